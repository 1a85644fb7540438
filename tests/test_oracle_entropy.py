"""Pins for the oracle's sampler and entropy estimator (no GPU).

Each test binds the C oracle to something other than itself: published
splitmix64 outputs, brute-force enumeration of the sampling predicate, special
cases with known entropy, a NumPy float32 re-computation of the bins, and the
closed forms of Lemma 2 (Gaussian) and of the Laplace distribution.
"""
import math

import numpy as np
import pytest

import edgc_inputs as gen
from oracle import edgc_oracle as orc


def test_mix64_matches_published_splitmix64_stream():
    # First outputs of the splitmix64 generator seeded with 0 (its public reference test
    # vector, stored under tests/golden/); counter c gives the (c+1)-th output.
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "splitmix64_seed0.txt")
    want = [int(line.split()[1], 16) for line in open(path) if line.strip() and not line.startswith("#")]
    assert len(want) == 3 and want[0] == 0xE220A8397B1DCDAF
    assert [orc.mix64(0, c) for c in range(len(want))] == want


@pytest.mark.parametrize("n,stride,chunk", [(1, 1, 1), (37, 1, 5), (1000, 7, 1), (1000, 7, 3),
                                             (1000, 10, 64), (4097, 100, 64), (513, 4, 128),
                                             (50, 100, 8)])
def test_sample_indices_brute_force(n, stride, chunk):
    for seed, step in [(0, 0), (0, 1), (123, 7), (2**63 + 5, 2**40)]:
        slot = orc.sample_slot(seed, step, stride)
        assert 0 <= slot < stride
        assert slot == orc.mix64(seed, step) % stride
        want = np.array([i for i in range(n) if (i // chunk) % stride == slot], dtype=np.uint64)
        got = orc.sample_indices(n, stride, chunk, seed, step)
        assert np.array_equal(got, want)
        if stride == 1:
            assert got.size == n


def test_slot_changes_with_step_and_covers_all_slots():
    slots = {orc.sample_slot(0, s, 10) for s in range(200)}
    assert slots == set(range(10))


def test_constant_tensor_has_zero_entropy():
    x = np.full(10000, 0.125, dtype=np.float32)
    r = orc.entropy(x, 1, 1, 0, 0, 256)
    assert r.H_bits == 0.0 and r.h_diff_nats == -math.inf
    assert r.counts[0] == 10000 and r.counts[1:].sum() == 0
    assert r.lo == r.hi == 0.125


@pytest.mark.parametrize("bins", [2, 256, 1024, 65536])
def test_equally_populated_bins_give_log2_bins(bins):
    # bin centres of [0, bins): every bin gets exactly `rep` samples
    rep = 3
    x = np.repeat(np.arange(bins, dtype=np.float32) + 0.5, rep)
    x = np.concatenate([x, np.array([0.0, float(bins)], dtype=np.float32)])  # pin lo/hi
    r = orc.entropy(x, 1, 1, 0, 0, bins)
    # the two range-pinning samples sit in the first and last bin
    c = np.full(bins, rep, dtype=np.uint64); c[0] += 1; c[-1] += 1
    assert np.array_equal(r.counts, c)
    r2 = orc.entropy(x[:-2], 1, 1, 0, 0, bins, value_range=(0.0, float(bins)))
    assert np.array_equal(r2.counts, np.full(bins, rep, dtype=np.uint64))
    assert r2.H_bits == pytest.approx(math.log2(bins), abs=1e-10)
    assert r2.h_diff_nats == pytest.approx(math.log(bins), abs=1e-10)   # width 1 => ln B


def test_two_values_half_half_is_one_bit_and_top_edge_goes_to_last_bin():
    x = np.array([-1.0] * 500 + [3.0] * 500, dtype=np.float32)
    r = orc.entropy(x, 1, 1, 0, 0, 64)
    assert r.H_bits == pytest.approx(1.0, abs=1e-12)
    assert r.counts[0] == 500 and r.counts[63] == 500      # x == hi lands in bin B-1


def test_counts_sum_permutation_invariance_and_nonfinite_skipped():
    x = gen.gaussian(50000, 1e-3, 3)
    x[[5, 77, 4000]] = [np.nan, np.inf, -np.inf]
    r = orc.entropy(x, 1, 1, 0, 0, 512)
    assert r.n_sampled == 50000 and r.n_nonfinite == 3
    assert int(r.counts.sum()) == 50000 - 3
    p = np.random.default_rng(1).permutation(x)
    rp = orc.entropy(p, 1, 1, 0, 0, 512)
    assert np.array_equal(r.counts, rp.counts) and r.H_bits == rp.H_bits
    with pytest.raises(orc.OracleError) as e:
        orc.entropy(np.full(10, np.nan, dtype=np.float32), 1, 1, 0, 0, 16)
    assert e.value.code == orc.ENONFINITE


def _numpy_fp32_counts(sample, bins, lo=None, hi=None):
    s = sample[np.isfinite(sample)].astype(np.float32)
    lo = np.float32(s.min() if lo is None else lo)
    hi = np.float32(s.max() if hi is None else hi)
    w = np.float32(hi - lo)
    scale = np.float32(np.float32(bins) / w)
    t = (s - lo).astype(np.float32)
    u = (t * scale).astype(np.float32)
    b = np.clip(np.trunc(u.astype(np.float64)), 0, bins - 1).astype(np.int64)
    return np.bincount(b, minlength=bins).astype(np.uint64), float(lo), float(hi)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("stride,chunk,bins", [(1, 1, 256), (100, 64, 256), (10, 1, 4096),
                                                (7, 33, 1000), (100, 64, 65536)])
def test_histogram_matches_numpy_float32_recomputation(dtype, stride, chunk, bins):
    n = 300_007
    x = gen.laplace_mixture(n, seed=5, dtype=dtype)
    r = orc.entropy(x, stride, chunk, 11, 3, bins)
    idx = orc.sample_indices(n, stride, chunk, 11, 3).astype(np.int64)
    vals = gen.bf16_bits_to_f32(x[idx]) if dtype == "bf16" else x[idx]
    want, lo, hi = _numpy_fp32_counts(vals, bins)
    assert r.n_sampled == idx.size
    assert (r.lo, r.hi) == (lo, hi)
    assert np.array_equal(r.counts, want)
    p = want[want > 0].astype(np.float64) / want.sum()
    assert r.H_bits == pytest.approx(float(-(p * np.log2(p)).sum()), abs=1e-10)
    w32 = float(np.float32(hi) - np.float32(lo))          # the fp32 range the bins are built on
    assert r.h_diff_nats == pytest.approx(r.H_bits * math.log(2) + math.log(w32 / bins), abs=1e-9)


def test_caller_range_clamps_outliers_to_edge_bins():
    x = np.array([-5.0, -1.0, -0.5, 0.0, 0.49, 0.5, 1.0, 9.0], dtype=np.float32)
    r = orc.entropy(x, 1, 1, 0, 0, 4, value_range=(-1.0, 1.0))
    # bins of width 0.5 over [-1, 1]: [-1,-.5) [-.5,0) [0,.5) [.5,1]
    assert r.counts.tolist() == [2, 1, 2, 3]
    assert (r.lo, r.hi) == (-1.0, 1.0)


@pytest.mark.parametrize("sigma", [1.0, 1e-3])
def test_gaussian_matches_lemma2_closed_form(sigma):
    # Lemma 2: H = ln sigma + 1/2 ln(2 pi e)
    x = gen.gaussian(4_000_000, sigma, 9)
    r = orc.entropy(x, 1, 1, 0, 0, 4096)
    want = math.log(sigma) + 0.5 * math.log(2 * math.pi * math.e)
    assert r.h_diff_nats == pytest.approx(want, abs=5e-3)


def test_rescaling_shifts_differential_entropy_only():
    x = gen.gaussian(200_000, 1e-2, 4)
    a = orc.entropy(x, 4, 16, 1, 2, 1024)
    b = orc.entropy((x * np.float32(8.0)).astype(np.float32), 4, 16, 1, 2, 1024)
    assert np.array_equal(a.counts, b.counts) and a.H_bits == b.H_bits   # power of two: exact
    assert b.h_diff_nats - a.h_diff_nats == pytest.approx(math.log(8.0), abs=1e-9)


def test_laplace_matches_textbook_entropy():
    # differential entropy of Laplace(0, b) is 1 + ln(2b)
    rng = np.random.default_rng(21)
    b = 2e-3
    x = rng.laplace(0.0, b, 4_000_000).astype(np.float32)
    r = orc.entropy(x, 1, 1, 0, 0, 8192)
    assert r.h_diff_nats == pytest.approx(1.0 + math.log(2 * b), abs=1e-2)


def test_subsample_tracks_full_entropy():
    # Sec. IV-B / ablation: a small beta still captures the entropy
    x = gen.laplace_mixture(2_000_000, seed=2)
    full = orc.entropy(x, 1, 1, 0, 0, 1024, value_range=(-0.05, 0.05))
    sub = orc.entropy(x, 20, 64, 0, 0, 1024, value_range=(-0.05, 0.05))
    assert abs(sub.n_sampled - 100_000) <= 64
    assert sub.H_bits == pytest.approx(full.H_bits, abs=0.03)


def test_bad_arguments_are_rejected():
    x = np.zeros(8, dtype=np.float32)
    for kw in [dict(stride=0), dict(chunk=0), dict(bins=0)]:
        a = dict(stride=1, chunk=1, bins=4); a.update(kw)
        with pytest.raises(orc.OracleError) as e:
            orc.entropy(x, a["stride"], a["chunk"], 0, 0, a["bins"])
        assert e.value.code == orc.EINVAL
