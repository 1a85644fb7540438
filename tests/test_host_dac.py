"""The library's host-only Dynamic Alignment Compressor arithmetic against the oracle on
seeded random inputs, plus its error codes.  No GPU."""
import math

import numpy as np
import pytest

import paper_2511_10333_amd as edgc
from oracle import dac_oracle as dac

CANDS = [2, 4, 8, 16, 32, 64, 128]


@pytest.mark.parametrize("seed", range(12))
def test_rank_bounds_matches_oracle(seed):
    rng = np.random.default_rng(seed)
    a_c, a_d = rng.uniform(5e-6, 100e-6, 2)
    b_c, b_d = rng.uniform(0.1e-6, 4e-6, 2)
    jitter = 1 + 0.2 * rng.standard_normal((len(CANDS), 2))         # measured times are not monotone
    per_rank = float(rng.integers(1 << 12, 1 << 18))
    tup = [(r, abs((a_c + b_c * r) * jitter[i, 0]), abs((a_d + b_d * r) * jitter[i, 1]), per_rank * r)
           for i, r in enumerate(CANDS)]
    costs = [edgc.RankCost(*t) for t in tup]
    d_orig = float(rng.integers(1 << 20, 1 << 28))
    for bw in np.geomspace(1e8, 2e12, 23):
        for div in (4.0, 4.7, 6.0):
            want = dac.rank_bounds(tup, d_orig, float(bw), div)
            got = edgc.rank_bounds(costs, d_orig, float(bw), div)
            assert (got.r_max, got.r_min) == want[:2]
            assert got.t_uncompressed == want[2] and got.t_com == want[3]     # same fp64 operations


@pytest.mark.parametrize("seed", range(8))
def test_fit_eta_matches_oracle(seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(1, 12))
    ranks = sorted(int(r) for r in rng.choice(np.arange(1, 200), n, replace=False))
    t = [float(rng.uniform(0.2e-3, 0.5e-3)) * r * float(1 + 0.1 * rng.standard_normal()) for r in ranks]
    t = [abs(x) + 1e-9 for x in t]
    eta_o, mape_o = dac.fit_eta(ranks, t)
    eta_g, mape_g = edgc.fit_eta(ranks, t)
    assert eta_g == pytest.approx(eta_o, rel=1e-14)
    assert mape_g == pytest.approx(mape_o, rel=1e-12, abs=1e-12)


@pytest.mark.parametrize("seed", range(12))
def test_stage_ranks_matches_oracle(seed):
    rng = np.random.default_rng(200 + seed)
    eta = float(rng.uniform(1e-5, 5e-3))
    r_min = int(rng.integers(1, 9))
    r_max = int(r_min + rng.integers(0, 120))
    r1 = int(rng.integers(r_min, r_max + 1))
    n_stages = int(rng.integers(1, 17))
    t_mb = float(rng.uniform(0, 20)) * eta if seed % 3 else float(rng.integers(0, 9)) * eta
    allowed = None
    if seed % 2:
        allowed = sorted(int(a) for a in rng.choice(np.arange(1, 160), int(rng.integers(1, 8)), replace=False))
    want = dac.stage_ranks(r1, t_mb, eta, r_min, r_max, n_stages, allowed)
    got = edgc.stage_ranks(r1, t_mb, eta, r_min, r_max, n_stages, allowed)
    assert got[0] == want[0]
    assert got[1] == pytest.approx(want[1], rel=1e-15)


def test_entropy_due_matches_oracle():
    for period in (1, 2, 3, 4, 10, 20, 1000):
        for t in list(range(45)) + [10 ** 12, 10 ** 12 + 1]:
            assert edgc.entropy_due(t, period) == dac.entropy_due(t, period)


def test_error_codes():
    good = [edgc.RankCost(4, 1.0, 1.0, 1.0), edgc.RankCost(8, 1.0, 1.0, 1.0)]
    EINVAL, ENONFINITE = -1, -5
    cases = [
        (lambda: edgc.rank_bounds([], 1.0, 1.0), EINVAL),
        (lambda: edgc.rank_bounds(good, 0.0, 1.0), EINVAL),
        (lambda: edgc.rank_bounds(good, 1.0, -1.0), EINVAL),
        (lambda: edgc.rank_bounds(good, 1.0, 1.0, 3.5), EINVAL),
        (lambda: edgc.rank_bounds(good, 1.0, 1.0, 6.5), EINVAL),
        (lambda: edgc.rank_bounds(good[::-1], 1.0, 1.0), EINVAL),
        (lambda: edgc.rank_bounds([edgc.RankCost(4, -1.0, 1.0, 1.0)], 1.0, 1.0), EINVAL),
        (lambda: edgc.rank_bounds([edgc.RankCost(4, math.nan, 1.0, 1.0)], 1.0, 1.0), ENONFINITE),
        (lambda: edgc.rank_bounds(good, math.inf, 1.0), ENONFINITE),
        (lambda: edgc.fit_eta([], []), EINVAL),
        (lambda: edgc.fit_eta([0], [1.0]), EINVAL),
        (lambda: edgc.fit_eta([1], [0.0]), EINVAL),
        (lambda: edgc.fit_eta([1], [math.nan]), ENONFINITE),
        (lambda: edgc.stage_ranks(8, 1.0, 0.0, 4, 64, 4), EINVAL),
        (lambda: edgc.stage_ranks(8, -1.0, 1.0, 4, 64, 4), EINVAL),
        (lambda: edgc.stage_ranks(8, 1.0, 1.0, 0, 64, 4), EINVAL),
        (lambda: edgc.stage_ranks(8, 1.0, 1.0, 65, 64, 4), EINVAL),
        (lambda: edgc.stage_ranks(8, 1.0, 1.0, 4, 64, 0), EINVAL),
        (lambda: edgc.stage_ranks(8, 1.0, 1.0, 4, 64, 4, [8, 4]), EINVAL),
        (lambda: edgc.stage_ranks(8, math.inf, 1.0, 4, 64, 4), ENONFINITE),
        (lambda: edgc.entropy_due(0, 0), EINVAL),
    ]
    for i, (call, code) in enumerate(cases):
        with pytest.raises(edgc.EdgcError) as e:
            call()
        assert e.value.code == code, i
