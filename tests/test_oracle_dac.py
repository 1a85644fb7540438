"""Pins for the oracle of the Dynamic Alignment Compressor's host arithmetic: values worked
out by hand from Sec. IV-D-1 (rank bounds, T_com = eta r), Algorithm 2 / Eq. 16 (stage
alignment) and Sec. IV-B (iteration sampling), plus closed forms and a library least-squares
routine for the fit."""
import math

import numpy as np
import pytest

from oracle import dac_oracle as dac

CANDS = [4, 8, 16, 32, 64, 128, 256]


def linear_costs(a_c, b_c, a_d, b_d, bytes_per_rank):
    return [(r, a_c + b_c * r, a_d + b_d * r, bytes_per_rank * r) for r in CANDS]


def test_rank_bounds_hand_example_32gbps():
    # T_c = 50us + 2us r, T_d = 30us + 1us r, D_c = 8192 r bytes, B = 4e9 B/s (32 Gbit/s),
    # D_orig = 4 MiB: plain exchange 1048.576 us; T_com = 80us + 5.048us r <= 1048.576us
    # <=> r <= 191.87  =>  r_max = 128 among the candidates
    costs = linear_costs(50e-6, 2e-6, 30e-6, 1e-6, 8192.0)
    r_max, r_min, t_plain, t_com = dac.rank_bounds(costs, 4194304.0, 4e9, 4.0)
    assert (r_max, r_min) == (128, 32)
    assert t_plain == pytest.approx(1048.576e-6, rel=1e-12)
    assert t_com[0] == pytest.approx(80e-6 + 5.048e-6 * 4, rel=1e-12)
    assert t_com[-1] == pytest.approx(80e-6 + 5.048e-6 * 256, rel=1e-12)
    # the footnote's range: r_max/6 <= r_min <= r_max/4
    assert dac.rank_bounds(costs, 4194304.0, 4e9, 6.0)[1] == 22        # ceil(21.33)
    assert dac.rank_bounds(costs, 4194304.0, 4e9, 5.0)[1] == 26        # ceil(25.6)


def test_rank_bounds_fast_link_never_pays():
    # 400 Gbit/s: plain exchange 83.886 us < the 80 us + 3.16 us r of any candidate
    costs = linear_costs(50e-6, 2e-6, 30e-6, 1e-6, 8192.0)
    r_max, r_min, _, _ = dac.rank_bounds(costs, 4194304.0, 50e9, 4.0)
    assert (r_max, r_min) == (0, 0)


def test_rank_bounds_threshold_matches_the_solved_inequality():
    # solve the inequality for r in closed form and compare over a sweep of bandwidths
    a, b, bytes_per_rank, d_orig = 75e-6, 2.5e-6, 16384.0, 64.0 * 2 ** 20
    costs = linear_costs(a / 3, b / 5, 2 * a / 3, 4 * b / 5, bytes_per_rank)
    for bw in np.geomspace(1e8, 1e12, 41):
        r_star = (d_orig / bw - a) / (b + bytes_per_rank / bw)
        want = max([r for r in CANDS if r <= r_star], default=0)
        assert dac.rank_bounds(costs, d_orig, bw, 4.0)[0] == want, bw


def test_rank_bounds_equality_counts_as_paying_and_first_violation_closes():
    # exactly equal times satisfy "<="
    costs = [(4, 1.0, 1.0, 0.0), (8, 2.0, 2.0, 0.0)]
    assert dac.rank_bounds(costs, 4.0, 1.0, 4.0)[0] == 8
    # rank 16 violates, rank 32 would satisfy again: the scan stopped at 16
    costs = [(8, 1.0, 0.0, 0.0), (16, 9.0, 0.0, 0.0), (32, 1.0, 0.0, 0.0)]
    assert dac.rank_bounds(costs, 4.0, 1.0, 4.0)[0] == 8
    # r_min never drops below 1
    assert dac.rank_bounds([(2, 0.0, 0.0, 0.0)], 4.0, 1.0, 6.0)[:2] == (2, 1)


def test_rank_bounds_rejects_bad_arguments():
    good = [(4, 1.0, 1.0, 1.0)]
    for args in [([], 1.0, 1.0, 4.0), (good, 0.0, 1.0, 4.0), (good, 1.0, 0.0, 4.0),
                 (good, 1.0, 1.0, 3.9), (good, 1.0, 1.0, 6.1),
                 ([(8, 1, 1, 1), (8, 1, 1, 1)], 1.0, 1.0, 4.0)]:
        with pytest.raises(ValueError):
            dac.rank_bounds(*args)


def test_fit_eta_hand_example():
    # ranks (1, 2), times (1, 3): eta = (1 + 6) / (1 + 4) = 1.4;
    # errors |1 - 1.4| / 1 = 0.4 and |3 - 2.8| / 3 = 1/15  =>  MAPE = 100 (0.4 + 1/15) / 2
    eta, mape = dac.fit_eta([1, 2], [1.0, 3.0])
    assert eta == pytest.approx(1.4, rel=1e-15)
    assert mape == pytest.approx(100.0 * (0.4 + 1.0 / 15.0) / 2.0, rel=1e-13)


def test_fit_eta_exact_line_and_library_least_squares():
    ranks = [4, 8, 16, 32, 64, 128]
    eta, mape = dac.fit_eta(ranks, [0.37e-3 * r for r in ranks])
    assert eta == pytest.approx(0.37e-3, rel=1e-14) and mape <= 1e-12
    rng = np.random.default_rng(5)
    t = 0.37e-3 * np.array(ranks) * (1 + 0.05 * rng.standard_normal(len(ranks)))
    eta, mape = dac.fit_eta(ranks, list(t))
    ref = np.linalg.lstsq(np.array(ranks, dtype=np.float64)[:, None], t, rcond=None)[0][0]
    assert eta == pytest.approx(ref, rel=1e-12)
    assert mape == pytest.approx(100 * np.mean(np.abs(t - ref * np.array(ranks)) / t), rel=1e-10)
    # scaling every time scales eta and leaves the percentage error alone
    eta2, mape2 = dac.fit_eta(ranks, list(3.0 * t))
    assert eta2 == pytest.approx(3 * eta, rel=1e-13) and mape2 == pytest.approx(mape, rel=1e-10)


def test_stage_ranks_hand_example():
    # eta = 2 ms per rank, stage 1 at rank 16 (32 ms), micro-batch backward 9 ms:
    # budgets 41, 50, 59 ms -> 20.5, 25, 29.5 -> ranks 20, 25, 29; r_max = 28 clamps the last
    ranks, t = dac.stage_ranks(16, 9e-3, 2e-3, 4, 28, 4)
    assert ranks == [16, 20, 25, 28]
    assert t == pytest.approx([32e-3, 40e-3, 50e-3, 56e-3], rel=1e-14)
    # allowed ranks: the largest one not above each of those
    assert dac.stage_ranks(16, 9e-3, 2e-3, 4, 28, 4, [4, 8, 16, 32])[0] == [16, 16, 16, 16]
    assert dac.stage_ranks(16, 9e-3, 2e-3, 4, 64, 4, [4, 8, 16, 24, 32])[0] == [16, 16, 24, 24]


def test_stage_ranks_offset_that_is_a_whole_number_of_ranks():
    # T_microBack = k eta  =>  Eq. 16 gives r_i = r_1 + (i - 1) k exactly, for awkward eta too
    for eta in (1e-3, 0.3e-3, 7.7e-5, 1.0 / 3.0):
        for k in (1, 3, 7):
            ranks, _ = dac.stage_ranks(5, k * eta, eta, 1, 1000, 6)
            assert ranks == [5 + i * k for i in range(6)], (eta, k)


def test_stage_ranks_single_stage_zero_offset_and_lower_clamp():
    assert dac.stage_ranks(12, 1e-3, 1e-3, 4, 64, 1)[0] == [12]
    assert dac.stage_ranks(12, 0.0, 1e-3, 4, 64, 3)[0] == [12, 12, 12]
    # a stage-1 rank below r_min (cannot come out of Algorithm 1, but the clamp still holds)
    assert dac.stage_ranks(2, 0.0, 1e-3, 4, 64, 2)[0] == [2, 4]
    # every later stage's budget is at least stage 1's: ranks never decrease
    ranks, t = dac.stage_ranks(9, 2.3e-3, 0.7e-3, 4, 64, 8)
    assert ranks == sorted(ranks) and all(r <= 64 for r in ranks)
    for i, r in enumerate(ranks[1:], start=1):
        assert 0.7e-3 * r <= 0.7e-3 * 9 + i * 2.3e-3 + 1e-12 or r == 4


def test_entropy_due_counts_alpha_of_the_window():
    # alpha = 1/4 over a 20-iteration window: 5 measurements, at 0, 4, 8, 12, 16
    due = [t for t in range(20) if dac.entropy_due(t, 4)]
    assert due == [0, 4, 8, 12, 16]
    assert all(dac.entropy_due(t, 1) for t in range(20))          # alpha = 1
    assert sum(dac.entropy_due(t, 20) for t in range(20)) == 1    # alpha = 5 %
    with pytest.raises(ValueError):
        dac.entropy_due(0, 0)
