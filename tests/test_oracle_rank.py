"""Pins for the oracle's CQM pieces (Lemma 1, Theorem 1, Theorem 3) and the
window rule (Sec. IV-D-2 warm-up, Algorithm 1).  No GPU."""
import math

import numpy as np
import pytest

from oracle import edgc_oracle as orc


def _ab(m, n):
    mm, nn = min(m, n), max(m, n)
    return (math.sqrt(nn) - math.sqrt(mm)) ** 2, (math.sqrt(nn) + math.sqrt(mm)) ** 2


@pytest.mark.parametrize("m,n", [(256, 512), (512, 256), (300, 300), (4096, 16384), (1, 7)])
def test_cdf_end_points_and_monotone(m, n):
    a, b = _ab(m, n)
    assert orc.mp_cdf(a, m, n) == 0.0
    assert orc.mp_cdf(b, m, n) == 1.0
    assert orc.mp_cdf(b * (1 - 1e-12), m, n) == pytest.approx(1.0, abs=1e-5)
    lam = np.linspace(a, b, 401)
    F = np.array([orc.mp_cdf(x, m, n) for x in lam])
    assert np.all(np.diff(F) >= -1e-15) and 0.0 <= F.min() and F.max() <= 1.0
    assert orc.mp_cdf(m, n, m) == orc.mp_cdf(m, m, n)          # shape order is irrelevant


@pytest.mark.parametrize("m,n", [(256, 512), (1024, 1024), (2048, 8192)])
def test_cdf_derivative_is_the_textbook_marchenko_pastur_density(m, n):
    # density of the eigenvalues of A A^T (unit-variance entries, m <= n):
    #   f(l) = sqrt((l - a)(b - l)) / (2 pi m l)
    a, b = _ab(m, n)
    mm = min(m, n)
    for t in [0.07, 0.3, 0.5, 0.8, 0.97]:
        lam = a + t * (b - a)
        h = 1e-5 * (b - a)
        num = (orc.mp_cdf(lam + h, m, n) - orc.mp_cdf(lam - h, m, n)) / (2 * h)
        want = math.sqrt((lam - a) * (b - lam)) / (2 * math.pi * mm * lam)
        assert num == pytest.approx(want, rel=2e-5)


def test_quantile_inverts_cdf():
    for p in [1e-4, 0.1, 0.5, 0.9, 1 - 1e-4]:
        lam = orc.mp_quantile(p, 640, 1920)
        assert orc.mp_cdf(lam, 640, 1920) == pytest.approx(p, abs=1e-12)


@pytest.mark.parametrize("m,n", [(256, 512), (512, 256), (384, 384)])
def test_g_table_invariants(m, n):
    g = orc.g_table(m, n)
    mm = min(m, n)
    assert g.shape == (mm + 1,) and g[mm] == 0.0
    assert np.all(np.diff(g) < 0)                            # strictly decreasing in r
    # sum of all sampled eigenvalues estimates ||A||_F^2 = m n
    assert g[0] ** 2 == pytest.approx(m * n, rel=2e-3)
    assert np.array_equal(g, orc.g_table(n, m))


def test_g_matches_svd_tails_of_a_gaussian_matrix():
    # Theorem 1: g(r) estimates ||A - A_r||_F of a unit-variance random matrix
    m, n = 256, 512
    A = np.random.default_rng(0).standard_normal((m, n))
    s = np.linalg.svd(A, compute_uv=False)
    g = orc.g_table(m, n)
    for r in [0, 1, 16, 64, 128, 200, 250]:
        truth = math.sqrt(float((s[r:] ** 2).sum()))
        assert g[r] == pytest.approx(truth, rel=0.012)


def _prm(**kw):
    base = dict(m=512, n=512, r_min=4, r_max=64, step_limit=8, allowed=None, eta=0.0,
                total_iters=0, min_warmup_frac=0.0, r_ref=0)
    base.update(kw)
    return orc.RankParams(**base)


def test_first_window_sets_reference_and_stays_in_warmup():
    st = orc.RankState()
    d = orc.select_rank(st, [1.0, 3.0], 2, _prm())
    assert d.rank == 0 and d.H_mean == 2.0 and st.have_ref == 1 and st.H_ref == 2.0
    assert st.compressing == 0 and st.iters_seen == 2


def test_unchanged_entropy_returns_reference_rank_and_keeps_warmup():
    st = orc.RankState()
    orc.select_rank(st, [2.0], 10, _prm())
    d = orc.select_rank(st, [2.0], 10, _prm())
    assert d.r_unclamped == 64          # g^{-1}(g(r_max)) = r_max
    assert d.rank == 0                  # r_new < r_max is required to leave warm-up


def test_theorem3_target_scales_with_exp_of_entropy_drop():
    prm = _prm()
    g = orc.g_table(512, 512)
    for dH in [math.log(2.0), 0.05, 0.5, -0.1]:
        st = orc.RankState()
        orc.select_rank(st, [0.0], 1, prm)
        d = orc.select_rank(st, [-dH], 1, prm)
        target = math.exp(dH) * g[64]
        want = int(np.argmax(g <= target))     # smallest r with g(r) <= target
        assert d.r_unclamped == want
        if dH > 0:
            assert d.r_unclamped < 64           # entropy down => rank down (Sec. IV-D-3)
        else:
            assert d.r_unclamped > 64           # entropy up => rank up


def test_algorithm1_step_limit_and_clamp_hand_table():
    prm = _prm(r_min=16, r_max=64, step_limit=8, eta=0.5)
    st = orc.RankState()
    orc.select_rank(st, [0.0], 1, prm)
    # a large entropy drop asks for rank 0: steps of 8 from r_max, then the r_min clamp
    seen = [orc.select_rank(st, [-3.0], 1, prm) for _ in range(8)]
    assert [d.rank for d in seen] == [56, 48, 40, 32, 24, 16, 16, 16]
    assert [d.T_com for d in seen] == [0.5 * r for r in [56, 48, 40, 32, 24, 16, 16, 16]]
    assert all(d.r_unclamped == 0 for d in seen)
    # entropy back above the reference: climb by 8 per window, clamp at r_max
    up = [orc.select_rank(st, [1.0], 1, prm).rank for _ in range(8)]
    assert up == [24, 32, 40, 48, 56, 64, 64, 64]


def test_small_moves_are_taken_directly():
    prm = _prm(r_min=4, r_max=64, step_limit=8)
    g = orc.g_table(512, 512)
    # pick the entropy drop that asks for exactly rank 60 (|60 - 64| <= 8)
    dH = math.log(g[60] / g[64]) + 1e-9
    st = orc.RankState()
    orc.select_rank(st, [0.0], 1, prm)
    d = orc.select_rank(st, [-dH], 1, prm)
    assert d.r_unclamped == 60 and d.rank == 60 and st.r_prev == 60


def test_allowed_set_snaps_up_but_state_stays_unsnapped():
    prm = _prm(r_min=4, r_max=64, step_limit=8, allowed=[4, 8, 16, 32, 64])
    st = orc.RankState()
    orc.select_rank(st, [0.0], 1, prm)
    ranks, states = [], []
    for _ in range(9):
        ranks.append(orc.select_rank(st, [-5.0], 1, prm).rank)
        states.append(st.r_prev)
    assert states == [56, 48, 40, 32, 24, 16, 8, 4, 4]
    assert ranks == [64, 64, 64, 32, 32, 16, 8, 4, 4]


def test_snapping_never_leaves_the_rank_bounds():
    # Sec. IV-D-1: r_max is where compression stops paying, and Algorithm 1 ends with the clamp to
    # [r_min, r_max]: with r_max = 48 the set {4, 8, 16, 32, 64} must never emit 64.  Hand table:
    # the state walks 40, 32, 24, ... down from r_ref = r_max = 48 and back up to 48.
    prm = _prm(r_min=6, r_max=48, step_limit=8, allowed=[4, 8, 16, 32, 64])
    st = orc.RankState()
    orc.select_rank(st, [0.0], 1, prm)
    down = [(orc.select_rank(st, [-5.0], 1, prm).rank, st.r_prev) for _ in range(7)]
    assert down == [(32, 40), (32, 32), (32, 24), (16, 16), (8, 8), (8, 6), (8, 6)]   # 4 < r_min is never emitted
    up = [(orc.select_rank(st, [1.0], 1, prm).rank, st.r_prev) for _ in range(7)]
    assert up == [(16, 14), (32, 22), (32, 30), (32, 38), (32, 46), (32, 48), (32, 48)]  # 64 > r_max: 32 instead
    # no allowed rank inside the bounds, or a lower bound of 0 (rank 0 means warm-up): rejected
    for bad in [_prm(r_min=33, r_max=63, allowed=[4, 8, 16, 32, 64]), _prm(r_min=0)]:
        with pytest.raises(orc.OracleError):
            orc.select_rank(orc.RankState(), [0.0], 1, bad)


def test_warmup_lasts_at_least_ten_percent():
    prm = _prm(total_iters=200, min_warmup_frac=0.10)
    st = orc.RankState()
    assert orc.select_rank(st, [0.0], 5, prm).rank == 0       # reference window, 5 iters
    assert orc.select_rank(st, [-1.0], 5, prm).rank == 0      # 10 iters seen < 20
    assert orc.select_rank(st, [-1.0], 5, prm).rank == 0      # 15
    d = orc.select_rank(st, [-1.0], 5, prm)                   # 20 >= 10 % of 200
    assert d.rank == 56 and st.compressing == 1


def test_reference_rank_override_lets_rank_rise_from_below():
    prm = _prm(r_min=4, r_max=64, step_limit=8, r_ref=4, allowed=[4, 8, 16, 32, 64])
    st = orc.RankState()
    orc.select_rank(st, [0.0], 1, prm)
    d = orc.select_rank(st, [0.0], 1, prm)
    assert d.r_unclamped == 4 and d.rank == 4                  # compression starts at r_ref
    d = orc.select_rank(st, [0.4], 1, prm)                     # entropy rose: asks for more
    assert d.r_unclamped > 12 and st.r_prev == 12 and d.rank == 16


def test_bad_parameters_rejected():
    st = orc.RankState()
    for prm in [_prm(r_max=0), _prm(r_max=1000), _prm(r_min=65), _prm(allowed=[8, 4])]:
        with pytest.raises(orc.OracleError):
            orc.select_rank(st, [0.0], 1, prm)
    with pytest.raises(orc.OracleError):
        orc.select_rank(st, [float("nan")], 1, _prm())
