"""Pins for the oracle's rank-r compressor with error feedback (no GPU).

NumPy/LAPACK (matmul, QR, SVD) in float64 is the independent side: each step
of the oracle is compared with the textbook routine it must reduce to, and
the whole is checked against invariants that fail on a dropped term, a wrong
sign or a transposed operand.
"""
import math

import numpy as np
import pytest
from scipy import stats

import edgc_inputs as gen
from oracle import edgc_oracle as orc


def _fro(a):
    return float(np.linalg.norm(np.asarray(a, dtype=np.float64)))


def _qr_pos(P):
    """Q-factor of the thin QR with a positive diagonal of R (unique for full column rank)."""
    Qf, R = np.linalg.qr(np.asarray(P, dtype=np.float64))
    sgn = np.sign(np.diag(R)); sgn[sgn == 0] = 1.0
    return Qf * sgn


def _q0(n, r, seed=0):
    Q = np.zeros((n, r), dtype=np.float32)
    orc.init_q(Q, 0, r, seed)
    return Q


def test_init_q_is_standard_normal_and_column_stable():
    Q = _q0(4096, 16, seed=3)
    flat = Q.astype(np.float64).ravel()
    assert abs(flat.mean()) < 0.02 and abs(flat.std() - 1.0) < 0.02
    assert stats.kstest(flat, "norm").pvalue > 1e-3
    assert abs(np.corrcoef(Q[:, 0], Q[:, 1])[0, 1]) < 0.06
    # growing the rank later reproduces the same columns (pure function of seed, row, column)
    Q2 = np.zeros((4096, 16), dtype=np.float32)
    orc.init_q(Q2, 0, 4, 3)
    orc.init_q(Q2, 4, 16, 3)
    assert np.array_equal(Q, Q2)
    Q3 = np.zeros((4096, 32), dtype=np.float32)
    orc.init_q(Q3, 0, 32, 3)
    assert np.array_equal(Q3[:, :16], Q)
    assert not np.array_equal(_q0(64, 4, seed=1), _q0(64, 4, seed=2))


@pytest.mark.parametrize("m,n,r", [(96, 160, 4), (160, 96, 7), (64, 64, 16)])
def test_each_step_reduces_to_the_library_routine(m, n, r):
    G = gen.lowrank_plus_noise(m, n, min(m, n, 32), 0.8, 1e-3, seed=1)
    E = (1e-2 * np.random.default_rng(5).standard_normal((m, n))).astype(np.float32)
    Q0 = _q0(n, r)
    P, Q1, D = orc.compress(G, E, Q0, r)
    assert np.array_equal(D, G + E)                                   # D = G + E_old, fp32
    Pn = D.astype(np.float64) @ Q0.astype(np.float64)                 # P = D Q
    Ph = _qr_pos(Pn)                                                  # orthonormalise
    assert _fro(P - Ph) / _fro(Ph) < 2e-6
    Qn = D.astype(np.float64).T @ P.astype(np.float64)                # Q = D^T P^
    assert _fro(Q1 - Qn) / _fro(Qn) < 1e-6
    out, En = orc.decompress(P, Q1, D, orc.F32)
    Mh = P.astype(np.float64) @ Q1.astype(np.float64).T               # M^ = P^ Q^T
    assert _fro(out - Mh) / _fro(Mh) < 1e-6
    assert np.array_equal(En, D - out)                                # E_new = D - M^, fp32
    for (i, j) in [(0, 0), (m - 1, n - 1), (3, 5)]:
        assert orc.reconstruct_one(P, Q1, i, j, orc.F32) == float(out[i, j])


@pytest.mark.parametrize("r", [1, 4, 8])
def test_exact_rank_r_matrix_is_reconstructed(r):
    M = gen.exact_rank(128, 192, r, seed=2)
    P, Q, D = orc.compress(M, None, _q0(192, r), r)
    out, E = orc.decompress(P, Q, D, orc.F32)
    assert _fro(M - out) / _fro(M) < 5e-6       # entries of M carry fp32 rounding of A B
    assert _fro(E) / _fro(M) < 5e-6


def test_invariants_orthonormal_orthogonal_residual_pythagoras():
    m, n, r = 256, 320, 8
    G = gen.lowrank_plus_noise(m, n, 64, 0.9, 1e-3, seed=4)
    P, Q, D = orc.compress(G, None, _q0(n, r), r)
    out, E = orc.decompress(P, Q, D, orc.F32)
    P64, Q64, D64, E64 = (a.astype(np.float64) for a in (P, Q, D, E))
    assert np.abs(P64.T @ P64 - np.eye(r)).max() < 1e-6               # P^T P = I
    assert np.abs(P64.T @ E64).max() < 1e-5 * _fro(D)                 # P^T E_new = 0
    assert _fro(E) ** 2 == pytest.approx(_fro(D) ** 2 - _fro(Q) ** 2, rel=1e-5)
    assert np.array_equal(D, out + E) or _fro(D - (out + E)) / _fro(D) < 1e-7


def test_eckart_young_bound_and_convergence_to_it():
    m, n, r = 192, 256, 6
    G = gen.lowrank_plus_noise(m, n, 48, 0.85, 1e-3, seed=6)
    s = np.linalg.svd(G.astype(np.float64), compute_uv=False)
    best = math.sqrt(float((s[r:] ** 2).sum()))
    Q = _q0(n, r)
    errs = []
    for _ in range(12):                       # repeated warm-started steps on a fixed matrix
        P, Q, D = orc.compress(G, None, Q, r)
        out, E = orc.decompress(P, Q, D, orc.F32)
        errs.append(_fro(E))
    assert all(e >= best * (1 - 1e-6) for e in errs)                  # never beats the SVD
    assert errs[-1] <= errs[0] and errs[-1] == pytest.approx(best, rel=2e-3)
    # more power iterations inside one call == the same number of warm-started calls
    P2, Q2, _ = orc.compress(G, None, _q0(n, r), r, power_iters=3)
    Qs = _q0(n, r)
    for _ in range(3):
        Ps, Qs, _ = orc.compress(G, None, Qs, r)
    assert np.array_equal(P2, Ps) and np.array_equal(Q2, Qs)


def test_rank_one_is_the_power_method():
    G = gen.lowrank_plus_noise(96, 128, 16, 0.5, 1e-4, seed=8)
    s = np.linalg.svd(G.astype(np.float64), compute_uv=False)
    Q = _q0(128, 1)
    for _ in range(15):
        P, Q, _ = orc.compress(G, None, Q, 1)
    assert _fro(Q) == pytest.approx(s[0], rel=1e-5)                   # ||Q|| -> sigma_1


def test_error_feedback_telescopes():
    m, n, r, T = 64, 96, 4, 6
    rng = np.random.default_rng(10)
    Q, E, acc_out = _q0(n, r), None, np.zeros((m, n))
    acc_g = np.zeros((m, n))
    for t in range(T):
        G = rng.standard_normal((m, n)).astype(np.float32)
        acc_g += G
        P, Q, D = orc.compress(G, E, Q, r)
        out, E = orc.decompress(P, Q, D, orc.F32)
        acc_out += out
    # sum_t out_t + E_T = sum_t G_t  (up to fp32 rounding of each D = G + E)
    assert _fro(acc_out + E - acc_g) / _fro(acc_g) < 1e-6


@pytest.mark.parametrize("code", ["f32", "bf16"])
def test_residual_in_factored_form_is_the_stored_residual(code):
    """What the deferred form of the library relies on: the residual the chain stores is exactly
    D - widen(M^ as transmitted), so a chain that keeps D and the factors and forms
    D_next = G + (D - M^) on the way walks through the same bits."""
    m, n, r, T = 48, 80, 4, 4
    rng = np.random.default_rng(12)
    dt = orc.BF16 if code == "bf16" else orc.F32
    Q, E, D_prev, out_prev = _q0(n, r), None, None, None
    for t in range(T):
        G = rng.standard_normal((m, n)).astype(np.float32)
        if code == "bf16":
            G = gen.to_bf16_bits(G)
        P, Q, D = orc.compress(G, E, Q, r)
        if D_prev is not None:                      # the same D from the factored form of E
            wide = gen.bf16_bits_to_f32(out_prev) if code == "bf16" else out_prev
            g32 = gen.bf16_bits_to_f32(G) if code == "bf16" else G
            assert np.array_equal(D, g32 + (D_prev - wide))
        out, E = orc.decompress(P, Q, D, dt)
        wide = gen.bf16_bits_to_f32(out) if code == "bf16" else out
        assert np.array_equal(E, D - wide)
        # and M^ is a function of the factors alone: recomputing it from (P, Q) gives the same bits
        out2, _ = orc.decompress(P, Q, np.zeros_like(D), dt)
        assert np.array_equal(out2, out)
        D_prev, out_prev = D, out


def test_zero_matrix_gives_zero_factors():
    Z = np.zeros((32, 48), dtype=np.float32)
    P, Q, D = orc.compress(Z, None, _q0(48, 4), 4)
    out, E = orc.decompress(P, Q, D, orc.F32)
    assert not P.any() and not Q.any() and not out.any() and not E.any()


def test_bf16_mode_rounds_operands_and_output():
    m, n, r = 96, 128, 8
    Gb = gen.lowrank_plus_noise(m, n, 32, 0.9, 1e-3, seed=12, dtype="bf16")
    G32 = gen.bf16_bits_to_f32(Gb)
    E = (1e-3 * np.random.default_rng(3).standard_normal((m, n))).astype(np.float32)
    Q0 = _q0(n, r)
    P, Q1, D = orc.compress(Gb, E, Q0, r)
    assert np.array_equal(D, G32 + E)

    def rb(a):                                  # independent RNE rounding through bf16
        return gen.bf16_bits_to_f32(gen.to_bf16_bits(a)).astype(np.float64)
    Pn = rb(D) @ rb(Q0)
    assert _fro(P - _qr_pos(Pn)) / math.sqrt(r) < 2e-6
    Qn = rb(D).T @ rb(P)
    assert _fro(Q1 - Qn) / _fro(Qn) < 1e-6
    out, En = orc.decompress(P, Q1, D, orc.BF16)
    assert out.dtype == np.uint16
    Mh = (rb(P) @ rb(Q1).T).astype(np.float32)
    assert np.array_equal(out, gen.to_bf16_bits(Mh))
    assert np.array_equal(En, D - gen.bf16_bits_to_f32(out))          # EF absorbs the rounding
    assert orc.reconstruct_one(P, Q1, 5, 7, orc.BF16) == float(gen.bf16_bits_to_f32(out[5:6, 7])[0])


def test_bf16_conversions_round_to_nearest_even():
    cases = {1.0: 0x3F80, 1.00390625: 0x3F80, 1.01171875: 0x3F82, -2.5: 0xC020, 0.0: 0x0000}
    for x, bits in cases.items():
        assert orc.f32_to_bf16_scalar(x) == bits
    x = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    assert all(orc.f32_to_bf16_scalar(float(v)) == int(b) for v, b in zip(x[:2000], gen.to_bf16_bits(x[:2000])))


def test_bad_arguments_rejected():
    G = np.zeros((8, 8), dtype=np.float32)
    with pytest.raises(orc.OracleError):
        orc.compress(G, None, _q0(8, 9), 9)           # r > min(m, n)
    with pytest.raises(orc.OracleError):
        orc.compress(G, None, _q0(8, 2), 2, power_iters=0)


def test_thread_count_does_not_change_any_result():
    # the oracle's OpenMP loops only split independent outputs: one thread and all threads agree bit for bit
    G = gen.lowrank_plus_noise(96, 200, 16, 0.9, 1e-3, seed=3)
    Q0 = np.zeros((200, 8), dtype=np.float32)
    orc.init_q(Q0, 0, 8, 5)
    n0 = orc.num_threads()
    try:
        outs = []
        for nt in (1, max(n0, 2)):
            orc.set_num_threads(nt)
            assert orc.num_threads() == nt
            P, Q, D = orc.compress(G, None, Q0, 8)
            out, E = orc.decompress(P, Q, D, orc.F32)
            outs.append((P, Q, D, out, E))
        for a, b in zip(*outs):
            assert np.array_equal(a, b)
    finally:
        orc.set_num_threads(n0)


def test_single_steps_equal_the_whole_step_and_numpy():
    # contract_p / orthonormalise / contract_q are the routines compress is made of: chained they give
    # compress bit for bit, on gathered rows / columns they give the corresponding rows of its result, and
    # each equals the plain NumPy product of the (rounded) operands
    for dtype, code in (("f32", orc.F32), ("bf16", orc.BF16)):
        G = gen.lowrank_plus_noise(150, 260, 24, 0.9, 1e-3, seed=8, dtype=dtype)
        E = gen.gaussian(150 * 260, 1e-4, 9).reshape(150, 260)
        Q0 = np.zeros((260, 12), dtype=np.float32)
        orc.init_q(Q0, 0, 12, 4)
        P, Q1, D = orc.compress(G, E, Q0, 12)
        P_raw = orc.contract_p(D, Q0, code)
        P_hat = orc.orthonormalise(P_raw)
        assert np.array_equal(P_hat, P)
        assert np.array_equal(orc.contract_q(D, P_hat, code), Q1)
        rows, cols = [0, 7, 149], [3, 259, 100]
        assert np.array_equal(orc.contract_p(D[rows], Q0, code), P_raw[rows])
        assert np.array_equal(orc.contract_q(D[:, cols], P_hat, code), Q1[cols])
        rnd = (lambda a: gen.bf16_bits_to_f32(gen.to_bf16_bits(a))) if dtype == "bf16" else (lambda a: a)
        want_p = rnd(D).astype(np.float64) @ rnd(Q0).astype(np.float64)
        assert np.abs(P_raw - want_p).max() <= 1e-6 * np.abs(want_p).max()
        want_q = rnd(D).astype(np.float64).T @ rnd(P_hat).astype(np.float64)
        assert np.abs(Q1 - want_q).max() <= 1e-6 * np.abs(want_q).max()
        # the orthonormalisation against NumPy's QR with the diagonal of R made positive
        Qn, Rn = np.linalg.qr(P_raw.astype(np.float64))
        Qn = Qn * np.sign(np.diag(Rn))
        assert np.abs(P_hat - Qn).max() <= 1e-5
