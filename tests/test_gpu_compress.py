"""GPU parity: edgc_init_q / edgc_compress / edgc_decompress against the CPU oracle.

Bar: D = G + E_old bit-exact (one fp32 add); P^, Q, M^ and E_new within 1e-3
relative Frobenius error for fp32 gradients and 1e-2 for bf16 gradients;
D = out + E_new exact up to the fp32 subtraction."""
import numpy as np
import pytest
import torch

import edgc_inputs as gen
import paper_2511_10333_amd as edgc
from oracle import edgc_oracle as orc
from gpu_util import ctx, rel_fro, to_dev, to_host

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-3, "bf16": 1e-2}


def _q0(n, r, seed=0, ld=None):
    Q = np.zeros((n, ld or r), dtype=np.float32)
    orc.init_q(Q, 0, r, seed)
    return Q


def _pad4(r):
    return (r + 3) // 4 * 4


def gpu_compress(G, E, Q0, r, power_iters=1, ld=None):
    """Runs edgc_compress on host arrays; returns (P, Q, D) as numpy."""
    m, n = G.shape
    Gd = to_dev(G)
    if ld is not None and ld != n:                        # embed in a wider row-major buffer
        wide = torch.zeros((m, ld), dtype=Gd.dtype, device="cuda")
        wide[:, :n] = Gd
        Gd = wide[:, :n]
    Ed = torch.empty((m, n), dtype=torch.float32, device="cuda") if E is None else to_dev(E)
    if E is None:
        Ed.fill_(float("nan"))                            # must never be read
    ldq = _pad4(r)
    Qd = torch.zeros((n, ldq), dtype=torch.float32, device="cuda")
    Qd[:, :r] = to_dev(np.ascontiguousarray(Q0[:, :r]))
    Pd = torch.full((m, ldq), 7.0, dtype=torch.float32, device="cuda")
    ctx().compress(Gd, Ed, E is None, Qd, Pd, r, power_iters)
    torch.cuda.synchronize()
    return to_host(Pd)[:, :r], to_host(Qd)[:, :r], to_host(Ed), (Pd, Qd, Ed)


def gpu_decompress(P, Q, D, dtype, r):
    m, n = D.shape
    ldq = _pad4(r)
    Pd = torch.zeros((m, ldq), dtype=torch.float32, device="cuda"); Pd[:, :r] = to_dev(np.ascontiguousarray(P))
    Qd = torch.zeros((n, ldq), dtype=torch.float32, device="cuda"); Qd[:, :r] = to_dev(np.ascontiguousarray(Q))
    Ed = to_dev(D)
    out = torch.empty((m, n), dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device="cuda")
    ctx().decompress(Pd, Qd, r, Ed, out)
    torch.cuda.synchronize()
    return to_host(out), to_host(Ed)


def _widen(out):
    return gen.bf16_bits_to_f32(out) if out.dtype == np.uint16 else out


def check_step(G, E, Q0, r, dtype, power_iters=1, ld=None, compare_factors=True):
    tol = TOL[dtype]
    Po, Qo, Do = orc.compress(G, E, Q0, r, power_iters)
    Pg, Qg, Dg, _ = gpu_compress(G, E, Q0, r, power_iters, ld)
    assert np.array_equal(Dg, Do), "D = G + E_old must be bit-exact"
    if compare_factors:
        assert rel_fro(Pg, Po) <= tol, f"P^ off by {rel_fro(Pg, Po):.2e}"
        assert rel_fro(Qg, Qo) <= tol, f"Q off by {rel_fro(Qg, Qo):.2e}"
    code = orc.BF16 if dtype == "bf16" else orc.F32
    # the reconstruction kernel on the oracle's factors ...
    out_o, E_o = orc.decompress(Po, Qo, Do, code)
    out_k, E_k = gpu_decompress(Po, Qo, Do, dtype, r)
    assert rel_fro(_widen(out_k), _widen(out_o)) <= tol
    assert rel_fro(E_k, E_o) <= tol or np.linalg.norm(E_k - E_o) <= tol * np.linalg.norm(Do)
    assert np.array_equal(E_k, Do - _widen(out_k)), "E_new = D - M^ as transmitted"
    # ... and the whole chain on the GPU's own factors
    out_g, E_g = gpu_decompress(Pg, Qg, Dg, dtype, r)
    assert rel_fro(_widen(out_g), _widen(out_o)) <= tol
    assert np.linalg.norm(E_g.astype(np.float64) - E_o) <= tol * np.linalg.norm(Do.astype(np.float64))
    return Pg, Qg, out_g, E_g


def test_init_q_matches_oracle():
    n, r = 5000, 24
    want = _q0(n, r, seed=11, ld=24)
    Qd = torch.full((n, 24), -3.0, dtype=torch.float32, device="cuda")
    ctx().init_q(Qd, 0, 8, 11)
    ctx().init_q(Qd, 8, 24, 11)                            # grown later: same values
    torch.cuda.synchronize()
    got = to_host(Qd)
    # both sides evaluate Box-Muller in fp64 and round once to fp32; libm differences can
    # flip that rounding only for a handful of values
    ulp = np.abs(got - want) / np.maximum(np.spacing(np.abs(want)), 1e-45)
    assert ulp.max() <= 1.0 and (ulp > 0).mean() < 1e-3


def test_config1_square_matrix_rank4():
    (_, G), = gen.workload_matrices("cfg1_1024sq_r4")
    Pg, Qg, out, E = check_step(G, None, _q0(1024, 4), 4, "f32")
    P64 = Pg.astype(np.float64)
    assert np.abs(P64.T @ P64 - np.eye(4)).max() < 1e-5          # orthonormal columns
    assert np.abs(P64.T @ E.astype(np.float64)).max() < 1e-4 * np.linalg.norm(G)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("m,n,r", [(256, 384, 8), (130, 260, 5), (200, 330, 16), (64, 64, 32),
                                    (384, 256, 48), (512, 640, 64), (300, 1000, 100), (1024, 512, 128),
                                    (33, 1027, 3)])
def test_shapes_tiles_and_ragged_tails(dtype, m, n, r):
    G = gen.lowrank_plus_noise(m, n, min(m, n, 96), 0.93, 1e-4, seed=m + n, dtype=dtype)
    E = (1e-3 * np.random.default_rng(r).standard_normal((m, n))).astype(np.float32)
    check_step(G, E, _q0(n, r), r, dtype)


@pytest.mark.parametrize("r", [15, 17, 31, 33, 63, 65, 97, 127])
def test_ranks_next_to_the_tile_edges_of_the_factorisation(r):
    # one column short of, and one past, a whole number of the 16-column tiles the Gram matrix is
    # factored in (and of the 32-column rank tiles of the passes): the padding columns must stay out
    G = gen.lowrank_plus_noise(320, 448, 160, 0.97, 1e-3, seed=r)
    Pg, Qg, out, E = check_step(G, None, _q0(448, r), r, "f32")
    P64 = Pg.astype(np.float64)
    assert np.abs(P64.T @ P64 - np.eye(r)).max() < 1e-5


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_strided_gradient_rows(dtype):
    G = gen.lowrank_plus_noise(192, 320, 32, 0.9, 1e-4, seed=5, dtype=dtype)
    check_step(G, None, _q0(320, 8), 8, dtype, ld=352)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_error_feedback_carried_over_steps_with_warm_start(dtype):
    m, n, r, T = 256, 512, 16, 4
    U, V = gen.orthonormal_factors(m, n, 64, 3)
    Qo = Qg = _q0(n, r)
    Eo = Eg = None
    code = orc.BF16 if dtype == "bf16" else orc.F32
    for t in range(T):
        G = gen.lowrank_plus_noise(m, n, 64, 0.9, 1e-3, seed=3, dtype=dtype, noise_seed=100 + t,
                                   factors=(U, V))
        Po, Qo, Do = orc.compress(G, Eo, Qo, r)
        out_o, Eo = orc.decompress(Po, Qo, Do, code)
        Pg, Qg, Dg, _ = gpu_compress(G, Eg, Qg, r)
        out_g, Eg = gpu_decompress(Pg, Qg, Dg, dtype, r)
        tol = TOL[dtype]
        assert rel_fro(Dg, Do) <= tol and rel_fro(Pg, Po) <= tol and rel_fro(Qg, Qo) <= tol
        assert rel_fro(_widen(out_g), _widen(out_o)) <= tol
        assert np.array_equal(Eg, Dg - _widen(out_g))


def test_exact_rank_r_matrix_is_reconstructed_on_device():
    M = gen.exact_rank(256, 384, 8, seed=2)
    Pg, Qg, out, E = check_step(M, None, _q0(384, 8), 8, "f32")
    assert rel_fro(out, M) < 1e-4      # two bf16 planes keep ~17 bits per operand


def test_rank_deficient_input_compares_reconstruction_only():
    # rank 3 matrix compressed at rank 8: trailing columns are orthogonalised noise, several
    # factorisations are valid; only M^ and the residual are unique
    M = gen.exact_rank(192, 256, 3, seed=4)
    check_step(M, None, _q0(256, 8), 8, "f32", compare_factors=False)


@pytest.mark.parametrize("m,n,r,dups", [
    # (column, the earlier column it repeats): in several blocks of four pivots and several 16-column tiles,
    # the last column among them
    (256, 320, 48, [(5, 2), (17, 3), (18, 16), (33, 1), (47, 40)]),
    (512, 640, 128, [(3, 0), (16, 15), (63, 20), (64, 63 - 1), (100, 99), (126, 7), (127, 125)]),
    (384, 256, 100, [(31, 30), (32, 31 - 1), (96, 50), (99, 98)]),
])
def test_repeated_start_columns_are_removed_and_the_rest_is_the_smaller_problem(m, n, r, dups):
    # Q0 with columns that repeat earlier ones: P = D Q0 has exactly dependent columns, whose pivots
    # the orthonormalisation must find zero.  Those columns of P^ and Q are exact zeros, and what is
    # left is the step at the smaller rank with the repeats taken out, which the oracle computes
    # (it would normalise the rounding noise a repeat leaves behind, a valid but different factor).
    G = gen.lowrank_plus_noise(m, n, 3 * r // 2, 0.97, 1e-3, seed=21)
    Q0 = _q0(n, r, seed=5)
    for c, o in dups:
        Q0[:, c] = Q0[:, o]
    dead = sorted(c for c, _ in dups)
    live = [c for c in range(r) if c not in dead]
    Pg, Qg, Dg, _ = gpu_compress(G, None, Q0, r)
    assert not Pg[:, dead].any() and not Qg[:, dead].any(), "a repeated column leaves a zero column in P^ and Q"
    Po, Qo, Do = orc.compress(G, None, np.ascontiguousarray(Q0[:, live]), len(live), 1)
    assert np.array_equal(Dg, Do)
    tol = TOL["f32"]
    assert rel_fro(Pg[:, live], Po) <= tol, f"P^ off by {rel_fro(Pg[:, live], Po):.2e}"
    assert rel_fro(Qg[:, live], Qo) <= tol, f"Q off by {rel_fro(Qg[:, live], Qo):.2e}"
    gram = Pg[:, live].astype(np.float64).T @ Pg[:, live].astype(np.float64)
    assert np.abs(gram - np.eye(len(live))).max() < 1e-5
    out_o, E_o = orc.decompress(Po, Qo, Do, orc.F32)
    out_g, E_g = gpu_decompress(Pg, Qg, Dg, "f32", r)
    assert rel_fro(out_g, out_o) <= tol
    assert np.array_equal(E_g, Dg - out_g)


def test_zero_matrix():
    Z = np.zeros((128, 192), dtype=np.float32)
    Pg, Qg, Dg, _ = gpu_compress(Z, None, _q0(192, 4), 4)
    assert not Pg.any() and not Qg.any() and not Dg.any()
    out, E = gpu_decompress(Pg, Qg, Dg, "f32", 4)
    assert not out.any() and not E.any()


def test_two_power_iterations():
    G = gen.lowrank_plus_noise(256, 320, 48, 0.85, 1e-3, seed=6)
    check_step(G, None, _q0(320, 6), 6, "f32", power_iters=2)


def test_rank_change_keeps_residual_and_leading_columns():
    m, n = 256, 384
    G = gen.lowrank_plus_noise(m, n, 64, 0.92, 1e-3, seed=7)
    Q8 = _q0(n, 8)
    Po, Qo, Do = orc.compress(G, None, Q8, 8)
    _, Eo = orc.decompress(Po, Qo, Do, orc.F32)
    # grow to rank 16: old columns kept, new ones from the seeded generator
    Q16 = _q0(n, 16)
    Q16[:, :8] = Qo
    G2 = gen.lowrank_plus_noise(m, n, 64, 0.92, 1e-3, seed=7, noise_seed=99)
    check_step(G2, Eo, Q16, 16, "f32")
    # shrink to rank 4: first columns only
    check_step(G2, Eo, Qo[:, :4].copy(), 4, "f32")


def test_bad_arguments_rejected_before_launch():
    c = ctx()
    G = torch.zeros((64, 96), device="cuda")
    E = torch.zeros((64, 96), device="cuda")
    Q = torch.zeros((96, 8), device="cuda")
    P = torch.zeros((64, 8), device="cuda")
    for r, it in [(0, 1), (65, 1), (8, 0)]:
        Qr = torch.zeros((96, max(_pad4(r), 4)), device="cuda")
        Pr = torch.zeros((64, max(_pad4(r), 4)), device="cuda")
        with pytest.raises(edgc.EdgcError) as e:
            c.compress(G, E, True, Qr, Pr, r, it)
        assert e.value.code == edgc.binding.EINVAL
    with pytest.raises(edgc.EdgcError):                    # ldq < r
        c.compress(G, E, True, Q, P, 12, 1)
    with pytest.raises(edgc.EdgcError):                    # larger than the context
        big = edgc.Context(0, 256, 16, 32, 32)
        big.compress(G, E, True, Q, P, 8, 1)
    with pytest.raises(edgc.EdgcError):                    # rank above the context's max_rank
        small = edgc.Context(0, 256, 4, 64, 96)
        small.compress(G, E, True, Q, P, 8, 1)
    # rows, columns and leading dimensions stop at 2^28 (the kernels keep lane offsets in 32 bits)
    # (straight through the C ABI: torch does not build a view with such a stride)
    L, EINVAL, big_ld = c._L, edgc.binding.EINVAL, (1 << 28) + 4
    assert L.edgc_compress(c._h, G.data_ptr(), edgc.F32, 64, 96, big_ld, E.data_ptr(), 1, Q.data_ptr(), 8,
                           P.data_ptr(), 8, 8, 1, None) == EINVAL
    assert L.edgc_decompress(c._h, P.data_ptr(), 8, Q.data_ptr(), 8, 64, 96, 8, E.data_ptr(), G.data_ptr(),
                             edgc.F32, big_ld, None) == EINVAL
    with pytest.raises(edgc.EdgcError):
        edgc.Context(0, 256, 16, (1 << 28) + 1, 64)
    with pytest.raises(edgc.EdgcError) as e:
        c.reserve_batch([((1 << 28) + 1, 64)])
    assert e.value.code == edgc.binding.EINVAL
    c.reserve_batch([(64, 96)])
    desc = (edgc.binding._Tensor * 1)()
    desc[0] = edgc.binding._Tensor(G.data_ptr(), G.data_ptr(), E.data_ptr(), Q.data_ptr(), P.data_ptr(),
                                   big_ld, 96, 64, 96, 8, 8, 1, 0)
    assert L.edgc_compress_batch(c._h, desc, 1, edgc.F32, 8, 1, None) == EINVAL
    desc[0].ld, desc[0].ld_out = 96, big_ld
    assert L.edgc_decompress_batch(c._h, desc, 1, edgc.F32, 8, None) == EINVAL


@pytest.mark.parametrize("name", ["cfg2_gpt_h2048_r16"])
def test_benchmark_workload_full_size(name):
    w = gen.WORKLOADS[name]
    for spec, G in gen.workload_matrices(name):
        check_step(G, None, _q0(spec.n, w["rank"]), w["rank"], w["dtype"])


@pytest.mark.parametrize("r", [32, 128])
def test_hidden5120_bf16_attention_projection_full_size(r):
    w = gen.WORKLOADS["cfg4_gpt_h5120_bf16"]
    G = gen.lowrank_plus_noise(5120, 5120, 512, w["decay"], w["noise"], 1, "bf16")
    check_step(G, None, _q0(5120, r), r, "bf16")


# ---------------------------------------------------------------------------
# rank-cost measurement (Sec. IV-D-1): the call runs the same two entry points, so what it
# leaves behind is one more valid step at the last rank; times are positive and sane
# ---------------------------------------------------------------------------
def test_measure_rank_costs_runs_the_two_calls_and_reports_bytes():
    m, n, ranks = 512, 768, [4, 8, 16, 32]
    g = gen.lowrank_plus_noise(m, n, 64, 0.9, 1e-4, 3)
    c = ctx()
    gd = to_dev(g)
    res, out = torch.empty((m, n), device="cuda"), torch.empty((m, n), device="cuda")
    Q, P = torch.empty((n, 32), device="cuda"), torch.empty((m, 32), device="cuda")
    costs = c.measure_rank_costs(gd, res, Q, P, out, ranks, reps=3)
    torch.cuda.synchronize()
    assert [k.rank for k in costs] == ranks
    for k in costs:
        assert 1e-6 < k.t_compress < 5e-3 and 1e-6 < k.t_decompress < 5e-3
        assert k.bytes_compressed == 4.0 * (m + n) * k.rank
    # the buffers hold the last round at rank 32: P orthonormal, out + E = D, and the
    # error-feedback sum over the 1 + 3 rounds since the residual was reset
    Ph = to_host(P).astype(np.float64)
    assert np.abs(Ph.T @ Ph - np.eye(32)).max() <= 1e-4
    # ... and they equal what the same sequence of plain calls leaves (one untimed round from
    # a zero residual and seeded Q columns, then three more)
    res2, out2 = torch.empty_like(res), torch.empty_like(out)
    Q2, P2 = torch.empty_like(Q), torch.empty_like(P)
    c.init_q(Q2, 0, 32, 0x5EED + 32)
    for rep in range(4):
        c.compress(gd, res2, rep == 0, Q2, P2, 32)
        c.decompress(P2, Q2, 32, res2, out2)
    torch.cuda.synchronize()
    assert torch.equal(res, res2) and torch.equal(out, out2) and torch.equal(P, P2) and torch.equal(Q, Q2)
    # the deferred form leaves the same factors and reconstruction, and D where the other leaves E;
    # its decompress only writes, so it is the cheaper of the two
    res3, out3 = torch.empty_like(res), torch.empty_like(out)
    Q3, P3 = torch.empty_like(Q), torch.empty_like(P)
    costs_d = c.measure_rank_costs(gd, res3, Q3, P3, out3, ranks, reps=3, deferred=True)
    torch.cuda.synchronize()
    assert torch.equal(out3, out) and torch.equal(P3, P) and torch.equal(Q3, Q)
    assert torch.equal(res3 - out3, res)
    assert all(1e-6 < k.t_decompress < 5e-3 and 1e-6 < k.t_compress < 5e-3 for k in costs_d)
    with pytest.raises(edgc.EdgcError):
        c.measure_rank_costs(gd, res, Q, P, gd, ranks, reps=3)           # aliasing refused
    with pytest.raises(edgc.EdgcError):
        c.measure_rank_costs(gd, res, Q, P, out, ranks, reps=0)
    with pytest.raises(edgc.EdgcError):
        c.measure_rank_costs(gd, res, Q, P, out, [8, 4], reps=1)


# ---------------------------------------------------------------------------
# measured device ceilings: the copy really copies, the figures are in a physical range, and
# bad arguments are refused before any launch
# ---------------------------------------------------------------------------
def test_measure_device_peaks_copies_and_reports_physical_figures():
    c = ctx()
    a = torch.randn(1 << 26, device="cuda")                 # 256 MiB
    b = torch.zeros_like(a)
    # after the call buf_b holds the copy of buf_a, except at its start, where the read and the
    # MFMA kernel left one float per thread (8 blocks per compute unit of 256 threads)
    pk = c.measure_device_peaks(a, b, reps=3)
    sink_floats = 8 * 256 * 256
    assert torch.equal(a[sink_floats:], b[sink_floats:])
    assert pk["bytes"] == a.numel() * 4
    assert 500.0 < pk["read_gbs"] < 20000.0 and 500.0 < pk["copy_gbs"] < 20000.0
    assert 500.0 < pk["write_gbs"] < 20000.0
    assert 100.0 < pk["mfma_bf16_tflops"] < 2600.0
    with pytest.raises(edgc.EdgcError):
        c.measure_device_peaks(a, a, reps=3)
    with pytest.raises(edgc.EdgcError):
        c.measure_device_peaks(a[:1024], b[:1024], reps=3)         # below the minimum size
    with pytest.raises(edgc.EdgcError):
        c.measure_device_peaks(a[1:1 + (1 << 22)], b[: 1 << 22], reps=3)   # misaligned
    with pytest.raises(edgc.EdgcError):
        c.measure_device_peaks(a, b, reps=0)
