"""GPU parity at the workload configurations: the large flat-buffer entropy sweep, a bf16
layer with the residual carried over steps at full size, and the dynamic-rate run
(entropy window -> rank, rank changes between steps with the residual preserved)."""
import math

import numpy as np
import pytest
import torch

import edgc_inputs as gen
import paper_2511_10333_amd as edgc
from oracle import edgc_oracle as orc
from gpu_util import ELEMENTWISE_TOL, ctx, elementwise_ratio, rel_fro, to_dev, to_host

pytestmark = pytest.mark.gpu


# ---------------------------------------------------------------------------
# entropy-only sweep on a flat Laplace-mixture buffer (a 2^26-element slice of the
# 1e9-element workload: same distribution, strides and bin counts)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_flat_buffer_entropy_sweep(dtype):
    n = (1 << 26) + 17
    x = gen.laplace_mixture(n, seed=0, dtype=dtype)
    xd = to_dev(x)
    c = ctx()
    for stride in (1000, 100, 10, 1):
        for bins in (256, 4096, 65536):
            ref = orc.entropy(x, stride, 64, 0, 5, bins)
            counts = torch.empty(bins, dtype=torch.int64, device="cuda")
            got = c.entropy_estimate(xd, stride, 64, 0, 5, bins, None, counts)
            assert (got.n_sampled, got.n_nonfinite, got.lo, got.hi) == (ref.n_sampled, 0, ref.lo, ref.hi)
            assert np.array_equal(counts.cpu().numpy().astype(np.uint64), ref.counts), (stride, bins)
            assert abs(got.H_bits - ref.H_bits) <= 1e-5 and abs(got.h_diff_nats - ref.h_diff_nats) <= 1e-5


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_flat_buffer_of_1e9_elements_sampled(dtype):
    """The flat buffer at its full size of 1e9 elements (generated on the device: Laplace(0, 1e-3)
    with 0.1 % of the values at 100 times the scale).  The oracle gets the sample: its own index
    set gathers the sampled elements, and its estimator runs over them with every element taken;
    counts are compared bit for bit, at strides 1000, 100 and 10 on three bin counts; with every
    element sampled the oracle reads the whole buffer (256, 4096 and 65536 bins)."""
    n = 1_000_000_000
    g = torch.Generator(device="cuda").manual_seed(3)
    x = torch.empty(n, device="cuda")
    x.exponential_(1.0, generator=g)                                   # |Laplace(0, 1)|
    sign = torch.empty(n, device="cuda").uniform_(-1.0, 1.0, generator=g)
    x.mul_(torch.sign(sign))
    x.mul_(torch.where(sign.abs() < 1e-3, 1e-1, 1e-3))                 # 0.1 % outliers at 100 x scale
    del sign
    if dtype == "bf16":
        x = x.bfloat16()
    c = ctx()
    for stride in (1000, 100, 10):
        idx = torch.from_numpy(orc.sample_indices(n, stride, 64, 0, 5).astype(np.int64)).cuda()
        sample = x[idx]
        del idx
        host = to_host(sample) if dtype == "bf16" else sample.cpu().numpy()
        del sample
        for bins in (256, 4096, 65536):
            ref = orc.entropy(host, 1, 1, 0, 0, bins)
            counts = torch.empty(bins, dtype=torch.int64, device="cuda")
            got = c.entropy_estimate(x, stride, 64, 0, 5, bins, None, counts)
            assert (got.n_sampled, got.n_nonfinite, got.lo, got.hi) == (ref.n_sampled, 0, ref.lo, ref.hi)
            assert got.n_sampled == host.size
            assert np.array_equal(counts.cpu().numpy().astype(np.uint64), ref.counts), (stride, bins)
            assert abs(got.H_bits - ref.H_bits) <= 1e-5 and abs(got.h_diff_nats - ref.h_diff_nats) <= 1e-5
    # every element sampled: the oracle reads the whole buffer, on all three bin counts (65536 bins: the
    # histogram no longer fits one LDS slice)
    host = to_host(x) if dtype == "bf16" else x.cpu().numpy()
    for bins in (256, 4096, 65536):
        ref = orc.entropy(host, 1, 64, 0, 5, bins)
        counts = torch.empty(bins, dtype=torch.int64, device="cuda")
        got = c.entropy_estimate(x, 1, 64, 0, 5, bins, None, counts)
        assert (got.n_sampled, got.n_nonfinite, got.lo, got.hi) == (n, 0, ref.lo, ref.hi), bins
        assert np.array_equal(counts.cpu().numpy().astype(np.uint64), ref.counts), bins
        assert abs(got.H_bits - ref.H_bits) <= 1e-5 and abs(got.h_diff_nats - ref.h_diff_nats) <= 1e-5, bins
    del x, host
    torch.cuda.empty_cache()


# ---------------------------------------------------------------------------
# hidden-5120 bf16 attention projection at ranks 32, 64 and 128: the same low-rank part with fresh
# noise every step, the error-feedback residual carried across 10 steps.  Every step the device path
# is run from the ORACLE's carried state (its residual and warm-started Q) and held to the one-step
# bar; the device's own chain runs beside it and is checked for what stays unique on a free run:
# D of the first step, error-feedback conservation and the size of the residual.  (At rank 128 the
# spectrum 0.97^i leaves the trailing directions of the subspace nearly degenerate: two free runs
# settle on slightly different bases, P of the two chains is 1.1e-2 apart after ten steps.)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("r", [32, 64, 128])
def test_hidden5120_bf16_residual_carried_over_ten_steps(r):
    m = n = 5120
    steps, tol = 10, 1e-2
    U, V = gen.orthonormal_factors(m, n, 512, 1)
    Q0 = np.zeros((n, r), dtype=np.float32)
    orc.init_q(Q0, 0, r, 0)
    c = ctx()
    Qd = to_dev(Q0); Pd = torch.empty((m, r), device="cuda")
    Ed = torch.empty((m, n), device="cuda"); out = torch.empty((m, n), dtype=torch.bfloat16, device="cuda")
    Pt = torch.empty((m, r), device="cuda"); ot = torch.empty((m, n), dtype=torch.bfloat16, device="cuda")
    Qo, Eo = Q0, None
    sumG = np.zeros((m, n)); sum_out = torch.zeros((m, n), dtype=torch.float64, device="cuda")
    for t in range(steps):
        G = gen.lowrank_plus_noise(m, n, 512, 0.97, 1e-4, 1, "bf16", noise_seed=50 + t, factors=(U, V))
        Gd = to_dev(G)
        E_prev, Q_prev = Eo, Qo
        Po, Qo, Do = orc.compress(G, E_prev, Q_prev, r)
        out_o, Eo = orc.decompress(Po, Qo, Do, orc.BF16)
        nD = np.linalg.norm(Do.astype(np.float64))
        # one step of the device path from the oracle's state
        Et = torch.empty((m, n), device="cuda") if E_prev is None else to_dev(E_prev)
        Qt = to_dev(Q_prev)
        c.compress(Gd, Et, E_prev is None, Qt, Pt, r)
        torch.cuda.synchronize()
        assert np.array_equal(to_host(Et), Do), t                  # D = G + E_old: one fp32 add
        c.decompress(Pt, Qt, r, Et, ot)
        torch.cuda.synchronize()
        assert rel_fro(to_host(Pt), Po) <= tol and rel_fro(to_host(Qt), Qo) <= tol, t
        got = gen.bf16_bits_to_f32(to_host(ot))
        assert rel_fro(got, gen.bf16_bits_to_f32(out_o)) <= tol, t
        assert elementwise_ratio(got, gen.bf16_bits_to_f32(out_o), Po, Qo) <= ELEMENTWISE_TOL["bf16"], t
        assert np.linalg.norm(to_host(Et).astype(np.float64) - Eo) <= tol * nD, t
        # the device's own chain
        c.compress(Gd, Ed, t == 0, Qd, Pd, r)
        if t == 0:
            torch.cuda.synchronize()
            assert np.array_equal(to_host(Ed), Do)
        c.decompress(Pd, Qd, r, Ed, out)
        torch.cuda.synchronize()
        sumG += gen.bf16_bits_to_f32(G)
        sum_out += out.double()
        if t in (0, steps - 1):
            Eg = to_host(Ed).astype(np.float64)
            lost = sumG - sum_out.cpu().numpy() - Eg
            assert np.linalg.norm(lost) <= 1e-5 * np.linalg.norm(sumG), t
            assert abs(np.linalg.norm(Eg) - np.linalg.norm(Eo.astype(np.float64))) <= 0.05 * nD, t
            assert rel_fro(gen.bf16_bits_to_f32(to_host(out)), gen.bf16_bits_to_f32(out_o)) <= 3 * tol, t


# ---------------------------------------------------------------------------
# dynamic-rate run on a hidden-256 replica of one pipeline stage: four layer gradients in
# one slab, spectrum decay ramping 0.90 -> 0.99 over 200 steps, entropy every step over a
# 20-step window, ranks in {4, 8, 16, 32, 64}; both sides run free (their own entropies,
# their own decisions, their own warm-started Q and residual)
# ---------------------------------------------------------------------------
# Two runs: the configuration's own ramp 0.90 -> 0.99 on a hidden-256 replica (the entropy rises, so the
# reference rank of Theorem 3 is set to r_min: with the paper's r0 = r_max such a run never leaves
# warm-up), and the ramp reversed, 0.99 -> 0.90, on a hidden-512 replica with the paper's own rule
# (r_ref = 0, i.e. r0 = r_max): the entropy falls and the rank comes down from r_max.
@pytest.mark.parametrize("hidden,d0,d1,r_ref", [(256, 0.90, 0.99, 4), (512, 0.99, 0.90, 0)])
def test_dynamic_rank_run_free_running(hidden, d0, d1, r_ref):
    steps, window = 200, 20
    shapes = [(hidden, 3 * hidden), (hidden, hidden), (hidden, 4 * hidden), (4 * hidden, hidden)]
    allowed = [4, 8, 16, 32, 64]
    r_max = 64
    prm = dict(m=hidden, n=hidden, r_min=4, r_max=r_max, step_limit=8, allowed=allowed, eta=1.0,
               total_iters=steps, min_warmup_frac=0.10, r_ref=r_ref)
    factors = [gen.orthonormal_factors(m, n, min(m, n), 30 + i) for i, (m, n) in enumerate(shapes)]
    sizes = [m * n for m, n in shapes]
    offs = np.concatenate([[0], np.cumsum(sizes)])
    c = ctx()
    slab = torch.empty(int(offs[-1]), device="cuda")
    layer_views = [slab[int(offs[i]):int(offs[i + 1])].view(m, n) for i, (m, n) in enumerate(shapes)]

    st_o, st_g = orc.RankState(), edgc.RankState()
    rank_o = rank_g = 0
    Hwin_o, Hwin_g = [], []
    Q_o = [np.zeros((n, r_max), dtype=np.float32) for _, n in shapes]
    for i, q in enumerate(Q_o):
        orc.init_q(q, 0, r_max, 100 + i)
    Q_g = [to_dev(q) for q in Q_o]
    P_g = [torch.empty((m, r_max), device="cuda") for m, _ in shapes]
    E_o = [None] * len(shapes)
    E_g = [torch.empty((m, n), device="cuda") for m, n in shapes]
    fresh = [True] * len(shapes)
    out_g = [torch.empty((m, n), device="cuda") for m, n in shapes]
    sumG = [np.zeros((m, n)) for m, n in shapes]
    sum_out = [torch.zeros((m, n), device="cuda", dtype=torch.float64) for m, n in shapes]
    ranks_seen = []
    for t in range(steps):
        decay = d0 + (d1 - d0) * t / (steps - 1)
        host = np.empty(int(offs[-1]), dtype=np.float32)
        for i, (m, n) in enumerate(shapes):
            g = gen.lowrank_plus_noise(m, n, min(m, n), decay, 1e-4, 7, noise_seed=1000 * i + t, factors=factors[i])
            host[int(offs[i]):int(offs[i + 1])] = g.reshape(-1)
        slab.copy_(torch.from_numpy(host))
        # entropy of the stage slab (every iteration: alpha = 1)
        e_o = orc.entropy(host, 100, 64, 3, t, 1024)
        e_g = c.entropy_estimate(slab, 100, 64, 3, t, 1024)
        assert abs(e_g.h_diff_nats - e_o.h_diff_nats) <= 1e-5 and e_g.n_sampled == e_o.n_sampled
        Hwin_o.append(e_o.h_diff_nats); Hwin_g.append(e_g.h_diff_nats)
        # compress / decompress every layer at the current rank (0 = warm-up: uncompressed)
        assert rank_o == rank_g
        if rank_o:
            r = rank_o
            check = (t % 10 == 9) or t == steps - 1 or (t % window == 0)
            for i, (m, n) in enumerate(shapes):
                G = host[int(offs[i]):int(offs[i + 1])].reshape(m, n)
                E_prev, Q_prev = E_o[i], Q_o[i][:, :r].copy()
                Po, Qn, Do = orc.compress(G, E_prev, Q_prev, r)
                Q_o[i][:, :r] = Qn
                out_o, E_o[i] = orc.decompress(Po, Qn, Do, orc.F32)
                c.compress(layer_views[i], E_g[i], fresh[i], Q_g[i], P_g[i], r)
                c.decompress(P_g[i], Q_g[i], r, E_g[i], out_g[i])
                fresh[i] = False
                sumG[i] += G
                sum_out[i] += out_g[i].double()
                if check:
                    torch.cuda.synchronize()
                    # free-running: with a slowly decaying spectrum the trailing directions of the
                    # rank-r subspace are nearly degenerate and the residual feeds back, so the two
                    # runs settle on different (equally valid) bases and drift apart; what stays
                    # unique is error-feedback conservation: everything the gradients carried is
                    # either in an output already or still in the residual
                    Eg = to_host(E_g[i]).astype(np.float64)
                    nD = np.linalg.norm(Do.astype(np.float64))
                    lost = sumG[i] - sum_out[i].cpu().numpy() - Eg
                    assert np.linalg.norm(lost) <= 1e-5 * np.linalg.norm(sumG[i]), (t, i, r)
                    # and the approximation quality stays comparable
                    assert abs(np.linalg.norm(Eg) - np.linalg.norm(E_o[i].astype(np.float64))) <= 0.1 * nD, (t, i, r)
                    # one step of the device path from the ORACLE's state: the one-step bar
                    Et = torch.empty((m, n), device="cuda") if E_prev is None else to_dev(E_prev)
                    Qt = torch.zeros((n, r_max), device="cuda"); Qt[:, :r] = to_dev(Q_prev)
                    Pt = torch.empty((m, r_max), device="cuda"); ot = torch.empty((m, n), device="cuda")
                    c.compress(layer_views[i], Et, E_prev is None, Qt, Pt, r)
                    c.decompress(Pt, Qt, r, Et, ot)
                    torch.cuda.synchronize()
                    assert rel_fro(to_host(Pt)[:, :r], Po) <= 1e-3 and rel_fro(to_host(Qt)[:, :r], Qn) <= 1e-3, (t, i, r)
                    assert rel_fro(to_host(ot), out_o) <= 1e-3, (t, i, r)
                    assert np.linalg.norm(to_host(Et).astype(np.float64) - E_o[i]) <= \
                        1e-3 * np.linalg.norm(Do.astype(np.float64)), (t, i, r)
        # window boundary: rank for the next window from this window's entropies
        if (t + 1) % window == 0:
            d_o = orc.select_rank(st_o, Hwin_o, window, orc.RankParams(**prm))
            d_g = edgc.select_rank(st_g, Hwin_g, window, edgc.RankParams(**prm))
            assert (d_o.rank, d_o.r_unclamped) == (d_g.rank, d_g.r_unclamped)
            rank_o, rank_g = d_o.rank, d_g.rank
            ranks_seen.append(rank_o)
            Hwin_o, Hwin_g = [], []
    torch.cuda.synchronize()
    assert ranks_seen[0] == 0                       # first window only fixes the reference
    assert len(set(r for r in ranks_seen if r)) >= 3, ranks_seen     # the rank really changed
    if d1 > d0:
        assert ranks_seen == sorted(ranks_seen)     # entropy rises with the flattening spectrum
    else:                                           # entropy falls: down from r_max once warm-up is over
        live = [r for r in ranks_seen if r]
        assert live[0] == r_max and live == sorted(live, reverse=True), ranks_seen


# ---------------------------------------------------------------------------
# layers of the dynamic-rate configuration at their real size (hidden 4096: attention projection
# and the two MLP matrices), across its rank range: step 0 from a zero residual, then one step
# from the ORACLE's residual and warm-started Q (teacher-forced), as the 200-step run at
# reduced size does at every check point
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("m,n,r", [(4096, 4096, 4), (4096, 4096, 64), (4096, 16384, 64), (16384, 4096, 32)])
def test_hidden4096_layer_full_size_teacher_forced(m, n, r):
    c = ctx()
    factors = gen.orthonormal_factors(m, n, 256, 77)
    Q0 = np.zeros((n, 64), dtype=np.float32)
    orc.init_q(Q0, 0, 64, 5)
    E_prev, Q_prev = None, np.ascontiguousarray(Q0[:, :r])
    for t, decay in enumerate((0.90, 0.99)):
        G = gen.lowrank_plus_noise(m, n, 256, decay, 1e-4, 7, noise_seed=900 + t, factors=factors)
        Po, Qn, Do = orc.compress(G, E_prev, Q_prev, r)
        out_o, E_o = orc.decompress(Po, Qn, Do, orc.F32)
        Gd = to_dev(G)
        Ed = torch.empty((m, n), device="cuda") if E_prev is None else to_dev(E_prev)
        Qd = torch.zeros((n, 64), device="cuda"); Qd[:, :r] = to_dev(Q_prev)
        Pd = torch.empty((m, 64), device="cuda"); out = torch.empty((m, n), device="cuda")
        c.compress(Gd, Ed, E_prev is None, Qd, Pd, r)
        assert np.array_equal(to_host(Ed), Do)
        c.decompress(Pd, Qd, r, Ed, out)
        torch.cuda.synchronize()
        assert rel_fro(to_host(Pd)[:, :r], Po) <= 1e-3 and rel_fro(to_host(Qd)[:, :r], Qn) <= 1e-3, (t, r)
        assert rel_fro(to_host(out), out_o) <= 1e-3, (t, r)
        assert np.linalg.norm(to_host(Ed).astype(np.float64) - E_o) <= 1e-3 * np.linalg.norm(Do.astype(np.float64))
        E_prev, Q_prev = E_o, Qn


# ---------------------------------------------------------------------------
# A rank change at the real layer size, from the ORACLE's state, through the calls a trainer makes:
# the deferred state of a step (D, P^, Q of the oracle) is loaded into the device buffers,
# edgc_residual_materialize_batch carries the subtraction out at the old rank, edgc_init_q seeds the
# columns a larger rank adds (a smaller rank keeps the leading ones), and the step at the new rank is
# compared with the oracle's step from its own residual and factors: the residual survives the change.
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("m,n,r1,r2", [(4096, 4096, 8, 16), (4096, 16384, 32, 64), (16384, 4096, 64, 32)])
def test_hidden4096_rank_change_full_size_teacher_forced(m, n, r1, r2):
    tol, ld, seed = 1e-3, 64, 5
    factors = gen.orthonormal_factors(m, n, 256, 77)
    Q0 = np.zeros((n, ld), dtype=np.float32)
    orc.init_q(Q0, 0, ld, seed)
    GA = gen.lowrank_plus_noise(m, n, 256, 0.90, 1e-4, 7, noise_seed=901, factors=factors)
    GB = gen.lowrank_plus_noise(m, n, 256, 0.95, 1e-4, 7, noise_seed=902, factors=factors)
    PA, QA, DA = orc.compress(GA, None, np.ascontiguousarray(Q0[:, :r1]), r1)
    _, EA = orc.decompress(PA, QA, DA, orc.F32)
    # the oracle's step at the new rank
    if r2 > r1:
        Qb = np.concatenate([QA, Q0[:, r1:r2]], axis=1)          # old columns kept, new ones seeded
    else:
        Qb = np.ascontiguousarray(QA[:, :r2])
    PB, QB, DB = orc.compress(GB, EA, Qb, r2)
    outB, EB = orc.decompress(PB, QB, DB, orc.F32)
    # the device: deferred state of step A in the buffers
    c = edgc.Context(0, max_bins=16, max_rank=ld, max_rows=64, max_cols=64)
    c.reserve_batch([(m, n)])
    res = to_dev(DA)
    Pd = torch.zeros((m, ld), device="cuda"); Pd[:, :r1] = to_dev(PA)
    Qd = torch.full((n, ld), float("nan"), device="cuda"); Qd[:, :r1] = to_dev(QA)
    out = torch.empty((m, n), device="cuda")
    ts = [edgc.Tensor(to_dev(GB), out, res, Qd, Pd, False)]
    c.residual_materialize_batch(ts, r1)
    torch.cuda.synchronize()
    nDA = np.linalg.norm(DA.astype(np.float64))
    assert np.linalg.norm(to_host(res).astype(np.float64) - EA) <= tol * nDA
    if r2 > r1:
        c.init_q(Qd, r1, r2, seed)
        torch.cuda.synchronize()
        assert rel_fro(to_host(Qd)[:, r1:r2], Q0[:, r1:r2]) <= 1e-6
    c.compress_batch(ts, r2, deferred=False)                     # the buffer holds E itself now
    torch.cuda.synchronize()
    assert rel_fro(to_host(res), DB) <= tol
    c.decompress_batch(ts, r2, deferred=True)
    torch.cuda.synchronize()
    assert rel_fro(to_host(Pd)[:, :r2], PB) <= tol and rel_fro(to_host(Qd)[:, :r2], QB) <= tol
    assert rel_fro(to_host(out), outB) <= tol
    assert elementwise_ratio(to_host(out), outB, PB, QB) <= ELEMENTWISE_TOL["f32"]
    c.close()
