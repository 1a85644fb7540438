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
from gpu_util import ctx, rel_fro, to_dev, to_host

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
    element sampled (4096 bins) the oracle reads the whole buffer."""
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
    # every element sampled: the oracle reads the whole buffer
    host = to_host(x) if dtype == "bf16" else x.cpu().numpy()
    ref = orc.entropy(host, 1, 64, 0, 5, 4096)
    counts = torch.empty(4096, dtype=torch.int64, device="cuda")
    got = c.entropy_estimate(x, 1, 64, 0, 5, 4096, None, counts)
    assert (got.n_sampled, got.n_nonfinite, got.lo, got.hi) == (n, 0, ref.lo, ref.hi)
    assert np.array_equal(counts.cpu().numpy().astype(np.uint64), ref.counts)
    assert abs(got.H_bits - ref.H_bits) <= 1e-5 and abs(got.h_diff_nats - ref.h_diff_nats) <= 1e-5
    del x, host
    torch.cuda.empty_cache()


# ---------------------------------------------------------------------------
# hidden-5120 bf16 attention projection, rank 64, residual carried over three steps
# ---------------------------------------------------------------------------
def test_hidden5120_bf16_residual_carried_over_steps():
    m = n = 5120
    r = 64
    U, V = gen.orthonormal_factors(m, n, 512, 1)
    Q0 = np.zeros((n, r), dtype=np.float32)
    orc.init_q(Q0, 0, r, 0)
    c = ctx()
    Qd = to_dev(Q0); Pd = torch.empty((m, r), device="cuda")
    Ed = torch.empty((m, n), device="cuda"); out = torch.empty((m, n), dtype=torch.bfloat16, device="cuda")
    Qo, Eo = Q0, None
    for t in range(3):
        G = gen.lowrank_plus_noise(m, n, 512, 0.97, 1e-4, 1, "bf16", noise_seed=50 + t, factors=(U, V))
        Po, Qo, Do = orc.compress(G, Eo, Qo, r)
        out_o, Eo = orc.decompress(Po, Qo, Do, orc.BF16)
        Gd = to_dev(G)
        c.compress(Gd, Ed, t == 0, Qd, Pd, r)
        torch.cuda.synchronize()
        assert rel_fro(to_host(Ed), Do) <= 1e-2                  # D (exact at t = 0)
        c.decompress(Pd, Qd, r, Ed, out)
        torch.cuda.synchronize()
        assert rel_fro(to_host(Pd), Po) <= 1e-2 and rel_fro(to_host(Qd), Qo) <= 1e-2
        assert rel_fro(gen.bf16_bits_to_f32(to_host(out)), gen.bf16_bits_to_f32(out_o)) <= 1e-2
        assert np.linalg.norm(to_host(Ed).astype(np.float64) - Eo) <= 1e-2 * np.linalg.norm(Do.astype(np.float64))
        if t == 0:
            assert np.array_equal(to_host(Ed) + gen.bf16_bits_to_f32(to_host(out)), Do) or \
                rel_fro(to_host(Ed) + gen.bf16_bits_to_f32(to_host(out)), Do) < 1e-6


# ---------------------------------------------------------------------------
# dynamic-rate run on a hidden-256 replica of one pipeline stage: four layer gradients in
# one slab, spectrum decay ramping 0.90 -> 0.99 over 200 steps, entropy every step over a
# 20-step window, ranks in {4, 8, 16, 32, 64}; both sides run free (their own entropies,
# their own decisions, their own warm-started Q and residual)
# ---------------------------------------------------------------------------
def test_dynamic_rank_run_free_running():
    hidden, steps, window = 256, 200, 20
    shapes = [(hidden, 3 * hidden), (hidden, hidden), (hidden, 4 * hidden), (4 * hidden, hidden)]
    allowed = [4, 8, 16, 32, 64]
    r_max = 64
    prm = dict(m=hidden, n=hidden, r_min=4, r_max=r_max, step_limit=8, allowed=allowed, eta=1.0,
               total_iters=steps, min_warmup_frac=0.10, r_ref=4)
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
        decay = 0.90 + 0.09 * t / (steps - 1)
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
    assert ranks_seen == sorted(ranks_seen)         # entropy rises with the flattening spectrum


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
