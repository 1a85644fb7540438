"""The compress in two phases (edgc_compress_p_batch, edgc_compress_q_batch): equal to the fused
call bit for bit, and — with the factors of two gradient shards averaged between the phases, the
way a data-parallel step exchanges them (Sec. II-B) — equal to the oracle's plain step on the
averaged gradient."""
import numpy as np
import pytest
import torch

import edgc_inputs as gen
import paper_2511_10333_amd as edgc
from oracle import edgc_oracle as orc
from gpu_util import rel_fro, to_dev, to_host
from test_gpu_batch import MIXED, Stage

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("deferred", [False, True])
@pytest.mark.parametrize("r", [8, 48, 128])
def test_two_phases_equal_the_fused_call_bit_for_bit(dtype, deferred, r):
    fused = Stage(MIXED, r, dtype, seed=5, deferred=deferred)
    split = Stage(MIXED, r, dtype, seed=5, deferred=deferred)
    for step in range(3):
        fused.step_device()
        split.ctx.compress_p_batch(split.t, r, deferred=deferred and step > 0)
        split.ctx.compress_q_batch(split.t, r)
        split.ctx.decompress_batch(split.t, r, deferred=deferred)
        torch.cuda.synchronize()
        for t in split.t:
            t.residual_is_zero = False
        for i, (a, b) in enumerate(zip(fused.t, split.t)):
            assert torch.equal(a.grad_out, b.grad_out), (step, i)
            if fused.compressed(i):
                assert torch.equal(a.P[:, :r], b.P[:, :r]) and torch.equal(a.Q[:, :r], b.Q[:, :r]), (step, i)
                assert torch.equal(a.residual, b.residual), (step, i)


def test_first_phase_leaves_the_plain_product():
    """After the first phase the residual buffer holds D = G + E and P holds D Q, not orthonormalised."""
    m, n, r = 320, 448, 16
    g = gen.lowrank_plus_noise(m, n, 40, 0.9, 1e-4, 7)
    e = (1e-3 * np.random.default_rng(1).standard_normal((m, n))).astype(np.float32)
    q = np.zeros((n, r), dtype=np.float32)
    orc.init_q(q, 0, r, 3)
    ctx = edgc.Context(0, max_rank=r, max_rows=64, max_cols=64)
    ctx.reserve_batch([(m, n)])
    t = edgc.Tensor(to_dev(g), torch.zeros((m, n), device="cuda"), to_dev(e), to_dev(q),
                    torch.zeros((m, r), device="cuda"), False)
    ctx.compress_p_batch([t], r)
    torch.cuda.synchronize()
    d = g + e
    assert np.array_equal(to_host(t.residual), d)
    assert rel_fro(to_host(t.P), d.astype(np.float64) @ q.astype(np.float64)) <= 1e-4
    assert np.array_equal(to_host(t.Q), q)                      # the warm start is untouched so far


@pytest.mark.parametrize("deferred", [False, True])
def test_two_shards_with_averaged_factors_match_the_oracle_on_the_averaged_gradient(deferred):
    """Two data-parallel shards on one GPU: each runs the first phase on its own gradient and
    residual, P is averaged, each runs the second phase on the averaged P, Q is averaged, each
    reconstructs.  By linearity this is the plain step on the averaged gradient with the averaged
    residual, which is what the oracle computes."""
    shapes, r, steps, shards = [(256, 384), (384, 256)], 8, 4, 2
    ctxs, ts = [], []
    q0 = []
    for i, (m, n) in enumerate(shapes):
        q = np.zeros((n, r), dtype=np.float32)
        orc.init_q(q, 0, r, 50 + i)
        q0.append(q)
    for k in range(shards):
        c = edgc.Context(0, max_rank=r, max_rows=64, max_cols=64)
        c.reserve_batch(shapes)
        ctxs.append(c)
        ts.append([edgc.Tensor(torch.zeros(s, device="cuda"), torch.zeros(s, device="cuda"),
                               torch.zeros(s, device="cuda"), to_dev(q0[i]),
                               torch.zeros((s[0], r), device="cuda"), True) for i, s in enumerate(shapes)])
    E_o = [None] * len(shapes)
    Q_o = [q.copy() for q in q0]
    for step in range(steps):
        g = [[gen.lowrank_plus_noise(s[0], s[1], 24, 0.9, 1e-4, 1000 + 100 * step + 10 * k + i)
              for i, s in enumerate(shapes)] for k in range(shards)]
        for k in range(shards):
            for i in range(len(shapes)):
                ts[k][i].grad = to_dev(g[k][i])
            ctxs[k].compress_p_batch(ts[k], r, deferred=deferred and step > 0)
        torch.cuda.synchronize()
        for i in range(len(shapes)):                      # stand-in for the all-reduce (mean) of P
            mean = sum(ts[k][i].P for k in range(shards)) / shards
            for k in range(shards):
                ts[k][i].P.copy_(mean)
        for k in range(shards):
            ctxs[k].compress_q_batch(ts[k], r)
        torch.cuda.synchronize()
        for i in range(len(shapes)):                      # ... and of Q
            mean = sum(ts[k][i].Q for k in range(shards)) / shards
            for k in range(shards):
                ts[k][i].Q.copy_(mean)
        for k in range(shards):
            ctxs[k].decompress_batch(ts[k], r, deferred=deferred)
            for t in ts[k]:
                t.residual_is_zero = False
        torch.cuda.synchronize()
        for i in range(len(shapes)):
            g_mean = (sum(x[i].astype(np.float64) for x in g) / shards).astype(np.float32)
            P_o, Qn, D_o = orc.compress(g_mean, E_o[i], Q_o[i], r)
            out_o, E_o[i] = orc.decompress(P_o, Qn, D_o, orc.F32)
            Q_o[i] = Qn
            for k in range(shards):
                assert torch.equal(ts[k][i].grad_out, ts[0][i].grad_out), "every shard reconstructs the same matrix"
                assert rel_fro(to_host(ts[k][i].P), P_o) <= 1e-3, (step, i, k)
                assert rel_fro(to_host(ts[k][i].Q), Qn) <= 1e-3, (step, i, k)
            assert rel_fro(to_host(ts[0][i].grad_out), out_o) <= 1e-3, (step, i)
            # the shards' residuals average to the oracle's
            res = sum(to_host(ts[k][i].residual).astype(np.float64) for k in range(shards)) / shards
            if deferred:
                res = res - to_host(ts[0][i].grad_out).astype(np.float64)       # the buffers keep D
            assert np.linalg.norm(res - E_o[i]) <= 1e-3 * np.linalg.norm(D_o.astype(np.float64)), (step, i)
