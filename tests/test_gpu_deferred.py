"""The deferred subtraction of the batched calls (the residual buffer keeps D = G + E between
steps and the next P-pass subtracts M^ = P^ Q^T itself): against the oracle's explicit
error-feedback chain (Sec. III-B / VII), and bit for bit against the library's own explicit
chain."""
import numpy as np
import pytest
import torch

import edgc_inputs as gen
import paper_2511_10333_amd as edgc
from oracle import edgc_oracle as orc
from gpu_util import rel_fro, to_dev, to_host
from test_gpu_batch import MIXED, Stage, TOL, _widen

pytestmark = pytest.mark.gpu

RAGGED = [(384, 640), (130, 70), (257, 129), (333, 1000), (100,), (1000, 62)]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("r", [4, 16, 48, 64, 128])
def test_deferred_chain_matches_oracle_over_three_steps(dtype, r):
    """Every step's factors and reconstruction against the oracle, whose chain stores E; the
    device buffer is compared with the oracle's D."""
    # a spectrum that is still well above the noise at index r, so that all r columns are determined
    st = Stage(RAGGED, r, dtype, seed=17 + r, deferred=True, signal_rank=max(48, 2 * r),
               decay=max(0.9, 0.1 ** (1.0 / r)))
    for _ in range(3):
        st.step_device()
        st.step_oracle_and_compare()
    # carrying the subtraction out leaves the oracle's E
    st.ctx.residual_materialize_batch(st.t, r)
    torch.cuda.synchronize()
    for i, t in enumerate(st.t):
        if st.compressed(i):
            nD = np.linalg.norm(st.E[i].astype(np.float64)) + np.linalg.norm(_widen(st.G[i]).astype(np.float64))
            assert np.linalg.norm(to_host(t.residual).astype(np.float64) - st.E[i]) <= TOL[dtype] * nD, i


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("r,power_iters", [(8, 1), (16, 1), (40, 1), (128, 1), (16, 2)])
def test_deferred_equals_explicit_chain_bit_for_bit(dtype, r, power_iters):
    """Same inputs through deferred = 0 and deferred = 1: the launch shapes agree, M^ is formed
    by the same instruction sequence in both, so every output is identical."""
    a = Stage(MIXED, r, dtype, seed=5, power_iters=power_iters)
    b = Stage(MIXED, r, dtype, seed=5, power_iters=power_iters, deferred=True)
    for step in range(4):
        a.step_device()
        b.step_device()
        for i, (x, y) in enumerate(zip(a.t, b.t)):
            assert torch.equal(x.grad_out, y.grad_out), (step, i)
            if a.compressed(i):
                assert torch.equal(x.P[:, :r], y.P[:, :r]) and torch.equal(x.Q[:, :r], y.Q[:, :r]), (step, i)
                # explicit: E = D - M^ in the buffer; deferred: D itself
                m_hat = y.grad_out.float()
                assert torch.equal(x.residual, y.residual - m_hat), (step, i)
    b.ctx.residual_materialize_batch(b.t, r)
    torch.cuda.synchronize()
    for i, (x, y) in enumerate(zip(a.t, b.t)):
        if a.compressed(i):
            assert torch.equal(x.residual, y.residual), i


def test_changing_over_between_the_two_forms_and_the_rank():
    """deferred steps at rank 16, the subtraction carried out, then rank 32 (new columns of Q
    seeded), entered with an explicit residual and left deferred again; the oracle runs the
    plain chain with the same rank change."""
    m, n, ld = 320, 448, 32
    g = [gen.lowrank_plus_noise(m, n, 40, 0.9, 1e-4, 70 + k, dtype="f32") for k in range(5)]
    q = np.zeros((n, ld), dtype=np.float32)
    orc.init_q(q, 0, 16, 1)
    ctx = edgc.Context(0, max_rank=32, max_rows=64, max_cols=64)
    ctx.reserve_batch([(m, n)])
    t = edgc.Tensor(to_dev(g[0]), torch.zeros((m, n), device="cuda"), torch.zeros((m, n), device="cuda"),
                    to_dev(q), torch.zeros((m, ld), device="cuda"), True)
    E, r = None, 16
    plan = [(16, False, True), (16, True, True),      # (rank, compress deferred, decompress deferred)
            (32, False, True), (32, True, False), (32, False, False)]
    for k, (rk, cdef, ddef) in enumerate(plan):
        if rk != r:                                   # rank change: E itself is needed, and new columns
            ctx.residual_materialize_batch([t], r)
            qd = torch.zeros((n, ld), device="cuda")
            ctx.init_q(qd, r, rk, 2)
            t.Q[:, r:rk] = qd[:, r:rk]
            orc.init_q(q, r, rk, 2)
            r = rk
        t.grad = to_dev(g[k])
        ctx.compress_batch([t], r, deferred=cdef)
        ctx.decompress_batch([t], r, deferred=ddef)
        torch.cuda.synchronize()
        t.residual_is_zero = False
        Po, Qo, Do = orc.compress(g[k], E, np.ascontiguousarray(q[:, :r]), r)
        out_o, E = orc.decompress(Po, Qo, Do, orc.F32)
        q[:, :r] = Qo
        nD = np.linalg.norm(Do.astype(np.float64))
        assert rel_fro(to_host(t.P)[:, :r], Po) <= 1e-3, k
        assert rel_fro(to_host(t.Q)[:, :r], Qo) <= 1e-3, k
        assert rel_fro(to_host(t.grad_out), out_o) <= 1e-3, k
        want = Do if ddef else E
        assert np.linalg.norm(to_host(t.residual).astype(np.float64) - want) <= 1e-3 * nD, k


def test_error_feedback_is_conserved_in_the_deferred_form():
    """Sum of the gradients = sum of the reconstructions + the residual still owed (Sec. VII), with
    fresh gradients every step; the residual owed is D - M^ of the last step."""
    shapes, r, steps = [(256, 384), (384, 256)], 8, 6
    st = Stage(shapes, r, "f32", seed=3, deferred=True)
    total_g = [np.zeros(s, dtype=np.float64) for s in shapes]
    total_out = [np.zeros(s, dtype=np.float64) for s in shapes]
    for k in range(steps):
        for i, s in enumerate(shapes):
            gk = gen.lowrank_plus_noise(s[0], s[1], 24, 0.9, 1e-4, 1000 + 10 * k + i, dtype="f32")
            st.t[i].grad = to_dev(gk)
            total_g[i] += gk
        st.step_device()
        for i in range(len(shapes)):
            total_out[i] += to_host(st.t[i].grad_out)
    st.ctx.residual_materialize_batch(st.t, r)
    torch.cuda.synchronize()
    for i in range(len(shapes)):
        owed = to_host(st.t[i].residual).astype(np.float64)
        assert np.linalg.norm(total_g[i] - total_out[i] - owed) <= 1e-5 * np.linalg.norm(total_g[i]), i


def test_full_size_bench_layout_deferred():
    """The benchmark's default workload at full size in the layout and mode bench.py times
    (two groups, deferred subtraction), three steps so that two of them subtract M^ on the way."""
    name = "cfg2_gpt_h2048_r16"
    w = gen.WORKLOADS[name]
    mats = [g for _, g in gen.workload_matrices(name)]
    order = sorted(range(len(mats)), key=lambda i: -mats[i].size)
    members, load = [[], []], [0, 0]
    for i in order:
        k = load.index(min(load))
        members[k].append(i)
        load[k] += mats[i].size
    for idx in members:
        st = Stage(None, w["rank"], w["dtype"], seed=w["seed"], mats=[mats[i] for i in sorted(idx)], deferred=True)
        for _ in range(3):
            st.step_device()
            st.step_oracle_and_compare()
        del st
        torch.cuda.empty_cache()


def test_descriptors_of_one_call_must_agree():
    st = Stage([(256, 256), (128, 384)], 8, "f32", seed=5)
    arr, code = st.ctx._marshal(st.t, deferred=True)
    arr[1].deferred = 0
    L = edgc.binding.load_library()
    assert L.edgc_compress_batch(st.ctx._h, arr, 2, code, 8, 1, None) == edgc.binding.EINVAL
    assert L.edgc_decompress_batch(st.ctx._h, arr, 2, code, 8, None) == edgc.binding.EINVAL
    arr[1].deferred = 2
    arr[0].deferred = 2
    assert L.edgc_compress_batch(st.ctx._h, arr, 2, code, 8, 1, None) == edgc.binding.EINVAL


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_deferred_with_strided_gradient_rows_and_more_tensors_than_one_launch_holds(dtype):
    """Gradient rows embedded in wider buffers (ld > n), and 21 tensors, which go through the
    kernels as a launch of 16 and one of 5."""
    st = Stage([(200, 328), (192, 192), (333, 100)], 24, dtype, seed=9, ragged_ld=True, deferred=True)
    for _ in range(3):
        st.step_device()
        st.step_oracle_and_compare()
    many = Stage([(64 + 8 * i, 96 + 4 * i) for i in range(21)], 8, dtype, seed=11, deferred=True)
    for _ in range(2):
        many.step_device()
        many.step_oracle_and_compare()


def test_deferred_hidden_5120_bf16_block_full_size():
    """The hidden-5120 bf16 block at rank 64 in the bench's two-group layout, deferred form:
    two steps, the second of which subtracts the first one's reconstruction on the way."""
    name = "cfg4_gpt_h5120_bf16"
    w = gen.WORKLOADS[name]
    mats = [g for _, g in gen.workload_matrices(name)]
    order = sorted(range(len(mats)), key=lambda i: -mats[i].size)
    members, load = [[], []], [0, 0]
    for i in order:
        k = load.index(min(load))
        members[k].append(i)
        load[k] += mats[i].size
    for idx in members:
        st = Stage(None, w["rank"], w["dtype"], seed=w["seed"], mats=[mats[i] for i in sorted(idx)], deferred=True)
        for _ in range(2):
            st.step_device()
            st.step_oracle_and_compare()
        del st
        torch.cuda.empty_cache()


def test_seeded_sweep_of_small_and_ragged_shapes_deferred_equals_explicit():
    """Forty seeded shapes between 2 and 700 per side (odd sizes, fewer columns than one stage,
    fewer rows than one wave, ranks that are no multiple of 4), both dtypes: two steps through
    either form must agree bit for bit, and the first step's D is G."""
    rng = np.random.default_rng(2024)
    for case in range(40):
        m, n = int(rng.integers(2, 700)), int(rng.integers(2, 700))
        r = int(rng.integers(1, min(m, n, 128) + 1))
        dtype = "bf16" if case % 2 else "f32"
        if edgc.tensor_bypassed(m, n, r):
            continue
        a = Stage([(m, n)], r, dtype, seed=case)
        b = Stage([(m, n)], r, dtype, seed=case, deferred=True)
        for step in range(2):
            a.step_device()
            b.step_device()
            x, y = a.t[0], b.t[0]
            assert torch.equal(x.grad_out, y.grad_out), (case, m, n, r, dtype, step)
            assert torch.equal(x.P[:, :r], y.P[:, :r]) and torch.equal(x.Q[:, :r], y.Q[:, :r]), (case, m, n, r, dtype, step)
            assert torch.equal(x.residual, y.residual - y.grad_out.float()), (case, m, n, r, dtype, step)
        del a, b


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_deferred_with_the_reconstruction_written_over_the_gradient(dtype):
    """grad_out may be the gradient buffer itself (the reconstruction replaces the gradient in place):
    the P-pass has read the gradient before the decompress of the same step overwrites it."""
    shapes, r = [(384, 640), (130, 260)], 16
    a = Stage(shapes, r, dtype, seed=4, deferred=True)
    b = Stage(shapes, r, dtype, seed=4, deferred=True)
    fresh = [t.grad.clone() for t in b.t]
    for t in b.t:
        t.grad_out = t.grad
    for step in range(3):
        for t, g in zip(b.t, fresh):
            t.grad.copy_(g)                                   # a new gradient arrives in the same buffer
        a.step_device()
        b.step_device()
        for i, (x, y) in enumerate(zip(a.t, b.t)):
            assert torch.equal(x.grad_out, y.grad), (step, i)
            assert torch.equal(x.residual, y.residual) and torch.equal(x.P, y.P) and torch.equal(x.Q, y.Q), (step, i)
