"""Batched compress / decompress (every tensor of a stage in one launch sequence) against the
oracle, tensor by tensor, and against the single-tensor entry points."""
import numpy as np
import pytest
import torch

import edgc_inputs as gen
import paper_2511_10333_amd as edgc
from oracle import edgc_oracle as orc
from gpu_util import ELEMENTWISE_TOL, elementwise_ratio, rel_fro, to_dev, to_host

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-3, "bf16": 1e-2}


def _widen(a):
    return gen.bf16_bits_to_f32(a) if a.dtype == np.uint16 else a


class Stage:
    """Host and device state of a list of gradient tensors that share one rank."""

    def __init__(self, shapes, r, dtype, seed=0, ragged_ld=False, mats=None, deferred=False, power_iters=1,
                 signal_rank=48, decay=0.9):
        """``mats``: ready-made 2-D gradients (host arrays) instead of generated ones.
        ``deferred``: the residual buffers keep D between steps (edgc_tensor.deferred)."""
        if mats is not None:
            shapes = [g.shape for g in mats]
        self.shapes, self.r, self.dtype = shapes, r, dtype
        self.deferred, self.power_iters, self.steps = deferred, power_iters, 0
        self.ctx = edgc.Context(0, max_rank=128, max_rows=64, max_cols=64)    # own scratch unused here
        self.ctx.reserve_batch([s if len(s) == 2 else (1, s[0]) for s in shapes])
        tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.G, self.Q, self.E = [], [], []
        self.t = []
        for i, s in enumerate(shapes):
            if len(s) == 1:                                   # 1-D tensor: never compressed
                g = gen.gaussian(s[0], 1e-3, seed + i).astype(np.float32)
                g = gen.to_bf16_bits(g) if dtype == "bf16" else g
                self.G.append(g); self.Q.append(None); self.E.append(None)
                self.t.append(edgc.Tensor(to_dev(g), torch.zeros(s[0], dtype=tdt, device="cuda")))
                continue
            m, n = s
            g = mats[i] if mats is not None else \
                gen.lowrank_plus_noise(m, n, min(m, n, signal_rank), decay, 1e-4, seed + i, dtype=dtype)
            self.G.append(g)
            if edgc.tensor_bypassed(m, n, r):
                self.Q.append(None); self.E.append(None)
                self.t.append(edgc.Tensor(to_dev(g), torch.zeros((m, n), dtype=tdt, device="cuda")))
                continue
            ldq = (r + 3) // 4 * 4
            q = np.zeros((n, ldq), dtype=np.float32)
            orc.init_q(q, 0, r, 100 + i)
            self.Q.append(q)
            self.E.append(None)
            gd = to_dev(g)
            if ragged_ld:                                     # rows embedded in a wider buffer
                wide = torch.zeros((m, n + 8), dtype=tdt, device="cuda")
                wide[:, :n] = gd
                gd = wide[:, :n]
            self.t.append(edgc.Tensor(gd, torch.zeros((m, n), dtype=tdt, device="cuda"),
                                      torch.full((m, n), float("nan"), device="cuda"), to_dev(q),
                                      torch.full((m, ldq), 7.0, device="cuda"), True))

    def compressed(self, i):
        return self.Q[i] is not None

    def step_device(self):
        # a deferred compress expects D and the factors of the step before: not on the first step
        self.ctx.compress_batch(self.t, self.r, power_iters=self.power_iters,
                                deferred=self.deferred and self.steps > 0)
        self.ctx.decompress_batch(self.t, self.r, deferred=self.deferred)
        torch.cuda.synchronize()
        self.steps += 1
        for t in self.t:
            t.residual_is_zero = False

    def step_oracle_and_compare(self):
        r, tol = self.r, TOL[self.dtype]
        code = orc.BF16 if self.dtype == "bf16" else orc.F32
        for i, g in enumerate(self.G):
            t = self.t[i]
            if not self.compressed(i):
                assert np.array_equal(to_host(t.grad_out).reshape(g.shape), g), f"tensor {i} must pass through"
                continue
            first = self.E[i] is None
            Po, Qo, Do = orc.compress(g, self.E[i], np.ascontiguousarray(self.Q[i][:, :r]), r)
            out_o, E_o = orc.decompress(Po, Qo, Do, code)
            self.Q[i][:, :r] = Qo
            self.E[i] = E_o
            nD = np.linalg.norm(Do.astype(np.float64))
            assert rel_fro(to_host(t.P)[:, :r], Po) <= tol, i
            assert rel_fro(to_host(t.Q)[:, :r], Qo) <= tol, i
            assert rel_fro(_widen(to_host(t.grad_out)), _widen(out_o)) <= tol, i
            # ... and element by element, |M^_ij - oracle| against ||p_i|| ||q_j|| (a few wrong elements of one
            # tile would not show in a Frobenius norm over the whole matrix)
            assert elementwise_ratio(_widen(to_host(t.grad_out)), _widen(out_o), Po, Qo) <= ELEMENTWISE_TOL[self.dtype], i
            if self.deferred:                                 # the buffer keeps D; E stays in factored form
                assert np.linalg.norm(to_host(t.residual).astype(np.float64) - Do) <= tol * nD, i
                if first:
                    assert np.array_equal(to_host(t.residual), Do.astype(np.float32)), i
                continue
            assert np.linalg.norm(to_host(t.residual).astype(np.float64) - E_o) <= tol * nD, i
            # D = M^ + E_new on the device (first step: its D is the oracle's D bit for bit)
            if first:
                assert rel_fro(to_host(t.residual) + _widen(to_host(t.grad_out)), Do) <= 1e-6


MIXED = [(384, 640), (100,), (130, 70), (6, 200), (257, 129), (512, 256), (64,)]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("r", [4, 16])
def test_mixed_stage_matches_oracle_over_three_steps(dtype, r):
    st = Stage(MIXED, r, dtype, seed=3)
    assert not st.compressed(1) and not st.compressed(6)          # 1-D
    assert st.compressed(3) == (not edgc.tensor_bypassed(6, 200, r))
    for _ in range(3):                                            # residual carried from step to step
        st.step_device()
        st.step_oracle_and_compare()


@pytest.mark.parametrize("name,rank,steps,deferred", [("cfg2_gpt_h2048_r16", 16, 2, False),
                                                      ("cfg4_gpt_h5120_bf16", 64, 1, False),
                                                      ("cfg4_gpt_h5120_bf16", 32, 2, True),
                                                      ("cfg4_gpt_h5120_bf16", 128, 2, True)])
def test_benchmark_workload_full_size_in_the_bench_layout(name, rank, steps, deferred):
    """The benchmark's matrices at full size against the oracle's whole steps, grouped as bench.py groups
    them (two groups balanced by size, largest first into the lighter one): two steps of the hidden-2048
    block so that the second carries a residual; the hidden-5120 bf16 block (20480 x 5120 included) for one
    step at rank 64 and, in the layout bench.py times (residual deferred: the second step runs the
    streaming P-pass that subtracts P^ Q^T on the way), for two steps at ranks 32 and 128."""
    w = gen.WORKLOADS[name]
    mats = [g for _, g in gen.workload_matrices(name)]
    order = sorted(range(len(mats)), key=lambda i: -mats[i].size)
    members, load = [[], []], [0, 0]
    for i in order:
        k = load.index(min(load))
        members[k].append(i)
        load[k] += mats[i].size
    assert sorted(members[0] + members[1]) == list(range(len(mats)))
    for idx in members:
        st = Stage(None, rank, w["dtype"], seed=w["seed"], mats=[mats[i] for i in sorted(idx)], deferred=deferred)
        for _ in range(steps):
            st.step_device()
            st.step_oracle_and_compare()
        del st
        torch.cuda.empty_cache()


def test_ragged_leading_dimension_and_rank_48():
    st = Stage([(200, 328), (192, 192), (333, 100)], 48, "f32", seed=9, ragged_ld=True)
    st.step_device()
    st.step_oracle_and_compare()


def test_more_tensors_than_one_group_holds():
    shapes = [(64 + 8 * i, 96 + 4 * i) for i in range(21)]        # 21 > 16 tensors per launch
    st = Stage(shapes, 8, "f32", seed=11)
    st.step_device()
    st.step_oracle_and_compare()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_batch_equals_single_tensor_calls(dtype):
    shapes, r = [(512, 768), (256, 1024), (1024, 256)], 16
    st = Stage(shapes, r, dtype, seed=21)
    single = edgc.Context(0, max_rank=128, max_rows=1024, max_cols=1024)
    ref = []
    for t in st.t:                                                 # same inputs through the single calls
        Q, P = t.Q.clone(), torch.empty_like(t.P)
        E, out = torch.empty_like(t.residual), torch.empty_like(t.grad_out)
        single.compress(t.grad, E, True, Q, P, r)
        single.decompress(P, Q, r, E, out)
        ref.append((P, Q, E, out))
    st.step_device()
    for t, (P, Q, E, out) in zip(st.t, ref):
        # the launch shapes differ (a batch shares the GPU among its tensors), so sums are taken
        # in another order: equal to rounding, not bit for bit
        assert rel_fro(to_host(t.P)[:, :r], to_host(P)[:, :r]) <= 2e-5
        assert rel_fro(to_host(t.Q)[:, :r], to_host(Q)[:, :r]) <= 2e-5
        assert rel_fro(_widen(to_host(t.grad_out)), _widen(to_host(out))) <= (1e-2 if dtype == "bf16" else 2e-5)
    # a batch of one has the single call's launch shape: bit for bit
    one = Stage([shapes[0]], r, dtype, seed=21)
    one.step_device()
    P, Q, E, out = ref[0]
    assert torch.equal(one.t[0].P[:, :r], P[:, :r]) and torch.equal(one.t[0].Q[:, :r], Q[:, :r])
    assert torch.equal(one.t[0].residual, E) and torch.equal(one.t[0].grad_out, out)


@pytest.mark.parametrize("deferred", [False, True])
def test_prepared_descriptors_give_the_same_bits_as_a_list(deferred):
    """binding.PreparedBatch builds the descriptor array once and rewrites only the two per-call
    flags: three steps through it equal three steps through the plain list bit for bit."""
    shapes, r = [(512, 768), (256, 1024), (1024, 256)], 16
    a = Stage(shapes, r, "bf16", seed=5, deferred=deferred)
    b = Stage(shapes, r, "bf16", seed=5, deferred=deferred)
    prep = edgc.PreparedBatch(b.t)
    for step in range(3):
        a.step_device()
        b.ctx.compress_batch(prep, r, deferred=deferred and step > 0)
        b.ctx.decompress_batch(prep, r, deferred=deferred)
        torch.cuda.synchronize()
        for t in b.t:
            t.residual_is_zero = False
        for ta, tb in zip(a.t, b.t):
            assert torch.equal(ta.P, tb.P) and torch.equal(ta.Q, tb.Q)
            assert torch.equal(ta.residual, tb.residual) and torch.equal(ta.grad_out, tb.grad_out)


def test_batch_rejects_bad_descriptors_before_launching():
    st = Stage([(256, 256), (128, 384)], 8, "f32", seed=5)
    before = [t.P.clone() for t in st.t]
    big = edgc.Tensor(torch.zeros((300, 256), device="cuda"), torch.zeros((300, 256), device="cuda"),
                      torch.zeros((300, 256), device="cuda"), torch.zeros((256, 8), device="cuda"),
                      torch.zeros((300, 8), device="cuda"), True)
    with pytest.raises(edgc.EdgcError):                            # larger than its slot
        st.ctx.compress_batch([big, st.t[1]], 8)
    with pytest.raises(edgc.EdgcError):                            # more tensors than slots
        st.ctx.compress_batch(st.t + [st.t[0]], 8)
    with pytest.raises(edgc.EdgcError):                            # rank above the context's
        st.ctx.compress_batch(st.t, 129)
    bad = edgc.Tensor(st.t[1].grad, st.t[1].grad_out, None, st.t[1].Q, st.t[1].P, True)
    with pytest.raises(edgc.EdgcError):                            # second descriptor is bad:
        st.ctx.compress_batch([st.t[0], bad], 8)                   # nothing of the first may run
    torch.cuda.synchronize()
    for t, p in zip(st.t, before):
        assert torch.equal(t.P, p)
    with pytest.raises(TypeError):
        st.ctx.compress_batch([st.t[0], edgc.Tensor(st.t[1].grad.bfloat16(), st.t[1].grad_out.bfloat16())], 8)
    st.ctx.compress_batch([], 8)                                   # empty batch: nothing to do
    st.ctx.decompress_batch([], 8)


# ---------------------------------------------------------------------------
# stage-level entropy over separate buffers: the union of the buffers' own samples
# ---------------------------------------------------------------------------
def _oracle_union_entropy(bufs, stride, chunk, seed, step, bins, value_range=None):
    """Each buffer's sample by the oracle's sampler, gathered and concatenated; the oracle's
    estimator then runs over that vector with every element sampled."""
    parts = []
    for b in bufs:
        idx = orc.sample_indices(b.size, stride, chunk, seed, step)
        parts.append(b.reshape(-1)[idx])
    cat = np.concatenate(parts)
    return orc.entropy(cat, 1, 1, 0, 0, bins, value_range), cat.size


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("stride,chunk,bins", [(100, 64, 1024), (10, 1, 256), (1, 64, 4096), (7, 48, 65536)])
def test_stage_entropy_over_separate_buffers(dtype, stride, chunk, bins):
    sizes = [1 << 20, 300_007, 64, 1, 2_000_003, 4096]
    bufs = [gen.laplace_mixture(n, 40 + i, dtype=dtype, scale=1e-3 * (1 + i)) for i, n in enumerate(sizes)]
    dev = [to_dev(b) for b in bufs]
    c = edgc.Context(0, max_bins=65536, max_rank=4, max_rows=64, max_cols=64)
    counts = torch.zeros(bins, dtype=torch.int64, device="cuda")
    for step in (0, 5):
        got = c.entropy_estimate(dev, stride, chunk, 9, step, bins, counts_out=counts)
        want, n_s = _oracle_union_entropy(bufs, stride, chunk, 9, step, bins)
        assert got.n_sampled == n_s == want.n_sampled
        assert (got.lo, got.hi) == (want.lo, want.hi)
        assert np.array_equal(counts.cpu().numpy().astype(np.uint64), want.counts), "bin counts are bit-exact"
        assert abs(got.H_bits - want.H_bits) <= 1e-5 and abs(got.h_diff_nats - want.h_diff_nats) <= 1e-5
    # a caller's range, and one buffer that is not 16-byte aligned (the group falls back to scalar loads)
    odd = [dev[0][1:], dev[1]]
    odd_host = [bufs[0][1:], bufs[1]]
    got = c.entropy_estimate(odd, stride, chunk, 9, 3, bins, value_range=(-2e-3, 2e-3))
    want, n_s = _oracle_union_entropy(odd_host, stride, chunk, 9, 3, bins, (-2e-3, 2e-3))
    assert got.n_sampled == n_s and abs(got.H_bits - want.H_bits) <= 1e-5
    # one buffer through the batch call is the single call
    a = c.entropy_estimate([dev[0]], stride, chunk, 9, 1, bins)
    b = c.entropy_estimate(dev[0], stride, chunk, 9, 1, bins)
    assert a == b
    with pytest.raises(edgc.EdgcError):
        c.entropy_estimate([dev[0]] * 33, stride, chunk, 9, 1, bins)
    with pytest.raises(edgc.EdgcError):
        c.entropy_estimate([], stride, chunk, 9, 1, bins)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_stage_entropy_large_union_sample(dtype):
    """A union sample large enough for the launch shapes of large samples (one block of 1024 threads
    per compute unit, whole-item rounds with the next loads in flight) over several buffers of
    different sizes, with a ragged tail and a few non-finite values."""
    sizes = [(1 << 25) + 5, 1 << 24, (1 << 23) + 64, 12_345_679]
    bufs = [gen.laplace_mixture(n, 70 + i, dtype=dtype, scale=1e-3 * (1 + i)) for i, n in enumerate(sizes)]
    nan, inf = (0x7fc0, 0x7f80) if dtype == "bf16" else (np.float32(np.nan), np.float32(np.inf))
    bufs[0][12345] = nan
    bufs[1][-1] = inf
    bufs[3][7] = nan
    dev = [to_dev(b) for b in bufs]
    c = edgc.Context(0, max_bins=65536, max_rank=4, max_rows=64, max_cols=64)
    for stride, chunk, bins in [(1, 64, 4096), (1, 64, 65536), (3, 64, 1024)]:
        counts = torch.zeros(bins, dtype=torch.int64, device="cuda")
        got = c.entropy_estimate(dev, stride, chunk, 9, 2, bins, counts_out=counts)
        want, n_s = _oracle_union_entropy(bufs, stride, chunk, 9, 2, bins)
        assert got.n_sampled == n_s == want.n_sampled
        assert got.n_nonfinite == want.n_nonfinite and (stride != 1 or got.n_nonfinite == 3)
        assert (got.lo, got.hi) == (want.lo, want.hi)
        assert np.array_equal(counts.cpu().numpy().astype(np.uint64), want.counts), (stride, bins)
        assert int(counts.sum()) == n_s - got.n_nonfinite
        assert abs(got.H_bits - want.H_bits) <= 1e-5 and abs(got.h_diff_nats - want.h_diff_nats) <= 1e-5
    c.close()


# ---------------------------------------------------------------------------
# the batched calls under HIP graph capture: no allocation, no synchronisation, no memset
# node inside them, so a captured step replays like the eager one
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("deferred", [False, True])
def test_batched_step_replays_from_a_hip_graph(deferred):
    shapes, r = [(384, 512), (256, 640), (100,)], 8
    eager = Stage(shapes, r, "f32", seed=31, deferred=deferred)
    graphed = Stage(shapes, r, "f32", seed=31, deferred=deferred)
    for st in (eager, graphed):                       # first step eagerly: it starts from a zero residual
        st.step_device()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    keep = [(t.residual.clone(), t.Q.clone(), t.P.clone()) if t.residual is not None else None for t in graphed.t]
    ent_out = torch.zeros(edgc.binding.ENTROPY_RESULT_BYTES, dtype=torch.uint8, pin_memory=True)
    flats = [t.grad.view(-1) for t in graphed.t]
    with torch.cuda.graph(g, stream=side, capture_error_mode="thread_local"):
        graphed.ctx.entropy_estimate_async(flats, 10, 64, 3, 0, 256, ent_out, stream=side)
        graphed.ctx.compress_batch(graphed.t, r, stream=side, deferred=deferred)
        graphed.ctx.decompress_batch(graphed.t, r, stream=side, deferred=deferred)
    torch.cuda.synchronize()
    ent_want = graphed.ctx.entropy_estimate(flats, 10, 64, 3, 0, 256)
    for t, k in zip(graphed.t, keep):                 # capture runs nothing, but make the state explicit
        if k is not None:
            t.residual.copy_(k[0]); t.Q.copy_(k[1]); t.P.copy_(k[2])
    for step in range(3):
        eager.step_device()
        g.replay()
        # eager work and a synchronisation between replays
        torch.cuda.synchronize()
        _ = (eager.t[0].grad_out * 2).sum().item()
        assert edgc.EntropyResult.from_buffer(ent_out.numpy().tobytes()) == ent_want, step
        ent_out.zero_()
        for a, b in zip(eager.t, graphed.t):
            assert torch.equal(a.grad_out, b.grad_out), step
            if a.residual is not None:
                assert torch.equal(a.residual, b.residual) and torch.equal(a.Q, b.Q) and torch.equal(a.P, b.P), step
