"""The whole 8-layer stage of the dynamic-rate configuration at full size (32 tensors, 1.61e9 fp32
elements, hidden 4096) in the layout bench.py times: two batched groups, one stage-level entropy
estimate, the residual in the deferred form, ranks changing between steps.  The CPU oracle cannot
run whole steps at this size in seconds, so its own steps are run on what it can take one by one:
the entropy of the 1 % sample (gathered, bit-exact counts), sampled elements of D (the recurrence
with the deferred subtraction, bit for bit), the oracle's P = D Q on gathered rows of D, its
orthonormalisation of the device's P (whole factor, one tensor of every shape; P^T P = I and
P = P^ R with R upper triangular and a positive diagonal for all of them), its Q = D^T P^ on gathered
columns of D, and its reconstruction of sampled elements.  The same walk runs over the
hidden-5120 block with bf16 gradients (its 20480 x 5120 matrix is the largest of the workloads)
at ranks 128, 32 and 64, and over a single matrix of more than 2^31 elements."""
import numpy as np
import pytest
import torch

import edgc_inputs as gen
import paper_2511_10333_amd as edgc
from oracle import edgc_oracle as orc

pytestmark = pytest.mark.gpu

STRIDE, CHUNK, BINS, SEED = 100, 64, 1024, 0
CASES = [
    # ranks per step: the kernels for ranks <= 32, <= 64 and > 64, changing up and down
    ("cfg5_stage8_h4096", "f32", [16, 16, 64, 64, 128, 8], 1_610_612_736),
    # the hidden-5120 block (its 20480 x 5120 matrix is the largest of the workloads) with bf16 gradients
    ("cfg4_gpt_h5120_bf16", "bf16", [128, 128, 32, 64], 314_572_800),
    # one matrix of more than 2^31 elements (an embedding-sized gradient): element and byte offsets
    # beyond 32 bits in every pass and in the sampler
    ((262144, 8704), "f32", [16, 16, 64], 2_281_701_376),
]


def _groups(sizes, k):
    order = sorted(range(len(sizes)), key=lambda i: -sizes[i])
    members, load = [[] for _ in range(k)], [0] * k
    for i in order:
        g = load.index(min(load))
        members[g].append(i)
        load[g] += sizes[i]
    return [sorted(m) for m in members]


@pytest.mark.parametrize("name,dtype,RANKS,elements", CASES)
def test_stage_at_full_size_sampled_against_the_oracle(name, dtype, RANKS, elements):
    if isinstance(name, tuple):
        shapes = [name]
    else:
        w = gen.WORKLOADS[name]
        shapes = [(s.m, s.n) for s in w["layers"]] * w.get("repeat", 1)
    assert sum(m * n for m, n in shapes) == elements
    NT = len(shapes)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    tol = 1e-2 if dtype == "bf16" else 1e-3
    code = orc.BF16 if dtype == "bf16" else orc.F32
    first_of_shape = {s: i for i, s in reversed(list(enumerate(shapes)))}
    dev = torch.device("cuda")
    rmax, kdim = max(RANKS), 24
    rng = np.random.default_rng(7)
    tg = torch.Generator(device="cuda").manual_seed(11)
    U = [torch.randn((m, kdim), device=dev, generator=tg) / np.sqrt(m) for m, _ in shapes]
    V = [torch.randn((n, kdim), device=dev, generator=tg) / np.sqrt(n) for _, n in shapes]
    G = [torch.empty(s, device=dev, dtype=tdt) for s in shapes]
    out = [torch.empty(s, device=dev, dtype=tdt) for s in shapes]
    res = [torch.empty(s, device=dev) for s in shapes]
    Q = [torch.zeros((n, rmax), device=dev) for _, n in shapes]
    P = [torch.zeros((m, rmax), device=dev) for m, _ in shapes]
    seeder = edgc.Context(0, max_bins=16, max_rank=4, max_rows=64, max_cols=64)
    for i in range(NT):
        seeder.init_q(Q[i], 0, RANKS[0], 900 + i)           # seeded start of the warm-started factor
    members = _groups([m * n for m, n in shapes], min(2, NT))
    ctxs, tens = [], []
    for idx in members:
        c = edgc.Context(0, max_bins=16, max_rank=rmax, max_rows=64, max_cols=64)
        c.reserve_batch([shapes[i] for i in idx])
        ctxs.append(c)
        tens.append([edgc.Tensor(G[i], out[i], res[i], Q[i], P[i], True) for i in idx])
    ectx = edgc.Context(0, max_bins=BINS, max_rank=4, max_rows=64, max_cols=64)
    counts = torch.zeros(BINS, dtype=torch.int64, device=dev)
    # sampled positions per tensor
    pos = [(rng.integers(0, m, 48), rng.integers(0, n, 48)) for m, n in shapes]
    rows = [rng.integers(0, m, 3) for m, _ in shapes]
    cols = [rng.integers(0, n, 3) for _, n in shapes]
    for (ii, jj), rr, cc, (m, n) in zip(pos, rows, cols, shapes):      # the far corner is always among them
        ii[-3:], jj[-3:] = [m - 1, m - 1, m - 2], [n - 1, 0, n - 2]
        rr[-1], cc[-1] = m - 1, n - 1
    idx_cache = {}
    r_prev, d_prev, out_prev = None, None, None
    for step, r in enumerate(RANKS):
        # fresh gradients: a low-rank part whose spectrum flattens with the step, plus noise
        decay = 0.80 + 0.03 * step
        s_vec = torch.tensor(decay ** np.arange(kdim), dtype=torch.float32, device=dev)
        for i in range(NT):
            if dtype == "bf16":
                tmp = torch.empty(shapes[i], device=dev).normal_(0.0, 1e-4, generator=tg)
                tmp.addmm_(U[i] * s_vec, V[i].t())
                G[i].copy_(tmp)
                del tmp
            else:
                G[i].normal_(0.0, 1e-4, generator=tg)
                G[i].addmm_(U[i] * s_vec, V[i].t())
        # --- entropy of the stage: the union of every buffer's own sample ---------------------------
        got = ectx.entropy_estimate([g.view(-1) for g in G], STRIDE, CHUNK, SEED, step, BINS, counts_out=counts)
        parts = []
        for g in G:
            key = (g.numel(), step)
            if key not in idx_cache:
                idx_cache[key] = torch.from_numpy(orc.sample_indices(g.numel(), STRIDE, CHUNK, SEED, step)
                                                  .astype(np.int64)).to(dev)
            parts.append(g.view(-1)[idx_cache[key]])
        sample = torch.cat(parts)
        sample = (sample.view(torch.int16).cpu().numpy().view(np.uint16) if dtype == "bf16" else sample.cpu().numpy())
        want = orc.entropy(sample, 1, 1, 0, 0, BINS)
        assert got.n_sampled == sample.size == want.n_sampled
        assert (got.lo, got.hi) == (want.lo, want.hi)
        assert np.array_equal(counts.cpu().numpy().astype(np.uint64), want.counts), step
        assert abs(got.H_bits - want.H_bits) <= 1e-5 and abs(got.h_diff_nats - want.h_diff_nats) <= 1e-5
        # --- rank change: the subtraction is carried out, new columns of Q are seeded ------------------
        deferred_in = step > 0
        if r_prev is not None and r != r_prev:
            for c, ts in zip(ctxs, tens):
                c.residual_materialize_batch(ts, r_prev)
            if r > r_prev:
                for i in range(NT):
                    seeder.init_q(Q[i], r_prev, r, 900 + i)
            deferred_in = False
        q_old = [q[:, :r].clone() for q in Q]
        torch.cuda.synchronize()
        # --- first phase: D and P = D Q -------------------------------------------------------------------
        for c, ts in zip(ctxs, tens):
            c.compress_p_batch(ts, r, deferred=deferred_in)
        torch.cuda.synchronize()
        p_raw = [p[:, :r].clone() for p in P]
        for i, (m, n) in enumerate(shapes):
            ii, jj = pos[i]
            d_now = res[i][ii, jj].cpu().numpy()
            g_now = G[i][ii, jj].float().cpu().numpy()
            if step == 0:
                assert np.array_equal(d_now, g_now), i
            else:
                # D = G + (D_prev - M^_prev) in the same fp32 operations, whether the subtraction was
                # deferred to this P-pass or carried out by the materialisation before a rank change
                assert np.array_equal(d_now, g_now + (d_prev[i] - out_prev[i])), (step, i)
            assert np.abs(d_now).max() > 0
            # the oracle's P = D Q on the gathered rows of D (its operand roundings included)
            rr = torch.from_numpy(np.asarray(rows[i], dtype=np.int64)).to(dev)
            want_rows = orc.contract_p(res[i][rr].cpu().numpy(), q_old[i].cpu().numpy(), code)
            got_rows = p_raw[i][rr].cpu().numpy()
            for k in range(len(rows[i])):
                assert np.linalg.norm(got_rows[k] - want_rows[k].astype(np.float64)) <= \
                    tol * np.linalg.norm(want_rows[k].astype(np.float64)) + 1e-12, (step, i, rows[i][k])
        # --- second phase: orthonormalisation and Q = D^T P^ ------------------------------------------
        for c, ts in zip(ctxs, tens):
            c.compress_q_batch(ts, r)
        torch.cuda.synchronize()
        for i, (m, n) in enumerate(shapes):
            ph = P[i][:, :r].double().cpu().numpy()
            pr = p_raw[i].double().cpu().numpy()
            assert np.abs(ph.T @ ph - np.eye(r)).max() <= 1e-5, (step, i)
            R = ph.T @ pr
            scale = np.abs(np.diag(R)).max()
            assert np.abs(np.tril(R, -1)).max() <= 1e-4 * scale and (np.diag(R) > 0).all(), (step, i)
            assert np.linalg.norm(ph @ R - pr) <= 1e-4 * np.linalg.norm(pr), (step, i)
            if first_of_shape[(m, n)] == i:         # the oracle's orthonormalisation of the same P, whole factor
                want_ph = orc.orthonormalise(p_raw[i].cpu().numpy())
                got_ph = P[i][:, :r].cpu().numpy()
                assert np.linalg.norm(got_ph.astype(np.float64) - want_ph) <= tol * np.sqrt(r), (step, i)
                assert np.abs(got_ph.astype(np.float64) - want_ph).max() <= tol * np.abs(want_ph).max(), (step, i)
            # the oracle's Q = D^T P^ on the gathered columns of D, from the device's P^
            cc = torch.from_numpy(np.asarray(cols[i], dtype=np.int64)).to(dev)
            want_q = orc.contract_q(res[i][:, cc].cpu().numpy(), P[i][:, :r].cpu().numpy(), code)
            got_q = Q[i][cc, :r].cpu().numpy()
            for k in range(len(cols[i])):
                assert np.linalg.norm(got_q[k] - want_q[k].astype(np.float64)) <= \
                    tol * np.linalg.norm(want_q[k].astype(np.float64)) + 1e-12, (step, i, cols[i][k])
        # --- reconstruction ------------------------------------------------------------------------------
        for c, ts in zip(ctxs, tens):
            c.decompress_batch(ts, r, deferred=True)
            for t in ts:
                t.residual_is_zero = False
        torch.cuda.synchronize()
        d_prev, out_prev = [], []
        for i, (m, n) in enumerate(shapes):
            ii, jj = pos[i]
            ti, tj = torch.from_numpy(ii).to(dev), torch.from_numpy(jj).to(dev)
            p32, q32 = P[i][ti, :r].cpu().numpy(), Q[i][tj, :r].cpu().numpy()
            ph, qh = p32.astype(np.float64), q32.astype(np.float64)
            # the oracle's reconstruction of the sampled elements (rounded to the gradient's dtype as it rounds)
            want_o = np.array([orc.reconstruct_one(p32[k:k + 1], q32[k:k + 1], 0, 0, code) for k in range(len(ii))])
            got_o = out[i][ii, jj].float().cpu().numpy()
            bound = tol * np.linalg.norm(ph, axis=1) * np.linalg.norm(qh, axis=1) + 1e-12
            assert (np.abs(got_o - want_o) <= bound).all(), (step, i)
            d_prev.append(res[i][ii, jj].cpu().numpy())
            out_prev.append(got_o)
        r_prev = r
    for c in ctxs + [ectx, seeder]:
        c.close()
