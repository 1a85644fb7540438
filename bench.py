#!/usr/bin/env python3
"""Benchmark of the EDGC hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic layer
gradients: the down-sampled entropy estimate (sample, range, histogram,
entropy) over every 2-D gradient of the workload, the host rank rule
(edgc_select_rank) on the entropies, whose decision is the rank the step
compresses at, and rank-r compress + decompress of every gradient with the
error-feedback residual carried from the previous step.  Inputs are resident
in HBM before the timed region starts.  Prints ONE JSON line.

Default: the hidden-5120 block with bf16 gradients (BASELINE config 4) at rank
128 is the headline (`value`, `roofline`, `cpu_baseline`); the same block at
ranks 32 and 64, the hidden-2048 fp32 block (config 2) and the 8-layer
hidden-4096 fp32 stage (config 5's shapes, fixed rank 64) are measured in the
same process and reported under `other_workloads`, and config 5's dynamic-rate
run (200 steps, window 20, ranks {4..64} chosen by edgc_select_rank, residual
kept across rank changes) under `dynamic`.

Layout of a step: the layers are split into two groups; each group goes
through the batched entry points (one launch sequence per group, on a stream
of its own, so that one group's small kernels run beside the other's streaming
passes); one stage-level entropy estimate over all the gradient buffers runs
on a third stream; the error-feedback residual is kept in the deferred form
(the buffer holds D = G + E, the next step's P-pass subtracts P^ Q^T on the
way; `--explicit-residual` stores E instead).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--rank R]
                    [--no-cpu-baseline] [--no-extras]
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published
BF16_MFMA_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA, published
METRIC = "gradient GB/s through entropy+rank-r compress/decompress; % HBM/MFMA roofline"
HEADLINE = ("cfg4_gpt_h5120_bf16", 128)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=HEADLINE[0])
    ap.add_argument("--rank", type=int, default=0, help="override the workload's rank (the default workload runs at 128)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the headline workload: leave out `other_workloads` and `dynamic`")
    ap.add_argument("--dynamic", action="store_true", help="only config 5's dynamic-rate run (the `dynamic` object)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device copy of 1 GiB five times (reference for the rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    ap.add_argument("--batch", type=int, default=2,
                    help="groups the layers are split into (balanced by size), each one launch sequence on its own stream")
    ap.add_argument("--explicit-residual", action="store_true",
                    help="keep E = D - M^ in the residual buffer between steps (the decompress reads D and writes E) "
                         "instead of the default deferred subtraction")
    ap.add_argument("--ent-strides", default="1000,100,10,1", help="cfg3_flat_1e9 only: the sampling strides to run")
    ap.add_argument("--ent-bins", default="256,4096,65536", help="cfg3_flat_1e9 only: the bin counts to run")
    ap.add_argument("--ent-dtypes", default="f32,bf16", help="cfg3_flat_1e9 only: the element types to run")
    ap.add_argument("--ent-chunk", type=int, default=64, help="cfg3_flat_1e9 only: elements per sampled chunk")
    ap.add_argument("--serial", action="store_true",
                    help="issue everything on ONE stream, also in the timed region: the run to put under "
                         "rocprofv3 --kernel-trace --stats, every kernel alone on the GPU")
    return ap.parse_args()


def traffic_from_profile(workload: str, rank: int, kernel: str, folder: str = None):
    """HBM-side bytes per launch of `kernel` from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary of this
    workload and rank under profiles/ (written by paper_2511_10333_amd/profile_summary.py from the counter CSVs);
    None when no such summary is there."""
    path = os.path.join(folder or os.path.join(ROOT, "profiles"), "traffic_%s_r%d.md" % (workload, rank))
    try:
        text = open(path).read()
    except OSError:
        return None, None
    m = re.search(r"^traffic_bytes_per_launch\s+%s\s+([0-9.eE+]+)\s*$" % re.escape(kernel), text, re.M)
    return (int(float(m.group(1))), os.path.relpath(path, ROOT)) if m else (None, None)


# ---------------------------------------------------------------------------------------------
# one workload at one rank, resident on the device
# ---------------------------------------------------------------------------------------------
class Workload:
    def __init__(self, torch, edgc, gen, name, rank, args, mats=None, allowed=None, r_min=None, r_ref=0,
                 window=1, total_iters=0, ref_shape=None):
        import numpy as np
        from paper_2511_10333_amd.binding import ENTROPY_RESULT_BYTES
        self.torch, self.edgc, self.name = torch, edgc, name
        w = self.w = gen.WORKLOADS[name]
        self.r_max = rank
        self.bf16 = w["dtype"] == "bf16"
        self.mats = mats if mats is not None else gen.workload_matrices(name)
        self.serial = args.serial
        self.skip_estimate = False    # only for the side measurement of what the estimate costs a step
        self.deferred = not args.explicit_residual
        self.NBUF = 3     # entropy results are read two steps after they are enqueued: the GPU never waits for the host
        n_groups = max(1, min(args.batch, len(self.mats)))
        self.streams = [torch.cuda.Stream() for _ in range(n_groups)]
        self.estream = torch.cuda.Stream()
        if args.serial:
            self.streams = [self.streams[0]] * n_groups
            self.estream = self.streams[0]
        ldf = (rank + 3) // 4 * 4
        self.layers = []
        self.qctx = qctx = edgc.Context(0, max_bins=16, max_rank=max(rank, 4), max_rows=64, max_cols=64)
        for li, (spec, g) in enumerate(self.mats):
            if isinstance(g, torch.Tensor):
                G = g
            elif self.bf16:
                G = torch.from_numpy(g.view(np.int16).copy()).cuda().view(torch.bfloat16)
            else:
                G = torch.from_numpy(g).cuda()
            Q = torch.zeros((spec.n, ldf), dtype=torch.float32, device="cuda")
            torch.cuda.synchronize()
            qctx.init_q(Q, 0, rank, w["seed"] + li)
            self.layers.append(dict(spec=spec, G=G, Q=Q,
                                    E=torch.empty((spec.m, spec.n), dtype=torch.float32, device="cuda"),
                                    P=torch.empty((spec.m, ldf), dtype=torch.float32, device="cuda"),
                                    out=torch.empty_like(G)))
        torch.cuda.synchronize()
        # groups: largest layer first into the lightest group
        order = sorted(range(len(self.layers)), key=lambda i: -self.layers[i]["spec"].m * self.layers[i]["spec"].n)
        members = [[] for _ in range(n_groups)]
        load = [0] * n_groups
        for i in order:
            k = load.index(min(load))
            members[k].append(i)
            load[k] += self.layers[i]["spec"].m * self.layers[i]["spec"].n
        self.groups = []
        for k, idx in enumerate(members):
            idx.sort()
            gctx = edgc.Context(0, max_bins=16, max_rank=max(rank, 4), max_rows=64, max_cols=64)
            gctx.reserve_batch([(self.layers[i]["spec"].m, self.layers[i]["spec"].n) for i in idx])
            tensors = [edgc.Tensor(self.layers[i]["G"], self.layers[i]["out"], self.layers[i]["E"], self.layers[i]["Q"],
                                   self.layers[i]["P"], True) for i in idx]
            self.groups.append(dict(ctx=gctx, tensors=tensors, prep=edgc.PreparedBatch(tensors), stream=self.streams[k], idx=idx))
        # ONE stage-level entropy estimate per step over all gradient buffers (the paper's rank is per stage)
        self.ectx = edgc.Context(0, max_bins=w["bins"], max_rank=4, max_rows=64, max_cols=64)
        self.flats = [L["G"].view(-1) for L in self.layers]
        # The first window is the reference of Theorem 3 (Sec. IV-D-2: the initial gradients); a run on fixed
        # synthetic gradients has no training behind it, so the reference window's estimate reads the gradients at
        # twice the scale (exact in bf16 and fp32): the entropy then falls by ln 2, as it does early in training,
        # the rule leaves warm-up and its decisions, not a constant, are the ranks the steps compress at.
        self.flats_ref = [(f * 2).contiguous() for f in self.flats]
        self.ent = [torch.empty(ENTROPY_RESULT_BYTES, dtype=torch.uint8, pin_memory=True) for _ in range(self.NBUF)]
        for st in set(self.streams + [self.estream]):
            with torch.cuda.stream(st):
                torch.zeros(1, device="cuda")    # a stream's hardware queue is set up at its first submission
        torch.cuda.synchronize()
        ref = min(self.mats, key=lambda t: t[0].m * t[0].n)[0]
        ref_m, ref_n = ref_shape if ref_shape else (ref.m, ref.n)     # the shape g(r; m, n) is evaluated at
        self.allowed = list(allowed) if allowed else [rank]
        self.prm = edgc.RankParams(ref_m, ref_n, r_min=r_min if r_min else rank, r_max=rank, step_limit=8,
                                   allowed=self.allowed, total_iters=total_iters, min_warmup_frac=0.10, r_ref=r_ref)
        self.window = window
        self.state = edgc.RankState()
        self.decisions = []
        self.H_window = []
        self.cur_rank = rank            # until the rule decides (rank 0 = warm-up: the start rank stays)
        self.rank_changes = []
        self.step_events = [[torch.cuda.Event() for _ in range(n_groups + 1)] for _ in range(self.NBUF)]
        self.t = 0
        self.grad_bytes = sum(s.m * s.n for s, _ in self.mats) * (2 if self.bf16 else 4)
        self.ctxs_all = [g["ctx"] for g in self.groups] + [self.ectx, self.qctx]

    # the rank rule consumes the entropies of step t-2 (on the host by now), so that one whole step is always
    # queued on the GPU while the host works; a decision is taken at the end of every window
    def rank_rule(self, t):
        if t < 2:
            return
        for ev in self.step_events[(t - 2) % self.NBUF]:
            ev.synchronize()
        res = self.edgc.EntropyResult.from_buffer(self.ent[(t - 2) % self.NBUF].numpy().tobytes())
        self.H_window.append(res.h_diff_nats)
        if len(self.H_window) < self.window:
            return
        d = self.edgc.select_rank(self.state, self.H_window, len(self.H_window), self.prm)
        self.H_window = []
        self.decisions.append(d.rank)
        if d.rank and d.rank != self.cur_rank:
            self.change_rank(d.rank, t)

    # Rank change between steps: the residual is preserved (the deferred form is carried out: E = D - M^ at the
    # old rank), Q keeps its leading columns and new ones are seeded (edgc_init_q); nothing is reallocated.
    def change_rank(self, r_new, t):
        torch = self.torch
        if self.cur_rank == 0:          # leaving warm-up: nothing was compressed yet, Q holds its seeded start
            self.rank_changes.append(dict(step=t, rank_from=0, rank_to=r_new, ms=0.0))
            self.cur_rank = r_new
            return
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        ev0.record(self.streams[0])
        for g in self.groups:
            if self.deferred and not g["tensors"][0].residual_is_zero:
                g["ctx"].residual_materialize_batch(g["tensors"], self.cur_rank, stream=self.streams[0])
            g["materialized"] = True
        if r_new > self.cur_rank:       # a shrink keeps the first r columns; a grow seeds the columns it adds
            for li, L in enumerate(self.layers):
                self.qctx.init_q(L["Q"], self.cur_rank, r_new, self.w["seed"] + li, stream=self.streams[0])
        ev1.record(self.streams[0])
        torch.cuda.synchronize()
        self.rank_changes.append(dict(step=t, rank_from=self.cur_rank, rank_to=r_new, ms=round(ev0.elapsed_time(ev1), 4)))
        self.cur_rank = r_new

    def step(self):
        t = self.t
        if not self.skip_estimate:
            self.rank_rule(t)
        r = self.cur_rank
        flats = self.flats_ref if t < self.window else self.flats
        if not self.skip_estimate:
            self.ectx.entropy_estimate_async(flats, self.w["stride"], self.w["chunk"], self.w["seed"], t, self.w["bins"],
                                             self.ent[t % self.NBUF], stream=self.estream)
        for g in self.groups if r else []:                  # rank 0: warm-up, the gradients go uncompressed
            first = g["tensors"][0].residual_is_zero
            explicit_in = g.pop("materialized", False)      # after a rank change the buffer holds E itself
            g["ctx"].compress_batch(g["prep"], r, stream=g["stream"],
                                    deferred=self.deferred and not first and not explicit_in)
            g["ctx"].decompress_batch(g["prep"], r, stream=g["stream"], deferred=self.deferred)
            for x in g["tensors"]:
                x.residual_is_zero = False
        for si, g in enumerate(self.groups):
            self.step_events[t % self.NBUF][si].record(g["stream"])
        self.step_events[t % self.NBUF][len(self.groups)].record(self.estream)
        self.t = t + 1

    def make_serial(self):
        for g in self.groups:
            g["stream"] = self.streams[0]
        self.estream = self.streams[0]

    def profile_steps(self, steps):
        """`steps` more steps on ONE stream, every launch between its own pair of HIP events."""
        self.torch.cuda.synchronize()
        self.make_serial()
        for c in self.ctxs_all:
            c.profile_begin(max_launches=steps * len(self.layers) * 16 + 64)
        for _ in range(steps):
            self.step()
        stats, overhead_us = {}, 0.0
        for c in self.ctxs_all:
            for name, s in c.profile_end().items():
                acc = stats.setdefault(name, dict(launches=0, total_ms=0.0, bytes=0.0, flops=0.0))
                for k in acc:
                    acc[k] += s[k]
                overhead_us = s["event_overhead_ms"] * 1e3
        return stats, overhead_us

    def close(self):
        self.torch.cuda.synchronize()
        for c in self.ctxs_all:
            c.close()


def kernel_table(stats, steps):
    out = {}
    for name, s in stats.items():
        if not s["launches"]:
            continue
        out[name] = dict(launches_per_step=round(s["launches"] / steps, 3),
                         avg_us=round(s["total_ms"] * 1e3 / s["launches"], 2),
                         gbs=round(s["bytes"] / (s["total_ms"] * 1e-3) / 1e9, 1) if s["total_ms"] > 0 else None,
                         tflops=round(s["flops"] / (s["total_ms"] * 1e-3) / 1e12, 2) if s["total_ms"] > 0 else None)
    return out


def measure(wl, steps, warmup):
    """W untimed steps, K timed steps between synchronisations, then the same K steps once more with every
    launch between HIP events on one stream."""
    torch = wl.torch
    for _ in range(warmup):
        wl.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        wl.step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms = (t1 - t0) * 1e3 / steps
    stats, overhead_us = wl.profile_steps(steps)
    dom = max(stats, key=lambda k: stats[k]["total_ms"])
    ds = stats[dom]
    achieved = ds["bytes"] / (ds["total_ms"] * 1e-3) / 1e9
    return dict(ms_per_step=ms, value=wl.grad_bytes / (ms * 1e-3) / 1e9,
                stats=stats, kernels=kernel_table(stats, steps), dominant=dom, achieved=achieved,
                avg_launch_us=ds["total_ms"] * 1e3 / ds["launches"], bytes_per_launch=ds["bytes"] / ds["launches"],
                event_overhead_us=overhead_us)


def arithmetic_of(bf16):
    return ("bf16 MFMA (32x32x16), fp32 accumulate: contraction operands rounded to bf16" if bf16 else
            "3 x bf16 MFMA (32x32x16) on operands split into two bf16 planes (~2^-17 relative per operand), fp32 accumulate")


def short_line(wl, m):
    """What `other_workloads` carries per workload."""
    return dict(workload=wl.name, rank=wl.r_max, dtype="bf16" if wl.bf16 else "f32", arithmetic=arithmetic_of(wl.bf16),
                layers=len(wl.layers), ms_per_step=round(m["ms_per_step"], 4), gradient_gbs=round(m["value"], 2),
                dominant_kernel=m["dominant"], dominant_gbs=round(m["achieved"], 1),
                dominant_frac_of_hbm_peak=round(m["achieved"] / HBM_PEAK_GBS, 4),
                kernels={k: dict(avg_us=v["avg_us"], gbs=v["gbs"]) for k, v in m["kernels"].items()},
                last_rank_decision=wl.decisions[-1] if wl.decisions else None)


def dynamic_run(torch, edgc, gen, args):
    """BASELINE config 5 at full size: one pipeline stage of 8 layers at hidden 4096 (32 fp32 tensors, 1.61e9
    elements), 200 steps, the spectrum decay of the gradients ramping from 0.90 to 0.99, per-step entropy, a
    20-step window, ranks {4, 8, 16, 32, 64} chosen by edgc_select_rank, the residual preserved across rank changes.
    The gradients of a step are formed on the device (U diag(d^i) V^T + noise from the workload's seeded factors:
    the trainer's part, outside the timed calls); the method's calls of every step are timed with HIP events."""
    import numpy as np
    name = "cfg5_stage8_h4096"
    w = gen.WORKLOADS[name]
    specs = w["layers"]
    k, rep, steps_total, window = w["k"], w["repeat"], 200, 20
    g = torch.Generator(device="cuda").manual_seed(w["seed"])
    factors, grads = [], []
    for spec in specs:
        # columns of variance 1/rows: orthonormal up to O(sqrt(k / rows)), which is all the timing needs
        U = torch.randn(spec.m, k, device="cuda", generator=g) / spec.m ** 0.5
        V = torch.randn(spec.n, k, device="cuda", generator=g) / spec.n ** 0.5
        Z = torch.randn(spec.m, spec.n, device="cuda", generator=g) * w["noise"]
        factors.append((U, V.T.contiguous(), Z))
        grads.append(torch.empty(spec.m, spec.n, device="cuda"))
    expo = torch.arange(k, device="cuda", dtype=torch.float32)

    def set_gradients(t):
        d = 0.90 + 0.09 * t / (steps_total - 1)
        s = torch.pow(torch.tensor(d, device="cuda"), expo)
        for (U, Vt, Z), G in zip(factors, grads):
            torch.addmm(Z, U * s, Vt, out=G)

    set_gradients(0)
    mats = [(gen.LayerSpec("L%d.%s" % (layer, spec.name), spec.m, spec.n), G)
            for layer in range(rep) for spec, G in zip(specs, grads)]
    # g(r; m, n) at the reference shape 128 x 128: which shape of a stage feeds g is the caller's choice, and at
    # this one the ramp's entropy change (1.1 nats) spans the allowed ranks; r_ref = 4: the run's entropy rises,
    # so compression starts at the lower bound (with the paper's r0 = r_max such a run never leaves warm-up)
    wl = Workload(torch, edgc, gen, name, 64, args, mats=mats, allowed=[4, 8, 16, 32, 64], r_min=4, r_ref=4,
                  window=window, total_iters=steps_total, ref_shape=(128, 128))
    wl.cur_rank = 0                  # warm-up (Sec. IV-D-2): no compression until the rule decides
    wl.flats_ref = wl.flats          # the ramp itself moves the entropy: no stand-in for the reference window
    per_rank = {}
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    wl.make_serial()                 # per-step event timing: everything on one stream
    for t in range(steps_total):
        set_gradients(t)
        torch.cuda.synchronize()
        ev[0].record(wl.streams[0])
        wl.step()
        ev[1].record(wl.streams[0])
        torch.cuda.synchronize()
        per_rank.setdefault(wl.cur_rank, []).append(ev[0].elapsed_time(ev[1]))
    out = dict(workload=name, what="config 5: 200 steps, decay 0.90 -> 0.99, window 20, ranks {4, 8, 16, 32, 64} from "
                                   "edgc_select_rank (r_ref = 4, g at 128x128), residual kept across rank changes; "
                                   "rank 0 = warm-up (entropy estimate only); one stream, HIP events around every "
                                   "step's calls (rank rule, entropy estimate, compress, decompress)",
               steps=steps_total, window=window, decisions=wl.decisions,
               ms_per_step_by_rank={str(r): dict(steps=len(v), ms=round(float(np.median(v)), 4),
                                                 gradient_gbs=round(wl.grad_bytes / (float(np.median(v)) * 1e-3) / 1e9, 1))
                                    for r, v in sorted(per_rank.items())},
               rank_changes=wl.rank_changes,
               rank_change_what="edgc_residual_materialize_batch over the stage (E = D - M^ at the old rank) plus "
                                "edgc_init_q of the new Q columns; ms from HIP events")
    wl.close()
    return out


def cpu_baseline_for(wl, torch):
    """The oracle as it stands on a bounded sample of the workload: its attention-projection gradient (the
    smallest matrix), one step = entropy of its 1 % sample + compress + decompress at the workload's rank; with
    all host threads and, on its first quarter of rows, with one."""
    import numpy as np
    from oracle import edgc_oracle as orc
    w, r = wl.w, wl.r_max
    li = min(range(len(wl.mats)), key=lambda i: wl.mats[i][0].m * wl.mats[i][0].n)
    spec, g = wl.mats[li]
    if isinstance(g, torch.Tensor):
        g = g.cpu().numpy() if not wl.bf16 else g.view(torch.int16).cpu().numpy().view(np.uint16)
    code = orc.BF16 if wl.bf16 else orc.F32
    esz = 2 if wl.bf16 else 4

    def one_step(G):
        Q0 = np.zeros((G.shape[1], r), dtype=np.float32)
        orc.init_q(Q0, 0, r, w["seed"] + li)
        t0 = time.perf_counter()
        orc.entropy(G.reshape(-1), w["stride"], w["chunk"], w["seed"], 0, w["bins"])
        P, Q1, D = orc.compress(G, None, Q0, r)
        orc.decompress(P, Q1, D, code)
        return time.perf_counter() - t0

    n_all = orc.num_threads()
    t_all = one_step(g)
    rows1 = max(r, spec.m // 4)
    g1 = np.ascontiguousarray(g[:rows1])
    orc.set_num_threads(1)
    try:
        t_one = one_step(g1)
    finally:
        orc.set_num_threads(n_all)
    return dict(value=round(g.size * esz / t_all / 1e9, 5), unit="GB/s", cores=n_all, kind="oracle",
                seconds=round(t_all, 2),
                sample="one step (entropy of the 1 %% sample, compress, decompress at rank %d) of the workload's %dx%d "
                       "%s gradient, oracle as it stands" % (r, spec.m, spec.n, spec.name),
                single_thread=dict(value=round(g1.size * esz / t_one / 1e9, 5), unit="GB/s", cores=1,
                                   seconds=round(t_one, 2),
                                   sample="the same step on the first %d rows of that gradient" % rows1))


def main() -> int:
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one rank's gradient shard, no collectives); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    import torch

    import edgc_inputs as gen
    import paper_2511_10333_amd as edgc

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")     # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4,
                          "launches": 5}))
        return 0

    if args.workload == "cfg3_flat_1e9":
        from bench_entropy import entropy_sweep
        return entropy_sweep(args, torch, edgc, METRIC, HBM_PEAK_GBS)

    if args.dynamic:
        print(json.dumps({"metric": METRIC, "dynamic": dynamic_run(torch, edgc, gen, args)}))
        return 0

    name = args.workload
    w = gen.WORKLOADS[name]
    r = args.rank or (HEADLINE[1] if name == HEADLINE[0] else w["rank"])
    t_setup = time.perf_counter()
    wl = Workload(torch, edgc, gen, name, r, args)
    m = measure(wl, args.steps, args.warmup)
    traffic, traffic_src = traffic_from_profile(name, r, m["dominant"])
    roofline = dict(bound="hbm", kernel=m["dominant"], achieved=round(m["achieved"], 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(m["achieved"] / HBM_PEAK_GBS, 4), traffic=traffic, traffic_from=traffic_src,
                    avg_launch_us=round(m["avg_launch_us"], 2),
                    algorithmic_bytes_per_launch=round(m["bytes_per_launch"]),
                    timing="HIP events around every launch (minus %.2f us, what an empty event pair reads); "
                           "second pass of the same K steps, launches serialised on one stream" % m["event_overhead_us"])
    # MFMA utilisation of the instruction issued, beside the most an HBM-bound pass could reach:
    # ceiling = min(1, arithmetic intensity / ridge), ridge = bf16 MFMA peak / HBM peak
    ridge = BF16_MFMA_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)
    st = m["stats"]
    mfma = {k: dict(tflops=v["tflops"], frac_of_bf16_peak=round(v["tflops"] / BF16_MFMA_PEAK_TFLOPS, 4),
                    flop_per_byte=round(st[k]["flops"] / st[k]["bytes"], 2),
                    ceiling=round(min(1.0, st[k]["flops"] / st[k]["bytes"] / ridge), 4))
            for k, v in m["kernels"].items()
            if k in ("k_pass_p", "k_pass_p_deferred", "k_pass_q", "k_decompress") and v["tflops"]}

    # what a plain copy, a plain read and a bf16 MFMA loop reach on this device
    pa = torch.ones(1 << 28, dtype=torch.float32, device="cuda")          # 1 GiB each
    pb = torch.empty_like(pa)
    torch.cuda.synchronize()
    peaks = wl.qctx.measure_device_peaks(pa, pb, reps=10)
    del pa, pb
    device_peaks = dict(copy_gbs=round(peaks["copy_gbs"], 1), read_gbs=round(peaks["read_gbs"], 1),
                        write_gbs=round(peaks["write_gbs"], 1),
                        mfma_bf16_tflops=round(peaks["mfma_bf16_tflops"], 1), bytes=peaks["bytes"],
                        what="plain copy (read + written bytes), plain read, plain fill, register-resident "
                             "32x32x16 bf16 MFMA loop; 10 launches each between one pair of events")
    # each streaming pass against the plain kernel of its own traffic mix: the P-pass reads and writes
    # (copy), the Q-pass only reads, the deferred decompress only writes
    against = {"k_pass_p_deferred": "copy_gbs", "k_pass_p": "copy_gbs", "k_pass_q": "read_gbs",
               "k_decompress": "write_gbs" if wl.deferred else "copy_gbs"}
    for k, ref in against.items():
        if k in m["kernels"] and m["kernels"][k].get("gbs"):
            m["kernels"][k]["frac_of_measured_" + ref[:-4]] = round(m["kernels"][k]["gbs"] / peaks[ref], 4)
    roofline["frac_of_measured_copy"] = round(m["achieved"] / peaks["copy_gbs"], 4)

    cpu_baseline = None if args.no_cpu_baseline else cpu_baseline_for(wl, torch)

    line = {
        "metric": METRIC,
        "value": round(m["value"], 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(m["ms_per_step"], 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if wl.bf16 else "f32", "arithmetic": arithmetic_of(wl.bf16),
        "data": "synthetic",
        "config": {"workload": name, "layers": ["%dx%d" % (s.m, s.n) for s, _ in wl.mats],
                   "rank": r, "stride": w["stride"], "chunk": w["chunk"], "bins": w["bins"],
                   "streams": 1 if args.serial else len(wl.groups), "entropy_streams": 0 if args.serial else 1,
                   "batch_groups": len(wl.groups), "residual": "deferred" if wl.deferred else "explicit",
                   "rank_rule": "edgc_select_rank every step on the stage entropy of step t-2, r_min = r_max = %d "
                                "(config 4 fixes the rank); its decision is the rank the step compresses at" % r,
                   "gradient_bytes_per_step": wl.grad_bytes},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "kernels": m["kernels"], "mfma": mfma,
        "device_peaks_measured": device_peaks,
        "last_rank_decision": wl.decisions[-1] if wl.decisions else None,
    }
    mats_keep = wl.mats
    wl.close()
    del wl
    torch.cuda.empty_cache()

    if not args.no_extras and name == HEADLINE[0] and not args.rank:
        others = []
        extra_steps = max(5, min(args.steps, 20))
        for ename, er in [(HEADLINE[0], 32), (HEADLINE[0], 64), ("cfg2_gpt_h2048_r16", 16), ("cfg5_stage8_h4096", 64)]:
            e = Workload(torch, edgc, gen, ename, er, args, mats=mats_keep if ename == HEADLINE[0] else None)
            others.append(short_line(e, measure(e, extra_steps, max(3, min(args.warmup, 5)))))
            others[-1]["steps"] = extra_steps
            e.close()
            del e
            torch.cuda.empty_cache()
        line["other_workloads"] = others
        # What the separate entropy estimate costs a step: the headline workload once more with the estimate
        # left out (NOT a valid step: the bound on what fusing the estimate into the P-pass could save)
        e = Workload(torch, edgc, gen, HEADLINE[0], HEADLINE[1], args, mats=mats_keep)
        e.skip_estimate = True
        for _ in range(args.warmup):
            e.step()
        torch.cuda.synchronize()
        tq0 = time.perf_counter()
        for _ in range(args.steps):
            e.step()
        torch.cuda.synchronize()
        ms_wo = (time.perf_counter() - tq0) * 1e3 / args.steps
        e.close()
        del e
        torch.cuda.empty_cache()
        line["entropy_estimate_cost"] = dict(
            ms_per_step=round(m["ms_per_step"], 4), ms_per_step_without_estimate=round(ms_wo, 4),
            difference_us=round((m["ms_per_step"] - ms_wo) * 1e3, 1),
            what="the headline workload again with the estimate's launches (and the rank rule's host call) left out: "
                 "what a step pays for the separate estimate (it runs on a stream of its own beside the passes), i.e. "
                 "the most a fused estimate could save")
        del mats_keep
        line["dynamic"] = dynamic_run(torch, edgc, gen, args)
    line["wall_seconds"] = round(time.perf_counter() - t_setup, 1)
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
