#!/usr/bin/env python3
"""Benchmark of the EDGC hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic layer
gradients: the down-sampled entropy estimate (sample, range, histogram,
entropy) of every 2-D gradient of the workload, the host rank rule on the
step's entropies, and rank-r compress + decompress of every gradient with the
error-feedback residual carried from the previous step.  Inputs are resident
in HBM before the timed region starts.  Prints ONE JSON line.

Default layout: the layers are split into two groups; each group goes through
the batched entry points (one launch sequence per group, on a stream of its
own, so that one group's small kernels run beside the other's streaming
passes); one stage-level entropy estimate over all the gradient buffers runs
on a third stream; the error-feedback residual is kept in the deferred form
(the buffer holds D = G + E, the next step's P-pass subtracts P^ Q^T on the
way; `--explicit-residual` stores E instead).  `--batch 0` runs one call chain
and one estimate per layer.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
BF16_MFMA_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA, published

# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# runs of this command (see profiles/), keyed by (workload, kernel, batch groups, form of the residual); None for a
# layout that has no such run recorded.
MEASURED_TRAFFIC_BYTES = {
    # profiles/k_pass_p_cfg2_explicit_residual_traffic.md: (2 x FETCH_SIZE + WRITE_SIZE) KiB per launch, the factors
    # coming from the same counters on a plain 1 GiB device copy (FETCH_SIZE reads half the bytes)
    ("cfg2_gpt_h2048_r16", "k_pass_p", 2, "explicit"): int((2 * 9.764e4 + 1.125e5) * 1024),
    # profiles/k_pass_p_deferred_cfg2_traffic.md, the same way
    ("cfg2_gpt_h2048_r16", "k_pass_p_deferred", 2, "deferred"): int((2 * 1.01527e5 + 1.12512e5) * 1024),
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg2_gpt_h2048_r16")
    ap.add_argument("--rank", type=int, default=0, help="override the workload's rank")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device copy of 1 GiB five times (reference for the rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    ap.add_argument("--graph", action="store_true",
                    help="replay the compress/decompress launches from a captured HIP graph instead of issuing "
                         "them eagerly (measured slower here: the graph's branches overlap less than the streams)")
    ap.add_argument("--no-graph", action="store_true", help="kept for compatibility: eager launches are the default")
    ap.add_argument("--batch", type=int, default=2,
                    help="N > 0 (default 2): compress/decompress through the batched entry points, the layers split "
                         "into N groups (balanced by size), each group one launch sequence on its own stream and one "
                         "stage-level entropy estimate; 0: one call chain per layer")
    ap.add_argument("--ent-streams", type=int, default=0,
                    help="streams the entropy estimates are spread over; 0 = one in batched mode (compress streams "
                         "+ entropy stream stay within the 4 hardware queues), else one per compress stream")
    ap.add_argument("--explicit-residual", action="store_true",
                    help="batched mode: keep E = D - M^ in the residual buffer between steps (the decompress reads D "
                         "and writes E) instead of the default deferred subtraction, where the buffer keeps D, the "
                         "decompress only writes the reconstruction and the next P-pass subtracts P^ Q^T on the way")
    ap.add_argument("--serial", action="store_true",
                    help="issue everything on ONE stream, also in the timed region (what the per-kernel second pass "
                         "always does): the run to put under rocprofv3 --kernel-trace --stats, every kernel alone on the GPU")
    ap.add_argument("--streams", type=int, default=0,
                    help="HIP streams (one library context each) the layers or groups are spread over; "
                         "0 = one per group in batched mode, else one per layer")
    return ap.parse_args()


def entropy_sweep(args, np, torch, edgc) -> int:
    """The entropy-only workload: one flat buffer of 1e9 elements (fp32, then bf16), Laplace(0, 1e-3)
    with 0.1 % of the values at 100 times the scale, generated on the device; sampling strides 1000,
    100, 10 and 1 (0.1 % to 100 %) times 256, 4096 and 65536 bins.  One "step" is one estimate
    (range, histogram, entropy) of one cell; the JSON line carries every cell and, as `value`, the
    100 % / 4096-bin cell of the fp32 buffer, whose two passes read the whole buffer twice."""
    from paper_2511_10333_amd.binding import ENTROPY_RESULT_BYTES, EntropyResult
    n, chunk, seed = 1_000_000_000, 64, 0
    strides, bins_list = (1000, 100, 10, 1), (256, 4096, 65536)
    ctx = edgc.Context(0, max_bins=65536, max_rank=4, max_rows=64, max_cols=64)
    out = torch.empty(ENTROPY_RESULT_BYTES, dtype=torch.uint8, pin_memory=True)
    g = torch.Generator(device="cuda").manual_seed(3)
    x32 = torch.empty(n, device="cuda")
    x32.exponential_(1.0, generator=g)                                  # |Laplace(0, 1)|
    sign = torch.empty(n, device="cuda").uniform_(-1.0, 1.0, generator=g)
    x32.mul_(torch.sign(sign))
    x32.mul_(torch.where(sign.abs() < 1e-3, 1e-1, 1e-3))               # 0.1 % outliers at 100 x the scale
    del sign
    bufs = {"f32": x32, "bf16": x32.bfloat16()}
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    cells, headline = [], None
    for dtype, x in bufs.items():
        esz = x.element_size()
        for stride in strides:
            reps = args.steps if stride > 1 else max(3, args.steps // 5)
            for bins in bins_list:
                for w in range(max(1, min(args.warmup, 3))):
                    ctx.entropy_estimate_async(x, stride, chunk, seed, w, bins, out)
                torch.cuda.synchronize()
                ev0.record()
                for t in range(reps):
                    ctx.entropy_estimate_async(x, stride, chunk, seed, t, bins, out)
                ev1.record()
                torch.cuda.synchronize()
                ms = ev0.elapsed_time(ev1) / reps
                res = EntropyResult.from_buffer(out.numpy().tobytes())
                # the same launches once more, each kernel between its own pair of events
                ctx.profile_begin(4 * reps + 8)
                for t in range(reps):
                    ctx.entropy_estimate_async(x, stride, chunk, seed, t, bins, out)
                torch.cuda.synchronize()
                ks = ctx.profile_end()
                kern = {k: dict(avg_us=round(v["total_ms"] * 1e3 / v["launches"], 2),
                                gbs=round(v["bytes"] / (v["total_ms"] * 1e-3) / 1e9, 1))
                        for k, v in ks.items() if v["launches"] and v["total_ms"] > 0}
                sample_bytes = res.n_sampled * esz
                cell = dict(dtype=dtype, stride=stride, bins=bins, n_sampled=res.n_sampled, ms=round(ms, 4),
                            gradient_gbs=round(n * esz / (ms * 1e-3) / 1e9, 1),
                            sample_gbs_two_passes=round(2 * sample_bytes / (ms * 1e-3) / 1e9, 1),
                            H_bits=round(res.H_bits, 6), kernels=kern)
                cells.append(cell)
                if dtype == "f32" and stride == 1 and bins == 4096:
                    headline = (cell, ms, ks, reps)
    cell, ms, ks, reps = headline
    dom = max(("k_minmax", "k_hist"), key=lambda k: ks[k]["total_ms"])
    achieved = ks[dom]["bytes"] / (ks[dom]["total_ms"] * 1e-3) / 1e9
    pa = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
    pb = torch.empty_like(pa)
    peaks = ctx.measure_device_peaks(pa, pb, reps=10)
    del pa, pb
    roofline = dict(bound="hbm", kernel=dom, achieved=round(achieved, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(achieved / HBM_PEAK_GBS, 4), traffic=None,
                    avg_launch_us=round(ks[dom]["total_ms"] * 1e3 / ks[dom]["launches"], 2),
                    algorithmic_bytes_per_launch=round(ks[dom]["bytes"] / ks[dom]["launches"]),
                    frac_of_measured_read=round(achieved / peaks["read_gbs"], 4),
                    timing="HIP events around every launch, second pass of the same estimates")
    cpu_baseline = None
    if not args.no_cpu_baseline:
        from oracle import edgc_oracle as orc
        host = x32[:100_000_000].cpu().numpy()
        tc0, k = time.perf_counter(), 0
        while True:
            orc.entropy(host, 1, chunk, seed, k, 4096)
            k += 1
            tc1 = time.perf_counter()
            if tc1 - tc0 >= 10.0 or k >= 50:
                break
        cpu_baseline = dict(value=round(k * host.nbytes / (tc1 - tc0) / 1e9, 4), unit="GB/s",
                            cores=orc.num_threads(), kind="oracle", seconds=round(tc1 - tc0, 2),
                            sample="%d estimates of the first 1e8 elements of the fp32 buffer, every element "
                                   "sampled, 4096 bins, oracle as it stands" % k)
    line = {
        "metric": "gradient GB/s through entropy+rank-r compress/decompress; % HBM/MFMA roofline",
        "value": cell["gradient_gbs"], "unit": "GB/s", "n_gpus": 1, "steps": reps, "warmup": min(args.warmup, 3),
        "ms_per_step": cell["ms"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "cfg3_flat_1e9", "what": "entropy estimate only; value = the 100 % / 4096-bin "
                   "cell of the fp32 buffer", "elements": n, "chunk": chunk, "strides": list(strides),
                   "bins": list(bins_list)},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "cells": cells,
        "device_peaks_measured": {k: (round(v, 1) if isinstance(v, float) else v) for k, v in peaks.items()},
    }
    print(json.dumps(line))
    return 0


def main() -> int:
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one rank's gradient shard, no collectives); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import edgc_inputs as gen
    import paper_2511_10333_amd as edgc
    from paper_2511_10333_amd.binding import ENTROPY_RESULT_BYTES

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
        return entropy_sweep(args, np, torch, edgc)

    w = gen.WORKLOADS[args.workload]
    r = args.rank or w["rank"]
    bf16 = w["dtype"] == "bf16"
    mats = gen.workload_matrices(args.workload)
    max_m = max(s.m for s, _ in mats)
    max_n = max(s.n for s, _ in mats)
    n_streams = args.streams or (min(args.batch, len(mats)) if args.batch > 0 else len(mats))
    # one context (scratch) per stream: independent layers overlap their small kernels
    ctxs = [edgc.Context(0, max_bins=w["bins"], max_rank=max(r, 4), max_rows=max_m, max_cols=max_n)
            for _ in range(n_streams)]
    streams = [torch.cuda.Stream() for _ in range(n_streams)]
    # the entropy estimate only reads the gradient and uses scratch of its own, so it runs on a
    # stream of its own beside the layer's compress/decompress chain
    n_ent = args.ent_streams or (1 if args.batch > 0 else n_streams)
    ent_streams = [torch.cuda.Stream() for _ in range(n_ent)] if (n_streams > 1 or args.ent_streams or args.batch > 0) else streams
    if args.serial:
        streams = [streams[0]] * n_streams
        ent_streams = [streams[0]] * n_ent
    n_ent = len(ent_streams)
    ctx = ctxs[0]

    NBUF = 3   # entropy results are read two steps after they are enqueued: the GPU never waits for the host
    # device state per layer: gradient, residual, warm-started Q, P, output
    layers = []
    for li, (spec, g) in enumerate(mats):
        if bf16:
            G = torch.from_numpy(g.view(np.int16).copy()).cuda().view(torch.bfloat16)
        else:
            G = torch.from_numpy(g).cuda()
        ldf = (r + 3) // 4 * 4
        Q = torch.zeros((spec.n, ldf), dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        # on the stream that will own the layer: the runtime sets a stream's hardware queue up at its
        # first submission (milliseconds), which belongs to the set-up, not to a step
        ctx.init_q(Q, 0, r, w["seed"] + li, stream=streams[li % n_streams])
        layers.append(dict(
            spec=spec, G=G, Q=Q, ctx=ctxs[li % n_streams], stream=streams[li % n_streams],
            estream=ent_streams[li % n_ent],
            E=torch.empty((spec.m, spec.n), dtype=torch.float32, device="cuda"),
            P=torch.empty((spec.m, ldf), dtype=torch.float32, device="cuda"),
            out=torch.empty_like(G), fresh=True,
            ent=[torch.empty(ENTROPY_RESULT_BYTES, dtype=torch.uint8, pin_memory=True) for _ in range(NBUF)],
        ))
    for st in ent_streams:
        with torch.cuda.stream(st):
            torch.zeros(1, device="cuda")     # first submission on the entropy stream, as above
    torch.cuda.synchronize()

    # batched mode: groups of layers, each with a context whose batch slots fit the group
    groups = []
    if args.batch > 0:
        order = sorted(range(len(layers)), key=lambda i: -layers[i]["spec"].m * layers[i]["spec"].n)
        members = [[] for _ in range(min(args.batch, len(layers)))]
        load = [0] * len(members)
        for i in order:                                  # largest first into the lightest group
            k = load.index(min(load))
            members[k].append(i)
            load[k] += layers[i]["spec"].m * layers[i]["spec"].n
        for k, idx in enumerate(members):
            idx.sort()
            gctx = edgc.Context(0, max_bins=16, max_rank=max(r, 4), max_rows=64, max_cols=64)
            gctx.reserve_batch([(layers[i]["spec"].m, layers[i]["spec"].n) for i in idx])
            tensors = [edgc.Tensor(layers[i]["G"], layers[i]["out"], layers[i]["E"], layers[i]["Q"],
                                   layers[i]["P"], True) for i in idx]
            groups.append(dict(ctx=gctx, tensors=tensors, stream=streams[k % n_streams]))
        # ONE stage-level entropy estimate per step over all gradient buffers of the workload
        # (the paper's rank is per stage), on a stream of its own
        stage = dict(ectx=edgc.Context(0, max_bins=w["bins"], max_rank=4, max_rows=64, max_cols=64),
                     estream=ent_streams[0], flats=[L["G"].view(-1) for L in layers],
                     ent=[torch.empty(ENTROPY_RESULT_BYTES, dtype=torch.uint8, pin_memory=True) for _ in range(NBUF)])
        ctxs_all = ctxs + [g["ctx"] for g in groups] + [stage["ectx"]]
    else:
        ctxs_all = ctxs

    ref = min(mats, key=lambda t: t[0].m * t[0].n)[0]
    prm = edgc.RankParams(ref.m, ref.n, r_min=r, r_max=r, step_limit=8, allowed=[r],
                          total_iters=args.steps + args.warmup, min_warmup_frac=0.10)
    state = edgc.RankState()
    decisions = []
    step_events = [[torch.cuda.Event() for _ in range(n_streams + n_ent)] for _ in range(NBUF)]
    counter = {"step": 0}

    for L in layers:
        L["flat"] = L["G"].view(-1)
    graph = {"g": None}

    def rank_rule(t):
        # the rank rule consumes the entropies of step t-2 (on the host by now), so that one
        # whole step is always queued on the GPU while the host works
        if t > 1:
            for ev in step_events[(t - 2) % NBUF]:
                ev.synchronize()
            H = [edgc.EntropyResult.from_buffer(x["ent"][(t - 2) % NBUF].numpy().tobytes()).h_diff_nats
                 for x in ([stage] if groups else layers)]
            decisions.append(edgc.select_rank(state, H, 1, prm))

    deferred = bool(groups) and not args.explicit_residual

    def compress_all():
        if groups:
            for g in groups:
                first = g["tensors"][0].residual_is_zero     # nothing to subtract yet
                g["ctx"].compress_batch(g["tensors"], r, stream=g["stream"], deferred=deferred and not first)
                g["ctx"].decompress_batch(g["tensors"], r, stream=g["stream"], deferred=deferred)
                for t in g["tensors"]:
                    t.residual_is_zero = False
            return
        for L in layers:
            c, st = L["ctx"], L["stream"]
            c.compress(L["G"], L["E"], L["fresh"], L["Q"], L["P"], r, stream=st)
            c.decompress(L["P"], L["Q"], r, L["E"], L["out"], stream=st)
            L["fresh"] = False

    def one_step():
        t = counter["step"]
        rank_rule(t)
        if graph["g"] is None:
            if groups:
                stage["ectx"].entropy_estimate_async(stage["flats"], w["stride"], w["chunk"], w["seed"], t,
                                                     w["bins"], stage["ent"][t % NBUF], stream=stage["estream"])
            else:
                for L in layers:
                    L["ctx"].entropy_estimate_async(L["flat"], w["stride"], w["chunk"], w["seed"], t,
                                                    w["bins"], L["ent"][t % NBUF], stream=L["estream"])
            compress_all()
            for si, st in enumerate(streams):
                step_events[t % NBUF][si].record(st)
            for si, st in enumerate(ent_streams):
                step_events[t % NBUF][n_streams + si].record(st)
        else:
            # entropy launches stay eager (their sampling slot changes with the step); the
            # compress + decompress launches of all layers are one captured graph
            if groups:
                stage["ectx"].entropy_estimate_async(stage["flats"], w["stride"], w["chunk"], w["seed"], t,
                                                     w["bins"], stage["ent"][t % NBUF], stream=stage["estream"])
            else:
                for L in layers:
                    L["ctx"].entropy_estimate_async(L["flat"], w["stride"], w["chunk"], w["seed"], t,
                                                    w["bins"], L["ent"][t % NBUF], stream=L["estream"])
            with torch.cuda.stream(main_stream):
                graph["g"].replay()
                for ev in step_events[t % NBUF][:n_streams]:
                    ev.record(main_stream)
            for si, st in enumerate(ent_streams):
                step_events[t % NBUF][n_streams + si].record(st)
        counter["step"] = t + 1

    main_stream = torch.cuda.Stream()

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    graphed = False
    if args.graph and not args.no_graph:
        try:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=main_stream, capture_error_mode="thread_local"):
                for st in streams:
                    st.wait_stream(main_stream)
                compress_all()
                for st in streams:
                    main_stream.wait_stream(st)
            graph["g"] = g
            graphed = True
            torch.cuda.synchronize()
            for _ in range(2):          # untimed replays
                one_step()
            torch.cuda.synchronize()
        except Exception as exc:        # fall back to eager launches
            print("bench.py: graph capture failed (%s); running eagerly" % exc, file=sys.stderr)
            graph["g"] = None
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step()
    t_issued = time.perf_counter()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    host_issue_ms = (t_issued - t0) * 1e3 / args.steps

    # host cost of issuing one step with an idle GPU behind it (no back-pressure)
    idle_issue = []
    for _ in range(5):
        torch.cuda.synchronize()
        ti0 = time.perf_counter()
        one_step()
        idle_issue.append((time.perf_counter() - ti0) * 1e3)
    torch.cuda.synchronize()
    host_issue_idle_ms = sorted(idle_issue)[len(idle_issue) // 2]

    elem_bytes = 2 if bf16 else 4
    grad_bytes = sum(s.m * s.n for s, _ in mats) * elem_bytes
    value = grad_bytes / (ms_per_step * 1e-3) / 1e9

    # second pass of the same K steps, launched eagerly on ONE stream so that every kernel has
    # the GPU to itself, each bracketed by HIP events on that stream
    graph["g"] = None
    torch.cuda.synchronize()
    for L in layers:
        L["stream"] = L["estream"] = streams[0]
    for g in groups:
        g["stream"] = streams[0]
    if groups:
        stage["estream"] = streams[0]
    ent_streams = [streams[0]] * n_ent
    for c in ctxs_all:
        c.profile_begin(max_launches=args.steps * len(layers) * 16 + 64)
    for _ in range(args.steps):
        one_step()
    stats = {}
    for c in ctxs_all:
        for name, sdict in c.profile_end().items():
            acc = stats.setdefault(name, dict(launches=0, total_ms=0.0, bytes=0.0, flops=0.0))
            for k in acc:
                acc[k] += sdict[k]
            event_overhead_us = sdict["event_overhead_ms"] * 1e3
    kernels = {}
    for name, s in stats.items():
        avg_us = s["total_ms"] * 1e3 / s["launches"]
        kernels[name] = dict(launches_per_step=s["launches"] / args.steps, avg_us=round(avg_us, 2),
                             gbs=round(s["bytes"] / (s["total_ms"] * 1e-3) / 1e9, 1) if s["total_ms"] > 0 else None,
                             tflops=round(s["flops"] / (s["total_ms"] * 1e-3) / 1e12, 2) if s["total_ms"] > 0 else None)
    dom = max(stats, key=lambda k: stats[k]["total_ms"])
    ds = stats[dom]
    achieved = ds["bytes"] / (ds["total_ms"] * 1e-3) / 1e9
    roofline = dict(bound="hbm", kernel=dom, achieved=round(achieved, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(achieved / HBM_PEAK_GBS, 4),
                    traffic=MEASURED_TRAFFIC_BYTES.get((args.workload, dom, len(groups),
                                                        "deferred" if deferred else "explicit")),
                    avg_launch_us=round(ds["total_ms"] * 1e3 / ds["launches"], 2),
                    algorithmic_bytes_per_launch=round(ds["bytes"] / ds["launches"]),
                    timing="HIP events around every launch (minus %.2f us, what an empty event pair reads); "
                           "second pass of the same K steps, launches serialised on one stream" % event_overhead_us)
    # MFMA utilisation of the instruction issued, beside the most an HBM-bound pass could reach:
    # ceiling = min(1, arithmetic intensity / ridge), ridge = bf16 MFMA peak / HBM peak
    ridge = BF16_MFMA_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)
    mfma = {k: dict(tflops=v["tflops"], frac_of_bf16_peak=round(v["tflops"] / BF16_MFMA_PEAK_TFLOPS, 4),
                    flop_per_byte=round(stats[k]["flops"] / stats[k]["bytes"], 2),
                    ceiling=round(min(1.0, stats[k]["flops"] / stats[k]["bytes"] / ridge), 4))
            for k, v in kernels.items()
            if k in ("k_pass_p", "k_pass_p_deferred", "k_pass_q", "k_decompress") and v["tflops"]}

    # what a plain copy, a plain read and a bf16 MFMA loop reach on this device (context beside the
    # published peaks the fractions above are taken against)
    pa = torch.ones(1 << 28, dtype=torch.float32, device="cuda")          # 1 GiB each
    pb = torch.empty_like(pa)
    torch.cuda.synchronize()
    peaks = ctxs[0].measure_device_peaks(pa, pb, reps=10)
    del pa, pb
    device_peaks = dict(copy_gbs=round(peaks["copy_gbs"], 1), read_gbs=round(peaks["read_gbs"], 1),
                        mfma_bf16_tflops=round(peaks["mfma_bf16_tflops"], 1), bytes=peaks["bytes"],
                        what="plain copy (read + written bytes), plain read, register-resident "
                             "32x32x16 bf16 MFMA loop; 10 launches each between one pair of events")
    roofline["frac_of_measured_copy"] = round(achieved / peaks["copy_gbs"], 4)

    cpu_baseline = None
    if not args.no_cpu_baseline:
        from oracle import edgc_oracle as orc
        q0s = []
        for li, (spec, g) in enumerate(mats):
            Q0 = np.zeros((spec.n, r), dtype=np.float32)
            orc.init_q(Q0, 0, r, w["seed"] + li)
            q0s.append(Q0)
        reps, tc0 = 0, time.perf_counter()
        while True:                      # whole steps until about 10 s of CPU work (at most 200 steps)
            if groups:
                # the stage-level estimate: every buffer's own sample, gathered, one histogram
                parts = [g.reshape(-1)[orc.sample_indices(g.size, w["stride"], w["chunk"], w["seed"], reps)]
                         for _, g in mats]
                orc.entropy(np.concatenate(parts), 1, 1, 0, 0, w["bins"])
            for li, (spec, g) in enumerate(mats):
                if not groups:
                    orc.entropy(g.reshape(-1), w["stride"], w["chunk"], w["seed"], reps, w["bins"])
                P, Q1, D = orc.compress(g, None, q0s[li], r)
                orc.decompress(P, Q1, D, orc.BF16 if bf16 else orc.F32)
            reps += 1
            tc1 = time.perf_counter()
            if tc1 - tc0 >= 10.0 or reps >= 200:
                break
        cpu_baseline = dict(value=round(reps * grad_bytes / (tc1 - tc0) / 1e9, 4), unit="GB/s",
                            cores=orc.num_threads(), kind="oracle", seconds=round(tc1 - tc0, 2),
                            sample="%d full steps of the workload (all %d matrices each), oracle as it stands"
                                   % (reps, len(mats)))

    line = {
        "metric": "gradient GB/s through entropy+rank-r compress/decompress; % HBM/MFMA roofline",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": args.workload, "layers": ["%dx%d" % (s.m, s.n) for s, _ in mats],
                   "rank": r, "stride": w["stride"], "chunk": w["chunk"], "bins": w["bins"],
                   "streams": 1 if args.serial else n_streams, "entropy_streams": 0 if args.serial else n_ent,
                   "hip_graph": graphed, "batch_groups": len(groups),
                   "residual": "deferred" if deferred else "explicit",
                   "gradient_bytes_per_step": grad_bytes},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "kernels": kernels, "mfma": mfma,
        "device_peaks_measured": device_peaks,
        "last_rank_decision": decisions[-1].rank if decisions else None,
        "host_issue_ms_per_step": round(host_issue_ms, 4),
        "host_issue_idle_gpu_ms_per_step": round(host_issue_idle_ms, 4),
    }
    print(json.dumps(line))
    for c in ctxs_all:
        c.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
