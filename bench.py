#!/usr/bin/env python3
"""Benchmark of the EDGC hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic layer
gradients: for every 2-D gradient of the workload, the down-sampled entropy
estimate (sample, range, histogram, entropy), the host rank rule on the
step's entropies, and rank-r compress + decompress with the error-feedback
residual carried from the previous step.  Inputs are resident in HBM before
the timed region starts.  Prints ONE JSON line.

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
# runs of this command (see profiles/); None until such a run has been recorded.
MEASURED_TRAFFIC_BYTES = {}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg2_gpt_h2048_r16")
    ap.add_argument("--rank", type=int, default=0, help="override the workload's rank")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    return ap.parse_args()


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

    w = gen.WORKLOADS[args.workload]
    r = args.rank or w["rank"]
    bf16 = w["dtype"] == "bf16"
    mats = gen.workload_matrices(args.workload)
    max_m = max(s.m for s, _ in mats)
    max_n = max(s.n for s, _ in mats)
    ctx = edgc.Context(0, max_bins=w["bins"], max_rank=max(r, 4), max_rows=max_m, max_cols=max_n)

    # device state per layer: gradient, residual, warm-started Q, P, output
    layers = []
    for li, (spec, g) in enumerate(mats):
        if bf16:
            G = torch.from_numpy(g.view(np.int16).copy()).cuda().view(torch.bfloat16)
        else:
            G = torch.from_numpy(g).cuda()
        ldf = (r + 3) // 4 * 4
        Q = torch.zeros((spec.n, ldf), dtype=torch.float32, device="cuda")
        ctx.init_q(Q, 0, r, w["seed"] + li)
        layers.append(dict(
            spec=spec, G=G, Q=Q,
            E=torch.empty((spec.m, spec.n), dtype=torch.float32, device="cuda"),
            P=torch.empty((spec.m, ldf), dtype=torch.float32, device="cuda"),
            out=torch.empty_like(G), fresh=True,
            ent=[torch.empty(ENTROPY_RESULT_BYTES, dtype=torch.uint8, pin_memory=True) for _ in range(2)],
        ))
    torch.cuda.synchronize()

    ref = min(mats, key=lambda t: t[0].m * t[0].n)[0]
    prm = edgc.RankParams(ref.m, ref.n, r_min=r, r_max=r, step_limit=8, allowed=[r],
                          total_iters=args.steps + args.warmup, min_warmup_frac=0.10)
    state = edgc.RankState()
    decisions = []
    step_events = [torch.cuda.Event(), torch.cuda.Event()]
    counter = {"step": 0}

    def one_step():
        t = counter["step"]
        # the rank rule consumes the entropies of the previous step (already on the host)
        if t > 0:
            step_events[(t - 1) & 1].synchronize()
            H = [edgc.EntropyResult.from_buffer(L["ent"][(t - 1) & 1].numpy().tobytes()).h_diff_nats
                 for L in layers]
            decisions.append(edgc.select_rank(state, H, 1, prm))
        for L in layers:
            ctx.entropy_estimate_async(L["G"].view(-1), w["stride"], w["chunk"], w["seed"], t, w["bins"],
                                       L["ent"][t & 1])
            ctx.compress(L["G"], L["E"], L["fresh"], L["Q"], L["P"], r)
            ctx.decompress(L["P"], L["Q"], r, L["E"], L["out"])
            L["fresh"] = False
        step_events[t & 1].record()
        counter["step"] = t + 1

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    elem_bytes = 2 if bf16 else 4
    grad_bytes = sum(s.m * s.n for s, _ in mats) * elem_bytes
    value = grad_bytes / (ms_per_step * 1e-3) / 1e9

    # second pass of the same K steps with every kernel bracketed by HIP events on its stream
    ctx.profile_begin(max_launches=args.steps * len(layers) * 16 + 64)
    for _ in range(args.steps):
        one_step()
    stats = ctx.profile_end()
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
                    traffic=MEASURED_TRAFFIC_BYTES.get((args.workload, dom)),
                    avg_launch_us=round(ds["total_ms"] * 1e3 / ds["launches"], 2),
                    algorithmic_bytes_per_launch=round(ds["bytes"] / ds["launches"]),
                    timing="HIP events around every launch, second pass of the same K steps")
    mfma = {k: dict(tflops=v["tflops"], frac_of_bf16_peak=round(v["tflops"] / BF16_MFMA_PEAK_TFLOPS, 4))
            for k, v in kernels.items() if k in ("k_pass_p", "k_pass_q", "k_decompress") and v["tflops"]}

    cpu_baseline = None
    if not args.no_cpu_baseline:
        from oracle import edgc_oracle as orc
        tc0 = time.perf_counter()
        for li, (spec, g) in enumerate(mats):
            orc.entropy(g.reshape(-1), w["stride"], w["chunk"], w["seed"], 0, w["bins"])
            Q0 = np.zeros((spec.n, r), dtype=np.float32)
            orc.init_q(Q0, 0, r, w["seed"] + li)
            P, Q1, D = orc.compress(g, None, Q0, r)
            orc.decompress(P, Q1, D, orc.BF16 if bf16 else orc.F32)
        tc1 = time.perf_counter()
        cpu_baseline = dict(value=round(grad_bytes / (tc1 - tc0) / 1e9, 4), unit="GB/s", cores=orc.num_threads(),
                            kind="oracle", seconds=round(tc1 - tc0, 2),
                            sample="one full step of the workload (all %d matrices), oracle as it stands" % len(mats))

    line = {
        "metric": "gradient GB/s through entropy+rank-r compress/decompress; % HBM/MFMA roofline",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": args.workload, "layers": ["%dx%d" % (s.m, s.n) for s, _ in mats],
                   "rank": r, "stride": w["stride"], "chunk": w["chunk"], "bins": w["bins"],
                   "gradient_bytes_per_step": grad_bytes},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "kernels": kernels, "mfma": mfma,
        "last_rank_decision": decisions[-1].rank if decisions else None,
    }
    print(json.dumps(line))
    ctx.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
