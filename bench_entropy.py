"""The entropy-only workload of bench.py (`--workload cfg3_flat_1e9`): BASELINE config 3, the
down-sampled entropy estimate alone on a flat buffer of 1e9 elements."""
from __future__ import annotations

import json
import time


def entropy_sweep(args, torch, edgc, metric, hbm_peak_gbs) -> int:
    """The entropy-only workload: one flat buffer of 1e9 elements (fp32, then bf16), Laplace(0, 1e-3)
    with 0.1 % of the values at 100 times the scale, generated on the device; sampling strides 1000,
    100, 10 and 1 (0.1 % to 100 %) times 256, 4096 and 65536 bins.  One "step" is one estimate
    (range, histogram, entropy) of one cell; the JSON line carries every cell and, as `value`, the
    100 % / 4096-bin cell of the fp32 buffer, whose two passes read the whole buffer twice.  A cell's
    `reads_of_sample` says how often its kernels read the sample (bf16 samples of 32 Mi elements or
    more are read once), `sample_gbs` = those reads x sample bytes / time."""
    from paper_2511_10333_amd.binding import ENTROPY_RESULT_BYTES, EntropyResult
    n, chunk, seed = 1_000_000_000, args.ent_chunk, 0
    strides = tuple(int(v) for v in args.ent_strides.split(","))
    bins_list = tuple(int(v) for v in args.ent_bins.split(","))
    dtypes = args.ent_dtypes.split(",")
    ctx = edgc.Context(0, max_bins=65536, max_rank=4, max_rows=64, max_cols=64)
    out = torch.empty(ENTROPY_RESULT_BYTES, dtype=torch.uint8, pin_memory=True)
    g = torch.Generator(device="cuda").manual_seed(3)
    x32 = torch.empty(n, device="cuda")
    x32.exponential_(1.0, generator=g)                                  # |Laplace(0, 1)|
    sign = torch.empty(n, device="cuda").uniform_(-1.0, 1.0, generator=g)
    x32.mul_(torch.sign(sign))
    x32.mul_(torch.where(sign.abs() < 1e-3, 1e-1, 1e-3))               # 0.1 % outliers at 100 x the scale
    del sign
    bufs = {k: v for k, v in (("f32", x32), ("bf16", x32.bfloat16() if "bf16" in dtypes else None)) if k in dtypes}
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
                ctx.profile_begin(6 * reps + 8)
                for t in range(reps):
                    ctx.entropy_estimate_async(x, stride, chunk, seed, t, bins, out)
                torch.cuda.synchronize()
                ks = ctx.profile_end()
                kern = {k: dict(avg_us=round(v["total_ms"] * 1e3 / v["launches"], 2),
                                gbs=round(v["bytes"] / (v["total_ms"] * 1e-3) / 1e9, 1))
                        for k, v in ks.items() if v["launches"] and v["total_ms"] > 0}
                sample_bytes = res.n_sampled * esz
                # reads of the sample: the range pass (not for bf16 counted by bit pattern) and one binning pass
                # (two for fp32 on more than 32768 bins without the 16-bit counters); kernels that only check
                # the overflow gate and return (a few microseconds, no bytes) do not count
                live = {k: v for k, v in kern.items() if v["avg_us"] >= 4.0 or k.startswith("k_wide")}
                reads = (1 if "k_minmax" in live else 0) + (1 if "k_wide_hist" in live else 0) + \
                        ((2 if bins > 32768 else 1) if "k_hist" in live else 0)
                cell = dict(dtype=dtype, stride=stride, bins=bins, n_sampled=res.n_sampled, ms=round(ms, 4),
                            gradient_gbs=round(n * esz / (ms * 1e-3) / 1e9, 1), reads_of_sample=reads,
                            sample_gbs=round(reads * sample_bytes / (ms * 1e-3) / 1e9, 1),
                            H_bits=round(res.H_bits, 6), kernels=kern)
                cells.append(cell)
                if (dtype == "f32" and stride == 1 and bins == 4096) or headline is None:
                    headline = (cell, ms, ks, reps)
    cell, ms, ks, reps = headline
    dom = max((k for k in ("k_minmax", "k_hist", "k_wide_hist") if k in ks and ks[k]["launches"]),
              key=lambda k: ks[k]["total_ms"])
    achieved = ks[dom]["bytes"] / (ks[dom]["total_ms"] * 1e-3) / 1e9
    pa = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
    pb = torch.empty_like(pa)
    peaks = ctx.measure_device_peaks(pa, pb, reps=10)
    del pa, pb
    roofline = dict(bound="hbm", kernel=dom, achieved=round(achieved, 1), peak=hbm_peak_gbs, unit="GB/s",
                    frac=round(achieved / hbm_peak_gbs, 4), traffic=None,
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
        "metric": metric,
        "value": cell["gradient_gbs"], "unit": "GB/s", "n_gpus": 1, "steps": reps, "warmup": min(args.warmup, 3),
        "ms_per_step": cell["ms"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cell["dtype"], "data": "synthetic",
        "config": {"workload": "cfg3_flat_1e9", "what": "entropy estimate only; value = the 100 % / 4096-bin "
                   "cell of the fp32 buffer (the first cell run when that one is not among them)", "elements": n, "chunk": chunk, "strides": list(strides),
                   "bins": list(bins_list)},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "cells": cells,
        "device_peaks_measured": {k: (round(v, 1) if isinstance(v, float) else v) for k, v in peaks.items()},
    }
    print(json.dumps(line))
    return 0

