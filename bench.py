#!/usr/bin/env python3
"""Benchmark of the cache look-up hot path on one MI355X.

One step = one pass of the whole look-up (query preparation, MFMA distance pass with
fused top-R, merge + fp32 re-scoring + vote + hit decision) over one batch of synthetic
queries, with cache, queries and workspace already resident in HBM.

Prints ONE JSON line: queries/s of the whole look-up, the roofline figures of the
dominant kernel (the distance pass, timed with HIP events on its own stream inside the
timed region) and the CPU oracle timed on a bounded sample of the same workload.
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

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E, published


def measured_traffic(kernel: str, workload: str):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary of this
    workload (FETCH_SIZE and WRITE_SIZE in KiB, each scaled by the plain-copy calibration factor
    recorded in the same file); None when there is no summary."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}.txt")
    if not os.path.exists(path):
        return None
    vals, factor = {}, {}
    for line in open(path):
        parts = line.split()
        for c in ("FETCH_SIZE", "WRITE_SIZE"):
            if line.startswith(f"fz::{kernel}") and c in parts:
                vals[c] = float(parts[parts.index(c) + 1])
            if line.startswith(f"{c} calibration") and "factor" in parts:
                factor[c] = float(parts[parts.index("factor") + 1])
    if set(vals) != {"FETCH_SIZE", "WRITE_SIZE"} or set(factor) != {"FETCH_SIZE", "WRITE_SIZE"}:
        return None
    return (vals["FETCH_SIZE"] * factor["FETCH_SIZE"] + vals["WRITE_SIZE"] * factor["WRITE_SIZE"]) * 1024.0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c2_batched")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle leg (profiling runs)")
    ap.add_argument("--cpu-sample", type=int, default=0, help="queries in the oracle sample (0 = per workload)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy three times (reference for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (one-GPU boxes; the path has no multi-GPU part); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2002_02645_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    binding.lib()   # fail loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    wl = synth.WORKLOADS[args.workload]
    if len(wl.layers) != 1:
        print("bench.py: single-layer workloads only (the cascade is measured by its own parity/bench test)",
              file=sys.stderr)
        return 2
    spec = wl.layers[0]
    t0 = time.time()
    data = synth.make_workload(wl, device=dev)
    L = data.layers[0]
    queries = data.queries[0]
    torch.cuda.synchronize()
    gen_s = time.time() - t0

    fc = binding.FreezeCache(1, dev)
    t0 = time.time()
    fc.build_layer(0, L.entries, L.labels, spec.num_classes)
    torch.cuda.synchronize()
    build_s = time.time() - t0

    b, k, thr, r = wl.batch, wl.k, wl.vote_thresholds[0], wl.rescore_r
    out = fc.alloc_outputs(b, k)
    stream = torch.cuda.current_stream()

    def step():
        fc.lookup(0, queries, k, thr, r, out=out)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    binding.freeze_profile_enable(fc.ctx, True)
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(args.steps):
        step()
    ev1.record(stream)
    torch.cuda.synchronize()
    wall_s = time.perf_counter() - t0
    stage_ms, calls = binding.freeze_profile_read(fc.ctx)
    binding.freeze_profile_enable(fc.ctx, False)
    ms_per_step = wall_s * 1e3 / args.steps
    ev_ms_per_step = ev0.elapsed_time(ev1) / args.steps
    qps = b * args.steps / wall_s

    # roofline of the dominant kernel (distance pass): algorithmic flops = 2 * B * N * d per launch
    dist_ms = stage_ms[1] / max(calls, 1)
    flops = 2.0 * b * spec.n * spec.d
    cache_bytes = float(spec.n) * spec.d * 2
    if b >= 64:
        achieved = flops / (dist_ms * 1e-3) / 1e12
        roofline = dict(bound="mfma", achieved=round(achieved, 2), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                        frac=round(achieved / PEAK_BF16_TFLOPS, 4), traffic=None)
    else:
        achieved = cache_bytes / (dist_ms * 1e-3) / 1e9
        roofline = dict(bound="hbm", achieved=round(achieved, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                        frac=round(achieved / PEAK_HBM_GBS, 4), traffic=None)
    roofline["kernel"] = "dist_topr_kernel" if b > 16 or spec.d > 1024 else "dist_skinny_kernel"
    roofline["traffic"] = measured_traffic(roofline["kernel"], wl.name)
    roofline["kernel_ms"] = round(dist_ms, 4)
    roofline["stage_ms"] = {"query_prep": round(stage_ms[0] / max(calls, 1), 4), "dist_topr": round(dist_ms, 4),
                            "finish": round(stage_ms[2] / max(calls, 1), 4)}

    result = {
        "metric": "queries/sec per layer lookup",
        "value": round(qps, 1),
        "unit": "queries/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: cache {spec.n}x{spec.d} bf16, batch {b}, k={k}, "
                               f"vote_threshold={thr}, rescore_r={r if r else 'default'}",
                   "event_ms_per_step": round(ev_ms_per_step, 4), "cache_build_s": round(build_s, 3),
                   "input_gen_s": round(gen_s, 2)},
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        from oracle import freeze_oracle as fo
        sample = args.cpu_sample or {"c2_batched": 128, "c3_wide": 16, "c1_tiny": 256}.get(wl.name, min(b, 64))
        sample = min(sample, b)
        g = torch.Generator().manual_seed(wl.seed + 999)
        pick = torch.randperm(b, generator=g)[:sample].sort().values
        q_h = queries[pick.to(dev)].cpu().numpy()
        e_h = synth.bf16_bits(L.entries) if L.entries.dtype == torch.bfloat16 else L.entries.cpu().numpy()
        l_h = L.labels.cpu().numpy()
        t0 = time.perf_counter()
        kk = min(k + 1, spec.n)   # one extra neighbour: tells a near-tie at the k-th place
        o_idx, o_dist, o_threads = fo.knn(q_h, e_h, kk)
        o_lab, o_votes, o_hit = fo.vote(l_h, o_idx[:, :k], spec.num_classes, thr)
        cpu_s = time.perf_counter() - t0
        ref = dict(idx=o_idx[:, :k], sqdist=o_dist, hit=o_hit, threads=o_threads)
        result["cpu_baseline"] = {"value": round(sample / cpu_s, 3), "unit": "queries/s", "cores": int(ref["threads"]),
                                  "kind": "oracle",
                                  "sample": f"{sample} of the {b} queries (seeded subset) against the full cache, "
                                            f"{cpu_s:.1f} s"}
        # the sample doubles as a parity spot check of the timed configuration
        got_idx = out["idx"][pick.to(dev)].cpu().numpy()
        got_hit = out["hit"][pick.to(dev)].cpu().numpy()
        gaps = np.diff(ref["sqdist"], axis=1) / np.maximum(ref["sqdist"][:, 1:], 1e-30)
        differ = (got_idx != ref["idx"]).any(axis=1)
        unexplained = int((differ & ~(gaps < 1e-4).any(axis=1)).sum())
        result["config"]["parity_sample"] = {"queries": int(sample), "identical": int((~differ).sum()),
                                             "differ_outside_near_tie": unexplained,
                                             "hit_equal": int((got_hit == ref["hit"]).sum())}
    if args.copy_calibration:
        src = torch.zeros(1 << 28, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.bitwise_not(src, out=dst)   # a plain elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        result["config"]["copy_calibration_bytes"] = 1 << 30
    fc.close()
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
