#!/usr/bin/env python3
"""Benchmark of the cache look-up hot path on one MI355X.

One step = one pass of the whole look-up (query preparation, MFMA distance pass, selection,
fp32 re-scoring, vote and hit decision; for the cascade workloads: all layers, with miss
compaction between them) over one batch of synthetic queries, with caches, queries and
workspace already resident in HBM.

Prints ONE JSON line: queries/s of the whole look-up, the roofline figures of the dominant
kernel (the distance pass, timed with HIP events on its own stream inside the timed region)
and the CPU oracle timed on a bounded sample of the same workload.  The headline workload is
c2_batched; without --workload the line also carries, under "other_workloads", the same block
(timing, roofline, cpu_baseline, parity sample) for every other benchmark configuration.
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
            if line.startswith(f"fz::{kernel}") and c in parts and c not in vals:
                vals[c] = float(parts[parts.index(c) + 1])
            if line.startswith(f"{c} calibration") and "factor" in parts:
                factor[c] = float(parts[parts.index("factor") + 1])
    if set(vals) != {"FETCH_SIZE", "WRITE_SIZE"} or set(factor) != {"FETCH_SIZE", "WRITE_SIZE"}:
        return None
    return (vals["FETCH_SIZE"] * factor["FETCH_SIZE"] + vals["WRITE_SIZE"] * factor["WRITE_SIZE"]) * 1024.0


def time_next_rows(torch, binding, dev):
    """Wall-clock times (synchronised, inputs resident) of the k-means cache and of the projection on
    seeded synthetic inputs: 50,000 points x 8,192 in 10 classes -> 200 centres; 1,024 outputs."""
    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        t0 = time.time()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.time() - t0) / reps * 1e3

    res = {"data": "synthetic", "kmeans": {}, "projection": []}
    g = torch.Generator(device=dev)
    g.manual_seed(20020264)
    n, d, kc, classes, nq = 50000, 8192, 200, 10, 10000
    cent = torch.randn(classes, d, device=dev, generator=g)
    cls = torch.randint(0, classes, (n,), device=dev, generator=g)
    pts = (cent[cls] + 0.8 * torch.randn(n, d, device=dev, generator=g)).contiguous()
    lab = cls.to(torch.int32)
    init = pts[:kc].clone()
    fc = binding.FreezeCache(1, dev)
    t1 = timed(lambda: fc.build_kmeans_layer(0, pts, lab, classes, init, 1), 3)
    t5 = timed(lambda: fc.build_kmeans_layer(0, pts, lab, classes, init, 5), 3)
    q = (cent[torch.randint(0, classes, (nq,), device=dev, generator=g)] +
         0.8 * torch.randn(nq, d, device=dev, generator=g)).contiguous()
    tl = timed(lambda: fc.lookup_confidence(0, q, 1, 0.01), 10)
    per_round = (t5 - t1) / 4
    # algorithmic bytes: a round reads every point twice in fp32 (assignment, update); a look-up reads its queries once
    round_bytes, lookup_bytes = 2.0 * n * d * 4, float(nq) * d * 4 + float(kc) * d * 2
    res["kmeans"] = {"points": n, "d": d, "centres": kc, "build_ms_1_round": round(t1, 3), "build_ms_5_rounds": round(t5, 3),
                     "ms_per_round": round(per_round, 3), "lookup_queries": nq, "lookup_ms": round(tl, 3),
                     "roofline_round": {"bound": "hbm", "achieved": round(round_bytes / per_round / 1e6, 1), "peak": PEAK_HBM_GBS,
                                        "unit": "GB/s", "frac": round(round_bytes / per_round / 1e6 / PEAK_HBM_GBS, 4),
                                        "bytes": round_bytes, "what": "whole round: centres -> cache, assignment look-up (k = 1) of every point, update"},
                     "roofline_lookup": {"bound": "hbm", "achieved": round(lookup_bytes / tl / 1e6, 1), "peak": PEAK_HBM_GBS,
                                         "unit": "GB/s", "frac": round(lookup_bytes / tl / 1e6 / PEAK_HBM_GBS, 4),
                                         "bytes": lookup_bytes, "what": "whole look-up with the k-means confidence"}}
    fc.close()
    del pts, q
    for (b, dd, m) in [(10000, 8192, 1024), (4096, 65536, 1024), (256, 65536, 1024)]:
        x = torch.randn(b, dd, device=dev, generator=g)
        w = (torch.randn(m, dd, device=dev, generator=g) / dd ** 0.5).to(torch.bfloat16)
        bias = torch.zeros(m, device=dev)
        fc = binding.FreezeCache(1, dev)
        fc.build_projection(0, w, bias)
        ms = timed(lambda: fc.project(0, x, True), 10)
        tf = 2.0 * b * dd * m / ms / 1e9
        io_bytes = float(b) * dd * 4 + float(m) * dd * 2 + float(b) * m * 4
        res["projection"].append({"inputs": b, "d": dd, "outputs": m, "ms": round(ms, 3), "TFLOPs": round(tf, 1),
                                  "roofline": {"bound": "mfma", "achieved": round(tf, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                                               "frac": round(tf / PEAK_BF16_TFLOPS, 4),
                                               "hbm_view": {"GBs": round(io_bytes / ms / 1e6, 1),
                                                            "frac_of_hbm_peak": round(io_bytes / ms / 1e6 / PEAK_HBM_GBS, 4)},
                                               "what": "whole call: fp32 -> bf16 conversion of x, MFMA product (stream-K), bias / ReLU"}})
        fc.close()
        del x, w
    return res


# oracle sample sizes: about 3-5 s of oracle time each on the machine's host cores (the run prints how
# many threads the oracle actually used)
CPU_SAMPLE = {"c1_tiny": 256, "c2_batched": 256, "c3_wide": 32, "c4_cascade": 16, "c4_cascade_noisy": 16,
              "c5_latency_b1": 1, "c5_latency_b8": 8}
STEPS = {"c1_tiny": 200, "c2_batched": 20, "c3_wide": 20, "c4_cascade": 6, "c4_cascade_noisy": 6,
         "c5_latency_b1": 200, "c5_latency_b8": 200}
ALL_WORKLOADS = ["c2_batched", "c1_tiny", "c3_wide", "c4_cascade", "c4_cascade_noisy", "c5_latency_b1", "c5_latency_b8"]


def run_workload(torch, np, binding, synth, dev, name, steps, warmup, cache_copies=0, cpu_baseline=True, cpu_sample=0,
                 data=None):
    """Times one workload and returns (result block, data).  `data` lets the two cascade variants,
    which differ in the cache labels only, share the generated activations."""
    wl = synth.WORKLOADS[name]
    nl = len(wl.layers)
    cascade = nl > 1
    t0 = time.time()
    if data is None:
        data = synth.make_workload(wl, device=dev)
    torch.cuda.synchronize()
    gen_s = time.time() - t0

    # A single-layer workload whose cache is small next to HBM is built twice and the steps
    # alternate between the copies, so that no step finds its cache in the memory-side cache
    # because the step before left it there.
    cache_gib = data.layers[0].spec.n * data.layers[0].spec.d * 2 / 2**30
    copies = cache_copies if cache_copies > 0 else (2 if (not cascade and cache_gib <= 2.0) else 1)
    if cascade:
        copies = 1
    fc = binding.FreezeCache(nl if cascade else copies, dev)
    verdicts = torch.zeros(3, dtype=torch.int64, device=dev)
    binding.freeze_lookup_stats_attach(fc.ctx, verdicts)
    t0 = time.time()
    for l, L in enumerate(data.layers):
        for c in range(copies):
            fc.build_layer(l + c, L.entries, L.labels, L.spec.num_classes)
    torch.cuda.synchronize()
    build_s = time.time() - t0

    b, k, r = wl.batch, wl.k, wl.rescore_r
    spec = wl.layers[0]
    stream = torch.cuda.current_stream()
    if cascade:
        out = dict(label=torch.empty(b, dtype=torch.int32, device=dev),
                   exit_layer=torch.empty(b, dtype=torch.int32, device=dev),
                   hits_per_layer=torch.empty(nl, dtype=torch.int64, device=dev))

        def step():
            fc.lookup_cascade(list(range(nl)), data.queries, k, list(wl.vote_thresholds), r, out=out)
    else:
        out = fc.alloc_outputs(b, k)
        turn = [0]

        def step():
            fc.lookup(turn[0] % copies, data.queries[0], k, wl.vote_thresholds[0], r, out=out)
            turn[0] += 1

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    verdicts.zero_()

    # the timed region brackets only the dominant kernel (the distance pass) with events: two per look-up,
    # or two per eighth look-up where a step is so short (C1, C5: 0.06 - 0.2 ms) that the 7 us of two event
    # records per call would be 4 - 12 % of what is being measured
    sampled_events = steps >= 100 and not cascade
    binding.freeze_profile_enable(fc.ctx, 3 if sampled_events else 2)
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(steps):
        step()
    ev1.record(stream)
    torch.cuda.synchronize()
    wall_s = time.perf_counter() - t0
    dist_calls = binding.freeze_profile_read_calls(fc.ctx)
    verdict_counts = [int(v) for v in verdicts.cpu().numpy()]
    # the same K steps twice more, outside the timed region: with events at every stage boundary
    # (the stage breakdown; four event records per look-up, which matter next to a 0.2 ms look-up
    # and not otherwise) and with none at all; both reported beside the timed region's figure
    binding.freeze_profile_enable(fc.ctx, 1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms_per_step_all_events = (time.perf_counter() - t0) * 1e3 / steps
    calls = binding.freeze_profile_read_calls(fc.ctx)
    binding.freeze_profile_enable(fc.ctx, 0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms_per_step_plain = (time.perf_counter() - t0) * 1e3 / steps
    ms_per_step = wall_s * 1e3 / steps
    ev_ms_per_step = ev0.elapsed_time(ev1) / steps
    qps = b * steps / wall_s

    # per-layer stage times: the recorded look-ups cycle through the layers
    per_layer = [[0.0, 0.0, 0.0] for _ in range(nl)]
    counted = [0] * nl
    for i, c in enumerate(calls):
        for j in range(3):
            per_layer[i % nl][j] += c[j]
        counted[i % nl] += 1
    per_layer = [[v / max(counted[l], 1) for v in per_layer[l]] for l in range(nl)]
    # per step: the stage times of its look-ups added up (kernel time without the gaps between calls)
    step_ms = sorted(sum(sum(c) for c in calls[i:i + nl]) for i in range(0, len(calls) - nl + 1, nl))

    # roofline of the dominant kernel: the distance pass of the (first) layer, from the events recorded
    # inside the timed region.
    # algorithmic flops per launch = 2 * B * N * d; algorithmic bytes (small batches) = N * d * 2
    first = [c[1] for i, c in enumerate(dist_calls) if i % nl == 0]
    dist_ms = sum(first) / max(len(first), 1)
    flops = 2.0 * b * spec.n * spec.d
    cache_bytes = float(spec.n) * spec.d * 2
    skinny = (not cascade) and b <= 16 and spec.d <= 1024
    if not skinny:
        achieved = flops / (dist_ms * 1e-3) / 1e12
        roofline = dict(bound="mfma", achieved=round(achieved, 2), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                        frac=round(achieved / PEAK_BF16_TFLOPS, 4), traffic=None)
        roofline["hbm_view"] = {"cache_stream_GBs": round(cache_bytes / (dist_ms * 1e-3) / 1e9, 1),
                                "frac_of_hbm_peak": round(cache_bytes / (dist_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
    else:
        achieved = cache_bytes / (dist_ms * 1e-3) / 1e9
        roofline = dict(bound="hbm", achieved=round(achieved, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                        frac=round(achieved / PEAK_HBM_GBS, 4), traffic=None)
    roofline["kernel"] = "dist_skinny_kernel" if skinny else "dist_topr_kernel"
    roofline["kernel_ms"] = round(dist_ms, 4)
    # (a cascade's profile averages the kernel over its four layers: no per-layer traffic figure)
    roofline["traffic"] = None if cascade else measured_traffic(roofline["kernel"], wl.name)
    roofline["traffic_source"] = (f"profiles/{roofline['kernel']}_{wl.name}.txt (rocprofv3 counters of an earlier run of "
                                  "this command; not measured in this run)") if roofline["traffic"] else None
    # stage breakdown from the run with events at every stage boundary (after the timed region)
    roofline["stage_ms"] = {"query_prep": round(per_layer[0][0], 4), "dist": round(per_layer[0][1], 4),
                            "select_rescore_vote": round(per_layer[0][2], 4)}

    config = {"workload": f"{wl.name}: " + ", ".join(f"cache {s.n}x{s.d} {'bf16' if s.store_bf16 else 'fp32'}"
                                                     for s in wl.layers)
                          + f", batch {b}, k={k}, vote_thresholds={list(wl.vote_thresholds)}, "
                            f"rescore_r={r if r else 'default'}",
              "event_ms_per_step": round(ev_ms_per_step, 4),
              "kernel_events_in_timed_region": ("every eighth look-up" if sampled_events else "every look-up"),
              "stage_sum_ms_median": round(step_ms[len(step_ms) // 2], 4) if step_ms else None,
              "stage_sum_ms_min": round(step_ms[0], 4) if step_ms else None,
              "ms_per_step_with_all_stage_events": round(ms_per_step_all_events, 4),
              "ms_per_step_without_stage_events": round(ms_per_step_plain, 4), "cache_build_s": round(build_s, 3), "cache_copies": copies,
              "input_gen_s": round(gen_s, 2),
              # how the timed look-ups were confirmed exact: at once / after the wider re-scoring / by the exact scan
              "certificate_verdicts": {"first_rescoring": verdict_counts[0], "wider_rescoring": verdict_counts[1],
                                       "exact_scan": verdict_counts[2]}}
    if cascade:
        hits = out["hits_per_layer"].cpu().numpy().astype(np.int64)
        entering = [b]
        for l in range(nl - 1):
            entering.append(int(entering[-1] - hits[l]))
        config["cascade"] = {
            "hits_per_layer": [int(h) for h in hits],
            "hit_fraction_of_entering": [round(float(hits[l]) / max(entering[l], 1), 4) for l in range(nl)],
            "entering_per_layer": entering,
            "fell_through": int(b - hits.sum()),
            "layer_stage_ms": [{"query_prep": round(p[0], 4), "dist": round(p[1], 4),
                                "select_rescore_vote": round(p[2], 4)} for p in per_layer],
            "layer_dist_tflops": [round(2.0 * entering[l] * wl.layers[l].n * wl.layers[l].d
                                        / max(per_layer[l][1] * 1e-3, 1e-9) / 1e12, 1) for l in range(nl)],
        }
        step_flops = sum(2.0 * entering[l] * wl.layers[l].n * wl.layers[l].d for l in range(nl))
    else:
        step_flops = flops
    # the whole step (every stage of every layer) against the same roof
    if skinny:
        roofline["frac_whole_step"] = round(cache_bytes / (ms_per_step * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)
    else:
        roofline["frac_whole_step"] = round(step_flops / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)

    result = {
        "metric": "queries/sec per layer lookup",
        "value": round(qps, 1),
        "unit": "queries/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        # the distance pass multiplies bf16 operands with fp32 accumulation; the re-scoring that decides
        # the reported neighbours and distances is fp32 against the stored values (bf16, or fp32 for C1)
        "dtype": "bf16",
        "rescoring_dtype": "f32",
        "cache_dtype": "bf16" if spec.store_bf16 else "f32",
        "data": "synthetic",
        "config": config,
        "roofline": roofline,
    }

    if cpu_baseline:
        from oracle import freeze_oracle as fo
        sample = min(cpu_sample or CPU_SAMPLE.get(wl.name, min(b, 64)), b)
        g = torch.Generator().manual_seed(wl.seed + 999)
        pick = torch.randperm(b, generator=g)[:sample].sort().values
        host_entries = [synth.bf16_bits(L.entries) if L.entries.dtype == torch.bfloat16 else L.entries.cpu().numpy()
                        for L in data.layers]
        host_labels = [L.labels.cpu().numpy() for L in data.layers]
        host_q = [q[pick.to(dev)].cpu().numpy() for q in data.queries]
        if cascade:
            t0 = time.perf_counter()
            o_lab, o_exit, _, o_threads = fo.cascade(host_q, host_entries, host_labels,
                                                     [L.spec.num_classes for L in data.layers], k, wl.vote_thresholds)
            cpu_s = time.perf_counter() - t0
            got_exit = out["exit_layer"][pick.to(dev)].cpu().numpy()
            got_lab = out["label"][pick.to(dev)].cpu().numpy()
            config["parity_sample"] = {"requests": int(sample),
                                       "exit_layer_equal": int((got_exit == o_exit).sum()),
                                       "label_equal": int((got_lab == o_lab).sum())}
            what = f"{sample} of the {b} requests (seeded subset) through the oracle's cascade"
        else:
            t0 = time.perf_counter()
            kk = min(k + 1, spec.n)   # one extra neighbour: tells a near-tie at the k-th place
            o_idx, o_dist, o_threads = fo.knn(host_q[0], host_entries[0], kk)
            o_lab, o_votes, o_hit = fo.vote(host_labels[0], o_idx[:, :k], spec.num_classes, wl.vote_thresholds[0])
            cpu_s = time.perf_counter() - t0
            got_idx = out["idx"][pick.to(dev)].cpu().numpy()
            got_hit = out["hit"][pick.to(dev)].cpu().numpy()
            gaps = np.diff(o_dist, axis=1) / np.maximum(o_dist[:, 1:], 1e-30)
            differ = (got_idx != o_idx[:, :k]).any(axis=1)
            config["parity_sample"] = {"queries": int(sample), "identical": int((~differ).sum()),
                                       "differ_outside_near_tie": int((differ & ~(gaps < 1e-4).any(axis=1)).sum()),
                                       "hit_equal": int((got_hit == o_hit).sum())}
            what = f"{sample} of the {b} queries (seeded subset) against the full cache"
        result["cpu_baseline"] = {"value": round(sample / cpu_s, 3), "unit": "queries/s", "cores": int(o_threads),
                                  "kind": "oracle", "sample": f"{what}, {cpu_s:.1f} s"}
        del host_entries, host_q
    fc.close()
    return result, data


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed steps of the headline workload (0 = 20)")
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="",
                    help="time this workload only; by default the headline workload c2_batched is followed by every "
                         "other benchmark configuration, reported under other_workloads of the same JSON line")
    ap.add_argument("--cache-copies", type=int, default=0,
                    help="identical copies of a single-layer cache the steps alternate between (0 = 2 when the cache is at most 2 GiB)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle leg (profiling runs)")
    ap.add_argument("--cpu-sample", type=int, default=0, help="queries in the oracle sample (0 = per workload)")
    ap.add_argument("--calibrate", action="store_true",
                    help="also measure what this GPU sustains on a pure MFMA loop and on a pure 1 GiB read")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy three times (reference for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--next-rows", action="store_true",
                    help="instead of a look-up workload, time the k-means cache (Sec. 4 of the paper) and the "
                         "projection in front of the look-up (Sec. 3) at the paper's scale; prints one JSON line")
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

    def copy_calibration():
        src = torch.zeros(1 << 28, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.bitwise_not(src, out=dst)   # a plain elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        return 1 << 30

    if args.next_rows:
        res = time_next_rows(torch, binding, dev)
        if args.copy_calibration:
            res["copy_calibration_bytes"] = copy_calibration()
        print(json.dumps(res))
        return 0

    head = args.workload or "c2_batched"
    result, data = run_workload(torch, np, binding, synth, dev, head, args.steps or STEPS.get(head, 20), args.warmup,
                                args.cache_copies, not args.no_cpu_baseline, args.cpu_sample)
    del data
    if not args.workload:
        # every other configuration, each with its own roofline / cpu_baseline / parity_sample block
        others, shared = [], None
        for name in ALL_WORKLOADS:
            if name == head:
                continue
            torch.cuda.empty_cache()
            reuse = shared if name == "c4_cascade_noisy" else None
            if reuse is not None:
                # same seeds, same activations: only the cache labels differ
                noisy = synth.make_workload_labels(synth.WORKLOADS[name])
                for L, lab in zip(reuse.layers, noisy):
                    L.labels = lab.to(dev)
            block, d = run_workload(torch, np, binding, synth, dev, name, STEPS.get(name, 20), args.warmup, 0,
                                    not args.no_cpu_baseline, 0, data=reuse)
            shared = d if name == "c4_cascade" else None
            del d
            for key in ("n_gpus", "higher_is_better", "scaling", "vs_baseline", "data"):
                block.pop(key, None)
            others.append(block)
        result["other_workloads"] = others

    if args.calibrate:
        scratch = torch.empty(1 << 22, dtype=torch.uint8, device=dev)
        tf, mhz = binding.freeze_calibrate_mfma(scratch)
        buf = torch.zeros(1 << 30, dtype=torch.uint8, device=dev)
        gbs = binding.freeze_calibrate_hbm_read(buf)
        del buf
        result["calibration"] = {"peaks_used": {"bf16_mfma_TFLOPs": PEAK_BF16_TFLOPS, "hbm_GBs": PEAK_HBM_GBS},
                                 "pure_mfma_loop_TFLOPs": round(tf, 1), "shader_clock_MHz_under_mfma": round(mhz),
                                 "pure_read_1GiB_GBs": round(gbs, 1)}
    if args.copy_calibration:
        result["config"]["copy_calibration_bytes"] = copy_calibration()
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
