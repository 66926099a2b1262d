#!/usr/bin/env python3
"""Benchmark of the multi-LoRA int4 layer step on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic rows: one
mlora_w4_layer_step call over all projections of the workload (group rows, shrink, base
product, expand).  Weights, adapters and rows are resident in HBM before the timed region;
R independently seeded copies of all tensors are cycled so that R * bytes >= 3 x 256 MiB and
every step streams its weights from HBM rather than from the last-level cache.

Prints ONE JSON line: value = algorithmic bytes per step / time per step (GB/s), with the time
per linear, the roofline block of the dominant kernel (HIP events around each of its launches)
and the CPU oracle timed on the host cores as a reported baseline.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0          # dense bf16, MI355X
CACHE_BYTES = 256 << 20
METRIC = "µs per multi-LoRA W4 linear + achieved HBM GB/s (% of 8 TB/s), 1 MI355X"

# HBM traffic per launch of the dominant kernel from rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE),
# scaled by a copy kernel of known size; see profiles/.  None until measured for a workload.
MEASURED_TRAFFIC = {"c2": 49030614}     # bytes per launch: profiles/layer_kernel_c2_hbm_traffic.txt


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="c2", help="c2 (default), c1, c3, c4_decode, c4_prefill, c5_up, c5_down")
    ap.add_argument("--mode", default="graph", choices=["graph", "eager"],
                    help="graph: the K steps are captured once in a HIP graph and replayed; "
                         "eager: one library call per step from Python")
    ap.add_argument("--copies", type=int, default=0, help="rotating copies (0 = enough to defeat the cache)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain device-to-device copies of 256 MiB (torch clone): a kernel of "
                         "known traffic next to which rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings "
                         "of the layer kernel can be scaled")
    ap.add_argument("--y-fp32", action="store_true")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path shards along N, see DESIGN.md); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2604_18655_amd as lib
    import workloads as wl
    from paper_2604_18655_amd import device

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    lib.load_library()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = wl.WORKLOADS[args.workload]
    y_dtype = lib.Y_FP32 if args.y_fp32 else lib.Y_BF16
    ysz = 4 if args.y_fp32 else 2
    M = w.M

    rows0 = wl.make_rows(w.row_map, M, w.projs[0].n_adapters, w.cfg_id)
    U = len(set(int(a) for a in rows0 if a >= 0))
    layer_bytes = sum(wl.algorithmic_bytes(p, M, U, ysz) for p in w.projs)
    layer_flops = sum(wl.algorithmic_flops(p, M) for p in w.projs)

    step_bytes, step_flops = layer_bytes * w.layers, layer_flops * w.layers

    # rotating copies: each "copy" is a full set of w.layers layers
    copies = args.copies or max(1, math.ceil(3 * CACHE_BYTES / step_bytes))
    t0 = time.time()
    plans, host_sets = [], []
    for c in range(copies):
        for layer in range(w.layers):
            probs, xs, rows = wl.make_layer(w, layer=c * w.layers + layer)
            projs = [device.upload_problem(p, dev) for p in probs]
            cache, dxs = {}, []
            for x in xs:
                if id(x) not in cache:
                    cache[id(x)] = device.to_device(x, dev)
                dxs.append(cache[id(x)])
            ra = torch.from_numpy(rows).to(dev)
            ys = [device.alloc_y(M, p.shape.N, y_dtype, dev) for p in probs]
            ws = device.alloc_workspace(projs, M, dev)
            plans.append(lib.LayerPlan(projs, dxs, ys, ra, M, y_dtype, ws))
            if c == 0 and layer == 0:
                host_sets.append((probs, xs, rows))
    torch.cuda.synchronize()
    setup_s = time.time() - t0
    calls_per_step = w.layers
    n_plans = len(plans)

    def run_step(i, stream=None):
        base = (i % copies) * calls_per_step
        for l in range(calls_per_step):
            plans[base + l].run(stream)

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        src.fill_(1)
        for _ in range(4):
            dst = src.clone()             # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    # ---- warm-up, then the timed region: exactly K steps between two synchronisations
    for i in range(args.warmup):
        run_step(i)
    torch.cuda.synchronize()

    K = args.steps
    # The timed region: exactly K steps between two synchronisations (wall clock), and the same
    # region between two HIP events recorded on the stream the launches go to, which gives the
    # average duration of the one kernel a layer call launches (launch gap included).
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if args.mode == "graph":
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for i in range(K):
                    run_step(args.warmup + i, side.cuda_stream)
        torch.cuda.current_stream().wait_stream(side)
        graph.replay()                    # untimed: first replay uploads the graph
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        ev0.record()
        graph.replay()
        ev1.record()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t_start
    else:
        t_start = time.perf_counter()
        ev0.record()
        for i in range(K):
            run_step(args.warmup + i)
        ev1.record()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t_start
    ms_per_step = elapsed * 1e3 / K
    gbs = step_bytes / (elapsed / K) / 1e9

    # ---- the dominant (only) kernel: one launch per 16 projections of a layer call
    launches_per_step = calls_per_step * math.ceil(len(w.projs) / 16)
    n_ev = K * launches_per_step
    kern_ms = ev0.elapsed_time(ev1) / n_ev
    base_bytes = step_bytes / launches_per_step
    achieved = base_bytes / (kern_ms * 1e-3) / 1e9
    wide = M >= 33                       # the library's kernel for 33 rows and more: bounded by the matrix units
    spg = w.projs[0].group // 32
    kernel_name = ("wide_kernel<%d>" % spg) if wide else \
        "layer_kernel<%s>" % ("1, 8" if M <= 8 else "1, 16" if M <= 16 else "2, 24" if M <= 24 else "2, 32")
    achieved_tflops = (step_flops / launches_per_step) / (kern_ms * 1e-3) / 1e12

    result = {
        "metric": METRIC,
        "value": round(gbs, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": f"{w.key}: {w.description}",
            "projections": [f"{p.name} {p.K}x{p.N}" for p in w.projs],
            "M": M, "group": w.projs[0].group, "rank": w.projs[0].rank,
            "n_adapters": w.projs[0].n_adapters, "distinct_adapters": U, "layers": w.layers,
            "y_dtype": "fp32" if args.y_fp32 else "bf16",
            "rotating_copies": copies, "launch_mode": args.mode,
        },
        "us_per_step": round(ms_per_step * 1e3, 3),
        "us_per_linear": round(ms_per_step * 1e3 / (len(w.projs) * w.layers), 3),
        "pct_of_hbm_peak": round(100.0 * gbs / HBM_PEAK_GBS, 2),
        "algorithmic_bytes_per_step": step_bytes,
        "tflops": round(step_flops / (elapsed / K) / 1e12, 3),
        "setup_s": round(setup_s, 1),
        "roofline": {
            "kernel": kernel_name,
            "bound": "mfma" if wide else "hbm",
            "achieved": round(achieved_tflops, 1) if wide else round(achieved, 1),
            "peak": MFMA_BF16_PEAK_TFLOPS if wide else HBM_PEAK_GBS,
            "unit": "TFLOP/s" if wide else "GB/s",
            "frac": round(achieved_tflops / MFMA_BF16_PEAK_TFLOPS, 4) if wide else round(achieved / HBM_PEAK_GBS, 4),
            "hbm_gbs": round(achieved, 1), "hbm_frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": MEASURED_TRAFFIC.get(w.key),
            "algorithmic_bytes_per_launch": int(base_bytes),
            "avg_launch_us": round(kern_ms * 1e3, 3),
            "launches_timed": n_ev,
            "timed_with": "two HIP events around the timed region on the launch stream",
        },
    }

    if not args.no_cpu_baseline:
        import oracle
        probs, xs, rows = host_sets[0]
        cores = oracle.max_threads()
        reps, t_cpu = 0, 0.0
        while t_cpu < 10.0 and reps < 1000:
            t1 = time.perf_counter()
            for p, x in zip(probs, xs):
                oracle.linear(p.wq, p.scales, p.shape.group, p.lora_a, p.lora_b, p.shape.alpha, x, rows)
            t_cpu += time.perf_counter() - t1
            reps += 1
        result["cpu_baseline"] = {
            "value": round(layer_bytes * reps / t_cpu / 1e9, 4),
            "unit": "GB/s",
            "cores": cores,
            "kind": "oracle",
            "sample": f"layer 0 of {w.key} ({len(probs)} projections, M={M}), {reps} repetitions, "
                      f"{t_cpu:.1f} s of fp64 loops on {cores} threads",
            "us_per_linear": round(t_cpu / reps / len(probs) * 1e6, 1),
        }
    print(json.dumps(result, ensure_ascii=False), flush=True)


if __name__ == "__main__":
    main()
