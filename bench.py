#!/usr/bin/env python3
"""Benchmark of the multi-LoRA int4 layer step on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic rows: ONE
mlora_w4_layer_step call over all projections of the workload (group rows, shrink, base
product, expand) -- for the default workload, c4_decode, the 112 projections of a 16-layer
stack at 32 rows, which the library runs as one launch.  Weights, adapters and rows are
resident in HBM before the timed region; R independently seeded copies of all tensors are
cycled so that R * bytes >= 3 x 256 MiB and every step streams its weights from HBM rather
than from the last-level cache.

Prints ONE JSON line: value = algorithmic bytes per step / time per step (GB/s), with the time
per linear, the roofline block of the dominant kernel (HIP events around its launches), the
same stack run in dependency order (q,k,v | o | gate,up | down: four calls per layer), the
error of one layer against the CPU oracle, and the oracle timed on the host cores as a
reported baseline.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0          # dense bf16, MI355X
CACHE_BYTES = 256 << 20
METRIC = "µs per multi-LoRA W4 linear + achieved HBM GB/s (% of 8 TB/s), 1 MI355X"
# which roofline bounds a workload (the others are reported beside it)
BOUND = {"c1": "hbm", "c2": "hbm", "c4_decode": "hbm", "c5_up": "hbm", "c5_down": "hbm",
         "c3": "mfma", "c3_interleaved": "mfma", "c4_prefill": "mfma"}
DEPENDENCY_ORDER = (("q", "k", "v"), ("o",), ("gate", "up"), ("down",))


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c4_decode",
                    help="c4_decode (default), c1, c2, c3, c4_prefill, c5_up, c5_down, c4_attention, c4_ds2d, c4_layer")
    ap.add_argument("--mode", default="graph", choices=["graph", "eager"],
                    help="graph: the K steps are captured once in a HIP graph and replayed; "
                         "eager: one library call per step from Python")
    ap.add_argument("--streams", type=int, default=1, help="output streams of the c4_ds2d workload")
    ap.add_argument("--copies", type=int, default=0, help="rotating copies (0 = enough to defeat the cache)")
    ap.add_argument("--per-layer-calls", action="store_true",
                    help="one library call (one launch) per layer instead of one per step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dependency-order", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain device-to-device copies of 256 MiB (torch clone): a kernel of "
                         "known traffic next to which rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings "
                         "of the layer kernel can be scaled")
    ap.add_argument("--y-fp32", action="store_true")
    ap.add_argument("--lora-int16", action="store_true",
                    help="LoRA stacks stored as int16 with one scale per stack, expanded by the library into a "
                         "bf16 pair of four times the rank (layer-step workloads c1..c5, not with --a8)")
    ap.add_argument("--a8", action="store_true",
                    help="int8 activations with one scale per tensor (mlora_w4a8_layer_step) instead of bf16")
    return ap.parse_args()


def measured_traffic(kernel_tag: str, workload: str):
    """HBM bytes per launch from the tracked rocprofv3 --pmc summary of this kernel and workload
    (profiles/<kernel>_<workload>_hbm_traffic.txt, line 'hbm_traffic_bytes_per_launch = N'), or
    None if no such summary is there."""
    path = os.path.join(ROOT, "profiles", f"{kernel_tag}_{workload}_hbm_traffic.txt")
    if not os.path.exists(path):
        return None, None
    m = re.search(r"hbm_traffic_bytes_per_launch\s*=\s*(\d+)", open(path).read())
    return (int(m.group(1)), os.path.relpath(path, ROOT)) if m else (None, None)


def bench_ds2d(args):
    """--workload c4_ds2d: the token side of a DS2D step (verification of the draft tree and
    drafting of the next one) on the logits of one stream of the paper's worked example: 30 rows
    (branch (3, 2), two forecast embeddings) of 128256 bf16 logits."""
    import numpy as np
    import torch

    import paper_2604_18655_amd as lib
    from oracle import ds2d as oracle_ds2d
    from workloads.ds2d import make_ds2d_inputs
    from workloads.generate import bf16_bits_to_f32

    lib.load_library()
    torch.cuda.set_device(0)
    S, m, branch, V = args.streams, 2, (3, 2), 128256
    T, R = lib.ds2d_rows(branch, m)
    call_bytes = S * R * V * 2
    copies = args.copies or (3 * CACHE_BYTES + call_bytes - 1) // call_bytes
    d = lib.Ds2dStep(S, m, branch, branch, V, lib.Y_BF16)
    t0 = time.time()
    logits0, tokens0 = make_ds2d_inputs(0, S, branch, m, V, True, accept=0.8)
    sets = []
    gen = torch.Generator(device="cuda").manual_seed(1234)
    for c in range(copies):
        if c == 0:
            lg = torch.from_numpy(logits0.view(np.int16)).cuda()
            tk = torch.from_numpy(tokens0).cuda()
        else:
            lg = (torch.randn((S * R, V), generator=gen, device="cuda") * 2.0).to(torch.bfloat16)
            tk = torch.randint(0, V, (S, T), generator=gen, device="cuda", dtype=torch.int32)
        outs = [torch.zeros(n, dtype=torch.int32, device="cuda") for n in (S, S * (m + 1), S * (m + 1), S * T)]
        ws = torch.empty(d.workspace_bytes(), dtype=torch.uint8, device="cuda")
        sets.append((lg, tk, outs, ws))
    torch.cuda.synchronize()
    setup_s = time.time() - t0

    def run_step(i, stream=None):
        lg, tk, outs, ws = sets[i % copies]
        d.run(lg, tk, outs[0], outs[1], outs[2], outs[3], ws, stream)

    for i in range(args.warmup):
        run_step(i)
    torch.cuda.synchronize()
    K = args.steps
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            for i in range(K):
                run_step(args.warmup + i, side.cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    graph.replay()
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    ev0.record()
    graph.replay()
    ev1.record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    call_s = ev0.elapsed_time(ev1) * 1e-3 / K

    # copy 0 against the oracle: every output is an integer and must match exactly
    ref = oracle_ds2d.step(branch, branch, m, bf16_bits_to_f32(logits0[:R]).astype(np.float64), tokens0[0])
    outs = [o.cpu().numpy() for o in sets[0][2]]
    a = len(ref["accepted_rows"]) - 1
    assert int(outs[0][0]) == a and list(outs[1][:a + 1]) == ref["accepted_rows"]
    assert list(outs[2][:a + 1]) == ref["emitted"] and list(outs[3][:T]) == ref["next_tokens"]
    gbs = call_bytes / (elapsed / K) / 1e9
    result = {
        "metric": "µs per DS2D verify-and-draft step + achieved HBM GB/s (% of 8 TB/s), 1 MI355X",
        "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": round(elapsed * 1e3 / K, 6), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "c4_ds2d: verification and drafting on the logits of one DS2D step",
                   "streams": S, "branch": list(branch), "forecast_embeddings": m, "rows": R, "vocab": V,
                   "rotating_copies": int(copies), "launch_mode": "graph"},
        "us_per_step": round(elapsed * 1e6 / K, 3), "pct_of_hbm_peak": round(100.0 * gbs / HBM_PEAK_GBS, 2),
        "algorithmic_bytes_per_step": call_bytes, "oracle_match": "exact", "setup_s": round(setup_s, 1),
        "roofline": {"kernel": "ds2d_best_partial<bf16> + ds2d_verify_draft (one call)", "bound": "hbm",
                     "achieved": round(call_bytes / call_s / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(call_bytes / call_s / 1e9 / HBM_PEAK_GBS, 4), "traffic": None,
                     "algorithmic_bytes_per_launch": int(call_bytes), "avg_launch_us": round(call_s * 1e6, 3),
                     "launches_timed": K,
                     "timed_with": "two HIP events around the timed region on the launch stream"},
    }
    if not args.no_cpu_baseline:
        t0 = time.perf_counter()
        n = 0
        while time.perf_counter() - t0 < 10.0:
            oracle_ds2d.step(branch, branch, m, bf16_bits_to_f32(logits0[:R]).astype(np.float64), tokens0[0])
            n += 1
        dt = (time.perf_counter() - t0) / n
        result["cpu_baseline"] = {"value": round(call_bytes / S / dt / 1e9, 4), "unit": "GB/s", "cores": 1,
                                  "kind": "oracle", "sample": f"{n} steps of one stream of the same workload, {dt:.2f} s each"}
    print(json.dumps(result))


def bench_layer(args):
    """--workload c4_layer: ONE decoder layer of the 1B-like model with its true dependencies, at the
    rows of the c4 decoding step (8 streams x 4 tree rows): rms scale, fused q/k/v (+ rotary
    encoding), masked tree attention, o (+ residual; leaves the sums of squares of its rows),
    fused gate/up (row scale from those sums, + SwiGLU), down (+ residual): 6 library calls, 7
    launches per step."""
    import numpy as np
    import torch

    import oracle
    import paper_2604_18655_amd as lib
    import workloads as wl
    from oracle import layer_glue as glue
    from paper_2604_18655_amd import device
    from paper_2604_18655_amd.decoder import DecoderLayerStep
    from workloads.generate import bf16_bits_to_f32, f32_to_bf16_bits

    lib.load_library()
    torch.cuda.set_device(0)
    S, R, Hq, Hkv, D, H, KV, F, Lp, cap = 8, 4, 32, 8, 64, 2048, 512, 8192, 2048, 128
    M, n_ad, rank = S * R, 8, 16
    parent, fc = np.asarray([-1, 0, 0, 1], np.int32), np.zeros(4, np.uint8)
    shapes = wl.llama1b_layer_shapes()
    rows = wl.make_rows("block:4", M, n_ad, 4)
    U = len(set(int(a) for a in rows if a >= 0))
    lin_bytes = sum(wl.algorithmic_bytes(p, M, U, 2) for p in shapes)
    copies = args.copies or 16
    t0 = time.time()
    layers, host0 = [], None
    att_bytes = 0
    for c in range(copies):
        mk = lambda i: wl.make_problem(shapes[i], 40, c, i)
        host = {"q": mk(0), "k": mk(1), "v": mk(2), "o": mk(3), "gate_up": wl.fuse_gate_up(mk(4), mk(5)), "down": mk(6)}
        dev = {k: device.upload_problem(p) for k, p in host.items()}
        inp = wl.make_attention_inputs(5000 + c, S, parent, fc, Hq, Hkv, D, Lp, 0, cap)
        dd = lambda a: device.to_device(a) if a.size else None
        k_new = torch.zeros((M, KV), dtype=torch.int16, device="cuda")
        v_new = torch.zeros((M, KV), dtype=torch.int16, device="cuda")
        att = lib.TreeAttention(Hq, Hkv, D, S, R, inp.scale, dd(inp.k_prefill), dd(inp.v_prefill), None, None,
                                dd(inp.k_stream), dd(inp.v_stream), torch.from_numpy(inp.len_stream).cuda(),
                                k_new, v_new, torch.from_numpy(inp.parent).cuda(),
                                torch.from_numpy(inp.is_forecast).cuda(), Lp, 0, cap)
        h = wl.make_x(M, H, 40, c, 9)
        ang = glue.rope_angles(np.random.default_rng(c).integers(0, 3000, M))
        cos, sin = np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)
        layer = DecoderLayerStep(dev["q"], dev["k"], dev["v"], dev["o"], dev["gate_up"], dev["down"], att,
                                 device.to_device(h), torch.from_numpy(cos).cuda(), torch.from_numpy(sin).cuda(),
                                 torch.from_numpy(rows).cuda(), M)
        layers.append(layer)
        if c == 0:
            host0 = (host, inp, h, cos, sin)
            att_bytes = 2 * 2 * Hkv * D * (Lp + int(inp.len_stream.sum())) + 2 * 2 * M * Hkv * D + 2 * 2 * M * Hq * D
    torch.cuda.synchronize()
    setup_s = time.time() - t0
    step_bytes = lin_bytes + att_bytes

    def run_step(i, stream=None):
        layers[i % copies].run(stream)

    for i in range(args.warmup):
        run_step(i)
    torch.cuda.synchronize()
    K = args.steps
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            for i in range(K):
                run_step(args.warmup + i, side.cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    graph.replay()
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    ev0.record()
    graph.replay()
    ev1.record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    step_s = ev0.elapsed_time(ev1) * 1e-3 / K
    for layer in layers:
        assert lib.workspace_status(layer.ws) == 0

    # copy 0 against the oracle's own chain (intermediates rounded to bf16 where the device stores bf16)
    host, inp, h, cos, sin = host0
    f64 = lambda bits: bf16_bits_to_f32(bits).astype(np.float64)
    rb = lambda y: f32_to_bf16_bits(y.astype(np.float32))
    lin = lambda key, x_bits, **kw: glue.fused_linear(host[key].wq, host[key].scales, 32, host[key].lora_a,
                                                      host[key].lora_b, 2.0, x_bits, rows, **kw)
    att_o = lambda q, k, v: oracle.tree_attention(q.reshape(M, Hq, D), inp.k_prefill, inp.v_prefill, inp.k_fprefix,
                                                  inp.v_fprefix, inp.k_stream, inp.v_stream, inp.len_stream,
                                                  k.reshape(M, Hkv, D), v.reshape(M, Hkv, D), inp.parent,
                                                  inp.is_forecast, S, inp.scale).reshape(M, Hq * D)

    def oracle_layer():
        s1 = glue.rms_scale(f64(h), 1e-5)
        rope = dict(row_scale=s1, pair_op="rope", cos=cos, sin=sin)
        q, k, v = rb(lin("q", h, **rope)), rb(lin("k", h, **rope)), rb(lin("v", h, row_scale=s1))
        h2 = rb(lin("o", rb(att_o(q, k, v)), residual_bits=h))
        act = rb(lin("gate_up", h2, row_scale=glue.rms_scale(f64(h2), 1e-5), pair_op="swiglu"))
        return lin("down", act, residual_bits=h2)

    t1 = time.perf_counter()
    ref = oracle_layer()
    t_cpu = time.perf_counter() - t1
    got = f64(layers[0].out.cpu().numpy().view(np.uint16))
    max_rel_err = float(np.max(np.abs(got - ref)) / np.max(np.abs(ref)))
    assert max_rel_err <= 2e-2, max_rel_err
    gbs = step_bytes / (elapsed / K) / 1e9
    result = {
        "metric": "µs per decoder layer step (7 multi-LoRA W4 projections + tree attention + glue) + achieved HBM GB/s, 1 MI355X",
        "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": round(elapsed * 1e3 / K, 6), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "c4_layer: one decoder layer of the 1B-like model in dependency order, 8 streams x 4 tree rows",
                   "M": M, "hidden": H, "kv_width": KV, "ffn": F, "n_q_heads": Hq, "n_kv_heads": Hkv, "head_dim": D,
                   "len_prefill": Lp, "cap_stream": cap, "group": 32, "rank": rank, "n_adapters": n_ad,
                   "distinct_adapters": U, "calls_per_step": 6, "launches_per_step": 7,
                   "rotating_copies": copies, "launch_mode": "graph"},
        "us_per_step": round(elapsed * 1e6 / K, 3), "pct_of_hbm_peak": round(100.0 * gbs / HBM_PEAK_GBS, 2),
        "algorithmic_bytes_per_step": int(step_bytes), "max_rel_err": float(f"{max_rel_err:.3e}"),
        "setup_s": round(setup_s, 1),
        "roofline": {"kernel": "layer_kernel<1, 16> x 4 + tree_attn_partial/combine + rms_scale_kernel (one step)",
                     "bound": "hbm", "achieved": round(step_bytes / step_s / 1e9, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(step_bytes / step_s / 1e9 / HBM_PEAK_GBS, 4), "traffic": None,
                     "algorithmic_bytes_per_launch": int(step_bytes), "avg_launch_us": round(step_s * 1e6, 3),
                     "launches_timed": K,
                     "timed_with": "two HIP events around the timed region on the launch stream"},
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = {"value": round(step_bytes / t_cpu / 1e9, 4), "unit": "GB/s",
                                  "cores": oracle.max_threads(), "kind": "oracle",
                                  "sample": f"one whole layer of the same workload, {t_cpu:.1f} s",
                                  "us_per_step": round(t_cpu * 1e6, 1)}
    print(json.dumps(result, ensure_ascii=False), flush=True)


def bench_attention(args):
    """--workload c4_attention: the masked tree attention of the 16-layer stack's decoding step
    (8 streams x 4 tree rows, 32 query heads on 8 kv heads of 64 features, 2048 prefill
    positions, up to 128 positions per stream), one call per layer, 16 calls per step."""
    import numpy as np
    import torch

    import oracle
    import paper_2604_18655_amd as lib
    import workloads as wl
    from paper_2604_18655_amd import device

    lib.load_library()
    torch.cuda.set_device(0)
    S, Hq, Hkv, D, Lp, Lf, cap, layers = 8, 32, 8, 64, 2048, 0, 128, 16
    parent, fc = np.asarray([-1, 0, 0, 1], np.int32), np.zeros(4, np.uint8)
    R, M = 4, 32
    copies = args.copies or 9                         # 9 x 16 layers x 6 MB > 3 x 256 MiB
    dev = lambda a: device.to_device(a) if a.size else None
    calls, host0 = [], None
    t0 = time.time()
    step_bytes = 0
    for c in range(copies):
        for layer in range(layers):
            inp = wl.make_attention_inputs(1000 + c * layers + layer, S, parent, fc, Hq, Hkv, D, Lp, Lf, cap)
            t = lib.TreeAttention(Hq, Hkv, D, S, R, inp.scale, dev(inp.k_prefill), dev(inp.v_prefill),
                                  dev(inp.k_fprefix), dev(inp.v_fprefix), dev(inp.k_stream), dev(inp.v_stream),
                                  torch.from_numpy(inp.len_stream).cuda(), dev(inp.k_new), dev(inp.v_new),
                                  torch.from_numpy(inp.parent).cuda(), torch.from_numpy(inp.is_forecast).cuda(),
                                  Lp, Lf, cap)
            q = device.to_device(inp.q)
            out = torch.empty((M, Hq, D), dtype=torch.int16, device="cuda")
            ws = torch.empty(max(t.workspace_bytes(), 256), dtype=torch.uint8, device="cuda")
            calls.append((t, q, out, ws))
            if c == 0:
                # what a call has to move at least once: visible keys and values, q, the rows' k and v, out
                step_bytes += 2 * 2 * Hkv * D * (Lp + Lf + int(inp.len_stream.sum())) + 2 * 2 * M * Hkv * D + 2 * 2 * M * Hq * D
            if c == 0 and layer == 0:
                host0 = inp
    torch.cuda.synchronize()
    setup_s = time.time() - t0

    def run_step(i, stream=None):
        base = (i % copies) * layers
        for t, q, out, ws in calls[base:base + layers]:
            t.run(q, out, lib.Y_BF16, ws, stream)

    for i in range(args.warmup):
        run_step(i)
    torch.cuda.synchronize()
    K = args.steps
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            for i in range(K):
                run_step(args.warmup + i, side.cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    graph.replay()
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    ev0.record()
    graph.replay()
    ev1.record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    call_s = ev0.elapsed_time(ev1) * 1e-3 / (K * layers)

    ref = oracle.tree_attention(host0.q, host0.k_prefill, host0.v_prefill, host0.k_fprefix, host0.v_fprefix,
                                host0.k_stream, host0.v_stream, host0.len_stream, host0.k_new, host0.v_new,
                                host0.parent, host0.is_forecast, S, host0.scale)
    got = device.y_to_numpy(calls[0][2].reshape(M, Hq * D)).reshape(M, Hq, D)
    max_rel_err = float(np.max(np.abs(got - ref)) / np.max(np.abs(ref)))
    assert max_rel_err <= 5e-3, max_rel_err
    gbs = step_bytes / (elapsed / K) / 1e9
    call_bytes = step_bytes / layers
    result = {
        "metric": "µs per masked tree attention call + achieved HBM GB/s (% of 8 TB/s), 1 MI355X",
        "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": round(elapsed * 1e3 / K, 6), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "c4_attention: tree attention of the 16-layer stack's decoding step, one call per layer",
                   "streams": S, "rows_per_stream": R, "n_q_heads": Hq, "n_kv_heads": Hkv, "head_dim": D,
                   "len_prefill": Lp, "len_fprefix": Lf, "cap_stream": cap, "layers": layers,
                   "rotating_copies": copies, "launch_mode": "graph"},
        "us_per_step": round(elapsed * 1e6 / K, 3), "us_per_call": round(elapsed * 1e6 / K / layers, 3),
        "pct_of_hbm_peak": round(100.0 * gbs / HBM_PEAK_GBS, 2), "algorithmic_bytes_per_step": step_bytes,
        "max_rel_err": float(f"{max_rel_err:.3e}"), "setup_s": round(setup_s, 1),
        "roofline": {"kernel": "tree_attn_partial<64> + tree_attn_combine<64> (one call)", "bound": "hbm",
                     "achieved": round(call_bytes / call_s / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(call_bytes / call_s / 1e9 / HBM_PEAK_GBS, 4), "traffic": None,
                     "algorithmic_bytes_per_launch": int(call_bytes), "avg_launch_us": round(call_s * 1e6, 3),
                     "launches_timed": K * layers,
                     "timed_with": "two HIP events around the timed region on the launch stream"},
    }
    if not args.no_cpu_baseline:
        reps, t_cpu = 0, 0.0
        while t_cpu < 10.0 and reps < 100:
            t1 = time.perf_counter()
            oracle.tree_attention(host0.q, host0.k_prefill, host0.v_prefill, host0.k_fprefix, host0.v_fprefix,
                                  host0.k_stream, host0.v_stream, host0.len_stream, host0.k_new, host0.v_new,
                                  host0.parent, host0.is_forecast, S, host0.scale)
            t_cpu += time.perf_counter() - t1
            reps += 1
        result["cpu_baseline"] = {"value": round(call_bytes * reps / t_cpu / 1e9, 4), "unit": "GB/s", "cores": 1,
                                  "kind": "oracle", "sample": f"layer 0, {reps} repetitions, {t_cpu:.1f} s of fp64 loops on 1 thread",
                                  "us_per_call": round(t_cpu / reps * 1e6, 1)}
    print(json.dumps(result, ensure_ascii=False), flush=True)


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path shards along N, see DESIGN.md); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    if args.a8 and args.lora_int16:
        print("bench.py: --a8 and --lora-int16 are separate variants", file=sys.stderr)
        sys.exit(2)
    if args.workload == "c4_ds2d":
        bench_ds2d(args)
        return
    if args.workload == "c4_layer":
        bench_layer(args)
        return
    if args.workload == "c4_attention":
        bench_attention(args)
        return

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
    n_proj = len(w.projs)

    rows0 = wl.make_rows(w.row_map, M, w.projs[0].n_adapters, w.cfg_id)
    U = len(set(int(a) for a in rows0 if a >= 0))
    layer_bytes = sum(wl.algorithmic_bytes(p, M, U, ysz) - (M * p.K if args.a8 else 0) for p in w.projs)   # int8 rows: half the bytes of x
    layer_flops = sum(wl.algorithmic_flops(p, M) for p in w.projs)
    step_bytes, step_flops = layer_bytes * w.layers, layer_flops * w.layers

    # rotating copies: each "copy" is a full set of w.layers layers
    copies = args.copies or max(2 if w.layers > 1 else 1, math.ceil(3 * CACHE_BYTES / step_bytes))
    t0 = time.time()
    sets = []                       # per copy: (projs, dxs, ys, ra) over all layers
    host_layer0 = None
    host_scales0 = None
    for c in range(copies):
        projs, dxs, ys, x_scales = [], [], [], []
        for layer in range(w.layers):
            if args.lora_int16:
                probs = [wl.make_problem_lora_int16(s_, w.cfg_id, c * w.layers + layer, i) for i, s_ in enumerate(w.projs)]
                _, xs, rows = wl.make_layer_inputs(w, layer=c * w.layers + layer)
                projs += [device.upload_problem_lora_int16(p, dev) for p in probs]
            else:
                probs, xs, rows = wl.make_layer(w, layer=c * w.layers + layer)
                projs += [device.upload_problem(p, dev) for p in probs]
            cache = {}
            if args.a8:
                xs = list(xs)
                for x in list(xs):
                    if id(x) not in cache:
                        xq, sc = wl.quantise_act_int8(wl.bf16_bits_to_f32(x))
                        cache[id(x)] = (torch.from_numpy(xq).to(dev), xq, float(sc))
                xs_q = [cache[id(x)][1] for x in xs]
                x_scales += [cache[id(x)][2] for x in xs]
                dxs += [cache[id(x)][0] for x in xs]
                if c == 0 and layer == 0:
                    host_scales0 = [cache[id(x)][2] for x in xs]
                xs = xs_q
            else:
                for x in xs:
                    if id(x) not in cache:
                        cache[id(x)] = device.to_device(x, dev)
                    dxs.append(cache[id(x)])
            ys += [device.alloc_y(M, p.shape.N, y_dtype, dev) for p in probs]
            if c == 0 and layer == 0:
                host_layer0 = (probs, xs, rows)
        ra = torch.from_numpy(rows).to(dev)
        sets.append((projs, dxs, ys, ra, x_scales))
    # one workspace per copy, sized for the whole step: the calls of a step follow each other on
    # one stream, and a workspace serves calls of any geometry one after another
    plans, dep_plans, workspaces = [], [], []
    for projs, dxs, ys, ra, x_scales in sets:
        if args.a8:
            ws = torch.zeros(max(lib.a8_workspace_bytes(projs, M), 256), dtype=torch.uint8, device=dev)
            workspaces.append(ws)
            plans.append([lib.LayerPlanA8(projs, dxs, x_scales, ys, ra, M, y_dtype, ws)])
            continue
        # (sized for the largest of the calls that will use it: the whole step, and each of the
        # dependency-order calls, whose smaller launches may be cut differently)
        names = [p.name for p in w.projs]
        dep_ok = n_proj == 7 and all(any(n in grp for grp in DEPENDENCY_ORDER) for n in names)
        need = lib.workspace_bytes(projs, M)
        if dep_ok:
            for grp in DEPENDENCY_ORDER:
                need = max(need, lib.workspace_bytes([projs[names.index(n)] for n in grp], M))
        ws = torch.zeros(max(need, 256), dtype=torch.uint8, device=dev)
        workspaces.append(ws)
        if args.per_layer_calls:
            plans.append([lib.LayerPlan(projs[l * n_proj:(l + 1) * n_proj], dxs[l * n_proj:(l + 1) * n_proj],
                                        ys[l * n_proj:(l + 1) * n_proj], ra, M, y_dtype, ws)
                          for l in range(w.layers)])
        else:
            plans.append([lib.LayerPlan(projs, dxs, ys, ra, M, y_dtype, ws)])
        if dep_ok:
            calls = []
            for l in range(w.layers):
                for grp in DEPENDENCY_ORDER:
                    idx = [l * n_proj + names.index(n) for n in grp]
                    calls.append(lib.LayerPlan([projs[i] for i in idx], [dxs[i] for i in idx],
                                               [ys[i] for i in idx], ra, M, y_dtype, ws))
            dep_plans.append(calls)
    torch.cuda.synchronize()
    setup_s = time.time() - t0
    calls_per_step = len(plans[0])

    def run_step(i, stream=None, table=plans):
        for plan in table[i % copies]:
            plan.run(stream)

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        src.fill_(1)
        for _ in range(4):
            dst = src.clone()             # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    def timed(table, K, warmup):
        """Exactly K steps between two synchronisations (wall clock), and the same region between
        two HIP events recorded on the stream the launches go to."""
        for i in range(warmup):
            run_step(i, None, table)
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        if args.mode == "graph":
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                with torch.cuda.graph(graph, stream=side):
                    for i in range(K):
                        run_step(warmup + i, side.cuda_stream, table)
            torch.cuda.current_stream().wait_stream(side)
            graph.replay()                    # untimed: the first replay uploads the graph
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
                run_step(warmup + i, None, table)
            ev1.record()
            torch.cuda.synchronize()
            elapsed = time.perf_counter() - t_start
        return elapsed, ev0.elapsed_time(ev1) * 1e-3

    K = args.steps
    elapsed, ev_s = timed(plans, K, args.warmup)
    ms_per_step = elapsed * 1e3 / K
    gbs = step_bytes / (elapsed / K) / 1e9

    # ---- after the timed region: no block gave up waiting, and the outputs are right
    for ws in workspaces:
        assert lib.workspace_status(ws) == 0, "a block gave up waiting for another: results invalid"
    import oracle
    from oracle import lora_int16 as lora_int16_oracle
    probs0, xs0, rows_h = host_layer0
    max_rel_err = 0.0
    sample = list(range(n_proj)) if M <= 64 else [0, n_proj - 1]
    msel = np.arange(M) if M <= 64 else np.unique(np.concatenate([[0, M - 1], np.arange(0, M, 37)]))
    for i in sample:
        p = probs0[i]
        if args.a8:
            ref = oracle.linear_a8(p.wq, p.scales, p.shape.group, p.lora_a, p.lora_b, p.shape.alpha,
                                   np.ascontiguousarray(xs0[i][msel]), host_scales0[i], np.ascontiguousarray(rows_h[msel]))
        elif args.lora_int16:
            ref = lora_int16_oracle.linear(p.wq, p.scales, p.shape.group, p.aq, p.s_a, p.bq, p.s_b, p.shape.alpha,
                                           np.ascontiguousarray(xs0[i][msel]), np.ascontiguousarray(rows_h[msel]))
        else:
            ref = oracle.linear(p.wq, p.scales, p.shape.group, p.lora_a, p.lora_b, p.shape.alpha,
                                np.ascontiguousarray(xs0[i][msel]), np.ascontiguousarray(rows_h[msel]))
        got = device.y_to_numpy(sets[0][2][i])[msel]
        max_rel_err = max(max_rel_err, float(np.max(np.abs(got - ref)) / np.max(np.abs(ref))))
    assert max_rel_err <= (2e-4 if args.y_fp32 else 5e-3), max_rel_err

    # ---- the dominant (only) kernel; which one and how many launches a call makes is asked of
    # the library itself
    info = lib.layer_step_plan(plans[0][0].keep[0], M)
    if args.a8:                                  # always blocks of four column tiles, one launch per 128 projections
        info = dict(info, wide=True, launches=math.ceil(len(plans[0][0].keep[0]) / 128))
    launches_per_step = calls_per_step * info["launches"]
    n_ev = K * launches_per_step
    kern_s = ev_s / n_ev
    base_bytes = step_bytes / launches_per_step
    achieved = base_bytes / kern_s / 1e9
    wide = info["wide"]
    spg = w.projs[0].group // 32
    kernel_name = ("wide_kernel<%d, %d, %s>" % (spg, 2 if M <= 32 else 4, "true" if args.a8 else "false")) if wide else \
        "layer_kernel<%s>" % ("1, 8" if M <= 8 else "1, 16" if info["rows_per_chunk"] == 16 else "2, 24" if M <= 24 else "2, 32")
    kernel_tag = ("wide_kernel_a8" if args.a8 else "wide_kernel") if wide else "layer_kernel"
    achieved_tflops = (step_flops / launches_per_step) / kern_s / 1e12
    bound = BOUND.get(w.key, "hbm")
    traffic, traffic_src = measured_traffic(kernel_tag, w.key) if not (args.per_layer_calls or args.lora_int16) else (None, None)

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
        "dtype": "int8 x int4 -> int32, fp32 scales" if args.a8 else "bf16",
        "data": "synthetic",
        "config": {
            "workload": f"{w.key}: {w.description}",
            "projections": [f"{p.name} {p.K}x{p.N}" for p in w.projs],
            "M": M, "group": w.projs[0].group, "rank": w.projs[0].rank,
            "n_adapters": w.projs[0].n_adapters, "distinct_adapters": U, "layers": w.layers,
            "y_dtype": "fp32" if args.y_fp32 else "bf16", "x_dtype": "int8, one scale per tensor" if args.a8 else "bf16",
            "rotating_copies": copies, "launch_mode": args.mode,
            "calls_per_step": calls_per_step,
            **({"lora": "int16 stacks, one scale each; served as a bf16 pair of rank %d (4x the bytes of the int16 "
                        "tensors, which are what the algorithmic bytes count)" % (4 * w.projs[0].rank)} if args.lora_int16 else {}),
        },
        "us_per_step": round(ms_per_step * 1e3, 3),
        "us_per_linear": round(ms_per_step * 1e3 / (n_proj * w.layers), 3),
        "pct_of_hbm_peak": round(100.0 * gbs / HBM_PEAK_GBS, 2),
        "algorithmic_bytes_per_step": step_bytes,
        "tflops": round(step_flops / (elapsed / K) / 1e12, 3),
        "max_rel_err": float(f"{max_rel_err:.3e}"),
        "status_word": 0,
        "setup_s": round(setup_s, 1),
        "roofline": {
            "kernel": kernel_name,
            "bound": bound,
            "achieved": round(achieved_tflops, 1) if bound == "mfma" else round(achieved, 1),
            "peak": MFMA_BF16_PEAK_TFLOPS if bound == "mfma" else HBM_PEAK_GBS,
            "unit": "TFLOP/s" if bound == "mfma" else "GB/s",
            "frac": round(achieved_tflops / MFMA_BF16_PEAK_TFLOPS, 4) if bound == "mfma" else round(achieved / HBM_PEAK_GBS, 4),
            "hbm_gbs": round(achieved, 1), "hbm_frac": round(achieved / HBM_PEAK_GBS, 4),
            "mfma_tflops": round(achieved_tflops, 1), "mfma_frac": round(achieved_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
            "traffic": traffic,
            "traffic_source": traffic_src,
            "algorithmic_bytes_per_launch": int(base_bytes),
            "avg_launch_us": round(kern_s * 1e6, 3),
            "launches_timed": n_ev,
            "timed_with": "two HIP events around the timed region on the launch stream",
        },
    }

    # per-step times of a short eager loop (one HIP event pair per step): spread, next to the mean above
    n_each = min(50, K)
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_each)]
    for i, (e0, e1) in enumerate(pairs):
        e0.record()
        run_step(args.warmup + i, None, plans)
        e1.record()
    torch.cuda.synchronize()
    each = sorted(e0.elapsed_time(e1) * 1e3 for e0, e1 in pairs)
    result["eager_per_step_us"] = {"n": n_each, "min": round(each[0], 3), "median": round(each[n_each // 2], 3),
                                   "max": round(each[-1], 3),
                                   "what": "one event pair per step, launched from Python one by one"}

    if dep_plans and not args.no_dependency_order:
        Kd = max(1, K // 4)
        el_d, _ = timed(dep_plans, Kd, min(args.warmup, 5))
        for ws in workspaces:
            assert lib.workspace_status(ws) == 0
        result["dependency_order"] = {
            "what": "the same stack as four calls per layer (q,k,v | o | gate,up | down), one workspace",
            "calls_per_step": len(dep_plans[0]), "steps": Kd,
            "us_per_step": round(el_d / Kd * 1e6, 3),
            "value": round(step_bytes / (el_d / Kd) / 1e9, 1), "unit": "GB/s",
            "pct_of_hbm_peak": round(100.0 * step_bytes / (el_d / Kd) / 1e9 / HBM_PEAK_GBS, 2),
        }

    if not args.no_cpu_baseline:
        cores = oracle.max_threads()
        reps, t_cpu = 0, 0.0
        while t_cpu < 10.0 and reps < 1000:
            t1 = time.perf_counter()
            for i, (p, x) in enumerate(zip(probs0, xs0)):
                if args.a8:
                    oracle.linear_a8(p.wq, p.scales, p.shape.group, p.lora_a, p.lora_b, p.shape.alpha, x, host_scales0[i], rows_h)
                elif args.lora_int16:
                    lora_int16_oracle.linear(p.wq, p.scales, p.shape.group, p.aq, p.s_a, p.bq, p.s_b, p.shape.alpha, x, rows_h)
                else:
                    oracle.linear(p.wq, p.scales, p.shape.group, p.lora_a, p.lora_b, p.shape.alpha, x, rows_h)
            t_cpu += time.perf_counter() - t1
            reps += 1
        result["cpu_baseline"] = {
            "value": round(layer_bytes * reps / t_cpu / 1e9, 4),
            "unit": "GB/s",
            "cores": cores,
            "kind": "oracle",
            "sample": f"layer 0 of {w.key} ({len(probs0)} projections, M={M}), {reps} repetitions, "
                      f"{t_cpu:.1f} s of fp64 loops on {cores} threads",
            "us_per_linear": round(t_cpu / reps / len(probs0) * 1e6, 1),
        }
        if w.key in ("c1", "c2", "c3") and not args.a8 and not args.lora_int16:
            # the small configurations also on ONE host thread (bounded the same way)
            oracle.set_threads(1)
            reps1, t1_cpu = 0, 0.0
            while t1_cpu < 10.0 and reps1 < 1000:
                t1 = time.perf_counter()
                for p, x in zip(probs0, xs0):
                    oracle.linear(p.wq, p.scales, p.shape.group, p.lora_a, p.lora_b, p.shape.alpha, x, rows_h)
                t1_cpu += time.perf_counter() - t1
                reps1 += 1
            oracle.set_threads(cores)
            result["cpu_baseline"]["single_thread"] = {
                "value": round(layer_bytes * reps1 / t1_cpu / 1e9, 4), "unit": "GB/s", "cores": 1,
                "us_per_linear": round(t1_cpu / reps1 / len(probs0) * 1e6, 1),
                "sample": f"the same layer, {reps1} repetitions, {t1_cpu:.1f} s on 1 thread"}
    print(json.dumps(result, ensure_ascii=False), flush=True)


if __name__ == "__main__":
    main()
