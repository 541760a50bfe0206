#!/usr/bin/env python3
"""Benchmark of the MoR analyse-select-quantize hot path on one MI355X.

A "step" is one pass of the whole path over the operand sweep of one Llama-style layer
(hidden 4096, ffn 14336, 8192 tokens): the 12 operands (activation 1x128, weights 128x128, gradients
per-tensor; Eq. 2, th = 4.5 %) go through ONE ``mor_analyze_quantize_batch`` call that also produces
each operand's selection statistics, on one stream, inputs already resident in HBM.  With
``--per-operand`` the same work is issued as 12 ``mor_analyze_quantize`` + 12 ``mor_select_stats`` calls.

Before the ``--warmup`` steps the step is run for ``--prewarm-ms`` of wall time and the JSON line says so
(``prewarm``): after an idle period (here: the seconds of host-side data generation) the GPU's power management
takes some tens of steps to settle -- the first handful run at full speed, the next twenty or so 5-10 % slower,
then the time per step becomes steady -- and a short warm-up would put the timed steps exactly into that window.

Prints ONE JSON line on stdout: whole-job throughput in GB/s of BF16 input, the roofline record
of the dominant kernel (timed live with HIP events recorded by the library around each kernel),
one measured row per configuration of the workload list (``configs``: the single operands at full size, each
rotated over enough buffer sets that the working set exceeds twice the 256 MB Infinity Cache), the further rows
of the method on the sweep's operands, and the CPU oracle timed on a bounded sample of the same workload.
Everything else goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak
META_BYTES = 17                # scale + amax + err_sum + nnz + mask per block
THRESHOLD = 0.045


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def csrc_sha256() -> str:
    """Hash of the kernel sources and the public header of this tree (what a rocprofv3 traffic measurement is tied to)."""
    import hashlib
    h = hashlib.sha256()
    base = os.path.join(ROOT, "paper_2512_22804_amd", "csrc")
    for f in sorted(os.listdir(base)) + [os.path.join("..", "..", "include", "mor.h")]:
        path = os.path.join(base, f)
        if os.path.isfile(path) and not f.endswith((".o", ".so")):
            h.update(os.path.basename(f).encode() + b"\0" + open(path, "rb").read())
    return h.hexdigest()[:16]


def algorithmic_bytes(kernel: str, n_elem: int, n_part: int, fallback_frac: float, fused: bool = False) -> float:
    """Bytes the method must move for one launch of `kernel` over an operand of n_elem elements.  `fused`: the
    per-tensor quantize pass also wrote the BF16 fallback (its decision was proven by the amax pass), so the
    copy pass moved nothing."""
    if kernel in ("sub1x128", "team_block"):
        return 2.0 * n_elem + n_elem + 2.0 * fallback_frac * n_elem + META_BYTES * n_part
    if kernel == "tensor_amax":
        return 2.0 * n_elem
    if kernel == "tensor_quant":
        return 2.0 * n_elem + n_elem + (2.0 * n_elem if fused else 0.0)
    if kernel == "fallback_copy":
        return 0.0 if fused else 4.0 * n_elem * fallback_frac
    if kernel in ("stats_partial",):
        return 9.0 * n_part
    return 0.0


def run_variants(ops, B, torch, dev, steps, log):
    """Times the further rows of the path on the same twelve operands: the paper's own tensor-level recipe
    (GAM scaling, one decision per tensor) at three partitions, E8M0 scales, the three-way recipe, 64 x 64 blocks,
    128 x 1 sub-columns, per-channel columns, fake quantization and de-quantization.  Each entry: ms per pass over
    all twelve operands, GB/s of BF16 input, algorithmic HBM GB/s and its fraction of the 8 TB/s peak."""
    n_total = sum(o["n"] for o in ops)
    results = []

    def timed(fn, iters):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        t0 = torch.cuda.Event(enable_timing=True); t1 = torch.cuda.Event(enable_timing=True)
        t0.record()
        for _ in range(iters):
            fn()
        t1.record()
        torch.cuda.synchronize()
        return t0.elapsed_time(t1) / iters

    def analyze_variant(name, gran_of, scope="partition", crit="mean_rel_err", scaling="fp32_amax", formats="e4m3|bf16", lean=False,
                        gam_group_rows=0):
        entries, outs = [], []
        for o in ops:
            gran = gran_of(o)
            params = B.make_params(o["params"].rows, o["params"].cols, gran, scope, crit, THRESHOLD, scaling=scaling, formats=formats,
                                   lean_fp8=lean, gam_group_rows=gam_group_rows)
            out = B.alloc_outputs(params, dev, want_bf16=True)
            out.workspace = None
            entries.append((params, o["x"], out, None))
            outs.append((o, gran, params, out))
        items = B.make_batch(entries)
        ws = torch.empty(max(16, B.mor_batch_workspace_bytes(items)), dtype=torch.uint8, device=dev)
        ms = timed(lambda: B.mor_analyze_quantize_batch(items, 1e-5, ws), steps)
        nbytes = 0.0
        n_fp8 = 0
        for o, gran, params, out in outs:
            mask = out.mask
            P = mask.numel()
            f = float((mask == 1).sum().item()) / P          # blocks are equal-sized here
            n_fp8 += int(round((1.0 - f) * o["n"]))
            n = o["n"]
            if gran == "tensor":
                b = 5.0 * n + 2.0 * n * f                       # amax pass + quantize pass (+ fallback written once)
                if lean:
                    b -= 1.0 * n * f                            # no FP8 payload for an operand known to stay in BF16
            else:
                b = 3.0 * n + META_BYTES * P
                if scope == "tensor" and ((scaling == "gam" and not gam_group_rows and gran in ("block128", "block64", "channel_row", "sub1x128", "sub128x1"))
                                          or gran == "channel_col"):
                    b += 2.0 * n * f                            # these inputs' BF16 decision is proven by the pre-pass: written by the block kernel
                elif scope == "tensor":
                    b += 4.0 * n * f                            # separate copy pass after the tensor-wide decision
                else:
                    b += 2.0 * n * f
                if gran == "channel_col":
                    b += 2.0 * n                                # column amax pass
                if scaling == "gam" and gran != "channel_col":      # (per-channel columns take the group amax from their column-amax pass)
                    b += 2.0 * n                                # group amax pre-pass (Algorithm 1, group loop)
            nbytes += b
        del outs, entries, items, ws
        rec = {"name": name, "ms": round(ms, 4), "input_gbs": round(2.0 * n_total / ms / 1e6, 1),
               "hbm_algorithmic_gbs": round(nbytes / ms / 1e6, 1), "hbm_frac_of_peak": round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 4),
               "fp8_pct_by_elements": round(100.0 * n_fp8 / n_total, 2)}
        log(f"[bench]   variant {name:34s} {ms:8.3f} ms  {rec['input_gbs']:8.1f} GB/s in  {rec['hbm_algorithmic_gbs']:8.1f} GB/s HBM "
            f"({100 * rec['hbm_frac_of_peak']:.1f} %)  FP8 {rec['fp8_pct_by_elements']:.1f} %")
        results.append(rec)
        torch.cuda.empty_cache()

    own = lambda o: o["gran"]
    const = lambda g: (lambda o: g)
    analyze_variant("hot_path_lean_fp8", own, lean=True)
    analyze_variant("gam_tensor_level_block128", const("block128"), scope="tensor", scaling="gam")
    analyze_variant("gam_tensor_level_block64", const("block64"), scope="tensor", scaling="gam")
    analyze_variant("gam_tensor_level_channel_row", const("channel_row"), scope="tensor", scaling="gam")
    analyze_variant("gam_tensor_level_channel_col", const("channel_col"), scope="tensor", scaling="gam")
    analyze_variant("gam_tensor_level_sub1x128", const("sub1x128"), scope="tensor", scaling="gam")
    analyze_variant("gam_tensor_level_sub128x1", const("sub128x1"), scope="tensor", scaling="gam")
    analyze_variant("gam_tensor_level_per_tensor", const("tensor"), scaling="gam")
    # Algorithm 1 with several groups per tensor: one mantissa per band of 128 rows, block decisions
    analyze_variant("gam_bands_of_128_rows_block128", const("block128"), scaling="gam", gam_group_rows=128)
    # the scaling ablation of Section 4.1.2 keeps the tensor-level decision and swaps the scaling algorithm
    analyze_variant("e8m0_tensor_level_block128", const("block128"), scope="tensor", scaling="e8m0")
    analyze_variant("fp32_amax_tensor_level_block128", const("block128"), scope="tensor")
    analyze_variant("e8m0_block128", const("block128"), scaling="e8m0")
    analyze_variant("two_way_eq3_block128", const("block128"), crit="e4m3_vs_e5m2")
    analyze_variant("three_way_eq3_block128", const("block128"), crit="e4m3_vs_e5m2", formats="e4m3|e5m2|bf16")
    analyze_variant("block64", const("block64"))
    analyze_variant("channel_row", const("channel_row"))
    analyze_variant("sub128x1", const("sub128x1"))
    analyze_variant("channel_col", const("channel_col"))

    # fake quantization at the sweep's own granularities, and de-quantization of the sweep's outputs
    metas, ys = [], []
    for o in ops:
        meta = B.alloc_outputs(o["params"], dev, want_bf16=False, want_fp8=False)
        metas.append(meta)
        ys.append(torch.empty_like(o["x"]))

    # the configuration of the paper's own experiments: fake quantization, tensor-level decision, GAM scales, 128x128 blocks
    for gran in ("block128", "channel_row"):
        entries, nbytes = [], 0.0
        for o, y in zip(ops, ys):
            pr = B.make_params(o["params"].rows, o["params"].cols, gran, "tensor", "mean_rel_err", THRESHOLD, scaling="gam")
            meta = B.alloc_outputs(pr, dev, want_bf16=False, want_fp8=False)
            entries.append((pr, o["x"], meta, None, y))
            # pre-pass 2, block pass 2 + 2 (these inputs' BF16 decisions are proven by the pre-pass, so nothing is copied afterwards)
            nbytes += 6.0 * o["n"] + META_BYTES * meta.mask.numel()
        items = B.make_batch(entries)
        ws = torch.empty(max(16, B.mor_batch_workspace_bytes(items)), dtype=torch.uint8, device=dev)
        ms = timed(lambda: B.mor_analyze_quantize_batch(items, 1e-5, ws), steps)
        rec = {"name": f"fake_gam_tensor_level_{gran}", "ms": round(ms, 4), "input_gbs": round(2.0 * n_total / ms / 1e6, 1),
               "hbm_algorithmic_gbs": round(nbytes / ms / 1e6, 1), "hbm_frac_of_peak": round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 4)}
        log(f"[bench]   variant {rec['name']:34s} {ms:8.3f} ms  {rec['input_gbs']:8.1f} GB/s in  {rec['hbm_algorithmic_gbs']:8.1f} GB/s HBM "
            f"({100 * rec['hbm_frac_of_peak']:.1f} %)")
        results.append(rec)
        del entries, items, ws

    fake_items = B.make_batch([(o["params"], o["x"], meta, None, y) for o, meta, y in zip(ops, metas, ys)])
    fake_ws = torch.empty(max(16, B.mor_batch_workspace_bytes(fake_items)), dtype=torch.uint8, device=dev)
    ms = timed(lambda: B.mor_analyze_quantize_batch(fake_items, 1e-5, fake_ws), steps)
    nbytes = sum((6.0 if o["gran"] == "tensor" else 4.0) * o["n"] + (0 if o["gran"] == "tensor" else META_BYTES * o["P"]) for o in ops)
    rec = {"name": "fake_quantize_cfg5", "ms": round(ms, 4), "input_gbs": round(2.0 * n_total / ms / 1e6, 1),
           "hbm_algorithmic_gbs": round(nbytes / ms / 1e6, 1), "hbm_frac_of_peak": round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 4)}
    log(f"[bench]   variant {rec['name']:34s} {ms:8.3f} ms  {rec['input_gbs']:8.1f} GB/s in  {rec['hbm_algorithmic_gbs']:8.1f} GB/s HBM "
        f"({100 * rec['hbm_frac_of_peak']:.1f} %)")
    results.append(rec)

    deq_items = B.make_dequant_batch([(o["params"], o["out"], y) for o, y in zip(ops, ys)])
    ms = timed(lambda: B.mor_dequantize_batch(deq_items), steps)
    nbytes = sum((3.0 + 1.0 * o["fallback_frac"]) * o["n"] for o in ops)      # FP8 blocks: 1 + 2; BF16 blocks: 2 + 2
    rec = {"name": "dequantize_cfg5", "ms": round(ms, 4), "input_gbs": round(2.0 * n_total / ms / 1e6, 1),
           "hbm_algorithmic_gbs": round(nbytes / ms / 1e6, 1), "hbm_frac_of_peak": round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 4)}
    log(f"[bench]   variant {rec['name']:34s} {ms:8.3f} ms  {rec['input_gbs']:8.1f} GB/s out {rec['hbm_algorithmic_gbs']:8.1f} GB/s HBM "
        f"({100 * rec['hbm_frac_of_peak']:.1f} %)")
    results.append(rec)
    return results


INFINITY_CACHE_BYTES = 256 << 20


def run_configs(B, W, torch, dev, log, target_ms=40.0):
    """One measured row per single-operand configuration of the workload list, each at full size: cfg1 (1024x1024, per
    tensor and 128x128: launch-latency-bound, flagged), cfg2 (activation, 1x128), cfg3 (weight, 128x128 and per tensor),
    cfg4 (gradient, 1x128 and 128x128) and cfg4b (the gradient whose chosen sub-channels are shrunk by half: a mixed
    mask with about 10 % fallback at 1x128).  A call = mor_analyze_quantize_batch with one item including its
    selection statistics.  Calls rotate over `buffer_sets` distinct sets of input / output buffers so that the bytes
    touched between two uses of a set exceed twice the Infinity Cache.  One rotation is captured in a HIP graph and
    replayed (calls of 10-80 us with two or three launches each are otherwise bound by the host's launch calls, which is
    reported beside it as `ms_eager_calls`); the GPU time of all replays is taken with one pair of events."""
    cases = []
    t0 = time.time()
    for name, xb, gran in W.cfg1():
        cases.append(("cfg1", xb, gran))
    for name, xb, gran in W.cfg2():
        cases.append(("cfg2", xb, gran))
    for name, xb, gran in W.cfg3():
        cases.append(("cfg3", xb, gran))
    for name, xb, gran in W.cfg4():
        cases.append(("cfg4", xb, gran))
    cases.append(("cfg4b", W.cfg4(tiny_half=True)[0][1], "sub1x128"))
    log(f"[bench] generated the single-operand configurations in {time.time() - t0:.1f}s")
    ev = B.HipEvents()
    rows_out = []
    dev_cache = {}
    for cfg, xb, gran in cases:
        rows, cols = xb.shape
        n = rows * cols
        params = B.make_params(rows, cols, gran, "partition", "mean_rel_err", THRESHOLD)
        P = B.mor_num_partitions(gran, rows, cols)
        set_bytes = 5 * n + META_BYTES * P                       # input, FP8 payload, BF16 fallback buffer, block outputs
        n_sets = max(2, 2 * INFINITY_CACHE_BYTES // set_bytes + 1)
        key = id(xb)
        if key not in dev_cache:                                 # the same host tensor serves both granularities of a config
            dev_cache.clear()
            x0 = torch.from_numpy(xb.view(np.int16)).to(dev)
            dev_cache[key] = [x0] + [x0.clone() for _ in range(n_sets - 1)]
        xs = dev_cache[key]
        while len(xs) < n_sets:
            xs.append(xs[0].clone())
        sets = []
        for k in range(n_sets):
            out = B.alloc_outputs(params, dev, want_bf16=True)
            out.workspace = None
            st = torch.zeros(B.STATS_BYTES, dtype=torch.uint8, device=dev)
            sets.append((B.make_batch([(params, xs[k], out, st)]), out, st, B.make_batch([(params, xs[k], out, None)])))
        ws = torch.empty(max(16, B.mor_batch_workspace_bytes(sets[0][0])), dtype=torch.uint8, device=dev)
        for entry in sets:                                        # warm-up: one rotation
            B.mor_analyze_quantize_batch(entry[0], 1e-5, ws)
        torch.cuda.synchronize()

        def rotation(reps, which=0):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                for entry in sets:
                    B.mor_analyze_quantize_batch(entry[which], 1e-5, ws)
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / (reps * n_sets)

        def graph_rotation(reps, which=0):
            """The same rotation captured once in a HIP graph and replayed: the launches are then issued by the GPU's command
            processor back to back, as a training loop that captures its step would issue them.  (The library only launches
            kernels: nothing else is recorded into the graph.)"""
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for entry in sets:
                    B.mor_analyze_quantize_batch(entry[which], 1e-5, ws)
            graph.replay()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                graph.replay()
            b.record()
            torch.cuda.synchronize()
            t = a.elapsed_time(b) / (reps * n_sets)
            del graph
            return t

        first = rotation(1)
        reps = max(2, min(2000, int(target_ms / max(first * n_sets, 1e-3))))
        ms_eager = rotation(reps)
        ms = graph_rotation(reps)
        ms_analyze = graph_rotation(reps, 3)                      # the same call without the selection statistics
        # the kernels of one call, bracketed by the library's own events
        prof = ev.new_profile(8)
        kern = {}
        for i in range(9):                                        # the first call after the idle gap is dropped; medians of the rest
            B.mor_analyze_quantize_batch(sets[i % n_sets][0], 1e-5, ws, prof)
            torch.cuda.synchronize()
            for k in range(prof.count):
                kn = B.KERNEL_NAMES[prof.kernel[k]]
                if i > 0:
                    kern.setdefault(kn, []).append(ev.elapsed_ms(prof.start[k], prof.stop[k]) * 1e3)
        kern = {k: round(float(np.median(v)), 2) for k, v in kern.items()}
        s = B.read_stats(sets[0][2])
        f = s["n_elem_bf16"] / float(n)
        fused = bool(s["flags"] & B.MOR_STATS_FLAG_FUSED_FALLBACK)
        if gran == "tensor":
            nbytes = sum(algorithmic_bytes(k, n, 1, f, fused) for k in ("tensor_amax", "tensor_quant", "fallback_copy"))
        else:
            nbytes = algorithmic_bytes("team_block", n, P, f)
        gbs = nbytes / ms / 1e6
        rec = {"config": cfg, "shape": [rows, cols], "granularity": gran, "elements": n, "buffer_sets": n_sets,
               "working_set_mb": round(n_sets * set_bytes / 1e6, 1), "calls_timed": reps * n_sets, "ms": round(ms, 5),
               "input_gbs": round(2.0 * n / ms / 1e6, 1), "algorithmic_bytes": int(nbytes),
               "hbm_algorithmic_gbs": round(gbs, 1), "hbm_frac_of_peak": round(gbs / HBM_PEAK_GBS, 4),
               "timing": "GPU time per call of a rotation over the buffer sets, captured in a HIP graph and replayed",
               "ms_eager_calls": round(ms_eager, 5),       # the same rotation issued call by call from Python: host-bound when above ms
               "ms_without_statistics": round(ms_analyze, 5),
               "hbm_frac_of_peak_without_statistics": round(nbytes / ms_analyze / 1e6 / HBM_PEAK_GBS, 4),
               "fp8_pct_by_elements": round(100.0 * s["n_elem_fp8"] / n, 3),
               "fp8_pct_by_blocks": round(100.0 * s["n_fp8_part"] / s["n_part"], 3),
               "near_threshold_blocks": s["n_near_threshold"], "mean_err": round(s["mean_err"], 6),
               "latency_bound": bool(nbytes / (HBM_PEAK_GBS * 1e9) < 5e-6),     # under 5 us of traffic at peak: launch latency dominates
               "kernels_us": kern}
        log(f"[bench]   config {cfg:6s} {rows}x{cols} {gran:9s} sets={n_sets:3d} {ms * 1e3:9.1f} us/call  {rec['input_gbs']:8.1f} GB/s in  "
            f"{gbs:8.1f} GB/s HBM ({100 * rec['hbm_frac_of_peak']:.1f} %; eager calls {ms_eager * 1e3:.1f} us; without statistics {ms_analyze * 1e3:.1f} us, "
            f"{100 * rec['hbm_frac_of_peak_without_statistics']:.1f} %)  FP8 {rec['fp8_pct_by_elements']:.2f} % of elements  kernels {kern}")
        rows_out.append(rec)
        del sets, ws
        torch.cuda.empty_cache()
    ev.destroy()
    return rows_out


KERNEL_GRAN = {"sub1x128": "sub1x128", "team_block": "block128", "tensor_amax": "tensor", "tensor_quant": "tensor",
               "fallback_copy": "tensor"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--row-div", type=int, default=1, help="divide every operand's rows (debug only; 1 = full workload)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--per-operand", action="store_true", help="one analyze + one stats call per operand instead of one batch call")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="kept for the profiling commands: the three plain 256 MiB device-to-device copies (reference for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE) are always run")
    ap.add_argument("--prewarm-ms", type=float, default=300.0,
                    help="run the step for this much wall time before the warm-up steps (reported as `prewarm`; 0: none)")
    ap.add_argument("--no-configs", action="store_true", help="skip the single-operand rows (cfg1-cfg4, cfg4b)")
    ap.add_argument("--no-variants", action="store_true", help="skip the timing of the further rows (GAM, three-way, partitions, fake quantization)")
    ap.add_argument("--cpu-passes", type=int, default=0, help="oracle passes over the sample (0: repeat until 10 s of oracle time)")
    ap.add_argument("--cpu-sample-div", type=int, default=1, help="oracle is timed on the first rows/N rows of every operand")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU only (no sharding, no collectives); --gpus must be 1.")
        return 2

    import torch
    from paper_2512_22804_amd import binding as B
    from paper_2512_22804_amd import workloads as W

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible; the HIP path has no CPU fallback.")
        return 3
    B.load()
    dev = torch.device("cuda:0")

    t0 = time.time()
    sweep = W.cfg5(row_div=args.row_div)
    log(f"[bench] generated {len(sweep)} operands in {time.time() - t0:.1f}s")

    ops = []
    for name, xb, gran in sweep:
        rows, cols = xb.shape
        params = B.make_params(rows, cols, gran, "partition", "mean_rel_err", THRESHOLD)
        x = torch.from_numpy(xb.view(np.int16)).to(dev)
        out = B.alloc_outputs(params, dev, want_bf16=True)
        stats = torch.zeros(B.STATS_BYTES, dtype=torch.uint8, device=dev)
        ops.append({"name": name, "gran": gran, "params": params, "x": x, "out": out, "stats": stats, "n": rows * cols,
                    "P": B.mor_num_partitions(gran, rows, cols), "host": xb})
    n_total = sum(o["n"] for o in ops)
    items = B.make_batch([(o["params"], o["x"], o["out"], o["stats"]) for o in ops])
    ws_bytes = B.mor_batch_workspace_bytes(items)
    batch_ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()

    def step(profiles=None):
        if not args.per_operand:
            B.mor_analyze_quantize_batch(items, 1e-5, batch_ws, profiles[0] if profiles is not None else None)
            return
        for i, o in enumerate(ops):
            if profiles is None:
                B.mor_analyze_quantize(o["params"], o["x"], o["out"])
            else:
                B.mor_analyze_quantize_profiled(o["params"], o["x"], o["out"], profiles[i])
            B.mor_select_stats(o["params"], o["out"].err_sum, o["out"].nnz, o["out"].mask, 1e-5, o["stats"])

    # reported pre-warm: bring the GPU's clocks / power state to steady state after the idle seconds of data generation
    prewarm_steps = 0
    t_pre = time.perf_counter()
    while args.prewarm_ms > 0 and (time.perf_counter() - t_pre) * 1e3 < args.prewarm_ms:
        for _ in range(10):
            step()
        torch.cuda.synchronize()
        prewarm_steps += 10
    prewarm_ms = (time.perf_counter() - t_pre) * 1e3
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    ms_per_step = elapsed / args.steps * 1e3
    value = 2.0 * n_total / (elapsed / args.steps) / 1e9
    log(f"[bench] pre-warm {prewarm_steps} steps ({prewarm_ms:.0f} ms), warm-up {args.warmup} steps; "
        f"{args.steps} timed steps, {ms_per_step:.4f} ms/step (wall clock, mean), {value:.1f} GB/s of BF16 input")

    # the same steps once more, each bracketed by its own pair of events: per-step GPU times in issue order, median, minimum
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for a, b in evs:
        a.record(); step(); b.record()
    torch.cuda.synchronize()
    in_order = [a.elapsed_time(b) for a, b in evs]
    per_step = sorted(in_order)
    ms_median, ms_min = per_step[len(per_step) // 2], per_step[0]
    ms_event_mean = sum(in_order) / len(in_order)
    log("[bench] per-step GPU time in issue order (ms): " + " ".join(f"{t:.4f}" for t in in_order[:64]) +
        (" ..." if len(in_order) > 64 else ""))
    log(f"[bench] per-step GPU time: mean {ms_event_mean:.4f} ms, median {ms_median:.4f} ms, min {ms_min:.4f} ms")

    # plain device-to-device copy of 256 MiB in the same run: the practical ceiling of a streaming kernel on this machine
    # (with --calibrate-copy these copies also calibrate rocprofv3's FETCH_SIZE / WRITE_SIZE counters)
    src = torch.zeros(256 << 20, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    c0 = torch.cuda.Event(enable_timing=True); c1 = torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(3):
        dst.copy_(src)
    c1.record()
    torch.cuda.synchronize()
    copy_gbs = 2.0 * 3 * (256 << 20) / (c0.elapsed_time(c1) * 1e-3) / 1e9
    log(f"[bench] plain 256 MiB device copy: {copy_gbs:.1f} GB/s (read + write)")
    del src, dst

    # selection result (after the timed region).  The batch call also reports, per operand, whether the quantize pass
    # wrote the fallback itself; in --per-operand mode one untimed batch call supplies that flag.
    if args.per_operand:
        B.mor_analyze_quantize_batch(items, 1e-5, batch_ws, None)
        torch.cuda.synchronize()
    stats = [B.read_stats(o["stats"]) for o in ops]
    fp8_elems = sum(s["n_elem_fp8"] for s in stats)
    fp8_parts = sum(s["n_fp8_part"] for s in stats)
    tot_parts = sum(s["n_part"] for s in stats)
    fp8_tensors = sum(1 for s in stats if s["n_bf16_part"] == 0)
    near = sum(s["n_near_threshold"] for s in stats)
    for o, s in zip(ops, stats):
        o["fallback_frac"] = s["n_elem_bf16"] / float(s["n_elem_fp8"] + s["n_elem_bf16"])
        o["fused_fallback"] = bool(s["flags"] & B.MOR_STATS_FLAG_FUSED_FALLBACK)
        log(f"[bench]   {o['name']:8s} {o['gran']:9s} {o['params'].rows}x{o['params'].cols} mean_err={s['mean_err']:.5f} "
            f"bf16_blocks={s['n_bf16_part']}/{s['n_part']}")

    # per-kernel timing: the same steps again with the library recording HIP events around each kernel
    ev = B.HipEvents()
    profiles = [ev.new_profile(8) for _ in ops]
    per_kernel = {}
    for it in range(args.steps):
        step(profiles)
        torch.cuda.synchronize()
        for o, pr in zip(ops, profiles):
            # a small 1x128 operand rides in extra workgroups of the 128x128 team launch (no launch of its own): its bytes
            # then belong to that launch
            seen = {B.KERNEL_NAMES[pr.kernel[k]] for k in range(pr.count)}
            sub_rides = not args.per_operand and "sub1x128" not in seen and "team_block" in seen
            for k in range(pr.count):
                kname = B.KERNEL_NAMES[pr.kernel[k]]
                ms = ev.elapsed_ms(pr.start[k], pr.stop[k])
                rec = per_kernel.setdefault(kname, {"ms": 0.0, "launches": 0, "bytes": 0.0})
                rec["ms"] += ms
                rec["launches"] += 1
                if args.per_operand:
                    rec["bytes"] += algorithmic_bytes(kname, o["n"], o["P"], o["fallback_frac"], o["fused_fallback"])
                else:      # a grouped launch covers every operand of that granularity
                    for q in ops:
                        if kname.startswith("stats"):
                            rec["bytes"] += algorithmic_bytes(kname, q["n"], q["P"], 0.0) if q["gran"] != "tensor" else 0.0
                        elif KERNEL_GRAN.get(kname) == q["gran"] or (sub_rides and kname == "team_block" and q["gran"] == "sub1x128"):
                            rec["bytes"] += algorithmic_bytes(kname, q["n"], q["P"], q["fallback_frac"], q["fused_fallback"])
            if not args.per_operand:
                break
    ev.destroy()
    for k, r in sorted(per_kernel.items(), key=lambda kv: -kv[1]["ms"]):
        gbs = r["bytes"] / (r["ms"] * 1e-3) / 1e9 if r["ms"] > 0 else 0.0
        log(f"[bench]   kernel {k:16s} launches={r['launches']:4d} avg={r['ms'] / r['launches'] * 1e3:9.1f} us "
            f"alg_bytes/launch={r['bytes'] / r['launches'] / 1e6:9.2f} MB  -> {gbs:7.1f} GB/s")
    dom_name, dom = max(per_kernel.items(), key=lambda kv: kv[1]["ms"])
    achieved = dom["bytes"] / (dom["ms"] * 1e-3) / 1e9
    traffic = None
    traffic_commit = traffic_sha = None
    tree_sha = csrc_sha256()
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath) and args.row_div == 1:
        try:
            tj = json.load(open(tpath))
            traffic = tj.get(dom_name, {}).get("bytes_per_launch")
            traffic_commit = tj.get("_measured_on", {}).get("commit")
            traffic_sha = tj.get("_measured_on", {}).get("csrc_sha256")
        except Exception:
            traffic = None
    if traffic is not None and traffic_sha != tree_sha:
        log(f"[bench] WARNING: profiles/hbm_traffic.json was measured on kernel sources {traffic_sha} (commit {traffic_commit}), "
            f"this tree's are {tree_sha}: roofline.traffic may be stale")
    roofline = {"bound": "hbm", "kernel": dom_name, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "traffic_commit": traffic_commit, "traffic_csrc_sha256": traffic_sha, "tree_csrc_sha256": tree_sha,
                "traffic_matches_tree": bool(traffic is not None and traffic_sha == tree_sha),
                "avg_launch_us": round(dom["ms"] / dom["launches"] * 1e3, 2),
                "algorithmic_bytes_per_launch": round(dom["bytes"] / dom["launches"], 1),
                "per_kernel": {k: {"avg_us": round(r["ms"] / r["launches"] * 1e3, 2),
                                   "gbs": round(r["bytes"] / (r["ms"] * 1e-3) / 1e9, 1) if r["ms"] > 0 else 0.0,
                                   "share_of_gpu_time": round(r["ms"] / sum(x["ms"] for x in per_kernel.values()), 4)}
                               for k, r in per_kernel.items()}}

    # whole-step algorithmic bytes -> achieved HBM GB/s of the step
    step_bytes = 0.0
    for o in ops:
        if o["gran"] == "tensor":
            step_bytes += sum(algorithmic_bytes(k, o["n"], 1, o["fallback_frac"], o["fused_fallback"])
                              for k in ("tensor_amax", "tensor_quant", "fallback_copy"))
        else:
            step_bytes += algorithmic_bytes("team_block" if o["gran"] == "block128" else o["gran"], o["n"], o["P"], o["fallback_frac"])
    step_gbs = step_bytes / (elapsed / args.steps) / 1e9

    configs = None
    if not args.no_configs and not args.per_operand and args.row_div == 1:
        configs = run_configs(B, W, torch, dev, log)

    variants = None
    if not args.no_variants and not args.per_operand:
        variants = run_variants(ops, B, torch, dev, min(args.steps, 10), log)

    cpu_baseline = None
    if not args.no_cpu_baseline:
        from oracle import mor_oracle as O      # the oracle is test infrastructure: timed here as a reported baseline only
        O.build()
        div = max(1, args.cpu_sample_div)
        n_cpu = 0
        t_cpu = 0.0
        passes = 0
        while passes < args.cpu_passes or (args.cpu_passes == 0 and t_cpu < 10.0 and passes < 16):
            for o in ops:
                rows = max(128, (o["host"].shape[0] // div) // 128 * 128)
                xs = np.ascontiguousarray(o["host"][:rows])
                tt = time.perf_counter()
                O.analyze_quantize(xs, o["gran"], "partition", "mean_rel_err", THRESHOLD)
                t_cpu += time.perf_counter() - tt
                n_cpu += xs.size
            passes += 1
        cpu_baseline = {"value": round(2.0 * n_cpu / t_cpu / 1e9, 4), "unit": "GB/s", "cores": O.threads(), "kind": "oracle",
                        "sample": f"{passes} passes over the first 1/{div} of the rows of each of the 12 operands "
                                  f"({n_cpu} elements in all, {t_cpu:.1f} s of oracle time)"}
        # one thread, on the activation operand alone (the first operand of the sweep), for scale
        O.set_threads(1)
        xs = np.ascontiguousarray(ops[0]["host"][:max(128, ops[0]["host"].shape[0] // 4)])
        tt = time.perf_counter()
        O.analyze_quantize(xs, ops[0]["gran"], "partition", "mean_rel_err", THRESHOLD)
        t1 = time.perf_counter() - tt
        O.set_threads(cpu_baseline["cores"])
        cpu_baseline["single_thread_value"] = round(2.0 * xs.size / t1 / 1e9, 4)
        cpu_baseline["single_thread_sample"] = f"first {xs.shape[0]} rows of X ({xs.size} elements, {t1:.1f} s)"
        log(f"[bench] cpu oracle: {cpu_baseline}")

    result = {
        "metric": "GB/s of BF16 input analysed+quantized (fraction of HBM peak); FP8-selected %",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "ms_per_step_median": round(ms_median, 4), "ms_per_step_min": round(ms_min, 4),
        "ms_per_step_event_mean": round(ms_event_mean, 4),
        "prewarm": {"steps": prewarm_steps, "ms": round(prewarm_ms, 1),
                    "why": "steady clocks: after the idle seconds of data generation the first ~5 steps run fast, the next ~20 "
                           "5-10 % slower, then the step time settles; the warm-up and timed steps follow this pre-warm unchanged"},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "cfg5: operand sweep of one Llama-style 8B layer (X 8192x4096 1x128; W_qkv 6144x4096, W_o 4096x4096, "
                               "W_gate/W_up 14336x4096, W_down 4096x14336 128x128; six same-shape gradients per-tensor); "
                               "Eq.2 th=4.5%; " + ("analyze_quantize + select_stats per operand" if args.per_operand else
                                                 "one analyze_quantize_batch call incl. statistics") + ", one stream",
                   "elements_per_step": n_total, "row_div": args.row_div, "criterion": "mean_rel_err", "threshold": THRESHOLD},
        "hbm_algorithmic_gbs": round(step_gbs, 1), "hbm_frac_of_peak": round(step_gbs / HBM_PEAK_GBS, 4),
        "plain_copy_gbs": round(copy_gbs, 1),
        "fp8_selected_pct": {"by_elements": round(100.0 * fp8_elems / n_total, 3), "by_blocks": round(100.0 * fp8_parts / tot_parts, 3),
                             "by_tensors": round(100.0 * fp8_tensors / len(ops), 3), "near_threshold_blocks": near},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "configs": configs,
        "further_rows": variants,
    }
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
