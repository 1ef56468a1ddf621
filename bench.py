#!/usr/bin/env python3
"""Throughput of the linear-angular attention layer on one MI355X.

A step is one whole forward of the layer (reduce + apply: every kernel of the
path) over one batch of synthetic, seeded inputs that are already resident in
HBM.  The bench rotates over several distinct input sets so the loop cannot be
served from the last-level cache.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 4]

Prints one JSON line: tokens/s, the roofline of the dominant kernel (algorithmic
bytes over its HIP-event-timed duration against the 8 TB/s HBM peak) and the CPU
oracle timed on the host cores (a baseline, not the target).
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

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E peak

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (scaled by a copy kernel
# of known size) are read from this committed summary; it names the sources it was measured on.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "forward_pmc_traffic.txt")
KERNEL_SOURCES = ("apply_mfma.hpp", "reduce_mfma.hpp", "fused_small.hpp", "tables.hpp", "formats.hpp",
                  "common.hpp", "apply_generic.hpp", "reduce_generic.hpp")


def kernel_source_digest() -> str:
    """sha256 over the forward kernels' source files (what a traffic figure is valid for)."""
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2211_10526_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic(workload: str):
    """{kernel: bytes per launch} for the workload from the committed PMC summary, and a note.
    Lines: `workload kernel FETCH_SIZE_KiB WRITE_SIZE_KiB fetch_scale write_scale`; a header line
    `sources <sha256>` names the kernel sources the counters were read on.  Figures measured on
    other sources than the ones in the tree are not reported."""
    if not os.path.exists(TRAFFIC_FILE):
        return None, "no committed PMC summary"
    digest, rows = None, {}
    with open(TRAFFIC_FILE) as f:
        for line in f:
            parts = line.split()
            if not parts or parts[0].startswith("#"):
                continue
            if parts[0] == "sources":
                digest = parts[1]
            elif parts[0] == workload and len(parts) >= 6:
                fetch, write, fs, ws = (float(x) for x in parts[2:6])
                rows[parts[1]] = (fetch * fs + write * ws) * 1024.0
    if not rows:
        return None, "workload not in the committed PMC summary"
    if digest != kernel_source_digest():
        return None, "kernel sources changed since the committed PMC summary was measured"
    return rows, None


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="4",
                    help="index (0-4) or name prefix of the benchmark workload; default the "
                         "largest one (bf16, B=2, heads=12, d=64, 128x128 grid, 9x9 DWConv)")
    ap.add_argument("--sets", type=int, default=6, help="distinct input sets to rotate over")
    ap.add_argument("--layout", choices=("dense", "fused"), default="dense",
                    help="dense: q, k, v, out contiguous [B,heads,N,d] (the benchmark configs); "
                         "fused: q, k, v slices of one [B,N,3,heads,d] tensor, out [B,N,heads*d]")
    ap.add_argument("--pairwise", choices=("sparse", "angular"), default=None,
                    help="time castling_attn_pairwise (masked softmax branch of Eq. 10 / exact "
                         "angular-kernel attention) instead of the layer; MFMA roofline")
    ap.add_argument("--downsample", action="store_true",
                    help="the workload as a downsampling layer: queries pooled to every second "
                         "row and column, residual query (dense layout)")
    ap.add_argument("--backward", action="store_true",
                    help="time castling_attn_backward (gradients of q, k, v, filters, bias) "
                         "instead of the forward layer (dense layout)")
    ap.add_argument("--per-call-filters", action="store_true",
                    help="pass the DWConv filters to every forward (their operand table is then "
                         "rebuilt per call) instead of registering them once before timing")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="first run three 256 MiB device-to-device copies: a kernel of known "
                         "traffic that scales the rocprofv3 FETCH_SIZE / WRITE_SIZE counters")
    return ap.parse_args()


def bench_pairwise(args, wl, sets, binding, inputs, torch):
    """K calls of castling_attn_pairwise over the rotating input sets; one JSON line.  The
    roofline is the dense bf16 / fp16 MFMA peak against the algorithmic flops 4 N^2 d per unit
    (one Q K^T and one P V; the kernel itself runs Q K^T twice for the softmax and P V on a
    two-part split of P)."""
    mode = binding.PAIR_SPARSE_SOFTMAX if args.pairwise == "sparse" else binding.PAIR_ANGULAR
    attn = binding.CastlingAttn.for_workload(wl)
    stream = torch.cuda.Stream()
    kept = torch.zeros(wl.units, dtype=torch.int64, device=sets[0]["q"].device)
    kw = dict(normalize=True, scale=8.0, threshold=0.02)

    def call(t):
        attn.pairwise(mode, t["q"], t["k"], t["v"], t["out"], kept=kept, stream=stream, **kw)

    steps = max(1, min(args.steps, int(2e8 // (wl.N * wl.N * wl.units // 1000 + 1)) + 1))
    with torch.cuda.stream(stream):
        for i in range(min(args.warmup, 3)):
            call(sets[i % len(sets)])
        stream.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(stream)
        for i in range(steps):
            call(sets[i % len(sets)])
        e1.record(stream)
        stream.synchronize()
        elapsed = time.perf_counter() - t0
        kernel_ms = e0.elapsed_time(e1) / steps
    flops = 4.0 * wl.units * wl.N * wl.N * wl.d
    achieved = flops / (kernel_ms * 1e-3) / 1e12
    peak = 2500.0  # TFLOP/s, dense bf16 / fp16 MFMA
    attn.destroy()
    print(json.dumps({
        "metric": f"pairwise {args.pairwise} attention tokens/s per layer",
        "value": round(wl.tokens * steps / elapsed, 1), "unit": "tokens/s", "n_gpus": 1,
        "steps": steps, "warmup": min(args.warmup, 3), "ms_per_step": round(elapsed * 1e3 / steps, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype,
        "data": "synthetic",
        "config": {"workload": wl.name, "B": wl.B, "heads": wl.heads, "d": wl.d, "N": wl.N,
                   "op": f"pairwise_{args.pairwise}", **kw,
                   "kept_per_unit": float(kept.float().mean().item())},
        "roofline": {"bound": "mfma", "kernel": "pairwise_attn_kernel", "achieved": round(achieved, 1),
                     "peak": peak, "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                     "traffic": None, "algorithmic_flops": flops, "kernel_ms": round(kernel_ms, 5)},
        "cpu_baseline": None,
    }))


def bench_backward(args, wl, sets, host0, binding, inputs, torch, nq):
    """K calls of castling_attn_backward over the rotating input sets; one JSON line.
    Algorithmic bytes of a backward: q, k, v, grad_out read and the three gradients written once
    (7 tensors; with --downsample q, grad_out and grad_q have a row per pooled query)."""
    dev = sets[0]["q"].device
    if args.downsample:
        attn = binding.CastlingAttn(binding.make_desc(
            wl.B, wl.heads, wl.N, wl.d, wl.grid_h, wl.grid_w, wl.dw_kernel, wl.dtype,
            flags=binding.FLAG_RESIDUAL_Q | binding.FLAG_TRAINING, q_pool=2))
    else:
        attn = binding.CastlingAttn.for_workload(wl, flags=binding.FLAG_TRAINING)
    stream = torch.cuda.Stream()
    for t in sets:
        t["g"] = torch.randn(t["q"].shape, device=dev).to(t["q"].dtype)
    grads = [torch.empty_like(sets[0]["q"]), torch.empty_like(sets[0]["k"]),
             torch.empty_like(sets[0]["k"])]
    gw = torch.empty(sets[0]["w"].shape, dtype=torch.float32, device=dev)
    gb = torch.empty((wl.heads, wl.d), dtype=torch.float32, device=dev)

    def call(t):
        attn.backward(t["q"], t["k"], t["v"], t["w"], t["g"], *grads, gw, gb, stream=stream)

    with torch.cuda.stream(stream):
        for i in range(args.warmup):
            call(sets[i % len(sets)])
        stream.synchronize()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(stream)
        for i in range(args.steps):
            call(sets[i % len(sets)])
        e1.record(stream)
        stream.synchronize()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        event_ms = e0.elapsed_time(e1) / args.steps
    tensor_bytes = wl.elems * wl.itemsize
    nbytes = 4 * tensor_bytes + 3 * (tensor_bytes * nq // wl.N)
    achieved = nbytes / (event_ms * 1e-3) / 1e9
    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        nb = 1
        xs = {n: inputs.to_f64(host0[n][:nb]) for n in ("q", "k", "v")}
        g64 = inputs.to_f64(sets[0]["g"][:nb].cpu())
        w64 = inputs.to_f64(host0["w"])
        if args.downsample:  # (the oracle has the definition only: O(Nq N d) per unit)
            oracle_bwd = lambda: oracle.backward_pooled_explicit(xs["q"], xs["k"], xs["v"], w64, g64,
                                                                 wl.grid_h, wl.grid_w)
        else:
            oracle_bwd = lambda: oracle.backward(xs["q"], xs["k"], xs["v"], w64, g64, wl.grid_h, wl.grid_w)
        c0 = time.perf_counter()
        oracle_bwd()
        first = time.perf_counter() - c0
        reps = max(1, min(200, int(10.0 / max(first, 1e-6))))
        c0 = time.perf_counter()
        for _ in range(reps):
            oracle_bwd()
        c1 = time.perf_counter() - c0
        cpu_baseline = {"value": round(reps * nb * wl.N / c1, 1), "unit": "tokens/s",
                        "cores": oracle.num_threads(), "kind": "oracle",
                        "sample": f"{nb} of {wl.B} batch images of the workload, {reps} passes of "
                                  f"the oracle's backward, fp64, {c1:.2f} s"}
    attn.destroy()
    print(json.dumps({
        "metric": "linear-angular attention backward tokens/s per layer",
        "value": round(wl.tokens * args.steps / elapsed, 1), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(elapsed * 1e3 / args.steps, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype,
        "data": "synthetic",
        "config": {"workload": wl.name, "B": wl.B, "heads": wl.heads, "d": wl.d, "N": wl.N,
                   "grid": [wl.grid_h, wl.grid_w], "dw_kernel": wl.dw_kernel, "op": "backward",
                   "queries_per_unit": nq,
                   "input_sets_rotated": len(sets)},
        "roofline": {"bound": "hbm", "kernel": "backward (all launches)", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": None, "algorithmic_bytes": nbytes, "kernel_ms": round(event_ms, 5)},
        "cpu_baseline": cpu_baseline,
    }))


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the layer's (batch, head) units are "
              "independent and would shard over GPUs without communication). Run with --gpus 1.",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2211_10526_amd import binding, inputs

    wl = inputs.workload(int(args.workload) if args.workload.isdigit() else args.workload)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    nq = -(-wl.grid_h // 2) * -(-wl.grid_w // 2) if args.downsample else wl.N
    if args.downsample and (args.layout != "dense" or args.pairwise):
        sys.exit("bench.py: --downsample goes with the dense layout of the layer")
    # distinct seeded input sets, all resident before timing starts
    sets = []
    for s in range(args.sets):
        x = inputs.make_inputs(wl, seed=wl.seed + s)
        if args.layout == "fused":
            qkv = torch.empty((wl.B, wl.N, 3, wl.heads, wl.d), dtype=x["q"].dtype, device=dev)
            for i, n in enumerate(("q", "k", "v")):
                qkv[:, :, i] = x[n].to(dev).permute(0, 2, 1, 3)
            t = {n: qkv[:, :, i] for i, n in enumerate(("q", "k", "v"))}
            t["w"] = x["w"].to(dev)
            t["out"] = torch.empty((wl.B, wl.N, wl.heads * wl.d), dtype=x["q"].dtype, device=dev)
        else:
            t = {n: x[n].to(dev) for n in ("q", "k", "v", "w")}
            if args.downsample:  # the pooled queries: as many rows of the drawn ones
                x["q"] = x["q"][:, :, :nq].contiguous()
                t["q"] = x["q"].to(dev)
            t["out"] = torch.empty_like(t["q"])
        sets.append(t)
        if s == 0:
            host0 = x
    if args.calibrate_copy:
        cx = torch.empty(128 * 1024 * 1024, dtype=torch.bfloat16, device=dev).normal_()
        cy = torch.empty_like(cx)
        for _ in range(3):
            cy.copy_(cx)
        torch.cuda.synchronize()
        del cx, cy
    if args.pairwise:
        return bench_pairwise(args, wl, sets, binding, inputs, torch)
    if args.backward:
        if args.layout != "dense":
            sys.exit("bench.py: --backward goes with the dense layout")
        return bench_backward(args, wl, sets, host0, binding, inputs, torch, nq)
    if args.layout == "fused":
        attn = binding.CastlingAttn.for_workload(
            wl, in_strides=binding.fused_qkv_strides(wl.heads, wl.N, wl.d),
            out_strides=binding.token_major_strides(wl.heads, wl.N, wl.d))
    elif args.downsample:
        attn = binding.CastlingAttn(binding.make_desc(
            wl.B, wl.heads, wl.N, wl.d, wl.grid_h, wl.grid_w, wl.dw_kernel, wl.dtype,
            flags=binding.FLAG_RESIDUAL_Q, q_pool=2))
    else:
        attn = binding.CastlingAttn.for_workload(wl)
    stream = torch.cuda.Stream()

    # The DWConv filters are constants of the model at inference: they are registered once (their
    # matrix-core operand table is built here, outside the timed region) and every forward uses
    # the registration.  --per-call-filters passes them to each forward instead.
    if not args.per_call_filters:
        attn.prepare_weights(sets[0]["w"], stream=stream)

    def fwd(t):
        attn.forward(t["q"], t["k"], t["v"], t["w"] if args.per_call_filters else None, None,
                     t["out"], stream=stream)

    with torch.cuda.stream(stream):
        for i in range(args.warmup):
            fwd(sets[i % len(sets)])
        stream.synchronize()
        torch.cuda.synchronize()

        # ---- timed region: exactly K whole forwards
        t0 = time.perf_counter()
        for i in range(args.steps):
            fwd(sets[i % len(sets)])
        stream.synchronize()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0

        # ---- per-kernel durations: K back-to-back launches of each half between two HIP
        # events recorded on the launch stream (same rotating inputs; the DWConv filters
        # are registered once so that the timed apply is the apply kernel alone; apply
        # reuses the state of the last reduce, its cost does not depend on the values)
        attn.prepare_weights(sets[0]["w"], stream=stream)
        e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        e[0].record(stream)
        for i in range(args.steps):
            t = sets[i % len(sets)]
            attn.reduce(t["k"], t["v"], stream=stream)
        e[1].record(stream)
        stream.synchronize()
        e[2].record(stream)
        for i in range(args.steps):
            t = sets[i % len(sets)]
            attn.apply(t["q"], t["v"], None, None, t["out"], stream=stream)
        e[3].record(stream)
        stream.synchronize()
        reduce_ms = e[0].elapsed_time(e[1]) / args.steps   # reduce + combine launches
        apply_ms = e[2].elapsed_time(e[3]) / args.steps
        staged_ms = reduce_ms + apply_ms

        # the same K forwards between HIP events (for handles whose forward is one kernel this
        # is that kernel's average duration)
        e[0].record(stream)
        for i in range(args.steps):
            fwd(sets[i % len(sets)])
        e[1].record(stream)
        stream.synchronize()
        forward_ms = e[0].elapsed_time(e[1]) / args.steps

    # a plain device-to-device copy on the same box, after the timed region: the practical
    # ceiling to read the fractions of the published peak against (256 MiB read + 256 MiB written)
    with torch.cuda.stream(stream):
        cx = torch.empty(128 * 1024 * 1024, dtype=torch.bfloat16, device=dev)
        cy = torch.empty_like(cx)
        cy.copy_(cx)
        stream.synchronize()
        e[0].record(stream)
        for _ in range(5):
            cy.copy_(cx)
        e[1].record(stream)
        stream.synchronize()
        copy_gbs = 5 * 2 * cx.numel() * 2 / (e[0].elapsed_time(e[1]) * 1e-3) / 1e9
        del cx, cy

    ms_per_step = elapsed * 1e3 / args.steps
    tokens_per_s = wl.tokens * args.steps / elapsed
    tensor_bytes = wl.elems * wl.itemsize
    q_bytes = tensor_bytes * nq // wl.N  # Q and out have one row per query
    layer_bytes = 2 * tensor_bytes + 2 * q_bytes
    if attn.num_launches() == 1:
        # the whole layer in one kernel: it reads Q, K, V once and writes out (4 tensors)
        kernels = {"fused_forward": (layer_bytes, forward_ms)}
    else:
        # algorithmic bytes: apply reads Q and V and writes out (3 tensors); reduce reads K and V
        kernels = {"apply": (tensor_bytes + 2 * q_bytes, apply_ms),
                   "reduce": (2 * tensor_bytes, reduce_ms)}
    dominant = max(kernels, key=lambda n: kernels[n][1])
    dom_bytes, dom_ms = kernels[dominant]
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9
    # measured HBM bytes per launch (dense layout of the plain layer only)
    traffic, traffic_note = (measured_traffic(wl.name) if args.layout == "dense" and not args.downsample
                             else (None, "no PMC summary for this layout"))
    roofline = {
        "bound": "hbm", "kernel": dominant, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
        "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
        "traffic": traffic.get(dominant) if traffic else None,
        "traffic_per_kernel": traffic, "traffic_forward": sum(traffic.values()) if traffic else None,
        "traffic_note": traffic_note,
        # all measured bytes of one forward over the step time: what the memory system delivers
        "traffic_forward_gbs": (round(sum(traffic.values()) / (ms_per_step * 1e-3) / 1e9, 1)
                                if traffic else None),
        "algorithmic_bytes": dom_bytes, "kernel_ms": round(dom_ms, 5),
        "reduce_ms": round(reduce_ms, 5), "apply_ms": round(apply_ms, 5),
        "staged_step_ms": round(staged_ms, 5),
        "layer_algorithmic_gbs_4tensor": round(layer_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "layer_frac_of_peak_4tensor": round(layer_bytes / (ms_per_step * 1e-3) / 1e9
                                            / HBM_PEAK_GBS, 4),
        "d2d_copy_gbs_same_run": round(copy_gbs, 1),
    }

    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        # bounded sample: as many whole (batch) images of the workload as fit ~10-30 s
        flops_per_unit = wl.N * wl.d * (4.0 * wl.d + 2.0 * wl.dw_kernel ** 2)
        est_s = flops_per_unit * wl.units / (0.4e9 * max(1, oracle.num_threads()))
        nb = max(1, min(wl.B, int(wl.B * 20.0 / max(est_s, 1e-9))))
        xs = {n: inputs.to_f64(host0[n][:nb]) for n in ("q", "k", "v")}
        w64 = inputs.to_f64(host0["w"])
        oracle_fwd = oracle.forward_pooled if args.downsample else oracle.forward
        c0 = time.perf_counter()
        oracle_fwd(xs["q"], xs["k"], xs["v"], w64, None, wl.grid_h, wl.grid_w)
        first = time.perf_counter() - c0
        # repeat whole passes up to about 10 s of CPU work (at most 200 passes)
        reps = max(1, min(200, int(10.0 / max(first, 1e-6))))
        c0 = time.perf_counter()
        for _ in range(reps):
            oracle_fwd(xs["q"], xs["k"], xs["v"], w64, None, wl.grid_h, wl.grid_w)
        c1 = time.perf_counter() - c0
        cpu_baseline = {
            "value": round(reps * nb * wl.N / c1, 1), "unit": "tokens/s",
            "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{nb} of {wl.B} batch images of the workload ({nb * wl.heads} of "
                      f"{wl.units} units), {reps} passes, fp64, {c1:.2f} s",
        }

    n_split = attn.num_splits()
    launches = attn.num_launches()
    attn.destroy()
    line = {
        "metric": "linear-angular attention tokens/s per layer",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype if wl.dtype != "f32" else "f32", "data": "synthetic",
        "config": {"workload": wl.name, "B": wl.B, "heads": wl.heads, "d": wl.d, "N": wl.N,
                   "grid": [wl.grid_h, wl.grid_w], "dw_kernel": wl.dw_kernel,
                   "layout": args.layout, "queries_per_unit": nq,
                   "input_sets_rotated": len(sets), "reduce_splits": n_split,
                   "kernels_per_forward": launches,
                   "filters": "per call" if args.per_call_filters else "registered once"},
        "roofline": roofline, "cpu_baseline": cpu_baseline,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
