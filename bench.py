#!/usr/bin/env python3
"""Benchmark of the tensor-contraction hot path on one MI355X.

    python bench.py --gpus 1 --steps K --warmup W [--workload NAME] [--hot] [--eager] [--no-operators]

A step is one call of the C ABI for the headline workload (default: the fp16 NHWC conv2d
16x56x56x64 -> 64, 3x3, stride 1, pad 1 with fp16 output), i.e. one pass of the whole path:
fused-iterator decode, tile decomposition, global->LDS copy stage, MFMA accumulation, fused
epilogue store.  Before the timed region the variants are measured once (tir_tune_*, the paper's
search reduced to a table; --no-tune keeps the built-in scoring rule).  Operands are resident in
device memory before the timed region.  By default the
K steps rotate over enough distinct operand / output sets to exceed the 256 MB memory-side cache
plus L2, so every step reads its inputs from HBM ("cold"); --hot reuses one set.  The K launches
are captured in one HIP graph (the kernels are microseconds long, a Python launch loop would
measure the host), replayed once inside the timed region; --eager launches them one by one.

Prints ONE JSON line.  `value` = algorithmic TFLOP/s of the whole run (2*M*N*K of the fused GEMM
view per step).  `roofline` prices the kernel against the dense fp16 MFMA peak; `cpu_baseline`
times the CPU oracle on the same workload on this machine's host cores; `operators` lists every other
benchmark configuration, plain and with a fused consumer (bias / ReLU / down-cast / int8
requantisation), hot cache, for context.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

PEAK_TFLOPS = {"f16": 2516.6, "bf16": 2516.6, "i8": 5033.2}   # 256 CU x 2.4 GHz x 4096 (8192) flop/clk/CU
HBM_GBS = 8000.0
CACHE_BYTES = 256e6 + 8 * 4e6     # memory-side cache + the eight L2s

# HBM bytes per launch of the headline kernel from rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), scaled
# by the same counters on a copy kernel of known size; see profiles/.  None until measured.
MEASURED_TRAFFIC_BYTES = {
    "c2a_conv56x64_f16": 7192720 + 6422528,      # FETCH_SIZE 3513.3 KiB x 1.9993, WRITE_SIZE 6272 KiB x 1.0
    "c4a_gemm4096_f16": 201415700 + 67108864,    # FETCH_SIZE 98382 KiB x 1.9993, WRITE_SIZE 65536 KiB x 1.0
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=480)
    ap.add_argument("--warmup", type=int, default=48)
    ap.add_argument("--workload", default="c2a_conv56x64_f16")
    ap.add_argument("--hot", action="store_true", help="reuse one operand set (cache-resident inputs)")
    ap.add_argument("--eager", action="store_true", help="launch step by step instead of one HIP graph")
    ap.add_argument("--no-operators", action="store_true", help="skip the per-operator context table")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-tune", action="store_true",
                    help="use the built-in scoring rule instead of measuring the variants first (tir_tune_*)")
    ap.add_argument("--profile-run", action="store_true",
                    help="only the headline timed region (for rocprofv3): no tuning trials, hot rerun, operator table, probe or oracle")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="instead of the workload, run 8 device-to-device copies of 64 MiB (a plain copy kernel of "
                         "known size, to scale the FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def make_sets(B, wl, count):
    a_bits, b_bits = wl.operands()
    bias = B.bias_to_device(wl)          # a few hundred bytes: shared by every set
    sets = []
    for _ in range(count):
        sets.append((B.to_device(a_bits, wl.dtype), B.to_device(b_bits, wl.dtype),
                     B.empty_out(B.out_shape(wl), wl.out), bias))
    return sets


def timed_run(torch, B, wl, sets, steps, warmup, eager, streaming=False):
    """Returns (wall seconds for `steps` launches, HIP-event seconds for the same region)."""
    stream = torch.cuda.Stream()
    n = len(sets)
    with torch.cuda.stream(stream):
        for i in range(warmup):
            B.run_workload(wl, *sets[i % n], stream=stream, streaming=streaming)
        torch.cuda.synchronize()
        graph = None
        if not eager:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for i in range(steps):
                    B.run_workload(wl, *sets[i % n], stream=stream, streaming=streaming)
            graph.replay()            # untimed: first replay uploads the graph
            torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record(stream)
        if graph is not None:
            graph.replay()
        else:
            for i in range(steps):
                B.run_workload(wl, *sets[i % n], stream=stream, streaming=streaming)
        e1.record(stream)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        return t1 - t0, e0.elapsed_time(e1) * 1e-3


def variant_of(B, wl):
    # (the variant query takes the output dtype; int8 output selects the requantising kernels)
    if wl.kind == "conv2d":
        return B.tir_conv2d_variant(wl.n, wl.h, wl.w, wl.c, wl.k, wl.r, wl.s, *wl.stride, *wl.pad, *wl.dil,
                                    wl.groups, wl.dtype, wl.out)
    b_rs, b_cs = (1, wl.K) if wl.trans_b else (wl.N, 1)
    return B.tir_gemm_variant(wl.batch, wl.M, wl.N, wl.K, wl.K, 1, b_rs, b_cs, wl.N, 1, wl.dtype, wl.out)


def mfma_ceiling(torch, B):
    """Sustained rate of a register-only fp16 MFMA loop (TFLOP/s): the practical ceiling of the matrix
    pipes under the power management, for constant and for random operands."""
    sink = torch.zeros(4, device="cuda:0")
    out = {}
    for label, rnd in (("const_operands", False), ("random_operands", True)):
        B.tir_probe_mfma_rate(sink, 200, rnd)
        torch.cuda.synchronize()
        best = 0.0
        for _ in range(3):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            flop = B.tir_probe_mfma_rate(sink, 2000, rnd)
            e1.record()
            torch.cuda.synchronize()
            best = max(best, flop / (e0.elapsed_time(e1) * 1e-3) / 1e12)
        out[label] = round(best, 1)
    return out


def attention_row(torch, B, I):
    """The two attention matmuls of configs[2] (QK^T, then PV) as ONE kernel with the softmax between them:
    192 heads of 128 x 128 x 64, fp16 in and out.  FLOPs count both matmuls; bytes Q, K, V and O once."""
    batch, M, N, d = 192, 128, 128, 64
    q = B.to_device(I.make_tensor("f16", "u", 3000, (batch, M, d)), "f16")
    k = B.to_device(I.make_tensor("f16", "u", 3001, (batch, N, d)), "f16")
    v = B.to_device(I.make_tensor("f16", "u", 3101, (batch, N, d)), "f16")
    o = B.empty_out((batch, M, d), "f16")
    stream = torch.cuda.Stream()
    steps = 200
    with torch.cuda.stream(stream):
        for _ in range(5):
            B.tir_attention(q, k, v, o, batch, M, N, d, 0.125, "f16", "f16", stream=stream)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for _ in range(steps):
                B.tir_attention(q, k, v, o, batch, M, N, d, 0.125, "f16", "f16", stream=stream)
        graph.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        graph.replay()
        e1.record(stream)
        torch.cuda.synchronize()
    sec = e0.elapsed_time(e1) * 1e-3 / steps
    flops = 2.0 * batch * M * N * d * 2
    nbytes = 2.0 * batch * (M * d + 2 * N * d + M * d)
    tf = flops / sec / 1e12
    return {"workload": "c3_attention_f16 (QK^T, softmax, PV in one kernel)", "variant": "attention_kernel<f16,f16,64>",
            "out": "f16", "fused": "softmax", "us": round(sec * 1e6, 3), "tflops": round(tf, 2),
            "frac_mfma_peak": round(tf / PEAK_TFLOPS["f16"], 4),
            "frac_attainable": round(tf / min(PEAK_TFLOPS["f16"], flops / nbytes * HBM_GBS / 1e3), 4),
            "gbs": round(nbytes / sec / 1e9, 1), "cache": "hot"}


def _graph_time(torch, fn, steps=100):
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for _ in range(5):
            fn(stream)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for _ in range(steps):
                fn(stream)
        graph.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        graph.replay()
        e1.record(stream)
        torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / steps


def other_conv_rows(torch, B, I, tune=True):
    """1-D, 3-D and transposed 2-D convolution (the rest of the paper's operator set), fp16, synthetic shapes."""
    rows = []

    def row(name, variant, sec, flops, nbytes):
        tf = flops / sec / 1e12
        rows.append({"workload": name, "variant": variant, "out": "f16", "fused": "",
                     "us": round(sec * 1e6, 3), "tflops": round(tf, 2), "frac_mfma_peak": round(tf / PEAK_TFLOPS["f16"], 4),
                     "frac_attainable": round(tf / min(PEAK_TFLOPS["f16"], flops / nbytes * HBM_GBS / 1e3), 4),
                     "gbs": round(nbytes / sec / 1e9, 1), "cache": "hot"})
    dev = lambda shape, seed: B.to_device(I.make_tensor("f16", "n0.1", seed, shape), "f16")
    # conv1d: 16 x 4096 x 128 -> 128, 9 taps
    N, L, C, K, R = 16, 4096, 128, 128, 9
    x, w, y = dev((N, L, C), 7000), dev((K, R, C), 7001), B.empty_out((N, L, K), "f16")
    if tune:      # a 1-D convolution is planned as the 2-D one on an image of height 1: same record
        B.tir_tune_conv2d(x, w, y, N, 1, L, C, K, 1, R, 1, 1, 0, 4, 1, 1, 1, "f16", "f16", reps=10)
    sec = _graph_time(torch, lambda st: B.tir_conv1d(x, w, y, N, L, C, K, R, 1, 4, 1, 1, "f16", "f16", stream=st))
    row("c1d_16x4096x128_k9_f16", B.tir_conv2d_variant(N, 1, L, C, K, 1, R, 1, 1, 0, 4, 1, 1, 1, "f16", "f16"), sec, 2.0 * N * L * K * R * C, 2.0 * (N * L * C + K * R * C + N * L * K))
    # conv3d: 1 x 10 x 16 x 16 x 128 -> 64, 3x3x3
    N, D, H, W, C, K = 1, 10, 16, 16, 128, 64
    x, w, y = dev((N, D, H, W, C), 7010), dev((K, 3, 3, 3, C), 7011), B.empty_out((N, D, H, W, K), "f16")
    if tune:
        B.tir_tune_conv3d(x, w, y, N, D, H, W, C, K, 3, 3, 3, (1, 1, 1), (1, 1, 1), (1, 1, 1), 1, "f16", "f16", reps=10)
    sec = _graph_time(torch, lambda st: B.tir_conv3d(x, w, y, N, D, H, W, C, K, 3, 3, 3, (1, 1, 1), (1, 1, 1), (1, 1, 1), 1, "f16", "f16", stream=st))
    row("c3d_10x16x16x128_k3_f16", B.tir_conv3d_variant(N, D, H, W, C, K, 3, 3, 3, (1, 1, 1), (1, 1, 1), (1, 1, 1), 1, "f16", "f16"), sec, 2.0 * N * D * H * W * K * 27 * C, 2.0 * (N * D * H * W * (C + K) + K * 27 * C))
    # transposed conv2d: 16 x 28 x 28 x 64 -> 56 x 56 x 64, 4x4, stride 2 (FLOPs of the taps that exist, not of the gather's zeros)
    N, H, W, C, K = 16, 28, 28, 64, 64
    x, w, y = dev((N, H, W, C), 7020), dev((K, 4, 4, C), 7021), B.empty_out((N, 56, 56, K), "f16")
    if tune:
        B.tir_tune_conv2d_transpose(x, w, y, N, H, W, C, K, 4, 4, (2, 2), (1, 1), (1, 1), (0, 0), 1, "f16", "f16", reps=10)
    sec = _graph_time(torch, lambda st: B.tir_conv2d_transpose(x, w, y, N, H, W, C, K, 4, 4, (2, 2), (1, 1), (1, 1), (0, 0), 1, "f16", "f16", stream=st))
    row("t2d_28x28x64_k4s2_f16", B.tir_conv2d_transpose_variant(N, H, W, C, K, 4, 4, (2, 2), (1, 1), (1, 1), (0, 0), 1, "f16", "f16"), sec, 2.0 * N * H * W * K * 16 * C, 2.0 * (N * H * W * C + K * 16 * C + N * 56 * 56 * K))
    return rows


def cpu_baseline(wl):
    """The oracle, as it stands, on this machine's host cores; whole workload, repeated for ~seconds."""
    import oracle
    from tests.parity import run_oracle
    a_bits, b_bits = wl.operands()
    sample_note = "whole workload"
    if wl.flops() > 4e10:     # 4096^3: 256 whole output rows are the bounded sample
        import dataclasses
        wl = dataclasses.replace(wl, M=256)
        a_bits = a_bits[:256].copy()
        sample_note = "256 of 4096 output rows"
    run_oracle(wl, a_bits, b_bits, oracle)     # warm (page in, build)
    reps, t = 0, 0.0
    while t < 3.0 and reps < 20:
        t0 = time.perf_counter()
        run_oracle(wl, a_bits, b_bits, oracle)
        t += time.perf_counter() - t0
        reps += 1
    return {"value": wl.flops() * reps / t / 1e12, "unit": "TFLOP/s", "cores": oracle.get_threads(),
            "kind": "oracle", "sample": f"{sample_note}, {reps} repetitions, fp64 direct loops incl. sum|a*b|"}


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (every output tile is independent: rows, batches and "
              "convolution groups would be sharded over GPUs without communication). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    import torch
    from paper_2207_04296_amd import binding as B
    from paper_2207_04296_amd import inputs as I

    if not torch.cuda.is_available():
        print("bench.py: no ROCm device visible", file=sys.stderr)
        sys.exit(2)
    B.lib()     # fails loudly if libtir.so was not built
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.ones(64 << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(8):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read_per_dispatch": 64 << 20, "bytes_written_per_dispatch": 64 << 20,
                                               "dispatches": 8}}))
        return
    if args.profile_run:
        args.no_operators = args.no_cpu_baseline = args.no_tune = True
    wl = I.WORKLOADS[args.workload]

    per_set = wl.min_bytes()
    nsets = 1 if args.hot else max(2, int(CACHE_BYTES * 1.25 / per_set) + 1)
    nsets = min(nsets, max(1, args.steps))
    sets = make_sets(B, wl, nsets)
    if not args.no_tune:      # untimed: measure the variants once, like a deployment that keeps its records
        B.tune_workload(wl, *sets[0], reps=10)
    # Cold run: inputs come from HBM and nothing reads an output again before 27 other launches have gone by, which
    # is what TIR_OUTPUT_STREAMING is for (see tir.h); the same run with cached outputs is reported next to it, and
    # the hot run and the operator table use the library's default (outputs stay cached for a consumer).
    streaming = not args.hot
    cold_cached_value = None
    wall, ev = timed_run(torch, B, wl, sets, args.steps, args.warmup, args.eager, streaming=streaming)
    if streaming and not args.profile_run:
        w3, _ = timed_run(torch, B, wl, sets, args.steps, args.warmup, args.eager)
        cold_cached_value = wl.flops() * args.steps / w3 / 1e12
    ms_per_step = wall * 1e3 / args.steps
    value = wl.flops() * args.steps / wall / 1e12
    peak = PEAK_TFLOPS[wl.dtype]
    launch_s = ev / args.steps
    achieved = wl.flops() / launch_s / 1e12
    traffic = MEASURED_TRAFFIC_BYTES.get(wl.name)

    hot_value = None
    if not args.hot and not args.profile_run:
        w2, _ = timed_run(torch, B, wl, sets[:1], args.steps, args.warmup, args.eager)
        hot_value = wl.flops() * args.steps / w2 / 1e12
    del sets

    operators = []
    if not args.no_operators:
        for name, o in list(I.WORKLOADS.items()) + list(I.FUSED_WORKLOADS.items()) + list(I.MORE_WORKLOADS.items()):
            k = 20 if o.flops() > 4e10 else 200
            s = make_sets(B, o, 1)
            if not args.no_tune:
                B.tune_workload(o, *s[0], reps=5 if o.flops() > 4e10 else 10)
            w_, e_ = timed_run(torch, B, o, s, k, 5, args.eager)
            tf = o.flops() * k / e_ / 1e12
            attain = min(PEAK_TFLOPS[o.dtype], o.flops() / o.min_bytes() * HBM_GBS / 1e3)
            operators.append({"workload": name, "variant": variant_of(B, o), "out": o.out,
                              "fused": ("bias " if o.ep_bias else "") + ("relu " if o.ep_relu else "") + ("requant" if o.ep_scale else ""),
                              "us": round(e_ / k * 1e6, 3),
                              "tflops": round(tf, 2), "frac_mfma_peak": round(tf / PEAK_TFLOPS[o.dtype], 4),
                              "frac_attainable": round(tf / attain, 4),
                              "gbs": round(o.min_bytes() * k / e_ / 1e9, 1), "cache": "hot"})
            del s
        operators.append(attention_row(torch, B, I))
        operators.extend(other_conv_rows(torch, B, I, tune=not args.no_tune))

    out = {
        "metric": "TFLOP/s and % of MI355X MFMA peak per operator (fp16 GEMM, conv2d)",
        "value": round(value, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": {"f16": "f16", "bf16": "bf16", "i8": "i8"}[wl.dtype],
        "data": "synthetic (seeded; ResNet-50- / BERT-base-shaped operator instances)",
        "config": {"workload": wl.name, "kind": wl.kind, "gemm_view_bMNK": list(wl.gemm_view()),
                   "out_dtype": wl.out, "variant": variant_of(B, wl),
                   "launch": "hip_graph" if not args.eager else "eager",
                   "selection": "scoring rule" if args.no_tune else "measured (tir_tune_*, untimed, before the run)",
                   "cache": "hot (one operand set)" if args.hot else f"cold (rotating {nsets} operand sets)",
                   "output_stores": "streaming (tir_set_output_policy: no launch reads an output again)" if streaming else "cached (library default)"},
        "frac_mfma_peak": round(value / peak, 4),
        "value_hot_cache": None if hot_value is None else round(hot_value, 3),
        "value_cold_cached_outputs": None if cold_cached_value is None else round(cold_cached_value, 3),
        "roofline": {"bound": "mfma", "achieved": round(achieved, 3), "peak": peak, "unit": "TFLOP/s",
                     "frac": round(achieved / peak, 4), "traffic": traffic,
                     "kernel": variant_of(B, wl), "avg_launch_us": round(launch_s * 1e6, 3),
                     "algorithmic_flop_per_launch": wl.flops(), "algorithmic_bytes_per_launch": wl.min_bytes()},
        "operators": operators,
        "mfma_sustained_tflops": None if args.profile_run else mfma_ceiling(torch, B),
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
