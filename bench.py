#!/usr/bin/env python3
"""Benchmark of the tensor-contraction hot path on one MI355X.

    python bench.py --gpus 1 --steps K --warmup W [--replays R] [--workload NAME] [--hot] [--no-operators]

A step is one call of the C ABI for the headline workload (default: the fp16 NHWC conv2d
16x56x56x64 -> 64, 3x3, stride 1, pad 1 with fp16 output), i.e. one pass of the whole path:
fused-iterator decode, tile decomposition, global->LDS copy stage, MFMA accumulation, fused
epilogue store.  Before the timed region the variants are measured once (tir_tune_*, the paper's
search reduced to a table; --no-tune keeps the built-in scoring rule, --records FILE loads kept
records instead of measuring and writes them after measuring).  Operands are resident in device
memory before the timed region.

Timing protocol.  The K steps are captured in one HIP graph (the kernels are microseconds long, a
Python launch loop measures the host as soon as a call takes it longer than the kernel lasts); the headline
workload is also timed as a plain loop over K calls, and the faster of the two ways is the one reported.  The timed region is one replay of that graph, bracketed
by device synchronisations and holding nothing else; it is repeated R times (default 31) and the MEDIAN replay is reported
(minimum and maximum beside it), so the line does not hang on one sample of a fraction of a
millisecond.  Cold mode (default): the K steps walk over enough distinct operand / output sets to
exceed the 256 MB memory-side cache plus the L2s - the number of sets does not depend on K - and
before every timed replay a 2 x 320 MB device copy (untimed) pushes whatever the previous replay
left out of the caches, so every step reads its inputs from HBM whatever K is.  --hot reuses one
set and skips the flush.  Outputs are written with the library's default (cached) policy; the same
run with streaming output stores is reported beside it.

Prints ONE JSON line.  `value` = algorithmic TFLOP/s of the median replay by the host clock
(2*M*N*K of the fused GEMM view per step).  `roofline` prices the headline kernel against the roof
that binds it (min of the MFMA peak and arithmetic intensity x 8 TB/s) with HIP-event times of
replays taken in turn with the host-clock ones (an event record is device work of its own and stays out of the
host-clock region); `roofline_gemm` is the same record for the 4096^3 fp16 GEMM; `cpu_baseline` times
the CPU oracle on the same workload on this machine's host cores; `operators` lists every other
benchmark configuration, plain and with a fused consumer, hot cache, and cold as well where the
roofline that binds them is HBM.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

PEAK_TFLOPS = {"f16": 2516.6, "bf16": 2516.6, "i8": 5033.2}   # 256 CU x 2.4 GHz x 4096 (8192) flop/clk/CU
HBM_GBS = 8000.0
CACHE_BYTES = 256e6 + 8 * 4e6     # memory-side cache + the eight L2s
FLUSH_BYTES = 320 << 20           # source and destination of the flush copy, each larger than the caches

# HBM-side bytes per launch from rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), each scaled by what the same counter
# reads for a device copy of known size; produced by `python -m paper_2207_04296_amd.profile`, which prints the line
# to paste here and writes the summary under profiles/.  Keyed by (workload, variant): a figure measured on another
# variant than the one timed is not reported.
MEASURED_TRAFFIC_BYTES = {
    ("c2a_conv56x64_f16", "f16_f16_patch256x64_conv"): 7251628 + 6422528,
    ("c4a_gemm4096_f16", "f16_f32_t256x128w4x2s3c4_ak_bn"): 268541908 + 67108864,
    ("c4a_gemm4096_f16", "f16_f32_t256x256w2x4s4r64_ak_bn"): 201499478 + 67108864,
    ("c4a_gemm4096_f16", "f16_f32_t256x256w2x4s3r64_ak_bn"): 201508049 + 67108864,
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--replays", type=int, default=31, help="timed replays of the K-step graph; the median is reported")
    ap.add_argument("--workload", default=None, help="headline workload (default c2a_conv56x64_f16); with --tune-only: tune just this one")
    ap.add_argument("--hot", action="store_true", help="reuse one operand set (cache-resident inputs), no flush")
    ap.add_argument("--no-operators", action="store_true", help="skip the per-operator context table")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-tune", action="store_true",
                    help="use the built-in scoring rule instead of measuring the variants first (tir_tune_*)")
    ap.add_argument("--records", default=None,
                    help="file of kept tuning records: loaded instead of measuring if it exists, written after measuring otherwise")
    ap.add_argument("--tune-only", action="store_true", help="measure the variants of every bench workload, write --records, exit")
    ap.add_argument("--profile-run", action="store_true",
                    help="only the headline timed region (for rocprofv3): no tuning trials (use --records), hot rerun, "
                         "operator table, probe or oracle; 2 replays (one by the host clock, one between events)")
    ap.add_argument("--variant", default=None,
                    help="launch this kernel variant (a name or part of one, as tir_debug_force_variant takes it) instead of the chosen one; "
                         "for profiles of a variant the measurement does not pick on the box at hand")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="instead of the workload, run 8 device-to-device copies of 64 MiB (a plain copy kernel of "
                         "known size, to scale the FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


class Harness:
    """Device plumbing shared by every measurement: one stream, its split-reduction workspace, the flush buffers."""

    def __init__(self, torch, B):
        self.torch, self.B = torch, B
        self.stream = torch.cuda.Stream()
        # reductions are split over workgroups only on a stream with a registered workspace (tir_set_workspace)
        self.ws = torch.empty(B.tir_workspace_bytes(), dtype=torch.uint8, device="cuda:0")
        B.tir_set_workspace(self.ws, stream=self.stream)
        self.flush_src = torch.ones(FLUSH_BYTES, dtype=torch.uint8, device="cuda:0")
        self.flush_dst = torch.empty_like(self.flush_src)
        torch.cuda.synchronize()

    def flush(self):
        """Push everything out of the L2s and the memory-side cache (enqueued on the harness stream)."""
        self.flush_dst.copy_(self.flush_src)

    def timed(self, launch, steps, warmup, replays, cold, eager=False):
        """launch(i, stream) enqueues step i.  Returns (wall seconds per replay, HIP-event seconds per replay), lists
        of `replays` samples each, taken in turn; one replay = `steps` launches, from one HIP graph or (eager) from a
        loop over the steps' calls."""
        torch = self.torch
        with torch.cuda.stream(self.stream):
            for i in range(warmup):
                launch(i, self.stream)
            torch.cuda.synchronize()
            graph = None
            if eager:
                def replay():
                    for i in range(steps):
                        launch(i, self.stream)
            else:
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=self.stream):
                    for i in range(steps):
                        launch(i, self.stream)
                replay = graph.replay
            replay()                  # untimed: the first replay uploads the graph
            torch.cuda.synchronize()
            walls, events = [], []
            for _ in range(replays):
                # one replay under the host clock with nothing else in the timed region ...
                if cold:
                    self.flush()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                replay()
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                walls.append(t1 - t0)
                # ... and one between HIP events on the launch stream (their records are device work of their own)
                if cold:
                    self.flush()
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                e0.record(self.stream)
                replay()
                e1.record(self.stream)
                torch.cuda.synchronize()
                events.append(e0.elapsed_time(e1) * 1e-3)
            del replay, graph
        return walls, events


def make_sets(B, wl, count):
    a_bits, b_bits = wl.operands()
    bias = B.bias_to_device(wl)          # a few hundred bytes: shared by every set
    sets = []
    for _ in range(count):
        sets.append((B.to_device(a_bits, wl.dtype), B.to_device(b_bits, wl.dtype),
                     B.empty_out(B.out_shape(wl), wl.out), bias))
    return sets


def cold_set_count(wl):
    """Distinct operand sets a cold run rotates over: 1.25 x the caches, whatever the step count."""
    return max(2, int(CACHE_BYTES * 1.25 / wl.min_bytes()) + 1)


def time_workload(H, wl, sets, steps, warmup, replays, cold, streaming=False, eager=False):
    n = len(sets)
    # (arguments marshalled once per operand set: an eager loop then spends its time per step in the library and the HIP runtime)
    calls = [H.B.prepare_workload(wl, *s, stream=H.stream, streaming=streaming) for s in sets]
    return H.timed(lambda i, st: calls[i % n](), steps, warmup, replays, cold, eager)


def stats(samples, scale=1.0):
    return {"median": round(statistics.median(samples) * scale, 6), "min": round(min(samples) * scale, 6),
            "max": round(max(samples) * scale, 6)}


def variant_of(B, wl):
    # (the variant query takes the output dtype; int8 output selects the requantising kernels)
    if wl.kind == "conv2d":
        return B.tir_conv2d_variant(wl.n, wl.h, wl.w, wl.c, wl.k, wl.r, wl.s, *wl.stride, *wl.pad, *wl.dil,
                                    wl.groups, wl.dtype, wl.out)
    b_rs, b_cs = (1, wl.K) if wl.trans_b else (wl.N, 1)
    return B.tir_gemm_variant(wl.batch, wl.M, wl.N, wl.K, wl.K, 1, b_rs, b_cs, wl.N, 1, wl.dtype, wl.out)


def roof(dtype, flops, nbytes):
    """The roof that binds: ("mfma" | "hbm", attainable TFLOP/s = min(peak, arithmetic intensity x 8 TB/s))."""
    peak = PEAK_TFLOPS[dtype]
    by_hbm = flops / nbytes * HBM_GBS / 1e3
    return ("hbm", by_hbm) if by_hbm < peak else ("mfma", peak)


def roofline_record(B, wl, event_s_per_launch, cache_note):
    """Roofline object of one kernel: achieved / peak in the unit of the roof that binds it, both fractions beside."""
    med = statistics.median(event_s_per_launch)
    flops, nbytes = wl.flops(), wl.min_bytes()
    bound, attain = roof(wl.dtype, flops, nbytes)
    tf = flops / med / 1e12
    gbs = nbytes / med / 1e9
    variant = variant_of(B, wl)
    traffic = MEASURED_TRAFFIC_BYTES.get((wl.name, variant))
    rec = {"bound": bound}
    if bound == "hbm":
        rec.update({"achieved": round(gbs, 1), "peak": HBM_GBS, "unit": "GB/s", "frac": round(gbs / HBM_GBS, 4)})
    else:
        rec.update({"achieved": round(tf, 3), "peak": PEAK_TFLOPS[wl.dtype], "unit": "TFLOP/s", "frac": round(tf / PEAK_TFLOPS[wl.dtype], 4)})
    rec.update({"traffic": traffic,
                "traffic_source": None if traffic is None else "profiles/ (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, copy-calibrated), same variant",
                "frac_mfma": round(tf / PEAK_TFLOPS[wl.dtype], 4), "frac_hbm": round(gbs / HBM_GBS, 4),
                "achieved_tflops": round(tf, 3), "achieved_gbs": round(gbs, 1),
                "attainable_tflops": round(attain, 1), "frac_attainable": round(tf / attain, 4),
                "kernel": variant, "workload": wl.name, "cache": cache_note,
                "avg_launch_us": round(med * 1e6, 3), "launch_us": stats(event_s_per_launch, 1e6),
                "algorithmic_flop_per_launch": flops, "algorithmic_bytes_per_launch": nbytes})
    return rec


def mfma_ceiling(torch, B):
    """Sustained rate of a register-only fp16 MFMA loop (TFLOP/s): the practical ceiling of the matrix
    pipes under the power management, for constant and for random operands."""
    sink = torch.zeros(8, dtype=torch.int32, device="cuda:0")
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
        w = [int(v) & 0xffffffff for v in sink.tolist()]      # one wave's view of the last run: counters before and after its loop
        cycles, ns = (w[3] - w[1]) & 0xffffffff, ((w[4] - w[2]) & 0xffffffff) * 10.0
        if ns > 0 and cycles > 0:
            out[label + "_shader_ghz"] = round(cycles / ns, 3)
            out[label + "_mfma_busy_share"] = round(2000 * 16 * 32 / cycles, 3)      # 16 MFMAs of 32 cycles per iteration
    return out


def op_row(name, variant, out, fused, dtype, sec, flops, nbytes, sec_cold=None):
    tf = flops / sec / 1e12
    bound, attain = roof(dtype, flops, nbytes)
    row = {"workload": name, "variant": variant, "out": out, "fused": fused, "us": round(sec * 1e6, 3), "tflops": round(tf, 2),
           "frac_mfma_peak": round(tf / PEAK_TFLOPS[dtype], 4), "bound": bound, "frac_attainable": round(tf / attain, 4),
           "gbs": round(nbytes / sec / 1e9, 1), "cache": "hot"}
    if sec_cold is not None:
        row.update({"us_cold": round(sec_cold * 1e6, 3), "gbs_cold": round(nbytes / sec_cold / 1e9, 1),
                    "frac_hbm_cold": round(nbytes / sec_cold / 1e9 / HBM_GBS, 4),
                    "frac_attainable_cold": round(flops / sec_cold / 1e12 / attain, 4)})
    return row


def attention_row(H, I):
    """The two attention matmuls of configs[2] (QK^T, then PV) as ONE kernel with the softmax between them:
    192 heads of 128 x 128 x 64, fp16 in and out.  FLOPs count both matmuls; bytes Q, K, V and O once."""
    B = H.B
    batch, M, N, d = 192, 128, 128, 64
    nbytes = 2.0 * batch * (M * d + 2 * N * d + M * d)

    def make():
        return (B.to_device(I.make_tensor("f16", "u", 3000, (batch, M, d)), "f16"), B.to_device(I.make_tensor("f16", "u", 3001, (batch, N, d)), "f16"),
                B.to_device(I.make_tensor("f16", "u", 3101, (batch, N, d)), "f16"), B.empty_out((batch, M, d), "f16"))
    sets = [make() for _ in range(max(2, int(CACHE_BYTES * 1.25 / nbytes) + 1))]
    _, ev_cold = H.timed(lambda i, st: B.tir_attention(*sets[i % len(sets)], batch, M, N, d, 0.125, "f16", "f16", stream=st), 40, 5, 7, True)
    _, ev = H.timed(lambda i, st: B.tir_attention(*sets[0], batch, M, N, d, 0.125, "f16", "f16", stream=st), 200, 5, 5, False)
    return op_row("c3_attention_f16 (QK^T, softmax, PV in one kernel)", "attention_kernel<f16,f16,64>", "f16", "softmax", "f16",
                  statistics.median(ev) / 200, 2.0 * batch * M * N * d * 2, nbytes, statistics.median(ev_cold) / 40)


def other_conv_rows(H, I, tune=True):
    """1-D, 3-D and transposed 2-D convolution (the rest of the paper's operator set), fp16, synthetic shapes."""
    B = H.B
    rows = []
    dev = lambda shape, seed: B.to_device(I.make_tensor("f16", "n0.1", seed, shape), "f16")
    hot = lambda fn: statistics.median(H.timed(lambda i, st: fn(st), 100, 5, 5, False)[1]) / 100
    # conv1d: 16 x 4096 x 128 -> 128, 9 taps
    N, L, C, K, R = 16, 4096, 128, 128, 9
    x, w, y = dev((N, L, C), 7000), dev((K, R, C), 7001), B.empty_out((N, L, K), "f16")
    if tune:      # a 1-D convolution is planned as the 2-D one on an image of height 1: same record
        B.tir_tune_conv2d(x, w, y, N, 1, L, C, K, 1, R, 1, 1, 0, 4, 1, 1, 1, "f16", "f16", reps=10, stream=H.stream)
    sec = hot(lambda st: B.tir_conv1d(x, w, y, N, L, C, K, R, 1, 4, 1, 1, "f16", "f16", stream=st))
    rows.append(op_row("c1d_16x4096x128_k9_f16", B.tir_conv2d_variant(N, 1, L, C, K, 1, R, 1, 1, 0, 4, 1, 1, 1, "f16", "f16"), "f16", "", "f16", sec,
                       2.0 * N * L * K * R * C, 2.0 * (N * L * C + K * R * C + N * L * K)))
    # conv3d: 1 x 10 x 16 x 16 x 128 -> 64, 3x3x3
    N, D, Hh, W, C, K = 1, 10, 16, 16, 128, 64
    x, w, y = dev((N, D, Hh, W, C), 7010), dev((K, 3, 3, 3, C), 7011), B.empty_out((N, D, Hh, W, K), "f16")
    if tune:
        B.tir_tune_conv3d(x, w, y, N, D, Hh, W, C, K, 3, 3, 3, (1, 1, 1), (1, 1, 1), (1, 1, 1), 1, "f16", "f16", reps=10, stream=H.stream)
    sec = hot(lambda st: B.tir_conv3d(x, w, y, N, D, Hh, W, C, K, 3, 3, 3, (1, 1, 1), (1, 1, 1), (1, 1, 1), 1, "f16", "f16", stream=st))
    rows.append(op_row("c3d_10x16x16x128_k3_f16", B.tir_conv3d_variant(N, D, Hh, W, C, K, 3, 3, 3, (1, 1, 1), (1, 1, 1), (1, 1, 1), 1, "f16", "f16"), "f16", "",
                       "f16", sec, 2.0 * N * D * Hh * W * K * 27 * C, 2.0 * (N * D * Hh * W * (C + K) + K * 27 * C)))
    # transposed conv2d: 16 x 28 x 28 x 64 -> 56 x 56 x 64, 4x4, stride 2 (FLOPs of the taps that exist, not of the gather's zeros)
    N, Hh, W, C, K = 16, 28, 28, 64, 64
    x, w, y = dev((N, Hh, W, C), 7020), dev((K, 4, 4, C), 7021), B.empty_out((N, 56, 56, K), "f16")
    if tune:
        B.tir_tune_conv2d_transpose(x, w, y, N, Hh, W, C, K, 4, 4, (2, 2), (1, 1), (1, 1), (0, 0), 1, "f16", "f16", reps=10, stream=H.stream)
    sec = hot(lambda st: B.tir_conv2d_transpose(x, w, y, N, Hh, W, C, K, 4, 4, (2, 2), (1, 1), (1, 1), (0, 0), 1, "f16", "f16", stream=st))
    rows.append(op_row("t2d_28x28x64_k4s2_f16", B.tir_conv2d_transpose_variant(N, Hh, W, C, K, 4, 4, (2, 2), (1, 1), (1, 1), (0, 0), 1, "f16", "f16"), "f16", "",
                       "f16", sec, 2.0 * N * Hh * W * K * 16 * C, 2.0 * (N * Hh * W * C + K * 16 * C + N * 56 * 56 * K)))
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


def all_bench_workloads(I):
    return list(I.WORKLOADS.items()) + list(I.FUSED_WORKLOADS.items()) + list(I.MORE_WORKLOADS.items())


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
    H = Harness(torch, B)
    have_records = bool(args.records) and os.path.exists(args.records)
    if have_records:
        B.tir_tune_load(args.records)
    measure = not args.no_tune and not have_records and not args.profile_run and not args.variant     # run tir_tune_* before timing
    selection = ("forced (--variant)" if args.variant else "kept records (tir_tune_load)" if have_records else
                 "measured (tir_tune_*, untimed, before the run)" if measure else "scoring rule")
    if args.variant:
        B.tir_debug_force_variant(args.variant)
        args.no_operators = True          # the other workloads have other variants

    if args.tune_only:
        for name, o in all_bench_workloads(I):
            if args.workload and name != args.workload:
                continue
            s = make_sets(B, o, 1)
            B.tune_workload(o, *s[0], reps=5 if o.flops() > 4e10 else 10, stream=H.stream)
            del s
        if not args.workload:
            other_conv_rows(H, I, tune=True)
        if args.records:
            B.tir_tune_save(args.records)
        print(json.dumps({"tuned": B.tir_tune_count(), "records": args.records}))
        return

    wl = I.WORKLOADS[args.workload or "c2a_conv56x64_f16"]
    steps, warmup = max(1, args.steps), max(0, args.warmup)
    replays = 1 if args.profile_run else max(1, args.replays)      # (each is two replays of the graph: one by the host clock, one between events)
    cold = not args.hot
    nsets = cold_set_count(wl) if cold else 1
    sets = make_sets(B, wl, nsets)
    if measure:               # untimed: measure the variants once, like a deployment that keeps its records
        B.tune_workload(wl, *sets[0], reps=10, stream=H.stream)

    # headline: the library's default output policy (cached).  The K steps are launched from one HIP graph and, in a run of
    # their own, by a plain loop over K calls; the line reports the faster way (a graph launch has a fixed cost of
    # 10 - 25 us on the device, which a short replay of microsecond kernels feels; a loop is bound by the host as soon as
    # a call takes it longer than the kernel lasts) and gives the other beside it.
    walls, events = time_workload(H, wl, sets, steps, warmup, replays, cold)
    launch_mode, other_value = "hip_graph", None
    if not args.profile_run:
        walls_e, events_e = time_workload(H, wl, sets, steps, warmup, replays, cold, eager=True)
        g_val, e_val = (wl.flops() * steps / statistics.median(x) / 1e12 for x in (walls, walls_e))
        if e_val > g_val:
            walls, events, launch_mode, other_value = walls_e, events_e, "eager", g_val
        else:
            other_value = e_val
    wall = statistics.median(walls)
    ms_per_step = wall * 1e3 / steps
    value = wl.flops() * steps / wall / 1e12
    peak = PEAK_TFLOPS[wl.dtype]
    cache_note = (f"cold (each replay walks {min(steps, nsets)} of {nsets} rotating operand sets = {nsets * wl.min_bytes() / 1e6:.0f} MB, "
                  f"2 x {FLUSH_BYTES >> 20} MiB flush copy before every timed replay)") if cold else "hot (one operand set)"
    roofline = roofline_record(B, wl, [e / steps for e in events], cache_note)

    streaming_value = hot_value = None
    if not args.profile_run:
        if cold:
            w3, _ = time_workload(H, wl, sets, steps, warmup, replays, True, streaming=True, eager=launch_mode == "eager")
            streaming_value = wl.flops() * steps / statistics.median(w3) / 1e12
            w2, _ = time_workload(H, wl, sets[:1], steps, warmup, replays, False)
            hot_value = wl.flops() * steps / statistics.median(w2) / 1e12
    del sets

    roofline_gemm = None
    if not args.profile_run and not args.no_operators and wl.name != "c4a_gemm4096_f16":
        g = I.WORKLOADS["c4a_gemm4096_f16"]
        gsets = make_sets(B, g, cold_set_count(g))
        if measure:
            B.tune_workload(g, *gsets[0], reps=5, stream=H.stream)
        _, gev = time_workload(H, g, gsets, 12, 4, 9, True)
        roofline_gemm = roofline_record(B, g, [e / 12 for e in gev],
                                        f"cold ({len(gsets)} rotating operand sets, flush copy before every timed replay of 12 launches)")
        del gsets

    operators = []
    if not args.no_operators and not args.profile_run:
        for name, o in all_bench_workloads(I):
            big = o.flops() > 4e10
            k = 20 if big else 200
            s = make_sets(B, o, 1)
            if measure:
                B.tune_workload(o, *s[0], reps=5 if big else 10, stream=H.stream)
            _, e_ = time_workload(H, o, s, k, 5, 5, False)
            sec_cold = None
            if roof(o.dtype, o.flops(), o.min_bytes())[0] == "hbm":
                # the roofline that binds this row is HBM bandwidth: only a cold run says anything about it
                cs = s + make_sets(B, o, cold_set_count(o) - 1)
                _, ec = time_workload(H, o, cs, 40, 5, 7, True)
                sec_cold = statistics.median(ec) / 40
                del cs
            operators.append(op_row(name, variant_of(B, o), o.out,
                                    ("bias " if o.ep_bias else "") + ("relu " if o.ep_relu else "") + ("requant" if o.ep_scale else ""),
                                    o.dtype, statistics.median(e_) / k, o.flops(), o.min_bytes(), sec_cold))
            del s
        operators.append(attention_row(H, I))
        operators.extend(other_conv_rows(H, I, tune=measure))
    if measure and args.records:
        B.tir_tune_save(args.records)

    out = {
        "metric": "TFLOP/s and % of MI355X MFMA peak per operator (fp16 GEMM, conv2d)",
        "value": round(value, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": {"f16": "f16", "bf16": "bf16", "i8": "i8"}[wl.dtype],
        "data": "synthetic (seeded; ResNet-50- / BERT-base-shaped operator instances)",
        "config": {"workload": wl.name, "kind": wl.kind, "gemm_view_bMNK": list(wl.gemm_view()),
                   "out_dtype": wl.out, "variant": variant_of(B, wl),
                   "launch": launch_mode + (" (K calls in a loop; faster here than one HIP graph of the K steps)" if launch_mode == "eager" else
                                            " (one graph of the K steps; faster here than K calls in a loop)" if other_value is not None else ""),
                   "selection": selection, "cache": cache_note,
                   "output_stores": "cached (library default)"},
        "timing": {"replays": replays, "reported": "median replay by the host clock; ms_per_step x steps = one replay; event-timed replays alternate with the host-clock ones",
                   "wall_ms_per_replay": stats(walls, 1e3), "event_ms_per_replay": stats(events, 1e3)},
        "frac_mfma_peak": round(value / peak, 4),
        "value_device_clock": round(wl.flops() * steps / statistics.median(events) / 1e12, 3),
        "value_other_launch_mode": None if other_value is None else {"launch": "hip_graph" if launch_mode == "eager" else "eager", "value": round(other_value, 3)},
        "value_hot_cache": None if hot_value is None else round(hot_value, 3),
        "value_cold_streaming_outputs": None if streaming_value is None else round(streaming_value, 3),
        "roofline": roofline,
        "roofline_gemm": roofline_gemm,
        "operators": operators,
        "mfma_sustained_tflops": None if args.profile_run else mfma_ceiling(torch, B),
    }
    if not args.no_cpu_baseline and not args.profile_run:
        out["cpu_baseline"] = cpu_baseline(wl)
    torch.cuda.synchronize()
    B.tir_set_workspace(None, stream=H.stream)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
