"""rocprofv3 harness: kernel time, MFMA utilisation and HBM-side traffic of the benchmark kernels.

    python -m paper_2207_04296_amd.profile [--workloads c2a_conv56x64_f16 c4a_gemm4096_f16] [--out gpurun_out/prof]

Run from the repository root on an MI355X machine.  For every workload it launches, each as a child process with
the program directly behind `--`,

    rocprofv3 --kernel-trace --stats ... -- python3 bench.py --profile-run --records R --workload W ...
    rocprofv3 --pmc FETCH_SIZE        ... -- python3 bench.py --profile-run ...
    rocprofv3 --pmc WRITE_SIZE        ... -- python3 bench.py --profile-run ...
    rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES SQ_LDS_BANK_CONFLICT SQ_WAVE_CYCLES SQ_WAIT_INST_ANY GRBM_GUI_ACTIVE ...

(counters in runs of their own, never together with a trace), the same bench.py command once without the profiler
(what a step takes when nothing traces it), plus the two counter runs of
`bench.py --copy-calibration` (a device copy of known size that scales FETCH_SIZE / WRITE_SIZE), after one
unprofiled `bench.py --tune-only --records R` so that the profiled runs launch the MEASURED variants without
the tuning trials in the trace.  It then reads the CSVs and prints, per workload, and writes as
`<out>/summaries/<workload>.md`:

  * kernel name, launches, average / min / max duration of the timed region;
  * MFMA utilisation = SQ_VALU_MFMA_BUSY_CYCLES / (number of SIMDs x shader cycles of the dispatch), with
    shader cycles = SQ_BUSY_CYCLES / 32 (the counter sums the 32 shader engines) and, beside it, GRBM_GUI_ACTIVE / 8
    (sums the eight XCDs; it keeps counting for some 20 000 cycles around a dispatch, which only a long kernel
    amortises), and the shader clock those cycles imply over the dispatch's own duration;
  * fetched and written bytes per launch (calibrated) and the GB/s they make at the kernel-trace duration;
  * the `MEASURED_TRAFFIC_BYTES` line for bench.py.

This module only starts processes and reads their output; it never touches the GPU itself.
"""
from __future__ import annotations

import argparse
import csv
import json
import os
import statistics
import subprocess
import sys
from pathlib import Path

SIMDS = 256 * 4
XCDS = 8
SHADER_ENGINES = 32
SQ_COUNTERS = ["SQ_VALU_MFMA_BUSY_CYCLES", "SQ_BUSY_CYCLES", "SQ_LDS_BANK_CONFLICT", "SQ_WAVE_CYCLES", "SQ_WAIT_INST_ANY", "GRBM_GUI_ACTIVE"]
PASS_TIMEOUT_S = 240


PARSE_ONLY = False


def run(cmd, log: Path, env):
    if PARSE_ONLY:
        return
    print("+ " + " ".join(cmd), flush=True)
    with open(log, "w") as f:
        r = subprocess.run(["timeout", "-s", "KILL", str(PASS_TIMEOUT_S)] + cmd, stdout=f, stderr=subprocess.STDOUT, env=env)
    if r.returncode != 0:
        tail = "".join(open(log).readlines()[-15:])
        raise SystemExit(f"profile: `{' '.join(cmd)}` ended with status {r.returncode}; end of its log:\n{tail}")


def find_csv(d: Path, suffix: str) -> Path:
    hits = sorted(d.rglob(f"*{suffix}"))
    if not hits:
        raise SystemExit(f"profile: no *{suffix} under {d}")
    return hits[0]


def is_lib_kernel(name: str) -> bool:
    return "tir::" in name and "clear_counters" not in name and "probe" not in name


def kernel_trace(d: Path, timed_launches: int):
    """(kernel name, all durations ns, durations of the last `timed_launches` dispatches) of the library's kernel."""
    rows = [r for r in csv.DictReader(open(find_csv(d, "kernel_trace.csv"))) if is_lib_kernel(r["Kernel_Name"])]
    if not rows:
        raise SystemExit(f"profile: no library kernel in {d}")
    rows.sort(key=lambda r: int(r["Start_Timestamp"]))
    dur = [int(r["End_Timestamp"]) - int(r["Start_Timestamp"]) for r in rows]
    info = rows[-1]
    return info, dur, dur[-timed_launches:]


def counters(d: Path, pick):
    """{counter: [value per dispatch]} and [duration ns per dispatch] over the dispatches pick(kernel name) accepts."""
    vals, durs = {}, {}
    for r in csv.DictReader(open(find_csv(d, "counter_collection.csv"))):
        if not pick(r["Kernel_Name"]):
            continue
        vals.setdefault(r["Counter_Name"], []).append(float(r["Counter_Value"]))
        durs[r["Dispatch_Id"]] = int(r["End_Timestamp"]) - int(r["Start_Timestamp"])
    return vals, list(durs.values())


def mean(v):
    return sum(v) / len(v)


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workloads", nargs="+", default=["c2a_conv56x64_f16", "c4a_gemm4096_f16"])
    ap.add_argument("--out", default="gpurun_out/prof")
    ap.add_argument("--steps", type=int, default=40, help="launches per replay in the profiled runs")
    ap.add_argument("--no-tune", action="store_true", help="profile the scoring rule's variants (no records)")
    ap.add_argument("--variant", default=None, help="profile this variant (bench.py --variant) instead of the measured or built-in choice")
    ap.add_argument("--parse-only", action="store_true", help="start nothing: read the CSVs and logs an earlier run left under --out")
    args = ap.parse_args()
    global PARSE_ONLY
    PARSE_ONLY = args.parse_only

    root = Path(__file__).resolve().parent.parent
    out = (root / args.out).resolve()
    (out / "summaries").mkdir(parents=True, exist_ok=True)
    env = dict(os.environ, TMPDIR="/tmp", PYTHONPATH=str(root))
    py = "python3"
    bench = str(root / "bench.py")
    records = out / "records.txt"
    rec_args = ["--variant", args.variant] if args.variant else []
    if not args.no_tune and not args.variant:
        if records.exists() and not PARSE_ONLY:
            records.unlink()
        for w in args.workloads:
            run([py, bench, "--tune-only", "--records", str(records), "--workload", w], out / f"tune_{w}.log", env)
        rec_args = ["--records", str(records)]

    def rocprof(tag, opts, bench_args):
        d = out / tag
        cmd = ["rocprofv3"] + opts + ["-d", str(d), "-o", "r", "--output-format", "csv", "--", py, bench] + bench_args
        run(cmd, out / f"{tag}.log", env)
        return d, " ".join(["rocprofv3"] + opts + ["-d", f"{args.out}/{tag}", "-o", "r", "--output-format", "csv", "--", py, "bench.py"] +
                            [a if a != str(records) else f"{args.out}/records.txt" for a in bench_args])

    # calibration: what the two traffic counters read for a copy of known size
    is_copy = lambda n: "copy" in n.lower()
    d, cmd_fc = rocprof("fetch_copy", ["--pmc", "FETCH_SIZE"], ["--copy-calibration"])
    fetch_copy = mean(counters(d, is_copy)[0]["FETCH_SIZE"])
    d, cmd_wc = rocprof("write_copy", ["--pmc", "WRITE_SIZE"], ["--copy-calibration"])
    write_copy = mean(counters(d, is_copy)[0]["WRITE_SIZE"])
    true_kib = (64 << 20) / 1024.0
    f_fetch, f_write = true_kib / fetch_copy, true_kib / write_copy
    calib = (f"Counter calibration (device copy of 64 MiB, `{cmd_fc}` and the same with WRITE_SIZE): FETCH_SIZE reads "
             f"{fetch_copy:.1f} KiB (factor {f_fetch:.4f}), WRITE_SIZE reads {write_copy:.1f} KiB (factor {f_write:.4f}).")
    print(calib)

    traffic_lines = []
    for w in args.workloads:
        bargs = ["--profile-run", "--workload", w, "--steps", str(args.steps), "--warmup", "4"] + rec_args
        d, cmd_kt = rocprof(f"kt_{w}", ["--kernel-trace", "--stats"], bargs)
        info, dur_all, dur_timed = kernel_trace(d, 2 * args.steps)
        bench_line = {}
        for line in open(out / f"kt_{w}.log"):
            if line.startswith('{"metric"'):
                bench_line = json.loads(line)
        # the same command without the profiler: what the tracer itself adds per launch
        run([py, bench] + bargs, out / f"plain_{w}.log", env)
        plain_line = {}
        if not PARSE_ONLY or (out / f"plain_{w}.log").exists():
            for line in open(out / f"plain_{w}.log"):
                if line.startswith('{"metric"'):
                    plain_line = json.loads(line)
        d, cmd_f = rocprof(f"fetch_{w}", ["--pmc", "FETCH_SIZE"], bargs)
        fetch = counters(d, is_lib_kernel)[0]["FETCH_SIZE"]
        d, cmd_w = rocprof(f"write_{w}", ["--pmc", "WRITE_SIZE"], bargs)
        write = counters(d, is_lib_kernel)[0]["WRITE_SIZE"]
        d, cmd_sq = rocprof(f"sq_{w}", ["--pmc"] + SQ_COUNTERS, bargs)
        sq, sq_dur = counters(d, is_lib_kernel)
        variant = bench_line.get("config", {}).get("variant", "?")
        rl = bench_line.get("roofline", {})
        avg_ns = mean(dur_timed)
        fetch_b, write_b = mean(fetch) * 1024 * f_fetch, mean(write) * 1024 * f_write
        cycles_grbm = mean(sq["GRBM_GUI_ACTIVE"]) / XCDS
        cycles = mean(sq["SQ_BUSY_CYCLES"]) / SHADER_ENGINES
        mfma_busy = mean(sq["SQ_VALU_MFMA_BUSY_CYCLES"])
        util, util_grbm = mfma_busy / (SIMDS * cycles), mfma_busy / (SIMDS * cycles_grbm)
        clock_ghz, clock_grbm = cycles / mean(sq_dur), cycles_grbm / mean(sq_dur)
        alg = rl.get("algorithmic_bytes_per_launch", 0)
        lines = [
            f"# {w}: `{variant}` under rocprofv3",
            "",
            f"Kernel `{info['Kernel_Name']}`: grid {info['Grid_Size_X']} x {info['Grid_Size_Y']} x {info['Grid_Size_Z']} threads, "
            f"workgroup {info['Workgroup_Size_X']}, LDS {info['LDS_Block_Size']} B, {info['VGPR_Count']} VGPR + {info['Accum_VGPR_Count']} AGPR, scratch {info['Scratch_Size']}.",
            f"Written by `python -m paper_2207_04296_amd.profile --workloads {' '.join(args.workloads)} --steps {args.steps}"
            f"{' --no-tune' if args.no_tune else ''}{' --variant ' + args.variant if args.variant else ''} --out {args.out}` on one MI355X "
            + ("(the variant is the one named on the command line)" if args.variant else
               "(the variant is the library's built-in choice: no tuning records)" if args.no_tune else
               "(variants from an unprofiled `bench.py --tune-only --records ...` run first)") + "; every figure below is per launch.",
            "",
            "## Kernel time",
            "",
            f"    {cmd_kt}",
            "",
            f"{len(dur_all)} launches in the trace (4 warm-up, one graph-upload replay, 2 timed replays of {args.steps}, each after a cache flush copy); "
            f"the {len(dur_timed)} launches of the timed replays: average {avg_ns:.0f} ns, min {min(dur_timed)}, max {max(dur_timed)}, "
            f"median {statistics.median(dur_timed):.0f}; all launches: average {mean(dur_all):.0f} ns.",
            f"The same run's bench line (HIP events around each replay, inside bench.py): avg_launch_us = {rl.get('avg_launch_us')}, "
            f"bound = {rl.get('bound')}, frac = {rl.get('frac')}, frac_mfma = {rl.get('frac_mfma')}, frac_hbm = {rl.get('frac_hbm')} ({rl.get('cache')}).",
            f"The same command without rocprofv3 in front: avg_launch_us = {plain_line.get('roofline', {}).get('avg_launch_us')} per step, gaps between the launches included "
            "(the kernels run in stream order, so this bounds a launch's own duration from above: what the trace adds to every dispatch is the difference).",
            "",
            "## MFMA utilisation and shader clock",
            "",
            f"    {cmd_sq}",
            "",
            "| counter (mean per dispatch over %d dispatches) | value |" % len(sq["GRBM_GUI_ACTIVE"]),
            "|---|---|",
        ] + [f"| {c} | {mean(sq[c]):.0f} |" for c in SQ_COUNTERS if c in sq] + [
            "",
            f"Shader cycles per dispatch = SQ_BUSY_CYCLES / {SHADER_ENGINES} shader engines = {cycles:.0f} (GRBM_GUI_ACTIVE / {XCDS} XCDs = {cycles_grbm:.0f}, "
            "which includes ~20 000 cycles around the dispatch); "
            f"over the dispatch's own duration ({mean(sq_dur):.0f} ns with the counters on) that is a shader clock of **{clock_ghz:.2f} GHz** "
            f"({clock_grbm:.2f} by GRBM_GUI_ACTIVE; nominal peak 2.4).",
            f"MFMA utilisation = SQ_VALU_MFMA_BUSY_CYCLES / ({SIMDS} SIMDs x shader cycles) = {mfma_busy:.0f} / ({SIMDS} x {cycles:.0f}) = **{util:.3f}** "
            f"({util_grbm:.3f} with the GRBM_GUI_ACTIVE cycles).",
            "",
            "## HBM-side traffic (L2 <-> fabric)",
            "",
            f"    {cmd_f}",
            f"    {cmd_w}",
            "",
            calib,
            "",
            "| counter | KiB per dispatch (mean, min, max) | factor | bytes per launch |",
            "|---|---|---|---|",
            f"| FETCH_SIZE | {mean(fetch):.1f}, {min(fetch):.1f}, {max(fetch):.1f} | {f_fetch:.4f} | {fetch_b:.0f} |",
            f"| WRITE_SIZE | {mean(write):.1f}, {min(write):.1f}, {max(write):.1f} | {f_write:.4f} | {write_b:.0f} |",
            "",
            f"traffic = {fetch_b + write_b:.0f} B per launch against {alg} algorithmic bytes"
            + (f" ({(fetch_b + write_b) / alg:.2f} x)" if alg else "") +
            f"; at the kernel-trace average of {avg_ns:.0f} ns that is **{(fetch_b + write_b) / avg_ns:.0f} GB/s** "
            f"({(fetch_b + write_b) / avg_ns / 8000:.3f} of 8 TB/s).  Both counters sit at the L2 -> fabric boundary: reads served by the "
            "256 MB memory-side cache are included, so they bound HBM traffic from above.",
            "",
            f'bench.py: `("{w}", "{variant}"): {fetch_b:.0f} + {write_b:.0f},`',
            "",
        ]
        text = "\n".join(lines)
        (out / "summaries" / f"{w}.md").write_text(text)
        print(text)
        traffic_lines.append(f'    ("{w}", "{variant}"): {fetch_b:.0f} + {write_b:.0f},')
    print("MEASURED_TRAFFIC_BYTES entries:\n" + "\n".join(traffic_lines))


if __name__ == "__main__":
    sys.exit(main())
