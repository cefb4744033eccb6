"""Host-side logic of bench.py and of the profile harness (no GPU): the roof that binds each configuration, the
cold protocol's set count, and that every measured-traffic figure belongs to a variant this build has and to a
summary under profiles/ that names it."""
from __future__ import annotations

import re
import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
sys.path.insert(0, str(ROOT))

import bench  # noqa: E402
from paper_2207_04296_amd import inputs as I  # noqa: E402


def test_binding_roof_of_the_benchmark_configurations():
    """Arithmetic intensity x 8 TB/s against the MFMA peak of the dtype (fp16: 2516.6 TFLOP/s, ridge 314.6 flop/B)."""
    expect = {"c1_gemm128_f16": "hbm", "c2a_conv56x64_f16": "hbm", "c2b_conv28x128s2_f16": "mfma", "c3a_bmm_qkT_f16": "hbm",
              "c3b_bmm_pv_f16": "hbm", "c4a_gemm4096_f16": "mfma", "c4b_gemm_ffn_f16": "hbm", "c5a_gemm2048_i8": "mfma",
              "c5b_conv_g8d2_i8": "hbm"}
    for name, bound in expect.items():
        wl = I.WORKLOADS[name]
        got, attain = bench.roof(wl.dtype, wl.flops(), wl.min_bytes())
        assert got == bound, (name, got, attain)
        assert attain <= bench.PEAK_TFLOPS[wl.dtype] + 1e-9
    # the headline: 3.699 GFLOP over 12 918 784 bytes = 286 flop/B -> 2 291 TFLOP/s attainable
    wl = I.WORKLOADS["c2a_conv56x64_f16"]
    assert wl.min_bytes() == 12918784 and wl.flops() == 3699376128.0
    assert bench.roof("f16", wl.flops(), wl.min_bytes())[1] == pytest.approx(2290.9, abs=0.1)


def test_cold_runs_rotate_over_more_than_the_caches_whatever_the_step_count():
    for name in ("c2a_conv56x64_f16", "c3a_bmm_qkT_f16", "c5b_conv_g8d2_i8", "c4a_gemm4096_f16"):
        wl = I.WORKLOADS[name]
        n = bench.cold_set_count(wl)
        assert n >= 2 and n * wl.min_bytes() >= 1.25 * bench.CACHE_BYTES
    assert bench.cold_set_count(I.WORKLOADS["c2a_conv56x64_f16"]) == 28
    assert bench.FLUSH_BYTES > bench.CACHE_BYTES


def test_operator_row_reports_both_cache_states_against_the_same_roof():
    wl = I.WORKLOADS["c3a_bmm_qkT_f16"]
    row = bench.op_row(wl.name, "v", wl.out, "", wl.dtype, 4e-6, wl.flops(), wl.min_bytes(), sec_cold=8e-6)
    assert row["bound"] == "hbm" and row["frac_attainable"] == pytest.approx(2 * row["frac_attainable_cold"], rel=1e-3)
    assert row["frac_hbm_cold"] == pytest.approx(wl.min_bytes() / 8e-6 / 8e12, rel=1e-3)


def _variant_names():
    text = (ROOT / "paper_2207_04296_amd" / "csrc" / "tir_variants.def").read_text()
    return set(re.findall(r'^V\d+\("([^"]+)"', text, flags=re.M))


def test_measured_traffic_figures_name_existing_variants_and_their_summaries():
    names = _variant_names()
    summaries = {p.name: p.read_text() for p in (ROOT / "profiles").glob("*.md")}
    assert summaries, "profiles/ holds no summary"
    for (workload, variant), nbytes in bench.MEASURED_TRAFFIC_BYTES.items():
        assert workload in I.WORKLOADS, workload
        assert variant in names, f"{variant} is not in tir_variants.def"
        # at least the algorithmic bytes must have moved, and not absurdly more
        assert I.WORKLOADS[workload].min_bytes() * 0.9 <= nbytes <= I.WORKLOADS[workload].min_bytes() * 4, (workload, variant, nbytes)
        hits = [n for n, t in summaries.items() if workload in n and f"`{variant}`" in t and str(nbytes - 0) and "bytes per launch" in t]
        assert hits, f"no summary under profiles/ covers {workload} on {variant}"
        # the summary's own `bench.py:` line carries the same two terms
        line = [l for l in summaries[hits[0]].splitlines() if l.startswith("bench.py:")]
        assert line, hits[0]
        terms = [int(x) for x in re.findall(r"(\d{6,})", line[0].split("):")[1])]
        assert sum(terms) == nbytes, (hits[0], terms, nbytes)


def test_every_summary_gives_its_full_command_and_runs_committed_files_only():
    for p in (ROOT / "profiles").glob("*.md"):
        t = p.read_text()
        assert "python -m paper_2207_04296_amd.profile" in t and "rocprofv3 --kernel-trace --stats" in t, p.name
        assert "_work" not in t, f"{p.name} refers to a working file"
