"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, rejects bad arguments before touching the device, and maps workgroup ids to
output tiles bijectively."""
import re
from pathlib import Path

import numpy as np
import pytest

from paper_2207_04296_amd import binding as B

ROOT = Path(__file__).resolve().parent.parent


def test_library_exports_every_declared_symbol():
    header = (ROOT / "include" / "tir.h").read_text()
    declared = set(re.findall(r"\b(tir_[a-z0-9_]+)\s*\(", header))
    assert {"tir_gemm", "tir_batch_matmul", "tir_conv2d", "tir_last_error"} <= declared
    L = B.lib()
    for name in sorted(declared):
        assert hasattr(L, name), f"libtir.so does not export {name}"
    assert declared == set(B.EXPORTS)
    assert B.tir_version() == "0.1"


GOOD = dict(M=64, N=64, K=64, a_rs=64, a_cs=1, b_rs=64, b_cs=1, c_rs=64, c_cs=1, in_dtype="f16", out_dtype="f32")
FAKE = 0x1000  # a non-null, 16-byte aligned "pointer"; never dereferenced because validation fails first


def _gemm(**over):
    a = dict(GOOD, **over)
    return B.tir_gemm_status(a.pop("A", FAKE), a.pop("Bp", FAKE), a.pop("C", FAKE), a["M"], a["N"], a["K"], a["a_rs"],
                             a["a_cs"], a["b_rs"], a["b_cs"], a["c_rs"], a["c_cs"], a["in_dtype"], a["out_dtype"])


@pytest.mark.parametrize("over,status", [
    (dict(M=-1), B.TIR_ERR_INVALID_ARG),
    (dict(K=-5), B.TIR_ERR_INVALID_ARG),
    (dict(a_rs=-64), B.TIR_ERR_INVALID_ARG),
    (dict(C=0), B.TIR_ERR_INVALID_ARG),
    (dict(A=0), B.TIR_ERR_INVALID_ARG),
    (dict(c_rs=0, c_cs=0), B.TIR_ERR_INVALID_ARG),
    (dict(in_dtype=7), B.TIR_ERR_INVALID_ARG),
    (dict(in_dtype="f16", out_dtype="i32"), B.TIR_ERR_UNSUPPORTED),
    (dict(in_dtype="i8", out_dtype="f32"), B.TIR_ERR_UNSUPPORTED),
    (dict(in_dtype="f32", out_dtype="f32"), B.TIR_ERR_UNSUPPORTED),
    (dict(in_dtype="bf16", out_dtype="f16"), B.TIR_ERR_UNSUPPORTED),
    (dict(M=2 ** 31), B.TIR_ERR_UNSUPPORTED),
    (dict(A=FAKE + 1), B.TIR_ERR_ALIGNMENT),
    (dict(C=FAKE + 2), B.TIR_ERR_ALIGNMENT),
])
def test_gemm_rejects_bad_arguments(over, status):
    assert _gemm(**over) == status
    assert B.last_error() != ""


def test_zero_sized_calls_are_noops_without_a_device():
    assert _gemm(M=0) == B.TIR_OK
    assert _gemm(N=0, A=0, Bp=0, C=0) == B.TIR_OK
    assert B.tir_batch_matmul_status(FAKE, FAKE, FAKE, 0, 8, 8, 8, 64, 8, 1, 64, 8, 1, 64, 8, 1, "f16", "f32") == B.TIR_OK
    assert B.tir_conv2d_status(FAKE, FAKE, FAKE, 0, 8, 8, 8, 8, 3, 3, 1, 1, 1, 1, 1, 1, 1, "f16", "f16") == B.TIR_OK


def test_bmm_rejects_overlapping_outputs():
    st = B.tir_batch_matmul_status(FAKE, FAKE, FAKE, 4, 8, 8, 8, 64, 8, 1, 64, 8, 1, 0, 8, 1, "f16", "f32")
    assert st == B.TIR_ERR_INVALID_ARG and "overlap" in B.last_error()


def _conv(**over):
    a = dict(N=1, H=8, W=8, C=8, K=8, R=3, S=3, sh=1, sw=1, ph=1, pw=1, dh=1, dw=1, g=1, i="f16", o="f16")
    a.update(over)
    return B.tir_conv2d_status(a.get("x", FAKE), a.get("w", FAKE), a.get("y", FAKE), a["N"], a["H"], a["W"], a["C"], a["K"],
                               a["R"], a["S"], a["sh"], a["sw"], a["ph"], a["pw"], a["dh"], a["dw"], a["g"], a["i"], a["o"])


@pytest.mark.parametrize("over,status", [
    (dict(g=3), B.TIR_ERR_INVALID_ARG),           # groups must divide C and K
    (dict(g=0), B.TIR_ERR_INVALID_ARG),
    (dict(C=8, K=12, g=8), B.TIR_ERR_INVALID_ARG),
    (dict(sh=0), B.TIR_ERR_INVALID_ARG),
    (dict(dw=0), B.TIR_ERR_INVALID_ARG),
    (dict(ph=-1), B.TIR_ERR_INVALID_ARG),
    (dict(H=2, W=2, ph=0, pw=0), B.TIR_ERR_INVALID_ARG),   # 3x3 filter does not fit: P <= 0
    (dict(H=0), B.TIR_ERR_INVALID_ARG),
    (dict(x=0), B.TIR_ERR_INVALID_ARG),
    (dict(H=20000), B.TIR_ERR_UNSUPPORTED),
    (dict(i="i8", o="f16"), B.TIR_ERR_UNSUPPORTED),
])
def test_conv_rejects_bad_arguments(over, status):
    assert _conv(**over) == status
    assert B.last_error() != ""


@pytest.mark.parametrize("tiles", [(1, 1), (16, 16), (7, 5), (3, 100), (49, 1), (2, 4), (13, 24), (196, 1)])
def test_block_to_tile_map_is_a_bijection(tiles):
    # the binding of block iterators to workgroup ids must cover every tile exactly once
    tm, tn = tiles
    seen = {B.tir_debug_tile_of_block(b, tm, tn) for b in range(tm * tn)}
    assert len(seen) == tm * tn
    assert all(0 <= a < tm and 0 <= b < tn for a, b in seen)


def test_division_by_launch_constants_is_exact():
    """The kernels decode output rows with multiply-and-shift constants; exact for every dividend below 2^31."""
    rng = np.random.default_rng(5)
    divisors = [1, 2, 3, 5, 7, 28, 49, 56, 784, 3136, 12544, 65535, 65536, 65537, 2**30 - 1, 2**30, 2**30 + 1, 2**31 - 1]
    divisors += [int(x) for x in rng.integers(1, 2**31, 40)]
    for d in divisors:
        edge = [0, 1, d - 1, d, d + 1, 2 * d - 1, 2 * d, 2**31 - 1, 2**31 - 2, (2**31 - 1) // d * d, (2**31 - 1) // d * d - 1]
        for m in edge + [int(x) for x in rng.integers(0, 2**31, 200)]:
            if 0 <= m < 2**31:
                assert B.tir_debug_fastdiv(d, m) == m // d, (d, m)


def test_variant_choice_reflects_layout():
    # row-major B is read N-major, a transposed B K-major; odd K falls back to the general kernel
    assert B.tir_gemm_variant(1, 4096, 4096, 4096, 4096, 1, 4096, 1, 4096, 1, "f16", "f32").endswith("ak_bn")
    assert B.tir_gemm_variant(1, 4096, 4096, 4096, 4096, 1, 1, 4096, 4096, 1, "f16", "f32").endswith("ak_bk")
    assert B.tir_gemm_variant(1, 100, 100, 37, 37, 1, 100, 1, 100, 1, "f16", "f32").endswith("generic")
    assert "conv" in B.tir_conv2d_variant(16, 56, 56, 64, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1, "f16", "f16")
    assert B.tir_conv2d_variant(1, 8, 8, 3, 8, 3, 3, 1, 1, 1, 1, 1, 1, 1, "f16", "f16").endswith("conv_generic")
    assert B.tir_gemm_variant(1, -1, 8, 8, 8, 1, 8, 1, 8, 1, "f16", "f32") == ""


# ------------------------------------------------------------------------------ measured-choice records
def _gemm_variant_512():
    return B.tir_gemm_variant(1, 512, 512, 512, 512, 1, 512, 1, 512, 1, "f16", "f32")


def test_tuning_records_load_save_and_steer_the_choice(tmp_path):
    """A record file names the variant per problem signature: loading it changes what the planner
    picks for exactly that signature, saving writes it back, clearing restores the scoring rule.
    (Record lines: kind dt out amode bmode batch M N K geom variant; row-major f16 -> f32 GEMM is
    dt 0, out 3, A k-major 0, B n-major 1.)"""
    B.tir_tune_clear()
    try:
        default = _gemm_variant_512()
        other = "f16_f32_t64x32w2x1s4_ak_bn"
        assert default and default != other and other in B.tir_debug_variant_names()
        rec = tmp_path / "records.txt"
        rec.write_text("tir-tune-records 1\n"
                       f"0 0 3 0 1 1 512 512 512 0 {other}\n"
                       "0 0 3 0 1 1 640 512 512 0 no_such_variant\n"              # unknown name: skipped
                       "0 0 3 0 1 1 768 512 512 0 i8_i32_t64x64w2x2s2_ak_bn\n"    # wrong dtype for the key: skipped
                       "0 0 3 0 1 1 896 512 512 0 f16_f32_t64x64w2x2s2_ak_bk\n"   # wrong copy mode for the key: skipped
                       "garbage line\n")
        B.tir_tune_load(rec)
        assert B.tir_tune_count() == 1
        assert _gemm_variant_512() == other
        # another signature (batch 2) is untouched
        B.tir_debug_force_variant("")
        batch2 = B.tir_gemm_variant(2, 512, 512, 512, 512, 1, 512, 1, 512, 1, "f16", "f32")
        assert batch2 and batch2 != other
        # a forced variant wins over a record
        B.tir_debug_force_variant("t128x128w2x2s2_")
        assert "t128x128w2x2s2_" in _gemm_variant_512()
        B.tir_debug_force_variant("")
        # save / clear / load round trip
        out = tmp_path / "saved.txt"
        B.tir_tune_save(out)
        lines = out.read_text().splitlines()
        assert lines[0] == "tir-tune-records 1" and lines[1:] == [f"0 0 3 0 1 1 512 512 512 0 {other} 1"]   # last field: reduction slices
        B.tir_tune_clear()
        assert B.tir_tune_count() == 0 and _gemm_variant_512() == default
        B.tir_tune_load(out)
        assert _gemm_variant_512() == other
    finally:
        B.tir_debug_force_variant("")
        B.tir_tune_clear()


def test_reduction_split_is_planned_only_where_it_fits(tmp_path):
    """A reduction can be split over several workgroups per output tile ("<variant>/z<slices>"): only by the fast
    kernels, only when every slice gets a stage, and the scoring rule asks for it when few tiles face a long K."""
    def gemm(M, N, K, batch=1):
        return B.tir_gemm_variant(batch, M, N, K, K, 1, 1, K, N, 1, "f16", "f32")
    B.tir_tune_clear()
    try:
        assert "/z" not in gemm(4096, 4096, 4096)                     # the tiles fill the CUs: no split
        auto = gemm(128, 128, 16384)
        assert "/z" in auto and 2 <= int(auto.split("/z")[1]) <= 8    # 1-4 tiles, 256 stages
        B.tir_debug_force_ksplit(4)
        assert gemm(128, 128, 16384).endswith("/z4")
        assert gemm(4096, 4096, 4096).endswith("/z4") is False       # workspace: 256 tiles x 4 slices x 256 KiB > 32 MiB
        assert "/z" not in gemm(128, 128, 128)                        # two stages cannot feed four slices
        assert gemm(128, 128, 256).endswith("/z4")                    # four stages can
        assert "/z" not in gemm(100, 100, 4001)                       # odd K: the general kernel does not split
        assert "/z" not in B.tir_conv2d_variant(1, 8, 8, 3, 8, 3, 3, 1, 1, 1, 1, 1, 1, 1, "f16", "f16")
        conv = B.tir_conv2d_variant(2, 14, 14, 256, 64, 3, 3, 1, 1, 1, 1, 1, 1, 1, "f16", "f16")
        assert conv.endswith("/z4") and "patch" not in conv
        B.tir_debug_force_ksplit(0)
        # a record carries the split; one that does not fit its problem is planned without it
        name = "f16_f32_t64x64w2x2s3_ak_bk"
        assert name in B.tir_debug_variant_names()
        rec = tmp_path / "split.txt"
        rec.write_text("tir-tune-records 1\n"
                       f"0 0 3 0 0 1 128 128 16384 0 {name} 6\n"
                       f"0 0 3 0 0 1 128 128 128 0 {name} 6\n"
                       f"0 0 3 0 0 1 128 128 256 0 {name} 99\n")           # out of range: skipped
        B.tir_tune_load(rec)
        assert B.tir_tune_count() == 2
        assert gemm(128, 128, 16384) == name + "/z6"
        assert gemm(128, 128, 128) == name
        out = tmp_path / "saved.txt"
        B.tir_tune_save(out)
        assert f"0 0 3 0 0 1 128 128 16384 0 {name} 6" in out.read_text().splitlines()
    finally:
        B.tir_debug_force_ksplit(0)
        B.tir_tune_clear()


def test_output_policy_is_a_checked_field_of_the_epilogue():
    """The cache policy of a call's output stores travels in its epilogue: 0 or 1, anything else is rejected on the host."""
    def call(streaming):
        ep = B.Epilogue(None, 0, 0.0, streaming)
        return B.lib().tir_gemm_fused(FAKE, FAKE, FAKE, 64, 64, 64, 64, 1, 64, 1, 64, 1, B.TIR_F16, B.TIR_F32, ep, None)
    assert call(7) == B.TIR_ERR_INVALID_ARG and "streaming" in B.last_error()
    assert call(-1) == B.TIR_ERR_INVALID_ARG
    assert B.make_epilogue() is None and B.make_epilogue(streaming=True).streaming == 1
    assert not hasattr(B.lib(), "tir_set_output_policy")       # no process-wide policy


def test_split_static_rejects_what_its_scratch_cannot_hold():
    """tir_gemm_split_static checks slices, the copy mode and the size of its static scratch before any HIP call."""
    def call(M=128, N=128, K=4096, slices=4, a_rs=None, in_dtype="f16", out_dtype="f32"):
        return B.tir_gemm_split_static_status(FAKE, FAKE, FAKE, M, N, K, a_rs or K, 1, 1, K, N, 1, in_dtype, out_dtype, None, slices)
    assert call(slices=1) == B.TIR_ERR_INVALID_ARG and "slices" in B.last_error()
    assert call(slices=65) == B.TIR_ERR_INVALID_ARG
    assert call(K=0) == B.TIR_ERR_INVALID_ARG
    assert call(M=0) == B.TIR_OK                                              # nothing to do
    assert call(K=4001, a_rs=4001) == B.TIR_ERR_UNSUPPORTED and "general kernel" in B.last_error()
    assert call(K=128, slices=4) == B.TIR_ERR_INVALID_ARG and "non-empty slices" in B.last_error()     # two stages, four slices
    # 4096 x 4096 outputs: at least 1024 tiles of 128 x 128 x 4 slices x 64 KiB = 256 MiB of partial sums
    assert call(M=4096, N=4096, K=4096, slices=4) == B.TIR_ERR_INVALID_ARG
    msg = B.last_error()
    assert str(B.TIR_STATIC_SCRATCH_BYTES) in msg and str(B.TIR_STATIC_SCRATCH_TILES) in msg, msg
    assert call(in_dtype="f16", out_dtype="i32") == B.TIR_ERR_UNSUPPORTED
    header = (ROOT / "include" / "tir.h").read_text()
    assert "#define TIR_STATIC_SCRATCH_BYTES (8u << 20)" in header and "#define TIR_STATIC_SCRATCH_TILES 1024" in header
    assert (B.TIR_STATIC_SCRATCH_BYTES, B.TIR_STATIC_SCRATCH_TILES) == (8 << 20, 1024)


def test_caller_workspace_arguments_are_checked():
    """tir_set_workspace rejects a buffer that is too small or not 256-byte aligned before it touches the device."""
    need = B.tir_workspace_bytes()
    assert need == (32 << 20) + 16384 * 4
    assert B.tir_set_workspace_status(FAKE, need - 1) == B.TIR_ERR_INVALID_ARG
    assert "tir_workspace_bytes" in B.last_error()
    assert B.tir_set_workspace_status(FAKE + 16, need) == B.TIR_ERR_ALIGNMENT


def test_tuning_record_files_are_validated(tmp_path):
    bad = tmp_path / "bad.txt"
    bad.write_text("something else\n")
    with pytest.raises(B.TirError) as e:
        B.tir_tune_load(bad)
    assert e.value.status == B.TIR_ERR_INVALID_ARG
    with pytest.raises(B.TirError):
        B.tir_tune_load(tmp_path / "missing.txt")
    with pytest.raises(B.TirError):
        B.tir_tune_save(tmp_path / "no_such_dir" / "x.txt")
    assert B.tir_tune_count() == 0


def test_tuning_rejects_bad_arguments_before_touching_the_device():
    import ctypes
    L = B.lib()
    us = ctypes.c_double(-1.0)
    # reps out of range, then an invalid problem: status codes, no launch
    st = L.tir_tune_batch_matmul(FAKE, FAKE, FAKE, 1, 64, 64, 64, 0, 64, 1, 0, 64, 1, 0, 64, 1, 0, 3, None, 0, ctypes.byref(us), None)
    assert st == B.TIR_ERR_INVALID_ARG and "reps" in B.last_error()
    st = L.tir_tune_batch_matmul(FAKE, FAKE, FAKE, 1, -4, 64, 64, 0, 64, 1, 0, 64, 1, 0, 64, 1, 0, 3, None, 3, ctypes.byref(us), None)
    assert st == B.TIR_ERR_INVALID_ARG
    # zero-sized problems are a successful no-op
    st = L.tir_tune_batch_matmul(FAKE, FAKE, FAKE, 1, 0, 64, 64, 0, 64, 1, 0, 64, 1, 0, 64, 1, 0, 3, None, 3, ctypes.byref(us), None)
    assert st == B.TIR_OK and us.value == 0.0 and B.tir_tune_count() == 0


def test_fused_entry_points_validate_the_epilogue_on_the_host():
    """Epilogue errors are status codes before any launch: int8 output only through the fused entry
    points and only with a finite positive scale; the bias pointer must be 4-byte aligned."""
    import ctypes
    L = B.lib()
    def gemm_fused(out, ep):
        return L.tir_gemm_fused(FAKE, FAKE, FAKE, 64, 64, 64, 64, 1, 64, 1, 64, 1, B.TIR_I8, out,
                                None if ep is None else ctypes.byref(ep), None)
    assert gemm_fused(B.TIR_I8, None) == B.TIR_ERR_UNSUPPORTED
    assert gemm_fused(B.TIR_I8, B.Epilogue(None, 0, 0.0)) == B.TIR_ERR_INVALID_ARG
    assert gemm_fused(B.TIR_I8, B.Epilogue(None, 0, float("nan"))) == B.TIR_ERR_INVALID_ARG
    assert gemm_fused(B.TIR_I32, B.Epilogue(FAKE + 2, 0, 0.0)) == B.TIR_ERR_ALIGNMENT
    assert gemm_fused(B.TIR_F16, B.Epilogue(None, 1, 1.0)) == B.TIR_ERR_UNSUPPORTED        # (I8, F16) is no pair
    assert B.tir_gemm_status(FAKE, FAKE, FAKE, 64, 64, 64, 64, 1, 64, 1, 64, 1, "i8", B.TIR_I8) == B.TIR_ERR_UNSUPPORTED
    # zero-sized fused calls are no-ops as well
    assert L.tir_gemm_fused(FAKE, FAKE, FAKE, 0, 64, 64, 64, 1, 64, 1, 64, 1, B.TIR_I8, B.TIR_I8,
                            ctypes.byref(B.Epilogue(None, 1, 0.5)), None) == B.TIR_OK
    # the variant query knows the requantising kernels
    assert B.tir_gemm_variant(1, 512, 512, 512, 512, 1, 512, 1, 512, 1, "i8", B.TIR_I8).startswith("i8_i8_")


def test_attention_rejects_bad_arguments_on_the_host():
    def st(**kw):
        a = dict(Q=FAKE, K=FAKE, V=FAKE, O=FAKE, batch=1, M=128, N=128, d=64, scale=0.125, i="f16", o="f16")
        a.update(kw)
        return B.tir_attention_status(a["Q"], a["K"], a["V"], a["O"], a["batch"], a["M"], a["N"], a["d"], a["scale"], a["i"], a["o"])
    assert st(d=96) == B.TIR_ERR_UNSUPPORTED and "head dimension" in B.last_error()
    assert st(N=0) == B.TIR_ERR_INVALID_ARG
    assert st(M=-1) == B.TIR_ERR_INVALID_ARG
    assert st(scale=float("inf")) == B.TIR_ERR_INVALID_ARG
    assert st(i="i8", o="i32") == B.TIR_ERR_UNSUPPORTED
    assert st(i="bf16", o="f16") == B.TIR_ERR_UNSUPPORTED
    assert st(V=0) == B.TIR_ERR_INVALID_ARG
    assert st(O=FAKE + 8) == B.TIR_ERR_ALIGNMENT
    assert st(M=0) == B.TIR_OK and st(batch=0) == B.TIR_OK          # nothing to do: no launch, no device needed


def test_conv1d_conv3d_and_transposed_conv_validate_on_the_host():
    L = B.lib()
    def c1(**kw):
        a = dict(N=1, L=32, C=16, K=16, R=3, stride=1, pad=1, dil=1, groups=1)
        a.update(kw)
        return L.tir_conv1d(FAKE, FAKE, FAKE, a["N"], a["L"], a["C"], a["K"], a["R"], a["stride"], a["pad"], a["dil"], a["groups"],
                            B.TIR_F16, B.TIR_F32, None, None)
    assert c1(stride=0) == B.TIR_ERR_INVALID_ARG
    assert c1(groups=3) == B.TIR_ERR_INVALID_ARG
    assert c1(L=2, R=5, pad=0) == B.TIR_ERR_INVALID_ARG          # empty output
    assert c1(N=0) == B.TIR_OK

    def c3(**kw):
        a = dict(N=1, D=4, H=8, W=8, C=16, K=16, T=3, R=3, S=3, s=(1, 1, 1), p=(1, 1, 1), d=(1, 1, 1), groups=1)
        a.update(kw)
        return L.tir_conv3d(FAKE, FAKE, FAKE, a["N"], a["D"], a["H"], a["W"], a["C"], a["K"], a["T"], a["R"], a["S"], *a["s"], *a["p"], *a["d"],
                            a["groups"], B.TIR_F16, B.TIR_F16, None, None)
    assert c3(D=0) == B.TIR_ERR_INVALID_ARG
    assert c3(d=(0, 1, 1)) == B.TIR_ERR_INVALID_ARG
    assert c3(p=(-1, 0, 0)) == B.TIR_ERR_INVALID_ARG
    assert c3(D=2, T=5, p=(0, 1, 1)) == B.TIR_ERR_INVALID_ARG    # empty output along the depth
    assert c3(D=20000) == B.TIR_ERR_UNSUPPORTED
    assert c3(N=0) == B.TIR_OK

    def ct(**kw):
        a = dict(N=1, H=8, W=8, C=16, K=16, R=3, S=3, s=(2, 2), p=(1, 1), d=(1, 1), op=(1, 1), groups=1)
        a.update(kw)
        return L.tir_conv2d_transpose(FAKE, FAKE, FAKE, a["N"], a["H"], a["W"], a["C"], a["K"], a["R"], a["S"], *a["s"], *a["p"], *a["d"], *a["op"],
                                      a["groups"], B.TIR_I8, B.TIR_I32, None, None)
    assert ct(op=(-1, 0)) == B.TIR_ERR_INVALID_ARG
    assert ct(s=(0, 1)) == B.TIR_ERR_INVALID_ARG
    assert ct(H=1, W=1, R=1, S=1, p=(1, 1), op=(0, 0), s=(1, 1)) == B.TIR_ERR_INVALID_ARG   # extent (1-1)*1 - 2 + 0 + 0 + 1 < 1
    assert ct(K=15, groups=2) == B.TIR_ERR_INVALID_ARG
    assert ct(H=1, s=(20000, 1), op=(0, 0)) == B.TIR_ERR_UNSUPPORTED    # the kernels keep remainders modulo the stride in 16 bits
    assert ct(N=0) == B.TIR_OK
    # by output phase: only undilated, strided, whole 128-byte channel blocks; the queries report how a problem would run
    q = lambda C, s, d, dt="f16": B.tir_conv2d_transpose_variant(2, 8, 8, C, 32, 4, 4, s, (1, 1), d, (0, 0), 1, dt, dt if dt != "i8" else "i32")
    assert q(64, (2, 2), (1, 1)).endswith("_conv/ph2x2")
    assert q(128, (1, 3), (1, 1)).endswith("_conv/ph1x3")
    assert q(128, (2, 2), (1, 1), "i8").endswith("_conv/ph2x2") and "ph" not in q(64, (2, 2), (1, 1), "i8")
    assert "convx" in q(64, (2, 2), (2, 1)) and "convx" in q(32, (2, 2), (1, 1)) and "convx" in q(64, (1, 1), (1, 1))
    assert B.tir_conv3d_variant(1, 10, 16, 16, 128, 64, 3, 3, 3, (1, 1, 1), (1, 1, 1), (1, 1, 1), 1, "f16", "f16").endswith("_convx/z6")
    assert B.tir_conv3d_variant(1, 0, 16, 16, 128, 64, 3, 3, 3, (1, 1, 1), (1, 1, 1), (1, 1, 1), 1, "f16", "f16") == ""


def test_variant_table_is_what_its_generator_writes():
    """csrc/tir_variants.def is generated (gen_variants.py): the committed table and the tile list must not drift apart,
    and every name must be unique."""
    import importlib.util
    import re
    from pathlib import Path
    csrc = Path(__file__).resolve().parent.parent / "paper_2207_04296_amd" / "csrc"
    spec = importlib.util.spec_from_file_location("gen_variants", csrc / "gen_variants.py")
    gen = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(gen)
    text = (csrc / "tir_variants.def").read_text()
    assert gen.render() == text, "run python paper_2207_04296_amd/csrc/gen_variants.py"
    names = re.findall(r'^V\d+\("([^"]+)"', text, flags=re.M)
    assert len(names) == len(set(names)) and len(names) > 600
