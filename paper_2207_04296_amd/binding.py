"""ctypes binding of libtir.so: same names as the C ABI, argument marshalling only.

Every operator call ends in one of the ``extern "C"`` entry points declared in ``include/tir.h``;
there is no Python or PyTorch fallback.  If the library has not been built, loading fails loudly.
PyTorch is used for device memory and streams only.
"""
from __future__ import annotations

import ctypes
from pathlib import Path

_PKG = Path(__file__).resolve().parent
_LIBPATH = _PKG / "libtir.so"

TIR_OK, TIR_ERR_INVALID_ARG, TIR_ERR_UNSUPPORTED, TIR_ERR_ALIGNMENT, TIR_ERR_LAUNCH = range(5)
TIR_F16, TIR_BF16, TIR_I8, TIR_F32, TIR_I32 = range(5)
DTYPE_CODES = {"f16": TIR_F16, "bf16": TIR_BF16, "i8": TIR_I8, "f32": TIR_F32, "i32": TIR_I32}

EXPORTS = ["tir_gemm", "tir_batch_matmul", "tir_conv2d", "tir_last_error", "tir_gemm_variant",
           "tir_conv2d_variant", "tir_debug_force_tile", "tir_debug_force_variant", "tir_debug_variant_count",
           "tir_debug_variant_name", "tir_debug_tile_of_block", "tir_probe_mfma_rate", "tir_version",
           "tir_tune_batch_matmul", "tir_tune_conv2d", "tir_tune_count", "tir_tune_clear", "tir_tune_save",
           "tir_tune_load", "tir_gemm_fused", "tir_batch_matmul_fused", "tir_conv2d_fused", "tir_attention",
           "tir_conv1d", "tir_conv3d", "tir_conv2d_transpose", "tir_debug_force_ksplit", "tir_debug_fastdiv",
           "tir_conv2d_transpose_variant", "tir_conv3d_variant", "tir_tune_conv3d", "tir_tune_conv2d_transpose",
           "tir_workspace_bytes", "tir_set_workspace", "tir_gemm_split_static"]


class Epilogue(ctypes.Structure):
    """struct tir_epilogue: bias pointer, relu flag, requantisation scale, cache policy of the output stores."""
    _fields_ = [("bias", ctypes.c_void_p), ("relu", ctypes.c_int), ("scale", ctypes.c_float), ("streaming", ctypes.c_int)]


def make_epilogue(bias=None, relu=False, scale=0.0, streaming=False):
    """ctypes tir_epilogue, or None when nothing is fused and the output policy is the default (the plain operator)."""
    if bias is None and not relu and not scale and not streaming:
        return None
    return Epilogue(_ptr(bias) or None, int(bool(relu)), float(scale), int(streaming))


class TirError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"tir status {status}: {message}")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    """Load libtir.so (built by ``python -m paper_2207_04296_amd.buildlib``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not _LIBPATH.exists():
        raise RuntimeError(f"{_LIBPATH} is missing: build it with `python -m paper_2207_04296_amd.buildlib` "
                           "(there is no fallback path)")
    # The library must share the HIP runtime that owns the caller's device memory.  PyTorch ships
    # its own libamdhip64 (same soname as the system one): importing torch first makes the dynamic
    # loader bind libtir.so to that copy instead of loading a second runtime.
    import torch  # noqa: F401
    L = ctypes.CDLL(str(_LIBPATH))
    i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
    L.tir_gemm.argtypes = [vp, vp, vp] + [i64] * 9 + [ci, ci, vp]
    L.tir_gemm.restype = ci
    L.tir_batch_matmul.argtypes = [vp, vp, vp] + [i64] * 13 + [ci, ci, vp]
    L.tir_batch_matmul.restype = ci
    L.tir_conv2d.argtypes = [vp, vp, vp] + [i64] * 7 + [ci] * 7 + [ci, ci, vp]
    L.tir_conv2d.restype = ci
    L.tir_last_error.restype = ctypes.c_char_p
    L.tir_gemm_variant.argtypes = [i64] * 10 + [ci, ci]
    L.tir_gemm_variant.restype = ctypes.c_char_p
    L.tir_conv2d_variant.argtypes = [i64] * 7 + [ci] * 7 + [ci, ci]
    L.tir_conv2d_variant.restype = ctypes.c_char_p
    L.tir_conv2d_transpose_variant.argtypes = [i64] * 7 + [ci] * 9 + [ci, ci]
    L.tir_conv2d_transpose_variant.restype = ctypes.c_char_p
    L.tir_debug_force_tile.argtypes = [ci, ci]
    L.tir_debug_force_tile.restype = None
    L.tir_debug_force_variant.argtypes = [ctypes.c_char_p]
    L.tir_debug_force_variant.restype = None
    L.tir_debug_fastdiv.argtypes = [ctypes.c_uint, ctypes.c_uint]
    L.tir_debug_fastdiv.restype = ctypes.c_uint
    L.tir_debug_force_ksplit.argtypes = [ctypes.c_int]
    L.tir_debug_force_ksplit.restype = None
    L.tir_debug_variant_count.restype = ci
    L.tir_debug_variant_name.argtypes = [ci]
    L.tir_debug_variant_name.restype = ctypes.c_char_p
    L.tir_debug_tile_of_block.argtypes = [ci, ci, ci, ctypes.POINTER(ci), ctypes.POINTER(ci)]
    L.tir_debug_tile_of_block.restype = None
    L.tir_probe_mfma_rate.argtypes = [vp, ci, ci, ctypes.POINTER(ctypes.c_double), vp]
    L.tir_probe_mfma_rate.restype = ci
    L.tir_version.restype = ctypes.c_char_p
    pd = ctypes.POINTER(ctypes.c_double)
    pe = ctypes.POINTER(Epilogue)
    L.tir_gemm_fused.argtypes = [vp, vp, vp] + [i64] * 9 + [ci, ci, pe, vp]
    L.tir_gemm_fused.restype = ci
    L.tir_batch_matmul_fused.argtypes = [vp, vp, vp] + [i64] * 13 + [ci, ci, pe, vp]
    L.tir_batch_matmul_fused.restype = ci
    L.tir_conv2d_fused.argtypes = [vp, vp, vp] + [i64] * 7 + [ci] * 7 + [ci, ci, pe, vp]
    L.tir_conv2d_fused.restype = ci
    L.tir_conv1d.argtypes = [vp, vp, vp] + [i64] * 5 + [ci] * 4 + [ci, ci, pe, vp]
    L.tir_conv1d.restype = ci
    L.tir_conv3d.argtypes = [vp, vp, vp] + [i64] * 9 + [ci] * 10 + [ci, ci, pe, vp]
    L.tir_conv3d.restype = ci
    L.tir_conv2d_transpose.argtypes = [vp, vp, vp] + [i64] * 7 + [ci] * 9 + [ci, ci, pe, vp]
    L.tir_conv2d_transpose.restype = ci
    L.tir_attention.argtypes = [vp, vp, vp, vp] + [i64] * 4 + [ctypes.c_float, ci, ci, vp]
    L.tir_attention.restype = ci
    L.tir_tune_batch_matmul.argtypes = [vp, vp, vp] + [i64] * 13 + [ci, ci, pe, ci, pd, vp]
    L.tir_tune_batch_matmul.restype = ci
    L.tir_tune_conv2d.argtypes = [vp, vp, vp] + [i64] * 7 + [ci] * 7 + [ci, ci, pe, ci, pd, vp]
    L.tir_tune_conv2d.restype = ci
    L.tir_tune_conv3d.argtypes = [vp, vp, vp] + [i64] * 9 + [ci] * 10 + [ci, ci, pe, ci, pd, vp]
    L.tir_tune_conv3d.restype = ci
    L.tir_tune_conv2d_transpose.argtypes = [vp, vp, vp] + [i64] * 7 + [ci] * 9 + [ci, ci, pe, ci, pd, vp]
    L.tir_tune_conv2d_transpose.restype = ci
    L.tir_conv3d_variant.argtypes = [i64] * 9 + [ci] * 10 + [ci, ci]
    L.tir_conv3d_variant.restype = ctypes.c_char_p
    L.tir_workspace_bytes.restype = ctypes.c_uint64
    L.tir_set_workspace.argtypes = [vp, vp, ctypes.c_uint64]
    L.tir_set_workspace.restype = ci
    L.tir_gemm_split_static.argtypes = [vp, vp, vp] + [i64] * 9 + [ci, ci, pe, ci, vp]
    L.tir_gemm_split_static.restype = ci
    L.tir_tune_count.restype = ci
    L.tir_tune_clear.restype = None
    L.tir_tune_save.argtypes = [ctypes.c_char_p]
    L.tir_tune_save.restype = ci
    L.tir_tune_load.argtypes = [ctypes.c_char_p]
    L.tir_tune_load.restype = ci
    _lib = L
    return L


def _ptr(t) -> int:
    """Device pointer of a torch tensor, or an int passed through."""
    if t is None:
        return 0
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _code(d) -> int:
    return DTYPE_CODES[d] if isinstance(d, str) else int(d)


def _check(status: int) -> None:
    if status != TIR_OK:
        raise TirError(status, lib().tir_last_error().decode())


def last_error() -> str:
    return lib().tir_last_error().decode()


def tir_gemm_status(A, B, C, M, N, K, a_rs, a_cs, b_rs, b_cs, c_rs, c_cs, in_dtype, out_dtype, stream=0) -> int:
    """Raw call returning the status code (used by the error-path tests; needs no GPU to fail)."""
    return lib().tir_gemm(_ptr(A), _ptr(B), _ptr(C), M, N, K, a_rs, a_cs, b_rs, b_cs, c_rs, c_cs,
                          _code(in_dtype), _code(out_dtype), stream)


def tir_batch_matmul_status(A, B, C, batch, M, N, K, a_bs, a_rs, a_cs, b_bs, b_rs, b_cs, c_bs, c_rs, c_cs,
                            in_dtype, out_dtype, stream=0) -> int:
    return lib().tir_batch_matmul(_ptr(A), _ptr(B), _ptr(C), batch, M, N, K, a_bs, a_rs, a_cs, b_bs, b_rs, b_cs,
                                  c_bs, c_rs, c_cs, _code(in_dtype), _code(out_dtype), stream)


def tir_conv2d_status(x, w, y, N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, groups,
                      in_dtype, out_dtype, stream=0) -> int:
    return lib().tir_conv2d(_ptr(x), _ptr(w), _ptr(y), N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w,
                            dil_h, dil_w, groups, _code(in_dtype), _code(out_dtype), stream)


def tir_gemm(A, B, C, M, N, K, a_rs, a_cs, b_rs, b_cs, c_rs, c_cs, in_dtype, out_dtype, stream=None) -> None:
    _check(tir_gemm_status(A, B, C, M, N, K, a_rs, a_cs, b_rs, b_cs, c_rs, c_cs, in_dtype, out_dtype,
                           _stream(stream)))


def tir_batch_matmul(A, B, C, batch, M, N, K, a_bs, a_rs, a_cs, b_bs, b_rs, b_cs, c_bs, c_rs, c_cs,
                     in_dtype, out_dtype, stream=None) -> None:
    _check(tir_batch_matmul_status(A, B, C, batch, M, N, K, a_bs, a_rs, a_cs, b_bs, b_rs, b_cs, c_bs, c_rs, c_cs,
                                   in_dtype, out_dtype, _stream(stream)))


def tir_conv2d(x, w, y, N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, groups,
               in_dtype, out_dtype, stream=None) -> None:
    _check(tir_conv2d_status(x, w, y, N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, groups,
                             in_dtype, out_dtype, _stream(stream)))


def tir_gemm_variant(batch, M, N, K, a_rs, a_cs, b_rs, b_cs, c_rs, c_cs, in_dtype, out_dtype) -> str:
    return lib().tir_gemm_variant(batch, M, N, K, a_rs, a_cs, b_rs, b_cs, c_rs, c_cs, _code(in_dtype),
                                  _code(out_dtype)).decode()


def tir_conv2d_variant(N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, groups, in_dtype,
                       out_dtype) -> str:
    return lib().tir_conv2d_variant(N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, groups,
                                    _code(in_dtype), _code(out_dtype)).decode()


def tir_conv2d_transpose_variant(N, H, W, C, K, R, S, stride, pad, dil, outpad, groups, in_dtype, out_dtype) -> str:
    return lib().tir_conv2d_transpose_variant(N, H, W, C, K, R, S, *stride, *pad, *dil, *outpad, groups, _code(in_dtype),
                                              _code(out_dtype)).decode()


def tir_debug_force_tile(bm: int, bn: int) -> None:
    lib().tir_debug_force_tile(bm, bn)


def tir_debug_force_variant(name_part: str) -> None:
    lib().tir_debug_force_variant((name_part or "").encode())


def tir_debug_fastdiv(d: int, m: int) -> int:
    return int(lib().tir_debug_fastdiv(d, m))


def tir_debug_force_ksplit(slices: int) -> None:
    lib().tir_debug_force_ksplit(int(slices))


TIR_STATIC_SCRATCH_BYTES, TIR_STATIC_SCRATCH_TILES = 8 << 20, 1024


def tir_gemm_split_static_status(A, B, C, M, N, K, a_rs, a_cs, b_rs, b_cs, c_rs, c_cs, in_dtype, out_dtype, ep, slices, stream=0) -> int:
    return lib().tir_gemm_split_static(_ptr(A), _ptr(B), _ptr(C), M, N, K, a_rs, a_cs, b_rs, b_cs, c_rs, c_cs, _code(in_dtype),
                                       _code(out_dtype), _ep_arg(ep), int(slices), stream)


def tir_gemm_split_static(A, B, C, M, N, K, a_rs, a_cs, b_rs, b_cs, c_rs, c_cs, in_dtype, out_dtype, ep=None, slices=2, stream=None) -> None:
    """tir_gemm_fused with the reduction split `slices` ways over the library's static device scratch (allocates nothing)."""
    _check(tir_gemm_split_static_status(A, B, C, M, N, K, a_rs, a_cs, b_rs, b_cs, c_rs, c_cs, in_dtype, out_dtype, ep, slices,
                                        _stream(stream)))


def tir_workspace_bytes() -> int:
    return int(lib().tir_workspace_bytes())


def tir_set_workspace_status(ws, nbytes: int, stream=0) -> int:
    """Raw call returning the status code (the size and alignment checks need no GPU)."""
    return lib().tir_set_workspace(stream or None, _ptr(ws) or None, int(nbytes))


def tir_set_workspace(ws, stream=None) -> None:
    """Hand the library a caller-owned uint8 device tensor for the split reductions launched on `stream`
    (None as `ws`: remove the registration, launches run unsplit).  The caller keeps the tensor alive."""
    nbytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(lib().tir_set_workspace(_stream(stream) or None, _ptr(ws) or None, nbytes))


def tir_debug_variant_names():
    L = lib()
    return [L.tir_debug_variant_name(i).decode() for i in range(L.tir_debug_variant_count())]


def tir_debug_tile_of_block(bid: int, tiles_m: int, tiles_n: int):
    tm, tn = ctypes.c_int(), ctypes.c_int()
    lib().tir_debug_tile_of_block(bid, tiles_m, tiles_n, ctypes.byref(tm), ctypes.byref(tn))
    return tm.value, tn.value


def tir_probe_mfma_rate(sink, iters: int, random_operands: bool, stream=None) -> float:
    """Enqueue the MFMA-rate probe; returns its FLOP count (time it with events around the call)."""
    flop = ctypes.c_double()
    _check(lib().tir_probe_mfma_rate(_ptr(sink), int(iters), int(bool(random_operands)), ctypes.byref(flop),
                                     _stream(stream)))
    return flop.value


def tir_version() -> str:
    return lib().tir_version().decode()


def _ep_arg(ep):
    return None if ep is None else ctypes.byref(ep)


def tir_gemm_fused(A, B, C, M, N, K, a_rs, a_cs, b_rs, b_cs, c_rs, c_cs, in_dtype, out_dtype, ep=None, stream=None) -> None:
    """ep: an Epilogue from make_epilogue(), or None for the plain operator."""
    _check(lib().tir_gemm_fused(_ptr(A), _ptr(B), _ptr(C), M, N, K, a_rs, a_cs, b_rs, b_cs, c_rs, c_cs, _code(in_dtype),
                                _code(out_dtype), _ep_arg(ep), _stream(stream)))


def tir_batch_matmul_fused(A, B, C, batch, M, N, K, a_bs, a_rs, a_cs, b_bs, b_rs, b_cs, c_bs, c_rs, c_cs,
                           in_dtype, out_dtype, ep=None, stream=None) -> None:
    _check(lib().tir_batch_matmul_fused(_ptr(A), _ptr(B), _ptr(C), batch, M, N, K, a_bs, a_rs, a_cs, b_bs, b_rs, b_cs,
                                        c_bs, c_rs, c_cs, _code(in_dtype), _code(out_dtype), _ep_arg(ep),
                                        _stream(stream)))


def tir_conv2d_fused(x, w, y, N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, groups,
                     in_dtype, out_dtype, ep=None, stream=None) -> None:
    _check(lib().tir_conv2d_fused(_ptr(x), _ptr(w), _ptr(y), N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w,
                                  dil_h, dil_w, groups, _code(in_dtype), _code(out_dtype), _ep_arg(ep),
                                  _stream(stream)))


def tir_conv1d(x, w, y, N, L, C, K, R, stride, pad, dil, groups, in_dtype, out_dtype, ep=None, stream=None) -> None:
    _check(lib().tir_conv1d(_ptr(x), _ptr(w), _ptr(y), N, L, C, K, R, stride, pad, dil, groups, _code(in_dtype),
                            _code(out_dtype), _ep_arg(ep), _stream(stream)))


def tir_conv3d(x, w, y, N, D, H, W, C, K, T, R, S, stride, pad, dil, groups, in_dtype, out_dtype, ep=None, stream=None) -> None:
    """stride, pad, dil: (depth, height, width) triples."""
    _check(lib().tir_conv3d(_ptr(x), _ptr(w), _ptr(y), N, D, H, W, C, K, T, R, S, *stride, *pad, *dil, groups,
                            _code(in_dtype), _code(out_dtype), _ep_arg(ep), _stream(stream)))


def tir_conv2d_transpose(x, w, y, N, H, W, C, K, R, S, stride, pad, dil, outpad, groups, in_dtype, out_dtype, ep=None,
                         stream=None) -> None:
    """stride, pad, dil, outpad: (height, width) pairs."""
    _check(lib().tir_conv2d_transpose(_ptr(x), _ptr(w), _ptr(y), N, H, W, C, K, R, S, *stride, *pad, *dil, *outpad, groups,
                                      _code(in_dtype), _code(out_dtype), _ep_arg(ep), _stream(stream)))


def tir_attention_status(Q, K, V, O, batch, M, N, d, scale, in_dtype, out_dtype, stream=0) -> int:
    return lib().tir_attention(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), batch, M, N, d, float(scale), _code(in_dtype),
                               _code(out_dtype), stream)


def tir_attention(Q, K, V, O, batch, M, N, d, scale, in_dtype, out_dtype, stream=None) -> None:
    """O[b] = softmax(scale * Q[b] K[b]^T) V[b]; Q [batch, M, d], K and V [batch, N, d], d in (64, 128)."""
    _check(tir_attention_status(Q, K, V, O, batch, M, N, d, scale, in_dtype, out_dtype, _stream(stream)))


def tir_tune_batch_matmul(A, B, C, batch, M, N, K, a_bs, a_rs, a_cs, b_bs, b_rs, b_cs, c_bs, c_rs, c_cs,
                          in_dtype, out_dtype, ep=None, reps=5, stream=None) -> float:
    """Measure every variant for this problem and record the fastest; returns its microseconds per launch."""
    us = ctypes.c_double()
    _check(lib().tir_tune_batch_matmul(_ptr(A), _ptr(B), _ptr(C), batch, M, N, K, a_bs, a_rs, a_cs, b_bs, b_rs, b_cs,
                                       c_bs, c_rs, c_cs, _code(in_dtype), _code(out_dtype), _ep_arg(ep), int(reps),
                                       ctypes.byref(us), _stream(stream)))
    return us.value


def tir_tune_conv2d(x, w, y, N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, groups,
                    in_dtype, out_dtype, ep=None, reps=5, stream=None) -> float:
    us = ctypes.c_double()
    _check(lib().tir_tune_conv2d(_ptr(x), _ptr(w), _ptr(y), N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w,
                                 dil_h, dil_w, groups, _code(in_dtype), _code(out_dtype), _ep_arg(ep), int(reps),
                                 ctypes.byref(us), _stream(stream)))
    return us.value


def tir_tune_conv3d(x, w, y, N, D, H, W, C, K, T, R, S, stride, pad, dil, groups, in_dtype, out_dtype, ep=None, reps=5,
                    stream=None) -> float:
    us = ctypes.c_double()
    _check(lib().tir_tune_conv3d(_ptr(x), _ptr(w), _ptr(y), N, D, H, W, C, K, T, R, S, *stride, *pad, *dil, groups,
                                 _code(in_dtype), _code(out_dtype), _ep_arg(ep), int(reps), ctypes.byref(us), _stream(stream)))
    return us.value


def tir_tune_conv2d_transpose(x, w, y, N, H, W, C, K, R, S, stride, pad, dil, outpad, groups, in_dtype, out_dtype, ep=None,
                              reps=5, stream=None) -> float:
    us = ctypes.c_double()
    _check(lib().tir_tune_conv2d_transpose(_ptr(x), _ptr(w), _ptr(y), N, H, W, C, K, R, S, *stride, *pad, *dil, *outpad, groups,
                                           _code(in_dtype), _code(out_dtype), _ep_arg(ep), int(reps), ctypes.byref(us),
                                           _stream(stream)))
    return us.value


def tir_conv3d_variant(N, D, H, W, C, K, T, R, S, stride, pad, dil, groups, in_dtype, out_dtype) -> str:
    return lib().tir_conv3d_variant(N, D, H, W, C, K, T, R, S, *stride, *pad, *dil, groups, _code(in_dtype),
                                    _code(out_dtype)).decode()


def tir_tune_count() -> int:
    return lib().tir_tune_count()


def tir_tune_clear() -> None:
    lib().tir_tune_clear()


def tir_tune_save(path) -> None:
    _check(lib().tir_tune_save(str(path).encode()))


def tir_tune_load(path) -> None:
    _check(lib().tir_tune_load(str(path).encode()))


# ------------------------------------------------------------------------------------------------
# device-memory plumbing for harnesses (bits <-> torch tensors); no arithmetic
# ------------------------------------------------------------------------------------------------
def to_device(bits, dtype: str, device="cuda:0"):
    """numpy raw bits (uint16 / int8) -> torch device tensor of the matching dtype."""
    import numpy as np
    import torch
    if dtype == "i8":
        return torch.from_numpy(np.ascontiguousarray(bits)).to(device)
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device)
    return t.view(torch.float16 if dtype == "f16" else torch.bfloat16)


def empty_out(shape, out_dtype: str, device="cuda:0"):
    import torch
    dt = {"f32": torch.float32, "i32": torch.int32, "f16": torch.float16, "bf16": torch.bfloat16, "i8": torch.int8}[out_dtype]
    return torch.empty(shape, dtype=dt, device=device)


def bias_to_device(wl, device="cuda:0"):
    """Device tensor of the workload's seeded bias (float32 / int32), or None."""
    import torch
    b = wl.bias_values()
    return None if b is None else torch.from_numpy(b).to(device)


def _wl_epilogue(wl, bias_dev, streaming=False):
    if wl.ep_bias and bias_dev is None:
        raise ValueError(f"{wl.name} has a fused bias: pass its device tensor (bias_to_device)")
    return make_epilogue(bias_dev if wl.ep_bias else None, wl.ep_relu, wl.ep_scale, streaming)


def run_workload(wl, a_dev, b_dev, c_dev, bias_dev=None, stream=None, streaming=False) -> None:
    """Launch one paper_2207_04296_amd.inputs.Workload on resident operands (streaming: non-temporal output stores)."""
    ep = _wl_epilogue(wl, bias_dev, streaming)
    if wl.kind == "conv2d":
        tir_conv2d_fused(a_dev, b_dev, c_dev, wl.n, wl.h, wl.w, wl.c, wl.k, wl.r, wl.s, wl.stride[0], wl.stride[1],
                         wl.pad[0], wl.pad[1], wl.dil[0], wl.dil[1], wl.groups, wl.dtype, wl.out, ep, stream)
        return
    M, N, K = wl.M, wl.N, wl.K
    b_rs, b_cs = (1, K) if wl.trans_b else (N, 1)
    if wl.kind == "gemm":
        tir_gemm_fused(a_dev, b_dev, c_dev, M, N, K, K, 1, b_rs, b_cs, N, 1, wl.dtype, wl.out, ep, stream)
    else:
        tir_batch_matmul_fused(a_dev, b_dev, c_dev, wl.batch, M, N, K, M * K, K, 1, K * N, b_rs, b_cs, M * N, N, 1,
                               wl.dtype, wl.out, ep, stream)


def prepare_workload(wl, a_dev, b_dev, c_dev, bias_dev=None, stream=None, streaming=False):
    """run_workload with the argument marshalling done once: returns a function of no arguments that launches
    the workload on these operands and this stream (for launch loops where the host's time per call matters)."""
    ep = _wl_epilogue(wl, bias_dev, streaming)            # kept alive by the closure below
    L, st = lib(), _stream(stream)
    a, b, c, ep_ref = _ptr(a_dev), _ptr(b_dev), _ptr(c_dev), _ep_arg(ep)
    dt, od = _code(wl.dtype), _code(wl.out)
    if wl.kind == "conv2d":
        fn = L.tir_conv2d_fused
        args = (a, b, c, wl.n, wl.h, wl.w, wl.c, wl.k, wl.r, wl.s, wl.stride[0], wl.stride[1], wl.pad[0], wl.pad[1],
                wl.dil[0], wl.dil[1], wl.groups, dt, od, ep_ref, st)
    else:
        M, N, K = wl.M, wl.N, wl.K
        b_rs, b_cs = (1, K) if wl.trans_b else (N, 1)
        if wl.kind == "gemm":
            fn = L.tir_gemm_fused
            args = (a, b, c, M, N, K, K, 1, b_rs, b_cs, N, 1, dt, od, ep_ref, st)
        else:
            fn = L.tir_batch_matmul_fused
            args = (a, b, c, wl.batch, M, N, K, M * K, K, 1, K * N, b_rs, b_cs, M * N, N, 1, dt, od, ep_ref, st)

    def launch(_keep=(a_dev, b_dev, c_dev, bias_dev, ep)) -> None:
        status = fn(*args)
        if status != TIR_OK:
            _check(status)

    return launch


def tune_workload(wl, a_dev, b_dev, c_dev, bias_dev=None, reps=5, stream=None) -> float:
    """tir_tune_* for one paper_2207_04296_amd.inputs.Workload; returns the winner's microseconds per launch."""
    ep = _wl_epilogue(wl, bias_dev)
    if wl.kind == "conv2d":
        return tir_tune_conv2d(a_dev, b_dev, c_dev, wl.n, wl.h, wl.w, wl.c, wl.k, wl.r, wl.s, wl.stride[0], wl.stride[1],
                               wl.pad[0], wl.pad[1], wl.dil[0], wl.dil[1], wl.groups, wl.dtype, wl.out, ep, reps, stream)
    M, N, K = wl.M, wl.N, wl.K
    b_rs, b_cs = (1, K) if wl.trans_b else (N, 1)
    if wl.kind == "gemm":
        return tir_tune_batch_matmul(a_dev, b_dev, c_dev, 1, M, N, K, 0, K, 1, 0, b_rs, b_cs, 0, N, 1, wl.dtype, wl.out,
                                     ep, reps, stream)
    return tir_tune_batch_matmul(a_dev, b_dev, c_dev, wl.batch, M, N, K, M * K, K, 1, K * N, b_rs, b_cs, M * N, N, 1,
                                 wl.dtype, wl.out, ep, reps, stream)


def out_shape(wl):
    if wl.kind == "conv2d":
        p, q = wl.out_hw()
        return (wl.n, p, q, wl.k)
    return (wl.batch, wl.M, wl.N) if wl.kind == "bmm" else (wl.M, wl.N)
