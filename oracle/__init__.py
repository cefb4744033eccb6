"""CPU oracle for the tensor-contraction operators: test infrastructure, not the product.

Only tests, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline`` leg may import this
package.  It wraps ``tir_oracle.c`` (plain C, fp64 / int64 direct loops following the operator
definitions in section 4.2 of the TensorIR paper) through ctypes and shares nothing with the HIP
path.  Inputs are raw bit arrays (``uint16`` for binary16 / bfloat16, ``int8``); outputs are
``float64`` (or ``int64`` for int8) numpy arrays, plus ``S = sum |a*b|`` for the parity bound.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "tir_oracle.c"
_LIB = _HERE / "liboracle.so"

F16, BF16, I8 = 0, 1, 2
_DTYPES = {"f16": F16, "bf16": BF16, "i8": I8}


def build(force: bool = False) -> Path:
    """Compile tir_oracle.c with gcc (OpenMP, -O2, no fast-math, no FMA contraction)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared", "-Wall",
               "-Wextra", "-o", str(_LIB), str(_SRC), "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(str(_LIB))
        i64, vp, dp = ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p
        lib.oracle_gemm.argtypes = [ctypes.c_int, vp, vp] + [i64] * 7 + [vp, dp]
        lib.oracle_gemm.restype = ctypes.c_int
        lib.oracle_batch_matmul.argtypes = [ctypes.c_int, vp, vp] + [i64] * 10 + [vp, dp]
        lib.oracle_batch_matmul.restype = ctypes.c_int
        lib.oracle_conv2d.argtypes = [ctypes.c_int, vp, vp] + [i64] * 14 + [vp, dp]
        lib.oracle_conv2d.restype = ctypes.c_int
        lib.oracle_conv_out_extent.argtypes = [i64] * 5
        lib.oracle_conv_out_extent.restype = i64
        lib.oracle_decode.argtypes = [ctypes.c_int, vp, i64, dp]
        lib.oracle_decode.restype = ctypes.c_int
        lib.oracle_epilogue_float.argtypes = [dp, dp, i64, i64, ctypes.POINTER(ctypes.c_float), ctypes.c_int]
        lib.oracle_epilogue_int.argtypes = [ctypes.POINTER(ctypes.c_int64), i64, i64, ctypes.POINTER(ctypes.c_int32),
                                            ctypes.c_int, ctypes.c_int, ctypes.c_float]
        pi64 = ctypes.POINTER(ctypes.c_int64)
        lib.oracle_conv1d.argtypes = [ctypes.c_int, vp, vp] + [i64] * 9 + [vp, dp]
        lib.oracle_conv3d.argtypes = [ctypes.c_int, vp, vp, i64, pi64, i64, i64, pi64, pi64, pi64, pi64, i64, vp, dp]
        lib.oracle_conv2d_transpose.argtypes = [ctypes.c_int, vp, vp] + [i64] * 7 + [pi64, pi64, pi64, pi64, i64, vp, dp]
        lib.oracle_conv_transpose_out_extent.restype = ctypes.c_int64
        lib.oracle_conv_transpose_out_extent.argtypes = [i64] * 6
        lib.oracle_attention.argtypes = [ctypes.c_int, vp, vp, vp] + [i64] * 5 + [ctypes.c_double, dp, dp]
        lib.oracle_set_threads.argtypes = [ctypes.c_int]
        lib.oracle_get_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def set_threads(n: int) -> None:
    _load().oracle_set_threads(int(n))


def get_threads() -> int:
    return int(_load().oracle_get_threads())


def _code(dtype: str) -> int:
    if dtype not in _DTYPES:
        raise ValueError(f"oracle: unknown dtype {dtype!r}")
    return _DTYPES[dtype]


def _check_bits(arr: np.ndarray, dtype: str) -> np.ndarray:
    want = np.int8 if dtype == "i8" else np.uint16
    if arr.dtype != want:
        raise TypeError(f"oracle: {dtype} operand must be raw bits of dtype {want}, got {arr.dtype}")
    return arr


def _ptr(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def _span(extents, strides) -> int:
    """Number of elements a strided view touches (1 + sum (extent-1)*stride), 0 if empty."""
    if any(e == 0 for e in extents):
        return 0
    return 1 + sum((e - 1) * s for e, s in zip(extents, strides))


def decode(dtype: str, bits: np.ndarray) -> np.ndarray:
    bits = np.ascontiguousarray(_check_bits(bits, dtype))
    out = np.empty(bits.shape, dtype=np.float64)
    rc = _load().oracle_decode(_code(dtype), _ptr(bits), bits.size, _ptr(out))
    if rc:
        raise RuntimeError(f"oracle_decode failed with {rc}")
    return out


def conv_out_extent(inp: int, filt: int, stride: int, pad: int, dil: int) -> int:
    return int(_load().oracle_conv_out_extent(inp, filt, stride, pad, dil))


def gemm(dtype: str, A: np.ndarray, B: np.ndarray, M: int, N: int, K: int,
         a_rs: int, a_cs: int, b_rs: int, b_cs: int, want_S: bool = True):
    """C[M,N] = A·B on flat bit buffers A, B with element strides; returns (C, S or None)."""
    A = np.ascontiguousarray(_check_bits(A, dtype)).ravel()
    B = np.ascontiguousarray(_check_bits(B, dtype)).ravel()
    if A.size < _span((M, K), (a_rs, a_cs)) or B.size < _span((K, N), (b_rs, b_cs)):
        raise ValueError("oracle.gemm: operand buffer smaller than the strided extent")
    is_int = dtype == "i8"
    C = np.empty((M, N), dtype=np.int64 if is_int else np.float64)
    S = None if (is_int or not want_S) else np.empty((M, N), dtype=np.float64)
    rc = _load().oracle_gemm(_code(dtype), _ptr(A), _ptr(B), M, N, K, a_rs, a_cs, b_rs, b_cs, _ptr(C),
                             _ptr(S) if S is not None else None)
    if rc:
        raise RuntimeError(f"oracle_gemm failed with {rc}")
    return C, S


def batch_matmul(dtype: str, A: np.ndarray, B: np.ndarray, batch: int, M: int, N: int, K: int,
                 a_bs: int, a_rs: int, a_cs: int, b_bs: int, b_rs: int, b_cs: int, want_S: bool = True):
    A = np.ascontiguousarray(_check_bits(A, dtype)).ravel()
    B = np.ascontiguousarray(_check_bits(B, dtype)).ravel()
    if A.size < _span((batch, M, K), (a_bs, a_rs, a_cs)) or B.size < _span((batch, K, N), (b_bs, b_rs, b_cs)):
        raise ValueError("oracle.batch_matmul: operand buffer smaller than the strided extent")
    is_int = dtype == "i8"
    C = np.empty((batch, M, N), dtype=np.int64 if is_int else np.float64)
    S = None if (is_int or not want_S) else np.empty((batch, M, N), dtype=np.float64)
    rc = _load().oracle_batch_matmul(_code(dtype), _ptr(A), _ptr(B), batch, M, N, K, a_bs, a_rs, a_cs,
                                     b_bs, b_rs, b_cs, _ptr(C), _ptr(S) if S is not None else None)
    if rc:
        raise RuntimeError(f"oracle_batch_matmul failed with {rc}")
    return C, S


def conv2d(dtype: str, x: np.ndarray, w: np.ndarray, stride=(1, 1), pad=(0, 0), dil=(1, 1), groups: int = 1,
           want_S: bool = True):
    """x: bits [N,H,W,C]; w: bits [K,R,S,C/groups]; returns (y [N,P,Q,K], Sabs or None)."""
    x = np.ascontiguousarray(_check_bits(x, dtype))
    w = np.ascontiguousarray(_check_bits(w, dtype))
    N, H, W, C = x.shape
    K, R, S_, Cg = w.shape
    if groups <= 0 or C % groups or K % groups or Cg != C // groups:
        raise ValueError("oracle.conv2d: inconsistent groups / channel counts")
    P = conv_out_extent(H, R, stride[0], pad[0], dil[0])
    Q = conv_out_extent(W, S_, stride[1], pad[1], dil[1])
    if P <= 0 or Q <= 0:
        raise ValueError("oracle.conv2d: empty output")
    is_int = dtype == "i8"
    y = np.empty((N, P, Q, K), dtype=np.int64 if is_int else np.float64)
    Sabs = None if (is_int or not want_S) else np.empty((N, P, Q, K), dtype=np.float64)
    rc = _load().oracle_conv2d(_code(dtype), _ptr(x), _ptr(w), N, H, W, C, K, R, S_, stride[0], stride[1],
                               pad[0], pad[1], dil[0], dil[1], groups, _ptr(y),
                               _ptr(Sabs) if Sabs is not None else None)
    if rc:
        raise RuntimeError(f"oracle_conv2d failed with {rc}")
    return y, Sabs


def epilogue(C: np.ndarray, S, bias=None, relu: bool = False, scale: float = 0.0):
    """Fused consumer applied to an operator result C (last axis = output column / channel): bias add,
    ReLU and, for integer C with scale > 0, requantisation to int8 codes.  Returns new (C, S)."""
    N = C.shape[-1]
    rows = C.size // N if N else 0
    lib = _load()
    if C.dtype == np.float64:
        if scale:
            raise ValueError("oracle.epilogue: requantisation is defined for int8 inputs only")
        C2 = np.ascontiguousarray(C).copy()
        S2 = None if S is None else np.ascontiguousarray(S).copy()
        b = None
        if bias is not None:
            b = np.ascontiguousarray(bias, dtype=np.float32)
            if b.shape != (N,):
                raise ValueError("oracle.epilogue: bias must have one float32 per output column")
        rc = lib.oracle_epilogue_float(C2.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                                       None if S2 is None else S2.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                                       rows, N, None if b is None else b.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
                                       int(bool(relu)))
        if rc:
            raise RuntimeError(f"oracle_epilogue_float failed with {rc}")
        return C2, S2
    if C.dtype != np.int64:
        raise ValueError("oracle.epilogue: C must be the float64 or int64 result of an oracle operator")
    C2 = np.ascontiguousarray(C).copy()
    b = None
    if bias is not None:
        b = np.ascontiguousarray(bias)
        if b.dtype != np.int32 or b.shape != (N,):
            raise ValueError("oracle.epilogue: bias must have one int32 per output column")
    rc = lib.oracle_epilogue_int(C2.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), rows, N,
                                 None if b is None else b.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                 int(bool(relu)), int(scale != 0.0), float(scale))
    if rc:
        raise RuntimeError(f"oracle_epilogue_int failed with {rc} (sum beyond int32, or scale not finite and positive)")
    return C2, None


def attention(dtype: str, Q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float, want_T: bool = True):
    """softmax(scale * Q K^T) V per batch.  Q: bits [batch, M, d], K: [batch, N, d], V: [batch, N, dv].
    Returns (O [batch, M, dv] float64, T or None) with T = sum_j P |V|."""
    if dtype not in ("f16", "bf16"):
        raise ValueError("oracle.attention: f16 or bf16 inputs")
    Q = np.ascontiguousarray(_check_bits(Q, dtype))
    K = np.ascontiguousarray(_check_bits(K, dtype))
    V = np.ascontiguousarray(_check_bits(V, dtype))
    batch, M, d = Q.shape
    _, N, dv = V.shape
    if K.shape != (batch, N, d) or V.shape[0] != batch or N < 1:
        raise ValueError("oracle.attention: inconsistent shapes")
    O = np.empty((batch, M, dv), dtype=np.float64)
    T = np.empty((batch, M, dv), dtype=np.float64) if want_T else None
    rc = _load().oracle_attention(_code(dtype), _ptr(Q), _ptr(K), _ptr(V), batch, M, N, d, dv, float(scale), _ptr(O),
                                  _ptr(T) if T is not None else None)
    if rc:
        raise RuntimeError(f"oracle_attention failed with {rc}")
    return O, T


def _i64arr(v):
    return (ctypes.c_int64 * len(v))(*[int(e) for e in v])


def _conv_out(is_int, shape, want_S):
    y = np.empty(shape, dtype=np.int64 if is_int else np.float64)
    S = None if (is_int or not want_S) else np.empty(shape, dtype=np.float64)
    return y, S


def conv1d(dtype: str, x: np.ndarray, w: np.ndarray, stride: int = 1, pad: int = 0, dil: int = 1, groups: int = 1,
           want_S: bool = True):
    """x: bits [N,L,C]; w: bits [K,R,C/groups]; returns (y [N,P,K], Sabs or None)."""
    x = np.ascontiguousarray(_check_bits(x, dtype)); w = np.ascontiguousarray(_check_bits(w, dtype))
    N, L, C = x.shape
    K, R, Cg = w.shape
    if groups <= 0 or C % groups or K % groups or Cg != C // groups:
        raise ValueError("oracle.conv1d: inconsistent groups / channel counts")
    P = conv_out_extent(L, R, stride, pad, dil)
    if P <= 0:
        raise ValueError("oracle.conv1d: empty output")
    y, S = _conv_out(dtype == "i8", (N, P, K), want_S)
    rc = _load().oracle_conv1d(_code(dtype), _ptr(x), _ptr(w), N, L, C, K, R, stride, pad, dil, groups, _ptr(y),
                               _ptr(S) if S is not None else None)
    if rc:
        raise RuntimeError(f"oracle_conv1d failed with {rc}")
    return y, S


def conv3d(dtype: str, x: np.ndarray, w: np.ndarray, stride=(1, 1, 1), pad=(0, 0, 0), dil=(1, 1, 1), groups: int = 1,
           want_S: bool = True):
    """x: bits [N,D,H,W,C]; w: bits [K,T,R,S,C/groups]; returns (y [N,OD,P,Q,K], Sabs or None)."""
    x = np.ascontiguousarray(_check_bits(x, dtype)); w = np.ascontiguousarray(_check_bits(w, dtype))
    N, D, H, W, C = x.shape
    K, T, R, S_, Cg = w.shape
    if groups <= 0 or C % groups or K % groups or Cg != C // groups:
        raise ValueError("oracle.conv3d: inconsistent groups / channel counts")
    out = [conv_out_extent(i, f, s, p, d) for i, f, s, p, d in zip((D, H, W), (T, R, S_), stride, pad, dil)]
    if min(out) <= 0:
        raise ValueError("oracle.conv3d: empty output")
    y, S = _conv_out(dtype == "i8", (N, *out, K), want_S)
    rc = _load().oracle_conv3d(_code(dtype), _ptr(x), _ptr(w), N, _i64arr((D, H, W)), C, K, _i64arr((T, R, S_)), _i64arr(stride),
                               _i64arr(pad), _i64arr(dil), groups, _ptr(y), _ptr(S) if S is not None else None)
    if rc:
        raise RuntimeError(f"oracle_conv3d failed with {rc}")
    return y, S


def conv_transpose_out_extent(inp: int, filt: int, stride: int, pad: int, dil: int, outpad: int) -> int:
    return int(_load().oracle_conv_transpose_out_extent(inp, filt, stride, pad, dil, outpad))


def conv2d_transpose(dtype: str, x: np.ndarray, w: np.ndarray, stride=(1, 1), pad=(0, 0), dil=(1, 1), outpad=(0, 0),
                     groups: int = 1, want_S: bool = True):
    """x: bits [N,H,W,C]; w: bits [K,R,S,C/groups] (output channel k, tap (r,s), input channel c of k's group);
    returns (y [N,P,Q,K], Sabs or None)."""
    x = np.ascontiguousarray(_check_bits(x, dtype)); w = np.ascontiguousarray(_check_bits(w, dtype))
    N, H, W, C = x.shape
    K, R, S_, Cg = w.shape
    if groups <= 0 or C % groups or K % groups or Cg != C // groups:
        raise ValueError("oracle.conv2d_transpose: inconsistent groups / channel counts")
    P = conv_transpose_out_extent(H, R, stride[0], pad[0], dil[0], outpad[0])
    Q = conv_transpose_out_extent(W, S_, stride[1], pad[1], dil[1], outpad[1])
    if P <= 0 or Q <= 0:
        raise ValueError("oracle.conv2d_transpose: empty output")
    y, S = _conv_out(dtype == "i8", (N, P, Q, K), want_S)
    rc = _load().oracle_conv2d_transpose(_code(dtype), _ptr(x), _ptr(w), N, H, W, C, K, R, S_, _i64arr(stride), _i64arr(pad),
                                         _i64arr(dil), _i64arr(outpad), groups, _ptr(y), _ptr(S) if S is not None else None)
    if rc:
        raise RuntimeError(f"oracle_conv2d_transpose failed with {rc}")
    return y, S
