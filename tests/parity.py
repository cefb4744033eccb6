"""Shared helpers of the GPU parity tests: run a workload through the C ABI and compare it with
the CPU oracle element by element.

Bar (per element):  int8 -> int32 bit-exact;  fp16 / bf16:  |gpu - oracle| <= 2e-3 * S + 1e-5 with
S = sum_k |a*b| from the oracle.  For 16-bit outputs the same bound holds because rounding the
fp32 accumulator to fp16 adds at most 2^-11 |c| <= 4.9e-4 S (bf16 outputs are only checked on data
whose |c| is well below S/2, see the callers).
"""
from __future__ import annotations

import numpy as np

RTOL_S = 2e-3
ATOL = 1e-5


def gpu_to_f64(t):
    import torch
    if t.dtype in (torch.int32, torch.int8):
        return t.cpu().numpy().astype(np.int64)
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def assert_close(gpu, ref, S, what=""):
    """gpu, ref: numpy arrays of identical shape; S None for integer data."""
    assert gpu.shape == ref.shape, f"{what}: shape {gpu.shape} vs {ref.shape}"
    if S is None:
        bad = np.flatnonzero(gpu.ravel() != ref.ravel())
        assert bad.size == 0, (f"{what}: {bad.size} of {gpu.size} integer outputs differ; first at flat index "
                               f"{bad[0]}: gpu={gpu.ravel()[bad[0]]} oracle={ref.ravel()[bad[0]]}")
        return 0.0
    assert np.all(np.isfinite(gpu)), f"{what}: non-finite GPU output"
    err = np.abs(gpu - ref)
    tol = RTOL_S * S + ATOL
    ratio = err / tol
    worst = int(np.argmax(ratio))
    assert ratio.ravel()[worst] <= 1.0, (f"{what}: max err/tol = {ratio.ravel()[worst]:.3g} at flat index {worst}: "
                                         f"gpu={gpu.ravel()[worst]!r} oracle={ref.ravel()[worst]!r} S={S.ravel()[worst]!r}")
    return float(ratio.ravel()[worst])


def run_gpu(wl, a_bits, b_bits, prefill=True, streaming=False):
    """Launch workload wl on cuda:0 through the C ABI; returns the output as float64 / int64 numpy."""
    import torch
    from paper_2207_04296_amd import binding as B
    a = B.to_device(a_bits, wl.dtype)
    b = B.to_device(b_bits, wl.dtype)
    c = B.empty_out(B.out_shape(wl), wl.out)
    if prefill:  # the result must overwrite whatever was there (reduction init)
        if c.dtype.is_floating_point:
            c.fill_(float("nan"))
        else:
            c.fill_(-77 if c.dtype == torch.int8 else -123456789)
    B.run_workload(wl, a, b, c, B.bias_to_device(wl), streaming=streaming)
    torch.cuda.synchronize()
    return gpu_to_f64(c)


def run_oracle(wl, a_bits, b_bits, oracle):
    """(result, S) of the workload incl. its fused consumer; S is None for integer results."""
    if wl.kind == "conv2d":
        C, S = oracle.conv2d(wl.dtype, a_bits, b_bits, wl.stride, wl.pad, wl.dil, wl.groups)
    else:
        b_rs, b_cs = (1, wl.K) if wl.trans_b else (wl.N, 1)
        if wl.kind == "gemm":
            C, S = oracle.gemm(wl.dtype, a_bits, b_bits, wl.M, wl.N, wl.K, wl.K, 1, b_rs, b_cs)
        else:
            C, S = oracle.batch_matmul(wl.dtype, a_bits, b_bits, wl.batch, wl.M, wl.N, wl.K, wl.M * wl.K, wl.K, 1,
                                       wl.K * wl.N, b_rs, b_cs)
    if wl.fused:
        C, S = oracle.epilogue(C, S, bias=wl.bias_values(), relu=wl.ep_relu, scale=wl.ep_scale)
    return C, S


def check_workload(wl, oracle, what=None):
    a_bits, b_bits = wl.operands()
    got = run_gpu(wl, a_bits, b_bits)
    ref, S = run_oracle(wl, a_bits, b_bits, oracle)
    return assert_close(got, ref, S, what or wl.name)


def variant_name(B, wl):
    """Name of the variant the library would launch for workload wl."""
    if wl.kind == "conv2d":
        return B.tir_conv2d_variant(wl.n, wl.h, wl.w, wl.c, wl.k, wl.r, wl.s, *wl.stride, *wl.pad, *wl.dil, wl.groups,
                                    wl.dtype, wl.out)
    b_rs, b_cs = (1, wl.K) if wl.trans_b else (wl.N, 1)
    return B.tir_gemm_variant(wl.batch if wl.kind == "bmm" else 1, wl.M, wl.N, wl.K, wl.K, 1, b_rs, b_cs, wl.N, 1,
                              wl.dtype, wl.out)

