"""tir_gemm_split_static (the entry point for callers that cannot allocate: its scratch is a static device array)
against tir_gemm_fused, the existing entry point it is a variant of, and against the oracle: two calls in a row
through the C ABI, the second on a smaller input, so that the scratch the first call left behind (partial sums of
more tiles and slices, counters) is what the second one starts from."""
import sys

import numpy as np
import pytest

from paper_2207_04296_amd import inputs as I
from tests import parity as PT

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def _fill(t):
    import torch
    t.fill_(float("nan")) if t.dtype.is_floating_point else t.fill_(-77 if t.dtype == torch.int8 else -123456789)


@pytest.mark.parametrize("dtype,out,fused", [("f16", "f32", False), ("bf16", "bf16", True), ("i8", "i32", False), ("i8", "i8", True)])
def test_split_static_matches_the_allocating_entry_point_twice_in_a_row(oracle, dtype, out, fused):
    import torch
    assert torch.cuda.is_available(), "GPU tests need a ROCm device"
    from paper_2207_04296_amd import binding as B
    B.lib()
    dist = "i" if dtype == "i8" else "u"
    # (M, N, K, slices): several ragged tiles and a K tail first, then a smaller problem with fewer slices
    for step, (M, N, K, slices) in enumerate([(200, 176, 4112, 5), (96, 80, 1024, 2)]):
        kw = dict(ep_bias=True, ep_relu=True, **({"ep_scale": 1.0 / 4000.0} if out == "i8" else {})) if fused else {}
        wl = I.Workload(f"static_split_{dtype}_{out}_{M}x{N}x{K}", "gemm", dtype, out, dist, 9300 + step, M=M, N=N, K=K, trans_b=True, **kw)
        a_bits, b_bits = wl.operands()
        ref, S = PT.run_oracle(wl, a_bits, b_bits, oracle)
        a, b = B.to_device(a_bits, dtype), B.to_device(b_bits, dtype)
        bias = B.bias_to_device(wl)
        ep = B.make_epilogue(bias if wl.ep_bias else None, wl.ep_relu, wl.ep_scale)
        c_static, c_plain = B.empty_out((M, N), out), B.empty_out((M, N), out)
        _fill(c_static); _fill(c_plain)
        _say(f"{wl.name}: tir_gemm_split_static, {slices} slices (call {step + 1} of 2)")
        B.tir_gemm_split_static(a, b, c_static, M, N, K, K, 1, 1, K, N, 1, dtype, out, ep, slices)
        _say(f"{wl.name}: tir_gemm_fused")
        B.tir_gemm_fused(a, b, c_plain, M, N, K, K, 1, 1, K, N, 1, dtype, out, ep)
        torch.cuda.synchronize()
        got, plain = PT.gpu_to_f64(c_static), PT.gpu_to_f64(c_plain)
        PT.assert_close(got, ref, S, f"{wl.name} on the static scratch vs the oracle")
        if S is None:
            assert np.array_equal(got, plain), f"{wl.name}: integer results differ from tir_gemm_fused"
        else:
            # both are within the tolerance of the exact result; against each other they differ by summation order only
            assert np.all(np.abs(got - plain) <= 2 * (PT.RTOL_S * S + PT.ATOL)), wl.name
        # the same call again gives the same bits: the sum does not depend on arrival order, the counters were reset
        c_again = B.empty_out((M, N), out)
        _fill(c_again)
        B.tir_gemm_split_static(a, b, c_again, M, N, K, K, 1, 1, K, N, 1, dtype, out, ep, slices)
        torch.cuda.synchronize()
        assert np.array_equal(PT.gpu_to_f64(c_again), got), f"{wl.name}: two identical calls differ"
