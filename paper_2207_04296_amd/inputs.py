"""Seeded synthetic inputs and the workload table (no operator arithmetic lives here).

Both sides of every parity test draw their operands from this module: the CPU oracle reads the
raw bit arrays directly, the HIP path gets the same bits after a host-to-device copy.  The
generator is counter based (splitmix64 of ``seed`` and the element index), so any slice of a
tensor can be regenerated without the rest.

The paper evaluates operator instances taken from ResNet-50, MobileNet-v2, BERT and ViT
(section 5.1) but prints neither their shapes nor any data; the table below holds ResNet-50- and
BERT-base-shaped stand-ins filled with seeded random values.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

_MASK = np.uint64(0xFFFFFFFFFFFFFFFF)


def splitmix64(seed: int, n: int, offset: int = 0) -> np.ndarray:
    """n successive outputs of splitmix64 started at state seed + (offset+1)*gamma, as uint64."""
    gamma = 0x9E3779B97F4A7C15
    idx = np.arange(offset + 1, offset + n + 1, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + idx * np.uint64(gamma)) & _MASK
        z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _MASK
        z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _MASK
        z = z ^ (z >> np.uint64(31))
    return z


def _unit(seed: int, n: int, offset: int = 0) -> np.ndarray:
    """Uniform doubles in [0, 1) with 53 random bits."""
    return (splitmix64(seed, n, offset) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))


def uniform_pm1(seed: int, n: int) -> np.ndarray:
    """U(-1, 1) in fp64."""
    return 2.0 * _unit(seed, n) - 1.0


def normal(seed: int, n: int, scale: float = 1.0) -> np.ndarray:
    """N(0, scale^2) in fp64 by Box-Muller on two independent uniform streams."""
    u1 = 1.0 - _unit(seed, n)                       # (0, 1]
    u2 = _unit(seed ^ 0x5DEECE66D, n, offset=1 << 40)
    return scale * np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def int8_uniform(seed: int, n: int) -> np.ndarray:
    """Uniform integers in [-127, 127] as int8."""
    z = splitmix64(seed, n) >> np.uint64(32)
    return ((z * np.uint64(255)) >> np.uint64(32)).astype(np.int64).astype(np.int8) - np.int8(127)


def to_f16_bits(v: np.ndarray) -> np.ndarray:
    """Round fp64 values to IEEE binary16 (nearest even) and return the bit patterns."""
    return np.asarray(v, dtype=np.float64).astype(np.float16).view(np.uint16)


def to_bf16_bits(v: np.ndarray) -> np.ndarray:
    """Round fp64 values to bfloat16 (nearest even, via binary32) and return the bit patterns."""
    u = np.asarray(v, dtype=np.float64).astype(np.float32).view(np.uint32).astype(np.uint64)
    rounded = (u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))) >> np.uint64(16)
    return rounded.astype(np.uint16)


def make_tensor(dtype: str, dist: str, seed: int, shape) -> np.ndarray:
    """Raw bits of a seeded tensor: uint16 for 'f16'/'bf16', int8 for 'i8'.

    dist: 'u' = U(-1,1); 'n0.1' = N(0,1)*0.1; 'i' = uniform integers in [-127,127]
    (for float dtypes 'i' gives small integer values, handy for exact tests).
    """
    n = int(np.prod(shape)) if len(shape) else 1
    if dtype == "i8":
        return int8_uniform(seed, n).reshape(shape)
    if dist == "u":
        v = uniform_pm1(seed, n)
    elif dist == "n0.1":
        v = normal(seed, n, 0.1)
    elif dist == "i":
        v = (int8_uniform(seed, n).astype(np.float64) / 16.0).round()
    else:
        raise ValueError(f"unknown distribution {dist!r}")
    bits = to_f16_bits(v) if dtype == "f16" else to_bf16_bits(v)
    return bits.reshape(shape)


# ---------------------------------------------------------------------------------------------
# Workload table
# ---------------------------------------------------------------------------------------------

@dataclass(frozen=True)
class Workload:
    """One operator instance. kind: 'gemm' | 'bmm' | 'conv2d'."""
    name: str
    kind: str
    dtype: str            # 'f16' | 'bf16' | 'i8'
    out: str              # 'f32' | 'f16' | 'bf16' | 'i32' | 'i8' (requantised, needs ep_scale)
    dist: str
    seed: int
    # gemm / bmm: C[batch,M,N] = A[batch,M,K] . B[batch,K,N]; trans_b: B stored [batch,N,K]
    batch: int = 1
    M: int = 0
    N: int = 0
    K: int = 0
    trans_b: bool = False
    # conv2d (NHWC input, KRSC filter)
    n: int = 0
    h: int = 0
    w: int = 0
    c: int = 0
    k: int = 0
    r: int = 0
    s: int = 0
    stride: tuple = (1, 1)
    pad: tuple = (0, 0)
    dil: tuple = (1, 1)
    groups: int = 1
    # fused consumer: bias per output column / channel, ReLU, requantisation scale (int8 output)
    ep_bias: bool = False
    ep_relu: bool = False
    ep_scale: float = 0.0
    note: str = field(default="", compare=False)

    @property
    def fused(self) -> bool:
        return self.ep_bias or self.ep_relu or self.ep_scale != 0.0

    def out_cols(self) -> int:
        return self.k if self.kind == "conv2d" else self.N

    def bias_values(self):
        """Seeded bias, one per output column: float32 N(0,1)*0.1 for float inputs, int32 multiples of 64
        in [-8128, 8128] for int8 inputs; None without ep_bias."""
        if not self.ep_bias:
            return None
        n = self.out_cols()
        if self.dtype == "i8":
            return int8_uniform(self.seed + 2, n).astype(np.int32) * np.int32(64)
        return normal(self.seed + 2, n, 0.1).astype(np.float32)

    def out_hw(self):
        p = (self.h + 2 * self.pad[0] - self.dil[0] * (self.r - 1) - 1) // self.stride[0] + 1
        q = (self.w + 2 * self.pad[1] - self.dil[1] * (self.s - 1) - 1) // self.stride[1] + 1
        return p, q

    def gemm_view(self):
        """(batch_or_groups, M, N, K) of the contraction after fusing iterators."""
        if self.kind == "conv2d":
            p, q = self.out_hw()
            return self.groups, self.n * p * q, self.k // self.groups, self.r * self.s * (self.c // self.groups)
        return self.batch, self.M, self.N, self.K

    def flops(self) -> float:
        b, m, n, k = self.gemm_view()
        return 2.0 * b * m * n * k

    def min_bytes(self) -> float:
        """Compulsory traffic: each operand read once, the output written once."""
        isz = 1 if self.dtype == "i8" else 2
        osz = {"f32": 4, "i32": 4, "f16": 2, "bf16": 2, "i8": 1}[self.out]
        extra = 4 * self.out_cols() if self.ep_bias else 0
        if self.kind == "conv2d":
            p, q = self.out_hw()
            return (isz * (self.n * self.h * self.w * self.c + self.k * self.r * self.s * (self.c // self.groups))
                    + osz * self.n * p * q * self.k + extra)
        return isz * self.batch * (self.M * self.K + self.K * self.N) + osz * self.batch * self.M * self.N + extra

    def operands(self):
        """Raw-bit host operands (a, b) of this workload, seeded."""
        if self.kind == "conv2d":
            x = make_tensor(self.dtype, self.dist, self.seed, (self.n, self.h, self.w, self.c))
            wt = make_tensor(self.dtype, self.dist, self.seed + 1, (self.k, self.r, self.s, self.c // self.groups))
            return x, wt
        ashape = (self.batch, self.M, self.K) if self.kind == "bmm" else (self.M, self.K)
        bmat = (self.N, self.K) if self.trans_b else (self.K, self.N)
        bshape = (self.batch,) + bmat if self.kind == "bmm" else bmat
        return (make_tensor(self.dtype, self.dist, self.seed, ashape),
                make_tensor(self.dtype, self.dist, self.seed + 1, bshape))


def _cfgs():
    w = []
    w.append(Workload("c1_gemm128_f16", "gemm", "f16", "f32", "u", 1000, M=128, N=128, K=128))
    w.append(Workload("c2a_conv56x64_f16", "conv2d", "f16", "f16", "n0.1", 2000, n=16, h=56, w=56, c=64, k=64,
                      r=3, s=3, stride=(1, 1), pad=(1, 1)))
    w.append(Workload("c2b_conv28x128s2_f16", "conv2d", "f16", "f16", "n0.1", 2100, n=16, h=28, w=28, c=128,
                      k=256, r=3, s=3, stride=(2, 2), pad=(1, 1)))
    w.append(Workload("c3a_bmm_qkT_f16", "bmm", "f16", "f32", "u", 3000, batch=192, M=128, N=128, K=64,
                      trans_b=True, note="K stored [192,128,64], transposed by strides"))
    w.append(Workload("c3b_bmm_pv_f16", "bmm", "f16", "f32", "u", 3100, batch=192, M=128, N=64, K=128))
    for dt, sd in (("f16", 4000), ("bf16", 4200)):
        w.append(Workload(f"c4a_gemm4096_{dt}", "gemm", dt, "f32", "u", sd, M=4096, N=4096, K=4096))
        w.append(Workload(f"c4b_gemm_ffn_{dt}", "gemm", dt, "f32", "u", sd + 100, M=2048, N=3072, K=768))
    w.append(Workload("c5a_gemm2048_i8", "gemm", "i8", "i32", "i", 5000, M=2048, N=2048, K=2048))
    w.append(Workload("c5b_conv_g8d2_i8", "conv2d", "i8", "i32", "i", 5100, n=8, h=28, w=28, c=256, k=256,
                      r=3, s=3, stride=(1, 1), pad=(2, 2), dil=(2, 2), groups=8))
    return {x.name: x for x in w}


def _fused_cfgs():
    """The same operator instances with a fused consumer (bias + ReLU, down-cast, int8 requantisation):
    the output bytes, which dominate the attention matmuls and the int8 convolution, shrink."""
    import dataclasses
    base = _cfgs()
    w = [
        dataclasses.replace(base["c2a_conv56x64_f16"], name="c2a_conv56x64_f16_bias_relu", ep_bias=True, ep_relu=True),
        dataclasses.replace(base["c3a_bmm_qkT_f16"], name="c3a_bmm_qkT_f16_out16", out="f16"),
        dataclasses.replace(base["c3b_bmm_pv_f16"], name="c3b_bmm_pv_f16_out16", out="f16"),
        dataclasses.replace(base["c4b_gemm_ffn_f16"], name="c4b_gemm_ffn_f16_bias_relu_out16", out="f16", ep_bias=True,
                            ep_relu=True),
        dataclasses.replace(base["c5a_gemm2048_i8"], name="c5a_gemm2048_i8_requant", out="i8", ep_bias=True,
                            ep_scale=1.0 / 4000.0),
        dataclasses.replace(base["c5b_conv_g8d2_i8"], name="c5b_conv_g8d2_i8_relu_requant", out="i8", ep_bias=True,
                            ep_relu=True, ep_scale=1.0 / 1500.0),
    ]
    return {x.name: x for x in w}


def _more_cfgs():
    """Operators of the paper's evaluation set beyond the five benchmark configurations that fit the 2-D
    convolution entry point: the depth-wise convolution of a MobileNet-style block (groups = channels)."""
    w = [
        Workload("dep_conv56x128_f16", "conv2d", "f16", "f16", "n0.1", 6000, n=16, h=56, w=56, c=128, k=128, r=3, s=3,
                 stride=(1, 1), pad=(1, 1), groups=128),
        Workload("dep_conv112x32s2_i8_requant", "conv2d", "i8", "i8", "i", 6100, n=16, h=112, w=112, c=32, k=32, r=3, s=3,
                 stride=(2, 2), pad=(1, 1), groups=32, ep_bias=True, ep_relu=True, ep_scale=1.0 / 400.0),
    ]
    return {x.name: x for x in w}


WORKLOADS = _cfgs()
FUSED_WORKLOADS = _fused_cfgs()
MORE_WORKLOADS = _more_cfgs()
