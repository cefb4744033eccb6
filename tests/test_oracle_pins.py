"""Pins for the CPU oracle: each checks it against something other than itself.

The paper prints no numeric worked example for these operators, so the pins are bit-pattern
decodes by numpy, per-element brute force with differently structured code, algebraic identities,
closed forms, the conv == im2col-GEMM rewrite of section 4.2, and torch's fp64 CPU convolution as
an independent library routine.
"""
import itertools

import numpy as np
import pytest

from paper_2207_04296_amd import inputs as I


# ----------------------------------------------------------------------------- decoders
def test_decode_every_f16_pattern(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.decode("f16", bits)
    want = bits.view(np.float16).astype(np.float64)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    m = ~np.isnan(want)
    assert np.array_equal(got[m], want[m])
    assert np.array_equal(np.signbit(got[m]), np.signbit(want[m]))


def test_decode_every_bf16_pattern(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.decode("bf16", bits)
    with np.errstate(invalid="ignore"):
        want = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    m = ~np.isnan(want)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(got[m], want[m])


def test_decode_int8(oracle):
    bits = np.arange(-128, 128, dtype=np.int8)
    assert np.array_equal(oracle.decode("i8", bits), np.arange(-128, 128, dtype=np.float64))


def test_known_f16_values(oracle):
    # values fixed by IEEE 754 binary16: 1.0, -2.0, 65504 (max), 2^-24 (min subnormal), 2^-14 (min normal)
    bits = np.array([0x3C00, 0xC000, 0x7BFF, 0x0001, 0x0400, 0x3555], dtype=np.uint16)
    want = [1.0, -2.0, 65504.0, 2.0 ** -24, 2.0 ** -14, 0.333251953125]
    assert oracle.decode("f16", bits).tolist() == want


# ----------------------------------------------------------------------------- helpers
def _vals(dtype, bits):
    """Independent decode through numpy (not through the oracle)."""
    if dtype == "i8":
        return bits.astype(np.int64)
    if dtype == "f16":
        return bits.view(np.float16).astype(np.float64)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _brute_gemm(a, b):
    """Per-element gather: one Python-level dot product per output element."""
    M, K = a.shape
    N = b.shape[1]
    out = np.zeros((M, N), dtype=a.dtype)
    for i, j in itertools.product(range(M), range(N)):
        out[i, j] = sum(a[i, k] * b[k, j] for k in range(K))
    return out


def _brute_conv(x, w, stride, pad, dil, groups):
    """Scatter formulation (loops over input pixels and taps, adds into the outputs they touch):
    structurally different from the oracle's gather loops."""
    N, H, W, C = x.shape
    K, R, S, Cg = w.shape
    P = (H + 2 * pad[0] - dil[0] * (R - 1) - 1) // stride[0] + 1
    Q = (W + 2 * pad[1] - dil[1] * (S - 1) - 1) // stride[1] + 1
    Kg = K // groups
    y = np.zeros((N, P, Q, K), dtype=x.dtype)
    for n, ih, iw, r, s in itertools.product(range(N), range(H), range(W), range(R), range(S)):
        ph = ih + pad[0] - r * dil[0]
        qw = iw + pad[1] - s * dil[1]
        if ph < 0 or qw < 0 or ph % stride[0] or qw % stride[1]:
            continue
        p, q = ph // stride[0], qw // stride[1]
        if p >= P or q >= Q:
            continue
        for k in range(K):
            g = k // Kg
            y[n, p, q, k] += np.dot(x[n, ih, iw, g * Cg:(g + 1) * Cg], w[k, r, s, :])
    return y


# ----------------------------------------------------------------------------- GEMM pins
@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (2, 3, 4), (5, 4, 3), (3, 5, 5), (4, 1, 5)])
def test_gemm_brute_force_tiny(oracle, dtype, M, N, K):
    A = I.make_tensor(dtype, "u", 11 + M, (M, K))
    B = I.make_tensor(dtype, "u", 12 + N, (K, N))
    C, S = oracle.gemm(dtype, A, B, M, N, K, K, 1, N, 1)
    a, b = _vals(dtype, A), _vals(dtype, B)
    want = _brute_gemm(a, b)
    if dtype == "i8":
        assert np.array_equal(C, want)
    else:
        np.testing.assert_allclose(C, want, rtol=0, atol=1e-13)
        np.testing.assert_allclose(S, _brute_gemm(np.abs(a), np.abs(b)), rtol=0, atol=1e-13)


@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
def test_gemm_strides_transposed_operands(oracle, dtype):
    # A stored as [K,M] and B stored as [N,K], addressed through strides; non-square so a
    # transposed-operand mistake changes the answer (or the shape).
    M, N, K = 4, 5, 3
    At = I.make_tensor(dtype, "u", 21, (K, M))
    Bt = I.make_tensor(dtype, "u", 22, (N, K))
    C, _ = oracle.gemm(dtype, At, Bt, M, N, K, 1, M, 1, K)
    want = _brute_gemm(_vals(dtype, At).T.copy(), _vals(dtype, Bt).T.copy())
    if dtype == "i8":
        assert np.array_equal(C, want)
    else:
        np.testing.assert_allclose(C, want, rtol=0, atol=1e-13)


@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
def test_gemm_identity(oracle, dtype):
    n = 17
    A = I.make_tensor(dtype, "u", 31, (n, n))
    one = {"f16": 0x3C00, "bf16": 0x3F80}.get(dtype, 1)
    eye = np.zeros((n, n), dtype=A.dtype)
    eye[np.arange(n), np.arange(n)] = one
    C1, _ = oracle.gemm(dtype, A, eye, n, n, n, n, 1, n, 1)
    C2, _ = oracle.gemm(dtype, eye, A, n, n, n, n, 1, n, 1)
    assert np.array_equal(C1, _vals(dtype, A))
    assert np.array_equal(C2, _vals(dtype, A))


def test_gemm_closed_forms(oracle):
    # A = 1, B = 1  =>  C = K ; A[i,k] = i, B[k,j] = j  =>  C = K*i*j  (all exactly representable)
    M, N, K = 33, 20, 47
    ones_a = np.full((M, K), 0x3C00, dtype=np.uint16)
    ones_b = np.full((K, N), 0x3C00, dtype=np.uint16)
    C, S = oracle.gemm("f16", ones_a, ones_b, M, N, K, K, 1, N, 1)
    assert np.all(C == K) and np.all(S == K)
    a = np.repeat(np.arange(M, dtype=np.float64)[:, None], K, axis=1)
    b = np.repeat(np.arange(N, dtype=np.float64)[None, :], K, axis=0)
    C, _ = oracle.gemm("f16", I.to_f16_bits(a), I.to_f16_bits(b), M, N, K, K, 1, N, 1)
    assert np.array_equal(C, K * np.outer(np.arange(M), np.arange(N)))
    # int8 at the largest magnitude the workloads reach: 2048 * 127 * 127 fits in int32
    a8 = np.full((2, 2048), 127, dtype=np.int8)
    b8 = np.full((2048, 3), -127, dtype=np.int8)
    C, _ = oracle.gemm("i8", a8, b8, 2, 3, 2048, 2048, 1, 3, 1)
    assert np.all(C == -2048 * 127 * 127) and abs(int(C[0, 0])) < 2 ** 31


def test_gemm_k_zero_is_reduction_init(oracle):
    C, S = oracle.gemm("f16", np.zeros(0, np.uint16), np.zeros(0, np.uint16), 3, 4, 0, 0, 1, 4, 1)
    assert np.all(C == 0) and np.all(S == 0)


@pytest.mark.parametrize("dtype", ["f16", "i8"])
def test_gemm_linearity_in_each_input(oracle, dtype):
    # small-integer-valued operands: every intermediate is exact, so linearity must hold exactly
    M, N, K = 9, 7, 13
    rng = np.random.default_rng(5)

    def enc(v):
        return v.astype(np.int8) if dtype == "i8" else I.to_f16_bits(v.astype(np.float64))

    A1, A2 = rng.integers(-7, 8, (M, K)), rng.integers(-7, 8, (M, K))
    B1, B2 = rng.integers(-7, 8, (K, N)), rng.integers(-7, 8, (K, N))
    f = lambda a, b: oracle.gemm(dtype, enc(a), enc(b), M, N, K, K, 1, N, 1)[0]
    assert np.array_equal(f(3 * A1 + A2, B1), 3 * f(A1, B1) + f(A2, B1))
    assert np.array_equal(f(A1, 3 * B1 + B2), 3 * f(A1, B1) + f(A1, B2))


def test_gemm_matches_numpy_matmul_medium(oracle):
    # library routine as the second opinion at a size spanning many rows / columns
    M, N, K = 70, 50, 90
    A = I.make_tensor("f16", "u", 41, (M, K))
    B = I.make_tensor("f16", "u", 42, (K, N))
    C, S = oracle.gemm("f16", A, B, M, N, K, K, 1, N, 1)
    a, b = _vals("f16", A), _vals("f16", B)
    np.testing.assert_allclose(C, a @ b, rtol=0, atol=1e-12)
    np.testing.assert_allclose(S, np.abs(a) @ np.abs(b), rtol=1e-14, atol=0)


# ----------------------------------------------------------------------------- BMM pins
@pytest.mark.parametrize("dtype", ["f16", "i8"])
def test_bmm_is_loop_of_gemms_and_broadcast(oracle, dtype):
    Bn, M, N, K = 3, 4, 5, 6
    A = I.make_tensor(dtype, "u", 51, (Bn, M, K))
    B = I.make_tensor(dtype, "u", 52, (Bn, N, K))       # stored transposed, like K in Q.K^T
    C, S = oracle.batch_matmul(dtype, A, B, Bn, M, N, K, M * K, K, 1, N * K, 1, K)
    a, b = _vals(dtype, A), _vals(dtype, B)
    want = np.einsum("bik,bjk->bij", a, b)
    if dtype == "i8":
        assert np.array_equal(C, want)
    else:
        np.testing.assert_allclose(C, want, rtol=0, atol=1e-13)
        np.testing.assert_allclose(S, np.einsum("bik,bjk->bij", np.abs(a), np.abs(b)), rtol=0, atol=1e-13)
    # batch stride 0 on B: every batch multiplies by the first matrix
    C0, _ = oracle.batch_matmul(dtype, A, B, Bn, M, N, K, M * K, K, 1, 0, 1, K)
    want0 = np.einsum("bik,jk->bij", a, b[0])
    if dtype == "i8":
        assert np.array_equal(C0, want0)
    else:
        np.testing.assert_allclose(C0, want0, rtol=0, atol=1e-13)


# ----------------------------------------------------------------------------- conv pins
_CONV_CASES = [
    # N,H,W,C,K,R,S, stride, pad, dil, groups
    (1, 5, 5, 2, 2, 3, 3, (1, 1), (0, 0), (1, 1), 1),
    (2, 5, 4, 4, 4, 3, 2, (2, 1), (1, 2), (1, 1), 2),
    (1, 5, 5, 4, 4, 2, 2, (1, 2), (2, 0), (2, 2), 4),     # depth-wise, dilated
    (2, 4, 5, 3, 2, 3, 3, (2, 2), (1, 1), (1, 2), 1),
    (1, 3, 3, 2, 4, 1, 1, (1, 1), (0, 0), (1, 1), 2),
    (1, 5, 5, 2, 2, 3, 3, (1, 1), (2, 2), (2, 2), 1),
]


@pytest.mark.parametrize("dtype", ["f16", "bf16", "i8"])
@pytest.mark.parametrize("case", _CONV_CASES)
def test_conv_brute_force_scatter(oracle, dtype, case):
    N, H, W, C, K, R, S, stride, pad, dil, groups = case
    x = I.make_tensor(dtype, "u", 61, (N, H, W, C))
    w = I.make_tensor(dtype, "u", 62, (K, R, S, C // groups))
    y, Sabs = oracle.conv2d(dtype, x, w, stride, pad, dil, groups)
    xv, wv = _vals(dtype, x), _vals(dtype, w)
    want = _brute_conv(xv, wv, stride, pad, dil, groups)
    assert y.shape == want.shape
    if dtype == "i8":
        assert np.array_equal(y, want)
    else:
        np.testing.assert_allclose(y, want, rtol=0, atol=1e-13)
        np.testing.assert_allclose(Sabs, _brute_conv(np.abs(xv), np.abs(wv), stride, pad, dil, groups),
                                   rtol=0, atol=1e-13)


def _im2col(xv, R, S, stride, pad, dil):
    """A_t[fuse(n,h,w), fuse(rh,rw,rc)] of section 4.2, materialised (zero rows for padding)."""
    N, H, W, C = xv.shape
    P = (H + 2 * pad[0] - dil[0] * (R - 1) - 1) // stride[0] + 1
    Q = (W + 2 * pad[1] - dil[1] * (S - 1) - 1) // stride[1] + 1
    xp = np.zeros((N, H + 2 * pad[0], W + 2 * pad[1], C), dtype=xv.dtype)
    xp[:, pad[0]:pad[0] + H, pad[1]:pad[1] + W, :] = xv
    cols = np.zeros((N, P, Q, R, S, C), dtype=xv.dtype)
    for r in range(R):
        for s in range(S):
            cols[:, :, :, r, s, :] = xp[:, r * dil[0]: r * dil[0] + (P - 1) * stride[0] + 1: stride[0],
                                        s * dil[1]: s * dil[1] + (Q - 1) * stride[1] + 1: stride[1], :]
    return cols.reshape(N * P * Q, R * S * C), (N, P, Q)


@pytest.mark.parametrize("stride,pad,dil", [((1, 1), (1, 1), (1, 1)), ((2, 2), (1, 1), (1, 1)),
                                            ((1, 1), (2, 2), (2, 2)), ((2, 1), (0, 3), (1, 2))])
def test_conv_equals_im2col_gemm_exact_int(oracle, stride, pad, dil):
    # Section 4.2: C_t[fuse(n,h,w), co] += A_t[fuse(n,h,w), fuse(rh,rw,rc)] * B_t[fuse(rh,rw,rc), co].
    # The GEMM side also goes through the oracle's GEMM, so the two operators pin each other and
    # both are pinned to numpy by the integer matmul below.
    N, H, W, C, K, R, S = 2, 9, 8, 6, 5, 3, 3
    x = I.make_tensor("i8", "i", 71, (N, H, W, C))
    w = I.make_tensor("i8", "i", 72, (K, R, S, C))
    y, _ = oracle.conv2d("i8", x, w, stride, pad, dil, 1)
    At, (n, p, q) = _im2col(x.astype(np.int64), R, S, stride, pad, dil)
    Bt = w.astype(np.int64).reshape(K, R * S * C).T            # [fuse(rh,rw,rc), co]
    assert np.array_equal(y.reshape(n * p * q, K), At @ Bt)
    Kd = R * S * C
    Cg, _ = oracle.gemm("i8", At.astype(np.int8), w.reshape(K, Kd), n * p * q, K, Kd, Kd, 1, 1, Kd)
    assert np.array_equal(y.reshape(n * p * q, K), Cg)


def test_conv_1x1_is_gemm(oracle):
    N, H, W, C, K = 2, 4, 3, 8, 5
    x = I.make_tensor("f16", "u", 81, (N, H, W, C))
    w = I.make_tensor("f16", "u", 82, (K, 1, 1, C))
    y, S1 = oracle.conv2d("f16", x, w)
    Cg, S2 = oracle.gemm("f16", x, w, N * H * W, K, C, C, 1, 1, C)
    assert np.array_equal(y.reshape(-1, K), Cg)
    assert np.array_equal(S1.reshape(-1, K), S2)
    np.testing.assert_allclose(Cg, _vals("f16", x).reshape(-1, C) @ _vals("f16", w).reshape(K, C).T, atol=1e-13)


def test_conv_delta_input_shows_filter_footprint(oracle):
    # a single 1 at (ih, iw, c0): y[p,q,k] = w[k,r,s,c0] where p*s_h - pad + r*d_h = ih etc.
    H = W = 9
    C, K, R, S = 3, 2, 3, 3
    stride, pad, dil = (2, 1), (2, 2), (2, 1)
    ih, iw, c0 = 4, 5, 1
    x = np.zeros((1, H, W, C), dtype=np.int8)
    x[0, ih, iw, c0] = 1
    w = I.make_tensor("i8", "i", 91, (K, R, S, C))
    y, _ = oracle.conv2d("i8", x, w, stride, pad, dil, 1)
    want = np.zeros_like(y)
    P, Q = y.shape[1:3]
    for r in range(R):
        for s in range(S):
            ph, qw = ih + pad[0] - r * dil[0], iw + pad[1] - s * dil[1]
            if ph >= 0 and qw >= 0 and ph % stride[0] == 0 and qw % stride[1] == 0:
                p, q = ph // stride[0], qw // stride[1]
                if p < P and q < Q:
                    want[0, p, q, :] += w[:, r, s, c0]
    assert np.array_equal(y, want) and np.count_nonzero(want) > 0


def test_conv_all_ones_counts_valid_taps(oracle):
    # x = 1, w = 1: y = (C/G) * (#taps whose input coordinate is inside the image), a closed form
    # that separates rows and columns.
    N, H, W, C, K, R, S, groups = 1, 7, 6, 4, 4, 3, 3, 2
    stride, pad, dil = (1, 2), (2, 1), (2, 1)
    x = np.ones((N, H, W, C), dtype=np.int8)
    w = np.ones((K, R, S, C // groups), dtype=np.int8)
    y, _ = oracle.conv2d("i8", x, w, stride, pad, dil, groups)
    P, Q = y.shape[1:3]
    rows = np.array([sum(0 <= p * stride[0] - pad[0] + r * dil[0] < H for r in range(R)) for p in range(P)])
    cols = np.array([sum(0 <= q * stride[1] - pad[1] + s * dil[1] < W for s in range(S)) for q in range(Q)])
    want = (C // groups) * np.outer(rows, cols)
    for k in range(K):
        assert np.array_equal(y[0, :, :, k], want)
    assert want.max() == R * S * (C // groups) and want.min() < want.max()


def test_conv_groups_are_independent_convs(oracle):
    N, H, W, C, K, R, S, G = 2, 6, 6, 8, 6, 3, 3, 2
    x = I.make_tensor("f16", "u", 101, (N, H, W, C))
    w = I.make_tensor("f16", "u", 102, (K, R, S, C // G))
    y, _ = oracle.conv2d("f16", x, w, (1, 1), (1, 1), (1, 1), G)
    Cg, Kg = C // G, K // G
    for g in range(G):
        yg, _ = oracle.conv2d("f16", np.ascontiguousarray(x[..., g * Cg:(g + 1) * Cg]),
                              np.ascontiguousarray(w[g * Kg:(g + 1) * Kg]), (1, 1), (1, 1), (1, 1), 1)
        assert np.array_equal(y[..., g * Kg:(g + 1) * Kg], yg)


@pytest.mark.parametrize("case", [
    (2, 12, 11, 8, 6, 3, 3, (1, 1), (1, 1), (1, 1), 1),
    (2, 12, 11, 8, 6, 3, 3, (2, 2), (1, 1), (1, 1), 1),
    (1, 13, 12, 8, 8, 3, 3, (1, 1), (2, 2), (2, 2), 4),
    (1, 10, 9, 6, 6, 5, 3, (2, 1), (2, 1), (1, 2), 6),
    (3, 7, 7, 4, 10, 1, 1, (1, 1), (0, 0), (1, 1), 2),
])
def test_conv_matches_torch_fp64_library(oracle, case):
    torch = pytest.importorskip("torch")
    N, H, W, C, K, R, S, stride, pad, dil, groups = case
    x = I.make_tensor("f16", "n0.1", 111, (N, H, W, C))
    w = I.make_tensor("f16", "n0.1", 112, (K, R, S, C // groups))
    y, _ = oracle.conv2d("f16", x, w, stride, pad, dil, groups)
    xt = torch.from_numpy(_vals("f16", x)).permute(0, 3, 1, 2)              # NCHW
    wt = torch.from_numpy(_vals("f16", w)).permute(0, 3, 1, 2)              # K,C/g,R,S
    ref = torch.nn.functional.conv2d(xt, wt, None, stride, pad, dil, groups).permute(0, 2, 3, 1).numpy()
    assert y.shape == ref.shape
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-12)


def test_conv_out_extent_rule(oracle):
    assert oracle.conv_out_extent(56, 3, 1, 1, 1) == 56
    assert oracle.conv_out_extent(28, 3, 2, 1, 1) == 14
    assert oracle.conv_out_extent(28, 3, 1, 2, 2) == 28
    assert oracle.conv_out_extent(2, 3, 1, 0, 1) == 0          # filter does not fit
    assert oracle.conv_out_extent(7, 3, 2, 0, 1) == 3


def test_conv_linearity_in_each_input(oracle):
    rng = np.random.default_rng(9)
    shape_x, shape_w = (1, 6, 6, 4), (4, 3, 3, 2)
    X1, X2 = rng.integers(-5, 6, shape_x), rng.integers(-5, 6, shape_x)
    W1, W2 = rng.integers(-5, 6, shape_w), rng.integers(-5, 6, shape_w)
    enc = lambda v: I.to_f16_bits(v.astype(np.float64))
    f = lambda x, w: oracle.conv2d("f16", enc(x), enc(w), (1, 1), (1, 1), (2, 2), 2)[0]
    assert np.array_equal(f(2 * X1 + X2, W1), 2 * f(X1, W1) + f(X2, W1))
    assert np.array_equal(f(X1, 2 * W1 + W2), 2 * f(X1, W1) + f(X1, W2))


# ------------------------------------------------------------------------------ fused consumers
def test_epilogue_float_hand_worked(oracle):
    """bias add and ReLU on a result small enough to check by eye; S grows by |bias| (the bias is one
    more term of the sum the tolerance is expressed in)."""
    C = np.array([[1.5, -2.0], [0.0, -0.25]])
    S = np.array([[3.0, 2.0], [1.0, 0.5]])
    bias = np.array([0.5, -1.0], dtype=np.float32)
    out, S2 = oracle.epilogue(C, S, bias=bias)
    assert out.tolist() == [[2.0, -3.0], [0.5, -1.25]]
    assert S2.tolist() == [[3.5, 3.0], [1.5, 1.5]]
    out, S2 = oracle.epilogue(C, S, bias=bias, relu=True)
    assert out.tolist() == [[2.0, 0.0], [0.5, 0.0]]
    out, S2 = oracle.epilogue(C, S, relu=True)
    assert out.tolist() == [[1.5, 0.0], [0.0, 0.0]] and S2.tolist() == S.tolist()
    out, _ = oracle.epilogue(C, None)
    assert out.tolist() == C.tolist() and out is not C
    # the bias is applied per output column of an N-d result (last axis)
    y = np.zeros((2, 3, 4, 2))
    out, _ = oracle.epilogue(y, None, bias=bias)
    assert np.all(out[..., 0] == 0.5) and np.all(out[..., 1] == -1.0)


def test_epilogue_int_hand_worked(oracle):
    """Requantisation: ties go to the even code, both signs, saturation at -128 / 127, ReLU comes
    before the scaling, the bias before the ReLU."""
    t = np.array([[1, 3, 5, -1, -3, 1000, -1000, 0]], dtype=np.int64)
    q, _ = oracle.epilogue(t, None, scale=0.5)
    assert q.tolist() == [[0, 2, 2, 0, -2, 127, -128, 0]]
    q, _ = oracle.epilogue(t, None, relu=True, scale=0.5)
    assert q.tolist() == [[0, 2, 2, 0, 0, 127, 0, 0]]
    bias = np.array([2, -2, 0, 1, 3, 0, 0, -7], dtype=np.int32)
    q, _ = oracle.epilogue(t, None, bias=bias)
    assert q.tolist() == [[3, 1, 5, 0, 0, 1000, -1000, -7]]
    q, _ = oracle.epilogue(t, None, bias=bias, relu=True, scale=1.0)
    assert q.tolist() == [[3, 1, 5, 0, 0, 127, 0, 0]]
    # the scaling is a binary32 product: 25 * 0.1f rounds to 2.5 exactly (-> 2), in binary64 it would be
    # 2.50000003... (-> 3)
    q, _ = oracle.epilogue(np.array([[25, 35]], dtype=np.int64), None, scale=float(np.float32(0.1)))
    assert q.tolist() == [[2, 4]]
    with pytest.raises(RuntimeError):
        oracle.epilogue(np.array([[2 ** 31 - 1]], dtype=np.int64), None, bias=np.array([1], dtype=np.int32))
    with pytest.raises(RuntimeError):
        oracle.epilogue(t, None, scale=-1.0)
    with pytest.raises(RuntimeError):
        oracle.epilogue(t, None, scale=float("inf"))


@pytest.mark.parametrize("scale", [0.0123, 1.0 / 3.0, 0.5, 2.0, 7.3e-4])
def test_epilogue_int_matches_numpy_float32(oracle, scale):
    """The same definition carried out by numpy: int32 -> float32, one float32 product, rint (ties to
    even), clip.  Values spread over both the linear and the saturated range."""
    rng = np.random.default_rng(int(scale * 1e6) + 5)
    span = int(min(2 ** 31 - 1, 400.0 / scale))
    t = rng.integers(-span, span, size=(37, 53), dtype=np.int64)
    bias = rng.integers(-1000, 1000, size=53).astype(np.int32)
    for relu in (False, True):
        got, _ = oracle.epilogue(t, None, bias=bias, relu=relu, scale=scale)
        u = t + bias.astype(np.int64)
        if relu:
            u = np.maximum(u, 0)
        f = u.astype(np.int32).astype(np.float32) * np.float32(scale)
        want = np.clip(np.rint(f), -128, 127).astype(np.int64)
        assert np.array_equal(got, want)
        assert got.min() == (-128 if not relu else 0) and got.max() == 127      # both regimes were exercised


# ------------------------------------------------------------------------------ attention head
def _f16(v):
    return I.to_f16_bits(np.asarray(v, dtype=np.float64))


def _dec16(bits):
    return bits.view(np.float16).astype(np.float64)


def test_attention_closed_forms(oracle):
    rng = np.random.default_rng(42)
    b, M, N, d, dv = 2, 5, 7, 8, 6
    V = _f16(rng.uniform(-1, 1, (b, N, dv)))
    K = _f16(rng.uniform(-1, 1, (b, N, d)))
    # Q = 0: every score is 0, the probabilities are uniform, the output is the mean of V's rows
    O, T = oracle.attention("f16", _f16(np.zeros((b, M, d))), K, V, 0.37)
    assert np.allclose(O, np.broadcast_to(_dec16(V).mean(axis=1, keepdims=True), O.shape), rtol=0, atol=1e-15)
    assert np.allclose(T, np.broadcast_to(np.abs(_dec16(V)).mean(axis=1, keepdims=True), T.shape), rtol=0, atol=1e-15)
    # a single key: the output is that key's value row, whatever the scores
    O1, _ = oracle.attention("f16", _f16(rng.uniform(-1, 1, (b, M, d))), K[:, :1], V[:, :1], 3.0)
    assert np.array_equal(O1, np.broadcast_to(_dec16(V[:, :1]), O1.shape))
    # one dominant key: queries equal to key 3 times a large scale pick value row 3
    Kd = np.zeros((1, N, d)); Kd[0, np.arange(N), np.arange(N)] = 1.0      # orthonormal keys
    Qd = np.zeros((1, 2, d)); Qd[0, 0, 3] = 1.0; Qd[0, 1, 5] = 1.0
    Od, _ = oracle.attention("f16", _f16(Qd), _f16(Kd), V[:1], 2000.0)
    assert np.allclose(Od[0, 0], _dec16(V)[0, 3], rtol=0, atol=1e-300) and np.allclose(Od[0, 1], _dec16(V)[0, 5], rtol=0, atol=1e-300)
    # two keys, scores 0 and ln 3 apart: probabilities 1/4 and 3/4
    K2 = np.zeros((1, 2, 2)); K2[0, 1, 0] = 1.0
    Q2 = np.zeros((1, 1, 2)); Q2[0, 0, 0] = 1.0
    V2 = np.array([[[8.0], [-4.0]]])
    O2, T2 = oracle.attention("f16", _f16(Q2), _f16(K2), _f16(V2), float(np.log(3.0)))
    assert abs(O2[0, 0, 0] - (0.25 * 8.0 + 0.75 * -4.0)) < 1e-14 and abs(T2[0, 0, 0] - (0.25 * 8.0 + 0.75 * 4.0)) < 1e-14


def test_attention_invariances(oracle):
    rng = np.random.default_rng(7)
    b, M, N, d, dv = 3, 9, 11, 16, 5
    Q = _f16(rng.uniform(-1, 1, (b, M, d))); K = _f16(rng.uniform(-1, 1, (b, N, d))); V = _f16(rng.uniform(-1, 1, (b, N, dv)))
    O, T = oracle.attention("f16", Q, K, V, 0.25)
    # the keys are a set: permuting keys and values together changes nothing (up to fp64 summation order)
    perm = rng.permutation(N)
    Op, Tp = oracle.attention("f16", Q, K[:, perm], V[:, perm], 0.25)
    assert np.allclose(O, Op, rtol=0, atol=1e-14) and np.allclose(T, Tp, rtol=0, atol=1e-14)
    # batches and query rows are independent
    O1, _ = oracle.attention("f16", Q[1:2, 2:5], K[1:2], V[1:2], 0.25)
    assert np.array_equal(O1[0], O[1, 2:5])
    # the output is a convex combination of value rows: inside their range, and T >= |O|
    vdec = _dec16(V)
    assert np.all(O <= vdec.max(axis=1, keepdims=True) + 1e-15) and np.all(O >= vdec.min(axis=1, keepdims=True) - 1e-15)
    assert np.all(T + 1e-15 >= np.abs(O))
    # scale 0 is uniform attention again
    O0, _ = oracle.attention("f16", Q, K, V, 0.0)
    assert np.allclose(O0, np.broadcast_to(vdec.mean(axis=1, keepdims=True), O0.shape), rtol=0, atol=1e-15)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_attention_matches_library_softmax_between_matmuls(oracle, dtype):
    """scipy's softmax between two numpy matmuls in fp64 (library routines, a different arrangement of
    the same definition), on shapes like one BERT head and on ragged ones."""
    from scipy.special import softmax
    for (b, M, N, d, dv, scale, seed) in [(2, 128, 128, 64, 64, 0.125, 1), (3, 17, 29, 24, 40, 0.3, 2), (1, 1, 300, 8, 8, 1.7, 3)]:
        Q = I.make_tensor(dtype, "u", 100 + seed, (b, M, d)); K = I.make_tensor(dtype, "u", 200 + seed, (b, N, d))
        V = I.make_tensor(dtype, "u", 300 + seed, (b, N, dv))
        q, k, v = oracle.decode(dtype, Q), oracle.decode(dtype, K), oracle.decode(dtype, V)
        P = softmax(scale * np.einsum("bic,bjc->bij", q, k), axis=-1)
        O, T = oracle.attention(dtype, Q, K, V, scale)
        assert np.allclose(O, P @ v, rtol=0, atol=1e-13)
        assert np.allclose(T, P @ np.abs(v), rtol=0, atol=1e-13)
        assert np.allclose(P.sum(axis=-1), 1.0, rtol=0, atol=1e-14)


# ------------------------------------------------------------------------------ conv1d / conv3d / transposed conv2d
def _smallint_bits(rng, shape):
    """fp16 bits of small integers: every product and sum below is exact in fp64."""
    return I.to_f16_bits(rng.integers(-3, 4, size=shape).astype(np.float64))


def test_conv1d_is_numpy_correlate_and_conv2d_with_unit_height(oracle):
    rng = np.random.default_rng(11)
    # one channel, one filter, no padding: numpy's own cross-correlation
    x = _smallint_bits(rng, (1, 40, 1)); w = _smallint_bits(rng, (1, 5, 1))
    y, _ = oracle.conv1d("f16", x, w)
    assert np.array_equal(y[0, :, 0], np.correlate(_dec16(x)[0, :, 0], _dec16(w)[0, :, 0], mode="valid"))
    # general case: the same numbers as the 2-D operator on an image of height 1
    for (stride, pad, dil, groups) in [(1, 0, 1, 1), (2, 3, 1, 2), (1, 2, 2, 4), (3, 1, 3, 1)]:
        x = _smallint_bits(rng, (2, 23, 8)); w = _smallint_bits(rng, (12, 3, 8 // groups))
        y, S = oracle.conv1d("f16", x, w, stride, pad, dil, groups)
        y2, S2 = oracle.conv2d("f16", x[:, None], w[:, None], (1, stride), (0, pad), (1, dil), groups)
        assert np.array_equal(y, y2[:, 0]) and np.array_equal(S, S2[:, 0])
    xi = rng.integers(-127, 128, size=(2, 17, 4)).astype(np.int8); wi = rng.integers(-127, 128, size=(6, 4, 2)).astype(np.int8)
    yi, _ = oracle.conv1d("i8", xi, wi, 2, 1, 1, 2)
    yi2, _ = oracle.conv2d("i8", xi[:, None], wi[:, None], (1, 2), (0, 1), (1, 1), 2)
    assert np.array_equal(yi, yi2[:, 0])


def test_conv3d_reduces_to_conv2d_and_to_a_sum_over_depth_taps(oracle):
    rng = np.random.default_rng(12)
    # depth 1, one depth tap: the 2-D operator
    x = _smallint_bits(rng, (2, 1, 9, 8, 6)); w = _smallint_bits(rng, (4, 1, 3, 2, 3))
    y, S = oracle.conv3d("f16", x, w, (1, 2, 1), (0, 1, 1), (1, 1, 2), 2)
    y2, S2 = oracle.conv2d("f16", x[:, 0], w[:, 0], (2, 1), (1, 1), (1, 2), 2)
    assert np.array_equal(y[:, 0], y2) and np.array_equal(S[:, 0], S2)
    # general: output depth o is the sum over depth taps t of 2-D convolutions of input slice o*s - pad + t*d
    N, D, H, W, C, K, T, R, S_ = 1, 7, 6, 5, 4, 6, 3, 2, 3
    sd, pd, dd = 2, 1, 2
    x = _smallint_bits(rng, (N, D, H, W, C)); w = _smallint_bits(rng, (K, T, R, S_, C))
    y, _ = oracle.conv3d("f16", x, w, (sd, 1, 2), (pd, 1, 0), (dd, 1, 1))
    OD = oracle.conv_out_extent(D, T, sd, pd, dd)
    assert y.shape[1] == OD == 3
    for o in range(OD):
        acc = 0.0
        for t in range(T):
            i_d = o * sd - pd + t * dd
            if 0 <= i_d < D:
                acc = acc + oracle.conv2d("f16", x[:, i_d], w[:, t], (1, 2), (1, 0), (1, 1))[0]
        assert np.array_equal(y[:, o], acc)


@pytest.mark.parametrize("case", [((1, 1, 1), (0, 0, 0), (1, 1, 1), 1), ((2, 1, 2), (1, 0, 2), (1, 2, 1), 1), ((1, 2, 1), (1, 1, 1), (2, 1, 1), 2)])
def test_conv3d_matches_torch_fp64_library(oracle, case):
    import torch
    stride, pad, dil, groups = case
    rng = np.random.default_rng(13)
    xb = I.make_tensor("f16", "u", 31, (2, 6, 7, 8, 4)); wb = I.make_tensor("f16", "u", 32, (6, 3, 2, 3, 4 // groups))
    y, _ = oracle.conv3d("f16", xb, wb, stride, pad, dil, groups)
    xt = torch.from_numpy(_dec16(xb)).permute(0, 4, 1, 2, 3); wt = torch.from_numpy(_dec16(wb)).permute(0, 4, 1, 2, 3)
    ref = torch.nn.functional.conv3d(xt, wt, None, stride, pad, dil, groups).permute(0, 2, 3, 4, 1).numpy()
    assert np.allclose(y, ref, rtol=0, atol=1e-12)


def test_conv2d_transpose_is_the_adjoint_of_conv2d(oracle):
    """<conv2d(x, w), y> == <x, conv2d_transpose(y, w^T)> for every x and y (exact on small integers), where w^T swaps
    the roles of the filter's channel axes; with it the transposed operator is pinned to the forward one."""
    rng = np.random.default_rng(14)
    for (stride, pad, dil, groups, H, W) in [((1, 1), (0, 0), (1, 1), 1, 6, 7), ((2, 2), (1, 1), (1, 1), 1, 9, 8), ((2, 3), (1, 0), (2, 1), 2, 11, 10),
                                              ((3, 1), (2, 1), (1, 2), 1, 10, 7)]:
        N, C, K, R, S_ = 2, 4, 6, 3, 2
        Cg, Kg = C // groups, K // groups
        xb = _smallint_bits(rng, (N, H, W, C)); wb = _smallint_bits(rng, (K, R, S_, Cg))
        fwd, _ = oracle.conv2d("f16", xb, wb, stride, pad, dil, groups)                    # [N,P,Q,K]
        P, Q = fwd.shape[1:3]
        yb = _smallint_bits(rng, (N, P, Q, K))
        # transposed filter: output channels of the adjoint are the forward input channels, group by group
        wf = _dec16(wb).reshape(groups, Kg, R, S_, Cg)
        wT = I.to_f16_bits(np.ascontiguousarray(wf.transpose(0, 4, 2, 3, 1)).reshape(C, R, S_, Kg))
        outpad = ((H + 2 * pad[0] - dil[0] * (R - 1) - 1) % stride[0], (W + 2 * pad[1] - dil[1] * (S_ - 1) - 1) % stride[1])
        back, _ = oracle.conv2d_transpose("f16", yb, wT, stride, pad, dil, outpad, groups)   # [N,H,W,C]
        assert back.shape == (N, H, W, C)
        assert np.sum(fwd * _dec16(yb)) == np.sum(_dec16(xb) * back)


@pytest.mark.parametrize("case", [((1, 1), (0, 0), (1, 1), (0, 0), 1), ((2, 2), (1, 1), (1, 1), (1, 1), 1), ((3, 2), (0, 2), (2, 1), (2, 0), 2)])
def test_conv2d_transpose_matches_torch_fp64_library(oracle, case):
    import torch
    stride, pad, dil, outpad, groups = case
    N, H, W, C, K, R, S_ = 2, 5, 6, 4, 6, 3, 2
    xb = I.make_tensor("f16", "u", 41, (N, H, W, C)); wb = I.make_tensor("f16", "u", 42, (K, R, S_, C // groups))
    y, S = oracle.conv2d_transpose("f16", xb, wb, stride, pad, dil, outpad, groups)
    # torch's layout: input [N,C,H,W], weight [C_in, C_out/groups, R, S]
    Cg, Kg = C // groups, K // groups
    wt = _dec16(wb).reshape(groups, Kg, R, S_, Cg).transpose(0, 4, 1, 2, 3).reshape(C, Kg, R, S_)
    ref = torch.nn.functional.conv_transpose2d(torch.from_numpy(_dec16(xb)).permute(0, 3, 1, 2), torch.from_numpy(np.ascontiguousarray(wt)),
                                               None, stride, pad, outpad, groups, dil).permute(0, 2, 3, 1).numpy()
    assert y.shape == ref.shape and np.allclose(y, ref, rtol=0, atol=1e-12)
    assert np.all(S + 1e-12 >= np.abs(y))
    # a single 1 in the input stamps the filter (times nothing else) into the output at stride spacing
    xd = np.zeros((1, H, W, C)); xd[0, 2, 3, 1] = 1.0
    yd, _ = oracle.conv2d_transpose("f16", I.to_f16_bits(xd), wb, stride, pad, dil, outpad, groups)
    g = 1 // Cg
    for r in range(R):
        for s in range(S_):
            oh, ow = 2 * stride[0] - pad[0] + r * dil[0], 3 * stride[1] - pad[1] + s * dil[1]
            if 0 <= oh < yd.shape[1] and 0 <= ow < yd.shape[2]:
                assert np.array_equal(yd[0, oh, ow, g * Kg:(g + 1) * Kg], _dec16(wb)[g * Kg:(g + 1) * Kg, r, s, 1 % Cg])
    assert np.count_nonzero(yd) <= R * S_ * Kg


# ------------------------------------------------------------------------------ int8 branches and S of the later convolution forms
def _brute_conv3d(x, w, stride, pad, dil, groups):
    """Per-output-element gather for the 3-D convolution (definition of sec. 5.1's C3D with the readings of
    the 2-D operator), on decoded values; index lists are built per element, nothing is shared with the oracle's loops."""
    N, D, H, W, C = x.shape
    K, T, R, S_, Cg = w.shape
    Kg = K // groups
    ext = [(i + 2 * p - d * (f - 1) - 1) // s + 1 for i, f, s, p, d in zip((D, H, W), (T, R, S_), stride, pad, dil)]
    y = np.zeros((N, *ext, K), dtype=x.dtype)
    for n, o, p, q, k in itertools.product(range(N), range(ext[0]), range(ext[1]), range(ext[2]), range(K)):
        g = k // Kg
        terms = []
        for t, r, s in itertools.product(range(T), range(R), range(S_)):
            i_d, ih, iw = (o * stride[0] - pad[0] + t * dil[0], p * stride[1] - pad[1] + r * dil[1], q * stride[2] - pad[2] + s * dil[2])
            if 0 <= i_d < D and 0 <= ih < H and 0 <= iw < W:
                terms.append(np.dot(x[n, i_d, ih, iw, g * Cg:(g + 1) * Cg], w[k, t, r, s]))
        y[n, o, p, q, k] = sum(terms)
    return y


def _brute_conv2d_transpose_gather(x, w, stride, pad, dil, outpad, groups):
    """The transposed convolution read as a GATHER (the oracle writes the scatter): output pixel (oh, ow) collects
    x[(oh + pad - r*dil) / stride] * w[r] for the taps where the division is exact and the quotient is an input pixel."""
    N, H, W, C = x.shape
    K, R, S_, Cg = w.shape
    Kg = K // groups
    P = (H - 1) * stride[0] - 2 * pad[0] + dil[0] * (R - 1) + outpad[0] + 1
    Q = (W - 1) * stride[1] - 2 * pad[1] + dil[1] * (S_ - 1) + outpad[1] + 1
    y = np.zeros((N, P, Q, K), dtype=x.dtype)
    for n, oh, ow, k in itertools.product(range(N), range(P), range(Q), range(K)):
        g = k // Kg
        acc = 0
        for r, s in itertools.product(range(R), range(S_)):
            nh, nw = oh + pad[0] - r * dil[0], ow + pad[1] - s * dil[1]
            if nh % stride[0] or nw % stride[1]:
                continue
            ih, iw = nh // stride[0], nw // stride[1]
            if 0 <= ih < H and 0 <= iw < W:
                acc = acc + np.dot(x[n, ih, iw, g * Cg:(g + 1) * Cg], w[k, r, s])
        y[n, oh, ow, k] = acc
    return y


_C3D_CASES = [((1, 1, 1), (0, 0, 0), (1, 1, 1), 1), ((2, 1, 2), (1, 0, 1), (1, 2, 1), 2), ((1, 2, 1), (1, 1, 2), (2, 1, 1), 4)]
_T2D_CASES = [((1, 1), (0, 0), (1, 1), (0, 0), 1), ((2, 2), (1, 1), (1, 1), (1, 0), 2), ((3, 2), (0, 2), (2, 1), (2, 1), 1), ((2, 3), (2, 0), (1, 2), (0, 2), 4)]


@pytest.mark.parametrize("case", _C3D_CASES)
def test_conv3d_int8_matches_brute_force_gather(oracle, case):
    """The int8 branch of the 3-D convolution has its own multiply-add line: full-range int8 data (so that a doubled
    or dropped product, a sign-extension slip or a narrow accumulator shows) against the per-element gather."""
    stride, pad, dil, groups = case
    rng = np.random.default_rng(101)
    x = rng.integers(-127, 128, size=(2, 4, 5, 4, 4)).astype(np.int8)
    w = rng.integers(-127, 128, size=(4, 2, 3, 2, 4 // groups)).astype(np.int8)
    y, S = oracle.conv3d("i8", x, w, stride, pad, dil, groups)
    assert S is None and y.dtype == np.int64
    assert np.array_equal(y, _brute_conv3d(x.astype(np.int64), w.astype(np.int64), stride, pad, dil, groups))


def test_conv3d_int8_is_a_sum_over_depth_taps_of_int8_conv2d(oracle):
    rng = np.random.default_rng(102)
    N, D, H, W, C, K, T, R, S_ = 1, 6, 5, 6, 8, 4, 3, 3, 2
    sd, pd, dd = 1, 1, 2
    x = rng.integers(-127, 128, size=(N, D, H, W, C)).astype(np.int8)
    w = rng.integers(-127, 128, size=(K, T, R, S_, C // 2)).astype(np.int8)
    y, _ = oracle.conv3d("i8", x, w, (sd, 2, 1), (pd, 1, 1), (dd, 1, 1), 2)
    OD = oracle.conv_out_extent(D, T, sd, pd, dd)
    assert y.shape[1] == OD
    for o in range(OD):
        acc = 0
        for t in range(T):
            i_d = o * sd - pd + t * dd
            if 0 <= i_d < D:
                acc = acc + oracle.conv2d("i8", np.ascontiguousarray(x[:, i_d]), np.ascontiguousarray(w[:, t]), (2, 1), (1, 1), (1, 1), 2)[0]
        assert np.array_equal(y[:, o], acc)
    # 127 * 127 * (taps * channels) must survive: the accumulator is wider than 16 and 32 bits of products
    xm = np.full((1, 3, 3, 3, 64), 127, dtype=np.int8); wm = np.full((1, 3, 3, 3, 64), -127, dtype=np.int8)
    ym, _ = oracle.conv3d("i8", xm, wm, (1, 1, 1), (0, 0, 0), (1, 1, 1), 1)
    assert ym.shape == (1, 1, 1, 1, 1) and int(ym[0, 0, 0, 0, 0]) == -127 * 127 * 27 * 64


@pytest.mark.parametrize("case", _T2D_CASES)
@pytest.mark.parametrize("dtype", ["i8", "f16"])
def test_conv2d_transpose_matches_brute_force_gather(oracle, case, dtype):
    """Scatter (oracle) against gather (here), int8 at full range and binary16 small integers (both exact)."""
    stride, pad, dil, outpad, groups = case
    rng = np.random.default_rng(103)
    N, H, W, C, K, R, S_ = 2, 4, 5, 4, 8, 3, 2
    if dtype == "i8":
        xb = rng.integers(-127, 128, size=(N, H, W, C)).astype(np.int8); wb = rng.integers(-127, 128, size=(K, R, S_, C // groups)).astype(np.int8)
        xv, wv = xb.astype(np.int64), wb.astype(np.int64)
    else:
        xb = _smallint_bits(rng, (N, H, W, C)); wb = _smallint_bits(rng, (K, R, S_, C // groups))
        xv, wv = _dec16(xb), _dec16(wb)
    y, S = oracle.conv2d_transpose(dtype, xb, wb, stride, pad, dil, outpad, groups)
    assert np.array_equal(y, _brute_conv2d_transpose_gather(xv, wv, stride, pad, dil, outpad, groups))
    if dtype != "i8":
        # S is the same operator applied to the absolute values: exactly, on this data
        assert np.array_equal(S, _brute_conv2d_transpose_gather(np.abs(xv), np.abs(wv), stride, pad, dil, outpad, groups))


def test_conv2d_transpose_int8_is_the_adjoint_of_int8_conv2d(oracle):
    """<conv2d(x, w), y> == <x, conv2d_transpose(y, w^T)> in exact integer arithmetic at full int8 range."""
    rng = np.random.default_rng(104)
    for (stride, pad, dil, groups, H, W) in [((1, 1), (0, 0), (1, 1), 1, 5, 6), ((2, 2), (1, 1), (1, 1), 2, 8, 7), ((3, 2), (1, 0), (1, 2), 1, 9, 8)]:
        N, C, K, R, S_ = 2, 4, 6, 3, 2
        Cg, Kg = C // groups, K // groups
        xb = rng.integers(-127, 128, size=(N, H, W, C)).astype(np.int8); wb = rng.integers(-127, 128, size=(K, R, S_, Cg)).astype(np.int8)
        fwd, _ = oracle.conv2d("i8", xb, wb, stride, pad, dil, groups)
        P, Q = fwd.shape[1:3]
        yb = rng.integers(-127, 128, size=(N, P, Q, K)).astype(np.int8)
        wT = np.ascontiguousarray(wb.reshape(groups, Kg, R, S_, Cg).transpose(0, 4, 2, 3, 1)).reshape(C, R, S_, Kg)
        outpad = ((H + 2 * pad[0] - dil[0] * (R - 1) - 1) % stride[0], (W + 2 * pad[1] - dil[1] * (S_ - 1) - 1) % stride[1])
        back, _ = oracle.conv2d_transpose("i8", yb, wT, stride, pad, dil, outpad, groups)
        assert back.shape == (N, H, W, C)
        assert int(np.sum(fwd * yb.astype(np.int64))) == int(np.sum(xb.astype(np.int64) * back))


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_S_of_every_convolution_form_is_the_operator_on_absolute_values(oracle, dtype):
    """The tolerance of every floating parity test is expressed in S = sum |x*w| over the operator's terms.  |x*w| =
    |x|*|w|, so S(x, w) must equal y(|x|, |w|), term by term in the same order: bit-identical."""
    def absbits(b):
        return (b & np.uint16(0x7fff)).astype(np.uint16)      # clearing the sign bit of binary16 / bfloat16 is |.|
    x2 = I.make_tensor(dtype, "u", 501, (2, 6, 7, 4)); w2 = I.make_tensor(dtype, "u", 502, (6, 3, 2, 2))
    y, S = oracle.conv2d(dtype, x2, w2, (2, 1), (1, 1), (1, 2), 2)
    assert np.array_equal(S, oracle.conv2d(dtype, absbits(x2), absbits(w2), (2, 1), (1, 1), (1, 2), 2)[0]) and np.any(S != np.abs(y))
    x1 = I.make_tensor(dtype, "u", 503, (2, 19, 4)); w1 = I.make_tensor(dtype, "u", 504, (6, 3, 2))
    y, S = oracle.conv1d(dtype, x1, w1, 2, 1, 2, 2)
    assert np.array_equal(S, oracle.conv1d(dtype, absbits(x1), absbits(w1), 2, 1, 2, 2)[0]) and np.any(S != np.abs(y))
    x3 = I.make_tensor(dtype, "u", 505, (1, 4, 5, 6, 4)); w3 = I.make_tensor(dtype, "u", 506, (4, 2, 3, 2, 2))
    y, S = oracle.conv3d(dtype, x3, w3, (1, 2, 1), (1, 1, 0), (2, 1, 1), 2)
    assert np.array_equal(S, oracle.conv3d(dtype, absbits(x3), absbits(w3), (1, 2, 1), (1, 1, 0), (2, 1, 1), 2)[0]) and np.any(S != np.abs(y))
    for (stride, pad, dil, outpad, groups) in _T2D_CASES:
        xt = I.make_tensor(dtype, "u", 507, (2, 4, 5, 4)); wt = I.make_tensor(dtype, "u", 508, (8, 3, 2, 4 // groups))
        y, S = oracle.conv2d_transpose(dtype, xt, wt, stride, pad, dil, outpad, groups)
        assert np.array_equal(S, oracle.conv2d_transpose(dtype, absbits(xt), absbits(wt), stride, pad, dil, outpad, groups)[0])
        assert np.any(S != np.abs(y))
    A = I.make_tensor(dtype, "u", 509, (7, 9)); Bm = I.make_tensor(dtype, "u", 510, (9, 5))
    C_, S = oracle.gemm(dtype, A, Bm, 7, 5, 9, 9, 1, 5, 1)
    assert np.array_equal(S, oracle.gemm(dtype, absbits(A), absbits(Bm), 7, 5, 9, 9, 1, 5, 1)[0])
