/*
 * CPU oracle for the tensor-contraction operators (test infrastructure, NOT the product).
 *
 * This file is the plain definition of the three operators the GPU library computes, written
 * as direct loops in fp64 (floating inputs) or int64 (int8 inputs).  It exists only so that
 * tests, the smoke check and the benchmark's cpu_baseline leg have something slow and obviously
 * correct to compare the HIP kernels with.  It shares no code, header, table or helper with
 * the GPU path and must never be called from it.
 *
 * What is computed (TensorIR paper, section 4.2):
 *   GEMM   C[x,y]     = sum_k A[x,k] * B[k,y]                      (Eq. 1, reduction init 0, sec. 3.1)
 *   BMM    C[b,i,j]   = sum_r A[b,i,r] * B[b,r,j]                  (sec. 4.2, b stays data-parallel)
 *   Conv2D C[n,h,w,co] = sum_{rh,rw,rc} A[n, h*s_h + rh*d_h - pad_h, w*s_w + rw*d_w - pad_w, g*Cg + rc]
 *                                        * W[co, rh, rw, rc]       (sec. 4.2 formula, NHWC)
 *     with the readings the paper leaves open: zero padding (taps outside the input add 0),
 *     cross-correlation (no filter flip), filter stored [K][R][S][C/groups], group of an output
 *     channel g = co / (K/groups), output extent floor((H + 2*pad - d*(R-1) - 1)/s) + 1.
 *
 * Inputs are the raw bits the GPU receives (IEEE binary16, bfloat16, or two's-complement int8);
 * each is decoded exactly to double / int64 here.  A product of two binary16 or two bfloat16
 * values is exact in double, so the only rounding is the fp64 summation (relative error
 * <= K * 2^-53 of sum|a*b|), far below the GPU tolerance.  For every output element the
 * side output S = sum |a*b| is produced as well; the parity bound is expressed in it.
 *
 * Every per-element sum runs over k in ascending order.  Loops over k sit outside the loop over
 * the output column only so that the innermost loop walks memory contiguously; each C[i,j] still
 * receives exactly the terms k = 0, 1, ..., K-1 in that order.
 *
 * Parity pins (tests/test_oracle_*.py): all 65536 binary16 / bfloat16 patterns against numpy's
 * own decode; brute-force per-element gathers on tiny shapes; identity matrices; conv ==
 * explicit im2col + matmul; 1x1 conv == GEMM; linearity; delta and all-ones closed forms; groups
 * == independent convs; fp64 library convolution (torch CPU) on strided/dilated/padded/grouped
 * cases; closed forms C = K and C = K*i*j; the fused consumers against hand-worked values (ties,
 * saturation, signs) and against the same arithmetic carried out in numpy's float32 / int64; the
 * attention head against closed forms (uniform attention, one dominant key, a single key), key
 * permutation invariance, shift invariance of the softmax, and scipy's softmax between two matmuls;
 * conv1d against numpy.correlate and the 2-D operator at height 1; conv3d against its reduction to
 * conv2d, a sum over depth taps (float and int8), a per-element gather at full int8 range and torch's
 * fp64 routine; the transposed convolution (written here as a scatter) against a per-element gather
 * (float and int8), the adjoint identity with conv2d (float and int8) and torch's fp64 routine; the
 * side output S of every operator against the same operator applied to |x|, |w|, bit for bit.
 * Each multiply-add line below (float and int8 branch of every function) and each S line is covered:
 * doubling a product or tripling an S term in any of them turns a pin red.  No function in this file
 * is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F16 = 0, ORACLE_BF16 = 1, ORACLE_I8 = 2 };
enum { ORACLE_OK = 0, ORACLE_BAD_ARG = 1, ORACLE_NO_MEMORY = 2 };

static int g_threads = 0; /* 0 = OpenMP default */

void oracle_set_threads(int n) { g_threads = n > 0 ? n : 0; }

int oracle_get_threads(void) {
#ifdef _OPENMP
    return g_threads > 0 ? g_threads : omp_get_max_threads();
#else
    return 1;
#endif
}

/* IEEE 754 binary16 -> double, exact (1 sign, 5 exponent bits with bias 15, 10 fraction bits). */
static double f16_bits_to_double(uint16_t h) {
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0) {
        v = ldexp((double)f, -24); /* zero or subnormal: f * 2^-10 * 2^-14 */
    } else if (e == 31) {
        v = f ? NAN : INFINITY;
    } else {
        v = ldexp((double)(1024 + f), e - 25); /* (1 + f/1024) * 2^(e-15) */
    }
    return sign ? -v : v;
}

/* bfloat16 is the upper half of an IEEE binary32. */
static double bf16_bits_to_double(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static double load_float(int dtype, const void* p, int64_t idx) {
    uint16_t bits = ((const uint16_t*)p)[idx];
    return dtype == ORACLE_F16 ? f16_bits_to_double(bits) : bf16_bits_to_double(bits);
}

/* Exposed so a test can pin the decoders against an independent decode of every bit pattern. */
int oracle_decode(int dtype, const void* bits, int64_t n, double* out) {
    if (n < 0 || (n > 0 && (!bits || !out))) return ORACLE_BAD_ARG;
    for (int64_t i = 0; i < n; ++i) {
        if (dtype == ORACLE_I8) out[i] = (double)((const int8_t*)bits)[i];
        else if (dtype == ORACLE_F16 || dtype == ORACLE_BF16) out[i] = load_float(dtype, bits, i);
        else return ORACLE_BAD_ARG;
    }
    return ORACLE_OK;
}

/* Gather a strided [rows, cols] operand into a dense row-major array of doubles / int64. */
static double* gather_f(int dtype, const void* p, int64_t rows, int64_t cols, int64_t rs, int64_t cs) {
    double* d = (double*)malloc(sizeof(double) * (size_t)(rows * cols > 0 ? rows * cols : 1));
    if (!d) return NULL;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) d[r * cols + c] = load_float(dtype, p, r * rs + c * cs);
    return d;
}

static int64_t* gather_i(const void* p, int64_t rows, int64_t cols, int64_t rs, int64_t cs) {
    int64_t* d = (int64_t*)malloc(sizeof(int64_t) * (size_t)(rows * cols > 0 ? rows * cols : 1));
    if (!d) return NULL;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) d[r * cols + c] = ((const int8_t*)p)[r * rs + c * cs];
    return d;
}

/*
 * GEMM, Eq. 1: C[i,j] = sum_k A[i,k] * B[k,j].  Element (i,k) of A sits at A[i*a_rs + k*a_cs],
 * element (k,j) of B at B[k*b_rs + j*b_cs] (strides in elements, non-negative).
 * C is dense row-major [M,N]: double for f16/bf16, int64 for int8.  S (double [M,N], may be NULL,
 * ignored for int8) receives sum_k |A[i,k] * B[k,j]|.  K = 0 gives C = 0.
 */
int oracle_gemm(int dtype, const void* A, const void* B, int64_t M, int64_t N, int64_t K,
                int64_t a_rs, int64_t a_cs, int64_t b_rs, int64_t b_cs, void* C, double* S) {
    if (M < 0 || N < 0 || K < 0) return ORACLE_BAD_ARG;
    if (dtype != ORACLE_F16 && dtype != ORACLE_BF16 && dtype != ORACLE_I8) return ORACLE_BAD_ARG;
    if (M == 0 || N == 0) return ORACLE_OK;
    if (!C || (K > 0 && (!A || !B))) return ORACLE_BAD_ARG;
    int nt = oracle_get_threads();
    (void)nt;
    if (dtype == ORACLE_I8) {
        int64_t* a = gather_i(A, M, K, a_rs, a_cs);
        int64_t* b = gather_i(B, K, N, b_rs, b_cs);
        if (!a || !b) { free(a); free(b); return ORACLE_NO_MEMORY; }
        int64_t* c = (int64_t*)C;
#pragma omp parallel for schedule(static) num_threads(nt)
        for (int64_t i = 0; i < M; ++i) {
            for (int64_t j = 0; j < N; ++j) c[i * N + j] = 0; /* reduction init */
            for (int64_t k = 0; k < K; ++k) {
                int64_t aik = a[i * K + k];
                for (int64_t j = 0; j < N; ++j) c[i * N + j] += aik * b[k * N + j];
            }
        }
        free(a); free(b);
        return ORACLE_OK;
    }
    double* a = gather_f(dtype, A, M, K, a_rs, a_cs);
    double* b = gather_f(dtype, B, K, N, b_rs, b_cs);
    if (!a || !b) { free(a); free(b); return ORACLE_NO_MEMORY; }
    double* c = (double*)C;
#pragma omp parallel for schedule(static) num_threads(nt)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) { c[i * N + j] = 0.0; if (S) S[i * N + j] = 0.0; }
        for (int64_t k = 0; k < K; ++k) {
            double aik = a[i * K + k];
            for (int64_t j = 0; j < N; ++j) {
                double t = aik * b[k * N + j];
                c[i * N + j] += t;
                if (S) S[i * N + j] += fabs(t);
            }
        }
    }
    free(a); free(b);
    return ORACLE_OK;
}

/*
 * Batched matmul: C[b,i,j] = sum_r A[b,i,r] * B[b,r,j]; the batch iterator maps to nothing in the
 * intrinsic and is a plain outer loop.  a_bs / b_bs are batch strides in elements (0 = the same
 * matrix for every batch).  C (and S) are dense [batch, M, N].
 */
int oracle_batch_matmul(int dtype, const void* A, const void* B, int64_t batch, int64_t M, int64_t N,
                        int64_t K, int64_t a_bs, int64_t a_rs, int64_t a_cs, int64_t b_bs, int64_t b_rs,
                        int64_t b_cs, void* C, double* S) {
    if (batch < 0) return ORACLE_BAD_ARG;
    size_t in_size = dtype == ORACLE_I8 ? 1 : 2;
    size_t out_size = 8;
    for (int64_t bi = 0; bi < batch; ++bi) {
        const char* a = A ? (const char*)A + (size_t)(bi * a_bs) * in_size : NULL;
        const char* b = B ? (const char*)B + (size_t)(bi * b_bs) * in_size : NULL;
        char* c = C ? (char*)C + (size_t)(bi * M * N) * out_size : NULL;
        double* s = S ? S + bi * M * N : NULL;
        int rc = oracle_gemm(dtype, a, b, M, N, K, a_rs, a_cs, b_rs, b_cs, c, s);
        if (rc != ORACLE_OK) return rc;
    }
    return ORACLE_OK;
}

/* Output extent of one spatial axis; <= 0 means the filter does not fit. */
int64_t oracle_conv_out_extent(int64_t in, int64_t filt, int64_t stride, int64_t pad, int64_t dil) {
    int64_t span = in + 2 * pad - dil * (filt - 1) - 1;
    if (span < 0) return 0;
    return span / stride + 1;
}

/*
 * Conv2D, direct loops.  x: [N,H,W,C] (NHWC), w: [K,R,S,C/groups], y (and Sabs): dense [N,P,Q,K].
 * y is double (f16/bf16) or int64 (int8).
 */
int oracle_conv2d(int dtype, const void* x, const void* w, int64_t N, int64_t H, int64_t W, int64_t C,
                  int64_t K, int64_t R, int64_t S, int64_t stride_h, int64_t stride_w, int64_t pad_h,
                  int64_t pad_w, int64_t dil_h, int64_t dil_w, int64_t groups, void* y, double* Sabs) {
    if (N < 0 || H <= 0 || W <= 0 || C <= 0 || K <= 0 || R <= 0 || S <= 0) return ORACLE_BAD_ARG;
    if (stride_h <= 0 || stride_w <= 0 || dil_h <= 0 || dil_w <= 0 || pad_h < 0 || pad_w < 0) return ORACLE_BAD_ARG;
    if (groups <= 0 || C % groups || K % groups) return ORACLE_BAD_ARG;
    if (dtype != ORACLE_F16 && dtype != ORACLE_BF16 && dtype != ORACLE_I8) return ORACLE_BAD_ARG;
    int64_t P = oracle_conv_out_extent(H, R, stride_h, pad_h, dil_h);
    int64_t Q = oracle_conv_out_extent(W, S, stride_w, pad_w, dil_w);
    if (P <= 0 || Q <= 0) return ORACLE_BAD_ARG;
    if (N == 0) return ORACLE_OK;
    if (!x || !w || !y) return ORACLE_BAD_ARG;
    int64_t Cg = C / groups, Kg = K / groups;
    int nt = oracle_get_threads();
    (void)nt;
    int is_int = dtype == ORACLE_I8;
    /* decode once; the loops below then read doubles / int64 */
    double* xf = NULL; double* wf = NULL; int64_t* xi = NULL; int64_t* wi = NULL;
    if (is_int) {
        xi = gather_i(x, 1, N * H * W * C, 0, 1);
        wi = gather_i(w, 1, K * R * S * Cg, 0, 1);
        if (!xi || !wi) { free(xi); free(wi); return ORACLE_NO_MEMORY; }
    } else {
        xf = gather_f(dtype, x, 1, N * H * W * C, 0, 1);
        wf = gather_f(dtype, w, 1, K * R * S * Cg, 0, 1);
        if (!xf || !wf) { free(xf); free(wf); return ORACLE_NO_MEMORY; }
    }
#pragma omp parallel for collapse(2) schedule(static) num_threads(nt)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t p = 0; p < P; ++p)
            for (int64_t q = 0; q < Q; ++q)
                for (int64_t k = 0; k < K; ++k) {
                    int64_t g = k / Kg;
                    double accf = 0.0, accs = 0.0;
                    int64_t acci = 0;
                    for (int64_t r = 0; r < R; ++r) {
                        int64_t ih = p * stride_h - pad_h + r * dil_h;
                        if (ih < 0 || ih >= H) continue; /* zero padding */
                        for (int64_t s = 0; s < S; ++s) {
                            int64_t iw = q * stride_w - pad_w + s * dil_w;
                            if (iw < 0 || iw >= W) continue;
                            int64_t xo = ((n * H + ih) * W + iw) * C + g * Cg;
                            int64_t wo = ((k * R + r) * S + s) * Cg;
                            for (int64_t c = 0; c < Cg; ++c) {
                                if (is_int) {
                                    acci += xi[xo + c] * wi[wo + c];
                                } else {
                                    double t = xf[xo + c] * wf[wo + c];
                                    accf += t;
                                    accs += fabs(t);
                                }
                            }
                        }
                    }
                    int64_t o = ((n * P + p) * Q + q) * K + k;
                    if (is_int) ((int64_t*)y)[o] = acci;
                    else { ((double*)y)[o] = accf; if (Sabs) Sabs[o] = accs; }
                }
    free(xf); free(wf); free(xi); free(wi);
    return ORACLE_OK;
}

/*
 * Fused consumers of the contraction (the paper's running example in its section-4 overview figure is a
 * matmul followed by ReLU; the consumer is computed behind the tensorized block instead of in a second
 * pass).  Both functions work in place on the row-major [rows][N] result of one of the operators above;
 * column j is the output column / output channel.
 *
 * Floating inputs:  t = C[i,j] + bias[j];  if relu: t = max(t, 0).  In fp64; S[i,j] (if given) grows by
 *   |bias[j]|, one more term of the sum the parity bound is expressed in.  bias may be NULL.
 * int8 inputs:      t = C[i,j] + bias[j] in int64 (must fit int32: else ORACLE_BAD_ARG);
 *   if relu: t = max(t, 0).  With requantise != 0 the value is then mapped to an int8 code in
 *   SINGLE precision, the precision the decision is taken in on the device as well:
 *       f = (float)(int32)t        (int32 -> binary32, round to nearest even)
 *       f = f * scale              (one binary32 multiplication)
 *       q = nearest integer to f, ties to even;  q = min(max(q, -128), 127)
 *   and C[i,j] = q.  scale must be finite and > 0.
 */
int oracle_epilogue_float(double* C, double* S, int64_t rows, int64_t N, const float* bias, int relu) {
    if (!C || rows < 0 || N < 0) return ORACLE_BAD_ARG;
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < N; ++j) {
            double t = C[i * N + j];
            if (bias) {
                t += (double)bias[j];
                if (S) S[i * N + j] += fabs((double)bias[j]);
            }
            if (relu && t < 0.0) t = 0.0;
            C[i * N + j] = t;
        }
    return ORACLE_OK;
}

int oracle_epilogue_int(int64_t* C, int64_t rows, int64_t N, const int32_t* bias, int relu, int requantise, float scale) {
    if (!C || rows < 0 || N < 0) return ORACLE_BAD_ARG;
    if (requantise && !(scale > 0.0f && scale <= 3.4028234663852886e38f)) return ORACLE_BAD_ARG;
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < N; ++j) {
            int64_t t = C[i * N + j];
            if (bias) t += (int64_t)bias[j];
            if (t < INT32_MIN || t > INT32_MAX) return ORACLE_BAD_ARG;
            if (relu && t < 0) t = 0;
            if (requantise) {
                volatile float f = (float)(int32_t)t;   /* volatile: each step is rounded to binary32, never kept wider */
                volatile float g = f * scale;
                float q = nearbyintf(g);                /* default rounding mode: to nearest, ties to even */
                if (q < -128.0f) q = -128.0f;
                if (q > 127.0f) q = 127.0f;
                t = (int64_t)q;
            }
            C[i * N + j] = t;
        }
    return ORACLE_OK;
}

/*
 * One attention head per batch: two contractions (Eq. 1 twice) with the row-wise softmax between
 * them computed in place - the two tensorized blocks of the paper's batched-matmul workload share one
 * tile instead of meeting in memory (sec. 2 and 3.2: blocks isolate sub-problems, which does not
 * prevent cooperation across blocks).  The softmax itself is the textbook definition, not the paper's.
 *
 *   S[b,i,j] = scale * sum_c Q[b,i,c] * K[b,j,c]          (K stored [N][d]: "Q . K^T")
 *   P[b,i,j] = exp(S[b,i,j] - max_j S[b,i,:]) / sum_j exp(S[b,i,j] - max_j S[b,i,:])
 *   O[b,i,e] = sum_j P[b,i,j] * V[b,j,e]
 *
 * Q: [batch][M][d], K: [batch][N][d], V: [batch][N][dv], dense, raw binary16 / bfloat16 bits.
 * Everything in fp64.  T[b,i,e] = sum_j P[b,i,j] * |V[b,j,e]| is the side output the parity bound is
 * expressed in (the probabilities are where the device rounds to 16 bits before the second product).
 * N must be >= 1.
 */
int oracle_attention(int dtype, const void* Q, const void* K, const void* V, int64_t batch, int64_t M, int64_t N,
                     int64_t d, int64_t dv, double scale, double* O, double* T) {
    if (dtype != ORACLE_F16 && dtype != ORACLE_BF16) return ORACLE_BAD_ARG;
    if (batch < 0 || M < 0 || N < 1 || d < 0 || dv < 0 || !O) return ORACLE_BAD_ARG;
    int failed = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(oracle_get_threads())
#endif
    for (int64_t bi = 0; bi < batch * M; ++bi) {
        const int64_t b = bi / M, i = bi % M;
        double* s = (double*)malloc((size_t)N * sizeof(double));
        if (!s) { failed = 1; continue; }
        double mx = 0.0;
        for (int64_t j = 0; j < N; ++j) {
            double acc = 0.0;
            for (int64_t c = 0; c < d; ++c)
                acc += load_float(dtype, Q, (b * M + i) * d + c) * load_float(dtype, K, (b * N + j) * d + c);
            s[j] = scale * acc;
            if (j == 0 || s[j] > mx) mx = s[j];
        }
        double denom = 0.0;
        for (int64_t j = 0; j < N; ++j) { s[j] = exp(s[j] - mx); denom += s[j]; }
        for (int64_t e = 0; e < dv; ++e) {
            double o = 0.0, t = 0.0;
            for (int64_t j = 0; j < N; ++j) {
                const double p = s[j] / denom, v = load_float(dtype, V, (b * N + j) * dv + e);
                o += p * v;
                t += p * fabs(v);
            }
            O[(b * M + i) * dv + e] = o;
            if (T) T[(b * M + i) * dv + e] = t;
        }
        free(s);
    }
    return failed ? ORACLE_NO_MEMORY : ORACLE_OK;
}

/*
 * The remaining convolution forms of the paper's operator set (sec. 5.1: 1D, 3D and transposed 2D
 * convolution next to the 2D, dilated and grouped ones above).  Same readings as oracle_conv2d: zero
 * padding, cross-correlation, channels-last activations, filter stored output-channel-major with the
 * channel innermost, contiguous channel groups, floor rule for the output extent.
 *
 * conv1d:  x [N][L][C],        w [K][R][C/g]         y[n,p,k] = sum_{r,c} x[n, p*s - pad + r*d, g*Cg + c] * w[k,r,c]
 * conv3d:  x [N][D][H][W][C],  w [K][T][R][S][C/g]   y[n,o,p,q,k] = sum_{t,r,s,c} x[n, o*s_d - pad_d + t*d_d, p*s_h - pad_h + r*d_h,
 *                                                                                  q*s_w - pad_w + s*d_w, g*Cg + c] * w[k,t,r,s,c]
 * conv2d_transpose (the adjoint of a strided convolution, written as the scatter that defines it):
 *          x [N][H][W][C],     w [K][R][S][C/g]      for every input pixel (ih, iw), tap (r, s) and channel c of group g:
 *              y[n, ih*s_h - pad_h + r*d_h, iw*s_w - pad_w + s*d_w, k] += x[n,ih,iw,g*Cg + c] * w[k,r,s,c]     (targets outside y dropped)
 *          output extent (H-1)*s_h - 2*pad_h + d_h*(R-1) + outpad_h + 1, likewise for the width.
 * S (float inputs) accumulates |x*w| over the same terms.  Arguments: int64 arrays dims / strides / pads / dils
 * of the spatial rank (1, 3 or 2).
 */
int oracle_conv1d(int dtype, const void* x, const void* w, int64_t N, int64_t L, int64_t C, int64_t K, int64_t R,
                  int64_t stride, int64_t pad, int64_t dil, int64_t groups, void* y, double* Sabs) {
    if (N < 0 || L <= 0 || C <= 0 || K <= 0 || R <= 0 || stride <= 0 || dil <= 0 || pad < 0 || groups <= 0 || C % groups || K % groups) return ORACLE_BAD_ARG;
    const int64_t P = oracle_conv_out_extent(L, R, stride, pad, dil);
    if (P <= 0) return ORACLE_BAD_ARG;
    const int is_int = dtype == ORACLE_I8;
    const int64_t Cg = C / groups, Kg = K / groups;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t p = 0; p < P; ++p)
            for (int64_t k = 0; k < K; ++k) {
                const int64_t g = k / Kg;
                double accf = 0.0, accs = 0.0;
                int64_t acci = 0;
                for (int64_t r = 0; r < R; ++r) {
                    const int64_t il = p * stride - pad + r * dil;
                    if (il < 0 || il >= L) continue;
                    for (int64_t c = 0; c < Cg; ++c) {
                        const int64_t xo = (n * L + il) * C + g * Cg + c, wo = (k * R + r) * Cg + c;
                        if (is_int) acci += (int64_t)((const int8_t*)x)[xo] * (int64_t)((const int8_t*)w)[wo];
                        else { const double t = load_float(dtype, x, xo) * load_float(dtype, w, wo); accf += t; accs += fabs(t); }
                    }
                }
                const int64_t o = (n * P + p) * K + k;
                if (is_int) ((int64_t*)y)[o] = acci;
                else { ((double*)y)[o] = accf; if (Sabs) Sabs[o] = accs; }
            }
    return ORACLE_OK;
}

int oracle_conv3d(int dtype, const void* x, const void* w, int64_t N, const int64_t* in_dhw, int64_t C, int64_t K,
                  const int64_t* filt_trs, const int64_t* stride, const int64_t* pad, const int64_t* dil, int64_t groups,
                  void* y, double* Sabs) {
    if (N < 0 || C <= 0 || K <= 0 || groups <= 0 || C % groups || K % groups) return ORACLE_BAD_ARG;
    int64_t out[3];
    for (int a = 0; a < 3; ++a) {
        if (in_dhw[a] <= 0 || filt_trs[a] <= 0 || stride[a] <= 0 || dil[a] <= 0 || pad[a] < 0) return ORACLE_BAD_ARG;
        out[a] = oracle_conv_out_extent(in_dhw[a], filt_trs[a], stride[a], pad[a], dil[a]);
        if (out[a] <= 0) return ORACLE_BAD_ARG;
    }
    const int is_int = dtype == ORACLE_I8;
    const int64_t D = in_dhw[0], H = in_dhw[1], W = in_dhw[2], T = filt_trs[0], R = filt_trs[1], S = filt_trs[2];
    const int64_t Cg = C / groups, Kg = K / groups;
#ifdef _OPENMP
#pragma omp parallel for collapse(2) schedule(static) num_threads(oracle_get_threads())
#endif
    for (int64_t n = 0; n < N; ++n)
        for (int64_t o = 0; o < out[0]; ++o)
            for (int64_t p = 0; p < out[1]; ++p)
                for (int64_t q = 0; q < out[2]; ++q)
                    for (int64_t k = 0; k < K; ++k) {
                        const int64_t g = k / Kg;
                        double accf = 0.0, accs = 0.0;
                        int64_t acci = 0;
                        for (int64_t t = 0; t < T; ++t) {
                            const int64_t id = o * stride[0] - pad[0] + t * dil[0];
                            if (id < 0 || id >= D) continue;
                            for (int64_t r = 0; r < R; ++r) {
                                const int64_t ih = p * stride[1] - pad[1] + r * dil[1];
                                if (ih < 0 || ih >= H) continue;
                                for (int64_t s = 0; s < S; ++s) {
                                    const int64_t iw = q * stride[2] - pad[2] + s * dil[2];
                                    if (iw < 0 || iw >= W) continue;
                                    const int64_t xo = (((n * D + id) * H + ih) * W + iw) * C + g * Cg;
                                    const int64_t wo = (((k * T + t) * R + r) * S + s) * Cg;
                                    for (int64_t c = 0; c < Cg; ++c) {
                                        if (is_int) acci += (int64_t)((const int8_t*)x)[xo + c] * (int64_t)((const int8_t*)w)[wo + c];
                                        else { const double v = load_float(dtype, x, xo + c) * load_float(dtype, w, wo + c); accf += v; accs += fabs(v); }
                                    }
                                }
                            }
                        }
                        const int64_t oo = (((n * out[0] + o) * out[1] + p) * out[2] + q) * K + k;
                        if (is_int) ((int64_t*)y)[oo] = acci;
                        else { ((double*)y)[oo] = accf; if (Sabs) Sabs[oo] = accs; }
                    }
    return ORACLE_OK;
}

int64_t oracle_conv_transpose_out_extent(int64_t in, int64_t filt, int64_t stride, int64_t pad, int64_t dil, int64_t outpad) {
    return (in - 1) * stride - 2 * pad + dil * (filt - 1) + outpad + 1;
}

int oracle_conv2d_transpose(int dtype, const void* x, const void* w, int64_t N, int64_t H, int64_t W, int64_t C, int64_t K,
                            int64_t R, int64_t S, const int64_t* stride, const int64_t* pad, const int64_t* dil,
                            const int64_t* outpad, int64_t groups, void* y, double* Sabs) {
    if (N < 0 || H <= 0 || W <= 0 || C <= 0 || K <= 0 || R <= 0 || S <= 0 || groups <= 0 || C % groups || K % groups) return ORACLE_BAD_ARG;
    for (int a = 0; a < 2; ++a)
        if (stride[a] <= 0 || dil[a] <= 0 || pad[a] < 0 || outpad[a] < 0) return ORACLE_BAD_ARG;
    const int64_t P = oracle_conv_transpose_out_extent(H, R, stride[0], pad[0], dil[0], outpad[0]);
    const int64_t Q = oracle_conv_transpose_out_extent(W, S, stride[1], pad[1], dil[1], outpad[1]);
    if (P <= 0 || Q <= 0) return ORACLE_BAD_ARG;
    const int is_int = dtype == ORACLE_I8;
    const int64_t Cg = C / groups, Kg = K / groups, total = N * P * Q * K;
    if (is_int) memset(y, 0, (size_t)total * sizeof(int64_t));
    else { memset(y, 0, (size_t)total * sizeof(double)); if (Sabs) memset(Sabs, 0, (size_t)total * sizeof(double)); }
    for (int64_t n = 0; n < N; ++n)
        for (int64_t ih = 0; ih < H; ++ih)
            for (int64_t iw = 0; iw < W; ++iw)
                for (int64_t r = 0; r < R; ++r) {
                    const int64_t oh = ih * stride[0] - pad[0] + r * dil[0];
                    if (oh < 0 || oh >= P) continue;
                    for (int64_t s = 0; s < S; ++s) {
                        const int64_t ow = iw * stride[1] - pad[1] + s * dil[1];
                        if (ow < 0 || ow >= Q) continue;
                        for (int64_t k = 0; k < K; ++k) {
                            const int64_t g = k / Kg;
                            const int64_t xo = ((n * H + ih) * W + iw) * C + g * Cg, wo = ((k * R + r) * S + s) * Cg;
                            const int64_t oo = ((n * P + oh) * Q + ow) * K + k;
                            for (int64_t c = 0; c < Cg; ++c) {
                                if (is_int) ((int64_t*)y)[oo] += (int64_t)((const int8_t*)x)[xo + c] * (int64_t)((const int8_t*)w)[wo + c];
                                else {
                                    const double v = load_float(dtype, x, xo + c) * load_float(dtype, w, wo + c);
                                    ((double*)y)[oo] += v;
                                    if (Sabs) Sabs[oo] += fabs(v);
                                }
                            }
                        }
                    }
                }
    return ORACLE_OK;
}
