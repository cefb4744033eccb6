/*
 * tir.h — C ABI of the MI355X (gfx950) tensor-contraction library.
 *
 * Three operators, each computed by decomposing its loop nest into blocks that map onto one
 * MFMA tile (the hardware tensor intrinsic C[x,y] += A[x,k] * B[k,y], TensorIR paper Eq. 1):
 *
 *   tir_gemm          C[x,y]       = sum_k A[x,k] * B[k,y]                     (Eq. 1)
 *   tir_batch_matmul  C[b,i,j]     = sum_r A[b,i,r] * B[b,r,j]                 (sec. 4.2; x,y,k -> i,j,r,
 *                                                                               b stays a data-parallel loop)
 *   tir_conv2d        C[n,h,w,co]  = sum A[n, h*s_h + rh*d_h - pad_h, w*s_w + rw*d_w - pad_w, rc]
 *                                        * W[co, rh, rw, rc]                   (sec. 4.2 Conv2D formula;
 *                       mapped onto Eq. 1 by ReIndex + fuse: x = fuse(n,h,w), y = co, k = fuse(rh,rw,rc))
 *
 * Common conventions
 *   - Every pointer is a DEVICE pointer owned by the caller.  The operator entry points never allocate or free
 *     device memory, never copy to the host and never synchronise: each call enqueues kernels on `stream` and
 *     returns, also while `stream` (or any other stream) is being captured.  The only calls that block or create
 *     HIP objects are the tuning calls (tir_tune_*), which say so.
 *   - One kernel path needs scratch memory: a reduction that is split over several workgroups per output tile
 *     (few small tiles facing a long K; the variant queries report it as "<variant>/z<slices>") keeps partial sums
 *     and arrival counters in a workspace.  The library owns none: it plans such a split only for launches on a
 *     stream for which the caller has registered a buffer (tir_set_workspace), and plans the same problem
 *     unsplit otherwise.  The result does not depend on the split's timing: the partial sums are added in a
 *     fixed order.  tir_gemm_split_static is the variant for callers that cannot provide a buffer either.
 *   - The output is fully overwritten (reduction init is 0; there is no alpha / beta), and must not
 *     overlap an input.
 *   - Inputs F16 / BF16 accumulate in fp32; input I8 accumulates in int32 (wrap-around on overflow,
 *     which inputs in [-127,127] with K <= 133000 cannot reach).
 *   - Allowed (in, out) pairs: (F16, F32) (F16, F16) (BF16, F32) (BF16, BF16) (I8, I32).
 *     16-bit outputs are rounded to nearest even from the fp32 accumulator.
 *   - Strides are in ELEMENTS and must be >= 0.  Any strides are accepted; the fast kernels need the
 *     reduction axis or the other axis of each input contiguous (stride 1), 16-byte aligned base
 *     pointers and leading strides that are multiples of 16 bytes, and a unit column stride on C.
 *     Everything else runs on a slower general kernel with the same results.
 *   - Return value: TIR_OK or an error code; on error nothing was launched and tir_last_error()
 *     describes the problem.  No C++ exception crosses this boundary.
 *   - Zero-sized M, N, batch (or conv batch N) is a successful no-op.  K == 0 zero-fills C.
 */
#ifndef TIR_H_
#define TIR_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TIR_OK = 0,
    TIR_ERR_INVALID_ARG = 1,  /* null pointer, negative size or stride, bad dtype code, groups not dividing */
    TIR_ERR_UNSUPPORTED = 2,  /* a (in, out) dtype pair outside the list above, or sizes beyond 2^31-1 */
    TIR_ERR_ALIGNMENT = 3,    /* pointer not aligned to its element size */
    TIR_ERR_LAUNCH = 4        /* the HIP runtime refused the launch; message holds hipGetErrorString */
} tir_status;

typedef enum { TIR_F16 = 0, TIR_BF16 = 1, TIR_I8 = 2, TIR_F32 = 3, TIR_I32 = 4 } tir_dtype;

/* Opaque stream handle: pass a hipStream_t (NULL = the default stream). */
typedef void* tir_stream;

/*
 * GEMM, Eq. 1.  Element (i,k) of A is A[i*a_rs + k*a_cs], (k,j) of B is B[k*b_rs + j*b_cs],
 * (i,j) of C is C[i*c_rs + j*c_cs].  Row-major operands: a_rs=K,a_cs=1, b_rs=N,b_cs=1, c_rs=N,c_cs=1;
 * a transposed operand is expressed by swapping its strides.
 */
tir_status tir_gemm(const void* A, const void* B, void* C, int64_t M, int64_t N, int64_t K,
                    int64_t a_rs, int64_t a_cs, int64_t b_rs, int64_t b_cs, int64_t c_rs, int64_t c_cs,
                    tir_dtype in, tir_dtype out, tir_stream stream);

/*
 * Batched matmul (sec. 4.2): C[b] = A[b] * B[b] for b < batch.  *_bs are batch strides in
 * elements; a_bs or b_bs may be 0 (the same matrix for every batch), c_bs must make the C
 * matrices disjoint.
 */
tir_status tir_batch_matmul(const void* A, const void* B, void* C, int64_t batch, int64_t M, int64_t N,
                            int64_t K, int64_t a_bs, int64_t a_rs, int64_t a_cs, int64_t b_bs, int64_t b_rs,
                            int64_t b_cs, int64_t c_bs, int64_t c_rs, int64_t c_cs, tir_dtype in,
                            tir_dtype out, tir_stream stream);

/*
 * 2-D convolution (sec. 4.2), cross-correlation with zero padding.
 *   x: [N,H,W,C] NHWC, dense.   w: [K,R,S,C/groups], dense (filter of output channel k, tap (r,s)).
 *   y: [N,P,Q,K] NHWC, dense, P = floor((H + 2*pad_h - dil_h*(R-1) - 1)/stride_h) + 1, Q likewise.
 *   Output channel k belongs to group k / (K/groups) and reads input channels
 *   [g*C/groups, (g+1)*C/groups).  groups must divide C and K; P and Q must be >= 1.
 * The im2col matrix is never materialised: input coordinates are recomputed from the fused
 * iterators inside the kernel.
 */
tir_status tir_conv2d(const void* x, const void* w, void* y, int64_t N, int64_t H, int64_t W, int64_t C,
                      int64_t K, int64_t R, int64_t S, int stride_h, int stride_w, int pad_h, int pad_w,
                      int dil_h, int dil_w, int groups, tir_dtype in, tir_dtype out, tir_stream stream);

/*
 * Fused consumers (the paper's running example, the overview figure of sec. 4, is a matmul followed by
 * ReLU: the element-wise consumer is computed behind the tensorized block, in the same kernel, instead
 * of in a second pass over C).  The *_fused entry points take the arguments of the plain ones plus an
 * epilogue; ep == NULL is the plain operator.  With t = the operator's sum for output column j
 * (GEMM / batched matmul: column of C, the same bias for every batch; conv2d: output channel k):
 *     t = t + bias[j]          if bias != NULL   (fp32 for F16 / BF16 inputs, int32 for I8 inputs;
 *                                                 device pointer, 4-byte aligned, N resp. K elements)
 *     t = max(t, 0)            if relu != 0
 *     out = convert(t)         F32 / I32: unchanged; F16 / BF16: round to nearest even;
 *                              I8 (inputs I8 only): clamp(rint((float)t * scale), -128, 127), the
 *                              product and the rounding in binary32, ties to even; scale must be
 *                              finite and > 0.  The int32 sum t must not overflow.
 * (I8, I8) is an allowed (in, out) pair for the fused entry points only; scale is ignored otherwise.
 *
 * streaming: cache policy of this call's output stores (0 or 1; anything else is TIR_ERR_INVALID_ARG).  Every
 * kernel writes its output through to memory during its epilogue.  With 0 (and for the entry points that take no
 * epilogue) the lines also stay in the caches, which is what a consumer launched next wants: in a chain of
 * 56x56x64 convolutions that each read the previous one's output a launch takes 7.5 us this way and 8.1 us with
 * streaming stores.  1 marks the stores non-temporal: for outputs that nothing reads soon - the last operator of a
 * graph, results copied out later, tensors larger than the caches.  Results are identical either way.
 */
typedef struct tir_epilogue {
    const void* bias;
    int relu;
    float scale;
    int streaming;
} tir_epilogue;

tir_status tir_gemm_fused(const void* A, const void* B, void* C, int64_t M, int64_t N, int64_t K, int64_t a_rs,
                          int64_t a_cs, int64_t b_rs, int64_t b_cs, int64_t c_rs, int64_t c_cs, tir_dtype in,
                          tir_dtype out, const tir_epilogue* ep, tir_stream stream);
tir_status tir_batch_matmul_fused(const void* A, const void* B, void* C, int64_t batch, int64_t M, int64_t N,
                                  int64_t K, int64_t a_bs, int64_t a_rs, int64_t a_cs, int64_t b_bs,
                                  int64_t b_rs, int64_t b_cs, int64_t c_bs, int64_t c_rs, int64_t c_cs,
                                  tir_dtype in, tir_dtype out, const tir_epilogue* ep, tir_stream stream);
tir_status tir_conv2d_fused(const void* x, const void* w, void* y, int64_t N, int64_t H, int64_t W, int64_t C,
                            int64_t K, int64_t R, int64_t S, int stride_h, int stride_w, int pad_h, int pad_w,
                            int dil_h, int dil_w, int groups, tir_dtype in, tir_dtype out,
                            const tir_epilogue* ep, tir_stream stream);

/*
 * The other convolution forms of the paper's operator set (sec. 5.1 evaluates 1-D, 3-D and transposed 2-D
 * convolution next to the 2-D, dilated and grouped ones).  Same conventions as tir_conv2d: channels-last
 * activations, filter stored output-channel-major with the channel innermost, zero padding,
 * cross-correlation, contiguous channel groups; ep (may be NULL) fuses a consumer as in tir_conv2d_fused.
 *
 * tir_conv1d:  x [N,L,C], w [K,R,C/groups], y [N,P,K], P = floor((L + 2*pad - dil*(R-1) - 1)/stride) + 1;
 *     y[n,p,k] = sum_{r,c} x[n, p*stride - pad + r*dil, g*C/groups + c] * w[k,r,c].
 * tir_conv3d:  x [N,D,H,W,C], w [K,T,R,S,C/groups], y [N,OD,P,Q,K] with the floor rule per axis;
 *     y[n,o,p,q,k] = sum_{t,r,s,c} x[n, o*stride_d - pad_d + t*dil_d, p*stride_h - pad_h + r*dil_h,
 *                                    q*stride_w - pad_w + s*dil_w, g*C/groups + c] * w[k,t,r,s,c].
 * tir_conv2d_transpose: the adjoint of a strided convolution.  x [N,H,W,C], w [K,R,S,C/groups] (output
 *     channel k, tap (r,s), input channel c of k's group), y [N,P,Q,K] with
 *     P = (H-1)*stride_h - 2*pad_h + dil_h*(R-1) + outpad_h + 1 (Q alike; outpad >= 0 only adds rows /
 *     columns that receive no or fewer contributions).  Every input pixel (ih, iw) adds
 *     x[n,ih,iw,g*C/groups + c] * w[k,r,s,c] to y[n, ih*stride_h - pad_h + r*dil_h, iw*stride_w - pad_w + s*dil_w, k]
 *     (targets outside y are dropped).  Computed as a gather: no atomics, the result is deterministic.
 *     Strided, undilated problems whose C/groups channels fill whole 128-byte blocks are computed per
 *     output phase (oh mod stride_h, ow mod stride_w): stride_h*stride_w stride-1 convolutions with the
 *     taps each phase can reach, in one launch (variant query: "<variant>/ph<stride_h>x<stride_w>");
 *     strides above 16383 are TIR_ERR_UNSUPPORTED.
 */
tir_status tir_conv1d(const void* x, const void* w, void* y, int64_t N, int64_t L, int64_t C, int64_t K, int64_t R,
                      int stride, int pad, int dil, int groups, tir_dtype in, tir_dtype out, const tir_epilogue* ep,
                      tir_stream stream);
tir_status tir_conv3d(const void* x, const void* w, void* y, int64_t N, int64_t D, int64_t H, int64_t W, int64_t C,
                      int64_t K, int64_t T, int64_t R, int64_t S, int stride_d, int stride_h, int stride_w, int pad_d,
                      int pad_h, int pad_w, int dil_d, int dil_h, int dil_w, int groups, tir_dtype in, tir_dtype out,
                      const tir_epilogue* ep, tir_stream stream);
tir_status tir_conv2d_transpose(const void* x, const void* w, void* y, int64_t N, int64_t H, int64_t W, int64_t C,
                                int64_t K, int64_t R, int64_t S, int stride_h, int stride_w, int pad_h, int pad_w,
                                int dil_h, int dil_w, int outpad_h, int outpad_w, int groups, tir_dtype in,
                                tir_dtype out, const tir_epilogue* ep, tir_stream stream);

/*
 * One attention head per batch, both contractions and the softmax between them in one kernel (the
 * two tensorized blocks of the batched-matmul workload share a tile; sec. 2 / 3.2 of the paper on blocks
 * as isolated sub-problems that still cooperate; the softmax is the textbook definition):
 *     S[b,i,j] = scale * sum_c Q[b,i,c] * K[b,j,c]
 *     P[b,i,:] = softmax over j of S[b,i,:]
 *     O[b,i,e] = sum_j P[b,i,j] * V[b,j,e]
 * Q: [batch][M][d], K: [batch][N][d], V: [batch][N][d], O: [batch][M][d], all dense, 16-byte aligned
 * device pointers.  d must be 64 or 128 (TIR_ERR_UNSUPPORTED otherwise).  in = F16 or BF16; out = the
 * same type or F32.  Scores and the softmax are fp32; the probabilities are rounded to the input type
 * before the second product, which accumulates in fp32.  N = 0 is an error (no keys), M = 0 or
 * batch = 0 a no-op.  scale must be finite.
 * Accuracy a caller gets, with T[b,i,e] = sum_j P[b,i,j] * |V[b,j,e]| of the exact probabilities:
 *   F16 inputs:  |O - exact| <= 2e-3 * T + 1e-5  (the bound of the plain operators; the rounding of P to binary16
 *                costs at most 2^-11 * T of it);
 *   BF16 inputs: |O - exact| <= 6e-3 * T + 1e-5  (P is rounded to bfloat16, 8 significant bits: that step alone
 *                is up to 2^-9 * T = 2e-3 * T), plus 2^-8 * |O| when the output is BF16 as well.
 */
tir_status tir_attention(const void* Q, const void* K, const void* V, void* O, int64_t batch, int64_t M, int64_t N,
                         int64_t d, float scale, tir_dtype in, tir_dtype out, tir_stream stream);

/* Message for the calling thread's last failed call ("" if none).  Never NULL; valid until the
 * thread's next failing call. */
const char* tir_last_error(void);

/*
 * Workspace for split reductions (see the conventions at the top): without one, no reduction is split over
 * workgroups.
 * tir_workspace_bytes: size the buffer must have (partial sums, then the arrival counters).
 * tir_set_workspace: from now on, launches on `stream` of the CURRENT device may split their reductions and keep
 * the partial sums in `ws` (device memory, 256-byte aligned, at least tir_workspace_bytes() bytes, owned by the
 * caller).  The call enqueues one small kernel on `stream` that zeroes the counters (a kernel, not a memset, so
 * the call may be captured) and returns; every launch leaves them zero again.  The buffer must stay allocated
 * until the work enqueued on `stream` has finished and a later tir_set_workspace has replaced or removed it;
 * ws = NULL removes the registration (later launches on `stream` run unsplit).  Two streams that may run at the
 * same time need two buffers: launches that share one race.  Tuning calls use the workspace of the stream they
 * are given and try split reductions only if it has one.
 * Errors: TIR_ERR_INVALID_ARG (buffer too small), TIR_ERR_ALIGNMENT, TIR_ERR_LAUNCH; the previous
 * registration stays in place then.
 */
uint64_t tir_workspace_bytes(void);
tir_status tir_set_workspace(tir_stream stream, void* ws, uint64_t bytes);

/*
 * GEMM with the reduction split over `slices` workgroups per output tile, for callers that can neither let a
 * library allocate nor hand it a buffer of their own: code under HIP graph capture, tight serving loops with a
 * fixed memory plan, harnesses that forbid hipMalloc.  Arguments and result as tir_gemm_fused (ep may be NULL);
 * the partial sums and arrival counters live in a static device array of the library, TIR_STATIC_SCRATCH_BYTES
 * of partial sums and TIR_STATIC_SCRATCH_TILES counters per GPU, held from the first call on that GPU until the
 * process ends.  The call allocates and frees nothing, does not synchronise, and enqueues on `stream` one small
 * kernel that zeroes the counters it will use, then the GEMM.
 *   slices: 2 .. 64, and at most the number of 128-byte stages of the reduction (K * element size / 128, rounded
 *     up), such that no slice is empty.
 *   Limits: the operands must qualify for the fast kernels (see "Strides" at the top; TIR_ERR_UNSUPPORTED
 *     otherwise), the tile chosen is at most 128 x 128, and tiles * slices * tile rows * tile columns * 4 bytes
 *     must fit TIR_STATIC_SCRATCH_BYTES and tiles must fit TIR_STATIC_SCRATCH_TILES: a problem beyond that is
 *     TIR_ERR_INVALID_ARG with a message that states both numbers.  Zero-sized M or N is a no-op; K == 0 is
 *     rejected (nothing to split).
 *   Every call on one GPU shares that GPU's array, which keeps the last call's contents: calls that may overlap
 *   on one GPU (two streams, two threads) race and must be serialised by the caller.  Calls on one stream are safe.
 */
#define TIR_STATIC_SCRATCH_BYTES (8u << 20)
#define TIR_STATIC_SCRATCH_TILES 1024
tir_status tir_gemm_split_static(const void* A, const void* B, void* C, int64_t M, int64_t N, int64_t K, int64_t a_rs,
                                 int64_t a_cs, int64_t b_rs, int64_t b_cs, int64_t c_rs, int64_t c_cs, tir_dtype in,
                                 tir_dtype out, const tir_epilogue* ep, int slices, tir_stream stream);

/*
 * Name of the kernel variant the next identical call would launch (for profiling harnesses), e.g.
 * "f16_f32_t256x256w2x4s2_ak_bn"; a "/z<slices>" suffix is the plan for a stream with a registered workspace.  Arguments as for tir_batch_matmul / tir_conv2d without pointers
 * being dereferenced; returns "" on invalid arguments.  The string is static.  out = TIR_I8 asks for the
 * requantising variant of the fused entry points.
 */
const char* tir_gemm_variant(int64_t batch, int64_t M, int64_t N, int64_t K, int64_t a_rs, int64_t a_cs,
                             int64_t b_rs, int64_t b_cs, int64_t c_rs, int64_t c_cs, tir_dtype in,
                             tir_dtype out);
const char* tir_conv2d_variant(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                               int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w,
                               int groups, tir_dtype in, tir_dtype out);
const char* tir_conv3d_variant(int64_t N, int64_t D, int64_t H, int64_t W, int64_t C, int64_t K, int64_t T, int64_t R,
                               int64_t S, int stride_d, int stride_h, int stride_w, int pad_d, int pad_h, int pad_w,
                               int dil_d, int dil_h, int dil_w, int groups, tir_dtype in, tir_dtype out);
/* Likewise for tir_conv2d_transpose; a strided problem computed per output phase reports
 * "<variant>/ph<stride_h>x<stride_w>" (see tir_conv2d_transpose). */
const char* tir_conv2d_transpose_variant(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                                         int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w,
                                         int outpad_h, int outpad_w, int groups, tir_dtype in, tir_dtype out);

/*
 * Choice of kernel variant by measurement (TensorIR paper sec. 4.4: candidates that differ only in the
 * loop structure around the fixed tensorized block are benchmarked on the device; the evaluation's
 * tuning-time discussion: kept records make a second search of the same operator unnecessary).
 *
 * tir_tune_batch_matmul / tir_tune_conv2d take the arguments of tir_batch_matmul_fused / tir_conv2d_fused
 * (batch = 1 with zero batch strides tunes tir_gemm; ep may be NULL), launch every compiled variant that computes this problem
 * - and, where few tiles face a long reduction and `stream` has a registered workspace, the same variant with the
 * reduction split over 2, 3, 4, 6 or 8 workgroups per tile - `reps` times on `stream`, time those within 10 % of the fastest five more
 * times in turn (each keeps its fastest round; a copy ring of three or more slots wins over a two-slot ring that is less than 2 % faster, the
 * trials' operands being warm in the caches), and record the winner under the problem's signature (dtypes, copy
 * modes implied by strides and alignment, extents, convolution geometry).  Later calls of the
 * operator entry points with the same signature use the recorded variant instead of the built-in
 * scoring rule.  Unlike every other call these BLOCK until the trial launches have finished, create
 * and destroy HIP events and graphs (each trial is a captured graph of `reps` launches, so that short
 * kernels are timed at the device's rate; with stream = NULL the trials run on a temporary stream
 * after a device synchronisation), and must not be called during stream capture.  The output buffer ends
 * up holding the operator's result (every variant computes the same values up to summation order).
 * *best_us (may be NULL) receives the winner's time per launch in microseconds (0 for empty problems).
 * reps must be in [1, 1000].
 *
 * Records are process-wide and thread-safe.  tir_tune_save writes them as text (one record per line,
 * variant by name, then the number of reduction slices), tir_tune_load merges a file into the table; lines naming a variant this build
 * does not have, or one that cannot compute the recorded signature, are skipped.
 */
tir_status tir_tune_batch_matmul(const void* A, const void* B, void* C, int64_t batch, int64_t M, int64_t N,
                                 int64_t K, int64_t a_bs, int64_t a_rs, int64_t a_cs, int64_t b_bs, int64_t b_rs,
                                 int64_t b_cs, int64_t c_bs, int64_t c_rs, int64_t c_cs, tir_dtype in,
                                 tir_dtype out, const tir_epilogue* ep, int reps, double* best_us,
                                 tir_stream stream);
tir_status tir_tune_conv2d(const void* x, const void* w, void* y, int64_t N, int64_t H, int64_t W, int64_t C,
                           int64_t K, int64_t R, int64_t S, int stride_h, int stride_w, int pad_h, int pad_w,
                           int dil_h, int dil_w, int groups, tir_dtype in, tir_dtype out,
                           const tir_epilogue* ep, int reps, double* best_us, tir_stream stream);
/* The same for tir_conv3d and tir_conv2d_transpose (arguments as for those entry points). */
tir_status tir_tune_conv3d(const void* x, const void* w, void* y, int64_t N, int64_t D, int64_t H, int64_t W, int64_t C,
                           int64_t K, int64_t T, int64_t R, int64_t S, int stride_d, int stride_h, int stride_w,
                           int pad_d, int pad_h, int pad_w, int dil_d, int dil_h, int dil_w, int groups, tir_dtype in,
                           tir_dtype out, const tir_epilogue* ep, int reps, double* best_us, tir_stream stream);
tir_status tir_tune_conv2d_transpose(const void* x, const void* w, void* y, int64_t N, int64_t H, int64_t W, int64_t C,
                                     int64_t K, int64_t R, int64_t S, int stride_h, int stride_w, int pad_h, int pad_w,
                                     int dil_h, int dil_w, int outpad_h, int outpad_w, int groups, tir_dtype in,
                                     tir_dtype out, const tir_epilogue* ep, int reps, double* best_us,
                                     tir_stream stream);
int tir_tune_count(void);                       /* number of records */
void tir_tune_clear(void);                      /* forget every record */
tir_status tir_tune_save(const char* path);     /* TIR_ERR_INVALID_ARG if the file cannot be written */
tir_status tir_tune_load(const char* path);     /* TIR_ERR_INVALID_ARG if it cannot be read or is not a record file */

/*
 * Testing / tuning hooks (process-wide, not thread-safe).
 * tir_debug_force_tile: make later calls use the bm x bn workgroup tile when the chosen copy mode
 * has such a variant (0,0 restores the automatic choice).
 * tir_debug_tile_of_block: host copy of the kernels' workgroup-id -> output-tile map (a bijection
 * of [0, tiles_m*tiles_n) that keeps the tiles of one L2 domain adjacent).
 */
void tir_debug_force_tile(int bm, int bn);
/* Force the first variant of the matching dtype / copy mode whose name contains name_part
 * ("" or NULL restores the automatic choice); tir_debug_variant_name enumerates the names. */
void tir_debug_force_variant(const char* name_part);
/* Make later calls split every tile's reduction over `slices` workgroups where the chosen variant, the
 * reduction's length and the stream's registered workspace allow it (0 or 1 restores the automatic choice, measured records
 * are ignored meanwhile).  The variant queries report a split as "<variant>/z<slices>". */
void tir_debug_force_ksplit(int slices);
int tir_debug_variant_count(void);
const char* tir_debug_variant_name(int i);
void tir_debug_tile_of_block(int bid, int tiles_m, int tiles_n, int* tm, int* tn);
/* Host copy of the kernels' division by a launch constant: m / d for d >= 1 and m < 2^31 through the
 * multiply-and-shift constants the planner derives from d (used to decode output rows into pixels). */
unsigned tir_debug_fastdiv(unsigned d, unsigned m);

/*
 * Measurement aid: enqueue a register-only fp16 MFMA loop (no memory traffic) of `iters` x 16 MFMAs
 * per wave on 1024 workgroups and report its FLOP count in *flop (may be NULL).  Timed by the
 * caller, it gives the rate the matrix pipes sustain at the clock the power management allows:
 * operands are constants (random_operands = 0) or pseudo-random values in (-1, 1).  `sink` is a
 * device pointer to at least 32 bytes, 4-byte aligned: word 0 is practically never written; one wave in the middle
 * of the grid stores the low words of the shader-clock counter and of the 100 MHz constant counter before its loop
 * (words 1, 2) and after it (words 3, 4).  (word 3 - word 1) / ((word 4 - word 2) * 10 ns) is the shader clock the
 * power management held, and iters * 16 * 32 / (word 3 - word 1) the share of those cycles that SIMD's matrix pipe
 * was busy (an MFMA of this shape occupies it for 32 cycles).
 */
tir_status tir_probe_mfma_rate(void* sink, int iters, int random_operands, double* flop, tir_stream stream);

/* Library version as "major.minor". */
const char* tir_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TIR_H_ */
