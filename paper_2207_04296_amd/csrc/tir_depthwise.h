// Depth-wise convolution (groups = channels, one filter per channel): the paper's DEP workload.  There
// is no contraction over channels, so nothing here maps onto a matrix intrinsic: the operator is bound
// by memory traffic and plain vector arithmetic, and the right decomposition is the direct one - each
// thread owns one output pixel x one 16-byte vector of channels, reads the R*S input vectors its taps
// touch (neighbouring pixels share them through the caches) and multiplies element by element with the
// filter taps, which the workgroup keeps in LDS as [tap][channel] in the accumulator's type.
//   y[n,p,q,c] = sum_{r,s} x[n, p*s_h - pad_h + r*d_h, q*s_w - pad_w + s*d_w, c] * w[c,r,s]      (sec. 4.2 formula with groups = C)
#pragma once
#include "tir_kernel.h"
#ifndef TIR_DW_NPIX
#define TIR_DW_NPIX 2
#endif
#define TIR_DW_NPIX_DEFAULT TIR_DW_NPIX

namespace tir {

template <int DT> struct DwIn;
template <> struct DwIn<DT_F16> {
    typedef float acc_e;
    static __device__ __forceinline__ float get(const uint4& v, int e) {
        typedef _Float16 h8 __attribute__((ext_vector_type(8)));
        return (float)__builtin_bit_cast(h8, v)[e];
    }
    static __device__ __forceinline__ float w(unsigned short bits) { return (float)__builtin_bit_cast(_Float16, bits); }
};
template <> struct DwIn<DT_BF16> {
    typedef float acc_e;
    static __device__ __forceinline__ float get(const uint4& v, int e) {
        const unsigned u = ((const unsigned*)&v)[e >> 1];
        return __uint_as_float((e & 1) ? (u & 0xffff0000u) : (u << 16));
    }
    static __device__ __forceinline__ float w(unsigned short bits) { return __uint_as_float((unsigned)bits << 16); }
};
template <> struct DwIn<DT_I8> {
    typedef int acc_e;
    static __device__ __forceinline__ int get(const uint4& v, int e) {
        const int u = (int)((const unsigned*)&v)[e >> 2];
        return (u << (24 - 8 * (e & 3))) >> 24;       // sign-extended byte e
    }
    static __device__ __forceinline__ int w(signed char bits) { return (int)bits; }
};

constexpr int kDwChannels = 64;     // channels per workgroup
constexpr int kDwPixPerThread = TIR_DW_NPIX_DEFAULT;
constexpr int kDwMaxTaps = 128;     // R*S limit of this kernel (the [tap][64] filter table in LDS)

// R3S3: the filter is 3x3 (the common case): the nine input vectors of a pixel are requested together.
template <int DT, int OUT, bool R3S3, bool STREAM>
__global__ void __launch_bounds__(256) depthwise_kernel(const Params p) {
    typedef typename DwIn<DT>::acc_e acc_e;
    typedef OutTraits<OUT> OT;
    typedef typename OT::type out_t;
    typedef typename std::conditional<DT == DT_I8, signed char, unsigned short>::type in_t;
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    constexpr int ES = elem_size(DT), VEC = 16 / ES;
    constexpr int CV = kDwChannels / VEC;            // channel vectors per workgroup
    constexpr int PP = 256 / CV;                     // pixels per pass of the workgroup
    constexpr int NPIX = kDwPixPerThread;            // pixels per thread

    __shared__ acc_e wt[R3S3 ? 1 : kDwMaxTaps * kDwChannels];

    const int tid = threadIdx.x;
    const int cv = tid % CV, pl = tid / CV;
    const int cbase = blockIdx.y * kDwChannels;
    const int c0 = cbase + cv * VEC;
    const int RS = p.R * p.S;
    const in_t* wsrc = (const in_t*)p.B;
    // 3x3: the thread's VEC channels x 9 taps are 9 consecutive 16-byte vectors of the filter (channel-major,
    // element (channel e, tap t) at position 9*e + t): they go to registers and stay there for all its pixels.
    uint4 wv[R3S3 ? 9 : 1];                  // kept packed: the multiply-add reads 16-bit operands directly
    if constexpr (R3S3) {
        if (c0 >= p.Cin) return;
#pragma unroll
        for (int i = 0; i < 9; ++i) wv[i] = ((const uint4*)(wsrc + (long long)c0 * 9))[i];
    } else {
        for (int idx = tid; idx < RS * kDwChannels; idx += 256) {
            const int t = idx / kDwChannels, ch = idx % kDwChannels;
            wt[idx] = cbase + ch < p.Cin ? DwIn<DT>::w(wsrc[(long long)(cbase + ch) * RS + t]) : (acc_e)0;
        }
    }
    // bias of the thread's channels (requested early: its latency overlaps the first input loads)
    acc_e bias_r[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) bias_r[e] = (p.bias && c0 < p.Cin) ? ((const acc_e*)p.bias)[c0 + e] : (acc_e)0;
    if constexpr (!R3S3) {
        __syncthreads();
        if (c0 >= p.Cin) return;
    }

    const int PQ = p.P * p.Q;
    // consecutive workgroup ids go to different XCDs (L2s): regroup them so that each XCD owns a contiguous
    // range of pixels and finds the rows its neighbouring taps share in its own L2
    int bx = blockIdx.x;
    {
        const int nb = (p.M + NPIX * PP - 1) / (NPIX * PP), nb8 = nb - nb % kXcds;      // = gridDim.x (a hidden argument, fetched late)
        if (bx < nb8) bx = (bx % kXcds) * (nb8 / kXcds) + bx / kXcds;
    }
    // taps outside the image read through the descriptor's range check: zeros, and no branch around the load
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void*)p.A, 0, (int)((long long)p.batch_imgs * p.H * p.W * p.Cin * ES), 0x00020000);
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(p.C, 0, (int)((long long)p.M * p.Cin * (int)sizeof(out_t)), 0x00020000);
    const acc_e* wcol = wt + (R3S3 ? 0 : cv * VEC);
#pragma unroll
    for (int j = 0; j < NPIX; ++j) {
        const int m = (bx * NPIX + j) * PP + pl;
        if (m >= p.M) break;
        const int img = (int)fastdiv((unsigned)m, p.div_pq_magic, p.div_pq_shift), rem = m - img * PQ;
        const int op = (int)fastdiv((unsigned)rem, p.div_q_magic, p.div_q_shift), oq = rem - op * p.Q;
        const int ih0 = op * p.stride_h - p.pad_h, iw0 = oq * p.stride_w - p.pad_w;
        const int pix0 = (img * p.H + ih0) * p.W + iw0;              // may be "negative": only used when the tap is valid
        acc_e acc[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] = 0;                    // reduction init
        auto tap_off = [&](int r, int s) -> int {
            const int ih = ih0 + r * p.dil_h, iw = iw0 + s * p.dil_w;
            const bool ok = (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
            return ok ? ((pix0 + r * p.dil_h * p.W + s * p.dil_w) * p.Cin + c0) * ES : (int)kOutOfRange;
        };
        if constexpr (R3S3) {
            u32x4 v[9];
#pragma unroll
            for (int t = 0; t < 9; ++t) v[t] = __builtin_amdgcn_raw_buffer_load_b128(rx, tap_off(t / 3, t % 3), 0, 0);
#pragma unroll
            for (int t = 0; t < 9; ++t) {
                const uint4 u = __builtin_bit_cast(uint4, v[t]);
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[e] += DwIn<DT>::get(u, e) * DwIn<DT>::get(wv[(9 * e + t) / VEC], (9 * e + t) % VEC);
            }
        } else {
            for (int r = 0; r < p.R; ++r)
                for (int s = 0; s < p.S; ++s) {
                    const uint4 u = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rx, tap_off(r, s), 0, 0));
                    const acc_e* wrow = wcol + (r * p.S + s) * kDwChannels;
#pragma unroll
                    for (int e = 0; e < VEC; ++e) acc[e] += DwIn<DT>::get(u, e) * wrow[e];
                }
        }
        alignas(16) out_t o[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) o[e] = finish_value<OUT>(consumer(acc[e], bias_r[e], p.relu), p.scale);
        constexpr int OB = VEC * (int)sizeof(out_t);                 // 16 .. 64 bytes
        static_assert(OB % 16 == 0, "");
        const int obyte = (m * p.Cin + c0) * (int)sizeof(out_t);     // < 2^31: checked by the host
#pragma unroll
        for (int b = 0; b < OB; b += 16)
            __builtin_amdgcn_raw_buffer_store_b128(*(const u32x4*)((const char*)o + b), ry, obyte + b, 0, STREAM ? TIR_STORE_AUX_STREAM : TIR_STORE_AUX);   // write-through, like every epilogue
    }
}

// 3x3 filter, undilated along the width, stride 1 or 2 there (SW): a thread owns four horizontally adjacent output
// pixels x one 16-byte channel vector.  Their taps touch 3 rows x NC = 3*SW + 3 consecutive input columns, loaded
// once (18 vectors for 4 pixels at stride 1 instead of 36) and all requested before the first multiply; row and
// column validity are decided once per row / column, so a tap's address costs three vector instructions instead
// of a dozen.  The one-pixel kernel above spent twice as many instructions on addresses as on multiply-adds.
// STREAM (the output policy) is a template parameter, not a branch: a branch around each store splits the pixel loop
// into blocks, and the compiler then waits for the previous pixel's stores before the next pixel's arithmetic
// (measured: 6.9 -> 8.8 us).
template <int DT, int OUT, int SW, bool STREAM>
__global__ void __launch_bounds__(256) depthwise3x3_blocked_kernel(const Params p) {
    typedef typename DwIn<DT>::acc_e acc_e;
    typedef OutTraits<OUT> OT;
    typedef typename OT::type out_t;
    typedef typename std::conditional<DT == DT_I8, signed char, unsigned short>::type in_t;
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    constexpr int ES = elem_size(DT), VEC = 16 / ES;
    constexpr int CV = kDwChannels / VEC;            // channel vectors per workgroup
    constexpr int PP = 256 / CV;                     // pixel groups per workgroup
    constexpr int NP = kDwBlockPix, NC = (NP - 1) * SW + 3;

    // every argument the kernel reads, fetched in one batch
    asm volatile("" ::"s"(p.A), "s"(p.B), "s"(p.C), "s"(p.M), "s"(p.bias), "s"(p.relu), "s"(p.scale), "s"(p.batch_imgs), "s"(p.H), "s"(p.W), "s"(p.Cin),
                 "s"(p.P), "s"(p.Q), "s"(p.stride_h), "s"(p.pad_h), "s"(p.pad_w), "s"(p.dil_h));
    asm volatile("" ::"s"(p.div_dwq_magic), "s"(p.div_dwq_shift), "s"(p.div_dwpq_magic), "s"(p.div_dwpq_shift));
    const int tid = threadIdx.x;
    const int cv = tid % CV, pl = tid / CV;
    const int c0 = blockIdx.y * kDwChannels + cv * VEC;
    if (c0 >= p.Cin) return;
    const in_t* wsrc = (const in_t*)p.B;
    uint4 wv[9];                                     // VEC channels x 9 taps, element (channel e, tap t) at 9*e + t
#pragma unroll
    for (int i = 0; i < 9; ++i) wv[i] = ((const uint4*)(wsrc + (long long)c0 * 9))[i];
    acc_e bias_r[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) bias_r[e] = p.bias ? ((const acc_e*)p.bias)[c0 + e] : (acc_e)0;

    const int QG = (p.Q + NP - 1) / NP;              // pixel groups per output row
    int bx = blockIdx.x;                             // each XCD owns a contiguous range of pixel groups (shared rows stay in its L2)
    {
        const int nb = (p.batch_imgs * p.P * QG + PP - 1) / PP, nb8 = nb - nb % kXcds;      // = gridDim.x (a hidden argument, fetched late)
        if (bx < nb8) bx = (bx % kXcds) * (nb8 / kXcds) + bx / kXcds;
    }
    const int gidx = bx * PP + pl;
    if (gidx >= p.batch_imgs * p.P * QG) return;
    const int img = (int)fastdiv((unsigned)gidx, p.div_dwpq_magic, p.div_dwpq_shift), rem = gidx - img * (p.P * QG);
    const int op = (int)fastdiv((unsigned)rem, p.div_dwq_magic, p.div_dwq_shift), oq0 = (rem - op * QG) * NP;
    const int ih0 = op * p.stride_h - p.pad_h, iw0 = oq0 * SW - p.pad_w;

    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void*)p.A, 0, (int)((long long)p.batch_imgs * p.H * p.W * p.Cin * ES), 0x00020000);
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(p.C, 0, (int)((long long)p.M * p.Cin * (int)sizeof(out_t)), 0x00020000);
    const int cstep = p.Cin * ES;                    // bytes from one input column to the next
    bool col_ok[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) col_ok[c] = (unsigned)(iw0 + c) < (unsigned)p.W;
    u32x4 v[3][NC];
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const int ih = ih0 + r * p.dil_h;
        const bool row_ok = (unsigned)ih < (unsigned)p.H;
        int row_off = (((img * p.H + ih) * p.W + iw0) * p.Cin + c0) * ES;           // only used where the tap is inside the image
        asm volatile("" : "+v"(row_off));      // (kept as one value: re-associated with the column, every load's address became a multiply)
#pragma unroll
        for (int c = 0; c < NC; ++c)
            v[r][c] = __builtin_amdgcn_raw_buffer_load_b128(rx, (row_ok && col_ok[c]) ? row_off + c * cstep : (int)kOutOfRange, 0, 0);
    }
    const int out_pix0 = (img * p.P + op) * p.Q + oq0;
#pragma unroll
    for (int j = 0; j < NP; ++j) {
        acc_e acc[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] = 0;                    // reduction init
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const uint4 u = __builtin_bit_cast(uint4, v[t / 3][j * SW + t % 3]);
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] += DwIn<DT>::get(u, e) * DwIn<DT>::get(wv[(9 * e + t) / VEC], (9 * e + t) % VEC);
        }
        alignas(16) out_t o[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) o[e] = finish_value<OUT>(consumer(acc[e], bias_r[e], p.relu), p.scale);
        constexpr int OB = VEC * (int)sizeof(out_t);
        const int obyte = oq0 + j < p.Q ? ((out_pix0 + j) * p.Cin + c0) * (int)sizeof(out_t) : (int)kOutOfRange;      // < 2^31: checked by the host
#pragma unroll
        for (int b = 0; b < OB; b += 16)
            __builtin_amdgcn_raw_buffer_store_b128(*(const u32x4*)((const char*)o + b), ry, obyte + b, 0, STREAM ? TIR_STORE_AUX_STREAM : TIR_STORE_AUX);
    }
}

typedef hipError_t (*dw_launch_fn)(const Params&, hipStream_t);
// (dt, out) -> launcher, or null when the pair is not compiled
dw_launch_fn depthwise_launcher(int dt, int out);

}  // namespace tir
