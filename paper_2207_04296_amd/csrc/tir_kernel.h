// The tensorized contraction kernel for gfx950 (CDNA4), one template for GEMM, batched matmul and
// implicit-im2col conv2d.
//
// Structure (names follow the TensorIR paper, sections 3.1 and 4):
//   - the output is cut into BM x BN workgroup tiles, each wave owns a TM x TN sub-tile made of
//     32x32 "blocks"; one block instance is one MFMA (the tensor intrinsic C[x,y] += A[x,k]*B[k,y]
//     over a 32 x 32 x (32 bytes of k) tile) and the reduction iterator k stays serial per tile;
//   - data movement is its own stage ("AutoCopy"): global -> registers -> LDS with 16-byte
//     vectors fetched cooperatively by the whole workgroup, two LDS stages so that the global
//     loads of K-slab i+1 are in flight while slab i is multiplied, and an XOR swizzle of the
//     16-byte columns instead of stride padding to keep the LDS reads free of bank conflicts;
//   - accumulators start at zero (reduction init) and the epilogue converts and stores them
//     straight from registers.
//
// One K-slab is 128 bytes of k per row (64 fp16/bf16 or 128 int8 values) = 4 MFMA k-steps.
#pragma once
#include <hip/hip_runtime.h>
#include <type_traits>
#include "tir_params.h"

namespace tir {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
typedef short i16x4 __attribute__((ext_vector_type(4)));

#define TIR_LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

// ---------------------------------------------------------------------------------------------
// Per input dtype: element size and the MFMA that consumes 16 bytes of k per lane.
// Operand layout of the 32x32 MFMAs (checked on hardware): lane l supplies row (l & 31) and the
// 16 bytes of k starting at 16*(l >> 5); D register r of lane l is element
// (row 8*(r/4) + 4*(l>>5) + r%4 of the first operand, row l&31 of the second operand).
// ---------------------------------------------------------------------------------------------
template <int DT> struct InTraits;
template <> struct InTraits<DT_F16> {
    static constexpr int ES = 2;
    typedef f32x16 acc_t;
    typedef float accs_t;
    static __device__ __forceinline__ acc_t mfma(const uint4& a, const uint4& b, acc_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};
template <> struct InTraits<DT_BF16> {
    static constexpr int ES = 2;
    typedef f32x16 acc_t;
    typedef float accs_t;
    static __device__ __forceinline__ acc_t mfma(const uint4& a, const uint4& b, acc_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct InTraits<DT_I8> {
    static constexpr int ES = 1;
    typedef i32x16 acc_t;
    typedef int accs_t;
    static __device__ __forceinline__ acc_t mfma(const uint4& a, const uint4& b, acc_t c) {
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(i32x4, a), __builtin_bit_cast(i32x4, b), c, 0, 0, 0);
    }
};

// Output conversion (round to nearest even for the 16-bit floats).
template <int OUT> struct OutTraits;
template <> struct OutTraits<DT_F32> {
    typedef float type;
    static __device__ __forceinline__ float cvt(float v) { return v; }
};
template <> struct OutTraits<DT_I32> {
    typedef int type;
    static __device__ __forceinline__ int cvt(int v) { return v; }
};
template <> struct OutTraits<DT_F16> {
    typedef _Float16 type;
    static __device__ __forceinline__ _Float16 cvt(float v) { return (_Float16)v; }
};
template <> struct OutTraits<DT_BF16> {
    typedef unsigned short type;
    static __device__ __forceinline__ unsigned short cvt(float v) {
        unsigned int u = __float_as_uint(v);
        if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40u);  // quiet NaN
        u += 0x7fffu + ((u >> 16) & 1u);
        return (unsigned short)(u >> 16);
    }
};

// Byte offset of 16-byte column `chunk` of `row` inside a [rows][128 B] K-major LDS tile.
// Column index XOR (row/2 mod 8): 16 consecutive rows read at one logical column then touch all
// 64 banks exactly once.
__device__ __forceinline__ int kmajor_off(int row, int chunk) {
    return row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4);
}

// XOR applied to the byte offset inside k-row `k` of an N-major LDS tile so that the k-rows one
// transposing read touches fall into different banks.
template <class C> __device__ __forceinline__ int nmajor_xor(int k) {
    return ((k / C::RPW) % C::NSEG) * C::SEG;
}

template <class C>
__global__ void __launch_bounds__(C::THREADS) contract_kernel(const Params p) {
    typedef InTraits<C::DT> IT;
    typedef OutTraits<C::OUT> OT;
    typedef typename IT::acc_t acc_t;
    constexpr int ES = C::ES, VEC = C::VEC, BK = C::BK;

    __shared__ __attribute__((aligned(16))) char smem[C::LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / C::WN, wn = wave % C::WN;

    int tm, tn;
    tile_of_block(blockIdx.x, p.tiles_m, p.tiles_n, &tm, &tn);
    const int m0 = tm * C::BM, n0 = tn * C::BN;
    const long long bz = blockIdx.y;

    const char* __restrict__ Ab = (const char*)p.A + bz * p.a_bs * ES;
    const char* __restrict__ Bb = (const char*)p.B + bz * p.b_bs * ES;

    // ---------------------------------------------------------------- copy-stage bookkeeping
    // A chunk q = tid + i*THREADS covers row q/8, 16-byte column q%8 of the [BM][128 B] tile.
    const int a_c = tid & 7;
    const int a_r0 = tid >> 3;
    constexpr int A_RSTEP = C::THREADS / 8;
    unsigned a_off[C::A_IT];       // A_KMAJOR: byte offset from the tile base; A_CONV: element base
    int a_hw[C::A_IT];             // A_CONV*: (ih0 << 16) | (iw0 & 0xffff) of the row's output pixel
    const char* a_tile = Ab;
    if constexpr (C::AMODE == A_KMAJOR) {
        a_tile = Ab + (long long)m0 * p.a_rs * ES;
#pragma unroll
        for (int i = 0; i < C::A_IT; ++i) {
            int r = a_r0 + i * A_RSTEP;
            int rc = m0 + r < p.M ? r : p.M - 1 - m0;   // rows past M re-read the last row; never stored
            a_off[i] = (unsigned)rc * (unsigned)(p.a_rs * ES) + a_c * 16;
        }
    } else if constexpr (C::AMODE == A_CONV || C::AMODE == A_CONV_GENERIC) {
        const int PQ = p.P * p.Q;
#pragma unroll
        for (int i = 0; i < C::A_IT; ++i) {
            int m = m0 + a_r0 + i * A_RSTEP;
            int ih0 = -30000, iw0 = 0, img = 0;
            if (m < p.M) {
                img = m / PQ;
                int rem = m - img * PQ;
                int op = rem / p.Q, oq = rem - op * p.Q;
                ih0 = op * p.stride_h - p.pad_h;
                iw0 = oq * p.stride_w - p.pad_w;
            }
            // element offset of (img, ih0, iw0, 0); may be "negative" (padding) - kept modulo 2^32
            a_off[i] = (((unsigned)img * (unsigned)p.H + (unsigned)ih0) * (unsigned)p.W + (unsigned)iw0) * (unsigned)p.Cin;
            a_hw[i] = (ih0 << 16) | (iw0 & 0xffff);
        }
    }

    // B chunk bookkeeping
    const int b_c = (C::BMODE == B_NMAJOR) ? tid % C::B_RC : (tid & 7);
    const int b_r0 = (C::BMODE == B_NMAJOR) ? tid / C::B_RC : (tid >> 3);
    constexpr int B_RSTEP = (C::BMODE == B_NMAJOR) ? C::THREADS / C::B_RC : C::THREADS / 8;
    unsigned b_off[C::B_IT];
    const char* b_tile = Bb;
    if constexpr (C::BMODE == B_KMAJOR) {
        b_tile = Bb + (long long)n0 * p.b_cs * ES;
#pragma unroll
        for (int i = 0; i < C::B_IT; ++i) {
            int r = b_r0 + i * B_RSTEP;
            int rc = n0 + r < p.N ? r : p.N - 1 - n0;
            b_off[i] = (unsigned)rc * (unsigned)(p.b_cs * ES) + b_c * 16;
        }
    } else if constexpr (C::BMODE == B_NMAJOR) {
        // k-row b_r0 + i*B_RSTEP of the slab, columns n0 + b_c*VEC ...; columns past N re-read column 0
        int col = n0 + b_c * VEC < p.N ? n0 + b_c * VEC : 0;
        b_tile = Bb + (long long)col * ES;   // per-thread base (not uniform)
#pragma unroll
        for (int i = 0; i < C::B_IT; ++i) b_off[i] = 0;
    }

    uint4 ra[C::A_IT], rb[C::B_IT];

    auto load_a = [&](int slab) {
        const int k0 = slab * BK;
        if constexpr (C::AMODE == A_KMAJOR) {
            const bool kv = k0 + a_c * VEC < p.K;
            const char* base = a_tile + (long long)k0 * ES;
#pragma unroll
            for (int i = 0; i < C::A_IT; ++i) {
                ra[i] = make_uint4(0, 0, 0, 0);
                if (kv) ra[i] = *(const uint4*)(base + a_off[i]);
            }
        } else if constexpr (C::AMODE == A_CONV) {
            // fuse(rh, rw, rc) -> (rh, rw, rc); a 16-byte vector never straddles a tap (Cg % VEC == 0)
            const int kb = k0 + a_c * VEC;
            const int tap = kb / p.Cg;
            const int cc = kb - tap * p.Cg;
            const int fr = tap / p.S, fs = tap - fr * p.S;
            const int dh = fr * p.dil_h, dw = fs * p.dil_w;
            const unsigned delta = (unsigned)((dh * p.W + dw) * p.Cin + cc);
            const bool kv = kb < p.K;
#pragma unroll
            for (int i = 0; i < C::A_IT; ++i) {
                int ih = (a_hw[i] >> 16) + dh;
                int iw = (int)(short)(a_hw[i] & 0xffff) + dw;
                bool ok = kv && (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
                ra[i] = make_uint4(0, 0, 0, 0);
                if (ok) ra[i] = *(const uint4*)(Ab + (long long)(int)(a_off[i] + delta) * ES);
            }
        } else if constexpr (C::AMODE == A_GENERIC) {
            typedef typename std::conditional<ES == 2, unsigned short, unsigned char>::type elem_t;
            const elem_t* A = (const elem_t*)Ab;
#pragma unroll
            for (int i = 0; i < C::A_IT; ++i) {
                alignas(16) elem_t v[VEC];
                const long long m = m0 + a_r0 + i * A_RSTEP;
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const long long k = k0 + a_c * VEC + e;
                    v[e] = (m < p.M && k < p.K) ? A[m * p.a_rs + k * p.a_cs] : (elem_t)0;
                }
                ra[i] = *(const uint4*)v;
            }
        } else {  // A_CONV_GENERIC: element-wise implicit im2col
            typedef typename std::conditional<ES == 2, unsigned short, unsigned char>::type elem_t;
            const elem_t* A = (const elem_t*)Ab;
#pragma unroll
            for (int i = 0; i < C::A_IT; ++i) {
                alignas(16) elem_t v[VEC];
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const int kb = k0 + a_c * VEC + e;
                    const int tap = kb / p.Cg;
                    const int cc = kb - tap * p.Cg;
                    const int fr = tap / p.S, fs = tap - fr * p.S;
                    const int dh = fr * p.dil_h, dw = fs * p.dil_w;
                    int ih = (a_hw[i] >> 16) + dh;
                    int iw = (int)(short)(a_hw[i] & 0xffff) + dw;
                    bool ok = kb < p.K && (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
                    v[e] = ok ? A[(long long)(int)(a_off[i] + (unsigned)((dh * p.W + dw) * p.Cin + cc))] : (elem_t)0;
                }
                ra[i] = *(const uint4*)v;
            }
        }
    };

    auto load_b = [&](int slab) {
        const int k0 = slab * BK;
        if constexpr (C::BMODE == B_KMAJOR) {
            const bool kv = k0 + b_c * VEC < p.K;
            const char* base = b_tile + (long long)k0 * ES;
#pragma unroll
            for (int i = 0; i < C::B_IT; ++i) {
                rb[i] = make_uint4(0, 0, 0, 0);
                if (kv) rb[i] = *(const uint4*)(base + b_off[i]);
            }
        } else if constexpr (C::BMODE == B_NMAJOR) {
#pragma unroll
            for (int i = 0; i < C::B_IT; ++i) {
                const int k = k0 + b_r0 + i * B_RSTEP;
                rb[i] = make_uint4(0, 0, 0, 0);
                if (k < p.K) rb[i] = *(const uint4*)(b_tile + (long long)k * p.b_rs * ES);
            }
        } else {  // B_GENERIC -> K-major LDS tile
            typedef typename std::conditional<ES == 2, unsigned short, unsigned char>::type elem_t;
            const elem_t* B = (const elem_t*)Bb;
#pragma unroll
            for (int i = 0; i < C::B_IT; ++i) {
                alignas(16) elem_t v[VEC];
                const long long n = n0 + b_r0 + i * B_RSTEP;
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const long long k = k0 + b_c * VEC + e;
                    v[e] = (n < p.N && k < p.K) ? B[k * p.b_rs + n * p.b_cs] : (elem_t)0;
                }
                rb[i] = *(const uint4*)v;
            }
        }
    };

    auto store_ab = [&](int buf) {
        char* sa = smem + buf * C::STAGE_BYTES;
        char* sb = sa + C::A_BYTES;
#pragma unroll
        for (int i = 0; i < C::A_IT; ++i) *(uint4*)(sa + kmajor_off(a_r0 + i * A_RSTEP, a_c)) = ra[i];
        if constexpr (C::BMODE == B_NMAJOR) {
#pragma unroll
            for (int i = 0; i < C::B_IT; ++i) {
                const int k = b_r0 + i * B_RSTEP;
                *(uint4*)(sb + k * C::BROW + ((b_c * 16) ^ nmajor_xor<C>(k))) = rb[i];
            }
        } else {
#pragma unroll
            for (int i = 0; i < C::B_IT; ++i) *(uint4*)(sb + kmajor_off(b_r0 + i * B_RSTEP, b_c)) = rb[i];
        }
    };

    // ---------------------------------------------------------------- MFMA-stage bookkeeping
    const int l31 = lane & 31, g = lane >> 5;
    const int a_frag_base = (wm * C::TM + l31) * 128;
    const int b_frag_base = (wn * C::TN + l31) * 128;
    const int sw = (l31 >> 1) & 7;    // (row>>1)&7 is the same for every 32-row block of this lane
    // transposing read of an N-major B tile works on groups of 16 lanes
    const int blk = lane >> 4, s16 = lane & 15;

    acc_t acc[C::MI][C::NI];
#pragma unroll
    for (int i = 0; i < C::MI; ++i)
#pragma unroll
        for (int j = 0; j < C::NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;   // reduction init

    auto compute = [&](int buf) {
        const char* sa = smem + buf * C::STAGE_BYTES;
        const char* sb = sa + C::A_BYTES;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            uint4 af[C::MI], bf[C::NI];
            const int col = ((2 * kk + g) ^ sw) << 4;
#pragma unroll
            for (int i = 0; i < C::MI; ++i) af[i] = *(const uint4*)(sa + a_frag_base + i * 32 * 128 + col);
            if constexpr (C::BMODE == B_NMAJOR) {
#pragma unroll
                for (int j = 0; j < C::NI; ++j) {
                    if constexpr (ES == 2) {
                        // 16-lane group `blk` covers columns 16*(blk&1).. of the 32-wide block and the
                        // k-group blk>>1; lane s fetches 4 values of k-row (s>>2) at columns 4*(s&3)..;
                        // after the transpose lane s holds 4 consecutive k of column s.
                        const int nloc = wn * C::TN + j * 32 + 16 * (blk & 1) + 4 * (s16 & 3);
                        i16x4 h[2];
#pragma unroll
                        for (int hh = 0; hh < 2; ++hh) {
                            const int k = kk * 16 + 8 * (blk >> 1) + 4 * hh + (s16 >> 2);
                            const char* ptr = sb + k * C::BROW + ((nloc * 2) ^ nmajor_xor<C>(k));
                            h[hh] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(TIR_LDS_PTR(i16x4, ptr));
                        }
                        bf[j] = make_uint4(0, 0, 0, 0);
                        __builtin_memcpy(&bf[j], &h[0], 8);
                        __builtin_memcpy((char*)&bf[j] + 8, &h[1], 8);
                    } else {
                        // int8: lane s fetches 8 values of k-row (s>>1) at columns 8*(s&1)..
                        const int nloc = wn * C::TN + j * 32 + 16 * (blk & 1) + 8 * (s16 & 1);
                        i32x2 h[2];
#pragma unroll
                        for (int hh = 0; hh < 2; ++hh) {
                            const int k = kk * 32 + 16 * (blk >> 1) + 8 * hh + (s16 >> 1);
                            const char* ptr = sb + k * C::BROW + (nloc ^ nmajor_xor<C>(k));
                            h[hh] = __builtin_amdgcn_ds_read_tr8_b64_v2i32(TIR_LDS_PTR(i32x2, ptr));
                        }
                        bf[j] = make_uint4((unsigned)h[0][0], (unsigned)h[0][1], (unsigned)h[1][0], (unsigned)h[1][1]);
                    }
                }
            } else {
#pragma unroll
                for (int j = 0; j < C::NI; ++j) bf[j] = *(const uint4*)(sb + b_frag_base + j * 32 * 128 + col);
            }
#pragma unroll
            for (int i = 0; i < C::MI; ++i)
#pragma unroll
                for (int j = 0; j < C::NI; ++j) acc[i][j] = IT::mfma(af[i], bf[j], acc[i][j]);
        }
    };

    // ---------------------------------------------------------------- main loop over K-slabs
    const int nslab = (p.K + BK - 1) / BK;
    if (nslab > 0) {
        load_a(0);
        load_b(0);
        store_ab(0);
        __syncthreads();
        for (int s = 0; s < nslab; ++s) {
            const int cur = s & 1;
            const bool more = s + 1 < nslab;
            if (more) {
                load_a(s + 1);
                load_b(s + 1);
            }
            compute(cur);
            if (more) store_ab(cur ^ 1);
            __syncthreads();
        }
    }

    // ---------------------------------------------------------------- fused epilogue
    typedef typename OT::type out_t;
    out_t* __restrict__ Cb = (out_t*)p.C + bz * p.c_bs;
#pragma unroll
    for (int i = 0; i < C::MI; ++i) {
#pragma unroll
        for (int j = 0; j < C::NI; ++j) {
            const int col = n0 + wn * C::TN + j * 32 + l31;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm * C::TM + i * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                if (row < p.M && col < p.N) Cb[(long long)row * p.c_rs + (long long)col * p.c_cs] = OT::cvt(acc[i][j][r]);
            }
        }
    }
}

}  // namespace tir
