// The tensorized contraction kernels for gfx950 (CDNA4): one template family for GEMM, batched
// matmul and implicit-im2col conv2d.
//
// Structure (names follow the TensorIR paper, sections 3.1 and 4):
//   - the output is cut into BM x BN workgroup tiles, each wave owns a TM x TN sub-tile made of
//     32x32 "blocks"; one block instance is one MFMA (the tensor intrinsic C[x,y] += A[x,k]*B[k,y]
//     over a 32 x 32 x (32 bytes of k) tile) and the reduction iterator k stays serial per tile;
//   - data movement is its own stage ("AutoCopy"): the whole workgroup fetches 16-byte vectors
//     cooperatively straight from global memory into LDS (buffer loads with the LDS destination,
//     no register hop; out-of-range lanes deliver zeros, which is the padding of ragged tiles),
//     two LDS stages so that K-slab i+1 is in flight while slab i is multiplied, and an XOR
//     swizzle of the 16-byte columns instead of stride padding to keep LDS reads conflict-free;
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
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
typedef short i16x4 __attribute__((ext_vector_type(4)));

#define TIR_LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))
// Nothing is scheduled across this point.
#define TIR_FENCE() __builtin_amdgcn_sched_barrier(0)

// ---------------------------------------------------------------------------------------------
// Per input dtype: the MFMA that consumes 16 bytes of k per lane.
// Operand layout of the 32x32 MFMAs (checked on hardware): lane l supplies row (l & 31) and the
// 16 bytes of k starting at 16*(l >> 5); D register r of lane l is element
// (row 8*(r/4) + 4*(l>>5) + r%4 of the first operand, row l&31 of the second operand).
// ---------------------------------------------------------------------------------------------
template <int DT> struct InTraits;
template <> struct InTraits<DT_F16> {
    typedef f32x16 acc_t;
    static __device__ __forceinline__ acc_t mfma(const uint4& a, const uint4& b, acc_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
};
template <> struct InTraits<DT_BF16> {
    typedef f32x16 acc_t;
    static __device__ __forceinline__ acc_t mfma(const uint4& a, const uint4& b, acc_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct InTraits<DT_I8> {
    typedef i32x16 acc_t;
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
// 64 banks exactly once.  The XOR is its own inverse, so the copy stage uses the same expression
// to find which logical column lands in a given physical slot.
__device__ __forceinline__ int kmajor_swz(int row) { return (row >> 1) & 7; }
__device__ __forceinline__ int kmajor_off(int row, int chunk) { return row * 128 + ((chunk ^ kmajor_swz(row)) << 4); }

// XOR applied to the byte offset inside k-row `k` of an N-major LDS tile so that the k-rows one
// transposing read touches fall into different banks.
template <class C> __device__ __forceinline__ int nmajor_xor(int k) { return ((k / C::RPW) % C::NSEG) * C::SEG; }

constexpr unsigned kOutOfRange = 0x80000000u;   // buffer offset no descriptor of this library reaches

// Raw buffer descriptor (4 SGPRs): base address, stride 0, byte count for the range check, and the
// gfx9-family data-format word.  Reads outside [0, bytes) return zeros.
__device__ __forceinline__ i32x4 make_rsrc(const void* base, long long bytes) {
    const unsigned n = bytes <= 0 ? 0u : (bytes > 0x7fffffffLL ? 0x7fffffffu : (unsigned)bytes);
    const unsigned long long a = (unsigned long long)base;
    i32x4 r;
    r[0] = (int)(unsigned)a;
    r[1] = (int)((unsigned)(a >> 32) & 0xffffu);
    r[2] = (int)n;
    r[3] = 0x00020000;
    return r;
}

// 16 bytes per lane from a buffer straight into LDS at lds_base + lane*16 (lds_base wave-uniform,
// passed through M0); lanes whose offset is outside the descriptor write zeros.  Written as inline
// assembly so that the compiler does not make later LDS reads of the *other* stage wait for it; the
// copy is published by copy_barrier() instead.
__device__ __forceinline__ void load_to_lds(const i32x4& rsrc, const char* lds_base, unsigned voffset) {
    const unsigned lds_addr = (unsigned)(unsigned long long)TIR_LDS_PTR(const char, lds_base);
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "buffer_load_dwordx4 %1, %2, 0 offen lds"
        :
        : "s"(lds_addr), "v"(voffset), "s"(rsrc)
        : "memory", "m0");
}

// Workgroup barrier that also publishes this wave's global->LDS copies (counted by vmcnt) and
// retires its LDS reads of the stage that is about to be overwritten.
__device__ __forceinline__ void copy_barrier() {
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// ---------------------------------------------------------------------------------------------
// MFMA stage: fragment addresses, fragment reads, accumulate.
// ---------------------------------------------------------------------------------------------
template <class C> struct Frag {
    int a_base, b_base, sw, g, blk, s16, wn_off;
    __device__ __forceinline__ Frag(int lane, int wm, int wn) {
        const int l31 = lane & 31;
        g = lane >> 5;
        a_base = (wm * C::TM + l31) * 128;
        b_base = (wn * C::TN + l31) * 128;
        sw = kmajor_swz(l31);          // (row>>1)&7 is the same for every 32-row block of this lane
        blk = lane >> 4;
        s16 = lane & 15;
        wn_off = wn * C::TN;
    }
    __device__ __forceinline__ void read_a(const char* sa, int kk, uint4* af) const {
        const int col = ((2 * kk + g) ^ sw) << 4;
#pragma unroll
        for (int i = 0; i < C::MI; ++i) af[i] = *(const uint4*)(sa + a_base + i * 32 * 128 + col);
    }
    __device__ __forceinline__ void read_b(const char* sb, int kk, uint4* bf) const {
        if constexpr (C::BMODE == B_NMAJOR) {
#pragma unroll
            for (int j = 0; j < C::NI; ++j) {
                if constexpr (C::ES == 2) {
                    // The transposing read works on groups of 16 lanes.  Group `blk` covers columns
                    // 16*(blk&1).. of the 32-wide block and the k-group blk>>1; lane s fetches 4 values
                    // of k-row (s>>2) at columns 4*(s&3)..; afterwards lane s holds 4 consecutive k of
                    // column s.
                    const int nloc = wn_off + j * 32 + 16 * (blk & 1) + 4 * (s16 & 3);
                    i16x4 h[2];
#pragma unroll
                    for (int hh = 0; hh < 2; ++hh) {
                        const int k = kk * 16 + 8 * (blk >> 1) + 4 * hh + (s16 >> 2);
                        const char* ptr = sb + k * C::BROW + ((nloc * 2) ^ nmajor_xor<C>(k));
                        h[hh] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(TIR_LDS_PTR(i16x4, ptr));
                    }
                    const i32x2 lo = __builtin_bit_cast(i32x2, h[0]), hi = __builtin_bit_cast(i32x2, h[1]);
                    bf[j] = make_uint4((unsigned)lo[0], (unsigned)lo[1], (unsigned)hi[0], (unsigned)hi[1]);
                } else {
                    // int8: lane s fetches 8 values of k-row (s>>1) at columns 8*(s&1)..
                    const int nloc = wn_off + j * 32 + 16 * (blk & 1) + 8 * (s16 & 1);
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
            const int col = ((2 * kk + g) ^ sw) << 4;
#pragma unroll
            for (int j = 0; j < C::NI; ++j) bf[j] = *(const uint4*)(sb + b_base + j * 32 * 128 + col);
        }
    }
};

template <class C, class acc_t>
__device__ __forceinline__ void mfma_block(const uint4* af, const uint4* bf, acc_t (&acc)[C::MI][C::NI]) {
#pragma unroll
    for (int i = 0; i < C::MI; ++i)
#pragma unroll
        for (int j = 0; j < C::NI; ++j) acc[i][j] = InTraits<C::DT>::mfma(af[i], bf[j], acc[i][j]);
}

// Fused epilogue: convert and store the accumulators (C is fully overwritten).
template <class C, class acc_t>
__device__ __forceinline__ void store_tile(const Params& p, long long bz, int m0, int n0, int wm, int wn, int lane,
                                           acc_t (&acc)[C::MI][C::NI]) {
    typedef OutTraits<C::OUT> OT;
    typedef typename OT::type out_t;
    out_t* __restrict__ Cb = (out_t*)p.C + bz * p.c_bs;
    const int l31 = lane & 31, g = lane >> 5;
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

// ---------------------------------------------------------------------------------------------
// Fast kernel: vector copy modes, global -> LDS without a register hop.
// ---------------------------------------------------------------------------------------------
template <class C>
__global__ void __launch_bounds__(C::THREADS) contract_direct_kernel(const Params p) {
    typedef typename InTraits<C::DT>::acc_t acc_t;
    constexpr int ES = C::ES, VEC = C::VEC, BK = C::BK;
    static_assert(C::AMODE == A_KMAJOR || C::AMODE == A_CONV, "");
    static_assert(C::BMODE == B_KMAJOR || C::BMODE == B_NMAJOR, "");

    __shared__ __attribute__((aligned(1024))) char smem[C::LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / C::WN, wn = wave % C::WN;

    int tm, tn;
    tile_of_block(blockIdx.x, p.tiles_m, p.tiles_n, &tm, &tn);
    const int m0 = tm * C::BM, n0 = tn * C::BN;
    const long long bz = blockIdx.y;

    const char* Ab = (const char*)p.A + bz * p.a_bs * ES;
    const char* Bb = (const char*)p.B + bz * p.b_bs * ES;

    // ------------------------------------------------------------ copy stage: A
    // LDS slot q = tid + i*THREADS is row q/8, physical 16-byte column q%8 of the [BM][128 B]
    // tile; the lane fetches the logical column that the swizzle stores there.
    constexpr int A_RSTEP = C::THREADS / 8;
    const int a_r0 = tid >> 3;
    const int a_lc = (tid & 7) ^ kmajor_swz(a_r0);      // same for every i: A_RSTEP is a multiple of 16
    static_assert(A_RSTEP % 16 == 0, "");
    unsigned a_off[C::A_IT];
    int a_hw[C::A_IT];
    const char* a_base = Ab;
    long long a_bytes = 0;     // valid bytes from a_base (at k = 0)
    if constexpr (C::AMODE == A_KMAJOR) {
        // rows past M start beyond the descriptor and read as zeros
        a_base = Ab + (long long)m0 * p.a_rs * ES;
        const int rows = p.M - m0 < C::BM ? p.M - m0 : C::BM;
        a_bytes = ((long long)(rows - 1) * p.a_rs + p.K) * ES;
#pragma unroll
        for (int i = 0; i < C::A_IT; ++i)
            a_off[i] = (unsigned)(a_r0 + i * A_RSTEP) * (unsigned)(p.a_rs * ES) + a_lc * 16;
    } else {
        // ReIndex: row m of A_t is output pixel (img, op, oq) = unfuse(m); keep the element offset of
        // its top-left input pixel and that pixel's coordinates.
        a_bytes = ((long long)p.M / (p.P * p.Q)) * p.H * p.W * p.Cin * ES - bz * p.a_bs * ES;
        const int PQ = p.P * p.Q;
#pragma unroll
        for (int i = 0; i < C::A_IT; ++i) {
            const int m = m0 + a_r0 + i * A_RSTEP;
            int ih0 = -30000, iw0 = 0, img = 0;
            if (m < p.M) {
                img = m / PQ;
                const int rem = m - img * PQ;
                const int op = rem / p.Q, oq = rem - op * p.Q;
                ih0 = op * p.stride_h - p.pad_h;
                iw0 = oq * p.stride_w - p.pad_w;
            }
            a_off[i] = (((unsigned)img * (unsigned)p.H + (unsigned)ih0) * (unsigned)p.W + (unsigned)iw0) * (unsigned)p.Cin;
            a_hw[i] = (ih0 << 16) | (iw0 & 0xffff);
        }
    }

    // ------------------------------------------------------------ copy stage: B
    constexpr int B_RSTEP = (C::BMODE == B_NMAJOR) ? C::THREADS / C::B_RC : C::THREADS / 8;
    const int b_r0 = (C::BMODE == B_NMAJOR) ? tid / C::B_RC : (tid >> 3);
    const int b_pc = (C::BMODE == B_NMAJOR) ? tid % C::B_RC : (tid & 7);
    unsigned b_off[C::B_IT];
    const char* b_base = Bb;
    long long b_bytes = 0;
    long long b_slab_step = 128;    // bytes the base advances per K-slab
    if constexpr (C::BMODE == B_KMAJOR) {
        static_assert(B_RSTEP % 16 == 0, "");
        b_base = Bb + (long long)n0 * p.b_cs * ES;
        const int rows = p.N - n0 < C::BN ? p.N - n0 : C::BN;
        b_bytes = ((long long)(rows - 1) * p.b_cs + p.K) * ES;
        const int b_lc = b_pc ^ kmajor_swz(b_r0);
#pragma unroll
        for (int i = 0; i < C::B_IT; ++i)
            b_off[i] = (unsigned)(b_r0 + i * B_RSTEP) * (unsigned)(p.b_cs * ES) + b_lc * 16;
    } else {
        // k-rows of the slab; rows past K start beyond the descriptor (b_rs >= N is checked by the
        // host), columns past N are switched off per lane
        b_base = Bb + (long long)n0 * ES;
        b_bytes = ((long long)(p.K - 1) * p.b_rs + (p.N - n0)) * ES;
        b_slab_step = (long long)BK * p.b_rs * ES;
#pragma unroll
        for (int i = 0; i < C::B_IT; ++i) {
            const int k = b_r0 + i * B_RSTEP;
            const int lb = (b_pc * 16) ^ nmajor_xor<C>(k);      // logical byte inside the k-row
            b_off[i] = (n0 + lb / ES < p.N) ? (unsigned)k * (unsigned)(p.b_rs * ES) + lb : kOutOfRange;
        }
    }

    auto issue = [&](int slab, int buf) {
        char* sa = smem + buf * C::STAGE_BYTES + wave * 1024;
        char* sb = sa + C::A_BYTES;
        const int k0 = slab * BK;
        if constexpr (C::AMODE == A_KMAJOR) {
            const i32x4 ra = make_rsrc(a_base + (long long)k0 * ES, a_bytes - (long long)k0 * ES);
            const bool kv = k0 + a_lc * VEC < p.K;      // K tail: the padding between rows is not zero
#pragma unroll
            for (int i = 0; i < C::A_IT; ++i) load_to_lds(ra, sa + i * C::THREADS * 16, kv ? a_off[i] : kOutOfRange);
        } else {
            // fuse(rh, rw, rc) -> (rh, rw, rc); a 16-byte vector never straddles a tap (Cg % VEC == 0)
            const i32x4 ra = make_rsrc(Ab, a_bytes);
            const int kb = k0 + a_lc * VEC;
            const int tap = kb / p.Cg;
            const int cc = kb - tap * p.Cg;
            const int fr = tap / p.S, fs = tap - fr * p.S;
            const int dh = fr * p.dil_h, dw = fs * p.dil_w;
            const unsigned delta = (unsigned)((dh * p.W + dw) * p.Cin + cc);
            const bool kv = kb < p.K;
#pragma unroll
            for (int i = 0; i < C::A_IT; ++i) {
                const int ih = (a_hw[i] >> 16) + dh;
                const int iw = (int)(short)(a_hw[i] & 0xffff) + dw;
                const bool ok = kv && (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
                load_to_lds(ra, sa + i * C::THREADS * 16, ok ? (a_off[i] + delta) * ES : kOutOfRange);
            }
        }
        if constexpr (C::BMODE == B_KMAJOR) {
            const i32x4 rb = make_rsrc(b_base + (long long)k0 * ES, b_bytes - (long long)k0 * ES);
            const int b_lc = b_pc ^ kmajor_swz(b_r0);
            const bool kv = k0 + b_lc * VEC < p.K;
#pragma unroll
            for (int i = 0; i < C::B_IT; ++i) load_to_lds(rb, sb + i * C::THREADS * 16, kv ? b_off[i] : kOutOfRange);
        } else {
            const i32x4 rb = make_rsrc(b_base + slab * b_slab_step, b_bytes - slab * b_slab_step);
#pragma unroll
            for (int i = 0; i < C::B_IT; ++i) load_to_lds(rb, sb + i * C::THREADS * 16, b_off[i]);
        }
    };

    // ------------------------------------------------------------ MFMA stage
    const Frag<C> frag(lane, wm, wn);
    acc_t acc[C::MI][C::NI];
#pragma unroll
    for (int i = 0; i < C::MI; ++i)
#pragma unroll
        for (int j = 0; j < C::NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;   // reduction init

    const int nslab = (p.K + BK - 1) / BK;
    if (nslab > 0) {
        uint4 af[2][C::MI], bf[2][C::NI];
        issue(0, 0);
        copy_barrier();
        frag.read_a(smem, 0, af[0]);
        frag.read_b(smem + C::A_BYTES, 0, bf[0]);
        for (int s = 0; s < nslab; ++s) {
            const int cur = s & 1;
            const char* sa = smem + cur * C::STAGE_BYTES;
            const char* sb = sa + C::A_BYTES;
            // the other stage was last read before the barrier that ended the previous iteration;
            // past the last slab the descriptors are empty and the copy writes zeros nobody reads
            issue(s + 1, cur ^ 1);
            // Fragments of k-step kk+1 are requested before the MFMAs of k-step kk are issued, so the
            // LDS latency hides behind the matrix pipe; the scheduling fences keep that order.
            TIR_FENCE();
            frag.read_a(sa, 1, af[1]);
            frag.read_b(sb, 1, bf[1]);
            TIR_FENCE();
            mfma_block<C>(af[0], bf[0], acc);
            TIR_FENCE();
            frag.read_a(sa, 2, af[0]);
            frag.read_b(sb, 2, bf[0]);
            TIR_FENCE();
            mfma_block<C>(af[1], bf[1], acc);
            TIR_FENCE();
            frag.read_a(sa, 3, af[1]);
            frag.read_b(sb, 3, bf[1]);
            TIR_FENCE();
            mfma_block<C>(af[0], bf[0], acc);
            TIR_FENCE();
            // slab s+1 has landed and every wave is done reading slab s
            copy_barrier();
            const char* na = smem + (cur ^ 1) * C::STAGE_BYTES;
            frag.read_a(na, 0, af[0]);
            frag.read_b(na + C::A_BYTES, 0, bf[0]);
            TIR_FENCE();
            mfma_block<C>(af[1], bf[1], acc);
            TIR_FENCE();
        }
    }

    store_tile<C>(p, bz, m0, n0, wm, wn, lane, acc);
}

// ---------------------------------------------------------------------------------------------
// General kernel: any strides / any channel count, element-wise loads staged through registers.
// Same LDS layout (both operands K-major) and the same MFMA stage as the fast kernel.
// ---------------------------------------------------------------------------------------------
template <class C>
__global__ void __launch_bounds__(C::THREADS) contract_staged_kernel(const Params p) {
    typedef typename InTraits<C::DT>::acc_t acc_t;
    constexpr int ES = C::ES, VEC = C::VEC, BK = C::BK;
    static_assert(C::AMODE == A_GENERIC || C::AMODE == A_CONV_GENERIC, "");
    static_assert(C::BMODE == B_GENERIC, "");
    typedef typename std::conditional<ES == 2, unsigned short, unsigned char>::type elem_t;

    __shared__ __attribute__((aligned(16))) char smem[C::LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / C::WN, wn = wave % C::WN;

    int tm, tn;
    tile_of_block(blockIdx.x, p.tiles_m, p.tiles_n, &tm, &tn);
    const int m0 = tm * C::BM, n0 = tn * C::BN;
    const long long bz = blockIdx.y;

    const elem_t* A = (const elem_t*)p.A + bz * p.a_bs;
    const elem_t* B = (const elem_t*)p.B + bz * p.b_bs;

    const int c8 = tid & 7;
    const int r0 = tid >> 3;
    constexpr int RSTEP = C::THREADS / 8;
    unsigned a_off[C::A_IT];
    int a_hw[C::A_IT];
    if constexpr (C::AMODE == A_CONV_GENERIC) {
        const int PQ = p.P * p.Q;
#pragma unroll
        for (int i = 0; i < C::A_IT; ++i) {
            const int m = m0 + r0 + i * RSTEP;
            int ih0 = -30000, iw0 = 0, img = 0;
            if (m < p.M) {
                img = m / PQ;
                const int rem = m - img * PQ;
                const int op = rem / p.Q, oq = rem - op * p.Q;
                ih0 = op * p.stride_h - p.pad_h;
                iw0 = oq * p.stride_w - p.pad_w;
            }
            a_off[i] = (((unsigned)img * (unsigned)p.H + (unsigned)ih0) * (unsigned)p.W + (unsigned)iw0) * (unsigned)p.Cin;
            a_hw[i] = (ih0 << 16) | (iw0 & 0xffff);
        }
    }

    uint4 ra[C::A_IT], rb[C::B_IT];

    auto load_ab = [&](int slab) {
        const int k0 = slab * BK;
#pragma unroll
        for (int i = 0; i < C::A_IT; ++i) {
            alignas(16) elem_t v[VEC];
            if constexpr (C::AMODE == A_GENERIC) {
                const long long m = m0 + r0 + i * RSTEP;
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const long long k = k0 + c8 * VEC + e;
                    v[e] = (m < p.M && k < p.K) ? A[m * p.a_rs + k * p.a_cs] : (elem_t)0;
                }
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const int kb = k0 + c8 * VEC + e;
                    const int tap = kb / p.Cg;
                    const int cc = kb - tap * p.Cg;
                    const int fr = tap / p.S, fs = tap - fr * p.S;
                    const int dh = fr * p.dil_h, dw = fs * p.dil_w;
                    const int ih = (a_hw[i] >> 16) + dh;
                    const int iw = (int)(short)(a_hw[i] & 0xffff) + dw;
                    const bool ok = kb < p.K && (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
                    v[e] = ok ? A[(long long)(int)(a_off[i] + (unsigned)((dh * p.W + dw) * p.Cin + cc))] : (elem_t)0;
                }
            }
            ra[i] = *(const uint4*)v;
        }
#pragma unroll
        for (int i = 0; i < C::B_IT; ++i) {
            alignas(16) elem_t v[VEC];
            const long long n = n0 + r0 + i * RSTEP;
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const long long k = k0 + c8 * VEC + e;
                v[e] = (n < p.N && k < p.K) ? B[k * p.b_rs + n * p.b_cs] : (elem_t)0;
            }
            rb[i] = *(const uint4*)v;
        }
    };
    auto store_ab = [&](int buf) {
        char* sa = smem + buf * C::STAGE_BYTES;
        char* sb = sa + C::A_BYTES;
#pragma unroll
        for (int i = 0; i < C::A_IT; ++i) *(uint4*)(sa + kmajor_off(r0 + i * RSTEP, c8)) = ra[i];
#pragma unroll
        for (int i = 0; i < C::B_IT; ++i) *(uint4*)(sb + kmajor_off(r0 + i * RSTEP, c8)) = rb[i];
    };

    const Frag<C> frag(lane, wm, wn);
    acc_t acc[C::MI][C::NI];
#pragma unroll
    for (int i = 0; i < C::MI; ++i)
#pragma unroll
        for (int j = 0; j < C::NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;   // reduction init

    const int nslab = (p.K + BK - 1) / BK;
    if (nslab > 0) {
        load_ab(0);
        store_ab(0);
        __syncthreads();
        for (int s = 0; s < nslab; ++s) {
            const int cur = s & 1;
            const bool more = s + 1 < nslab;
            if (more) load_ab(s + 1);
            const char* sa = smem + cur * C::STAGE_BYTES;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                uint4 af[C::MI], bf[C::NI];
                frag.read_a(sa, kk, af);
                frag.read_b(sa + C::A_BYTES, kk, bf);
                mfma_block<C>(af, bf, acc);
            }
            if (more) store_ab(cur ^ 1);
            __syncthreads();
        }
    }

    store_tile<C>(p, bz, m0, n0, wm, wn, lane, acc);
}

}  // namespace tir
