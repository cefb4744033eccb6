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
// One LDS stage holds ROWB = 64, 128 or 256 bytes of k per row (e.g. 32, 64 or 128 fp16 values) = 2, 4 or 8
// MFMA k-steps; the stages form a ring that the copy stage fills NSTAGE-1 stages ahead of the MFMAs.
#pragma once
#include <hip/hip_runtime.h>
#include <type_traits>
#include "tir_params.h"

// Cache policy bits of the epilogue's buffer stores (0 = default write-back through L2): write-through at system
// scope, which spreads the write-back over the epilogue instead of leaving it to the end of the kernel ...
#ifndef TIR_STORE_AUX
#define TIR_STORE_AUX 17
#endif
// ... and, for outputs that nothing reads soon (Params::store_nt, the caller's choice), non-temporal as well: the lines
// are not kept in L2.  Measured on the 56x56x64 convolution: 7.4 instead of 9.0 us per launch when inputs come from
// HBM and the output is not read again, but 8.1 instead of 7.5 us per launch in a chain of convolutions that each
// read what the previous one wrote.
#define TIR_STORE_AUX_STREAM (TIR_STORE_AUX | 2)

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
        return __builtin_bit_cast(unsigned short, (__bf16)v);      // gfx950 converts in hardware (v_cvt_pk_bf16_f32: nearest even, quiet NaN)
    }
};

template <> struct OutTraits<DT_I8> {
    typedef signed char type;       // requantised int8 codes; produced by finish_value(), which needs the scale
};

// The fused consumer behind the tensorized block: bias add, ReLU, conversion to the output type.
// For int8 output the int32 sum is scaled in binary32 and rounded to the nearest code, ties to even
// (v_rndne_f32), then saturated.
template <class E> __device__ __forceinline__ E consumer(E acc, E bias, int relu) {
    // ReLU as a clamp from below at a uniform floor (0, or the lowest value = no clamp): add, compare, select per value,
    // with nothing uniform left inside the per-value code.  A NaN fails the comparison and stays a NaN.
    const E floor = relu ? (E)0 : (std::is_same<E, float>::value ? (E)(-__builtin_inff()) : (E)(-2147483647 - 1));
    const E t = acc + bias;
    return t < floor ? floor : t;
}
template <int OUT, class E> __device__ __forceinline__ typename OutTraits<OUT>::type finish_value(E t, float scale) {
    if constexpr (OUT == DT_I8) {
        float f = (float)t * scale;
        f = __builtin_rintf(f);
        f = __builtin_amdgcn_fmed3f(f, -128.0f, 127.0f);       // saturate: the median of the value and the two limits, one instruction
        return (signed char)(int)f;
    } else {
        return OutTraits<OUT>::cvt(t);
    }
}
// One output value through the buffer descriptor rc (1, 2 or 4 bytes).
template <int AUX = TIR_STORE_AUX, class T> __device__ __forceinline__ void store_value(T v, __amdgpu_buffer_rsrc_t rc, int voff, int soff) {
    if constexpr (sizeof(T) == 4) __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), rc, voff, soff, AUX);
    else if constexpr (sizeof(T) == 2) __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(unsigned short, v), rc, voff, soff, AUX);
    else __builtin_amdgcn_raw_buffer_store_b8(__builtin_bit_cast(unsigned char, v), rc, voff, soff, AUX);
}

// Convert and store the 16 accumulator registers of one 32x32 block (register r is row
// 8*(r/4) + r%4 of the lane's row group).  The plain operator sends its accumulators to the store
// unit with at most a type conversion; the consumer's extra instructions only run when one is fused
// (`fused` is uniform).
template <int OUT, int AUX, class ACC, class E>
__device__ __forceinline__ void store_block_as(const ACC& a, bool fused, E bias, int relu, float scale,
                                               __amdgpu_buffer_rsrc_t rc, int voff, int row_bytes) {
    if (fused) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
            store_value<AUX>(finish_value<OUT>(consumer((E)a[r], bias, relu), scale), rc, voff, (8 * (r >> 2) + (r & 3)) * row_bytes);
    } else {
#pragma unroll
        for (int r = 0; r < 16; ++r)
            store_value<AUX>(finish_value<OUT>((E)a[r], scale), rc, voff, (8 * (r >> 2) + (r & 3)) * row_bytes);
    }
}
// ... with the cache policy the launch asks for (`stream` is uniform).
template <int OUT, class ACC, class E>
__device__ __forceinline__ void store_block(const ACC& a, bool fused, E bias, int relu, float scale,
                                            __amdgpu_buffer_rsrc_t rc, int voff, int row_bytes, bool stream) {
    if (stream) store_block_as<OUT, TIR_STORE_AUX_STREAM>(a, fused, bias, relu, scale, rc, voff, row_bytes);
    else store_block_as<OUT, TIR_STORE_AUX>(a, fused, bias, relu, scale, rc, voff, row_bytes);
}

// K-major LDS tile: [rows][ROWB bytes], 16-byte columns XOR-swizzled by the row so that the 16
// rows one ds_read_b128 phase touches at a fixed logical column fall on all 64 banks exactly once
// (ROWB 256: column ^ (row mod 16); ROWB 128: column ^ (row/2 mod 8); ROWB 64: column ^ (row/4 mod 4)).  The XOR is its own inverse,
// so the copy stage uses the same expression to find which logical column a physical slot holds.
template <int ROWB> __device__ __forceinline__ int kmajor_swz(int row) {
    return ROWB == 256 ? (row & 15) : ROWB == 128 ? ((row >> 1) & 7) : ((row >> 2) & 3);
}
template <int ROWB> __device__ __forceinline__ int kmajor_off(int row, int chunk) {
    return row * ROWB + ((chunk ^ kmajor_swz<ROWB>(row)) << 4);
}

// XOR applied to the byte offset inside k-row `k` of an N-major LDS tile so that the k-rows one
// transposing read touches fall into different banks.
template <class C> __device__ __forceinline__ int nmajor_xor(int k) { return ((k / C::RPW) % C::NSEG) * C::SEG; }


constexpr unsigned kOutOfRange = 0x80000000u;   // buffer offset no descriptor of this library reaches

// Raw buffer descriptor (4 SGPRs): base address, stride 0, byte count for the range check, and the
// gfx9-family data-format word.  Reads outside [0, bytes) return zeros.
__device__ __forceinline__ i32x4 make_rsrc(const void* base, long long bytes) {
    const unsigned n = bytes <= 0 ? 0u : (bytes > 0x7fffffffLL ? 0x7fffffffu : (unsigned)bytes);
    const unsigned long long a = (unsigned long long)base;
    // the descriptor must sit in scalar registers: readfirstlane is free for values the compiler already
    // knows to be uniform and forces the others
    i32x4 r;
    r[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)a);
    r[1] = __builtin_amdgcn_readfirstlane((int)((unsigned)(a >> 32) & 0xffffu));
    r[2] = __builtin_amdgcn_readfirstlane((int)n);
    r[3] = 0x00020000;
    return r;
}

// The same for a byte count the host has already bounded by 2^31 - 1 (every K-major and convolution operand):
// the 64-bit clamp above compiles to vector compares of uniform values whose results travel back to the scalar
// unit, twice per descriptor and stage.
__device__ __forceinline__ i32x4 make_rsrc32(const void* base, unsigned bytes) {
    const unsigned long long a = (unsigned long long)base;
    i32x4 r;
    r[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)a);
    r[1] = __builtin_amdgcn_readfirstlane((int)((unsigned)(a >> 32) & 0xffffu));
    r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
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
// ... with the non-temporal hint, for operand bytes that (almost) no other workgroup of the launch reads again: they then do
// not push the lines the workgroups share out of the caches.  Measured with the operands coming from memory: the headline
// convolution's input 8.6 -> 8.2 us, the fused attention's Q, K, V 7.05 -> 6.63, no change with warm caches.  On operands
// that many workgroups re-read (a filter, the panels of a GEMM) it costs as much and more, and on the operands of batched
// matmuls with one tile per batch entry it trades 10 % from memory against 8 % from the caches: those keep the plain copy.
__device__ __forceinline__ void load_to_lds_nt(const i32x4& rsrc, const char* lds_base, unsigned voffset) {
    const unsigned lds_addr = (unsigned)(unsigned long long)TIR_LDS_PTR(const char, lds_base);
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "buffer_load_dwordx4 %1, %2, 0 offen nt lds"
        :
        : "s"(lds_addr), "v"(voffset), "s"(rsrc)
        : "memory", "m0");
}

// Kernel arguments are fetched lazily, a few at a time, each fetch an exposed scalar-memory latency
// of several hundred cycles.  Naming the fields a kernel needs before its first copy in one asm
// statement makes the compiler fetch them in one batch at the very start.
__device__ __forceinline__ void prefetch_args(const Params& p, bool conv) {
    asm volatile("" ::"s"(p.A), "s"(p.B), "s"(p.C), "s"(p.M), "s"(p.N), "s"(p.K), "s"(p.tiles_m), "s"(p.tiles_n),
                 "s"(p.c_fast), "s"(p.ksplit), "s"(p.div_gw_magic), "s"(p.div_gw_shift));
    asm volatile("" ::"s"(p.a_bs), "s"(p.b_bs), "s"(p.c_bs), "s"(p.a_rs), "s"(p.b_rs), "s"(p.b_cs), "s"(p.c_rs), "s"(p.c_cs), "s"(p.bias_bs),
                 "s"(p.bias), "s"(p.relu), "s"(p.scale), "s"(p.ws), "s"(p.batch_imgs), "s"(p.store_nt));
    if (conv) {
        asm volatile("" ::"s"(p.H), "s"(p.W), "s"(p.Cin), "s"(p.Cg), "s"(p.P), "s"(p.Q), "s"(p.S), "s"(p.stride_h), "s"(p.stride_w), "s"(p.pad_h),
                     "s"(p.pad_w), "s"(p.dil_h), "s"(p.dil_w));
        asm volatile("" ::"s"(p.div_pq_magic), "s"(p.div_q_magic), "s"(p.div_pq_shift), "s"(p.div_q_shift), "s"(p.div_cg_magic), "s"(p.div_s_magic),
                     "s"(p.div_cg_shift), "s"(p.div_s_shift), "s"(p.phases_h));
    }
}

// Workgroup barrier that also publishes this wave's global->LDS copies (counted by vmcnt; all but
// the newest PENDING must have landed) and retires its LDS reads of the slot that is refilled next.
template <int PENDING> __device__ __forceinline__ void copy_barrier() {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(PENDING) : "memory");
}

// s_waitcnt takes an immediate; this waits until at most n (wave-uniform, capped at 63) vector-memory
// operations of the wave are outstanding.
__device__ __forceinline__ void wait_vmcnt_upto(int n) {
#define TIR_W(k) case k: asm volatile("s_waitcnt vmcnt(" #k ")" ::: "memory"); break;
#define TIR_W4(k) TIR_W(k) TIR_W(k + 1) TIR_W(k + 2) TIR_W(k + 3)
#define TIR_W16(k) TIR_W4(k) TIR_W4(k + 4) TIR_W4(k + 8) TIR_W4(k + 12)
    switch (n < 0 ? 0 : (n > 63 ? 63 : n)) {
        TIR_W16(0) TIR_W16(16) TIR_W16(32) TIR_W16(48)
        default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
    }
#undef TIR_W16
#undef TIR_W4
#undef TIR_W
}

// ---------------------------------------------------------------------------------------------
// MFMA stage: fragment addresses, fragment reads, accumulate.
// ---------------------------------------------------------------------------------------------
template <class C> struct Frag {
    int a_base, b_base, sw, g, blk, s16, wn_off;
    __device__ __forceinline__ Frag(int lane, int wm, int wn) {
        const int l31 = lane & 31;
        g = lane >> 5;
        a_base = (wm * C::TM + l31) * C::ROWB;
        b_base = (wn * C::TN + l31) * C::ROWB;
        sw = kmajor_swz<C::ROWB>(l31);   // the swizzle repeats every 16 rows: same for every 32-row block
        blk = lane >> 4;
        s16 = lane & 15;
        wn_off = wn * C::TN;
    }
    __device__ __forceinline__ uint4 read_a1(const char* sa, int kk, int i) const {
        const int col = ((2 * kk + g) ^ sw) << 4;
        return *(const uint4*)(sa + a_base + i * 32 * C::ROWB + col);
    }
    __device__ __forceinline__ void read_a(const char* sa, int kk, uint4* af) const {
#pragma unroll
        for (int i = 0; i < C::MI; ++i) af[i] = read_a1(sa, kk, i);
    }
    __device__ __forceinline__ void read_b(const char* sb, int kk, uint4* bf) const {
#pragma unroll
        for (int j = 0; j < C::NI; ++j) bf[j] = read_b1(sb, kk, j);
    }
    __device__ __forceinline__ uint4 read_b1(const char* sb, int kk, int j) const {
        uint4 out;
        if constexpr (C::BMODE == B_NMAJOR) {
            {
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
                    out = make_uint4((unsigned)lo[0], (unsigned)lo[1], (unsigned)hi[0], (unsigned)hi[1]);
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
                    out = make_uint4((unsigned)h[0][0], (unsigned)h[0][1], (unsigned)h[1][0], (unsigned)h[1][1]);
                }
            }
        } else {
            const int col = ((2 * kk + g) ^ sw) << 4;
            out = *(const uint4*)(sb + b_base + j * 32 * C::ROWB + col);
        }
        return out;
    }
};

template <class C, class acc_t>
__device__ __forceinline__ void mfma_block(const uint4* af, const uint4* bf, acc_t (&acc)[C::MI][C::NI]) {
#pragma unroll
    for (int i = 0; i < C::MI; ++i)
#pragma unroll
        for (int j = 0; j < C::NI; ++j) acc[i][j] = InTraits<C::DT>::mfma(af[i], bf[j], acc[i][j]);
}

// The lane's bias values (one per 32-column block of its wave tile), requested at kernel start: the
// vector usually misses every cache, and a load in the epilogue would expose that whole latency.
template <class C, class E>
__device__ __forceinline__ void load_bias(const Params& p, long long bz, int n0, int wn, int lane, E (&bias_r)[C::NI]) {
    // through a buffer descriptor that covers the tile's valid columns, or nothing at all without a
    // bias: lanes outside it read 0 and no branch is needed
    const int cols = p.N - n0 < C::BN ? p.N - n0 : C::BN;
    const E* base = (const E*)p.bias + bz * p.bias_bs + n0;
    const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, p.bias ? cols * 4 : 0, 0x00020000);
#pragma unroll
    for (int j = 0; j < C::NI; ++j) {
        const int col = wn * C::TN + j * 32 + (lane & 31);
        bias_r[j] = __builtin_bit_cast(E, __builtin_amdgcn_raw_buffer_load_b32(rb, col * 4, 0, 0));
    }
}

// Fused epilogue: convert and store the accumulators (C is fully overwritten).
// With a unit column stride the stores go through a buffer descriptor that covers exactly the valid
// part of this workgroup's tile: rows past M fall outside it and are dropped by the hardware, columns
// past N are switched off per lane, and the row offset is a scalar, so a store costs no vector ALU
// work.  Other C strides take the element-wise path.
template <class C, class acc_t>
__device__ __forceinline__ void store_tile(const Params& p, long long bz, int m0, int n0, int wm, int wn, int lane,
                                           acc_t (&acc)[C::MI][C::NI],
                                           const typename std::conditional<std::is_same<acc_t, f32x16>::value, float, int>::type (&bias_r)[C::NI]) {
    typedef OutTraits<C::OUT> OT;
    typedef typename OT::type out_t;
    typedef typename std::conditional<std::is_same<acc_t, f32x16>::value, float, int>::type acc_e;
    constexpr int OS = (int)sizeof(out_t);
    out_t* __restrict__ Cb = (out_t*)p.C + bz * p.c_bs;
    const int l31 = lane & 31, g = lane >> 5;
    const int cols = p.N - n0 < C::BN ? p.N - n0 : C::BN;
    const bool fused = p.bias != nullptr || p.relu != 0;      // uniform; int8 output alone only changes finish_value
    // Loads and stores retire through one counter, in order: the wait for the bias values (requested
    // at kernel start) must sit before the first store, or it would wait for stores as well.
#pragma unroll
    for (int j = 0; j < C::NI; ++j) asm volatile("" ::"v"(bias_r[j]));
    if (p.c_fast) {
        const int rows = p.M - m0 < C::BM ? p.M - m0 : C::BM;
        const long long bytes = ((long long)(rows - 1) * p.c_rs + cols) * OS;
        const __amdgpu_buffer_rsrc_t rc = __builtin_amdgcn_make_buffer_rsrc(
            (void*)(Cb + (long long)m0 * p.c_rs + n0), 0, (int)(bytes > 0x7fffffffLL ? 0x7fffffffLL : bytes), 0x00020000);
        const int row_bytes = (int)p.c_rs * OS;
#pragma unroll
        for (int i = 0; i < C::MI; ++i) {
#pragma unroll
            for (int j = 0; j < C::NI; ++j) {
                const int col = wn * C::TN + j * 32 + l31;
                const int row0 = wm * C::TM + i * 32 + 4 * g;
                const unsigned voff = col < cols ? (unsigned)(row0 * row_bytes + col * OS) : kOutOfRange;
                store_block<C::OUT>(acc[i][j], fused, bias_r[j], p.relu, p.scale, rc, (int)voff, row_bytes, p.store_nt != 0);
            }
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < C::MI; ++i) {
#pragma unroll
        for (int j = 0; j < C::NI; ++j) {
            const int col = n0 + wn * C::TN + j * 32 + l31;
            const acc_e b = bias_r[j];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm * C::TM + i * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                if (row < p.M && col < p.N)
                    Cb[(long long)row * p.c_rs + (long long)col * p.c_cs] = finish_value<C::OUT>(consumer(acc[i][j][r], b, p.relu), p.scale);
            }
        }
    }
}

// Epilogue of one output phase of a transposed convolution: row m of the tile is pixel (img, op, oq) of the
// phase's grid, i.e. pixel (op*phases_h + ph, oq*phases_w + pw) of the output image.  Rows are decoded with
// the host's division constants; rows past M and pixels past the output's edge (extents not divisible by the
// phase count) are switched off.
template <class C, class acc_t>
__device__ __forceinline__ void store_tile_phase(const Params& p, long long bz, int m0, int n0, int wm, int wn, int lane,
                                                 acc_t (&acc)[C::MI][C::NI],
                                                 const typename std::conditional<std::is_same<acc_t, f32x16>::value, float, int>::type (&bias_r)[C::NI],
                                                 int ph, int pw) {
    typedef typename OutTraits<C::OUT>::type out_t;
    constexpr int OS = (int)sizeof(out_t);
    const int l31 = lane & 31, g = lane >> 5;
    const int cols = p.N - n0 < C::BN ? p.N - n0 : C::BN;
    const int PQ = p.P * p.Q;
    const long long total = (long long)p.batch_imgs * p.P_full * p.Q_full * p.c_rs * OS;      // bytes of the whole output
    const __amdgpu_buffer_rsrc_t rc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)((out_t*)p.C + bz * p.c_bs + n0), 0, (int)(total - (bz * p.c_bs + n0) * OS), 0x00020000);
#pragma unroll
    for (int j = 0; j < C::NI; ++j) asm volatile("" ::"v"(bias_r[j]));
    unsigned col_off[C::NI];        // the lane's column inside the descriptor, or out of range
#pragma unroll
    for (int j = 0; j < C::NI; ++j) {
        const int col = wn * C::TN + j * 32 + l31;
        col_off[j] = col < cols ? (unsigned)(col * OS) : kOutOfRange;
    }
    // FUSED: a consumer is fused (else the accumulators go out with a conversion at most); STREAM: non-temporal stores.
    auto emit = [&](auto fused_flag, auto stream_flag) __attribute__((always_inline)) {
        constexpr bool FUSED = decltype(fused_flag)::value;
        constexpr int AUX = decltype(stream_flag)::value ? TIR_STORE_AUX_STREAM : TIR_STORE_AUX;
#pragma unroll
        for (int i = 0; i < C::MI; ++i) {
            // The 32 rows of block i are decoded once, row l31 by lane l31 (both half-waves alike); accumulator register r
            // holds row 8*(r/4) + r%4 (+ 4 in the upper half-wave), whose offset comes over from the lane that decoded it.
            // Decoding per register instead cost 16 divisions per lane and block: 4 us of this epilogue were address arithmetic.
            const unsigned m = (unsigned)(m0 + wm * C::TM + i * 32 + l31);
            const unsigned img = fastdiv(m, p.div_pq_magic, p.div_pq_shift);
            const unsigned rem = m - img * (unsigned)PQ;
            const unsigned op = fastdiv(rem, p.div_q_magic, p.div_q_shift);
            const unsigned oq = rem - op * (unsigned)p.Q;
            const int oh = (int)op * p.phases_h + ph, ow = (int)oq * p.phases_w + pw;
            const bool row_ok = (int)m < p.M && oh < p.P_full && ow < p.Q_full;
            // (< 2^31: the host bounds the output's bytes; an invalid row stays out of range whatever column is added)
            const unsigned pixv = row_ok ? ((img * (unsigned)p.P_full + (unsigned)oh) * (unsigned)p.Q_full + (unsigned)ow) * (unsigned)(p.c_rs * OS) : kOutOfRange;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = 8 * (r >> 2) + (r & 3);
                const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)pixv, row), hi = (unsigned)__builtin_amdgcn_readlane((int)pixv, row + 4);
                const unsigned pix = g ? hi : lo;
#pragma unroll
                for (int j = 0; j < C::NI; ++j) {
                    const unsigned voff = col_off[j] != kOutOfRange ? pix + col_off[j] : kOutOfRange;
                    const auto t = FUSED ? consumer(acc[i][j][r], bias_r[j], p.relu) : acc[i][j][r];
                    store_value<AUX>(finish_value<C::OUT>(t, p.scale), rc, (int)voff, 0);
                }
            }
        }
    };
    const bool fused = p.bias != nullptr || p.relu != 0;      // uniform, like the cache policy
    if (fused) {
        if (p.store_nt) emit(std::true_type(), std::true_type());
        else emit(std::true_type(), std::false_type());
    } else {
        if (p.store_nt) emit(std::false_type(), std::true_type());
        else emit(std::false_type(), std::false_type());
    }
}

// ---------------------------------------------------------------------------------------------
// Fast kernel: vector copy modes, global -> LDS without a register hop, NSTAGE-deep copy ring.
//
// Stage h of the reduction lives in ring slot h % NSTAGE.  Iteration h of the main loop
//   (1) multiplies k-steps 0 .. KSTEPS-LA-1 of stage h while it requests the fragments LA k-steps ahead
//       from LDS and issues the global->LDS copy of stage h+NSTAGE-1 (its slot held stage
//       h-1, which every wave finished reading before the previous barrier);
//   (2) waits until this wave's copy of stage h+1 has landed and joins the workgroup barrier;
//   (3) multiplies the last LA k-steps of stage h while requesting the first fragments of stage h+1.
// The last NSTAGE-1 iterations have no stage left to copy and skip that part of (1).
// A wave issues one instruction per ~4 cycles whatever its kind, and at one or two waves per SIMD all of
// them are exposed: slots and stages advance by counters (no h % NSTAGE), divisions by launch constants
// are multiply-and-shift, and nothing is recomputed per stage that a counter can carry.
// With one wave per SIMD nothing else hides latency, so MFMAs and side work (LDS reads, copy
// issue) are interleaved one by one in program order and scheduling fences keep that order.
// ---------------------------------------------------------------------------------------------
template <class C>
__global__ void __launch_bounds__(C::THREADS) contract_direct_kernel(const Params p) {
    typedef typename InTraits<C::DT>::acc_t acc_t;
    constexpr int ES = C::ES, VEC = C::VEC, BK = C::BK, ROWB = C::ROWB, NSTAGE = C::NSTAGE, KSTEPS = C::KSTEPS;
    constexpr int L = C::A_IT + C::B_IT;      // copy instructions per wave and stage
    static_assert(C::AMODE == A_KMAJOR || C::AMODE == A_CONV || C::AMODE == A_CONVX, "");
    static_assert(C::BMODE == B_KMAJOR || C::BMODE == B_NMAJOR, "");
    static_assert((NSTAGE - 2) * L <= 63, "vmcnt range");

    __shared__ __attribute__((aligned(1024))) char smem[C::LDS_BYTES];
    prefetch_args(p, C::AMODE != A_KMAJOR);

    // reduction group kgrp owns the stages s with s % KW == kgrp; inside the group, thread tid of SUB.
    // With copy waves (CW > 0) the waves past the multiplying ones only copy: thread tid of CT, wave `wave` of CW.
    constexpr bool SPEC = C::CW > 0;
    const int lane = threadIdx.x & 63;
    const int wave_wg = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool copier = SPEC && wave_wg >= C::WM * C::WN;        // wave-uniform
    const int kgrp = C::KW == 1 ? 0 : wave_wg / (C::WM * C::WN);
    const int wave = wave_wg - (copier ? C::WM * C::WN : kgrp * (C::WM * C::WN));
    const int tid = (int)threadIdx.x - (copier ? C::SUB : kgrp * C::SUB);
    const int wm = wave / C::WN, wn = wave % C::WN;
    char* const ring = smem + kgrp * C::RING_BYTES;

    int tm, tn;
    tile_of_block(blockIdx.x, p.tiles_m, p.tiles_n, p.div_gw_magic, p.div_gw_shift, &tm, &tn);
    const int m0 = tm * C::BM, n0 = tn * C::BN;
    long long bz = blockIdx.y;

    // Transposed convolution by output phase: this grid.y entry is (phase, group).  The phase's pixels are a
    // stride-1 convolution with every phases-th filter tap, taken backwards (cursor tap (fr, fs) is filter tap
    // (f_r0 - phases_h*fr, f_s0 - phases_w*fs)); tap count, padding and with them K differ per phase.
    int cS = p.S, cK = p.K, cpad_h = p.pad_h, cpad_w = p.pad_w;
    int f_r0 = 0, f_s0 = 0, ph = 0, pw = 0;
    bool phased = false;
    if constexpr (C::AMODE == A_CONV) {
        phased = p.phases_h != 0;
        if (phased) {
            auto div_h = [&](int v) { return (int)fastdiv((unsigned)v, p.div_phh_magic, p.div_phh_shift); };    // v >= 0
            auto div_w = [&](int v) { return (int)fastdiv((unsigned)v, p.div_phw_magic, p.div_phw_shift); };
            const int phase = (int)fastdiv((unsigned)bz, p.div_grp_magic, p.div_grp_shift);
            bz -= (long long)phase * p.conv_groups;
            ph = div_w(phase);
            pw = phase - ph * p.phases_w;
            const int qh = div_h(ph + p.t_pad_h), qw = div_w(pw + p.t_pad_w);
            const int r0 = ph + p.t_pad_h - qh * p.phases_h, s0 = pw + p.t_pad_w - qw * p.phases_w;
            const int cR = p.R > r0 ? div_h(p.R - r0 + p.phases_h - 1) : 0;
            cS = p.S > s0 ? div_w(p.S - s0 + p.phases_w - 1) : 0;
            cpad_h = (cR - 1) - qh;       // (ph + t_pad_h - r0) / phases_h
            cpad_w = (cS - 1) - qw;
            f_r0 = r0 + p.phases_h * (cR - 1);
            f_s0 = s0 + p.phases_w * (cS - 1);
            cK = cR * cS * p.Cg;                          // 0 for a phase no tap reaches: its pixels get the empty sum
        }
    }

    const char* Ab = (const char*)p.A + bz * p.a_bs * ES;
    const char* Bb = (const char*)p.B + bz * p.b_bs * ES;
    const int nh_all = (cK + BK - 1) / BK;              // stages of the reduction
    // this workgroup's slice of them (grid.z slices of nh_slice consecutive stages; the host makes every slice non-empty)
    const int nh_slice = p.ksplit > 1 ? (nh_all + p.ksplit - 1) / p.ksplit : nh_all;
    const int s_begin = (int)blockIdx.z * nh_slice;
    const int s_end = s_begin + nh_slice < nh_all ? s_begin + nh_slice : nh_all;
    const int nh = (s_end - s_begin + C::KW - 1) / C::KW;   // ... per group (the last one may be empty for some groups)
    const bool ktail = (cK % BK) != 0;                  // last stage is partly beyond K

    // ------------------------------------------------------------ copy stage: A
    // LDS slot q = tid + i*THREADS is row q/RCH, physical 16-byte column q%RCH of the [BM][ROWB]
    // tile; the lane fetches the logical column that the swizzle stores there.
    const int a_r0 = tid / C::RCH;
    const int a_lc = (tid % C::RCH) ^ kmajor_swz<ROWB>(a_r0);   // same for every i (K_RSTEP % 16 == 0)
    unsigned a_off[C::A_IT];
    int a_hw[C::A_IT];
    int a_dz[C::AMODE == A_CONVX ? C::A_IT : 1];       // general decode: first input depth of the row's output pixel
    int a_res[C::AMODE == A_CONVX ? C::A_IT : 1];      // ... and the remainders of its tap-(0,0) coordinates modulo the up-sampling
    const char* a_base = Ab;
    long long a_bytes = 0;     // valid bytes from a_base (at k = 0)
    if constexpr (C::AMODE == A_KMAJOR) {
        // rows past M start beyond the descriptor and read as zeros
        a_base = Ab + (long long)m0 * p.a_rs * ES;
        const int rows = p.M - m0 < C::BM ? p.M - m0 : C::BM;
        a_bytes = ((long long)(rows - 1) * p.a_rs + p.K) * ES;
#pragma unroll
        for (int i = 0; i < C::A_IT; ++i)
            a_off[i] = (unsigned)(a_r0 + i * C::K_RSTEP) * (unsigned)(p.a_rs * ES) + a_lc * 16;
    } else if constexpr (C::AMODE == A_CONVX) {
        // ReIndex with a depth axis: row m of A_t is output pixel (img, od, op, oq) = unfuse(m); keep the
        // pixel index of the image's first pixel and the (possibly up-sampled) coordinates of tap (0,0,0)
        const int PQ = p.P * p.Q, OPQ = p.OD * PQ;
        a_bytes = (long long)p.batch_imgs * p.D * p.H * p.W * p.Cin * ES - bz * p.a_bs * ES;
#pragma unroll
        for (int i = 0; i < C::A_IT; ++i) {
            const int m = m0 + a_r0 + i * C::K_RSTEP;
            int id0 = 0, ih0 = -30000, iw0 = 0, img = 0;
            if (m < p.M) {
                img = (int)fastdiv((unsigned)m, p.div_opq_magic, p.div_opq_shift);
                const int rem = m - img * OPQ;
                const int od = (int)fastdiv((unsigned)rem, p.div_pq_magic, p.div_pq_shift), rem2 = rem - od * PQ;
                const int op = (int)fastdiv((unsigned)rem2, p.div_q_magic, p.div_q_shift), oq = rem2 - op * p.Q;
                id0 = od * p.stride_d - p.pad_d;
                ih0 = op * p.stride_h - p.pad_h;
                iw0 = oq * p.stride_w - p.pad_w;
            }
            // coordinate = up * quotient + remainder (floor division, once per row): tap offsets are uniform per
            // stage, so whether a tap hits an input pixel is decided by adding remainders, without a division
            int qh = ih0, qw = iw0;
            if (p.up_h != 1 || p.up_w != 1) {       // (uniform; a 3-D convolution never divides)
                qh = ih0 >= 0 ? ih0 / p.up_h : -((-ih0 + p.up_h - 1) / p.up_h);
                qw = iw0 >= 0 ? iw0 / p.up_w : -((-iw0 + p.up_w - 1) / p.up_w);
            }
            a_off[i] = (unsigned)img * (unsigned)(p.D * p.H * p.W);
            a_dz[i] = id0;
            a_hw[i] = (qh << 16) | (qw & 0xffff);
            a_res[i] = ((ih0 - qh * p.up_h) << 16) | (iw0 - qw * p.up_w);
        }
    } else {
        // ReIndex: row m of A_t is output pixel (img, op, oq) = unfuse(m); keep the element offset of
        // its top-left input pixel and that pixel's coordinates.
        a_bytes = (long long)p.batch_imgs * p.H * p.W * p.Cin * ES - bz * p.a_bs * ES;
        const int PQ = p.P * p.Q;
#pragma unroll
        for (int i = 0; i < C::A_IT; ++i) {
            const int m = m0 + a_r0 + i * C::K_RSTEP;
            // (decoded for rows past M too - the arithmetic is total - and then moved out of the image: no branch)
            const int img = (int)fastdiv((unsigned)m, p.div_pq_magic, p.div_pq_shift);
            const int rem = m - img * PQ;
            const int op = (int)fastdiv((unsigned)rem, p.div_q_magic, p.div_q_shift), oq = rem - op * p.Q;
            const int ih0 = m < p.M ? op * p.stride_h - cpad_h : -30000;
            const int iw0 = oq * p.stride_w - cpad_w;
            a_off[i] = (((unsigned)img * (unsigned)p.H + (unsigned)ih0) * (unsigned)p.W + (unsigned)iw0) * (unsigned)(p.Cin * ES);    // bytes, modulo 2^32
            a_hw[i] = (ih0 << 16) | (iw0 & 0xffff);
        }
    }

    // ------------------------------------------------------------ copy stage: B
    const int b_r0 = tid / C::RCH;                      // K-major only: row, physical and logical column of the thread's chunk
    const int b_pc = tid % C::RCH;
    const int b_lc = b_pc ^ kmajor_swz<ROWB>(b_r0);
    unsigned b_off[C::B_IT];
    const char* b_base = Bb;
    long long b_bytes = 0;
    long long b_step = ROWB;    // bytes the base advances per stage
    if constexpr (C::BMODE == B_KMAJOR) {
        b_base = Bb + (long long)n0 * p.b_cs * ES;
        const int rows = p.N - n0 < C::BN ? p.N - n0 : C::BN;
        b_bytes = ((long long)(rows - 1) * p.b_cs + p.K) * ES;
#pragma unroll
        for (int i = 0; i < C::B_IT; ++i)
            b_off[i] = (unsigned)(b_r0 + i * C::K_RSTEP) * (unsigned)(p.b_cs * ES) + b_lc * 16;
    } else {
        // k-rows of the stage; rows past K start beyond the descriptor (b_rs >= N is checked by the
        // host), columns past N are switched off per lane
        b_base = Bb + (long long)n0 * ES;
        b_bytes = ((long long)(p.K - 1) * p.b_rs + (p.N - n0)) * ES;
        b_step = (long long)BK * p.b_rs * ES;
#pragma unroll
        for (int i = 0; i < C::B_IT; ++i) {
            // the copying threads' i-th pass covers 16-byte chunks i*CT .. of the tile (k-rows of B_RC chunks, any count)
            const int chunk = i * C::CT + tid;
            const int k = chunk / C::B_RC, pc = chunk - k * C::B_RC;
            const int lb = (pc * 16) ^ nmajor_xor<C>(k);        // logical byte inside the k-row
            b_off[i] = (n0 + lb / ES < p.N) ? (unsigned)k * (unsigned)(p.b_rs * ES) + lb : kOutOfRange;
        }
    }

    // Per-stage copy state: descriptors (SGPRs) and, for the convolution, this stage's offsets and
    // the scalar tap cursor (filter row, filter column, channel offset of the next stage).
    const bool conv_uniform_tap = (C::AMODE == A_CONV || C::AMODE == A_CONVX) && (p.Cg % BK == 0);
    int conv_ft = 0, conv_fr = 0, conv_fs = 0, conv_cc = 0;
    auto conv_advance = [&](int stages) {                // move the tap cursor `stages` stages ahead
        conv_cc += stages * BK;
        while (conv_cc >= p.Cg) {
            conv_cc -= p.Cg;
            if (++conv_fs == cS) {
                conv_fs = 0;
                ++conv_fr;
                if constexpr (C::AMODE == A_CONVX) {
                    if (conv_fr == p.R) { conv_fr = 0; ++conv_ft; }
                }
            }
        }
    };
    if (conv_uniform_tap) conv_advance(s_begin + kgrp);
    // One stage ahead, branch-free (Cg is a multiple of the stage's k extent: at most one tap boundary per stage).
    auto conv_step = [&]() {
        conv_cc += BK;
        const bool tap_end = conv_cc >= p.Cg;
        conv_cc = tap_end ? 0 : conv_cc;
        conv_fs += tap_end ? 1 : 0;
        const bool row_end = conv_fs == cS;
        conv_fs = row_end ? 0 : conv_fs;
        conv_fr += row_end ? 1 : 0;
        if constexpr (C::AMODE == A_CONVX) {
            const bool plane_end = conv_fr == p.R;
            conv_fr = plane_end ? 0 : conv_fr;
            conv_ft += plane_end ? 1 : 0;
        }
    };
    i32x4 ra, rb;
    unsigned a_voff[C::A_IT];
    // Is tap offset d (rows in the high half, columns in the low half) of the packed pixel coordinates hw inside the
    // image?  Both 16-bit sums at once: a coordinate is inside iff clamping it to the last row / column (unsigned, so
    // negative ones are huge) leaves it unchanged.  The host keeps every coordinate within (-2^15, 2^16).
    typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
    const u16x2 hw_last = {(unsigned short)(p.W - 1), (unsigned short)(p.H - 1)};
    auto inside = [&](int hw, u16x2 d) -> bool {
        const u16x2 c = __builtin_bit_cast(u16x2, hw) + d;
        return __builtin_bit_cast(unsigned, __builtin_elementwise_min(c, hw_last)) == __builtin_bit_cast(unsigned, c);
    };
    char* lds_dst = ring;    // wave-uniform destination of this wave's first A chunk
    int c_slot = 0;          // ring slot and reduction stage of the next copy_begin (stages are prepared in order)
    int c_stage = s_begin + kgrp;

    // Prepare the copy of the next stage (descriptors, predicates) - stages are prepared strictly in order, the
    // counters above say which one is next; the loads themselves are issued one by one through copy_unit() so
    // that they can be interleaved with MFMAs.
    auto copy_begin = [&]() __attribute__((always_inline)) {
        lds_dst = ring + c_slot * C::STAGE_BYTES + wave * 1024;
        const int stage = c_stage;                                   // stage of the whole reduction
        c_slot = c_slot + 1 == NSTAGE ? 0 : c_slot + 1;
        c_stage += C::KW;
        const int nh = nh_all;
        const int tap_fr = conv_fr, tap_fs = conv_fs, tap_cc = conv_cc;    // the stage's tap, before the cursor moves on
        const bool live = stage < s_end;   // past the end: empty descriptors, the copies write zeros (they add nothing)
        if constexpr (C::AMODE == A_KMAJOR) {
            ra = make_rsrc32(a_base + (long long)stage * ROWB, live ? (unsigned)a_bytes - (unsigned)stage * ROWB : 0u);
            if (ktail && stage == nh - 1) {
                // K tail: the bytes between K and the row stride are not zero, switch those lanes off
                const bool kv = stage * BK + a_lc * VEC < p.K;
#pragma unroll
                for (int i = 0; i < C::A_IT; ++i) a_off[i] = kv ? a_off[i] : kOutOfRange;
            }
#pragma unroll
            for (int i = 0; i < C::A_IT; ++i) a_voff[i] = a_off[i];
        } else if constexpr (C::AMODE == A_CONVX) {
            // fuse(rt, rh, rw, rc) -> (rt, rh, rw, rc), per lane; taps step by tap_sign, and with up > 1 only
            // coordinates divisible by it are input pixels (the transposed convolution read as a gather)
            ra = make_rsrc32(Ab, live ? (unsigned)a_bytes : 0u);
            int ft, fr, fs, cc;
            bool kv;
            if (conv_uniform_tap) {
                // Cg is a multiple of the stage's k extent: one tap per stage, decoded by the scalar cursor
                ft = conv_ft; fr = conv_fr; fs = conv_fs;
                cc = conv_cc + a_lc * VEC;
                kv = live;
#pragma unroll
                for (int kw = 0; kw < C::KW; ++kw) conv_step();
            } else {
                const int kb = stage * BK + a_lc * VEC;
                const int tap = (int)fastdiv((unsigned)kb, p.div_cg_magic, p.div_cg_shift);
                cc = kb - tap * p.Cg;
                const int RS = p.R * p.S;
                ft = (int)fastdiv((unsigned)tap, p.div_rs_magic, p.div_rs_shift);
                const int rs = tap - ft * RS;
                fr = (int)fastdiv((unsigned)rs, p.div_s_magic, p.div_s_shift);
                fs = rs - fr * p.S;
                kv = kb < p.K;
            }
            // tap offset = up * quotient + remainder too (scalar in the one-tap-per-stage case); the sum of the two
            // remainders is 0 or up exactly when the tap lands on an input pixel
            const int dd = ft * p.dil_d, dh = p.tap_sign * fr * p.dil_h, dw = p.tap_sign * fs * p.dil_w;
            int dqh = dh, drh = 0, dqw = dw, drw = 0;
            if (p.up_h != 1 || p.up_w != 1) {       // (uniform; a 3-D convolution never divides)
                dqh = dh >= 0 ? dh / p.up_h : -((-dh + p.up_h - 1) / p.up_h); drh = dh - dqh * p.up_h;
                dqw = dw >= 0 ? dw / p.up_w : -((-dw + p.up_w - 1) / p.up_w); drw = dw - dqw * p.up_w;
            }
#pragma unroll
            for (int i = 0; i < C::A_IT; ++i) {
                const int idn = a_dz[i] + dd;
                const int sh = (a_res[i] >> 16) + drh, sw = (a_res[i] & 0xffff) + drw;
                const int ih = (a_hw[i] >> 16) + dqh + (sh == p.up_h ? 1 : 0);
                const int iw = (int)(short)(a_hw[i] & 0xffff) + dqw + (sw == p.up_w ? 1 : 0);
                const bool ok = kv && (unsigned)idn < (unsigned)p.D && (sh == 0 || sh == p.up_h) && (sw == 0 || sw == p.up_w) &&
                                (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
                a_voff[i] = ok ? ((a_off[i] + (unsigned)((idn * p.H + ih) * p.W + iw)) * (unsigned)p.Cin + (unsigned)cc) * ES : kOutOfRange;
            }
        } else {
            // fuse(rh, rw, rc) -> (rh, rw, rc); a 16-byte vector never straddles a tap (Cg % VEC == 0)
            ra = make_rsrc32(Ab, live ? (unsigned)a_bytes : 0u);
            if (conv_uniform_tap) {
                // Cg is a multiple of the stage's k extent: the whole stage belongs to one tap, so the tap
                // decode is scalar and advances incrementally (stages are prepared in order)
                const int dh = conv_fr * p.dil_h, dw = conv_fs * p.dil_w;
                const unsigned delta = (unsigned)(((dh * p.W + dw) * p.Cin + conv_cc) * ES) + a_lc * 16;
                // not live: the descriptor is empty (K = R*S*Cg is a multiple of the stage extent here)
                const u16x2 d_hw = {(unsigned short)dw, (unsigned short)dh};
#pragma unroll
                for (int i = 0; i < C::A_IT; ++i) a_voff[i] = inside(a_hw[i], d_hw) ? a_off[i] + delta : kOutOfRange;
#pragma unroll
                for (int kw = 0; kw < C::KW; ++kw) conv_step();
            } else {
                const int kb = stage * BK + a_lc * VEC;
                const int tap = (int)fastdiv((unsigned)kb, p.div_cg_magic, p.div_cg_shift);
                const int cc = kb - tap * p.Cg;
                const int fr = (int)fastdiv((unsigned)tap, p.div_s_magic, p.div_s_shift), fs = tap - fr * p.S;
                const int dh = fr * p.dil_h, dw = fs * p.dil_w;
                const unsigned delta = (unsigned)(((dh * p.W + dw) * p.Cin + cc) * ES);
                const bool kv = kb < p.K;
                const u16x2 d_hw = {(unsigned short)dw, (unsigned short)dh};
#pragma unroll
                for (int i = 0; i < C::A_IT; ++i) a_voff[i] = (kv && inside(a_hw[i], d_hw)) ? a_off[i] + delta : kOutOfRange;
            }
        }
        if constexpr (C::BMODE == B_KMAJOR) {
            // k offset of the stage inside a filter row: consecutive, or (by phase) that of the tap it stands for
            long long kb = (long long)stage * ROWB;
            if constexpr (C::AMODE == A_CONV) {
                if (phased) kb = (long long)(((f_r0 - p.phases_h * tap_fr) * p.S + (f_s0 - p.phases_w * tap_fs)) * p.Cg + tap_cc) * ES;
            }
            rb = make_rsrc32(b_base + kb, live ? (unsigned)b_bytes - (unsigned)kb : 0u);
            if (ktail && stage == nh - 1) {
                const bool kv = stage * BK + b_lc * VEC < p.K;
#pragma unroll
                for (int i = 0; i < C::B_IT; ++i) b_off[i] = kv ? b_off[i] : kOutOfRange;
            }
        } else {
            // a stage reads BK k-rows: the descriptor covers exactly those (32-bit size, bounded by the host for
            // 128 rows), or what is left of B in the last stage, so that rows past K stay out of range
            const unsigned b_window = (unsigned)(((long long)(BK - 1) * p.b_rs + (p.N - n0)) * ES);
            const unsigned b_left = (stage + 1) * BK <= p.K ? b_window : (unsigned)(b_bytes - stage * b_step);
            rb = make_rsrc32(b_base + stage * b_step, live ? b_left : 0u);
        }
    };
    // u-th copy instruction of the prepared stage (u < L): A chunks first, then B chunks.
    auto copy_unit = [&](int u) __attribute__((always_inline)) {
        if (u < C::A_IT) load_to_lds(ra, lds_dst + u * C::CT * 16, a_voff[u]);
        else load_to_lds(rb, lds_dst + C::A_BYTES + (u - C::A_IT) * C::CT * 16, b_off[u - C::A_IT]);
    };

    // ------------------------------------------------------------ copy waves
    // Issuing a global->LDS load holds the issuing wave for about 40 ns (measured: 75 ticks of the 1.9 GHz
    // counter per load, against 90 for a whole LDS read round trip), and the address arithmetic of the copy
    // comes on top: with four to six loads per wave and stage that is a third of a small tile's stage time
    // during which the wave feeds no MFMA.  Copy waves take all of it off the multiplying waves.  Both roles
    // meet at one barrier per stage: the copy waves arrive when the next stage has landed, the multiplying
    // waves when they have read the current one (whose slot the copy waves refill right after).
    if constexpr (SPEC) {
        if (copier) {
            if (nh > 0) {
                // (stages past the last one are not copied: see the multiplying waves' loop below)
#pragma unroll
                for (int st = 0; st < NSTAGE - 1; ++st) {
                    if (st < nh) {
                        copy_begin();
#pragma unroll
                        for (int u = 0; u < L; ++u) copy_unit(u);
                    }
                }
                if (nh >= NSTAGE - 1) copy_barrier<(NSTAGE - 2) * L>();
                else copy_barrier<0>();
                for (int h = 0; h < nh; ++h) {
                    if (h + NSTAGE - 1 < nh) {
                        copy_begin();
#pragma unroll
                        for (int u = 0; u < L; ++u) copy_unit(u);
                        copy_barrier<(NSTAGE - 2) * L>();
                    } else {
                        copy_barrier<0>();
                    }
                }
            }
            return;
        }
    }

    // ------------------------------------------------------------ MFMA stage
    const Frag<C> frag(lane, wm, wn);
    acc_t acc[C::MI][C::NI];
#pragma unroll
    for (int i = 0; i < C::MI; ++i)
#pragma unroll
        for (int j = 0; j < C::NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;   // reduction init

    typedef typename std::conditional<std::is_same<acc_t, f32x16>::value, float, int>::type acc_e;
    acc_e bias_r[C::NI];
    load_bias<C>(p, bz, n0, wn, lane, bias_r);

    // Fragment look-ahead: the fragments of k-step g are requested while k-step g - LA multiplies, into one of
    // LA + 1 register sets.  A wave with one or two MFMAs per k-step has 32-64 cycles of them in flight, less
    // than an LDS read's round trip, and stalls every k-step with a look-ahead of one.
    constexpr int LA = C::LA, NSET = LA + 1;
    static_assert(KSTEPS % NSET == 0 && LA < KSTEPS, "fragment sets rotate per k-step and must line up per stage");
    uint4 af[NSET][C::MI], bf[NSET][C::NI];

    // One k-step: the MI*NI MFMAs on fragment set `set`, interleaved with `nside` units of side
    // work: first the fragment reads of (ra_s, rb_s, rk) into set `into`, then copy units
    // [v0, v0 + nv).
    auto kstep = [&](int set, int into, const char* ra_s, const char* rb_s, int rk, int v0, int nv) __attribute__((always_inline)) {
        constexpr int NM = C::MI * C::NI;
        constexpr int NR = C::MI + C::NI;
        const int nside = NR + nv;
#pragma unroll
        for (int t = 0; t < NM; ++t) {
            acc[t / C::NI][t % C::NI] = InTraits<C::DT>::mfma(af[set][t / C::NI], bf[set][t % C::NI], acc[t / C::NI][t % C::NI]);
            TIR_FENCE();
#pragma unroll
            for (int u = t * nside / NM; u < (t + 1) * nside / NM; ++u) {
                if (u < C::MI) af[into][u] = frag.read_a1(ra_s, rk, u);
                else if (u < NR) bf[into][u - C::MI] = frag.read_b1(rb_s, rk, u - C::MI);
                else copy_unit(v0 + u - NR);
                TIR_FENCE();
            }
        }
    };

    if (nh > 0) {
        // prologue: fill NSTAGE-1 slots, wait for stage 0
        if constexpr (!SPEC) {
#pragma unroll
            for (int st = 0; st < NSTAGE - 1; ++st) {
                if (st < nh) {
                    copy_begin();
#pragma unroll
                    for (int u = 0; u < L; ++u) copy_unit(u);
                }
            }
        }
        if (nh >= NSTAGE - 1) copy_barrier<(NSTAGE - 2) * L>();
        else copy_barrier<0>();
#pragma unroll
        for (int kk = 0; kk < LA; ++kk) {
            frag.read_a(ring, kk, af[kk]);
            frag.read_b(ring + C::A_BYTES, kk, bf[kk]);
        }
        TIR_FENCE();

        // Copy units the multiplying waves issue per stage, and per k-step.  With a look-ahead of one they all
        // precede the barrier; with a longer one (rings of three slots or more) the barrier comes LA k-steps before the
        // stage's end and the units are spread over the whole stage, U_PRE of them before the barrier.
        constexpr int LM = SPEC ? 0 : L;
        constexpr int KS_COPY = LA == 1 ? KSTEPS - 1 : KSTEPS;
        constexpr int VPK = (LM + KS_COPY - 1) / KS_COPY;
        constexpr int U_PRE = (KSTEPS - LA) * VPK < LM ? (KSTEPS - LA) * VPK : LM;
        static_assert(NSTAGE >= 3 || LA == 1, "a ring of two copies the very stage the barrier waits for");
        int r_off = 0;                                             // byte offset of stage h's ring slot (h % NSTAGE, without the division)
        // One iteration of the loop described above; COPY: stage h+NSTAGE-1 exists and is copied meanwhile.  The last
        // NSTAGE-1 iterations have nothing left to copy (a copy instruction costs its wave ~60 cycles even when its
        // descriptor is empty, and short reductions are mostly tail): they wait for everything still in flight.
        auto iteration = [&](int h, auto copy_flag) __attribute__((always_inline)) {
            constexpr bool COPY = decltype(copy_flag)::value;
            constexpr int LC = COPY ? LM : 0;
            const char* sa = ring + r_off;
            const char* sb = sa + C::A_BYTES;
            r_off = r_off + C::STAGE_BYTES == NSTAGE * C::STAGE_BYTES ? 0 : r_off + C::STAGE_BYTES;
            const char* na = ring + r_off;
            if constexpr (!SPEC && COPY) copy_begin();
            TIR_FENCE();
#pragma unroll
            for (int kk = 0; kk < KSTEPS; ++kk) {
                // Before the first read of stage h+1: this wave's copy of it has landed (the copies issued after it
                // may be in flight: NSTAGE-3 whole stages and this iteration's first U_PRE units); after the barrier
                // everybody's has, and every wave is done reading stage h-1's slot ... and stage h (its last
                // fragments are in registers).
                if (kk == KSTEPS - LA) copy_barrier<COPY ? (NSTAGE - 3) * L + (SPEC ? L : U_PRE) : 0>();
                const int v0 = kk * VPK;
                const int nv = v0 + VPK <= LC ? VPK : (LC > v0 ? LC - v0 : 0);
                const int rk = kk + LA;
                if (rk < KSTEPS) kstep(kk % NSET, rk % NSET, sa, sb, rk, v0, nv);
                else kstep(kk % NSET, rk % NSET, na, na + C::A_BYTES, rk - KSTEPS, v0, nv);
            }
        };
        int h = 0;
        for (; h + NSTAGE - 1 < nh; ++h) iteration(h, std::true_type());
        for (; h < nh; ++h) iteration(h, std::false_type());
        // (nothing is in flight any more: the last iterations waited for every copy)
    }

    if constexpr (C::KW > 1) {
        // The groups' partial sums meet in LDS (every copy has landed and, after the barrier, every
        // wave is past its last fragment read): group 1 writes its accumulators, group 0 adds and stores.
        typedef typename std::conditional<std::is_same<acc_t, f32x16>::value, float, int>::type acc_e;
        typedef acc_e acc_e4 __attribute__((ext_vector_type(4)));
        acc_e4* xch = (acc_e4*)(smem + wave * (C::MI * C::NI * 4096));
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (kgrp != 0) {
#pragma unroll
            for (int i = 0; i < C::MI; ++i)
#pragma unroll
                for (int j = 0; j < C::NI; ++j)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        acc_e4 v;
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = acc[i][j][r4 * 4 + e];
                        xch[((i * C::NI + j) * 4 + r4) * 64 + lane] = v;
                    }
        }
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (kgrp != 0) return;
#pragma unroll
        for (int i = 0; i < C::MI; ++i)
#pragma unroll
            for (int j = 0; j < C::NI; ++j)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const acc_e4 v = xch[((i * C::NI + j) * 4 + r4) * 64 + lane];
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[i][j][r4 * 4 + e] += v[e];
                }
    }
    // (Tiles above 128x128 have no split: their partial sums would be 256 KiB and more per slice, and the code below
    // would push the big tiles' register allocation into scratch memory.  The host plans accordingly.)
    if (C::BM * C::BN <= kSplitMaxTile && p.ksplit > 1) {
        // Reduction split over workgroups.  Every slice leaves its partial sums in the workspace (one
        // 16-byte vector per lane and store: whole lines) and counts itself at the tile's counter; the
        // slice that finds every other one already counted adds all partial sums - its own included,
        // from memory, in slice order, so the rounding does not depend on the order of arrival - and
        // finishes the tile.  Nobody waits for anybody.
        // The slices of a tile run on different XCDs, whose L2s do not see each other's lines: the partial
        // sums are written through to memory and read past the caches (system-scope stores and loads);
        // a release / acquire fence pair would write back and invalidate a whole L2 per workgroup instead
        // (measured: 50-100 us per launch).  The stores have left the L2 when their counter drains, which
        // is before the workgroup's arrival is counted.
        typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
        constexpr int SLICE_BYTES = C::BM * C::BN * 4;
        constexpr int kSystemScope = 17;                         // sc0 | sc1
        const long long tile_lin = bz * ((long long)p.tiles_m * p.tiles_n) + blockIdx.x;
        const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
            (char*)p.ws + tile_lin * p.ksplit * SLICE_BYTES, 0, p.ksplit * SLICE_BYTES, 0x00020000);
        const int lane_off = (wave * (C::MI * C::NI * 4 * 64) + lane) * 16;     // block (i, j), quarter r4: + ((i*NI + j)*4 + r4) * 1024
#pragma unroll
        for (int i = 0; i < C::MI; ++i)
#pragma unroll
            for (int j = 0; j < C::NI; ++j)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    u32x4 v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const acc_e t = acc[i][j][r4 * 4 + e];      // a copy: bit_cast applied to a vector element reads element 0
                        v[e] = __builtin_bit_cast(unsigned, t);
                    }
                    __builtin_amdgcn_raw_buffer_store_b128(v, rw, lane_off + ((i * C::NI + j) * 4 + r4) * 1024,
                                                           (int)blockIdx.z * SLICE_BYTES, kSystemScope);
                }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");        // this wave's partial sums are in memory
        __syncthreads();                                        // ... and every wave's
        unsigned* const flag = (unsigned*)smem;                 // the rings are idle: every wave is past its last read
        if (threadIdx.x == 0) *flag = __hip_atomic_fetch_add(p.ws_count + tile_lin, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        __syncthreads();
        if (*flag != (unsigned)p.ksplit - 1u) return;
        if (threadIdx.x == 0) __hip_atomic_store(p.ws_count + tile_lin, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);   // ready for the next launch
#pragma unroll
        for (int i = 0; i < C::MI; ++i)
#pragma unroll
            for (int j = 0; j < C::NI; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
        // G slices of one 32x32 block are requested together (a load from memory takes longer than adding a
        // slice) and added in slice order; slices past the last one are switched off and add zeros
        constexpr int G = C::MI * C::NI >= 4 ? 2 : 4;      // (four at a time would push the 64x64 wave tiles' registers into scratch)
        for (int z0 = 0; z0 < p.ksplit; z0 += G) {
#pragma unroll
            for (int blk = 0; blk < C::MI * C::NI; ++blk) {
                u32x4 part[G][4];
#pragma unroll
                for (int g = 0; g < G; ++g)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4)
                        part[g][r4] = __builtin_amdgcn_raw_buffer_load_b128(rw, z0 + g < p.ksplit ? lane_off + (blk * 4 + r4) * 1024 : (int)kOutOfRange,
                                                                            (z0 + g) * SLICE_BYTES, kSystemScope);
#pragma unroll
                for (int g = 0; g < G; ++g)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4)
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const unsigned t = part[g][r4][e];
                            acc[blk / C::NI][blk % C::NI][r4 * 4 + e] += __builtin_bit_cast(acc_e, t);
                        }
            }
        }
    }
    if constexpr (C::AMODE == A_CONV) {
        if (phased) {
            store_tile_phase<C>(p, bz, m0, n0, wm, wn, lane, acc, bias_r, ph, pw);
            return;
        }
    }
    store_tile<C>(p, bz, m0, n0, wm, wn, lane, acc, bias_r);
}

// ---------------------------------------------------------------------------------------------
// Convolution with an LDS-resident input patch (channels per group = 128 bytes per pixel).
//
// The implicit-GEMM kernel above sends the im2col matrix A_t through the global->LDS copy, i.e.
// every input pixel R*S times.  Here the ReIndex step is applied on the LDS side instead: a
// workgroup owns 256 consecutive output pixels of one image, copies the input rows they touch
// (full width plus the zero halo, which out-of-range lanes of the copy deliver) into LDS once, and
// the MFMA A-fragments of tap (rh, rw) are read from that patch at
//     pixel(p*s_h + rh*d_h, q*s_w + rw*d_w)
// - the same formula as the paper's A_r[n,h,w,rh,rw,rc], evaluated per LDS read.  The filter of the
// 64 output channels is LDS-resident too: R*S slabs of [64 output channels][128 B], requested a few
// taps ahead.
// One LDS row per patch pixel, same XOR swizzle as the K-major tiles (keyed by the pixel index).
// 8 waves: four copy, four multiply; multiplying wave w owns output pixels [64w, 64w+64) x 64 output
// channels (2x2 MFMA blocks).
// ---------------------------------------------------------------------------------------------
template <int DT, int OUT>
__global__ void __launch_bounds__(512) conv_patch_kernel(const Params p) {
    typedef typename InTraits<DT>::acc_t acc_t;
    typedef OutTraits<OUT> OT;
    typedef typename OT::type out_t;
    constexpr int ES = elem_size(DT), OS = (int)sizeof(out_t);
    constexpr int SLAB = 64 * 128;              // one filter tap: 64 output channels x 128 B

    __shared__ __attribute__((aligned(1024))) char smem[160 * 1024];
    // every argument the kernel reads, fetched in one batch (see prefetch_args)
    asm volatile("" ::"s"(p.A), "s"(p.B), "s"(p.C), "s"(p.N), "s"(p.K), "s"(p.tiles_m), "s"(p.tiles_n), "s"(p.c_rs), "s"(p.bias), "s"(p.bias_bs),
                 "s"(p.relu), "s"(p.scale), "s"(p.batch_imgs), "s"(p.PW), "s"(p.store_nt));
    asm volatile("" ::"s"(p.H), "s"(p.W), "s"(p.Cin), "s"(p.Cg), "s"(p.P), "s"(p.Q), "s"(p.R), "s"(p.S), "s"(p.stride_h), "s"(p.stride_w), "s"(p.pad_h),
                 "s"(p.pad_w), "s"(p.dil_h), "s"(p.dil_w));
    asm volatile("" ::"s"(p.div_q_magic), "s"(p.div_q_shift), "s"(p.div_tn_magic), "s"(p.div_tn_shift), "s"(p.div_tm_magic), "s"(p.div_tm_shift),
                 "s"(p.div_pw_magic), "s"(p.div_pw_shift));
    asm volatile("" ::"s"(p.tap_px[0]), "s"(p.tap_px[1]), "s"(p.tap_px[2]), "s"(p.tap_px[3]), "s"(p.tap_px[4]), "s"(p.tap_px[5]), "s"(p.tap_px[6]),
                 "s"(p.tap_px[7]), "s"(p.tap_px[8]));
    char* const s_filt = smem;                  // R*S slabs, then the patch (the host checked that both fit)
    char* const s_patch = smem + p.R * p.S * SLAB;

    // Waves 0-3 copy (half of the patch, then the filter), waves 4-7 copy the other half of the patch and multiply.  A global->LDS copy instruction occupies its wave for
    // far longer than an MFMA does, and a wave issues in order: if the multiplying waves issued the
    // copies themselves, the matrix pipes would idle behind every one of them.  The copy role goes to
    // the first four waves because the second wave of each SIMD starts ~0.3 us after the first.
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool copier = wave < 4;
    const int cw = wave & 3;                    // index within the role
    const int tid = threadIdx.x & 255;          // thread index within the role
    const int lane = tid & 63;
    const int l31 = lane & 31, g = lane >> 5;

    // workgroup -> (image, pixel tile, channel tile); group = blockIdx.y
    // Workgroups go to the 8 L2 domains round-robin by launch index: give each domain a run of consecutive tiles,
    // so that the input rows two neighbouring pixel tiles share (the halo) are fetched into one L2 once.
    const int nwg = p.batch_imgs * p.tiles_m * p.tiles_n;       // = gridDim.x, without the late fetch of a hidden argument
    const int xq = nwg >> 3, xr = nwg & 7, xf = blockIdx.x & 7;
    const int bid = xf * xq + (xf < xr ? xf : xr) + (blockIdx.x >> 3);
    const int rest = (int)fastdiv((unsigned)bid, p.div_tn_magic, p.div_tn_shift);
    const int nt = bid - rest * p.tiles_n;
    const int img = (int)fastdiv((unsigned)rest, p.div_tm_magic, p.div_tm_shift);
    const int tix = rest - img * p.tiles_m;     // tiles_m = pixel tiles per image here
    const int grp = blockIdx.y;
    const int PQ = p.P * p.Q;
    const int m_first = tix * 256;
    const int m_cnt = PQ - m_first < 256 ? PQ - m_first : 256;
    const int n0 = nt * 64;
    const int ncols = p.N - n0 < 64 ? p.N - n0 : 64;          // N = output channels per group
    const int RS = p.R * p.S;

    // patch geometry: output rows p_a..p_b of this image, input rows ih_base .. ih_base + nrows - 1
    const int p_a = (int)fastdiv((unsigned)m_first, p.div_q_magic, p.div_q_shift), p_b = (int)fastdiv((unsigned)(m_first + m_cnt - 1), p.div_q_magic, p.div_q_shift);
    const int ih_base = p_a * p.stride_h - p.pad_h;
    const int nrows = (p_b - p_a) * p.stride_h + (p.R - 1) * p.dil_h + 1;
    const int PW = p.PW;                        // patch columns: (Q-1)*s_w + (S-1)*d_w + 1 rounded up to 8, the first is iw = -pad_w
    const int U = PW >> 3;                      // a copy instruction moves one unit: 8 consecutive pixels of one patch row (1 KiB)

    // Passes [first, last) of the patch copy; a pass is four units (32 pixels x 128 B), one per wave of the role.
    const int nit = (nrows * U + 3) >> 2;
    // The multiplying waves are idle until the patch is in: they copy its second half (measured 3/8 .. 8/8 for
    // the copy waves' share: one half each is fastest, 7.8 vs 8.45 us on the 56x56x64 benchmark convolution).
    const int nsplit = (nit + 1) / 2;
    // The role's passes [c_it, c_last) of the patch copy, one copy instruction per call.
    // Unit u = 4*pass + cw is row u / U, columns 8*(u % U) .. of the patch: row and first column are uniform, so
    // the address is a scalar base plus a constant of the lane and validity is one comparison per lane (columns;
    // a row outside the image compares against a width of 0).  Per-lane decoding of each pixel made a copy
    // instruction cost ~270 cycles to issue; this form costs about what a filter slab's does.
    const i32x4 rx = make_rsrc32((const char*)p.A, (unsigned)((long long)p.batch_imgs * p.H * p.W * p.Cin * ES));      // < 2^31: the host checks
    const int pix_bytes = p.Cin * ES;
    const int lp = lane >> 3;                                           // pixel of the unit
    // LDS slot (pixel lp, physical column lane & 7) holds logical column (lane & 7) ^ key(pixel index); the pixel
    // index is 8*u + lp with u = cw mod 4 throughout, so the key (4*(cw & 1) + lp / 2) mod 8 is a constant of the lane
    const unsigned lane_off = (unsigned)(lp * pix_bytes + grp * p.Cg * ES + (((lane & 7) ^ ((4 * (cw & 1) + (lp >> 1)) & 7)) << 4));
    int c_it = copier ? 0 : nsplit;
    const int c_last = copier ? nsplit : nit;
    const int u0 = 4 * c_it + cw;
    int ur = (int)fastdiv((unsigned)u0, p.div_pw_magic, p.div_pw_shift), uc = u0 - ur * U;          // (the host's constants divide by U)
    char* c_dst = s_patch + c_it * 4096 + cw * 1024;
    auto copy_step = [&]() __attribute__((always_inline)) {
        if (c_it < c_last) {
            const int ih = ih_base + ur, iw0 = 8 * uc - p.pad_w;
            const unsigned wlim = (ur < nrows && (unsigned)ih < (unsigned)p.H) ? (unsigned)p.W : 0u;
            const unsigned base = (unsigned)(((img * p.H + ih) * p.W + iw0) * pix_bytes);          // modulo 2^32; used only for pixels that exist
            const unsigned voff = (unsigned)(iw0 + lp) < wlim ? base + lane_off : kOutOfRange;
            load_to_lds_nt(rx, c_dst, voff);       // (a pixel is read by one workgroup, halo rows by two)
            c_dst += 4096;
            uc += 4;
            while (uc >= U) { uc -= U; ++ur; }
            ++c_it;
        }
    };

    if (copier) {
        // ------------------------------------------------------------ copy: patch, then one filter slab per tap
        while (c_it < c_last) copy_step();
        const long long Kd = p.K;                               // R*S*Cg
        const char* wbase = (const char*)p.B + ((long long)grp * p.N + n0) * Kd * ES;
        unsigned w_off[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int q2 = j * 256 + tid;
            const int n = q2 >> 3;
            const int lc = (q2 & 7) ^ kmajor_swz<128>(n);
            w_off[j] = n < ncols ? (unsigned)(n * (int)Kd * ES) + lc * 16 : kOutOfRange;
        }
        auto issue_slab = [&](int t) {
            const i32x4 rw = make_rsrc32(wbase + (long long)t * p.Cg * ES, (unsigned)(((long long)(ncols - 1) * Kd + p.Cg) * ES));
            char* dst = s_filt + t * SLAB + cw * 1024;
            load_to_lds(rw, dst, w_off[0]);
            load_to_lds(rw, dst + 4096, w_off[1]);
        };
        // Barrier t releases tap t: it needs the patch and slabs <= t+1 (the tap's last k-steps already
        // fetch fragments of tap t+1).  Copies complete in issue order, so "slab t+1 has landed" is "at
        // most 2*(issued - (t+2)) copy instructions of this wave outstanding".  Slabs are issued a few
        // taps ahead only, so that barrier 0 does not wait for the whole filter to be requested.
        constexpr int AHEAD = 3;
        int issued = 0;
        for (int t = 0; t < RS; ++t) {
            // (before barrier 0 only what the first tap and its successor need plus one: every copy requested ahead of it
            // is queued in front of the patch's last rows at the L2, which every workgroup of the launch asks at once)
            const int ahead = t == 0 ? 1 : AHEAD;
            const int want = t + 2 + ahead < RS ? t + 2 + ahead : RS;
            for (; issued < want; ++issued) issue_slab(issued);
            wait_vmcnt_upto(2 * (issued - (t + 2)));
            __builtin_amdgcn_s_barrier();
        }
        return;
    }

    while (c_it < c_last) copy_step();            // this role's share of the patch

    // ------------------------------------------------------------ fragment addressing
    // lane's output pixel of MFMA block i: m = 64*cw + 32*i + l31 -> patch pixel of tap (0,0)
    int base_px[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        int m = cw * 64 + i * 32 + l31;
        if (m >= m_cnt) m = m_cnt - 1;                         // rows past the tile re-read its last pixel; never stored
        const int mm = m_first + m;
        const int op = (int)fastdiv((unsigned)mm, p.div_q_magic, p.div_q_shift), oq = mm - op * p.Q;
        base_px[i] = (op - p_a) * p.stride_h * PW + oq * p.stride_w;
    }
    // Fragment addresses as byte offsets into smem.  A 128-byte row holds 16-byte column (2*kk + g) of k-step kk at physical
    // column (2*kk + g) ^ key: the k-step only flips bits 5 and 6 of the address, so a lane keeps the address of k-step 0
    // per tap (A: patch row of its pixel under that tap; B: its filter row in that tap's slab) and every read costs one
    // XOR.  With one multiplying wave per SIMD, whatever stands between two MFMAs beyond the 32 cycles the first one
    // takes leaves the matrix pipe idle: decoding pixel and swizzle in front of each read was a chain of five
    // dependent vector instructions.
    const int patch_base = p.R * p.S * SLAB;
    auto a_off0 = [&](int tap_px, int i) -> unsigned {
        const int px = base_px[i] + tap_px;
        return (unsigned)(patch_base + px * 128 + ((g ^ kmajor_swz<128>(px)) << 4));
    };
    const unsigned b_lane = (unsigned)(l31 * 128 + ((g ^ kmajor_swz<128>(l31)) << 4));        // + tap * SLAB, + 4096 for the second block
    auto read_at = [&](unsigned off0, int kk, int add) -> uint4 { return *(const uint4*)(smem + ((off0 ^ (unsigned)(kk << 5)) + add)); };

    acc_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;       // reduction init

    // the lane's two bias values, requested now: in the epilogue the load's latency would be exposed
    typedef typename std::conditional<std::is_same<acc_t, f32x16>::value, float, int>::type acc_e;
    acc_e bias_r[2];
    {
        const acc_e* base = (const acc_e*)p.bias + (long long)grp * p.bias_bs + n0;
        const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, p.bias ? ncols * 4 : 0, 0x00020000);
#pragma unroll
        for (int j = 0; j < 2; ++j) bias_r[j] = __builtin_bit_cast(acc_e, __builtin_amdgcn_raw_buffer_load_b32(rb, (j * 32 + l31) * 4, 0, 0));
    }

    // Fragment sets: k-step kk of every tap uses set kk, fetched two k-steps ahead (a k-step is only
    // four MFMAs long here, one k-step of lookahead would not cover the LDS latency).
    uint4 af[4][2], bf[4][2];
    const int row_step = p.dil_h * PW, col_step = p.dil_w;

    // Up to nine taps (3x3 and smaller filters): the loop over the taps is unrolled and the address of every fragment of
    // every tap is worked out here, after the wave's copies have been requested and while they land.  A wave issues in
    // order and this one is alone on its SIMD: in the generic loop below the tap cursor, the next tap's addresses and an
    // XOR per read stand between the MFMAs (770 cycles per tap against the 512 of its MFMAs and ~570 for the same
    // MFMAs issued from registers alone; 650 this way).  Measured against this placement: the arithmetic between the
    // copy instructions (the copies go out later: slower than not unrolling at all), and the last six taps' addresses
    // behind the MFMAs of taps 0 and 1 (1 % slower).
    unsigned aT[9][2][4];                         // [tap][pixel block][k-step]; the host lists the taps' patch offsets
    auto tap_addresses = [&](int t, int i) __attribute__((always_inline)) {
        const unsigned a0 = a_off0(p.tap_px[t], i);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            aT[t][i][kk] = a0 ^ (unsigned)(kk << 5);
            asm volatile("" : "+v"(aT[t][i][kk]));                    // here and now, in a register: not again next to its use
        }
    };
    if (RS <= 9) {
#pragma unroll
        for (int t = 0; t < 9; ++t)
#pragma unroll
            for (int i = 0; i < 2; ++i) tap_addresses(t, i);
    }

    if (RS <= 9) {
        // filter rows: slab t starts t * SLAB bytes on, which the read's offset field holds up to 64 KiB: two bases
        const char* bK[4][2];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            unsigned b0 = b_lane ^ (unsigned)(kk << 5), b1 = b0 + 32768;
            asm volatile("" : "+v"(b0), "+v"(b1));
            bK[kk][0] = smem + b0;
            bK[kk][1] = smem + b1;
        }
        auto read_b = [&](int t, int kk, int j) __attribute__((always_inline)) -> uint4 {
            return t < 8 ? *(const uint4*)(bK[kk][0] + t * SLAB + j * 4096) : *(const uint4*)(bK[kk][1] + (t * SLAB - 32768) + j * 4096);
        };
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // this wave's patch copies (and its bias) have landed
        __builtin_amdgcn_s_barrier();             // barrier 0: patch, slabs 0 and 1 are in LDS
        asm volatile("" ::: "memory");
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                af[kk][i] = *(const uint4*)(smem + aT[0][i][kk]);
                bf[kk][i] = read_b(0, kk, i);
            }
        TIR_FENCE();
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            if (t < RS) {
                if (t > 0) {
                    __builtin_amdgcn_s_barrier();     // barrier t: slab t+1 is in LDS
                    asm volatile("" ::: "memory");
                }
                TIR_FENCE();
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    // two k-steps ahead: same tap for kk < 2, the next tap's first k-steps otherwise; one read behind each MFMA
                    const int rk = (kk + 2) & 3, rt = kk < 2 ? t : t + 1;
                    acc[0][0] = InTraits<DT>::mfma(af[kk][0], bf[kk][0], acc[0][0]);
                    TIR_FENCE();
                    if (rt < 9) af[rk][0] = *(const uint4*)(smem + aT[rt][0][rk]);
                    TIR_FENCE();
                    acc[0][1] = InTraits<DT>::mfma(af[kk][0], bf[kk][1], acc[0][1]);
                    TIR_FENCE();
                    if (rt < 9) bf[rk][0] = read_b(rt, rk, 0);
                    TIR_FENCE();
                    acc[1][0] = InTraits<DT>::mfma(af[kk][1], bf[kk][0], acc[1][0]);
                    TIR_FENCE();
                    if (rt < 9) af[rk][1] = *(const uint4*)(smem + aT[rt][1][rk]);
                    TIR_FENCE();
                    acc[1][1] = InTraits<DT>::mfma(af[kk][1], bf[kk][1], acc[1][1]);
                    TIR_FENCE();
                    if (rt < 9) bf[rk][1] = read_b(rt, rk, 1);
                    TIR_FENCE();
                }
            }
        }
    } else {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");          // this wave's patch copies (and its bias) have landed
    __builtin_amdgcn_s_barrier();                 // barrier 0: patch, slabs 0 and 1 are in LDS
    asm volatile("" ::: "memory");
    constexpr int LOOK = 2;      // k-steps of lookahead (1, 2 and 3 measure alike)
    unsigned cA[2] = {a_off0(0, 0), a_off0(0, 1)}, cB = b_lane;      // k-step 0 of the current tap
    unsigned nA[2] = {cA[0], cA[1]}, nB = cB;                        // ... of the next one
#pragma unroll
    for (int kk = 0; kk < LOOK; ++kk)
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            af[kk][i] = read_at(cA[i], kk, 0);
            bf[kk][i] = read_at(cB, kk, i * 4096);
        }
    TIR_FENCE();

    // The tap cursor advances by additions under the tap's first MFMA, and the next tap's addresses (needed two k-steps
    // later) are worked out under the back-to-back MFMA pairs of the first two k-steps; an iteration ends on such a pair,
    // which covers the loop branch and the barrier.
    int tap_px = 0, row_px = 0, fs = 0;           // patch offsets of the current tap and of its filter row's first tap; filter column
    for (int t = 0; t < RS; ++t) {
        if (t > 0) {
            __builtin_amdgcn_s_barrier();         // barrier t: slab t+1 is in LDS
            asm volatile("" ::: "memory");
        }
        int next_px = tap_px;                     // (the last tap prefetches itself: those fragments are never used)
        TIR_FENCE();
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            // two k-steps ahead: same tap for kk < 2, the next tap's first k-steps otherwise
            const int rk = (kk + LOOK) & 3;
            const bool ahead = kk >= 4 - LOOK;
            acc[0][0] = InTraits<DT>::mfma(af[kk][0], bf[kk][0], acc[0][0]);
            TIR_FENCE();
            if (kk == 0) {
                const bool more = t + 1 < RS, wrap = fs + 1 == p.S;
                const int adv = wrap ? row_px + row_step : tap_px + col_step;
                next_px = more ? adv : tap_px;
                row_px = wrap ? row_px + row_step : row_px;
                fs = wrap ? 0 : fs + 1;
                nB = more ? cB + SLAB : cB;
            }
            af[rk][0] = read_at(ahead ? nA[0] : cA[0], rk, 0);
            bf[rk][0] = read_at(ahead ? nB : cB, rk, 0);
            TIR_FENCE();
            acc[0][1] = InTraits<DT>::mfma(af[kk][0], bf[kk][1], acc[0][1]);
            TIR_FENCE();
            af[rk][1] = read_at(ahead ? nA[1] : cA[1], rk, 0);
            bf[rk][1] = read_at(ahead ? nB : cB, rk, 4096);
            TIR_FENCE();
            acc[1][0] = InTraits<DT>::mfma(af[kk][1], bf[kk][0], acc[1][0]);
            acc[1][1] = InTraits<DT>::mfma(af[kk][1], bf[kk][1], acc[1][1]);
            TIR_FENCE();
            if (kk < 2) {                         // under the pair: 64 cycles of cover for five dependent instructions
                nA[kk] = a_off0(next_px, kk);
                TIR_FENCE();
            }
        }
        tap_px = next_px;
        cA[0] = nA[0]; cA[1] = nA[1]; cB = nB;
    }
    }

    // ------------------------------------------------------------ fused epilogue (NHWC rows are output pixels)
    out_t* ybase = (out_t*)p.C + ((long long)img * PQ + m_first) * p.c_rs + (long long)grp * p.N + n0;
    const bool fused = p.bias != nullptr || p.relu != 0;
    // (loads and stores retire through one counter, in order: wait for the bias before the first store)
    asm volatile("" ::"v"(bias_r[0]), "v"(bias_r[1]));
    const long long bytes = ((long long)(m_cnt - 1) * p.c_rs + ncols) * OS;
    const __amdgpu_buffer_rsrc_t rc = __builtin_amdgcn_make_buffer_rsrc((void*)ybase, 0, (int)bytes, 0x00020000);
    const int row_bytes = (int)p.c_rs * OS;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = j * 32 + l31;
            const int row0 = cw * 64 + i * 32 + 4 * g;
            const unsigned voff = col < ncols ? (unsigned)(row0 * row_bytes + col * OS) : kOutOfRange;
            store_block<OUT>(acc[i][j], fused, bias_r[j], p.relu, p.scale, rc, (int)voff, row_bytes, p.store_nt != 0);
        }
    }
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
    static_assert(C::BMODE == B_GENERIC && C::ROWB == 128 && C::NSTAGE == 2, "");
    typedef typename std::conditional<ES == 2, unsigned short, unsigned char>::type elem_t;

    __shared__ __attribute__((aligned(16))) char smem[C::LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / C::WN, wn = wave % C::WN;

    int tm, tn;
    tile_of_block(blockIdx.x, p.tiles_m, p.tiles_n, p.div_gw_magic, p.div_gw_shift, &tm, &tn);
    const int m0 = tm * C::BM, n0 = tn * C::BN;
    const long long bz = blockIdx.y;

    const elem_t* A = (const elem_t*)p.A + bz * p.a_bs;
    const elem_t* B = (const elem_t*)p.B + bz * p.b_bs;

    const int c8 = tid & 7;
    const int r0 = tid >> 3;
    constexpr int RSTEP = C::THREADS / 8;
    unsigned a_off[C::A_IT];
    int a_hw[C::A_IT], a_dz[C::A_IT];
    if constexpr (C::AMODE == A_CONV_GENERIC) {
        // general decode (depth axis, transposed form); a plain 2-D convolution has OD = D = T = 1, up = 1
        const int PQ = p.P * p.Q, OPQ = p.OD * PQ;
#pragma unroll
        for (int i = 0; i < C::A_IT; ++i) {
            const int m = m0 + r0 + i * RSTEP;
            int id0 = 0, ih0 = -30000, iw0 = 0, img = 0;
            if (m < p.M) {
                img = m / OPQ;
                const int rem = m - img * OPQ;
                const int od = rem / PQ, rem2 = rem - od * PQ;
                const int op = rem2 / p.Q, oq = rem2 - op * p.Q;
                id0 = od * p.stride_d - p.pad_d;
                ih0 = op * p.stride_h - p.pad_h;
                iw0 = oq * p.stride_w - p.pad_w;
            }
            a_off[i] = (unsigned)img * (unsigned)(p.D * p.H * p.W);
            a_dz[i] = id0;
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
                    const int RS = p.R * p.S;
                    const int ft = tap / RS, rs = tap - ft * RS;
                    const int fr = rs / p.S, fs = rs - fr * p.S;
                    const int idn = a_dz[i] + ft * p.dil_d;
                    int ih = (a_hw[i] >> 16) + p.tap_sign * fr * p.dil_h;
                    int iw = (int)(short)(a_hw[i] & 0xffff) + p.tap_sign * fs * p.dil_w;
                    bool ok = kb < p.K && (unsigned)idn < (unsigned)p.D && ih >= 0 && iw >= 0;
                    const int qh = ih / p.up_h, qw = iw / p.up_w;
                    ok = ok && qh * p.up_h == ih && qw * p.up_w == iw && qh < p.H && qw < p.W;
                    v[e] = ok ? A[(long long)(a_off[i] + (unsigned)((idn * p.H + qh) * p.W + qw)) * p.Cin + cc] : (elem_t)0;
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
        for (int i = 0; i < C::A_IT; ++i) *(uint4*)(sa + kmajor_off<128>(r0 + i * RSTEP, c8)) = ra[i];
#pragma unroll
        for (int i = 0; i < C::B_IT; ++i) *(uint4*)(sb + kmajor_off<128>(r0 + i * RSTEP, c8)) = rb[i];
    };

    const Frag<C> frag(lane, wm, wn);
    acc_t acc[C::MI][C::NI];
#pragma unroll
    for (int i = 0; i < C::MI; ++i)
#pragma unroll
        for (int j = 0; j < C::NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;   // reduction init

    typedef typename std::conditional<std::is_same<acc_t, f32x16>::value, float, int>::type acc_e;
    acc_e bias_r[C::NI];
    load_bias<C>(p, bz, n0, wn, lane, bias_r);

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
            for (int kk = 0; kk < C::KSTEPS; ++kk) {
                uint4 af[C::MI], bf[C::NI];
                frag.read_a(sa, kk, af);
                frag.read_b(sa + C::A_BYTES, kk, bf);
                mfma_block<C>(af, bf, acc);
            }
            if (more) store_ab(cur ^ 1);
            __syncthreads();
        }
    }

    store_tile<C>(p, bz, m0, n0, wm, wn, lane, acc, bias_r);
}

}  // namespace tir
