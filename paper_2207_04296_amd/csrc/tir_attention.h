// One attention head per (batch, 128-query tile): S = scale * Q K^T, row softmax, O = P V, in one
// kernel.  Both contractions are tensorized blocks (Eq. 1 of the TensorIR paper, mapped onto the
// 32x32x16 MFMA) that share the workgroup's tile instead of meeting in memory: the probabilities never
// leave the registers (sec. 2 / 3.2: blocks isolate the two sub-problems, which does not prevent
// cooperation across them).  The softmax is the textbook one, computed online over 128-key chunks.
//
// Both products are computed transposed, S^T = K Q^T and O^T = V^T P^T, so that the second MFMA
// operand - whose row index is the lane - is the query in both: every lane then owns one query row,
// the row maximum / row sum are reductions over the lane's own registers plus one exchange between
// the two half-waves, rescaling O by exp(m_old - m_new) is a per-lane scalar multiply, and the
// probabilities come out of the first MFMA already in the register layout the second one reads them
// in (the k-order of an MFMA is free as long as both operands use the same one; V^T is fetched with
// the transposing LDS read in the order the probabilities happen to have).
#pragma once
#include "tir_kernel.h"

namespace tir {

struct AttnParams {
    const void* Q;   // [batch][M][D]
    const void* K;   // [batch][N][D]
    const void* V;   // [batch][N][D]
    void* O;         // [batch][M][D]
    int M, N, batch;
    int tiles_m;     // ceil(M / 128)
    float scale_log2e;   // scale * log2(e): the softmax runs in base 2
    unsigned div_tm_magic;   // workgroup id / tiles_m as multiply-and-shift (make_fastdiv)
    int div_tm_shift;
    int store_nt;            // the output is not read again soon: non-temporal stores (see TIR_STORE_AUX_STREAM)
};

template <int DT> struct PackP;
template <> struct PackP<DT_F16> {
    static __device__ __forceinline__ unsigned two(float a, float b) {
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        h2 v = {(_Float16)a, (_Float16)b};
        return __builtin_bit_cast(unsigned, v);
    }
};
template <> struct PackP<DT_BF16> {
    static __device__ __forceinline__ unsigned two(float a, float b) {
        typedef __bf16 b2 __attribute__((ext_vector_type(2)));
        b2 v = {(__bf16)a, (__bf16)b};          // one v_cvt_pk_bf16_f32
        return __builtin_bit_cast(unsigned, v);
    }
};

// DT: f16 / bf16 inputs, OUT: same 16-bit type or f32, DH: head dimension (64 or 128) of Q, K and V.
template <int DT, int OUT, int DH>
__global__ void __launch_bounds__(256) attention_kernel(const AttnParams p) {
    typedef OutTraits<OUT> OT;
    typedef typename OT::type out_t;
    constexpr int OS = (int)sizeof(out_t);
    constexpr int ROW = DH * 2;                 // bytes of one Q / K / V row
    constexpr int HALVES = DH / 64;             // 128-byte column groups of a K-major row
    constexpr int TILE = 128 * ROW;             // one 128-row tile
    constexpr int KSTEPS = DH / 16;             // MFMA k-steps over the head dimension
    constexpr int DB = DH / 32;                 // 32-wide blocks of the output's head dimension
    constexpr int VRC = ROW / 16;               // 16-byte chunks per V row
    // V tile [key][ROW] with the transposing-read swizzle: byte offset XOR ((key / RPW) % NSEG) * 64
    constexpr int WIN = ROW < 256 ? ROW : 256;
    constexpr int NSEG = WIN / 64, RPW = 256 / WIN;
    static_assert(DH == 64 || DH == 128, "head dimension");
    static_assert(TILE * 5 <= 160 * 1024, "Q + two stages of K and V");

    __shared__ __attribute__((aligned(1024))) char smem[5 * TILE];
    char* const s_q = smem;
    auto s_k = [&](int st) { return smem + TILE + st * 2 * TILE; };
    auto s_v = [&](int st) { return smem + 2 * TILE + st * 2 * TILE; };

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l31 = lane & 31, g = lane >> 5;
    const int blk = lane >> 4, s16 = lane & 15;

    const long long b = fastdiv(blockIdx.x, p.div_tm_magic, p.div_tm_shift);
    const int tm = (int)blockIdx.x - (int)b * p.tiles_m;
    const int m0 = tm * 128;
    const int rows_q = p.M - m0 < 128 ? p.M - m0 : 128;
    const int nchunk = (p.N + 127) / 128;

    // ------------------------------------------------------------ copy stage
    // K-major tile (Q, K): slot q = tid + i*256 is row q / (8*HALVES)... kept as HALVES sub-tiles of
    // [128 rows][128 B] so that the row swizzle of the GEMM kernels applies unchanged.
    auto copy_kmajor = [&](const char* base, long long valid_bytes, char* dst, bool nt) {
        const i32x4 r = make_rsrc(base, valid_bytes);
#pragma unroll
        for (int h = 0; h < HALVES; ++h)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int q = tid + i * 256;              // 1024 chunks of 16 B per sub-tile
                const int row = q >> 3;
                const int lc = (q & 7) ^ kmajor_swz<128>(row);
                if (nt) load_to_lds_nt(r, dst + h * (128 * 128) + i * 4096 + wave * 1024, (unsigned)(row * ROW + h * 128 + lc * 16));
                else load_to_lds(r, dst + h * (128 * 128) + i * 4096 + wave * 1024, (unsigned)(row * ROW + h * 128 + lc * 16));
            }
    };
    auto copy_v = [&](const char* base, long long valid_bytes, char* dst, bool nt) {
        const i32x4 r = make_rsrc(base, valid_bytes);
#pragma unroll
        for (int i = 0; i < 4 * HALVES; ++i) {
            const int q = tid + i * 256;
            const int key = q / VRC;
            const int lb = ((q % VRC) * 16) ^ (((key / RPW) % NSEG) * 64);
            if (nt) load_to_lds_nt(r, dst + i * 4096 + wave * 1024, (unsigned)(key * ROW + lb));
            else load_to_lds(r, dst + i * 4096 + wave * 1024, (unsigned)(key * ROW + lb));
        }
    };
    const char* Qb = (const char*)p.Q + ((b * p.M + m0) * (long long)ROW);
    const char* Kb = (const char*)p.K + b * p.N * (long long)ROW;
    const char* Vb = (const char*)p.V + b * p.N * (long long)ROW;
    // Non-temporal copies for what one workgroup alone reads - the queries always, keys and values when one tile holds all
    // queries of a head: 7.05 -> 6.63 us on the benchmark's 192 heads with the operands coming from memory, no change from the caches.
    const bool kv_once = p.tiles_m == 1;
    auto copy_chunk = [&](int c) {
        const long long left = (long long)(p.N - c * 128) * ROW;      // rows past N lie outside the descriptor: zeros
        copy_kmajor(Kb + (long long)c * TILE, left, s_k(c & 1), kv_once);
        copy_v(Vb + (long long)c * TILE, left, s_v(c & 1), kv_once);
    };
    copy_kmajor(Qb, (long long)rows_q * ROW, s_q, true);
    copy_chunk(0);
    // Q and the first keys are enough to start on the scores: the first values (the newest 4*HALVES
    // copies of this wave) may still be in flight, they are waited for before the second product
    wait_vmcnt_upto(4 * HALVES);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    // ------------------------------------------------------------ this wave's queries, as MFMA operands
    const int swl = kmajor_swz<128>(l31);            // rows 32*w + l31 and 32*jb + l31 share it (period 16)
    uint4 qf[KSTEPS];
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks)
        qf[ks] = *(const uint4*)(s_q + (ks >> 2) * (128 * 128) + (wave * 32 + l31) * 128 + ((((ks & 3) * 2 + g) ^ swl) << 4));

    f32x16 acc_o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[db][r] = 0.f;          // reduction init
    float m_run = -__builtin_inff(), l_run = 0.f;

    for (int c = 0; c < nchunk; ++c) {
        if (c + 1 < nchunk) copy_chunk(c + 1);        // its stage was last read before the previous barrier
        const char* sk = s_k(c & 1);
        const char* sv = s_v(c & 1);

        // S^T = K Q^T: rows = keys (registers), columns = queries (lanes)
        f32x16 acc_s[4];
#pragma unroll
        for (int jb = 0; jb < 4; ++jb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_s[jb][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
                const uint4 kf = *(const uint4*)(sk + (ks >> 2) * (128 * 128) + (jb * 32 + l31) * 128 + ((((ks & 3) * 2 + g) ^ swl) << 4));
                acc_s[jb] = InTraits<DT>::mfma(kf, qf[ks], acc_s[jb]);
            }
        }
        // scores in base 2; keys past N (only in the last chunk) drop out of the softmax
        const bool ragged = (c + 1) * 128 > p.N;
        float mx = -__builtin_inff();
#pragma unroll
        for (int jb = 0; jb < 4; ++jb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float s = acc_s[jb][r] * p.scale_log2e;
                if (ragged && c * 128 + jb * 32 + 8 * (r >> 2) + 4 * g + (r & 3) >= p.N) s = -__builtin_inff();
                acc_s[jb][r] = s;
                mx = __builtin_fmaxf(mx, s);
            }
        mx = __builtin_fmaxf(mx, __shfl_xor(mx, 32));           // the other half-wave holds the query's other keys
        const float m_new = __builtin_fmaxf(m_run, mx);          // finite: every chunk has at least one valid key
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        float lsum = 0.f;
        uint4 pf[4][2];                                           // P^T fragments: key block jb, k-step s
#pragma unroll
        for (int jb = 0; jb < 4; ++jb) {
            float pr[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                pr[r] = __builtin_amdgcn_exp2f(acc_s[jb][r] - m_new);
                lsum += pr[r];
            }
#pragma unroll
            for (int s = 0; s < 2; ++s)
                pf[jb][s] = make_uint4(PackP<DT>::two(pr[8 * s + 0], pr[8 * s + 1]), PackP<DT>::two(pr[8 * s + 2], pr[8 * s + 3]),
                                       PackP<DT>::two(pr[8 * s + 4], pr[8 * s + 5]), PackP<DT>::two(pr[8 * s + 6], pr[8 * s + 7]));
        }
        l_run = l_run * alpha + lsum;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_o[db][r] *= alpha;

        if (c == 0) {
            // the first values: everything but the next chunk's copies (issued after them) has landed
            wait_vmcnt_upto(nchunk > 1 ? 8 * HALVES : 0);
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        }
        // O^T += V^T P^T.  Position (g, 4*hh + e) of k-step s in key block jb is key
        // 32*jb + 16*s + 8*hh + 4*g + e - the order the probabilities sit in the registers above.
#pragma unroll
        for (int jb = 0; jb < 4; ++jb)
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    i16x4 h[2];
#pragma unroll
                    for (int hh = 0; hh < 2; ++hh) {
                        const int key = jb * 32 + s * 16 + hh * 8 + 4 * (blk >> 1) + (s16 >> 2);
                        const int col = db * 32 + 16 * (blk & 1) + 4 * (s16 & 3);
                        const char* ptr = sv + key * ROW + ((col * 2) ^ (((key / RPW) % NSEG) * 64));
                        h[hh] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(TIR_LDS_PTR(i16x4, ptr));
                    }
                    const i32x2 lo = __builtin_bit_cast(i32x2, h[0]), hi = __builtin_bit_cast(i32x2, h[1]);
                    const uint4 vf = make_uint4((unsigned)lo[0], (unsigned)lo[1], (unsigned)hi[0], (unsigned)hi[1]);
                    acc_o[db] = InTraits<DT>::mfma(vf, pf[jb][s], acc_o[db]);
                }

        // the next chunk has landed (this wave's part); after the barrier everybody's has, and every
        // wave is done reading this chunk's stage
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    }

    // ------------------------------------------------------------ normalise, stage through LDS, store rows
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = 1.0f / l_tot;
    constexpr int ORB = DH * OS;                     // bytes of one output row
    char* const s_o = smem + TILE;                   // the K / V stages are free now (ORB * 128 <= 4 * TILE)
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            // registers 4*q4 .. 4*q4+3 are head-dimension columns dv0 .. dv0+3 of query 32*wave + l31
            const int row = wave * 32 + l31;
            const int dv0 = db * 32 + 8 * q4 + 4 * g;
            char* dst = s_o + row * ORB + ((dv0 * OS) ^ ((row & 7) << 4));
            alignas(16) out_t v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = OT::cvt(acc_o[db][4 * q4 + e] * inv);
            if constexpr (OS == 4) *(uint4*)dst = *(const uint4*)v;
            else *(uint2*)dst = *(const uint2*)v;
        }
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    {
        char* Ob = (char*)p.O + (b * p.M + m0) * (long long)ORB;
        const __amdgpu_buffer_rsrc_t ro = __builtin_amdgcn_make_buffer_rsrc((void*)Ob, 0, rows_q * ORB, 0x00020000);
        constexpr int ORC = ORB / 16;                // 16-byte chunks per output row
#pragma unroll
        for (int i = 0; i < 128 * ORC / 256; ++i) {
            const int q = tid + i * 256;
            const int row = q / ORC, pc = q % ORC;
            typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
            const u32x4 v = *(const u32x4*)(s_o + row * ORB + ((pc * 16) ^ ((row & 7) << 4)));
            if (p.store_nt) __builtin_amdgcn_raw_buffer_store_b128(v, ro, row * ORB + pc * 16, 0, TIR_STORE_AUX_STREAM);
            else __builtin_amdgcn_raw_buffer_store_b128(v, ro, row * ORB + pc * 16, 0, TIR_STORE_AUX);   // rows past M: outside the descriptor
        }
    }
}

typedef hipError_t (*attn_launch_fn)(const AttnParams&, hipStream_t);
// (dt, out, head dimension) -> launcher, or null when the combination is not compiled
attn_launch_fn attention_launcher(int dt, int out, int dh);

}  // namespace tir
