// Kernel parameter block and small host/device helpers shared by the host dispatcher and the
// gfx950 kernels.  Nothing here is visible across the C ABI.
#pragma once
#include <cstddef>
#include <stdint.h>

namespace tir {

enum : int { DT_F16 = 0, DT_BF16 = 1, DT_I8 = 2, DT_F32 = 3, DT_I32 = 4 };

// How the A (x,k) tile and the B (k,y) tile are fetched from global memory.
enum : int {
    A_KMAJOR = 0,   // A[x][k], k contiguous, 16-byte vectors
    A_CONV = 1,     // implicit im2col of an NHWC tensor, channel vectors of 16 bytes
    A_GENERIC = 2,  // any strides, element-wise loads
    A_CONV_GENERIC = 3,  // implicit im2col, element-wise (C/groups not a multiple of the vector)
    A_CONV_PATCH = 4,    // convolution reading its taps from an LDS-resident input patch (128 B per pixel)
    A_DEPTHWISE = 6,     // depth-wise 2-D convolution (one filter per channel): direct kernel, no matrix intrinsic
    A_CONVX = 5          // implicit im2col with the general coordinate decode: a depth axis (3-D convolution) and the
                         // transposed form (taps step backwards, only every up-th coordinate is an input pixel)
};
enum : int {
    B_KMAJOR = 0,   // B stored [y][k], k contiguous (a "transposed" B, or a KRSC filter)
    B_NMAJOR = 1,   // B stored [k][y], y contiguous (row-major B); transposed on the LDS read
    B_GENERIC = 2   // any strides, element-wise loads
};

// Kernel arguments.  The block is fetched through the scalar cache 64 bytes at a time and a kernel's first copy waits
// for every field it needs, so what all kernels read sits in the first three lines and the convolution-only fields
// follow (the kernels name their fields up front, which makes the compiler fetch them in one batch).
struct Params {
    // ---- line 0
    const void* A;
    const void* B;
    void* C;
    int M, N, K;      // extents of one contraction (per batch / per group)
    int batch;        // number of independent contractions (grid.y)
    int tiles_m, tiles_n;
    int c_fast;       // C has unit column stride, disjoint rows and 31-bit tile offsets: buffer-store epilogue
    // reduction split over workgroups (fast kernels): ksplit slices (grid.z) reduce consecutive runs of stages
    // of one output tile; each writes its partial sums to ws, the slice that arrives last at the tile's counter
    // adds all of them in slice order (the sum does not depend on who is last) and runs the epilogue
    int ksplit;          // 1: no split, ws and ws_count unused
    // Divisions by launch constants as multiply-and-shift (make_fastdiv; m < 2^31).  A runtime
    // integer division is a chain of ~25 dependent instructions, and the kernels' first copy waits for several.
    unsigned div_gw_magic;                   // id / (kGroupM * tiles_n): the workgroup -> tile map
    int div_gw_shift;
    // ---- line 1
    long long a_bs, b_bs, c_bs;                 // per-batch offsets, in elements
    long long a_rs, a_cs, b_rs, b_cs, c_rs;     // element strides; for conv: a_* unused
    // ---- line 2
    long long c_cs;
    // fused consumer: out = cvt(relu(acc + bias[column])); bias is fp32 (float inputs) or int32 (int8 inputs)
    const void* bias;    // null: no bias
    long long bias_bs;   // bias elements between consecutive grid.y slices (conv groups: channels per group; batches: 0)
    int relu;
    float scale;         // int8 output only: code = clamp(rint(float(t) * scale), -128, 127)
    void* ws;            // partial sums: [grid.y][tile][slice][BM*BN] accumulator elements (4 bytes each)
    unsigned* ws_count;  // [grid.y][tile] arrival counters, zero between launches (the last slice resets its tile's)
    int batch_imgs;   // convolutions: images in x (for the descriptor)
    int PW;           // patch kernel: columns of the LDS-resident input patch (a multiple of 8)
    int store_nt;     // the caller does not read the output again soon: non-temporal epilogue stores (see TIR_STORE_AUX_STREAM)
    int reserved0;
    // ---- convolution geometry (A_CONV*): x is [n][H][W][Cin], one group reads Cg channels
    int H, W, Cin, Cg, P, Q, R, S;
    int stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
    unsigned div_pq_magic, div_q_magic;      // m / (P*Q) and m / Q: output row -> (image, row, column)
    int div_pq_shift, div_q_shift;
    unsigned div_cg_magic, div_s_magic, div_rs_magic;      // k / Cg, tap / S, tap / (R*S): per-lane tap decode when a stage spans taps
    int div_cg_shift, div_s_shift, div_rs_shift;
    unsigned div_tn_magic, div_tm_magic, div_pw_magic;     // patch kernel: id / tiles_n, id / tiles_m, copy unit / (PW / 8)
    int div_tn_shift, div_tm_shift, div_pw_shift;
    int tap_px[9];    // patch kernel, filters of up to nine taps: patch pixel offset (r*dil_h*PW + s*dil_w) of tap t = r*S + s; taps past the last repeat it
    // Transposed convolution by output phase (A_CONV variants; phases_h = 0: off).  The output pixels with
    // (oh mod phases_h, ow mod phases_w) = (ph, pw) form a stride-1 convolution of the input with the filter taps
    // r = r0 + phases_h*t, r0 = (ph + t_pad_h) mod phases_h (likewise in w): grid.y enumerates (phase, group), the
    // kernel derives that phase's tap subset, padding and output pixels.  P, Q are then the extents of one phase's
    // pixel grid (ceil(P_full / phases_h) ...), M = images * P * Q, R, S, K those of the whole filter.
    int phases_h, phases_w, t_pad_h, t_pad_w, P_full, Q_full, conv_groups;
    unsigned div_grp_magic, div_phh_magic, div_phw_magic;  // by phase: / conv_groups, / phases_h, / phases_w
    int div_grp_shift, div_phh_shift, div_phw_shift;
    // general convolution decode (A_CONVX, A_CONV_GENERIC); a plain 2-D convolution has D = T = OD = 1, stride_d = dil_d = 1,
    // pad_d = 0, tap_sign = 1, up_h = up_w = 1.  Input coordinate of output pixel (o, p, q) and tap (t, r, s):
    //   depth  o*stride_d - pad_d + t*dil_d
    //   height (p*stride_h - pad_h + tap_sign*r*dil_h) / up_h   if divisible by up_h, else the tap reads zero; width alike
    int D, T, OD, stride_d, pad_d, dil_d;
    int tap_sign, up_h, up_w;
    unsigned div_opq_magic;                  // m / (OD*P*Q): with a depth axis
    int div_opq_shift;
    unsigned div_dwq_magic, div_dwpq_magic;                // depth-wise, pixel blocks: / ceil(Q / kDwBlockPix), / (P * that)
    int div_dwq_shift, div_dwpq_shift;
};
static_assert(offsetof(Params, a_bs) == 64 && offsetof(Params, c_cs) == 128 && offsetof(Params, H) == 192, "the lines described above");

// Exact unsigned division of m < 2^31 by a fixed d >= 1 without a branch or a special case: with s = ceil(log2 d)
// and magic = floor(2^32 * (2^s - d) / d) + 1 < 2^32,  m / d = (mulhi(m, magic) + m) >> s  (the round-up method of
// Granlund and Montgomery; m < 2^31 keeps the sum inside 32 bits).  d = 1 gives magic 0, shift 0.
struct FastDiv {
    unsigned magic;
    int shift;
};
inline FastDiv make_fastdiv(unsigned d) {
    FastDiv f = {0u, 0};
    if (d <= 1) return f;
    int s = 0;
    while ((1ull << s) < d) ++s;
    f.magic = (unsigned)(((1ull << (32 + s)) / d) + 1ull - (1ull << 32));
    f.shift = s;
    return f;
}
__host__ __device__ inline unsigned fastdiv(unsigned m, unsigned magic, int shift) {
#if defined(__HIP_DEVICE_COMPILE__)
    return (__umulhi(m, magic) + m) >> shift;
#else
    return ((unsigned)(((unsigned long long)m * magic) >> 32) + m) >> shift;
#endif
}

// Adjacent output pixels one thread of the blocked depth-wise kernel owns.
constexpr int kDwBlockPix = 4;      // measured 2, 4, 8: 8.5 / 7.2 / 6.9 us at stride 1 (16x56x56x128 fp16), 7.1 / 6.2 / 9.8 us at stride 2 (int8)

// Largest workgroup tile (rows x columns) whose reduction may be split over workgroups.
constexpr int kSplitMaxTile = 128 * 128;

// Number of XCDs (L2 domains) workgroups are dealt to round-robin by the dispatcher.
constexpr int kXcds = 8;
// Tile rows walked together before moving to the next tile column (L2 reuse of the B tile).
constexpr int kGroupM = 4;

// Map a linear workgroup id to an output tile.  Consecutive hardware ids land on different XCDs,
// so ids are first regrouped such that each XCD owns a contiguous run of logical tiles (its L2
// then sees few distinct A/B panels), and logical tiles walk kGroupM tile-rows at a time.
// The map is a bijection from [0, tiles_m*tiles_n) onto the tile grid.
// (gw_magic, gw_shift) = make_fastdiv(kGroupM * tiles_n).
__host__ __device__ inline void tile_of_block(int bid, int tiles_m, int tiles_n, unsigned gw_magic, int gw_shift, int* tm, int* tn) {
    int nb = tiles_m * tiles_n;
    int nb8 = nb - nb % kXcds;
    int logical = bid;
    if (bid < nb8) logical = (bid % kXcds) * (nb8 / kXcds) + bid / kXcds;
    int width = kGroupM * tiles_n;
    int group = (int)fastdiv((unsigned)logical, gw_magic, gw_shift);
    int first_m = group * kGroupM;
    int in_group = logical - group * width;
    // tile rows in this group: kGroupM, fewer in the last one; the division by 1 .. 4 as constants of fastdiv
    int gsz = tiles_m - first_m < kGroupM ? tiles_m - first_m : kGroupM;
    static_assert(kGroupM == 4, "the constants below are those of 1, 2, 3 and 4");
    unsigned g_magic = gsz == 3 ? 0x55555556u : (gsz == 1 ? 0u : 1u);
    int g_shift = gsz >= 3 ? 2 : gsz - 1;
    int q = (int)fastdiv((unsigned)in_group, g_magic, g_shift);
    *tm = first_m + in_group - q * gsz;
    *tn = q;
}

constexpr int const_gcd(int a, int b) { return b == 0 ? a : const_gcd(b, a % b); }
constexpr int elem_size(int dt) { return dt == DT_I8 ? 1 : (dt == DT_F16 || dt == DT_BF16) ? 2 : 4; }

// Compile-time shape of one kernel variant: BM x BN workgroup tile, WM x WN waves, ROWB bytes of k
// per LDS row and stage (128 or 64), NSTAGE LDS stages in the copy ring, KW reduction groups: KW
// sets of WM x WN waves share the output tile, group g reduces the stages s with s % KW == g through
// a ring of its own, and the partial sums are added through LDS before the store.  CW > 0 adds CW
// waves that do nothing but the global->LDS copy (the multiplying waves then issue none).
template <int DT_, int OUT_, int BM_, int BN_, int WM_, int WN_, int AMODE_, int BMODE_, int ROWB_ = 128, int NSTAGE_ = 2, int KW_ = 1, int CW_ = 0>
struct Cfg {
    static constexpr int DT = DT_, OUT = OUT_, BM = BM_, BN = BN_, WM = WM_, WN = WN_;
    static constexpr int AMODE = AMODE_, BMODE = BMODE_, ROWB = ROWB_, NSTAGE = NSTAGE_, KW = KW_, CW = CW_;
    static constexpr int SUB = WM * WN * 64;      // threads of one reduction group
    static constexpr int CT = CW ? CW * 64 : SUB; // threads that share the copy of a stage
    static constexpr int THREADS = SUB * KW + CW * 64;
    static constexpr int ES = elem_size(DT);
    static constexpr int VEC = 16 / ES;        // elements per 16-byte vector
    static constexpr int BK = ROWB / ES;       // elements of k per stage
    static constexpr int KSTEPS = ROWB / 32;   // MFMA k-steps per stage (each eats 32 bytes of k per row)
    static constexpr int RCH = ROWB / 16;      // 16-byte columns per K-major row
    static constexpr int TM = BM / WM, TN = BN / WN;
    static constexpr int MI = TM / 32, NI = TN / 32;
    // k-steps by which the LDS fragment reads run ahead of the MFMAs that use them: three where a k-step is one or two
    // MFMAs (shorter than an LDS round trip) and the ring has three slots or more, else one (with two slots the stage the
    // early barrier waits for is the one whose copy the iteration has just requested)
    static constexpr int LA = (MI * NI <= 2 && KSTEPS % 4 == 0 && NSTAGE >= 3) ? 3 : 1;
    static constexpr int A_BYTES = BM * ROWB, B_BYTES = BN * ROWB;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int RING_BYTES = NSTAGE * STAGE_BYTES;   // one reduction group's ring
    static constexpr int LDS_BYTES = KW * RING_BYTES;
    static constexpr int A_IT = BM * RCH / CT;    // 16-byte chunks per copying thread per stage
    static constexpr int B_IT = BN * RCH / CT;
    static constexpr int K_RSTEP = CT / RCH;          // K-major rows covered by one pass of the copying threads
    // N-major B tile in LDS: BK k-rows of BN*ES bytes
    static constexpr int BROW = BN * ES;
    static constexpr int B_RC = BROW / 16;          // 16-byte chunks per k-row
    static constexpr int SEG = (ES == 2) ? 64 : 32; // bytes one half-wave reads per k-row on the transposing read
    // A transposing read touches 256 / SEG consecutive k-rows at one SEG-byte segment each; they must fall into
    // different SEG-byte groups of the 256-byte bank sweep.  Row r starts in group r * (BROW / SEG) mod (256 / SEG):
    // that visits 256 / SEG / NSEG groups, with period RPW, where NSEG = gcd(BROW / SEG, 256 / SEG); XORing
    // (r / RPW) mod NSEG into the segment index spreads the rows over the rest.  (BROW a multiple of 256: all rows
    // start alike and the XOR does everything; BROW / SEG odd, e.g. 96 fp16 columns: the stride alone does.)
    static constexpr int SEGS_PER_SWEEP = 256 / SEG, SEGS_PER_ROW = BROW / SEG;
    static constexpr int NSEG = const_gcd(SEGS_PER_ROW, SEGS_PER_SWEEP);
    static constexpr int RPW = SEGS_PER_SWEEP / NSEG;
    static_assert(ROWB == 256 || ROWB == 128 || ROWB == 64, "");
    static_assert(TM % 32 == 0 && TN % 32 == 0, "wave tile must be a multiple of the 32x32 MFMA block");
    static_assert((BM * RCH) % CT == 0 && (BN * RCH) % CT == 0, "copy must divide evenly");
    static_assert(K_RSTEP % 16 == 0, "the K-major swizzle must repeat with the copy's row step");
    static_assert(BMODE != B_NMAJOR || (BROW % SEG == 0 && BROW % (NSEG * SEG) == 0), "N-major tile: whole segments, XOR closed inside a row");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of one CU");
    static_assert(KW >= 1 && KW <= 2 && THREADS <= 1024 && (CW == 0 || KW == 1), "");
    static_assert((KW - 1) * BM * BN * 4 <= LDS_BYTES, "the partial sums of the other groups must fit the rings");
};

}  // namespace tir
