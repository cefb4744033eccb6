// C-ABI entry points: argument validation, choice of kernel variant, launch.
// Everything a caller can get wrong is caught here, before any HIP call, so that a bad call
// never reaches a kernel.  See include/tir.h for the contract.
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <map>
#include <mutex>
#include <tuple>
#include <utility>
#include <vector>

#include "tir.h"
#include "tir_launch.h"
#include "tir_attention.h"
#include "tir_depthwise.h"

namespace tir {

// ------------------------------------------------------------------------------- MFMA rate probe
// Register-only MFMA loop: 4 waves per workgroup, 16 independent 32x32 accumulators per wave, no
// memory traffic inside the loop.  What it sustains is the practical ceiling of the matrix pipes at
// the clock the power management allows for the given operand statistics.
typedef _Float16 probe_f16x8 __attribute__((ext_vector_type(8)));
typedef float probe_f32x16 __attribute__((ext_vector_type(16)));

__global__ void __launch_bounds__(256) mfma_probe_kernel(float* sink, int iters, int random_operands) {
    probe_f32x16 acc[16];
    for (int i = 0; i < 16; ++i)
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    probe_f16x8 a, b;
    unsigned x = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    for (int e = 0; e < 8; ++e) {
        x ^= x >> 15; x *= 2246822519u; x ^= x >> 13;
        a[e] = (_Float16)(random_operands ? ((x & 0xffff) / 32768.0f - 1.0f) : 1.0f);
        x *= 3266489917u; x ^= x >> 16;
        b[e] = (_Float16)(random_operands ? ((x & 0xffff) / 32768.0f - 1.0f) : 0.5f);
    }
    // Shader-clock counter and 100 MHz wall counter before and after the loop, as one wave in the middle of the grid sees
    // them (raw low words, stored right away so that nothing stays live across the loop): cycles / time is the clock the
    // power management held during the loop.
    const bool reporter = blockIdx.x == gridDim.x / 2 && threadIdx.x == 0;
    unsigned* const stamps = (unsigned*)sink;
    if (reporter) {
        stamps[1] = (unsigned)__builtin_amdgcn_s_memtime();
        stamps[2] = (unsigned)__builtin_amdgcn_s_memrealtime();
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < 16; ++i)
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    if (s == 123.456f) sink[0] = s;      // keeps the loop alive, practically never stores
    if (reporter) {
        stamps[3] = (unsigned)__builtin_amdgcn_s_memtime();
        stamps[4] = (unsigned)__builtin_amdgcn_s_memrealtime();
    }
}

// ------------------------------------------------------------------------------- variant table
#define TIR_ROW(name, DT, OUT, BM, BN, WM, WN, AM, BMO, RB, NS, KW, CW) \
    {name, DT, OUT, BM, BN, WM, WN, AM, BMO, RB, NS, KW, CW, &launch_cfg<Cfg<DT, OUT, BM, BN, WM, WN, AM, BMO, RB, NS, KW, CW>>},
#define V0 TIR_ROW
#define V1 TIR_ROW
#define V2 TIR_ROW
#define V3 TIR_ROW
#define V4 TIR_ROW
#define V5 TIR_ROW
static const Variant kVariants[] = {
#include "tir_variants.def"
};
static const int kNumVariants = (int)(sizeof(kVariants) / sizeof(kVariants[0]));

// The depth-wise kernel is not a tile variant: one entry per dtype pair, filled on first use.
static const Variant* depthwise_variant(int dt, int out) {
    static Variant table[6] = {
        {"f16_f16_depthwise", DT_F16, DT_F16, 0, 0, 0, 0, A_DEPTHWISE, B_GENERIC, 0, 0, 1, 0, nullptr},
        {"f16_f32_depthwise", DT_F16, DT_F32, 0, 0, 0, 0, A_DEPTHWISE, B_GENERIC, 0, 0, 1, 0, nullptr},
        {"bf16_bf16_depthwise", DT_BF16, DT_BF16, 0, 0, 0, 0, A_DEPTHWISE, B_GENERIC, 0, 0, 1, 0, nullptr},
        {"bf16_f32_depthwise", DT_BF16, DT_F32, 0, 0, 0, 0, A_DEPTHWISE, B_GENERIC, 0, 0, 1, 0, nullptr},
        {"i8_i32_depthwise", DT_I8, DT_I32, 0, 0, 0, 0, A_DEPTHWISE, B_GENERIC, 0, 0, 1, 0, nullptr},
        {"i8_i8_depthwise", DT_I8, DT_I8, 0, 0, 0, 0, A_DEPTHWISE, B_GENERIC, 0, 0, 1, 0, nullptr},
    };
    for (Variant& v : table)
        if (v.dt == dt && v.out == out) {
            if (!v.fn) v.fn = depthwise_launcher(dt, out);      // idempotent: racing threads store the same pointer
            return v.fn ? &v : nullptr;
        }
    return nullptr;
}

static thread_local char g_err[512] = "";
static int g_force_bm = 0, g_force_bn = 0, g_force_ksplit = 0;
static char g_force_name[64] = "";

static tir_status fail(tir_status st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}

static const int64_t kMaxExtent = 2147483647LL;
static const double kCUs = 256.0;

static bool dtype_pair_ok(int in, int out, bool fused) {
    return (in == TIR_F16 && (out == TIR_F32 || out == TIR_F16)) ||
           (in == TIR_BF16 && (out == TIR_F32 || out == TIR_BF16)) || (in == TIR_I8 && out == TIR_I32) ||
           (fused && in == TIR_I8 && out == TIR_I8);
}

// The epilogue variant queries assume for int8 output.
static const tir_epilogue kQueryRequant = {nullptr, 0, 1.0f};

static bool aligned(const void* p, uintptr_t a) { return ((uintptr_t)p % a) == 0; }

// Do byte offsets inside one tile of at most 256 rows of `stride` elements (the last one `width` elements wide) fit
// 31 bits?  (stride * 256 + width) * es < 2^31 - 1, written so that no product can overflow for strides up to 2^63.
static bool fits_tile_offsets(int64_t stride, int64_t width, int64_t es) {
    const int64_t room = kMaxExtent / es - width;
    return room > 0 && stride < (room + 255) / 256 && (stride * 256 + width) * es < kMaxExtent;
}

// ------------------------------------------------------------------------------- measured choices
// Records of tir_tune_*: for a problem signature, the variant that ran fastest on this device.
// kind 0 = (batched) GEMM, 1 = convolution; geom packs the convolution geometry that the GEMM view
// (batch, M, N, K) does not show.  A record only ever names a variant that computes the same result.
struct TuneKey {
    int kind, dt, out, amode, bmode;
    int64_t batch, M, N, K;
    uint64_t geom;
    bool operator<(const TuneKey& o) const {
        return std::tie(kind, dt, out, amode, bmode, batch, M, N, K, geom) <
               std::tie(o.kind, o.dt, o.out, o.amode, o.bmode, o.batch, o.M, o.N, o.K, o.geom);
    }
};
// A kernel variant plus the number of workgroups that share one tile's reduction (1 = no split).
struct Choice {
    const Variant* v;
    int ksplit;
};
static const Choice kNoChoice = {nullptr, 1};
static std::mutex g_tune_mu;
static std::map<TuneKey, Choice> g_tuned;
// set by the tuner around its trial launches on the calling thread: the choice to plan with
static thread_local Choice g_trial = {nullptr, 1};

static Choice tuned_lookup(const TuneKey& k) {
    std::lock_guard<std::mutex> lock(g_tune_mu);
    auto it = g_tuned.find(k);
    return it == g_tuned.end() ? kNoChoice : it->second;
}

// ------------------------------------------------------------------------------- split reduction
// Scratch of the reduction split over workgroups: the slices' partial sums and one arrival counter per output
// tile.  The library owns no such memory: a caller registers a buffer per (device, stream) with tir_set_workspace
// (launches on one stream follow each other, so they can share it; launches on different streams may overlap and
// need their own), or calls tir_gemm_split_static, whose scratch is a static device array.
static const int64_t kWsBytes = 32ll << 20;      // partial sums of a registered workspace
static const int64_t kWsTiles = 16384;           // ... and its counters
struct Workspace {
    void* partial;
    unsigned* count;
};
static std::mutex g_ws_mu;
static std::map<std::pair<int, hipStream_t>, Workspace> g_ws;

// What a plan may use for split reductions: room for partial sums and counters (bytes = 0: none, never split),
// and the slice count a caller insists on (force > 1: only variants that can split that way are considered,
// measured records and the scoring rule's own idea of a split are ignored).
struct SplitLimits {
    int64_t bytes, tiles;
    int force;
};
static const SplitLimits kNoSplit = {0, 0, 0};
static const SplitLimits kRegisteredSplit = {kWsBytes, kWsTiles, 0};      // a registered workspace (also what the variant queries assume)

// Arrival counters start at zero; every launch leaves them at zero again (the last workgroup of a tile resets its counter).
__global__ void __launch_bounds__(256) clear_counters_kernel(unsigned* count, int n) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) count[i] = 0;
}

// Can variant v reduce a problem of `tiles` output tiles per batch entry in ks slices?
static bool split_fits(const Variant* v, int ks, int64_t batch, int64_t tiles, int64_t K, const SplitLimits& sl) {
    if (ks == 1) return true;
    if (ks < 1 || ks > 64 || sl.bytes <= 0) return false;
    if (v->amode != A_KMAJOR && v->amode != A_CONV && v->amode != A_CONVX) return false;      // the fast kernel only
    if (v->bm * v->bn > kSplitMaxTile) return false;
    const int64_t stages = (K * elem_size(v->dt) + v->rowb - 1) / v->rowb;
    const int64_t per = (stages + ks - 1) / ks;
    if ((ks - 1) * per >= stages) return false;       // a slice would be empty
    if (batch > 65535 || batch * tiles > sl.tiles) return false;
    return batch * tiles * ks * v->bm * v->bn * 4 <= sl.bytes;
}

// The split a launch on `stream` of the current device may use: that of its registered workspace, or none.
static SplitLimits stream_split_limits(hipStream_t stream) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return kNoSplit;
    }
    std::lock_guard<std::mutex> lock(g_ws_mu);
    return g_ws.count(std::make_pair(dev, stream)) ? kRegisteredSplit : kNoSplit;
}

// The kernels divide by these launch constants through multiply-and-shift (see Params).
static void set_divisors(Params& p) {
    auto put = [](unsigned d, unsigned* magic, int* shift) {
        const FastDiv f = make_fastdiv(d < 1 ? 1u : d);
        *magic = f.magic;
        *shift = f.shift;
    };
    put((unsigned)(kGroupM * p.tiles_n), &p.div_gw_magic, &p.div_gw_shift);
    put((unsigned)p.tiles_n, &p.div_tn_magic, &p.div_tn_shift);
    put((unsigned)p.tiles_m, &p.div_tm_magic, &p.div_tm_shift);
    put((unsigned)(p.PW / 8), &p.div_pw_magic, &p.div_pw_shift);      // copy units (8 pixels) per patch row
    put((unsigned)p.Q, &p.div_q_magic, &p.div_q_shift);
    put((unsigned)(p.P * p.Q), &p.div_pq_magic, &p.div_pq_shift);
    put((unsigned)(p.OD < 1 ? 1 : p.OD) * (unsigned)(p.P * p.Q), &p.div_opq_magic, &p.div_opq_shift);
    put((unsigned)p.Cg, &p.div_cg_magic, &p.div_cg_shift);
    put((unsigned)p.S, &p.div_s_magic, &p.div_s_shift);
    put((unsigned)(p.R * p.S), &p.div_rs_magic, &p.div_rs_shift);
    put((unsigned)p.conv_groups, &p.div_grp_magic, &p.div_grp_shift);
    put((unsigned)p.phases_h, &p.div_phh_magic, &p.div_phh_shift);
    put((unsigned)p.phases_w, &p.div_phw_magic, &p.div_phw_shift);
    const unsigned qg = (unsigned)((p.Q + kDwBlockPix - 1) / kDwBlockPix);
    put(qg, &p.div_dwq_magic, &p.div_dwq_shift);
    put((unsigned)p.P * qg, &p.div_dwpq_magic, &p.div_dwpq_shift);
}

static uint64_t hash_fields(const int64_t* f, int n) {
    // the fields of a convolution's geometry do not fit 64 bits side by side: mix them instead (FNV-1a)
    uint64_t h = 1469598103934665603ull;
    for (int i = 0; i < n; ++i)
        for (int b = 0; b < 8; ++b) { h ^= (uint64_t)((f[i] >> (8 * b)) & 0xff); h *= 1099511628211ull; }
    return h;
}

// Pick a variant for (dt, out, amode, bmode).  This is the hand-made stand-in for the paper's
// search over tilings (sec. 4.4): every listed tile is scored by
//   padding efficiency  x  how evenly its workgroups fill the 256 CUs  x  bytes-per-flop factor,
// where the last term favours tiles that need fewer global->LDS bytes per MFMA (bm*bn/(bm+bn),
// saturating at the 256x256 tile).  Among equal tiles the ring depth is chosen by occupancy:
// deep rings when one workgroup per CU must hide the global latency alone, shallow ones when
// several workgroups share a CU (their LDS must fit side by side) or the reduction is short.
//
// A reduction much longer than the tile grid is wide (few small tiles, many stages) is split over several
// workgroups per tile, as many as fill the CUs once while each keeps at least eight stages.
static Choice pick(int dt, int out, int amode, int bmode, int64_t batch, int64_t M, int64_t N, int64_t K, const SplitLimits& sl, int max_rowb = 256) {
    Choice best = kNoChoice;
    double best_score = -1.0;
    const int es = elem_size(dt);
    for (int i = 0; i < kNumVariants; ++i) {
        const Variant* v = &kVariants[i];
        if (v->dt != dt || v->out != out || v->amode != amode || v->bmode != bmode || v->rowb > max_rowb) continue;
        const int64_t tiles_1 = ((M + v->bm - 1) / v->bm) * ((N + v->bn - 1) / v->bn);
        const int want_ks = sl.force > 1 ? sl.force : g_force_ksplit;
        const int forced_ks = (want_ks > 1 && split_fits(v, want_ks, batch, tiles_1, K, sl)) ? want_ks : 1;
        if (sl.force > 1 && forced_ks != sl.force) continue;          // the caller insists on this split
        if (g_force_name[0] && strstr(v->name, g_force_name)) return Choice{v, forced_ks};          // testing / tuning overrides
        if (g_force_bm && v->bm == g_force_bm && v->bn == g_force_bn && v->kw == 1 && v->cw == 0) return Choice{v, forced_ks};
        const double tm = (double)((M + v->bm - 1) / v->bm), tn = (double)((N + v->bn - 1) / v->bn);
        int ks = forced_ks;
        // (the partial sums' trip through memory costs about 4 us for a 64x64 tile and grows with the tile: it pays
        // only for small tiles whose wave groups face two dozen stages or more)
        if (!want_ks && sl.bytes > 0 && v->bm * v->bn <= 64 * 64) {
            const int64_t stages = (K * es + v->rowb - 1) / v->rowb;
            int64_t want = stages / v->kw >= 24 ? (int64_t)kCUs / (tiles_1 * batch) : 1;
            if (want > stages / (8 * v->kw)) want = stages / (8 * v->kw);
            if (want > 8) want = 8;
            while (want > 1 && !split_fits(v, (int)want, batch, tiles_1, K, sl)) --want;
            if (want > 1) ks = (int)want;
        }
        const double tiles = tm * tn * (double)batch * ks;
        const double eff = ((double)M * (double)N) / (tm * v->bm * tn * v->bn);
        const double rounds = tiles <= kCUs ? 1.0 : (double)((int64_t)(tiles + kCUs - 1) / kCUs);
        const double fill = tiles / (rounds * kCUs);
        double intensity = (double)v->bm * v->bn / (double)(v->bm + v->bn) / 128.0;
        if (intensity > 1.0) intensity = 1.0;
        double score = eff * fill * (0.25 + 0.75 * intensity);
        // ring depth: stages beyond the number of K-slabs are useless; with more than one
        // workgroup per CU prefer rings that let two of them be resident (LDS <= 80 KB)
        const int64_t nslab = (K * es + v->rowb - 1) / v->rowb;
        const int lds = (v->bm + v->bn) * v->rowb * v->nstage * v->kw;
        double depth = 1.0;
        if (v->kw > 1) {
            // two reduction groups pay for the exchange of partial sums: only for small tiles in a single
            // round of workgroups (nothing else on the CU hides the copy latency) facing a long reduction
            if (tiles > kCUs || nslab < 4 * v->kw || v->bm * v->bn > 64 * 64) continue;
            depth += 0.05;
        }
        // copy waves pay off once a stage is worth the extra waves: measured -8 .. -17 % on 128x128 and larger
        // tiles of mid-size GEMMs, a loss on the narrow ones
        // (and -13 % on a 64x64-tile convolution with 18 stages once the stages are 256 bytes)
        if (v->cw) depth += ((v->bm * v->bn >= 128 * 128 && nslab >= 8) ? 0.04 : (v->rowb == 256 && tiles <= kCUs && nslab >= 8) ? 0.07 : -0.04);
        else if (v->rowb == 256) depth -= 0.04;
        if (nslab < v->nstage) depth -= 0.02 * (v->nstage - (int)nslab);
        if (tiles > kCUs && lds > 80 * 1024) depth -= 0.03;
        else if (tiles <= kCUs) depth += 0.01 * v->nstage;
        else depth += 0.005 * v->nstage;
        score *= depth * (1.0 - 0.03 * (ks - 1));       // the partial sums' round trip
        if (score > best_score) { best_score = score; best = Choice{v, ks}; }
    }
    return best;
}

// by phase, a stage must hold channels of one tap
static bool tuned_or_trial_mismatch(const Variant* v, int64_t group_channel_bytes) {
    return v->amode == A_CONV && group_channel_bytes % v->rowb != 0 && !g_trial.v;
}

struct Plan {
    const Variant* v;
    Params p;
    TuneKey key;        // signature of the problem for the measured-choice records
    bool patch_ok;      // convolution: the LDS-resident-patch kernel may run this problem
};

// The variant a plan uses: the tuner's trial variant, else a measured record, else the scoring rule.
static Choice choose(const TuneKey& key, int64_t batch, int64_t M, int64_t N, int64_t K, const SplitLimits& sl) {
    if (sl.force > 1) return pick(key.dt, key.out, key.amode, key.bmode, batch, M, N, K, sl);
    if (g_trial.v) return g_trial;
    if (!g_force_name[0] && !g_force_bm && !g_force_ksplit) {
        const Choice t = tuned_lookup(key);
        if (t.v) return t;
    }
    return pick(key.dt, key.out, key.amode, key.bmode, batch, M, N, K, sl);
}

static tir_status check_common(const void* A, const void* B, const void* C, int in, int out, const tir_epilogue* ep) {
    if (in < 0 || in > TIR_I32 || out < 0 || out > TIR_I32) return fail(TIR_ERR_INVALID_ARG, "unknown dtype code (in=%d out=%d)", in, out);
    if (!dtype_pair_ok(in, out, ep != nullptr)) return fail(TIR_ERR_UNSUPPORTED, "unsupported (in, out) dtype pair (%d, %d)", in, out);
    if (ep) {
        if (ep->streaming != 0 && ep->streaming != 1) return fail(TIR_ERR_INVALID_ARG, "epilogue: streaming must be 0 or 1 (got %d)", ep->streaming);
        if (!aligned(ep->bias, 4)) return fail(TIR_ERR_ALIGNMENT, "bias pointer not aligned to 4 bytes");
        if (out == TIR_I8 && !(ep->scale > 0.0f && ep->scale <= 3.402823466e38f))
            return fail(TIR_ERR_INVALID_ARG, "int8 output needs a finite scale > 0");
    }
    const int es = elem_size(in), os = elem_size(out);
    if (!aligned(A, es) || !aligned(B, es)) return fail(TIR_ERR_ALIGNMENT, "input pointer not aligned to its element size");
    if (!aligned(C, os)) return fail(TIR_ERR_ALIGNMENT, "output pointer not aligned to its element size");
    return TIR_OK;
}

// Build the launch plan of a (batched) GEMM.  Pointers may be null only for planning (variant query).
static tir_status plan_gemm(bool need_ptrs, const void* A, const void* B, void* C, int64_t batch, int64_t M, int64_t N,
                            int64_t K, int64_t a_bs, int64_t a_rs, int64_t a_cs, int64_t b_bs, int64_t b_rs,
                            int64_t b_cs, int64_t c_bs, int64_t c_rs, int64_t c_cs, int in, int out, const tir_epilogue* ep,
                            const SplitLimits& sl, Plan* plan) {
    plan->v = nullptr;
    plan->key.kind = -1;        // no signature yet
    tir_status st = check_common(A, B, C, in, out, ep);
    if (st != TIR_OK) return st;
    if (batch < 0 || M < 0 || N < 0 || K < 0) return fail(TIR_ERR_INVALID_ARG, "negative extent (batch=%lld M=%lld N=%lld K=%lld)", (long long)batch, (long long)M, (long long)N, (long long)K);
    if (a_bs < 0 || a_rs < 0 || a_cs < 0 || b_bs < 0 || b_rs < 0 || b_cs < 0 || c_bs < 0 || c_rs < 0 || c_cs < 0)
        return fail(TIR_ERR_INVALID_ARG, "negative stride");
    if (M > kMaxExtent || N > kMaxExtent || K > kMaxExtent || batch > kMaxExtent)
        return fail(TIR_ERR_UNSUPPORTED, "extent beyond 2^31-1");
    if (batch == 0 || M == 0 || N == 0) return TIR_OK;  // nothing to do, plan->v stays null
    if (need_ptrs) {
        if (!C) return fail(TIR_ERR_INVALID_ARG, "C is null");
        if (K > 0 && (!A || !B)) return fail(TIR_ERR_INVALID_ARG, "A or B is null");
    }
    if (M > 1 && N > 1 && c_rs == 0 && c_cs == 0) return fail(TIR_ERR_INVALID_ARG, "C strides are both zero");
    if (batch > 1 && c_bs == 0) return fail(TIR_ERR_INVALID_ARG, "c_bs is zero: the C matrices of different batches overlap");

    const int es = elem_size(in);
    const int vec = 16 / es;
    const bool k_vec = K % vec == 0;
    int amode = A_GENERIC, bmode = B_GENERIC;
    // fast copy modes need 16-byte vectors along the contiguous axis
    // (rows must not overlap: the copy stage relies on "row r+1 starts after row r ends" to turn
    // rows past the edge into out-of-range reads; byte offsets inside one tile must fit 31 bits)
    if (a_cs == 1 && k_vec && a_rs % vec == 0 && a_bs % vec == 0 && aligned(A, 16) && (a_rs >= K || M == 1) &&
        fits_tile_offsets(a_rs, K, es)) amode = A_KMAJOR;
    if (b_rs == 1 && k_vec && b_cs % vec == 0 && b_bs % vec == 0 && aligned(B, 16) && (b_cs >= K || N == 1) &&
        fits_tile_offsets(b_cs, K, es)) bmode = B_KMAJOR;
    else if (b_cs == 1 && N % vec == 0 && b_rs % vec == 0 && b_bs % vec == 0 && aligned(B, 16) && b_rs >= N &&
             fits_tile_offsets(b_rs, N, es)) bmode = B_NMAJOR;
    if (amode == A_GENERIC || bmode == B_GENERIC) { amode = A_GENERIC; bmode = B_GENERIC; }

    plan->key = TuneKey{0, in, out, amode, bmode, batch, M, N, K, 0};
    plan->patch_ok = false;
    const Choice ch = choose(plan->key, batch, M, N, K, sl);
    const Variant* v = ch.v;
    if (!v) return fail(TIR_ERR_UNSUPPORTED, "no kernel variant for this dtype / layout / forced tile");
    Params& p = plan->p;
    memset(&p, 0, sizeof p);
    p.ksplit = split_fits(v, ch.ksplit, batch, ((M + v->bm - 1) / v->bm) * ((N + v->bn - 1) / v->bn), K, sl) ? ch.ksplit : 1;
    p.A = A; p.B = B; p.C = C;
    p.M = (int)M; p.N = (int)N; p.K = (int)K;
    p.batch = (int)batch;
    p.tiles_m = (int)((M + v->bm - 1) / v->bm);
    p.tiles_n = (int)((N + v->bn - 1) / v->bn);
    if ((int64_t)p.tiles_m * p.tiles_n > kMaxExtent) return fail(TIR_ERR_UNSUPPORTED, "too many output tiles");
    p.a_bs = a_bs; p.b_bs = b_bs; p.c_bs = c_bs;
    p.a_rs = a_rs; p.a_cs = a_cs; p.b_rs = b_rs; p.b_cs = b_cs; p.c_rs = c_rs; p.c_cs = c_cs;
    p.c_fast = (c_cs == 1 && (c_rs >= N || M == 1) && fits_tile_offsets(c_rs, N, elem_size(out))) ? 1 : 0;
    if (ep) { p.bias = ep->bias; p.bias_bs = 0; p.relu = ep->relu != 0; p.scale = ep->scale; p.store_nt = ep->streaming; }
    set_divisors(p);
    plan->v = v;
    return TIR_OK;
}

static int64_t conv_extent(int64_t in, int64_t filt, int64_t stride, int64_t pad, int64_t dil) {
    int64_t span = in + 2 * pad - dil * (filt - 1) - 1;
    return span < 0 ? 0 : span / stride + 1;
}

// Geometry of a convolution in the general form the kernels decode: a depth axis (D = T = 1 for 1-D / 2-D) and the
// transposed 2-D form (the adjoint of a strided convolution).
struct ConvGeom {
    int64_t N, D, H, W, C, K, T, R, S;
    int stride_d, stride_h, stride_w, pad_d, pad_h, pad_w, dil_d, dil_h, dil_w;
    int groups;
    bool transposed;
    int outpad_h, outpad_w;      // transposed only
};

static tir_status plan_conv_geom(bool need_ptrs, const void* x, const void* w, void* y, const ConvGeom& g, int in, int out,
                                 const tir_epilogue* ep, const SplitLimits& sl, Plan* plan) {
    plan->v = nullptr;
    tir_status st = check_common(x, w, y, in, out, ep);
    if (st != TIR_OK) return st;
    const int64_t N = g.N, D = g.D, H = g.H, W = g.W, C = g.C, K = g.K, T = g.T, R = g.R, S = g.S;
    const int groups = g.groups;
    if (N < 0 || D <= 0 || H <= 0 || W <= 0 || C <= 0 || K <= 0 || T <= 0 || R <= 0 || S <= 0)
        return fail(TIR_ERR_INVALID_ARG, "non-positive extent (N=%lld D=%lld H=%lld W=%lld C=%lld K=%lld T=%lld R=%lld S=%lld)", (long long)N, (long long)D, (long long)H, (long long)W, (long long)C, (long long)K, (long long)T, (long long)R, (long long)S);
    if (g.stride_d <= 0 || g.stride_h <= 0 || g.stride_w <= 0 || g.dil_d <= 0 || g.dil_h <= 0 || g.dil_w <= 0 || g.pad_d < 0 || g.pad_h < 0 || g.pad_w < 0)
        return fail(TIR_ERR_INVALID_ARG, "stride and dilation must be positive, padding non-negative");
    if (g.transposed && (g.outpad_h < 0 || g.outpad_w < 0)) return fail(TIR_ERR_INVALID_ARG, "output padding must be non-negative");
    if (g.transposed && (g.stride_h > 16383 || g.stride_w > 16383)) return fail(TIR_ERR_UNSUPPORTED, "transposed convolution: stride beyond 16383");
    if (groups <= 0 || C % groups != 0 || K % groups != 0)
        return fail(TIR_ERR_INVALID_ARG, "groups=%d must divide C=%lld and K=%lld", groups, (long long)C, (long long)K);
    int64_t OD = 1, P, Q;
    if (g.transposed) {
        // extent of the adjoint: (in - 1) * stride - 2 * pad + dil * (filt - 1) + outpad + 1
        P = (H - 1) * g.stride_h - 2 * g.pad_h + (int64_t)g.dil_h * (R - 1) + g.outpad_h + 1;
        Q = (W - 1) * g.stride_w - 2 * g.pad_w + (int64_t)g.dil_w * (S - 1) + g.outpad_w + 1;
    } else {
        OD = conv_extent(D, T, g.stride_d, g.pad_d, g.dil_d);
        P = conv_extent(H, R, g.stride_h, g.pad_h, g.dil_h);
        Q = conv_extent(W, S, g.stride_w, g.pad_w, g.dil_w);
    }
    if (OD <= 0 || P <= 0 || Q <= 0) return fail(TIR_ERR_INVALID_ARG, "empty output: the dilated filter does not fit the padded input");
    // the kernels keep input coordinates in 16 bits and element offsets in 32 bits
    if (D > 16383 || H > 16383 || W > 16383 || g.pad_d > 8191 || g.pad_h > 8191 || g.pad_w > 8191 || (T - 1) * g.dil_d > 8191 ||
        (R - 1) * g.dil_h > 8191 || (S - 1) * g.dil_w > 8191 || P + g.pad_h > 32000 || Q + g.pad_w > 32000)
        return fail(TIR_ERR_UNSUPPORTED, "spatial extent, padding or dilated filter span too large");
    const int64_t Cg = C / groups, Kg = K / groups;
    const int64_t Mg = N * OD * P * Q, Kd = T * R * S * Cg;
    if (N * D * H * W * C > kMaxExtent || Mg > kMaxExtent || Kd > kMaxExtent || Mg * K > (int64_t)1 << 40)
        return fail(TIR_ERR_UNSUPPORTED, "tensor too large for 32-bit element offsets");
    if (N == 0) return TIR_OK;
    if (need_ptrs && (!x || !w || !y)) return fail(TIR_ERR_INVALID_ARG, "x, w or y is null");

    const int es = elem_size(in);
    const int vec = 16 / es;
    const bool plain2d = !g.transposed && D == 1 && T == 1;      // the 2-D kernels (scalar tap cursor, LDS-resident patch) apply
    int amode = A_CONV_GENERIC, bmode = B_GENERIC;
    if (Cg % vec == 0 && aligned(x, 16) && aligned(w, 16) && N * D * H * W * C * es < kMaxExtent && (Kd * 256 + Kd) * es < kMaxExtent) {
        amode = plain2d ? A_CONV : A_CONVX;
        bmode = B_KMAJOR;
    }
    // A strided transposed convolution multiplies mostly structural zeros when read as one gather (only every
    // stride-th tap meets an input pixel).  Undilated, with whole stages per tap (one stage = 128 bytes of channels),
    // it is computed per output phase instead: stride_h*stride_w stride-1 convolutions with a tap subset each, all
    // in one launch of the 2-D kernels (a forced general-decode variant keeps the gather).
    const int64_t phases = (int64_t)g.stride_h * g.stride_w;
    const int64_t Pp = (P + g.stride_h - 1) / g.stride_h, Qp = (Q + g.stride_w - 1) / g.stride_w;      // pixel grid of one phase
    const bool phased = g.transposed && amode == A_CONVX && phases > 1 && g.dil_h == 1 && g.dil_w == 1 && (Cg * es) % 128 == 0 &&
                        groups * phases <= 65535 && N * P * Q * K * elem_size(out) < kMaxExtent && N * Pp * Qp <= kMaxExtent &&
                        !(g_force_name[0] && (strstr(g_force_name, "convx") || strstr(g_force_name, "generic")));
    if (phased) amode = A_CONV;
    // LDS-resident input patch: one pixel of one group is exactly one 128-byte LDS row, the input rows
    // that 256 consecutive output pixels touch (rows padded to 8 pixels, copied in passes of 32) fit beside the R*S filter slabs
    const int64_t span_out = (255 + Q - 1) / Q < P - 1 ? (255 + Q - 1) / Q : P - 1;   // output rows a tile can span, minus one
    const int64_t span_rows = span_out * g.stride_h + (R - 1) * g.dil_h + 1;
    const int64_t patch_w = ((Q - 1) * g.stride_w + (S - 1) * g.dil_w + 1 + 7) / 8 * 8;      // patch rows are copied in units of 8 pixels
    const bool patch_ok = amode == A_CONV && !phased && Cg * es == 128 && P * Q >= 128 && (span_rows * patch_w + 31) / 32 * 4096 + R * S * 8192 <= 160 * 1024 &&
                          (K * 256 + Kg) * elem_size(out) < kMaxExtent;
    plan->patch_ok = patch_ok;
    // records are kept under the implicit-GEMM signature; a record (or a trial) may name either kernel family
    const int64_t geom[21] = {N, groups, D, H, W, T, R, S, g.stride_d, g.stride_h, g.stride_w, g.pad_d, g.pad_h, g.pad_w, g.dil_d, g.dil_h, g.dil_w,
                              g.transposed ? 1 : 0, g.transposed ? g.outpad_h : 0, g.transposed ? g.outpad_w : 0, 0};
    plan->key = TuneKey{1, in, out, amode, bmode, groups * N, OD * P * Q, Kg, Kd, hash_fields(geom, 21)};
    // the tile grid the variants are scored on: by phase, every phase is a batch entry of its own with a share of the taps
    const int64_t sc_batch = phased ? groups * phases : groups, sc_M = phased ? N * Pp * Qp : Mg, sc_K = phased ? (Kd + phases - 1) / phases : Kd;
    Choice ch = kNoChoice;
    // depth-wise (one input and one output channel per group): the direct kernel, unless a test forces a tile variant
    if (plain2d && Cg == 1 && Kg == 1 && C % vec == 0 && R * S <= kDwMaxTaps && aligned(x, 16) && aligned(w, 16) && aligned(y, 16) &&
        N * H * W * C * es < kMaxExtent && Mg * K * elem_size(out) < kMaxExtent && !g_trial.v &&
        !g_force_name[0] && !g_force_bm)
        ch.v = depthwise_variant(in, out);
    const bool depthwise = ch.v != nullptr;
    if (depthwise) amode = A_DEPTHWISE;
    else if (g_trial.v) ch = g_trial;
    else if (!g_force_name[0] && !g_force_bm && !g_force_ksplit) ch = tuned_lookup(plan->key);
    if (ch.v && ch.v->amode == A_CONV_PATCH && !patch_ok) ch = kNoChoice;
    if (!ch.v) {
        const bool use_patch = patch_ok && !g_force_ksplit && (!g_force_name[0] || strstr(g_force_name, "patch"));
        if (use_patch) ch = pick(in, out, A_CONV_PATCH, bmode, groups * N, P * Q, Kg, Kd, sl);
        else ch = pick(in, out, amode, bmode, sc_batch, sc_M, Kg, sc_K, sl, phased ? (int)(Cg * es >= 256 && (Cg * es) % 256 == 0 ? 256 : 128) : 256);
    }
    if (phased && ch.v && tuned_or_trial_mismatch(ch.v, Cg * es)) ch = pick(in, out, amode, bmode, sc_batch, sc_M, Kg, sc_K, sl, 128);
    const Variant* v = ch.v;
    if (v && v->amode == A_CONV_PATCH) amode = A_CONV_PATCH;
    if (!v) return fail(TIR_ERR_UNSUPPORTED, "no kernel variant for this dtype / forced tile");
    Params& p = plan->p;
    memset(&p, 0, sizeof p);
    p.ksplit = (!depthwise && !phased && split_fits(v, ch.ksplit, groups, ((Mg + v->bm - 1) / v->bm) * ((Kg + v->bn - 1) / v->bn), Kd, sl)) ? ch.ksplit : 1;
    p.A = x; p.B = w; p.C = y;
    p.M = (int)Mg; p.N = (int)Kg; p.K = (int)Kd;
    p.batch = depthwise ? 1 : groups;                 // the depth-wise kernel covers every channel in one launch
    p.tiles_m = depthwise ? 1 : (int)((Mg + v->bm - 1) / v->bm);
    p.tiles_n = depthwise ? 1 : (int)((Kg + v->bn - 1) / v->bn);
    if (amode == A_CONV_PATCH) {
        p.tiles_m = (int)((P * Q + 255) / 256);      // pixel tiles per image
        p.PW = (int)patch_w;
        for (int t = 0; t < 9; ++t) {
            const int64_t tt = t < R * S ? t : R * S - 1;
            p.tap_px[t] = R * S <= 9 ? (int)((tt / S) * g.dil_h * patch_w + (tt % S) * g.dil_w) : 0;
        }
    }
    p.batch_imgs = (int)N;
    p.a_bs = Cg;            // a group starts Cg channels further
    p.b_bs = Kg * Kd;       // filters of one group are contiguous
    p.c_bs = Kg;
    p.a_rs = 0; p.a_cs = 1;
    p.b_rs = 1; p.b_cs = Kd;          // B[k][y] = w[y][k]: the filter (output channel major, channel innermost) is B stored K-major
    p.c_rs = K; p.c_cs = 1;           // the channels-last output is C_t[fuse(n,o,h,w)][co]
    p.c_fast = ((K * 256 + Kg) * elem_size(out) < kMaxExtent) ? 1 : 0;
    if (ep) { p.bias = ep->bias; p.bias_bs = Kg; p.relu = ep->relu != 0; p.scale = ep->scale; p.store_nt = ep->streaming; }
    p.H = (int)H; p.W = (int)W; p.Cin = (int)C; p.Cg = (int)Cg; p.P = (int)P; p.Q = (int)Q; p.R = (int)R; p.S = (int)S;
    p.D = (int)D; p.T = (int)T; p.OD = (int)OD;
    p.stride_d = g.stride_d; p.pad_d = g.pad_d; p.dil_d = g.dil_d;
    p.dil_h = g.dil_h; p.dil_w = g.dil_w;
    if (phased) {
        if (v->amode != A_CONV || (Cg * es) % v->rowb != 0)
            return fail(TIR_ERR_UNSUPPORTED, "transposed convolution by phase needs a 2-D implicit-GEMM variant whose stages hold one tap (got %s)", v->name);
        p.M = (int)(N * Pp * Qp);
        p.batch = (int)(groups * phases);
        p.tiles_m = (int)((p.M + v->bm - 1) / v->bm);
        p.P = (int)Pp; p.Q = (int)Qp; p.P_full = (int)P; p.Q_full = (int)Q;
        p.phases_h = g.stride_h; p.phases_w = g.stride_w; p.t_pad_h = g.pad_h; p.t_pad_w = g.pad_w;
        p.conv_groups = groups;
        p.stride_h = 1; p.stride_w = 1; p.pad_h = 0; p.pad_w = 0;      // per phase, derived by the kernel
        p.tap_sign = 1; p.up_h = 1; p.up_w = 1;
    } else if (g.transposed) {
        // gather form of the adjoint: output pixel oh reads input (oh + pad - r*dil) / stride where that is an integer
        p.stride_h = 1; p.stride_w = 1; p.pad_h = -g.pad_h; p.pad_w = -g.pad_w;
        p.tap_sign = -1; p.up_h = g.stride_h; p.up_w = g.stride_w;
    } else {
        p.stride_h = g.stride_h; p.stride_w = g.stride_w; p.pad_h = g.pad_h; p.pad_w = g.pad_w;
        p.tap_sign = 1; p.up_h = 1; p.up_w = 1;
    }
    set_divisors(p);
    plan->v = v;
    return TIR_OK;
}

static tir_status plan_conv(bool need_ptrs, const void* x, const void* w, void* y, int64_t N, int64_t H, int64_t W,
                            int64_t C, int64_t K, int64_t R, int64_t S, int stride_h, int stride_w, int pad_h,
                            int pad_w, int dil_h, int dil_w, int groups, int in, int out, const tir_epilogue* ep, const SplitLimits& sl,
                            Plan* plan) {
    const ConvGeom g = {N, 1, H, W, C, K, 1, R, S, 1, stride_h, stride_w, 0, pad_h, pad_w, 1, dil_h, dil_w, groups, false, 0, 0};
    return plan_conv_geom(need_ptrs, x, w, y, g, in, out, ep, sl, plan);
}

// Give a plan with a split reduction the workspace registered for its stream (the plan was made with that stream's
// limits; should the registration have gone meanwhile, the same variant runs unsplit).
static tir_status attach_workspace(Plan* plan, hipStream_t stream) {
    if (!plan->v || plan->p.ksplit <= 1) return TIR_OK;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(TIR_ERR_LAUNCH, "hipGetDevice failed: %s", hipGetErrorString(e));
    std::lock_guard<std::mutex> lock(g_ws_mu);
    auto it = g_ws.find(std::make_pair(dev, stream));
    if (it == g_ws.end()) {
        plan->p.ksplit = 1;
        return TIR_OK;
    }
    plan->p.ws = it->second.partial;
    plan->p.ws_count = it->second.count;
    return TIR_OK;
}

static tir_status run(const Plan& plan, hipStream_t stream) {
    if (!plan.v) return TIR_OK;
    if (plan.p.ksplit > 1 && (!plan.p.ws || !plan.p.ws_count || plan.p.batch > 65535))
        return fail(TIR_ERR_LAUNCH, "split reduction planned without its workspace");
    // grid.y is limited to 65535: launch the batch in slices
    const int es = elem_size(plan.v->dt), os = elem_size(plan.v->out);
    const int total = plan.p.batch;
    for (int b0 = 0; b0 < total; b0 += 65535) {
        Params p = plan.p;
        p.batch = total - b0 < 65535 ? total - b0 : 65535;
        p.A = (const char*)plan.p.A + (long long)b0 * p.a_bs * es;
        p.B = (const char*)plan.p.B + (long long)b0 * p.b_bs * es;
        p.C = (char*)plan.p.C + (long long)b0 * p.c_bs * os;
        if (p.bias) p.bias = (const char*)plan.p.bias + (long long)b0 * p.bias_bs * 4;
        hipError_t e = plan.v->fn(p, stream);
        if (e != hipSuccess) return fail(TIR_ERR_LAUNCH, "launch of %s failed: %s", plan.v->name, hipGetErrorString(e));
    }
    return TIR_OK;
}

static tir_status launch(Plan& plan, hipStream_t stream) {
    tir_status st = attach_workspace(&plan, stream);
    if (st != TIR_OK) return st;
    return run(plan, stream);
}

// ------------------------------------------------------------------------------- tuning by measurement
static bool record_fits(const TuneKey& k, const Variant* v) {
    if (v->dt != k.dt || v->out != k.out) return false;
    if (v->amode == k.amode && v->bmode == k.bmode) return true;
    return k.kind == 1 && k.amode == A_CONV && k.bmode == B_KMAJOR && v->amode == A_CONV_PATCH;   // re-checked against the shape when used
}

struct TrialGuard {
    ~TrialGuard() { g_trial = kNoChoice; }
};

// Run every variant that can compute the problem `make_plan` describes, `reps` times each, and record
// the fastest.  make_plan(Plan*) builds the launch plan honouring g_trial.
template <class MakePlan>
static tir_status tune_problem(MakePlan make_plan, int reps, hipStream_t stream, double* best_us, const char** best_name) {
    if (best_us) *best_us = 0.0;
    if (best_name) *best_name = "";
    if (reps <= 0 || reps > 1000) return fail(TIR_ERR_INVALID_ARG, "reps must be in [1, 1000]");
    if (g_force_name[0] || g_force_bm || g_force_ksplit) return fail(TIR_ERR_INVALID_ARG, "tuning while a variant or tile is forced");
    Plan base;
    g_trial = kNoChoice;
    tir_status st = make_plan(&base);
    if (st != TIR_OK) return st;
    if (!base.v) return TIR_OK;                       // zero-sized problem: nothing to measure
    hipEvent_t e0, e1;
    hipError_t ce = hipEventCreate(&e0);
    if (ce != hipSuccess) return fail(TIR_ERR_LAUNCH, "hipEventCreate failed: %s", hipGetErrorString(ce));
    ce = hipEventCreate(&e1);
    if (ce != hipSuccess) {
        (void)hipEventDestroy(e0);
        return fail(TIR_ERR_LAUNCH, "hipEventCreate failed: %s", hipGetErrorString(ce));
    }
    // the legacy default stream cannot be captured: trials then run on a stream of their own (which borrows the
    // caller's stream's workspace: everything queued there has finished, and the trials finish before the call returns)
    const hipStream_t caller_stream = stream;
    hipStream_t own = nullptr;
    if (!stream) {
        ce = hipStreamCreateWithFlags(&own, hipStreamNonBlocking);
        if (ce == hipSuccess) ce = hipDeviceSynchronize();      // work already queued on the default stream comes first
        if (ce != hipSuccess) {
            (void)hipEventDestroy(e0);
            (void)hipEventDestroy(e1);
            if (own) (void)hipStreamDestroy(own);
            return fail(TIR_ERR_LAUNCH, "tuning: cannot create a stream: %s", hipGetErrorString(ce));
        }
        stream = own;
    }
    TrialGuard guard;
    Choice best = kNoChoice;
    float best_ms = 0.f;
    std::vector<std::pair<Choice, float>> tried;      // every variant that was measured, with its time per launch
    // n launches of plan pl captured into one HIP graph and replayed (launched one by one, kernels of a few
    // microseconds would be timed at the host's launch rate, not the device's); ms per launch in *ms_out
    auto timed_plan = [&](const Plan& pl, int n, float* ms_out) -> tir_status {
        hipGraph_t graph = nullptr;
        hipGraphExec_t exec = nullptr;
        float ms = 0.f;
        hipError_t e = hipStreamBeginCapture(stream, hipStreamCaptureModeThreadLocal);
        if (e != hipSuccess) return fail(TIR_ERR_LAUNCH, "tuning: stream capture failed: %s", hipGetErrorString(e));
        tir_status s2 = TIR_OK;
        for (int r = 0; r < n && s2 == TIR_OK; ++r) s2 = run(pl, stream);
        e = hipStreamEndCapture(stream, &graph);
        if (s2 == TIR_OK && e == hipSuccess) e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
        if (s2 == TIR_OK && e == hipSuccess) e = hipGraphLaunch(exec, stream);            // upload + first run, untimed
        if (s2 == TIR_OK && e == hipSuccess) e = hipEventRecord(e0, stream);
        if (s2 == TIR_OK && e == hipSuccess) e = hipGraphLaunch(exec, stream);
        if (s2 == TIR_OK && e == hipSuccess) e = hipEventRecord(e1, stream);
        if (s2 == TIR_OK && e == hipSuccess) e = hipEventSynchronize(e1);
        if (s2 == TIR_OK && e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (exec) (void)hipGraphExecDestroy(exec);
        if (graph) (void)hipGraphDestroy(graph);
        if (s2 != TIR_OK) return s2;
        if (e != hipSuccess) return fail(TIR_ERR_LAUNCH, "tuning run of %s failed: %s", pl.v->name, hipGetErrorString(e));
        *ms_out = ms / (float)n;
        return TIR_OK;
    };
    if (base.v->amode == A_DEPTHWISE) {
        // The direct depth-wise kernel is not a tile variant and the planner prefers it whatever a record says:
        // there is nothing to choose, so it is timed (best_us is the time of the kernel that will run) and no
        // record is written.
        st = timed_plan(base, reps, &best_ms);
        (void)hipEventDestroy(e0);
        (void)hipEventDestroy(e1);
        if (own) (void)hipStreamDestroy(own);
        if (st == TIR_OK) {
            if (best_us) *best_us = (double)best_ms * 1e3;
            if (best_name) *best_name = base.v->name;
        }
        return st;
    }
    // reduction splits tried per variant (where the variant, the workspace and the reduction's length allow
    // them and the workgroups still fit two rounds of the CUs)
    static const int kSplits[] = {1, 2, 3, 4, 6, 8};
    for (int i = 0; i < kNumVariants * 6 && st == TIR_OK; ++i) {
        const Variant* v = &kVariants[i / 6];
        const int ks = kSplits[i % 6];
        if (!record_fits(base.key, v) || (v->amode == A_CONV_PATCH && !base.patch_ok)) continue;
        g_trial = Choice{v, ks};
        Plan pl;
        st = make_plan(&pl);
        if (st == TIR_ERR_UNSUPPORTED) { st = TIR_OK; continue; }      // this variant cannot run the problem
        if (st == TIR_OK) st = attach_workspace(&pl, caller_stream);
        if (st != TIR_OK) break;
        if (pl.p.ksplit != ks) continue;              // this split does not apply
        if (ks > 1) {
            const int64_t wgs = (int64_t)pl.p.tiles_m * pl.p.tiles_n * pl.p.batch * ks;
            const int64_t stages = ((int64_t)pl.p.K * elem_size(v->dt) + v->rowb - 1) / v->rowb;
            if (wgs > 2 * (int64_t)kCUs || stages / ks < 2) continue;
        }
        // one launch first (a variant several times slower than the best so far is not worth `reps`
        // more), then the measured batch; every HIP call is checked, the first failure ends the tuning
        float ms = 0.f;
        auto timed = [&](int n) -> tir_status { return timed_plan(pl, n, &ms); };
        st = timed(1);
        if (st != TIR_OK) break;
        if (best.v && ms > 4.f * best_ms + 0.05f) continue;
        st = timed(reps);
        if (st != TIR_OK) break;
        tried.push_back({Choice{v, ks}, ms});
        if (!best.v || ms < best_ms) { best = Choice{v, ks}; best_ms = ms; }
    }
    // Play-off.  One timing per variant is good to a few per cent (clocks move with the power the previous trial
    // drew), and the variants near the top are often closer than that: those within 10 % of the fastest are timed
    // again, five rounds in turn, and each keeps its fastest round.
    if (st == TIR_OK && best.v) {
        std::vector<std::pair<Choice, float>> top;
        for (const auto& t : tried)
            if (t.second <= 1.10f * best_ms) top.push_back(t);
        for (int round = 0; round < 5 && st == TIR_OK && top.size() > 1; ++round) {
            for (auto& t : top) {
                g_trial = t.first;
                Plan pl;
                st = make_plan(&pl);
                if (st == TIR_OK) st = attach_workspace(&pl, caller_stream);
                float ms = 0.f;
                if (st == TIR_OK) st = timed_plan(pl, reps, &ms);
                if (st != TIR_OK) break;
                if (ms < t.second) t.second = ms;
            }
        }
        if (st == TIR_OK) {
            for (const auto& t : top)
                if (t.second < best_ms) { best = t.first; best_ms = t.second; }
            // The trials run on operands that sit in the caches.  If a two-slot ring is the fastest, a ring of three or more
            // slots within 2 % of it wins instead: two slots lose most when the operands come from memory (4096-cube GEMM: the
            // two-slot 256x256 tile is 7 % slower cold than hot, the three- and four-slot ones are not).  Rings deeper than three
            // earn no such bonus: their longer prologue delays the first stage of a cold launch (2048-cube int8 GEMM on 128x128
            // tiles, four slots against three: the same 11.2 us hot, 17.1 - 18.8 against 16.0 - 16.3 us cold).
            if (best.v->nstage < 3) {
                const float fastest = best_ms;
                for (const auto& t : top)
                    if (t.second <= 1.02f * fastest && t.first.v->nstage >= 3 && (best.v->nstage < 3 || t.second < best_ms)) {
                        best = t.first;
                        best_ms = t.second;
                    }
            }
        }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (own) (void)hipStreamDestroy(own);
    if (st != TIR_OK) return st;
    if (best.v) {
        std::lock_guard<std::mutex> lock(g_tune_mu);
        g_tuned[base.key] = best;
        if (best_us) *best_us = (double)best_ms * 1e3;
        if (best_name) *best_name = best.v->name;
    }
    return TIR_OK;
}

}  // namespace tir

using namespace tir;

extern "C" {

tir_status tir_gemm_fused(const void* A, const void* B, void* C, int64_t M, int64_t N, int64_t K, int64_t a_rs,
                          int64_t a_cs, int64_t b_rs, int64_t b_cs, int64_t c_rs, int64_t c_cs, tir_dtype in,
                          tir_dtype out, const tir_epilogue* ep, tir_stream stream) {
    Plan plan;
    tir_status st = plan_gemm(true, A, B, C, 1, M, N, K, 0, a_rs, a_cs, 0, b_rs, b_cs, 0, c_rs, c_cs, (int)in, (int)out, ep, stream_split_limits((hipStream_t)stream), &plan);
    if (st != TIR_OK) return st;
    return launch(plan, (hipStream_t)stream);
}

tir_status tir_batch_matmul_fused(const void* A, const void* B, void* C, int64_t batch, int64_t M, int64_t N, int64_t K,
                                  int64_t a_bs, int64_t a_rs, int64_t a_cs, int64_t b_bs, int64_t b_rs, int64_t b_cs,
                                  int64_t c_bs, int64_t c_rs, int64_t c_cs, tir_dtype in, tir_dtype out,
                                  const tir_epilogue* ep, tir_stream stream) {
    Plan plan;
    tir_status st = plan_gemm(true, A, B, C, batch, M, N, K, a_bs, a_rs, a_cs, b_bs, b_rs, b_cs, c_bs, c_rs, c_cs, (int)in, (int)out, ep, stream_split_limits((hipStream_t)stream), &plan);
    if (st != TIR_OK) return st;
    return launch(plan, (hipStream_t)stream);
}

tir_status tir_conv2d_fused(const void* x, const void* w, void* y, int64_t N, int64_t H, int64_t W, int64_t C, int64_t K,
                            int64_t R, int64_t S, int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w,
                            int groups, tir_dtype in, tir_dtype out, const tir_epilogue* ep, tir_stream stream) {
    Plan plan;
    tir_status st = plan_conv(true, x, w, y, N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, groups, (int)in, (int)out, ep, stream_split_limits((hipStream_t)stream), &plan);
    if (st != TIR_OK) return st;
    return launch(plan, (hipStream_t)stream);
}

tir_status tir_gemm(const void* A, const void* B, void* C, int64_t M, int64_t N, int64_t K, int64_t a_rs,
                    int64_t a_cs, int64_t b_rs, int64_t b_cs, int64_t c_rs, int64_t c_cs, tir_dtype in,
                    tir_dtype out, tir_stream stream) {
    return tir_gemm_fused(A, B, C, M, N, K, a_rs, a_cs, b_rs, b_cs, c_rs, c_cs, in, out, nullptr, stream);
}

tir_status tir_batch_matmul(const void* A, const void* B, void* C, int64_t batch, int64_t M, int64_t N, int64_t K,
                            int64_t a_bs, int64_t a_rs, int64_t a_cs, int64_t b_bs, int64_t b_rs, int64_t b_cs,
                            int64_t c_bs, int64_t c_rs, int64_t c_cs, tir_dtype in, tir_dtype out,
                            tir_stream stream) {
    return tir_batch_matmul_fused(A, B, C, batch, M, N, K, a_bs, a_rs, a_cs, b_bs, b_rs, b_cs, c_bs, c_rs, c_cs, in, out, nullptr, stream);
}

tir_status tir_conv2d(const void* x, const void* w, void* y, int64_t N, int64_t H, int64_t W, int64_t C, int64_t K,
                      int64_t R, int64_t S, int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w,
                      int groups, tir_dtype in, tir_dtype out, tir_stream stream) {
    return tir_conv2d_fused(x, w, y, N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, groups, in, out, nullptr, stream);
}

const char* tir_last_error(void) { return g_err; }

// "<variant>" or "<variant>/z<slices>" for a plan with a split reduction
static const char* plan_name(const Plan& plan) {
    static thread_local char buf[160];
    if (!plan.v) return "";
    if (plan.p.phases_h) snprintf(buf, sizeof buf, "%s/ph%dx%d", plan.v->name, plan.p.phases_h, plan.p.phases_w);
    else if (plan.p.ksplit > 1) snprintf(buf, sizeof buf, "%s/z%d", plan.v->name, plan.p.ksplit);
    else return plan.v->name;
    return buf;
}

const char* tir_gemm_variant(int64_t batch, int64_t M, int64_t N, int64_t K, int64_t a_rs, int64_t a_cs, int64_t b_rs,
                             int64_t b_cs, int64_t c_rs, int64_t c_cs, tir_dtype in, tir_dtype out) {
    Plan plan;
    // batch strides of dense operands, only their divisibility matters for the choice
    tir_status st = plan_gemm(false, nullptr, nullptr, nullptr, batch, M, N, K, M * K, a_rs, a_cs, K * N, b_rs, b_cs, M * N, c_rs, c_cs, (int)in, (int)out, out == TIR_I8 ? &kQueryRequant : nullptr, kRegisteredSplit, &plan);
    return st == TIR_OK ? plan_name(plan) : "";
}

const char* tir_conv2d_variant(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                               int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w, int groups,
                               tir_dtype in, tir_dtype out) {
    Plan plan;
    tir_status st = plan_conv(false, nullptr, nullptr, nullptr, N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, groups, (int)in, (int)out, out == TIR_I8 ? &kQueryRequant : nullptr, kRegisteredSplit, &plan);
    return st == TIR_OK ? plan_name(plan) : "";
}

const char* tir_conv3d_variant(int64_t N, int64_t D, int64_t H, int64_t W, int64_t C, int64_t K, int64_t T, int64_t R,
                               int64_t S, int stride_d, int stride_h, int stride_w, int pad_d, int pad_h, int pad_w,
                               int dil_d, int dil_h, int dil_w, int groups, tir_dtype in, tir_dtype out) {
    const ConvGeom g = {N, D, H, W, C, K, T, R, S, stride_d, stride_h, stride_w, pad_d, pad_h, pad_w, dil_d, dil_h, dil_w, groups, false, 0, 0};
    Plan plan;
    tir_status st = plan_conv_geom(false, nullptr, nullptr, nullptr, g, (int)in, (int)out, out == TIR_I8 ? &kQueryRequant : nullptr, kRegisteredSplit, &plan);
    return st == TIR_OK ? plan_name(plan) : "";
}

const char* tir_conv2d_transpose_variant(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                                         int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w,
                                         int outpad_h, int outpad_w, int groups, tir_dtype in, tir_dtype out) {
    const ConvGeom g = {N, 1, H, W, C, K, 1, R, S, 1, stride_h, stride_w, 0, pad_h, pad_w, 1, dil_h, dil_w, groups, true, outpad_h, outpad_w};
    Plan plan;
    tir_status st = plan_conv_geom(false, nullptr, nullptr, nullptr, g, (int)in, (int)out, out == TIR_I8 ? &kQueryRequant : nullptr, kRegisteredSplit, &plan);
    return st == TIR_OK ? plan_name(plan) : "";
}

void tir_debug_force_tile(int bm, int bn) {
    g_force_bm = bm;
    g_force_bn = bn;
}

uint64_t tir_workspace_bytes(void) { return (uint64_t)(kWsBytes + kWsTiles * 4); }

tir_status tir_set_workspace(tir_stream stream_, void* ws, uint64_t bytes) {
    hipStream_t stream = (hipStream_t)stream_;
    if (ws) {
        if (bytes < tir_workspace_bytes())
            return fail(TIR_ERR_INVALID_ARG, "workspace of %llu bytes, tir_workspace_bytes() = %llu are needed", (unsigned long long)bytes,
                        (unsigned long long)tir_workspace_bytes());
        if ((uintptr_t)ws & 255) return fail(TIR_ERR_ALIGNMENT, "workspace not aligned to 256 bytes");
    }
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(TIR_ERR_LAUNCH, "hipGetDevice failed: %s", hipGetErrorString(e));
    std::lock_guard<std::mutex> lock(g_ws_mu);
    const std::pair<int, hipStream_t> key(dev, stream);
    if (!ws) {
        g_ws.erase(key);
        return TIR_OK;
    }
    unsigned* count = (unsigned*)((char*)ws + kWsBytes);
    hipLaunchKernelGGL(clear_counters_kernel, dim3((unsigned)(kWsTiles / 256)), dim3(256), 0, stream, count, (int)kWsTiles);
    e = hipGetLastError();
    if (e != hipSuccess) return fail(TIR_ERR_LAUNCH, "clearing the workspace counters failed: %s", hipGetErrorString(e));
    g_ws[key] = Workspace{ws, count};
    return TIR_OK;
}

void tir_debug_force_ksplit(int slices) { g_force_ksplit = slices > 1 ? slices : 0; }

void tir_debug_force_variant(const char* name_part) {
    snprintf(g_force_name, sizeof g_force_name, "%s", name_part ? name_part : "");
}

int tir_debug_variant_count(void) { return kNumVariants; }

const char* tir_debug_variant_name(int i) { return (i >= 0 && i < kNumVariants) ? kVariants[i].name : ""; }

void tir_debug_tile_of_block(int bid, int tiles_m, int tiles_n, int* tm, int* tn) {
    const FastDiv gw = make_fastdiv((unsigned)(kGroupM * tiles_n));
    tile_of_block(bid, tiles_m, tiles_n, gw.magic, gw.shift, tm, tn);
}

unsigned tir_debug_fastdiv(unsigned d, unsigned m) {
    const FastDiv f = make_fastdiv(d);
    return fastdiv(m, f.magic, f.shift);
}

tir_status tir_probe_mfma_rate(void* sink, int iters, int random_operands, double* flop, tir_stream stream) {
    if (!sink || iters <= 0) return fail(TIR_ERR_INVALID_ARG, "tir_probe_mfma_rate: sink is null or iters <= 0");
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(1024), dim3(256), 0, (hipStream_t)stream, (float*)sink, iters, random_operands);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(TIR_ERR_LAUNCH, "probe launch failed: %s", hipGetErrorString(e));
    if (flop) *flop = 1024.0 * 4.0 * (double)iters * 16.0 * 32768.0;
    return TIR_OK;
}

tir_status tir_tune_batch_matmul(const void* A, const void* B, void* C, int64_t batch, int64_t M, int64_t N, int64_t K,
                                 int64_t a_bs, int64_t a_rs, int64_t a_cs, int64_t b_bs, int64_t b_rs, int64_t b_cs,
                                 int64_t c_bs, int64_t c_rs, int64_t c_cs, tir_dtype in, tir_dtype out,
                                 const tir_epilogue* ep, int reps, double* best_us, tir_stream stream) {
    const SplitLimits sl = stream_split_limits((hipStream_t)stream);
    auto make = [&](Plan* pl) {
        return plan_gemm(true, A, B, C, batch, M, N, K, a_bs, a_rs, a_cs, b_bs, b_rs, b_cs, c_bs, c_rs, c_cs, (int)in, (int)out, ep, sl, pl);
    };
    return tune_problem(make, reps, (hipStream_t)stream, best_us, nullptr);
}

tir_status tir_tune_conv2d(const void* x, const void* w, void* y, int64_t N, int64_t H, int64_t W, int64_t C, int64_t K,
                           int64_t R, int64_t S, int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w,
                           int groups, tir_dtype in, tir_dtype out, const tir_epilogue* ep, int reps, double* best_us,
                           tir_stream stream) {
    const SplitLimits sl = stream_split_limits((hipStream_t)stream);
    auto make = [&](Plan* pl) {
        return plan_conv(true, x, w, y, N, H, W, C, K, R, S, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, groups, (int)in, (int)out, ep, sl, pl);
    };
    return tune_problem(make, reps, (hipStream_t)stream, best_us, nullptr);
}

tir_status tir_tune_conv3d(const void* x, const void* w, void* y, int64_t N, int64_t D, int64_t H, int64_t W, int64_t C,
                           int64_t K, int64_t T, int64_t R, int64_t S, int stride_d, int stride_h, int stride_w,
                           int pad_d, int pad_h, int pad_w, int dil_d, int dil_h, int dil_w, int groups, tir_dtype in,
                           tir_dtype out, const tir_epilogue* ep, int reps, double* best_us, tir_stream stream) {
    const ConvGeom g = {N, D, H, W, C, K, T, R, S, stride_d, stride_h, stride_w, pad_d, pad_h, pad_w, dil_d, dil_h, dil_w, groups, false, 0, 0};
    const SplitLimits sl = stream_split_limits((hipStream_t)stream);
    auto make = [&](Plan* pl) { return plan_conv_geom(true, x, w, y, g, (int)in, (int)out, ep, sl, pl); };
    return tune_problem(make, reps, (hipStream_t)stream, best_us, nullptr);
}

tir_status tir_tune_conv2d_transpose(const void* x, const void* w, void* y, int64_t N, int64_t H, int64_t W, int64_t C,
                                     int64_t K, int64_t R, int64_t S, int stride_h, int stride_w, int pad_h, int pad_w,
                                     int dil_h, int dil_w, int outpad_h, int outpad_w, int groups, tir_dtype in,
                                     tir_dtype out, const tir_epilogue* ep, int reps, double* best_us,
                                     tir_stream stream) {
    const ConvGeom g = {N, 1, H, W, C, K, 1, R, S, 1, stride_h, stride_w, 0, pad_h, pad_w, 1, dil_h, dil_w, groups, true, outpad_h, outpad_w};
    const SplitLimits sl = stream_split_limits((hipStream_t)stream);
    auto make = [&](Plan* pl) { return plan_conv_geom(true, x, w, y, g, (int)in, (int)out, ep, sl, pl); };
    return tune_problem(make, reps, (hipStream_t)stream, best_us, nullptr);
}

int tir_tune_count(void) {
    std::lock_guard<std::mutex> lock(g_tune_mu);
    return (int)g_tuned.size();
}

void tir_tune_clear(void) {
    std::lock_guard<std::mutex> lock(g_tune_mu);
    g_tuned.clear();
}

tir_status tir_tune_save(const char* path) {
    if (!path) return fail(TIR_ERR_INVALID_ARG, "path is null");
    FILE* f = fopen(path, "w");
    if (!f) return fail(TIR_ERR_INVALID_ARG, "cannot open %s for writing", path);
    std::lock_guard<std::mutex> lock(g_tune_mu);
    fprintf(f, "tir-tune-records 1\n");
    for (const auto& kv : g_tuned) {
        const TuneKey& k = kv.first;
        fprintf(f, "%d %d %d %d %d %lld %lld %lld %lld %llu %s %d\n", k.kind, k.dt, k.out, k.amode, k.bmode, (long long)k.batch,
                (long long)k.M, (long long)k.N, (long long)k.K, (unsigned long long)k.geom, kv.second.v->name, kv.second.ksplit);
    }
    const bool ok = fclose(f) == 0;
    return ok ? TIR_OK : fail(TIR_ERR_INVALID_ARG, "writing %s failed", path);
}

tir_status tir_tune_load(const char* path) {
    if (!path) return fail(TIR_ERR_INVALID_ARG, "path is null");
    FILE* f = fopen(path, "r");
    if (!f) return fail(TIR_ERR_INVALID_ARG, "cannot open %s", path);
    char line[512];
    int version = 0;
    if (!fgets(line, sizeof line, f) || sscanf(line, "tir-tune-records %d", &version) != 1 || version != 1) {
        fclose(f);
        return fail(TIR_ERR_INVALID_ARG, "%s is not a version-1 record file", path);
    }
    std::lock_guard<std::mutex> lock(g_tune_mu);
    while (fgets(line, sizeof line, f)) {
        TuneKey k;
        long long b, m, n, kk;
        unsigned long long geom;
        char name[128];
        int ks = 1;                                     // last field: slices of a split reduction (absent = 1)
        if (sscanf(line, "%d %d %d %d %d %lld %lld %lld %lld %llu %127s %d", &k.kind, &k.dt, &k.out, &k.amode, &k.bmode, &b, &m, &n, &kk,
                   &geom, name, &ks) < 11 || ks < 1 || ks > 64)
            continue;                                   // malformed line: ignored
        k.batch = b; k.M = m; k.N = n; k.K = kk; k.geom = geom;
        // records of another build may name variants this one does not have, or that do not fit the key
        for (int i = 0; i < kNumVariants; ++i)
            if (strcmp(kVariants[i].name, name) == 0 && record_fits(k, &kVariants[i])) {
                g_tuned[k] = Choice{&kVariants[i], ks};      // a split that does not fit the problem is dropped when planned
                break;
            }
    }
    fclose(f);
    return TIR_OK;
}

tir_status tir_attention(const void* Q, const void* K, const void* V, void* O, int64_t batch, int64_t M, int64_t N,
                         int64_t d, float scale, tir_dtype in, tir_dtype out, tir_stream stream) {
    if ((int)in < 0 || (int)in > TIR_I32 || (int)out < 0 || (int)out > TIR_I32) return fail(TIR_ERR_INVALID_ARG, "unknown dtype code (in=%d out=%d)", (int)in, (int)out);
    if (!((in == TIR_F16 && (out == TIR_F16 || out == TIR_F32)) || (in == TIR_BF16 && (out == TIR_BF16 || out == TIR_F32))))
        return fail(TIR_ERR_UNSUPPORTED, "attention: unsupported (in, out) dtype pair (%d, %d)", (int)in, (int)out);
    if (batch < 0 || M < 0 || N < 0 || d < 0) return fail(TIR_ERR_INVALID_ARG, "negative extent (batch=%lld M=%lld N=%lld d=%lld)", (long long)batch, (long long)M, (long long)N, (long long)d);
    if (d != 64 && d != 128) return fail(TIR_ERR_UNSUPPORTED, "attention: head dimension %lld (64 and 128 are compiled)", (long long)d);
    if (!(scale == scale) || scale > 3.0e38f || scale < -3.0e38f) return fail(TIR_ERR_INVALID_ARG, "attention: scale must be finite");
    if (batch == 0 || M == 0) return TIR_OK;
    if (N == 0) return fail(TIR_ERR_INVALID_ARG, "attention: the softmax over zero keys is undefined (N = 0)");
    if (!Q || !K || !V || !O) return fail(TIR_ERR_INVALID_ARG, "Q, K, V or O is null");
    if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(O, 16)) return fail(TIR_ERR_ALIGNMENT, "attention: Q, K, V and O must be 16-byte aligned");
    const int64_t tiles_m = (M + 127) / 128;
    if (M > kMaxExtent || N > kMaxExtent || batch * tiles_m > kMaxExtent) return fail(TIR_ERR_UNSUPPORTED, "extent beyond 2^31-1");
    attn_launch_fn fn = attention_launcher((int)in, (int)out, (int)d);
    if (!fn) return fail(TIR_ERR_UNSUPPORTED, "attention: no kernel for this dtype pair / head dimension");
    AttnParams p;
    p.Q = Q; p.K = K; p.V = V; p.O = O;
    p.M = (int)M; p.N = (int)N; p.batch = (int)batch; p.tiles_m = (int)tiles_m;
    p.scale_log2e = scale * 1.44269504088896340736f;
    const FastDiv dtm = make_fastdiv((unsigned)tiles_m);
    p.div_tm_magic = dtm.magic; p.div_tm_shift = dtm.shift;
    hipError_t e = fn(p, (hipStream_t)stream);
    if (e != hipSuccess) return fail(TIR_ERR_LAUNCH, "attention launch failed: %s", hipGetErrorString(e));
    return TIR_OK;
}

tir_status tir_conv1d(const void* x, const void* w, void* y, int64_t N, int64_t L, int64_t C, int64_t K, int64_t R,
                      int stride, int pad, int dil, int groups, tir_dtype in, tir_dtype out, const tir_epilogue* ep,
                      tir_stream stream) {
    // a 1-D convolution is the 2-D one on an image of height 1 with a filter of height 1
    Plan plan;
    tir_status st = plan_conv(true, x, w, y, N, 1, L, C, K, 1, R, 1, stride, 0, pad, 1, dil, groups, (int)in, (int)out, ep, stream_split_limits((hipStream_t)stream), &plan);
    if (st != TIR_OK) return st;
    return launch(plan, (hipStream_t)stream);
}

tir_status tir_conv3d(const void* x, const void* w, void* y, int64_t N, int64_t D, int64_t H, int64_t W, int64_t C,
                      int64_t K, int64_t T, int64_t R, int64_t S, int stride_d, int stride_h, int stride_w, int pad_d,
                      int pad_h, int pad_w, int dil_d, int dil_h, int dil_w, int groups, tir_dtype in, tir_dtype out,
                      const tir_epilogue* ep, tir_stream stream) {
    const ConvGeom g = {N, D, H, W, C, K, T, R, S, stride_d, stride_h, stride_w, pad_d, pad_h, pad_w, dil_d, dil_h, dil_w, groups, false, 0, 0};
    Plan plan;
    tir_status st = plan_conv_geom(true, x, w, y, g, (int)in, (int)out, ep, stream_split_limits((hipStream_t)stream), &plan);
    if (st != TIR_OK) return st;
    return launch(plan, (hipStream_t)stream);
}

tir_status tir_conv2d_transpose(const void* x, const void* w, void* y, int64_t N, int64_t H, int64_t W, int64_t C,
                                int64_t K, int64_t R, int64_t S, int stride_h, int stride_w, int pad_h, int pad_w,
                                int dil_h, int dil_w, int outpad_h, int outpad_w, int groups, tir_dtype in, tir_dtype out,
                                const tir_epilogue* ep, tir_stream stream) {
    const ConvGeom g = {N, 1, H, W, C, K, 1, R, S, 1, stride_h, stride_w, 0, pad_h, pad_w, 1, dil_h, dil_w, groups, true, outpad_h, outpad_w};
    Plan plan;
    tir_status st = plan_conv_geom(true, x, w, y, g, (int)in, (int)out, ep, stream_split_limits((hipStream_t)stream), &plan);
    if (st != TIR_OK) return st;
    return launch(plan, (hipStream_t)stream);
}

// ------------------------------------------------------------------------------- split GEMM on static scratch
}  // extern "C"

namespace tir {
// Partial sums, then arrival counters, of tir_gemm_split_static.  In host code this name is only a handle for
// hipGetSymbolAddress: every use of the memory goes through the per-device address kept in g_static_ptr.
static __device__ __align__(256) unsigned char scratch[TIR_STATIC_SCRATCH_BYTES + TIR_STATIC_SCRATCH_TILES * 4];
static const int kMaxDevices = 64;
static std::mutex g_static_mu;
static void* g_static_ptr[kMaxDevices] = {};

// Address of the current device's copy of `scratch` (looked up once per device).
static tir_status static_scratch(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(TIR_ERR_LAUNCH, "hipGetDevice failed: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(TIR_ERR_UNSUPPORTED, "device index %d beyond %d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return fail(TIR_ERR_LAUNCH, "hipGetSymbolAddress of the static scratch failed on device %d: %s", dev, hipGetErrorString(e));
        }
        g_static_ptr[dev] = ptr;
    }
    *out = g_static_ptr[dev];
    return TIR_OK;
}
}  // namespace tir

extern "C" {

tir_status tir_gemm_split_static(const void* A, const void* B, void* C, int64_t M, int64_t N, int64_t K, int64_t a_rs,
                                 int64_t a_cs, int64_t b_rs, int64_t b_cs, int64_t c_rs, int64_t c_cs, tir_dtype in,
                                 tir_dtype out, const tir_epilogue* ep, int slices, tir_stream stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    if (slices < 2 || slices > 64) return fail(TIR_ERR_INVALID_ARG, "tir_gemm_split_static: slices = %d, must be in [2, 64]", slices);
    if (K == 0) return fail(TIR_ERR_INVALID_ARG, "tir_gemm_split_static: K = 0, there is no reduction to split");
    const SplitLimits sl = {(int64_t)TIR_STATIC_SCRATCH_BYTES, (int64_t)TIR_STATIC_SCRATCH_TILES, slices};
    Plan plan;
    tir_status st = plan_gemm(true, A, B, C, 1, M, N, K, 0, a_rs, a_cs, 0, b_rs, b_cs, 0, c_rs, c_cs, (int)in, (int)out, ep, sl, &plan);
    if (st == TIR_ERR_UNSUPPORTED && plan.key.kind == 0 && !plan.v) {
        // no variant splits this problem `slices` ways inside the static scratch: say which limit it is
        if (plan.key.amode != A_KMAJOR)
            return fail(TIR_ERR_UNSUPPORTED, "tir_gemm_split_static: operand strides / alignment need the general kernel, which has no split reduction");
        const SplitLimits any = {(int64_t)1 << 60, (int64_t)1 << 40, slices};
        const Choice c = pick(plan.key.dt, plan.key.out, plan.key.amode, plan.key.bmode, 1, M, N, K, any);
        if (c.v) {
            const int64_t tiles = ((M + c.v->bm - 1) / c.v->bm) * ((N + c.v->bn - 1) / c.v->bn);
            return fail(TIR_ERR_INVALID_ARG, "tir_gemm_split_static: %lld tiles x %d slices need %lld bytes of partial sums and %lld counters; the static scratch holds %u bytes and %d counters",
                        (long long)tiles, slices, (long long)(tiles * slices * c.v->bm * c.v->bn * 4), (long long)tiles, (unsigned)TIR_STATIC_SCRATCH_BYTES, (int)TIR_STATIC_SCRATCH_TILES);
        }
        return fail(TIR_ERR_INVALID_ARG, "tir_gemm_split_static: a reduction of K = %lld cannot be cut into %d non-empty slices of whole stages", (long long)K, slices);
    }
    if (st != TIR_OK) return st;
    if (!plan.v) return TIR_OK;                       // M or N is zero
    if (plan.p.ksplit != slices) return fail(TIR_ERR_UNSUPPORTED, "tir_gemm_split_static: variant %s cannot split %d ways", plan.v->name, slices);
    void* base = nullptr;
    st = static_scratch(&base);
    if (st != TIR_OK) return st;
    plan.p.ws = base;
    plan.p.ws_count = (unsigned*)((char*)base + TIR_STATIC_SCRATCH_BYTES);
    // The array keeps whatever the last call left: the counters of the tiles this launch uses start at zero
    // (a kernel, not a memset: the call may be captured into a graph).
    const int ntiles = plan.p.tiles_m * plan.p.tiles_n;
    hipLaunchKernelGGL(clear_counters_kernel, dim3((unsigned)((ntiles + 255) / 256)), dim3(256), 0, stream, plan.p.ws_count, ntiles);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(TIR_ERR_LAUNCH, "clearing the static scratch counters failed: %s", hipGetErrorString(e));
    return run(plan, stream);
}

const char* tir_version(void) { return "0.1"; }

}  // extern "C"
