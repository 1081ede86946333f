// Host side of libcks: argument checking, tile selection and kernel launches
// behind the C ABI declared in include/cks.h.  gfx950 only.
#include "../../include/cks.h"

#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <atomic>
#include <cstring>
#include <mutex>
#include <set>
#include <utility>

#include "cks_pack.h"
#include "cks_patch_fwd.h"
#include "cks_patch_gemm.h"
#include "cks_pixel_dma.h"
#include "cks_pixel_gemm.h"
#include "cks_rowrun_dma.h"
#include "cks_rowrun_gemm.h"
#include "cks_scatter_deconv.h"
#include "cks_sweep_deconv.h"
#include "cks_strip_fwd.h"
#include "cks_strip_wgrad.h"

// Scratch memory of cks_dilated_conv2d_wgrad_noalloc_hw: one array per GPU, part of the loaded code object,
// held until the process ends.  In host code the array's name only stands for the symbol; its device
// address is looked up once per device (static_scratch) and only that address is handed to kernels.
static __device__ __align__(256) unsigned char scratch[CKS_STATIC_SCRATCH_BYTES];

namespace {

using namespace cks;

constexpr int kCUs = 256;  // compute units of one MI355X

// Tuning experiments: a library built with -DCKS_TUNING reads CKS_TUNE_* environment variables that
// force other tiles, segment counts and load paths for A/B measurements, and carries the kernel
// instantiations only they can select.  The product build defines nothing of it: tune() is then a
// constant and every branch that depends on it disappears.
#ifdef CKS_TUNING
constexpr bool kTuning = true;
inline const char *tune(const char *name) { return getenv(name); }
#else
constexpr bool kTuning = false;
constexpr const char *tune(const char *) { return nullptr; }
#endif

thread_local int g_last_hip_error = 0;

// cks_plan_hw runs the very code path of an entry point with this recorder installed: launch() then
// writes the kernel's name and launch shape into the text instead of enqueuing anything.
struct PlanRecorder {
    char *text;
    size_t cap, len;
    bool truncated;
};
thread_local PlanRecorder *g_plan = nullptr;

struct Geo {
    int N, C, H, W, OC, FH, FW;
    int sh, sw, ph, pw;   // stride and padding per axis (Table I: <sh sw>, <ph pw>)
    int OH, OW;
    bool same_on_both_axes() const { return sh == sw && ph == pw; }
};

inline bool fits_i31(long long v) { return v > 0 && v < (1LL << 31); }

int check_geo(Geo &g, int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || OC <= 0 || FH <= 0 || FW <= 0) return CKS_ERR_SHAPE;
    if (sh < 1 || sw < 1 || ph < 0 || pw < 0) return CKS_ERR_SHAPE;
    if ((long long)H + 2LL * ph < FH || (long long)W + 2LL * pw < FW) return CKS_ERR_SHAPE;
    if (ph > (1 << 20) || pw > (1 << 20) || sh > (1 << 20) || sw > (1 << 20)) return CKS_ERR_SHAPE;
    g = Geo{N, C, H, W, OC, FH, FW, sh, sw, ph, pw, (H + 2 * ph - FH) / sh + 1, (W + 2 * pw - FW) / sw + 1};
    if (!fits_i31((long long)N * H * W * C) || !fits_i31((long long)OC * FH * FW * C) ||
        !fits_i31((long long)N * g.OH * g.OW * OC))
        return CKS_ERR_SHAPE;
    return CKS_OK;
}

inline int hip_fail(hipError_t e)
{
    g_last_hip_error = (int)e;
    return CKS_ERR_HIP;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Kernels that need more than 64 KB of dynamic LDS must be told so once per
// device; the call is a driver round trip, so the (kernel, device) pairs already
// configured (for the full 160 KB) are remembered.
inline hipError_t allow_large_lds(const void *kernel)
{
    static std::mutex mu;
    static std::set<std::pair<const void *, int>> done;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    if (done.count({kernel, dev})) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e == hipSuccess) done.insert({kernel, dev});
    return e;
}

// Device address of this GPU's copy of `scratch`, looked up on the first call per device.
constexpr int kMaxDevices = 64;
int static_scratch(void **out)
{
    static std::mutex mu;
    static std::atomic<void *> known[kMaxDevices];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return CKS_ERR_UNSUPPORTED;
    void *p = known[dev].load(std::memory_order_acquire);
    if (!p) {
        std::lock_guard<std::mutex> lock(mu);
        p = known[dev].load(std::memory_order_relaxed);
        if (!p) {
            e = hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess) return hip_fail(e);
            if (!p) return CKS_ERR_UNSUPPORTED;
            known[dev].store(p, std::memory_order_release);
        }
    }
    *out = p;
    return CKS_OK;
}

// A kernel's name as the demangler prints its instantiation, e.g. "rowrun_gemm_dma<2, 64, 64, 2, 2>":
// base name, integer template arguments, then boolean ones.
struct KName {
    const char *base;
    int nInts;
    int ints[8];
    int nBools;
    bool bools[2];
};
inline KName kname(const char *base) { return KName{base, 0, {}, 0, {}}; }
template <typename... I>
inline KName kname(const char *base, I... ints)
{
    KName k{base, (int)sizeof...(I), {(int)ints...}, 0, {}};
    return k;
}
inline KName with_bools(KName k, bool a) { k.nBools = 1; k.bools[0] = a; return k; }
inline KName with_bools(KName k, bool a, bool b) { k.nBools = 2; k.bools[0] = a; k.bools[1] = b; return k; }

void record_launch(const KName &k, long long blocks, int threads, size_t lds)
{
    PlanRecorder &R = *g_plan;
    char one[192];
    int n = snprintf(one, sizeof one, "%s", k.base);
    if (k.nInts + k.nBools > 0) {
        n += snprintf(one + n, sizeof one - n, "<");
        for (int i = 0; i < k.nInts; ++i) n += snprintf(one + n, sizeof one - n, i ? ", %d" : "%d", k.ints[i]);
        for (int i = 0; i < k.nBools; ++i)
            n += snprintf(one + n, sizeof one - n, (i || k.nInts) ? ", %s" : "%s", k.bools[i] ? "true" : "false");
        n += snprintf(one + n, sizeof one - n, ">");
    }
    n += snprintf(one + n, sizeof one - n, " [%lld x %d, lds %zu]\n", blocks, threads, lds);
    if (R.text && R.len + (size_t)n + 1 <= R.cap) {
        memcpy(R.text + R.len, one, (size_t)n + 1);
        R.len += (size_t)n;
    } else {
        R.truncated = true;
    }
}

template <typename K, typename... A>
int launch_args(const KName &name, K kernel, int blocks, size_t lds, hipStream_t st, int threads, const A &...args)
{
    if (lds > 160 * 1024) return CKS_ERR_SHAPE;
    if (const char *t = tune("CKS_TUNE_WG_PER_CU")) {   // cap the workgroups resident per compute unit
        const int n = atoi(t);
        if (n > 0) {
            const size_t want = (size_t)(160 * 1024 / n) / 256 * 256;
            if (want > lds) lds = want;
        }
    }
    if (g_plan) {
        record_launch(name, blocks, threads, lds);
        return CKS_OK;
    }
    if (lds > 64 * 1024) {
        hipError_t e = allow_large_lds(reinterpret_cast<const void *>(kernel));
        if (e != hipSuccess) return hip_fail(e);
    }
    hipLaunchKernelGGL(kernel, dim3(blocks), dim3(threads), lds, st, args...);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? CKS_OK : hip_fail(e);
}

template <typename K, typename P>
int launch(const KName &name, K kernel, const P &params, int blocks, size_t lds, hipStream_t st, int threads = kThreads)
{
    return launch_args(name, kernel, blocks, lds, st, threads, params);
}

// ---------------------------------------------------------------- ConvV2 / KS-deconv Stage 2&3

// untrimmed: the ablation's operators without filter trimming (plain convolution, KS-deconv of Algorithm 2); they
// exist for the 64x64 tile loaded straight into LDS only.
template <int OP, int BM, int BN, int WM, int WN>
int launch_rowrun(RowRunParams P, int rows, int cols, bool vec, hipStream_t st, bool untrimmed = false)
{
    P.mTiles = (rows + BM - 1) / BM;
    P.nTiles = (cols + BN - 1) / BN;
    const long long items = (long long)P.itemsH * P.itemsW;
    const long long total = items * P.mTiles * P.nTiles;
    // Bands: at least four per die if there are enough items, at most one row of items each.  With few
    // items (under 16 per die) that deals the dies unequal shares -- 49 positions of 32 tiles dealt position
    // by position kept one die busy 25 % longer than the mean -- so bands are then two workgroups: every die
    // gets the same mix of positions whatever their number (79 -> 86 % on that layer; what the dies' caches
    // lose in locality did not show).  Not for KS-deconv with several classes: its class-major list wants
    // neighbouring positions on one die (bands of 16 or 64 workgroups instead of 32 cost 12 points on the
    // stride-2 benchmark layer).
    P.pairFlip = op_is_fwd(OP) || (P.sh == 1 && P.sw == 1);
    // (KS-deconv with several classes: two per die -- on the 16x16 stride-2 benchmark layer a band is then a whole
    // row of positions, every compute unit still holds one tile of each class, and the layer runs 2 points faster
    // than with half rows; smaller or larger bands put two tiles of the dearest class on one compute unit: -13 points)
    long long g = items / ((P.pairFlip ? 4 : 2) * kXcds);
    g = g < 1 ? 1 : (g > P.itemsW ? P.itemsW : g);
    long long bandBlocks = P.pairFlip && items < 16 * kXcds ? 2 : g * P.mTiles * P.nTiles;
    if (const char *t = tune("CKS_TUNE_BAND")) { if (atoi(t) > 0) bandBlocks = atoi(t); }   // tuning experiments only
    // whole rounds of 8 bands go to the dies band by band, the rest in 8 equal pieces (banded_work)
    const long long rounds = total / (bandBlocks * kXcds);
    const long long covered = rounds * kXcds * bandBlocks, remPerDie = (total - covered + kXcds - 1) / kXcds;
    // (whole groups of 32 workgroups per die: banded_work permutes within them; the surplus workgroups exit at once)
    const long long perDie = (rounds * bandBlocks + remPerDie + 31) / 32 * 32;
    const long long blocks = perDie * kXcds;
    if (!fits_i31(blocks)) return CKS_ERR_SHAPE;
    P.total = (int)total;
    P.fullSlots = (int)(rounds * bandBlocks); P.remPerDie = (int)remPerDie; P.covered = (int)covered;
    P.bandBlocks = (int)bandBlocks;
    P.dBand = make_fastdiv(P.bandBlocks);
    P.dNT = make_fastdiv(P.nTiles);
    P.dMT = make_fastdiv(P.mTiles);
    P.dItemsW = make_fastdiv(P.itemsW);
    P.dSh = make_fastdiv(P.sh);
    P.dSw = make_fastdiv(P.sw);
    P.pmodsH = P.ph % P.sh;
    P.pmodsW = P.pw % P.sw;
    {
        // output rows of a tile are one image apart
        const long long rowO = op_is_fwd(OP) ? (long long)P.OH * P.OW * P.OC : (long long)P.IH * P.IW * P.IC;
        P.bufStore = rowO * BM * 4 < (1LL << 31) && !tune("CKS_TUNE_NO_BUFFER_STORES");
    }
    const size_t lds = rowrun_lds_bytes<BM, BN>();
    // Fast loads need: 16-byte vectors, every run a whole number of 32-float
    // chunks (the run is a multiple of the contracted channel count), and the
    // tile's rows within 2 GiB of its first one.
    const long long kch = op_is_fwd(OP) ? P.IC : P.OC;
    const long long rowA = op_is_fwd(OP) ? (long long)P.IH * P.IW * P.IC : (long long)P.OH * P.OW * P.OC;
    const long long rowB = op_is_fwd(OP) ? (long long)P.FH * P.FW * P.IC : (long long)P.CHp * P.CWp * P.OC;
    // the default tiles also exist with their chunks loaded straight into LDS (same conditions as the fast loads)
    constexpr bool kHasDma = (BM == 64 && BN == 64 && WM == 2 && WN == 2) ||
                             (BM == 128 && BN == 32 && WM == 4 && WN == 1 && !op_b_k_major(OP));   // (the K-major filter tile is laid out for 64 columns)
    // (kernels that only a tuning build can select are not instantiated otherwise)
    const bool dma = kHasDma && !tune("CKS_TUNE_NO_LDS_DIRECT");
    constexpr bool kAlwaysDma = kHasDma && !kTuning;
    if (untrimmed) {
        if constexpr ((OP == OP_FWD || OP == OP_DECONV_W) && BM == 64 && BN == 64) {
            const bool fast = vec && kch % 32 == 0 && (rowA * BM + rowA) * 4 < (1LL << 31) && (OP == OP_DECONV_W || (rowB * BN + rowB) * 4 < (1LL << 31));
            if (fast)
                return launch(with_bools(kname("rowrun_gemm_dma", OP, BM, BN, WM, WN), false), rowrun_gemm_dma<OP, BM, BN, WM, WN, false>, P,
                              (int)blocks, rowrun_dma_lds_bytes<BM, BN>(), st);
        }
        return CKS_ERR_UNSUPPORTED;
    }
    if constexpr (op_b_k_major(OP)) {
        // the caller has checked deconv_in_place_ok / fwd_transposed_ok: only the fast-load variants exist
        if constexpr (kHasDma)
            if (dma) return launch(with_bools(kname("rowrun_gemm_dma", OP, BM, BN, WM, WN), true), rowrun_gemm_dma<OP, BM, BN, WM, WN>, P, (int)blocks, rowrun_dma_lds_bytes<BM, BN>(), st);
        if constexpr (!kAlwaysDma)
            return launch(kname("rowrun_gemm", OP, BM, BN, WM, WN, LOAD_FAST), rowrun_gemm<OP, BM, BN, WM, WN, LOAD_FAST>, P, (int)blocks, lds, st);
    } else {
        const bool fast = vec && kch % 32 == 0 && (rowA * BM + rowA) * 4 < (1LL << 31) && (rowB * BN + rowB) * 4 < (1LL << 31) &&
                          !tune("CKS_TUNE_NO_FAST_LOADS");
        if constexpr (kHasDma)
            if (fast && dma) return launch(with_bools(kname("rowrun_gemm_dma", OP, BM, BN, WM, WN), true), rowrun_gemm_dma<OP, BM, BN, WM, WN>, P, (int)blocks, rowrun_dma_lds_bytes<BM, BN>(), st);
        if constexpr (!kAlwaysDma)
            if (fast) return launch(kname("rowrun_gemm", OP, BM, BN, WM, WN, LOAD_FAST), rowrun_gemm<OP, BM, BN, WM, WN, LOAD_FAST>, P, (int)blocks, lds, st);
        if (vec) return launch(kname("rowrun_gemm", OP, BM, BN, WM, WN, LOAD_VEC), rowrun_gemm<OP, BM, BN, WM, WN, LOAD_VEC>, P, (int)blocks, lds, st);
        return launch(kname("rowrun_gemm", OP, BM, BN, WM, WN, LOAD_SCALAR), rowrun_gemm<OP, BM, BN, WM, WN, LOAD_SCALAR>, P, (int)blocks, lds, st);
    }
    return CKS_ERR_UNSUPPORTED;   // not reached
}

// KS-deconv can take its sub-kernels straight from the OHWI filter (no Stage 1 launch, no
// workspace) when the fast-load variant applies: whole 32-channel chunks of OC, 16-byte vectors,
// tile rows of dY within 2 GiB of the first (for the largest tile, 128 rows), the filter below 2 GiB.
bool deconv_in_place_ok(const Geo &g, const float *dY, const float *Wt)
{
    const long long rowA = (long long)g.OH * g.OW * g.OC, w = (long long)g.OC * g.FH * g.FW * g.C;
    return g.OC % 32 == 0 && g.C % 4 == 0 && aligned16(dY) && aligned16(Wt) && rowA * 129 * 4 < (1LL << 31) &&
           w * 4 < (1LL << 31) && !tune("CKS_TUNE_NO_FAST_LOADS") && !tune("CKS_TUNE_SPLIT_DECONV");
}

template <int OP>
int dispatch_rowrun(const RowRunParams &P, int rows, int cols, bool vec, hipStream_t st, bool untrimmed = false)
{
    const long long positions = (long long)P.itemsH * P.itemsW;
    // rows = batch, cols = output channels of this operator.  Measured on all
    // benchmark layers: once the K loop is free of vector-ALU work, 64x64 tiles
    // beat the larger ones by 5-15 points (more workgroups per compute unit, whose
    // load/store phases overlap each other's MFMA phases, and finer balance).
    int bm = 64;
    int bn = cols >= 48 ? 64 : 32;
    if (bn == 32) bm = 128;
    (void)positions;
#ifdef CKS_TUNING
    if (const char *t = tune("CKS_TUNE_ROWRUN")) sscanf(t, "%d,%d", &bm, &bn);
    if (bm == 128 && bn == 128) return launch_rowrun<OP, 128, 128, 2, 2>(P, rows, cols, vec, st);
    if (bm == 128 && bn == 64) return launch_rowrun<OP, 128, 64, 2, 2>(P, rows, cols, vec, st);
    if (bm == 64 && bn == 128) return launch_rowrun<OP, 64, 128, 2, 2>(P, rows, cols, vec, st);
#endif
    if (bm == 64 && bn == 64) return launch_rowrun<OP, 64, 64, 2, 2>(P, rows, cols, vec, st, untrimmed);
    return launch_rowrun<OP, 128, 32, 4, 1>(P, rows, cols, vec, st, untrimmed);
}

template <int OP>
RowRunParams rowrun_params(const Geo &g, const float *A, const float *B, float *Out)
{
    RowRunParams P{};
    P.A = A; P.B = B; P.Out = Out;
    P.N = g.N; P.IC = g.C; P.IH = g.H; P.IW = g.W; P.OC = g.OC; P.OH = g.OH; P.OW = g.OW;
    P.FH = g.FH; P.FW = g.FW; P.sh = g.sh; P.sw = g.sw; P.ph = g.ph; P.pw = g.pw;
    P.CHp = (g.FH + g.sh - 1) / g.sh;
    P.CWp = (g.FW + g.sw - 1) / g.sw;
    if (op_is_fwd(OP)) {
        P.itemsH = g.OH; P.itemsW = g.OW;
        P.rotH = ((g.ph + g.sh - 1) / g.sh) % g.OH;       // output rows whose window starts in the padding
        P.rotW = ((g.pw + g.sw - 1) / g.sw) % g.OW;
    } else {
        P.itemsH = g.H; P.itemsW = g.W;
        P.rotH = 0; P.rotW = 0;   // the class-major list is rotated class by class (class_major_index)
    }
    return P;
}

size_t split_bytes(int C, int OC, int FH, int FW, int sh, int sw)
{
    return sizeof(float) * (size_t)sh * sw * C * ((FH + sh - 1) / sh) * ((FW + sw - 1) / sw) * OC;
}

template <int MODE>
int launch_pack(const float *Wt, float *Out, int C, int OC, int FH, int FW, int sh, int sw, hipStream_t st)
{
    PackParams P{};
    P.W = Wt; P.Out = Out; P.IC = C; P.OC = OC; P.FH = FH; P.FW = FW; P.sh = sh; P.sw = sw;
    P.CHp = (FH + sh - 1) / sh;
    P.CWp = (FW + sw - 1) / sw;
    P.ocTiles = (OC + 31) / 32;
    P.icTiles = (C + 31) / 32;
    const long long slots = MODE == PACK_SPLIT ? (long long)sh * sw * P.CHp * P.CWp : (long long)FH * FW;
    const long long blocks = slots * P.ocTiles * P.icTiles;
    if (!fits_i31(blocks)) return CKS_ERR_SHAPE;
    return launch(kname("pack_filter", MODE), pack_filter<MODE>, P, (int)blocks, 0, st);
}

// ---------------------------------------------------------------- Sk-dilated

constexpr int kStripWgradGroups = kCUs;   // strip_wgrad: one workgroup (= one segment) per compute unit

// Few-channel geometries the strip kernels are instantiated for: 1 = 7x7 / stride 2 / 3 channels (ImageNet
// stems), 2 = 3x3 / stride 1 / 3 channels, 3 = 3x3 / stride 2 / 3 channels (small-image stems); 0 = none.
// All with the same stride and padding on both axes.
inline int strip_geometry(const Geo &g)
{
    const int FH = g.FH, FW = g.FW, C = g.C, s = g.sh;
    if (!g.same_on_both_axes() || C != 3 || FH != FW) return 0;
    if (FH == 7 && s == 2) return 1;
    if (FH == 3 && s == 1) return 2;
    if (FH == 3 && s == 2) return 3;
    return 0;
}

template <int FH, int FW, int IC, int S>
int launch_strip_fwd(const Geo &g, const float *X, const float *Wt, float *Y, hipStream_t st)
{
    using SG = StripGeo<FH, FW, IC, S>;
    StripFwdParams Q{};
    Q.X = X; Q.W = Wt; Q.Y = Y;
    Q.N = g.N; Q.IH = g.H; Q.IW = g.W; Q.OC = g.OC; Q.OH = g.OH; Q.OW = g.OW; Q.p = g.ph;
    Q.nBands = (g.OW + 15) / 16;
    Q.nRowTiles = (g.OH + 3) / 4;
    Q.nT = (g.OC + 63) / 64;
    const long long tiles = (long long)g.N * Q.nBands * Q.nRowTiles;
    if (!fits_i31(tiles * Q.nT)) return CKS_ERR_SHAPE;
    Q.tiles = (int)tiles;
    int per_cu = 2;   // workgroups per compute unit
    if (const char *t = tune("CKS_TUNE_STRIP_FWD")) per_cu = atoi(t) > 0 ? atoi(t) : 2;   // tuning experiments only
    const int groups = Q.tiles < per_cu * kCUs ? Q.tiles : per_cu * kCUs;
    Q.tilesPerBlock = (Q.tiles + groups - 1) / groups;
    const int blocks = ((Q.tiles + Q.tilesPerBlock - 1) / Q.tilesPerBlock) * Q.nT;
    return launch(kname("strip_fwd", FH, FW, IC, S), strip_fwd<FH, FW, IC, S>, Q, blocks, SG::lds_bytes(), st, kStripThreads);
}

template <int FH, int FW, int IC, int S>
int launch_strip_wgrad(const Geo &g, int GZ, const float *X, const float *dY, float *part, bool veca, hipStream_t st)
{
    StripWgradParams Q{};
    Q.X = X; Q.dY = dY; Q.part = part;
    Q.N = g.N; Q.IH = g.H; Q.IW = g.W; Q.OC = g.OC; Q.OH = g.OH; Q.OW = g.OW; Q.p = g.ph;
    Q.nBands = (g.OW + 15) / 16;
    Q.nRowTiles = (g.OH + 3) / 4;
    Q.tiles = g.N * Q.nBands * Q.nRowTiles;
    Q.tilesPerBlock = (Q.tiles + GZ - 1) / GZ;
    const size_t lds = strip_wgrad_lds_bytes<FH, FW, IC, S>();
    if (veca) return launch(with_bools(kname("strip_wgrad", FH, FW, IC, S), true), strip_wgrad<FH, FW, IC, S, true>, Q, GZ, lds, st, kStripThreads);
    return launch(with_bools(kname("strip_wgrad", FH, FW, IC, S), false), strip_wgrad<FH, FW, IC, S, false>, Q, GZ, lds, st, kStripThreads);
}

struct WgradPlan {
    int patch;    // 0: one tile per filter tap (pixel_gemm); 1..3: all taps in one tile (patch_gemm); 4: strip_wgrad
    int variant, bm, bn, mTiles, nTiles, GZ;
};

// Tile variants of pixel_gemm: {BM, BN, KC, WAVES_M, WAVES_N, WAVES_K}
constexpr int kWgradVariants[][6] = {
    {128, 128, 16, 2, 2, 1},  // 0
    {128, 64, 32, 2, 1, 2},   // 1
    {64, 128, 32, 1, 2, 2},   // 2
    {64, 64, 32, 1, 1, 4},    // 3
    {64, 64, 16, 2, 2, 1},    // 4
    {128, 64, 16, 2, 2, 1},   // 5
    {64, 128, 16, 2, 2, 1},   // 6
};

// G_Z (Section IV.C: the number of segments trades parallelism against the
// memory for partial sums) is derived from the compute-unit count, see below.
// Segments (G_Z of Section IV.C's map-reduce) for `tiles` output tiles over K pixels.
long long wgrad_segments(long long tiles, long long K)
{
    // Just under four workgroups per compute unit (measured: 1008 workgroups beat 1152 by 2-4 points,
    // a fifth workgroup on half of the compute units costs more than the others' idle eighth), an
    // even number of segments (odd counts lose 5 points: the workgroups are dealt to the 8 dies in
    // contiguous ranges of segments), segments of at least 256 pixels; never fewer than 8 segments
    // while that leaves at most 16 workgroups per compute unit (8 segments beat 7 or 9 by 10-15 %).
    long long gz = 4LL * kCUs / tiles;
    if (gz >= kXcds) gz &= ~1LL;
    else if (tiles * kXcds <= 16LL * kCUs) gz = kXcds;
    if (tiles * kXcds > 16LL * kCUs) {
        // Many tiles (> 2 per compute unit): still up to four segments of at least 1024 pixels (eight
        // up to 1024 tiles).  The finer grain evens out the compute units' shares and keeps a segment's
        // X / dY rows in L2 while all its tiles use them (measured on 512-channel 5x5 layers: 4
        // segments 74-85 % of peak, one segment 57-69 %; on 576 tiles with 12544 pixels: 8 segments
        // 88.8 %, 4 segments 85.7 %).
        const long long most = tiles <= 1024 ? 8 : 4;
        gz = K / 1024 < most ? K / 1024 : most;
    }
    while (gz > 1 && K / gz < 256) gz = gz > kXcds ? gz - kXcds : gz / 2;
    return gz < 1 ? 1 : gz;
}

WgradPlan plan_wgrad(const Geo &g)
{
    WgradPlan w;
    w.patch = 0;
    const char *tw = tune("CKS_TUNE_WGRAD");   // "variant[,G_Z]": tuning experiments only
    // Few input channels: a per-tap tile would be narrower than an MFMA block.
    // Put the whole filter patch (J = FH*FW*IC columns) into one tile if it
    // fits 5, 10 or 18 column blocks without wasting more than 30 % of them.
    const long long J = (long long)g.FH * g.FW * g.C;
    // image stems: input strip in LDS (strip_wgrad), one segment per workgroup
    // (an image of X and one of dY, plus a tile's rows below it, are each addressed with 31 bits of bytes)
    if (strip_geometry(g) && g.OC <= 64 && (long long)g.H * g.W * g.C * 4 < (1LL << 31) &&
        ((long long)g.OH + 4) * g.OW * g.OC * 4 < (1LL << 31) && !tw && !tune("CKS_TUNE_NO_STRIP_WGRAD")) {
        const long long tiles = (long long)g.N * ((g.OW + 15) / 16) * ((g.OH + 3) / 4);
        if (fits_i31(tiles)) {
            w.patch = 4;
            w.variant = -1;
            w.bm = 64; w.bn = 160;
            w.mTiles = 1; w.nTiles = 1;
            const int groups = tiles < kStripWgradGroups ? (int)tiles : kStripWgradGroups;
            const int per = (int)((tiles + groups - 1) / groups);
            w.GZ = (int)((tiles + per - 1) / per);
            return w;
        }
    }
    if (g.C < 48 && J <= 576 && !(tw && tw[0] == 't')) {
        const int nb = J <= 160 ? 5 : (J <= 320 ? 10 : 18);
        if (10 * J >= 7 * 32 * nb) {
            w.patch = nb == 5 ? 1 : (nb == 10 ? 2 : 3);
            w.variant = -1;
            w.bm = 64; w.bn = 32 * nb;
            w.mTiles = (g.OC + 63) / 64; w.nTiles = 1;
            const long long K = (long long)g.N * g.OH * g.OW;
            // workgroups per compute unit that fit its LDS: one for the 18-block tile, else two
            long long gz = ((w.patch == 3 ? 1LL : 2LL) * kCUs + w.mTiles - 1) / w.mTiles;
            gz = gz < K / 256 ? gz : K / 256;
            if (tw && tw[0] == 'p') {
                const int z = atoi(tw + 1);
                if (z > 0) gz = z;
            }
            if (gz < 1) gz = 1;
            w.GZ = (int)gz;
            return w;
        }
    }
    // 64-wide channel tiles; 128 output channels per tile only for a middling number of tiles
    // and a long contraction axis (measured: 128x128 tiles lose 5-8 points on every layer, 128x64
    // gain 3 on 576 tiles with 12544 pixels, lose 4 on 576 tiles with 4096 pixels or on 1600 tiles)
    const long long tiles64 = (long long)g.FH * g.FW * ((g.OC + 63) / 64) * ((g.C + 63) / 64);
    // The 64x64 tile also exists with its chunks loaded straight into LDS (whole chunks of 32 images, 16-byte
    // vectors), which is worth more than the wider tile (576 tiles, 12544 pixels: 88.8 against 87.5 %; 400
    // tiles: +5 points) -- unless its workgroups would come to between 4 and 8 per compute unit, where the
    // uneven shares cost more (144 tiles: 1152 workgroups 69 %, the wider tile's 1008 workgroups 79 %).
    const long long K = (long long)g.N * g.OH * g.OW;
    const bool lds_direct = g.N % 32 == 0 && g.C % 4 == 0 && g.OC % 4 == 0;
    const long long wgs64 = tiles64 * wgrad_segments(tiles64, K);
    const bool prefer64 = lds_direct && (wgs64 <= 4LL * kCUs || wgs64 >= 8LL * kCUs);
    w.variant = (!prefer64 && g.OC >= 96 && tiles64 > 128 && tiles64 <= 1024 && K >= 8192) ? 5 : 4;
    long long gz_override = 0;
    if (const char *t = tw) {
        int v = -1, z = 0;
        if (t[0] == 't') ++t;
        if (sscanf(t, "%d,%d", &v, &z) >= 1 && v >= 0 && v < 7) w.variant = v;
        gz_override = z;
    }
    w.bm = kWgradVariants[w.variant][0];
    w.bn = kWgradVariants[w.variant][1];
    w.mTiles = (g.OC + w.bm - 1) / w.bm;
    w.nTiles = (g.C + w.bn - 1) / w.bn;
    const long long tiles = (long long)g.FH * g.FW * w.mTiles * w.nTiles;
    long long gz = wgrad_segments(tiles, K);
    if (gz_override > 0) gz = gz_override;
    if (gz < 1) gz = 1;
    if (gz > 512) gz = 512;
    w.GZ = (int)gz;
    return w;
}

template <int BM, int BN, int KC, int WM, int WN, int WK>
int launch_pixel(PixelGemmParams P, bool veca, bool vecb, hipStream_t st, bool untrimmed = false)
{
    const size_t lds = pixel_lds_bytes<BM, BN, KC>();
    const int blocks = P.perXcd * kXcds;
    P.dNT = make_fastdiv(P.nTiles);
    P.dMT = make_fastdiv(P.mTiles);
    P.dTaps = make_fastdiv(P.FH * P.FW);
    P.dFW = make_fastdiv(P.FW);
    P.dSh = make_fastdiv(P.sh);
    P.dSw = make_fastdiv(P.sw);
    P.dGZ = make_fastdiv(P.GZ);
    P.dNC = make_fastdiv(P.N / KC > 0 ? P.N / KC : 1);
    P.bufStore = P.sliceElems * 4 < (1LL << 31) && !tune("CKS_TUNE_NO_BUFFER_STORES");
    // batch-inner ordering with scalar chunk offsets (see pixel_gemm_fast)
    // (its ceiling divisions shift their numerators by (FH + FW) strides: keep that within 31 bits)
    const long long smax = P.sh > P.sw ? P.sh : P.sw;
    const bool fast = veca && vecb && P.N % KC == 0 && (long long)P.N * P.IH * P.IW * P.IC * 4 < (1LL << 31) &&
                      (long long)P.N * P.OH * P.OW * P.OC * 4 < (1LL << 31) &&
                      (P.FH + P.FW + 2) * smax + P.IH + P.IW + P.FH + P.FW < (1LL << 30) && !tune("CKS_TUNE_NO_FAST_LOADS");
    if constexpr (BM == 64 && BN == 64 && KC == 16 && WM == 2 && WN == 2 && WK == 1) {
        // the default tile also exists with its chunks (32 images) loaded straight into LDS
        if (fast && P.N % kPixelDmaKC == 0 && !tune("CKS_TUNE_NO_LDS_DIRECT")) {
            P.dNC = make_fastdiv(P.N / kPixelDmaKC);
            if (untrimmed) return launch(with_bools(kname("pixel_gemm_dma"), false), pixel_gemm_dma<false>, P, blocks, pixel_dma_lds_bytes(), st);
            return launch(with_bools(kname("pixel_gemm_dma"), true), pixel_gemm_dma<true>, P, blocks, pixel_dma_lds_bytes(), st);
        }
    }
    if (untrimmed) return CKS_ERR_UNSUPPORTED;   // Algorithm 3 exists for the tile loaded straight into LDS only
    if (fast) return launch(kname("pixel_gemm_fast", BM, BN, KC, WM, WN, WK), pixel_gemm_fast<BM, BN, KC, WM, WN, WK>, P, blocks, lds, st);
    if (veca && vecb) return launch(with_bools(kname("pixel_gemm", BM, BN, KC, WM, WN, WK), true, true), pixel_gemm<BM, BN, KC, WM, WN, WK, true, true>, P, blocks, lds, st);
    if (veca) return launch(with_bools(kname("pixel_gemm", BM, BN, KC, WM, WN, WK), true, false), pixel_gemm<BM, BN, KC, WM, WN, WK, true, false>, P, blocks, lds, st);
    if (vecb) return launch(with_bools(kname("pixel_gemm", BM, BN, KC, WM, WN, WK), false, true), pixel_gemm<BM, BN, KC, WM, WN, WK, false, true>, P, blocks, lds, st);
    return launch(with_bools(kname("pixel_gemm", BM, BN, KC, WM, WN, WK), false, false), pixel_gemm<BM, BN, KC, WM, WN, WK, false, false>, P, blocks, lds, st);
}

template <int WM, int WN, int WK, int NBW, int KC>
int launch_patch(PatchGemmParams P, bool veca, bool vecb, hipStream_t st)
{
    const size_t lds = patch_lds_bytes<WM, WN, NBW, KC>();
    const int blocks = P.perXcd * kXcds;
    // batch-inner ordering with scalar chunk offsets (see patch_gemm_fast)
    const bool fast = veca && P.N % KC == 0 && (long long)P.N * P.IH * P.IW * P.IC * 4 < (1LL << 31) &&
                      (long long)P.N * P.OH * P.OW * P.OC * 4 < (1LL << 31) && !tune("CKS_TUNE_NO_FAST_LOADS");
    // (with 4-byte items, i.e. IC not a multiple of 4, the pixel order coalesces better: neighbouring patches overlap)
    if (fast && vecb) return launch(with_bools(kname("patch_gemm_fast", WM, WN, WK, NBW, KC), true), patch_gemm_fast<WM, WN, WK, NBW, KC, true>, P, blocks, lds, st);
    if (veca && vecb) return launch(with_bools(kname("patch_gemm", WM, WN, WK, NBW, KC), true, true), patch_gemm<WM, WN, WK, NBW, KC, true, true>, P, blocks, lds, st);
    if (veca) return launch(with_bools(kname("patch_gemm", WM, WN, WK, NBW, KC), true, false), patch_gemm<WM, WN, WK, NBW, KC, true, false>, P, blocks, lds, st);
    if (vecb) return launch(with_bools(kname("patch_gemm", WM, WN, WK, NBW, KC), false, true), patch_gemm<WM, WN, WK, NBW, KC, false, true>, P, blocks, lds, st);
    return launch(with_bools(kname("patch_gemm", WM, WN, WK, NBW, KC), false, false), patch_gemm<WM, WN, WK, NBW, KC, false, false>, P, blocks, lds, st);
}


int64_t useful_macs(const Geo &g)
{
    auto S = [](int I, int F, int O, int s, int p) {
        int64_t t = 0;
        for (int o = 0; o < O; ++o) {
            int i0 = o * s - p;
            int lo = -i0 > 0 ? -i0 : 0, hi = I - i0 < F ? I - i0 : F;
            if (hi > lo) t += hi - lo;
        }
        return t;
    };
    return (int64_t)g.N * g.C * g.OC * S(g.H, g.FH, g.OH, g.sh, g.ph) * S(g.W, g.FW, g.OW, g.sw, g.pw);
}

// Few-channel KS-deconv (tap-stationary GEMM + LDS composing): geometry limits of scatter_deconv.
struct ScatterPlan {
    bool ok;
    int NB;             // 16-column blocks (template parameter to use)
    ScatterDeconvParams P;
    int blocks;
    size_t headBytes, rowheadBytes;   // side buffers in the workspace, in this order
};

ScatterPlan plan_scatter(const Geo &g)
{
    ScatterPlan S{};
    if (!g.same_on_both_axes()) return S;
    const int N = g.N, C = g.C, H = g.H, W = g.W, OC = g.OC, FH = g.FH, FW = g.FW, stride = g.sh, padding = g.ph;
    const int J = FH * FW * C, sic = stride * C;
    if (C >= 8 || OC > 64 || OC % 4 != 0 || J > 160) return S;
    if ((long long)H * W * C * 4 >= (1LL << 31)) return S;   // an image is one raw buffer
    ScatterDeconvParams &P = S.P;
    P.N = N; P.IC = C; P.IH = H; P.IW = W; P.OC = OC; P.OH = g.OH; P.OW = g.OW;
    P.FH = FH; P.FW = FW; P.s = stride; P.p = padding;
    P.nBands = (g.OW + 15) / 16;
    P.nTiles = (g.OH + 3) / 4;
    P.OVF = (FW > stride ? FW - stride : 0) * C;
    P.SW = 16 * sic + P.OVF;
    const int touched = (15 * stride + FW) * C;
    const int rest = (W + padding) * C - 16 * (P.nBands - 1) * sic;   // dX floats from the last band's start to the row's end
    P.SWlast = touched > rest ? touched : rest;
    if (P.SW > kScatterRP || P.SWlast > kScatterRP || touched > kScatterRP) return S;
    if ((FW + stride - 1) / stride > kScatterMaxTB || (FH + stride - 1) / stride > kScatterMaxTB) return S;
    P.slots = 8 + (FH - 1) / stride;   // rows being composed (4) + rows being produced (4) + history
    const int rowsEnd = (4 * P.nTiles - 1) * stride + FH, rowsImg = H + padding;
    P.nFlush = ((rowsEnd > rowsImg ? rowsEnd : rowsImg) + 4 * stride - 1) / (4 * stride);
    P.KP = (OC + 15) / 16 * 16;
    S.NB = J <= 64 ? 4 : 10;
    if (scatter_deconv_lds_bytes(S.NB, P.slots, FH) > 160 * 1024) return S;
    if (!fits_i31((long long)N * P.nBands * H) || P.OVF > kThreads) return S;   // add_heads indexes rows with 32 bits
    const long long steps = (long long)N * P.nBands * P.nTiles;
    if (!fits_i31(steps)) return S;
    P.steps = (int)steps;
    P.HR = FH > stride ? FH - stride : 0;
    // One workgroup per compute unit, each with an equal run of consecutive sweep steps; a run that
    // starts inside a band shares HR dX rows with the run before it (rowhead).  Two such row heads of
    // neighbouring bands must not meet in a dX row (their column overlap would be added to twice at
    // once): if they would, every workgroup gets whole bands instead.
    P.stepsPerBlock = (int)((steps + kCUs - 1) / kCUs);
    if (P.stepsPerBlock % P.nTiles != 0) {
        bool clash = false;
        int prevBand = -2, prevT0 = 0;
        const int blocks = (P.steps + P.stepsPerBlock - 1) / P.stepsPerBlock;
        for (int b = 1; b < blocks && !clash; ++b) {
            const long long u0 = (long long)b * P.stepsPerBlock;
            const int band = (int)(u0 / P.nTiles), t0 = (int)(u0 % P.nTiles);
            if (t0 == 0) continue;
            if (band == prevBand) clash = true;   // two heads in one band: not handled
            if (band == prevBand + 1 && band % P.nBands != 0) {
                const int a = prevT0 * 4 * stride, c2 = t0 * 4 * stride;
                if (a < c2 + P.HR && c2 < a + P.HR) clash = true;
            }
            prevBand = band; prevT0 = t0;
        }
        if (clash || P.HR == 0 || P.stepsPerBlock < P.nTiles) P.stepsPerBlock = (P.stepsPerBlock + P.nTiles - 1) / P.nTiles * P.nTiles;
    }
    S.blocks = (P.steps + P.stepsPerBlock - 1) / P.stepsPerBlock;
    S.headBytes = ((size_t)N * (P.nBands - 1) * H * P.OVF * sizeof(float) + 255) / 256 * 256;
    S.rowheadBytes = P.stepsPerBlock % P.nTiles != 0 ? (size_t)S.blocks * P.HR * kScatterRP * sizeof(float) : 0;
    S.ok = true;
    return S;
}

// Image-stem KS-deconv on the 4x4x1 matrix instruction (sweep_deconv): the shapes it is built for.
// 0: none; 1: 7x7 stride 2 padding 3 on the width, 3 input channels, 64 output channels.
int sweep_geometry(const Geo &g)
{
    if (tune("CKS_TUNE_NO_SWEEP")) return 0;
    if (g.sh != g.sw) return 0;
    // the two tensors are one raw buffer each, and rows of all windows are counted with 31 bits
    if ((long long)g.N * g.OH * g.OW * g.OC * 4 >= (1LL << 31) || (long long)g.N * g.H * g.W * g.C * 4 >= (1LL << 31)) return 0;
    if (g.FH == 7 && g.FW == 7 && g.sh == 2 && g.pw == 3 && g.C == 3 && g.OC == 64) return 1;
    return 0;
}

template <int FH, int FW, int S, int PW, int IC, int OCQ>
int launch_sweep_deconv(const Geo &g, const float *dY, const float *Wt, float *dX, hipStream_t st)
{
    SweepDeconvParams P{};
    P.dY = dY; P.W = Wt; P.dX = dX;
    P.N = g.N; P.OH = g.OH; P.OW = g.OW; P.OC = g.OC; P.IH = g.H; P.IW = g.W; P.ph = g.ph;
    const int need = (g.W + S - 1) / S;
    P.OWv = need > g.OW ? need : g.OW;
    using G = SweepShape<FH, FW, S, PW, IC, OCQ>;
    const long long line = (long long)g.N * P.OWv;
    const long long nWin = (line + G::ADV - 1) / G::ADV, rows = nWin * g.OH;
    if (!fits_i31(rows) || !fits_i31(nWin * 64)) return CKS_ERR_SHAPE;
    P.nWin = (int)nWin;
    // one wave per SIMD, every wave an equal run of consecutive rows
    const long long waves = rows < 4LL * kCUs ? rows : 4LL * kCUs;
    P.per = (int)(rows / waves); P.rem = (int)(rows % waves);
    P.dOWv = make_fastdiv(P.OWv); P.dOH = make_fastdiv(g.OH);
    const int blocks = (int)((waves + 3) / 4);
    return launch(kname("sweep_deconv", FH, FW, S, PW, IC, OCQ), sweep_deconv<FH, FW, S, PW, IC, OCQ>, P, blocks, 0, st);
}

size_t deconv_workspace(const Geo &g)
{
    const size_t split = split_bytes(g.C, g.OC, g.FH, g.FW, g.sh, g.sw);
    const ScatterPlan S = plan_scatter(g);
    return S.ok && S.headBytes + S.rowheadBytes > split ? S.headBytes + S.rowheadBytes : split;
}

size_t wgrad_workspace(const Geo &g)
{
    const WgradPlan w = plan_wgrad(g);
    return w.GZ > 1 ? sizeof(float) * (size_t)w.GZ * g.OC * g.FH * g.FW * g.C : 0;
}

int conv_fwd(const Geo &g, const float *X, const float *Wt, float *Y, hipStream_t st)
{
    if (!X || !Wt || !Y) return CKS_ERR_NULL;
    const int N = g.N, C = g.C, H = g.H, W = g.W, OC = g.OC, FH = g.FH, FW = g.FW;
    // image stems: input strip in LDS, addressing known at compile time
    // (an image of X and one of Y are each addressed with 31 bits of bytes)
    if ((long long)H * W * C * 4 < (1LL << 31) && (long long)g.OH * g.OW * OC * 4 < (1LL << 31) && !tune("CKS_TUNE_NO_STRIP_FWD")) {
        switch (strip_geometry(g)) {
            case 1: return launch_strip_fwd<7, 7, 3, 2>(g, X, Wt, Y, st);
            case 2: return launch_strip_fwd<3, 3, 3, 1>(g, X, Wt, Y, st);
            case 3: return launch_strip_fwd<3, 3, 3, 2>(g, X, Wt, Y, st);
            default: break;
        }
    }
    // Other layers with very few input channels: one GEMM over all pixels with the
    // whole filter patch as contraction axis and the filter resident in LDS.
    const int KP = (FH * FW * C + 15) / 16 * 16;
    if (C < 8 && KP <= kPatchFwdMaxKP && (long long)N * H * W * C * 4 < (1LL << 31) &&
        (long long)N * g.OH * g.OW * OC * 4 < (1LL << 31) && !tune("CKS_TUNE_NO_PATCH_FWD")) {
        PatchFwdParams Q{};
        Q.X = X; Q.W = Wt; Q.Y = Y;
        Q.N = N; Q.IC = C; Q.IH = H; Q.IW = W; Q.OC = OC; Q.OH = g.OH; Q.OW = g.OW;
        Q.FH = FH; Q.FW = FW; Q.sh = g.sh; Q.sw = g.sw; Q.ph = g.ph; Q.pw = g.pw;
        Q.KP = KP;
        Q.nT = (OC + 63) / 64;
        Q.mTiles = (int)(((long long)N * g.OH * g.OW + 63) / 64);
        const int groups = Q.mTiles < kCUs ? Q.mTiles : kCUs;    // one workgroup per compute unit (LDS)
        Q.tilesPerBlock = (Q.mTiles + groups - 1) / groups;
        const long long blocks = (long long)((Q.mTiles + Q.tilesPerBlock - 1) / Q.tilesPerBlock) * Q.nT;
        if (!fits_i31(blocks)) return CKS_ERR_SHAPE;
        return launch(kname("patch_fwd"), patch_fwd, Q, (int)blocks, patch_fwd_lds_bytes(KP), st, kPatchFwdThreads);
    }
    const bool vec = (C % 4 == 0) && aligned16(X) && aligned16(Wt);
    return dispatch_rowrun<OP_FWD>(rowrun_params<OP_FWD>(g, X, Wt, Y), N, OC, vec, st);
}

// ConvV2 on the transposed filter Wtt[FH][FW][C][OC] (Section IV.A, last paragraph).  For one tap the filter
// is then a K x N matrix (ic x oc) with N contiguous; its 32 x 64 chunks go to LDS as they lie.  Needs whole
// 32-channel chunks of C, 16-byte vectors, tile rows of X within 2 GiB of the first, the filter below 2 GiB.
bool fwd_transposed_ok(const Geo &g, const float *X, const float *Wtt)
{
    const long long rowA = (long long)g.H * g.W * g.C, w = (long long)g.OC * g.FH * g.FW * g.C;
    return g.C % 32 == 0 && g.OC % 4 == 0 && aligned16(X) && aligned16(Wtt) && rowA * 129 * 4 < (1LL << 31) && w * 4 < (1LL << 31);
}

int conv_fwd_transposed(const Geo &g, const float *X, const float *Wtt, float *Y, hipStream_t st)
{
    if (!X || !Wtt || !Y) return CKS_ERR_NULL;
    if (!fwd_transposed_ok(g, X, Wtt)) return CKS_ERR_UNSUPPORTED;
    return dispatch_rowrun<OP_FWD_T>(rowrun_params<OP_FWD_T>(g, X, Wtt, Y), g.N, g.OC, true, st);
}

// The operators with filter trimming switched off (Section IV: the plain convolution that ConvV2 improves on, and
// KS-deconv as Algorithm 2 states it before the V2 of Algorithm 2B), for the ablation.  Same kernels, same work
// lists; every position contracts its whole window and the cells outside the data are read as zeros.
int conv_fwd_untrimmed(const Geo &g, const float *X, const float *Wt, float *Y, hipStream_t st)
{
    if (!X || !Wt || !Y) return CKS_ERR_NULL;
    if (g.OC < 48 || g.C % 4 != 0 || !aligned16(X) || !aligned16(Wt)) return CKS_ERR_UNSUPPORTED;
    return dispatch_rowrun<OP_FWD>(rowrun_params<OP_FWD>(g, X, Wt, Y), g.N, g.OC, true, st, true);
}

int deconv_untrimmed(const Geo &g, const float *dY, const float *Wt, float *dX, hipStream_t st)
{
    if (!dY || !Wt || !dX) return CKS_ERR_NULL;
    if (g.C < 48 || !deconv_in_place_ok(g, dY, Wt)) return CKS_ERR_UNSUPPORTED;
    return dispatch_rowrun<OP_DECONV_W>(rowrun_params<OP_DECONV_W>(g, dY, Wt, dX), g.N, g.C, true, st, true);
}

int kernel_split(const float *Wt, float *Cs, int C, int OC, int FH, int FW, int sh, int sw, hipStream_t st)
{
    if (C <= 0 || OC <= 0 || FH <= 0 || FW <= 0 || sh < 1 || sw < 1 || sh > (1 << 20) || sw > (1 << 20)) return CKS_ERR_SHAPE;
    if (!fits_i31((long long)(split_bytes(C, OC, FH, FW, sh, sw) / sizeof(float)))) return CKS_ERR_SHAPE;
    if (!Wt || !Cs) return CKS_ERR_NULL;
    return launch_pack<PACK_SPLIT>(Wt, Cs, C, OC, FH, FW, sh, sw, st);
}

int deconv_presplit(const Geo &g, const float *dY, const float *Cs, float *dX, hipStream_t st)
{
    if (!fits_i31((long long)(split_bytes(g.C, g.OC, g.FH, g.FW, g.sh, g.sw) / sizeof(float)))) return CKS_ERR_SHAPE;
    if (!dY || !Cs || !dX) return CKS_ERR_NULL;
    const bool vec = (g.OC % 4 == 0) && aligned16(dY) && aligned16(Cs);
    return dispatch_rowrun<OP_DECONV>(rowrun_params<OP_DECONV>(g, dY, Cs, dX), g.N, g.C, vec, st);
}

int deconv(const Geo &g, const float *dY, const float *Wt, float *dX, void *ws, size_t ws_bytes, hipStream_t st)
{
    const int N = g.N, C = g.C, H = g.H, W = g.W, OC = g.OC, FH = g.FH, FW = g.FW;
    if (!fits_i31((long long)(split_bytes(C, OC, FH, FW, g.sh, g.sw) / sizeof(float)))) return CKS_ERR_SHAPE;
    if (!dY || !Wt || !dX) return CKS_ERR_NULL;
    // (the variant that reads the filter in place uses no workspace: it may then be NULL)
    // (its 16-byte loads want dY aligned; it uses no workspace)
    if (sweep_geometry(g) == 1 && aligned16(dY)) return launch_sweep_deconv<7, 7, 2, 3, 3, 4>(g, dY, Wt, dX, st);
    const bool have_ws = ws && ws_bytes >= deconv_workspace(g);
    ScatterPlan S = plan_scatter(g);
    if (S.ok && !have_ws) return CKS_ERR_WORKSPACE;
    if (S.ok && aligned16(dY) && aligned16(ws) && !tune("CKS_TUNE_NO_SCATTER")) {
        const int stride = g.sh, padding = g.ph;   // the same on both axes (plan_scatter)
        S.P.dY = dY; S.P.W = Wt; S.P.dX = dX; S.P.head = (float *)ws;
        S.P.rowhead = (float *)((char *)ws + S.headBytes);
        const bool stem = FH == 7 && FW == 7 && C == 3 && stride == 2 && OC == 64;
        if (stem) S.P.slots = kScatterStemSlots;
        const size_t lds = scatter_deconv_lds_bytes(S.NB, S.P.slots, FH);
        int rc;
        if (S.NB == 4) rc = launch(with_bools(kname("scatter_deconv", 4), false), scatter_deconv<4, false>, S.P, S.blocks, lds, st, kScatterThreads);
        else if (stem) rc = launch(with_bools(kname("scatter_deconv", 10), true), scatter_deconv<10, true>, S.P, S.blocks, lds, st, kScatterStemThreads);
        else rc = launch(with_bools(kname("scatter_deconv", 10), false), scatter_deconv<10, false>, S.P, S.blocks, lds, st, kScatterThreads);
        if (rc != CKS_OK) return rc;
        const bool bandPart = S.P.nBands > 1 && S.P.OVF > 0;
        if (bandPart || S.rowheadBytes) {
            HeadsParams B{};
            B.head = (const float *)ws; B.rowhead = S.rowheadBytes ? S.P.rowhead : nullptr; B.dX = dX;
            B.N = N; B.IC = C; B.IH = H; B.IW = W; B.s = stride; B.p = padding; B.nBands = S.P.nBands; B.nTiles = S.P.nTiles;
            B.OVF = S.P.OVF; B.SW = S.P.SW; B.SWlast = S.P.SWlast; B.HR = S.P.HR; B.stepsPerBlock = S.P.stepsPerBlock; B.blocks = S.blocks;
            while ((kHeadFloats << B.xwShift) < S.P.OVF) ++B.xwShift;   // OVF <= 256 floats (plan_scatter): at most a workgroup
            B.dIH = make_fastdiv(H); B.dBandsLeft = make_fastdiv(S.P.nBands > 1 ? S.P.nBands - 1 : 1); B.dSteps = make_fastdiv(S.P.stepsPerBlock);
            if (bandPart) {
                const long long rows = (long long)N * (S.P.nBands - 1) * H;   // plan_scatter has checked that this fits 31 bits
                const long long rpb = kThreads >> B.xwShift;
                B.rows = (int)rows;
                B.bandBlocks = (int)((rows + rpb - 1) / rpb);
            }
            const int per = kThreads / kScatterRP;
            const long long rowBlocks = S.rowheadBytes ? ((long long)S.blocks * S.P.HR + per - 1) / per : 0;
            if (!fits_i31(B.bandBlocks + rowBlocks)) return CKS_ERR_SHAPE;
            rc = launch(kname("add_heads"), add_heads, B, (int)(B.bandBlocks + rowBlocks), 0, st);
        }
        return rc;
    }
    if (deconv_in_place_ok(g, dY, Wt))
        return dispatch_rowrun<OP_DECONV_W>(rowrun_params<OP_DECONV_W>(g, dY, Wt, dX), N, C, true, st);
    if (!have_ws) return CKS_ERR_WORKSPACE;
    int rc = kernel_split(Wt, (float *)ws, C, OC, FH, FW, g.sh, g.sw, st);
    if (rc != CKS_OK) return rc;
    return deconv_presplit(g, dY, (const float *)ws, dX, st);
}

int wgrad_partials(const Geo &g, const float *X, const float *dY, float *part, hipStream_t st, bool untrimmed = false)
{
    if (!X || !dY || !part) return CKS_ERR_NULL;
    const int N = g.N, C = g.C, H = g.H, W = g.W, OC = g.OC, FH = g.FH, FW = g.FW;
    const WgradPlan w = plan_wgrad(g);
    if (untrimmed && (w.patch || w.variant != 4)) return CKS_ERR_UNSUPPORTED;
    const bool veca = (OC % 4 == 0) && aligned16(dY);
    const bool vecb = (C % 4 == 0) && aligned16(X);
    if (w.patch == 4) {
        switch (strip_geometry(g)) {
            case 1: return launch_strip_wgrad<7, 7, 3, 2>(g, w.GZ, X, dY, part, veca, st);
            case 2: return launch_strip_wgrad<3, 3, 3, 1>(g, w.GZ, X, dY, part, veca, st);
            case 3: return launch_strip_wgrad<3, 3, 3, 2>(g, w.GZ, X, dY, part, veca, st);
            default: return CKS_ERR_UNSUPPORTED;
        }
    }
    if (w.patch) {
        PatchGemmParams Q{};
        Q.X = X; Q.dY = dY; Q.Out = part;
        Q.N = N; Q.IC = C; Q.IH = H; Q.IW = W; Q.OC = OC; Q.OH = g.OH; Q.OW = g.OW;
        Q.FH = FH; Q.FW = FW; Q.sh = g.sh; Q.sw = g.sw; Q.ph = g.ph; Q.pw = g.pw;
        Q.GZ = w.GZ; Q.mTiles = w.mTiles;
        Q.total = w.GZ * w.mTiles;
        Q.perXcd = (Q.total + kXcds - 1) / kXcds;
        Q.sliceElems = (long)OC * FH * FW * C;
        switch (w.patch) {
            case 1: return launch_patch<2, 1, 2, 5, 32>(Q, veca, vecb, st);
            case 2: return launch_patch<2, 2, 1, 5, 16>(Q, veca, vecb, st);
            default: return launch_patch<2, 2, 1, 9, 16>(Q, veca, vecb, st);
        }
    }
    const long long total = (long long)w.GZ * FH * FW * w.mTiles * w.nTiles;
    if (!fits_i31(total + kXcds)) return CKS_ERR_SHAPE;

    PixelGemmParams P{};
    P.X = X; P.dY = dY; P.Out = part;
    P.N = N; P.IC = C; P.IH = H; P.IW = W; P.OC = OC; P.OH = g.OH; P.OW = g.OW;
    P.FH = FH; P.FW = FW; P.sh = g.sh; P.sw = g.sw; P.ph = g.ph; P.pw = g.pw;
    P.GZ = w.GZ; P.mTiles = w.mTiles; P.nTiles = w.nTiles;
    P.total = (int)total;
    P.perXcd = (P.total + kXcds - 1) / kXcds;
    P.sliceElems = (long)OC * FH * FW * C;
    switch (w.variant) {
#ifdef CKS_TUNING
        case 0: return launch_pixel<128, 128, 16, 2, 2, 1>(P, veca, vecb, st);
        case 1: return launch_pixel<128, 64, 32, 2, 1, 2>(P, veca, vecb, st);
        case 2: return launch_pixel<64, 128, 32, 1, 2, 2>(P, veca, vecb, st);
        case 3: return launch_pixel<64, 64, 32, 1, 1, 4>(P, veca, vecb, st);
        case 6: return launch_pixel<64, 128, 16, 2, 2, 1>(P, veca, vecb, st);
#endif
        case 4: return launch_pixel<64, 64, 16, 2, 2, 1>(P, veca, vecb, st, untrimmed);
        case 5: return launch_pixel<128, 64, 16, 2, 2, 1>(P, veca, vecb, st);
        default: return CKS_ERR_UNSUPPORTED;
    }
}

int wgrad(const Geo &g, const float *X, const float *dY, float *dW, void *ws, size_t ws_bytes, void *stream, bool untrimmed = false)
{
    if (!X || !dY || !dW) return CKS_ERR_NULL;
    const int GZ = plan_wgrad(g).GZ;
    const long slice = (long)g.OC * g.FH * g.FW * g.C;
    if (GZ == 1)  // one segment: its "partial" result is the result
        return wgrad_partials(g, X, dY, dW, (hipStream_t)stream, untrimmed);
    if (!ws || ws_bytes < sizeof(float) * (size_t)GZ * slice) return CKS_ERR_WORKSPACE;
    int rc = wgrad_partials(g, X, dY, (float *)ws, (hipStream_t)stream, untrimmed);
    if (rc != CKS_OK) return rc;
    return cks_reduce_partials((const float *)ws, dW, slice, GZ, stream);
}

}  // namespace

extern "C" {

// ---- stride and padding per axis

int cks_out_dims_hw(int H, int W, int FH, int FW, int sh, int sw, int ph, int pw, int *OH, int *OW)
{
    Geo g;
    int rc = check_geo(g, 1, 1, H, W, 1, FH, FW, sh, sw, ph, pw);
    if (rc != CKS_OK) return rc;
    if (OH) *OH = g.OH;
    if (OW) *OW = g.OW;
    return CKS_OK;
}

int64_t cks_useful_macs_hw(int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw)
{
    Geo g;
    if (check_geo(g, N, C, H, W, OC, FH, FW, sh, sw, ph, pw) != CKS_OK) return -1;
    return useful_macs(g);
}

size_t cks_conv2d_fwd_workspace_hw(int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw)
{
    (void)N; (void)C; (void)H; (void)W; (void)OC; (void)FH; (void)FW; (void)sh; (void)sw; (void)ph; (void)pw;
    return 0;  // the forward operator reads the filter in its given layout
}

size_t cks_deconv2d_workspace_hw(int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw)
{
    Geo g;
    if (check_geo(g, N, C, H, W, OC, FH, FW, sh, sw, ph, pw) != CKS_OK) return 0;
    return deconv_workspace(g);
}

size_t cks_dilated_conv2d_wgrad_workspace_hw(int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw)
{
    Geo g;
    if (check_geo(g, N, C, H, W, OC, FH, FW, sh, sw, ph, pw) != CKS_OK) return 0;
    return wgrad_workspace(g);
}

int cks_conv2d_fwd_hw(const float *X, const float *Wt, float *Y,
                      int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
                      void *ws, size_t ws_bytes, void *stream)
{
    (void)ws; (void)ws_bytes;
    Geo g;
    int rc = check_geo(g, N, C, H, W, OC, FH, FW, sh, sw, ph, pw);
    if (rc != CKS_OK) return rc;
    return conv_fwd(g, X, Wt, Y, (hipStream_t)stream);
}

int cks_deconv2d_hw(const float *dY, const float *Wt, float *dX,
                    int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
                    void *ws, size_t ws_bytes, void *stream)
{
    Geo g;
    int rc = check_geo(g, N, C, H, W, OC, FH, FW, sh, sw, ph, pw);
    if (rc != CKS_OK) return rc;
    return deconv(g, dY, Wt, dX, ws, ws_bytes, (hipStream_t)stream);
}

int cks_dilated_conv2d_wgrad_hw(const float *X, const float *dY, float *dW,
                                int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
                                void *ws, size_t ws_bytes, void *stream)
{
    Geo g;
    int rc = check_geo(g, N, C, H, W, OC, FH, FW, sh, sw, ph, pw);
    if (rc != CKS_OK) return rc;
    return wgrad(g, X, dY, dW, ws, ws_bytes, stream);
}

int cks_dilated_conv2d_wgrad_noalloc_hw(const float *X, const float *dY, float *dW,
                                        int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
                                        void *stream)
{
    Geo g;
    int rc = check_geo(g, N, C, H, W, OC, FH, FW, sh, sw, ph, pw);
    if (rc != CKS_OK) return rc;
    if (!X || !dY || !dW) return CKS_ERR_NULL;
    const size_t need = wgrad_workspace(g);
    if (need > CKS_STATIC_SCRATCH_BYTES) return CKS_ERR_SCRATCH;
    void *ptr = nullptr;
    if (need > 0 && !g_plan) {
        rc = static_scratch(&ptr);
        if (rc != CKS_OK) return rc;
    }
    // every element of the partial sums is written before the aggregation reads it: nothing to clear
    return wgrad(g, X, dY, dW, ptr, need, stream);
}

// ---- one stride and one padding for both axes

int cks_out_dims(int H, int W, int FH, int FW, int stride, int padding, int *OH, int *OW)
{
    return cks_out_dims_hw(H, W, FH, FW, stride, stride, padding, padding, OH, OW);
}

int64_t cks_useful_macs(int N, int C, int H, int W, int OC, int FH, int FW, int stride, int padding)
{
    return cks_useful_macs_hw(N, C, H, W, OC, FH, FW, stride, stride, padding, padding);
}

size_t cks_conv2d_fwd_workspace(int N, int C, int H, int W, int OC, int FH, int FW, int stride, int padding)
{
    return cks_conv2d_fwd_workspace_hw(N, C, H, W, OC, FH, FW, stride, stride, padding, padding);
}

size_t cks_deconv2d_workspace(int N, int C, int H, int W, int OC, int FH, int FW, int stride, int padding)
{
    return cks_deconv2d_workspace_hw(N, C, H, W, OC, FH, FW, stride, stride, padding, padding);
}

size_t cks_dilated_conv2d_wgrad_workspace(int N, int C, int H, int W, int OC, int FH, int FW, int stride, int padding)
{
    return cks_dilated_conv2d_wgrad_workspace_hw(N, C, H, W, OC, FH, FW, stride, stride, padding, padding);
}

int cks_conv2d_fwd(const float *X, const float *Wt, float *Y,
                   int N, int C, int H, int W, int OC, int FH, int FW, int stride, int padding,
                   void *ws, size_t ws_bytes, void *stream)
{
    return cks_conv2d_fwd_hw(X, Wt, Y, N, C, H, W, OC, FH, FW, stride, stride, padding, padding, ws, ws_bytes, stream);
}

int cks_deconv2d(const float *dY, const float *Wt, float *dX,
                 int N, int C, int H, int W, int OC, int FH, int FW, int stride, int padding,
                 void *ws, size_t ws_bytes, void *stream)
{
    return cks_deconv2d_hw(dY, Wt, dX, N, C, H, W, OC, FH, FW, stride, stride, padding, padding, ws, ws_bytes, stream);
}

int cks_dilated_conv2d_wgrad(const float *X, const float *dY, float *dW,
                             int N, int C, int H, int W, int OC, int FH, int FW, int stride, int padding,
                             void *ws, size_t ws_bytes, void *stream)
{
    return cks_dilated_conv2d_wgrad_hw(X, dY, dW, N, C, H, W, OC, FH, FW, stride, stride, padding, padding, ws, ws_bytes, stream);
}

// ---- stages

size_t cks_kernel_split_bytes_hw(int C, int OC, int FH, int FW, int sh, int sw)
{
    if (C <= 0 || OC <= 0 || FH <= 0 || FW <= 0 || sh < 1 || sw < 1) return 0;
    return split_bytes(C, OC, FH, FW, sh, sw);
}

size_t cks_kernel_split_bytes(int C, int OC, int FH, int FW, int stride)
{
    return cks_kernel_split_bytes_hw(C, OC, FH, FW, stride, stride);
}

int cks_kernel_split_hw(const float *Wt, float *Cs, int C, int OC, int FH, int FW, int sh, int sw, void *stream)
{
    return kernel_split(Wt, Cs, C, OC, FH, FW, sh, sw, (hipStream_t)stream);
}

int cks_kernel_split(const float *Wt, float *Cs, int C, int OC, int FH, int FW, int stride, void *stream)
{
    return cks_kernel_split_hw(Wt, Cs, C, OC, FH, FW, stride, stride, stream);
}

int cks_filter_transpose(const float *Wt, float *Wout, int C, int OC, int FH, int FW, void *stream)
{
    if (C <= 0 || OC <= 0 || FH <= 0 || FW <= 0) return CKS_ERR_SHAPE;
    if (!fits_i31((long long)C * OC * FH * FW)) return CKS_ERR_SHAPE;
    if (!Wt || !Wout) return CKS_ERR_NULL;
    return launch_pack<PACK_TRANSPOSE>(Wt, Wout, C, OC, FH, FW, 1, 1, (hipStream_t)stream);
}

int cks_conv2d_fwd_transposed_hw(const float *X, const float *Wtt, float *Y,
                                 int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
                                 void *stream)
{
    Geo g;
    int rc = check_geo(g, N, C, H, W, OC, FH, FW, sh, sw, ph, pw);
    if (rc != CKS_OK) return rc;
    return conv_fwd_transposed(g, X, Wtt, Y, (hipStream_t)stream);
}

int cks_conv2d_fwd_transposed(const float *X, const float *Wtt, float *Y,
                              int N, int C, int H, int W, int OC, int FH, int FW, int stride, int padding,
                              void *stream)
{
    return cks_conv2d_fwd_transposed_hw(X, Wtt, Y, N, C, H, W, OC, FH, FW, stride, stride, padding, padding, stream);
}

int cks_conv2d_fwd_untrimmed_hw(const float *X, const float *Wt, float *Y,
                                int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
                                void *stream)
{
    Geo g;
    int rc = check_geo(g, N, C, H, W, OC, FH, FW, sh, sw, ph, pw);
    if (rc != CKS_OK) return rc;
    return conv_fwd_untrimmed(g, X, Wt, Y, (hipStream_t)stream);
}

int cks_deconv2d_untrimmed_hw(const float *dY, const float *Wt, float *dX,
                              int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
                              void *stream)
{
    Geo g;
    int rc = check_geo(g, N, C, H, W, OC, FH, FW, sh, sw, ph, pw);
    if (rc != CKS_OK) return rc;
    return deconv_untrimmed(g, dY, Wt, dX, (hipStream_t)stream);
}

int cks_dilated_conv2d_wgrad_untrimmed_hw(const float *X, const float *dY, float *dW,
                                          int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
                                          void *ws, size_t ws_bytes, void *stream)
{
    Geo g;
    int rc = check_geo(g, N, C, H, W, OC, FH, FW, sh, sw, ph, pw);
    if (rc != CKS_OK) return rc;
    return wgrad(g, X, dY, dW, ws, ws_bytes, stream, true);
}

int cks_deconv2d_presplit_hw(const float *dY, const float *Cs, float *dX,
                             int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
                             void *stream)
{
    Geo g;
    int rc = check_geo(g, N, C, H, W, OC, FH, FW, sh, sw, ph, pw);
    if (rc != CKS_OK) return rc;
    return deconv_presplit(g, dY, Cs, dX, (hipStream_t)stream);
}

int cks_deconv2d_presplit(const float *dY, const float *Cs, float *dX,
                          int N, int C, int H, int W, int OC, int FH, int FW, int stride, int padding,
                          void *stream)
{
    return cks_deconv2d_presplit_hw(dY, Cs, dX, N, C, H, W, OC, FH, FW, stride, stride, padding, padding, stream);
}

int cks_dilated_conv2d_wgrad_segments_hw(int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw)
{
    Geo g;
    if (check_geo(g, N, C, H, W, OC, FH, FW, sh, sw, ph, pw) != CKS_OK) return 0;
    return plan_wgrad(g).GZ;
}

int cks_dilated_conv2d_wgrad_segments(int N, int C, int H, int W, int OC, int FH, int FW, int stride, int padding)
{
    return cks_dilated_conv2d_wgrad_segments_hw(N, C, H, W, OC, FH, FW, stride, stride, padding, padding);
}

int cks_dilated_conv2d_wgrad_partials_hw(const float *X, const float *dY, float *part,
                                         int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
                                         void *stream)
{
    Geo g;
    int rc = check_geo(g, N, C, H, W, OC, FH, FW, sh, sw, ph, pw);
    if (rc != CKS_OK) return rc;
    return wgrad_partials(g, X, dY, part, (hipStream_t)stream);
}

int cks_dilated_conv2d_wgrad_partials(const float *X, const float *dY, float *part,
                                      int N, int C, int H, int W, int OC, int FH, int FW, int stride, int padding,
                                      void *stream)
{
    return cks_dilated_conv2d_wgrad_partials_hw(X, dY, part, N, C, H, W, OC, FH, FW, stride, stride, padding, padding, stream);
}

int cks_reduce_partials(const float *part, float *dW, int64_t elems, int segments, void *stream)
{
    if (elems <= 0 || segments < 1 || !fits_i31(elems)) return CKS_ERR_SHAPE;
    if (!part || !dW) return CKS_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    const bool vec = elems % 4 == 0 && aligned16(part) && aligned16(dW);
    const int zl = segments >= 32 ? 16 : 1;                 // z-lanes per element
    const long per_block = (long)(kThreads / zl) * (vec ? 4 : 1);
    const int blocks = (int)((elems + per_block - 1) / per_block);
    const long n = (long)elems;
    if (zl == 16 && vec) return launch_args(kname("reduce_slices", 16, 4), reduce_slices<16, 4>, blocks, 0, st, kThreads, part, dW, n, segments);
    if (zl == 16) return launch_args(kname("reduce_slices", 16, 1), reduce_slices<16, 1>, blocks, 0, st, kThreads, part, dW, n, segments);
    if (vec) return launch_args(kname("reduce_slices", 1, 4), reduce_slices<1, 4>, blocks, 0, st, kThreads, part, dW, n, segments);
    return launch_args(kname("reduce_slices", 1, 1), reduce_slices<1, 1>, blocks, 0, st, kThreads, part, dW, n, segments);
}

// ---- which kernels a call would enqueue (host only)

int cks_plan_hw(int op, int N, int C, int H, int W, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
                unsigned only_4byte_aligned, char *text, size_t text_bytes)
{
    Geo g;
    int rc = check_geo(g, N, C, H, W, OC, FH, FW, sh, sw, ph, pw);
    if (rc != CKS_OK) return rc;
    if (!text || text_bytes == 0) return CKS_ERR_NULL;
    // Stand-in addresses with the requested alignment; no entry point reads or writes through a
    // pointer on the host, and with the recorder installed nothing reaches the device.
    auto ptr = [&](int i) { return reinterpret_cast<float *>((uintptr_t)0x10000000u * (uintptr_t)(i + 1) + ((only_4byte_aligned >> i) & 1u) * 4u); };
    float *a = ptr(0), *b = ptr(1), *c = ptr(2), *ws = ptr(3);
    PlanRecorder R{text, text_bytes, 0, false};
    text[0] = 0;
    g_plan = &R;
    switch (op) {
        case CKS_OP_CONV2D_FWD: rc = conv_fwd(g, a, b, c, nullptr); break;
        case CKS_OP_DECONV2D: rc = deconv(g, a, b, c, ws, deconv_workspace(g), nullptr); break;
        case CKS_OP_DILATED_CONV2D_WGRAD: rc = wgrad(g, a, b, c, ws, wgrad_workspace(g), nullptr); break;
        case CKS_OP_KERNEL_SPLIT: rc = kernel_split(a, b, C, OC, FH, FW, sh, sw, nullptr); break;
        case CKS_OP_DECONV2D_PRESPLIT: rc = deconv_presplit(g, a, b, c, nullptr); break;
        case CKS_OP_FILTER_TRANSPOSE: rc = cks_filter_transpose(a, b, C, OC, FH, FW, nullptr); break;
        case CKS_OP_WGRAD_PARTIALS: rc = wgrad_partials(g, a, b, c, nullptr); break;
        case CKS_OP_REDUCE_PARTIALS: rc = cks_reduce_partials(a, b, (int64_t)OC * FH * FW * C, plan_wgrad(g).GZ, nullptr); break;
        case CKS_OP_CONV2D_FWD_TRANSPOSED: rc = conv_fwd_transposed(g, a, b, c, nullptr); break;
        case CKS_OP_CONV2D_FWD_UNTRIMMED: rc = conv_fwd_untrimmed(g, a, b, c, nullptr); break;
        case CKS_OP_DECONV2D_UNTRIMMED: rc = deconv_untrimmed(g, a, b, c, nullptr); break;
        case CKS_OP_WGRAD_UNTRIMMED: rc = wgrad(g, a, b, c, ws, wgrad_workspace(g), nullptr, true); break;
        default: rc = CKS_ERR_UNSUPPORTED; break;
    }
    g_plan = nullptr;
    if (rc == CKS_OK && R.truncated) rc = CKS_ERR_WORKSPACE;
    return rc;
}

const char *cks_strerror(int status)
{
    switch (status) {
        case CKS_OK: return "success";
        case CKS_ERR_NULL: return "a required pointer is NULL";
        case CKS_ERR_SHAPE: return "invalid or too large tensor geometry";
        case CKS_ERR_WORKSPACE: return "workspace missing or too small";
        case CKS_ERR_HIP: return "HIP runtime error (see cks_last_hip_error)";
        case CKS_ERR_UNSUPPORTED: return "this entry point has no kernel for the geometry or pointer alignment";
        case CKS_ERR_SCRATCH: return "the call needs more scratch memory than the library's static buffer holds";
        default: return "unknown status";
    }
}

int cks_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
