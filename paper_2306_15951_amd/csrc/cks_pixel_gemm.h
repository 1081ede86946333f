// Sk-dilated-V2 (Algorithm 3B) as a split-K fp32-MFMA GEMM, plus the reduction
// of the split (Section IV.C, paragraph on map-reduce).
//
// For one filter tap (fh,fw):
//     dW[oc, fh, fw, ic] = sum over n, oh in [oh_s,oh_e), ow in [ow_s,ow_e)
//                          dY[n, oh, ow, oc] * X[n, fh-ph+oh*sh, fw-pw+ow*sw, ic]
// i.e. a GEMM with rows oc, columns ic and the contraction index k running over
// the pixels (n,oh,ow) of the tap's trimmed range.  dY is read exactly as it is
// stored (no zero is ever inserted), X with a leaping step (sh, sw).  One k is one
// contiguous OC-row of dY and one contiguous IC-row of X.
//
// The contraction axis is split at two levels:
//   * between workgroups: segment z of G_Z writes its partial result to slice z
//     of the workspace; a second kernel adds the slices in a fixed order;
//   * inside a workgroup whose tile is smaller than 128x128: the WAVES_K waves
//     that share a tile each take every WAVES_K-th part of a K-chunk, so that
//     every wave still owns a 64x64 block of accumulators, and their results
//     are added through LDS in a fixed tree before the store.
#pragma once
#include "cks_device.h"

namespace cks {

struct PixelGemmParams {
    const float *X;
    const float *dY;
    float *Out;  // [GZ][OC][FH][FW][IC] partial sums (or dW itself when GZ == 1)
    int N, IC, IH, IW, OC, OH, OW, FH, FW;
    int sh, sw, ph, pw;   // stride and padding per axis
    int GZ, mTiles, nTiles, total, perXcd;
    long sliceElems;  // OC*FH*FW*IC
    // divisors of the work decoding, prepared on the host (see FastDiv)
    FastDiv dNT, dMT, dTaps, dFW, dSh, dSw, dGZ, dNC;   // nTiles, mTiles, FH*FW, FW, sh, sw, GZ, N/KC (chunks per pixel of pixel_gemm_fast)
    int bufStore;     // a slice is below 2 GiB: full tiles are stored through a buffer descriptor
};

// Pixel counter inside a tap's trimmed range: k = (n*nOH + a)*nOW + b.
struct Pix { int n, a, b; };
// "advance by d" without division:  d = (qn*nOH + rh)*nOW + rw
struct PixStep { int qn, rh, rw; };

__device__ inline PixStep make_step(int d, int nOH, int nOW)
{
    PixStep st;
    int q = d / nOW;
    st.rw = d - q * nOW;
    st.qn = q / nOH;
    st.rh = q - st.qn * nOH;
    return st;
}
__device__ inline Pix advance(Pix x, PixStep st, int nOH, int nOW)
{
    x.b += st.rw;
    int c = x.b >= nOW;
    x.b -= c ? nOW : 0;
    x.a += st.rh + c;
    c = x.a >= nOH;
    x.a -= c ? nOH : 0;
    x.n += st.qn + c;
    return x;
}

// Shared tail of the filter-gradient kernels: add the WAVES_K partial tiles (in
// each round the upper half of the remaining waves hands its accumulators to
// the lower half through LDS: a fixed tree) and store the tile to slice z.
template <int TM, int TN, int WAVES_M, int WAVES_N, int WAVES_K>
__device__ inline void wgrad_tile_epilogue(floatx16 (&acc)[TM][TN], float *smem, const PixelGemmParams &P, int z, int tap,
                                           int m0, int n0, int wm, int wn, int wk, int lane)
{
    if (WAVES_K > 1) {
        float4 *red = reinterpret_cast<float4 *>(smem);
#pragma unroll
        for (int h = WAVES_K / 2; h >= 1; h /= 2) {
            // slot of the (wm, wn, wk - h) tile: TM*TN*4 float4 per lane
            if (wk >= h && wk < 2 * h) {
                float4 *dst = red + (size_t)(((wm * WAVES_N + wn) * h + (wk - h)) * TM * TN * 4) * 64 + lane;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            dst[((i * TN + j) * 4 + q) * 64] = make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1],
                                                                           acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
            }
            __syncthreads();
            if (wk < h) {
                const float4 *src = red + (size_t)(((wm * WAVES_N + wn) * h + wk) * TM * TN * 4) * 64 + lane;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const float4 v = src[((i * TN + j) * 4 + q) * 64];
                            acc[i][j][4 * q] += v.x;
                            acc[i][j][4 * q + 1] += v.y;
                            acc[i][j][4 * q + 2] += v.z;
                            acc[i][j][4 * q + 3] += v.w;
                        }
            }
            __syncthreads();
        }
        if (wk != 0) return;
    }
    float *out = P.Out + (long)z * P.sliceElems;
    if (P.bufStore && m0 + WAVES_M * TM * 32 <= P.OC) {
        // A tile with all its output channels: the slice as a raw buffer, lane part of the offset once,
        // row part as a scalar offset (not range-checked by the hardware: hence full tiles only); an
        // input channel past the end carries an offset beyond the buffer.  No vector arithmetic per store.
        const __amdgpu_buffer_rsrc_t rsO = __builtin_amdgcn_make_buffer_rsrc(out, 0, (int)(P.sliceElems * 4), 0x00020000);
        const int rowB = P.FH * P.FW * P.IC * 4;   // bytes between output channels
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int ic = n0 + (wn * TN + j) * 32 + (lane & 31);
                const int oc0 = m0 + (wm * TM + i) * 32 + 4 * (lane >> 5);
                const int voff = ic < P.IC ? oc0 * rowB + (tap * P.IC + ic) * 4 : (int)0x80000000u;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[i][j][r]), rsO, voff, (8 * (r >> 2) + (r & 3)) * rowB, 0);
            }
        return;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int ic = n0 + (wn * TN + j) * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int oc = m0 + (wm * TM + i) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (oc < P.OC && ic < P.IC) out[((long)oc * P.FH * P.FW + tap) * P.IC + ic] = acc[i][j][r];
            }
        }
}

template <int BM, int BN, int KC>
constexpr size_t pixel_lds_bytes() { return (size_t)2 * KC * (BM + 32 + BN + 32) * sizeof(float); }

template <int BM, int BN, int KC, int WAVES_M, int WAVES_N, int WAVES_K, bool VECA, bool VECB>
__global__ void __launch_bounds__(kThreads) pixel_gemm(const PixelGemmParams P)
{
    constexpr int LDA = BM + 32, LDB = BN + 32;   // +32: the two lane halves (k, k+1) hit disjoint banks
    constexpr int TM = BM / (WAVES_M * 32), TN = BN / (WAVES_N * 32);
    constexpr int PA = BM / 64, PB = BN / 64;     // 16-byte loads per thread and pixel row
    constexpr int PK = KC / 16;                   // pixel rows per thread and chunk
    constexpr int KW = KC / WAVES_K;              // k handled by one wave per chunk
    static_assert(WAVES_M * WAVES_N * WAVES_K == 4 && TM >= 1 && TN >= 1 && PA >= 1 && PB >= 1 && PK >= 1 &&
                  KW % 2 == 0, "tile shape");
    static_assert((size_t)(WAVES_K / 2) * WAVES_M * WAVES_N * TM * TN * 1024 * 4 <= pixel_lds_bytes<BM, BN, KC>(),
                  "the wave reduction reuses the staging buffers");

    extern __shared__ __align__(16) float smem[];
    float *As = smem;                 // [2][KC][LDA]   dY rows
    float *Bs = smem + 2 * KC * LDA;  // [2][KC][LDB]   X rows

    const int work = xcd_contiguous_work(blockIdx.x, P.perXcd);
    if (work >= P.total) return;
    const int nt = work % P.nTiles;
    const int mt = (work / P.nTiles) % P.mTiles;
    const int tap = (work / (P.nTiles * P.mTiles)) % (P.FH * P.FW);
    const int z = work / (P.nTiles * P.mTiles * P.FH * P.FW);
    const int fh = tap / P.FW, fw = tap - fh * P.FW;
    const int m0 = mt * BM, n0 = nt * BN;

    // Algorithm 3B: the (oh,ow) whose X element exists for this tap.
    const int ih_s = fh - P.ph, iw_s = fw - P.pw;
    const int oh_s = max(cdiv_any(-ih_s, P.sh), 0), oh_e = min(P.OH, cdiv_any(P.IH - ih_s, P.sh));
    const int ow_s = max(cdiv_any(-iw_s, P.sw), 0), ow_e = min(P.OW, cdiv_any(P.IW - iw_s, P.sw));
    const int nOH = max(oh_e - oh_s, 0), nOW = max(ow_e - ow_s, 0);
    const int Kt = P.N * nOH * nOW;
    const int seg = ((Kt + P.GZ - 1) / P.GZ + KC - 1) / KC * KC;
    const int kbeg = min(z * seg, Kt), kend = min(kbeg + seg, Kt);
    const int T = (kend - kbeg + KC - 1) / KC;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wk = wave % WAVES_K, wn = (wave / WAVES_K) % WAVES_N, wm = wave / (WAVES_K * WAVES_N);

    // Staging: thread (lr, lc) fetches pixel rows lr, lr+16, .. of a chunk, 16
    // bytes at channel lc (+64, ...) of both operands.
    const int lr = tid >> 4, lc = (tid & 15) * 4;
    Pix px[PK];
    PixStep stepKC = {0, 0, 0};
    if (T > 0) {
        const PixStep step16 = make_step(16, nOH, nOW);
        stepKC = make_step(KC, nOH, nOW);
        const int k = kbeg + lr, q = k / nOW;
        px[0].b = k - q * nOW;
        px[0].n = q / nOH;
        px[0].a = q - px[0].n * nOH;
#pragma unroll
        for (int r = 1; r < PK; ++r) px[r] = advance(px[r - 1], step16, nOH, nOW);
    } else {
#pragma unroll
        for (int r = 0; r < PK; ++r) px[r] = Pix{0, 0, 0};
    }
    int kcur = kbeg + lr;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // The loads of chunk t+1 are issued before chunk t is multiplied out of LDS
    // and stored to the other LDS buffer after it.
    struct Stage { float4 a[PK][PA], b[PK][PB]; };
    Stage S0;
    auto gload = [&](Stage &S) {
#pragma unroll
        for (int r = 0; r < PK; ++r) {
            const bool live = kcur + 16 * r < kend;   // dead rows (past the segment) read nothing: zeros
            const int oh = oh_s + px[r].a, ow = ow_s + px[r].b;
            const float *ya = P.dY + (((long)px[r].n * P.OH + oh) * P.OW + ow) * P.OC + m0 + lc;
            const float *xb =
                P.X + (((long)px[r].n * P.IH + (oh * P.sh + ih_s)) * P.IW + (ow * P.sw + iw_s)) * P.IC + n0 + lc;
#pragma unroll
            for (int i = 0; i < PA; ++i) S.a[r][i] = load4<VECA>(ya + 64 * i, live ? P.OC - (m0 + lc + 64 * i) : 0);
#pragma unroll
            for (int i = 0; i < PB; ++i) S.b[r][i] = load4<VECB>(xb + 64 * i, live ? P.IC - (n0 + lc + 64 * i) : 0);
            px[r] = advance(px[r], stepKC, nOH, nOW);   // same row of the next chunk
        }
        kcur += KC;
    };
    auto sstore = [&](const Stage &S, int buf) {
#pragma unroll
        for (int r = 0; r < PK; ++r) {
#pragma unroll
            for (int i = 0; i < PA; ++i)
                *reinterpret_cast<float4 *>(&As[(buf * KC + lr + 16 * r) * LDA + lc + 64 * i]) = S.a[r][i];
#pragma unroll
            for (int i = 0; i < PB; ++i)
                *reinterpret_cast<float4 *>(&Bs[(buf * KC + lr + 16 * r) * LDB + lc + 64 * i]) = S.b[r][i];
        }
    };
    const int fcol = lane & 31, fk = wk * KW + (lane >> 5);
    const float *const Ar = As + fk * LDA + wm * TM * 32 + fcol, *const Br = Bs + fk * LDB + wn * TN * 32 + fcol;
    auto compute = [&](int buf) {   // fragments of step kk+1 are requested before the MFMAs of step kk
        float a[TM], b[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) a[i] = Ar[buf * KC * LDA + i * 32];
#pragma unroll
        for (int j = 0; j < TN; ++j) b[j] = Br[buf * KC * LDB + j * 32];
#pragma unroll
        for (int kk = 0; kk < KW / 2; ++kk) {
            float an[TM], bn[TN];
            if (kk + 1 < KW / 2) {
#pragma unroll
                for (int i = 0; i < TM; ++i) an[i] = Ar[(buf * KC + kk * 2 + 2) * LDA + i * 32];
#pragma unroll
                for (int j = 0; j < TN; ++j) bn[j] = Br[(buf * KC + kk * 2 + 2) * LDB + j * 32];
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = mfma32(a[i], b[j], acc[i][j]);
            if (kk + 1 < KW / 2) {
#pragma unroll
                for (int i = 0; i < TM; ++i) a[i] = an[i];
#pragma unroll
                for (int j = 0; j < TN; ++j) b[j] = bn[j];
            }
            // pin the order: the LDS reads of the next step, then this step's MFMAs
            __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, TM * TN, 0);
        }
    };

    // two chunks per loop pass with literal buffer numbers and no branch around the
    // MFMAs (the accumulators stay in place); an odd chunk count is peeled off in front
    const int odd = T & 1;
    gload(S0);          // chunk 0 (zeros when the segment is empty)
    if (odd) sstore(S0, 1); else sstore(S0, 0);
    __syncthreads();
    auto iteration = [&](int buf) {
        gload(S0);      // next chunk; past the end of the segment every row is dead
        compute(buf);
        sstore(S0, buf ^ 1);
        __syncthreads();
    };
    if (odd) iteration(1);
    for (int t = odd; t < T; t += 2) {
        iteration(0);
        iteration(1);
    }

    wgrad_tile_epilogue<TM, TN, WAVES_M, WAVES_N, WAVES_K>(acc, smem, P, z, tap, m0, n0, wm, wn, wk, lane);
}

// The same GEMM with the contraction index ordered (oh, ow) outer, batch n
// inner: a K-chunk is KC consecutive images at one (oh,ow) of the tap's trimmed
// range.  Then the address of a chunk is a per-lane constant (image and channel
// of the lane) plus one scalar offset ((oh,ow) and first image of the chunk),
// so the loop issues buffer loads with a scalar offset and no vector ALU
// instruction for addressing -- VALU instructions and MFMAs of one SIMD do not
// overlap, so each one removed from the loop is MFMA time won.  Needs N to be a
// multiple of KC, 16-byte aligned tensors with channel counts that are
// multiples of 4, and tensors below 2 GiB; the pixel-ordered kernel above
// handles everything else.
template <int BM, int BN, int KC, int WAVES_M, int WAVES_N, int WAVES_K>
__global__ void __launch_bounds__(kThreads) pixel_gemm_fast(const PixelGemmParams P)
{
    constexpr int LDA = BM + 32, LDB = BN + 32;
    constexpr int TM = BM / (WAVES_M * 32), TN = BN / (WAVES_N * 32);
    constexpr int PA = BM / 64, PB = BN / 64;
    constexpr int PK = KC / 16;
    constexpr int KW = KC / WAVES_K;
    static_assert(WAVES_M * WAVES_N * WAVES_K == 4 && TM >= 1 && TN >= 1 && PA >= 1 && PB >= 1 && PK >= 1 &&
                  KW % 2 == 0, "tile shape");

    extern __shared__ __align__(16) float smem[];
    float *As = smem;                 // [2][KC][LDA]   dY rows
    float *Bs = smem + 2 * KC * LDA;  // [2][KC][LDB]   X rows

    const int work = xcd_contiguous_work(blockIdx.x, P.perXcd);
    if (work >= P.total) return;
    const int q1 = fdiv(work, P.dNT), nt = work - q1 * P.nTiles;
    const int q2 = fdiv(q1, P.dMT), mt = q1 - q2 * P.mTiles;
    const int z = fdiv(q2, P.dTaps), tap = q2 - z * P.dTaps.d;
    const int fh = fdiv(tap, P.dFW), fw = tap - fh * P.FW;
    const int m0 = mt * BM, n0 = nt * BN;

    // Algorithm 3B: the (oh,ow) whose X element exists for this tap.  ceil(a/s) for a of either sign
    // (a > -(FH + FW)): shift the numerator by a multiple of s that makes it non-negative.
    const int ih_s = fh - P.ph, iw_s = fw - P.pw;
    const int shiftK = P.FH + P.FW;
    auto cdiv_s = [&](int a, const FastDiv &d) { return fdiv(a + shiftK * d.d + d.d - 1, d) - shiftK; };
    const int oh_s = max(cdiv_s(-ih_s, P.dSh), 0), oh_e = min(P.OH, cdiv_s(P.IH - ih_s, P.dSh));
    const int ow_s = max(cdiv_s(-iw_s, P.dSw), 0), ow_e = min(P.OW, cdiv_s(P.IW - iw_s, P.dSw));
    const int nOH = max(oh_e - oh_s, 0), nOW = max(ow_e - ow_s, 0);
    const int NC = P.dNC.d;                        // chunks per (oh,ow): N / KC
    const int Ct = nOH * nOW * NC;                 // chunks of this tap
    // segment z of G_Z: the chunks are dealt evenly, the first Ct mod G_Z segments get one more
    const int seg = fdiv(Ct, P.dGZ), extra = Ct - seg * P.GZ;
    const int cbeg = z * seg + min(z, extra), T = seg + (z < extra ? 1 : 0);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wk = wave % WAVES_K, wn = (wave / WAVES_K) % WAVES_N, wm = wave / (WAVES_K * WAVES_N);

    // per-lane part of the addresses: image lr (+16, ...) of the chunk, channels lc (+64, ...)
    const int lr = tid >> 4, lc = (tid & 15) * 4;
    unsigned va[PK][PA], vb[PK][PB];
#pragma unroll
    for (int r = 0; r < PK; ++r) {
#pragma unroll
        for (int i = 0; i < PA; ++i)   // channels past the end are clamped (loaded twice, never stored)
            va[r][i] = (unsigned)(((lr + 16 * r) * P.OH * P.OW * P.OC + min(m0 + lc + 64 * i, P.OC - 4)) * 4);
#pragma unroll
        for (int i = 0; i < PB; ++i)
            vb[r][i] = (unsigned)(((lr + 16 * r) * P.IH * P.IW * P.IC + min(n0 + lc + 64 * i, P.IC - 4)) * 4);
    }
    const __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(P.dY), 0, -1, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsB = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(P.X), 0, -1, 0x00020000);

    // scalar part: position and first image of the chunk being loaded
    int nch = 0, pa_ = 0, pb_ = 0;
    if (T > 0) {
        const int pos = fdiv(cbeg, P.dNC);
        nch = cbeg - pos * NC;
        pa_ = pos / nOW;
        pb_ = pos - pa_ * nOW;
    }

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    struct Stage { float4 a[PK][PA], b[PK][PB]; };
    Stage S0;
    auto gload = [&](bool live) {
        if (!live) return;   // uniform
        const int oh = oh_s + pa_, ow = ow_s + pb_, n1 = nch * KC;
        const int sa = (((n1 * P.OH + oh) * P.OW + ow) * P.OC) * 4;
        const int sb = (((n1 * P.IH + oh * P.sh + ih_s) * P.IW + ow * P.sw + iw_s) * P.IC) * 4;
#pragma unroll
        for (int r = 0; r < PK; ++r) {
#pragma unroll
            for (int i = 0; i < PA; ++i)
                S0.a[r][i] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(rsA, va[r][i], sa, 0));
#pragma unroll
            for (int i = 0; i < PB; ++i)
                S0.b[r][i] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(rsB, vb[r][i], sb, 0));
        }
        if (++nch == NC) { nch = 0; if (++pb_ == nOW) { pb_ = 0; ++pa_; } }
    };
    float *const Aw = As + lr * LDA + lc, *const Bw = Bs + lr * LDB + lc;
    auto sstore = [&](int buf) {
#pragma unroll
        for (int r = 0; r < PK; ++r) {
#pragma unroll
            for (int i = 0; i < PA; ++i) *reinterpret_cast<float4 *>(Aw + (buf * KC + 16 * r) * LDA + 64 * i) = S0.a[r][i];
#pragma unroll
            for (int i = 0; i < PB; ++i) *reinterpret_cast<float4 *>(Bw + (buf * KC + 16 * r) * LDB + 64 * i) = S0.b[r][i];
        }
    };
    const int fcol = lane & 31, fk = wk * KW + (lane >> 5);
    const float *const Ar = As + fk * LDA + wm * TM * 32 + fcol, *const Br = Bs + fk * LDB + wn * TN * 32 + fcol;
    auto compute = [&](int buf) {   // fragments of step kk+1 are requested before the MFMAs of step kk
        float a[TM], b[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) a[i] = Ar[buf * KC * LDA + i * 32];
#pragma unroll
        for (int j = 0; j < TN; ++j) b[j] = Br[buf * KC * LDB + j * 32];
#pragma unroll
        for (int kk = 0; kk < KW / 2; ++kk) {
            float an[TM], bn[TN];
            if (kk + 1 < KW / 2) {
#pragma unroll
                for (int i = 0; i < TM; ++i) an[i] = Ar[(buf * KC + kk * 2 + 2) * LDA + i * 32];
#pragma unroll
                for (int j = 0; j < TN; ++j) bn[j] = Br[(buf * KC + kk * 2 + 2) * LDB + j * 32];
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = mfma32(a[i], b[j], acc[i][j]);
            if (kk + 1 < KW / 2) {
#pragma unroll
                for (int i = 0; i < TM; ++i) a[i] = an[i];
#pragma unroll
                for (int j = 0; j < TN; ++j) b[j] = bn[j];
            }
            // pin the order: the LDS reads of the next step, then this step's MFMAs
            __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, TM * TN, 0);
        }
    };

    // two chunks per loop pass with literal buffer numbers; an odd count is peeled off in front
    const int odd = T & 1;
    gload(T > 0);
    if (T > 0) { if (odd) sstore(1); else sstore(0); }
    __syncthreads();
    auto iteration = [&](int t, int buf) {
        gload(t + 1 < T);
        compute(buf);
        if (t + 1 < T) sstore(buf ^ 1);
        __syncthreads();
    };
    if (odd) iteration(0, 1);
    for (int t = odd; t < T; t += 2) {
        iteration(t, 0);
        iteration(t + 1, 1);
    }

    wgrad_tile_epilogue<TM, TN, WAVES_M, WAVES_N, WAVES_K>(acc, smem, P, z, tap, m0, n0, wm, wn, wk, lane);
}

// dW[e] = sum_z part[z][e] in a fixed association, so two runs agree bit for
// bit: z-lane l of ZL adds slices l, l+ZL, l+2ZL, ... in ascending order, then
// the ZL lane sums are added in ascending lane order.  A workgroup covers
// (256/ZL)*VW consecutive elements; VW = 4 uses 16-byte accesses.
template <int ZL, int VW>
__global__ void __launch_bounds__(kThreads) reduce_slices(const float *part, float *dW, long elems, int GZ)
{
    constexpr int COLS = kThreads / ZL;
    __shared__ float red[ZL > 1 ? kThreads * VW : 1];
    const int col = threadIdx.x % COLS, zl = threadIdx.x / COLS;
    const long e = ((long)blockIdx.x * COLS + col) * VW;
    float s[VW];
#pragma unroll
    for (int v = 0; v < VW; ++v) s[v] = 0.f;
    if (e < elems) {
        const float *p = part + e + (long)zl * elems;
        const long step = (long)ZL * elems;
        // eight slices are requested before the first is added (the additions stay in ascending order): a
        // thread that waited for each load in turn would spend the kernel on memory latency
        int z = zl;
        for (; z + 7 * ZL < GZ; z += 8 * ZL, p += 8 * step) {
            if (VW == 4) {
                float4 t[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) t[u] = *reinterpret_cast<const float4 *>(p + u * step);
#pragma unroll
                for (int u = 0; u < 8; ++u) { s[0] += t[u].x; s[VW > 1 ? 1 : 0] += t[u].y; s[VW > 2 ? 2 : 0] += t[u].z; s[VW > 3 ? 3 : 0] += t[u].w; }
            } else {
                float t[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) t[u] = p[u * step];
#pragma unroll
                for (int u = 0; u < 8; ++u) s[0] += t[u];
            }
        }
        for (; z + 3 * ZL < GZ; z += 4 * ZL, p += 4 * step) {
            if (VW == 4) {
                float4 t[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) t[u] = *reinterpret_cast<const float4 *>(p + u * step);
#pragma unroll
                for (int u = 0; u < 4; ++u) { s[0] += t[u].x; s[VW > 1 ? 1 : 0] += t[u].y; s[VW > 2 ? 2 : 0] += t[u].z; s[VW > 3 ? 3 : 0] += t[u].w; }
            } else {
                float t[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) t[u] = p[u * step];
#pragma unroll
                for (int u = 0; u < 4; ++u) s[0] += t[u];
            }
        }
        for (; z < GZ; z += ZL, p += step) {
            if (VW == 4) {
                const float4 t = *reinterpret_cast<const float4 *>(p);
                s[0] += t.x; s[VW > 1 ? 1 : 0] += t.y; s[VW > 2 ? 2 : 0] += t.z; s[VW > 3 ? 3 : 0] += t.w;
            } else {
                s[0] += p[0];
            }
        }
    }
    if (ZL > 1) {
#pragma unroll
        for (int v = 0; v < VW; ++v) red[(zl * VW + v) * COLS + col] = s[v];
        __syncthreads();
        if (zl != 0 || e >= elems) return;
#pragma unroll
        for (int v = 0; v < VW; ++v) {
            float t = red[v * COLS + col];
            for (int l = 1; l < ZL; ++l) t += red[(l * VW + v) * COLS + col];
            s[v] = t;
        }
    } else if (e >= elems) {
        return;
    }
    if (VW == 4) *reinterpret_cast<float4 *>(dW + e) = make_float4(s[0], s[VW > 1 ? 1 : 0], s[VW > 2 ? 2 : 0], s[VW > 3 ? 3 : 0]);
    else dW[e] = s[0];
}

}  // namespace cks
