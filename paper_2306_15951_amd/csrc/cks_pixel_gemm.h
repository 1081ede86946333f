// Sk-dilated-V2 (Algorithm 3B) as a split-K fp32-MFMA GEMM, plus the reduction
// of the split (Section IV.C, paragraph on map-reduce).
//
// For one filter tap (fh,fw):
//     dW[oc, fh, fw, ic] = sum over n, oh in [oh_s,oh_e), ow in [ow_s,ow_e)
//                          dY[n, oh, ow, oc] * X[n, fh-p+oh*s, fw-p+ow*s, ic]
// i.e. a GEMM with rows oc, columns ic and the contraction index k running over
// the pixels (n,oh,ow) of the tap's trimmed range.  dY is read exactly as it is
// stored (no zero is ever inserted), X with a leaping step s.  One k is one
// contiguous OC-row of dY and one contiguous IC-row of X.
//
// A workgroup owns (segment z of the pixel range, tap, BM oc, BN ic).  Segment
// z of G_Z writes its partial result to slice z of the workspace; a second
// kernel adds the slices in a fixed order.
#pragma once
#include "cks_device.h"

namespace cks {

struct PixelGemmParams {
    const float *X;
    const float *dY;
    float *Out;  // [GZ][OC][FH][FW][IC] partial sums (or dW itself when GZ == 1)
    int N, IC, IH, IW, OC, OH, OW, FH, FW, s, p;
    int GZ, mTiles, nTiles, total, perXcd;
    long sliceElems;  // OC*FH*FW*IC
};

// "advance a pixel counter by d" without division:  d = qn*(nOH*nOW) + rh*nOW + rw
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

template <int BM, int BN>
constexpr size_t pixel_lds_bytes() { return (size_t)2 * 16 * (BM + 32 + BN + 32) * sizeof(float); }

template <int BM, int BN, int WAVES_M, int WAVES_N, bool VECA, bool VECB>
__global__ void __launch_bounds__(kThreads) pixel_gemm(const PixelGemmParams P)
{
    constexpr int KC = 16;
    constexpr int LDA = BM + 32, LDB = BN + 32;   // +32: the two lane halves (k, k+1) hit disjoint banks
    constexpr int TM = BM / (WAVES_M * 32), TN = BN / (WAVES_N * 32);
    constexpr int PA = BM / 64, PB = BN / 64;
    static_assert(WAVES_M * WAVES_N == 4 && TM >= 1 && TN >= 1 && PA >= 1 && PB >= 1, "tile shape");

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
    const int ih_s = fh - P.p, iw_s = fw - P.p;
    const int oh_s = max(cdiv_any(-ih_s, P.s), 0), oh_e = min(P.OH, cdiv_any(P.IH - ih_s, P.s));
    const int ow_s = max(cdiv_any(-iw_s, P.s), 0), ow_e = min(P.OW, cdiv_any(P.IW - iw_s, P.s));
    const int nOH = max(oh_e - oh_s, 0), nOW = max(ow_e - ow_s, 0);
    const int Kt = P.N * nOH * nOW;
    const int seg = ((Kt + P.GZ - 1) / P.GZ + KC - 1) / KC * KC;
    const int kbeg = min(z * seg, Kt), kend = min(kbeg + seg, Kt);
    const int T = (kend - kbeg + KC - 1) / KC;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    // Staging: thread (lr, lc) fetches pixel kbeg + t*KC + lr, 16 bytes at
    // channel lc (+64, ...) of both operands.  (n, a, b) is that pixel's
    // (image, row, column) inside the trimmed range, advanced by carries.
    const int lr = tid >> 4, lc = (tid & 15) * 4;
    int pn = 0, pa_ = 0, pb_ = 0;
    PixStep stepKC = {0, 0, 0};
    if (T > 0) {
        int k = kbeg + lr;
        int q = k / nOW;
        pb_ = k - q * nOW;
        pn = q / nOH;
        pa_ = q - pn * nOH;
        stepKC = make_step(KC, nOH, nOW);
    }
    int kcur = kbeg + lr;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    float4 ra[PA], rb[PB];
    auto gload = [&]() {
        const bool live = kcur < kend;
        const int oh = oh_s + pa_, ow = ow_s + pb_;
        const float *ya = P.dY + (((long)pn * P.OH + oh) * P.OW + ow) * P.OC + m0 + lc;
        const float *xb = P.X + (((long)pn * P.IH + (oh * P.s + ih_s)) * P.IW + (ow * P.s + iw_s)) * P.IC + n0 + lc;
#pragma unroll
        for (int i = 0; i < PA; ++i) ra[i] = load4<VECA>(ya + 64 * i, live ? P.OC - (m0 + lc + 64 * i) : 0);
#pragma unroll
        for (int i = 0; i < PB; ++i) rb[i] = load4<VECB>(xb + 64 * i, live ? P.IC - (n0 + lc + 64 * i) : 0);
        // advance to the same row of the next chunk
        kcur += KC;
        pb_ += stepKC.rw;
        int c = pb_ >= nOW;
        pb_ -= c ? nOW : 0;
        pa_ += stepKC.rh + c;
        c = pa_ >= nOH;
        pa_ -= c ? nOH : 0;
        pn += stepKC.qn + c;
    };
    auto sstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < PA; ++i) *reinterpret_cast<float4 *>(&As[(buf * KC + lr) * LDA + lc + 64 * i]) = ra[i];
#pragma unroll
        for (int i = 0; i < PB; ++i) *reinterpret_cast<float4 *>(&Bs[(buf * KC + lr) * LDB + lc + 64 * i]) = rb[i];
    };

    if (T > 0) {
        gload();
        sstore(0);
    }
    __syncthreads();
    const int fcol = lane & 31, fk = lane >> 5;
    for (int t = 0; t < T; ++t) {
        const int buf = t & 1;
        const bool more = t + 1 < T;
        if (more) gload();
        const float *Ab = As + (buf * KC + fk) * LDA + wm * TM * 32 + fcol;
        const float *Bb = Bs + (buf * KC + fk) * LDB + wn * TN * 32 + fcol;
#pragma unroll
        for (int kk = 0; kk < KC / 2; ++kk) {
            float a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = Ab[kk * 2 * LDA + i * 32];
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = Bb[kk * 2 * LDB + j * 32];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = mfma32(a[i], b[j], acc[i][j]);
        }
        if (more) sstore(buf ^ 1);
        __syncthreads();
    }

    float *out = P.Out + (long)z * P.sliceElems;
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

// dW[e] = sum_z part[z][e], z ascending: a fixed order, so two runs agree bit for bit.
__global__ void __launch_bounds__(kThreads) reduce_slices(const float *part, float *dW, long elems, int GZ)
{
    const long e = (long)blockIdx.x * kThreads + threadIdx.x;
    if (e >= elems) return;
    float s = 0.f;
    for (int z = 0; z < GZ; ++z) s += part[(long)z * elems + e];
    dW[e] = s;
}

}  // namespace cks
