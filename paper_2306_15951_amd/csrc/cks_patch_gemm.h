// Sk-dilated (Algorithm 3) for layers with few input channels: all filter taps
// in one GEMM tile.
//
// When IC is small a per-tap tile (rows oc, columns ic) is far narrower than an
// MFMA block, and every tap re-reads dY.  Here the GEMM columns are the whole
// filter patch j' = (fh, fw, ic), J = FH*FW*IC of them:
//     dW[oc, j'] = sum over pixels (n,oh,ow)  dY[n,oh,ow,oc] * patch[(n,oh,ow), j']
//     patch[(n,oh,ow), (fh,fw,ic)] = X[n, oh*s-p+fh, ow*s-p+fw, ic]   (0 outside X)
// dY is read exactly as stored (nothing is ever inserted) and once; X is read
// with the leaping step s (Section IV.C).  In NHWC one filter row of the patch
// is FW*IC contiguous floats of X, so a patch is FH contiguous segments.
// Border pixels get zeros for the taps that fall into the padding instead of a
// per-tap trimmed range: with one tile for all taps the range cannot be cut per
// tap.  (Padded taps are 1.5 % of the work on a 7x7/s2 stem layer, 4 % on a
// 32x32 3x3 layer; layers with many channels use the per-tap kernel, which
// trims exactly.)
//
// Tile: BM = 32*WAVES_M output channels x NB*32 patch columns, every wave owns
// one 32-row block and NBW column blocks; WAVES_K waves share a tile and split
// each K-chunk, their partial tiles are added through LDS in a fixed tree.
// The contraction axis is also split between workgroups (G_Z segments), as in
// the per-tap kernel.
#pragma once
#include "cks_pixel_gemm.h"

namespace cks {

struct PatchGemmParams {
    const float *X;
    const float *dY;
    float *Out;  // [GZ][OC][FH*FW*IC]
    int N, IC, IH, IW, OC, OH, OW, FH, FW, s, p;
    int GZ, mTiles, total, perXcd;
    long sliceElems;
};

template <int WAVES_M, int WAVES_N, int NBW, int KC>
constexpr size_t patch_lds_bytes() { return (size_t)2 * KC * (32 * WAVES_M + 32 + 32 * WAVES_N * NBW + 32) * sizeof(float); }

template <int WAVES_M, int WAVES_N, int WAVES_K, int NBW, int KC, bool VECA, bool VECB>
__global__ void __launch_bounds__(kThreads) patch_gemm(const PatchGemmParams P)
{
    constexpr int BM = 32 * WAVES_M, BN = 32 * WAVES_N * NBW;
    constexpr int LDA = BM + 32, LDB = BN + 32;
    constexpr int LPP = kThreads / KC;                 // lanes that share one pixel row of a chunk
    constexpr int VW = VECB ? 4 : 1;                   // floats per patch item
    constexpr int NI = (BN / VW + LPP - 1) / LPP;      // patch items per lane
    constexpr int NA = (BM / 4 + LPP - 1) / LPP;       // 16-byte dY pieces per lane
    constexpr int KW = KC / WAVES_K;
    static_assert(WAVES_M * WAVES_N * WAVES_K == 4 && KW % 2 == 0 && kThreads % KC == 0, "tile shape");
    static_assert((size_t)(WAVES_K / 2) * WAVES_M * WAVES_N * NBW * 4096 <= patch_lds_bytes<WAVES_M, WAVES_N, NBW, KC>(),
                  "the wave reduction reuses the staging buffers");

    extern __shared__ __align__(16) float smem[];
    float *As = smem;                 // [2][KC][LDA]  dY rows
    float *Bs = smem + 2 * KC * LDA;  // [2][KC][LDB]  patches

    const int work = xcd_contiguous_work(blockIdx.x, P.perXcd);
    if (work >= P.total) return;
    const int mt = work % P.mTiles, z = work / P.mTiles;
    const int m0 = mt * BM;
    const int L = P.FW * P.IC, J = P.FH * L;

    const int Kt = P.N * P.OH * P.OW;
    const int seg = ((Kt + P.GZ - 1) / P.GZ + KC - 1) / KC * KC;
    const int kbeg = min(z * seg, Kt), kend = min(kbeg + seg, Kt);
    const int T = (kend - kbeg + KC - 1) / KC;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wk = wave % WAVES_K, wn = (wave / WAVES_K) % WAVES_N, wm = wave / (WAVES_K * WAVES_N);

    // Staging: LPP lanes share pixel kbeg + t*KC + lp; lane lq of them fetches
    // patch items lq, lq+LPP, ... (an item is VW consecutive floats of one
    // filter row) and dY pieces lq, lq+LPP, ...
    const int lp = tid / LPP, lq = tid % LPP;
    int item_off[NI], item_code[NI];   // offset inside the patch; (fh << 16 | column inside the filter row)
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int jf = (lq + LPP * i) * VW;   // flat patch column of the item
        if (jf < J) {
            const int fh = jf / L, j = jf - fh * L;
            item_off[i] = fh * P.IW * P.IC + j;
            item_code[i] = (fh << 16) | j;
        } else {
            item_off[i] = 0;
            item_code[i] = 0x7fff0000;        // filter row that never exists: stages zeros
        }
    }
    Pix px = {0, 0, 0};
    PixStep stepKC = {0, 0, 0};
    if (T > 0) {
        stepKC = make_step(KC, P.OH, P.OW);
        const int k = kbeg + lp, q = k / P.OW;
        px.b = k - q * P.OW;
        px.n = q / P.OH;
        px.a = q - px.n * P.OH;
    }
    int kcur = kbeg + lp;

    floatx16 acc[NBW];
#pragma unroll
    for (int j = 0; j < NBW; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;

    float4 ra[NA];
    float4 rbv[VECB ? NI : 1];
    float rbs[VECB ? 1 : NI];
    auto gload = [&]() {
        const bool live = kcur < kend;
        const int ih0 = px.a * P.s - P.p, iw0 = px.b * P.s - P.p;     // top-left corner of the patch in X
        const float *ya = P.dY + (((long)px.n * P.OH + px.a) * P.OW + px.b) * P.OC + m0;
        const float *xb = P.X + (((long)px.n * P.IH + ih0) * P.IW + iw0) * P.IC;
        // filter rows / columns of this pixel's patch that lie inside X
        const int fh_lo = live ? max(-ih0, 0) : P.FH, fh_hi = min(P.IH - ih0, P.FH);
        const int j_lo = max(-iw0, 0) * P.IC, j_hi = min(P.IW - iw0, P.FW) * P.IC;
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int c = (lq + LPP * i) * 4;
            ra[i] = load4<VECA>(ya + c, (live && c < BM) ? P.OC - (m0 + c) : 0);
        }
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int fh = item_code[i] >> 16, j = item_code[i] & 0xffff;
            const bool ok = fh >= fh_lo && fh < fh_hi && j >= j_lo && j < j_hi;
            if (VECB) {
                rbv[VECB ? i : 0] = ok ? *reinterpret_cast<const float4 *>(xb + item_off[i]) : make_float4(0.f, 0.f, 0.f, 0.f);
            } else {
                rbs[VECB ? 0 : i] = ok ? xb[item_off[i]] : 0.f;
            }
        }
        px = advance(px, stepKC, P.OH, P.OW);
        kcur += KC;
    };
    auto sstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int c = (lq + LPP * i) * 4;
            if (c < BM) *reinterpret_cast<float4 *>(&As[(buf * KC + lp) * LDA + c]) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int jf = (lq + LPP * i) * VW;
            if (jf < BN) {
                if (VECB) *reinterpret_cast<float4 *>(&Bs[(buf * KC + lp) * LDB + jf]) = rbv[VECB ? i : 0];
                else Bs[(buf * KC + lp) * LDB + jf] = rbs[VECB ? 0 : i];
            }
        }
    };
    const int fcol = lane & 31, fk = wk * KW + (lane >> 5);
    auto compute = [&](int buf) {
        const float *Ab = As + (buf * KC + fk) * LDA + wm * 32 + fcol;
        const float *Bb = Bs + (buf * KC + fk) * LDB + wn * NBW * 32 + fcol;
#pragma unroll
        for (int kk = 0; kk < KW / 2; ++kk) {
            const float a = Ab[kk * 2 * LDA];
            float b[NBW];
#pragma unroll
            for (int j = 0; j < NBW; ++j) b[j] = Bb[kk * 2 * LDB + j * 32];
#pragma unroll
            for (int j = 0; j < NBW; ++j) acc[j] = mfma32(a, b[j], acc[j]);
        }
    };

    gload();          // chunk 0 (zeros when the segment is empty)
    sstore(0);
    __syncthreads();
    for (int t = 0; t < T; ++t) {
        gload();      // chunk t+1; past the end of the segment every row is dead
        compute(t & 1);
        sstore((t + 1) & 1);
        __syncthreads();
    }

    if (WAVES_K > 1) {
        float4 *red = reinterpret_cast<float4 *>(smem);
#pragma unroll
        for (int h = WAVES_K / 2; h >= 1; h /= 2) {
            if (wk >= h && wk < 2 * h) {
                float4 *dst = red + (size_t)(((wm * WAVES_N + wn) * h + (wk - h)) * NBW * 4) * 64 + lane;
#pragma unroll
                for (int j = 0; j < NBW; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        dst[(j * 4 + q) * 64] =
                            make_float4(acc[j][4 * q], acc[j][4 * q + 1], acc[j][4 * q + 2], acc[j][4 * q + 3]);
            }
            __syncthreads();
            if (wk < h) {
                const float4 *src = red + (size_t)(((wm * WAVES_N + wn) * h + wk) * NBW * 4) * 64 + lane;
#pragma unroll
                for (int j = 0; j < NBW; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float4 v = src[(j * 4 + q) * 64];
                        acc[j][4 * q] += v.x;
                        acc[j][4 * q + 1] += v.y;
                        acc[j][4 * q + 2] += v.z;
                        acc[j][4 * q + 3] += v.w;
                    }
            }
            __syncthreads();
        }
        if (wk != 0) return;
    }

    float *out = P.Out + (long)z * P.sliceElems;
#pragma unroll
    for (int j = 0; j < NBW; ++j) {
        const int jf = (wn * NBW + j) * 32 + (lane & 31);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int oc = m0 + wm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            if (oc < P.OC && jf < J) out[(long)oc * J + jf] = acc[j][r];
        }
    }
}

}  // namespace cks
