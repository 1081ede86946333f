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
    int N, IC, IH, IW, OC, OH, OW, FH, FW;
    int sh, sw, ph, pw;   // stride and padding per axis
    int GZ, mTiles, total, perXcd;
    long sliceElems;
};

// Shared tail: add the WAVES_K partial tiles through LDS (fixed tree) and store.
template <int WAVES_M, int WAVES_N, int WAVES_K, int NBW>
__device__ inline void patch_tile_epilogue(floatx16 (&acc)[NBW], float *smem, const PatchGemmParams &P, int z, int m0, int J,
                                           int wm, int wn, int wk, int lane)
{
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
        const int ih0 = px.a * P.sh - P.ph, iw0 = px.b * P.sw - P.pw;     // top-left corner of the patch in X
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
    const float *const Ar = As + fk * LDA + wm * 32 + fcol, *const Br = Bs + fk * LDB + wn * NBW * 32 + fcol;
    // The fragments of step kk+1 are requested from LDS before the MFMAs of step
    // kk are issued: with one wave per SIMD nothing else would cover that latency.
    auto compute = [&](int buf) {
        float a = Ar[buf * KC * LDA], b[NBW];
#pragma unroll
        for (int j = 0; j < NBW; ++j) b[j] = Br[buf * KC * LDB + j * 32];
#pragma unroll
        for (int kk = 0; kk < KW / 2; ++kk) {
            float an = 0.f, bn[NBW];
            if (kk + 1 < KW / 2) {
                an = Ar[(buf * KC + kk * 2 + 2) * LDA];
#pragma unroll
                for (int j = 0; j < NBW; ++j) bn[j] = Br[(buf * KC + kk * 2 + 2) * LDB + j * 32];
            }
#pragma unroll
            for (int j = 0; j < NBW; ++j) acc[j] = mfma32(a, b[j], acc[j]);
            if (kk + 1 < KW / 2) {
                a = an;
#pragma unroll
                for (int j = 0; j < NBW; ++j) b[j] = bn[j];
            }
            // pin the order: the LDS reads of the next step, then this step's MFMAs
            __builtin_amdgcn_sched_group_barrier(0x100, NBW + 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, NBW, 0);
        }
    };

    // two chunks per loop pass with literal buffer numbers and no branch around the
    // MFMAs (the accumulators stay in place); an odd chunk count is peeled off in front
    const int odd = T & 1;
    gload();          // chunk 0 (zeros when the segment is empty)
    if (odd) sstore(1); else sstore(0);
    __syncthreads();
    auto iteration = [&](int buf) {
        gload();      // next chunk; past the end of the segment every row is dead
        compute(buf);
        sstore(buf ^ 1);
        __syncthreads();
    };
    if (odd) iteration(1);
    for (int t = odd; t < T; t += 2) {
        iteration(0);
        iteration(1);
    }

    patch_tile_epilogue<WAVES_M, WAVES_N, WAVES_K, NBW>(acc, smem, P, z, m0, J, wm, wn, wk, lane);
}

// The same GEMM with the contraction index ordered (oh, ow) outer, batch inner:
// a K-chunk is KC consecutive images at one output position.  The address of
// a chunk is then a per-lane constant (image of the lane, item inside the
// patch) plus one scalar offset, and whether a tap lies in the padding is the
// same for the whole chunk: positions whose patch lies wholly inside X (all but
// the border) load without any mask or address arithmetic in vector
// registers.  Needs N to be a multiple of KC, OC a multiple of 4, 16-byte
// aligned dY and tensors below 2 GiB.
template <int WAVES_M, int WAVES_N, int WAVES_K, int NBW, int KC, bool VECB>
__global__ void __launch_bounds__(kThreads) patch_gemm_fast(const PatchGemmParams P)
{
    constexpr int BM = 32 * WAVES_M, BN = 32 * WAVES_N * NBW;
    constexpr int LDA = BM + 32, LDB = BN + 32;
    constexpr int LPP = kThreads / KC;
    constexpr int VW = VECB ? 4 : 1;
    constexpr int NI = (BN / VW + LPP - 1) / LPP;
    constexpr int NA = (BM / 4 + LPP - 1) / LPP;
    constexpr int KW = KC / WAVES_K;
    static_assert(WAVES_M * WAVES_N * WAVES_K == 4 && KW % 2 == 0 && kThreads % KC == 0, "tile shape");

    extern __shared__ __align__(16) float smem[];
    float *As = smem;                 // [2][KC][LDA]  dY rows
    float *Bs = smem + 2 * KC * LDA;  // [2][KC][LDB]  patches

    const int work = xcd_contiguous_work(blockIdx.x, P.perXcd);
    if (work >= P.total) return;
    const int mt = work % P.mTiles, z = work / P.mTiles;
    const int m0 = mt * BM;
    const int L = P.FW * P.IC, J = P.FH * L;

    const int NC = P.N / KC;                  // chunks per output position
    const int Ct = P.OH * P.OW * NC;
    // segment z of G_Z: the chunks are dealt evenly, the first Ct mod G_Z segments get one more
    const int seg = Ct / P.GZ, extra = Ct - seg * P.GZ;
    const int cbeg = z * seg + min(z, extra), T = seg + (z < extra ? 1 : 0);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wk = wave % WAVES_K, wn = (wave / WAVES_K) % WAVES_N, wm = wave / (WAVES_K * WAVES_N);

    // zero the patch tiles once: columns J.. of the padded tile are never staged
    for (int i = tid; i < 2 * KC * LDB; i += kThreads) Bs[i] = 0.f;

    // per-lane constants: image lp of the chunk; patch items lq, lq+LPP, ...; dY pieces lq, lq+LPP, ...
    const int lp = tid / LPP, lq = tid % LPP;
    const int imgX = P.IH * P.IW * P.IC, imgY = P.OH * P.OW * P.OC;
    int item_off[NI], item_code[NI];   // float offset inside the patch; (fh << 16 | column inside the filter row)
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int jf = (lq + LPP * i) * VW;
        if (jf < J) {
            const int fh = jf / L, j = jf - fh * L;
            item_off[i] = lp * imgX + fh * P.IW * P.IC + j;
            item_code[i] = (fh << 16) | j;
        } else {
            item_off[i] = 0;
            item_code[i] = 0x7fff0000;   // no such filter row
        }
    }
    unsigned va[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) va[i] = (unsigned)((lp * imgY + min(m0 + (lq + LPP * i) * 4, P.OC - 4)) * 4);
    const __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(P.dY), 0, -1, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsB = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(P.X), 0, -1, 0x00020000);

    int nch = 0, oh = 0, ow = 0;   // chunk being loaded
    if (T > 0) {
        nch = cbeg % NC;
        const int pos = cbeg / NC;
        oh = pos / P.OW;
        ow = pos - oh * P.OW;
    }

    floatx16 acc[NBW];
#pragma unroll
    for (int j = 0; j < NBW; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;

    float4 ra[NA];
    float4 rbv[VECB ? NI : 1];
    float rbs[VECB ? 1 : NI];
    auto gload = [&](bool live) {
        if (!live) return;   // uniform
        const int n1 = nch * KC;
        const int ih0 = oh * P.sh - P.ph, iw0 = ow * P.sw - P.pw;     // top-left corner of the patches of this chunk
        const int sa = (((n1 * P.OH + oh) * P.OW + ow) * P.OC) * 4;
#pragma unroll
        for (int i = 0; i < NA; ++i)
            if ((lq + LPP * i) * 4 < BM) ra[i] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(rsA, va[i], sa, 0));
        const bool inside = ih0 >= 0 && iw0 >= 0 && ih0 + P.FH <= P.IH && iw0 + P.FW <= P.IW;   // uniform
        if (inside) {
            const int sb = ((n1 * P.IH + ih0) * P.IW + iw0) * P.IC * 4;
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                if ((lq + LPP * i) * VW < J) {
                    if (VECB) rbv[VECB ? i : 0] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(rsB, item_off[i] * 4, sb, 0));
                    else rbs[VECB ? 0 : i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsB, item_off[i] * 4, sb, 0));
                }
            }
        } else {
            // border position: taps in the padding are not read and enter as zeros
            const int corner = (ih0 * P.IW + iw0) * P.IC;            // may be negative
            const int sb = n1 * imgX * 4;
            const int fh_lo = max(-ih0, 0), fh_hi = min(P.IH - ih0, P.FH);
            const int j_lo = max(-iw0, 0) * P.IC, j_hi = min(P.IW - iw0, P.FW) * P.IC;
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const int fh = item_code[i] >> 16, j = item_code[i] & 0xffff;
                const bool ok = fh >= fh_lo && fh < fh_hi && j >= j_lo && j < j_hi;
                if (VECB) {
                    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (ok) v = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(rsB, (item_off[i] + corner) * 4, sb, 0));
                    rbv[VECB ? i : 0] = v;
                } else {
                    float v = 0.f;
                    if (ok) v = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsB, (item_off[i] + corner) * 4, sb, 0));
                    rbs[VECB ? 0 : i] = v;
                }
            }
        }
        if (++nch == NC) { nch = 0; if (++ow == P.OW) { ow = 0; ++oh; } }
    };
    float *const Aw = As + lp * LDA + lq * 4, *const Bw = Bs + lp * LDB + lq * VW;
    auto sstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NA; ++i)
            if ((lq + LPP * i) * 4 < BM) *reinterpret_cast<float4 *>(Aw + buf * KC * LDA + LPP * i * 4) = ra[i];
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            if ((lq + LPP * i) * VW < J) {
                if (VECB) *reinterpret_cast<float4 *>(Bw + buf * KC * LDB + LPP * i * VW) = rbv[VECB ? i : 0];
                else Bw[buf * KC * LDB + LPP * i * VW] = rbs[VECB ? 0 : i];
            }
        }
    };
    const int fcol = lane & 31, fk = wk * KW + (lane >> 5);
    const float *const Ar = As + fk * LDA + wm * 32 + fcol, *const Br = Bs + fk * LDB + wn * NBW * 32 + fcol;
    auto compute = [&](int buf) {   // fragments of step kk+1 are requested before the MFMAs of step kk
        float a = Ar[buf * KC * LDA], b[NBW];
#pragma unroll
        for (int j = 0; j < NBW; ++j) b[j] = Br[buf * KC * LDB + j * 32];
#pragma unroll
        for (int kk = 0; kk < KW / 2; ++kk) {
            float an = 0.f, bn[NBW];
            if (kk + 1 < KW / 2) {
                an = Ar[(buf * KC + kk * 2 + 2) * LDA];
#pragma unroll
                for (int j = 0; j < NBW; ++j) bn[j] = Br[(buf * KC + kk * 2 + 2) * LDB + j * 32];
            }
#pragma unroll
            for (int j = 0; j < NBW; ++j) acc[j] = mfma32(a, b[j], acc[j]);
            if (kk + 1 < KW / 2) {
                a = an;
#pragma unroll
                for (int j = 0; j < NBW; ++j) b[j] = bn[j];
            }
            // pin the order: the LDS reads of the next step, then this step's MFMAs
            __builtin_amdgcn_sched_group_barrier(0x100, NBW + 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, NBW, 0);
        }
    };

    const int odd = T & 1;
    __syncthreads();   // the zero fill above is complete
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

    patch_tile_epilogue<WAVES_M, WAVES_N, WAVES_K, NBW>(acc, smem, P, z, m0, J, wm, wn, wk, lane);
}

}  // namespace cks
