// ConvV2 for layers with few input channels (image stems): the whole filter
// patch is the contraction axis.
//
// With IC = 3 a filter row (fw, ic) is 21 floats, so the per-position kernel
// spends a padded 32-float K-chunk on each of them and re-stages the filter for
// every position.  Here
//     Y[(n,oh,ow), oc] = sum_{j'} patch[(n,oh,ow), j'] * W[oc, j'],   j' = (fh,fw,ic), J = FH*FW*IC
// is one GEMM over all output pixels: rows = 64 consecutive pixels, columns = 64
// output channels, K = J rounded up to 16.  The filter slice W[oc0..oc0+64][J]
// (already K-contiguous in OHWI) is staged into LDS once per workgroup, which
// then walks a contiguous range of pixel tiles; only the patches stream.
// A patch is FH contiguous segments of FW*IC floats of X; taps that fall into
// the padding are not read and enter as zeros (Algorithm 1's trimmed range,
// realised as a per-pixel mask because one tile mixes positions with different
// trims; such taps are 1.5 % of a 224x224 7x7/s2/p3 layer).
#pragma once
#include "cks_device.h"

namespace cks {

struct PatchFwdParams {
    const float *X;
    const float *W;
    float *Y;
    int N, IC, IH, IW, OC, OH, OW, FH, FW;
    int sh, sw, ph, pw;   // stride and padding per axis
    int KP;             // J rounded up to a multiple of 16 (<= 192)
    int nT;             // 64-wide output-channel tiles
    int tilesPerBlock;  // pixel tiles each workgroup walks
    int mTiles;         // ceil(N*OH*OW / 64)
};

constexpr int kPatchFwdMaxKP = 192;
constexpr int kPatchFwdThreads = 512;   // 4 MFMA waves + 4 staging waves
inline size_t patch_fwd_lds_bytes(int KP) { return (size_t)3 * 64 * (KP + 4) * sizeof(float); }

// Waves 0-3 multiply pixel tile t out of LDS and store it; waves 4-7 meanwhile
// fetch the patches of tile t+1 and write them to the other LDS buffer.  Each
// SIMD hosts one wave of either kind, so address arithmetic and loads run in
// the shadow of the MFMAs.  One workgroup barrier per tile.
__global__ void __launch_bounds__(kPatchFwdThreads) patch_fwd(const PatchFwdParams P)
{
    constexpr int PASSES = kPatchFwdMaxKP / 64;   // patch columns per lane
    extern __shared__ __align__(16) float smem[];
    const int LDK = P.KP + 4;
    float *Ws = smem;                  // [64][LDK]   filter slice
    float *As = smem + 64 * LDK;       // [2][64][LDK] patches of a pixel tile

    const int nt = blockIdx.x % P.nT, g = blockIdx.x / P.nT;
    const int oc0 = nt * 64;
    const int L = P.FW * P.IC, J = P.FH * L;
    const int M = P.N * P.OH * P.OW;   // fits: Y has fewer than 2^31 elements
    const int tile_beg = g * P.tilesPerBlock, tile_end = min(tile_beg + P.tilesPerBlock, P.mTiles);
    if (tile_beg >= tile_end) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: role and pixel arithmetic stay scalar

    // zero the three LDS tiles once (K padding columns are never written again), then stage W
    for (int i = tid; i < 3 * 64 * LDK; i += kPatchFwdThreads) smem[i] = 0.f;
    __syncthreads();
    for (int i = tid; i < 64 * J; i += kPatchFwdThreads) {
        const int r = i / J, j = i - r * J;
        if (oc0 + r < P.OC) Ws[r * LDK + j] = P.W[(long)(oc0 + r) * J + j];
    }

    // X as a raw buffer of its exact size (the host checks that X and Y are below
    // 2 GiB): an offset of 2 GiB is out of range whatever scalar offset is added.
    const int img = P.IH * P.IW * P.IC;   // floats per image
    const __amdgpu_buffer_rsrc_t rsX = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(P.X), 0, P.N * img * 4, 0x00020000);
    constexpr int kBeyond = (int)0x80000000u;

    if (wave >= 4) {
        // ---------------- staging waves: wave pw fetches pixels 16pw .. 16pw+15 of a tile.
        // Lane l handles patch columns j' = l, l+64, l+128.  A group of 16 pixels
        // whose patches lie wholly inside X and in one image row is fetched with
        // buffer loads "lane constant + scalar pixel offset": no vector ALU work.
        const int pw = wave - 4;
        int col_off[PASSES], col_fh[PASSES], col_j[PASSES];
#pragma unroll
        for (int q = 0; q < PASSES; ++q) {
            const int jf = lane + 64 * q;
            if (jf < J) {
                col_fh[q] = jf / L;
                col_j[q] = jf - col_fh[q] * L;
                col_off[q] = col_fh[q] * P.IW * P.IC + col_j[q];
            } else {
                col_fh[q] = 1 << 20;   // never inside a patch
                col_j[q] = 0;
                col_off[q] = 0;        // reads element 0 of the patch; never staged
            }
        }
        float stage[16][PASSES];
        auto fetch = [&](int tile, int buf) {
            if (tile >= tile_end) return;   // uniform
            const int m0 = tile * 64 + pw * 16;
            int ow = m0 % P.OW;
            const int t2 = m0 / P.OW;
            int oh = t2 % P.OH;
            int n = t2 / P.OH;
            const int ih0 = oh * P.sh - P.ph, iw0 = ow * P.sw - P.pw;
            const bool fast = m0 + 16 <= M && ow + 16 <= P.OW && ih0 >= 0 && ih0 + P.FH <= P.IH && iw0 >= 0 &&
                              iw0 + 15 * P.sw + P.FW <= P.IW;
            if (fast) {
                const int s0 = ((n * P.IH + ih0) * P.IW + iw0) * P.IC * 4, ds = P.sw * P.IC * 4;
#pragma unroll
                for (int i = 0; i < 16; ++i)
#pragma unroll
                    for (int q = 0; q < PASSES; ++q)
                        stage[i][q] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsX, col_off[q] * 4, s0 + i * ds, 0));
            } else {
                // Border group: per pixel the valid filter rows / columns are scalar
                // ranges; a lane whose tap is in the padding (or whose pixel is past
                // the end) sends an offset beyond the descriptor's size, for which a
                // buffer load returns zero without touching memory.  No branches, so
                // all 48 loads are in flight together.
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const bool live = m0 + i < M;
                    const int h0 = oh * P.sh - P.ph, w0 = ow * P.sw - P.pw;
                    const int corner4 = (h0 * P.IW + w0) * P.IC * 4;   // may be negative
                    const int fh_lo = max(-h0, 0), j_lo = max(-w0, 0) * P.IC;
                    const unsigned fh_n = live ? (unsigned)max(min(P.IH - h0, P.FH) - fh_lo, 0) : 0u;
                    const unsigned j_n = (unsigned)max(min(P.IW - w0, P.FW) * P.IC - j_lo, 0);
                    const int sn = (live ? n : 0) * img * 4;
#pragma unroll
                    for (int q = 0; q < PASSES; ++q) {
                        const bool ok = ((unsigned)(col_fh[q] - fh_lo) < fh_n) & ((unsigned)(col_j[q] - j_lo) < j_n);
                        const int voff = ok ? corner4 + col_off[q] * 4 : kBeyond;
                        stage[i][q] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsX, voff, sn, 0));
                    }
                    if (++ow == P.OW) { ow = 0; if (++oh == P.OH) { oh = 0; ++n; } }
                }
            }
#pragma unroll
            for (int q = 0; q < PASSES; ++q) {
                const int jf = lane + 64 * q;
                if (jf < J) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) As[(buf * 64 + pw * 16 + i) * LDK + jf] = stage[i][q];
                }
            }
        };
        fetch(tile_beg, 0);
        __syncthreads();
        for (int tile = tile_beg; tile < tile_end; ++tile) {
            fetch(tile + 1, (tile + 1 - tile_beg) & 1);   // reads nothing past the workgroup's range
            __syncthreads();
        }
        return;
    }

    // ---------------- MFMA waves: 2 x 2 blocks of 32 pixels x 32 channels
    const int wm = wave >> 1, wn = wave & 1;
    const int frow = lane & 31, fk = (lane >> 5) * 4;
    const int nks = P.KP >> 3;   // even: KP is a multiple of 16
    const __amdgpu_buffer_rsrc_t rsY = __builtin_amdgcn_make_buffer_rsrc(P.Y, 0, -1, 0x00020000);
    const int col = oc0 + wn * 32 + (lane & 31);
    const int vrow0 = wm * 32 + 4 * (lane >> 5);
    __syncthreads();
    for (int tile = tile_beg; tile < tile_end; ++tile) {
        const int buf = (tile - tile_beg) & 1;
        floatx16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
        const float *Ab = As + (buf * 64 + wm * 32 + frow) * LDK + fk;
        const float *Bb = Ws + (wn * 32 + frow) * LDK + fk;
        // fragments of step ks+1 are requested before the MFMAs of step ks are issued
        float4 a0 = *reinterpret_cast<const float4 *>(Ab), b0 = *reinterpret_cast<const float4 *>(Bb);
        for (int ks = 0; ks < nks; ks += 2) {
            const float4 a1 = *reinterpret_cast<const float4 *>(Ab + ks * 8 + 8);
            const float4 b1 = *reinterpret_cast<const float4 *>(Bb + ks * 8 + 8);
            acc = mfma32(a0.x, b0.x, acc);
            acc = mfma32(a0.y, b0.y, acc);
            acc = mfma32(a0.z, b0.z, acc);
            acc = mfma32(a0.w, b0.w, acc);
            if (ks + 2 < nks) {
                a0 = *reinterpret_cast<const float4 *>(Ab + ks * 8 + 16);
                b0 = *reinterpret_cast<const float4 *>(Bb + ks * 8 + 16);
            }
            acc = mfma32(a1.x, b1.x, acc);
            acc = mfma32(a1.y, b1.y, acc);
            acc = mfma32(a1.z, b1.z, acc);
            acc = mfma32(a1.w, b1.w, acc);
        }
        // a full tile is stored with "lane constant + scalar tile offset" addressing
        const bool full = tile * 64 + 64 <= M && oc0 + 64 <= P.OC;   // uniform
        if (full) {
            const int st = tile * 64 * P.OC * 4;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[r]), rsY,
                                                      ((vrow0 + 8 * (r >> 2) + (r & 3)) * P.OC + col) * 4, st, 0);
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = tile * 64 + vrow0 + 8 * (r >> 2) + (r & 3);
                if (row < M && col < P.OC) P.Y[(long)row * P.OC + col] = acc[r];
            }
        }
        __syncthreads();
    }
}

}  // namespace cks
