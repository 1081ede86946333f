// Sk-dilated (filter gradient) for image stems whose geometry is known at
// compile time.
//
//     dW[oc, (fh,fw,ic)] = sum_{n,oh,ow} dY[n,oh,ow,oc] * X[n, oh*s-p+fh, ow*s-p+fw, ic]
// is a GEMM with rows = output channels, columns = the J = FH*FW*IC taps and
// the output pixels as contraction axis: dY is used as it is (Algorithm 3 never
// inserts the zeros of the dilated dY; reading X at stride s is its leaping
// access).  As in strip_fwd the X operand is never gathered into patches: the
// staging waves copy the tile's input strip to LDS as it lies in memory (zeros
// where it overlaps the padding), and the MFMA lane that owns tap k of pixel
// (th,tw) reads  strip[rowoff(th,tw) + koff(k)] - a lane constant plus a
// constant of the K step.
//
// The pixel axis is cut into segments (Section IV.C's map-reduce over G_Z
// parts): one workgroup per segment walks a contiguous range of 4 x 16 pixel
// tiles.  MFMA wave w contracts tile row w (16 pixels, 8 K steps) into its own
// 64 x J accumulator (2 x NB blocks of 32x32); at the end the four waves' sums
// are added in a fixed order through LDS and the segment's partial dW goes to
// part[segment][OC][J].  Waves 4-7 meanwhile stage the next tile's strip and dY rows.
#pragma once
#include "cks_device.h"
#include "cks_strip_fwd.h"

namespace cks {

struct StripWgradParams {
    const float *X;
    const float *dY;
    float *part;        // [blocks][OC][J]
    int N, IH, IW, OC, OH, OW, p;
    int nBands;         // ceil(OW / 16)
    int nRowTiles;      // ceil(OH / 4)
    int tiles;          // N * nBands * nRowTiles
    int tilesPerBlock;
};

constexpr int kStripWgradLDY = 68;   // dY tile pitch: 64 channels + 4
template <int FH, int FW, int IC, int S>
constexpr size_t strip_wgrad_lds_bytes()
{
    using G = StripGeo<FH, FW, IC, S>;
    constexpr size_t run = 2 * 64 * kStripWgradLDY + 2 * G::STRIP;
    constexpr size_t red = (size_t)2 * ((G::J + 31) / 32) * 16 * 64;   // one wave's accumulators
    return (run > red ? run : red) * sizeof(float);
}

// VEC: dY rows may be read as float4 (OC % 4 == 0 and a 16-byte aligned dY)
template <int FH, int FW, int IC, int S, bool VEC>
__global__ void __launch_bounds__(kStripThreads) strip_wgrad(const StripWgradParams P)
{
    using G = StripGeo<FH, FW, IC, S>;
    constexpr int L = G::L, J = G::J, RP = G::RP, STRIP = G::STRIP;
    constexpr int NB = (J + 31) / 32;          // column blocks
    constexpr int LDY = kStripWgradLDY, ABUF = 64 * LDY;
    extern __shared__ __align__(16) float smem[];
    float *As = smem;                 // [2][64 pixels][LDY]
    float *Ss = smem + 2 * ABUF;      // [2][STRIP]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tile_beg = blockIdx.x * P.tilesPerBlock, tile_end = min(tile_beg + P.tilesPerBlock, P.tiles);

    for (int i = tid; i < 2 * ABUF + 2 * STRIP; i += kStripThreads) smem[i] = 0.f;
    __syncthreads();

    auto decode = [&](int tile, int &n, int &c, int &t) {
        t = tile % P.nRowTiles;
        const int q = tile / P.nRowTiles;
        c = q % P.nBands;
        n = q / P.nBands;
    };

    floatx16 acc[2][NB];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mb][nb][r] = 0.f;

    if (wave >= 4) {
        // ---------------------------------------------------------------- staging waves
        const int pw = wave - 4, ptid = tid - 256;
        StripStager<G> stager;
        // (written for instruction count, see StripStager: a tile cursor advanced without divisions, one dY
        // descriptor per image, 32-bit scalar row offsets, no per-row tests when the tile's rows all exist)
        int fn, fc, ft, ftile = tile_beg;   // the tile fetched next
        decode(tile_beg < P.tiles ? tile_beg : 0, fn, fc, ft);
        // dY: tile row th is min(16, OW-ow0)*OC contiguous floats; thread f takes floats 4f..4f+3 of it
        const bool a_lane = 4 * ptid < 16 * P.OC;
        const int a_px = a_lane ? (4 * ptid) / P.OC : 0, a_oc = a_lane ? 4 * ptid - a_px * P.OC : 0;
        float *a_dst = As + a_px * LDY + a_oc;   // VEC: OC % 4 == 0, the four floats are one pixel's
        float4 areg[4];
        constexpr int kBeyond = (int)0x80000000u;
        const int imgY = P.OH * P.OW * P.OC;     // floats of dY per image (the host checks: below 2 GiB)
        int a_band = -1, a_voff[VEC ? 1 : 4];    // byte offsets of this thread's floats in a tile row, or kBeyond
        int a_img = -1;
        __amdgpu_buffer_rsrc_t rs;               // image a_img of dY
        auto fetch = [&]() {
            if (ftile >= tile_end) return;   // uniform
            // (made scalar explicitly: the cursor is uniform, but lives across divergent code)
            const int n = __builtin_amdgcn_readfirstlane(fn), c = __builtin_amdgcn_readfirstlane(fc), t = __builtin_amdgcn_readfirstlane(ft);
            ++ftile;
            if (++ft == P.nRowTiles) { ft = 0; if (++fc == P.nBands) { fc = 0; ++fn; } }
            if (n != a_img) {   // uniform, and before the lanes part ways: the descriptor stays in scalar registers
                a_img = n;
                rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(P.dY + (long)n * imgY), 0, imgY * 4, 0x00020000);
            }
            stager.fetch(P.X, n, c, t, pw, lane, P.IH, P.IW, P.p);
            if (!a_lane) return;
            const int ow0 = c * 16;
            if (c != a_band) {   // uniform: floats past the last output column of the band read as zero
                a_band = c;
                const int a_bytes = min(16, P.OW - ow0) * P.OC * 4;
#pragma unroll
                for (int i = 0; i < (VEC ? 1 : 4); ++i) a_voff[i] = 16 * ptid + 4 * i < a_bytes ? 16 * ptid + 4 * i : kBeyond;
            }
            int soff = ((4 * t) * P.OW + ow0) * P.OC * 4;
            const int rowB = P.OW * P.OC * 4;
            if (VEC && 4 * t + 4 <= P.OH) {   // uniform
#pragma unroll
                for (int th = 0; th < 4; ++th, soff += rowB)
                    areg[th] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(rs, a_voff[0], soff, 0));
                return;
            }
#pragma unroll
            for (int th = 0; th < 4; ++th, soff += rowB) {
                const bool in = 4 * t + th < P.OH;   // uniform; a row below the map reads as zero
                if constexpr (VEC) {
                    areg[th] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(rs, in ? a_voff[0] : kBeyond, soff, 0));
                } else {
                    areg[th].x = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, in ? a_voff[0] : kBeyond, soff, 0));
                    areg[th].y = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, in ? a_voff[VEC ? 0 : 1] : kBeyond, soff, 0));
                    areg[th].z = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, in ? a_voff[VEC ? 0 : 2] : kBeyond, soff, 0));
                    areg[th].w = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, in ? a_voff[VEC ? 0 : 3] : kBeyond, soff, 0));
                }
            }
        };
        auto stage = [&](int tile, int buf) {
            if (tile >= tile_end) return;
            stager.stage(Ss + buf * STRIP, pw, lane);
            if (!a_lane) return;
            float *d = a_dst + buf * ABUF;
#pragma unroll
            for (int th = 0; th < 4; ++th) {
                if constexpr (VEC) {
                    *reinterpret_cast<float4 *>(d + th * 16 * LDY) = areg[th];
                } else {
                    // the four floats may straddle pixels: place each by its own (pixel, channel)
                    const float e[4] = {areg[th].x, areg[th].y, areg[th].z, areg[th].w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int f = 4 * ptid + i, px = f / P.OC, oc = f - px * P.OC;
                        As[buf * ABUF + (th * 16 + px) * LDY + oc] = e[i];
                    }
                }
            }
        };
        fetch();                 // tile_beg
        stage(tile_beg, 0);
        fetch();                 // tile_beg + 1
        __syncthreads();
        // the loads of tile t+2 are issued as soon as the registers of tile t+1 have gone to LDS: they
        // have a whole tile's time to arrive
        for (int tile = tile_beg; tile < tile_end; ++tile) {
            stage(tile + 1, (tile + 1 - tile_beg) & 1);
            fetch();             // tile + 2
            __syncthreads();
        }
    } else {
        // ---------------------------------------------------------------- MFMA waves: wave w contracts tile row w
        // 32x32x2 MFMA: lane l supplies A[m = l%32][k = l/32] and B[k = l/32][n = l%32]; here m is an
        // output channel, n a tap and k a pixel: K step t covers pixels tw = 2t (lanes 0-31), 2t+1 (32-63).
        const int h = lane >> 5, l32 = lane & 31;
        const float *a_base[2];
        const float *b_base[NB];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) a_base[mb] = As + (wave * 16 + h) * LDY + 32 * mb + l32;   // + 2t*LDY
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int k = 32 * nb + l32;
            const int koff = k < J ? (k / L) * RP + k % L : 0;   // columns past J are computed and dropped
            b_base[nb] = Ss + wave * S * RP + h * S * IC + koff;   // + 2t*S*IC
        }
        __syncthreads();
        for (int tile = tile_beg; tile < tile_end; ++tile) {
            const int buf = (tile - tile_beg) & 1;
            const int sa = buf * ABUF, ss = buf * STRIP;
            float av[2][2], bv[2][NB];   // [step parity][block]
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) av[0][mb] = a_base[mb][sa];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) bv[0][nb] = b_base[nb][ss];
            __builtin_amdgcn_sched_group_barrier(0x100, 2 + NB, 0);
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int cur = t & 1, nxt = cur ^ 1;
                if (t < 7) {
#pragma unroll
                    for (int mb = 0; mb < 2; ++mb) av[nxt][mb] = a_base[mb][sa + 2 * (t + 1) * LDY];
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) bv[nxt][nb] = b_base[nb][ss + 2 * (t + 1) * S * IC];
                }
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) acc[mb][nb] = mfma32(av[cur][mb], bv[cur][nb], acc[mb][nb]);
                // pin the order: the LDS reads of the next step, then this step's MFMAs
                if (t < 7) __builtin_amdgcn_sched_group_barrier(0x100, 2 + NB, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 2 * NB, 0);
            }
            __syncthreads();
        }
    }

    // -------------------------------------------------------------------- sum of the four waves, fixed order
    // (all eight waves pass the same barriers; LDS is free now)
    float *R = smem;   // [2*NB blocks][16 registers][64 lanes]
    for (int src = 1; src < 4; ++src) {
        __syncthreads();
        if (wave == src) {
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) R[((mb * NB + nb) * 16 + r) * 64 + lane] = acc[mb][nb][r];
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[mb][nb][r] += R[((mb * NB + nb) * 16 + r) * 64 + lane];
        }
    }
    if (wave == 0) {
        float *out = P.part + (long)blockIdx.x * P.OC * J;
        const int h = lane >> 5, l32 = lane & 31;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int k = 32 * nb + l32;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int oc = 32 * mb + 8 * (r >> 2) + 4 * h + (r & 3);
                    if (oc < P.OC && k < J) out[(long)oc * J + k] = acc[mb][nb][r];
                }
            }
    }
}

}  // namespace cks
