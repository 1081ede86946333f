// Sk-dilated-V2 (Algorithm 3B), general path: pixel_gemm_fast of cks_pixel_gemm.h with its K-chunks fetched
// straight into LDS (see cks_rowrun_dma.h for why, and for the inline-assembly fragment reads).
//
// Same GEMM (rows = output channels, columns = input channels, contraction over the pixels of the tap's trimmed
// range, batch innermost), same split of the contraction axis into G_Z segments, same tile store.  A K-chunk is 32
// consecutive images at one (oh,ow): 32 k-rows of 64 dY channels and 32 k-rows of 64 X channels, each k-row 256
// contiguous bytes in memory.  A wave's LDS-direct load moves four such rows (16 lanes x 16 bytes each); the LDS
// tile is therefore K-major, [32 k][64 channels], unpadded.  Lane l of an MFMA supplies channel l % 32 at k = 2 t +
// l / 32 in step t: the two lane halves read rows of different parity at the same column, so the 16-byte pieces of
// odd k-rows are stored with bit 3 of their position flipped (column ^ 32), which puts the halves into different
// bank halves.  Steps t and t + 1 are two rows apart: one ds_read2_b32 fetches both.
#pragma once
#include "cks_pixel_gemm.h"
#include "cks_rowrun_dma.h"

namespace cks {

constexpr int kPixelDmaKC = 32;
constexpr size_t pixel_dma_lds_bytes() { return (size_t)2 * kPixelDmaKC * (64 + 64) * sizeof(float); }

// Two floats OFF0 and OFF1 rows of 64 floats behind addr: the rows of a K-major [k][64] tile.
template <int OFF0, int OFF1>
__device__ __forceinline__ floatx2v lds_read2_rows64(unsigned addr)
{
    static_assert(OFF0 >= 0 && OFF0 < 256 && OFF1 >= 0 && OFF1 < 256, "ds_read2st64 offsets are 8-bit counts of 64 dwords");
    floatx2v v = {0.f, 0.f};
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("ds_read2st64_b32 %0, %1 offset0:%2 offset1:%3" : "=v"(v) : "v"(addr), "n"(OFF0), "n"(OFF1));
#else
    (void)addr;
#endif
    return v;
}
template <int PENDING>
__device__ __forceinline__ void lds_wait(floatx2v &a, floatx2v &b)
{
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a), "+v"(b) : "n"(PENDING));
#endif
}

// MFMA steps 2 G and 2 G + 1 of a chunk in LDS buffer BUF (32 rows behind buffer 0), then the following pairs.
// A lane's operands of step t are in row 2 t + h of its column: the pair (2 G, 2 G + 1) is rows 4 G and 4 G + 2
// behind the lane's address.  The reads of pair G + 1 are issued before the MFMAs of pair G.
template <int BUF, int G>
__device__ __forceinline__ void pixel_dma_pairs(unsigned a_addr, unsigned b_addr, floatx2v (&a)[8], floatx2v (&b)[8], floatx16 &acc)
{
    if constexpr (G == 0) {
        a[0] = lds_read2_rows64<32 * BUF, 32 * BUF + 2>(a_addr);
        b[0] = lds_read2_rows64<32 * BUF, 32 * BUF + 2>(b_addr);
    }
    if constexpr (G + 1 < 8) {
        a[G + 1] = lds_read2_rows64<32 * BUF + 4 * (G + 1), 32 * BUF + 4 * (G + 1) + 2>(a_addr);
        b[G + 1] = lds_read2_rows64<32 * BUF + 4 * (G + 1), 32 * BUF + 4 * (G + 1) + 2>(b_addr);
        lds_wait<2>(a[G], b[G]);
    } else {
        lds_wait<0>(a[G], b[G]);
    }
    acc = mfma32(a[G].x, b[G].x, acc);
    acc = mfma32(a[G].y, b[G].y, acc);
    if constexpr (G + 1 < 8) pixel_dma_pairs<BUF, G + 1>(a_addr, b_addr, a, b, acc);
}

// 64 x 64 tile, 2 x 2 waves of one 32x32 block each, P.dNC = N / 32.
// TRIM = false: Sk-dilated before its V2 (Algorithm 3), for the ablation -- every tap visits all (oh,ow), and a
// chunk whose leaped-to X pixel lies outside the input is fetched through a descriptor of zero length, i.e. as zeros.
template <bool TRIM = true>
__global__ void __launch_bounds__(kThreads) pixel_gemm_dma(const PixelGemmParams P)
{
    constexpr int BM = 64, BN = 64, KC = kPixelDmaKC;

    extern __shared__ __align__(16) float smem[];
    float *As = smem;                 // [2][32][64]   dY rows
    float *Bs = smem + 2 * KC * BM;   // [2][32][64]   X rows

    const int work = xcd_contiguous_work(blockIdx.x, P.perXcd);
    if (work >= P.total) return;
    const int q1 = fdiv(work, P.dNT), nt = work - q1 * P.nTiles;
    const int q2 = fdiv(q1, P.dMT), mt = q1 - q2 * P.mTiles;
    const int z = fdiv(q2, P.dTaps), tap = q2 - z * P.dTaps.d;
    const int fh = fdiv(tap, P.dFW), fw = tap - fh * P.FW;
    const int m0 = mt * BM, n0 = nt * BN;

    // Algorithm 3B: the (oh,ow) whose X element exists for this tap (see pixel_gemm_fast)
    const int ih_s = fh - P.ph, iw_s = fw - P.pw;
    const int shiftK = P.FH + P.FW;
    auto cdiv_s = [&](int a, const FastDiv &d) { return fdiv(a + shiftK * d.d + d.d - 1, d) - shiftK; };
    const int oh_s = TRIM ? max(cdiv_s(-ih_s, P.dSh), 0) : 0, oh_e = TRIM ? min(P.OH, cdiv_s(P.IH - ih_s, P.dSh)) : P.OH;
    const int ow_s = TRIM ? max(cdiv_s(-iw_s, P.dSw), 0) : 0, ow_e = TRIM ? min(P.OW, cdiv_s(P.IW - iw_s, P.dSw)) : P.OW;
    const int nOH = max(oh_e - oh_s, 0), nOW = max(ow_e - ow_s, 0);
    const int NC = P.dNC.d;                        // chunks per (oh,ow): N / 32
    const int Ct = nOH * nOW * NC;                 // chunks of this tap
    // segment z of G_Z: the chunks are dealt evenly, the first Ct mod G_Z segments get one more
    const int seg = fdiv(Ct, P.dGZ), extra = Ct - seg * P.GZ;
    const int cbeg = z * seg + min(z, extra), T = seg + (z < extra ? 1 : 0);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int h = lane >> 5, l32 = lane & 31;

    // global side: load q of this wave fills k-rows 4 * (2 wave + q) .. + 3; lane l: k-row + l / 16, LDS piece position
    // l % 16, global piece (l % 16) ^ (8 * (k & 1)).  Channels past the end are clamped (loaded twice, never stored).
    unsigned va[2], vb[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int k = 4 * (2 * wave + q) + (lane >> 4);
        const int piece = (lane & 15) ^ (8 * (k & 1));
        va[q] = (unsigned)((k * P.OH * P.OW * P.OC + min(m0 + 4 * piece, P.OC - 4)) * 4);
        vb[q] = (unsigned)((k * P.IH * P.IW * P.IC + min(n0 + 4 * piece, P.IC - 4)) * 4);
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
    auto gload = [&](int buf) {   // buf is a literal at every call
        const int oh = oh_s + pa_, ow = ow_s + pb_, n1 = nch * KC;
        const int sa = (((n1 * P.OH + oh) * P.OW + ow) * P.OC) * 4;
        const int sb = (((n1 * P.IH + oh * P.sh + ih_s) * P.IW + ow * P.sw + iw_s) * P.IC) * 4;
        // untrimmed: a pixel outside the input is read through a descriptor of length 0 (wave-uniform: one scalar select)
        const bool inside = TRIM || ((unsigned)(oh * P.sh + ih_s) < (unsigned)P.IH && (unsigned)(ow * P.sw + iw_s) < (unsigned)P.IW);
        const __amdgpu_buffer_rsrc_t rsBc = TRIM ? rsB : __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(P.X), 0, __builtin_amdgcn_readfirstlane(inside ? -1 : 0), 0x00020000);
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            load16_to_lds(rsA, As + buf * KC * BM + (2 * wave + q) * 256, va[q], sa);
            load16_to_lds(rsBc, Bs + buf * KC * BN + (2 * wave + q) * 256, vb[q], sb);
        }
        if (++nch == NC) { nch = 0; if (++pb_ == nOW) { pb_ = 0; ++pa_; } }
    };

    // LDS side: this lane's column, row h of buffer 0 (rows are immediates from there)
    const unsigned a_addr = (unsigned)(size_t)(lds_float_t *)(As + h * BM + ((wm * 32 + l32) ^ (32 * h)));
    const unsigned b_addr = (unsigned)(size_t)(lds_float_t *)(Bs + h * BN + ((wn * 32 + l32) ^ (32 * h)));

    floatx16 acc[1][1];
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[0][0][r] = 0.f;

    auto compute = [&](auto buf_c) {
        floatx2v a[8], b[8];
        pixel_dma_pairs<decltype(buf_c)::value, 0>(a_addr, b_addr, a, b, acc[0][0]);
    };
    using B0 = std::integral_constant<int, 0>;
    using B1 = std::integral_constant<int, 1>;
    auto chunk_end = [&]() {
        vmem_wait_all();
        __syncthreads();
    };

    if (T > 0) {
        const int odd = T & 1;
        if (odd) gload(1); else gload(0);
        chunk_end();
        int t = 0;
        if (odd) {
            if (T > 1) gload(0);
            compute(B1{});
            chunk_end();
            t = 1;
        }
        for (; t < T; t += 2) {
            gload(1);                       // chunk t + 1 exists: T - t is even
            compute(B0{});
            chunk_end();
            if (t + 2 < T) gload(0);
            compute(B1{});
            chunk_end();
        }
    }

    wgrad_tile_epilogue<1, 1, 2, 2, 1>(acc, smem, P, z, tap, m0, n0, wm, wn, 0, lane);
}

}  // namespace cks
