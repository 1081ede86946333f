// ConvV2 for image stems whose geometry is known at compile time.
//
// With IC = 3 the filter row (fw, ic) that the per-position kernel contracts
// over is 21 floats; a tile of output pixels, however, reads a small dense
// strip of X.  This kernel stages that strip in LDS as it lies in memory -
// rows of the input, (TH-1)*s + FH of them, ((TW-1)*s + FW)*IC floats each -
// and lets the MFMA lanes pick the patch elements out of it:
//     Y[(th,tw), oc] = sum_{k=(fh,fw,ic)} strip[th*s + fh][(tw*s + fw)*IC + ic] * W[oc][k].
// The element of pixel (th,tw) for k is at  rowoff(th,tw) + fh*RP + (fw*IC+ic):
// a lane constant plus a constant of the K step, i.e. one ds_read_b32 with an
// immediate offset and no address arithmetic.  The strip holds zeros where it
// overlaps the padding, which is Algorithm 1's trimmed range realised per tile
// (a tile mixes positions with different trims); those zeros are written by
// the staging waves, X itself is read unpadded.  K runs over the J = FH*FW*IC
// real taps only (plus one zero if J is odd).
//
// Waves 0-3 (2 x 2 blocks of 32 pixels x 32 channels, 32x32x2 MFMA) multiply
// tile t while waves 4-7 fetch the strip of tile t+1 into the other buffer.  The
// filter slice W[oc0..oc0+64][J] stays in LDS for the life of the workgroup,
// which walks a contiguous range of tiles (tiles run down a band of TW columns,
// so successive strips overlap in L2).  Global accesses are buffer accesses
// "lane constant + scalar"; what falls outside a row or the tensor is out of
// range of its descriptor and reads as zero / is dropped.
#pragma once
#include "cks_device.h"

namespace cks {

struct StripFwdParams {
    const float *X;
    const float *W;
    float *Y;
    int N, IH, IW, OC, OH, OW, p;
    int nBands;         // ceil(OW / 16)
    int nRowTiles;      // ceil(OH / 4)
    int nT;             // 64-wide output-channel tiles
    int tiles;          // N * nBands * nRowTiles
    int tilesPerBlock;
};

constexpr int kStripThreads = 512;

template <int FH, int FW, int IC, int S>
struct StripGeo {
    static constexpr int TH = 4, TW = 16, IC_ = IC, S_ = S;
    static constexpr int L = FW * IC, J = FH * L, STEPS = (J + 1) / 2;
    static constexpr int SR = (TH - 1) * S + FH;              // strip rows
    static constexpr int SWF = ((TW - 1) * S + FW) * IC;      // strip floats per row
    static constexpr int PASSES = (SWF + 63) / 64;            // 64-lane passes that cover a row
    // Row pitch: SWF + 1 modulo the 64 banks (neighbouring rows then start 48 or 55 banks apart, which keeps the
    // MFMA lanes' reads conflict-free), and at least 64 * PASSES, so that the staging waves can write whole
    // passes without masking lanes (the floats past SWF are never read).
    static constexpr int RP = SWF + 1 + (64 * PASSES - (SWF + 1) + 63) / 64 * 64;
    static constexpr int SRA = (SR + 3) / 4 * 4;              // rows allocated: every staging wave the same number
    static constexpr int STRIP = SRA * RP + 1;                // + one word that stays zero
    static constexpr int LDW = (2 * STEPS) | 1;               // filter row pitch, odd: conflict-free column reads
    static constexpr size_t lds_bytes() { return (size_t)(64 * LDW + 2 * STRIP) * sizeof(float); }
};

// Staging of a tile's input strip by four waves: wave pw takes strip rows pw, pw+4, ..., lane l the
// floats l, l+64, ... of a row.  The image is one raw buffer, the row a scalar offset; floats that
// lie outside the row (left/right padding) carry an offset beyond the buffer and read as zero,
// rows outside the image are not read and staged as zeros.
// A wave that shares its SIMD with an MFMA wave gets an issue slot only every few dozen cycles, whatever
// the instruction, so this path is written for instruction count: a strip whose rows all lie inside the
// image (most) is fetched without per-row tests, and the LDS writes are unconditional.
template <class G>
struct StripStager {
    static constexpr int RROWS = G::SRA / 4;
    static constexpr int kBeyond = (int)0x80000000u;
    float v[RROWS][G::PASSES];
    int voff[G::PASSES], vlast[G::PASSES];   // byte offsets of this lane's floats in an image row; the same for the wave's last row
    int band = -1, img = -1;
    __amdgpu_buffer_rsrc_t rs;   // image img of X

    // tile = (image n, band c of 16 output columns, row tile t of 4 output rows); all wave-uniform
    __device__ __forceinline__ void fetch(const float *X, int n, int c, int t, int pw, int lane, int IH, int IW, int p)
    {
        const int rowFloats = IW * G::IC_;
        if (c != band) {   // uniform: where this band's strip floats lie in an image row
            band = c;
            const int x0 = (c * 16 * G::S_ - p) * G::IC_;
#pragma unroll
            for (int q = 0; q < G::PASSES; ++q) {
                const int x = lane + 64 * q;
                voff[q] = (x < G::SWF && x0 + x >= 0 && x0 + x < rowFloats) ? (x0 + x) * 4 : kBeyond;
                vlast[q] = pw + 4 * (RROWS - 1) < G::SR ? voff[q] : kBeyond;   // (the rows past SR exist in LDS only)
            }
        }
        if (n != img) {   // uniform: one descriptor per image
            img = n;
            rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(X) + (long)n * IH * rowFloats, 0, IH * rowFloats * 4, 0x00020000);
        }
        const int ih0 = 4 * t * G::S_ - p, rowB = rowFloats * 4;
        static_assert(4 * (RROWS - 1) < G::SR, "only a wave's last row can lie past the strip");
        if (ih0 >= 0 && ih0 + G::SR <= IH) {
            // straight-line: a lane that has nothing to fetch carries an offset beyond the image, and the
            // range check looks at that offset only, so the row offset of a row past SR does no harm
            int soff = (ih0 + pw) * rowB;
#pragma unroll
            for (int j = 0; j < RROWS; ++j, soff += 4 * rowB)
#pragma unroll
                for (int q = 0; q < G::PASSES; ++q)
                    v[j][q] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, j == RROWS - 1 ? vlast[q] : voff[q], soff, 0));
            return;
        }
#pragma unroll
        for (int j = 0; j < RROWS; ++j) {
            const int ih = ih0 + pw + 4 * j;
            const bool in = pw + 4 * j < G::SR && ih >= 0 && ih < IH;   // uniform
#pragma unroll
            for (int q = 0; q < G::PASSES; ++q)
                v[j][q] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, in ? voff[q] : kBeyond, in ? ih * rowB : 0, 0));
        }
    }
    // strip: start of the strip buffer to fill.  Whole passes and all RROWS rows are written: what lies
    // past SWF or SR is never read.
    __device__ __forceinline__ void stage(float *strip, int pw, int lane) const
    {
        float *dst = strip + pw * G::RP + lane;
#pragma unroll
        for (int j = 0; j < RROWS; ++j)
#pragma unroll
            for (int q = 0; q < G::PASSES; ++q) dst[4 * j * G::RP + 64 * q] = v[j][q];
    }
};

// The K loop, unrolled in groups of kStripGroup steps: the LDS reads of group g+1 are issued, then
// the MFMAs of group g (order pinned; the compiler would sink each read to its use).  Every read
// is "lane constant + immediate".
constexpr int kStripGroup = 6;   // 12 reads in flight: the LDS counter tracks at most 15
template <class G, int GI>
struct StripKLoop {
    static constexpr int BEG = GI * kStripGroup;
    static constexpr int END = BEG + kStripGroup < G::STEPS ? BEG + kStripGroup : G::STEPS;
    static constexpr int NEXT_END = END + kStripGroup < G::STEPS ? END + kStripGroup : G::STEPS;
    __device__ static __forceinline__ void load(float *av, float *bv, int beg, int end, const float *a_same,
                                                const float *a_wrap, const float *a_last, const float *b_ptr)
    {
#pragma unroll
        for (int t = beg; t < end; ++t) {
            const int k0 = 2 * t, fh0 = k0 / G::L, j0 = k0 % G::L;
            const float *ap = (k0 + 1 >= G::J) ? a_last : (j0 + 1 < G::L ? a_same : a_wrap);
            av[t] = ap[fh0 * G::RP + j0];
            bv[t] = b_ptr[k0];
        }
    }
    __device__ static __forceinline__ void run(float *av, float *bv, floatx16 &acc, const float *a_same, const float *a_wrap,
                                               const float *a_last, const float *b_ptr)
    {
        if constexpr (GI == 0) {
            load(av, bv, BEG, END, a_same, a_wrap, a_last, b_ptr);
            __builtin_amdgcn_sched_group_barrier(0x100, 2 * (END - BEG), 0);
        }
        if constexpr (END < G::STEPS) load(av, bv, END, NEXT_END, a_same, a_wrap, a_last, b_ptr);
#pragma unroll
        for (int t = BEG; t < END; ++t) acc = mfma32(av[t], bv[t], acc);
        if constexpr (END < G::STEPS) __builtin_amdgcn_sched_group_barrier(0x100, 2 * (NEXT_END - END), 0);
        __builtin_amdgcn_sched_group_barrier(0x008, END - BEG, 0);
        if constexpr (END < G::STEPS) StripKLoop<G, GI + 1>::run(av, bv, acc, a_same, a_wrap, a_last, b_ptr);
    }
};

template <int FH, int FW, int IC, int S>
__global__ void __launch_bounds__(kStripThreads) strip_fwd(const StripFwdParams P)
{
    using G = StripGeo<FH, FW, IC, S>;
    constexpr int L = G::L, J = G::J, RP = G::RP, STRIP = G::STRIP, LDW = G::LDW;
    constexpr int kBeyond = (int)0x80000000u;   // an offset outside every descriptor used here
    extern __shared__ __align__(16) float smem[];
    float *Ws = smem;                 // [64][LDW]
    float *Ss = smem + 64 * LDW;      // [2][STRIP]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nt = blockIdx.x % P.nT, g = blockIdx.x / P.nT;
    const int oc0 = nt * 64;
    const int tile_beg = g * P.tilesPerBlock, tile_end = min(tile_beg + P.tilesPerBlock, P.tiles);
    if (tile_beg >= tile_end) return;

    for (int i = tid; i < 64 * LDW + 2 * STRIP; i += kStripThreads) smem[i] = 0.f;
    __syncthreads();
    for (int i = tid; i < 64 * J; i += kStripThreads) {
        const int r = i / J, j = i - r * J;
        if (oc0 + r < P.OC) Ws[r * LDW + j] = P.W[(long)(oc0 + r) * J + j];
    }

    // tile index -> (image, band, row tile); row tiles fastest, so a workgroup runs down a band.  Decoded once;
    // every wave then advances its own cursor (divisions by kernel arguments run on the vector ALU).
    int cn, cc, ct;
    {
        ct = tile_beg % P.nRowTiles;
        const int q = tile_beg / P.nRowTiles;
        cc = q % P.nBands;
        cn = q / P.nBands;
    }
    auto advance = [&]() {
        if (++ct == P.nRowTiles) { ct = 0; if (++cc == P.nBands) { cc = 0; ++cn; } }
    };

    if (wave >= 4) {
        // ---------------------------------------------------------------- staging waves
        const int pw = wave - 4;
        StripStager<G> stager;
        int ftile = tile_beg;   // the tile fetched next: the cursor's
        auto fetch = [&]() {
            if (ftile >= tile_end) return;   // uniform
            ++ftile;
            stager.fetch(P.X, __builtin_amdgcn_readfirstlane(cn), __builtin_amdgcn_readfirstlane(cc),
                         __builtin_amdgcn_readfirstlane(ct), pw, lane, P.IH, P.IW, P.p);
            advance();
        };
        auto stage = [&](int tile, int buf) {
            if (tile < tile_end) stager.stage(Ss + buf * STRIP, pw, lane);
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
        return;
    }

    // -------------------------------------------------------------------- MFMA waves
    // 32x32x2 MFMA: lane l supplies A[m = l%32][k = l/32] and B[k = l/32][n = l%32]; result
    // register r holds D[m = 8*(r/4) + 4*(l/32) + r%4][n = l%32].
    const int wm = wave >> 1, wn = wave & 1;
    const int m = wm * 32 + (lane & 31), h = lane >> 5;
    const int th = m >> 4, tw = m & 15;
    const int rowoff = th * S * RP + tw * S * IC;
    // K step t covers k = 2t (lanes 0-31) and 2t+1 (lanes 32-63).  Within a filter row the second
    // is the next float; at a row's last float it is the first float of the next strip row; past
    // the last tap it is the word that stays zero.
    const float *a_same = Ss + rowoff + h;
    const float *a_wrap = Ss + rowoff + h * (RP - (L - 1));
    constexpr int kLastImm = ((J - 1) / L) * RP + (J - 1) % L;
    const float *a_last = h ? Ss + (STRIP - 1) - kLastImm : Ss + rowoff;
    const float *b_ptr = Ws + (wn * 32 + (lane & 31)) * LDW + h;

    // Y: pixel (th, tw) of the tile is row oh0+th, column ow0+tw.  One descriptor per image, the tile row a
    // scalar offset; a lane whose channel or tile column does not exist carries an offset beyond the image
    // (set when the band changes: only a row's last band can be narrower than 16 columns).
    const int col = oc0 + wn * 32 + (lane & 31);
    int yoff[8];   // register r -> tile column 8*((r/4)%2) + 4h + r%4; tile row 2*wm + r/8
    int yimg = -1, yband = -1;
    __amdgpu_buffer_rsrc_t rsY;
    const int imgY = P.OH * P.OW * P.OC;   // floats of Y per image (the host checks: below 2 GiB)

    __syncthreads();
    for (int tile = tile_beg; tile < tile_end; ++tile) {
        const int sb = ((tile - tile_beg) & 1) * STRIP;
        floatx16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
        float av[G::STEPS], bv[G::STEPS];
        StripKLoop<G, 0>::run(av, bv, acc, a_same + sb, a_wrap + sb, a_last + sb, b_ptr);

        const int n = __builtin_amdgcn_readfirstlane(cn), c = __builtin_amdgcn_readfirstlane(cc),
                  tt = __builtin_amdgcn_readfirstlane(ct);
        advance();
        const int ow0 = c * 16;
        if (n != yimg) {   // uniform
            yimg = n;
            rsY = __builtin_amdgcn_make_buffer_rsrc(P.Y + (long)n * imgY, 0, imgY * 4, 0x00020000);
        }
        if (c != yband) {   // uniform
            yband = c;
            const int cols = min(16, P.OW - ow0);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int twe = 8 * (e >> 2) + 4 * h + (e & 3);
                yoff[e] = (col < P.OC && twe < cols) ? (twe * P.OC + col) * 4 : kBeyond;
            }
        }
        const int oh0 = 4 * tt + 2 * wm, rowB = P.OW * P.OC * 4;
        int soff = (oh0 * P.OW + ow0) * P.OC * 4;
#pragma unroll
        for (int half = 0; half < 2; ++half, soff += rowB) {
            if (oh0 + half < P.OH) {   // uniform (the scalar offset takes no part in the range check)
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[8 * half + e]), rsY, yoff[e], soff, 0);
            }
        }
        __syncthreads();
    }
}

}  // namespace cks
