// KS-deconv (Algorithm 2 Stage 2&3 / Algorithm 2B) for image stems -- very few input channels, a large filter, a
// stride above 1 -- on the 4x4x1 matrix instruction.
//
// With IC = 3 the s*s sub-convolutions of kernel split have three output columns each: a 16- or 32-wide MFMA tile
// would be a fifth full.  v_mfma_f32_4x4x1_16b_f32 multiplies sixteen independent 4x1 by 1x4 blocks; with its A
// operand broadcast from one block (cbsz = 4, abid = b) it computes, in every lane,
//
//     D[i][lane] += A[4 b + i] * B[lane],      i = 0..3
//
// i.e. four outputs per lane from one B value per lane, at the full fp32 matrix rate.  Here a lane is a dY column
// (ow), B is dY[n, oh, ow, oc] and the four A values are four consecutive "columns" (fh, fw, ic) of W[oc]: the
// products W[oc, fh, fw, ic] * dY[n, oh, ow, oc] are exactly the real-tap, real-element products of KS-deconv, laid
// out tap-stationary: P[(fh, fw, ic)][ow].  One A register holds the four columns of 16 output channels (one per
// block), so a chunk of 16 output channels is 16 instructions per group of four columns with b as an immediate.
//
// Stage 3 (dX[s oh - p + fh, s ow - p + fw, ic] = sum of P) is done where it is cheapest:
//   * down the rows in the accumulators themselves.  A wave sweeps its 64 columns from the top of the image to the
//     bottom; row oh + 1 adds to the same dX row through filter row fh - s what row oh added through fh.  Columns
//     are ordered fh-major, CPF per filter row with CPF padded until s * CPF is a multiple of 4: the first
//     instruction of a row's group g then takes group g + s CPF / 4 of the previous row as its C operand, which
//     moves every partial sum s filter rows up while it is being added to.  After a row, the first s filter rows
//     hold finished dX rows.
//   * along the row between lanes, once per finished dX row: x = s q + r collects, for every fw = s d + r + pw, the
//     lane d to the left (ds_bpermute).  A wave owns the outputs of its lanes HL .. 63 - HR, whose neighbours it holds;
//     windows of 64 lanes advance by 64 - HL - HR over the line of all images' columns, so only every 61st column
//     (stem) is computed twice and nothing is ever added in memory: no workspace, no second launch, one thread per
//     dX element, a fixed order of every sum.
//
// Work is dealt in equal runs of consecutive (window, row) steps, one run per wave, one wave per SIMD (the kernel
// holds the whole filter, 4 x NG registers, NG accumulators of 4 and two chunks of dY).  A run that starts inside an
// image first visits the up to NB - 1 rows above it for the filter rows that reach into its own dX rows, and one
// that ends inside an image skips the filter rows that reach below it: blocks of s filter rows are switched on and
// off by a wave-uniform mask, so no product is computed twice.
//
// What limits it (measured with per-wave time stamps and a probe of the instruction mix): next to back-to-back
// 8-cycle matrix instructions, whose operands keep the register file busy, every other instruction that moves a
// vector register costs matrix time -- a vector ALU instruction or an LDS write about 10 cycles, a 16-byte load
// about 30, a store about 60, reading an accumulator that was just written about 30 -- and a wave alone on its SIMD
// hides none of it.  A row is 2496 matrix instructions (19 968 cycles) and takes 23 300: the lane exchange and the
// stores of the finished rows (about 2 000; they are issued in two steps a chunk apart, because the exchange has a
// long latency) and the loads and block branches of the four chunks (about 1 300).  Variants that were measured and
// are not here: fetching dY once per d with shifted addresses and keeping the sums output-aligned (no exchange, but
// four times the loads: the texture addresser becomes the bottleneck, 173 us against 150) and passing dY through an
// LDS tile for that (the tile traffic costs what the exchange did, 170 us).
#pragma once
#include "cks_device.h"

namespace cks {

struct SweepDeconvParams {
    const float *dY, *W;
    float *dX;
    int N, OH, OW, OC, IH, IW, ph;
    int OWv;        // columns per image in the line of all columns: max(OW, ceil(IW / s)); columns >= OW hold no dY
    int nWin;       // windows of 64 lanes over that line
    int per, rem;   // rows (window-major) per wave: per, the first rem waves one more
    FastDiv dOWv, dOH;
};

template <int FH, int FW, int S, int PW, int IC, int OCQ>
struct SweepShape {
    static constexpr int cpf() { int c = FW * IC; while ((S * c) % 4 != 0) ++c; return c; }
    static constexpr int CPF = cpf();             // columns per filter row (padded)
    static constexpr int NCOL = FH * CPF;
    static constexpr int NG = (NCOL + 3) / 4;     // groups of 4 columns: one accumulator of 4 registers each
    static constexpr int SG = S * CPF / 4;        // groups per block of S filter rows
    static constexpr int NB = (FH + S - 1) / S;   // blocks
    // x = S q + r takes fw = S d + r + PW from lane q - d
    static constexpr bool has(int r, int fw) { return ((fw - r - PW) % S + S) % S == 0; }
    static constexpr int delta(int r, int fw) { return (fw - r - PW) / S; }   // exact where has(r, fw)
    static constexpr int dmax() { int m = 0; for (int r = 0; r < S; ++r) for (int fw = 0; fw < FW; ++fw) if (has(r, fw) && delta(r, fw) > m) m = delta(r, fw); return m; }
    static constexpr int dmin() { int m = 0; for (int r = 0; r < S; ++r) for (int fw = 0; fw < FW; ++fw) if (has(r, fw) && delta(r, fw) < m) m = delta(r, fw); return m; }
    static constexpr int HL = dmax(), HR = -dmin();
    static constexpr int ADV = 64 - HL - HR;      // lanes a window owns
    static_assert(PW < FW && HL + HR < 32 && NG * 4 <= 200, "shape outside what the kernel holds in registers");
};

template <int ABID>
__device__ __forceinline__ floatx4 mfma4_bcast(float a, float b, floatx4 c)
{
    return __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, c, 4, ABID, 0);
}
// (the block number is an immediate of the instruction)
__device__ __forceinline__ floatx4 mfma4_bcast_n(int abid, float a, float b, floatx4 c)
{
    switch (abid) {
        case 0: return mfma4_bcast<0>(a, b, c);
        case 1: return mfma4_bcast<1>(a, b, c);
        case 2: return mfma4_bcast<2>(a, b, c);
        case 3: return mfma4_bcast<3>(a, b, c);
        case 4: return mfma4_bcast<4>(a, b, c);
        case 5: return mfma4_bcast<5>(a, b, c);
        case 6: return mfma4_bcast<6>(a, b, c);
        case 7: return mfma4_bcast<7>(a, b, c);
        case 8: return mfma4_bcast<8>(a, b, c);
        case 9: return mfma4_bcast<9>(a, b, c);
        case 10: return mfma4_bcast<10>(a, b, c);
        case 11: return mfma4_bcast<11>(a, b, c);
        case 12: return mfma4_bcast<12>(a, b, c);
        case 13: return mfma4_bcast<13>(a, b, c);
        case 14: return mfma4_bcast<14>(a, b, c);
        default: return mfma4_bcast<15>(a, b, c);
    }
}

// 16 output channels of one dY row into the accumulators.  FIRST: the row's first chunk, which also moves every
// partial sum S filter rows up (C operand = the group one block further down; past the last filter row: zero).
// Blocks are processed upwards, so a block reads its lower neighbour before that one is overwritten.
// `between(blk)` is called before block blk: the caller issues the next chunk's loads there, one at a time, so that
// they do not queue up behind each other in front of the matrix instructions.
template <typename G, bool FIRST, typename Between>
__device__ __forceinline__ void sweep_chunk(floatx4 (&acc)[G::NG], const float (&w)[G::NG], const floatx4 (&b)[4], unsigned mask, Between between)
{
#pragma unroll
    for (int blk = 0; blk < G::NB; ++blk) {
        between(blk);
        if (mask & (1u << blk)) {   // wave-uniform
#pragma unroll
            for (int o = 0; o < 16; ++o) {
#pragma unroll
                for (int g = blk * G::SG; g < (blk + 1) * G::SG && g < G::NG; ++g) {
                    floatx4 c = acc[g];
                    if (FIRST && o == 0) {
                        if (g + G::SG < G::NG) c = acc[g + G::SG];
                        else c = floatx4{0.f, 0.f, 0.f, 0.f};
                    }
                    acc[g] = mfma4_bcast_n(o, w[g], b[o >> 2][o & 3], c);
                }
            }
        }
    }
}

template <int FH, int FW, int S, int PW, int IC, int OCQ>
__global__ void __launch_bounds__(kThreads) sweep_deconv(const SweepDeconvParams P)
{
    using G = SweepShape<FH, FW, S, PW, IC, OCQ>;
    constexpr int NG = G::NG, SG = G::SG, NB = G::NB, CPF = G::CPF, HL = G::HL, HR = G::HR;
    constexpr int OC = 16 * OCQ;
    static_assert(OCQ % 2 == 0, "the chunks of a row alternate between two register sets");

    const int lane = threadIdx.x & 63;
    const int wid = blockIdx.x * (kThreads / 64) + __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    int p = wid * P.per + min(wid, P.rem);
    const int end = p + P.per + (wid < P.rem ? 1 : 0);

    // The filter goes through LDS once, in the kernel's column order with the padding columns as zeros:
    // wl[oc][4 NG].  The A operand of group g for the 16 output channels of chunk q is, in lane 4 b + i,
    // wl[16 q + b][4 g + i]; every wave then keeps its OCQ x NG operands in registers.  (Each wave gathering
    // them from global memory cost the four waves of a compute unit 600 scattered loads: 8 us.)
    constexpr int WROW = 4 * NG;
    __shared__ float wl[OC * WROW];
    {
        // (all loads first, then all stores: one trip through memory instead of one per element)
        constexpr int PER = (OC * WROW + kThreads - 1) / kThreads;
        float v[PER];
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            const int i = threadIdx.x + k * kThreads;
            const int oc = i / WROW, col = i - oc * WROW, fh = col / CPF, rem = col - fh * CPF;
            v[k] = i < OC * WROW && fh < FH && rem < FW * IC ? P.W[(oc * FH + fh) * (FW * IC) + rem] : 0.f;
        }
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            const int i = threadIdx.x + k * kThreads;
            if (i < OC * WROW) wl[i] = v[k];
        }
    }
    __syncthreads();
    if (p >= end) return;
    const float *wlane = wl + (lane >> 2) * WROW + (lane & 3);
    float w[OCQ][NG];
#pragma unroll
    for (int q = 0; q < OCQ; ++q)
#pragma unroll
        for (int g = 0; g < NG; ++g) w[q][g] = wlane[q * 16 * WROW + 4 * g];

    const __amdgpu_buffer_rsrc_t rsY = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(P.dY), 0, P.N * P.OH * P.OW * OC * 4, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsX = __builtin_amdgcn_make_buffer_rsrc(P.dX, 0, P.N * P.IH * P.IW * IC * 4, 0x00020000);
    const int rowY = P.OW * OC * 4, rowX = P.IW * IC * 4;   // bytes

    floatx4 acc[NG];

    while (p < end) {
        // ---- a piece: rows [r0, r1) of window win
        const int win = fdiv(p, P.dOH), r0 = p - win * P.OH;
        const int r1 = min(P.OH, r0 + (end - p));
        const bool runEnds = r1 < P.OH;   // the rows below are another wave's

        const int c = win * G::ADV - HL + lane;
        const bool valid = c >= 0 && c < P.N * P.OWv;
        const int cc = valid ? c : 0;
        const int n = fdiv(cc, P.dOWv), ow = cc - n * P.OWv;
        const unsigned ldoff = valid && ow < P.OW ? (unsigned)(((n * P.OH) * P.OW + ow) * OC * 4) : 0x80000000u;   // out of range: reads 0
        const bool owner = valid && lane >= HL && lane < 64 - HR;
        const int stbase = ((n * P.IH) * P.IW + S * ow) * IC * 4;

#pragma unroll
        for (int g = 0; g < NG; ++g) acc[g] = floatx4{0.f, 0.f, 0.f, 0.f};

        // 4 of the 16 output channels of chunk q of row oh
        auto loadB = [&](floatx4 (&b)[4], int oh, int q, int j) {
            b[j] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rsY, ldoff, oh * rowY + q * 64 + 16 * j, 0));
        };

        // A finished block of S dX rows (row t = S oh + fh - ph) is composed along the row and stored in two steps
        // with a chunk of the next row between them: the exchange between lanes has a long latency and this wave is
        // alone on its SIMD.  take(): every column of the block to the lane that adds it (x = S q + r takes
        // fw = S d + r + PW from lane q - d); the accumulators may be overwritten once it is issued.
        float moved[S][FW * IC];
        auto take = [&]() {
#pragma unroll
            for (int fh = 0; fh < S; ++fh)
#pragma unroll
                for (int fw = 0; fw < FW; ++fw) {
                    int d = 0;
#pragma unroll
                    for (int r = 0; r < S; ++r) if (G::has(r, fw)) d = G::delta(r, fw);
#pragma unroll
                    for (int ic = 0; ic < IC; ++ic) {
                        const int col = fh * CPF + fw * IC + ic;
                        float v = acc[col / 4][col % 4];
                        if (d != 0) v = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(((lane - d) & 63) * 4, __builtin_bit_cast(int, v)));
                        moved[fh][fw * IC + ic] = v;
                    }
                }
        };
        // put(): add and store what take() moved for row block oh; part = fh * S + r, or all parts (-1)
        auto put = [&](int oh, int part) {
#pragma unroll
            for (int fh = 0; fh < S; ++fh) {
                const int t = S * oh + fh - P.ph;
                if (t < 0 || t >= P.IH) continue;   // wave-uniform
#pragma unroll
                for (int r = 0; r < S; ++r) {
                    if (part >= 0 && part != fh * S + r) continue;
                    float out[IC];
#pragma unroll
                    for (int ic = 0; ic < IC; ++ic) out[ic] = 0.f;
#pragma unroll
                    for (int fw = 0; fw < FW; ++fw) {
                        if (!G::has(r, fw)) continue;
                        const int d = G::delta(r, fw);
                        const bool ok = ow - d >= 0 && ow - d < P.OWv;   // the neighbour is a column of the same image
#pragma unroll
                        for (int ic = 0; ic < IC; ++ic) out[ic] += d == 0 || ok ? moved[fh][fw * IC + ic] : 0.f;
                    }
                    const unsigned off = owner && S * ow + r < P.IW ? (unsigned)(stbase + r * IC * 4) : 0x80000000u;   // out of range: dropped
                    if constexpr (IC == 3) {
                        typedef unsigned uint3v __attribute__((ext_vector_type(3)));
                        __builtin_amdgcn_raw_buffer_store_b96(uint3v{__float_as_uint(out[0]), __float_as_uint(out[1]), __float_as_uint(out[2])}, rsX, off, t * rowX, 0);
                    } else {
#pragma unroll
                        for (int ic = 0; ic < IC; ++ic)
                            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(out[ic]), rsX, off, t * rowX + ic * 4, 0);
                    }
                }
            }
        };

        const int oh0 = max(r0 - (NB - 1), 0);
        floatx4 bA[4], bB[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) loadB(bA, oh0, 0, j);

        bool pending = false;   // take() of the row above has been issued, its put() has not
        auto row = [&](int oh, unsigned mask) {
            const bool takes = oh >= r0;
#pragma unroll
            for (int q = 0; q < OCQ; q += 2) {
                // The next chunk's operands are fetched before the blocks of this one: of its 4 dY loads one before each
                // block (the rest, if there are fewer than 4 blocks, before the first), and the filter registers of a
                // block before that block.  So go the parts of the put() of the row above, in the row's second chunk,
                // and the take() of this row: before block 1 of its last chunk, when block 0 is finished.
                auto nextB = [&](int blk) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) if ((j < NB ? j : 0) == blk) loadB(bB, oh, q + 1, j);
                };
                if (q == 0) sweep_chunk<G, true>(acc, w[q], bA, mask, nextB);
                else sweep_chunk<G, false>(acc, w[q], bA, mask, nextB);
                auto nextA = [&](int blk) {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if ((j < NB ? j : 0) == blk) {
                            if (q + 2 < OCQ) loadB(bA, oh, q + 2, j);
                            else if (oh + 1 < r1) loadB(bA, oh + 1, 0, j);
                        }

                    if (q == 0 && pending) {
#pragma unroll
                        for (int part = 0; part < S * S; ++part) if ((part < NB ? part : 0) == blk) put(oh - 1, part);
                    }
                    if (q + 2 == OCQ && blk == (NB > 2 ? 2 : NB > 1 ? 1 : 0) && takes) take();
                };
                sweep_chunk<G, false>(acc, w[q + 1], bB, mask, nextA);
            }
            if (NB == 1 && takes) take();   // (a single block is finished only now)
            pending = takes;
        };
        for (int oh = oh0; oh < r1; ++oh) {
            // blocks [lo, hi): filter rows that reach dX rows of this run
            const int lo = max(r0 - oh, 0), hi = runEnds ? min(r1 - oh, NB) : NB;
            const unsigned mask = ((1u << hi) - 1u) & ~((1u << lo) - 1u);
            row(oh, mask);
        }
        if (pending) put(r1 - 1, -1);
        if (!runEnds) {
            // the bottom of the image: what the last rows left in the lower blocks, then rows nothing reaches (zeros)
            for (int oh = P.OH; S * oh - P.ph < P.IH; ++oh) {
#pragma unroll
                for (int g = 0; g < NG; ++g) {
                    if (g + SG < NG) acc[g] = acc[g + SG];
                    else acc[g] = floatx4{0.f, 0.f, 0.f, 0.f};
                }
                take();
                put(oh, -1);
            }
        }
        p += r1 - r0;
    }
}

}  // namespace cks
