// KS-deconv for layers with few input channels (image stems).
//
// Kernel split turns the input gradient into stride^2 small convolutions whose
// GEMMs have IC output columns each; with IC = 3 an MFMA tile would be 9 % full.
// This kernel therefore keeps the sub-kernels' arithmetic (only real filter taps
// meet real dY elements; no zero of the dilated dY is ever touched) but runs it
// tap-stationary: for a row of 16 dY pixels
//     P[ow, (fh,fw,ic)] = sum_oc dY[n,oh,ow,oc] * W[oc,fh,fw,ic]
// is one dense GEMM (rows = pixels, columns = J = FH*FW*IC, K = OC), and the
// composing phase of the paper's Stage 3 is
//     dX[n, oh*s-p+fh, ow*s-p+fw, ic] = sum over the (oh,fh), (ow,fw) that map there of P.
// Columns with equal (fh mod s, fw mod s) are one sub-kernel; their targets
// interleave exactly as the sub-kernels' outputs do.  The sum is separable and is
// taken in two steps, both in a fixed order (the result does not depend on timing):
//   1. along the row:  Q[oh][fh][x] = sum_{tb} P[v-tb, (fh, b+s*tb, ic)] for ring
//      float x = (v*s+b)*IC+ic, by the wave that computed P, through a wave-private
//      LDS scratch (the MFMA result layout has the addends in different lanes);
//   2. across rows:    dX row (ih+p) = sum_{fh = (ih+p) mod s, +s, ...} Q[(ih+p-fh)/s][fh],
//      by the staging waves when the sweep has passed the row, from a ring of Q rows.
// A band of 16 dY columns of one image is swept top to bottom, four dY rows (one
// per MFMA wave) per step; the steps of all bands, in order, are dealt to the
// workgroups in equal consecutive runs.  Neighbouring bands overlap in (FW - s) dX
// pixel columns, and a run that starts inside a band shares (FH - s) dX rows with
// the run above it: a workgroup writes its share of such columns and rows to small
// side buffers, and add_heads adds them to dX afterwards, so no two workgroups
// ever add to one address.
//
// Every global access is a buffer access "lane constant + scalar" against a
// per-row descriptor: rows and pixels outside the tensors fall outside the
// descriptor and read as zero or are dropped on store.
#pragma once
#include "cks_device.h"

namespace cks {

typedef float floatx4 __attribute__((ext_vector_type(4)));

struct ScatterDeconvParams {
    const float *dY;
    const float *W;     // OHWI
    float *dX;
    float *head;        // [N][nBands-1][IH][OVF]: a band's share of the columns it has in common with its left neighbour
    float *rowhead;     // [workgroups][HR][kScatterRP]: a workgroup's share of the rows its first segment has in
                        // common with the rows above (written only if that segment starts inside a band)
    int N, IC, IH, IW, OC, OH, OW, FH, FW, s, p;
    int nBands;         // ceil(OW / 16)
    int nTiles;         // ceil(OH / 4): steps of a band's sweep
    int nFlush;         // output steps of 4*s dX rows each that a whole band needs
    int steps;          // N * nBands * nTiles
    int stepsPerBlock;  // consecutive steps (band-major) a workgroup works through
    int SW;             // floats of a dX row a band writes (from its first touched float)
    int SWlast;         // the same for the last band (includes dX columns no pixel reaches)
    int OVF;            // floats per row shared with the left neighbour: max(FW - s, 0) * IC
    int HR;             // rows shared with the rows above: max(FH - s, 0)
    int slots;          // Q ring: dY rows kept
    int KP;             // OC rounded up to 16
};

constexpr int kScatterThreads = 512;       // 4 MFMA waves + 4 staging waves
constexpr int kScatterStemThreads = 768;   // 8 MFMA waves (two per dY row) + 4 staging waves
constexpr int kScatterLDK = 68;    // K <= 64, +4 keeps 16-row fragments conflict free
constexpr int kScatterPP = 20;     // scratch floats per column: 16 pixels + 4 (bank skew, keeps float4 alignment)
constexpr int kScatterRP = 128;    // floats per Q row
constexpr int kScatterMaxTB = 4;   // taps per sub-kernel row and column: ceil(FW / s), ceil(FH / s) <= 4
constexpr int kScatterStemSlots = 16;  // stem: depth of the Q ring (11 rows are needed; a power of two makes the slot a mask)
constexpr int kScatterStemKeep = 2;   // stem: K groups (of 4) whose filter fragments an MFMA wave keeps in registers
inline size_t scatter_deconv_lds_bytes(int NB, int slots, int FH)
{
    return ((size_t)NB * 16 * kScatterLDK + (size_t)4 * NB * 16 * kScatterPP + ((size_t)slots * FH + 1 + 4) * kScatterRP) * sizeof(float);
}

// One pass of a stem MFMA wave (OC = 64: four K groups of 16): NBH column blocks of P for its dY
// row, and step 1 for NFH filter rows of the row it computed in the previous pass (that P is still
// in the wave's scratch, which is overwritten only at the end of this pass).  The filter fragments
// of K group u+1 are requested before the MFMAs of group u are issued and one filter row's gather
// reads ride along with each group and are summed and written during the next one.  The order is
// pinned (the compiler would sink every read to its use), and never more than 15 LDS reads are
// outstanding at a wait, which is all the counter can express.  The fragments of the first kScatterStemKeep groups
// never change and stay in registers (wk): a pass starts its MFMAs without waiting for LDS.
//
// Step 1 on the stem: lane l of gather q takes pixel column 2v + q (v = l / 3) and channel l mod 3,
// so that its taps tb = 0 .. 3 - q sit at gs[q] + tb * (6 PP - 1) + fh * 21 PP: one lane constant,
// the rest immediates, and the 64 lanes of a read fall into 64 different banks.  A tap that reaches
// before pixel 0 or past pixel 15 of its column lands in pad slots, which stay zero.  The sum is
// float 6v + 3q + l mod 3 of the Q row (qrow points at float 6v + l mod 3).
template <int NBH, int NFH, bool MFMAS>
__device__ __forceinline__ void scatter_stem_pass(const float4 (&a)[4], const float4 (&wk)[kScatterStemKeep][6], const float *Bp,
                                                  const float *const (&gs)[2], float *qrow, float *Pst)
{
    constexpr int LDK = kScatterLDK, PP = kScatterPP, RP = kScatterRP, MAXTB = kScatterMaxTB;
    constexpr int TAP = 6 * PP - 1, FHS = 21 * PP;   // scratch floats from one tap / filter row to the next
    if constexpr (MFMAS) {
        floatx4 acc[NBH];
#pragma unroll
        for (int b = 0; b < NBH; ++b) acc[b] = floatx4{0.f, 0.f, 0.f, 0.f};
        constexpr int KEEP = kScatterStemKeep;
        static_assert(KEEP >= 1 && KEEP <= 3, "the first group's fragments are resident, the last group's are not");
        float4 wc[NBH], wn[NBH];
        float g[2][MAXTB];   // the addends of one filter row: summed and written during the next group
#pragma unroll
        for (int b = 0; b < NBH; ++b) wc[b] = wk[0][b];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const bool loads = u < 3 && u + 1 >= KEEP;   // the next group's fragments come from LDS
            const bool sums = u >= 1 && u - 1 < NFH, gathers = u < NFH;
            if (loads) {
#pragma unroll
                for (int b = 0; b < NBH; ++b) wn[b] = *reinterpret_cast<const float4 *>(Bp + b * 16 * LDK + 16 * (u + 1));
            } else if (u < 3) {
#pragma unroll
                for (int b = 0; b < NBH; ++b) wn[b] = wk[u + 1 < KEEP ? u + 1 : 0][b];
            }
            if (sums) {
                qrow[(u - 1) * RP] = (g[0][0] + g[0][1]) + (g[0][2] + g[0][3]);
                qrow[(u - 1) * RP + 3] = (g[1][0] + g[1][1]) + g[1][2];
            }
            if (gathers) {
#pragma unroll
                for (int q = 0; q < 2; ++q)
#pragma unroll
                    for (int tb = 0; tb < MAXTB - q; ++tb) g[q][tb] = gs[q][tb * TAP + u * FHS];
            }
#pragma unroll
            for (int b = 0; b < NBH; ++b) {
                acc[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u].x, wc[b].x, acc[b], 0, 0, 0);
                acc[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u].y, wc[b].y, acc[b], 0, 0, 0);
                acc[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u].z, wc[b].z, acc[b], 0, 0, 0);
                acc[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u].w, wc[b].w, acc[b], 0, 0, 0);
            }
            if (loads) __builtin_amdgcn_sched_group_barrier(0x100, NBH, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
            if (sums) {
                __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);
                __builtin_amdgcn_sched_group_barrier(0x200, 2, 0);
            }
            if (gathers) __builtin_amdgcn_sched_group_barrier(0x100, 2 * MAXTB - 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 4 * NBH - 8, 0);
#pragma unroll
            for (int b = 0; b < NBH; ++b) wc[b] = wn[b];
        }
        if constexpr (NFH == 4) {
            qrow[3 * RP] = (g[0][0] + g[0][1]) + (g[0][2] + g[0][3]);
            qrow[3 * RP + 3] = (g[1][0] + g[1][1]) + g[1][2];
        }
#pragma unroll
        for (int b = 0; b < NBH; ++b)
            *reinterpret_cast<float4 *>(Pst + b * 16 * PP) = float4{acc[b][0], acc[b][1], acc[b][2], acc[b][3]};
    } else {
        float g[NFH][2][MAXTB];
#pragma unroll
        for (int fh = 0; fh < NFH; ++fh)
#pragma unroll
            for (int q = 0; q < 2; ++q)
#pragma unroll
                for (int tb = 0; tb < MAXTB - q; ++tb) g[fh][q][tb] = gs[q][tb * TAP + fh * FHS];
#pragma unroll
        for (int fh = 0; fh < NFH; ++fh) {
            qrow[fh * RP] = (g[fh][0][0] + g[fh][0][1]) + (g[fh][0][2] + g[fh][0][3]);
            qrow[fh * RP + 3] = (g[fh][1][0] + g[fh][1][1]) + g[fh][1][2];
        }
    }
}

// NB: 16-column blocks of the GEMM (J <= 16 NB).  STEM: the geometry is the
// 7x7 / stride 2 / 3-channel stem, known at compile time, so that every LDS
// access of the composing steps is "lane constant + immediate".
template <int NB, bool STEM>
__global__ void __launch_bounds__(STEM ? kScatterStemThreads : kScatterThreads) scatter_deconv(const ScatterDeconvParams P)
{
    constexpr int THREADS = STEM ? kScatterStemThreads : kScatterThreads, NCW = THREADS / 64 - 4;   // MFMA waves
    constexpr int LDK = kScatterLDK, PP = kScatterPP, RP = kScatterRP, MAXTB = kScatterMaxTB;
    constexpr int kBeyond = (int)0x80000000u;   // an offset outside every descriptor used here
    const int FH = STEM ? 7 : P.FH, FW = STEM ? 7 : P.FW, IC = STEM ? 3 : P.IC, S = STEM ? 2 : P.s;
    const int SLOTS = STEM ? kScatterStemSlots : P.slots;
    extern __shared__ __align__(16) float smem[];
    float *Bs = smem;                           // [NB*16][LDK]       filter, column-major: Bs[j'][oc]
    float *Ps = Bs + NB * 16 * LDK;             // [4][NB*16][PP]     per-wave P scratch
    float *Qs = Ps + 4 * NB * 16 * PP;          // [slots][FH][RP]    ring of row-composed dY rows
    const float *Qzero = Qs + SLOTS * FH * RP;   // [RP]               stays zero

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int L = FW * IC, J = FH * L;
    const int rows4s = 4 * S;
    float *Qdump = Qs + (SLOTS * FH + 1) * RP;   // [4][RP] receives what must go nowhere

    // All of LDS starts at zero (pad columns, pad slots, the ring); then the filter, transposed.
    // stem: filter rows 0-3 are columns 0..83, rows 4-6 start at column 96 (one MFMA wave each);
    // its filter is requested before the zero fill so that the loads are all in flight at once.
    const int ldsFloats = NB * 16 * LDK + 4 * NB * 16 * PP + (SLOTS * FH + 1 + 4) * RP;   // a multiple of 4
    constexpr int WREGS = STEM ? (64 * 7 * 7 * 3 + THREADS - 1) / THREADS : 1;
    float wreg[WREGS];
    if constexpr (STEM) {
        const __amdgpu_buffer_rsrc_t rsW = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(P.W), 0, P.OC * J * 4, 0x00020000);
#pragma unroll
        for (int k = 0; k < WREGS; ++k)
            wreg[k] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsW, (tid + k * THREADS) * 4, 0, 0));   // past the end: 0
    }
    for (int i = tid; i < ldsFloats / 4; i += THREADS) reinterpret_cast<float4 *>(smem)[i] = float4{0.f, 0.f, 0.f, 0.f};
    __syncthreads();
    if constexpr (STEM) {
#pragma unroll
        for (int k = 0; k < WREGS; ++k) {
            const int i = tid + k * THREADS;
            const int oc = i / J, j = i - oc * J;
            if (i < P.OC * J) Bs[(j >= 4 * L ? j + (96 - 4 * L) : j) * LDK + oc] = wreg[k];
        }
    } else {
        for (int i = tid; i < P.OC * J; i += THREADS) {
            const int oc = i / J, j = i - oc * J;
            Bs[j * LDK + oc] = P.W[i];
        }
    }
    __syncthreads();

    // This workgroup's share of the sweep steps, cut into segments at band ends.  A segment
    // (band, steps [t0,t1)) composes the dX rows [4 t0 s, 4 t1 s + HR) (to the band's end if t1 is the
    // last step); of those, the first HR rows (if t0 > 0) also receive from the steps above and go to
    // rowhead, the last HR rows (if t1 is not the last step) are completed by the next segment's rowhead.
    const int u0 = blockIdx.x * P.stepsPerBlock, u1 = min(u0 + P.stepsPerBlock, P.steps);
    constexpr int DELAY = STEM ? 2 : 1;   // passes by which the output step trails a tile's MFMAs

    if (wave >= NCW) {
        // ------------------------------------------------------------ staging waves: step 2 and the stores
        // These waves issue few instructions, each of which would otherwise queue behind the MFMA
        // wave of the same SIMD.
        __builtin_amdgcn_s_setprio(3);
        const int pw = wave - NCW;
        const int rowFloats = P.IW * IC;
        for (int u = u0; u < u1;) {
            const int band = u / P.nTiles, t0 = u - band * P.nTiles, t1 = min(P.nTiles, t0 + (u1 - u));
            const int n = band / P.nBands, c = band - n * P.nBands;
            u += t1 - t0;
            // Q float x of this band is dX float (16 c s - p)*IC + x of its image row.  The image (and
            // the side buffers) are raw buffers, the row a scalar offset; lanes outside the row or not
            // written by this band carry an offset beyond them.
            const int sw = c == P.nBands - 1 ? P.SWlast : P.SW;
            const int x0 = (c * 16 * S - P.p) * IC;
            int voffX[2], voffH[2], voffR[2];
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int x = lane + 64 * q;
                const bool inrow = x < sw && x0 + x >= 0 && x0 + x < rowFloats;
                voffX[q] = (inrow && !(c > 0 && x < P.OVF)) ? (x0 + x) * 4 : kBeyond;
                voffH[q] = (c > 0 && x < P.OVF) ? x * 4 : kBeyond;
                voffR[q] = inrow ? x * 4 : kBeyond;
            }
            const __amdgpu_buffer_rsrc_t rsX =
                __builtin_amdgcn_make_buffer_rsrc(P.dX + (long)n * P.IH * rowFloats, 0, P.IH * rowFloats * 4, 0x00020000);
            const __amdgpu_buffer_rsrc_t rsH = __builtin_amdgcn_make_buffer_rsrc(
                P.head + ((long)n * (P.nBands - 1) + max(c - 1, 0)) * P.IH * P.OVF, 0, c > 0 ? P.IH * P.OVF * 4 : 0, 0x00020000);
            const __amdgpu_buffer_rsrc_t rsR = __builtin_amdgcn_make_buffer_rsrc(
                P.rowhead + (long)blockIdx.x * P.HR * RP, 0, t0 > 0 ? P.HR * RP * 4 : 0, 0x00020000);
            const bool last = t1 == P.nTiles;
            const int rowBeg = t0 * rows4s, rowEnd = last ? P.nFlush * rows4s : t1 * rows4s + P.HR;
            const int kEnd = (rowEnd + rows4s - 1) / rows4s;
            const int ohBeg = 4 * t0, ohEnd = min(P.OH, 4 * t1);
            // stem: output steps whose 8 rows all lie in the image and draw on dY rows of this segment
            // only (4k-3 .. 4k+3) need none of the checks below
            const int kFirst = max(t0 + 1, (P.p + 7) / 8);   // row 8k - p is not above the image
            const int kPlain = STEM ? min(t1, P.IH + P.p >= 8 ? (P.IH + P.p - 8) / 8 + 1 : 0) : 0;   // row 8k + 7 - p not below it
            for (int i = t0; i < kEnd + DELAY; ++i) {
                const int k = i - DELAY;   // rows [k*4s, (k+1)*4s) are complete once step 1 of tile k is done
                if (STEM && k >= kFirst && k < kPlain) {
                    float v0[2][MAXTB], v1[2][MAXTB];
#pragma unroll
                    for (int j = 0; j < 2; ++j) {   // rows 8k + pw and 8k + pw + 4 = oh*2 + fh: fh = (pw & 1) + 2t, oh = 4k + pw/2 + 2j - t
#pragma unroll
                        for (int t = 0; t < MAXTB; ++t) {
                            const int fh = (pw & 1) + 2 * t, slot = (4 * k + (pw >> 1) + 2 * j - t) & (kScatterStemSlots - 1);
                            const float *qp = (fh < 7 ? Qs + (slot * 7 + fh) * RP : Qzero) + lane;
                            v0[j][t] = qp[0];
                            v1[j][t] = qp[64];
                        }
                    }
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const int soff = (8 * k + pw + 4 * j - P.p) * rowFloats * 4, soffH = (8 * k + pw + 4 * j - P.p) * P.OVF * 4;
                        const float sum0 = (v0[j][0] + v0[j][1]) + (v0[j][2] + v0[j][3]);
                        const float sum1 = (v1[j][0] + v1[j][1]) + (v1[j][2] + v1[j][3]);
                        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(sum0), rsX, voffX[0], soff, 0);
                        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(sum1), rsX, voffX[1], soff, 0);
                        if (c > 0) {
                            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(sum0), rsH, voffH[0], soffH, 0);
                            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(sum1), rsH, voffH[1], soffH, 0);
                        }
                    }
                } else if (k >= t0) {
#pragma unroll 2
                    for (int r = pw; r < rows4s; r += 4) {
                        const int row = k * rows4s + r;   // = ih + p
                        const int ih = row - P.p;
                        if (row >= rowEnd || ih < 0 || ih >= P.IH) continue;   // uniform
                        // row = oh*s + fh: fh = r mod s + t*s, oh = 4k + r/s - t.  All reads are issued before
                        // the first add; a term that does not exist reads the zero row behind the ring.
                        const int fh0 = r % S, ohTop = 4 * k + r / S;
                        float v0[MAXTB], v1[MAXTB];
#pragma unroll
                        for (int t = 0; t < MAXTB; ++t) {
                            const int fh = fh0 + t * S, oh = ohTop - t;
                            const bool ok = fh < FH && oh >= ohBeg && oh < ohEnd;   // uniform
                            const float *qp = (ok ? Qs + ((oh % SLOTS) * FH + fh) * RP : Qzero) + lane;
                            v0[t] = qp[0];
                            v1[t] = qp[64];
                        }
                        const float sum0 = (v0[0] + v0[1]) + (v0[2] + v0[3]);
                        const float sum1 = (v1[0] + v1[1]) + (v1[2] + v1[3]);
                        if (t0 > 0 && row < rowBeg + P.HR) {
                            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(sum0), rsR, voffR[0], (row - rowBeg) * RP * 4, 0);
                            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(sum1), rsR, voffR[1], (row - rowBeg) * RP * 4, 0);
                        } else {
                            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(sum0), rsX, voffX[0], ih * rowFloats * 4, 0);
                            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(sum1), rsX, voffX[1], ih * rowFloats * 4, 0);
                            if (c > 0) {
                                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(sum0), rsH, voffH[0], ih * P.OVF * 4, 0);
                                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(sum1), rsH, voffH[1], ih * P.OVF * 4, 0);
                            }
                        }
                    }
                }
                __syncthreads();
            }
        }
        return;
    }

    // ---------------------------------------------------------------- MFMA waves: a wave owns dY row 4i + wrow of step i
    // 16x16x4 MFMA: lane l supplies A[m = l%16][k = l/16] and B[k = l/16][n = l%16];
    // result register r holds D[m = 4*(l/16) + r][n = l%16].
    // Stem: waves 0-3 take filter rows 0-3 (column blocks 0-5) of dY rows 0-3 of the step, waves 4-7
    // filter rows 4-6 (blocks 6-9): each SIMD then hosts two MFMA waves that fill each other's stalls.
    const int lm = lane & 15, lk = lane >> 4;
    const int KU = P.KP >> 4;
    const int wrow = STEM ? (wave & 3) : wave, half = STEM ? (wave >> 2) : 0;
    const int colBase = half ? 96 : 0, fhBase = half ? 4 : 0;
    // A straight from global: pixel lm, channels 16u + 4lk .. +3 (channels past OC are out of range)
    int a_voff[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) a_voff[u] = (16 * u + 4 * lk < P.OC) ? (lm * P.OC + 16 * u + 4 * lk) * 4 : kBeyond;
    float4 areg[4];
    // step 1, lane constants: ring float x = lane + 64q is pixel column pwx = x / IC (= v*s + b), channel ic
    float *Pw = Ps + (wrow * NB * 16 + colBase) * PP;   // this wave's columns of its row's scratch
    const float *gat[2][MAXTB];   // general geometry: one address per tap
    const float *gs[2];           // stem: one address per gather, see scatter_stem_pass
    int qx = lane;                // stem: the Q row float of this lane's first gather
    const int fhStride = L * PP;
    if constexpr (STEM) {
        // lanes past the last pixel column (l >= 57 / 54) sit at "pixel 19", from where every tap
        // reads a pad slot: their Q positions (dX floats no pixel reaches) hold zeros
        const int v = min(lane / 3, 19), ic = lane % 3;
#pragma unroll
        for (int q = 0; q < 2; ++q) gs[q] = Pw + (3 * q + ic) * PP + v;
        qx = 6 * v + ic;   // <= 116: the idle lanes all write their zeros to floats 114 .. 119
    } else {
        const int touched = (15 * S + FW) * IC;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int x = lane + 64 * q;
            const int pwx = x / IC, ic = x - pwx * IC, b = pwx % S, v = pwx / S;
#pragma unroll
            for (int tb = 0; tb < MAXTB; ++tb) {
                // column (fh=0, fw=b+s*tb, ic), pixel v-tb; + fh*L*PP selects the filter row.  A tap that does
                // not exist reads pad slot 16 of column fh*L instead, which is never written and stays zero.
                const bool ok = x < touched && b + S * tb < FW && v - tb >= 0 && v - tb < 16;
                gat[q][tb] = ok ? Pw + ((b + S * tb) * IC + ic) * PP + v - tb : Pw + 16;
            }
        }
    }
    float *Pst = Pw + lm * PP + 4 * lk;   // + b*16*PP: P[pixels 4lk..4lk+3][column 16b + lm]
    const float *Bp = Bs + (colBase + lm) * LDK + 4 * lk;
    float4 wk[kScatterStemKeep][6];   // stem: this wave's filter fragments of the first K groups (4 blocks in the second half)
    if constexpr (STEM) {
#pragma unroll
        for (int u = 0; u < kScatterStemKeep; ++u)
#pragma unroll
            for (int b = 0; b < 6; ++b)
                wk[u][b] = (b < 4 || half == 0) ? *reinterpret_cast<const float4 *>(Bp + b * 16 * LDK + 16 * u) : float4{0.f, 0.f, 0.f, 0.f};
    }

    for (int u = u0; u < u1;) {
        const int band = u / P.nTiles, t0 = u - band * P.nTiles, t1 = min(P.nTiles, t0 + (u1 - u));
        const int n = band / P.nBands, c = band - n * P.nBands;
        u += t1 - t0;
        const int ow0 = c * 16;
        const int a_bytes = min(16, P.OW - ow0) * P.OC * 4;
        auto fetch = [&](int i) {
            const int oh = 4 * i + wrow;
            const long off = (((long)n * P.OH + min(oh, P.OH - 1)) * P.OW + ow0) * P.OC;
            const __amdgpu_buffer_rsrc_t rs =
                __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(P.dY + off), 0, oh < P.OH ? a_bytes : 0, 0x00020000);
#pragma unroll
            for (int uu = 0; uu < 4; ++uu)
                areg[uu] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(rs, a_voff[uu], 0, 0));
        };
        const bool last = t1 == P.nTiles;
        const int rowEnd = last ? P.nFlush * rows4s : t1 * rows4s + P.HR;
        const int kEnd = (rowEnd + rows4s - 1) / rows4s;
        fetch(t0);
        if constexpr (STEM) {
            for (int i = t0; i < kEnd + DELAY; ++i) {
                // Q rows of dY row 4(i-1) + wrow.  In a segment's first pass the scratch holds nothing of
                // this segment: what is gathered goes to the dump row.
                float *qrow = (i > t0 ? Qs + (((4 * (i - 1) + wrow) % SLOTS) * 7 + fhBase) * RP : Qdump) + qx;
                if (i < t1) {   // uniform
                    float4 a[4];
#pragma unroll
                    for (int uu = 0; uu < 4; ++uu) a[uu] = areg[uu];
                    if (i + 1 < t1) fetch(i + 1);   // in flight during this step's MFMAs
                    if (half == 0) scatter_stem_pass<6, 4, true>(a, wk, Bp, gs, qrow, Pst);
                    else scatter_stem_pass<4, 3, true>(a, wk, Bp, gs, qrow, Pst);
                } else if (i == t1) {
                    // the segment's last dY rows: step 1 on its own
                    float4 a[4];
                    if (half == 0) scatter_stem_pass<6, 4, false>(a, wk, Bp, gs, qrow, Pst);
                    else scatter_stem_pass<4, 3, false>(a, wk, Bp, gs, qrow, Pst);
                }
                __syncthreads();
            }
        } else {
            for (int i = t0; i < kEnd + DELAY; ++i) {
                if (i < t1) {   // uniform
                    floatx4 acc[NB];
#pragma unroll
                    for (int b = 0; b < NB; ++b) acc[b] = floatx4{0.f, 0.f, 0.f, 0.f};
                    float4 a[4];
#pragma unroll
                    for (int uu = 0; uu < 4; ++uu) a[uu] = areg[uu];
                    if (i + 1 < t1) fetch(i + 1);   // in flight during this step's MFMAs
#pragma unroll
                    for (int uu = 0; uu < 4; ++uu) {
                        if (uu < KU) {
#pragma unroll
                            for (int b = 0; b < NB; ++b) {
                                const float4 w4 = *reinterpret_cast<const float4 *>(Bp + b * 16 * LDK + 16 * uu);
                                acc[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[uu].x, w4.x, acc[b], 0, 0, 0);
                                acc[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[uu].y, w4.y, acc[b], 0, 0, 0);
                                acc[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[uu].z, w4.z, acc[b], 0, 0, 0);
                                acc[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[uu].w, w4.w, acc[b], 0, 0, 0);
                            }
                        }
                    }
#pragma unroll
                    for (int b = 0; b < NB; ++b)
                        *reinterpret_cast<float4 *>(Pst + b * 16 * PP) = float4{acc[b][0], acc[b][1], acc[b][2], acc[b][3]};
                    // the scratch is private to this wave: its LDS accesses complete in order
                    float *qrow = Qs + (((4 * i + wrow) % SLOTS) * FH) * RP + lane;
                    for (int fh = 0; fh < FH; ++fh) {
#pragma unroll
                        for (int q = 0; q < 2; ++q) {
                            float sum = 0.f;
#pragma unroll
                            for (int tb = 0; tb < MAXTB; ++tb) sum += gat[q][tb][fh * fhStride];
                            qrow[fh * RP + 64 * q] = sum;
                        }
                    }
                }
                __syncthreads();
            }
        }
    }
}

// What the side buffers hold is added to dX by one launch, every dX element by one thread:
//   band part: dX[n, ih, (16 c s - p)*IC + x] += head[n][c-1][ih][x] for every band c >= 1, x < OVF;
//   row part:  dX rows [4 t0 s, 4 t0 s + HR) of the band a workgroup's first segment lies in += that
//              workgroup's rowhead, if the segment starts inside the band.
// Where a row head crosses the columns that two bands share, the band part's thread adds it as
// well (after head) and the row part leaves those columns alone.  The host has checked
// that at most one workgroup starts inside a band and that no two row heads meet in a dX element.
constexpr int kHeadFloats = 1;   // measured: more floats per thread (fewer, longer threads) is slower
struct HeadsParams {
    const float *head;
    const float *rowhead;   // null: no workgroup starts inside a band
    float *dX;
    int N, IC, IH, IW, s, p, nBands, nTiles, OVF, SW, SWlast, HR, stepsPerBlock, blocks;
    int rows;         // band part: N * (nBands-1) * IH rows of OVF floats (0 if there is no band part)
    int xwShift;      // a row is shared by 2^xwShift threads, kHeadFloats consecutive floats each
    int bandBlocks;   // workgroups of the band part; the row part's follow
    FastDiv dIH, dBandsLeft, dSteps;   // IH, nBands - 1, stepsPerBlock
};

__global__ void __launch_bounds__(kThreads) add_heads(const HeadsParams P)
{
    const int rowFloats = P.IW * P.IC;
    if ((int)blockIdx.x < P.bandBlocks) {
        const int row = blockIdx.x * (kThreads >> P.xwShift) + (threadIdx.x >> P.xwShift), x0 = (threadIdx.x & ((1 << P.xwShift) - 1)) * kHeadFloats;
        if (row >= P.rows || x0 >= P.OVF) return;
        const int t = fdiv(row, P.dIH), ih = row - t * P.IH;
        const int n = fdiv(t, P.dBandsLeft), c = t - n * (P.nBands - 1) + 1;
        const int col0 = (16 * c * P.s - P.p) * P.IC + x0;
        // row heads that cross these columns: of the workgroup that starts inside this band (from its
        // float 0) and of the one that starts inside the left neighbour (from its float 16 s IC)
        const float *rh[2] = {nullptr, nullptr};
        if (P.rowhead) {
#pragma unroll
            for (int side = 0; side < 2; ++side) {
                const int first = (n * P.nBands + c - side) * P.nTiles, g = fdiv(first, P.dSteps) + 1;   // first run starting after the band's first step
                if (g >= P.blocks) continue;
                const int t0 = g * P.stepsPerBlock - first, r = ih + P.p - t0 * 4 * P.s;
                if (t0 < P.nTiles && r >= 0 && r < P.HR) rh[side] = P.rowhead + ((long)g * P.HR + r) * kScatterRP + side * 16 * P.s * P.IC;
            }
        }
        const float *hp = P.head + (long)row * P.OVF;
        float *dp = P.dX + ((long)n * P.IH + ih) * rowFloats;
        // every load before the first store: the compiler cannot know that the buffers are distinct
        float v[kHeadFloats], d[kHeadFloats];
        bool ok[kHeadFloats];
#pragma unroll
        for (int j = 0; j < kHeadFloats; ++j) {
            const int x = x0 + j, col = col0 + j;
            ok[j] = x < P.OVF && col >= 0 && col < rowFloats;
            v[j] = ok[j] ? hp[x] : 0.f;
            d[j] = ok[j] ? dp[col] : 0.f;
            if (ok[j] && rh[0]) v[j] += rh[0][x];
            if (ok[j] && rh[1]) v[j] += rh[1][x];
        }
#pragma unroll
        for (int j = 0; j < kHeadFloats; ++j)
            if (ok[j]) dp[col0 + j] = d[j] + v[j];
        return;
    }
    const int per = kThreads / kScatterRP;   // rows per workgroup
    const int hr = (blockIdx.x - P.bandBlocks) * per + threadIdx.x / kScatterRP, x = threadIdx.x % kScatterRP;
    if (hr >= P.blocks * P.HR) return;
    const int g = hr / P.HR, r = hr - g * P.HR;
    const int u0 = g * P.stepsPerBlock;
    const int band = u0 / P.nTiles, t0 = u0 - band * P.nTiles;
    if (t0 == 0) return;
    const int n = band / P.nBands, c = band - n * P.nBands;
    const int ih = t0 * 4 * P.s + r - P.p;
    const int sw = c == P.nBands - 1 ? P.SWlast : P.SW;
    const int col = (16 * c * P.s - P.p) * P.IC + x;
    if (ih < 0 || ih >= P.IH || x >= sw || col < 0 || col >= rowFloats) return;
    if (P.OVF > 0 && ((c > 0 && x < P.OVF) || (c < P.nBands - 1 && x >= 16 * P.s * P.IC))) return;   // the band part's
    P.dX[((long)n * P.IH + ih) * rowFloats + col] += P.rowhead[(long)hr * kScatterRP + x];
}

}  // namespace cks
