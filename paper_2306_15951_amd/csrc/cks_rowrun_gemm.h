// ConvV2 (Algorithm 1) and KS-deconv-V2 Stage 2&3 (Algorithm 2B) as one
// position-uniform fp32-MFMA GEMM.
//
// Both operators have the same shape once an output POSITION is fixed
// ((oh,ow) of Y, resp. (ih,iw) of dX):
//
//     Out[n, pos, j] = sum over trimmed taps, channel  A[n, tap, ch] * B[j, tap, ch]
//
// with n the batch index (GEMM rows), j the output channel (GEMM columns), and
// the trimmed tap range the SAME for every n and j.  Better still, in NHWC
// the taps of one filter row are adjacent pixels, so for one fh (resp. ch) the
// contraction index (fw, ic) is one contiguous run of (fw_e - fw_s)*IC floats
// in the activation row AND in the filter row:
//
//   ConvV2:    A = X,  B = W[oc][fh][fw][ic]              run over (fw, ic)
//   KS-deconv: A = dY, B = Cs[y][x][ic][ch][cw][oc]       run over (cw, oc)
//   KS-deconv without Stage 1: A = dY, B = W itself.  Sub-kernel (y,x)'s tap (ch,cw) is the filter tap
//              (y + (CH-1-ch) sh, x + (CW-1-cw) sw); for it W[oc][fh][fw][ic] is a K x N matrix (oc x ic) with
//              N contiguous.  It is staged into LDS as it lies (K-major) and the B fragments are read one
//              float per MFMA instead of four: Stage 1 then costs nothing at all.
//
// So a workgroup owns (position, 128/64 batch rows, 128/64/32 channels), knows its
// trim as scalars, and walks  nruns x ceil(L/32)  K-chunks; trimming costs
// nothing but two pointer offsets and a shorter loop (the realisation of
// trimming that Section IV.A describes), no lane ever multiplies a padded
// or inserted zero, and no per-element bounds test exists in the loop.
#pragma once
#include "cks_device.h"

namespace cks {

// OP_DECONV_W: KS-deconv Stage 2&3 that takes its sub-kernels straight from the OHWI filter (see below)
// OP_FWD_T:    ConvV2 on the transposed filter Wt[FH][FW][IC][OC] of Section IV.A (last paragraph): for one tap
//              the filter is a K x N matrix (ic x oc) with N contiguous, staged K-major like OP_DECONV_W's
enum { OP_FWD = 0, OP_DECONV = 1, OP_DECONV_W = 2, OP_FWD_T = 3 };
constexpr bool op_is_fwd(int op) { return op == OP_FWD || op == OP_FWD_T; }        // positions are those of Y
constexpr bool op_b_k_major(int op) { return op == OP_DECONV_W || op == OP_FWD_T; }  // B chunk = 32 k-rows x BN columns

struct RowRunParams {
    const float *A;   // X (fwd) or dY (deconv)
    const float *B;   // W (fwd) or split kernels Cs (deconv)
    float *Out;       // Y (fwd) or dX (deconv)
    int N, IC, IH, IW, OC, OH, OW, FH, FW;
    int sh, sw, ph, pw;   // stride and padding per axis (Table I: <sh sw>, <ph pw>)
    int CHp, CWp;     // ceil(FH/sh), ceil(FW/sw): padded sub-kernel extents
    // Work decomposition: one output position (of Y, resp. dX) times one tile.
    // Positions are issued roughly most expensive first: ConvV2's list starts at
    // (rotH, rotW), the first position with an untrimmed window, and wraps
    // around to the border; KS-deconv lists the positions class by class (larger
    // sub-kernels first) and does the same within each class (rotH = rotW = 0).
    int itemsH, itemsW;   // grid of positions
    int rotH, rotW;
    int mTiles, nTiles;
    int bandBlocks;       // workgroups per band = items per band * mTiles * nTiles
    int total;            // workgroups with work
    // divisors of the work decoding, prepared on the host (see FastDiv)
    FastDiv dBand, dNT, dMT, dItemsW, dSh, dSw;
    int pmodsH, pmodsW;   // ph mod sh, pw mod sw
    int bufStore;         // the tile's BM output rows span less than 2 GiB: stores go through a buffer descriptor
    int pairFlip;         // see banded_work
    int fullSlots, remPerDie, covered;   // see banded_work
};

struct RunSet {
    long a0, b0, o0;          // float offsets of the first run in A-row 0, B-row 0, Out-row 0
    long aRun, bRun;          // float distance between consecutive runs
    long bCw;                 // OP_DECONV_W: float distance between consecutive cw (negative: the rotation)
    long strideA, strideB, strideO;
    int nruns, L, NC;         // runs, floats per run, number of output channels
    // untrimmed variant only: run r, tap column c of the window is A pixel (h0 + r, w0 + c), which exists if
    // it lies inside hLim x wLim (Algorithm 2 / the plain convolution read zeros elsewhere)
    int h0, w0, hLim, wLim;
};

// The a-th index of [0, I) when indices are listed class by class, class
// y = (i + p) mod s, y = 0, 1, ...  (sub-kernel extents shrink with y, so the
// classes with most work come first).  Within a class the list starts at its first
// index whose window over dY is not cut at the low end and wraps around to those
// that are: every class then runs from its dearest to its cheapest positions, and
// the list as a whole from the dearest class to the cheapest.  (Rotating the list
// as a whole instead moves a row of the dearest class behind the cheapest one: on a
// layer whose workgroups are all resident at once that row is dispatched last, gets
// what is left of the issue slots and finishes last -- 7 % on the stride-2 benchmark layer.)
__device__ inline int class_major_index(int a, int I, const FastDiv &dS, int pmods, int F, int p)
{
    const int s = dS.d;
    for (int y = 0; y < s; ++y) {
        int i0 = y - pmods;   // first index of class y: (y - p) mod s
        if (i0 < 0) i0 += s;
        int cnt = i0 < I ? fdiv(I - 1 - i0, dS) + 1 : 0;
        if (a < cnt) {
            // index i0 + j s has window start q0 + j - (CH - 1): cut at the low end while j < CH - 1 - q0
            const int CH = y < F ? fdiv(F - y + s - 1, dS) : 0, q0 = fdiv(i0 + p - y, dS);
            const int lead = min(max(CH - 1 - q0, 0), cnt);
            int j = a + lead;
            if (j >= cnt) j -= cnt;
            return i0 + j * s;
        }
        a -= cnt;
    }
    return 0;  // not reached for 0 <= a < I
}

// Trim and addressing of one output position: (oh,ow) of Y for ConvV2, (ih,iw)
// of dX for KS-deconv.
// TRIM = false: the whole window is contracted, as in the plain convolution and in KS-deconv before its V2
// (Algorithm 2); the caller supplies zeros for the window's cells outside the data.
template <int OP, bool TRIM = true>
__device__ inline RunSet decode_position(const RowRunParams &P, int ph, int pw)
{
    RunSet R;
    R.bCw = 0;
    if (op_is_fwd(OP)) {
        // Algorithm 1: trim [fh_s,fh_e) x [fw_s,fw_e) of the filter at (oh,ow).
        const int oh = ph, ow = pw;
        int ih_s = oh * P.sh - P.ph, iw_s = ow * P.sw - P.pw;
        int fh_s = max(-ih_s, 0), fh_e = min(P.IH - ih_s, P.FH);
        int fw_s = max(-iw_s, 0), fw_e = min(P.IW - iw_s, P.FW);
        if (!TRIM) { fh_s = 0; fh_e = P.FH; fw_s = 0; fw_e = P.FW; }
        R.h0 = ih_s; R.w0 = iw_s; R.hLim = P.IH; R.wLim = P.IW;
        R.nruns = max(fh_e - fh_s, 0);
        R.L = max(fw_e - fw_s, 0) * P.IC;
        R.a0 = ((long)(ih_s + fh_s) * P.IW + (iw_s + fw_s)) * P.IC;
        R.aRun = (long)P.IW * P.IC;
        R.strideA = (long)P.IH * P.IW * P.IC;
        if (OP == OP_FWD_T) {
            // run r is filter row fh_s + r of Wt[FH][FW][IC][OC]; within it the taps fw_s.. follow each other
            // IC*OC floats apart, and consecutive k (input channels) are OC floats apart
            R.strideB = P.OC;
            R.b0 = ((long)fh_s * P.FW + fw_s) * P.IC * P.OC;
            R.bRun = (long)P.FW * P.IC * P.OC;
            R.bCw = (long)P.IC * P.OC;
        } else {
            R.b0 = ((long)fh_s * P.FW + fw_s) * P.IC;
            R.bRun = (long)P.FW * P.IC;
            R.strideB = (long)P.FH * P.FW * P.IC;
        }
        R.o0 = ((long)oh * P.OW + ow) * P.OC;
        R.strideO = (long)P.OH * P.OW * P.OC;
        R.NC = P.OC;
    } else {
        // Algorithm 2B: class (y,x) of (ih,iw), its sub-kernel extent CH x CW,
        // the window start (oh_s,ow_s) in dY and the trim [ch_s,ch_e) x [cw_s,cw_e).
        const int ih = ph, iw = pw;
        const int qh = fdiv(ih + P.ph, P.dSh), qw = fdiv(iw + P.pw, P.dSw);
        int y = ih + P.ph - qh * P.sh, x = iw + P.pw - qw * P.sw;
        int CH = y < P.FH ? fdiv(P.FH - y + P.sh - 1, P.dSh) : 0;
        int CW = x < P.FW ? fdiv(P.FW - x + P.sw - 1, P.dSw) : 0;
        int oh_s = qh - (CH - 1), ow_s = qw - (CW - 1);
        int ch_s = max(-oh_s, 0), ch_e = min(P.OH - oh_s, CH);
        int cw_s = max(-ow_s, 0), cw_e = min(P.OW - ow_s, CW);
        if (!TRIM) { ch_s = 0; ch_e = CH; cw_s = 0; cw_e = CW; }
        R.h0 = oh_s; R.w0 = ow_s; R.hLim = P.OH; R.wLim = P.OW;
        R.nruns = max(ch_e - ch_s, 0);
        R.L = max(cw_e - cw_s, 0) * P.OC;
        R.a0 = ((long)(oh_s + ch_s) * P.OW + (ow_s + cw_s)) * P.OC;
        R.aRun = (long)P.OW * P.OC;
        R.strideA = (long)P.OH * P.OW * P.OC;
        if (OP == OP_DECONV_W) {
            // run r is sub-kernel row ch_s + r = filter row y + (CH-1-ch_s-r) sh; likewise the columns
            R.strideB = (long)P.FH * P.FW * P.IC;
            R.b0 = ((long)(y + (CH - 1 - ch_s) * P.sh) * P.FW + (x + (CW - 1 - cw_s) * P.sw)) * P.IC;
            R.bRun = -(long)P.sh * P.FW * P.IC;
            R.bCw = -(long)P.sw * P.IC;
        } else {
            R.strideB = (long)P.CHp * P.CWp * P.OC;
            R.b0 = (long)(y * P.sw + x) * P.IC * R.strideB + ((long)ch_s * P.CWp + cw_s) * P.OC;
            R.bRun = (long)P.CWp * P.OC;
        }
        R.o0 = ((long)ih * P.IW + iw) * P.IC;   // Stage 3: the class result lands at its own (ih,iw)
        R.strideO = (long)P.IH * P.IW * P.IC;
        R.NC = P.IC;
    }
    if (R.nruns == 0 || R.L == 0) { R.nruns = 0; R.L = 0; R.a0 = 0; R.b0 = 0; }
    return R;
}

// Hardware hands workgroup b to die b % 8.  Work is cut into bands of
// bandBlocks consecutive workgroups (tiles of neighbouring items, which share
// operands and so that die's L2); bands go to the dies in a serpentine order,
// so every die gets the same mix of expensive interior and cheap border items.
// That covers the whole rounds of 8 bands (slots below fullSlots of every die, workgroups below
// `covered`); what is left -- less than a round -- is cut into 8 equal contiguous pieces of remPerDie
// workgroups, one per die: a 49th band as a whole would keep one die busy a seventh longer than the others.
// Within a die the hardware deals consecutive workgroups to its 32 compute units round-robin (observed:
// workgroups j and j + 32 of a die share a compute unit), and items are listed expensive first: with `flip`
// every second group of 32 is walked backwards, so that the workgroups resident together on a compute unit
// are an expensive and a cheap one rather than two of a kind.  (Not for KS-deconv with several classes: its
// list is class-major, workgroups 32 apart are neighbouring positions of different classes that read the
// same dY rows, and sharing a compute unit's cache is worth more there: -12 points on cfg2 when flipped.)
// A slot without work returns P.total.
__device__ inline int banded_work(int bid, const RowRunParams &P)
{
    const int xcd = bid % kXcds;
    int slot = bid / kXcds;
    if (P.pairFlip && (slot & 32)) slot ^= 31;
    if (slot < P.fullSlots) {
        const int round = fdiv(slot, P.dBand);
        const int band = round * kXcds + ((round & 1) ? kXcds - 1 - xcd : xcd);
        return band * P.dBand.d + (slot - round * P.dBand.d);
    }
    const int j = slot - P.fullSlots;
    return j < P.remPerDie ? P.covered + xcd * P.remPerDie + j : P.total;
}

// Store of a workgroup's tile (shared by the kernels of this file and of cks_rowrun_dma.h).  Every output
// element of the tile is stored, also when the trimmed range was empty (then it is +0.0).  32 lanes
// write 128 contiguous bytes.
template <int BM, int BN, int WAVES_M, int WAVES_N, int TM, int TN>
__device__ inline void rowrun_store_tile(floatx16 (&acc)[TM][TN], const RowRunParams &P, const RunSet &R, int m0, int n0,
                                              int wm, int wn, int lane)
{
    if (P.bufStore && m0 + BM <= P.N) {
        // A full tile's rows as one raw buffer: lane part of the offset once, row part as a scalar
        // offset (which the hardware does not range-check: hence full tiles only), no vector
        // arithmetic per store.  A column past the channels carries an offset beyond the buffer.
        const __amdgpu_buffer_rsrc_t rsO = __builtin_amdgcn_make_buffer_rsrc(
            P.Out + (long)m0 * R.strideO, 0, (int)(BM * R.strideO * 4), 0x00020000);
        const int so = (int)R.strideO * 4, o0b = (int)R.o0 * 4;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = n0 + (wn * TN + j) * 32 + (lane & 31);
                const int voff = col < R.NC ? ((wm * TM + i) * 32 + 4 * (lane >> 5)) * so + col * 4 : (int)0x80000000u;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[i][j][r]), rsO, voff,
                                                          o0b + (8 * (r >> 2) + (r & 3)) * so, 0);
            }
        return;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + (wn * TN + j) * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + (wm * TM + i) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (row < P.N && col < R.NC) P.Out[(long)row * R.strideO + R.o0 + col] = acc[i][j][r];
            }
        }
}

// Workgroup tile BM (batch rows) x BN (channels), K-chunk of 32 floats, LDS
// double-buffered, rows padded to 36 floats so that the 16-byte fragment reads
// of 32 consecutive rows spread over all banks.  4 waves as WAVES_M x WAVES_N,
// each owning (BM/WAVES_M) x (BN/WAVES_N) as 32x32 MFMA blocks.
template <int BM, int BN>
constexpr size_t rowrun_lds_bytes() { return (size_t)2 * (BM + BN) * 36 * sizeof(float); }

// LOAD selects how the K-chunks are fetched:
//   LOAD_SCALAR  4-byte loads, every element masked (any channel count, any alignment)
//   LOAD_VEC     16-byte loads, masked per 4 floats (channel count multiple of 4, 16-byte aligned)
//   LOAD_FAST    16-byte buffer loads with one scalar offset per chunk: the per-lane
//                offsets are computed once, the run length is a multiple of 32 (no
//                partial chunk, nothing to mask), so the loop issues no vector ALU
//                instruction for addressing.  VALU instructions and MFMAs of one SIMD
//                do not overlap, so every one removed from the loop is MFMA time won.
enum { LOAD_SCALAR = 0, LOAD_VEC = 1, LOAD_FAST = 2 };

template <int OP, int BM, int BN, int WAVES_M, int WAVES_N, int LOAD>
__global__ void __launch_bounds__(kThreads) rowrun_gemm(const RowRunParams P)
{
    constexpr bool VEC = LOAD != LOAD_SCALAR;
    constexpr int KC = 32, LDK = KC + 4;
    constexpr int TM = BM / (WAVES_M * 32), TN = BN / (WAVES_N * 32);
    constexpr int PA = BM / 32, PB = BN / 32;
    static_assert(WAVES_M * WAVES_N == 4 && TM >= 1 && TN >= 1, "4 waves per workgroup");
    // OP_DECONV_W: B chunk = 32 output channels (K) x BN input channels, staged K-major (OP_FWD_T: 32 input
    // channels x BN output channels)
    constexpr bool BK = op_b_k_major(OP);
    constexpr int LDB = BN + 4, TPR = BN / 4, RPP = kThreads / TPR;   // floats per k-row, threads / rows per staging pass
    static_assert(!BK || LOAD == LOAD_FAST, "the filter is read in place only by the fast-load variant");
    static_assert(!BK || 2 * KC * LDB <= 2 * BN * LDK, "the K-major B buffers fit the LDS of the row-major ones");

    extern __shared__ __align__(16) float smem[];
    float *As = smem;                 // [2][BM][LDK]
    float *Bs = smem + 2 * BM * LDK;  // [2][BN][LDK]

    const int work = banded_work(blockIdx.x, P);
    if (work >= P.total) return;
    const int wq = fdiv(work, P.dNT), nt = work - wq * P.nTiles;
    const int item = fdiv(wq, P.dMT), mt = wq - item * P.mTiles;
    int ph = fdiv(item, P.dItemsW), pw = item - ph * P.itemsW;
    ph += P.rotH; if (ph >= P.itemsH) ph -= P.itemsH;   // rotH < itemsH
    pw += P.rotW; if (pw >= P.itemsW) pw -= P.itemsW;
    if (!op_is_fwd(OP)) {
        ph = class_major_index(ph, P.IH, P.dSh, P.pmodsH, P.FH, P.ph);
        pw = class_major_index(pw, P.IW, P.dSw, P.pmodsW, P.FW, P.pw);
    }
    const int m0 = mt * BM, n0 = nt * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    // Global -> LDS staging: 8 threads cover one 32-float row chunk (128 B).
    const int lr = tid >> 3, lc = (tid & 7) * 4;
    const int frow = lane & 31, fk = (lane >> 5) * 4;

    const RunSet R = decode_position<OP>(P, ph, pw);

    const int cpr = (R.L + KC - 1) / KC;  // chunks per run
    const int T = R.nruns * cpr;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // Row addresses of this thread's staging loads.  Rows past the end of the
    // batch / channel range are clamped (loaded twice, never stored).
    const float *pa[PA], *pb[PB];
    unsigned va[PA], vb[PB];   // LOAD_FAST: byte offsets from the workgroup's base
#pragma unroll
    for (int i = 0; i < PA; ++i) {
        const int r = min(m0 + lr + 32 * i, P.N - 1);
        pa[i] = P.A + (long)r * R.strideA + R.a0 + lc;
        va[i] = (unsigned)(((long)(r - m0) * R.strideA + lc) * 4);
    }
    const int brow = tid / TPR, bcol = (tid % TPR) * 4;   // BK: k-row (output channel of the chunk) and column of this thread
#pragma unroll
    for (int i = 0; i < PB; ++i) {
        const int c = min(n0 + lr + 32 * i, R.NC - 1);
        pb[i] = P.B + (long)c * R.strideB + R.b0 + lc;
        // BK: a column past the last input channel would be the next tap's (or, at the very end of the
        // filter, past the allocation): it carries an offset beyond the buffer and reads as zero
        vb[i] = BK ? (n0 + bcol < R.NC ? (unsigned)(((long)(brow + RPP * i) * R.strideB + bcol) * 4) : 0x80000000u)
                   : (unsigned)(((long)(c - n0) * R.strideB + lc) * 4);
    }
    const __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(P.A + (long)min(m0, P.N - 1) * R.strideA + R.a0), 0, -1, 0x00020000);
    // BK: the filter from column n0 on, as a buffer of its true size
    const __amdgpu_buffer_rsrc_t rsB =
        BK ? __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(P.B + n0), 0,
                                               (int)(((long)P.OC * P.FH * P.FW * P.IC - n0) * 4), 0x00020000)
           : __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(P.B + (long)min(n0, R.NC - 1) * R.strideB + R.b0), 0, -1,
                                               0x00020000);
    const int ocChunks = (op_is_fwd(OP) ? P.IC : P.OC) / KC;   // BK: chunks per tap of a run (the contracted channels)

    // One register set: the loads of chunk t+1 are issued before chunk t is
    // multiplied out of LDS and stored to the other LDS buffer after it.  (A
    // second set, two chunks ahead, was measured to be slower.)
    struct Stage { float4 a[PA], b[PB]; };
    Stage S0;
    // `live` false: nothing is read; the masked modes then stage zeros.
    int cwi = 0, occ = 0;   // BK: the chunk being loaded is contracted channels 32*occ.. of the run's tap number cwi
    auto gload = [&](Stage &S, int run, int ck, bool live) {
        if (LOAD == LOAD_FAST) {
            if (!live) return;   // uniform
            const int sa = (int)((run * R.aRun + ck * KC) * 4);
            const int sb = BK ? (int)((R.b0 + run * R.bRun + cwi * R.bCw + (long)occ * KC * R.strideB) * 4)
                              : (int)((run * R.bRun + ck * KC) * 4);
#pragma unroll
            for (int i = 0; i < PA; ++i)
                S.a[i] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(rsA, va[i], sa, 0));
#pragma unroll
            for (int i = 0; i < PB; ++i)
                S.b[i] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(rsB, vb[i], sb, 0));
        } else {
            const long oa = run * R.aRun + ck * KC, ob = run * R.bRun + ck * KC;
            const int valid = live ? R.L - ck * KC - lc : 0;
#pragma unroll
            for (int i = 0; i < PA; ++i) S.a[i] = load4<VEC>(pa[i] + oa, valid);
#pragma unroll
            for (int i = 0; i < PB; ++i) S.b[i] = load4<VEC>(pb[i] + ob, valid);
        }
    };
    // buf is a compile-time constant in the loop below, so every LDS access is
    // "thread base + immediate"
    float *const Aw = As + lr * LDK + lc, *const Bw = Bs + lr * LDK + lc, *const Bwk = Bs + brow * LDB + bcol;
    auto sstore = [&](const Stage &S, int buf) {
#pragma unroll
        for (int i = 0; i < PA; ++i) *reinterpret_cast<float4 *>(Aw + (buf * BM + 32 * i) * LDK) = S.a[i];
#pragma unroll
        for (int i = 0; i < PB; ++i) {
            if (BK) *reinterpret_cast<float4 *>(Bwk + (buf * KC + RPP * i) * LDB) = S.b[i];
            else *reinterpret_cast<float4 *>(Bw + (buf * BN + 32 * i) * LDK) = S.b[i];
        }
    };

    // MFMA fragments: lane l reads 4 consecutive k of row (l%32); the two lane
    // halves take k-groups 4 apart, so one 16-byte read feeds 4 MFMAs.  A chunk
    // shorter than 32 is zero-filled in LDS, so every chunk runs the same 4 steps
    // and the accumulators never leave their registers.
    const float *const Ar = As + (wm * TM * 32 + frow) * LDK + fk, *const Br = Bs + (wn * TN * 32 + frow) * LDK + fk;
    // K-major B: one base per (buffer, k-group of 8), so that the four rows a lane reads are within the
    // 1 KB an LDS read pair can address beyond its base (anything larger costs a VALU add in the loop)
    typedef __attribute__((address_space(3))) const float lds_cfloat;
    lds_cfloat *brk[2][KC / 8];   // LDS addresses, made opaque so that each stays in a register of its own
#pragma unroll
    for (int bf = 0; bf < 2; ++bf)
#pragma unroll
        for (int kk = 0; kk < KC / 8; ++kk) {
            lds_cfloat *q = (lds_cfloat *)(Bs + ((bf * KC + kk * 8) + fk) * LDB + wn * TN * 32 + frow);
            asm volatile("" : "+v"(q));
            brk[bf][kk] = q;
        }
    auto compute = [&](int buf) {
#pragma unroll
        for (int kk = 0; kk < KC / 8; ++kk) {
            float4 a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const float4 *>(Ar + (buf * BM + i * 32) * LDK + kk * 8);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if (BK) {
                    // K-major: the lane's four k (fk .. fk+3) are four rows
                    lds_cfloat *q = brk[buf][kk] + j * 32;
                    b[j] = float4{q[0], q[LDB], q[2 * LDB], q[3 * LDB]};
                } else {
                    b[j] = *reinterpret_cast<const float4 *>(Br + (buf * BN + j * 32) * LDK + kk * 8);
                }
            }
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = mfma32(reinterpret_cast<const float *>(&a[i])[e],
                                           reinterpret_cast<const float *>(&b[j])[e], acc[i][j]);
        }
    };

    int run = 0, ck = 0;   // chunk being loaded
    auto next_chunk = [&]() {
        if (BK && ++occ == ocChunks) { occ = 0; ++cwi; }
        if (++ck == cpr) { ck = 0; ++run; cwi = 0; occ = 0; }
    };
    // The loop body handles two chunks with literal buffer numbers (all LDS
    // addresses become immediates) and no branch around the MFMAs (so the
    // accumulators stay in place).  An odd chunk count is peeled off in front:
    // chunk 0 then starts in buffer 1.
    const int odd = T & 1;
    gload(S0, 0, 0, T > 0);
    if (LOAD != LOAD_FAST || T > 0) {
        if (odd) sstore(S0, 1); else sstore(S0, 0);
    }
    __syncthreads();
    auto iteration = [&](int t, int buf) {   // buf is a literal at every call
        next_chunk();
        gload(S0, run, ck, t + 1 < T);
        compute(buf);
        if (LOAD != LOAD_FAST || t + 1 < T) sstore(S0, buf ^ 1);
        __syncthreads();
    };
    if (odd) iteration(0, 1);
    for (int t = odd; t < T; t += 2) {
        iteration(t, 0);
        iteration(t + 1, 1);
    }

    rowrun_store_tile<BM, BN, WAVES_M, WAVES_N>(acc, P, R, m0, n0, wm, wn, lane);
}

}  // namespace cks
