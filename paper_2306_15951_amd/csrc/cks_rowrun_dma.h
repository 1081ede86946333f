// ConvV2 / KS-deconv-V2 Stage 2&3: the position-uniform GEMM of cks_rowrun_gemm.h with its K-chunks
// fetched straight into LDS.
//
// Same work decomposition, same trim (decode_position), same tile store as rowrun_gemm; what differs is the
// way a K-chunk gets from global memory to the MFMA operands.  rowrun_gemm loads 16 bytes per lane into
// registers and writes them to LDS with ds_write_b128; measured in a probe of the bare loop, that register
// round trip costs 13 points of matrix-core time with four workgroups on a compute unit and 22 with two.
// Here each lane's 16 bytes go from the buffer load directly into LDS ("buffer_load_dwordx4 ... lds": the
// wave's 64 pieces land at LDS base + 16 * lane, base in M0), no vector register is written and no LDS
// store instruction issued.
//
// Because the hardware fixes where a lane's piece lands, the LDS tile cannot be padded against bank
// conflicts; instead the 16-byte pieces of a row are permuted:
//   row-major operand (A always; B of ConvV2 and of the pre-split KS-deconv): tile [rows][32 floats], piece
//     c (0..7) of row r is stored at piece position c ^ ((r >> 1) & 7).  The 16 lanes that the LDS serves
//     together read one piece each from 16 consecutive rows: 8 even and 8 odd rows, which differ in bit 5
//     of the bank number and, within each parity, in all 8 piece positions.
//   K-major operand (B of the KS-deconv that reads the filter in place and of ConvV2 on the transposed
//     filter): tile [32 k][BN floats], piece c of
//     k-row k is stored at piece position c ^ (8 * ((k >> 2) & 1)) -- the two lane halves of a fragment
//     read rows k and k + 4 at the same column and now fall into different bank halves.
// A lane simply fetches the global piece that belongs at its fixed LDS position.
//
// The compiler makes every LDS read it can see wait for all LDS-direct loads in flight (it cannot tell
// that they go to the other buffer), which would serialise loading and multiplying.  The fragment reads
// are therefore inline assembly with hand-placed waits; their addresses are "lane constant + immediate".
#pragma once
#include <type_traits>

#include "cks_lds_direct.h"
#include "cks_rowrun_gemm.h"

namespace cks {

template <int BM, int BN>
constexpr size_t rowrun_dma_lds_bytes() { return (size_t)2 * (BM + BN) * 32 * sizeof(float); }

// TRIM = false: the ablation's untrimmed operators (plain convolution; KS-deconv of Algorithm 2) -- every
// position contracts its whole window, and a chunk whose A pixel lies outside the data is fetched through a
// descriptor of zero length, i.e. as zeros, which the matrix cores then multiply like any other operand.
template <int OP, int BM, int BN, int WAVES_M, int WAVES_N, bool TRIM = true>
__global__ void __launch_bounds__(kThreads) rowrun_gemm_dma(const RowRunParams P)
{
    constexpr int KC = 32;
    constexpr int TM = BM / (WAVES_M * 32), TN = BN / (WAVES_N * 32);
    constexpr int IA = BM / 32, IB = BN / 32;      // LDS-direct loads per wave and chunk (1 KB each)
    constexpr bool BK = op_b_k_major(OP);
    constexpr int ABUF = BM * KC * 4, BBUF = BN * KC * 4;   // bytes per buffer
    static_assert(WAVES_M * WAVES_N == 4 && TM >= 1 && TN >= 1 && TM <= 2 && TN <= 2, "4 waves, up to 2 x 2 blocks each");
    static_assert(!BK || (BN == 64 && TN == 1), "the K-major tile is laid out for 64 columns, one block per wave");

    extern __shared__ __align__(16) float smem[];
    float *As = smem;                      // [2][BM][32]
    float *Bs = smem + 2 * BM * KC;        // [2][BN][32], or [2][32][BN] (K-major)

    const int work = banded_work(blockIdx.x, P);
    if (work >= P.total) return;
    const int wq = fdiv(work, P.dNT), nt = work - wq * P.nTiles;
    const int item = fdiv(wq, P.dMT), mt = wq - item * P.mTiles;
    int ph = fdiv(item, P.dItemsW), pw = item - ph * P.itemsW;
    ph += P.rotH; if (ph >= P.itemsH) ph -= P.itemsH;
    pw += P.rotW; if (pw >= P.itemsW) pw -= P.itemsW;
    if (!op_is_fwd(OP)) {
        ph = class_major_index(ph, P.IH, P.dSh, P.pmodsH, P.FH, P.ph);
        pw = class_major_index(pw, P.IW, P.dSw, P.pmodsW, P.FW, P.pw);
    }
    const int m0 = mt * BM, n0 = nt * BN;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: LDS-direct loads take their LDS base from M0
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int frow = lane & 31, h = lane >> 5;

    const RunSet R = decode_position<OP, TRIM>(P, ph, pw);
    const int cpr = R.L / KC;             // chunks per run (the host launches this kernel only if L % 32 == 0)
    const int T = R.nruns * cpr;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // ---- global side: load q of this wave fills rows 8 * (IA * wave + q) .. + 7 of the A tile; lane l row + l / 8,
    // LDS piece position l % 8, hence global piece (l % 8) ^ ((row >> 1) & 7).  Rows past the end of the batch /
    // channel range are clamped (loaded twice, never stored).
    unsigned va[IA], vb[IB];
#pragma unroll
    for (int q = 0; q < IA; ++q) {
        const int row = 8 * (IA * wave + q) + (lane >> 3);
        const int piece = (lane & 7) ^ ((row >> 1) & 7);
        const int r = min(m0 + row, P.N - 1);
        va[q] = (unsigned)(((long)(r - min(m0, P.N - 1)) * R.strideA + piece * 4) * 4);
    }
#pragma unroll
    for (int q = 0; q < IB; ++q) {
        if (BK) {
            // K-major: load q fills k-rows 4 * (IB * wave + q) .. + 3 (16 pieces of 4 columns each); lane l k-row + l / 16,
            // LDS piece position l % 16, global piece (l % 16) ^ (8 * ((k >> 2) & 1)).  A column past the last input
            // channel would be the next tap's (or past the allocation): it carries an offset beyond the buffer.
            const int k = 4 * (IB * wave + q) + (lane >> 4);
            const int piece = (lane & 15) ^ (8 * ((k >> 2) & 1));
            vb[q] = n0 + 4 * piece < R.NC ? (unsigned)(((long)k * R.strideB + 4 * piece) * 4) : 0x80000000u;
        } else {
            const int row = 8 * (IB * wave + q) + (lane >> 3);
            const int piece = (lane & 7) ^ ((row >> 1) & 7);
            const int c = min(n0 + row, R.NC - 1);
            vb[q] = (unsigned)(((long)(c - min(n0, R.NC - 1)) * R.strideB + piece * 4) * 4);
        }
    }
    float *const baseA = const_cast<float *>(P.A + (long)min(m0, P.N - 1) * R.strideA + R.a0);
    const __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc(baseA, 0, -1, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsB =
        BK ? __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(P.B + n0), 0, (int)(((long)P.OC * P.FH * P.FW * P.IC - n0) * 4), 0x00020000)
           : __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(P.B + (long)min(n0, R.NC - 1) * R.strideB + R.b0), 0, -1, 0x00020000);
    const int ocChunks = (op_is_fwd(OP) ? P.IC : P.OC) / KC;   // chunks per tap of a run (the contracted channels)

    int run = 0, ck = 0, cwi = 0, occ = 0;   // chunk being loaded: contracted channels 32*occ.. of the run's tap number cwi
    auto next_chunk = [&]() {
        if ((BK || !TRIM) && ++occ == ocChunks) { occ = 0; ++cwi; }
        if (++ck == cpr) { ck = 0; ++run; cwi = 0; occ = 0; }
    };
    auto gload = [&](int buf) {   // buf is a literal at every call
        const int sa = (int)((run * R.aRun + ck * KC) * 4);
        // untrimmed: a chunk outside the data is read through a descriptor of length 0 (wave-uniform: one scalar select)
        const bool inside = TRIM || ((unsigned)(R.h0 + run) < (unsigned)R.hLim && (unsigned)(R.w0 + cwi) < (unsigned)R.wLim);
        const __amdgpu_buffer_rsrc_t rsAc = TRIM ? rsA : __builtin_amdgcn_make_buffer_rsrc(baseA, 0, __builtin_amdgcn_readfirstlane(inside ? -1 : 0), 0x00020000);
        const int sb = BK ? (int)((R.b0 + run * R.bRun + cwi * R.bCw + (long)occ * KC * R.strideB) * 4)
                          : (int)((run * R.bRun + ck * KC) * 4);
#pragma unroll
        for (int q = 0; q < IA; ++q)
            load16_to_lds(rsAc, As + buf * BM * KC + (IA * wave + q) * 256, va[q], sa);
#pragma unroll
        for (int q = 0; q < IB; ++q)
            load16_to_lds(rsB, Bs + buf * BN * KC + (IB * wave + q) * 256, vb[q], sb);
    };

    // ---- LDS side: byte addresses of this lane's fragments in buffer 0, one per group of 8 k (kk = 0..3).
    // A (and row-major B): row (block row + lane % 32), piece 2 kk + h permuted by the row; further blocks of 32
    // rows and buffer 1 are immediates (32 rows do not change (row >> 1) & 7).
    // K-major B: column (block column + lane % 32) of k-rows 8 kk + 4 h .. + 3; the permutation depends on h only.
    unsigned pa[4], pb[4];
    unsigned pbk[2][4];   // K-major B: the read pairs have no room for a buffer offset, so one address per buffer
    {
        const int ra = wm * TM * 32 + frow, rb = wn * TN * 32 + frow;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            pa[kk] = (unsigned)(size_t)(lds_float_t *)(As + ra * KC + 4 * ((2 * kk + h) ^ ((ra >> 1) & 7)));
            if (BK) {
                const int col = rb ^ (32 * h);   // piece ^ 8 == column ^ 32
                pb[kk] = 0;
                pbk[0][kk] = (unsigned)(size_t)(lds_float_t *)(Bs + (8 * kk + 4 * h) * BN + col);
                pbk[1][kk] = pbk[0][kk] + BBUF;
            } else {
                pbk[0][kk] = pbk[1][kk] = 0;
                pb[kk] = (unsigned)(size_t)(lds_float_t *)(Bs + rb * KC + 4 * ((2 * kk + h) ^ ((rb >> 1) & 7)));
            }
        }
    }

    // One K-chunk out of LDS buffer BUF: the fragment reads of k-group kk + 1 are issued before the MFMAs of
    // group kk; each wait names the values it releases, which orders the MFMAs behind it.
    auto read_a = [&](auto buf_c, int kk, floatx4v(&a)[TM]) {
        constexpr int BUF = decltype(buf_c)::value;
        a[0] = lds_read_b128<BUF * ABUF>(pa[kk]);
        if constexpr (TM > 1) a[1] = lds_read_b128<BUF * ABUF + 32 * KC * 4>(pa[kk]);
    };
    auto read_b = [&](auto buf_c, int kk, floatx4v(&b)[TN]) {
        constexpr int BUF = decltype(buf_c)::value;
        if constexpr (BK) {
            // four k-rows of one column: rows are BN floats apart
            const floatx2v lo = lds_read2_b32<0, BN>(pbk[BUF][kk]), hi = lds_read2_b32<2 * BN, 3 * BN>(pbk[BUF][kk]);
            b[0] = floatx4v{lo.x, lo.y, hi.x, hi.y};
        } else {
            b[0] = lds_read_b128<BUF * BBUF>(pb[kk]);
            if constexpr (TN > 1) b[1] = lds_read_b128<BUF * BBUF + 32 * KC * 4>(pb[kk]);
        }
    };
    auto release = [&](floatx4v(&a)[TM], floatx4v(&b)[TN], auto last_c) {
        // reads of the next group (issued after these) may stay in flight unless this is the last group
        constexpr int PENDING = decltype(last_c)::value ? 0 : TM + (BK ? 2 * TN : TN);
        if constexpr (TM == 1 && TN == 1) lds_wait<PENDING>(a[0], b[0]);
        else if constexpr (TM == 2 && TN == 1) lds_wait<PENDING>(a[0], a[1], b[0]);
        else if constexpr (TM == 1 && TN == 2) lds_wait<PENDING>(a[0], b[0], b[1]);
        else lds_wait<PENDING>(a[0], a[1], b[0], b[1]);
    };
    auto mfmas = [&](const floatx4v(&a)[TM], const floatx4v(&b)[TN]) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = mfma32(a[i][e], b[j][e], acc[i][j]);
    };
    auto compute = [&](auto buf_c) {
        floatx4v a0[TM], b0[TN], a1[TM], b1[TN];
        read_a(buf_c, 0, a0); read_b(buf_c, 0, b0);
        read_a(buf_c, 1, a1); read_b(buf_c, 1, b1);
        release(a0, b0, std::false_type{});
        mfmas(a0, b0);
        read_a(buf_c, 2, a0); read_b(buf_c, 2, b0);
        release(a1, b1, std::false_type{});
        mfmas(a1, b1);
        read_a(buf_c, 3, a1); read_b(buf_c, 3, b1);
        release(a0, b0, std::false_type{});
        mfmas(a0, b0);
        release(a1, b1, std::true_type{});
        mfmas(a1, b1);
    };
    // the loads issued during this iteration have landed, and every wave is done reading the buffer that the
    // next iteration's loads overwrite
    auto chunk_end = [&]() {
        vmem_wait_all();
        __syncthreads();
    };
    using B0 = std::integral_constant<int, 0>;
    using B1 = std::integral_constant<int, 1>;

    // Two chunks per loop pass with literal buffer numbers; an odd chunk count is peeled off in front
    // (chunk 0 then starts in buffer 1).
    if (T > 0) {
        const int odd = T & 1;
        if (odd) gload(1); else gload(0);
        chunk_end();
        int t = 0;
        if (odd) {
            if (T > 1) { next_chunk(); gload(0); }
            compute(B1{});
            chunk_end();
            t = 1;
        }
        for (; t < T; t += 2) {
            next_chunk();
            gload(1);                       // chunk t + 1 exists: T - t is even
            compute(B0{});
            chunk_end();
            if (t + 2 < T) { next_chunk(); gload(0); }
            compute(B1{});
            chunk_end();
        }
    }

    rowrun_store_tile<BM, BN, WAVES_M, WAVES_N>(acc, P, R, m0, n0, wm, wn, lane);
}

}  // namespace cks
