// Filter re-layout kernels: KS-deconv Stage 1 (kernel split, Algorithm 2
// Stage 1) and the filter transposition of Section IV.A.  Both move every
// filter element once and exchange the roles of the two channel axes, so they
// are one 32x32 LDS-tiled transpose with two different address maps: reads are
// contiguous along IC, writes contiguous along OC.
#pragma once
#include "cks_device.h"

namespace cks {

enum { PACK_SPLIT = 0, PACK_TRANSPOSE = 1 };

struct PackParams {
    const float *W;   // [OC][FH][FW][IC]
    float *Out;       // PACK_SPLIT: [sh][sw][IC][CHp][CWp][OC]   PACK_TRANSPOSE: [FH][FW][IC][OC]
    int IC, OC, FH, FW, sh, sw, CHp, CWp;
    int ocTiles, icTiles;
};

template <int MODE>
__global__ void __launch_bounds__(kThreads) pack_filter(const PackParams P)
{
    __shared__ float tile[32][33];
    int b = blockIdx.x;
    const int ot = b % P.ocTiles; b /= P.ocTiles;
    const int it = b % P.icTiles; b /= P.icTiles;
    const int slot = b;  // spatial slot of the output

    int fh, fw;
    long out_base;   // float offset of Out[slot-part][ic = 0][...][oc = 0]
    long out_ic;     // float distance between consecutive ic
    bool live = true;
    if (MODE == PACK_SPLIT) {
        // slot = ((y*sw + x)*CHp + ch)*CWp + cw.  Sub-kernel (y,x) has CH x CW
        // taps; tap (ch,cw) is filter tap (y + (CH-1-ch)*sh, x + (CW-1-cw)*sw):
        // the rotated filter sampled with steps sh, sw.  Slots beyond (CH,CW) are
        // the zero padding of the 6-D tensor and are written as zeros.
        const int cw = slot % P.CWp, ch = (slot / P.CWp) % P.CHp;
        const int yx = slot / (P.CWp * P.CHp);
        const int y = yx / P.sw, x = yx - y * P.sw;
        const int CH = y < P.FH ? (P.FH - y + P.sh - 1) / P.sh : 0;
        const int CW = x < P.FW ? (P.FW - x + P.sw - 1) / P.sw : 0;
        fh = y + (CH - 1 - ch) * P.sh;
        fw = x + (CW - 1 - cw) * P.sw;
        live = ch < CH && cw < CW;
        out_ic = (long)P.CHp * P.CWp * P.OC;
        out_base = (long)yx * P.IC * out_ic + ((long)ch * P.CWp + cw) * P.OC;
    } else {
        fh = slot / P.FW;
        fw = slot - fh * P.FW;
        out_ic = P.OC;
        out_base = (long)slot * P.IC * P.OC;
    }

    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int oc0 = ot * 32, ic0 = it * 32;
#pragma unroll
    for (int r = ty; r < 32; r += 8) {
        const int oc = oc0 + r, ic = ic0 + tx;
        float v = 0.f;
        if (live && oc < P.OC && ic < P.IC) v = P.W[(((long)oc * P.FH + fh) * P.FW + fw) * P.IC + ic];
        tile[r][tx] = v;
    }
    __syncthreads();
#pragma unroll
    for (int r = ty; r < 32; r += 8) {
        const int ic = ic0 + r, oc = oc0 + tx;
        if (ic < P.IC && oc < P.OC) P.Out[out_base + (long)ic * out_ic + oc] = tile[tx][r];
    }
}

}  // namespace cks
