/*
 * CPU oracle for the three operators of a 2-D convolutional layer.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the slow, plain definition that the GPU
 * library is checked against; nothing in the product path may call it.  It
 * shares no code, header, table or helper with the HIP kernels.
 *
 * What is computed (paper: Section IV, Eq. (1)-(3); tensor shapes from the
 * paragraph introducing Eq. (1); notation of Table I):
 *
 *   X  [N][IH][IW][IC]    input feature maps            (float)
 *   W  [OC][FH][FW][IC]   filters                       (float)
 *   Y  [N][OH][OW][OC]    output feature maps
 *   OH = floor((IH + 2 ph - FH) / sh) + 1, OW likewise with pw, sw  (the
 *        paper never writes this down; it is the only reading that fits
 *        Table III and the worked example of Fig. 1/4)
 *
 * Stride and padding are given per axis, <sh sw> and <ph pw> of Table I; the
 * paper's algorithms are printed with both and its examples use sh = sw,
 * ph = pw.
 *
 *   Eq. (1)  Y  = conv2D(X, W)              zero padding made explicit
 *   Eq. (2)  dX = deconv2D(dY, rot180(W))   zero insertion made explicit
 *   Eq. (3)  dW = dilated_conv2D(X, dY)     dilation made explicit
 *
 * The method of the paper is exact: it only leaves out terms whose factor is a
 * padded or inserted zero (Section III).  So the oracle is the textbook
 * operator with every such zero physically present in a materialised tensor,
 * and NOT the trimmed / split / leaping algorithms of the appendix.
 *
 * Arithmetic: inputs are float, every product and sum is carried in double,
 * results are returned as double (the caller rounds if it wants to).  Loop
 * order is fixed.  OpenMP is used over the list of output elements only.
 *
 * Every operator takes an optional list of flat output indices ("sample").
 * With sample == NULL all outputs are produced, out[] has the full size; with a
 * list, out[i] is the output element whose flat index is sample[i].  Both modes
 * evaluate the same per-element function on the same materialised tensors.
 *
 * Pins (see tests): a 7-deep brute-force scatter loop (cko_brute, below, which
 * shares nothing with the three operators but the index relation
 * ih = oh*sh - ph + fh), an independent library convolution, the adjoint
 * identities, finite differences, closed forms and the paper's worked example.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Threads the parallel loops below will use (for reporting only). */
int cko_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int out_dim(int I, int F, int s, int p)
{
    int t = I + 2 * p - F;
    if (t < 0) return 0;
    return t / s + 1;
}

int cko_out_dim(int I, int F, int s, int p) { return out_dim(I, F, s, p); }

static int bad_geometry(int N, int IC, int IH, int IW, int OC, int FH, int FW, int sh, int sw, int ph, int pw)
{
    if (N <= 0 || IC <= 0 || IH <= 0 || IW <= 0 || OC <= 0 || FH <= 0 || FW <= 0) return 1;
    if (sh < 1 || sw < 1 || ph < 0 || pw < 0) return 1;
    if (IH + 2 * ph < FH || IW + 2 * pw < FW) return 1;
    return 0;
}

/* X with an explicit border of zeros, ph rows above and below, pw columns left
 * and right: [N][IH+2ph][IW+2pw][IC]. */
static float *make_padded(const float *X, int N, int IH, int IW, int IC, int ph, int pw)
{
    size_t PH = (size_t)IH + 2 * ph, PW = (size_t)IW + 2 * pw;
    float *Xp = (float *)calloc((size_t)N * PH * PW * IC, sizeof(float));
    if (!Xp) return NULL;
    for (int n = 0; n < N; ++n)
        for (int ih = 0; ih < IH; ++ih)
            memcpy(Xp + (((size_t)n * PH + ih + ph) * PW + pw) * IC,
                   X + (((size_t)n * IH + ih) * IW) * IC, (size_t)IW * IC * sizeof(float));
    return Xp;
}

/* dY with (sh-1) / (sw-1) explicit zeros between vertical / horizontal
 * neighbours: [N][(OH-1)sh+1][(OW-1)sw+1][OC]
 * (Section III, second paragraph on backward propagation; Table III, O^p). */
static float *make_dilated(const float *dY, int N, int OH, int OW, int OC, int sh, int sw)
{
    size_t DH = (size_t)(OH - 1) * sh + 1, DW = (size_t)(OW - 1) * sw + 1;
    float *D = (float *)calloc((size_t)N * DH * DW * OC, sizeof(float));
    if (!D) return NULL;
    for (int n = 0; n < N; ++n)
        for (int oh = 0; oh < OH; ++oh)
            for (int ow = 0; ow < OW; ++ow)
                memcpy(D + (((size_t)n * DH + (size_t)oh * sh) * DW + (size_t)ow * sw) * OC,
                       dY + (((size_t)n * OH + oh) * OW + ow) * OC, (size_t)OC * sizeof(float));
    return D;
}

/* ------------------------------------------------------------------ Eq. (1) */

int cko_conv_fwd(const float *X, const float *W, double *Y,
                 int N, int IC, int IH, int IW, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
                 const int64_t *sample, int64_t nsample)
{
    if (bad_geometry(N, IC, IH, IW, OC, FH, FW, sh, sw, ph, pw)) return -2;
    const int OH = out_dim(IH, FH, sh, ph), OW = out_dim(IW, FW, sw, pw);
    const size_t PH = (size_t)IH + 2 * ph, PW = (size_t)IW + 2 * pw;
    float *Xp = make_padded(X, N, IH, IW, IC, ph, pw);
    if (!Xp) return -9;
    const int64_t total = sample ? nsample : (int64_t)N * OH * OW * OC;
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < total; ++e) {
        int64_t idx = sample ? sample[e] : e;
        int oc = (int)(idx % OC); idx /= OC;
        int ow = (int)(idx % OW); idx /= OW;
        int oh = (int)(idx % OH); idx /= OH;
        int n = (int)idx;
        double acc = 0.0;
        for (int fh = 0; fh < FH; ++fh)
            for (int fw = 0; fw < FW; ++fw) {
                const float *xr = Xp + (((size_t)n * PH + (size_t)oh * sh + fh) * PW + (size_t)ow * sw + fw) * IC;
                const float *wr = W + (((size_t)oc * FH + fh) * FW + fw) * IC;
                for (int ic = 0; ic < IC; ++ic) acc += (double)xr[ic] * (double)wr[ic];
            }
        Y[e] = acc;
    }
    free(Xp);
    return 0;
}

/* ------------------------------------------------------------------ Eq. (2) */

int cko_deconv(const float *dY, const float *W, double *dX,
               int N, int IC, int IH, int IW, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
               const int64_t *sample, int64_t nsample)
{
    if (bad_geometry(N, IC, IH, IW, OC, FH, FW, sh, sw, ph, pw)) return -2;
    const int OH = out_dim(IH, FH, sh, ph), OW = out_dim(IW, FW, sw, pw);
    /* Canvas: the zero-inserted gradient laid on zeros so that a unit-stride
     * correlation with the rotated filter yields exactly IH x IW outputs.
     * Cell (oh*sh + FH-1-ph, ow*sw + FW-1-pw) holds dY[oh][ow]; cells that would
     * fall outside are ones no dX element can see, and are dropped. */
    const size_t CH = (size_t)IH + FH - 1, CW = (size_t)IW + FW - 1;
    float *Z = (float *)calloc((size_t)N * CH * CW * OC, sizeof(float));
    float *Wr = (float *)malloc((size_t)OC * FH * FW * IC * sizeof(float));
    if (!Z || !Wr) { free(Z); free(Wr); return -9; }
    for (int n = 0; n < N; ++n)
        for (int oh = 0; oh < OH; ++oh)
            for (int ow = 0; ow < OW; ++ow) {
                long th = (long)oh * sh + FH - 1 - ph, tw = (long)ow * sw + FW - 1 - pw;
                if (th < 0 || tw < 0 || th >= (long)CH || tw >= (long)CW) continue;
                memcpy(Z + (((size_t)n * CH + th) * CW + tw) * OC,
                       dY + (((size_t)n * OH + oh) * OW + ow) * OC, (size_t)OC * sizeof(float));
            }
    /* rot180: flip both spatial axes, channels untouched. */
    for (int oc = 0; oc < OC; ++oc)
        for (int a = 0; a < FH; ++a)
            for (int b = 0; b < FW; ++b)
                memcpy(Wr + (((size_t)oc * FH + a) * FW + b) * IC,
                       W + (((size_t)oc * FH + (FH - 1 - a)) * FW + (FW - 1 - b)) * IC,
                       (size_t)IC * sizeof(float));
    const int64_t total = sample ? nsample : (int64_t)N * IH * IW * IC;
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < total; ++e) {
        int64_t idx = sample ? sample[e] : e;
        int ic = (int)(idx % IC); idx /= IC;
        int iw = (int)(idx % IW); idx /= IW;
        int ih = (int)(idx % IH); idx /= IH;
        int n = (int)idx;
        double acc = 0.0;
        for (int a = 0; a < FH; ++a)
            for (int b = 0; b < FW; ++b) {
                const float *zr = Z + (((size_t)n * CH + ih + a) * CW + iw + b) * OC;
                for (int oc = 0; oc < OC; ++oc)
                    acc += (double)zr[oc] * (double)Wr[(((size_t)oc * FH + a) * FW + b) * IC + ic];
            }
        dX[e] = acc;
    }
    free(Z);
    free(Wr);
    return 0;
}

/* ------------------------------------------------------------------ Eq. (3) */

int cko_wgrad(const float *X, const float *dY, double *dW,
              int N, int IC, int IH, int IW, int OC, int FH, int FW, int sh, int sw, int ph, int pw,
              const int64_t *sample, int64_t nsample)
{
    if (bad_geometry(N, IC, IH, IW, OC, FH, FW, sh, sw, ph, pw)) return -2;
    const int OH = out_dim(IH, FH, sh, ph), OW = out_dim(IW, FW, sw, pw);
    const size_t PH = (size_t)IH + 2 * ph, PW = (size_t)IW + 2 * pw;
    const size_t DH = (size_t)(OH - 1) * sh + 1, DW = (size_t)(OW - 1) * sw + 1;
    float *Xp = make_padded(X, N, IH, IW, IC, ph, pw);
    float *D = make_dilated(dY, N, OH, OW, OC, sh, sw);
    if (!Xp || !D) { free(Xp); free(D); return -9; }
    const int64_t total = sample ? nsample : (int64_t)OC * FH * FW * IC;
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < total; ++e) {
        int64_t idx = sample ? sample[e] : e;
        int ic = (int)(idx % IC); idx /= IC;
        int fw = (int)(idx % FW); idx /= FW;
        int fh = (int)(idx % FH); idx /= FH;
        int oc = (int)idx;
        double acc = 0.0;
        for (int n = 0; n < N; ++n)
            for (size_t a = 0; a < DH; ++a)
                for (size_t b = 0; b < DW; ++b)
                    acc += (double)Xp[(((size_t)n * PH + fh + a) * PW + fw + b) * IC + ic] *
                           (double)D[(((size_t)n * DH + a) * DW + b) * OC + oc];
        dW[e] = acc;
    }
    free(Xp);
    free(D);
    return 0;
}

/* ------------------------------------------------- brute-force cross-check
 * One 7-deep loop over (n, oh, ow, oc, fh, fw, ic).  Each in-range index tuple
 * contributes x*w to Y, dy*w to dX and x*dy to dW.  No padding, insertion,
 * dilation or rotation is ever formed; small inputs only (serial). */
int cko_brute(const float *X, const float *W, const float *dY,
              double *Y, double *dX, double *dW,
              int N, int IC, int IH, int IW, int OC, int FH, int FW, int sh, int sw, int ph, int pw)
{
    if (bad_geometry(N, IC, IH, IW, OC, FH, FW, sh, sw, ph, pw)) return -2;
    const int OH = out_dim(IH, FH, sh, ph), OW = out_dim(IW, FW, sw, pw);
    memset(Y, 0, sizeof(double) * (size_t)N * OH * OW * OC);
    memset(dX, 0, sizeof(double) * (size_t)N * IH * IW * IC);
    memset(dW, 0, sizeof(double) * (size_t)OC * FH * FW * IC);
    for (int n = 0; n < N; ++n)
    for (int oh = 0; oh < OH; ++oh)
    for (int ow = 0; ow < OW; ++ow)
    for (int oc = 0; oc < OC; ++oc)
    for (int fh = 0; fh < FH; ++fh)
    for (int fw = 0; fw < FW; ++fw)
    for (int ic = 0; ic < IC; ++ic) {
        int ih = oh * sh - ph + fh, iw = ow * sw - pw + fw;
        if (ih < 0 || ih >= IH || iw < 0 || iw >= IW) continue;
        size_t xi = (((size_t)n * IH + ih) * IW + iw) * IC + ic;
        size_t wi = (((size_t)oc * FH + fh) * FW + fw) * IC + ic;
        size_t yi = (((size_t)n * OH + oh) * OW + ow) * OC + oc;
        Y[yi]  += (double)X[xi] * (double)W[wi];
        dX[xi] += (double)dY[yi] * (double)W[wi];
        dW[wi] += (double)X[xi] * (double)dY[yi];
    }
    return 0;
}

/* ------------------------------------------------------------ data movement
 * Filter transposition, Section IV.A last paragraph:
 *   W[OC][FH][FW][IC] -> Wt[FH][FW][IC][OC]. */
int cko_filter_transpose(const float *W, float *Wt, int OC, int FH, int FW, int IC)
{
    if (OC <= 0 || FH <= 0 || FW <= 0 || IC <= 0) return -2;
    for (int oc = 0; oc < OC; ++oc)
        for (int fh = 0; fh < FH; ++fh)
            for (int fw = 0; fw < FW; ++fw)
                for (int ic = 0; ic < IC; ++ic)
                    Wt[(((size_t)fh * FW + fw) * IC + ic) * OC + oc] =
                        W[(((size_t)oc * FH + fh) * FW + fw) * IC + ic];
    return 0;
}

static int cdiv_pos(int a, int b) { return (a + b - 1) / b; } /* a >= 0, b > 0 */

/* Kernel split, Section IV.B Stage 1 and Algorithm 2 (Stage 1), in the paper's
 * own 6-D layout  C[sh][sw][OC][ceil(FH/sh)][ceil(FW/sw)][IC], zero-initialised.
 * Sub-kernel (y,x) has ceil((FH-y)/sh) x ceil((FW-x)/sw) taps (none if that is
 * <= 0, which happens when a stride exceeds the filter); tap (ch,cw) of it is
 * the filter tap
 *   fh = y + (oph - ch)*sh,  fw = x + (opw - cw)*sw,   oph = CH_y - 1,
 * i.e. the rotated filter sampled with steps sh, sw.  Entries outside stay zero. */
int cko_kernel_split(const float *W, float *Cs, int OC, int FH, int FW, int IC, int sh, int sw)
{
    if (OC <= 0 || FH <= 0 || FW <= 0 || IC <= 0 || sh < 1 || sw < 1) return -2;
    const int CHp = cdiv_pos(FH, sh), CWp = cdiv_pos(FW, sw);
    memset(Cs, 0, sizeof(float) * (size_t)sh * sw * OC * CHp * CWp * IC);
    for (int y = 0; y < sh; ++y)
        for (int x = 0; x < sw; ++x) {
            int CHy = y < FH ? cdiv_pos(FH - y, sh) : 0;
            int CWx = x < FW ? cdiv_pos(FW - x, sw) : 0;
            int oph = CHy - 1, opw = CWx - 1;
            for (int oc = 0; oc < OC; ++oc)
                for (int ch = 0; ch < CHy; ++ch)
                    for (int cw = 0; cw < CWx; ++cw) {
                        int fh = y + (oph - ch) * sh, fw = x + (opw - cw) * sw;
                        if (fh < 0 || fh >= FH || fw < 0 || fw >= FW) continue;
                        for (int ic = 0; ic < IC; ++ic)
                            Cs[(((((size_t)y * sw + x) * OC + oc) * CHp + ch) * CWp + cw) * IC + ic] =
                                W[(((size_t)oc * FH + fh) * FW + fw) * IC + ic];
                    }
        }
    return 0;
}

/* ------------------------------------------------------------- cost counting
 * counts[0] dense MACs of Eq. (1): every tap of every patch, padded zeros
 *           included  (Table III, T_Conv / 2)
 * counts[1] useful MACs: index tuples whose input element really exists; the
 *           same set is contracted by all three operators
 * counts[2] nominal MACs of the zero-inserting deconvolution (T_Deconv / 2)
 * counts[3] nominal MACs of the dilating filter gradient (T_Dilated / 2, with
 *           the batch factor N that the printed formula leaves out)
 * Counted by enumeration, not by formula, so the tests can pin the formulas. */
int cko_mac_counts(int64_t *counts, int N, int IC, int IH, int IW, int OC, int FH, int FW, int sh, int sw, int ph, int pw)
{
    if (bad_geometry(N, IC, IH, IW, OC, FH, FW, sh, sw, ph, pw)) return -2;
    const int OH = out_dim(IH, FH, sh, ph), OW = out_dim(IW, FW, sw, pw);
    int64_t dense = 0, useful = 0;
    for (int oh = 0; oh < OH; ++oh)
        for (int ow = 0; ow < OW; ++ow)
            for (int fh = 0; fh < FH; ++fh)
                for (int fw = 0; fw < FW; ++fw) {
                    int ih = oh * sh - ph + fh, iw = ow * sw - pw + fw;
                    ++dense;
                    if (ih >= 0 && ih < IH && iw >= 0 && iw < IW) ++useful;
                }
    int64_t ch = (int64_t)N * IC * OC;
    counts[0] = dense * ch;
    counts[1] = useful * ch;
    counts[2] = (int64_t)IH * IW * FH * FW * ch;
    counts[3] = (int64_t)((OH - 1) * sh + 1) * ((OW - 1) * sw + 1) * FH * FW * ch;
    return 0;
}
