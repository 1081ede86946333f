/*
 * Sanitizer run of the CPU oracle -- TEST INFRASTRUCTURE, like cks_oracle.c, which this file includes.
 *
 * Built by tests/test_sanitizers.py as one executable with -fsanitize=address,undefined and run on the
 * CPU: every function of the oracle is driven over small geometries (strides 1-3 per axis, padding from
 * 0 to beyond the filter, stride larger than the filter, remainder rows, full and sampled mode), so that
 * an out-of-bounds access or undefined arithmetic in the materialised-zero tensors aborts the run.  The
 * three operators are also compared with the 7-deep brute-force loop (exact: integer-valued inputs).
 * Prints the number of geometries and exits 0, or says what differed and exits 1.
 */
#include "cks_oracle.c"

#include <stdio.h>

static unsigned long long state = 88172645463325252ULL;
static int small_int(void)   /* -3 .. 3 */
{
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (int)(state % 7ULL) - 3;
}

static float *filled(size_t n)
{
    float *p = (float *)malloc((n ? n : 1) * sizeof(float));
    for (size_t i = 0; i < n; ++i) p[i] = (float)small_int();
    return p;
}

static int differ(const double *a, const double *b, size_t n, const char *what, const int *g)
{
    for (size_t i = 0; i < n; ++i)
        if (a[i] != b[i]) {
            printf("%s differs at %zu: %g vs %g (N=%d IC=%d IH=%d IW=%d OC=%d FH=%d FW=%d sh=%d sw=%d ph=%d pw=%d)\n",
                   what, i, a[i], b[i], g[0], g[1], g[2], g[3], g[4], g[5], g[6], g[7], g[8], g[9], g[10]);
            return 1;
        }
    return 0;
}

static int one(const int *g)
{
    const int N = g[0], IC = g[1], IH = g[2], IW = g[3], OC = g[4], FH = g[5], FW = g[6], sh = g[7], sw = g[8], ph = g[9], pw = g[10];
    if (IH + 2 * ph < FH || IW + 2 * pw < FW) return 0;
    const int OH = cko_out_dim(IH, FH, sh, ph), OW = cko_out_dim(IW, FW, sw, pw);
    const size_t nx = (size_t)N * IH * IW * IC, nw = (size_t)OC * FH * FW * IC, ny = (size_t)N * OH * OW * OC;
    float *X = filled(nx), *W = filled(nw), *dY = filled(ny);
    double *Y = malloc(ny * sizeof(double)), *dX = malloc(nx * sizeof(double)), *dW = malloc(nw * sizeof(double));
    double *Yb = malloc(ny * sizeof(double)), *dXb = malloc(nx * sizeof(double)), *dWb = malloc(nw * sizeof(double));
    int bad = 0;
    bad |= cko_conv_fwd(X, W, Y, N, IC, IH, IW, OC, FH, FW, sh, sw, ph, pw, NULL, 0);
    bad |= cko_deconv(dY, W, dX, N, IC, IH, IW, OC, FH, FW, sh, sw, ph, pw, NULL, 0);
    bad |= cko_wgrad(X, dY, dW, N, IC, IH, IW, OC, FH, FW, sh, sw, ph, pw, NULL, 0);
    bad |= cko_brute(X, W, dY, Yb, dXb, dWb, N, IC, IH, IW, OC, FH, FW, sh, sw, ph, pw);
    if (bad) { printf("an operator rejected a valid geometry\n"); return 1; }
    bad |= differ(Y, Yb, ny, "conv_fwd", g) | differ(dX, dXb, nx, "deconv", g) | differ(dW, dWb, nw, "wgrad", g);
    /* sampled mode: first, last and a middle element of each result */
    int64_t s[3];
    double o[3];
    s[0] = 0; s[1] = (int64_t)ny / 2; s[2] = (int64_t)ny - 1;
    bad |= cko_conv_fwd(X, W, o, N, IC, IH, IW, OC, FH, FW, sh, sw, ph, pw, s, 3);
    for (int i = 0; i < 3; ++i) bad |= o[i] != Y[s[i]];
    s[1] = (int64_t)nx / 2; s[2] = (int64_t)nx - 1;
    bad |= cko_deconv(dY, W, o, N, IC, IH, IW, OC, FH, FW, sh, sw, ph, pw, s, 3);
    for (int i = 0; i < 3; ++i) bad |= o[i] != dX[s[i]];
    s[1] = (int64_t)nw / 2; s[2] = (int64_t)nw - 1;
    bad |= cko_wgrad(X, dY, o, N, IC, IH, IW, OC, FH, FW, sh, sw, ph, pw, s, 3);
    for (int i = 0; i < 3; ++i) bad |= o[i] != dW[s[i]];
    if (bad) printf("sampled mode differs from full mode\n");
    /* data movement and counting */
    float *Wt = malloc((nw ? nw : 1) * sizeof(float));
    const size_t nc = (size_t)sh * sw * OC * ((FH + sh - 1) / sh) * ((FW + sw - 1) / sw) * IC;
    float *Cs = malloc((nc ? nc : 1) * sizeof(float));
    bad |= cko_filter_transpose(W, Wt, OC, FH, FW, IC);
    bad |= cko_kernel_split(W, Cs, OC, FH, FW, IC, sh, sw);
    double sumC = 0;                 /* the split is a partition of the filter: every tap once, zeros elsewhere */
    for (size_t i = 0; i < nw; ++i) sumC += W[i];
    double sumS = 0;
    for (size_t i = 0; i < nc; ++i) sumS += Cs[i];
    if (sumS != sumC) { printf("kernel split does not hold every tap once\n"); bad = 1; }
    int64_t counts[4];
    bad |= cko_mac_counts(counts, N, IC, IH, IW, OC, FH, FW, sh, sw, ph, pw);
    if (counts[1] > counts[0]) { printf("more useful than dense multiply-adds\n"); bad = 1; }
    free(X); free(W); free(dY); free(Y); free(dX); free(dW); free(Yb); free(dXb); free(dWb); free(Wt); free(Cs);
    return bad;
}

int main(void)
{
    int done = 0, bad = 0;
    const int maps[][2] = {{1, 1}, {3, 4}, {4, 4}, {5, 7}, {8, 6}};
    const int filters[][2] = {{1, 1}, {2, 3}, {3, 3}, {4, 2}, {5, 5}};
    for (unsigned m = 0; m < sizeof maps / sizeof maps[0]; ++m)
        for (unsigned f = 0; f < sizeof filters / sizeof filters[0]; ++f)
            for (int sh = 1; sh <= 3; ++sh)
                for (int sw = 1; sw <= 3; sw += 2)
                    for (int ph = 0; ph <= 5; ph += (ph < 2 ? 1 : 3))
                        for (int pw = 0; pw <= 4; pw += 2) {
                            const int g[11] = {2, 3, maps[m][0], maps[m][1], 2, filters[f][0], filters[f][1], sh, sw, ph, pw};
                            if (maps[m][0] + 2 * ph < filters[f][0] || maps[m][1] + 2 * pw < filters[f][1]) continue;
                            bad |= one(g);
                            ++done;
                        }
    /* rejected geometries must not touch memory */
    double dummy[1];
    float fdummy[1] = {0};
    if (cko_conv_fwd(fdummy, fdummy, dummy, 1, 1, 2, 2, 1, 5, 5, 1, 1, 1, 1, NULL, 0) == 0) { printf("filter larger than the padded input accepted\n"); bad = 1; }
    if (cko_conv_fwd(fdummy, fdummy, dummy, 1, 1, 2, 2, 1, 1, 1, 0, 1, 0, 0, NULL, 0) == 0) { printf("stride 0 accepted\n"); bad = 1; }
    printf("%d geometries %s\n", done, bad ? "FAILED" : "ok");
    return bad ? 1 : 0;
}
