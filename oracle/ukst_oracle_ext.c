/*
 * TEST INFRASTRUCTURE ONLY -- CPU oracle for the two generalisations the paper's Sec. 5 points to:
 * transpose convolution with a general stride s (s*s parity classes instead of four) and dilated
 * convolution evaluated on segregated input feature maps.  Plain, slow, fp64; nothing in the
 * product path may call this file, and it shares nothing with the HIP kernels.
 *
 * Layouts as in ukst_oracle.c: x [B][Cin][H][W], w [Cout][Cin][n][n] used as printed (no flip),
 * y / S [B][Cout][OH][OW]; S = sum of |x*w| over the same terms (tolerance scale), may be NULL.
 *
 * Stride-s transpose convolution (Algorithm 1 with s-1 zeros between neighbouring pixels instead
 * of one; s = 2 is the paper's case):
 *   ukst_oracle_strided_naive      -- ORACLE OF RECORD: bed-of-nails upsample to s(H-1)+1, zero-pad
 *                                     by P, stride-1 n x n window.  OH = s(H-1) + 2P - n + 2.
 *   ukst_oracle_strided_segregated -- check only: Algorithm 2 with s*s sub-kernels
 *                                     k_rc[u][v] = K[r+s*u][c+s*v], class picked per output pixel.
 * Dilated convolution (Sec. 5: the KERNEL is upsampled with the bed of nails, then an ordinary
 * convolution is applied; dilation d puts d-1 zeros between neighbouring taps):
 *   ukst_oracle_dilated_naive      -- ORACLE OF RECORD: build the (d(n-1)+1)-sided kernel with the
 *                                     zeros in it, zero-pad the input by P, stride-1 window.
 *                                     OH = H + 2P - d(n-1).
 *   ukst_oracle_dilated_segregated -- check only: the input is split into d*d sub-sampled maps
 *                                     x_pq[i][j] = xpad[p+d*i][q+d*j]; each is convolved with the
 *                                     unmodified n x n kernel and the results are interleaved.
 *
 * Return: 0 ok, 1 bad argument, 2 out of memory.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

static int bad_common(const double *x, const double *w, double *y, int B, int Cin, int Cout, int H,
                      int W, int n, int P)
{
    if (!x || !w || !y) return 1;
    if (B < 1 || Cin < 1 || Cout < 1 || H < 1 || W < 1 || n < 1 || P < 0) return 1;
    return 0;
}

int ukst_oracle_strided_naive(const double *x, const double *w, double *y, double *S, int B, int Cin,
                              int Cout, int H, int W, int n, int P, int s)
{
    if (bad_common(x, w, y, B, Cin, Cout, H, W, n, P) || s < 1) return 1;
    const int UH = s * (H - 1) + 1 + 2 * P, UW = s * (W - 1) + 1 + 2 * P; /* upsampled + padded */
    const int OH = UH - n + 1, OW = UW - n + 1;
    if (OH < 1 || OW < 1) return 1;
    const int total = B * Cout;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(| : err)
    for (int p = 0; p < total; ++p) {
        const int b = p / Cout, co = p % Cout;
        double *U = (double *)malloc(sizeof(double) * (size_t)UH * UW);
        if (!U) { err |= 2; continue; }
        double *yp = y + (size_t)p * OH * OW;
        double *sp = S ? S + (size_t)p * OH * OW : NULL;
        memset(yp, 0, sizeof(double) * (size_t)OH * OW);
        if (sp) memset(sp, 0, sizeof(double) * (size_t)OH * OW);
        for (int ci = 0; ci < Cin; ++ci) {
            const double *xp = x + ((size_t)b * Cin + ci) * H * W;
            const double *wp = w + ((size_t)co * Cin + ci) * n * n;
            /* bed of nails with s-1 zeros between pixels: U[s*i][s*j] = I[i][j], shifted by P */
            memset(U, 0, sizeof(double) * (size_t)UH * UW);
            for (int i = 0; i < H; ++i)
                for (int j = 0; j < W; ++j)
                    U[(size_t)(P + s * i) * UW + (P + s * j)] = xp[(size_t)i * W + j];
            for (int oy = 0; oy < OH; ++oy)
                for (int ox = 0; ox < OW; ++ox) {
                    double acc = 0.0, mag = 0.0;
                    for (int a = 0; a < n; ++a)
                        for (int c = 0; c < n; ++c) {
                            const double t = U[(size_t)(oy + a) * UW + (ox + c)] * wp[a * n + c];
                            acc += t;
                            mag += fabs(t);
                        }
                    yp[(size_t)oy * OW + ox] += acc;
                    if (sp) sp[(size_t)oy * OW + ox] += mag;
                }
        }
        free(U);
    }
    return err;
}

/* Algorithm 2 for stride s.  Tap a of output row oy meets a pixel only where oy + a - P is a
 * multiple of s: the row class is r = (P - oy) mod s, its taps are r, r+s, r+2s, ... and tap r+s*u
 * reads input row (oy + r - P)/s + u.  The s*s sub-kernels are built explicitly first. */
int ukst_oracle_strided_segregated(const double *x, const double *w, double *y, double *S, int B,
                                   int Cin, int Cout, int H, int W, int n, int P, int s)
{
    if (bad_common(x, w, y, B, Cin, Cout, H, W, n, P) || s < 1) return 1;
    const int OH = s * (H - 1) + 2 * P - n + 2, OW = s * (W - 1) + 2 * P - n + 2;
    if (OH < 1 || OW < 1) return 1;
    const int T = (n + s - 1) / s; /* largest sub-kernel side */
    double *sub = (double *)malloc(sizeof(double) * (size_t)s * s * T * T);
    if (!sub) return 2;
    for (int b = 0; b < B; ++b)
        for (int co = 0; co < Cout; ++co) {
            double *yp = y + ((size_t)b * Cout + co) * OH * OW;
            double *sp = S ? S + ((size_t)b * Cout + co) * OH * OW : NULL;
            memset(yp, 0, sizeof(double) * (size_t)OH * OW);
            if (sp) memset(sp, 0, sizeof(double) * (size_t)OH * OW);
            for (int ci = 0; ci < Cin; ++ci) {
                const double *xp = x + ((size_t)b * Cin + ci) * H * W;
                const double *wp = w + ((size_t)co * Cin + ci) * n * n;
                /* sub-kernel (r, c): taps r + s*u, c + s*v of the kernel */
                memset(sub, 0, sizeof(double) * (size_t)s * s * T * T);
                for (int r = 0; r < s; ++r)
                    for (int c = 0; c < s; ++c)
                        for (int u = 0; r + s * u < n; ++u)
                            for (int v = 0; c + s * v < n; ++v)
                                sub[(((size_t)r * s + c) * T + u) * T + v] = wp[(r + s * u) * n + (c + s * v)];
                for (int oy = 0; oy < OH; ++oy) {
                    const int r = ((P - oy) % s + s) % s;
                    const int Tr = r < n ? (n - r + s - 1) / s : 0;
                    const int i0 = (oy + r - P) / s; /* exact: oy + r - P is a multiple of s */
                    for (int ox = 0; ox < OW; ++ox) {
                        const int c = ((P - ox) % s + s) % s;
                        const int Tc = c < n ? (n - c + s - 1) / s : 0;
                        const int j0 = (ox + c - P) / s;
                        double acc = 0.0, mag = 0.0;
                        for (int u = 0; u < Tr; ++u) {
                            const int i = i0 + u;
                            if (i < 0 || i >= H) continue;
                            for (int v = 0; v < Tc; ++v) {
                                const int j = j0 + v;
                                if (j < 0 || j >= W) continue;
                                const double t = xp[(size_t)i * W + j] *
                                                 sub[(((size_t)r * s + c) * T + u) * T + v];
                                acc += t;
                                mag += fabs(t);
                            }
                        }
                        yp[(size_t)oy * OW + ox] += acc;
                        if (sp) sp[(size_t)oy * OW + ox] += mag;
                    }
                }
            }
        }
    free(sub);
    return 0;
}

int ukst_oracle_dilated_naive(const double *x, const double *w, double *y, double *S, int B, int Cin,
                              int Cout, int H, int W, int n, int P, int d)
{
    if (bad_common(x, w, y, B, Cin, Cout, H, W, n, P) || d < 1) return 1;
    const int nd = d * (n - 1) + 1;        /* side of the upsampled kernel */
    const int PH = H + 2 * P, PW = W + 2 * P; /* zero-padded input */
    const int OH = PH - nd + 1, OW = PW - nd + 1;
    if (OH < 1 || OW < 1) return 1;
    const int total = B * Cout;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(| : err)
    for (int p = 0; p < total; ++p) {
        const int b = p / Cout, co = p % Cout;
        double *Xp = (double *)malloc(sizeof(double) * (size_t)PH * PW);
        double *Kd = (double *)malloc(sizeof(double) * (size_t)nd * nd);
        if (!Xp || !Kd) { err |= 2; free(Xp); free(Kd); continue; }
        double *yp = y + (size_t)p * OH * OW;
        double *sp = S ? S + (size_t)p * OH * OW : NULL;
        memset(yp, 0, sizeof(double) * (size_t)OH * OW);
        if (sp) memset(sp, 0, sizeof(double) * (size_t)OH * OW);
        for (int ci = 0; ci < Cin; ++ci) {
            const double *xp = x + ((size_t)b * Cin + ci) * H * W;
            const double *wp = w + ((size_t)co * Cin + ci) * n * n;
            /* bed of nails on the KERNEL: Kd[d*a][d*c] = K[a][c], zeros elsewhere */
            memset(Kd, 0, sizeof(double) * (size_t)nd * nd);
            for (int a = 0; a < n; ++a)
                for (int c = 0; c < n; ++c) Kd[(size_t)(d * a) * nd + d * c] = wp[a * n + c];
            memset(Xp, 0, sizeof(double) * (size_t)PH * PW);
            for (int i = 0; i < H; ++i)
                for (int j = 0; j < W; ++j) Xp[(size_t)(P + i) * PW + (P + j)] = xp[(size_t)i * W + j];
            for (int oy = 0; oy < OH; ++oy)
                for (int ox = 0; ox < OW; ++ox) {
                    double acc = 0.0, mag = 0.0;
                    for (int a = 0; a < nd; ++a)
                        for (int c = 0; c < nd; ++c) {
                            const double t = Xp[(size_t)(oy + a) * PW + (ox + c)] * Kd[(size_t)a * nd + c];
                            acc += t;
                            mag += fabs(t);
                        }
                    yp[(size_t)oy * OW + ox] += acc;
                    if (sp) sp[(size_t)oy * OW + ox] += mag;
                }
        }
        free(Xp);
        free(Kd);
    }
    return err;
}

/* Segregated input: output pixel (oy, ox) only ever meets padded-input pixels whose coordinates
 * are congruent to (oy, ox) modulo d.  Split the padded input into its d*d sub-sampled maps,
 * correlate each with the unmodified kernel (dense, stride 1) and interleave the results. */
int ukst_oracle_dilated_segregated(const double *x, const double *w, double *y, double *S, int B,
                                   int Cin, int Cout, int H, int W, int n, int P, int d)
{
    if (bad_common(x, w, y, B, Cin, Cout, H, W, n, P) || d < 1) return 1;
    const int PH = H + 2 * P, PW = W + 2 * P;
    const int OH = PH - d * (n - 1), OW = PW - d * (n - 1);
    if (OH < 1 || OW < 1) return 1;
    const int SH = (PH + d - 1) / d, SW = (PW + d - 1) / d; /* largest sub-map */
    double *sub = (double *)malloc(sizeof(double) * (size_t)SH * SW);
    if (!sub) return 2;
    memset(y, 0, sizeof(double) * (size_t)B * Cout * OH * OW);
    if (S) memset(S, 0, sizeof(double) * (size_t)B * Cout * OH * OW);
    for (int b = 0; b < B; ++b)
        for (int ci = 0; ci < Cin; ++ci) {
            const double *xp = x + ((size_t)b * Cin + ci) * H * W;
            for (int p = 0; p < d; ++p)
                for (int q = 0; q < d; ++q) {
                    /* sub-map (p, q) of the padded input: rows p, p+d, ...; columns q, q+d, ... */
                    const int sh = p < PH ? (PH - p + d - 1) / d : 0;
                    const int sw = q < PW ? (PW - q + d - 1) / d : 0;
                    for (int i = 0; i < sh; ++i)
                        for (int j = 0; j < sw; ++j) {
                            const int pi = p + d * i - P, pj = q + d * j - P;
                            sub[(size_t)i * SW + j] =
                                (pi >= 0 && pi < H && pj >= 0 && pj < W) ? xp[(size_t)pi * W + pj] : 0.0;
                        }
                    /* dense n x n window over the sub-map; its outputs are rows p, p+d, ... of y */
                    for (int co = 0; co < Cout; ++co) {
                        const double *wp = w + ((size_t)co * Cin + ci) * n * n;
                        double *yp = y + ((size_t)b * Cout + co) * OH * OW;
                        double *sp = S ? S + ((size_t)b * Cout + co) * OH * OW : NULL;
                        for (int i = 0; i + n <= sh; ++i) {
                            const int oy = p + d * i;
                            if (oy >= OH) break;
                            for (int j = 0; j + n <= sw; ++j) {
                                const int ox = q + d * j;
                                if (ox >= OW) break;
                                double acc = 0.0, mag = 0.0;
                                for (int a = 0; a < n; ++a)
                                    for (int c = 0; c < n; ++c) {
                                        const double t = sub[(size_t)(i + a) * SW + (j + c)] * wp[a * n + c];
                                        acc += t;
                                        mag += fabs(t);
                                    }
                                yp[(size_t)oy * OW + ox] += acc;
                                if (sp) sp[(size_t)oy * OW + ox] += mag;
                            }
                        }
                    }
                }
        }
    free(sub);
    return 0;
}
