/*
 * TEST INFRASTRUCTURE ONLY -- CPU oracle for stride-2 transpose convolution.
 *
 * Plain, slow, fp64.  Nothing in the product path may call this file; it exists so that the
 * tests, the smoke check and the benchmark's cpu_baseline leg have an independent statement
 * of what the GPU library must compute.  It shares no code, header, table or helper with the
 * HIP kernels.
 *
 * Layouts (all row-major, contiguous, double):
 *   x [B][Cin][H][W]      input feature maps
 *   w [Cout][Cin][n][n]   kernel, used as printed (no flip: Eqs. 1-4 multiply in[i+u] by k[u])
 *   y [B][Cout][OH][OW]   OH = 2H+2P-n, OW = 2W+2P-n   (Sec. 1: (2N-n) for P = 0)
 *   S [B][Cout][OH][OW]   sum of |x*w| over the same terms (tolerance scale); may be NULL
 *
 * Three formulations:
 *   ukst_oracle_naive      -- the ORACLE OF RECORD: Algorithm 1 (bed-of-nails upsample, then a
 *                             stride-1 n x n window), with the upsampled map zero-padded by P
 *                             on every side (Fig. 2 / Sec. 3.4) and summed over input channels
 *                             (Table 4 kernels are n x n x Cin x Cout).
 *   ukst_oracle_scatter    -- check only: every input pixel adds x*w[a][c] at stride 2.
 *   ukst_oracle_segregated -- check only: Algorithm 2 + Eqs. 1-4 + the padding rule of Sec. 3.4
 *                             (four parity sub-kernels, picked per output pixel).
 * The last two exist to pin the first; they are written separately on purpose.
 *
 * Planes are selected by an optional list so that the benchmark can time a bounded sample:
 * plane p = b*Cout + co; planes == NULL means all B*Cout planes.  Unselected planes of y/S are
 * left untouched.
 *
 * Return: 0 ok, 1 bad argument, 2 out of memory.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int ukst_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int bad_args(const double *x, const double *w, double *y, int B, int Cin, int Cout,
                    int H, int W, int n, int P)
{
    if (!x || !w || !y) return 1;
    if (B < 1 || Cin < 1 || Cout < 1 || H < 1 || W < 1 || n < 1 || P < 0) return 1;
    if (2 * H + 2 * P - n < 1 || 2 * W + 2 * P - n < 1) return 1;
    return 0;
}

/* Algorithm 1, generalised to batch / channels / H != W / padding P. */
int ukst_oracle_naive(const double *x, const double *w, double *y, double *S, int B, int Cin,
                      int Cout, int H, int W, int n, int P, const int *planes, int nplanes)
{
    if (bad_args(x, w, y, B, Cin, Cout, H, W, n, P)) return 1;
    const int OH = 2 * H + 2 * P - n, OW = 2 * W + 2 * P - n;
    const int UH = 2 * H - 1 + 2 * P, UW = 2 * W - 1 + 2 * P; /* upsampled + padded */
    const int total = planes ? nplanes : B * Cout;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(| : err)
    for (int t = 0; t < total; ++t) {
        const int p = planes ? planes[t] : t;
        if (p < 0 || p >= B * Cout) { err |= 1; continue; }
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
            /* bed of nails: U[2i][2j] = I[i][j], shifted by the padding P */
            memset(U, 0, sizeof(double) * (size_t)UH * UW);
            for (int i = 0; i < H; ++i)
                for (int j = 0; j < W; ++j)
                    U[(size_t)(P + 2 * i) * UW + (P + 2 * j)] = xp[(size_t)i * W + j];
            /* stride-1 n x n window over U */
            for (int oy = 0; oy < OH; ++oy)
                for (int ox = 0; ox < OW; ++ox) {
                    double acc = 0.0, mag = 0.0;
                    for (int a = 0; a < n; ++a)
                        for (int c = 0; c < n; ++c) {
                            const double t2 = U[(size_t)(oy + a) * UW + (ox + c)] * wp[a * n + c];
                            acc += t2;
                            mag += fabs(t2);
                        }
                    yp[(size_t)oy * OW + ox] += acc;
                    if (sp) sp[(size_t)oy * OW + ox] += mag;
                }
        }
        free(U);
    }
    return err;
}

/* Scatter view: input pixel (i,j) sits at (P+2i, P+2j) of the padded upsampled map, and the
 * window of output (oy,ox) covers it with tap (a,c) = (P+2i-oy, P+2j-ox). */
int ukst_oracle_scatter(const double *x, const double *w, double *y, double *S, int B, int Cin,
                        int Cout, int H, int W, int n, int P)
{
    if (bad_args(x, w, y, B, Cin, Cout, H, W, n, P)) return 1;
    const int OH = 2 * H + 2 * P - n, OW = 2 * W + 2 * P - n;
    const size_t plane = (size_t)OH * OW;
    memset(y, 0, sizeof(double) * plane * B * Cout);
    if (S) memset(S, 0, sizeof(double) * plane * B * Cout);
    for (int b = 0; b < B; ++b)
        for (int co = 0; co < Cout; ++co)
            for (int ci = 0; ci < Cin; ++ci)
                for (int i = 0; i < H; ++i)
                    for (int j = 0; j < W; ++j) {
                        const double xv = x[(((size_t)b * Cin + ci) * H + i) * W + j];
                        for (int a = 0; a < n; ++a) {
                            const int oy = 2 * i + P - a;
                            if (oy < 0 || oy >= OH) continue;
                            for (int c = 0; c < n; ++c) {
                                const int ox = 2 * j + P - c;
                                if (ox < 0 || ox >= OW) continue;
                                const double t2 =
                                    xv * w[(((size_t)co * Cin + ci) * n + a) * n + c];
                                const size_t o = ((size_t)b * Cout + co) * plane +
                                                 (size_t)oy * OW + ox;
                                y[o] += t2;
                                if (S) S[o] += fabs(t2);
                            }
                        }
                    }
    return 0;
}

/* Algorithm 2 with the sub-kernels of Sec. 3.1-3.2 built explicitly first:
 * k_rs[u][v] = K[r+2u][s+2v], sizes ceil/floor(n/2).  With padding P the class of an output
 * pixel is the parity of (coordinate + P) -- this is the "order flips for odd P" rule of
 * Sec. 3.4 -- and the window may overhang the input by floor(P/2), treated as zeros. */
int ukst_oracle_segregated(const double *x, const double *w, double *y, double *S, int B,
                           int Cin, int Cout, int H, int W, int n, int P)
{
    if (bad_args(x, w, y, B, Cin, Cout, H, W, n, P)) return 1;
    const int OH = 2 * H + 2 * P - n, OW = 2 * W + 2 * P - n;
    const int hi = (n + 1) / 2, lo = n / 2; /* ceil(n/2), floor(n/2) */
    double *k[2][2];
    int rows[2] = {hi, lo}, cols[2] = {hi, lo};
    for (int r = 0; r < 2; ++r)
        for (int s = 0; s < 2; ++s) {
            k[r][s] = (double *)malloc(sizeof(double) * (size_t)(hi * hi + 1));
            if (!k[r][s]) return 2;
        }
    for (int b = 0; b < B; ++b)
        for (int co = 0; co < Cout; ++co) {
            double *yp = y + ((size_t)b * Cout + co) * OH * OW;
            double *sp = S ? S + ((size_t)b * Cout + co) * OH * OW : NULL;
            for (size_t t = 0; t < (size_t)OH * OW; ++t) { yp[t] = 0.0; if (sp) sp[t] = 0.0; }
            for (int ci = 0; ci < Cin; ++ci) {
                const double *xp = x + ((size_t)b * Cin + ci) * H * W;
                const double *K = w + ((size_t)co * Cin + ci) * n * n;
                for (int r = 0; r < 2; ++r)
                    for (int s = 0; s < 2; ++s)
                        for (int u = 0; u < rows[r]; ++u)
                            for (int v = 0; v < cols[s]; ++v)
                                k[r][s][u * cols[s] + v] = K[(r + 2 * u) * n + (s + 2 * v)];
                for (int oy = 0; oy < OH; ++oy)
                    for (int ox = 0; ox < OW; ++ox) {
                        const int r = (oy + P) % 2, s = (ox + P) % 2;
                        const int R = rows[r], C = cols[s];
                        /* first input row/col under the window: ceil((oy-P)/2) */
                        const int i0 = (oy + r - P) / 2, j0 = (ox + s - P) / 2;
                        double acc = 0.0, mag = 0.0;
                        for (int u = 0; u < R; ++u)
                            for (int v = 0; v < C; ++v) {
                                const int i = i0 + u, j = j0 + v;
                                if (i < 0 || i >= H || j < 0 || j >= W) continue;
                                const double t2 = xp[(size_t)i * W + j] * k[r][s][u * C + v];
                                acc += t2;
                                mag += fabs(t2);
                            }
                        yp[(size_t)oy * OW + ox] += acc;
                        if (sp) sp[(size_t)oy * OW + ox] += mag;
                    }
            }
        }
    for (int r = 0; r < 2; ++r)
        for (int s = 0; s < 2; ++s) free(k[r][s]);
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * Backward pass.  The paper evaluates the forward layer only; training a generator also needs
 * the two gradients of the same linear map.  Both are written here as the adjoint of
 * Algorithm 1 taken step by step (Algorithm 1: U = bed of nails of the input, padded by P;
 * y = stride-1 n x n window over U, no flip), for the loss  L = sum(dy * y):
 *
 *   ukst_oracle_grad_input   dL/dx: the window step's adjoint spreads every dy over the n x n
 *                            cells of U its window covered (dU[oy+a][ox+c] += dy * w[a][c]);
 *                            the bed-of-nails step's adjoint reads dU back at the cells that
 *                            hold input pixels (dx[i][j] = dU[P+2i][P+2j]) and drops the rest.
 *   ukst_oracle_grad_weight  dL/dw: U is built exactly as in the forward pass and
 *                            dw[a][c] = sum over output pixels of dy[oy][ox] * U[oy+a][ox+c].
 *
 * Layouts as above; dy [B][Cout][OH][OW], dx [B][Cin][H][W], dw [Cout][Cin][n][n].
 * S (optional) receives the sum of the absolute values of the same products (tolerance scale).
 * Pinned in tests/test_oracle_backward_pins.py against the forward oracle (adjoint identity,
 * element by element through unit vectors), hand-worked values and a library autograd.
 */
static int bad_args3(const void *p0, const void *p1, const void *p2, int B, int Cin, int Cout,
                     int H, int W, int n, int P)
{
    if (!p0 || !p1 || !p2) return 1;
    if (B < 1 || Cin < 1 || Cout < 1 || H < 1 || W < 1 || n < 1 || P < 0) return 1;
    if (2 * H + 2 * P - n < 1 || 2 * W + 2 * P - n < 1) return 1;
    return 0;
}

int ukst_oracle_grad_input(const double *dy, const double *w, double *dx, double *S, int B,
                           int Cin, int Cout, int H, int W, int n, int P)
{
    if (bad_args3(dy, w, dx, B, Cin, Cout, H, W, n, P)) return 1;
    const int OH = 2 * H + 2 * P - n, OW = 2 * W + 2 * P - n;
    const int UH = 2 * H - 1 + 2 * P, UW = 2 * W - 1 + 2 * P;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(| : err)
    for (int p = 0; p < B * Cin; ++p) {
        const int b = p / Cin, ci = p % Cin;
        double *dU = (double *)calloc((size_t)UH * UW, sizeof(double));
        double *aU = (double *)calloc((size_t)UH * UW, sizeof(double));
        if (!dU || !aU) { err |= 2; free(dU); free(aU); continue; }
        for (int co = 0; co < Cout; ++co) {
            const double *dyp = dy + ((size_t)b * Cout + co) * OH * OW;
            const double *wp = w + ((size_t)co * Cin + ci) * n * n;
            for (int oy = 0; oy < OH; ++oy)
                for (int ox = 0; ox < OW; ++ox)
                    for (int a = 0; a < n; ++a)
                        for (int c = 0; c < n; ++c) {
                            const double t = dyp[(size_t)oy * OW + ox] * wp[a * n + c];
                            dU[(size_t)(oy + a) * UW + (ox + c)] += t;
                            aU[(size_t)(oy + a) * UW + (ox + c)] += fabs(t);
                        }
        }
        for (int i = 0; i < H; ++i)
            for (int j = 0; j < W; ++j) {
                dx[(size_t)p * H * W + (size_t)i * W + j] = dU[(size_t)(P + 2 * i) * UW + (P + 2 * j)];
                if (S) S[(size_t)p * H * W + (size_t)i * W + j] = aU[(size_t)(P + 2 * i) * UW + (P + 2 * j)];
            }
        free(dU);
        free(aU);
    }
    return err;
}

int ukst_oracle_grad_weight(const double *x, const double *dy, double *dw, double *S, int B,
                            int Cin, int Cout, int H, int W, int n, int P)
{
    if (bad_args3(x, dy, dw, B, Cin, Cout, H, W, n, P)) return 1;
    const int OH = 2 * H + 2 * P - n, OW = 2 * W + 2 * P - n;
    const int UH = 2 * H - 1 + 2 * P, UW = 2 * W - 1 + 2 * P;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(| : err)
    for (int ci = 0; ci < Cin; ++ci) {
        double *U = (double *)malloc(sizeof(double) * (size_t)UH * UW);
        if (!U) { err |= 2; continue; }
        for (int co = 0; co < Cout; ++co)
            for (int t = 0; t < n * n; ++t) {
                dw[((size_t)co * Cin + ci) * n * n + t] = 0.0;
                if (S) S[((size_t)co * Cin + ci) * n * n + t] = 0.0;
            }
        for (int b = 0; b < B; ++b) {
            const double *xp = x + ((size_t)b * Cin + ci) * H * W;
            memset(U, 0, sizeof(double) * (size_t)UH * UW);
            for (int i = 0; i < H; ++i)
                for (int j = 0; j < W; ++j)
                    U[(size_t)(P + 2 * i) * UW + (P + 2 * j)] = xp[(size_t)i * W + j];
            for (int co = 0; co < Cout; ++co) {
                const double *dyp = dy + ((size_t)b * Cout + co) * OH * OW;
                double *dwp = dw + ((size_t)co * Cin + ci) * n * n;
                double *sp = S ? S + ((size_t)co * Cin + ci) * n * n : NULL;
                for (int a = 0; a < n; ++a)
                    for (int c = 0; c < n; ++c) {
                        double acc = 0.0, mag = 0.0;
                        for (int oy = 0; oy < OH; ++oy)
                            for (int ox = 0; ox < OW; ++ox) {
                                const double t = dyp[(size_t)oy * OW + ox] *
                                                 U[(size_t)(oy + a) * UW + (ox + c)];
                                acc += t;
                                mag += fabs(t);
                            }
                        dwp[a * n + c] += acc;
                        if (sp) sp[a * n + c] += mag;
                    }
            }
        }
        free(U);
    }
    return err;
}
