/*
 * The oracle's pins once more, from plain C, for a build of oracle/oracle.c under
 * -fsanitize=address,undefined (test infrastructure; tests/test_sanitize.py builds and runs it).
 * The Python pins of tests/test_oracle_*.py go through ctypes, where a stray read or write of
 * the oracle's index arithmetic would go unnoticed as long as the numbers come out right; here
 * every buffer is exactly as large as the interface says, so the sanitizer sees any access
 * outside it.  Checks: the hand-worked example of the three passes (Section 2's equations;
 * the values of tests/golden/hand_conv_3x3.txt), impulse responses, plane selections against the
 * full result (first, last, repeated and out-of-order planes), kernel as large as the image,
 * closed-form transforms (DFT definition of the Supplement), inverse after forward with
 * zero padding and crop in 1-D and 2-D, the O(n^4) 2-D definition, and the convolution
 * theorem (Section 2) on a ragged shape.
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void oracle_conv_fprop(const double *x, const double *w, double *y, int S, int f, int fo, int h, int wd,
                       int kh, int kw, const long *sel, long nsel);
void oracle_conv_bprop(const double *gy, const double *w, double *gx, int S, int f, int fo, int h, int wd,
                       int kh, int kw, const long *sel, long nsel);
void oracle_conv_accgrad(const double *x, const double *gy, double *gw, int S, int f, int fo, int h, int wd,
                         int kh, int kw, const long *sel, long nsel);
void oracle_dft_r2c_1d(const double *in, double *out, long B, int n_in, int n);
void oracle_idft_c2r_1d(const double *in, double *out, long B, int n, int n_out);
void oracle_dft_r2c_2d(const double *in, double *out, long B, int h_in, int w_in, int n);
void oracle_idft_c2r_2d(const double *in, double *out, long B, int n, int h_out, int w_out);
void oracle_dft2_bruteforce(const double *in, double *out, int n);

static int bad = 0;
static void expect(int ok, const char *what) {
    printf("%-58s %s\n", what, ok ? "ok" : "FAIL");
    if (!ok) ++bad;
}
static double maxdiff(const double *a, const double *b, size_t n) {
    double m = 0;
    for (size_t i = 0; i < n; ++i) { const double d = fabs(a[i] - b[i]); if (d > m) m = d; }
    return m;
}
static unsigned long long rs = 88172645463325252ull;
static double rnd(void) {   /* xorshift64, uniform in [-1, 1) */
    rs ^= rs << 13; rs ^= rs >> 7; rs ^= rs << 17;
    return (double)(rs >> 11) / 4503599627370496.0 - 1.0;
}
static double *randoms(size_t n) {
    double *p = (double *)malloc(n * sizeof(double));
    for (size_t i = 0; i < n; ++i) p[i] = rnd();
    return p;
}

static void hand_example(void) {
    const double x[9] = {1, 2, 3, 4, 5, 6, 7, 8, 9}, w[4] = {1, 0, 0, -1}, gy[4] = {1, 1, 1, 1};
    const double y_ref[4] = {-4, -4, -4, -4}, gx_ref[9] = {1, 1, 0, 1, 0, -1, 0, -1, -1}, gw_ref[4] = {12, 16, 24, 28};
    double y[4], gx[9], gw[4];
    oracle_conv_fprop(x, w, y, 1, 1, 1, 3, 3, 2, 2, NULL, 0);
    oracle_conv_bprop(gy, w, gx, 1, 1, 1, 3, 3, 2, 2, NULL, 0);
    oracle_conv_accgrad(x, gy, gw, 1, 1, 1, 3, 3, 2, 2, NULL, 0);
    expect(maxdiff(y, y_ref, 4) == 0 && maxdiff(gx, gx_ref, 9) == 0 && maxdiff(gw, gw_ref, 4) == 0,
           "hand example: fprop, bprop, accGrad");
}

static void impulses(void) {
    /* x = delta at (p, q): y[a, b] = w[p - a, q - b];  w = delta at (u0, v0): y[a, b] = x[a + u0, b + v0] */
    enum { H = 6, W = 7, KH = 3, KW = 2, OH = H - KH + 1, OW = W - KW + 1 };
    double x[H * W], *w = randoms(KH * KW), y[OH * OW];
    memset(x, 0, sizeof x);
    const int p = 3, q = 4;
    x[p * W + q] = 1.0;
    oracle_conv_fprop(x, w, y, 1, 1, 1, H, W, KH, KW, NULL, 0);
    int ok = 1;
    for (int a = 0; a < OH; ++a)
        for (int b = 0; b < OW; ++b) {
            const int u = p - a, v = q - b;
            const double want = (u >= 0 && u < KH && v >= 0 && v < KW) ? w[u * KW + v] : 0.0;
            if (y[a * OW + b] != want) ok = 0;
        }
    expect(ok, "impulse image: y[a,b] = w[p-a, q-b]");
    double *xr = randoms(H * W), wd[KH * KW];
    memset(wd, 0, sizeof wd);
    wd[2 * KW + 1] = 1.0;
    oracle_conv_fprop(xr, wd, y, 1, 1, 1, H, W, KH, KW, NULL, 0);
    ok = 1;
    for (int a = 0; a < OH; ++a)
        for (int b = 0; b < OW; ++b) if (y[a * OW + b] != xr[(a + 2) * W + (b + 1)]) ok = 0;
    expect(ok, "impulse kernel: y[a,b] = x[a+u0, b+v0]");
    free(w); free(xr);
}

static void selections(void) {
    enum { S = 3, F = 2, FO = 4, H = 5, W = 4, KH = 2, KW = 3, OH = H - KH + 1, OW = W - KW + 1 };
    double *x = randoms(S * F * H * W), *w = randoms(FO * F * KH * KW), *gy = randoms(S * FO * OH * OW);
    double y[S * FO * OH * OW], gx[S * F * H * W], gw[FO * F * KH * KW];
    oracle_conv_fprop(x, w, y, S, F, FO, H, W, KH, KW, NULL, 0);
    oracle_conv_bprop(gy, w, gx, S, F, FO, H, W, KH, KW, NULL, 0);
    oracle_conv_accgrad(x, gy, gw, S, F, FO, H, W, KH, KW, NULL, 0);
    const long sy[4] = {S * FO - 1, 0, 5, 5}, sx[3] = {S * F - 1, 2, 0}, sw[3] = {FO * F - 1, 0, 3};
    double ys[4 * OH * OW], gxs[3 * H * W], gws[3 * KH * KW];
    oracle_conv_fprop(x, w, ys, S, F, FO, H, W, KH, KW, sy, 4);
    oracle_conv_bprop(gy, w, gxs, S, F, FO, H, W, KH, KW, sx, 3);
    oracle_conv_accgrad(x, gy, gws, S, F, FO, H, W, KH, KW, sw, 3);
    int ok = 1;
    for (int r = 0; r < 4; ++r) if (maxdiff(ys + r * OH * OW, y + sy[r] * OH * OW, OH * OW) != 0) ok = 0;
    for (int r = 0; r < 3; ++r) if (maxdiff(gxs + r * H * W, gx + sx[r] * H * W, H * W) != 0) ok = 0;
    for (int r = 0; r < 3; ++r) if (maxdiff(gws + r * KH * KW, gw + sw[r] * KH * KW, KH * KW) != 0) ok = 0;
    expect(ok, "plane selections equal the full result");
    /* adjoint identity: <fprop(x, w), gy> = <x, bprop(gy, w)> = <w, accGrad(x, gy)> */
    double a = 0, b = 0, c = 0;
    for (int i = 0; i < S * FO * OH * OW; ++i) a += y[i] * gy[i];
    for (int i = 0; i < S * F * H * W; ++i) b += x[i] * gx[i];
    for (int i = 0; i < FO * F * KH * KW; ++i) c += w[i] * gw[i];
    expect(fabs(a - b) < 1e-12 * fabs(a) + 1e-12 && fabs(a - c) < 1e-12 * fabs(a) + 1e-12, "adjoint identity of the three passes");
    /* kernel as large as the image: one output pixel, the plain inner product */
    double one[1], dot = 0;
    oracle_conv_fprop(x, x, one, 1, 1, 1, H, W, H, W, NULL, 0);
    for (int i = 0; i < H * W; ++i) dot += x[i] * x[i];
    expect(fabs(one[0] - dot) < 1e-13, "kernel as large as the image");
    free(x); free(w); free(gy);
}

static void transforms(void) {
    /* delta -> all ones; constant -> n at bin 0; n = 4 by hand: x = (1, 2, 3, 4) -> (10, -2 + 2i, -2) */
    double d[8] = {1, 0, 0, 0, 0, 0, 0, 0}, D[5 * 2];
    oracle_dft_r2c_1d(d, D, 1, 8, 8);
    int ok = 1;
    for (int k = 0; k < 5; ++k) if (fabs(D[2 * k] - 1) > 1e-15 || fabs(D[2 * k + 1]) > 1e-15) ok = 0;
    const double x4[4] = {1, 2, 3, 4};
    double X4[3 * 2];
    oracle_dft_r2c_1d(x4, X4, 1, 4, 4);
    const double want[6] = {10, 0, -2, 2, -2, 0};
    if (maxdiff(X4, want, 6) > 1e-14) ok = 0;
    expect(ok, "closed forms: delta, n = 4 by hand");
    /* zero padding from n_in < n, every supported kind of length, inverse with crop gives the input back */
    ok = 1;
    const int sizes[] = {2, 8, 12, 14, 18, 20, 36, 64};
    for (unsigned t = 0; t < sizeof sizes / sizeof *sizes; ++t) {
        const int n = sizes[t], n_in = n > 3 ? n - 3 : n, nb = n / 2 + 1;
        const long B = 3;
        double *x = randoms(B * n_in), *X = (double *)malloc(sizeof(double) * B * nb * 2), *back = (double *)malloc(sizeof(double) * B * n_in);
        oracle_dft_r2c_1d(x, X, B, n_in, n);
        oracle_idft_c2r_1d(X, back, B, n, n_in);
        if (maxdiff(x, back, B * n_in) > 1e-13) ok = 0;
        free(x); free(X); free(back);
    }
    expect(ok, "1-D inverse of forward with padding and crop");
    ok = 1;
    for (unsigned t = 0; t < 5; ++t) {
        const int n = sizes[t + 1], h_in = n - 3, w_in = n - 1, nb = n / 2 + 1;
        const long B = 2;
        double *x = randoms(B * h_in * w_in), *X = (double *)malloc(sizeof(double) * B * n * nb * 2);
        double *back = (double *)malloc(sizeof(double) * B * h_in * w_in);
        oracle_dft_r2c_2d(x, X, B, h_in, w_in, n);
        oracle_idft_c2r_2d(X, back, B, n, h_in, w_in);
        if (maxdiff(x, back, B * h_in * w_in) > 1e-12) ok = 0;
        free(x); free(X); free(back);
    }
    expect(ok, "2-D inverse of forward with padding and crop");
    /* separable 2-D transform against the four-index definition */
    enum { N = 6, NB = N / 2 + 1 };
    double *x = randoms(N * N), X[N * NB * 2], full[N * N * 2];
    oracle_dft_r2c_2d(x, X, 1, N, N, N);
    oracle_dft2_bruteforce(x, full, N);
    ok = 1;
    for (int k1 = 0; k1 < N; ++k1)
        for (int k2 = 0; k2 < NB; ++k2)
            for (int c = 0; c < 2; ++c)
                if (fabs(X[(k1 * NB + k2) * 2 + c] - full[(k1 * N + k2) * 2 + c]) > 1e-12) ok = 0;
    expect(ok, "2-D transform equals the O(n^4) definition");
    free(x);
}

static void convolution_theorem(void) {
    /* fprop = crop(IDFT(DFT(x) . conj(DFT(w)))), summed over input planes, on a ragged shape */
    enum { F = 2, H = 7, W = 5, KH = 3, KW = 2, N = 8, NB = N / 2 + 1, OH = H - KH + 1, OW = W - KW + 1 };
    double *x = randoms(F * H * W), *w = randoms(F * KH * KW), y[OH * OW];
    oracle_conv_fprop(x, w, y, 1, F, 1, H, W, KH, KW, NULL, 0);
    double XF[F * N * NB * 2], WF[F * N * NB * 2], YF[N * NB * 2], back[OH * OW];
    oracle_dft_r2c_2d(x, XF, F, H, W, N);
    oracle_dft_r2c_2d(w, WF, F, KH, KW, N);
    memset(YF, 0, sizeof YF);
    for (int i = 0; i < F; ++i)
        for (int b = 0; b < N * NB; ++b) {
            const double xr = XF[(i * N * NB + b) * 2], xi = XF[(i * N * NB + b) * 2 + 1];
            const double wr = WF[(i * N * NB + b) * 2], wi = WF[(i * N * NB + b) * 2 + 1];
            YF[2 * b] += xr * wr + xi * wi;
            YF[2 * b + 1] += xi * wr - xr * wi;
        }
    oracle_idft_c2r_2d(YF, back, 1, N, OH, OW);
    expect(maxdiff(y, back, OH * OW) < 1e-12, "convolution theorem: fprop through the transforms");
    free(x); free(w);
}

int main(void) {
    hand_example();
    impulses();
    selections();
    transforms();
    convolution_theorem();
    printf(bad ? "%d checks FAILED\n" : "all checks passed\n", bad);
    return bad ? 1 : 0;
}
