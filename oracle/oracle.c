/*
 * CPU oracle for frequency-domain convolution (fbfft paper, arXiv 1412.7580).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP path is checked against.  It shares no code, header, table or helper
 * with the HIP library and must never be called from the product path; only
 * the tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * Everything is fp64.  Tensors are dense row-major "BDHW" (Section 3.1):
 *   input       x [S][f ][h ][w ]
 *   weight      w [f'][f][kh][kw]
 *   output      y [S][f'][oh][ow],  oh = h-kh+1, ow = w-kw+1  (valid-only, Section 2)
 * Each function optionally takes a list of output planes to compute, so that
 * a sample of a large problem can be evaluated; sel == NULL means all planes,
 * and results are then written densely in plane order.  With a selection the
 * r-th selected plane is written at out + r*plane_size.
 *
 * Pins (tests/test_oracle_*.py): hand-worked example, brute force in a second
 * language, impulse responses, 1x1 kernels against a matrix product, the
 * adjoint identity tying the three passes together, finite differences,
 * library correlation/convolution, closed-form DFTs, Parseval, shift theorem,
 * a non-separable O(n^4) 2-D DFT, and the convolution theorem connecting the
 * direct passes with the DFT functions.
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

#ifndef M_PI
#define M_PI 3.14159265358979323846264338327950288
#endif

/* ---------------------------------------------------------------------- */
/* Time-domain passes (Section 2, the three displayed equations)          */
/* ---------------------------------------------------------------------- */

/* fprop: y(s,j) = sum_i x(s,i) (star) w(j,i)   -- valid cross-correlation,
 * y[s,j,a,b] = sum_{i,u,v} x[s,i,a+u,b+v] * w[j,i,u,v].                   */
void oracle_conv_fprop(const double *x, const double *w, double *y,
                       int S, int f, int fo, int h, int wd, int kh, int kw,
                       const long *sel, long nsel)
{
    const int oh = h - kh + 1, ow = wd - kw + 1;
    const long nplanes = sel ? nsel : (long)S * fo;
#pragma omp parallel for schedule(dynamic, 1)
    for (long r = 0; r < nplanes; ++r) {
        const long pl = sel ? sel[r] : r;
        const int s = (int)(pl / fo), j = (int)(pl % fo);
        double *yp = y + r * (long)oh * ow;
        for (long t = 0; t < (long)oh * ow; ++t) yp[t] = 0.0;
        for (int i = 0; i < f; ++i) {
            const double *xp = x + ((long)s * f + i) * h * wd;
            const double *wp = w + ((long)j * f + i) * kh * kw;
            for (int u = 0; u < kh; ++u)
                for (int v = 0; v < kw; ++v) {
                    const double c = wp[u * kw + v];
                    for (int a = 0; a < oh; ++a)
                        for (int b = 0; b < ow; ++b)
                            yp[a * ow + b] += xp[(a + u) * wd + (b + v)] * c;
                }
        }
    }
}

/* bprop: dL/dx(s,i) = sum_j dL/dy(s,j) * w(j,i)  -- true (full) convolution,
 * gx[s,i,p,q] = sum_{j,u,v} gy[s,j,p-u,q-v] * w[j,i,u,v], out-of-range gy = 0. */
void oracle_conv_bprop(const double *gy, const double *w, double *gx,
                       int S, int f, int fo, int h, int wd, int kh, int kw,
                       const long *sel, long nsel)
{
    const int oh = h - kh + 1, ow = wd - kw + 1;
    const long nplanes = sel ? nsel : (long)S * f;
#pragma omp parallel for schedule(dynamic, 1)
    for (long r = 0; r < nplanes; ++r) {
        const long pl = sel ? sel[r] : r;
        const int s = (int)(pl / f), i = (int)(pl % f);
        double *gp = gx + r * (long)h * wd;
        for (long t = 0; t < (long)h * wd; ++t) gp[t] = 0.0;
        for (int j = 0; j < fo; ++j) {
            const double *gyp = gy + ((long)s * fo + j) * oh * ow;
            const double *wp = w + ((long)j * f + i) * kh * kw;
            for (int u = 0; u < kh; ++u)
                for (int v = 0; v < kw; ++v) {
                    const double c = wp[u * kw + v];
                    /* p-u = a in [0,oh), q-v = b in [0,ow) */
                    for (int a = 0; a < oh; ++a)
                        for (int b = 0; b < ow; ++b)
                            gp[(a + u) * wd + (b + v)] += gyp[a * ow + b] * c;
                }
        }
    }
}

/* accGrad: dL/dw(j,i) = sum_s dL/dy(s,j) (star) x(s,i); the index form is the
 * one the tiling discussion of Section 6 writes out (sum_i x_{j+i} z_i):
 * gw[j,i,u,v] = sum_{s,a,b} gy[s,j,a,b] * x[s,i,a+u,b+v].                  */
void oracle_conv_accgrad(const double *x, const double *gy, double *gw,
                         int S, int f, int fo, int h, int wd, int kh, int kw,
                         const long *sel, long nsel)
{
    const int oh = h - kh + 1, ow = wd - kw + 1;
    const long nplanes = sel ? nsel : (long)fo * f;
#pragma omp parallel for schedule(dynamic, 1)
    for (long r = 0; r < nplanes; ++r) {
        const long pl = sel ? sel[r] : r;
        const int j = (int)(pl / f), i = (int)(pl % f);
        double *gp = gw + r * (long)kh * kw;
        for (int u = 0; u < kh; ++u)
            for (int v = 0; v < kw; ++v) {
                double acc = 0.0;
                for (int s = 0; s < S; ++s) {
                    const double *xp = x + ((long)s * f + i) * h * wd;
                    const double *gyp = gy + ((long)s * fo + j) * oh * ow;
                    for (int a = 0; a < oh; ++a)
                        for (int b = 0; b < ow; ++b)
                            acc += gyp[a * ow + b] * xp[(a + u) * wd + (b + v)];
                }
                gp[u * kw + v] = acc;
            }
    }
}

/* ---------------------------------------------------------------------- */
/* Naive DFT (Supplement, "Decimation in Time vs Frequency", first        */
/* display): X_k = sum_j x_j exp(-2 pi i j k / n).  O(n^2) per line.      */
/* ---------------------------------------------------------------------- */

/* exp(sign * 2 pi i * (m mod n) / n); the argument is reduced in integers
 * first so that cos/sin only ever see angles in [0, 2 pi).               */
static void root_of_unity(long m, int n, int sign, double *re, double *im)
{
    long r = m % n;
    if (r < 0) r += n;
    const double ang = 2.0 * M_PI * (double)r / (double)n;
    *re = cos(ang);
    *im = sign * sin(ang);
}

/* 1-D real-to-complex: in [B][n_in] (zero-padded to n), out [B][n/2+1][2]. */
void oracle_dft_r2c_1d(const double *in, double *out, long B, int n_in, int n)
{
    const int nb = n / 2 + 1;
#pragma omp parallel for schedule(static)
    for (long t = 0; t < B; ++t) {
        const double *x = in + t * n_in;
        double *X = out + t * nb * 2;
        for (int k = 0; k < nb; ++k) {
            double ar = 0.0, ai = 0.0;
            for (int j = 0; j < n_in; ++j) {
                double c, s;
                root_of_unity((long)j * k, n, -1, &c, &s);
                ar += x[j] * c;
                ai += x[j] * s;
            }
            X[2 * k] = ar;
            X[2 * k + 1] = ai;
        }
    }
}

/* 1-D complex-to-real inverse: in [B][n/2+1][2] (Hermitian half), out
 * [B][n_out] = first n_out samples of (1/n) sum_k Xfull_k exp(+2 pi i j k/n).
 * Xfull_{n-k} = conj(X_k); only the real part of the sum is kept (imaginary
 * parts of the self-conjugate bins 0 and n/2 therefore do not matter).   */
void oracle_idft_c2r_1d(const double *in, double *out, long B, int n, int n_out)
{
    const int nb = n / 2 + 1;
#pragma omp parallel for schedule(static)
    for (long t = 0; t < B; ++t) {
        const double *X = in + t * nb * 2;
        double *x = out + t * n_out;
        for (int j = 0; j < n_out; ++j) {
            double acc = 0.0;
            for (int k = 0; k < n; ++k) {
                double xr, xi, c, s;
                if (k < nb) { xr = X[2 * k]; xi = X[2 * k + 1]; }
                else        { xr = X[2 * (n - k)]; xi = -X[2 * (n - k) + 1]; }
                root_of_unity((long)j * k, n, +1, &c, &s);
                acc += xr * c - xi * s;          /* Re{(xr+i xi)(c+i s)} */
            }
            x[j] = acc / n;
        }
    }
}

/* 2-D real-to-complex: in [B][h_in][w_in] zero-padded to n x n,
 * out [B][n][n/2+1][2]; Hermitian half kept along the innermost (w) axis,
 * the layout of the frequency tensors in Table 1.  Separable: 1-D DFT along
 * w keeping n/2+1 bins, then a full-length 1-D DFT along h.              */
void oracle_dft_r2c_2d(const double *in, double *out, long B, int h_in, int w_in, int n)
{
    const int nb = n / 2 + 1;
#pragma omp parallel
    {
        double *row = (double *)malloc(sizeof(double) * (size_t)h_in * nb * 2);
#pragma omp for schedule(static)
        for (long t = 0; t < B; ++t) {
            const double *x = in + t * (long)h_in * w_in;
            double *X = out + t * (long)n * nb * 2;
            for (int a = 0; a < h_in; ++a)
                for (int k2 = 0; k2 < nb; ++k2) {
                    double ar = 0.0, ai = 0.0;
                    for (int b = 0; b < w_in; ++b) {
                        double c, s;
                        root_of_unity((long)b * k2, n, -1, &c, &s);
                        ar += x[a * w_in + b] * c;
                        ai += x[a * w_in + b] * s;
                    }
                    row[(a * nb + k2) * 2] = ar;
                    row[(a * nb + k2) * 2 + 1] = ai;
                }
            for (int k1 = 0; k1 < n; ++k1)
                for (int k2 = 0; k2 < nb; ++k2) {
                    double ar = 0.0, ai = 0.0;
                    for (int a = 0; a < h_in; ++a) {
                        double c, s;
                        root_of_unity((long)a * k1, n, -1, &c, &s);
                        const double rr = row[(a * nb + k2) * 2], ri = row[(a * nb + k2) * 2 + 1];
                        ar += rr * c - ri * s;
                        ai += rr * s + ri * c;
                    }
                    X[(k1 * nb + k2) * 2] = ar;
                    X[(k1 * nb + k2) * 2 + 1] = ai;
                }
        }
        free(row);
    }
}

/* 2-D complex-to-real inverse with crop: in [B][n][n/2+1][2], out
 * [B][h_out][w_out] = top-left corner of the real n x n inverse, scaled by
 * 1/n^2 (the clipping step that ends each pass in Section 3.1).          */
void oracle_idft_c2r_2d(const double *in, double *out, long B, int n, int h_out, int w_out)
{
    const int nb = n / 2 + 1;
#pragma omp parallel
    {
        /* col[a][k2] = sum_k1 X[k1][k2] exp(+2 pi i a k1 / n) for a < h_out */
        double *col = (double *)malloc(sizeof(double) * (size_t)h_out * nb * 2);
#pragma omp for schedule(static)
        for (long t = 0; t < B; ++t) {
            const double *X = in + t * (long)n * nb * 2;
            double *x = out + t * (long)h_out * w_out;
            for (int a = 0; a < h_out; ++a)
                for (int k2 = 0; k2 < nb; ++k2) {
                    double ar = 0.0, ai = 0.0;
                    for (int k1 = 0; k1 < n; ++k1) {
                        double c, s;
                        root_of_unity((long)a * k1, n, +1, &c, &s);
                        const double xr = X[(k1 * nb + k2) * 2], xi = X[(k1 * nb + k2) * 2 + 1];
                        ar += xr * c - xi * s;
                        ai += xr * s + xi * c;
                    }
                    col[(a * nb + k2) * 2] = ar;
                    col[(a * nb + k2) * 2 + 1] = ai;
                }
            for (int a = 0; a < h_out; ++a)
                for (int b = 0; b < w_out; ++b) {
                    double acc = 0.0;
                    for (int k2 = 0; k2 < n; ++k2) {
                        double xr, xi, c, s;
                        if (k2 < nb) { xr = col[(a * nb + k2) * 2]; xi = col[(a * nb + k2) * 2 + 1]; }
                        else { xr = col[(a * nb + (n - k2)) * 2]; xi = -col[(a * nb + (n - k2)) * 2 + 1]; }
                        root_of_unity((long)b * k2, n, +1, &c, &s);
                        acc += xr * c - xi * s;
                    }
                    x[a * w_out + b] = acc / ((double)n * n);
                }
        }
        free(col);
    }
}

/* Full complex 2-D DFT of one real n x n array by the non-separable
 * four-index definition, O(n^4): used only to pin oracle_dft_r2c_2d.     */
void oracle_dft2_bruteforce(const double *in, double *out, int n)
{
    for (int k1 = 0; k1 < n; ++k1)
        for (int k2 = 0; k2 < n; ++k2) {
            double ar = 0.0, ai = 0.0;
            for (int a = 0; a < n; ++a)
                for (int b = 0; b < n; ++b) {
                    double c, s;
                    root_of_unity((long)a * k1 + (long)b * k2, n, -1, &c, &s);
                    ar += in[a * n + b] * c;
                    ai += in[a * n + b] * s;
                }
            out[(k1 * n + k2) * 2] = ar;
            out[(k1 * n + k2) * 2 + 1] = ai;
        }
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    n = omp_get_max_threads();
#endif
    return n;
}
