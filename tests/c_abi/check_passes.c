/*
 * Plain-C caller of the library's ABI: no Python, no PyTorch.  Allocates device memory with the
 * HIP runtime, runs the three passes (ordinary and zero-padded), a tiled fprop and a 1-D
 * transform through include/fftconv.h, and compares every result with the fp64 oracle
 * (oracle/oracle.c, linked in: this program is test infrastructure).  Prints one line per
 * check and exits 0 only if every max|err| / max|ref| is within its bound (1e-4 for the
 * convolutions, 1e-5 for the transform).
 */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "fftconv.h"

void oracle_conv_fprop(const double *x, const double *w, double *y, int S, int f, int fo, int h, int wd,
                       int kh, int kw, const long *sel, long nsel);
void oracle_conv_bprop(const double *gy, const double *w, double *gx, int S, int f, int fo, int h, int wd,
                       int kh, int kw, const long *sel, long nsel);
void oracle_conv_accgrad(const double *x, const double *gy, double *gw, int S, int f, int fo, int h, int wd,
                         int kh, int kw, const long *sel, long nsel);
void oracle_dft_r2c_1d(const double *in, double *out, long B, int n_in, int n);

#define HIP_OK(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { \
    fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_)); exit(2); } } while (0)
#define FC_OK(call) do { int s_ = (call); if (s_ != FFTCONV_OK) { \
    fprintf(stderr, "%s: %s\n", #call, fftconv_status_string(s_)); exit(2); } } while (0)

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static float uniform_pm1(void) {          /* xorshift64*, values in [-1, 1) with 24 random bits */
    rng_state ^= rng_state >> 12; rng_state ^= rng_state << 25; rng_state ^= rng_state >> 27;
    return (float)((rng_state * 0x2545F4914F6CDD1Dull) >> 40) * (2.0f / 16777216.0f) - 1.0f;
}

static float *host_random(size_t n) {
    float *p = (float *)malloc(n * sizeof(float));
    for (size_t i = 0; i < n; ++i) p[i] = uniform_pm1();
    return p;
}
static double *widen(const float *p, size_t n) {
    double *d = (double *)malloc(n * sizeof(double));
    for (size_t i = 0; i < n; ++i) d[i] = p[i];
    return d;
}
static float *to_device(const float *h, size_t n) {
    float *d;
    HIP_OK(hipMalloc((void **)&d, n * sizeof(float)));
    HIP_OK(hipMemcpy(d, h, n * sizeof(float), hipMemcpyHostToDevice));
    return d;
}
static int check(const char *what, const float *dev, const double *ref, size_t n, double tol) {
    float *got = (float *)malloc(n * sizeof(float));
    HIP_OK(hipDeviceSynchronize());
    HIP_OK(hipMemcpy(got, dev, n * sizeof(float), hipMemcpyDeviceToHost));
    double err = 0, mx = 0;
    for (size_t i = 0; i < n; ++i) {
        const double e = fabs((double)got[i] - ref[i]);
        if (e > err) err = e;
        if (fabs(ref[i]) > mx) mx = fabs(ref[i]);
    }
    free(got);
    const double rel = err / mx;
    printf("%-28s max|err|/max|ref| = %.3e  %s\n", what, rel, rel <= tol ? "ok" : "FAIL");
    return rel <= tol ? 0 : 1;
}

/* `check_passes --time`: microseconds per fprop of the smallest benchmark layer (S = f = f' = 16,
 * 13x13, 3x3) driven from C, where no interpreter stands between two launches: the ordinary call,
 * the call on weights transformed ahead, and the one-launch kernel. */
static int time_small_layer(fftconv_handle hd) {
    const int S = 16, f = 16, fo = 16, h = 13, w = 13, k = 3, o = h - k + 1, reps = 2000;
    const size_t nx = (size_t)S * f * h * w, nw = (size_t)fo * f * k * k, ny = (size_t)S * fo * o * o;
    float *x = host_random(nx), *wt = host_random(nw);
    float *dx = to_device(x, nx), *dw = to_device(wt, nw), *dy;
    void *ws, *wf;
    const size_t wsb = fftconv_workspace_bytes(FFTCONV_FPROP, S, f, fo, h, w, k, k);
    const size_t wfb = fftconv_weights_bytes(f, fo, h, w, k, k, 0, 0);
    HIP_OK(hipMalloc((void **)&dy, ny * sizeof(float)));
    HIP_OK(hipMalloc(&ws, wsb));
    HIP_OK(hipMalloc(&wf, wfb));
    FC_OK(fft_conv_transform_weights(hd, dw, wf, wfb, f, fo, h, w, k, k, 0, 0));
    hipEvent_t e0, e1;
    HIP_OK(hipEventCreate(&e0)); HIP_OK(hipEventCreate(&e1));
    for (int variant = 0; variant < 3; ++variant) {
        float ms = 0;
        for (int r = -50; r < reps; ++r) {          /* 50 untimed calls first */
            if (r == 0) HIP_OK(hipEventRecord(e0, 0));
            if (variant == 0) FC_OK(fft_conv_fprop(hd, dx, dw, dy, S, f, fo, h, w, k, k, ws, wsb));
            else if (variant == 1) FC_OK(fft_conv_fprop_weights(hd, dx, wf, wfb, dy, S, f, fo, h, w, k, k, 0, 0, ws, wsb));
            else FC_OK(fft_conv_fprop_fused(hd, dx, wf, wfb, dy, S, f, fo, h, w, k, k));
        }
        HIP_OK(hipEventRecord(e1, 0));
        HIP_OK(hipEventSynchronize(e1));
        HIP_OK(hipEventElapsedTime(&ms, e0, e1));
        printf("%-34s %.2f us per call\n", variant == 0 ? "fft_conv_fprop" : variant == 1 ? "fft_conv_fprop_weights" : "fft_conv_fprop_fused",
               ms * 1e3 / reps);
    }
    return 0;
}

int main(int argc, char **argv) {
    int bad = 0;
    fftconv_handle hd;
    FC_OK(fftconv_create(&hd, 0));
    if (argc > 1 && strcmp(argv[1], "--time") == 0) return time_small_layer(hd);

    /* ---- one layer, three passes, ordinary and through a forced tile basis */
    const int S = 3, f = 5, fo = 4, h = 21, w = 18, kh = 3, kw = 5, oh = h - kh + 1, ow = w - kw + 1;
    const size_t nx = (size_t)S * f * h * w, nw = (size_t)fo * f * kh * kw, ny = (size_t)S * fo * oh * ow;
    float *x = host_random(nx), *wt = host_random(nw), *gy = host_random(ny);
    double *xd = widen(x, nx), *wd = widen(wt, nw), *gyd = widen(gy, ny);
    double *ry = (double *)malloc(ny * sizeof(double)), *rgx = (double *)malloc(nx * sizeof(double)),
           *rgw = (double *)malloc(nw * sizeof(double));
    oracle_conv_fprop(xd, wd, ry, S, f, fo, h, w, kh, kw, NULL, 0);
    oracle_conv_bprop(gyd, wd, rgx, S, f, fo, h, w, kh, kw, NULL, 0);
    oracle_conv_accgrad(xd, gyd, rgw, S, f, fo, h, w, kh, kw, NULL, 0);
    float *dx = to_device(x, nx), *dw = to_device(wt, nw), *dgy = to_device(gy, ny);
    float *dy, *dgx, *dgw;
    HIP_OK(hipMalloc((void **)&dy, ny * sizeof(float)));
    HIP_OK(hipMalloc((void **)&dgx, nx * sizeof(float)));
    HIP_OK(hipMalloc((void **)&dgw, nw * sizeof(float)));
    FC_OK(fft_conv_fprop(hd, dx, dw, dy, S, f, fo, h, w, kh, kw, NULL, 0));
    bad += check("fft_conv_fprop", dy, ry, ny, 1e-4);
    FC_OK(fft_conv_bprop(hd, dgy, dw, dgx, S, f, fo, h, w, kh, kw, NULL, 0));
    bad += check("fft_conv_bprop", dgx, rgx, nx, 1e-4);
    FC_OK(fft_conv_accgrad(hd, dx, dgy, dgw, S, f, fo, h, w, kh, kw, 1.0f, 0, NULL, 0));
    bad += check("fft_conv_accgrad", dgw, rgw, nw, 1e-4);
    HIP_OK(hipMemset(dy, 0, ny * sizeof(float)));
    {   /* caller-supplied workspace of exactly the advertised size */
        const size_t need = fftconv_tiled_workspace_bytes(FFTCONV_FPROP, S, f, fo, h, w, kh, kw, 8);
        void *ws;
        HIP_OK(hipMalloc(&ws, need));
        FC_OK(fft_conv_fprop_tiled(hd, dx, dw, dy, S, f, fo, h, w, kh, kw, 8, ws, need));
        bad += check("fft_conv_fprop_tiled (n=8)", dy, ry, ny, 1e-4);
        if (fft_conv_fprop_tiled(hd, dx, dw, dy, S, f, fo, h, w, kh, kw, 8, ws, need - 256) !=
            FFTCONV_WORKSPACE_TOO_SMALL) { printf("short workspace not rejected  FAIL\n"); ++bad; }
        HIP_OK(hipFree(ws));
    }
    {   /* transform reuse: fprop_save + backward */
        const size_t sb = fftconv_saved_bytes(S, f, fo, h, w, kh, kw);
        void *saved;
        HIP_OK(hipMalloc(&saved, sb));
        FC_OK(fft_conv_fprop_save(hd, dx, dw, dy, S, f, fo, h, w, kh, kw, saved, sb, NULL, 0));
        FC_OK(fft_conv_backward(hd, dgy, dgx, dgw, S, f, fo, h, w, kh, kw, 1.0f, 0, saved, sb, NULL, 0));
        bad += check("fft_conv_fprop_save", dy, ry, ny, 1e-4);
        bad += check("fft_conv_backward gx", dgx, rgx, nx, 1e-4);
        bad += check("fft_conv_backward gw", dgw, rgw, nw, 1e-4);
        HIP_OK(hipFree(saved));
    }

    /* ---- the same layer with a zero border of (2, 1): oracle on an explicitly padded copy */
    {
        const int ph = 2, pw = 1, hp = h + 2 * ph, wp = w + 2 * pw, ohp = hp - kh + 1, owp = wp - kw + 1;
        const size_t nxp = (size_t)S * f * hp * wp, nyp = (size_t)S * fo * ohp * owp;
        double *xp = (double *)calloc(nxp, sizeof(double)), *ryp = (double *)malloc(nyp * sizeof(double));
        for (int p = 0; p < S * f; ++p)
            for (int r = 0; r < h; ++r)
                for (int c = 0; c < w; ++c)
                    xp[((size_t)p * hp + r + ph) * wp + c + pw] = xd[((size_t)p * h + r) * w + c];
        oracle_conv_fprop(xp, wd, ryp, S, f, fo, hp, wp, kh, kw, NULL, 0);
        float *dyp;
        HIP_OK(hipMalloc((void **)&dyp, nyp * sizeof(float)));
        FC_OK(fft_conv_fprop_padded(hd, dx, dw, dyp, S, f, fo, h, w, kh, kw, ph, pw, NULL, 0));
        bad += check("fft_conv_fprop_padded (2,1)", dyp, ryp, nyp, 1e-4);
        HIP_OK(hipFree(dyp));
        free(xp); free(ryp);
    }

    /* ---- which basis the layer above ran on: 21 x 18 calls for a rectangular 24 x 18 */
    {
        int nr = 0, nc = 0;
        const int tiled = fftconv_layer_basis(h, w, kh, kw, 0, 0, &nr, &nc);
        if (tiled != 0 || nr != 24 || nc != 18) { printf("layer basis %d x %d (tiled %d)  FAIL\n", nr, nc, tiled); ++bad; }
    }

    /* ---- a small layer on weights transformed ahead: fprop and bprop as one launch each */
    {
        const int S2 = 2, f2 = 8, fo2 = 8, h2 = 13, k2 = 3, o2 = h2 - k2 + 1;
        const size_t nx2 = (size_t)S2 * f2 * h2 * h2, nw2 = (size_t)fo2 * f2 * k2 * k2, ny2 = (size_t)S2 * fo2 * o2 * o2;
        float *x2 = host_random(nx2), *w2 = host_random(nw2), *g2 = host_random(ny2);
        double *x2d = widen(x2, nx2), *w2d = widen(w2, nw2), *g2d = widen(g2, ny2);
        double *ry2 = (double *)malloc(ny2 * sizeof(double)), *rgx2 = (double *)malloc(nx2 * sizeof(double));
        oracle_conv_fprop(x2d, w2d, ry2, S2, f2, fo2, h2, h2, k2, k2, NULL, 0);
        oracle_conv_bprop(g2d, w2d, rgx2, S2, f2, fo2, h2, h2, k2, k2, NULL, 0);
        float *dx2 = to_device(x2, nx2), *dw2 = to_device(w2, nw2), *dg2 = to_device(g2, ny2), *dy2, *dgx2;
        HIP_OK(hipMalloc((void **)&dy2, ny2 * sizeof(float)));
        HIP_OK(hipMalloc((void **)&dgx2, nx2 * sizeof(float)));
        const size_t wb = fftconv_weights_bytes(f2, fo2, h2, h2, k2, k2, 0, 0);
        void *wf;
        HIP_OK(hipMalloc(&wf, wb));
        FC_OK(fft_conv_transform_weights(hd, dw2, wf, wb, f2, fo2, h2, h2, k2, k2, 0, 0));
        FC_OK(fft_conv_fprop_fused(hd, dx2, wf, wb, dy2, S2, f2, fo2, h2, h2, k2, k2));
        bad += check("fft_conv_fprop_fused", dy2, ry2, ny2, 1e-4);
        FC_OK(fft_conv_bprop_fused(hd, dg2, wf, wb, dgx2, S2, f2, fo2, h2, h2, k2, k2));
        bad += check("fft_conv_bprop_fused", dgx2, rgx2, nx2, 1e-4);
        /* accGrad of the same layer as one launch (needs no weights: it reduces over the samples) */
        {
            double *rgw2 = (double *)malloc(nw2 * sizeof(double));
            oracle_conv_accgrad(x2d, g2d, rgw2, S2, f2, fo2, h2, h2, k2, k2, NULL, 0);
            float *dgw2;
            HIP_OK(hipMalloc((void **)&dgw2, nw2 * sizeof(float)));
            FC_OK(fft_conv_accgrad_fused(hd, dx2, dg2, dgw2, S2, f2, fo2, h2, h2, k2, k2, 1.0f, 0));
            bad += check("fft_conv_accgrad_fused", dgw2, rgw2, nw2, 1e-4);
            HIP_OK(hipFree(dgw2));
            free(rgw2);
        }
        HIP_OK(hipFree(dx2)); HIP_OK(hipFree(dw2)); HIP_OK(hipFree(dg2)); HIP_OK(hipFree(dy2)); HIP_OK(hipFree(dgx2));
        HIP_OK(hipFree(wf));
        free(x2); free(w2); free(g2); free(x2d); free(w2d); free(g2d); free(ry2); free(rgx2);
    }

    /* ---- a batch of 1-D transforms: 1000 signals of 61 samples, n = 64 */
    {
        const long B = 1000; const int n_in = 61, n = 64, nb = n / 2 + 1;
        float *s = host_random((size_t)B * n_in);
        double *sd = widen(s, (size_t)B * n_in), *rX = (double *)malloc((size_t)B * nb * 2 * sizeof(double));
        oracle_dft_r2c_1d(sd, rX, B, n_in, n);
        float *ds = to_device(s, (size_t)B * n_in), *dX;
        HIP_OK(hipMalloc((void **)&dX, (size_t)B * nb * 2 * sizeof(float)));
        FC_OK(fft_r2c_1d(hd, ds, dX, B, n_in, n));
        bad += check("fft_r2c_1d (n=64)", dX, rX, (size_t)B * nb * 2, 1e-5);
        HIP_OK(hipFree(ds)); HIP_OK(hipFree(dX));
        free(s); free(sd); free(rX);
    }

    /* ---- argument errors come back as statuses, nothing is launched */
    if (fft_conv_fprop(hd, dx, dw, dy, S, f, fo, 2, 2, kh, kw, NULL, 0) != FFTCONV_INVALID_ARG) { printf("bad shape accepted  FAIL\n"); ++bad; }
    if (fft_r2c_1d(hd, dx, dy, 1, 8, 44) != FFTCONV_UNSUPPORTED) { printf("bad size accepted  FAIL\n"); ++bad; }

    FC_OK(fftconv_destroy(hd));
    printf(bad ? "FAILED (%d)\n" : "all checks passed\n", bad);
    return bad ? 1 : 0;
}
