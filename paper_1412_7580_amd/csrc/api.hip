// C ABI of the library (include/fftconv.h): argument checks, workspace, and the three pass
// pipelines of Table 1 of the fbfft paper expressed as four launches on one stream:
//   FFT2D(operand A) -> FFT2D(operand B) -> per-bin complex contraction -> IFFT2D + clip.
// The frequency-domain forms used for the two passes the paper leaves as "similar"
// (Section 2) follow from the DFT shift property:
//   fprop   Y  = sum_i  X_si  . conj(W_ji)
//   bprop   GX = sum_j  GY_sj . W_ji
//   accGrad GW = sum_s  conj(GY_sj) . X_si
// each followed by the inverse transform and a crop at the origin.
#include "../../include/fftconv.h"
#include "kernels.hpp"

#include <new>

using namespace fc;

struct fftconv_ctx {
    int device;
    hipStream_t stream;
    void *ws;
    size_t ws_bytes;
    int profiling;
    hipEvent_t ev[8];   // start/stop pair per stage
    int ev_valid;
    char last_hip_error[256];
};

static int basis_size(int h, int w) {
    int m = h > w ? h : w, n = 8;
    while (n < m) n <<= 1;
    return n;
}

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct PassPlan {
    int N, bins;
    long planesA, planesB, planesC;
    int hA, wA, hB, wB, hC, wC;
    bool conjA, conjB;
    int M, Nn, K;
    long a_rs, a_cs, b_rs, b_cs, c_rs, c_cs;
    FreqLayout lay;
    size_t offA, offB, offC, total;
};

static int make_plan(int pass, int S, int f, int fo, int h, int w, int kh, int kw, PassPlan *p) {
    if (S <= 0 || f <= 0 || fo <= 0 || h <= 0 || w <= 0 || kh <= 0 || kw <= 0) return FFTCONV_INVALID_ARG;
    if (kh > h || kw > w) return FFTCONV_INVALID_ARG;
    if (pass < 0 || pass > 2) return FFTCONV_INVALID_ARG;
    const int N = basis_size(h, w);
    if (N > 128) return FFTCONV_UNSUPPORTED;
    const int oh = h - kh + 1, ow = w - kw + 1;
    p->N = N;
    p->bins = N * (N / 2 + 1);
    p->lay.tsh = fft2d_tile_log2(N);
    p->lay.bins = p->bins;
    p->conjA = p->conjB = false;
    switch (pass) {
        case FFTCONV_FPROP:
            p->planesA = (long)S * f;  p->hA = h;  p->wA = w;
            p->planesB = (long)fo * f; p->hB = kh; p->wB = kw; p->conjB = true;
            p->planesC = (long)S * fo; p->hC = oh; p->wC = ow;
            p->M = S; p->Nn = fo; p->K = f;
            p->a_rs = f;  p->a_cs = 1;     // A(s,i) = XF[s][i]
            p->b_rs = 1;  p->b_cs = f;     // B(i,j) = conj WF[j][i]
            p->c_rs = fo; p->c_cs = 1;     // C(s,j) = YF[s][j]
            break;
        case FFTCONV_BPROP:
            p->planesA = (long)S * fo; p->hA = oh; p->wA = ow;
            p->planesB = (long)fo * f; p->hB = kh; p->wB = kw;
            p->planesC = (long)S * f;  p->hC = h;  p->wC = w;
            p->M = S; p->Nn = f; p->K = fo;
            p->a_rs = fo; p->a_cs = 1;     // A(s,j) = GYF[s][j]
            p->b_rs = f;  p->b_cs = 1;     // B(j,i) = WF[j][i]
            p->c_rs = f;  p->c_cs = 1;     // C(s,i) = GXF[s][i]
            break;
        default:
            p->planesA = (long)S * fo; p->hA = oh; p->wA = ow; p->conjA = true;
            p->planesB = (long)S * f;  p->hB = h;  p->wB = w;
            p->planesC = (long)fo * f; p->hC = kh; p->wC = kw;
            p->M = fo; p->Nn = f; p->K = S;
            p->a_rs = 1;  p->a_cs = fo;    // A(j,s) = conj GYF[s][j]
            p->b_rs = f;  p->b_cs = 1;     // B(s,i) = XF[s][i]
            p->c_rs = f;  p->c_cs = 1;     // C(j,i) = GWF[j][i]
            break;
    }
    p->offA = 0;
    p->offB = align_up(p->offA + p->lay.floats(p->planesA) * sizeof(float), 256);
    p->offC = align_up(p->offB + p->lay.floats(p->planesB) * sizeof(float), 256);
    p->total = align_up(p->offC + p->lay.floats(p->planesC) * sizeof(float), 256);
    return FFTCONV_OK;
}

static int hip_fail(fftconv_ctx *c, hipError_t e) {
    if (c) snprintf(c->last_hip_error, sizeof(c->last_hip_error), "HIP error: %s", hipGetErrorString(e));
    return FFTCONV_HIP_ERROR;
}

static int run_pass(fftconv_ctx *c, int pass, const float *opA, const float *opB, float *out,
                    int S, int f, int fo, int h, int w, int kh, int kw, float scale, int accumulate,
                    void *ws, size_t ws_bytes) {
    if (!c || !opA || !opB || !out) return FFTCONV_INVALID_ARG;
    PassPlan p;
    int rc = make_plan(pass, S, f, fo, h, w, kh, kw, &p);
    if (rc != FFTCONV_OK) return rc;
    hipError_t e;
    if (ws) {
        if (ws_bytes < p.total) return FFTCONV_WORKSPACE_TOO_SMALL;
    } else {
        if (c->ws_bytes < p.total) {
            if (c->ws) {
                if ((e = hipStreamSynchronize(c->stream)) != hipSuccess) return hip_fail(c, e);
                (void)hipFree(c->ws);
                c->ws = nullptr; c->ws_bytes = 0;
            }
            if ((e = hipMalloc(&c->ws, p.total)) != hipSuccess) return hip_fail(c, e);
            c->ws_bytes = p.total;
        }
        ws = c->ws;
    }
    float *AF = reinterpret_cast<float *>(static_cast<char *>(ws) + p.offA);
    float *BF = reinterpret_cast<float *>(static_cast<char *>(ws) + p.offB);
    float *CF = reinterpret_cast<float *>(static_cast<char *>(ws) + p.offC);
    const bool prof = c->profiling != 0;
    c->ev_valid = 0;
    auto ctx = [&](int stage) {
        return prof ? LaunchCtx{c->stream, c->ev[2 * stage], c->ev[2 * stage + 1]}
                    : LaunchCtx{c->stream, nullptr, nullptr};
    };

    if ((e = launch_fft2d_r2c(opA, AF, p.planesA, p.hA, p.wA, p.N, true, p.conjA, ctx(0))) != hipSuccess) return hip_fail(c, e);
    if ((e = launch_fft2d_r2c(opB, BF, p.planesB, p.hB, p.wB, p.N, true, p.conjB, ctx(1))) != hipSuccess) return hip_fail(c, e);
    GemmOperand ga{AF, p.lay, p.a_rs, p.a_cs}, gb{BF, p.lay, p.b_rs, p.b_cs};
    if ((e = launch_cgemm_bins(ga, gb, CF, p.lay, p.c_rs, p.c_cs, p.M, p.Nn, p.K, p.bins, ctx(2))) != hipSuccess) return hip_fail(c, e);
    const float s = scale / ((float)p.N * (float)p.N);
    if ((e = launch_fft2d_c2r(CF, out, p.planesC, p.N, p.hC, p.wC, true, s, accumulate != 0, ctx(3))) != hipSuccess) return hip_fail(c, e);
    if (prof) c->ev_valid = 1;
    return FFTCONV_OK;
}

extern "C" {

int fftconv_create(fftconv_handle *out, int device) {
    if (!out) return FFTCONV_INVALID_ARG;
    *out = nullptr;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) return FFTCONV_HIP_ERROR;
    if (hipSetDevice(device) != hipSuccess) return FFTCONV_HIP_ERROR;
    fftconv_ctx *c = new (std::nothrow) fftconv_ctx();
    if (!c) return FFTCONV_HIP_ERROR;
    c->device = device; c->stream = nullptr; c->ws = nullptr; c->ws_bytes = 0;
    c->profiling = 0; c->ev_valid = 0; c->last_hip_error[0] = 0;
    for (int i = 0; i < 8; ++i)
        if (hipEventCreate(&c->ev[i]) != hipSuccess) { delete c; return FFTCONV_HIP_ERROR; }
    *out = c;
    return FFTCONV_OK;
}

int fftconv_destroy(fftconv_handle h) {
    if (!h) return FFTCONV_INVALID_ARG;
    if (h->ws) (void)hipFree(h->ws);
    for (int i = 0; i < 8; ++i) (void)hipEventDestroy(h->ev[i]);
    delete h;
    return FFTCONV_OK;
}

int fftconv_set_stream(fftconv_handle h, void *stream) {
    if (!h) return FFTCONV_INVALID_ARG;
    h->stream = static_cast<hipStream_t>(stream);
    return FFTCONV_OK;
}

const char *fftconv_status_string(int status) {
    switch (status) {
        case FFTCONV_OK: return "ok";
        case FFTCONV_INVALID_ARG: return "invalid argument";
        case FFTCONV_UNSUPPORTED: return "unsupported Fourier basis size (must be 8..128)";
        case FFTCONV_WORKSPACE_TOO_SMALL: return "workspace too small";
        case FFTCONV_HIP_ERROR: return "HIP runtime error";
        default: return "unknown status";
    }
}

size_t fftconv_workspace_bytes(int pass, int S, int f, int fo, int h, int w, int kh, int kw) {
    PassPlan p;
    if (make_plan(pass, S, f, fo, h, w, kh, kw, &p) != FFTCONV_OK) return 0;
    return p.total;
}

int fft_conv_fprop(fftconv_handle hd, const float *x, const float *wt, float *y,
                   int S, int f, int fo, int h, int w, int kh, int kw, void *ws, size_t ws_bytes) {
    return run_pass(hd, FFTCONV_FPROP, x, wt, y, S, f, fo, h, w, kh, kw, 1.0f, 0, ws, ws_bytes);
}

int fft_conv_bprop(fftconv_handle hd, const float *gy, const float *wt, float *gx,
                   int S, int f, int fo, int h, int w, int kh, int kw, void *ws, size_t ws_bytes) {
    return run_pass(hd, FFTCONV_BPROP, gy, wt, gx, S, f, fo, h, w, kh, kw, 1.0f, 0, ws, ws_bytes);
}

int fft_conv_accgrad(fftconv_handle hd, const float *x, const float *gy, float *gw,
                     int S, int f, int fo, int h, int w, int kh, int kw,
                     float scale, int accumulate, void *ws, size_t ws_bytes) {
    return run_pass(hd, FFTCONV_ACCGRAD, gy, x, gw, S, f, fo, h, w, kh, kw, scale, accumulate, ws, ws_bytes);
}

static bool fft_size_ok(int n) { return n == 8 || n == 16 || n == 32 || n == 64 || n == 128; }

int fft_r2c_1d(fftconv_handle hd, const float *in, float *out, long B, int n_in, int n) {
    if (!hd || B < 0 || n_in <= 0 || (B > 0 && (!in || !out))) return FFTCONV_INVALID_ARG;
    if (!fft_size_ok(n)) return FFTCONV_UNSUPPORTED;
    if (n_in > n) return FFTCONV_INVALID_ARG;
    hipError_t e = launch_fft1d_r2c(in, out, B, n_in, n, LaunchCtx{hd->stream, nullptr, nullptr});
    return e == hipSuccess ? FFTCONV_OK : hip_fail(hd, e);
}

int fft_c2r_1d(fftconv_handle hd, const float *in, float *out, long B, int n, int n_out) {
    if (!hd || B < 0 || n_out <= 0 || (B > 0 && (!in || !out))) return FFTCONV_INVALID_ARG;
    if (!fft_size_ok(n)) return FFTCONV_UNSUPPORTED;
    if (n_out > n) return FFTCONV_INVALID_ARG;
    hipError_t e = launch_fft1d_c2r(in, out, B, n, n_out, LaunchCtx{hd->stream, nullptr, nullptr});
    return e == hipSuccess ? FFTCONV_OK : hip_fail(hd, e);
}

int fft_r2c_2d(fftconv_handle hd, const float *in, float *out, long B, int h_in, int w_in, int n) {
    if (!hd || B < 0 || h_in <= 0 || w_in <= 0 || (B > 0 && (!in || !out))) return FFTCONV_INVALID_ARG;
    if (!fft_size_ok(n)) return FFTCONV_UNSUPPORTED;
    if (h_in > n || w_in > n) return FFTCONV_INVALID_ARG;
    hipError_t e = launch_fft2d_r2c(in, out, B, h_in, w_in, n, false, false, LaunchCtx{hd->stream, nullptr, nullptr});
    return e == hipSuccess ? FFTCONV_OK : hip_fail(hd, e);
}

int fft_c2r_2d(fftconv_handle hd, const float *in, float *out, long B, int n, int h_out, int w_out) {
    if (!hd || B < 0 || h_out <= 0 || w_out <= 0 || (B > 0 && (!in || !out))) return FFTCONV_INVALID_ARG;
    if (!fft_size_ok(n)) return FFTCONV_UNSUPPORTED;
    if (h_out > n || w_out > n) return FFTCONV_INVALID_ARG;
    const float s = 1.0f / ((float)n * (float)n);
    hipError_t e = launch_fft2d_c2r(in, out, B, n, h_out, w_out, false, s, false, LaunchCtx{hd->stream, nullptr, nullptr});
    return e == hipSuccess ? FFTCONV_OK : hip_fail(hd, e);
}

int fftconv_set_profiling(fftconv_handle h, int enabled) {
    if (!h) return FFTCONV_INVALID_ARG;
    h->profiling = enabled ? 1 : 0;
    h->ev_valid = 0;
    return FFTCONV_OK;
}

int fftconv_last_stage_ms(fftconv_handle h, float ms_out[4]) {
    if (!h || !ms_out) return FFTCONV_INVALID_ARG;
    if (!h->ev_valid) return FFTCONV_INVALID_ARG;
    hipError_t e = hipEventSynchronize(h->ev[7]);
    if (e != hipSuccess) return hip_fail(h, e);
    for (int i = 0; i < 4; ++i)
        if ((e = hipEventElapsedTime(&ms_out[i], h->ev[2 * i], h->ev[2 * i + 1])) != hipSuccess) return hip_fail(h, e);
    return FFTCONV_OK;
}

}  // extern "C"
