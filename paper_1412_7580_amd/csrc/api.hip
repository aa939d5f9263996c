// C ABI of the library (include/fftconv.h): argument checks, workspace, and the three pass
// pipelines of Table 1 of the fbfft paper expressed as four launches on one stream:
//   FFT2D(operand A) -> FFT2D(operand B) -> per-bin complex contraction -> IFFT2D + clip.
// The frequency-domain forms used for the two passes the paper leaves as "similar"
// (Section 2) follow from the DFT shift property:
//   fprop   Y  = sum_i  X_si  . conj(W_ji)
//   bprop   GX = sum_j  GY_sj . W_ji
//   accGrad GW = sum_s  conj(GY_sj) . X_si
// each followed by the inverse transform and a crop at the origin.
#include <cstdlib>
#include "../../include/fftconv.h"
#include "kernels.hpp"

#include <mutex>
#include <new>

using namespace fc;

constexpr int kMaxKernels = 8;

// Scratch for fft_conv_fprop_static, the entry point for callers that cannot allocate: the three
// frequency-domain tensors of one fprop live in this array instead of a workspace.  Every GPU
// the library runs on holds its own copy, at its own address, until the process ends.  In host
// code the array's name is only a handle for hipGetSymbolAddress; the address that kernels and
// copies take is the one looked up per device in static_scratch_for().
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char fftconv_static_scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static void *g_static_scratch[kMaxDevices];   // device address of the array on each GPU, once looked up
static std::mutex g_static_scratch_mutex;

// Device address of the static scratch array on `device`, which must be the current device.
static hipError_t static_scratch_for(int device, void **out) {
    *out = nullptr;
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_static_scratch_mutex);
    if (!g_static_scratch[device]) {
        void *ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(fftconv_static_scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_static_scratch[device] = ptr;
    }
    *out = g_static_scratch[device];
    return hipSuccess;
}

struct PassPlan;
struct PlanCache;

struct fftconv_ctx {
    int device;
    GemmSwitches sw;        // A/B switches of the contraction, read from the environment at creation
    PlanCache *plans;       // plans of the layer shapes seen so far
    hipStream_t stream;
    void *ws;
    size_t ws_bytes;
    void *static_scratch;   // this device's copy of fftconv_static_scratch (device address)
    int profiling;
    hipEvent_t ev[2 * 8];   // start/stop pair per kernel of the last call
    int nk;                 // kernels of the last call that carry events
    const char *label[8];   // what each of them is (see fftconv_last_kernel_label)
    char last_hip_error[256];
};

// Fourier bases of the 2-D transforms: the powers of two 8 ... 128 (Section 5 of the paper) and,
// between them, sizes 2^a * {3, 5, 7, 9} from the search space of Section 3.4: one odd factor
// everywhere, and 10, 18 and 36, which close the widest gaps of that ladder below 40 (the
// sizes with a factor 15 measured slower than the next power of two and are left out).
static const int kBases[] = {8, 10, 12, 14, 16, 18, 20, 24, 28, 32, 36, 40, 48, 56, 64, 80, 96, 112, 128};
static bool basis_ok(int n) {
    for (int b : kBases) if (b == n) return true;
    return false;
}
// Smallest basis that holds an h x w image; above 128 for images that none holds.
static int basis_size(int h, int w) {
    const int m = h > w ? h : w;
    for (int b : kBases) if (b >= m) return b;
    return 256;
}

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct PassPlan {
    int N, bins;
    bool rect;          // rectangular basis Nr x Nc (untiled, unpadded layers only); N = the larger side
    int Nr, Nc;
    long planesA, planesB, planesC;
    int hA, wA, hB, wB, hC, wC;
    bool conjA, conjB;
    int M, Nn, K;
    long a_rs, a_cs, b_rs, b_cs, c_rs, c_cs;
    FreqLayout lay;
    size_t offA, offB, offC, total;
    // Tiling (Section 6 of the paper): which operands are windows of larger images, and how.
    bool tiled;
    bool viewA, viewB, viewC;
    PlaneView vA, vB, vC;
};

static int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Tile basis used when the caller leaves the choice to the library: the basis that minimises
// (number of tiles) x (bins per tile) x (relative cost of a bin at that basis).  The first two
// factors count the contraction's work and the frequency tensors' size; the tile count is the
// mean over the three passes (fprop and accGrad tile the output, bprop the input), so that all
// passes of a layer get the same basis and can share transforms.  The third factor is measured
// (time of the three passes per tile-bin on 224x224 5x5 and 3x3, 160x160 11x11 and 72x72 7x7
// layers on this chip, relative to basis 32): flat from 16 to 32, about 10 % more from 40 to 56,
// 20 % at 64, more at the small bases (many tiny planes, long reductions in accGrad), and
// 2.4 .. 2.9x from 80 on (one plane per workgroup, scalar gathers in the contraction).
// Output tiles are (n - kh + 1) x (n - kw + 1).
static double basis_weight(int n) {
    return n <= 8 ? 1.6 : n <= 12 ? 1.2 : n <= 14 ? 1.1 : n <= 16 ? 1.05 : n <= 32 ? 1.0 : n <= 56 ? 1.1 : n <= 64 ? 1.2
                                                                                          : n <= 112 ? 2.4 : 2.9;
}
static double basis_cost(int n, int h, int w, int kh, int kw) {
    const int oh = h - kh + 1, ow = w - kw + 1, dy = n - kh + 1, dx = n - kw + 1;
    const double tiles = (2.0 * ceil_div(oh, dy) * ceil_div(ow, dx) + (double)ceil_div(h, dy) * ceil_div(w, dx)) / 3.0;
    return tiles * n * (n / 2 + 1) * basis_weight(n);
}
static int pick_tile_basis(int h, int w, int kh, int kw, double *cost_out = nullptr) {
    int best = 0;
    double best_cost = 0;
    for (int n : kBases) {
        if (n < kh || n < kw) continue;
        const double cost = basis_cost(n, h, w, kh, kw);
        if (!best || cost < best_cost) { best = n; best_cost = cost; }
    }
    if (cost_out) *cost_out = best_cost;
    return best;
}

// tile_n: -1 = the ordinary entry points: tile when the layer needs it (basis above 128) or
// when the estimate says tiling is clearly cheaper (in practice the layers whose untiled basis
// would be 80 or more: measured 2..5x faster tiled at a basis between 24 and 64); 0 = tile with
// the library's choice of basis; else use basis tile_n, tiled unless it holds the whole image.
// ph, pw: rows / columns of zeros around every input image (Section 2's p_h, p_w); the output
// is then (h + 2 ph - kh + 1) x (w + 2 pw - kw + 1).  Padded layers always run on windows (a
// single window per image when the padded image fits the basis): the padding is the part of
// a window that lies outside the image and reads as zero.
static int make_plan(int pass, int S, int f, int fo, int h, int w, int kh, int kw, PassPlan *p, int tile_n = -1,
                     int ph = 0, int pw = 0) {
    if (S <= 0 || f <= 0 || fo <= 0 || h <= 0 || w <= 0 || kh <= 0 || kw <= 0) return FFTCONV_INVALID_ARG;
    if (ph < 0 || pw < 0) return FFTCONV_INVALID_ARG;
    const int hp = h + 2 * ph, wp = w + 2 * pw;             // padded image
    if (kh > hp || kw > wp) return FFTCONV_INVALID_ARG;
    if (pass < 0 || pass > 2) return FFTCONV_INVALID_ARG;
    if (tile_n > 0 && (!basis_ok(tile_n) || tile_n < kh || tile_n < kw)) return FFTCONV_INVALID_ARG;
    int N = basis_size(hp, wp);
    bool tiled = tile_n >= 0 || ph > 0 || pw > 0;
    // a named basis that holds the whole (unpadded) image: the ordinary untiled plan at that basis
    const bool whole = tile_n > 0 && ph == 0 && pw == 0 && tile_n >= h && tile_n >= w;
    if (whole) { tiled = false; N = tile_n; }
    if (tiled && tile_n < 0) tile_n = 0;
    if (N > 128) { tiled = true; if (tile_n < 0) tile_n = 0; }
    // each side on the smallest basis that holds it, where the rectangular kernels exist
    int nr = N, nc = N;
    if (!tiled && !whole) {
        nr = basis_size(h, 1); nc = basis_size(1, w);
        if (nr == nc || !fft2d_rect_supported(nr, nc)) nr = nc = N;
    }
    if (!tiled && !whole) {
        double cost = 0;
        const int tn = pick_tile_basis(hp, wp, kh, kw, &cost);
        if (tn && tn < N && cost < 0.8 * nr * (nc / 2 + 1) * basis_weight(N)) { tiled = true; tile_n = tn; }
    }
    if (tiled && tile_n == 0) tile_n = pick_tile_basis(hp, wp, kh, kw);
    if (tiled && tile_n == 0) return FFTCONV_UNSUPPORTED;   // kernel larger than every basis
    if (tiled) N = tile_n;
    const int oh = hp - kh + 1, ow = wp - kw + 1;
    const int dy = N - kh + 1, dx = N - kw + 1;             // output tile (tiled plans only)
    p->N = N;
    p->bins = fft2d_layout_bins(N);
    p->lay.tsh = fft2d_tile_log2(N);
    p->rect = false; p->Nr = p->Nc = N;
    if (!tiled && !whole && nr != nc) {
        p->rect = true; p->Nr = nr; p->Nc = nc;
        p->bins = fft2d_rect_layout_bins(nr, nc);
        p->lay.tsh = fft2d_rect_tile_log2(nr, nc);
    }
    p->lay.bins = p->bins;
    p->conjA = p->conjB = false;
    p->tiled = tiled;
    p->viewA = p->viewB = p->viewC = false;
    p->vA = p->vB = p->vC = PlaneView{};
    auto imin = [](int a, int b) { return a < b ? a : b; };
    switch (pass) {
        case FFTCONV_FPROP: {
            long Sm = S;
            p->hA = h;  p->wA = w;  p->hC = oh; p->wC = ow;
            if (tiled) {
                // y[a0 + r] needs padded x[a0 + r + u]: windows of N rows starting ph rows
                // before the tile origin
                const int nty = ceil_div(oh, dy), ntx = ceil_div(ow, dx);
                Sm = (long)S * nty * ntx;
                p->viewA = true; p->vA = PlaneView{f, nty, ntx, dy, dx, -ph, -pw, h, w};
                p->hA = imin(N, h + ph); p->wA = imin(N, w + pw);
                p->viewC = true; p->vC = PlaneView{fo, nty, ntx, dy, dx, 0, 0, oh, ow};
                p->hC = imin(dy, oh); p->wC = imin(dx, ow);
            }
            p->planesA = Sm * f;
            p->planesB = (long)fo * f; p->hB = kh; p->wB = kw; p->conjB = true;
            p->planesC = Sm * fo;
            p->M = (int)Sm; p->Nn = fo; p->K = f;
            p->a_rs = f;  p->a_cs = 1;     // A(s,i) = XF[s][i]
            p->b_rs = 1;  p->b_cs = f;     // B(i,j) = conj WF[j][i]
            p->c_rs = fo; p->c_cs = 1;     // C(s,j) = YF[s][j]
            break;
        }
        case FFTCONV_BPROP: {
            long Sm = S;
            p->hA = oh; p->wA = ow; p->hC = h;  p->wC = w;
            if (tiled) {
                // gx[p0 + t] = sum_u gy[p0 + t + ph - u] w[u]: windows of N rows starting
                // kh - 1 - ph rows before the tile origin; the cyclic result is valid from row
                // kh - 1 on
                const int nty = ceil_div(h, dy), ntx = ceil_div(w, dx);
                Sm = (long)S * nty * ntx;
                p->viewA = true; p->vA = PlaneView{fo, nty, ntx, dy, dx, ph - (kh - 1), pw - (kw - 1), oh, ow};
                p->hA = N; p->wA = N;
                p->viewC = true; p->vC = PlaneView{f, nty, ntx, dy, dx, kh - 1, kw - 1, h, w};
                p->hC = imin(dy, h); p->wC = imin(dx, w);
            }
            p->planesA = Sm * fo;
            p->planesB = (long)fo * f; p->hB = kh; p->wB = kw;
            p->planesC = Sm * f;
            p->M = (int)Sm; p->Nn = f; p->K = fo;
            p->a_rs = fo; p->a_cs = 1;     // A(s,j) = GYF[s][j]
            p->b_rs = f;  p->b_cs = 1;     // B(j,i) = WF[j][i]
            p->c_rs = f;  p->c_cs = 1;     // C(s,i) = GXF[s][i]
            break;
        }
        default: {
            long Sm = S;
            p->hA = oh; p->wA = ow; p->hB = h;  p->wB = w;
            if (tiled) {
                // gw[u] = sum over samples and tiles of (gy tile) correlated with (padded x
                // window): the tile index joins the sample index in the reduction
                const int nty = ceil_div(oh, dy), ntx = ceil_div(ow, dx);
                Sm = (long)S * nty * ntx;
                p->viewA = true; p->vA = PlaneView{fo, nty, ntx, dy, dx, 0, 0, oh, ow};
                p->hA = imin(dy, oh); p->wA = imin(dx, ow);
                p->viewB = true; p->vB = PlaneView{f, nty, ntx, dy, dx, -ph, -pw, h, w};
                p->hB = imin(N, h + ph); p->wB = imin(N, w + pw);
            }
            p->planesA = Sm * fo; p->conjA = true;
            p->planesB = Sm * f;
            p->planesC = (long)fo * f; p->hC = kh; p->wC = kw;
            p->M = fo; p->Nn = f; p->K = (int)Sm;
            p->a_rs = 1;  p->a_cs = fo;    // A(j,s) = conj GYF[s][j]
            p->b_rs = f;  p->b_cs = 1;     // B(s,i) = XF[s][i]
            p->c_rs = f;  p->c_cs = 1;     // C(j,i) = GWF[j][i]
            break;
        }
    }
    if (p->planesA > 0x7fffffffL || p->planesB > 0x7fffffffL || p->planesC > 0x7fffffffL) return FFTCONV_UNSUPPORTED;
    p->offA = 0;
    p->offB = align_up(p->offA + p->lay.floats(p->planesA) * sizeof(float), 256);
    p->offC = align_up(p->offB + p->lay.floats(p->planesB) * sizeof(float), 256);
    p->total = align_up(p->offC + p->lay.floats(p->planesC) * sizeof(float), 256);
    return FFTCONV_OK;
}

// Plans by layer shape, kept in the handle (the per-problem-size strategy cache of Section 3.4 of
// the paper): a call on a shape seen before skips the basis choice and tiling arithmetic.  A
// small ring, searched linearly; a training loop cycles through a handful of layer shapes.
struct PlanKey {
    int v[11];   // pass, S, f, fo, h, w, kh, kw, tile_n, ph, pw
    bool operator==(const PlanKey &o) const {
        for (int i = 0; i < 11; ++i) if (v[i] != o.v[i]) return false;
        return true;
    }
};
struct PlanCache {
    static constexpr int kSlots = 48;
    PlanKey key[kSlots];
    PassPlan plan[kSlots];
    int used = 0, next = 0;
};

// make_plan through the handle's cache (only valid plans are kept).
static int cached_plan(fftconv_ctx *c, int pass, int S, int f, int fo, int h, int w, int kh, int kw, PassPlan *p,
                       int tile_n = -1, int ph = 0, int pw = 0) {
    if (!c || !c->plans) return make_plan(pass, S, f, fo, h, w, kh, kw, p, tile_n, ph, pw);
    PlanCache &pc = *c->plans;
    const PlanKey k{{pass, S, f, fo, h, w, kh, kw, tile_n, ph, pw}};
    for (int i = 0; i < pc.used; ++i)
        if (pc.key[i] == k) { *p = pc.plan[i]; return FFTCONV_OK; }
    const int rc = make_plan(pass, S, f, fo, h, w, kh, kw, p, tile_n, ph, pw);
    if (rc != FFTCONV_OK) return rc;
    const int slot = pc.used < PlanCache::kSlots ? pc.used++ : (pc.next = (pc.next + 1) % PlanCache::kSlots);
    pc.key[slot] = k; pc.plan[slot] = *p;
    return FFTCONV_OK;
}

static int hip_fail(fftconv_ctx *c, hipError_t e) {
    if (c) snprintf(c->last_hip_error, sizeof(c->last_hip_error), "HIP error: %s", hipGetErrorString(e));
    return FFTCONV_HIP_ERROR;
}

static int get_workspace(fftconv_ctx *c, size_t need, void **ws, size_t ws_bytes) {
    if (*ws) return ws_bytes < need ? FFTCONV_WORKSPACE_TOO_SMALL : FFTCONV_OK;
    hipError_t e;
    if (c->ws_bytes < need) {
        // Growing means a synchronisation, a free and an allocation: none of them may happen
        // while the stream is being captured into a graph.  Such a caller passes a workspace (or
        // makes one eager call first, after which the handle's buffer is large enough).
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(c->stream, &cap) == hipSuccess && cap != hipStreamCaptureStatusNone)
            return FFTCONV_WORKSPACE_TOO_SMALL;
        if (c->ws) {
            if ((e = hipStreamSynchronize(c->stream)) != hipSuccess) return hip_fail(c, e);
            (void)hipFree(c->ws);
            c->ws = nullptr; c->ws_bytes = 0;
        }
        if ((e = hipMalloc(&c->ws, need)) != hipSuccess) return hip_fail(c, e);
        c->ws_bytes = need;
    }
    *ws = c->ws;
    return FFTCONV_OK;
}

// Launch context for the next kernel of the current call: with profiling on, each kernel gets
// its own start/stop event pair (kMaxKernels per call).
static LaunchCtx next_ctx(fftconv_ctx *c, const char *label) {
    if (!c->profiling || c->nk >= kMaxKernels) return LaunchCtx{c->stream, nullptr, nullptr, &c->sw};
    const int k = c->nk++;
    c->label[k] = label;
    return LaunchCtx{c->stream, c->ev[2 * k], c->ev[2 * k + 1], &c->sw};
}

static float *at(void *base, size_t off) { return reinterpret_cast<float *>(static_cast<char *>(base) + off); }

// One operand's forward transform into the plane-tiled layout of the plan's basis.
static hipError_t transform(const PassPlan &p, const float *in, float *out, long planes, int h, int w, LaunchCtx lc,
                            const PlaneView *view = nullptr) {
    if (p.rect) {
        const FwdOperand op{in, out, planes, h, w, nullptr};
        return launch_fft2d_r2c_rect(&op, 1, p.Nr, p.Nc, lc);
    }
    return launch_fft2d_r2c(in, out, planes, h, w, p.N, true, lc, view);
}

// Whether two forward transforms of basis N (layout tile 2^tsh planes) go out as one launch.
// Two short kernels would queue behind each other's ramp-up and tail (measured 14 us of 204 per
// step on the 32-basis layer; 28 -> 21 us on a 64-channel 36x36 layer, 38 -> 32 at 45x45 on basis 48,
// 63 -> 48 for the windows and weights of a 160x160 layer tiled at basis 64), so they share a
// launch up to basis 56.  At 64 every block of a shared launch gets the LDS footprint of the
// operand with more rows, which costs the other one occupancy: shared only when that other
// operand is the smaller one (the 31x31 weights of the 64-basis benchmark layer, 16384 planes
// against 4096 of x: 129 us apart, 143 shared).  From 80 on (one plane per workgroup) apart.
static bool share_forward(int N, int tsh, int hA, long planesA, int hB, long planesB) {
    if (tsh >= 3 || N <= 56) return true;
    if (N > 64) return false;
    const int lo = hA < hB ? hA : hB, hi = hA < hB ? hB : hA;
    if (4 * lo >= 3 * hi) return true;        // about the same footprint (gy and the weights there: 118 -> 112 us)
    return hA < hB ? planesA <= planesB : planesB <= planesA;
}

// Forward transforms of both operands of a pass, as one launch where share_forward says so.
// Profiling reports a shared launch as one entry ("fft.ab"), separate ones as "fft.a", "fft.b".
static hipError_t forward_pair(fftconv_ctx *c, const PassPlan &p, const float *a, float *AF,
                               const float *b, float *BF) {
    const PlaneView *va = p.viewA ? &p.vA : nullptr, *vb = p.viewB ? &p.vB : nullptr;
    if (p.rect) {
        FwdOperand ops[2] = {{a, AF, p.planesA, p.hA, p.wA, nullptr}, {b, BF, p.planesB, p.hB, p.wB, nullptr}};
        return launch_fft2d_r2c_rect(ops, 2, p.Nr, p.Nc, next_ctx(c, "fft.ab"));
    }
    if (share_forward(p.N, p.lay.tsh, p.hA, p.planesA, p.hB, p.planesB)) {
        FwdOperand ops[2] = {{a, AF, p.planesA, p.hA, p.wA, va}, {b, BF, p.planesB, p.hB, p.wB, vb}};
        return launch_fft2d_r2c_multi(ops, 2, p.N, next_ctx(c, "fft.ab"));
    }
    hipError_t e = transform(p, a, AF, p.planesA, p.hA, p.wA, next_ctx(c, "fft.a"), va);
    if (e != hipSuccess) return e;
    return transform(p, b, BF, p.planesB, p.hB, p.wB, next_ctx(c, "fft.b"), vb);
}

// The contraction of one pass as the kernels see it.
static GemmProblem gemm_problem(const PassPlan &p, const float *AF, const float *BF, float *CF) {
    GemmProblem g;
    g.A = GemmOperand{AF, p.lay, p.a_rs, p.a_cs, p.conjA};
    g.B = GemmOperand{BF, p.lay, p.b_rs, p.b_cs, p.conjB};
    g.C = CF; g.layC = p.lay; g.C_rs = p.c_rs; g.C_cs = p.c_cs;
    g.M = p.M; g.N = p.Nn; g.K = p.K; g.bins = p.bins;
    return g;
}

// Inverse transform + crop of one pass's product (1/N^2 folded into the output scale).
static hipError_t invert(fftconv_ctx *c, const PassPlan &p, const float *CF, float *out, float scale, int accumulate) {
    const float s = scale / ((float)p.Nr * (float)p.Nc);
    if (p.rect) return launch_fft2d_c2r_rect(CF, out, p.planesC, p.Nr, p.Nc, p.hC, p.wC, s, accumulate != 0, next_ctx(c, "ifft"));
    return launch_fft2d_c2r(CF, out, p.planesC, p.N, p.hC, p.wC, true, s, accumulate != 0, next_ctx(c, "ifft"),
                            p.viewC ? &p.vC : nullptr);
}

// The two inverse transforms of the backward pass (gx from plan pb, gw from plan pa): one
// launch where the basis has one inverse kernel for every operand, else one after the other.
static hipError_t invert_pair(fftconv_ctx *c, const PassPlan &pb, const float *GXF, float *gx, const PassPlan &pa,
                              const float *GWF, float *gw, float scale, int accumulate) {
    if (pb.rect && pa.rect && pb.Nr == pa.Nr && pb.Nc == pa.Nc) {
        const float sb = 1.0f / ((float)pb.Nr * (float)pb.Nc), sa = scale * sb;
        const InvOperand ops[2] = {{GXF, gx, pb.planesC, pb.hC, pb.wC, sb, false, nullptr},
                                   {GWF, gw, pa.planesC, pa.hC, pa.wC, sa, accumulate != 0, nullptr}};
        const int nk = c->nk;
        const hipError_t e = launch_fft2d_c2r_rect_pair(ops, pb.Nr, pb.Nc, next_ctx(c, "ifft.pair"));
        if (e != hipErrorNotSupported) return e;
        c->nk = nk;
    }
    if (!pb.rect && !pa.rect && pb.N == pa.N) {
        const float sb = 1.0f / ((float)pb.N * (float)pb.N), sa = scale / ((float)pa.N * (float)pa.N);
        const InvOperand ops[2] = {{GXF, gx, pb.planesC, pb.hC, pb.wC, sb, false, pb.viewC ? &pb.vC : nullptr},
                                   {GWF, gw, pa.planesC, pa.hC, pa.wC, sa, accumulate != 0, pa.viewC ? &pa.vC : nullptr}};
        const int nk = c->nk;
        const hipError_t e = launch_fft2d_c2r_pair(ops, pb.N, next_ctx(c, "ifft.pair"));
        if (e != hipErrorNotSupported) return e;
        c->nk = nk;   // nothing was launched: give the event pair back
    }
    if (hipError_t e = invert(c, pb, GXF, gx, 1.0f, 0); e != hipSuccess) return e;
    return invert(c, pa, GWF, gw, scale, accumulate);
}

// Contraction + inverse transform of one pass, operands already in the frequency domain.
static hipError_t contract_and_invert(fftconv_ctx *c, const PassPlan &p, const float *AF, const float *BF,
                                      float *CF, float *out, float scale, int accumulate) {
    const GemmProblem g = gemm_problem(p, AF, BF, CF);
    if (hipError_t e = launch_cgemm_bins(g.A, g.B, g.C, g.layC, g.C_rs, g.C_cs, g.M, g.N, g.K, g.bins, next_ctx(c, "contraction")); e != hipSuccess) return e;
    return invert(c, p, CF, out, scale, accumulate);
}

static int run_pass(fftconv_ctx *c, int pass, const float *opA, const float *opB, float *out,
                    int S, int f, int fo, int h, int w, int kh, int kw, float scale, int accumulate,
                    void *ws, size_t ws_bytes, int tile_n = -1, int ph = 0, int pw = 0) {
    if (!c || !opA || !opB || !out) return FFTCONV_INVALID_ARG;
    PassPlan p;
    int rc = cached_plan(c, pass, S, f, fo, h, w, kh, kw, &p, tile_n, ph, pw);
    if (rc != FFTCONV_OK) return rc;
    // accGrad of a layer of few samples or very small images runs as ONE launch (as the
    // weights-ahead fprop / bprop of small layers do): no workspace is touched then.
    if (pass == FFTCONV_ACCGRAD && tile_n < 0 && !p.tiled && !p.rect && ph == 0 && pw == 0 &&
        fused_accgrad_pays(p.N, S, f, fo)) {
        c->nk = 0;
        const hipError_t e1 = launch_fused_accgrad(opA, opB, out, S, f, fo, h, w, kh, kw, p.N, scale, accumulate,
                                                   next_ctx(c, "fused"));
        if (e1 == hipSuccess) return FFTCONV_OK;
        if (e1 != hipErrorInvalidValue) return hip_fail(c, e1);   // (invalid value: the planes do not fit the kernel's LDS plan)
    }
    if ((rc = get_workspace(c, p.total, &ws, ws_bytes)) != FFTCONV_OK) return rc;
    float *AF = at(ws, p.offA), *BF = at(ws, p.offB), *CF = at(ws, p.offC);
    c->nk = 0;
    hipError_t e;
    if ((e = forward_pair(c, p, opA, AF, opB, BF)) != hipSuccess) return hip_fail(c, e);
    if ((e = contract_and_invert(c, p, AF, BF, CF, out, scale, accumulate)) != hipSuccess) return hip_fail(c, e);
    return FFTCONV_OK;
}

// fprop / bprop with the weights already in the frequency domain (wf from
// fft_conv_transform_weights): one forward transform, the contraction, the inverse.
static int run_pass_weights(fftconv_ctx *c, int pass, const float *opA, const void *wf, size_t wf_bytes, float *out,
                            int S, int f, int fo, int h, int w, int kh, int kw, int ph, int pw,
                            void *ws, size_t ws_bytes) {
    if (!c || !opA || !wf || !out) return FFTCONV_INVALID_ARG;
    PassPlan p;
    int rc = cached_plan(c, pass, S, f, fo, h, w, kh, kw, &p, -1, ph, pw);
    if (rc != FFTCONV_OK) return rc;
    if (wf_bytes < align_up(p.lay.floats(p.planesB) * sizeof(float), 256)) return FFTCONV_WORKSPACE_TOO_SMALL;
    // Latency-bound layers (a few dozen small planes) run as ONE launch: three launches of a few
    // microseconds each cost more than their arithmetic (Section 6 plans such an integration).
    // The one-launch kernels carry one sample per workgroup, so they pay while the samples are a
    // single round of workgroups.
    if (!p.tiled && !p.rect && ph == 0 && pw == 0 && S <= 512) {
        const float *wff = static_cast<const float *>(wf);
        const bool ok = pass == FFTCONV_FPROP ? fused_fprop_supported(p.N, f, fo, wff) : fused_bprop_supported(p.N, f, fo, wff);
        if (ok) {
            c->nk = 0;
            const hipError_t e = pass == FFTCONV_FPROP
                                     ? launch_fused_fprop(opA, wff, out, S, f, fo, h, w, kh, kw, p.N, next_ctx(c, "fused"))
                                     : launch_fused_bprop(opA, wff, out, S, f, fo, h, w, kh, kw, p.N, next_ctx(c, "fused"));
            if (e == hipSuccess) return FFTCONV_OK;
            if (e != hipErrorInvalidValue) return hip_fail(c, e);   // (invalid value: the planes do not fit the kernel's LDS plan)
        }
    }
    if ((rc = get_workspace(c, p.total, &ws, ws_bytes)) != FFTCONV_OK) return rc;
    float *AF = at(ws, p.offA), *CF = at(ws, p.offC);
    c->nk = 0;
    hipError_t e = transform(p, opA, AF, p.planesA, p.hA, p.wA, next_ctx(c, "fft.a"), p.viewA ? &p.vA : nullptr);
    if (e != hipSuccess) return hip_fail(c, e);
    if ((e = contract_and_invert(c, p, AF, static_cast<const float *>(wf), CF, out, 1.0f, 0)) != hipSuccess) return hip_fail(c, e);
    return FFTCONV_OK;
}

// Layout of the buffer that carries the input and weight transforms from fprop to the
// backward call: [XF | WF], each in the plane-tiled layout of the layer's basis.
struct SavedPlan {
    size_t offX, offW, total;
};
static SavedPlan saved_plan(const PassPlan &fp) {
    SavedPlan s;
    s.offX = 0;
    s.offW = align_up(fp.lay.floats(fp.planesA) * sizeof(float), 256);
    s.total = align_up(s.offW + fp.lay.floats(fp.planesB) * sizeof(float), 256);
    return s;
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
    c->profiling = 0; c->nk = 0; c->last_hip_error[0] = 0;
    c->static_scratch = nullptr;
    c->sw = read_gemm_switches();
    c->plans = new (std::nothrow) PlanCache();   // without it every call plans afresh
    // this device's copy of the static scratch array (the device is current here)
    if (static_scratch_for(device, &c->static_scratch) != hipSuccess) { delete c->plans; delete c; return FFTCONV_HIP_ERROR; }
    for (int i = 0; i < 2 * kMaxKernels; ++i)
        if (hipEventCreate(&c->ev[i]) != hipSuccess) {
            for (int j = 0; j < i; ++j) (void)hipEventDestroy(c->ev[j]);
            delete c->plans; delete c;
            return FFTCONV_HIP_ERROR;
        }
    *out = c;
    return FFTCONV_OK;
}

int fftconv_destroy(fftconv_handle h) {
    if (!h) return FFTCONV_INVALID_ARG;
    if (h->ws) (void)hipFree(h->ws);
    for (int i = 0; i < 2 * kMaxKernels; ++i) (void)hipEventDestroy(h->ev[i]);
    delete h->plans;
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
        case FFTCONV_UNSUPPORTED: return "unsupported transform size or layer shape for this entry point";
        case FFTCONV_WORKSPACE_TOO_SMALL: return "workspace too small";
        case FFTCONV_HIP_ERROR: return "HIP runtime error";
        case FFTCONV_STATIC_SCRATCH_EXCEEDED: return "layer needs more scratch than the library's static buffer holds";
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

size_t fftconv_static_scratch_bytes(void) { return kStaticScratchBytes; }

int fft_conv_fprop_static(fftconv_handle hd, const float *x, const float *wt, float *y,
                          int S, int f, int fo, int h, int w, int kh, int kw) {
    if (!hd || !x || !wt || !y) return FFTCONV_INVALID_ARG;
    PassPlan p;
    const int rc = cached_plan(hd, FFTCONV_FPROP, S, f, fo, h, w, kh, kw, &p);
    if (rc != FFTCONV_OK) return rc;
    if (p.total > kStaticScratchBytes) return FFTCONV_STATIC_SCRATCH_EXCEEDED;
    if (!hd->static_scratch) return FFTCONV_HIP_ERROR;
    // the same pipeline as fft_conv_fprop with the device's static array as the workspace: every
    // frequency-domain element that is read was written by this call's transforms first, so
    // nothing of the array needs clearing between calls
    return run_pass(hd, FFTCONV_FPROP, x, wt, y, S, f, fo, h, w, kh, kw, 1.0f, 0, hd->static_scratch,
                    kStaticScratchBytes);
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

size_t fftconv_tiled_workspace_bytes(int pass, int S, int f, int fo, int h, int w, int kh, int kw, int tile_n) {
    PassPlan p;
    if (tile_n < 0 || make_plan(pass, S, f, fo, h, w, kh, kw, &p, tile_n) != FFTCONV_OK) return 0;
    return p.total;
}

int fftconv_layer_basis(int h, int w, int kh, int kw, int pad_h, int pad_w, int *n_rows, int *n_cols) {
    PassPlan p;
    const int rc = make_plan(FFTCONV_FPROP, 1, 1, 1, h, w, kh, kw, &p, -1, pad_h, pad_w);
    if (rc != FFTCONV_OK) return -rc;
    if (n_rows) *n_rows = p.Nr;
    if (n_cols) *n_cols = p.Nc;
    return p.tiled ? 1 : 0;
}

int fftconv_describe_plan(int pass, int S, int f, int fo, int h, int w, int kh, int kw, int tile_n,
                          int pad_h, int pad_w, long *out, int cap) {
    PassPlan p;
    const int rc = make_plan(pass, S, f, fo, h, w, kh, kw, &p, tile_n, pad_h, pad_w);
    if (rc != FFTCONV_OK) return -rc;
    long v[61];
    int n = 0;
    v[n++] = p.Nr; v[n++] = p.Nc; v[n++] = p.tiled; v[n++] = p.rect; v[n++] = p.bins; v[n++] = p.lay.tsh;
    v[n++] = p.planesA; v[n++] = p.planesB; v[n++] = p.planesC;
    v[n++] = p.hA; v[n++] = p.wA; v[n++] = p.hB; v[n++] = p.wB; v[n++] = p.hC; v[n++] = p.wC;
    v[n++] = p.M; v[n++] = p.Nn; v[n++] = p.K;
    v[n++] = p.conjA; v[n++] = p.conjB;
    v[n++] = p.a_rs; v[n++] = p.a_cs; v[n++] = p.b_rs; v[n++] = p.b_cs; v[n++] = p.c_rs; v[n++] = p.c_cs;
    v[n++] = (long)p.offA; v[n++] = (long)p.offB; v[n++] = (long)p.offC; v[n++] = (long)p.total;
    v[n++] = (long)(p.lay.floats(p.planesA) * sizeof(float));
    const bool has[3] = {p.viewA, p.viewB, p.viewC};
    const PlaneView *views[3] = {&p.vA, &p.vB, &p.vC};
    for (int i = 0; i < 3; ++i) {
        const PlaneView &q = *views[i];
        v[n++] = has[i]; v[n++] = q.C; v[n++] = q.nty; v[n++] = q.ntx; v[n++] = q.dy; v[n++] = q.dx;
        v[n++] = q.oy; v[n++] = q.ox; v[n++] = q.H; v[n++] = q.W;
    }
    for (int i = 0; i < n && i < cap; ++i) if (out) out[i] = v[i];
    return n;
}

int fftconv_tile_basis(int h, int w, int kh, int kw, int tile_n) {
    PassPlan p;
    if (tile_n < 0 || make_plan(FFTCONV_FPROP, 1, 1, 1, h, w, kh, kw, &p, tile_n) != FFTCONV_OK) return 0;
    return p.N;
}

int fft_conv_fprop_tiled(fftconv_handle hd, const float *x, const float *wt, float *y,
                         int S, int f, int fo, int h, int w, int kh, int kw, int tile_n,
                         void *ws, size_t ws_bytes) {
    if (tile_n < 0) return FFTCONV_INVALID_ARG;
    return run_pass(hd, FFTCONV_FPROP, x, wt, y, S, f, fo, h, w, kh, kw, 1.0f, 0, ws, ws_bytes, tile_n);
}

int fft_conv_bprop_tiled(fftconv_handle hd, const float *gy, const float *wt, float *gx,
                         int S, int f, int fo, int h, int w, int kh, int kw, int tile_n,
                         void *ws, size_t ws_bytes) {
    if (tile_n < 0) return FFTCONV_INVALID_ARG;
    return run_pass(hd, FFTCONV_BPROP, gy, wt, gx, S, f, fo, h, w, kh, kw, 1.0f, 0, ws, ws_bytes, tile_n);
}

int fft_conv_accgrad_tiled(fftconv_handle hd, const float *x, const float *gy, float *gw,
                           int S, int f, int fo, int h, int w, int kh, int kw,
                           float scale, int accumulate, int tile_n, void *ws, size_t ws_bytes) {
    if (tile_n < 0) return FFTCONV_INVALID_ARG;
    return run_pass(hd, FFTCONV_ACCGRAD, gy, x, gw, S, f, fo, h, w, kh, kw, scale, accumulate, ws, ws_bytes, tile_n);
}

int fftconv_autotune_basis(fftconv_handle hd, const float *x, const float *wt, const float *gy,
                           float *y, float *gx, float *gw, int S, int f, int fo, int h, int w, int kh, int kw,
                           int reps, int *basis_out, float *ms_out) {
    if (!hd || !x || !wt || !gy || !y || !gx || !gw || !basis_out || reps <= 0) return FFTCONV_INVALID_ARG;
    *basis_out = 0;
    PassPlan probe;
    if (int st = make_plan(FFTCONV_FPROP, S, f, fo, h, w, kh, kw, &probe, 0); st != FFTCONV_OK) return st;
    // Candidates: every basis that holds the kernel and whose estimated cost is within 3x of
    // the lowest estimate (the rest are far off and would only cost workspace and time).
    double low = 0;
    for (int n : kBases)
        if (n >= kh && n >= kw) { const double c = basis_cost(n, h, w, kh, kw); if (low == 0 || c < low) low = c; }
    hipEvent_t t0, t1;
    if (hipEventCreate(&t0) != hipSuccess) return FFTCONV_HIP_ERROR;
    if (hipEventCreate(&t1) != hipSuccess) { (void)hipEventDestroy(t0); return FFTCONV_HIP_ERROR; }
    const int was_profiling = hd->profiling;
    hd->profiling = 0;
    int status = FFTCONV_OK, best = 0;
    float best_ms = 0;
    auto step = [&](int n) -> int {
        int st;
        if ((st = run_pass(hd, FFTCONV_FPROP, x, wt, y, S, f, fo, h, w, kh, kw, 1.0f, 0, nullptr, 0, n)) != FFTCONV_OK) return st;
        if ((st = run_pass(hd, FFTCONV_BPROP, gy, wt, gx, S, f, fo, h, w, kh, kw, 1.0f, 0, nullptr, 0, n)) != FFTCONV_OK) return st;
        return run_pass(hd, FFTCONV_ACCGRAD, gy, x, gw, S, f, fo, h, w, kh, kw, 1.0f, 0, nullptr, 0, n);
    };
    for (int n : kBases) {
        if (n < kh || n < kw || basis_cost(n, h, w, kh, kw) > 3.0 * low) continue;
        if ((status = step(n)) != FFTCONV_OK) break;                       // warm-up, grows the workspace
        hipError_t e = hipEventRecord(t0, hd->stream);
        for (int r = 0; r < reps && status == FFTCONV_OK; ++r) status = step(n);
        if (status != FFTCONV_OK) break;
        if (e == hipSuccess) e = hipEventRecord(t1, hd->stream);
        if (e == hipSuccess) e = hipEventSynchronize(t1);
        float ms = 0;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, t0, t1);
        if (e != hipSuccess) { status = hip_fail(hd, e); break; }
        ms /= (float)reps;
        if (!best || ms < best_ms) { best = n; best_ms = ms; }
    }
    hd->profiling = was_profiling;
    (void)hipEventDestroy(t0); (void)hipEventDestroy(t1);
    if (status != FFTCONV_OK) return status;
    // leave the outputs as the chosen basis computes them
    if ((status = step(best)) != FFTCONV_OK) return status;
    *basis_out = best;
    if (ms_out) *ms_out = best_ms;
    return FFTCONV_OK;
}

size_t fftconv_padded_workspace_bytes(int pass, int S, int f, int fo, int h, int w, int kh, int kw,
                                      int pad_h, int pad_w) {
    PassPlan p;
    if (make_plan(pass, S, f, fo, h, w, kh, kw, &p, -1, pad_h, pad_w) != FFTCONV_OK) return 0;
    return p.total;
}

int fft_conv_fprop_padded(fftconv_handle hd, const float *x, const float *wt, float *y,
                          int S, int f, int fo, int h, int w, int kh, int kw, int pad_h, int pad_w,
                          void *ws, size_t ws_bytes) {
    return run_pass(hd, FFTCONV_FPROP, x, wt, y, S, f, fo, h, w, kh, kw, 1.0f, 0, ws, ws_bytes, -1, pad_h, pad_w);
}

int fft_conv_bprop_padded(fftconv_handle hd, const float *gy, const float *wt, float *gx,
                          int S, int f, int fo, int h, int w, int kh, int kw, int pad_h, int pad_w,
                          void *ws, size_t ws_bytes) {
    return run_pass(hd, FFTCONV_BPROP, gy, wt, gx, S, f, fo, h, w, kh, kw, 1.0f, 0, ws, ws_bytes, -1, pad_h, pad_w);
}

int fft_conv_accgrad_padded(fftconv_handle hd, const float *x, const float *gy, float *gw,
                            int S, int f, int fo, int h, int w, int kh, int kw, int pad_h, int pad_w,
                            float scale, int accumulate, void *ws, size_t ws_bytes) {
    return run_pass(hd, FFTCONV_ACCGRAD, gy, x, gw, S, f, fo, h, w, kh, kw, scale, accumulate, ws, ws_bytes, -1,
                    pad_h, pad_w);
}

static bool fft_size_ok(int n) { return n == 2 || n == 4 || basis_ok(n); }
// 1-D transforms go one octave further (the range of Section 5.3 of the paper).
static bool fft1d_size_ok(int n) { return fft_size_ok(n) || n == 160 || n == 192 || n == 224 || n == 256; }

int fft_r2c_1d(fftconv_handle hd, const float *in, float *out, long B, int n_in, int n) {
    if (!hd || B < 0 || n_in <= 0 || (B > 0 && (!in || !out))) return FFTCONV_INVALID_ARG;
    if (!fft1d_size_ok(n)) return FFTCONV_UNSUPPORTED;
    if (n_in > n) return FFTCONV_INVALID_ARG;
    hipError_t e = launch_fft1d_r2c(in, out, B, n_in, n, LaunchCtx{hd->stream, nullptr, nullptr});
    return e == hipSuccess ? FFTCONV_OK : hip_fail(hd, e);
}

int fft_c2r_1d(fftconv_handle hd, const float *in, float *out, long B, int n, int n_out) {
    if (!hd || B < 0 || n_out <= 0 || (B > 0 && (!in || !out))) return FFTCONV_INVALID_ARG;
    if (!fft1d_size_ok(n)) return FFTCONV_UNSUPPORTED;
    if (n_out > n) return FFTCONV_INVALID_ARG;
    hipError_t e = launch_fft1d_c2r(in, out, B, n, n_out, LaunchCtx{hd->stream, nullptr, nullptr});
    return e == hipSuccess ? FFTCONV_OK : hip_fail(hd, e);
}

int fft_r2c_2d(fftconv_handle hd, const float *in, float *out, long B, int h_in, int w_in, int n) {
    if (!hd || B < 0 || h_in <= 0 || w_in <= 0 || (B > 0 && (!in || !out))) return FFTCONV_INVALID_ARG;
    if (!fft_size_ok(n)) return FFTCONV_UNSUPPORTED;
    if (h_in > n || w_in > n) return FFTCONV_INVALID_ARG;
    hipError_t e = launch_fft2d_r2c(in, out, B, h_in, w_in, n, false, LaunchCtx{hd->stream, nullptr, nullptr});
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
    h->nk = 0;
    return FFTCONV_OK;
}

const char *fftconv_last_kernel_label(fftconv_handle h, int i) {
    if (!h || !h->profiling || i < 0 || i >= h->nk) return "";
    return h->label[i];
}

int fftconv_last_kernel_ms(fftconv_handle h, float *ms_out, int capacity, int *count) {
    if (!h || !ms_out || !count || capacity < 0) return FFTCONV_INVALID_ARG;
    *count = 0;
    if (!h->profiling || h->nk == 0) return FFTCONV_INVALID_ARG;
    hipError_t e = hipEventSynchronize(h->ev[2 * (h->nk - 1) + 1]);
    if (e != hipSuccess) return hip_fail(h, e);
    const int n = h->nk < capacity ? h->nk : capacity;
    for (int i = 0; i < n; ++i)
        if ((e = hipEventElapsedTime(&ms_out[i], h->ev[2 * i], h->ev[2 * i + 1])) != hipSuccess) return hip_fail(h, e);
    *count = n;
    return FFTCONV_OK;
}

static size_t saved_bytes_impl(int S, int f, int fo, int h, int w, int kh, int kw, int ph, int pw, int tile_n = -1) {
    PassPlan p;
    if (make_plan(FFTCONV_FPROP, S, f, fo, h, w, kh, kw, &p, tile_n, ph, pw) != FFTCONV_OK) return 0;
    return saved_plan(p).total;
}

size_t fftconv_saved_bytes(int S, int f, int fo, int h, int w, int kh, int kw) {
    return saved_bytes_impl(S, f, fo, h, w, kh, kw, 0, 0);
}

size_t fftconv_saved_bytes_padded(int S, int f, int fo, int h, int w, int kh, int kw, int pad_h, int pad_w) {
    return saved_bytes_impl(S, f, fo, h, w, kh, kw, pad_h, pad_w);
}

size_t fftconv_saved_bytes_tiled(int S, int f, int fo, int h, int w, int kh, int kw, int tile_n) {
    return tile_n < 0 ? 0 : saved_bytes_impl(S, f, fo, h, w, kh, kw, 0, 0, tile_n);
}

// Workspace of fft_conv_backward: [GYF for bprop | GYF for accGrad (tiled layers only: the two
// passes cut gy into different windows) | GXF | GWF], one product buffer per pass because the
// two contractions may run in one launch.
struct BackwardPlan {
    size_t offGYb, offGYa, offGX, offGW, total;
};
static BackwardPlan backward_plan(const PassPlan &pb, const PassPlan &pa) {
    BackwardPlan b;
    b.offGYb = 0;
    b.offGYa = 0;
    size_t at = align_up(pb.lay.floats(pb.planesA) * sizeof(float), 256);
    if (pb.tiled) { b.offGYa = at; at += align_up(pa.lay.floats(pa.planesA) * sizeof(float), 256); }
    b.offGX = at; at += align_up(pb.lay.floats(pb.planesC) * sizeof(float), 256);
    b.offGW = at; at += align_up(pa.lay.floats(pa.planesC) * sizeof(float), 256);
    b.total = at;
    return b;
}

static size_t backward_workspace_impl(int S, int f, int fo, int h, int w, int kh, int kw, int ph, int pw,
                                      int tile_n = -1) {
    PassPlan pb, pa;
    if (make_plan(FFTCONV_BPROP, S, f, fo, h, w, kh, kw, &pb, tile_n, ph, pw) != FFTCONV_OK) return 0;
    if (make_plan(FFTCONV_ACCGRAD, S, f, fo, h, w, kh, kw, &pa, tile_n, ph, pw) != FFTCONV_OK) return 0;
    return backward_plan(pb, pa).total;
}

size_t fftconv_backward_workspace_bytes(int S, int f, int fo, int h, int w, int kh, int kw) {
    return backward_workspace_impl(S, f, fo, h, w, kh, kw, 0, 0);
}

size_t fftconv_backward_workspace_bytes_padded(int S, int f, int fo, int h, int w, int kh, int kw,
                                               int pad_h, int pad_w) {
    return backward_workspace_impl(S, f, fo, h, w, kh, kw, pad_h, pad_w);
}

size_t fftconv_backward_workspace_bytes_tiled(int S, int f, int fo, int h, int w, int kh, int kw, int tile_n) {
    return tile_n < 0 ? 0 : backward_workspace_impl(S, f, fo, h, w, kh, kw, 0, 0, tile_n);
}

}  // extern "C"

static int fprop_save_impl(fftconv_handle hd, const float *x, const float *wt, float *y,
                           int S, int f, int fo, int h, int w, int kh, int kw, int ph, int pw,
                           void *saved, size_t saved_bytes, void *ws, size_t ws_bytes, int tile_n = -1) {
    if (!hd || !x || !wt || !y || !saved) return FFTCONV_INVALID_ARG;
    PassPlan p;
    int rc = cached_plan(hd, FFTCONV_FPROP, S, f, fo, h, w, kh, kw, &p, tile_n, ph, pw);
    if (rc != FFTCONV_OK) return rc;
    const SavedPlan sp = saved_plan(p);
    if (saved_bytes < sp.total) return FFTCONV_WORKSPACE_TOO_SMALL;
    const size_t need = align_up(p.lay.floats(p.planesC) * sizeof(float), 256);
    if ((rc = get_workspace(hd, need, &ws, ws_bytes)) != FFTCONV_OK) return rc;
    float *XF = at(saved, sp.offX), *WF = at(saved, sp.offW), *YF = at(ws, 0);
    hd->nk = 0;
    hipError_t e;
    if ((e = forward_pair(hd, p, x, XF, wt, WF)) != hipSuccess) return hip_fail(hd, e);
    if ((e = contract_and_invert(hd, p, XF, WF, YF, y, 1.0f, 0)) != hipSuccess) return hip_fail(hd, e);
    return FFTCONV_OK;
}

static int backward_impl(fftconv_handle hd, const float *gy, float *gx, float *gw,
                         int S, int f, int fo, int h, int w, int kh, int kw, int ph, int pw,
                         float scale, int accumulate, const void *saved, size_t saved_bytes,
                         void *ws, size_t ws_bytes, int tile_n = -1) {
    if (!hd || !gy || !saved || (!gx && !gw)) return FFTCONV_INVALID_ARG;
    PassPlan pf, pb, pa;
    int rc = cached_plan(hd, FFTCONV_FPROP, S, f, fo, h, w, kh, kw, &pf, tile_n, ph, pw);
    if (rc != FFTCONV_OK) return rc;
    if ((rc = cached_plan(hd, FFTCONV_BPROP, S, f, fo, h, w, kh, kw, &pb, tile_n, ph, pw)) != FFTCONV_OK) return rc;
    if ((rc = cached_plan(hd, FFTCONV_ACCGRAD, S, f, fo, h, w, kh, kw, &pa, tile_n, ph, pw)) != FFTCONV_OK) return rc;
    const SavedPlan sp = saved_plan(pf);
    if (saved_bytes < sp.total) return FFTCONV_WORKSPACE_TOO_SMALL;
    const BackwardPlan bp = backward_plan(pb, pa);
    if ((rc = get_workspace(hd, bp.total, &ws, ws_bytes)) != FFTCONV_OK) return rc;
    const float *XF = at(const_cast<void *>(saved), sp.offX), *WF = at(const_cast<void *>(saved), sp.offW);
    float *GYF = at(ws, bp.offGYb), *GYFa = at(ws, bp.offGYa);
    float *GXF = at(ws, bp.offGX), *GWF = at(ws, bp.offGW);
    hd->nk = 0;
    hipError_t e;
    if (!pb.tiled) {
        if ((e = transform(pb, gy, GYF, pb.planesA, pb.hA, pb.wA, next_ctx(hd, "fft.a"))) != hipSuccess) return hip_fail(hd, e);
    } else {
        // gy cut twice: overlapping windows for bprop, disjoint tiles for accGrad
        if (gx && gw && share_forward(pb.N, pb.lay.tsh, pb.hA, pb.planesA, pa.hA, pa.planesA)) {   // as for the two operands of a pass
            FwdOperand ops[2] = {{gy, GYF, pb.planesA, pb.hA, pb.wA, &pb.vA}, {gy, GYFa, pa.planesA, pa.hA, pa.wA, &pa.vA}};
            if ((e = launch_fft2d_r2c_multi(ops, 2, pb.N, next_ctx(hd, "fft.ab"))) != hipSuccess) return hip_fail(hd, e);
        } else {
            if (gx && (e = launch_fft2d_r2c(gy, GYF, pb.planesA, pb.hA, pb.wA, pb.N, true, next_ctx(hd, "fft.a"),
                                            &pb.vA)) != hipSuccess) return hip_fail(hd, e);
            if (gw && (e = launch_fft2d_r2c(gy, GYFa, pa.planesA, pa.hA, pa.wA, pa.N, true, next_ctx(hd, "fft.b"),
                                            &pa.vA)) != hipSuccess) return hip_fail(hd, e);
        }
    }
    // bprop: GX = GY . W ; accGrad: GW = conj(GY) . X  (operand A of both plans is GYF)
    if (gx && gw) {
        const GemmProblem qb = gemm_problem(pb, GYF, WF, GXF), qa = gemm_problem(pa, GYFa, XF, GWF);
        if (cgemm_pair_supported(qb, qa, &hd->sw)) {
            // both contractions in one launch, then the two inverse transforms
            // (the one with the longer reduction first: its workgroups run longest)
            const bool a_first = pa.K >= pb.K;
            if ((e = launch_cgemm_pair(a_first ? qa : qb, a_first ? qb : qa, next_ctx(hd, "contraction.pair"))) != hipSuccess) return hip_fail(hd, e);
            if ((e = invert_pair(hd, pb, GXF, gx, pa, GWF, gw, scale, accumulate)) != hipSuccess) return hip_fail(hd, e);
            return FFTCONV_OK;
        }
    }
    if (gx && (e = contract_and_invert(hd, pb, GYF, WF, GXF, gx, 1.0f, 0)) != hipSuccess) return hip_fail(hd, e);
    if (gw && (e = contract_and_invert(hd, pa, GYFa, XF, GWF, gw, scale, accumulate)) != hipSuccess) return hip_fail(hd, e);
    return FFTCONV_OK;
}

extern "C" {

int fft_conv_fprop_save(fftconv_handle hd, const float *x, const float *wt, float *y,
                        int S, int f, int fo, int h, int w, int kh, int kw,
                        void *saved, size_t saved_bytes, void *ws, size_t ws_bytes) {
    return fprop_save_impl(hd, x, wt, y, S, f, fo, h, w, kh, kw, 0, 0, saved, saved_bytes, ws, ws_bytes);
}

int fft_conv_backward(fftconv_handle hd, const float *gy, float *gx, float *gw,
                      int S, int f, int fo, int h, int w, int kh, int kw,
                      float scale, int accumulate, const void *saved, size_t saved_bytes,
                      void *ws, size_t ws_bytes) {
    return backward_impl(hd, gy, gx, gw, S, f, fo, h, w, kh, kw, 0, 0, scale, accumulate, saved, saved_bytes, ws,
                         ws_bytes);
}

int fft_conv_fprop_save_padded(fftconv_handle hd, const float *x, const float *wt, float *y,
                               int S, int f, int fo, int h, int w, int kh, int kw, int pad_h, int pad_w,
                               void *saved, size_t saved_bytes, void *ws, size_t ws_bytes) {
    return fprop_save_impl(hd, x, wt, y, S, f, fo, h, w, kh, kw, pad_h, pad_w, saved, saved_bytes, ws, ws_bytes);
}

int fft_conv_backward_padded(fftconv_handle hd, const float *gy, float *gx, float *gw,
                             int S, int f, int fo, int h, int w, int kh, int kw, int pad_h, int pad_w,
                             float scale, int accumulate, const void *saved, size_t saved_bytes,
                             void *ws, size_t ws_bytes) {
    return backward_impl(hd, gy, gx, gw, S, f, fo, h, w, kh, kw, pad_h, pad_w, scale, accumulate, saved,
                         saved_bytes, ws, ws_bytes);
}

int fft_conv_fprop_save_tiled(fftconv_handle hd, const float *x, const float *wt, float *y,
                              int S, int f, int fo, int h, int w, int kh, int kw, int tile_n,
                              void *saved, size_t saved_bytes, void *ws, size_t ws_bytes) {
    if (tile_n < 0) return FFTCONV_INVALID_ARG;
    return fprop_save_impl(hd, x, wt, y, S, f, fo, h, w, kh, kw, 0, 0, saved, saved_bytes, ws, ws_bytes, tile_n);
}

int fft_conv_backward_tiled(fftconv_handle hd, const float *gy, float *gx, float *gw,
                            int S, int f, int fo, int h, int w, int kh, int kw, int tile_n,
                            float scale, int accumulate, const void *saved, size_t saved_bytes,
                            void *ws, size_t ws_bytes) {
    if (tile_n < 0) return FFTCONV_INVALID_ARG;
    return backward_impl(hd, gy, gx, gw, S, f, fo, h, w, kh, kw, 0, 0, scale, accumulate, saved, saved_bytes, ws,
                         ws_bytes, tile_n);
}

size_t fftconv_weights_bytes(int f, int fo, int h, int w, int kh, int kw, int pad_h, int pad_w) {
    PassPlan p;
    if (make_plan(FFTCONV_FPROP, 1, f, fo, h, w, kh, kw, &p, -1, pad_h, pad_w) != FFTCONV_OK) return 0;
    return align_up(p.lay.floats(p.planesB) * sizeof(float), 256);
}

int fft_conv_transform_weights(fftconv_handle hd, const float *wt, void *wf, size_t wf_bytes,
                               int f, int fo, int h, int w, int kh, int kw, int pad_h, int pad_w) {
    if (!hd || !wt || !wf) return FFTCONV_INVALID_ARG;
    PassPlan p;
    int rc = cached_plan(hd, FFTCONV_FPROP, 1, f, fo, h, w, kh, kw, &p, -1, pad_h, pad_w);
    if (rc != FFTCONV_OK) return rc;
    if (wf_bytes < align_up(p.lay.floats(p.planesB) * sizeof(float), 256)) return FFTCONV_WORKSPACE_TOO_SMALL;
    hd->nk = 0;
    hipError_t e = transform(p, wt, static_cast<float *>(wf), p.planesB, p.hB, p.wB, next_ctx(hd, "fft.b"));
    return e == hipSuccess ? FFTCONV_OK : hip_fail(hd, e);
}

int fft_conv_fprop_weights(fftconv_handle hd, const float *x, const void *wf, size_t wf_bytes, float *y,
                           int S, int f, int fo, int h, int w, int kh, int kw, int pad_h, int pad_w,
                           void *ws, size_t ws_bytes) {
    return run_pass_weights(hd, FFTCONV_FPROP, x, wf, wf_bytes, y, S, f, fo, h, w, kh, kw, pad_h, pad_w, ws, ws_bytes);
}

int fft_conv_bprop_weights(fftconv_handle hd, const float *gy, const void *wf, size_t wf_bytes, float *gx,
                           int S, int f, int fo, int h, int w, int kh, int kw, int pad_h, int pad_w,
                           void *ws, size_t ws_bytes) {
    return run_pass_weights(hd, FFTCONV_BPROP, gy, wf, wf_bytes, gx, S, f, fo, h, w, kh, kw, pad_h, pad_w, ws, ws_bytes);
}

int fft_conv_fprop_fused(fftconv_handle hd, const float *x, const void *wf, size_t wf_bytes, float *y,
                         int S, int f, int fo, int h, int w, int kh, int kw) {
    if (!hd || !x || !wf || !y) return FFTCONV_INVALID_ARG;
    PassPlan p;
    int rc = cached_plan(hd, FFTCONV_FPROP, S, f, fo, h, w, kh, kw, &p);
    if (rc != FFTCONV_OK) return rc;
    if (wf_bytes < align_up(p.lay.floats(p.planesB) * sizeof(float), 256)) return FFTCONV_WORKSPACE_TOO_SMALL;
    if (p.tiled || p.rect || !fused_fprop_supported(p.N, f, fo, static_cast<const float *>(wf))) return FFTCONV_UNSUPPORTED;
    hd->nk = 0;
    const hipError_t e = launch_fused_fprop(x, static_cast<const float *>(wf), y, S, f, fo, h, w, kh, kw, p.N, next_ctx(hd, "fused"));
    if (e == hipErrorInvalidValue) return FFTCONV_UNSUPPORTED;   // the layer's planes do not fit the kernel's LDS plan
    return e == hipSuccess ? FFTCONV_OK : hip_fail(hd, e);
}

int fft_conv_bprop_fused(fftconv_handle hd, const float *gy, const void *wf, size_t wf_bytes, float *gx,
                         int S, int f, int fo, int h, int w, int kh, int kw) {
    if (!hd || !gy || !wf || !gx) return FFTCONV_INVALID_ARG;
    PassPlan p;
    int rc = cached_plan(hd, FFTCONV_BPROP, S, f, fo, h, w, kh, kw, &p);
    if (rc != FFTCONV_OK) return rc;
    if (wf_bytes < align_up(p.lay.floats(p.planesB) * sizeof(float), 256)) return FFTCONV_WORKSPACE_TOO_SMALL;
    if (p.tiled || p.rect || !fused_bprop_supported(p.N, f, fo, static_cast<const float *>(wf))) return FFTCONV_UNSUPPORTED;
    hd->nk = 0;
    const hipError_t e = launch_fused_bprop(gy, static_cast<const float *>(wf), gx, S, f, fo, h, w, kh, kw, p.N, next_ctx(hd, "fused"));
    if (e == hipErrorInvalidValue) return FFTCONV_UNSUPPORTED;   // the layer's planes do not fit the kernel's LDS plan
    return e == hipSuccess ? FFTCONV_OK : hip_fail(hd, e);
}

int fft_conv_accgrad_fused(fftconv_handle hd, const float *x, const float *gy, float *gw,
                           int S, int f, int fo, int h, int w, int kh, int kw, float scale, int accumulate) {
    if (!hd || !gy || !x || !gw) return FFTCONV_INVALID_ARG;
    PassPlan p;
    int rc = cached_plan(hd, FFTCONV_ACCGRAD, S, f, fo, h, w, kh, kw, &p);
    if (rc != FFTCONV_OK) return rc;
    if (p.tiled || p.rect || !fused_accgrad_supported(p.N, S, f, fo)) return FFTCONV_UNSUPPORTED;
    hd->nk = 0;
    const hipError_t e = launch_fused_accgrad(gy, x, gw, S, f, fo, h, w, kh, kw, p.N, scale, accumulate, next_ctx(hd, "fused"));
    if (e == hipErrorInvalidValue) return FFTCONV_UNSUPPORTED;   // the layer's planes do not fit the kernel's LDS plan
    return e == hipSuccess ? FFTCONV_OK : hip_fail(hd, e);
}

}  // extern "C"
