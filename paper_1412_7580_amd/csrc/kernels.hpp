// Internal launch interface between the C ABI (api.hip) and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>

namespace fc {

// Where a kernel is launched and, optionally, a pair of events that the runtime attaches to
// that one dispatch (their elapsed time is the kernel's own execution time, without the gaps
// that events recorded between launches would include).
// Switches of the contraction for A/B runs (environment variables FFTCONV_GEMM_TILE, _NO_TAIL,
// _NO_PAIR, _NO_BINGROUP, _NO_FAST and FFTCONV_BG_TILE), read once when a handle is created; none
// changes a result beyond rounding.  All off by default.
struct GemmSwitches {
    int tile = -1;          // 0..5: another tile shape, single kernels only; -1: the default
    bool no_tail = false, no_pair = false, no_bingroup = false, no_fast = false;
    int bg_tile = 0;        // per-wave tile of the four-bins-per-line kernel
};
GemmSwitches read_gemm_switches();

struct LaunchCtx {
    hipStream_t stream;
    hipEvent_t start, stop;
    const GemmSwitches *sw = nullptr;   // contraction launches: the handle's switches (nullptr: defaults)
};

template <class K, class P>
inline void launch_kernel(K kernel, dim3 grid, dim3 block, size_t lds, const LaunchCtx &lc, const P &prm) {
    if (lc.start || lc.stop) hipExtLaunchKernelGGL(kernel, grid, block, (unsigned)lds, lc.stream, lc.start, lc.stop, 0, prm);
    else hipLaunchKernelGGL(kernel, grid, block, lds, lc.stream, prm);
}

// Raise a kernel's dynamic-LDS limit when it needs more than the default 64 KB.  The runtime
// call is made once per kernel function and size class (the largest request so far is kept),
// not on every launch.
hipError_t allow_big_lds(const void *fn, size_t bytes);

// Private frequency-domain layout used between the FFT stages and the contraction
// ("plane-tiled, bin-major, planar"):
//     F[plane / T][bin][c][plane % T],   bin = k1 * (N/2+1) + k2,  c = 0 real, 1 imaginary
// T (a power of two) is the number of consecutive planes one FFT workgroup transforms, so
// every workgroup writes one contiguous block and, for one bin, a run of T floats.  The
// contraction gathers such runs.  This plays the role of the paper's HWBD tensors of Table 1
// without ever materialising the BDHW frequency tensors or the three transposes.
struct FreqLayout {
    int tsh;    // log2(T)
    int bins;   // bin stride of a plane tile: N * (N/2 + 1) rounded up to a multiple of 8
    __host__ __device__ size_t index(long plane, int bin, int c) const {
        const long pt = plane >> tsh;
        const long pl = plane & ((1L << tsh) - 1);
        return (size_t)((((pt * bins + bin) * 2 + c) << tsh) + pl);
    }
    // Offset of plane x relative to plane 0 for a fixed bin and component.  For x = a + b with
    // no carry out of the low tsh bits of a and b (e.g. a a multiple of the tile, or both below
    // it with a + b below it too), part(a + b) = part(a) + part(b).
    __host__ __device__ size_t part(int x) const {
        return ((size_t)(x >> tsh) * bins * 2 << tsh) + (size_t)(x & ((1 << tsh) - 1));
    }
    size_t floats(long planes) const {
        const long T = 1L << tsh;
        return (size_t)((planes + T - 1) / T) * T * bins * 2;
    }
};

// How the planes of a tiled operand map to memory (tiling of large inputs into small
// transforms, Section 6 of the paper).  Plane p = (sample-tile m, channel p % C) with
// m = (s * nty + ty) * ntx + tx, and the plane's data is a window of image (s, channel):
//   forward: rows ty*dy + oy ... of H, columns tx*dx + ox ... of W; elements outside the
//            image read as 0 (the origin may be negative);
//   inverse: rows oy ... and columns ox ... of the transform's output go to rows ty*dy ...
//            and columns tx*dx ... of the image; elements outside the image are dropped.
struct PlaneView {
    int C;
    int nty, ntx;
    int dy, dx;
    int oy, ox;
    int H, W;
    int Cimg = 0;   // channels per sample of the image tensor when the view selects C of them (0: C)
};

// Planes per workgroup (= layout tile) of the 2-D kernels for basis N.
int fft2d_tile_log2(int N);
// Bins per plane tile of the layout for basis N: N * (N/2 + 1) rounded up to a multiple of 8 (of
// 32 for the bases with runs of 4 planes), so that the contraction can always cut the bins into
// equal chunks per XCD (and whole 128-byte lines).  The padding bins, which only bases with an
// odd factor have, are never written by the transforms nor read by the inverse; the
// contraction multiplies whatever they hold into the padding bins of its output.
int fft2d_layout_bins(int N);

// 2-D R2C of `planes` planes [h_in x w_in] zero-padded to N x N.
//   conv layout: out = FreqLayout buffer (tile = fft2d_tile_log2(N)).
//   natural layout: out = [planes][N][N/2+1][2].
// With a view, `in` is the image tensor and h_in x w_in the window size.
hipError_t launch_fft2d_r2c(const float *in, float *out, long planes, int h_in, int w_in, int N,
                            bool conv_layout, LaunchCtx st, const PlaneView *view = nullptr);

// The same transform of up to three operand tensors (plane-tiled layout) in ONE launch.
struct FwdOperand {
    const float *in;
    float *out;
    long planes;
    int h_in, w_in;
    const PlaneView *view = nullptr;
};
hipError_t launch_fft2d_r2c_multi(const FwdOperand *ops, int nops, int N, LaunchCtx st);

// The same on a rectangular basis nr x nc (nr rows, nc columns; both at most 32 and different),
// plane-tiled layout only, whole planes only (no windows).  The layout then has
// bin = k1 * (nc/2+1) + k2 with the tile and bin count given by these functions.
bool fft2d_rect_supported(int nr, int nc);
int fft2d_rect_tile_log2(int nr, int nc);
int fft2d_rect_layout_bins(int nr, int nc);
hipError_t launch_fft2d_r2c_rect(const FwdOperand *ops, int nops, int nr, int nc, LaunchCtx st);   // nops 1 or 2
hipError_t launch_fft2d_c2r_rect(const float *in, float *out, long planes, int nr, int nc, int h_out, int w_out,
                                 float scale, bool accumulate, LaunchCtx st);

// 2-D C2R + crop.  out[planes][h_out][w_out] = scale * real inverse (the caller folds 1/N^2
// into `scale`), added to the previous contents when accumulate is set.
// With a view (plane-tiled layout only), `out` is the image tensor and h_out x w_out the size
// of the window taken from each transform at offset (view->oy, view->ox).
hipError_t launch_fft2d_c2r(const float *in, float *out, long planes, int N, int h_out, int w_out,
                            bool conv_layout, float scale, bool accumulate, LaunchCtx st,
                            const PlaneView *view = nullptr);

// Two inverse transforms of the plane-tiled layout in ONE launch (the two products of the
// backward pass), for the bases up to 32.  hipErrorNotSupported for the others: the caller then
// launches them one after the other.
struct InvOperand {
    const float *in;
    float *out;
    long planes;
    int h_out, w_out;
    float scale;
    bool accumulate;
    const PlaneView *view = nullptr;
};
hipError_t launch_fft2d_c2r_pair(const InvOperand *ops, int N, LaunchCtx st);
// The same on a rectangular basis (whole planes only).
hipError_t launch_fft2d_c2r_rect_pair(const InvOperand *ops, int nr, int nc, LaunchCtx st);

// One-launch fprop of a small layer (basis N <= 16, f and f' within one plane tile): one
// workgroup per sample; wf is the weight transform in the layout of basis N.
bool fused_fprop_supported(int N, int f, int fo, const float *wf);
hipError_t launch_fused_fprop(const float *x, const float *wf, float *y, int S, int f, int fo, int h, int w,
                              int kh, int kw, int N, LaunchCtx st);

// bprop likewise (GX_i = sum_j GY_j . W_ji): one workgroup per sample, same support rule.
bool fused_bprop_supported(int N, int f, int fo, const float *wf);
hipError_t launch_fused_bprop(const float *gy, const float *wf, float *gx, int S, int f, int fo, int h, int w,
                              int kh, int kw, int N, LaunchCtx st);

// One-launch accGrad of a small layer (basis N <= 16, all S samples of a block of output and input
// channels within one plane tile): one workgroup per block of (j, i) pairs, which transforms the
// planes of gy and x it needs itself, reduces over the samples and inverts its own products.
bool fused_accgrad_supported(int N, int S, int f, int fo);
bool fused_accgrad_pays(int N, int S, int f, int fo);     // ... and measured faster than three launches
hipError_t launch_fused_accgrad(const float *gy, const float *x, float *gw, int S, int f, int fo, int h, int w,
                                int kh, int kw, int N, float scale, int accumulate, LaunchCtx st);

hipError_t launch_fft1d_r2c(const float *in, float *out, long B, int n_in, int n, LaunchCtx st);
hipError_t launch_fft1d_c2r(const float *in, float *out, long B, int n, int n_out, LaunchCtx st);

// Per-bin complex contraction  C[b](m,n) = sum_k A'[b](m,k) * B'[b](k,n)  over all bins, where
// X' is X or its complex conjugate.  Operand element (row r, col c) of X lives at plane
// r * X_rs + c * X_cs  of its layout.
struct GemmOperand {
    const float *ptr;
    FreqLayout lay;
    long rs, cs;       // plane strides of the (row, col) indices
    bool conj;         // use the complex conjugate of the stored values
};
hipError_t launch_cgemm_bins(GemmOperand A, GemmOperand B, float *C, FreqLayout layC, long C_rs,
                             long C_cs, int M, int N, int K, int bins, LaunchCtx st);

// Two independent contractions in one launch (see cgemm_pair_kernel).  Possible when both
// can use 16-byte gathers and neither is a case for the four-bins-per-line kernel.
struct GemmProblem {
    GemmOperand A, B;
    float *C;
    FreqLayout layC;
    long C_rs, C_cs;
    int M, N, K, bins;
};
bool cgemm_pair_supported(const GemmProblem &g1, const GemmProblem &g2, const GemmSwitches *sw = nullptr);
hipError_t launch_cgemm_pair(const GemmProblem &g1, const GemmProblem &g2, LaunchCtx st);

}  // namespace fc
