/*
 * fftconv -- frequency-domain convolution for CNN layers on AMD gfx950 (MI355X).
 *
 * C ABI of the hot path of "Fast Convolutional Nets With fbfft" (arXiv 1412.7580):
 * the three convolution passes of Section 2 computed as in Section 3.1 / Table 1
 * (2-D real FFT of both zero-padded operands -> per-frequency complex product that
 * reduces over planes -> inverse FFT clipped to the valid region), plus the batched
 * small 1-D / 2-D real FFTs of Section 5 as stand-alone calls.
 *
 * Conventions common to every call
 *  - All tensor pointers are DEVICE pointers to dense, row-major fp32 memory owned by
 *    the caller ("BDHW", innermost = image row, Section 3.1).  Inputs are never
 *    modified; outputs are fully overwritten (except fft_conv_accgrad with
 *    accumulate != 0).  Input and output ranges must not overlap.
 *  - Work is enqueued on the handle's stream and the call returns without waiting for
 *    it.  A handle must not be used from two threads at once, nor may two of its calls
 *    overlap on different streams: the frequency-domain buffers are one reused set per
 *    handle (the buffer policy of Section 3.3).
 *  - Every function returns an fftconv_status; arguments are validated before anything
 *    is launched, so on an error other than FFTCONV_HIP_ERROR no device work was issued.
 *  - The Fourier basis is the smallest supported size that holds the image (8 ... 128: the
 *    powers of two of the paper's 2-D kernels, Section 5.3, and sizes 2^a x {3, 5, 7, 9} between
 *    them), square, or rectangular (each side on its own size) when both sides are at most
 *    32 and differ.  Layers that would need a larger basis, and layers for which it is
 *    clearly cheaper, are tiled (Section 6): the passes then run on windows of the images
 *    with a small basis, with identical results.  fftconv_layer_basis() tells which.
 */
#ifndef FFTCONV_H
#define FFTCONV_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fftconv_ctx *fftconv_handle;

typedef enum {
    FFTCONV_OK = 0,
    FFTCONV_INVALID_ARG = 1,         /* null pointer, non-positive size, kernel larger than input, n_in > n ... */
    FFTCONV_UNSUPPORTED = 2,         /* transform size that is not one of the bases; kernel larger than 128 */
    FFTCONV_WORKSPACE_TOO_SMALL = 3, /* caller-supplied workspace smaller than fftconv_workspace_bytes() */
    FFTCONV_HIP_ERROR = 4,           /* allocation or launch failure reported by the HIP runtime */
    FFTCONV_STATIC_SCRATCH_EXCEEDED = 5 /* fft_conv_fprop_static: the layer needs more than fftconv_static_scratch_bytes() */
} fftconv_status;

enum { FFTCONV_FPROP = 0, FFTCONV_BPROP = 1, FFTCONV_ACCGRAD = 2 };

/* Create a handle bound to HIP device `device` (made current for the call).  The handle
 * starts on the null stream and owns no workspace until one is needed. */
int fftconv_create(fftconv_handle *out, int device);
/* Free the handle and any workspace it owns.  Pending work must have completed. */
int fftconv_destroy(fftconv_handle h);
/* `stream` is a hipStream_t passed as void*; NULL selects the null stream. */
int fftconv_set_stream(fftconv_handle h, void *stream);
const char *fftconv_status_string(int status);

/* The basis the ordinary (and padded, saved-transform and weights-ahead) entry points use for a
 * layer: *n_rows x *n_cols (equal unless rectangular).  Returns 0 when the layer runs whole on
 * that basis, 1 when it is tiled with that basis, and a negative fftconv_status for invalid
 * or unsupported shapes.  Host only. */
int fftconv_layer_basis(int h, int w, int kh, int kw, int pad_h, int pad_w, int *n_rows, int *n_cols);

/* Bytes of device scratch one pass needs: the three frequency-domain tensors of Table 1
 * (both operands and the product), Hermitian half, complex fp32, in the library's private
 * bin-major layout.  Returns 0 for invalid or unsupported shapes. */
size_t fftconv_workspace_bytes(int pass, int S, int f, int fo, int h, int w, int kh, int kw);

/*
 * The three passes (Section 2; pipeline of Table 1; clipping sizes of Section 3.1).
 *   S minibatch, f input planes, fo output planes (f'), h x w input, kh x kw kernel,
 *   oh = h-kh+1, ow = w-kw+1.  Stride 1, no margin padding (Section 2 excludes strides).
 * Fourier basis: the smallest of 8, 10, 12, 14, 16, 18, 20, 24, 28, 32, 36, 40, 48, 56, 64 that
 * holds the image (the powers of two of Section 5 and, between them, sizes 2^a x {3, 5, 7, 9} of
 * the search space of Section 3.4); larger images are tiled (see the tiled passes below).  The
 * basis is square, N x N with N chosen for max(h, w), except that an image whose sides both
 * fit 32 and call for different sizes gets a rectangular basis N_h x N_w, each side the
 * smallest size that holds it (Section 3.1 only asks that every operand fit the common
 * basis).  The same basis serves all three passes of a layer.
 * `ws`/`ws_bytes`: optional caller-owned device scratch of at least
 * fftconv_workspace_bytes(); with ws == NULL the handle grows and reuses its own buffer
 * (hipMalloc on first use or growth only; growth waits for the stream first).  While the
 * handle's stream is being captured into a graph the buffer cannot grow: a call that would need
 * to returns FFTCONV_WORKSPACE_TOO_SMALL (pass a workspace, or make one eager call first).
 */

/* fprop: y(s,j) = sum_i x(s,i) (star) w(j,i)  -- valid cross-correlation.
 * x[S,f,h,w], wt[fo,f,kh,kw] -> y[S,fo,oh,ow]. */
int fft_conv_fprop(fftconv_handle hd, const float *x, const float *wt, float *y,
                   int S, int f, int fo, int h, int w, int kh, int kw,
                   void *ws, size_t ws_bytes);

/*
 * fprop for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, result and kernels as
 * fft_conv_fprop, but the three frequency-domain tensors live in an array that is part of the
 * library's device code (32 MiB, fftconv_static_scratch_bytes(); every GPU the library runs on
 * holds one copy until the process ends) instead of a workspace: the call makes no allocation
 * of any kind.  A layer whose fprop needs more (fftconv_workspace_bytes(FFTCONV_FPROP, ...) above
 * that size) gives FFTCONV_STATIC_SCRATCH_EXCEEDED and nothing is launched; other errors as for
 * fft_conv_fprop.  All calls on one GPU, from every handle, share that GPU's array: two such
 * calls that overlap in time on one GPU (different streams or handles) race and give wrong
 * results; calls that follow each other on one stream are fine, and nothing of the array has
 * to be cleared between them (every element a call reads, it has written before).
 */
size_t fftconv_static_scratch_bytes(void);
int fft_conv_fprop_static(fftconv_handle hd, const float *x, const float *wt, float *y,
                          int S, int f, int fo, int h, int w, int kh, int kw);

/* bprop: dL/dx(s,i) = sum_j dL/dy(s,j) * w(j,i)  -- full convolution, reduces over fo.
 * gy[S,fo,oh,ow], wt[fo,f,kh,kw] -> gx[S,f,h,w]. */
int fft_conv_bprop(fftconv_handle hd, const float *gy, const float *wt, float *gx,
                   int S, int f, int fo, int h, int w, int kh, int kw,
                   void *ws, size_t ws_bytes);

/* accGrad: dL/dw(j,i) = sum_s dL/dy(s,j) (star) x(s,i)  -- reduces over the minibatch.
 * x[S,f,h,w], gy[S,fo,oh,ow] -> gw[fo,f,kh,kw] = scale * result (+ previous gw if
 * accumulate != 0).  Layers of few samples or very small images (those fft_conv_accgrad_fused
 * supports, with samples x frequency bins up to 900) run as one launch by themselves and then
 * touch no workspace. */
int fft_conv_accgrad(fftconv_handle hd, const float *x, const float *gy, float *gw,
                     int S, int f, int fo, int h, int w, int kh, int kw,
                     float scale, int accumulate, void *ws, size_t ws_bytes);

/*
 * Tiled passes (the tiling strategy of Section 6).  An output tile of d rows needs d + kh - 1
 * input rows, so a large convolution splits into many small ones on a basis of
 * tile_n = d + kh - 1 (columns alike): fprop and bprop by overlapping input windows, accGrad
 * by summing the per-tile correlations, the tile index joining the minibatch index in the
 * reduction.  Results equal those of the untiled calls up to rounding.  tile_n is one of the
 * bases 8, 10, 12, 14, 16, 18, 20, 24, 28, 32, 36, 40, 48, 56, 64, 80, 96, 112, 128, at least
 * max(kh, kw); 0 lets the library choose (the basis with the lowest estimated cost: tiles x bins per tile x a
 * measured per-basis factor).  A tile_n that holds the whole image (tile_n >= max(h, w)) runs
 * the untiled pipeline at that basis: this is how a caller names the Fourier basis of a layer.
 * The entry points above tile by themselves, with the library's choice, when max(h, w) > 128
 * and when the estimate is clearly below that of the untiled basis (in practice: layers whose
 * untiled basis is 80 or more).  Arguments, layouts and errors as for the untiled calls;
 * tile_n < 0, not a basis or smaller than the kernel gives FFTCONV_INVALID_ARG.
 */
size_t fftconv_tiled_workspace_bytes(int pass, int S, int f, int fo, int h, int w, int kh, int kw, int tile_n);
/* The basis a tiled call with this tile_n uses (host only; 0 for invalid arguments). */
int fftconv_tile_basis(int h, int w, int kh, int kw, int tile_n);
int fft_conv_fprop_tiled(fftconv_handle hd, const float *x, const float *wt, float *y,
                         int S, int f, int fo, int h, int w, int kh, int kw, int tile_n,
                         void *ws, size_t ws_bytes);
int fft_conv_bprop_tiled(fftconv_handle hd, const float *gy, const float *wt, float *gx,
                         int S, int f, int fo, int h, int w, int kh, int kw, int tile_n,
                         void *ws, size_t ws_bytes);
int fft_conv_accgrad_tiled(fftconv_handle hd, const float *x, const float *gy, float *gw,
                           int S, int f, int fo, int h, int w, int kh, int kw,
                           float scale, int accumulate, int tile_n, void *ws, size_t ws_bytes);

/*
 * Basis selection by measurement (the strategy selection of Section 3.4, here over the Fourier
 * basis alone): runs fprop, bprop and accGrad of the layer at every basis that holds the
 * kernel and whose estimated cost is within 3x of the lowest estimate, `reps` times each after
 * one untimed run, and returns the basis with the shortest time for the three passes in
 * *basis_out, for use as tile_n of the calls above (the caller caches it per layer shape).
 * *ms_out, if not NULL, receives that time in milliseconds.  x, wt, gy are the layer's
 * operands (device, read only); y, gx, gw (device) are overwritten and hold the chosen basis's
 * results on return.  Uses the handle's own workspace, which grows to the largest candidate's
 * need.  Synchronous: returns after the last run has finished.  Errors as for the passes;
 * reps <= 0 or a NULL pointer other than ms_out gives FFTCONV_INVALID_ARG.  The candidates are
 * the square bases; for a non-square image whose sides both fit 32 the ordinary entry points
 * use a rectangular basis (see fftconv_layer_basis), which is not among them and is usually
 * the faster choice there.
 */
int fftconv_autotune_basis(fftconv_handle hd, const float *x, const float *wt, const float *gy,
                           float *y, float *gx, float *gw, int S, int f, int fo, int h, int w, int kh, int kw,
                           int reps, int *basis_out, float *ms_out);

/*
 * The plan of one pass as numbers (host only; for tests of the planner, which check on the CPU
 * that the windows, crops and buffer offsets of every layer shape stay inside their tensors and
 * that a plain re-enactment of the plan gives the convolution).  tile_n: -1 as the ordinary
 * entry points choose, else as for the tiled passes.  Writes min(cap, count) values to out and
 * returns count (61), or a negative fftconv_status.  Values, in order: basis rows, basis
 * columns, tiled, rectangular, bins per plane tile of the layout, log2(planes per layout tile);
 * planes of operand A, operand B, product C; window / crop sizes hA, wA, hB, wB, hC, wC;
 * contraction sizes M, N, K; conjugate A, conjugate B; plane strides of A(m,k): row, column, of
 * B(k,n), of C(m,n); workspace offsets of A, B, C and total bytes; bytes of A's buffer; then for
 * A, B and C ten values each: is a window view, channels, tiles down, tiles across, tile step
 * rows, columns, window offset rows, columns, image rows, columns.
 */
int fftconv_describe_plan(int pass, int S, int f, int fo, int h, int w, int kh, int kw, int tile_n,
                          int pad_h, int pad_w, long *out, int cap);

/*
 * Passes of a layer whose input images are surrounded by pad_h rows and pad_w columns of zeros
 * on every side (the p_h, p_w of Section 2).  No padded copy of x is made: the padding is the
 * part of a window that falls outside the image (the implicit zero padding of Section 5.1).
 * x[S,f,h,w] and gx keep their unpadded shape; y and gy are
 * [S,fo,h+2pad_h-kh+1,w+2pad_w-kw+1].  With pad_h = pad_w = 0 these are the ordinary passes.
 * Negative padding or a kernel larger than the padded image gives FFTCONV_INVALID_ARG.
 */
size_t fftconv_padded_workspace_bytes(int pass, int S, int f, int fo, int h, int w, int kh, int kw,
                                      int pad_h, int pad_w);
int fft_conv_fprop_padded(fftconv_handle hd, const float *x, const float *wt, float *y,
                          int S, int f, int fo, int h, int w, int kh, int kw, int pad_h, int pad_w,
                          void *ws, size_t ws_bytes);
int fft_conv_bprop_padded(fftconv_handle hd, const float *gy, const float *wt, float *gx,
                          int S, int f, int fo, int h, int w, int kh, int kw, int pad_h, int pad_w,
                          void *ws, size_t ws_bytes);
int fft_conv_accgrad_padded(fftconv_handle hd, const float *x, const float *gy, float *gw,
                            int S, int f, int fo, int h, int w, int kh, int kw, int pad_h, int pad_w,
                            float scale, int accumulate, void *ws, size_t ws_bytes);
/* The transform-reuse pair (see fft_conv_fprop_save / fft_conv_backward below) for a padded
 * layer; the same padding must be given to all four functions. */
size_t fftconv_saved_bytes_padded(int S, int f, int fo, int h, int w, int kh, int kw, int pad_h, int pad_w);
size_t fftconv_backward_workspace_bytes_padded(int S, int f, int fo, int h, int w, int kh, int kw,
                                               int pad_h, int pad_w);
int fft_conv_fprop_save_padded(fftconv_handle hd, const float *x, const float *wt, float *y,
                               int S, int f, int fo, int h, int w, int kh, int kw, int pad_h, int pad_w,
                               void *saved, size_t saved_bytes, void *ws, size_t ws_bytes);
int fft_conv_backward_padded(fftconv_handle hd, const float *gy, float *gx, float *gw,
                             int S, int f, int fo, int h, int w, int kh, int kw, int pad_h, int pad_w,
                             float scale, int accumulate, const void *saved, size_t saved_bytes,
                             void *ws, size_t ws_bytes);
/* The transform-reuse pair on a named basis (tile_n as for the tiled passes, e.g. the result
 * of fftconv_autotune_basis); the same tile_n must be given to all four functions. */
size_t fftconv_saved_bytes_tiled(int S, int f, int fo, int h, int w, int kh, int kw, int tile_n);
size_t fftconv_backward_workspace_bytes_tiled(int S, int f, int fo, int h, int w, int kh, int kw, int tile_n);
int fft_conv_fprop_save_tiled(fftconv_handle hd, const float *x, const float *wt, float *y,
                              int S, int f, int fo, int h, int w, int kh, int kw, int tile_n,
                              void *saved, size_t saved_bytes, void *ws, size_t ws_bytes);
int fft_conv_backward_tiled(fftconv_handle hd, const float *gy, float *gx, float *gw,
                            int S, int f, int fo, int h, int w, int kh, int kw, int tile_n,
                            float scale, int accumulate, const void *saved, size_t saved_bytes,
                            void *ws, size_t ws_bytes);

/*
 * Weights transformed ahead of the passes that use them (the second opportunity Section 6
 * lists and forgoes: precomputing the FFTs of the weight tensors; once per optimiser step in
 * training, once for all in inference).  fft_conv_transform_weights leaves the transform of
 * wt[fo,f,kh,kw] for a layer of h x w images (padded by pad_h, pad_w; 0 for none) in the caller's
 * device buffer wf of at least fftconv_weights_bytes() bytes (contents private; valid for
 * every minibatch size).  fft_conv_fprop_weights / fft_conv_bprop_weights then equal
 * fft_conv_fprop(_padded) / fft_conv_bprop(_padded) with one forward transform instead of two.
 * The transform may run on another handle and stream than the passes (the caller orders
 * them).  Workspace as for the ordinary passes; a short wf gives FFTCONV_WORKSPACE_TOO_SMALL.
 * Small layers (those fft_conv_fprop_fused / fft_conv_bprop_fused support, up to 512 samples)
 * run as one launch by themselves and then touch no workspace.
 */
size_t fftconv_weights_bytes(int f, int fo, int h, int w, int kh, int kw, int pad_h, int pad_w);
int fft_conv_transform_weights(fftconv_handle hd, const float *wt, void *wf, size_t wf_bytes,
                               int f, int fo, int h, int w, int kh, int kw, int pad_h, int pad_w);
int fft_conv_fprop_weights(fftconv_handle hd, const float *x, const void *wf, size_t wf_bytes, float *y,
                           int S, int f, int fo, int h, int w, int kh, int kw, int pad_h, int pad_w,
                           void *ws, size_t ws_bytes);
int fft_conv_bprop_weights(fftconv_handle hd, const float *gy, const void *wf, size_t wf_bytes, float *gx,
                           int S, int f, int fo, int h, int w, int kh, int kw, int pad_h, int pad_w,
                           void *ws, size_t ws_bytes);

/*
 * fprop of a small layer in ONE launch, on weights transformed ahead (wf from
 * fft_conv_transform_weights with pad 0): for the latency-bound regime, where the three launches
 * of fft_conv_fprop_weights cost more than the arithmetic (Section 6 plans such an integration
 * of the matrix product with the transform kernels).  One workgroup carries one sample through
 * transform, contraction and inverse; it needs no workspace.  Same result as fft_conv_fprop up
 * to rounding.  Supported when the layer's basis is square and at most 16 (unpadded images),
 * f is a multiple of 4 that divides 32 (64 at basis 8), fo <= 32 (64) and
 * bins x f x fo <= 40000 (bins = N (N/2 + 1) of the layer's basis N; e.g. 16 x 16 planes at
 * basis 14 or 16): otherwise FFTCONV_UNSUPPORTED, and the caller uses fft_conv_fprop_weights.
 */
int fft_conv_fprop_fused(fftconv_handle hd, const float *x, const void *wf, size_t wf_bytes, float *y,
                         int S, int f, int fo, int h, int w, int kh, int kw);

/*
 * bprop of a small layer in ONE launch, the counterpart of fft_conv_fprop_fused (same weights
 * buffer wf, same support rule with the same f and fo, same error behaviour): one workgroup
 * carries one sample's fo gradient planes gy through transform, product GX_i = sum_j GY_j . W_ji
 * and inverse with crop to h x w.  gy [S, fo, h-kh+1, w-kw+1] (device, read only), gx
 * [S, f, h, w] (device, overwritten).  Same result as fft_conv_bprop up to rounding.
 */
int fft_conv_bprop_fused(fftconv_handle hd, const float *gy, const void *wf, size_t wf_bytes, float *gx,
                         int S, int f, int fo, int h, int w, int kh, int kw);

/*
 * accGrad of a small layer in ONE launch (Section 6's planned integration of the product with
 * the transforms, for the pass that reduces over the samples).  The launch has no dependence
 * between workgroups: each owns a block of output channels and a block of input channels,
 * transforms the planes of gy and x of those channels for all S samples itself, sums
 * conj(GY_sj) . X_si over the samples per frequency and inverts its own products with the crop to
 * kh x kw; a plane is therefore transformed by several workgroups.  Arguments, scale and
 * accumulate as for fft_conv_accgrad; same result up to rounding; no workspace.  Supported for
 * untiled, unpadded layers on a square basis of at most 16 with at most 32 samples (64 on basis
 * 8) and at most 256 channel blocks: otherwise FFTCONV_UNSUPPORTED, and the caller uses
 * fft_conv_accgrad.
 */
int fft_conv_accgrad_fused(fftconv_handle hd, const float *x, const float *gy, float *gw,
                           int S, int f, int fo, int h, int w, int kh, int kw, float scale, int accumulate);

/*
 * Stand-alone batched real FFTs (Section 5).  X_k = sum_j x_j exp(-2 pi i jk/n)
 * (Supplement, DFT definition); n is a power of two in 2..128 (256 for the 1-D calls: the
 * sizes of Section 5.3) or one of 10, 12, 14, 18, 20, 24, 28, 36, 40, 48, 56, 80, 96, 112 (and
 * 160, 192, 224 for the 1-D calls): 2^a x {3, 5, 7, 9}, sizes Section 3.2 takes from cuFFT; any other n
 * gives FFTCONV_UNSUPPORTED.  Inputs shorter than n are
 * zero-padded implicitly while loading (the clipping of Section 5.1), no padded copy is
 * made.  Complex data are interleaved (re,im) fp32; only the Hermitian half
 * k = 0..n/2 along the innermost axis is stored (Table 1), in natural bin order.
 * The inverse calls are true inverses (scaled by 1/n per dimension) that keep the first
 * n_out (h_out x w_out) samples.  Their input must be the transform of a real signal.  In
 * 1-D that constrains only bins 0 and n/2, whose imaginary parts are not looked at.  In 2-D the
 * two self-conjugate columns k2 = 0 and k2 = n/2 must be Hermitian along the other axis,
 * X[k1][k2] = conj(X[(n - k1) % n][k2]) (every transform of real data, and every product of such
 * transforms, is); the inverse relies on it, and for input without that symmetry the result is
 * unspecified (no error is reported).  Columns 0 < k2 < n/2 are unconstrained.  B = 0 is a
 * no-op that returns FFTCONV_OK (pointers may then be NULL).
 */
/* in[B,n_in] -> out[B,n/2+1,2];  1 <= n_in <= n. */
int fft_r2c_1d(fftconv_handle hd, const float *in, float *out, long B, int n_in, int n);
/* in[B,n/2+1,2] -> out[B,n_out];  1 <= n_out <= n. */
int fft_c2r_1d(fftconv_handle hd, const float *in, float *out, long B, int n, int n_out);
/* in[B,h_in,w_in] -> out[B,n,n/2+1,2]. */
int fft_r2c_2d(fftconv_handle hd, const float *in, float *out, long B, int h_in, int w_in, int n);
/* in[B,n,n/2+1,2] -> out[B,h_out,w_out]. */
int fft_c2r_2d(fftconv_handle hd, const float *in, float *out, long B, int n, int h_out, int w_out);

/*
 * Reuse of transforms between the passes of one layer (the first of the two opportunities
 * Section 6 of the paper lists and forgoes for lack of memory: keeping transforms that a
 * layer's passes share).  fft_conv_fprop_save computes the same y as fft_conv_fprop and leaves the
 * transforms of x and wt in the caller's `saved` buffer (device memory, at least
 * fftconv_saved_bytes(), contents private).  fft_conv_backward then computes gx (as
 * fft_conv_bprop) and gw (as fft_conv_accgrad, with scale / accumulate) from gy and that
 * buffer, transforming gy once: three forward transforms per layer and step instead of six.
 * Either of gx, gw may be NULL to skip that half.  `saved` must come from
 * fft_conv_fprop_save with the same shape arguments and x, wt unchanged since.
 * `ws` as for the passes; sizes: fftconv_workspace_bytes(FFTCONV_FPROP, ...) is enough for
 * fft_conv_fprop_save, fftconv_backward_workspace_bytes() for fft_conv_backward.
 */
size_t fftconv_saved_bytes(int S, int f, int fo, int h, int w, int kh, int kw);
size_t fftconv_backward_workspace_bytes(int S, int f, int fo, int h, int w, int kh, int kw);
int fft_conv_fprop_save(fftconv_handle hd, const float *x, const float *wt, float *y,
                        int S, int f, int fo, int h, int w, int kh, int kw,
                        void *saved, size_t saved_bytes, void *ws, size_t ws_bytes);
int fft_conv_backward(fftconv_handle hd, const float *gy, float *gx, float *gw,
                      int S, int f, int fo, int h, int w, int kh, int kw,
                      float scale, int accumulate, const void *saved, size_t saved_bytes,
                      void *ws, size_t ws_bytes);

/*
 * Per-kernel timing of the last convolution call, for roofline reporting.
 * With profiling enabled every kernel of a convolution call is launched with a start/stop
 * HIP event pair attached to that dispatch on the handle's stream.
 * fftconv_last_kernel_ms() waits for the last call and writes the execution times in
 * milliseconds, in launch order, to ms_out[0 .. *count) (at most 8 kernels per call);
 * fftconv_last_kernel_label(h, i) names kernel i of that list (a static string, "" when there
 * is no such entry):
 *   "fft.ab"  forward FFT of both operands in one launch; "fft.a", "fft.b" when they are two
 *             launches or there is only one operand to transform (a = first operand of the pass:
 *             x for fprop, gy for bprop, accGrad and fft_conv_backward; b = weights, or x for
 *             accGrad; fft_conv_backward on a tiled layer cuts gy twice: a for bprop, b for accGrad)
 *   "contraction"       per-bin contraction of one pass
 *   "contraction.pair"  the bprop and accGrad contractions of fft_conv_backward in one launch
 *   "ifft", "ifft.pair" inverse FFT + clip of one product, or of gx and gw in one launch
 *   "fused"             the one-launch passes
 * fft_conv_fprop / bprop / accgrad / fprop_save give 3 or 4 entries (1 when the pass runs as one
 * launch); fft_conv_backward gives
 * fft of gy, then contraction and ifft for gx and again for gw (5), or 4 or 3 with shared launches.
 * Off by default.
 */
int fftconv_set_profiling(fftconv_handle h, int enabled);
int fftconv_last_kernel_ms(fftconv_handle h, float *ms_out, int capacity, int *count);
const char *fftconv_last_kernel_label(fftconv_handle h, int i);

#ifdef __cplusplus
}
#endif
#endif /* FFTCONV_H */
