// One-launch fprop for small layers (the latency-bound regime: a few microseconds per kernel,
// where three launches cost more than the arithmetic).  Section 6 of the fbfft paper plans
// matrix products integrated with the transform kernels to avoid separate launches; here one
// workgroup carries one sample through the whole pass:
//   R2C of its f input planes (spectra stay in LDS)  ->  Y_j = sum_i X_i . conj(W_ji) per bin
//   on the vector ALUs (one sample is a matrix-vector product per bin: no tile for the matrix
//   cores), W from the weight transform computed ahead  ->  C2R + crop of its f' planes.
// No workgroup waits for another one, so there is no grid-wide synchronisation.
#include "fft_kernels_impl.hpp"

namespace fc {

struct FusedParams {
    Fwd2dParams fwd;           // in = x (first sample), planes = f
    Inv2dParams inv;           // out = y (first sample), planes = f'
    const float *wf;           // weight transform in the layout fwd.lay, plane = j * f + i
    int f, fo;
    long x_stride, y_stride;   // floats per sample
    int img;                   // float offset of the second LDS image (the product's)
};

template <int L, int G, int T>
__global__ void __launch_bounds__(T *(L * G / 2) * G) fused_fprop_kernel(FusedParams fp) {
    constexpr int N = L * G, NH = N / 2, NB = NH + 1, BT = T * NH * G, BINS = N * NB;
    extern __shared__ float smem[];
    const int tid = threadIdx.x;
    const long s = blockIdx.x;

    Fwd2dParams fw = fp.fwd;
    fw.in += s * fp.x_stride;
    fft2d_r2c_body<L, G, T, true, true, true>(fw, 0);      // X[(bin * 2 + c) * T + i] at smem

    // One output (bin, j) per lane and round; consecutive lanes take consecutive j, so the X
    // reads of a bin are LDS broadcasts and the W reads of neighbouring j are contiguous (the f
    // planes j * f .. j * f + f - 1 lie in one run of the layout because f divides T).  (Gathering W
    // for several outputs at once, or for the first ones ahead of the forward transform,
    // measured slower: 14.0 against 11.7 us on the 16-plane 13x13 layer.)
    float *yimg = smem + fp.img;
    const int f = fp.f, fo = fp.fo;
    for (int o = tid; o < BINS * fo; o += BT) {
        const int bin = o / fo, j = o - bin * fo;
        const float *wr = fp.wf + fp.fwd.lay.index((long)j * f, bin, 0);
        const float *wi = wr + T;
        const float *xr = smem + (bin * 2) * T, *xi = xr + T;
        float yr = 0.f, yi = 0.f;
#pragma unroll 4
        for (int i = 0; i < f; i += 4) {
            const float4 a = *reinterpret_cast<const float4 *>(wr + i), b = *reinterpret_cast<const float4 *>(wi + i);
            const float4 p = *reinterpret_cast<const float4 *>(xr + i), q = *reinterpret_cast<const float4 *>(xi + i);
            // x . conj(w) = (xr wr + xi wi) + i (xi wr - xr wi)
            yr += p.x * a.x + q.x * b.x + p.y * a.y + q.y * b.y + p.z * a.z + q.z * b.z + p.w * a.w + q.w * b.w;
            yi += q.x * a.x - p.x * b.x + q.y * a.y - p.y * b.y + q.z * a.z - p.z * b.z + q.w * a.w - p.w * b.w;
        }
        yimg[(bin * 2) * T + j] = yr;
        yimg[(bin * 2 + 1) * T + j] = yi;
    }
    __syncthreads();

    Inv2dParams iv = fp.inv;
    iv.out += s * fp.y_stride;
    fft2d_c2r_body<L, G, T, true, false, true>(iv, 0, yimg);
}

// bprop the same way: R2C of the sample's f' planes of gy (spectra stay in LDS) ->
// GX_i = sum_j GY_j . W_ji per bin (no conjugate) -> C2R + crop of its f planes.  A lane forms
// four consecutive input planes i of one bin: the four W values of one j are then one 16-byte
// load (planes j * f + i .. + 3 lie in one run of the layout because f divides T), and the GY
// reads of a bin are LDS broadcasts.
template <int L, int G, int T>
__global__ void __launch_bounds__(T *(L * G / 2) * G) fused_bprop_kernel(FusedParams fp) {
    constexpr int N = L * G, NH = N / 2, NB = NH + 1, BT = T * NH * G, BINS = N * NB;
    extern __shared__ float smem[];
    const int tid = threadIdx.x;
    const long s = blockIdx.x;

    Fwd2dParams fw = fp.fwd;
    fw.in += s * fp.x_stride;
    fft2d_r2c_body<L, G, T, true, true, true>(fw, 0);      // GY[(bin * 2 + c) * T + j] at smem

    float *ximg = smem + fp.img;
    const int f = fp.f, fo = fp.fo, f4 = f >> 2;
    for (int o = tid; o < BINS * f4; o += BT) {
        const int bin = o / f4, i = (o - bin * f4) << 2;
        const float *gr = smem + (bin * 2) * T, *gi = gr + T;
        float4 xr = make_float4(0.f, 0.f, 0.f, 0.f), xi = xr;
#pragma unroll 4
        for (int j = 0; j < fo; ++j) {
            const float *wr = fp.wf + fp.fwd.lay.index((long)j * f + i, bin, 0);
            const float4 a = *reinterpret_cast<const float4 *>(wr), b = *reinterpret_cast<const float4 *>(wr + T);
            const float yr = gr[j], yi = gi[j];
            // gy . w = (yr wr - yi wi) + i (yr wi + yi wr)
            xr.x += yr * a.x - yi * b.x; xi.x += yr * b.x + yi * a.x;
            xr.y += yr * a.y - yi * b.y; xi.y += yr * b.y + yi * a.y;
            xr.z += yr * a.z - yi * b.z; xi.z += yr * b.z + yi * a.z;
            xr.w += yr * a.w - yi * b.w; xi.w += yr * b.w + yi * a.w;
        }
        *reinterpret_cast<float4 *>(ximg + (bin * 2) * T + i) = xr;
        *reinterpret_cast<float4 *>(ximg + (bin * 2 + 1) * T + i) = xi;
    }
    __syncthreads();

    Inv2dParams iv = fp.inv;
    iv.out += s * fp.y_stride;
    fft2d_c2r_body<L, G, T, true, false, true>(iv, 0, ximg);
}

template <int L, int G, int T>
static hipError_t run_fused(const float *x, const float *wf, float *y, int S, int f, int fo, int h, int w,
                            int kh, int kw, LaunchCtx st, bool bprop = false) {
    // fprop: in = x (f planes of h x w), out = y (f' planes of oh x ow); bprop: in = gy (f' planes of
    // oh x ow), out = gx (f planes of h x w)
    constexpr int N = L * G, NH = N / 2, NB = NH + 1, BT = T * NH * G;
    FusedParams fp;
    size_t lds_fwd = 0;
    const int fh = h - kh + 1, fw_ = w - kw + 1;
    const int in_planes = bprop ? fo : f, in_h = bprop ? fh : h, in_w = bprop ? fw_ : w;
    const int out_planes = bprop ? f : fo;
    fp.fwd = make_fwd2d<L, G, T>(x, nullptr, in_planes, in_h, in_w, &lds_fwd, nullptr);
    const int oh = bprop ? h : fh, ow = bprop ? w : fw_;
    Inv2dParams &iv = fp.inv;
    iv.in = nullptr; iv.out = y; iv.planes = out_planes; iv.h_out = oh; iv.w_out = ow;
    iv.MPS = MidLayout<L, G>::inv_plane(oh) | 1;
    iv.lay = fp.fwd.lay;
    iv.scale = 1.0f / ((float)N * (float)N); iv.accumulate = 0;
    iv.vec_ok = 0; iv.in_vec_ok = 0; iv.tiled = 0; iv.info_off = 0; iv.tw_off = 0; iv.win_h = iv.win_w = 0;
    iv.div_w = iv.div_h = MagicDiv{0}; iv.view = PlaneView{};
    fp.wf = wf; fp.f = f; fp.fo = fo;
    fp.x_stride = (long)in_planes * in_h * in_w; fp.y_stride = (long)out_planes * oh * ow;
    const size_t img = (size_t)T * N * NB * 2;           // floats of one LDS image
    // the first region holds, one after the other in time, the forward staging and transposed
    // data, the spectra X, and the inverse's transposed data and output block; the product's
    // image lies behind it
    size_t first = img * sizeof(float);
    if (lds_fwd > first) first = lds_fwd;
    if ((size_t)T * iv.MPS * sizeof(float2) > first) first = (size_t)T * iv.MPS * sizeof(float2);
    if (((size_t)T * oh * ow + 3) * sizeof(float) > first) first = ((size_t)T * oh * ow + 3) * sizeof(float);
    first = (first + 15) / 16 * 16;
    fp.img = (int)(first / sizeof(float));
    const size_t lds = first + img * sizeof(float);
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    auto k = bprop ? fused_bprop_kernel<L, G, T> : fused_fprop_kernel<L, G, T>;
    if (hipError_t e = allow_big_lds((const void *)k, lds); e != hipSuccess) return e;
    launch_kernel(k, dim3((unsigned)S), dim3(BT), lds, st, fp);
    return hipGetLastError();
}

bool fused_fprop_supported(int N, int f, int fo, const float *wf) {
    const int tsh = fft2d_tile_log2(N);
    if (tsh < 5 || N > 16) return false;                // bases 8 .. 16: 32 or 64 planes per tile
    const int T = 1 << tsh;
    // bins x weight planes up to 40000: beyond that the vector-ALU product stage takes longer
    // than the launches it saves (measured at basis 14: 16 x 16 planes 10.1 us against 14.9 for
    // the three-launch path, 16 x 32 13.2 against 14.6, 32 x 16 19.3 against 15.9, 32 x 32 31 against 16)
    return f <= T && fo <= T && (long)N * (N / 2 + 1) * f * fo <= 40000 && f % 4 == 0 && T % f == 0 &&
           ((size_t)wf & 15) == 0;
}

hipError_t launch_fused_fprop(const float *x, const float *wf, float *y, int S, int f, int fo, int h, int w,
                              int kh, int kw, int N, LaunchCtx st) {
    if (!fused_fprop_supported(N, f, fo, wf) || h > N || w > N) return hipErrorInvalidValue;
    switch (N) {
        // lane pairs: twice the lanes for the product stage, whose W gathers set its pace
        case 8: return run_fused<4, 2, 64>(x, wf, y, S, f, fo, h, w, kh, kw, st);
        case 10: return run_fused<5, 2, 32>(x, wf, y, S, f, fo, h, w, kh, kw, st);
        case 12: return run_fused<6, 2, 32>(x, wf, y, S, f, fo, h, w, kh, kw, st);
        case 14: return run_fused<7, 2, 32>(x, wf, y, S, f, fo, h, w, kh, kw, st);
        case 16: return run_fused<8, 2, 32>(x, wf, y, S, f, fo, h, w, kh, kw, st);
        default: return hipErrorInvalidValue;
    }
}

// The same rule with the roles of f and f' as they are in bprop: the reduction runs over f'.
bool fused_bprop_supported(int N, int f, int fo, const float *wf) {
    return fused_fprop_supported(N, f, fo, wf);
}

hipError_t launch_fused_bprop(const float *gy, const float *wf, float *gx, int S, int f, int fo, int h, int w,
                              int kh, int kw, int N, LaunchCtx st) {
    if (!fused_bprop_supported(N, f, fo, wf) || h > N || w > N) return hipErrorInvalidValue;
    switch (N) {
        case 8: return run_fused<4, 2, 64>(gy, wf, gx, S, f, fo, h, w, kh, kw, st, true);
        case 10: return run_fused<5, 2, 32>(gy, wf, gx, S, f, fo, h, w, kh, kw, st, true);
        case 12: return run_fused<6, 2, 32>(gy, wf, gx, S, f, fo, h, w, kh, kw, st, true);
        case 14: return run_fused<7, 2, 32>(gy, wf, gx, S, f, fo, h, w, kh, kw, st, true);
        case 16: return run_fused<8, 2, 32>(gy, wf, gx, S, f, fo, h, w, kh, kw, st, true);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace fc
