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

// accGrad in one launch.  GW_ji = sum_s conj(GY_sj) . X_si reduces over the samples, so a workgroup
// that is to work alone needs every sample's planes of the channels it owns: it takes a block of
// JB output channels and IB input channels, transforms the S x JB planes of gy and the S x IB
// planes of x itself (each set within one plane tile, gathered through a view that selects the
// block's channels of every sample), forms the JB x IB products per bin on the vector ALUs and
// inverts them with the crop to kh x kw.  A plane of x is transformed by f' / JB workgroups: the
// price of having no dependence between workgroups, affordable while the whole layer is a few
// microseconds of arithmetic.  Measured (back-to-back calls, us, one launch against the three of
// fft_conv_accgrad): 16 samples of 16 x 16 planes 7x7 10.1 / 13.6; 2 samples of 64 x 64 planes 13x13
// 12.0 / 16.7; 8 of 64 x 64 15.7 / 16.8; 8 of 32 x 32 15.2 / 15.4; 16 of 16 x 16 13x13 16.3 / 14.6
// (in the kernel: transforms 8.0, products 3.9, inverse 2.7); 32 of 16 x 16 17.9 / 15.4: it pays for
// few samples or very small images, which is when fft_conv_accgrad takes it by itself.
struct FusedAccParams {
    Fwd2dParams fg, fx;        // in = gy / x (first sample, channel 0); planes = S * JB / S * IB
    Inv2dParams inv;           // out = gw (pair (0, 0)); planes = JB * IB
    int S, JB, IB, nib;        // nib = f / IB blocks of input channels
    int QP;                    // JB * IB rounded up to a power of two
    long gy_plane, x_plane, gw_plane;   // floats per plane
    int f;
    int imgB, imgC;            // float offsets of the second and third LDS image
};

// The workgroup is two sets of BT threads: the first transforms the block's planes of gy, the
// second, at the same time and in its own part of LDS, those of x.
template <int L, int G, int T>
__global__ void __launch_bounds__(2 * T *(L * G / 2) * G) fused_accgrad_kernel(FusedAccParams ap) {
    constexpr int N = L * G, NH = N / 2, NB = NH + 1, BT = T * NH * G, BINS = N * NB;
    static_assert(BT % 64 == 0, "the two thread sets are whole waves");
    extern __shared__ float smem[];
    const int tid = threadIdx.x;
    const int jb = blockIdx.x / ap.nib, ib = blockIdx.x - jb * ap.nib;
    const bool second = __builtin_amdgcn_readfirstlane(tid >= BT) != 0;    // (uniform over a wave)
    const int t = second ? tid - BT : tid;

    {
        Fwd2dParams fw = second ? ap.fx : ap.fg;
        fw.in += second ? (long)ib * ap.IB * ap.x_plane : (long)jb * ap.JB * ap.gy_plane;
        // GY[(bin * 2 + c) * T + s * JB + jj] at smem, X[(bin * 2 + c) * T + s * IB + ii] at smem + imgB
        fft2d_r2c_body<L, G, T, true, true, true>(fw, 0, t, second ? (unsigned)ap.imgB : 0u);
    }

    // Products: a wave takes a few bins at a time; for one bin its lanes are (pair q = (jj, ii),
    // sample group), so that the planes read by the lanes of a wave differ (or coincide: a
    // broadcast) and the LDS reads meet no bank twice -- lanes on different bins would all read the
    // same plane index, i.e. the same bank.  Each lane sums its samples, then the groups of a pair
    // are added up by a butterfly of lane exchanges; UB bins go through that together so that the
    // exchanges of one overlap with those of the others.
    constexpr int UB = 4, NW = 2 * BT / 64;
    const float *ximg = smem + ap.imgB;
    float *wimg = smem + ap.imgC;
    const int S = ap.S, JB = ap.JB, IB = ap.IB, Q = JB * IB, QP = ap.QP;   // QP: Q rounded up to a power of two
    const int lane = tid & 63, wave = tid >> 6;
    const int q = lane & (QP - 1), sg = lane / QP, nsg = 64 / QP;
    const bool live = q < Q;
    const int jj = live ? q / IB : 0, ii = live ? q - jj * IB : 0;
    for (int b0 = wave * UB; b0 < BINS; b0 += NW * UB) {
        float wr[UB], wi[UB];
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            const int bin = b0 + u < BINS ? b0 + u : BINS - 1;
            const float *gr = smem + (bin * 2) * T + jj, *gi = gr + T;
            const float *xr = ximg + (bin * 2) * T + ii, *xi = xr + T;
            wr[u] = 0.f; wi[u] = 0.f;
            if (live) {
                for (int s = sg; s < S; s += nsg) {
                    const float a = gr[s * JB], b = gi[s * JB], c = xr[s * IB], d = xi[s * IB];
                    // conj(gy) . x = (a c + b d) + i (a d - b c)
                    wr[u] += a * c + b * d;
                    wi[u] += a * d - b * c;
                }
            }
        }
        for (int m = QP; m < 64; m <<= 1) {
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                wr[u] += __shfl_xor(wr[u], m, 64);
                wi[u] += __shfl_xor(wi[u], m, 64);
            }
        }
        if (live && sg == 0) {
#pragma unroll
            for (int u = 0; u < UB; ++u)
                if (b0 + u < BINS) {
                    wimg[((b0 + u) * 2) * T + q] = wr[u];
                    wimg[((b0 + u) * 2 + 1) * T + q] = wi[u];
                }
        }
    }
    __syncthreads();

    Inv2dParams iv = ap.inv;
    iv.out += ((long)jb * JB * ap.f + (long)ib * IB) * ap.gw_plane;
    if (second) iv.planes = 0;      // (the second thread set only passes the barriers)
    fft2d_c2r_body<L, G, T, true, false, true>(iv, 0, wimg, t);
}

// Channel blocks (JB of f', IB of f; divisors, so that no block is ragged) with S * JB, S * IB and
// JB * IB within one plane tile, chosen to transform the fewest planes over the whole grid.
static bool accgrad_blocks(int T, int S, int f, int fo, int *JB, int *IB) {
    double best = 0.0;
    *JB = *IB = 0;
    for (int j = 1; j <= fo && S * j <= T; ++j) {
        if (fo % j) continue;
        for (int i = 1; i <= f && S * i <= T && j * i <= T; ++i) {
            if (f % i) continue;
            const double cost = 1.0 / j + 1.0 / i;      // planes transformed ~ S f f' (1/IB + 1/JB)
            if (*JB == 0 || cost < best) { best = cost; *JB = j; *IB = i; }
        }
    }
    return *JB != 0;
}

bool fused_accgrad_supported(int N, int S, int f, int fo) {
    const int tsh = fft2d_tile_log2(N);
    if (tsh < 5 || N > 16) return false;                // bases 8 .. 16: 32 or 64 planes per tile
    int JB, IB;
    if (!accgrad_blocks(1 << tsh, S, f, fo, &JB, &IB)) return false;
    // one round of workgroups at most, each transforming S (JB + IB) planes of its own
    return (long)(fo / JB) * (f / IB) <= 256;
}

// Where the one launch measured faster than the three of the ordinary pass: few samples or very
// small images (samples x bins up to 900: 8 samples at basis 14, 16 at basis 8).
bool fused_accgrad_pays(int N, int S, int f, int fo) {
    return fused_accgrad_supported(N, S, f, fo) && (long)S * N * (N / 2 + 1) <= 900;
}

template <int L, int G, int T>
static hipError_t run_fused_accgrad(const float *gy, const float *x, float *gw, int S, int f, int fo, int h, int w,
                                    int kh, int kw, float scale, int accumulate, LaunchCtx st) {
    constexpr int N = L * G, NH = N / 2, NB = NH + 1, BT = T * NH * G;
    const int oh = h - kh + 1, ow = w - kw + 1;
    FusedAccParams ap;
    if (!accgrad_blocks(T, S, f, fo, &ap.JB, &ap.IB)) return hipErrorInvalidValue;
    ap.S = S; ap.f = f; ap.nib = f / ap.IB;
    ap.QP = 1;
    while (ap.QP < ap.JB * ap.IB) ap.QP <<= 1;
    ap.gy_plane = (long)oh * ow; ap.x_plane = (long)h * w; ap.gw_plane = (long)kh * kw;
    // views: plane p of a set = (sample p / C, channel p % C of the block) of a tensor with Cimg channels
    const PlaneView vg{ap.JB, 1, 1, N, N, 0, 0, oh, ow, fo}, vx{ap.IB, 1, 1, N, N, 0, 0, h, w, f},
        vo{ap.IB, 1, 1, N, N, 0, 0, kh, kw, f};
    size_t lds_g = 0, lds_x = 0, lds_i = 0;
    bool istage = false;
    ap.fg = make_fwd2d<L, G, T>(gy, nullptr, (long)S * ap.JB, oh, ow, &lds_g, &vg);
    ap.fx = make_fwd2d<L, G, T>(x, nullptr, (long)S * ap.IB, h, w, &lds_x, &vx);
    // LDS is what limits this kernel: stage the planes with the plain odd strides instead of the
    // bank-spreading ones (up to 34 floats per row of 8), which the transforms read equally well
    auto compact = [](Fwd2dParams &p, size_t *lds) {
        p.RS = p.w_in | 1;
        p.IPS = (p.h_in * p.RS) | 1;
        const size_t a = ((size_t)T * p.IPS + N) * sizeof(float), b = (size_t)T * p.MPS * sizeof(float2);
        *lds = a > b ? a : b;
    };
    compact(ap.fg, &lds_g);
    compact(ap.fx, &lds_x);
    ap.inv = make_inv2d<L, G, T>(nullptr, gw, (long)ap.JB * ap.IB, kh, kw, true, scale / ((float)N * (float)N),
                                 accumulate != 0, &vo, &lds_i, &istage);
    const size_t img = (size_t)T * N * NB * 2 * sizeof(float);      // bytes of one LDS image
    // Two regions of equal size, one per thread set, each holding its forward transform's staging
    // and transposed data and then its spectra (the first later also the inverse's transposed data
    // and output block); the products' image behind them, the two origin tables last.
    size_t first = img;
    if (lds_g > first) first = lds_g;
    if (lds_x > first) first = lds_x;
    const size_t inv_a = (size_t)T * ap.inv.MPS * sizeof(float2), inv_b = ((size_t)T * kh * kw + 3) * sizeof(float);
    if (inv_a > first) first = inv_a;
    if (inv_b > first) first = inv_b;
    first = (first + 15) / 16 * 16;
    ap.imgB = (int)(first / sizeof(float));
    ap.imgC = (int)(2 * first / sizeof(float));
    int info0 = 0, info1 = 0;
    size_t lds = with_origin_table(2 * first + img, T, &info0);
    lds = with_origin_table(lds, T, &info1);
    ap.fg.info_off = ap.inv.info_off = info0;
    ap.fx.info_off = info1 - ap.imgB;          // relative to the second region
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    auto k = fused_accgrad_kernel<L, G, T>;
    if (hipError_t e = allow_big_lds((const void *)k, lds); e != hipSuccess) return e;
    launch_kernel(k, dim3((unsigned)((fo / ap.JB) * ap.nib)), dim3(2 * BT), lds, st, ap);
    return hipGetLastError();
}

hipError_t launch_fused_accgrad(const float *gy, const float *x, float *gw, int S, int f, int fo, int h, int w,
                                int kh, int kw, int N, float scale, int accumulate, LaunchCtx st) {
    if (!fused_accgrad_supported(N, S, f, fo) || h > N || w > N) return hipErrorInvalidValue;
    switch (N) {
        case 8: return run_fused_accgrad<4, 2, 64>(gy, x, gw, S, f, fo, h, w, kh, kw, scale, accumulate, st);
        case 10: return run_fused_accgrad<5, 2, 32>(gy, x, gw, S, f, fo, h, w, kh, kw, scale, accumulate, st);
        case 12: return run_fused_accgrad<6, 2, 32>(gy, x, gw, S, f, fo, h, w, kh, kw, scale, accumulate, st);
        case 14: return run_fused_accgrad<7, 2, 32>(gy, x, gw, S, f, fo, h, w, kh, kw, scale, accumulate, st);
        case 16: return run_fused_accgrad<8, 2, 32>(gy, x, gw, S, f, fo, h, w, kh, kw, scale, accumulate, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace fc
