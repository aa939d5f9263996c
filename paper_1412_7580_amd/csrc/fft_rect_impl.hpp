// 2-D transforms on a rectangular Fourier basis NR x NC (NR rows, NC columns, both from the
// bases up to 32), for the convolution passes of images that are far from square (Section 2
// allows any h x w; zero-padding to a common basis, Section 3.1, only needs each dimension to
// hold its operand).  Plane-tiled frequency layout only, no windows.  The kernels follow the
// square ones (rows two at a time as one complex line, LDS transpose, columns; slot 0 of a
// half spectrum holds the packed pair of real bins) with the line length, lanes per line and
// registers per lane chosen per dimension: NR = LH * GH, NC = LW * GW.
#pragma once
#include "fft_kernels_impl.hpp"

namespace fc {

template <int LH, int GH, int LW, int GW>
struct RectShape {
    static constexpr int NR = LH * GH, NC = LW * GW, RH = NR / 2, CH = NC / 2, NB = CH + 1;
    // planes per workgroup = tile of the layout: as for the square basis of the larger side
    static constexpr int T = (NR >= 18 || NC >= 18) ? 16 : 32;
    static constexpr int ROW_LANES = T * GW * RH;   // (lane in line, plane, row pair)
    static constexpr int COL_LANES = T * GH * CH;   // (lane in line, plane, column slot)
    static constexpr int BT = ROW_LANES > COL_LANES ? ROW_LANES : COL_LANES;
    static constexpr int MRS = CH | 1;              // LDS row stride of the half spectra (float2)
};

struct RectFwdParams {
    const float *in;
    float *out;
    long planes;
    int h_in, w_in;
    int RS, IPS;      // LDS row / plane stride of the staged input (floats, odd)
    int MPS;          // LDS plane stride of the row-transformed data (float2, odd)
    MagicDiv div_wv, div_h;
    int vecw;
    FreqLayout lay;
    int linear;
};

template <int LH, int GH, int LW, int GW>
__device__ __forceinline__ void fft2d_r2c_rect_body(const RectFwdParams &prm, unsigned block) {
    typedef RectShape<LH, GH, LW, GW> S;
    constexpr int NR = S::NR, RH = S::RH, CH = S::CH, NB = S::NB, T = S::T, BT = S::BT, MRS = S::MRS;
    constexpr int NA = SplitRegs<LW, GW>::A, NBR = SplitRegs<LW, GW>::B;
    extern __shared__ float smem[];
    float *sin = smem;
    float2 *mid = reinterpret_cast<float2 *>(smem);

    const int tid = threadIdx.x;
    const long p0 = (long)block * T;
    const int h_in = prm.h_in, w_in = prm.w_in, hw = h_in * w_in;
    const long left = prm.planes - p0;
    const int np = left < T ? (int)left : T;

    {   // stage the block's planes (contiguous in memory) into LDS
        const float *src = prm.in + p0 * hw;
        if (prm.linear) {
            sin = smem + misalign4(src);
            stage_linear<BT>(sin, src, (unsigned)np * hw, tid, true);
        } else {
            const unsigned rows = (unsigned)np * h_in;
            if (prm.vecw == 4)
                stage_padded<BT, 4, 24>(sin, src, rows, w_in, h_in, prm.RS, prm.IPS, prm.div_wv, prm.div_h, tid);
            else if (prm.vecw == 2)
                stage_padded<BT, 2, 12>(sin, src, rows, w_in, h_in, prm.RS, prm.IPS, prm.div_wv, prm.div_h, tid);
            else
                stage_padded<BT, 1, 8>(sin, src, rows, w_in, h_in, prm.RS, prm.IPS, prm.div_wv, prm.div_h, tid);
        }
    }
    __syncthreads();

    // ---- rows (length NC): lane group = (plane p, rows ra and rb packed as ra + i rb)
    const int H2 = (h_in + 1) >> 1;
    const int g = tid % GW, p = (tid / GW) % T, rp = tid / (GW * T);
    const bool row_active = rp < H2 && p < np;
    const int ra = rp, rb = rp + H2;
    const bool hasb = rb < h_in;
    float are[NA], aim[NA], bre[NBR], bim[NBR];
    if (row_active) {
        float re[LW], im[LW];
        const float *pa = sin + p * prm.IPS + ra * prm.RS;
        const float *pb = sin + p * prm.IPS + rb * prm.RS;
#pragma unroll
        for (int m = 0; m < LW; ++m) {
            const int j = g + GW * m;
            const bool in = j < w_in;
            re[m] = in ? pa[j] : 0.0f;
            im[m] = (in && hasb) ? pb[j] : 0.0f;
        }
        fft_group<LW, GW, -1>(re, im, g);
        split_two_real<LW, GW>(re, im, g, are, aim, bre, bim);
    }
    __syncthreads();   // the staged input may be overwritten
    if (row_active) {
        float2 *mp = mid + p * prm.MPS;
        if constexpr (GW == 1) {
#pragma unroll
            for (int k = 0; k < CH; ++k) mp[ra * MRS + k] = make_float2(are[k], aim[k]);
            if (hasb) {
#pragma unroll
                for (int k = 0; k < CH; ++k) mp[rb * MRS + k] = make_float2(bre[k], bim[k]);
            }
        } else {
            const int row = (g & 1) ? rb : ra;
            if (!(g & 1) || hasb) {
#pragma unroll
                for (int k = 0; k < LW; ++k) mp[row * MRS + split_slot<LW, GW>(g, k)] = make_float2(are[k], aim[k]);
            }
        }
    }
    __syncthreads();

    // ---- columns (length NR): lane group = (plane cp, column slot cc); slot 0 is the packed
    //      pair of real columns k2 = 0 and k2 = NC/2
    const int cg = tid % GH, cp = (tid / GH) % T, cc = tid / (GH * T);
    if (cp >= np || cc >= CH) return;
    float re[LH], im[LH];
    {
        const float2 *mp = mid + cp * prm.MPS + cc;
#pragma unroll
        for (int m = 0; m < LH; ++m) {
            const int r = cg + GH * m;
            float2 v = make_float2(0.f, 0.f);
            if (r < h_in) v = mp[r * MRS];
            re[m] = v.x; im[m] = v.y;
        }
        fft_group<LH, GH, -1>(re, im, cg);
    }
    float *base = prm.out + prm.lay.index(p0, 0, 0) + cp;
    auto st = [&](int k1, int k2, float vr, float vi) {
        const unsigned idx = (unsigned)((k1 * NB + k2) * 2) * T;
        base[idx] = vr;
        base[idx + T] = vi;
    };
    if (cc != 0) {
#pragma unroll
        for (int k = 0; k < LH; ++k) st(k + LH * group_block<GH>(cg), cc, re[k], im[k]);
    } else {
        constexpr int UA = SplitRegs<LH, GH>::A, UB = SplitRegs<LH, GH>::B;
        float ur[UA], ui[UA], vr[UB], vi[UB];
        split_two_real<LH, GH>(re, im, cg, ur, ui, vr, vi);
        if constexpr (GH == 1) {
            st(0, 0, ur[0], 0.f);  st(RH, 0, ui[0], 0.f);
            st(0, CH, vr[0], 0.f); st(RH, CH, vi[0], 0.f);
#pragma unroll
            for (int k = 1; k < RH; ++k) {
                st(k, 0, ur[k], ui[k]);  st(NR - k, 0, ur[k], -ui[k]);
                st(k, CH, vr[k], vi[k]); st(NR - k, CH, vr[k], -vi[k]);
            }
        } else {
            const int k2 = (cg & 1) ? CH : 0;   // even lanes: column 0, odd lanes: column NC/2
#pragma unroll
            for (int k = 0; k < LH; ++k) {
                const int k1 = split_slot<LH, GH>(cg, k);
                if (k1 == 0) {
                    st(0, k2, ur[k], 0.f);
                    st(RH, k2, ui[k], 0.f);
                } else {
                    st(k1, k2, ur[k], ui[k]);
                    st(NR - k1, k2, ur[k], -ui[k]);
                }
            }
        }
    }
}

// Both operands of a pass in one launch: the blocks of operand o are [first[o], first[o+1]).
struct RectFwdPair {
    RectFwdParams op[2];
    unsigned first[3];
};

template <int LH, int GH, int LW, int GW>
__global__ void __launch_bounds__((RectShape<LH, GH, LW, GW>::BT)) fft2d_r2c_rect_kernel(RectFwdPair m) {
    const unsigned b = blockIdx.x;
    const int o = b >= m.first[1];
    fft2d_r2c_rect_body<LH, GH, LW, GW>(m.op[o], b - m.first[o]);
}

struct RectInvParams {
    const float *in;
    float *out;
    long planes;
    int h_out, w_out;
    int MPS;
    FreqLayout lay;
    float scale;
    int accumulate;
};

template <int LH, int GH, int LW, int GW>
__device__ __forceinline__ void fft2d_c2r_rect_body(const RectInvParams &prm, unsigned block) {
    typedef RectShape<LH, GH, LW, GW> S;
    constexpr int NC = S::NC, CH = S::CH, NB = S::NB, T = S::T, BT = S::BT, MRS = S::MRS;
    extern __shared__ float smem[];
    float2 *mid = reinterpret_cast<float2 *>(smem);

    const int tid = threadIdx.x;
    const long p0 = (long)block * T;
    const int h_out = prm.h_out, w_out = prm.w_out;
    float *sout = smem + misalign4(prm.out + p0 * (long)h_out * w_out);
    const long left = prm.planes - p0;
    const int np = left < T ? (int)left : T;

    {   // ---- columns (inverse along k1) for column slot cc of plane cp
        const int cg = tid % GH, cp = (tid / GH) % T, cc = tid / (GH * T);
        if (cp < np && cc < CH) {
            float cre[LH], cim[LH];
            const float *base = prm.in + prm.lay.index(p0, 0, 0) + cp;
#pragma unroll
            for (int m = 0; m < LH; ++m) {
                const int k1 = cg + GH * m;
                const float *q = base + (size_t)((k1 * NB + cc) * 2) * T;
                float xr = q[0], xi = q[T];
                if (cc == 0) {   // pack columns 0 and NC/2:  z = y0 + i yN
                    const float *qn = base + (size_t)((k1 * NB + CH) * 2) * T;
                    const float nr = qn[0], ni = qn[T];
                    xr -= ni; xi += nr;
                }
                cre[m] = xr; cim[m] = xi;
            }
            fft_group<LH, GH, +1>(cre, cim, cg);
            float2 *mp = mid + cp * prm.MPS + cc;
            const int a0 = LH * group_block<GH>(cg);
#pragma unroll
            for (int k = 0; k < LH; ++k) {
                if (a0 + k < h_out) mp[(a0 + k) * MRS] = make_float2(cre[k], cim[k]);
            }
        }
    }
    __syncthreads();

    // ---- rows (inverse along k2), rows ra and rb packed as ra + i rb
    const int H2 = (h_out + 1) >> 1;
    const int g = tid % GW, p = (tid / GW) % T, rp = tid / (GW * T);
    const bool active = rp < H2 && p < np;
    const int ra = rp, rb = rp + H2;
    const bool hasb = rb < h_out;
    float re[LW], im[LW];
    if (active) {
        const float2 *A = mid + p * prm.MPS + ra * MRS;
        const float2 *B = mid + p * prm.MPS + (hasb ? rb : ra) * MRS;
#pragma unroll
        for (int m = 0; m < LW; ++m) {
            const int k2 = g + GW * m;
            const int slot = (k2 == CH) ? 0 : (k2 < CH ? k2 : NC - k2);
            const float2 a = A[slot];
            float2 b = B[slot];
            if (!hasb) b = make_float2(0.f, 0.f);
            float xr, xi;
            if (k2 == 0) { xr = a.x; xi = b.x; }
            else if (k2 == CH) { xr = a.y; xi = b.y; }
            else if (k2 < CH) { xr = a.x - b.y; xi = a.y + b.x; }
            else { xr = a.x + b.y; xi = b.x - a.y; }
            re[m] = xr; im[m] = xi;
        }
        fft_group<LW, GW, +1>(re, im, g);
    }
    __syncthreads();   // all reads of `mid` done; the area becomes the output block
    if (active) {
        float *oa = sout + (p * h_out + ra) * w_out;
        float *ob = sout + (p * h_out + rb) * w_out;
#pragma unroll
        for (int k = 0; k < LW; ++k) {
            const int b = k + LW * group_block<GW>(g);
            if (b < w_out) {
                oa[b] = re[k] * prm.scale;
                if (hasb) ob[b] = im[k] * prm.scale;
            }
        }
    }
    __syncthreads();
    unstage_linear<BT>(prm.out + p0 * (long)h_out * w_out, sout, (unsigned)np * h_out * w_out, tid, true,
                       prm.accumulate != 0);
}

template <int LH, int GH, int LW, int GW>
__global__ void __launch_bounds__((RectShape<LH, GH, LW, GW>::BT)) fft2d_c2r_rect_kernel(RectInvParams prm) {
    fft2d_c2r_rect_body<LH, GH, LW, GW>(prm, blockIdx.x);
}

// The inverse transforms of the two products of the backward pass in one launch: the blocks of
// operand o are [first[o], first[o+1]).
struct RectInvPair {
    RectInvParams op[2];
    unsigned first[3];
};

template <int LH, int GH, int LW, int GW>
__global__ void __launch_bounds__((RectShape<LH, GH, LW, GW>::BT)) fft2d_c2r_rect_pair_kernel(RectInvPair m) {
    const unsigned b = blockIdx.x;
    const int o = b >= m.first[1];
    fft2d_c2r_rect_body<LH, GH, LW, GW>(m.op[o], b - m.first[o]);
}

// Tile and bin count of the plane-tiled layout of a rectangular basis.
inline int rect_tile_log2(int nr, int nc) { return (nr >= 18 || nc >= 18) ? 4 : 5; }
inline int rect_layout_bins(int nr, int nc) { return (nr * (nc / 2 + 1) + 7) / 8 * 8; }

template <int LH, int GH, int LW, int GW>
static RectFwdParams make_fwd_rect(const FwdOperand &op, size_t *lds) {
    typedef RectShape<LH, GH, LW, GW> S;
    const int h_in = op.h_in, w_in = op.w_in;
    RectFwdParams prm;
    prm.in = op.in; prm.out = op.out; prm.planes = op.planes; prm.h_in = h_in; prm.w_in = w_in;
    prm.RS = w_in | 1;
    prm.IPS = (h_in * prm.RS) | 1;
    prm.MPS = (h_in * S::MRS) | 1;
    prm.vecw = (((size_t)op.in & 15) == 0 && w_in % 4 == 0) ? 4 : ((((size_t)op.in & 7) == 0 && w_in % 2 == 0) ? 2 : 1);
    prm.div_wv = make_magic((unsigned)(w_in / prm.vecw));
    prm.div_h = make_magic((unsigned)h_in);
    prm.lay.tsh = rect_tile_log2(S::NR, S::NC);
    prm.lay.bins = rect_layout_bins(S::NR, S::NC);
    prm.linear = (prm.RS == w_in && prm.IPS == h_in * w_in) ? 1 : 0;
    const size_t a = ((size_t)S::T * prm.IPS + S::NC + 4) * sizeof(float), b = (size_t)S::T * prm.MPS * sizeof(float2);
    *lds = a > b ? a : b;
    return prm;
}

// One or two operand tensors (whole planes) in one launch.
template <int LH, int GH, int LW, int GW>
static hipError_t run_fwd_rect(const FwdOperand *ops, int nops, LaunchCtx st) {
    typedef RectShape<LH, GH, LW, GW> S;
    RectFwdPair m;
    size_t lds = 0;
    unsigned blocks = 0;
    for (int o = 0; o < 2; ++o) {
        m.first[o] = blocks;
        if (o < nops) {
            size_t l;
            m.op[o] = make_fwd_rect<LH, GH, LW, GW>(ops[o], &l);
            if (l > lds) lds = l;
            blocks += (unsigned)((ops[o].planes + S::T - 1) / S::T);
        } else {
            m.op[o] = m.op[0];
        }
    }
    m.first[2] = blocks;
    if (blocks == 0) return hipSuccess;
    auto k = fft2d_r2c_rect_kernel<LH, GH, LW, GW>;
    if (hipError_t e = allow_big_lds((const void *)k, lds); e != hipSuccess) return e;
    launch_kernel(k, dim3(blocks), dim3(S::BT), lds, st, m);
    return hipGetLastError();
}

template <int LH, int GH, int LW, int GW>
static RectInvParams make_inv_rect(const float *in, float *out, long planes, int h_out, int w_out, float scale,
                                   bool accumulate, size_t *lds) {
    typedef RectShape<LH, GH, LW, GW> S;
    RectInvParams prm;
    prm.in = in; prm.out = out; prm.planes = planes; prm.h_out = h_out; prm.w_out = w_out;
    prm.MPS = (h_out * S::MRS) | 1;
    prm.lay.tsh = rect_tile_log2(S::NR, S::NC);
    prm.lay.bins = rect_layout_bins(S::NR, S::NC);
    prm.scale = scale; prm.accumulate = accumulate ? 1 : 0;
    const size_t a = (size_t)S::T * prm.MPS * sizeof(float2), b = ((size_t)S::T * h_out * w_out + 3) * sizeof(float);
    *lds = a > b ? a : b;
    return prm;
}

template <int LH, int GH, int LW, int GW>
static hipError_t run_inv_rect(const float *in, float *out, long planes, int h_out, int w_out, float scale,
                               bool accumulate, LaunchCtx st) {
    typedef RectShape<LH, GH, LW, GW> S;
    size_t lds;
    const RectInvParams prm = make_inv_rect<LH, GH, LW, GW>(in, out, planes, h_out, w_out, scale, accumulate, &lds);
    auto k = fft2d_c2r_rect_kernel<LH, GH, LW, GW>;
    if (hipError_t e = allow_big_lds((const void *)k, lds); e != hipSuccess) return e;
    launch_kernel(k, dim3((unsigned)((planes + S::T - 1) / S::T)), dim3(S::BT), lds, st, prm);
    return hipGetLastError();
}

template <int LH, int GH, int LW, int GW>
static hipError_t run_inv_rect_pair(const InvOperand *ops, LaunchCtx st) {
    typedef RectShape<LH, GH, LW, GW> S;
    RectInvPair m;
    size_t lds = 0;
    unsigned blocks = 0;
    for (int o = 0; o < 2; ++o) {
        size_t l;
        m.first[o] = blocks;
        m.op[o] = make_inv_rect<LH, GH, LW, GW>(ops[o].in, ops[o].out, ops[o].planes, ops[o].h_out, ops[o].w_out,
                                                ops[o].scale, ops[o].accumulate, &l);
        if (l > lds) lds = l;
        blocks += (unsigned)((ops[o].planes + S::T - 1) / S::T);
    }
    m.first[2] = blocks;
    if (blocks == 0) return hipSuccess;
    auto k = fft2d_c2r_rect_pair_kernel<LH, GH, LW, GW>;
    if (hipError_t e = allow_big_lds((const void *)k, lds); e != hipSuccess) return e;
    launch_kernel(k, dim3(blocks), dim3(S::BT), lds, st, m);
    return hipGetLastError();
}

// Registers per lane and lanes per line of a side of the basis: one lane up to 16, two above.
template <int N> struct RectSide { static constexpr int G = N <= 16 ? 1 : 2, L = N / G; };

// Calls f(<NR>, <NC>) for the pair of supported sides (8 .. 32), or returns false.
template <class F>
static bool rect_dispatch(int nr, int nc, F &&f) {
    auto cols = [&](auto R) -> bool {
        constexpr int NR = decltype(R)::value;
        switch (nc) {
#define RECT_COL(NC_) case NC_: if constexpr (NR != NC_) { f(R, std::integral_constant<int, NC_>{}); return true; } return false;
            RECT_COL(8) RECT_COL(10) RECT_COL(12) RECT_COL(14) RECT_COL(16) RECT_COL(18) RECT_COL(20) RECT_COL(24) RECT_COL(28) RECT_COL(32)
#undef RECT_COL
            default: return false;
        }
    };
    switch (nr) {
#define RECT_ROW(NR_) case NR_: return cols(std::integral_constant<int, NR_>{});
        RECT_ROW(8) RECT_ROW(10) RECT_ROW(12) RECT_ROW(14) RECT_ROW(16) RECT_ROW(18) RECT_ROW(20) RECT_ROW(24) RECT_ROW(28) RECT_ROW(32)
#undef RECT_ROW
        default: return false;
    }
}

}  // namespace fc
