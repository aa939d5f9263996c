// Batched small real FFT kernels for gfx950 as templates over (L, G, T): 2-D R2C, 2-D C2R with
// crop, 1-D R2C, 1-D C2R, and the host-side launch helpers that size their LDS.  The .hip
// files that include this header instantiate them for their share of the supported sizes.
//
// What is computed: Section 5 of the fbfft paper (batched 1-D / 2-D FFTs with implicit zero
// padding by clipped loads, Hermitian-half output, two real lines packed into one complex
// transform, n/2 instead of n/2+1 column transforms), and the clipped inverse of Section 3.1.
// How: one workgroup owns T consecutive planes; planes are staged through LDS with coalesced
// global accesses, each lane (or group of G lanes) transforms a whole line of N = L*G points in
// registers (fft_core.hpp), and the row <-> column transpose is an LDS round trip.
#pragma once
#include "fft_core.hpp"
#include "kernels.hpp"

namespace fc {

// ------------------------------------------------------------------ small helpers
struct MagicDiv {
    unsigned long long m;   // ceil(2^32 / d); exact quotient for x * d < 2^32
};
static inline MagicDiv make_magic(unsigned d) { return MagicDiv{((1ull << 32) + d - 1) / d}; }
__device__ __forceinline__ unsigned mdiv(unsigned x, MagicDiv md) {
    return (unsigned)(((unsigned long long)x * md.m) >> 32);
}

// Bank layout of the row-transformed data ("mid") that the 2-D kernels keep in LDS between their
// two phases, rows of N/2 float2.  With G >= 4 lanes per line, G lanes of a half-wave work on
// the same column of G rows (forward: consecutive rows; inverse: rows L apart) or on G blocks of
// L entries of one row; with a row stride of N/2 (a multiple of 16 from N = 64 on) they would
// all meet on one bank pair.  Measured on the stand-alone 128x128 forward kernel: 80 % of the
// LDS cycles were bank conflicts.  Three paddings, none for G < 4:
//   row stride:  G consecutive rows spread evenly over the banks: stride 4 or 12 modulo 16
//                float2 (rows 8 banks apart), for G = 4 also 8 (16 banks apart);
//   slot (forward, G = 8): entry s of a row sits at s + s / L, one float2 between blocks;
//   row block (inverse): row a sits (a / L) * RP float2 further, RP = 32 / G.
template <int L, int G>
struct MidLayout {
    static constexpr int N = L * G, NH = N / 2;
    static constexpr bool slots = (G == 8);
    static constexpr int need = NH + (slots ? NH / L : 0);
    static constexpr int pick() {
        if (G < 4) return NH;
        for (int v = need;; ++v)
            if (v % 16 == 4 || v % 16 == 12 || (G == 4 && v % 16 == 8)) return v;
    }
    static constexpr int MRS = pick();                 // row stride, float2
    static constexpr int RP = (G < 4) ? 0 : 32 / G;    // inverse: extra float2 per block of L rows
    __host__ __device__ static constexpr int slot(int s) { return slots ? s + s / L : s; }
    __host__ __device__ static constexpr int row(int a) { return a * MRS + (a / L) * RP; }
    // float2 per plane for h rows: forward (no row blocks) and inverse
    static constexpr int fwd_plane(int h) { return h * MRS; }
    static constexpr int inv_plane(int h) { return h * MRS + (h / L + 1) * RP; }
};

// Floats by which a global address lies past a 16-byte boundary (0..3).
__device__ __forceinline__ unsigned misalign4(const float *p) { return (unsigned)(((size_t)p >> 2) & 3); }

// Copy `total` contiguous floats from global memory into LDS at the same offsets.  Loads are
// issued in batches of U per lane before any LDS store so that many are in flight at once;
// 16-byte loads are used when `vec_ok`: dst and src lie equally far past a 16-byte boundary
// (the caller shifts its LDS image by misalign4(src)); the up to 3 floats before the first
// boundary and after the last one are copied singly.
template <int BT, int U = 8>
__device__ __forceinline__ void stage_linear(float *dst, const float *src, unsigned total, int tid,
                                             bool vec_ok) {
    unsigned done = 0;
    if (vec_ok) {
        unsigned head = (4 - misalign4(src)) & 3;
        if (head > total) head = total;
        if ((unsigned)tid < head) dst[tid] = src[tid];
        const unsigned total4 = (total - head) >> 2;
        const float4 *s4 = reinterpret_cast<const float4 *>(src + head);
        float4 *d4 = reinterpret_cast<float4 *>(dst + head);
        for (unsigned base = tid; base < total4; base += BT * U) {
            float4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const unsigned i = base + u * BT;
                v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (i < total4) v[u] = s4[i];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const unsigned i = base + u * BT;
                if (i < total4) d4[i] = v[u];
            }
        }
        done = head + (total4 << 2);
    }
    for (unsigned base = done + tid; base < total; base += BT * U) {
        float v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const unsigned i = base + u * BT;
            v[u] = 0.f;
            if (i < total) v[u] = src[i];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const unsigned i = base + u * BT;
            if (i < total) dst[i] = v[u];
        }
    }
}

// Copy `total` floats from LDS to contiguous global memory (optionally accumulating); vec_ok
// as for stage_linear, with the roles of dst and src exchanged.
template <int BT>
__device__ __forceinline__ void unstage_linear(float *dst, const float *src, unsigned total, int tid,
                                               bool vec_ok, bool accumulate) {
    unsigned done = 0;
    if (vec_ok && !accumulate) {
        unsigned head = (4 - misalign4(dst)) & 3;
        if (head > total) head = total;
        if ((unsigned)tid < head) dst[tid] = src[tid];
        const unsigned total4 = (total - head) >> 2;
        const float4 *s4 = reinterpret_cast<const float4 *>(src + head);
        float4 *d4 = reinterpret_cast<float4 *>(dst + head);
        for (unsigned i = tid; i < total4; i += BT) d4[i] = s4[i];
        done = head + (total4 << 2);
    }
    if (accumulate) {
        for (unsigned i = done + tid; i < total; i += BT) dst[i] += src[i];
    } else {
        for (unsigned i = done + tid; i < total; i += BT) dst[i] = src[i];
    }
}


// Copy a contiguous block of `rows` rows of w floats (consecutive planes of h rows each) into
// an LDS image with padded strides (row stride rs, plane stride ps), V floats per load
// (V divides w; the block start is V*4-byte aligned).  Batched like stage_linear.
// FPL: floats per lane of the largest block the kernel can be given (2 N / G).  The batch is
// sized so that such a block is in flight as ONE batch of up to sixteen loads per lane (four
// 64 x 64 planes on 256 lanes: sixteen 16-byte loads): a second batch would wait for the first
// one's round trip to memory before it is even issued.
template <int BT, int V, int FPL>
__device__ __forceinline__ void stage_padded(float *dst, const float *src, unsigned rows, unsigned w,
                                             unsigned h, unsigned rs, unsigned ps, MagicDiv div_wv,
                                             MagicDiv div_h, int tid) {
    constexpr int U = FPL / V < 4 ? 4 : (FPL / V > 16 ? 16 : FPL / V);
    typedef float vec_t __attribute__((ext_vector_type(V)));
    const unsigned wv = w / V, total = rows * wv;
    const vec_t *sv = reinterpret_cast<const vec_t *>(src);
    for (unsigned base = tid; base < total; base += BT * U) {
        vec_t v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const unsigned e = base + u * BT;
            v[u] = vec_t(0.f);
            if (e < total) v[u] = sv[e];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const unsigned e = base + u * BT;
            if (e < total) {
                const unsigned row = mdiv(e, div_wv);
                const unsigned c = (e - row * wv) * V;
                const unsigned pl = mdiv(row, div_h);
                float *d = dst + pl * ps + (row - pl * h) * rs + c;
#pragma unroll
                for (int q = 0; q < V; ++q) d[q] = v[u][q];
            }
        }
    }
}

// ------------------------------------------------------------------ tiled operands
// Image offset and window origin (before the view's oy / ox) of plane p of a tiled operand.
struct PlaneOrigin {
    long long base;
    int y0, x0;
};
__device__ __forceinline__ PlaneOrigin plane_origin(const PlaneView &v, long p) {
    const long m = p / v.C;
    const int ch = (int)(p - m * v.C);
    const long q = m / v.ntx;
    const int tx = (int)(m - q * v.ntx);
    const long s = q / v.nty;
    const int ty = (int)(q - s * v.nty);
    const int cimg = v.Cimg ? v.Cimg : v.C;
    return PlaneOrigin{((s * cimg + ch) * (long long)v.H) * v.W, ty * v.dy, tx * v.dx};
}

// Per-workgroup table of the origins of its np planes, kept in LDS at `info`
// (T x 16 bytes: bases, then y0, then x0).
template <int T>
struct OriginTable {
    long long *base;
    int *y0, *x0;
    __device__ __forceinline__ explicit OriginTable(float *info)
        : base(reinterpret_cast<long long *>(info)), y0(reinterpret_cast<int *>(info + 2 * T)), x0(y0 + T) {}
    __device__ __forceinline__ void fill(const PlaneView &v, long p0, int np, int tid) {
        if (tid < np) {
            const PlaneOrigin o = plane_origin(v, p0 + tid);
            base[tid] = o.base; y0[tid] = o.y0; x0[tid] = o.x0;
        }
        __syncthreads();
    }
};

// Gather the h x w windows of np planes into an LDS image with row stride rs and plane
// stride ps; elements outside the H x W image become 0.  V floats per load: V = 4 needs every
// window column origin, W, w and the image base to be multiples of 4 floats, so that a
// group of 4 lies wholly inside or outside the image and is 16-byte aligned; div_w divides
// by w / V.
template <int BT, int T, int V>
__device__ __forceinline__ void stage_windows(float *dst, const float *img, const PlaneView &v,
                                              const OriginTable<T> &tab, int np, unsigned h, unsigned w,
                                              unsigned rs, unsigned ps, MagicDiv div_w, MagicDiv div_h, int tid) {
    constexpr int U = (V == 1) ? 8 : 4;
    typedef float vec_t __attribute__((ext_vector_type(V)));
    const unsigned wv = w / V, total = (unsigned)np * h * wv;
    for (unsigned b = tid; b < total; b += BT * U) {
        vec_t val[U];
        unsigned off[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const unsigned e = b + u * BT;
            val[u] = vec_t(0.f); off[u] = 0;
            if (e < total) {
                const unsigned row = mdiv(e, div_w);
                const unsigned c = (e - row * wv) * V;
                const unsigned pl = mdiv(row, div_h);
                const unsigned r = row - pl * h;
                off[u] = pl * ps + r * rs + c;
                const int gy = tab.y0[pl] + v.oy + (int)r, gx = tab.x0[pl] + v.ox + (int)c;
                if ((unsigned)gy < (unsigned)v.H && (unsigned)gx < (unsigned)v.W)
                    val[u] = *reinterpret_cast<const vec_t *>(img + tab.base[pl] + (long long)gy * v.W + gx);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (b + u * BT < total) {
#pragma unroll
                for (int q = 0; q < V; ++q) dst[off[u] + q] = val[u][q];
            }
    }
}

// Scatter the h x w windows at offset (oy, ox) of an LDS image of np planes of sh x sw floats
// to their places in the H x W images; elements outside the image are dropped.  V = 4 under the
// same alignment conditions as for the gather, plus sw and ox multiples of 4.
template <int BT, int T, int V>
__device__ __forceinline__ void unstage_windows(float *img, const float *src, const PlaneView &v,
                                                const OriginTable<T> &tab, int np, unsigned h, unsigned w,
                                                unsigned sh, unsigned sw, MagicDiv div_w, MagicDiv div_h,
                                                int tid, bool accumulate) {
    typedef float vec_t __attribute__((ext_vector_type(V)));
    const unsigned wv = w / V, total = (unsigned)np * h * wv;
    for (unsigned e = tid; e < total; e += BT) {
        const unsigned row = mdiv(e, div_w);
        const unsigned c = (e - row * wv) * V;
        const unsigned pl = mdiv(row, div_h);
        const unsigned r = row - pl * h;
        const int gy = tab.y0[pl] + (int)r, gx = tab.x0[pl] + (int)c;
        if (gy < v.H && gx < v.W) {
            vec_t *d = reinterpret_cast<vec_t *>(img + tab.base[pl] + (long long)gy * v.W + gx);
            const vec_t val = *reinterpret_cast<const vec_t *>(src + (pl * sh + r + v.oy) * sw + c + v.ox);
            if (accumulate) *d += val; else *d = val;
        }
    }
}

// ------------------------------------------------------------------ 2-D forward
struct Fwd2dParams {
    const float *in;
    float *out;
    long planes;
    int h_in, w_in;
    int RS, IPS;      // LDS row / plane stride of the staged input (floats, odd)
    int MPS;          // LDS plane stride of the row-transformed data (float2, odd)
    MagicDiv div_wv, div_h;   // row length in load vectors, rows per plane
    int vecw;                 // floats per staging load when the image is padded: 4, 2 or 1
    FreqLayout lay;
    int linear;       // staged planes need no padding: LDS image == global image
    int vec_ok;       // (unused by the linear staging, which adapts to the block's alignment)
    int out_vec_ok;   // output base and every block start are 16-byte aligned
    int tiled;        // planes are windows of images (view); origin table at LDS float info_off
    int info_off;
    int tw_off;       // lines of four or eight lanes: twiddle table at LDS float tw_off
    PlaneView view;
};

// How the forward kernels write the plane-tiled layout.  With runs of 16 planes or more a lane's
// 4-byte stores fill whole 64-byte segments.  With short runs (8 planes at basis 32, 4 from 36 on)
// the same stores are 16- or 32-byte pieces at twice that stride, half of every 64-byte request
// empty, and the time goes into issuing them: on the 64-basis layer the stores were 40 % of the
// weight transform's time (85 us with, 52 us without them; a plain fill of as many bytes takes
// 43).  There the two lanes of a pair swap halves, so that one instruction writes the real and
// the imaginary run of a bin side by side (85 -> 74 us; assembling the block in LDS and writing it
// with linear 16-byte stores, in halves to keep the occupancy, came to 76 and cost the smaller
// transforms 10 .. 25 %).
template <int G, int T> constexpr bool kPairedStores = (G > 1) && (T <= 8);

// Store helpers for the two output layouts.  `base` is uniform over the workgroup (block
// or LDS image start) and the lane's part of the address is a 32-bit element offset, so that a
// store costs one 32-bit add instead of 64-bit pointer arithmetic.
template <int N, int T, bool CONV>
struct BinStore {
    float *base;
    unsigned lane_off;  // CONV: plane within the tile; natural: plane * N * (N/2+1) (in float2)
    __device__ __forceinline__ void operator()(int k1, int k2, float re, float im) const {
        constexpr int NB = N / 2 + 1;
        if constexpr (CONV) {
            const unsigned idx = lane_off + (unsigned)((k1 * NB + k2) * 2) * T;
            base[idx] = re;
            base[idx + T] = im;
        } else {
            reinterpret_cast<float2 *>(base)[lane_off + (unsigned)(k1 * NB + k2)] = make_float2(re, im);
        }
    }
};

// KEEP (with CONV and OSTAGE): stop once the block's spectra stand in LDS, as the image
// smem[(bin * 2 + c) * T + plane], and leave them there for the caller (after a barrier).
// tid_sub / lds_off: a part of a larger workgroup (BT consecutive threads, numbered from 0 in
// tid_sub) runs the transform in its own part of LDS, lds_off floats (a multiple of 4) from the
// start; every thread of the workgroup must then make a call of this function, since its barriers
// are the workgroup's.
template <int L, int G, int T, bool CONV, bool OSTAGE, bool KEEP = false>
__device__ __forceinline__ void fft2d_r2c_body(const Fwd2dParams &prm, unsigned block, int tid_sub = -1,
                                               unsigned lds_off = 0) {
    static_assert(!KEEP || (CONV && OSTAGE), "KEEP leaves the plane-tiled image in LDS");
    constexpr int N = L * G, NH = N / 2, NB = NH + 1, BT = T * NH * G, MRS = MidLayout<L, G>::MRS;
    constexpr int NA = SplitRegs<L, G>::A;   // registers of split spectrum per lane
    constexpr int NBR = SplitRegs<L, G>::B;
    extern __shared__ float smem_dyn[];
    float *const smem = smem_dyn + lds_off;
    float *sin = smem;
    float2 *mid = reinterpret_cast<float2 *>(smem);

    const int tid = tid_sub < 0 ? (int)threadIdx.x : tid_sub;
    const long p0 = (long)block * T;
    const int h_in = prm.h_in, w_in = prm.w_in, hw = h_in * w_in;
    const long left = prm.planes - p0;
    const int np = left < T ? (int)left : T;

    load_group_twiddles<L, G, BT>(smem + prm.tw_off, tid);   // used after the next barrier
    // ---- stage the contiguous block of np planes into LDS (coalesced reads)
    bool windows = false;
    if constexpr (CONV) windows = prm.tiled != 0;   // only the plane-tiled layout is used with views
    if (windows) {
        OriginTable<T> tab(smem + prm.info_off);
        tab.fill(prm.view, p0, np, tid);
        if (prm.vecw == 4)
            stage_windows<BT, T, 4>(sin, prm.in, prm.view, tab, np, h_in, w_in, prm.RS, prm.IPS, prm.div_wv,
                                    prm.div_h, tid);
        else
            stage_windows<BT, T, 1>(sin, prm.in, prm.view, tab, np, h_in, w_in, prm.RS, prm.IPS, prm.div_wv,
                                    prm.div_h, tid);
    } else {
        const float *src = prm.in + p0 * hw;
        if (prm.linear) {
            sin = smem + misalign4(src);   // the LDS image shares the block's 16-byte phase
            stage_linear<BT>(sin, src, (unsigned)np * hw, tid, true);
        } else {
            const unsigned rows = (unsigned)np * h_in;
            constexpr int FPL = 2 * N / G;
            if (prm.vecw == 4)
                stage_padded<BT, 4, FPL>(sin, src, rows, w_in, h_in, prm.RS, prm.IPS, prm.div_wv, prm.div_h, tid);
            else if (prm.vecw == 2)
                stage_padded<BT, 2, FPL>(sin, src, rows, w_in, h_in, prm.RS, prm.IPS, prm.div_wv, prm.div_h, tid);
            else
                stage_padded<BT, 1, FPL>(sin, src, rows, w_in, h_in, prm.RS, prm.IPS, prm.div_wv, prm.div_h, tid);
        }
    }
    __syncthreads();

    // ---- row phase: lane (pair) = (plane p, rows ra and rb packed as ra + i rb)
    const int H2 = (h_in + 1) >> 1;
    const int g = tid % G, p = (tid / G) % T, rp = tid / (G * T);
    const bool row_active = rp < H2 && p < np;
    const int ra = rp, rb = rp + H2;
    const bool hasb = rb < h_in;
    float are[NA], aim[NA], bre[NBR], bim[NBR];
    if (row_active) {
        float re[L], im[L];
        // (Conditional reads: the compiler turns them into uniform branches that skip the
        // loads of the zero padding; measured faster than unconditional reads plus selects,
        // which cost registers and occupancy on the two-lane kernels.)
        const float *pa = sin + p * prm.IPS + ra * prm.RS;
        const float *pb = sin + p * prm.IPS + rb * prm.RS;
#pragma unroll
        for (int m = 0; m < L; ++m) {
            const int j = g + G * m;
            const bool in = j < w_in;
            re[m] = in ? pa[j] : 0.0f;
            im[m] = (in && hasb) ? pb[j] : 0.0f;
        }
        fft_lines<L, G, -1>(re, im, g, smem + prm.tw_off);
        split_two_real<L, G, kDeferHalf<G>>(re, im, g, are, aim, bre, bim);   // (doubled: halved in the column phase)
    }
    __syncthreads();   // every lane has read its rows; the staging area may be overwritten
    if (row_active) {
        float2 *mp = mid + p * prm.MPS;
        if constexpr (G == 1) {
#pragma unroll
            for (int k = 0; k < NH; ++k) mp[ra * MRS + k] = make_float2(are[k], aim[k]);
            if (hasb) {
#pragma unroll
                for (int k = 0; k < NH; ++k) mp[rb * MRS + k] = make_float2(bre[k], bim[k]);
            }
        } else {
            const int row = (g & 1) ? rb : ra;
            if (!(g & 1) || hasb) {
#pragma unroll
                for (int k = 0; k < L; ++k)
                    mp[row * MRS + MidLayout<L, G>::slot(split_slot<L, G>(g, k))] = make_float2(are[k], aim[k]);
            }
        }
    }
    __syncthreads();

    // ---- column phase: lane (pair) = (plane cp, column slot cc); slot 0 is the packed pair
    //      of real columns k2 = 0 and k2 = N/2.
    int cg, cp, cc;
    if constexpr (CONV) { cg = tid % G; cp = (tid / G) % T; cc = tid / (G * T); }
    else { cg = tid % G; cc = (tid / G) % NH; cp = tid / (G * NH); }
    const bool col_active = cp < np;

    float re[L], im[L];
    if (col_active) {
        const float2 *mp = mid + cp * prm.MPS + MidLayout<L, G>::slot(cc);
#pragma unroll
        for (int m = 0; m < L; ++m) {
            const int r = cg + G * m;
            float2 v = make_float2(0.f, 0.f);
            if (r < h_in) v = mp[r * MRS];
            re[m] = v.x; im[m] = v.y;
        }
        fft_lines<L, G, -1, kDeferHalf<G>>(re, im, cg, smem + prm.tw_off);
    }

    // Results go either straight to global memory or, when OSTAGE, into an LDS image of the
    // block's output (which is one contiguous range in both layouts) that is then written
    // out with 16-byte coalesced stores.
    BinStore<N, T, CONV> st;
    st.lane_off = CONV ? (unsigned)cp : (unsigned)cp * N * NB;
    if constexpr (OSTAGE) {
        __syncthreads();   // every lane has read `mid`; the image overlays it
        st.base = smem;
    } else {
        if constexpr (CONV) st.base = prm.out + prm.lay.index(p0, 0, 0);
        else st.base = prm.out + (size_t)p0 * N * NB * 2;
    }

    if (col_active) {
        if (cc != 0) {
            if constexpr (CONV && !OSTAGE && kPairedStores<G, T>) {
                // The two lanes of a pair (cg, cg ^ 1) hold the same bins k2 of two different rows.
                // They swap halves: the even lane writes the real parts of both rows, the odd lane
                // the imaginary parts, so that one store instruction fills the real and the
                // imaginary run of a bin, and with the neighbouring columns whole 64-byte segments.
                const bool odd = (cg & 1) != 0;
                const int row_e = L * group_block<G>(cg & ~1), row_o = L * group_block<G>(cg | 1);
                float *pe = st.base + st.lane_off + (unsigned)(((row_e * NB + cc) * 2 + (odd ? 1 : 0)) * T);
                float *po = st.base + st.lane_off + (unsigned)(((row_o * NB + cc) * 2 + (odd ? 1 : 0)) * T);
#pragma unroll
                for (int k = 0; k < L; ++k) {
                    const float got = lane_xor1(odd ? re[k] : im[k]);
                    pe[(k * NB * 2) * T] = odd ? got : re[k];
                    po[(k * NB * 2) * T] = odd ? im[k] : got;
                }
            } else {
#pragma unroll
                for (int k = 0; k < L; ++k) st(k + L * group_block<G>(cg), cc, re[k], im[k]);
            }
        } else {
            float ur[NA], ui[NA], vr[NBR], vi[NBR];
            split_two_real<L, G>(re, im, cg, ur, ui, vr, vi);
            if constexpr (G == 1) {
                st(0, 0, ur[0], 0.f);  st(NH, 0, ui[0], 0.f);
                st(0, NH, vr[0], 0.f); st(NH, NH, vi[0], 0.f);
#pragma unroll
                for (int k = 1; k < NH; ++k) {
                    st(k, 0, ur[k], ui[k]);  st(N - k, 0, ur[k], -ui[k]);
                    st(k, NH, vr[k], vi[k]); st(N - k, NH, vr[k], -vi[k]);
                }
            } else {
                // even lanes hold the spectrum of column 0, odd lanes that of column N/2
                const int k2 = (cg & 1) ? NH : 0;
#pragma unroll
                for (int k = 0; k < L; ++k) {
                    const int k1 = split_slot<L, G>(cg, k);
                    if (k1 == 0) {                       // packed real bins 0 and N/2
                        st(0, k2, ur[k], 0.f);
                        st(NH, k2, ui[k], 0.f);
                    } else {
                        st(k1, k2, ur[k], ui[k]);
                        st(N - k1, k2, ur[k], -ui[k]);
                    }
                }
            }
        }
    }
    if constexpr (OSTAGE) {
        __syncthreads();
        if constexpr (KEEP) return;
        if constexpr (CONV) {
            // whole tile, including the padding planes of a ragged last tile
            unstage_linear<BT>(prm.out + prm.lay.index(p0, 0, 0), smem, (unsigned)T * N * NB * 2, tid,
                               prm.out_vec_ok != 0, false);
        } else {
            unstage_linear<BT>(prm.out + (size_t)p0 * N * NB * 2, smem, (unsigned)np * N * NB * 2, tid,
                               prm.out_vec_ok != 0, false);
        }
    }
}

template <int L, int G, int T, bool CONV, bool OSTAGE>
__global__ void __launch_bounds__(T *(L * G / 2) * G) fft2d_r2c_kernel(Fwd2dParams prm) {
    fft2d_r2c_body<L, G, T, CONV, OSTAGE>(prm, blockIdx.x);
}

// Up to three operand tensors transformed by one launch (plane-tiled layout only): the blocks
// of operand o are [first[o], first[o+1]).  Short transforms of several operands fill the chip
// together instead of queueing behind each other's ramp-up and tail.
struct FwdMultiParams {
    Fwd2dParams op[3];
    unsigned first[4];
};

template <int L, int G, int T>
__global__ void __launch_bounds__(T *(L * G / 2) * G) fft2d_r2c_multi_kernel(FwdMultiParams m) {
    const unsigned b = blockIdx.x;
    const int o = (b >= m.first[1]) + (b >= m.first[2]);
    fft2d_r2c_body<L, G, T, true, false>(m.op[o], b - m.first[o]);
}

// ------------------------------------------------------------------ 2-D inverse + crop
struct Inv2dParams {
    const float *in;
    float *out;
    long planes;
    int h_out, w_out;
    int MPS;          // LDS plane stride of the column-transformed data (float2, odd)
    FreqLayout lay;
    float scale;
    int accumulate;
    int vec_ok;       // tiled outputs: the windows can be scattered with 16-byte stores
    int in_vec_ok;    // natural layout only: input base is 16-byte aligned
    int tiled;        // outputs are windows of images (view); origin table at LDS float info_off
    int info_off;
    int win_h, win_w; // tiled: size of the window taken at (view.oy, view.ox) of the h_out x w_out block
    int tw_off;       // lines of four or eight lanes: twiddle table at LDS float tw_off
    MagicDiv div_w, div_h;
    PlaneView view;
};

// PRE (plane-tiled layout only): the block's input already stands in LDS at pre_img, laid out
// like one tile of the layout ((bin * 2 + c) * T + plane), beyond the first
// max(T * MPS float2, T * h_out * w_out + 3 floats) of LDS, which this function uses.
// tid_sub: as for the forward body (threads of a larger workgroup beyond the BT that do the work call
// with a plan of no planes and still pass the barriers).
template <int L, int G, int T, bool CONV, bool ISTAGE, bool PRE = false>
__device__ __forceinline__ void fft2d_c2r_body(const Inv2dParams &prm, unsigned block, const float *pre_img = nullptr,
                                               int tid_sub = -1) {
    static_assert(!PRE || (CONV && !ISTAGE), "a preloaded tile is in the plane-tiled layout and needs no staging");
    constexpr int N = L * G, NH = N / 2, NB = NH + 1, BT = T * NH * G;
    typedef MidLayout<L, G> ML;
    extern __shared__ float smem[];
    float2 *mid = reinterpret_cast<float2 *>(smem);

    const int tid = tid_sub < 0 ? (int)threadIdx.x : tid_sub;
    const long p0 = (long)block * T;
    // the output block assembled in LDS shares the 16-byte phase of its place in global memory
    // (contiguous outputs only; scattered windows keep an aligned image)
    float *sout = smem;
    if (!(CONV && prm.tiled)) sout += misalign4(prm.out + p0 * (long)prm.h_out * prm.w_out);
    const long left = prm.planes - p0;
    const int np = left < T ? (int)left : T;
    const int h_out = prm.h_out, w_out = prm.w_out;

    // ---- column phase (inverse along k1) for column slot cc of plane cp.  In the natural
    //      layout the block's input is one contiguous range: bring it into LDS with wide
    //      coalesced loads first, then pick the strided column elements out of LDS.
    {
        int cg, cp, cc;
        if constexpr (CONV) { cg = tid % G; cp = (tid / G) % T; cc = tid / (G * T); }
        else { cg = tid % G; cc = (tid / G) % NH; cp = tid / (G * NH); }
        if constexpr (kLdsTwiddles<G>) {
            load_group_twiddles<L, G, BT>(smem + prm.tw_off, tid);
            if constexpr (!ISTAGE) __syncthreads();   // (the staging below ends with a barrier)
        }
        if constexpr (ISTAGE) {
            if constexpr (CONV)   // whole tile (its padding planes are simply not used)
                stage_linear<BT>(smem, prm.in + prm.lay.index(p0, 0, 0), (unsigned)T * N * NB * 2, tid,
                                 prm.in_vec_ok != 0);
            else
                stage_linear<BT>(smem, prm.in + (size_t)p0 * N * NB * 2, (unsigned)np * N * NB * 2, tid,
                                 prm.in_vec_ok != 0);
            __syncthreads();
        }
        float cre[L], cim[L];
        if (cp < np) {
            if constexpr (CONV) {
                const float *base = (PRE ? pre_img : ISTAGE ? smem : prm.in + prm.lay.index(p0, 0, 0)) + cp;
                const int tsh = prm.lay.tsh;
#pragma unroll
                for (int m = 0; m < L; ++m) {
                    const int k1 = cg + G * m;
                    const float *q = base + ((size_t)((k1 * NB + cc) * 2) << tsh);
                    float xr = q[0], xi = q[(size_t)1 << tsh];
                    if (cc == 0) {   // pack columns 0 and N/2:  z = y0 + i yN
                        const float *qn = base + ((size_t)((k1 * NB + NH) * 2) << tsh);
                        const float nr = qn[0], ni = qn[(size_t)1 << tsh];
                        xr -= ni; xi += nr;
                    }
                    cre[m] = xr; cim[m] = xi;
                }
            } else {
                const float2 *base = reinterpret_cast<const float2 *>(smem) + cp * N * NB;
#pragma unroll
                for (int m = 0; m < L; ++m) {
                    const int k1 = cg + G * m;
                    float2 v = base[k1 * NB + cc];
                    if (cc == 0) {
                        const float2 u = base[k1 * NB + NH];
                        v.x -= u.y; v.y += u.x;
                    }
                    cre[m] = v.x; cim[m] = v.y;
                }
            }
            fft_lines<L, G, +1>(cre, cim, cg, smem + prm.tw_off);
        }
        if constexpr (ISTAGE) __syncthreads();   // staged input fully consumed; `mid` overlays it
        if (cp < np) {
            // row a = k + L * block: k rows plus `block` whole blocks of L rows
            const int blk = group_block<G>(cg);
            float2 *mp = mid + cp * prm.MPS + cc + blk * (L * ML::MRS + ML::RP);
#pragma unroll
            for (int k = 0; k < L; ++k) {
                if (k + L * blk < h_out) mp[k * ML::MRS] = make_float2(cre[k], cim[k]);
            }
        }
    }
    __syncthreads();

    // ---- row phase (inverse along k2), rows ra and rb packed as ra + i rb
    const int H2 = (h_out + 1) >> 1;
    const int g = tid % G, p = (tid / G) % T, rp = tid / (G * T);
    const bool active = rp < H2 && p < np;
    const int ra = rp, rb = rp + H2;
    const bool hasb = rb < h_out;
    float re[L], im[L];
    if (active) {
        const float2 *A = mid + p * prm.MPS + ML::row(ra);
        const float2 *B = mid + p * prm.MPS + ML::row(hasb ? rb : ra);
#pragma unroll
        for (int m = 0; m < L; ++m) {
            const int k2 = g + G * m;
            const int slot = (k2 == NH) ? 0 : (k2 < NH ? k2 : N - k2);
            const float2 a = A[slot];
            float2 b = B[slot];
            if (!hasb) b = make_float2(0.f, 0.f);
            float xr, xi;
            if (k2 == 0) { xr = a.x; xi = b.x; }
            else if (k2 == NH) { xr = a.y; xi = b.y; }
            else if (k2 < NH) { xr = a.x - b.y; xi = a.y + b.x; }
            else { xr = a.x + b.y; xi = b.x - a.y; }
            re[m] = xr; im[m] = xi;
        }
        fft_lines<L, G, +1>(re, im, g, smem + prm.tw_off);
    }
    __syncthreads();   // all reads of `mid` done; reuse the area as the output block
    if (active) {
        float *oa = sout + (p * h_out + ra) * w_out;
        float *ob = sout + (p * h_out + rb) * w_out;
#pragma unroll
        for (int k = 0; k < L; ++k) {
            const int b = k + L * group_block<G>(g);
            if (b < w_out) {
                oa[b] = re[k] * prm.scale;
                if (hasb) ob[b] = im[k] * prm.scale;
            }
        }
    }
    __syncthreads();
    if constexpr (CONV) {
        if (prm.tiled) {
            OriginTable<T> tab(smem + prm.info_off);
            tab.fill(prm.view, p0, np, tid);
            if (prm.vec_ok)
                unstage_windows<BT, T, 4>(prm.out, sout, prm.view, tab, np, prm.win_h, prm.win_w, h_out, w_out,
                                          prm.div_w, prm.div_h, tid, prm.accumulate != 0);
            else
                unstage_windows<BT, T, 1>(prm.out, sout, prm.view, tab, np, prm.win_h, prm.win_w, h_out, w_out,
                                          prm.div_w, prm.div_h, tid, prm.accumulate != 0);
            return;
        }
    }
    {
        float *dst = prm.out + p0 * (long)h_out * w_out;
        const unsigned total = (unsigned)np * h_out * w_out;
        unstage_linear<BT>(dst, sout, total, tid, true, prm.accumulate != 0);
    }
}

template <int L, int G, int T, bool CONV, bool ISTAGE>
__global__ void __launch_bounds__(T *(L * G / 2) * G) fft2d_c2r_kernel(Inv2dParams prm) {
    fft2d_c2r_body<L, G, T, CONV, ISTAGE>(prm, blockIdx.x);
}


// Two inverse transforms (plane-tiled layout, both staged through LDS) in ONE launch: the blocks
// of operand o are [first[o], first[o+1]).  For the two products of fft_conv_backward (gx and gw),
// whose grids are short: one ramp-up and one tail instead of two.
struct InvPairParams {
    Inv2dParams op[2];
    unsigned first[3];
};

template <int L, int G, int T>
__global__ void __launch_bounds__(T *(L * G / 2) * G) fft2d_c2r_pair_kernel(InvPairParams m) {
    const unsigned b = blockIdx.x;
    const int o = b >= m.first[1];
    fft2d_c2r_body<L, G, T, true, true>(m.op[o], b - m.first[o]);
}

// ------------------------------------------------------------------ 1-D forward
struct Fwd1dParams {
    const float *in;
    float *out;
    long B;
    int n_in, RS;
    MagicDiv div_n;
    int linear, vec_ok, out_vec_ok;
    int tw_off;       // lines of four or eight lanes: twiddle table at LDS float tw_off
};

template <int L, int G, int TB>
__global__ void __launch_bounds__(TB / 2 * G) fft1d_r2c_kernel(Fwd1dParams prm) {
    constexpr int N = L * G, NH = N / 2, NB = NH + 1, BT = TB / 2 * G;
    constexpr int NA = SplitRegs<L, G>::A;
    constexpr int NBR = SplitRegs<L, G>::B;
    extern __shared__ float smem[];
    float *sin = smem;
    float2 *sout = reinterpret_cast<float2 *>(smem);

    const int tid = threadIdx.x;
    const long b0 = (long)blockIdx.x * TB;
    const long left = prm.B - b0;
    const int nb = left < TB ? (int)left : TB;
    const int n_in = prm.n_in;
    load_group_twiddles<L, G, BT>(smem + prm.tw_off, tid);   // used after the next barrier
    {
        const float *src = prm.in + b0 * n_in;
        const unsigned total = (unsigned)nb * n_in;
        if (prm.linear) {
            stage_linear<BT>(sin, src, total, tid, prm.vec_ok != 0);
        } else {
            constexpr int U = 8;
            for (unsigned base = tid; base < total; base += BT * U) {
                float v[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const unsigned e = base + u * BT;
                    v[u] = 0.f;
                    if (e < total) v[u] = src[e];
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const unsigned e = base + u * BT;
                    if (e < total) {
                        const unsigned sg = mdiv(e, prm.div_n);
                        sin[sg * prm.RS + (e - sg * n_in)] = v[u];
                    }
                }
            }
        }
    }
    __syncthreads();
    const int g = tid % G, pr = tid / G;
    const int sa = 2 * pr, sb = 2 * pr + 1;
    const bool active = sa < nb, hasb = sb < nb;
    float are[NA], aim[NA], bre[NBR], bim[NBR];
    if (active) {
        float re[L], im[L];
        const float *pa = sin + sa * prm.RS, *pb = sin + (hasb ? sb : sa) * prm.RS;
#pragma unroll
        for (int m = 0; m < L; ++m) {
            const int j = g + G * m;
            const float va = pa[j], vb = pb[j];     // unconditional; LDS has N floats of slack
            const bool in = j < n_in;
            re[m] = in ? va : 0.f;
            im[m] = (in && hasb) ? vb : 0.f;
        }
        fft_lines<L, G, -1>(re, im, g, smem + prm.tw_off);
        split_two_real<L, G>(re, im, g, are, aim, bre, bim);
    }
    __syncthreads();
    if (active) {
        if constexpr (G == 1) {
            float2 *oa = sout + sa * NB, *ob = sout + sb * NB;
            oa[0] = make_float2(are[0], 0.f); oa[NH] = make_float2(aim[0], 0.f);
#pragma unroll
            for (int k = 1; k < NH; ++k) oa[k] = make_float2(are[k], aim[k]);
            if (hasb) {
                ob[0] = make_float2(bre[0], 0.f); ob[NH] = make_float2(bim[0], 0.f);
#pragma unroll
                for (int k = 1; k < NH; ++k) ob[k] = make_float2(bre[k], bim[k]);
            }
        } else {
            if (!(g & 1) || hasb) {
                float2 *o = sout + ((g & 1) ? sb : sa) * NB;
#pragma unroll
                for (int k = 0; k < L; ++k) {
                    const int j = split_slot<L, G>(g, k);
                    if (j == 0) { o[0] = make_float2(are[k], 0.f); o[NH] = make_float2(aim[k], 0.f); }
                    else o[j] = make_float2(are[k], aim[k]);
                }
            }
        }
    }
    __syncthreads();
    {
        float *dst = prm.out + b0 * NB * 2;
        const unsigned total = (unsigned)nb * NB * 2;
        unstage_linear<BT>(dst, smem, total, tid, prm.out_vec_ok != 0, false);
    }
}

// ------------------------------------------------------------------ 1-D inverse
struct Inv1dParams {
    const float *in;
    float *out;
    long B;
    int n_out;
    float scale;
    int in_vec_ok, out_vec_ok;
    int tw_off;       // lines of four or eight lanes: twiddle table at LDS float tw_off
};

template <int L, int G, int TB>
__global__ void __launch_bounds__(TB / 2 * G) fft1d_c2r_kernel(Inv1dParams prm) {
    constexpr int N = L * G, NH = N / 2, NB = NH + 1, BT = TB / 2 * G;
    extern __shared__ float smem[];
    float2 *sin = reinterpret_cast<float2 *>(smem);
    float *sout = smem;

    const int tid = threadIdx.x;
    const long b0 = (long)blockIdx.x * TB;
    const long left = prm.B - b0;
    const int nb = left < TB ? (int)left : TB;
    const int n_out = prm.n_out;
    load_group_twiddles<L, G, BT>(smem + prm.tw_off, tid);   // used after the next barrier
    {
        const float *src = prm.in + b0 * NB * 2;
        const unsigned total = (unsigned)nb * NB * 2;
        stage_linear<BT>(smem, src, total, tid, prm.in_vec_ok != 0);
    }
    __syncthreads();
    const int g = tid % G, pr = tid / G;
    const int sa = 2 * pr, sb = 2 * pr + 1;
    const bool active = sa < nb, hasb = sb < nb;
    float re[L], im[L];
    if (active) {
        const float2 *A = sin + sa * NB, *Bp = sin + (hasb ? sb : sa) * NB;
#pragma unroll
        for (int m = 0; m < L; ++m) {
            const int k2 = g + G * m;
            const int slot = k2 <= NH ? k2 : N - k2;
            float2 a = A[slot];
            float2 b = Bp[slot];
            if (!hasb) b = make_float2(0.f, 0.f);
            if (k2 == 0 || k2 == NH) { a.y = 0.f; b.y = 0.f; }
            else if (k2 > NH) { a.y = -a.y; b.y = -b.y; }
            re[m] = a.x - b.y;
            im[m] = a.y + b.x;
        }
        fft_lines<L, G, +1>(re, im, g, smem + prm.tw_off);
    }
    __syncthreads();
    if (active) {
        float *oa = sout + sa * n_out, *ob = sout + sb * n_out;
#pragma unroll
        for (int k = 0; k < L; ++k) {
            const int b = k + L * group_block<G>(g);
            if (b < n_out) {
                oa[b] = re[k] * prm.scale;
                if (hasb) ob[b] = im[k] * prm.scale;
            }
        }
    }
    __syncthreads();
    {
        float *dst = prm.out + b0 * n_out;
        const unsigned total = (unsigned)nb * n_out;
        unstage_linear<BT>(dst, sout, total, tid, prm.out_vec_ok != 0, false);
    }
}

// ------------------------------------------------------------------ launch helpers
template <int L, int G, int T>
static Fwd2dParams make_fwd2d(const float *in, float *out, long planes, int h_in, int w_in, size_t *lds,
                              const PlaneView *view = nullptr) {
    constexpr int N = L * G, NH = N / 2;
    Fwd2dParams prm;
    prm.in = in; prm.out = out; prm.planes = planes; prm.h_in = h_in; prm.w_in = w_in;
    // LDS strides of the staged planes.  Odd strides by default: when w_in and h_in*w_in are
    // already odd the block is copied as it lies in memory, with 16-byte loads (that plain copy
    // measured worth more than any bank layout).  When padding is needed anyway and lanes work
    // in groups, pick the strides that spread a half-wave over all 32 banks: row-phase lanes are
    // ordered (lane-in-group g, plane p, row pair rp) and read element g + G*m of their rows,
    // bank = g + rp*RS + p*IPS (mod 32), so RS = G and IPS = G * (row pairs per 32 lanes) mod 32.
    prm.RS = w_in | 1;
    prm.IPS = (h_in * prm.RS) | 1;
    if (G > 1 && !(prm.RS == w_in && prm.IPS == h_in * w_in)) {
        auto up_to_residue = [](int v, int r) { return v + ((r - v) % 32 + 32) % 32; };
        const int rows32 = 32 / (G * T) > 0 ? 32 / (G * T) : 1;
        prm.RS = up_to_residue(w_in, G);
        prm.IPS = up_to_residue(h_in * prm.RS, (G * rows32) % 32);
    }
    prm.MPS = MidLayout<L, G>::fwd_plane(h_in) | 1;
    prm.vecw = (((size_t)in & 15) == 0 && w_in % 4 == 0) ? 4 : ((((size_t)in & 7) == 0 && w_in % 2 == 0) ? 2 : 1);
    prm.div_wv = make_magic((unsigned)(w_in / prm.vecw));
    prm.div_h = make_magic((unsigned)h_in);
    prm.lay.tsh = fft2d_tile_log2(N);
    prm.lay.bins = fft2d_layout_bins(N);
    prm.linear = (prm.RS == w_in && prm.IPS == h_in * w_in) ? 1 : 0;
    prm.vec_ok = (((size_t)in & 15) == 0 && ((size_t)T * h_in * w_in) % 4 == 0) ? 1 : 0;
    prm.out_vec_ok = (((size_t)out & 15) == 0 && ((size_t)T * N * (NH + 1) * 2) % 4 == 0) ? 1 : 0;
    const size_t a = ((size_t)T * prm.IPS + N) * sizeof(float), b = (size_t)T * prm.MPS * sizeof(float2);
    *lds = a > b ? a : b;
    prm.tiled = 0; prm.info_off = 0; prm.tw_off = 0; prm.view = PlaneView{};
    if (view) {   // gathered windows: scalar loads, padded image, origin table behind everything else
        prm.tiled = 1; prm.view = *view;
        prm.linear = 0;
        const bool v4 = ((size_t)in & 15) == 0 && view->W % 4 == 0 && view->dx % 4 == 0 && view->ox % 4 == 0 &&
                        w_in % 4 == 0;
        prm.vecw = v4 ? 4 : 1;
        prm.div_wv = make_magic((unsigned)(w_in / prm.vecw));
    }
    return prm;
}

// LDS bytes of a launch whose lines of four or eight lanes keep their twiddle table behind `lds` bytes of
// other data; *tw_off receives the table's offset in floats.
template <int L, int G>
static inline size_t with_twiddle_table(size_t lds, int *tw_off) {
    *tw_off = 0;
    if constexpr (!kLdsTwiddles<G>) return lds;
    const size_t at = (lds + 7) / 8 * 8;
    *tw_off = (int)(at / sizeof(float));
    return at + kGroupTwiddleFloats<L, G> * sizeof(float);
}

// LDS bytes of a launch whose blocks keep an origin table of T planes behind `lds` bytes of
// other data; *info_off receives the table's offset in floats.
static inline size_t with_origin_table(size_t lds, int T, int *info_off) {
    const size_t at = (lds + 7) / 8 * 8;
    *info_off = (int)(at / sizeof(float));
    return at + (size_t)T * 16;
}

// CONV_TOO = false: only the natural-layout kernel is instantiated (conv must be false).
template <int L, int G, int T, bool CONV_TOO = true>
static hipError_t run_fwd2d(const float *in, float *out, long planes, int h_in, int w_in,
                            bool conv, LaunchCtx st, const PlaneView *view) {
    constexpr int N = L * G, NH = N / 2, BT = T * NH * G;
    size_t lds;
    Fwd2dParams prm = make_fwd2d<L, G, T>(in, out, planes, h_in, w_in, &lds, view);
    // Measured: staging the output through LDS pays for the natural layout (short runs per
    // lane otherwise) and costs for the plane-tiled layout, whose direct stores already fill
    // whole runs of T planes.
    const bool ostage = !conv;
    if (ostage) {
        const size_t c = (size_t)T * N * (NH + 1) * 2 * sizeof(float);
        if (c > lds) lds = c;
    }
    lds = with_twiddle_table<L, G>(lds, &prm.tw_off);
    if (prm.tiled) lds = with_origin_table(lds, T, &prm.info_off);
    const unsigned grid = (unsigned)((planes + T - 1) / T);
    hipError_t e;
    auto go = [&](auto k) -> hipError_t {
        if ((e = allow_big_lds((const void *)k, lds)) != hipSuccess) return e;
        launch_kernel(k, dim3(grid), dim3(BT), lds, st, prm);
        return hipGetLastError();
    };
    if constexpr (CONV_TOO) {
        if (conv) return go(fft2d_r2c_kernel<L, G, T, true, false>);
    } else {
        if (conv) return hipErrorInvalidValue;
    }
    return go(fft2d_r2c_kernel<L, G, T, false, true>);
}

template <int L, int G, int T>
static hipError_t run_fwd2d_multi(const FwdOperand *ops, int nops, LaunchCtx st) {
    constexpr int N = L * G, NH = N / 2, BT = T * NH * G;
    FwdMultiParams m;
    size_t lds = 0;
    unsigned blocks = 0;
    for (int o = 0; o < 3; ++o) {
        m.first[o] = blocks;
        if (o < nops) {
            size_t l;
            m.op[o] = make_fwd2d<L, G, T>(ops[o].in, ops[o].out, ops[o].planes, ops[o].h_in, ops[o].w_in, &l,
                                          ops[o].view);
            if (l > lds) lds = l;
            blocks += (unsigned)((ops[o].planes + T - 1) / T);
        } else {
            m.op[o] = m.op[0];
        }
    }
    m.first[3] = blocks;
    for (int o = nops; o < 3; ++o) m.first[o] = blocks;   // unused operands own no blocks
    {   // one twiddle table position for all operands, behind the largest footprint
        int tw_off = 0;
        lds = with_twiddle_table<L, G>(lds, &tw_off);
        for (int o = 0; o < 3; ++o) m.op[o].tw_off = tw_off;
    }
    {   // one origin table position for all operands, behind everything else
        int info_off = 0;
        bool any = false;
        for (int o = 0; o < nops; ++o) any = any || m.op[o].tiled;
        if (any) {
            lds = with_origin_table(lds, T, &info_off);
            for (int o = 0; o < 3; ++o) m.op[o].info_off = info_off;
        }
    }
    auto k = fft2d_r2c_multi_kernel<L, G, T>;
    hipError_t e;
    if ((e = allow_big_lds((const void *)k, lds)) != hipSuccess) return e;
    launch_kernel(k, dim3(blocks), dim3(BT), lds, st, m);
    return hipGetLastError();
}

// Parameters and LDS bytes of one inverse launch; *istage_out tells whether the plane-tiled input
// is staged through LDS (always for the natural layout).
template <int L, int G, int T>
static Inv2dParams make_inv2d(const float *in, float *out, long planes, int h_out, int w_out, bool conv, float scale,
                              bool accumulate, const PlaneView *view, size_t *lds_out, bool *istage_out,
                              bool force_stage = false) {
    constexpr int N = L * G, NH = N / 2;
    Inv2dParams prm;
    prm.tiled = 0; prm.info_off = 0; prm.win_h = prm.win_w = 0; prm.view = PlaneView{};
    prm.div_w = prm.div_h = MagicDiv{0};
    bool tiled_vec = false;
    if (view) {
        // the block assembled in LDS spans the transform's rows / columns up to the window's end
        prm.tiled = 1; prm.view = *view;
        prm.win_h = h_out; prm.win_w = w_out;
        tiled_vec = ((size_t)out & 15) == 0 && view->W % 4 == 0 && view->dx % 4 == 0 && view->ox % 4 == 0 &&
                    w_out % 4 == 0;    // then the LDS block's row length ox + w_out is a multiple of 4 too
        prm.div_w = make_magic((unsigned)(tiled_vec ? w_out / 4 : w_out)); prm.div_h = make_magic((unsigned)h_out);
        h_out += view->oy; w_out += view->ox;
    }
    prm.in = in; prm.out = out; prm.planes = planes; prm.h_out = h_out; prm.w_out = w_out;
    prm.MPS = MidLayout<L, G>::inv_plane(h_out) | 1;
    prm.lay.tsh = fft2d_tile_log2(N);
    prm.lay.bins = fft2d_layout_bins(N);
    prm.scale = scale; prm.accumulate = accumulate ? 1 : 0;
    prm.vec_ok = (((size_t)out & 15) == 0 && ((size_t)T * h_out * w_out) % 4 == 0) ? 1 : 0;
    if (view) prm.vec_ok = tiled_vec ? 1 : 0;   // tiled: 16-byte scatter of the windows
    prm.in_vec_ok = (((size_t)in & 15) == 0 && ((size_t)T * N * (NH + 1) * 2) % 4 == 0) ? 1 : 0;
    const size_t a = (size_t)T * prm.MPS * sizeof(float2), b = ((size_t)T * h_out * w_out + 3) * sizeof(float);
    size_t lds = a > b ? a : b;
    // Stage the block's (contiguous) input through LDS with 16-byte loads: always for the
    // natural layout; for the plane-tiled layout it measured faster except for the small
    // bases (32 or 64 planes per workgroup) when most of the output is kept.
    const bool istage = force_stage || !conv || T <= 16 || 2 * h_out <= N;
    if (istage) {
        const size_t c = (size_t)T * N * (NH + 1) * sizeof(float2);
        if (c > lds) lds = c;
    }
    *lds_out = lds;
    *istage_out = istage;
    return prm;
}

template <int L, int G, int T, bool CONV_TOO = true>
static hipError_t run_inv2d(const float *in, float *out, long planes, int h_out, int w_out,
                            bool conv, float scale, bool accumulate, LaunchCtx st, const PlaneView *view) {
    constexpr int N = L * G, NH = N / 2, BT = T * NH * G;
    size_t lds;
    bool istage;
    Inv2dParams prm = make_inv2d<L, G, T>(in, out, planes, h_out, w_out, conv, scale, accumulate, view, &lds, &istage);
    lds = with_twiddle_table<L, G>(lds, &prm.tw_off);
    if (prm.tiled) lds = with_origin_table(lds, T, &prm.info_off);
    const unsigned grid = (unsigned)((planes + T - 1) / T);
    hipError_t e;
    auto go = [&](auto k) -> hipError_t {
        if ((e = allow_big_lds((const void *)k, lds)) != hipSuccess) return e;
        launch_kernel(k, dim3(grid), dim3(BT), lds, st, prm);
        return hipGetLastError();
    };
    if constexpr (CONV_TOO) {
        if (conv) return istage ? go(fft2d_c2r_kernel<L, G, T, true, true>) : go(fft2d_c2r_kernel<L, G, T, true, false>);
    } else {
        if (conv) return hipErrorInvalidValue;
    }
    return go(fft2d_c2r_kernel<L, G, T, false, true>);
}

// Two operands in one launch; both run the variant that stages the plane-tiled input through
// LDS (the only one for T <= 16).
template <int L, int G, int T>
static hipError_t run_inv2d_pair(const InvOperand *ops, LaunchCtx st) {
    constexpr int N = L * G, NH = N / 2, BT = T * NH * G;
    InvPairParams m;
    size_t lds = 0;
    unsigned blocks = 0;
    bool any_tiled = false;
    for (int o = 0; o < 2; ++o) {
        size_t l;
        bool istage;
        m.first[o] = blocks;
        m.op[o] = make_inv2d<L, G, T>(ops[o].in, ops[o].out, ops[o].planes, ops[o].h_out, ops[o].w_out, true,
                                      ops[o].scale, ops[o].accumulate, ops[o].view, &l, &istage, true);
        if (l > lds) lds = l;
        any_tiled = any_tiled || m.op[o].tiled;
        blocks += (unsigned)((ops[o].planes + T - 1) / T);
    }
    m.first[2] = blocks;
    int tw_off = 0, info_off = 0;
    lds = with_twiddle_table<L, G>(lds, &tw_off);
    if (any_tiled) lds = with_origin_table(lds, T, &info_off);
    for (int o = 0; o < 2; ++o) { m.op[o].tw_off = tw_off; m.op[o].info_off = info_off; }
    if (blocks == 0) return hipSuccess;
    auto k = fft2d_c2r_pair_kernel<L, G, T>;
    if (hipError_t e = allow_big_lds((const void *)k, lds); e != hipSuccess) return e;
    launch_kernel(k, dim3(blocks), dim3(BT), lds, st, m);
    return hipGetLastError();
}

template <int L, int G, int TB>
static hipError_t run_fwd1d(const float *in, float *out, long B, int n_in, LaunchCtx st) {
    constexpr int N = L * G, NB = N / 2 + 1, BT = TB / 2 * G;
    Fwd1dParams prm;
    prm.in = in; prm.out = out; prm.B = B; prm.n_in = n_in; prm.RS = n_in | 1;
    prm.div_n = make_magic((unsigned)n_in);
    prm.linear = (prm.RS == n_in) ? 1 : 0;
    prm.vec_ok = (((size_t)in & 15) == 0 && ((size_t)TB * n_in) % 4 == 0) ? 1 : 0;
    prm.out_vec_ok = (((size_t)out & 15) == 0 && ((size_t)TB * NB * 2) % 4 == 0) ? 1 : 0;
    const size_t a = ((size_t)TB * prm.RS + N) * sizeof(float), b = (size_t)TB * NB * sizeof(float2);
    const size_t lds = with_twiddle_table<L, G>(a > b ? a : b, &prm.tw_off);
    auto k = fft1d_r2c_kernel<L, G, TB>;
    hipError_t e;
    if ((e = allow_big_lds((const void *)k, lds)) != hipSuccess) return e;
    launch_kernel(k, dim3((unsigned)((B + TB - 1) / TB)), dim3(BT), lds, st, prm);
    return hipGetLastError();
}

template <int L, int G, int TB>
static hipError_t run_inv1d(const float *in, float *out, long B, int n_out, LaunchCtx st) {
    constexpr int N = L * G, NB = N / 2 + 1, BT = TB / 2 * G;
    Inv1dParams prm;
    prm.in = in; prm.out = out; prm.B = B; prm.n_out = n_out; prm.scale = 1.0f / (float)N;
    prm.in_vec_ok = (((size_t)in & 15) == 0 && ((size_t)TB * NB * 2) % 4 == 0) ? 1 : 0;
    prm.out_vec_ok = (((size_t)out & 15) == 0 && ((size_t)TB * n_out) % 4 == 0) ? 1 : 0;
    const size_t a = (size_t)TB * NB * sizeof(float2), b = (size_t)TB * n_out * sizeof(float);
    const size_t lds = with_twiddle_table<L, G>(a > b ? a : b, &prm.tw_off);
    auto k = fft1d_c2r_kernel<L, G, TB>;
    hipError_t e;
    if ((e = allow_big_lds((const void *)k, lds)) != hipSuccess) return e;
    launch_kernel(k, dim3((unsigned)((B + TB - 1) / TB)), dim3(BT), lds, st, prm);
    return hipGetLastError();
}


// Sizes with an odd factor (12 ... 224), instantiated in their own translation units; the
// launch_* functions of kernels.hpp forward every size that is not a power of two here.
hipError_t launch_fft2d_r2c_mixed(const float *in, float *out, long planes, int h_in, int w_in, int N,
                                  bool conv, LaunchCtx st, const PlaneView *view);
hipError_t launch_fft2d_r2c_multi_mixed(const FwdOperand *ops, int nops, int N, LaunchCtx st);
hipError_t launch_fft2d_c2r_mixed(const float *in, float *out, long planes, int N, int h_out, int w_out,
                                  bool conv, float scale, bool accumulate, LaunchCtx st, const PlaneView *view);
// Natural-layout choices that differ from the convolution path's (fft_kernels_natural.hip);
// hipErrorNotSupported for the sizes without one.
hipError_t launch_fft2d_r2c_natural(const float *in, float *out, long planes, int h_in, int w_in, int N, LaunchCtx st);
hipError_t launch_fft2d_c2r_natural(const float *in, float *out, long planes, int N, int h_out, int w_out,
                                    float scale, bool accumulate, LaunchCtx st);
hipError_t launch_fft2d_c2r_pair_mixed(const InvOperand *ops, int N, LaunchCtx st);
hipError_t launch_fft1d_r2c_mixed(const float *in, float *out, long B, int n_in, int n, LaunchCtx st);
hipError_t launch_fft1d_c2r_mixed(const float *in, float *out, long B, int n, int n_out, LaunchCtx st);

}  // namespace fc
