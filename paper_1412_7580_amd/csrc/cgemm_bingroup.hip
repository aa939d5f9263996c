// Per-bin complex contraction for plane-tiled layouts with runs of 4 planes (Fourier basis 64).
//
// Same operation as cgemm_kernels.hip (the Cgemm row of Table 1 of the fbfft paper), other
// blocking.  With T = 4 a 128-byte line of a frequency tensor holds 4 planes x (re, im) x 4
// consecutive bins, so a kernel that works on one bin uses 1/4 of every line it touches and
// the rest is fetched again for the neighbouring bins.  Here a workgroup takes four
// consecutive bins at once: its 256 lanes load whole lines (8 lanes x 16 bytes per line), the
// line's eight (bin, component) pieces go to eight LDS regions, and wave w multiplies bin w.
#include "gemm_params.hpp"

#include <cstdlib>

namespace fc {

// Loader of a (ROWS x TK) operand tile of four bins.  Lane tid handles float4 number tid % 8
// of a line, i.e. region = (bin - b0) * 2 + component, for units tid / 8 + 32 * i.
template <int ROWS, int TK, int STRIDE, int RSTR, bool KF>
struct GroupLoader {
    static constexpr int UNITS = ROWS * TK / 4;
    static constexpr int NV = (UNITS + 31) / 32;
    float4 v[NV];

    __device__ __forceinline__ void load(const float *base, int bins, long rs, long cs, int b0,
                                         int r0, int k0, int R, int K, int tid) {
        const int j = tid & 7, ub = tid >> 3;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int u = ub + 32 * i;
            int rr, kk;
            if constexpr (KF) { kk = (u % (TK / 4)) * 4; rr = u / (TK / 4); }
            else { rr = (u % (ROWS / 4)) * 4; kk = u / (ROWS / 4); }
            v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (u < UNITS && r0 + rr < R && k0 + kk < K) {
                const long plane = (r0 + rr) * rs + (k0 + kk) * cs;
                const size_t idx = (size_t)((plane >> 2) * bins + b0) * 8 + j * 4;
                v[i] = *reinterpret_cast<const float4 *>(base + idx);
            }
        }
    }

    // Fast addressing (the strided matrix index moves in whole plane tiles, see fast_addressing()
    // in cgemm_kernels.hip): the element index splits into a part that is uniform over the
    // workgroup and changes with the K tile, left to the scalar unit (tile_base), and a per-lane
    // byte offset that never changes, computed once (prepare).  A gather then costs no vector
    // arithmetic and no 64-bit address registers.
    unsigned boff[NV];
    __device__ __forceinline__ void prepare(int bins, long rs, long cs, int r0, int R, int tid) {
        const int j = tid & 7, ub = tid >> 3;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int u = ub + 32 * i;
            int rr, kk;
            if constexpr (KF) { kk = (u % (TK / 4)) * 4; rr = u / (TK / 4); }
            else { rr = (u % (ROWS / 4)) * 4; kk = u / (ROWS / 4); }
            size_t o;
            if constexpr (KF) o = (size_t)rr * (rs >> 2) + (kk >> 2);
            else o = (size_t)(rr >> 2) + (size_t)kk * (cs >> 2);
            o = o * bins * 8 + j * 4;
            boff[i] = (u < UNITS && r0 + rr < R) ? (unsigned)(o * sizeof(float)) : 0xffffffffu;
        }
    }
    static __device__ __forceinline__ const char *tile_base(const float *base, int bins, long rs, long cs, int b0,
                                                            int r0, int k0) {
        size_t o;
        if constexpr (KF) o = (size_t)r0 * (rs >> 2) + (k0 >> 2);
        else o = (size_t)(r0 >> 2) + (size_t)k0 * (cs >> 2);
        return reinterpret_cast<const char *>(base + (o * bins + b0) * 8);
    }
    __device__ __forceinline__ void load_fast(const char *ub, int k0, int K, int tid) {
        const int ubi = tid >> 3;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int u = ubi + 32 * i;
            int kk;
            if constexpr (KF) kk = (u % (TK / 4)) * 4;
            else kk = u / (ROWS / 4);
            v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (boff[i] != 0xffffffffu && k0 + kk < K) v[i] = *reinterpret_cast<const float4 *>(ub + boff[i]);
        }
    }

    // LDS image: region-major, inside a region [k][row] with row stride STRIDE.
    __device__ __forceinline__ void store(float *dst, int tid) const {
        const int j = tid & 7, ub = tid >> 3;
        float *d = dst + j * RSTR;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int u = ub + 32 * i;
            if (u < UNITS) {
                if constexpr (KF) {
                    const int kk = (u % (TK / 4)) * 4, rr = u / (TK / 4);
                    d[(kk + 0) * STRIDE + rr] = v[i].x; d[(kk + 1) * STRIDE + rr] = v[i].y;
                    d[(kk + 2) * STRIDE + rr] = v[i].z; d[(kk + 3) * STRIDE + rr] = v[i].w;
                } else {
                    const int rr = (u % (ROWS / 4)) * 4, kk = u / (ROWS / 4);
                    float2 *q = reinterpret_cast<float2 *>(d + kk * STRIDE + rr);
                    q[0] = make_float2(v[i].x, v[i].y);
                    q[1] = make_float2(v[i].z, v[i].w);
                }
            }
        }
    }
};

// FAST: fast addressing (GroupLoader::prepare) of both operands and of the result.  C4 layer, us per
// pass (fprop / bprop / accGrad), same box: 107 / 100 / 117 without, 100 / 93 / 103 with it.  (Loads of
// two K tiles in flight instead of one need 64 more registers: at three waves per SIMD that
// build spilled, at two it measured 117 / 108 / 140.)
template <int FM, int FN, int TK, bool AKF, bool BKF, bool FAST>
__global__ void __launch_bounds__(256, (FM * FN == 1 && AKF == BKF ? 4 : 1)) cgemm_bingroup_kernel(GemmParams prm) {
    constexpr int TM = 32 * FM, TN = 32 * FN;
    constexpr int SA = TM + 2, SB = TN + 2;
    // region strides: odd (scalar transposing stores spread over banks) or even (float2 stores)
    constexpr int RA = TK * SA + (AKF ? 1 : 2), RB = TK * SB + (BKF ? 1 : 2);
    extern __shared__ float smem[];
    float *As = smem;              // [8 regions][RA]
    float *Bs = smem + 8 * RA;     // [8 regions][RB]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tiles = prm.tiles_m * prm.tiles_n;
    const int groups_per_xcd = prm.bins / 4 / kXcds;
    const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
    const int b0 = (xcd * groups_per_xcd + slot / tiles) * 4;
    const int tile = slot % tiles;
    const int m0 = (tile / prm.tiles_n) * TM, n0 = (tile % prm.tiles_n) * TN;
    const int M = prm.M, N = prm.N, K = prm.K, bins = prm.bins;

    // Three real products per complex product (Gauss): P1 = Ar Br, P2 = Ai Bi,
    // P3 = (Ar + Ai)(Br + Bi);  Cr = P1 - P2,  Ci = P3 - P1 - P2.
    floatx16 acc_p1[FM][FN], acc_p2[FM][FN], acc_p3[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) { acc_p1[i][j][v] = 0.f; acc_p2[i][j][v] = 0.f; acc_p3[i][j][v] = 0.f; }

    GroupLoader<TM, TK, SA, RA, AKF> la;
    GroupLoader<TN, TK, SB, RB, BKF> lb;
    const int nkt = (K + TK - 1) / TK;
    if constexpr (FAST) {
        la.prepare(bins, prm.a_rs, prm.a_cs, m0, M, tid);
        lb.prepare(bins, prm.b_cs, prm.b_rs, n0, N, tid);
    }
    auto fetch = [&](int kt) {
        if constexpr (FAST) {
            la.load_fast(la.tile_base(prm.A, bins, prm.a_rs, prm.a_cs, b0, m0, kt * TK), kt * TK, K, tid);
            lb.load_fast(lb.tile_base(prm.B, bins, prm.b_cs, prm.b_rs, b0, n0, kt * TK), kt * TK, K, tid);
        } else {
            la.load(prm.A, bins, prm.a_rs, prm.a_cs, b0, m0, kt * TK, M, K, tid);
            lb.load(prm.B, bins, prm.b_cs, prm.b_rs, b0, n0, kt * TK, N, K, tid);
        }
    };
    fetch(0);
    la.store(As, tid);
    lb.store(Bs, tid);
    __syncthreads();

    const int lrow = lane & 31, lk = lane >> 5;
    const float *a0 = As + (2 * wave) * RA + lrow;
    const float *b0p = Bs + (2 * wave) * RB + lrow;
    for (int kt = 0; kt < nkt; ++kt) {
        const bool more = kt + 1 < nkt;
        if (more) fetch(kt + 1);
#pragma unroll
        for (int ks = 0; ks < TK; ks += 2) {
            float a_re[FM], a_im[FM], a_sm[FM], b_re[FN], b_im[FN], b_sm[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i) {
                a_re[i] = a0[(ks + lk) * SA + i * 32];
                a_im[i] = flip(a0[RA + (ks + lk) * SA + i * 32], prm.a_sign);
                a_sm[i] = a_re[i] + a_im[i];
            }
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                b_re[j] = b0p[(ks + lk) * SB + j * 32];
                b_im[j] = flip(b0p[RB + (ks + lk) * SB + j * 32], prm.b_sign);
                b_sm[j] = b_re[j] + b_im[j];
            }
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    acc_p1[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_re[i], b_re[j], acc_p1[i][j], 0, 0, 0);
                    acc_p2[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_im[i], b_im[j], acc_p2[i][j], 0, 0, 0);
                    acc_p3[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_sm[i], b_sm[j], acc_p3[i][j], 0, 0, 0);
                }
        }
        if (more) {
            __syncthreads();      // every wave is done reading this tile
            la.store(As, tid);
            lb.store(Bs, tid);
            __syncthreads();
        }
    }

    // Epilogue.  D layout of the 32x32x2 MFMA: lane l, register v -> row 8*(v/4) + 4*(l/32) + v%4,
    // col l%32.  The four waves drop their tiles into an LDS image laid out like the global
    // lines (per (row, 4 columns): 4 bins x (re, im) x 4 planes, padded to 36 floats so that
    // the scalar stores spread over the banks); then 8 lanes write each 128-byte line.
    constexpr int LSTR = 36;
    constexpr int NQ = TN / 4;
    __syncthreads();               // all waves are done with the operand tiles
    float *img = smem;
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const int nn = j * 32 + lrow;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int mm = i * 32 + 8 * (v / 4) + 4 * lk + (v % 4);
                float *q = img + (mm * NQ + (nn >> 2)) * LSTR + wave * 8 + (nn & 3);
                const float p1 = acc_p1[i][j][v], p2 = acc_p2[i][j][v];
                q[0] = p1 - p2;
                q[4] = acc_p3[i][j][v] - p1 - p2;
            }
        }
    __syncthreads();
    if constexpr (FAST) {
        // rows ub / NQ + it * (32 / NQ), column quad ub % NQ: the index is a uniform base, a per-lane
        // offset and a uniform step per round
        static_assert(32 % NQ == 0, "a round of 32 units covers whole rows");
        const int jq = tid & 7, ub = tid >> 3;
        const size_t crs4 = (size_t)(prm.c_rs >> 2);
        char *cb = reinterpret_cast<char *>(prm.C + (((size_t)m0 * crs4 + (n0 >> 2)) * bins + b0) * 8);
        const int mm0 = ub / NQ, nq = ub % NQ;
        const unsigned loff = (unsigned)((((size_t)mm0 * crs4 + nq) * bins * 8 + jq * 4) * sizeof(float));
        const size_t step = (size_t)(32 / NQ) * crs4 * bins * 8 * sizeof(float);
        const bool col_ok = n0 + 4 * nq < N;
#pragma unroll
        for (int it = 0; it < TM * NQ / 32; ++it) {
            const int mm = mm0 + it * (32 / NQ);
            if (col_ok && m0 + mm < M)
                *reinterpret_cast<float4 *>(cb + it * step + loff) =
                    *reinterpret_cast<const float4 *>(img + (ub + 32 * it) * LSTR + jq * 4);
        }
    } else {
        const int jq = tid & 7, ub = tid >> 3;
#pragma unroll
        for (int u = ub; u < TM * NQ; u += 32) {
            const int mm = u / NQ, nq = u % NQ;
            const int m = m0 + mm, n = n0 + 4 * nq;
            if (m < M && n < N) {
                const long plane = m * prm.c_rs + n;
                const size_t idx = (size_t)((plane >> 2) * bins + b0) * 8 + jq * 4;
                *reinterpret_cast<float4 *>(prm.C + idx) = *reinterpret_cast<const float4 *>(img + u * LSTR + jq * 4);
            }
        }
    }
}

template <int FM, int FN, int TK, bool AKF, bool BKF, bool FAST = false>
static hipError_t run_bg(GemmParams prm, LaunchCtx st) {
    constexpr int TM = 32 * FM, TN = 32 * FN;
    constexpr int RA = TK * (TM + 2) + (AKF ? 1 : 2), RB = TK * (TN + 2) + (BKF ? 1 : 2);
    prm.tiles_m = (prm.M + TM - 1) / TM;
    prm.tiles_n = (prm.N + TN - 1) / TN;
    const long grid = (long)(prm.bins / 4) * prm.tiles_m * prm.tiles_n;
    size_t lds = (size_t)8 * (RA + RB) * sizeof(float);
    const size_t img = (size_t)TM * (TN / 4) * 36 * sizeof(float);
    if (img > lds) lds = img;
    auto k = cgemm_bingroup_kernel<FM, FN, TK, AKF, BKF, FAST>;
    if (hipError_t e = allow_big_lds((const void *)k, lds); e != hipSuccess) return e;
    launch_kernel(k, dim3((unsigned)grid), dim3(256), lds, st, prm);
    return hipGetLastError();
}

template <bool AKF, bool BKF>
static hipError_t dispatch_bg(int shape, const GemmParams &prm, LaunchCtx st) {
    switch (shape) {
        case 0: return prm.fast ? run_bg<1, 1, 16, AKF, BKF, true>(prm, st) : run_bg<1, 1, 16, AKF, BKF>(prm, st);
        case 1: return run_bg<1, 2, 16, AKF, BKF>(prm, st);
        case 2: return run_bg<2, 1, 16, AKF, BKF>(prm, st);
        case 3: return run_bg<2, 2, 16, AKF, BKF>(prm, st);
        default: return hipErrorInvalidValue;
    }
}

// Per-wave tile (rows x cols of one bin): 0 32x32, 1 32x64, 2 64x32, 3 64x64.
hipError_t launch_cgemm_bingroup(const GemmParams &prm, bool akf, bool bkf, LaunchCtx st) {
    const int shape = st.sw ? st.sw->bg_tile : 0;   // 0 measured fastest for every pass of the 64-basis layer
    if (akf && bkf) return dispatch_bg<true, true>(shape, prm, st);
    if (akf && !bkf) return dispatch_bg<true, false>(shape, prm, st);
    if (!akf && !bkf) return dispatch_bg<false, false>(shape, prm, st);
    return dispatch_bg<false, true>(shape, prm, st);
}

}  // namespace fc
