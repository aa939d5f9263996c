// Per-frequency-bin complex contraction on the fp32 matrix cores of gfx950.
//
// This is the Cgemm step of Table 1 of the fbfft paper (one small complex matrix product
// per frequency bin, reducing over f for fprop, f' for bprop and S for accGrad), done as one
// launch over all bins instead of a batched library call on transposed tensors.  A complex
// product is three real MFMA products on planar operands (Gauss's trick; the operand sums
// are one VALU add per value read from LDS):
//     P1 += Ar*Br,  P2 += Ai*Bi,  P3 += (Ar+Ai)*(Br+Bi);   Cr = P1 - P2,  Ci = P3 - P1 - P2
// Operands are gathered straight from the FFT kernels' plane-tiled layout (kernels.hpp), so
// the three explicit transposes of the paper's pipeline never exist.
//
// Workgroup = 4 waves (WGM x WGN), each wave owns FM x FN MFMA tiles of 32x32 (re and im
// accumulators).  K is walked in tiles of TK through a double-buffered LDS image
// As[c][k][m], Bs[c][k][n]; the next tile's global loads are in flight while the current
// one is multiplied.  Bins are dealt to the 8 XCDs in contiguous chunks (workgroup i runs
// on XCD i % 8), so that the tiles of one bin, and neighbouring bins that share cache
// lines in the plane-tiled layout, meet in the same L2.
#include "kernels.hpp"
#include "gemm_params.hpp"

#include <cstdlib>
#include <type_traits>

namespace fc {

template <int I, int E, class F>
__device__ __forceinline__ void static_for_gemm(F &&f) {
    if constexpr (I < E) {
        f(std::integral_constant<int, I>{});
        static_for_gemm<I + 1, E>(f);
    }
}




// Loader of one operand tile (ROWS x TK) with the "row" index being m (or n) and the
// reduction index k.  KF: k is the contiguous plane index (else the row index is).
// VEC: 16-byte gathers (needs plane runs of >= 4, aligned starts and extents).
template <int ROWS, int TK, int STRIDE, bool KF, bool VEC, int NT>
struct TileLoader {
    static constexpr int NV = VEC ? (ROWS * TK / 4 + NT - 1) / NT : (ROWS * TK + NT - 1) / NT;
    float4 vr[VEC ? NV : 1], vi[VEC ? NV : 1];
    float sr[VEC ? 1 : NV], si[VEC ? 1 : NV];
    unsigned boff[VEC ? NV : 1];   // fast addressing: byte offset of vector i from the tile's uniform base

    // Fast addressing (16-byte gathers whose strided index moves in whole plane tiles, see
    // fast_addressing()): the element index splits into a part that is uniform over the
    // workgroup and changes with the K tile, which the scalar unit computes, and a per-lane
    // part that never changes, computed here once.  A gather then costs no vector arithmetic.
    __device__ __forceinline__ void prepare_fast(const FreqLayout &lay, long rs, long cs, int r0, int R, int tid) {
        static_assert(VEC, "fast addressing is for 16-byte gathers");
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int v = tid + i * NT;
            int rr, kk;
            if constexpr (KF) { kk = (v % (TK / 4)) * 4; rr = v / (TK / 4); }
            else { rr = (v % (ROWS / 4)) * 4; kk = v / (ROWS / 4); }
            size_t o;
            if constexpr (KF) o = (size_t)rr * rs * lay.bins * 2 + lay.part(kk);
            else o = lay.part(rr) + (size_t)kk * cs * lay.bins * 2;
            boff[i] = (v < ROWS * TK / 4 && r0 + rr < R) ? (unsigned)(o * sizeof(float)) : 0xffffffffu;
        }
    }
    // ub: uniform base of this K tile (real parts); the imaginary parts lie im_bytes further.
    __device__ __forceinline__ void load_fast(const char *ub, unsigned im_bytes, int k0, int K, int tid) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int v = tid + i * NT;
            int kk;
            if constexpr (KF) kk = (v % (TK / 4)) * 4;
            else kk = v / (ROWS / 4);
            vr[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            vi[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (boff[i] != 0xffffffffu && k0 + kk < K) {
                vr[i] = *reinterpret_cast<const float4 *>(ub + boff[i]);
                vi[i] = *reinterpret_cast<const float4 *>(ub + im_bytes + boff[i]);
            }
        }
    }

    __device__ __forceinline__ void load(const float *base, const FreqLayout &lay, long rs, long cs,
                                         int bin, int r0, int k0, int R, int K, int tid) {
        const size_t im_off = (size_t)1 << lay.tsh;
        if constexpr (VEC) {
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                const int v = tid + i * NT;
                int rr, kk;
                if constexpr (KF) { kk = (v % (TK / 4)) * 4; rr = v / (TK / 4); }
                else { rr = (v % (ROWS / 4)) * 4; kk = v / (ROWS / 4); }
                vr[i] = make_float4(0.f, 0.f, 0.f, 0.f);
                vi[i] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (v < ROWS * TK / 4 && r0 + rr < R && k0 + kk < K) {
                    const size_t idx = lay.index((r0 + rr) * rs + (k0 + kk) * cs, bin, 0);
                    vr[i] = *reinterpret_cast<const float4 *>(base + idx);
                    vi[i] = *reinterpret_cast<const float4 *>(base + idx + im_off);
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                const int e = tid + i * NT;
                int rr, kk;
                if constexpr (KF) { kk = e % TK; rr = e / TK; }
                else { rr = e % ROWS; kk = e / ROWS; }
                sr[i] = 0.f; si[i] = 0.f;
                if (e < ROWS * TK && r0 + rr < R && k0 + kk < K) {
                    const size_t idx = lay.index((r0 + rr) * rs + (k0 + kk) * cs, bin, 0);
                    sr[i] = base[idx];
                    si[i] = base[idx + im_off];
                }
            }
        }
    }

    // LDS image: dst[c][k][row], row stride STRIDE, component stride TK*STRIDE.
    __device__ __forceinline__ void store(float *dst, int tid) const {
        float *d0 = dst, *d1 = dst + TK * STRIDE;
        if constexpr (VEC) {
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                const int v = tid + i * NT;
                if (v < ROWS * TK / 4) {
                    if constexpr (KF) {
                        const int kk = (v % (TK / 4)) * 4, rr = v / (TK / 4);
                        d0[(kk + 0) * STRIDE + rr] = vr[i].x; d0[(kk + 1) * STRIDE + rr] = vr[i].y;
                        d0[(kk + 2) * STRIDE + rr] = vr[i].z; d0[(kk + 3) * STRIDE + rr] = vr[i].w;
                        d1[(kk + 0) * STRIDE + rr] = vi[i].x; d1[(kk + 1) * STRIDE + rr] = vi[i].y;
                        d1[(kk + 2) * STRIDE + rr] = vi[i].z; d1[(kk + 3) * STRIDE + rr] = vi[i].w;
                    } else {
                        const int rr = (v % (ROWS / 4)) * 4, kk = v / (ROWS / 4);
                        float2 *q0 = reinterpret_cast<float2 *>(d0 + kk * STRIDE + rr);
                        float2 *q1 = reinterpret_cast<float2 *>(d1 + kk * STRIDE + rr);
                        q0[0] = make_float2(vr[i].x, vr[i].y); q0[1] = make_float2(vr[i].z, vr[i].w);
                        q1[0] = make_float2(vi[i].x, vi[i].y); q1[1] = make_float2(vi[i].z, vi[i].w);
                    }
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                const int e = tid + i * NT;
                if (e < ROWS * TK) {
                    int rr, kk;
                    if constexpr (KF) { kk = e % TK; rr = e / TK; }
                    else { rr = e % ROWS; kk = e / ROWS; }
                    d0[kk * STRIDE + rr] = sr[i];
                    d1[kk * STRIDE + rr] = si[i];
                }
            }
        }
    }
};

// Uniform part of the addresses of one operand tile under fast addressing: rows from r0 (row
// stride rs planes), reduction indices from k0 (stride cs planes), real parts.
template <bool KF>
__device__ __forceinline__ const char *tile_base(const float *base, const FreqLayout &lay, long rs, long cs,
                                                 int bin, int r0, int k0) {
    size_t o = (size_t)bin * (2u << lay.tsh);
    if constexpr (KF) o += (size_t)r0 * rs * lay.bins * 2 + lay.part(k0);
    else o += lay.part(r0) + (size_t)k0 * cs * lay.bins * 2;
    return reinterpret_cast<const char *>(base + o);
}

// One workgroup's share of the contraction: workgroup number wg of prm's grid.
template <int WGM, int WGN, int FM, int FN, int TK, bool AKF, bool BKF, bool VEC, int PD>
__device__ __forceinline__ void cgemm_bins_body(const GemmParams &prm, const unsigned wg) {
    constexpr int NT = 64 * WGM * WGN;
    constexpr int TM = WGM * FM * 32, TN = WGN * FN * 32;
    constexpr int SA = TM + 2, SB = TN + 2;        // +2: conflict-free transposing stores
    constexpr int ABUF = 2 * TK * SA, BBUF = 2 * TK * SB;
    extern __shared__ float smem[];
    float *As = smem;                 // [2 buffers][2 comps][TK][SA]
    float *Bs = smem + 2 * ABUF;      // [2 buffers][2 comps][TK][SB]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;

    // XCD-aware decomposition of the flat workgroup index (see file header).
    const int tiles = prm.tiles_m * prm.tiles_n;
    const int xcd = wg % kXcds, slot = wg / kXcds;
    const int bins_per_xcd = prm.bins / kXcds;
    const int bin = xcd * bins_per_xcd + slot / tiles;
    const int tile = slot % tiles;
    const int tm = tile / prm.tiles_n, tn = tile % prm.tiles_n;
    const int m0 = tm * TM, n0 = tn * TN;
    const int M = prm.M, N = prm.N, K = prm.K;

    // Three real products per complex product (Gauss): P1 = Ar Br, P2 = Ai Bi,
    // P3 = (Ar + Ai)(Br + Bi);  Cr = P1 - P2,  Ci = P3 - P1 - P2.
    floatx16 acc_p1[FM][FN], acc_p2[FM][FN], acc_p3[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) { acc_p1[i][j][v] = 0.f; acc_p2[i][j][v] = 0.f; acc_p3[i][j][v] = 0.f; }

    // Register staging for PD tiles ahead: tile t travels global -> la/lb[t % PD] -> LDS buffer
    // t % 2.  With a short reduction (K of a few tiles) every gather is in flight before the
    // first MFMA; with a long one a single tile ahead is enough.
    TileLoader<TM, TK, SA, AKF, VEC, NT> la[PD];
    TileLoader<TN, TK, SB, BKF, VEC, NT> lb[PD];
    const int nkt = (K + TK - 1) / TK;
    bool fast = false;
    if constexpr (VEC) fast = prm.fast != 0;
    if constexpr (VEC) {
        if (fast) {
#pragma unroll
            for (int d = 0; d < PD; ++d) {
                la[d].prepare_fast(prm.layA, prm.a_rs, prm.a_cs, m0, M, tid);
                lb[d].prepare_fast(prm.layB, prm.b_cs, prm.b_rs, n0, N, tid);
            }
        }
    }
    auto issue = [&](auto &xa, auto &xb, int kt) {
        if constexpr (VEC) {
            if (fast) {
                xa.load_fast(tile_base<AKF>(prm.A, prm.layA, prm.a_rs, prm.a_cs, bin, m0, kt * TK),
                             4u << prm.layA.tsh, kt * TK, K, tid);
                xb.load_fast(tile_base<BKF>(prm.B, prm.layB, prm.b_cs, prm.b_rs, bin, n0, kt * TK),
                             4u << prm.layB.tsh, kt * TK, K, tid);
                return;
            }
        }
        xa.load(prm.A, prm.layA, prm.a_rs, prm.a_cs, bin, m0, kt * TK, M, K, tid);
        // B(k, n): row index of the loader is n, so swap the strides
        xb.load(prm.B, prm.layB, prm.b_cs, prm.b_rs, bin, n0, kt * TK, N, K, tid);
    };
    static_for_gemm<0, PD>([&](auto dd) {
        constexpr int d = decltype(dd)::value;
        if (d < nkt) issue(la[d], lb[d], d);
    });
    la[0].store(As, tid);
    lb[0].store(Bs, tid);
    if (PD < nkt) issue(la[0], lb[0], PD);
    __syncthreads();

    const int lrow = lane & 31, lk = lane >> 5;
    // The k-steps of the tile in LDS buffer cur, software-pipelined: the LDS reads of step
    // s + 1 are issued before the MFMAs of step s, so a wave on its own keeps the matrix
    // pipe fed.  mid() runs half way through the tile.
    struct Frag { float a_re[FM], a_im[FM], b_re[FN], b_im[FN]; };
    auto read_frag = [&](Frag &f, const float *a0, const float *b0, int ks) {
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            f.a_re[i] = a0[(ks + lk) * SA + i * 32];
            f.a_im[i] = a0[TK * SA + (ks + lk) * SA + i * 32];
        }
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            f.b_re[j] = b0[(ks + lk) * SB + j * 32];
            f.b_im[j] = b0[TK * SB + (ks + lk) * SB + j * 32];
        }
    };
    auto mma = [&](const Frag &f) {
        float a_im[FM], a_sm[FM], b_im[FN], b_sm[FN];
#pragma unroll
        for (int i = 0; i < FM; ++i) { a_im[i] = flip(f.a_im[i], prm.a_sign); a_sm[i] = f.a_re[i] + a_im[i]; }
#pragma unroll
        for (int j = 0; j < FN; ++j) { b_im[j] = flip(f.b_im[j], prm.b_sign); b_sm[j] = f.b_re[j] + b_im[j]; }
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                acc_p1[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a_re[i], f.b_re[j], acc_p1[i][j], 0, 0, 0);
                acc_p2[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_im[i], b_im[j], acc_p2[i][j], 0, 0, 0);
                acc_p3[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_sm[i], b_sm[j], acc_p3[i][j], 0, 0, 0);
            }
    };
    auto compute = [&](int cur, auto &&mid) {
        const float *a0 = As + cur * ABUF + (wm * FM * 32 + lrow);
        const float *b0 = Bs + cur * BBUF + (wn * FN * 32 + lrow);
        Frag f[2];
        read_frag(f[0], a0, b0, 0);
        static_for_gemm<0, TK / 2>([&](auto ss) {
            constexpr int st = decltype(ss)::value;
            if constexpr (st + 1 < TK / 2) read_frag(f[(st + 1) & 1], a0, b0, 2 * (st + 1));
            __builtin_amdgcn_sched_barrier(0);
            mma(f[st & 1]);
            if constexpr (st == TK / 4 - 1) mid();
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    // Iteration kt multiplies tile kt out of LDS buffer kt & 1.  Half way through, tile kt + 1
    // moves from its registers into the other buffer (which every wave left at the barrier
    // that ended iteration kt - 1) and the freed registers take the gathers of tile
    // kt + 1 + PD, so that between two tiles a wave only passes a barrier.
    for (int kt0 = 0; kt0 < nkt; kt0 += PD) {
        static_for_gemm<0, PD>([&](auto dd) {
            constexpr int d = decltype(dd)::value;
            constexpr int dn = (d + 1) % PD;
            const int kt = kt0 + d;
            if (kt < nkt) {
                const int cur = kt & 1;
                compute(cur, [&]() {
                    if (kt + 1 < nkt) {
                        la[dn].store(As + (cur ^ 1) * ABUF, tid);
                        lb[dn].store(Bs + (cur ^ 1) * BBUF, tid);
                        if (kt + 1 + PD < nkt) issue(la[dn], lb[dn], kt + 1 + PD);
                    }
                });
                if (kt + 1 < nkt) __syncthreads();
            }
        });
    }

    // D layout of the 32x32x2 MFMA: lane l, register v -> row 8*(v/4) + 4*(l/32) + v%4, col l%32.
    const size_t cim = (size_t)1 << prm.layC.tsh;
    if (fast) {
        // C(m, n) with n the contiguous plane index and the row stride a whole number of plane
        // tiles: uniform base per register v (scalar unit), one per-lane byte offset
        const size_t row = (size_t)prm.c_rs * prm.layC.bins * 2;          // floats per step of m
        char *cb = reinterpret_cast<char *>(prm.C + (size_t)bin * (2u << prm.layC.tsh) + prm.layC.part(n0) + (size_t)m0 * row);
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const int nl = (wn * FN + j) * 32 + lrow, ml = (wm * FM + i) * 32 + 4 * lk;
                const unsigned lo = (unsigned)((ml * row + prm.layC.part(nl)) * sizeof(float));
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int mv = 8 * (v / 4) + (v % 4);
                    if (m0 + ml + mv < M && n0 + nl < N) {
                        char *q = cb + (size_t)mv * row * sizeof(float) + lo;
                        const float p1 = acc_p1[i][j][v], p2 = acc_p2[i][j][v];
                        *reinterpret_cast<float *>(q) = p1 - p2;
                        *reinterpret_cast<float *>(q + cim * sizeof(float)) = acc_p3[i][j][v] - p1 - p2;
                    }
                }
            }
        return;
    }
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const int n = n0 + (wn * FN + j) * 32 + lrow;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + (wm * FM + i) * 32 + 8 * (v / 4) + 4 * lk + (v % 4);
                if (m < M && n < N) {
                    const size_t idx = prm.layC.index(m * prm.c_rs + n * prm.c_cs, bin, 0);
                    const float p1 = acc_p1[i][j][v], p2 = acc_p2[i][j][v];
                    prm.C[idx] = p1 - p2;
                    prm.C[idx + cim] = acc_p3[i][j][v] - p1 - p2;
                }
            }
        }
}

template <int WGM, int WGN, int FM, int FN, int TK, bool AKF, bool BKF, bool VEC, int MINB, int PD>
__global__ void __launch_bounds__(64 * WGM * WGN, MINB) cgemm_bins_kernel(GemmParams prm) {
    cgemm_bins_body<WGM, WGN, FM, FN, TK, AKF, BKF, VEC, PD>(prm, blockIdx.x);
}

// One 32x32 quadrant (quad = 2 * row half + column half) of the 64x64 tile that workgroup
// number vwg of prm's grid would compute, with the reduction split over the four waves: wave w
// takes k-steps w and w + 4 of every K tile, the four partial tiles meet in LDS and each wave
// sums and stores a quarter of the rows.  A quarter of the serial MFMA chain per wave, and PD
// tiles of gathers in flight from the start: this is for workgroups that run when most of
// the chip has drained (see cgemm_tail_kernel).
template <int TK, bool AKF, bool BKF, int PD>
__device__ __forceinline__ void cgemm_quadrant_body(const GemmParams &prm, const unsigned vwg, const int quad) {
    constexpr int NT = 256, TQ = 32, SQ = TQ + 2;
    constexpr int QBUF = 2 * TK * SQ;
    static_assert(TK == 16, "two k-step pairs per wave and K tile");
    extern __shared__ float smem[];
    float *As = smem;                 // [2 buffers][2 comps][TK][SQ]
    float *Bs = smem + 2 * QBUF;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tiles = prm.tiles_m * prm.tiles_n;
    const int xcd = vwg % kXcds, slot = vwg / kXcds;
    const int bins_per_xcd = prm.bins / kXcds;
    const int bin = xcd * bins_per_xcd + slot / tiles;
    const int tile = slot % tiles;
    const int m0 = (tile / prm.tiles_n) * 64 + (quad >> 1) * TQ, n0 = (tile % prm.tiles_n) * 64 + (quad & 1) * TQ;
    const int M = prm.M, N = prm.N, K = prm.K;
    if (m0 >= M || n0 >= N) return;   // uniform over the workgroup

    floatx16 p1, p2, p3;
#pragma unroll
    for (int v = 0; v < 16; ++v) { p1[v] = 0.f; p2[v] = 0.f; p3[v] = 0.f; }

    TileLoader<TQ, TK, SQ, AKF, true, NT> la[PD];
    TileLoader<TQ, TK, SQ, BKF, true, NT> lb[PD];
    const int nkt = (K + TK - 1) / TK;
    const bool fast = prm.fast != 0;
    if (fast) {
#pragma unroll
        for (int d = 0; d < PD; ++d) {
            la[d].prepare_fast(prm.layA, prm.a_rs, prm.a_cs, m0, M, tid);
            lb[d].prepare_fast(prm.layB, prm.b_cs, prm.b_rs, n0, N, tid);
        }
    }
    auto issue = [&](auto &xa, auto &xb, int kt) {
        if (fast) {
            xa.load_fast(tile_base<AKF>(prm.A, prm.layA, prm.a_rs, prm.a_cs, bin, m0, kt * TK),
                         4u << prm.layA.tsh, kt * TK, K, tid);
            xb.load_fast(tile_base<BKF>(prm.B, prm.layB, prm.b_cs, prm.b_rs, bin, n0, kt * TK),
                         4u << prm.layB.tsh, kt * TK, K, tid);
            return;
        }
        xa.load(prm.A, prm.layA, prm.a_rs, prm.a_cs, bin, m0, kt * TK, M, K, tid);
        xb.load(prm.B, prm.layB, prm.b_cs, prm.b_rs, bin, n0, kt * TK, N, K, tid);
    };
    static_for_gemm<0, PD>([&](auto dd) {
        constexpr int d = decltype(dd)::value;
        if (d < nkt) issue(la[d], lb[d], d);
    });
    la[0].store(As, tid);
    lb[0].store(Bs, tid);
    if (PD < nkt) issue(la[0], lb[0], PD);
    __syncthreads();

    const int lrow = lane & 31, lk = lane >> 5;
    auto compute = [&](int cur) {
        const float *a0 = As + cur * QBUF + lrow, *b0 = Bs + cur * QBUF + lrow;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int k = 2 * (wave + 4 * h) + lk;
            const float a_re = a0[k * SQ], a_im = flip(a0[TK * SQ + k * SQ], prm.a_sign);
            const float b_re = b0[k * SQ], b_im = flip(b0[TK * SQ + k * SQ], prm.b_sign);
            p1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a_re, b_re, p1, 0, 0, 0);
            p2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a_im, b_im, p2, 0, 0, 0);
            p3 = __builtin_amdgcn_mfma_f32_32x32x2f32(a_re + a_im, b_re + b_im, p3, 0, 0, 0);
        }
    };
    for (int kt0 = 0; kt0 < nkt; kt0 += PD) {
        static_for_gemm<0, PD>([&](auto dd) {
            constexpr int d = decltype(dd)::value;
            constexpr int dn = (d + 1) % PD;
            const int kt = kt0 + d;
            if (kt < nkt) {
                const int cur = kt & 1;
                if (kt + 1 < nkt) {
                    // buffer cur ^ 1 was last read in iteration kt - 1, which every wave has left
                    la[dn].store(As + (cur ^ 1) * QBUF, tid);
                    lb[dn].store(Bs + (cur ^ 1) * QBUF, tid);
                    if (kt + 1 + PD < nkt) issue(la[dn], lb[dn], kt + 1 + PD);
                }
                compute(cur);
                if (kt + 1 < nkt) __syncthreads();
            }
        });
    }

    // Partial tiles [wave][component][register][lane] -> LDS; wave w then owns registers
    // 4w .. 4w+3, i.e. rows 8w + 4*(lane/32) + 0..3 of the quadrant (D layout of the MFMA).
    __syncthreads();                  // every wave is done with the operand tiles
    float *red = smem;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        red[((wave * 2 + 0) * 16 + v) * 64 + lane] = p1[v] - p2[v];
        red[((wave * 2 + 1) * 16 + v) * 64 + lane] = p3[v] - p1[v] - p2[v];
    }
    __syncthreads();
    const size_t cim = (size_t)1 << prm.layC.tsh;
    const int n = n0 + lrow;
#pragma unroll
    for (int vv = 0; vv < 4; ++vv) {
        const int v = wave * 4 + vv;
        float cr = 0.f, ci = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            cr += red[((w * 2 + 0) * 16 + v) * 64 + lane];
            ci += red[((w * 2 + 1) * 16 + v) * 64 + lane];
        }
        const int m = m0 + 8 * wave + 4 * lk + vv;
        if (m < M && n < N) {
            size_t idx;
            if (fast) idx = (size_t)bin * (2u << prm.layC.tsh) + prm.layC.part(n0) + prm.layC.part(lrow) +
                            (size_t)m * prm.c_rs * prm.layC.bins * 2;
            else idx = prm.layC.index(m * prm.c_rs + n * prm.c_cs, bin, 0);
            prm.C[idx] = cr;
            prm.C[idx + cim] = ci;
        }
    }
}

// The 64x64 contraction with a split tail.  A grid that is a little more than a whole number
// of rounds (resident workgroups: four per compute unit) leaves its last few workgroups to
// run alone, each at the latency of its own loads and MFMA chain, while the rest of the chip
// idles (measured on the 27x27 layer: 64 of 1088 workgroups, 11 of 28 us).  Those last tiles are
// cut into quadrants: workgroups [split_from, grid) are quadrant workgroups, four per tile,
// numbered so that a tile's quadrants run on the XCD that its bin's other tiles ran on.
template <bool AKF, bool BKF>
__global__ void __launch_bounds__(256, 3) cgemm_tail_kernel(GemmParams prm) {
    if (blockIdx.x < prm.split_from) {
        cgemm_bins_body<2, 2, 1, 1, 16, AKF, BKF, true, 1>(prm, blockIdx.x);
    } else {
        const unsigned r = blockIdx.x - prm.split_from;
        const unsigned x = r % kXcds, u = r / kXcds;
        cgemm_quadrant_body<16, AKF, BKF, 2>(prm, prm.split_from + kXcds * (u / 4) + x, (int)(u % 4));
    }
}

// Two independent contractions in one launch (the two backward passes of a layer share
// their first operand and neither waits for the other): workgroups [0, n1) work on p1, the
// rest on p2.  One grid means one ramp-up and one tail instead of two, and the second
// problem's workgroups fill the slots that the first one's stragglers leave idle.
struct GemmPairParams {
    GemmParams p1, p2;
    unsigned n1;       // workgroups of p1
    unsigned split2;   // p2's workgroups from this number on are cut into quadrants (as in
                       // cgemm_tail_kernel); equal to p2's workgroup count when none are
};
template <bool AKF1, bool BKF1, bool AKF2, bool BKF2>
__global__ void __launch_bounds__(256, 3) cgemm_pair_kernel(GemmPairParams pp) {
    if (blockIdx.x < pp.n1) {
        cgemm_bins_body<2, 2, 1, 1, 16, AKF1, BKF1, true, 1>(pp.p1, blockIdx.x);
        return;
    }
    const unsigned b = blockIdx.x - pp.n1;
    if (b < pp.split2) {
        cgemm_bins_body<2, 2, 1, 1, 16, AKF2, BKF2, true, 1>(pp.p2, b);
    } else {
        const unsigned r = b - pp.split2;
        const unsigned x = r % kXcds, u = r / kXcds;
        cgemm_quadrant_body<16, AKF2, BKF2, 2>(pp.p2, pp.split2 + kXcds * (u / 4) + x, (int)(u % 4));
    }
}

template <int WGM, int WGN, int FM, int FN, int TK, bool AKF, bool BKF, bool VEC, int MINB, int PD = 1>
static hipError_t run_gemm(GemmParams prm, LaunchCtx st) {
    constexpr int TM = WGM * FM * 32, TN = WGN * FN * 32;
    prm.tiles_m = (prm.M + TM - 1) / TM;
    prm.tiles_n = (prm.N + TN - 1) / TN;
    const long grid = (long)prm.bins * prm.tiles_m * prm.tiles_n;
    const size_t lds = (size_t)(2 * 2 * TK * (TM + 2) + 2 * 2 * TK * (TN + 2)) * sizeof(float);
    auto k = cgemm_bins_kernel<WGM, WGN, FM, FN, TK, AKF, BKF, VEC, MINB, PD>;
    if (hipError_t e = allow_big_lds((const void *)k, lds); e != hipSuccess) return e;
    launch_kernel(k, dim3((unsigned)grid), dim3(64 * WGM * WGN), lds, st, prm);
    return hipGetLastError();
}

// Tile shapes (M x N on four waves): 0 128x128, 1 64x128, 2 128x64, 3 64x64; 4 and 5 are 64x64
// with 2 and 4 tiles of register staging ahead.  3 is the default, the others are kept for
// A/B runs.  1-, 2- and 8-wave workgroups and TK = 8 / 32 were also measured; none beat 3.
template <bool AKF, bool BKF, bool VEC>
static hipError_t dispatch_tile(int shape, GemmParams prm, LaunchCtx st) {
    switch (shape) {
        case 0: return run_gemm<2, 2, 2, 2, 16, AKF, BKF, VEC, 1>(prm, st);
        case 1: return run_gemm<2, 2, 1, 2, 16, AKF, BKF, VEC, 2>(prm, st);
        case 2: return run_gemm<2, 2, 2, 1, 16, AKF, BKF, VEC, 2>(prm, st);
        case 3: return run_gemm<2, 2, 1, 1, 16, AKF, BKF, VEC, 3>(prm, st);
        case 4: return run_gemm<2, 2, 1, 1, 16, AKF, BKF, VEC, 3, 2>(prm, st);
        case 5: return run_gemm<2, 2, 1, 1, 16, AKF, BKF, VEC, 3, 4>(prm, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_cgemm_bingroup(const GemmParams &prm, bool akf, bool bkf, LaunchCtx st);

GemmSwitches read_gemm_switches() {
    GemmSwitches s;
    auto on = [](const char *name) { const char *e = getenv(name); return e && atoi(e) != 0; };
    if (const char *e = getenv("FFTCONV_GEMM_TILE")) s.tile = atoi(e);
    s.no_tail = on("FFTCONV_GEMM_NO_TAIL");
    s.no_pair = on("FFTCONV_GEMM_NO_PAIR");
    s.no_bingroup = on("FFTCONV_GEMM_NO_BINGROUP");
    s.no_fast = on("FFTCONV_GEMM_NO_FAST");
    if (const char *e = getenv("FFTCONV_BG_TILE")) s.bg_tile = atoi(e);
    return s;
}
static const GemmSwitches kDefaultSwitches{};
static const GemmSwitches &switches_of(const GemmSwitches *sw) { return sw ? *sw : kDefaultSwitches; }

// 64x64 tiles on four waves with one tile of register staging ahead (shape 3) measured fastest
// for every layer shape tried (more workgroups in flight beat the larger tiles' operand reuse
// and the deeper staging's registers).
static int pick_tile(const GemmSwitches &sw) { return sw.tile >= 0 ? sw.tile : 3; }

// Fast addressing of an operand (see TileLoader::prepare_fast): one index of the matrix is the
// contiguous plane index, the other moves `stride` planes per step.  When that stride is a
// whole number of plane tiles, a step of the strided index adds a constant to the element index,
// whatever the contiguous index is, so addresses split into a uniform part and a per-lane
// part.  The per-lane part must fit an unsigned 32-bit byte offset: 64 steps of the strided index.
static bool fast_addressing(const FreqLayout &lay, long stride, int bins) {
    const long T = 1L << lay.tsh;
    if (stride <= 0 || stride % T != 0) return false;
    return (double)stride * bins * 2 * 4 * 65 < 2147483648.0;
}

// Kernel parameters of one contraction and the kernel variant it can use.
struct Prepared {
    GemmParams prm;
    bool akf, bkf;     // the reduction index is the contiguous plane index of A / B
    bool vec;          // 16-byte gathers are possible
    bool bingroup;     // the four-bins-per-line kernel applies
};

static hipError_t prepare(const GemmOperand &A, const GemmOperand &B, float *C, FreqLayout layC, long C_rs,
                          long C_cs, int M, int N, int K, int bins, const GemmSwitches &sw, Prepared *out) {
    if (bins % kXcds != 0) return hipErrorInvalidValue;   // N*(N/2+1) with N >= 8 always is
    GemmParams &prm = out->prm;
    prm.A = A.ptr; prm.B = B.ptr; prm.C = C;
    prm.layA = A.lay; prm.layB = B.lay; prm.layC = layC;
    prm.a_rs = A.rs; prm.a_cs = A.cs; prm.b_rs = B.rs; prm.b_cs = B.cs;
    prm.c_rs = C_rs; prm.c_cs = C_cs;
    prm.M = M; prm.N = N; prm.K = K; prm.bins = bins;
    prm.tiles_m = prm.tiles_n = 0;
    prm.split_from = 0xffffffffu;
    prm.a_sign = A.conj ? 0x80000000u : 0u;
    prm.b_sign = B.conj ? 0x80000000u : 0u;
    const bool akf = (A.cs == 1), bkf = (B.rs == 1);
    // 16-byte gathers need: runs of >= 4 planes, the contiguous index a multiple of 4 at every
    // vector start (tile origins are), its extent a multiple of 4, and the other stride too.
    auto vec_ok = [](const FreqLayout &l, long contiguous_extent, long other_stride, const float *p) {
        return l.tsh >= 2 && contiguous_extent % 4 == 0 && other_stride % 4 == 0 && ((size_t)p & 15) == 0;
    };
    const bool va = akf ? vec_ok(A.lay, K, A.rs, A.ptr) : (A.rs == 1 && vec_ok(A.lay, M, A.cs, A.ptr));
    const bool vb = bkf ? vec_ok(B.lay, K, B.cs, B.ptr) : (B.cs == 1 && vec_ok(B.lay, N, B.rs, B.ptr));
    out->akf = akf; out->bkf = bkf; out->vec = va && vb;
    prm.fast = (out->vec && fast_addressing(A.lay, akf ? A.rs : A.cs, bins) &&
                fast_addressing(B.lay, bkf ? B.cs : B.rs, bins) && C_cs == 1 && fast_addressing(layC, C_rs, bins) &&
                !sw.no_fast) ? 1 : 0;
    // Layouts with runs of 4 planes (basis 64) put four bins in every 128-byte line: the
    // bin-group kernel loads whole lines and multiplies the four bins side by side.
    out->bingroup = out->vec && !sw.no_bingroup && A.lay.tsh == 2 && B.lay.tsh == 2 && layC.tsh == 2 &&
                    bins % (4 * kXcds) == 0 && (akf || A.rs == 1) && (bkf || B.cs == 1) && C_cs == 1 &&
                    C_rs % 4 == 0 && N % 4 == 0 && ((size_t)C & 15) == 0;
    return hipSuccess;
}

// Workgroups of the 64x64 kernel that are resident at once (four per compute unit: LDS).
static long resident_workgroups() {
    static long slots = 0;
    if (!slots) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
        slots = 4L * cus;
    }
    return slots;
}

template <bool AKF, bool BKF>
static hipError_t run_tail(GemmParams prm, long full, long rem, LaunchCtx st) {
    prm.split_from = (unsigned)full;
    const size_t lds = (size_t)(2 * 2 * 16 * 66 + 2 * 2 * 16 * 66) * sizeof(float);   // >= the quadrant's 32 KB
    auto k = cgemm_tail_kernel<AKF, BKF>;
    if (hipError_t e = allow_big_lds((const void *)k, lds); e != hipSuccess) return e;
    launch_kernel(k, dim3((unsigned)(full + 4 * rem)), dim3(256), lds, st, prm);
    return hipGetLastError();
}

static hipError_t launch_prepared(const Prepared &q, LaunchCtx st) {
    const GemmParams &prm = q.prm;
    const GemmSwitches &sw = switches_of(st.sw);
    if (q.bingroup) return launch_cgemm_bingroup(prm, q.akf, q.bkf, st);
    const int shape = pick_tile(sw);
    if (q.vec && shape == 3 && sw.tile < 0 && !sw.no_tail) {
        // a short last round (at most a quarter of the resident workgroups): split its tiles
        GemmParams p2 = prm;
        p2.tiles_m = (p2.M + 63) / 64; p2.tiles_n = (p2.N + 63) / 64;
        const long total = (long)p2.bins * p2.tiles_m * p2.tiles_n, slots = resident_workgroups();
        const long rem = total % slots, full = total - rem;
        if (full > 0 && rem > 0 && 4 * rem <= slots && rem % kXcds == 0 && full % kXcds == 0) {
            if (q.akf && q.bkf) return run_tail<true, true>(p2, full, rem, st);
            if (q.akf && !q.bkf) return run_tail<true, false>(p2, full, rem, st);
            if (!q.akf && !q.bkf) return run_tail<false, false>(p2, full, rem, st);
            return run_tail<false, true>(p2, full, rem, st);
        }
    }
    if (q.vec) {
        if (q.akf && q.bkf) return dispatch_tile<true, true, true>(shape, prm, st);
        if (q.akf && !q.bkf) return dispatch_tile<true, false, true>(shape, prm, st);
        if (!q.akf && !q.bkf) return dispatch_tile<false, false, true>(shape, prm, st);
        return dispatch_tile<false, true, true>(shape, prm, st);
    }
    if (q.akf && q.bkf) return dispatch_tile<true, true, false>(shape, prm, st);
    if (q.akf && !q.bkf) return dispatch_tile<true, false, false>(shape, prm, st);
    if (!q.akf && !q.bkf) return dispatch_tile<false, false, false>(shape, prm, st);
    return dispatch_tile<false, true, false>(shape, prm, st);
}

hipError_t launch_cgemm_bins(GemmOperand A, GemmOperand B, float *C, FreqLayout layC, long C_rs,
                             long C_cs, int M, int N, int K, int bins, LaunchCtx st) {
    Prepared q;
    if (hipError_t e = prepare(A, B, C, layC, C_rs, C_cs, M, N, K, bins, switches_of(st.sw), &q); e != hipSuccess) return e;
    return launch_prepared(q, st);
}

template <bool AKF1, bool BKF1, bool AKF2, bool BKF2>
static hipError_t run_pair(GemmPairParams &pp, LaunchCtx st) {
    constexpr int TM = 64, TN = 64, TK = 16;
    for (GemmParams *g : {&pp.p1, &pp.p2}) {
        g->tiles_m = (g->M + TM - 1) / TM;
        g->tiles_n = (g->N + TN - 1) / TN;
    }
    const long n1 = (long)pp.p1.bins * pp.p1.tiles_m * pp.p1.tiles_n;
    const long n2 = (long)pp.p2.bins * pp.p2.tiles_m * pp.p2.tiles_n;
    pp.n1 = (unsigned)n1;     // a multiple of the XCD count, as bins is
    // a short last round (at most a quarter of the resident workgroups), all of it p2's: split
    // its tiles into quadrants (the 27x27 layer on basis 28: 424 + 848 workgroups, 248 left over)
    const long slots = resident_workgroups(), rem = (n1 + n2) % slots, full = n1 + n2 - rem;
    long split = n2;
    if (!switches_of(st.sw).no_tail && full > 0 && rem > 0 && 4 * rem <= slots && rem <= n2 && rem % kXcds == 0 &&
        (n2 - rem) % kXcds == 0)
        split = n2 - rem;
    pp.split2 = (unsigned)split;
    const size_t lds = (size_t)(2 * 2 * TK * (TM + 2) + 2 * 2 * TK * (TN + 2)) * sizeof(float);   // >= the quadrant's
    auto k = cgemm_pair_kernel<AKF1, BKF1, AKF2, BKF2>;
    if (hipError_t e = allow_big_lds((const void *)k, lds); e != hipSuccess) return e;
    launch_kernel(k, dim3((unsigned)(n1 + split + 4 * (n2 - split))), dim3(256), lds, st, pp);
    return hipGetLastError();
}

template <bool AKF1, bool BKF1>
static hipError_t pair_second(const Prepared &q2, GemmPairParams &pp, LaunchCtx st) {
    if (q2.akf && q2.bkf) return run_pair<AKF1, BKF1, true, true>(pp, st);
    if (q2.akf && !q2.bkf) return run_pair<AKF1, BKF1, true, false>(pp, st);
    if (!q2.akf && !q2.bkf) return run_pair<AKF1, BKF1, false, false>(pp, st);
    return run_pair<AKF1, BKF1, false, true>(pp, st);
}

bool cgemm_pair_supported(const GemmProblem &g1, const GemmProblem &g2, const GemmSwitches *swp) {
    const GemmSwitches &sw = switches_of(swp);
    if (sw.tile >= 0) return false;       // A/B runs of single-kernel shapes
    if (sw.no_pair) return false;
    Prepared q1, q2;
    if (prepare(g1.A, g1.B, g1.C, g1.layC, g1.C_rs, g1.C_cs, g1.M, g1.N, g1.K, g1.bins, sw, &q1) != hipSuccess) return false;
    if (prepare(g2.A, g2.B, g2.C, g2.layC, g2.C_rs, g2.C_cs, g2.M, g2.N, g2.K, g2.bins, sw, &q2) != hipSuccess) return false;
    return q1.vec && q2.vec && !q1.bingroup && !q2.bingroup;
}

hipError_t launch_cgemm_pair(const GemmProblem &g1, const GemmProblem &g2, LaunchCtx st) {
    Prepared q1, q2;
    const GemmSwitches &sw = switches_of(st.sw);
    if (hipError_t e = prepare(g1.A, g1.B, g1.C, g1.layC, g1.C_rs, g1.C_cs, g1.M, g1.N, g1.K, g1.bins, sw, &q1); e != hipSuccess) return e;
    if (hipError_t e = prepare(g2.A, g2.B, g2.C, g2.layC, g2.C_rs, g2.C_cs, g2.M, g2.N, g2.K, g2.bins, sw, &q2); e != hipSuccess) return e;
    if (!(q1.vec && q2.vec) || q1.bingroup || q2.bingroup) return hipErrorInvalidValue;
    GemmPairParams pp;
    pp.p1 = q1.prm; pp.p2 = q2.prm; pp.n1 = 0;
    if (q1.akf && q1.bkf) return pair_second<true, true>(q2, pp, st);
    if (q1.akf && !q1.bkf) return pair_second<true, false>(q2, pp, st);
    if (!q1.akf && !q1.bkf) return pair_second<false, false>(q2, pp, st);
    return pair_second<false, true>(q2, pp, st);
}

}  // namespace fc
