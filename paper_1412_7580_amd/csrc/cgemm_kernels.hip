// Per-frequency-bin complex contraction on the fp32 matrix cores of gfx950.
//
// This is the Cgemm step of Table 1 of the fbfft paper (one small complex matrix product
// per frequency bin, reducing over f for fprop, f' for bprop and S for accGrad), done as one
// launch over all bins instead of a batched library call on transposed tensors.  A complex
// product is four real MFMA products on planar operands:
//     Cr += Ar*Br + (-Ai)*Bi ,   Ci += Ar*Bi + Ai*Br
// Operands are gathered straight from the FFT kernels' plane-tiled layout (kernels.hpp), so
// the three explicit transposes of the paper's pipeline never exist.
#include "kernels.hpp"

namespace fc {

typedef float floatx16 __attribute__((ext_vector_type(16)));

struct GemmParams {
    const float *A, *B;
    float *C;
    FreqLayout layA, layB, layC;
    long a_rs, a_cs, b_rs, b_cs, c_rs, c_cs;
    int M, N, K, bins;
    int tiles_m, tiles_n;
    int a_kfast, b_kfast;   // which index is contiguous in planes (coalescing of the gather)
};

constexpr int GEMM_TK = 16;
constexpr int GEMM_PAD = 4;

// Workgroup = 4 waves arranged WGM x WGN; each wave owns FM x FN MFMA tiles of 32x32.
template <int WGM, int WGN, int FM, int FN>
__global__ void __launch_bounds__(256) cgemm_bins_kernel(GemmParams prm) {
    static_assert(WGM * WGN == 4, "four waves per workgroup");
    constexpr int TM = WGM * FM * 32, TN = WGN * FN * 32, TK = GEMM_TK;
    constexpr int SA = TM + GEMM_PAD, SB = TN + GEMM_PAD;
    constexpr int EA = TM * TK / 256, EB = TN * TK / 256;
    __shared__ float As[2][TK][SA];
    __shared__ float Bs[2][TK][SB];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    int bid = blockIdx.x;
    const int tn = bid % prm.tiles_n; bid /= prm.tiles_n;
    const int tm = bid % prm.tiles_m;
    const int bin = bid / prm.tiles_m;
    const int m0 = tm * TM, n0 = tn * TN;
    const int M = prm.M, N = prm.N, K = prm.K;

    floatx16 acc_re[FM][FN], acc_im[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) { acc_re[i][j][v] = 0.f; acc_im[i][j][v] = 0.f; }

    float ra_re[EA], ra_im[EA], rb_re[EB], rb_im[EB];

    auto load_tiles = [&](int k0) {
#pragma unroll
        for (int i = 0; i < EA; ++i) {
            const int e = tid + i * 256;
            int mm, kk;
            if (prm.a_kfast) { kk = e % TK; mm = e / TK; } else { mm = e % TM; kk = e / TM; }
            const int m = m0 + mm, k = k0 + kk;
            float xr = 0.f, xi = 0.f;
            if (m < M && k < K) {
                const size_t idx = prm.layA.index(m * prm.a_rs + k * prm.a_cs, bin, 0);
                xr = prm.A[idx];
                xi = prm.A[idx + ((size_t)1 << prm.layA.tsh)];
            }
            ra_re[i] = xr; ra_im[i] = xi;
        }
#pragma unroll
        for (int i = 0; i < EB; ++i) {
            const int e = tid + i * 256;
            int nn, kk;
            if (prm.b_kfast) { kk = e % TK; nn = e / TK; } else { nn = e % TN; kk = e / TN; }
            const int n = n0 + nn, k = k0 + kk;
            float xr = 0.f, xi = 0.f;
            if (n < N && k < K) {
                const size_t idx = prm.layB.index(k * prm.b_rs + n * prm.b_cs, bin, 0);
                xr = prm.B[idx];
                xi = prm.B[idx + ((size_t)1 << prm.layB.tsh)];
            }
            rb_re[i] = xr; rb_im[i] = xi;
        }
    };
    auto store_tiles = [&]() {
#pragma unroll
        for (int i = 0; i < EA; ++i) {
            const int e = tid + i * 256;
            int mm, kk;
            if (prm.a_kfast) { kk = e % TK; mm = e / TK; } else { mm = e % TM; kk = e / TM; }
            As[0][kk][mm] = ra_re[i];
            As[1][kk][mm] = ra_im[i];
        }
#pragma unroll
        for (int i = 0; i < EB; ++i) {
            const int e = tid + i * 256;
            int nn, kk;
            if (prm.b_kfast) { kk = e % TK; nn = e / TK; } else { nn = e % TN; kk = e / TN; }
            Bs[0][kk][nn] = rb_re[i];
            Bs[1][kk][nn] = rb_im[i];
        }
    };

    const int nkt = (K + TK - 1) / TK;
    load_tiles(0);
    store_tiles();
    __syncthreads();
    const int lrow = lane & 31, lk = lane >> 5;
    for (int kt = 0; kt < nkt; ++kt) {
        if (kt + 1 < nkt) load_tiles((kt + 1) * TK);
#pragma unroll
        for (int ks = 0; ks < TK; ks += 2) {
            float a_re[FM], a_im[FM], a_in[FM], b_re[FN], b_im[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i) {
                const int mm = (wm * FM + i) * 32 + lrow;
                a_re[i] = As[0][ks + lk][mm];
                a_im[i] = As[1][ks + lk][mm];
                a_in[i] = -a_im[i];
            }
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const int nn = (wn * FN + j) * 32 + lrow;
                b_re[j] = Bs[0][ks + lk][nn];
                b_im[j] = Bs[1][ks + lk][nn];
            }
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    acc_re[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_re[i], b_re[j], acc_re[i][j], 0, 0, 0);
                    acc_im[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_re[i], b_im[j], acc_im[i][j], 0, 0, 0);
                    acc_re[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_in[i], b_im[j], acc_re[i][j], 0, 0, 0);
                    acc_im[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_im[i], b_re[j], acc_im[i][j], 0, 0, 0);
                }
        }
        __syncthreads();
        if (kt + 1 < nkt) {
            store_tiles();
            __syncthreads();
        }
    }

    // D layout of the 32x32x2 MFMA: lane l, register v -> row 8*(v/4) + 4*(l/32) + v%4, col l%32.
    const size_t cim = (size_t)1 << prm.layC.tsh;
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
                    prm.C[idx] = acc_re[i][j][v];
                    prm.C[idx + cim] = acc_im[i][j][v];
                }
            }
        }
}

template <int WGM, int WGN, int FM, int FN>
static hipError_t run_gemm(GemmParams prm, hipStream_t st) {
    constexpr int TM = WGM * FM * 32, TN = WGN * FN * 32;
    prm.tiles_m = (prm.M + TM - 1) / TM;
    prm.tiles_n = (prm.N + TN - 1) / TN;
    const long grid = (long)prm.bins * prm.tiles_m * prm.tiles_n;
    hipLaunchKernelGGL((cgemm_bins_kernel<WGM, WGN, FM, FN>), dim3((unsigned)grid), dim3(256), 0, st, prm);
    return hipGetLastError();
}

hipError_t launch_cgemm_bins(GemmOperand A, GemmOperand B, float *C, FreqLayout layC, long C_rs,
                             long C_cs, int M, int N, int K, int bins, hipStream_t st) {
    GemmParams prm;
    prm.A = A.ptr; prm.B = B.ptr; prm.C = C;
    prm.layA = A.lay; prm.layB = B.lay; prm.layC = layC;
    prm.a_rs = A.rs; prm.a_cs = A.cs; prm.b_rs = B.rs; prm.b_cs = B.cs;
    prm.c_rs = C_rs; prm.c_cs = C_cs;
    prm.M = M; prm.N = N; prm.K = K; prm.bins = bins;
    prm.a_kfast = (A.cs == 1);
    prm.b_kfast = (B.rs == 1);
    auto wgs = [&](int tm, int tn) { return (long)bins * ((M + tm - 1) / tm) * ((N + tn - 1) / tn); };
    if (M <= 32) return run_gemm<1, 4, 1, 1>(prm, st);
    if (M > 64 && N > 64 && wgs(128, 128) >= 512) return run_gemm<2, 2, 2, 2>(prm, st);
    if (N > 64 && wgs(64, 128) >= 512) return run_gemm<2, 2, 1, 2>(prm, st);
    if (M > 64 && wgs(128, 64) >= 512) return run_gemm<2, 2, 2, 1>(prm, st);
    return run_gemm<2, 2, 1, 1>(prm, st);
}

}  // namespace fc
