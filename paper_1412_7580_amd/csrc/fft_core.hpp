// In-register small FFT building blocks for gfx950 (wave64).
//
// A length-N line (N = L*G, G in {1,2,4}) is transformed by G adjacent lanes.  Lane g holds
// the decimated samples x[g + G*m], m < L, in L complex registers, runs an L-point FFT on
// them with fully static register indexing (straight-line code, twiddles are immediates),
// and, for G > 1, finishes with log2(G) radix-2 decimation-in-time steps across the lane
// group through DPP quad-permutes.  Afterwards each lane holds a block of L consecutive bins.
//
// This replaces the one-element-per-lane warp-shuffle butterflies of Section 5.2 of the
// fbfft paper: on CDNA every cross-lane permute other than DPP goes through the LDS pipe,
// the very bottleneck Section 6 reports, so the butterflies stay inside a lane and only the
// last one or two stages of the two largest sizes cross lanes.
#pragma once
#include <hip/hip_runtime.h>
#include <type_traits>

namespace fc {

// ---------------------------------------------------------------- compile-time twiddles
constexpr double kPi = 3.14159265358979323846264338327950288;

constexpr double sin_small(double x) {  // |x| <= pi/4, Taylor, error < 1e-17
    double x2 = x * x, term = x, sum = x;
    for (int i = 1; i < 14; ++i) { term *= -x2 / double((2 * i) * (2 * i + 1)); sum += term; }
    return sum;
}
constexpr double cos_small(double x) {
    double x2 = x * x, term = 1.0, sum = 1.0;
    for (int i = 1; i < 14; ++i) { term *= -x2 / double((2 * i - 1) * (2 * i)); sum += term; }
    return sum;
}
struct cplx_d { double re, im; };
// exp(+2 pi i k / n), by octant reduction so that exact values (0, +-1) and symmetries come
// out exactly.  Powers of two up to 1024 keep their own path (angles in 1024ths of a turn);
// any other n reduces 8k/n to an octant and a remainder.
constexpr cplx_d unit_root(int k, int n) {
    const bool pow2 = (n & (n - 1)) == 0 && n <= 1024;
    int q = 0;
    double c = 0, s = 0;
    if (pow2) {
        int K = ((k % n) + n) % n * (1024 / n);
        q = K / 256;
        int r = K % 256;
        if (r <= 128) { double a = 2.0 * kPi * r / 1024.0; c = cos_small(a); s = sin_small(a); }
        else { double a = 2.0 * kPi * (256 - r) / 1024.0; c = sin_small(a); s = cos_small(a); }
        if (r == 0) { c = 1.0; s = 0.0; }
    } else {
        const int t = 8 * (((k % n) + n) % n);
        const int oct = t / n, rem = t % n;          // angle = (oct + rem / n) * pi / 4
        q = oct / 2;
        if (oct % 2 == 0) { double a = kPi * rem / (4.0 * n); c = cos_small(a); s = sin_small(a); }
        else { double a = kPi * (n - rem) / (4.0 * n); c = sin_small(a); s = cos_small(a); }
        if (rem == 0 && oct % 2 == 0) { c = 1.0; s = 0.0; }
    }
    switch (q) {
        case 0: return {c, s};
        case 1: return {-s, c};
        case 2: return {-c, -s};
        default: return {s, -c};
    }
}

template <int I, int E, class F>
__device__ __forceinline__ void static_for(F &&f) {
    if constexpr (I < E) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, E>(f);
    }
}

// ---------------------------------------------------------------- L-point FFT in registers
// DIR = -1 forward (exp(-2 pi i jk/L)), +1 inverse (unscaled).  Natural order in and out.
template <int L, int DIR>
__device__ __forceinline__ void fft_leaf(float (&re)[L], float (&im)[L]) {
    if constexpr (L == 2) {
        float ar = re[0], ai = im[0], br = re[1], bi = im[1];
        re[0] = ar + br; im[0] = ai + bi;
        re[1] = ar - br; im[1] = ai - bi;
    } else if constexpr (L == 4) {
        // radix-4 butterfly
        float s0r = re[0] + re[2], s0i = im[0] + im[2];
        float d0r = re[0] - re[2], d0i = im[0] - im[2];
        float s1r = re[1] + re[3], s1i = im[1] + im[3];
        float d1r = re[1] - re[3], d1i = im[1] - im[3];
        re[0] = s0r + s1r; im[0] = s0i + s1i;
        re[2] = s0r - s1r; im[2] = s0i - s1i;
        if constexpr (DIR < 0) {   // X1 = d0 - i d1, X3 = d0 + i d1
            re[1] = d0r + d1i; im[1] = d0i - d1r;
            re[3] = d0r - d1i; im[3] = d0i + d1r;
        } else {                   // X1 = d0 + i d1, X3 = d0 - i d1
            re[1] = d0r - d1i; im[1] = d0i + d1r;
            re[3] = d0r + d1i; im[3] = d0i - d1r;
        }
    } else if constexpr (L % 2 == 1) {
        // Odd length (3, 5, 7, ...): the definition, with the samples m and L - m paired so that
        // bins k and L - k share their products:
        //   X_k, X_{L-k} = x_0 + sum_m cos(2 pi mk/L) (x_m + x_{L-m})  +-  DIR i sum_m sin(2 pi mk/L) (x_m - x_{L-m})
        constexpr int H = (L - 1) / 2;
        float ar[H], ai[H], br[H], bi[H];
        float s0r = re[0], s0i = im[0];
#pragma unroll
        for (int m = 1; m <= H; ++m) {
            ar[m - 1] = re[m] + re[L - m]; ai[m - 1] = im[m] + im[L - m];
            br[m - 1] = re[m] - re[L - m]; bi[m - 1] = im[m] - im[L - m];
            s0r += ar[m - 1]; s0i += ai[m - 1];
        }
        const float x0r = re[0], x0i = im[0];
        re[0] = s0r; im[0] = s0i;
        static_for<1, H + 1>([&](auto kk) {
            constexpr int k = decltype(kk)::value;
            float pr = x0r, pi = x0i, qr = 0.f, qi = 0.f;
            static_for<1, H + 1>([&](auto mm) {
                constexpr int m = decltype(mm)::value;
                constexpr cplx_d w = unit_root((m * k) % L, L);
                constexpr float c = (float)w.re, s = (float)w.im;
                pr += c * ar[m - 1]; pi += c * ai[m - 1];
                qr += s * br[m - 1]; qi += s * bi[m - 1];
            });
            if constexpr (DIR < 0) {   // X_k = P - i Q, X_{L-k} = P + i Q
                re[k] = pr + qi; im[k] = pi - qr;
                re[L - k] = pr - qi; im[L - k] = pi + qr;
            } else {
                re[k] = pr - qi; im[k] = pi + qr;
                re[L - k] = pr + qi; im[L - k] = pi - qr;
            }
        });
    } else {
        constexpr int H = L / 2;
        float er[H], ei[H], pr[H], pi[H];
#pragma unroll
        for (int m = 0; m < H; ++m) {
            er[m] = re[2 * m]; ei[m] = im[2 * m];
            pr[m] = re[2 * m + 1]; pi[m] = im[2 * m + 1];
        }
        fft_leaf<H, DIR>(er, ei);
        fft_leaf<H, DIR>(pr, pi);
        static_for<0, H>([&](auto kk) {
            constexpr int k = decltype(kk)::value;
            float tr, ti;
            if constexpr (k == 0) {
                tr = pr[k]; ti = pi[k];
            } else if constexpr (4 * k == L) {          // multiply by DIR * i
                if constexpr (DIR < 0) { tr = pi[k]; ti = -pr[k]; }
                else { tr = -pi[k]; ti = pr[k]; }
            } else {
                constexpr cplx_d w = unit_root(DIR * k, L);
                constexpr float wr = (float)w.re, wi = (float)w.im;
                tr = wr * pr[k] - wi * pi[k];
                ti = wr * pi[k] + wi * pr[k];
            }
            re[k] = er[k] + tr; im[k] = ei[k] + ti;
            re[k + H] = er[k] - tr; im[k + H] = ei[k] - ti;
        });
    }
}

// ---------------------------------------------------------------- cross-lane helpers
// Value held by lane ^ 1 / ^ 2 / ^ 3 of the same quad: DPP quad_perm.
template <int CTRL>
__device__ __forceinline__ float quad_dpp(float v) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float lane_xor1(float v) { return quad_dpp<0xB1>(v); }   // [1,0,3,2]
__device__ __forceinline__ float lane_xor2(float v) { return quad_dpp<0x4E>(v); }   // [2,3,0,1]
__device__ __forceinline__ float lane_xor3(float v) { return quad_dpp<0x1B>(v); }   // [3,2,1,0]
// Lane ^ 7 of the same group of eight: DPP row_half_mirror; lane ^ 4 = (lane ^ 7) ^ 3.
__device__ __forceinline__ float lane_xor7(float v) { return quad_dpp<0x141>(v); }
__device__ __forceinline__ float lane_xor4(float v) { return lane_xor3(lane_xor7(v)); }

// Block of output bins held by lane g after fft_group: lane g holds X[k + L*group_block(g)].
template <int G>
__device__ __forceinline__ int group_block(int g) {
    if constexpr (G == 4) return ((g & 1) << 1) | (g >> 1);
    else if constexpr (G == 8) return ((g & 1) << 2) | (g & 2) | (g >> 2);
    else return g;
}

// N = L*G point FFT over G adjacent lanes (G = 1, 2, 4 or 8).  On entry lane g holds x[g + G*m]
// in register m; on exit lane g holds X[k + L*group_block<G>(g)] in register k.  All G lanes
// of a group must be active together.  The cross-lane part is one (G = 2) or two (G = 4)
// radix-2 decimation-in-time steps: the upper lane of each pair multiplies by the step's
// twiddle, the pair swaps values through DPP and forms sum / difference.
// HALF (lane pairs only): the result is scaled by 1/2, at no cost: the factor goes into the
// twiddles of the cross-lane step, whose product every lane forms anyway.
template <int L, int G, int DIR, bool HALF = false>
__device__ __forceinline__ void fft_group(float (&re)[L], float (&im)[L], int g) {
    static_assert(G == 1 || G == 2 || G == 4 || G == 8, "one, two, four or eight lanes per line");
    static_assert(!HALF || G == 2, "the free scaling exists for lane pairs");
    constexpr double SCALE = HALF ? 0.5 : 1.0;
    fft_leaf<L, DIR>(re, im);
    if constexpr (G == 2) {
        float sgn = g ? -1.0f : 1.0f;
        // (opaque to the compiler: knowing that it is +-1 it would form both the sum and the
        // difference and select between them, three instructions where a product and a sum do)
        asm volatile("" : "+v"(sgn));
        static_for<0, L>([&](auto kk) {
            constexpr int k = decltype(kk)::value;
            constexpr cplx_d w = unit_root(DIR * k, 2 * L);
            constexpr float cr = (float)(SCALE * w.re), ci = (float)(SCALE * w.im), one = (float)SCALE;
            const float wr = g ? cr : one, wi = g ? ci : 0.0f;
            const float tr = wr * re[k] - wi * im[k];
            const float ti = wr * im[k] + wi * re[k];
            const float qr = lane_xor1(tr), qi = lane_xor1(ti);
            re[k] = qr + sgn * tr;
            im[k] = qi + sgn * ti;
        });
    } else if constexpr (G == 4) {
        const bool up = (g >> 1) != 0, odd = (g & 1) != 0, last = g == 3;
        const float s1 = up ? -1.0f : 1.0f, s2 = odd ? -1.0f : 1.0f;
        static_for<0, L>([&](auto kk) {
            constexpr int k = decltype(kk)::value;
            // step 1, lanes (0,2) and (1,3): even/odd halves of the 2L-point sub-transforms
            constexpr cplx_d w1 = unit_root(DIR * k, 2 * L);
            constexpr float c1 = (float)w1.re, d1 = (float)w1.im;
            const float w1r = up ? c1 : 1.0f, w1i = up ? d1 : 0.0f;
            const float tr = w1r * re[k] - w1i * im[k];
            const float ti = w1r * im[k] + w1i * re[k];
            const float ar = lane_xor2(tr) + s1 * tr;
            const float ai = lane_xor2(ti) + s1 * ti;
            // step 2, lanes (0,1) and (2,3): twiddle w_N^k on lane 1, w_N^(k+L) on lane 3
            constexpr cplx_d w2 = unit_root(DIR * k, 4 * L), w3 = unit_root(DIR * (k + L), 4 * L);
            constexpr float c2 = (float)w2.re, d2 = (float)w2.im, c3 = (float)w3.re, d3 = (float)w3.im;
            const float w2r = odd ? (last ? c3 : c2) : 1.0f, w2i = odd ? (last ? d3 : d2) : 0.0f;
            const float ur = w2r * ar - w2i * ai;
            const float ui = w2r * ai + w2i * ar;
            re[k] = lane_xor1(ur) + s2 * ur;
            im[k] = lane_xor1(ui) + s2 * ui;
        });
    } else if constexpr (G == 8) {
        // Three steps, pairing lanes g ^ 4, g ^ 2, g ^ 1.  With g = 4u + 2v + o: step 1 joins
        // the stride-8 sequences g and g + 4 (twiddle w_2L^k on u = 1), step 2 the stride-4
        // sequences (twiddle w_4L^(k + L u) on v = 1), step 3 the two stride-2 sequences
        // (twiddle w_8L^(k + L u + 2L v) on o = 1); each lane keeps the sum (bit clear) or the
        // difference (bit set), so lane g ends with block u + 2v + 4o.
        const bool u = (g & 4) != 0, v = (g & 2) != 0, o = (g & 1) != 0;
        const float s1 = u ? -1.0f : 1.0f, s2 = v ? -1.0f : 1.0f, s3 = o ? -1.0f : 1.0f;
        static_for<0, L>([&](auto kk) {
            constexpr int k = decltype(kk)::value;
            constexpr cplx_d w1 = unit_root(DIR * k, 2 * L);
            constexpr float c1 = (float)w1.re, d1 = (float)w1.im;
            const float w1r = u ? c1 : 1.0f, w1i = u ? d1 : 0.0f;
            const float tr = w1r * re[k] - w1i * im[k];
            const float ti = w1r * im[k] + w1i * re[k];
            const float ar = lane_xor4(tr) + s1 * tr;
            const float ai = lane_xor4(ti) + s1 * ti;
            constexpr cplx_d w20 = unit_root(DIR * k, 4 * L), w21 = unit_root(DIR * (k + L), 4 * L);
            constexpr float c20 = (float)w20.re, d20 = (float)w20.im, c21 = (float)w21.re, d21 = (float)w21.im;
            const float w2r = v ? (u ? c21 : c20) : 1.0f, w2i = v ? (u ? d21 : d20) : 0.0f;
            const float br = w2r * ar - w2i * ai;
            const float bi = w2r * ai + w2i * ar;
            const float cr = lane_xor2(br) + s2 * br;
            const float ci = lane_xor2(bi) + s2 * bi;
            constexpr cplx_d w30 = unit_root(DIR * k, 8 * L), w31 = unit_root(DIR * (k + L), 8 * L),
                             w32 = unit_root(DIR * (k + 2 * L), 8 * L), w33 = unit_root(DIR * (k + 3 * L), 8 * L);
            constexpr float c30 = (float)w30.re, d30 = (float)w30.im, c31 = (float)w31.re, d31 = (float)w31.im,
                            c32 = (float)w32.re, d32 = (float)w32.im, c33 = (float)w33.re, d33 = (float)w33.im;
            const float w3r = o ? (v ? (u ? c33 : c32) : (u ? c31 : c30)) : 1.0f;
            const float w3i = o ? (v ? (u ? d33 : d32) : (u ? d31 : d30)) : 0.0f;
            const float er = w3r * cr - w3i * ci;
            const float ei = w3r * ci + w3i * cr;
            re[k] = lane_xor1(er) + s3 * er;
            im[k] = lane_xor1(ei) + s3 * ei;
        });
    }
}

// The per-lane twiddles of the cross-lane steps of a line spread over G lanes, as a table for
// kernels that keep it in LDS: entry (step s, register k, lane g) is the factor lane g applies
// to register k before step s (1 for the lanes that keep their value), for DIR = +1; the
// other direction uses the conjugate.  Step s pairs lanes that differ in bit log2(G)-1-s of g;
// the exponent collects the bits already used (see fft_group).  One 8-byte LDS read replaces
// the selects among compile-time constants (up to four constants moved into registers and
// three selects per component), a third of the vector instructions of the eight-lane kernels.
template <int G> constexpr int kGroupSteps = G == 8 ? 3 : G == 4 ? 2 : 1;
// Lines of four or eight lanes read the table; lane pairs keep the immediates (one select per
// component; with the table the 32x32 transforms measured 2..6 % slower).
template <int G> constexpr bool kLdsTwiddles = G >= 4;
template <int L, int G> constexpr int kGroupTwiddleFloats = kLdsTwiddles<G> ? kGroupSteps<G> * L * G * 2 : 0;

template <int L, int G>
struct GroupTwiddles {
    float v[kGroupSteps<G> * L * G * 2];
    constexpr GroupTwiddles() : v{} {
        constexpr int S = kGroupSteps<G>;
        for (int s = 0; s < S; ++s)
            for (int k = 0; k < L; ++k)
                for (int g = 0; g < G; ++g) {
                    const bool on = ((g >> (S - 1 - s)) & 1) != 0;
                    int e = k;
                    for (int t = 0; t < s; ++t) e += ((g >> (S - 1 - t)) & 1) * (L << t);
                    const cplx_d w = on ? unit_root(e, (2 << s) * L) : cplx_d{1.0, 0.0};
                    v[((s * L + k) * G + g) * 2 + 0] = (float)w.re;
                    v[((s * L + k) * G + g) * 2 + 1] = (float)w.im;
                }
    }
};
template <int L, int G> __device__ const GroupTwiddles<L, G> kGroupTwiddles{};

// Copy the table to LDS (all threads of the workgroup; a barrier must follow before use).
template <int L, int G, int BT>
__device__ __forceinline__ void load_group_twiddles(float *dst, int tid) {
    if constexpr (kLdsTwiddles<G>) {
        for (int i = tid; i < kGroupTwiddleFloats<L, G>; i += BT) dst[i] = kGroupTwiddles<L, G>.v[i];
    }
}

// fft_group<L, G, DIR> for G = 4 or 8 with the twiddles read from the LDS copy of the table; tw
// points at this lane's entry of (step 0, register 0).
template <int L, int G, int DIR>
__device__ __forceinline__ void fft_group_lds(float (&re)[L], float (&im)[L], int g, const float2 *tw) {
    static_assert(G == 4 || G == 8, "four or eight lanes per line");
    fft_leaf<L, DIR>(re, im);
    constexpr float D = (float)DIR;
    auto twiddle = [&](const float2 w, float &xr, float &xi) {
        const float tr = w.x * xr - D * w.y * xi;
        const float ti = w.x * xi + D * w.y * xr;
        xr = tr; xi = ti;
    };
    if constexpr (G == 8) {
        const float s1 = (g & 4) ? -1.0f : 1.0f, s2 = (g & 2) ? -1.0f : 1.0f, s3 = (g & 1) ? -1.0f : 1.0f;
        static_for<0, L>([&](auto kk) {
            constexpr int k = decltype(kk)::value;
            float xr = re[k], xi = im[k];
            twiddle(tw[(0 * L + k) * 8], xr, xi);
            float yr = lane_xor4(xr) + s1 * xr, yi = lane_xor4(xi) + s1 * xi;
            twiddle(tw[(1 * L + k) * 8], yr, yi);
            float zr = lane_xor2(yr) + s2 * yr, zi = lane_xor2(yi) + s2 * yi;
            twiddle(tw[(2 * L + k) * 8], zr, zi);
            re[k] = lane_xor1(zr) + s3 * zr;
            im[k] = lane_xor1(zi) + s3 * zi;
        });
    } else {
        const float s1 = (g & 2) ? -1.0f : 1.0f, s2 = (g & 1) ? -1.0f : 1.0f;
        static_for<0, L>([&](auto kk) {
            constexpr int k = decltype(kk)::value;
            float xr = re[k], xi = im[k];
            twiddle(tw[(0 * L + k) * 4], xr, xi);
            float yr = lane_xor2(xr) + s1 * xr, yi = lane_xor2(xi) + s1 * xi;
            twiddle(tw[(1 * L + k) * 4], yr, yi);
            re[k] = lane_xor1(yr) + s2 * yr;
            im[k] = lane_xor1(yi) + s2 * yi;
        });
    }
}

// The line transform as the kernels call it: lines of four or eight lanes take their twiddles
// from the table at `tw` in LDS, the others have them as immediates.
template <int L, int G, int DIR, bool HALF = false>
__device__ __forceinline__ void fft_lines(float (&re)[L], float (&im)[L], int g, const float *tw) {
    if constexpr (kLdsTwiddles<G>) fft_group_lds<L, G, DIR>(re, im, g, reinterpret_cast<const float2 *>(tw) + g);
    else fft_group<L, G, DIR, HALF>(re, im, g);
}

// Whether the forward 2-D kernels move the factor 1/2 of the two-for-one split of their row phase
// into the column transform (lane pairs: see fft_group's HALF).  The row phase then leaves twice
// the row spectra, the column phase halves them again; results are unchanged bit for bit,
// since halving is exact.
template <int G> constexpr bool kDeferHalf = G == 2;

// Number of registers of split spectrum a lane keeps (see split_two_real).
template <int L, int G> struct SplitRegs { static constexpr int A = (G == 1) ? L / 2 : L, B = (G == 1) ? L / 2 : 1; };

// Slot (0 .. N/2-1) of the half spectrum that register k of lane g holds after
// split_two_real for G > 1; slot 0 is the packed pair of real bins (X_0, X_{N/2}).
template <int L, int G>
__device__ __forceinline__ int split_slot(int g, int k) {
    if constexpr (G == 2) return (g && k) ? L - k : k;
    else if constexpr (G == 8) {
        // even lanes hold bins k + L b of the first line (b = group_block(g) < 4); odd lanes hold
        // bin N - (k + L b) of the second line (b >= 4), the Nyquist bin packed into slot 0
        const int b = group_block<8>(g);
        if (!(g & 1)) return k + L * b;
        if (k) return L * (7 - b) + L - k;
        return b == 4 ? 0 : L * (8 - b);
    } else {
        switch (g) {
            case 0: return k;
            case 2: return L + k;
            case 3: return k ? L - k : L;
            default: return k ? 2 * L - k : 0;
        }
    }
}

// After a forward fft_group of z = a + i b (a, b real lines), split the spectrum into the
// spectra of a and b (the standard two-for-one trick the paper cites in Section 5.2).
// With NH = L*G/2 slots per line, slot 0 holding the two real bins (X_0, X_{N/2}) as (re, im):
//   G == 1: are/aim[k], bre/bim[k] for k < NH are slot k of a and of b.
//   G  > 1: even lanes get line a, odd lanes line b; register k holds slot split_slot(g, k).
//           Both are returned in are/aim.
// TWICE: leave out the factor 1/2 (the spectra come out doubled; G > 1 only).
template <int L, int G, bool TWICE = false>
__device__ __forceinline__ void split_two_real(const float (&re)[L], const float (&im)[L], int g,
                                               float (&are)[SplitRegs<L, G>::A],
                                               float (&aim)[SplitRegs<L, G>::A],
                                               float (&bre)[SplitRegs<L, G>::B],
                                               float (&bim)[SplitRegs<L, G>::B]) {
    static_assert(!TWICE || G == 2, "the doubled split is used with lane pairs only");
    if constexpr (G == 1) {
        constexpr int NH = L / 2;
        are[0] = re[0]; aim[0] = re[NH];
        bre[0] = im[0]; bim[0] = im[NH];
#pragma unroll
        for (int k = 1; k < NH; ++k) {
            const float xr = re[k], xi = im[k], yr = re[L - k], yi = im[L - k];
            are[k] = 0.5f * (xr + yr); aim[k] = 0.5f * (xi - yi);
            bre[k] = 0.5f * (xi + yi); bim[k] = 0.5f * (yr - xr);
        }
    } else {
        // Every lane pairs its own Z[j] with Z[N-j] fetched from the mirror lane.  Even lanes
        // form A[j] = (own + conj(other)) / 2, odd lanes B[N-j] = (other - conj(own)) / (2i).
        const bool odd = (g & 1) != 0;
        {   // register 0: bins 0, N/2 (and N/4, 3N/4 for G = 4) pair up with the neighbour lane
            const float o0r = lane_xor1(re[0]), o0i = lane_xor1(im[0]);
            if constexpr (G == 2) {
                constexpr float two = TWICE ? 2.0f : 1.0f;
                are[0] = two * (odd ? o0i : re[0]);
                aim[0] = two * (odd ? im[0] : o0r);
            } else if constexpr (G == 4) {
                const float a_r = 0.5f * (re[0] + o0r), a_i = 0.5f * (im[0] - o0i);
                const float b_r = 0.5f * (o0i + im[0]), b_i = 0.5f * (re[0] - o0r);
                const bool up = (g >> 1) != 0;
                are[0] = up ? (odd ? b_r : a_r) : (odd ? o0i : re[0]);
                aim[0] = up ? (odd ? b_i : a_i) : (odd ? im[0] : o0r);
            } else {
                // G = 8: bin L b pairs with bin L (8 - b): lanes 0,1 hold bins 0 and N/2, lanes 2,3
                // are neighbours, lanes 4..7 pair up as (4,7) and (5,6)
                const bool hi = (g & 4) != 0;
                const float p3r = lane_xor3(re[0]), p3i = lane_xor3(im[0]);
                const float pr = hi ? p3r : o0r, pi = hi ? p3i : o0i;
                const float a_r = 0.5f * (re[0] + pr), a_i = 0.5f * (im[0] - pi);
                const float b_r = 0.5f * (pi + im[0]), b_i = 0.5f * (re[0] - pr);
                const bool first = g < 2;
                are[0] = first ? (odd ? o0i : re[0]) : (odd ? b_r : a_r);
                aim[0] = first ? (odd ? im[0] : o0r) : (odd ? b_i : a_i);
            }
        }
        static_for<1, L>([&](auto kk) {
            constexpr int k = decltype(kk)::value;
            float orr, oi;
            if constexpr (G == 2) { orr = lane_xor1(re[L - k]); oi = lane_xor1(im[L - k]); }
            else if constexpr (G == 4) { orr = lane_xor3(re[L - k]); oi = lane_xor3(im[L - k]); }
            else { orr = lane_xor7(re[L - k]); oi = lane_xor7(im[L - k]); }
            constexpr float h = TWICE ? 1.0f : 0.5f;
            const float a_r = h * (re[k] + orr), a_i = h * (im[k] - oi);
            const float b_r = h * (oi + im[k]), b_i = h * (re[k] - orr);
            are[k] = odd ? b_r : a_r;
            aim[k] = odd ? b_i : a_i;
        });
        bre[0] = 0.f; bim[0] = 0.f;
    }
}

}  // namespace fc
