// Parameters shared by the contraction kernels.
#pragma once
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
    unsigned a_sign, b_sign;   // 0x80000000 to conjugate the operand (flips Im on the way to the MFMA)
    unsigned split_from;       // cgemm_tail_kernel: first workgroup index of the quadrant workgroups
    int fast;                  // addresses split into a uniform and a per-lane part (fast_addressing())
};

__device__ __forceinline__ float flip(float v, unsigned sign) {
    return __builtin_bit_cast(float, __builtin_bit_cast(unsigned, v) ^ sign);
}

constexpr int kXcds = 8;   // workgroup i is placed on XCD i % kXcds

}  // namespace fc
