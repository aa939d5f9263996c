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
};

constexpr int kXcds = 8;   // workgroup i is placed on XCD i % kXcds

}  // namespace fc
