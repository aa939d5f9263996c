// Stand-alone 2-D transforms (natural layout [plane][N][N/2+1]) of the sizes where the best
// split of a line over lanes and the best number of planes per workgroup differ from the
// convolution path's.  There the planes per workgroup are the tile of the frequency layout;
// here nothing ties them, and smaller workgroups measured faster: more of them are resident,
// so loads, butterflies and stores of different workgroups overlap better.  Measured on
// 256 MiB batches of (n-3) x (n-3) inputs, same process, TB/s, the convolution path's choice ->
// the one here (first sweep; a second one, after the cross-lane twiddles of four- and
// eight-lane lines had moved to an LDS table, shifted 16, 32, 40, 48 and 56 by another 1..6 %
// towards more lanes per line and fewer planes):
//   forward  14: 5.36 -> 5.97   16: 5.31 -> 5.74   20: 5.56 -> 5.73   24: 5.31 -> 5.77   28: 5.32 -> 5.52
//            32: 5.03 -> 5.44   56: 4.37 -> 4.75   64: 4.01 -> 4.70
//   inverse   8: 5.57 -> 5.98   12: 4.48 -> 5.96   16: 5.43 -> 5.51   24: 4.95 -> 5.51   28: 4.70 -> 5.42
//            32: 5.23 -> 5.54   56: 4.83 -> 5.00   64: 4.65 -> 5.03
#include "fft_kernels_impl.hpp"

namespace fc {

// Returns hipErrorNotSupported for the sizes that keep the convolution path's choice.
hipError_t launch_fft2d_r2c_natural(const float *in, float *out, long planes, int h_in, int w_in, int N, LaunchCtx st) {
    switch (N) {
        case 10: return run_fwd2d<5, 2, 32, false>(in, out, planes, h_in, w_in, false, st, nullptr);
        case 18: return run_fwd2d<9, 2, 8, false>(in, out, planes, h_in, w_in, false, st, nullptr);
        case 14: return run_fwd2d<7, 2, 16, false>(in, out, planes, h_in, w_in, false, st, nullptr);
        case 16: return run_fwd2d<8, 2, 4, false>(in, out, planes, h_in, w_in, false, st, nullptr);
        case 20: return run_fwd2d<10, 2, 8, false>(in, out, planes, h_in, w_in, false, st, nullptr);
        case 24: return run_fwd2d<12, 2, 4, false>(in, out, planes, h_in, w_in, false, st, nullptr);
        case 28: return run_fwd2d<14, 2, 4, false>(in, out, planes, h_in, w_in, false, st, nullptr);
        case 32: return run_fwd2d<8, 4, 4, false>(in, out, planes, h_in, w_in, false, st, nullptr);
        case 36: return run_fwd2d<18, 2, 4, false>(in, out, planes, h_in, w_in, false, st, nullptr);   // (9,4,4): 4.4..4.8 -> 5.0..5.2 TB/s
        case 48: return run_fwd2d<12, 4, 2, false>(in, out, planes, h_in, w_in, false, st, nullptr);
        case 56: return run_fwd2d<7, 8, 2, false>(in, out, planes, h_in, w_in, false, st, nullptr);
        case 64: return run_fwd2d<8, 8, 1, false>(in, out, planes, h_in, w_in, false, st, nullptr);
        default: return hipErrorNotSupported;
    }
}

hipError_t launch_fft2d_c2r_natural(const float *in, float *out, long planes, int N, int h_out, int w_out,
                                    float scale, bool accumulate, LaunchCtx st) {
    switch (N) {
        case 18: return run_inv2d<9, 2, 8, false>(in, out, planes, h_out, w_out, false, scale, accumulate, st, nullptr);
        case 8: return run_inv2d<4, 2, 64, false>(in, out, planes, h_out, w_out, false, scale, accumulate, st, nullptr);
        case 12: return run_inv2d<6, 2, 32, false>(in, out, planes, h_out, w_out, false, scale, accumulate, st, nullptr);
        case 16: return run_inv2d<8, 2, 16, false>(in, out, planes, h_out, w_out, false, scale, accumulate, st, nullptr);
        case 24: return run_inv2d<6, 4, 4, false>(in, out, planes, h_out, w_out, false, scale, accumulate, st, nullptr);
        case 28: return run_inv2d<7, 4, 8, false>(in, out, planes, h_out, w_out, false, scale, accumulate, st, nullptr);
        case 32: return run_inv2d<8, 4, 2, false>(in, out, planes, h_out, w_out, false, scale, accumulate, st, nullptr);
        case 40: return run_inv2d<10, 4, 2, false>(in, out, planes, h_out, w_out, false, scale, accumulate, st, nullptr);
        case 48: return run_inv2d<12, 4, 2, false>(in, out, planes, h_out, w_out, false, scale, accumulate, st, nullptr);
        case 56: return run_inv2d<14, 4, 2, false>(in, out, planes, h_out, w_out, false, scale, accumulate, st, nullptr);
        case 64: return run_inv2d<8, 8, 1, false>(in, out, planes, h_out, w_out, false, scale, accumulate, st, nullptr);
        default: return hipErrorNotSupported;
    }
}

}  // namespace fc
