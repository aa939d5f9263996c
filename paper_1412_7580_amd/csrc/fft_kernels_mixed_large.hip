// 2-D transforms of the sizes 36, 40, 48, 56, 80, 96 and 112 (an odd factor 3, 5, 7 or 9 in the
// per-lane part of the line), and the dispatch of every size that is not a power of two.
#include "fft_kernels_impl.hpp"

namespace fc {

// Lanes per line, measured on 64-channel layers of 11x11 ... 54x54 images: the forward
// transforms like long per-lane parts (one lane per line up to 28, e.g. basis 20: 13.7 us
// against 18.1 with lane pairs; four lanes from 40 to 56), the inverses mostly shorter ones, as
// for the powers of two.

hipError_t launch_fft2d_r2c_multi_small(const FwdOperand *ops, int nops, int N, LaunchCtx st);
hipError_t launch_fft2d_r2c_small(const float *in, float *out, long planes, int h_in, int w_in, int N,
                                  bool conv, LaunchCtx st, const PlaneView *view);
hipError_t launch_fft2d_c2r_small(const float *in, float *out, long planes, int N, int h_out, int w_out,
                                  bool conv, float scale, bool accumulate, LaunchCtx st, const PlaneView *view);

hipError_t launch_fft2d_r2c_multi_mixed(const FwdOperand *ops, int nops, int N, LaunchCtx st) {
    switch (N) {
        case 36: return run_fwd2d_multi<9, 4, 4>(ops, nops, st);
        case 40: return run_fwd2d_multi<10, 4, 4>(ops, nops, st);
        case 48: return run_fwd2d_multi<12, 4, 4>(ops, nops, st);
        case 56: return run_fwd2d_multi<14, 4, 4>(ops, nops, st);
        case 80: return run_fwd2d_multi<10, 8, 1>(ops, nops, st);
        case 96: return run_fwd2d_multi<12, 8, 1>(ops, nops, st);
        case 112: return run_fwd2d_multi<14, 8, 1>(ops, nops, st);
        default: return launch_fft2d_r2c_multi_small(ops, nops, N, st);
    }
}

hipError_t launch_fft2d_r2c_mixed(const float *in, float *out, long planes, int h_in, int w_in, int N,
                                  bool conv, LaunchCtx st, const PlaneView *view) {
    switch (N) {
        case 36: return run_fwd2d<9, 4, 4>(in, out, planes, h_in, w_in, conv, st, view);
        case 40: return run_fwd2d<10, 4, 4>(in, out, planes, h_in, w_in, conv, st, view);
        case 48: return run_fwd2d<12, 4, 4>(in, out, planes, h_in, w_in, conv, st, view);
        case 56: return run_fwd2d<14, 4, 4>(in, out, planes, h_in, w_in, conv, st, view);
        case 80: return run_fwd2d<10, 8, 1>(in, out, planes, h_in, w_in, conv, st, view);
        case 96: return run_fwd2d<12, 8, 1>(in, out, planes, h_in, w_in, conv, st, view);
        case 112: return run_fwd2d<14, 8, 1>(in, out, planes, h_in, w_in, conv, st, view);
        default: return launch_fft2d_r2c_small(in, out, planes, h_in, w_in, N, conv, st, view);
    }
}

hipError_t launch_fft2d_c2r_mixed(const float *in, float *out, long planes, int N, int h_out, int w_out,
                                  bool conv, float scale, bool accumulate, LaunchCtx st, const PlaneView *view) {
    switch (N) {
        case 36: return run_inv2d<9, 4, 4>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);   // (18,2): 8.2 -> 10.5 us for the weight gradients of a 36x36 layer
        case 40: return run_inv2d<10, 4, 4>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        case 48: return run_inv2d<12, 4, 4>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        case 56: return run_inv2d<14, 4, 4>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        case 80: return run_inv2d<10, 8, 1>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        case 96: return run_inv2d<12, 8, 1>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        case 112: return run_inv2d<14, 8, 1>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        default: return launch_fft2d_c2r_small(in, out, planes, N, h_out, w_out, conv, scale, accumulate, st, view);
    }
}

hipError_t launch_fft2d_c2r_pair_small(const InvOperand *ops, int N, LaunchCtx st);

// (From 36 on the backward pass never pairs its products: the contractions of those bases go out
// as separate launches, each followed by its inverse transform.)
hipError_t launch_fft2d_c2r_pair_mixed(const InvOperand *ops, int N, LaunchCtx st) {
    return launch_fft2d_c2r_pair_small(ops, N, st);
}

}  // namespace fc
