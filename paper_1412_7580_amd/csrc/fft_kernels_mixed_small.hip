// 2-D transforms of the sizes 12, 14, 20, 24 and 28 (one odd factor 3, 5 or 7 in the
// per-lane part of the line, see fft_core.hpp), the small half of the bases Section 3.2 of the
// fbfft paper reaches through cuFFT.
#include "fft_kernels_impl.hpp"

namespace fc {

// Lanes per line, measured on 64-channel layers of 11x11 ... 54x54 images: the forward
// transforms like long per-lane parts (one lane per line up to 14, two up to 28, four up to 56),
// the inverses shorter ones, as for the powers of two.

hipError_t launch_fft2d_r2c_multi_small(const FwdOperand *ops, int nops, int N, LaunchCtx st) {
    switch (N) {
        case 12: return run_fwd2d_multi<12, 1, 32>(ops, nops, st);
        case 14: return run_fwd2d_multi<14, 1, 32>(ops, nops, st);
        case 20: return run_fwd2d_multi<10, 2, 16>(ops, nops, st);
        case 24: return run_fwd2d_multi<12, 2, 16>(ops, nops, st);
        case 28: return run_fwd2d_multi<14, 2, 16>(ops, nops, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_fft2d_r2c_small(const float *in, float *out, long planes, int h_in, int w_in, int N,
                                  bool conv, LaunchCtx st, const PlaneView *view) {
    switch (N) {
        case 12: return run_fwd2d<12, 1, 32>(in, out, planes, h_in, w_in, conv, st, view);
        case 14: return run_fwd2d<14, 1, 32>(in, out, planes, h_in, w_in, conv, st, view);
        case 20: return run_fwd2d<10, 2, 16>(in, out, planes, h_in, w_in, conv, st, view);
        case 24: return run_fwd2d<12, 2, 16>(in, out, planes, h_in, w_in, conv, st, view);
        case 28: return run_fwd2d<14, 2, 16>(in, out, planes, h_in, w_in, conv, st, view);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_fft2d_c2r_small(const float *in, float *out, long planes, int N, int h_out, int w_out,
                                  bool conv, float scale, bool accumulate, LaunchCtx st, const PlaneView *view) {
    switch (N) {
        case 12: return run_inv2d<3, 4, 32>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        case 14: return run_inv2d<7, 2, 32>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        case 20: return run_inv2d<10, 2, 16>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        case 24: return run_inv2d<6, 4, 16>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        case 28:
            // lane pairs when nearly all rows are kept (27x27 input gradients: 13.9 us against 14.7),
            // four lanes per line otherwise (5x5 weight gradients: 6.5 against 6.8)
            if (conv && 4 * (h_out + (view ? view->oy : 0)) > 3 * 28)
                return run_inv2d<14, 2, 16>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
            return run_inv2d<7, 4, 16>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace fc
