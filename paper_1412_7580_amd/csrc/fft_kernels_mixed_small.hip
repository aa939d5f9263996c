// 2-D transforms of the sizes 10, 12, 14, 18, 20, 24 and 28 (an odd factor 3, 5, 7 or 9 in the
// per-lane part of the line, see fft_core.hpp), the small half of the bases Section 3.2 of the
// fbfft paper reaches through cuFFT.
#include "fft_kernels_impl.hpp"

namespace fc {

// Lanes per line, measured on 64-channel layers of 11x11 ... 54x54 images: the forward
// transforms like long per-lane parts (one lane per line up to 28, e.g. basis 20: 13.7 us
// against 18.1 with lane pairs; four lanes from 40 to 56), the inverses mostly shorter ones, as
// for the powers of two.

hipError_t launch_fft2d_r2c_multi_small(const FwdOperand *ops, int nops, int N, LaunchCtx st) {
    switch (N) {
        case 10: return run_fwd2d_multi<10, 1, 32>(ops, nops, st);
        case 12: return run_fwd2d_multi<12, 1, 32>(ops, nops, st);
        case 18: return run_fwd2d_multi<18, 1, 16>(ops, nops, st);   // (9,2): 12.8 -> 15.3 us on an 18x18 layer
        case 14: return run_fwd2d_multi<14, 1, 32>(ops, nops, st);
        case 20: {
            // one lane per line on grids of a few rounds of workgroups (18x18 layer: 13.7 us against
            // 18.1), lane pairs on large tiled grids (224x224 in 16x16 tiles: 547 us against 616)
            long planes = 0;
            for (int o = 0; o < nops; ++o) planes += ops[o].planes;
            if (planes > 32768) return run_fwd2d_multi<10, 2, 16>(ops, nops, st);
            return run_fwd2d_multi<20, 1, 16>(ops, nops, st);
        }
        case 24: return run_fwd2d_multi<24, 1, 16>(ops, nops, st);
        case 28: return run_fwd2d_multi<28, 1, 16>(ops, nops, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_fft2d_r2c_small(const float *in, float *out, long planes, int h_in, int w_in, int N,
                                  bool conv, LaunchCtx st, const PlaneView *view) {
    switch (N) {
        case 10: return run_fwd2d<10, 1, 32>(in, out, planes, h_in, w_in, conv, st, view);
        case 12: return run_fwd2d<12, 1, 32>(in, out, planes, h_in, w_in, conv, st, view);
        case 18: return run_fwd2d<18, 1, 16>(in, out, planes, h_in, w_in, conv, st, view);
        case 14: return run_fwd2d<14, 1, 32>(in, out, planes, h_in, w_in, conv, st, view);
        // (the natural layout, whose batches are large, keeps lane pairs: 4.9 against 4.7 TB/s at 28)
        case 20:
            if (!conv || planes > 32768) return run_fwd2d<10, 2, 16>(in, out, planes, h_in, w_in, conv, st, view);
            return run_fwd2d<20, 1, 16>(in, out, planes, h_in, w_in, conv, st, view);
        case 24:
            if (!conv) return run_fwd2d<12, 2, 16>(in, out, planes, h_in, w_in, conv, st, view);
            return run_fwd2d<24, 1, 16>(in, out, planes, h_in, w_in, conv, st, view);
        case 28:
            if (!conv) return run_fwd2d<14, 2, 16>(in, out, planes, h_in, w_in, conv, st, view);
            return run_fwd2d<28, 1, 16>(in, out, planes, h_in, w_in, conv, st, view);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_fft2d_c2r_small(const float *in, float *out, long planes, int N, int h_out, int w_out,
                                  bool conv, float scale, bool accumulate, LaunchCtx st, const PlaneView *view) {
    switch (N) {
        case 10: return run_inv2d<5, 2, 32>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        case 12: return run_inv2d<3, 4, 32>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        case 18: return run_inv2d<9, 2, 16>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        case 14: return run_inv2d<7, 2, 32>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        case 20:
            if (!conv) return run_inv2d<10, 2, 16>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
            return run_inv2d<20, 1, 16>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        case 24: return run_inv2d<6, 4, 16>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        case 28:
            // one lane per line when nearly all rows are kept (27x27 input gradients: 13.5 us
            // against 14.1), four otherwise (5x5 weight gradients: 6.6 against 8.0)
            if (conv && 4 * (h_out + (view ? view->oy : 0)) > 3 * 28)
                return run_inv2d<28, 1, 16>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
            return run_inv2d<7, 4, 16>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        default: return hipErrorInvalidValue;
    }
}

// One inverse kernel for both products of the backward pass.  Where the separate launches would
// pick different kernels by the rows kept (28), the choice for the larger operand serves both.
// Measured on 64-channel layers, fft_conv_backward in us, two launches -> one: basis 18 44.6 -> 40.4,
// 20 49.8 -> 44.4, 24 59.5 -> 55.4; the 27x27 layer at basis 28: inverse transforms 13.7 + 6.9 -> 16.0 with
// (28,1) for both (23.7 with (7,4), the weight gradients' own choice); 13x13 with 384 channels at
// basis 14: 21.5 + 26.1 -> 42.0.
hipError_t launch_fft2d_c2r_pair_small(const InvOperand *ops, int N, LaunchCtx st) {
    switch (N) {
        case 10: return run_inv2d_pair<5, 2, 32>(ops, st);
        case 12: return run_inv2d_pair<3, 4, 32>(ops, st);
        case 14: return run_inv2d_pair<7, 2, 32>(ops, st);
        case 18: return run_inv2d_pair<9, 2, 16>(ops, st);
        case 20: return run_inv2d_pair<20, 1, 16>(ops, st);
        case 24: return run_inv2d_pair<6, 4, 16>(ops, st);
        case 28: return run_inv2d_pair<28, 1, 16>(ops, st);
        default: return hipErrorNotSupported;
    }
}

}  // namespace fc
