// 2-D transforms of the sizes 12, 14, 20, 24 and 28 (one odd factor 3, 5 or 7 in the
// per-lane part of the line, see fft_core.hpp), the small half of the bases Section 3.2 of the
// fbfft paper reaches through cuFFT.
#include "fft_kernels_impl.hpp"

#include <cstdlib>

namespace fc {

#define FC_ALT(name) (getenv(name) != nullptr)

hipError_t launch_fft2d_r2c_multi_small(const FwdOperand *ops, int nops, int N, LaunchCtx st) {
    switch (N) {
        case 12: return FC_ALT("FFTCONV_ALT12") ? run_fwd2d_multi<3, 4, 32>(ops, nops, st) : run_fwd2d_multi<6, 2, 32>(ops, nops, st);
        case 14: return run_fwd2d_multi<7, 2, 32>(ops, nops, st);
        case 20: return FC_ALT("FFTCONV_ALT20") ? run_fwd2d_multi<10, 2, 16>(ops, nops, st) : run_fwd2d_multi<5, 4, 16>(ops, nops, st);
        case 24: return FC_ALT("FFTCONV_ALT24") ? run_fwd2d_multi<12, 2, 16>(ops, nops, st) : run_fwd2d_multi<6, 4, 16>(ops, nops, st);
        case 28: return FC_ALT("FFTCONV_ALT28") ? run_fwd2d_multi<14, 2, 16>(ops, nops, st) : run_fwd2d_multi<7, 4, 16>(ops, nops, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_fft2d_r2c_small(const float *in, float *out, long planes, int h_in, int w_in, int N,
                                  bool conv, LaunchCtx st, const PlaneView *view) {
    switch (N) {
        case 12: return FC_ALT("FFTCONV_ALT12") ? run_fwd2d<3, 4, 32>(in, out, planes, h_in, w_in, conv, st, view) : run_fwd2d<6, 2, 32>(in, out, planes, h_in, w_in, conv, st, view);
        case 14: return run_fwd2d<7, 2, 32>(in, out, planes, h_in, w_in, conv, st, view);
        case 20: return FC_ALT("FFTCONV_ALT20") ? run_fwd2d<10, 2, 16>(in, out, planes, h_in, w_in, conv, st, view) : run_fwd2d<5, 4, 16>(in, out, planes, h_in, w_in, conv, st, view);
        case 24: return FC_ALT("FFTCONV_ALT24") ? run_fwd2d<12, 2, 16>(in, out, planes, h_in, w_in, conv, st, view) : run_fwd2d<6, 4, 16>(in, out, planes, h_in, w_in, conv, st, view);
        case 28: return FC_ALT("FFTCONV_ALT28") ? run_fwd2d<14, 2, 16>(in, out, planes, h_in, w_in, conv, st, view) : run_fwd2d<7, 4, 16>(in, out, planes, h_in, w_in, conv, st, view);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_fft2d_c2r_small(const float *in, float *out, long planes, int N, int h_out, int w_out,
                                  bool conv, float scale, bool accumulate, LaunchCtx st, const PlaneView *view) {
    switch (N) {
        case 12: return FC_ALT("FFTCONV_IALT12") ? run_inv2d<3, 4, 32>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view) : run_inv2d<6, 2, 32>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        case 14: return run_inv2d<7, 2, 32>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        case 20: return FC_ALT("FFTCONV_IALT20") ? run_inv2d<10, 2, 16>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view) : run_inv2d<5, 4, 16>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        case 24: return FC_ALT("FFTCONV_IALT24") ? run_inv2d<12, 2, 16>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view) : run_inv2d<6, 4, 16>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        case 28: return FC_ALT("FFTCONV_IALT28") ? run_inv2d<14, 2, 16>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view) : run_inv2d<7, 4, 16>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace fc
