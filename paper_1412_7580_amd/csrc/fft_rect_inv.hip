// Inverse transforms on rectangular bases (see fft_rect_impl.hpp).
#include "fft_rect_impl.hpp"

namespace fc {

hipError_t launch_fft2d_c2r_rect(const float *in, float *out, long planes, int nr, int nc, int h_out, int w_out,
                                 float scale, bool accumulate, LaunchCtx st) {
    if (planes <= 0) return hipSuccess;
    if (h_out < 1 || w_out < 1 || h_out > nr || w_out > nc) return hipErrorInvalidValue;
    hipError_t e = hipErrorInvalidValue;
    rect_dispatch(nr, nc, [&](auto R, auto C) {
        typedef RectSide<decltype(R)::value> SR;
        typedef RectSide<decltype(C)::value> SC;
        e = run_inv_rect<SR::L, SR::G, SC::L, SC::G>(in, out, planes, h_out, w_out, scale, accumulate, st);
    });
    return e;
}

hipError_t launch_fft2d_c2r_rect_pair(const InvOperand *ops, int nr, int nc, LaunchCtx st) {
    for (int o = 0; o < 2; ++o) {
        if (ops[o].planes <= 0 || ops[o].view) return hipErrorNotSupported;
        if (ops[o].h_out < 1 || ops[o].w_out < 1 || ops[o].h_out > nr || ops[o].w_out > nc) return hipErrorInvalidValue;
    }
    hipError_t e = hipErrorNotSupported;
    rect_dispatch(nr, nc, [&](auto R, auto C) {
        typedef RectSide<decltype(R)::value> SR;
        typedef RectSide<decltype(C)::value> SC;
        e = run_inv_rect_pair<SR::L, SR::G, SC::L, SC::G>(ops, st);
    });
    return e;
}

}  // namespace fc
