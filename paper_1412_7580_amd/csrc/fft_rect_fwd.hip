// Forward transforms on rectangular bases (see fft_rect_impl.hpp).
#include "fft_rect_impl.hpp"

namespace fc {

bool fft2d_rect_supported(int nr, int nc) {
    return rect_dispatch(nr, nc, [](auto, auto) {});
}
int fft2d_rect_tile_log2(int nr, int nc) { return rect_tile_log2(nr, nc); }
int fft2d_rect_layout_bins(int nr, int nc) { return rect_layout_bins(nr, nc); }

hipError_t launch_fft2d_r2c_rect(const FwdOperand *ops, int nops, int nr, int nc, LaunchCtx st) {
    if (nops < 1 || nops > 2) return hipErrorInvalidValue;
    for (int o = 0; o < nops; ++o) {
        if (ops[o].planes < 0 || ops[o].view) return hipErrorInvalidValue;
        if (ops[o].h_in < 1 || ops[o].w_in < 1 || ops[o].h_in > nr || ops[o].w_in > nc) return hipErrorInvalidValue;
    }
    hipError_t e = hipErrorInvalidValue;
    rect_dispatch(nr, nc, [&](auto R, auto C) {
        typedef RectSide<decltype(R)::value> SR;
        typedef RectSide<decltype(C)::value> SC;
        e = run_fwd_rect<SR::L, SR::G, SC::L, SC::G>(ops, nops, st);
    });
    return e;
}

}  // namespace fc
