// 1-D transforms of the sizes with an odd factor 3, 5, 7 or 9: 10 ... 224.  Eight lanes per line
// from 40 on (and at 24), as for the powers of two (more lanes with shorter register transforms
// measured faster at every size there).  Signals per workgroup from a sweep of the base choice
// against a half, a quarter and another lane split, same process (e.g. n = 96: 128 -> 64 signals
// 5.21 / 5.11 -> 5.55 / 5.35 TB/s; n = 24: (6,4) 256 -> (3,8) 128 5.60 / 5.59 -> 5.73 / 5.83; the sizes from
// 160 on keep 64: halving it costs 5..10 %).
#include "fft_kernels_impl.hpp"

namespace fc {

hipError_t launch_fft1d_r2c_mixed(const float *in, float *out, long B, int n_in, int n, LaunchCtx st) {
    switch (n) {
        case 10: return run_fwd1d<5, 2, 256>(in, out, B, n_in, st);
        case 12: return run_fwd1d<3, 4, 128>(in, out, B, n_in, st);
        case 18: return run_fwd1d<9, 2, 256>(in, out, B, n_in, st);
        case 36: return run_fwd1d<9, 4, 128>(in, out, B, n_in, st);
        case 14: return run_fwd1d<7, 2, 256>(in, out, B, n_in, st);
        case 20: return run_fwd1d<5, 4, 128>(in, out, B, n_in, st);
        case 24: return run_fwd1d<3, 8, 128>(in, out, B, n_in, st);
        case 28: return run_fwd1d<7, 4, 64>(in, out, B, n_in, st);
        case 40: return run_fwd1d<5, 8, 32>(in, out, B, n_in, st);
        case 48: return run_fwd1d<6, 8, 64>(in, out, B, n_in, st);
        case 56: return run_fwd1d<7, 8, 64>(in, out, B, n_in, st);
        case 80: return run_fwd1d<10, 8, 32>(in, out, B, n_in, st);
        case 96: return run_fwd1d<12, 8, 64>(in, out, B, n_in, st);
        case 112: return run_fwd1d<14, 8, 64>(in, out, B, n_in, st);
        case 160: return run_fwd1d<20, 8, 64>(in, out, B, n_in, st);
        case 192: return run_fwd1d<24, 8, 64>(in, out, B, n_in, st);
        case 224: return run_fwd1d<28, 8, 64>(in, out, B, n_in, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_fft1d_c2r_mixed(const float *in, float *out, long B, int n, int n_out, LaunchCtx st) {
    switch (n) {
        case 10: return run_inv1d<5, 2, 256>(in, out, B, n_out, st);
        case 12: return run_inv1d<3, 4, 128>(in, out, B, n_out, st);
        case 18: return run_inv1d<9, 2, 256>(in, out, B, n_out, st);
        case 36: return run_inv1d<9, 4, 128>(in, out, B, n_out, st);
        case 14: return run_inv1d<7, 2, 256>(in, out, B, n_out, st);
        case 20: return run_inv1d<5, 4, 128>(in, out, B, n_out, st);
        case 24: return run_inv1d<3, 8, 128>(in, out, B, n_out, st);
        case 28: return run_inv1d<7, 4, 64>(in, out, B, n_out, st);
        case 40: return run_inv1d<5, 8, 32>(in, out, B, n_out, st);
        case 48: return run_inv1d<6, 8, 64>(in, out, B, n_out, st);
        case 56: return run_inv1d<7, 8, 64>(in, out, B, n_out, st);
        case 80: return run_inv1d<10, 8, 32>(in, out, B, n_out, st);
        case 96: return run_inv1d<12, 8, 64>(in, out, B, n_out, st);
        case 112: return run_inv1d<14, 8, 64>(in, out, B, n_out, st);
        case 160: return run_inv1d<20, 8, 64>(in, out, B, n_out, st);
        case 192: return run_inv1d<24, 8, 64>(in, out, B, n_out, st);
        case 224: return run_inv1d<28, 8, 64>(in, out, B, n_out, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace fc
