// Launchers of the batched FFT kernels (fft_kernels_impl.hpp): the power-of-two sizes of
// Section 5 of the fbfft paper (8 ... 128 in 2-D, 8 ... 256 in 1-D) are instantiated here; sizes
// with an odd factor go to the fft_kernels_mixed*.hip files.
#include "fft_kernels_impl.hpp"

#include <cstdlib>
#include <mutex>
#include <unordered_map>

namespace fc {

hipError_t allow_big_lds(const void *fn, size_t bytes) {
    if (bytes <= 64 * 1024) return hipSuccess;
    static std::mutex mu;
    static std::unordered_map<const void *, size_t> granted;
    std::lock_guard<std::mutex> lock(mu);
    size_t &have = granted[fn];
    if (have >= bytes) return hipSuccess;
    const size_t ask = 160 * 1024;   // the whole LDS of a gfx950 compute unit
    const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)ask);
    if (e == hipSuccess) have = ask;
    return e;
}

// Planes per workgroup (= tile of the frequency layout) by size class: 64 at 8, 32 up to 16, 16
// up to 28, 4 up to 64, 1 above.  Basis 32 takes 8: with four lanes per line and eight planes
// its transforms are 5 .. 25 % faster than any 16-plane variant (more, smaller workgroups), which
// outweighs the contraction's loss from runs of 8 planes instead of 16 (0 .. 15 %) on every layer
// measured (27x27 step 146.4 -> 143.5 us, 224x224 in 32x32 tiles 1480 -> 1420, 55x55 780 -> 745);
// at 20 .. 28 the one-lane-per-line 16-plane kernels stay ahead (basis 28: 125 us against 127 .. 132).
int fft2d_tile_log2(int N) {
    switch (N) {
        case 8: return 6;
        case 10: case 12: case 14: case 16: return 5;
        case 18: case 20: case 24: case 28: return 4;
        case 32: return 3;
        case 36: case 40: case 48: case 56: case 64: return 2;
        case 80: case 96: case 112: case 128: return 0;
        default: return -1;
    }
}

int fft2d_layout_bins(int N) {
    const int bins = N * (N / 2 + 1), unit = fft2d_tile_log2(N) == 2 ? 32 : 8;
    return (bins + unit - 1) / unit * unit;
}

hipError_t launch_fft2d_r2c_multi(const FwdOperand *ops, int nops, int N, LaunchCtx st) {
    if (nops < 1 || nops > 3) return hipErrorInvalidValue;
    for (int o = 0; o < nops; ++o)
        if (ops[o].planes <= 0) return hipErrorInvalidValue;
    switch (N) {
        case 8: return run_fwd2d_multi<8, 1, 64>(ops, nops, st);
        case 16: return run_fwd2d_multi<16, 1, 32>(ops, nops, st);
        case 32: return run_fwd2d_multi<8, 4, 8>(ops, nops, st);
        case 64: return run_fwd2d_multi<32, 2, 4>(ops, nops, st);
        case 128: return run_fwd2d_multi<16, 8, 1>(ops, nops, st);
        default: return launch_fft2d_r2c_multi_mixed(ops, nops, N, st);
    }
}

hipError_t launch_fft2d_r2c(const float *in, float *out, long planes, int h_in, int w_in, int N,
                            bool conv, LaunchCtx st, const PlaneView *view) {
    if (planes <= 0) return hipSuccess;
    if (view && !conv) return hipErrorInvalidValue;
    if (!conv) {
        const hipError_t e = launch_fft2d_r2c_natural(in, out, planes, h_in, w_in, N, st);
        if (e != hipErrorNotSupported) return e;
    }
    switch (N) {
        // sizes 2 and 4: stand-alone transforms only (Section 5 covers 2 ... 256; no convolution basis)
        case 2: return conv ? hipErrorInvalidValue : run_fwd2d<2, 1, 64>(in, out, planes, h_in, w_in, conv, st, view);
        case 4: return conv ? hipErrorInvalidValue : run_fwd2d<4, 1, 64>(in, out, planes, h_in, w_in, conv, st, view);
        case 8: return run_fwd2d<8, 1, 64>(in, out, planes, h_in, w_in, conv, st, view);
        case 16: return run_fwd2d<16, 1, 32>(in, out, planes, h_in, w_in, conv, st, view);   // (8,2): 12 % slower
        case 32: return run_fwd2d<8, 4, 8>(in, out, planes, h_in, w_in, conv, st, view);   // 16 planes: (16,2) 5 % slower, (32,1) 8 %
        case 64:
            // Lane pairs ((64,1): 25 % slower), except for inputs of more than 52 rows: their four
            // planes of row-transformed data (1 KB per row) leave room for two workgroups per compute
            // unit only, and twice the waves on four lanes per line then hide more latency
            // (4096 planes 64x64: 45.7 -> 41.2 us; but 34x34: 25.8 -> 31.5, 31x31: 74 -> 84)
            if (conv && h_in > 52) return run_fwd2d<16, 4, 4>(in, out, planes, h_in, w_in, conv, st, view);
            return run_fwd2d<32, 2, 4>(in, out, planes, h_in, w_in, conv, st, view);
        case 128: return run_fwd2d<16, 8, 1>(in, out, planes, h_in, w_in, conv, st, view);
        default: return launch_fft2d_r2c_mixed(in, out, planes, h_in, w_in, N, conv, st, view);
    }
}

hipError_t launch_fft2d_c2r(const float *in, float *out, long planes, int N, int h_out, int w_out,
                            bool conv, float scale, bool accumulate, LaunchCtx st, const PlaneView *view) {
    if (planes <= 0) return hipSuccess;
    if (view && (!conv || view->oy + h_out > N || view->ox + w_out > N)) return hipErrorInvalidValue;
    const int rows = h_out + (view ? view->oy : 0);   // rows of the transform that are computed
    if (!conv) {
        const hipError_t e = launch_fft2d_c2r_natural(in, out, planes, N, h_out, w_out, scale, accumulate, st);
        if (e != hipErrorNotSupported) return e;
    }
    switch (N) {
        case 2: return conv ? hipErrorInvalidValue : run_inv2d<2, 1, 64>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        case 4: return conv ? hipErrorInvalidValue : run_inv2d<4, 1, 64>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        case 8: return run_inv2d<8, 1, 64>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        case 16:
            // lane pairs when at most half the rows are kept (3x3 weight gradients: 29 us against
            // 36 on the 13x13 layer), one lane per line otherwise (19 us against 23)
            if (conv && 2 * rows <= 16) return run_inv2d<8, 2, 32>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
            return run_inv2d<16, 1, 32>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        case 32:
            // (with 16 planes per workgroup: (32,1) 15.0 us on the 27x27 layer, (16,2) 16.1; this: 14.3)
            return run_inv2d<8, 4, 8>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        // the inverse gains from more lanes per line (fewer registers, shorter serial chains):
        // eight per line since their cross-lane twiddles come from the LDS table (31x31 crops of the
        // 64-basis layer: 85 us with (16,4), 74 with (8,8); 34x34 outputs 29.4 -> 24.8; before the table
        // (16,4) was ahead whenever at most three quarters of the rows were kept)
        case 64: return run_inv2d<8, 8, 4>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        case 128: return run_inv2d<16, 8, 1>(in, out, planes, h_out, w_out, conv, scale, accumulate, st, view);
        default: return launch_fft2d_c2r_mixed(in, out, planes, N, h_out, w_out, conv, scale, accumulate, st, view);
    }
}

hipError_t launch_fft2d_c2r_pair(const InvOperand *ops, int N, LaunchCtx st) {
    for (int o = 0; o < 2; ++o) {
        const int rows = ops[o].h_out + (ops[o].view ? ops[o].view->oy : 0), cols = ops[o].w_out + (ops[o].view ? ops[o].view->ox : 0);
        if (ops[o].planes <= 0 || rows > N || cols > N) return hipErrorNotSupported;
    }
    switch (N) {
        case 16: return run_inv2d_pair<16, 1, 32>(ops, st);   // 22.1 + 29.7 -> 52.5 us at 384 channels: the launch gap
        case 32: return run_inv2d_pair<8, 4, 8>(ops, st);
        default: return launch_fft2d_c2r_pair_mixed(ops, N, st);
    }
}

// Lanes per line of the 1-D kernels: more lanes with shorter register FFTs measured faster at
// every size (fewer registers per lane, more loads in flight), e.g. n = 64: (8,8) 5.3 TB/s against
// (32,2) 4.8; n = 256: (32,8) 4.2 against (64,4) 2.7; (2,4) at n = 8 lost.  Signals per workgroup
// (third argument): smaller workgroups overlap their load, transform and store phases better;
// same process, TB/s R2C / C2R: n = 16 512 -> 256 signals 5.49 / 5.65 -> 5.96 / 5.80; n = 32 (8,4) 256 ->
// (4,8) 128 (eight lanes since the cross-lane twiddles come from LDS) 5.32 / 5.47 -> 5.86 / 5.84; n = 64
// 128 -> 32 5.37 / 5.42 -> 5.61 / 5.56; n = 128 128 -> 64 4.57..5.01 / 4.59..4.88 -> 5.14..5.18 / 5.06..5.17;
// n = 256 keeps 64 (32: 4.04 against 4.08).
hipError_t launch_fft1d_r2c(const float *in, float *out, long B, int n_in, int n, LaunchCtx st) {
    if (B <= 0) return hipSuccess;
    switch (n) {
        case 2: return run_fwd1d<2, 1, 1024>(in, out, B, n_in, st);
        case 4: return run_fwd1d<4, 1, 1024>(in, out, B, n_in, st);
        case 8: return run_fwd1d<4, 2, 512>(in, out, B, n_in, st);
        case 16: return run_fwd1d<4, 4, 256>(in, out, B, n_in, st);
        case 32: return run_fwd1d<4, 8, 128>(in, out, B, n_in, st);
        case 64: return run_fwd1d<8, 8, 32>(in, out, B, n_in, st);
        case 128: return run_fwd1d<16, 8, 64>(in, out, B, n_in, st);
        case 256: return run_fwd1d<32, 8, 64>(in, out, B, n_in, st);
        default: return launch_fft1d_r2c_mixed(in, out, B, n_in, n, st);
    }
}

hipError_t launch_fft1d_c2r(const float *in, float *out, long B, int n, int n_out, LaunchCtx st) {
    if (B <= 0) return hipSuccess;
    switch (n) {
        case 2: return run_inv1d<2, 1, 1024>(in, out, B, n_out, st);
        case 4: return run_inv1d<4, 1, 1024>(in, out, B, n_out, st);
        case 8: return run_inv1d<4, 2, 512>(in, out, B, n_out, st);
        case 16: return run_inv1d<4, 4, 256>(in, out, B, n_out, st);
        case 32: return run_inv1d<4, 8, 128>(in, out, B, n_out, st);
        case 64: return run_inv1d<8, 8, 32>(in, out, B, n_out, st);
        case 128: return run_inv1d<16, 8, 64>(in, out, B, n_out, st);
        case 256: return run_inv1d<32, 8, 64>(in, out, B, n_out, st);
        default: return launch_fft1d_c2r_mixed(in, out, B, n, n_out, st);
    }
}

}  // namespace fc
