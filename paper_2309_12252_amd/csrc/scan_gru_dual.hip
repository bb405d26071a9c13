// Dual (transposed, time-reversed) scan of the backward derivative (Sec. 3.1.1 eq. 7) for the GRU cell with small
// state sizes (n <= 8): the single-pass scan kernel with the transposed Jacobians computed in registers from the
// trajectory, so the backward pass neither writes nor reads the n*n matrices.
#include "scan_valu_kernel.h"

namespace deer {

namespace {

template <typename S, int N, int L>
hipError_t launch_dual_nl(const ScanParams& p, const GruFeed& gf, hipStream_t s) {
    constexpr int W = 8;
    dim3 grid((unsigned)((long long)p.B * p.tiles));
    if (gf.d <= 4) hipLaunchKernelGGL((scan_valu_kernel<S, N, L, W, true, 4>), grid, dim3(64 * W), 0, s, p, gf);
    else hipLaunchKernelGGL((scan_valu_kernel<S, N, L, W, true, 8>), grid, dim3(64 * W), 0, s, p, gf);
    return hipGetLastError();
}

template <typename S, int N>
hipError_t launch_dual_n(const ScanParams& p, const GruFeed& gf, hipStream_t s) {
    switch (p.L) {
        case 1: return launch_dual_nl<S, N, 1>(p, gf, s);
        case 2: return launch_dual_nl<S, N, 2>(p, gf, s);
        case 4: return launch_dual_nl<S, N, 4>(p, gf, s);
        case 8: return launch_dual_nl<S, N, 8>(p, gf, s);
        case 10: if constexpr (sizeof(S) == 4 && N == 8) return launch_dual_nl<S, N, 10>(p, gf, s); else return hipErrorInvalidValue;
        case 12: if constexpr (sizeof(S) == 4 && N == 8) return launch_dual_nl<S, N, 12>(p, gf, s); else return hipErrorInvalidValue;
        case 16: if constexpr (sizeof(S) == 4) return launch_dual_nl<S, N, 16>(p, gf, s); else return hipErrorInvalidValue;
        default: return hipErrorInvalidValue;
    }
}

template <typename S>
hipError_t launch_dual_s(int n, const ScanParams& p, const GruFeed& gf, hipStream_t s) {
    switch (n) {
        case 1: return launch_dual_n<S, 1>(p, gf, s);
        case 2: return launch_dual_n<S, 2>(p, gf, s);
        case 4: return launch_dual_n<S, 4>(p, gf, s);
        case 8: return launch_dual_n<S, 8>(p, gf, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

// the tile shapes of the fused forward step with eight wavefronts
bool scan_gru_dual_supported(int dtype, int n, int d, int L, int W) {
    return W == 8 && scan_gru_fused_supported(dtype, n, d, L, W);
}

hipError_t launch_scan_gru_dual(int dtype, int n, const ScanParams& p, const void* theta, const void* x, int d,
                                hipStream_t s) {
    if (!p.reverse || p.delta || !p.yold || !scan_gru_dual_supported(dtype, n, d, p.L, p.W)) return hipErrorInvalidValue;
    const GruFeed gf{theta, x, d};
    return dtype == 0 ? launch_dual_s<float>(n, p, gf, s) : launch_dual_s<double>(n, p, gf, s);
}

}  // namespace deer
