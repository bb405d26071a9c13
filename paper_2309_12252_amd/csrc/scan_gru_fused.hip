// Newton step of the GRU cell for small state sizes (n <= 8) in one launch: the single-pass scan
// kernel with the cell's Jacobian and right-hand side (Sec. 3.1 eq. 3 and 5) computed in registers where
// the plain scan loads its pairs.  The n*n matrices are never written to or read from HBM; a launch
// reads the previous iterate and the inputs and writes the next iterate (Sec. 3.2, Sec. 3.4 eq. 11).
#include "scan_valu_kernel.h"

namespace deer {

namespace {

template <typename S, int N, int L, int W, int DP>
hipError_t launch_fused_nlwd(const ScanParams& p, const GruFeed& gf, hipStream_t s) {
    dim3 grid((unsigned)((long long)p.B * p.tiles));
    hipLaunchKernelGGL((scan_valu_kernel<S, N, L, W, false, DP>), grid, dim3(64 * W), 0, s, p, gf);
    return hipGetLastError();
}

template <typename S, int N, int L, int W>
hipError_t launch_fused_nlw(const ScanParams& p, const GruFeed& gf, hipStream_t s) {
    if (gf.d <= 4) return launch_fused_nlwd<S, N, L, W, 4>(p, gf, s);
    if (gf.d <= 8) return launch_fused_nlwd<S, N, L, W, 8>(p, gf, s);
    return hipErrorInvalidValue;
}

template <typename S, int N, int L>
hipError_t launch_fused_nl(const ScanParams& p, const GruFeed& gf, hipStream_t s) {
    if (p.W == 8) return launch_fused_nlw<S, N, L, 8>(p, gf, s);
    if constexpr (N >= 4) {   // wavefront 0 scans one wavefront total per group: 64 / n >= W
        if (p.W == 4) return launch_fused_nlw<S, N, L, 4>(p, gf, s);
    }
    return hipErrorInvalidValue;
}

template <typename S, int N>
hipError_t launch_fused_n(const ScanParams& p, const GruFeed& gf, hipStream_t s) {
    switch (p.L) {
        case 1: return launch_fused_nl<S, N, 1>(p, gf, s);
        case 2: return launch_fused_nl<S, N, 2>(p, gf, s);
        case 4: return launch_fused_nl<S, N, 4>(p, gf, s);
        case 8: return launch_fused_nl<S, N, 8>(p, gf, s);
        case 10: if constexpr (sizeof(S) == 4 && N == 8) return launch_fused_nl<S, N, 10>(p, gf, s); else return hipErrorInvalidValue;
        case 12: if constexpr (sizeof(S) == 4 && N == 8) return launch_fused_nl<S, N, 12>(p, gf, s); else return hipErrorInvalidValue;
        case 16: if constexpr (sizeof(S) == 4) return launch_fused_nl<S, N, 16>(p, gf, s); else return hipErrorInvalidValue;
        default: return hipErrorInvalidValue;
    }
}

template <typename S>
hipError_t launch_fused_s(int n, const ScanParams& p, const GruFeed& gf, hipStream_t s) {
    switch (n) {
        case 1: return launch_fused_n<S, 1>(p, gf, s);
        case 2: return launch_fused_n<S, 2>(p, gf, s);
        case 4: return launch_fused_n<S, 4>(p, gf, s);
        case 8: return launch_fused_n<S, 8>(p, gf, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

// mirrors the instantiations reachable through launch_fused_s
bool scan_gru_fused_supported(int dtype, int n, int d, int L, int W) {
    if (!(n == 1 || n == 2 || n == 4 || n == 8) || d < 1 || d > 8) return false;
    if (!(W == 8 || (W == 4 && n >= 4))) return false;
    if (L == 1 || L == 2 || L == 4 || L == 8) return true;
    if (dtype != 0) return false;
    return L == 16 || (n == 8 && (L == 10 || L == 12));
}

hipError_t launch_scan_gru_fused(int dtype, int n, const ScanParams& p, const void* theta, const void* x, int d,
                                 hipStream_t s) {
    if (p.reverse || p.delta || !p.yold) return hipErrorInvalidValue;
    const GruFeed gf{theta, x, d};
    return dtype == 0 ? launch_fused_s<float>(n, p, gf, s) : launch_fused_s<double>(n, p, gf, s);
}

}  // namespace deer
