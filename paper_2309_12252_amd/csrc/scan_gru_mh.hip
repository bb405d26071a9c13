// Multi-head GRU with strides (Sec. 4.4, App. B.4): the fused Newton step and the dual scan of the small-n kernel
// with the launch's sequences being the strided recurrences of the heads (scan_valu_kernel<..., MH = true>: per-head
// parameters, positions s * H * n scalars apart, per-recurrence length).  Heads fold into the batch dimension of the
// scan; nothing else of the kernel changes.
#include "scan_valu_kernel.h"

namespace deer {

namespace {

template <typename S, int N, int L>
hipError_t launch_mh_nl(const ScanParams& p, const GruFeed& gf, hipStream_t s) {
    dim3 grid((unsigned)((long long)p.B * p.tiles));
    if (p.reverse)
        hipLaunchKernelGGL((scan_valu_kernel<S, N, L, 8, true, 8, false, true>), grid, dim3(64 * 8), 0, s, p, gf);
    else
        hipLaunchKernelGGL((scan_valu_kernel<S, N, L, 8, false, 8, false, true>), grid, dim3(64 * 8), 0, s, p, gf);
    return hipGetLastError();
}

template <typename S, int N>
hipError_t launch_mh_n(const ScanParams& p, const GruFeed& gf, hipStream_t s) {
    switch (p.L) {
        case 1: return launch_mh_nl<S, N, 1>(p, gf, s);
        case 2: return launch_mh_nl<S, N, 2>(p, gf, s);
        case 4: return launch_mh_nl<S, N, 4>(p, gf, s);
        default: return hipErrorInvalidValue;
    }
}

template <typename S>
hipError_t launch_mh_s(int n, const ScanParams& p, const GruFeed& gf, hipStream_t s) {
    switch (n) {
        case 2: return launch_mh_n<S, 2>(p, gf, s);
        case 4: return launch_mh_n<S, 4>(p, gf, s);
        case 8: return launch_mh_n<S, 8>(p, gf, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool scan_gru_mh_supported(int dtype, int n, int d, int L) {
    (void)dtype;
    return (n == 2 || n == 4 || n == 8) && d >= 1 && d <= 8 && (L == 1 || L == 2 || L == 4);
}

hipError_t launch_scan_gru_mh(int dtype, int n, const ScanParams& p, const void* theta, const void* x, int d, hipStream_t s) {
    if (!scan_gru_mh_supported(dtype, n, d, p.L) || p.W != 8 || p.delta || !p.yold || p.mh_H < 1 || p.mh_K < 1 || !p.mh_table)
        return hipErrorInvalidValue;
    if (p.reverse && !p.bv) return hipErrorInvalidValue;
    const GruFeed gf{theta, x, d};
    return dtype == 0 ? launch_mh_s<float>(n, p, gf, s) : launch_mh_s<double>(n, p, gf, s);
}

}  // namespace deer
