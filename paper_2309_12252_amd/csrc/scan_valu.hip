// Inverse linear operator for small state sizes (n <= 8): single-pass blocked associative scan
// over affine pairs (A | b) with the operator of Sec. 3.3 eq. 10, on the vector ALUs with DPP
// cross-lane operands.
//
// Data layout in registers: a pair is spread over the n consecutive lanes of a "group"; lane i of
// the group holds row i of the matrix (n registers) and entry i of the vector.  A wavefront holds
// 64/n groups.  The product of two matrices needs, in lane i, row i of the left factor (own
// registers) and every row of the right factor (the other lanes of the same group); those come in
// through DPP operands (quad_perm broadcasts inside a quad; for n = 8 one half-row mirror first makes
// every lane see the other quad of its group next to its own), so a product costs n*n
// multiply-adds per lane and no LDS traffic.  Global loads are coalesced: a group reads the n*n
// contiguous scalars of its matrix.
//
// Structure of one tile (WAVES wavefronts, L scan positions per group, WAVES * 64/n * L per tile):
//   1. every group loads its L consecutive pairs into registers and composes them serially;
//   2. the groups of a wavefront are scanned with a log-step scan (shuffles by whole groups);
//   3. wavefront totals meet in LDS; wavefront 0 scans them the same way, which gives the tile total
//      and the prefix in front of every wavefront;
//   4. tiles of one sequence are chained through HBM by decoupled look-back: a tile publishes its
//      total (state AGGREGATE), inspects up to 64 predecessors at once, and folds their totals
//      forward from the nearest predecessor whose inclusive carry is known (state INCLUSIVE); the
//      totals are fetched by all groups in parallel, one predecessor per group, and applied in
//      order.  Only the vector part of the carry is needed, so the fold is matrix-vector work.
//      Published data travels as self-validating tagged words (no fences, no cache maintenance).
//      Tiles take their index from an atomic ticket, so every predecessor of a running tile has
//      started, which makes the waiting deadlock free; waits are bounded anyway;
//   5. every group turns the carry into its own starting state and walks its register-resident
//      pairs again (y <- A y + b), writing y and reducing max|y - y_previous_iterate| for the
//      convergence test.  The matrices are read from HBM exactly once.
#include "scan_valu_kernel.h"

namespace deer {

namespace {

template <typename S, int N, int L, int W>
hipError_t launch_nlw(const ScanParams& p, hipStream_t s) {
    dim3 grid((unsigned)((long long)p.B * p.tiles));
    if (p.add_identity) {
        // matrices stored as A - I: reverse scans of state sizes the ODE form uses
        if constexpr (N >= 2) {
            if (!p.reverse) return hipErrorInvalidValue;
            hipLaunchKernelGGL((scan_valu_kernel<S, N, L, W, true, 0, true>), grid, dim3(64 * W), 0, s, p, GruFeed{});
        } else {
            return hipErrorInvalidValue;
        }
    } else if (p.reverse)
        hipLaunchKernelGGL((scan_valu_kernel<S, N, L, W, true, 0>), grid, dim3(64 * W), 0, s, p, GruFeed{});
    else
        hipLaunchKernelGGL((scan_valu_kernel<S, N, L, W, false, 0>), grid, dim3(64 * W), 0, s, p, GruFeed{});
    return hipGetLastError();
}

template <typename S, int N, int L>
hipError_t launch_nl(const ScanParams& p, hipStream_t s) {
    return launch_nlw<S, N, L, 8>(p, s);
}

template <typename S, int N>
hipError_t launch_n(const ScanParams& p, hipStream_t s) {
    switch (p.L) {
        case 1: return launch_nl<S, N, 1>(p, s);
        case 2: return launch_nl<S, N, 2>(p, s);
        case 4: return launch_nl<S, N, 4>(p, s);
        case 8: return launch_nl<S, N, 8>(p, s);
        case 10: if constexpr (sizeof(S) == 4) return launch_nl<S, N, 10>(p, s); else return hipErrorInvalidValue;
        case 12: if constexpr (sizeof(S) == 4) return launch_nl<S, N, 12>(p, s); else return hipErrorInvalidValue;
        case 16: if constexpr (sizeof(S) == 4) return launch_nl<S, N, 16>(p, s); else return hipErrorInvalidValue;
        case 24: if constexpr (sizeof(S) == 4 && N == 4) return launch_nl<S, N, 24>(p, s); else return hipErrorInvalidValue;
        case 32: if constexpr (sizeof(S) == 4 && N == 2) return launch_nl<S, N, 32>(p, s); else return hipErrorInvalidValue;
        default: return hipErrorInvalidValue;
    }
}

template <typename S>
hipError_t launch_s(int n, const ScanParams& p, hipStream_t s) {
    switch (n) {
        case 1: return launch_n<S, 1>(p, s);
        case 2: return launch_n<S, 2>(p, s);
        case 4: return launch_n<S, 4>(p, s);
        case 8: return launch_n<S, 8>(p, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

int scan_valu_tile(int n, int L, int W) { return W * (64 / n) * L; }

hipError_t launch_scan_valu(int dtype, int n, const ScanParams& p, hipStream_t s) {
    if (p.W != 8) return hipErrorInvalidValue;
    return dtype == 0 ? launch_s<float>(n, p, s) : launch_s<double>(n, p, s);
}

}  // namespace deer
