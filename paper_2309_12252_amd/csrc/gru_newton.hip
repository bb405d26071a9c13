// All Newton iterations of a small GRU problem in one launch (n <= 8, d <= 8).
//
// Every tile of every sequence gets a workgroup and all of them are resident at the same time (the
// host checks the grid against the device's capacity before choosing this kernel).  A lane keeps the
// iterate at its L positions and the input projections W x + b in registers for the whole solve; an
// iteration computes the pairs (J | f - J h) of Sec. 3.1 eq. 3 and 5 from the registers, runs the tile scan
// with look-back exactly like the one-step kernel (tags carry the iteration's own epoch), and takes
// the new iterate from the second walk.  The state entering a group in the new iterate is the h of that
// group's first position in the next iteration, so iterations exchange nothing but the look-back words.
// The convergence test of Sec. 3.2 / App. B.1 needs the maximum over all tiles: per iteration every
// workgroup publishes its maximum in a slot of its own and collects everybody's (bounded waits).  This
// is also a grid barrier, which keeps an iteration's published words from being overwritten while in use.
// Compared with one launch per iteration this removes the dispatch gap between dependent launches
// (about 13 us on this part), the reloads of x and of the iterate, and all but the last store.
#include "scan_valu_kernel.h"

namespace deer {

namespace {

template <typename S, int N, int L, int W, int DP>
__global__ __launch_bounds__(64 * W) void gru_newton_kernel(NewtonParams q) {
    constexpr int NG = 64 / N;
    constexpr int TILE = W * NG * L;
    __shared__ TileShared<S, N, W> sh;
    __shared__ int s_stop;
    __shared__ S s_red[W];

    const ScanParams& p = q.scan;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int group = lane / N;
    const int i = lane % N;
    // static tile assignment: nothing waits for a workgroup that is not running
    const int b = (int)(blockIdx.x % (unsigned)p.B);
    const int t = (int)(blockIdx.x / (unsigned)p.B);
    const long long T = p.T;
    const long long e0 = (long long)t * TILE + (long long)(wave * NG + group) * L;
    const bool full = (long long)(t + 1) * TILE <= T;

    // Constant over the solve and parked in LDS, so that they occupy registers only while the pairs are
    // formed: the hidden-to-hidden rows (a small table shared by all groups) and this lane's input
    // projections W x + b.
    __shared__ S sU[N][3 * N + 1];         // row i: U_r | U_z | U_c (natural column order), b_hc
    __shared__ S sP[3 * L][64 * W];        // [3 l + gate][thread]
    {
        GruRow<S, N, DP> w0;
        load_gru_row<S, N, DP>(q.feed, i, w0);
        const S* __restrict__ xb = reinterpret_cast<const S*>(q.feed.x) + (long long)b * T * q.feed.d;
        S pr[L], pq[L], pc[L];
        if (full) gru_project<S, N, L, DP, true>(w0, xb, q.feed.d, T, e0, pr, pq, pc);
        else gru_project<S, N, L, DP, false>(w0, xb, q.feed.d, T, e0, pr, pq, pc);
#pragma unroll
        for (int l = 0; l < L; ++l) {
            sP[3 * l][tid] = pr[l];
            sP[3 * l + 1][tid] = pq[l];
            sP[3 * l + 2][tid] = pc[l];
        }
        if (tid < N) {
            const S* __restrict__ th = reinterpret_cast<const S*>(q.feed.theta);
            const S* __restrict__ U = th + 3 * N * q.feed.d;
            for (int c = 0; c < N; ++c) {
                sU[tid][c] = U[tid * N + c];
                sU[tid][N + c] = U[(N + tid) * N + c];
                sU[tid][2 * N + c] = U[(2 * N + tid) * N + c];
            }
            sU[tid][3 * N] = U[3 * N * N + 3 * N + tid];
        }
    }
    __syncthreads();

    // iterate 0: the guess (zeros without one) at this group's positions and in front of them
    const S* __restrict__ gb = p.yold ? reinterpret_cast<const S*>(p.yold) + (long long)b * p.strideOld : nullptr;
    S yv[L], h0;
#pragma unroll
    for (int l = 0; l < L; ++l) {
        const long long e = (e0 + l < T) ? e0 + l : T - 1;
        yv[l] = gb ? gb[e * N + i] : S(0);
    }
    {
        const long long ef = e0 < T ? e0 : T;
        const S* y0p = reinterpret_cast<const S*>(p.y0);
        const S a = gb ? gb[(ef > 0 ? ef - 1 : 0) * N + i] : S(0);
        const S c0 = y0p ? y0p[(long long)b * N + i] : S(0);
        h0 = ef > 0 ? a : c0;
    }

    if (tid == 0) sh.failed = 0;   // (the first barrier inside tile_carry orders this before any use)
    const S tol = (S)q.tol;
    // After an error of e the next one is about e^2 (Newton): below this threshold the coming iteration is
    // expected to be the last one, and the work for the one after it is not started ahead of the test.
    const S spec_thr = (S)sqrt(q.tol);

    S Ar[L][N], be[L], Pex[N], pex = S(0), Mt[N], vt = S(0);
#pragma unroll
    for (int c = 0; c < N; ++c) Mt[c] = S(0);
    // First half of an iteration, all inside the workgroup: the pairs from the current iterate (yv, h0), their
    // composition and the scans inside the tile.  Nothing is published.
    auto local_half = [&]() {
        // weights and projections come back from LDS; the indices pass through an opaque statement so that
        // the loads stay inside the loop (hoisted, the values would hold registers for the whole solve)
        int ri = i, ti = tid;
        asm volatile("" : "+v"(ri), "+v"(ti));
        GruRow<S, N, DP> w;
#pragma unroll
        for (int c = 0; c < N; ++c) {
            const int col = swz_col<N>(c, i);
            w.Ur[c] = sU[ri][col];
            w.Uz[c] = sU[ri][N + col];
            w.Uc[c] = sU[ri][2 * N + col];
            w.E[c] = (col == i) ? S(1) : S(0);
        }
        w.bh = sU[ri][3 * N];
        S pr[L], pq[L], pc[L];
#pragma unroll
        for (int l = 0; l < L; ++l) {
            pr[l] = sP[3 * l][ti];
            pq[l] = sP[3 * l + 1][ti];
            pc[l] = sP[3 * l + 2][ti];
        }
        if (full) gru_rows<S, N, L, DP, true>(w, pr, pq, pc, h0, yv, T, e0, Ar, be);
        else gru_rows<S, N, L, DP, false>(w, pr, pq, pc, h0, yv, T, e0, Ar, be);
        tile_local<S, N, L, W>(p, sh, Ar, be, (long long)b * p.tiles, t, Pex, pex, Mt, vt);
    };

    const unsigned G = gridDim.x + q.extra_workgroups;   // (extra: test hook, see NewtonParams)
    // Second half of the convergence test of iteration kk: collect the maxima of all workgroups (bounded
    // wait), record the result for the host, and say whether the solve stops here.
    S elast = S(INFINITY);
    bool gave_up = false;   // a wait of this workgroup ran out: the solve is abandoned, the caller solves again
    auto collect = [&](int kk, S own) -> bool {
        unsigned long long* bank = q.barrier + (size_t)(kk & 1) * G * TaggedWords<S>::per_scalar;
        const unsigned tagK = ((p.epoch + (unsigned)kk) << 2) | TILE_INCLUSIVE;
        S gm = S(0);
        bool ok = true;
        for (unsigned j = tid; j < G && G > 1u && ok; j += 64 * W) {   // a single workgroup has nobody to wait for
            S v = S(0);
            unsigned spins = 0;
            while (!TaggedWords<S>::get(bank, j, tagK, v)) {
                // give up after the bound, or as soon as another workgroup has given up; the first thread whose
                // wait runs out raises the status word at once, so nobody else waits out a bound of its own
                if (++spins > q.spin_limit ||
                    ((spins & 1023u) == 0u && __hip_atomic_load(p.status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u)) {
                    ok = false;
                    atomicOr(p.status, 2u);
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
            }
            gm = v > gm ? v : gm;
        }
        if (G == 1u) gm = own;   // (every wavefront's own maximum; combined across wavefronts below)
        gm = wave_max<S>(gm);
        const bool wave_ok = __ballot(!ok) == 0ull;
        __syncthreads();   // s_red is reused
        if (lane == 0) s_red[wave] = gm;
        if (tid == 0) s_stop = 0;
        __syncthreads();
        if (lane == 0 && !wave_ok) s_stop = 1;
        S e = s_red[0];
#pragma unroll
        for (int v = 1; v < W; ++v) e = s_red[v] > e ? s_red[v] : e;
        __syncthreads();
        const bool stop = s_stop != 0 || !(e > tol) || e >= S(INFINITY);
        gave_up = gave_up || s_stop != 0;
        if (blockIdx.x == 0 && tid == 0) {   // the record for the host (host-visible memory)
            const S rec = s_stop != 0 ? S(INFINITY) : e;
            if constexpr (sizeof(S) == 4) *reinterpret_cast<float*>(q.err + kk) = rec;
            else *reinterpret_cast<double*>(q.err + kk) = rec;
        }
        elast = e;
        return stop;
    };

    // Iteration k = local half, look-back, second walk, test.  The test is split: the workgroup publishes
    // its maximum right after the walk, and collects everybody's either at once or -- when another iteration
    // is expected -- only after the local half of that next iteration, which needs nothing from the other
    // workgroups, publishes nothing and leaves the new iterate alone (so it is simply dropped if the test
    // says stop).  All conditions are the same in every workgroup.
    int k = 0;            // iterations whose walk is done
    bool pending = false; // the test of iteration k-1 has not been collected yet
    S own = S(0);
    for (;;) {
        DEER_STAMP(p, (long long)b * p.tiles + t, 0, tid == 0);
        local_half();
        if (pending) {
            const bool stop = collect(k - 1, own);
            if (stop || k >= q.max_iter) break;
        }
        // The bases of the published-word regions pass through an opaque statement every iteration: the
        // look-back's many addresses are then recomputed per iteration instead of being hoisted out of the
        // loop, where they would occupy registers for the whole solve.
        ScanParams pk = p;
        asm volatile("" : "+v"(pk.aggW), "+v"(pk.inclW));
        tile_lookback<S, N, W>(pk, sh, (long long)b * p.tiles, t, p.epoch + (unsigned)k, Mt, vt,
                               p.y0 ? reinterpret_cast<const S*>(p.y0) + (long long)b * N : nullptr);
        S y = tile_start_state<S, N, W>(sh, Pex, pex, wave, i);
        h0 = y;   // the new iterate in front of this group's first position
        S emax = S(0);
#pragma unroll
        for (int l = 0; l < L; ++l) {
            y = group_matvec<S, N>(Ar[l], be[l], y);
            if (full || e0 + l < T) {
                const S dq = abs_or_inf<S>(y - yv[l]);
                emax = dq > emax ? dq : emax;
            }
            yv[l] = y;
        }
        DEER_STAMP(p, (long long)b * p.tiles + t, 6, tid == 0);
        // A tile whose look-back gave up has no valid iterate: it reports an infinite change, which stops
        // every workgroup at the test and tells the host to look at the status word.
        if (sh.failed) emax = S(INFINITY);
        // First half of the test: every workgroup publishes its own maximum as a tagged word in its own
        // slot (plain stores to distinct addresses, no atomic read-modify-write on a shared word).  The slots
        // alternate between two banks by iteration parity: nobody can be two iterations ahead of a workgroup
        // that has not collected the previous test.  The exchange is also the grid barrier that keeps an
        // iteration's look-back words from being overwritten while in use.
        emax = wave_max<S>(emax);
        own = emax;
        if (lane == 0) s_red[wave] = emax;
        __syncthreads();
        if (tid == 0) {
            S m = s_red[0];
#pragma unroll
            for (int v = 1; v < W; ++v) m = s_red[v] > m ? s_red[v] : m;
            TaggedWords<S>::put(q.barrier + (size_t)(k & 1) * G * TaggedWords<S>::per_scalar, blockIdx.x, m,
                                ((p.epoch + (unsigned)k) << 2) | TILE_INCLUSIVE);
        }
        ++k;
#ifdef DEER_SCAN_TIMING
        if (p.timing && tid == 0) p.timing[((long long)b * p.tiles + t) * 16 + 7] = wall_clock64();
#endif
        // After an error of e the next one is about e^2 (Newton): with the last known error above the
        // threshold one more iteration is expected and its local half runs before the collection.
        pending = (k < q.max_iter) && (elast > spec_thr) && G > 1u;
        if (!pending) {
            const bool stop = collect(k - 1, own);
            if (stop || k >= q.max_iter) break;
        }
    }

    // An abandoned solve leaves the output alone: it may be the caller's initial guess (d_y_guess == d_y), which
    // the launch-by-launch solve that follows starts from.
    S* __restrict__ ob = reinterpret_cast<S*>(p.out) + (long long)b * p.strideOut;
    if (!gave_up && !sh.failed) {
#pragma unroll
        for (int l = 0; l < L; ++l)
            if (full || e0 + l < T) __builtin_nontemporal_store(yv[l], ob + (e0 + l) * N + i);
    }
    if (blockIdx.x == 0 && tid == 0) *q.result = k;
}

template <typename S, int N, int L, int DP>
struct Variant {
    static constexpr int W = 8;
    static hipError_t launch(const NewtonParams& q, hipStream_t s) {
        dim3 grid((unsigned)((long long)q.scan.B * q.scan.tiles));
        hipLaunchKernelGGL((gru_newton_kernel<S, N, L, W, DP>), grid, dim3(64 * W), 0, s, q);
        return hipGetLastError();
    }
    static int capacity() {
        int dev = 0, per_cu = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, gru_newton_kernel<S, N, L, W, DP>, 64 * W, 0) != hipSuccess)
            return 0;
        return per_cu * prop.multiProcessorCount;
    }
};

// op = 0: launch, op = 1: capacity.  Returns hipError_t for a launch, the capacity otherwise (0: no such variant).
template <typename S, int N, int L>
int dispatch_nl(int op, int d, const NewtonParams* q, hipStream_t s) {
    if (d <= 4) return op == 0 ? (int)Variant<S, N, L, 4>::launch(*q, s) : Variant<S, N, L, 4>::capacity();
    return op == 0 ? (int)Variant<S, N, L, 8>::launch(*q, s) : Variant<S, N, L, 8>::capacity();
}

template <typename S, int N>
int dispatch_n(int op, int L, int d, const NewtonParams* q, hipStream_t s) {
    switch (L) {
        case 1: return dispatch_nl<S, N, 1>(op, d, q, s);
        case 2: return dispatch_nl<S, N, 2>(op, d, q, s);
        case 4: return dispatch_nl<S, N, 4>(op, d, q, s);
        case 8: return dispatch_nl<S, N, 8>(op, d, q, s);
        case 10: if constexpr (sizeof(S) == 4 && N == 8) return dispatch_nl<S, N, 10>(op, d, q, s); else break;
        case 12: if constexpr (sizeof(S) == 4 && N == 8) return dispatch_nl<S, N, 12>(op, d, q, s); else break;
        case 16: if constexpr (sizeof(S) == 4) return dispatch_nl<S, N, 16>(op, d, q, s); else break;
        default: break;
    }
    return op == 0 ? (int)hipErrorInvalidValue : 0;
}

template <typename S>
int dispatch_s(int op, int n, int L, int d, const NewtonParams* q, hipStream_t s) {
    switch (n) {
        case 1: return dispatch_n<S, 1>(op, L, d, q, s);
        case 2: return dispatch_n<S, 2>(op, L, d, q, s);
        case 4: return dispatch_n<S, 4>(op, L, d, q, s);
        case 8: return dispatch_n<S, 8>(op, L, d, q, s);
        default: return op == 0 ? (int)hipErrorInvalidValue : 0;
    }
}

}  // namespace

int gru_newton_capacity(int dtype, int n, int d, int L) {
    if (d < 1 || d > 8) return 0;
    return dtype == 0 ? dispatch_s<float>(1, n, L, d, nullptr, nullptr) : dispatch_s<double>(1, n, L, d, nullptr, nullptr);
}

hipError_t launch_gru_newton(int dtype, int n, const NewtonParams& q, hipStream_t s) {
    if (q.scan.W != 8 || q.scan.reverse || q.scan.delta || q.max_iter < 1) return hipErrorInvalidValue;
    return (hipError_t)(dtype == 0 ? dispatch_s<float>(0, n, q.scan.L, q.feed.d, &q, s)
                                   : dispatch_s<double>(0, n, q.scan.L, q.feed.d, &q, s));
}

}  // namespace deer
