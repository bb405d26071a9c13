// Inverse linear operator for small state sizes (n <= 8): single-pass blocked associative scan
// over affine pairs (A | b) with the operator of Sec. 3.3 eq. 10, on the vector ALUs.
//
// Structure of one tile (256 threads, L scan positions per lane, 256*L positions per tile):
//   1. every lane composes its L consecutive pairs serially into one pair held in registers;
//   2. the 64 lane pairs of a wavefront are scanned with a log-step (Kogge-Stone) scan using
//      cross-lane shuffles; each lane keeps the exclusive prefix of its wavefront;
//   3. the four wavefront totals meet in LDS and give the tile total;
//   4. tiles of one sequence are chained through HBM by decoupled look-back: a tile publishes its
//      total (flag AGGREGATE), inspects up to 64 predecessors at once, and folds their totals
//      forward from the nearest predecessor whose inclusive carry is already known (flag
//      INCLUSIVE).  Only the vector part of the carry is needed, so the fold is matrix-vector
//      work.  Tiles take their index from an atomic ticket, so every predecessor of a running
//      tile has started, which makes the waiting deadlock free; waits are bounded anyway.
//   5. every lane turns the carry into its own starting state and walks its L positions again
//      (y <- A y + b), writing y and reducing max|y - y_previous_iterate| for the convergence test.
#include "deer_common.h"

namespace deer {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

// scan position k of one sequence -> registers.  Reverse mode: vector index T-1-k, matrix = transpose
// of the one stored at index T-k, none (zero) for k = 0.
template <typename S, int N, bool REV>
__device__ __forceinline__ void load_elem(const S* __restrict__ Ab, const S* __restrict__ bb, int T, int k,
                                          S* Am, S* bvv) {
    if constexpr (!REV) {
        vload<S, N * N>(Am, Ab + (long long)k * (N * N));
        vload<S, N>(bvv, bb + (long long)k * N);
    } else {
        vload<S, N>(bvv, bb + (long long)(T - 1 - k) * N);
        if (k == 0) {
#pragma unroll
            for (int q = 0; q < N * N; ++q) Am[q] = S(0);
        } else {
            S tmp[N * N];
            vload<S, N * N>(tmp, Ab + (long long)(T - k) * (N * N));
#pragma unroll
            for (int r = 0; r < N; ++r)
#pragma unroll
                for (int c = 0; c < N; ++c) Am[r * N + c] = tmp[c * N + r];
        }
    }
}

// (M | v) <- (Am | bvv) after (M | v):  M <- Am M,  v <- Am v + bvv   (column by column, in place)
template <typename S, int N>
__device__ __forceinline__ void apply_left(const S* Am, const S* bvv, S* M, S* v) {
#pragma unroll
    for (int c = 0; c < N; ++c) {
        S col[N];
#pragma unroll
        for (int r = 0; r < N; ++r) {
            S s = S(0);
#pragma unroll
            for (int k = 0; k < N; ++k) s += Am[r * N + k] * M[k * N + c];
            col[r] = s;
        }
#pragma unroll
        for (int r = 0; r < N; ++r) M[r * N + c] = col[r];
    }
    S nv[N];
#pragma unroll
    for (int r = 0; r < N; ++r) {
        S s = bvv[r];
#pragma unroll
        for (int k = 0; k < N; ++k) s += Am[r * N + k] * v[k];
        nv[r] = s;
    }
#pragma unroll
    for (int r = 0; r < N; ++r) v[r] = nv[r];
}

// (M | v) <- (M | v) after (Mo | vo):  v <- M vo + v,  M <- M Mo   (row by row, in place)
template <typename S, int N>
__device__ __forceinline__ void apply_right(S* M, S* v, const S* Mo, const S* vo) {
#pragma unroll
    for (int r = 0; r < N; ++r) {
        S row[N];
        S s = v[r];
#pragma unroll
        for (int k = 0; k < N; ++k) s += M[r * N + k] * vo[k];
#pragma unroll
        for (int c = 0; c < N; ++c) {
            S a = S(0);
#pragma unroll
            for (int k = 0; k < N; ++k) a += M[r * N + k] * Mo[k * N + c];
            row[c] = a;
        }
        v[r] = s;
#pragma unroll
        for (int c = 0; c < N; ++c) M[r * N + c] = row[c];
    }
}

// y <- M y + v
template <typename S, int N>
__device__ __forceinline__ void matvec(const S* M, const S* v, S* y) {
    S ny[N];
#pragma unroll
    for (int r = 0; r < N; ++r) {
        S s = v[r];
#pragma unroll
        for (int k = 0; k < N; ++k) s += M[r * N + k] * y[k];
        ny[r] = s;
    }
#pragma unroll
    for (int r = 0; r < N; ++r) y[r] = ny[r];
}

template <typename S, int N, bool REV>
__global__ __launch_bounds__(kThreads) void scan_valu_kernel(ScanParams p) {
    __shared__ unsigned s_ticket;
    __shared__ S sAggM[kWaves][N * N];
    __shared__ S sAggv[kWaves][N];
    __shared__ S sP[2][N * N];
    __shared__ S sPv[2][N];
    __shared__ S sCarry[N];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;

    if (tid == 0) s_ticket = atomicAdd(p.ticket, 1u);
    __syncthreads();
    const unsigned tk = s_ticket;
    const int b = (int)(tk % (unsigned)p.B);
    const int t = (int)(tk / (unsigned)p.B);
    if (t >= p.tiles) return;

    const S* __restrict__ Ab = reinterpret_cast<const S*>(p.A) + (long long)b * p.strideA;
    const S* __restrict__ bb = reinterpret_cast<const S*>(p.bv) + (long long)b * p.strideb;
    S* __restrict__ ob = reinterpret_cast<S*>(p.out) + (long long)b * p.strideOut;
    const S* __restrict__ oldb =
        p.yold ? reinterpret_cast<const S*>(p.yold) + (long long)b * p.strideOld : nullptr;

    const int L = p.L;
    const long long e0 = (long long)t * (kThreads * L) + (long long)tid * L;

    // ---- 1. serial composition of this lane's positions ----
    S M[N * N], v[N];
#pragma unroll
    for (int q = 0; q < N * N; ++q) M[q] = ((q / N) == (q % N)) ? S(1) : S(0);
#pragma unroll
    for (int q = 0; q < N; ++q) v[q] = S(0);
    for (int i = 0; i < L; ++i) {
        const long long e = e0 + i;
        if (e < p.T) {
            S Am[N * N], bvv[N];
            load_elem<S, N, REV>(Ab, bb, p.T, (int)e, Am, bvv);
            apply_left<S, N>(Am, bvv, M, v);
        }
    }

    // ---- 2. inclusive scan over the lanes of the wavefront ----
#pragma unroll 1
    for (int dlt = 1; dlt < 64; dlt <<= 1) {
        S Mo[N * N], vo[N];
#pragma unroll
        for (int q = 0; q < N * N; ++q) Mo[q] = __shfl_up(M[q], dlt);
#pragma unroll
        for (int q = 0; q < N; ++q) vo[q] = __shfl_up(v[q], dlt);
        if (lane >= dlt) apply_right<S, N>(M, v, Mo, vo);
    }
    if (lane == 63) {
#pragma unroll
        for (int q = 0; q < N * N; ++q) sAggM[wave][q] = M[q];
#pragma unroll
        for (int q = 0; q < N; ++q) sAggv[wave][q] = v[q];
    }
    // exclusive prefix of the lane within its wavefront
#pragma unroll
    for (int q = 0; q < N * N; ++q) {
        S u = __shfl_up(M[q], 1);
        M[q] = lane == 0 ? (((q / N) == (q % N)) ? S(1) : S(0)) : u;
    }
#pragma unroll
    for (int q = 0; q < N; ++q) {
        S u = __shfl_up(v[q], 1);
        v[q] = lane == 0 ? S(0) : u;
    }
    __syncthreads();

    // ---- 3. tile total = wavefront totals composed in order ----
    int cur = 0;
    if (tid < N * N) sP[0][tid] = sAggM[0][tid];
    if (tid < N) sPv[0][tid] = sAggv[0][tid];
    __syncthreads();
    for (int w = 1; w < kWaves; ++w) {
        if (tid < N * N) {
            const int r = tid / N, c = tid % N;
            S s = S(0);
#pragma unroll
            for (int k = 0; k < N; ++k) s += sAggM[w][r * N + k] * sP[cur][k * N + c];
            sP[cur ^ 1][tid] = s;
        }
        if (tid < N) {
            S s = sAggv[w][tid];
#pragma unroll
            for (int k = 0; k < N; ++k) s += sAggM[w][tid * N + k] * sPv[cur][k];
            sPv[cur ^ 1][tid] = s;
        }
        __syncthreads();
        cur ^= 1;
    }

    // ---- 4. publish the total, look back for the carry, publish the inclusive carry ----
    const long long slot = (long long)b * p.tiles + t;
    if (wave == 0) {
        S* gM = reinterpret_cast<S*>(p.aggM) + slot * (N * N);
        S* gv = reinterpret_cast<S*>(p.aggv) + slot * N;
        S* gi = reinterpret_cast<S*>(p.incl) + slot * N;
        const unsigned tag = p.epoch << 2;
        if (t > 0) {
            for (int q = lane; q < N * N; q += 64) gM[q] = sP[cur][q];
            if (lane < N) gv[lane] = sPv[cur][lane];
            __threadfence();
            if (lane == 0) flag_store(&p.flags[slot], tag | TILE_AGGREGATE);
        }

        // lane j inspects predecessor t-1-j; index -1 is the given initial state
        const int idx = t - 1 - lane;
        int k = -1;
        unsigned spins = 0;
        while (true) {
            unsigned st;
            if (idx >= 0) {
                const unsigned f = flag_load(&p.flags[(long long)b * p.tiles + idx]);
                st = ((f >> 2) == p.epoch) ? (f & 3u) : TILE_INVALID;
            } else {
                st = (idx == -1) ? TILE_INCLUSIVE : 3u;
            }
            const unsigned long long incl_mask = __ballot(st == TILE_INCLUSIVE);
            const unsigned long long wait_mask = __ballot(st == TILE_INVALID);
            if (incl_mask != 0ull) {
                const int first = __ffsll((long long)incl_mask) - 1;
                const unsigned long long below = (first == 0) ? 0ull : ((1ull << first) - 1ull);
                if ((wait_mask & below) == 0ull) { k = first; break; }
            }
            if (++spins > kSpinLimit) break;
            __builtin_amdgcn_s_sleep(2);
        }

        S y[N];
#pragma unroll
        for (int q = 0; q < N; ++q) y[q] = S(0);
        if (k < 0) {
            if (lane == 0) atomicOr(p.status, 1u);
        } else {
            S Mp[N * N], vp[N];
#pragma unroll
            for (int q = 0; q < N * N; ++q) Mp[q] = S(0);
#pragma unroll
            for (int q = 0; q < N; ++q) vp[q] = S(0);
            if (lane < k) {
                const long long ps = (long long)b * p.tiles + idx;
                const S* pM = reinterpret_cast<const S*>(p.aggM) + ps * (N * N);
                const S* pv = reinterpret_cast<const S*>(p.aggv) + ps * N;
#pragma unroll
                for (int q = 0; q < N * N; ++q) Mp[q] = coherent_load(pM + q);
#pragma unroll
                for (int q = 0; q < N; ++q) vp[q] = coherent_load(pv + q);
            } else if (lane == k) {
                if (idx >= 0) {
                    const S* pi = reinterpret_cast<const S*>(p.incl) + ((long long)b * p.tiles + idx) * N;
#pragma unroll
                    for (int q = 0; q < N; ++q) y[q] = coherent_load(pi + q);
                } else if (p.y0) {
                    const S* y0b = reinterpret_cast<const S*>(p.y0) + (long long)b * N;
#pragma unroll
                    for (int q = 0; q < N; ++q) y[q] = y0b[q];
                }
            }
            // fold forward: lane j turns the carry before tile t-1-j into the carry after it
            for (int j = k - 1; j >= 0; --j) {
                S yin[N];
#pragma unroll
                for (int q = 0; q < N; ++q) yin[q] = __shfl(y[q], j + 1);
                if (lane == j) {
#pragma unroll
                    for (int q = 0; q < N; ++q) y[q] = yin[q];
                    matvec<S, N>(Mp, vp, y);
                }
            }
        }
        S c[N];
#pragma unroll
        for (int q = 0; q < N; ++q) c[q] = __shfl(y[q], 0);
        if (lane < N) {
            S s = sPv[cur][lane];
#pragma unroll
            for (int q = 0; q < N; ++q) s += sP[cur][lane * N + q] * c[q];
            gi[lane] = s;
        }
        __threadfence();
        if (lane == 0) {
            flag_store(&p.flags[slot], tag | TILE_INCLUSIVE);
#pragma unroll
            for (int q = 0; q < N; ++q) sCarry[q] = c[q];
        }
    }
    __syncthreads();

    // ---- 5. starting state of this lane, then the second walk ----
    S y[N];
#pragma unroll
    for (int q = 0; q < N; ++q) y[q] = sCarry[q];
    for (int w = 0; w < wave; ++w) matvec<S, N>(sAggM[w], sAggv[w], y);
    matvec<S, N>(M, v, y);

    S emax = S(0);
    for (int i = 0; i < L; ++i) {
        const long long e = e0 + i;
        if (e < p.T) {
            S Am[N * N], bvv[N];
            load_elem<S, N, REV>(Ab, bb, p.T, (int)e, Am, bvv);
            matvec<S, N>(Am, bvv, y);
            const long long oi = (REV ? (long long)(p.T - 1 - e) : e) * N;
            if (oldb) {
                S yo[N], wv[N];
                vload<S, N>(yo, oldb + oi);
#pragma unroll
                for (int q = 0; q < N; ++q) {
                    wv[q] = p.delta ? yo[q] + y[q] : y[q];
                    const S dq = abs_or_inf<S>(p.delta ? y[q] : y[q] - yo[q]);
                    emax = dq > emax ? dq : emax;
                }
                vstore<S, N>(ob + oi, wv);
            } else {
                vstore<S, N>(ob + oi, y);
            }
        }
    }
    if (p.err) {
        emax = wave_max<S>(emax);
        if (lane == 0) err_atomic_max(p.err, emax);
    }
}

template <typename S, int N>
hipError_t launch_n(const ScanParams& p, hipStream_t s) {
    dim3 grid((unsigned)((long long)p.B * p.tiles));
    if (p.reverse)
        hipLaunchKernelGGL((scan_valu_kernel<S, N, true>), grid, dim3(kThreads), 0, s, p);
    else
        hipLaunchKernelGGL((scan_valu_kernel<S, N, false>), grid, dim3(kThreads), 0, s, p);
    return hipGetLastError();
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

int scan_valu_tile(int n, int L) { (void)n; return kThreads * L; }

hipError_t launch_scan_valu(int dtype, int n, const ScanParams& p, hipStream_t s) {
    return dtype == 0 ? launch_s<float>(n, p, s) : launch_s<double>(n, p, s);
}

}  // namespace deer
