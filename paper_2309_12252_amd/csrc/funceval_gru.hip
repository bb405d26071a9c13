// GRU cell kernels.
//   gru_funceval_kernel: for every sequence position, f(h, x), the Jacobian J = df/dh and the
//     right-hand side of the linear recurrence, rhs = f - J h (the paper carries G = -J and
//     z = f + G h, Sec. 3.1 eq. 3 and 5; the sign is folded so that y_i = J_i y_{i-1} + rhs_i).
//     h is the previous iterate shifted by one position, y0 at the first position (Sec. 3.2).
//   gru_vjp_kernel: vector-Jacobian product of f with the scanned cotangent lam at every position
//     (Sec. 3.1.1 eq. 7, outer bracket): dL/dx per position, dL/dy0, and per-wavefront partial sums
//     of dL/dtheta that gru_vjp_reduce_kernel adds up in a fixed order (run-to-run identical).
//
// Cell (gates r, z, candidate c; reset applied after the hidden projection):
//   r = sig(W_r x + b_r + U_r h)   z = sig(W_z x + b_z + U_z h)
//   q = U_c h + b_hc               c = tanh(W_c x + b_c + r q)        f = (1 - z) c + z h
//   J = diag(z) + diag((h - c) z (1 - z)) U_z + diag((1 - z)(1 - c^2)) [diag(r) U_c + diag(q r (1 - r)) U_r]
//
// Work split: one thread per (position, state row i).  Row i of J needs only row i of the gates
// and of U, so threads never talk to each other in the forward kernel; the n threads of a position
// sit in consecutive lanes and write n*n consecutive scalars of J (fully coalesced).  U rows live in
// registers, W (runtime input size) in LDS with an odd row stride.
#include "deer_common.h"

namespace deer {

namespace {

constexpr int kThreads = 256;
constexpr int kMaxD = 32;   // largest input size (the kernels are instantiated for unroll widths 16 and 32)

// fp32: hardware exp2 and reciprocal (absolute error below 3e-7), as in the fused step
__device__ __forceinline__ float sigmoid_(float a) { return feed_sigmoid(a); }
__device__ __forceinline__ double sigmoid_(double a) { return 1.0 / (1.0 + exp(-a)); }
__device__ __forceinline__ float tanh_(float a) { return feed_tanh(a); }
__device__ __forceinline__ double tanh_(double a) { return tanh(a); }

template <typename S, int N>
struct RowWeights {
    S Ur[N], Uz[N], Uc[N];
    S br, bz, bc, bh;
};

template <typename S, int N>
__device__ __forceinline__ void load_row_weights(const S* __restrict__ theta, int d, int i, RowWeights<S, N>& w,
                                                 S* sW, int ds, int tid) {
    for (int q = tid; q < 3 * N * d; q += kThreads) sW[(q / d) * ds + (q % d)] = theta[q];
    const S* U = theta + 3 * N * d;
    const S* bias = U + 3 * N * N;
    vload<S, N>(w.Ur, U + (long long)(i)*N);
    vload<S, N>(w.Uz, U + (long long)(N + i) * N);
    vload<S, N>(w.Uc, U + (long long)(2 * N + i) * N);
    w.br = bias[i];
    w.bz = bias[N + i];
    w.bc = bias[2 * N + i];
    w.bh = bias[3 * N + i];
}

template <typename S, int N>
struct Gates {
    S r, z, q, c, hi;
};

// gates of row i at (h, x); DX: the input width the x loops are unrolled for (d <= DX)
template <typename S, int N, int DX>
__global__ __launch_bounds__(kThreads) void gru_funceval_kernel(GruParams p) {
    if (gate_closed<S>(p.gate)) return;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    S* sW = reinterpret_cast<S*>(smem_raw);
    const int tid = threadIdx.x;
    const int d = p.d, ds = d | 1;
    constexpr int SPB = kThreads / N;   // positions per block pass
    const int i = tid % N;
    const int sg = tid / N;
    const S* __restrict__ theta = reinterpret_cast<const S*>(p.theta);
    const S* __restrict__ x = reinterpret_cast<const S*>(p.x);
    const S* __restrict__ y0 = reinterpret_cast<const S*>(p.y0);
    const S* __restrict__ y = reinterpret_cast<const S*>(p.y);
    S* __restrict__ J = reinterpret_cast<S*>(p.J);
    S* __restrict__ rhs = reinterpret_cast<S*>(p.rhs);

    RowWeights<S, N> w;
    load_row_weights<S, N>(theta, d, i, w, sW, ds, tid);
    __syncthreads();

    const long long total = (long long)p.B * p.T;
    const long long stride = (long long)gridDim.x * SPB;
    // Software pipeline: the operands of the next position are requested before the current one is
    // computed, so the loop does not expose a memory round trip per position.
    S hn[N], hin = S(0), xn[DX];
    auto fetch = [&](long long s) {
        const long long bi = s / p.T;
        const int ti = (int)(s - bi * p.T);
        const S* hp = (ti == 0) ? (y0 + bi * N) : (y + (s - 1) * N);
        vload<S, N>(hn, hp);
        hin = hp[i];
#pragma unroll
        for (int k = 0; k < DX; ++k) xn[k] = (k < d) ? x[s * d + k] : S(0);
    };
    long long s = (long long)blockIdx.x * SPB + sg;
    if (s < total) fetch(s);
    for (; s < total; s += stride) {
        S h[N], xv[DX];
#pragma unroll
        for (int j = 0; j < N; ++j) h[j] = hn[j];
#pragma unroll
        for (int k = 0; k < DX; ++k) xv[k] = xn[k];
        const S hi = hin;
        if (s + stride < total) fetch(s + stride);
        S ar = w.br, az = w.bz, ac = w.bc, q = w.bh;
#pragma unroll
        for (int k = 0; k < DX; ++k) {
            if (k < d) {
                ar += sW[(i)*ds + k] * xv[k];
                az += sW[(N + i) * ds + k] * xv[k];
                ac += sW[(2 * N + i) * ds + k] * xv[k];
            }
        }
#pragma unroll
        for (int j = 0; j < N; ++j) {
            ar += w.Ur[j] * h[j];
            az += w.Uz[j] * h[j];
            q += w.Uc[j] * h[j];
        }
        Gates<S, N> g;
        g.r = sigmoid_(ar);
        g.z = sigmoid_(az);
        g.q = q;
        g.c = tanh_(ac + g.r * q);
        const S f = (S(1) - g.z) * g.c + g.z * hi;
        const S pz = (hi - g.c) * g.z * (S(1) - g.z);
        const S sc = (S(1) - g.z) * (S(1) - g.c * g.c);
        const S sr = sc * g.r;
        const S st = sc * g.q * g.r * (S(1) - g.r);
        S Jrow[N];
        S acc = f;
#pragma unroll
        for (int j = 0; j < N; ++j) {
            S jv = pz * w.Uz[j] + sr * w.Uc[j] + st * w.Ur[j];
            jv += (j == i) ? g.z : S(0);
            Jrow[j] = jv;
            acc -= jv * h[j];
        }
        vstore<S, N>(J + (s * N + i) * N, Jrow);
        rhs[s * N + i] = acc;
    }
}

// sum over the lanes that hold the same state row (lane stride N inside a wavefront)
template <typename S, int N>
__device__ __forceinline__ S sum_same_row(S v) {
#pragma unroll
    for (int o = N; o < 64; o <<= 1) v += __shfl_xor(v, o);
    return v;
}
// sum over the N lanes of one position
template <typename S, int N>
__device__ __forceinline__ S sum_position(S v) {
#pragma unroll
    for (int o = 1; o < N; o <<= 1) v += __shfl_xor(v, o);
    return v;
}

// Sum of DP per-lane values over the N lanes of a position when DP <= N: the lanes first halve the number
// of values they carry while doubling the lanes each value has been summed over (log2 DP rounds, DP - 1
// shuffles in all), then finish with log2(N / DP) ordinary rounds.  Lane i ends up with the complete sum of
// value number i / (N / DP).  Fixed order, DP - 1 + log2(N / DP) shuffles instead of DP * log2 N.
template <typename S, int N, int DP>
__device__ __forceinline__ S reduce_scatter_position(const S* v, int i) {
    static_assert(DP <= N, "more values than lanes");
    S cur[DP];
#pragma unroll
    for (int k = 0; k < DP; ++k) cur[k] = v[k];
    int o = N / 2;
#pragma unroll
    for (int m = DP; m > 1; m >>= 1) {
        const bool up = (i & o) != 0;
#pragma unroll
        for (int j = 0; j < m / 2; ++j) {
            const S keep = up ? cur[j + m / 2] : cur[j];
            const S send = up ? cur[j] : cur[j + m / 2];
            cur[j] = keep + __shfl_xor(send, o);
        }
        o >>= 1;
    }
    S r = cur[0];
#pragma unroll
    for (int q = N / DP / 2; q >= 1; q >>= 1) r += __shfl_xor(r, q);
    return r;
}

// DP: the input width the x loops are unrolled for (d <= DP).
// MH: multi-head GRU with strides (Sec. 4.4, App. B.4).  Arrays are [batch][time][head][channel]; blockIdx.y is the
// head, which has its own parameters and partial rows and looks back st = 2^(head mod K) steps.  The first st positions
// of a head all start from y0, so dL/dy0 collects st terms: each goes to p.dy0_parts[batch][head][time] and a second
// kernel adds them in order.
template <typename S, int N, int DP, bool MH = false>
__global__ __launch_bounds__(kThreads) void gru_vjp_kernel(GruVjpParams p) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    S* sW = reinterpret_cast<S*>(smem_raw);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int d = p.d, ds = d | 1;
    constexpr int SPB = kThreads / N;
    const int i = tid % N;
    const int sg = tid / N;
    const S* __restrict__ theta = reinterpret_cast<const S*>(p.theta);
    const S* __restrict__ x = reinterpret_cast<const S*>(p.x);
    const S* __restrict__ y0 = reinterpret_cast<const S*>(p.y0);
    const S* __restrict__ y = reinterpret_cast<const S*>(p.y);
    const S* __restrict__ lam = reinterpret_cast<const S*>(p.lam);
    S* __restrict__ dx = reinterpret_cast<S*>(p.dx);
    S* __restrict__ dy0 = reinterpret_cast<S*>(MH ? p.dy0_parts : p.dy0);
    const long long P = 3LL * N * d + 3LL * N * N + 4LL * N;
    const int hd = MH ? (int)blockIdx.y : 0;
    const int H = MH ? p.H : 1;
    const int st = MH ? (1 << (hd % p.K)) : 1;
    const int smax = MH ? (1 << (p.K - 1)) : 1;
    if constexpr (MH) theta += (long long)hd * P;

    RowWeights<S, N> w;
    load_row_weights<S, N>(theta, d, i, w, sW, ds, tid);
    __syncthreads();

    S aUr[N], aUz[N], aUc[N], aWr[DP], aWz[DP], aWc[DP];
    S abr = S(0), abz = S(0), abc = S(0), abh = S(0);
#pragma unroll
    for (int j = 0; j < N; ++j) aUr[j] = aUz[j] = aUc[j] = S(0);
#pragma unroll
    for (int k = 0; k < DP; ++k) aWr[k] = aWz[k] = aWc[k] = S(0);

    const long long total = (long long)p.B * p.T;
    // every thread of a block runs the same number of passes so that the shuffles below always
    // see whole positions; a pass past the end contributes zeros
    const long long passes = (total + (long long)gridDim.x * SPB - 1) / ((long long)gridDim.x * SPB);
    // Software pipeline: the operands of the next pass are requested before the current one is computed, so a
    // pass does not expose a memory round trip (the accumulators leave room for two wavefronts per SIMD only).
    S hn[N], hin = S(0), xn[DP], lmn = S(0);
    auto fetch = [&](long long it) {
        const long long s = (it * gridDim.x + blockIdx.x) * SPB + sg;
        const bool live = s < total;
        const long long sc_ = live ? s : 0;
        const long long bi = sc_ / p.T;
        const int ti = (int)(sc_ - bi * p.T);
        const long long at = MH ? (sc_ * H + hd) : sc_;   // element index of this position in the [batch][time][head] grid
        const S* hp = (ti < st) ? (y0 + (MH ? bi * H + hd : bi) * N) : (y + (at - (long long)st * H) * N);
        vload<S, N>(hn, hp);
        hin = hp[i];
#pragma unroll
        for (int k = 0; k < DP; ++k) xn[k] = (k < d) ? x[at * d + k] : S(0);
        lmn = live ? lam[at * N + i] : S(0);
    };
    if (passes > 0) fetch(0);
    for (long long it = 0; it < passes; ++it) {
        const long long s = (it * gridDim.x + blockIdx.x) * SPB + sg;
        const bool live = s < total;
        const long long sc_ = live ? s : 0;
        const long long bi = sc_ / p.T;
        const int ti = (int)(sc_ - bi * p.T);
        const long long at = MH ? (sc_ * H + hd) : sc_;
        S h[N], xp[DP];
#pragma unroll
        for (int j = 0; j < N; ++j) h[j] = hn[j];
#pragma unroll
        for (int k = 0; k < DP; ++k) xp[k] = xn[k];
        const S hi = hin;
        const S lm = lmn;
        if (it + 1 < passes) fetch(it + 1);
        Gates<S, N> g;
        {
            S ar = w.br, az = w.bz, ac = w.bc, q = w.bh;
#pragma unroll
            for (int k = 0; k < DP; ++k) {
                if (k < d) {
                    ar += sW[(i)*ds + k] * xp[k];
                    az += sW[(N + i) * ds + k] * xp[k];
                    ac += sW[(2 * N + i) * ds + k] * xp[k];
                }
            }
#pragma unroll
            for (int j = 0; j < N; ++j) {
                ar += w.Ur[j] * h[j];
                az += w.Uz[j] * h[j];
                q += w.Uc[j] * h[j];
            }
            g.r = sigmoid_(ar);
            g.z = sigmoid_(az);
            g.q = q;
            g.c = tanh_(ac + g.r * q);
        }
        const S dcand = lm * (S(1) - g.z);
        const S dac = dcand * (S(1) - g.c * g.c);
        const S daz = lm * (hi - g.c) * g.z * (S(1) - g.z);
        const S dq = dac * g.r;
        const S dar = dac * g.q * g.r * (S(1) - g.r);
#pragma unroll
        for (int j = 0; j < N; ++j) {
            aUr[j] += dar * h[j];
            aUz[j] += daz * h[j];
            aUc[j] += dq * h[j];
        }
        abr += dar; abz += daz; abc += dac; abh += dq;
        S dxp[DP];
#pragma unroll
        for (int k = 0; k < DP; ++k) {
            dxp[k] = S(0);
            if (k < d) {
                const S xv = xp[k];
                aWr[k] += dar * xv;
                aWz[k] += daz * xv;
                aWc[k] += dac * xv;
                dxp[k] = sW[(i)*ds + k] * dar + sW[(N + i) * ds + k] * daz + sW[(2 * N + i) * ds + k] * dac;
            }
        }
        if (dx) {
            if constexpr (DP <= N) {
                const S tot = reduce_scatter_position<S, N, DP>(dxp, i);
                const int k = i / (N / DP);
                if (live && (i % (N / DP)) == 0 && k < d) dx[at * d + k] = tot;
            } else {
#pragma unroll
                for (int k = 0; k < DP; ++k) {
                    if (k < d) {
                        const S part = sum_position<S, N>(dxp[k]);
                        if (live && i == (k % N)) dx[at * d + k] = part;
                    }
                }
            }
        }
        if (dy0 && ti < st) {
            // dL/dy0 = J_1^T lam_1, row j: z_j lam_j + sum_i (U_r[i][j] dar_i + U_z[i][j] daz_i + U_c[i][j] dq_i)
            // (strided heads: one such term for each of the first st positions)
#pragma unroll
            for (int j = 0; j < N; ++j) {
                S part = w.Ur[j] * dar + w.Uz[j] * daz + w.Uc[j] * dq;
                part += (j == i) ? g.z * lm : S(0);
                part = sum_position<S, N>(part);
                if (live && i == j) dy0[(MH ? ((bi * H + hd) * smax + ti) : bi) * N + j] = part;
            }
        }
    }

    // per-wavefront partial sums, written without atomics: row (block * 4 + wave) of p.partial (of this head's rows)
    S* __restrict__ prow = reinterpret_cast<S*>(p.partial) +
                           (((long long)hd * gridDim.x + blockIdx.x) * (kThreads / 64) + (tid >> 6)) * P;
    const bool writer = lane < N;   // the first position group of the wavefront holds the totals
#pragma unroll
    for (int k = 0; k < DP; ++k) {
        if (k < d) {
            const S a = sum_same_row<S, N>(aWr[k]), b = sum_same_row<S, N>(aWz[k]), c = sum_same_row<S, N>(aWc[k]);
            if (writer) {
                prow[(long long)(i)*d + k] = a;
                prow[(long long)(N + i) * d + k] = b;
                prow[(long long)(2 * N + i) * d + k] = c;
            }
        }
    }
    S* pU = prow + 3LL * N * d;
#pragma unroll
    for (int j = 0; j < N; ++j) {
        const S a = sum_same_row<S, N>(aUr[j]), b = sum_same_row<S, N>(aUz[j]), c = sum_same_row<S, N>(aUc[j]);
        if (writer) {
            pU[(long long)(i)*N + j] = a;
            pU[(long long)(N + i) * N + j] = b;
            pU[(long long)(2 * N + i) * N + j] = c;
        }
    }
    S* pb = pU + 3LL * N * N;
    {
        const S a = sum_same_row<S, N>(abr), b = sum_same_row<S, N>(abz), c = sum_same_row<S, N>(abc),
                e = sum_same_row<S, N>(abh);
        if (writer) {
            pb[i] = a;
            pb[N + i] = b;
            pb[2 * N + i] = c;
            pb[3 * N + i] = e;
        }
    }
}

// Final sum of the per-wavefront partial rows in a fixed order (run-to-run identical): a block of 256
// threads owns 16 consecutive parameters; thread (g, q) adds the rows g, g+16, g+32, ... of parameter q in
// that order (eight independent loads in flight at a time), then the 16 strided sums meet in LDS and are
// added in the order g = 0..15.
template <typename S>
__global__ __launch_bounds__(256) void gru_vjp_reduce_kernel(const S* __restrict__ partial, S* __restrict__ dtheta,
                                                             long long P, int rows) {
    __shared__ S part[16][17];
    const int ql = threadIdx.x & 15, g = threadIdx.x >> 4;
    const long long q = (long long)blockIdx.x * 16 + ql;
    // (blockIdx.y: one set of rows and one output vector per head of a multi-head GRU)
    partial += (long long)blockIdx.y * rows * P;
    dtheta += (long long)blockIdx.y * P;
    S acc = S(0);
    if (q < P) {
        int r = g;
        for (; r + 7 * 16 < rows; r += 8 * 16) {
            S v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = partial[(long long)(r + 16 * u) * P + q];
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += v[u];
        }
        for (; r < rows; r += 16) acc += partial[(long long)r * P + q];
    }
    part[g][ql] = acc;
    __syncthreads();
    if (g == 0 && q < P) {
        S s = part[0][ql];
#pragma unroll
        for (int u = 1; u < 16; ++u) s += part[u][ql];
        dtheta[q] = s;
    }
}

template <typename S, int N>
hipError_t launch_fe(const GruParams& p, hipStream_t s) {
    constexpr int SPB = kThreads / N;
    const long long total = (long long)p.B * p.T;
    long long blocks = (total + SPB - 1) / SPB;
    if (blocks > 256 * 8) blocks = 256 * 8;
    if (blocks < 1) blocks = 1;
    const size_t shmem = (size_t)3 * N * (p.d | 1) * sizeof(S);
    if (p.d <= 16) hipLaunchKernelGGL((gru_funceval_kernel<S, N, 16>), dim3((unsigned)blocks), dim3(kThreads), shmem, s, p);
    else hipLaunchKernelGGL((gru_funceval_kernel<S, N, 32>), dim3((unsigned)blocks), dim3(kThreads), shmem, s, p);
    return hipGetLastError();
}

template <typename S>
hipError_t launch_fe_s(const GruParams& p, hipStream_t s) {
    switch (p.n) {
        case 1: return launch_fe<S, 1>(p, s);
        case 2: return launch_fe<S, 2>(p, s);
        case 4: return launch_fe<S, 4>(p, s);
        case 8: return launch_fe<S, 8>(p, s);
        case 16: return launch_fe<S, 16>(p, s);
        case 32: return launch_fe<S, 32>(p, s);
        case 64:   // fp32 only
            if constexpr (sizeof(S) == 4) return launch_fe<S, 64>(p, s);
            return hipErrorInvalidValue;
        default: return hipErrorInvalidValue;
    }
}

template <typename S, int N>
hipError_t launch_vjp(const GruVjpParams& p, hipStream_t s) {
    const size_t shmem = (size_t)3 * N * (p.d | 1) * sizeof(S);
    if (p.d <= 4) hipLaunchKernelGGL((gru_vjp_kernel<S, N, 4>), dim3((unsigned)p.blocks), dim3(kThreads), shmem, s, p);
    else if (p.d <= 8) hipLaunchKernelGGL((gru_vjp_kernel<S, N, 8>), dim3((unsigned)p.blocks), dim3(kThreads), shmem, s, p);
    else if (p.d <= 16) hipLaunchKernelGGL((gru_vjp_kernel<S, N, 16>), dim3((unsigned)p.blocks), dim3(kThreads), shmem, s, p);
    else hipLaunchKernelGGL((gru_vjp_kernel<S, N, 32>), dim3((unsigned)p.blocks), dim3(kThreads), shmem, s, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const long long P = 3LL * N * p.d + 3LL * N * N + 4LL * N;
    hipLaunchKernelGGL((gru_vjp_reduce_kernel<S>), dim3((unsigned)((P + 15) / 16)), dim3(256), 0, s,
                       reinterpret_cast<const S*>(p.partial), reinterpret_cast<S*>(p.dtheta), P,
                       p.blocks * (kThreads / 64));
    return hipGetLastError();
}

// dL/dy0 of a multi-head GRU: the terms of the first st positions of every head, added in time order
template <typename S>
__global__ __launch_bounds__(256) void gru_dy0_mh_kernel(const S* __restrict__ parts, S* __restrict__ dy0, int B, int T, int H,
                                                         int K, int n) {
    const long long q = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= (long long)B * H * n) return;
    const int j = (int)(q % n);
    const long long bh = q / n;
    const int hd = (int)(bh % H);
    const int smax = 1 << (K - 1);
    int st = 1 << (hd % K);
    if (st > T) st = T;
    S acc = S(0);
    for (int t = 0; t < st; ++t) acc += parts[(bh * smax + t) * n + j];
    dy0[q] = acc;
}

template <typename S, int N>
hipError_t launch_vjp_mh(const GruVjpParams& p, hipStream_t s) {
    const size_t shmem = (size_t)3 * N * (p.d | 1) * sizeof(S);
    hipLaunchKernelGGL((gru_vjp_kernel<S, N, 8, true>), dim3((unsigned)p.blocks, (unsigned)p.H), dim3(kThreads), shmem, s, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const long long P = 3LL * N * p.d + 3LL * N * N + 4LL * N;
    hipLaunchKernelGGL((gru_vjp_reduce_kernel<S>), dim3((unsigned)((P + 15) / 16), (unsigned)p.H), dim3(256), 0, s,
                       reinterpret_cast<const S*>(p.partial), reinterpret_cast<S*>(p.dtheta), P, p.blocks * (kThreads / 64));
    e = hipGetLastError();
    if (e != hipSuccess || !p.dy0) return e;
    const long long q = (long long)p.B * p.H * N;
    hipLaunchKernelGGL((gru_dy0_mh_kernel<S>), dim3((unsigned)((q + 255) / 256)), dim3(256), 0, s,
                       reinterpret_cast<const S*>(p.dy0_parts), reinterpret_cast<S*>(p.dy0), p.B, p.T, p.H, p.K, N);
    return hipGetLastError();
}

template <typename S>
hipError_t launch_vjp_mh_s(const GruVjpParams& p, hipStream_t s) {
    switch (p.n) {
        case 2: return launch_vjp_mh<S, 2>(p, s);
        case 4: return launch_vjp_mh<S, 4>(p, s);
        case 8: return launch_vjp_mh<S, 8>(p, s);
        default: return hipErrorInvalidValue;
    }
}

template <typename S>
hipError_t launch_vjp_s(const GruVjpParams& p, hipStream_t s) {
    switch (p.n) {
        case 1: return launch_vjp<S, 1>(p, s);
        case 2: return launch_vjp<S, 2>(p, s);
        case 4: return launch_vjp<S, 4>(p, s);
        case 8: return launch_vjp<S, 8>(p, s);
        case 16: return launch_vjp<S, 16>(p, s);
        case 32: return launch_vjp<S, 32>(p, s);
        case 64:   // fp32 only
            if constexpr (sizeof(S) == 4) return launch_vjp<S, 64>(p, s);
            return hipErrorInvalidValue;
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

int gru_vjp_blocks(int n, long long steps) {
    const int spb = kThreads / n;
    long long blocks = (steps + spb - 1) / spb;
    // (n = 16: the matrix-core kernel fits three wavefronts per SIMD, i.e. 768 blocks of four)
    if (blocks > (n == 16 ? 768 : 512)) blocks = (n == 16 ? 768 : 512);
    if (blocks < 1) blocks = 1;
    return (int)blocks;
}

// ---- embedding of a state size without kernels of its own into the next larger one ----
// The cell with n channels is run as a cell with np >= n channels whose extra rows and columns of every weight and
// bias are zero.  Extra channels then obey h' = h / 2 and stay at the zero they start from, and the real channels never
// see them (their columns of U are zero): the recurrence, its Jacobians, the Newton iterates and the cotangents of
// the real channels are exactly those of the n-channel cell.
template <typename S>
__global__ __launch_bounds__(256) void pad_rows_kernel(const S* __restrict__ src, S* __restrict__ dst, long long rows, int n, int np,
                                                      int unpack) {
    // pack: dst[rows][np] <- src[rows][n] with zeros behind; unpack: dst[rows][n] <- src[rows][np]
    const long long total = rows * (unpack ? n : np);
    for (long long q = (long long)blockIdx.x * blockDim.x + threadIdx.x; q < total; q += (long long)gridDim.x * blockDim.x) {
        if (unpack) {
            const long long r = q / n;
            const int c = (int)(q % n);
            dst[q] = src[r * np + c];
        } else {
            const long long r = q / np;
            const int c = (int)(q % np);
            dst[q] = c < n ? src[r * n + c] : S(0);
        }
    }
}

// theta of the GRU cell: W[3n,d] | U[3n,n] | b[3n] | b_hc[n]  <->  the same blocks for np channels
template <typename S>
__global__ __launch_bounds__(256) void pad_gru_theta_kernel(const S* __restrict__ src, S* __restrict__ dst, int n, int np, int d,
                                                           int unpack) {
    const long long Pp = 3LL * np * d + 3LL * np * np + 4LL * np;
    for (long long q = (long long)blockIdx.x * blockDim.x + threadIdx.x; q < Pp; q += (long long)gridDim.x * blockDim.x) {
        // position of entry q of the padded layout in the small one, or -1
        long long at = -1, r = q;
        if (r < 3LL * np * d) {
            const int gate = (int)(r / ((long long)np * d)), row = (int)((r / d) % np), col = (int)(r % d);
            if (row < n) at = ((long long)gate * n + row) * d + col;
        } else if ((r -= 3LL * np * d) < 3LL * np * np) {
            const int gate = (int)(r / ((long long)np * np)), row = (int)((r / np) % np), col = (int)(r % np);
            if (row < n && col < n) at = 3LL * n * d + ((long long)gate * n + row) * n + col;
        } else {
            r -= 3LL * np * np;   // four bias vectors of np entries
            const int which = (int)(r / np), row = (int)(r % np);
            if (row < n) at = 3LL * n * d + 3LL * n * n + (long long)which * n + row;
        }
        if (unpack) {
            if (at >= 0) dst[at] = src[q];
        } else {
            dst[q] = at >= 0 ? src[at] : S(0);
        }
    }
}

hipError_t launch_pad_rows(int dtype, const void* src, void* dst, long long rows, int n, int np, int unpack, hipStream_t s) {
    if (rows < 1) return hipSuccess;
    long long blocks = (rows * np + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    if (dtype == 0)
        hipLaunchKernelGGL((pad_rows_kernel<float>), dim3((unsigned)blocks), dim3(256), 0, s, reinterpret_cast<const float*>(src),
                           reinterpret_cast<float*>(dst), rows, n, np, unpack);
    else
        hipLaunchKernelGGL((pad_rows_kernel<double>), dim3((unsigned)blocks), dim3(256), 0, s, reinterpret_cast<const double*>(src),
                           reinterpret_cast<double*>(dst), rows, n, np, unpack);
    return hipGetLastError();
}

hipError_t launch_pad_gru_theta(int dtype, const void* src, void* dst, int n, int np, int d, int unpack, hipStream_t s) {
    const long long Pp = 3LL * np * d + 3LL * np * np + 4LL * np;
    const unsigned blocks = (unsigned)((Pp + 255) / 256);
    if (dtype == 0)
        hipLaunchKernelGGL((pad_gru_theta_kernel<float>), dim3(blocks), dim3(256), 0, s, reinterpret_cast<const float*>(src),
                           reinterpret_cast<float*>(dst), n, np, d, unpack);
    else
        hipLaunchKernelGGL((pad_gru_theta_kernel<double>), dim3(blocks), dim3(256), 0, s, reinterpret_cast<const double*>(src),
                           reinterpret_cast<double*>(dst), n, np, d, unpack);
    return hipGetLastError();
}

hipError_t launch_partial_reduce(int dtype, const void* partial, void* out, long long P, int rows, hipStream_t s) {
    if (P < 1 || rows < 1) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((P + 15) / 16));
    if (dtype == 0)
        hipLaunchKernelGGL((gru_vjp_reduce_kernel<float>), grid, dim3(256), 0, s, reinterpret_cast<const float*>(partial),
                           reinterpret_cast<float*>(out), P, rows);
    else
        hipLaunchKernelGGL((gru_vjp_reduce_kernel<double>), grid, dim3(256), 0, s, reinterpret_cast<const double*>(partial),
                           reinterpret_cast<double*>(out), P, rows);
    return hipGetLastError();
}

hipError_t launch_gru_funceval(int dtype, const GruParams& p, hipStream_t s) {
    if (p.d < 1 || p.d > kMaxD) return hipErrorInvalidValue;
    return dtype == 0 ? launch_fe_s<float>(p, s) : launch_fe_s<double>(p, s);
}

hipError_t launch_gru_vjp(int dtype, const GruVjpParams& p, hipStream_t s) {
    if (p.d < 1 || p.d > kMaxD) return hipErrorInvalidValue;
    if (p.H > 1 || p.K > 1) {   // multi-head GRU with strides
        if (p.d > 8 || p.H < 1 || p.K < 1 || !p.dy0_parts) return hipErrorInvalidValue;
        return dtype == 0 ? launch_vjp_mh_s<float>(p, s) : launch_vjp_mh_s<double>(p, s);
    }
    return dtype == 0 ? launch_vjp_s<float>(p, s) : launch_vjp_s<double>(p, s);
}

}  // namespace deer
