// LSTM cell kernels (Sec. 3.4 names the LSTM as an instance of the recurrence y_i = f(y_{i-1}, x_i)).
//   u units, state y = (h | c) of 2u entries, gates in the order input, forget, candidate, output:
//     i = sig(W_i x + U_i h + b_i)   f = sig(W_f x + U_f h + b_f)   g = tanh(W_g x + U_g h + b_g)   o = sig(W_o x + U_o h + b_o)
//     c' = f c + i g                 h' = o tanh(c')
//   theta = W[4u,d] | U[4u,u] | b[4u].
//   lstm_funceval_kernel: at every position the Jacobian J = d(h' | c')/d(h | c) and rhs = f - J y of the linear
//     recurrence the scan solves (Sec. 3.1 eq. 3 and 5 with the sign folded as for the GRU), at the previous iterate
//     shifted by one position.  Rows of unit j:
//       dc'_j/dh = c_j f_j(1-f_j) U_f[j] + g_j i_j(1-i_j) U_i[j] + i_j(1-g_j^2) U_g[j],   dc'_j/dc_j = f_j
//       dh'_j/dh = tanh(c'_j) o_j(1-o_j) U_o[j] + o_j(1-tanh^2 c'_j) dc'_j/dh,            dh'_j/dc_j = o_j(1-tanh^2 c'_j) f_j
//   lstm_vjp_kernel: vector-Jacobian product of the cell with the scanned cotangent at every position (Sec. 3.1.1
//     eq. 7, outer bracket): dL/dx, dL/dy0 and per-wavefront partial sums of dL/dtheta for the fixed-order reduction.
//
// The state travels in rows of np >= 2u scalars (np: the scan's state size; entries past 2u are zero and the kernels
// keep them zero: their rows of J and rhs are written as zeros).  One thread per (position, unit); a wavefront holds
// 64 / u positions (the remaining lanes idle), so the u threads of a position can exchange values by shuffles.
// The shape is a run-time argument (u <= 16, d <= 8); the weights sit in LDS with odd row strides.
#include "deer_common.h"

namespace deer {

namespace {

constexpr int kThreads = 256;
constexpr int kMaxU = 16;
constexpr int kMaxDx = 8;

__device__ __forceinline__ float sig_(float a) { return feed_sigmoid(a); }
__device__ __forceinline__ double sig_(double a) { return 1.0 / (1.0 + exp(-a)); }
__device__ __forceinline__ float th_(float a) { return feed_tanh(a); }
__device__ __forceinline__ double th_(double a) { return tanh(a); }

template <typename S>
struct LstmShared {
    S* W;   // [4u][ds], ds = d | 1
    S* U;   // [4u][us], us = u | 1
    S* b;   // [4u]
};

template <typename S>
__device__ __forceinline__ LstmShared<S> stage_weights(const S* __restrict__ theta, int u, int d, S* smem, int tid) {
    const int ds = d | 1, us = u | 1;
    LstmShared<S> w;
    w.W = smem;
    w.U = w.W + 4 * u * ds;
    w.b = w.U + 4 * u * us;
    for (int q = tid; q < 4 * u * d; q += kThreads) w.W[(q / d) * ds + (q % d)] = theta[q];
    const S* Ug = theta + 4 * u * d;
    for (int q = tid; q < 4 * u * u; q += kThreads) w.U[(q / u) * us + (q % u)] = Ug[q];
    const S* bg = Ug + 4 * u * u;
    for (int q = tid; q < 4 * u; q += kThreads) w.b[q] = bg[q];
    return w;
}

__host__ __device__ inline size_t lstm_smem_scalars(int u, int d) { return (size_t)4 * u * (d | 1) + (size_t)4 * u * (u | 1) + (size_t)4 * u; }

template <typename S>
struct LstmGates {
    S i, f, g, o, cn, tc;
};

// gates of unit j at (h, x)
template <typename S>
__device__ __forceinline__ LstmGates<S> lstm_gates(const LstmShared<S>& w, int u, int d, int j, const S* h, const S* xv, S cj) {
    const int ds = d | 1, us = u | 1;
    S a[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) a[q] = w.b[q * u + j];
#pragma unroll
    for (int k = 0; k < kMaxDx; ++k)
        if (k < d) {
#pragma unroll
            for (int q = 0; q < 4; ++q) a[q] += w.W[(q * u + j) * ds + k] * xv[k];
        }
#pragma unroll
    for (int k = 0; k < kMaxU; ++k)
        if (k < u) {
#pragma unroll
            for (int q = 0; q < 4; ++q) a[q] += w.U[(q * u + j) * us + k] * h[k];
        }
    LstmGates<S> g;
    g.i = sig_(a[0]);
    g.f = sig_(a[1]);
    g.g = th_(a[2]);
    g.o = sig_(a[3]);
    g.cn = g.f * cj + g.i * g.g;
    g.tc = th_(g.cn);
    return g;
}

// a row of np <= 32 scalars (np a power of two) from registers to memory
template <typename S>
__device__ __forceinline__ void store_row(S* dst, const S* row, int np) {
    if (np < 4) {
#pragma unroll
        for (int k = 0; k < 2; ++k)
            if (k < np) dst[k] = row[k];
        return;
    }
#pragma unroll
    for (int k4 = 0; k4 < 2 * kMaxU / 4; ++k4)
        if (4 * k4 < np) vstore<S, 4>(dst + 4 * k4, row + 4 * k4);
}

template <typename S>
__global__ __launch_bounds__(kThreads) void lstm_funceval_kernel(GruParams p) {
    if (gate_closed<S>(p.gate)) return;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int u = p.units, d = p.d, np = p.n, us = u | 1;
    const LstmShared<S> w = stage_weights<S>(reinterpret_cast<const S*>(p.theta), u, d, reinterpret_cast<S*>(smem_raw), tid);
    __syncthreads();
    const int PW = 64 / u;                 // positions per wavefront
    const int pg = lane / u, j = lane % u;
    const bool worker = pg < PW;
    const S* __restrict__ x = reinterpret_cast<const S*>(p.x);
    const S* __restrict__ y0 = reinterpret_cast<const S*>(p.y0);
    const S* __restrict__ y = reinterpret_cast<const S*>(p.y);
    S* __restrict__ J = reinterpret_cast<S*>(p.J);
    S* __restrict__ rhs = reinterpret_cast<S*>(p.rhs);
    const long long total = (long long)p.B * p.T;
    const long long stride = (long long)gridDim.x * (kThreads / 64) * PW;
    for (long long s = ((long long)blockIdx.x * (kThreads / 64) + wave) * PW + pg; worker && s < total; s += stride) {
        const long long bi = s / p.T;
        const int ti = (int)(s - bi * p.T);
        const S* yp = (ti == 0) ? (y0 + bi * np) : (y + (s - 1) * np);
        S h[kMaxU], xv[kMaxDx];
#pragma unroll
        for (int k = 0; k < kMaxU; ++k) h[k] = (k < u) ? yp[k] : S(0);
#pragma unroll
        for (int k = 0; k < kMaxDx; ++k) xv[k] = (k < d) ? x[s * d + k] : S(0);
        const S cj = yp[u + j];
        const LstmGates<S> g = lstm_gates<S>(w, u, d, j, h, xv, cj);
        const S dti = g.i * (S(1) - g.i), dtf = g.f * (S(1) - g.f), dtg = S(1) - g.g * g.g, dto = g.o * (S(1) - g.o);
        const S dtc = S(1) - g.tc * g.tc;
        const S ci = g.g * dti, cf = cj * dtf, cg = g.i * dtg;   // factors of U_i, U_f, U_g in dc'/dh
        const S ho = g.tc * dto, hc = g.o * dtc;                 // factor of U_o and of dc'/dh in dh'/dh
        S* Jh = J + (s * np + j) * np;         // row of h'_j
        S* Jc = J + (s * np + u + j) * np;     // row of c'_j
        S acch = g.o * g.tc, accc = g.cn;      // rhs = f - J y
        // the two rows are put together in registers and leave as 16-byte stores (a row is np scalars, np = 4, 8, 16 or 32;
        // np = 2 takes scalar stores)
        S rowh[2 * kMaxU], rowc[2 * kMaxU];
#pragma unroll
        for (int k = 0; k < 2 * kMaxU; ++k) {
            rowc[k] = (k == u + j) ? g.f : S(0);
            rowh[k] = (k == u + j) ? hc * g.f : S(0);
        }
#pragma unroll
        for (int k = 0; k < kMaxU; ++k)
            if (k < u) {
                const S vc = ci * w.U[(j)*us + k] + cf * w.U[(u + j) * us + k] + cg * w.U[(2 * u + j) * us + k];
                const S vh = ho * w.U[(3 * u + j) * us + k] + hc * vc;
                accc -= vc * h[k];
                acch -= vh * h[k];
                rowc[k] = vc;
                rowh[k] = vh;
            }
        store_row<S>(Jh, rowh, np);
        store_row<S>(Jc, rowc, np);
        accc -= g.f * cj;
        acch -= hc * g.f * cj;
        rhs[s * np + j] = acch;
        rhs[s * np + u + j] = accc;
        // rows past the state: zeros (the extra entries of the embedded state stay at zero)
        for (int r = 2 * u + j; r < np; r += u) {
            for (int k = 0; k < np; ++k) J[(s * np + r) * np + k] = S(0);
            rhs[s * np + r] = S(0);
        }
    }
}

template <typename S>
__global__ __launch_bounds__(kThreads) void lstm_vjp_kernel(GruVjpParams p) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int u = p.units, d = p.d, np = p.n, us = u | 1, ds = d | 1;
    S* smem = reinterpret_cast<S*>(smem_raw);
    const LstmShared<S> w = stage_weights<S>(reinterpret_cast<const S*>(p.theta), u, d, smem, tid);
    S* s_red = smem + ((lstm_smem_scalars(u, d) + 3) & ~(size_t)3);   // [4 waves][64 lanes] for the final sums
    __syncthreads();
    const int PW = 64 / u;
    const int pg = lane / u, j = lane % u;
    const bool worker = pg < PW;
    const int base = pg * u;               // first lane of this position's group
    const S* __restrict__ x = reinterpret_cast<const S*>(p.x);
    const S* __restrict__ y0 = reinterpret_cast<const S*>(p.y0);
    const S* __restrict__ y = reinterpret_cast<const S*>(p.y);
    const S* __restrict__ lam = reinterpret_cast<const S*>(p.lam);
    S* __restrict__ dx = reinterpret_cast<S*>(p.dx);
    S* __restrict__ dy0 = reinterpret_cast<S*>(p.dy0);

    S aU[4][kMaxU], aW[4][kMaxDx], ab[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        ab[q] = S(0);
#pragma unroll
        for (int k = 0; k < kMaxU; ++k) aU[q][k] = S(0);
#pragma unroll
        for (int k = 0; k < kMaxDx; ++k) aW[q][k] = S(0);
    }
    const long long total = (long long)p.B * p.T;
    const long long per_pass = (long long)gridDim.x * (kThreads / 64) * PW;
    const long long passes = (total + per_pass - 1) / per_pass;   // every lane runs them all: the shuffles need whole wavefronts
    for (long long it = 0; it < passes; ++it) {
        const long long s = it * per_pass + ((long long)blockIdx.x * (kThreads / 64) + wave) * PW + pg;
        const bool live = worker && s < total;
        const long long sc = live ? s : 0;
        const long long bi = sc / p.T;
        const int ti = (int)(sc - bi * p.T);
        const S* yp = (ti == 0) ? (y0 + bi * np) : (y + (sc - 1) * np);
        S h[kMaxU], xv[kMaxDx];
#pragma unroll
        for (int k = 0; k < kMaxU; ++k) h[k] = (k < u) ? yp[k] : S(0);
#pragma unroll
        for (int k = 0; k < kMaxDx; ++k) xv[k] = (k < d) ? x[sc * d + k] : S(0);
        const S cj = yp[u + j];
        const S lh = live ? lam[sc * np + j] : S(0), lc = live ? lam[sc * np + u + j] : S(0);
        const LstmGates<S> g = lstm_gates<S>(w, u, d, j, h, xv, cj);
        const S dcn = lc + lh * g.o * (S(1) - g.tc * g.tc);
        S da[4];
        da[0] = dcn * g.g * g.i * (S(1) - g.i);
        da[1] = dcn * cj * g.f * (S(1) - g.f);
        da[2] = dcn * g.i * (S(1) - g.g * g.g);
        da[3] = lh * g.tc * g.o * (S(1) - g.o);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            ab[q] += da[q];
#pragma unroll
            for (int k = 0; k < kMaxU; ++k) aU[q][k] += da[q] * h[k];
#pragma unroll
            for (int k = 0; k < kMaxDx; ++k) aW[q][k] += da[q] * xv[k];
        }
        // dL/dx[m] = sum over units and gates of W_q[unit][m] da_q[unit]; dL/dh_prev[k] likewise with U_q[unit][k]:
        // lane j of the group sums entry m = j (and j + u, ...) over the group's units, whose da arrive by shuffles
        const bool want_dy0 = dy0 != nullptr && ti == 0;   // (same for all lanes of a group)
        // (every lane runs the same shuffles; the entries a lane has no use for are dropped)
        S sh = S(0);
        for (int m = 0; m < u; ++m) {
#pragma unroll
            for (int q = 0; q < 4; ++q) sh += w.U[(q * u + m) * us + j] * __shfl(da[q], base + m);
        }
        for (int m0 = 0; m0 < d; m0 += u) {
            const int mx = m0 + j;                 // the input channel this lane sums in this round
            const int mc = mx < d ? mx : d - 1;
            S a = S(0);
            for (int m = 0; m < u; ++m) {
#pragma unroll
                for (int q = 0; q < 4; ++q) a += w.W[(q * u + m) * ds + mc] * __shfl(da[q], base + m);
            }
            if (live && dx && mx < d) dx[sc * d + mx] = a;
        }
        if (live && want_dy0) {
            dy0[bi * np + j] = sh;
            dy0[bi * np + u + j] = dcn * g.f;
            for (int r = 2 * u + j; r < np; r += u) dy0[bi * np + r] = S(0);
        }
    }

    // per-wavefront partial sums: the lanes j, j + u, j + 2u, ... of a wavefront hold the same unit
    const long long P = 4LL * u * d + 4LL * u * u + 4LL * u;
    S* __restrict__ prow = reinterpret_cast<S*>(p.partial) + ((long long)blockIdx.x * (kThreads / 64) + wave) * P;
    S* red = s_red + wave * 64;
    auto group_total = [&](S v) -> S {
        red[lane] = worker ? v : S(0);
        __builtin_amdgcn_wave_barrier();
        S t = S(0);
        for (int g2 = 0; g2 < PW; ++g2) t += red[g2 * u + j];
        __builtin_amdgcn_wave_barrier();
        return t;
    };
#pragma unroll
    for (int q = 0; q < 4; ++q) {
#pragma unroll
        for (int k = 0; k < kMaxDx; ++k) {
            const S t = group_total(aW[q][k]);
            if (lane < u && k < d) prow[(long long)(q * u + j) * d + k] = t;
        }
#pragma unroll
        for (int k = 0; k < kMaxU; ++k) {
            const S t = group_total(aU[q][k]);
            if (lane < u && k < u) prow[4LL * u * d + (long long)(q * u + j) * u + k] = t;
        }
        const S t = group_total(ab[q]);
        if (lane < u) prow[4LL * u * d + 4LL * u * u + q * u + j] = t;
    }
}

// ---------------------------------------------------------------------------------------------------------------
// LEM cell (the cell of the paper's last experiment; equations of the cited publication): u units, state (y | z),
// step dt, row blocks of theta in the order 1 | 2 | z | y:
//     s1 = dt sig(W_1 x + U_1 y + b_1)    s2 = dt sig(W_2 x + U_2 y + b_2)
//     z' = (1 - s1) z + s1 tanh(W_z x + U_z y + b_z)
//     y' = (1 - s2) y + s2 tanh(W_y x + U_y z' + b_y)
// Rows of the Jacobian d(y' | z')/d(y | z) of unit j, with c1 = ds1 (g_z - z), c2 = s1 (1 - g_z^2), ds = s (1 - s / dt):
//     dz'_j/dy = c1_j U_1[j] + c2_j U_z[j],                         dz'_j/dz_j = 1 - s1_j
//     dy'_j/dy = s2_j (1 - g_y^2) sum_m U_y[j][m] dz'_m/dy + ds2_j (g_y - y_j) U_2[j] + (1 - s2_j) e_j
//     dy'_j/dz_k = s2_j (1 - g_y^2) U_y[j][k] (1 - s1_k)
// The y update sees the new z of all units: every lane runs every pass so that the units of a position can exchange
// z', c1, c2 and s1 by shuffles.

template <typename S>
struct LemGates {
    S s1, s2, gz, zn, gy;
};

// gates of unit j; znv receives z' of all units of the position (lanes base .. base + u - 1)
template <typename S>
__device__ __forceinline__ LemGates<S> lem_gates(const LstmShared<S>& w, int u, int d, S dt, int j, int base, const S* yv,
                                                 const S* xv, S zj, S* znv) {
    const int ds = d | 1, us = u | 1;
    S a[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) a[q] = w.b[q * u + j];
#pragma unroll
    for (int k = 0; k < kMaxDx; ++k)
        if (k < d) {
#pragma unroll
            for (int q = 0; q < 4; ++q) a[q] += w.W[(q * u + j) * ds + k] * xv[k];
        }
#pragma unroll
    for (int k = 0; k < kMaxU; ++k)
        if (k < u) {
#pragma unroll
            for (int q = 0; q < 3; ++q) a[q] += w.U[(q * u + j) * us + k] * yv[k];
        }
    LemGates<S> g;
    g.s1 = dt * sig_(a[0]);
    g.s2 = dt * sig_(a[1]);
    g.gz = th_(a[2]);
    g.zn = (S(1) - g.s1) * zj + g.s1 * g.gz;
#pragma unroll
    for (int k = 0; k < kMaxU; ++k) znv[k] = __shfl(g.zn, base + (k < u ? k : 0));
#pragma unroll
    for (int k = 0; k < kMaxU; ++k)
        if (k < u) a[3] += w.U[(3 * u + j) * us + k] * znv[k];
    g.gy = th_(a[3]);
    return g;
}

// UC: the number of units when it is 2, 4, 8 or 16 and the scan's state size is exactly 2 UC (the rows of the Jacobian are
// then put together in registers and leave as 16-byte stores); 0: any shape, scalar stores
template <typename S, int UC>
__global__ __launch_bounds__(kThreads) void lem_funceval_kernel(GruParams p) {
    if (gate_closed<S>(p.gate)) return;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int u = UC > 0 ? UC : p.units, d = p.d, np = UC > 0 ? 2 * UC : p.n, us = u | 1;
    const S dt = (S)p.dt;
    const LstmShared<S> w = stage_weights<S>(reinterpret_cast<const S*>(p.theta), u, d, reinterpret_cast<S*>(smem_raw), tid);
    S* sMw = reinterpret_cast<S*>(smem_raw) + ((lstm_smem_scalars(u, d) + 3) & ~(size_t)3) + (size_t)wave * 64 * us;   // [64 lanes][us]
    __syncthreads();
    const int PW = 64 / u;
    const int pg = lane / u, j = lane % u;
    const bool worker = pg < PW;
    const int base = worker ? pg * u : 0;
    const S* __restrict__ x = reinterpret_cast<const S*>(p.x);
    const S* __restrict__ y0 = reinterpret_cast<const S*>(p.y0);
    const S* __restrict__ y = reinterpret_cast<const S*>(p.y);
    S* __restrict__ J = reinterpret_cast<S*>(p.J);
    S* __restrict__ rhs = reinterpret_cast<S*>(p.rhs);
    const long long total = (long long)p.B * p.T;
    const long long per_pass = (long long)gridDim.x * (kThreads / 64) * PW;
    const long long passes = (total + per_pass - 1) / per_pass;
    for (long long it = 0; it < passes; ++it) {
        const long long s = it * per_pass + ((long long)blockIdx.x * (kThreads / 64) + wave) * PW + pg;
        const bool live = worker && s < total;
        const long long sc = live ? s : 0;
        const long long bi = sc / p.T;
        const int ti = (int)(sc - bi * p.T);
        const S* sp = (ti == 0) ? (y0 + bi * np) : (y + (sc - 1) * np);
        S yv[kMaxU], zv[kMaxU], xv[kMaxDx], znv[kMaxU];
#pragma unroll
        for (int k = 0; k < kMaxU; ++k) {
            yv[k] = (k < u) ? sp[k] : S(0);
            zv[k] = (k < u) ? sp[u + k] : S(0);
        }
#pragma unroll
        for (int k = 0; k < kMaxDx; ++k) xv[k] = (k < d) ? x[sc * d + k] : S(0);
        const S yj = sp[j], zj = sp[u + j];
        const LemGates<S> g = lem_gates<S>(w, u, d, dt, j, base, yv, xv, zj, znv);
        const S ds1 = g.s1 * (S(1) - g.s1 / dt), ds2 = g.s2 * (S(1) - g.s2 / dt);
        const S c1 = ds1 * (g.gz - zj), c2 = g.s1 * (S(1) - g.gz * g.gz);
        const S dgy = g.s2 * (S(1) - g.gy * g.gy);
        const S c3 = ds2 * (g.gy - yj);
        // row j of dz'/dy goes to the wavefront's LDS slice: the rows of dy'/dy need all of them (U_y times that matrix)
        S mrow[kMaxU], s1v[kMaxU];
#pragma unroll
        for (int k = 0; k < kMaxU; ++k) {
            mrow[k] = (k < u) ? c1 * w.U[(j)*us + k] + c2 * w.U[(2 * u + j) * us + k] : S(0);
            if (k < u) sMw[lane * us + k] = mrow[k];
            s1v[k] = __shfl(g.s1, base + (k < u ? k : 0));
        }
        __builtin_amdgcn_wave_barrier();
        S chain[kMaxU];   // chain[k] = sum over m of U_y[j][m] dz'_m/dy_k
#pragma unroll
        for (int k = 0; k < kMaxU; ++k) chain[k] = S(0);
#pragma unroll
        for (int m = 0; m < kMaxU; ++m)
            if (m < u) {
                const S uym = w.U[(3 * u + j) * us + m];
#pragma unroll
                for (int k = 0; k < kMaxU; ++k)
                    if (k < u) chain[k] += uym * sMw[(base + m) * us + k];
            }
        __builtin_amdgcn_wave_barrier();
        if (live) {
            S* Jy = J + (s * np + j) * np;        // row of y'_j
            S* Jz = J + (s * np + u + j) * np;    // row of z'_j
            S accy = (S(1) - g.s2) * yj + g.s2 * g.gy, accz = g.zn;   // rhs = f - J (y | z)
            if constexpr (UC > 0) {
                S rowy[2 * UC], rowz[2 * UC];
#pragma unroll
                for (int k = 0; k < UC; ++k) {
                    const S vz = mrow[k];
                    S vy = dgy * chain[k] + c3 * w.U[(u + j) * us + k];
                    if (k == j) vy += S(1) - g.s2;
                    const S vyz = dgy * w.U[(3 * u + j) * us + k] * (S(1) - s1v[k]);
                    accz -= vz * yv[k];
                    accy -= vy * yv[k] + vyz * zv[k];
                    rowz[k] = vz;
                    rowy[k] = vy;
                    rowy[UC + k] = vyz;
                    rowz[UC + k] = (k == j) ? S(1) - g.s1 : S(0);
                }
                accz -= (S(1) - g.s1) * zj;
                vstore<S, 2 * UC>(Jy, rowy);
                vstore<S, 2 * UC>(Jz, rowz);
                rhs[s * np + j] = accy;
                rhs[s * np + u + j] = accz;
                continue;
            }
#pragma unroll
            for (int k = 0; k < kMaxU; ++k)
                if (k < u) {
                    const S vz = mrow[k];
                    S vy = dgy * chain[k] + c3 * w.U[(u + j) * us + k];
                    if (k == j) vy += S(1) - g.s2;
                    const S vyz = dgy * w.U[(3 * u + j) * us + k] * (S(1) - s1v[k]);
                    accz -= vz * yv[k];
                    accy -= vy * yv[k] + vyz * zv[k];
                    Jz[k] = vz;
                    Jy[k] = vy;
                    Jy[u + k] = vyz;
                    Jz[u + k] = (k == j) ? S(1) - g.s1 : S(0);
                }
            accz -= (S(1) - g.s1) * zj;
            for (int k = 2 * u; k < np; ++k) { Jy[k] = S(0); Jz[k] = S(0); }
            rhs[s * np + j] = accy;
            rhs[s * np + u + j] = accz;
            for (int r = 2 * u + j; r < np; r += u) {
                for (int k = 0; k < np; ++k) J[(s * np + r) * np + k] = S(0);
                rhs[s * np + r] = S(0);
            }
        }
    }
}

template <typename S>
__global__ __launch_bounds__(kThreads) void lem_vjp_kernel(GruVjpParams p) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int u = p.units, d = p.d, np = p.n, us = u | 1, ds = d | 1;
    const S dt = (S)p.dt;
    S* smem = reinterpret_cast<S*>(smem_raw);
    const LstmShared<S> w = stage_weights<S>(reinterpret_cast<const S*>(p.theta), u, d, smem, tid);
    S* s_red = smem + ((lstm_smem_scalars(u, d) + 3) & ~(size_t)3);   // [4 waves][64 lanes] for the final sums
    __syncthreads();
    const int PW = 64 / u;
    const int pg = lane / u, j = lane % u;
    const bool worker = pg < PW;
    const int base = worker ? pg * u : 0;
    const S* __restrict__ x = reinterpret_cast<const S*>(p.x);
    const S* __restrict__ y0 = reinterpret_cast<const S*>(p.y0);
    const S* __restrict__ y = reinterpret_cast<const S*>(p.y);
    const S* __restrict__ lam = reinterpret_cast<const S*>(p.lam);
    S* __restrict__ dx = reinterpret_cast<S*>(p.dx);
    S* __restrict__ dy0 = reinterpret_cast<S*>(p.dy0);

    S aU[4][kMaxU], aW[4][kMaxDx], ab[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        ab[q] = S(0);
#pragma unroll
        for (int k = 0; k < kMaxU; ++k) aU[q][k] = S(0);
#pragma unroll
        for (int k = 0; k < kMaxDx; ++k) aW[q][k] = S(0);
    }
    const long long total = (long long)p.B * p.T;
    const long long per_pass = (long long)gridDim.x * (kThreads / 64) * PW;
    const long long passes = (total + per_pass - 1) / per_pass;
    for (long long it = 0; it < passes; ++it) {
        const long long s = it * per_pass + ((long long)blockIdx.x * (kThreads / 64) + wave) * PW + pg;
        const bool live = worker && s < total;
        const long long sc = live ? s : 0;
        const long long bi = sc / p.T;
        const int ti = (int)(sc - bi * p.T);
        const S* sp = (ti == 0) ? (y0 + bi * np) : (y + (sc - 1) * np);
        S yv[kMaxU], xv[kMaxDx], znv[kMaxU];
#pragma unroll
        for (int k = 0; k < kMaxU; ++k) yv[k] = (k < u) ? sp[k] : S(0);
#pragma unroll
        for (int k = 0; k < kMaxDx; ++k) xv[k] = (k < d) ? x[sc * d + k] : S(0);
        const S yj = sp[j], zj = sp[u + j];
        const S ly = live ? lam[sc * np + j] : S(0), lz = live ? lam[sc * np + u + j] : S(0);
        const LemGates<S> g = lem_gates<S>(w, u, d, dt, j, base, yv, xv, zj, znv);
        // pre-activation cotangents, row blocks 1 | 2 | z | y  (da[0] and da[2] need dL/dz' of this unit, which collects
        // the y update's cotangents of all units through U_y)
        S da[4];
        da[3] = ly * g.s2 * (S(1) - g.gy * g.gy);
        da[1] = ly * (g.gy - yj) * g.s2 * (S(1) - g.s2 / dt);
        S dzn = lz;
        for (int m = 0; m < u; ++m) dzn += w.U[(3 * u + m) * us + j] * __shfl(da[3], base + m);
        da[0] = dzn * (g.gz - zj) * g.s1 * (S(1) - g.s1 / dt);
        da[2] = dzn * g.s1 * (S(1) - g.gz * g.gz);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            ab[q] += da[q];
#pragma unroll
            for (int k = 0; k < kMaxDx; ++k) aW[q][k] += da[q] * xv[k];
        }
#pragma unroll
        for (int k = 0; k < kMaxU; ++k) {
            aU[0][k] += da[0] * yv[k];
            aU[1][k] += da[1] * yv[k];
            aU[2][k] += da[2] * yv[k];
            aU[3][k] += da[3] * (k < u ? znv[k] : S(0));
        }
        const bool want_dy0 = dy0 != nullptr && ti == 0;
        S sh = S(0);   // dL/dy_prev[j] through the three blocks that read y
        for (int m = 0; m < u; ++m) {
#pragma unroll
            for (int q = 0; q < 3; ++q) sh += w.U[(q * u + m) * us + j] * __shfl(da[q], base + m);
        }
        for (int m0 = 0; m0 < d; m0 += u) {
            const int mx = m0 + j;
            const int mc = mx < d ? mx : d - 1;
            S a = S(0);
            for (int m = 0; m < u; ++m) {
#pragma unroll
                for (int q = 0; q < 4; ++q) a += w.W[(q * u + m) * ds + mc] * __shfl(da[q], base + m);
            }
            if (live && dx && mx < d) dx[sc * d + mx] = a;
        }
        if (live && want_dy0) {
            dy0[bi * np + j] = sh + ly * (S(1) - g.s2);
            dy0[bi * np + u + j] = dzn * (S(1) - g.s1);
            for (int r = 2 * u + j; r < np; r += u) dy0[bi * np + r] = S(0);
        }
    }

    const long long P = 4LL * u * d + 4LL * u * u + 4LL * u;
    S* __restrict__ prow = reinterpret_cast<S*>(p.partial) + ((long long)blockIdx.x * (kThreads / 64) + wave) * P;
    S* red = s_red + wave * 64;
    auto group_total = [&](S v) -> S {
        red[lane] = worker ? v : S(0);
        __builtin_amdgcn_wave_barrier();
        S t = S(0);
        for (int g2 = 0; g2 < PW; ++g2) t += red[g2 * u + j];
        __builtin_amdgcn_wave_barrier();
        return t;
    };
#pragma unroll
    for (int q = 0; q < 4; ++q) {
#pragma unroll
        for (int k = 0; k < kMaxDx; ++k) {
            const S t = group_total(aW[q][k]);
            if (lane < u && k < d) prow[(long long)(q * u + j) * d + k] = t;
        }
#pragma unroll
        for (int k = 0; k < kMaxU; ++k) {
            const S t = group_total(aU[q][k]);
            if (lane < u && k < u) prow[4LL * u * d + (long long)(q * u + j) * u + k] = t;
        }
        const S t = group_total(ab[q]);
        if (lane < u) prow[4LL * u * d + 4LL * u * u + q * u + j] = t;
    }
}

template <typename S>
hipError_t launch_lem_fe(const GruParams& p, hipStream_t s) {
    const int PW = 64 / p.units;
    const long long total = (long long)p.B * p.T;
    long long blocks = (total + 4 * PW - 1) / (4 * PW);
    if (blocks > 2048) blocks = 2048;
    if (blocks < 1) blocks = 1;
    const size_t shmem = (((lstm_smem_scalars(p.units, p.d) + 3) & ~(size_t)3) + (size_t)4 * 64 * (p.units | 1)) * sizeof(S);
    const dim3 grid((unsigned)blocks), blk(kThreads);
    int uc = (p.n == 2 * p.units) ? p.units : 0;
    if (sizeof(S) == 8 && uc == 16) uc = 0;   // (64 fp64 row entries in registers spill)
    if (uc == 16) hipLaunchKernelGGL((lem_funceval_kernel<S, 16>), grid, blk, shmem, s, p);
    else if (uc == 8) hipLaunchKernelGGL((lem_funceval_kernel<S, 8>), grid, blk, shmem, s, p);
    else if (uc == 4) hipLaunchKernelGGL((lem_funceval_kernel<S, 4>), grid, blk, shmem, s, p);
    else if (uc == 2) hipLaunchKernelGGL((lem_funceval_kernel<S, 2>), grid, blk, shmem, s, p);
    else hipLaunchKernelGGL((lem_funceval_kernel<S, 0>), grid, blk, shmem, s, p);
    return hipGetLastError();
}

template <typename S>
hipError_t launch_lem_vj(const GruVjpParams& p, hipStream_t s) {
    const size_t shmem = (((lstm_smem_scalars(p.units, p.d) + 3) & ~(size_t)3) + 4 * 64) * sizeof(S);
    hipLaunchKernelGGL((lem_vjp_kernel<S>), dim3((unsigned)p.blocks), dim3(kThreads), shmem, s, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const long long P = 4LL * p.units * p.d + 4LL * p.units * p.units + 4LL * p.units;
    return launch_partial_reduce(sizeof(S) == 4 ? 0 : 1, p.partial, p.dtheta, P, p.blocks * (kThreads / 64), s);
}

template <typename S>
hipError_t launch_fe(const GruParams& p, hipStream_t s) {
    const int PW = 64 / p.units;
    const long long total = (long long)p.B * p.T;
    long long blocks = (total + 4 * PW - 1) / (4 * PW);
    if (blocks > 2048) blocks = 2048;
    if (blocks < 1) blocks = 1;
    const size_t shmem = lstm_smem_scalars(p.units, p.d) * sizeof(S);
    hipLaunchKernelGGL((lstm_funceval_kernel<S>), dim3((unsigned)blocks), dim3(kThreads), shmem, s, p);
    return hipGetLastError();
}

template <typename S>
hipError_t launch_vj(const GruVjpParams& p, hipStream_t s) {
    const size_t shmem = (((lstm_smem_scalars(p.units, p.d) + 3) & ~(size_t)3) + 4 * 64) * sizeof(S);
    hipLaunchKernelGGL((lstm_vjp_kernel<S>), dim3((unsigned)p.blocks), dim3(kThreads), shmem, s, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const long long P = 4LL * p.units * p.d + 4LL * p.units * p.units + 4LL * p.units;
    return launch_partial_reduce(sizeof(S) == 4 ? 0 : 1, p.partial, p.dtheta, P, p.blocks * (kThreads / 64), s);
}

}  // namespace

bool lstm_supported(int units, int d) { return units >= 1 && units <= kMaxU && d >= 1 && d <= kMaxDx; }

int lstm_vjp_blocks(int units, long long steps) {
    const int PW = 64 / units;
    long long blocks = (steps + 4 * PW - 1) / (4 * PW);
    if (blocks > 512) blocks = 512;
    if (blocks < 1) blocks = 1;
    return (int)blocks;
}

hipError_t launch_lstm_funceval(int dtype, const GruParams& p, hipStream_t s) {
    if (!lstm_supported(p.units, p.d) || p.n < 2 * p.units) return hipErrorInvalidValue;
    return dtype == 0 ? launch_fe<float>(p, s) : launch_fe<double>(p, s);
}

hipError_t launch_lstm_vjp(int dtype, const GruVjpParams& p, hipStream_t s) {
    if (!lstm_supported(p.units, p.d) || p.n < 2 * p.units) return hipErrorInvalidValue;
    return dtype == 0 ? launch_vj<float>(p, s) : launch_vj<double>(p, s);
}

hipError_t launch_lem_funceval(int dtype, const GruParams& p, hipStream_t s) {
    if (!lstm_supported(p.units, p.d) || p.n < 2 * p.units || !(p.dt > 0.0)) return hipErrorInvalidValue;
    return dtype == 0 ? launch_lem_fe<float>(p, s) : launch_lem_fe<double>(p, s);
}

hipError_t launch_lem_vjp(int dtype, const GruVjpParams& p, hipStream_t s) {
    if (!lstm_supported(p.units, p.d) || p.n < 2 * p.units || !(p.dt > 0.0)) return hipErrorInvalidValue;
    return dtype == 0 ? launch_lem_vj<float>(p, s) : launch_lem_vj<double>(p, s);
}

}  // namespace deer
