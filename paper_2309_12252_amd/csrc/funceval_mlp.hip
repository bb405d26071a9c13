// NeuralODE kernels: dy/dt = f(y), f an MLP with two tanh hidden layers (Sec. 3.3).
//   mlp_funceval_kernel: at every grid point of the current iterate, f(y), J = df/dy =
//     W3 D2 W2 D1 W1 (D = diag(1 - tanh^2)), and the pair the paper's linear ODE uses:
//     G = -J and z = f + G y (Sec. 3.1 eq. 5, Sec. 3.3 eq. 8).
//   ode_discretise_kernel: per interval, midpoint values Gc = (G_i + G_{i+1})/2, zc likewise,
//     Gbar = exp(-Gc dt) and zbar = Gc^{-1}(I - Gbar) zc (Sec. 3.3 eq. 9), the latter evaluated as
//     dt * phi1(-Gc dt) zc with phi1(X) = sum_k X^k/(k+1)!, which equals the printed formula when
//     Gc is invertible and stays finite when it is not.  The kernel hands the scan the pair
//     (Gbar | res) with res = Gbar y_i + zbar - y_{i+1}, the residual of the current iterate: the
//     scan then solves for the correction y_next - y, which is the same Newton step in exact
//     arithmetic but keeps fp32 rounding relative to the (small) correction instead of to y.
//   pin_first_kernel: y[b,0,:] = y0[b,:] (the first grid point is the initial condition).
//
// mlp_funceval work split (generic kernel: fp64, n < 8): the n threads of a grid point sit in
// consecutive lanes; thread j owns column j of J and the hidden units j, j+n, j+2n, ... of both
// layers; activations are shared with cross-lane shuffles.  Weights are read with wave-uniform
// addresses (scalar loads).  fp32 with n = 8 runs on the matrix cores (mlp_funceval_mfma_kernel).
#include "deer_common.h"

namespace deer {

namespace {

constexpr int kThreads = 256;

// fp32: hardware exp2 and reciprocal (absolute error below 3e-7)
__device__ __forceinline__ float tanh_(float a) { return feed_tanh(a); }
__device__ __forceinline__ double tanh_(double a) { return tanh(a); }

template <typename S, int N, int W>
__global__ __launch_bounds__(kThreads) void mlp_funceval_kernel(MlpParams p) {
    if (gate_closed<S>(p.gate)) return;
    static_assert(W % N == 0, "hidden width must be a multiple of the state size");
    constexpr int UPT = W / N;   // hidden units per thread
    constexpr int SPB = kThreads / N;
    const int tid = threadIdx.x;
    const int j = tid % N;
    const int sg = tid / N;
    const int lane = tid & 63;
    const int base = lane - j;   // first lane of this grid point's group
    const S* __restrict__ th = reinterpret_cast<const S*>(p.theta);
    const S* __restrict__ W1 = th;                 // [W][N]
    const S* __restrict__ b1 = W1 + W * N;         // [W]
    const S* __restrict__ W2 = b1 + W;             // [W][W]
    const S* __restrict__ b2 = W2 + W * W;         // [W]
    const S* __restrict__ W3 = b2 + W;             // [N][W]
    const S* __restrict__ b3 = W3 + N * W;         // [N]
    const S* __restrict__ y = reinterpret_cast<const S*>(p.y);
    S* __restrict__ G = reinterpret_cast<S*>(p.G);
    S* __restrict__ z = reinterpret_cast<S*>(p.z);

    const long long total = (long long)p.B * p.T;
    const long long passes = (total + (long long)gridDim.x * SPB - 1) / ((long long)gridDim.x * SPB);
    for (long long it = 0; it < passes; ++it) {
        const long long s = (it * gridDim.x + blockIdx.x) * SPB + sg;
        const bool live = s < total;
        const long long sc = live ? s : 0;
        S yv[N];
        vload<S, N>(yv, y + sc * N);

        // layer 1: this thread's units, then all-gather
        S a1[W];
        {
            S mine[UPT];
#pragma unroll
            for (int u = 0; u < UPT; ++u) {
                const int m = u * N + j;
                S a = b1[m];
#pragma unroll
                for (int k = 0; k < N; ++k) a += W1[m * N + k] * yv[k];
                mine[u] = tanh_(a);
            }
#pragma unroll
            for (int u = 0; u < UPT; ++u)
#pragma unroll
                for (int q = 0; q < N; ++q) a1[u * N + q] = __shfl(mine[u], base + q);
        }
        // layer 2
        S a2[W];
        {
            S mine[UPT];
#pragma unroll
            for (int u = 0; u < UPT; ++u) {
                const int m = u * N + j;
                S a = b2[m];
#pragma unroll
                for (int k = 0; k < W; ++k) a += W2[m * W + k] * a1[k];
                mine[u] = tanh_(a);
            }
#pragma unroll
            for (int u = 0; u < UPT; ++u)
#pragma unroll
                for (int q = 0; q < N; ++q) a2[u * N + q] = __shfl(mine[u], base + q);
        }
        // f_j
        S fj = b3[j];
#pragma unroll
        for (int k = 0; k < W; ++k) fj += W3[j * W + k] * a2[k];

        // column j of J: W3 D2 W2 D1 W1[:, j]
        S u1[W];
#pragma unroll
        for (int m = 0; m < W; ++m) u1[m] = (S(1) - a1[m] * a1[m]) * W1[m * N + j];
        S u2[W];
#pragma unroll
        for (int m = 0; m < W; ++m) {
            S a = S(0);
#pragma unroll
            for (int k = 0; k < W; ++k) a += W2[m * W + k] * u1[k];
            u2[m] = (S(1) - a2[m] * a2[m]) * a;
        }
        const S yj = y[sc * N + j];
#pragma unroll
        for (int i = 0; i < N; ++i) {
            S a = S(0);
#pragma unroll
            for (int k = 0; k < W; ++k) a += W3[i * W + k] * u2[k];
            // a = J[i][j];  G = -J;  z_i = f_i + sum_j G[i][j] y_j
            if (live) G[(sc * N + i) * N + j] = -a;
            S part = -a * yj;
#pragma unroll
            for (int o = 1; o < N; o <<= 1) part += __shfl_xor(part, o);
            const S fi = __shfl(fj, base + i);
            if (live && j == i) z[sc * N + i] = fi + part;
        }
    }
}

// ---- MLP field on the matrix cores (fp32, n = 8, hidden width a multiple of 16) ----
//
// A wavefront handles 16 grid points at a time.  All products run on v_mfma_f32_16x16x4f32; matrices
// flow from one stage to the next in accumulator layout, which is directly a valid B operand (lane
// group g, register v = row 4g + v of a 16-row block), so no stage needs a transpose:
//   Z1 = W1 Y + b1 (columns = the 16 points), A1 = tanh Z1, D1 = 1 - A1^2
//   Z2 = W2 A1 + b2,                         A2 = tanh Z2, D2 = 1 - A2^2
//   f  = W3 A2 + b3
//   J y = W3 D2 W2 D1 (W1 y): the same chain applied to D1 * (Z1 - b1)        -> z = f - J y
//   J   = W3 D2 W2 D1 W1 for every point: the columns of the right factor are (point, j) pairs, 16 at a
//         time (two points x 8 columns); D1 and D2 of the right point reach a lane by one shuffle each.
// Rows 8..15 of the W3 products are padding (n = 8).
typedef float mlp_acc __attribute__((ext_vector_type(4)));

template <int WB, bool JONLY>   // hidden width / 16; JONLY: Jacobians only (z is written as zeros)
// (width 16 and 32: four wavefronts per SIMD through the launch bounds -- the compiler's own choice of three,
// with part of the operands in accumulation registers, measured 8 % slower, five with spills 10 % slower)
__global__ __launch_bounds__(kThreads, WB <= 2 ? 4 : 1) void mlp_funceval_mfma_kernel(MlpParams p) {
    if (gate_closed<float>(p.gate)) return;
    constexpr int W = 16 * WB, N = 8;
    const int lane = threadIdx.x & 63;
    const int g = lane >> 4, c = lane & 15;
    const float* __restrict__ th = reinterpret_cast<const float*>(p.theta);
    const float* __restrict__ W1 = th;
    const float* __restrict__ b1 = W1 + W * N;
    const float* __restrict__ W2 = b1 + W;
    const float* __restrict__ b2 = W2 + W * W;
    const float* __restrict__ W3 = b2 + W;
    const float* __restrict__ b3 = W3 + N * W;
    const float* __restrict__ y = reinterpret_cast<const float*>(p.y);
    float* __restrict__ G = reinterpret_cast<float*>(p.G);
    float* __restrict__ z = reinterpret_cast<float*>(p.z);

    // weights in operand layouts (c doubles as the row index r of A operands)
    float w1a[WB][2];          // A operand of stage 1: W1[16I + c][4kk + g]
    mlp_acc b1c[WB], b2c[WB];  // biases in accumulator layout: b[16I + 4g + v]
    float w2a[WB][WB][4];      // A operand: W2[16I + c][16K + 4g + v]
    float w3a[WB][4];          // A operand: W3[c][16K + 4g + v], rows >= 8 are zero
    mlp_acc b3c;
    float w1b[WB][4];          // W1[16K + 4g + v][c & 7], the column factor of D1 W1
#pragma unroll
    for (int I = 0; I < WB; ++I) {
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) w1a[I][kk] = W1[(16 * I + c) * N + 4 * kk + g];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            b1c[I][v] = b1[16 * I + 4 * g + v];
            b2c[I][v] = b2[16 * I + 4 * g + v];
            w1b[I][v] = W1[(16 * I + 4 * g + v) * N + (c & 7)];
            w3a[I][v] = (c < N) ? W3[c * W + 16 * I + 4 * g + v] : 0.0f;
        }
#pragma unroll
        for (int K = 0; K < WB; ++K)
#pragma unroll
            for (int v = 0; v < 4; ++v) w2a[I][K][v] = W2[(16 * I + c) * W + 16 * K + 4 * g + v];
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) b3c[v] = (4 * g + v < N) ? b3[4 * g + v] : 0.0f;

    const long long total = (long long)p.B * p.T;
    const long long nblk = (total + 15) / 16;
    const long long wave0 = ((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const long long nwaves = ((long long)gridDim.x * blockDim.x) >> 6;
    for (long long blk = wave0; blk < nblk; blk += nwaves) {
        const long long s0 = blk * 16;
        const long long sc = (s0 + c < total) ? s0 + c : total - 1;
        float yb[2];
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) yb[kk] = y[sc * N + 4 * kk + g];

        mlp_acc a1[WB], d1[WB], q1[WB];
#pragma unroll
        for (int I = 0; I < WB; ++I) {
            mlp_acc acc = b1c[I];
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(w1a[I][kk], yb[kk], acc, 0, 0, 0);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float t = feed_tanh(acc[v]);
                a1[I][v] = t;
                d1[I][v] = 1.0f - t * t;
                q1[I][v] = d1[I][v] * (acc[v] - b1c[I][v]);
            }
        }
        mlp_acc a2[WB], d2[WB], q2[WB];
#pragma unroll
        for (int I = 0; I < WB; ++I) {
            mlp_acc acc = b2c[I], accq = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int K = 0; K < WB; ++K)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(w2a[I][K][v], a1[K][v], acc, 0, 0, 0);
                    if constexpr (!JONLY) accq = __builtin_amdgcn_mfma_f32_16x16x4f32(w2a[I][K][v], q1[K][v], accq, 0, 0, 0);
                }
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float t = feed_tanh(acc[v]);
                a2[I][v] = t;
                d2[I][v] = 1.0f - t * t;
                q2[I][v] = d2[I][v] * accq[v];
            }
        }
        {
            mlp_acc f = b3c, jy = {0.f, 0.f, 0.f, 0.f};
            if constexpr (JONLY) {
                f = mlp_acc{0.f, 0.f, 0.f, 0.f};
            } else {
#pragma unroll
                for (int K = 0; K < WB; ++K)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        f = __builtin_amdgcn_mfma_f32_16x16x4f32(w3a[K][v], a2[K][v], f, 0, 0, 0);
                        jy = __builtin_amdgcn_mfma_f32_16x16x4f32(w3a[K][v], q2[K][v], jy, 0, 0, 0);
                    }
            }
            // z = f + G y = f - J y at point s0 + c, rows 4g + v < 8
            if (g < 2 && s0 + c < total) {
#pragma unroll
                for (int v = 0; v < 4; ++v) z[(s0 + c) * N + 4 * g + v] = f[v] - jy[v];
            }
        }
        // Jacobians, two points (16 columns) per round
#pragma unroll 2
        for (int cb = 0; cb < 8; ++cb) {
            const int src = (lane & 48) + 2 * cb + ((lane >> 3) & 1);   // lane holding D of this column's point
            float u1[WB][4];
#pragma unroll
            for (int K = 0; K < WB; ++K)
#pragma unroll
                for (int v = 0; v < 4; ++v) u1[K][v] = __shfl(d1[K][v], src) * w1b[K][v];
            float u2[WB][4];
#pragma unroll
            for (int I = 0; I < WB; ++I) {
                mlp_acc t = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int K = 0; K < WB; ++K)
#pragma unroll
                    for (int v = 0; v < 4; ++v) t = __builtin_amdgcn_mfma_f32_16x16x4f32(w2a[I][K][v], u1[K][v], t, 0, 0, 0);
#pragma unroll
                for (int v = 0; v < 4; ++v) u2[I][v] = __shfl(d2[I][v], src) * t[v];
            }
            mlp_acc jb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int K = 0; K < WB; ++K)
#pragma unroll
                for (int v = 0; v < 4; ++v) jb = __builtin_amdgcn_mfma_f32_16x16x4f32(w3a[K][v], u2[K][v], jb, 0, 0, 0);
            const long long sp = s0 + 2 * cb + (c >> 3);
            if (g < 2 && sp < total) {
#pragma unroll
                for (int v = 0; v < 4; ++v) G[(sp * N + 4 * g + v) * N + (c & 7)] = -jb[v];
            }
        }
    }
}

// ---- ODE discretisation: one thread per interval, n x n matrices in registers ----

template <typename S, int N>
__device__ __forceinline__ void matmul_reg(const S* A, const S* Bm, S* C) {
#pragma unroll
    for (int r = 0; r < N; ++r)
#pragma unroll
        for (int c = 0; c < N; ++c) {
            S s = S(0);
#pragma unroll
            for (int k = 0; k < N; ++k) s += A[r * N + k] * Bm[k * N + c];
            C[r * N + c] = s;
        }
}

template <typename S> struct SeriesTol;
template <> struct SeriesTol<float> { static constexpr float v = 1e-10f; };
template <> struct SeriesTol<double> { static constexpr double v = 1e-19; };

// D = exp(X) - I and pv = phi1(X) v for one n x n matrix held in registers (X is overwritten by its scaled
// copy): scaling so that the max-row-sum norm is at most 1/2, Taylor series, then the doublings undone.
template <typename S, int N, bool VEC = true>
__device__ __forceinline__ void expm1_phi1v(S* X, const S* zc, S* D, S* pv, bool need_matrix = true) {
    S norm = S(0);
#pragma unroll
    for (int r = 0; r < N; ++r) {
        S s = S(0);
#pragma unroll
        for (int c = 0; c < N; ++c) s += (X[r * N + c] < S(0) ? -X[r * N + c] : X[r * N + c]);
        norm = s > norm ? s : norm;
    }
    int sq = 0;
    S scale = S(1);
    while (norm > S(0.5) && sq < 40) { norm *= S(0.5); scale *= S(0.5); ++sq; }
    if (!(norm == norm)) sq = 0;
#pragma unroll
    for (int k = 0; k < N * N; ++k) X[k] *= scale;

    // Taylor series of D = exp(X) - I (matrix, identity left out so that nothing of size |X| is
    // rounded against 1) and of phi1(X) zc (vector), up to the first power K whose bound norm^K/K! is
    // below the working precision.  The matrix series runs in Horner form from the innermost bracket,
    //   D = (..((X/K + I) X/(K-1) + I) X/(K-2) ..+ I) X/1,
    // by right-multiplications, which update a matrix row by row in place: two live matrices instead of the
    // three a term-by-term sum needs.
    int K = 1;
    {
        S bound = norm;
        while (K < 24 && !(bound < SeriesTol<S>::v)) { ++K; bound *= norm / (S)K; }
    }
    // (a caller that wants the vector alone passes need_matrix = false: the matrix is then formed only where the
    // scaling has to be undone, which takes it)
    const bool with_matrix = need_matrix || sq > 0;
    if (with_matrix) {
        const S invK = S(1) / (S)K;
#pragma unroll
        for (int e = 0; e < N * N; ++e) D[e] = X[e] * invK;
    }
    for (int k = K - 1; with_matrix && k >= 1; --k) {
        const S invk = S(1) / (S)k;
#pragma unroll
        for (int r = 0; r < N; ++r) {
            S nr[N];
#pragma unroll
            for (int c = 0; c < N; ++c) {
                S s = X[r * N + c];
#pragma unroll
                for (int q = 0; q < N; ++q) s += D[r * N + q] * X[q * N + c];
                nr[c] = s * invk;
            }
#pragma unroll
            for (int c = 0; c < N; ++c) D[r * N + c] = nr[c];
        }
    }
    if constexpr (VEC) {
        S wv[N];
#pragma unroll
        for (int k = 0; k < N; ++k) { pv[k] = zc[k]; wv[k] = zc[k]; }
        for (int k = 1; k <= K; ++k) {
            // w_k = X w_{k-1} / (k+1)
            S nw[N];
            const S inv1 = S(1) / (S)(k + 1);
#pragma unroll
            for (int r = 0; r < N; ++r) {
                S s = S(0);
#pragma unroll
                for (int c = 0; c < N; ++c) s += X[r * N + c] * wv[c];
                nw[r] = s * inv1;
            }
#pragma unroll
            for (int r = 0; r < N; ++r) { wv[r] = nw[r]; pv[r] += nw[r]; }
        }
    }
    // undo the scaling: phi1(2X) v = (exp(X) + I) phi1(X) v / 2 = phi1(X) v + D phi1(X) v / 2,
    // exp(2X) - I = 2D + D^2
    for (int sstep = 0; sstep < sq; ++sstep) {
        if constexpr (VEC) {
            S nv[N];
#pragma unroll
            for (int r = 0; r < N; ++r) {
                S s = S(0);
#pragma unroll
                for (int c = 0; c < N; ++c) s += D[r * N + c] * pv[c];
                nv[r] = pv[r] + S(0.5) * s;
            }
#pragma unroll
            for (int r = 0; r < N; ++r) pv[r] = nv[r];
        }
        // (X is dead by now: it holds the copy of D that the update needs)
#pragma unroll
        for (int e = 0; e < N * N; ++e) X[e] = D[e];
#pragma unroll
        for (int r = 0; r < N; ++r)
#pragma unroll
            for (int c = 0; c < N; ++c) {
                S s = S(0);
#pragma unroll
                for (int q = 0; q < N; ++q) s += X[r * N + q] * X[q * N + c];
                D[r * N + c] = S(2) * X[r * N + c] + s;
            }
    }
}

// (two wavefronts per SIMD wanted: for n = 8 in fp32 the matrices of a thread just fit 256 registers)
// MATONLY: the backward pass wants the matrices alone (no vector series, no residual; z, y and res are not touched)
template <typename S, int N, bool MATONLY>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(sizeof(S) == 4 ? 2 : 1)))
void ode_discretise_kernel(OdeDiscParams p) {
    if (gate_closed<S>(p.gate)) return;
    const long long nint = (long long)p.B * (p.T - 1);
    const long long q = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (q >= nint) return;
    const long long bi = q / (p.T - 1);
    const long long i = q - bi * (p.T - 1);
    const S* __restrict__ G = reinterpret_cast<const S*>(p.G) + (bi * p.T + i) * (N * N);
    const S* __restrict__ z = reinterpret_cast<const S*>(p.z) + (bi * p.T + i) * N;
    const S* __restrict__ y = reinterpret_cast<const S*>(p.y) + (bi * p.T + i) * N;
    S* __restrict__ Gbar = reinterpret_cast<S*>(p.Gbar) + q * (N * N);
    S* __restrict__ res = reinterpret_cast<S*>(p.res) + q * N;
    const S dt = (S)p.dt;

    // X = -Gc dt / 2^sq with max-row-sum norm at most 1/2
    S X[N * N], zc[N];
    {
        S G0[N * N], G1[N * N];
        vload<S, N * N>(G0, G);
        vload<S, N * N>(G1, G + N * N);
#pragma unroll
        for (int k = 0; k < N * N; ++k) X[k] = S(-0.5) * (G0[k] + G1[k]) * dt;
        if constexpr (!MATONLY) {
            S z0[N], z1[N];
            vload<S, N>(z0, z);
            vload<S, N>(z1, z + N);
#pragma unroll
            for (int k = 0; k < N; ++k) zc[k] = S(0.5) * (z0[k] + z1[k]);
        }
    }
    S D[N * N], pv[N];
    expm1_phi1v<S, N, !MATONLY>(X, zc, D, pv);
    if constexpr (MATONLY) {
        if (!p.minus_identity) {
#pragma unroll
            for (int e = 0; e < N * N; ++e) D[e] += ((e / N) == (e % N)) ? S(1) : S(0);
        }
        vstore<S, N * N>(Gbar, D);
        return;
    }
    // residual of the current iterate in the discretised recurrence (Sec. 3.3 eq. 9):
    // res = Gbar y_i + zbar - y_{i+1} = D y_i + dt phi1 zc - (y_{i+1} - y_i)
    S y0v[N], y1v[N], rv[N];
    vload<S, N>(y0v, y);
    vload<S, N>(y1v, y + N);
#pragma unroll
    for (int r = 0; r < N; ++r) {
        S s = S(0);
#pragma unroll
        for (int c = 0; c < N; ++c) s += D[r * N + c] * y0v[c];
        rv[r] = (s + dt * pv[r]) - (y1v[r] - y0v[r]);
    }
    if (!p.minus_identity) {
#pragma unroll
        for (int e = 0; e < N * N; ++e) D[e] += ((e / N) == (e % N)) ? S(1) : S(0);
    }
    vstore<S, N * N>(Gbar, D);
    vstore<S, N>(res, rv);
}

// Dual of the discretisation for the backward derivative (Sec. 3.1.1 eq. 7 on the operator of Sec. 3.3
// eq. 8-9): one thread per interval i computes u_i = dt phi1(X_i)^T lam_{i+1} = dt phi1(X_i^T) lam_{i+1} with
// X_i = -(G_i + G_{i+1}) dt / 2, the weight with which the cotangent lam enters df/dtheta at the two ends of
// the interval, and, for the first interval, dL/dy0 = g_0 + exp(X_0)^T lam_1.
template <typename S, int N>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(sizeof(S) == 4 ? 2 : 1)))
void ode_dual_kernel(OdeDualParams p) {
    const long long nint = (long long)p.B * (p.T - 1);
    const long long q = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (q >= nint) return;
    const long long bi = q / (p.T - 1);
    const long long i = q - bi * (p.T - 1);
    const S* __restrict__ G = reinterpret_cast<const S*>(p.G) + (bi * p.T + i) * (N * N);
    const S* __restrict__ lam = reinterpret_cast<const S*>(p.lam) + q * N;   // lam at grid point i + 1
    S* __restrict__ u = reinterpret_cast<S*>(p.u) + q * N;
    const S dt = (S)p.dt;
    S X[N * N], lv[N];
    {
        S G0[N * N], G1[N * N];
        vload<S, N * N>(G0, G);
        vload<S, N * N>(G1, G + N * N);
        vload<S, N>(lv, lam);
#pragma unroll
        for (int r = 0; r < N; ++r)
#pragma unroll
            for (int c = 0; c < N; ++c) X[r * N + c] = S(-0.5) * (G0[c * N + r] + G1[c * N + r]) * dt;
    }
    S D[N * N], pv[N];
    const bool first = i == 0 && p.dy0;   // the first interval also yields dL/dy0, which takes the matrix
    expm1_phi1v<S, N>(X, lv, D, pv, first);
    S uv[N];
#pragma unroll
    for (int r = 0; r < N; ++r) uv[r] = dt * pv[r];
    vstore<S, N>(u, uv);
    if (first) {
        const S* __restrict__ g0 = reinterpret_cast<const S*>(p.g) + bi * p.T * N;
        S* __restrict__ out = reinterpret_cast<S*>(p.dy0) + bi * N;
#pragma unroll
        for (int r = 0; r < N; ++r) {
            S s = lv[r];
#pragma unroll
            for (int c = 0; c < N; ++c) s += D[r * N + c] * lv[c];
            out[r] = g0[r] + s;
        }
    }
}

// Residual of an approximate solution lam0 of the dual recurrence over grid points 1..T-1,
//   res_i = g_i - lam0_i + lam0_{i+1} + D_i^T lam0_{i+1}   (res_{T-1} = g_{T-1} - lam0_{T-1}),
// with D_i = exp(X_i) - I: the identity never meets D, so the residual keeps the digits of D that a product
// with the rounded I + D loses.  One thread per (grid point, row).
template <typename S, int N>
__global__ __launch_bounds__(kThreads) void ode_dual_residual_kernel(const S* __restrict__ D, const S* __restrict__ g,
                                                                     const S* __restrict__ lam0, S* __restrict__ res,
                                                                     int B, int T) {
    const long long T1 = T - 1;
    const long long total = (long long)B * T1 * N;
    const long long q = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (q >= total) return;
    const int r = (int)(q % N);
    const long long pi = q / N;            // (sequence, grid point - 1)
    const long long bi = pi / T1, i1 = pi - bi * T1;
    const S gi = g[(bi * T + i1 + 1) * N + r];
    S acc = gi - lam0[pi * N + r];
    if (i1 + 1 < T1) {
        const S* __restrict__ ln = lam0 + (pi + 1) * N;
        const S* __restrict__ Di = D + (bi * T1 + i1 + 1) * (N * N);   // interval from grid point i1+1 to i1+2
        S s = S(0);
#pragma unroll
        for (int c = 0; c < N; ++c) s += Di[c * N + r] * ln[c];
        acc = (acc + ln[r]) + s;
    }
    res[pi * N + r] = acc;
}

template <typename S>
__global__ __launch_bounds__(256) void pin_first_kernel(S* __restrict__ y, const S* __restrict__ y0, int B, int T,
                                                        int n) {
    const long long q = (long long)blockIdx.x * 256 + threadIdx.x;
    if (q >= (long long)B * n) return;
    const long long b = q / n;
    const int c = (int)(q - b * n);
    y[b * T * n + c] = y0[q];
}

__global__ __launch_bounds__(256) void fill_zero_kernel(uint4* __restrict__ p, size_t n16) {
    const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
    for (size_t q = (size_t)blockIdx.x * 256 + threadIdx.x; q < n16; q += (size_t)gridDim.x * 256) p[q] = zero;
}

// zero two ranges in one launch: a (16-byte aligned, n16a uint4) and b (4-byte aligned, nwb words)
__global__ __launch_bounds__(256) void fill_zero2_kernel(uint4* __restrict__ a, size_t n16a, unsigned* __restrict__ b,
                                                         size_t nwb) {
    const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
    const size_t stride = (size_t)gridDim.x * 256;
    const size_t first = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (size_t q = first; q < n16a; q += stride) a[q] = zero;
    size_t head = ((16 - (reinterpret_cast<uintptr_t>(b) & 15)) & 15) / 4;   // words in front of the aligned body
    if (head > nwb) head = nwb;
    const size_t body = (nwb - head) / 4;
    uint4* bb = reinterpret_cast<uint4*>(b + head);
    for (size_t q = first; q < body; q += stride) bb[q] = zero;
    if (first < head) b[first] = 0u;
    const size_t tail0 = head + 4 * body;
    if (tail0 + first < nwb) b[tail0 + first] = 0u;   // fewer than 4 words
}

template <typename S, int N, int W>
hipError_t launch_mlp_nw(const MlpParams& p, hipStream_t s) {
    constexpr int SPB = kThreads / N;
    const long long total = (long long)p.B * p.T;
    long long blocks = (total + SPB - 1) / SPB;
    if (blocks > 256 * 8) blocks = 256 * 8;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL((mlp_funceval_kernel<S, N, W>), dim3((unsigned)blocks), dim3(kThreads), 0, s, p);
    return hipGetLastError();
}

template <typename S, int N>
hipError_t launch_mlp_n(const MlpParams& p, hipStream_t s) {
    switch (p.width) {
        case 16: if constexpr (16 % N == 0) return launch_mlp_nw<S, N, 16>(p, s); else return hipErrorInvalidValue;
        case 32: if constexpr (32 % N == 0) return launch_mlp_nw<S, N, 32>(p, s); else return hipErrorInvalidValue;
        case 64: if constexpr (64 % N == 0) return launch_mlp_nw<S, N, 64>(p, s); else return hipErrorInvalidValue;
        default: return hipErrorInvalidValue;
    }
}

template <typename S>
hipError_t launch_mlp_s(const MlpParams& p, hipStream_t s) {
    switch (p.n) {
        case 2: return launch_mlp_n<S, 2>(p, s);
        case 4: return launch_mlp_n<S, 4>(p, s);
        case 8: return launch_mlp_n<S, 8>(p, s);
        default: return hipErrorInvalidValue;
    }
}

template <typename S>
hipError_t launch_disc_s(const OdeDiscParams& p, hipStream_t s) {
    const long long nint = (long long)p.B * (p.T - 1);
    dim3 grid((unsigned)((nint + kThreads - 1) / kThreads));
    switch (p.n) {
        case 2:
            if (p.matrix_only) hipLaunchKernelGGL((ode_discretise_kernel<S, 2, true>), grid, dim3(kThreads), 0, s, p);
            else hipLaunchKernelGGL((ode_discretise_kernel<S, 2, false>), grid, dim3(kThreads), 0, s, p);
            break;
        case 4:
            if (p.matrix_only) hipLaunchKernelGGL((ode_discretise_kernel<S, 4, true>), grid, dim3(kThreads), 0, s, p);
            else hipLaunchKernelGGL((ode_discretise_kernel<S, 4, false>), grid, dim3(kThreads), 0, s, p);
            break;
        case 8:
            if (p.matrix_only) hipLaunchKernelGGL((ode_discretise_kernel<S, 8, true>), grid, dim3(kThreads), 0, s, p);
            else hipLaunchKernelGGL((ode_discretise_kernel<S, 8, false>), grid, dim3(kThreads), 0, s, p);
            break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <typename S>
hipError_t launch_dual_s(const OdeDualParams& p, hipStream_t s) {
    const long long nint = (long long)p.B * (p.T - 1);
    const unsigned blocks = (unsigned)((nint + kThreads - 1) / kThreads);
    switch (p.n) {
        case 2: hipLaunchKernelGGL((ode_dual_kernel<S, 2>), dim3(blocks), dim3(kThreads), 0, s, p); break;
        case 4: hipLaunchKernelGGL((ode_dual_kernel<S, 4>), dim3(blocks), dim3(kThreads), 0, s, p); break;
        case 8: hipLaunchKernelGGL((ode_dual_kernel<S, 8>), dim3(blocks), dim3(kThreads), 0, s, p); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_mlp_funceval(int dtype, const MlpParams& p, hipStream_t s) {
    if (dtype == 0 && p.n == 8 && (p.width == 16 || p.width == 32 || p.width == 64)) {
        const long long nblk = ((long long)p.B * p.T + 15) / 16;   // one wavefront per 16 grid points
        long long blocks = (nblk + 3) / 4;
        if (blocks > 256 * 4) blocks = 256 * 4;
        if (blocks < 1) blocks = 1;
        dim3 grid((unsigned)blocks), blk(kThreads);
        if (p.jac_only) {
            if (p.width == 16) hipLaunchKernelGGL((mlp_funceval_mfma_kernel<1, true>), grid, blk, 0, s, p);
            else if (p.width == 32) hipLaunchKernelGGL((mlp_funceval_mfma_kernel<2, true>), grid, blk, 0, s, p);
            else hipLaunchKernelGGL((mlp_funceval_mfma_kernel<4, true>), grid, blk, 0, s, p);
        } else {
            if (p.width == 16) hipLaunchKernelGGL((mlp_funceval_mfma_kernel<1, false>), grid, blk, 0, s, p);
            else if (p.width == 32) hipLaunchKernelGGL((mlp_funceval_mfma_kernel<2, false>), grid, blk, 0, s, p);
            else hipLaunchKernelGGL((mlp_funceval_mfma_kernel<4, false>), grid, blk, 0, s, p);
        }
        return hipGetLastError();
    }
    return dtype == 0 ? launch_mlp_s<float>(p, s) : launch_mlp_s<double>(p, s);
}

hipError_t launch_ode_discretise(int dtype, const OdeDiscParams& p, hipStream_t s) {
    return dtype == 0 ? launch_disc_s<float>(p, s) : launch_disc_s<double>(p, s);
}

hipError_t launch_ode_dual(int dtype, const OdeDualParams& p, hipStream_t s) {
    if (p.T < 2) return hipErrorInvalidValue;
    return dtype == 0 ? launch_dual_s<float>(p, s) : launch_dual_s<double>(p, s);
}

template <typename S>
static hipError_t launch_residual_s(const void* D, const void* g, const void* lam0, void* res, int B, int T, int n,
                                    hipStream_t s) {
    const long long total = (long long)B * (T - 1) * n;
    const dim3 grid((unsigned)((total + kThreads - 1) / kThreads));
    const S* Dp = reinterpret_cast<const S*>(D);
    const S* gp = reinterpret_cast<const S*>(g);
    const S* lp = reinterpret_cast<const S*>(lam0);
    S* rp = reinterpret_cast<S*>(res);
    switch (n) {
        case 2: hipLaunchKernelGGL((ode_dual_residual_kernel<S, 2>), grid, dim3(kThreads), 0, s, Dp, gp, lp, rp, B, T); break;
        case 4: hipLaunchKernelGGL((ode_dual_residual_kernel<S, 4>), grid, dim3(kThreads), 0, s, Dp, gp, lp, rp, B, T); break;
        case 8: hipLaunchKernelGGL((ode_dual_residual_kernel<S, 8>), grid, dim3(kThreads), 0, s, Dp, gp, lp, rp, B, T); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_ode_dual_residual(int dtype, const void* D, const void* g, const void* lam0, void* res, int B, int T,
                                    int n, hipStream_t s) {
    if (T < 2) return hipErrorInvalidValue;
    return dtype == 0 ? launch_residual_s<float>(D, g, lam0, res, B, T, n, s)
                      : launch_residual_s<double>(D, g, lam0, res, B, T, n, s);
}

__global__ void copy_word_kernel(unsigned* __restrict__ dst, const unsigned* __restrict__ src) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *dst = *src;
}

hipError_t launch_copy_word(void* dst, const void* src, hipStream_t s) {
    hipLaunchKernelGGL(copy_word_kernel, dim3(1), dim3(64), 0, s, reinterpret_cast<unsigned*>(dst),
                       reinterpret_cast<const unsigned*>(src));
    return hipGetLastError();
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
    // bytes must be a multiple of 16 and p 16-byte aligned (workspace sections are)
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, s, reinterpret_cast<uint4*>(p), n16);
    return hipGetLastError();
}

hipError_t launch_fill_zero2(void* a, size_t abytes, void* b, size_t bbytes, hipStream_t s) {
    // a: 16-byte aligned, abytes a multiple of 16; b: 4-byte aligned, bbytes a multiple of 4
    const size_t n16 = abytes / 16, nw = bbytes / 4;
    size_t most = n16 > nw / 4 ? n16 : nw / 4;
    size_t blocks = (most + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(fill_zero2_kernel, dim3((unsigned)blocks), dim3(256), 0, s, reinterpret_cast<uint4*>(a), n16,
                       reinterpret_cast<unsigned*>(b), nw);
    return hipGetLastError();
}

hipError_t launch_pin_first(int dtype, void* y, const void* y0, int B, int T, int n, hipStream_t s) {
    const long long q = (long long)B * n;
    dim3 grid((unsigned)((q + 255) / 256));
    if (dtype == 0)
        hipLaunchKernelGGL((pin_first_kernel<float>), grid, dim3(256), 0, s, (float*)y, (const float*)y0, B, T, n);
    else
        hipLaunchKernelGGL((pin_first_kernel<double>), grid, dim3(256), 0, s, (double*)y, (const double*)y0, B, T, n);
    return hipGetLastError();
}

}  // namespace deer
