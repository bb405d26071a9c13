// MLP vector field of any depth and either activation (Sec. 3.3; the two-body network of App. B.2 has six
// linear layers with softplus on all but the last): the field kernel and the vector-Jacobian product for
// every shape the two-hidden-layer tanh kernels do not take.
//
//   f(y) = W_out s(W_L s(... s(W_1 y + b_1) ...) + b_L) + b_out,   s = tanh or softplus,
//   theta = W_1[w,n], b_1[w], (W_l[w,w], b_l[w]) for l = 2..L, W_out[n,w], b_out[n].
//
// mlp_gen_funceval_kernel: f and J = df/dy = W_out D_L W_L ... D_1 W_1 (D_l = diag s'(pre-activation)) by
// carrying S_l = d(a_l)/dy, a w x n matrix, through the layers next to the activations (forward mode: one
// pass, nothing of the earlier layers is kept); output G = -J and z = f + G y (Sec. 3.1 eq. 5, Sec. 3.3 eq. 8).
// mlp_gen_vjp_kernel: the reverse sweep at every grid point and the sums over the grid points of the outer
// products that make dL/dtheta (Sec. 3.1.1 eq. 7, outer bracket), as in the two-layer kernel: phase A leaves
// every point's activations and pre-activation cotangents as a row in LDS, phase B sums 4 x 4 blocks of
// (cotangent) x (layer input) over the points in registers; one partial row per block, added by the
// fixed-order reduction.
//
// fp32 with n = 8 and width 32 or 64 runs both on the matrix cores (mlp_gen_funceval_mfma_kernel,
// mlp_gen_vjp_mfma_kernel, described where they are defined); the kernels described here serve every other shape.
//
// Both kernels take the shape at run time.  A block of 256 threads handles `pts` grid points at a time with
// 256 / pts threads per point, which share the hidden units of a layer; a point's state is a row in LDS
// (row length = 4 mod 32 words, so that the 16-byte reads of consecutive points fall on different banks).
// The weights are read from memory as they are (rows by 16-byte loads, the same address in all lanes of a
// point group); the reverse sweep reads them down a column.
#include "deer_common.h"

namespace deer {

namespace {

constexpr int kThreads = 256;

__host__ __device__ inline int ceil4(int v) { return (v + 3) & ~3; }

template <typename S> struct Act;
template <> struct Act<float> {
    static __device__ __forceinline__ float tanh_(float a) { return feed_tanh(a); }
    static __device__ __forceinline__ float softplus(float a) { return fmaxf(a, 0.0f) + log1pf(expf(-fabsf(a))); }
    static __device__ __forceinline__ float sigmoid(float a) { return 1.0f / (1.0f + expf(-a)); }
    static __device__ __forceinline__ float one_minus_exp_neg(float a) { return -expm1f(-a); }
};
template <> struct Act<double> {
    static __device__ __forceinline__ double tanh_(double a) { return tanh(a); }
    static __device__ __forceinline__ double softplus(double a) { return fmax(a, 0.0) + log1p(exp(-fabs(a))); }
    static __device__ __forceinline__ double sigmoid(double a) { return 1.0 / (1.0 + exp(-a)); }
    static __device__ __forceinline__ double one_minus_exp_neg(double a) { return -expm1(-a); }
};

// activation and its derivative at pre-activation `pre`
template <typename S>
__device__ __forceinline__ void act_both(int kind, S pre, S& a, S& da) {
    if (kind == 0) {
        a = Act<S>::tanh_(pre);
        da = S(1) - a * a;
    } else {
        a = Act<S>::softplus(pre);
        da = Act<S>::sigmoid(pre);
    }
}
// derivative from the activation's value: tanh' = 1 - a^2, softplus' = sigmoid(pre) = 1 - exp(-a)
template <typename S>
__device__ __forceinline__ S dact_from_value(int kind, S a) {
    return kind == 0 ? S(1) - a * a : Act<S>::one_minus_exp_neg(a);
}

// offset of layer l (0-based hidden layers 0..L-1, L = the output layer) inside theta
__host__ __device__ inline long long layer_offset(int n, int w, int l) {
    if (l == 0) return 0;
    return (long long)w * n + w + (long long)(l - 1) * ((long long)w * w + w);
}
__host__ __device__ inline long long gen_theta_len(int n, int w, int L) { return layer_offset(n, w, L) + (long long)n * w + n; }

// ---------------------------------------------------------------------------------------------------------
// field + Jacobian on the matrix cores (fp32, n = 8, hidden width 16 * WB, L hidden layers)
// ---------------------------------------------------------------------------------------------------------
// The two-hidden-layer kernel's scheme for any depth: a wavefront handles 16 grid points as the columns of
// 16 x 16 x 4 products whose results stay in accumulator layout (a valid B operand of the next product):
//   values      A_1 = s(W_1 Y + b_1), A_l = s(W_l A_{l-1} + b_l), f = W_out A_L + b_out
//   J y         Q_1 = D_1 (W_1 Y), Q_l = D_l (W_l Q_{l-1}), J y = W_out Q_L            (z = f - J y)
//   Jacobians   16 columns (two points x 8 state entries) at a time: U_1 = D_1 W_1, U_l = D_l (W_l U_{l-1}),
//               J = W_out U_L; the derivative factors D_l of a column's point come from that point's lane by
//               one shuffle each.
// The derivative factors of all layers stay in registers (L * WB * 4); the weights are A operands read from
// LDS (rows padded to W + 4 words: 16-byte reads, lanes of a row group on different banks).
typedef float gacc __attribute__((ext_vector_type(4)));

// softplus and its derivative (the logistic function) from one exp2, one log2 and one reciprocal of the hardware:
// absolute errors below 3e-7
__device__ __forceinline__ void fast_act(int kind, float pre, float& a, float& da) {
    if (kind == 0) {
        a = feed_tanh(pre);
        da = 1.0f - a * a;
    } else {
        const float e = __builtin_amdgcn_exp2f(-1.44269504088896341f * fabsf(pre));   // exp(-|pre|) in (0, 1]
        const float r = __builtin_amdgcn_rcpf(1.0f + e);
        a = fmaxf(pre, 0.0f) + 0.693147180559945309f * __builtin_amdgcn_logf(1.0f + e);
        da = pre >= 0.0f ? r : e * r;
    }
}

template <int WB, int L>
__global__ __launch_bounds__(kThreads) void mlp_gen_funceval_mfma_kernel(MlpParams p) {
    if (gate_closed<float>(p.gate)) return;
    constexpr int W = 16 * WB, N = 8, WS = W + 4, W1S = 12;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    float* sW1 = reinterpret_cast<float*>(smem_raw);   // [W][W1S]: W_1, 8 columns used
    float* sWh = sW1 + W * W1S;                        // [L - 1][W][WS]
    float* sWo = sWh + (L - 1) * W * WS;               // [16][WS]: W_out, rows 8..15 zero
    float* sb = sWo + 16 * WS;                         // [L][W] hidden biases, then [16] output bias (entries 8..15 zero)
    const int tid = threadIdx.x, lane = tid & 63;
    const int g = lane >> 4, c = lane & 15;
    const float* __restrict__ th = reinterpret_cast<const float*>(p.theta);
    const int kind = p.act;
    for (int q = tid; q < W * N; q += kThreads) sW1[(q / N) * W1S + (q % N)] = th[q];
    for (int q = tid; q < W; q += kThreads) sb[q] = th[W * N + q];
    for (int l = 1; l < L; ++l) {
        const float* src = th + layer_offset(N, W, l);
        for (int q = tid; q < W * W; q += kThreads) sWh[((l - 1) * W + q / W) * WS + (q % W)] = src[q];
        for (int q = tid; q < W; q += kThreads) sb[l * W + q] = src[W * W + q];
    }
    {
        const float* src = th + layer_offset(N, W, L);
        for (int q = tid; q < 16 * W; q += kThreads) sWo[(q / W) * WS + (q % W)] = (q / W < N) ? src[q] : 0.0f;
        if (tid < 16) sb[L * W + tid] = (tid < N) ? src[N * W + tid] : 0.0f;
    }
    __syncthreads();

    const float* __restrict__ y = reinterpret_cast<const float*>(p.y);
    float* __restrict__ G = reinterpret_cast<float*>(p.G);
    float* __restrict__ z = reinterpret_cast<float*>(p.z);
    float w1b[WB][4];   // W_1[16K + 4g + v][c & 7]: the column factor of D_1 W_1
#pragma unroll
    for (int K = 0; K < WB; ++K)
#pragma unroll
        for (int v = 0; v < 4; ++v) w1b[K][v] = sW1[(16 * K + 4 * g + v) * W1S + (c & 7)];

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

        gacc a[WB], q[WB], d[L][WB];
        // layer 1
#pragma unroll
        for (int I = 0; I < WB; ++I) {
            gacc bias, acc;
#pragma unroll
            for (int v = 0; v < 4; ++v) bias[v] = sb[16 * I + 4 * g + v];
            acc = bias;
#pragma unroll
            for (int kk = 0; kk < 2; ++kk)
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(sW1[(16 * I + c) * W1S + 4 * kk + g], yb[kk], acc, 0, 0, 0);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float av, dv;
                fast_act(kind, acc[v], av, dv);
                a[I][v] = av;
                d[0][I][v] = dv;
                q[I][v] = dv * (acc[v] - bias[v]);
            }
        }
        // hidden layers 2..L
#pragma unroll
        for (int l = 1; l < L; ++l) {
            gacc an[WB], qn[WB];
#pragma unroll
            for (int I = 0; I < WB; ++I) {
                gacc acc, accq = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[v] = sb[l * W + 16 * I + 4 * g + v];
#pragma unroll
                for (int K = 0; K < WB; ++K) {
                    float wa[4];
                    vload<float, 4>(wa, &sWh[((l - 1) * W + 16 * I + c) * WS + 16 * K + 4 * g]);
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[v], a[K][v], acc, 0, 0, 0);
                        if (!p.jac_only) accq = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[v], q[K][v], accq, 0, 0, 0);
                    }
                }
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    float av, dv;
                    fast_act(kind, acc[v], av, dv);
                    an[I][v] = av;
                    d[l][I][v] = dv;
                    qn[I][v] = dv * accq[v];
                }
            }
#pragma unroll
            for (int I = 0; I < WB; ++I) { a[I] = an[I]; q[I] = qn[I]; }
        }
        // output layer: z = f - J y at point s0 + c, rows 4g + v < 8
        {
            gacc f = {0.f, 0.f, 0.f, 0.f}, jy = {0.f, 0.f, 0.f, 0.f};
            if (!p.jac_only) {
#pragma unroll
                for (int v = 0; v < 4; ++v) f[v] = sb[L * W + 4 * g + v];
#pragma unroll
                for (int K = 0; K < WB; ++K) {
                    float wa[4];
                    vload<float, 4>(wa, &sWo[c * WS + 16 * K + 4 * g]);
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        f = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[v], a[K][v], f, 0, 0, 0);
                        jy = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[v], q[K][v], jy, 0, 0, 0);
                    }
                }
            }
            if (g < 2 && s0 + c < total) {
#pragma unroll
                for (int v = 0; v < 4; ++v) z[(s0 + c) * N + 4 * g + v] = f[v] - jy[v];
            }
        }
        // Jacobians, two points (16 columns) per round
#pragma unroll 1
        for (int cb = 0; cb < 8; ++cb) {
            const int src = (lane & 48) + 2 * cb + ((lane >> 3) & 1);   // lane holding the factors of this column's point
            // (an offset the compiler cannot see through: the weight reads of a round stay in the round instead of being
            // hoisted into hundreds of registers in front of the loop)
            int zoff = 0;
            asm volatile("" : "+v"(zoff));
            float u[WB][4];
#pragma unroll
            for (int K = 0; K < WB; ++K)
#pragma unroll
                for (int v = 0; v < 4; ++v) u[K][v] = __shfl(d[0][K][v], src) * w1b[K][v];
#pragma unroll
            for (int l = 1; l < L; ++l) {
                float un[WB][4];
#pragma unroll
                for (int I = 0; I < WB; ++I) {
                    gacc t = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int K = 0; K < WB; ++K) {
                        float wa[4];
                        vload<float, 4>(wa, &sWh[((l - 1) * W + 16 * I + c) * WS + 16 * K + 4 * g + zoff]);
#pragma unroll
                        for (int v = 0; v < 4; ++v) t = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[v], u[K][v], t, 0, 0, 0);
                    }
#pragma unroll
                    for (int v = 0; v < 4; ++v) un[I][v] = __shfl(d[l][I][v], src) * t[v];
                }
#pragma unroll
                for (int I = 0; I < WB; ++I)
#pragma unroll
                    for (int v = 0; v < 4; ++v) u[I][v] = un[I][v];
            }
            gacc jb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int K = 0; K < WB; ++K) {
                float wa[4];
                vload<float, 4>(wa, &sWo[c * WS + 16 * K + 4 * g + zoff]);
#pragma unroll
                for (int v = 0; v < 4; ++v) jb = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[v], u[K][v], jb, 0, 0, 0);
            }
            const long long sp = s0 + 2 * cb + (c >> 3);
            if (g < 2 && sp < total) {
#pragma unroll
                for (int v = 0; v < 4; ++v) G[(sp * N + 4 * g + v) * N + (c & 7)] = -jb[v];
            }
        }
    }
}

size_t fe_mfma_smem(int W, int L) { return ((size_t)W * 12 + (size_t)(L - 1) * W * (W + 4) + 16 * (size_t)(W + 4) + (size_t)L * W + 16) * 4; }

template <int WB, int L>
hipError_t launch_fe_mfma_wl(const MlpParams& p, hipStream_t s) {
    const size_t shmem = fe_mfma_smem(16 * WB, L);
    static bool attr_set = false;   // more than 64 KB of dynamic LDS needs the attribute (set once per instantiation)
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&mlp_gen_funceval_mfma_kernel<WB, L>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const long long nblk = ((long long)p.B * p.T + 15) / 16;
    long long blocks = (nblk + 3) / 4;
    if (blocks > 512) blocks = 512;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL((mlp_gen_funceval_mfma_kernel<WB, L>), dim3((unsigned)blocks), dim3(kThreads), shmem, s, p);
    return hipGetLastError();
}

template <int WB>
hipError_t launch_fe_mfma_w(const MlpParams& p, hipStream_t s) {
    switch (p.nhid) {
        case 1: return launch_fe_mfma_wl<WB, 1>(p, s);
        case 2: return launch_fe_mfma_wl<WB, 2>(p, s);
        case 3: return launch_fe_mfma_wl<WB, 3>(p, s);
        case 4: return launch_fe_mfma_wl<WB, 4>(p, s);
        case 5: return launch_fe_mfma_wl<WB, 5>(p, s);
        default: return hipErrorInvalidValue;
    }
}

bool fe_mfma_supported(int dtype, int n, int width, int nhid) {
    return dtype == 0 && n == 8 && (width == 32 || width == 64) && nhid >= 1 && nhid <= 5;
}

// ---------------------------------------------------------------------------------------------------------
// vector-Jacobian product on the matrix cores (fp32, n = 8, hidden width 16 * WB, L hidden layers)
// ---------------------------------------------------------------------------------------------------------
// dL/dtheta = sum over grid points j of (df/dtheta)(y_j)^T w_j, w_j = (u_j + u_{j-1}) / 2 (Sec. 3.1.1 eq. 7, outer
// bracket, ODE form).  The accumulators of all layers do not fit the registers of a wavefront (width 64: 64 per
// hidden layer), so blockIdx.y names the layer a block accumulates: 0 = (W_1, b_1), l = (W_{l+1}, b_{l+1}),
// L = (W_out, b_out).  Every block runs the forward pass of its 16-point tiles (it needs the derivative factors
// of the layers above its own) and the reverse pass down to its layer, all as 16 x 16 x 4 products in accumulator
// layout as in the field kernel (weights from LDS; for the reverse products they are read down a column, row
// stride = 4 mod 64 words: no bank conflicts); its layer's cotangent and input then cross a wavefront-private LDS
// tile so that the grid points land on the contraction index of the outer-product sum.  One partial row per
// wavefront (each block fills its layer's slice of the row), the fixed-order reduction adds the rows.
template <int WB, int L>
__global__ __launch_bounds__(kThreads) void mlp_gen_vjp_mfma_kernel(MlpVjpParams p) {
    constexpr int W = 16 * WB, N = 8, WS = W + 4, W1S = 12, LD = 17, kWaves = kThreads / 64;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    float* sW1 = reinterpret_cast<float*>(smem_raw);   // [W][W1S]
    float* sWh = sW1 + W * W1S;                        // [L - 1][W][WS]
    float* sWo = sWh + (L - 1) * W * WS;               // [16][WS], rows 8..15 zero
    float* sb = sWo + 16 * WS;                         // [L][W] (+ 16 unused)
    float* sD = sb + L * W + 16;                       // [kWaves][2 W][LD]: cotangent rows | input rows of the block's layer
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, c = lane & 15;
    const int grp = blockIdx.y;
    const int kind = p.act;
    const float* __restrict__ th = reinterpret_cast<const float*>(p.theta);
    for (int q = tid; q < W * N; q += kThreads) sW1[(q / N) * W1S + (q % N)] = th[q];
    for (int q = tid; q < W; q += kThreads) sb[q] = th[W * N + q];
    for (int l = 1; l < L; ++l) {
        const float* src = th + layer_offset(N, W, l);
        for (int q = tid; q < W * W; q += kThreads) sWh[((l - 1) * W + q / W) * WS + (q % W)] = src[q];
        for (int q = tid; q < W; q += kThreads) sb[l * W + q] = src[W * W + q];
    }
    {
        const float* src = th + layer_offset(N, W, L);
        for (int q = tid; q < 16 * W; q += kThreads) sWo[(q / W) * WS + (q % W)] = (q / W < N) ? src[q] : 0.0f;
    }
    float* myD = sD + (size_t)wave * 2 * W * LD;
    for (int q = lane; q < 2 * W * LD; q += 64) myD[q] = 0.0f;   // (rows that a layer does not use stay zero)
    __syncthreads();

    const float* __restrict__ yg = reinterpret_cast<const float*>(p.y);
    const float* __restrict__ ug = reinterpret_cast<const float*>(p.u);
    gacc acc[WB][WB], accB[WB];
#pragma unroll
    for (int I = 0; I < WB; ++I) {
        accB[I] = gacc{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int J = 0; J < WB; ++J) acc[I][J] = gacc{0.f, 0.f, 0.f, 0.f};
    }
    const long long total = (long long)p.B * p.T;
    const long long tiles = (total + 15) / 16;
    const long long tstride = (long long)gridDim.x * kWaves;
    for (long long tile = (long long)blockIdx.x * kWaves + wave; tile < tiles; tile += tstride) {
        const long long s0 = tile * 16;
        const long long sc = s0 + c;
        const bool live = sc < total;
        const long long scl = live ? sc : 0;
        float yB[2];
#pragma unroll
        for (int m = 0; m < 2; ++m) yB[m] = live ? yg[scl * N + 4 * m + g] : 0.0f;
        // w in accumulator layout: entries 4g .. 4g+3 of point c (zero for g >= 2 and past the end)
        gacc wA = {0.f, 0.f, 0.f, 0.f};
        if (live && g < 2) {
            const long long b = sc / p.T, j = sc - b * p.T;
            float4 ua = {0.f, 0.f, 0.f, 0.f}, ub = {0.f, 0.f, 0.f, 0.f};
            if (j + 1 < p.T) ua = *reinterpret_cast<const float4*>(ug + (b * (p.T - 1) + j) * N + 4 * g);
            if (j > 0) ub = *reinterpret_cast<const float4*>(ug + (b * (p.T - 1) + j - 1) * N + 4 * g);
            wA = gacc{0.5f * (ua.x + ub.x), 0.5f * (ua.y + ub.y), 0.5f * (ua.z + ub.z), 0.5f * (ua.w + ub.w)};
        }

        // ---- forward: activations (the one entering the block's layer is kept) and derivative factors ----
        gacc a[WB], ain[WB], dact[L][WB];
#pragma unroll
        for (int I = 0; I < WB; ++I) {
            gacc z;
#pragma unroll
            for (int v = 0; v < 4; ++v) z[v] = sb[16 * I + 4 * g + v];
#pragma unroll
            for (int m = 0; m < 2; ++m) z = __builtin_amdgcn_mfma_f32_16x16x4f32(sW1[(16 * I + c) * W1S + 4 * m + g], yB[m], z, 0, 0, 0);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float av, dv;
                fast_act(kind, z[v], av, dv);
                a[I][v] = live ? av : 0.0f;
                dact[0][I][v] = dv;
            }
            ain[I] = a[I];
        }
#pragma unroll
        for (int l = 1; l < L; ++l) {
            gacc an[WB];
#pragma unroll
            for (int I = 0; I < WB; ++I) {
                gacc z;
#pragma unroll
                for (int v = 0; v < 4; ++v) z[v] = sb[l * W + 16 * I + 4 * g + v];
#pragma unroll
                for (int K = 0; K < WB; ++K) {
                    float wa[4];
                    vload<float, 4>(wa, &sWh[((l - 1) * W + 16 * I + c) * WS + 16 * K + 4 * g]);
#pragma unroll
                    for (int v = 0; v < 4; ++v) z = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[v], a[K][v], z, 0, 0, 0);
                }
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    float av, dv;
                    fast_act(kind, z[v], av, dv);
                    an[I][v] = live ? av : 0.0f;
                    dact[l][I][v] = dv;
                }
            }
#pragma unroll
            for (int I = 0; I < WB; ++I) {
                a[I] = an[I];
                if (l < grp) ain[I] = an[I];   // ain = output of hidden layer min(grp, L) - 1 (grp >= 1)
            }
        }

        // ---- reverse, down to the block's layer: dcur = cotangent of the pre-activation of hidden layer l ----
        gacc dcur[WB];
        if (grp < L) {
#pragma unroll
            for (int I = 0; I < WB; ++I) {
                gacc z = {0.f, 0.f, 0.f, 0.f};
                // k-step v: lane group g supplies entry 4g + v of w (zero from g = 2 on); A[i = c][k = g] = W_out[4g + v][16 I + c]
#pragma unroll
                for (int v = 0; v < 4; ++v) z = __builtin_amdgcn_mfma_f32_16x16x4f32(sWo[(4 * g + v) * WS + 16 * I + c], wA[v], z, 0, 0, 0);
#pragma unroll
                for (int v = 0; v < 4; ++v) dcur[I][v] = z[v] * dact[L - 1][I][v];
            }
#pragma unroll
            for (int l = L - 2; l >= 0; --l) {
                if (l >= grp) {   // (uniform)
                    gacc dn[WB];
#pragma unroll
                    for (int I = 0; I < WB; ++I) {
                        gacc z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int K = 0; K < WB; ++K)
#pragma unroll
                            for (int v = 0; v < 4; ++v)
                                z = __builtin_amdgcn_mfma_f32_16x16x4f32(sWh[(l * W + 16 * K + 4 * g + v) * WS + 16 * I + c], dcur[K][v], z, 0, 0, 0);
#pragma unroll
                        for (int v = 0; v < 4; ++v) dn[I][v] = z[v] * dact[l][I][v];
                    }
#pragma unroll
                    for (int I = 0; I < WB; ++I) dcur[I] = dn[I];
                }
            }
        }

        // ---- the layer's cotangent (rows 0 .. W-1 of the tile) and input (rows W .. 2W-1) with the points as columns ----
        if (grp == L) {
            if (g < 2) {
#pragma unroll
                for (int v = 0; v < 4; ++v) myD[(4 * g + v) * LD + c] = wA[v];
            }
            accB[0] += wA;
        } else {
#pragma unroll
            for (int I = 0; I < WB; ++I) {
#pragma unroll
                for (int v = 0; v < 4; ++v) myD[(16 * I + 4 * g + v) * LD + c] = dcur[I][v];
                accB[I] += dcur[I];
            }
        }
        if (grp > 0) {
#pragma unroll
            for (int I = 0; I < WB; ++I)
#pragma unroll
                for (int v = 0; v < 4; ++v) myD[(W + 16 * I + 4 * g + v) * LD + c] = ain[I][v];
        }
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            // A[i = c][k = g -> point 4m + g] from the cotangent rows, B[k = g -> point 4m + g][j = c] from the input rows
            const int at = c * LD + 4 * m + g;
            float td[WB], tin[WB];
#pragma unroll
            for (int I = 0; I < WB; ++I) {
                td[I] = myD[(16 * I) * LD + at];
                tin[I] = myD[(W + 16 * I) * LD + at];
            }
            if (grp == 0) {
                const long long sp = s0 + 4 * m + g;
                const float yK = (c < N && sp < total) ? yg[sp * N + c] : 0.0f;   // entry c of point 4m + g
#pragma unroll
                for (int I = 0; I < WB; ++I) acc[I][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(td[I], yK, acc[I][0], 0, 0, 0);
            } else if (grp == L) {
#pragma unroll
                for (int J = 0; J < WB; ++J) acc[0][J] = __builtin_amdgcn_mfma_f32_16x16x4f32(td[0], tin[J], acc[0][J], 0, 0, 0);
            } else {
#pragma unroll
                for (int I = 0; I < WB; ++I)
#pragma unroll
                    for (int J = 0; J < WB; ++J) acc[I][J] = __builtin_amdgcn_mfma_f32_16x16x4f32(td[I], tin[J], acc[I][J], 0, 0, 0);
            }
        }
    }

    // ---- this layer's slice of the wavefront's partial row ----
    const long long P = gen_theta_len(N, W, L);
    float* __restrict__ prow = reinterpret_cast<float*>(p.partial) + ((long long)blockIdx.x * kWaves + wave) * P;
    const long long base = layer_offset(N, W, grp);
#pragma unroll
    for (int I = 0; I < WB; ++I)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = 16 * I + 4 * g + v;
            float sbias = accB[I][v];
#pragma unroll
            for (int o = 1; o < 16; o <<= 1) sbias += __shfl_xor(sbias, o);
            if (grp == 0) {
                if (c < N) prow[base + row * N + c] = acc[I][0][v];
                if (c == 0) prow[base + W * N + row] = sbias;
            } else if (grp == L) {
                if (I == 0 && g < 2) {
#pragma unroll
                    for (int J = 0; J < WB; ++J) prow[base + (4 * g + v) * W + 16 * J + c] = acc[0][J][v];
                    if (c == 0) prow[base + N * W + 4 * g + v] = sbias;
                }
            } else {
#pragma unroll
                for (int J = 0; J < WB; ++J) prow[base + row * W + 16 * J + c] = acc[I][J][v];
                if (c == 0) prow[base + W * W + row] = sbias;
            }
        }
}

size_t vj_mfma_smem(int W, int L) { return ((size_t)W * 12 + (size_t)(L - 1) * W * (W + 4) + 16 * (size_t)(W + 4) + (size_t)L * W + 16 + 4 * 2 * (size_t)W * 17) * 4; }

template <int WB, int L>
hipError_t launch_vj_mfma_wl(const MlpVjpParams& p, int blocks, hipStream_t s) {
    const size_t shmem = vj_mfma_smem(16 * WB, L);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&mlp_gen_vjp_mfma_kernel<WB, L>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((mlp_gen_vjp_mfma_kernel<WB, L>), dim3((unsigned)blocks, (unsigned)(L + 1)), dim3(kThreads), shmem, s, p);
    return hipGetLastError();
}

template <int WB>
hipError_t launch_vj_mfma_w(const MlpVjpParams& p, int blocks, hipStream_t s) {
    switch (p.nhid) {
        case 1: return launch_vj_mfma_wl<WB, 1>(p, blocks, s);
        case 2: return launch_vj_mfma_wl<WB, 2>(p, blocks, s);
        case 3: return launch_vj_mfma_wl<WB, 3>(p, blocks, s);
        case 4: return launch_vj_mfma_wl<WB, 4>(p, blocks, s);
        case 5: return launch_vj_mfma_wl<WB, 5>(p, blocks, s);
        default: return hipErrorInvalidValue;
    }
}

// ---------------------------------------------------------------------------------------------------------
// field + Jacobian
// ---------------------------------------------------------------------------------------------------------
struct FeRow {
    int a[2], S[2], y, len, np;
    __host__ __device__ FeRow(int n, int w) {
        np = ceil4(n);
        a[0] = 0; a[1] = w; S[0] = 2 * w; S[1] = 2 * w + w * np; y = 2 * w + 2 * w * np;
        len = y + np;
        while ((len & 31) != 4) len += 4;
    }
};

template <typename S>
__global__ __launch_bounds__(kThreads) void mlp_gen_funceval_kernel(MlpParams p, int pts) {
    if (gate_closed<S>(p.gate)) return;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    S* rows = reinterpret_cast<S*>(smem_raw);
    const int n = p.n, w = p.width, L = p.nhid, kind = p.act;
    const FeRow rl(n, w);
    const int np = rl.np;
    const int tid = threadIdx.x;
    const int split = kThreads / pts;
    const int pt = tid % pts, part = tid / pts;
    const S* __restrict__ th = reinterpret_cast<const S*>(p.theta);
    const S* __restrict__ yg = reinterpret_cast<const S*>(p.y);
    S* __restrict__ Gg = reinterpret_cast<S*>(p.G);
    S* __restrict__ zg = reinterpret_cast<S*>(p.z);
    const long long total = (long long)p.B * p.T;
    const long long chunks = (total + pts - 1) / pts;
    S* R = rows + (size_t)pt * rl.len;

    for (long long ch = blockIdx.x; ch < chunks; ch += gridDim.x) {
        const long long gp = ch * pts + pt;
        const bool valid = gp < total;
        if (part == 0) {
            for (int k = 0; k < np; ++k) R[rl.y + k] = (valid && k < n) ? yg[gp * n + k] : S(0);
        }
        __syncthreads();
        // layer 1: a = s(W_1 y + b_1), S = D_1 W_1
        {
            const S* __restrict__ W1 = th;
            const S* __restrict__ b1 = th + (long long)w * n;
            for (int h = part; h < w; h += split) {
                S pre = b1[h];
                for (int k = 0; k < n; ++k) pre += W1[h * n + k] * R[rl.y + k];
                S a, da;
                act_both<S>(kind, pre, a, da);
                R[rl.a[0] + h] = a;
                for (int k = 0; k < np; ++k) R[rl.S[0] + h * np + k] = (k < n) ? da * W1[h * n + k] : S(0);
            }
        }
        __syncthreads();
        // layers 2..L: a' = s(W a + b), S' = D (W S)
        int cur = 0;
        for (int l = 1; l < L; ++l) {
            const S* __restrict__ Wl = th + layer_offset(n, w, l);
            const S* __restrict__ bl = Wl + (long long)w * w;
            const S* ain = R + rl.a[cur];
            const S* Sin = R + rl.S[cur];
            for (int h = part; h < w; h += split) {
                S pre = bl[h];
                S t[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) t[j] = S(0);
                for (int k = 0; k < w; k += 4) {
                    S wv[4], av[4];
                    vload<S, 4>(wv, Wl + (long long)h * w + k);
                    vload<S, 4>(av, ain + k);
#pragma unroll
                    for (int kk = 0; kk < 4; ++kk) {
                        pre += wv[kk] * av[kk];
                        S sv[8];
                        vload<S, 4>(sv, Sin + (k + kk) * np);
                        if (np > 4) vload<S, 4>(sv + 4, Sin + (k + kk) * np + 4);
#pragma unroll
                        for (int j = 0; j < 4; ++j) t[j] += wv[kk] * sv[j];
                        if (np > 4) {
#pragma unroll
                            for (int j = 4; j < 8; ++j) t[j] += wv[kk] * sv[j];
                        }
                    }
                }
                S a, da;
                act_both<S>(kind, pre, a, da);
                R[rl.a[cur ^ 1] + h] = a;
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (j < np) R[rl.S[cur ^ 1] + h * np + j] = da * t[j];
            }
            cur ^= 1;
            __syncthreads();
        }
        // output layer: f = W_out a + b_out, J = W_out S; G = -J, z = f - J y
        {
            const S* __restrict__ Wo = th + layer_offset(n, w, L);
            const S* __restrict__ bo = Wo + (long long)n * w;
            const S* ain = R + rl.a[cur];
            const S* Sin = R + rl.S[cur];
            for (int i = part; i < n; i += split) {
                S f = bo[i];
                S t[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) t[j] = S(0);
                for (int k = 0; k < w; k += 4) {
                    S wv[4], av[4];
                    vload<S, 4>(wv, Wo + (long long)i * w + k);
                    vload<S, 4>(av, ain + k);
#pragma unroll
                    for (int kk = 0; kk < 4; ++kk) {
                        f += wv[kk] * av[kk];
                        S sv[8];
                        vload<S, 4>(sv, Sin + (k + kk) * np);
                        if (np > 4) vload<S, 4>(sv + 4, Sin + (k + kk) * np + 4);
#pragma unroll
                        for (int j = 0; j < 4; ++j) t[j] += wv[kk] * sv[j];
                        if (np > 4) {
#pragma unroll
                            for (int j = 4; j < 8; ++j) t[j] += wv[kk] * sv[j];
                        }
                    }
                }
                if (valid) {
                    S jy = S(0);
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (j < n) {
                            jy += t[j] * R[rl.y + j];
                            Gg[(gp * n + i) * n + j] = -t[j];
                        }
                    zg[gp * n + i] = p.jac_only ? S(0) : f - jy;
                }
            }
        }
        __syncthreads();
    }
}

template <typename S>
int fe_points(int n, int w, size_t* bytes) {
    const FeRow rl(n, w);
    int pts = 64;
    while (pts > 4 && (size_t)pts * rl.len * sizeof(S) > (size_t)48 * 1024) pts >>= 1;
    *bytes = (size_t)pts * rl.len * sizeof(S);
    return pts;
}

template <typename S>
hipError_t launch_fe(const MlpParams& p, hipStream_t s) {
    size_t bytes = 0;
    const int pts = fe_points<S>(p.n, p.width, &bytes);
    if (bytes > (size_t)150 * 1024) return hipErrorInvalidValue;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(mlp_gen_funceval_kernel<S>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) return e;
    const long long total = (long long)p.B * p.T;
    long long blocks = (total + pts - 1) / pts;
    if (blocks > 2048) blocks = 2048;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL((mlp_gen_funceval_kernel<S>), dim3((unsigned)blocks), dim3(kThreads), bytes, s, p, pts);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------------
// vector-Jacobian product with the parameter-gradient sums
// ---------------------------------------------------------------------------------------------------------
constexpr int kMaxTasks = 5;   // 4 x 4 blocks per thread (width 64, five hidden layers, n = 8: 1,170 tasks over 256 threads)

// a point's row: a_1..a_L | d_1..d_L (cotangents of the pre-activations) | y | w | 1
struct VjRow {
    int a, d, y, w, one, len;
    __host__ __device__ VjRow(int n, int width, int L) {
        a = 0; d = L * width; y = 2 * L * width; w = y + ceil4(n); one = w + ceil4(n);
        len = one + 4;
        while ((len & 31) != 4) len += 4;
    }
};

struct Task {
    int uo, vo, out, rs, nr, nc;
};

__host__ __device__ inline int gen_task_count(int n, int w, int L) {
    const int wb = w / 4, nb = ceil4(n) / 4;
    return wb * nb + wb + (L - 1) * (wb * wb + wb) + nb * wb + nb;
}

// task number q: four entries of one field of the row (rows of the block) times four entries of another
__device__ __forceinline__ bool make_task(int q, int n, int w, int L, const VjRow& rl, Task& t) {
    const int wb = w / 4, nb = ceil4(n) / 4;
    int r = q;
    if (r < wb * nb) {   // dW_1[h][k] = sum d_1[h] y[k]
        const int hb = r / nb, kb = r % nb;
        t = Task{rl.d + 4 * hb, rl.y + 4 * kb, 4 * hb * n + 4 * kb, n, 4, (n - 4 * kb) < 4 ? (n - 4 * kb) : 4};
        return true;
    }
    r -= wb * nb;
    if (r < wb) {        // db_1
        t = Task{rl.d + 4 * r, rl.one, w * n + 4 * r, 1, 4, 1};
        return true;
    }
    r -= wb;
    for (int l = 1; l < L; ++l) {
        const int base = (int)layer_offset(n, w, l);
        if (r < wb * wb) {   // dW_{l+1}[h][k] = sum d_{l+1}[h] a_l[k]
            const int hb = r / wb, kb = r % wb;
            t = Task{rl.d + l * w + 4 * hb, rl.a + (l - 1) * w + 4 * kb, base + 4 * hb * w + 4 * kb, w, 4, 4};
            return true;
        }
        r -= wb * wb;
        if (r < wb) {
            t = Task{rl.d + l * w + 4 * r, rl.one, base + w * w + 4 * r, 1, 4, 1};
            return true;
        }
        r -= wb;
    }
    const int base = (int)layer_offset(n, w, L);
    if (r < nb * wb) {   // dW_out[i][h] = sum w[i] a_L[h]
        const int rb = r / wb, hb = r % wb;
        t = Task{rl.w + 4 * rb, rl.a + (L - 1) * w + 4 * hb, base + 4 * rb * w + 4 * hb, w, (n - 4 * rb) < 4 ? (n - 4 * rb) : 4, 4};
        return true;
    }
    r -= nb * wb;
    if (r < nb) {        // db_out
        t = Task{rl.w + 4 * r, rl.one, base + n * w + 4 * r, 1, (n - 4 * r) < 4 ? (n - 4 * r) : 4, 1};
        return true;
    }
    return false;
}

template <typename S>
__global__ __launch_bounds__(kThreads) void mlp_gen_vjp_kernel(MlpVjpParams p, int pts) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    S* rows = reinterpret_cast<S*>(smem_raw);
    const int n = p.n, w = p.width, L = p.nhid, kind = p.act;
    const VjRow rl(n, w, L);
    const int tid = threadIdx.x;
    const S* __restrict__ th = reinterpret_cast<const S*>(p.theta);
    const int split = kThreads / pts;
    const int pt = tid % pts, part = tid / pts;

    S acc[kMaxTasks][16];
    Task task[kMaxTasks];
    bool has[kMaxTasks];
#pragma unroll
    for (int k = 0; k < kMaxTasks; ++k) {
        has[k] = make_task(tid + kThreads * k, n, w, L, rl, task[k]);
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[k][e] = S(0);
    }

    const long long total = (long long)p.B * p.T;
    const long long chunks = (total + pts - 1) / pts;
    const S* __restrict__ yg = reinterpret_cast<const S*>(p.y);
    const S* __restrict__ ug = reinterpret_cast<const S*>(p.u);
    S* R = rows + (size_t)pt * rl.len;

    for (long long ch = blockIdx.x; ch < chunks; ch += gridDim.x) {
        // ---- phase A: forward and reverse sweep at every point of the chunk ----
        const long long gp = ch * pts + pt;
        const bool valid = gp < total;
        if (part == 0) {
            const long long b = valid ? gp / p.T : 0, j = valid ? gp % p.T : 0;
            for (int k = 0; k < ceil4(n); ++k) {
                S yv = S(0), wv = S(0);
                if (valid && k < n) {
                    yv = yg[gp * n + k];
                    const S ua = (j + 1 < p.T) ? ug[(b * (p.T - 1) + j) * n + k] : S(0);
                    const S ub = (j > 0) ? ug[(b * (p.T - 1) + j - 1) * n + k] : S(0);
                    wv = S(0.5) * (ua + ub);
                }
                R[rl.y + k] = yv;
                R[rl.w + k] = wv;
            }
            for (int k = 0; k < 4; ++k) R[rl.one + k] = (valid && k == 0) ? S(1) : S(0);
        }
        __syncthreads();
        {
            const S* __restrict__ W1 = th;
            const S* __restrict__ b1 = th + (long long)w * n;
            for (int h = part; h < w; h += split) {
                S pre = b1[h];
                for (int k = 0; k < n; ++k) pre += W1[h * n + k] * R[rl.y + k];
                S a, da;
                act_both<S>(kind, pre, a, da);
                R[rl.a + h] = a;
            }
        }
        __syncthreads();
        for (int l = 1; l < L; ++l) {
            const S* __restrict__ Wl = th + layer_offset(n, w, l);
            const S* __restrict__ bl = Wl + (long long)w * w;
            const S* ain = R + rl.a + (l - 1) * w;
            for (int h = part; h < w; h += split) {
                S pre = bl[h];
                for (int k = 0; k < w; k += 4) {
                    S wv[4], av[4];
                    vload<S, 4>(wv, Wl + (long long)h * w + k);
                    vload<S, 4>(av, ain + k);
                    pre += wv[0] * av[0] + wv[1] * av[1] + wv[2] * av[2] + wv[3] * av[3];
                }
                S a, da;
                act_both<S>(kind, pre, a, da);
                R[rl.a + l * w + h] = a;
            }
            __syncthreads();
        }
        // d_L = (W_out^T w) s'(.), then d_l = (W_{l+1}^T d_{l+1}) s'(.) down to l = 1
        {
            const S* __restrict__ Wo = th + layer_offset(n, w, L);
            for (int h = part; h < w; h += split) {
                S s = S(0);
                for (int r = 0; r < n; ++r) s += Wo[(long long)r * w + h] * R[rl.w + r];
                R[rl.d + (L - 1) * w + h] = s * dact_from_value<S>(kind, R[rl.a + (L - 1) * w + h]);
            }
        }
        __syncthreads();
        for (int l = L - 1; l >= 1; --l) {
            const S* __restrict__ Wn = th + layer_offset(n, w, l);   // weights of hidden layer l + 1 (0-based l)
            const S* dn = R + rl.d + l * w;
            for (int h = part; h < w; h += split) {
                S s = S(0);
                for (int m = 0; m < w; m += 4) {
                    S dv[4];
                    vload<S, 4>(dv, dn + m);
                    s += Wn[(long long)m * w + h] * dv[0] + Wn[(long long)(m + 1) * w + h] * dv[1] +
                         Wn[(long long)(m + 2) * w + h] * dv[2] + Wn[(long long)(m + 3) * w + h] * dv[3];
                }
                R[rl.d + (l - 1) * w + h] = s * dact_from_value<S>(kind, R[rl.a + (l - 1) * w + h]);
            }
            __syncthreads();
        }

        // ---- phase B: outer products summed over the points of the chunk ----
#pragma unroll
        for (int k = 0; k < kMaxTasks; ++k) {
            if (has[k]) {
                for (int q = 0; q < pts; ++q) {
                    const S* Rq = rows + (size_t)q * rl.len;
                    S uv[4], vv[4];
                    vload<S, 4>(uv, Rq + task[k].uo);
                    vload<S, 4>(vv, Rq + task[k].vo);
#pragma unroll
                    for (int a = 0; a < 4; ++a)
#pragma unroll
                        for (int c = 0; c < 4; ++c) acc[k][a * 4 + c] += uv[a] * vv[c];
                }
            }
        }
        __syncthreads();
    }

    S* __restrict__ out = reinterpret_cast<S*>(p.partial) + (size_t)blockIdx.x * (size_t)gen_theta_len(n, w, L);
#pragma unroll
    for (int k = 0; k < kMaxTasks; ++k) {
        if (has[k]) {
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (a < task[k].nr && c < task[k].nc) out[task[k].out + a * task[k].rs + c] = acc[k][a * 4 + c];
        }
    }
}

template <typename S>
int vj_points(int n, int w, int L, size_t* bytes) {
    const VjRow rl(n, w, L);
    int pts = 64;
    while (pts > 8 && (size_t)pts * rl.len * sizeof(S) > (size_t)64 * 1024) pts >>= 1;
    *bytes = (size_t)pts * rl.len * sizeof(S);
    return pts;
}

template <typename S>
hipError_t launch_vj(const MlpVjpParams& p, hipStream_t s) {
    size_t bytes = 0;
    const int pts = vj_points<S>(p.n, p.width, p.nhid, &bytes);
    if (bytes > (size_t)150 * 1024) return hipErrorInvalidValue;
    if (gen_task_count(p.n, p.width, p.nhid) > kThreads * kMaxTasks) return hipErrorInvalidValue;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(mlp_gen_vjp_kernel<S>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((mlp_gen_vjp_kernel<S>), dim3((unsigned)p.blocks), dim3(kThreads), bytes, s, p, pts);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_partial_reduce(sizeof(S) == 4 ? 0 : 1, p.partial, p.dtheta, gen_theta_len(p.n, p.width, p.nhid), p.blocks, s);
}

}  // namespace

bool mlp_general_supported(int n, int width, int nhid, int act) {
    return n >= 1 && n <= 8 && width >= 4 && width <= 64 && (width & 3) == 0 && nhid >= 1 && nhid <= 5 &&
           (act == 0 || act == 1) && gen_task_count(n, width, nhid) <= kThreads * kMaxTasks;
}

int mlp_general_vjp_blocks(int dtype, int n, int width, int nhid, long long points) {
    size_t bytes = 0;
    const int pts = dtype == 0 ? vj_points<float>(n, width, nhid, &bytes) : vj_points<double>(n, width, nhid, &bytes);
    long long chunks = (points + pts - 1) / pts;
    if (chunks > 512) chunks = 512;
    if (chunks < 1) chunks = 1;
    return (int)chunks;
}

hipError_t launch_mlp_general_funceval(int dtype, const MlpParams& p, hipStream_t s) {
    if (!mlp_general_supported(p.n, p.width, p.nhid, p.act)) return hipErrorInvalidValue;
    // fp32, n = 8, width 32 or 64: on the matrix cores (DEER_MLP_MFMA=0 keeps the vector-ALU kernel)
    const char* e = getenv("DEER_MLP_MFMA");   // (read per call: the tests run both kernels in one process)
    const bool mfma = !(e && *e && atoi(e) == 0);
    if (mfma && fe_mfma_supported(dtype, p.n, p.width, p.nhid)) return p.width == 32 ? launch_fe_mfma_w<2>(p, s) : launch_fe_mfma_w<4>(p, s);
    return dtype == 0 ? launch_fe<float>(p, s) : launch_fe<double>(p, s);
}

hipError_t launch_mlp_general_vjp(int dtype, const MlpVjpParams& p, hipStream_t s) {
    if (!mlp_general_supported(p.n, p.width, p.nhid, p.act) || p.T < 2) return hipErrorInvalidValue;
    const char* e = getenv("DEER_MLP_MFMA");
    if (!(e && *e && atoi(e) == 0) && fe_mfma_supported(dtype, p.n, p.width, p.nhid) && p.blocks >= 1) {
        // the partial region holds p.blocks * 4 rows: that many wavefront rows at most, and one block per CU by its LDS
        const int blocks = p.blocks < 256 ? p.blocks : 256;
        hipError_t err = p.width == 32 ? launch_vj_mfma_w<2>(p, blocks, s) : launch_vj_mfma_w<4>(p, blocks, s);
        if (err != hipSuccess) return err;
        return launch_partial_reduce(0, p.partial, p.dtheta, gen_theta_len(p.n, p.width, p.nhid), blocks * 4, s);
    }
    return dtype == 0 ? launch_vj<float>(p, s) : launch_vj<double>(p, s);
}

}  // namespace deer
