// Backward derivative of the MLP vector field on the matrix cores (fp32, n = 8, width 16, 32 or 64): the same
// sums as mlp_vjp_kernel (Sec. 3.1.1 eq. 7, outer bracket, ODE form) -- dL/dtheta = sum over grid points j of
// (df/dtheta)(y_j)^T w_j, w_j = (u_j + u_{j-1}) / 2 -- with every contraction as 16 x 16 x 4 MFMAs.
//
// A wavefront takes 16 consecutive grid points as the column tile (lane = 16 g + c: column c, lane group g).
//   1. forward: Z1 = W1 Y + b1, A1 = tanh Z1, Z2 = W2 A1 + b2, A2 = tanh Z2.  Weight rows are the A operands
//      (resident in registers), y the B operand of the first product; A1 stays in its accumulators and is the B operand
//      of the second product (k-step v takes the rows {4g + v} of a 16-row block, the A operand's columns are
//      picked to match);
//   2. reverse: D2 = (W3^T w) (1 - A2^2), D1 = (W2^T D2) (1 - A1^2), the same way with the weights read down
//      their columns; w arrives in accumulator layout as 16-byte loads;
//   3. dW3 += w A2^T, dW2 += D2 A1^T, dW1 += D1 Y^T have the grid points on the k index: w, A2, D2, A1, D1 cross
//      a wavefront-private LDS tile (lane (g, i) reads entry i of point 4m + g), y is read a second time in that
//      layout from memory;
//   4. the bias sums stay per lane and are added over the 16 columns once, at the end.
// Accumulators live in registers over all passes; every wavefront writes one partial row.
#include "deer_common.h"

namespace deer {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kN = 8;     // state size
constexpr int kLD = 17;   // LDS row stride of the 16-column blocks

typedef float acc4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ acc4 mfma(float a, float b, acc4 c) { return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0); }

// rows of the per-wavefront LDS tile: w (16, the upper 8 zero) | a2 | d2 | a1 | d1
template <int WB>
struct Tile {
    static constexpr int W = 16 * WB;
    static constexpr int u = 0, a2 = 16, d2 = 16 + W, a1 = 16 + 2 * W, d1 = 16 + 3 * W, rows = 16 + 4 * W;
};

template <int WB>
__global__ __launch_bounds__(kThreads) void mlp_vjp_mfma_kernel(MlpVjpParams p) {
    constexpr int W = 16 * WB;
    using T = Tile<WB>;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    float* sD = reinterpret_cast<float*>(smem_raw);    // [kWaves][T::rows][kLD]
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, c = lane & 15;
    const float* __restrict__ th = reinterpret_cast<const float*>(p.theta);
    constexpr int oW1 = 0, ob1 = W * kN, oW2 = ob1 + W, ob2 = oW2 + W * W, oW3 = ob2 + W, ob3 = oW3 + kN * W;
    const float* __restrict__ yg = reinterpret_cast<const float*>(p.y);
    const float* __restrict__ ug = reinterpret_cast<const float*>(p.u);

    // every weight as the A operand of the product it enters, resident in registers (an operand read from LDS in
    // front of each MFMA leaves the matrix cores waiting for it)
    float w1A[WB][2], w2A[WB][WB][4], w2T[WB][WB][4], w3T[WB][4];
    acc4 b1A[WB], b2A[WB];
#pragma unroll
    for (int I = 0; I < WB; ++I) {
#pragma unroll
        for (int m = 0; m < 2; ++m) w1A[I][m] = th[oW1 + (16 * I + c) * kN + 4 * m + g];
#pragma unroll
        for (int K = 0; K < WB; ++K)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                w2A[I][K][v] = th[oW2 + (16 * I + c) * W + 16 * K + 4 * g + v];
                w2T[I][K][v] = th[oW2 + (16 * K + 4 * g + v) * W + 16 * I + c];
            }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            w3T[I][v] = (g < 2) ? th[oW3 + (4 * g + v) * W + 16 * I + c] : 0.0f;   // rows 8..15 of the padded block
            b1A[I][v] = th[ob1 + 16 * I + 4 * g + v];
            b2A[I][v] = th[ob2 + 16 * I + 4 * g + v];
        }
    }

    float* myD = sD + (size_t)wave * T::rows * kLD;
    // the upper half of the w block never changes
    for (int q = lane; q < 8 * kLD; q += 64) myD[(T::u + 8) * kLD + q] = 0.0f;

    acc4 accW2[WB][WB], accW1[WB], accW3[WB], accB1[WB], accB2[WB], accB3;
#pragma unroll
    for (int I = 0; I < WB; ++I) {
        accW1[I] = acc4{0.f, 0.f, 0.f, 0.f};
        accW3[I] = acc4{0.f, 0.f, 0.f, 0.f};
        accB1[I] = acc4{0.f, 0.f, 0.f, 0.f};
        accB2[I] = acc4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int J = 0; J < WB; ++J) accW2[I][J] = acc4{0.f, 0.f, 0.f, 0.f};
    }
    accB3 = acc4{0.f, 0.f, 0.f, 0.f};

    const long long total = (long long)p.B * p.T;
    const long long tiles = (total + 15) / 16;
    const long long tstride = (long long)gridDim.x * kWaves;
    // operands of one tile
    struct Operands {
        float yB[2];    // y as B operand of the first product: entry 4m + g of point c
        float yK[4];    // y as B operand of dW1: entry c of point 4m + g
        float4 ua, ub;  // u_j and u_{j-1}, entries 4g .. 4g+3 of point c (g < 2)
    };
    auto request = [&](long long tile, Operands& o) {
        const long long s0 = tile * 16;
        const long long sc = s0 + c;
        const bool live = sc < total;
        const long long scl = live ? sc : 0;
#pragma unroll
        for (int m = 0; m < 2; ++m) o.yB[m] = live ? yg[scl * kN + 4 * m + g] : 0.0f;
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const long long sp = s0 + 4 * m + g;
            o.yK[m] = (c < kN && sp < total) ? yg[sp * kN + c] : 0.0f;
        }
        o.ua = float4{0.f, 0.f, 0.f, 0.f};
        o.ub = float4{0.f, 0.f, 0.f, 0.f};
        if (live && g < 2) {
            const long long b = sc / p.T, j = sc - b * p.T;
            if (j + 1 < p.T) o.ua = *reinterpret_cast<const float4*>(ug + (b * (p.T - 1) + j) * kN + 4 * g);
            if (j > 0) o.ub = *reinterpret_cast<const float4*>(ug + (b * (p.T - 1) + j - 1) * kN + 4 * g);
        }
    };
    // software pipeline: the (few) operands of the next tile are requested before the current one is worked on
    Operands nxt;
    {
        const long long first = (long long)blockIdx.x * kWaves + wave;
        if (first < tiles) request(first, nxt);
    }
    for (long long tile = (long long)blockIdx.x * kWaves + wave; tile < tiles; tile += tstride) {
        const bool live = tile * 16 + c < total;
        const Operands o = nxt;
        if (tile + tstride < tiles) request(tile + tstride, nxt);
        const float (&yB)[2] = o.yB;
        const float (&yK)[4] = o.yK;
        // w in accumulator layout (zero for g >= 2 and past the end)
        const acc4 wA = {0.5f * (o.ua.x + o.ub.x), 0.5f * (o.ua.y + o.ub.y), 0.5f * (o.ua.z + o.ub.z), 0.5f * (o.ua.w + o.ub.w)};

        // ---- 1. forward ----
        acc4 a1[WB], a2[WB];
#pragma unroll
        for (int I = 0; I < WB; ++I) {
            acc4 z = b1A[I];
#pragma unroll
            for (int m = 0; m < 2; ++m) z = mfma(w1A[I][m], yB[m], z);
#pragma unroll
            for (int v = 0; v < 4; ++v) a1[I][v] = live ? feed_tanh(z[v]) : 0.0f;
        }
#pragma unroll
        for (int I = 0; I < WB; ++I) {
            acc4 z = b2A[I];
#pragma unroll
            for (int K = 0; K < WB; ++K)
#pragma unroll
                for (int v = 0; v < 4; ++v) z = mfma(w2A[I][K][v], a1[K][v], z);
#pragma unroll
            for (int v = 0; v < 4; ++v) a2[I][v] = live ? feed_tanh(z[v]) : 0.0f;
        }

        // ---- 2. reverse ----
        acc4 d1[WB], d2[WB];
#pragma unroll
        for (int I = 0; I < WB; ++I) {
            acc4 z = {0.f, 0.f, 0.f, 0.f};
            // k-step v: lane group g supplies entry 4g + v of w (zero from g = 2 on); A[i = c][k = g] = W3[4g + v][16 I + c]
#pragma unroll
            for (int v = 0; v < 4; ++v) z = mfma(w3T[I][v], wA[v], z);
#pragma unroll
            for (int v = 0; v < 4; ++v) d2[I][v] = z[v] * (1.0f - a2[I][v] * a2[I][v]);
        }
#pragma unroll
        for (int I = 0; I < WB; ++I) {
            acc4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int K = 0; K < WB; ++K)
#pragma unroll
                for (int v = 0; v < 4; ++v) z = mfma(w2T[I][K][v], d2[K][v], z);
#pragma unroll
            for (int v = 0; v < 4; ++v) d1[I][v] = z[v] * (1.0f - a1[I][v] * a1[I][v]);
        }

        // ---- 3. the five fields cross to the layout with the points on the k index ----
        if (g < 2) {
#pragma unroll
            for (int v = 0; v < 4; ++v) myD[(T::u + 4 * g + v) * kLD + c] = wA[v];
        }
#pragma unroll
        for (int I = 0; I < WB; ++I)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = 16 * I + 4 * g + v;
                myD[(T::a2 + row) * kLD + c] = a2[I][v];
                myD[(T::d2 + row) * kLD + c] = d2[I][v];
                myD[(T::a1 + row) * kLD + c] = a1[I][v];
                myD[(T::d1 + row) * kLD + c] = d1[I][v];
            }
        accB3 += wA;
#pragma unroll
        for (int I = 0; I < WB; ++I) {
            accB2[I] += d2[I];
            accB1[I] += d1[I];
        }
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            // A[i = c][k = g -> point 4m + g], B[k = g -> point 4m + g][j = c]
            const int at = c * kLD + 4 * m + g;
            const float tu = myD[T::u * kLD + at];
            float ta2[WB], td2[WB], ta1[WB], td1[WB];
#pragma unroll
            for (int I = 0; I < WB; ++I) {
                ta2[I] = myD[(T::a2 + 16 * I) * kLD + at];
                td2[I] = myD[(T::d2 + 16 * I) * kLD + at];
                ta1[I] = myD[(T::a1 + 16 * I) * kLD + at];
                td1[I] = myD[(T::d1 + 16 * I) * kLD + at];
            }
#pragma unroll
            for (int I = 0; I < WB; ++I) {
                accW3[I] = mfma(tu, ta2[I], accW3[I]);
                accW1[I] = mfma(td1[I], yK[m], accW1[I]);
#pragma unroll
                for (int J = 0; J < WB; ++J) accW2[I][J] = mfma(td2[I], ta1[J], accW2[I][J]);
            }
        }
    }

    // ---- partial row of this wavefront ----
    constexpr long long P = ob3 + kN;
    float* __restrict__ prow = reinterpret_cast<float*>(p.partial) + ((long long)blockIdx.x * kWaves + wave) * P;
#pragma unroll
    for (int I = 0; I < WB; ++I)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = 16 * I + 4 * g + v;
            if (c < kN) prow[oW1 + row * kN + c] = accW1[I][v];
#pragma unroll
            for (int J = 0; J < WB; ++J) prow[oW2 + row * W + 16 * J + c] = accW2[I][J][v];
            if (g < 2) prow[oW3 + (4 * g + v) * W + 16 * I + c] = accW3[I][v];
            float s1 = accB1[I][v], s2 = accB2[I][v];
#pragma unroll
            for (int o = 1; o < 16; o <<= 1) {
                s1 += __shfl_xor(s1, o);
                s2 += __shfl_xor(s2, o);
            }
            if (c == 0) { prow[ob1 + row] = s1; prow[ob2 + row] = s2; }
        }
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        float s = accB3[v];
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) s += __shfl_xor(s, o);
        if (c == 0 && g < 2) prow[ob3 + 4 * g + v] = s;
    }
}

template <int WB>
size_t shmem_bytes() {
    return (size_t)kWaves * Tile<WB>::rows * kLD * sizeof(float);
}

template <int WB>
hipError_t launch_w(const MlpVjpParams& p, hipStream_t s) {
    const size_t bytes = shmem_bytes<WB>();
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(mlp_vjp_mfma_kernel<WB>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((mlp_vjp_mfma_kernel<WB>), dim3((unsigned)p.blocks), dim3(kThreads), bytes, s, p);
    return hipGetLastError();
}

}  // namespace

bool mlp_vjp_mfma_supported(int dtype, int n, int width) { return dtype == 0 && n == kN && (width == 16 || width == 32 || width == 64); }

// launches the kernel only; the caller adds the partial rows (blocks * 4 of them) with launch_partial_reduce
hipError_t launch_mlp_vjp_mfma(const MlpVjpParams& p, hipStream_t s) {
    if (!mlp_vjp_mfma_supported(0, p.n, p.width) || p.T < 2 || p.blocks < 1) return hipErrorInvalidValue;
    return p.width == 16 ? launch_w<1>(p, s) : (p.width == 32 ? launch_w<2>(p, s) : launch_w<4>(p, s));
}

}  // namespace deer
