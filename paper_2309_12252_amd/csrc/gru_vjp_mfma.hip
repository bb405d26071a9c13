// Vector-Jacobian product of the GRU cell on the matrix cores (fp32, n = 16 or 32, d <= 16): the same
// quantities as gru_vjp_kernel (Sec. 3.1.1 eq. 7, outer bracket) -- dL/dx per position, dL/dy0, and partial
// rows of dL/dtheta for the fixed-order reduction -- with every contraction as 16 x 16 x 4 MFMAs.
//
// A wavefront takes 16 consecutive positions as the column tile (lane = 16 g + c: column c, lane group g).
//   1. gate pre-activations  a_r, a_z = U h + W x + b,  q = U_c h + b_hc,  a_c' = W_c x + b_c : rows of the
//      weights are the A operands (U resident in registers, W read from LDS), h and x of the 16 positions
//      the B operands (lane (g, c) supplies entry 4m + g of position c in k-step m);
//   2. cotangents in accumulator layout (lane (g, c): rows 4g .. 4g+3 of a 16-row block, position c), where
//      lam and h arrive as 16-byte loads:  dac = lam (1 - z)(1 - c^2), daz = lam (h - c) z (1 - z),
//      dq = dac r, dar = dac q r (1 - r);
//   3. dL/dx = sum over gates of W_g^T d_g straight from those registers: k-step v takes the rows
//      {16 I + 4g + v}, and the A operand's columns are picked to match;
//   4. dU_g += d_g H^T and dW_g += d_g X^T have the positions on the k index: the cotangent blocks cross a
//      wavefront-private LDS tile to become A operands, h and x are read a second time as B operands
//      (lane (g, j): entry j of position 4m + g);
//   5. the bias sums stay per lane and are added over the 16 columns once, at the end.
// Accumulators live in registers over all passes; every wavefront writes one partial row.
#include "deer_common.h"

namespace deer {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kDP = 16;   // inputs are padded to 16 columns (zeros)
constexpr int kLD = 17;   // LDS row stride of the 16-column blocks

typedef float acc4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ acc4 mfma(float a, float b, acc4 c) { return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0); }

template <int N>
__global__ __launch_bounds__(kThreads, N == 32 ? 2 : 1) void gru_vjp_mfma_kernel(GruVjpParams p) {
    constexpr int NB = N / 16;   // 16-row blocks
    constexpr int KH = N / 4;    // k-steps over the state
    extern __shared__ __align__(16) unsigned char smem_raw[];
    float* sW = reinterpret_cast<float*>(smem_raw);   // [3N][kLD] input weights, columns >= d zero
    float* sB = sW + 3 * N * kLD;                      // [4N] biases r | z | c | hc
    float* sD = sB + 4 * N;                            // [kWaves][5][N][kLD] cotangent blocks (dar, daz, dac, dq, z lam)
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, c = lane & 15;
    const int d = p.d;
    const float* __restrict__ theta = reinterpret_cast<const float*>(p.theta);
    const float* __restrict__ U = theta + 3 * N * d;
    const float* __restrict__ bias = U + 3 * N * N;
    const float* __restrict__ x = reinterpret_cast<const float*>(p.x);
    const float* __restrict__ y0 = reinterpret_cast<const float*>(p.y0);
    const float* __restrict__ y = reinterpret_cast<const float*>(p.y);
    const float* __restrict__ lam = reinterpret_cast<const float*>(p.lam);
    float* __restrict__ dx = reinterpret_cast<float*>(p.dx);
    float* __restrict__ dy0 = reinterpret_cast<float*>(p.dy0);

    for (int q = tid; q < 3 * N * kLD; q += kThreads) {
        const int row = q / kLD, col = q - row * kLD;
        sW[q] = (col < d) ? theta[row * d + col] : 0.0f;
    }
    for (int q = tid; q < 4 * N; q += kThreads) sB[q] = bias[q];
    // hidden-to-hidden weights as A operands: uA[gate][I][m] = U_gate[16 I + c][4 m + g]
    float uA[3][NB][KH];
#pragma unroll
    for (int a = 0; a < 3; ++a)
#pragma unroll
        for (int I = 0; I < NB; ++I)
#pragma unroll
            for (int m = 0; m < KH; ++m) uA[a][I][m] = U[(a * N + 16 * I + c) * N + 4 * m + g];
    __syncthreads();

    float* myD = sD + (size_t)wave * 5 * N * kLD;
    acc4 accU[3][NB][NB], accW[3][NB], accB[4][NB];
#pragma unroll
    for (int a = 0; a < 3; ++a)
#pragma unroll
        for (int I = 0; I < NB; ++I) {
            accW[a][I] = acc4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int J = 0; J < NB; ++J) accU[a][I][J] = acc4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int I = 0; I < NB; ++I) accB[a][I] = acc4{0.f, 0.f, 0.f, 0.f};

    const long long total = (long long)p.B * p.T;
    const long long tiles = (total + 15) / 16;
    // state in front of position s (y0 at the first position of a sequence); positions past the end read position 0
    const bool narrow = total < (1LL << 31);   // 32-bit division is several times cheaper than the 64-bit one
    auto hrow = [&](long long s) -> const float* {
        const long long sc = s < total ? s : 0;
        const long long bi = narrow ? (long long)((unsigned)sc / (unsigned)p.T) : sc / p.T;
        return (sc - bi * p.T == 0) ? (y0 + bi * N) : (y + (sc - 1) * N);
    };

    // operands of one tile, in the layouts described above
    struct Operands {
        float hB[KH], xB[4];
        acc4 lamA[NB], hA[NB];
        float hK[4][NB], xK[4];
    };
    auto request = [&](long long tile, Operands& o) {
        const long long s0 = tile * 16;
        const long long sc = s0 + c;            // this lane's column position
        const bool live = sc < total;
        const long long scl = live ? sc : 0;
        const float* hc = hrow(sc);
#pragma unroll
        for (int m = 0; m < KH; ++m) o.hB[m] = hc[4 * m + g];
#pragma unroll
        for (int m = 0; m < 4; ++m) o.xB[m] = (4 * m + g < d) ? x[scl * d + 4 * m + g] : 0.0f;
#pragma unroll
        for (int I = 0; I < NB; ++I) {
            const float4 lv = *reinterpret_cast<const float4*>(lam + scl * N + 16 * I + 4 * g);
            const float4 hv = *reinterpret_cast<const float4*>(hc + 16 * I + 4 * g);
            o.lamA[I] = live ? acc4{lv.x, lv.y, lv.z, lv.w} : acc4{0.f, 0.f, 0.f, 0.f};
            o.hA[I] = acc4{hv.x, hv.y, hv.z, hv.w};
        }
        // second view for the products over positions: lane (g, j) reads entry j of position 4 m + g
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const long long sp = s0 + 4 * m + g;
            const float* hp = hrow(sp);
#pragma unroll
            for (int J = 0; J < NB; ++J) o.hK[m][J] = hp[16 * J + c];
            o.xK[m] = (c < d && sp < total) ? x[sp * d + c] : 0.0f;
        }
    };
    const long long tstride = (long long)gridDim.x * kWaves;
    for (long long tile = (long long)blockIdx.x * kWaves + wave; tile < tiles; tile += tstride) {
        const long long s0 = tile * 16;
        const long long sc = s0 + c;
        const bool live = sc < total;
        // (requesting the next tile's operands one pass ahead costs a wavefront of occupancy and measured slower)
        Operands o;
        request(tile, o);
        const float (&hB)[KH] = o.hB;
        const float (&xB)[4] = o.xB;
        const acc4 (&lamA)[NB] = o.lamA;
        const acc4 (&hA)[NB] = o.hA;
        const float (&hK)[4][NB] = o.hK;
        const float (&xK)[4] = o.xK;

        // ---- 1. gates ----
        acc4 dar[NB], daz[NB], dac[NB], dq[NB];
#pragma unroll
        for (int I = 0; I < NB; ++I) {
            acc4 ar, az, aq, ac;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                ar[v] = sB[16 * I + 4 * g + v];
                az[v] = sB[N + 16 * I + 4 * g + v];
                ac[v] = sB[2 * N + 16 * I + 4 * g + v];
                aq[v] = sB[3 * N + 16 * I + 4 * g + v];
            }
#pragma unroll
            for (int m = 0; m < KH; ++m) {
                ar = mfma(uA[0][I][m], hB[m], ar);
                az = mfma(uA[1][I][m], hB[m], az);
                aq = mfma(uA[2][I][m], hB[m], aq);
            }
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                ar = mfma(sW[(16 * I + c) * kLD + 4 * m + g], xB[m], ar);
                az = mfma(sW[(N + 16 * I + c) * kLD + 4 * m + g], xB[m], az);
                ac = mfma(sW[(2 * N + 16 * I + c) * kLD + 4 * m + g], xB[m], ac);
            }
            // ---- 2. cotangents ----
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float r = feed_sigmoid(ar[v]), z = feed_sigmoid(az[v]);
                const float cc = feed_tanh(ac[v] + r * aq[v]);
                const float lm = lamA[I][v], hi = hA[I][v];
                const float dcand = lm * (1.0f - z);
                const float vac = dcand * (1.0f - cc * cc);
                dac[I][v] = vac;
                daz[I][v] = lm * (hi - cc) * z * (1.0f - z);
                dq[I][v] = vac * r;
                dar[I][v] = vac * aq[v] * r * (1.0f - r);
                const int row = 16 * I + 4 * g + v;
                myD[(0 * N + row) * kLD + c] = dar[I][v];
                myD[(1 * N + row) * kLD + c] = daz[I][v];
                myD[(2 * N + row) * kLD + c] = dac[I][v];
                myD[(3 * N + row) * kLD + c] = dq[I][v];
                myD[(4 * N + row) * kLD + c] = z * lm;
            }
            accB[0][I] += dar[I];
            accB[1][I] += daz[I];
            accB[2][I] += dac[I];
            accB[3][I] += dq[I];
        }

        // ---- 3. dL/dx: rows (input index) 4g + v of position c ----
        if (dx) {
            acc4 ax = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int I = 0; I < NB; ++I)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    // k-step v: lane group g supplies row 16 I + 4g + v of the cotangent; A[i = c][k = g] = W[that row][c]
                    const int row = 16 * I + 4 * g + v;
                    ax = mfma(sW[row * kLD + c], dar[I][v], ax);
                    ax = mfma(sW[(N + row) * kLD + c], daz[I][v], ax);
                    ax = mfma(sW[(2 * N + row) * kLD + c], dac[I][v], ax);
                }
            if (live) {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (4 * g + v < d) dx[sc * d + 4 * g + v] = ax[v];
            }
        }

        // ---- 4. dU += d H^T, dW += d X^T (k = positions) ----
#pragma unroll
        for (int I = 0; I < NB; ++I)
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                // A[i = c -> row 16 I + c][k = g -> position 4 m + g]
                const int at = (16 * I + c) * kLD + 4 * m + g;
                const float tr = myD[0 * N * kLD + at], tz = myD[1 * N * kLD + at];
                const float tc = myD[2 * N * kLD + at], tq = myD[3 * N * kLD + at];
#pragma unroll
                for (int J = 0; J < NB; ++J) {
                    accU[0][I][J] = mfma(tr, hK[m][J], accU[0][I][J]);
                    accU[1][I][J] = mfma(tz, hK[m][J], accU[1][I][J]);
                    accU[2][I][J] = mfma(tq, hK[m][J], accU[2][I][J]);
                }
                accW[0][I] = mfma(tr, xK[m], accW[0][I]);
                accW[1][I] = mfma(tz, xK[m], accW[1][I]);
                accW[2][I] = mfma(tc, xK[m], accW[2][I]);
            }

        // ---- dL/dy0 = J_1^T lam_1 at the first position of a sequence (rare: one column of a few tiles) ----
        if (dy0) {
            for (int c0 = 0; c0 < 16; ++c0) {
                const long long sp = s0 + c0;
                if (sp >= total) break;
                const long long bi = sp / p.T;
                if (sp - bi * p.T != 0) continue;
                if (lane < N) {
                    float s = myD[(4 * N + lane) * kLD + c0];   // z_j lam_j
                    for (int i = 0; i < N; ++i) {
                        s += U[(0 * N + i) * N + lane] * myD[(0 * N + i) * kLD + c0];
                        s += U[(1 * N + i) * N + lane] * myD[(1 * N + i) * kLD + c0];
                        s += U[(2 * N + i) * N + lane] * myD[(3 * N + i) * kLD + c0];
                    }
                    dy0[bi * N + lane] = s;
                }
            }
        }
    }

    // ---- partial row of this wavefront ----
    const long long P = 3LL * N * d + 3LL * N * N + 4LL * N;
    float* __restrict__ prow = reinterpret_cast<float*>(p.partial) + ((long long)blockIdx.x * kWaves + wave) * P;
    float* pU = prow + 3LL * N * d;
    float* pb = pU + 3LL * N * N;
#pragma unroll
    for (int a = 0; a < 3; ++a)
#pragma unroll
        for (int I = 0; I < NB; ++I)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = a * N + 16 * I + 4 * g + v;
                if (c < d) prow[(long long)row * d + c] = accW[a][I][v];
#pragma unroll
                for (int J = 0; J < NB; ++J) pU[(long long)row * N + 16 * J + c] = accU[a][I][J][v];
            }
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int I = 0; I < NB; ++I)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float s = accB[a][I][v];
                s += __shfl_xor(s, 1);
                s += __shfl_xor(s, 2);
                s += __shfl_xor(s, 4);
                s += __shfl_xor(s, 8);
                if (c == 0) pb[a * N + 16 * I + 4 * g + v] = s;
            }
}

template <int N>
hipError_t launch_n(const GruVjpParams& p, hipStream_t s) {
    const size_t shmem = ((size_t)3 * N * kLD + 4 * N + (size_t)kWaves * 5 * N * kLD) * sizeof(float);
    hipLaunchKernelGGL((gru_vjp_mfma_kernel<N>), dim3((unsigned)p.blocks), dim3(kThreads), shmem, s, p);
    return hipGetLastError();
}

}  // namespace

bool gru_vjp_mfma_supported(int dtype, int n, int d) { return dtype == 0 && (n == 16 || n == 32) && d >= 1 && d <= kDP; }

// launches the kernel only; the caller adds the partial rows (blocks * 4 of them) with launch_partial_reduce
hipError_t launch_gru_vjp_mfma(const GruVjpParams& p, hipStream_t s) {
    if (!gru_vjp_mfma_supported(0, p.n, p.d)) return hipErrorInvalidValue;
    return p.n == 16 ? launch_n<16>(p, s) : launch_n<32>(p, s);
}

}  // namespace deer
