// Backward derivative of the MLP vector field over a whole trajectory (Sec. 3.1.1 eq. 7, outer bracket,
// for the ODE form): dL/dtheta = sum over grid points j of (df/dtheta)(y_j)^T w_j with
// w_j = (u_j + u_{j-1}) / 2, u_i = dt phi1(X_i)^T lam_{i+1} from the dual discretisation (u_{-1} = u_{T-1} = 0).
//
// Field: f(y) = W3 tanh(W2 tanh(W1 y + b1) + b2) + b3; theta = W1[w,n], b1[w], W2[w,w], b2[w], W3[n,w], b3[n].
// Reverse sweep at one point: a1 = tanh(W1 y + b1), a2 = tanh(W2 a1 + b2),
//   d2 = (W3^T w) (1 - a2^2),  d1 = (W2^T d2) (1 - a1^2),
//   dW3 += w a2^T, db3 += w, dW2 += d2 a1^T, db2 += d2, dW1 += d1 y^T, db1 += d1.
//
// Work split.  A block of 256 threads takes chunks of PTS grid points (grid-stride).  Phase A: the hidden
// units of a layer are dealt out to 256 / PTS threads per point; every thread writes its activations into
// the point's row in LDS (point-major: a1 | a2 | d1 | d2 | y | w | 1).  Phase B: the outer products are summed
// over the points in 4 x 4 register blocks -- a task is four entries of one field of the row times four
// entries of another (the trailing 1 gives the bias gradients) -- by two thread groups that take the even
// and the odd points.  Accumulators stay in registers across chunks; at the end every group writes one
// partial row, and a second kernel adds the rows in a fixed order, so the result is run-to-run identical.
#include "deer_common.h"

namespace deer {

namespace {

constexpr int kThreads = 256;
constexpr int kMaxTasks = 3;   // 4 x 4 blocks per thread (width 64: 354 tasks over 128 threads)

// fp32: hardware exp2 and reciprocal (absolute error below 3e-7)
__device__ __forceinline__ float tanh_(float a) { return feed_tanh(a); }
__device__ __forceinline__ double tanh_(double a) { return tanh(a); }

__host__ __device__ inline int ceil4(int v) { return (v + 3) & ~3; }

// offsets inside a point's row, in scalars
struct RowLayout {
    int a1, a2, d1, d2, y, w, one, len;
    __host__ __device__ RowLayout(int n, int width) {
        a1 = 0; a2 = width; d1 = 2 * width; d2 = 3 * width;
        y = 4 * width; w = y + ceil4(n); one = w + ceil4(n);
        len = one + 4;       // "1" padded to four entries
        // row length = 4 (mod 32) words: the 16-byte reads of consecutive points then fall on different banks
        while ((len & 31) != 4) len += 4;
    }
};
// offsets of the staged weights in LDS: W1, b1, W2, b2, W3^T, W2^T
struct WeightLayout {
    int W1, b1, W2, b2, W3T, W2T, len;
    __host__ __device__ WeightLayout(int n, int width) {
        W1 = 0; b1 = W1 + width * n; W2 = b1 + width; b2 = W2 + width * width;
        W3T = b2 + width; W2T = W3T + width * n; len = W2T + width * width;
    }
};

// One 4 x 4 task: rows of field U (offset uo) times columns of field V (offset vo); out: parameter offset of
// entry (0,0), strides, and how many rows / columns are real.
struct Task {
    int uo, vo, out, rs, nr, nc;
};

// task number q for state size n and hidden width w (see the work split above); false past the last task
__device__ __forceinline__ bool make_task(int q, int n, int w, const RowLayout& rl, Task& t) {
    const int wb = w / 4, nb = ceil4(n) / 4;
    const int oW1 = 0, ob1 = w * n, oW2 = ob1 + w, ob2 = oW2 + w * w, oW3 = ob2 + w, ob3 = oW3 + n * w;
    int r = q;
    if (r < wb * nb) {   // dW1[h][k] = sum d1[h] y[k]
        const int hb = r / nb, kb = r % nb;
        t = Task{rl.d1 + 4 * hb, rl.y + 4 * kb, oW1 + 4 * hb * n + 4 * kb, n, 4, (n - 4 * kb) < 4 ? (n - 4 * kb) : 4};
        return true;
    }
    r -= wb * nb;
    if (r < wb) {        // db1[h] = sum d1[h]
        t = Task{rl.d1 + 4 * r, rl.one, ob1 + 4 * r, 1, 4, 1};
        return true;
    }
    r -= wb;
    if (r < wb * wb) {   // dW2[h][k] = sum d2[h] a1[k]
        const int hb = r / wb, kb = r % wb;
        t = Task{rl.d2 + 4 * hb, rl.a1 + 4 * kb, oW2 + 4 * hb * w + 4 * kb, w, 4, 4};
        return true;
    }
    r -= wb * wb;
    if (r < wb) {        // db2
        t = Task{rl.d2 + 4 * r, rl.one, ob2 + 4 * r, 1, 4, 1};
        return true;
    }
    r -= wb;
    if (r < nb * wb) {   // dW3[r][h] = sum w[r] a2[h]
        const int rb = r / wb, hb = r % wb;
        t = Task{rl.w + 4 * rb, rl.a2 + 4 * hb, oW3 + 4 * rb * w + 4 * hb, w, (n - 4 * rb) < 4 ? (n - 4 * rb) : 4, 4};
        return true;
    }
    r -= nb * wb;
    if (r < nb) {        // db3
        t = Task{rl.w + 4 * r, rl.one, ob3 + 4 * r, 1, (n - 4 * r) < 4 ? (n - 4 * r) : 4, 1};
        return true;
    }
    return false;
}

__host__ __device__ inline int task_count(int n, int w) {
    const int wb = w / 4, nb = ceil4(n) / 4;
    return wb * nb + wb + wb * wb + wb + nb * wb + nb;
}

template <typename S>
__global__ __launch_bounds__(kThreads) void mlp_vjp_kernel(MlpVjpParams p, int pts) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    S* sW = reinterpret_cast<S*>(smem_raw);
    const int n = p.n, w = p.width;
    const RowLayout rl(n, w);
    const WeightLayout wl(n, w);
    S* rows = sW + ((wl.len + 3) & ~3);
    const int tid = threadIdx.x;
    const S* __restrict__ th = reinterpret_cast<const S*>(p.theta);

    // stage the weights (and the two transposes the reverse sweep reads row-wise)
    {
        const int oW1 = 0, ob1 = w * n, oW2 = ob1 + w, ob2 = oW2 + w * w, oW3 = ob2 + w;
        for (int q = tid; q < w * n; q += kThreads) sW[wl.W1 + q] = th[oW1 + q];
        for (int q = tid; q < w; q += kThreads) { sW[wl.b1 + q] = th[ob1 + q]; sW[wl.b2 + q] = th[ob2 + q]; }
        for (int q = tid; q < w * w; q += kThreads) {
            const S v = th[oW2 + q];
            sW[wl.W2 + q] = v;
            sW[wl.W2T + (q % w) * w + (q / w)] = v;
        }
        for (int q = tid; q < n * w; q += kThreads) sW[wl.W3T + (q % w) * n + (q / w)] = th[oW3 + q];
    }

    const int split = kThreads / pts;      // threads per point in phase A
    const int pt = tid % pts, part = tid / pts;
    const int grp = tid >> 7, tl = tid & 127;   // phase B: two groups of 128 threads
    S acc[kMaxTasks][16];
    Task task[kMaxTasks];
    bool has[kMaxTasks];
#pragma unroll
    for (int k = 0; k < kMaxTasks; ++k) {
        has[k] = make_task(tl + 128 * k, n, w, rl, task[k]);
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[k][e] = S(0);
    }

    const long long total = (long long)p.B * p.T;
    const long long chunks = (total + pts - 1) / pts;
    const S* __restrict__ yg = reinterpret_cast<const S*>(p.y);
    const S* __restrict__ ug = reinterpret_cast<const S*>(p.u);
    __syncthreads();

    for (long long ch = blockIdx.x; ch < chunks; ch += gridDim.x) {
        // ---- phase A: the reverse sweep at every point of the chunk ----
        S* R = rows + (size_t)pt * rl.len;
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
        // (all inner products run over four entries at a time: 16-byte LDS reads of the point's row and of
        // the weights, which every lane of a wavefront reads at the same address)
        for (int h = part; h < w; h += split) {
            S a = sW[wl.b1 + h];
            if ((n & 3) == 0) {
                for (int k = 0; k < n; k += 4) {
                    S wv[4], yv[4];
                    vload<S, 4>(wv, sW + wl.W1 + h * n + k);
                    vload<S, 4>(yv, R + rl.y + k);
                    a += wv[0] * yv[0] + wv[1] * yv[1] + wv[2] * yv[2] + wv[3] * yv[3];
                }
            } else {
                for (int k = 0; k < n; ++k) a += sW[wl.W1 + h * n + k] * R[rl.y + k];
            }
            R[rl.a1 + h] = tanh_(a);
        }
        __syncthreads();
        for (int h = part; h < w; h += split) {
            S a = sW[wl.b2 + h];
            for (int k = 0; k < w; k += 4) {
                S wv[4], av[4];
                vload<S, 4>(wv, sW + wl.W2 + h * w + k);
                vload<S, 4>(av, R + rl.a1 + k);
                a += wv[0] * av[0] + wv[1] * av[1] + wv[2] * av[2] + wv[3] * av[3];
            }
            R[rl.a2 + h] = tanh_(a);
        }
        __syncthreads();
        for (int h = part; h < w; h += split) {
            S s = S(0);
            if ((n & 3) == 0) {
                for (int r = 0; r < n; r += 4) {
                    S wv[4], cv[4];
                    vload<S, 4>(wv, sW + wl.W3T + h * n + r);
                    vload<S, 4>(cv, R + rl.w + r);
                    s += wv[0] * cv[0] + wv[1] * cv[1] + wv[2] * cv[2] + wv[3] * cv[3];
                }
            } else {
                for (int r = 0; r < n; ++r) s += sW[wl.W3T + h * n + r] * R[rl.w + r];
            }
            const S a2 = R[rl.a2 + h];
            R[rl.d2 + h] = s * (S(1) - a2 * a2);
        }
        __syncthreads();
        for (int h = part; h < w; h += split) {
            S s = S(0);
            for (int k = 0; k < w; k += 4) {
                S wv[4], dv[4];
                vload<S, 4>(wv, sW + wl.W2T + h * w + k);
                vload<S, 4>(dv, R + rl.d2 + k);
                s += wv[0] * dv[0] + wv[1] * dv[1] + wv[2] * dv[2] + wv[3] * dv[3];
            }
            const S a1 = R[rl.a1 + h];
            R[rl.d1 + h] = s * (S(1) - a1 * a1);
        }
        __syncthreads();

        // ---- phase B: outer products summed over the points of the chunk ----
#pragma unroll
        for (int k = 0; k < kMaxTasks; ++k) {
            if (has[k]) {
                for (int q = grp; q < pts; q += 2) {
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

    // one partial row per thread group
    S* __restrict__ out = reinterpret_cast<S*>(p.partial) + ((size_t)blockIdx.x * 2 + grp) * (size_t)(wl.W3T + n * w + n);   // row of theta_count entries
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

long long theta_len(int n, int w) { return (long long)w * n + w + (long long)w * w + w + (long long)n * w + n; }

// points per chunk so that weights and rows fit the LDS budget (a power of two between 32 and 128)
template <typename S>
int choose_points(int n, int w, size_t* bytes) {
    const RowLayout rl(n, w);
    const WeightLayout wl(n, w);
    const size_t wbytes = (size_t)((wl.len + 3) & ~3) * sizeof(S);
    int pts = 128;
    while (pts > 32 && wbytes + (size_t)pts * rl.len * sizeof(S) > (size_t)56 * 1024) pts >>= 1;   // three blocks per compute unit
    *bytes = wbytes + (size_t)pts * rl.len * sizeof(S);
    return pts;
}

template <typename S>
hipError_t launch_s(const MlpVjpParams& p, hipStream_t s) {
    size_t bytes = 0;
    const int pts = choose_points<S>(p.n, p.width, &bytes);
    if (bytes > (size_t)150 * 1024) return hipErrorInvalidValue;
    if (task_count(p.n, p.width) > 128 * kMaxTasks) return hipErrorInvalidValue;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(mlp_vjp_kernel<S>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((mlp_vjp_kernel<S>), dim3((unsigned)p.blocks), dim3(kThreads), bytes, s, p, pts);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_partial_reduce(sizeof(S) == 4 ? 0 : 1, p.partial, p.dtheta, theta_len(p.n, p.width), p.blocks * 2, s);
}

}  // namespace

int mlp_vjp_blocks(int dtype, int n, int width, long long points) {
    size_t bytes = 0;
    const int pts = dtype == 0 ? choose_points<float>(n, width, &bytes) : choose_points<double>(n, width, &bytes);
    long long chunks = (points + pts - 1) / pts;
    if (chunks > 768) chunks = 768;
    if (chunks < 1) chunks = 1;
    return (int)chunks;
}

hipError_t launch_mlp_vjp(int dtype, const MlpVjpParams& p, hipStream_t s) {
    if (p.n < 1 || p.n > 8 || p.width < 4 || p.width > 64 || (p.width & 3) != 0 || p.T < 2) return hipErrorInvalidValue;
    return dtype == 0 ? launch_s<float>(p, s) : launch_s<double>(p, s);
}

}  // namespace deer
