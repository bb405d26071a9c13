// Shared declarations of the DEER HIP library (device helpers and the launch interface
// between the host driver and the kernel translation units).  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace deer {

// Device-side iteration control: kernels of Newton iteration k are enqueued before the error of
// iteration k-1 has been read back.  They look at that error themselves and return at once when it
// already met the tolerance (or was never written, which reads as zero), so a batch of iterations
// can be enqueued without a host round trip in between.
struct Gate {
    const void* prev_err;   // raw bits of the previous iteration's max|dy| (same scalar type), or nullptr
    double tol;
};
template <typename S>
__device__ __forceinline__ bool gate_closed(const Gate& g) {
    if (!g.prev_err) return false;
    const S e = *reinterpret_cast<const S*>(g.prev_err);
    return (double)e <= g.tol;
}

// ---------------------------------------------------------------------------------------
// Scan launch description.  One launch solves y_k = A_k y_{k-1} + b_k, k = 0..T-1 (scan
// positions), for B sequences (Sec. 3.3 eq. 9-10, Sec. 3.4 eq. 11).  In reverse mode scan
// position k stands for array index T-1-k and uses the TRANSPOSE of the matrix stored at
// index T-k (none for k = 0), which is the dual operator of Sec. 3.1.1 eq. 7.
// All strides are per sequence and counted in scalars.
// ---------------------------------------------------------------------------------------
struct ScanParams {
    const void* A;       // [B][T][n][n]
    const void* bv;      // [B][T][n]
    const void* y0;      // [B][n] or nullptr (zeros)
    void* out;           // [B][T][n]
    const void* yold;    // previous iterate laid out like out, or nullptr (no error reduction)
    long long strideA, strideb, strideOut, strideOld;
    int B, T;
    int L;               // scan positions per lane group (VALU kernel)
    int W;               // wavefronts per tile (VALU kernel): 4 or 8
    int tiles;           // tiles per sequence
    int reverse;
    int delta;           // 1: the scan solves for a correction; out = yold + y and the error is max|y|
    int add_identity;    // VALU kernel, reverse scans: 1 = the stored matrices are A - I (the identity is added on load)
    unsigned epoch;      // tags carry (epoch << 2) | state, so words of earlier launches need no clearing
    unsigned long long* aggW;   // [B * tiles][(n*n + n) * words per scalar] tile totals (M row-major, then v)
    unsigned long long* inclW;  // [B * tiles][n * words per scalar] inclusive carry after the tile
    unsigned* ticket;    // tile dispenser for this launch (zero on entry)
    void* err;           // max |out - yold| as raw bits of a non-negative scalar, or nullptr
    unsigned* status;    // set non-zero when a bounded wait ran out
    Gate gate;
    // multi-head GRU with strides (kernels instantiated with MH only): heads, stride levels, parameters per head, and
    // the list of one batch entry's tiles (p.tiles entries: head << 26 | first time index << 19 | tile of its recurrence)
    int mh_H, mh_K;
    long long mh_P;
    const unsigned* mh_table;
#ifdef DEER_SCAN_TIMING
    unsigned long long* timing;   // development builds only: [B * tiles][16] timestamps of the tile's phases
#endif
};

#ifdef DEER_SCAN_TIMING
#define DEER_STAMP(p, slot, j, cond) do { if ((p).timing && (cond)) (p).timing[(slot) * 16 + (j)] = wall_clock64(); } while (0)
// per wavefront (up to 8 per tile, two stamps each), in the upper half of the segment
#define DEER_STAMPW(p, slot, wave, j, cond) do { if ((p).timing && (cond)) (p).timing[((size_t)1 << 19) + ((slot) * 8 + (wave)) * 2 + (j)] = wall_clock64(); } while (0)
#else
#define DEER_STAMP(p, slot, j, cond) do { } while (0)
#define DEER_STAMPW(p, slot, wave, j, cond) do { } while (0)
#endif

// Source of the pairs when the GRU cell is evaluated inside the scan: the pair at position e is
// (J_e | f_e - J_e h_e) with h_e the previous iterate at e-1 (y0 for e = 0), Sec. 3.1 eq. 3 and 5 with the
// sign folded as in the stand-alone cell kernel.  theta uses that kernel's layout.
struct GruFeed {
    const void* theta;
    const void* x;   // [B][T][d]
    int d;           // <= DP
};

// Activations of the fused GRU steps.
// fp32: hardware exp2 and reciprocal (about 1 ulp each).  The absolute error of both functions stays
// below 3e-7, far inside the convergence tolerance of the fp32 iteration; overflow of exp2 gives the
// correct limits (1/inf = 0).
__device__ __forceinline__ float feed_sigmoid(float a) {
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504088896341f * a));
}
__device__ __forceinline__ float feed_tanh(float a) {
    return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(2.88539008177792681f * a));
}
__device__ __forceinline__ double feed_sigmoid(double a) { return 1.0 / (1.0 + exp(-a)); }
__device__ __forceinline__ double feed_tanh(double a) { return tanh(a); }

// One launch that runs all Newton iterations of a GRU problem (n <= 8) whose tiles are all resident.
struct NewtonParams {
    ScanParams scan;           // y0, out, yold = initial guess or nullptr (zeros), shapes, published-word regions,
                               // epoch of the first iteration (iteration k uses epoch + k), status
    GruFeed feed;
    unsigned long long* err;      // [max_iter] 8-byte slots: max|dy| of every iteration, for the host (may be
                                  // host-mapped memory); an infinite entry also stands for a wait that ran out
    unsigned long long* barrier;  // [2][workgroups][words per scalar] tagged words, no valid tag on entry
    int* result;               // number of iterations performed (may be host-mapped memory)
    double tol;
    int max_iter;              // >= 1
    unsigned spin_limit;       // polls before a wait in the grid barrier gives up (kSpinLimit in production)
    unsigned extra_workgroups; // test hook: the barrier also expects this many workgroups that do not exist,
                               // so it runs into its limit and the failure path can be exercised
};

enum : unsigned { TILE_INVALID = 0u, TILE_AGGREGATE = 1u, TILE_INCLUSIVE = 2u };
constexpr unsigned kSpinLimit = 1u << 22;   // polls before a waiting tile gives up

// ---------------------------------------------------------------------------------------
// Device helpers
// ---------------------------------------------------------------------------------------

template <int BYTES> struct VecOf;
template <> struct VecOf<16> { using type = uint4; };
template <> struct VecOf<8> { using type = uint2; };
template <> struct VecOf<4> { using type = unsigned; };

// Copy COUNT scalars between a register array and memory with the widest access that divides
// COUNT * sizeof(S); the address must be aligned to that width (guaranteed by the layouts used).
template <typename S, int COUNT>
__device__ __forceinline__ void vload(S* dst, const S* __restrict__ src) {
    constexpr int bytes = COUNT * (int)sizeof(S);
    constexpr int W = (bytes % 16 == 0) ? 16 : ((bytes % 8 == 0) ? 8 : 4);
    using V = typename VecOf<W>::type;
    constexpr int NV = bytes / W;
    constexpr int PER = W / (int)sizeof(S);
    static_assert(W >= (int)sizeof(S), "scalar wider than access");
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        V v = reinterpret_cast<const V*>(src)[i];
        const S* p = reinterpret_cast<const S*>(&v);
#pragma unroll
        for (int j = 0; j < PER; ++j) dst[i * PER + j] = p[j];
    }
}

template <typename S, int COUNT>
__device__ __forceinline__ void vstore(S* __restrict__ dst, const S* src) {
    constexpr int bytes = COUNT * (int)sizeof(S);
    constexpr int W = (bytes % 16 == 0) ? 16 : ((bytes % 8 == 0) ? 8 : 4);
    using V = typename VecOf<W>::type;
    constexpr int NV = bytes / W;
    constexpr int PER = W / (int)sizeof(S);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        V v;
        S* p = reinterpret_cast<S*>(&v);
#pragma unroll
        for (int j = 0; j < PER; ++j) p[j] = src[i * PER + j];
        reinterpret_cast<V*>(dst)[i] = v;
    }
}

// ---------------------------------------------------------------------------------------
// Self-validating words for data handed from one workgroup to another inside a launch.
// Every 32 bits of payload travel in one 64-bit word together with a 32-bit tag
// (launch epoch << 2 | state), written and read with single 64-bit agent-scope atomics.  A reader
// accepts a word only if its tag matches, so no ordering between the words, no fence and no cache
// write-back or invalidation is needed: a word is either the expected one or not there yet.
// ---------------------------------------------------------------------------------------
template <typename S> struct TaggedWords;
template <> struct TaggedWords<float> {
    static constexpr int per_scalar = 1;
    static __device__ __forceinline__ void put(unsigned long long* base, long long idx, float v, unsigned tag) {
        __hip_atomic_store(base + idx, ((unsigned long long)tag << 32) | __float_as_uint(v), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    }
    static __device__ __forceinline__ bool get(const unsigned long long* base, long long idx, unsigned tag, float& v) {
        const unsigned long long w = __hip_atomic_load(base + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        v = __uint_as_float((unsigned)(w & 0xffffffffull));
        return (unsigned)(w >> 32) == tag;
    }
};
template <> struct TaggedWords<double> {
    static constexpr int per_scalar = 2;
    static __device__ __forceinline__ void put(unsigned long long* base, long long idx, double v, unsigned tag) {
        const unsigned long long u = (unsigned long long)__double_as_longlong(v);
        __hip_atomic_store(base + 2 * idx, ((unsigned long long)tag << 32) | (u & 0xffffffffull), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(base + 2 * idx + 1, ((unsigned long long)tag << 32) | (u >> 32), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    }
    static __device__ __forceinline__ bool get(const unsigned long long* base, long long idx, unsigned tag, double& v) {
        const unsigned long long lo = __hip_atomic_load(base + 2 * idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned long long hi = __hip_atomic_load(base + 2 * idx + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        v = __longlong_as_double((long long)((hi << 32) | (lo & 0xffffffffull)));
        return (unsigned)(lo >> 32) == tag && (unsigned)(hi >> 32) == tag;
    }
};
// read a word that is known to be on its way; gives up (returns false) after kSpinLimit polls
template <typename S>
__device__ __forceinline__ bool tagged_get_wait(const unsigned long long* base, long long idx, unsigned tag, S& v) {
    unsigned spins = 0;
    while (!TaggedWords<S>::get(base, idx, tag, v)) {
        if (++spins > kSpinLimit) return false;
        __builtin_amdgcn_s_sleep(1);
    }
    return true;
}

// max-reduce a non-negative value (NaN mapped to +inf by the caller) into *err as raw bits
// (the stored maximum only grows: a value that does not exceed what a plain load sees cannot change it, and skipping
// its read-modify-write keeps a launch with hundreds of thousands of wavefronts from queueing on one address)
__device__ __forceinline__ void err_atomic_max(void* err, float v) {
    unsigned* p = reinterpret_cast<unsigned*>(err);
    const unsigned bits = __float_as_uint(v);
    if (bits > __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(p, bits);
}
__device__ __forceinline__ void err_atomic_max(void* err, double v) {
    unsigned long long* p = reinterpret_cast<unsigned long long*>(err);
    const unsigned long long bits = (unsigned long long)__double_as_longlong(v);
    if (bits > __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(p, bits);
}

template <typename S>
__device__ __forceinline__ S abs_or_inf(S d) {
    d = d < S(0) ? -d : d;
    // a NaN difference must not be lost in the max: report +inf instead
    return (d == d) ? d : S(INFINITY);
}

template <typename S>
__device__ __forceinline__ S wave_max(S v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        S u = __shfl_xor(v, o);
        v = u > v ? u : v;
    }
    return v;
}

// ---------------------------------------------------------------------------------------
// Launchers implemented in the kernel translation units.  Each returns hipGetLastError().
// ---------------------------------------------------------------------------------------
struct GruParams {
    const void* theta; const void* x; const void* y0; const void* y;  // y: current iterate [B,T,n]
    void* J; void* rhs;                                               // outputs [B,T,n,n], [B,T,n]
    int B, T, n, d;
    Gate gate;
    int units;         // LSTM and LEM kernels: units of the cell (n is then the scan's state size, >= 2 units); 0 otherwise
    double dt;         // LEM kernels: the cell's step
};

struct GruVjpParams {
    const void* theta; const void* x; const void* y0; const void* y; const void* lam;
    void* dx;          // [B,T,d] or nullptr
    void* dy0;         // [B,n] or nullptr
    void* partial;     // [blocks][theta_count] per-block partial sums
    void* dtheta;      // [theta_count]
    int B, T, n, d;
    int blocks;
    int H, K;          // multi-head GRU with strides: heads and stride levels (0 or 1: the plain GRU); arrays are then
                       // [B][T][H][.], theta and dtheta [H][theta_count], partial [H][blocks * 4][theta_count]
    void* dy0_parts;   // multi-head: [B][H][2^(K-1)][n] scratch for the terms of dL/dy0
    int units;         // LSTM and LEM kernels: units of the cell (n: the scan's state size); 0 otherwise
    double dt;         // LEM kernels: the cell's step
};

struct MlpParams {
    const void* theta; const void* y;     // y [B,T,n]
    void* G; void* z;                     // outputs: G = -df/dy [B,T,n,n], z = f + G y [B,T,n]
    int B, T, n, width;
    Gate gate;
    int jac_only;                         // != 0: only G is wanted (the backward pass); kernels may write zeros to z
    int nhid, act;                        // hidden layers and activation (0 tanh, 1 softplus): read by the general kernels only
};

struct OdeDiscParams {
    const void* G; const void* z;         // [B,T,n,n], [B,T,n]
    const void* y;                        // current iterate [B,T,n]
    void* Gbar; void* res;                // [B,T-1,n,n] exp(-Gc dt), [B,T-1,n] residual of the iterate
    int B, T, n;
    double dt;
    Gate gate;
    int minus_identity;                   // 1: Gbar holds exp(-Gc dt) - I (nothing of size dt is rounded against 1)
    int matrix_only;                      // 1: only Gbar is wanted (the backward pass): z, y and res are not touched
};

struct OdeDualParams {
    const void* G;                        // [B,T,n,n] G = -df/dy at the trajectory
    const void* lam;                      // [B,T-1,n] scanned cotangent at grid points 1..T-1
    const void* g;                        // [B,T,n] dL/dy (entry 0 is read when dy0 is given)
    void* u;                              // [B,T-1,n] dt phi1(X_i)^T lam_{i+1}
    void* dy0;                            // [B,n] or nullptr
    int B, T, n;
    double dt;
};

struct MlpVjpParams {
    const void* theta; const void* y;     // y [B,T,n]
    const void* u;                        // [B,T-1,n] from the dual discretisation
    void* partial;                        // [blocks][theta_count] per-block partial sums
    void* dtheta;                         // [theta_count]
    int B, T, n, width;
    int blocks;
    int nhid, act;                        // as in MlpParams
};

hipError_t launch_scan_valu(int dtype, int n, const ScanParams& p, hipStream_t s);
hipError_t launch_scan_mfma(int dtype, int n, const ScanParams& p, hipStream_t s);
// MFMA scan with the GRU cell evaluated in place of the loads (fp32, forward, n = 16 or 32, d <= 16)
bool scan_mfma_fused_supported(int dtype, int n, int d);
int scan_mfma_fused_tile(int n);   // scan positions per tile of the fused step
hipError_t launch_scan_mfma_fused(int n, const ScanParams& p, const void* theta, const void* x, int d, hipStream_t s);
int scan_valu_tile(int n, int L, int W);   // scan positions per tile
// scan with the GRU cell evaluated in place of the loads (forward, n <= 8, d <= 8); p.A / p.bv unused
bool scan_gru_fused_supported(int dtype, int n, int d, int L, int W);
// all iterations in one launch: workgroups the current device holds at once (0: no such variant), launcher
int gru_newton_capacity(int dtype, int n, int d, int L);
hipError_t launch_gru_newton(int dtype, int n, const NewtonParams& q, hipStream_t s);
hipError_t launch_scan_gru_fused(int dtype, int n, const ScanParams& p, const void* theta, const void* x, int d,
                                 hipStream_t s);
// the same for the dual scan of the backward derivative (p.reverse set, p.yold = trajectory, p.bv = cotangent)
bool scan_gru_dual_supported(int dtype, int n, int d, int L, int W);
hipError_t launch_scan_gru_dual(int dtype, int n, const ScanParams& p, const void* theta, const void* x, int d,
                                hipStream_t s);
// the fused step and its dual for the strided heads of a multi-head GRU (p.mh_* set; p.B = batch * p.mh_Sper)
bool scan_gru_mh_supported(int dtype, int n, int d, int L);
hipError_t launch_scan_gru_mh(int dtype, int n, const ScanParams& p, const void* theta, const void* x, int d, hipStream_t s);
int scan_mfma_tile(int dtype, int n);
hipError_t launch_gru_funceval(int dtype, const GruParams& p, hipStream_t s);
hipError_t launch_gru_vjp(int dtype, const GruVjpParams& p, hipStream_t s);
// the same on the matrix cores (fp32, n = 16 or 32, d <= 16): kernel only, partial rows = blocks * 4
bool gru_vjp_mfma_supported(int dtype, int n, int d);
hipError_t launch_gru_vjp_mfma(const GruVjpParams& p, hipStream_t s);
int gru_vjp_blocks(int n, long long steps);
// LSTM cell (p.units units, state (h | c) in rows of p.n >= 2 units scalars): Jacobian + right-hand side, and the
// vector-Jacobian product with its reduction (partial rows = blocks * 4)
bool lstm_supported(int units, int d);
int lstm_vjp_blocks(int units, long long steps);
hipError_t launch_lstm_funceval(int dtype, const GruParams& p, hipStream_t s);
hipError_t launch_lstm_vjp(int dtype, const GruVjpParams& p, hipStream_t s);
// LEM cell (same shapes and parameter layout as the LSTM: units 1..16, d 1..8; p.dt is the step)
hipError_t launch_lem_funceval(int dtype, const GruParams& p, hipStream_t s);
hipError_t launch_lem_vjp(int dtype, const GruVjpParams& p, hipStream_t s);
hipError_t launch_mlp_funceval(int dtype, const MlpParams& p, hipStream_t s);
hipError_t launch_ode_discretise(int dtype, const OdeDiscParams& p, hipStream_t s);
hipError_t launch_ode_dual(int dtype, const OdeDualParams& p, hipStream_t s);
// residual of an approximate solution lam0 of the dual recurrence lam_i = g_i + (I + D_{i+1})^T lam_{i+1} over grid
// points 1..T-1 (D [B,T-1,n,n] = Gbar - I, g [B,T,n], lam0 and res [B,T-1,n]), evaluated without forming I + D
hipError_t launch_ode_dual_residual(int dtype, const void* D, const void* g, const void* lam0, void* res, int B, int T,
                                    int n, hipStream_t s);
// VJP of the MLP field with the parameter-gradient reduction; blocks from mlp_vjp_blocks()
int mlp_vjp_blocks(int dtype, int n, int width, long long points);
hipError_t launch_mlp_vjp(int dtype, const MlpVjpParams& p, hipStream_t s);
// the same sums on the matrix cores (fp32, n = 8, width 16, 32 or 64); writes p.blocks * 4 partial rows and leaves
// their addition (launch_partial_reduce) to the caller
bool mlp_vjp_mfma_supported(int dtype, int n, int width);
hipError_t launch_mlp_vjp_mfma(const MlpVjpParams& p, hipStream_t s);
// MLP field of any depth (1..5 hidden layers) and activation (tanh, softplus): field + Jacobian, and the
// vector-Jacobian product with its reduction (partial rows = p.blocks, from mlp_general_vjp_blocks())
bool mlp_general_supported(int n, int width, int nhid, int act);
int mlp_general_vjp_blocks(int dtype, int n, int width, int nhid, long long points);
hipError_t launch_mlp_general_funceval(int dtype, const MlpParams& p, hipStream_t s);
hipError_t launch_mlp_general_vjp(int dtype, const MlpVjpParams& p, hipStream_t s);
// fixed-order sum of partial rows [rows][P] into out[P]
hipError_t launch_partial_reduce(int dtype, const void* partial, void* out, long long P, int rows, hipStream_t s);
// zero-padding of the channel axis (rows of n scalars <-> rows of np) and of the GRU parameters, both directions
hipError_t launch_pad_rows(int dtype, const void* src, void* dst, long long rows, int n, int np, int unpack, hipStream_t s);
hipError_t launch_pad_gru_theta(int dtype, const void* src, void* dst, int n, int np, int d, int unpack, hipStream_t s);
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s);
hipError_t launch_fill_zero2(void* a, size_t abytes, void* b, size_t bbytes, hipStream_t s);
hipError_t launch_copy_word(void* dst, const void* src, hipStream_t s);   // one 32-bit word, device to device
hipError_t launch_pin_first(int dtype, void* y, const void* y0, int B, int T, int n, hipStream_t s);

}  // namespace deer
