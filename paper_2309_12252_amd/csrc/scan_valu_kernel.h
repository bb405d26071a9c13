// Kernel template of the single-pass scan for small state sizes (n <= 8) and its DPP helpers.
// Included by the translation units that instantiate it: the plain scan (pairs read from memory)
// and the scan with the GRU cell evaluated in place of the loads.
#pragma once
#include "deer_common.h"

namespace deer {

namespace {

// ---- DPP helpers ----
template <int CTRL, int BANK_MASK, bool BOUND>
__device__ __forceinline__ float dpp(float old, float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(x), CTRL, 0xf, BANK_MASK, BOUND));
}
template <int CTRL, int BANK_MASK, bool BOUND>
__device__ __forceinline__ double dpp(double old, double x) {
    const long long u = __double_as_longlong(x), o = __double_as_longlong(old);
    const int lo = __builtin_amdgcn_update_dpp((int)(o & 0xffffffffll), (int)(u & 0xffffffffll), CTRL, 0xf, BANK_MASK, BOUND);
    const int hi = __builtin_amdgcn_update_dpp((int)(o >> 32), (int)(u >> 32), CTRL, 0xf, BANK_MASK, BOUND);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
// broadcast of lane q of every quad
template <int Q, typename S>
__device__ __forceinline__ S quad_bcast(S x) { return dpp<0x55 * Q, 0xf, true>(S(0), x); }

// For n = 8 a group is two quads.  mirror(x) reverses the group (lane i gets the value of lane 7 - i),
// so every lane sees the other quad's four values next to its own quad's.  Broadcasting lane k of
// the own quad of x gives entry 4*hi + k of the group (hi = 1 in the upper quad); broadcasting lane
// 3 - k of the own quad of mirror(x) gives entry 4*(1 - hi) + k.  A dot product of a register row with
// the group's values thus takes the row SWIZZLED: slot s holds column s ^ (4*hi), i.e. the halves of
// the row are swapped in the lanes of the upper quad.  Every left factor below is kept in that
// form (for n < 8 the swizzle is the identity).
template <typename S, int N>
__device__ __forceinline__ S mirror(S x) {
    if constexpr (N == 8) return dpp<0x141, 0xf, true>(S(0), x);
    else return x;
}
// column held by slot s of a swizzled row in lane i of the group
template <int N>
__device__ __forceinline__ int swz_col(int s, int i) {
    if constexpr (N == 8) return s ^ (i & 4);
    else return s;
}
template <typename S, int N>
__device__ __forceinline__ void swizzle_row(const S* nat, S* out, int i) {
    if constexpr (N == 8) {
        const bool hi = (i & 4) != 0;
#pragma unroll
        for (int s = 0; s < 8; ++s) out[s] = hi ? nat[s ^ 4] : nat[s];
    } else {
#pragma unroll
        for (int s = 0; s < N; ++s) out[s] = nat[s];
    }
}
// N scalars of a row-major matrix row at `row`, swizzled for lane i (two half loads for n = 8)
template <typename S, int N>
__device__ __forceinline__ void load_swizzled(S* out, const S* __restrict__ row, int i) {
    if constexpr (N == 8) {
        const int h = i & 4;
        vload<S, 4>(out, row + h);
        vload<S, 4>(out + 4, row + (4 - h));
    } else {
        vload<S, N>(out, row);
    }
}
// value of x in the lane that slot s of a swizzled row refers to (xm: mirror(x))
template <typename S, int N, int s>
__device__ __forceinline__ S fetch(S x, S xm) {
    if constexpr (N == 1) return x;
    else if constexpr (N == 2) return dpp<(s == 0 ? 0xA0 : 0xF5), 0xf, true>(S(0), x);
    else if constexpr (N == 4) return quad_bcast<s>(x);
    else if constexpr (s < 4) return quad_bcast<s>(x);
    else return quad_bcast<7 - s>(xm);
}

// acc += sum_s Ls[s] * (value of x in the lane slot s refers to)
template <typename S, int N, int s = 0>
struct RowDot {
    static __device__ __forceinline__ void run(const S* Ls, S x, S xm, S& acc) {
        acc += Ls[s] * fetch<S, N, s>(x, xm);
        if constexpr (s + 1 < N) RowDot<S, N, s + 1>::run(Ls, x, xm, acc);
    }
};

#include "scan_valu_dpp.inc"

// acc[0..K) += (swizzled row Ls) . (column values spread over the group), K columns given in x
template <typename S, int N, int K>
__device__ __forceinline__ void row_dots(const S* Ls, const S* x, S* acc) {
    if constexpr (sizeof(S) == 4 && N == 8 && (K == 4 || K == 1)) {
        float xm[K];
#pragma unroll
        for (int c = 0; c < K; ++c) xm[c] = mirror<float, 8>(x[c]);
        if constexpr (K == 4) dpp_dot8_4(Ls, x, xm, acc); else dpp_dot8_1(Ls, x, xm, acc);
    } else if constexpr (sizeof(S) == 4 && N == 4 && (K == 4 || K == 1)) {
        if constexpr (K == 4) dpp_dot4_4(Ls, x, acc); else dpp_dot4_1(Ls, x, acc);
    } else if constexpr (sizeof(S) == 4 && N == 2 && (K == 2 || K == 1)) {
        if constexpr (K == 2) dpp_dot2_2(Ls, x, acc); else dpp_dot2_1(Ls, x, acc);
    } else {
#pragma unroll
        for (int c = 0; c < K; ++c) RowDot<S, N>::run(Ls, x[c], mirror<S, N>(x[c]), acc[c]);
    }
}

// Lr: row i of the left matrix, swizzled.  (M | v): right pair, lane i holds row i / entry i in natural
// column order.  Result (natural order): row i of Lmat * M and entry i of Lmat * v + add.
// Must be called by whole wavefronts (the cross-lane operands come from every lane of the group).
template <typename S, int N>
__device__ __forceinline__ void group_apply(const S* Lr, S add, S* M, S& v) {
    constexpr int K = (N >= 4) ? 4 : N;   // columns per block
    S R[N];
#pragma unroll
    for (int c = 0; c < N; ++c) R[c] = S(0);
#pragma unroll
    for (int c0 = 0; c0 < N; c0 += K) row_dots<S, N, K>(Lr, M + c0, R + c0);
    S nv = add;
    row_dots<S, N, 1>(Lr, &v, &nv);
#pragma unroll
    for (int c = 0; c < N; ++c) M[c] = R[c];
    v = nv;
}
// entry i of Lmat * y + add, y spread over the group
template <typename S, int N>
__device__ __forceinline__ S group_matvec(const S* Lr, S add, S y) {
    S nv = add;
    row_dots<S, N, 1>(Lr, &y, &nv);
    return nv;
}

// Rows i (swizzled) of the matrices at scan positions e0 .. e0+L-1 of one sequence and entries i of
// their vectors.  Reverse mode: vector index T-1-e, matrix = transpose of the one stored at index T-e,
// zero for e = 0.  FULL: all positions are inside the sequence (and e0 > 0 in reverse mode), so one
// base address with constant offsets serves all loads.  Otherwise branch free with clamping (positions
// past the end read the last valid one and are then replaced by the identity pair): with
// straight-line code the compiler keeps the loads in order and lets the first products start while
// later positions are still in flight.
template <typename S, int N, int L, bool REV, bool FULL, bool ADDI = false, bool SKIPB = false>
__device__ __forceinline__ void load_pairs(const S* __restrict__ Ab, const S* __restrict__ bb, long long T,
                                           long long e0, int i, S (*Ar)[N], S* be) {
    constexpr S addI = ADDI ? S(1) : S(0);   // ADDI: the stored matrices are A - I
    constexpr int H = (N == 8) ? 4 : 0;
    const int h = (N == 8) ? (i & 4) : 0;
    if constexpr (FULL && !REV) {
        const S* rowa = Ab + e0 * (N * N) + i * N + h;         // first half of the swizzled row
        const S* rowb = Ab + e0 * (N * N) + i * N + (H - h);   // second half (n = 8)
        const S* bp = bb + e0 * N + i;
#pragma unroll
        for (int l = 0; l < L; ++l) {
            if constexpr (N == 8) {
                vload<S, 4>(Ar[l], rowa + l * (N * N));
                vload<S, 4>(Ar[l] + 4, rowb + l * (N * N));
            } else {
                vload<S, N>(Ar[l], rowa + l * (N * N));
            }
            if constexpr (!SKIPB) be[l] = bp[l * N];   // (SKIPB: the vectors come through the staged loads)
        }
    } else if constexpr (FULL && REV) {
        // column i of the matrix stored at index T - e, rows in swizzled order
        const S* cola = Ab + (T - e0) * (N * N) + h * N + i;
        const S* colb = Ab + (T - e0) * (N * N) + (H - h) * N + i;
        const S* bp = bb + (T - 1 - e0) * N + i;
#pragma unroll
        for (int l = 0; l < L; ++l) {
#pragma unroll
            for (int s = 0; s < N; ++s)
                Ar[l][s] = (N == 8 && s >= 4) ? colb[(s - 4) * N - l * (N * N)] : cola[s * N - l * (N * N)];
            be[l] = bp[-l * N];
        }
    } else {
#pragma unroll
        for (int l = 0; l < L; ++l) {
            const long long e = e0 + l;
            const bool past = e >= T;
            const long long ec = past ? T - 1 : e;
            S row[N], bv;
            if constexpr (!REV) {
                load_swizzled<S, N>(row, Ab + ec * (N * N) + i * N, i);
                bv = bb[ec * N + i];
            } else {
                bv = bb[(T - 1 - ec) * N + i];
                const long long em = ec == 0 ? 1 : ec;   // position 0 has no matrix; any valid one is read and dropped
                const S* mat = Ab + (T - em) * (N * N);
                const S* lo = mat + h * N + i;
                const S* hi = mat + (H - h) * N + i;
#pragma unroll
                for (int s = 0; s < N; ++s) {
                    const S* src = (N == 8 && s >= 4) ? hi + (s - 4) * N : lo + s * N;
                    row[s] = (T > 1) ? *src : S(0);
                }
                if (ec == 0) {
#pragma unroll
                    for (int s = 0; s < N; ++s) row[s] = (swz_col<N>(s, i) == i) ? -addI : S(0);   // stays zero below
                }
            }
#pragma unroll
            for (int s = 0; s < N; ++s) Ar[l][s] = past ? ((swz_col<N>(s, i) == i) ? S(1) - addI : S(0)) : row[s];
            be[l] = past ? S(0) : bv;
        }
    }
    // matrices stored without their identity: put it back (slot s of lane i holds column swz_col(s, i))
    if constexpr (ADDI) {
#pragma unroll
        for (int l = 0; l < L; ++l)
#pragma unroll
            for (int s = 0; s < N; ++s) Ar[l][s] += (swz_col<N>(s, i) == i) ? S(1) : S(0);
    }
}


// Staged loads and stores for n = 2 (fp32, forward, tiles inside the sequence; the code also handles n = 4 and
// n = 8, see the measurements below).  A group's rows are short (8 bytes), so a lane-per-row load instruction
// touches one cache line per group and every line
// is visited by many instructions; with eight wavefronts in flight the lines do not survive in the
// first-level cache between visits.  Here every lane loads contiguous 16-byte pieces of the wavefront's
// chunk instead (each line is touched by one instruction), the pieces cross a wavefront-private LDS region
// (one 16-byte pad per group run keeps the reads off each other's banks), and every lane reads its own
// rows back.  LC positions per group and pass.
template <int N, int L>
struct Staged {
    // Measured on chip-filling streams: n = 2 goes from 2.2 to 4.2 TB/s (with 32 positions per group); n = 4 and
    // n = 8, whose rows are whole 16-byte loads, lose with any part staged (matrices at n = 4: 3.9 against 4.2 TB/s;
    // vectors and results only: 4.0 against 4.2 at n = 4, 3.1 against 3.45 at n = 8), so they stay with direct accesses.
    static constexpr bool use = N == 2 && (L % 8 == 0);   // vectors in, results out
    static constexpr bool useA = use && N == 2;           // matrices too
    static constexpr int NG = 64 / N;
    static constexpr int LC = (N == 2) ? ((L % 16 == 0) ? 16 : 8) : 8;   // positions per group and pass
    static constexpr int MU = N * N / 4;            // 16-byte pieces per matrix
    static constexpr int RUNA = LC * MU;            // pieces per group and pass, matrices
    static constexpr int RUNB = LC * N / 4;         // pieces per group and pass, vectors
    static constexpr int TOTA = NG * RUNA, TOTB = NG * RUNB;
    static constexpr int IN4 = (useA ? TOTA + NG : 0) + TOTB + NG, OUT4 = NG * (L * N / 4) + NG;
    static constexpr int U4 = use ? (IN4 > OUT4 ? IN4 : OUT4) : 1;   // pieces of LDS per wavefront
};

// (the staging region is written as 16-byte pieces and read as scalars: both through types that may alias
// anything, so the compiler keeps the reads behind the writes)
typedef uint4 __attribute__((may_alias)) staged_piece;
typedef float __attribute__((may_alias)) staged_scalar;

template <int N, int L>
__device__ __forceinline__ void load_pairs_staged(const float* __restrict__ Ab, const float* __restrict__ bb,
                                                  long long ew, int lane, staged_piece* st, float (*Ar)[N], float* be) {
    using P = Staged<N, L>;
    constexpr int NG = P::NG, LC = P::LC, MU = P::MU, RUNA = P::RUNA, RUNB = P::RUNB;
    static_assert((!P::useA || P::TOTA % 64 == 0) && P::TOTB % 64 == 0, "whole load instructions");
    constexpr int KA = P::useA ? P::TOTA / 64 : 0;
    const int group = lane / N, i = lane % N;
    staged_piece* stA = st;
    staged_piece* stB = st + (P::useA ? P::TOTA + NG : 0);
#pragma unroll
    for (int l0 = 0; l0 < L; l0 += LC) {
        uint4 va[KA > 0 ? KA : 1], vb[P::TOTB / 64];
#pragma unroll
        for (int k = 0; k < KA; ++k) {
            const int u = k * 64 + lane, g = u / RUNA, o = u % RUNA;
            va[k] = reinterpret_cast<const uint4*>(Ab + (ew + (long long)g * L + l0) * (N * N))[o];
        }
#pragma unroll
        for (int k = 0; k < P::TOTB / 64; ++k) {
            const int u = k * 64 + lane, g = u / RUNB, o = u % RUNB;
            vb[k] = reinterpret_cast<const uint4*>(bb + (ew + (long long)g * L + l0) * N)[o];
        }
        if (l0 > 0) __builtin_amdgcn_wave_barrier();   // the previous pass has been read
#pragma unroll
        for (int k = 0; k < KA; ++k) {
            const int u = k * 64 + lane;
            stA[u + u / RUNA] = va[k];
        }
#pragma unroll
        for (int k = 0; k < P::TOTB / 64; ++k) {
            const int u = k * 64 + lane;
            stB[u + u / RUNB] = vb[k];
        }
        __builtin_amdgcn_wave_barrier();
        const staged_scalar* rowsA = reinterpret_cast<const staged_scalar*>(stA + group * (RUNA + 1)) + i * N;
        const staged_scalar* rowsB = reinterpret_cast<const staged_scalar*>(stB + group * (RUNB + 1)) + i;
#pragma unroll
        for (int l = 0; l < LC; ++l) {
            if constexpr (P::useA) {
#pragma unroll
                for (int c = 0; c < N; ++c) Ar[l0 + l][c] = rowsA[l * (N * N) + c];
            }
            float bv = rowsB[l * N];
            // The vectors come back from LDS two to a register pair, and the composition's assembly blocks
            // accumulate into a copy of each vector: with the pair's halves used directly the compiler (ROCm
            // 7.2) dropped that copy for every second position and the block overwrote the vector the
            // second walk still needs.  Passing each value through an opaque statement gives it a register
            // of its own.
            asm volatile("" : "+v"(bv));
            be[l0 + l] = bv;
        }
    }
}

// The other direction for the results: every lane leaves entry i of its L positions in the wavefront's LDS region
// and the wavefront writes its chunk of the output as contiguous 16-byte pieces.
template <int N, int L>
__device__ __forceinline__ void store_staged(float* __restrict__ ob, long long ew, int lane, staged_piece* st, const float* w) {
    constexpr int NG = 64 / N;
    constexpr int RUN = L * N / 4;        // pieces per group
    constexpr int TOT = NG * RUN;
    static_assert(TOT % 64 == 0 && TOT + NG <= Staged<N, L>::U4, "whole store instructions inside the region");
    const int group = lane / N, i = lane % N;
    __builtin_amdgcn_wave_barrier();
    staged_scalar* mine = reinterpret_cast<staged_scalar*>(st + group * (RUN + 1)) + i;
#pragma unroll
    for (int l = 0; l < L; ++l) mine[l * N] = w[l];
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int k = 0; k < TOT / 64; ++k) {
        const int u = k * 64 + lane;
        const staged_piece v = st[u + u / RUN];
        reinterpret_cast<uint4*>(ob + ew * N)[u] = v;
    }
}

// entry i of the previous iterate (or any array laid out like the output) at positions e0 .. e0+L-1
// (psy: scalars between consecutive positions of the sequence, N unless the sequence is a strided head)
template <typename S, int N, int L, bool REV, bool FULL>
__device__ __forceinline__ void load_previous(const S* __restrict__ src, long long T, long long e0, int i, S* yo,
                                              long long psy = N) {
    if constexpr (FULL) {
        const S* bp = src + (REV ? (T - 1 - e0) : e0) * psy + i;
#pragma unroll
        for (int l = 0; l < L; ++l) yo[l] = bp[REV ? -l * psy : l * psy];
    } else {
#pragma unroll
        for (int l = 0; l < L; ++l) {
            const long long e = (e0 + l < T) ? e0 + l : T - 1;
            yo[l] = src[(REV ? (T - 1 - e) : e) * psy + i];
        }
    }
}

// Row i of the GRU cell's weights in the layouts the fused step uses
template <typename S, int N, int DP>
struct GruRow {
    S Ur[N], Uz[N], Uc[N];   // rows of the hidden-to-hidden matrices, swizzled
    S E[N];                  // row i of the identity, swizzled
    S Wr[DP], Wz[DP], Wc[DP];
    S br, bz, bc, bh;
};

template <typename S, int N, int DP>
__device__ __forceinline__ void load_gru_row(const GruFeed& gf, int i, GruRow<S, N, DP>& w) {
    const S* __restrict__ th = reinterpret_cast<const S*>(gf.theta);
    const int d = gf.d;
    const S* __restrict__ U = th + 3 * N * d;
    const S* __restrict__ bias = U + 3 * N * N;
    load_swizzled<S, N>(w.Ur, U + i * N, i);
    load_swizzled<S, N>(w.Uz, U + (N + i) * N, i);
    load_swizzled<S, N>(w.Uc, U + (2 * N + i) * N, i);
#pragma unroll
    for (int j = 0; j < N; ++j) w.E[j] = (swz_col<N>(j, i) == i) ? S(1) : S(0);
#pragma unroll
    for (int k = 0; k < DP; ++k) {
        const int kc = k < d ? k : d - 1;   // columns past d read a valid one and count as zero
        const S a = th[i * d + kc], bq = th[(N + i) * d + kc], c = th[(2 * N + i) * d + kc];
        w.Wr[k] = k < d ? a : S(0);
        w.Wz[k] = k < d ? bq : S(0);
        w.Wc[k] = k < d ? c : S(0);
    }
    w.br = bias[i]; w.bz = bias[N + i]; w.bc = bias[2 * N + i]; w.bh = bias[3 * N + i];
}

// input projections W x + b of row i at positions e0 .. e0+L-1 (xb: inputs of the sequence)
template <typename S, int N, int L, int DP, bool FULL>
__device__ __forceinline__ void gru_project(const GruRow<S, N, DP>& w, const S* __restrict__ xb, int d, long long T,
                                            long long e0, S* pr, S* pq, S* pc, long long psx = -1) {
    if (psx < 0) psx = d;   // scalars between the inputs of consecutive positions
#pragma unroll
    for (int l = 0; l < L; ++l) {
        const long long e = (FULL || e0 + l < T) ? e0 + l : T - 1;
        S ar = w.br, az = w.bz, ac = w.bc;
#pragma unroll
        for (int k = 0; k < DP; ++k) {
            const S xv = xb[e * psx + (k < d ? k : d - 1)];
            ar += w.Wr[k] * xv;
            az += w.Wz[k] * xv;
            ac += w.Wc[k] * xv;
        }
        pr[l] = ar; pq[l] = az; pc[l] = ac;
    }
}

// Rows i of the pairs (J_e | f_e - J_e h_e) at positions e0 .. e0+L-1.  h: entry i of the state in front
// of the first position; yo: entries i of the previous iterate at these positions (h of the next one).
template <typename S, int N, int L, int DP, bool FULL>
__device__ __forceinline__ void gru_rows(const GruRow<S, N, DP>& w, const S* pr, const S* pq, const S* pc, S h,
                                         const S* yo, long long T, long long e0, S (*Ar)[N], S* be) {
#pragma unroll
    for (int l = 0; l < L; ++l) {
        S ar = pr[l], az = pq[l], ac = pc[l], q = w.bh;
        row_dots<S, N, 1>(w.Ur, &h, &ar);
        row_dots<S, N, 1>(w.Uz, &h, &az);
        row_dots<S, N, 1>(w.Uc, &h, &q);
        const S r = feed_sigmoid(ar), z = feed_sigmoid(az);
        const S c = feed_tanh(ac + r * q);
        const S f = (S(1) - z) * c + z * h;
        const S pz = (h - c) * z * (S(1) - z);
        const S sc = (S(1) - z) * (S(1) - c * c);
        const S sr = sc * r;
        const S st = sc * q * r * (S(1) - r);
        S Jrow[N];
#pragma unroll
        for (int j = 0; j < N; ++j) Jrow[j] = pz * w.Uz[j] + (sr * w.Uc[j] + (st * w.Ur[j] + z * w.E[j]));
        S Jh = S(0);
        row_dots<S, N, 1>(Jrow, &h, &Jh);
        if constexpr (FULL) {
#pragma unroll
            for (int j = 0; j < N; ++j) Ar[l][j] = Jrow[j];
            be[l] = f - Jh;
        } else {
            const bool past = e0 + l >= T;
#pragma unroll
            for (int j = 0; j < N; ++j) Ar[l][j] = past ? w.E[j] : Jrow[j];
            be[l] = past ? S(0) : f - Jh;
        }
        h = yo[l];
    }
}

// The pairs of positions e0 .. e0+L-1 from the GRU cell.  yo: previous iterate at these positions
// (already requested); oldb: previous iterate of the sequence; DP: input width the x loops are unrolled for.
// (gf.theta: this sequence's parameters; xb: its inputs; y0row: its initial state or nullptr; psy, psx: scalars between
// consecutive positions of the trajectory and of the inputs)
template <typename S, int N, int L, int DP, bool FULL>
__device__ __forceinline__ void gru_pairs(const GruFeed& gf, const S* __restrict__ xb, const S* __restrict__ y0row,
                                          const S* __restrict__ oldb, long long T, long long e0, int i, const S* yo,
                                          S (*Ar)[N], S* be, long long psy, long long psx) {
    GruRow<S, N, DP> w;
    load_gru_row<S, N, DP>(gf, i, w);
    // state in front of the first position of this group
    S h;
    {
        const long long ef = e0 < T ? e0 : T;
        const S a = oldb[(ef > 0 ? ef - 1 : 0) * psy + i];
        const S c0 = y0row ? y0row[i] : S(0);
        h = ef > 0 ? a : c0;
    }
    // input projections of all positions first: their loads are all in flight before the
    // cross-lane products start (those are opaque to the scheduler, loads do not move across them)
    S pr[L], pq[L], pc[L];
    gru_project<S, N, L, DP, FULL>(w, xb, gf.d, T, e0, pr, pq, pc, psx);
    gru_rows<S, N, L, DP, FULL>(w, pr, pq, pc, h, yo, T, e0, Ar, be);
}

// slot s of row i of the transposed Jacobian: J[c][i] with c the column slot s refers to, i.e. the row factors of
// lane c times column i of the weights (Tz, Tc, Tr: that column, rows in swizzled order)
template <typename S, int N, int s = 0>
struct DualRow {
    static __device__ __forceinline__ void run(const S* Tz, const S* Tc, const S* Tr, const S* E, S pz, S pzm, S sr, S srm,
                                               S st, S stm, S z, S* out) {
        out[s] = fetch<S, N, s>(pz, pzm) * Tz[s] + (fetch<S, N, s>(sr, srm) * Tc[s] + (fetch<S, N, s>(st, stm) * Tr[s] + z * E[s]));
        if constexpr (s + 1 < N) DualRow<S, N, s + 1>::run(Tz, Tc, Tr, E, pz, pzm, sr, srm, st, stm, z, out);
    }
};

// Matrices of the dual scan (Sec. 3.1.1 eq. 7) from the GRU cell: scan position e carries time T-1-e and the
// transpose of the Jacobian at time T-e, a function of the state at time T-1-e (yv: entry i at the L positions, in
// scan order) and the input at time T-e.  Position 0 has no matrix (zero); positions past the end get the identity.
// Must be called by whole wavefronts.
template <typename S, int N, int L, int DP, bool FULL>
__device__ __forceinline__ void gru_pairs_dual(const GruFeed& gf, const S* __restrict__ xb, long long T, long long e0, int i,
                                               const S* yv, S (*Ar)[N], long long psx) {
    GruRow<S, N, DP> w;
    load_gru_row<S, N, DP>(gf, i, w);
    const int d = gf.d;
    const S* __restrict__ U = reinterpret_cast<const S*>(gf.theta) + 3 * N * d;
    S Tr[N], Tz[N], Tc[N];
#pragma unroll
    for (int s = 0; s < N; ++s) {
        const int c = swz_col<N>(s, i);
        Tr[s] = U[c * N + i];
        Tz[s] = U[(N + c) * N + i];
        Tc[s] = U[(2 * N + c) * N + i];
    }
    S pr[L], pq[L], pc[L];
#pragma unroll
    for (int l = 0; l < L; ++l) {
        long long tj = T - (e0 + l);
        if constexpr (!FULL) {
            tj = tj > T - 1 ? T - 1 : tj;
            tj = tj < 0 ? 0 : tj;
        }
        S ar = w.br, az = w.bz, ac = w.bc;
#pragma unroll
        for (int k = 0; k < DP; ++k) {
            const S xv = xb[tj * psx + (k < d ? k : d - 1)];
            ar += w.Wr[k] * xv;
            az += w.Wz[k] * xv;
            ac += w.Wc[k] * xv;
        }
        pr[l] = ar; pq[l] = az; pc[l] = ac;
    }
#pragma unroll
    for (int l = 0; l < L; ++l) {
        S h = yv[l];
        S ar = pr[l], az = pq[l], ac = pc[l], q = w.bh;
        row_dots<S, N, 1>(w.Ur, &h, &ar);
        row_dots<S, N, 1>(w.Uz, &h, &az);
        row_dots<S, N, 1>(w.Uc, &h, &q);
        const S r = feed_sigmoid(ar), z = feed_sigmoid(az);
        const S c = feed_tanh(ac + r * q);
        const S pz = (h - c) * z * (S(1) - z);
        const S sc = (S(1) - z) * (S(1) - c * c);
        const S sr = sc * r;
        const S st = sc * q * r * (S(1) - r);
        S row[N];
        DualRow<S, N>::run(Tz, Tc, Tr, w.E, pz, mirror<S, N>(pz), sr, mirror<S, N>(sr), st, mirror<S, N>(st), z, row);
        if constexpr (FULL) {
#pragma unroll
            for (int s = 0; s < N; ++s) Ar[l][s] = row[s];
        } else {
            const long long e = e0 + l;
#pragma unroll
            for (int s = 0; s < N; ++s) Ar[l][s] = (e >= T) ? w.E[s] : (e == 0 ? S(0) : row[s]);
        }
    }
}

// Inclusive log-step scan over the groups of a wavefront.  (M | v): this group's pair, lane i holds
// row i.  Afterwards group g holds pair_g o ... o pair_0.
// seg (a power of two): the groups fall into aligned runs of seg groups that are scanned separately (64 / N or more:
// one run).
template <typename S, int N>
__device__ __forceinline__ void scan_groups(S* M, S& v, int group, int i, int ngroups_active, int seg = 64 / N) {
    constexpr int NG = 64 / N;
#pragma unroll
    for (int d = 1; d < NG; d <<= 1) {
        if (d >= ngroups_active || d >= seg) break;   // uniform
        S Mo[N], vo;
#pragma unroll
        for (int c = 0; c < N; ++c) Mo[c] = __shfl_up(M[c], d * N);
        vo = __shfl_up(v, d * N);
        // (mine) after (other): rows of mine times other
        const S keepv = v;
        S keepM[N], leftM[N];
#pragma unroll
        for (int c = 0; c < N; ++c) keepM[c] = M[c];
        swizzle_row<S, N>(keepM, leftM, i);
        group_apply<S, N>(leftM, keepv, Mo, vo);
        const bool upd = (group & (seg - 1)) >= d;
#pragma unroll
        for (int c = 0; c < N; ++c) M[c] = upd ? Mo[c] : keepM[c];
        v = upd ? vo : keepv;
    }
}

// LDS of one tile
template <typename S, int N, int W>
struct TileShared {
    S M[W][N * N];    // wavefront totals
    S v[W][N];
    S EM[W][N * N];   // prefix in front of each wavefront (exclusive)
    S Ev[W][N];
    S carry[N];       // state entering the tile
    int failed;       // set (never cleared) by tile_carry when a bounded wait ran out
};

// Steps 1b-3 of a tile, all inside the workgroup: composition of the group's L pairs, scan over the
// groups of every wavefront, scan of the wavefront totals by wavefront 0.  Called by all threads (one
// barrier).  Out: (Pex | pex) the prefix of this group inside its wavefront (row i, swizzled); sh.EM/Ev the
// prefixes in front of the wavefronts; in wavefront 0, group W-1: (Mt | vt) the tile total (natural order).
template <typename S, int N, int L, int W>
// seg: wavefronts per sequence when the tile holds W / seg independent short sequences, one per aligned run of seg
// wavefronts (W: the tile belongs to one sequence); the prefixes then restart at every run.
__device__ __forceinline__ void tile_local(const ScanParams& p, TileShared<S, N, W>& sh, const S (*Ar)[N], const S* be,
                                           long long seq0, int t, S* Pex, S& pex, S* Mt, S& vt, int seg = W) {
    constexpr int NG = 64 / N;
    static_assert(NG >= W, "wavefront 0 scans one wavefront total per group");
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int group = lane / N;
    const int i = lane % N;
    const long long slot = seq0 + t;
    (void)slot;
    S M[N], v;
#pragma unroll
    for (int c = 0; c < N; ++c) M[c] = (c == i) ? S(1) : S(0);
    v = S(0);
#pragma unroll
    for (int l = 0; l < L; ++l) group_apply<S, N>(Ar[l], be[l], M, v);

    // ---- 2. scan over the groups of the wavefront; keep the exclusive prefix ----
    scan_groups<S, N>(M, v, group, i, NG);
    if (group == NG - 1) {
#pragma unroll
        for (int c = 0; c < N; ++c) sh.M[wave][i * N + c] = M[c];
        sh.v[wave][i] = v;
    }
    {
        S nat[N];
#pragma unroll
        for (int c = 0; c < N; ++c) {
            const S u = __shfl_up(M[c], N);
            nat[c] = group == 0 ? ((c == i) ? S(1) : S(0)) : u;
        }
        swizzle_row<S, N>(nat, Pex, i);
        const S u = __shfl_up(v, N);
        pex = group == 0 ? S(0) : u;
    }
    __syncthreads();

    // ---- 3. wavefront 0: scan of the wavefront totals; 4. look-back ----
    DEER_STAMP(p, slot, 1, tid == 0);
    if (wave == 0) {
        {
            // groups beyond the number of wavefronts hold the identity pair
            const bool has = group < W;
            const int gw = has ? group : W - 1;
#pragma unroll
            for (int c = 0; c < N; ++c) {
                const S u = sh.M[gw][i * N + c];
                Mt[c] = has ? u : ((c == i) ? S(1) : S(0));
            }
            const S u = sh.v[gw][i];
            vt = has ? u : S(0);
        }
        scan_groups<S, N>(Mt, vt, group, i, W, seg);
        // group g now holds the prefix through wavefront g: it is the prefix in front of wavefront g+1 (the identity
        // where a new sequence starts)
        if (group < W - 1) {
            const bool fresh = ((group + 1) & (seg - 1)) == 0;
#pragma unroll
            for (int c = 0; c < N; ++c) sh.EM[group + 1][i * N + c] = fresh ? ((c == i) ? S(1) : S(0)) : Mt[c];
            sh.Ev[group + 1][i] = fresh ? S(0) : vt;
        }
    }
}

// Step 4 of a tile: publication of the tile total and the look-back along sequence b (tile t of p.tiles;
// tags carry `epoch`).  Called by all threads; ends with a barrier after which sh.carry holds the state
// entering the tile.  (Mt | vt): the tile total as left by tile_local.
template <typename S, int N, int W>
__device__ __forceinline__ void tile_lookback(const ScanParams& p, TileShared<S, N, W>& sh, long long seq0, int t, unsigned epoch,
                                              const S* Mt, S vt, const S* y0row) {   // y0row: initial state of this sequence or nullptr (zeros)
    constexpr int NG = 64 / N;
    constexpr int WS = TaggedWords<S>::per_scalar;
    constexpr int AGG_WORDS = (N * N + N) * WS;   // words of one published tile total
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int group = lane / N;
    const int i = lane % N;
    const long long slot = seq0 + t;
    (void)tid;
    if (wave == 0) {
        const unsigned tagA = (epoch << 2) | TILE_AGGREGATE;
        const unsigned tagI = (epoch << 2) | TILE_INCLUSIVE;
        const unsigned long long* aggSeq = p.aggW + seq0 * AGG_WORDS;
        const unsigned long long* inclSeq = p.inclW + seq0 * (N * WS);
        if (t > 0 && group == W - 1) {
            unsigned long long* mine = p.aggW + slot * AGG_WORDS;
#pragma unroll
            for (int c = 0; c < N; ++c) TaggedWords<S>::put(mine, i * N + c, Mt[c], tagA);
            TaggedWords<S>::put(mine, N * N + i, vt, tagA);
        }
        DEER_STAMP(p, slot, 2, lane == 0);

        // lane j inspects predecessor t-1-j (index -1 is the given initial state): inclusive carry
        // known, total known, or nothing yet, judged by one word of each
        int k = -1;
        {
            const int idx = t - 1 - lane;
            unsigned spins = 0;
            while (true) {
                unsigned st;
                if (idx >= 0) {
                    S dummy;
                    if (TaggedWords<S>::get(inclSeq + (long long)idx * (N * WS), 0, tagI, dummy)) st = TILE_INCLUSIVE;
                    else if (TaggedWords<S>::get(aggSeq + (long long)idx * AGG_WORDS, N * N, tagA, dummy)) st = TILE_AGGREGATE;
                    else st = TILE_INVALID;
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
                __builtin_amdgcn_s_sleep(1);
            }
        }
        DEER_STAMP(p, slot, 3, lane == 0);

        // carry: entry i in the lanes of group 0
        S y = S(0);
        bool ok = k >= 0;
        if (ok) {
            const int far = t - 1 - k;   // tile whose inclusive carry is known (-1: the initial state)
            if (group == 0) {
                if (far >= 0) ok = tagged_get_wait<S>(inclSeq + (long long)far * (N * WS), i, tagI, y);
                else if (y0row) y = y0row[i];
            }
            // fold the totals of tiles far+1 .. t-1 forward, NG of them per round: group g fetches
            // tile q0 + g, then the running value walks through the groups in order
            for (int q0 = far + 1; q0 <= t - 1; q0 += NG) {
                const int q = q0 + group;
                const bool valid = q <= t - 1;
                S Lr[N], hv;
                {
                    // groups past the last predecessor re-read it and then act as the identity pair
                    const unsigned long long* src = aggSeq + (long long)(valid ? q : t - 1) * AGG_WORDS;
                    // all words are requested at once; the per-word wait is only a fallback for the
                    // rare case that a word of a total is still in flight when its first word is seen
                    S row[N], u;
                    bool got = true;
#pragma unroll
                    for (int c = 0; c < N; ++c) got = TaggedWords<S>::get(src, i * N + swz_col<N>(c, i), tagA, row[c]) && got;
                    got = TaggedWords<S>::get(src, N * N + i, tagA, u) && got;
                    if (__ballot(!got) != 0ull) {
#pragma unroll
                        for (int c = 0; c < N; ++c) ok = tagged_get_wait<S>(src, i * N + swz_col<N>(c, i), tagA, row[c]) && ok;
                        ok = tagged_get_wait<S>(src, N * N + i, tagA, u) && ok;
                    }
                    hv = valid ? u : S(0);
#pragma unroll
                    for (int c = 0; c < N; ++c) Lr[c] = valid ? row[c] : ((swz_col<N>(c, i) == i) ? S(1) : S(0));
                }
#pragma unroll 1
                for (int g = 0; g < NG; ++g) {
                    const S ny = group_matvec<S, N>(Lr, hv, y);
                    if (group == g) y = ny;
                    const S pass = __shfl_up(y, N);
                    if (group == g + 1) y = pass;
                }
                // the running value sits in the last group: bring it back to group 0
                const S back = __shfl(y, i + (NG - 1) * N);
                if (group == 0) y = back;
            }
        }
        if (__ballot(!ok) != 0ull) {
            if (lane == 0) {
                atomicOr(p.status, 1u);
                sh.failed = 1;
            }
        }
        DEER_STAMP(p, slot, 4, lane == 0);
#ifdef DEER_SCAN_TIMING
        if (p.timing && lane == 0) p.timing[slot * 16 + 7] = (unsigned long long)(k < 0 ? 0 : k);
#endif
        if (group == 0) sh.carry[i] = y;
        // inclusive carry of this tile: (tile total) applied to the carry
        if (group == W - 1) {
            const S c = sh.carry[i];
            S left[N];
            swizzle_row<S, N>(Mt, left, i);
            TaggedWords<S>::put(p.inclW + slot * (N * WS), i, group_matvec<S, N>(left, vt, c), tagI);
        }
        DEER_STAMP(p, slot, 5, lane == 0);
    }
    __syncthreads();

}

// Step 4 with the work spread over two wavefronts.  While wavefront 0 is still scanning the wavefront totals
// (end of tile_local), wavefront 1 already looks for the state entering the tile; wavefront 0 publishes the
// tile total when it has it, and the inclusive carry after the barrier.  The first poll asks for everything it
// is likely to need in the same round trip: lane j reads the state of predecessor t-1-j as in
// tile_lookback, and group g also reads the inclusive carry and the total of predecessor t-1-g.  If the
// nearest predecessor with a known carry is among those and all words have arrived, the carry is folded
// forward through the groups at once.  Otherwise the search goes on exactly as in tile_lookback (light
// polls, then one fetch).  Called by all threads after tile_local; ends like tile_lookback.
template <typename S, int N, int W>
__device__ __forceinline__ void tile_lookback_split(const ScanParams& p, TileShared<S, N, W>& sh, long long seq0, int t,
                                                    unsigned epoch, const S* Mt, S vt, const S* y0row) {
    static_assert(W >= 2, "one wavefront publishes while another looks back");
    constexpr int NG = 64 / N;
    constexpr int WS = TaggedWords<S>::per_scalar;
    constexpr int AGG_WORDS = (N * N + N) * WS;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int group = lane / N;
    const int i = lane % N;
    const long long slot = seq0 + t;
    (void)slot;
    const unsigned tagA = (epoch << 2) | TILE_AGGREGATE;
    const unsigned tagI = (epoch << 2) | TILE_INCLUSIVE;
    if (wave == 0) {
        if (t > 0 && group == W - 1) {
            unsigned long long* mine = p.aggW + slot * AGG_WORDS;
#pragma unroll
            for (int c = 0; c < N; ++c) TaggedWords<S>::put(mine, i * N + c, Mt[c], tagA);
            TaggedWords<S>::put(mine, N * N + i, vt, tagA);
        }
        DEER_STAMP(p, slot, 2, lane == 0);
    } else if (wave == 1) {
        const unsigned long long* aggSeq = p.aggW + seq0 * AGG_WORDS;
        const unsigned long long* inclSeq = p.inclW + seq0 * (N * WS);
        int k = -1;
        bool fast = false;
        S Lr[N], hv = S(0), cv = S(0);
        {
            const int idx = t - 1 - lane;     // predecessor whose state this lane inspects
            const int qs = t - 1 - group;     // predecessor whose words this group reads ahead (first poll only)
            unsigned spins = 0;
            while (true) {
                unsigned st;
                if (idx >= 0) {
                    S dummy;
                    if (TaggedWords<S>::get(inclSeq + (long long)idx * (N * WS), 0, tagI, dummy)) st = TILE_INCLUSIVE;
                    else if (TaggedWords<S>::get(aggSeq + (long long)idx * AGG_WORDS, N * N, tagA, dummy)) st = TILE_AGGREGATE;
                    else st = TILE_INVALID;
                } else {
                    st = (idx == -1) ? TILE_INCLUSIVE : 3u;
                }
                bool gotA = false, gotI = false;
                if (spins == 0) {
                    if (qs >= 0) {
                        const unsigned long long* src = aggSeq + (long long)qs * AGG_WORDS;
                        gotA = true;
#pragma unroll
                        for (int c = 0; c < N; ++c) gotA = TaggedWords<S>::get(src, i * N + swz_col<N>(c, i), tagA, Lr[c]) && gotA;
                        gotA = TaggedWords<S>::get(src, N * N + i, tagA, hv) && gotA;
                        gotI = TaggedWords<S>::get(inclSeq + (long long)qs * (N * WS), i, tagI, cv);
                    } else if (qs == -1) {
                        gotI = true;
                        cv = y0row ? y0row[i] : S(0);
                    }
                }
                const unsigned long long incl_mask = __ballot(st == TILE_INCLUSIVE);
                const unsigned long long wait_mask = __ballot(st == TILE_INVALID);
                if (incl_mask != 0ull) {
                    const int first = __ffsll((long long)incl_mask) - 1;
                    const unsigned long long below = (first == 0) ? 0ull : ((1ull << first) - 1ull);
                    if ((wait_mask & below) == 0ull) {
                        k = first;
                        if (spins == 0 && k < NG) {
                            const unsigned long long a_mask = __ballot(gotA), i_mask = __ballot(gotI);
                            const unsigned long long needA = (k == 0) ? 0ull : ((1ull << (k * N)) - 1ull);
                            const unsigned long long needI = ((1ull << N) - 1ull) << (k * N);
                            fast = (a_mask & needA) == needA && (i_mask & needI) == needI;
                        }
                        break;
                    }
                }
                if (++spins > kSpinLimit) break;
                __builtin_amdgcn_s_sleep(1);
            }
        }
        DEER_STAMP(p, slot, 3, lane == 0);
        S y = S(0);
        bool ok = k >= 0;
        if (ok && fast) {
            // group k holds the known carry, groups k-1 .. 0 the totals to apply, nearest predecessor last
            y = cv;
            for (int g = k - 1; g >= 0; --g) {
                const S pass = __shfl_down(y, N);
                const S ny = group_matvec<S, N>(Lr, hv, pass);
                if (group == g) y = ny;
            }
        } else if (ok) {
            const int far = t - 1 - k;   // tile whose inclusive carry is known (-1: the initial state)
            if (group == 0) {
                if (far >= 0) ok = tagged_get_wait<S>(inclSeq + (long long)far * (N * WS), i, tagI, y);
                else if (y0row) y = y0row[i];
            }
            for (int q0 = far + 1; q0 <= t - 1; q0 += NG) {
                const int q = q0 + group;
                const bool valid = q <= t - 1;
                const unsigned long long* src = aggSeq + (long long)(valid ? q : t - 1) * AGG_WORDS;
                S row[N], u;
                bool got = true;
#pragma unroll
                for (int c = 0; c < N; ++c) got = TaggedWords<S>::get(src, i * N + swz_col<N>(c, i), tagA, row[c]) && got;
                got = TaggedWords<S>::get(src, N * N + i, tagA, u) && got;
                if (__ballot(!got) != 0ull) {
#pragma unroll
                    for (int c = 0; c < N; ++c) ok = tagged_get_wait<S>(src, i * N + swz_col<N>(c, i), tagA, row[c]) && ok;
                    ok = tagged_get_wait<S>(src, N * N + i, tagA, u) && ok;
                }
                hv = valid ? u : S(0);
#pragma unroll
                for (int c = 0; c < N; ++c) Lr[c] = valid ? row[c] : ((swz_col<N>(c, i) == i) ? S(1) : S(0));
#pragma unroll 1
                for (int g = 0; g < NG; ++g) {
                    const S ny = group_matvec<S, N>(Lr, hv, y);
                    if (group == g) y = ny;
                    const S pass = __shfl_up(y, N);
                    if (group == g + 1) y = pass;
                }
                const S back = __shfl(y, i + (NG - 1) * N);
                if (group == 0) y = back;
            }
        }
        if (__ballot(!ok) != 0ull) {
            if (lane == 0) {
                atomicOr(p.status, 1u);
                sh.failed = 1;
            }
        }
        DEER_STAMP(p, slot, 4, lane == 0);
        if (group == 0) sh.carry[i] = y;
    }
    __syncthreads();
    if (wave == 0) {
        // inclusive carry of this tile: (tile total) applied to the carry
        const S c = sh.carry[i];
        S left[N];
        swizzle_row<S, N>(Mt, left, i);
        const S incl = group_matvec<S, N>(left, vt, c);
        if (group == W - 1) TaggedWords<S>::put(p.inclW + slot * (N * WS), i, incl, tagI);
        DEER_STAMP(p, slot, 5, lane == 0);
    }
}

// Steps 1b-4 in one go (see tile_local, tile_lookback and tile_lookback_split).
template <typename S, int N, int L, int W, bool SPLIT = false>
__device__ __forceinline__ void tile_carry(const ScanParams& p, TileShared<S, N, W>& sh, const S (*Ar)[N], const S* be,
                                           long long seq0, int t, unsigned epoch, S* Pex, S& pex, const S* y0row, int seg = W) {
    S Mt[N], vt = S(0);
#pragma unroll
    for (int c = 0; c < N; ++c) Mt[c] = S(0);
    tile_local<S, N, L, W>(p, sh, Ar, be, seq0, t, Pex, pex, Mt, vt, seg);
    if constexpr (SPLIT) tile_lookback_split<S, N, W>(p, sh, seq0, t, epoch, Mt, vt, y0row);
    else tile_lookback<S, N, W>(p, sh, seq0, t, epoch, Mt, vt, y0row);
}

// Step 5a: the state in front of this group's first position (entry i), from the tile's carry
template <typename S, int N, int W>
__device__ __forceinline__ S tile_start_state(const TileShared<S, N, W>& sh, const S* Pex, S pex, int wave, int i) {
    S y = sh.carry[i];
    if (wave > 0) {
        S row[N];
#pragma unroll
        for (int c = 0; c < N; ++c) row[c] = sh.EM[wave][i * N + swz_col<N>(c, i)];
        y = group_matvec<S, N>(row, sh.Ev[wave][i], y);
    }
    y = group_matvec<S, N>(Pex, pex, y);

    return y;
}

// DP = 0: pairs are read from p.A / p.bv.  DP > 0: pairs come from the GRU cell, DP being the input width the x
// loops are unrolled for: forward, the Newton step at the previous iterate p.yold; with REV, the dual scan with
// the transposed Jacobians at the trajectory p.yold and the vectors from p.bv (no convergence measure).  ADDI: the stored matrices are A - I (the identity
// is added on load; used by the dual recurrence of the ODE form, whose matrices are I + O(dt)).
// MH (with DP > 0): the launch's sequences are the strided heads of a multi-head GRU (Sec. 4.4, App. B.4).  Arrays are
// [batch][time][head][channel]; head h has its own parameters (gf.theta + h * p.mh_P) and looks back s = 2^(h mod p.mh_K)
// steps, so it falls into s independent recurrences over the times r, r + s, r + 2s, ...; each is a sequence of the scan:
// its positions lie s * H * N scalars apart and its length is ceil((T - r) / s).  The launch's tiles are the tiles of all
// recurrences of all p.B batch entries, listed in p.mh_table.
template <typename S, int N, int L, int W, bool REV, int DP, bool ADDI = false, bool MH = false>
__global__ __launch_bounds__(64 * W) void scan_valu_kernel(ScanParams p, GruFeed gf) {
    constexpr bool DUAL = DP > 0 && REV;
    static_assert(!ADDI || DP == 0, "only stored matrices can lack their identity");
    static_assert(!MH || DP > 0, "strided heads exist for the GRU feed only");
    constexpr int NG = 64 / N;        // groups per wavefront
    constexpr int TILE = W * NG * L;  // scan positions per tile

    __shared__ unsigned s_ticket;
    __shared__ TileShared<S, N, W> sh;
    constexpr bool STAGED = DP == 0 && !REV && !ADDI && sizeof(S) == 4 && Staged<N, L>::use;
    __shared__ uint4 s_stage[STAGED ? W : 1][Staged<N, L>::U4];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int group = lane / N;
    const int i = lane % N;

    if (gate_closed<S>(p.gate)) return;
    if (tid == 0) s_ticket = atomicAdd(p.ticket, 1u);
    __syncthreads();
    const unsigned tk = s_ticket;
    const int b = (int)(tk % (unsigned)p.B);
    int t = (int)(tk / (unsigned)p.B);
    if (t >= p.tiles) return;
    long long seq0 = (long long)b * p.tiles;   // slot of the sequence's first tile in the published-word regions

    const S* __restrict__ Ab = reinterpret_cast<const S*>(p.A) + (long long)b * p.strideA;
    const S* __restrict__ bb = reinterpret_cast<const S*>(p.bv) + (long long)b * p.strideb;
    S* __restrict__ ob = reinterpret_cast<S*>(p.out) + (long long)b * p.strideOut;
    const S* __restrict__ oldb =
        p.yold ? reinterpret_cast<const S*>(p.yold) + (long long)b * p.strideOld : nullptr;
    long long T = p.T;
    int seg = W, wv = wave;          // wavefronts per sequence in this tile and this wavefront's index among them (multi-head)
    long long psy = N, psx = gf.d;   // scalars between consecutive positions of the trajectory and of the inputs
    const S* __restrict__ xb = nullptr;
    const S* __restrict__ y0row = nullptr;
    if constexpr (!MH) {
        if constexpr (DP > 0) xb = reinterpret_cast<const S*>(gf.x) + (long long)b * T * gf.d;
        if (p.y0) y0row = reinterpret_cast<const S*>(p.y0) + (long long)b * N;
    }
    if constexpr (MH) {
        // p.tiles counts the tiles of one batch entry over all its recurrences; the table lists them head by head,
        // recurrence by recurrence, tile by tile: head (6 bits) | first time index r (7 bits) | log2 of the recurrences
        // packed into the tile (2 bits) | tile (17 bits).  The tiles of a recurrence are consecutive entries, so its
        // published words are consecutive slots.  Short recurrences share a tile: 2^pack of them (same head, first time
        // indices r, r + 1, ...), each on an aligned run of W >> pack wavefronts, each starting from the head's y0.
        const int H = p.mh_H;
        const int entry = t;
        const unsigned ent = p.mh_table[entry];
        const int h = (int)(ent >> 26);
        const int lp = (int)((ent >> 17) & 3u);
        seg = W >> lp;
        const int r = (int)((ent >> 19) & 127u) + wave / seg;
        wv = wave & (seg - 1);
        t = (int)(ent & 0x1ffffu);
        seq0 = (long long)b * p.tiles + entry - t;
        const long long bi = b;
        const long long s = 1LL << (h % p.mh_K);
        const long long Tfull = p.T;
        T = (Tfull - r + s - 1) / s;
        psy = s * H * N;
        psx = s * H * (long long)gf.d;
        const long long first = ((bi * Tfull + r) * H + h);
        ob = reinterpret_cast<S*>(p.out) + first * N;
        oldb = reinterpret_cast<const S*>(p.yold) + first * N;
        bb = reinterpret_cast<const S*>(p.bv) + first * N;
        xb = reinterpret_cast<const S*>(gf.x) + first * gf.d;
        if (p.y0) y0row = reinterpret_cast<const S*>(p.y0) + (bi * H + h) * N;
        gf.theta = reinterpret_cast<const S*>(gf.theta) + (long long)h * p.mh_P;
    }
    const long long e0 = (long long)t * TILE + (long long)(wv * NG + group) * L;
    const long long slot = seq0 + t;
    DEER_STAMP(p, slot, 0, tid == 0);

    // ---- 1. this group's pairs (kept for the second walk), then their composition ----
    // A tile that lies completely inside the sequence takes the FULL variants: one base address with
    // constant offsets and no end-of-sequence handling.
    // (per wavefront where short sequences share the tile)
    const bool full = (MH && seg < W) ? (!REV && (long long)(wv + 1) * (NG * L) <= T)
                                      : ((long long)(t + 1) * TILE <= T && (!REV || t > 0));
    S Ar[L][N], be[L], yo[L];
    if (full) {
        if constexpr (STAGED) {
            if constexpr (!Staged<N, L>::useA) load_pairs<S, N, L, REV, true, ADDI, true>(Ab, bb, T, e0, i, Ar, be);
            load_pairs_staged<N, L>(Ab, bb, (long long)t * TILE + (long long)wave * (NG * L), lane, reinterpret_cast<staged_piece*>(s_stage[wave]), Ar, be);
        } else if constexpr (DP == 0) {
            load_pairs<S, N, L, REV, true, ADDI>(Ab, bb, T, e0, i, Ar, be);
        }
        if constexpr (DP == 0 && N <= 4) {
            // (without a previous iterate nothing is loaded; measured +6 % at n = 4, while the n = 8 kernel, at
            // its register limit, is a few per cent slower with the branch and keeps the unconditional loads)
            if (oldb) load_previous<S, N, L, REV, true>(oldb, T, e0, i, yo);
            else {
#pragma unroll
                for (int l = 0; l < L; ++l) yo[l] = S(0);
            }
        } else {
            load_previous<S, N, L, REV, true>(oldb ? oldb : bb, T, e0, i, yo, psy);
        }
        if constexpr (DP > 0 && !REV) gru_pairs<S, N, L, DP, true>(gf, xb, y0row, oldb, T, e0, i, yo, Ar, be, psy, psx);
        if constexpr (DUAL) {
            load_previous<S, N, L, true, true>(bb, T, e0, i, be, psy);
            gru_pairs_dual<S, N, L, DP, true>(gf, xb, T, e0, i, yo, Ar, psx);
        }
    } else {
        if constexpr (DP == 0) load_pairs<S, N, L, REV, false, ADDI>(Ab, bb, T, e0, i, Ar, be);
        load_previous<S, N, L, REV, false>(oldb ? oldb : bb, T, e0, i, yo, psy);
        if constexpr (DP > 0 && !REV) gru_pairs<S, N, L, DP, false>(gf, xb, y0row, oldb, T, e0, i, yo, Ar, be, psy, psx);
        if constexpr (DUAL) {
            load_previous<S, N, L, true, false>(bb, T, e0, i, be, psy);
#pragma unroll
            for (int l = 0; l < L; ++l) be[l] = (e0 + l < T) ? be[l] : S(0);
            gru_pairs_dual<S, N, L, DP, false>(gf, xb, T, e0, i, yo, Ar, psx);
        }
    }
    S Pex[N], pex;
    // plain scans of n <= 4 look back on wavefront 1 while wavefront 0 scans the wavefront totals (measured on
    // chip-filling streams: +5 % at n = 4, +12 % at n = 2; at n = 8 the extra registers cost more than it gains)
    tile_carry<S, N, L, W, DP == 0 && N <= 4>(p, sh, Ar, be, seq0, t, p.epoch, Pex, pex, y0row, seg);

    // ---- 5. starting state of this group, then the second walk over the resident pairs ----
    S y = tile_start_state<S, N, W>(sh, Pex, pex, wave, i);

    S emax = S(0);
    S wout[STAGED ? L : 1];
#pragma unroll
    for (int l = 0; l < L; ++l) {
        const long long e = e0 + l;
        y = group_matvec<S, N>(Ar[l], be[l], y);
        if (full || e < T) {
            const long long oi = (REV ? (T - 1 - e) : e) * psy + i;
            S w = y;
            if (!DUAL && oldb) {
                const S dq = abs_or_inf<S>(p.delta ? y : y - yo[l]);
                emax = dq > emax ? dq : emax;
                if (p.delta) w += yo[l];
            }
            if constexpr (STAGED) {
                if (full) wout[l] = w;
                else ob[oi] = w;
            } else {
                ob[oi] = w;
            }
        }
    }
    if constexpr (STAGED) {
        if (full)
            store_staged<N, L>(ob, (long long)t * TILE + (long long)wave * (NG * L), lane,
                               reinterpret_cast<staged_piece*>(s_stage[wave]), wout);
    }
    if (p.err) {
        emax = wave_max<S>(emax);
        if (lane == 0) err_atomic_max(p.err, emax);
    }
    DEER_STAMP(p, slot, 6, tid == 0);
}

}  // namespace

}  // namespace deer
