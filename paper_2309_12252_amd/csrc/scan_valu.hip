// Inverse linear operator for small state sizes (n <= 8): single-pass blocked associative scan
// over affine pairs (A | b) with the operator of Sec. 3.3 eq. 10, on the vector ALUs with DPP
// cross-lane operands.
//
// Data layout in registers: a pair is spread over the n consecutive lanes of a "group"; lane i of
// the group holds row i of the matrix (n registers) and entry i of the vector.  A wavefront holds
// 64/n groups.  The product of two matrices needs, in lane i, row i of the left factor (own
// registers) and every row of the right factor (the other lanes of the same group); those come in
// through DPP moves (quad_perm broadcasts inside a quad; for n = 8 two bank-masked row shifts first
// make every lane see the lower and the upper quad of its group), so a product costs n*n
// multiply-adds per lane and no LDS traffic.  Global loads are coalesced: a group reads the n*n
// contiguous scalars of its matrix.
//
// Structure of one tile (WAVES wavefronts, L scan positions per group, WAVES * 64/n * L per tile):
//   1. every group loads its L consecutive pairs into registers and composes them serially;
//   2. the groups of a wavefront are scanned with a log-step scan (shuffles by whole groups);
//   3. wavefront totals meet in LDS; wavefront 0 scans them the same way, which gives the tile total
//      and the prefix in front of every wavefront;
//   4. tiles of one sequence are chained through HBM by decoupled look-back: a tile publishes its
//      total (state AGGREGATE), inspects up to 64 predecessors at once, and folds their totals
//      forward from the nearest predecessor whose inclusive carry is known (state INCLUSIVE); the
//      totals are fetched by all groups in parallel, one predecessor per group, and applied in
//      order.  Only the vector part of the carry is needed, so the fold is matrix-vector work.
//      Published data travels as self-validating tagged words (no fences, no cache maintenance).
//      Tiles take their index from an atomic ticket, so every predecessor of a running tile has
//      started, which makes the waiting deadlock free; waits are bounded anyway;
//   5. every group turns the carry into its own starting state and walks its register-resident
//      pairs again (y <- A y + b), writing y and reducing max|y - y_previous_iterate| for the
//      convergence test.  The matrices are read from HBM exactly once.
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

// For n = 8 a group is two quads.  lower_copy(x): every lane gets x from the lower quad's lane at its
// own position (row_shr:4 written only in the upper quads); upper_copy(x) the other way round
// (row_shl:4 written only in the lower quads).  A quad broadcast of these copies then delivers row s
// of the group to all 8 lanes.
template <typename S, int N>
__device__ __forceinline__ S lower_copy(S x) {
    if constexpr (N == 8) return dpp<0x114, 0xA, false>(x, x);
    else return x;
}
template <typename S, int N>
__device__ __forceinline__ S upper_copy(S x) {
    if constexpr (N == 8) return dpp<0x104, 0x5, false>(x, x);
    else return x;
}
// value of x held by lane s of the group (xa, xb: lower_copy / upper_copy of x)
template <typename S, int N, int s>
__device__ __forceinline__ S fetch(S xa, S xb) {
    if constexpr (N == 1) return xa;
    else if constexpr (N == 2) return dpp<(s == 0 ? 0xA0 : 0xF5), 0xf, true>(S(0), xa);
    else if constexpr (N == 4) return quad_bcast<s>(xa);
    else if constexpr (s < 4) return quad_bcast<s>(xa);
    else return quad_bcast<s - 4>(xb);
}

// acc += sum_s Lr[s] * (value of x in lane s of the group)
template <typename S, int N, int s = 0>
struct RowDot {
    static __device__ __forceinline__ void run(const S* Lr, S xa, S xb, S& acc) {
        acc += Lr[s] * fetch<S, N, s>(xa, xb);
        if constexpr (s + 1 < N) RowDot<S, N, s + 1>::run(Lr, xa, xb, acc);
    }
};

#include "scan_valu_dpp.inc"

// acc[0..K) += sum_s Lr[s] * (column value in lane s of the group), K columns given in x
template <typename S, int N, int K>
__device__ __forceinline__ void row_dots(const S* Lr, const S* x, S* acc) {
    if constexpr (sizeof(S) == 4 && N == 8 && (K == 4 || K == 1)) {
        float xa[K], xb[K];
#pragma unroll
        for (int c = 0; c < K; ++c) { xa[c] = lower_copy<float, 8>(x[c]); xb[c] = upper_copy<float, 8>(x[c]); }
        if constexpr (K == 4) dpp_dot8_4(Lr, xa, xb, acc); else dpp_dot8_1(Lr, xa, xb, acc);
    } else if constexpr (sizeof(S) == 4 && N == 4 && (K == 4 || K == 1)) {
        if constexpr (K == 4) dpp_dot4_4(Lr, x, acc); else dpp_dot4_1(Lr, x, acc);
    } else if constexpr (sizeof(S) == 4 && N == 2 && (K == 2 || K == 1)) {
        if constexpr (K == 2) dpp_dot2_2(Lr, x, acc); else dpp_dot2_1(Lr, x, acc);
    } else {
#pragma unroll
        for (int c = 0; c < K; ++c) RowDot<S, N>::run(Lr, lower_copy<S, N>(x[c]), upper_copy<S, N>(x[c]), acc[c]);
    }
}

// Lr: row i of the left matrix.  (M | v): right pair, lane i holds row i / entry i.
// Result: row i of Lmat * M and entry i of Lmat * v + add.
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

// Row i of the matrix at scan position e of one sequence and entry i of its vector.
// Reverse mode: vector index T-1-e, matrix = transpose of the one stored at index T-e, zero for e = 0.
// Branch free on purpose (positions past the end read the last valid one and are then replaced by the
// identity pair): with straight-line code the compiler keeps the loads in order and lets the first
// products start while later positions are still in flight.
template <typename S, int N, bool REV>
__device__ __forceinline__ void load_row(const S* __restrict__ Ab, const S* __restrict__ bb, long long T,
                                         long long e, int i, S* Lr, S& bi) {
    const bool past = e >= T;
    const long long ec = past ? T - 1 : e;
    S row[N], bv;
    if constexpr (!REV) {
        vload<S, N>(row, Ab + ec * (N * N) + i * N);
        bv = bb[ec * N + i];
    } else {
        bv = bb[(T - 1 - ec) * N + i];
        const long long em = ec == 0 ? 1 : ec;   // position 0 has no matrix; any valid one is read and dropped
        const S* mat = Ab + (T - em) * (N * N);
#pragma unroll
        for (int s = 0; s < N; ++s) row[s] = (T > 1) ? mat[s * N + i] : S(0);
        if (ec == 0) {
#pragma unroll
            for (int s = 0; s < N; ++s) row[s] = S(0);
        }
    }
#pragma unroll
    for (int s = 0; s < N; ++s) Lr[s] = past ? ((s == i) ? S(1) : S(0)) : row[s];
    bi = past ? S(0) : bv;
}

// Inclusive log-step scan over the groups of a wavefront.  (M | v): this group's pair, lane i holds
// row i.  Afterwards group g holds pair_g o ... o pair_0.
template <typename S, int N>
__device__ __forceinline__ void scan_groups(S* M, S& v, int group, int ngroups_active) {
    constexpr int NG = 64 / N;
#pragma unroll
    for (int d = 1; d < NG; d <<= 1) {
        if (d >= ngroups_active) break;   // uniform
        S Mo[N], vo;
#pragma unroll
        for (int c = 0; c < N; ++c) Mo[c] = __shfl_up(M[c], d * N);
        vo = __shfl_up(v, d * N);
        // (mine) after (other): rows of mine times other
        const S keepv = v;
        S keepM[N];
#pragma unroll
        for (int c = 0; c < N; ++c) keepM[c] = M[c];
        group_apply<S, N>(keepM, keepv, Mo, vo);
        const bool upd = group >= d;
#pragma unroll
        for (int c = 0; c < N; ++c) M[c] = upd ? Mo[c] : keepM[c];
        v = upd ? vo : keepv;
    }
}

template <typename S, int N, int L, int W, bool REV>
__global__ __launch_bounds__(64 * W) void scan_valu_kernel(ScanParams p) {
    constexpr int NG = 64 / N;        // groups per wavefront
    constexpr int TILE = W * NG * L;  // scan positions per tile
    constexpr int WS = TaggedWords<S>::per_scalar;
    constexpr int AGG_WORDS = (N * N + N) * WS;   // words of one published tile total
    static_assert(NG >= W, "wavefront 0 scans one wavefront total per group");

    __shared__ unsigned s_ticket;
    __shared__ S sM[W][N * N];    // wavefront totals
    __shared__ S sv[W][N];
    __shared__ S sEM[W][N * N];   // prefix in front of each wavefront (exclusive)
    __shared__ S sEv[W][N];
    __shared__ S sCarry[N];

    if (gate_closed<S>(p.gate)) return;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int group = lane / N;
    const int i = lane % N;

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
    const long long T = p.T;
    const long long e0 = (long long)t * TILE + (long long)(wave * NG + group) * L;
    const long long slot = (long long)b * p.tiles + t;
    DEER_STAMP(p, slot, 0, tid == 0);

    // ---- 1. load this group's pairs (kept for the second walk) and compose them ----
    S Ar[L][N], be[L];
#pragma unroll
    for (int l = 0; l < L; ++l) load_row<S, N, REV>(Ab, bb, T, e0 + l, i, Ar[l], be[l]);
    // the previous iterate at this group's positions, requested now so that it is there for step 5
    S yo[L];
#pragma unroll
    for (int l = 0; l < L; ++l) {
        const long long e = (e0 + l < T) ? e0 + l : T - 1;
        const S* src = oldb ? oldb : bb;   // branch free: without a previous iterate the value is unused
        yo[l] = src[(REV ? (T - 1 - e) : e) * N + i];
    }
    S M[N], v;
#pragma unroll
    for (int c = 0; c < N; ++c) M[c] = (c == i) ? S(1) : S(0);
    v = S(0);
#pragma unroll
    for (int l = 0; l < L; ++l) group_apply<S, N>(Ar[l], be[l], M, v);

    // ---- 2. scan over the groups of the wavefront; keep the exclusive prefix ----
    scan_groups<S, N>(M, v, group, NG);
    if (group == NG - 1) {
#pragma unroll
        for (int c = 0; c < N; ++c) sM[wave][i * N + c] = M[c];
        sv[wave][i] = v;
    }
    S Pex[N], pex;   // exclusive prefix of this group inside its wavefront (row i)
    {
#pragma unroll
        for (int c = 0; c < N; ++c) {
            const S u = __shfl_up(M[c], N);
            Pex[c] = group == 0 ? ((c == i) ? S(1) : S(0)) : u;
        }
        const S u = __shfl_up(v, N);
        pex = group == 0 ? S(0) : u;
    }
    __syncthreads();

    // ---- 3. wavefront 0: scan of the wavefront totals; 4. look-back ----
    DEER_STAMP(p, slot, 1, tid == 0);
    if (wave == 0) {
        S Mt[N], vt;
        {
            // groups beyond the number of wavefronts hold the identity pair
            const bool has = group < W;
            const int gw = has ? group : W - 1;
#pragma unroll
            for (int c = 0; c < N; ++c) {
                const S u = sM[gw][i * N + c];
                Mt[c] = has ? u : ((c == i) ? S(1) : S(0));
            }
            const S u = sv[gw][i];
            vt = has ? u : S(0);
        }
        scan_groups<S, N>(Mt, vt, group, W);
        // group g now holds the prefix through wavefront g: it is the prefix in front of wavefront g+1
        if (group < W - 1) {
#pragma unroll
            for (int c = 0; c < N; ++c) sEM[group + 1][i * N + c] = Mt[c];
            sEv[group + 1][i] = vt;
        }
        const unsigned tagA = (p.epoch << 2) | TILE_AGGREGATE;
        const unsigned tagI = (p.epoch << 2) | TILE_INCLUSIVE;
        const unsigned long long* aggSeq = p.aggW + (long long)b * p.tiles * AGG_WORDS;
        const unsigned long long* inclSeq = p.inclW + (long long)b * p.tiles * (N * WS);
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
                else if (p.y0) y = reinterpret_cast<const S*>(p.y0)[(long long)b * N + i];
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
                    for (int c = 0; c < N; ++c) got = TaggedWords<S>::get(src, i * N + c, tagA, row[c]) && got;
                    got = TaggedWords<S>::get(src, N * N + i, tagA, u) && got;
                    if (__ballot(!got) != 0ull) {
#pragma unroll
                        for (int c = 0; c < N; ++c) ok = tagged_get_wait<S>(src, i * N + c, tagA, row[c]) && ok;
                        ok = tagged_get_wait<S>(src, N * N + i, tagA, u) && ok;
                    }
                    hv = valid ? u : S(0);
#pragma unroll
                    for (int c = 0; c < N; ++c) Lr[c] = valid ? row[c] : ((c == i) ? S(1) : S(0));
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
            if (lane == 0) atomicOr(p.status, 1u);
        }
        DEER_STAMP(p, slot, 4, lane == 0);
#ifdef DEER_SCAN_TIMING
        if (p.timing && lane == 0) p.timing[slot * 8 + 7] = (unsigned long long)(k < 0 ? 0 : k);
#endif
        if (group == 0) sCarry[i] = y;
        // inclusive carry of this tile: (tile total) applied to the carry
        if (group == W - 1) {
            const S c = sCarry[i];
            TaggedWords<S>::put(p.inclW + slot * (N * WS), i, group_matvec<S, N>(Mt, vt, c), tagI);
        }
        DEER_STAMP(p, slot, 5, lane == 0);
    }
    __syncthreads();

    // ---- 5. starting state of this group, then the second walk over the resident pairs ----
    S y = sCarry[i];
    if (wave > 0) {
        S row[N];
#pragma unroll
        for (int c = 0; c < N; ++c) row[c] = sEM[wave][i * N + c];
        y = group_matvec<S, N>(row, sEv[wave][i], y);
    }
    y = group_matvec<S, N>(Pex, pex, y);

    S emax = S(0);
#pragma unroll
    for (int l = 0; l < L; ++l) {
        const long long e = e0 + l;
        y = group_matvec<S, N>(Ar[l], be[l], y);
        if (e < T) {
            const long long oi = (REV ? (T - 1 - e) : e) * N + i;
            S w = y;
            if (oldb) {
                const S dq = abs_or_inf<S>(p.delta ? y : y - yo[l]);
                emax = dq > emax ? dq : emax;
                if (p.delta) w += yo[l];
            }
            ob[oi] = w;
        }
    }
    if (p.err) {
        emax = wave_max<S>(emax);
        if (lane == 0) err_atomic_max(p.err, emax);
    }
    DEER_STAMP(p, slot, 6, tid == 0);
}

template <typename S, int N, int L, int W>
hipError_t launch_nlw(const ScanParams& p, hipStream_t s) {
    dim3 grid((unsigned)((long long)p.B * p.tiles));
    if (p.reverse)
        hipLaunchKernelGGL((scan_valu_kernel<S, N, L, W, true>), grid, dim3(64 * W), 0, s, p);
    else
        hipLaunchKernelGGL((scan_valu_kernel<S, N, L, W, false>), grid, dim3(64 * W), 0, s, p);
    return hipGetLastError();
}

template <typename S, int N, int L>
hipError_t launch_nl(const ScanParams& p, hipStream_t s) {
    return launch_nlw<S, N, L, 8>(p, s);
}

template <typename S, int N>
hipError_t launch_n(const ScanParams& p, hipStream_t s) {
    switch (p.L) {
        case 1: return launch_nl<S, N, 1>(p, s);
        case 2: return launch_nl<S, N, 2>(p, s);
        case 4: return launch_nl<S, N, 4>(p, s);
        case 8: return launch_nl<S, N, 8>(p, s);
        case 10: if constexpr (sizeof(S) == 4) return launch_nl<S, N, 10>(p, s); else return hipErrorInvalidValue;
        case 12: if constexpr (sizeof(S) == 4) return launch_nl<S, N, 12>(p, s); else return hipErrorInvalidValue;
        case 16: if constexpr (sizeof(S) == 4) return launch_nl<S, N, 16>(p, s); else return hipErrorInvalidValue;
        default: return hipErrorInvalidValue;
    }
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

int scan_valu_tile(int n, int L, int W) { return W * (64 / n) * L; }

hipError_t launch_scan_valu(int dtype, int n, const ScanParams& p, hipStream_t s) {
    if (p.W != 8) return hipErrorInvalidValue;
    return dtype == 0 ? launch_s<float>(n, p, s) : launch_s<double>(n, p, s);
}

}  // namespace deer
