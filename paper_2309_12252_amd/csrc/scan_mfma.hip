// Inverse linear operator for n = 16 and n = 32: single-pass blocked associative scan over affine
// pairs (A | b) with the operator of Sec. 3.3 eq. 10, the matrix-matrix part on the matrix cores.
//
// Every n x n matrix is handled as (n/16)^2 blocks of 16 x 16 and multiplied with the 16x16x4 MFMA
// instruction:
//   A operand  : lane (g = lane/16, r = lane%16) supplies A[r][g]           (16 x 4 slice)
//   B operand  : lane (g, c = lane%16)           supplies B[g][c]           (4 x 16 slice)
//   accumulator: lane (g, c), register v         holds    D[4g + v][c] (fp32) or D[4v + g][c] (fp64)
// A running product P is kept in accumulator layout.  Register v of a block of P, used directly as
// the B operand, is the 4 x 16 slice made of rows {idx(g, v)}; the matching A operand is the 16 x 4
// slice made of columns {idx(g, v)}.  For fp32 (idx = 4g + v) that is one contiguous 4-scalar load
// per lane from a row-major matrix; for fp64 (idx = 4v + g) four strided loads.  So P <- A_t P needs
// no data movement between accumulators and operands.
//
// Structure of one tile (WAVES wavefronts, LW scan positions per wavefront):
//   1. each wavefront loads its LW pairs into registers (A-operand layout) and composes them
//      serially: P <- A_t P on the matrix cores, v <- A_t v + b_t on the vector ALUs;
//   2. wavefront totals meet in LDS and are composed into the tile total by a tree over the
//      wavefronts (log2(WAVES) rounds of one product each);
//   3. decoupled look-back across tiles through HBM as in the small-n kernel (tile index from an
//      atomic ticket, totals and inclusive carries published as self-validating tagged words,
//      window of 64 predecessors, forward fold of totals from the nearest known inclusive carry with
//      the next total requested while the current one is applied, bounded waits);
//   4. each wavefront derives its starting state from the carry and walks its register-resident
//      pairs again (y <- A_t y + b_t), writing y and reducing max|y - y_previous_iterate|.
#include "deer_common.h"

namespace deer {

namespace {

template <typename S> struct Mfma;
template <> struct Mfma<float> {
    using Acc = float __attribute__((ext_vector_type(4)));
    static __device__ __forceinline__ Acc run(float a, float b, Acc c) {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
};
template <> struct Mfma<double> {
    using Acc = double __attribute__((ext_vector_type(4)));
    static __device__ __forceinline__ Acc run(double a, double b, Acc c) {
        return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
    }
};

// Index (row of an accumulator block, or k inside a 16-wide slice) that register v of lane group g
// stands for.  The fp32 instruction keeps rows 4g + v in lane group g, the fp64 one rows 4v + g.
template <typename S> struct Lay;
template <> struct Lay<float> {
    static constexpr bool contiguous = true;
    static __device__ __forceinline__ int idx(int g, int v) { return 4 * g + v; }
};
template <> struct Lay<double> {
    static constexpr bool contiguous = false;
    static __device__ __forceinline__ int idx(int g, int v) { return 4 * v + g; }
};

// x + (x of the lane 32 away) and x + (x of the lane 16 away) with the gfx950 lane-swap instructions: the
// swap of a register with itself leaves the lower (even) half in one result and the upper (odd) half in the
// other, in every lane.  Vector ALU only, no trip through the LDS crossbar.
__device__ __forceinline__ float plus_lane32(float x) {
    const unsigned u = __float_as_uint(x);
    const auto q = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(q[0]) + __uint_as_float(q[1]);
}
__device__ __forceinline__ float plus_lane16(float x) {
    const unsigned u = __float_as_uint(x);
    const auto q = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    return __uint_as_float(q[0]) + __uint_as_float(q[1]);
}
__device__ __forceinline__ double plus_lane32(double x) {
    const unsigned long long u = (unsigned long long)__double_as_longlong(x);
    const unsigned lo = (unsigned)u, hi = (unsigned)(u >> 32);
    const auto a = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
    const auto b = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
    return __longlong_as_double((long long)(((unsigned long long)b[0] << 32) | a[0])) +
           __longlong_as_double((long long)(((unsigned long long)b[1] << 32) | a[1]));
}
__device__ __forceinline__ double plus_lane16(double x) {
    const unsigned long long u = (unsigned long long)__double_as_longlong(x);
    const unsigned lo = (unsigned)u, hi = (unsigned)(u >> 32);
    const auto a = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
    const auto b = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
    return __longlong_as_double((long long)(((unsigned long long)b[0] << 32) | a[0])) +
           __longlong_as_double((long long)(((unsigned long long)b[1] << 32) | a[1]));
}

// Four sums over the 16 lanes of a row at once: lane r ends with the total of q[r & 3].  Lanes first trade the values they
// do not keep (with the neighbour, then with the other pair of the quad), the two rotations then add the four quads, which
// hold the same selection.  11 instructions instead of the 19 of four separate sums and a select.
__device__ __forceinline__ float row_sum16_select4(const float q[4], int r) {
    const bool odd = r & 1, upper = r & 2;
    const float k0 = odd ? q[1] : q[0], s0 = odd ? q[0] : q[1];
    const float k1 = odd ? q[3] : q[2], s1 = odd ? q[2] : q[3];
    const float u0 = k0 + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(s0), 0xB1, 0xf, 0xf, true));   // quad_perm 1,0,3,2
    const float u1 = k1 + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(s1), 0xB1, 0xf, 0xf, true));
    const float k = upper ? u1 : u0, s = upper ? u0 : u1;
    float w = k + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(s), 0x4E, 0xf, 0xf, true));             // quad_perm 2,3,0,1
    w += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(w), 0x124, 0xf, 0xf, true));                     // row_ror 4
    w += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(w), 0x128, 0xf, 0xf, true));                     // row_ror 8
    return w;
}
__device__ __forceinline__ double row_sum16_select4(const double*, int) { return 0.0; }   // fp64 walks the chain instead

// sum over the four lane groups g (lanes r, r+16, r+32, r+48)
template <typename S>
__device__ __forceinline__ S sum_groups(S v) {
    return plus_lane32(plus_lane16(v));
}

// FUSE: the pairs are not loaded but computed from the GRU cell at the previous iterate (p.yold), Sec. 3.1
// eq. 3 and 5: J in A-operand layout straight from the gate values and the weights (kept in LDS in that
// layout), rhs = f - J h.  fp32 only.  FUSE with REV is the dual scan of Sec. 3.1.1 eq. 7 with the transposed
// Jacobians computed the same way at the trajectory p.yold (scan position e carries time T-1-e: its matrix is
// the transpose of the Jacobian at time T-e, which depends on the state at T-1-e and the input at T-e; the
// vector is still loaded from p.bv); no convergence measure is taken.
template <typename S, int N, int LW, int WAVES, bool REV, bool FUSE>
__global__ __launch_bounds__(64 * WAVES, 2) void scan_mfma_kernel(ScanParams p, GruFeed gf) {
    static_assert(!FUSE || sizeof(S) == 4, "the fused cell feeds fp32 scans only");
    constexpr bool DUAL = FUSE && REV;
    constexpr int NB = N / 16;
    // fp32: the composition leaves the running pair of every position in the registers of its factor, so the second
    // walk is L independent products with the carry instead of a chain through cross-lane gathers
    constexpr bool PAR = sizeof(S) == 4;
    // plain forward fp32 scan, n = 16: the first pair of a wavefront is loaded in accumulator layout straight away -- it is
    // the running product after one position -- instead of in operand layout for a product with the identity (measured:
    // +10 % at n = 16, nothing at n = 32, and with the cell inside the scan the extra assembly spills)
    constexpr bool SKIP0 = PAR && !REV && !FUSE && N == 16;
    constexpr int LD = N + 1;   // LDS row stride of a wavefront total
    constexpr int TILE = LW * WAVES;
    using Acc = typename Mfma<S>::Acc;

    __shared__ unsigned s_ticket;
    __shared__ S sM[WAVES][N * LD];   // wavefront totals, row-major, padded rows
    __shared__ S sv[WAVES][N];
    __shared__ S sP[WAVES / 2][N * LD];   // partial totals handed between the rounds of the tree
    __shared__ S sPv[WAVES / 2][N];
    __shared__ S sT[N * LD];          // tile total
    __shared__ S sTv[N];
    __shared__ S sC[WAVES][N];        // carry entering each wavefront
    constexpr int HOPS = (sizeof(S) == 4) ? (N == 64 ? 2 : 8) : 2;   // predecessor totals staged in LDS per round
    __shared__ int s_k;               // hops between this tile and the nearest known inclusive carry
    __shared__ int s_ok;
    // fused cell: rows of [U_gate | W_gate (16 columns, zero padded)] per gate, and the four bias vectors
    constexpr int LDU = N + 16 + 4;
    __shared__ __align__(16) S sU[FUSE ? 3 : 1][FUSE ? N : 1][FUSE ? LDU : 1];
    __shared__ __align__(16) S sB[FUSE ? 4 : 1][FUSE ? N : 1];
    // per wavefront: p_z, s_r, s_t, z and rhs of its LW positions, [scalar][position][row]
    // The staged predecessor totals share their memory: the scalars are last read when the matrices are assembled, the
    // totals are first staged after the barriers of the tree.
    constexpr int NSC = DUAL ? 4 : 5;
    constexpr int SS_ELEMS = FUSE ? WAVES * NSC * LW * N : 1;
    constexpr int HOP_ELEMS = HOPS * (N * LD + N);
    __shared__ __align__(16) S sRaw[SS_ELEMS > HOP_ELEMS ? SS_ELEMS : HOP_ELEMS];
    S (*sHop)[N * LD + N] = reinterpret_cast<S (*)[N * LD + N]>(sRaw);
    S (*sS)[NSC][FUSE ? LW : 1][FUSE ? N : 1] = reinterpret_cast<S (*)[NSC][FUSE ? LW : 1][FUSE ? N : 1]>(sRaw);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    // Segment of the tile (in scan order) of each wavefront.  Wavefronts w and w + 4 of a workgroup share a SIMD, and the
    // rounds of the tree keep the segments 0, 2, 4, 6, then 0 and 4, busy: those go to four different SIMDs, and each SIMD's
    // second wavefront takes the odd segment that evens out the serial carry steps of step 4 (segment s makes s of them).
    const int pw = tid >> 6;
    // (four-wavefront workgroups have a SIMD per wavefront and keep the plain order: measured faster)
    const int wave = (WAVES < 8) ? pw : ((pw < WAVES / 2) ? 2 * pw : (WAVES - 1) - 2 * (pw - WAVES / 2));
    const int g = lane >> 4;
    const int r = lane & 15;

    if (gate_closed<S>(p.gate)) return;
    if (tid == 0) s_ticket = atomicAdd(p.ticket, 1u);
    // the cell's weights go to LDS while the ticket is on its way (the barrier below covers both)
    if constexpr (FUSE) {
        const S* __restrict__ th = reinterpret_cast<const S*>(gf.theta);
        const int d = gf.d;
        const S* __restrict__ U = th + 3 * N * d;
        const S* __restrict__ bias = U + 3 * N * N;
        // sixteen threads per row, four columns each (the last 16 - (N + 16) / 4 of them idle): one 16-byte load and
        // store per gate for the U part, guarded scalars for the d input columns
        const int c4 = tid & 15;
        for (int row = tid >> 4; row < N; row += 4 * WAVES) {
            if (c4 < (N + 16) / 4) {
#pragma unroll
                for (int gate = 0; gate < 3; ++gate) {
                    S val[4];
                    if (4 * c4 < N) {
                        vload<S, 4>(val, U + (gate * N + row) * N + 4 * c4);
                    } else {
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const int col = 4 * c4 + v - N;
                            val[v] = (col < d) ? th[(gate * N + row) * d + col] : S(0);
                        }
                    }
                    vstore<S, 4>(&sU[gate][row][4 * c4], val);
                }
            }
        }
        if (tid < 4 * N) sB[tid / N][tid % N] = bias[tid];
    }
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
    const long long e0 = (long long)t * TILE + (long long)wave * LW;
    const long long slot = (long long)b * p.tiles + t;
    DEER_STAMP(p, slot, 0, tid == 0);

    // ---- 1a. load this wavefront's pairs ----
    // Branch free on purpose (positions past the end read the last valid one and are then replaced by
    // the identity pair): with straight-line code the compiler keeps the loads in order and lets the
    // first products start while later positions are still in flight.
    S a[LW][NB][NB][4];   // a[i][I][K][v] = A_e[16I + r][16K + idx(g, v)]
    S bel[LW][NB];        // bel[i][I]     = b_e[16I + r]
    S yo[LW][NB];         // previous iterate at the same positions (for step 4)
#pragma unroll
    for (int i = 0; i < (FUSE ? 0 : LW); ++i) {
        const long long e = e0 + i;
        const bool past = e >= p.T;
        const long long ec = past ? (long long)p.T - 1 : e;
        const long long vi = (REV ? ((long long)p.T - 1 - ec) : ec) * N;
        if constexpr (!REV) {
            const S* Ae = Ab + ec * (N * N);
#pragma unroll
            for (int I = 0; I < NB; ++I)
#pragma unroll
                for (int K = 0; K < NB; ++K) {
                    if (SKIP0 && i == 0) {
                        // accumulator layout: rows 16I + idx(g, v), column 16K + r
#pragma unroll
                        for (int v = 0; v < 4; ++v) a[i][I][K][v] = Ae[(16 * I + Lay<S>::idx(g, v)) * N + 16 * K + r];
                    } else if constexpr (Lay<S>::contiguous) {
                        vload<S, 4>(a[i][I][K], Ae + (16 * I + r) * N + 16 * K + 4 * g);
                    } else {
#pragma unroll
                        for (int v = 0; v < 4; ++v)
                            a[i][I][K][v] = Ae[(16 * I + r) * N + 16 * K + Lay<S>::idx(g, v)];
                    }
                }
        } else {
            // dual operator: transpose of the matrix stored at index T-e; position 0 has none (zero):
            // any valid matrix is read and dropped
            const long long em = ec == 0 ? 1 : ec;
            const S* Ae = Ab + ((long long)p.T - em) * (N * N);
#pragma unroll
            for (int I = 0; I < NB; ++I)
#pragma unroll
                for (int K = 0; K < NB; ++K)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const S u = (p.T > 1) ? Ae[(16 * K + Lay<S>::idx(g, v)) * N + 16 * I + r] : S(0);
                        a[i][I][K][v] = (ec == 0) ? S(0) : u;
                    }
        }
#pragma unroll
        for (int I = 0; I < NB; ++I) {
            const S bv = bb[vi + 16 * I + r];
            bel[i][I] = past ? S(0) : bv;
#pragma unroll
            for (int K = 0; K < NB; ++K)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    a[i][I][K][v] = past ? ((I == K && r == Lay<S>::idx(g, v)) ? S(1) : S(0)) : a[i][I][K][v];
        }
    }
#pragma unroll
    for (int i = 0; i < LW; ++i) {
        const long long e = (e0 + i < p.T) ? e0 + i : (long long)p.T - 1;
        const S* src = oldb ? oldb : bb;   // branch free: without a previous iterate the value is unused
#pragma unroll
        for (int I = 0; I < NB; ++I) {
            if constexpr (DUAL) {
                // no previous iterate in the dual scan; its vector (the cotangent) is requested here instead
                yo[i][I] = S(0);
                const S bv = bb[((long long)p.T - 1 - e) * N + 16 * I + r];
                bel[i][I] = (e0 + i < p.T) ? bv : S(0);
            } else {
                yo[i][I] = src[(REV ? ((long long)p.T - 1 - e) : e) * N + 16 * I + r];
            }
        }
    }

    DEER_STAMP(p, slot, 8, tid == 0);
    if constexpr (FUSE) {
        // The cell at all LW positions of this wavefront at once.  Gate pre-activations are products on the
        // matrix cores with the positions as columns: S_gate = U_gate H, H[:, c] = state in front of position
        // c, and W_gate X likewise; A operands are read from the weight rows in LDS, B operands are one scalar
        // of h (or x) per lane and k-step.  The results come in accumulator layout -- lane (g, c) holds rows
        // 4g..4g+3 (per 16-row block) of position c -- where the gates, f, the three row factors of J, z and
        // rhs = f - J h are plain elementwise work (J h = p_z (U_z h) + s_r (U_c h) + s_t (U_r h) + z h uses
        // the same products again).  The five per-row scalars then cross to the layout the composition
        // needs (lane (., r) <-> row r, one position after the other) through a private LDS slice.
        const int d = gf.d;
        const S* __restrict__ xb = reinterpret_cast<const S*>(gf.x) + (long long)b * p.T * d;
        const S* __restrict__ y0p = reinterpret_cast<const S*>(p.y0);
        S (*sSw)[LW][N] = sS[wave];
        // n = 32 with eight positions per wavefront: two neighbouring wavefronts share the work by row block instead of
        // by position -- each takes one 16-row block of the 16 positions of the pair, so that all 16 columns of every
        // matrix instruction and all lanes of the elementwise part carry a position -- and exchange the scalars through
        // their LDS slices (one more barrier).
        constexpr bool PAIR = NB == 2 && LW == 8 && WAVES % 2 == 0;
        const long long e0g = PAIR ? (long long)t * TILE + (long long)(wave & ~1) * LW : e0;
#pragma unroll
        for (int cb = 0; cb < (PAIR ? 1 : (LW + 15) / 16); ++cb) {
        const int c = PAIR ? r : ((16 * cb + r < LW) ? 16 * cb + r : LW - 1);   // position handled as a column (lanes beyond LW repeat the last)
        const long long ecol = e0g + c;
        const S* hp;
        long long exl;
        if constexpr (!REV) {
            const long long ecl = ecol < p.T ? ecol : (long long)p.T;     // past the end: the last state (result unused)
            hp = (ecl > 0) ? oldb + (ecl - 1) * N : (y0p ? y0p + (long long)b * N : nullptr);
            exl = ecol < p.T ? ecol : (long long)p.T - 1;
        } else {
            // Jacobian at time T - e; position 0 and positions past the end have none: any valid one is computed and dropped
            long long tj = (long long)p.T - ecol;
            tj = tj > (long long)p.T - 1 ? (long long)p.T - 1 : tj;
            tj = tj < 0 ? 0 : tj;
            exl = tj;
            hp = oldb + (tj > 0 ? tj - 1 : 0) * N;
        }
        S hB[N / 4], xB[4];
#pragma unroll
        for (int kk = 0; kk < N / 4; ++kk) hB[kk] = hp ? hp[4 * kk + g] : S(0);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int k = 4 * kk + g;
            xB[kk] = xb[exl * d + (k < d ? k : d - 1)];   // weights beyond d are zero
        }
        S (*sSd)[LW][N] = PAIR ? sS[(wave & ~1) + (c >> 3)] : sSw;
        const int cl = PAIR ? (c & 7) : c;
#pragma unroll
        for (int Iq = 0; Iq < (PAIR ? 1 : NB); ++Iq) {
            const int I = PAIR ? (wave & 1) : Iq;
            Acc uh[3], wx[3];
#pragma unroll
            for (int gate = 0; gate < 3; ++gate) {
                Acc acc = {S(0), S(0), S(0), S(0)};
#pragma unroll
                for (int kk = 0; kk < N / 4; ++kk) acc = Mfma<S>::run(sU[gate][16 * I + r][4 * kk + g], hB[kk], acc);
                uh[gate] = acc;
                Acc accx = {S(0), S(0), S(0), S(0)};
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
                    if (4 * kk < d) accx = Mfma<S>::run(sU[gate][16 * I + r][N + 4 * kk + g], xB[kk], accx);
                wx[gate] = accx;
            }
            S hrow[4], br[4], bz[4], bc[4], bh[4];
            if (hp) vload<S, 4>(hrow, hp + 16 * I + 4 * g);
            else {
#pragma unroll
                for (int v = 0; v < 4; ++v) hrow[v] = S(0);
            }
            vload<S, 4>(br, &sB[0][16 * I + 4 * g]);
            vload<S, 4>(bz, &sB[1][16 * I + 4 * g]);
            vload<S, 4>(bc, &sB[2][16 * I + 4 * g]);
            vload<S, 4>(bh, &sB[3][16 * I + 4 * g]);
            S o_pz[4], o_sr[4], o_st[4], o_z[4], o_rhs[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const S rg = feed_sigmoid(uh[0][v] + wx[0][v] + br[v]);
                const S z = feed_sigmoid(uh[1][v] + wx[1][v] + bz[v]);
                const S q = uh[2][v] + bh[v];
                const S cc = feed_tanh(wx[2][v] + bc[v] + rg * q);
                const S h = hrow[v];
                const S f = (S(1) - z) * cc + z * h;
                const S pz = (h - cc) * z * (S(1) - z);
                const S sc = (S(1) - z) * (S(1) - cc * cc);
                const S sr = sc * rg;
                const S st = sc * q * rg * (S(1) - rg);
                o_pz[v] = pz; o_sr[v] = sr; o_st[v] = st; o_z[v] = z;
                o_rhs[v] = f - (pz * uh[1][v] + (sr * uh[2][v] + (st * uh[0][v] + z * h)));
            }
            (void)o_rhs;
            if (PAIR || 16 * cb + r < LW) {
                vstore<S, 4>(&sSd[0][cl][16 * I + 4 * g], o_pz);
                vstore<S, 4>(&sSd[1][cl][16 * I + 4 * g], o_sr);
                vstore<S, 4>(&sSd[2][cl][16 * I + 4 * g], o_st);
                vstore<S, 4>(&sSd[3][cl][16 * I + 4 * g], o_z);
                if constexpr (!DUAL) vstore<S, 4>(&sSd[4][cl][16 * I + 4 * g], o_rhs);
            }
        }
        }   // column batches
        if constexpr (PAIR) __syncthreads();
        DEER_STAMP(p, slot, 9, tid == 0);
        // dual scan: the transposed Jacobian in A-operand layout, a[i][I][K][v] = J[16K + 4g + v][16I + r]: the
        // row factors come four at a time, the weights are read down a column
        if constexpr (DUAL) {
            // the diagonal as arithmetic (a select on the lane's own indices would become a branch around the read)
            S dsel[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) dsel[v] = (4 * g + v == r) ? S(1) : S(0);
#pragma unroll
            for (int i = 0; i < LW; ++i) {
                const long long e = e0 + i;
                const S live = (e >= p.T || e == 0) ? S(0) : S(1);   // no matrix at position 0 (zero) and past the end
                const S unit = (e >= p.T) ? S(1) : S(0);             // ... where the pair is the identity
#pragma unroll
                for (int K = 0; K < NB; ++K) {
                    S pz[4], sr[4], st[4], zz[4];
                    vload<S, 4>(pz, &sSw[0][i][16 * K + 4 * g]);
                    vload<S, 4>(sr, &sSw[1][i][16 * K + 4 * g]);
                    vload<S, 4>(st, &sSw[2][i][16 * K + 4 * g]);
                    vload<S, 4>(zz, &sSw[3][i][16 * K + 4 * g]);
#pragma unroll
                    for (int I = 0; I < NB; ++I) {
                        const int col = 16 * I + r;
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const int row = 16 * K + 4 * g + v;
                            S jv = pz[v] * sU[1][row][col] + (sr[v] * sU[2][row][col] + st[v] * sU[0][row][col]);
                            if (I == K) jv += dsel[v] * zz[v];
                            jv *= live;
                            if (I == K) jv += dsel[v] * unit;
                            a[i][I][K][v] = jv;
                        }
                    }
                }
            }
        }
        // J of every position in A-operand layout from its row's three factors (weights from LDS in that layout)
        // (a position past the end takes the factors 0, 0, 0, 1 and the vector 0: the identity pair, at five selects a
        // row instead of one per entry; the diagonal term is one multiply-add with the lane's own 0/1 indicator)
        S dsel[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) dsel[v] = (r == Lay<S>::idx(g, v)) ? S(1) : S(0);
#pragma unroll
        for (int i = 0; i < (DUAL ? 0 : LW); ++i) {
            const bool past = e0 + i >= p.T;
#pragma unroll
            for (int I = 0; I < NB; ++I) {
                const int row = 16 * I + r;
                const S pz = past ? S(0) : sSw[0][i][row], sr = past ? S(0) : sSw[1][i][row];
                const S st = past ? S(0) : sSw[2][i][row], zz = past ? S(1) : sSw[3][i][row];
                const S rhs = sSw[4][i][row];
#pragma unroll
                for (int K = 0; K < NB; ++K) {
                    S Ur[4], Uz[4], Uc[4];
                    vload<S, 4>(Ur, &sU[0][row][16 * K + 4 * g]);
                    vload<S, 4>(Uz, &sU[1][row][16 * K + 4 * g]);
                    vload<S, 4>(Uc, &sU[2][row][16 * K + 4 * g]);
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        S jv = pz * Uz[v] + (sr * Uc[v] + st * Ur[v]);
                        if (I == K) jv += dsel[v] * zz;
                        a[i][I][K][v] = jv;
                    }
                }
                bel[i][I] = past ? S(0) : rhs;
            }
        }
    }

    DEER_STAMP(p, slot, 10, tid == 0);
    DEER_STAMPW(p, slot, wave, 0, lane == 0);
    // ---- 1b. serial composition: P <- A_e P (MFMA), vec <- A_e vec + b_e (VALU) ----
    Acc P[NB][NB];
#pragma unroll
    for (int I = 0; I < NB; ++I)
#pragma unroll
        for (int J = 0; J < NB; ++J)
#pragma unroll
            for (int v = 0; v < 4; ++v) P[I][J][v] = (I == J && Lay<S>::idx(g, v) == r) ? S(1) : S(0);
    S vr[NB];        // vec in row layout:    vr[I]    = vec[16I + r]
    S vc[NB][4];     // vec in column layout: vc[K][v] = vec[16K + idx(g, v)]
#pragma unroll
    for (int I = 0; I < NB; ++I) {
        vr[I] = S(0);
#pragma unroll
        for (int v = 0; v < 4; ++v) vc[I][v] = S(0);
    }
    if constexpr (SKIP0) {
        // after one position the running pair is the first pair itself (already in accumulator layout, and in its place
        // for the second walk)
#pragma unroll
        for (int I = 0; I < NB; ++I) {
#pragma unroll
            for (int J = 0; J < NB; ++J)
#pragma unroll
                for (int v = 0; v < 4; ++v) P[I][J][v] = a[0][I][J][v];
            vr[I] = bel[0][I];
        }
#pragma unroll
        for (int K = 0; K < NB; ++K)
#pragma unroll
            for (int v = 0; v < 4; ++v) vc[K][v] = __shfl(vr[K], Lay<S>::idx(g, v));
    }
#pragma unroll
    for (int i = (SKIP0 ? 1 : 0); i < LW; ++i) {
        Acc Pn[NB][NB];
#pragma unroll
        for (int I = 0; I < NB; ++I)
#pragma unroll
            for (int J = 0; J < NB; ++J) {
                Acc acc = {S(0), S(0), S(0), S(0)};
#pragma unroll
                for (int K = 0; K < NB; ++K)
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc = Mfma<S>::run(a[i][I][K][v], P[K][J][v], acc);
                Pn[I][J] = acc;
            }
#pragma unroll
        for (int I = 0; I < NB; ++I) {
            S s = S(0);
#pragma unroll
            for (int K = 0; K < NB; ++K)
#pragma unroll
                for (int v = 0; v < 4; ++v) s += a[i][I][K][v] * vc[K][v];
            vr[I] = sum_groups<S>(s) + bel[i][I];
        }
#pragma unroll
        for (int K = 0; K < NB; ++K)
#pragma unroll
            for (int v = 0; v < 4; ++v) vc[K][v] = __shfl(vr[K], Lay<S>::idx(g, v));
#pragma unroll
        for (int I = 0; I < NB; ++I)
#pragma unroll
            for (int J = 0; J < NB; ++J) P[I][J] = Pn[I][J];
        if constexpr (PAR) {
            // the factor is not needed again: keep the running pair (accumulator layout: rows 4g + v, column r) in its place
#pragma unroll
            for (int I = 0; I < NB; ++I) {
#pragma unroll
                for (int J = 0; J < NB; ++J)
#pragma unroll
                    for (int v = 0; v < 4; ++v) a[i][I][J][v] = Pn[I][J][v];
                bel[i][I] = vr[I];
            }
        }
    }

    DEER_STAMP(p, slot, 11, tid == 0);
    DEER_STAMPW(p, slot, wave, 1, lane == 0);
    // wavefront total -> LDS (row-major)
#pragma unroll
    for (int I = 0; I < NB; ++I) {
#pragma unroll
        for (int J = 0; J < NB; ++J)
#pragma unroll
            for (int v = 0; v < 4; ++v) sM[wave][(16 * I + Lay<S>::idx(g, v)) * LD + 16 * J + r] = P[I][J][v];
        if (g == 0) sv[wave][16 * I + r] = vr[I];
    }
    __syncthreads();

    // ---- 2. tile total by a tree over the wavefronts: in round `stride` wavefront w (a multiple of
    // 2*stride) composes the partial total that starts at w + stride (left factor, read from LDS in
    // A-operand layout) with its own (right factor, still in its accumulators), so no partial total is
    // ever re-loaded into accumulator layout.  log2(WAVES) rounds instead of WAVES - 1 serial products.
    DEER_STAMP(p, slot, 1, tid == 0);
#pragma unroll 1
    for (int stride = 1; stride < WAVES; stride <<= 1) {
        if (stride > 1) {
            // partial totals of the previous round that are a left factor in this round; in front of the last round
            // wavefront 0 also leaves the total of the tile's first half (slot 0 has no other use): the carries of
            // the second half start from it in step 4
            if ((wave % (2 * stride)) == stride || (2 * stride == WAVES && wave == 0)) {
#pragma unroll
                for (int I = 0; I < NB; ++I) {
#pragma unroll
                    for (int J = 0; J < NB; ++J)
#pragma unroll
                        for (int v = 0; v < 4; ++v) sP[wave / 2][(16 * I + Lay<S>::idx(g, v)) * LD + 16 * J + r] = P[I][J][v];
                    if (g == 0) sPv[wave / 2][16 * I + r] = vr[I];
                }
            }
            __syncthreads();
        }
        if ((wave % (2 * stride)) == 0) {
            const int src = wave + stride;
            const S* Ml = (stride == 1) ? sM[src] : sP[src / 2];
            const S* vl = (stride == 1) ? sv[src] : sPv[src / 2];
            S am[NB][NB][4];
#pragma unroll
            for (int I = 0; I < NB; ++I)
#pragma unroll
                for (int K = 0; K < NB; ++K)
#pragma unroll
                    for (int v = 0; v < 4; ++v) am[I][K][v] = Ml[(16 * I + r) * LD + 16 * K + Lay<S>::idx(g, v)];
            Acc Pn[NB][NB];
#pragma unroll
            for (int I = 0; I < NB; ++I)
#pragma unroll
                for (int J = 0; J < NB; ++J) {
                    Acc acc = {S(0), S(0), S(0), S(0)};
#pragma unroll
                    for (int K = 0; K < NB; ++K)
#pragma unroll
                        for (int v = 0; v < 4; ++v) acc = Mfma<S>::run(am[I][K][v], P[K][J][v], acc);
                    Pn[I][J] = acc;
                }
#pragma unroll
            for (int I = 0; I < NB; ++I) {
                S sacc = S(0);
#pragma unroll
                for (int K = 0; K < NB; ++K)
#pragma unroll
                    for (int v = 0; v < 4; ++v) sacc += am[I][K][v] * vc[K][v];
                vr[I] = sum_groups<S>(sacc) + vl[16 * I + r];
            }
#pragma unroll
            for (int K = 0; K < NB; ++K)
#pragma unroll
                for (int v = 0; v < 4; ++v) vc[K][v] = __shfl(vr[K], Lay<S>::idx(g, v));
#pragma unroll
            for (int I = 0; I < NB; ++I)
#pragma unroll
                for (int J = 0; J < NB; ++J) P[I][J] = Pn[I][J];
        }
        DEER_STAMP(p, slot, (stride == 1 ? 12 : (stride == 2 ? 13 : 14)), tid == 0);
    }

    // ---- 3. look-back (wavefront 0 now holds the tile total) ----
    // The tile total goes to LDS (for the inclusive carry); from there the other wavefronts send it to HBM for the
    // successors (tagged words, consecutive lanes to consecutive words) while wavefront 0 already looks back.
    if (wave == 0) {
#pragma unroll
        for (int I = 0; I < NB; ++I) {
#pragma unroll
            for (int J = 0; J < NB; ++J)
#pragma unroll
                for (int v = 0; v < 4; ++v) sT[(16 * I + Lay<S>::idx(g, v)) * LD + 16 * J + r] = P[I][J][v];
            if (g == 0) sTv[16 * I + r] = vr[I];
        }
    }
    __syncthreads();
    if (wave != 0) {
        if (t > 0) {
            constexpr int WS = TaggedWords<S>::per_scalar;
            constexpr int AGG_WORDS = (N * N + N) * WS;
            const unsigned tagA = (p.epoch << 2) | TILE_AGGREGATE;
            unsigned long long* mine = p.aggW + slot * AGG_WORDS;
            for (int e = tid - 64; e < N * N + N; e += 64 * (WAVES - 1)) {
                const S val = (e < N * N) ? sT[(e / N) * LD + (e % N)] : sTv[e - N * N];
                TaggedWords<S>::put(mine, e, val, tagA);
            }
        }
    } else {
        constexpr int WS = TaggedWords<S>::per_scalar;
        constexpr int AGG_WORDS = (N * N + N) * WS;
        const unsigned tagA = (p.epoch << 2) | TILE_AGGREGATE;
        const unsigned tagI = (p.epoch << 2) | TILE_INCLUSIVE;
        const unsigned long long* aggSeq = p.aggW + (long long)b * p.tiles * AGG_WORDS;
        const unsigned long long* inclSeq = p.inclW + (long long)b * p.tiles * (N * WS);
        DEER_STAMP(p, slot, 2, lane == 0);
        // lane j inspects predecessor t-1-j (index -1 is the given initial state): inclusive carry
        // known, total known, or nothing yet, judged by one word of each
        const int idx = t - 1 - lane;
        int k = -1;
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

        DEER_STAMP(p, slot, 3, lane == 0);
        if (lane == 0) { s_k = k; s_ok = 1; }
    }
    __syncthreads();

    // ---- 3b. fold the totals of the k predecessors between the known inclusive carry and this tile.
    // All wavefronts stage the totals into LDS (coalesced tagged words, HOPS tiles per round); wavefront
    // 0 applies them in order, one matrix row per lane, with the running carry in sC[0].
    {
        constexpr int WS = TaggedWords<S>::per_scalar;
        constexpr int AGG_WORDS = (N * N + N) * WS;
        const unsigned tagA = (p.epoch << 2) | TILE_AGGREGATE;
        const unsigned tagI = (p.epoch << 2) | TILE_INCLUSIVE;
        const unsigned long long* aggSeq = p.aggW + (long long)b * p.tiles * AGG_WORDS;
        const unsigned long long* inclSeq = p.inclW + (long long)b * p.tiles * (N * WS);
        const int k = s_k;
        const int far = t - 1 - k;   // tile whose inclusive carry is known (-1: the initial state)
        bool ok = k >= 0;
        if (wave == 0 && lane < N) {
            S y = S(0);
            if (ok) {
                if (far >= 0) ok = tagged_get_wait<S>(inclSeq + (long long)far * (N * WS), lane, tagI, y);
                else if (p.y0) y = reinterpret_cast<const S*>(p.y0)[(long long)b * N + lane];
            }
            sC[0][lane] = y;
        }
        for (int q0 = far + 1; k >= 0 && q0 <= t - 1; q0 += HOPS) {   // uniform: k, far and t are the same for every thread
            const int nh = (t - q0 < HOPS) ? (t - q0) : HOPS;
            // every lane requests all its words of all its tiles before looking at any of them
            constexpr int TOT = N * N + N;
            constexpr int PER = (TOT + 63) / 64;              // words per lane and tile
            constexpr int HPW = (HOPS + WAVES - 1) / WAVES;   // tiles per wavefront and round
            S vals[HPW][PER];
            bool got = true;
#pragma unroll
            for (int hh = 0; hh < HPW; ++hh) {
                const int h = wave + hh * WAVES;
                if (h < nh) {
                    const unsigned long long* src = aggSeq + (long long)(q0 + h) * AGG_WORDS;
#pragma unroll
                    for (int j = 0; j < PER; ++j) {
                        const int e = lane + 64 * j;
                        if (e < TOT) got = TaggedWords<S>::get(src, e, tagA, vals[hh][j]) && got;
                    }
                }
            }
            if (__ballot(!got) != 0ull) {
                // rare: part of a total was still in flight; wait for it word by word
#pragma unroll
                for (int hh = 0; hh < HPW; ++hh) {
                    const int h = wave + hh * WAVES;
                    if (h < nh) {
                        const unsigned long long* src = aggSeq + (long long)(q0 + h) * AGG_WORDS;
#pragma unroll
                        for (int j = 0; j < PER; ++j) {
                            const int e = lane + 64 * j;
                            if (e < TOT) ok = tagged_get_wait<S>(src, e, tagA, vals[hh][j]) && ok;
                        }
                    }
                }
            }
#pragma unroll
            for (int hh = 0; hh < HPW; ++hh) {
                const int h = wave + hh * WAVES;
                if (h < nh) {
#pragma unroll
                    for (int j = 0; j < PER; ++j) {
                        const int e = lane + 64 * j;
                        if (e < TOT) {
                            const int dst = (e < N * N) ? ((e / N) * LD + (e % N)) : (N * LD + (e - N * N));
                            sHop[h][dst] = vals[hh][j];
                        }
                    }
                }
            }
            __syncthreads();
            if (wave == 0) {
                for (int h = 0; h < nh; ++h) {
                    S acc = S(0);
                    if (lane < N) {
                        acc = sHop[h][N * LD + lane];
#pragma unroll 8
                        for (int q = 0; q < N; ++q) acc += sHop[h][lane * LD + q] * sC[0][q];
                    }
                    if (lane < N) sC[0][lane] = acc;
                }
            }
            __syncthreads();
        }
        if (!ok) s_ok = 0;
        if (wave == 0) {
            DEER_STAMP(p, slot, 4, lane == 0);
#ifdef DEER_SCAN_TIMING
            if (p.timing && lane == 0) p.timing[slot * 16 + 7] = (unsigned long long)(k < 0 ? 0 : k);
#endif
            // inclusive carry of this tile = (tile total) applied to the carry
            if (lane < N) {
                S sacc = sTv[lane];
                for (int q = 0; q < N; ++q) sacc += sT[lane * LD + q] * sC[0][q];
                TaggedWords<S>::put(p.inclW + slot * (N * WS), lane, sacc, tagI);
            }
            DEER_STAMP(p, slot, 5, lane == 0);
        }
    }
    __syncthreads();
    if (tid == 0 && s_ok == 0) atomicOr(p.status, 1u);

    // ---- 4. carry entering this wavefront, then the second walk over the resident pairs ----
    const int w0 = (WAVES >= 4 && wave >= WAVES / 2) ? WAVES / 2 : 0;
    if (w0 > 0) {
        // second half of the tile: (total of the first half) applied to the tile's carry
        S s = S(0);
        if (lane < N) {
            s = sPv[0][lane];
            for (int q = 0; q < N; ++q) s += sP[0][lane * LD + q] * sC[0][q];
        }
        if (lane < N) sC[wave][lane] = s;
    }
    for (int w = w0; w < wave; ++w) {
        // sC[wave] <- M_w * (carry entering w) + v_w, built up in place from sC[0]
        S s = S(0);
        if (lane < N) {
            const S* cin = (w == 0) ? sC[0] : sC[wave];
            s = sv[w][lane];
            for (int q = 0; q < N; ++q) s += sM[w][lane * LD + q] * cin[q];
        }
        if (lane < N) sC[wave][lane] = s;
    }
    S emax = S(0);
    if constexpr (PAR) {
        // y_e = (running matrix of e) carry + (running vector of e): lane (g, r) multiplies its column r of rows 4g + v
        // with entry r of the carry; the sums over the row's 16 lanes leave y[16 I + 4g + (r & 3)] in lane r of row g, and
        // the four lanes r = 4g .. 4g+3 of each row own the 16 entries in memory order
        S cr[NB];
#pragma unroll
        for (int J = 0; J < NB; ++J) cr[J] = sC[wave][16 * J + r];
        const bool owner = (r >> 2) == g;
#pragma unroll
        for (int i = 0; i < LW; ++i) {
            const long long e = e0 + i;
            const long long oi = (REV ? ((long long)p.T - 1 - e) : e) * N;
#pragma unroll
            for (int I = 0; I < NB; ++I) {
                S t[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    S q = S(0);
#pragma unroll
                    for (int J = 0; J < NB; ++J) q += a[i][I][J][v] * cr[J];
                    t[v] = q;
                }
                const S y = row_sum16_select4(t, r) + bel[i][I];
                if (e < p.T && owner) {
                    S wv = y;
                    if (!DUAL && oldb) {
                        const S dq = abs_or_inf<S>(p.delta ? y : y - yo[i][I]);
                        emax = dq > emax ? dq : emax;
                        if (p.delta) wv += yo[i][I];
                    }
                    ob[oi + 16 * I + r] = wv;
                }
            }
        }
    }
    S yc[NB][4], yr[NB];
#pragma unroll
    for (int K = 0; K < NB; ++K)
#pragma unroll
        for (int v = 0; v < 4; ++v) yc[K][v] = sC[wave][16 * K + Lay<S>::idx(g, v)];

#pragma unroll
    for (int i = 0; i < (PAR ? 0 : LW); ++i) {
        const long long e = e0 + i;
#pragma unroll
        for (int I = 0; I < NB; ++I) {
            S s = S(0);
#pragma unroll
            for (int K = 0; K < NB; ++K)
#pragma unroll
                for (int v = 0; v < 4; ++v) s += a[i][I][K][v] * yc[K][v];
            yr[I] = sum_groups<S>(s) + bel[i][I];
        }
        if (e < p.T && g == 0) {
            const long long oi = (REV ? ((long long)p.T - 1 - e) : e) * N;
#pragma unroll
            for (int I = 0; I < NB; ++I) {
                S wv = yr[I];
                if (!DUAL && oldb) {
                    const S dq = abs_or_inf<S>(p.delta ? yr[I] : yr[I] - yo[i][I]);
                    emax = dq > emax ? dq : emax;
                    if (p.delta) wv += yo[i][I];
                }
                ob[oi + 16 * I + r] = wv;
            }
        }
#pragma unroll
        for (int K = 0; K < NB; ++K)
#pragma unroll
            for (int v = 0; v < 4; ++v) yc[K][v] = __shfl(yr[K], Lay<S>::idx(g, v));
    }
    if (p.err) {
        emax = wave_max<S>(emax);
        if (lane == 0) err_atomic_max(p.err, emax);
    }
    DEER_STAMP(p, slot, 6, tid == 0);
}

template <typename S, int N> struct MfmaShape;
template <> struct MfmaShape<float, 16> { static constexpr int LW = 16, WAVES = 4; };
template <> struct MfmaShape<float, 32> { static constexpr int LW = 8, WAVES = 8; };
// n = 64 (fp32 only): 64 registers per matrix, two positions per wavefront; four wavefronts, because the wavefront totals
// (16.6 KB each) fill the LDS
template <> struct MfmaShape<float, 64> { static constexpr int LW = 2, WAVES = 4; };
template <> struct MfmaShape<double, 16> { static constexpr int LW = 8, WAVES = 8; };
template <> struct MfmaShape<double, 32> { static constexpr int LW = 4, WAVES = 8; };

template <typename S, int N>
hipError_t launch_n(const ScanParams& p, hipStream_t s) {
    constexpr int LW = MfmaShape<S, N>::LW, WAVES = MfmaShape<S, N>::WAVES;
    dim3 grid((unsigned)((long long)p.B * p.tiles));
    if (p.reverse)
        hipLaunchKernelGGL((scan_mfma_kernel<S, N, LW, WAVES, true, false>), grid, dim3(64 * WAVES), 0, s, p, GruFeed{});
    else
        hipLaunchKernelGGL((scan_mfma_kernel<S, N, LW, WAVES, false, false>), grid, dim3(64 * WAVES), 0, s, p, GruFeed{});
    return hipGetLastError();
}

// Tile shapes of the fused step.  n = 16: longer serial runs than the plain scan (the per-tile latencies --
// ticket, weight fill, first loads -- weigh more than the 4 MFMAs per position), as long as the registers hold.
template <int N> struct MfmaFusedShape;
template <> struct MfmaFusedShape<16> { static constexpr int LW = 24, WAVES = 4; };
template <> struct MfmaFusedShape<32> { static constexpr int LW = 8, WAVES = 8; };
template <int N>
hipError_t launch_fused_n(const ScanParams& p, const GruFeed& gf, hipStream_t s) {
    constexpr int LW = MfmaFusedShape<N>::LW, WAVES = MfmaFusedShape<N>::WAVES;
    dim3 grid((unsigned)((long long)p.B * p.tiles));
    if (p.reverse)   // the dual scan runs on the tile shape of the plain scan (n = 16: three wavefronts per SIMD; 24 positions
                     // per wavefront measured 10 % slower)
        hipLaunchKernelGGL((scan_mfma_kernel<float, N, MfmaShape<float, N>::LW, MfmaShape<float, N>::WAVES, true, true>), grid,
                           dim3(64 * MfmaShape<float, N>::WAVES), 0, s, p, gf);
    else
        hipLaunchKernelGGL((scan_mfma_kernel<float, N, LW, WAVES, false, true>), grid, dim3(64 * WAVES), 0, s, p, gf);
    return hipGetLastError();
}

}  // namespace

int scan_mfma_tile(int dtype, int n) {
    if (dtype == 0 && n == 64) return MfmaShape<float, 64>::LW * MfmaShape<float, 64>::WAVES;
    if (dtype == 0) return n == 16 ? MfmaShape<float, 16>::LW * MfmaShape<float, 16>::WAVES
                                   : MfmaShape<float, 32>::LW * MfmaShape<float, 32>::WAVES;
    return n == 16 ? MfmaShape<double, 16>::LW * MfmaShape<double, 16>::WAVES
                   : MfmaShape<double, 32>::LW * MfmaShape<double, 32>::WAVES;
}

int scan_mfma_fused_tile(int n) {
    return n == 16 ? MfmaFusedShape<16>::LW * MfmaFusedShape<16>::WAVES : MfmaFusedShape<32>::LW * MfmaFusedShape<32>::WAVES;
}

bool scan_mfma_fused_supported(int dtype, int n, int d) { return dtype == 0 && (n == 16 || n == 32) && d >= 1 && d <= 16; }

hipError_t launch_scan_mfma_fused(int n, const ScanParams& p, const void* theta, const void* x, int d, hipStream_t s) {
    if (!scan_mfma_fused_supported(0, n, d) || p.delta || !p.yold) return hipErrorInvalidValue;
    const GruFeed gf{theta, x, d};
    return n == 16 ? launch_fused_n<16>(p, gf, s) : launch_fused_n<32>(p, gf, s);
}

hipError_t launch_scan_mfma(int dtype, int n, const ScanParams& p, hipStream_t s) {
    if (n == 64) return dtype == 0 ? launch_n<float, 64>(p, s) : hipErrorInvalidValue;
    if (n != 16 && n != 32) return hipErrorInvalidValue;
    if (dtype == 0) return n == 16 ? launch_n<float, 16>(p, s) : launch_n<float, 32>(p, s);
    return n == 16 ? launch_n<double, 16>(p, s) : launch_n<double, 32>(p, s);
}

}  // namespace deer
