/*
 * deer.h -- C ABI of the DEER hot path for one AMD MI355X (gfx950).
 *
 * DEER (arxiv 2309.12252) evaluates a non-linear recurrence y_i = f(y_{i-1}, x_i)
 * (Sec. 3.4) or an ODE dy/dt = f(y) on a time grid (Sec. 3.3) by the fixed-point
 * iteration  y <- L_G^{-1}[ f(y_shifted) + G y_shifted ],  G = -df/dy  (Sec. 3.1
 * eq. 3 and 5), where L_G^{-1} solves a linear recurrence with an associative scan
 * over affine pairs (Sec. 3.3 eq. 9-10, Sec. 3.4 eq. 11).  Gradients take one
 * application of the transposed, reversed operator followed by the vector-Jacobian
 * product of f (Sec. 3.1.1 eq. 7).
 *
 * Conventions for every entry point
 *   - Pointers named d_* are DEVICE pointers owned by the caller; all other
 *     pointers are HOST pointers owned by the caller.  The library allocates no
 *     device memory: the caller hands in a workspace of deer_workspace_bytes().
 *     (deer_create() allocates a few hundred bytes of pinned HOST memory and the
 *     HIP events of the context; deer_destroy() frees them.)
 *   - Arrays are dense, row-major, in the dtype of the configuration (fp32 or
 *     fp64).  d_* arrays must be 16-byte aligned.
 *   - Work is enqueued on the HIP stream given to deer_create().  deer_eval()
 *     synchronises that stream (it reads the convergence error back) and returns
 *     with its outputs complete; deer_grad() and deer_linrec_solve() synchronise
 *     before returning as well.
 *   - Every call returns a deer_status; nothing throws or aborts across the ABI.
 *     After a non-OK status deer_last_error() describes what went wrong.
 *   - Calls on one context must not overlap in time.
 *
 * The model
 *   GRU cell (the paper names the cell but prints no equations; this is the
 *   reading used, gates r, z and candidate c, reset applied after the hidden
 *   projection):
 *       r = sigmoid(W_r x + b_r + U_r h)     z = sigmoid(W_z x + b_z + U_z h)
 *       q = U_c h + b_hc                     c = tanh(W_c x + b_c + r * q)
 *       f(h, x) = (1 - z) * c + z * h
 *     theta (flat): W[3n,d] (rows r|z|c), U[3n,n] (rows r|z|c), b[3n] (r|z|c), b_hc[n].
 *   LSTM cell (Sec. 3.4 names it as an instance of the recurrence; cell = DEER_CELL_LSTM, n = number of units u,
 *   1..16, d = 1..8).  The state is y = (h | c) with 2u entries, so y0 is [B,2u] and y, the guess and dL/dy are
 *   [B,T,2u]; gates in the order input, forget, candidate, output:
 *       i = sigmoid(W_i x + U_i h + b_i)   f = sigmoid(W_f x + U_f h + b_f)
 *       g = tanh(W_g x + U_g h + b_g)      o = sigmoid(W_o x + U_o h + b_o)
 *       c' = f * c + i * g                 h' = o * tanh(c')
 *     theta (flat): W[4u,d], U[4u,u], b[4u].  An iteration is a Jacobian kernel followed by the scan over the 2u x 2u
 *     Jacobians (embedded in the next state size with a scan kernel).
 *   LEM cell (the cell of the paper's last experiment, which trains it with DEER; the paper prints no equations, the
 *   ones of the publication it cites are used; cell = DEER_CELL_LEM, n = number of units u, 1..16, d = 1..8, t1 = the
 *   cell's step dt > 0).  The state is (y | z) with 2u entries, laid out like the LSTM's; two learned time scales:
 *       s1 = dt * sigmoid(W_1 x + U_1 y + b_1)   s2 = dt * sigmoid(W_2 x + U_2 y + b_2)
 *       z' = (1 - s1) * z + s1 * tanh(W_z x + U_z y + b_z)
 *       y' = (1 - s2) * y + s2 * tanh(W_y x + U_y z' + b_y)
 *     theta (flat): W[4u,d], U[4u,u], b[4u], row blocks in the order 1 | 2 | z | y.  Kernels as for the LSTM.
 *   Multi-head GRU with strides (Sec. 4.4, App. B.4; heads > 1 or stride_levels > 1): the state is H heads of n
 *   channels, every head a GRU cell of its own on its own d input channels, and head h looks back
 *   s_h = 2^(h mod K) steps instead of one (the K stride levels are dealt out to the heads in turn):
 *       y[b,i,h,:] = f_h(y[b,i-s_h,h,:], x[b,i,h,:]),  with y0[b,h,:] in place of y[b,i-s_h,h,:] while i < s_h.
 *     Arrays: x [B,T,H,d], y0 [B,H,n], y / guess / dL/dy [B,T,H,n], dL/dx [B,T,H,d], dL/dy0 [B,H,n];
 *     theta and dL/dtheta [H][theta of one cell]; deer_theta_count() returns the total.  n = 2, 4 or 8, d <= 8,
 *     H <= 64, K <= 8.  A head that takes all input channels is obtained by projecting the inputs beforehand
 *     (a plain matrix product outside this library).
 *   MLP vector field (autonomous), L hidden layers of width w with activation s = tanh or softplus
 *   (s(a) = log(1 + exp(a)); App. B.2 uses six linear layers with softplus on all but the last):
 *       f(y) = W_out s(W_L s(... s(W_1 y + b_1) ...) + b_L) + b_out
 *     theta (flat): W_1[w,n], b_1[w], then W_l[w,w], b_l[w] for l = 2..L, then W_out[n,w], b_out[n].
 *   Two tanh layers of width 16, 32 or 64 (a multiple of n) have kernels of their own (fp32 with n = 8: on
 *   the matrix cores); every other depth, width and the softplus activation run general kernels.
 */
#ifndef DEER_H
#define DEER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DEER_OK = 0,
    DEER_ERR_INVALID_ARG = 1,  /* NULL where a pointer is required, non-positive size, bad enum          */
    DEER_ERR_UNSUPPORTED = 2,  /* a shape or mode this build has no kernel for                           */
    DEER_ERR_WORKSPACE = 3,    /* workspace NULL, misaligned or smaller than deer_workspace_bytes()      */
    DEER_ERR_HIP = 4,          /* a HIP runtime call failed, or a kernel reported an internal time-out   */
    DEER_ERR_NONFINITE = 5     /* the iteration produced a NaN/Inf; outputs hold the last iterate        */
} deer_status;

typedef enum { DEER_CELL_GRU = 0, DEER_CELL_MLP_ODE = 1, DEER_CELL_LSTM = 2, DEER_CELL_LEM = 3 } deer_cell;
typedef enum { DEER_F32 = 0, DEER_F64 = 1 } deer_dtype;
typedef enum { DEER_ACT_TANH = 0, DEER_ACT_SOFTPLUS = 1 } deer_activation;

typedef struct {
    int32_t cell;               /* deer_cell                                                             */
    int32_t dtype;              /* deer_dtype                                                            */
    int32_t B;                  /* batch: independent sequences                                          */
    int32_t T;                  /* GRU: number of steps; MLP_ODE: number of grid points (>= 2)           */
    int32_t n;                  /* state size.  GRU: 1..64, above 32 in fp32 only (1, 2, 4, 8, 16, 32, 64 have  */
                                /* kernels of their own; any other size runs embedded in the next of     */
                                /* those, with identical results);                                       */
                                /* MLP_ODE: 2, 4 or 8; multi-head GRU: 2, 4 or 8 per head; LSTM and LEM: */
                                /* the number of units u, 1..16 (the state has 2u entries)               */
    int32_t d;                  /* GRU input size (1..32); LSTM and LEM: 1..8; ignored for MLP_ODE       */
    int32_t mlp_width;          /* MLP_ODE hidden width w: a multiple of 4, 4..64; ignored for GRU       */
    int32_t mlp_hidden_layers;  /* MLP_ODE: hidden layers L, 1..5 (L + 1 linear layers)                  */
    double t0, t1;              /* MLP_ODE: uniform grid t_j = t0 + j (t1 - t0)/(T - 1); LEM: t1 = step dt */
    int32_t mlp_activation;     /* MLP_ODE: deer_activation of the hidden layers (0 = tanh)              */
    int32_t heads;              /* GRU: number of heads H (0 or 1: the plain cell); see "multi-head GRU"  */
    int32_t stride_levels;      /* GRU: stride levels K (0 or 1: every head has stride 1)                */
    int32_t reserved;           /* must be 0                                                             */
} deer_config;

typedef struct deer_ctx deer_ctx; /* opaque, host memory owned by the library */

/* Accumulated per-kernel device time, filled while profiling is on (see deer_set_profiling). */
typedef struct {
    double funceval_ms;   int64_t funceval_launches;   /* f, Jacobian and right-hand side            */
    double discretise_ms; int64_t discretise_launches; /* ODE only: exp(-G dt), phi1; in deer_grad also   */
                                                       /* the residual and the dual discretisation       */
    double scan_ms;       int64_t scan_launches;       /* inverse linear operator (+ fused max|dy|)  */
    double vjp_ms;        int64_t vjp_launches;        /* VJP of f + parameter-gradient reduction    */
    double fused_ms;      int64_t fused_launches;      /* GRU: cell + scan + max|dy| in one launch;   */
                                                       /* in deer_grad: cell inside the reverse scan  */
    double newton_ms;     int64_t newton_launches;     /* GRU, small problems: a whole solve in one   */
    int64_t newton_iterations;                         /* Newton iterations inside those launches     */
} deer_profile;

/* Number of parameters in the flat theta of this configuration (layouts above); 0 if invalid. */
size_t deer_theta_count(const deer_config* cfg);

/* Bytes of device workspace deer_create() needs for cfg: a second trajectory buffer, the words the scan's
 * tiles publish for each other, counters, partial sums of dL/dtheta -- and, only where a kernel pair exchanges
 * them through memory (MLP_ODE; GRU in fp64 with n >= 16, with d beyond what the in-scan cell takes, or with the
 * DEER_FUSED / DEER_GRAD_FUSED knobs at 0), the Jacobian stream [B,T,n,n] and the right-hand side, the O(n^2 T)
 * memory of Sec. 3.5.  Where the cell is evaluated inside the scans the workspace is O(n T).
 * The environment variables listed under "Environment" below are read here and in deer_create(); both calls must
 * see the same values. */
deer_status deer_workspace_bytes(const deer_config* cfg, size_t* bytes);

/* Create a context.  d_workspace (device, 256-byte aligned, >= deer_workspace_bytes) stays owned by
 * the caller and must outlive the context; the library may overwrite all of it in any call.
 * hip_stream is a hipStream_t (NULL = the default stream).  On failure *out is NULL. */
deer_status deer_create(const deer_config* cfg, void* d_workspace, size_t workspace_bytes,
                        void* hip_stream, deer_ctx** out);

/* Forward evaluation by DEER (Sec. 3.1 eq. 3 with eq. 5; iteration control as in App. B.1).
 *   d_theta   in  parameters, deer_theta_count() entries
 *   d_x       in  GRU: inputs [B,T,d]; MLP_ODE: ignored (may be NULL)
 *   d_y0      in  initial state [B,n]
 *   d_y_guess in  initial guess [B,T,n], or NULL for all zeros (the paper's benchmarks start from
 *                 zeros; a previous solution can be passed as a warm start, Sec. 3.1)
 *   tol       in  stop when err = max|y_next - y| <= tol (paper: 1e-4 fp32, 1e-7 fp64)
 *   max_iter  in  at most this many iterations (>= 0)
 *   d_y       out GRU: y[b,i-1,:] = y_i for i = 1..T.  MLP_ODE: y[b,j,:] = y(t_j), y[b,0,:] = y0;
 *                 the first grid point is pinned to y0 in every iterate, so err runs over j >= 1
 *   iters     out number of iterations (linear solves) performed, including the one whose err met tol
 *   final_err out err of the last iteration (1e10 if max_iter == 0)
 *   converged out 1 if final_err <= tol else 0.  Not converging is not an error: DEER_OK is returned
 *                 with iters == max_iter (Newton's method may diverge far from the solution, Sec. 3.5).
 * The convergence test is global over batch, time and state.  DEER_ERR_NONFINITE if err is NaN/Inf.
 * d_y doubles as one of the two iterate buffers: it is overwritten during the call; d_y_guess may be
 * the same buffer as d_y.  How the iterations are put on the device does not change the result and is
 * chosen from the shapes: for the GRU with n <= 8 the cell is evaluated inside the scan kernel (the
 * Jacobians never reach memory), and when all tiles of the problem fit on the device at once the
 * whole solve is one kernel launch; for n = 16, 32 in fp32 the cell is evaluated inside the matrix-core
 * scan; otherwise an iteration is a Jacobian kernel followed by a scan kernel (see "Environment").
 * The Jacobians of the last iteration are not kept for deer_grad(): Sec. 3.1.1 offers that as a way to trade memory
 * for speed, this library always recomputes them at the trajectory it is given (exact for any trajectory, and the
 * O(n^2 T) buffer is not needed), so there is no save-the-Jacobian option in deer_config. */
deer_status deer_eval(deer_ctx* ctx, const void* d_theta, const void* d_x, const void* d_y0,
                      const void* d_y_guess, double tol, int32_t max_iter, void* d_y,
                      int32_t* iters, double* final_err, int32_t* converged);

/* Backward derivative (Sec. 3.1.1 eq. 7): the cotangent g = dL/dy is pushed through the transposed,
 * time-reversed linear operator (one reverse scan), then through the vector-Jacobian product of f.
 * The Jacobians are recomputed at the trajectory d_y that is passed in, so the trajectory may
 * come from deer_eval() or from a sequential evaluation (Sec. 3.1.1, last paragraph).
 *   GRU:     lam_T = g_T, lam_i = g_i + J_{i+1}^T lam_{i+1};  dL/dtheta = sum_i (df/dtheta)_i^T lam_i, same for x.
 *   MLP_ODE: on the discretised operator of Sec. 3.3 eq. 8-9 with G frozen at the trajectory:
 *            lam_{T-1} = g_{T-1}, lam_j = g_j + Gbar_j^T lam_{j+1};  dL/dy0 = lam_0;
 *            dL/dtheta = sum_j (df/dtheta)(y_j)^T w_j,  w_j = (P_j^T lam_{j+1} + P_{j-1}^T lam_j) / 2,
 *            P_j = dt phi1(-Gc_j dt) (terms outside the grid dropped).  This is the derivative eq. 7 defines;
 *            it differs from the derivative of the discrete solution by O(dt^2).  d_x, d_y0 and d_dLdx are
 *            ignored (the field is autonomous and y[:,0,:] is the initial state).
 *   d_y        in  trajectory [B,T,n]          d_dLdy   in  g = dL/dy [B,T,n]
 *   d_dLdx     out [B,T,d], or NULL to skip    d_dLdtheta out [theta_count] (overwritten, not accumulated)
 *   d_dLdy0    out [B,n], or NULL to skip
 * The parameter gradient is summed in a fixed order: two calls with the same inputs return the same bits.
 * For the GRU the transposed Jacobians are computed inside the reverse scan wherever deer_eval() evaluates the
 * cell inside the forward scan (n <= 8 with d <= 8; fp32 n = 16, 32 with d <= 16), and in fp32 with n = 16, 32
 * the vector-Jacobian product runs on the matrix cores (so does the MLP field's for fp32, n = 8 and width 16,
 * 32 or 64); see "Environment" for the knobs that select the separate kernels instead. */
deer_status deer_grad(deer_ctx* ctx, const void* d_theta, const void* d_x, const void* d_y0,
                      const void* d_y, const void* d_dLdy, void* d_dLdx, void* d_dLdtheta,
                      void* d_dLdy0);

/* The inverse linear operator alone (Sec. 3.3 eq. 9-10, Sec. 3.4 eq. 11):
 * y_i = A_i y_{i-1} + b_i for i = 1..T from y_0, for B independent sequences, by the blocked
 * associative scan.  Shapes come from the context (B, T, n, dtype).
 * (plain GRU-shaped contexts with n = 1, 2, 4, 8, 16 or 32 only).
 *   d_A [B,T,n,n]   d_b [B,T,n]   d_y0 [B,n] (NULL = zeros)   d_y out [B,T,n]
 *   reverse != 0 applies the dual (transposed, time-reversed) operator of Sec. 3.1.1 eq. 7 instead:
 *   y_T = b_T, y_i = b_i + A_{i+1}^T y_{i+1}; d_y0 is ignored.  A is read as stored and transposed
 *   on the fly. */
deer_status deer_linrec_solve(deer_ctx* ctx, const void* d_A, const void* d_b, const void* d_y0,
                              void* d_y, int32_t reverse);

/* deer_linrec_solve() for callers that cannot allocate device memory or hand in a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The same scan kernels run, but the words their
 * tiles publish for each other, the tile dispenser and the status word live in a static device array inside the
 * library (64 MiB; every GPU the library runs on holds its own copy until the process ends) instead of a workspace,
 * and no context is needed.  The call allocates nothing (no hipMalloc/hipFree, no pinned host memory, no events),
 * enqueues three kernels on hip_stream (a fill that clears the part of the array it uses, the scan, a one-word
 * copy) and returns without synchronising: outputs are complete when the stream reaches that point.
 *   dtype, B, T, n   as in deer_config (n = 1, 2, 4, 8, 16 or 32)
 *   d_A [B,T,n,n]  d_b [B,T,n]  d_y0 [B,n] or NULL (zeros)  d_y out [B,T,n]  reverse: as in deer_linrec_solve()
 *   hip_stream     hipStream_t (NULL = the default stream)
 *   d_status       out, DEVICE int32, or NULL: 0, or non-zero if a tile waited too long for its predecessors
 *                  (then d_y is not valid); the host-side return value cannot report that without a synchronisation
 * Limit: the published words of all tiles must fit the array; a shape beyond it is rejected with
 * DEER_ERR_WORKSPACE before anything is enqueued (n = 32: about 480,000 positions in all; n = 8: several 10^7).
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two threads) race.
 * Returns DEER_OK once everything is enqueued; errors are reported through deer_last_error(NULL). */
deer_status deer_linrec_solve_static(int32_t dtype, int32_t B, int32_t T, int32_t n, const void* d_A, const void* d_b,
                                     const void* d_y0, void* d_y, int32_t reverse, void* hip_stream,
                                     int32_t* d_status);

/* Switch per-kernel timing with HIP events on the context's stream on or off (off by default;
 * turning it on resets the accumulated numbers), and read the numbers accumulated so far. */
deer_status deer_set_profiling(deer_ctx* ctx, int32_t on);
deer_status deer_get_profile(deer_ctx* ctx, deer_profile* out);

/* Text of the last error on this context (never NULL; valid until the next call on ctx).
 * With ctx == NULL: the last error of a failed deer_create()/deer_workspace_bytes() on this thread. */
const char* deer_last_error(const deer_ctx* ctx);

/* Free the context (host memory and HIP events only; the workspace stays with the caller). */
void deer_destroy(deer_ctx* ctx);

/* Environment.  Every variable the library reads; all are meant for tests and measurements, none changes a
 * result beyond rounding.  Read by deer_workspace_bytes() and deer_create() (the plan and the workspace size
 * depend on them), except DEER_VJP_MFMA and DEER_MLP_MFMA, which deer_grad() / deer_eval() read at each call.
 *   DEER_FUSED=0        GRU: run the cell kernel and the plain scan as two launches per iteration (needs the
 *                       Jacobian stream in the workspace) instead of the scan with the cell inside
 *   DEER_GRAD_FUSED=0   GRU deer_grad(): Jacobian kernel + plain reverse scan instead of the reverse scan with the
 *                       cell inside (needs the Jacobian stream in the workspace)
 *   DEER_ONE_LAUNCH=0   GRU, n <= 8: one launch per iteration even when the whole solve fits one launch
 *   DEER_FUSED_L, DEER_FUSED_W, DEER_SCAN_L
 *                       tile shapes of the n <= 8 kernels: positions per lane group (1, 2, 4, 8, 10, 12, 16; 24 for
 *                       the plain n = 4 scan) and wavefronts per tile (4 or 8); ignored when no such variant exists
 *   DEER_BATCH          Newton iterations enqueued per host round trip on a fresh context (1..8, default 4)
 *   DEER_VJP_MFMA=0     vector-ALU kernels for the vector-Jacobian products instead of the matrix-core ones
 *   DEER_MLP_MFMA=0     MLP fields outside the two-layer tanh shapes (fp32, n = 8, width 32 or 64): vector-ALU field
 *                       kernel instead of the matrix-core one
 * Test hooks (exercise paths that ordinary runs reach rarely; never set them in production):
 *   DEER_EPOCH0         first launch epoch of the context (default 1), to reach the wrap-around of the 30-bit
 *                       epoch that tags published words
 *   DEER_TEST_SPIN_LIMIT, DEER_TEST_EXTRA_WORKGROUPS
 *                       polls before a wait in the one-launch solve gives up, and a number (1..4) of workgroups
 *                       that solve also waits for although they do not exist: together they force the give-up path,
 *                       after which deer_eval() solves launch by launch */

#ifdef __cplusplus
}
#endif
#endif /* DEER_H */
