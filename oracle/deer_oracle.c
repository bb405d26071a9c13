/*
 * deer_oracle.c -- plain CPU fp64 oracle for the DEER hot path (arxiv 2309.12252).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It exists so that the GPU
 * library can be checked against something slow and obviously right.  Only
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 * It shares no code, header, table or helper with the HIP path.
 *
 * Everything is fp64, row-major, host memory, one loop per mathematical index.
 * No blocking, fusion or reordering beyond what the paper's equations state.
 *
 * What follows the paper and where:
 *   - sequential evaluation y_i = f(y_{i-1}, x_i)            Sec. 3.4
 *   - DEER iteration y <- L_G^{-1}[ f(y_shift) + G y_shift ],
 *     G = -df/dy, err = max|y_next - y|, loop while
 *     err > tol and iter < max_iter, err starts at 1e10      Sec. 3.1 eq. 3, 5; App. B.1
 *   - RNN inverse operator  y_i + G_i y_{i-1} = z_i           Sec. 3.4 eq. 11
 *   - ODE inverse operator  y_{i+1} = Gbar_i y_i + zbar_i,
 *     Gbar = exp(-G dt), zbar = G^{-1}(I - Gbar) z,
 *     midpoint values of G and z                              Sec. 3.3 eq. 8, 9; Table 3
 *   - associative operator on pairs (Gbar | zbar)             Sec. 3.3 eq. 10
 *   - backward derivative through the dual operator           Sec. 3.1.1 eq. 7
 *     (recurrence form, and the ODE form on the discretised operator)
 *
 * Readings where the paper is silent:
 *   - GRU cell: gates r, z, candidate c with the reset gate applied after the
 *     hidden projection; biases on the three input projections and on the
 *     candidate's hidden projection:
 *         r = sig(W_r x + b_r + U_r h)      z = sig(W_z x + b_z + U_z h)
 *         q = U_c h + b_hc                  c = tanh(W_c x + b_c + r*q)
 *         h' = (1 - z)*c + z*h
 *     theta = W[3n,d] (rows r|z|c), U[3n,n] (rows r|z|c), b[3n], b_hc[n].
 *   - MLP field: f(y) = W_out s(... s(W_1 y + b_1) ...) + b_out with
 *     nhid hidden layers of equal width and activation s = tanh, or softplus
 *     s(a) = log(1 + exp(a)) (the activation of the paper's two-body network,
 *     App. B.2: six linear layers, softplus on all but the last); theta = W_1[w,n], b_1[w],
 *     (W_k[w,w], b_k[w]) for k = 2..nhid, W_out[n,w], b_out[n]; nhid = 0 is
 *     the linear field W_out[n,n] y + b_out.
 *   - LSTM cell (Sec. 3.4 names it as an instance of the recurrence): u units, state y = (h | c) of 2u
 *     entries, gates in the order input, forget, candidate, output:
 *         i = sig(W_i x + U_i h + b_i)   f = sig(W_f x + U_f h + b_f)
 *         g = tanh(W_g x + U_g h + b_g)  o = sig(W_o x + U_o h + b_o)
 *         c' = f*c + i*g                 h' = o*tanh(c')
 *     theta = W[4u,d], U[4u,u], b[4u].  (The cell torch.nn.LSTMCell computes with its second bias at zero.)
 *   - LEM cell (the cell of the paper's last experiment, App. B.5 in the arXiv numbering: "long expressive memory";
 *     the paper prints no equations, the ones of the cited publication are used): u units, state (y | z) of 2u
 *     entries, step dt, two learned time scales:
 *         s1 = dt*sig(W_1 x + U_1 y + b_1)       s2 = dt*sig(W_2 x + U_2 y + b_2)
 *         z' = (1 - s1)*z + s1*tanh(W_z x + U_z y + b_z)
 *         y' = (1 - s2)*y + s2*tanh(W_y x + U_y z' + b_y)
 *     theta = W[4u,d], U[4u,u], b[4u], row blocks in the order 1 | 2 | z | y.  PARITY UNPINNED for the cell's
 *     definition (no library cell to compare with offline); its Jacobian and vector-Jacobian product are pinned to
 *     finite differences and autograd of the cell function.
 *   - affine RNN cell (a test hook, used to pin "Newton is exact for linear
 *     f"): f(h, x) = A h + Bm x + c, theta = A[n,n], Bm[n,d], c[n].
 *   - one global convergence test over batch, time and state; the returned
 *     iteration count is the number of linear solves performed.
 *   - ODE: the first grid point is pinned to y0 in every iterate, so err runs
 *     over grid points 1..T-1; G^{-1}(I - exp(-G dt)) is evaluated as
 *     dt * phi1(-G dt), phi1(A) = sum_k A^k/(k+1)!, which is the same matrix
 *     when G is invertible and stays defined when it is not.
 *
 * Parity pins live in tests/ (library GRU cell and autograd, finite
 * differences, closed forms, SciPy expm, RK4, brute force).
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_CELL_GRU 0
#define ORACLE_CELL_MLP 1
#define ORACLE_CELL_AFFINE 2
#define ORACLE_CELL_LSTM 3
#define ORACLE_CELL_LEM 4

typedef struct {
    int cell;   /* ORACLE_CELL_* */
    int n;      /* state size */
    int d;      /* input size (GRU, AFFINE); ignored for MLP */
    int width;  /* MLP hidden width */
    int nhid;   /* MLP number of hidden layers */
    int act;    /* MLP activation: 0 tanh, 1 softplus */
    double dt;  /* LEM: the step dt */
} oracle_cell;

static double sigmoid(double a) { return 1.0 / (1.0 + exp(-a)); }

long oracle_theta_count(const oracle_cell* c) {
    long n = c->n, d = c->d, w = c->width;
    if (c->cell == ORACLE_CELL_GRU) return 3 * n * d + 3 * n * n + 3 * n + n;
    if (c->cell == ORACLE_CELL_AFFINE) return n * n + n * d + n;
    if (c->cell == ORACLE_CELL_LSTM || c->cell == ORACLE_CELL_LEM) { long u = n / 2; return 4 * u * d + 4 * u * u + 4 * u; }
    if (c->nhid == 0) return n * n + n;
    return (w * n + w) + (long)(c->nhid - 1) * (w * w + w) + (n * w + n);
}

/* ------------------------------------------------------------------ GRU -- */

/* gate values of the GRU cell at (h, x); each output has n entries */
static void gru_gates(int n, int d, const double* th, const double* h, const double* x,
                      double* r, double* z, double* q, double* c) {
    const double* W = th;                 /* [3n, d] */
    const double* U = W + 3 * n * d;      /* [3n, n] */
    const double* b = U + 3 * n * n;      /* [3n]    */
    const double* bhc = b + 3 * n;        /* [n]     */
    for (int i = 0; i < n; i++) {
        double ar = b[i], az = b[n + i], ac = b[2 * n + i], qi = bhc[i];
        for (int k = 0; k < d; k++) {
            ar += W[(i)*d + k] * x[k];
            az += W[(n + i) * d + k] * x[k];
            ac += W[(2 * n + i) * d + k] * x[k];
        }
        for (int j = 0; j < n; j++) {
            ar += U[(i)*n + j] * h[j];
            az += U[(n + i) * n + j] * h[j];
            qi += U[(2 * n + i) * n + j] * h[j];
        }
        r[i] = sigmoid(ar);
        z[i] = sigmoid(az);
        q[i] = qi;
        c[i] = tanh(ac + r[i] * qi);
    }
}

static void gru_f(int n, int d, const double* th, const double* h, const double* x, double* out) {
    double* r = malloc(4 * n * sizeof(double));
    double *z = r + n, *q = z + n, *c = q + n;
    gru_gates(n, d, th, h, x, r, z, q, c);
    for (int i = 0; i < n; i++) out[i] = (1.0 - z[i]) * c[i] + z[i] * h[i];
    free(r);
}

/* J[i][j] = d h'_i / d h_j */
static void gru_jac(int n, int d, const double* th, const double* h, const double* x, double* J) {
    const double* U = th + 3 * n * d;
    const double *Ur = U, *Uz = U + n * n, *Uc = U + 2 * n * n;
    double* r = malloc(4 * n * sizeof(double));
    double *z = r + n, *q = z + n, *c = q + n;
    gru_gates(n, d, th, h, x, r, z, q, c);
    for (int i = 0; i < n; i++) {
        double dz = z[i] * (1.0 - z[i]);   /* sigmoid' at the z gate */
        double dr = r[i] * (1.0 - r[i]);   /* sigmoid' at the r gate */
        double dc = 1.0 - c[i] * c[i];     /* tanh' at the candidate */
        for (int j = 0; j < n; j++) {
            double dzi = dz * Uz[i * n + j];                              /* dz_i/dh_j */
            double dci = dc * (dr * Ur[i * n + j] * q[i] + r[i] * Uc[i * n + j]); /* dc_i/dh_j */
            J[i * n + j] = (h[i] - c[i]) * dzi + (1.0 - z[i]) * dci + (i == j ? z[i] : 0.0);
        }
    }
    free(r);
}

/* vector-Jacobian products of the GRU cell for an output cotangent lam:
 * dtheta += lam^T df/dtheta, dx = lam^T df/dx, dh = lam^T df/dh. */
static void gru_vjp(int n, int d, const double* th, const double* h, const double* x,
                    const double* lam, double* dtheta, double* dx, double* dh) {
    const double* W = th;
    const double* U = W + 3 * n * d;
    double* dW = dtheta;
    double* dU = dW + 3 * n * d;
    double* db = dU + 3 * n * n;
    double* dbhc = db + 3 * n;
    double* r = malloc(4 * n * sizeof(double));
    double *z = r + n, *q = z + n, *c = q + n;
    gru_gates(n, d, th, h, x, r, z, q, c);
    for (int k = 0; k < d; k++) dx[k] = 0.0;
    for (int j = 0; j < n; j++) dh[j] = z[j] * lam[j];   /* direct path h -> h' */
    for (int i = 0; i < n; i++) {
        double dcand = lam[i] * (1.0 - z[i]);                 /* dL/dc_i          */
        double dac = dcand * (1.0 - c[i] * c[i]);             /* pre-tanh         */
        double daz = lam[i] * (h[i] - c[i]) * z[i] * (1.0 - z[i]); /* pre-sigmoid z */
        double dq = dac * r[i];                               /* dL/dq_i          */
        double dar = dac * q[i] * r[i] * (1.0 - r[i]);        /* pre-sigmoid r    */
        for (int k = 0; k < d; k++) {
            dW[(i)*d + k] += dar * x[k];
            dW[(n + i) * d + k] += daz * x[k];
            dW[(2 * n + i) * d + k] += dac * x[k];
            dx[k] += W[(i)*d + k] * dar + W[(n + i) * d + k] * daz + W[(2 * n + i) * d + k] * dac;
        }
        for (int j = 0; j < n; j++) {
            dU[(i)*n + j] += dar * h[j];
            dU[(n + i) * n + j] += daz * h[j];
            dU[(2 * n + i) * n + j] += dq * h[j];
            dh[j] += U[(i)*n + j] * dar + U[(n + i) * n + j] * daz + U[(2 * n + i) * n + j] * dq;
        }
        db[i] += dar;
        db[n + i] += daz;
        db[2 * n + i] += dac;
        dbhc[i] += dq;
    }
    free(r);
}

/* ------------------------------------------------------------------ MLP -- */

/* activation and its derivative at pre-activation a */
static double mlp_act(int kind, double a) {
    if (kind == 0) return tanh(a);
    return a > 0.0 ? a + log1p(exp(-a)) : log1p(exp(a));   /* log(1 + e^a) without overflow */
}
static double mlp_dact(int kind, double a) {
    if (kind == 0) { double t = tanh(a); return 1.0 - t * t; }
    return sigmoid(a);
}

/* forward pass keeping every layer's activations: act[l] (l = 0..nhid-1), width w, and (when dact is
 * not NULL) the derivative of the activation at every unit */
static void mlp_forward_d(const oracle_cell* c, const double* th, const double* y, double* act, double* dact, double* out) {
    int n = c->n, w = c->width, L = c->nhid;
    const double* p = th;
    const double* in = y;
    int nin = n;
    for (int l = 0; l < L; l++) {
        const double* Wl = p;
        const double* bl = p + w * nin;
        for (int i = 0; i < w; i++) {
            double a = bl[i];
            for (int j = 0; j < nin; j++) a += Wl[i * nin + j] * in[j];
            act[l * w + i] = mlp_act(c->act, a);
            if (dact) dact[l * w + i] = mlp_dact(c->act, a);
        }
        p += w * nin + w;
        in = act + l * w;
        nin = w;
    }
    const double* Wo = p;
    const double* bo = p + n * nin;
    for (int i = 0; i < n; i++) {
        double a = bo[i];
        for (int j = 0; j < nin; j++) a += Wo[i * nin + j] * in[j];
        out[i] = a;
    }
}

static void mlp_forward(const oracle_cell* c, const double* th, const double* y, double* act, double* out) {
    mlp_forward_d(c, th, y, act, NULL, out);
}

static void mlp_f(const oracle_cell* c, const double* th, const double* y, double* out) {
    double* act = malloc((size_t)(c->nhid * c->width + 1) * sizeof(double));
    mlp_forward(c, th, y, act, out);
    free(act);
}

/* J = W_out D_L W_L ... D_1 W_1, D_l = diag(s'(pre-activation of layer l)): propagate the n
 * columns of the identity through the layers (forward mode). */
static void mlp_jac(const oracle_cell* c, const double* th, const double* y, double* J) {
    int n = c->n, w = c->width, L = c->nhid;
    int big = (w > n ? w : n);
    double* act = malloc((size_t)(L * w + 1) * sizeof(double));
    double* out = malloc((size_t)n * sizeof(double));
    double* S = malloc((size_t)big * n * sizeof(double));   /* d(layer input)/dy, [nin, n] */
    double* S2 = malloc((size_t)big * n * sizeof(double));
    double* dac = malloc((size_t)(L * w + 1) * sizeof(double));
    mlp_forward_d(c, th, y, act, dac, out);
    for (int i = 0; i < n; i++)
        for (int j = 0; j < n; j++) S[i * n + j] = (i == j ? 1.0 : 0.0);
    const double* p = th;
    int nin = n;
    for (int l = 0; l < L; l++) {
        const double* Wl = p;
        for (int i = 0; i < w; i++) {
            double dact = dac[l * w + i];
            for (int j = 0; j < n; j++) {
                double s = 0.0;
                for (int k = 0; k < nin; k++) s += Wl[i * nin + k] * S[k * n + j];
                S2[i * n + j] = dact * s;
            }
        }
        memcpy(S, S2, (size_t)w * n * sizeof(double));
        p += w * nin + w;
        nin = w;
    }
    const double* Wo = p;
    for (int i = 0; i < n; i++)
        for (int j = 0; j < n; j++) {
            double s = 0.0;
            for (int k = 0; k < nin; k++) s += Wo[i * nin + k] * S[k * n + j];
            J[i * n + j] = s;
        }
    free(act); free(out); free(S); free(S2); free(dac);
}

/* ----------------------------------------------------------------- LSTM -- */

/* gate values at (y = (h | c), x); each output has u entries; cn = c', tc = tanh(c') */
static void lstm_gates(int u, int d, const double* th, const double* y, const double* x,
                       double* gi, double* gf, double* gg, double* go, double* cn, double* tc) {
    const double* W = th;                 /* [4u, d] */
    const double* U = W + 4 * u * d;      /* [4u, u] */
    const double* b = U + 4 * u * u;      /* [4u]    */
    const double* h = y;
    const double* c = y + u;
    for (int j = 0; j < u; j++) {
        double a[4];
        for (int q = 0; q < 4; q++) {
            a[q] = b[q * u + j];
            for (int k = 0; k < d; k++) a[q] += W[(q * u + j) * d + k] * x[k];
            for (int k = 0; k < u; k++) a[q] += U[(q * u + j) * u + k] * h[k];
        }
        gi[j] = sigmoid(a[0]);
        gf[j] = sigmoid(a[1]);
        gg[j] = tanh(a[2]);
        go[j] = sigmoid(a[3]);
        cn[j] = gf[j] * c[j] + gi[j] * gg[j];
        tc[j] = tanh(cn[j]);
    }
}

static void lstm_f(int u, int d, const double* th, const double* y, const double* x, double* out) {
    double* g = malloc(6 * u * sizeof(double));
    lstm_gates(u, d, th, y, x, g, g + u, g + 2 * u, g + 3 * u, g + 4 * u, g + 5 * u);
    for (int j = 0; j < u; j++) {
        out[j] = g[3 * u + j] * g[5 * u + j];   /* h' = o tanh(c') */
        out[u + j] = g[4 * u + j];              /* c'              */
    }
    free(g);
}

/* J = d(h' | c') / d(h | c), 2u x 2u, row-major */
static void lstm_jac(int u, int d, const double* th, const double* y, const double* x, double* J) {
    const double* U = th + 4 * u * d;
    const double* c = y + u;
    int n = 2 * u;
    double* g = malloc(6 * u * sizeof(double));
    double *gi = g, *gf = g + u, *gg = g + 2 * u, *go = g + 3 * u, *tc = g + 5 * u;
    lstm_gates(u, d, th, y, x, gi, gf, gg, go, g + 4 * u, tc);
    memset(J, 0, (size_t)n * n * sizeof(double));
    for (int j = 0; j < u; j++) {
        double dti = gi[j] * (1.0 - gi[j]), dtf = gf[j] * (1.0 - gf[j]);
        double dtg = 1.0 - gg[j] * gg[j], dto = go[j] * (1.0 - go[j]);
        double dtc = 1.0 - tc[j] * tc[j];
        for (int k = 0; k < u; k++) {
            /* dc'_j/dh_k */
            double dc = c[j] * dtf * U[(u + j) * u + k] + gg[j] * dti * U[(j)*u + k] + gi[j] * dtg * U[(2 * u + j) * u + k];
            J[(u + j) * n + k] = dc;
            /* dh'_j/dh_k */
            J[j * n + k] = tc[j] * dto * U[(3 * u + j) * u + k] + go[j] * dtc * dc;
        }
        J[(u + j) * n + u + j] = gf[j];                 /* dc'_j/dc_j */
        J[j * n + u + j] = go[j] * dtc * gf[j];         /* dh'_j/dc_j */
    }
    free(g);
}

/* vector-Jacobian products for an output cotangent lam = (lam_h | lam_c): dtheta += ..., dx, dy overwritten */
static void lstm_vjp(int u, int d, const double* th, const double* y, const double* x,
                     const double* lam, double* dtheta, double* dx, double* dy) {
    const double* W = th;
    const double* U = W + 4 * u * d;
    double* dW = dtheta;
    double* dU = dW + 4 * u * d;
    double* db = dU + 4 * u * u;
    const double* h = y;
    const double* c = y + u;
    double* g = malloc(6 * u * sizeof(double));
    double *gi = g, *gf = g + u, *gg = g + 2 * u, *go = g + 3 * u, *tc = g + 5 * u;
    lstm_gates(u, d, th, y, x, gi, gf, gg, go, g + 4 * u, tc);
    for (int k = 0; k < d; k++) dx[k] = 0.0;
    for (int k = 0; k < 2 * u; k++) dy[k] = 0.0;
    for (int j = 0; j < u; j++) {
        double dcn = lam[u + j] + lam[j] * go[j] * (1.0 - tc[j] * tc[j]);   /* dL/dc'_j */
        double da[4];
        da[0] = dcn * gg[j] * gi[j] * (1.0 - gi[j]);           /* input gate, pre-sigmoid   */
        da[1] = dcn * c[j] * gf[j] * (1.0 - gf[j]);            /* forget gate               */
        da[2] = dcn * gi[j] * (1.0 - gg[j] * gg[j]);           /* candidate, pre-tanh       */
        da[3] = lam[j] * tc[j] * go[j] * (1.0 - go[j]);        /* output gate               */
        dy[u + j] += dcn * gf[j];                              /* direct path c -> c'       */
        for (int q = 0; q < 4; q++) {
            for (int k = 0; k < d; k++) {
                dW[(q * u + j) * d + k] += da[q] * x[k];
                dx[k] += W[(q * u + j) * d + k] * da[q];
            }
            for (int k = 0; k < u; k++) {
                dU[(q * u + j) * u + k] += da[q] * h[k];
                dy[k] += U[(q * u + j) * u + k] * da[q];
            }
            db[q * u + j] += da[q];
        }
    }
    free(g);
}

/* ------------------------------------------------------------------ LEM -- */

/* s1, s2 (time scales, dt included), gz = tanh(.) of the z update, zn = z', gy = tanh(.) of the y update; u entries each */
static void lem_gates(int u, int d, double dt, const double* th, const double* s, const double* x,
                      double* s1, double* s2, double* gz, double* zn, double* gy) {
    const double* W = th;                 /* [4u, d] */
    const double* U = W + 4 * u * d;      /* [4u, u] */
    const double* b = U + 4 * u * u;      /* [4u]    */
    const double* y = s;
    const double* z = s + u;
    for (int j = 0; j < u; j++) {
        double a[3];
        for (int q = 0; q < 3; q++) {
            a[q] = b[q * u + j];
            for (int k = 0; k < d; k++) a[q] += W[(q * u + j) * d + k] * x[k];
            for (int k = 0; k < u; k++) a[q] += U[(q * u + j) * u + k] * y[k];
        }
        s1[j] = dt * sigmoid(a[0]);
        s2[j] = dt * sigmoid(a[1]);
        gz[j] = tanh(a[2]);
        zn[j] = (1.0 - s1[j]) * z[j] + s1[j] * gz[j];
    }
    for (int j = 0; j < u; j++) {   /* the y update sees the new z */
        double a = b[3 * u + j];
        for (int k = 0; k < d; k++) a += W[(3 * u + j) * d + k] * x[k];
        for (int k = 0; k < u; k++) a += U[(3 * u + j) * u + k] * zn[k];
        gy[j] = tanh(a);
    }
}

static void lem_f(int u, int d, double dt, const double* th, const double* s, const double* x, double* out) {
    double* g = malloc(5 * u * sizeof(double));
    double *s2 = g + u, *zn = g + 3 * u, *gy = g + 4 * u;
    lem_gates(u, d, dt, th, s, x, g, s2, g + 2 * u, zn, gy);
    for (int j = 0; j < u; j++) {
        out[j] = (1.0 - s2[j]) * s[j] + s2[j] * gy[j];
        out[u + j] = zn[j];
    }
    free(g);
}

/* J = d(y' | z') / d(y | z), 2u x 2u, row-major */
static void lem_jac(int u, int d, double dt, const double* th, const double* s, const double* x, double* J) {
    const double* U = th + 4 * u * d;
    const double* y = s;
    const double* z = s + u;
    int n = 2 * u;
    double* g = malloc(5 * u * sizeof(double));
    double *s1 = g, *s2 = g + u, *gz = g + 2 * u, *gy = g + 4 * u;
    lem_gates(u, d, dt, th, s, x, s1, s2, gz, g + 3 * u, gy);
    memset(J, 0, (size_t)n * n * sizeof(double));
    /* rows of z': dz'_j/dy_k and dz'_j/dz_j;  d s1_j / d a = s1_j (1 - s1_j / dt) */
    for (int j = 0; j < u; j++) {
        double ds1 = s1[j] * (1.0 - s1[j] / dt);
        for (int k = 0; k < u; k++)
            J[(u + j) * n + k] = ds1 * (gz[j] - z[j]) * U[(j)*u + k] + s1[j] * (1.0 - gz[j] * gz[j]) * U[(2 * u + j) * u + k];
        J[(u + j) * n + u + j] = 1.0 - s1[j];
    }
    /* rows of y': through s2 (depends on y), the direct term, and tanh(. U_y z') */
    for (int j = 0; j < u; j++) {
        double ds2 = s2[j] * (1.0 - s2[j] / dt);
        double dgy = s2[j] * (1.0 - gy[j] * gy[j]);
        for (int k = 0; k < n; k++) {
            double acc = 0.0;
            for (int m = 0; m < u; m++) acc += U[(3 * u + j) * u + m] * J[(u + m) * n + k];
            J[j * n + k] = dgy * acc;
        }
        for (int k = 0; k < u; k++) J[j * n + k] += ds2 * (gy[j] - y[j]) * U[(u + j) * u + k];
        J[j * n + j] += 1.0 - s2[j];
    }
    free(g);
}

/* vector-Jacobian products for an output cotangent lam = (lam_y | lam_z): dtheta += ..., dx, ds overwritten */
static void lem_vjp(int u, int d, double dt, const double* th, const double* s, const double* x,
                    const double* lam, double* dtheta, double* dx, double* ds) {
    const double* W = th;
    const double* U = W + 4 * u * d;
    double* dW = dtheta;
    double* dU = dW + 4 * u * d;
    double* db = dU + 4 * u * u;
    const double* y = s;
    const double* z = s + u;
    double* g = malloc(6 * u * sizeof(double));
    double *s1 = g, *s2 = g + u, *gz = g + 2 * u, *zn = g + 3 * u, *gy = g + 4 * u, *dzn = g + 5 * u;
    lem_gates(u, d, dt, th, s, x, s1, s2, gz, zn, gy);
    for (int k = 0; k < d; k++) dx[k] = 0.0;
    for (int k = 0; k < 2 * u; k++) ds[k] = 0.0;
    for (int m = 0; m < u; m++) dzn[m] = lam[u + m];
    /* the y update: pre-activations of s2 (block 1) and of tanh(W_y x + U_y z' + b_y) (block 3) */
    for (int j = 0; j < u; j++) {
        double da2 = lam[j] * (gy[j] - y[j]) * s2[j] * (1.0 - s2[j] / dt);
        double day = lam[j] * s2[j] * (1.0 - gy[j] * gy[j]);
        ds[j] += lam[j] * (1.0 - s2[j]);
        for (int k = 0; k < d; k++) {
            dW[(u + j) * d + k] += da2 * x[k];
            dW[(3 * u + j) * d + k] += day * x[k];
            dx[k] += W[(u + j) * d + k] * da2 + W[(3 * u + j) * d + k] * day;
        }
        for (int k = 0; k < u; k++) {
            dU[(u + j) * u + k] += da2 * y[k];
            dU[(3 * u + j) * u + k] += day * zn[k];
            ds[k] += U[(u + j) * u + k] * da2;
            dzn[k] += U[(3 * u + j) * u + k] * day;
        }
        db[u + j] += da2;
        db[3 * u + j] += day;
    }
    /* the z update: pre-activations of s1 (block 0) and of tanh(W_z x + U_z y + b_z) (block 2) */
    for (int j = 0; j < u; j++) {
        double da1 = dzn[j] * (gz[j] - z[j]) * s1[j] * (1.0 - s1[j] / dt);
        double daz = dzn[j] * s1[j] * (1.0 - gz[j] * gz[j]);
        ds[u + j] += dzn[j] * (1.0 - s1[j]);
        for (int k = 0; k < d; k++) {
            dW[(j)*d + k] += da1 * x[k];
            dW[(2 * u + j) * d + k] += daz * x[k];
            dx[k] += W[(j)*d + k] * da1 + W[(2 * u + j) * d + k] * daz;
        }
        for (int k = 0; k < u; k++) {
            dU[(j)*u + k] += da1 * y[k];
            dU[(2 * u + j) * u + k] += daz * y[k];
            ds[k] += U[(j)*u + k] * da1 + U[(2 * u + j) * u + k] * daz;
        }
        db[j] += da1;
        db[2 * u + j] += daz;
    }
    free(g);
}

/* --------------------------------------------------------------- affine -- */

static void affine_f(int n, int d, const double* th, const double* h, const double* x, double* out) {
    const double* A = th;
    const double* Bm = A + n * n;
    const double* cc = Bm + n * d;
    for (int i = 0; i < n; i++) {
        double a = cc[i];
        for (int j = 0; j < n; j++) a += A[i * n + j] * h[j];
        for (int k = 0; k < d; k++) a += Bm[i * d + k] * x[k];
        out[i] = a;
    }
}

/* ------------------------------------------------------ cell dispatchers -- */

void oracle_cell_f(const oracle_cell* c, const double* th, const double* h, const double* x, double* out) {
    if (c->cell == ORACLE_CELL_GRU) gru_f(c->n, c->d, th, h, x, out);
    else if (c->cell == ORACLE_CELL_LSTM) lstm_f(c->n / 2, c->d, th, h, x, out);
    else if (c->cell == ORACLE_CELL_LEM) lem_f(c->n / 2, c->d, c->dt, th, h, x, out);
    else if (c->cell == ORACLE_CELL_MLP) mlp_f(c, th, h, out);
    else affine_f(c->n, c->d, th, h, x, out);
}

void oracle_cell_jac(const oracle_cell* c, const double* th, const double* h, const double* x, double* J) {
    if (c->cell == ORACLE_CELL_GRU) gru_jac(c->n, c->d, th, h, x, J);
    else if (c->cell == ORACLE_CELL_LSTM) lstm_jac(c->n / 2, c->d, th, h, x, J);
    else if (c->cell == ORACLE_CELL_LEM) lem_jac(c->n / 2, c->d, c->dt, th, h, x, J);
    else if (c->cell == ORACLE_CELL_MLP) mlp_jac(c, th, h, J);
    else memcpy(J, th, (size_t)c->n * c->n * sizeof(double));
}

/* GRU only. dtheta is accumulated into; dx and dh are overwritten. */
void oracle_gru_vjp(int n, int d, const double* th, const double* h, const double* x,
                    const double* lam, double* dtheta, double* dx, double* dh) {
    gru_vjp(n, d, th, h, x, lam, dtheta, dx, dh);
}

/* GRU, LSTM and LEM: vector-Jacobian products of the cell; dtheta is accumulated into, dx and dh overwritten */
void oracle_cell_vjp(const oracle_cell* c, const double* th, const double* h, const double* x,
                     const double* lam, double* dtheta, double* dx, double* dh) {
    if (c->cell == ORACLE_CELL_GRU) gru_vjp(c->n, c->d, th, h, x, lam, dtheta, dx, dh);
    else if (c->cell == ORACLE_CELL_LEM) lem_vjp(c->n / 2, c->d, c->dt, th, h, x, lam, dtheta, dx, dh);
    else lstm_vjp(c->n / 2, c->d, th, h, x, lam, dtheta, dx, dh);
}

/* --------------------------------------------- affine pairs and the scan -- */

/* Sec. 3.3 eq. 10: (Gi | zi) is the earlier element, (Gj | zj) the later one;
 * result = (Gj Gi | Gj zi + zj).  Outputs must not alias the inputs. */
void oracle_affine_combine(int n, const double* Gi, const double* zi, const double* Gj, const double* zj,
                           double* Gout, double* zout) {
    for (int r = 0; r < n; r++) {
        for (int c = 0; c < n; c++) {
            double s = 0.0;
            for (int k = 0; k < n; k++) s += Gj[r * n + k] * Gi[k * n + c];
            Gout[r * n + c] = s;
        }
        double s = zj[r];
        for (int k = 0; k < n; k++) s += Gj[r * n + k] * zi[k];
        zout[r] = s;
    }
}

/* Sec. 3.3 eq. 9 / Sec. 3.4 eq. 11 solved one step after the other:
 * y_i = Gbar_i y_{i-1} + zbar_i, i = 1..T, y_0 given; y holds y_1..y_T. */
void oracle_linrec_serial(int n, long T, const double* Gbar, const double* zbar, const double* y0, double* y) {
    const double* prev = y0;
    for (long i = 0; i < T; i++) {
        const double* G = Gbar + i * n * n;
        for (int r = 0; r < n; r++) {
            double s = zbar[i * n + r];
            for (int k = 0; k < n; k++) s += G[r * n + k] * prev[k];
            y[i * n + r] = s;
        }
        prev = y + i * n;
    }
}

/* The same result through the definition with the associative operator:
 * running value c <- c . element_i, started at c_0 = (I | y0); y_i is the
 * vector part of the running value (Sec. 3.3, text after eq. 10). */
void oracle_affine_scan(int n, long T, const double* Gbar, const double* zbar, const double* y0, double* y) {
    double* G = malloc((size_t)n * n * sizeof(double));
    double* z = malloc((size_t)n * sizeof(double));
    double* G2 = malloc((size_t)n * n * sizeof(double));
    double* z2 = malloc((size_t)n * sizeof(double));
    for (int r = 0; r < n; r++) {
        for (int c = 0; c < n; c++) G[r * n + c] = (r == c ? 1.0 : 0.0);
        z[r] = y0[r];
    }
    for (long i = 0; i < T; i++) {
        oracle_affine_combine(n, G, z, Gbar + i * n * n, zbar + i * n, G2, z2);
        memcpy(G, G2, (size_t)n * n * sizeof(double));
        memcpy(z, z2, (size_t)n * sizeof(double));
        memcpy(y + i * n, z, (size_t)n * sizeof(double));
    }
    free(G); free(z); free(G2); free(z2);
}

/* ------------------------------------------------ sequential evaluation -- */

/* y[b, i-1] = y_i = f(y_{i-1}, x_i), i = 1..T (Sec. 3.4). x is [B,T,d], y0 [B,n], y [B,T,n]. */
void oracle_seq_eval(const oracle_cell* c, const double* th, long B, long T, const double* x,
                     const double* y0, double* y, int nthreads) {
    int n = c->n, d = c->d;
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for num_threads(nthreads) schedule(static)
    for (long b = 0; b < B; b++) {
        const double* h = y0 + b * n;
        for (long i = 0; i < T; i++) {
            double* out = y + (b * T + i) * n;
            oracle_cell_f(c, th, h, x ? x + (b * T + i) * d : NULL, out);
            h = out;
        }
    }
}

/* ------------------------------------------------------- DEER for an RNN -- */

/* DEER iteration for y_i = f(y_{i-1}, x_i) (Sec. 3.1 eq. 3 and 5, Sec. 3.4 eq. 11, App. B.1).
 * guess may be NULL (zeros). err_hist (may be NULL) receives err after every iteration
 * (max_iter entries at most). Returns the number of iterations (linear solves) done. */
int oracle_deer_eval(const oracle_cell* c, const double* th, long B, long T, const double* x,
                     const double* y0, const double* guess, double tol, int max_iter,
                     double* y, double* final_err, double* err_hist, int nthreads) {
    int n = c->n, d = c->d;
    size_t total = (size_t)B * T * n;
    double* ynew = malloc(total * sizeof(double));
    if (guess) memcpy(y, guess, total * sizeof(double));
    else memset(y, 0, total * sizeof(double));
    if (nthreads < 1) nthreads = 1;
    double err = 1e10;
    int iter = 0;
    while (err > tol && iter < max_iter) {
        double errmax = 0.0;
        int bad = 0;
#pragma omp parallel for num_threads(nthreads) schedule(static) reduction(max : errmax) reduction(| : bad)
        for (long b = 0; b < B; b++) {
            double* f = malloc((size_t)(3 * n + n * n) * sizeof(double));
            double *zv = f + n, *G = zv + n;
            for (long i = 0; i < T; i++) {
                /* shifter: the argument of f at position i is the previous iterate at i-1 */
                const double* hs = (i == 0 ? y0 + b * n : y + (b * T + i - 1) * n);
                const double* xi = x ? x + (b * T + i) * d : NULL;
                oracle_cell_f(c, th, hs, xi, f);
                oracle_cell_jac(c, th, hs, xi, G);
                for (int k = 0; k < n * n; k++) G[k] = -G[k];               /* G = -df/dy  */
                for (int r = 0; r < n; r++) {                                /* z = f + G y */
                    double s = f[r];
                    for (int k = 0; k < n; k++) s += G[r * n + k] * hs[k];
                    zv[r] = s;
                }
                /* inverse operator: y_i + G_i y_{i-1} = z_i with the new y_{i-1} */
                const double* hp = (i == 0 ? y0 + b * n : ynew + (b * T + i - 1) * n);
                for (int r = 0; r < n; r++) {
                    double s = zv[r];
                    for (int k = 0; k < n; k++) s -= G[r * n + k] * hp[k];
                    ynew[(b * T + i) * n + r] = s;
                    double dlt = fabs(s - y[(b * T + i) * n + r]);
                    if (dlt > errmax) errmax = dlt;
                    if (!(dlt == dlt) || isinf(dlt)) bad = 1;
                }
            }
            free(f);
        }
        err = bad ? NAN : errmax;
        memcpy(y, ynew, total * sizeof(double));
        if (err_hist) err_hist[iter] = err;
        iter++;
    }
    if (final_err) *final_err = err;
    free(ynew);
    return iter;
}

/* ---------------------------------------------- backward derivative, GRU -- */

/* Sec. 3.1.1 eq. 7 for the RNN operator (L y)_i = y_i + G_i y_{i-1}, G_i = -J_i:
 * first lam = (dL/dy) L_G^{-1}, i.e. lam_T = g_T, lam_i = g_i - G_{i+1}^T lam_{i+1};
 * then the vector-Jacobian product of f with lam at every position.
 * J_i is evaluated at the given trajectory y (h = y_{i-1}, y_0 for i = 1).
 * g, y: [B,T,n]; outputs dtheta [theta_count] (overwritten), dx [B,T,d], dy0 [B,n]. */
void oracle_gru_grad(int n, int d, const double* th, long B, long T, const double* x,
                     const double* y0, const double* y, const double* g,
                     double* dtheta, double* dx, double* dy0) {
    long P = 3L * n * d + 3L * n * n + 4L * n;
    memset(dtheta, 0, (size_t)P * sizeof(double));
    double* lam = malloc((size_t)T * n * sizeof(double));
    double* G = malloc((size_t)n * n * sizeof(double));
    double* dh = malloc((size_t)n * sizeof(double));
    for (long b = 0; b < B; b++) {
        for (long i = T - 1; i >= 0; i--) {
            for (int r = 0; r < n; r++) lam[i * n + r] = g[(b * T + i) * n + r];
            if (i < T - 1) {
                /* G_{i+1} uses h = y_i and x_{i+1} */
                gru_jac(n, d, th, y + (b * T + i) * n, x + (b * T + i + 1) * d, G);
                for (int k = 0; k < n * n; k++) G[k] = -G[k];
                for (int r = 0; r < n; r++) {
                    double s = 0.0;
                    for (int k = 0; k < n; k++) s += G[k * n + r] * lam[(i + 1) * n + k];
                    lam[i * n + r] -= s;
                }
            }
        }
        for (long i = 0; i < T; i++) {
            const double* h = (i == 0 ? y0 + b * n : y + (b * T + i - 1) * n);
            gru_vjp(n, d, th, h, x + (b * T + i) * d, lam + i * n, dtheta, dx + (b * T + i) * d, dh);
            if (i == 0) memcpy(dy0 + b * n, dh, (size_t)n * sizeof(double));
        }
    }
    free(lam); free(G); free(dh);
}

/* The same backward derivative (Sec. 3.1.1 eq. 7) for any recurrent cell with a vector-Jacobian product
 * (GRU, LSTM); c->n is the state size. */
void oracle_rnn_grad(const oracle_cell* c, const double* th, long B, long T, const double* x,
                     const double* y0, const double* y, const double* g,
                     double* dtheta, double* dx, double* dy0) {
    int n = c->n, d = c->d;
    long P = oracle_theta_count(c);
    memset(dtheta, 0, (size_t)P * sizeof(double));
    double* lam = malloc((size_t)T * n * sizeof(double));
    double* J = malloc((size_t)n * n * sizeof(double));
    double* dh = malloc((size_t)n * sizeof(double));
    for (long b = 0; b < B; b++) {
        for (long i = T - 1; i >= 0; i--) {
            for (int r = 0; r < n; r++) lam[i * n + r] = g[(b * T + i) * n + r];
            if (i < T - 1) {
                oracle_cell_jac(c, th, y + (b * T + i) * n, x + (b * T + i + 1) * d, J);   /* J_{i+1} at h = y_i */
                for (int r = 0; r < n; r++) {
                    double a = 0.0;
                    for (int k = 0; k < n; k++) a += J[k * n + r] * lam[(i + 1) * n + k];
                    lam[i * n + r] += a;
                }
            }
        }
        for (long i = 0; i < T; i++) {
            const double* h = (i == 0 ? y0 + b * n : y + (b * T + i - 1) * n);
            oracle_cell_vjp(c, th, h, x + (b * T + i) * d, lam + i * n, dtheta, dx + (b * T + i) * d, dh);
            if (i == 0) memcpy(dy0 + b * n, dh, (size_t)n * sizeof(double));
        }
    }
    free(lam); free(J); free(dh);
}

/* ----------------------------------------- multi-head GRU with strides -- */

/* Sec. 4.4 / App. B.4: the state is split into H heads of n channels, every head a GRU of its own
 * (parameters th[h], inputs x[b,i,h,:]), and head h looks back s_h = 2^(h mod K) steps instead of one
 * (K stride levels dealt out to the heads in turn):
 *     y[b,i,h] = f_h( y[b,i-s_h,h], x[b,i,h] ),   y[b,i-s_h,h] = y0[b,h] for i < s_h
 * (0-based i).  Layouts: x [B,T,H,d], y0 [B,H,n], y [B,T,H,n], th [H][theta_count]. */
static long mh_stride(int h, int K) { return 1L << (h % K); }

void oracle_mh_seq_eval(int n, int d, int H, int K, const double* th, long B, long T, const double* x,
                        const double* y0, double* y, int nthreads) {
    long P = 3L * n * d + 3L * n * n + 4L * n;
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for num_threads(nthreads) schedule(static)
    for (long bh = 0; bh < B * H; bh++) {
        long b = bh / H;
        int h = (int)(bh % H);
        long s = mh_stride(h, K);
        for (long i = 0; i < T; i++) {
            const double* prev = (i >= s ? y + ((b * T + i - s) * H + h) * n : y0 + (b * H + h) * n);
            gru_f(n, d, th + h * P, prev, x + ((b * T + i) * H + h) * d, y + ((b * T + i) * H + h) * n);
        }
    }
}

/* DEER for the same recurrence: the shifter hands f the previous iterate s_h steps back, the linear
 * operator is (L y)_i = y_i + G_i y_{i-s_h} (Sec. 3.4 eq. 11 with that delay), solved serially; one
 * convergence test over batch, time, heads and channels (App. B.1). */
int oracle_mh_deer_eval(int n, int d, int H, int K, const double* th, long B, long T, const double* x,
                        const double* y0, const double* guess, double tol, int max_iter,
                        double* y, double* final_err, double* err_hist, int nthreads) {
    long P = 3L * n * d + 3L * n * n + 4L * n;
    size_t total = (size_t)B * T * H * n;
    double* ynew = malloc(total * sizeof(double));
    if (guess) memcpy(y, guess, total * sizeof(double));
    else memset(y, 0, total * sizeof(double));
    if (nthreads < 1) nthreads = 1;
    double err = 1e10;
    int iter = 0;
    while (err > tol && iter < max_iter) {
        double errmax = 0.0;
        int bad = 0;
#pragma omp parallel for num_threads(nthreads) schedule(static) reduction(max : errmax) reduction(| : bad)
        for (long bh = 0; bh < B * H; bh++) {
            long b = bh / H;
            int h = (int)(bh % H);
            long s = mh_stride(h, K);
            const double* thh = th + h * P;
            double* f = malloc((size_t)(2 * n + n * n) * sizeof(double));
            double *zv = f + n, *G = zv + n;
            for (long i = 0; i < T; i++) {
                const double* hs = (i >= s ? y + ((b * T + i - s) * H + h) * n : y0 + (b * H + h) * n);
                const double* xi = x + ((b * T + i) * H + h) * d;
                gru_f(n, d, thh, hs, xi, f);
                gru_jac(n, d, thh, hs, xi, G);
                for (int k = 0; k < n * n; k++) G[k] = -G[k];
                for (int r = 0; r < n; r++) {
                    double a = f[r];
                    for (int k = 0; k < n; k++) a += G[r * n + k] * hs[k];
                    zv[r] = a;
                }
                const double* hp = (i >= s ? ynew + ((b * T + i - s) * H + h) * n : y0 + (b * H + h) * n);
                for (int r = 0; r < n; r++) {
                    double a = zv[r];
                    for (int k = 0; k < n; k++) a -= G[r * n + k] * hp[k];
                    size_t at = (size_t)((b * T + i) * H + h) * n + r;
                    ynew[at] = a;
                    double dlt = fabs(a - y[at]);
                    if (dlt > errmax) errmax = dlt;
                    if (!(dlt == dlt) || isinf(dlt)) bad = 1;
                }
            }
            free(f);
        }
        err = bad ? NAN : errmax;
        memcpy(y, ynew, total * sizeof(double));
        if (err_hist) err_hist[iter] = err;
        iter++;
    }
    if (final_err) *final_err = err;
    free(ynew);
    return iter;
}

/* Backward derivative (Sec. 3.1.1 eq. 7) for the strided operator: lam_i = g_i + J_{i+s}^T lam_{i+s}
 * (no term when i + s >= T), J_{i+s} evaluated at h = y_i and x_{i+s}; then the vector-Jacobian product
 * of f_h at every position; the first s positions of a head all start from y0, so dL/dy0 collects s terms.
 * Outputs: dtheta [H][theta_count] (overwritten), dx [B,T,H,d], dy0 [B,H,n]. */
void oracle_mh_gru_grad(int n, int d, int H, int K, const double* th, long B, long T, const double* x,
                        const double* y0, const double* y, const double* g,
                        double* dtheta, double* dx, double* dy0) {
    long P = 3L * n * d + 3L * n * n + 4L * n;
    memset(dtheta, 0, (size_t)H * P * sizeof(double));
    memset(dy0, 0, (size_t)B * H * n * sizeof(double));
    double* lam = malloc((size_t)T * n * sizeof(double));
    double* G = malloc((size_t)n * n * sizeof(double));
    double* dh = malloc((size_t)n * sizeof(double));
    for (long b = 0; b < B; b++)
        for (int h = 0; h < H; h++) {
            long s = mh_stride(h, K);
            const double* thh = th + h * P;
            for (long i = T - 1; i >= 0; i--) {
                for (int r = 0; r < n; r++) lam[i * n + r] = g[((b * T + i) * H + h) * n + r];
                if (i + s < T) {
                    gru_jac(n, d, thh, y + ((b * T + i) * H + h) * n, x + ((b * T + i + s) * H + h) * d, G);
                    for (int r = 0; r < n; r++) {
                        double a = 0.0;
                        for (int k = 0; k < n; k++) a += G[k * n + r] * lam[(i + s) * n + k];
                        lam[i * n + r] += a;
                    }
                }
            }
            for (long i = 0; i < T; i++) {
                const double* hs = (i >= s ? y + ((b * T + i - s) * H + h) * n : y0 + (b * H + h) * n);
                gru_vjp(n, d, thh, hs, x + ((b * T + i) * H + h) * d, lam + i * n, dtheta + h * P,
                        dx + ((b * T + i) * H + h) * d, dh);
                if (i < s)
                    for (int r = 0; r < n; r++) dy0[(b * H + h) * n + r] += dh[r];
            }
        }
    free(lam); free(G); free(dh);
}

/* ------------------------------------------- matrix exponential and phi1 -- */

static void matmul(int n, const double* A, const double* Bm, double* C) {
    for (int r = 0; r < n; r++)
        for (int c = 0; c < n; c++) {
            double s = 0.0;
            for (int k = 0; k < n; k++) s += A[r * n + k] * Bm[k * n + c];
            C[r * n + c] = s;
        }
}

/* E = exp(A) and P = phi1(A) = sum_{k>=0} A^k/(k+1)!  (so that A P = E - I).
 * Taylor series on A/2^s with the max-row-sum norm of A/2^s at most 1/2, summed
 * until a term no longer changes the sum, then s doublings:
 * exp(2X) = exp(X)^2, phi1(2X) = (exp(X) + I) phi1(X) / 2. */
void oracle_expm_phi1(int n, const double* A, double* E, double* P) {
    size_t nn = (size_t)n * n;
    double* X = malloc(4 * nn * sizeof(double));
    double *term = X + nn, *tmp = term + nn, *tmp2 = tmp + nn;
    double norm = 0.0;
    for (int r = 0; r < n; r++) {
        double s = 0.0;
        for (int c = 0; c < n; c++) s += fabs(A[r * n + c]);
        if (s > norm) norm = s;
    }
    int s = 0;
    while (norm > 0.5 && s < 60) { norm *= 0.5; s++; }
    double scale = ldexp(1.0, -s);
    for (size_t k = 0; k < nn; k++) X[k] = A[k] * scale;
    for (int r = 0; r < n; r++)
        for (int c = 0; c < n; c++) {
            double id = (r == c ? 1.0 : 0.0);
            term[r * n + c] = id;   /* X^0/0! */
            E[r * n + c] = id;
            P[r * n + c] = id;      /* X^0/1! */
        }
    for (int k = 1; k <= 40; k++) {
        matmul(n, term, X, tmp);
        double tmax = 0.0;
        for (size_t q = 0; q < nn; q++) {
            term[q] = tmp[q] / k;                 /* X^k/k!      */
            E[q] += term[q];
            P[q] += term[q] / (k + 1);            /* X^k/(k+1)!  */
            if (fabs(term[q]) > tmax) tmax = fabs(term[q]);
        }
        if (tmax < 1e-30) break;
    }
    for (int j = 0; j < s; j++) {
        for (int r = 0; r < n; r++)
            for (int c = 0; c < n; c++) tmp[r * n + c] = 0.5 * (E[r * n + c] + (r == c ? 1.0 : 0.0));
        matmul(n, tmp, P, tmp2);
        memcpy(P, tmp2, nn * sizeof(double));
        matmul(n, E, E, tmp);
        memcpy(E, tmp, nn * sizeof(double));
    }
    free(X);
}

/* One interval of the ODE inverse operator (Sec. 3.3 eq. 9 with midpoint values):
 * Gc = (G0 + G1)/2, zc = (z0 + z1)/2, Gbar = exp(-Gc dt), zbar = Gc^{-1}(I - Gbar) zc
 * computed as dt * phi1(-Gc dt) zc. */
void oracle_ode_discretise(int n, const double* G0, const double* z0, const double* G1, const double* z1,
                           double dt, double* Gbar, double* zbar) {
    size_t nn = (size_t)n * n;
    double* M = malloc((2 * nn + n) * sizeof(double));
    double *Ph = M + nn, *zc = Ph + nn;
    for (size_t k = 0; k < nn; k++) M[k] = -0.5 * (G0[k] + G1[k]) * dt;
    for (int r = 0; r < n; r++) zc[r] = 0.5 * (z0[r] + z1[r]);
    oracle_expm_phi1(n, M, Gbar, Ph);
    for (int r = 0; r < n; r++) {
        double s = 0.0;
        for (int k = 0; k < n; k++) s += Ph[r * n + k] * zc[k];
        zbar[r] = dt * s;
    }
    free(M);
}

/* -------------------------------------------------------- DEER for an ODE -- */

/* dy/dt = f(y) on the uniform grid t_j = t0 + j dt, dt = (t1 - t0)/(T - 1), j = 0..T-1
 * (Sec. 3.3).  Each iteration: G_j = -df/dy(y_j), z_j = f(y_j) + G_j y_j at every grid
 * point of the previous iterate; then y_{i+1} = Gbar_i y_i + zbar_i from y_0 = y0.
 * y: [B,T,n] with y[:,0] = y0.  guess may be NULL (zeros); its first point is replaced by y0. */
int oracle_ode_deer_eval(const oracle_cell* c, const double* th, long B, long T, double t0, double t1,
                         const double* y0, const double* guess, double tol, int max_iter,
                         double* y, double* final_err, double* err_hist, int nthreads) {
    int n = c->n;
    size_t nn = (size_t)n * n;
    size_t total = (size_t)B * T * n;
    double dt = (t1 - t0) / (double)(T - 1);
    double* ynew = malloc(total * sizeof(double));
    if (guess) memcpy(y, guess, total * sizeof(double));
    else memset(y, 0, total * sizeof(double));
    for (long b = 0; b < B; b++) memcpy(y + b * T * n, y0 + b * n, (size_t)n * sizeof(double));
    if (nthreads < 1) nthreads = 1;
    double err = 1e10;
    int iter = 0;
    while (err > tol && iter < max_iter) {
        double errmax = 0.0;
        int bad = 0;
#pragma omp parallel for num_threads(nthreads) schedule(static) reduction(max : errmax) reduction(| : bad)
        for (long b = 0; b < B; b++) {
            double* buf = malloc((3 * nn + 5 * n) * sizeof(double));
            double *Ga = buf, *Gb = Ga + nn, *Gbar = Gb + nn;
            double *za = Gbar + nn, *zb = za + n, *zbar = zb + n, *f = zbar + n;
            const double* yb = y + b * T * n;
            double* ynb = ynew + b * T * n;
            memcpy(ynb, y0 + b * n, (size_t)n * sizeof(double));
            /* G and z at grid point 0 */
            mlp_f(c, th, yb, f);
            mlp_jac(c, th, yb, Ga);
            for (size_t k = 0; k < nn; k++) Ga[k] = -Ga[k];
            for (int r = 0; r < n; r++) {
                double s = f[r];
                for (int k = 0; k < n; k++) s += Ga[r * n + k] * yb[k];
                za[r] = s;
            }
            for (long i = 0; i + 1 < T; i++) {
                const double* y1 = yb + (i + 1) * n;
                mlp_f(c, th, y1, f);
                mlp_jac(c, th, y1, Gb);
                for (size_t k = 0; k < nn; k++) Gb[k] = -Gb[k];
                for (int r = 0; r < n; r++) {
                    double s = f[r];
                    for (int k = 0; k < n; k++) s += Gb[r * n + k] * y1[k];
                    zb[r] = s;
                }
                oracle_ode_discretise(n, Ga, za, Gb, zb, dt, Gbar, zbar);
                for (int r = 0; r < n; r++) {
                    double s = zbar[r];
                    for (int k = 0; k < n; k++) s += Gbar[r * n + k] * ynb[i * n + k];
                    ynb[(i + 1) * n + r] = s;
                    double dlt = fabs(s - yb[(i + 1) * n + r]);
                    if (dlt > errmax) errmax = dlt;
                    if (!(dlt == dlt) || isinf(dlt)) bad = 1;
                }
                memcpy(Ga, Gb, nn * sizeof(double));
                memcpy(za, zb, (size_t)n * sizeof(double));
            }
            free(buf);
        }
        err = bad ? NAN : errmax;
        memcpy(y, ynew, total * sizeof(double));
        if (err_hist) err_hist[iter] = err;
        iter++;
    }
    if (final_err) *final_err = err;
    free(ynew);
    return iter;
}

/* ------------------------------------- backward derivative for the ODE form -- */

/* Vector-Jacobian product of the MLP field at one point: dth += (df/dtheta)^T w,
 * dy = (df/dy)^T w.  Reverse-mode sweep through the layers of mlp_forward. */
static void mlp_vjp(const oracle_cell* c, const double* th, const double* y, const double* w,
                    double* dth, double* dy) {
    int n = c->n, wd = c->width, L = c->nhid;
    int big = (wd > n ? wd : n);
    double* act = malloc((size_t)(L * wd + 1) * sizeof(double));
    double* out = malloc((size_t)n * sizeof(double));
    double* up = malloc((size_t)big * sizeof(double));     /* dL/d(output of the current layer) */
    double* down = malloc((size_t)big * sizeof(double));   /* dL/d(input of the current layer) */
    double* dac = malloc((size_t)(L * wd + 1) * sizeof(double));
    mlp_forward_d(c, th, y, act, dac, out);
    /* offsets of the layers inside theta */
    size_t* off = malloc((size_t)(L + 1) * sizeof(size_t));
    size_t o = 0;
    int nin = n;
    for (int l = 0; l < L; l++) { off[l] = o; o += (size_t)wd * nin + wd; nin = wd; }
    off[L] = o;
    /* output layer: f = W_out in + b_out */
    {
        const double* in = (L > 0 ? act + (L - 1) * wd : y);
        const double* Wo = th + off[L];
        double* dWo = dth + off[L];
        double* dbo = dWo + (size_t)n * nin;
        for (int i = 0; i < n; i++) {
            for (int j = 0; j < nin; j++) dWo[i * nin + j] += w[i] * in[j];
            dbo[i] += w[i];
        }
        for (int j = 0; j < nin; j++) {
            double sacc = 0.0;
            for (int i = 0; i < n; i++) sacc += Wo[i * nin + j] * w[i];
            up[j] = sacc;
        }
    }
    /* hidden layers, last to first: act_l = s(W_l in + b_l) */
    for (int l = L - 1; l >= 0; l--) {
        int lin = (l == 0 ? n : wd);
        const double* in = (l == 0 ? y : act + (l - 1) * wd);
        const double* Wl = th + off[l];
        double* dWl = dth + off[l];
        double* dbl = dWl + (size_t)wd * lin;
        for (int j = 0; j < lin; j++) down[j] = 0.0;
        for (int i = 0; i < wd; i++) {
            double dpre = up[i] * dac[l * wd + i];
            for (int j = 0; j < lin; j++) {
                dWl[i * lin + j] += dpre * in[j];
                down[j] += Wl[i * lin + j] * dpre;
            }
            dbl[i] += dpre;
        }
        memcpy(up, down, (size_t)lin * sizeof(double));
    }
    memcpy(dy, up, (size_t)n * sizeof(double));
    free(act); free(out); free(up); free(down); free(off); free(dac);
}

void oracle_mlp_vjp(const oracle_cell* c, const double* th, const double* y, const double* w,
                    double* dth, double* dy) {
    mlp_vjp(c, th, y, w, dth, dy);
}

/* Backward derivative of a loss L(y_0..y_{T-1}) for dy/dt = f(y, theta) on the grid of
 * oracle_ode_deer_eval (Sec. 3.1.1 eq. 7 applied to the discretised operator of Sec. 3.3 eq. 8-9).
 * With G frozen at the trajectory, a perturbation of theta moves the right-hand side by
 * df_j = (df/dtheta)(y_j) dtheta and the trajectory by
 *     dy_{j+1} = Gbar_j dy_j + P_j (df_j + df_{j+1})/2,   P_j = dt phi1(-Gc_j dt),  dy_0 = dy0,
 * so with g_j = dL/dy_j
 *     lam_{T-1} = g_{T-1},  lam_j = g_j + Gbar_j^T lam_{j+1}                  (dual operator)
 *     w_j = ( P_j^T lam_{j+1} [j < T-1]  +  P_{j-1}^T lam_j [j > 0] ) / 2
 *     dL/dtheta = sum_j (df/dtheta)(y_j)^T w_j,    dL/dy0 = lam_0.
 * This is the derivative eq. 7 defines (the explicit dependence of f on theta pushed through
 * L_G^{-1}); it differs from the derivative of the discrete solution by O(dt^2), because the latter
 * also sees Gbar change with theta.  y: [B,T,n] trajectory, g: [B,T,n]; dth is overwritten. */
void oracle_ode_grad(const oracle_cell* c, const double* th, long B, long T, double t0, double t1,
                     const double* y, const double* g, double* dth, double* dy0) {
    int n = c->n;
    size_t nn = (size_t)n * n;
    double dt = (t1 - t0) / (double)(T - 1);
    long nth = oracle_theta_count(c);
    for (long k = 0; k < nth; k++) dth[k] = 0.0;
    double* G = malloc((size_t)T * nn * sizeof(double));
    double* Gbar = malloc((size_t)(T - 1) * nn * sizeof(double));
    double* P = malloc((size_t)(T - 1) * nn * sizeof(double));
    double* lam = malloc((size_t)T * n * sizeof(double));
    double* M = malloc(nn * sizeof(double));
    double* w = malloc((size_t)n * sizeof(double));
    double* dyj = malloc((size_t)n * sizeof(double));
    for (long b = 0; b < B; b++) {
        const double* yb = y + b * T * n;
        const double* gb = g + b * T * n;
        for (long j = 0; j < T; j++) {
            mlp_jac(c, th, yb + j * n, G + j * nn);
            for (size_t k = 0; k < nn; k++) G[j * nn + k] = -G[j * nn + k];
        }
        for (long j = 0; j + 1 < T; j++) {
            for (size_t k = 0; k < nn; k++) M[k] = -0.5 * (G[j * nn + k] + G[(j + 1) * nn + k]) * dt;
            oracle_expm_phi1(n, M, Gbar + j * nn, P + j * nn);
            for (size_t k = 0; k < nn; k++) P[j * nn + k] *= dt;
        }
        memcpy(lam + (T - 1) * n, gb + (T - 1) * n, (size_t)n * sizeof(double));
        for (long j = T - 2; j >= 0; j--)
            for (int r = 0; r < n; r++) {
                double sacc = gb[j * n + r];
                for (int k = 0; k < n; k++) sacc += Gbar[j * nn + k * n + r] * lam[(j + 1) * n + k];
                lam[j * n + r] = sacc;
            }
        for (long j = 0; j < T; j++) {
            for (int r = 0; r < n; r++) {
                double sacc = 0.0;
                if (j + 1 < T)
                    for (int k = 0; k < n; k++) sacc += P[j * nn + k * n + r] * lam[(j + 1) * n + k];
                if (j > 0)
                    for (int k = 0; k < n; k++) sacc += P[(j - 1) * nn + k * n + r] * lam[j * n + k];
                w[r] = 0.5 * sacc;
            }
            mlp_vjp(c, th, yb + j * n, w, dth, dyj);
        }
        memcpy(dy0 + b * n, lam, (size_t)n * sizeof(double));
    }
    free(G); free(Gbar); free(P); free(lam); free(M); free(w); free(dyj);
}

int oracle_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
