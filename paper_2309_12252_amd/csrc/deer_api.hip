// Host driver and C ABI of the DEER library (see include/deer.h for the contract).
// The driver owns no device memory: it carves the caller's workspace into the Jacobian stream,
// the right-hand side, a second trajectory buffer, scan tile descriptors and a few counters.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/deer.h"
#include "deer_common.h"

using namespace deer;

namespace {

constexpr int kSlots = 256;          // ticket / error slots, one per scan launch between refills
constexpr size_t kAlign = 256;
constexpr int kMaxEvents = 24;      // timed launches between two host synchronisations

thread_local std::string g_last_error;

// Scratch of deer_linrec_solve_static(): the words the scan's tiles publish for each other, the tile dispenser
// and the status word live in this array instead of a caller-provided workspace.  Every GPU the library runs
// on holds its own copy, at its own address, until the process ends.  In host code the array's name is only
// a handle for hipGetSymbolAddress(); kernels and fills get the per-device address kept in g_static_ptr.
constexpr size_t kStaticBytes = (size_t)64 << 20;
constexpr int kMaxDevices = 64;
__device__ __align__(256) unsigned char deer_static_scratch[kStaticBytes];
std::mutex g_static_mutex;
void* g_static_ptr[kMaxDevices] = {};
#ifdef DEER_SCAN_TIMING
// development builds only (-DDEER_SCAN_TIMING): the kernels stamp the phases of every tile into a region at the
// end of the caller's workspace (deer_workspace_bytes() grows by kTimingBytes); deer_debug_timing(ctx) returns it
constexpr size_t kTimingBytes = (size_t)1 << 26;
#endif

size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Plan {
    size_t esz;          // bytes per scalar
    int scan_T;          // scan positions per sequence
    int tile;            // scan positions per tile
    int tiles;           // tiles per sequence
    int L;               // positions per lane group (VALU scan)
    int W;               // wavefronts per tile (VALU scan)
    bool mfma;
    bool fused;          // GRU with n <= 8: Newton steps run the scan with the cell evaluated in place
    int fused_L, fused_W, fused_tiles;
    bool mh;             // multi-head GRU with strides: the scan's sequences are the heads' strided recurrences
    int mh_H, mh_K;      // heads, stride levels
    size_t off_dy0parts, off_mhtable;
    bool grad_fused;     // deer_grad computes the transposed Jacobians inside the reverse scan
    bool need_J;         // some kernel of this plan reads or writes the Jacobian stream [B,T,n,n] and the right-hand side
    int vjp_blocks;
    // byte offsets into the workspace
    size_t off_J, off_rhs, off_ybuf, off_Gbar, off_zbar, off_aggW, off_inclW, off_barrier, off_ctl, off_partial, off_timing, total;
};

// cells whose state is two halves of n units each (n of the configuration = units): LSTM (h | c), LEM (y | z)
bool two_part_cell(int cell) { return cell == DEER_CELL_LSTM || cell == DEER_CELL_LEM; }

size_t theta_count(const deer_config* c) {
    const size_t n = (size_t)c->n;
    if (c->cell == DEER_CELL_GRU) return (size_t)(c->heads > 1 ? c->heads : 1) * (3 * n * (size_t)c->d + 3 * n * n + 4 * n);
    if (two_part_cell(c->cell)) {
        const size_t u = c->reserved > 0 ? (size_t)c->reserved : n;   // (the configuration the kernels run keeps the units there)
        return 4 * u * (size_t)c->d + 4 * u * u + 4 * u;
    }
    const size_t w = (size_t)c->mlp_width;
    const size_t L = c->mlp_hidden_layers >= 1 ? (size_t)c->mlp_hidden_layers : 1;
    return (w * n + w) + (L - 1) * (w * w + w) + (n * w + n);
}

// the two-hidden-layer tanh field has kernels of its own (on the matrix cores for fp32, n = 8); every other depth
// and the softplus activation run the general kernels
bool mlp_fast_path(const deer_config* c) {
    const int w = c->mlp_width;
    return c->mlp_hidden_layers == 2 && c->mlp_activation == DEER_ACT_TANH && (w == 16 || w == 32 || w == 64) && w % c->n == 0;
}

int env_int(const char* name, int dflt) {
    const char* s = std::getenv(name);
    if (!s || !*s) return dflt;
    return std::atoi(s);
}

bool validate(const deer_config* c, std::string& why) {
    if (!c) { why = "config is NULL"; return false; }
    if (c->cell != DEER_CELL_GRU && c->cell != DEER_CELL_MLP_ODE && !two_part_cell(c->cell)) { why = "unknown cell"; return false; }
    if (c->dtype != DEER_F32 && c->dtype != DEER_F64) { why = "unknown dtype"; return false; }
    if (c->B < 1 || c->T < 1 || c->n < 1) { why = "B, T and n must be positive"; return false; }
    if ((long long)c->B * c->T > (1LL << 31) - 1) { why = "B*T must fit 31 bits"; return false; }
    if (c->heads < 0 || c->stride_levels < 0 || c->reserved != 0) { why = "heads and stride_levels must be >= 0 and reserved 0"; return false; }
    if (c->cell != DEER_CELL_GRU && (c->heads > 1 || c->stride_levels > 1)) { why = "heads and strides exist for the GRU only"; return false; }
    return true;
}

// smallest state size with kernels of its own that holds n channels (0: none)
int native_n(int n) {
    for (int v = 1; v <= 64; v <<= 1)
        if (n <= v) return v;
    return 0;
}

bool is_multihead(const deer_config* c);

// The configuration the kernels run: a plain GRU whose state size has no kernels of its own is embedded in the next
// size that has (zero rows and columns in every weight: the extra channels stay at zero and the real ones never see
// them, so iterates, iteration counts and gradients are those of the original cell).
deer_config internal_config(const deer_config* user) {
    deer_config c = *user;
    if (c.cell == DEER_CELL_GRU && !is_multihead(user) && native_n(c.n) > 0) c.n = native_n(c.n);
    if (two_part_cell(c.cell)) {   // state (h | c) or (y | z) of 2 units entries in the next state size with a scan kernel
        c.reserved = user->n;
        c.n = native_n(2 * user->n);
    }
    return c;
}

bool is_multihead(const deer_config* c) { return c->cell == DEER_CELL_GRU && (c->heads > 1 || c->stride_levels > 1); }

bool supported(const deer_config* c, std::string& why) {
    const int n = c->n;
    if (is_multihead(c)) {
        const int H = c->heads > 1 ? c->heads : 1, K = c->stride_levels > 1 ? c->stride_levels : 1;
        if (!(n == 2 || n == 4 || n == 8) || c->d < 1 || c->d > 8) { why = "multi-head GRU: state size per head must be 2, 4 or 8 and input size per head 1..8"; return false; }
        if (H > 64 || K > 8) { why = "multi-head GRU: at most 64 heads and 8 stride levels"; return false; }
        if ((long long)c->B * c->T * H > (1LL << 31) - 1) { why = "B*T*heads must fit 31 bits"; return false; }
        if (c->T > (1 << 22)) { why = "multi-head GRU: at most 4,194,304 steps (17 bits of tile index per recurrence)"; return false; }
        if (env_int("DEER_FUSED", 1) == 0 || env_int("DEER_GRAD_FUSED", 1) == 0) { why = "multi-head GRU runs only with the cell inside the scans"; return false; }
        return true;
    }
    if (two_part_cell(c->cell)) {
        if (!lstm_supported(n, c->d)) { why = "LSTM and LEM: 1..16 units and input size 1..8"; return false; }
        if (c->cell == DEER_CELL_LEM && !(c->t1 > 0.0)) { why = "LEM: t1 holds the cell's step and must be positive"; return false; }
        return true;
    }
    if (c->cell == DEER_CELL_GRU) {
        // 1, 2, 4, 8, 16, 32 and (fp32) 64 have kernels; the sizes in between run embedded in the next one of those
        if (n > 64) { why = "GRU state size must be at most 64"; return false; }
        if (n > 32 && c->dtype != DEER_F32) { why = "GRU state sizes above 32 run in fp32 only"; return false; }
        if (c->d < 1 || c->d > 32) { why = "GRU input size must be 1..32"; return false; }
    } else {
        if (!(n == 2 || n == 4 || n == 8)) { why = "MLP_ODE state size must be 2, 4 or 8"; return false; }
        if (c->mlp_activation != DEER_ACT_TANH && c->mlp_activation != DEER_ACT_SOFTPLUS) { why = "unknown MLP activation"; return false; }
        if (c->mlp_hidden_layers < 1 || c->mlp_hidden_layers > 5) { why = "MLP_ODE needs 1 to 5 hidden layers"; return false; }
        const int w = c->mlp_width;
        if (w < 4 || w > 64 || (w & 3) != 0) { why = "MLP_ODE hidden width must be a multiple of 4 between 4 and 64"; return false; }
        if (!mlp_fast_path(c) && !mlp_general_supported(n, w, c->mlp_hidden_layers, c->mlp_activation)) {
            why = "MLP_ODE: no kernel for this width, depth and activation";
            return false;
        }
        if (c->T < 2) { why = "MLP_ODE needs at least 2 grid points"; return false; }
        if (!(c->t1 > c->t0)) { why = "MLP_ODE needs t1 > t0"; return false; }
    }
    return true;
}

// Multi-head GRU: the tiles of one batch entry, head by head, recurrence by recurrence (first time index r < stride),
// tile by tile: head << 26 | r << 19 | pack << 17 | tile.  The kernels read this list instead of decoding a ticket.
// Recurrences of at most half a tile share one: 2^pack of them (first time indices r .. r + 2^pack - 1), each on
// an eighth, a quarter or half of the tile's eight wavefronts.
std::vector<unsigned> mh_table(const deer_config* c, int tile) {
    const int H = c->heads > 1 ? c->heads : 1, K = c->stride_levels > 1 ? c->stride_levels : 1;
    std::vector<unsigned> v;
    for (int h = 0; h < H; ++h) {
        const long long s = 1LL << (h % K);
        const long long nrec = s < (long long)c->T ? s : (long long)c->T;   // recurrences that have a position
        const long long len0 = ((long long)c->T + s - 1) / s;              // the longest of them (r = 0)
        int pack = 0;
        while (pack < 3 && len0 * (2LL << pack) <= tile && (2LL << pack) <= nrec) ++pack;
        long long r = 0;
        for (; pack > 0 && r + (1LL << pack) <= nrec; r += 1LL << pack)
            v.push_back((unsigned)h << 26 | (unsigned)r << 19 | (unsigned)pack << 17);
        for (; r < nrec; ++r) {
            const long long len = ((long long)c->T - r + s - 1) / s;
            for (long long t = 0; t * tile < len; ++t) v.push_back((unsigned)h << 26 | (unsigned)r << 19 | (unsigned)t);
        }
    }
    return v;
}

Plan make_plan(const deer_config* c) {
    Plan p{};
    p.esz = c->dtype == DEER_F32 ? 4 : 8;
    const size_t n = (size_t)c->n, B = (size_t)c->B, T = (size_t)c->T;
    const bool ode = c->cell == DEER_CELL_MLP_ODE;
    p.scan_T = ode ? c->T - 1 : c->T;
    p.mh = is_multihead(c);
    if (p.mh) {
        // every head's strided recurrences are sequences of the fused small-n kernel (eight wavefronts per tile);
        // positions per lane group from the same kind of estimate as below, over the real tiles of all recurrences
        const int H = c->heads > 1 ? c->heads : 1, K = c->stride_levels > 1 ? c->stride_levels : 1;
        p.mh_H = H; p.mh_K = K;
        p.mfma = false; p.W = 8; p.L = 1; p.fused = true; p.fused_W = 8;
        static const int kLm[] = {1, 2, 4};
        double best = 1e300;
        int forced = env_int("DEER_FUSED_L", 0);
        for (int q = 0; q < 3; ++q) {
            const long long tiles = (long long)B * (long long)mh_table(c, scan_valu_tile(c->n, kLm[q], 8)).size();
            double est = (double)((tiles + 255) / 256) * (5.0 + 1.6 * kLm[q]);
            if (forced == kLm[q]) est = -1.0;
            if (est < best) { best = est; p.fused_L = kLm[q]; }
        }
        const int tile = scan_valu_tile(c->n, p.fused_L, 8);
        p.fused_tiles = (int)mh_table(c, tile).size();   // tiles of one batch entry over all its recurrences
        p.tile = tile; p.tiles = p.fused_tiles;
        p.grad_fused = true; p.need_J = false;
        long long vb = ((long long)B * (long long)T + 31) / 32;
        p.vjp_blocks = (int)(vb > 128 ? 128 : (vb < 1 ? 1 : vb));
        size_t off = 0;
        auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
        p.off_J = take(0); p.off_rhs = take(0);
        p.off_ybuf = take(B * T * (size_t)H * n * p.esz);
        p.off_Gbar = take(0); p.off_zbar = take(0);
        const size_t nt = B * (size_t)p.fused_tiles;
        p.off_mhtable = take((size_t)p.fused_tiles * 4);
        p.off_aggW = take(nt * (n * n + n) * (p.esz / 4) * 8);
        p.off_inclW = take(nt * n * (p.esz / 4) * 8);
        p.off_barrier = take(0);
        p.off_ctl = take((size_t)kSlots * 4 + (size_t)kSlots * 8 + 16);
        p.off_partial = take((size_t)H * p.vjp_blocks * 4 * (theta_count(c) / H) * p.esz);
        p.off_dy0parts = take(B * (size_t)H * ((size_t)1 << (K - 1)) * n * p.esz);
#ifdef DEER_SCAN_TIMING
        p.off_timing = take(kTimingBytes);
#endif
        p.total = off;
        return p;
    }
    p.mfma = c->n >= 16;
    if (p.mfma) {
        p.L = 0;
        p.tile = scan_mfma_tile(c->dtype, c->n);
    } else {
        // Positions per group of lanes.  Measured on MI355X: a tile lives for about (5 + 1.05 L)
        // microseconds and the chip holds one tile per compute unit, so a launch takes
        // ceil(tiles / 256) such rounds; longer serial runs amortise the per-tile look-back, and the
        // longest one wins as soon as it still leaves a tile for half of the compute units.
        // (fp64 keeps L <= 4 for n = 8 and <= 8 otherwise: registers.)
        const int W = 8;
        p.W = W;
        static const int kL32[] = {1, 2, 4, 8, 10, 12, 16};
        static const int kL64[] = {1, 2, 4, 8};
        const int* cand = c->dtype == DEER_F32 ? kL32 : kL64;
        int ncand = c->dtype == DEER_F32 ? 7 : ((c->n == 8) ? 3 : 4);
        int L = cand[0];
        double best = 1e300;
        for (int q = 0; q < ncand; ++q) {
            const long long tile = scan_valu_tile(c->n, cand[q], W);
            const long long tiles = (long long)B * ((p.scan_T + tile - 1) / tile);
            double est = (double)((tiles + 255) / 256) * (5.0 + 1.05 * cand[q]);
            if (q == ncand - 1 && tiles >= 128) est = 0.0;
            if (est < best) { best = est; L = cand[q]; }
        }
        const int forced = env_int("DEER_SCAN_L", 0);
        for (int q = 0; q < ncand; ++q)
            if (forced == cand[q]) L = forced;
        // n = 4 in fp32 has registers for 24 positions per group: measured 4 % faster than 16 on streams that
        // still give every compute unit a tile
        if (c->dtype == DEER_F32 && c->n == 4) {
            const long long tile24 = scan_valu_tile(4, 24, W);
            const bool fills = (long long)B * ((p.scan_T + tile24 - 1) / tile24) >= 256;
            if (forced == 24 || (forced == 0 && L == 16 && fills)) L = 24;
        }
        // n = 2 in fp32: 32 positions per group (three registers each) once the launch still gives every
        // compute unit a tile; the fixed per-tile latencies are most of a tile's life at this size
        if (c->dtype == DEER_F32 && c->n == 2) {
            const long long tile32 = scan_valu_tile(2, 32, W);
            const bool fills = (long long)B * ((p.scan_T + tile32 - 1) / tile32) >= 256;
            if (forced == 32 || (forced == 0 && L == 16 && fills)) L = 32;
        }
        p.L = L;
        p.tile = scan_valu_tile(c->n, p.L, p.W);
    }
    p.tiles = (p.scan_T + p.tile - 1) / p.tile;
    if (p.tiles < 1) p.tiles = 1;
    p.fused = false;
    p.fused_tiles = 0;
    const bool gru = c->cell == DEER_CELL_GRU;
    if (gru && !p.mfma && c->d <= 8 && env_int("DEER_FUSED", 1) != 0) {
        // The fused step spends more time per position on arithmetic and none on loading matrices:
        // shorter serial runs than the plain scan, so that more tiles are in flight.
        static const int kLf[] = {1, 2, 4, 8, 10, 12, 16};
        const int ncand = c->dtype == DEER_F32 ? 7 : ((c->n == 8) ? 3 : 4);
        int L = kLf[0];
        double best = 1e300;
        for (int q = 0; q < ncand; ++q) {
            if (!scan_gru_fused_supported(c->dtype, c->n, c->d, kLf[q], 8)) continue;
            const long long tile = scan_valu_tile(c->n, kLf[q], p.W);
            const long long tiles = (long long)B * ((p.scan_T + tile - 1) / tile);
            // per tile: a fixed part, the serial run (cheaper for small n), and the look-back along the
            // sequence when it has more than one tile
            const double per_pos = c->n == 8 ? 1.6 : (c->n == 4 ? 0.8 : 0.5);
            const double est = (double)((tiles + 255) / 256) * (5.0 + per_pos * kLf[q]) + (tiles > (long long)B ? 4.0 : 0.0);
            if (est < best) { best = est; L = kLf[q]; }
        }
        // tuning knobs: honoured when the requested variant exists
        p.fused_W = 8;
        const int fl = env_int("DEER_FUSED_L", 0), fw = env_int("DEER_FUSED_W", 0);
        if (fw > 0 && scan_gru_fused_supported(c->dtype, c->n, c->d, L, fw)) p.fused_W = fw;
        if (fl > 0 && scan_gru_fused_supported(c->dtype, c->n, c->d, fl, p.fused_W)) L = fl;
        if (scan_gru_fused_supported(c->dtype, c->n, c->d, L, p.fused_W)) {
            p.fused = true;
            p.fused_L = L;
            const int tile = scan_valu_tile(c->n, L, p.fused_W);
            p.fused_tiles = (p.scan_T + tile - 1) / tile;
            if (p.fused_tiles < 1) p.fused_tiles = 1;
        }
    }
    if (gru && p.mfma && env_int("DEER_FUSED", 1) != 0 && scan_mfma_fused_supported(c->dtype, c->n, c->d)) {
        p.fused = true;   // the MFMA scan with the cell inside (its own tile shape)
        p.fused_L = 0;
        p.fused_W = 0;
        const int ft = scan_mfma_fused_tile(c->n);
        p.fused_tiles = (p.scan_T + ft - 1) / ft;
        if (p.fused_tiles < 1) p.fused_tiles = 1;
    }
    p.vjp_blocks = c->cell == DEER_CELL_GRU    ? gru_vjp_blocks(c->n, (long long)B * T)
                   : two_part_cell(c->cell) ? lstm_vjp_blocks(c->reserved, (long long)B * T)
                   : mlp_fast_path(c)       ? mlp_vjp_blocks(c->dtype, c->n, c->mlp_width, (long long)B * T)
                                            : mlp_general_vjp_blocks(c->dtype, c->n, c->mlp_width, c->mlp_hidden_layers, (long long)B * T);

    p.grad_fused = p.fused && env_int("DEER_GRAD_FUSED", 1) != 0 &&
                   (p.mfma || scan_gru_dual_supported(c->dtype, c->n, c->d, p.fused_L, p.fused_W));
    // The Jacobians exist in memory only where a kernel pair exchanges them: the ODE form, and the GRU sizes (or
    // knob settings) whose forward or backward pass runs the cell kernel followed by the plain scan.  With the
    // cell inside both scans the workspace is O(n T) instead of the O(n^2 T) of Sec. 3.5.
    p.need_J = ode || !p.fused || !p.grad_fused;

    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
    p.off_J = take(p.need_J ? B * T * n * n * p.esz : 0);
    p.off_rhs = take(p.need_J ? B * T * n * p.esz : 0);
    p.off_ybuf = take(B * T * n * p.esz);
    p.off_Gbar = take(ode ? B * (T - 1) * n * n * p.esz : 0);
    p.off_zbar = take(ode ? B * (T - 1) * n * p.esz : 0);
    const size_t nt = B * (size_t)(p.tiles > p.fused_tiles ? p.tiles : p.fused_tiles);
    // published tile totals and carries: one 64-bit tagged word per 32 bits of payload
    p.off_aggW = take(nt * (n * n + n) * (p.esz / 4) * 8);
    p.off_inclW = take(nt * n * (p.esz / 4) * 8);
    // slots of the one-launch solve's grid barrier (two banks, one tagged scalar per workgroup)
    p.off_barrier = take(p.fused ? 2 * (B * (size_t)p.fused_tiles + 4) * (p.esz / 4) * 8 : 0);   // (+4: test hook)
    p.off_ctl = take((size_t)kSlots * 4 + (size_t)kSlots * 8 + 16);   // tickets, err bits, status
    // partial rows of dL/dtheta: four per block (one per wavefront), two per block in the vector-ALU MLP kernel (one per thread group)
    p.off_partial = take((size_t)p.vjp_blocks * 4 * theta_count(c) * p.esz);
#ifdef DEER_SCAN_TIMING
    p.off_timing = take(kTimingBytes);
#endif
    p.total = off;
    return p;
}

}  // namespace

// Regions behind the kernels' own workspace that hold the embedded copies of a padded configuration
struct PadPlan {
    bool on;
    size_t off_theta, off_y0, off_y, off_g, off_dtheta, off_dy0, total;
};

static PadPlan make_pad_plan(const deer_config* user, const deer_config* in, size_t base) {
    PadPlan q{};
    const int user_state = two_part_cell(user->cell) ? 2 * user->n : user->n;
    q.on = in->n != user_state;
    q.total = base;
    if (!q.on) return q;
    const size_t esz = in->dtype == DEER_F32 ? 4 : 8;
    const size_t B = (size_t)in->B, T = (size_t)in->T, np = (size_t)in->n;
    size_t off = base;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
    const size_t P = theta_count(in);
    q.off_theta = take(P * esz);
    q.off_y0 = take(B * np * esz);
    q.off_y = take(B * T * np * esz);
    q.off_g = take(B * T * np * esz);
    q.off_dtheta = take(P * esz);
    q.off_dy0 = take(B * np * esz);
    q.total = off;
    return q;
}

struct deer_ctx {
    deer_config user;    // the configuration as the caller gave it
    PadPlan pad;
    deer_config cfg;
    Plan plan;
    hipStream_t stream;
    char* ws;
    unsigned epoch;
    void* h_err;            // pinned: kSlots * 8 bytes of error words, then the status word and a result word
    void* d_h_err;          // the same memory as the device sees it
    int batch;              // Newton iterations enqueued per host round trip when nothing better is known
    int last_iters;         // iterations the previous deer_eval() took (0: none yet)
    bool one_launch;        // GRU, n <= 8, every tile resident at once: all iterations run in one launch
    unsigned test_spin_limit, test_extra_workgroups;   // test hooks of the one-launch solve's grid barrier
    bool profiling;
    deer_profile prof;
    hipEvent_t ev[2 * kMaxEvents];
    int ev_kind[kMaxEvents];
    int ev_iter[kMaxEvents];   // Newton iteration the launch belongs to (-1: always counted)
    int ev_used;
    std::string last_error;
};

namespace {

enum { KIND_FUNCEVAL = 0, KIND_DISC = 1, KIND_SCAN = 2, KIND_VJP = 3, KIND_FUSED = 4, KIND_NEWTON = 5 };

deer_status fail(deer_ctx* ctx, deer_status st, const std::string& msg) {
    if (ctx) ctx->last_error = msg;
    g_last_error = msg;
    return st;
}

#define HIPCHK(ctx, expr)                                                                       \
    do {                                                                                        \
        hipError_t e_ = (expr);                                                                 \
        if (e_ != hipSuccess)                                                                   \
            return fail(ctx, DEER_ERR_HIP, std::string(#expr) + ": " + hipGetErrorString(e_));  \
    } while (0)

unsigned* ctl_ticket(deer_ctx* c, int slot) { return reinterpret_cast<unsigned*>(c->ws + c->plan.off_ctl) + slot; }
void* ctl_err(deer_ctx* c, int slot) { return c->ws + c->plan.off_ctl + (size_t)kSlots * 4 + (size_t)slot * 8; }
unsigned* ctl_status(deer_ctx* c) {
    return reinterpret_cast<unsigned*>(c->ws + c->plan.off_ctl + (size_t)kSlots * 4 + (size_t)kSlots * 8);
}
size_t ctl_bytes() { return align_up((size_t)kSlots * 4 + (size_t)kSlots * 8 + 16); }

void prof_begin(deer_ctx* c, int kind, int iter = -1) {
    if (!c->profiling || c->ev_used >= kMaxEvents) return;
    c->ev_kind[c->ev_used] = kind;
    c->ev_iter[c->ev_used] = iter;
    (void)hipEventRecord(c->ev[2 * c->ev_used], c->stream);
}
void prof_end(deer_ctx* c) {
    if (!c->profiling || c->ev_used >= kMaxEvents) return;
    (void)hipEventRecord(c->ev[2 * c->ev_used + 1], c->stream);
    c->ev_used++;
}
// Call after the stream has been synchronised.  Launches of Newton iterations >= iters_done were
// enqueued ahead of the convergence test and returned at once: they are not counted.
void prof_collect(deer_ctx* c, int iters_done = 1 << 30) {
    for (int i = 0; i < c->ev_used; ++i) {
        if (c->ev_iter[i] >= iters_done) continue;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, c->ev[2 * i], c->ev[2 * i + 1]) != hipSuccess) continue;
        switch (c->ev_kind[i]) {
            case KIND_FUNCEVAL: c->prof.funceval_ms += ms; c->prof.funceval_launches++; break;
            case KIND_DISC: c->prof.discretise_ms += ms; c->prof.discretise_launches++; break;
            case KIND_SCAN: c->prof.scan_ms += ms; c->prof.scan_launches++; break;
            case KIND_FUSED: c->prof.fused_ms += ms; c->prof.fused_launches++; break;
            case KIND_NEWTON: c->prof.newton_ms += ms; c->prof.newton_launches++; break;
            default: c->prof.vjp_ms += ms; c->prof.vjp_launches++; break;
        }
    }
    c->ev_used = 0;
}

// One scan launch over the context's shapes.
hipError_t run_scan(deer_ctx* c, const void* A, const void* bv, const void* y0, void* out, const void* yold,
                    long long strideA, long long strideb, long long strideOut, int reverse, int slot, bool want_err,
                    int delta = 0, Gate gate = Gate{nullptr, 0.0}, int iter = -1, const void* fused_theta = nullptr,
                    const void* fused_x = nullptr, int add_identity = 0) {
    const deer_config& g = c->cfg;
    ScanParams p{};
    p.A = A; p.bv = bv; p.y0 = y0; p.out = out; p.yold = yold;
    p.strideA = strideA; p.strideb = strideb; p.strideOut = strideOut; p.strideOld = strideOut;
    p.B = g.B; p.T = c->plan.scan_T; p.L = c->plan.L; p.tiles = c->plan.tiles; p.reverse = reverse; p.delta = delta; p.add_identity = add_identity;
    p.epoch = ++c->epoch;   // reserve_epochs() keeps this below 2^30
    p.aggW = reinterpret_cast<unsigned long long*>(c->ws + c->plan.off_aggW);
    p.inclW = reinterpret_cast<unsigned long long*>(c->ws + c->plan.off_inclW);
    p.W = c->plan.W;
    p.ticket = ctl_ticket(c, slot);
    p.err = want_err ? ctl_err(c, slot) : nullptr;
    p.status = ctl_status(c);
    p.gate = gate;
#ifdef DEER_SCAN_TIMING
    // eight segments of 2^20 words, one per launch in turn, so consecutive launches can be compared
    p.timing = reinterpret_cast<unsigned long long*>(c->ws + c->plan.off_timing) + (size_t)(p.epoch & 7u) * ((size_t)1 << 20);
#endif
    hipError_t e;
    if (fused_theta && c->plan.mh) {
        p.L = c->plan.fused_L;
        p.W = 8;
        p.tiles = c->plan.fused_tiles;
        p.mh_H = c->plan.mh_H; p.mh_K = c->plan.mh_K;
        p.mh_table = reinterpret_cast<const unsigned*>(c->ws + c->plan.off_mhtable);
        p.mh_P = (long long)(theta_count(&g) / (size_t)c->plan.mh_H);
        prof_begin(c, KIND_FUSED, iter);
        e = launch_scan_gru_mh(g.dtype, g.n, p, fused_theta, fused_x, g.d, c->stream);
    } else if (fused_theta && c->plan.mfma) {
        p.tiles = reverse ? c->plan.tiles : c->plan.fused_tiles;   // the dual scan keeps the plain scan's tile shape
        prof_begin(c, KIND_FUSED, iter);
        e = launch_scan_mfma_fused(g.n, p, fused_theta, fused_x, g.d, c->stream);
    } else if (fused_theta) {
        p.L = c->plan.fused_L;
        p.W = c->plan.fused_W;
        p.tiles = c->plan.fused_tiles;
        prof_begin(c, KIND_FUSED, iter);
        e = reverse ? launch_scan_gru_dual(g.dtype, g.n, p, fused_theta, fused_x, g.d, c->stream)
                    : launch_scan_gru_fused(g.dtype, g.n, p, fused_theta, fused_x, g.d, c->stream);
    } else {
        prof_begin(c, KIND_SCAN, iter);
        e = c->plan.mfma ? launch_scan_mfma(g.dtype, g.n, p, c->stream) : launch_scan_valu(g.dtype, g.n, p, c->stream);
    }
    prof_end(c);
    return e;
}

// Tags carry a 30-bit launch epoch.  Before `count` more epochs are handed out: if they would not fit,
// start again from 1 and clear everything published so far (stale words must not carry a tag that will be
// used again).  Called at points where no launch of this context is using the published words any more
// in stream order: the clearing kernel is enqueued on the same stream.
deer_status reserve_epochs(deer_ctx* c, unsigned count) {
    if (c->epoch + count + 1u >= (1u << 30)) {
        HIPCHK(c, launch_fill_zero(c->ws + c->plan.off_aggW, c->plan.off_ctl - c->plan.off_aggW, c->stream));
        c->epoch = 0;
    }
    return DEER_OK;
}

// Clears tickets, error slots and the status word; at most kSlots launches follow before the next call.
deer_status zero_ctl(deer_ctx* c) {
    deer_status st = reserve_epochs(c, (unsigned)kSlots + 8u);
    if (st != DEER_OK) return st;
    HIPCHK(c, launch_fill_zero(c->ws + c->plan.off_ctl, ctl_bytes(), c->stream));
    return DEER_OK;
}

deer_status check_status(deer_ctx* c) {
    unsigned st = 0;
    HIPCHK(c, hipMemcpyAsync(c->h_err, ctl_status(c), 4, hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    std::memcpy(&st, c->h_err, 4);
    if (st != 0) return fail(c, DEER_ERR_HIP, "scan kernel: a tile waited too long for its predecessors");
    return DEER_OK;
}

// *busy is set when the one-launch solve gave up waiting (the device is shared with other work): the caller
// then takes the launch-per-iteration path
deer_status eval_one_launch(bool* busy, deer_ctx* c, const void* d_theta, const void* d_x, const void* d_y0, const void* d_y_guess,
                            double tol, int32_t max_iter, void* d_y, int32_t* iters, double* final_err,
                            int32_t* converged) {
    const deer_config& g = c->cfg;
    const size_t n = (size_t)g.n, T = (size_t)g.T;
    // No clearing launch in front: the kernel draws no tickets, writes every word the host reads, and the
    // status word is zero unless a previous solve failed (which re-zeroes it below).
    deer_status st = DEER_OK;
    NewtonParams q{};
    ScanParams& p = q.scan;
    p.y0 = d_y0; p.out = d_y; p.yold = d_y_guess;
    p.strideOut = (long long)(T * n); p.strideOld = (long long)(T * n);
    p.B = g.B; p.T = g.T; p.L = c->plan.fused_L; p.W = 8; p.tiles = c->plan.fused_tiles;
    st = reserve_epochs(c, (unsigned)max_iter + 1u);
    if (st != DEER_OK) return st;
    p.epoch = c->epoch + 1;
    c->epoch += (unsigned)max_iter + 1u;
    p.aggW = reinterpret_cast<unsigned long long*>(c->ws + c->plan.off_aggW);
    p.inclW = reinterpret_cast<unsigned long long*>(c->ws + c->plan.off_inclW);
    p.status = ctl_status(c);
    p.gate = Gate{nullptr, 0.0};
    q.feed = GruFeed{d_theta, d_x, g.d};
    // The kernel writes its per-iteration record and the iteration count straight into pinned host memory:
    // no copy back, the stream synchronisation alone makes them visible.
    char* h = reinterpret_cast<char*>(c->h_err);
    q.err = reinterpret_cast<unsigned long long*>(c->d_h_err);
    q.result = reinterpret_cast<int*>(reinterpret_cast<char*>(c->d_h_err) + (size_t)kSlots * 8 + 4);
    q.barrier = reinterpret_cast<unsigned long long*>(c->ws + c->plan.off_barrier);
    q.tol = tol;
    q.max_iter = max_iter;
    q.spin_limit = c->test_spin_limit;
    q.extra_workgroups = c->test_extra_workgroups;
    std::memset(h + (size_t)kSlots * 8, 0, 8);
#ifdef DEER_SCAN_TIMING
    p.timing = reinterpret_cast<unsigned long long*>(c->ws + c->plan.off_timing);
#endif
    prof_begin(c, KIND_NEWTON);
    HIPCHK(c, launch_gru_newton(g.dtype, g.n, q, c->stream));
    prof_end(c);
    HIPCHK(c, hipStreamSynchronize(c->stream));
    int it = 0;
    std::memcpy(&it, h + (size_t)kSlots * 8 + 4, 4);
    prof_collect(c);
    double last = 0.0;
    if (it >= 1 && it <= max_iter) {
        if (g.dtype == DEER_F32) {
            float f;
            std::memcpy(&f, h + (size_t)(it - 1) * 8, 4);
            last = (double)f;
        } else {
            std::memcpy(&last, h + (size_t)(it - 1) * 8, 8);
        }
    }
    if (it < 1 || it > max_iter || !std::isfinite(last)) {
        // either the iteration blew up or a wait ran out: the status word on the device tells which
        unsigned status = 0;
        HIPCHK(c, hipMemcpyAsync(h + (size_t)kSlots * 8, ctl_status(c), 4, hipMemcpyDeviceToHost, c->stream));
        HIPCHK(c, hipStreamSynchronize(c->stream));
        std::memcpy(&status, h + (size_t)kSlots * 8, 4);
        if (status != 0) {
            HIPCHK(c, launch_fill_zero(c->ws + c->plan.off_ctl, ctl_bytes(), c->stream));
            *busy = true;
            return DEER_OK;
        }
    }
    if (it < 1 || it > max_iter) return fail(c, DEER_ERR_HIP, "one-launch solve returned an impossible iteration count");
    double err;
    if (g.dtype == DEER_F32) {
        float f;
        std::memcpy(&f, h + (size_t)(it - 1) * 8, 4);
        err = (double)f;
    } else {
        std::memcpy(&err, h + (size_t)(it - 1) * 8, 8);
    }
    if (c->profiling) c->prof.newton_iterations += it;
    c->last_iters = it;
    *iters = it;
    *final_err = err;
    *converged = (err <= tol) ? 1 : 0;
    if (!std::isfinite(err)) return fail(c, DEER_ERR_NONFINITE, "the iteration produced a non-finite value");
    return DEER_OK;
}

}  // namespace

extern "C" {

size_t deer_theta_count(const deer_config* cfg) {
    std::string why;
    if (!validate(cfg, why)) return 0;
    return theta_count(cfg);
}

deer_status deer_workspace_bytes(const deer_config* cfg, size_t* bytes) {
    std::string why;
    if (!bytes) return fail(nullptr, DEER_ERR_INVALID_ARG, "bytes is NULL");
    if (!validate(cfg, why)) return fail(nullptr, DEER_ERR_INVALID_ARG, why);
    if (!supported(cfg, why)) return fail(nullptr, DEER_ERR_UNSUPPORTED, why);
    const deer_config in = internal_config(cfg);
    *bytes = make_pad_plan(cfg, &in, make_plan(&in).total).total;
    return DEER_OK;
}

deer_status deer_create(const deer_config* cfg, void* d_workspace, size_t workspace_bytes, void* hip_stream,
                        deer_ctx** out) {
    if (!out) return fail(nullptr, DEER_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    std::string why;
    if (!validate(cfg, why)) return fail(nullptr, DEER_ERR_INVALID_ARG, why);
    if (!supported(cfg, why)) return fail(nullptr, DEER_ERR_UNSUPPORTED, why);
    const deer_config user_cfg = *cfg;
    const deer_config in_cfg = internal_config(cfg);
    cfg = &in_cfg;   // from here on: the configuration the kernels run
    Plan plan = make_plan(cfg);
    const PadPlan pad = make_pad_plan(&user_cfg, cfg, plan.total);
    if (!d_workspace || (reinterpret_cast<uintptr_t>(d_workspace) % kAlign) != 0 || workspace_bytes < pad.total)
        return fail(nullptr, DEER_ERR_WORKSPACE, "workspace is NULL, misaligned or too small");
    deer_ctx* c = new (std::nothrow) deer_ctx();
    if (!c) return fail(nullptr, DEER_ERR_INVALID_ARG, "out of host memory");
    c->user = user_cfg;
    c->pad = pad;
    c->cfg = *cfg;
    c->plan = plan;
    c->stream = reinterpret_cast<hipStream_t>(hip_stream);
    c->ws = reinterpret_cast<char*>(d_workspace);
    c->epoch = 0;
    c->h_err = nullptr;
    c->profiling = false;
    c->prof = deer_profile{};
    c->ev_used = 0;
    for (auto& e : c->ev) e = nullptr;
    hipError_t e = hipHostMalloc(&c->h_err, (size_t)kSlots * 8 + 16, hipHostMallocMapped);
    c->d_h_err = nullptr;
    if (e == hipSuccess) e = hipHostGetDevicePointer(&c->d_h_err, c->h_err, 0);
    for (int i = 0; i < 2 * kMaxEvents && e == hipSuccess; ++i) e = hipEventCreate(&c->ev[i]);
    c->batch = env_int("DEER_BATCH", 4);
    c->last_iters = 0;
    if (c->batch < 1) c->batch = 1;
    if (c->batch > 8) c->batch = 8;
    std::vector<unsigned> table;   // (lives until the synchronisation below)
    if (e == hipSuccess && plan.mh) {
        table = mh_table(cfg, plan.tile);
        e = hipMemcpyAsync(c->ws + plan.off_mhtable, table.data(), table.size() * 4, hipMemcpyHostToDevice, c->stream);
    }
    if (e == hipSuccess) e = launch_fill_zero(c->ws + plan.off_ctl, ctl_bytes(), c->stream);
    // tagged words must not carry a valid tag by accident: epochs start at 1, so zeros never match
    if (e == hipSuccess)
        e = launch_fill_zero(c->ws + plan.off_aggW, plan.off_ctl - plan.off_aggW, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) {
        std::string msg = std::string("deer_create: ") + hipGetErrorString(e);
        deer_destroy(c);
        return fail(nullptr, DEER_ERR_HIP, msg);
    }
    c->epoch = 1;
    {
        // test hook: start the epoch counter somewhere else (e.g. just below its wrap-around)
        const int e0 = env_int("DEER_EPOCH0", 0);
        if (e0 > 0 && (unsigned)e0 < (1u << 30)) c->epoch = (unsigned)e0;
    }
    {
        // test hooks: make the grid barrier of the one-launch solve give up (it then reports a failure and
        // deer_eval solves launch by launch)
        const int sl = env_int("DEER_TEST_SPIN_LIMIT", 0), xw = env_int("DEER_TEST_EXTRA_WORKGROUPS", 0);
        c->test_spin_limit = sl > 0 ? (unsigned)sl : kSpinLimit;
        c->test_extra_workgroups = (xw > 0 && xw <= 4) ? (unsigned)xw : 0u;
    }
    c->one_launch = false;
    if (plan.fused && !plan.mh && plan.fused_W == 8 && env_int("DEER_ONE_LAUNCH", 1) != 0) {
        const long long grid = (long long)cfg->B * plan.fused_tiles;
        c->one_launch = grid <= (long long)gru_newton_capacity(cfg->dtype, cfg->n, cfg->d, plan.fused_L);
    }
    *out = c;
    return DEER_OK;
}

static deer_status eval_impl(deer_ctx* c, const void* d_theta, const void* d_x, const void* d_y0, const void* d_y_guess,
                             double tol, int32_t max_iter, void* d_y, int32_t* iters, double* final_err, int32_t* converged);

deer_status deer_eval(deer_ctx* c, const void* d_theta, const void* d_x, const void* d_y0, const void* d_y_guess,
                      double tol, int32_t max_iter, void* d_y, int32_t* iters, double* final_err,
                      int32_t* converged) {
    if (!c) return fail(nullptr, DEER_ERR_INVALID_ARG, "ctx is NULL");
    if (!c->pad.on) return eval_impl(c, d_theta, d_x, d_y0, d_y_guess, tol, max_iter, d_y, iters, final_err, converged);
    // embedded state size: zero-padded copies of the parameters, the initial state and the guess go in, the real
    // channels of the result come out
    if (!d_theta || !d_y0 || !d_y || !d_x) return fail(c, DEER_ERR_INVALID_ARG, "a required pointer is NULL");
    const deer_config& g = c->cfg;
    const bool lstm = two_part_cell(g.cell);   // its kernels take the parameters as they are
    const int n = lstm ? 2 * c->user.n : c->user.n, np = g.n;
    const long long rows = (long long)g.B * g.T;
    char* pth = c->ws + c->pad.off_theta;
    char* py0 = c->ws + c->pad.off_y0;
    char* py = c->ws + c->pad.off_y;
    if (!lstm) HIPCHK(c, launch_pad_gru_theta(g.dtype, d_theta, pth, n, np, g.d, 0, c->stream));
    HIPCHK(c, launch_pad_rows(g.dtype, d_y0, py0, g.B, n, np, 0, c->stream));
    if (d_y_guess) HIPCHK(c, launch_pad_rows(g.dtype, d_y_guess, py, rows, n, np, 0, c->stream));
    const deer_status st = eval_impl(c, lstm ? d_theta : pth, d_x, py0, d_y_guess ? py : nullptr, tol, max_iter, py, iters, final_err, converged);
    if (st != DEER_OK && st != DEER_ERR_NONFINITE) return st;
    HIPCHK(c, launch_pad_rows(g.dtype, py, d_y, rows, n, np, 1, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    return st;
}

static deer_status eval_impl(deer_ctx* c, const void* d_theta, const void* d_x, const void* d_y0, const void* d_y_guess,
                             double tol, int32_t max_iter, void* d_y, int32_t* iters, double* final_err, int32_t* converged) {
    const deer_config& g = c->cfg;
    const bool ode = g.cell == DEER_CELL_MLP_ODE;
    if (!d_theta || !d_y0 || !d_y || (!ode && !d_x)) return fail(c, DEER_ERR_INVALID_ARG, "a required pointer is NULL");
    if (!iters || !final_err || !converged) return fail(c, DEER_ERR_INVALID_ARG, "an output pointer is NULL");
    if (max_iter < 0 || !(tol >= 0.0)) return fail(c, DEER_ERR_INVALID_ARG, "max_iter and tol must be >= 0");

    const size_t esz = c->plan.esz;
    const size_t n = (size_t)g.n, B = (size_t)g.B, T = (size_t)g.T;
    const size_t ybytes = B * T * n * esz * (size_t)(c->plan.mh ? c->plan.mh_H : 1);
    char* J = c->ws + c->plan.off_J;
    char* rhs = c->ws + c->plan.off_rhs;

    if (c->one_launch && max_iter >= 1 && max_iter <= kSlots) {
        bool busy = false;
        deer_status s1 = eval_one_launch(&busy, c, d_theta, d_x, d_y0, d_y_guess, tol, max_iter, d_y, iters, final_err, converged);
        if (!busy) return s1;
        // a workgroup waited too long for the others (the device is shared): solve again launch by launch.  An
        // abandoned solve may have stored part of its last iterate: a guess that shares the output buffer is
        // no longer the caller's, so the solve starts from zeros instead.
        if (d_y_guess == d_y) d_y_guess = nullptr;
    }

    // Iteration k reads buf[k & 1] and writes buf[(k + 1) & 1].  The buffers are ordered so that the
    // iterate expected to be the last one (same count as the previous call on this context) lands in d_y
    // without a final copy.
    const int expect = c->last_iters > 0 ? c->last_iters : 1;
    char* buf[2];
    buf[expect & 1] = reinterpret_cast<char*>(d_y);
    buf[(expect + 1) & 1] = c->ws + c->plan.off_ybuf;

    deer_status st = DEER_OK;
    if (d_y_guess) {
        st = zero_ctl(c);
        if (st != DEER_OK) return st;
        if (d_y_guess != buf[0])
            HIPCHK(c, hipMemcpyAsync(buf[0], d_y_guess, ybytes, hipMemcpyDeviceToDevice, c->stream));
    } else {
        st = reserve_epochs(c, (unsigned)kSlots + 8u);
        if (st != DEER_OK) return st;
        HIPCHK(c, launch_fill_zero2(c->ws + c->plan.off_ctl, ctl_bytes(), buf[0], ybytes, c->stream));
    }
    if (ode) {
        HIPCHK(c, launch_pin_first(g.dtype, buf[0], d_y0, g.B, g.T, g.n, c->stream));
        HIPCHK(c, launch_pin_first(g.dtype, buf[1], d_y0, g.B, g.T, g.n, c->stream));
    }

    // Up to nb iterations are enqueued per host round trip; from the second one of a batch on, the
    // kernels check the previous iteration's error on the device and return at once when it already
    // met tol.  The first batch is as long as the previous call's iteration count (a solver called
    // again on similar input converges in about as many steps), later ones are short.
    double err = 1e10;
    int it = 0;
    bool nonfinite = false;
    unsigned status = 0;
    while (err > tol && it < max_iter && !nonfinite) {
        const int slot0 = it % kSlots;
        if (it > 0 && slot0 == 0) {
            st = zero_ctl(c);
            if (st != DEER_OK) return st;
        }
        int want = c->batch;
        if (it == 0 && c->last_iters > 0) want = c->last_iters < 8 ? c->last_iters : 8;
        if (it > 0 && c->last_iters > 0) want = 2;
        int nb = max_iter - it;
        if (nb > want) nb = want;
        if (nb > kSlots - slot0) nb = kSlots - slot0;
        for (int j = 0; j < nb; ++j) {
            const int k = it + j, slot = slot0 + j;
            char* src = buf[k & 1];
            char* dst = buf[(k + 1) & 1];
            const Gate gate = (j == 0) ? Gate{nullptr, 0.0} : Gate{ctl_err(c, slot - 1), tol};
            if (c->plan.fused) {
                // cell and scan in one launch; the matrices stay in registers
                HIPCHK(c, run_scan(c, nullptr, nullptr, d_y0, dst, src, 0, 0, (long long)(T * n), 0, slot, true, 0, gate,
                                   k, d_theta, d_x));
            } else if (!ode) {
                GruParams gp{d_theta, d_x, d_y0, src, J, rhs, g.B, g.T, g.n, g.d, gate, two_part_cell(g.cell) ? g.reserved : 0, g.t1};
                prof_begin(c, KIND_FUNCEVAL, k);
                HIPCHK(c, g.cell == DEER_CELL_LSTM  ? launch_lstm_funceval(g.dtype, gp, c->stream)
                          : g.cell == DEER_CELL_LEM ? launch_lem_funceval(g.dtype, gp, c->stream)
                                                    : launch_gru_funceval(g.dtype, gp, c->stream));
                prof_end(c);
                HIPCHK(c, run_scan(c, J, rhs, d_y0, dst, src, (long long)(T * n * n), (long long)(T * n),
                                   (long long)(T * n), 0, slot, true, 0, gate, k));
            } else {
                char* Gbar = c->ws + c->plan.off_Gbar;
                char* zbar = c->ws + c->plan.off_zbar;
                MlpParams mp{d_theta, src, J, rhs, g.B, g.T, g.n, g.mlp_width, gate, 0, g.mlp_hidden_layers, g.mlp_activation};
                prof_begin(c, KIND_FUNCEVAL, k);
                HIPCHK(c, mlp_fast_path(&g) ? launch_mlp_funceval(g.dtype, mp, c->stream)
                                            : launch_mlp_general_funceval(g.dtype, mp, c->stream));
                prof_end(c);
                OdeDiscParams dp{J, rhs, src, Gbar, zbar, g.B, g.T, g.n, (g.t1 - g.t0) / (double)(g.T - 1), gate, 0, 0};
                prof_begin(c, KIND_DISC, k);
                HIPCHK(c, launch_ode_discretise(g.dtype, dp, c->stream));
                prof_end(c);
                // correction form: the scan solves delta_{i+1} = Gbar_i delta_i + res_i from delta_0 = 0 and
                // writes y_next = y + delta at positions 1..T-1; position 0 stays y0
                HIPCHK(c, run_scan(c, Gbar, zbar, nullptr, dst + n * esz, src + n * esz, (long long)((T - 1) * n * n),
                                   (long long)((T - 1) * n), (long long)(T * n), 0, slot, true, 1, gate, k));
            }
        }
        // error words of the batch and the status word come back with one synchronisation
        char* h = reinterpret_cast<char*>(c->h_err);
        HIPCHK(c, hipMemcpyAsync(h, ctl_err(c, slot0), (size_t)nb * 8, hipMemcpyDeviceToHost, c->stream));
        HIPCHK(c, hipMemcpyAsync(h + (size_t)kSlots * 8, ctl_status(c), 4, hipMemcpyDeviceToHost, c->stream));
        HIPCHK(c, hipStreamSynchronize(c->stream));
        std::memcpy(&status, h + (size_t)kSlots * 8, 4);
        for (int j = 0; j < nb; ++j) {
            const char* ep = h + (size_t)j * 8;
            if (g.dtype == DEER_F32) {
                float f;
                std::memcpy(&f, ep, 4);
                err = (double)f;
            } else {
                std::memcpy(&err, ep, 8);
            }
            ++it;
            if (!std::isfinite(err)) { nonfinite = true; break; }
            if (!(err > tol)) break;
        }
        prof_collect(c, it);
        if (status != 0) break;
    }
    if (it > 0) c->last_iters = it;
    char* fin = buf[it & 1];
    if (fin != reinterpret_cast<char*>(d_y)) {
        HIPCHK(c, hipMemcpyAsync(d_y, fin, ybytes, hipMemcpyDeviceToDevice, c->stream));
        HIPCHK(c, hipStreamSynchronize(c->stream));
    }
    if (status != 0) st = fail(c, DEER_ERR_HIP, "scan kernel: a tile waited too long for its predecessors");
    *iters = it;
    *final_err = err;
    *converged = (err <= tol) ? 1 : 0;
    if (st != DEER_OK) return st;
    if (nonfinite) return fail(c, DEER_ERR_NONFINITE, "the iteration produced a non-finite value");
    return DEER_OK;
}

// Backward derivative for the ODE form (Sec. 3.1.1 eq. 7 on the discretised operator of Sec. 3.3 eq. 8-9):
// G = -df/dy at the trajectory, Gbar_i = exp(-(G_i + G_{i+1}) dt / 2), the reverse scan
// lam_{T-1} = g_{T-1}, lam_i = g_i + Gbar_i^T lam_{i+1} for i >= 1, then per interval
// u_i = dt phi1(.)^T lam_{i+1} (and dL/dy0 = g_0 + Gbar_0^T lam_1), and the VJP of f with
// w_j = (u_j + u_{j-1}) / 2 at every grid point.
static deer_status grad_ode(deer_ctx* c, const void* d_theta, const void* d_y, const void* d_dLdy, void* d_dLdtheta,
                            void* d_dLdy0) {
    const deer_config& g = c->cfg;
    if (!d_theta || !d_y || !d_dLdy || !d_dLdtheta) return fail(c, DEER_ERR_INVALID_ARG, "a required pointer is NULL");
    const size_t n = (size_t)g.n, T = (size_t)g.T, esz = (size_t)c->plan.esz;
    char* G = c->ws + c->plan.off_J;
    char* z = c->ws + c->plan.off_rhs;       // z of the field evaluation, then the residual, then u
    char* res = z;
    char* u = z;
    char* lam0 = c->ws + c->plan.off_ybuf;   // first pass of the reverse scan
    char* lam = c->ws + c->plan.off_zbar;    // [B,T-1,n]: lam at grid points 1..T-1
    char* Dm = c->ws + c->plan.off_Gbar;
    const double dt = (g.t1 - g.t0) / (double)(g.T - 1);
    const Gate open{nullptr, 0.0};

    deer_status st = zero_ctl(c);
    if (st != DEER_OK) return st;
    MlpParams mp{d_theta, d_y, G, z, g.B, g.T, g.n, g.mlp_width, open, 1, g.mlp_hidden_layers, g.mlp_activation};   // the backward pass needs G only
    prof_begin(c, KIND_FUNCEVAL);
    HIPCHK(c, mlp_fast_path(&g) ? launch_mlp_funceval(g.dtype, mp, c->stream) : launch_mlp_general_funceval(g.dtype, mp, c->stream));
    prof_end(c);
    // D_i = Gbar_i - I, the matrices alone
    OdeDiscParams dp{G, z, d_y, Dm, lam, g.B, g.T, g.n, dt, open, 1, 1};
    prof_begin(c, KIND_DISC);
    HIPCHK(c, launch_ode_discretise(g.dtype, dp, c->stream));
    prof_end(c);
    // Reverse scan over grid points 1..T-1 (matrices D_1..D_{T-2}; D_0 serves dL/dy0 only), twice: the scan
    // works on I + D rounded to the working precision, which perturbs the generator by eps / |D|; one step of
    // iterative refinement with the residual evaluated on D itself removes that (it matters in fp32 only,
    // where it costs a second scan: 1.4e-4 against 1e-5 relative error of lam at T = 1e5).
    const char* gvec = reinterpret_cast<const char*>(d_dLdy) + n * esz;
    const long long sD = (long long)((T - 1) * n * n), sg = (long long)(T * n), sl = (long long)((T - 1) * n);
    const bool refine = g.dtype == DEER_F32;
    HIPCHK(c, run_scan(c, Dm, gvec, nullptr, refine ? lam0 : lam, nullptr, sD, sg, sl, 1, 0, false, 0, open, -1, nullptr,
                       nullptr, 1));
    if (refine) {
        prof_begin(c, KIND_DISC);
        HIPCHK(c, launch_ode_dual_residual(g.dtype, Dm, d_dLdy, lam0, res, g.B, g.T, g.n, c->stream));
        prof_end(c);
        HIPCHK(c, run_scan(c, Dm, res, nullptr, lam, lam0, sD, sl, sl, 1, 1, false, 1, open, -1, nullptr, nullptr, 1));
    }
    OdeDualParams up{G, lam, d_dLdy, u, d_dLdy0, g.B, g.T, g.n, dt};
    prof_begin(c, KIND_DISC);
    HIPCHK(c, launch_ode_dual(g.dtype, up, c->stream));
    prof_end(c);
    MlpVjpParams vp{d_theta, d_y, u, c->ws + c->plan.off_partial, d_dLdtheta, g.B, g.T, g.n, g.mlp_width, c->plan.vjp_blocks,
                    g.mlp_hidden_layers, g.mlp_activation};
    prof_begin(c, KIND_VJP);
    if (!mlp_fast_path(&g)) {
        HIPCHK(c, launch_mlp_general_vjp(g.dtype, vp, c->stream));
    } else if (mlp_vjp_mfma_supported(g.dtype, g.n, g.mlp_width) && env_int("DEER_VJP_MFMA", 1) != 0) {
        if (vp.blocks > 512) vp.blocks = 512;   // two wavefronts per SIMD by registers: 512 blocks of four fill the chip once
        HIPCHK(c, launch_mlp_vjp_mfma(vp, c->stream));
        HIPCHK(c, launch_partial_reduce(g.dtype, vp.partial, d_dLdtheta, (long long)theta_count(&g), vp.blocks * 4, c->stream));
    } else {
        HIPCHK(c, launch_mlp_vjp(g.dtype, vp, c->stream));
    }
    prof_end(c);
    st = check_status(c);
    prof_collect(c);
    return st;
}

static deer_status grad_impl(deer_ctx* c, const void* d_theta, const void* d_x, const void* d_y0, const void* d_y,
                             const void* d_dLdy, void* d_dLdx, void* d_dLdtheta, void* d_dLdy0);

deer_status deer_grad(deer_ctx* c, const void* d_theta, const void* d_x, const void* d_y0, const void* d_y,
                      const void* d_dLdy, void* d_dLdx, void* d_dLdtheta, void* d_dLdy0) {
    if (!c) return fail(nullptr, DEER_ERR_INVALID_ARG, "ctx is NULL");
    if (!c->pad.on) return grad_impl(c, d_theta, d_x, d_y0, d_y, d_dLdy, d_dLdx, d_dLdtheta, d_dLdy0);
    // embedded state size: padded copies in, the real entries of the gradients out (the cotangent of the extra
    // channels is zero and stays zero through the dual recurrence)
    if (!d_theta || !d_x || !d_y0 || !d_y || !d_dLdy || !d_dLdtheta) return fail(c, DEER_ERR_INVALID_ARG, "a required pointer is NULL");
    const deer_config& g = c->cfg;
    const bool lstm = two_part_cell(g.cell);
    const int n = lstm ? 2 * c->user.n : c->user.n, np = g.n;
    const long long rows = (long long)g.B * g.T;
    char* pth = c->ws + c->pad.off_theta;
    char* py0 = c->ws + c->pad.off_y0;
    char* py = c->ws + c->pad.off_y;
    char* pg = c->ws + c->pad.off_g;
    char* pdth = c->ws + c->pad.off_dtheta;
    char* pdy0 = c->ws + c->pad.off_dy0;
    if (!lstm) HIPCHK(c, launch_pad_gru_theta(g.dtype, d_theta, pth, n, np, g.d, 0, c->stream));
    HIPCHK(c, launch_pad_rows(g.dtype, d_y0, py0, g.B, n, np, 0, c->stream));
    HIPCHK(c, launch_pad_rows(g.dtype, d_y, py, rows, n, np, 0, c->stream));
    HIPCHK(c, launch_pad_rows(g.dtype, d_dLdy, pg, rows, n, np, 0, c->stream));
    const deer_status st = grad_impl(c, lstm ? d_theta : pth, d_x, py0, py, pg, d_dLdx, lstm ? d_dLdtheta : pdth, d_dLdy0 ? pdy0 : nullptr);
    if (st != DEER_OK) return st;
    if (!lstm) HIPCHK(c, launch_pad_gru_theta(g.dtype, pdth, d_dLdtheta, n, np, g.d, 1, c->stream));
    if (d_dLdy0) HIPCHK(c, launch_pad_rows(g.dtype, pdy0, d_dLdy0, g.B, n, np, 1, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    return DEER_OK;
}

static deer_status grad_impl(deer_ctx* c, const void* d_theta, const void* d_x, const void* d_y0, const void* d_y,
                             const void* d_dLdy, void* d_dLdx, void* d_dLdtheta, void* d_dLdy0) {
    if (!c) return fail(nullptr, DEER_ERR_INVALID_ARG, "ctx is NULL");
    const deer_config& g = c->cfg;
    if (g.cell == DEER_CELL_MLP_ODE) return grad_ode(c, d_theta, d_y, d_dLdy, d_dLdtheta, d_dLdy0);
    if (!d_theta || !d_x || !d_y0 || !d_y || !d_dLdy || !d_dLdtheta)
        return fail(c, DEER_ERR_INVALID_ARG, "a required pointer is NULL");
    const size_t n = (size_t)g.n, T = (size_t)g.T;
    char* J = c->ws + c->plan.off_J;
    char* rhs = c->ws + c->plan.off_rhs;
    char* lam = c->ws + c->plan.off_ybuf;

    deer_status st = zero_ctl(c);
    if (st != DEER_OK) return st;
    if (c->plan.grad_fused) {
        // lam = (dL/dy) L_G^{-1} with the transposed Jacobians computed inside the reverse scan (they never reach memory)
        HIPCHK(c, run_scan(c, nullptr, d_dLdy, nullptr, lam, d_y, 0, (long long)(T * n), (long long)(T * n), 1, 0, false, 0,
                           Gate{nullptr, 0.0}, -1, d_theta, d_x));
    } else {
        // Jacobians at the given trajectory (the right-hand side output is not used)
        GruParams gp{d_theta, d_x, d_y0, d_y, J, rhs, g.B, g.T, g.n, g.d, Gate{nullptr, 0.0}, two_part_cell(g.cell) ? g.reserved : 0, g.t1};
        prof_begin(c, KIND_FUNCEVAL);
        HIPCHK(c, g.cell == DEER_CELL_LSTM  ? launch_lstm_funceval(g.dtype, gp, c->stream)
                  : g.cell == DEER_CELL_LEM ? launch_lem_funceval(g.dtype, gp, c->stream)
                                            : launch_gru_funceval(g.dtype, gp, c->stream));
        prof_end(c);
        // lam = (dL/dy) L_G^{-1}: reverse scan with transposed Jacobians
        HIPCHK(c, run_scan(c, J, d_dLdy, nullptr, lam, nullptr, (long long)(T * n * n), (long long)(T * n),
                           (long long)(T * n), 1, 0, false));
    }
    GruVjpParams vp{d_theta, d_x, d_y0, d_y, lam, d_dLdx, d_dLdy0, c->ws + c->plan.off_partial, d_dLdtheta,
                    g.B, g.T, g.n, g.d, c->plan.vjp_blocks, c->plan.mh ? c->plan.mh_H : 0, c->plan.mh ? c->plan.mh_K : 0,
                    c->plan.mh ? c->ws + c->plan.off_dy0parts : nullptr, two_part_cell(g.cell) ? g.reserved : 0, g.t1};
    prof_begin(c, KIND_VJP);
    if (g.cell == DEER_CELL_LSTM) {
        HIPCHK(c, launch_lstm_vjp(g.dtype, vp, c->stream));
    } else if (g.cell == DEER_CELL_LEM) {
        HIPCHK(c, launch_lem_vjp(g.dtype, vp, c->stream));
    } else if (!c->plan.mh && gru_vjp_mfma_supported(g.dtype, g.n, g.d) && env_int("DEER_VJP_MFMA", 1) != 0) {
        HIPCHK(c, launch_gru_vjp_mfma(vp, c->stream));
        HIPCHK(c, launch_partial_reduce(g.dtype, vp.partial, d_dLdtheta, (long long)theta_count(&g), vp.blocks * 4, c->stream));
    } else {
        HIPCHK(c, launch_gru_vjp(g.dtype, vp, c->stream));
    }
    prof_end(c);
    st = check_status(c);
    prof_collect(c);
    return st;
}

deer_status deer_linrec_solve(deer_ctx* c, const void* d_A, const void* d_b, const void* d_y0, void* d_y,
                              int32_t reverse) {
    if (!c) return fail(nullptr, DEER_ERR_INVALID_ARG, "ctx is NULL");
    const deer_config& g = c->cfg;
    if (!d_A || !d_b || !d_y) return fail(c, DEER_ERR_INVALID_ARG, "a required pointer is NULL");
    if (g.cell != DEER_CELL_GRU || c->plan.mh || c->pad.on || c->user.cell != DEER_CELL_GRU)
        return fail(c, DEER_ERR_UNSUPPORTED, "deer_linrec_solve needs a plain GRU-shaped context of state size 1, 2, 4, 8, 16 or 32");
    const size_t n = (size_t)g.n, T = (size_t)g.T;
    deer_status st = zero_ctl(c);
    if (st != DEER_OK) return st;
    HIPCHK(c, run_scan(c, d_A, d_b, reverse ? nullptr : d_y0, d_y, nullptr, (long long)(T * n * n),
                       (long long)(T * n), (long long)(T * n), reverse ? 1 : 0, 0, false));
    st = check_status(c);
    prof_collect(c);
    return st;
}

deer_status deer_set_profiling(deer_ctx* c, int32_t on) {
    if (!c) return fail(nullptr, DEER_ERR_INVALID_ARG, "ctx is NULL");
    c->profiling = on != 0;
    if (on) c->prof = deer_profile{};
    c->ev_used = 0;
    return DEER_OK;
}

deer_status deer_get_profile(deer_ctx* c, deer_profile* out) {
    if (!c || !out) return fail(c, DEER_ERR_INVALID_ARG, "NULL argument");
    *out = c->prof;
    return DEER_OK;
}

#ifdef DEER_SCAN_TIMING
void* deer_debug_timing(deer_ctx* c) { return c ? c->ws + c->plan.off_timing : nullptr; }
#endif

deer_status deer_linrec_solve_static(int32_t dtype, int32_t B, int32_t T, int32_t n, const void* d_A, const void* d_b,
                                     const void* d_y0, void* d_y, int32_t reverse, void* hip_stream, int32_t* d_status) {
    deer_config cfg{};
    cfg.cell = DEER_CELL_GRU;
    cfg.dtype = dtype;
    cfg.B = B;
    cfg.T = T;
    cfg.n = n;
    cfg.d = 1;
    std::string why;
    if (!validate(&cfg, why)) return fail(nullptr, DEER_ERR_INVALID_ARG, why);
    if (!supported(&cfg, why)) return fail(nullptr, DEER_ERR_UNSUPPORTED, why);
    if (native_n(n) != n) return fail(nullptr, DEER_ERR_UNSUPPORTED, "the scan alone needs a state size of 1, 2, 4, 8, 16, 32 or (fp32) 64");
    if (!d_A || !d_b || !d_y) return fail(nullptr, DEER_ERR_INVALID_ARG, "a required pointer is NULL");
    // the part of the plan the scan uses, re-based to the start of the static array
    Plan plan = make_plan(&cfg);
    const size_t base = plan.off_aggW;
    const size_t need = plan.off_ctl - base + ctl_bytes();
    if (need > kStaticBytes)
        return fail(nullptr, DEER_ERR_WORKSPACE,
                    "deer_linrec_solve_static: B * tiles of this shape need " + std::to_string(need) +
                        " bytes of published words, the static scratch holds " + std::to_string(kStaticBytes));
    plan.off_aggW -= base;
    plan.off_inclW -= base;
    plan.off_barrier -= base;
    plan.off_ctl -= base;

    // address of this device's copy of the array, looked up once per device with that device current
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(nullptr, DEER_ERR_HIP, std::string("hipGetDevice: ") + hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(nullptr, DEER_ERR_UNSUPPORTED, "device index beyond the table of static scratch addresses");
    void* scratch = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_static_mutex);
        if (!g_static_ptr[dev]) {
            void* ptr = nullptr;
            e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(deer_static_scratch));
            if (e != hipSuccess || !ptr)
                return fail(nullptr, DEER_ERR_HIP, std::string("hipGetSymbolAddress(deer_static_scratch): ") + hipGetErrorString(e));
            g_static_ptr[dev] = ptr;
        }
        scratch = g_static_ptr[dev];
    }

    // a context on the stack (host memory only) that points the scan at the static array
    deer_ctx c;
    c.user = cfg;
    c.pad = PadPlan{};
    c.cfg = cfg;
    c.plan = plan;
    c.stream = reinterpret_cast<hipStream_t>(hip_stream);
    c.ws = reinterpret_cast<char*>(scratch);
    c.epoch = 1;   // the same tag in every call: everything published by the previous call is cleared below
    c.h_err = nullptr;
    c.d_h_err = nullptr;
    c.profiling = false;
    c.ev_used = 0;
    // The array keeps the last call's contents: clear the published words (their tags would match again), the
    // tile dispenser and the status word, with a fill kernel on the caller's stream.
    e = launch_fill_zero(scratch, need, c.stream);
    if (e != hipSuccess) return fail(nullptr, DEER_ERR_HIP, std::string("fill launch: ") + hipGetErrorString(e));
    const size_t nn = (size_t)n, TT = (size_t)T;
    e = run_scan(&c, d_A, d_b, reverse ? nullptr : d_y0, d_y, nullptr, (long long)(TT * nn * nn), (long long)(TT * nn),
                 (long long)(TT * nn), reverse ? 1 : 0, 0, false);
    if (e != hipSuccess) return fail(nullptr, DEER_ERR_HIP, std::string("scan launch: ") + hipGetErrorString(e));
    if (d_status) {
        e = launch_copy_word(d_status, ctl_status(&c), c.stream);
        if (e != hipSuccess) return fail(nullptr, DEER_ERR_HIP, std::string("status copy launch: ") + hipGetErrorString(e));
    }
    return DEER_OK;
}

const char* deer_last_error(const deer_ctx* c) {
    return c ? c->last_error.c_str() : g_last_error.c_str();
}

void deer_destroy(deer_ctx* c) {
    if (!c) return;
    for (auto& e : c->ev)
        if (e) (void)hipEventDestroy(e);
    if (c->h_err) (void)hipHostFree(c->h_err);
    delete c;
}

}  // extern "C"
