// C ABI of the library (see include/pararnn.h): argument checks, workspace
// layout, tile-shape choice and the enqueue sequence.  No kernel code here.
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include <initializer_list>

#include "../../include/pararnn.h"
#include "dense.h"
#include "launch.h"

using namespace pararnn;

namespace {

struct CellInfo { int G, S, PR; };

bool cell_info(int cell, CellInfo *ci)
{
    switch (cell) {
    case PARARNN_GRU_DIAG: *ci = {3, 1, 6}; return true;
    case PARARNN_LSTM_DIAG: *ci = {4, 2, 8}; return true;
    case PARARNN_TANH_DENSE: *ci = {1, 1, 0}; return true;
    case PARARNN_LINEAR_DIAG: *ci = {1, 1, 2}; return true;
    case PARARNN_PARALSTM_DIAG: *ci = {3, 2, 8}; return true;
    }
    return false;
}

size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }

// process-wide switch for launches that run several Newton iterations (pararnn_set_fused)
int g_fused_enabled = 1;
int g_fused_head = 5;      // iterations in the first launch of a solve to a tolerance (0 = none)

// process-wide tile-shape override: {vec, ll, c, w}; vec = 0 none, -1 not yet read from the environment
int g_tile_override[4] = {-1, 0, 0, 0};

// Tile shape for a problem.  The table is the result of sweeps on MI355X over
// the compiled shapes (fp32 and bf16 storage, forward and backward, GRU and
// LSTM at 2^25..2^30 timestep-channels): one channel per lane (two for bf16
// forward) with 128..256-byte row segments and 128..256 steps per tile.
// PARARNN_TILE="vec,ll,c,w" or pararnn_set_tile() overrides it (tuning aid; the
// combination must be one that is compiled in and allowed by H and alignment).
TileCfg choose_tile(int cell_kind, int dtype, bool backward, int H, int align_elems, bool fused = false)
{
    int vmax = 1;
    if (H % 4 == 0 && align_elems >= 4) vmax = 4;
    else if (H % 2 == 0 && align_elems >= 2) vmax = 2;
    TileCfg cfg = {1, 2, 8, 8};                          // 32 channels x 128 steps
    const bool lstm = cell_kind == PARARNN_LSTM_DIAG || cell_kind == PARARNN_PARALSTM_DIAG, bf = dtype == PARARNN_BF16;
    if (H <= 8) {
        cfg = {1, 8, 4, 2};                              // 8 channels x 64 steps
    } else if (H <= 32) {
        cfg = {1, 2, 8, 8};
    } else if (fused) {
        // the fused blocks are bound by vector arithmetic, not by HBM: long per-thread chunks spread the
        // per-thread cost of the wave / workgroup / look-back levels over more cell evaluations
        if (lstm) cfg = {1, 1, 16, 4};                   // 64 channels x 64 steps
        else cfg = {1, 1, 12, 8};                        // 64 channels x 96 steps
    } else if (!backward) {
        if (lstm) cfg = {1, 1, 8, 16};                   // 64 channels x 128 steps
        else if (bf && vmax >= 2) cfg = {2, 2, 8, 8};    // 64 channels x 128 steps
        else cfg = {1, 1, 8, 16};                        // 64 channels x 128 steps
    } else {
        if (cell_kind == PARARNN_PARALSTM_DIAG) cfg = {1, 1, 12, 8};   // 64 channels x 96 steps
        else if (lstm) cfg = {1, 1, 16, 8};              // 64 channels x 128 steps
        else if (bf) cfg = {1, 1, 8, 8};                 // 64 channels x 64 steps
        else cfg = {1, 2, 8, 16};                        // 32 channels x 256 steps
    }
    if (g_tile_override[0] == -1) {
        g_tile_override[0] = 0;
        const char *e = getenv("PARARNN_TILE");
        int v, l, c, w;
        if (e && sscanf(e, "%d,%d,%d,%d", &v, &l, &c, &w) == 4) {
            g_tile_override[0] = v; g_tile_override[1] = l; g_tile_override[2] = c; g_tile_override[3] = w;
        }
    }
    if (g_tile_override[0] > 0 && g_tile_override[0] <= vmax) {
        cfg.vec = g_tile_override[0]; cfg.ll = g_tile_override[1];
        cfg.c = g_tile_override[2]; cfg.w = g_tile_override[3];
    }
    return cfg;
}

struct Layout {
    ScanGeom g;
    TileCfg cfg;
    size_t off_rec, n_rec, off_bnd, off_iter, off_part, total;
};

// Workspace: [Ctrl | carry records (rec_slots sets) | boundary rows | fp32 iterate (bf16 forward) |
// parameter-gradient partials (backward)]
Layout make_layout(int cell_kind, const CellInfo &ci, int dtype, int B, int L, int H, bool backward, int align_elems,
                   bool fused = false, int rec_slots = 1, const TileCfg *force = nullptr)
{
    Layout lo;
    lo.cfg = force ? *force : choose_tile(cell_kind, dtype, backward, H, align_elems, fused);
    const int CW = (kWave / lo.cfg.ll) * lo.cfg.vec, T = lo.cfg.c * lo.cfg.ll * lo.cfg.w;
    ScanGeom &g = lo.g;
    g.B = B; g.L = L; g.H = H; g.T = T;
    g.n_lt = (L + T - 1) / T;
    g.n_cg = (H + CW - 1) / CW;
    g.n_groups = B * g.n_cg;
    g.n_tiles = g.n_groups * g.n_lt;
    const size_t NW = (size_t)ci.S * ci.S + 2 * ci.S;
    size_t off = round256(sizeof(Ctrl));
    lo.n_rec = (size_t)g.n_tiles * NW * CW;
    lo.off_rec = off;   off += round256(lo.n_rec * (size_t)rec_slots * sizeof(unsigned long long));
    lo.off_bnd = off;
    if (!backward) off += round256((size_t)2 * g.n_lt * B * ci.S * H * sizeof(float));
    lo.off_iter = off;
    if (!backward && dtype == PARARNN_BF16) off += round256((size_t)B * L * ci.S * H * sizeof(float));
    lo.off_part = off;
    if (backward) off += round256((size_t)g.n_lt * B * ci.PR * H * sizeof(float));
    lo.total = off;
    return lo;
}

bool dims_ok(int B, int L, int H)
{
    if (B < 1 || L < 1 || H < 1) return false;
    // keep every element count inside size_t/int ranges the kernels assume
    const double n = (double)B * (double)L * (double)H;
    return n < 3.0e10 && (double)B * H < 2.0e9 && L < (1 << 30);
}

bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }

// widest vector (in elements of size esz: 4, 2 or 1) every pointer in the list allows; NULL allows any
int align_elems(size_t esz, std::initializer_list<const void *> ptrs)
{
    int a = 4;
    for (const void *p : ptrs) {
        if (!p) continue;
        const int here = aligned(p, 4 * esz) ? 4 : aligned(p, 2 * esz) ? 2 : 1;
        if (here < a) a = here;
    }
    return a;
}

// Iterations the next launch of a solve performs: `done` of max_iter are behind it, `n_fused`
// carry-record slots are available (0: every launch is one iteration).  The first launch takes
// n_fused, the following ones 1, 2, 4, ... capped by n_fused and by what is left.
int next_block_size(int done, int launches, int max_iter, int n_fused)
{
    int K = 1;
    if (n_fused > 0) {
        if (launches == 0) K = n_fused;
        else K = launches - 1 < 30 ? 1 << (launches - 1) : n_fused;
        if (K > n_fused) K = n_fused;
    }
    if (K > max_iter - done) K = max_iter - done;
    return K;
}

// n_fused = number of carry-record slots the workspace holds (0: none; fused launches are not used).
// tol < 0: the whole fixed-count solve is one fused launch of n_fused = max_iter iterations.
// tol >= 0: the solve is a sequence of launches, each checked by the stopping test on the
// device: a fused block of n_fused iterations from the initial guess, then blocks of 1, 2,
// 4, ... (at most n_fused) iterations from the iterate; a block of one iteration is the
// per-iteration kernel.  Launches after the one that met the tolerance return at once, and
// there are O(max_iter / n_fused) of them instead of max_iter.
template <class Cell>
int forward_diag(const CellInfo &ci, int dtype, const Layout &lo, FwdArgs &a, hipStream_t st, void *h,
                 int status0, int max_iter, int n_fused)
{
    char *ws = reinterpret_cast<char *>(a.ctrl);
    const bool bf = dtype == PARARNN_BF16;
    const bool to_tol = a.tol >= 0.0f;
    hipError_t e;
    a.hit = bf ? reinterpret_cast<float *>(ws + lo.off_iter) : static_cast<float *>(h);
    e = launch_reset(a.ctrl, a.rec, lo.n_rec * (size_t)(n_fused > 0 ? n_fused : 1), a.iters_out, status0, st);
    if (e != hipSuccess) return PARARNN_HIP_ERROR;
    if (max_iter == 0) {
        // only the initial guess is asked for; otherwise the first iteration computes it on the fly
        e = bf ? Kernels<Cell, unsigned short>::init_guess(lo.cfg.vec, a, st) : Kernels<Cell, float>::init_guess(lo.cfg.vec, a, st);
        if (e != hipSuccess) return PARARNN_HIP_ERROR;
    }
    FusedArgs f;
    memset(&f, 0, sizeof(f));
    f.g = a.g; f.params = a.params; f.u = a.u; f.h0 = a.h0; f.h = h;
    f.rec = a.rec; f.rec_stride = lo.n_rec;
    f.gmaxk = reinterpret_cast<unsigned int *>(ws + 64);
    f.ctrl = a.ctrl; f.iters_out = a.iters_out; f.trace = a.trace;
    f.head = to_tol ? 1 : 0; f.max_iter = max_iter; f.tol = a.tol;
    f.hit = to_tol ? a.hit : nullptr;
    f.bnd = a.bnd;
    int done = 0, cur = 0;
    for (int launches = 0; done < max_iter; ++launches) {
        const int K = next_block_size(done, launches, max_iter, n_fused);
        if (n_fused > 0 && (K > 1 || done == 0)) {
            f.n_iters = K; f.k0 = done; f.bnd_cur = cur;
            e = bf ? Kernels<Cell, unsigned short>::newton_fused(lo.cfg, f, st) : Kernels<Cell, float>::newton_fused(lo.cfg, f, st);
        } else {
            a.k = done + 1; a.bnd_cur = cur;
            e = bf ? Kernels<Cell, unsigned short>::newton_iter(lo.cfg, a, done == 0, st)
                   : Kernels<Cell, float>::newton_iter(lo.cfg, a, done == 0, st);
        }
        if (e != hipSuccess) return e == hipErrorInvalidValue ? PARARNN_UNSUPPORTED : PARARNN_HIP_ERROR;
        done += K;
        cur ^= 1;
    }
    if (bf && !(n_fused > 0 && !to_tol)) {
        // rounds the fp32 iterate into the output; skipped on the device when a fused block
        // already wrote the final iterate
        e = launch_store_bf16(a.hit, h, (size_t)lo.g.B * lo.g.L * ci.S * lo.g.H, a.ctrl, st);
        if (e != hipSuccess) return PARARNN_HIP_ERROR;
    }
    return PARARNN_OK;
}

template <class Cell>
int backward_diag(const CellInfo &ci, int dtype, const Layout &lo, BwdArgs &a, hipStream_t st, float *dparams)
{
    hipError_t e = launch_reset(a.ctrl, a.rec, lo.n_rec, nullptr, 0, st);
    if (e != hipSuccess) return PARARNN_HIP_ERROR;
    e = dtype == PARARNN_BF16 ? Kernels<Cell, unsigned short>::backward(lo.cfg, a, st)
                              : Kernels<Cell, float>::backward(lo.cfg, a, st);
    if (e != hipSuccess) return e == hipErrorInvalidValue ? PARARNN_UNSUPPORTED : PARARNN_HIP_ERROR;
    e = launch_param_reduce(a.part, dparams, lo.g.n_lt * lo.g.B, ci.PR * lo.g.H, st);
    return e == hipSuccess ? PARARNN_OK : PARARNN_HIP_ERROR;
}

}  // namespace

extern "C" {

const char *pararnn_status_string(int status)
{
    switch (status) {
    case PARARNN_OK: return "OK";
    case PARARNN_NOT_CONVERGED: return "NOT_CONVERGED";
    case PARARNN_INVALID_ARG: return "INVALID_ARG";
    case PARARNN_WORKSPACE_TOO_SMALL: return "WORKSPACE_TOO_SMALL";
    case PARARNN_HIP_ERROR: return "HIP_ERROR";
    case PARARNN_NONFINITE: return "NONFINITE";
    case PARARNN_UNSUPPORTED: return "UNSUPPORTED";
    case PARARNN_INTERNAL: return "INTERNAL";
    }
    return "UNKNOWN";
}

int pararnn_version(void) { return 100; }

int pararnn_set_tile(int vec, int ll, int c, int w)
{
    if (vec == 0) { g_tile_override[0] = 0; return PARARNN_OK; }
    bool known = false;
#define PARARNN_CASE(V, LLv, C, W) known = known || (vec == V && ll == LLv && c == C && w == W);
    PARARNN_SHAPES(PARARNN_CASE)
#undef PARARNN_CASE
    if (!known) return PARARNN_UNSUPPORTED;
    g_tile_override[0] = vec; g_tile_override[1] = ll; g_tile_override[2] = c; g_tile_override[3] = w;
    return PARARNN_OK;
}

int pararnn_cell_gates(int cell)
{
    CellInfo ci;
    return cell_info(cell, &ci) ? ci.G : -1;
}

int pararnn_cell_state(int cell)
{
    CellInfo ci;
    return cell_info(cell, &ci) ? ci.S : -1;
}

size_t pararnn_workspace_bytes(int cell, int dtype, int B, int L, int H, int backward)
{
    CellInfo ci;
    if (!cell_info(cell, &ci) || (dtype != PARARNN_F32 && dtype != PARARNN_BF16) || !dims_ok(B, L, H)) return 0;
    if (cell == PARARNN_TANH_DENSE) return dense_workspace_bytes(dtype, B, L, H, backward);
    // the size must not depend on pointer alignment: take the larger footprint when they differ
    size_t need = 0;
    for (int al = 1; al <= 4; al *= 2) {
        const Layout lo = make_layout(cell, ci, dtype, B, L, H, backward != 0, al);
        if (lo.total > need) need = lo.total;
        if (!backward && g_fused_enabled && g_fused_head > 0) {
            const Layout lf = make_layout(cell, ci, dtype, B, L, H, false, al, true, g_fused_head);
            if (lf.total > need) need = lf.total;
        }
    }
    return need;
}

size_t pararnn_workspace_bytes_fused(int cell, int dtype, int B, int L, int H, int n_iters)
{
    CellInfo ci;
    if (!cell_info(cell, &ci) || (dtype != PARARNN_F32 && dtype != PARARNN_BF16) || !dims_ok(B, L, H)) return 0;
    size_t need = pararnn_workspace_bytes(cell, dtype, B, L, H, 0);
    if (cell == PARARNN_TANH_DENSE || n_iters < 1 || n_iters > kMaxFused) return need;
    for (int al = 1; al <= 4; al *= 2) {
        const Layout lf = make_layout(cell, ci, dtype, B, L, H, false, al, true, n_iters);
        if (lf.off_bnd > need) need = lf.off_bnd;
    }
    return need;
}

int pararnn_set_fused(int enable)
{
    g_fused_enabled = enable ? 1 : 0;
    return PARARNN_OK;
}

int pararnn_solve_plan(float tol, int max_iter, int *block_sizes, int capacity)
{
    if (max_iter < 0 || tol != tol || (capacity > 0 && !block_sizes)) return -1;
    int n_fused = 0;
    if (g_fused_enabled && max_iter >= 1)
        n_fused = tol < 0.0f ? (max_iter <= kMaxFused ? max_iter : 0) : (max_iter < g_fused_head ? max_iter : g_fused_head);
    int done = 0, launches = 0;
    for (; done < max_iter; ++launches) {
        const int K = next_block_size(done, launches, max_iter, n_fused);
        if (launches < capacity) block_sizes[launches] = K;
        done += K;
    }
    return launches;
}

int pararnn_set_fused_head(int n_iters)
{
    if (n_iters < 0 || n_iters > kMaxFused) return PARARNN_INVALID_ARG;
    g_fused_head = n_iters;
    return PARARNN_OK;
}

int pararnn_forward(int cell, int dtype, const float *params, const void *u, const void *h0, int B, int L,
                    int H, float tol, int max_iter, void *h, int *iters, float *delta_trace, void *workspace,
                    size_t workspace_bytes, void *hip_stream)
{
    CellInfo ci;
    if (!cell_info(cell, &ci) || (dtype != PARARNN_F32 && dtype != PARARNN_BF16)) return PARARNN_INVALID_ARG;
    if (!dims_ok(B, L, H) || max_iter < 0 || !params || !u || !h || !iters || !workspace) return PARARNN_INVALID_ARG;
    if (tol != tol) return PARARNN_INVALID_ARG;
    if (!aligned(workspace, 256) || !aligned(params, 4) || !aligned(iters, 4)) return PARARNN_INVALID_ARG;
    const size_t esz = dtype == PARARNN_BF16 ? 2 : 4;
    if (!aligned(u, esz) || !aligned(h, esz) || (h0 && !aligned(h0, esz))) return PARARNN_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int status0 = tol < 0.0f ? PARARNN_OK : PARARNN_NOT_CONVERGED;

    if (cell == PARARNN_TANH_DENSE)
        return dense_forward(dtype, params, u, h0, B, L, H, tol, max_iter, h, iters, delta_trace, workspace,
                             workspace_bytes, st);

    int al = align_elems(esz, {u, h, h0});
    const int alp = align_elems(4, {params});
    if (alp < al) al = alp;
    // Fused launches need one carry-record slot per iteration they run; they are used when the
    // workspace holds those: the whole solve when the count is fixed (tol < 0), else its first
    // g_fused_head iterations.
    Layout lo = make_layout(cell, ci, dtype, B, L, H, false, al);
    int n_fused = 0;
    if (g_fused_enabled && max_iter >= 1) {
        const int want = tol < 0.0f ? (max_iter <= kMaxFused ? max_iter : 0)
                                    : (max_iter < g_fused_head ? max_iter : g_fused_head);
        if (want > 0) {
            const Layout lf = make_layout(cell, ci, dtype, B, L, H, false, al, true, want);
            if (workspace_bytes >= (tol < 0.0f ? lf.off_bnd : lf.total)) {
                lo = lf;
                n_fused = want;
            }
        }
    }
    if (n_fused == 0 && workspace_bytes < lo.total) return PARARNN_WORKSPACE_TOO_SMALL;
    char *ws = static_cast<char *>(workspace);
    FwdArgs a;
    memset(&a, 0, sizeof(a));
    a.g = lo.g;
    a.params = params; a.u = u; a.h0 = h0; a.jac = nullptr;
    a.bnd = reinterpret_cast<float *>(ws + lo.off_bnd);
    a.rec = reinterpret_cast<unsigned long long *>(ws + lo.off_rec);
    a.ctrl = reinterpret_cast<Ctrl *>(ws);
    a.iters_out = iters; a.trace = delta_trace;
    a.k = 0; a.max_iter = max_iter; a.tol = tol;
    switch (cell) {
    case PARARNN_GRU_DIAG: return forward_diag<GruDiag>(ci, dtype, lo, a, st, h, status0, max_iter, n_fused);
    case PARARNN_LSTM_DIAG: return forward_diag<LstmDiag>(ci, dtype, lo, a, st, h, status0, max_iter, n_fused);
    case PARARNN_LINEAR_DIAG: return forward_diag<LinearDiag>(ci, dtype, lo, a, st, h, status0, max_iter, n_fused);
    case PARARNN_PARALSTM_DIAG: return forward_diag<ParaLstmDiag>(ci, dtype, lo, a, st, h, status0, max_iter, n_fused);
    }
    return PARARNN_INVALID_ARG;
}

int pararnn_backward(int cell, int dtype, const float *params, const void *u, const void *h0, const void *h,
                     const void *dL_dh, int B, int L, int H, void *dL_du, float *dL_dparams, void *dL_dh0,
                     void *workspace, size_t workspace_bytes, void *hip_stream)
{
    CellInfo ci;
    if (!cell_info(cell, &ci) || (dtype != PARARNN_F32 && dtype != PARARNN_BF16)) return PARARNN_INVALID_ARG;
    if (!dims_ok(B, L, H) || !params || !u || !h || !dL_dh || !dL_du || !dL_dparams || !workspace)
        return PARARNN_INVALID_ARG;
    const size_t esz = dtype == PARARNN_BF16 ? 2 : 4;
    if (!aligned(workspace, 256) || !aligned(params, 4) || !aligned(dL_dparams, 4) || !aligned(u, esz) ||
        !aligned(h, esz) || !aligned(dL_dh, esz) || !aligned(dL_du, esz) || (h0 && !aligned(h0, esz)) ||
        (dL_dh0 && !aligned(dL_dh0, esz)))
        return PARARNN_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (cell == PARARNN_TANH_DENSE)
        return dense_backward(dtype, params, u, h0, h, dL_dh, B, L, H, dL_du, dL_dparams, dL_dh0, workspace,
                              workspace_bytes, st);

    int al = align_elems(esz, {u, h, h0, dL_dh, dL_du, dL_dh0});
    const int alp = align_elems(4, {params, dL_dparams});
    if (alp < al) al = alp;
    const Layout lo = make_layout(cell, ci, dtype, B, L, H, true, al);
    if (workspace_bytes < lo.total) return PARARNN_WORKSPACE_TOO_SMALL;
    char *ws = static_cast<char *>(workspace);
    BwdArgs a;
    memset(&a, 0, sizeof(a));
    a.g = lo.g;
    a.params = params; a.u = u; a.h0 = h0; a.h = h; a.gl = dL_dh; a.jac = nullptr;
    a.du = dL_du; a.dh0 = dL_dh0;
    a.part = reinterpret_cast<float *>(ws + lo.off_part);
    a.rec = reinterpret_cast<unsigned long long *>(ws + lo.off_rec);
    a.ctrl = reinterpret_cast<Ctrl *>(ws);
    switch (cell) {
    case PARARNN_GRU_DIAG: return backward_diag<GruDiag>(ci, dtype, lo, a, st, dL_dparams);
    case PARARNN_LSTM_DIAG: return backward_diag<LstmDiag>(ci, dtype, lo, a, st, dL_dparams);
    case PARARNN_LINEAR_DIAG: return backward_diag<LinearDiag>(ci, dtype, lo, a, st, dL_dparams);
    case PARARNN_PARALSTM_DIAG: return backward_diag<ParaLstmDiag>(ci, dtype, lo, a, st, dL_dparams);
    }
    return PARARNN_INVALID_ARG;
}

}  // extern "C" (reopened below, after the scan helpers)

namespace {

// the scan on its own: kind 0 diagonal, 1..3 blocks of 2x2, 3x3, 4x4
bool scan_kind_ok(int kind) { return kind >= 0 && kind <= 3; }

Layout scan_layout(int kind, int reverse, int B, int L, int H, int al)
{
    const int S = kind + 1;
    const CellInfo ci = {S, S, 0};
    if (S <= 2)
        return make_layout(S == 1 ? PARARNN_GRU_DIAG : PARARNN_LSTM_DIAG, ci, PARARNN_F32, B, L, H, reverse != 0, al);
    // 3x3 and 4x4 blocks keep 12 / 20 floats per step in registers: four steps per thread
    const TileCfg cfg = H <= 8 ? TileCfg{1, 8, 4, 2} : TileCfg{1, 1, 4, 8};
    return make_layout(PARARNN_LSTM_DIAG, ci, PARARNN_F32, B, L, H, reverse != 0, al, false, 1, &cfg);
}

template <int S>
hipError_t scan_launch(const Layout &lo, int reverse, const float *J, const float *r, float *delta, Ctrl *ctrl,
                       unsigned long long *rec, int *scratch_iters, hipStream_t st)
{
    if (!reverse) {
        FwdArgs a;
        memset(&a, 0, sizeof(a));
        a.g = lo.g; a.u = r; a.jac = J; a.hit = delta;
        a.rec = rec; a.ctrl = ctrl;
        a.bnd = nullptr; a.iters_out = scratch_iters; a.trace = nullptr;
        a.k = 1; a.max_iter = 1; a.tol = -1.0f;
        return Kernels<RawScan<S>, float>::newton_iter(lo.cfg, a, false, st);
    }
    BwdArgs a;
    memset(&a, 0, sizeof(a));
    a.g = lo.g; a.gl = r; a.jac = J; a.du = delta; a.dh0 = nullptr; a.part = nullptr;
    a.rec = rec; a.ctrl = ctrl;
    return Kernels<RawScan<S>, float>::backward(lo.cfg, a, st);
}

}  // namespace

extern "C" {

size_t pararnn_affine_scan_workspace_bytes(int kind, int reverse, int B, int L, int H)
{
    if (!scan_kind_ok(kind) || !dims_ok(B, L, H)) return 0;
    size_t need = 0;
    for (int al = 1; al <= 4; al *= 2) {
        const Layout lo = scan_layout(kind, reverse, B, L, H, al);
        if (lo.total > need) need = lo.total;
    }
    return need;
}

int pararnn_affine_scan(int kind, int reverse, const float *J, const float *r, int B, int L, int H, float *delta,
                        void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!scan_kind_ok(kind) || !dims_ok(B, L, H) || !J || !r || !delta || !workspace) return PARARNN_INVALID_ARG;
    if (!aligned(workspace, 256) || !aligned(J, 4) || !aligned(r, 4) || !aligned(delta, 4)) return PARARNN_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int al = align_elems(4, {J, r, delta});
    const Layout lo = scan_layout(kind, reverse, B, L, H, al);
    if (workspace_bytes < lo.total) return PARARNN_WORKSPACE_TOO_SMALL;
    char *ws = static_cast<char *>(workspace);
    Ctrl *ctrl = reinterpret_cast<Ctrl *>(ws);
    unsigned long long *rec = reinterpret_cast<unsigned long long *>(ws + lo.off_rec);
    // a device int[2] for the (unused) iteration result lives in the control block's padding
    int *scratch_iters = reinterpret_cast<int *>(&ctrl->pad[0]);
    hipError_t e = launch_reset(ctrl, rec, lo.n_rec, nullptr, 0, st);
    if (e != hipSuccess) return PARARNN_HIP_ERROR;
    switch (kind) {
    case 0: e = scan_launch<1>(lo, reverse, J, r, delta, ctrl, rec, scratch_iters, st); break;
    case 1: e = scan_launch<2>(lo, reverse, J, r, delta, ctrl, rec, scratch_iters, st); break;
    case 2: e = scan_launch<3>(lo, reverse, J, r, delta, ctrl, rec, scratch_iters, st); break;
    default: e = scan_launch<4>(lo, reverse, J, r, delta, ctrl, rec, scratch_iters, st); break;
    }
    if (e != hipSuccess) return e == hipErrorInvalidValue ? PARARNN_UNSUPPORTED : PARARNN_HIP_ERROR;
    return PARARNN_OK;
}

int pararnn_dense_chunk(void) { return dense_chunk(); }

int pararnn_dense_chunk_products(const float *W, const float *d, int B, int L, int H, float *A, void *workspace,
                                 size_t workspace_bytes, void *hip_stream)
{
    if (!dims_ok(B, L, H) || !W || !d || !A || !workspace) return PARARNN_INVALID_ARG;
    if (!aligned(workspace, 256)) return PARARNN_INVALID_ARG;
    if (workspace_bytes < 256) return PARARNN_WORKSPACE_TOO_SMALL;
    return dense_chunk_products(W, d, B, L, H, A, workspace, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
