// Host-side driver of the diagonal / small-block paths, generic in the cell:
// argument checks, workspace layout, tile-shape choice and the enqueue
// sequence of a forward solve (Sec. 2, Alg. 1a) and of a backward pass (Eq. (6)).
// Used by the C ABI of the built-in cells and by libraries that add a cell of
// their own (pararnn_cell.h).  No kernel code here.
#pragma once
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <initializer_list>

#include "../pararnn.h"
#include "launch.h"

namespace pararnn {

// G gate pre-activations per step, S state values per channel, PR parameter rows of H floats;
// kind is the PARARNN_* constant of a built-in cell, -1 for any other cell
struct CellInfo { int G, S, PR, kind; };

// Process-wide settings of the library (pararnn_set_fused, pararnn_set_fused_head,
// pararnn_set_tile); one instance, owned by libpararnn.so.
struct Settings {
    int fused_enabled;     // launches that run several Newton iterations are allowed
    int fused_head;        // iterations in the first launch of a solve to a tolerance (0 = none)
    int tile[4];           // tile-shape override {vec, ll, c, w}; vec = 0 none, -1 not yet read from the environment
    unsigned int spin_limit;   // polls of one predecessor before a tile gives up (pararnn_set_spin_limit)
    int stage_enabled;         // kernels that copy their inputs straight into LDS are allowed (pararnn_set_staging)
    int fused_tail;            // the blocks after a solve's first launch share one persistent launch (pararnn_set_fused_tail)
    int ws_reuse;              // the caller promises that nothing else writes to a workspace between calls (pararnn_set_workspace_reuse)
    int streaming;             // streamed accesses of the HBM-bound kernels: 0 chosen by size, 1 never, 2 always (pararnn_set_streaming)
};
Settings &settings();

// Choices of one forward solve.  The C ABI's plain entry points take them from the process-wide
// settings; pararnn_forward_ex takes them from its options argument, so that two threads with
// different wishes do not meet in the settings.
struct SolveOpts {
    int fused_enabled;     // launches that run several Newton iterations are allowed
    int fused_head;        // iterations in the first launch of a solve to a tolerance (0 = none)
};
inline SolveOpts default_opts()
{
    const Settings &s = settings();
    return {s.fused_enabled, s.fused_head};
}

inline size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }

// The memory-side cache of the device (256 MiB) keeps what a launch wrote or read for the next one when
// it is left room.  A per-iteration launch reads u and reads and rewrites the fp32 iterate: u is
// streamed as soon as the two together exceed that cache (the iterate then has it to itself: measured
// 8 % on 0.8 GB of u with a 0.27 GB iterate), the iterate too once it is larger than twice the cache,
// where nothing of it survives until the next launch and streamed accesses are the faster ones (3 %).
constexpr size_t kMemCacheBytes = (size_t)256 << 20;
inline int forward_stream_level(size_t u_bytes, size_t iterate_bytes)
{
    const int mode = settings().streaming;
    if (mode == 1) return 0;
    if (mode == 2) return 2;
    if (iterate_bytes > 2 * kMemCacheBytes) return 2;
    return u_bytes + iterate_bytes > kMemCacheBytes ? 1 : 0;
}
// The backward kernel for bf16 storage reads and writes every byte once: streamed when its tensors
// together exceed twice the cache (4 % on 17 GB).  The fp32 kernels gain nothing either way (measured).
inline int backward_stream(size_t bytes)
{
    const int mode = settings().streaming;
    if (mode == 1) return 0;
    if (mode == 2) return 1;
    return bytes > 2 * kMemCacheBytes ? 1 : 0;
}

// Tile shape for a problem.  The table is the result of sweeps on MI355X over
// the compiled shapes (fp32 and bf16 storage, forward and backward, GRU and
// LSTM at 2^25..2^30 timestep-channels): one channel per lane
// with 128..256-byte row segments and 64..128 steps per tile.
// PARARNN_TILE="vec,ll,c,w" or pararnn_set_tile() overrides it (tuning aid; the
// combination must be one that is compiled in and allowed by H and alignment).
inline TileCfg choose_tile(const CellInfo &ci, int dtype, bool backward, int H, int align_elems, bool fused = false)
{
    int vmax = 1;
    if (H % 4 == 0 && align_elems >= 4) vmax = 4;
    else if (H % 2 == 0 && align_elems >= 2) vmax = 2;
    TileCfg cfg = {1, 2, 8, 8};                          // 32 channels x 128 steps
    const bool lstm = ci.S >= 2, bf = dtype == PARARNN_BF16;
    if (H <= 8) {
        cfg = {1, 8, 4, 2};                              // 8 channels x 64 steps
    } else if (ci.S >= 4) {
        // 4x4 blocks: 20 prefix values per step; four steps per thread (a few registers spill in the
        // fused and backward kernels, the next larger shape spills a hundred)
        cfg = {1, 1, 4, 8};                              // 64 channels x 32 steps
    } else if (ci.S == 3) {
        // 3x3 blocks: a step keeps S*S + S prefix values in registers; eight steps per thread is the
        // most that fits without spilling (190-230 registers, two waves per SIMD) and measured
        // fastest forward, fused and backward alike
        cfg = {1, 1, 8, 8};                              // 64 channels x 64 steps
    } else if (H <= 32) {
        cfg = {1, 2, 8, 8};
    } else if (fused) {
        // the fused blocks are bound by vector arithmetic, not by HBM: long per-thread chunks spread the
        // per-thread cost of the wave / workgroup / look-back levels over more cell evaluations
        if (lstm) cfg = {1, 1, 16, 4};                   // 64 channels x 64 steps
        else cfg = {1, 1, 12, 8};                        // 64 channels x 96 steps
    } else if (!backward) {
        if (lstm) cfg = {1, 1, 8, 16};                   // 64 channels x 128 steps
        else if (bf) cfg = {1, 1, 16, 8};                // 64 channels x 128 steps (3 % faster than two channels per lane on config 5)
        else cfg = {1, 1, 8, 16};                        // 64 channels x 128 steps
    } else {
        if (ci.kind == PARARNN_PARALSTM_DIAG) cfg = {1, 1, 12, 8};   // 64 channels x 96 steps
        else if (lstm && !bf) cfg = {1, 2, 8, 8};        // 32 channels x 128 steps (3 % faster than 64 x 128 on config 3)
        else if (lstm) cfg = {1, 1, 16, 8};              // 64 channels x 128 steps
        else if (bf) cfg = {1, 1, 8, 8};                 // 64 channels x 64 steps
        else cfg = {1, 1, 8, 16};                        // 64 channels x 128 steps (3-4 % faster than 32 x 256 on config 2)
    }
    int *ov = settings().tile;
    if (ov[0] == -1) {
        ov[0] = 0;
        const char *e = getenv("PARARNN_TILE");
        int v, l, c, w;
        if (e && sscanf(e, "%d,%d,%d,%d", &v, &l, &c, &w) == 4) {
            ov[0] = v; ov[1] = l; ov[2] = c; ov[3] = w;
        }
    }
    if (ov[0] > 0 && ov[0] <= vmax) {
        cfg.vec = ov[0]; cfg.ll = ov[1]; cfg.c = ov[2]; cfg.w = ov[3];
    }
    return cfg;
}

struct Layout {
    ScanGeom g;
    TileCfg cfg;
    size_t off_rec, n_rec, off_bnd, off_iter, off_part, total;
};

// What decides where a call's carry records lie and how they are read: two calls with the same
// signature on the same workspace use every record word for the same thing.  Never 0.
inline unsigned long long layout_signature(int pass, const CellInfo &ci, int dtype, const Layout &lo, int rec_slots)
{
    unsigned long long h = 1469598103934665603ull;
    const long long v[] = {pass, ci.kind, ci.S, ci.G, ci.PR, dtype, lo.g.B, lo.g.L, lo.g.H, lo.g.T, lo.g.n_lt, lo.g.n_cg,
                           lo.cfg.vec, lo.cfg.ll, lo.cfg.c, lo.cfg.w, rec_slots, (long long)lo.n_rec,
                           (long long)lo.off_rec, (long long)lo.total};
    for (long long x : v) {
        for (int i = 0; i < 8; ++i) {
            h ^= (unsigned long long)(x >> (8 * i)) & 0xffull;
            h *= 1099511628211ull;
        }
    }
    return h ? h : 1ull;
}

// largest max_iter whose epochs fit below the per-call number in a record tag (tag = epoch * 4 + state,
// epoch = number * 1024 + iteration)
constexpr int kMaxIterWithReuse = 1000;

// Workspace: [Ctrl | carry records (rec_slots sets) | boundary rows | fp32 iterate (bf16 forward) |
// parameter-gradient partials (backward)]
inline Layout make_layout(const CellInfo &ci, int dtype, int B, int L, int H, bool backward, int align_elems,
                          bool fused = false, int rec_slots = 1, const TileCfg *force = nullptr)
{
    Layout lo;
    lo.cfg = force ? *force : choose_tile(ci, dtype, backward, H, align_elems, fused);
    const int CW = (kWave / lo.cfg.ll) * lo.cfg.vec, T = lo.cfg.c * lo.cfg.ll * lo.cfg.w;
    ScanGeom &g = lo.g;
    g.B = B; g.L = L; g.H = H; g.T = T;
    g.n_lt = (L + T - 1) / T;
    g.n_cg = (H + CW - 1) / CW;
    g.n_groups = B * g.n_cg;
    g.n_tiles = g.n_groups * g.n_lt;
    g.spin_limit = settings().spin_limit;
    g.epoch_base = 0;
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

inline bool dims_ok(int B, int L, int H)
{
    if (B < 1 || L < 1 || H < 1) return false;
    // keep every element count inside size_t/int ranges the kernels assume.  The bound on H keeps the
    // 32-bit byte offsets of the buffer instructions in range: a wave addresses up to 128 rows of H
    // elements of 4 bytes from its base (8 segments x 4 steps x 4 gates, or 2 x 16 x 4)
    const double n = (double)B * (double)L * (double)H;
    return n < 3.0e10 && (double)B * H < 2.0e9 && L < (1 << 30) && H <= (1 << 22);
}

inline bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }

// widest vector (in elements of size esz: 4, 2 or 1) every pointer in the list allows; NULL allows any
inline int align_elems(size_t esz, std::initializer_list<const void *> ptrs)
{
    int a = 4;
    for (const void *p : ptrs) {
        if (!p) continue;
        const int here = aligned(p, 4 * esz) ? 4 : aligned(p, 2 * esz) ? 2 : 1;
        if (here < a) a = here;
    }
    return a;
}

// Carry-record slots a solve would like to have: the whole solve when the count is fixed
// (tol < 0) and short enough, else its first fused_head iterations; 0 = no fused launches.
inline int fused_slots_wanted(float tol, int max_iter, const SolveOpts &s = default_opts())
{
    if (!s.fused_enabled || max_iter < 1) return 0;
    if (tol < 0.0f) return max_iter <= kMaxFused ? max_iter : 0;
    return max_iter < s.fused_head ? max_iter : s.fused_head;
}

// Workspace size of a forward solve to a tolerance (or of a backward pass); does not depend on
// pointer alignment: the larger footprint is taken when the layouts differ.
inline size_t diag_workspace_bytes(const CellInfo &ci, int dtype, int B, int L, int H, bool backward,
                                   const SolveOpts &s = default_opts())
{
    size_t need = 0;
    for (int al = 1; al <= 4; al *= 2) {
        const Layout lo = make_layout(ci, dtype, B, L, H, backward, al);
        if (lo.total > need) need = lo.total;
        if (!backward && s.fused_enabled && s.fused_head > 0) {
            const Layout lf = make_layout(ci, dtype, B, L, H, false, al, true, s.fused_head);
            if (lf.total > need) need = lf.total;
        }
    }
    return need;
}

// Workspace size of a fixed-count solve of n_iters iterations in one launch.
inline size_t diag_workspace_bytes_fused(const CellInfo &ci, int dtype, int B, int L, int H, int n_iters)
{
    size_t need = diag_workspace_bytes(ci, dtype, B, L, H, false);
    if (n_iters < 1 || n_iters > kMaxFused) return need;
    for (int al = 1; al <= 4; al *= 2) {
        const Layout lf = make_layout(ci, dtype, B, L, H, false, al, true, n_iters);
        if (lf.off_bnd > need) need = lf.off_bnd;
    }
    return need;
}

// n_fused = number of carry-record slots the workspace holds (0: none; fused launches are not used).
// tol < 0: the whole fixed-count solve is one fused launch of n_fused = max_iter iterations.
// tol >= 0: the solve is a sequence of launches, each checked by the stopping test on the
// device: a fused block of n_fused iterations from the initial guess, then blocks of 1, 2,
// 4, ... (at most n_fused) iterations from the iterate; a block of one iteration that is a
// launch of its own is the per-iteration kernel.  With `tail` the blocks after the second share
// ONE launch of the fused kernel, which returns at once when the tolerance was met before;
// without it every block is a launch of its own.  Launches after the one that met the
// tolerance return at once.
template <class Cell>
int forward_diag(const CellInfo &ci, int dtype, const Layout &lo, FwdArgs &a, hipStream_t st, void *h,
                 int status0, int max_iter, int n_fused)
{
    char *ws = reinterpret_cast<char *>(a.ctrl);
    const bool bf = dtype == PARARNN_BF16;
    const bool to_tol = a.tol >= 0.0f;
    hipError_t e;
    a.hit = bf ? reinterpret_cast<float *>(ws + lo.off_iter) : static_cast<float *>(h);
    const int slots = n_fused > 0 ? n_fused : 1;
    bool fill = true;
    if (max_iter <= kMaxIterWithReuse) a.g.epoch_base = workspace_epoch(ws, layout_signature(0, ci, dtype, lo, slots), st, &fill);
    else workspace_forget(ws);
    e = launch_reset(a.ctrl, a.rec, fill ? lo.n_rec * (size_t)slots : 0, a.iters_out, status0, st);
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
    f.n_slots = n_fused; f.spin_limit = settings().spin_limit;
    const bool tail = settings().fused_tail != 0;
    int done = 0, cur = 0;
    for (int launches = 0; done < max_iter; ++launches) {
        const int K = next_block_size(done, launches, max_iter, n_fused);
        if (to_tol && n_fused > 0 && launches == 2 && tail) {
            // everything after the second block in one launch that goes through the plan on the device (the
            // second block is one iteration, which the per-iteration kernel does faster than a fused block)
            f.n_iters = K; f.k0 = done; f.epoch0 = f.g.epoch_base + (unsigned int)done; f.bnd_cur = cur; f.tail = 1; f.launch_no = launches;
            e = bf ? Kernels<Cell, unsigned short>::newton_fused(lo.cfg, f, st) : Kernels<Cell, float>::newton_fused(lo.cfg, f, st);
            if (e != hipSuccess) return e == hipErrorInvalidValue ? PARARNN_UNSUPPORTED : PARARNN_HIP_ERROR;
            break;
        }
        if (n_fused > 0 && (K > 1 || done == 0)) {
            f.n_iters = K; f.k0 = done; f.epoch0 = f.g.epoch_base + (unsigned int)done; f.bnd_cur = cur; f.tail = 0; f.launch_no = launches;
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
    bool fill = true;
    a.g.epoch_base = workspace_epoch(a.ctrl, layout_signature(1, ci, dtype, lo, 1), st, &fill);
    hipError_t e = launch_reset(a.ctrl, a.rec, fill ? lo.n_rec : 0, nullptr, 0, st);
    if (e != hipSuccess) return PARARNN_HIP_ERROR;
    e = dtype == PARARNN_BF16 ? Kernels<Cell, unsigned short>::backward(lo.cfg, a, st)
                              : Kernels<Cell, float>::backward(lo.cfg, a, st);
    if (e != hipSuccess) return e == hipErrorInvalidValue ? PARARNN_UNSUPPORTED : PARARNN_HIP_ERROR;
    e = launch_param_reduce(a.part, dparams, lo.g.n_lt * lo.g.B, ci.PR * lo.g.H, st);
    return e == hipSuccess ? PARARNN_OK : PARARNN_HIP_ERROR;
}

// Argument checks shared by every forward entry point; PARARNN_OK or the status to return.
inline int check_forward_args(int dtype, const float *params, const void *u, const void *h0, int B, int L, int H,
                              float tol, int max_iter, void *h, int *iters, void *workspace)
{
    if (dtype != PARARNN_F32 && dtype != PARARNN_BF16) return PARARNN_INVALID_ARG;
    if (!dims_ok(B, L, H) || max_iter < 0 || !params || !u || !h || !iters || !workspace) return PARARNN_INVALID_ARG;
    if (tol != tol) return PARARNN_INVALID_ARG;
    if (!aligned(workspace, 256) || !aligned(params, 4) || !aligned(iters, 4)) return PARARNN_INVALID_ARG;
    const size_t esz = dtype == PARARNN_BF16 ? 2 : 4;
    if (!aligned(u, esz) || !aligned(h, esz) || (h0 && !aligned(h0, esz))) return PARARNN_INVALID_ARG;
    return PARARNN_OK;
}

inline int check_backward_args(int dtype, const float *params, const void *u, const void *h0, const void *h,
                               const void *dL_dh, int B, int L, int H, void *dL_du, float *dL_dparams, void *dL_dh0,
                               void *workspace)
{
    if (dtype != PARARNN_F32 && dtype != PARARNN_BF16) return PARARNN_INVALID_ARG;
    if (!dims_ok(B, L, H) || !params || !u || !h || !dL_dh || !dL_du || !dL_dparams || !workspace)
        return PARARNN_INVALID_ARG;
    const size_t esz = dtype == PARARNN_BF16 ? 2 : 4;
    if (!aligned(workspace, 256) || !aligned(params, 4) || !aligned(dL_dparams, 4) || !aligned(u, esz) ||
        !aligned(h, esz) || !aligned(dL_dh, esz) || !aligned(dL_du, esz) || (h0 && !aligned(h0, esz)) ||
        (dL_dh0 && !aligned(dL_dh0, esz)))
        return PARARNN_INVALID_ARG;
    return PARARNN_OK;
}

// A forward solve with checked arguments: layout, then the launches.
template <class Cell>
int forward_solve(const CellInfo &ci, int dtype, const float *params, const void *u, const void *h0, int B, int L,
                  int H, float tol, int max_iter, void *h, int *iters, float *delta_trace, void *workspace,
                  size_t workspace_bytes, hipStream_t st, const SolveOpts &opts = default_opts())
{
    const size_t esz = dtype == PARARNN_BF16 ? 2 : 4;
    const int status0 = tol < 0.0f ? PARARNN_OK : PARARNN_NOT_CONVERGED;
    int al = align_elems(esz, {u, h, h0});
    const int alp = align_elems(4, {params});
    if (alp < al) al = alp;
    // Fused launches need one carry-record slot per iteration they run; they are used when the
    // workspace holds those.
    Layout lo = make_layout(ci, dtype, B, L, H, false, al);
    int n_fused = 0;
    const int want = fused_slots_wanted(tol, max_iter, opts);
    if (want > 0) {
        const Layout lf = make_layout(ci, dtype, B, L, H, false, al, true, want);
        if (workspace_bytes >= (tol < 0.0f ? lf.off_bnd : lf.total)) {
            lo = lf;
            n_fused = want;
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
    {
        const size_t n = (size_t)B * L * H, esz = dtype == PARARNN_BF16 ? 2 : 4;
        a.stream = forward_stream_level(n * ci.G * esz, n * ci.S * sizeof(float));
    }
    const int rc = forward_diag<Cell>(ci, dtype, lo, a, st, h, status0, max_iter, n_fused);
    if (rc != PARARNN_OK) workspace_forget(workspace);
    return rc;
}

// Residual max-norm of given states (App. A); out is a device float.
inline int check_residual_args(int dtype, const float *params, const void *u, const void *h0, const void *h, int B,
                               int L, int H, float *out)
{
    if (dtype != PARARNN_F32 && dtype != PARARNN_BF16) return PARARNN_INVALID_ARG;
    if (!dims_ok(B, L, H) || !params || !u || !h || !out) return PARARNN_INVALID_ARG;
    const size_t esz = dtype == PARARNN_BF16 ? 2 : 4;
    if (!aligned(params, 4) || !aligned(out, 4) || !aligned(u, esz) || !aligned(h, esz) || (h0 && !aligned(h0, esz)))
        return PARARNN_INVALID_ARG;
    return PARARNN_OK;
}

template <class Cell>
int residual_norm_diag(int dtype, const float *params, const void *u, const void *h0, const void *h, int B, int L,
                       int H, float *out, hipStream_t st)
{
    const size_t esz = dtype == PARARNN_BF16 ? 2 : 4;
    int al = align_elems(esz, {u, h, h0});
    const int alp = align_elems(4, {params});
    if (alp < al) al = alp;
    const int vec = (H % 4 == 0 && al >= 4) ? 4 : (H % 2 == 0 && al >= 2) ? 2 : 1;
    ResArgs a;
    memset(&a, 0, sizeof(a));
    a.B = B; a.L = L; a.H = H;
    a.params = params; a.u = u; a.h0 = h0; a.h = h;
    a.out = reinterpret_cast<unsigned int *>(out);
    if (launch_zero_words(a.out, 1, st) != hipSuccess) return PARARNN_HIP_ERROR;
    const hipError_t e = dtype == PARARNN_BF16 ? Kernels<Cell, unsigned short>::residual_norm(vec, a, st)
                                               : Kernels<Cell, float>::residual_norm(vec, a, st);
    return e == hipSuccess ? PARARNN_OK : PARARNN_HIP_ERROR;
}

// A backward pass with checked arguments.
template <class Cell>
int backward_pass(const CellInfo &ci, int dtype, const float *params, const void *u, const void *h0, const void *h,
                  const void *dL_dh, int B, int L, int H, void *dL_du, float *dL_dparams, void *dL_dh0,
                  void *workspace, size_t workspace_bytes, hipStream_t st)
{
    const size_t esz = dtype == PARARNN_BF16 ? 2 : 4;
    int al = align_elems(esz, {u, h, h0, dL_dh, dL_du, dL_dh0});
    const int alp = align_elems(4, {params, dL_dparams});
    if (alp < al) al = alp;
    const Layout lo = make_layout(ci, dtype, B, L, H, true, al);
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
    // rows that the kernel may copy straight into LDS, 16 bytes per lane: bf16 rows that start on 16-byte
    // boundaries, and row offsets that stay inside the 32-bit range of a buffer instruction
    a.stage = settings().stage_enabled && dtype == PARARNN_BF16 && H % 8 == 0 && aligned(u, 16) && aligned(h, 16) &&
              aligned(dL_dh, 16) && (double)H * 2.0 * (16.0 * ci.G) < 4.0e9;
    a.stream = dtype == PARARNN_BF16 ? backward_stream((size_t)B * L * H * 2 * (2 * ci.G + 2 * ci.S)) : 0;
    const int rc = backward_diag<Cell>(ci, dtype, lo, a, st, dL_dparams);
    if (rc != PARARNN_OK) workspace_forget(workspace);
    return rc;
}

}  // namespace pararnn
