// C ABI of the library (see include/pararnn.h) for the built-in cells; the
// cell-generic host driver is driver.h.  No kernel code here.
#include <mutex>
#include <unordered_map>

#include "dense.h"
#include "cells.h"
#include "pararnn/driver.h"
#include "proj.h"

using namespace pararnn;

namespace pararnn {

Settings &settings()
{
    static Settings s = {1, 5, {-1, 0, 0, 0}, kSpinLimit, 1, 1, 0, 0};
    return s;
}

// ---- workspaces the caller has promised to leave alone between calls
namespace {
struct WorkspaceNote {
    unsigned long long sig;    // layout signature of the last call that used the workspace
    unsigned int number;       // that call's number (1 .. 2^20 - 1)
};
std::mutex g_ws_mutex;
std::unordered_map<unsigned long long, WorkspaceNote> g_ws_notes;      // by device and address

unsigned long long ws_key(const void *workspace)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) dev = 0;
    return ((unsigned long long)(unsigned int)dev << 56) ^ (unsigned long long)(uintptr_t)workspace;
}
}  // namespace

unsigned int workspace_epoch(void *workspace, unsigned long long layout_sig, hipStream_t st, bool *fill)
{
    *fill = true;
    const unsigned long long key = ws_key(workspace);
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    const bool capturing = hipStreamIsCapturing(st, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone;
    if (!settings().ws_reuse || capturing) {
        g_ws_notes.erase(key);
        return 0u;
    }
    WorkspaceNote &n = g_ws_notes[key];                // a new note has sig 0, which no call has
    if (n.sig == layout_sig && n.number >= 1u && n.number < (1u << 20) - 1u) {
        ++n.number;
        *fill = false;
    } else {
        n.sig = layout_sig;
        n.number = 1u;
    }
    return n.number << 10;
}

void workspace_forget(void *workspace)
{
    const unsigned long long key = ws_key(workspace);
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    g_ws_notes.erase(key);
}

}  // namespace pararnn

// Scratch of pararnn_forward_noalloc: one copy per GPU the library runs on, held until the process
// ends.  In host code the array's name is only a handle for hipGetSymbolAddress; kernels get the
// device address that call returned.
static __device__ __align__(256) unsigned char scratch[PARARNN_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];    // device address of `scratch` on each device, once looked up

// Device address of the current device's copy of `scratch` (looked up once per device, with that
// device current), or NULL when the runtime refuses.
void *scratch_on_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

bool cell_info(int cell, CellInfo *ci)
{
    switch (cell) {
    case PARARNN_GRU_DIAG: *ci = {3, 1, 6, cell}; return true;
    case PARARNN_LSTM_DIAG: *ci = {4, 2, 8, cell}; return true;
    case PARARNN_TANH_DENSE: *ci = {1, 1, 0, cell}; return true;
    case PARARNN_LINEAR_DIAG: *ci = {1, 1, 2, cell}; return true;
    case PARARNN_PARALSTM_DIAG: *ci = {3, 2, 8, cell}; return true;
    }
    return false;
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

int pararnn_device_info(int *info, int capacity)
{
    static const hipDeviceAttribute_t what[] = {hipDeviceAttributeMultiprocessorCount, hipDeviceAttributeClockRate,
                                                hipDeviceAttributeMemoryClockRate, hipDeviceAttributeMemoryBusWidth,
                                                hipDeviceAttributeL2CacheSize,
                                                hipDeviceAttributeMaxSharedMemoryPerBlock};
    const int n = (int)(sizeof(what) / sizeof(what[0]));
    int dev = 0;
    if (!info || capacity < n) return -1;
    if (hipGetDevice(&dev) != hipSuccess) return -1;
    for (int i = 0; i < n; ++i)
        if (hipDeviceGetAttribute(&info[i], what[i], dev) != hipSuccess) info[i] = -1;
    return n;
}

int pararnn_set_tile(int vec, int ll, int c, int w)
{
    int *ov = settings().tile;
    if (vec == 0) { ov[0] = 0; return PARARNN_OK; }
    bool known = false;
#define PARARNN_CASE(V, LLv, C, W) known = known || (vec == V && ll == LLv && c == C && w == W);
    PARARNN_SHAPES(PARARNN_CASE)
#undef PARARNN_CASE
    if (!known) return PARARNN_UNSUPPORTED;
    ov[0] = vec; ov[1] = ll; ov[2] = c; ov[3] = w;
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
    return diag_workspace_bytes(ci, dtype, B, L, H, backward != 0);
}

size_t pararnn_workspace_bytes_fused(int cell, int dtype, int B, int L, int H, int n_iters)
{
    CellInfo ci;
    if (!cell_info(cell, &ci) || (dtype != PARARNN_F32 && dtype != PARARNN_BF16) || !dims_ok(B, L, H)) return 0;
    if (cell == PARARNN_TANH_DENSE) return dense_workspace_bytes(dtype, B, L, H, 0);
    return diag_workspace_bytes_fused(ci, dtype, B, L, H, n_iters);
}

int pararnn_set_spin_limit(unsigned int polls)
{
    settings().spin_limit = polls ? polls : kSpinLimit;
    return PARARNN_OK;
}

int pararnn_set_staging(int enable)
{
    settings().stage_enabled = enable ? 1 : 0;
    return proj_set_dma(enable);
}

int pararnn_set_streaming(int mode)
{
    if (mode < 0 || mode > 2) return PARARNN_INVALID_ARG;
    settings().streaming = mode;
    return PARARNN_OK;
}

int pararnn_set_fused(int enable)
{
    settings().fused_enabled = enable ? 1 : 0;
    return PARARNN_OK;
}

int pararnn_set_fused_tail(int enable)
{
    settings().fused_tail = enable ? 1 : 0;
    return PARARNN_OK;
}

int pararnn_set_workspace_reuse(int enable)
{
    settings().ws_reuse = enable ? 1 : 0;
    return PARARNN_OK;
}

int pararnn_solve_plan(float tol, int max_iter, int *block_sizes, int capacity)
{
    if (max_iter < 0 || tol != tol || (capacity > 0 && !block_sizes)) return -1;
    const int n_fused = fused_slots_wanted(tol, max_iter);
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
    settings().fused_head = n_iters;
    return PARARNN_OK;
}

}  // extern "C"

namespace {

// options of pararnn_forward_ex -> the driver's choices; false when a field is out of range
bool solve_opts(const pararnn_solve_options_t *o, SolveOpts *out)
{
    *out = default_opts();
    if (!o) return true;
    if (o->first_block < -1 || o->first_block > kMaxFused || o->fused < -1 || o->fused > 1) return false;
    if (o->first_block >= 0) out->fused_head = o->first_block;
    if (o->fused >= 0) out->fused_enabled = o->fused;
    return true;
}

int forward_with(int cell, int dtype, const float *params, const void *u, const void *h0, int B, int L, int H,
                 float tol, int max_iter, void *h, int *iters, float *delta_trace, void *workspace,
                 size_t workspace_bytes, void *hip_stream, const SolveOpts &opts)
{
    CellInfo ci;
    if (!cell_info(cell, &ci)) return PARARNN_INVALID_ARG;
    const int bad = check_forward_args(dtype, params, u, h0, B, L, H, tol, max_iter, h, iters, workspace);
    if (bad != PARARNN_OK) return bad;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
#define PARARNN_FWD(Cell)                                                                                   \
    forward_solve<Cell>(ci, dtype, params, u, h0, B, L, H, tol, max_iter, h, iters, delta_trace, workspace, \
                        workspace_bytes, st, opts)
    switch (cell) {
    case PARARNN_TANH_DENSE:
        workspace_forget(workspace);
        return dense_forward(dtype, params, u, h0, B, L, H, tol, max_iter, h, iters, delta_trace, workspace,
                             workspace_bytes, st);
    case PARARNN_GRU_DIAG: return PARARNN_FWD(GruDiag);
    case PARARNN_LSTM_DIAG: return PARARNN_FWD(LstmDiag);
    case PARARNN_LINEAR_DIAG: return PARARNN_FWD(LinearDiag);
    case PARARNN_PARALSTM_DIAG: return PARARNN_FWD(ParaLstmDiag);
    }
#undef PARARNN_FWD
    return PARARNN_INVALID_ARG;
}

}  // namespace

extern "C" {

int pararnn_forward(int cell, int dtype, const float *params, const void *u, const void *h0, int B, int L,
                    int H, float tol, int max_iter, void *h, int *iters, float *delta_trace, void *workspace,
                    size_t workspace_bytes, void *hip_stream)
{
    return forward_with(cell, dtype, params, u, h0, B, L, H, tol, max_iter, h, iters, delta_trace, workspace,
                        workspace_bytes, hip_stream, default_opts());
}

int pararnn_forward_ex(int cell, int dtype, const float *params, const void *u, const void *h0, int B, int L,
                       int H, float tol, int max_iter, void *h, int *iters, float *delta_trace, void *workspace,
                       size_t workspace_bytes, void *hip_stream, const pararnn_solve_options_t *options)
{
    SolveOpts opts;
    if (!solve_opts(options, &opts)) return PARARNN_INVALID_ARG;
    return forward_with(cell, dtype, params, u, h0, B, L, H, tol, max_iter, h, iters, delta_trace, workspace,
                        workspace_bytes, hip_stream, opts);
}

size_t pararnn_workspace_bytes_ex(int cell, int dtype, int B, int L, int H, const pararnn_solve_options_t *options)
{
    CellInfo ci;
    SolveOpts opts;
    if (!cell_info(cell, &ci) || (dtype != PARARNN_F32 && dtype != PARARNN_BF16) || !dims_ok(B, L, H)) return 0;
    if (!solve_opts(options, &opts)) return 0;
    if (cell == PARARNN_TANH_DENSE) return dense_workspace_bytes(dtype, B, L, H, 0);
    return diag_workspace_bytes(ci, dtype, B, L, H, false, opts);
}

int pararnn_solve_plan_ex(float tol, int max_iter, const pararnn_solve_options_t *options, int *block_sizes, int capacity)
{
    SolveOpts opts;
    if (max_iter < 0 || tol != tol || (capacity > 0 && !block_sizes) || !solve_opts(options, &opts)) return -1;
    const int n_fused = fused_slots_wanted(tol, max_iter, opts);
    int done = 0, launches = 0;
    for (; done < max_iter; ++launches) {
        const int K = next_block_size(done, launches, max_iter, n_fused);
        if (launches < capacity) block_sizes[launches] = K;
        done += K;
    }
    return launches;
}

int pararnn_forward_noalloc(int cell, int dtype, const float *params, const void *u, const void *h0, int B, int L,
                            int H, float tol, int max_iter, void *h, int *iters, float *delta_trace,
                            void *hip_stream)
{
    void *ptr = scratch_on_current_device();
    if (!ptr) return PARARNN_HIP_ERROR;
    // the same solve as pararnn_forward with the static array as its workspace: the launch sequence
    // clears what must start at zero (control block, carry records) with a kernel of its own, and a
    // problem whose smallest workspace exceeds the array is refused with WORKSPACE_TOO_SMALL
    return pararnn_forward(cell, dtype, params, u, h0, B, L, H, tol, max_iter, h, iters, delta_trace, ptr,
                           (size_t)PARARNN_NOALLOC_SCRATCH_BYTES, hip_stream);
}

int pararnn_backward(int cell, int dtype, const float *params, const void *u, const void *h0, const void *h,
                     const void *dL_dh, int B, int L, int H, void *dL_du, float *dL_dparams, void *dL_dh0,
                     void *workspace, size_t workspace_bytes, void *hip_stream)
{
    CellInfo ci;
    if (!cell_info(cell, &ci)) return PARARNN_INVALID_ARG;
    const int bad = check_backward_args(dtype, params, u, h0, h, dL_dh, B, L, H, dL_du, dL_dparams, dL_dh0, workspace);
    if (bad != PARARNN_OK) return bad;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
#define PARARNN_BWD(Cell)                                                                                  \
    backward_pass<Cell>(ci, dtype, params, u, h0, h, dL_dh, B, L, H, dL_du, dL_dparams, dL_dh0, workspace, \
                        workspace_bytes, st)
    switch (cell) {
    case PARARNN_TANH_DENSE:
        workspace_forget(workspace);
        return dense_backward(dtype, params, u, h0, h, dL_dh, B, L, H, dL_du, dL_dparams, dL_dh0, workspace,
                              workspace_bytes, st);
    case PARARNN_GRU_DIAG: return PARARNN_BWD(GruDiag);
    case PARARNN_LSTM_DIAG: return PARARNN_BWD(LstmDiag);
    case PARARNN_LINEAR_DIAG: return PARARNN_BWD(LinearDiag);
    case PARARNN_PARALSTM_DIAG: return PARARNN_BWD(ParaLstmDiag);
    }
#undef PARARNN_BWD
    return PARARNN_INVALID_ARG;
}

int pararnn_residual_norm(int cell, int dtype, const float *params, const void *u, const void *h0, const void *h,
                          int B, int L, int H, float *out, void *hip_stream)
{
    CellInfo ci;
    if (!cell_info(cell, &ci)) return PARARNN_INVALID_ARG;
    const int bad = check_residual_args(dtype, params, u, h0, h, B, L, H, out);
    if (bad != PARARNN_OK) return bad;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
#define PARARNN_RES(Cell) residual_norm_diag<Cell>(dtype, params, u, h0, h, B, L, H, out, st)
    switch (cell) {
    case PARARNN_TANH_DENSE: return dense_residual_norm(dtype, params, u, h0, h, B, L, H, out, st);
    case PARARNN_GRU_DIAG: return PARARNN_RES(GruDiag);
    case PARARNN_LSTM_DIAG: return PARARNN_RES(LstmDiag);
    case PARARNN_LINEAR_DIAG: return PARARNN_RES(LinearDiag);
    case PARARNN_PARALSTM_DIAG: return PARARNN_RES(ParaLstmDiag);
    }
#undef PARARNN_RES
    return PARARNN_INVALID_ARG;
}

}  // extern "C" (reopened below, after the scan helpers)

namespace {

// the scan on its own: kind 0 diagonal, 1..3 blocks of 2x2, 3x3, 4x4
bool scan_kind_ok(int kind) { return kind >= 0 && kind <= 3; }

Layout scan_layout(int kind, int reverse, int B, int L, int H, int al)
{
    const int S = kind + 1;
    const CellInfo ci = {S, S, 0, -1};
    if (S <= 2) return make_layout(ci, PARARNN_F32, B, L, H, reverse != 0, al);
    // 3x3 and 4x4 blocks keep 12 / 20 floats per step in registers: four steps per thread
    const TileCfg cfg = H <= 8 ? TileCfg{1, 8, 4, 2} : TileCfg{1, 1, 4, 8};
    return make_layout(ci, PARARNN_F32, B, L, H, reverse != 0, al, false, 1, &cfg);
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
    workspace_forget(workspace);
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

size_t pararnn_input_projection_workspace_bytes(int dtype, int B, int L, int H, int G, int n_heads, int backward)
{
    return proj_workspace_bytes(dtype, B, L, H, G, n_heads, backward);
}

int pararnn_input_projection(int dtype, const void *x, const float *Wx, const float *bias, int B, int L, int H,
                             int G, int n_heads, void *u, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!x || !Wx || !u || !workspace || !aligned(workspace, 256)) return PARARNN_INVALID_ARG;
    workspace_forget(workspace);
    return proj_forward(dtype, x, Wx, bias, B, L, H, G, n_heads, u, workspace, workspace_bytes,
                        static_cast<hipStream_t>(hip_stream));
}

int pararnn_input_projection_backward(int dtype, const void *x, const float *Wx, const void *du, int B, int L,
                                      int H, int G, int n_heads, void *dx, float *dWx, float *dbias,
                                      void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!x || !Wx || !du || !workspace || !aligned(workspace, 256) || (dbias && !dWx)) return PARARNN_INVALID_ARG;
    workspace_forget(workspace);
    return proj_backward(dtype, x, Wx, du, B, L, H, G, n_heads, dx, dWx, dbias, workspace, workspace_bytes,
                         static_cast<hipStream_t>(hip_stream));
}

int pararnn_dense_chunk(void) { return dense_chunk(); }

int pararnn_set_dense_products(int mode) { return dense_set_products(mode); }

int pararnn_set_dense_jacobian(int mode) { return dense_set_jacobian(mode); }

int pararnn_set_dense_tail(int mode) { return dense_set_one_launch(mode); }

int pararnn_dense_chunk_products(const float *W, const float *d, int B, int L, int H, float *A, void *workspace,
                                 size_t workspace_bytes, void *hip_stream)
{
    if (!dims_ok(B, L, H) || !W || !d || !A || !workspace) return PARARNN_INVALID_ARG;
    if (!aligned(workspace, 256)) return PARARNN_INVALID_ARG;
    if (workspace_bytes < 256) return PARARNN_WORKSPACE_TOO_SMALL;
    workspace_forget(workspace);
    return dense_chunk_products(W, d, B, L, H, A, workspace, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
