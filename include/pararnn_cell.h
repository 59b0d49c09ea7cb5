/*
 * pararnn_cell.h - adding a recurrent cell of your own (HIP C++, gfx950).
 *
 * The paper's framework lets a user define a new cell by its recurrence step
 * and its Jacobian and then reuses the Newton solver and the parallel
 * reduction unchanged (App. D.3: the recurrence-step and Jacobian hooks of the
 * cell implementation class).  This header is that hook for this library: a
 * cell is a struct of four per-channel device functions; PARARNN_DEFINE_CELL
 * instantiates every kernel of the diagonal / small-block path for it (fused
 * Newton blocks, per-iteration kernel, backward scan, fp32 and bf16 storage)
 * and emits a C ABI with the same argument lists as pararnn_forward /
 * pararnn_backward of pararnn.h, minus the `cell` argument.
 *
 * A cell struct provides
 *
 *     static constexpr int G;    gate pre-activations per step and channel: u is [B][L][G][H]
 *     static constexpr int S;    state values per channel (1: diagonal Jacobian; 2, 3, 4: blocks of that size)
 *     static constexpr int P;    parameter rows: params is [P][H] fp32
 *     static constexpr int NC;   coefficients handed from bwd_prep to bwd_emit
 *
 *     // Eq. (1): F[S] = f(hp[S], u[G]) for one channel; p[P] are that channel's parameters
 *     __device__ static void step(const float *p, const float *hp, const float *u, float *F);
 *     // the same F plus J[S*S] = dF/dhp, row-major: J[a*S+b] = dF_a/dhp_b   (the J_l of Eq. (3))
 *     __device__ static void step_and_jacobian(const float *p, const float *hp, const float *u,
 *                                              float *F, float *J);
 *     // backward, Eq. (6): J as above and NC numbers k[] of the cell's choosing ...
 *     __device__ static void bwd_prep(const float *p, const float *hp, const float *u, float *J, float *k);
 *     // ... from which, given lam[S] = dL/dF, du[G] = (dF/du)^T lam is written and
 *     // (dF/dp_i)^T lam is ADDED to acc[i] for each of the P parameters
 *     __device__ static void bwd_emit(const float *k, const float *lam, float *du, float *acc);
 *
 * All four are called once per (timestep, channel); they must be pure functions
 * of their arguments.  Build the file that holds the cell and the macro with
 * `python -m paper_2510_21450_amd.build --cell my_cell.hip -o libmy_cell.so`
 * (same compiler flags as the library, linked against libpararnn.so, which
 * supplies the cell-independent kernels and the process-wide settings).
 *
 * PARARNN_DEFINE_CELL(Cell, name) exports (all host functions; pointers as in pararnn.h):
 *     int    name_gates(void), name_state(void), name_param_rows(void);
 *     size_t name_workspace_bytes(int dtype, int B, int L, int H, int backward);
 *     size_t name_workspace_bytes_fused(int dtype, int B, int L, int H, int n_iters);
 *     int    name_forward(int dtype, params, u, h0, B, L, H, tol, max_iter, h, iters, delta_trace,
 *                         workspace, workspace_bytes, hip_stream);
 *     int    name_backward(int dtype, params, u, h0, h, dL_dh, B, L, H, dL_du, dL_dparams, dL_dh0,
 *                          workspace, workspace_bytes, hip_stream);
 *     int    name_residual_norm(int dtype, params, u, h0, h, B, L, H, out, hip_stream);
 * with the semantics, status codes and error behaviour of the pararnn_* functions
 * of the same name.
 *
 * Tile shapes: the automatic choice depends on S.  For S = 3 (4) only the shapes with one channel
 * per lane and at most 8 (4) timesteps per thread are instantiated (larger ones would keep more
 * prefix values per thread than the register file holds); a shape forced with pararnn_set_tile
 * outside them makes the call return PARARNN_UNSUPPORTED.
 */
#ifndef PARARNN_CELL_H
#define PARARNN_CELL_H

#include "pararnn/driver.h"
#include "pararnn/launch_impl.h"

namespace pararnn {

// Presents a cell written to the four-function contract above to the kernels.  The kernels'
// optional pre-scaled ("folded") gate arithmetic is not used: u and the parameters reach the
// cell unchanged.
template <class Impl> struct UserCell {
    static_assert(Impl::S >= 1 && Impl::S <= 4, "state values per channel: 1 to 4");
    static_assert(Impl::G >= 1 && Impl::P >= 1 && Impl::NC >= 1, "G, P and NC must be positive");
    static constexpr int G = Impl::G, S = Impl::S, PR = Impl::P, NC = Impl::NC, PQ = 0;

    __device__ __forceinline__ static void fold_params(const float *, float *) {}
    __device__ __forceinline__ static void fold_u(const float *, float *) {}

    template <bool FOLD = false>
    __device__ __forceinline__ static void step(const float *p, const float *hp, const float *u, float *F,
                                                const float * = nullptr)
    {
        Impl::step(p, hp, u, F);
    }
    template <bool FOLD = false>
    __device__ __forceinline__ static void fwd(const float *p, const float *hp, const float *u, float *F, float *J,
                                               const float * = nullptr)
    {
        Impl::step_and_jacobian(p, hp, u, F, J);
    }
    __device__ __forceinline__ static void bwd_prep(const float *p, const float *hp, const float *u, float *J,
                                                    float *k)
    {
        Impl::bwd_prep(p, hp, u, J, k);
    }
    __device__ __forceinline__ static void bwd_emit(const float *k, const float *lam, float *du, float *acc)
    {
        Impl::bwd_emit(k, lam, du, acc);
    }
};

}  // namespace pararnn

#define PARARNN_DEFINE_CELL(Impl, name)                                                                           \
    namespace pararnn {                                                                                           \
    template struct Kernels<UserCell<Impl>, float>;                                                               \
    template struct Kernels<UserCell<Impl>, unsigned short>;                                                      \
    }                                                                                                             \
    extern "C" {                                                                                                  \
    int name##_gates(void) { return Impl::G; }                                                                    \
    int name##_state(void) { return Impl::S; }                                                                    \
    int name##_param_rows(void) { return Impl::P; }                                                               \
    size_t name##_workspace_bytes(int dtype, int B, int L, int H, int backward)                                   \
    {                                                                                                             \
        const pararnn::CellInfo ci = {Impl::G, Impl::S, Impl::P, -1};                                             \
        if ((dtype != PARARNN_F32 && dtype != PARARNN_BF16) || !pararnn::dims_ok(B, L, H)) return 0;              \
        return pararnn::diag_workspace_bytes(ci, dtype, B, L, H, backward != 0);                                  \
    }                                                                                                             \
    size_t name##_workspace_bytes_fused(int dtype, int B, int L, int H, int n_iters)                              \
    {                                                                                                             \
        const pararnn::CellInfo ci = {Impl::G, Impl::S, Impl::P, -1};                                             \
        if ((dtype != PARARNN_F32 && dtype != PARARNN_BF16) || !pararnn::dims_ok(B, L, H)) return 0;              \
        return pararnn::diag_workspace_bytes_fused(ci, dtype, B, L, H, n_iters);                                  \
    }                                                                                                             \
    int name##_forward(int dtype, const float *params, const void *u, const void *h0, int B, int L, int H,        \
                       float tol, int max_iter, void *h, int *iters, float *delta_trace, void *workspace,         \
                       size_t workspace_bytes, void *hip_stream)                                                  \
    {                                                                                                             \
        const pararnn::CellInfo ci = {Impl::G, Impl::S, Impl::P, -1};                                             \
        const int bad = pararnn::check_forward_args(dtype, params, u, h0, B, L, H, tol, max_iter, h, iters,       \
                                                    workspace);                                                   \
        if (bad != PARARNN_OK) return bad;                                                                        \
        return pararnn::forward_solve<pararnn::UserCell<Impl>>(ci, dtype, params, u, h0, B, L, H, tol, max_iter,  \
                                                               h, iters, delta_trace, workspace, workspace_bytes, \
                                                               static_cast<hipStream_t>(hip_stream));             \
    }                                                                                                             \
    int name##_residual_norm(int dtype, const float *params, const void *u, const void *h0, const void *h,        \
                             int B, int L, int H, float *out, void *hip_stream)                                   \
    {                                                                                                             \
        const int bad = pararnn::check_residual_args(dtype, params, u, h0, h, B, L, H, out);                      \
        if (bad != PARARNN_OK) return bad;                                                                        \
        return pararnn::residual_norm_diag<pararnn::UserCell<Impl>>(dtype, params, u, h0, h, B, L, H, out,        \
                                                                    static_cast<hipStream_t>(hip_stream));        \
    }                                                                                                             \
    int name##_backward(int dtype, const float *params, const void *u, const void *h0, const void *h,             \
                        const void *dL_dh, int B, int L, int H, void *dL_du, float *dL_dparams, void *dL_dh0,     \
                        void *workspace, size_t workspace_bytes, void *hip_stream)                                \
    {                                                                                                             \
        const pararnn::CellInfo ci = {Impl::G, Impl::S, Impl::P, -1};                                             \
        const int bad = pararnn::check_backward_args(dtype, params, u, h0, h, dL_dh, B, L, H, dL_du, dL_dparams,  \
                                                     dL_dh0, workspace);                                          \
        if (bad != PARARNN_OK) return bad;                                                                        \
        return pararnn::backward_pass<pararnn::UserCell<Impl>>(ci, dtype, params, u, h0, h, dL_dh, B, L, H,       \
                                                               dL_du, dL_dparams, dL_dh0, workspace,              \
                                                               workspace_bytes,                                   \
                                                               static_cast<hipStream_t>(hip_stream));             \
    }                                                                                                             \
    }

#endif /* PARARNN_CELL_H */
