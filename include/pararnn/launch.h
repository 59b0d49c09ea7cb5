// Host-side launch interface between the C ABI and the per-cell kernel
// instantiations (each cell / storage type is compiled in its own file).
#pragma once
#include "fused_kernels.h"

namespace pararnn {

struct TileCfg {
    int vec;  // channels per lane
    int ll;   // segments along L inside a wave (64/ll lanes each)
    int c;    // timesteps per thread
    int w;    // waves per workgroup
};

// Tile shapes compiled for every cell: X(VEC, LL, C, W).  A tile covers
// (64/LL)*VEC channels x C*LL*W timesteps.  Measured on MI355X the narrow
// shapes (one or two channels per lane: few registers, many resident waves)
// beat wide vector loads; the automatic choice is in pararnn_api.hip.
#define PARARNN_SHAPES(X)                                                                       \
    X(1, 1, 8, 16) X(1, 2, 8, 16) X(1, 2, 16, 4) X(1, 2, 8, 8) X(1, 1, 8, 8) X(2, 2, 8, 8)            \
    X(1, 1, 16, 8) X(1, 1, 4, 8) X(1, 8, 4, 2) X(4, 4, 8, 8) X(2, 4, 8, 8) X(1, 1, 16, 4) X(1, 1, 12, 8)
// channels per lane compiled for the element-wise kernels
#define PARARNN_VECS(X) X(1) X(2) X(4)

template <class Cell, typename UT> struct Kernels {
    static hipError_t init_guess(int vec, const FwdArgs &a, hipStream_t st);
    static hipError_t residual_norm(int vec, const ResArgs &a, hipStream_t st);
    // fold_guess: this is iteration 1 and the initial guess is computed inside it
    static hipError_t newton_iter(const TileCfg &cfg, const FwdArgs &a, bool fold_guess, hipStream_t st);
    static hipError_t backward(const TileCfg &cfg, const BwdArgs &a, hipStream_t st);
    // all iterations of a fixed-count solve in one launch
    static hipError_t newton_fused(const TileCfg &cfg, const FusedArgs &a, hipStream_t st);
};

hipError_t launch_reset(Ctrl *ctrl, unsigned long long *rec, size_t n_rec, int *iters_out, int status0,
                        hipStream_t st);
// ctrl may be NULL; otherwise the pass is skipped on the device when ctrl->h_final is set
hipError_t launch_store_bf16(const float *src, void *dst, size_t n, const Ctrl *ctrl, hipStream_t st);
// n 32-bit words of zeros, written by a kernel (no memset node when a caller captures a graph)
hipError_t launch_zero_words(unsigned int *dst, int n, hipStream_t st);
hipError_t launch_param_reduce(const float *part, float *out, int n_terms, int n_out, hipStream_t st);
int device_cu_count();

// Workspaces that are reused across calls (pararnn_set_workspace_reuse).  Returns the number this call adds
// to the epoch in its record tags and sets *fill to whether the carry records have to be cleared: not when
// the last call that used this workspace on this device had the same layout signature, in which case its
// records carry another number and read as empty.  Without the caller's promise, under stream capture (a
// captured launch sequence would replay one number) and for a new address or signature: 0 / 1 and *fill = true.
unsigned int workspace_epoch(void *workspace, unsigned long long layout_sig, hipStream_t st, bool *fill);
// The library no longer knows what this workspace holds (a call on it failed, or ran without a signature).
void workspace_forget(void *workspace);

}  // namespace pararnn
