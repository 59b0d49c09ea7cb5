// Host entry points of the dense-Jacobian path (h' = tanh(W h + u)).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace pararnn {

size_t dense_workspace_bytes(int dtype, int B, int L, int H, int backward);
int dense_forward(int dtype, const float *W, const void *u, const void *h0, int B, int L, int H, float tol,
                  int max_iter, void *h, int *iters, float *delta_trace, void *workspace, size_t workspace_bytes,
                  hipStream_t st);

// Adjoint scan and gradients at the forward result h: du [B][L][H], dW [H][H], dh0 [B][H] (or NULL).
int dense_backward(int dtype, const float *W, const void *u, const void *h0, const void *h, const void *g, int B,
                   int L, int H, void *du, float *dW, void *dh0, void *workspace, size_t workspace_bytes,
                   hipStream_t st);

// max |h_l - tanh(W h_{l-1} + u_l)| over everything (App. A), to a device float
int dense_residual_norm(int dtype, const float *W, const void *u, const void *h0, const void *h, int B, int L, int H,
                        float *out, hipStream_t st);

// Timesteps per chunk of the dense scan, and its composition kernel alone:
// A[b][c] = J_e ... J_s, J_l = diag(d_l) W, for the chunks 1 .. n_c-2 (the ones the
// scan needs); ctrl_scratch is 256 bytes of device memory.
int dense_chunk();
// Arithmetic of the chunk products of forward solves: 0 fp32 (default), 1 three bf16 terms, 2 one bf16 term.
int dense_set_products(int mode);
// Jacobian of the linear solves of forward solves: 0 full (Newton, default), 1 its diagonal (quasi-Newton).
int dense_set_jacobian(int mode);
// Launch structure of forward solves: 1 launches per phase for the first iterations, one persistent launch for the
// rest (default); 0 launches per phase throughout; 2 the persistent launch from the first iteration.
int dense_set_one_launch(int mode);
int dense_chunk_products(const float *W, const float *d, int B, int L, int H, float *A, void *ctrl_scratch,
                         hipStream_t st);

}  // namespace pararnn
