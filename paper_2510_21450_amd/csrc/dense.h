// Host entry points of the dense-Jacobian path (h' = tanh(W h + u)).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace pararnn {

size_t dense_workspace_bytes(int dtype, int B, int L, int H, int backward);
int dense_forward(int dtype, const float *W, const void *u, const void *h0, int B, int L, int H, float tol,
                  int max_iter, void *h, int *iters, float *delta_trace, void *workspace, size_t workspace_bytes,
                  hipStream_t st);

}  // namespace pararnn
