// Host entry points of the input projection u = B x + b and its derivatives
// (matrix-core kernels in proj_kernels.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace pararnn {

size_t proj_workspace_bytes(int dtype, int B, int L, int H, int G, int n_heads, int backward);
int proj_forward(int dtype, const void *x, const float *Wx, const float *bias, int B, int L, int H, int G,
                 int n_heads, void *u, void *workspace, size_t workspace_bytes, hipStream_t st);
// dx, dWx may be NULL (not wanted); dbias needs dWx
int proj_backward(int dtype, const void *x, const float *Wx, const void *du, int B, int L, int H, int G, int n_heads,
                  void *dx, float *dWx, float *dbias, void *workspace, size_t workspace_bytes, hipStream_t st);

// bf16 storage: the NT products (forward, dx) copy their operand tiles straight into LDS (1, default) or stage them
// through registers like the fp32-storage kernels (0)
int proj_set_dma(int on);

}  // namespace pararnn
