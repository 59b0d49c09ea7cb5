// Small helper kernels shared by all paths, and their launchers.
#include "pararnn/launch.h"

namespace pararnn {

// Clears the control block and the carry records of a call (their tags must
// not survive from an earlier call), and sets the result of a solve that
// performs no iteration.
__global__ void reset_kernel(Ctrl *ctrl, unsigned long long *rec, size_t n_rec, int *iters_out, int status0)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < 64) reinterpret_cast<unsigned int *>(ctrl)[i] = 0u;     // the whole 256-byte control block
    __syncthreads();
    if (i == 0) {
        ctrl->status = status0;
        if (iters_out) { iters_out[0] = 0; iters_out[1] = status0; }
    }
    // two records per store (the array is 256-byte aligned); the odd last one separately
    ulonglong2 *rec2 = reinterpret_cast<ulonglong2 *>(rec);
    const size_t n2 = n_rec / 2;
    for (size_t j = i; j < n2; j += (size_t)gridDim.x * blockDim.x) rec2[j] = make_ulonglong2(0ull, 0ull);
    if (i == 0 && (n_rec & 1)) rec[n_rec - 1] = 0ull;
}

__global__ void zero_words_kernel(unsigned int *dst, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = 0u;
}

// bf16 storage: round the converged fp32 iterate once into the output.
__global__ __launch_bounds__(256) void store_bf16_kernel(const float *src, unsigned short *dst, size_t n4,
                                                         const Ctrl *ctrl)
{
    if (ctrl && ctrl->h_final) return;            // the output was already written in its final form
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (size_t)gridDim.x * blockDim.x) {
        float v[4];
        load_vec<4>(src + 4 * i, v);
        store_vec<4>(dst + 4 * i, v);
    }
}

__global__ __launch_bounds__(256) void store_bf16_scalar_kernel(const float *src, unsigned short *dst, size_t n,
                                                                const Ctrl *ctrl)
{
    if (ctrl && ctrl->h_final) return;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = f32_to_bf16(src[i]);
}

__global__ void store_bf16_tail_kernel(const float *src, unsigned short *dst, int n, const Ctrl *ctrl)
{
    if (ctrl && ctrl->h_final) return;
    if ((int)threadIdx.x < n) dst[threadIdx.x] = f32_to_bf16(src[threadIdx.x]);
}

// dL/dparams[i] = sum over the n_terms (tile, sequence) partials part[t][i].
// A block owns 64 outputs; its 16 slices of 64 threads sum interleaved terms
// with independent accumulators, then the slices are added in a fixed order,
// so the result does not depend on scheduling.
__global__ __launch_bounds__(1024) void param_reduce_kernel(const float *part, float *out, int n_terms, int n_out)
{
    __shared__ float s_sum[16][64];
    const int o = threadIdx.x & 63, slice = threadIdx.x >> 6;
    const int i = blockIdx.x * 64 + o;
    float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
    if (i < n_out) {
        int t = slice;
        for (; t + 48 < n_terms; t += 64) {
            a0 += part[(size_t)t * n_out + i];
            a1 += part[(size_t)(t + 16) * n_out + i];
            a2 += part[(size_t)(t + 32) * n_out + i];
            a3 += part[(size_t)(t + 48) * n_out + i];
        }
        for (; t < n_terms; t += 16) a0 += part[(size_t)t * n_out + i];
    }
    s_sum[slice][o] = (a0 + a1) + (a2 + a3);
    __syncthreads();
    if (slice == 0 && i < n_out) {
        float s = 0.0f;
#pragma unroll
        for (int k = 0; k < 16; ++k) s += s_sum[k][o];
        out[i] = s;
    }
}

}  // namespace pararnn

namespace pararnn {

hipError_t launch_reset(Ctrl *ctrl, unsigned long long *rec, size_t n_rec, int *iters_out, int status0,
                        hipStream_t st)
{
    size_t blocks = (n_rec / 2 + 255) / 256;
    if (blocks < 1) blocks = 1;
    const size_t cap = (size_t)device_cu_count() * 32;
    if (blocks > cap) blocks = cap;
    hipLaunchKernelGGL(reset_kernel, dim3((unsigned)blocks), dim3(256), 0, st, ctrl, rec, n_rec, iters_out,
                       status0);
    return hipGetLastError();
}

hipError_t launch_zero_words(unsigned int *dst, int n, hipStream_t st)
{
    hipLaunchKernelGGL(zero_words_kernel, dim3((n + 63) / 64), dim3(64), 0, st, dst, n);
    return hipGetLastError();
}

hipError_t launch_store_bf16(const float *src, void *dst, size_t n, const Ctrl *ctrl, hipStream_t st)
{
    // four values per thread (16-byte loads, 8-byte stores) where both pointers allow it, else one
    if (reinterpret_cast<uintptr_t>(dst) % 8 != 0 || reinterpret_cast<uintptr_t>(src) % 16 != 0) {
        size_t blocks = (n + 255) / 256;
        const size_t cap = (size_t)device_cu_count() * 32;
        if (blocks > cap) blocks = cap;
        hipLaunchKernelGGL(store_bf16_scalar_kernel, dim3((unsigned)blocks), dim3(256), 0, st, src,
                           static_cast<unsigned short *>(dst), n, ctrl);
        return hipGetLastError();
    }
    const size_t n4 = n / 4;
    if (n4) {
        size_t blocks = (n4 + 255) / 256;
        const size_t cap = (size_t)device_cu_count() * 32;
        if (blocks > cap) blocks = cap;
        hipLaunchKernelGGL(store_bf16_kernel, dim3((unsigned)blocks), dim3(256), 0, st, src,
                           static_cast<unsigned short *>(dst), n4, ctrl);
    }
    if (n % 4) {
        hipLaunchKernelGGL(store_bf16_tail_kernel, dim3(1), dim3(64), 0, st, src + 4 * n4,
                           static_cast<unsigned short *>(dst) + 4 * n4, (int)(n % 4), ctrl);
    }
    return hipGetLastError();
}

hipError_t launch_param_reduce(const float *part, float *out, int n_terms, int n_out, hipStream_t st)
{
    hipLaunchKernelGGL(param_reduce_kernel, dim3((n_out + 63) / 64), dim3(1024), 0, st, part, out, n_terms, n_out);
    return hipGetLastError();
}

int device_cu_count()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            cus = n;
        else
            cus = 256;
    }
    return cus;
}

}  // namespace pararnn

