// Dense-Jacobian path: h' = tanh(W h + u), J_l = diag(1 - F_l^2) W (the generic
// dense case of Sec. 2.1), H = 64, fp32.
//
// One Newton iteration (Alg. 1a) is five launches:
//   residual  F_l = tanh(W h_{l-1} + u_l), d_l = 1 - F_l^2, r_l = F_l - h_l   (Eq. (3))
//   chunk_products   A_c = J_e ... J_s for every chunk of CD timesteps: the
//             64x64x64 Jacobian compositions of the scan, on the matrix cores
//             (v_mfma_f32_32x32x2_f32), one wave per (sequence, chunk)
//   sweep (local)    b_c = solution at the chunk's end for a zero input
//   carry            x_c = A_c x_{c-1} + b_c, sequential over the chunks of a sequence
//   sweep (final)    delta_l = J_l delta_{l-1} + r_l from x_{c-1}; h += delta; max|delta|
// The sweeps batch 32 sequences per wave so that the mat-vecs W delta of
// different sequences become one MFMA product W [delta_b]; the per-sequence
// factor d_l is applied to the product afterwards.
//
// MFMA operand trick: the 32x32 accumulator layout (lane = column, register v
// of lane half h = row 8*(v/4) + 4*h + v%4) is used unchanged as the B operand
// of the next product; the k-pair an instruction consumes is then (row(v,0),
// row(v,1)), and W is held in registers permuted to supply exactly those
// columns as the A operand.  No layout change is ever needed between products.
#include "../../include/pararnn.h"
#include "common.h"
#include "dense.h"
#include "launch.h"

#include <string.h>

#include <type_traits>

namespace pararnn {

namespace {

constexpr int DH = 64;          // hidden size this path is built for
constexpr int CD = 16;          // timesteps per chunk
typedef float f16v __attribute__((ext_vector_type(16)));

struct DenseArgs {
    const float *W;      // [64][64] row-major
    const float *u;      // [B][L][64]
    const float *h0;     // [B][64] or NULL
    float *h;            // [B][L][64] iterate, in place
    float *d;            // [B][L][64]
    float *r;            // [B][L][64]
    float *Ac;           // [B][n_c][64][64] row-major chunk products
    float *bc;           // [B][n_c][64] chunk-local end values
    float *xc;           // [B][n_c][64] delta at each chunk's end
    Ctrl *ctrl;
    int *iters_out;
    float *trace;
    int B, L, n_c;
    int k, max_iter;
    float tol;
};

__device__ __forceinline__ int mfma_row(int v, int half) { return 8 * (v >> 2) + 4 * half + (v & 3); }

// W in A-operand form: wr[mt][kt][v] = W[32 mt + lane%32][32 kt + row(v, lane/32)]
__device__ __forceinline__ void load_w_operand(const float *W, int lane, float (&wr)[2][2][16])
{
    const int n = lane & 31, half = lane >> 5;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int v = 0; v < 16; ++v) wr[mt][kt][v] = W[(32 * mt + n) * DH + 32 * kt + mfma_row(v, half)];
}

// ---------------------------------------------------------------- residual
// F = tanh(W h_{l-1} + u_l) for 32 consecutive rows (b, l) per wave as one MFMA
// product W [h_{l-1} rows]; lane = row, registers = channels (accumulator
// layout), so every access is a float4 inside a 256-byte row.
// mode 0: write d = 1 - F^2 and r = F - h for the current iterate;
// mode 1: write the initial guess h = tanh(W h0 + u) (App. A).
__global__ __launch_bounds__(256) void dense_residual_kernel(const DenseArgs a, int mode)
{
    if (a.ctrl->stop) return;
    const int lane = threadIdx.x & 63, n = lane & 31, half = lane >> 5;
    const int wave = blockIdx.x * 4 + (threadIdx.x >> 6), n_waves = gridDim.x * 4;
    const size_t rows = (size_t)a.B * a.L;
    const size_t n_items = (rows + 31) / 32;
    float wr[2][2][16];
    load_w_operand(a.W, lane, wr);
    for (size_t item = wave; item < n_items; item += n_waves) {
        const size_t row = item * 32 + n;
        const bool ok = row < rows;
        const int l = ok ? (int)(row % a.L) : 0;
        const size_t b = ok ? row / a.L : 0;
        // previous state of this row: h0 (or zero) at l = 0 and for the guess, else the row before
        const float *hp = nullptr;
        if (ok) {
            if (mode == 1 || l == 0) hp = a.h0 ? a.h0 + b * DH : nullptr;
            else hp = a.h + (row - 1) * DH;
        }
        f16v X[2], Y[2];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
                if (hp) t = *reinterpret_cast<const float4 *>(hp + 32 * kt + 8 * g + 4 * half);
                X[kt][4 * g] = t.x; X[kt][4 * g + 1] = t.y; X[kt][4 * g + 2] = t.z; X[kt][4 * g + 3] = t.w;
            }
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int v = 0; v < 16; ++v) Y[mt][v] = 0.0f;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                Y[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(wr[0][kt][v], X[kt][v], Y[0], 0, 0, 0);
                Y[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(wr[1][kt][v], X[kt][v], Y[1], 0, 0, 0);
            }
        if (ok) {
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const size_t off = row * DH + 32 * mt + 8 * g + 4 * half;
                    const float4 uv = *reinterpret_cast<const float4 *>(a.u + off);
                    float4 F;
                    F.x = fast_tanh(Y[mt][4 * g] + uv.x); F.y = fast_tanh(Y[mt][4 * g + 1] + uv.y);
                    F.z = fast_tanh(Y[mt][4 * g + 2] + uv.z); F.w = fast_tanh(Y[mt][4 * g + 3] + uv.w);
                    if (mode == 1) {
                        *reinterpret_cast<float4 *>(a.h + off) = F;
                    } else {
                        const float4 hv = *reinterpret_cast<const float4 *>(a.h + off);
                        *reinterpret_cast<float4 *>(a.d + off) =
                            make_float4(fmaf(-F.x, F.x, 1.0f), fmaf(-F.y, F.y, 1.0f), fmaf(-F.z, F.z, 1.0f), fmaf(-F.w, F.w, 1.0f));
                        *reinterpret_cast<float4 *>(a.r + off) = make_float4(F.x - hv.x, F.y - hv.y, F.z - hv.z, F.w - hv.w);
                    }
                }
        }
    }
}

// ------------------------------------------------------------ chunk products
// A_c = J_e ... J_{s+1} J_s with J_l = diag(d_l) W, one wave per (b, chunk).
// Chunk 0 and the last chunk are skipped: nothing enters chunk 0 (delta_0 = 0)
// and nothing follows the last one.
__global__ __launch_bounds__(256) void dense_chunk_products_kernel(const DenseArgs a)
{
    if (a.ctrl->stop) return;
    const int lane = threadIdx.x & 63, n = lane & 31, half = lane >> 5;
    const int item = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int per_seq = a.n_c - 2;
    if (per_seq <= 0 || item >= a.B * per_seq) return;
    const int b = item / per_seq, c = 1 + item % per_seq;
    const int ls = c * CD, le = min(a.L, ls + CD);

    float wr[2][2][16];
    load_w_operand(a.W, lane, wr);

    // P = J_ls in accumulator layout: P[mt][nt][v] = d[row] W[row][32 nt + n]
    f16v P[2][2];
    const float *dl = a.d + ((size_t)b * a.L + ls) * DH;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = 32 * mt + mfma_row(v, half);
            const float dv = dl[row];
            P[mt][0][v] = dv * a.W[row * DH + n];
            P[mt][1][v] = dv * a.W[row * DH + 32 + n];
        }
    // the row factors d_l of all later steps up front, so that the product loop never waits on memory
    float dpre[CD][2];
#pragma unroll
    for (int i = 1; i < CD; ++i) {
        const bool ok = ls + i < le;
        dpre[i][0] = ok ? dl[i * DH + n] : 0.0f;
        dpre[i][1] = ok ? dl[i * DH + 32 + n] : 0.0f;
    }
#pragma unroll 1
    for (int i = 1; i < CD; ++i) {
        if (ls + i >= le) break;
        float d0 = 0.0f, d1 = 0.0f;
#pragma unroll
        for (int q = 1; q < CD; ++q)
            if (q == i) { d0 = dpre[q][0]; d1 = dpre[q][1]; }
        f16v Q[2][2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                for (int v = 0; v < 16; ++v) Q[mt][nt][v] = 0.0f;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float a0 = wr[0][kt][v] * d0, a1 = wr[1][kt][v] * d1;
                const float b0 = P[kt][0][v], b1 = P[kt][1][v];
                Q[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, Q[0][0], 0, 0, 0);
                Q[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, Q[0][1], 0, 0, 0);
                Q[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, Q[1][0], 0, 0, 0);
                Q[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, Q[1][1], 0, 0, 0);
            }
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) P[mt][nt] = Q[mt][nt];
    }
    float *out = a.Ac + ((size_t)b * a.n_c + c) * DH * DH;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int v = 0; v < 16; ++v) out[(32 * mt + mfma_row(v, half)) * DH + 32 * nt + n] = P[mt][nt][v];
}

// The last workgroup of the final sweep closes the iteration: stopping test,
// results, reset of the counters (same protocol as the scan kernels).
__device__ __forceinline__ void finish_iteration(const DenseArgs &a, float block_max)
{
    Ctrl *ctrl = a.ctrl;
    atomicMax(&ctrl->gmax_bits, __float_as_uint(block_max));
    __threadfence();
    const unsigned int prev = atomicAdd(&ctrl->done, 1u);
    if (prev == gridDim.x - 1) {
        __threadfence();
        const float mk = __uint_as_float(atomicMax(&ctrl->gmax_bits, 0u));
        int status, stop = 0;
        if (a.trace) a.trace[a.k - 1] = mk;
        if (!(mk - mk == 0.0f)) { status = kStNonFinite; stop = 1; }
        else if (a.tol >= 0.0f && mk <= a.tol) { status = kStOk; stop = 1; }
        else status = a.tol < 0.0f ? kStOk : kStNotConverged;
        a.iters_out[0] = a.k;
        a.iters_out[1] = status;
        ctrl->iters = a.k;
        ctrl->status = status;
        ctrl->stop = stop;
        ctrl->done = 0u;
        ctrl->gmax_bits = 0u;
        __threadfence();
    }
}

// -------------------------------------------------------------------- sweeps
// X <- diag(d_l) (W X) + r_l over the steps of one chunk for 32 sequences at
// once: X is 64 channels x 32 sequences in accumulator layout (2 row tiles).
// final = 0: X starts at 0, only the end value is kept (b_c).
// final = 1: X starts at x_{c-1}; every step updates h and feeds max|delta|.
template <int FINAL>
__global__ __launch_bounds__(256) void dense_sweep_kernel(const DenseArgs a)
{
    __shared__ float s_max[4];
    if (a.ctrl->stop) return;
    const int lane = threadIdx.x & 63, n = lane & 31, half = lane >> 5, w = threadIdx.x >> 6;
    const int n_bt = (a.B + 31) / 32;
    const int item = blockIdx.x * 4 + w;
    float wmax = 0.0f;
    if (item < a.n_c * n_bt) {
        const int c = item / n_bt, bt = item - c * n_bt;
        const int b = bt * 32 + n;
        const bool b_ok = b < a.B;
        const bool full = bt * 32 + 32 <= a.B;          // wave-uniform: no guards needed in the loop
        const int ls = c * CD, le = min(a.L, ls + CD);
        float wr[2][2][16];
        load_w_operand(a.W, lane, wr);
        f16v X[2];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int v = 0; v < 16; ++v) X[kt][v] = 0.0f;
        if (FINAL && c > 0 && b_ok) {
            const float *x0 = a.xc + ((size_t)b * a.n_c + (c - 1)) * DH;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const float4 t = *reinterpret_cast<const float4 *>(x0 + 32 * kt + 8 * g + 4 * half);
                    X[kt][4 * g] = t.x; X[kt][4 * g + 1] = t.y; X[kt][4 * g + 2] = t.z; X[kt][4 * g + 3] = t.w;
                }
        }
        // rows of an invalid lane are read from sequence B-1 (valid memory) and
        // multiplied by zero; only stores are guarded, and only in ragged tiles
        const size_t brow = (size_t)(b_ok ? b : a.B - 1) * a.L;
        const float keep = b_ok ? 1.0f : 0.0f;
        auto sweep = [&](auto guard) {
            constexpr bool kGuard = decltype(guard)::value;
            // d, r (and h) of the next step are fetched before the products of
            // this step are issued, so their latency hides behind the MFMAs
            float4 dc[8], rc[8], hc[FINAL ? 8 : 1], dn[8], rn[8], hn[FINAL ? 8 : 1];
            auto fetch = [&](int l, float4 (&dd)[8], float4 (&rr)[8], float4 (&hh)[FINAL ? 8 : 1]) {
                const size_t off = (brow + l) * DH;
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const int ch = 32 * (q >> 2) + 8 * (q & 3) + 4 * half;
                    dd[q] = *reinterpret_cast<const float4 *>(a.d + off + ch);
                    rr[q] = *reinterpret_cast<const float4 *>(a.r + off + ch);
                    if constexpr (FINAL != 0) hh[q] = *reinterpret_cast<const float4 *>(a.h + off + ch);
                }
            };
            fetch(ls, dc, rc, hc);
            for (int l = ls; l < le; ++l) {
                fetch(min(l + 1, le - 1), dn, rn, hn);
                const size_t off = (brow + l) * DH;
                f16v Y[2];
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) Y[mt][v] = 0.0f;
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        Y[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(wr[0][kt][v], X[kt][v], Y[0], 0, 0, 0);
                        Y[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(wr[1][kt][v], X[kt][v], Y[1], 0, 0, 0);
                    }
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const int mt = q >> 2, g = q & 3;
                    const int ch = 32 * mt + 8 * g + 4 * half;
                    float4 dv = dc[q], rv = rc[q];
                    if constexpr (kGuard) {
                        dv.x *= keep; dv.y *= keep; dv.z *= keep; dv.w *= keep;
                        rv.x *= keep; rv.y *= keep; rv.z *= keep; rv.w *= keep;
                    }
                    const float x0 = fmaf(dv.x, Y[mt][4 * g], rv.x), x1 = fmaf(dv.y, Y[mt][4 * g + 1], rv.y);
                    const float x2 = fmaf(dv.z, Y[mt][4 * g + 2], rv.z), x3 = fmaf(dv.w, Y[mt][4 * g + 3], rv.w);
                    X[mt][4 * g] = x0; X[mt][4 * g + 1] = x1; X[mt][4 * g + 2] = x2; X[mt][4 * g + 3] = x3;
                    if constexpr (FINAL != 0) {
                        float4 hv = hc[q];
                        hv.x += x0; hv.y += x1; hv.z += x2; hv.w += x3;
                        if (!kGuard || b_ok) *reinterpret_cast<float4 *>(a.h + off + ch) = hv;
                        wmax = nanmax(nanmax(nanmax(nanmax(wmax, __builtin_fabsf(x0)), __builtin_fabsf(x1)),
                                             __builtin_fabsf(x2)), __builtin_fabsf(x3));
                    }
                }
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    dc[q] = dn[q]; rc[q] = rn[q];
                    if constexpr (FINAL != 0) hc[q] = hn[q];
                }
            }
        };
        if (full) sweep(std::false_type{});
        else sweep(std::true_type{});
        if (!FINAL && b_ok) {
            float *out = a.bc + ((size_t)b * a.n_c + c) * DH;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    *reinterpret_cast<float4 *>(out + 32 * mt + 8 * g + 4 * half) =
                        make_float4(X[mt][4 * g], X[mt][4 * g + 1], X[mt][4 * g + 2], X[mt][4 * g + 3]);
        }
    }
    if (FINAL) {
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) wmax = nanmax(wmax, __shfl_xor(wmax, off, 64));
        if (lane == 0) s_max[w] = wmax;
        __syncthreads();
        if (threadIdx.x == 0)
            finish_iteration(a, nanmax(nanmax(s_max[0], s_max[1]), nanmax(s_max[2], s_max[3])));
    }
}

// --------------------------------------------------------------------- carry
// x_c = A_c x_{c-1} + b_c for c = 0 .. n_c-2 (x_{-1} = 0, so x_0 = b_0); one
// wave per sequence, lane = row of A_c.  The rows of the next four chunks are
// in flight while one is used (the chain is otherwise bound by memory latency);
// the loop body is branch-free (indices are clamped instead) so that the loads
// really stay outstanding; x is broadcast lane by lane (v_readlane).
__global__ __launch_bounds__(64) void dense_carry_kernel(const DenseArgs a)
{
    constexpr int DEPTH = 4;
    if (a.ctrl->stop) return;
    const int lane = threadIdx.x, b = blockIdx.x;
    const float *bcb = a.bc + (size_t)b * a.n_c * DH + lane;
    float *xcb = a.xc + (size_t)b * a.n_c * DH + lane;
    const float *Ab = a.Ac + ((size_t)b * a.n_c * DH + lane) * DH;     // row `lane` of chunk 0
    float x = bcb[0];
    xcb[0] = x;
    const int last = a.n_c - 2;                       // last chunk whose end value is needed
    if (last < 1) return;
    float4 buf[DEPTH][DH / 4];
    float bb[DEPTH];
#pragma unroll
    for (int k = 0; k < DEPTH; ++k) {
        const int c = min(1 + k, last);
#pragma unroll
        for (int j = 0; j < DH / 4; ++j)
            buf[k][j] = *reinterpret_cast<const float4 *>(Ab + (size_t)c * DH * DH + 4 * j);
        bb[k] = bcb[(size_t)c * DH];
    }
    for (int base = 1; base <= last; base += DEPTH) {
#pragma unroll
        for (int k = 0; k < DEPTH; ++k) {
            const int c = base + k;
            float s0 = bb[k], s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
            const unsigned int xb = __float_as_uint(x);
#pragma unroll
            for (int j = 0; j < DH / 4; ++j) {
                s0 = fmaf(buf[k][j].x, __uint_as_float(__builtin_amdgcn_readlane(xb, 4 * j)), s0);
                s1 = fmaf(buf[k][j].y, __uint_as_float(__builtin_amdgcn_readlane(xb, 4 * j + 1)), s1);
                s2 = fmaf(buf[k][j].z, __uint_as_float(__builtin_amdgcn_readlane(xb, 4 * j + 2)), s2);
                s3 = fmaf(buf[k][j].w, __uint_as_float(__builtin_amdgcn_readlane(xb, 4 * j + 3)), s3);
            }
            // past the end the value is simply kept (and rewritten to the last slot)
            x = c <= last ? (s0 + s1) + (s2 + s3) : x;
            xcb[(size_t)min(c, last) * DH] = x;
            const int cn = min(c + DEPTH, last);
#pragma unroll
            for (int j = 0; j < DH / 4; ++j)
                buf[k][j] = *reinterpret_cast<const float4 *>(Ab + (size_t)cn * DH * DH + 4 * j);
            bb[k] = bcb[(size_t)cn * DH];
        }
    }
}

size_t r256(size_t x) { return (x + 255) & ~(size_t)255; }

struct DenseLayout { size_t off_d, off_r, off_A, off_b, off_x, total; int n_c; };

DenseLayout dense_layout(int B, int L)
{
    DenseLayout lo;
    lo.n_c = (L + CD - 1) / CD;
    size_t off = r256(sizeof(Ctrl));
    lo.off_d = off; off += r256((size_t)B * L * DH * 4);
    lo.off_r = off; off += r256((size_t)B * L * DH * 4);
    lo.off_A = off; off += r256((size_t)B * lo.n_c * DH * DH * 4);
    lo.off_b = off; off += r256((size_t)B * lo.n_c * DH * 4);
    lo.off_x = off; off += r256((size_t)B * lo.n_c * DH * 4);
    lo.total = off;
    return lo;
}

}  // namespace

int dense_chunk() { return CD; }

int dense_chunk_products(const float *W, const float *d, int B, int L, int H, float *A, void *ctrl_scratch,
                         hipStream_t st)
{
    if (H != DH) return PARARNN_UNSUPPORTED;
    if (((uintptr_t)W | (uintptr_t)d | (uintptr_t)A) % 16) return PARARNN_UNSUPPORTED;
    DenseArgs a;
    memset(&a, 0, sizeof(a));
    a.W = W; a.d = const_cast<float *>(d); a.Ac = A;
    a.ctrl = static_cast<Ctrl *>(ctrl_scratch);
    a.B = B; a.L = L; a.n_c = (L + CD - 1) / CD;
    if (launch_reset(a.ctrl, nullptr, 0, nullptr, 0, st) != hipSuccess) return PARARNN_HIP_ERROR;
    const int n_prod = B * (a.n_c - 2);
    if (n_prod > 0)
        hipLaunchKernelGGL(dense_chunk_products_kernel, dim3((n_prod + 3) / 4), dim3(256), 0, st, a);
    return hipGetLastError() == hipSuccess ? PARARNN_OK : PARARNN_HIP_ERROR;
}

size_t dense_workspace_bytes(int dtype, int B, int L, int H, int backward)
{
    if (dtype != PARARNN_F32 || H != DH || backward) return 256;
    return dense_layout(B, L).total;
}

int dense_forward(int dtype, const float *W, const void *u, const void *h0, int B, int L, int H, float tol,
                  int max_iter, void *h, int *iters, float *delta_trace, void *workspace, size_t workspace_bytes,
                  hipStream_t st)
{
    if (dtype != PARARNN_F32 || H != DH) return PARARNN_UNSUPPORTED;
    if (((uintptr_t)W | (uintptr_t)u | (uintptr_t)h | (uintptr_t)h0) % 16) return PARARNN_UNSUPPORTED;
    const DenseLayout lo = dense_layout(B, L);
    if (workspace_bytes < lo.total) return PARARNN_WORKSPACE_TOO_SMALL;
    char *ws = static_cast<char *>(workspace);
    DenseArgs a;
    a.W = W; a.u = static_cast<const float *>(u); a.h0 = static_cast<const float *>(h0);
    a.h = static_cast<float *>(h);
    a.d = reinterpret_cast<float *>(ws + lo.off_d);
    a.r = reinterpret_cast<float *>(ws + lo.off_r);
    a.Ac = reinterpret_cast<float *>(ws + lo.off_A);
    a.bc = reinterpret_cast<float *>(ws + lo.off_b);
    a.xc = reinterpret_cast<float *>(ws + lo.off_x);
    a.ctrl = reinterpret_cast<Ctrl *>(ws);
    a.iters_out = iters; a.trace = delta_trace;
    a.B = B; a.L = L; a.n_c = lo.n_c; a.k = 0; a.max_iter = max_iter; a.tol = tol;

    const int status0 = tol < 0.0f ? PARARNN_OK : PARARNN_NOT_CONVERGED;
    if (launch_reset(a.ctrl, nullptr, 0, iters, status0, st) != hipSuccess) return PARARNN_HIP_ERROR;
    const size_t res_items = ((size_t)B * L + 31) / 32;
    const int res_blocks = (int)((res_items + 3) / 4 < 512 ? (res_items + 3) / 4 : 512);
    hipLaunchKernelGGL(dense_residual_kernel, dim3(res_blocks), dim3(256), 0, st, a, 1);
    const int n_prod = B * (lo.n_c - 2);
    const int n_sweep = lo.n_c * ((B + 31) / 32);
    for (int k = 1; k <= max_iter; ++k) {
        a.k = k;
        hipLaunchKernelGGL(dense_residual_kernel, dim3(res_blocks), dim3(256), 0, st, a, 0);
        if (n_prod > 0)
            hipLaunchKernelGGL(dense_chunk_products_kernel, dim3((n_prod + 3) / 4), dim3(256), 0, st, a);
        hipLaunchKernelGGL(dense_sweep_kernel<0>, dim3((n_sweep + 3) / 4), dim3(256), 0, st, a);
        hipLaunchKernelGGL(dense_carry_kernel, dim3(B), dim3(64), 0, st, a);
        hipLaunchKernelGGL(dense_sweep_kernel<1>, dim3((n_sweep + 3) / 4), dim3(256), 0, st, a);
    }
    return hipGetLastError() == hipSuccess ? PARARNN_OK : PARARNN_HIP_ERROR;
}

}  // namespace pararnn
