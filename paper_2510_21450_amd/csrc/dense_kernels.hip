// Dense-Jacobian path: h' = tanh(W h + u), J_l = diag(1 - F_l^2) W (the generic
// dense case of Sec. 2.1), H = 64, fp32.
//
// One Newton iteration (Alg. 1a) is four launches (chunk_products and the local sweep share one):
//   residual  F_l = tanh(W h_{l-1} + u_l), d_l = 1 - F_l^2, r_l = F_l - h_l   (Eq. (3))
//   chunk_products   A_c = J_e ... J_s for every chunk of CD timesteps: the
//             64x64x64 Jacobian compositions of the scan, on the matrix cores
//             (v_mfma_f32_32x32x2_f32), one wave per (sequence, chunk)
//   sweep (local)    b_c = solution at the chunk's end for a zero input
//   carry            x_c = A_c x_{c-1} + b_c, sequential over the chunks of a sequence
//   sweep (final)    delta_l = J_l delta_{l-1} + r_l from x_{c-1}; h += delta; max|delta|
// The sweeps batch 16 (sequence, chunk) columns per workgroup so that the
// mat-vecs W delta of different columns become one MFMA product W [delta];
// the per-column factor d_l is applied to the product afterwards.
//
// Backward (Eq. (6)): with mu_l = d_l * lam_l (which is dL/du_l) the adjoint
// recurrence lam_l = g_l + W^T (d_{l+1} * lam_{l+1}) becomes
//   mu_l = diag(d_l) W^T mu_{l+1} + d_l * g_l,
// the same affine recurrence as the forward solve with W^T in place of W, the
// time axis reversed and r_l = d_l * g_l: the same kernels run it (rev = 1,
// W = the transposed matrix), followed by dL/dh0 = W^T mu_1 and
// dL/dW = sum_{b,l} mu_l h_{l-1}^T (one more MFMA reduction).
//
// MFMA operand trick: the 32x32 accumulator layout (lane = column, register v
// of lane half h = row 8*(v/4) + 4*h + v%4) is used unchanged as the B operand
// of the next product; the k-pair an instruction consumes is then (row(v,0),
// row(v,1)), and W is held in registers permuted to supply exactly those
// columns as the A operand.  No layout change is ever needed between products.
#include "pararnn.h"
#include "pararnn/common.h"
#include "dense.h"
#include "pararnn/driver.h"
#include "pararnn/launch.h"

#include <string.h>

#include <type_traits>

namespace pararnn {

namespace {

constexpr int DH = 64;          // hidden size this path is built for
constexpr int CD = 16;          // timesteps per chunk
typedef float f16v __attribute__((ext_vector_type(16)));
typedef float f4v __attribute__((ext_vector_type(4)));
typedef __bf16 bf2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf8v __attribute__((ext_vector_type(8)));
typedef unsigned int u4v __attribute__((ext_vector_type(4)));

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
    float *hend;         // [B][n_c][64] the iterate at each chunk's last step, as it was before this iteration's update (or NULL)
    Ctrl *ctrl;
    int *iters_out;
    float *trace;
    int B, L, n_c;
    int k, max_iter;
    float tol;
    // backward
    const float *g;      // dL/dh [B][L][64]
    float *du;           // out [B][L][64]: mu
    int rev;             // 1: scan step t of the recurrence is timestep L-1-t
    unsigned int *norm;  // residual max-norm only: bits of the result, zero on entry
    unsigned int *gmax;  // one-launch solve only: where the final sweep leaves max|delta| of this iteration
    unsigned int spin_limit;   // one-launch solve only: polls of a grid-wide barrier before a workgroup gives up
};

// row of the [B][L][64] arrays that scan step t of sequence b touches
__device__ __forceinline__ size_t scan_row(const DenseArgs &a, size_t b, int t)
{
    return b * a.L + (a.rev ? a.L - 1 - t : t);
}

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
            for (int g = 0; g < 4; ++g) {
                // rows(4g .. 4g+3, half) are four consecutive columns of W
                const float4 t = *reinterpret_cast<const float4 *>(W + (32 * mt + n) * DH + 32 * kt + 8 * g + 4 * half);
                wr[mt][kt][4 * g] = t.x; wr[mt][kt][4 * g + 1] = t.y; wr[mt][kt][4 * g + 2] = t.z; wr[mt][kt][4 * g + 3] = t.w;
            }
}

// W in A-operand form for the 16x16x4 products of wave w:
// wa[ww][v] = W[16w + n][16ww + 4g + v], lane = (n = lane % 16, g = lane / 16)
__device__ __forceinline__ void load_w_operand16(const float *W, int w, int n, int g, float (&wa)[4][4])
{
#pragma unroll
    for (int ww = 0; ww < 4; ++ww) {
        const f4v t = *reinterpret_cast<const f4v *>(W + (16 * w + n) * DH + 16 * ww + 4 * g);
#pragma unroll
        for (int v = 0; v < 4; ++v) wa[ww][v] = t[v];
    }
}

// ---------------------------------------------------------------- residual
// F = tanh(W h_{l-1} + u_l) for 16 consecutive rows (b, l) per workgroup as one
// 64 x 64 x 16 product W [h_{l-1} rows] on v_mfma_f32_16x16x4_f32: wave w owns
// channels 16w .. 16w+15, lane (n = lane % 16, g = lane / 16) ends up with
// channels 16w + 4g .. +3 of row n, so u, h, d and r move as float4.  The B
// operand of k-step (ww, v) is component v of the float4 at channels
// 16ww + 4g of the previous state, read straight from memory.
// mode 0: write d = 1 - F^2 and r = F - h for the current iterate;
// mode 1: write the initial guess h = tanh(W h0 + u) (App. A);
// mode 2: write nothing but max |F - h| over all rows to a.norm (no control block is read);
// mode 3: as mode 0, but d is the diagonal of the Jacobian, (1 - F^2) * W_ii (quasi-Newton);
// mode 4: modes 1 and 0 in one pass: the initial guess is written, and the residual and row factors of the
//         first iteration are formed from it.  The guess of the row before, which the residual needs, is
//         recomputed rather than read (it is tanh(W h0 + u_{l-1}), and W h0 is one product per row's sequence,
//         shared with the row's own guess): same bits as the two launches, one pass over u instead of two and
//         none over h.
__device__ __forceinline__ void residual_body(const DenseArgs &a, int mode)
{
    float nmax = 0.0f;
    f4v wdiag = {1.0f, 1.0f, 1.0f, 1.0f};
    if (mode == 3) {
        const int c0 = 16 * __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) + 4 * (int)((threadIdx.x & 63) >> 4);
#pragma unroll
        for (int v = 0; v < 4; ++v) wdiag[v] = a.W[(c0 + v) * DH + c0 + v];
    }
    const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int n = lane & 15, g = lane >> 4;
    const int chn = 16 * w + 4 * g;
    const size_t rows = (size_t)a.B * a.L;
    const size_t n_items = (rows + 15) / 16;
    float wa[4][4];
    load_w_operand16(a.W, w, n, g, wa);
    const f4v zero = {0.0f, 0.0f, 0.0f, 0.0f};
    __shared__ f4v s_c[4][64];
    for (size_t item = blockIdx.x; item < n_items; item += gridDim.x) {
        const size_t row = item * 16 + n;
        const bool ok = row < rows;
        const int l = ok ? (int)(row % a.L) : 0;
        const size_t b = ok ? row / a.L : 0;
        if (mode == 4) {
            // W h0 of this row's sequence: own part (channels chn ..) and, through LDS, every wave's part
            f4v cbo = zero, cbk[4] = {zero, zero, zero, zero};
            f4v h0k[4] = {zero, zero, zero, zero};
            if (a.h0) {
#pragma unroll
                for (int ww = 0; ww < 4; ++ww)
                    if (ok) h0k[ww] = *reinterpret_cast<const f4v *>(a.h0 + b * DH + 16 * ww + 4 * g);
                f4v c0 = zero, c1 = zero;
#pragma unroll
                for (int ww = 0; ww < 4; ww += 2)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        c0 = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[ww][v], h0k[ww][v], c0, 0, 0, 0);
                        c1 = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[ww + 1][v], h0k[ww + 1][v], c1, 0, 0, 0);
                    }
                cbo = c0 + c1;
                __syncthreads();                      // the previous item's reads of s_c
                s_c[w][lane] = cbo;
                __syncthreads();
#pragma unroll
                for (int ww = 0; ww < 4; ++ww) cbk[ww] = s_c[ww][lane];
            }
            f4v uv = zero;
            f4v xb[4] = {zero, zero, zero, zero};
            if (ok) {
                uv = *reinterpret_cast<const f4v *>(a.u + row * DH + chn);
                if (l == 0) {
#pragma unroll
                    for (int ww = 0; ww < 4; ++ww) xb[ww] = h0k[ww];
                } else {
#pragma unroll
                    for (int ww = 0; ww < 4; ++ww) {
                        const f4v y = cbk[ww] + *reinterpret_cast<const f4v *>(a.u + (row - 1) * DH + 16 * ww + 4 * g);
#pragma unroll
                        for (int v = 0; v < 4; ++v) xb[ww][v] = fast_tanh(y[v]);
                    }
                }
            }
            f4v acc0 = zero, acc1 = zero;
#pragma unroll
            for (int ww = 0; ww < 4; ww += 2)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[ww][v], xb[ww][v], acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[ww + 1][v], xb[ww + 1][v], acc1, 0, 0, 0);
                }
            if (ok) {
                const f4v y0 = cbo + uv, y = acc0 + acc1 + uv;
                f4v hv, F;
#pragma unroll
                for (int v = 0; v < 4; ++v) { hv[v] = fast_tanh(y0[v]); F[v] = fast_tanh(y[v]); }
                *reinterpret_cast<f4v *>(a.h + row * DH + chn) = hv;
                *reinterpret_cast<f4v *>(a.d + row * DH + chn) = (1.0f - F * F) * wdiag;
                *reinterpret_cast<f4v *>(a.r + row * DH + chn) = F - hv;
            }
            continue;
        }
        // previous state of this row: h0 (or zero) at l = 0 and for the guess, else the row before
        const float *hp = nullptr;
        if (ok) {
            if (mode == 1 || l == 0) hp = a.h0 ? a.h0 + b * DH : nullptr;
            else hp = a.h + (row - 1) * DH;
        }
        f4v xb[4];
#pragma unroll
        for (int ww = 0; ww < 4; ++ww) xb[ww] = hp ? *reinterpret_cast<const f4v *>(hp + 16 * ww + 4 * g) : zero;
        f4v uv = zero, hv = zero;
        if (ok) {
            uv = *reinterpret_cast<const f4v *>(a.u + row * DH + chn);
            if (mode != 1) hv = *reinterpret_cast<const f4v *>(a.h + row * DH + chn);
        }
        f4v acc0 = zero, acc1 = zero;
#pragma unroll
        for (int ww = 0; ww < 4; ww += 2)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[ww][v], xb[ww][v], acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[ww + 1][v], xb[ww + 1][v], acc1, 0, 0, 0);
            }
        if (ok) {
            const f4v y = acc0 + acc1 + uv;
            f4v F;
#pragma unroll
            for (int v = 0; v < 4; ++v) F[v] = fast_tanh(y[v]);
            if (mode == 1) {
                *reinterpret_cast<f4v *>(a.h + row * DH + chn) = F;
            } else if (mode == 2) {
#pragma unroll
                for (int v = 0; v < 4; ++v) nmax = nanmax(nmax, fabsf(hv[v] - F[v]));
            } else {
                *reinterpret_cast<f4v *>(a.d + row * DH + chn) = (1.0f - F * F) * wdiag;
                *reinterpret_cast<f4v *>(a.r + row * DH + chn) = F - hv;
            }
        }
    }
    if (mode == 2) {
        // one atomic per workgroup: they all go to one address
        __shared__ float s_nmax[4];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) nmax = nanmax(nmax, __shfl_xor(nmax, off, 64));
        if (lane == 0) s_nmax[w] = nmax;
        __syncthreads();
        if (threadIdx.x == 0) {
            nmax = nanmax(nanmax(s_nmax[0], s_nmax[1]), nanmax(s_nmax[2], s_nmax[3]));
            atomicMax(a.norm, nmax != nmax ? 0x7fc00000u : __float_as_uint(nmax));
        }
    }
}

__global__ __launch_bounds__(256) void dense_residual_kernel(const DenseArgs a, int mode)
{
    if (mode != 2 && a.ctrl->stop) return;
    residual_body(a, mode);
}

// ------------------------------------------------------------ chunk products
// A_c = J_e ... J_{s+1} J_s with J_l = diag(d_l) W, one wave per (b, chunk).
// Chunk 0 and the last chunk are skipped: nothing enters chunk 0 (delta_0 = 0)
// and nothing follows the last one.
__device__ __forceinline__ void chunk_products_body(const DenseArgs &a, int block)
{
    const int lane = threadIdx.x & 63, n = lane & 31, half = lane >> 5;
    const int item = block * 4 + (threadIdx.x >> 6);
    const int per_seq = a.n_c - 2;
    if (per_seq <= 0 || item >= a.B * per_seq) return;
    const int b = item / per_seq, c = 1 + item % per_seq;
    const int ls = c * CD, n_steps = min(a.L, ls + CD) - ls;

    float wr[2][2][16];
    load_w_operand(a.W, lane, wr);

    // P = J_ls in accumulator layout: P[mt][nt][v] = d[row] W[row][32 nt + n]
    f16v P[2][2], Q[2][2];
    const float *dl0 = a.d + scan_row(a, b, ls) * DH;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = 32 * mt + mfma_row(v, half);
            const float dv = dl0[row];
            P[mt][0][v] = dv * a.W[row * DH + n];
            P[mt][1][v] = dv * a.W[row * DH + 32 + n];
        }
    // dst = diag(d) W src.  The two products alternate between P and Q, so no
    // accumulator is ever copied: the result of one step is the B operand of the next.
    auto compose = [&](const f16v(&src)[2][2], f16v(&dst)[2][2], float d0, float d1) {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                for (int v = 0; v < 16; ++v) dst[mt][nt][v] = 0.0f;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float a0 = wr[0][kt][v] * d0, a1 = wr[1][kt][v] * d1;
                const float b0 = src[kt][0][v], b1 = src[kt][1][v];
                dst[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, dst[0][0], 0, 0, 0);
                dst[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, dst[0][1], 0, 0, 0);
                dst[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, dst[1][0], 0, 0, 0);
                dst[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, dst[1][1], 0, 0, 0);
            }
    };
    // row factors of the next two steps are fetched while the current two run
    // (indices clamped to the chunk: the extra values are never used)
    auto dload = [&](int i, int hi) { return a.d[scan_row(a, b, ls + min(i, n_steps - 1)) * DH + 32 * hi + n]; };
    float da0 = dload(1, 0), da1 = dload(1, 1), db0 = dload(2, 0), db1 = dload(2, 1);
    int i = 1;
#pragma unroll 1
    for (; i + 1 < n_steps; i += 2) {
        const float na0 = dload(i + 2, 0), na1 = dload(i + 2, 1), nb0 = dload(i + 3, 0), nb1 = dload(i + 3, 1);
        compose(P, Q, da0, da1);
        compose(Q, P, db0, db1);
        da0 = na0; da1 = na1; db0 = nb0; db1 = nb1;
    }
    const bool odd = i < n_steps;                 // one step left: the result ends up in Q
    if (odd) compose(P, Q, da0, da1);
    float *out = a.Ac + ((size_t)b * a.n_c + c) * DH * DH;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                out[(32 * mt + mfma_row(v, half)) * DH + 32 * nt + n] = odd ? Q[mt][nt][v] : P[mt][nt][v];
}

// ------------------------------------------- chunk products, bf16 matrix cores
// The same compositions with the operands split into bf16 terms (an inexact
// Jacobian for the Newton step: the residual stays fp32, so the solve converges to
// the same states; only the carries x_c are computed from approximate A_c).
// TERMS = 3: x = hi + lo with hi = bf16(x), lo = bf16(x - hi), and
//   W B ~ W_hi B_hi + W_hi B_lo + W_lo B_hi   (relative error ~2^-16 per product);
// TERMS = 1: W_hi B_hi only (~2^-8).
// v_mfma_f32_32x32x16_bf16 takes eight consecutive k per lane half.  As in the
// fp32 kernel the accumulator is fed back as the B operand without a layout
// change: k-slot j of lane half g of k-block kb stands for row
// 16 kb + 8 (j / 4) + 4 g + j % 4 of the 32-row block, which is accumulator
// register 8 kb + j, and W is held in registers with its columns in that order.
// The row factor d_l is applied to the fp32 result, so W's split is done once.
__device__ __forceinline__ unsigned int pack_bf16(float x0, float x1)
{
    const bf2v p = {(__bf16)x0, (__bf16)x1};
    return __builtin_bit_cast(unsigned int, p);
}

// registers 8 kb .. 8 kb + 7 of an accumulator as bf16 operand(s)
template <int TERMS>
__device__ __forceinline__ void split_operand(const f16v &x, int kb, bf8v &hi, bf8v &lo)
{
    u4v ph, pl = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float x0 = x[8 * kb + 2 * j], x1 = x[8 * kb + 2 * j + 1];
        const unsigned int pk = pack_bf16(x0, x1);
        ph[j] = pk;
        if (TERMS > 1) {
            const float h0 = __builtin_bit_cast(float, pk << 16), h1 = __builtin_bit_cast(float, pk & 0xffff0000u);
            pl[j] = pack_bf16(x0 - h0, x1 - h1);
        }
    }
    hi = __builtin_bit_cast(bf8v, ph);
    lo = __builtin_bit_cast(bf8v, pl);
}

template <int TERMS>
__device__ __forceinline__ void chunk_products_bf16_body(const DenseArgs &a, int block)
{
    const int lane = threadIdx.x & 63, n = lane & 31, half = lane >> 5;
    const int item = block * 4 + (threadIdx.x >> 6);
    const int per_seq = a.n_c - 2;
    if (per_seq <= 0 || item >= a.B * per_seq) return;
    const int b = item / per_seq, c = 1 + item % per_seq;
    const int ls = c * CD, n_steps = min(a.L, ls + CD) - ls;

    // W as A operands: whi[mt][kt][kb] slot j = W[32 mt + n][32 kt + 16 kb + 8 (j/4) + 4 half + j%4]
    bf8v whi[2][2][2], wlo[2][2][2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                f16v t;
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const f4v w4 = *reinterpret_cast<const f4v *>(a.W + (32 * mt + n) * DH + 32 * kt + 16 * kb + 8 * q + 4 * half);
#pragma unroll
                    for (int e = 0; e < 4; ++e) t[4 * q + e] = w4[e];
                }
                split_operand<TERMS>(t, 0, whi[mt][kt][kb], wlo[mt][kt][kb]);
            }

    // The row factors of the chunk go through LDS (one region per wave): rows of d arrive as
    // coalesced float4 loads and are read back in accumulator order, dq[mt][q] =
    // d[32 mt + 8 q + 4 half .. +3], the same 16 bytes for all lanes of a half.  Only this
    // wave touches its region, and a wave's LDS operations complete in order.
    __shared__ __attribute__((aligned(16))) float s_d[4][CD][DH];
    float(*sd)[DH] = s_d[threadIdx.x >> 6];
#pragma unroll
    for (int j = 0; j < CD / 4; ++j) {
        const int i = 4 * j + (lane >> 4);
        const f4v t = *reinterpret_cast<const f4v *>(a.d + scan_row(a, b, ls + min(i, n_steps - 1)) * DH + 4 * (lane & 15));
        *reinterpret_cast<f4v *>(&sd[i][4 * (lane & 15)]) = t;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    auto dload = [&](int i, f4v(&dq)[2][4]) {
        const int ii = min(i, CD - 1);                // the value past the last step is never used
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int q = 0; q < 4; ++q) dq[mt][q] = *reinterpret_cast<const f4v *>(&sd[ii][32 * mt + 8 * q + 4 * half]);
    };
    // acc = J_ls in accumulator layout: acc[mt][nt][v] = d[row] W[row][32 nt + n]
    f16v acc[2][2];
    {
        f4v d0[2][4];
        dload(0, d0);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = 32 * mt + mfma_row(v, half);
                const float dv = d0[mt][v >> 2][v & 3];
                acc[mt][0][v] = dv * a.W[row * DH + n];
                acc[mt][1][v] = dv * a.W[row * DH + 32 + n];
            }
    }
    f4v dcur[2][4], dnext[2][4];
    dload(1, dcur);
#pragma unroll 1
    for (int i = 1; i < n_steps; ++i) {
        dload(i + 1, dnext);
        bf8v bhi[2][2][2], blo[2][2][2];              // [kt][nt][kb]
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) split_operand<TERMS>(acc[kt][nt], kb, bhi[kt][nt][kb], blo[kt][nt][kb]);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                f16v s;
#pragma unroll
                for (int v = 0; v < 16; ++v) s[v] = 0.0f;
                if (TERMS > 1) {
                    // the small terms first
#pragma unroll
                    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                        for (int kb = 0; kb < 2; ++kb) {
                            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(whi[mt][kt][kb], blo[kt][nt][kb], s, 0, 0, 0);
                            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wlo[mt][kt][kb], bhi[kt][nt][kb], s, 0, 0, 0);
                        }
                }
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb)
                        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(whi[mt][kt][kb], bhi[kt][nt][kb], s, 0, 0, 0);
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[mt][nt][v] = s[v] * dcur[mt][v >> 2][v & 3];
            }
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int q = 0; q < 4; ++q) dcur[mt][q] = dnext[mt][q];
    }
    float *out = a.Ac + ((size_t)b * a.n_c + c) * DH * DH;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int v = 0; v < 16; ++v) out[(32 * mt + mfma_row(v, half)) * DH + 32 * nt + n] = acc[mt][nt][v];
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
// x <- diag(d_l) (W x) + r_l over the CD steps of a chunk.  The chain is
// sequential, so what counts is the latency of one step; every (sequence,
// chunk) pair is an independent column, and one workgroup advances 16 columns
// with the 64 x 64 x 16 product of a step split over its four waves: wave w
// owns rows 16w .. 16w+15 and issues 16 v_mfma_f32_16x16x4_f32.
//
// Operand layout: the 16x16 accumulator gives lane (n = lane % 16, g = lane / 16)
// the rows 16w + 4g + v, v = 0..3, of column n.  Each wave drops its float4 into
// LDS at [w][lane]; for the next step every wave reads the four float4 at
// [ww][lane], ww = 0..3, and uses component v of wave ww's value as the B
// operand of k-step (ww, v), whose four k-slots (one per lane group g) are then
// the rows 16ww + 4g + v.  W is held in registers in the matching A-operand
// order, so the exchange is one float4 write and four conflict-free float4
// reads per step, with no index arithmetic.
//
// d and r (and h) of all CD steps are loaded before the chain starts; the barrier
// between steps orders LDS only.
// final = 0: x starts at 0, only the end value is kept (b_c).
// final = 1: x starts at x_{c-1}; afterwards h += delta and max|delta|.
// BWD: the backward recurrence (r_l = d_l * g_l; the final sweep writes mu = dL/du and nothing else).
// LATE_H: the iterate's rows are read after the chain instead of before it (48 fewer registers held
// through the chain; the one-launch solve shares its register budget with the chunk products).
//
// Forward solves: the delta of a chunk's last step exists twice, as the end of this chain and as the carried
// value x_c that every later chunk started from; the update takes x_c, so that the iterate at a chunk's last
// step is (old value + x_c), which the next chunk's column can form by itself.  The chunk-local sweep leaves the
// old values of those steps in a.hend for that purpose (the final sweeps of neighbouring chunks run side by side
// and update h in place).
// NEXT (final forward sweep): the residual and row factors of the NEXT iteration are formed here, from the
// new rows this column holds, instead of by a launch of their own that would read the iterate again:
// row l needs the new h_{l-1} (for l = ls: hend + x_{c-1}, or h0) and the new h_l.  Same products in the same
// order as dense_residual_kernel, so both give the same bits.
template <int FINAL, bool BWD, bool LATE_H = false, bool NEXT = false>
__device__ __forceinline__ void sweep_body(const DenseArgs &a, int block)
{
    static_assert(!NEXT || (FINAL && !BWD && !LATE_H), "the next residual belongs to the forward final sweep");
    __shared__ f4v s_x[2][4][64];
    __shared__ float s_max[4];
    const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int n = lane & 15, g = lane >> 4;
    const int n_cols = a.B * a.n_c;
    const int col = block * 16 + n;
    const bool ok = col < n_cols;
    const int cc = ok ? col : n_cols - 1;         // a column past the end reads valid memory and stores nothing
    const int b = cc / a.n_c, c = cc - b * a.n_c;
    const int ls = c * CD;
    const int chn = 16 * w + 4 * g;               // first of this lane's four channels

    float wa[4][4];
    load_w_operand16(a.W, w, n, g, wa);
    const f4v zero = {0.0f, 0.0f, 0.0f, 0.0f};
    f4v dv[CD], rv[CD], hv[(FINAL && !BWD && !LATE_H) ? CD : 1];
#pragma unroll
    for (int i = 0; i < CD; ++i) {
        const int l = ls + i;
        const size_t off = scan_row(a, b, min(l, a.L - 1)) * DH + chn;
        dv[i] = *reinterpret_cast<const f4v *>(a.d + off);
        if (BWD) rv[i] = dv[i] * *reinterpret_cast<const f4v *>(a.g + off);
        else rv[i] = *reinterpret_cast<const f4v *>(a.r + off);
        if (FINAL && !BWD && !LATE_H) hv[i] = *reinterpret_cast<const f4v *>(a.h + off);
        if (!(ok && l < a.L)) { dv[i] = zero; rv[i] = zero; }     // steps past the end leave x = 0
    }
    f4v x = zero;
    if (FINAL && ok && c > 0) x = *reinterpret_cast<const f4v *>(a.xc + ((size_t)b * a.n_c + (c - 1)) * DH + chn);
    // forward: the carried delta of this chunk's last step, and (chunk-local sweep) the iterate there
    const bool carried_end = !BWD && a.hend && ok && c < a.n_c - 1;
    f4v xend = zero;
    if (FINAL && carried_end) xend = *reinterpret_cast<const f4v *>(a.xc + ((size_t)b * a.n_c + c) * DH + chn);
    if (!FINAL && carried_end)
        *reinterpret_cast<f4v *>(a.hend + ((size_t)b * a.n_c + c) * DH + chn) =
            *reinterpret_cast<const f4v *>(a.h + ((size_t)b * a.L + ls + CD - 1) * DH + chn);
    const f4v xstart = x;
    s_x[0][w][lane] = x;
    lds_barrier();
#pragma unroll
    for (int i = 0; i < CD; ++i) {
        f4v acc0 = zero, acc1 = zero;
#pragma unroll
        for (int ww = 0; ww < 4; ww += 2) {
            const f4v xa = s_x[i & 1][ww][lane], xb = s_x[i & 1][ww + 1][lane];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[ww][v], xa[v], acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[ww + 1][v], xb[v], acc1, 0, 0, 0);
            }
        }
        x = dv[i] * (acc0 + acc1) + rv[i];
        if (FINAL) rv[i] = x;                     // delta_l, applied to h after the chain
        if (i + 1 < CD) {
            s_x[(i + 1) & 1][w][lane] = x;
            lds_barrier();
        }
    }
    if (!FINAL) {
        if (ok) *reinterpret_cast<f4v *>(a.bc + ((size_t)b * a.n_c + c) * DH + chn) = x;
        return;
    }
    if (BWD) {
#pragma unroll
        for (int i = 0; i < CD; ++i) {
            const int l = ls + i;
            if (ok && l < a.L) *reinterpret_cast<f4v *>(a.du + scan_row(a, b, l) * DH + chn) = rv[i];
        }
        return;
    }
    if (carried_end) rv[CD - 1] = xend;
    float wmax = 0.0f;
    if constexpr (NEXT) {
        // u of this column's rows (the registers of the row factors are free now)
        f4v uv[CD];
#pragma unroll
        for (int i = 0; i < CD; ++i)
            uv[i] = *reinterpret_cast<const f4v *>(a.u + ((size_t)b * a.L + min(ls + i, a.L - 1)) * DH + chn);
        // the state in front of the column's first row
        f4v hprev = zero;
        if (ok) {
            if (c == 0) {
                if (a.h0) hprev = *reinterpret_cast<const f4v *>(a.h0 + (size_t)b * DH + chn);
            } else {
                hprev = *reinterpret_cast<const f4v *>(a.hend + ((size_t)b * a.n_c + (c - 1)) * DH + chn) + xstart;
            }
        }
        // every wave needs all 64 values of each state: slot i holds the state in front of row i
        __shared__ f4v s_h[CD][4][64];
        s_h[0][w][lane] = hprev;
#pragma unroll
        for (int i = 0; i < CD; ++i) {
            const int l = ls + i;
#pragma unroll
            for (int v = 0; v < 4; ++v) wmax = nanmax(wmax, __builtin_fabsf(rv[i][v]));
            rv[i] = hv[i] + rv[i];                                  // the new row
            if (ok && l < a.L) *reinterpret_cast<f4v *>(a.h + ((size_t)b * a.L + l) * DH + chn) = rv[i];
            if (i + 1 < CD) s_h[i + 1][w][lane] = rv[i];
        }
        lds_barrier();
#pragma unroll
        for (int i = 0; i < CD; ++i) {
            const int l = ls + i;
            f4v acc0 = zero, acc1 = zero;
#pragma unroll
            for (int ww = 0; ww < 4; ww += 2) {
                const f4v xa = s_h[i][ww][lane], xb = s_h[i][ww + 1][lane];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[ww][v], xa[v], acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[ww + 1][v], xb[v], acc1, 0, 0, 0);
                }
            }
            if (ok && l < a.L) {
                const f4v y = acc0 + acc1 + uv[i];
                f4v F;
#pragma unroll
                for (int v = 0; v < 4; ++v) F[v] = fast_tanh(y[v]);
                const size_t off = ((size_t)b * a.L + l) * DH + chn;
                *reinterpret_cast<f4v *>(a.d + off) = (1.0f - F * F);
                *reinterpret_cast<f4v *>(a.r + off) = F - rv[i];
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < CD; ++i) {
            const int l = ls + i;
            if (ok && l < a.L) {
                f4v *hp = reinterpret_cast<f4v *>(a.h + ((size_t)b * a.L + l) * DH + chn);
                if (LATE_H) *hp = *hp + rv[i];
                else *hp = hv[i] + rv[i];
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) wmax = nanmax(wmax, __builtin_fabsf(rv[i][v]));
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) wmax = nanmax(wmax, __shfl_xor(wmax, off, 64));
    if (lane == 0) s_max[w] = wmax;
    __syncthreads();
    if (threadIdx.x == 0) {
        const float bm = nanmax(nanmax(s_max[0], s_max[1]), nanmax(s_max[2], s_max[3]));
        if (a.gmax) atomicMax(a.gmax, __float_as_uint(bm));       // the one-launch solve decides after its barrier
        else finish_iteration(a, bm);
    }
}

// The final sweep of an iteration (or of the backward pass).  NEXT: it also leaves the residual and the row
// factors of the next iteration.
template <bool BWD, bool NEXT = false>
__global__ __launch_bounds__(256) void dense_final_sweep_kernel(const DenseArgs a)
{
    if (a.ctrl->stop) return;
    sweep_body<1, BWD, false, NEXT>(a, blockIdx.x);
}

// Chunk products and chunk-local sweeps need only d and r, and nothing of each
// other: one launch runs both.  The first n_sweep workgroups take the sweeps,
// whose sequential chains are bound by latency and so start first; the rest
// compose the chunk products, which keep the matrix cores busy meanwhile.
// PROD: how the chunk products are formed: 0 fp32, 1 three bf16 terms, 2 one bf16 term
template <bool BWD, int PROD>
__global__ __launch_bounds__(256, 2) void dense_products_sweep_kernel(const DenseArgs a, int n_sweep)
{
    if (a.ctrl->stop) return;
    if ((int)blockIdx.x < n_sweep) sweep_body<0, BWD>(a, blockIdx.x);
    else if (PROD == 0) chunk_products_body(a, (int)blockIdx.x - n_sweep);
    else chunk_products_bf16_body<PROD == 1 ? 3 : 1>(a, (int)blockIdx.x - n_sweep);
}

// process-wide choice of the product arithmetic of forward solves (pararnn_set_dense_products)
int g_dense_products = 0;
int g_dense_jacobian = 0;       // 0: the full Jacobian (Newton), 1: its diagonal (quasi-Newton)
int g_dense_one_launch = 1;     // 1: the first kDenseHead iterations as launches per phase, the rest in one persistent
                                // launch; 0: launches per phase throughout; 2: the persistent launch from the start
constexpr int kDenseHead = 6;


void launch_products_sweep(int prod, int blocks, hipStream_t st, const DenseArgs &a, int n_sweep)
{
    if (prod == 1) hipLaunchKernelGGL((dense_products_sweep_kernel<false, 1>), dim3(blocks), dim3(256), 0, st, a, n_sweep);
    else if (prod == 2) hipLaunchKernelGGL((dense_products_sweep_kernel<false, 2>), dim3(blocks), dim3(256), 0, st, a, n_sweep);
    else hipLaunchKernelGGL((dense_products_sweep_kernel<false, 0>), dim3(blocks), dim3(256), 0, st, a, n_sweep);
}

// --------------------------------------------------------------------- carry
// x_c = A_c x_{c-1} + b_c for c = 0 .. n_c-2 (x_{-1} = 0, so x_0 = b_0), one
// workgroup per sequence.  Lane (row = lane / 4, q = lane % 4) of wave w holds
// columns 16j + 4q .. 16j + 4q + 3, j = 0..3, of row 16w + row of A_c (so that the
// four lanes of a quad load 64 contiguous bytes at a time): sixteen FMAs against x from
// LDS, two DPP adds across the quad, and the row's new value goes back to LDS.
// The matrices of the next DEPTH chunks are in flight meanwhile; the loop body
// is branch-free around the loads (indices are clamped) and its barrier orders
// LDS only, so those loads stay outstanding across steps.
__device__ __forceinline__ void carry_body(const DenseArgs &a, int b)
{
    constexpr int DEPTH = 8;
    __shared__ __attribute__((aligned(16))) float s_x[2][DH];
    const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int row = 16 * w + (lane >> 2), q = lane & 3;
    const float *bcb = a.bc + (size_t)b * a.n_c * DH + row;
    float *xcb = a.xc + (size_t)b * a.n_c * DH + row;
    const float *Ab = a.Ac + ((size_t)b * a.n_c * DH + row) * DH + 4 * q;    // this lane's first columns, chunk 0
    const int last = a.n_c - 2;                       // last chunk whose end value is needed
    {
        const float x0 = bcb[0];
        if (q == 0) { s_x[0][row] = x0; xcb[0] = x0; }
    }
    if (last < 1) return;
    f4v buf[DEPTH][4];
    float bb[DEPTH];
#pragma unroll
    for (int k = 0; k < DEPTH; ++k) {
        const int c = min(1 + k, last);
#pragma unroll
        for (int j = 0; j < 4; ++j) buf[k][j] = *reinterpret_cast<const f4v *>(Ab + (size_t)c * DH * DH + 16 * j);
        bb[k] = bcb[(size_t)c * DH];
    }
    lds_barrier();
    int cur = 0;
    for (int base = 1; base <= last; base += DEPTH) {
#pragma unroll
        for (int k = 0; k < DEPTH; ++k) {
            const int c = base + k;
            const f4v *xs = reinterpret_cast<const f4v *>(&s_x[cur][4 * q]);
            f4v s = buf[k][0] * xs[0];
#pragma unroll
            for (int j = 1; j < 4; ++j) s = buf[k][j] * xs[4 * j] + s;
            float t = (s[0] + s[1]) + (s[2] + s[3]);
            t += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, t), 0xB1, 0xf, 0xf, false));
            t += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, t), 0x4E, 0xf, 0xf, false));
            const float xn = t + bb[k];
            // past the last chunk nothing is written and the buffers do not flip
            if (c <= last) {
                if (q == 0) { s_x[cur ^ 1][row] = xn; xcb[(size_t)c * DH] = xn; }
                cur ^= 1;
            }
            const int cn = min(c + DEPTH, last);
#pragma unroll
            for (int j = 0; j < 4; ++j) buf[k][j] = *reinterpret_cast<const f4v *>(Ab + (size_t)cn * DH * DH + 16 * j);
            bb[k] = bcb[(size_t)cn * DH];
            lds_barrier();
        }
    }
}

__global__ __launch_bounds__(256) void dense_carry_kernel(const DenseArgs a)
{
    if (a.ctrl->stop) return;
    carry_body(a, blockIdx.x);
}

// ------------------------------------------------- the whole solve in one launch
// Newton iterations of a forward solve in ONE persistent launch: the phases of an
// iteration (residual; chunk products + chunk-local sweeps; carry; final sweep) are
// separated by grid-wide barriers instead of kernel boundaries, the stopping test is
// taken by every workgroup from the same device-wide maximum right after the last
// barrier of an iteration, and the launch ends with the iteration that met the
// tolerance: no launch is enqueued for iterations that never run.  The grid is what
// the device holds at once (every workgroup is resident, so every barrier is reached
// by all of them); a barrier wait is bounded like the look-back waits of the scan
// kernels and ends the launch with status INTERNAL if it ever runs out.
//
// Words 16.. of the control block: [0], [1] max|delta| bits of odd / even iterations,
// [2] barrier arrivals (monotone), [3] ticket of the chunk-product workgroup items.
__device__ __forceinline__ bool grid_barrier(unsigned int *arrivals, unsigned int &generation, unsigned int spin_limit)
{
    __shared__ int s_ok;
    __syncthreads();
    if (threadIdx.x == 0) {
        __threadfence();                              // this workgroup's writes, before it arrives
        ++generation;
        const unsigned int target = generation * gridDim.x;
        atomicAdd(arrivals, 1u);
        unsigned int spins = 0;
        int ok = 1;
        while (__hip_atomic_load(arrivals, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            if (++spins >= spin_limit) { ok = 0; break; }
            __builtin_amdgcn_s_sleep(16);             // about half a microsecond: hundreds of workgroups poll one word
        }
        __threadfence();                              // the others' writes, after all have arrived
        s_ok = ok;
    }
    __syncthreads();
    return s_ok != 0;
}

// Each phase is a function of its own (not inlined): the phases keep W and their row addresses
// in registers in different layouts, and inlined into one body the compiler would carry all of
// them through the whole iteration loop and spill.  A phase reads the launch's arguments from the
// kernel-argument block and gets what changes per iteration by value.
__device__ __attribute__((noinline)) void phase_residual(const DenseArgs *ap, int mode)
{
    const DenseArgs a = *ap;
    residual_body(a, mode);
}

template <int PROD>
__device__ __attribute__((noinline)) void phase_products_sweeps(const DenseArgs *ap, unsigned int *ticket, int n_sweep,
                                                              int n_prod_blocks)
{
    __shared__ unsigned int s_t;
    const DenseArgs a = *ap;
    // chunk-local sweeps first (sequential chains, bound by latency), then the chunk products,
    // handed out by a ticket so that the workgroups that swept do not finish last
    for (int blk = blockIdx.x; blk < n_sweep; blk += gridDim.x) {
        sweep_body<0, false>(a, blk);
        __syncthreads();
    }
    for (;;) {
        if (threadIdx.x == 0) s_t = atomicAdd(ticket, 1u);
        __syncthreads();
        const unsigned int t = __builtin_amdgcn_readfirstlane(s_t);
        __syncthreads();
        if (t >= (unsigned int)n_prod_blocks) break;
        if (PROD == 0) chunk_products_body(a, (int)t);
        else chunk_products_bf16_body<PROD == 1 ? 3 : 1>(a, (int)t);
    }
}

__device__ __attribute__((noinline)) void phase_carry(const DenseArgs *ap)
{
    const DenseArgs a = *ap;
    for (int b = blockIdx.x; b < a.B; b += gridDim.x) {
        carry_body(a, b);
        __syncthreads();
    }
}

__device__ __attribute__((noinline)) void phase_final_sweep(const DenseArgs *ap, unsigned int *gmax, int n_sweep)
{
    DenseArgs a = *ap;
    a.gmax = gmax;
    for (int blk = blockIdx.x; blk < n_sweep; blk += gridDim.x) {
        sweep_body<1, false, true>(a, blk);
        __syncthreads();
    }
}

// k_first = 1: the solve from the initial guess; k_first > 1: iterations k_first .. max_iter of a
// solve whose earlier iterations ran as separate launches (nothing to do when one of them ended it).
template <int PROD>
__global__ __launch_bounds__(256, 2) void dense_newton_kernel(const DenseArgs a, int n_sweep, int n_prod_blocks,
                                                              int k_first)
{
    Ctrl *ctrl = a.ctrl;
    if (ctrl->stop) return;
    unsigned int *aux = reinterpret_cast<unsigned int *>(ctrl) + 16;
    unsigned int generation = 0;
    bool alive = true;
    if (k_first == 1) {
        // initial guess h^0_l = tanh(W h0 + u_l) (App. A); rows are independent
        phase_residual(&a, 1);
        alive = grid_barrier(aux + 2, generation, a.spin_limit);
    }
    int k = k_first;
    for (; alive && k <= a.max_iter; ++k) {
        unsigned int *gmax = aux + (k & 1);
        phase_residual(&a, 0);
        if (!(alive = grid_barrier(aux + 2, generation, a.spin_limit))) break;
        phase_products_sweeps<PROD>(&a, aux + 3, n_sweep, n_prod_blocks);
        if (!(alive = grid_barrier(aux + 2, generation, a.spin_limit))) break;
        phase_carry(&a);
        if (!(alive = grid_barrier(aux + 2, generation, a.spin_limit))) break;
        phase_final_sweep(&a, gmax, n_sweep);
        if (!(alive = grid_barrier(aux + 2, generation, a.spin_limit))) break;
        // every workgroup reads the same maximum and takes the same decision
        const float mk = __uint_as_float(__hip_atomic_load(gmax, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        int status, stop = 0;
        if (!(mk - mk == 0.0f)) { status = kStNonFinite; stop = 1; }
        else if (a.tol >= 0.0f && mk <= a.tol) { status = kStOk; stop = 1; }
        else status = a.tol < 0.0f ? kStOk : kStNotConverged;
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            if (a.trace) a.trace[k - 1] = mk;
            a.iters_out[0] = k;
            a.iters_out[1] = status;
            ctrl->iters = k;
            ctrl->status = status;
            ctrl->stop = stop;
            // for the next iteration: its maximum slot was last read two iterations ago, and the
            // product ticket is not drawn again before two more barriers
            aux[(k + 1) & 1] = 0u;
            aux[3] = 0u;
        }
        if (stop) break;
    }
    if (!alive && threadIdx.x == 0) {
        atomicExch(&ctrl->status, kStInternal);
        a.iters_out[1] = kStInternal;
    }
}

void launch_newton(int prod, int grid, hipStream_t st, const DenseArgs &a, int n_sweep, int n_prod_blocks, int k_first)
{
    if (prod == 1) hipLaunchKernelGGL((dense_newton_kernel<1>), dim3(grid), dim3(256), 0, st, a, n_sweep, n_prod_blocks, k_first);
    else if (prod == 2) hipLaunchKernelGGL((dense_newton_kernel<2>), dim3(grid), dim3(256), 0, st, a, n_sweep, n_prod_blocks, k_first);
    else hipLaunchKernelGGL((dense_newton_kernel<0>), dim3(grid), dim3(256), 0, st, a, n_sweep, n_prod_blocks, k_first);
}

// workgroups of the one-launch solve: what the device holds at once
int newton_grid(int prod)
{
    static int cap[3] = {0, 0, 0};
    if (cap[prod] == 0) {
        int per_cu = 0;
        hipError_t e;
        if (prod == 1) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, dense_newton_kernel<1>, 256, 0);
        else if (prod == 2) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, dense_newton_kernel<2>, 256, 0);
        else e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, dense_newton_kernel<0>, 256, 0);
        if (e != hipSuccess || per_cu < 1) per_cu = 1;
        cap[prod] = per_cu * device_cu_count();
    }
    return cap[prod];
}

// ------------------------------------------------------------ backward extras
// Wt = W^T (16 KB)
__global__ __launch_bounds__(256) void dense_transpose_kernel(const float *W, float *Wt)
{
    for (int i = threadIdx.x; i < DH * DH; i += 256) Wt[(i % DH) * DH + i / DH] = W[i];
}

// dL/dh0[b] = W^T mu_{b,0}: thread j sums over the rows i of W
__global__ __launch_bounds__(64) void dense_dh0_kernel(const float *W, const float *mu, int L, float *dh0)
{
    const int b = blockIdx.x, j = threadIdx.x;
    const float *m = mu + (size_t)b * L * DH;
    float s = 0.0f;
    for (int i = 0; i < DH; ++i) s = fmaf(W[i * DH + j], m[i], s);
    dh0[(size_t)b * DH + j] = s;
}

// Partial sums of dL/dW = sum over rows (b, l) of mu_l h_{l-1}^T: wave p sums its
// contiguous share of the rows as 64 x 64 x (rows) products on
// v_mfma_f32_32x32x2_f32 (two rows per instruction: A = mu, B = h_{l-1}) and
// writes part[p][64][64]; the partials are added in a fixed order afterwards.
__global__ __launch_bounds__(256) void dense_dw_kernel(const DenseArgs a, float *part, int rows_per_wave)
{
    const int lane = threadIdx.x & 63, n = lane & 31, half = lane >> 5;
    const int p = blockIdx.x * 4 + (threadIdx.x >> 6);
    const size_t rows = (size_t)a.B * a.L;
    const size_t r0 = (size_t)p * rows_per_wave;
    const size_t r1 = r0 + rows_per_wave < rows ? r0 + rows_per_wave : rows;
    f16v Q[2][2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int v = 0; v < 16; ++v) Q[mt][nt][v] = 0.0f;
    for (size_t r = r0; r < r1; r += 2) {
        const size_t row = r + half;               // this lane half's row of the pair
        const bool ok = row < r1;
        float m0 = 0.0f, m1 = 0.0f, h0v = 0.0f, h1v = 0.0f;
        if (ok) {
            m0 = a.du[row * DH + n];
            m1 = a.du[row * DH + 32 + n];
            const int l = (int)(row % a.L);
            const float *hp = l == 0 ? (a.h0 ? a.h0 + (row / a.L) * DH : nullptr) : a.h + (row - 1) * DH;
            if (hp) { h0v = hp[n]; h1v = hp[32 + n]; }
        }
        Q[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(m0, h0v, Q[0][0], 0, 0, 0);
        Q[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(m0, h1v, Q[0][1], 0, 0, 0);
        Q[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(m1, h0v, Q[1][0], 0, 0, 0);
        Q[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(m1, h1v, Q[1][1], 0, 0, 0);
    }
    float *out = part + (size_t)p * DH * DH;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int v = 0; v < 16; ++v) out[(32 * mt + mfma_row(v, half)) * DH + 32 * nt + n] = Q[mt][nt][v];
}

size_t r256(size_t x) { return (x + 255) & ~(size_t)255; }

struct DenseLayout { size_t off_d, off_r, off_A, off_b, off_x, off_hend, total; int n_c; };

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
    lo.off_hend = off; off += r256((size_t)B * lo.n_c * DH * 4);
    lo.total = off;
    return lo;
}

}  // namespace

int dense_chunk() { return CD; }

int dense_set_products(int mode)
{
    if (mode < 0 || mode > 2) return PARARNN_INVALID_ARG;
    g_dense_products = mode;
    return PARARNN_OK;
}

int dense_set_one_launch(int mode)
{
    if (mode < 0 || mode > 2) return PARARNN_INVALID_ARG;
    g_dense_one_launch = mode;
    return PARARNN_OK;
}

int dense_set_jacobian(int mode)
{
    if (mode < 0 || mode > 1) return PARARNN_INVALID_ARG;
    g_dense_jacobian = mode;
    return PARARNN_OK;
}

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
        launch_products_sweep(g_dense_products, (n_prod + 3) / 4, st, a, 0);
    return hipGetLastError() == hipSuccess ? PARARNN_OK : PARARNN_HIP_ERROR;
}

// waves that share the rows of the dL/dW reduction (a multiple of 4: whole workgroups)
int dw_waves(int B, int L)
{
    const size_t rows = (size_t)B * L;
    size_t wv = (rows + 63) / 64;                 // at least 64 rows per wave
    if (wv > 1024) wv = 1024;
    return (int)((wv + 3) / 4 * 4);
}

size_t dense_workspace_bytes(int dtype, int B, int L, int H, int backward)
{
    if (dtype != PARARNN_F32 || H != DH) return 256;
    const DenseLayout lo = dense_layout(B, L);
    if (!backward) return lo.total;
    // the forward layout, then W^T and the dL/dW partials
    return lo.total + r256((size_t)DH * DH * 4) + r256((size_t)dw_waves(B, L) * DH * DH * 4);
}

int dense_backward(int dtype, const float *W, const void *u, const void *h0, const void *h, const void *g, int B,
                   int L, int H, void *du, float *dW, void *dh0, void *workspace, size_t workspace_bytes,
                   hipStream_t st)
{
    if (dtype != PARARNN_F32 || H != DH) return PARARNN_UNSUPPORTED;
    if (((uintptr_t)W | (uintptr_t)u | (uintptr_t)h | (uintptr_t)h0 | (uintptr_t)g | (uintptr_t)du) % 16)
        return PARARNN_UNSUPPORTED;
    if (workspace_bytes < dense_workspace_bytes(dtype, B, L, H, 1)) return PARARNN_WORKSPACE_TOO_SMALL;
    const DenseLayout lo = dense_layout(B, L);
    char *ws = static_cast<char *>(workspace);
    float *Wt = reinterpret_cast<float *>(ws + lo.total);
    float *part = reinterpret_cast<float *>(ws + lo.total + r256((size_t)DH * DH * 4));
    DenseArgs a;
    memset(&a, 0, sizeof(a));
    a.u = static_cast<const float *>(u); a.h0 = static_cast<const float *>(h0);
    a.h = const_cast<float *>(static_cast<const float *>(h));       // only read on this path
    a.d = reinterpret_cast<float *>(ws + lo.off_d);
    a.r = reinterpret_cast<float *>(ws + lo.off_r);
    a.Ac = reinterpret_cast<float *>(ws + lo.off_A);
    a.bc = reinterpret_cast<float *>(ws + lo.off_b);
    a.xc = reinterpret_cast<float *>(ws + lo.off_x);
    a.ctrl = reinterpret_cast<Ctrl *>(ws);
    a.g = static_cast<const float *>(g); a.du = static_cast<float *>(du);
    a.B = B; a.L = L; a.n_c = lo.n_c;
    if (launch_reset(a.ctrl, nullptr, 0, nullptr, 0, st) != hipSuccess) return PARARNN_HIP_ERROR;
    hipLaunchKernelGGL(dense_transpose_kernel, dim3(1), dim3(256), 0, st, W, Wt);
    // d_l = 1 - tanh^2(W h_{l-1} + u_l) at the given states (forward addressing, W itself)
    const size_t res_items = ((size_t)B * L + 15) / 16;
    const size_t res_cap = (size_t)device_cu_count() * 8;
    const int res_blocks = (int)(res_items < res_cap ? res_items : res_cap);
    a.W = W; a.rev = 0;
    hipLaunchKernelGGL(dense_residual_kernel, dim3(res_blocks), dim3(256), 0, st, a, 0);
    // the reverse scan with W^T
    a.W = Wt; a.rev = 1;
    const int n_prod = B * (lo.n_c - 2);
    const int n_sweep = (B * lo.n_c + 15) / 16;
    const int n_prod_blocks = n_prod > 0 ? (n_prod + 3) / 4 : 0;
    // always fp32 products: this is one linear solve, not an iteration that would correct an inexact one
    hipLaunchKernelGGL((dense_products_sweep_kernel<true, 0>), dim3(n_sweep + n_prod_blocks), dim3(256), 0, st, a, n_sweep);
    hipLaunchKernelGGL(dense_carry_kernel, dim3(B), dim3(256), 0, st, a);
    hipLaunchKernelGGL(dense_final_sweep_kernel<true>, dim3(n_sweep), dim3(256), 0, st, a);
    // step-local gradients
    if (dh0) hipLaunchKernelGGL(dense_dh0_kernel, dim3(B), dim3(64), 0, st, W, a.du, L, static_cast<float *>(dh0));
    const int wv = dw_waves(B, L);
    const size_t rows = (size_t)B * L;
    int rows_per_wave = (int)((rows + wv - 1) / wv);
    rows_per_wave += rows_per_wave & 1;           // pairs of rows
    hipLaunchKernelGGL(dense_dw_kernel, dim3(wv / 4), dim3(256), 0, st, a, part, rows_per_wave);
    if (hipGetLastError() != hipSuccess) return PARARNN_HIP_ERROR;
    return launch_param_reduce(part, dW, wv, DH * DH, st) == hipSuccess ? PARARNN_OK : PARARNN_HIP_ERROR;
}

int dense_residual_norm(int dtype, const float *W, const void *u, const void *h0, const void *h, int B, int L, int H,
                        float *out, hipStream_t st)
{
    if (dtype != PARARNN_F32 || H != DH) return PARARNN_UNSUPPORTED;
    if (((uintptr_t)W | (uintptr_t)u | (uintptr_t)h | (uintptr_t)h0) % 16) return PARARNN_UNSUPPORTED;
    DenseArgs a;
    memset(&a, 0, sizeof(a));
    a.W = W; a.u = static_cast<const float *>(u); a.h0 = static_cast<const float *>(h0);
    a.h = const_cast<float *>(static_cast<const float *>(h));        // mode 2 only reads it
    a.B = B; a.L = L;
    a.norm = reinterpret_cast<unsigned int *>(out);
    if (launch_zero_words(a.norm, 1, st) != hipSuccess) return PARARNN_HIP_ERROR;
    const size_t res_items = ((size_t)B * L + 15) / 16;
    const size_t res_cap = (size_t)device_cu_count() * 4;
    const int res_blocks = (int)(res_items < res_cap ? res_items : res_cap);
    hipLaunchKernelGGL(dense_residual_kernel, dim3(res_blocks), dim3(256), 0, st, a, 2);
    return hipGetLastError() == hipSuccess ? PARARNN_OK : PARARNN_HIP_ERROR;
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
    memset(&a, 0, sizeof(a));
    a.W = W; a.u = static_cast<const float *>(u); a.h0 = static_cast<const float *>(h0);
    a.h = static_cast<float *>(h);
    a.d = reinterpret_cast<float *>(ws + lo.off_d);
    a.r = reinterpret_cast<float *>(ws + lo.off_r);
    a.Ac = reinterpret_cast<float *>(ws + lo.off_A);
    a.bc = reinterpret_cast<float *>(ws + lo.off_b);
    a.xc = reinterpret_cast<float *>(ws + lo.off_x);
    a.hend = reinterpret_cast<float *>(ws + lo.off_hend);
    a.ctrl = reinterpret_cast<Ctrl *>(ws);
    a.iters_out = iters; a.trace = delta_trace;
    a.B = B; a.L = L; a.n_c = lo.n_c; a.k = 0; a.max_iter = max_iter; a.tol = tol;

    const int status0 = tol < 0.0f ? PARARNN_OK : PARARNN_NOT_CONVERGED;
    const size_t res_items = ((size_t)B * L + 15) / 16;           // one workgroup per 16 rows, a few rounds at most
    const size_t res_cap = (size_t)device_cu_count() * 8;
    const int res_blocks = (int)(res_items < res_cap ? res_items : res_cap);
    if (g_dense_jacobian == 1) {
        // Quasi-Newton: J_l is replaced by its diagonal (1 - F_l^2) * W_ii, so the linear solve is the
        // diagonal scan over 64 independent channels per sequence; no matrix products.  The scan adds
        // its result to h itself; its carry records live where the chunk products would (always
        // large enough).
        const CellInfo ci = {1, 1, 0, -1};
        const Layout sl = make_layout(ci, PARARNN_F32, B, L, DH, false, 4);
        unsigned long long *rec = reinterpret_cast<unsigned long long *>(ws + lo.off_A);
        if (lo.off_A + sl.n_rec * sizeof(unsigned long long) > lo.off_b) return PARARNN_WORKSPACE_TOO_SMALL;   // cannot happen: 24 B of records per 64 steps against 16 KB of products per 16
        if (launch_reset(a.ctrl, rec, sl.n_rec, iters, status0, st) != hipSuccess) return PARARNN_HIP_ERROR;
        hipLaunchKernelGGL(dense_residual_kernel, dim3(res_blocks), dim3(256), 0, st, a, 1);
        FwdArgs f;
        memset(&f, 0, sizeof(f));
        f.g = sl.g;
        f.u = a.r; f.jac = a.d; f.hit = a.h; f.raw_add = 1;
        f.rec = rec; f.ctrl = a.ctrl;
        f.iters_out = iters; f.trace = delta_trace;
        f.max_iter = max_iter; f.tol = tol;
        for (int k = 1; k <= max_iter; ++k) {
            hipLaunchKernelGGL(dense_residual_kernel, dim3(res_blocks), dim3(256), 0, st, a, 3);
            f.k = k;
            const hipError_t e = Kernels<RawScan<1>, float>::newton_iter(sl.cfg, f, false, st);
            if (e != hipSuccess) return PARARNN_HIP_ERROR;
        }
        return hipGetLastError() == hipSuccess ? PARARNN_OK : PARARNN_HIP_ERROR;
    }
    if (launch_reset(a.ctrl, nullptr, 0, iters, status0, st) != hipSuccess) return PARARNN_HIP_ERROR;
    const int n_prod = B * (lo.n_c - 2);
    const int n_prod_blocks = n_prod > 0 ? (n_prod + 3) / 4 : 0;
    const int n_sweep = (B * lo.n_c + 15) / 16;       // workgroups: 16 (sequence, chunk) columns each
    // Launch plan.  The first iterations run as separate launches per phase (each phase at the occupancy
    // that suits it: that is the fast way while the solve is running); what is left of max_iter runs in ONE
    // persistent launch that iterates on the device and returns at once when the solve has already ended.
    // A solve that converges within the head therefore costs one idle launch instead of four per
    // iteration up to max_iter.
    // A fixed-count solve (tol < 0) runs every iteration it is given: nothing is idle, so it stays on the fast path.
    const int head = g_dense_one_launch == 2 ? 0
                     : (g_dense_one_launch == 0 || tol < 0.0f) ? max_iter
                     : (max_iter < kDenseHead ? max_iter : kDenseHead);
    // the initial guess (all a solve of zero iterations returns); the persistent launch makes its own when it starts the solve
    if (max_iter == 0) hipLaunchKernelGGL(dense_residual_kernel, dim3(res_blocks), dim3(256), 0, st, a, 1);
    for (int k = 1; k <= head; ++k) {
        a.k = k;
        // the initial guess and the residual of iteration 1 in one launch; the final sweep of an iteration
        // leaves the next one's
        if (k == 1) hipLaunchKernelGGL(dense_residual_kernel, dim3(res_blocks), dim3(256), 0, st, a, 4);
        launch_products_sweep(g_dense_products, n_sweep + n_prod_blocks, st, a, n_sweep);
        hipLaunchKernelGGL(dense_carry_kernel, dim3(B), dim3(256), 0, st, a);
        if (k < max_iter) hipLaunchKernelGGL((dense_final_sweep_kernel<false, true>), dim3(n_sweep), dim3(256), 0, st, a);
        else hipLaunchKernelGGL((dense_final_sweep_kernel<false, false>), dim3(n_sweep), dim3(256), 0, st, a);
    }
    if (head < max_iter) {
        a.spin_limit = settings().spin_limit;
        const int cap = newton_grid(g_dense_products);
        const size_t most = res_items > (size_t)(n_sweep + n_prod_blocks) ? res_items : (size_t)(n_sweep + n_prod_blocks);
        const int grid = (int)(most < (size_t)cap ? (most < 1 ? 1 : most) : (size_t)cap);
        launch_newton(g_dense_products, grid, st, a, n_sweep, n_prod_blocks, head + 1);
    }
    return hipGetLastError() == hipSuccess ? PARARNN_OK : PARARNN_HIP_ERROR;
}

}  // namespace pararnn
