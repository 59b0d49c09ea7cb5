// Input projection of the cells: u_g = B_g x + b_g for every gate g (the input
// terms of Eq. (7a) / (7b)), with multi-head, i.e. block-diagonal, B_g (App. C),
// and the derivatives of that map.  These are dense contractions and run on the
// matrix cores: operands rounded to bf16, fp32 accumulation
// (v_mfma_f32_32x32x16_bf16), the arithmetic of the paper's mixed-precision
// training set-up.  The bias add and the [B][L][G][H] layout of u are the GEMM's
// epilogue: u is written once, in the form the Newton kernels read.
//
//   forward   u[m][g][h]   = sum_j Wx[g][h][j] x[m][head(h) dh + j] + bias[g][h]
//   backward  dx[m][k dh+j] = sum_g sum_i du[m][g][k dh + i] Wx[g][k dh + i][j]
//             dWx[g][h][j] = sum_m du[m][g][h] x[m][head(h) dh + j]
//             dbias[g][h]  = sum_m du[m][g][h]
//
// forward and dx are "NT" products C[m][n] = sum_k A[m][k] B[n][k] with both
// operands contiguous in k (dx uses a transposed bf16 copy of the weights);
// dWx reduces over the rows m, which are the strided dimension of both of its
// operands, so its loader transposes on the way into LDS, and it is split over
// row ranges whose partial results are added in a fixed order afterwards.
//
// Tiles: 128 x 128 outputs per workgroup of four waves (64 x 64 per wave, four
// 32 x 32 accumulators), 64 k per step, both operand tiles in LDS as rows of 64
// bf16 with a pitch of 144 bytes (the 16-byte fragments of 16 consecutive rows
// then cover all 64 banks once), double buffered: the global loads of step s+1
// are in flight while step s is multiplied.
#include "../../include/pararnn.h"
#include "common.h"
#include "launch.h"
#include "proj.h"

#include <stdint.h>
#include <string.h>

namespace pararnn {

namespace {

typedef float f16v __attribute__((ext_vector_type(16)));
typedef float f4v __attribute__((ext_vector_type(4)));
typedef float f2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf8v __attribute__((ext_vector_type(8)));
typedef unsigned int u4v __attribute__((ext_vector_type(4)));

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int PITCH = BK + 8;            // bf16 elements per LDS row (144 bytes)

__device__ __forceinline__ unsigned int pack2(float x0, float x1)
{
    const bf2v p = {(__bf16)x0, (__bf16)x1};
    return __builtin_bit_cast(unsigned int, p);
}

// eight consecutive elements as packed bf16
__device__ __forceinline__ u4v load8(const unsigned short *p) { return *reinterpret_cast<const u4v *>(p); }
__device__ __forceinline__ u4v load8(const float *p)
{
    const f4v a = *reinterpret_cast<const f4v *>(p), b = *reinterpret_cast<const f4v *>(p + 4);
    const u4v r = {pack2(a[0], a[1]), pack2(a[2], a[3]), pack2(b[0], b[1]), pack2(b[2], b[3])};
    return r;
}

__device__ __forceinline__ void store1(float *p, float v) { *p = v; }
__device__ __forceinline__ void store1(unsigned short *p, float v) { *p = f32_to_bf16(v); }

__device__ __forceinline__ int acc_row(int v, int half) { return 8 * (v >> 2) + 4 * half + (v & 3); }

// one 64-k step of a 64 x 64 wave tile from the LDS operand tiles
__device__ __forceinline__ void mma_step(const unsigned short *sa, const unsigned short *sb, int wm, int wn, int l32,
                                         int half, f16v (&acc)[2][2])
{
#pragma unroll
    for (int kb = 0; kb < BK / 16; ++kb) {
        bf8v fa[2], fb[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            fa[i] = *reinterpret_cast<const bf8v *>(sa + (64 * wm + 32 * i + l32) * PITCH + 16 * kb + 8 * half);
            fb[i] = *reinterpret_cast<const bf8v *>(sb + (64 * wn + 32 * i + l32) * PITCH + 16 * kb + 8 * half);
        }
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[mi], fb[ni], acc[mi][ni], 0, 0, 0);
    }
}

// ------------------------------------------------------------------ NT product
struct GemmArgs {
    const void *A;                 // [M][lda], storage type AT
    const unsigned short *Bw;      // bf16 [N][ldb]
    void *C;                       // [M][ldc], storage type CT
    const float *bias;             // indexed like the columns of C (same batch offsets), or NULL
    long long lda, ldb, ldc;
    int M, N, K;                   // K a multiple of BK
    int kseg;                      // k of A lives at (k / kseg) * kseg_stride + k % kseg; kseg a multiple of BK
    long long kseg_stride;
    int nz0, n_batch;              // batch index z = z1 * nz0 + z0
    long long a_off[2], b_off[2], c_off[2];     // element offsets per unit of z0, z1
    int tiles_m, tiles_n, per_xcd;
};

// Workgroups are dealt to the eight XCDs round-robin by the dispatcher; renumbering
// them so that each XCD works through a contiguous range of tiles keeps the tiles
// that share a row block of A (all n tiles, gates and heads of it) on one L2.
template <typename AT, typename CT>
__global__ __launch_bounds__(256, 2) void proj_gemm_nt_kernel(const GemmArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned short s_a[2][BM * PITCH];
    __shared__ __attribute__((aligned(16))) unsigned short s_b[2][BN * PITCH];
    const long long id = (long long)(blockIdx.x & 7) * a.per_xcd + (blockIdx.x >> 3);
    const int inner_n = a.tiles_n * a.n_batch;
    if (id >= (long long)a.tiles_m * inner_n) return;
    const int mt = (int)(id / inner_n), inner = (int)(id % inner_n);
    const int nt = inner % a.tiles_n, z = inner / a.tiles_n;
    const int z0 = z % a.nz0, z1 = z / a.nz0;
    const AT *A = static_cast<const AT *>(a.A) + z0 * a.a_off[0] + z1 * a.a_off[1];
    const unsigned short *Bw = a.Bw + z0 * a.b_off[0] + z1 * a.b_off[1];
    const long long coff = z0 * a.c_off[0] + z1 * a.c_off[1];
    const int m0 = mt * BM, n0 = nt * BN;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, wm = w >> 1, wn = w & 1;
    const int half = lane >> 5, l32 = lane & 31;

    // a thread stages four 16-byte pieces of each operand tile per step: piece q = tid + 256 i
    // is k-chunk q % 8 of tile row q / 8
    u4v ra[4], rb[4];
    const u4v zero4 = {0u, 0u, 0u, 0u};
    auto load_stage = [&](int k0) {
        const long long kbase = (long long)(k0 / a.kseg) * a.kseg_stride + k0 % a.kseg;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int q = tid + 256 * i, row = q >> 3, c = q & 7;
            const int gm = m0 + row, gn = n0 + row;
            ra[i] = gm < a.M ? load8(A + (long long)gm * a.lda + kbase + 8 * c) : zero4;
            rb[i] = gn < a.N ? load8(Bw + (long long)gn * a.ldb + k0 + 8 * c) : zero4;
        }
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int q = tid + 256 * i, row = q >> 3, c = q & 7;
            *reinterpret_cast<u4v *>(&s_a[buf][row * PITCH + 8 * c]) = ra[i];
            *reinterpret_cast<u4v *>(&s_b[buf][row * PITCH + 8 * c]) = rb[i];
        }
    };
    f16v acc[2][2];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

    const int nk = a.K / BK;
    load_stage(0);
    store_stage(0);
    __syncthreads();
    for (int s = 0; s < nk; ++s) {
        if (s + 1 < nk) load_stage((s + 1) * BK);
        mma_step(s_a[s & 1], s_b[s & 1], wm, wn, l32, half, acc);
        if (s + 1 < nk) store_stage((s + 1) & 1);
        __syncthreads();
    }
    // epilogue: bias, storage type, the caller's layout; a lane owns one column
    CT *C = static_cast<CT *>(a.C) + coff;
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
        const int col = n0 + 64 * wn + 32 * ni + l32;
        if (col >= a.N) continue;
        const float bv = a.bias ? a.bias[coff + col] : 0.0f;
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + 64 * wm + 32 * mi + acc_row(v, half);
                if (row < a.M) store1(C + (long long)row * a.ldc + col, acc[mi][ni][v] + bv);
            }
    }
}

// --------------------------------------------------- dWx and dbias (TN product)
struct DwArgs {
    const void *du;        // [M][G][H], storage type AT
    const void *x;         // [M][H]
    float *part;           // [S][G][H][dh] partial sums of dWx
    float *dbpart;         // [S][G][H] partial sums of dbias, or NULL
    int M, H, G, heads, dh;
    int S, rows_per_split; // rows_per_split a multiple of BK
    int tiles;             // 128-wide tiles per dh
};

// two adjacent channels of eight consecutive rows -> one 16-byte k-run per channel
template <typename AT> struct PairLoad;
template <> struct PairLoad<unsigned short> {
    __device__ __forceinline__ static void run(const unsigned short *p, long long ld, int m, int m_end, bool ok,
                                               u4v &c0, u4v &c1, float &s0, float &s1)
    {
        unsigned int v[8];
#pragma unroll
        for (int r = 0; r < 8; ++r)
            v[r] = (ok && m + r < m_end) ? *reinterpret_cast<const unsigned int *>(p + (long long)(m + r) * ld) : 0u;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            c0[k] = (v[2 * k] & 0xffffu) | (v[2 * k + 1] << 16);
            c1[k] = (v[2 * k] >> 16) | (v[2 * k + 1] & 0xffff0000u);
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            s0 += __builtin_bit_cast(float, v[r] << 16);
            s1 += __builtin_bit_cast(float, v[r] & 0xffff0000u);
        }
    }
};
template <> struct PairLoad<float> {
    __device__ __forceinline__ static void run(const float *p, long long ld, int m, int m_end, bool ok, u4v &c0,
                                               u4v &c1, float &s0, float &s1)
    {
        f2v v[8];
        const f2v zero2 = {0.0f, 0.0f};
#pragma unroll
        for (int r = 0; r < 8; ++r)
            v[r] = (ok && m + r < m_end) ? *reinterpret_cast<const f2v *>(p + (long long)(m + r) * ld) : zero2;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            c0[k] = pack2(v[2 * k][0], v[2 * k + 1][0]);
            c1[k] = pack2(v[2 * k][1], v[2 * k + 1][1]);
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) { s0 += v[r][0]; s1 += v[r][1]; }
    }
};

// One workgroup: a 128 x 128 tile of dWx[g][head] for one row range.  Tile rows are
// the output channels i (operand du), tile columns the input channels j (operand x);
// k runs over the rows m of the range.
template <typename AT>
__global__ __launch_bounds__(256, 2) void proj_dw_kernel(const DwArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned short s_a[2][BM * PITCH];
    __shared__ __attribute__((aligned(16))) unsigned short s_b[2][BN * PITCH];
    __shared__ float s_db[4][BM];
    int id = blockIdx.x;
    const int tj = id % a.tiles; id /= a.tiles;
    const int ti = id % a.tiles; id /= a.tiles;
    const int head = id % a.heads; id /= a.heads;
    const int g = id % a.G;
    const int s = id / a.G;
    const int i0 = ti * BM, j0 = tj * BN;
    const int m_begin = s * a.rows_per_split;
    const int m_end = min(a.M, m_begin + a.rows_per_split);
    const long long ld_du = (long long)a.G * a.H, ld_x = a.H;
    const AT *du = static_cast<const AT *>(a.du) + (long long)g * a.H + head * a.dh + i0;
    const AT *x = static_cast<const AT *>(a.x) + head * a.dh + j0;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, wm = w >> 1, wn = w & 1;
    const int half = lane >> 5, l32 = lane & 31;
    // staging item (channel pair p, row group mg + 4 i): rows 8 (mg + 4 i) .. +7 of the 64-row step
    const int p = tid & 63, mg = tid >> 6;
    const bool ok_a = i0 + 2 * p < a.dh, ok_b = j0 + 2 * p < a.dh;     // dh is even: a pair is valid or not as a whole

    u4v ra[2][2], rb[2][2];
    float sdb0 = 0.0f, sdb1 = 0.0f, unused0 = 0.0f, unused1 = 0.0f;
    auto load_stage = [&](int m0) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int m = m0 + 8 * (mg + 4 * i);
            PairLoad<AT>::run(du + 2 * p, ld_du, m, m_end, ok_a, ra[i][0], ra[i][1], sdb0, sdb1);
            PairLoad<AT>::run(x + 2 * p, ld_x, m, m_end, ok_b, rb[i][0], rb[i][1], unused0, unused1);
        }
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int k = 8 * (mg + 4 * i);
            *reinterpret_cast<u4v *>(&s_a[buf][(2 * p) * PITCH + k]) = ra[i][0];
            *reinterpret_cast<u4v *>(&s_a[buf][(2 * p + 1) * PITCH + k]) = ra[i][1];
            *reinterpret_cast<u4v *>(&s_b[buf][(2 * p) * PITCH + k]) = rb[i][0];
            *reinterpret_cast<u4v *>(&s_b[buf][(2 * p + 1) * PITCH + k]) = rb[i][1];
        }
    };
    f16v acc[2][2];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

    const int nk = m_end > m_begin ? (m_end - m_begin + BK - 1) / BK : 0;
    if (nk > 0) {
        load_stage(m_begin);
        store_stage(0);
    }
    __syncthreads();
    for (int st = 0; st < nk; ++st) {
        if (st + 1 < nk) load_stage(m_begin + (st + 1) * BK);
        mma_step(s_a[st & 1], s_b[st & 1], wm, wn, l32, half, acc);
        if (st + 1 < nk) store_stage((st + 1) & 1);
        __syncthreads();
    }
    float *out = a.part + (((long long)s * a.G + g) * a.H + head * a.dh + i0) * a.dh + j0;
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
        const int col = 64 * wn + 32 * ni + l32;
        if (j0 + col >= a.dh) continue;
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = 64 * wm + 32 * mi + acc_row(v, half);
                if (i0 + row < a.dh) out[(long long)row * a.dh + col] = acc[mi][ni][v];
            }
    }
    // column sums of du seen by this workgroup (the tj = 0 tiles cover every channel once)
    if (a.dbpart && tj == 0) {
        s_db[mg][2 * p] = sdb0;
        s_db[mg][2 * p + 1] = sdb1;
        __syncthreads();
        if (tid < BM && i0 + tid < a.dh)
            a.dbpart[((long long)s * a.G + g) * a.H + head * a.dh + i0 + tid] =
                (s_db[0][tid] + s_db[1][tid]) + (s_db[2][tid] + s_db[3][tid]);
    }
}

// ------------------------------------------------------------- weight copies
// Wb = bf16(Wx), same layout [G][H][dh]
__global__ __launch_bounds__(256) void proj_wb_kernel(const float *Wx, unsigned short *Wb, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        Wb[i] = f32_to_bf16(Wx[i]);
}

// Wt[head][j][g dh + i] = bf16(Wx[g][head dh + i][j]): the B operand of the dx product
__global__ __launch_bounds__(256) void proj_wt_kernel(const float *Wx, unsigned short *Wt, int G, int H, int dh)
{
    const size_t n = (size_t)G * H * dh;
    for (size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x; o < n; o += (size_t)gridDim.x * blockDim.x) {
        const int i = (int)(o % dh);
        const int g = (int)((o / dh) % G);
        const int j = (int)((o / ((size_t)dh * G)) % dh);
        const int head = (int)(o / ((size_t)dh * G * dh));
        Wt[o] = f32_to_bf16(Wx[((size_t)g * H + (size_t)head * dh + i) * dh + j]);
    }
}

size_t r256(size_t x) { return (x + 255) & ~(size_t)255; }

bool shapes_ok(int dtype, int B, int L, int H, int G, int n_heads)
{
    if (dtype != PARARNN_F32 && dtype != PARARNN_BF16) return false;
    if (B < 1 || L < 1 || H < 1 || G < 1 || G > 8 || n_heads < 1 || H % n_heads) return false;
    const double rows = (double)B * (double)L;
    return rows < 2.0e9 && rows * G * H < 3.0e10;
}

// row ranges of the dWx reduction: enough workgroups to fill the device, whole 64-row steps
void dw_split(int M, int base_tiles, int *S, int *rows_per_split)
{
    int want = (2048 + base_tiles - 1) / base_tiles;
    if (want < 1) want = 1;
    if (want > 64) want = 64;
    int rps = (M + want - 1) / want;
    rps = (rps + BK - 1) / BK * BK;
    if (rps < 4 * BK) rps = 4 * BK;
    *rows_per_split = rps;
    *S = (M + rps - 1) / rps;
}

struct ProjLayout {
    size_t off_w, off_part, off_db, total;
    int S, rows_per_split, tiles;
};

ProjLayout proj_layout(int B, int L, int H, int G, int n_heads, int backward)
{
    ProjLayout lo;
    const int dh = H / n_heads;
    const size_t nw = (size_t)G * H * dh;
    size_t off = 0;
    lo.off_w = off; off += r256(nw * sizeof(unsigned short));
    lo.tiles = (dh + BM - 1) / BM;
    lo.S = 0; lo.rows_per_split = 0;
    lo.off_part = lo.off_db = off;
    if (backward) {
        dw_split(B * L, lo.tiles * lo.tiles * G * n_heads, &lo.S, &lo.rows_per_split);
        lo.off_part = off; off += r256((size_t)lo.S * nw * sizeof(float));
        lo.off_db = off;   off += r256((size_t)lo.S * G * H * sizeof(float));
    }
    lo.total = off < 256 ? 256 : off;
    return lo;
}

template <typename AT, typename CT> hipError_t launch_nt(GemmArgs &g, hipStream_t st)
{
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + BN - 1) / BN;
    const long long total = (long long)g.tiles_m * g.tiles_n * g.n_batch;
    g.per_xcd = (int)((total + 7) / 8);
    hipLaunchKernelGGL((proj_gemm_nt_kernel<AT, CT>), dim3((unsigned)(8 * g.per_xcd)), dim3(256), 0, st, g);
    return hipGetLastError();
}

int elementwise_blocks(size_t n)
{
    size_t blocks = (n + 255) / 256;
    const size_t cap = (size_t)device_cu_count() * 16;
    return (int)(blocks < cap ? blocks : cap);
}

}  // namespace

size_t proj_workspace_bytes(int dtype, int B, int L, int H, int G, int n_heads, int backward)
{
    if (!shapes_ok(dtype, B, L, H, G, n_heads) || (H / n_heads) % BK) return 0;
    return proj_layout(B, L, H, G, n_heads, backward).total;
}

int proj_forward(int dtype, const void *x, const float *Wx, const float *bias, int B, int L, int H, int G,
                 int n_heads, void *u, void *workspace, size_t workspace_bytes, hipStream_t st)
{
    if (!shapes_ok(dtype, B, L, H, G, n_heads)) return PARARNN_INVALID_ARG;
    const int dh = H / n_heads;
    if (dh % BK) return PARARNN_UNSUPPORTED;
    if (((uintptr_t)x | (uintptr_t)Wx | (uintptr_t)u | (uintptr_t)workspace) % 16) return PARARNN_UNSUPPORTED;
    const ProjLayout lo = proj_layout(B, L, H, G, n_heads, 0);
    if (workspace_bytes < lo.total) return PARARNN_WORKSPACE_TOO_SMALL;
    unsigned short *Wb = reinterpret_cast<unsigned short *>(static_cast<char *>(workspace) + lo.off_w);
    const size_t nw = (size_t)G * H * dh;
    hipLaunchKernelGGL(proj_wb_kernel, dim3(elementwise_blocks(nw)), dim3(256), 0, st, Wx, Wb, nw);
    GemmArgs g;
    memset(&g, 0, sizeof(g));
    g.A = x; g.Bw = Wb; g.C = u; g.bias = bias;
    g.lda = H; g.ldb = dh; g.ldc = (long long)G * H;
    g.M = B * L; g.N = dh; g.K = dh;
    g.kseg = dh; g.kseg_stride = 0;
    g.nz0 = n_heads; g.n_batch = n_heads * G;          // z0 = head, z1 = gate
    g.a_off[0] = dh; g.a_off[1] = 0;
    g.b_off[0] = (long long)dh * dh; g.b_off[1] = (long long)H * dh;
    g.c_off[0] = dh; g.c_off[1] = H;
    const hipError_t e = dtype == PARARNN_BF16 ? launch_nt<unsigned short, unsigned short>(g, st) : launch_nt<float, float>(g, st);
    return e == hipSuccess ? PARARNN_OK : PARARNN_HIP_ERROR;
}

int proj_backward(int dtype, const void *x, const float *Wx, const void *du, int B, int L, int H, int G, int n_heads,
                  void *dx, float *dWx, float *dbias, void *workspace, size_t workspace_bytes, hipStream_t st)
{
    if (!shapes_ok(dtype, B, L, H, G, n_heads)) return PARARNN_INVALID_ARG;
    const int dh = H / n_heads;
    if (dh % BK) return PARARNN_UNSUPPORTED;
    if (((uintptr_t)x | (uintptr_t)Wx | (uintptr_t)du | (uintptr_t)dx | (uintptr_t)workspace) % 16) return PARARNN_UNSUPPORTED;
    const ProjLayout lo = proj_layout(B, L, H, G, n_heads, 1);
    if (workspace_bytes < lo.total) return PARARNN_WORKSPACE_TOO_SMALL;
    char *ws = static_cast<char *>(workspace);
    const size_t nw = (size_t)G * H * dh;
    const bool bf = dtype == PARARNN_BF16;
    hipError_t e = hipSuccess;
    if (dx) {
        unsigned short *Wt = reinterpret_cast<unsigned short *>(ws + lo.off_w);
        hipLaunchKernelGGL(proj_wt_kernel, dim3(elementwise_blocks(nw)), dim3(256), 0, st, Wx, Wt, G, H, dh);
        GemmArgs g;
        memset(&g, 0, sizeof(g));
        g.A = du; g.Bw = Wt; g.C = dx; g.bias = nullptr;
        g.lda = (long long)G * H; g.ldb = (long long)G * dh; g.ldc = H;
        g.M = B * L; g.N = dh; g.K = G * dh;
        g.kseg = dh; g.kseg_stride = H;                 // k = (gate, i): gates are H apart in a row of du
        g.nz0 = n_heads; g.n_batch = n_heads;           // z0 = head
        g.a_off[0] = dh; g.b_off[0] = (long long)dh * G * dh; g.c_off[0] = dh;
        e = bf ? launch_nt<unsigned short, unsigned short>(g, st) : launch_nt<float, float>(g, st);
        if (e != hipSuccess) return PARARNN_HIP_ERROR;
    }
    if (dWx) {
        DwArgs a;
        memset(&a, 0, sizeof(a));
        a.du = du; a.x = x;
        a.part = reinterpret_cast<float *>(ws + lo.off_part);
        a.dbpart = dbias ? reinterpret_cast<float *>(ws + lo.off_db) : nullptr;
        a.M = B * L; a.H = H; a.G = G; a.heads = n_heads; a.dh = dh;
        a.S = lo.S; a.rows_per_split = lo.rows_per_split; a.tiles = lo.tiles;
        const int blocks = lo.tiles * lo.tiles * n_heads * G * lo.S;
        if (bf) hipLaunchKernelGGL(proj_dw_kernel<unsigned short>, dim3(blocks), dim3(256), 0, st, a);
        else hipLaunchKernelGGL(proj_dw_kernel<float>, dim3(blocks), dim3(256), 0, st, a);
        if (hipGetLastError() != hipSuccess) return PARARNN_HIP_ERROR;
        if (launch_param_reduce(a.part, dWx, lo.S, (int)nw, st) != hipSuccess) return PARARNN_HIP_ERROR;
        if (dbias && launch_param_reduce(a.dbpart, dbias, lo.S, G * H, st) != hipSuccess) return PARARNN_HIP_ERROR;
    }
    return PARARNN_OK;
}

}  // namespace pararnn
