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
// 32 x 32 accumulators), 64 k per step, both operand tiles in LDS in k-chunk-major
// order (fragment reads are contiguous), double buffered, the global loads of the
// next two steps in flight while a step is multiplied.
#include "pararnn.h"
#include "pararnn/common.h"
#include "pararnn/launch.h"
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
// An operand tile in LDS: eight planes, one per 16-byte k-chunk, each holding that chunk of the
// 128 rows back to back, planes 16 bytes further apart than their size.
constexpr int PLANE = 128 * 8 + 8;       // bf16 elements from one plane to the next
constexpr int TILE = 8 * PLANE;          // bf16 elements of a tile

__device__ __forceinline__ unsigned int pack2(float x0, float x1)
{
    const bf2v p = {(__bf16)x0, (__bf16)x1};
    return __builtin_bit_cast(unsigned int, p);
}

// eight consecutive elements as fetched, and as packed bf16
struct Raw8f {
    f4v lo, hi;
};
__device__ __forceinline__ u4v load8(const unsigned short *p) { return *reinterpret_cast<const u4v *>(p); }
__device__ __forceinline__ Raw8f load8(const float *p)
{
    Raw8f r;
    r.lo = *reinterpret_cast<const f4v *>(p);
    r.hi = *reinterpret_cast<const f4v *>(p + 4);
    return r;
}
__device__ __forceinline__ u4v to_bf16x8(const u4v &v) { return v; }
__device__ __forceinline__ u4v to_bf16x8(const Raw8f &v)
{
    const u4v r = {pack2(v.lo[0], v.lo[1]), pack2(v.lo[2], v.lo[3]), pack2(v.hi[0], v.hi[1]), pack2(v.hi[2], v.hi[3])};
    return r;
}
template <typename AT> struct Raw8 { typedef u4v type; };
template <> struct Raw8<float> { typedef Raw8f type; };

// four consecutive outputs in the storage type
__device__ __forceinline__ void store4(float *p, const f4v &v) { *reinterpret_cast<f4v *>(p) = v; }
__device__ __forceinline__ void store4(unsigned short *p, const f4v &v)
{
    *reinterpret_cast<uint2 *>(p) = make_uint2(pack2(v[0], v[1]), pack2(v[2], v[3]));
}

__device__ __forceinline__ int acc_row(int v, int half) { return 8 * (v >> 2) + 4 * half + (v & 3); }

// Element offset of 16-byte chunk `chunk` (0..7) of row `row` in an LDS operand tile.  A
// fragment read (32 consecutive rows, one chunk per lane half) is 512 contiguous bytes; the
// eight chunks of a row, stored by eight neighbouring lanes, fall into eight different
// 16-byte bank groups because of the 16 bytes between planes.
__device__ __forceinline__ int lds_off(int row, int chunk) { return chunk * PLANE + row * 8; }

// one 64-k step of a 64 x 64 wave tile from the LDS operand tiles.  PREFETCH: the fragments
// of the next 16 k are requested before the products of the current 16 k are issued (the
// scheduling barriers keep that order), so that LDS latency is paid once per step, not four
// times; it costs 16 registers, which only the bf16 NT kernel has to spare.
template <bool PREFETCH>
__device__ __forceinline__ void mma_step(const unsigned short *sa, const unsigned short *sb, int wm, int wn, int l32,
                                         int half, f16v (&acc)[2][2])
{
    auto read = [&](int kb, bf8v(&a)[2], bf8v(&b)[2]) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            a[i] = *reinterpret_cast<const bf8v *>(sa + lds_off(64 * wm + 32 * i + l32, 2 * kb + half));
            b[i] = *reinterpret_cast<const bf8v *>(sb + lds_off(64 * wn + 32 * i + l32, 2 * kb + half));
        }
    };
    if constexpr (PREFETCH) {
        bf8v fa[2][2], fb[2][2];
        read(0, fa[0], fb[0]);
#pragma unroll
        for (int kb = 0; kb < BK / 16; ++kb) {
            if (kb + 1 < BK / 16) read(kb + 1, fa[(kb + 1) & 1], fb[(kb + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kb & 1][mi], fb[kb & 1][ni], acc[mi][ni], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {
#pragma unroll
        for (int kb = 0; kb < BK / 16; ++kb) {
            bf8v fa[2], fb[2];
            read(kb, fa, fb);
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[mi], fb[ni], acc[mi][ni], 0, 0, 0);
        }
    }
}

// The step loop of both products.  Step t is multiplied from LDS buffer t % 2 while the
// global loads of steps t+1 and t+2 are outstanding in two register sets (memory latency
// is several times the duration of a step).  load(set) fetches the next step in stream
// order, store(buf, set) puts a fetched step into an LDS buffer (buf = -1: into none) and
// may publish through LDS what load() needs at its next call, compute(buf) multiplies.
// Loads and stores are issued unconditionally, also past the end of the stream (load()
// then has to deliver something harmless, which is stored and never multiplied): with
// no branch around them the compiler can wait for exactly the older register set while
// the younger loads stay in flight.  For the same reason load() must not touch what it
// fetched: conversion, zeroing of rows past the end and transposition happen in store().
// done() is asked after every step and must give every thread the same answer: the
// barriers are uniform.
template <class Stage, class Load, class Store, class Compute, class Done>
__device__ __forceinline__ void two_ahead(Load load, Store store, Compute compute, Done done)
{
    Stage r0, r1;
    load(r0);
    store(0, r0);
    __syncthreads();
    load(r1);
    store(-1, r1);            // nothing goes to a buffer: only what load() wants published through LDS
    __syncthreads();
    for (;;) {
        // a step from buffer 0; set 0 is free, set 1 holds the next step
        load(r0);
        compute(0);
        store(1, r1);
        __syncthreads();
        if (done()) break;
        // a step from buffer 1; set 1 is free, set 0 holds the next step
        load(r1);
        compute(1);
        store(0, r0);
        __syncthreads();
        if (done()) break;
    }
}

// The same with one register set: the loads of step t+1 are outstanding while step t is
// multiplied.  For stages too large to hold twice (fp32 rows before their transposition).
template <class Stage, class Load, class Store, class Compute, class Done>
__device__ __forceinline__ void one_ahead(Load load, Store store, Compute compute, Done done)
{
    Stage r;
    load(r);
    store(0, r);
    __syncthreads();
    for (int t = 0;; ++t) {
        load(r);
        compute(t & 1);
        store((t + 1) & 1, r);
        __syncthreads();
        if (done()) break;
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
    int tiles_m, tiles_n;
    int *tickets;                  // eight counters, zero at launch: the next tile number of each XCD
    int draw;                      // tile numbers taken per draw (copy-to-LDS kernel)
};

// Persistent workgroups, each walking a list of output tiles; the (tile, k-step) pairs
// of that list form one flat stream of steps, so that the loads of a tile's first steps
// are in flight while the previous tile is still being multiplied.  Step t is multiplied
// from LDS buffer t % 2 while the global loads of steps t+1 and t+2 are outstanding in two
// register sets (memory latency is several times the duration of a step).
//
// Workgroups are dealt to the eight XCDs round-robin by the dispatcher; tile numbers are
// assigned so that each XCD works through a contiguous range, neighbours in time being
// the tiles that share a row block of A (all n tiles, gates and heads of it): they meet
// in one L2.
template <typename AT, typename CT, bool BIAS>
__global__ __launch_bounds__(256, 2) void proj_gemm_nt_kernel(const GemmArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned short s_a[2][TILE];
    __shared__ __attribute__((aligned(16))) unsigned short s_b[2][TILE];
    __shared__ int s_ring[8];
    const int xcd = blockIdx.x & 7;
    const int inner_n = a.tiles_n * a.n_batch;
    // This XCD owns the row blocks [xcd * mx, (xcd + 1) * mx).  Its (row block, inner) grid is
    // cut into patches of 8 x 8 tiles (smaller at the edges), numbered one after the other, and
    // its workgroups draw numbers from a counter: whatever their relative speed they are inside
    // one or two neighbouring patches at any time, whose 8 + 8 operand panels stay in that
    // XCD's L2.
    const int mx = (a.tiles_m + 7) / 8;
    int my_rows = a.tiles_m - xcd * mx;            // row blocks of this XCD
    if (my_rows > mx) my_rows = mx;
    if (my_rows <= 0) return;
    const int n_local = my_rows * inner_n;
    auto decode = [&](int local, int &mt, int &inner) {
        const int pm = local / (8 * inner_n), rem = local - pm * 8 * inner_n;
        const int hm = min(8, my_rows - 8 * pm);                 // rows of this patch row
        const int pn = rem / (8 * hm), rem2 = rem - pn * 8 * hm;
        const int hn = min(8, inner_n - 8 * pn);                 // columns of this patch
        mt = xcd * mx + 8 * pm + rem2 / hn;
        inner = 8 * pn + rem2 % hn;
    };
    const int nk = a.K / BK;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, wm = w >> 1, wn = w & 1;
    const int half = lane >> 5, l32 = lane & 31;
    // Thread 0 draws the number of this workgroup's n-th tile and leaves it in s_ring[n % 8]
    // (n_local or more: the XCD's list is used up); everybody reads it after a later barrier.
    // At most three tiles are drawn ahead of the one being multiplied.
    if (tid == 0) s_ring[0] = atomicAdd(a.tickets + xcd, 1);
    __syncthreads();
    if (s_ring[0] >= n_local) return;

    struct Tile {
        const AT *A;
        const unsigned short *Bw;
        long long coff;
        int m0, n0;
    };
    auto tile_of = [&](int local) {
        int mt, inner;
        decode(local, mt, inner);
        const int nt = inner % a.tiles_n, z = inner / a.tiles_n;
        const int z0 = z % a.nz0, z1 = z / a.nz0;
        Tile t;
        t.A = static_cast<const AT *>(a.A) + z0 * a.a_off[0] + z1 * a.a_off[1];
        t.Bw = a.Bw + z0 * a.b_off[0] + z1 * a.b_off[1];
        t.coff = z0 * a.c_off[0] + z1 * a.c_off[1];
        t.m0 = mt * BM; t.n0 = nt * BN;
        return t;
    };
    // a thread stages four 16-byte pieces of each operand tile per step: piece q = tid + 256 i
    // is k-chunk q % 8 of the tile row below: eight lanes cover one row (eight bank groups), and
    // the two rows of sixteen consecutive lanes are eight apart (the other eight)
    auto piece_row = [](int q) { return ((q >> 4) & 7) + 8 * ((q >> 3) & 1) + 16 * (q >> 7); };
    const u4v zero4 = {0u, 0u, 0u, 0u};
    // the loading side: tile number ln of this workgroup, k-step lks of it; l_switch: the tile
    // is finished and the next load starts the tile drawn meanwhile; l_end: there was none
    Tile lt = tile_of(s_ring[0]);
    int ln = 0, lks = 0;
    bool l_switch = false, l_end = false;
    // the number drawn for tile ln + 1: requested when the last step of tile ln is fetched,
    // put into the ring by the store() that follows (the request's latency passes meanwhile)
    int drawn = 0;
    bool drawn_pending = false;
    struct Stage {
        typename Raw8<AT>::type a[4];
        u4v b[4];
        unsigned int valid;            // bit i: row of a[i] exists, bit 4 + i: row of b[i] exists
    };
    // per tile: where this thread's four pieces of each operand start (k = 0), and which of their
    // rows exist; rows past the end read the last row (valid memory) and are stored as zeros
    const AT *pa[4];
    const unsigned short *pb[4];
    unsigned int l_valid = 0u;
    auto point_at = [&](const Tile &t) {
        l_valid = 0u;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int q = tid + 256 * i, row = piece_row(q), c = q & 7;
            const int gm = t.m0 + row, gn = t.n0 + row;
            pa[i] = t.A + (long long)min(gm, a.M - 1) * a.lda + 8 * c;
            pb[i] = t.Bw + (long long)min(gn, a.N - 1) * a.ldb + 8 * c;
            l_valid |= (gm < a.M ? 1u : 0u) << i | (gn < a.N ? 16u : 0u) << i;
        }
    };
    point_at(lt);
    auto load_next = [&](Stage &r) {
        if (l_switch) {
            const int t = s_ring[(ln + 1) & 7];
            if (t >= n_local) {
                l_end = true;              // from here on the last step is fetched again (never multiplied)
            } else {
                lt = tile_of(t);
                point_at(lt);
                ++ln;
                lks = 0;
            }
            l_switch = false;
        }
        const bool last_step = !l_end && lks + 1 == nk;
        if (last_step && tid == 0) drawn = atomicAdd(a.tickets + xcd, 1);
        const int k0 = lks * BK;
        const long long kbase = (long long)(k0 / a.kseg) * a.kseg_stride + k0 % a.kseg;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            r.a[i] = load8(pa[i] + kbase);
            r.b[i] = load8(pb[i] + k0);
        }
        r.valid = l_valid;
        if (last_step) {
            drawn_pending = true;
            l_switch = true;
        } else if (!l_end) {
            ++lks;
        }
    };
    auto store_stage = [&](int buf, const Stage &r) {
        if (drawn_pending) {
            if (tid == 0) s_ring[(ln + 1) & 7] = drawn;
            drawn_pending = false;
        }
        if (buf < 0) return;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int q = tid + 256 * i, row = piece_row(q), c = q & 7;
            *reinterpret_cast<u4v *>(&s_a[buf][lds_off(row, c)]) = (r.valid >> i & 1u) ? to_bf16x8(r.a[i]) : zero4;
            *reinterpret_cast<u4v *>(&s_b[buf][lds_off(row, c)]) = (r.valid >> (4 + i) & 1u) ? r.b[i] : zero4;
        }
    };
    f16v acc[2][2];
    auto clear_acc = [&]() {
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;
    };
    // The product is formed transposed, acc[ni][mi] = (W tile)(A tile)^T: a lane then owns one
    // ROW of C and, per group of four accumulator registers, four consecutive columns, so the
    // epilogue (bias, storage type, the caller's layout) stores 8 or 16 bytes per lane.
    Tile ct = lt;                      // tile being multiplied: number cn of this workgroup
    int cn = 0, cks = 0;
    bool c_end = false;
    auto finish_step = [&](int buf) {
        if (++cks < nk) return;
        // Epilogue.  The accumulators go through LDS so that a wave's global stores are whole
        // row segments (16 bytes per lane, neighbouring lanes neighbouring addresses): each
        // wave transposes its 64 x 64 part in two passes of 32 rows, in its own quarter of the
        // operand buffer that has just been multiplied (free once every wave is past this
        // step).  16-byte chunk c of row r sits at chunk position c ^ (r % chunks per row).
        __syncthreads();
        constexpr int EPC = 16 / (int)sizeof(CT);          // elements per 16-byte chunk
        constexpr int CPR = 64 / EPC;                      // chunks per 64-column row
        CT *stage = reinterpret_cast<CT *>(w < 2 ? s_a[buf] : s_b[buf]) + (w & 1) * (32 * 64);
        CT *C = static_cast<CT *>(a.C) + ct.coff;
        const int col0 = ct.n0 + 64 * wn;                  // N is a multiple of 64: all 64 columns exist or none
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = 32 * ni + 8 * q + 4 * half;      // this lane's four columns, row l32
                    f4v o = {acc[ni][mi][4 * q], acc[ni][mi][4 * q + 1], acc[ni][mi][4 * q + 2], acc[ni][mi][4 * q + 3]};
                    if (BIAS) o += *reinterpret_cast<const f4v *>(a.bias + ct.coff + min(col0, a.N - 64) + col);
                    store4(stage + l32 * 64 + ((col / EPC) ^ (l32 & (CPR - 1))) * EPC + col % EPC, o);
                }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            constexpr int RPI = 64 / CPR;                  // rows per store instruction
#pragma unroll
            for (int it = 0; it < 32 / RPI; ++it) {
                const int r = it * RPI + lane / CPR, cc = lane % CPR;
                const u4v v = *reinterpret_cast<const u4v *>(stage + r * 64 + (cc ^ (r & (CPR - 1))) * EPC);
                const int row = ct.m0 + 64 * wm + 32 * mi + r;
                if (row < a.M && col0 < a.N) *reinterpret_cast<u4v *>(C + (long long)row * a.ldc + col0 + cc * EPC) = v;
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        clear_acc();
        cks = 0;
        const int t = s_ring[++cn & 7];     // drawn at least one barrier ago
        if (t >= n_local) c_end = true;
        else ct = tile_of(t);
    };
    clear_acc();

    two_ahead<Stage>(load_next, store_stage,
                     [&](int buf) {
                         mma_step<sizeof(AT) == 2>(s_b[buf], s_a[buf], wn, wm, l32, half, acc);
                         finish_step(buf);
                     },
                     [&]() { return c_end; });
}

// ------------------------------- NT product, bf16 operands copied straight into LDS
// The same product for bf16 storage and K >= 128, built around buffer loads whose destination
// is LDS: operand tiles never pass through registers, and a step costs a wave eight copy
// instructions instead of loads, conversions and LDS stores.
//
//   tile     256 x 256 outputs per workgroup of eight waves (2 x 4; 128 rows x 64 columns per
//            wave = eight 32 x 32 accumulators), 64 k per step; one workgroup per CU
//   LDS      two stages of (256 + 256) rows x 128 bytes = 128 KB.  A copy instruction moves
//            64 x 16 bytes to consecutive LDS addresses, lane i to base + 16 i: 8 rows of a
//            stage, and 8 whole 128-byte lines of memory (with 32 k per step an instruction
//            took half of 16 lines, and the other half of every line was fetched again a step
//            later: the copies alone then took as long as the whole kernel does now).  Which
//            16-byte k-chunk of its row a lane fetches is free, and chosen so that chunk c of
//            row r lies at position c ^ swz(r) of the row: the eight lanes of a row still read
//            one line, and the fragment reads of the multiply (32 rows, one chunk each) spread
//            over all banks, whether 8 or 16 lanes are served per cycle.
//   step T   four rounds of (fragments of the next 16 k, eight products of the current 16 k);
//            before the last round: own copies of step T + 1 landed, own reads of step T done,
//            barrier; then the first fragments of step T + 1 are read and the copies of step
//            T + 2 start into the stage step T has just left.  One barrier per step, LDS
//            latency behind eight products, memory latency behind one step.
//   waits    the copies are issued from inline assembly, so the compiler neither knows nor
//            waits for them; at the one wait of a step the copies of step T + 1 are the only
//            loads the wave has outstanding, so the kernel waits for "no memory operation
//            outstanding", or for "at most sixteen" when the sixteen stores of an output tile
//            were issued after those copies: vector-memory operations of a wave complete in
//            issue order on this architecture (its single counter is used that way by every
//            compiled kernel), and waiting for the stores to drain cost a tenth of the time.
//   tiles    drawn from the per-XCD counters like above, a few consecutive numbers per draw
//            (the compiler waits for the atomic's result with every copy in flight, which
//            stalls the drawing wave; per draw, not per tile), and put into the ring one tile
//            ahead.
namespace dma {
constexpr int BM = 256, BN = 256, BK = 64;
constexpr int OP = 256 * BK;             // bf16 elements of one operand tile of a stage
constexpr int STAGE = 2 * OP;            // A tile, then W tile
}  // namespace dma

__device__ __forceinline__ int dma_swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }

__device__ __forceinline__ unsigned int uniform(unsigned int v) { return __builtin_amdgcn_readfirstlane(v); }

// buffer descriptor words for the assembly forms: base, no stride, whole 4 GiB window
__device__ __forceinline__ u4v rsrc_words(const void *p)
{
    const unsigned long long v = (unsigned long long)p;
    const u4v r = {uniform((unsigned int)v), uniform((unsigned int)(v >> 32) & 0xffffu), 0xffffffffu, 0x27000u};
    return r;
}

__device__ __forceinline__ unsigned int lds_address(const void *p)
{
    return (unsigned int)(unsigned long long)(__attribute__((address_space(3))) const void *)p;
}

// 64 x 16 bytes (64 x 4 bytes) from rsrc + voff + soff to LDS lds_base + 16 (4) * lane.  The five wait
// states in front of the load are the ones a vector-memory instruction needs after a vector instruction
// (v_readfirstlane, v_readlane of a spilled value) has written one of its scalar operands; the compiler
// inserts them for its own instructions and not for what is inside an asm statement.  They also cover
// the wait state between the write of M0 and its use.
__device__ __forceinline__ void copy_to_lds_16(unsigned int lds_base, const u4v &rsrc, unsigned int voff, unsigned int soff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 4\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :: "s"(uniform(lds_base)), "v"(voff), "s"(rsrc), "s"(uniform(soff)) : "memory", "m0");
}
__device__ __forceinline__ void copy_to_lds_4(unsigned int lds_base, const u4v &rsrc, unsigned int voff, unsigned int soff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 4\n\tbuffer_load_dword %1, %2, %3 offen lds"
                 :: "s"(uniform(lds_base)), "v"(voff), "s"(rsrc), "s"(uniform(soff)) : "memory", "m0");
}

template <bool BIAS>
__global__ __launch_bounds__(512) void proj_gemm_nt_dma_kernel(const GemmArgs a)
{
    constexpr int BM = dma::BM, BN = dma::BN, BK = dma::BK, OP = dma::OP, STAGE = dma::STAGE;
    __shared__ __attribute__((aligned(16))) unsigned short s_op[2][STAGE];
    __shared__ __attribute__((aligned(16))) unsigned short s_epi[8][32 * 32];
    __shared__ __attribute__((aligned(16))) float s_bias[4][8][64];
    __shared__ int s_ring[8];
    const int xcd = blockIdx.x & 7;
    const int inner_n = a.tiles_n * a.n_batch;
    // the XCD's (row block, inner) grid in patches of 8 x 8 tiles, as in proj_gemm_nt_kernel
    const int mx = (a.tiles_m + 7) / 8;
    int my_rows = a.tiles_m - xcd * mx;
    if (my_rows > mx) my_rows = mx;
    if (my_rows <= 0) return;
    const int n_local = my_rows * inner_n;
    const int nk = a.K / BK;
    const int tid = threadIdx.x, lane = tid & 63, w = (int)uniform((unsigned int)tid >> 6), wm = w >> 2, wn = w & 3;
    const int half = lane >> 5, l32 = lane & 31;
    if (tid == 0) s_ring[0] = atomicAdd(a.tickets + xcd, a.draw);
    __syncthreads();
    const int first = (int)uniform((unsigned int)s_ring[0]);
    if (first >= n_local) return;

    struct Tile {
        const unsigned short *A, *Bw;
        long long coff;
        int m0, n0;
    };
    auto tile_of = [&](int local) {
        const int pm = local / (8 * inner_n), rem = local - pm * 8 * inner_n;
        const int hm = min(8, my_rows - 8 * pm);
        const int pn = rem / (8 * hm), rem2 = rem - pn * 8 * hm;
        const int hn = min(8, inner_n - 8 * pn);
        const int mt = xcd * mx + 8 * pm + rem2 / hn, inner = 8 * pn + rem2 % hn;
        const int nt = inner % a.tiles_n, z = inner / a.tiles_n;
        const int z0 = z % a.nz0, z1 = z / a.nz0;
        Tile t;
        t.A = static_cast<const unsigned short *>(a.A) + z0 * a.a_off[0] + z1 * a.a_off[1];
        t.Bw = a.Bw + z0 * a.b_off[0] + z1 * a.b_off[1];
        t.coff = z0 * a.c_off[0] + z1 * a.c_off[1];
        t.m0 = mt * BM; t.n0 = nt * BN;
        return t;
    };

    // ---- the copying side: tile number ln of this workgroup, k-step lks of it.  A wave copies rows
    //      32 w .. 32 w + 31 of both operand tiles, eight rows (eight lanes each) per instruction.
    const unsigned int lds_op = lds_address(&s_op[0][0]);
    const int lrow = lane >> 3;
    u4v ra, rb, rbias;
    unsigned int va[4], vb[4], vbias = 0u;
    int ln = 0, lks = 0;
    long long seg_base = 0;                // element offset of the current k-segment in a row of A
    int kin = 0;                           // k within the segment
    bool l_end = false;
    auto point_at = [&](const Tile &t) {
        ra = rsrc_words(t.A + (long long)t.m0 * a.lda);
        rb = rsrc_words(t.Bw + (long long)t.n0 * a.ldb);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            // rows past the end read the last row (valid memory); their products are never stored
            const int row = 32 * w + 8 * j + lrow;
            const unsigned int chunk = (unsigned int)((lane & 7) ^ dma_swz(8 * j + lrow));
            const int gm = min(t.m0 + row, a.M - 1) - t.m0, gn = min(t.n0 + row, a.N - 1) - t.n0;
            va[j] = (unsigned int)gm * (unsigned int)a.lda * 2u + chunk * 16u;
            vb[j] = (unsigned int)gn * (unsigned int)a.ldb * 2u + chunk * 16u;
        }
        if (BIAS) {
            rbias = rsrc_words(a.bias + t.coff);
            vbias = (unsigned int)min(t.n0 + 64 * wn + lane, a.N - 1) * 4u;
        }
        seg_base = 0; kin = 0;
    };
    // thread 0: the numbers drawn and not yet handed out
    int next_no = first + 1, left = a.draw - 1;
    auto draw = [&]() {
        // the number of tile ln + 1 goes into the ring; it is read after at least one barrier
        if (tid == 0) {
            if (left == 0) {
                next_no = atomicAdd(a.tickets + xcd, a.draw);
                left = a.draw;
            }
            s_ring[(ln + 1) & 7] = next_no++;
            --left;
        }
    };
    // the copies of the next step in stream order, into stage `buf`
    auto issue = [&](int buf) {
        if (lks == nk) {
            const int t = (int)uniform((unsigned int)s_ring[(ln + 1) & 7]);      // written at least a barrier ago
            if (t >= n_local) {
                l_end = true;
                return;
            }
            point_at(tile_of(t));
            ++ln;
            lks = 0;
        }
        if (lks == 0) {
            draw();
            if (BIAS) copy_to_lds_4(lds_address(&s_bias[ln & 3][w][0]), rbias, vbias, 0u);
        }
        const unsigned int soa = (unsigned int)((seg_base + kin) * 2), sob = (unsigned int)(lks * BK) * 2u;
        const unsigned int dst = lds_op + (unsigned int)buf * (STAGE * 2u) + (unsigned int)(32 * w) * (BK * 2u);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            copy_to_lds_16(dst + (unsigned int)j * (8u * BK * 2u), ra, va[j], soa);
            copy_to_lds_16(dst + OP * 2u + (unsigned int)j * (8u * BK * 2u), rb, vb[j], sob);
        }
        ++lks;
        kin += BK;
        if (kin == a.kseg) {
            kin = 0;
            seg_base += a.kseg_stride;
        }
    };

    // ---- the multiplying side
    // byte offset of this lane's fragment piece within a 32-row block, for the four 16-k rounds of a step
    unsigned int fo[4];
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) fo[kb] = (unsigned int)l32 * 128u + (unsigned int)((2 * kb + half) ^ dma_swz(l32)) * 16u;
    auto read_frags = [&](int buf, int kb, bf8v (&fa)[4], bf8v (&fw)[2]) {
        const char *base = reinterpret_cast<const char *>(&s_op[buf][0]) + fo[kb];
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) fa[mi] = *reinterpret_cast<const bf8v *>(base + (128 * wm + 32 * mi) * (BK * 2));
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) fw[ni] = *reinterpret_cast<const bf8v *>(base + OP * 2 + (64 * wn + 32 * ni) * (BK * 2));
    };
    f16v acc[2][4];
    auto clear_acc = [&]() {
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[ni][mi][v] = 0.0f;
    };
    // acc[ni][mi] = (W rows)(A rows)^T: a lane owns row l32 of the A block and, per four registers,
    // four consecutive columns
    auto multiply = [&](const bf8v (&fa)[4], const bf8v (&fw)[2]) {
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
                acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[ni], fa[mi], acc[ni][mi], 0, 0, 0);
    };
    Tile ct = tile_of(first);
    int cn = 0, cks = 0;
    bool stores_behind = false;            // an output tile was stored after the copies the next wait is for
    auto epilogue = [&]() {
        // 16 rows x 64 columns at a time through this wave's LDS patch (2 KB), so that a global store
        // instruction writes eight whole 128-byte lines; 16-byte chunk c of patch row r sits at chunk
        // position c ^ (r % 8).  Rows and columns past the end fall outside the buffer descriptor and are
        // dropped, so the number of store instructions never depends on the data: sixteen.
        unsigned short *stage = &s_epi[w][0];
        const int rows_here = a.M - (ct.m0 + 128 * wm);                   // valid rows of this wave's part (may be <= 0)
        const bool cols_here = ct.n0 + 64 * wn < a.N;                     // N is a multiple of 64: all 64 columns or none
        unsigned short *C = static_cast<unsigned short *>(a.C) + ct.coff + (long long)(ct.m0 + 128 * wm) * a.ldc + ct.n0 + 64 * wn;
        const long long valid = (rows_here > 0 && cols_here) ? (long long)(min(rows_here, 128) - 1) * a.ldc * 2 + 128 : 0;
        const buf_rsrc rc = __builtin_amdgcn_make_buffer_rsrc(C, 0, (int)valid, 0x27000);
        const int r16 = l32 & 15;
        // this lane's bias values, read once: between the patch writes below the compiler keeps LDS
        // accesses in order, and every read would wait out the LDS latency by itself
        f4v bias4[2][4];
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f4v zero = {0.0f, 0.0f, 0.0f, 0.0f};
                bias4[ni][q] = BIAS ? *reinterpret_cast<const f4v *>(&s_bias[cn & 3][w][32 * ni + 8 * q + 4 * half]) : zero;
            }
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int ph = 0; ph < 2; ++ph) {                              // rows 16 ph .. 16 ph + 15 of the 32-row block
                if ((l32 >> 4) == ph) {
#pragma unroll
                    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            f4v o = {acc[ni][mi][4 * q], acc[ni][mi][4 * q + 1], acc[ni][mi][4 * q + 2], acc[ni][mi][4 * q + 3]};
                            if (BIAS) o += bias4[ni][q];
                            store4(stage + r16 * 64 + ((4 * ni + q) ^ (r16 & 7)) * 8 + 4 * half, o);
                        }
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int it = 0; it < 2; ++it) {
                    const int r = 8 * it + (lane >> 3), cc = lane & 7;
                    const u4v v = *reinterpret_cast<const u4v *>(stage + r * 64 + (cc ^ (r & 7)) * 8);
                    const unsigned int off = (unsigned int)(32 * mi + 16 * ph + r) * (unsigned int)a.ldc * 2u + (unsigned int)cc * 16u;
                    __builtin_amdgcn_raw_buffer_store_b128(v, rc, off, 0, 0);
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                __builtin_amdgcn_wave_barrier();
            }
    };

    // ---- prologue: two steps on their way, the first one landed
    point_at(ct);
    issue(0);
    issue(1);
    asm volatile("s_waitcnt vmcnt(8)" ::: "memory");       // the eight copies of the second step may be outstanding
    asm volatile("s_barrier" ::: "memory");
    bf8v fa0[4], fw0[2], fa1[4], fw1[2];
    read_frags(0, 0, fa0, fw0);
    clear_acc();

    for (int T = 0;; ++T) {
        const int buf = T & 1;
        read_frags(buf, 1, fa1, fw1);
        __builtin_amdgcn_sched_barrier(0);
        multiply(fa0, fw0);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(buf, 2, fa0, fw0);
        __builtin_amdgcn_sched_barrier(0);
        multiply(fa1, fw1);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(buf, 3, fa1, fw1);
        __builtin_amdgcn_sched_barrier(0);
        multiply(fa0, fw0);
        __builtin_amdgcn_sched_barrier(0);
        // own copies of step T + 1 have landed, own reads of this stage are done; after the barrier
        // everybody's.  Behind those copies the wave has issued nothing, or the sixteen stores of an output tile.
        if (stores_behind) asm volatile("s_waitcnt vmcnt(16) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        stores_behind = false;
        read_frags(buf ^ 1, 0, fa0, fw0);
        if (!l_end) issue(buf);
        __builtin_amdgcn_sched_barrier(0);
        multiply(fa1, fw1);
        __builtin_amdgcn_sched_barrier(0);
        if (++cks == nk) {
            epilogue();
            stores_behind = true;
            clear_acc();
            cks = 0;
            const int nt = (int)uniform((unsigned int)s_ring[++cn & 7]);
            if (nt >= n_local) break;
            ct = tile_of(nt);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// ------------------------------- NT product, fp32 A and C, operands copied straight into LDS
// The kernel above for fp32 storage: rows of A arrive as fp32 (32 k = 128 bytes per row and step) and
// are rounded to bf16 when a lane reads its fragment (two 16-byte reads and four conversions per
// fragment); W is the bf16 copy, 32 k = 64 bytes per row and step, sixteen rows per copy instruction,
// 16-byte chunk c of row r at position c ^ (r / 4 % 4): sixteen rows of a fragment read then cover all
// banks once.  A step is two rounds of eight products; a stage is 32 KB of A and 16 KB of W.  A wave owns
// 64 rows of A x 128 rows of W (the fp32 fragments are the costly ones in registers: two per round instead
// of four).  With 32 k per step a step's products last a quarter of a microsecond, far less than a trip to
// memory, so there are three stages and the copies run two steps ahead; that takes all of LDS, and output
// tiles leave straight from the registers.
namespace dmaf {
constexpr int BK = 32;
constexpr int OPA = 256 * BK * 4;        // bytes of the A tile of a stage
constexpr int STAGE = OPA + 256 * BK * 2;  // A tile, then W tile
}  // namespace dmaf

__device__ __forceinline__ int dmaf_wswz(int row) { return (row >> 2) & 3; }

template <bool BIAS>
__global__ __launch_bounds__(512) void proj_gemm_nt_dma_f32_kernel(const GemmArgs a)
{
    constexpr int BM = dma::BM, BN = dma::BN, BK = dmaf::BK, OPA = dmaf::OPA, STAGE = dmaf::STAGE;
    __shared__ __attribute__((aligned(16))) unsigned char s_op[3][STAGE];
    __shared__ __attribute__((aligned(16))) float s_bias[2][8][128];
    __shared__ int s_ring[8];
    const int xcd = blockIdx.x & 7;
    const int inner_n = a.tiles_n * a.n_batch;
    // the XCD's (row block, inner) grid in patches of 8 x 8 tiles, as in proj_gemm_nt_kernel
    const int mx = (a.tiles_m + 7) / 8;
    int my_rows = a.tiles_m - xcd * mx;
    if (my_rows > mx) my_rows = mx;
    if (my_rows <= 0) return;
    const int n_local = my_rows * inner_n;
    const int nk = a.K / BK;
    const int tid = threadIdx.x, lane = tid & 63, w = (int)uniform((unsigned int)tid >> 6), wm = w & 3, wn = w >> 2;
    const int half = lane >> 5, l32 = lane & 31;
    if (tid == 0) s_ring[0] = atomicAdd(a.tickets + xcd, a.draw);
    __syncthreads();
    const int first = (int)uniform((unsigned int)s_ring[0]);
    if (first >= n_local) return;

    struct Tile {
        const float *A;
        const unsigned short *Bw;
        long long coff;
        int m0, n0;
    };
    auto tile_of = [&](int local) {
        const int pm = local / (8 * inner_n), rem = local - pm * 8 * inner_n;
        const int hm = min(8, my_rows - 8 * pm);
        const int pn = rem / (8 * hm), rem2 = rem - pn * 8 * hm;
        const int hn = min(8, inner_n - 8 * pn);
        const int mt = xcd * mx + 8 * pm + rem2 / hn, inner = 8 * pn + rem2 % hn;
        const int nt = inner % a.tiles_n, z = inner / a.tiles_n;
        const int z0 = z % a.nz0, z1 = z / a.nz0;
        Tile t;
        t.A = static_cast<const float *>(a.A) + z0 * a.a_off[0] + z1 * a.a_off[1];
        t.Bw = a.Bw + z0 * a.b_off[0] + z1 * a.b_off[1];
        t.coff = z0 * a.c_off[0] + z1 * a.c_off[1];
        t.m0 = mt * BM; t.n0 = nt * BN;
        return t;
    };

    // ---- the copying side: tile number ln of this workgroup, k-step lks of it.  A wave copies rows
    //      32 w .. 32 w + 31 of both operand tiles: eight rows of A (eight lanes each) or sixteen rows
    //      of W (four lanes each) per instruction.
    const unsigned int lds_op = lds_address(&s_op[0][0]);
    const int lrow = lane >> 3;
    u4v ra, rb, rbias;
    unsigned int va[4], vb[2], vbias[2] = {0u, 0u};
    int ln = 0, lks = 0;
    long long seg_base = 0;                // element offset of the current k-segment in a row of A
    int kin = 0;                           // k within the segment
    bool l_end = false;
    auto point_at = [&](const Tile &t) {
        ra = rsrc_words(t.A + (long long)t.m0 * a.lda);
        rb = rsrc_words(t.Bw + (long long)t.n0 * a.ldb);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            // rows past the end read the last row (valid memory); their products are never stored
            const int row = 32 * w + 8 * j + lrow;
            const unsigned int chunk = (unsigned int)((lane & 7) ^ dma_swz(8 * j + lrow));
            const int gm = min(t.m0 + row, a.M - 1) - t.m0;
            va[j] = (unsigned int)gm * (unsigned int)a.lda * 4u + chunk * 16u;
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int row = 32 * w + 16 * j + (lane >> 2);
            const unsigned int chunk = (unsigned int)((lane & 3) ^ dmaf_wswz(row));
            const int gn = min(t.n0 + row, a.N - 1) - t.n0;
            vb[j] = (unsigned int)gn * (unsigned int)a.ldb * 2u + chunk * 16u;
        }
        if (BIAS) {
            rbias = rsrc_words(a.bias + t.coff);
#pragma unroll
            for (int j = 0; j < 2; ++j) vbias[j] = (unsigned int)min(t.n0 + 128 * wn + 64 * j + lane, a.N - 1) * 4u;
        }
        seg_base = 0; kin = 0;
    };
    // thread 0: the numbers drawn and not yet handed out
    int next_no = first + 1, left = a.draw - 1;
    auto draw = [&]() {
        // the number of tile ln + 1 goes into the ring; it is read after at least one barrier
        if (tid == 0) {
            if (left == 0) {
                next_no = atomicAdd(a.tickets + xcd, a.draw);
                left = a.draw;
            }
            s_ring[(ln + 1) & 7] = next_no++;
            --left;
        }
    };
    // the copies of the next step in stream order, into stage `buf`
    auto issue = [&](int buf) {
        if (lks == nk) {
            const int t = (int)uniform((unsigned int)s_ring[(ln + 1) & 7]);      // written at least a barrier ago
            if (t >= n_local) {
                l_end = true;
                return;
            }
            point_at(tile_of(t));
            ++ln;
            lks = 0;
        }
        if (lks == 0) {
            draw();
            if (BIAS) {
#pragma unroll
                for (int j = 0; j < 2; ++j) copy_to_lds_4(lds_address(&s_bias[ln & 1][w][64 * j]), rbias, vbias[j], 0u);
            }
        }
        const unsigned int soa = (unsigned int)((seg_base + kin) * 4), sob = (unsigned int)(lks * BK) * 2u;
        const unsigned int dst = lds_op + (unsigned int)buf * (unsigned int)STAGE;
#pragma unroll
        for (int j = 0; j < 4; ++j) copy_to_lds_16(dst + (unsigned int)(32 * w + 8 * j) * 128u, ra, va[j], soa);
#pragma unroll
        for (int j = 0; j < 2; ++j) copy_to_lds_16(dst + OPA + (unsigned int)(32 * w + 16 * j) * 64u, rb, vb[j], sob);
        ++lks;
        kin += BK;
        if (kin == a.kseg) {
            kin = 0;
            seg_base += a.kseg_stride;
        }
    };

    // ---- the multiplying side
    // byte offsets of this lane's fragment pieces within a 32-row block, for the two 16-k rounds of a step:
    // eight fp32 of an A row (two chunks, rounded to bf16 here), eight bf16 of a W row (one chunk)
    unsigned int foa[2][2], fow[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int e = 0; e < 2; ++e) foa[kb][e] = (unsigned int)l32 * 128u + (unsigned int)((4 * kb + 2 * half + e) ^ dma_swz(l32)) * 16u;
        fow[kb] = (unsigned int)OPA + (unsigned int)l32 * 64u + (unsigned int)((2 * kb + half) ^ dmaf_wswz(l32)) * 16u;
    }
    auto read_frags = [&](int buf, int kb, bf8v (&fa)[2], bf8v (&fw)[4]) {
        const unsigned char *base = &s_op[buf][0];
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
            const unsigned char *row = base + (64 * wm + 32 * mi) * 128;
            const f4v lo = *reinterpret_cast<const f4v *>(row + foa[kb][0]), hi = *reinterpret_cast<const f4v *>(row + foa[kb][1]);
            const u4v r = {pack2(lo[0], lo[1]), pack2(lo[2], lo[3]), pack2(hi[0], hi[1]), pack2(hi[2], hi[3])};
            fa[mi] = __builtin_bit_cast(bf8v, r);
        }
#pragma unroll
        for (int ni = 0; ni < 4; ++ni) fw[ni] = *reinterpret_cast<const bf8v *>(base + fow[kb] + (128 * wn + 32 * ni) * 64);
    };
    f16v acc[4][2];
    auto clear_acc = [&]() {
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[ni][mi][v] = 0.0f;
    };
    // acc[ni][mi] = (W rows)(A rows)^T: a lane owns row l32 of the A block and, per four registers,
    // four consecutive columns
    auto multiply = [&](const bf8v (&fa)[2], const bf8v (&fw)[4]) {
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int ni = 0; ni < 4; ++ni)
                acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[ni], fa[mi], acc[ni][mi], 0, 0, 0);
    };
    Tile ct = tile_of(first);
    int cn = 0, cks = 0;
    auto epilogue = [&]() {
        // straight from the registers: a lane owns row l32 of each 32 x 32 block and, per four registers, four
        // consecutive columns, so a store instruction writes 32 bytes of 32 rows (all of LDS belongs to the
        // three stages).  Rows and columns past the end fall outside the buffer descriptor and are dropped, so
        // the number of store instructions never depends on the data: thirty-two.
        const int rows_here = a.M - (ct.m0 + 64 * wm);                    // valid rows of this wave's part (may be <= 0)
        const int cols_here = min(a.N - (ct.n0 + 128 * wn), 128);         // valid columns: a multiple of 64 (may be <= 0)
        float *C = static_cast<float *>(a.C) + ct.coff + (long long)(ct.m0 + 64 * wm) * a.ldc + ct.n0 + 128 * wn;
        const long long valid = (rows_here > 0 && cols_here > 0) ? (long long)(min(rows_here, 64) - 1) * a.ldc * 4 + 512 : 0;
        const buf_rsrc rc = __builtin_amdgcn_make_buffer_rsrc(C, 0, (int)valid, 0x27000);
        const unsigned int lane_off = (unsigned int)l32 * (unsigned int)a.ldc * 4u + (unsigned int)half * 16u;
        const float *bias_w = &s_bias[cn & 1][w][4 * half];
#pragma unroll
        for (int ni = 0; ni < 4; ++ni) {
            // columns past the end (a part that is only half there) go beyond the descriptor too
            const unsigned int col_off = 32 * ni < cols_here ? (unsigned int)(32 * ni) * 4u : 0x80000000u;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f4v zero = {0.0f, 0.0f, 0.0f, 0.0f};
                const f4v b4 = BIAS ? *reinterpret_cast<const f4v *>(bias_w + 32 * ni + 8 * q) : zero;
#pragma unroll
                for (int mi = 0; mi < 2; ++mi) {
                    f4v o = {acc[ni][mi][4 * q], acc[ni][mi][4 * q + 1], acc[ni][mi][4 * q + 2], acc[ni][mi][4 * q + 3]};
                    if (BIAS) o += b4;
                    const unsigned int off = lane_off + (unsigned int)(32 * mi) * (unsigned int)a.ldc * 4u + col_off + (unsigned int)(8 * q) * 4u;
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u4v, o), rc, off, 0, 0);
                }
            }
        }
    };

    // ---- prologue: three steps on their way, the first one landed
    point_at(ct);
    issue(0);
    issue(1);
    issue(2);
    asm volatile("s_waitcnt vmcnt(12)" ::: "memory");      // the copies of the second and third step may be outstanding
    asm volatile("s_barrier" ::: "memory");
    bf8v fa0[2], fw0[4], fa1[2], fw1[4];
    read_frags(0, 0, fa0, fw0);
    clear_acc();

    // Step T is multiplied from stage T % 3 while the copies of steps T + 1 and T + 2 are under way; after the
    // barrier of step T its stage takes the copies of step T + 3.  At that barrier the copies of step T + 1 must
    // have landed; behind them the wave has issued the six copies of step T + 2 (unless the list of steps has
    // ended) and, for two steps after an output tile, its 32 stores.
    int st = 0;                            // T % 3
    int stores_behind = 0;                 // steps for which the stores of an output tile are still behind the copies waited for
    for (;;) {
        read_frags(st, 1, fa1, fw1);
        __builtin_amdgcn_sched_barrier(0);
        multiply(fa0, fw0);
        __builtin_amdgcn_sched_barrier(0);
        if (stores_behind) {
            if (!l_end) asm volatile("s_waitcnt vmcnt(38) lgkmcnt(0)\n\ts_barrier" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(32) lgkmcnt(0)\n\ts_barrier" ::: "memory");
            --stores_behind;
        } else {
            if (!l_end) asm volatile("s_waitcnt vmcnt(6) lgkmcnt(0)\n\ts_barrier" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        }
        // the copies first: the arithmetic of a tile change needs the registers the fp32 fragments would hold
        if (!l_end) issue(st);
        st = st == 2 ? 0 : st + 1;
        __builtin_amdgcn_sched_barrier(0);
        read_frags(st, 0, fa0, fw0);
        __builtin_amdgcn_sched_barrier(0);
        multiply(fa1, fw1);
        __builtin_amdgcn_sched_barrier(0);
        if (++cks == nk) {
            epilogue();
            stores_behind = 2;
            clear_acc();
            cks = 0;
            const int nt = (int)uniform((unsigned int)s_ring[++cn & 7]);
            if (nt >= n_local) break;
            ct = tile_of(nt);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}


// --------------------------------------------------- dWx and dbias (TN product)
struct DwArgs {
    const void *du;        // [M][G][H], storage type AT
    const void *x;         // [M][H]
    float *part;           // [S][G][H][dh] partial sums of dWx
    float *dbpart;         // [S][G][H] partial sums of dbias, or NULL
    int M, H, G, heads, dh;
    int S, rows_per_split; // rows_per_split a multiple of BK
    int tiles;             // tiles per dh (128 wide; 256 wide for the copy-to-LDS kernel)
    int n_blocks, per_xcd; // tiles^2 * G * heads * S workgroups, an eighth of them (rounded up)
};

// Four adjacent channels of eight consecutive rows as fetched; transposed in registers into
// one 16-byte k-run per channel (rows that do not count become zeros), plus column sums.
template <typename AT> struct QuadRows;
template <> struct QuadRows<unsigned short> {
    uint2 v[8];
    int n_valid;
    __device__ __forceinline__ void load(const unsigned short *p, long long ld, int m, int m_last, int n_valid_)
    {
        // rows m .. m + 7, those past m_last replaced by m_last (valid memory, counted as zeros)
        const unsigned short *base = p + (long long)min(m, m_last) * ld;
        const int dm = max(m_last - m, 0), ldi = (int)ld;
#pragma unroll
        for (int r = 0; r < 8; ++r) v[r] = *reinterpret_cast<const uint2 *>(base + min(r, dm) * ldi);
        n_valid = n_valid_;
    }
    __device__ __forceinline__ void transpose(u4v (&c)[4], float (&s)[4]) const
    {
        uint2 t[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) t[r] = r < n_valid ? v[r] : make_uint2(0u, 0u);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            c[0][k] = (t[2 * k].x & 0xffffu) | (t[2 * k + 1].x << 16);
            c[1][k] = (t[2 * k].x >> 16) | (t[2 * k + 1].x & 0xffff0000u);
            c[2][k] = (t[2 * k].y & 0xffffu) | (t[2 * k + 1].y << 16);
            c[3][k] = (t[2 * k].y >> 16) | (t[2 * k + 1].y & 0xffff0000u);
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            s[0] += __builtin_bit_cast(float, t[r].x << 16);
            s[1] += __builtin_bit_cast(float, t[r].x & 0xffff0000u);
            s[2] += __builtin_bit_cast(float, t[r].y << 16);
            s[3] += __builtin_bit_cast(float, t[r].y & 0xffff0000u);
        }
    }
};
template <> struct QuadRows<float> {
    f4v v[8];
    int n_valid;
    __device__ __forceinline__ void load(const float *p, long long ld, int m, int m_last, int n_valid_)
    {
        const float *base = p + (long long)min(m, m_last) * ld;
        const int dm = max(m_last - m, 0), ldi = (int)ld;
#pragma unroll
        for (int r = 0; r < 8; ++r) v[r] = *reinterpret_cast<const f4v *>(base + min(r, dm) * ldi);
        n_valid = n_valid_;
    }
    __device__ __forceinline__ void transpose(u4v (&c)[4], float (&s)[4]) const
    {
        const f4v zero = {0.0f, 0.0f, 0.0f, 0.0f};
        f4v t[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) t[r] = r < n_valid ? v[r] : zero;
#pragma unroll
        for (int ch = 0; ch < 4; ++ch)
#pragma unroll
            for (int k = 0; k < 4; ++k) c[ch][k] = pack2(t[2 * k][ch], t[2 * k + 1][ch]);
#pragma unroll
        for (int r = 0; r < 8; ++r)
#pragma unroll
            for (int ch = 0; ch < 4; ++ch) s[ch] += t[r][ch];
    }
};

// One workgroup: a 128 x 128 tile of dWx[g][head] for one row range.  Tile rows are
// the output channels i (operand du), tile columns the input channels j (operand x);
// k runs over the rows m of the range, 64 per step.  A thread stages channels
// 4 c4 .. 4 c4 + 3 of rows 8 rg .. 8 rg + 7 of the step for both operands.
template <typename AT>
__global__ __launch_bounds__(256, 2) void proj_dw_kernel(const DwArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned short s_a[2][TILE];
    __shared__ __attribute__((aligned(16))) unsigned short s_b[2][TILE];
    __shared__ float s_db[8][BM];
    // Workgroups go to the eight XCDs round-robin; numbering them so that each XCD works through a
    // contiguous range keeps the tiles that share operand panels (the tiles of one (head, range):
    // x is common to its gates, du to its column tiles) on one L2 at about the same time.
    int id = (int)(blockIdx.x & 7) * a.per_xcd + (int)(blockIdx.x >> 3);
    if (id >= a.n_blocks) return;
    const int tj = id % a.tiles; id /= a.tiles;
    const int ti = id % a.tiles; id /= a.tiles;
    const int g = id % a.G; id /= a.G;
    const int head = id % a.heads;
    const int s = id / a.heads;
    const int i0 = ti * BM, j0 = tj * BN;
    const int m_begin = s * a.rows_per_split;
    const int m_end = min(a.M, m_begin + a.rows_per_split);
    const long long ld_du = (long long)a.G * a.H, ld_x = a.H;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, wm = w >> 1, wn = w & 1;
    const int half = lane >> 5, l32 = lane & 31;
    const int c4 = tid & 31, rg = tid >> 5;
    // dh is a multiple of 64: a quad of channels is valid or not as a whole; an invalid one reads
    // the tile's first quad (valid memory) and counts as zeros
    const bool ok_a = i0 + 4 * c4 < a.dh, ok_b = j0 + 4 * c4 < a.dh;
    const AT *du = static_cast<const AT *>(a.du) + (long long)g * a.H + head * a.dh + i0 + (ok_a ? 4 * c4 : 0);
    const AT *x = static_cast<const AT *>(a.x) + head * a.dh + j0 + (ok_b ? 4 * c4 : 0);

    float sdb[4] = {0.0f, 0.0f, 0.0f, 0.0f}, unused[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    struct Stage {
        QuadRows<AT> a, b;
    };
    int m_next = m_begin;
    auto load_next = [&](Stage &r) {
        // past the end of the range the last step is fetched again and counts as zeros
        const bool real = m_next < m_end;
        const int m = (real ? m_next : m_next - BK) + 8 * rg;
        const int n_valid = real ? m_end - m : 0;      // rows of this thread's group that count
        r.a.load(du, ld_du, m, a.M - 1, ok_a ? n_valid : 0);
        r.b.load(x, ld_x, m, a.M - 1, ok_b ? n_valid : 0);
        if (real) m_next += BK;
    };
    auto store_stage = [&](int buf, const Stage &r) {
        if (buf < 0) return;
        u4v ca[4], cb[4];
        r.a.transpose(ca, sdb);
        r.b.transpose(cb, unused);
        // lane c4 stores its channels in the order ch = (i + c4 / 2) % 4: the eight neighbouring lanes
        // of a 16-byte store pass then hit eight different 16-byte bank groups
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int ch = (i + (c4 >> 1)) & 3;
            const u4v va = ch == 0 ? ca[0] : ch == 1 ? ca[1] : ch == 2 ? ca[2] : ca[3];
            const u4v vb = ch == 0 ? cb[0] : ch == 1 ? cb[1] : ch == 2 ? cb[2] : cb[3];
            *reinterpret_cast<u4v *>(&s_a[buf][lds_off(4 * c4 + ch, rg)]) = va;
            *reinterpret_cast<u4v *>(&s_b[buf][lds_off(4 * c4 + ch, rg)]) = vb;
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
    int steps_done = 0;
    auto compute = [&](int buf) {
        mma_step<false>(s_a[buf], s_b[buf], wm, wn, l32, half, acc);
        ++steps_done;
    };
    auto done = [&]() { return steps_done >= nk; };
    if (nk > 0) {
        if constexpr (sizeof(AT) == 4) one_ahead<Stage>(load_next, store_stage, compute, done);
        else two_ahead<Stage>(load_next, store_stage, compute, done);
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
#pragma unroll
        for (int ch = 0; ch < 4; ++ch) s_db[rg][4 * c4 + ch] = sdb[ch];
        __syncthreads();
        if (tid < BM && i0 + tid < a.dh) {
            float t = 0.0f;
#pragma unroll
            for (int q = 0; q < 8; ++q) t += s_db[q][tid];
            a.dbpart[((long long)s * a.G + g) * a.H + head * a.dh + i0 + tid] = t;
        }
    }
}

// ------------------------------- dWx and dbias, bf16 operands copied straight into LDS
// The same sums for bf16 storage and wide heads: 256 x 256 outputs per workgroup of eight waves
// (2 x 4; a wave owns 128 output channels i x 64 input channels j), 64 rows m per step, operand rows
// copied from memory to LDS as they are, 512 bytes of du and of x per row.
//
//   LDS      two stages of (64 + 64) rows x 512 bytes = 128 KB.  A copy instruction moves two rows;
//            16-byte chunk c of row r lies at position c ^ dw_swz(r) of its row.
//   reads    the products need, per lane, eight consecutive m of one channel: a column of the
//            stage.  ds_read_b64_tr_b16 hands a lane four of them: the sixteen lanes of a group read
//            8 bytes each, four lanes per row over four rows (32 bytes = 16 channels of a row), and
//            lane i of the group receives the i-th channel of the four rows.  With the chunk
//            positions above the four rows of a group lie in four different parts of the banks.
//   rows     past the end of a range lie beyond the buffer descriptor, which is rebuilt for every
//            step (base at the step's first row, extent to the end of the range): the copy writes
//            zeros for them, so they add nothing.  Tile columns past dh hold whatever follows in the
//            row (a neighbouring head or gate; zeros past the end of the tensor) and their sums are
//            not stored.
//   dbias    the column sums of du come from one more product per round, with an operand of ones,
//            in the tiles of the first column block; the wave with wn = mi does block mi.
namespace dwd {
constexpr int BT = 256, BK = 64;
constexpr int OP = BK * BT;              // bf16 elements of one operand's rows of a step
constexpr int STAGE = 2 * OP;            // du rows, then x rows
}  // namespace dwd

// position of 16-byte chunk c in stage row r: c ^ dw_swz(r).  Rows r .. r + 3 (r a multiple of four) get
// four different values both in bits 1-2 and in bits 2-3 of the chunk index: the four rows of a transposing
// read then lie in different 32-byte quarters of a 128-byte window and in different 64-byte quarters of a
// 256-byte window of the banks, whichever the LDS serves per cycle.
__device__ __forceinline__ int dw_swz(int row) { return (0xca60 >> (4 * (row & 3))) & 15; }       // 0, 6, 10, 12

typedef short s4v __attribute__((ext_vector_type(4)));
typedef short s8v __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) char *lds_char_ptr;
typedef __attribute__((address_space(3))) s4v *lds_s4v_ptr;

__global__ __launch_bounds__(512) void proj_dw_dma_kernel(const DwArgs a)
{
    constexpr int BT = dwd::BT, BK = dwd::BK, OP = dwd::OP, STAGE = dwd::STAGE;
    __shared__ __attribute__((aligned(16))) unsigned short s_op[2][STAGE];
    // Workgroups go to the eight XCDs round-robin and an XCD runs 32 of its contiguous range at a
    // time: the tiles of a (gate, head, range) are numbered in strips of four tile rows, down the strip's columns,
    // so that 32 consecutive ones cover 4 x 8 tiles (8 x panels, 4 du panels) where a head has that many.
    int id = (int)(blockIdx.x & 7) * a.per_xcd + (int)(blockIdx.x >> 3);
    if (id >= a.n_blocks) return;
    const int per_grid = a.tiles * a.tiles;
    const int in_grid = id % per_grid; id /= per_grid;
    const int strip = in_grid / (4 * a.tiles), in_strip = in_grid - strip * 4 * a.tiles;
    const int hs = min(4, a.tiles - 4 * strip);
    const int tj = in_strip / hs, ti = 4 * strip + in_strip % hs;
    const int g = id % a.G; id /= a.G;
    const int head = id % a.heads;
    const int s = id / a.heads;
    const int i0 = ti * BT, j0 = tj * BT;
    const int m_begin = s * a.rows_per_split;
    const int rows = min(a.M, m_begin + a.rows_per_split) - m_begin;
    const int nk = (rows + BK - 1) / BK;
    if (nk <= 0) return;
    const int tid = threadIdx.x, lane = tid & 63, w = (int)uniform((unsigned int)tid >> 6), wm = w >> 2, wn = w & 3;
    const int half = lane >> 5, l32 = lane & 31;
    const bool do_db = a.dbpart && tj == 0;

    // ---- the copying side: a wave copies rows 8 w .. 8 w + 7 of both operands' steps, two rows per instruction
    const long long ld_du = (long long)a.G * a.H, ld_x = a.H;
    const long long col_du = (long long)g * a.H + head * a.dh + i0, col_x = (long long)head * a.dh + j0;
    unsigned long long p_du = (unsigned long long)(static_cast<const unsigned short *>(a.du) + (long long)m_begin * ld_du + col_du);
    unsigned long long p_x = (unsigned long long)(static_cast<const unsigned short *>(a.x) + (long long)m_begin * ld_x + col_x);
    // bytes from there that belong to the range: whole rows, and the tile's columns of the last one
    long long rem_du = ((long long)(rows - 1) * ld_du + min((long long)BT, ld_du - col_du)) * 2;
    long long rem_x = ((long long)(rows - 1) * ld_x + min((long long)BT, ld_x - col_x)) * 2;
    unsigned int va[4], vb[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = 8 * w + 2 * j + (lane >> 5);
        const unsigned int chunk = (unsigned int)((lane & 31) ^ dw_swz(row));
        va[j] = (unsigned int)row * (unsigned int)ld_du * 2u + chunk * 16u;
        vb[j] = (unsigned int)row * (unsigned int)ld_x * 2u + chunk * 16u;
    }
    const unsigned int lds_op = lds_address(&s_op[0][0]);
    const lds_char_ptr lds_zero = (lds_char_ptr)&s_op[0][0] - lds_op;       // LDS address 0, as a pointer
    auto words = [&](unsigned long long p, long long rem) {
        const unsigned int n = rem <= 0 ? 0u : rem > 0xffffffffll ? 0xffffffffu : (unsigned int)rem;
        const u4v r = {uniform((unsigned int)p), uniform((unsigned int)(p >> 32) & 0xffffu), uniform(n), 0x27000u};
        return r;
    };
    auto issue = [&](int buf) {
        const u4v ra = words(p_du, rem_du), rb = words(p_x, rem_x);
        const unsigned int dst = lds_op + (unsigned int)buf * (STAGE * 2u) + (unsigned int)(8 * w) * (BT * 2u);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            copy_to_lds_16(dst + (unsigned int)j * (2u * BT * 2u), ra, va[j], 0u);
            copy_to_lds_16(dst + OP * 2u + (unsigned int)j * (2u * BT * 2u), rb, vb[j], 0u);
        }
        p_du += (unsigned long long)(BK * ld_du * 2); rem_du -= BK * ld_du * 2;
        p_x += (unsigned long long)(BK * ld_x * 2);   rem_x -= BK * ld_x * 2;
    };

    // ---- the multiplying side
    // this lane's place in a transposing read: row rr of the four, the 8 bytes at channel 16 hi + 4 (lane % 4) of
    // the 32-channel block.  The block's first chunk is a multiple of four and the lane's chunk within the block
    // is 2 hi + lo, so its position is (block chunk ^ high bits of the row's mask) + ((2 hi + lo) ^ low bits):
    // one lane offset per value of the block chunk's bits 2-3.
    const int rr = (lane & 15) >> 2, mask = dw_swz(rr);
    const int in_block = (2 * ((lane >> 4) & 1) + ((lane & 3) >> 1)) ^ (mask & 3);
    const unsigned int rowpart = (unsigned int)(8 * half + rr) * (BT * 2u) + (unsigned int)(lane & 1) * 8u;
    unsigned int o_du[4], o_x[2];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
        o_du[mi] = lds_op + rowpart + (unsigned int)(((16 * wm + 4 * mi) ^ (mask & 12)) + in_block) * 16u;
#pragma unroll
    for (int nj = 0; nj < 2; ++nj)
        o_x[nj] = lds_op + OP * 2u + rowpart + (unsigned int)(((8 * wn + 4 * nj) ^ (mask & 12)) + in_block) * 16u;
    auto read8 = [&](unsigned int addr) {
        const s4v q0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4v_ptr)(lds_zero + addr));
        const s4v q1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4v_ptr)(lds_zero + addr + 4u * BT * 2u));
        const s8v t = __builtin_shufflevector(q0, q1, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf8v, t);
    };
    auto read_frags = [&](int buf, int kb, bf8v (&fd)[4], bf8v (&fx)[2]) {
        const unsigned int base = (unsigned int)buf * (STAGE * 2u) + (unsigned int)(16 * kb) * (BT * 2u);
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) fd[mi] = read8(o_du[mi] + base);
#pragma unroll
        for (int nj = 0; nj < 2; ++nj) fx[nj] = read8(o_x[nj] + base);
    };
    f16v acc[2][4], accdb;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        accdb[v] = 0.0f;
#pragma unroll
        for (int nj = 0; nj < 2; ++nj)
#pragma unroll
            for (int mi = 0; mi < 4; ++mi) acc[nj][mi][v] = 0.0f;
    }
    const __bf16 one = (__bf16)1.0f;
    const bf8v ones = {one, one, one, one, one, one, one, one};
    // acc[nj][mi] = (x columns)^T (du columns): a lane owns channel l32 of the du block and, per four
    // registers, four consecutive channels of x
    auto multiply = [&](const bf8v (&fd)[4], const bf8v (&fx)[2]) {
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) {
#pragma unroll
            for (int nj = 0; nj < 2; ++nj)
                acc[nj][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[nj], fd[mi], acc[nj][mi], 0, 0, 0);
            if (do_db && wn == mi) accdb = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, fd[mi], accdb, 0, 0, 0);
        }
    };

    // ---- two steps on their way, the first one landed
    issue(0);
    if (nk > 1) {
        issue(1);
        asm volatile("s_waitcnt vmcnt(8)" ::: "memory");   // the eight copies of the second step may be outstanding
    } else {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    asm volatile("s_barrier" ::: "memory");
    bf8v fd0[4], fx0[2], fd1[4], fx1[2];
    read_frags(0, 0, fd0, fx0);
    for (int T = 0; T < nk; ++T) {
        const int buf = T & 1;
        read_frags(buf, 1, fd1, fx1);
        __builtin_amdgcn_sched_barrier(0);
        multiply(fd0, fx0);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(buf, 2, fd0, fx0);
        __builtin_amdgcn_sched_barrier(0);
        multiply(fd1, fx1);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(buf, 3, fd1, fx1);
        __builtin_amdgcn_sched_barrier(0);
        multiply(fd0, fx0);
        __builtin_amdgcn_sched_barrier(0);
        // own copies of step T + 1 (the only memory operations outstanding) have landed, own reads of this
        // stage are done; after the barrier everybody's
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        read_frags(buf ^ 1, 0, fd0, fx0);                  // after the last step: stale rows, not used
        if (T + 2 < nk) issue(buf);
        __builtin_amdgcn_sched_barrier(0);
        multiply(fd1, fx1);
        __builtin_amdgcn_sched_barrier(0);
    }

    float *out = a.part + (((long long)s * a.G + g) * a.H + (long long)head * a.dh) * a.dh;
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
        const int i = i0 + 128 * wm + 32 * mi + l32;
        if (i >= a.dh) continue;
#pragma unroll
        for (int nj = 0; nj < 2; ++nj)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int j = j0 + 64 * wn + 32 * nj + 8 * q + 4 * half;       // dh is a multiple of 4
                if (j >= a.dh) continue;
                const f4v o = {acc[nj][mi][4 * q], acc[nj][mi][4 * q + 1], acc[nj][mi][4 * q + 2], acc[nj][mi][4 * q + 3]};
                *reinterpret_cast<f4v *>(out + (long long)i * a.dh + j) = o;
            }
    }
    if (do_db && half == 0) {
        // every row of the product with ones holds the column sums
        const int i = i0 + 128 * wm + 32 * wn + l32;
        if (i < a.dh) a.dbpart[((long long)s * a.G + g) * a.H + (long long)head * a.dh + i] = accdb[0];
    }
}

// ------------------------------------------------------------- weight copies
// Wb = bf16(Wx), same layout [G][H][dh]
__global__ __launch_bounds__(256) void proj_wb_kernel(const float *Wx, unsigned short *Wb, size_t n, int *tickets)
{
    if (blockIdx.x == 0 && threadIdx.x < 8) tickets[threadIdx.x] = 0;      // for the product that follows
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        Wb[i] = f32_to_bf16(Wx[i]);
}

// Wt[head][j][g dh + i] = bf16(Wx[g][head dh + i][j]): the B operand of the dx product
__global__ __launch_bounds__(256) void proj_wt_kernel(const float *Wx, unsigned short *Wt, int G, int H, int dh,
                                                      int *tickets)
{
    if (blockIdx.x == 0 && threadIdx.x < 8) tickets[threadIdx.x] = 0;      // for the product that follows
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

int g_proj_dma = 1;        // bf16 NT products use the copy-to-LDS kernel where it applies (proj_set_dma)

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

// The same for the copy-to-LDS kernel, one workgroup per compute unit: the number of ranges with the least
// estimated time, from the rounds of workgroups the device needs (a step of a 256 x 256 tile takes a compute
// unit about 2.3 us, a workgroup's start and output tile about 6 us) and the partial sums that have to be
// written and read again (about 4 TB/s); at least four steps per range.
void dw_dma_split(int M, int G, int H, int dh, int n_heads, int *S, int *rows_per_split)
{
    const int cus = device_cu_count() > 0 ? device_cu_count() : 256;
    const int tiles = (dh + dwd::BT - 1) / dwd::BT;
    const long long base_tiles = (long long)tiles * tiles * G * n_heads;
    const double nw = (double)G * H * dh;
    int best = 1;
    double best_us = 0.0;
    for (int s = 1; s <= 64; ++s) {
        int rps = (M + s - 1) / s;
        rps = (rps + dwd::BK - 1) / dwd::BK * dwd::BK;
        if (s > 1 && rps < 4 * dwd::BK) break;
        const int ranges = (M + rps - 1) / rps;
        const long long rounds = (base_tiles * ranges + cus - 1) / cus;
        const double us = (double)rounds * ((double)(rps / dwd::BK) * 2.3 + 6.0) + (ranges > 1 ? (double)ranges * nw * 8.0 / 4.0e6 : 0.0);
        if (s == 1 || us < best_us) { best_us = us; best = ranges; }
    }
    int rps = (M + best - 1) / best;
    rps = (rps + dwd::BK - 1) / dwd::BK * dwd::BK;
    *rows_per_split = rps;
    *S = (M + rps - 1) / rps;
}

// the copy-to-LDS kernel's 256-wide tiles against the 128-wide ones: taken where they cover dh with at most
// half as much again of idle tile area
bool dw_dma_shape_ok(int H, int G, int dh)
{
    const double t2 = (double)((dh + dwd::BT - 1) / dwd::BT * dwd::BT), t1 = (double)((dh + BM - 1) / BM * BM);
    return dh % 8 == 0 && H % 8 == 0 && (long long)G * H < (1 << 22) && t2 * t2 <= 1.5 * t1 * t1;
}

struct ProjLayout {
    size_t off_tickets, off_w, off_part, off_db, total;
    int S, rows_per_split, tiles;
    int S2, rows_per_split2, tiles2;       // the copy-to-LDS dWx kernel's ranges and 256-wide tiles (S2 = 0: not offered)
};

ProjLayout proj_layout(int B, int L, int H, int G, int n_heads, int backward)
{
    ProjLayout lo;
    const int dh = H / n_heads;
    const size_t nw = (size_t)G * H * dh;
    size_t off = 0;
    lo.off_tickets = off; off += 256;
    lo.off_w = off; off += r256(nw * sizeof(unsigned short));
    lo.tiles = (dh + BM - 1) / BM;
    lo.S = 0; lo.rows_per_split = 0;
    lo.S2 = 0; lo.rows_per_split2 = 0; lo.tiles2 = 0;
    lo.off_part = lo.off_db = off;
    if (backward) {
        dw_split(B * L, lo.tiles * lo.tiles * G * n_heads, &lo.S, &lo.rows_per_split);
        // room for either kernel's partial sums, so that the size does not depend on proj_set_dma
        if (dw_dma_shape_ok(H, G, dh)) {
            lo.tiles2 = (dh + dwd::BT - 1) / dwd::BT;
            dw_dma_split(B * L, G, H, dh, n_heads, &lo.S2, &lo.rows_per_split2);
        }
        const size_t s_max = (size_t)(lo.S > lo.S2 ? lo.S : lo.S2);
        lo.off_part = off; off += r256(s_max * nw * sizeof(float));
        lo.off_db = off;   off += r256(s_max * G * H * sizeof(float));
    }
    lo.total = off < 256 ? 256 : off;
    return lo;
}

template <typename AT, typename CT> hipError_t launch_nt(GemmArgs &g, hipStream_t st)
{
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + BN - 1) / BN;
    // two workgroups per compute unit (their LDS and registers allow no more), the same number on every XCD
    int slots = 2 * device_cu_count() / 8;
    if (slots < 1) slots = 1;
    if (slots > 64) slots = 64;                      // a patch of tiles has 64 members
    if (g.bias) hipLaunchKernelGGL((proj_gemm_nt_kernel<AT, CT, true>), dim3((unsigned)(8 * slots)), dim3(256), 0, st, g);
    else hipLaunchKernelGGL((proj_gemm_nt_kernel<AT, CT, false>), dim3((unsigned)(8 * slots)), dim3(256), 0, st, g);
    return hipGetLastError();
}

// the copy-to-LDS kernel: bf16 storage, at least two 64-k steps per tile, k-segments in whole steps, row
// offsets of a 256-row tile within 32 bits
bool nt_dma_ok(const GemmArgs &g)
{
    return g.K >= 2 * dma::BK && g.K % dma::BK == 0 && g.kseg % dma::BK == 0 && g.N % 64 == 0 &&
           g.lda < (1 << 22) && g.ldb < (1 << 22) && g.ldc < (1 << 22) && g.lda % 8 == 0 && g.ldb % 8 == 0 && g.ldc % 8 == 0;
}

// the same for fp32 A and C: 32-k steps
bool nt_dma_f32_ok(const GemmArgs &g)
{
    return g.K >= 3 * dmaf::BK && g.K % dmaf::BK == 0 && g.kseg % dmaf::BK == 0 && g.N % 64 == 0 &&
           g.lda < (1 << 22) && g.ldb < (1 << 22) && g.ldc < (1 << 22) && g.lda % 4 == 0 && g.ldb % 8 == 0 && g.ldc % 4 == 0;
}

hipError_t launch_nt_dma_f32(GemmArgs &g, hipStream_t st)
{
    g.tiles_m = (g.M + dma::BM - 1) / dma::BM;
    g.tiles_n = (g.N + dma::BN - 1) / dma::BN;
    int slots = device_cu_count() / 8;
    if (slots < 1) slots = 1;
    if (slots > 64) slots = 64;
    const long long per_wg = ((long long)(g.tiles_m + 7) / 8) * g.tiles_n * g.n_batch / slots;
    g.draw = per_wg >= 32 ? 4 : per_wg >= 16 ? 2 : 1;
    if (g.bias) hipLaunchKernelGGL((proj_gemm_nt_dma_f32_kernel<true>), dim3((unsigned)(8 * slots)), dim3(512), 0, st, g);
    else hipLaunchKernelGGL((proj_gemm_nt_dma_f32_kernel<false>), dim3((unsigned)(8 * slots)), dim3(512), 0, st, g);
    return hipGetLastError();
}

hipError_t launch_nt_dma(GemmArgs &g, hipStream_t st)
{
    g.tiles_m = (g.M + dma::BM - 1) / dma::BM;
    g.tiles_n = (g.N + dma::BN - 1) / dma::BN;
    // one workgroup per compute unit (its LDS allows no more), the same number on every XCD
    int slots = device_cu_count() / 8;
    if (slots < 1) slots = 1;
    if (slots > 64) slots = 64;
    // numbers per draw: about an eighth of a workgroup's share, four at most (the tail of a launch is then a few
    // tiles out of hundreds), one where a workgroup gets few tiles
    const long long per_wg = ((long long)(g.tiles_m + 7) / 8) * g.tiles_n * g.n_batch / slots;
    g.draw = per_wg >= 32 ? 4 : per_wg >= 16 ? 2 : 1;
    if (g.bias) hipLaunchKernelGGL((proj_gemm_nt_dma_kernel<true>), dim3((unsigned)(8 * slots)), dim3(512), 0, st, g);
    else hipLaunchKernelGGL((proj_gemm_nt_dma_kernel<false>), dim3((unsigned)(8 * slots)), dim3(512), 0, st, g);
    return hipGetLastError();
}

int elementwise_blocks(size_t n)
{
    size_t blocks = (n + 255) / 256;
    const size_t cap = (size_t)device_cu_count() * 16;
    return (int)(blocks < cap ? blocks : cap);
}

}  // namespace

int proj_set_dma(int on)
{
    g_proj_dma = on ? 1 : 0;
    return PARARNN_OK;
}

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
    int *tickets = reinterpret_cast<int *>(static_cast<char *>(workspace) + lo.off_tickets);
    hipLaunchKernelGGL(proj_wb_kernel, dim3(elementwise_blocks(nw)), dim3(256), 0, st, Wx, Wb, nw, tickets);
    GemmArgs g;
    memset(&g, 0, sizeof(g));
    g.A = x; g.Bw = Wb; g.C = u; g.bias = bias; g.tickets = tickets;
    g.lda = H; g.ldb = dh; g.ldc = (long long)G * H;
    g.M = B * L; g.N = dh; g.K = dh;
    g.kseg = dh; g.kseg_stride = 0;
    g.nz0 = G; g.n_batch = n_heads * G;                // z0 = gate, z1 = head: the tiles that read the same
    g.a_off[0] = 0; g.a_off[1] = dh;                   // columns of x (all gates of a head) are neighbours
    g.b_off[0] = (long long)H * dh; g.b_off[1] = (long long)dh * dh;
    g.c_off[0] = H; g.c_off[1] = dh;
    // fp32 storage: the copy-to-LDS kernel stores its output in 32-byte pieces, which costs more than its loads
    // gain once the output is four times the input (measured: 8-25 % faster with three gates, 1-9 % slower with four)
    const hipError_t e = dtype != PARARNN_BF16
                             ? ((g_proj_dma && nt_dma_f32_ok(g) && G <= 3) ? launch_nt_dma_f32(g, st) : launch_nt<float, float>(g, st))
                         : (g_proj_dma && nt_dma_ok(g)) ? launch_nt_dma(g, st) : launch_nt<unsigned short, unsigned short>(g, st);
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
        int *tickets = reinterpret_cast<int *>(ws + lo.off_tickets);
        hipLaunchKernelGGL(proj_wt_kernel, dim3(elementwise_blocks(nw)), dim3(256), 0, st, Wx, Wt, G, H, dh, tickets);
        GemmArgs g;
        memset(&g, 0, sizeof(g));
        g.A = du; g.Bw = Wt; g.C = dx; g.bias = nullptr; g.tickets = tickets;
        g.lda = (long long)G * H; g.ldb = (long long)G * dh; g.ldc = H;
        g.M = B * L; g.N = dh; g.K = G * dh;
        g.kseg = dh; g.kseg_stride = H;                 // k = (gate, i): gates are H apart in a row of du
        g.nz0 = n_heads; g.n_batch = n_heads;           // z0 = head
        g.a_off[0] = dh; g.b_off[0] = (long long)dh * G * dh; g.c_off[0] = dh;
        e = !bf ? ((g_proj_dma && nt_dma_f32_ok(g)) ? launch_nt_dma_f32(g, st) : launch_nt<float, float>(g, st))
            : (g_proj_dma && nt_dma_ok(g)) ? launch_nt_dma(g, st) : launch_nt<unsigned short, unsigned short>(g, st);
        if (e != hipSuccess) return PARARNN_HIP_ERROR;
    }
    if (dWx) {
        DwArgs a;
        memset(&a, 0, sizeof(a));
        a.du = du; a.x = x;
        a.part = reinterpret_cast<float *>(ws + lo.off_part);
        a.dbpart = dbias ? reinterpret_cast<float *>(ws + lo.off_db) : nullptr;
        a.M = B * L; a.H = H; a.G = G; a.heads = n_heads; a.dh = dh;
        const bool copy_kernel = bf && g_proj_dma && lo.S2 > 0;
        a.S = copy_kernel ? lo.S2 : lo.S;
        if (a.S == 1) {                                 // one range: its sums are the results
            a.part = dWx;
            if (dbias) a.dbpart = dbias;
        }
        a.rows_per_split = copy_kernel ? lo.rows_per_split2 : lo.rows_per_split;
        a.tiles = copy_kernel ? lo.tiles2 : lo.tiles;
        a.n_blocks = a.tiles * a.tiles * n_heads * G * a.S;
        a.per_xcd = (a.n_blocks + 7) / 8;
        const int blocks = 8 * a.per_xcd;
        if (copy_kernel) hipLaunchKernelGGL(proj_dw_dma_kernel, dim3(blocks), dim3(512), 0, st, a);
        else if (bf) hipLaunchKernelGGL(proj_dw_kernel<unsigned short>, dim3(blocks), dim3(256), 0, st, a);
        else hipLaunchKernelGGL(proj_dw_kernel<float>, dim3(blocks), dim3(256), 0, st, a);
        if (hipGetLastError() != hipSuccess) return PARARNN_HIP_ERROR;
        if (a.S > 1) {
            if (launch_param_reduce(a.part, dWx, a.S, (int)nw, st) != hipSuccess) return PARARNN_HIP_ERROR;
            if (dbias && launch_param_reduce(a.dbpart, dbias, a.S, G * H, st) != hipSuccess) return PARARNN_HIP_ERROR;
        }
    }
    return PARARNN_OK;
}

}  // namespace pararnn
