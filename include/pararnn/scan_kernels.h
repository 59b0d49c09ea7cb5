// Fused Newton-iteration kernel and fused backward kernel for cells with a
// diagonal (S = 1) or 2x2-block (S = 2) Jacobian.
//
// Work decomposition.  A "tile" is CW = (64/LL)*VEC channels of one sequence x
// T = C*LL*W consecutive timesteps:
//   lane   -> (segment, channel slot): the 64 lanes of a wave are LL segments
//             of 64/LL lanes; a lane owns VEC adjacent channels (H is the
//             contiguous axis, so each segment reads rows of (64/LL)*VEC*4
//             contiguous bytes) and C consecutive timesteps, which it reduces
//             sequentially in registers (the thread-level forward substitution
//             of the paper's App. D.2)
//   wave   -> the LL segments hold consecutive chunks of the same channels and
//             are combined by a Kogge-Stone scan with cross-lane shuffles
//   block  -> W waves take consecutive stretches; their aggregates are
//             combined through LDS
//   grid   -> tiles along L are chained by a decoupled look-back: a tile
//             publishes its aggregate affine map (A, b), then walks back over
//             its predecessors until it meets one whose inclusive value
//             (delta at the tile's end) is known.  Tiles are handed out by an
//             atomic ticket, channel groups fastest, so a tile's predecessors
//             have always started before it and every wait terminates.
// The affine maps compose as (A2,b2) o (A1,b1) = (A2 A1, A2 b1 + b2); because
// delta_0 = 0 the inclusive value of a tile is just a state vector.
//
// Nothing but u, the iterate and the new iterate crosses HBM per Newton
// iteration: residual, Jacobian, scan, update and max|delta| are fused.
#pragma once
#include <type_traits>

#include "common.h"

namespace pararnn {

// test/profiling "cell": J and r come from memory (pararnn_affine_scan)
template <int S_> struct RawScan {
    static constexpr int G = S_, S = S_, PR = 0, NC = 1;
    static constexpr bool kRaw = true;
};
template <class Cell, class = void> struct IsRaw { static constexpr bool value = false; };
template <class Cell> struct IsRaw<Cell, decltype((void)Cell::kRaw)> { static constexpr bool value = true; };

struct ScanGeom {
    int B, L, H;
    int T;         // timesteps per tile
    int n_lt;      // tiles along L
    int n_cg;      // channel groups per sequence
    int n_groups;  // B * n_cg
    int n_tiles;   // n_groups * n_lt
    unsigned int spin_limit;   // polls of one predecessor before a tile gives up
    unsigned int epoch_base;   // added to the epoch in every record tag of this call (0 unless the workspace is reused)
};

struct FwdArgs {
    ScanGeom g;
    const float *params;
    const void *u;       // [B][L][G][H], fp32 or bf16
    const void *h0;      // [B][S][H] in u's type, or NULL
    const float *jac;    // raw scans only: [B][L][S*S][H]
    float *hit;          // fp32 iterate [B][L][S][H], updated in place (raw scans: the output delta)
    int raw_add;         // raw scans only: add delta to what hit holds instead of overwriting it
    float *bnd;          // [2][n_lt][B][S][H]: iterate at each tile's last step
    int bnd_cur;         // which of the two holds the rows of the iterate being read (the other is written)
    unsigned long long *rec; // carry records [n_groups][n_lt][S*S + 2S][CW] of {value, tag}
    Ctrl *ctrl;
    int *iters_out;      // device int[2]
    float *trace;        // device float[max_iter] or NULL
    int k;               // Newton iteration (1-based); also the flag epoch
    int max_iter;
    float tol;
    int stream;          // cache policy of interior tiles: 0 plain accesses, 1 u is read as a stream, 2 the iterate as well
};

// arguments of the residual max-norm (App. A)
struct ResArgs {
    int B, L, H;
    const float *params;
    const void *u;       // [B][L][G][H]
    const void *h0;      // [B][S][H] or NULL
    const void *h;       // states [B][L][S][H] in storage type
    unsigned int *out;   // bits of the result, a non-negative float (or a NaN); zero on entry
};

struct BwdArgs {
    ScanGeom g;
    const float *params;
    const void *u;
    const void *h0;
    const void *h;       // forward result [B][L][S][H] in storage type
    const void *gl;      // dL/dh [B][L][S][H]
    const float *jac;    // raw scans only
    void *du;            // out [B][L][G][H]
    void *dh0;           // out [B][S][H] or NULL
    float *part;         // parameter-gradient partials [n_lt][B][PR][H]
    unsigned long long *rec;
    Ctrl *ctrl;
    int stage;           // the tensors allow the LDS-staged kernel variant (16-byte aligned rows)
    int stream;          // bf16 storage: interior tiles read and write their rows as streams
};

// ------------------------------------------------------------ small matrix ops
// Row-major S x S blocks in registers; outputs may alias inputs.  S = 1 and 2 (the
// cells) are written out; larger blocks (the scan on its own, S = 3, 4) loop.
// y = A x (S x S times S)
template <int S>
__device__ __forceinline__ void mat_vec(const float *A, const float *x, float *y)
{
    if constexpr (S == 1) {
        y[0] = A[0] * x[0];
    } else if constexpr (S == 2) {
        const float y0 = fmaf(A[0], x[0], A[1] * x[1]);
        const float y1 = fmaf(A[2], x[0], A[3] * x[1]);
        y[0] = y0; y[1] = y1;
    } else {
        float t[S];
#pragma unroll
        for (int i = 0; i < S; ++i) {
            float s = A[i * S] * x[0];
#pragma unroll
            for (int k = 1; k < S; ++k) s = fmaf(A[i * S + k], x[k], s);
            t[i] = s;
        }
#pragma unroll
        for (int i = 0; i < S; ++i) y[i] = t[i];
    }
}
// y = A x + b
template <int S>
__device__ __forceinline__ void affine(const float *A, const float *x, const float *b, float *y)
{
    if constexpr (S == 1) {
        y[0] = fmaf(A[0], x[0], b[0]);
    } else if constexpr (S == 2) {
        const float y0 = fmaf(A[0], x[0], fmaf(A[1], x[1], b[0]));
        const float y1 = fmaf(A[2], x[0], fmaf(A[3], x[1], b[1]));
        y[0] = y0;
        y[1] = y1;
    } else {
        float t[S];
#pragma unroll
        for (int i = 0; i < S; ++i) {
            float s = b[i];
#pragma unroll
            for (int k = 0; k < S; ++k) s = fmaf(A[i * S + k], x[k], s);
            t[i] = s;
        }
#pragma unroll
        for (int i = 0; i < S; ++i) y[i] = t[i];
    }
}
// C = A B
template <int S>
__device__ __forceinline__ void mat_mul(const float *A, const float *Bm, float *Cm)
{
    if constexpr (S == 1) {
        Cm[0] = A[0] * Bm[0];
    } else if constexpr (S == 2) {
        const float c0 = fmaf(A[0], Bm[0], A[1] * Bm[2]);
        const float c1 = fmaf(A[0], Bm[1], A[1] * Bm[3]);
        const float c2 = fmaf(A[2], Bm[0], A[3] * Bm[2]);
        const float c3 = fmaf(A[2], Bm[1], A[3] * Bm[3]);
        Cm[0] = c0; Cm[1] = c1; Cm[2] = c2; Cm[3] = c3;
    } else {
        float t[S * S];
#pragma unroll
        for (int i = 0; i < S; ++i)
#pragma unroll
            for (int j = 0; j < S; ++j) {
                float s = A[i * S] * Bm[j];
#pragma unroll
                for (int k = 1; k < S; ++k) s = fmaf(A[i * S + k], Bm[k * S + j], s);
                t[i * S + j] = s;
            }
#pragma unroll
        for (int e = 0; e < S * S; ++e) Cm[e] = t[e];
    }
}
template <int S> __device__ __forceinline__ void set_identity(float *A)
{
#pragma unroll
    for (int i = 0; i < S; ++i)
#pragma unroll
        for (int j = 0; j < S; ++j) A[i * S + j] = i == j ? 1.0f : 0.0f;
}
template <int S> __device__ __forceinline__ void transpose_inplace(float *A)
{
#pragma unroll
    for (int i = 0; i < S; ++i)
#pragma unroll
        for (int j = i + 1; j < S; ++j) {
            const float t = A[i * S + j];
            A[i * S + j] = A[j * S + i];
            A[j * S + i] = t;
        }
}

// (accA, accB) <- (J, r) o (accA, accB): apply one more step after the prefix
template <int S>
__device__ __forceinline__ void push_step(const float *J, const float *r, float *accA, float *accB)
{
    affine<S>(J, accB, r, accB);
    mat_mul<S>(J, accA, accA);
}

// compose: (accA, accB) <- (accA, accB) o (pA, pB): the map p is applied first
template <int S>
__device__ __forceinline__ void compose_after(const float *pA, const float *pB, float *accA, float *accB)
{
    affine<S>(accA, pB, accB, accB);
    mat_mul<S>(accA, pA, accA);
}

// ------------------------------------------------ cross-workgroup carry records
// Every published float travels in its own 64-bit word {value, tag} written and
// read with one relaxed agent-scope atomic access, so a word validates itself
// and no fence (an L2 write-back on this chip) is needed.  tag = epoch*4+state.
typedef unsigned long long rec_t;

__device__ __forceinline__ rec_t rec_pack(float v, unsigned int tag)
{
    return ((rec_t)tag << 32) | (rec_t)__float_as_uint(v);
}
__device__ __forceinline__ void rec_store(rec_t *p, float v, unsigned int tag)
{
    __hip_atomic_store(p, rec_pack(v, tag), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ rec_t rec_load(const rec_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Value entering tile `lt` of chain `grp`, obtained by walking over the
// predecessors in direction `dir` (-1: towards l = 0, forward scan; +1: towards
// l = L, reverse scan) until one with a known inclusive value is met.  Called
// by a whole wave; lanes with active = true own VEC channels starting at
// column `col` of the group, the others only keep the control flow uniform.
// Returns false when the bounded wait ran out (carry is then zero).
template <int S, int VEC, int CW>
__device__ __forceinline__ bool lookback(unsigned int spin_limit, const rec_t *rec_base, int n_lt, int grp, int lt, int dir,
                                         unsigned int epoch, int col, bool active, float (&carry)[S][VEC])
{
    constexpr int SS = S * S, NW = SS + 2 * S;
    const unsigned int tag_agg = epoch * 4u + kFlagAgg, tag_inc = epoch * 4u + kFlagIncl;
    float LA[VEC][SS], LB[VEC][S];
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
        set_identity<S>(LA[v]);
#pragma unroll
        for (int s = 0; s < S; ++s) LB[v][s] = 0.0f;
    }
    int j = lt + dir;
    unsigned int spins = 0;
    for (;;) {
        const rec_t *rj = rec_base + ((size_t)grp * n_lt + j) * (NW * CW) + col;
        // inclusive value and aggregate of tile j, asked for together: one trip to memory per look
        rec_t wi[S][VEC], wa[SS + S][VEC];
#pragma unroll
        for (int s = 0; s < S; ++s)
#pragma unroll
            for (int v = 0; v < VEC; ++v) wi[s][v] = active ? rec_load(rj + (SS + S + s) * CW + v) : 0;
#pragma unroll
        for (int e = 0; e < SS + S; ++e)
#pragma unroll
            for (int v = 0; v < VEC; ++v) wa[e][v] = active ? rec_load(rj + e * CW + v) : 0;
        bool ok = true;
#pragma unroll
        for (int s = 0; s < S; ++s)
#pragma unroll
            for (int v = 0; v < VEC; ++v) ok &= (unsigned int)(wi[s][v] >> 32) == tag_inc;
        if (__all(ok || !active)) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                float x[S], y[S];
#pragma unroll
                for (int s = 0; s < S; ++s) x[s] = __uint_as_float((unsigned int)wi[s][v]);
                affine<S>(LA[v], x, LB[v], y);
#pragma unroll
                for (int s = 0; s < S; ++s) carry[s][v] = y[s];
            }
            return true;
        }
        ok = true;
#pragma unroll
        for (int e = 0; e < SS + S; ++e)
#pragma unroll
            for (int v = 0; v < VEC; ++v) ok &= (unsigned int)(wa[e][v] >> 32) == tag_agg;
        if (__all(ok || !active)) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                float A1[SS], b1[S];
#pragma unroll
                for (int e = 0; e < SS; ++e) A1[e] = __uint_as_float((unsigned int)wa[e][v]);
#pragma unroll
                for (int s = 0; s < S; ++s) b1[s] = __uint_as_float((unsigned int)wa[SS + s][v]);
                compose_after<S>(A1, b1, LA[v], LB[v]);
            }
            j += dir;
            spins = 0;
            if (j < 0 || j >= n_lt) {   // ran past the end of the chain: the value there is 0
#pragma unroll
                for (int v = 0; v < VEC; ++v)
#pragma unroll
                    for (int s = 0; s < S; ++s) carry[s][v] = LB[v][s];
                return true;
            }
            continue;
        }
        if (++spins >= spin_limit) {
#pragma unroll
            for (int v = 0; v < VEC; ++v)
#pragma unroll
                for (int s = 0; s < S; ++s) carry[s][v] = 0.0f;
            return false;
        }
        __builtin_amdgcn_s_sleep(1);
    }
}

// One look at the neighbour in direction `dir`: true, and its inclusive value in `carry`, when that is already
// there.  The tile then has no need to publish its own aggregate (two thirds of a tile's record words): whoever
// asks this tile will find its inclusive value, which follows at once.  Called like lookback().
template <int S, int VEC, int CW>
__device__ __forceinline__ bool neighbour_inclusive(const rec_t *rec_base, int n_lt, int grp, int lt, int dir,
                                                    unsigned int epoch, int col, bool active, float (&carry)[S][VEC])
{
    constexpr int SS = S * S, NW = SS + 2 * S;
    const unsigned int tag_inc = epoch * 4u + kFlagIncl;
    const rec_t *rj = rec_base + ((size_t)grp * n_lt + (lt + dir)) * (NW * CW) + col;
    rec_t wi[S][VEC];
    bool ok = true;
#pragma unroll
    for (int s = 0; s < S; ++s)
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            wi[s][v] = active ? rec_load(rj + (SS + S + s) * CW + v) : 0;
            ok = ok && (unsigned int)(wi[s][v] >> 32) == tag_inc;
        }
    if (!__all(ok || !active)) return false;
#pragma unroll
    for (int s = 0; s < S; ++s)
#pragma unroll
        for (int v = 0; v < VEC; ++v) carry[s][v] = __uint_as_float((unsigned int)wi[s][v]);
    return true;
}

template <int N, int VEC, int CW>
__device__ __forceinline__ void publish(rec_t *rec_rows, const float (&val)[N][VEC], unsigned int tag, int col,
                                        bool active)
{
    if (active) {
#pragma unroll
        for (int e = 0; e < N; ++e)
#pragma unroll
            for (int v = 0; v < VEC; ++v) rec_store(rec_rows + e * CW + col + v, val[e][v], tag);
    }
}

__device__ __forceinline__ float wave_nanmax(float m)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = nanmax(m, __shfl_xor(m, off, 64));
    return m;
}

// ======================================================================
// One Newton iteration (Alg. 1a body): residual + Jacobian (Eq. (3)), prefix
// scan of Eq. (4), update, max|delta|, and the device-side stopping test.
// ======================================================================
// FIRST = true is iteration 1 with the initial guess folded in: the old iterate
// h^0_l = f(h0, u_l) (App. A) is computed from u on the fly instead of being read
// (one extra row of u per chunk supplies h^0_{l0-1}), so no separate pass
// writes and re-reads the guess.
template <class Cell, int VEC, int LL, int C, int W, typename UT, bool FIRST>
__global__ __launch_bounds__(kWave *W) void newton_iter_kernel(const FwdArgs a)
{
    constexpr int S = Cell::S, G = Cell::G, SS = S * S, PR = Cell::PR;
    constexpr int LPS = kWave / LL, CW = LPS * VEC, NW = SS + 2 * S, T = C * LL * W;
    constexpr bool kRaw = IsRaw<Cell>::value;
    __shared__ float s_A[W][SS][CW];
    __shared__ float s_b[W][S][CW];
    __shared__ float s_carry[S][CW];
    __shared__ float s_max[W];
    __shared__ unsigned int s_ticket;

    Ctrl *ctrl = a.ctrl;
    if (ctrl->stop) return;
    const ScanGeom &g = a.g;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // wave-uniform: keep it scalar
    const int seg = lane / LPS, col = (lane % LPS) * VEC;
    const unsigned int epoch = g.epoch_base + (unsigned int)a.k;
    const UT *u = static_cast<const UT *>(a.u);
    const int cur = a.bnd_cur, nxt = cur ^ 1;
    // max |delta| as its bit pattern: for non-negative floats the unsigned order is the float order, and
    // NaN patterns sort above infinity, so one integer max both orders the values and keeps a NaN
    unsigned int wmax_bits = 0u;
    bool internal_error = false;

    for (;;) {
        if (threadIdx.x == 0) s_ticket = atomicAdd(&ctrl->ticket, 1u);
        __syncthreads();
        // the ticket comes through LDS; make it scalar so that the whole tile geometry is computed on the SALU
        const unsigned int t = __builtin_amdgcn_readfirstlane(s_ticket);
        if (t >= (unsigned int)g.n_tiles) break;
        const int grp = (int)(t % (unsigned int)g.n_groups), lt = (int)(t / (unsigned int)g.n_groups);
        const int b = grp / g.n_cg, cg = grp - b * g.n_cg;
        const int ch = cg * CW + col;
        const bool ch_ok = ch < g.H;
        const int l0 = lt * T + (w * LL + seg) * C;
        const size_t seq = (size_t)b * g.L;
        // interior tiles address memory as buffer resource (scalar base of the wave's first row)
        // + one per-lane byte offset + a scalar row offset: no per-load vector address arithmetic
        const int wl = lt * T + w * (LL * C);
        const unsigned int Hn = (unsigned int)g.H;
        const size_t row_w = seq + (size_t)wl;
        const buf_rsrc ru = make_rsrc(u + row_w * G * Hn + (size_t)cg * CW);
        const buf_rsrc rh = make_rsrc(a.hit + row_w * S * Hn + (size_t)cg * CW);
        const buf_rsrc rj = make_rsrc(kRaw ? a.jac + row_w * SS * Hn + (size_t)cg * CW : nullptr);
        const unsigned int vu = ((unsigned int)(seg * (C * G)) * Hn + col) * (unsigned int)sizeof(UT);
        const unsigned int vh = ((unsigned int)(seg * (C * S)) * Hn + col) * 4u;
        const unsigned int vj = ((unsigned int)(seg * (C * SS)) * Hn + col) * 4u;

        float p[VEC][PR > 0 ? PR : 1];
        if constexpr (PR > 0) {
#pragma unroll
            for (int r = 0; r < PR; ++r) {
                float tmp[VEC];
#pragma unroll
                for (int v = 0; v < VEC; ++v) tmp[v] = 0.0f;
                if (ch_ok) load_vec<VEC>(a.params + (size_t)r * g.H + ch, tmp);
#pragma unroll
                for (int v = 0; v < VEC; ++v) p[v][r] = tmp[v];
            }
        }

        // ---- loads: u and the old iterate for the C steps of this thread, kept
        // raw so that all of them are in flight together; tiles that lie fully
        // inside the tensor take the unguarded path
        using RawU = typename RawVec<UT, VEC>::type;
        using RawF = typename RawVec<float, VEC>::type;
        RawU uur[C][G], uhalo[FIRST ? G : 1];
        RawF hor[FIRST ? 1 : C][S], jrr[kRaw ? C : 1][kRaw ? SS : 1];
        float hprev[S][VEC];
        const bool full_tile = (lt + 1) * T <= g.L && (cg + 1) * CW <= g.H;
        auto load_inputs = [&](auto guard, auto stream) {
            constexpr bool kGuard = decltype(guard)::value;
            constexpr int kAuxU = decltype(stream)::value >= 1 ? kAuxStream : kAuxNone;
            constexpr int kAuxHld = decltype(stream)::value >= 2 ? kAuxStream : kAuxNone;
#pragma unroll
            for (int i = 0; i < C; ++i) {
                const int l = l0 + i;
                const bool ok = !kGuard || (ch_ok && l < g.L);
#pragma unroll
                for (int q = 0; q < G; ++q) {
                    if constexpr (!kGuard) uur[i][q] = buf_load<UT, VEC, kAuxU>(ru, vu, (unsigned int)(i * G + q) * Hn * (unsigned int)sizeof(UT));
                    else if (ok) uur[i][q] = load_raw<UT, VEC>(u + ((seq + l) * G + q) * g.H + ch);
                    else uur[i][q] = zero_raw<UT, VEC>();
                }
                if constexpr (!FIRST) {
#pragma unroll
                    for (int s = 0; s < S; ++s) {
                        if (!kRaw || a.raw_add) {
                            if constexpr (!kGuard) hor[i][s] = buf_load<float, VEC, kAuxHld>(rh, vh, (unsigned int)(i * S + s) * Hn * 4u);
                            else if (ok) hor[i][s] = load_raw<float, VEC>(a.hit + ((seq + l) * S + s) * g.H + ch);
                            else hor[i][s] = zero_raw<float, VEC>();
                        } else {
                            hor[i][s] = zero_raw<float, VEC>();
                        }
                    }
                }
                if constexpr (kRaw) {
#pragma unroll
                    for (int e = 0; e < SS; ++e) {
                        if constexpr (!kGuard) jrr[i][e] = buf_load<float, VEC>(rj, vj, (unsigned int)(i * SS + e) * Hn * 4u);
                        else if (ok) jrr[i][e] = load_raw<float, VEC>(a.jac + ((seq + l) * SS + e) * g.H + ch);
                        else jrr[i][e] = zero_raw<float, VEC>();
                    }
                }
            }
        };
        // which tensors are streamed is the host's choice (they stay out of the caches' way when the
        // iteration's working set is larger than the memory-side cache)
        if (!full_tile) load_inputs(std::true_type{}, std::integral_constant<int, 0>{});
        else if (a.stream >= 2) load_inputs(std::false_type{}, std::integral_constant<int, 2>{});
        else if (a.stream == 1) load_inputs(std::false_type{}, std::integral_constant<int, 1>{});
        else load_inputs(std::false_type{}, std::integral_constant<int, 0>{});
        if constexpr (FIRST) {
#pragma unroll
            for (int q = 0; q < G; ++q) {
                uhalo[q] = zero_raw<UT, VEC>();
                if (ch_ok && l0 > 0 && l0 <= g.L) uhalo[q] = load_raw<UT, VEC>(u + ((seq + l0 - 1) * G + q) * Hn + ch);
            }
        }
        // state entering the chunk: h0, the previous tile's boundary row, or
        // the row just before the chunk (still the old iterate: every store of
        // this tile comes after the barriers below)
#pragma unroll
        for (int s = 0; s < S; ++s) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) hprev[s][v] = 0.0f;
            if constexpr (FIRST) {
                if (ch_ok && a.h0) load_vec<VEC>(static_cast<const UT *>(a.h0) + ((size_t)b * S + s) * g.H + ch, hprev[s]);
            } else if constexpr (!kRaw) {
                if (ch_ok && l0 <= g.L) {
                    if (l0 == 0) {
                        if (a.h0) load_vec<VEC>(static_cast<const UT *>(a.h0) + ((size_t)b * S + s) * g.H + ch, hprev[s]);
                    } else if (w == 0 && seg == 0) {
                        load_vec<VEC>(a.bnd + ((((size_t)cur * g.n_lt + (lt - 1)) * g.B + b) * S + s) * g.H + ch, hprev[s]);
                    } else {
                        load_vec<VEC>(a.hit + ((seq + l0 - 1) * S + s) * g.H + ch, hprev[s]);
                    }
                }
            }
        }

        // ---- thread level: local prefix (PA_i, qb_i) after each of the C steps
        float PA[C][VEC][SS], qb[C][VEC][S], accA[VEC][SS], accB[VEC][S];
        float uu[C][G][VEC], ho[C][S][VEC], jr[kRaw ? C : 1][kRaw ? SS : 1][VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            set_identity<S>(accA[v]);
#pragma unroll
            for (int s = 0; s < S; ++s) accB[v][s] = 0.0f;
        }
        float h0v[FIRST ? S : 1][VEC];
        if constexpr (FIRST) {
            // hprev holds h0 here; the state entering the chunk is the guess of
            // the row before it, f(h0, u_{l0-1}), or h0 itself at the sequence start
#pragma unroll
            for (int s = 0; s < S; ++s)
#pragma unroll
                for (int v = 0; v < VEC; ++v) h0v[s][v] = hprev[s][v];
            if (l0 > 0) {
                float uh[G][VEC];
#pragma unroll
                for (int q = 0; q < G; ++q) raw_to_float<UT, VEC>(uhalo[q], uh[q]);
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    float h1[S], ug[G], F0[S];
#pragma unroll
                    for (int s = 0; s < S; ++s) h1[s] = h0v[s][v];
#pragma unroll
                    for (int q = 0; q < G; ++q) ug[q] = uh[q][v];
                    Cell::step(p[v], h1, ug, F0);
#pragma unroll
                    for (int s = 0; s < S; ++s) hprev[s][v] = F0[s];
                }
            }
        }
#pragma unroll
        for (int i = 0; i < C; ++i) {
#pragma unroll
            for (int q = 0; q < G; ++q) raw_to_float<UT, VEC>(uur[i][q], uu[i][q]);
            if constexpr (FIRST) {
                // old iterate = initial guess h^0_l = f(h0, u_l)
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    float h1[S], ug[G], F0[S];
#pragma unroll
                    for (int s = 0; s < S; ++s) h1[s] = h0v[s][v];
#pragma unroll
                    for (int q = 0; q < G; ++q) ug[q] = uu[i][q][v];
                    Cell::step(p[v], h1, ug, F0);
#pragma unroll
                    for (int s = 0; s < S; ++s) ho[i][s][v] = F0[s];
                }
            } else {
#pragma unroll
                for (int s = 0; s < S; ++s) raw_to_float<float, VEC>(hor[i][s], ho[i][s]);
            }
            if constexpr (kRaw) {
#pragma unroll
                for (int e = 0; e < SS; ++e) raw_to_float<float, VEC>(jrr[i][e], jr[i][e]);
            }
            if (l0 + i < g.L) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    float J[SS], r[S];
                    if constexpr (kRaw) {
#pragma unroll
                        for (int e = 0; e < SS; ++e) J[e] = jr[i][e][v];
#pragma unroll
                        for (int s = 0; s < S; ++s) r[s] = uu[i][s][v];
                    } else {
                        float hp[S], ug[G], F[S];
#pragma unroll
                        for (int s = 0; s < S; ++s) hp[s] = i == 0 ? hprev[s][v] : ho[i - 1][s][v];
#pragma unroll
                        for (int q = 0; q < G; ++q) ug[q] = uu[i][q][v];
                        Cell::fwd(p[v], hp, ug, F, J);
#pragma unroll
                        for (int s = 0; s < S; ++s) r[s] = F[s] - ho[i][s][v];
                    }
                    push_step<S>(J, r, accA[v], accB[v]);
                }
            }
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
#pragma unroll
                for (int e = 0; e < SS; ++e) PA[i][v][e] = accA[v][e];
#pragma unroll
                for (int s = 0; s < S; ++s) qb[i][v][s] = accB[v][s];
            }
        }

        // ---- wave level: Kogge-Stone scan over the LL segments of the wave
        // (lanes seg*LPS.. hold consecutive chunks of the same channels)
        float lexA[VEC][SS], lexB[VEC][S];   // map of the segments before this one
        if constexpr (LL > 1) {
#pragma unroll
            for (int d = 1; d < LL; d <<= 1) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    float pA[SS], pB[S];
#pragma unroll
                    for (int e = 0; e < SS; ++e) pA[e] = __shfl_up(accA[v][e], d * LPS, 64);
#pragma unroll
                    for (int s = 0; s < S; ++s) pB[s] = __shfl_up(accB[v][s], d * LPS, 64);
                    if (seg >= d) compose_after<S>(pA, pB, accA[v], accB[v]);
                }
            }
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
#pragma unroll
                for (int e = 0; e < SS; ++e) lexA[v][e] = __shfl_up(accA[v][e], LPS, 64);
#pragma unroll
                for (int s = 0; s < S; ++s) lexB[v][s] = __shfl_up(accB[v][s], LPS, 64);
                if (seg == 0) {
                    set_identity<S>(lexA[v]);
#pragma unroll
                    for (int s = 0; s < S; ++s) lexB[v][s] = 0.0f;
                }
            }
        }

        // ---- workgroup level: wave aggregates through LDS
        if (seg == LL - 1) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
#pragma unroll
                for (int e = 0; e < SS; ++e) s_A[w][e][col + v] = accA[v][e];
#pragma unroll
                for (int s = 0; s < S; ++s) s_b[w][s][col + v] = accB[v][s];
            }
        }
        __syncthreads();

        // map of the waves before this one (all waves) / of the whole tile (wave 0)
        float exA[VEC][SS], exB[VEC][S];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            set_identity<S>(exA[v]);
#pragma unroll
            for (int s = 0; s < S; ++s) exB[v][s] = 0.0f;
        }
        const int upto = w == 0 ? W : w;
        for (int j = 0; j < upto; ++j) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                float Aj[SS], bj[S];
#pragma unroll
                for (int e = 0; e < SS; ++e) Aj[e] = s_A[j][e][col + v];
#pragma unroll
                for (int s = 0; s < S; ++s) bj[s] = s_b[j][s][col + v];
                push_step<S>(Aj, bj, exA[v], exB[v]);
            }
        }
        if (w == 0) {
            // ---- grid level: decoupled look-back along L, lanes of segment 0
            float tileA[SS][VEC], tileB[S][VEC], carry[S][VEC];
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
#pragma unroll
                for (int e = 0; e < SS; ++e) tileA[e][v] = exA[v][e];
#pragma unroll
                for (int s = 0; s < S; ++s) { tileB[s][v] = exB[v][s]; exB[v][s] = 0.0f; carry[s][v] = 0.0f; }
                set_identity<S>(exA[v]);
            }
            const bool active = seg == 0;
            const bool has_next = lt + 1 < g.n_lt;
            rec_t *rec = a.rec + ((size_t)grp * g.n_lt + lt) * (NW * CW);
            if (lt > 0 && !neighbour_inclusive<S, VEC, CW>(a.rec, g.n_lt, grp, lt, -1, epoch, col, active, carry)) {
                if (has_next) {
                    float ab[SS + S][VEC];
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
#pragma unroll
                        for (int e = 0; e < SS; ++e) ab[e][v] = tileA[e][v];
#pragma unroll
                        for (int s = 0; s < S; ++s) ab[SS + s][v] = tileB[s][v];
                    }
                    publish<SS + S, VEC, CW>(rec, ab, epoch * 4u + kFlagAgg, col, active);
                }
                if (!lookback<S, VEC, CW>(g.spin_limit, a.rec, g.n_lt, grp, lt, -1, epoch, col, active, carry))
                    internal_error = true;
            }
            if (has_next) {
                float inc[S][VEC];
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    float A1[SS], x[S], b1[S], y[S];
#pragma unroll
                    for (int e = 0; e < SS; ++e) A1[e] = tileA[e][v];
#pragma unroll
                    for (int s = 0; s < S; ++s) { x[s] = carry[s][v]; b1[s] = tileB[s][v]; }
                    affine<S>(A1, x, b1, y);
#pragma unroll
                    for (int s = 0; s < S; ++s) inc[s][v] = y[s];
                }
                publish<S, VEC, CW>(rec + (SS + S) * CW, inc, epoch * 4u + kFlagIncl, col, active);
            }
            if (active) {
#pragma unroll
                for (int s = 0; s < S; ++s)
#pragma unroll
                    for (int v = 0; v < VEC; ++v) s_carry[s][col + v] = carry[s][v];
            }
        }
        __syncthreads();

        // ---- back-substitution: delta entering this chunk, then every step
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            float cin[S], din[S];
#pragma unroll
            for (int s = 0; s < S; ++s) cin[s] = s_carry[s][col + v];
            affine<S>(exA[v], cin, exB[v], din);
            if constexpr (LL > 1) affine<S>(lexA[v], din, lexB[v], din);
#pragma unroll
            for (int i = 0; i < C; ++i) {
                float d[S];
                affine<S>(PA[i][v], din, qb[i][v], d);
#pragma unroll
                for (int s = 0; s < S; ++s) {
                    ho[i][s][v] += d[s];
                    if (ch_ok && l0 + i < g.L) wmax_bits = max(wmax_bits, __float_as_uint(d[s]) & 0x7fffffffu);
                }
            }
        }
        if (full_tile && a.stream >= 2) {
#pragma unroll
            for (int i = 0; i < C; ++i)
#pragma unroll
                for (int s = 0; s < S; ++s) buf_store<float, VEC, kAuxStream>(rh, vh, (unsigned int)(i * S + s) * Hn * 4u, ho[i][s]);
        } else if (full_tile) {
#pragma unroll
            for (int i = 0; i < C; ++i)
#pragma unroll
                for (int s = 0; s < S; ++s) buf_store<float, VEC>(rh, vh, (unsigned int)(i * S + s) * Hn * 4u, ho[i][s]);
        } else {
#pragma unroll
            for (int i = 0; i < C; ++i) {
                const int l = l0 + i;
                if (ch_ok && l < g.L) {
#pragma unroll
                    for (int s = 0; s < S; ++s) store_vec<VEC>(a.hit + ((seq + l) * S + s) * g.H + ch, ho[i][s]);
                }
            }
        }
        if constexpr (!kRaw) {
            if (ch_ok && w == W - 1 && seg == LL - 1 && lt + 1 < g.n_lt) {
#pragma unroll
                for (int s = 0; s < S; ++s)
                    store_vec<VEC>(a.bnd + ((((size_t)nxt * g.n_lt + lt) * g.B + b) * S + s) * g.H + ch, ho[C - 1][s]);
            }
        }
    }

    // ---- convergence reduction and, in the last workgroup, the stopping test
    float wmax = wave_nanmax(__uint_as_float(wmax_bits));
    if (lane == 0) s_max[w] = wmax;
    if (internal_error && lane == 0) atomicExch(&ctrl->status, kStInternal);
    __syncthreads();
    if (threadIdx.x == 0) {
        float m = 0.0f;
#pragma unroll
        for (int j = 0; j < W; ++j) m = nanmax(m, s_max[j]);
        atomicMax(&ctrl->gmax_bits, __float_as_uint(m));
        __threadfence();
        const unsigned int prev = atomicAdd(&ctrl->done, 1u);
        if (prev == gridDim.x - 1) {
            __threadfence();
            const float mk = __uint_as_float(atomicMax(&ctrl->gmax_bits, 0u));
            int status = atomicAdd(&ctrl->status, 0), stop = 0;
            if (a.trace) a.trace[a.k - 1] = mk;
            if (status == kStInternal) {
                stop = 1;
            } else if (!(mk - mk == 0.0f)) {
                status = kStNonFinite;
                stop = 1;
            } else if (a.tol >= 0.0f && mk <= a.tol) {
                status = kStOk;
                stop = 1;
            } else {
                status = a.tol < 0.0f ? kStOk : kStNotConverged;
            }
            a.iters_out[0] = a.k;
            a.iters_out[1] = status;
            ctrl->iters = a.k;
            ctrl->status = status;
            ctrl->stop = stop;
            ctrl->ticket = 0u;
            ctrl->done = 0u;
            ctrl->gmax_bits = 0u;
            __threadfence();
        }
    }
}

// Residual max-norm of given states (App. A, the observable of the convergence
// figure): max |h_l - f(h_{l-1}, u_l)| over everything.  A thread owns VEC channels
// and kResRun consecutive steps, so each state row is read once as h_l and carried
// in registers as h_{l-1} of the next step (plus one extra row per run).  One
// atomic max per workgroup; NaNs propagate (their bit pattern orders above +inf).
constexpr int kResRun = 8;

template <class Cell, int VEC, typename UT>
__global__ __launch_bounds__(256) void residual_norm_kernel(const ResArgs a)
{
    constexpr int S = Cell::S, G = Cell::G, PR = Cell::PR;
    __shared__ float s_max[4];
    const int hv = a.H / VEC;
    const int n_runs = (a.L + kResRun - 1) / kResRun;
    const size_t n = (size_t)a.B * n_runs * hv;
    const UT *u = static_cast<const UT *>(a.u), *h = static_cast<const UT *>(a.h);
    float m = 0.0f;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (size_t)gridDim.x * blockDim.x) {
        const int ch = (int)(idx % hv) * VEC;
        const size_t br = idx / hv;
        const int l0 = (int)(br % n_runs) * kResRun;
        const size_t b = br / n_runs;
        const int l1 = min(a.L, l0 + kResRun);
        float p[VEC][PR], hp[S][VEC];
#pragma unroll
        for (int r = 0; r < PR; ++r) {
            float tmp[VEC];
            load_vec<VEC>(a.params + (size_t)r * a.H + ch, tmp);
#pragma unroll
            for (int v = 0; v < VEC; ++v) p[v][r] = tmp[v];
        }
#pragma unroll
        for (int s = 0; s < S; ++s) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) hp[s][v] = 0.0f;
            if (l0 > 0) load_vec<VEC>(h + ((b * a.L + l0 - 1) * S + s) * a.H + ch, hp[s]);
            else if (a.h0) load_vec<VEC>(static_cast<const UT *>(a.h0) + (b * S + s) * a.H + ch, hp[s]);
        }
        for (int l = l0; l < l1; ++l) {
            const size_t row = b * a.L + l;
            float uu[G][VEC], hl[S][VEC];
#pragma unroll
            for (int q = 0; q < G; ++q) load_vec<VEC>(u + (row * G + q) * a.H + ch, uu[q]);
#pragma unroll
            for (int s = 0; s < S; ++s) load_vec<VEC>(h + (row * S + s) * a.H + ch, hl[s]);
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                float h1[S], u1[G], F[S];
#pragma unroll
                for (int s = 0; s < S; ++s) h1[s] = hp[s][v];
#pragma unroll
                for (int q = 0; q < G; ++q) u1[q] = uu[q][v];
                Cell::step(p[v], h1, u1, F);
#pragma unroll
                for (int s = 0; s < S; ++s) {
                    m = nanmax(m, fabsf(hl[s][v] - F[s]));
                    hp[s][v] = hl[s][v];
                }
            }
        }
    }
    m = wave_nanmax(m);
    if ((threadIdx.x & 63) == 0) s_max[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        m = nanmax(nanmax(s_max[0], s_max[1]), nanmax(s_max[2], s_max[3]));
        atomicMax(a.out, m != m ? 0x7fc00000u : __float_as_uint(m));
    }
}

// Initial guess h^0_l = f(h0, u_l) for every l (App. A), plus the boundary rows
// the first iteration reads.  One thread per (b, l, VEC channels).
template <class Cell, int VEC, typename UT>
__global__ __launch_bounds__(256) void init_guess_kernel(const FwdArgs a)
{
    constexpr int S = Cell::S, G = Cell::G, PR = Cell::PR;
    const ScanGeom &g = a.g;
    const int hv = g.H / VEC;
    const size_t n = (size_t)g.B * g.L * hv;
    const UT *u = static_cast<const UT *>(a.u);
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n; idx += (size_t)gridDim.x * blockDim.x) {
        const int ch = (int)(idx % hv) * VEC;
        const size_t bl = idx / hv;
        const int l = (int)(bl % g.L), b = (int)(bl / g.L);
        float p[VEC][PR], uu[G][VEC], hp[S][VEC], out[S][VEC];
#pragma unroll
        for (int r = 0; r < PR; ++r) {
            float tmp[VEC];
            load_vec<VEC>(a.params + (size_t)r * g.H + ch, tmp);
#pragma unroll
            for (int v = 0; v < VEC; ++v) p[v][r] = tmp[v];
        }
#pragma unroll
        for (int q = 0; q < G; ++q) load_vec<VEC>(u + (bl * G + q) * g.H + ch, uu[q]);
#pragma unroll
        for (int s = 0; s < S; ++s) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) hp[s][v] = 0.0f;
            if (a.h0) load_vec<VEC>(static_cast<const UT *>(a.h0) + ((size_t)b * S + s) * g.H + ch, hp[s]);
        }
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            float h1[S], u1[G], F[S];
#pragma unroll
            for (int s = 0; s < S; ++s) h1[s] = hp[s][v];
#pragma unroll
            for (int q = 0; q < G; ++q) u1[q] = uu[q][v];
            Cell::step(p[v], h1, u1, F);
#pragma unroll
            for (int s = 0; s < S; ++s) out[s][v] = F[s];
        }
#pragma unroll
        for (int s = 0; s < S; ++s) store_vec<VEC>(a.hit + (bl * S + s) * g.H + ch, out[s]);
        if ((l + 1) % g.T == 0 && (l + 1) / g.T < g.n_lt) {
            const int lt = (l + 1) / g.T - 1;
            // iteration 1 reads boundary buffer 1 (k & 1)
#pragma unroll
            for (int s = 0; s < S; ++s)
                store_vec<VEC>(a.bnd + ((((size_t)1 * g.n_lt + lt) * g.B + b) * S + s) * g.H + ch, out[s]);
        }
    }
}


// ======================================================================
// Backward (Eq. (6)) as one reverse scan.  With nu_l = J_l^T lam_l the adjoint
// recurrence lam_{l-1} = J_l^T lam_l + g_{l-1} reads
//     nu_l = J_l^T nu_{l+1} + J_l^T g_l,   nu_{L+1} = 0,   lam_l = g_l + nu_{l+1},
// so element l of the scan needs only step l's own data (h_{l-1}, u_l, g_l).
// dL/dh0 = nu_1.  Parameter gradients are reduced per tile into `part`
// and summed by param_reduce_kernel (fixed order: bit-reproducible).
// ======================================================================
//
// STAGE = true (bf16 storage, one channel per lane, one segment per wave, C a
// multiple of 8): the inputs of a tile do not pass through registers on their way
// from memory.  Every wave copies the rows of its own C steps straight into LDS
// (buffer loads with the LDS destination: 8 rows of 64 bf16 = 1 KiB per
// instruction) one tile ahead, so the loads of the next tile are in flight during
// the whole of the current tile's arithmetic, look-forward and stores, and cost
// no registers.  A workgroup therefore holds two tickets, the tile it works on
// and the one it has staged; tickets are still handed out in increasing order
// and a workgroup works through its own in that order, so the tile with the
// smallest unfinished ticket never waits for an unfinished one and every wait
// ends as before.  Tiles at the ragged edges of the tensor and the first tile of
// a sequence (its h_{l-1} rows start before the sequence) take the register path.
template <class Cell, int VEC, int LL, int C, int W, typename UT, bool STAGE = false>
__global__ __launch_bounds__(kWave *W) void backward_kernel(const BwdArgs a)
{
    constexpr int S = Cell::S, G = Cell::G, SS = S * S, PR = Cell::PR, NC = Cell::NC;
    constexpr int LPS = kWave / LL, CW = LPS * VEC, NW = SS + 2 * S, T = C * LL * W;
    constexpr bool kRaw = IsRaw<Cell>::value;
    constexpr int PRX = PR > 0 ? PR : 1;
    constexpr int LDSROWS = (SS + S) > PRX ? (SS + S) : PRX;
    static_assert(!STAGE || (sizeof(UT) == 2 && VEC == 1 && LL == 1 && C % 8 == 0 && !kRaw),
                  "the staged variant is built for bf16 storage, one channel per lane, C % 8 == 0");
    // staged rows of one wave, 64 bf16 (32 words) each: u_l (C*G rows), h_{l-1} (C*S), g_l (C*S)
    constexpr int kRowsU = C * G, kRowsS = C * S;
    constexpr int kStageWords = STAGE ? (kRowsU + 2 * kRowsS) * 32 : 1;
    __shared__ float s_buf[W][LDSROWS][CW];   // wave aggregates, then gradient partials
    __shared__ float s_carry[S][CW];
    __shared__ unsigned int s_ticket;
    __shared__ unsigned int s_first[2];
    __shared__ __attribute__((aligned(16))) unsigned int s_stage[STAGE ? W : 1][kStageWords];

    Ctrl *ctrl = a.ctrl;
    const ScanGeom &g = a.g;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // wave-uniform: keep it scalar
    const int seg = lane / LPS, col = (lane % LPS) * VEC;
    const unsigned int epoch = g.epoch_base + 1u;
    const UT *u = static_cast<const UT *>(a.u);
    const UT *hres = static_cast<const UT *>(a.h);
    const UT *gl = static_cast<const UT *>(a.gl);
    UT *du = static_cast<UT *>(a.du);
    bool internal_error = false;

    // parameters of the channels this lane owns in channel group cg_
    auto load_params = [&](int cg_, float (&dst)[VEC][PRX]) {
#pragma unroll
        for (int r = 0; r < PRX; ++r) {
            float tmp[VEC];
#pragma unroll
            for (int v = 0; v < VEC; ++v) tmp[v] = 0.0f;
            if constexpr (STAGE) {
                // no branch, so that nothing waits for the value before it is used: channels past the
                // end read the last channel's parameters and are masked where results are stored
                const int chn_ = min(cg_ * CW + col, g.H - 1);
                if (PR > 0) tmp[0] = a.params[(size_t)r * g.H + chn_];
            } else {
                if (PR > 0 && cg_ * CW + col < g.H) load_vec<VEC>(a.params + (size_t)r * g.H + cg_ * CW + col, tmp);
            }
#pragma unroll
            for (int v = 0; v < VEC; ++v) dst[v][r] = tmp[v];
        }
    };
    float pn[VEC][PRX];      // staged variant: parameters of the next tile
#pragma unroll
    for (int v = 0; v < VEC; ++v)
#pragma unroll
        for (int r = 0; r < PRX; ++r) pn[v][r] = 0.0f;

    // ---- staged variant: which tiles go through LDS, and the copy of a tile's rows
    auto stageable = [&](unsigned int t_) -> bool {
        if constexpr (!STAGE) {
            return false;
        } else {
            if (!a.stage || t_ >= (unsigned int)g.n_tiles) return false;
            const int grp_ = (int)(t_ % (unsigned int)g.n_groups);
            const int lt_ = g.n_lt - 1 - (int)(t_ / (unsigned int)g.n_groups);
            const int cg_ = grp_ % g.n_cg;
            return lt_ > 0 && (lt_ + 1) * T <= g.L && (cg_ + 1) * CW <= g.H;
        }
    };
    auto stage_tile_as = [&](unsigned int t_, auto stream) {
        if constexpr (STAGE) {
            constexpr int kAux = decltype(stream)::value ? kAuxStream : kAuxNone;
            typedef __attribute__((address_space(3))) void *lds_ptr;
            const int grp_ = (int)(t_ % (unsigned int)g.n_groups);
            const int lt_ = g.n_lt - 1 - (int)(t_ / (unsigned int)g.n_groups);
            const int b_ = grp_ / g.n_cg, cg_ = grp_ - b_ * g.n_cg;
            const unsigned int Hn_ = (unsigned int)g.H;
            const size_t row_ = (size_t)b_ * g.L + (size_t)(lt_ * T + w * C);      // first step of this wave
            // lane -> one of 8 rows, 16 bytes of its 128
            const unsigned int voff = (unsigned int)(lane >> 3) * Hn_ * 2u + (unsigned int)(lane & 7) * 16u;
            const buf_rsrc su = make_rsrc(u + row_ * G * Hn_ + (size_t)cg_ * CW);
            const buf_rsrc sh = make_rsrc(hres + (row_ - 1) * S * Hn_ + (size_t)cg_ * CW);   // h_{l-1}: lt_ > 0
            const buf_rsrc sg = make_rsrc(gl + row_ * S * Hn_ + (size_t)cg_ * CW);
#pragma unroll
            for (int j = 0; j < kRowsU / 8; ++j)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(su, (lds_ptr)&s_stage[w][j * 256], 16, voff,
                                                         (unsigned int)(j * 8) * Hn_ * 2u, 0, kAux);
#pragma unroll
            for (int j = 0; j < kRowsS / 8; ++j) {
                __builtin_amdgcn_raw_ptr_buffer_load_lds(sh, (lds_ptr)&s_stage[w][(kRowsU / 8 + j) * 256], 16, voff,
                                                         (unsigned int)(j * 8) * Hn_ * 2u, 0, kAux);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(sg, (lds_ptr)&s_stage[w][((kRowsU + kRowsS) / 8 + j) * 256], 16,
                                                         voff, (unsigned int)(j * 8) * Hn_ * 2u, 0, kAux);
            }
        }
    };
    auto stage_tile = [&](unsigned int t_) {
        if (a.stream) stage_tile_as(t_, std::true_type{});
        else stage_tile_as(t_, std::false_type{});
    };
    unsigned int t = 0, t_next = 0;
    bool cur_staged = false;
    if constexpr (STAGE) {
        if (threadIdx.x == 0) {
            s_first[0] = atomicAdd(&ctrl->ticket, 1u);
            s_first[1] = atomicAdd(&ctrl->ticket, 1u);
        }
        __syncthreads();
        t = __builtin_amdgcn_readfirstlane(s_first[0]);
        t_next = __builtin_amdgcn_readfirstlane(s_first[1]);
        cur_staged = stageable(t);
        if (cur_staged) stage_tile(t);
        if (t < (unsigned int)g.n_tiles) load_params((int)(t % (unsigned int)g.n_groups) % g.n_cg, pn);
    }

    for (;;) {
        if constexpr (STAGE) {
            // the workgroup's third ticket, read after the first barrier below; the barrier here keeps
            // the previous tile's reads of s_buf (gradient partials) ahead of this tile's writes
            lds_barrier();
            if (t >= (unsigned int)g.n_tiles) break;
            if (threadIdx.x == 0) s_ticket = atomicAdd(&ctrl->ticket, 1u);
        } else {
            if (threadIdx.x == 0) s_ticket = atomicAdd(&ctrl->ticket, 1u);
            __syncthreads();
            // the ticket comes through LDS; make it scalar so that the whole tile geometry is computed on the SALU
            t = __builtin_amdgcn_readfirstlane(s_ticket);
            if (t >= (unsigned int)g.n_tiles) break;
        }
        const int grp = (int)(t % (unsigned int)g.n_groups);
        const int lt = g.n_lt - 1 - (int)(t / (unsigned int)g.n_groups);   // from the end of the sequence
        const int b = grp / g.n_cg, cg = grp - b * g.n_cg;
        const int ch = cg * CW + col;
        const bool ch_ok = ch < g.H;
        const int l0 = lt * T + (w * LL + seg) * C;
        const size_t seq = (size_t)b * g.L;
        const int wl = lt * T + w * (LL * C);
        const unsigned int Hn = (unsigned int)g.H;
        const size_t row_w = seq + (size_t)wl;
        const buf_rsrc ru = make_rsrc(u + row_w * G * Hn + (size_t)cg * CW);
        const buf_rsrc rdu = make_rsrc(du + row_w * G * Hn + (size_t)cg * CW);
        const buf_rsrc rg = make_rsrc(gl + row_w * S * Hn + (size_t)cg * CW);
        // h one row earlier (address arithmetic on the integer value: for the very first row of the tensor
        // the base lies one row before the buffer and is never dereferenced, since l = 0 reads h0)
        const buf_rsrc rh1 = make_rsrc(reinterpret_cast<const void *>(reinterpret_cast<uintptr_t>(hres) +
                                       (row_w * S * Hn + (size_t)cg * CW) * sizeof(UT) - (size_t)S * Hn * sizeof(UT)));
        const buf_rsrc rj = make_rsrc(kRaw ? a.jac + row_w * SS * Hn + (size_t)cg * CW : nullptr);
        const unsigned int vu = ((unsigned int)(seg * (C * G)) * Hn + col) * (unsigned int)sizeof(UT);
        const unsigned int vh = ((unsigned int)(seg * (C * S)) * Hn + col) * (unsigned int)sizeof(UT);
        const unsigned int vj = ((unsigned int)(seg * (C * SS)) * Hn + col) * 4u;

        float p[VEC][PRX];
        if constexpr (PR > 0) {
            if constexpr (STAGE) {
                // loaded one tile ahead, like the staged rows
#pragma unroll
                for (int v = 0; v < VEC; ++v)
#pragma unroll
                    for (int r = 0; r < PR; ++r) p[v][r] = pn[v][r];
            } else {
                load_params(cg, p);
            }
        }

        // ---- loads: u_l, h_{l-1}, g_l for the C steps of this thread (raw, all
        // in flight together; unguarded for tiles fully inside the tensor)
        using RawU = typename RawVec<UT, VEC>::type;
        using RawF = typename RawVec<float, VEC>::type;
        RawU uur[kRaw ? 1 : C][kRaw ? 1 : G], hpr[C][S], ggr[C][S];
        RawF jrr[kRaw ? C : 1][kRaw ? SS : 1];
        const bool full_tile = (lt + 1) * T <= g.L && (cg + 1) * CW <= g.H;
        auto load_inputs = [&](auto guard) {
            constexpr bool kGuard = decltype(guard)::value;
#pragma unroll
            for (int i = 0; i < C; ++i) {
                const int l = l0 + i;
                const bool ok = !kGuard || (ch_ok && l < g.L);
                if constexpr (!kRaw) {
#pragma unroll
                    for (int q = 0; q < G; ++q) {
                        if constexpr (!kGuard) uur[i][q] = buf_load<UT, VEC>(ru, vu, (unsigned int)(i * G + q) * Hn * (unsigned int)sizeof(UT));
                        else if (ok) uur[i][q] = load_raw<UT, VEC>(u + ((seq + l) * G + q) * g.H + ch);
                        else uur[i][q] = zero_raw<UT, VEC>();
                    }
                }
#pragma unroll
                for (int s = 0; s < S; ++s) {
                    if constexpr (!kGuard) ggr[i][s] = buf_load<UT, VEC>(rg, vh, (unsigned int)(i * S + s) * Hn * (unsigned int)sizeof(UT));
                    else if (ok) ggr[i][s] = load_raw<UT, VEC>(gl + ((seq + l) * S + s) * g.H + ch);
                    else ggr[i][s] = zero_raw<UT, VEC>();
                    hpr[i][s] = zero_raw<UT, VEC>();
                    if constexpr (!kRaw) {
                        if (ok) {
                            if (i > 0 || l > 0) {        // only a chunk's first step can be l = 0
                                if constexpr (!kGuard) hpr[i][s] = buf_load<UT, VEC>(rh1, vh, (unsigned int)(i * S + s) * Hn * (unsigned int)sizeof(UT));
                                else hpr[i][s] = load_raw<UT, VEC>(hres + ((seq + l - 1) * S + s) * g.H + ch);
                            } else if (a.h0) {
                                hpr[i][s] = load_raw<UT, VEC>(static_cast<const UT *>(a.h0) + ((size_t)b * S + s) * g.H + ch);
                            }
                        }
                    }
                }
                if constexpr (kRaw) {
#pragma unroll
                    for (int e = 0; e < SS; ++e) {
                        if constexpr (!kGuard) jrr[i][e] = buf_load<float, VEC>(rj, vj, (unsigned int)(i * SS + e) * Hn * 4u);
                        else if (ok) jrr[i][e] = load_raw<float, VEC>(a.jac + ((seq + l) * SS + e) * g.H + ch);
                        else jrr[i][e] = zero_raw<float, VEC>();
                    }
                }
            }
        };
        // ---- thread level, right to left.  For step i keep the map from the
        // value entering the chunk on the right (nu_in) to lam_i:
        //     lam_i = PX_i nu_in + qx_i,   PX_i = prod_{j>i} J_j^T,  qx_i = g_i + q_{i+1}
        float PX[C][VEC][SS], qx[C][VEC][S], kk[C][VEC][NC], accA[VEC][SS], accB[VEC][S];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            set_identity<S>(accA[v]);
#pragma unroll
            for (int s = 0; s < S; ++s) accB[v][s] = 0.0f;
        }
        // from_lds: the step's inputs are read from this wave's staged rows as they are needed
        // (no registers hold them), else from the registers load_inputs filled
        auto thread_level = [&](auto from_lds) {
            constexpr bool kLds = decltype(from_lds)::value;
#pragma unroll
            for (int i = C - 1; i >= 0; --i) {
                float uu1[G][VEC], hp1[S][VEC], gg1[S][VEC], jr1[kRaw ? SS : 1][VEC];
                if constexpr (kLds) {
                    const unsigned short *sp = reinterpret_cast<const unsigned short *>(&s_stage[w][0]);
#pragma unroll
                    for (int q = 0; q < G; ++q) uu1[q][0] = bf16_to_f32(sp[(i * G + q) * 64 + lane]);
#pragma unroll
                    for (int s = 0; s < S; ++s) {
                        hp1[s][0] = bf16_to_f32(sp[(kRowsU + i * S + s) * 64 + lane]);
                        gg1[s][0] = bf16_to_f32(sp[(kRowsU + kRowsS + i * S + s) * 64 + lane]);
                    }
                } else {
                    if constexpr (!kRaw) {
#pragma unroll
                        for (int q = 0; q < G; ++q) raw_to_float<UT, VEC>(uur[i][q], uu1[q]);
                    } else {
#pragma unroll
                        for (int e = 0; e < SS; ++e) raw_to_float<float, VEC>(jrr[i][e], jr1[e]);
                    }
#pragma unroll
                    for (int s = 0; s < S; ++s) {
                        raw_to_float<UT, VEC>(hpr[i][s], hp1[s]);
                        raw_to_float<UT, VEC>(ggr[i][s], gg1[s]);
                    }
                }
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
#pragma unroll
                    for (int e = 0; e < SS; ++e) PX[i][v][e] = accA[v][e];
#pragma unroll
                    for (int s = 0; s < S; ++s) qx[i][v][s] = accB[v][s] + gg1[s][v];
                }
                if (kLds || l0 + i < g.L) {
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        float J[SS], zero[S];
                        if constexpr (kRaw) {
#pragma unroll
                            for (int e = 0; e < SS; ++e) J[e] = jr1[e][v];
                        } else {
                            float h1[S], ug[G];
#pragma unroll
                            for (int s = 0; s < S; ++s) h1[s] = hp1[s][v];
#pragma unroll
                            for (int q = 0; q < G; ++q) ug[q] = uu1[q][v];
                            Cell::bwd_prep(p[v], h1, ug, J, kk[i][v]);
                        }
                        transpose_inplace<S>(J);
#pragma unroll
                        for (int s = 0; s < S; ++s) zero[s] = 0.0f;
                        // nu_i = J^T (g_i + nu_{i+1}):  accB = J^T qx_i,  accA = J^T accA
                        affine<S>(J, qx[i][v], zero, accB[v]);
                        mat_mul<S>(J, accA[v], accA[v]);
                    }
                }
            }
        };
        bool next_staged = false;
        if constexpr (STAGE) {
            if (cur_staged) {
                // this wave's rows were copied by this wave: its own copies have landed once its
                // outstanding-memory count is zero
                __builtin_amdgcn_s_waitcnt(0);
                thread_level(std::true_type{});
                __builtin_amdgcn_s_waitcnt(0);       // every row has been read before it is overwritten
            } else {
                if (full_tile) load_inputs(std::false_type{});
                else load_inputs(std::true_type{});
                thread_level(std::false_type{});
                __builtin_amdgcn_s_waitcnt(0);
            }
            // the next tile: its rows on their way into LDS, its parameters into registers, while this
            // tile goes through the scan levels, the look-forward, the gradient formulas and its stores
            next_staged = stageable(t_next);
            if (next_staged) stage_tile(t_next);
            if (t_next < (unsigned int)g.n_tiles) load_params((int)(t_next % (unsigned int)g.n_groups) % g.n_cg, pn);
        } else {
            if (full_tile) load_inputs(std::false_type{});
            else load_inputs(std::true_type{});
            thread_level(std::false_type{});
        }
        // chunk aggregate before the wave-level scan overwrites it (nu at the chunk's first step)
        float cA[VEC][SS], cB[VEC][S];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
#pragma unroll
            for (int e = 0; e < SS; ++e) cA[v][e] = accA[v][e];
#pragma unroll
            for (int s = 0; s < S; ++s) cB[v][s] = accB[v][s];
        }

        // ---- wave level: suffix scan over the segments to the right
        float lexA[VEC][SS], lexB[VEC][S];
        if constexpr (LL > 1) {
#pragma unroll
            for (int d = 1; d < LL; d <<= 1) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    float pA[SS], pB[S];
#pragma unroll
                    for (int e = 0; e < SS; ++e) pA[e] = __shfl_down(accA[v][e], d * LPS, 64);
#pragma unroll
                    for (int s = 0; s < S; ++s) pB[s] = __shfl_down(accB[v][s], d * LPS, 64);
                    if (seg + d < LL) compose_after<S>(pA, pB, accA[v], accB[v]);
                }
            }
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
#pragma unroll
                for (int e = 0; e < SS; ++e) lexA[v][e] = __shfl_down(accA[v][e], LPS, 64);
#pragma unroll
                for (int s = 0; s < S; ++s) lexB[v][s] = __shfl_down(accB[v][s], LPS, 64);
                if (seg == LL - 1) {
                    set_identity<S>(lexA[v]);
#pragma unroll
                    for (int s = 0; s < S; ++s) lexB[v][s] = 0.0f;
                }
            }
        }

        // ---- workgroup level
        if (seg == 0) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
#pragma unroll
                for (int e = 0; e < SS; ++e) s_buf[w][e][col + v] = accA[v][e];
#pragma unroll
                for (int s = 0; s < S; ++s) s_buf[w][SS + s][col + v] = accB[v][s];
            }
        }
        if constexpr (STAGE) lds_barrier_keep_vmem();
        else __syncthreads();
        unsigned int t_after = 0;
        if constexpr (STAGE) t_after = __builtin_amdgcn_readfirstlane(s_ticket);
        // map of the waves after this one; wave W-1 also forms the tile
        // aggregate and runs the look-forward
        float exA[VEC][SS], exB[VEC][S];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            set_identity<S>(exA[v]);
#pragma unroll
            for (int s = 0; s < S; ++s) exB[v][s] = 0.0f;
        }
        const int down_to = w == W - 1 ? 0 : w + 1;
        for (int j = W - 1; j >= down_to; --j) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                float Aj[SS], bj[S];
#pragma unroll
                for (int e = 0; e < SS; ++e) Aj[e] = s_buf[j][e][col + v];
#pragma unroll
                for (int s = 0; s < S; ++s) bj[s] = s_buf[j][SS + s][col + v];
                push_step<S>(Aj, bj, exA[v], exB[v]);
            }
        }
        if (w == W - 1) {
            float tileA[SS][VEC], tileB[S][VEC], carry[S][VEC];
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
#pragma unroll
                for (int e = 0; e < SS; ++e) tileA[e][v] = exA[v][e];
#pragma unroll
                for (int s = 0; s < S; ++s) { tileB[s][v] = exB[v][s]; exB[v][s] = 0.0f; carry[s][v] = 0.0f; }
                set_identity<S>(exA[v]);
            }
            const bool active = seg == 0;
            const bool has_next = lt > 0;            // a tile to the left will ask
            rec_t *rec = a.rec + ((size_t)grp * g.n_lt + lt) * (NW * CW);
            if (lt + 1 < g.n_lt && !neighbour_inclusive<S, VEC, CW>(a.rec, g.n_lt, grp, lt, +1, epoch, col, active, carry)) {
                if (has_next) {
                    float ab[SS + S][VEC];
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
#pragma unroll
                        for (int e = 0; e < SS; ++e) ab[e][v] = tileA[e][v];
#pragma unroll
                        for (int s = 0; s < S; ++s) ab[SS + s][v] = tileB[s][v];
                    }
                    publish<SS + S, VEC, CW>(rec, ab, epoch * 4u + kFlagAgg, col, active);
                }
                if (!lookback<S, VEC, CW>(g.spin_limit, a.rec, g.n_lt, grp, lt, +1, epoch, col, active, carry))
                    internal_error = true;
            }
            if (has_next) {
                float inc[S][VEC];
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    float A1[SS], x[S], b1[S], y[S];
#pragma unroll
                    for (int e = 0; e < SS; ++e) A1[e] = tileA[e][v];
#pragma unroll
                    for (int s = 0; s < S; ++s) { x[s] = carry[s][v]; b1[s] = tileB[s][v]; }
                    affine<S>(A1, x, b1, y);
#pragma unroll
                    for (int s = 0; s < S; ++s) inc[s][v] = y[s];
                }
                publish<S, VEC, CW>(rec + (SS + S) * CW, inc, epoch * 4u + kFlagIncl, col, active);
            }
            if (active) {
#pragma unroll
                for (int s = 0; s < S; ++s)
#pragma unroll
                    for (int v = 0; v < VEC; ++v) s_carry[s][col + v] = carry[s][v];
            }
        }
        if constexpr (STAGE) lds_barrier_keep_vmem();
        else __syncthreads();

        // ---- back-substitution: lam for every step, then du and the
        // parameter-gradient contributions
        float acc[VEC][PRX];
#pragma unroll
        for (int v = 0; v < VEC; ++v)
#pragma unroll
            for (int r = 0; r < PRX; ++r) acc[v][r] = 0.0f;
        float duv[C][G][VEC];
        float nu0[S][VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            float cin[S], nin[S];
#pragma unroll
            for (int s = 0; s < S; ++s) cin[s] = s_carry[s][col + v];
            affine<S>(exA[v], cin, exB[v], nin);      // nu entering this wave from the right
            if constexpr (LL > 1) affine<S>(lexA[v], nin, lexB[v], nin);   // ... entering this chunk
#pragma unroll
            for (int i = 0; i < C; ++i) {
                float lam[S], d1[G];
                affine<S>(PX[i][v], nin, qx[i][v], lam);
                if constexpr (kRaw) {
#pragma unroll
                    for (int s = 0; s < S; ++s) d1[s] = lam[s];
                } else {
                    if (l0 + i < g.L) Cell::bwd_emit(kk[i][v], lam, d1, acc[v]);
                }
#pragma unroll
                for (int q = 0; q < G; ++q) duv[i][q][v] = d1[q];
            }
            // nu at the chunk's first step (dL/dh0 when that step is l = 0)
            float n0[S];
            affine<S>(cA[v], nin, cB[v], n0);
#pragma unroll
            for (int s = 0; s < S; ++s) nu0[s][v] = n0[s];
        }
        if (STAGE && full_tile && a.stream) {
#pragma unroll
            for (int i = 0; i < C; ++i)
#pragma unroll
                for (int q = 0; q < G; ++q)
                    buf_store<UT, VEC, kAuxStream>(rdu, vu, (unsigned int)(i * G + q) * Hn * (unsigned int)sizeof(UT), duv[i][q]);
        } else if (full_tile) {
#pragma unroll
            for (int i = 0; i < C; ++i)
#pragma unroll
                for (int q = 0; q < G; ++q)
                    buf_store<UT, VEC>(rdu, vu, (unsigned int)(i * G + q) * Hn * (unsigned int)sizeof(UT), duv[i][q]);
        } else {
#pragma unroll
            for (int i = 0; i < C; ++i) {
                const int l = l0 + i;
                if (ch_ok && l < g.L) {
#pragma unroll
                    for (int q = 0; q < G; ++q) store_vec<VEC>(du + ((seq + l) * G + q) * g.H + ch, duv[i][q]);
                }
            }
        }
        if (a.dh0 && ch_ok && l0 == 0) {
#pragma unroll
            for (int s = 0; s < S; ++s)
                store_vec<VEC>(static_cast<UT *>(a.dh0) + ((size_t)b * S + s) * g.H + ch, nu0[s]);
        }
        if constexpr (PR > 0) {
            // sum the accumulators over the segments of the wave, then over the waves
            if constexpr (LL > 1) {
#pragma unroll
                for (int d = LL / 2; d >= 1; d >>= 1)
#pragma unroll
                    for (int v = 0; v < VEC; ++v)
#pragma unroll
                        for (int r = 0; r < PR; ++r) acc[v][r] += __shfl_down(acc[v][r], d * LPS, 64);
            }
            if (seg == 0) {
#pragma unroll
                for (int v = 0; v < VEC; ++v)
#pragma unroll
                    for (int r = 0; r < PR; ++r) s_buf[w][r][col + v] = acc[v][r];
            }
            if constexpr (STAGE) lds_barrier_keep_vmem();
            else __syncthreads();
            for (int idx = threadIdx.x; idx < PR * CW; idx += kWave * W) {
                const int r = idx / CW, c = idx - r * CW;
                float s = 0.0f;
#pragma unroll
                for (int j = 0; j < W; ++j) s += s_buf[j][r][c];
                const int chn = cg * CW + c;
                if (chn < g.H) a.part[(((size_t)lt * g.B + b) * PR + r) * g.H + chn] = s;
            }
        }
        if constexpr (STAGE) {
            t = t_next;
            t_next = t_after;
            cur_staged = next_staged;
        }
    }
    if (internal_error && lane == 0) atomicExch(&ctrl->status, kStInternal);
}

}  // namespace pararnn
