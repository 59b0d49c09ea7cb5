// K Newton iterations in one launch (the paper's "fully fused" mode, Sec. 4
// item 3 and App. D.3, where N_its is fixed and there is no stopping test): u
// is read once, the K iterations run on registers, h is written once.  Traffic
// per timestep-channel drops from K * (u + 2 h) to u + h.
//
// Two uses.  A fixed-count solve (tol < 0) runs entirely here.  A solve to a
// tolerance is a sequence of such blocks of K iterations: the maximum of |delta|
// is kept per iteration, the last workgroup reports the first iteration that
// met the tolerance, and the returned state is the iterate at the end of the
// block, i.e. the converged one refined by the iterations that were already in
// flight.  The first block starts from the initial guess (k0 = 0); a later one
// (k0 > 0) starts from the fp32 iterate and the tile-boundary rows its
// predecessor left behind, exactly as the per-iteration kernel does, and may be
// mixed with launches of that kernel.  With `tail` set one launch runs ALL the
// blocks that are left of a solve (sizes 1, 2, 4, ... as next_block_size gives
// them), separated by grid-wide barriers: after a block every workgroup learns
// from the control block whether the solve has ended, and a solve that met the
// tolerance early costs one such launch instead of a dozen that return at once.  The grid of such a launch is what the device holds at once
// (as for every launch of this kernel), so every barrier is reached by all.
//
// Same tile decomposition and the same look-back as newton_iter_kernel, with one
// carry-record slot per iteration: tile t at iteration k waits only for tile
// t-1 at iteration k, and tile t-1 never waits for tile t, so a tile may run
// ahead by any number of iterations and every wait ends.
//
// The state that enters a chunk, h_{l0-1}, belongs to another lane; it is kept
// up to date without any exchange because the delta that enters the chunk IS the
// update of that state: h^k_{l0-1} = h^{k-1}_{l0-1} + delta^k_{l0-1}.
#pragma once
#include "scan_kernels.h"

namespace pararnn {

constexpr int kMaxFused = 8;    // iterations one fused launch may run

struct FusedArgs {
    ScanGeom g;
    const float *params;
    const void *u;
    const void *h0;
    void *h;                 // out [B][L][S][H] in storage type
    unsigned long long *rec; // [n_iters][n_groups][n_lt][NW][CW]
    size_t rec_stride;       // words per iteration
    unsigned int *gmaxk;     // [kMaxFused] max |delta| bits per iteration (zeroed by the reset kernel)
    Ctrl *ctrl;
    int *iters_out;
    float *trace;
    int n_iters;
    // block of a solve to a tolerance (head != 0)
    int head;
    int k0;                  // iterations performed before this launch
    unsigned int epoch0;     // g.epoch_base + k0: the record tags' epoch of iteration k of this launch is epoch0 + k
    int max_iter;            // of the whole solve
    float tol;
    float *hit;              // fp32 iterate, read when k0 > 0 and written when more launches may follow;
                             // the output h itself for fp32 storage
    float *bnd;              // [2][n_lt][B][S][H] tile-boundary rows, see FwdArgs
    int bnd_cur;             // buffer read (k0 > 0); the other one is written
    // tail != 0: after this block the following ones of the plan, in the same launch
    int tail;
    int launch_no;           // position of this block in the plan (0 = the first launch of the solve)
    int n_slots;             // carry-record slots = largest block
    unsigned int spin_limit; // polls of a grid-wide barrier before it gives up
};

// Iterations of the next block of a solve: `done` of max_iter are behind it, `n_fused` carry-record
// slots are available (0: every block is one iteration).  The first block takes n_fused, the
// following ones 1, 2, 4, ... capped by n_fused and by what is left.
__host__ __device__ inline int next_block_size(int done, int launches, int max_iter, int n_fused)
{
    int K = 1;
    if (n_fused > 0) {
        if (launches == 0) K = n_fused;
        else K = launches - 1 < 30 ? 1 << (launches - 1) : n_fused;
        if (K > n_fused) K = n_fused;
    }
    if (K > max_iter - done) K = max_iter - done;
    return K;
}

// All workgroups of the launch meet here; false when the wait ran out (some workgroup never
// arrived: the launch then ends with status INTERNAL instead of hanging).  `arrivals` counts up over
// the launch, `generation` is the caller's count of barriers passed.
__device__ __forceinline__ bool fused_grid_barrier(unsigned int *arrivals, unsigned int &generation, unsigned int spin_limit)
{
    __shared__ int s_ok;
    __syncthreads();
    ++generation;                                     // by every thread: the count stays a scalar
    if (threadIdx.x == 0) {
        __threadfence();                              // this workgroup's writes, before it arrives
        const unsigned int target = generation * gridDim.x;
        atomicAdd(arrivals, 1u);
        unsigned int spins = 0;
        int ok = 1;
        while (__hip_atomic_load(arrivals, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            if (++spins >= spin_limit) { ok = 0; break; }
            __builtin_amdgcn_s_sleep(16);
        }
        __threadfence();                              // the others' writes, after all have arrived
        s_ok = ok;
    }
    __syncthreads();
    // as a scalar: a branch on a per-lane value would make the caller's loop variables per-lane values too
    return __builtin_amdgcn_readfirstlane(s_ok) != 0;
}

// S rows of CW record words (8 bytes each, consecutive columns) from memory straight into LDS, 16
// bytes per lane, past the L2 like every record access (sc1), issued from an asm statement so that
// the compiler neither tracks nor waits for it: the caller waits (s_waitcnt vmcnt) before it reads
// dst.  A record word lies inside one aligned 16-byte piece, which the memory system serves in one
// access, so a word is still seen whole.  M0 holds the LDS address; the wait states are the ones a
// vector-memory instruction needs after its scalar operands were written.
template <int S, int CW>
__device__ __forceinline__ void early_look(rec_t (*dst)[CW], const rec_t *src, int lane)
{
    typedef unsigned int u4 __attribute__((ext_vector_type(4)));
    const unsigned long long p = (unsigned long long)src;
    const u4 rsrc = {(unsigned int)__builtin_amdgcn_readfirstlane((unsigned int)p),
                     (unsigned int)__builtin_amdgcn_readfirstlane((unsigned int)(p >> 32)) & 0xffffu, 0xffffffffu, 0x27000u};
    const unsigned int lds = (unsigned int)(unsigned long long)(__attribute__((address_space(3))) const void *)&dst[0][0];
    if (lane < CW / 2) {
#pragma unroll
        for (int s = 0; s < S; ++s)
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 4\n\tbuffer_load_dwordx4 %1, %2, %3 offen sc1 lds"
                         ::"s"((unsigned int)__builtin_amdgcn_readfirstlane(lds + (unsigned int)(s * CW * 8))),
                         "v"((unsigned int)lane * 16u), "s"(rsrc), "s"((unsigned int)(s * CW * 8))
                         : "memory", "m0");
    }
}

// Waves per SIMD the register allocation must leave room for: four (128 registers) for scalar states with
// chunks of up to 12 steps and two (256) for 2 x 2 blocks, whose default shapes sit at those limits; no
// demand otherwise.
template <class Cell, int VEC, int C> constexpr int fused_min_waves()
{
    return Cell::S == 1 && VEC == 1 && C <= 12 ? 4 : (Cell::S == 2 && VEC == 1 ? 2 : 1);
}

// TAIL: the launch goes on with the following blocks of the plan (a.tail is set); a variant of its own
// because the block's size and position are then loop variables that stay in registers, where the
// one-block variant re-reads them from the kernel arguments, and the first block of the bf16 GRU
// sits one register short of losing a wave per SIMD
template <class Cell, int VEC, int LL, int C, int W, typename UT, bool TAIL = false>
__global__ __launch_bounds__(kWave *W) __attribute__((amdgpu_waves_per_eu(fused_min_waves<Cell, VEC, C>())))
void newton_fused_kernel(const FusedArgs a)
{
    constexpr int S = Cell::S, G = Cell::G, SS = S * S, PR = Cell::PR;
    constexpr int LPS = kWave / LL, CW = LPS * VEC, NW = SS + 2 * S, T = C * LL * W;
    __shared__ float s_A[W][SS][CW];
    __shared__ float s_b[W][S][CW];
    __shared__ float s_carry[S][CW];
    __shared__ float s_incl[S][CW];
    constexpr bool kEarly = CW <= 128;                 // a row of records fits one copy instruction (64 lanes x 16 bytes)
    __shared__ __attribute__((aligned(16))) rec_t s_pre[kEarly ? S : 1][kEarly ? CW : 2];
    __shared__ unsigned int s_maxk[kMaxFused];
    __shared__ unsigned int s_ticket;

    Ctrl *ctrl = a.ctrl;
    if (ctrl->stop) return;
    const ScanGeom &g = a.g;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int seg = lane / LPS, col = (lane % LPS) * VEC;
    const UT *u = static_cast<const UT *>(a.u);
    UT *hout = static_cast<UT *>(a.h);
    int K = a.n_iters, k0 = a.k0, bnd_cur = a.bnd_cur, launch_no = a.launch_no;
    unsigned int generation = 0;
    bool internal_error = false;

  for (;;) {                              // the blocks of this launch: one, or the rest of the plan (tail)
    const bool resume = k0 > 0;
    if (threadIdx.x < kMaxFused) s_maxk[threadIdx.x] = 0u;

    for (;;) {
        if (threadIdx.x == 0) s_ticket = atomicAdd(&ctrl->ticket, 1u);
        __syncthreads();
        const unsigned int t = __builtin_amdgcn_readfirstlane(s_ticket);
        if (t >= (unsigned int)g.n_tiles) break;
        const int grp = (int)(t % (unsigned int)g.n_groups), lt = (int)(t / (unsigned int)g.n_groups);
        const int b = grp / g.n_cg, cg = grp - b * g.n_cg;
        const int ch = cg * CW + col;
        const bool ch_ok = ch < g.H;
        const int l0 = lt * T + (w * LL + seg) * C;
        const size_t seq = (size_t)b * g.L;
        const int wl = lt * T + w * (LL * C);
        const unsigned int Hn = (unsigned int)g.H;
        const size_t row_w = seq + (size_t)wl;
        const buf_rsrc ru = make_rsrc(u + row_w * G * Hn + (size_t)cg * CW);
        const buf_rsrc rho = make_rsrc(hout + row_w * S * Hn + (size_t)cg * CW);
        const unsigned int vu = ((unsigned int)(seg * (C * G)) * Hn + col) * (unsigned int)sizeof(UT);
        const unsigned int vh = ((unsigned int)(seg * (C * S)) * Hn + col) * (unsigned int)sizeof(UT);
        const bool full_tile = (lt + 1) * T <= g.L && (cg + 1) * CW <= g.H;

        float p[VEC][PR];
#pragma unroll
        for (int r = 0; r < PR; ++r) {
            float tmp[VEC];
#pragma unroll
            for (int v = 0; v < VEC; ++v) tmp[v] = 0.0f;
            if (ch_ok) load_vec<VEC>(a.params + (size_t)r * g.H + ch, tmp);
#pragma unroll
            for (int v = 0; v < VEC; ++v) p[v][r] = tmp[v];
        }
        // weights scaled for the folded gate arithmetic (u is folded once below, then reused K times)
        float pq[VEC][Cell::PQ > 0 ? Cell::PQ : 1];
#pragma unroll
        for (int v = 0; v < VEC; ++v) Cell::fold_params(p[v], pq[v]);

        // ---- u for the C steps of this thread (kept for all iterations), the row before, h0
        using RawU = typename RawVec<UT, VEC>::type;
        RawU uur[C][G], uhalo[G];
        auto load_inputs = [&](auto guard) {
            constexpr bool kGuard = decltype(guard)::value;
#pragma unroll
            for (int i = 0; i < C; ++i) {
                const int l = l0 + i;
                const bool ok = !kGuard || (ch_ok && l < g.L);
#pragma unroll
                for (int q = 0; q < G; ++q) {
                    if constexpr (!kGuard) uur[i][q] = buf_load<UT, VEC>(ru, vu, (unsigned int)(i * G + q) * Hn * (unsigned int)sizeof(UT));
                    else if (ok) uur[i][q] = load_raw<UT, VEC>(u + ((seq + l) * G + q) * g.H + ch);
                    else uur[i][q] = zero_raw<UT, VEC>();
                }
            }
        };
        // a new tile's loads go out ahead of the arithmetic of the waves that share the SIMD
        __builtin_amdgcn_s_setprio(2);
        if (full_tile) load_inputs(std::false_type{});
        else load_inputs(std::true_type{});
#pragma unroll
        for (int q = 0; q < G; ++q) {
            uhalo[q] = zero_raw<UT, VEC>();
            if (ch_ok && l0 > 0 && l0 <= g.L) uhalo[q] = load_raw<UT, VEC>(u + ((seq + l0 - 1) * G + q) * Hn + ch);
        }
        float h0v[S][VEC], hprev[S][VEC];
#pragma unroll
        for (int s = 0; s < S; ++s) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) h0v[s][v] = 0.0f;
            if (ch_ok && a.h0) load_vec<VEC>(static_cast<const UT *>(a.h0) + ((size_t)b * S + s) * g.H + ch, h0v[s]);
        }

        // ---- initial guess h^0_l = f(h0, u_l) (App. A) for the own steps and for the row before the chunk;
        //      a resumed solve reads both from the iterate instead
        float uu[C][G][VEC], ho[C][S][VEC];
#pragma unroll
        for (int i = 0; i < C; ++i) {
#pragma unroll
            for (int q = 0; q < G; ++q) raw_to_float<UT, VEC>(uur[i][q], uu[i][q]);
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                float ug[G];
#pragma unroll
                for (int q = 0; q < G; ++q) ug[q] = uu[i][q][v];
                Cell::fold_u(p[v], ug);
#pragma unroll
                for (int q = 0; q < G; ++q) uu[i][q][v] = ug[q];
            }
            if (resume) {
#pragma unroll
                for (int s = 0; s < S; ++s) {
#pragma unroll
                    for (int v = 0; v < VEC; ++v) ho[i][s][v] = 0.0f;
                    if (ch_ok && l0 + i < g.L) load_vec<VEC>(a.hit + ((seq + l0 + i) * S + s) * g.H + ch, ho[i][s]);
                }
                continue;
            }
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                float h1[S], ug[G], F0[S];
#pragma unroll
                for (int s = 0; s < S; ++s) h1[s] = h0v[s][v];
#pragma unroll
                for (int q = 0; q < G; ++q) ug[q] = uu[i][q][v];
                Cell::template step<true>(p[v], h1, ug, F0, pq[v]);
#pragma unroll
                for (int s = 0; s < S; ++s) ho[i][s][v] = F0[s];
            }
        }
#pragma unroll
        for (int s = 0; s < S; ++s)
#pragma unroll
            for (int v = 0; v < VEC; ++v) hprev[s][v] = h0v[s][v];
        if (resume) {
            // the previous tile's boundary row, or the row just before the chunk (still the old
            // iterate: every store of this tile comes after the barriers below)
            if (ch_ok && l0 > 0 && l0 <= g.L) {
#pragma unroll
                for (int s = 0; s < S; ++s) {
                    if (w == 0 && seg == 0)
                        load_vec<VEC>(a.bnd + ((((size_t)bnd_cur * g.n_lt + (lt - 1)) * g.B + b) * S + s) * g.H + ch, hprev[s]);
                    else
                        load_vec<VEC>(a.hit + ((seq + l0 - 1) * S + s) * g.H + ch, hprev[s]);
                }
            }
        } else if (l0 > 0) {
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
                Cell::fold_u(p[v], ug);
                Cell::template step<true>(p[v], h1, ug, F0, pq[v]);
#pragma unroll
                for (int s = 0; s < S; ++s) hprev[s][v] = F0[s];
            }
        }

        // The K iterations.  Interior tiles run the thread-level pass and the back-substitution without
        // bounds tests (the C cell evaluations of a thread are independent, they read the previous iterate,
        // and without branches between them the compiler interleaves their dependency chains).  mode 0 / 1:
        // the whole iteration loop exists in both forms and the choice is made once per tile, which spares
        // the register shuffling where two forms meet inside the loop (6 % on the GRU); mode 2: one loop
        // that chooses inside each phase, for cells whose state no longer fits the registers twice over
        // (2x2 blocks and larger: the doubled loop costs them a wave per SIMD).
        __builtin_amdgcn_s_setprio(0);
        auto iterations = [&](auto mode) {
            constexpr int kMode = decltype(mode)::value;
            // nothing in flight when the loop starts (the inputs have been used by now, what remains are the
            // last tile's stores): inside the loop the only load a wave may wait for is then the early look
            // at the predecessor's record, and the thread-level pass runs while it travels
            __builtin_amdgcn_s_waitcnt(0x0F70);       // vmcnt(0) only
            // ---- the predecessor's inclusive value of an iteration is asked for one iteration ahead (the
            //      first one here) and looked at when the workgroup level needs it: a tile whose predecessor
            //      is that far ahead finds its carry waiting instead of paying a round trip to memory, about
            //      as long as the rest of an iteration, while its other waves wait.  The record rows travel
            //      straight into LDS (early_look): no register is their destination, so the compiled code
            //      has no wait for them; wave 0 waits where it reads them.
            const bool looks_back = kEarly && w == 0 && lt > 0;
            const rec_t *pre_src = a.rec + ((size_t)grp * g.n_lt + (lt > 0 ? lt - 1 : 0)) * (NW * CW) + (SS + S) * CW;
            if (looks_back) early_look<S, CW>(s_pre, pre_src, lane);
#pragma unroll 1
            for (int k = 1; k <= K; ++k) {
                // unique within the call; the one-block variant takes the sum of the constant part from the kernel
                // arguments (one more value that lives through the block costs it registers it does not have)
                const unsigned int epoch = TAIL ? g.epoch_base + (unsigned int)(k0 + k) : a.epoch0 + (unsigned int)k;
                unsigned long long *reck = a.rec + (size_t)(k - 1) * a.rec_stride;

                // ---- thread level
                float PA[C][VEC][SS], qb[C][VEC][S], accA[VEC][SS], accB[VEC][S];
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    set_identity<S>(accA[v]);
#pragma unroll
                    for (int s = 0; s < S; ++s) accB[v][s] = 0.0f;
                }
                auto thread_level = [&](auto gd) {
                    constexpr bool kG = decltype(gd)::value;
#pragma unroll
                    for (int i = 0; i < C; ++i) {
                        if (!kG || l0 + i < g.L) {
#pragma unroll
                            for (int v = 0; v < VEC; ++v) {
                                float J[SS], r[S], hp[S], ug[G], F[S];
#pragma unroll
                                for (int s = 0; s < S; ++s) hp[s] = i == 0 ? hprev[s][v] : ho[i - 1][s][v];
#pragma unroll
                                for (int q = 0; q < G; ++q) ug[q] = uu[i][q][v];
                                Cell::template fwd<true>(p[v], hp, ug, F, J, pq[v]);
#pragma unroll
                                for (int s = 0; s < S; ++s) r[s] = F[s] - ho[i][s][v];
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
                };
                if constexpr (kMode == 2) {
                    if (full_tile) thread_level(std::false_type{});
                    else thread_level(std::true_type{});
                } else {
                    thread_level(std::integral_constant<bool, kMode == 1>{});
                }

                // ---- wave level
                float lexA[VEC][SS], lexB[VEC][S];
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

                // ---- workgroup level
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
                if (w == 0) {
                    // seven waves wait at the next barrier for what this one does now: it goes first on its SIMD
                    __builtin_amdgcn_s_setprio(3);
                    // the early look is waited for here, by the only wave that has one in flight (and no
                    // stores of its own in flight unless it took the slow path below an iteration ago)
                    rec_t pre[S][VEC];
                    if constexpr (kEarly) {
                        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
                        for (int s = 0; s < S; ++s)
#pragma unroll
                            for (int v = 0; v < VEC; ++v) pre[s][v] = s_pre[s][col + v];
                    } else {
#pragma unroll
                        for (int s = 0; s < S; ++s)
#pragma unroll
                            for (int v = 0; v < VEC; ++v) pre[s][v] = 0;
                    }
                    // ---- workgroup level, by wave 0 alone: it walks the waves' aggregates once, leaving in
                    //      place of each the composition of the waves before it, and ends with the tile's
                    //      aggregate.  (Every wave used to compose its own prefix from the same values: W/2
                    //      steps per wave instead of W in all, on the vector ALUs that bound this kernel.)
                    float exA[VEC][SS], exB[VEC][S];
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        set_identity<S>(exA[v]);
#pragma unroll
                        for (int s = 0; s < S; ++s) exB[v][s] = 0.0f;
                    }
                    if constexpr (S == 1) {
                        // the aggregates in batches of JB LDS reads (one latency per batch instead of one per
                        // wave), composed in registers, the prefixes written back in one batch
                        constexpr int JB = W % 4 == 0 ? 4 : (W % 2 == 0 ? 2 : 1);
#pragma unroll
                        for (int j0 = 0; j0 < W; j0 += JB) {
                            float Aw[JB][VEC][SS], bw[JB][VEC][S];
#pragma unroll
                            for (int j = 0; j < JB; ++j)
#pragma unroll
                                for (int v = 0; v < VEC; ++v) {
#pragma unroll
                                    for (int e = 0; e < SS; ++e) Aw[j][v][e] = s_A[j0 + j][e][col + v];
#pragma unroll
                                    for (int s = 0; s < S; ++s) bw[j][v][s] = s_b[j0 + j][s][col + v];
                                }
#pragma unroll
                            for (int j = 0; j < JB; ++j)
#pragma unroll
                                for (int v = 0; v < VEC; ++v) {
                                    float Aj[SS], bj[S];
#pragma unroll
                                    for (int e = 0; e < SS; ++e) { Aj[e] = Aw[j][v][e]; Aw[j][v][e] = exA[v][e]; }
#pragma unroll
                                    for (int s = 0; s < S; ++s) { bj[s] = bw[j][v][s]; bw[j][v][s] = exB[v][s]; }
                                    push_step<S>(Aj, bj, exA[v], exB[v]);
                                }
#pragma unroll
                            for (int j = 0; j < JB; ++j)
#pragma unroll
                                for (int v = 0; v < VEC; ++v) {
#pragma unroll
                                    for (int e = 0; e < SS; ++e) s_A[j0 + j][e][col + v] = Aw[j][v][e];
#pragma unroll
                                    for (int s = 0; s < S; ++s) s_b[j0 + j][s][col + v] = bw[j][v][s];
                                }
                        }
                    } else {
#pragma unroll
                        for (int j = 0; j < W; ++j) {
#pragma unroll
                            for (int v = 0; v < VEC; ++v) {
                                float Aj[SS], bj[S];
#pragma unroll
                                for (int e = 0; e < SS; ++e) {
                                    Aj[e] = s_A[j][e][col + v];
                                    s_A[j][e][col + v] = exA[v][e];
                                }
#pragma unroll
                                for (int s = 0; s < S; ++s) {
                                    bj[s] = s_b[j][s][col + v];
                                    s_b[j][s][col + v] = exB[v][s];
                                }
                                push_step<S>(Aj, bj, exA[v], exB[v]);
                            }
                        }
                    }
                    // ---- grid level: look-back within this iteration's record slot
                    float tileA[SS][VEC], tileB[S][VEC], carry[S][VEC];
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
#pragma unroll
                        for (int e = 0; e < SS; ++e) tileA[e][v] = exA[v][e];
#pragma unroll
                        for (int s = 0; s < S; ++s) { tileB[s][v] = exB[v][s]; carry[s][v] = 0.0f; }
                    }
                    const bool active = seg == 0;
                    const bool has_next = lt + 1 < g.n_lt;
                    rec_t *rec = reck + ((size_t)grp * g.n_lt + lt) * (NW * CW);
                    bool early = lt > 0;
#pragma unroll
                    for (int s = 0; s < S; ++s)
#pragma unroll
                        for (int v = 0; v < VEC; ++v) {
                            early = early && (unsigned int)(pre[s][v] >> 32) == epoch * 4u + kFlagIncl;
                            carry[s][v] = __uint_as_float((unsigned int)pre[s][v]);
                        }
                    early = kEarly && __all(early || !active) && lt > 0;
                    if (!early) {                 // also the first tile of a chain: nothing enters it
#pragma unroll
                        for (int s = 0; s < S; ++s)
#pragma unroll
                            for (int v = 0; v < VEC; ++v) carry[s][v] = 0.0f;
                    }
                    if (looks_back && k < K) early_look<S, CW>(s_pre, pre_src + (size_t)k * a.rec_stride, lane);
                    if (lt > 0 && !early) {
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
                        if (!lookback<S, VEC, CW>(g.spin_limit, reck, g.n_lt, grp, lt, -1, epoch, col, active, carry))
                            internal_error = true;
                    }
                    // ---- the carry, for every wave to apply its own prefix to (it lives in the lanes of segment
                    //      0), and the tile's inclusive value in the form a look-back over this tile's aggregate
                    //      would give it (same bits whichever way a successor comes by it), for the last wave to
                    //      publish
                    if (active) {
#pragma unroll
                        for (int v = 0; v < VEC; ++v) {
                            float A1[SS], x[S], b1[S], y[S];
#pragma unroll
                            for (int e = 0; e < SS; ++e) A1[e] = tileA[e][v];
#pragma unroll
                            for (int s = 0; s < S; ++s) { x[s] = carry[s][v]; b1[s] = tileB[s][v]; }
                            affine<S>(A1, x, b1, y);
#pragma unroll
                            for (int s = 0; s < S; ++s) {
                                s_carry[s][col + v] = carry[s][v];
                                s_incl[s][col + v] = y[s];
                            }
                        }
                    }
                    __builtin_amdgcn_s_setprio(0);
                }
                __syncthreads();

                // ---- back-substitution; the delta entering the chunk also updates the state before it
                // ---- the tile's inclusive value leaves through the last wave, which never waits for a load
                //      inside the loop: the store's way to memory is then nobody's waiting time (wave 0 would
                //      meet it at its next wait for the early look)
                if (w == W - 1 && lt + 1 < g.n_lt) {
                    float inc[S][VEC];
#pragma unroll
                    for (int s = 0; s < S; ++s)
#pragma unroll
                        for (int v = 0; v < VEC; ++v) inc[s][v] = s_incl[s][col + v];
                    publish<S, VEC, CW>(reck + ((size_t)grp * g.n_lt + lt) * (NW * CW) + (SS + S) * CW, inc,
                                        epoch * 4u + kFlagIncl, col, seg == 0);
                }
                unsigned int wmax_bits = 0u;
                auto back_substitute = [&](auto gd) {
                    constexpr bool kG = decltype(gd)::value;
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        // the delta that enters this wave's first step: its prefix applied to the tile's carry
                        float din[S], cin[S], Aw[SS], bw[S];
#pragma unroll
                        for (int e = 0; e < SS; ++e) Aw[e] = s_A[w][e][col + v];
#pragma unroll
                        for (int s = 0; s < S; ++s) { bw[s] = s_b[w][s][col + v]; cin[s] = s_carry[s][col + v]; }
                        affine<S>(Aw, cin, bw, din);
                        if constexpr (LL > 1) affine<S>(lexA[v], din, lexB[v], din);
#pragma unroll
                        for (int s = 0; s < S; ++s) hprev[s][v] += din[s];
#pragma unroll
                        for (int i = 0; i < C; ++i) {
                            float d[S];
                            affine<S>(PA[i][v], din, qb[i][v], d);
#pragma unroll
                            for (int s = 0; s < S; ++s) {
                                ho[i][s][v] += d[s];
                                if (!kG || (ch_ok && l0 + i < g.L))
                                    wmax_bits = max(wmax_bits, __float_as_uint(d[s]) & 0x7fffffffu);
                            }
                        }
                    }
                };
                if constexpr (kMode == 2) {
                    if (full_tile) back_substitute(std::false_type{});
                    else back_substitute(std::true_type{});
                } else {
                    back_substitute(std::integral_constant<bool, kMode == 1>{});
                }
                const unsigned int wave_bits = wave_max_u32(wmax_bits);
                if (lane == 0) atomicMax(&s_maxk[k - 1], wave_bits);
                // a wave rewrites its own s_A / s_b entries before the next iteration's first barrier; wave 0 reads
                // them all after it
            }
        };
        if constexpr (S == 1) {
            if (full_tile) iterations(std::integral_constant<int, 0>{});
            else iterations(std::integral_constant<int, 1>{});
        } else {
            iterations(std::integral_constant<int, 2>{});
        }

        // from here to the first iteration of the workgroup's next tile (stores, ticket, loads, initial guess)
        // its waves go ahead of the other workgroup's iterations on the SIMDs they share
        __builtin_amdgcn_s_setprio(2);
        // ---- what a following per-iteration launch needs: the fp32 iterate and the tile's last row
        if (a.head && k0 + K < a.max_iter) {
            if (a.hit && static_cast<void *>(a.hit) != a.h) {
#pragma unroll
                for (int i = 0; i < C; ++i) {
                    const int l = l0 + i;
                    if (ch_ok && l < g.L) {
#pragma unroll
                        for (int s = 0; s < S; ++s) store_vec<VEC>(a.hit + ((seq + l) * S + s) * g.H + ch, ho[i][s]);
                    }
                }
            }
            if (ch_ok && w == W - 1 && seg == LL - 1 && lt + 1 < g.n_lt) {
                const int nxt = bnd_cur ^ 1;
#pragma unroll
                for (int s = 0; s < S; ++s)
                    store_vec<VEC>(a.bnd + ((((size_t)nxt * g.n_lt + lt) * g.B + b) * S + s) * g.H + ch, ho[C - 1][s]);
            }
        }

        // ---- the result, once
        if (full_tile) {
#pragma unroll
            for (int i = 0; i < C; ++i)
#pragma unroll
                for (int s = 0; s < S; ++s)
                    buf_store<UT, VEC>(rho, vh, (unsigned int)(i * S + s) * Hn * (unsigned int)sizeof(UT), ho[i][s]);
        } else {
#pragma unroll
            for (int i = 0; i < C; ++i) {
                const int l = l0 + i;
                if (ch_ok && l < g.L) {
#pragma unroll
                    for (int s = 0; s < S; ++s) store_vec<VEC>(hout + ((seq + l) * S + s) * g.H + ch, ho[i][s]);
                }
            }
        }
    }

    // ---- per-iteration maxima; the last workgroup writes the results
    if (internal_error && lane == 0) atomicExch(&ctrl->status, kStInternal);
    __syncthreads();
    if ((int)threadIdx.x < K) atomicMax(&a.gmaxk[threadIdx.x], s_maxk[threadIdx.x]);
    __syncthreads();
    if (threadIdx.x == 0) {
        __threadfence();
        const unsigned int prev = atomicAdd(&ctrl->done, 1u);
        if (prev == gridDim.x - 1) {
            __threadfence();
            const bool internal = atomicAdd(&ctrl->status, 0) == kStInternal;
            int status = internal ? kStInternal : (a.head ? kStNotConverged : kStOk);
            int iters = K, stop = (a.head && !internal) ? 0 : 1;
            bool ended = false;
            iters += k0;
            for (int k = 0; k < K; ++k) {
                const float mk = __uint_as_float(atomicExch(&a.gmaxk[k], 0u));   // zero again for the next block
                if (ended) continue;                  // iterations past the end are not reported
                if (a.trace) a.trace[k0 + k] = mk;
                if (internal) continue;
                if (!(mk - mk == 0.0f)) { status = kStNonFinite; iters = k0 + k + 1; stop = 1; ended = true; }
                else if (a.head && mk <= a.tol) { status = kStOk; iters = k0 + k + 1; stop = 1; ended = true; }
            }
            a.iters_out[0] = iters;
            a.iters_out[1] = status;
            ctrl->iters = iters;
            ctrl->status = status;
            ctrl->stop = stop;
            ctrl->h_final = (stop || k0 + K >= a.max_iter) ? 1 : 0;
            ctrl->ticket = 0u;
            ctrl->done = 0u;
            __threadfence();
        }
    }
    if constexpr (!TAIL) {
        break;
    } else {
    // ---- the next block of the plan, if the solve goes on
    if (!fused_grid_barrier(&ctrl->pad[0], generation, a.spin_limit)) {
        if (threadIdx.x == 0) {
            atomicExch(&ctrl->status, kStInternal);
            a.iters_out[1] = kStInternal;
            ctrl->stop = 1;
        }
        break;
    }
    if (__builtin_amdgcn_readfirstlane(__hip_atomic_load(&ctrl->stop, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) break;
    k0 += K;
    if (k0 >= a.max_iter) break;
    bnd_cur ^= 1;
    ++launch_no;
    K = next_block_size(k0, launch_no, a.max_iter, a.n_slots);
    }
  }
}

}  // namespace pararnn
