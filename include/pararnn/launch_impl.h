// Definitions of Kernels<Cell, UT>; included only by the inst_*.hip files.
#pragma once
#include "launch.h"

namespace pararnn {

// workgroups of a persistent launch: what fits on the device at once
template <typename K> static int persistent_grid(K kernel, int threads, int n_tiles)
{
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, 0) != hipSuccess || per_cu < 1)
        per_cu = 1;
    const long long cap = (long long)per_cu * device_cu_count();
    return (int)(n_tiles < cap ? n_tiles : cap);
}

// Tile shapes instantiated for a cell.  Blocks of 3x3 and larger keep S*S + S prefix values per
// step in registers: beyond eight (3x3) or four (4x4) steps per thread and one channel per lane the
// kernels spill by the hundred, so those shapes are not built (the launch reports UNSUPPORTED).
template <class Cell, int VEC, int C> constexpr bool shape_offered()
{
    return Cell::S <= 2 || (VEC == 1 && C <= (Cell::S == 3 ? 8 : 4));
}

// static LDS of the forward kernels must stay within 64 KiB
template <class Cell, int VEC, int LL, int W> constexpr bool forward_fits_lds()
{
    constexpr int S = Cell::S, SS = S * S;
    return (size_t)(W * (SS + S) + 4 * S) * (kWave / LL) * VEC * sizeof(float) + 4 * W + 64 <= 65536;
}

// static LDS of the backward kernel must stay within 64 KiB
template <class Cell, int VEC, int LL, int W> constexpr bool backward_fits_lds()
{
    constexpr int S = Cell::S, SS = S * S, PRX = Cell::PR > 0 ? Cell::PR : 1;
    constexpr int rows = (SS + S) > PRX ? (SS + S) : PRX;
    return (size_t)(W * rows + S) * (kWave / LL) * VEC * sizeof(float) + 16 <= 65536;
}

template <class Cell, typename UT>
hipError_t Kernels<Cell, UT>::init_guess(int vec, const FwdArgs &a, hipStream_t st)
{
    if constexpr (IsRaw<Cell>::value) {
        return hipErrorInvalidValue;
    } else {
        const size_t n = (size_t)a.g.B * a.g.L * (a.g.H / vec);
        size_t blocks = (n + 255) / 256;
        const size_t cap = (size_t)device_cu_count() * 32;
        if (blocks > cap) blocks = cap;
#define PARARNN_CASE(V)                                                                       \
    if (vec == V) {                                                                           \
        hipLaunchKernelGGL((init_guess_kernel<Cell, V, UT>), dim3((unsigned)blocks), dim3(256), 0, st, a); \
        return hipGetLastError();                                                             \
    }
        PARARNN_VECS(PARARNN_CASE)
#undef PARARNN_CASE
        return hipErrorInvalidValue;
    }
}

template <class Cell, typename UT>
hipError_t Kernels<Cell, UT>::residual_norm(int vec, const ResArgs &a, hipStream_t st)
{
    if constexpr (IsRaw<Cell>::value) {
        return hipErrorInvalidValue;
    } else {
        const size_t n = (size_t)a.B * ((a.L + kResRun - 1) / kResRun) * (a.H / vec);
        size_t blocks = (n + 255) / 256;
        const size_t cap = (size_t)device_cu_count() * 8;
        if (blocks > cap) blocks = cap;
#define PARARNN_CASE(V)                                                                       \
    if (vec == V) {                                                                           \
        hipLaunchKernelGGL((residual_norm_kernel<Cell, V, UT>), dim3((unsigned)blocks), dim3(256), 0, st, a); \
        return hipGetLastError();                                                             \
    }
        PARARNN_VECS(PARARNN_CASE)
#undef PARARNN_CASE
        return hipErrorInvalidValue;
    }
}

template <class Cell, typename UT>
hipError_t Kernels<Cell, UT>::newton_iter(const TileCfg &cfg, const FwdArgs &a, bool fold_guess, hipStream_t st)
{
#define PARARNN_CASE(V, LLv, C, W)                                                             \
    if (cfg.vec == V && cfg.ll == LLv && cfg.c == C && cfg.w == W) {                           \
        if constexpr (shape_offered<Cell, V, C>() && forward_fits_lds<Cell, V, LLv, W>()) {    \
            static int grid_cap[2] = {0, 0}; /* per instantiation */                           \
            constexpr bool kFoldGuess = !IsRaw<Cell>::value;                                   \
            const int first = (kFoldGuess && fold_guess) ? 1 : 0;                              \
            auto kern = newton_iter_kernel<Cell, V, LLv, C, W, UT, false>;                     \
            if constexpr (kFoldGuess) {                                                        \
                if (first) kern = newton_iter_kernel<Cell, V, LLv, C, W, UT, true>;            \
            }                                                                                  \
            if (grid_cap[first] == 0) grid_cap[first] = persistent_grid(kern, kWave * W, 1 << 30); \
            const int grid = a.g.n_tiles < grid_cap[first] ? a.g.n_tiles : grid_cap[first];    \
            hipLaunchKernelGGL(kern, dim3(grid), dim3(kWave * W), 0, st, a);                   \
            return hipGetLastError();                                                          \
        } else {                                                                               \
            return hipErrorInvalidValue;                                                       \
        }                                                                                      \
    }
    PARARNN_SHAPES(PARARNN_CASE)
#undef PARARNN_CASE
    return hipErrorInvalidValue;
}

template <class Cell, typename UT>
hipError_t Kernels<Cell, UT>::newton_fused(const TileCfg &cfg, const FusedArgs &a, hipStream_t st)
{
    if constexpr (IsRaw<Cell>::value) {
        return hipErrorInvalidValue;
    } else {
#define PARARNN_CASE(V, LLv, C, W)                                                             \
    if (cfg.vec == V && cfg.ll == LLv && cfg.c == C && cfg.w == W) {                           \
        if constexpr (shape_offered<Cell, V, C>()) {                                           \
            static int grid_cap[2] = {0, 0};                                                   \
            const int tl = a.tail ? 1 : 0;                                                     \
            auto kern = a.tail ? newton_fused_kernel<Cell, V, LLv, C, W, UT, true>             \
                               : newton_fused_kernel<Cell, V, LLv, C, W, UT, false>;           \
            if (grid_cap[tl] == 0) grid_cap[tl] = persistent_grid(kern, kWave * W, 1 << 30);   \
            const int grid = a.g.n_tiles < grid_cap[tl] ? a.g.n_tiles : grid_cap[tl];          \
            hipLaunchKernelGGL(kern, dim3(grid), dim3(kWave * W), 0, st, a);                   \
            return hipGetLastError();                                                          \
        } else {                                                                               \
            return hipErrorInvalidValue;                                                       \
        }                                                                                      \
    }
        PARARNN_SHAPES(PARARNN_CASE)
#undef PARARNN_CASE
        return hipErrorInvalidValue;
    }
}

// The LDS-staged variant of the backward kernel exists for bf16 storage, one channel per lane, one
// segment per wave and steps per thread in multiples of 8 (one copy instruction moves 8 rows).
template <class Cell, int VEC, int LL, int C, typename UT> constexpr bool backward_stage_offered()
{
    return !IsRaw<Cell>::value && sizeof(UT) == 2 && VEC == 1 && LL == 1 && C % 8 == 0;
}

// static LDS of the staged backward kernel: its staging rows on top of the plain kernel's
template <class Cell, int C, int W> constexpr bool backward_stage_fits_lds()
{
    constexpr int S = Cell::S, SS = S * S, PRX = Cell::PR > 0 ? Cell::PR : 1;
    constexpr int rows = (SS + S) > PRX ? (SS + S) : PRX;
    return (size_t)(W * rows + S) * kWave * sizeof(float) + (size_t)W * C * (Cell::G + 2 * S) * 128 + 64 <= 65536;
}

template <class Cell, typename UT>
hipError_t Kernels<Cell, UT>::backward(const TileCfg &cfg, const BwdArgs &a, hipStream_t st)
{
#define PARARNN_CASE(V, LLv, C, W)                                                             \
    if (cfg.vec == V && cfg.ll == LLv && cfg.c == C && cfg.w == W) {                           \
        if constexpr (shape_offered<Cell, V, C>() && backward_fits_lds<Cell, V, LLv, W>()) {   \
            static int grid_cap[2] = {0, 0};                                                   \
            auto kern = backward_kernel<Cell, V, LLv, C, W, UT, false>;                        \
            int staged = 0;                                                                    \
            if constexpr (backward_stage_offered<Cell, V, LLv, C, UT>()) {                     \
                if constexpr (backward_stage_fits_lds<Cell, C, W>()) {                         \
                    if (a.stage) {                                                             \
                        kern = backward_kernel<Cell, V, LLv, C, W, UT, true>;                  \
                        staged = 1;                                                            \
                    }                                                                          \
                }                                                                              \
            }                                                                                  \
            if (grid_cap[staged] == 0) grid_cap[staged] = persistent_grid(kern, kWave * W, 1 << 30); \
            const int grid = a.g.n_tiles < grid_cap[staged] ? a.g.n_tiles : grid_cap[staged];  \
            hipLaunchKernelGGL(kern, dim3(grid), dim3(kWave * W), 0, st, a);                   \
            return hipGetLastError();                                                          \
        } else {                                                                               \
            return hipErrorInvalidValue;                                                       \
        }                                                                                      \
    }
    PARARNN_SHAPES(PARARNN_CASE)
#undef PARARNN_CASE
    return hipErrorInvalidValue;
}

}  // namespace pararnn
