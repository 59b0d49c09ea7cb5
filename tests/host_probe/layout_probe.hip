// Host-only probe of the workspace layout the driver computes (include/pararnn/driver.h):
// prints, for one problem and one tile shape, the byte ranges of the workspace regions and the
// largest index each kernel-side formula can produce, so that a CPU test can check that every
// access stays inside its region.  The index expressions below restate the kernels' own
// (scan_kernels.h / fused_kernels.h: record words, boundary rows, iterate, gradient partials and
// the 32-bit byte offsets of the buffer instructions) at their extreme arguments.  No device call.
#include <stdio.h>
#include <stdlib.h>

#include "pararnn/driver.h"

using namespace pararnn;

int main(int argc, char **argv)
{
    if (argc != 14) {
        fprintf(stderr, "usage: G S PR dtype B L H backward vec ll c w slots\n");
        return 2;
    }
    int v[13];
    for (int i = 0; i < 13; ++i) v[i] = atoi(argv[i + 1]);
    const CellInfo ci = {v[0], v[1], v[2], -1};
    const int dtype = v[3], B = v[4], L = v[5], H = v[6];
    const bool backward = v[7] != 0;
    const TileCfg cfg = {v[8], v[9], v[10], v[11]};
    const int slots = v[12];
    const Layout lo = make_layout(ci, dtype, B, L, H, backward, 4, slots > 1, slots, &cfg);
    const ScanGeom &g = lo.g;
    const size_t S = ci.S, G = ci.G, SS = S * S, NW = SS + 2 * S;
    const size_t CW = (size_t)(64 / cfg.ll) * cfg.vec, T = (size_t)cfg.c * cfg.ll * cfg.w;
    const size_t esz = dtype == PARARNN_BF16 ? 2 : 4;
    // largest record word index: last slot, last group, last tile, last word row, last column
    const size_t rec_max = (size_t)(slots - 1) * lo.n_rec + ((size_t)(g.n_groups - 1) * g.n_lt + (g.n_lt - 1)) * (NW * CW) +
                           (NW - 1) * CW + (CW - 1);
    // boundary rows [2][n_lt][B][S][H], largest index
    const size_t bnd_max = ((((size_t)1 * g.n_lt + (g.n_lt - 1)) * B + (B - 1)) * S + (S - 1)) * H + (H - 1);
    const size_t iter_max = (size_t)B * L * S * H - 1;
    const size_t part_max = (((size_t)(g.n_lt - 1) * B + (B - 1)) * ci.PR + (ci.PR > 0 ? ci.PR - 1 : 0)) * H + (H - 1);
    // 32-bit byte offsets of an interior tile's buffer accesses from the wave's base: lane part + row part
    const double voff_u = ((double)(cfg.ll - 1) * cfg.c * G * H + (CW - 1)) * esz;
    const double soff_u = ((double)(cfg.c - 1) * G + (G - 1)) * H * esz;
    const double voff_h = ((double)(cfg.ll - 1) * cfg.c * S * H + (CW - 1)) * 4.0;
    const double soff_h = ((double)(cfg.c - 1) * S + (S - 1)) * H * 4.0;
    printf("{\"total\": %zu, \"off_rec\": %zu, \"n_rec\": %zu, \"off_bnd\": %zu, \"off_iter\": %zu, \"off_part\": %zu, "
           "\"n_tiles\": %d, \"n_groups\": %d, \"n_lt\": %d, \"T\": %zu, \"CW\": %zu, \"rec_max\": %zu, \"bnd_max\": %zu, "
           "\"iter_max\": %zu, \"part_max\": %zu, \"off32_u\": %.0f, \"off32_h\": %.0f, \"tiles_exact\": %d}\n",
           lo.total, lo.off_rec, lo.n_rec, lo.off_bnd, lo.off_iter, lo.off_part, g.n_tiles, g.n_groups, g.n_lt, T, CW,
           rec_max, bnd_max, iter_max, part_max, voff_u + soff_u, voff_h + soff_h,
           (int)((long long)g.n_groups * g.n_lt == (long long)g.n_tiles));
    return 0;
}
