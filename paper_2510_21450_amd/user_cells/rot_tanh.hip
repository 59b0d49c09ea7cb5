// Example of a cell written from scratch against the four-function contract of
// pararnn_cell.h, with two state values per channel, i.e. a 2x2 Jacobian block
// (the block-diagonal structure of Sec. 2.1 / Eq. (8b), not tied to an LSTM):
//
//     p' = tanh(a p - b q + u_1),   q' = tanh(b p + a q + u_2)
//
// a per-channel rotation-scaling followed by tanh.  params [2][H] = (a, b).
// Exports rot_tanh_forward / rot_tanh_backward / ...
#include "pararnn_cell.h"

struct RotTanh {
    static constexpr int G = 2, S = 2, P = 2, NC = 4;

    __device__ __forceinline__ static void step(const float *p, const float *hp, const float *u, float *F)
    {
        F[0] = pararnn::fast_tanh(fmaf(p[0], hp[0], fmaf(-p[1], hp[1], u[0])));
        F[1] = pararnn::fast_tanh(fmaf(p[1], hp[0], fmaf(p[0], hp[1], u[1])));
    }

    __device__ __forceinline__ static void step_and_jacobian(const float *p, const float *hp, const float *u,
                                                             float *F, float *J)
    {
        step(p, hp, u, F);
        const float d0 = fmaf(-F[0], F[0], 1.0f), d1 = fmaf(-F[1], F[1], 1.0f);
        J[0] = d0 * p[0];
        J[1] = -d0 * p[1];
        J[2] = d1 * p[1];
        J[3] = d1 * p[0];
    }

    // k = (1 - p'^2, 1 - q'^2, p, q)
    __device__ __forceinline__ static void bwd_prep(const float *p, const float *hp, const float *u, float *J,
                                                    float *k)
    {
        float F[2];
        step_and_jacobian(p, hp, u, F, J);
        k[0] = fmaf(-F[0], F[0], 1.0f);
        k[1] = fmaf(-F[1], F[1], 1.0f);
        k[2] = hp[0];
        k[3] = hp[1];
    }

    __device__ __forceinline__ static void bwd_emit(const float *k, const float *lam, float *du, float *acc)
    {
        du[0] = lam[0] * k[0];
        du[1] = lam[1] * k[1];
        acc[0] += fmaf(du[0], k[2], du[1] * k[3]);
        acc[1] += fmaf(du[1], k[2], -du[0] * k[3]);
    }
};

PARARNN_DEFINE_CELL(RotTanh, rot_tanh)
