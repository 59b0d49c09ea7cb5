// Example of a cell with three state values per channel, i.e. 3x3 Jacobian blocks (the
// block-diagonal structure of Sec. 2.1 beyond the LSTM's 2x2), written against the
// four-function contract of pararnn_cell.h:
//
//     x'_a = tanh(sum_b m_ab x_b + u_a),   a, b = 0..2
//
// every channel has its own 3x3 matrix m.  params [9][H]: rows m_00, m_01, m_02, m_10, ...
// Exports tri_tanh_forward / tri_tanh_backward / ...
#include "pararnn_cell.h"

struct TriTanh {
    static constexpr int G = 3, S = 3, P = 9, NC = 6;

    __device__ __forceinline__ static void step(const float *p, const float *hp, const float *u, float *F)
    {
#pragma unroll
        for (int a = 0; a < 3; ++a)
            F[a] = pararnn::fast_tanh(fmaf(p[3 * a], hp[0], fmaf(p[3 * a + 1], hp[1], fmaf(p[3 * a + 2], hp[2], u[a]))));
    }

    // J[3 a + b] = (1 - x'_a^2) m_ab
    __device__ __forceinline__ static void step_and_jacobian(const float *p, const float *hp, const float *u,
                                                             float *F, float *J)
    {
        step(p, hp, u, F);
#pragma unroll
        for (int a = 0; a < 3; ++a) {
            const float d = fmaf(-F[a], F[a], 1.0f);
#pragma unroll
            for (int b = 0; b < 3; ++b) J[3 * a + b] = d * p[3 * a + b];
        }
    }

    // k = (1 - x'_0^2, 1 - x'_1^2, 1 - x'_2^2, x_0, x_1, x_2)
    __device__ __forceinline__ static void bwd_prep(const float *p, const float *hp, const float *u, float *J,
                                                    float *k)
    {
        float F[3];
        step_and_jacobian(p, hp, u, F, J);
#pragma unroll
        for (int a = 0; a < 3; ++a) {
            k[a] = fmaf(-F[a], F[a], 1.0f);
            k[3 + a] = hp[a];
        }
    }

    // du_a = lam_a (1 - x'_a^2);  dL/dm_ab += du_a x_b
    __device__ __forceinline__ static void bwd_emit(const float *k, const float *lam, float *du, float *acc)
    {
#pragma unroll
        for (int a = 0; a < 3; ++a) {
            du[a] = lam[a] * k[a];
#pragma unroll
            for (int b = 0; b < 3; ++b) acc[3 * a + b] = fmaf(du[a], k[3 + b], acc[3 * a + b]);
        }
    }
};

PARARNN_DEFINE_CELL(TriTanh, tri_tanh)
