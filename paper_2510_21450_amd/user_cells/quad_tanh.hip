// The 3x3 example cell (tri_tanh.hip) with four state values per channel, i.e. 4x4 Jacobian
// blocks, the largest block size the cell header offers:
//
//     x'_a = tanh(sum_b m_ab x_b + u_a),   a, b = 0..3
//
// every channel has its own 4x4 matrix m.  params [16][H]: rows m_00, m_01, m_02, m_03, m_10, ...
// Exports quad_tanh_forward / quad_tanh_backward / ...
#include "pararnn_cell.h"

struct QuadTanh {
    static constexpr int N = 4;
    static constexpr int G = N, S = N, P = N * N, NC = 2 * N;

    __device__ __forceinline__ static void step(const float *p, const float *hp, const float *u, float *F)
    {
#pragma unroll
        for (int a = 0; a < N; ++a) {
            float s = u[a];
#pragma unroll
            for (int b = 0; b < N; ++b) s = fmaf(p[N * a + b], hp[b], s);
            F[a] = pararnn::fast_tanh(s);
        }
    }

    // J[N a + b] = (1 - x'_a^2) m_ab
    __device__ __forceinline__ static void step_and_jacobian(const float *p, const float *hp, const float *u,
                                                             float *F, float *J)
    {
        step(p, hp, u, F);
#pragma unroll
        for (int a = 0; a < N; ++a) {
            const float d = fmaf(-F[a], F[a], 1.0f);
#pragma unroll
            for (int b = 0; b < N; ++b) J[N * a + b] = d * p[N * a + b];
        }
    }

    // k = (1 - x'_a^2 for a = 0..3, then x_0 .. x_3)
    __device__ __forceinline__ static void bwd_prep(const float *p, const float *hp, const float *u, float *J,
                                                    float *k)
    {
        float F[N];
        step_and_jacobian(p, hp, u, F, J);
#pragma unroll
        for (int a = 0; a < N; ++a) {
            k[a] = fmaf(-F[a], F[a], 1.0f);
            k[N + a] = hp[a];
        }
    }

    // du_a = lam_a (1 - x'_a^2);  dL/dm_ab += du_a x_b
    __device__ __forceinline__ static void bwd_emit(const float *k, const float *lam, float *du, float *acc)
    {
#pragma unroll
        for (int a = 0; a < N; ++a) {
            du[a] = lam[a] * k[a];
#pragma unroll
            for (int b = 0; b < N; ++b) acc[N * a + b] = fmaf(du[a], k[N + b], acc[N * a + b]);
        }
    }
};

PARARNN_DEFINE_CELL(QuadTanh, quad_tanh)
