/*
 * pararnn_nonlin.h - the diagonal GRU with selectable nonlinearities.
 *
 * The paper's GRU cell takes its three nonlinearities as parameters of the cell
 * (App. D.3: update, reset and state nonlinearity; sigmoid, sigmoid, tanh by
 * default).  Here they are template arguments: GruDiagNl<NU, NR, NS> is Eq. (7a)
 * with diagonal recurrent weights (Eq. (9))
 *
 *     z = NU(a_z h + u_z + b_z),  r = NR(a_r h + u_r + b_r),
 *     c = NS(a_c (r h) + u_c + b_c),  h' = (1 - z) h + z c,
 *
 * written to the cell contract of pararnn_cell.h, so that
 *
 *     using Cell = pararnn::GruDiagNl<pararnn::NlSigmoid, pararnn::NlSigmoid, pararnn::NlSoftsign>;
 *     PARARNN_DEFINE_CELL(Cell, gru_softsign)
 *
 * is a complete library for that variant.  Parameters [2][3][H]: a_z, a_r, a_c,
 * then b_z, b_r, b_c (the layout of the built-in GRU).
 *
 * A nonlinearity is a struct with f(x) and d(x, y) = f'(x), where y = f(x) is
 * passed along so that derivatives which are cheaper from the output can use it.
 */
#ifndef PARARNN_NONLIN_H
#define PARARNN_NONLIN_H

#include "pararnn/common.h"

namespace pararnn {

struct NlSigmoid {
    __device__ __forceinline__ static float f(float x) { return fast_sigmoid(x); }
    __device__ __forceinline__ static float d(float, float y) { return y * (1.0f - y); }
};
struct NlTanh {
    __device__ __forceinline__ static float f(float x) { return fast_tanh(x); }
    __device__ __forceinline__ static float d(float, float y) { return fmaf(-y, y, 1.0f); }
};
struct NlIdentity {
    __device__ __forceinline__ static float f(float x) { return x; }
    __device__ __forceinline__ static float d(float, float) { return 1.0f; }
};
// x / (1 + |x|); derivative 1 / (1 + |x|)^2 = (1 - |y|)^2
struct NlSoftsign {
    __device__ __forceinline__ static float f(float x) { return x * __builtin_amdgcn_rcpf(1.0f + fabsf(x)); }
    __device__ __forceinline__ static float d(float, float y)
    {
        const float t = 1.0f - fabsf(y);
        return t * t;
    }
};

// Jacobian, Eq. (8a) with general nonlinearities:
//   k_z = (c - h) NU'(.), k_c = z NS'(.), k_r = k_c a_c h NR'(.)   (dF/du_z, dF/du_c, dF/du_r)
//   J   = (1 - z) + a_z k_z + a_c r k_c + a_r k_r
template <class NU, class NR, class NS> struct GruDiagNl {
    static constexpr int G = 3, S = 1, P = 6, NC = 5;

    __device__ __forceinline__ static void step(const float *p, const float *hp, const float *u, float *F)
    {
        const float h = hp[0];
        const float z = NU::f(fmaf(p[0], h, u[0] + p[3]));
        const float r = NR::f(fmaf(p[1], h, u[1] + p[4]));
        const float c = NS::f(fmaf(p[2], r * h, u[2] + p[5]));
        F[0] = fmaf(z, c - h, h);
    }

    __device__ __forceinline__ static void coefs(const float *p, float h, const float *u, float &F, float &J,
                                                 float &kz, float &kr, float &kc, float &rh)
    {
        const float xz = fmaf(p[0], h, u[0] + p[3]), xr = fmaf(p[1], h, u[1] + p[4]);
        const float z = NU::f(xz), r = NR::f(xr);
        rh = r * h;
        const float xc = fmaf(p[2], rh, u[2] + p[5]);
        const float c = NS::f(xc);
        const float cmh = c - h;
        F = fmaf(z, cmh, h);
        kz = cmh * NU::d(xz, z);
        kc = z * NS::d(xc, c);
        const float ackc = p[2] * kc;
        kr = ackc * (h * NR::d(xr, r));
        J = fmaf(p[0], kz, 1.0f - z);
        J = fmaf(ackc, r, J);
        J = fmaf(p[1], kr, J);
    }

    __device__ __forceinline__ static void step_and_jacobian(const float *p, const float *hp, const float *u,
                                                             float *F, float *J)
    {
        float kz, kr, kc, rh;
        coefs(p, hp[0], u, F[0], J[0], kz, kr, kc, rh);
    }

    // k = (k_z, k_r, k_c, h, r h): the last two are d(pre-activation)/d(a_*)
    __device__ __forceinline__ static void bwd_prep(const float *p, const float *hp, const float *u, float *J,
                                                    float *k)
    {
        float F;
        coefs(p, hp[0], u, F, J[0], k[0], k[1], k[2], k[4]);
        k[3] = hp[0];
    }

    __device__ __forceinline__ static void bwd_emit(const float *k, const float *lam, float *du, float *acc)
    {
        du[0] = lam[0] * k[0];
        du[1] = lam[0] * k[1];
        du[2] = lam[0] * k[2];
        acc[0] = fmaf(du[0], k[3], acc[0]);
        acc[1] = fmaf(du[1], k[3], acc[1]);
        acc[2] = fmaf(du[2], k[4], acc[2]);
        acc[3] += du[0];
        acc[4] += du[1];
        acc[5] += du[2];
    }
};

}  // namespace pararnn

#endif /* PARARNN_NONLIN_H */
