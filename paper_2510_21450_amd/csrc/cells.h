// Per-channel cell arithmetic for the diagonal and 2x2-block paths.
//
// Every function works on ONE channel: p[] holds that channel's PR parameter
// rows ([2][G]: recurrent weights then biases), hp[] the previous state (S
// values), u[] the G pre-activations.  J is row-major S x S with
// J[p*S+q] = d(out_p)/d(in_q).
//
// step<true> / fwd<true> are the folded forms: u[] then holds fold_u()'s output
// (the gate inputs u + b scaled for the exp2-based nonlinearities) and q[] the
// PQ scaled weights from fold_params(); p[] is still needed for the Jacobian.
//
// Backward (Sec. 2, Eq. (6)): bwd_prep returns J and NC coefficients from which
// bwd_emit maps the incoming adjoint lam (dL/d state_l) to dL/du_l and adds this
// step's contribution to the PR parameter-gradient accumulators.
#pragma once
#include "pararnn/common.h"

namespace pararnn {

// Sec. 3, Eq. (7a) with the diagonal weights of Eq. (9); Jacobian Eq. (8a).
struct GruDiag {
    static constexpr int G = 3, S = 1, PR = 6, NC = 5, PQ = 3;

    __device__ __forceinline__ static void fold_params(const float *p, float *q)
    {
        q[0] = kSigFold * p[0]; q[1] = kSigFold * p[1]; q[2] = kTanhFold * p[2];
    }
    __device__ __forceinline__ static void fold_u(const float *p, float *u)
    {
        u[0] = kSigFold * (u[0] + p[3]); u[1] = kSigFold * (u[1] + p[4]); u[2] = kTanhFold * (u[2] + p[5]);
    }

    template <bool FOLD>
    __device__ __forceinline__ static void gates(const float *p, const float *q, float h, const float *u, float &z,
                                                 float &r, float &rh, float &c)
    {
        z = gate_sigmoid<FOLD>(gate_in<FOLD>(p[0], FOLD ? q[0] : 0.0f, h, u[0], p[3]));
        r = gate_sigmoid<FOLD>(gate_in<FOLD>(p[1], FOLD ? q[1] : 0.0f, h, u[1], p[4]));
        rh = r * h;
        c = gate_tanh<FOLD>(gate_in<FOLD>(p[2], FOLD ? q[2] : 0.0f, rh, u[2], p[5]));
    }

    template <bool FOLD = false>
    __device__ __forceinline__ static void step(const float *p, const float *hp, const float *u, float *F,
                                                const float *q = nullptr)
    {
        float z, r, rh, c;
        gates<FOLD>(p, q, hp[0], u, z, r, rh, c);
        F[0] = fmaf(z, c - hp[0], hp[0]);
    }

    // k_z = (c-h) z(1-z), k_c = z (1-c^2), k_r = k_c a_c h r(1-r) are df/du_z,
    // df/du_c, df/du_r;  J = (1-z) + a_z k_z + a_c r k_c + a_r k_r  (Eq. (8a)).
    template <bool FOLD>
    __device__ __forceinline__ static void coefs(const float *p, const float *q, float h, const float *u, float &F,
                                                 float &J, float &kz, float &kr, float &kc, float &rh)
    {
        float z, r, c;
        gates<FOLD>(p, q, h, u, z, r, rh, c);
        const float cmh = c - h, omz = 1.0f - z;
        F = fmaf(z, cmh, h);
        kz = cmh * (z * omz);
        kc = z * fmaf(-c, c, 1.0f);
        const float ackc = p[2] * kc;
        kr = ackc * (rh * (1.0f - r));
        J = fmaf(p[0], kz, omz);
        J = fmaf(ackc, r, J);
        J = fmaf(p[1], kr, J);
    }

    // The forward pass needs F and J only: J = (1-z) + a_z k_z + a_c k_c (r + a_r r h (1-r)), which
    // skips k_r as a value of its own (one instruction fewer per evaluation than coefs).
    template <bool FOLD = false>
    __device__ __forceinline__ static void fwd(const float *p, const float *hp, const float *u, float *F, float *J,
                                               const float *q = nullptr)
    {
        float z, r, rh, c;
        const float h = hp[0];
        gates<FOLD>(p, q, h, u, z, r, rh, c);
        const float cmh = c - h, omz = 1.0f - z;
        F[0] = fmaf(z, cmh, h);
        const float kz = cmh * (z * omz);
        const float ackc = p[2] * (z * fmaf(-c, c, 1.0f));
        const float t = fmaf(p[1], rh * (1.0f - r), r);
        J[0] = fmaf(ackc, t, fmaf(p[0], kz, omz));
    }

    __device__ __forceinline__ static void bwd_prep(const float *p, const float *hp, const float *u,
                                                    float *J, float *k)
    {
        float F;
        coefs<false>(p, nullptr, hp[0], u, F, J[0], k[0], k[1], k[2], k[4]);
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

// LSTM-style cell with separate input/forget gates that all read h_{l-1}
// through diagonal weights; state (c, h); 2x2 Jacobian block per channel (the
// block structure of Eq. (8b)).
struct LstmDiag {
    static constexpr int G = 4, S = 2, PR = 8, NC = 6, PQ = 4;

    __device__ __forceinline__ static void fold_params(const float *p, float *q)
    {
        q[0] = kSigFold * p[0]; q[1] = kSigFold * p[1]; q[2] = kSigFold * p[2]; q[3] = kTanhFold * p[3];
    }
    __device__ __forceinline__ static void fold_u(const float *p, float *u)
    {
        u[0] = kSigFold * (u[0] + p[4]); u[1] = kSigFold * (u[1] + p[5]);
        u[2] = kSigFold * (u[2] + p[6]); u[3] = kTanhFold * (u[3] + p[7]);
    }

    template <bool FOLD>
    __device__ __forceinline__ static void gates(const float *p, const float *q, float h, const float *u, float &i,
                                                 float &f, float &o, float &g)
    {
        i = gate_sigmoid<FOLD>(gate_in<FOLD>(p[0], FOLD ? q[0] : 0.0f, h, u[0], p[4]));
        f = gate_sigmoid<FOLD>(gate_in<FOLD>(p[1], FOLD ? q[1] : 0.0f, h, u[1], p[5]));
        o = gate_sigmoid<FOLD>(gate_in<FOLD>(p[2], FOLD ? q[2] : 0.0f, h, u[2], p[6]));
        g = gate_tanh<FOLD>(gate_in<FOLD>(p[3], FOLD ? q[3] : 0.0f, h, u[3], p[7]));
    }

    template <bool FOLD = false>
    __device__ __forceinline__ static void step(const float *p, const float *hp, const float *u, float *F,
                                                const float *q = nullptr)
    {
        float i, f, o, g;
        gates<FOLD>(p, q, hp[1], u, i, f, o, g);
        F[0] = fmaf(f, hp[0], i * g);
        F[1] = o * fast_tanh(F[0]);
    }

    // k[0..3] = d c'/d u_{i,f,g-slot order i,f,o,g} with k[2] = d h'/d u_o,
    // k[4] = o (1 - tanh(c')^2) = d h'/d c', k[5] = h.
    template <bool FOLD>
    __device__ __forceinline__ static void coefs(const float *p, const float *q, const float *hp, const float *u,
                                                 float *F, float *J, float *k)
    {
        const float c = hp[0], h = hp[1];
        float i, f, o, g;
        gates<FOLD>(p, q, h, u, i, f, o, g);
        const float cn = fmaf(f, c, i * g);
        const float t = fast_tanh(cn);
        F[0] = cn;
        F[1] = o * t;
        k[0] = g * (i * (1.0f - i));
        k[1] = c * (f * (1.0f - f));
        k[2] = t * (o * (1.0f - o));
        k[3] = i * fmaf(-g, g, 1.0f);
        k[4] = o * fmaf(-t, t, 1.0f);
        k[5] = h;
        const float jch = fmaf(k[0], p[0], fmaf(k[1], p[1], k[3] * p[3]));
        J[0] = f;
        J[1] = jch;
        J[2] = k[4] * f;
        J[3] = fmaf(k[2], p[2], k[4] * jch);
    }

    template <bool FOLD = false>
    __device__ __forceinline__ static void fwd(const float *p, const float *hp, const float *u, float *F, float *J,
                                               const float *q = nullptr)
    {
        float k[NC];
        coefs<FOLD>(p, q, hp, u, F, J, k);
    }

    __device__ __forceinline__ static void bwd_prep(const float *p, const float *hp, const float *u,
                                                    float *J, float *k)
    {
        float F[2];
        coefs<false>(p, nullptr, hp, u, F, J, k);
    }

    __device__ __forceinline__ static void bwd_emit(const float *k, const float *lam, float *du, float *acc)
    {
        const float dcn = fmaf(lam[1], k[4], lam[0]);
        du[0] = dcn * k[0];
        du[1] = dcn * k[1];
        du[2] = lam[1] * k[2];
        du[3] = dcn * k[3];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            acc[g] = fmaf(du[g], k[5], acc[g]);
            acc[4 + g] += du[g];
        }
    }
};

// The paper's ParaLSTM: Sec. 3, Eq. (7b) with diagonal A_*, C_* (Eq. (9)) -- input
// and forget gates combined, peepholes from c_{l-1} into f and from the new c
// into o, candidate nonlinearity tanh.  Jacobian blocks: Eq. (8b).
// Parameter rows: a_f, a_z, a_o, c_f, c_o, b_f, b_z, b_o.  Gates (f, z, o).
struct ParaLstmDiag {
    static constexpr int G = 3, S = 2, PR = 8, NC = 8, PQ = 5;

    // q = scaled a_f, a_z, a_o, c_f, c_o
    __device__ __forceinline__ static void fold_params(const float *p, float *q)
    {
        q[0] = kSigFold * p[0]; q[1] = kTanhFold * p[1]; q[2] = kSigFold * p[2];
        q[3] = kSigFold * p[3]; q[4] = kSigFold * p[4];
    }
    __device__ __forceinline__ static void fold_u(const float *p, float *u)
    {
        u[0] = kSigFold * (u[0] + p[5]); u[1] = kTanhFold * (u[1] + p[6]); u[2] = kSigFold * (u[2] + p[7]);
    }

    // f and z from the previous state; o needs the new c
    template <bool FOLD>
    __device__ __forceinline__ static void gates_fz(const float *p, const float *q, float c, float h, const float *u,
                                                    float &f, float &z)
    {
        if constexpr (FOLD) {
            f = gate_sigmoid<true>(fmaf(q[0], h, fmaf(q[3], c, u[0])));
            z = gate_tanh<true>(fmaf(q[1], h, u[1]));
        } else {
            f = fast_sigmoid(fmaf(p[0], h, fmaf(p[3], c, u[0] + p[5])));
            z = fast_tanh(fmaf(p[1], h, u[1] + p[6]));
        }
    }
    template <bool FOLD>
    __device__ __forceinline__ static float gate_o(const float *p, const float *q, float cn, float h, const float *u)
    {
        if constexpr (FOLD) return gate_sigmoid<true>(fmaf(q[2], h, fmaf(q[4], cn, u[2])));
        else return fast_sigmoid(fmaf(p[2], h, fmaf(p[4], cn, u[2] + p[7])));
    }

    template <bool FOLD = false>
    __device__ __forceinline__ static void step(const float *p, const float *hp, const float *u, float *F,
                                                const float *q = nullptr)
    {
        const float c = hp[0], h = hp[1];
        float f, z;
        gates_fz<FOLD>(p, q, c, h, u, f, z);
        const float cn = fmaf(f, c - z, z);
        const float o = gate_o<FOLD>(p, q, cn, h, u);
        F[0] = cn;
        F[1] = o * fast_tanh(cn);
    }

    // k[0] = d c'/d u_f = (c - z) f(1-f), k[1] = d c'/d u_z = (1-f)(1-z^2),
    // k[2] = d h'/d u_o = t o(1-o), k[3] = o (1-t^2), k[4] = c_o, k[5] = h, k[6] = c, k[7] = c'.
    template <bool FOLD>
    __device__ __forceinline__ static void coefs(const float *p, const float *q, const float *hp, const float *u,
                                                 float *F, float *J, float *k)
    {
        const float c = hp[0], h = hp[1];
        float f, z;
        gates_fz<FOLD>(p, q, c, h, u, f, z);
        const float cmz = c - z;
        const float cn = fmaf(f, cmz, z);
        const float o = gate_o<FOLD>(p, q, cn, h, u);
        const float t = fast_tanh(cn);
        F[0] = cn;
        F[1] = o * t;
        k[0] = cmz * (f * (1.0f - f));
        k[1] = (1.0f - f) * fmaf(-z, z, 1.0f);
        k[2] = t * (o * (1.0f - o));
        k[3] = o * fmaf(-t, t, 1.0f);
        k[4] = p[4];
        k[5] = h;
        k[6] = c;
        k[7] = cn;
        const float jcc = fmaf(k[0], p[3], f);
        const float jch = fmaf(k[0], p[0], k[1] * p[1]);
        const float hc = fmaf(k[2], p[4], k[3]);          // d h'/d c' including the peephole of o
        J[0] = jcc;
        J[1] = jch;
        J[2] = hc * jcc;
        J[3] = fmaf(k[2], p[2], hc * jch);
    }

    template <bool FOLD = false>
    __device__ __forceinline__ static void fwd(const float *p, const float *hp, const float *u, float *F, float *J,
                                               const float *q = nullptr)
    {
        float k[NC];
        coefs<FOLD>(p, q, hp, u, F, J, k);
    }

    __device__ __forceinline__ static void bwd_prep(const float *p, const float *hp, const float *u,
                                                    float *J, float *k)
    {
        float F[2];
        coefs<false>(p, nullptr, hp, u, F, J, k);
    }

    __device__ __forceinline__ static void bwd_emit(const float *k, const float *lam, float *du, float *acc)
    {
        const float dpo = lam[1] * k[2];
        const float dcn = fmaf(lam[1], k[3], fmaf(dpo, k[4], lam[0]));
        const float dpf = dcn * k[0], dpz = dcn * k[1];
        du[0] = dpf;
        du[1] = dpz;
        du[2] = dpo;
        acc[0] = fmaf(dpf, k[5], acc[0]);
        acc[1] = fmaf(dpz, k[5], acc[1]);
        acc[2] = fmaf(dpo, k[5], acc[2]);
        acc[3] = fmaf(dpf, k[6], acc[3]);
        acc[4] = fmaf(dpo, k[7], acc[4]);
        acc[5] += dpf;
        acc[6] += dpz;
        acc[7] += dpo;
    }
};

// Linear SSM of the footnote in Sec. 2: f = a h + u + b, J = a.
struct LinearDiag {
    static constexpr int G = 1, S = 1, PR = 2, NC = 1, PQ = 0;

    __device__ __forceinline__ static void fold_params(const float *, float *) {}
    __device__ __forceinline__ static void fold_u(const float *p, float *u) { u[0] += p[1]; }

    template <bool FOLD = false>
    __device__ __forceinline__ static void step(const float *p, const float *hp, const float *u, float *F,
                                                const float * = nullptr)
    {
        F[0] = fmaf(p[0], hp[0], FOLD ? u[0] : u[0] + p[1]);
    }
    template <bool FOLD = false>
    __device__ __forceinline__ static void fwd(const float *p, const float *hp, const float *u, float *F, float *J,
                                               const float * = nullptr)
    {
        step<FOLD>(p, hp, u, F);
        J[0] = p[0];
    }
    __device__ __forceinline__ static void bwd_prep(const float *p, const float *hp, const float *, float *J, float *k)
    {
        J[0] = p[0];
        k[0] = hp[0];
    }
    __device__ __forceinline__ static void bwd_emit(const float *k, const float *lam, float *du, float *acc)
    {
        du[0] = lam[0];
        acc[0] = fmaf(lam[0], k[0], acc[0]);
        acc[1] += lam[0];
    }
};

}  // namespace pararnn
