/*
 * CPU oracle for the sequence-parallel application of a nonlinear RNN.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
 * sequential implementation of what the method computes, used only by the
 * tests, the smoke check and the benchmark's CPU-baseline leg.  It shares no
 * code, header, table or helper with the HIP library and neither side
 * includes or links the other.
 *
 * What it follows (ParaRNN, arXiv 2510.21450):
 *   - Sec. 2, Eq. (1): the recurrence h_l = f(h_{l-1}, x_l)       -> oracle_seq_unroll
 *   - Sec. 2, Eq. (3) + Alg. 1a: Newton on the stacked system     -> oracle_newton
 *   - Sec. 2, Eq. (4): forward substitution of the linearised,
 *     block bi-diagonal system                                    -> oracle_forward_substitution
 *   - Sec. 2, Alg. 1b: the naive parallel reduction               -> oracle_parallel_reduce
 *   - Sec. 2, Eq. (6): the backward (adjoint) recurrence          -> oracle_backward
 *   - Sec. 3, Eq. (7a) with the diagonal weights of Eq. (9): GRU  -> cell 0
 *   - Sec. 3, Eq. (8a): its Jacobian                              -> oracle_cell_jacobian
 *   - Sec. 3, Eq. (7b) / (8b) with diagonal A_*, C_* (Eq. (9)): the
 *     CIFG LSTM with peepholes (ParaLSTM) and its 2x2 Jacobian    -> cell 4
 *   - App. A: the initial guess h^0_l = f(h_0, x_l)               -> oracle_newton
 *   - Sec. 1 / Sec. 2.1: the quasi-Newton variant of prior work, Newton with
 *     every Jacobian replaced by its diagonal                     -> oracle_newton_diag
 *   - App. A: the max-norm of the residual of Eq. (2), the
 *     quantity its convergence figure plots per iteration         -> oracle_residual_norm
 *   - Sec. 3, Eq. (7a) / (7b): the input terms B_* x_l + b_* of all gates,
 *     with the multi-head (block-diagonal) input matrices of App. C     -> oracle_input_projection
 *     and the derivatives of that map                                   -> oracle_input_projection_backward
 *   - App. D.3: the GRU's update / reset / state nonlinearities are
 *     parameters of the cell: Eq. (7a) / (8a) with each of them chosen
 *     from sigmoid, tanh, identity, softsign                      -> cells 100..163
 *   - Sec. 2.1 (block-diagonal Jacobians): a cell written only to
 *     exercise 2x2 blocks that do not come from an LSTM, a per-channel
 *     rotation-scaling followed by tanh                           -> cell 5
 *     and cells with 3x3 and 4x4 blocks (N state values per channel
 *     mixed by a per-channel N x N matrix, then tanh)             -> cells 6, 7
 *
 * Precision: REAL is double unless the file is compiled with -DREAL=float
 * (a second build used only to look at fp32 iteration traces).
 *
 * Layouts (H contiguous): u [B][L][G][H]; h, g [B][L][S][H]; h0 [B][S][H];
 * params for the diagonal cells [2][G][H] (recurrent weights, then biases),
 * for the dense cell W[H][H] row-major, for the ParaLSTM [8][H] = (a_f, a_z,
 * a_o, c_f, c_o, b_f, b_z, b_o).  Gate order GRU (z,r,c), LSTM (i,f,o,g),
 * ParaLSTM (f,z,o); LSTM state order (c,h).  Cells 100 + 16 nu + 4 nr + ns
 * (nu, nr, ns in 0..3 = sigmoid, tanh, identity, softsign) share the GRU's
 * layouts.  Cell 5: params [2][H] = (a, b), u [2][H], state (p, q):
 * p' = tanh(a p - b q + u_1), q' = tanh(b p + a q + u_2).
 *
 * Parity pins: every function here is checked by tests that do not call it to
 * produce their own expected value (closed forms, finite differences, brute
 * force of Eq. (5), invariants); none is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#ifndef REAL
#define REAL double
#endif

enum { CELL_GRU_DIAG = 0, CELL_LSTM_DIAG = 1, CELL_TANH_DENSE = 2, CELL_LINEAR_DIAG = 3, CELL_PARALSTM_DIAG = 4,
       CELL_ROT_TANH = 5, CELL_TRI_TANH = 6, CELL_QUAD_TANH = 7, CELL_GRU_NL = 100 /* .. 163 */ };
enum { NL_SIGMOID = 0, NL_TANH = 1, NL_IDENTITY = 2, NL_SOFTSIGN = 3 };
enum { ST_OK = 0, ST_NOT_CONVERGED = 1, ST_INVALID = 2, ST_NONFINITE = 5 };
/* BLOCK3 / BLOCK4: [N][N][H] with N = 3 / 4, J[a][b] = dF_a/dh_b */
enum { JAC_DIAG = 0, JAC_BLOCK2 = 1, JAC_DENSE = 2, JAC_BLOCK3 = 3, JAC_BLOCK4 = 4 };
static int block_dim(int kind) { return kind == JAC_BLOCK3 ? 3 : kind == JAC_BLOCK4 ? 4 : 0; }
/* state values per channel of the cells that mix them with a per-channel N x N matrix, else 0 */
static int mix_dim(int cell);

static REAL sigmoid(REAL x) { return (REAL)1 / ((REAL)1 + (REAL)exp(-(double)x)); }
static REAL tanh_r(REAL x) { return (REAL)tanh((double)x); }

static int is_gru_nl(int cell) { return cell >= CELL_GRU_NL && cell < CELL_GRU_NL + 64; }

/* a nonlinearity by number and its derivative, both as functions of the pre-activation */
static REAL nl_f(int kind, REAL x)
{
    if (kind == NL_SIGMOID) return sigmoid(x);
    if (kind == NL_TANH) return tanh_r(x);
    if (kind == NL_SOFTSIGN) return x / ((REAL)1 + (REAL)fabs((double)x));
    return x;
}

static REAL nl_d(int kind, REAL x)
{
    if (kind == NL_SIGMOID) { REAL s = sigmoid(x); return s * ((REAL)1 - s); }
    if (kind == NL_TANH) { REAL t = tanh_r(x); return (REAL)1 - t * t; }
    if (kind == NL_SOFTSIGN) { REAL q = (REAL)1 + (REAL)fabs((double)x); return (REAL)1 / (q * q); }
    return (REAL)1;
}

int oracle_real_bytes(void) { return (int)sizeof(REAL); }

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int mix_dim(int cell) { return cell == CELL_TRI_TANH ? 3 : cell == CELL_QUAD_TANH ? 4 : 0; }

int oracle_gates(int cell)
{
    switch (cell) {
    case CELL_GRU_DIAG: return 3;
    case CELL_LSTM_DIAG: return 4;
    case CELL_TANH_DENSE: return 1;
    case CELL_LINEAR_DIAG: return 1;
    case CELL_PARALSTM_DIAG: return 3;
    case CELL_ROT_TANH: return 2;
    case CELL_TRI_TANH: return 3;
    case CELL_QUAD_TANH: return 4;
    }
    return is_gru_nl(cell) ? 3 : -1;
}

int oracle_state(int cell)
{
    if (cell == CELL_LSTM_DIAG || cell == CELL_PARALSTM_DIAG || cell == CELL_ROT_TANH) return 2;
    if (mix_dim(cell)) return mix_dim(cell);
    return (cell >= 0 && cell <= 3) || is_gru_nl(cell) ? 1 : -1;
}

int oracle_jac_kind(int cell)
{
    if (cell == CELL_LSTM_DIAG || cell == CELL_PARALSTM_DIAG || cell == CELL_ROT_TANH) return JAC_BLOCK2;
    if (cell == CELL_TANH_DENSE) return JAC_DENSE;
    if (cell == CELL_TRI_TANH) return JAC_BLOCK3;
    if (cell == CELL_QUAD_TANH) return JAC_BLOCK4;
    return JAC_DIAG;
}

/* number of REALs one Jacobian J_l occupies */
static size_t jac_size(int kind, int H)
{
    if (kind == JAC_DIAG) return (size_t)H;
    if (kind == JAC_BLOCK2) return (size_t)4 * H;       /* [2][2][H] */
    if (block_dim(kind)) return (size_t)block_dim(kind) * block_dim(kind) * H;
    return (size_t)H * H;                               /* [H][H] row-major */
}

static size_t param_count(int cell, int H)
{
    if (cell == CELL_TANH_DENSE) return (size_t)H * H;
    if (cell == CELL_PARALSTM_DIAG) return (size_t)8 * H;
    if (cell == CELL_ROT_TANH) return (size_t)2 * H;
    if (mix_dim(cell)) return (size_t)mix_dim(cell) * mix_dim(cell) * H;
    return (size_t)2 * oracle_gates(cell) * H;
}

/* ------------------------------------------------------------------ cells */

/* One application of the recurrence step f, Eq. (1).
 * hp: previous state [S][H]; u: pre-activations [G][H]; out: new state [S][H]. */
void oracle_cell_step(int cell, int H, const REAL *params, const REAL *hp, const REAL *u, REAL *out)
{
    int j;
    if (cell == CELL_GRU_DIAG) {
        /* Eq. (7a) with A_* = diag(a_*) (Eq. (9)) and u = B x + b precomputed;
         * an extra bias b_* is part of params. */
        const REAL *a = params, *b = params + 3 * H;
        for (j = 0; j < H; ++j) {
            REAL h = hp[j];
            REAL z = sigmoid(a[0 * H + j] * h + u[0 * H + j] + b[0 * H + j]);
            REAL r = sigmoid(a[1 * H + j] * h + u[1 * H + j] + b[1 * H + j]);
            REAL c = tanh_r(a[2 * H + j] * (r * h) + u[2 * H + j] + b[2 * H + j]);
            out[j] = ((REAL)1 - z) * h + z * c;
        }
    } else if (cell == CELL_LSTM_DIAG) {
        /* LSTM-style cell of the benchmark: separate input and forget gates,
         * all gates read h_{l-1} through diagonal weights; state (c,h). */
        const REAL *w = params, *b = params + 4 * H;
        const REAL *cp = hp, *hh = hp + H;
        for (j = 0; j < H; ++j) {
            REAL h = hh[j];
            REAL i = sigmoid(w[0 * H + j] * h + u[0 * H + j] + b[0 * H + j]);
            REAL f = sigmoid(w[1 * H + j] * h + u[1 * H + j] + b[1 * H + j]);
            REAL o = sigmoid(w[2 * H + j] * h + u[2 * H + j] + b[2 * H + j]);
            REAL g = tanh_r(w[3 * H + j] * h + u[3 * H + j] + b[3 * H + j]);
            REAL cn = f * cp[j] + i * g;
            out[j] = cn;
            out[H + j] = o * tanh_r(cn);
        }
    } else if (cell == CELL_PARALSTM_DIAG) {
        /* Eq. (7b) with A_* = diag(a_*), C_* = diag(c_*) (Eq. (9)): input and
         * forget gates combined, peepholes from c_{l-1} into f and from the
         * NEW c_l into o; the candidate nonlinearity sigma_z is taken as tanh. */
        const REAL *af = params, *az = params + H, *ao = params + 2 * H, *cf = params + 3 * H,
                   *co = params + 4 * H, *bf = params + 5 * H, *bz = params + 6 * H, *bo = params + 7 * H;
        const REAL *cp = hp, *hh = hp + H;
        for (j = 0; j < H; ++j) {
            REAL h = hh[j], c = cp[j];
            REAL f = sigmoid(af[j] * h + u[0 * H + j] + cf[j] * c + bf[j]);
            REAL z = tanh_r(az[j] * h + u[1 * H + j] + bz[j]);
            REAL cn = f * c + ((REAL)1 - f) * z;
            REAL o = sigmoid(ao[j] * h + u[2 * H + j] + co[j] * cn + bo[j]);
            out[j] = cn;
            out[H + j] = o * tanh_r(cn);
        }
    } else if (is_gru_nl(cell)) {
        /* Eq. (7a) with diagonal weights and the three nonlinearities chosen by number */
        const int nu = ((cell - CELL_GRU_NL) >> 4) & 3, nr = ((cell - CELL_GRU_NL) >> 2) & 3, ns = (cell - CELL_GRU_NL) & 3;
        const REAL *a = params, *b = params + 3 * H;
        for (j = 0; j < H; ++j) {
            REAL h = hp[j];
            REAL z = nl_f(nu, a[0 * H + j] * h + u[0 * H + j] + b[0 * H + j]);
            REAL r = nl_f(nr, a[1 * H + j] * h + u[1 * H + j] + b[1 * H + j]);
            REAL c = nl_f(ns, a[2 * H + j] * (r * h) + u[2 * H + j] + b[2 * H + j]);
            out[j] = ((REAL)1 - z) * h + z * c;
        }
    } else if (cell == CELL_ROT_TANH) {
        const REAL *a = params, *b = params + H;
        for (j = 0; j < H; ++j) {
            REAL p = hp[j], q = hp[H + j];
            out[j] = tanh_r(a[j] * p - b[j] * q + u[j]);
            out[H + j] = tanh_r(b[j] * p + a[j] * q + u[H + j]);
        }
    } else if (mix_dim(cell)) {
        /* N state values per channel mixed by that channel's own N x N matrix m (params [N][N][H]):
         * x'_a = tanh(sum_b m_ab x_b + u_a); a cell with N x N Jacobian blocks (Sec. 2.1), N = 3, 4 */
        const int N = mix_dim(cell);
        int a, b;
        for (j = 0; j < H; ++j)
            for (a = 0; a < N; ++a) {
                REAL s = u[a * H + j];
                for (b = 0; b < N; ++b) s += params[(N * a + b) * H + j] * hp[b * H + j];
                out[a * H + j] = tanh_r(s);
            }
    } else if (cell == CELL_TANH_DENSE) {
        /* generic dense-Jacobian cell: h' = tanh(W h + u) (Sec. 2.1) */
        int i;
        for (i = 0; i < H; ++i) {
            REAL s = u[i];
            for (j = 0; j < H; ++j) s += params[(size_t)i * H + j] * hp[j];
            out[i] = tanh_r(s);
        }
    } else {
        /* linear SSM of the footnote in Sec. 2: f = a h + u (+ b) */
        for (j = 0; j < H; ++j) out[j] = params[j] * hp[j] + u[j] + params[H + j];
    }
}

/* Jacobian of f with respect to the previous state, evaluated at (hp, u).
 * This is the J_l of Eq. (3): the derivative of equation l with respect to
 * its own input h_{l-1}.  Layout by kind: diag [H]; block2 [2][2][H] with
 * J[p][q] = d(out_p)/d(in_q), p,q in (c,h); dense [H][H] row-major. */
void oracle_cell_jacobian(int cell, int H, const REAL *params, const REAL *hp, const REAL *u, REAL *J)
{
    int j;
    if (cell == CELL_GRU_DIAG) {
        /* Eq. (8a) with diagonal A_*: every factor is a per-channel scalar. */
        const REAL *a = params, *b = params + 3 * H;
        for (j = 0; j < H; ++j) {
            REAL h = hp[j];
            REAL z = sigmoid(a[0 * H + j] * h + u[0 * H + j] + b[0 * H + j]);
            REAL r = sigmoid(a[1 * H + j] * h + u[1 * H + j] + b[1 * H + j]);
            REAL c = tanh_r(a[2 * H + j] * (r * h) + u[2 * H + j] + b[2 * H + j]);
            REAL dz = z * ((REAL)1 - z), dr = r * ((REAL)1 - r), dc = (REAL)1 - c * c;
            J[j] = ((REAL)1 - z) + (c - h) * dz * a[0 * H + j]
                 + z * dc * a[2 * H + j] * (r + h * dr * a[1 * H + j]);
        }
    } else if (cell == CELL_LSTM_DIAG) {
        const REAL *w = params, *b = params + 4 * H;
        const REAL *cp = hp, *hh = hp + H;
        for (j = 0; j < H; ++j) {
            REAL h = hh[j], c = cp[j];
            REAL i = sigmoid(w[0 * H + j] * h + u[0 * H + j] + b[0 * H + j]);
            REAL f = sigmoid(w[1 * H + j] * h + u[1 * H + j] + b[1 * H + j]);
            REAL o = sigmoid(w[2 * H + j] * h + u[2 * H + j] + b[2 * H + j]);
            REAL g = tanh_r(w[3 * H + j] * h + u[3 * H + j] + b[3 * H + j]);
            REAL t = tanh_r(f * c + i * g);
            REAL Jch = c * f * ((REAL)1 - f) * w[1 * H + j] + g * i * ((REAL)1 - i) * w[0 * H + j]
                     + i * ((REAL)1 - g * g) * w[3 * H + j];
            J[0 * H + j] = f;                                          /* dc'/dc */
            J[1 * H + j] = Jch;                                        /* dc'/dh */
            J[2 * H + j] = o * ((REAL)1 - t * t) * f;                  /* dh'/dc */
            J[3 * H + j] = t * o * ((REAL)1 - o) * w[2 * H + j] + o * ((REAL)1 - t * t) * Jch; /* dh'/dh */
        }
    } else if (cell == CELL_PARALSTM_DIAG) {
        /* Eq. (8b) with diagonal A_*, C_*: every block is a per-channel scalar. */
        const REAL *af = params, *az = params + H, *ao = params + 2 * H, *cf = params + 3 * H,
                   *co = params + 4 * H, *bf = params + 5 * H, *bz = params + 6 * H, *bo = params + 7 * H;
        const REAL *cp = hp, *hh = hp + H;
        for (j = 0; j < H; ++j) {
            REAL h = hh[j], c = cp[j];
            REAL f = sigmoid(af[j] * h + u[0 * H + j] + cf[j] * c + bf[j]);
            REAL z = tanh_r(az[j] * h + u[1 * H + j] + bz[j]);
            REAL cn = f * c + ((REAL)1 - f) * z;
            REAL o = sigmoid(ao[j] * h + u[2 * H + j] + co[j] * cn + bo[j]);
            REAL t = tanh_r(cn);
            REAL sf = f * ((REAL)1 - f), so = o * ((REAL)1 - o), sz = (REAL)1 - z * z, st = (REAL)1 - t * t;
            REAL Jcc = f + (c - z) * sf * cf[j];
            REAL Jch = (c - z) * sf * af[j] + ((REAL)1 - f) * sz * az[j];
            J[0 * H + j] = Jcc;
            J[1 * H + j] = Jch;
            J[2 * H + j] = (t * so * co[j] + o * st) * Jcc;
            J[3 * H + j] = t * so * (ao[j] + co[j] * Jch) + o * st * Jch;
        }
    } else if (is_gru_nl(cell)) {
        /* Eq. (8a) with sigma' and tanh' replaced by the chosen nonlinearities' derivatives */
        const int nu = ((cell - CELL_GRU_NL) >> 4) & 3, nr = ((cell - CELL_GRU_NL) >> 2) & 3, ns = (cell - CELL_GRU_NL) & 3;
        const REAL *a = params, *b = params + 3 * H;
        for (j = 0; j < H; ++j) {
            REAL h = hp[j];
            REAL xz = a[0 * H + j] * h + u[0 * H + j] + b[0 * H + j];
            REAL xr = a[1 * H + j] * h + u[1 * H + j] + b[1 * H + j];
            REAL z = nl_f(nu, xz), r = nl_f(nr, xr);
            REAL xc = a[2 * H + j] * (r * h) + u[2 * H + j] + b[2 * H + j];
            REAL c = nl_f(ns, xc);
            J[j] = ((REAL)1 - z) + (c - h) * nl_d(nu, xz) * a[0 * H + j]
                 + z * nl_d(ns, xc) * a[2 * H + j] * (r + h * nl_d(nr, xr) * a[1 * H + j]);
        }
    } else if (cell == CELL_ROT_TANH) {
        const REAL *a = params, *b = params + H;
        for (j = 0; j < H; ++j) {
            REAL p = hp[j], q = hp[H + j];
            REAL t1 = tanh_r(a[j] * p - b[j] * q + u[j]), t2 = tanh_r(b[j] * p + a[j] * q + u[H + j]);
            REAL d1 = (REAL)1 - t1 * t1, d2 = (REAL)1 - t2 * t2;
            J[0 * H + j] = d1 * a[j];
            J[1 * H + j] = -d1 * b[j];
            J[2 * H + j] = d2 * b[j];
            J[3 * H + j] = d2 * a[j];
        }
    } else if (mix_dim(cell)) {
        const int N = mix_dim(cell);
        int a, b;
        for (j = 0; j < H; ++j)
            for (a = 0; a < N; ++a) {
                REAL s = u[a * H + j], t;
                for (b = 0; b < N; ++b) s += params[(N * a + b) * H + j] * hp[b * H + j];
                t = tanh_r(s);
                for (b = 0; b < N; ++b) J[(N * a + b) * H + j] = ((REAL)1 - t * t) * params[(N * a + b) * H + j];
            }
    } else if (cell == CELL_TANH_DENSE) {
        int i;
        for (i = 0; i < H; ++i) {
            REAL s = u[i], d;
            for (j = 0; j < H; ++j) s += params[(size_t)i * H + j] * hp[j];
            d = tanh_r(s);
            d = (REAL)1 - d * d;
            for (j = 0; j < H; ++j) J[(size_t)i * H + j] = d * params[(size_t)i * H + j];
        }
    } else {
        for (j = 0; j < H; ++j) J[j] = params[j];
    }
}

/* y = J x for one Jacobian of the given kind; x, y are [S][H]. */
static void jac_apply(int kind, int H, const REAL *J, const REAL *x, REAL *y)
{
    int i, j;
    if (kind == JAC_DIAG) {
        for (j = 0; j < H; ++j) y[j] = J[j] * x[j];
    } else if (kind == JAC_BLOCK2) {
        for (j = 0; j < H; ++j) {
            REAL xc = x[j], xh = x[H + j];
            y[j] = J[0 * H + j] * xc + J[1 * H + j] * xh;
            y[H + j] = J[2 * H + j] * xc + J[3 * H + j] * xh;
        }
    } else if (block_dim(kind)) {
        const int N = block_dim(kind);
        int q;
        for (j = 0; j < H; ++j)
            for (i = 0; i < N; ++i) {
                REAL s = J[(N * i) * H + j] * x[j];
                for (q = 1; q < N; ++q) s += J[(N * i + q) * H + j] * x[q * H + j];
                y[i * H + j] = s;
            }
    } else {
        for (i = 0; i < H; ++i) {
            REAL s = 0;
            for (j = 0; j < H; ++j) s += J[(size_t)i * H + j] * x[j];
            y[i] = s;
        }
    }
}

/* J <- diag(J): zero every entry d(out_i)/d(in_j) with i != j (state values of all channels
 * counted as one vector, so the 2x2 blocks lose J_ch and J_hc) */
static void jac_keep_diagonal(int kind, int H, REAL *J)
{
    int i, j;
    if (kind == JAC_BLOCK2) {
        for (j = 0; j < H; ++j) J[1 * H + j] = J[2 * H + j] = 0;
    } else if (block_dim(kind)) {
        const int N = block_dim(kind);
        for (i = 0; i < N * N; ++i)
            if (i % (N + 1) != 0)
                for (j = 0; j < H; ++j) J[i * H + j] = 0;
    } else if (kind != JAC_DIAG) {
        for (i = 0; i < H; ++i)
            for (j = 0; j < H; ++j)
                if (i != j) J[(size_t)i * H + j] = 0;
    }
}

/* C = A B for two Jacobians of the same kind */
static void jac_mul(int kind, int H, const REAL *A, const REAL *Bm, REAL *C)
{
    int i, j, k;
    if (kind == JAC_DIAG) {
        for (j = 0; j < H; ++j) C[j] = A[j] * Bm[j];
    } else if (kind == JAC_BLOCK2) {
        for (j = 0; j < H; ++j) {
            REAL a00 = A[0 * H + j], a01 = A[1 * H + j], a10 = A[2 * H + j], a11 = A[3 * H + j];
            REAL b00 = Bm[0 * H + j], b01 = Bm[1 * H + j], b10 = Bm[2 * H + j], b11 = Bm[3 * H + j];
            C[0 * H + j] = a00 * b00 + a01 * b10;
            C[1 * H + j] = a00 * b01 + a01 * b11;
            C[2 * H + j] = a10 * b00 + a11 * b10;
            C[3 * H + j] = a10 * b01 + a11 * b11;
        }
    } else if (block_dim(kind)) {
        const int N = block_dim(kind);
        int q;
        for (j = 0; j < H; ++j)
            for (i = 0; i < N; ++i)
                for (k = 0; k < N; ++k) {
                    REAL s = A[(N * i) * H + j] * Bm[k * H + j];
                    for (q = 1; q < N; ++q) s += A[(N * i + q) * H + j] * Bm[(N * q + k) * H + j];
                    C[(N * i + k) * H + j] = s;
                }
    } else {
        for (i = 0; i < H; ++i)
            for (j = 0; j < H; ++j) {
                REAL s = 0;
                for (k = 0; k < H; ++k) s += A[(size_t)i * H + k] * Bm[(size_t)k * H + j];
                C[(size_t)i * H + j] = s;
            }
    }
}

/* ------------------------------------------------- sequential application */

/* Eq. (1): h_l = f(h_{l-1}, u_l), l = 1..L, from h0 (NULL = zeros). */
void oracle_seq_unroll(int cell, int B, int L, int H, const REAL *params, const REAL *u,
                       const REAL *h0, REAL *h)
{
    const int G = oracle_gates(cell), S = oracle_state(cell);
    int b;
#pragma omp parallel for schedule(static)
    for (b = 0; b < B; ++b) {
        REAL *zero = (REAL *)calloc((size_t)S * H, sizeof(REAL));
        int l;
        for (l = 0; l < L; ++l) {
            const REAL *hp = l == 0 ? (h0 ? h0 + (size_t)b * S * H : zero)
                                    : h + ((size_t)b * L + (l - 1)) * S * H;
            oracle_cell_step(cell, H, params, hp, u + ((size_t)b * L + l) * G * H,
                             h + ((size_t)b * L + l) * S * H);
        }
        free(zero);
    }
}

/* App. A (the convergence figure's observable): how far given states are from
 * solving the stacked system Eq. (2), in max-norm:
 *     max over b, l, state value, channel of | h_l - f(h_{l-1}, u_l) |,  h_0 = h0 (NULL = zeros).
 * A NaN anywhere gives NaN. */
REAL oracle_residual_norm(int cell, int B, int L, int H, const REAL *params, const REAL *u,
                          const REAL *h0, const REAL *h)
{
    const int G = oracle_gates(cell), S = oracle_state(cell);
    const size_t n = (size_t)S * H;
    REAL *zero = (REAL *)calloc(n, sizeof(REAL)), *F = (REAL *)malloc(n * sizeof(REAL));
    REAL m = 0;
    int b, l;
    size_t i;
    for (b = 0; b < B; ++b)
        for (l = 0; l < L; ++l) {
            const REAL *hl = h + ((size_t)b * L + l) * n;
            const REAL *hp = l == 0 ? (h0 ? h0 + (size_t)b * n : zero) : hl - n;
            oracle_cell_step(cell, H, params, hp, u + ((size_t)b * L + l) * G * H, F);
            for (i = 0; i < n; ++i) {
                const REAL e = (REAL)fabs((double)(hl[i] - F[i]));
                if (e > m || e != e) m = e;
                if (m != m) break;
            }
        }
    free(zero);
    free(F);
    return m;
}

/* ----------------------------------------------- linear solvers, one sequence */

/* Eq. (4): delta_l = J_l delta_{l-1} + r_l with delta_0 = 0 (row 1 of Eq. (3)
 * has no sub-diagonal block).  J [L][jac_size], r and delta [L][S*H]. */
void oracle_forward_substitution(int kind, int L, int H, const REAL *J, const REAL *r, REAL *delta)
{
    const int S = kind == JAC_BLOCK2 ? 2 : block_dim(kind) ? block_dim(kind) : 1;
    const size_t n = (size_t)S * H, js = jac_size(kind, H);
    int l;
    size_t j;
    for (l = 0; l < L; ++l) {
        if (l == 0) {
            for (j = 0; j < n; ++j) delta[j] = r[j];
        } else {
            jac_apply(kind, H, J + (size_t)l * js, delta + (size_t)(l - 1) * n, delta + (size_t)l * n);
            for (j = 0; j < n; ++j) delta[(size_t)l * n + j] += r[(size_t)l * n + j];
        }
    }
}

/* Alg. 1b, the naive parallel reduction: A_l = -J_l, delta_l = r_l, then for
 * i = 0..ceil(log2 L)-1 every equation l >= 2^i (0-based) is reduced with the
 * one 2^i before it:  delta_l -= A_l delta_{l-2^i};  A_l = -A_l A_{l-2^i}.
 * The partner index is read as l - 2^i (the printed "+1" would pair an
 * equation with itself at i = 0).  The first equation has no sub-diagonal
 * block, so its A is zero.  The "parfor" is honoured by reading only values
 * of the previous step (two buffers). */
void oracle_parallel_reduce(int kind, int L, int H, const REAL *J, const REAL *r, REAL *delta)
{
    const int S = kind == JAC_BLOCK2 ? 2 : block_dim(kind) ? block_dim(kind) : 1;
    const size_t n = (size_t)S * H, js = jac_size(kind, H);
    REAL *A = (REAL *)malloc(sizeof(REAL) * js * L), *A2 = (REAL *)malloc(sizeof(REAL) * js * L);
    REAL *d = (REAL *)malloc(sizeof(REAL) * n * L), *d2 = (REAL *)malloc(sizeof(REAL) * n * L);
    REAL *tmp = (REAL *)malloc(sizeof(REAL) * (js > n ? js : n));
    size_t j;
    int l;
    long stride;
    for (j = 0; j < js * (size_t)L; ++j) A[j] = -J[j];
    for (j = 0; j < js; ++j) A[j] = 0;
    memcpy(d, r, sizeof(REAL) * n * L);
    for (stride = 1; stride < L; stride *= 2) {
        memcpy(A2, A, sizeof(REAL) * js * L);
        memcpy(d2, d, sizeof(REAL) * n * L);
        for (l = (int)stride; l < L; ++l) {
            const REAL *Al = A + (size_t)l * js;
            jac_apply(kind, H, Al, d + (size_t)(l - stride) * n, tmp);
            for (j = 0; j < n; ++j) d2[(size_t)l * n + j] = d[(size_t)l * n + j] - tmp[j];
            jac_mul(kind, H, Al, A + (size_t)(l - stride) * js, tmp);
            for (j = 0; j < js; ++j) A2[(size_t)l * js + j] = -tmp[j];
        }
        { REAL *t = A; A = A2; A2 = t; }
        { REAL *t = d; d = d2; d2 = t; }
    }
    memcpy(delta, d, sizeof(REAL) * n * L);
    free(A); free(A2); free(d); free(d2); free(tmp);
}

/* ------------------------------------------------------------------ Newton */

static REAL nanmax(REAL m, REAL a) { return (a > m || a != a) ? a : m; }

/* Alg. 1a with Eq. (4) as the inner solver.
 *   h^0_l = f(h0, u_l) for all l                        (App. A; reduces to
 *                                                        f(0, x_l) for h0 = 0)
 *   for k = 1..max_iter:
 *       J_l = df/dh (h^{k-1}_{l-1}, u_l),  r_l = f(h^{k-1}_{l-1}, u_l) - h^{k-1}_l
 *       delta = forward substitution;  h^k = h^{k-1} + delta
 *       m_k = max |delta| over the whole batch;  stop when m_k <= tol
 * tol < 0: run exactly max_iter iterations.  trace (or NULL) receives m_k.
 * iters = number of linear solves performed.  Returns the status.
 * diag_only != 0: the quasi-Newton variant Sec. 1 and Sec. 2.1 mention (prior work): every
 * J_l is replaced by its diagonal before the linear solve, nothing else changes. */
static int newton_impl(int cell, int B, int L, int H, const REAL *params, const REAL *u, const REAL *h0,
                       REAL tol, int max_iter, REAL *h, int *iters, REAL *trace, int diag_only)
{
    const int G = oracle_gates(cell), S = oracle_state(cell), kind = oracle_jac_kind(cell);
    const size_t n = (size_t)S * H, js = jac_size(kind, H);
    int b, k, status;
    if (G < 0 || B < 1 || L < 1 || H < 1 || max_iter < 0) return ST_INVALID;

#pragma omp parallel for schedule(static)
    for (b = 0; b < B; ++b) {
        REAL *zero = (REAL *)calloc(n, sizeof(REAL));
        const REAL *hstart = h0 ? h0 + (size_t)b * n : zero;
        int l;
        for (l = 0; l < L; ++l)
            oracle_cell_step(cell, H, params, hstart, u + ((size_t)b * L + l) * G * H,
                             h + ((size_t)b * L + l) * n);
        free(zero);
    }

    *iters = 0;
    status = tol < 0 ? ST_OK : ST_NOT_CONVERGED;
    for (k = 1; k <= max_iter; ++k) {
        REAL *mb = (REAL *)calloc((size_t)B, sizeof(REAL));
        REAL m = 0;
#pragma omp parallel for schedule(static)
        for (b = 0; b < B; ++b) {
            REAL *zero = (REAL *)calloc(n, sizeof(REAL));
            REAL *J = (REAL *)malloc(sizeof(REAL) * js * L);
            REAL *r = (REAL *)malloc(sizeof(REAL) * n * L);
            REAL *d = (REAL *)malloc(sizeof(REAL) * n * L);
            REAL *hb = h + (size_t)b * L * n;
            REAL mm = 0;
            int l;
            size_t j;
            for (l = 0; l < L; ++l) {
                const REAL *hp = l == 0 ? (h0 ? h0 + (size_t)b * n : zero) : hb + (size_t)(l - 1) * n;
                const REAL *ul = u + ((size_t)b * L + l) * G * H;
                oracle_cell_step(cell, H, params, hp, ul, r + (size_t)l * n);
                for (j = 0; j < n; ++j) r[(size_t)l * n + j] -= hb[(size_t)l * n + j];
                oracle_cell_jacobian(cell, H, params, hp, ul, J + (size_t)l * js);
                if (diag_only) jac_keep_diagonal(kind, H, J + (size_t)l * js);
            }
            oracle_forward_substitution(kind, L, H, J, r, d);
            for (j = 0; j < n * (size_t)L; ++j) {
                hb[j] += d[j];
                mm = nanmax(mm, (REAL)fabs((double)d[j]));
            }
            mb[b] = mm;
            free(zero); free(J); free(r); free(d);
        }
        for (b = 0; b < B; ++b) m = nanmax(m, mb[b]);
        free(mb);
        *iters = k;
        if (trace) trace[k - 1] = m;
        if (!(m - m == 0)) { status = ST_NONFINITE; break; }   /* inf or nan */
        if (tol >= 0 && m <= tol) { status = ST_OK; break; }
    }
    return status;
}

int oracle_newton(int cell, int B, int L, int H, const REAL *params, const REAL *u, const REAL *h0,
                  REAL tol, int max_iter, REAL *h, int *iters, REAL *trace)
{
    return newton_impl(cell, B, L, H, params, u, h0, tol, max_iter, h, iters, trace, 0);
}

int oracle_newton_diag(int cell, int B, int L, int H, const REAL *params, const REAL *u, const REAL *h0,
                       REAL tol, int max_iter, REAL *h, int *iters, REAL *trace)
{
    return newton_impl(cell, B, L, H, params, u, h0, tol, max_iter, h, iters, trace, 1);
}

/* ----------------------------------------------------------------- backward */

/* Eq. (6): with lam_L = g_L, for l = L..1
 *     (step-local chain rule through f at (h_{l-1}, u_l) with incoming lam_l)
 *     du_l = (df/du_l)^T lam_l,  dparams += (df/dparams)^T lam_l,
 *     lam_{l-1} = J_l^T lam_l + g_{l-1}
 * h is the forward result; dh0 (or NULL) receives J_1^T lam_1.
 * The step-local derivatives are reverse-mode differentiation of the cell
 * written out by hand; the paper obtains them from autograd. */
void oracle_backward(int cell, int B, int L, int H, const REAL *params, const REAL *u,
                     const REAL *h0, const REAL *h, const REAL *g, REAL *du, REAL *dparams, REAL *dh0)
{
    const int G = oracle_gates(cell), S = oracle_state(cell);
    const size_t n = (size_t)S * H, np = param_count(cell, H);
    REAL *dpb = (REAL *)calloc(np * (size_t)B, sizeof(REAL));
    int b;
    size_t q;
#pragma omp parallel for schedule(static)
    for (b = 0; b < B; ++b) {
        REAL *zero = (REAL *)calloc(n, sizeof(REAL));
        REAL *lam = (REAL *)malloc(sizeof(REAL) * n), *lprev = (REAL *)malloc(sizeof(REAL) * n);
        REAL *dp = dpb + (size_t)b * np;
        int l, j;
        memcpy(lam, g + ((size_t)b * L + (L - 1)) * n, sizeof(REAL) * n);
        for (l = L - 1; l >= 0; --l) {
            const REAL *hp = l == 0 ? (h0 ? h0 + (size_t)b * n : zero) : h + ((size_t)b * L + (l - 1)) * n;
            const REAL *ul = u + ((size_t)b * L + l) * G * H;
            REAL *dul = du + ((size_t)b * L + l) * G * H;
            if (cell == CELL_GRU_DIAG) {
                const REAL *a = params, *bb = params + 3 * H;
                for (j = 0; j < H; ++j) {
                    REAL hh = hp[j], lm = lam[j];
                    REAL z = sigmoid(a[0 * H + j] * hh + ul[0 * H + j] + bb[0 * H + j]);
                    REAL r = sigmoid(a[1 * H + j] * hh + ul[1 * H + j] + bb[1 * H + j]);
                    REAL c = tanh_r(a[2 * H + j] * (r * hh) + ul[2 * H + j] + bb[2 * H + j]);
                    /* h' = (1-z) h + z c */
                    REAL d_z = lm * (c - hh), d_c = lm * z, d_h = lm * ((REAL)1 - z);
                    REAL d_pc = d_c * ((REAL)1 - c * c);          /* through tanh */
                    REAL d_rh = d_pc * a[2 * H + j];              /* through a_c (r h) */
                    REAL d_r = d_rh * hh, d_pr, d_pz;
                    d_h += d_rh * r;
                    d_pr = d_r * r * ((REAL)1 - r);               /* through sigmoid */
                    d_h += d_pr * a[1 * H + j];
                    d_pz = d_z * z * ((REAL)1 - z);
                    d_h += d_pz * a[0 * H + j];
                    dul[0 * H + j] = d_pz; dul[1 * H + j] = d_pr; dul[2 * H + j] = d_pc;
                    dp[0 * H + j] += d_pz * hh; dp[1 * H + j] += d_pr * hh; dp[2 * H + j] += d_pc * (r * hh);
                    dp[3 * H + j] += d_pz; dp[4 * H + j] += d_pr; dp[5 * H + j] += d_pc;
                    lprev[j] = d_h;
                }
            } else if (cell == CELL_LSTM_DIAG) {
                const REAL *w = params, *bb = params + 4 * H;
                for (j = 0; j < H; ++j) {
                    REAL c = hp[j], hh = hp[H + j], lc = lam[j], lh = lam[H + j];
                    REAL i = sigmoid(w[0 * H + j] * hh + ul[0 * H + j] + bb[0 * H + j]);
                    REAL f = sigmoid(w[1 * H + j] * hh + ul[1 * H + j] + bb[1 * H + j]);
                    REAL o = sigmoid(w[2 * H + j] * hh + ul[2 * H + j] + bb[2 * H + j]);
                    REAL gg = tanh_r(w[3 * H + j] * hh + ul[3 * H + j] + bb[3 * H + j]);
                    REAL t = tanh_r(f * c + i * gg);
                    /* h' = o t,  c' = f c + i g */
                    REAL d_o = lh * t, d_cn = lc + lh * o * ((REAL)1 - t * t);
                    REAL d_f = d_cn * c, d_i = d_cn * gg, d_g = d_cn * i;
                    REAL d_pi = d_i * i * ((REAL)1 - i), d_pf = d_f * f * ((REAL)1 - f);
                    REAL d_po = d_o * o * ((REAL)1 - o), d_pg = d_g * ((REAL)1 - gg * gg);
                    dul[0 * H + j] = d_pi; dul[1 * H + j] = d_pf; dul[2 * H + j] = d_po; dul[3 * H + j] = d_pg;
                    dp[0 * H + j] += d_pi * hh; dp[1 * H + j] += d_pf * hh;
                    dp[2 * H + j] += d_po * hh; dp[3 * H + j] += d_pg * hh;
                    dp[4 * H + j] += d_pi; dp[5 * H + j] += d_pf; dp[6 * H + j] += d_po; dp[7 * H + j] += d_pg;
                    lprev[j] = d_cn * f;
                    lprev[H + j] = d_pi * w[0 * H + j] + d_pf * w[1 * H + j] + d_po * w[2 * H + j]
                                 + d_pg * w[3 * H + j];
                }
            } else if (cell == CELL_PARALSTM_DIAG) {
                const REAL *af = params, *az = params + H, *ao = params + 2 * H, *cf = params + 3 * H,
                           *co = params + 4 * H, *bf = params + 5 * H, *bz = params + 6 * H, *bo = params + 7 * H;
                for (j = 0; j < H; ++j) {
                    REAL c = hp[j], hh = hp[H + j], lc = lam[j], lh = lam[H + j];
                    REAL f = sigmoid(af[j] * hh + ul[0 * H + j] + cf[j] * c + bf[j]);
                    REAL z = tanh_r(az[j] * hh + ul[1 * H + j] + bz[j]);
                    REAL cn = f * c + ((REAL)1 - f) * z;
                    REAL o = sigmoid(ao[j] * hh + ul[2 * H + j] + co[j] * cn + bo[j]);
                    REAL t = tanh_r(cn);
                    /* h' = o t;  o reads the new c through its peephole */
                    REAL d_o = lh * t;
                    REAL d_po = d_o * o * ((REAL)1 - o);
                    REAL d_cn = lc + lh * o * ((REAL)1 - t * t) + d_po * co[j];
                    /* c' = f c + (1 - f) z */
                    REAL d_f = d_cn * (c - z), d_z = d_cn * ((REAL)1 - f);
                    REAL d_pf = d_f * f * ((REAL)1 - f), d_pz = d_z * ((REAL)1 - z * z);
                    dul[0 * H + j] = d_pf; dul[1 * H + j] = d_pz; dul[2 * H + j] = d_po;
                    dp[0 * H + j] += d_pf * hh; dp[1 * H + j] += d_pz * hh; dp[2 * H + j] += d_po * hh;
                    dp[3 * H + j] += d_pf * c;  dp[4 * H + j] += d_po * cn;
                    dp[5 * H + j] += d_pf; dp[6 * H + j] += d_pz; dp[7 * H + j] += d_po;
                    lprev[j] = d_cn * f + d_pf * cf[j];
                    lprev[H + j] = d_pf * af[j] + d_pz * az[j] + d_po * ao[j];
                }
            } else if (is_gru_nl(cell)) {
                const int nu = ((cell - CELL_GRU_NL) >> 4) & 3, nr = ((cell - CELL_GRU_NL) >> 2) & 3,
                          ns = (cell - CELL_GRU_NL) & 3;
                const REAL *a = params, *bb = params + 3 * H;
                for (j = 0; j < H; ++j) {
                    REAL hh = hp[j], lm = lam[j];
                    REAL xz = a[0 * H + j] * hh + ul[0 * H + j] + bb[0 * H + j];
                    REAL xr = a[1 * H + j] * hh + ul[1 * H + j] + bb[1 * H + j];
                    REAL z = nl_f(nu, xz), r = nl_f(nr, xr);
                    REAL xc = a[2 * H + j] * (r * hh) + ul[2 * H + j] + bb[2 * H + j];
                    REAL c = nl_f(ns, xc);
                    /* h' = (1-z) h + z c, taken apart from the output backwards */
                    REAL d_z = lm * (c - hh), d_c = lm * z, d_h = lm * ((REAL)1 - z);
                    REAL d_pc = d_c * nl_d(ns, xc);
                    REAL d_rh = d_pc * a[2 * H + j];
                    REAL d_r = d_rh * hh, d_pr, d_pz;
                    d_h += d_rh * r;
                    d_pr = d_r * nl_d(nr, xr);
                    d_h += d_pr * a[1 * H + j];
                    d_pz = d_z * nl_d(nu, xz);
                    d_h += d_pz * a[0 * H + j];
                    dul[0 * H + j] = d_pz; dul[1 * H + j] = d_pr; dul[2 * H + j] = d_pc;
                    dp[0 * H + j] += d_pz * hh; dp[1 * H + j] += d_pr * hh; dp[2 * H + j] += d_pc * (r * hh);
                    dp[3 * H + j] += d_pz; dp[4 * H + j] += d_pr; dp[5 * H + j] += d_pc;
                    lprev[j] = d_h;
                }
            } else if (cell == CELL_ROT_TANH) {
                const REAL *a = params, *bb = params + H;
                for (j = 0; j < H; ++j) {
                    REAL p = hp[j], q = hp[H + j];
                    REAL t1 = tanh_r(a[j] * p - bb[j] * q + ul[j]), t2 = tanh_r(bb[j] * p + a[j] * q + ul[H + j]);
                    REAL d1 = lam[j] * ((REAL)1 - t1 * t1), d2 = lam[H + j] * ((REAL)1 - t2 * t2);
                    dul[j] = d1; dul[H + j] = d2;
                    dp[j] += d1 * p + d2 * q;
                    dp[H + j] += -d1 * q + d2 * p;
                    lprev[j] = a[j] * d1 + bb[j] * d2;
                    lprev[H + j] = -bb[j] * d1 + a[j] * d2;
                }
            } else if (mix_dim(cell)) {
                const int N = mix_dim(cell);
                int a, c;
                for (j = 0; j < H; ++j) {
                    REAL d[4];
                    for (a = 0; a < N; ++a) {
                        REAL s = ul[a * H + j], t;
                        for (c = 0; c < N; ++c) s += params[(N * a + c) * H + j] * hp[c * H + j];
                        t = tanh_r(s);
                        d[a] = lam[a * H + j] * ((REAL)1 - t * t);              /* through tanh */
                        dul[a * H + j] = d[a];
                        for (c = 0; c < N; ++c) dp[(N * a + c) * H + j] += d[a] * hp[c * H + j];
                    }
                    for (c = 0; c < N; ++c) {
                        REAL s = params[c * H + j] * d[0];
                        for (a = 1; a < N; ++a) s += params[(N * a + c) * H + j] * d[a];
                        lprev[c * H + j] = s;
                    }
                }
            } else if (cell == CELL_TANH_DENSE) {
                const REAL *hl = h + ((size_t)b * L + l) * n;
                int i;
                for (j = 0; j < H; ++j) lprev[j] = 0;
                for (i = 0; i < H; ++i) {
                    REAL d_pre = lam[i] * ((REAL)1 - hl[i] * hl[i]);   /* h_l = tanh(pre) */
                    dul[i] = d_pre;
                    for (j = 0; j < H; ++j) {
                        dp[(size_t)i * H + j] += d_pre * hp[j];
                        lprev[j] += params[(size_t)i * H + j] * d_pre;
                    }
                }
            } else {
                for (j = 0; j < H; ++j) {
                    dul[j] = lam[j];
                    dp[j] += lam[j] * hp[j];
                    dp[H + j] += lam[j];
                    lprev[j] = params[j] * lam[j];
                }
            }
            if (l > 0) {
                const REAL *gp = g + ((size_t)b * L + (l - 1)) * n;
                for (j = 0; j < (int)n; ++j) lam[j] = lprev[j] + gp[j];
            } else if (dh0) {
                memcpy(dh0 + (size_t)b * n, lprev, sizeof(REAL) * n);
            }
        }
        free(zero); free(lam); free(lprev);
    }
    for (q = 0; q < np; ++q) {
        REAL s = 0;
        for (b = 0; b < B; ++b) s += dpb[(size_t)b * np + q];
        dparams[q] = s;
    }
    free(dpb);
}

/* ------------------------------------------------------- input projection */

/* The gate pre-activations that feed the recurrence: for every row m = (b, l),
 * gate g and channel h,
 *     u[m][g][h] = sum_j Wx[g][h][j] x[m][head(h) * dh + j] + bias[g][h],
 * dh = H / n_heads, head(h) = h / dh: each head's dh outputs read only that
 * head's dh inputs (App. C), i.e. the input matrix B_g of Eq. (7a) / (7b) is
 * block diagonal with n_heads blocks; n_heads = 1 is a full matrix.
 * x [rows][H], Wx [G][H][dh], bias [G][H] or NULL, u [rows][G][H]. */
void oracle_input_projection(int rows, int H, int G, int n_heads, const REAL *x, const REAL *Wx,
                             const REAL *bias, REAL *u)
{
    const int dh = H / n_heads;
    int m;
#pragma omp parallel for schedule(static)
    for (m = 0; m < rows; ++m) {
        int g, h, j;
        for (g = 0; g < G; ++g)
            for (h = 0; h < H; ++h) {
                const REAL *w = Wx + ((size_t)g * H + h) * dh;
                const REAL *xr = x + (size_t)m * H + (size_t)(h / dh) * dh;
                REAL s = bias ? bias[(size_t)g * H + h] : (REAL)0;
                for (j = 0; j < dh; ++j) s += w[j] * xr[j];
                u[((size_t)m * G + g) * H + h] = s;
            }
    }
}

/* Derivatives of the map above for an incoming du = dL/du:
 *     dx[m][head*dh + j]   = sum_g sum_{h in head} du[m][g][h] Wx[g][h][j]
 *     dWx[g][h][j]         = sum_m du[m][g][h] x[m][head(h)*dh + j]
 *     dbias[g][h]          = sum_m du[m][g][h]
 * dbias may be NULL. */
void oracle_input_projection_backward(int rows, int H, int G, int n_heads, const REAL *x, const REAL *Wx,
                                      const REAL *du, REAL *dx, REAL *dWx, REAL *dbias)
{
    const int dh = H / n_heads;
    int m, q;
#pragma omp parallel for schedule(static)
    for (m = 0; m < rows; ++m) {
        int g, h, j;
        REAL *dxr = dx + (size_t)m * H;
        for (j = 0; j < H; ++j) dxr[j] = 0;
        for (g = 0; g < G; ++g)
            for (h = 0; h < H; ++h) {
                const REAL d = du[((size_t)m * G + g) * H + h];
                const REAL *w = Wx + ((size_t)g * H + h) * dh;
                REAL *dxh = dxr + (size_t)(h / dh) * dh;
                for (j = 0; j < dh; ++j) dxh[j] += d * w[j];
            }
    }
#pragma omp parallel for schedule(static)
    for (q = 0; q < G * H; ++q) {
        const int h = q % H;
        int j;
        REAL *dw = dWx + (size_t)q * dh;
        REAL sb = 0;
        for (j = 0; j < dh; ++j) dw[j] = 0;
        for (m = 0; m < rows; ++m) {
            const REAL d = du[(size_t)m * G * H + q];
            const REAL *xr = x + (size_t)m * H + (size_t)(h / dh) * dh;
            for (j = 0; j < dh; ++j) dw[j] += d * xr[j];
            sb += d;
        }
        if (dbias) dbias[q] = sb;
    }
}
