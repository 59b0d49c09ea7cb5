"""Pins for the CPU oracle: each check compares an oracle routine with
something the paper or plain mathematics fixes, never with the routine
itself.  All fp64, tiny sizes, no GPU.

Citations are to ParaRNN (arXiv 2510.21450) by section / equation.
"""
import itertools
import math

import numpy as np
import pytest

NL_CELLS = ["gru_nl:tanh,softsign,identity", "gru_nl:sigmoid,sigmoid,softsign", "gru_nl:softsign,tanh,sigmoid"]
DIAG_CELLS = ["gru_diag", "linear_diag"] + NL_CELLS
BLOCK2_CELLS = ["lstm_diag", "paralstm_diag", "rot_tanh"]
BLOCK3_CELLS = ["tri_tanh", "quad_tanh"]          # 3x3 and 4x4 blocks
ALL_CELLS = ["gru_diag", "lstm_diag", "tanh_dense", "linear_diag", "paralstm_diag", "rot_tanh", "tri_tanh", "quad_tanh"] + NL_CELLS


def sig(x):
    return 1.0 / (1.0 + math.exp(-x))


def rand_params(oracle, cell, H, rng, bound=0.9, bias=True):
    G, S = oracle.dims(cell)
    if cell == "tanh_dense":
        return rng.normal(0, 0.8 / math.sqrt(H), (H, H))
    if cell == "paralstm_diag":          # a_f, a_z, a_o, c_f, c_o, then biases b_f, b_z, b_o
        p = np.zeros((8, H))
        p[:5] = rng.uniform(-bound, bound, (5, H))
        if bias:
            p[5:] = rng.normal(0, 0.3, (3, H))
        return p
    if cell in ("tri_tanh", "quad_tanh"):    # the per-channel N x N matrix, [N][N][H] as N*N rows
        return rng.uniform(-bound / 2, bound / 2, (S * S, H)) * (1.0 if S == 3 else 0.75)
    if cell == "rot_tanh":               # a, b of the per-channel rotation-scaling
        return rng.uniform(-bound / 1.5, bound / 1.5, (2, H))
    p = np.zeros((2, G, H))
    p[0] = rng.uniform(-bound, bound, (G, H))
    if bias:
        p[1] = rng.normal(0, 0.3, (G, H))
    return p


def rand_problem(oracle, cell, B, L, H, seed, bound=0.9, h0=True):
    rng = np.random.default_rng(seed)
    G, S = oracle.dims(cell)
    params = rand_params(oracle, cell, H, rng, bound)
    u = rng.normal(0, 1, (B, L, G, H))
    h0v = rng.normal(0, 0.3, (B, S, H)) if h0 else None
    return params, u, h0v


# ---------------------------------------------------------------- cell forward

def test_gru_step_hand_values(oracle_mod):
    """Eq. (7a) with Eq. (9), typed out for one channel with python's math."""
    o = oracle_mod
    az, ar, ac, bz, br, bc = 0.7, -0.4, 0.55, 0.1, -0.2, 0.05
    uz, ur, uc, h = 0.3, -1.1, 0.8, 0.6
    z = sig(az * h + uz + bz)
    r = sig(ar * h + ur + br)
    c = math.tanh(ac * (r * h) + uc + bc)
    want = (1 - z) * h + z * c
    p = np.array([[[az], [ar], [ac]], [[bz], [br], [bc]]])
    got = o.cell_step("gru_diag", p, [[h]], [[uz], [ur], [uc]])
    assert got.shape == (1, 1)
    assert abs(got[0, 0] - want) < 1e-15
    # all weights, biases and inputs zero: z = r = 1/2, c = 0 -> h' = h/2
    got = o.cell_step("gru_diag", np.zeros((2, 3, 1)), [[0.8]], np.zeros((3, 1)))
    assert abs(got[0, 0] - 0.4) < 1e-16


def test_gru_channels_do_not_mix_and_gate_order(oracle_mod):
    """Eq. (9): d_h independent 1-D cells; gate order (z, r, c)."""
    o = oracle_mod
    rng = np.random.default_rng(0)
    H = 5
    p = rand_params(o, "gru_diag", H, rng)
    hp = rng.normal(0, 0.5, (1, H))
    u = rng.normal(0, 1, (3, H))
    full = o.cell_step("gru_diag", p, hp, u)
    for j in range(H):
        one = o.cell_step("gru_diag", p[:, :, j:j + 1], hp[:, j:j + 1], u[:, j:j + 1])
        assert one[0, 0] == full[0, j]
    # a huge positive u_z forces z -> 1, h' -> c = tanh(a_c r h + u_c): identifies slot 0 as z
    u2 = u.copy(); u2[0] = 50.0
    got = o.cell_step("gru_diag", p, hp, u2)
    r = 1 / (1 + np.exp(-(p[0, 1] * hp[0] + u2[1] + p[1, 1])))
    want = np.tanh(p[0, 2] * r * hp[0] + u2[2] + p[1, 2])
    assert np.allclose(got[0], want, atol=1e-14)
    # a hugely negative u_z forces z -> 0, h' -> h
    u2[0] = -50.0
    assert np.allclose(o.cell_step("gru_diag", p, hp, u2)[0], hp[0], atol=1e-14)


def test_lstm_step_hand_values(oracle_mod):
    """The benchmark's LSTM-style cell: i,f,o = sigmoid(w h + u + b),
    g = tanh(.), c' = f c + i g, h' = o tanh(c'); state order (c, h)."""
    o = oracle_mod
    w = [0.3, -0.6, 0.8, 0.45]
    b = [0.0, 1.0, 0.0, 0.0]
    u = [0.2, -0.3, 0.9, -1.2]
    c, h = 0.7, -0.35
    i = sig(w[0] * h + u[0] + b[0]); f = sig(w[1] * h + u[1] + b[1])
    oo = sig(w[2] * h + u[2] + b[2]); g = math.tanh(w[3] * h + u[3] + b[3])
    cn = f * c + i * g
    hn = oo * math.tanh(cn)
    p = np.array([[[x] for x in w], [[x] for x in b]])
    got = o.cell_step("lstm_diag", p, [[c], [h]], [[x] for x in u])
    assert abs(got[0, 0] - cn) < 1e-15 and abs(got[1, 0] - hn) < 1e-15
    # w = 0, u = 0, b_f = 1: f = sigmoid(1), i = o = 1/2, g = 0
    p0 = np.zeros((2, 4, 1)); p0[1, 1] = 1.0
    got = o.cell_step("lstm_diag", p0, [[c], [h]], np.zeros((4, 1)))
    assert abs(got[0, 0] - sig(1.0) * c) < 1e-15
    assert abs(got[1, 0] - 0.5 * math.tanh(sig(1.0) * c)) < 1e-15


def test_paralstm_step_hand_values(oracle_mod):
    """Eq. (7b) with Eq. (9): f = sig(a_f h + u_f + c_f c + b_f), z = tanh(a_z h + u_z + b_z),
    c' = f c + (1-f) z, o = sig(a_o h + u_o + c_o c' + b_o) (peephole on the NEW c), h' = o tanh(c')."""
    o = oracle_mod
    af, az, ao, cf, co, bf, bz, bo = 0.4, -0.7, 0.6, 0.5, -0.3, 0.2, -0.1, 0.05
    uf, uz, uo, c, h = 0.3, -0.8, 0.9, 0.7, -0.45
    f = sig(af * h + uf + cf * c + bf)
    z = math.tanh(az * h + uz + bz)
    cn = f * c + (1 - f) * z
    oo = sig(ao * h + uo + co * cn + bo)
    hn = oo * math.tanh(cn)
    p = np.array([[x] for x in (af, az, ao, cf, co, bf, bz, bo)])
    got = o.cell_step("paralstm_diag", p, [[c], [h]], [[uf], [uz], [uo]])
    assert abs(got[0, 0] - cn) < 1e-15 and abs(got[1, 0] - hn) < 1e-15
    # the o peephole reads the new c: with a_o = u_o = b_o = 0 and a huge c_o the gate saturates by sign(c')
    p2 = p.copy(); p2[2] = 0; p2[7] = 0; p2[4] = 1e4
    got = o.cell_step("paralstm_diag", p2, [[c], [h]], [[uf], [uz], [0.0]])
    assert abs(got[1, 0] - (math.tanh(cn) if cn > 0 else 0.0)) < 1e-12
    # f -> 1 keeps c (CIFG: the input gate is 1 - f)
    got = o.cell_step("paralstm_diag", p, [[c], [h]], [[60.0], [uz], [uo]])
    assert abs(got[0, 0] - c) < 1e-14


def test_dense_step_is_tanh_of_matvec(oracle_mod):
    o = oracle_mod
    rng = np.random.default_rng(1)
    H = 6
    W = rng.normal(0, 0.4, (H, H))
    hp = rng.normal(0, 0.5, (1, H)); u = rng.normal(0, 1, (1, H))
    got = o.cell_step("tanh_dense", W, hp, u)
    assert np.allclose(got[0], np.tanh(W @ hp[0] + u[0]), atol=1e-15)
    # row-major W[i][j] multiplies h_j: a matrix with a single entry tells rows from columns
    W1 = np.zeros((H, H)); W1[1, 4] = 0.9
    got = o.cell_step("tanh_dense", W1, hp, np.zeros((1, H)))
    want = np.zeros(H); want[1] = math.tanh(0.9 * hp[0, 4])
    assert np.allclose(got[0], want, atol=1e-16)


def test_bounded_state_invariant(oracle_mod):
    """GRU: h' is a convex combination of h and tanh(.) so |h_l| < 1 when
    |h_0| <= 1; LSTM: |h_l| < 1 since h' = o tanh(c')."""
    o = oracle_mod
    for cell in ("gru_diag", "lstm_diag", "paralstm_diag"):
        params, u, h0 = rand_problem(o, cell, 2, 200, 7, seed=3)
        u *= 3.0
        h = o.seq_unroll(cell, params, u, None)
        hh = h[:, :, -1, :]
        assert np.all(np.abs(hh) < 1.0)


# ------------------------------------------------------------------ Jacobians

@pytest.mark.parametrize("cell", ALL_CELLS)
def test_jacobian_matches_central_differences(oracle_mod, cell):
    """Eq. (8a) (and the 2x2 / dense analogues) against finite differences of f."""
    o = oracle_mod
    rng = np.random.default_rng(11)
    H = 4
    G, S = o.dims(cell)
    params = rand_params(o, cell, H, rng)
    hp = rng.normal(0, 0.6, (S, H)); u = rng.normal(0, 1, (G, H))
    J = o.cell_jacobian(cell, params, hp, u)
    eps = 1e-6
    n = S * H
    Jfd = np.zeros((n, n))
    for q in range(n):
        e = np.zeros(n); e[q] = eps
        fp = o.cell_step(cell, params, hp + e.reshape(S, H), u).ravel()
        fm = o.cell_step(cell, params, hp - e.reshape(S, H), u).ravel()
        Jfd[:, q] = (fp - fm) / (2 * eps)
    if cell in DIAG_CELLS:
        Jfull = np.diag(J)
    elif cell in BLOCK2_CELLS + BLOCK3_CELLS:
        Jfull = np.zeros((n, n))
        for p_, q_ in itertools.product(range(S), range(S)):
            Jfull[p_ * H:(p_ + 1) * H, q_ * H:(q_ + 1) * H] = np.diag(J[p_, q_])
    else:
        Jfull = J
    assert np.max(np.abs(Jfull - Jfd)) < 1e-8


def test_gru_jacobian_uses_candidate_minus_previous_state(oracle_mod):
    """The (c - h_{l-1}) factor of Eq. (8a): with a_r = a_c = 0 the Jacobian is
    (1-z) + (c-h) z(1-z) a_z with c = tanh(u_c) free of h."""
    o = oracle_mod
    az, h, uz, uc = 0.8, 0.3, 0.4, -0.7
    p = np.zeros((2, 3, 1)); p[0, 0, 0] = az
    z = sig(az * h + uz); c = math.tanh(uc)
    want = (1 - z) + (c - h) * z * (1 - z) * az
    got = o.cell_jacobian("gru_diag", p, [[h]], [[uz], [0.0], [uc]])
    assert abs(got[0] - want) < 1e-15


# ---------------------------------------------------------------- linear solves

def _rand_system(kind, L, H, rng, scale=0.9):
    if kind == "diag":
        return rng.uniform(-scale, scale, (L, H)), rng.normal(0, 1, (L, H))
    if kind == "block2":
        return rng.uniform(-scale, scale, (L, 2, 2, H)), rng.normal(0, 1, (L, 2, H))
    if kind in ("block3", "block4"):
        N = int(kind[-1])
        return rng.uniform(-scale / 1.5, scale / 1.5, (L, N, N, H)) * 3 / N, rng.normal(0, 1, (L, N, H))
    return rng.normal(0, scale / math.sqrt(H), (L, H, H)), rng.normal(0, 1, (L, H))


def _dense_view(kind, J, H):
    """Expand any Jacobian layout into full (S*H)x(S*H) matrices."""
    L = J.shape[0]
    if kind == "diag":
        return np.stack([np.diag(J[l]) for l in range(L)])
    if kind in ("block2", "block3", "block4"):
        S = J.shape[1]
        out = np.zeros((L, S * H, S * H))
        for l in range(L):
            for p_, q_ in itertools.product(range(S), range(S)):
                out[l, p_ * H:(p_ + 1) * H, q_ * H:(q_ + 1) * H] = np.diag(J[l, p_, q_])
        return out
    return J


@pytest.mark.parametrize("kind", ["diag", "block2", "block3", "block4", "dense"])
def test_forward_substitution_equals_unrolled_sum(oracle_mod, kind):
    """Eq. (5): delta_l = sum_{s<=l} (J_l J_{l-1} ... J_{s+1}) r_s, by brute force."""
    o = oracle_mod
    rng = np.random.default_rng(5)
    H = 3
    for L in range(1, 9):
        J, r = _rand_system(kind, L, H, rng)
        got = o.forward_substitution(kind, J, r).reshape(L, -1)
        Jd = _dense_view(kind, J, H); rv = r.reshape(L, -1)
        for l in range(L):
            want = np.zeros(rv.shape[1])
            for s in range(l + 1):
                prod = np.eye(rv.shape[1])
                for t in range(l, s, -1):          # J_l J_{l-1} ... J_{s+1}
                    prod = prod @ Jd[t]
                want += prod @ rv[s]
            assert np.allclose(got[l], want, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("kind", ["diag", "block2", "block3", "block4", "dense"])
def test_parallel_reduce_equals_dense_solve(oracle_mod, kind):
    """Alg. 1b solves the block bi-diagonal system of Eq. (3): compare with a
    dense LAPACK solve of (I - subdiag(J)) delta = r, for every L up to 70
    (non powers of two included) and also with forward substitution."""
    o = oracle_mod
    rng = np.random.default_rng(6)
    H = 2
    for L in list(range(1, 34)) + [47, 64, 65, 70]:
        J, r = _rand_system(kind, L, H, rng)
        Jd = _dense_view(kind, J, H); rv = r.reshape(L, -1)
        n = rv.shape[1]
        M = np.eye(L * n)
        for l in range(1, L):
            M[l * n:(l + 1) * n, (l - 1) * n:l * n] = -Jd[l]
        want = np.linalg.solve(M, rv.ravel()).reshape(L, n)
        got_pr = o.parallel_reduce(kind, J, r).reshape(L, n)
        got_fs = o.forward_substitution(kind, J, r).reshape(L, n)
        assert np.allclose(got_pr, want, rtol=1e-10, atol=1e-11)
        assert np.allclose(got_fs, want, rtol=1e-10, atol=1e-11)


def test_linear_cell_closed_form(oracle_mod):
    """Footnote of Sec. 2: f = a h + u.  Constant a, u give the geometric sum
    h_l = a^l h_0 + u (1 - a^l)/(1 - a)."""
    o = oracle_mod
    a, uu, h0, L = 0.83, 0.4, -0.6, 40
    p = np.zeros((2, 1, 1)); p[0, 0, 0] = a
    u = np.full((1, L, 1, 1), uu)
    h = o.seq_unroll("linear_diag", p, u, np.array([[[h0]]]))
    for l in range(1, L + 1):
        want = a ** l * h0 + uu * (1 - a ** l) / (1 - a)
        assert abs(h[0, l - 1, 0, 0] - want) < 1e-14


# ----------------------------------------------------------------------- Newton

def test_linear_cell_one_newton_solve_is_exact(oracle_mod):
    """Footnote of Sec. 2: for a linear cell the Jacobian is the transition
    itself and one Newton update recovers the output."""
    o = oracle_mod
    params, u, h0 = rand_problem(o, "linear_diag", 2, 50, 3, seed=8)
    ref = o.seq_unroll("linear_diag", params, u, h0)
    h1, iters, st, tr = o.newton("linear_diag", params, u, h0, tol=-1.0, max_iter=1)
    assert iters == 1 and st == 0
    assert np.max(np.abs(h1 - ref)) < 1e-13
    # with a stopping test a second solve confirms (delta ~ 0): iters == 2
    h2, iters, st, tr = o.newton("linear_diag", params, u, h0, tol=1e-9, max_iter=10)
    assert iters == 2 and st == 0 and tr[1] < 1e-12
    # GRU with a_* = 0 is linear in h (J = 1 - z): same property
    params, u, h0 = rand_problem(o, "gru_diag", 2, 50, 3, seed=9)
    params[0] = 0.0
    ref = o.seq_unroll("gru_diag", params, u, h0)
    h1, iters, st, _ = o.newton("gru_diag", params, u, h0, tol=-1.0, max_iter=1)
    assert np.max(np.abs(h1 - ref)) < 1e-13


@pytest.mark.parametrize("cell", ["gru_diag", "lstm_diag", "tanh_dense", "paralstm_diag", "tri_tanh", "quad_tanh"])
def test_newton_first_k_states_exact_after_k_iterations(oracle_mod, cell):
    """Sec. 2.1: convergence in at most L Newton steps is guaranteed because
    after k solves the first k states equal the sequential result, whatever the
    weights.  Deliberately expansive weights (|a| up to 3)."""
    o = oracle_mod
    B, L, H = 2, 12, 3
    params, u, h0 = rand_problem(o, cell, B, L, H, seed=21, bound=3.0)
    if cell == "tanh_dense":
        params = params * 4.0
    ref = o.seq_unroll(cell, params, u, h0)
    for k in range(0, L + 1):
        hk, iters, st, _ = o.newton(cell, params, u, h0, tol=-1.0, max_iter=k)
        assert iters == k
        # the initial guess f(h0, u_1) is already exact for l = 1, so after k
        # solves states 1..k+1 are exact
        upto = min(L, k + 1)
        assert np.max(np.abs(hk[:, :upto] - ref[:, :upto])) < 1e-11, (cell, k)
    hL, iters, st, _ = o.newton(cell, params, u, h0, tol=-1.0, max_iter=L)
    assert np.max(np.abs(hL - ref)) < 1e-11


@pytest.mark.parametrize("cell", ["gru_diag", "lstm_diag", "tanh_dense", "paralstm_diag", "tri_tanh", "quad_tanh"])
def test_newton_converges_quadratically_to_the_unroll(oracle_mod, cell):
    """App. A: the residual falls to machine precision in a handful of
    iterations; the converged iterate is the sequential result of Eq. (1)."""
    o = oracle_mod
    params, u, h0 = rand_problem(o, cell, 3, 128, 4, seed=31)
    ref = o.seq_unroll(cell, params, u, h0)
    h, iters, st, tr = o.newton(cell, params, u, h0, tol=1e-12, max_iter=64)
    assert st == 0 and iters < 20
    assert np.max(np.abs(h - ref)) < 1e-12
    # quadratic tail: once below 1e-2, each step at least squares the error
    # up to a modest constant
    small = [t for t in tr if t < 1e-2]
    for a, b in zip(small[:-1], small[1:]):
        assert b < 50 * a * a + 1e-14
    # the fixed point does not depend on tol once converged
    h2, it2, _, _ = o.newton(cell, params, u, h0, tol=1e-9, max_iter=64)
    assert it2 <= iters and np.max(np.abs(h2 - ref)) < 1e-9


def test_newton_initial_guess_and_iteration_edge_cases(oracle_mod):
    o = oracle_mod
    params, u, h0 = rand_problem(o, "gru_diag", 2, 9, 3, seed=41)
    # max_iter = 0: h is the initial guess f(h0, u_l) for every l (App. A)
    hg, iters, st, tr = o.newton("gru_diag", params, u, h0, tol=1e-6, max_iter=0)
    assert iters == 0 and st == 1 and len(tr) == 0
    for b in range(2):
        for l in range(9):
            want = o.cell_step("gru_diag", params, h0[b], u[b, l])
            assert np.array_equal(hg[b, l], want)
    # h0 = None means zeros (Sec. 2: h_0 = 0)
    hz, _, _, _ = o.newton("gru_diag", params, u, None, tol=1e-6, max_iter=0)
    hz2, _, _, _ = o.newton("gru_diag", params, u, np.zeros_like(h0), tol=1e-6, max_iter=0)
    assert np.array_equal(hz, hz2)
    # tol < 0: exactly max_iter solves, status OK
    _, iters, st, tr = o.newton("gru_diag", params, u, h0, tol=-1.0, max_iter=7)
    assert iters == 7 and st == 0 and len(tr) == 7
    # L = 1: the guess is exact, the first solve returns delta = 0
    _, iters, st, tr = o.newton("gru_diag", params, u[:, :1], h0, tol=0.0, max_iter=5)
    assert iters == 1 and st == 0 and tr[0] == 0.0
    # not converged: h is the last iterate, iters = max_iter
    _, iters, st, _ = o.newton("gru_diag", params, u, h0, tol=1e-300, max_iter=2)
    assert iters == 2 and st == 1
    # a NaN in the input is reported
    u2 = u.copy(); u2[0, 3, 0, 0] = np.nan
    _, iters, st, _ = o.newton("gru_diag", params, u2, h0, tol=1e-6, max_iter=5)
    assert st == 5 and iters == 1


def test_newton_stops_on_batch_wide_max(oracle_mod):
    """The stopping test takes the max over the whole batch (App. A takes the
    max on batches): solving two sequences together needs as many solves as
    the slower of the two alone."""
    o = oracle_mod
    params, u, h0 = rand_problem(o, "gru_diag", 2, 200, 2, seed=51)
    u[1] *= 3.0
    it = [o.newton("gru_diag", params, u[b:b + 1], h0[b:b + 1], tol=1e-10)[1] for b in range(2)]
    both = o.newton("gru_diag", params, u, h0, tol=1e-10)[1]
    assert both == max(it)


# --------------------------------------------------------------------- backward

@pytest.mark.parametrize("cell", ALL_CELLS)
def test_backward_matches_finite_differences(oracle_mod, cell):
    """Eq. (6) and the step-local gradients against central differences of
    the scalar loss sum(g * h) through the sequential recurrence."""
    o = oracle_mod
    B, L, H = 2, 7, 3
    params, u, h0 = rand_problem(o, cell, B, L, H, seed=61)
    G, S = o.dims(cell)
    rng = np.random.default_rng(62)
    g = rng.normal(0, 1, (B, L, S, H))

    def loss(p, uu, hh0):
        return float(np.sum(g * o.seq_unroll(cell, p, uu, hh0)))

    h = o.seq_unroll(cell, params, u, h0)
    du, dp, dh0 = o.backward(cell, params, u, h0, h, g)
    eps = 1e-6

    def fd(arr, idx, which):
        a1 = arr.copy(); a2 = arr.copy()
        a1[idx] += eps; a2[idx] -= eps
        args1 = {"p": params, "u": u, "h0": h0}; args2 = dict(args1)
        args1[which] = a1; args2[which] = a2
        return (loss(args1["p"], args1["u"], args1["h0"]) - loss(args2["p"], args2["u"], args2["h0"])) / (2 * eps)

    for idx in np.ndindex(*params.shape):
        assert abs(dp[idx] - fd(params, idx, "p")) < 2e-8 * max(1.0, abs(dp[idx])), ("dparams", idx)
    for idx in np.ndindex(*h0.shape):
        assert abs(dh0[idx] - fd(h0, idx, "h0")) < 2e-8 * max(1.0, abs(dh0[idx])), ("dh0", idx)
    for idx in list(np.ndindex(*u.shape))[::5]:
        assert abs(du[idx] - fd(u, idx, "u")) < 2e-8 * max(1.0, abs(du[idx])), ("du", idx)


@pytest.mark.parametrize("cell", ["gru_diag", "lstm_diag", "paralstm_diag"])
def test_backward_dummy_loss_sum_h_squared(oracle_mod, cell):
    """App. B's dummy loss L(h) = sum_l h_l^2, i.e. g_l = 2 h_l."""
    o = oracle_mod
    params, u, h0 = rand_problem(o, cell, 1, 10, 2, seed=71)
    h = o.seq_unroll(cell, params, u, h0)
    du, dp, dh0 = o.backward(cell, params, u, h0, h, 2 * h)
    eps = 1e-6
    for idx in np.ndindex(*h0.shape):
        a1 = h0.copy(); a2 = h0.copy(); a1[idx] += eps; a2[idx] -= eps
        fdv = (np.sum(o.seq_unroll(cell, params, u, a1) ** 2) - np.sum(o.seq_unroll(cell, params, u, a2) ** 2)) / (2 * eps)
        assert abs(dh0[idx] - fdv) < 1e-7


@pytest.mark.parametrize("cell", ["gru_diag", "lstm_diag", "tanh_dense", "paralstm_diag"])
def test_adjoint_identity_between_forward_solve_and_backward(oracle_mod, cell):
    """Eq. (6) is the transpose of the solve of Eq. (3)/(4): for the solution
    operator S of delta_l = J_l delta_{l-1} + r_l and the reverse recurrence
    lam_{l-1} = J_l^T lam_l + g_{l-1},  <g, S r> = <lam, r>.
    lam is recovered from oracle_backward through du of a cell whose df/du is
    known: for the linear cell du = lam; here we use dh0 and the identity on
    J-weighted sums instead, with J from oracle_cell_jacobian."""
    o = oracle_mod
    B, L, H = 1, 9, 3
    params, u, h0 = rand_problem(o, cell, B, L, H, seed=81)
    G, S = o.dims(cell)
    rng = np.random.default_rng(82)
    h = o.seq_unroll(cell, params, u, h0)
    g = rng.normal(0, 1, (B, L, S, H))
    # Jacobians at the converged states
    kind = {"gru_diag": "diag", "lstm_diag": "block2", "paralstm_diag": "block2", "tanh_dense": "dense"}[cell]
    Js = [o.cell_jacobian(cell, params, h0[0] if l == 0 else h[0, l - 1], u[0, l]) for l in range(L)]
    J = np.stack(Js)
    r = rng.normal(0, 1, (L, S, H))
    delta = o.forward_substitution(kind, J, r)
    # lam by the reverse recurrence with explicitly transposed dense matrices
    Jd = _dense_view(kind, J, H)
    lam = np.zeros((L, S * H))
    lam[L - 1] = g[0, L - 1].ravel()
    for l in range(L - 1, 0, -1):
        lam[l - 1] = Jd[l].T @ lam[l] + g[0, l - 1].ravel()
    lhs = float(np.sum(g[0] * delta))
    rhs = float(np.sum(lam * r.reshape(L, -1)))
    assert abs(lhs - rhs) < 1e-11 * max(1.0, abs(lhs))
    # and oracle_backward's dh0 is J_1^T lam_1
    _, _, dh0 = o.backward(cell, params, u, h0, h, g)
    assert np.allclose(dh0[0].ravel(), Jd[0].T @ lam[0], rtol=1e-12, atol=1e-13)


def test_linear_cell_backward_du_is_lambda(oracle_mod):
    """For f = a h + u: du_l = lam_l = sum_{s>=l} a^{s-l} g_s (closed form)."""
    o = oracle_mod
    a, L = 0.7, 12
    p = np.zeros((2, 1, 1)); p[0, 0, 0] = a
    rng = np.random.default_rng(91)
    u = rng.normal(0, 1, (1, L, 1, 1)); g = rng.normal(0, 1, (1, L, 1, 1))
    h = o.seq_unroll("linear_diag", p, u, None)
    du, dp, dh0 = o.backward("linear_diag", p, u, None, h, g)
    for l in range(L):
        want = sum(a ** (s - l) * g[0, s, 0, 0] for s in range(l, L))
        assert abs(du[0, l, 0, 0] - want) < 1e-13
    assert abs(dh0[0, 0, 0] - a * du[0, 0, 0, 0]) < 1e-13
    # bias gradient = sum of lam; weight gradient = sum lam_l h_{l-1}
    assert abs(dp[1, 0, 0] - du.sum()) < 1e-12
    hprev = np.concatenate([[0.0], h[0, :-1, 0, 0]])
    assert abs(dp[0, 0, 0] - np.sum(du[0, :, 0, 0] * hprev)) < 1e-12


# ------------------------------------- selectable nonlinearities, 2x2 example cell

def test_gru_with_default_nonlinearities_is_the_gru(oracle_mod):
    """App. D.3: sigmoid, sigmoid, tanh are the defaults, so the selectable form
    must reproduce Eq. (7a) / (8a) / (6) of the plain GRU exactly."""
    o = oracle_mod
    params, u, h0 = rand_problem(o, "gru_diag", 2, 9, 5, seed=91)
    nl = "gru_nl:sigmoid,sigmoid,tanh"
    assert np.array_equal(o.seq_unroll(nl, params, u, h0), o.seq_unroll("gru_diag", params, u, h0))
    assert np.array_equal(o.cell_jacobian(nl, params, h0[0], u[0, 0]), o.cell_jacobian("gru_diag", params, h0[0], u[0, 0]))
    h = o.seq_unroll("gru_diag", params, u, h0)
    g = np.random.default_rng(92).normal(0, 1, h.shape)
    for a, b in zip(o.backward(nl, params, u, h0, h, g), o.backward("gru_diag", params, u, h0, h, g)):
        assert np.allclose(a, b, rtol=1e-13, atol=1e-15)      # products associate differently


@pytest.mark.parametrize("state_nl", ["identity", "tanh", "softsign"])
def test_gru_state_nonlinearity_alone(oracle_mod, state_nl):
    """With identity update / reset gates held at z = r = 1 (a_z = a_r = 0, u_z = u_r = 1)
    Eq. (7a) collapses to h' = NS(a_c h + u_c + b_c): the linear cell of the Sec. 2
    footnote for identity, the dense tanh cell with a diagonal W for tanh, and
    x / (1 + |x|) with its known values for softsign."""
    o = oracle_mod
    rng = np.random.default_rng(93)
    H, L = 4, 6
    params = np.zeros((2, 3, H)); params[0, 2] = rng.uniform(-0.9, 0.9, H); params[1, 2] = rng.normal(0, 0.3, H)
    u = rng.normal(0, 1, (1, L, 3, H)); u[:, :, :2] = 1.0
    h0 = rng.normal(0, 0.3, (1, 1, H))
    h = o.seq_unroll(f"gru_nl:identity,identity,{state_nl}", params, u, h0)
    if state_nl == "identity":
        lin = np.stack([params[0, 2], params[1, 2]])[:, None, :]
        assert np.allclose(h, o.seq_unroll("linear_diag", lin, u[:, :, 2:3], h0), rtol=0, atol=1e-15)
    elif state_nl == "tanh":
        W = np.diag(params[0, 2])
        ref = o.seq_unroll("tanh_dense", W, u[:, :, 2:3] + params[1, 2], h0)
        assert np.allclose(h, ref, rtol=0, atol=1e-15)
    else:
        pz = np.zeros((2, 3, 1))
        for x, y in ((0.0, 0.0), (1.0, 0.5), (-1.0, -0.5), (3.0, 0.75), (-7.0, -0.875)):
            uu = np.array([1.0, 1.0, x]).reshape(1, 1, 3, 1)
            assert o.seq_unroll("gru_nl:identity,identity,softsign", pz, uu, None)[0, 0, 0, 0] == y


def test_gru_gate_nonlinearities_reach_the_right_gates(oracle_mod):
    """Which of the three selectors acts on which gate: with a_* = 0 the step is
    h' = (1 - z) h + z c with z = NU(u_z), c = NS(u_c) and r unused; with a_c = 1,
    u_c = 0 and identity state nonlinearity c = NR(u_r) h."""
    o = oracle_mod
    pz = np.zeros((2, 3, 1))
    h0 = np.full((1, 1, 1), 0.25)
    uu = np.array([1.0, -7.0, 3.0]).reshape(1, 1, 3, 1)
    # z = softsign(1) = 1/2, c = softsign(3) = 3/4 -> h' = (0.25 + 0.75) / 2
    assert o.seq_unroll("gru_nl:softsign,sigmoid,softsign", pz, uu, h0)[0, 0, 0, 0] == 0.5
    # z = identity(1) = 1 -> h' = c = identity(3)
    assert o.seq_unroll("gru_nl:identity,tanh,identity", pz, uu, h0)[0, 0, 0, 0] == 3.0
    pc = pz.copy(); pc[0, 2, 0] = 1.0
    uu = np.array([1.0, -7.0, 0.0]).reshape(1, 1, 3, 1)
    # z = 1, c = a_c * softsign(-7) * h = -7/8 * 1/4
    assert o.seq_unroll("gru_nl:identity,softsign,identity", pc, uu, h0)[0, 0, 0, 0] == -0.875 * 0.25


def test_rot_tanh_is_the_dense_cell_with_a_2x2_matrix(oracle_mod):
    """One channel of the 2x2 example cell is h' = tanh(W h + u) with
    W = [[a, -b], [b, a]]: step, Jacobian, Newton solve and backward must agree
    with the dense cell at H = 2 (dL/da = dW_00 + dW_11, dL/db = dW_10 - dW_01)."""
    o = oracle_mod
    rng = np.random.default_rng(95)
    a, b = 0.55, -0.4
    L = 12
    W = np.array([[a, -b], [b, a]])
    u = rng.normal(0, 1, (1, L, 1, 2)); h0 = rng.normal(0, 0.3, (1, 1, 2))
    pr = np.array([[a], [b]])
    ur = u.reshape(1, L, 2, 1); h0r = h0.reshape(1, 2, 1)
    hd = o.seq_unroll("tanh_dense", W, u, h0)
    hr = o.seq_unroll("rot_tanh", pr, ur, h0r)
    assert np.allclose(hr.reshape(L, 2), hd.reshape(L, 2), rtol=0, atol=1e-15)
    Jd = o.cell_jacobian("tanh_dense", W, h0[0], u[0, 0])
    Jr = o.cell_jacobian("rot_tanh", pr, h0r[0], ur[0, 0])
    assert np.allclose(Jr.reshape(2, 2), Jd, rtol=0, atol=1e-15)
    nd = o.newton("tanh_dense", W, u, h0, tol=1e-12, max_iter=20)
    nr = o.newton("rot_tanh", pr, ur, h0r, tol=1e-12, max_iter=20)
    assert nd[1] == nr[1] and np.allclose(nd[3], nr[3], rtol=1e-9, atol=1e-15)
    g = rng.normal(0, 1, (1, L, 1, 2))
    dud, dWd, dh0d = o.backward("tanh_dense", W, u, h0, hd, g)
    dur, dpr, dh0r = o.backward("rot_tanh", pr, ur, h0r, hr, g.reshape(1, L, 2, 1))
    assert np.allclose(dur.reshape(L, 2), dud.reshape(L, 2), rtol=0, atol=1e-14)
    assert np.allclose(dh0r.ravel(), dh0d.ravel(), rtol=0, atol=1e-14)
    assert np.allclose(dpr.ravel(), [dWd[0, 0] + dWd[1, 1], dWd[1, 0] - dWd[0, 1]], rtol=0, atol=1e-13)


@pytest.mark.parametrize("cell,N", [("tri_tanh", 3), ("quad_tanh", 4)])
def test_mixing_cells_are_the_dense_cell_with_an_nxn_matrix_per_channel(oracle_mod, cell, N):
    """Each channel of the N x N-block example cells is h' = tanh(M h + u) with that channel's own
    matrix M: step, Jacobian, Newton solve (both Jacobian modes) and backward must agree with the
    dense cell at H = N, channel by channel (channels do not mix)."""
    o = oracle_mod
    rng = np.random.default_rng(96)
    L, H = 10, 2
    M = rng.uniform(-0.45, 0.45, (H, N, N)) * 3 / N          # M[channel][a][b]
    pt = np.transpose(M, (1, 2, 0)).reshape(N * N, H)        # rows m_ab, channels last
    ut = rng.normal(0, 1, (1, L, N, H)); h0t = rng.normal(0, 0.3, (1, N, H)); gt = rng.normal(0, 1, (1, L, N, H))
    ht = o.seq_unroll(cell, pt, ut, h0t)
    Jt = o.cell_jacobian(cell, pt, h0t[0], ut[0, 0])
    nt = o.newton(cell, pt, ut, h0t, tol=-1.0, max_iter=3)
    qt = o.newton(cell, pt, ut, h0t, tol=-1.0, max_iter=3, jacobian="diagonal")
    dut, dpt, dh0t = o.backward(cell, pt, ut, h0t, ht, gt)
    for ch in range(H):
        W = M[ch]
        u = ut[:, :, :, ch].reshape(1, L, 1, N); h0 = h0t[:, :, ch].reshape(1, 1, N); g = gt[:, :, :, ch].reshape(1, L, 1, N)
        hd = o.seq_unroll("tanh_dense", W, u, h0)
        assert np.allclose(ht[0, :, :, ch], hd.reshape(L, N), rtol=0, atol=1e-15)
        assert np.allclose(Jt[:, :, ch], o.cell_jacobian("tanh_dense", W, h0[0], u[0, 0]), rtol=0, atol=1e-15)
        nd = o.newton("tanh_dense", W, u, h0, tol=-1.0, max_iter=3)
        qd = o.newton("tanh_dense", W, u, h0, tol=-1.0, max_iter=3, jacobian="diagonal")
        assert np.allclose(nt[0][0, :, :, ch], nd[0].reshape(L, N), rtol=0, atol=1e-14)
        assert np.allclose(qt[0][0, :, :, ch], qd[0].reshape(L, N), rtol=0, atol=1e-14)
        dud, dWd, dh0d = o.backward("tanh_dense", W, u, h0, hd, g)
        assert np.allclose(dut[0, :, :, ch], dud.reshape(L, N), rtol=0, atol=1e-14)
        assert np.allclose(dh0t[0, :, ch], dh0d.ravel(), rtol=0, atol=1e-14)
        assert np.allclose(dpt[:, ch].reshape(N, N), dWd, rtol=0, atol=1e-13)


# ---------------------------------------------------------- input projection

@pytest.mark.parametrize("n_heads", [1, 2, 4])
def test_input_projection_is_a_block_diagonal_matrix_product(oracle_mod, n_heads):
    """Eq. (7a): u_g = B_g x + b_g.  With n_heads heads B_g is block diagonal
    (App. C); expanding it to a full H x H matrix, the map is a plain matrix
    product, here numpy's."""
    o = oracle_mod
    rng = np.random.default_rng(101 + n_heads)
    Bt, L, H, G = 2, 5, 8, 3
    dh = H // n_heads
    x = rng.normal(0, 1, (Bt, L, H)); Wx = rng.normal(0, 1, (G, H, dh)); b = rng.normal(0, 1, (G, H))
    full = np.zeros((G, H, H))
    for h in range(H):
        k = h // dh
        full[:, h, k * dh:(k + 1) * dh] = Wx[:, h, :]
    ref = np.einsum("blj,ghj->blgh", x, full) + b
    assert np.allclose(o.input_projection(x, Wx, b, n_heads), ref, rtol=0, atol=1e-13)
    assert np.allclose(o.input_projection(x, Wx, None, n_heads), ref - b, rtol=0, atol=1e-13)
    # heads do not mix: changing head 0's inputs leaves the other heads' outputs alone
    if n_heads > 1:
        x2 = x.copy(); x2[..., :dh] += 1.0
        u1, u2 = o.input_projection(x, Wx, b, n_heads), o.input_projection(x2, Wx, b, n_heads)
        assert np.array_equal(u1[..., dh:], u2[..., dh:]) and not np.allclose(u1[..., :dh], u2[..., :dh])


@pytest.mark.parametrize("n_heads", [1, 2])
def test_input_projection_backward_matches_finite_differences(oracle_mod, n_heads):
    o = oracle_mod
    rng = np.random.default_rng(111)
    rows, H, G = 6, 4, 3
    dh = H // n_heads
    x = rng.normal(0, 1, (rows, H)); Wx = rng.normal(0, 1, (G, H, dh)); b = rng.normal(0, 1, (G, H))
    w = rng.normal(0, 1, (rows, G, H))
    loss = lambda xx, WW, bb: float(np.sum(w * o.input_projection(xx, WW, bb, n_heads)))
    dx, dW, db = o.input_projection_backward(x, Wx, w, n_heads)
    eps = 1e-6
    for arr, grad, which in ((x, dx, 0), (Wx, dW, 1), (b, db, 2)):
        for idx in np.ndindex(*arr.shape):
            a1 = arr.copy(); a2 = arr.copy(); a1[idx] += eps; a2[idx] -= eps
            args1 = [x, Wx, b]; args2 = [x, Wx, b]
            args1[which] = a1; args2[which] = a2
            fd = (loss(*args1) - loss(*args2)) / (2 * eps)
            assert abs(grad[idx] - fd) < 1e-7 * max(1.0, abs(fd)), (which, idx)


# ------------------------------------------------------- residual max-norm (App. A)

@pytest.mark.parametrize("cell", ALL_CELLS)
def test_residual_norm_vanishes_on_the_recurrence_only(oracle_mod, cell):
    """The states of Eq. (1) solve Eq. (2) exactly (the same function on the same numbers), with
    the h0 they started from and with no other."""
    o = oracle_mod
    H = 64 if cell == "tanh_dense" else 5
    params, u, h0 = rand_problem(o, cell, 2, 9, H, seed=71)
    h = o.seq_unroll(cell, params, u, h0)
    assert o.residual_norm(cell, params, u, h0, h) == 0.0
    # with h0 left out only row 1 of Eq. (2) is violated: by f(0, u_1) - h_1
    want = max(np.max(np.abs(o.cell_step(cell, params, np.zeros_like(h0[b]), u[b, 0]) - h[b, 0])) for b in range(2))
    assert want > 1e-3
    assert o.residual_norm(cell, params, u, None, h) == pytest.approx(want, rel=1e-14)


def test_residual_norm_linear_cell_closed_form(oracle_mod):
    """f = a h + u (footnote of Sec. 2): the residual of arbitrary states is a h_{l-1} + u_l - h_l,
    typed out with numpy."""
    o = oracle_mod
    rng = np.random.default_rng(72)
    B, L, H = 3, 7, 4
    params = np.zeros((2, 1, H)); params[0] = rng.uniform(-0.9, 0.9, (1, H))
    u = rng.normal(0, 1, (B, L, 1, H)); h = rng.normal(0, 1, (B, L, 1, H)); h0 = rng.normal(0, 1, (B, 1, H))
    prev = np.concatenate([h0[:, None], h[:, :-1]], axis=1)
    want = np.max(np.abs(params[0][None, None] * prev + u - h))
    assert o.residual_norm("linear_diag", params, u, h0, h) == pytest.approx(want, rel=1e-15)


@pytest.mark.parametrize("cell", ["gru_diag", "lstm_diag", "paralstm_diag", "tanh_dense", "rot_tanh"])
def test_residual_norm_of_one_perturbed_state(oracle_mod, cell):
    """One state value of the exact trajectory moved by eps, at step l0: equation l0 is off by eps
    and equation l0 + 1 by f(h_l0 + eps e) - h_{l0+1}; every other equation still holds.  Pins which
    state each equation reads (a shift the wrong way, or a wrong batch / state index, changes the
    value) and that the maximum runs over everything."""
    o = oracle_mod
    H = 64 if cell == "tanh_dense" else 3
    B, L = 2, 6
    params, u, h0 = rand_problem(o, cell, B, L, H, seed=73)
    h = o.seq_unroll(cell, params, u, h0)
    S = h.shape[2]
    eps = 0.25
    for b, l0, s, ch in [(0, 0, 0, 0), (1, 3, S - 1, H - 1), (1, L - 1, 0, 1)]:
        hh = h.copy()
        hh[b, l0, s, ch] += eps
        nxt = 0.0 if l0 == L - 1 else np.max(np.abs(o.cell_step(cell, params, hh[b, l0], u[b, l0 + 1]) - h[b, l0 + 1]))
        assert o.residual_norm(cell, params, u, h0, hh) == pytest.approx(max(eps, nxt), rel=1e-13), (b, l0, s, ch)
    hh = h.copy()
    hh[1, 2, 0, 0] = np.nan
    assert math.isnan(o.residual_norm(cell, params, u, h0, hh))


@pytest.mark.parametrize("cell", ["gru_diag", "paralstm_diag", "tanh_dense"])
def test_residual_norm_along_newton(oracle_mod, cell):
    """App. A's convergence figure: the residual max-norm of the Newton iterates drops to rounding
    level within a handful of iterations, quadratically at the end (each value at most the square
    root scale of the one before is too strict for the first steps, so: the last three values above
    the floor shrink faster than linearly, and the floor is reached by iteration 7)."""
    o = oracle_mod
    H = 64 if cell == "tanh_dense" else 6
    params, u, h0 = rand_problem(o, cell, 2, 200, H, seed=74)
    norms = []
    for k in range(9):
        hk = o.newton(cell, params, u, h0, tol=-1.0, max_iter=k)[0]
        norms.append(o.residual_norm(cell, params, u, h0, hk))
    assert norms[0] > 1e-2                                   # the initial guess is not the solution
    assert min(norms[:8]) < 1e-13, norms
    above = [x for x in norms if x > 1e-12]
    assert len(above) <= 7, norms
    if len(above) >= 3:
        assert above[-1] / above[-2] < above[-2] / above[-3], norms      # super-linear at the end
    # App. A's guess h^0_l = f(h0, u_l) satisfies the first equation exactly
    h_guess = o.newton(cell, params, u, h0, tol=-1.0, max_iter=0)[0]
    assert o.residual_norm(cell, params, u[:, :1], h0, h_guess[:, :1]) == 0.0


# ------------------------------------- quasi-Newton with diagonal Jacobians (Sec. 1, Sec. 2.1)

@pytest.mark.parametrize("cell", DIAG_CELLS)
def test_quasi_newton_is_newton_for_diagonal_cells(oracle_mod, cell):
    """Eq. (9): these cells' Jacobians are diagonal already, so dropping off-diagonal entries
    changes nothing, bit for bit."""
    o = oracle_mod
    params, u, h0 = rand_problem(o, cell, 2, 40, 5, seed=81)
    a = o.newton(cell, params, u, h0, tol=1e-10, max_iter=30)
    b = o.newton(cell, params, u, h0, tol=1e-10, max_iter=30, jacobian="diagonal")
    assert a[1] == b[1] and a[2] == b[2] and np.array_equal(a[0], b[0]) and np.array_equal(a[3], b[3])


def _diag_of(J, kind):
    """The Jacobian of all state values of one step as a dense matrix, off-diagonal entries dropped."""
    if kind == "dense":
        return np.diag(np.diag(J))
    H = J.shape[-1]                      # 2x2 blocks [2][2][H] -> diag(J_cc, J_hh) of size 2H
    return np.diag(np.concatenate([J[0, 0], J[1, 1]]))


@pytest.mark.parametrize("cell,kind,H", [("tanh_dense", "dense", 4), ("lstm_diag", "block", 3), ("paralstm_diag", "block", 3),
                                          ("rot_tanh", "block", 2)])
def test_quasi_newton_iterates_by_a_global_solve(oracle_mod, cell, kind, H):
    """Each quasi-Newton iterate re-derived without forward substitution: assemble the block
    bi-diagonal matrix of Eq. (3) with diag(J_l) below the identity blocks, as one (L n) x (L n)
    matrix, and solve it with LAPACK; the Jacobians and the cell come from the routines pinned
    above (finite differences, hand values)."""
    o = oracle_mod
    B, L = 1, 6
    params, u, h0 = rand_problem(o, cell, B, L, H, seed=82)
    S = o.dims(cell)[1]
    n = S * H
    h = np.stack([o.cell_step(cell, params, h0[0], u[0, l]) for l in range(L)])          # App. A's guess
    for k in range(1, 5):
        M = np.eye(L * n)
        r = np.zeros(L * n)
        for l in range(L):
            hp = h0[0] if l == 0 else h[l - 1]
            r[l * n:(l + 1) * n] = (o.cell_step(cell, params, hp, u[0, l]) - h[l]).reshape(-1)
            if l > 0:
                M[l * n:(l + 1) * n, (l - 1) * n:l * n] = -_diag_of(o.cell_jacobian(cell, params, hp, u[0, l]), kind)
        delta = np.linalg.solve(M, r).reshape(L, S, H)
        h = h + delta
        got, it, st, tr = o.newton(cell, params, u, h0, tol=-1.0, max_iter=k, jacobian="diagonal")
        assert it == k and np.max(np.abs(got[0] - h)) < 1e-13, k
        assert tr[-1] == pytest.approx(np.max(np.abs(delta)), rel=1e-12)
    # and it is not Newton: with the full Jacobian the same iterate is elsewhere
    full = o.newton(cell, params, u, h0, tol=-1.0, max_iter=2)[0]
    quasi = o.newton(cell, params, u, h0, tol=-1.0, max_iter=2, jacobian="diagonal")[0]
    assert np.max(np.abs(full - quasi)) > 1e-6


@pytest.mark.parametrize("cell", ["tanh_dense", "lstm_diag", "paralstm_diag"])
def test_quasi_newton_is_causal_and_reaches_the_recurrence(oracle_mod, cell):
    """The system is lower block-triangular with identity diagonal blocks, whatever stands below
    them: the guess solves step 1 and iteration k makes step k + 1 exact, so the recurrence's states
    are reached after at most L - 1 iterations, however poor the approximation; it converges to the
    same states as Newton, only linearly (more iterations than Newton here)."""
    o = oracle_mod
    H = 64 if cell == "tanh_dense" else 4
    L = 12
    params, u, h0 = rand_problem(o, cell, 2, L, H, seed=83)
    ref = o.seq_unroll(cell, params, u, h0)
    for k in (0, 1, 4, L - 1):
        hk = o.newton(cell, params, u, h0, tol=-1.0, max_iter=k, jacobian="diagonal")[0]
        assert np.max(np.abs(hk[:, :k + 1] - ref[:, :k + 1])) < 1e-14, k
    params, u, h0 = rand_problem(o, cell, 2, 300, H, seed=84)
    ref = o.seq_unroll(cell, params, u, h0)
    hq, itq, stq, trq = o.newton(cell, params, u, h0, tol=1e-9, max_iter=300, jacobian="diagonal")
    hn, itn, stn, _ = o.newton(cell, params, u, h0, tol=1e-9, max_iter=300)
    assert stq == 0 and stn == 0 and itq > itn
    assert np.max(np.abs(hq - ref)) < 1e-8 and np.max(np.abs(hn - ref)) < 1e-12
