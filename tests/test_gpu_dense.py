"""GPU parity of the dense-Jacobian path (h' = tanh(W h + u), H = 64): the MFMA
scan against the CPU oracle, including benchmark configuration 4 at full size."""
import json
import os

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from workloads import CONFIGS, make_inputs      # noqa: E402
from workloads.rng import normal                 # noqa: E402
from parity_util import well_posed_tol, elt_err  # noqa: E402

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "newton_traces.json")


def relerr(got, ref):
    got = np.asarray(got, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    return float(np.max(np.abs(got - ref)) / max(np.max(np.abs(ref)), 1e-30))


def f64(t):
    return None if t is None else t.detach().to("cpu", torch.float64).numpy()


@pytest.mark.parametrize("shape", [(1, 1), (1, 16), (2, 17), (3, 50), (33, 100), (5, 257), (64, 32)])
@pytest.mark.parametrize("with_h0", [False, True])
def test_dense_small(oracle_mod, shape, with_h0):
    import paper_2510_21450_amd as P
    B, L = shape
    H = 64
    print(f"dense B={B} L={L} h0={with_h0}", flush=True)
    W = normal(900 + L, 5, (H, H), std=0.8 / H ** 0.5, device="cuda")
    u = normal(900 + L, 1, (B, L, 1, H), device="cuda")
    h0 = normal(900 + L, 3, (B, 1, H), std=0.3, device="cuda") if with_h0 else None
    Wn, un, h0n = f64(W), f64(u), f64(h0)
    ref = oracle_mod.seq_unroll("tanh_dense", Wn, un, h0n)
    # fixed iteration counts: iterate k matches the oracle's iterate k
    for k in (0, 1, 2):
        h, iters, _ = P.forward("tanh_dense", W, u, h0, tol=-1.0, max_iter=k)
        hk, _, _, _ = oracle_mod.newton("tanh_dense", Wn, un, h0n, tol=-1.0, max_iter=k)
        assert tuple(int(x) for x in iters.cpu()) == (k, 0)
        assert relerr(f64(h), hk) <= 2e-5, k
    tol, want = well_posed_tol(oracle_mod, "tanh_dense", Wn, un, h0n, max_iter=32, probe_tol=1e-4)
    h, iters, tr = P.forward("tanh_dense", W, u, h0, tol=tol, max_iter=32, trace=True)
    torch.cuda.synchronize()
    it, st = (int(x) for x in iters.cpu())
    assert st == 0
    assert relerr(f64(h), ref) <= 1e-5
    assert it == want, (it, want, tol, tr.cpu().numpy()[:it])


@pytest.mark.parametrize("shape", [(2, 48), (3, 70), (5, 160)])
def test_chunk_products_match_plain_matrix_products(shape):
    """The MFMA composition kernel alone against numpy's fp64 matrix products:
    A[b][c] = J_e ... J_s with J_l = diag(d_l) W over each chunk (Alg. 1b's
    Jacobian update accumulated over a chunk)."""
    import paper_2510_21450_amd as P
    B, L = shape
    H = 64
    W = normal(77, 5, (H, H), std=0.8 / H ** 0.5, device="cuda")
    d = (1.0 - torch.tanh(normal(77, 1, (B, L, H), device="cuda")) ** 2).contiguous()
    A = P.dense_chunk_products(W, d)
    torch.cuda.synchronize()
    chunk = P.dense_chunk()
    n_c = (L + chunk - 1) // chunk
    Wn, dn, An = f64(W), f64(d), f64(A)
    assert A.shape == (B, n_c, H, H)
    for b in range(B):
        for c in range(1, n_c - 1):
            ref = np.eye(H)
            for l in range(c * chunk, min(L, (c + 1) * chunk)):
                ref = (dn[b, l][:, None] * Wn) @ ref
            assert relerr(An[b, c], ref) <= 1e-5, (b, c)
        assert not An[b, 0].any() and not An[b, n_c - 1].any()     # not needed by the scan, not written


def test_dense_zero_weights_is_tanh_of_input(oracle_mod):
    import paper_2510_21450_amd as P
    B, L, H = 2, 40, 64
    W = torch.zeros(H, H, device="cuda")
    u = normal(5, 1, (B, L, 1, H), device="cuda")
    h, iters, tr = P.forward("tanh_dense", W, u, None, tol=1e-6, max_iter=8, trace=True)
    assert tuple(int(x) for x in iters.cpu()) == (1, 0)          # guess exact, one confirming solve
    assert relerr(f64(h), np.tanh(f64(u))) <= 1e-6


def test_dense_unsupported_shapes_are_refused():
    import paper_2510_21450_amd as P
    W = torch.zeros(32, 32, device="cuda")
    u = torch.zeros(1, 4, 1, 32, device="cuda")
    with pytest.raises(RuntimeError, match="UNSUPPORTED"):
        P.forward("tanh_dense", W, u, None)


def test_config_c4_full_size(oracle_mod):
    """Benchmark configuration 4: B=64, L=1024, H=64, max_iter 32, forward."""
    import paper_2510_21450_amd as P
    w = CONFIGS["C4"]
    d = make_inputs(w, device="cuda")
    h, iters, tr = P.forward(w.cell, d["params"], d["u"], None, tol=w.tol, max_iter=w.max_iter, trace=True)
    torch.cuda.synchronize()
    it, st = (int(x) for x in iters.cpu())
    assert st == 0
    ref = oracle_mod.seq_unroll(w.cell, f64(d["params"]), f64(d["u"]), None)
    e, ee = relerr(f64(h), ref), elt_err(f64(h), ref)
    with open(GOLDEN) as f:
        gold = json.load(f)["C4"]
    want = next(k for k, m in enumerate(gold["f32"], start=1) if m <= w.tol)
    assert want == next(k for k, m in enumerate(gold["f64"], start=1) if m <= w.tol)
    print(f"C4: iters={it} (oracle {want}) rel err h={e:.2e} element-wise (floor 1e-3 max|ref|) {ee:.2e} "
          f"trace={tr.cpu().numpy()[:it]}", flush=True)
    assert it == want
    assert e <= 1e-5 and ee <= 1e-3
    got = tr.cpu().numpy()[:it]
    for k in range(it):
        if gold["f64"][k] > 1e-3:
            assert abs(got[k] - gold["f64"][k]) <= 2e-3 * gold["f64"][k]


@pytest.mark.parametrize("shape", [(1, 1), (1, 16), (2, 17), (3, 50), (33, 100), (5, 257), (64, 33)])
@pytest.mark.parametrize("with_h0", [False, True])
def test_dense_backward_small(oracle_mod, as_stored, shape, with_h0):
    """Eq. (6) for the dense cell: the reverse scan with W^T on the matrix cores,
    dL/du, dL/dW and dL/dh0 against the oracle's reverse sweep, both at the oracle's states."""
    import paper_2510_21450_amd as P
    B, L = shape
    H = 64
    print(f"dense backward B={B} L={L} h0={with_h0}", flush=True)
    W = normal(700 + L, 5, (H, H), std=0.8 / H ** 0.5, device="cuda")
    u = normal(700 + L, 1, (B, L, 1, H), device="cuda")
    h0 = normal(700 + L, 3, (B, 1, H), std=0.3, device="cuda") if with_h0 else None
    g = normal(700 + L, 4, (B, L, 1, H), device="cuda")
    h = as_stored(oracle_mod.seq_unroll("tanh_dense", f64(W), f64(u), f64(h0)), u)
    du, dW, dh0 = P.backward("tanh_dense", W, u, h0, h, g)
    torch.cuda.synchronize()
    rdu, rdW, rdh0 = oracle_mod.backward("tanh_dense", f64(W), f64(u), f64(h0), f64(h), f64(g))
    assert relerr(f64(du), rdu) <= 1e-5
    assert relerr(f64(dW), rdW) <= 1e-5
    assert relerr(f64(dh0), rdh0) <= 1e-5
    # dL/dh0 may be skipped; a second call gives the same bits (fixed summation order)
    du2, dW2, none = P.backward("tanh_dense", W, u, h0, h, g, want_dh0=False)
    torch.cuda.synchronize()
    assert none is None and torch.equal(du, du2) and torch.equal(dW, dW2)


def test_dense_backward_config_c4(oracle_mod, as_stored):
    """Backward at config 4's size (B=64, L=1024), compared on whole sequences
    (the oracle handles a subset of the batch; dL/dW is checked for that subset
    by running the library on it alone)."""
    import paper_2510_21450_amd as P
    w = CONFIGS["C4"]
    d = make_inputs(w, device="cuda")
    W, u = d["params"], d["u"]
    g = normal(w.seed, 4, (w.B, w.L, 1, w.H), device="cuda")
    h, iters, _ = P.forward(w.cell, W, u, None, tol=w.tol, max_iter=w.max_iter)
    sel = [0, 31, 63]
    idx = torch.as_tensor(sel, device="cuda")
    us, gs = u.index_select(0, idx).contiguous(), g.index_select(0, idx).contiguous()
    # sequences are independent in dL/du and dL/dh0: the compared ones are evaluated on both sides
    # at the oracle's states
    hs = as_stored(oracle_mod.seq_unroll(w.cell, f64(W), f64(us), None), h)
    assert relerr(f64(h.index_select(0, idx)), f64(hs)) <= 1e-5
    h.index_copy_(0, idx, hs)
    du, dW, dh0 = P.backward(w.cell, W, u, None, h, g)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(du).all()) and bool(torch.isfinite(dW).all())
    rdu, rdW, rdh0 = oracle_mod.backward(w.cell, f64(W), f64(us), None, f64(hs), f64(gs))
    assert relerr(f64(du.index_select(0, idx)), rdu) <= 1e-5
    assert relerr(f64(dh0.index_select(0, idx)), rdh0) <= 1e-5
    _, dWs, _ = P.backward(w.cell, W, us, None, hs, gs)
    assert relerr(f64(dWs), rdW) <= 1e-5
    # the full-batch dL/dW is the sum over sequences: compare with per-sequence runs added up in fp64
    acc = np.zeros((w.H, w.H))
    for b in range(0, w.B, 16):
        sl = slice(b, b + 16)
        acc += f64(P.backward(w.cell, W, u[sl].contiguous(), None, h[sl].contiguous(), g[sl].contiguous())[1])
    assert relerr(f64(dW), acc) <= 1e-5


# ---------------------------------------------------- inexact Jacobian products

@pytest.fixture
def products_mode():
    """Sets the product arithmetic for one test and always restores fp32."""
    import paper_2510_21450_amd as P
    yield P.set_dense_products
    P.set_dense_products(0)


@pytest.mark.parametrize("mode,bound", [(1, 1e-4), (2, 2e-2)])
@pytest.mark.parametrize("shape", [(2, 48), (3, 70), (5, 160)])
def test_chunk_products_in_bf16_terms(products_mode, mode, bound, shape):
    """The compositions from bf16 terms against numpy's fp64 products: three
    terms lose about 2^-16 per product, one term about 2^-8; 15 products per chunk."""
    import paper_2510_21450_amd as P
    B, L = shape
    H = 64
    W = normal(78, 5, (H, H), std=0.8 / H ** 0.5, device="cuda")
    d = (1.0 - torch.tanh(normal(78, 1, (B, L, H), device="cuda")) ** 2).contiguous()
    products_mode(mode)
    A = P.dense_chunk_products(W, d)
    torch.cuda.synchronize()
    chunk = P.dense_chunk()
    n_c = (L + chunk - 1) // chunk
    Wn, dn, An = f64(W), f64(d), f64(A)
    worst = 0.0
    for b in range(B):
        for c in range(1, n_c - 1):
            ref = np.eye(H)
            for l in range(c * chunk, min(L, (c + 1) * chunk)):
                ref = (dn[b, l][:, None] * Wn) @ ref
            worst = max(worst, relerr(An[b, c], ref))
    print(f"mode {mode} {shape}: worst norm-wise error of a chunk product {worst:.2e}", flush=True)
    assert worst <= bound
    assert worst >= 1e-7          # it is not the fp32 kernel that ran


@pytest.mark.parametrize("mode,extra", [(1, 1), (2, 12)])
@pytest.mark.parametrize("shape", [(3, 50), (33, 100), (5, 257), (64, 1024)])
def test_dense_solve_with_inexact_products_reaches_the_same_states(oracle_mod, as_stored, products_mode, mode, extra, shape):
    """Inexact Newton: with approximate Jacobian products and the fp32 residual the
    solve still ends at the recurrence's states (1e-5 against the sequential
    unroll), the stopping test still holds what it promises, and the iteration
    count is at least Newton's and exceeds it by a few at most."""
    import paper_2510_21450_amd as P
    B, L = shape
    H = 64
    W = normal(950 + L, 5, (H, H), std=0.8 / H ** 0.5, device="cuda")
    u = normal(950 + L, 1, (B, L, 1, H), device="cuda")
    h0 = normal(950 + L, 3, (B, 1, H), std=0.3, device="cuda")
    Wn, un, h0n = f64(W), f64(u), f64(h0)
    ref = oracle_mod.seq_unroll("tanh_dense", Wn, un, h0n)
    tol = 1e-5
    _, it32, st32, _ = oracle_mod.newton("tanh_dense", Wn, un, h0n, tol=tol, max_iter=32, precision="f32")
    assert st32 == 0
    products_mode(mode)
    h, iters, tr = P.forward("tanh_dense", W, u, h0, tol=tol, max_iter=32, trace=True)
    torch.cuda.synchronize()
    it, st = (int(x) for x in iters.cpu())
    tr = tr.cpu().numpy()[:it]
    print(f"mode {mode} {shape}: {it} iterations (Newton {it32}), trace {tr}", flush=True)
    assert st == 0 and tr[-1] <= tol and (it == 1 or tr[-2] > tol)
    assert relerr(f64(h), ref) <= 1e-5
    assert it32 - 1 <= it <= it32 + extra
    # the backward pass is unaffected by the mode (always fp32 products)
    g = normal(951 + L, 4, (B, L, 1, H), device="cuda")
    hs = as_stored(ref, h)
    du, dW, dh0 = P.backward("tanh_dense", W, u, h0, hs, g)
    torch.cuda.synchronize()
    rdu, rdW, rdh0 = oracle_mod.backward("tanh_dense", Wn, un, h0n, f64(hs), f64(g))
    assert relerr(f64(du), rdu) <= 1e-5 and relerr(f64(dW), rdW) <= 1e-5 and relerr(f64(dh0), rdh0) <= 1e-5


# ------------------------------------------- quasi-Newton: diagonal of the Jacobian

@pytest.fixture
def jacobian_mode():
    """Sets the Jacobian of the dense path's linear solves for one test and always restores the full one."""
    import paper_2510_21450_amd as P
    yield P.set_dense_jacobian
    P.set_dense_jacobian(0)


@pytest.mark.parametrize("shape", [(1, 1), (2, 17), (3, 64), (3, 65), (5, 257), (64, 33), (2, 1000)])
def test_dense_quasi_newton_against_the_oracle(oracle_mod, jacobian_mode, shape):
    """pararnn_set_dense_jacobian(1): every iterate, the per-iteration maxima and the iteration
    count against the oracle's quasi-Newton (Newton with J_l replaced by its diagonal)."""
    import paper_2510_21450_amd as P
    B, L = shape
    H = 64
    print(f"dense quasi-Newton B={B} L={L}", flush=True)
    W = normal(970 + L, 5, (H, H), std=0.8 / H ** 0.5, device="cuda")
    u = normal(970 + L, 1, (B, L, 1, H), device="cuda")
    h0 = normal(970 + L, 3, (B, 1, H), std=0.3, device="cuda")
    Wn, un, h0n = f64(W), f64(u), f64(h0)
    jacobian_mode(1)
    for k in (0, 1, 2, 5):
        h, iters, tr = P.forward("tanh_dense", W, u, h0, tol=-1.0, max_iter=k, trace=True)
        torch.cuda.synchronize()
        hk, _, _, trk = oracle_mod.newton("tanh_dense", Wn, un, h0n, tol=-1.0, max_iter=k, jacobian="diagonal")
        assert tuple(int(x) for x in iters.cpu()) == (k, 0)
        assert relerr(f64(h), hk) <= 1e-5, k
        assert np.allclose(tr.cpu().numpy()[:k], trk, rtol=1e-3, atol=1e-6), k
    # linear convergence leaves little room between consecutive maxima: the tolerance is put in the middle
    # (in the logarithm) of a step of the oracle's fp64 and fp32 traces, with 20 % room on both sides, and
    # the count is then compared exactly
    tol, want = well_posed_tol(oracle_mod, "tanh_dense", Wn, un, h0n, max_iter=200, margin=1.2, probe_tol=1e-5,
                               jacobian="diagonal")
    h, iters, tr = P.forward("tanh_dense", W, u, h0, tol=tol, max_iter=200, trace=True)
    torch.cuda.synchronize()
    it, st = (int(x) for x in iters.cpu())
    h64, it64, st64, tr64 = oracle_mod.newton("tanh_dense", Wn, un, h0n, tol=tol, max_iter=200, jacobian="diagonal")
    tn, itn = well_posed_tol(oracle_mod, "tanh_dense", Wn, un, h0n, max_iter=200, probe_tol=1e-5)
    assert st == 0 and st64 == 0 and it64 == want
    print(f"  {it} iterations at tol {tol:.3g} (oracle {it64}; Newton {itn} at {tn:.3g})", flush=True)
    assert it == it64, (it, it64, tol, tr.cpu().numpy()[:it], tr64)
    assert it64 >= itn
    assert relerr(f64(h), h64) <= 1e-5
    assert relerr(f64(h), oracle_mod.seq_unroll("tanh_dense", Wn, un, h0n)) <= max(1e-5, 20 * tol)   # error at the stop is of the order of tol
    # the full Jacobian again: Newton's count
    jacobian_mode(0)
    _, iters, _ = P.forward("tanh_dense", W, u, h0, tol=tn, max_iter=200)
    assert int(iters.cpu()[0]) == itn


def test_dense_quasi_newton_config_c4(oracle_mod, jacobian_mode):
    """Benchmark configuration 4 with the diagonal approximation: same states, more iterations."""
    import paper_2510_21450_amd as P
    w = CONFIGS["C4"]
    d = make_inputs(w, device="cuda")
    Wn, un = f64(d["params"]), f64(d["u"])
    jacobian_mode(1)
    h, iters, tr = P.forward(w.cell, d["params"], d["u"], None, tol=w.tol, max_iter=w.max_iter, trace=True)
    torch.cuda.synchronize()
    it, st = (int(x) for x in iters.cpu())
    h64, it64, st64, tr64 = oracle_mod.newton(w.cell, Wn, un, None, tol=w.tol, max_iter=w.max_iter, jacobian="diagonal")
    _, it32, _, tr32 = oracle_mod.newton(w.cell, Wn, un, None, tol=w.tol, max_iter=w.max_iter, jacobian="diagonal",
                                         precision="f32")
    print(f"C4 quasi-Newton: {it} iterations (oracle {it64}), status {st} (oracle {st64}), trace {tr.cpu().numpy()[:it]}", flush=True)
    # the configuration's tolerance is given; the oracle's fp64 and fp32 traces both clear it by 5 % on each
    # side (linear convergence: consecutive maxima are a factor 1.5-2 apart), so the count is compared exactly
    assert it32 == it64 and all(t[-1] <= w.tol / 1.05 and t[-2] >= 1.05 * w.tol for t in (tr32, tr64)), (tr32, tr64)
    assert (it, st) == (it64, st64)
    assert relerr(f64(h), h64) <= 1e-5
    assert np.allclose(tr.cpu().numpy()[:min(it, it64)], tr64[:min(it, it64)], rtol=2e-3)


@pytest.mark.parametrize("mode", [0, 1])
def test_dense_iteration_control_edge_cases(oracle_mod, jacobian_mode, mode):
    """The dense cell under both Jacobian modes: max_iter = 0 gives the initial guess, tol = 0 runs
    to max_iter with NOT_CONVERGED, L = 1 needs one solve with a zero update, a NaN in the input
    ends the solve with NONFINITE after its first iteration: statuses and counts as the oracle's."""
    import paper_2510_21450_amd as P
    B, L, H = 2, 40, 64
    W = normal(990, 5, (H, H), std=0.8 / H ** 0.5, device="cuda")
    u = normal(990, 1, (B, L, 1, H), device="cuda")
    h0 = normal(990, 3, (B, 1, H), std=0.3, device="cuda")
    Wn, un, h0n = f64(W), f64(u), f64(h0)
    jac = "full" if mode == 0 else "diagonal"
    jacobian_mode(mode)
    h, iters, _ = P.forward("tanh_dense", W, u, h0, tol=1e-6, max_iter=0)
    hg = oracle_mod.newton("tanh_dense", Wn, un, h0n, tol=1e-6, max_iter=0, jacobian=jac)[0]
    assert int(iters.cpu()[0]) == 0 and relerr(f64(h), hg) <= 1e-5
    h, iters, _ = P.forward("tanh_dense", W, u, h0, tol=0.0, max_iter=2)
    _, ito, sto, _ = oracle_mod.newton("tanh_dense", Wn, un, h0n, tol=0.0, max_iter=2, jacobian=jac)
    assert tuple(int(x) for x in iters.cpu()) == (ito, sto) == (2, 1)
    h, iters, tr = P.forward("tanh_dense", W, u[:, :1].contiguous(), h0, tol=0.0, max_iter=5, trace=True)
    assert tuple(int(x) for x in iters.cpu()) == (1, 0) and float(tr[0]) == 0.0
    u2 = u.clone(); u2[1, 3, 0, 7] = float("nan")
    h, iters, _ = P.forward("tanh_dense", W, u2, h0, tol=1e-6, max_iter=5)
    _, ito, sto, _ = oracle_mod.newton("tanh_dense", Wn, f64(u2), h0n, tol=1e-6, max_iter=5, jacobian=jac)
    assert tuple(int(x) for x in iters.cpu()) == (ito, sto) == (1, 5)


# ------------------------------------------- launch plans of the forward solve

@pytest.fixture
def tail_mode():
    """Sets the launch plan of the dense path's forward solves for one test and always restores the default."""
    import paper_2510_21450_amd as P
    yield P.set_dense_tail
    P.set_dense_tail(1)


@pytest.mark.parametrize("shape", [(3, 50), (33, 100), (5, 257)])
def test_dense_launch_plans_agree(oracle_mod, tail_mode, shape):
    """The same solve as launches per phase throughout (0), as six iterations of launches per phase and
    one persistent launch for the rest (1, the default), and as one persistent launch from the start
    (2): bit-identical states, the same iteration count, status and trace -- for a solve to a tolerance,
    for one that runs out of iterations inside the persistent launch, for fixed-count solves on both
    sides of the hand-over, for max_iter = 0 and for a NaN in the input."""
    import paper_2510_21450_amd as P
    B, L = shape
    H = 64
    W = normal(940 + L, 5, (H, H), std=0.8 / H ** 0.5, device="cuda")
    u = normal(940 + L, 1, (B, L, 1, H), device="cuda")
    h0 = normal(940 + L, 3, (B, 1, H), std=0.3, device="cuda")
    Wn, un, h0n = f64(W), f64(u), f64(h0)
    tol, want = well_posed_tol(oracle_mod, "tanh_dense", Wn, un, h0n, max_iter=32, probe_tol=1e-4)
    u_nan = u.clone(); u_nan[0, L // 2, 0, 5] = float("nan")
    cases = [dict(u=u, tol=tol, max_iter=32), dict(u=u, tol=0.0, max_iter=9), dict(u=u, tol=-1.0, max_iter=3),
             dict(u=u, tol=-1.0, max_iter=8), dict(u=u, tol=1e-30, max_iter=7), dict(u=u, tol=tol, max_iter=0),
             dict(u=u_nan, tol=tol, max_iter=32)]
    for case in cases:
        got = []
        for mode in (0, 1, 2):
            print(f"dense plans B={B} L={L} tol={case['tol']} max_iter={case['max_iter']} mode={mode}", flush=True)
            tail_mode(mode)
            h, iters, tr = P.forward("tanh_dense", W, case["u"], h0, tol=case["tol"], max_iter=case["max_iter"], trace=True)
            torch.cuda.synchronize()
            got.append((h.clone(), iters.cpu().tolist(), tr.cpu().numpy().copy()))
        for mode, (h, it, tr) in zip((1, 2), got[1:]):
            what = (case["tol"], case["max_iter"], mode)
            assert it == got[0][1], (what, it, got[0][1])
            assert np.array_equal(tr, got[0][2], equal_nan=True), what
            # bit for bit, except that a NaN may carry another sign or payload
            differ = (h.view(torch.int32) != got[0][0].view(torch.int32)) & ~(torch.isnan(h) & torch.isnan(got[0][0]))
            assert not bool(differ.any()), (what, int(differ.sum()), torch.nonzero(differ)[:6].tolist(),
                                            h[differ][:6].tolist(), got[0][0][differ][:6].tolist())
    # and the first case is the oracle's solve
    tail_mode(1)
    h, iters, _ = P.forward("tanh_dense", W, u, h0, tol=tol, max_iter=32)
    assert iters.cpu().tolist() == [want, 0]
    assert relerr(f64(h), oracle_mod.seq_unroll("tanh_dense", Wn, un, h0n)) <= 1e-5


def test_dense_persistent_launch_gives_up_after_a_bounded_wait(tail_mode):
    """The grid-wide barriers of the persistent launch wait a bounded number of polls.  With the limit
    forced to one poll a workgroup that is not the last to arrive gives up: every workgroup still
    exits, the status says INTERNAL (or the solve went through), and the next call works."""
    import paper_2510_21450_amd as P
    w = CONFIGS["C4"].scaled(B=16, L=512)
    d = make_inputs(w, device="cuda")
    seen = set()
    try:
        P.set_spin_limit(1)
        tail_mode(2)
        for rep in range(3):
            _, iters, _ = P.forward(w.cell, d["params"], d["u"], None, tol=w.tol, max_iter=8)
            torch.cuda.synchronize()
            seen.add(P.status_string(int(iters.cpu()[1])))
    finally:
        P.set_spin_limit(0)
    print(f"dense persistent launch, one poll: statuses {sorted(seen)}", flush=True)
    assert seen <= {"OK", "INTERNAL", "NOT_CONVERGED"}
    h, iters, _ = P.forward(w.cell, d["params"], d["u"], None, tol=w.tol, max_iter=32)
    torch.cuda.synchronize()
    assert int(iters.cpu()[1]) == 0
