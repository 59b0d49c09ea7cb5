"""GPU parity of the cells added through include/pararnn_cell.h (the example
libraries under paper_2510_21450_amd/user_cells/): the GRU with other nonlinearities
(selectable nonlinearities, App. D.3: a softsign state; identity, softsign and tanh reset gates with
tanh, identity and softsign states.  The update gate stays a sigmoid: with a range beyond [0, 1] the
step h' = (1 - z) h + z c expands the state wherever z < 0 and the recurrence itself diverges on
sequences of a few hundred steps, in the oracle as on the GPU) and from-scratch cells with
2x2, 3x3 and 4x4 Jacobian blocks.  Same bars as the built-in cells: fp32 1e-5 norm-wise
against the fp64 oracle, bf16 storage 2e-2, iteration counts exact (the tolerance
of every case sits inside a jump of the oracle's fp64 and fp32 traces)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from workloads.rng import normal, uniform_sym               # noqa: E402
from parity_util import well_posed_tol                      # noqa: E402

TOL_F32 = 1e-5
TOL_BF16 = 2e-2
TOL_CHAIN = 3e-5        # forward and backward run by each side on its own: the backward's 1e-5 plus the effect of states that differ by <= 1e-5
ORACLE_NAME = {"gru_softsign": "gru_nl:sigmoid,sigmoid,softsign", "rot_tanh": "rot_tanh", "tri_tanh": "tri_tanh",
               "quad_tanh": "quad_tanh", "gru_sigmoid_identity_tanh": "gru_nl:sigmoid,identity,tanh",
               "gru_sigmoid_softsign_identity": "gru_nl:sigmoid,softsign,identity",
               "gru_sigmoid_tanh_softsign": "gru_nl:sigmoid,tanh,softsign"}
ALL_CELLS = list(ORACLE_NAME)


def relerr(got, ref):
    got = np.asarray(got, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    return float(np.max(np.abs(got - ref)) / max(np.max(np.abs(ref)), 1e-30))


def to_np(t):
    return None if t is None else t.detach().to("cpu", torch.float64).numpy()


def problem(cell, B, L, H, seed, dtype=torch.float32):
    dev = "cuda"
    if cell.name == "rot_tanh":
        params = uniform_sym(seed, 2, (2, H), 0.6, device=dev)
    elif cell.name == "tri_tanh":
        params = uniform_sym(seed, 2, (9, H), 0.45, device=dev)
    elif cell.name == "quad_tanh":
        params = uniform_sym(seed, 2, (16, H), 0.34, device=dev)
    else:
        params = torch.zeros(2, cell.G, H, device=dev)
        params[0] = uniform_sym(seed, 2, (cell.G, H), 0.9, device=dev)
        params[1] = normal(seed, 6, (cell.G, H), std=0.3, device=dev)
    u = normal(seed, 1, (B, L, cell.G, H), dtype=dtype, device=dev)
    h0 = normal(seed, 3, (B, cell.S, H), std=0.3, dtype=dtype, device=dev)
    g = normal(seed, 4, (B, L, cell.S, H), dtype=dtype, device=dev)
    return params, u, h0, g


SHAPES = [(1, 1, 8), (2, 33, 1), (2, 100, 24), (3, 257, 68), (2, 1000, 130), (1, 65, 6), (2, 3000, 64)]


@pytest.mark.parametrize("name", ALL_CELLS)
@pytest.mark.parametrize("shape", SHAPES)
def test_user_cell_forward_backward_f32(oracle_mod, as_stored, name, shape):
    import paper_2510_21450_amd as P
    cell = P.example_cell(name)
    oname = ORACLE_NAME[name]
    assert (cell.G, cell.S) == oracle_mod.dims(oname)
    B, L, H = shape
    print(f"case {name} B={B} L={L} H={H}", flush=True)
    params, u, h0, g = problem(cell, B, L, H, seed=3000 + L * 7 + H)
    pn, un, h0n, gn = to_np(params), to_np(u), to_np(h0), to_np(g)
    tol, want = well_posed_tol(oracle_mod, oname, pn, un, h0n, max_iter=40)
    h, iters, tr = P.forward(cell, params, u, h0, tol=tol, max_iter=40, trace=True)
    torch.cuda.synchronize()
    it, st = (int(x) for x in iters.cpu())
    ref = oracle_mod.seq_unroll(oname, pn, un, h0n)
    assert st == 0, P.status_string(st)
    assert relerr(to_np(h), ref) <= TOL_F32
    assert it == want, (it, want, tol, tr.cpu().numpy()[:it])
    hs = as_stored(ref, h)          # backward: both sides at the oracle's states
    du, dp, dh0 = P.backward(cell, params, u, h0, hs, g)
    torch.cuda.synchronize()
    rdu, rdp, rdh0 = oracle_mod.backward(oname, pn, un, h0n, to_np(hs), gn)
    assert relerr(to_np(du), rdu) <= TOL_F32
    assert relerr(to_np(dp), rdp) <= TOL_F32
    assert relerr(to_np(dh0), rdh0) <= TOL_F32


@pytest.mark.parametrize("name", ALL_CELLS)
@pytest.mark.parametrize("fused", [True, False])
def test_user_cell_per_iteration_and_fused_paths_agree(oracle_mod, name, fused):
    """Every launch kind is instantiated for a user cell: fused blocks (default),
    one kernel per iteration, a fixed-count solve in one launch; each against the
    oracle's iterate after the same number of iterations."""
    import paper_2510_21450_amd as P
    cell = P.example_cell(name)
    oname = ORACLE_NAME[name]
    params, u, h0, _ = problem(cell, 2, 700, 96, seed=3100)
    pn, un, h0n = to_np(params), to_np(u), to_np(h0)
    P.set_fused(fused)
    try:
        for n_it in (1, 3):
            h, iters, tr = P.forward(cell, params, u, h0, tol=-1.0, max_iter=n_it, trace=True)
            torch.cuda.synchronize()
            ref, _, _, rtr = oracle_mod.newton(oname, pn, un, h0n, tol=-1.0, max_iter=n_it)
            assert tuple(int(x) for x in iters.cpu()) == (n_it, 0)
            assert relerr(to_np(h), ref) <= TOL_F32
            assert np.allclose(tr.cpu().numpy()[:n_it], rtr, rtol=1e-3, atol=1e-6)
    finally:
        P.set_fused(True)


@pytest.mark.parametrize("name", ALL_CELLS)
def test_user_cell_bf16_storage(oracle_mod, as_stored, name):
    import paper_2510_21450_amd as P
    cell = P.example_cell(name)
    oname = ORACLE_NAME[name]
    params, u, h0, g = problem(cell, 2, 900, 128, seed=3200, dtype=torch.bfloat16)
    h, iters, _ = P.forward(cell, params, u, h0, tol=1e-3, max_iter=40)
    torch.cuda.synchronize()
    assert int(iters.cpu()[1]) == 0
    pn, un, h0n, gn = to_np(params), to_np(u), to_np(h0), to_np(g)
    ref = oracle_mod.seq_unroll(oname, pn, un, h0n)
    assert relerr(to_np(h), ref) <= TOL_BF16
    hs = as_stored(ref, h)
    du, dp, dh0 = P.backward(cell, params, u, h0, hs, g)
    torch.cuda.synchronize()
    rdu, rdp, rdh0 = oracle_mod.backward(oname, pn, un, h0n, to_np(hs), gn)
    assert relerr(to_np(du), rdu) <= TOL_BF16 and relerr(to_np(dp), rdp) <= TOL_BF16 and relerr(to_np(dh0), rdh0) <= TOL_BF16


def test_user_cell_through_autograd(oracle_mod):
    import paper_2510_21450_amd as P
    cell = P.example_cell("rot_tanh")
    params, u, h0, w = problem(cell, 2, 300, 64, seed=3300)
    params.requires_grad_(True); u.requires_grad_(True); h0.requires_grad_(True)
    h, iters = P.rnn_apply(cell, params, u, h0, tol=1e-5, max_iter=40)
    assert int(iters.cpu()[1]) == 0
    (h * w).sum().backward()
    # each side runs its own chain here: the oracle's reverse sweep is taken at the oracle's states
    ref = oracle_mod.seq_unroll("rot_tanh", to_np(params), to_np(u), to_np(h0))
    rdu, rdp, rdh0 = oracle_mod.backward("rot_tanh", to_np(params), to_np(u), to_np(h0), ref, to_np(w))
    errs = (relerr(to_np(h), ref), relerr(to_np(u.grad), rdu), relerr(to_np(params.grad), rdp), relerr(to_np(h0.grad), rdh0))
    print(f"autograd chain rot_tanh: rel err h, du, dparams, dh0 = {errs}", flush=True)
    assert errs[0] <= TOL_F32 and max(errs[1:]) <= TOL_CHAIN


def test_block_cells_refuse_tile_shapes_that_are_not_built():
    """For 3x3 and 4x4 blocks only the tile shapes with few steps per thread are instantiated: a
    forced shape outside them is refused by the host (UNSUPPORTED), an offered one works."""
    import paper_2510_21450_amd as P
    for name, offered, refused in (("tri_tanh", (1, 1, 4, 8), (1, 1, 16, 8)), ("quad_tanh", (1, 8, 4, 2), (1, 1, 8, 8))):
        cell = P.example_cell(name)
        params, u, h0, g = problem(cell, 2, 200, 64, seed=3400)
        try:
            P.set_tile(*refused)
            with pytest.raises(RuntimeError, match="UNSUPPORTED"):
                P.forward(cell, params, u, h0, tol=1e-5, max_iter=8)
            with pytest.raises(RuntimeError, match="UNSUPPORTED"):
                P.backward(cell, params, u, h0, torch.zeros_like(g), g)
            P.set_tile(*offered)
            h, iters, _ = P.forward(cell, params, u, h0, tol=1e-5, max_iter=40)
            torch.cuda.synchronize()
            assert int(iters.cpu()[1]) == 0
        finally:
            P.set_tile(0)
