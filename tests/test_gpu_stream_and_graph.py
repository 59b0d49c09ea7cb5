"""The library only enqueues work: a forward solve and a backward pass can be
recorded into a HIP graph (no host synchronisation, no allocation, no memset
node inside) and replayed, and they run correctly on a non-default stream."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

# Where each side runs the whole chain on its own (forward solve, then the backward pass at its own
# states) the gradients differ by the backward pass's own 1e-5 plus the effect of the <= 1e-5
# difference between the two sets of states, which the adjoint recursion carries along a sequence.
CHAIN_TOL = 3e-5

from workloads import CONFIGS, make_inputs, cell_dims      # noqa: E402


def f64(t):
    return None if t is None else t.detach().to("cpu", torch.float64).numpy()


def relerr(got, ref):
    return float(np.max(np.abs(got - ref)) / max(np.max(np.abs(ref)), 1e-30))


def test_forward_and_backward_replay_from_a_graph(oracle_mod):
    import paper_2510_21450_amd as P
    w = CONFIGS["C2"].scaled(B=2, L=600, H=192)
    G, S = cell_dims(w.cell)
    d = make_inputs(w, device="cuda")
    params, u, g = d["params"], d["u"], d["g"]
    ws_f = torch.empty(P.workspace_bytes(w.cell, u.dtype, w.B, w.L, w.H), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(P.workspace_bytes(w.cell, u.dtype, w.B, w.L, w.H, True), dtype=torch.uint8, device="cuda")
    h = torch.empty((w.B, w.L, S, w.H), device="cuda")
    outs = (torch.empty_like(u), torch.empty_like(params), torch.empty((w.B, S, w.H), device="cuda"))
    # eager reference
    h_e, it_e, _ = P.forward(w.cell, params, u, None, tol=w.tol, max_iter=16, workspace=ws_f)
    du_e, dp_e, dh0_e = P.backward(w.cell, params, u, None, h_e, g, workspace=ws_b)
    torch.cuda.synchronize()
    it_e = it_e.cpu().clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            _, iters, _ = P.forward(w.cell, params, u, None, tol=w.tol, max_iter=16, workspace=ws_f, out=h)
            P.backward(w.cell, params, u, None, h, g, workspace=ws_b, out=outs)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        # clobber the outputs, do unrelated eager work, then replay
        h.fill_(float("nan")); outs[0].zero_(); outs[1].zero_(); outs[2].zero_(); iters.zero_()
        _ = (u.float() * 2).sum().item()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(iters.cpu(), it_e), rep
        assert torch.equal(h, h_e), rep
        assert torch.equal(outs[0], du_e) and torch.equal(outs[2], dh0_e), rep
        assert torch.equal(outs[1], dp_e), rep            # fixed-order reduction: bit-reproducible
    ref = oracle_mod.seq_unroll(w.cell, f64(params), f64(u), None)
    assert relerr(f64(h), ref) <= 1e-5


@pytest.mark.parametrize("jacobian", [0, 1])
def test_dense_solve_and_residual_norm_replay_from_a_graph(jacobian):
    """The dense cell's solve (Newton, and the quasi-Newton mode chosen at capture time) followed by
    the residual max-norm of its result, recorded into a HIP graph and replayed with eager work in
    between: every replay equals the eager result bit for bit."""
    import paper_2510_21450_amd as P
    from workloads.rng import normal
    B, L, H = 3, 300, 64
    W = normal(77, 5, (H, H), std=0.8 / H ** 0.5, device="cuda")
    u = normal(77, 1, (B, L, 1, H), device="cuda")
    h0 = normal(77, 3, (B, 1, H), std=0.3, device="cuda")
    ws = torch.empty(P.workspace_bytes("tanh_dense", u.dtype, B, L, H), dtype=torch.uint8, device="cuda")
    h = torch.empty_like(u)
    rn = torch.empty(1, device="cuda")
    P.set_dense_jacobian(jacobian)
    try:
        h_e, it_e, _ = P.forward("tanh_dense", W, u, h0, tol=1e-5, max_iter=60, workspace=ws)
        rn_e = P.residual_norm("tanh_dense", W, u, h0, h_e)
        torch.cuda.synchronize()
        h_e, it_e, rn_e = h_e.clone(), it_e.cpu().clone(), rn_e.cpu().clone()
        assert int(it_e[1]) == 0 and float(rn_e) < 1e-4
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                _, iters, _ = P.forward("tanh_dense", W, u, h0, tol=1e-5, max_iter=60, workspace=ws, out=h)
                P.residual_norm("tanh_dense", W, u, h0, h, out=rn)
        torch.cuda.current_stream().wait_stream(side)
    finally:
        P.set_dense_jacobian(0)
    for rep in range(3):
        h.fill_(float("nan")); iters.zero_(); rn.fill_(7.0)
        _ = (u * 2).sum().item()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(iters.cpu(), it_e) and torch.equal(h, h_e) and torch.equal(rn.cpu(), rn_e), rep


def test_runs_on_a_side_stream(oracle_mod, as_stored):
    import paper_2510_21450_amd as P
    w = CONFIGS["C3"].scaled(B=2, L=300, H=96)
    d = make_inputs(w, device="cuda")
    ref = oracle_mod.seq_unroll(w.cell, f64(d["params"]), f64(d["u"]), None)
    hs = as_stored(ref, d["u"])             # backward: both sides at the oracle's states
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        h, iters, _ = P.forward(w.cell, d["params"], d["u"], None, tol=w.tol, max_iter=32)
        du, dp, dh0 = P.backward(w.cell, d["params"], d["u"], None, hs, d["g"])
    s.synchronize()
    assert int(iters.cpu()[1]) == 0
    assert relerr(f64(h), ref) <= 1e-5
    rdu, rdp, rdh0 = oracle_mod.backward(w.cell, f64(d["params"]), f64(d["u"]), None, f64(hs), f64(d["g"]))
    assert relerr(f64(du), rdu) <= 1e-5 and relerr(f64(dp), rdp) <= 1e-5


def test_repeated_calls_share_a_workspace_and_are_bit_reproducible():
    import paper_2510_21450_amd as P
    w = CONFIGS["C2"].scaled(B=3, L=1000, H=200)
    d = make_inputs(w, device="cuda")
    ws = torch.empty(P.workspace_bytes(w.cell, d["u"].dtype, w.B, w.L, w.H), dtype=torch.uint8, device="cuda")
    ws.fill_(0xAB)           # the workspace needs no initialisation
    first = None
    for rep in range(4):
        h, iters, tr = P.forward(w.cell, d["params"], d["u"], None, tol=w.tol, max_iter=32, trace=True, workspace=ws)
        torch.cuda.synchronize()
        cur = (h.clone(), iters.cpu().clone(), tr.cpu().clone())
        if first is None:
            first = cur
        else:
            assert torch.equal(cur[0], first[0]) and torch.equal(cur[1], first[1]) and torch.equal(cur[2], first[2])


@pytest.mark.parametrize("cell", ["gru_diag", "lstm_diag"])
def test_lookback_stress_many_small_tiles(cell, oracle_mod):
    """The carry chain under stress: the smallest tile shape (8 channels x 64
    steps) on long sequences gives hundreds of tiles per chain and thousands of
    workgroups racing for tickets; whatever order they run in, forward and
    backward must give the same bits every time, and the oracle's result."""
    import paper_2510_21450_amd as P
    w = CONFIGS["C2" if cell == "gru_diag" else "C3"].scaled(B=4, L=20000, H=8)
    d = make_inputs(w, device="cuda")
    ws = torch.empty(P.workspace_bytes(w.cell, d["u"].dtype, w.B, w.L, w.H), dtype=torch.uint8, device="cuda")
    ws.random_(0, 255)       # garbage, including tags that look almost valid
    first = None
    for rep in range(12):
        h, iters, _ = P.forward(w.cell, d["params"], d["u"], d["h0"], tol=w.tol, max_iter=32, workspace=ws)
        du, dp, dh0 = P.backward(w.cell, d["params"], d["u"], d["h0"], h, d["g"])
        torch.cuda.synchronize()
        cur = (h.clone(), iters.cpu().clone(), du.clone(), dp.clone(), dh0.clone())
        if first is None:
            first = cur
            assert int(cur[1][1]) == 0
        else:
            assert all(torch.equal(a, b) for a, b in zip(cur, first)), rep
    f64 = lambda t: None if t is None else t.detach().to("cpu", torch.float64).numpy()
    ref = oracle_mod.seq_unroll(w.cell, f64(d["params"]), f64(d["u"]), f64(d["h0"]))
    err = float(np.max(np.abs(f64(first[0]) - ref)) / np.max(np.abs(ref)))
    assert err <= 1e-5, err


@pytest.mark.parametrize("cell", ["gru_diag", "lstm_diag", "tanh_dense"])
def test_autograd_wrapper_matches_oracle_gradients(cell, oracle_mod):
    """rnn_apply inside a PyTorch graph: loss = sum(w * h), gradients with respect
    to params, u and h0 against the oracle's chain (its own states, then its reverse sweep).
    Each side runs forward and backward on its own here, so the bound is CHAIN_TOL."""
    import numpy as np
    import paper_2510_21450_amd as P
    from workloads.rng import normal, uniform_sym
    G, S = P.cell_dims(cell)
    B, L, H = 2, 300, 64
    if cell == "tanh_dense":
        params = normal(41, 5, (H, H), std=0.8 / H ** 0.5, device="cuda")
    else:
        params = torch.zeros(2, G, H, device="cuda")
        params[0] = uniform_sym(41, 2, (G, H), 0.9, device="cuda")
    u = normal(41, 1, (B, L, G, H), device="cuda")
    h0 = normal(41, 3, (B, S, H), std=0.3, device="cuda")
    w = normal(41, 4, (B, L, S, H), device="cuda")
    params.requires_grad_(True); u.requires_grad_(True); h0.requires_grad_(True)
    h, iters = P.rnn_apply(cell, params, u, h0, tol=1e-5, max_iter=40)
    assert int(iters.cpu()[1]) == 0 and not iters.requires_grad
    (h * w).sum().backward()
    f64 = lambda t: t.detach().to("cpu", torch.float64).numpy()
    ref = oracle_mod.seq_unroll(cell, f64(params), f64(u), f64(h0))
    rdu, rdp, rdh0 = oracle_mod.backward(cell, f64(params), f64(u), f64(h0), ref, f64(w))
    rel = lambda a, b: float(np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-30))
    errs = (rel(f64(h), ref), rel(f64(u.grad), rdu), rel(f64(params.grad), rdp), rel(f64(h0.grad), rdh0))
    print(f"autograd chain {cell}: rel err h, du, dparams, dh0 = {errs}", flush=True)
    assert errs[0] <= 1e-5 and max(errs[1:]) <= CHAIN_TOL
    # without h0 the wrapper asks for no dL/dh0
    u2 = u.detach().clone().requires_grad_(True)
    h2, _ = P.rnn_apply(cell, params.detach(), u2, None, tol=1e-5, max_iter=40)
    h2.sum().backward()
    assert u2.grad is not None and bool(torch.isfinite(u2.grad).all())


@pytest.mark.parametrize("cell", ["gru_diag", "lstm_diag"])
def test_bounded_wait_gives_up_cleanly(cell, oracle_mod):
    """The look-back wait is bounded: with the limit forced to a single poll from the
    host, a tile whose predecessor has not published yet gives up, the status becomes
    INTERNAL (or the solve happens to succeed), every wave exits, and the next call
    with the default limit is correct again.  Forward (fused blocks and one launch
    per iteration) and backward."""
    import paper_2510_21450_amd as P
    w = CONFIGS["C2" if cell == "gru_diag" else "C3"].scaled(B=4, L=20000, H=64)
    d = make_inputs(w, device="cuda")
    try:
        P.set_spin_limit(1)
        seen = set()
        for fused in (True, False):
            P.set_fused(fused)
            for rep in range(3):
                h, iters, _ = P.forward(w.cell, d["params"], d["u"], d["h0"], tol=w.tol, max_iter=8)
                du, dp, dh0 = P.backward(w.cell, d["params"], d["u"], d["h0"], h, d["g"])
                torch.cuda.synchronize()
                seen.add(P.status_string(int(iters.cpu()[1])))
        print(f"{cell}: statuses with one poll: {sorted(seen)}", flush=True)
        assert seen <= {"OK", "INTERNAL", "NOT_CONVERGED"}
    finally:
        P.set_spin_limit(0)
        P.set_fused(True)
    h, iters, _ = P.forward(w.cell, d["params"], d["u"], d["h0"], tol=w.tol, max_iter=32)
    torch.cuda.synchronize()
    assert int(iters.cpu()[1]) == 0
    ref = oracle_mod.seq_unroll(w.cell, f64(d["params"]), f64(d["u"]), f64(d["h0"]))
    assert relerr(f64(h), ref) <= 1e-5
