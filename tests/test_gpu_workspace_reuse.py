"""pararnn_set_workspace_reuse: with the caller's promise that nothing else writes to a workspace
between calls, the carry records are not cleared again for a call of the same layout (their tags carry a
per-call number instead).  Results must be the bits of the default path, whatever the workspace held."""
import os
import sys

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
from workloads import CONFIGS, make_inputs, cell_dims      # noqa: E402


def run_pair(P, w, d, ws_f, ws_b, max_iter=16, first_block=-1):
    h, iters, tr = P.forward_ex(w.cell, d["params"], d["u"], d["h0"], tol=w.tol, max_iter=max_iter, first_block=first_block,
                                trace=True, workspace=ws_f)
    du, dp, dh0 = P.backward(w.cell, d["params"], d["u"], d["h0"], h, d["g"], workspace=ws_b)
    torch.cuda.synchronize()
    return h.clone(), iters.cpu().clone(), tr.cpu().clone(), du.clone(), dp.clone(), dh0.clone()


def same(a, b):
    return all(torch.equal(x, y) for x, y in zip(a, b))


@pytest.mark.parametrize("name,dtype", [("C2", "f32"), ("C3", "f32"), ("C5", "bf16")])
def test_reused_workspaces_give_the_same_bits(name, dtype):
    """Five calls in a row on the same two workspaces with different inputs each time (so that every
    record of the call before holds a valid-looking value of another problem), several tiles per
    sequence, first blocks short enough that the tail launch and the per-iteration kernel run too;
    then another shape on the same memory, and the first shape again."""
    import paper_2510_21450_amd as P
    base = CONFIGS[name]
    w = base.scaled(B=3, L=1500, H=136)
    w2 = base.scaled(B=2, L=700, H=264)
    sizes = [P.workspace_bytes(x.cell, torch.bfloat16 if dtype == "bf16" else torch.float32, x.B, x.L, x.H, bw)
             for x in (w, w2) for bw in (False, True)]
    ws_f = torch.empty(max(sizes), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(max(sizes), dtype=torch.uint8, device="cuda")
    problems = []
    for k in range(5):
        wk = (w if k != 3 else w2).scaled(seed=base.seed + 10 * k)
        problems.append((wk, make_inputs(wk, device="cuda")))
    want = []
    for wk, d in problems:
        ws_f.random_(0, 256); ws_b.random_(0, 256)          # the default path does not care what it finds
        want.append(run_pair(P, wk, d, ws_f, ws_b, first_block=2))
    try:
        P.set_workspace_reuse(True)
        ws_f.random_(0, 256); ws_b.random_(0, 256)          # first use of these addresses: cleared like always
        for rep in range(2):
            for k, (wk, d) in enumerate(problems):
                print(f"workspace reuse {name} round {rep} problem {k}", flush=True)
                got = run_pair(P, wk, d, ws_f, ws_b, first_block=2)
                assert same(got, want[k]), (rep, k)
        # another entry point of the library on the same memory: the next call clears again
        d0 = problems[0][1]
        G, S = cell_dims(w.cell)
        if S == 1:
            J = torch.rand((2, 300, 64), device="cuda") * 0.5
            r = torch.randn((2, 300, 64), device="cuda")
            P.affine_scan(J, r, workspace=ws_f)             # a small scan: its records overwrite the start of the solve's
        else:
            ws_f.random_(0, 256)
            P.set_workspace_reuse(False)                    # what a caller must do before writing there itself ...
            P.forward(w.cell, d0["params"], d0["u"], d0["h0"], tol=w.tol, max_iter=16, workspace=ws_f)
            P.set_workspace_reuse(True)                     # ... and the call without the promise has forgotten the workspace
        got = run_pair(P, problems[0][0], d0, ws_f, ws_b, first_block=2)
        assert same(got, want[0])
    finally:
        P.set_workspace_reuse(False)
    # and the default again
    ws_f.random_(0, 256); ws_b.random_(0, 256)
    assert same(run_pair(P, problems[1][0], problems[1][1], ws_f, ws_b, first_block=2), want[1])


def test_reuse_under_graph_capture_clears_every_time():
    """A captured launch sequence replays one call number, so calls that are being captured clear their
    records: replays with changing inputs give the eager results."""
    import paper_2510_21450_amd as P
    w = CONFIGS["C2"].scaled(B=2, L=900, H=192)
    G, S = cell_dims(w.cell)
    d = make_inputs(w, device="cuda")
    params, u, g = d["params"], d["u"].clone(), d["g"]
    ws_f = torch.empty(P.workspace_bytes(w.cell, u.dtype, w.B, w.L, w.H), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(P.workspace_bytes(w.cell, u.dtype, w.B, w.L, w.H, True), dtype=torch.uint8, device="cuda")
    h = torch.empty((w.B, w.L, S, w.H), device="cuda")
    outs = (torch.empty_like(u), torch.empty_like(params), torch.empty((w.B, S, w.H), device="cuda"))
    try:
        P.set_workspace_reuse(True)
        P.forward(w.cell, params, u, None, tol=w.tol, max_iter=16, workspace=ws_f)       # the addresses are known now
        P.backward(w.cell, params, u, None, h.zero_(), g, workspace=ws_b)
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                _, iters, _ = P.forward(w.cell, params, u, None, tol=w.tol, max_iter=16, workspace=ws_f, out=h)
                P.backward(w.cell, params, u, None, h, g, workspace=ws_b, out=outs)
        torch.cuda.current_stream().wait_stream(side)
        for rep in range(3):
            u.copy_(d["u"] * (1.0 + 0.25 * rep))
            graph.replay()
            torch.cuda.synchronize()
            got = (h.clone(), iters.cpu().clone(), outs[0].clone(), outs[1].clone(), outs[2].clone())
            P.set_workspace_reuse(False)
            ws2_f, ws2_b = torch.empty_like(ws_f), torch.empty_like(ws_b)
            h_e, it_e, _ = P.forward(w.cell, params, u, None, tol=w.tol, max_iter=16, workspace=ws2_f)
            du_e, dp_e, dh0_e = P.backward(w.cell, params, u, None, h_e, g, workspace=ws2_b)
            torch.cuda.synchronize()
            P.set_workspace_reuse(True)
            assert same(got, (h_e, it_e.cpu(), du_e, dp_e, dh0_e)), rep
    finally:
        P.set_workspace_reuse(False)


def test_reuse_on_the_library_own_scratch():
    """pararnn_forward_noalloc keeps its workspace inside the library, so the promise holds by itself:
    the same problem twice (second call: records not cleared), another input, a smaller shape (another
    layout: cleared), against pararnn_forward on a caller's workspace."""
    import paper_2510_21450_amd as P
    from workloads.rng import normal, uniform_sym
    cell = "gru_diag"
    G, S = cell_dims(cell)

    def solve(B, L, H, seed, scale):
        params = torch.zeros(2, G, H, device="cuda")
        params[0] = uniform_sym(seed, 2, (G, H), 0.9, device="cuda")
        u = normal(seed, 1, (B, L, G, H), device="cuda") * scale
        h0 = normal(seed, 3, (B, S, H), std=0.3, device="cuda")
        P.set_workspace_reuse(False)
        h_ref, it_ref, _ = P.forward(cell, params, u, h0, tol=1e-5, max_iter=24)
        torch.cuda.synchronize()
        P.set_workspace_reuse(True)
        h = torch.full((B, L, S, H), float("nan"), device="cuda")
        iters = torch.full((2,), -1, dtype=torch.int32, device="cuda")
        code = P.forward_noalloc(cell, params, u, h0, 1e-5, 24, h, iters)
        torch.cuda.synchronize()
        assert code == 0, P.status_string(code)
        assert iters.cpu().tolist() == it_ref.cpu().tolist() and torch.equal(h, h_ref)

    try:
        for B, L, H, seed, scale in ((2, 1200, 128, 71, 1.0), (2, 1200, 128, 71, 1.0), (2, 1200, 128, 72, 1.3),
                                     (1, 500, 64, 73, 1.0), (2, 1200, 128, 71, 0.7)):
            print(f"noalloc with reuse B={B} L={L} H={H} seed={seed} scale={scale}", flush=True)
            solve(B, L, H, seed, scale)
    finally:
        P.set_workspace_reuse(False)
