"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on
identical seeded inputs.  fp32 results must agree to 1e-5 (norm-wise max
relative error: max|x - ref| / max|ref| per tensor), bf16-storage results to
2e-2, iteration counts exactly."""
import json
import os

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from workloads import CONFIGS, make_inputs, cell_dims      # noqa: E402
from workloads.rng import normal, uniform_sym               # noqa: E402
from parity_util import well_posed_tol                      # noqa: E402

TOL_F32 = 1e-5
TOL_BF16 = 2e-2
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "newton_traces.json")


@pytest.fixture(scope="module")
def P():
    import paper_2510_21450_amd as P
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return P


def relerr(got, ref):
    """max |got - ref| / max |ref| (norm-wise, infinity norm)."""
    got = np.asarray(got, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    return float(np.max(np.abs(got - ref)) / max(np.max(np.abs(ref)), 1e-30))


def to_np(t):
    return None if t is None else t.detach().to("cpu", torch.float64).numpy()


def problem(cell, B, L, H, seed, dtype=torch.float32, h0=True, bias=True, bound=0.9):
    """Random problem with nonzero biases and h0, on the GPU, plus fp64 host copies."""
    G, S = cell_dims(cell)
    dev = "cuda"
    if cell == "tanh_dense":
        params = normal(seed, 5, (H, H), std=0.8 / H ** 0.5, device=dev)
    elif cell == "paralstm_diag":       # a_f, a_z, a_o, c_f, c_o, b_f, b_z, b_o
        params = torch.zeros(8, H, device=dev)
        params[:5] = uniform_sym(seed, 2, (5, H), bound, device=dev)
        if bias:
            params[5:] = normal(seed, 6, (3, H), std=0.3, device=dev)
    else:
        params = torch.zeros(2, G, H, device=dev)
        params[0] = uniform_sym(seed, 2, (G, H), bound, device=dev)
        if bias:
            params[1] = normal(seed, 6, (G, H), std=0.3, device=dev)
    u = normal(seed, 1, (B, L, G, H), dtype=dtype, device=dev)
    h0t = normal(seed, 3, (B, S, H), std=0.3, dtype=dtype, device=dev) if h0 else None
    g = normal(seed, 4, (B, L, S, H), dtype=dtype, device=dev)
    return params, u, h0t, g


SHAPES = [(1, 1, 8), (1, 2, 4), (2, 33, 1), (2, 100, 24), (3, 257, 68), (2, 1000, 130), (1, 31, 64),
          (1, 32, 256), (2, 64, 512), (1, 65, 6)]


@pytest.mark.parametrize("cell", ["gru_diag", "lstm_diag", "paralstm_diag"])
@pytest.mark.parametrize("shape", SHAPES)
def test_forward_backward_f32_small(P, oracle_mod, as_stored, cell, shape):
    B, L, H = shape
    print(f"case {cell} B={B} L={L} H={H}", flush=True)
    params, u, h0, g = problem(cell, B, L, H, seed=1000 + L * 7 + H)
    pn, un, h0n, gn = to_np(params), to_np(u), to_np(h0), to_np(g)
    # a tolerance inside a jump of the oracle's fp64 and fp32 traces (8x room on both sides): the
    # iteration count is then well defined and compared exactly
    tol, want = well_posed_tol(oracle_mod, cell, pn, un, h0n, max_iter=40)
    h, iters, tr = P.forward(cell, params, u, h0, tol=tol, max_iter=40, trace=True)
    torch.cuda.synchronize()
    it, st = (int(x) for x in iters.cpu())
    ref = oracle_mod.seq_unroll(cell, pn, un, h0n)
    assert st == 0, P.status_string(st)
    assert relerr(to_np(h), ref) <= TOL_F32
    assert it == want, (it, want, tol, tr.cpu().numpy()[:it])
    # backward: both sides at the oracle's states
    hs = as_stored(ref, h)
    du, dp, dh0 = P.backward(cell, params, u, h0, hs, g)
    torch.cuda.synchronize()
    rdu, rdp, rdh0 = oracle_mod.backward(cell, pn, un, h0n, to_np(hs), gn)
    assert relerr(to_np(du), rdu) <= TOL_F32
    assert relerr(to_np(dp), rdp) <= TOL_F32
    assert relerr(to_np(dh0), rdh0) <= TOL_F32


def test_config_c1(P, oracle_mod):
    """Benchmark configuration 1: GRU, B=1, L=64, H=8, tol 1e-6, max_iter 64, forward."""
    w = CONFIGS["C1"]
    d = make_inputs(w, device="cuda")
    h, iters, tr = P.forward(w.cell, d["params"], d["u"], d["h0"], tol=w.tol, max_iter=w.max_iter, trace=True)
    torch.cuda.synchronize()
    it, st = (int(x) for x in iters.cpu())
    pn, un = to_np(d["params"]), to_np(d["u"])
    ref = oracle_mod.seq_unroll(w.cell, pn, un, None)
    assert st == 0 and relerr(to_np(h), ref) <= TOL_F32
    _, it32, _, tr32 = oracle_mod.newton(w.cell, pn, un, None, tol=w.tol, max_iter=w.max_iter, precision="f32")
    assert it == it32 == 5
    got = tr.cpu().numpy()[:it]
    # before the fp32 floor the per-iteration maxima agree closely
    assert np.allclose(got[:3], tr32[:3], rtol=1e-3)
    assert np.allclose(got[3], tr32[3], rtol=5e-2)     # 6.7e-6: fp32 rounding (~1e-7) shows


def test_linear_cell_one_solve_is_exact(P, oracle_mod):
    params, u, h0, _ = problem("linear_diag", 2, 300, 40, seed=7)
    h, iters, _ = P.forward("linear_diag", params, u, h0, tol=-1.0, max_iter=1)
    torch.cuda.synchronize()
    ref = oracle_mod.seq_unroll("linear_diag", to_np(params), to_np(u), to_np(h0))
    assert tuple(int(x) for x in iters.cpu()) == (1, 0)
    assert relerr(to_np(h), ref) <= TOL_F32
    # with a stopping test the second solve confirms: iters == 2
    h, iters, tr = P.forward("linear_diag", params, u, h0, tol=1e-4, max_iter=10, trace=True)
    assert tuple(int(x) for x in iters.cpu()) == (2, 0)


def test_iteration_control_edge_cases(P, oracle_mod):
    cell = "gru_diag"
    params, u, h0, _ = problem(cell, 2, 70, 12, seed=11)
    pn, un, h0n = to_np(params), to_np(u), to_np(h0)
    # max_iter = 0: the initial guess f(h0, u_l)
    h, iters, _ = P.forward(cell, params, u, h0, tol=1e-6, max_iter=0)
    hg, _, _, _ = oracle_mod.newton(cell, pn, un, h0n, tol=1e-6, max_iter=0)
    assert tuple(int(x) for x in iters.cpu()) == (0, 1)
    assert relerr(to_np(h), hg) <= TOL_F32
    # tol < 0: exactly max_iter solves, status OK; iterate k matches the oracle's iterate k
    for k in (1, 2, 3):
        h, iters, _ = P.forward(cell, params, u, h0, tol=-1.0, max_iter=k)
        hk, _, _, _ = oracle_mod.newton(cell, pn, un, h0n, tol=-1.0, max_iter=k)
        assert tuple(int(x) for x in iters.cpu()) == (k, 0)
        assert relerr(to_np(h), hk) <= 2e-5
    # not converged: last iterate, iters = max_iter, status NOT_CONVERGED
    h, iters, _ = P.forward(cell, params, u, h0, tol=0.0, max_iter=2)
    assert tuple(int(x) for x in iters.cpu()) == (2, 1)
    # L = 1: the guess is exact; one solve with delta = 0
    h, iters, tr = P.forward(cell, params, u[:, :1].contiguous(), h0, tol=0.0, max_iter=5, trace=True)
    assert tuple(int(x) for x in iters.cpu()) == (1, 0) and float(tr[0]) == 0.0
    # NaN in the input -> NONFINITE after the first solve
    u2 = u.clone(); u2[0, 3, 0, 0] = float("nan")
    h, iters, _ = P.forward(cell, params, u2, h0, tol=1e-6, max_iter=5)
    assert tuple(int(x) for x in iters.cpu()) == (1, 5)
    # h0 = None is zeros
    ha, _, _ = P.forward(cell, params, u, None, tol=1e-6, max_iter=20)
    hb, _, _ = P.forward(cell, params, u, torch.zeros_like(h0), tol=1e-6, max_iter=20)
    assert torch.equal(ha, hb)


def _misaligned(t, elems=1):
    """A contiguous copy of t whose data pointer is off by `elems` elements from the allocation."""
    flat = torch.empty(t.numel() + elems, dtype=t.dtype, device=t.device)
    out = flat[elems:].view(t.shape)
    out.copy_(t)
    assert out.is_contiguous() and out.data_ptr() % 16 != 0
    return out


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_pointers_without_vector_alignment(P, oracle_mod, as_stored, dtype):
    """Buffers that are only element-aligned (and an H that allows no vector
    width) must still work: the library falls back to narrower accesses."""
    cell = "gru_diag"
    bound = TOL_F32 if dtype == torch.float32 else TOL_BF16
    for H in (64, 66, 67):
        params, u, h0, g = problem(cell, 2, 150, H, seed=31 + H, dtype=dtype)
        pn, un, h0n, gn = to_np(params), to_np(u), to_np(h0), to_np(g)
        ref = oracle_mod.seq_unroll(cell, pn, un, h0n)
        hs = as_stored(ref, u)
        try:
            P.set_tile(2, 2, 8, 8)       # asks for 2 channels per lane; refused silently when not allowed
            um, h0m, gm, pm = _misaligned(u), _misaligned(h0), _misaligned(g), _misaligned(params)
            h, iters, _ = P.forward(cell, pm, um, h0m, tol=1e-5, max_iter=40)
            du, dp, dh0 = P.backward(cell, pm, um, h0m, _misaligned(hs), gm)
            torch.cuda.synchronize()
        finally:
            P.set_tile(0)
        assert int(iters.cpu()[1]) == 0
        assert relerr(to_np(h), ref) <= bound
        rdu, rdp, rdh0 = oracle_mod.backward(cell, pn, un, h0n, to_np(hs), gn)
        assert relerr(to_np(du), rdu) <= bound and relerr(to_np(dp), rdp) <= bound and relerr(to_np(dh0), rdh0) <= bound


def test_many_short_sequences_and_one_long(P, oracle_mod, as_stored):
    """Extreme aspect ratios: B*H large with tiny L, and one long sequence with few channels."""
    for cell, (B, L, H) in (("gru_diag", (300, 3, 40)), ("lstm_diag", (1, 20000, 8)), ("paralstm_diag", (64, 1, 130))):
        params, u, h0, g = problem(cell, B, L, H, seed=B + L)
        pn, un, h0n, gn = to_np(params), to_np(u), to_np(h0), to_np(g)
        ref = oracle_mod.seq_unroll(cell, pn, un, h0n)
        hs = as_stored(ref, u)
        h, iters, _ = P.forward(cell, params, u, h0, tol=1e-5, max_iter=40)
        du, dp, dh0 = P.backward(cell, params, u, h0, hs, g)
        torch.cuda.synchronize()
        assert int(iters.cpu()[1]) == 0
        assert relerr(to_np(h), ref) <= TOL_F32, (cell, B, L, H)
        rdu, rdp, rdh0 = oracle_mod.backward(cell, pn, un, h0n, to_np(hs), gn)
        assert relerr(to_np(du), rdu) <= TOL_F32 and relerr(to_np(dp), rdp) <= TOL_F32 and relerr(to_np(dh0), rdh0) <= TOL_F32


def test_invalid_arguments_are_rejected(P):
    params, u, h0, _ = problem("gru_diag", 1, 8, 8, seed=3)
    with pytest.raises(RuntimeError, match="INVALID_ARG"):
        P.forward("gru_diag", params, u, h0, tol=float("nan"))
    with pytest.raises(RuntimeError, match="INVALID_ARG"):
        P.forward("gru_diag", params, u, h0, max_iter=-1)
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(RuntimeError, match="WORKSPACE_TOO_SMALL"):
        P.forward("gru_diag", params, u, h0, workspace=small)


TILE_SHAPES = [(1, 1, 8, 16), (1, 2, 8, 16), (1, 2, 16, 4), (1, 2, 8, 8), (1, 1, 8, 8), (2, 2, 8, 8), (1, 1, 4, 8), (1, 1, 16, 8),
               (1, 8, 4, 2), (4, 4, 8, 8), (2, 4, 8, 8), (1, 1, 16, 4), (1, 1, 12, 8)]


@pytest.mark.parametrize("cell", ["gru_diag", "lstm_diag", "paralstm_diag"])
@pytest.mark.parametrize("tile", TILE_SHAPES)
def test_every_tile_shape(P, oracle_mod, as_stored, cell, tile):
    """Every compiled tile shape (channels per lane, segments per wave, steps
    per thread, waves per workgroup) on a problem spanning several tiles with
    ragged tails in L and H."""
    B, L, H = 2, 1100, 200
    print(f"tile {tile} {cell}", flush=True)
    params, u, h0, g = problem(cell, B, L, H, seed=4242)
    pn, un, h0n, gn = to_np(params), to_np(u), to_np(h0), to_np(g)
    ref = oracle_mod.seq_unroll(cell, pn, un, h0n)
    hs = as_stored(ref, u)
    try:
        P.set_tile(*tile)
        h, iters, _ = P.forward(cell, params, u, h0, tol=1e-5, max_iter=40)
        try:
            du, dp, dh0 = P.backward(cell, params, u, h0, hs, g)
        except RuntimeError as e:
            # wide LSTM tiles exceed the backward kernel's 64 KiB of LDS and are refused by the host
            if "UNSUPPORTED" in str(e) and cell != "gru_diag" and tile[0] * 64 // tile[1] * tile[3] >= 2048:
                pytest.skip("tile shape not offered for the LSTM backward kernel (LDS)")
            raise
        torch.cuda.synchronize()
    finally:
        P.set_tile(0)
    it, st = (int(x) for x in iters.cpu())
    assert st == 0
    assert relerr(to_np(h), ref) <= TOL_F32
    rdu, rdp, rdh0 = oracle_mod.backward(cell, pn, un, h0n, to_np(hs), gn)
    assert relerr(to_np(du), rdu) <= TOL_F32
    assert relerr(to_np(dp), rdp) <= TOL_F32
    assert relerr(to_np(dh0), rdh0) <= TOL_F32


@pytest.mark.parametrize("cell", ["gru_diag", "lstm_diag", "paralstm_diag"])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_fixed_count_solve_in_one_launch(P, oracle_mod, cell, dtype):
    """tol < 0 (the paper's fixed N_its): all iterations in one launch must give
    the oracle's iterate K, and the same iterate as one launch per iteration."""
    B, L, H = 2, 700, 100
    params, u, h0, _ = problem(cell, B, L, H, seed=2024, dtype=dtype)
    pn, un, h0n = to_np(params), to_np(u), to_np(h0)
    bound = 2e-5 if dtype == torch.float32 else TOL_BF16
    for tile in [None, (1, 2, 8, 8), (2, 2, 8, 8), (1, 1, 4, 8)]:
        for K in (1, 2, 3, 5, 8):
            print(f"fused {cell} {dtype} tile={tile} K={K}", flush=True)
            try:
                if tile:
                    P.set_tile(*tile)
                assert P.workspace_bytes_fused(cell, dtype, B, L, H, K) >= P.workspace_bytes(cell, dtype, B, L, H)
                hf, it_f, tr_f = P.forward(cell, params, u, h0, tol=-1.0, max_iter=K, trace=True)
                P.set_fused(False)
                hi, it_i, tr_i = P.forward(cell, params, u, h0, tol=-1.0, max_iter=K, trace=True)
                torch.cuda.synchronize()
            finally:
                P.set_fused(True)
                P.set_tile(0)
            hk, _, _, trk = oracle_mod.newton(cell, pn, un, h0n, tol=-1.0, max_iter=K)
            assert tuple(int(x) for x in it_f.cpu()) == (K, 0) == tuple(int(x) for x in it_i.cpu())
            assert relerr(to_np(hf), hk) <= bound
            assert relerr(to_np(hf), to_np(hi)) <= (2e-6 if dtype == torch.float32 else 1e-2)
            got = tr_f.cpu().numpy()[:K]
            for k in range(K):
                if trk[k] > 1e-4:
                    assert abs(got[k] - trk[k]) <= 2e-3 * trk[k], (k, got, trk)
    # a NaN in the input is reported with the first iteration it shows up in
    u2 = u.clone(); u2[0, 3, 0, 0] = float("nan")
    _, it, _ = P.forward(cell, params, u2, h0, tol=-1.0, max_iter=3)
    assert tuple(int(x) for x in it.cpu()) == (1, 5)


@pytest.mark.parametrize("S", [3, 4])
@pytest.mark.parametrize("reverse", [False, True])
def test_affine_scan_larger_blocks(P, oracle_mod, S, reverse):
    """3x3 and 4x4 block-diagonal Jacobians (cells with S state values per channel):
    every channel is an S x S recurrence, which the oracle solves as a dense one."""
    for (B, L, H) in [(1, 1, 4), (2, 33, 6), (2, 100, 37), (1, 257, 64), (2, 1025, 70)]:
        print(f"scan blocks {S}x{S} reverse={reverse} B={B} L={L} H={H}", flush=True)
        seed = 800 + L + S
        J = uniform_sym(seed, 1, (B, L, S, S, H), 0.45, device="cuda")
        r = normal(seed, 2, (B, L, S, H), device="cuda")
        d = P.affine_scan(J, r, reverse=reverse)
        torch.cuda.synchronize()
        Jn, rn, dn = to_np(J), to_np(r), to_np(d)
        worst = 0.0
        for b in range(B):
            for ch in range(H):
                Jc = np.ascontiguousarray(Jn[b, :, :, :, ch])          # [L][S][S]
                rc = np.ascontiguousarray(rn[b, :, :, ch])             # [L][S]
                if not reverse:
                    ref = oracle_mod.forward_substitution("dense", Jc, rc)
                else:
                    Jt = np.ascontiguousarray(Jc[::-1].transpose(0, 2, 1))
                    Js = np.zeros_like(Jt); Js[1:] = Jt[:-1]
                    ref = oracle_mod.forward_substitution("dense", Js, np.ascontiguousarray(rc[::-1]))[::-1]
                worst = max(worst, relerr(dn[b, :, :, ch], ref.reshape(L, S)))
        assert worst <= TOL_F32, (S, reverse, L, worst)


@pytest.mark.parametrize("cell", ["gru_diag", "lstm_diag", "paralstm_diag"])
@pytest.mark.parametrize("shape", [(3, 257, 68), (1, 65, 6), (2, 1000, 130), (1, 129, 64), (4, 64, 31)])
def test_fused_blocks_ragged_shapes(P, oracle_mod, cell, shape):
    """Resumed blocks on shapes with ragged tiles along L and H (and the small-H
    tile shape): a first block too short to converge, so that the solve ends in
    a resumed fused block or in the single-iteration launch."""
    B, L, H = shape
    params, u, h0, _ = problem(cell, B, L, H, seed=300 + L + H)
    pn, un, h0n = to_np(params), to_np(u), to_np(h0)
    ref = oracle_mod.seq_unroll(cell, pn, un, h0n)
    tol, it64 = well_posed_tol(oracle_mod, cell, pn, un, h0n, max_iter=40)
    try:
        for head in (1, 2, 3, 4, 8):
            print(f"ragged blocks {cell} {shape} head={head}", flush=True)
            P.set_fused_head(head)
            h, iters, tr = P.forward(cell, params, u, h0, tol=tol, max_iter=40, trace=True)
            torch.cuda.synchronize()
            it, st = (int(x) for x in iters.cpu())
            assert st == 0
            assert it == it64, (it, it64, tol)
            assert relerr(to_np(h), ref) <= TOL_F32
    finally:
        P.set_fused_head(5)


@pytest.mark.parametrize("cell", ["gru_diag", "lstm_diag", "paralstm_diag"])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_solve_to_tolerance_in_fused_blocks(P, oracle_mod, cell, dtype):
    """A solve to a tolerance is a sequence of launches: a fused block from the
    initial guess, then blocks of 1, 2, 4, ... iterations from the iterate.  For
    every size of the first block the tolerance is met in a different launch
    (inside the first block, in the single-iteration launch after it, inside a
    resumed fused block) or never; `iters`, status and trace must be those of the
    oracle's Newton, and h the converged state, whichever launch ended the solve."""
    B, L, H = 2, 700, 100
    params, u, h0, _ = problem(cell, B, L, H, seed=77, dtype=dtype)
    pn, un, h0n = to_np(params), to_np(u), to_np(h0)
    ref = oracle_mod.seq_unroll(cell, pn, un, h0n)
    bound = TOL_F32 if dtype == torch.float32 else TOL_BF16
    # the tolerance sits in the middle of the last jump of the oracle's trace, so that the
    # stopping decision has a clear margin in fp64 and in fp32
    tr0 = oracle_mod.newton(cell, pn, un, h0n, tol=1e-5, max_iter=40)[3]
    tol = max(float(np.sqrt(tr0[-2] * tr0[-1])), 2e-6)
    _, it64, _, tr64 = oracle_mod.newton(cell, pn, un, h0n, tol=tol, max_iter=40)
    _, it32, _, tr32 = oracle_mod.newton(cell, pn, un, h0n, tol=tol, max_iter=40, precision="f32")
    assert it64 == it32 == len(tr0) and it64 >= 4, (it64, it32)
    k = it64 - 1
    assert min(tr64[k - 1], tr32[k - 1]) >= 8 * tol and max(tr64[k], tr32[k]) <= tol / 8, (tr64, tr32)
    try:
        for head in (0, 1, 2, 3, 4, 5, 6, 8):
            for tile in (None, (1, 2, 8, 8), (2, 2, 8, 8), (4, 4, 8, 8)):
                for max_iter in (40, it64, it64 - 1, 2):
                    print(f"blocks {cell} {dtype} head={head} tile={tile} max_iter={max_iter}", flush=True)
                    P.set_fused_head(head)
                    if tile:
                        P.set_tile(*tile)
                    h, iters, tr = P.forward(cell, params, u, h0, tol=tol, max_iter=max_iter, trace=True)
                    torch.cuda.synchronize()
                    P.set_tile(0)
                    it, st = (int(x) for x in iters.cpu())
                    if max_iter >= it64:
                        assert (it, st) == (it64, 0), (it, st, it64)
                        assert relerr(to_np(h), ref) <= bound
                    else:
                        assert (it, st) == (max_iter, 1), (it, st)
                        hk = oracle_mod.newton(cell, pn, un, h0n, tol=tol, max_iter=max_iter)[0]
                        assert relerr(to_np(h), hk) <= (2e-5 if dtype == torch.float32 else TOL_BF16)
                    got = tr.cpu().numpy()[:it]
                    for j in range(it):
                        if tr64[j] > 1e-4:
                            assert abs(got[j] - tr64[j]) <= 5e-3 * tr64[j], (j, got, tr64)
        # the same solve with one launch per iteration agrees on everything but the extra refinement of h
        P.set_fused_head(5)
        hf, itf, _ = P.forward(cell, params, u, h0, tol=tol, max_iter=40)
        P.set_fused(False)
        hi, iti, _ = P.forward(cell, params, u, h0, tol=tol, max_iter=40)
        torch.cuda.synchronize()
        assert tuple(int(x) for x in itf.cpu()) == tuple(int(x) for x in iti.cpu())
        assert relerr(to_np(hf), to_np(hi)) <= (1e-5 if dtype == torch.float32 else 1e-2)
    finally:
        P.set_fused(True)
        P.set_fused_head(5)
        P.set_tile(0)


@pytest.mark.parametrize("kind", ["diag", "block2"])
@pytest.mark.parametrize("reverse", [False, True])
def test_affine_scan_matches_forward_substitution(P, oracle_mod, kind, reverse):
    """The scan on its own (random J, r) against Eq. (4) at tile-boundary
    lengths; reverse = the adjoint recurrence of Eq. (6)."""
    H = 70
    for L in (1, 2, 31, 32, 33, 63, 64, 65, 100, 257, 1025):
        print(f"scan {kind} reverse={reverse} L={L}", flush=True)
        B = 2
        seed = 500 + L
        if kind == "diag":
            J = uniform_sym(seed, 1, (B, L, H), 0.95, device="cuda")
            r = normal(seed, 2, (B, L, H), device="cuda")
        else:
            J = uniform_sym(seed, 1, (B, L, 2, 2, H), 0.6, device="cuda")
            r = normal(seed, 2, (B, L, 2, H), device="cuda")
        d = P.affine_scan(J, r, reverse=reverse)
        torch.cuda.synchronize()
        Jn, rn = to_np(J), to_np(r)
        for b in range(B):
            if not reverse:
                ref = oracle_mod.forward_substitution(kind, Jn[b], rn[b])
            else:
                # lam_l = J_{l+1}^T lam_{l+1} + r_l: flip time, shift J by one, transpose
                Jt = Jn[b][::-1].copy()
                if kind == "block2":
                    Jt = Jt.transpose(0, 2, 1, 3).copy()
                Js = np.zeros_like(Jt); Js[1:] = Jt[:-1]
                ref = oracle_mod.forward_substitution(kind, Js, rn[b][::-1].copy())[::-1]
            assert relerr(to_np(d[b]), ref) <= TOL_F32, (kind, reverse, L)


@pytest.mark.parametrize("cell", ["gru_diag", "lstm_diag", "paralstm_diag"])
def test_bf16_storage(P, oracle_mod, as_stored, cell):
    """bf16 storage, fp32 arithmetic: the oracle takes the bf16-rounded inputs
    as exact and computes in fp64; bound 2e-2."""
    B, L, H = 2, 300, 136
    params, u, h0, g = problem(cell, B, L, H, seed=77, dtype=torch.bfloat16)
    pn, un, h0n, gn = to_np(params), to_np(u), to_np(h0), to_np(g)
    tol, want = well_posed_tol(oracle_mod, cell, pn, un, h0n, max_iter=40)
    h, iters, _ = P.forward(cell, params, u, h0, tol=tol, max_iter=40)
    torch.cuda.synchronize()
    it, st = (int(x) for x in iters.cpu())
    ref = oracle_mod.seq_unroll(cell, pn, un, h0n)
    assert st == 0 and h.dtype == torch.bfloat16
    assert relerr(to_np(h), ref) <= TOL_BF16
    assert it == want, (it, want, tol)       # the iterate is fp32 under bf16 storage: the count is the fp32 solve's
    hs = as_stored(ref, h)                      # the oracle's states rounded to bf16, for both sides
    du, dp, dh0 = P.backward(cell, params, u, h0, hs, g)
    torch.cuda.synchronize()
    rdu, rdp, rdh0 = oracle_mod.backward(cell, pn, un, h0n, to_np(hs), gn)
    assert relerr(to_np(du), rdu) <= TOL_BF16
    assert relerr(to_np(dp), rdp) <= TOL_BF16
    assert relerr(to_np(dh0), rdh0) <= TOL_BF16


def _tie_problem(B, L, H):
    """linear_diag under bf16 storage with dyadic values whose exact fp32 results sit on, just above and just
    below the midpoint of two bf16 neighbours, with both signs: channel c takes pattern c % 6."""
    a_pat = [2.0 ** -8, 2.0 ** -8, 2.0 ** -8 + 2.0 ** -20, 2.0 ** -8 - 2.0 ** -20, 2.0 ** -8, 2.0 ** -8]
    x_pat = [1.0, 1.0 + 2.0 ** -7, 1.0, 1.0, 1.0, 1.0 + 2.0 ** -7]
    s_pat = [1.0, 1.0, 1.0, 1.0, -1.0, -1.0]
    ch = torch.arange(H) % 6
    a = torch.tensor(a_pat, dtype=torch.float32)[ch]
    x = torch.tensor(x_pat, dtype=torch.float32)[ch]
    s = torch.tensor(s_pat, dtype=torch.float32)[ch]
    params = torch.zeros(2, 1, H)
    params[0, 0] = a
    first = (s * x).to(torch.bfloat16)            # exactly representable: the cast changes nothing
    assert torch.equal(first.float(), s * x)
    one = s.to(torch.bfloat16)
    return params.cuda(), first, one


def test_bf16_stores_round_to_nearest_even_on_ties(P, oracle_mod):
    """Every kernel that writes a bf16 output, driven onto exact ties: the fp32 results 1 + 2^-8 and
    1 + 2^-7 + 2^-8 (and their negatives) are halfway between two bf16 values and must go to the even
    one, values 2^-20 off the midpoint to the nearer one.  Bits are compared with the oracle's fp64
    result (exact for these dyadic inputs) rounded to bf16 on the CPU, nearest-even."""
    cell = "linear_diag"
    for H in (8, 64, 67, 256):
        B = 2
        params, first, one = _tie_problem(B, 1, H)
        # forward, L = 1: h_1 = a h0 + u_1 with h0 = +-1, u_1 = +-x
        u = first.view(1, 1, 1, H).expand(B, 1, 1, H).contiguous().cuda()
        h0 = one.view(1, 1, H).expand(B, 1, H).contiguous().cuda()
        ref = oracle_mod.seq_unroll(cell, to_np(params), to_np(u), to_np(h0))
        want = torch.from_numpy(ref).to(torch.bfloat16)
        # the cases really are ties: the exact result is not a bf16 value in the first two patterns
        assert not np.array_equal(want.double().numpy(), ref)
        paths = {"fused block epilogue": dict(tol=1e-6, max_iter=8),
                 "fixed-count fused launch": dict(tol=-1.0, max_iter=3),
                 "initial guess + rounding pass": dict(tol=1e-6, max_iter=0)}
        for name, kw in paths.items():
            print(f"bf16 ties H={H}: {name}", flush=True)
            h, _, _ = P.forward(cell, params, u, h0, **kw)
            torch.cuda.synchronize()
            assert torch.equal(h.cpu().view(torch.int16), want.view(torch.int16)), (H, name)
        P.set_fused(False)
        try:
            print(f"bf16 ties H={H}: per-iteration kernel + rounding pass", flush=True)
            h, _, _ = P.forward(cell, params, u, h0, tol=1e-6, max_iter=8)
            torch.cuda.synchronize()
        finally:
            P.set_fused(True)
        assert torch.equal(h.cpu().view(torch.int16), want.view(torch.int16)), H
        # backward, L = 2 at states h = 0: lam_2 = g_2, lam_1 = g_1 + a g_2 = dL/du_1 (ties for g_2 = +-1,
        # g_1 = +-x), dL/dh0 = a lam_1 (the same ties scaled by a power of two in the tie patterns)
        u2 = torch.zeros(B, 2, 1, H, dtype=torch.bfloat16, device="cuda")
        hs = torch.zeros(B, 2, 1, H, dtype=torch.bfloat16, device="cuda")
        g = torch.stack([first, one]).view(1, 2, 1, H).expand(B, 2, 1, H).contiguous().cuda()
        print(f"bf16 ties H={H}: backward", flush=True)
        du, dp, dh0 = P.backward(cell, params, u2, None, hs, g)
        torch.cuda.synchronize()
        rdu, rdp, rdh0 = oracle_mod.backward(cell, to_np(params), to_np(u2), None, to_np(hs), to_np(g))
        want_du, want_dh0 = torch.from_numpy(rdu).to(torch.bfloat16), torch.from_numpy(rdh0).to(torch.bfloat16)
        assert not np.array_equal(want_du.double().numpy(), rdu)
        assert torch.equal(du.cpu().view(torch.int16), want_du.view(torch.int16)), H
        assert torch.equal(dh0.cpu().view(torch.int16), want_dh0.view(torch.int16)), H


@pytest.mark.parametrize("cell", ["gru_diag", "lstm_diag", "paralstm_diag"])
def test_backward_inputs_staged_through_lds(P, oracle_mod, as_stored, cell):
    """bf16 storage: the backward kernel copies the rows of a tile straight from memory into LDS one
    tile ahead (interior tiles; edge tiles and the first tile of a sequence load through registers).
    Same arithmetic either way: bit-identical outputs with the staging switched off, and both within
    the bf16 bound of the oracle.  Shapes with ragged tiles in L and H, and L below one tile."""
    for (B, L, H), tile in (((2, 1100, 200), None), ((3, 700, 64), None), ((2, 50, 72), None), ((1, 2100, 136), (1, 1, 8, 16)),
                            ((2, 900, 128), (1, 1, 16, 4))):
        print(f"staged backward {cell} B={B} L={L} H={H} tile={tile}", flush=True)
        params, u, h0, g = problem(cell, B, L, H, seed=900 + L, dtype=torch.bfloat16)
        pn, un, h0n, gn = to_np(params), to_np(u), to_np(h0), to_np(g)
        hs = as_stored(oracle_mod.seq_unroll(cell, pn, un, h0n), u)
        outs = []
        try:
            if tile:
                P.set_tile(*tile)
            for staging in (True, False):
                P.set_staging(staging)
                outs.append(P.backward(cell, params, u, h0, hs, g))
            torch.cuda.synchronize()
        finally:
            P.set_staging(True)
            P.set_tile(0)
        for a, b in zip(*outs):
            assert torch.equal(a, b)
        rdu, rdp, rdh0 = oracle_mod.backward(cell, pn, un, h0n, to_np(hs), gn)
        du, dp, dh0 = outs[0]
        assert relerr(to_np(du), rdu) <= TOL_BF16 and relerr(to_np(dp), rdp) <= TOL_BF16
        assert relerr(to_np(dh0), rdh0) <= TOL_BF16


@pytest.mark.parametrize("cell,dtype", [("gru_diag", torch.float32), ("lstm_diag", torch.float32), ("gru_diag", torch.bfloat16)])
def test_streamed_tile_accesses_give_the_same_bits(P, oracle_mod, as_stored, cell, dtype):
    """pararnn_set_streaming: the per-iteration forward kernel and the bf16 backward kernel with their
    interior tiles' accesses marked as streamed (mode 2; what large problems get by themselves) against
    plain accesses (mode 1).  Only the cache policy differs: same bits, iteration count and trace; the
    plain result is checked against the oracle."""
    B, L, H = 2, 1100, 200
    params, u, h0, g = problem(cell, B, L, H, seed=4242, dtype=dtype)
    pn, un, h0n = to_np(params), to_np(u), to_np(h0)
    fwd, bwd = [], []
    try:
        P.set_fused(False)                      # one launch per iteration: the kernel that takes the flag
        for mode in (1, 2, 0):
            print(f"streaming mode {mode} {cell} {dtype}", flush=True)
            P.set_streaming(mode)
            h, iters, trace = P.forward(cell, params, u, h0, tol=-1.0, max_iter=6, trace=True)
            fwd.append((h, trace, iters))
            bwd.append(P.backward(cell, params, u, h0, h, g))
        torch.cuda.synchronize()
    finally:
        P.set_streaming(0)
        P.set_fused(True)
    for other in (1, 2):
        for a, b in zip(fwd[0], fwd[other]):
            assert torch.equal(a, b)
        for a, b in zip(bwd[0], bwd[other]):
            assert torch.equal(a, b)
    ref = oracle_mod.seq_unroll(cell, pn, un, h0n)
    tol_h = TOL_BF16 if dtype == torch.bfloat16 else TOL_F32
    assert relerr(to_np(fwd[0][0]), ref) <= tol_h
    with pytest.raises(RuntimeError):
        P.set_streaming(3)


@pytest.mark.parametrize("cell,dtype", [("gru_diag", torch.float32), ("lstm_diag", torch.float32), ("gru_diag", torch.bfloat16)])
def test_blocks_after_the_first_in_one_launch(P, oracle_mod, cell, dtype):
    """The rest of a solve's plan in one persistent launch (pararnn_set_fused_tail, the default) against one
    launch per block: a first block of 1, 2 or 3 iterations and the one iteration that follows it leave
    more to blocks of 2 and 4 that the tail launch separates by grid-wide barriers.  Iteration count, status and trace are the
    oracle's either way; the traces of the two agree to rounding (a block of one iteration is the fused
    kernel in the one and the per-iteration kernel in the other), h is the converged state."""
    B, L, H = 3, 1500, 200
    params, u, h0, _ = problem(cell, B, L, H, seed=616, dtype=dtype)
    pn, un, h0n = to_np(params), to_np(u), to_np(h0)
    ref = oracle_mod.seq_unroll(cell, pn, un, h0n)
    tol, want = well_posed_tol(oracle_mod, cell, pn, un, h0n, max_iter=40)
    assert want >= 5
    for first_block in (1, 2, 3):
        out = {}
        for tail in (True, False):
            print(f"tail launch {cell} {dtype} first_block={first_block} tail={tail}", flush=True)
            try:
                P.set_fused_tail(tail)
                h, iters, tr = P.forward_ex(cell, params, u, h0, tol=tol, max_iter=40, first_block=first_block, trace=True)
                torch.cuda.synchronize()
            finally:
                P.set_fused_tail(True)
            assert tuple(int(x) for x in iters.cpu()) == (want, 0)
            assert relerr(to_np(h), ref) <= (TOL_F32 if dtype == torch.float32 else TOL_BF16)
            out[tail] = tr[:want].cpu().numpy().astype(np.float64)
        big = out[False] > 1e-4                       # above the rounding floor of the updates
        assert np.all(np.abs(out[True] - out[False])[big] <= 1e-3 * out[False][big])


@pytest.mark.gpu
def test_tail_launch_with_a_full_grid(P, oracle_mod):
    """The same on config 2's shape, where the persistent grid is as large as the device holds and every
    workgroup walks many tiles per block: a first block of 1 and the iteration after it leave three or more
    iterations to the tail launch (blocks of 2 and 4).  Checked against the oracle's sequential unroll on sampled channels."""
    from workloads import CONFIGS, make_inputs
    w = CONFIGS["C2"]
    d = make_inputs(w, device="cuda")
    params, u, h0 = d["params"], d["u"], d["h0"]
    res = {}
    for tail in (True, False):
        print(f"tail launch, full grid, tail={tail}", flush=True)
        try:
            P.set_fused_tail(tail)
            h, iters, tr = P.forward_ex(w.cell, params, u, h0, tol=w.tol, max_iter=w.max_iter, first_block=1, trace=True)
            torch.cuda.synchronize()
        finally:
            P.set_fused_tail(True)
        res[tail] = (h, tuple(int(x) for x in iters.cpu()), tr)
    assert res[True][1] == res[False][1] and res[True][1][1] == 0 and res[True][1][0] >= 4
    assert float((res[True][0] - res[False][0]).abs().max()) <= 1e-5
    idx = torch.tensor([0, 1, 63, 64, 500, 1023], device="cuda")
    ref = oracle_mod.seq_unroll(w.cell, to_np(params.index_select(-1, idx)), to_np(u.index_select(-1, idx)),
                                None if h0 is None else to_np(h0.index_select(-1, idx)))
    assert relerr(to_np(res[True][0].index_select(-1, idx)), ref) <= TOL_F32


@pytest.mark.parametrize("cell", ["gru_diag", "lstm_diag"])
def test_forward_ex_options_travel_with_the_call(P, oracle_mod, cell):
    """pararnn_forward_ex: the first launch runs `first_block` iterations (3 = the paper's fixed
    count); whichever launch the tolerance is met in, iteration count, status and trace are the
    oracle's, h is the converged state, and the process-wide settings stay as they were."""
    B, L, H = 2, 900, 136
    params, u, h0, _ = problem(cell, B, L, H, seed=515)
    pn, un, h0n = to_np(params), to_np(u), to_np(h0)
    ref = oracle_mod.seq_unroll(cell, pn, un, h0n)
    tol, want = well_posed_tol(oracle_mod, cell, pn, un, h0n, max_iter=40)
    plan_before = P.solve_plan(tol, 40)
    for first_block, fused in ((3, -1), (1, -1), (0, -1), (8, -1), (-1, 0), (-1, -1)):
        print(f"forward_ex {cell} first_block={first_block} fused={fused}", flush=True)
        h, iters, tr = P.forward_ex(cell, params, u, h0, tol=tol, max_iter=40, first_block=first_block, fused=fused,
                                    trace=True)
        torch.cuda.synchronize()
        assert tuple(int(x) for x in iters.cpu()) == (want, 0)
        assert relerr(to_np(h), ref) <= TOL_F32
        plan = P.solve_plan_ex(tol, 40, first_block=first_block, fused=fused)
        assert sum(plan) == 40 and plan[0] == (1 if fused == 0 or first_block == 0 else (5 if first_block < 0 else first_block))
    assert P.solve_plan(tol, 40) == plan_before
    with pytest.raises(RuntimeError, match="INVALID_ARG"):
        P.forward_ex(cell, params, u, h0, tol=tol, max_iter=40, first_block=9)
