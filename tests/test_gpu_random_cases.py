"""Seeded random sweep over cells, storage types, shapes (ragged in L and H, L
down to 1), tile shapes, sizes of the first fused block and iteration limits:
forward and backward against the oracle, case by case."""
import random

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from test_gpu_parity import problem, relerr, to_np      # noqa: E402
from parity_util import well_posed_tol                   # noqa: E402

TILES = [None, None, None, (1, 1, 8, 16), (1, 2, 8, 16), (1, 2, 16, 4), (1, 2, 8, 8), (1, 1, 8, 8), (2, 2, 8, 8),
         (1, 1, 4, 8), (1, 1, 16, 8), (1, 8, 4, 2), (4, 4, 8, 8), (2, 4, 8, 8), (1, 1, 16, 4), (1, 1, 12, 8)]


@pytest.mark.parametrize("seed", [11, 12])
def test_random_cases(oracle_mod, as_stored, seed):
    import paper_2510_21450_amd as P
    rnd = random.Random(seed)
    for case in range(120):
        cell = rnd.choice(["gru_diag", "lstm_diag", "paralstm_diag"])
        dtype = rnd.choice([torch.float32, torch.float32, torch.bfloat16])
        B = rnd.randint(1, 4)
        L = rnd.choice([1, 2, 3, rnd.randint(4, 200), rnd.randint(200, 1500), rnd.randint(1500, 4000)])
        H = rnd.choice([1, 2, 7, 8, 9, 31, 32, 33, 64, 65, rnd.randint(66, 300)])
        head, tile = rnd.randint(0, 8), rnd.choice(TILES)
        max_iter, use_h0 = rnd.choice([40, 40, 40, 3, 6]), rnd.random() < 0.7
        what = f"case {seed}/{case}: {cell} {dtype} B={B} L={L} H={H} head={head} tile={tile} max_iter={max_iter} h0={use_h0}"
        print(what, flush=True)
        params, u, h0, g = problem(cell, B, L, H, seed=5000 + 1000 * seed + case, dtype=dtype, h0=use_h0)
        pn, un, h0n, gn = to_np(params), to_np(u), to_np(h0), to_np(g)
        bound = 1e-5 if dtype == torch.float32 else 2e-2
        # the tolerance sits inside a jump of the oracle's fp64 and fp32 traces, so the iteration count and
        # the status are well defined for every case: the solve needs `need` iterations and is given max_iter
        tol, need = well_posed_tol(oracle_mod, cell, pn, un, h0n, max_iter=40)
        want_it, want_st = (need, 0) if need <= max_iter else (max_iter, 1)
        # the states the backward pass is evaluated at, for both sides: the oracle's (the
        # recurrence's where the solve converges, else the iterate after max_iter steps)
        if want_st == 0:
            ref = oracle_mod.seq_unroll(cell, pn, un, h0n)
        else:
            ref, itk, stk, _ = oracle_mod.newton(cell, pn, un, h0n, tol=tol, max_iter=max_iter)
            assert (itk, stk) == (want_it, want_st), what
        hs = as_stored(ref, u)
        try:
            P.set_fused_head(head)
            if tile:
                P.set_tile(*tile)
            # every tile shape in TILES is built for these cells, forward and backward: nothing may be refused
            h, iters, tr = P.forward(cell, params, u, h0, tol=tol, max_iter=max_iter, trace=True)
            du, dp, dh0 = P.backward(cell, params, u, h0, hs, g)
            torch.cuda.synchronize()
        finally:
            P.set_tile(0)
            P.set_fused_head(5)
        it, st = (int(x) for x in iters.cpu())
        assert (it, st) == (want_it, want_st), (what, it, st, want_it, want_st, tol, tr.cpu().numpy()[:it])
        # a converged solve against the recurrence itself; an iterate that has not converged against the
        # oracle's iterate after the same number of steps (2e-5: rounding differences of iterate k - 1 pass
        # through one more Newton step, as in the fixed-count tests)
        assert relerr(to_np(h), ref) <= (bound if want_st == 0 else max(bound, 2e-5)), what
        rdu, rdp, rdh0 = oracle_mod.backward(cell, pn, un, h0n, to_np(hs), gn)
        assert relerr(to_np(du), rdu) <= bound and relerr(to_np(dp), rdp) <= bound, what
        assert relerr(to_np(dh0), rdh0) <= bound, what
