"""Helpers shared by the GPU parity tests (no arithmetic of the method here).

Error metrics: `relerr` is the norm-wise bound the parity bar is stated in
(max |x - ref| / max |ref| per tensor); `elt_err` is the element-wise relative
error with an absolute floor of 1e-3 * max |ref| (states cross zero, so a plain
element-wise relative error has no bound).

`well_posed_tol` picks a stopping tolerance for which the iteration count of a
solve is well defined, so that every test can compare it exactly: Newton's
updates fall quadratically (1e-1, 1e-2, 1e-4, 1e-8 ...) until they reach the
fp32 rounding floor, and `iters` is unambiguous only when `tol` sits inside one
of those jumps with room on both sides in fp64 and in fp32 arithmetic alike.
The tolerance is taken from the oracle's own traces, never from the GPU's."""
import numpy as np
import torch

MARGIN = 8.0          # the update that stops the solve is <= tol / MARGIN, the one before it >= MARGIN * tol
TOL_FLOOR = 2e-6      # tolerances stay above the fp32 rounding floor of the updates (1e-7 .. 1e-6 here)


def relerr(got, ref):
    """max |got - ref| / max |ref| (norm-wise, infinity norm)."""
    got = np.asarray(got, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    return float(np.max(np.abs(got - ref)) / max(np.max(np.abs(ref)), 1e-30))


def elt_err(got, ref):
    """max_i |got_i - ref_i| / max(|ref_i|, 1e-3 * max |ref|)."""
    got = np.asarray(got, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    floor = 1e-3 * max(float(np.max(np.abs(ref))), 1e-30)
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), floor)))


def to_np(t):
    return None if t is None else t.detach().to("cpu", torch.float64).numpy()


def well_posed_tol(oracle_mod, cell, params, u, h0, max_iter=40, margin=MARGIN, probe_tol=1e-5, floor=TOL_FLOOR,
                   **newton_kw):
    """(tol, iters): a tolerance inside a jump of the oracle's update trace such that, in the
    oracle's fp64 AND fp32 arithmetic, update `iters` is <= tol / margin and update `iters - 1`
    is >= margin * tol.  The jump closest to `probe_tol` is taken (the last one of a solve to
    probe_tol); raises if the traces have no such jump (the case is ill-posed: change it)."""
    t64 = oracle_mod.newton(cell, params, u, h0, tol=probe_tol, max_iter=max_iter, precision="f64", **newton_kw)[3]
    t32 = oracle_mod.newton(cell, params, u, h0, tol=probe_tol, max_iter=max_iter, precision="f32", **newton_kw)[3]
    n = min(len(t64), len(t32))
    for k in range(n - 1, -1, -1):
        hi = max(float(t64[k]), float(t32[k]))                  # the update that has to pass the test
        lo = min(float(t64[k - 1]), float(t32[k - 1])) if k > 0 else float("inf")
        if k > 0:
            tol = max(float(np.sqrt(max(hi, 1e-300) * lo)), floor)
        else:
            tol = max(margin * hi, probe_tol)
        earlier = min([float(min(a, b)) for a, b in zip(t64[:k], t32[:k])], default=float("inf"))
        if hi * margin <= tol and tol * margin <= lo and tol * margin <= earlier:
            return tol, k + 1
    raise AssertionError(f"no tolerance with a {margin}x margin in both precisions: fp64 {t64}, fp32 {t32}")
