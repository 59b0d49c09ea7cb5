"""Python access to the CPU oracle (oracle/pararnn_oracle.c) through ctypes.

Test infrastructure only: imported by tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py, never by the product package.  Arrays are numpy,
C-contiguous, in the oracle's precision (float64 by default; `precision="f32"`
selects the second build of the same C file, used to inspect fp32 iteration
traces).  Argument marshalling only: all arithmetic is in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "pararnn_oracle.c")
_LIBS = {}

CELLS = {"gru_diag": 0, "lstm_diag": 1, "tanh_dense": 2, "linear_diag": 3, "paralstm_diag": 4, "rot_tanh": 5, "tri_tanh": 6, "quad_tanh": 7}
NONLIN = {"sigmoid": 0, "tanh": 1, "identity": 2, "softsign": 3}


def cell_id(cell: str) -> int:
    """Number of a cell; "gru_nl:<update>,<reset>,<state>" names the GRU with those nonlinearities."""
    if cell.startswith("gru_nl:"):
        nu, nr, ns = (NONLIN[s] for s in cell[len("gru_nl:"):].split(","))
        return 100 + 16 * nu + 4 * nr + ns
    return CELLS[cell]


STATUS = {0: "OK", 1: "NOT_CONVERGED", 2: "INVALID_ARG", 5: "NONFINITE"}
JAC_KIND = {"diag": 0, "block2": 1, "dense": 2, "block3": 3, "block4": 4}


def _lib_path(precision):
    return os.path.join(_DIR, f"liboracle_{precision}.so")


def build(force: bool = False) -> None:
    """Compile the oracle with gcc: -O2, no fast-math, OpenMP over the batch."""
    for precision, real in (("f64", "double"), ("f32", "float")):
        out = _lib_path(precision)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-Wextra",
               f"-DREAL={real}", "-o", out, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    _LIBS.clear()


def _lib(precision="f64"):
    if precision not in _LIBS:
        build()
        lib = ctypes.CDLL(_lib_path(precision))
        assert lib.oracle_real_bytes() == (8 if precision == "f64" else 4)
        _LIBS[precision] = lib
    return _LIBS[precision]


def _np_t(precision):
    return np.float64 if precision == "f64" else np.float32


def _c(a, precision):
    if a is None:
        return None, None
    a = np.ascontiguousarray(a, dtype=_np_t(precision))
    return a, a.ctypes.data_as(ctypes.c_void_p)


def dims(cell: str):
    lib = _lib()
    return lib.oracle_gates(cell_id(cell)), lib.oracle_state(cell_id(cell))


def num_threads() -> int:
    return _lib().oracle_num_threads()


def cell_step(cell, params, hp, u, precision="f64"):
    """f(hp, u) for one timestep: hp [S][H], u [G][H] -> [S][H]."""
    lib = _lib(precision)
    hp_a, hp_p = _c(hp, precision)
    H = hp_a.shape[-1]
    _, pp = _c(params, precision)
    _, up = _c(u, precision)
    out = np.empty_like(hp_a)
    lib.oracle_cell_step(cell_id(cell), H, pp, hp_p, up, out.ctypes.data_as(ctypes.c_void_p))
    return out


def cell_jacobian(cell, params, hp, u, precision="f64"):
    """J = df/dh at (hp, u): diag [H]; lstm [2][2][H]; dense [H][H]."""
    lib = _lib(precision)
    hp_a, hp_p = _c(hp, precision)
    H = hp_a.shape[-1]
    _, pp = _c(params, precision)
    _, up = _c(u, precision)
    shape = {0: (H,), 1: (2, 2, H), 2: (H, H), 3: (3, 3, H), 4: (4, 4, H)}[lib.oracle_jac_kind(cell_id(cell))]
    out = np.empty(shape, dtype=_np_t(precision))
    lib.oracle_cell_jacobian(cell_id(cell), H, pp, hp_p, up, out.ctypes.data_as(ctypes.c_void_p))
    return out


def seq_unroll(cell, params, u, h0=None, precision="f64"):
    """Eq. (1). u [B][L][G][H] -> h [B][L][S][H]."""
    lib = _lib(precision)
    u_a, up = _c(u, precision)
    B, L, G, H = u_a.shape
    S = lib.oracle_state(cell_id(cell))
    assert G == lib.oracle_gates(cell_id(cell))
    _, pp = _c(params, precision)
    _h0, h0p = _c(h0, precision)
    h = np.empty((B, L, S, H), dtype=_np_t(precision))
    lib.oracle_seq_unroll(cell_id(cell), B, L, H, pp, up, h0p, h.ctypes.data_as(ctypes.c_void_p))
    return h


def residual_norm(cell, params, u, h0, h, precision="f64"):
    """App. A: max |h_l - f(h_{l-1}, u_l)| over the batch, all steps, state values and channels."""
    lib = _lib(precision)
    u_a, up = _c(u, precision)
    B, L, G, H = u_a.shape
    h_a, hp = _c(h, precision)
    assert h_a.shape == (B, L, lib.oracle_state(cell_id(cell)), H)
    _, pp = _c(params, precision)
    _h0, h0p = _c(h0, precision)
    fn = lib.oracle_residual_norm
    fn.restype = ctypes.c_double if precision == "f64" else ctypes.c_float
    return float(fn(cell_id(cell), B, L, H, pp, up, h0p, hp))


def _solver(name, kind, J, r, precision):
    lib = _lib(precision)
    r_a, rp = _c(r, precision)
    L = r_a.shape[0]
    H = r_a.shape[-1]
    _J, Jp = _c(J, precision)
    d = np.empty_like(r_a)
    getattr(lib, name)(JAC_KIND[kind], L, H, Jp, rp, d.ctypes.data_as(ctypes.c_void_p))
    return d


def forward_substitution(kind, J, r, precision="f64"):
    """Eq. (4) on one sequence. J [L][...], r [L][S][H] (or [L][H]) -> delta."""
    return _solver("oracle_forward_substitution", kind, J, r, precision)


def parallel_reduce(kind, J, r, precision="f64"):
    """Alg. 1b on one sequence; same arguments as forward_substitution."""
    return _solver("oracle_parallel_reduce", kind, J, r, precision)


def newton(cell, params, u, h0=None, tol=1e-6, max_iter=64, precision="f64", jacobian="full"):
    """Alg. 1a with Eq. (4). Returns (h, iters, status, trace[iters]).
    jacobian="diagonal": the quasi-Newton variant (every J_l replaced by its diagonal)."""
    assert jacobian in ("full", "diagonal")
    lib = _lib(precision)
    u_a, up = _c(u, precision)
    B, L, G, H = u_a.shape
    S = lib.oracle_state(cell_id(cell))
    _, pp = _c(params, precision)
    _h0, h0p = _c(h0, precision)
    h = np.empty((B, L, S, H), dtype=_np_t(precision))
    iters = ctypes.c_int(0)
    trace = np.zeros(max(max_iter, 1), dtype=_np_t(precision))
    real = ctypes.c_double if precision == "f64" else ctypes.c_float
    fn = lib.oracle_newton if jacobian == "full" else lib.oracle_newton_diag
    fn.argtypes = [ctypes.c_int] * 4 + [ctypes.c_void_p] * 3 + [real, ctypes.c_int,
                   ctypes.c_void_p, ctypes.POINTER(ctypes.c_int), ctypes.c_void_p]
    st = fn(cell_id(cell), B, L, H, pp, up, h0p, tol, max_iter,
            h.ctypes.data_as(ctypes.c_void_p), ctypes.byref(iters),
            trace.ctypes.data_as(ctypes.c_void_p))
    return h, iters.value, st, trace[:iters.value].copy()


def backward(cell, params, u, h0, h, g, precision="f64"):
    """Eq. (6) + step-local chain rule. Returns (du, dparams, dh0)."""
    lib = _lib(precision)
    u_a, up = _c(u, precision)
    B, L, G, H = u_a.shape
    S = lib.oracle_state(cell_id(cell))
    p_a, pp = _c(params, precision)
    _h0, h0p = _c(h0, precision)
    _h, hp = _c(h, precision)
    _g, gp = _c(g, precision)
    du = np.empty_like(u_a)
    dparams = np.empty_like(p_a)
    dh0 = np.empty((B, S, H), dtype=_np_t(precision))
    lib.oracle_backward(cell_id(cell), B, L, H, pp, up, h0p, hp, gp,
                        du.ctypes.data_as(ctypes.c_void_p), dparams.ctypes.data_as(ctypes.c_void_p),
                        dh0.ctypes.data_as(ctypes.c_void_p))
    return du, dparams, dh0


def input_projection(x, Wx, bias=None, n_heads=1, precision="f64"):
    """u = B x + b for all gates (Eq. (7a) / (7b) input terms, multi-head per App. C).
    x [..., H], Wx [G][H][H / n_heads], bias [G][H] or None -> u [..., G, H]."""
    lib = _lib(precision)
    x_a, xp = _c(x, precision)
    w_a, wp = _c(Wx, precision)
    G, H, dh = w_a.shape
    assert x_a.shape[-1] == H and dh * n_heads == H
    _b, bp = _c(bias, precision)
    rows = x_a.size // H
    u = np.empty(x_a.shape[:-1] + (G, H), dtype=_np_t(precision))
    lib.oracle_input_projection(rows, H, G, n_heads, xp, wp, bp, u.ctypes.data_as(ctypes.c_void_p))
    return u


def input_projection_backward(x, Wx, du, n_heads=1, precision="f64"):
    """Returns (dx, dWx, dbias) for du = dL/du of input_projection."""
    lib = _lib(precision)
    x_a, xp = _c(x, precision)
    w_a, wp = _c(Wx, precision)
    du_a, dup = _c(du, precision)
    G, H, dh = w_a.shape
    rows = x_a.size // H
    assert du_a.shape == x_a.shape[:-1] + (G, H)
    dx = np.empty_like(x_a)
    dW = np.empty_like(w_a)
    db = np.empty((G, H), dtype=_np_t(precision))
    lib.oracle_input_projection_backward(rows, H, G, n_heads, xp, wp, dup, dx.ctypes.data_as(ctypes.c_void_p),
                                         dW.ctypes.data_as(ctypes.c_void_p), db.ctypes.data_as(ctypes.c_void_p))
    return dx, dW, db
