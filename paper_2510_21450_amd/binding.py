"""ctypes binding: one Python function per entry point of include/pararnn.h,
same names without the prefix.  Argument marshalling only."""
from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libpararnn.so")

CELLS = {"gru_diag": 0, "lstm_diag": 1, "tanh_dense": 2, "linear_diag": 3, "paralstm_diag": 4}
DTYPES = {torch.float32: 0, torch.bfloat16: 1}
STATUS = {0: "OK", 1: "NOT_CONVERGED", 2: "INVALID_ARG", 3: "WORKSPACE_TOO_SMALL", 4: "HIP_ERROR",
          5: "NONFINITE", 6: "UNSUPPORTED", 7: "INTERNAL"}

if not os.path.exists(_LIB_PATH):
    raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2510_21450_amd.build` "
                      "(there is no CPU fallback)")

_lib = ctypes.CDLL(_LIB_PATH)
for _name in ("pararnn_input_projection", "pararnn_residual_norm", "pararnn_set_dense_jacobian", "pararnn_device_info", "pararnn_set_dense_products", "pararnn_solve_plan", "pararnn_affine_scan_workspace_bytes"):
    if not hasattr(_lib, _name):
        raise ImportError(f"{_LIB_PATH} is older than this binding ({_name} is missing): rebuild it with "
                          "`python -m paper_2510_21450_amd.build`")
_vp, _i, _f, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
_lib.pararnn_status_string.restype = ctypes.c_char_p
_lib.pararnn_status_string.argtypes = [_i]
_lib.pararnn_version.restype = _i
_lib.pararnn_device_info.restype = _i
_lib.pararnn_device_info.argtypes = [ctypes.POINTER(ctypes.c_int), _i]
_lib.pararnn_set_tile.argtypes = [_i] * 4
_lib.pararnn_set_tile.restype = _i
_lib.pararnn_cell_gates.argtypes = [_i]
_lib.pararnn_cell_state.argtypes = [_i]
_lib.pararnn_workspace_bytes.restype = _sz
_lib.pararnn_workspace_bytes.argtypes = [_i] * 6
_lib.pararnn_workspace_bytes_fused.restype = _sz
_lib.pararnn_workspace_bytes_fused.argtypes = [_i] * 6
_lib.pararnn_set_fused.argtypes = [_i]
_lib.pararnn_set_fused_tail.argtypes = [_i]
_lib.pararnn_set_workspace_reuse.argtypes = [_i]
_lib.pararnn_set_staging.argtypes = [_i]
_lib.pararnn_set_streaming.argtypes = [_i]
_lib.pararnn_set_dense_products.argtypes = [_i]
_lib.pararnn_set_fused_head.argtypes = [_i]
_lib.pararnn_solve_plan.restype = _i
_lib.pararnn_solve_plan.argtypes = [ctypes.c_float, _i, ctypes.POINTER(ctypes.c_int), _i]
_lib.pararnn_forward.restype = _i
_lib.pararnn_forward.argtypes = [_i, _i, _vp, _vp, _vp, _i, _i, _i, _f, _i, _vp, _vp, _vp, _vp, _sz, _vp]
class _SolveOptions(ctypes.Structure):
    _fields_ = [("first_block", ctypes.c_int), ("fused", ctypes.c_int)]


_lib.pararnn_forward_ex.restype = _i
_lib.pararnn_forward_ex.argtypes = [_i, _i, _vp, _vp, _vp, _i, _i, _i, _f, _i, _vp, _vp, _vp, _vp, _sz, _vp,
                                    ctypes.POINTER(_SolveOptions)]
_lib.pararnn_workspace_bytes_ex.restype = _sz
_lib.pararnn_workspace_bytes_ex.argtypes = [_i, _i, _i, _i, _i, ctypes.POINTER(_SolveOptions)]
_lib.pararnn_solve_plan_ex.restype = _i
_lib.pararnn_solve_plan_ex.argtypes = [ctypes.c_float, _i, ctypes.POINTER(_SolveOptions), ctypes.POINTER(ctypes.c_int), _i]
_lib.pararnn_forward_noalloc.restype = _i
_lib.pararnn_forward_noalloc.argtypes = [_i, _i, _vp, _vp, _vp, _i, _i, _i, _f, _i, _vp, _vp, _vp, _vp]
_lib.pararnn_backward.restype = _i
_lib.pararnn_backward.argtypes = [_i, _i, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.pararnn_dense_chunk_products.restype = _i
_lib.pararnn_dense_chunk_products.argtypes = [_vp, _vp, _i, _i, _i, _vp, _vp, _sz, _vp]
_lib.pararnn_affine_scan.restype = _i
_lib.pararnn_affine_scan_workspace_bytes.restype = _sz
_lib.pararnn_affine_scan_workspace_bytes.argtypes = [_i] * 5
_lib.pararnn_affine_scan.argtypes = [_i, _i, _vp, _vp, _i, _i, _i, _vp, _vp, _sz, _vp]


_FWD_ARGS = [_i, _vp, _vp, _vp, _i, _i, _i, _f, _i, _vp, _vp, _vp, _vp, _sz, _vp]
_BWD_ARGS = [_i, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _vp, _vp, _vp, _vp, _sz, _vp]
_RES_ARGS = [_i, _vp, _vp, _vp, _vp, _i, _i, _i, _vp, _vp]
_lib.pararnn_residual_norm.restype = _i
_lib.pararnn_residual_norm.argtypes = [_i] + _RES_ARGS


class _BuiltinCell:
    """Entry points of one built-in cell: the pararnn_* functions with the cell number bound."""

    def __init__(self, name):
        self.name = name
        c = CELLS[name]
        self.G, self.S = _lib.pararnn_cell_gates(c), _lib.pararnn_cell_state(c)
        self.what = "pararnn"
        self.ws = lambda *a: _lib.pararnn_workspace_bytes(c, *a)
        self.ws_fused = lambda *a: _lib.pararnn_workspace_bytes_fused(c, *a)
        self.fwd = lambda *a: _lib.pararnn_forward(c, *a)
        self.bwd = lambda *a: _lib.pararnn_backward(c, *a)
        self.res = lambda *a: _lib.pararnn_residual_norm(c, *a)


class UserCell:
    """A cell from a library built with PARARNN_DEFINE_CELL(Cell, name) (include/pararnn_cell.h):
    pass the object wherever the functions of this module take a cell name."""

    def __init__(self, lib_path: str, name: str):
        if not os.path.exists(lib_path):
            raise ImportError(f"{lib_path} is missing: build it with `python -m paper_2510_21450_amd.build --cell ...`")
        self.name, self.what = name, name
        self._lib = lib = ctypes.CDLL(lib_path)
        f = lambda s: getattr(lib, f"{name}_{s}")
        self.G, self.S, self.param_rows = f("gates")(), f("state")(), f("param_rows")()
        self.ws, self.ws_fused, self.fwd, self.bwd = f("workspace_bytes"), f("workspace_bytes_fused"), f("forward"), f("backward")
        self.ws.restype = self.ws_fused.restype = _sz
        self.ws.argtypes = self.ws_fused.argtypes = [_i] * 5
        self.fwd.restype = self.bwd.restype = _i
        self.fwd.argtypes, self.bwd.argtypes = _FWD_ARGS, _BWD_ARGS
        self.res = f("residual_norm")
        self.res.restype, self.res.argtypes = _i, _RES_ARGS


_builtin = {}


def _api(cell):
    if isinstance(cell, UserCell):
        return cell
    if cell not in _builtin:
        _builtin[cell] = _BuiltinCell(cell)
    return _builtin[cell]


def example_cell(name: str) -> UserCell:
    """One of the example cells shipped under user_cells/ ("gru_softsign", "gru_sigmoid_identity_tanh",
    "gru_sigmoid_softsign_identity", "gru_sigmoid_tanh_softsign", "rot_tanh", "tri_tanh", "quad_tanh")."""
    return UserCell(os.path.join(_PKG, f"libpararnn_{name}.so"), name)


def set_tile(vec: int = 0, ll: int = 0, c: int = 0, w: int = 0) -> None:
    """pararnn_set_tile: force a compiled tile shape (vec = 0: automatic)."""
    _raise(_lib.pararnn_set_tile(vec, ll, c, w), "pararnn_set_tile")


def set_dense_products(mode: int = 0) -> None:
    """pararnn_set_dense_products: 0 fp32 Jacobian products (default), 1 three bf16 terms, 2 one bf16 term."""
    _raise(_lib.pararnn_set_dense_products(int(mode)), "pararnn_set_dense_products")


def device_info() -> dict:
    """pararnn_device_info as a dict (None where the runtime gives no answer)."""
    buf = (ctypes.c_int * 8)()
    n = _lib.pararnn_device_info(buf, 8)
    if n < 6:
        raise RuntimeError("pararnn_device_info failed")
    keys = ("compute_units", "clock_khz", "memory_clock_khz", "memory_bus_bits", "l2_bytes", "lds_bytes_per_workgroup")
    return {k: (int(buf[i]) if buf[i] >= 0 else None) for i, k in enumerate(keys)}


def set_dense_jacobian(mode: int = 0) -> None:
    """pararnn_set_dense_jacobian: 0 the full Jacobian (Newton, default), 1 its diagonal (quasi-Newton)."""
    _raise(_lib.pararnn_set_dense_jacobian(int(mode)), "pararnn_set_dense_jacobian")


def set_dense_tail(mode: int = 1) -> None:
    """pararnn_set_dense_tail: 1 launches per phase for six iterations, then one persistent launch (default);
    0 launches per phase throughout; 2 the persistent launch from the start."""
    _raise(_lib.pararnn_set_dense_tail(int(mode)), "pararnn_set_dense_tail")


def dense_chunk() -> int:
    return _lib.pararnn_dense_chunk()


def dense_chunk_products(W, d, out=None, stream=None):
    """pararnn_dense_chunk_products.  W [H][H], d [B][L][H] -> A [B][n_c][H][H]
    (chunks 1 .. n_c-2 written, the rest zero)."""
    B, L, H = d.shape
    _check(W, "W", torch.float32, (H, H))
    _check(d, "d", torch.float32)
    n_c = (L + dense_chunk() - 1) // dense_chunk()
    A = torch.zeros((B, n_c, H, H), dtype=torch.float32, device=d.device) if out is None else out
    ws = torch.empty(256, dtype=torch.uint8, device=d.device)
    code = _lib.pararnn_dense_chunk_products(_ptr(W), _ptr(d), B, L, H, _ptr(A), _ptr(ws), ws.numel(), _stream(stream))
    _raise(code, "pararnn_dense_chunk_products")
    return A


def lib_path() -> str:
    return _LIB_PATH


def version() -> int:
    return _lib.pararnn_version()


def status_string(code: int) -> str:
    return _lib.pararnn_status_string(code).decode()


def cell_dims(cell):
    """(gates G, state values S) of a cell (a built-in cell's name or a UserCell)."""
    a = _api(cell)
    return a.G, a.S


def workspace_bytes(cell, dtype, B: int, L: int, H: int, backward: bool = False) -> int:
    return _api(cell).ws(DTYPES[dtype], B, L, H, int(backward))


def workspace_bytes_fused(cell, dtype, B: int, L: int, H: int, n_iters: int) -> int:
    return _api(cell).ws_fused(DTYPES[dtype], B, L, H, n_iters)


def set_spin_limit(polls: int = 0) -> None:
    """pararnn_set_spin_limit: polls of a predecessor's carry record before a tile gives up (0 = default)."""
    _lib.pararnn_set_spin_limit.argtypes = [ctypes.c_uint]
    _raise(_lib.pararnn_set_spin_limit(int(polls)), "pararnn_set_spin_limit")


def set_fused(enable: bool = True) -> None:
    """pararnn_set_fused: allow (default) or forbid the fused multi-iteration launches."""
    _raise(_lib.pararnn_set_fused(int(enable)), "pararnn_set_fused")


def set_staging(enable: bool = True) -> None:
    """pararnn_set_staging: allow (default) or forbid the kernel variants that stage their inputs through LDS."""
    _raise(_lib.pararnn_set_staging(int(enable)), "pararnn_set_staging")


def solve_plan(tol: float, max_iter: int):
    """pararnn_solve_plan: Newton iterations per launch of a solve with the current settings."""
    buf = (ctypes.c_int * max(1, max_iter))()
    n = _lib.pararnn_solve_plan(float(tol), int(max_iter), buf, max(1, max_iter))
    if n < 0:
        raise ValueError("pararnn_solve_plan: invalid arguments")
    return [buf[i] for i in range(n)]


def set_streaming(mode: int = 0) -> None:
    """pararnn_set_streaming: streamed tile accesses of the memory-bound kernels chosen by size (0, default),
    never (1) or always (2)."""
    _raise(_lib.pararnn_set_streaming(int(mode)), "pararnn_set_streaming")


def set_workspace_reuse(enable: bool = False) -> None:
    """pararnn_set_workspace_reuse: the caller's promise that nothing else writes to a workspace between the
    library's calls on it; the carry records are then not cleared again for a call of the same layout."""
    _raise(_lib.pararnn_set_workspace_reuse(int(enable)), "pararnn_set_workspace_reuse")


def set_fused_tail(enable: bool = True) -> None:
    """pararnn_set_fused_tail: the blocks after a solve's first launch share one persistent launch (default)
    or are launches of their own."""
    _raise(_lib.pararnn_set_fused_tail(int(enable)), "pararnn_set_fused_tail")


def set_fused_head(n_iters: int = 5) -> None:
    """pararnn_set_fused_head: iterations a solve to a tolerance runs in its first launch (0 = none)."""
    _raise(_lib.pararnn_set_fused_head(int(n_iters)), "pararnn_set_fused_head")


def _ptr(t):
    return None if t is None else t.data_ptr()


def _check(t, name, dtype, shape=None):
    if not t.is_cuda:
        raise ValueError(f"{name} must be a CUDA tensor")
    if t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def _workspace(nbytes, device, workspace):
    if workspace is None:
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
    return workspace


def _raise(code, what):
    if code != 0:
        raise RuntimeError(f"{what} failed: {status_string(code)} ({code})")


def forward(cell, params, u, h0=None, tol: float = 1e-6, max_iter: int = 64, trace: bool = False,
            workspace=None, stream=None, out=None):
    """pararnn_forward (or <name>_forward of a UserCell).  u [B][L][G][H] (fp32 or bf16), params fp32.
    Returns (h, iters, delta_trace): iters is a DEVICE int32[2] tensor
    {iterations, status} (no synchronisation happens here), delta_trace a
    device float[max_iter] tensor or None."""
    G, S = cell_dims(cell)
    B, L, Gu, H = u.shape
    dt = u.dtype
    _check(u, "u", dt, (B, L, G, H))
    _check(params, "params", torch.float32)
    if h0 is not None:
        _check(h0, "h0", dt, (B, S, H))
    h = torch.empty((B, L, S, H), dtype=dt, device=u.device) if out is None else out
    _check(h, "h", dt, (B, L, S, H))
    iters = torch.empty(2, dtype=torch.int32, device=u.device)
    tr = torch.zeros(max(max_iter, 1), dtype=torch.float32, device=u.device) if trace else None
    need = workspace_bytes_fused(cell, dt, B, L, H, max_iter) if tol < 0 else workspace_bytes(cell, dt, B, L, H, False)
    ws = _workspace(need, u.device, workspace)
    api = _api(cell)
    code = api.fwd(DTYPES[dt], _ptr(params), _ptr(u), _ptr(h0), B, L, H, tol, max_iter,
                   _ptr(h), _ptr(iters), _ptr(tr), _ptr(ws), ws.numel(), _stream(stream))
    _raise(code, f"{api.what}_forward")
    return h, iters, tr


def forward_ex(cell, params, u, h0=None, tol: float = 1e-6, max_iter: int = 64, first_block: int = -1, fused: int = -1,
               trace: bool = False, workspace=None, stream=None, out=None):
    """pararnn_forward_ex (built-in cells): `forward` with the size of the first fused block and the
    fused switch as arguments of the call (-1 = the library's setting).  Same return values."""
    G, S = cell_dims(cell)
    B, L, Gu, H = u.shape
    dt = u.dtype
    _check(u, "u", dt, (B, L, G, H))
    _check(params, "params", torch.float32)
    if h0 is not None:
        _check(h0, "h0", dt, (B, S, H))
    h = torch.empty((B, L, S, H), dtype=dt, device=u.device) if out is None else out
    _check(h, "h", dt, (B, L, S, H))
    iters = torch.empty(2, dtype=torch.int32, device=u.device)
    tr = torch.zeros(max(max_iter, 1), dtype=torch.float32, device=u.device) if trace else None
    opt = _SolveOptions(int(first_block), int(fused))
    need = max(_lib.pararnn_workspace_bytes_ex(CELLS[cell], DTYPES[dt], B, L, H, ctypes.byref(opt)),
               workspace_bytes_fused(cell, dt, B, L, H, max_iter) if tol < 0 else 0)
    ws = _workspace(need, u.device, workspace)
    code = _lib.pararnn_forward_ex(CELLS[cell], DTYPES[dt], _ptr(params), _ptr(u), _ptr(h0), B, L, H, tol, max_iter,
                                   _ptr(h), _ptr(iters), _ptr(tr), _ptr(ws), ws.numel(), _stream(stream),
                                   ctypes.byref(opt))
    _raise(code, "pararnn_forward_ex")
    return h, iters, tr


def solve_plan_ex(tol: float, max_iter: int, first_block: int = -1, fused: int = -1):
    """pararnn_solve_plan_ex: Newton iterations per launch of a solve with the given options."""
    buf = (ctypes.c_int * max(1, max_iter))()
    opt = _SolveOptions(int(first_block), int(fused))
    n = _lib.pararnn_solve_plan_ex(float(tol), int(max_iter), ctypes.byref(opt), buf, max(1, max_iter))
    if n < 0:
        raise ValueError("pararnn_solve_plan_ex: invalid arguments")
    return [buf[i] for i in range(n)]


def forward_noalloc(cell, params, u, h0, tol, max_iter, out, iters, delta_trace=None, stream=None):
    """pararnn_forward_noalloc (built-in cells): the solve of `forward` on the library's static
    scratch array.  Nothing is allocated here either: `out` [B][L][S][H], `iters` (device int32[2])
    and, if wanted, `delta_trace` (device float[max_iter]) are the caller's.  Returns the C status
    code (0 = enqueued); a problem too large for the array gives WORKSPACE_TOO_SMALL (3)."""
    G, S = cell_dims(cell)
    B, L, Gu, H = u.shape
    dt = u.dtype
    _check(u, "u", dt, (B, L, G, H))
    _check(params, "params", torch.float32)
    if h0 is not None:
        _check(h0, "h0", dt, (B, S, H))
    _check(out, "h", dt, (B, L, S, H))
    _check(iters, "iters", torch.int32, (2,))
    if delta_trace is not None:
        _check(delta_trace, "delta_trace", torch.float32, (max(max_iter, 1),))
    return _lib.pararnn_forward_noalloc(CELLS[cell], DTYPES[dt], _ptr(params), _ptr(u), _ptr(h0), B, L, H, tol,
                                        max_iter, _ptr(out), _ptr(iters), _ptr(delta_trace), _stream(stream))


def backward(cell, params, u, h0, h, dL_dh, want_dh0: bool = True, workspace=None, stream=None, out=None):
    """pararnn_backward.  Returns (dL_du, dL_dparams, dL_dh0 or None); `out`
    may hold a preallocated (dL_du, dL_dparams, dL_dh0) triple."""
    G, S = cell_dims(cell)
    B, L, Gu, H = u.shape
    dt = u.dtype
    _check(u, "u", dt, (B, L, G, H))
    _check(params, "params", torch.float32)
    _check(h, "h", dt, (B, L, S, H))
    _check(dL_dh, "dL_dh", dt, (B, L, S, H))
    if h0 is not None:
        _check(h0, "h0", dt, (B, S, H))
    if out is not None:
        du, dparams, dh0 = out
        _check(du, "dL_du", dt, u.shape)
        _check(dparams, "dL_dparams", torch.float32, params.shape)
        if dh0 is not None:
            _check(dh0, "dL_dh0", dt, (B, S, H))
    else:
        du = torch.empty_like(u)
        dparams = torch.empty_like(params)
        dh0 = torch.empty((B, S, H), dtype=dt, device=u.device) if want_dh0 else None
    ws = _workspace(workspace_bytes(cell, dt, B, L, H, True), u.device, workspace)
    api = _api(cell)
    code = api.bwd(DTYPES[dt], _ptr(params), _ptr(u), _ptr(h0), _ptr(h), _ptr(dL_dh),
                   B, L, H, _ptr(du), _ptr(dparams), _ptr(dh0), _ptr(ws), ws.numel(), _stream(stream))
    _raise(code, f"{api.what}_backward")
    return du, dparams, dh0


def residual_norm(cell, params, u, h0, h, stream=None, out=None):
    """pararnn_residual_norm: max |h_l - f(h_{l-1}, u_l)| of the given states, as a device float[1]."""
    G, S = cell_dims(cell)
    B, L, Gu, H = u.shape
    dt = u.dtype
    _check(u, "u", dt, (B, L, G, H))
    _check(params, "params", torch.float32)
    _check(h, "h", dt, (B, L, S, H))
    if h0 is not None:
        _check(h0, "h0", dt, (B, S, H))
    if out is None:
        out = torch.empty(1, dtype=torch.float32, device=u.device)
    _check(out, "out", torch.float32, (1,))
    api = _api(cell)
    code = api.res(DTYPES[dt], _ptr(params), _ptr(u), _ptr(h0), _ptr(h), B, L, H, _ptr(out), _stream(stream))
    _raise(code, f"{api.what}_residual_norm")
    return out


_lib.pararnn_input_projection_workspace_bytes.restype = _sz
_lib.pararnn_input_projection_workspace_bytes.argtypes = [_i] * 7
_lib.pararnn_input_projection.restype = _i
_lib.pararnn_input_projection.argtypes = [_i, _vp, _vp, _vp, _i, _i, _i, _i, _i, _vp, _vp, _sz, _vp]
_lib.pararnn_input_projection_backward.restype = _i
_lib.pararnn_input_projection_backward.argtypes = [_i, _vp, _vp, _vp, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _sz, _vp]


def input_projection_workspace_bytes(dtype, B: int, L: int, H: int, G: int, n_heads: int = 1, backward: bool = False) -> int:
    return _lib.pararnn_input_projection_workspace_bytes(DTYPES[dtype], B, L, H, G, n_heads, int(backward))


def input_projection(x, Wx, bias=None, n_heads: int = 1, workspace=None, stream=None, out=None):
    """pararnn_input_projection.  x [B][L][H], Wx fp32 [G][H][H / n_heads], bias fp32 [G][H] or None
    -> u [B][L][G][H] of x's dtype."""
    B, L, H = x.shape
    G = Wx.shape[0]
    dt = x.dtype
    _check(x, "x", dt, (B, L, H))
    _check(Wx, "Wx", torch.float32, (G, H, H // n_heads))
    if bias is not None:
        _check(bias, "bias", torch.float32, (G, H))
    u = torch.empty((B, L, G, H), dtype=dt, device=x.device) if out is None else out
    _check(u, "u", dt, (B, L, G, H))
    ws = _workspace(input_projection_workspace_bytes(dt, B, L, H, G, n_heads), x.device, workspace)
    code = _lib.pararnn_input_projection(DTYPES[dt], _ptr(x), _ptr(Wx), _ptr(bias), B, L, H, G, n_heads, _ptr(u),
                                         _ptr(ws), ws.numel(), _stream(stream))
    _raise(code, "pararnn_input_projection")
    return u


def input_projection_backward(x, Wx, du, n_heads: int = 1, want_dx: bool = True, want_dw: bool = True,
                              want_dbias: bool = True, workspace=None, stream=None):
    """pararnn_input_projection_backward.  Returns (dx, dWx, dbias); entries not wanted are None."""
    B, L, H = x.shape
    G = Wx.shape[0]
    dt = x.dtype
    _check(x, "x", dt, (B, L, H))
    _check(Wx, "Wx", torch.float32, (G, H, H // n_heads))
    _check(du, "du", dt, (B, L, G, H))
    dx = torch.empty_like(x) if want_dx else None
    dW = torch.empty_like(Wx) if want_dw else None
    db = torch.empty((G, H), dtype=torch.float32, device=x.device) if want_dbias else None
    ws = _workspace(input_projection_workspace_bytes(dt, B, L, H, G, n_heads, True), x.device, workspace)
    code = _lib.pararnn_input_projection_backward(DTYPES[dt], _ptr(x), _ptr(Wx), _ptr(du), B, L, H, G, n_heads,
                                                  _ptr(dx), _ptr(dW), _ptr(db), _ptr(ws), ws.numel(), _stream(stream))
    _raise(code, "pararnn_input_projection_backward")
    return dx, dW, db


def affine_scan(J, r, reverse: bool = False, workspace=None, stream=None):
    """pararnn_affine_scan.  J [B][L][H] (diagonal) or [B][L][S][S][H] (blocks,
    S = 2, 3, 4); r [B][L][S][H] or [B][L][H].  Returns delta with r's shape."""
    B, L = r.shape[0], r.shape[1]
    H = r.shape[-1]
    if J.dim() == 3:
        kind = 0
        _check(J, "J", torch.float32, (B, L, H))
    else:
        S = J.shape[2]
        if J.dim() != 5 or S not in (2, 3, 4):
            raise ValueError("J must be [B][L][H] or [B][L][S][S][H] with S in 2..4")
        kind = S - 1
        _check(J, "J", torch.float32, (B, L, S, S, H))
    _check(r, "r", torch.float32)
    delta = torch.empty_like(r)
    ws = _workspace(_lib.pararnn_affine_scan_workspace_bytes(kind, int(reverse), B, L, H), r.device, workspace)
    code = _lib.pararnn_affine_scan(kind, int(reverse), _ptr(J), _ptr(r), B, L, H, _ptr(delta), _ptr(ws),
                                    ws.numel(), _stream(stream))
    _raise(code, "pararnn_affine_scan")
    return delta
