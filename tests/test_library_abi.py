"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every function include/pararnn.h declares, and its host logic (status
strings, cell tables, workspace sizes, tile-shape hook, argument validation
that happens before any device work) behaves as the header says."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "pararnn.h")
LIB = os.path.join(ROOT, "paper_2510_21450_amd", "libpararnn.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2510_21450_amd import build
        build.build()
    return ctypes.CDLL(LIB)


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(pararnn_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_boundary():
    names = declared_functions()
    for must in ("pararnn_forward", "pararnn_backward", "pararnn_workspace_bytes", "pararnn_affine_scan"):
        assert must in names


def test_every_declared_symbol_is_exported(lib):
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} is declared in pararnn.h but not exported"


def test_status_strings_and_cell_tables(lib):
    lib.pararnn_status_string.restype = ctypes.c_char_p
    want = {0: "OK", 1: "NOT_CONVERGED", 2: "INVALID_ARG", 3: "WORKSPACE_TOO_SMALL", 4: "HIP_ERROR",
            5: "NONFINITE", 6: "UNSUPPORTED", 7: "INTERNAL", 99: "UNKNOWN"}
    for code, s in want.items():
        assert lib.pararnn_status_string(code).decode() == s
    assert lib.pararnn_version() >= 100
    assert [(lib.pararnn_cell_gates(c), lib.pararnn_cell_state(c)) for c in range(5)] == [(3, 1), (4, 2), (1, 1), (1, 1), (3, 2)]
    assert lib.pararnn_cell_gates(7) == -1 and lib.pararnn_cell_state(-1) == -1


def test_workspace_bytes(lib):
    ws = lib.pararnn_workspace_bytes
    ws.restype = ctypes.c_size_t
    ws.argtypes = [ctypes.c_int] * 6
    # invalid requests give 0
    assert ws(9, 0, 1, 1, 1, 0) == 0 and ws(0, 5, 1, 1, 1, 0) == 0 and ws(0, 0, 0, 8, 8, 0) == 0
    assert ws(0, 0, 4, -1, 8, 0) == 0
    small = ws(0, 0, 1, 64, 8, 0)
    assert small >= 256 and small % 256 == 0
    # grows with the problem; bf16 forward also holds the fp32 iterate
    f32 = ws(0, 0, 16, 4096, 1024, 0)
    bf = ws(0, 1, 16, 4096, 1024, 0)
    assert f32 > small and bf >= f32 + 16 * 4096 * 1024 * 4
    # the fp32 workspace (carry records for the fused first launch, boundary rows) is small next
    # to the tensors (u alone is 805 MB)
    assert f32 < 192 << 20
    # backward workspace holds the per-tile parameter-gradient partials
    assert ws(0, 0, 16, 4096, 1024, 1) > 0
    # dense path: d, r, chunk products
    assert ws(2, 0, 64, 1024, 64, 0) >= 2 * 64 * 1024 * 64 * 4 + 64 * 64 * 64 * 64 * 4


def test_input_projection_host_checks(lib):
    """Workspace sizes and the refusals that need no device."""
    vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    ws = lib.pararnn_input_projection_workspace_bytes
    ws.restype = sz
    ws.argtypes = [i] * 7
    fwd = ws(1, 16, 4096, 1024, 3, 4, 0)
    bwd = ws(1, 16, 4096, 1024, 3, 4, 1)
    assert fwd >= 3 * 1024 * 256 * 2 and fwd % 256 == 0            # the bf16 copy of the weights
    assert bwd > fwd + 3 * 1024 * 256 * 4                          # + partial sums of the weight gradient
    assert ws(0, 1, 4, 96, 3, 1, 0) == 0 and ws(0, 1, 4, 128, 3, 3, 0) == 0 and ws(2, 1, 4, 128, 3, 1, 0) == 0
    assert ws(0, 1, 4, 128, 9, 1, 0) == 0 and ws(0, 0, 4, 128, 3, 1, 0) == 0
    f = lib.pararnn_input_projection
    f.restype = i
    f.argtypes = [i, vp, vp, vp, i, i, i, i, i, vp, vp, sz, vp]
    p = 0x1000
    assert f(0, None, p, None, 1, 4, 128, 3, 1, p, p, 1 << 20, None) == 2          # x NULL
    assert f(0, p, p, None, 1, 4, 128, 3, 1, p, p + 8, 1 << 20, None) == 2         # workspace alignment
    assert f(0, p, p, None, 1, 4, 128, 3, 3, p, p, 1 << 20, None) == 2             # heads do not divide H
    assert f(0, p, p, None, 1, 4, 96, 3, 1, p, p, 1 << 20, None) == 6              # dh not a multiple of 64
    assert f(0, p + 4, p, None, 1, 4, 128, 3, 1, p, p, 1 << 20, None) == 6         # x not 16-byte aligned
    assert f(0, p, p, None, 1, 4, 128, 3, 1, p, p, 256, None) == 3                 # WORKSPACE_TOO_SMALL
    b = lib.pararnn_input_projection_backward
    b.restype = i
    b.argtypes = [i, vp, vp, vp, i, i, i, i, i, vp, vp, vp, vp, sz, vp]
    assert b(0, p, p, None, 1, 4, 128, 3, 1, p, p, p, p, 1 << 20, None) == 2       # du NULL
    assert b(0, p, p, p, 1, 4, 128, 3, 1, p, None, p, p, 1 << 20, None) == 2       # dbias without dWx
    assert b(0, p, p, p, 1, 4, 128, 3, 1, p, p, p, p, 256, None) == 3


def test_spin_limit_hook(lib):
    sl = lib.pararnn_set_spin_limit
    sl.argtypes = [ctypes.c_uint]
    assert sl(1) == 0 and sl(0) == 0          # 0 restores the default


def test_dense_products_switch(lib):
    sp = lib.pararnn_set_dense_products
    assert sp(1) == 0 and sp(2) == 0 and sp(0) == 0
    assert sp(3) == 2 and sp(-1) == 2


def test_dense_tail_switch(lib):
    st = lib.pararnn_set_dense_tail
    assert st(0) == 0 and st(2) == 0 and st(1) == 0
    assert st(3) == 2 and st(-1) == 2


def test_dense_jacobian_switch(lib):
    sj = lib.pararnn_set_dense_jacobian
    assert sj(1) == 0 and sj(0) == 0
    assert sj(2) == 2 and sj(-1) == 2


def test_tile_hook(lib):
    st = lib.pararnn_set_tile
    assert st(4, 4, 8, 8) == 0          # a compiled shape
    assert st(3, 1, 8, 8) == 6          # UNSUPPORTED
    assert st(4, 4, 8, 7) == 6
    assert st(1, 1, 8, 16) == 0
    assert st(0, 0, 0, 0) == 0          # back to automatic


def test_host_side_argument_validation(lib):
    """These requests are refused before any device call is made."""
    f = lib.pararnn_forward
    f.restype = ctypes.c_int
    vp, i, fl, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    f.argtypes = [i, i, vp, vp, vp, i, i, i, fl, i, vp, vp, vp, vp, sz, vp]
    p = 0x1000  # any aligned non-null address: it is never dereferenced on these paths
    INVALID = 2
    assert f(9, 0, p, p, None, 1, 8, 8, 1e-6, 4, p, p, None, p, 1 << 20, None) == INVALID      # cell
    assert f(0, 3, p, p, None, 1, 8, 8, 1e-6, 4, p, p, None, p, 1 << 20, None) == INVALID      # dtype
    assert f(0, 0, p, p, None, 0, 8, 8, 1e-6, 4, p, p, None, p, 1 << 20, None) == INVALID      # B = 0
    assert f(0, 0, p, p, None, 1, 8, 8, 1e-6, -1, p, p, None, p, 1 << 20, None) == INVALID     # max_iter
    assert f(0, 0, None, p, None, 1, 8, 8, 1e-6, 4, p, p, None, p, 1 << 20, None) == INVALID   # params NULL
    assert f(0, 0, p, p, None, 1, 8, 8, float("nan"), 4, p, p, None, p, 1 << 20, None) == INVALID
    assert f(0, 0, p, p, None, 1, 8, 8, 1e-6, 4, p, p, None, p + 8, 1 << 20, None) == INVALID  # workspace alignment
    assert f(0, 0, p, p, None, 1, 8, 8, 1e-6, 4, p, p, None, p, 16, None) == 3                 # WORKSPACE_TOO_SMALL
    b = lib.pararnn_backward
    b.restype = ctypes.c_int
    b.argtypes = [i, i, vp, vp, vp, vp, vp, i, i, i, vp, vp, vp, vp, sz, vp]
    assert b(0, 0, p, p, None, p, None, 1, 8, 8, p, p, None, p, 1 << 20, None) == INVALID      # dL_dh NULL
    assert b(2, 0, p, p, None, p, p, 1, 8, 32, p, p, None, p, 1 << 20, None) == 6              # dense path: H = 64 only
    assert b(2, 0, p, p, None, p, p, 1, 8, 64, p, p, None, p, 4096, None) == 3                 # dense backward workspace
    s = lib.pararnn_affine_scan
    s.restype = ctypes.c_int
    s.argtypes = [i, i, vp, vp, i, i, i, vp, vp, sz, vp]
    assert s(4, 0, p, p, 1, 8, 8, p, p, 1 << 20, None) == INVALID and s(-1, 0, p, p, 1, 8, 8, p, p, 1 << 20, None) == INVALID
    assert s(3, 0, p, p, 1, 8, 8, p, p, 16, None) == 3            # 4x4 blocks are a valid kind
    sw = lib.pararnn_affine_scan_workspace_bytes
    sw.restype = ctypes.c_size_t
    sw.argtypes = [i] * 5
    assert sw(4, 0, 1, 8, 8) == 0 and 0 < sw(0, 0, 2, 100, 64) < sw(1, 0, 2, 100, 64) < sw(3, 0, 2, 100, 64)
    assert s(0, 0, p, p, 1, 8, 8, p, p, 16, None) == 3


@pytest.mark.parametrize("name,gsp", [("gru_softsign", (3, 1, 6)), ("gru_sigmoid_identity_tanh", (3, 1, 6)),
                                      ("gru_sigmoid_softsign_identity", (3, 1, 6)), ("gru_sigmoid_tanh_softsign", (3, 1, 6)), ("rot_tanh", (2, 2, 2)), ("tri_tanh", (3, 3, 9)),
                                      ("quad_tanh", (4, 4, 16))])
def test_user_cell_libraries_export_their_abi(lib, name, gsp):
    """A library made by PARARNN_DEFINE_CELL (include/pararnn_cell.h) exports the functions the
    header lists and validates arguments like the built-in entry points."""
    path = os.path.join(ROOT, "paper_2510_21450_amd", f"libpararnn_{name}.so")
    if not os.path.exists(path):
        from paper_2510_21450_amd import build
        build.build_examples()
    ul = ctypes.CDLL(path)
    for fn in ("gates", "state", "param_rows", "workspace_bytes", "workspace_bytes_fused", "forward", "backward",
               "residual_norm"):
        assert hasattr(ul, f"{name}_{fn}")
    f = lambda s: getattr(ul, f"{name}_{s}")
    assert (f("gates")(), f("state")(), f("param_rows")()) == gsp
    ws = f("workspace_bytes")
    ws.restype = ctypes.c_size_t
    ws.argtypes = [ctypes.c_int] * 5
    assert ws(3, 1, 8, 8, 0) == 0 and ws(0, 0, 8, 8, 0) == 0
    assert ws(0, 2, 1000, 64, 0) >= 256 and ws(1, 2, 1000, 64, 0) >= ws(0, 2, 1000, 64, 0) + 2 * 1000 * gsp[1] * 64 * 4
    vp, i, fl, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    fw = f("forward")
    fw.restype = ctypes.c_int
    fw.argtypes = [i, vp, vp, vp, i, i, i, fl, i, vp, vp, vp, vp, sz, vp]
    p = 0x1000
    assert fw(3, p, p, None, 1, 8, 8, 1e-6, 4, p, p, None, p, 1 << 20, None) == 2       # dtype
    assert fw(0, None, p, None, 1, 8, 8, 1e-6, 4, p, p, None, p, 1 << 20, None) == 2    # params NULL
    assert fw(0, p, p, None, 1, 8, 8, 1e-6, 4, p, p, None, p, 16, None) == 3            # WORKSPACE_TOO_SMALL
    bw = f("backward")
    bw.restype = ctypes.c_int
    bw.argtypes = [i, vp, vp, vp, vp, vp, i, i, i, vp, vp, vp, vp, sz, vp]
    assert bw(0, p, p, None, p, None, 1, 8, 8, p, p, None, p, 1 << 20, None) == 2       # dL_dh NULL
    assert bw(0, p, p, None, p, p, 1, 8, 8, p, p, None, p, 16, None) == 3
    rn = f("residual_norm")
    rn.restype = ctypes.c_int
    rn.argtypes = [i, vp, vp, vp, vp, i, i, i, vp, vp]
    assert rn(0, p, p, None, p, 1, 8, 8, None, None) == 2                                # out NULL
    assert rn(0, p, p, None, p, 0, 8, 8, p, None) == 2                                   # B = 0
    # the settings are the main library's: switching fused launches off shrinks this library's workspace too
    big = ws(0, 4, 4096, 256, 0)
    lib.pararnn_set_fused(0)
    try:
        assert ws(0, 4, 4096, 256, 0) < big
    finally:
        lib.pararnn_set_fused(1)


def test_python_binding_refuses_cpu_tensors():
    import torch
    import paper_2510_21450_amd as P
    with pytest.raises(ValueError, match="CUDA"):
        P.forward("gru_diag", torch.zeros(2, 3, 8), torch.zeros(1, 4, 3, 8))


def test_solve_plan(lib):
    """The launch schedule of a solve: a first fused block, then blocks of 1, 2, 4, ...
    iterations capped by the size of the first; sizes add up to max_iter."""
    plan = lib.pararnn_solve_plan
    plan.restype = ctypes.c_int
    plan.argtypes = [ctypes.c_float, ctypes.c_int, ctypes.POINTER(ctypes.c_int), ctypes.c_int]
    buf = (ctypes.c_int * 256)()

    def blocks(tol, max_iter):
        n = plan(tol, max_iter, buf, 256)
        assert 0 <= n <= 256
        return [buf[i] for i in range(n)]

    try:
        assert lib.pararnn_set_fused_head(5) == 0 and lib.pararnn_set_fused(1) == 0
        assert blocks(1e-5, 64) == [5, 1, 2, 4] + [5] * 10 + [2]
        assert blocks(1e-5, 5) == [5] and blocks(1e-5, 3) == [3] and blocks(1e-5, 0) == []
        assert blocks(1e-5, 6) == [5, 1] and blocks(1e-5, 9) == [5, 1, 2, 1]
        # fixed-count solves: one launch up to 8 iterations, else one launch per iteration
        assert blocks(-1.0, 3) == [3] and blocks(-1.0, 8) == [8] and blocks(-1.0, 10) == [1] * 10
        for head in range(0, 9):
            assert lib.pararnn_set_fused_head(head) == 0
            for max_iter in (1, 2, 7, 8, 9, 31, 64, 200):
                b = blocks(1e-6, max_iter)
                assert sum(b) == max_iter and all(1 <= k <= max(head, 1) for k in b)
                assert b[0] == (min(head, max_iter) if head else 1)
                if head >= 4:
                    assert len(b) <= 4 + max_iter // head + 1
        assert lib.pararnn_set_fused_head(9) == 2 and lib.pararnn_set_fused_head(-1) == 2
        lib.pararnn_set_fused_head(5)
        # more launches than the caller has room for: the count is still returned
        assert plan(1e-5, 64, buf, 2) == 15 and plan(1e-5, -1, buf, 2) == -1
        lib.pararnn_set_fused(0)
        assert blocks(1e-5, 7) == [1] * 7 and blocks(-1.0, 3) == [1] * 3
    finally:
        lib.pararnn_set_fused(1)
        lib.pararnn_set_fused_head(5)


def test_residual_norm_host_checks(lib):
    """Refusals of pararnn_residual_norm that need no device."""
    vp, i = ctypes.c_void_p, ctypes.c_int
    f = lib.pararnn_residual_norm
    f.restype = i
    f.argtypes = [i, i, vp, vp, vp, vp, i, i, i, vp, vp]
    p = 0x1000
    assert f(0, 0, p, p, None, p, 1, 4, 8, None, None) == 2            # out NULL
    assert f(0, 0, p, None, None, p, 1, 4, 8, p, None) == 2            # u NULL
    assert f(9, 0, p, p, None, p, 1, 4, 8, p, None) == 2               # unknown cell
    assert f(0, 2, p, p, None, p, 1, 4, 8, p, None) == 2               # unknown dtype
    assert f(0, 0, p, p, None, p, 1, 0, 8, p, None) == 2               # L = 0
    assert f(0, 0, p, p + 2, None, p, 1, 4, 8, p, None) == 2           # fp32 u at an odd 2-byte address
    assert f(2, 1, p, p, None, p, 1, 4, 64, p, None) == 6              # dense cell: fp32 only
    assert f(2, 0, p, p, None, p, 1, 4, 32, p, None) == 6              # dense cell: H = 64 only


def test_device_info_argument_checks(lib):
    """pararnn_device_info refuses a missing or short buffer (no device is needed for that)."""
    f = lib.pararnn_device_info
    f.restype = ctypes.c_int
    f.argtypes = [ctypes.POINTER(ctypes.c_int), ctypes.c_int]
    buf = (ctypes.c_int * 8)()
    assert f(None, 8) == -1 and f(buf, 5) == -1


class SolveOptions(ctypes.Structure):
    _fields_ = [("first_block", ctypes.c_int), ("fused", ctypes.c_int)]


def test_per_call_solve_options(lib):
    """pararnn_forward_ex / pararnn_workspace_bytes_ex / pararnn_solve_plan_ex take the size of the first
    fused block and the fused switch with the call: same plans and sizes as the process-wide setters
    give, without touching them; fields out of range are refused."""
    vp, i, fl, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    opt_p = ctypes.POINTER(SolveOptions)
    plan = lib.pararnn_solve_plan_ex
    plan.restype = i
    plan.argtypes = [fl, i, opt_p, ctypes.POINTER(i), i]
    plan0 = lib.pararnn_solve_plan
    plan0.restype = i
    plan0.argtypes = [fl, i, ctypes.POINTER(i), i]
    wsx = lib.pararnn_workspace_bytes_ex
    wsx.restype = sz
    wsx.argtypes = [i, i, i, i, i, opt_p]
    ws = lib.pararnn_workspace_bytes
    ws.restype = sz
    ws.argtypes = [i] * 6
    buf = (i * 64)()

    def blocks(tol, max_iter, **kw):
        o = SolveOptions(kw.get("first_block", -1), kw.get("fused", -1))
        n = plan(tol, max_iter, ctypes.byref(o), buf, 64)
        return [buf[k] for k in range(n)]

    lib.pararnn_set_fused_head(5)
    lib.pararnn_set_fused(1)
    # the paper's three iterations as the first launch
    assert blocks(1e-5, 10, first_block=3) == [3, 1, 2, 3, 1]
    assert blocks(1e-5, 10) == [5, 1, 2, 2] and blocks(1e-5, 10, first_block=0) == [1] * 10
    assert blocks(1e-5, 10, fused=0) == [1] * 10 and blocks(-1.0, 3, fused=0) == [1, 1, 1]
    assert plan(1e-5, 10, None, buf, 64) == plan0(1e-5, 10, buf, 64)
    # the process-wide settings were not touched
    n = plan0(1e-5, 10, buf, 64)
    assert [buf[k] for k in range(n)] == [5, 1, 2, 2]
    for bad in (SolveOptions(9, -1), SolveOptions(-2, -1), SolveOptions(3, 2), SolveOptions(3, -2)):
        assert plan(1e-5, 10, ctypes.byref(bad), buf, 64) == -1
        assert wsx(0, 0, 4, 4096, 256, ctypes.byref(bad)) == 0
    # workspace: one record slot per iteration of the first block
    dflt = ws(0, 0, 4, 4096, 256, 0)
    assert wsx(0, 0, 4, 4096, 256, None) == dflt
    three, none = wsx(0, 0, 4, 4096, 256, ctypes.byref(SolveOptions(3, -1))), wsx(0, 0, 4, 4096, 256, ctypes.byref(SolveOptions(0, -1)))
    assert none < three < dflt
    lib.pararnn_set_fused_head(3)
    try:
        assert ws(0, 0, 4, 4096, 256, 0) == three
        assert wsx(0, 0, 4, 4096, 256, ctypes.byref(SolveOptions(5, -1))) == dflt
    finally:
        lib.pararnn_set_fused_head(5)
    f = lib.pararnn_forward_ex
    f.restype = i
    f.argtypes = [i, i, vp, vp, vp, i, i, i, fl, i, vp, vp, vp, vp, sz, vp, opt_p]
    p = 0x1000
    assert f(0, 0, p, p, None, 1, 8, 8, 1e-6, 4, p, p, None, p, 1 << 20, None, ctypes.byref(SolveOptions(9, -1))) == 2
    assert f(0, 0, p, p, None, 1, 8, 8, 1e-6, 4, p, p, None, p, 16, None, ctypes.byref(SolveOptions(3, -1))) == 3
    assert f(0, 0, None, p, None, 1, 8, 8, 1e-6, 4, p, p, None, p, 1 << 20, None, None) == 2


def test_channel_count_bound(lib):
    """H beyond 2^22 would overflow the 32-bit row offsets of the kernels' buffer instructions: refused."""
    ws = lib.pararnn_workspace_bytes
    ws.restype = ctypes.c_size_t
    ws.argtypes = [ctypes.c_int] * 6
    assert ws(0, 0, 1, 4, 1 << 22, 0) > 0 and ws(0, 0, 1, 4, (1 << 22) + 64, 0) == 0
    f = lib.pararnn_forward
    f.restype = ctypes.c_int
    vp, i, fl, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    f.argtypes = [i, i, vp, vp, vp, i, i, i, fl, i, vp, vp, vp, vp, sz, vp]
    p = 0x1000
    assert f(0, 0, p, p, None, 1, 4, (1 << 22) + 64, 1e-6, 4, p, p, None, p, 1 << 30, None) == 2


def test_user_cell_builds_from_the_public_headers_alone(tmp_path):
    """A cell written against include/pararnn_cell.h compiles with nothing but -I include: the
    headers a cell library needs (driver, kernels, launchers) are shipped under include/pararnn/."""
    import shutil
    import subprocess
    src = tmp_path / "my_cell.hip"
    shutil.copy(os.path.join(ROOT, "paper_2510_21450_amd", "user_cells", "quad_tanh.hip"), src)
    cmd = ["/opt/rocm/bin/hipcc", "--offload-arch=gfx950", "-O1", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", f"-I{os.path.join(ROOT, 'include')}",
           "-c", str(src), "-o", str(tmp_path / "my_cell.o")]
    r = subprocess.run(cmd, cwd=tmp_path, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    text = open(src).read() + open(os.path.join(ROOT, "include", "pararnn_cell.h")).read() \
        + open(os.path.join(ROOT, "include", "pararnn_nonlin.h")).read()
    assert "csrc" not in text and "../" not in text.replace("../pararnn.h", "")
