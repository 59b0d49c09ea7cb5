"""MI355X-native sequence-parallel RNN application (Newton + affine prefix scan).

Thin Python binding over the C ABI of libpararnn.so (include/pararnn.h).
PyTorch is used for device memory and streams only; every step of the method
runs in the HIP kernels.  The library must have been built
(`python -m paper_2510_21450_amd.build`): the binding is loaded on first use of
any name below and raises ImportError when the library is missing or older
than the binding (there is no CPU fallback).  Only the `build` submodule works
without the library.
"""
import importlib

_BINDING = ["CELLS", "DTYPES", "STATUS", "UserCell", "example_cell", "affine_scan", "backward", "cell_dims",
            "dense_chunk", "dense_chunk_products", "device_info", "forward", "forward_ex", "forward_noalloc", "input_projection", "input_projection_backward",
            "input_projection_workspace_bytes", "lib_path", "residual_norm", "set_dense_jacobian", "set_dense_tail", "set_dense_products", "set_fused", "set_fused_tail", "set_workspace_reuse",
            "set_fused_head", "set_spin_limit", "set_staging", "set_streaming", "set_tile", "solve_plan", "solve_plan_ex", "status_string", "version", "workspace_bytes",
            "workspace_bytes_fused"]
_AUTOGRAD = ["rnn_apply", "rnn_layer", "input_projection_apply"]
__all__ = _AUTOGRAD + _BINDING


def __getattr__(name):
    if name in _BINDING:
        return getattr(importlib.import_module(".binding", __name__), name)
    if name in _AUTOGRAD:
        return getattr(importlib.import_module(".autograd", __name__), name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")
