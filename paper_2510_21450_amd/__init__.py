"""MI355X-native sequence-parallel RNN application (Newton + affine prefix scan).

Thin Python binding over the C ABI of libpararnn.so (include/pararnn.h).
PyTorch is used for device memory and streams only; every step of the method
runs in the HIP kernels.  The library must have been built
(`python -m paper_2510_21450_amd.build`); importing without it fails.
"""
from .binding import (CELLS, DTYPES, STATUS, UserCell, example_cell, affine_scan, backward, cell_dims, dense_chunk, dense_chunk_products, forward, lib_path, set_fused, set_fused_head, set_tile, solve_plan,
                      status_string, version, workspace_bytes, workspace_bytes_fused)
from .autograd import rnn_apply

__all__ = ["rnn_apply", "UserCell", "example_cell", "CELLS", "DTYPES", "STATUS", "affine_scan", "backward", "cell_dims", "dense_chunk", "dense_chunk_products", "forward", "lib_path", "set_fused", "set_fused_head", "set_tile", "solve_plan",
           "status_string", "version", "workspace_bytes", "workspace_bytes_fused"]
