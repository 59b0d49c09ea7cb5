"""The five benchmark workloads: shapes, seeds and value distributions.

Tensor layouts (H contiguous everywhere):
  u      [B][L][G][H]   pre-activations, G gates per channel
  h, g   [B][L][S][H]   state / loss gradient, S state values per channel
  h0     [B][S][H]
  params diag cells: [2][G][H] = recurrent weights then biases (fp32)
         dense cell: W[H][H] row-major (fp32)
         ParaLSTM (CIFG + peepholes): [8][H] = a_f, a_z, a_o, c_f, c_o, b_f, b_z, b_o
Gate order: GRU (z, r, c); LSTM (i, f, o, g); ParaLSTM (f, z, o).  LSTM state order (c, h).
Streams of the generator: 1 = u, 2 = weights, 3 = h0, 4 = dL/dh, 5 = W.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
import torch

from .rng import normal, uniform_sym

BASE_SEED = 20251021

# cell name -> (gates G, state size S)
_DIMS = {"gru_diag": (3, 1), "lstm_diag": (4, 2), "tanh_dense": (1, 1), "linear_diag": (1, 1),
         "paralstm_diag": (3, 2)}


def cell_dims(cell: str):
    return _DIMS[cell]


@dataclass(frozen=True)
class Workload:
    name: str
    cell: str
    dtype: str          # storage of u, h0, h, g, du: "f32" or "bf16"
    B: int
    L: int
    H: int
    tol: float
    max_iter: int
    backward: bool
    seed: int
    h0_std: float = 0.0  # 0 -> h0 is all zeros
    w_bound: float = 0.9
    w_std_dense: float = 0.8

    def scaled(self, **kw) -> "Workload":
        """Same recipe at another size (used for cut-down parity cases)."""
        return replace(self, **kw)


CONFIGS = {
    "C1": Workload("C1", "gru_diag", "f32", 1, 64, 8, 1e-6, 64, False, BASE_SEED + 0),
    "C2": Workload("C2", "gru_diag", "f32", 16, 4096, 1024, 1e-5, 64, True, BASE_SEED + 1),
    "C3": Workload("C3", "lstm_diag", "f32", 8, 2048, 2048, 2e-5, 64, True, BASE_SEED + 2),
    "C4": Workload("C4", "tanh_dense", "f32", 64, 1024, 64, 1e-3, 32, False, BASE_SEED + 3),
    "C5": Workload("C5", "gru_diag", "bf16", 4, 65536, 4096, 2e-5, 64, True, BASE_SEED + 4,
                   h0_std=0.1),
}


# Beyond the five: the paper's own ParaLSTM cell (Eq. (7b)) on config 3's shapes and recipe.
EXTRA_CONFIGS = {
    "X3": Workload("X3", "paralstm_diag", "f32", 8, 2048, 2048, 1e-4, 64, True, BASE_SEED + 5),
}
ALL_CONFIGS = {**CONFIGS, **EXTRA_CONFIGS}


def _storage(dtype: str):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]


def make_inputs(w: Workload, device="cpu", need_g: bool | None = None) -> dict:
    """Generate params, u, h0 (None = zeros) and, for backward workloads, g."""
    G, S = cell_dims(w.cell)
    st = _storage(w.dtype)
    out = {}
    if w.cell == "tanh_dense":
        out["params"] = normal(w.seed, 5, (w.H, w.H), std=w.w_std_dense / w.H ** 0.5,
                               dtype=torch.float32, device=device)
    else:
        if w.cell == "paralstm_diag":
            # a_f, a_z, a_o, c_f, c_o ~ U(-bound, bound); b_f = +1, b_z = b_o = 0
            p = torch.zeros(8, w.H, dtype=torch.float32, device=device)
            p[:5] = uniform_sym(w.seed, 2, (5, w.H), w.w_bound, dtype=torch.float32, device=device)
            p[5] = 1.0
        else:
            p = torch.zeros(2, G, w.H, dtype=torch.float32, device=device)
            p[0] = uniform_sym(w.seed, 2, (G, w.H), w.w_bound, dtype=torch.float32, device=device)
            if w.cell == "lstm_diag":
                p[1, 1] = 1.0          # forget-gate bias +1
        out["params"] = p
    out["u"] = normal(w.seed, 1, (w.B, w.L, G, w.H), dtype=st, device=device)
    out["h0"] = (normal(w.seed, 3, (w.B, S, w.H), std=w.h0_std, dtype=st, device=device)
                 if w.h0_std > 0 else None)
    if w.backward if need_g is None else need_g:
        out["g"] = normal(w.seed, 4, (w.B, w.L, S, w.H), dtype=st, device=device)
    return out
