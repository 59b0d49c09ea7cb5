"""The seeded input generator: determinism, slice-wise regeneration,
distributions, bf16 rounding mode, and the shapes of the five workloads."""
import math

import numpy as np
import torch

from workloads import CONFIGS, make_inputs, normal, uniform01, uniform_sym, cell_dims
from workloads.rng import _key, _mix_int


def test_counter_based_and_deterministic():
    a = uniform01(7, 1, 1000)
    b = uniform01(7, 1, 1000)
    assert torch.equal(a, b)
    # any slice can be regenerated on its own
    assert torch.equal(uniform01(7, 1, 100, start=300), a[300:400])
    # streams and seeds are independent
    assert not torch.equal(uniform01(7, 2, 1000), a) and not torch.equal(uniform01(8, 1, 1000), a)
    assert float(a.min()) > 0.0 and float(a.max()) < 1.0
    # bit pattern agrees with a pure-python splitmix64
    k = _key(7, 1)
    want = [(float(_mix_int(i * 0x9E3779B97F4A7C15 + k) >> 11) + 0.5) / 2.0 ** 53 for i in range(5)]
    assert [float(x) for x in a[:5]] == want


def test_chunked_generation_matches_one_shot(monkeypatch):
    import workloads.rng as rng
    x = normal(3, 1, (5000,), dtype=torch.float64)
    monkeypatch.setattr(rng, "_CHUNK", 1024)
    y = normal(3, 1, (5000,), dtype=torch.float64)
    assert torch.equal(x, y)


def test_distributions():
    n = 400000
    z = normal(11, 1, (n,), dtype=torch.float64)
    assert abs(float(z.mean())) < 0.01 and abs(float(z.std()) - 1.0) < 0.01
    assert abs(float((z ** 3).mean())) < 0.03 and abs(float((z ** 4).mean()) - 3.0) < 0.1
    z2 = normal(11, 1, (n,), std=0.1, dtype=torch.float64)
    assert torch.allclose(z2, 0.1 * z)
    u = uniform_sym(11, 2, (n,), 0.9, dtype=torch.float64)
    assert float(u.abs().max()) < 0.9 and abs(float(u.mean())) < 0.01
    assert abs(float(u.std()) - 0.9 / math.sqrt(3)) < 0.01


def test_bf16_cast_rounds_to_nearest_even():
    # 1 + 2^-8 is exactly halfway between bf16 neighbours 1 and 1 + 2^-7: ties go to even (1.0);
    # 1 + 3*2^-8 is halfway between 1 + 2^-7 and 1 + 2^-6: even is 1 + 2^-6
    x = torch.tensor([1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20], dtype=torch.float32)
    y = x.to(torch.bfloat16).to(torch.float32)
    assert y.tolist() == [1.0, 1.0 + 2 ** -6, 1.0 + 2 ** -7]


def test_workload_shapes_and_recipes():
    expect = {"C1": ("gru_diag", "f32", 1, 64, 8), "C2": ("gru_diag", "f32", 16, 4096, 1024),
              "C3": ("lstm_diag", "f32", 8, 2048, 2048), "C4": ("tanh_dense", "f32", 64, 1024, 64),
              "C5": ("gru_diag", "bf16", 4, 65536, 4096)}
    for name, (cell, dt, B, L, H) in expect.items():
        w = CONFIGS[name]
        assert (w.cell, w.dtype, w.B, w.L, w.H) == (cell, dt, B, L, H)
    assert CONFIGS["C1"].tol == 1e-6 and CONFIGS["C1"].max_iter == 64 and CONFIGS["C4"].max_iter == 32
    assert not CONFIGS["C1"].backward and not CONFIGS["C4"].backward
    assert all(CONFIGS[c].backward for c in ("C2", "C3", "C5"))
    # small instances of each recipe
    w = CONFIGS["C3"].scaled(B=2, L=5, H=6)
    d = make_inputs(w)
    G, S = cell_dims(w.cell)
    assert d["params"].shape == (2, 4, 6) and d["u"].shape == (2, 5, 4, 6) and d["g"].shape == (2, 5, 2, 6)
    assert float(d["params"][0].abs().max()) < 0.9
    assert torch.equal(d["params"][1], torch.tensor([[0.0] * 6, [1.0] * 6, [0.0] * 6, [0.0] * 6]))   # b_f = +1
    assert d["h0"] is None
    w = CONFIGS["C5"].scaled(B=2, L=8, H=16)
    d = make_inputs(w)
    assert d["u"].dtype == torch.bfloat16 and d["h0"].dtype == torch.bfloat16 and d["params"].dtype == torch.float32
    assert 0.0 < float(d["h0"].float().std()) < 0.2
    w = CONFIGS["C4"].scaled(B=2, L=3)
    d = make_inputs(w)
    assert d["params"].shape == (64, 64) and abs(float(d["params"].std()) - 0.1) < 0.01
