"""Writes tests/golden/newton_traces.json: the oracle's max|delta h| per Newton
iteration (Alg. 1a with Eq. (4) as inner solver) on the full-size benchmark
workloads, in fp64 and in fp32.  Calls only oracle/ and the input generator.

The stopping test is global over the batch, so a workload is processed in
channel slices with a fixed iteration count (tol < 0) and the per-iteration
maxima are combined with max().  The diagonal cells' channels are independent,
so a slice of channels is moved into the batch axis to use all host threads.

Usage: python tests/golden/make_traces.py [C1 C2 ... X3]   (C5 takes ~15 min)
"""
import json
import os
import sys

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle                                   # noqa: E402
from workloads import ALL_CONFIGS as CONFIGS, make_inputs      # noqa: E402

OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "newton_traces.json")
N_ITERS = 9


def traces_for(name):
    w = CONFIGS[name]
    d = make_inputs(w, need_g=False)
    res = {"B": w.B, "L": w.L, "H": w.H, "cell": w.cell, "dtype": w.dtype, "seed": w.seed}
    params = d["params"].double().numpy()
    for prec in ("f64", "f32"):
        m = np.zeros(N_ITERS)
        if w.cell == "tanh_dense":
            u = d["u"].double().numpy()
            _, _, _, tr = oracle.newton(w.cell, params, u, None, tol=-1.0, max_iter=N_ITERS, precision=prec)
            m = np.maximum(m, tr)
        else:
            step = min(w.H, 64)
            group = 8                                   # slices handled per call
            for c0 in range(0, w.H, step * group):
                sl = slice(c0, min(w.H, c0 + step * group))
                us = d["u"][..., sl].double().numpy()          # [B][L][G][hs]
                B, L, G, hs = us.shape
                nb = hs // step
                # channels -> batch: [B][L][G][nb][step] -> [B*nb][L][G][step]
                us = us.reshape(B, L, G, nb, step).transpose(0, 3, 1, 2, 4).reshape(B * nb, L, G, step)
                ps = params[..., sl]
                h0 = None
                if d["h0"] is not None:
                    h0 = d["h0"][..., sl].double().numpy()
                    S = h0.shape[1]
                    h0 = h0.reshape(B, S, nb, step).transpose(0, 2, 1, 3).reshape(B * nb, S, step)
                tr_all = np.zeros(N_ITERS)
                for k in range(nb):
                    pk = ps[..., k * step:(k + 1) * step]
                    uk = us[k::nb]
                    hk = None if h0 is None else h0[k::nb]
                    _, _, _, tr = oracle.newton(w.cell, pk, uk, hk, tol=-1.0, max_iter=N_ITERS, precision=prec)
                    tr_all = np.maximum(tr_all, tr)
                m = np.maximum(m, tr_all)
                print(name, prec, "channels", sl, " ".join("%.2e" % x for x in m), flush=True)
        res[prec] = [float(x) for x in m]
    return res


def main():
    names = sys.argv[1:] or ["C1", "C2", "C3", "C4"]
    data = {}
    if os.path.exists(OUT):
        with open(OUT) as f:
            data = json.load(f)
    for n in names:
        data[n] = traces_for(n)
        with open(OUT, "w") as f:
            json.dump(data, f, indent=1, sort_keys=True)
        print(n, "f64", data[n]["f64"], "\n  f32", data[n]["f32"], flush=True)


if __name__ == "__main__":
    main()
