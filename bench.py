"""Benchmark of the hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: the
forward Newton solve (initial guess + Newton iterations until max|dh| <= tol)
and, for workloads that have one, the backward adjoint scan.  Inputs are
resident in HBM before the timed region.

Prints ONE JSON line: whole-job throughput in timestep-channels/s, the roofline
record of the dominant kernel (the fused block of Newton iterations; for the
dense cell the Jacobian-composition kernel) measured live with device events,
and the CPU oracle timed on the host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_F32_PEAK_TFLOPS = 157.3   # MI355X dense fp32 matrix peak, published
# fp32 vector peak of the instructions this build may use: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz x 2 (FMA).
# The published 157.3 TFLOP/s needs packed two-wide FMAs, which the build switches off.
VALU_F32_PEAK_TFLOPS = 78.6
FUSED_HEAD = 5                 # iterations in the first launch of a solve (the library's default)
# algorithmic bytes per timestep-channel (per-iteration kernel: read u + read iterate + write iterate;
# fused block: read u + write h, plus the fp32 iterate it leaves for later launches under bf16 storage;
# backward: read h, u, g + write du), storage sizes per workload
ALGO_BYTES = {
    "C1": {"iter": 20, "block": 16, "bwd": 32}, "C2": {"iter": 20, "block": 16, "bwd": 32},
    "C3": {"iter": 32, "block": 24, "bwd": 48}, "C5": {"iter": 14, "block": 12, "bwd": 16},
    "X3": {"iter": 28, "block": 20, "bwd": 40},     # ParaLSTM: 3 gates, state (c, h)
}
# algorithmic fp32 operations per timestep-channel and Newton iteration (cell, Jacobian, residual, the
# thread-level scan step and the back-substitution; +, -, *, / and exp count one each)
ALGO_FLOPS = {"gru_diag": 49, "lstm_diag": 93, "paralstm_diag": 92}
# From rocprofv3 --pmc passes over this file's own run (profiles/newton_fused_*.txt), per launch of the first
# fused block: HBM bytes moved (FETCH_SIZE / WRITE_SIZE scaled by their reading for a plain copy of known
# size), and the cycles its vector ALUs were busy summed over the 1024 SIMDs (4 x SQ_ACTIVE_INST_VALU).
MEASURED_TRAFFIC = {"C2": 1204.1e6, "C3": 1044.3e6, "C5": 15036.7e6,
                    "C4": 81.6e6}   # C4: the stand-alone chunk-products launch (d in, 3968 products of 16 KB out)
MEASURED_VALU_BUSY_CYCLES = {"C2": 1.1165e9, "C3": 0.9917e9, "C5": 1.8168e10}


def note(msg):
    """Progress on stderr (stdout carries the one JSON line)."""
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def time_events(fn, reps):
    import torch
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in evs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return [a.elapsed_time(b) for a, b in evs]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="C2", choices=["C1", "C2", "C3", "C4", "C5", "X3"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no sharding or collectives are part of it); "
                 "run with --gpus 1")

    import torch
    import paper_2510_21450_amd as P
    from workloads import ALL_CONFIGS as CONFIGS, make_inputs, cell_dims

    torch.cuda.set_device(0)
    P.set_fused_head(FUSED_HEAD)
    w = CONFIGS[args.config]
    G, S = cell_dims(w.cell)
    d = make_inputs(w, device="cuda")
    params, u, h0, g = d["params"], d["u"], d["h0"], d.get("g")
    N = w.B * w.L * w.H
    ws_f = torch.empty(P.workspace_bytes(w.cell, u.dtype, w.B, w.L, w.H, False), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(max(256, P.workspace_bytes(w.cell, u.dtype, w.B, w.L, w.H, True)), dtype=torch.uint8, device="cuda")
    h_out = torch.empty((w.B, w.L, S, w.H), dtype=u.dtype, device="cuda")
    state = {}

    def step():
        h, iters, _ = P.forward(w.cell, params, u, h0, tol=w.tol, max_iter=w.max_iter, workspace=ws_f, out=h_out)
        state["iters"] = iters
        if w.backward:
            state["grads"] = P.backward(w.cell, params, u, h0, h, g, workspace=ws_b)

    note(f"inputs ready: {w.name} {w.cell} {w.dtype} B={w.B} L={w.L} H={w.H}")
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    iters, status = (int(x) for x in state["iters"].cpu())
    note(f"{args.steps} timed steps: {ms_per_step:.4f} ms per step, iters={iters}")
    t_steps = sorted(time_events(step, max(args.steps, 20)))      # per step, device events: minimum and median

    # ---- per-kernel figures with device events on the launch stream
    def fwd_fixed(m):
        return lambda: P.forward(w.cell, params, u, h0, tol=-1.0, max_iter=m, workspace=ws_f, out=h_out)

    # one launch per iteration (the path without fused blocks): time per Newton iteration
    P.set_fused(False)
    m_lo, m_hi = 2, 10
    for m in (m_lo, m_hi):
        fwd_fixed(m)()
    t_lo = time_events(fwd_fixed(m_lo), 10)
    t_hi = time_events(fwd_fixed(m_hi), 10)
    P.set_fused(True)
    t_iter_ms = (sum(t_hi) / len(t_hi) - sum(t_lo) / len(t_lo)) / (m_hi - m_lo)
    t_iter_min_ms = (min(t_hi) - min(t_lo)) / (m_hi - m_lo)
    t_fwd = time_events(lambda: P.forward(w.cell, params, u, h0, tol=w.tol, max_iter=w.max_iter, workspace=ws_f,
                                          out=h_out), 10)
    detail = {"iters": iters, "status": P.status_string(status), "tol": w.tol, "max_iter": w.max_iter,
              "ms_per_step_min": t_steps[0], "ms_per_step_median": t_steps[len(t_steps) // 2],
              "launches": P.solve_plan(w.tol, w.max_iter) if w.cell != "tanh_dense" else None,
              "t_fwd_ms": sum(t_fwd) / len(t_fwd), "t_fwd_min_ms": min(t_fwd),
              "t_iter_ms": t_iter_ms, "t_iter_min_ms": t_iter_min_ms}
    # what the runtime reports for this device, beside the published figures the rooflines use
    props = torch.cuda.get_device_properties(0)
    dev = {"name": props.name, "arch": getattr(props, "gcnArchName", None), "memory_gib": props.total_memory / 2 ** 30}
    dev.update(P.device_info())
    detail["device"] = dev
    if w.cell == "tanh_dense":
        # the scan composes one 64x64 Jacobian product (2 H^3 flop) per timestep
        flops_iter = 2.0 * w.H ** 3 * w.B * w.L
        chunk = P.dense_chunk()
        n_c = (w.L + chunk - 1) // chunk
        flops_kernel = 2.0 * w.H ** 3 * w.B * max(0, n_c - 2) * (chunk - 1)
        detail["iter_tflops"] = flops_iter / (t_iter_ms * 1e-3) / 1e12
        detail["iter_frac_mfma"] = detail["iter_tflops"] / MFMA_F32_PEAK_TFLOPS
        # the composition kernel alone, same launch as inside the solve, on Jacobian factors of the same
        # distribution (d = 1 - tanh^2 of the converged states)
        dfac = (1.0 - h_out.view(w.B, w.L, w.H) ** 2).contiguous()
        Aout = torch.zeros((w.B, n_c, w.H, w.H), dtype=torch.float32, device="cuda")
        P.dense_chunk_products(params, dfac, out=Aout)
        t_ks = time_events(lambda: P.dense_chunk_products(params, dfac, out=Aout), 20)
        t_k = sum(t_ks) / len(t_ks)
        ach = flops_kernel / (t_k * 1e-3) / 1e12
        detail["chunk_products_ms"] = t_k
        # not part of the step (config 4 is forward only): the adjoint scan of the same cell
        gd = torch.randn_like(h_out)
        ws_db = torch.empty(P.workspace_bytes(w.cell, u.dtype, w.B, w.L, w.H, True), dtype=torch.uint8, device="cuda")
        dense_bwd = lambda: P.backward(w.cell, params, u, h0, h_out, gd, workspace=ws_db)
        dense_bwd()
        t_db = time_events(dense_bwd, 10)
        detail["dense_backward_ms"] = sum(t_db) / len(t_db)
        # inexact Newton (opt-in, not the timed step): Jacobian products from bf16 terms, fp32 residual
        inexact = {}
        for mode, name in ((1, "bf16x3"), (2, "bf16")):
            P.set_dense_products(mode)
            try:
                solve = lambda: P.forward(w.cell, params, u, h0, tol=w.tol, max_iter=w.max_iter, workspace=ws_f, out=h_out)
                _, it_m, _ = solve()
                t_m = time_events(solve, 10)
                t_km = time_events(lambda: P.dense_chunk_products(params, dfac, out=Aout), 10)
                it_m = [int(x) for x in it_m.cpu()]
                inexact[name] = {"t_fwd_ms": sum(t_m) / len(t_m), "iters": it_m[0], "status": P.status_string(it_m[1]),
                                 "chunk_products_ms": sum(t_km) / len(t_km)}
            finally:
                P.set_dense_products(0)
        detail["inexact_products"] = inexact
        # not part of the timed step: the quasi-Newton ablation (the Jacobian replaced by its diagonal,
        # a diagonal scan instead of the matrix products; linear convergence, more iterations)
        P.set_dense_jacobian(1)
        try:
            solve = lambda: P.forward(w.cell, params, u, h0, tol=w.tol, max_iter=w.max_iter, workspace=ws_f, out=h_out)
            _, it_q, _ = solve()
            t_q = time_events(solve, 10)
            it_q = [int(x) for x in it_q.cpu()]
            detail["quasi_newton_diagonal"] = {"t_fwd_ms": sum(t_q) / len(t_q), "iters": it_q[0],
                                               "status": P.status_string(it_q[1])}
        finally:
            P.set_dense_jacobian(0)
        P.forward(w.cell, params, u, h0, tol=w.tol, max_iter=w.max_iter, workspace=ws_f, out=h_out)
        roofline = {"bound": "mfma", "kernel": "dense_products_sweep_kernel (chunk products part)", "achieved": ach,
                    "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": ach / MFMA_F32_PEAK_TFLOPS, "traffic": MEASURED_TRAFFIC.get(args.config)}
    else:
        ab = ALGO_BYTES[args.config]
        iter_gbs = ab["iter"] * N / (t_iter_ms * 1e-3) / 1e9
        detail.update({"iter_bytes_per_elt": ab["iter"], "iter_gbs": iter_gbs, "iter_frac_hbm": iter_gbs / HBM_PEAK_GBS})
        # The dominant launch of a solve: its first fused block of FUSED_HEAD iterations from the initial
        # guess (u read once, the iterate in registers, h written once).  Timed as the library runs it
        # inside a solve: a tolerance that is met at once ends the solve after this launch, which still
        # performs all its iterations; the call also holds the reset of the carry records and one
        # launch that returns at once.
        K0 = min(FUSED_HEAD, w.max_iter)
        block = lambda: P.forward(w.cell, params, u, h0, tol=3.0e38, max_iter=K0 + 1, workspace=ws_f, out=h_out)
        block()
        t_blk = time_events(block, 10)
        t_block_ms = sum(t_blk) / len(t_blk)
        flops = ALGO_FLOPS[w.cell] * float(N) * K0
        ach = flops / (t_block_ms * 1e-3) / 1e12
        detail.update({"fused_block_iterations": K0, "t_block_ms": t_block_ms, "t_block_min_ms": min(t_blk),
                       "block_flops_per_elt_iter": ALGO_FLOPS[w.cell],
                       "block_bytes_per_elt": ab["block"],
                       "block_gbs": ab["block"] * N / (t_block_ms * 1e-3) / 1e9,
                       # what one launch per iteration would have had to move for the same iterations
                       "block_equivalent_per_iteration_gbs": ab["iter"] * N * K0 / (t_block_ms * 1e-3) / 1e9})
        busy = MEASURED_VALU_BUSY_CYCLES.get(args.config)
        if busy:
            # share of the launch during which the vector ALUs were issuing (1024 SIMDs at 2.4 GHz)
            detail["block_valu_busy_frac"] = busy / (t_block_ms * 1e-3 * 1024 * 2.4e9)
        roofline = {"bound": "alu", "kernel": "newton_fused_kernel", "achieved": ach, "peak": VALU_F32_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": ach / VALU_F32_PEAK_TFLOPS, "traffic": MEASURED_TRAFFIC.get(args.config)}
    if w.cell != "tanh_dense":
        # the paper's operating mode: a fixed N_its = 3 and no stopping test (tol < 0), which the library
        # runs in one launch (u read once, h written once)
        ws_3 = torch.empty(P.workspace_bytes_fused(w.cell, u.dtype, w.B, w.L, w.H, 3), dtype=torch.uint8, device="cuda")
        fixed3 = lambda: P.forward(w.cell, params, u, h0, tol=-1.0, max_iter=3, workspace=ws_3, out=h_out)
        fixed3()
        t_f3 = time_events(fixed3, 10)
        detail["fixed_3_iterations_one_launch_ms"] = sum(t_f3) / len(t_f3)
        del ws_3
    if w.backward:
        ab = ALGO_BYTES[args.config]
        h, _, _ = P.forward(w.cell, params, u, h0, tol=w.tol, max_iter=w.max_iter, workspace=ws_f, out=h_out)
        t_bwd = time_events(lambda: P.backward(w.cell, params, u, h0, h, g, workspace=ws_b), 10)
        detail.update({"t_bwd_ms": sum(t_bwd) / len(t_bwd), "t_bwd_min_ms": min(t_bwd),
                       "bwd_bytes_per_elt": ab["bwd"],
                       "bwd_gbs": ab["bwd"] * N / (sum(t_bwd) / len(t_bwd) * 1e-3) / 1e9})
        detail["bwd_frac_hbm"] = detail["bwd_gbs"] / HBM_PEAK_GBS

    # not part of the timed step: the residual max-norm of the result (the paper's convergence
    # observable), one pass over u and h
    h, _, _ = P.forward(w.cell, params, u, h0, tol=w.tol, max_iter=w.max_iter, workspace=ws_f, out=h_out)
    rn_out = torch.empty(1, dtype=torch.float32, device="cuda")
    rn = lambda: P.residual_norm(w.cell, params, u, h0, h, out=rn_out)
    rn()
    t_rn = time_events(rn, 10)
    G_, S_ = u.shape[2], h.shape[2]
    detail["residual_norm"] = {"value": float(rn_out.cpu()), "ms": sum(t_rn) / len(t_rn),
                               "bytes_per_elt": (G_ + S_) * u.element_size(),
                               "gbs": (G_ + S_) * u.element_size() * N / (sum(t_rn) / len(t_rn) * 1e-3) / 1e9}

    if w.cell != "tanh_dense" and w.H % 256 == 0:
        # not part of the timed step: the input projection u = Bx + b in front of the solve and its
        # derivatives behind the backward pass, four heads (the paper's 400M .. 7B models), same shapes
        G = u.shape[2]
        heads = 4
        dh = w.H // heads
        xin = torch.randn((w.B, w.L, w.H), device="cuda").to(u.dtype)
        Wx = torch.randn((G, w.H, dh), device="cuda") / dh ** 0.5
        bx = torch.randn((G, w.H), device="cuda")
        ws_p = torch.empty(P.input_projection_workspace_bytes(u.dtype, w.B, w.L, w.H, G, heads, True),
                           dtype=torch.uint8, device="cuda")
        u_p = torch.empty_like(u)
        pf = lambda: P.input_projection(xin, Wx, bx, n_heads=heads, workspace=ws_p, out=u_p)
        pb = lambda: P.input_projection_backward(xin, Wx, u_p, n_heads=heads, workspace=ws_p)
        pf(); pb()
        t_pf, t_pb = time_events(pf, 5), time_events(pb, 5)
        t_pf, t_pb = sum(t_pf) / len(t_pf), sum(t_pb) / len(t_pb)
        es = u.element_size()
        flops = 2.0 * N * G * dh
        detail["input_projection"] = {
            "n_heads": heads, "arithmetic": "bf16 operands, fp32 accumulation",
            "fwd_ms": t_pf, "fwd_tflops": flops / (t_pf * 1e-3) / 1e12,
            "fwd_gbs": (N + N * G) * es / (t_pf * 1e-3) / 1e9,
            "bwd_ms": t_pb, "bwd_tflops": 2 * flops / (t_pb * 1e-3) / 1e12,
            "bwd_gbs": (2 * N + 2 * N * G) * es / (t_pb * 1e-3) / 1e9}
        del xin, u_p, ws_p
    note("per-kernel timings done")
    # a plain copy of known size, as the reference for hardware byte counters
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    t_copy = time_events(lambda: dst.copy_(src), 5)
    detail["copy_1GiB_gbs"] = 2 * src.numel() * 4 / (min(t_copy) * 1e-3) / 1e9
    del src, dst

    cpu = None
    if not args.no_cpu_baseline:
        note("timing the CPU oracle on its sample")
        cpu = cpu_baseline(w, d)

    out = {
        "metric": "Newton-solve timesteps*channels/s (fwd+bwd), % HBM roofline, 1 MI355X",
        "value": N / (ms_per_step * 1e-3), "unit": "timestep-channels/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.cell} {w.dtype} B={w.B} L={w.L} H={w.H} "
                               f"{'forward+backward' if w.backward else 'forward'}",
                   "tol": w.tol, "max_iter": w.max_iter},
        "roofline": roofline, "cpu_baseline": cpu, "detail": detail,
    }
    print(json.dumps(out))


def cpu_baseline(w, d):
    """The CPU oracle as it stands (fp64 Newton with forward substitution +
    adjoint recurrence), timed on the host cores on a bounded sample of the same
    workload: whole sequences, all of them when the work stays near 1e8
    timestep-channels, else the first sequences and, for the diagonal cells
    (whose channels are independent), the first channels."""
    import numpy as np
    import oracle
    oracle.build()
    threads = oracle.num_threads()
    budget = 1.0e8
    Bs, Hs = w.B, w.H
    if w.cell == "tanh_dense":
        Bs = int(max(1, min(w.B, budget // (w.L * w.H))))
    elif w.B * w.L * w.H > budget:
        Hs = int(max(1, min(w.H, budget // (w.B * w.L))))
    f64 = lambda t: None if t is None else t[:Bs, ..., :Hs].cpu().double().numpy()
    params = d["params"].cpu().double().numpy()
    if w.cell != "tanh_dense":
        params = np.ascontiguousarray(params[..., :Hs])
    u, h0 = f64(d["u"]), f64(d["h0"])
    t0 = time.perf_counter()
    h, it, st, _ = oracle.newton(w.cell, params, u, h0, tol=w.tol, max_iter=w.max_iter)
    t1 = time.perf_counter()
    tb = 0.0
    if w.backward:
        g = f64(d["g"])
        oracle.backward(w.cell, params, u, h0, h, g)
        tb = time.perf_counter() - t1
    n = Bs * w.L * Hs
    # the plain sequential application (Eq. (1)) of one sequence in fp32 on one core: the paper's
    # "naive sequential" reference point
    u1 = None if u is None else u[:1]
    h01 = None if h0 is None else h0[:1]
    t2 = time.perf_counter()
    oracle.seq_unroll(w.cell, params, u1, h01, precision="f32")
    t_seq = time.perf_counter() - t2
    extra = {"seq_unroll_f32_1core": w.L * Hs / t_seq}
    # the oracle spreads whole sequences over the OpenMP threads
    return {"value": n / ((t1 - t0) + tb), "unit": "timestep-channels/s", "cores": min(threads, Bs),
            "kind": "oracle", "sample": f"{Bs} of {w.B} sequences, {Hs} of {w.H} channels, full L, fp64, "
                                        f"{it} Newton iterations ({t1 - t0:.2f} s) + backward ({tb:.2f} s)", **extra}


if __name__ == "__main__":
    main()
