"""Benchmark of the hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: the
forward Newton solve (initial guess + Newton iterations until max|dh| <= tol)
and, for workloads that have one, the backward adjoint scan.  Inputs are
resident in HBM before the timed region.

Prints ONE JSON line.  The headline (`value`, `ms_per_step`, `roofline`) is the
largest single-GPU workload, config 5 (2^30 timestep-channels, bf16 storage,
fp32 arithmetic); `detail.configs` carries the other four configurations measured
in the same run (time per step, iterations, status, dominant kernel, roofline
fraction, algorithmic and counter bytes).  Kernel-level figures are measured live
with device events on the launch stream; hardware-counter figures (HBM traffic,
vector-ALU busy cycles) are read from profiles/counters.json, which
bench_profile.py writes from rocprofv3 passes over this file, and are printed as
null unless that file was made from the kernel sources this run uses.  The CPU
oracle is timed on the host cores on a bounded sample of the headline workload.

`--config X` makes X the headline; `--only` skips the other configurations.
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "Newton-solve timesteps*channels/s (fwd+bwd), % HBM roofline, 1 MI355X"
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_F32_PEAK_TFLOPS = 157.3   # MI355X dense fp32 matrix peak, published
# fp32 vector peak, published: 256 CUs x 4 SIMDs x 32 lanes x 2.4 GHz x 2 (FMA).  A SIMD issues a plain
# (not packed) wave-wide fp32 instruction every 2 cycles and a transcendental one (v_exp_f32, v_rcp_f32)
# every 8, measured with loops of independent instructions at full occupancy; packed forms are off.
VALU_F32_PEAK_TFLOPS = 157.3
VALU_CYCLES_PLAIN, VALU_CYCLES_TRANS = 2.0, 8.0
SIMDS, CLOCK_HZ = 1024, 2.4e9
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
COUNTERS_JSON = os.path.join(ROOT, "profiles", "counters.json")
KERNEL_SOURCES = [os.path.join(ROOT, "paper_2510_21450_amd", "csrc"), os.path.join(ROOT, "include", "pararnn")]


def note(msg):
    """Progress on stderr (stdout carries the one JSON line)."""
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def source_hash():
    """Hash of the kernel sources the library is built from: the stamp that ties a counter file to a build."""
    h = hashlib.sha256()
    for folder in KERNEL_SOURCES:
        for name in sorted(os.listdir(folder)):
            if name.endswith((".h", ".hip")):
                h.update(name.encode())
                h.update(open(os.path.join(folder, name), "rb").read())
    return h.hexdigest()[:16]


def load_counters(version):
    """profiles/counters.json when it was made from these kernel sources and this library version, else {}."""
    try:
        c = json.load(open(COUNTERS_JSON))
    except (OSError, ValueError):
        return {}, "profiles/counters.json is missing"
    if c.get("source_hash") != source_hash() or c.get("pararnn_version") != version:
        return {}, "profiles/counters.json was made from other kernel sources: counter figures are null"
    return c.get("configs", {}), None


def time_events(fn, reps):
    import torch
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in evs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return [a.elapsed_time(b) for a, b in evs]


def mean(v):
    return sum(v) / len(v)


def workload_string(w):
    store = "bf16 storage / fp32 arithmetic" if w.dtype == "bf16" else "fp32"
    return (f"{w.name}: {w.cell} {store} B={w.B} L={w.L} H={w.H} "
            f"{'forward+backward' if w.backward else 'forward'}")


class Run:
    """One workload resident on the GPU, with the step the benchmark times."""

    def __init__(self, P, torch, name):
        from workloads import ALL_CONFIGS, make_inputs, cell_dims
        self.P, self.torch, self.name = P, torch, name
        self.w = w = ALL_CONFIGS[name]
        self.G, self.S = cell_dims(w.cell)
        self.d = d = make_inputs(w, device="cuda")
        self.params, self.u, self.h0, self.g = d["params"], d["u"], d["h0"], d.get("g")
        self.N = w.B * w.L * w.H
        dt = self.u.dtype
        self.ws_f = torch.empty(P.workspace_bytes(w.cell, dt, w.B, w.L, w.H, False), dtype=torch.uint8, device="cuda")
        self.ws_b = torch.empty(max(256, P.workspace_bytes(w.cell, dt, w.B, w.L, w.H, True)), dtype=torch.uint8,
                                device="cuda")
        self.h_out = torch.empty((w.B, w.L, self.S, w.H), dtype=dt, device="cuda")
        self.bwd_out = None
        if w.backward:
            self.bwd_out = (torch.empty_like(self.u), torch.empty_like(self.params),
                            torch.empty((w.B, self.S, w.H), dtype=dt, device="cuda"))
        self.iters = None

    def forward(self, tol=None, max_iter=None):
        w = self.w
        h, iters, _ = self.P.forward(w.cell, self.params, self.u, self.h0, tol=w.tol if tol is None else tol,
                                     max_iter=w.max_iter if max_iter is None else max_iter, workspace=self.ws_f,
                                     out=self.h_out)
        return h, iters

    def backward(self, h):
        w = self.w
        return self.P.backward(w.cell, self.params, self.u, self.h0, h, self.g, workspace=self.ws_b, out=self.bwd_out)

    def step(self):
        h, self.iters = self.forward()
        if self.w.backward:
            self.backward(h)

    def timed_steps(self, steps, warmup):
        torch = self.torch
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps


PROJ_HEADS = 4


def projection_applies(w):
    return w.cell != "tanh_dense" and w.H % (64 * PROJ_HEADS) == 0


def projection_calls(run):
    """Forward and backward of the input projection on the workload's shapes (four heads); the tensors
    stay alive with the returned closures."""
    P, torch, w = run.P, run.torch, run.w
    u = run.d["u"]
    G, heads = run.G, PROJ_HEADS
    dh = w.H // heads
    xin = torch.randn((w.B, w.L, w.H), device="cuda").to(u.dtype)
    Wx = torch.randn((G, w.H, dh), device="cuda") / dh ** 0.5
    bx = torch.randn((G, w.H), device="cuda")
    ws_p = torch.empty(P.input_projection_workspace_bytes(u.dtype, w.B, w.L, w.H, G, heads, True),
                       dtype=torch.uint8, device="cuda")
    u_p = torch.empty_like(u)
    pf = lambda: P.input_projection(xin, Wx, bx, n_heads=heads, workspace=ws_p, out=u_p)
    pb = lambda: P.input_projection_backward(xin, Wx, u_p, n_heads=heads, workspace=ws_p)
    return pf, pb, dh


def kernel_figures(run, reps, counters):
    """Per-kernel timings of one workload (device events on the launch stream) and its roofline record."""
    P, torch, w, N = run.P, run.torch, run.w, run.N
    cnt = counters.get(run.name, {})
    out = {}
    if w.cell == "tanh_dense":
        # one launch sequence per iteration: time per Newton iteration from fixed-count solves
        m_lo, m_hi = 2, 10
        for m in (m_lo, m_hi):
            run.forward(tol=-1.0, max_iter=m)
        t_lo = time_events(lambda: run.forward(tol=-1.0, max_iter=m_lo), reps)
        t_hi = time_events(lambda: run.forward(tol=-1.0, max_iter=m_hi), reps)
        t_iter_ms = (mean(t_hi) - mean(t_lo)) / (m_hi - m_lo)
        # the scan composes one 64x64 Jacobian product (2 H^3 flop) per timestep
        flops_iter = 2.0 * w.H ** 3 * w.B * w.L
        chunk = P.dense_chunk()
        n_c = (w.L + chunk - 1) // chunk
        flops_kernel = 2.0 * w.H ** 3 * w.B * max(0, n_c - 2) * (chunk - 1)
        out.update({"t_iter_ms": t_iter_ms, "iter_tflops": flops_iter / (t_iter_ms * 1e-3) / 1e12})
        out["iter_frac_mfma"] = out["iter_tflops"] / MFMA_F32_PEAK_TFLOPS
        # the composition kernel alone, same launch as inside the solve, on Jacobian factors of the same
        # distribution (d = 1 - tanh^2 of the converged states)
        run.forward()
        dfac = (1.0 - run.h_out.view(w.B, w.L, w.H) ** 2).contiguous()
        Aout = torch.zeros((w.B, n_c, w.H, w.H), dtype=torch.float32, device="cuda")
        P.dense_chunk_products(run.params, dfac, out=Aout)
        t_k = mean(time_events(lambda: P.dense_chunk_products(run.params, dfac, out=Aout), 2 * reps))
        ach = flops_kernel / (t_k * 1e-3) / 1e12
        out["chunk_products_ms"] = t_k
        out["algorithmic_flops_per_launch"] = flops_kernel
        out["roofline"] = {"bound": "mfma", "kernel": "dense_products_sweep_kernel (chunk products part)",
                           "achieved": ach, "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                           "frac": ach / MFMA_F32_PEAK_TFLOPS, "traffic": cnt.get("dominant", {}).get("traffic_bytes")}
        run.extra = (dfac, Aout)
        return out
    ab = ALGO_BYTES[run.name]
    # one launch per iteration (the path without fused blocks): time per Newton iteration
    P.set_fused(False)
    try:
        m_lo, m_hi = 2, 10
        for m in (m_lo, m_hi):
            run.forward(tol=-1.0, max_iter=m)
        t_lo = time_events(lambda: run.forward(tol=-1.0, max_iter=m_lo), reps)
        t_hi = time_events(lambda: run.forward(tol=-1.0, max_iter=m_hi), reps)
    finally:
        P.set_fused(True)
    t_iter_ms = (mean(t_hi) - mean(t_lo)) / (m_hi - m_lo)
    iter_gbs = ab["iter"] * N / (t_iter_ms * 1e-3) / 1e9
    out.update({"t_iter_ms": t_iter_ms, "t_iter_min_ms": (min(t_hi) - min(t_lo)) / (m_hi - m_lo),
                "iter_bytes_per_elt": ab["iter"], "iter_gbs": iter_gbs, "iter_frac_hbm": iter_gbs / HBM_PEAK_GBS,
                "iter_traffic_bytes": cnt.get("iter", {}).get("traffic_bytes")})
    # The dominant launch of a solve: its first fused block of FUSED_HEAD iterations from the initial
    # guess (u read once, the iterate in registers, h written once).  Timed as the library runs it
    # inside a solve: a tolerance that is met at once ends the solve after this launch, which still
    # performs all its iterations; the call also holds the reset of the control block and one
    # launch that returns at once.
    K0 = min(FUSED_HEAD, w.max_iter)
    block = lambda: run.forward(tol=3.0e38, max_iter=K0 + 1)
    block()
    t_blk = time_events(block, reps)
    t_block_ms = mean(t_blk)
    flops = ALGO_FLOPS[w.cell] * float(N) * K0
    ach = flops / (t_block_ms * 1e-3) / 1e12
    out.update({"fused_block_iterations": K0, "t_block_ms": t_block_ms, "t_block_min_ms": min(t_blk),
                "block_flops_per_elt_iter": ALGO_FLOPS[w.cell], "block_bytes_per_elt": ab["block"],
                "block_gbs": ab["block"] * N / (t_block_ms * 1e-3) / 1e9,
                # what one launch per iteration would have had to move for the same iterations
                "block_equivalent_per_iteration_gbs": ab["iter"] * N * K0 / (t_block_ms * 1e-3) / 1e9})
    busy = cnt.get("dominant", {}).get("valu_busy_cycles")
    # share of the launch during which the vector ALUs were issuing (1024 SIMDs at 2.4 GHz)
    out["block_valu_busy_frac"] = busy / (t_block_ms * 1e-3 * 1024 * 2.4e9) if busy else None
    # the launch's own instruction mix at the issue rates above: the time the vector ALUs need for the
    # instructions the kernel executes (counted by the profiler), at the nominal clock
    dom = cnt.get("dominant", {})
    if dom.get("valu_insts_per_elt_iter") and dom.get("trans_insts_per_elt_iter") is not None:
        vi, ti = dom["valu_insts_per_elt_iter"], dom["trans_insts_per_elt_iter"]
        cyc = float(N) * K0 / 64.0 * ((vi - ti) * VALU_CYCLES_PLAIN + ti * VALU_CYCLES_TRANS)
        t_issue_ms = cyc / (SIMDS * CLOCK_HZ) * 1e3
        out["block_issue_bound_ms"] = t_issue_ms
        out["block_issue_bound_frac"] = t_issue_ms / t_block_ms
    else:
        out["block_issue_bound_ms"] = out["block_issue_bound_frac"] = None
    out["roofline"] = {"bound": "alu", "kernel": "newton_fused_kernel (first block of a solve)", "achieved": ach,
                       "peak": VALU_F32_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": ach / VALU_F32_PEAK_TFLOPS,
                       "traffic": cnt.get("dominant", {}).get("traffic_bytes")}
    out["algorithmic_bytes_per_launch"] = ab["block"] * N
    if w.backward:
        h, _ = run.forward()
        run.backward(h)
        t_bwd = time_events(lambda: run.backward(h), reps)
        gbs = ab["bwd"] * N / (mean(t_bwd) * 1e-3) / 1e9
        out.update({"t_bwd_ms": mean(t_bwd), "t_bwd_min_ms": min(t_bwd), "bwd_bytes_per_elt": ab["bwd"],
                    "bwd_gbs": gbs, "bwd_frac_hbm": gbs / HBM_PEAK_GBS,
                    "bwd_traffic_bytes": cnt.get("bwd", {}).get("traffic_bytes")})
    return out


def measure(P, torch, name, steps, warmup, reps, counters, headline):
    """ms per step, iterations, status and kernel figures of one workload."""
    run = Run(P, torch, name)
    w = run.w
    note(f"inputs ready: {workload_string(w)}")
    ms = run.timed_steps(steps, warmup)
    iters, status = (int(x) for x in run.iters.cpu())
    note(f"{name}: {steps} timed steps: {ms:.4f} ms per step, iters={iters} status={P.status_string(status)}")
    rec = {"workload": workload_string(w), "tol": w.tol, "max_iter": w.max_iter, "steps": steps, "warmup": warmup,
           "ms_per_step": ms, "value": run.N / (ms * 1e-3), "iters": iters, "status": P.status_string(status)}
    t_steps = sorted(time_events(run.step, max(steps, 20) if headline else min(steps, 20)))
    rec.update({"ms_per_step_min": t_steps[0], "ms_per_step_median": t_steps[len(t_steps) // 2]})
    t_fwd = time_events(lambda: run.forward(), reps)
    rec.update({"t_fwd_ms": mean(t_fwd), "t_fwd_min_ms": min(t_fwd)})
    if w.B * w.L * w.H < 1 << 16:
        # launch-latency bound: no roofline is claimed for it
        rec["roofline"] = None
        rec["dominant_kernel"] = "newton_fused_kernel (launch latency: no roofline claimed)"
    else:
        rec.update(kernel_figures(run, reps, counters))
        rec["dominant_kernel"] = rec["roofline"]["kernel"]
    return run, rec


def headline_extras(run, rec, reps, counters):
    """Figures beside the timed step, for the headline workload only."""
    P, torch, w, N = run.P, run.torch, run.w, run.N
    u, params, h0 = run.u, run.params, run.h0
    # blocks of Newton iterations of the plan; the first two are launches of their own, the rest share one
    rec["blocks"] = P.solve_plan(w.tol, w.max_iter) if w.cell != "tanh_dense" else None
    rec["launches_per_solve"] = min(len(rec["blocks"]), 3) if rec["blocks"] is not None else None
    if w.cell != "tanh_dense":
        # the same step under pararnn_set_workspace_reuse (the caller's promise that nothing else writes to the
        # two workspaces between calls: true for this loop): the carry records are not cleared again
        try:
            P.set_workspace_reuse(True)
            ms = run.timed_steps(20, 3)
        finally:
            P.set_workspace_reuse(False)
        rec["workspace_reuse"] = {"ms_per_step": ms, "value": N / (ms * 1e-3),
                                  "note": "opt-in mode, not the headline: pararnn_set_workspace_reuse(1)"}
    if w.cell == "tanh_dense":
        dfac, Aout = run.extra
        # not part of the step (config 4 is forward only): the adjoint scan of the same cell
        gd = torch.randn_like(run.h_out)
        ws_db = torch.empty(P.workspace_bytes(w.cell, u.dtype, w.B, w.L, w.H, True), dtype=torch.uint8, device="cuda")
        dense_bwd = lambda: P.backward(w.cell, params, u, h0, run.h_out, gd, workspace=ws_db)
        dense_bwd()
        rec["dense_backward_ms"] = mean(time_events(dense_bwd, reps))
        # inexact Newton (opt-in, not the timed step): Jacobian products from bf16 terms, fp32 residual
        inexact = {}
        for mode, name in ((1, "bf16x3"), (2, "bf16")):
            P.set_dense_products(mode)
            try:
                _, it_m = run.forward()
                t_m = time_events(lambda: run.forward(), reps)
                t_km = time_events(lambda: P.dense_chunk_products(params, dfac, out=Aout), reps)
                it_m = [int(x) for x in it_m.cpu()]
                inexact[name] = {"t_fwd_ms": mean(t_m), "iters": it_m[0], "status": P.status_string(it_m[1]),
                                 "chunk_products_ms": mean(t_km)}
            finally:
                P.set_dense_products(0)
        rec["inexact_products"] = inexact
        # not part of the timed step: the quasi-Newton ablation (the Jacobian replaced by its diagonal,
        # a diagonal scan instead of the matrix products; linear convergence, more iterations)
        P.set_dense_jacobian(1)
        try:
            _, it_q = run.forward()
            t_q = time_events(lambda: run.forward(), reps)
            it_q = [int(x) for x in it_q.cpu()]
            rec["quasi_newton_diagonal"] = {"t_fwd_ms": mean(t_q), "iters": it_q[0], "status": P.status_string(it_q[1])}
        finally:
            P.set_dense_jacobian(0)
        run.forward()
    else:
        # the paper's operating mode: a fixed N_its = 3 and no stopping test (tol < 0), which the library
        # runs in one launch (u read once, h written once)
        ws_3 = torch.empty(P.workspace_bytes_fused(w.cell, u.dtype, w.B, w.L, w.H, 3), dtype=torch.uint8, device="cuda")
        fixed3 = lambda: P.forward(w.cell, params, u, h0, tol=-1.0, max_iter=3, workspace=ws_3, out=run.h_out)
        fixed3()
        rec["fixed_3_iterations_one_launch_ms"] = mean(time_events(fixed3, reps))
        del ws_3
    # not part of the timed step: the residual max-norm of the result (the paper's convergence
    # observable), one pass over u and h
    h, _ = run.forward()
    rn_out = torch.empty(1, dtype=torch.float32, device="cuda")
    rn = lambda: P.residual_norm(w.cell, params, u, h0, h, out=rn_out)
    rn()
    t_rn = mean(time_events(rn, reps))
    bpe = (run.G + run.S) * u.element_size()
    rec["residual_norm"] = {"value": float(rn_out.cpu()), "ms": t_rn, "bytes_per_elt": bpe,
                            "gbs": bpe * N / (t_rn * 1e-3) / 1e9}
    if projection_applies(w):
        # not part of the timed step: the input projection u = Bx + b in front of the solve and its
        # derivatives behind the backward pass, four heads (the paper's 400M .. 7B models), same shapes
        pf, pb, dh = projection_calls(run)
        pf(); pb()
        t_pf, t_pb = mean(time_events(pf, 5)), mean(time_events(pb, 5))
        es = u.element_size()
        G = run.G
        flops = 2.0 * N * G * dh
        pr = {"n_heads": PROJ_HEADS, "arithmetic": "bf16 operands, fp32 accumulation",
              "fwd_ms": t_pf, "fwd_tflops": flops / (t_pf * 1e-3) / 1e12,
              "fwd_gbs": (N + N * G) * es / (t_pf * 1e-3) / 1e9,
              "bwd_ms": t_pb, "bwd_tflops": 2 * flops / (t_pb * 1e-3) / 1e12,
              "bwd_gbs": (2 * N + 2 * N * G) * es / (t_pb * 1e-3) / 1e9}
        # per kernel, from the committed counter passes (null when they were made from other sources)
        cnt = counters.get(run.name, {})
        for cname in ("proj_fwd", "proj_dx", "proj_dw"):
            c = cnt.get(cname)
            pr[cname] = None if not c else {
                "kernel": c["kernel"], "avg_us": c["avg_us"], "traffic_bytes": c["traffic_bytes"],
                "algorithmic_bytes": c.get("algorithmic_bytes"), "tflops": c.get("tflops"),
                "mfma_busy_frac": c.get("mfma_busy_frac")}
        rec["input_projection"] = pr


def profile_pass(P, torch, name):
    """What bench_profile.py runs under rocprofv3: a few steps of one workload, each kernel class of the
    solve on its own, and a plain copy of known size (the reference for the hardware byte counters)."""
    run = Run(P, torch, name)
    w = run.w
    for _ in range(3):
        run.step()
    if w.cell == "tanh_dense":
        kernel_figures(run, 3, {})
    else:
        K0 = min(FUSED_HEAD, w.max_iter)
        for _ in range(3):
            run.forward(tol=3.0e38, max_iter=K0 + 1)
        P.set_fused(False)
        for _ in range(3):
            run.forward(tol=-1.0, max_iter=3)
        P.set_fused(True)
        if projection_applies(w):
            pf, pb, _ = projection_calls(run)
            for _ in range(3):
                pf()
                pb()
    src = torch.empty(1 << 26, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)          # 256 MiB read, 256 MiB written
    torch.cuda.synchronize()
    print(json.dumps({"profile_pass": name, "copy_bytes_each_way": src.numel() * 4, "N": run.N, "version": P.version()}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="C5", choices=["C1", "C2", "C3", "C4", "C5", "X3"],
                    help="the headline workload (default: the largest single-GPU configuration)")
    ap.add_argument("--only", action="store_true", help="measure the headline workload only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-pass", action="store_true", help="short run of --config for rocprofv3 (bench_profile.py)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no sharding or collectives are part of it); "
                 "run with --gpus 1")

    import torch
    import paper_2510_21450_amd as P

    torch.cuda.set_device(0)
    P.set_fused_head(FUSED_HEAD)
    if args.profile_pass:
        profile_pass(P, torch, args.config)
        return
    counters, why = load_counters(P.version())
    if why:
        note(why)

    run, rec = measure(P, torch, args.config, args.steps, args.warmup, 10, counters, True)
    headline_extras(run, rec, 10, counters)
    note("headline workload done")
    # what the runtime reports for this device, beside the published figures the rooflines use
    props = torch.cuda.get_device_properties(0)
    dev = {"name": props.name, "arch": getattr(props, "gcnArchName", None), "memory_gib": props.total_memory / 2 ** 30}
    dev.update(P.device_info())
    # a plain copy of known size, as the reference for hardware byte counters
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    t_copy = time_events(lambda: dst.copy_(src), 5)
    copy_gbs = 2 * src.numel() * 4 / (min(t_copy) * 1e-3) / 1e9
    del src, dst

    cpu = None
    if not args.no_cpu_baseline:
        note("timing the CPU oracle on its sample")
        cpu = cpu_baseline(run.w, run.d)
    w = run.w
    del run
    torch.cuda.empty_cache()

    others = {}
    if not args.only:
        for name in ("C1", "C2", "C3", "C4", "C5"):
            if name == args.config:
                continue
            r, other = measure(P, torch, name, min(args.steps, 50), min(args.warmup, 10), 5, counters, False)
            others[name] = other
            del r
            torch.cuda.empty_cache()

    roofline = rec.pop("roofline")
    detail = {k: v for k, v in rec.items() if k not in ("workload", "tol", "max_iter", "steps", "warmup", "ms_per_step",
                                                        "value")}
    detail["device"] = dev
    detail["copy_1GiB_gbs"] = copy_gbs
    detail["counters"] = {"file": "profiles/counters.json", "source_hash": source_hash(), "usable": why is None}
    detail["configs"] = others
    out = {
        "metric": METRIC, "value": rec["value"], "unit": "timestep-channels/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": rec["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": workload_string(w), "tol": w.tol, "max_iter": w.max_iter},
        "roofline": roofline, "cpu_baseline": cpu, "detail": detail,
    }
    print(json.dumps(out))


def cpu_baseline(w, d):
    """The CPU oracle as it stands, timed on the host cores on a bounded sample of the same workload.

    The oracle itself runs the sequences of a batch on OpenMP threads; the workloads have fewer
    sequences than the host has cores, so the sample is cut into single-sequence pieces that are
    handed to a pool of as many threads as the oracle's OpenMP would use (the machine's CPU share):
    whole sequences, and for the diagonal cells, whose channels are independent recurrences, blocks
    of channels.  Every piece is one oracle call (fp64 Newton with forward substitution to the
    workload's tolerance, then the adjoint recurrence); `value` is the sample's timestep-channels over
    the wall time of the pool.  Beside it: the plain sequential application (Eq. (1)) in fp32, on one
    core (the paper's "naive sequential" point of comparison) and on all cores."""
    import concurrent.futures as cf
    import numpy as np
    import oracle
    oracle.build()
    threads = oracle.num_threads()
    budget = 1.0e8                               # timestep-channels in the sample
    dense = w.cell == "tanh_dense"
    if dense:
        Bs = int(max(1, min(w.B, budget // (w.L * w.H))))
        pieces = [(b, 0, w.H) for b in range(Bs)]
    else:
        # channel blocks of 64 (one cache line of fp64 per row and gate would be 8; 64 keeps calls long)
        per_seq = max(1, int(budget // w.L))     # channels in the sample, over all its sequences
        Bs = min(w.B, max(1, threads))
        Hc = 64 if w.H >= 64 else w.H
        blocks = max(1, min(w.H // Hc, per_seq // (Hc * Bs)))
        # a multiple of the thread count, so that the pool ends together
        n_pieces = max(1, (Bs * blocks) // threads) * threads if Bs * blocks >= threads else Bs * blocks
        pieces = [(i % Bs, (i // Bs) * Hc, Hc) for i in range(n_pieces)]
    used = min(threads, len(pieces))

    def inputs(piece, dtype):
        b, c0, hc = piece
        cut = lambda t: None if t is None else np.ascontiguousarray(t[b:b + 1, ..., c0:c0 + hc].cpu().to(dtype).numpy())
        params = d["params"].cpu().to(dtype).numpy()
        if not dense:
            params = np.ascontiguousarray(params[..., c0:c0 + hc])
        return params, cut(d["u"]), cut(d["h0"]), cut(d.get("g"))

    import ctypes
    import torch
    gomp = ctypes.CDLL("libgomp.so.1")
    data64 = [inputs(p, torch.float64) for p in pieces]

    def solve(x):
        params, u, h0, g = x
        gomp.omp_set_num_threads(1)              # per calling thread: one piece, one thread
        t0 = time.perf_counter()
        h, it, st, _ = oracle.newton(w.cell, params, u, h0, tol=w.tol, max_iter=w.max_iter)
        t1 = time.perf_counter()
        if w.backward:
            oracle.backward(w.cell, params, u, h0, h, g)
        return it, t1 - t0, time.perf_counter() - t1

    with cf.ThreadPoolExecutor(max_workers=used) as ex:
        t0 = time.perf_counter()
        res = list(ex.map(solve, data64))
        t_oracle = time.perf_counter() - t0
    n = sum(p[2] for p in pieces) * w.L
    its = [r[0] for r in res]
    del data64
    data32 = [inputs(p, torch.float32)[:3] for p in pieces]
    def unroll(x):
        gomp.omp_set_num_threads(1)
        return oracle.seq_unroll(w.cell, x[0], x[1], x[2], precision="f32")

    t0 = time.perf_counter()
    unroll(data32[0])
    t_seq1 = time.perf_counter() - t0
    with cf.ThreadPoolExecutor(max_workers=used) as ex:
        t0 = time.perf_counter()
        list(ex.map(unroll, data32))
        t_seq = time.perf_counter() - t0
    return {"value": n / t_oracle, "unit": "timestep-channels/s", "cores": used, "kind": "oracle",
            "nproc": os.cpu_count(), "omp_max_threads": threads,
            "sample": f"{len(pieces)} pieces of one sequence x {pieces[0][2]} channels x full L "
                      f"({n} of {w.B * w.L * w.H} timestep-channels), fp64, each solved to the workload's tolerance "
                      f"({min(its)}-{max(its)} Newton iterations) + backward: {t_oracle:.2f} s on {used} threads "
                      f"(forward {sum(r[1] for r in res):.1f} + backward {sum(r[2] for r in res):.1f} thread-seconds)",
            "seq_unroll_f32_1core": pieces[0][2] * w.L / t_seq1,
            "seq_unroll_f32_allcores": n / t_seq, "seq_unroll_threads": used}


if __name__ == "__main__":
    main()
