"""Hardware-counter figures for bench.py, from rocprofv3 passes over bench.py itself.

For every requested workload this runs, as separate passes of the same command
(`python3 bench.py --config X --profile-pass`: a few steps of the workload, each
kernel class of the solve on its own, and a plain device copy of known size):

    rocprofv3 --kernel-trace --stats        per-kernel durations
    rocprofv3 --pmc FETCH_SIZE              bytes fetched from HBM, per dispatch
    rocprofv3 --pmc WRITE_SIZE              bytes written to HBM, per dispatch
    rocprofv3 --pmc <issue counters>        vector-ALU / matrix-pipe busy cycles, instruction counts

and writes

    profiles/counters.json                  what bench.py prints as `traffic` and busy fractions, stamped
                                            with the library version and a hash of the kernel sources
                                            (bench.py prints null for a file made from other sources)
    profiles/<kernel>_<workload>.txt        the short summary of each workload's passes

The byte counters are calibrated on the copy in the same run: a copy of n bytes
fetches n and writes n, so the factor of each counter is n over what it read.
Raw rocprofv3 output goes to an untracked scratch folder (RAW_OUT below), with a second copy of the summaries
and of counters.json.  Run on the machine with the GPU, from the repository root:

    python3 bench_profile.py C5 C2 C3 C4
"""
import collections
import csv
import json
import os
import re
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
RAW_OUT = os.path.join(ROOT, "gpurun_out", "profile")     # raw profiler output and a second copy of the results: not tracked
sys.path.insert(0, ROOT)
import bench  # noqa: E402  (constants and the source hash; nothing here touches the GPU)

PROFILE_NAMES = {"C2": "newton_fused_gru_f32_C2", "C3": "newton_fused_lstm_f32_C3", "C4": "dense_scan_f32_C4",
                 "C5": "newton_fused_gru_bf16_C5", "X3": "newton_fused_paralstm_f32_X3"}
ISSUE_COUNTERS = {
    "diag": "SQ_INSTS_VALU SQ_INSTS_VALU_TRANS_F32 SQ_INSTS_SALU SQ_WAVES SQ_BUSY_CYCLES SQ_ACTIVE_INST_VALU "
            "SQ_VALU_MFMA_BUSY_CYCLES SQ_LDS_BANK_CONFLICT GRBM_GUI_ACTIVE",
    "dense": "SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES SQ_INSTS_VALU_MFMA_MOPS_F32 SQ_WAVES GRBM_GUI_ACTIVE",
}
PASS_TIMEOUT_S = 170


def short(name):
    name = name.replace("(anonymous namespace)::", "")
    name = re.sub(r"\(.*", "", name).replace("void ", "").replace("pararnn::", "")
    return name[:96]


def run_pass(cfg, tag, rocprof_args, outdir):
    """One rocprofv3 pass of bench.py's profile run; returns the path prefix of its CSV files."""
    d = os.path.join(outdir, tag)
    os.makedirs(d, exist_ok=True)
    cmd = ["rocprofv3", *rocprof_args, "--output-format", "csv", "-d", d, "-o", tag, "--",
           "python3", os.path.join(ROOT, "bench.py"), "--config", cfg, "--profile-pass"]
    env = dict(os.environ, TMPDIR="/tmp", PYTHONPATH=ROOT)
    print(f"[profile] {cfg} {tag}: {' '.join(cmd)}", flush=True)
    t0 = time.time()
    with open(os.path.join(d, "run.log"), "w") as log:
        r = subprocess.run(["timeout", "-s", "KILL", str(PASS_TIMEOUT_S), *cmd], cwd="/tmp", env=env, stdout=log,
                           stderr=subprocess.STDOUT)
    print(f"[profile] {cfg} {tag}: exit {r.returncode} after {time.time() - t0:.0f} s", flush=True)
    if r.returncode != 0:
        tail = open(os.path.join(d, "run.log")).read()[-1500:]
        raise SystemExit(f"pass {tag} of {cfg} failed (exit {r.returncode}); nothing further is run\n{tail}")
    return os.path.join(d, tag), " ".join(cmd[:cmd.index("--") + 1] + ["python3", "bench.py", "--config", cfg, "--profile-pass"])


def durations(prefix):
    by = collections.defaultdict(list)
    for r in csv.DictReader(open(prefix + "_kernel_trace.csv")):
        by[short(r["Kernel_Name"])].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    return by


def counter_rows(prefix):
    """{kernel: {counter: [(value, duration_us), ...]}}"""
    by = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(prefix + "_counter_collection.csv")):
        dur = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3
        by[short(r["Kernel_Name"])][r["Counter_Name"]].append((float(r["Counter_Value"]), dur))
    return by


def classes(kind):
    """Launch classes of a workload: name -> (kernel-name pattern, which dispatches of it)."""
    if kind == "dense":
        return {"dominant": (r"^dense_products_sweep_kernel<false", "work"),
                "residual": (r"^dense_residual_kernel", "work"),
                "carry": (r"^dense_carry_kernel", "work"),
                "final_sweep": (r"^dense_final_sweep_kernel<false", "work")}
    return {"dominant": (r"^newton_fused_kernel<", "longest"),          # first block of a solve
            "iter": (r"^newton_iter_kernel<.*false>$", "work"),        # one iteration per launch, from the iterate
            "bwd": (r"^backward_kernel<", "work"),
            # the input projection in front of the solve (four heads; not part of the timed step)
            "proj_fwd": (r"^proj_gemm_nt(_dma(_f32)?)?_kernel<.*true>", "work"),
            "proj_dx": (r"^proj_gemm_nt(_dma(_f32)?)?_kernel<.*false>", "work"),
            "proj_dw": (r"^proj_dw_(dma_)?kernel", "work")}


def pick(values, how):
    """values: [(x, duration_us)].  'longest': the class within 15 % of the longest dispatch; 'work': > 10 us."""
    if not values:
        return []
    dmax = max(d for _, d in values)
    if how == "longest":
        return [x for x, d in values if d >= 0.85 * dmax]
    return [x for x, d in values if d >= 10.0]


def mean(v):
    return sum(v) / len(v) if v else None


def profile_config(cfg, outdir):
    from workloads import ALL_CONFIGS
    w = ALL_CONFIGS[cfg]
    kind = "dense" if w.cell == "tanh_dense" else "diag"
    d = os.path.join(outdir, cfg)
    kt, cmd_kt = run_pass(cfg, "kt", ["--kernel-trace", "--stats"], d)
    fe, cmd_fe = run_pass(cfg, "fetch", ["--pmc", "FETCH_SIZE"], d)
    wr, cmd_wr = run_pass(cfg, "write", ["--pmc", "WRITE_SIZE"], d)
    ex, cmd_ex = run_pass(cfg, "issue", ["--pmc", *ISSUE_COUNTERS[kind].split()], d)
    meta = [json.loads(l) for l in open(os.path.join(d, "kt", "run.log")) if l.startswith("{")][-1]
    dur, fetch, write, issue = durations(kt), counter_rows(fe), counter_rows(wr), counter_rows(ex)

    # calibration: the device copy of known size (the largest copy kernel dispatches)
    def copy_reading(rows, counter):
        vals = [x for k, cs in rows.items() if "copyBuffer" in k for x, dd in cs[counter] if dd >= 20.0]
        top = max(vals)
        return mean([v for v in vals if v >= 0.9 * top]) * 1024.0
    n_copy = float(meta["copy_bytes_each_way"])
    f_fetch, f_write = n_copy / copy_reading(fetch, "FETCH_SIZE"), n_copy / copy_reading(write, "WRITE_SIZE")

    rec, lines = {}, []
    for cname, (pat, how) in classes(kind).items():
        names = [k for k in dur if re.search(pat, k)]
        if not names:
            continue
        # the shape that does the work: the one with the largest total time in the trace
        k = max(names, key=lambda n: sum(dur[n]))
        dsel = pick([(x, x) for x in dur[k]], how)
        fb = mean(pick(fetch[k]["FETCH_SIZE"], how))
        wb = mean(pick(write[k]["WRITE_SIZE"], how))
        r = {"kernel": k, "dispatches": len(dsel), "avg_us": mean(dsel), "min_us": min(dsel), "max_us": max(dsel),
             "fetch_bytes": fb * 1024.0 * f_fetch, "write_bytes": wb * 1024.0 * f_write}
        r["traffic_bytes"] = r["fetch_bytes"] + r["write_bytes"]
        for counter, vals in issue[k].items():
            v = mean(pick(vals, how))
            if v is not None:
                r[counter] = v
        if "SQ_ACTIVE_INST_VALU" in r:
            # the counter ticks once per 4 cycles of a busy vector ALU, summed over the SIMDs
            r["valu_busy_cycles"] = 4.0 * r["SQ_ACTIVE_INST_VALU"]
        rec[cname] = r
    # algorithmic bytes / flops beside the counters
    N = float(meta["N"])
    if kind == "diag":
        ab = bench.ALGO_BYTES[cfg]
        algo = {"dominant": ab["block"] * N, "iter": ab["iter"] * N, "bwd": ab["bwd"] * N}
        for c, a in algo.items():
            if c in rec:
                rec[c]["algorithmic_bytes"] = a
                rec[c]["traffic_over_algorithmic"] = rec[c]["traffic_bytes"] / a
        # projection: bytes of x and u (du, dx); flops of one product set
        from workloads import cell_dims
        G = cell_dims(w.cell)[0]
        es = 2.0 if w.dtype == "bf16" else 4.0
        pflops = 2.0 * N * G * (w.H // bench.PROJ_HEADS)
        for c in ("proj_fwd", "proj_dx", "proj_dw"):
            if c in rec:
                rec[c]["algorithmic_bytes"] = (N + N * G) * es
                rec[c]["traffic_over_algorithmic"] = rec[c]["traffic_bytes"] / rec[c]["algorithmic_bytes"]
                rec[c]["flops"] = pflops
                rec[c]["tflops"] = pflops / (rec[c]["avg_us"] * 1e-6) / 1e12
                if "SQ_VALU_MFMA_BUSY_CYCLES" in rec[c] and "GRBM_GUI_ACTIVE" in rec[c]:
                    rec[c]["mfma_busy_frac"] = rec[c]["SQ_VALU_MFMA_BUSY_CYCLES"] / 1024.0 / (rec[c]["GRBM_GUI_ACTIVE"] / 8.0)
        if "dominant" in rec and "SQ_INSTS_VALU" in rec["dominant"]:
            K0 = min(bench.FUSED_HEAD, w.max_iter)
            rec["dominant"]["valu_insts_per_elt_iter"] = rec["dominant"]["SQ_INSTS_VALU"] * 64.0 / (N * K0)
            rec["dominant"]["trans_insts_per_elt_iter"] = rec["dominant"]["SQ_INSTS_VALU_TRANS_F32"] * 64.0 / (N * K0)
    rec["calibration"] = {"copy_bytes_each_way": n_copy, "fetch_factor": f_fetch, "write_factor": f_write}

    # ---- the text summary
    lines.append(f"Workload: {bench.workload_string(w)} (N = {int(N)} timestep-channels)")
    lines.append(f"Library version {meta.get('version')}, kernel-source hash {bench.source_hash()}")
    lines.append("Commands (cwd /tmp, TMPDIR=/tmp, PYTHONPATH=<repository>; separate passes of the same command), "
                 "written by `python3 bench_profile.py " + cfg + "`:")
    for c in (cmd_kt, cmd_fe, cmd_wr, cmd_ex):
        lines.append("  " + c.replace(d + "/", "OUT/"))
    lines.append("")
    lines.append(f"Byte-counter calibration on the device copy of {int(n_copy)} bytes in the same run: "
                 f"bytes fetched = {f_fetch:.3f} x FETCH_SIZE KiB x 1024, bytes written = {f_write:.3f} x WRITE_SIZE KiB x 1024")
    lines.append("")
    lines.append("Launch classes (dominant = first fused block of a solve / chunk products; averages per launch):")
    for cname, r in rec.items():
        if cname == "calibration":
            continue
        lines.append(f"  {cname}: {r['kernel']}")
        lines.append(f"      {r['dispatches']} launches, avg {r['avg_us']:.1f} us (min {r['min_us']:.1f}, max {r['max_us']:.1f})")
        s = f"      HBM read {r['fetch_bytes'] / 1e6:.1f} MB + written {r['write_bytes'] / 1e6:.1f} MB = {r['traffic_bytes'] / 1e6:.1f} MB"
        if "algorithmic_bytes" in r:
            s += (f"; algorithmic {r['algorithmic_bytes'] / 1e6:.1f} MB (x{r['traffic_over_algorithmic']:.3f}); "
                  f"{r['algorithmic_bytes'] / r['avg_us'] / 1e3:.0f} GB/s algorithmic = "
                  f"{r['algorithmic_bytes'] / r['avg_us'] / 1e3 / bench.HBM_PEAK_GBS:.3f} of {bench.HBM_PEAK_GBS:.0f}")
        if "tflops" in r:
            s += f"; {r['tflops']:.0f} TFLOP/s = {r['tflops'] / 2500.0:.3f} of the 2500 dense bf16 peak"
        lines.append(s)
        extra = [f"{k} {v:.4g}" for k, v in r.items() if k.startswith(("SQ_", "GRBM_"))]
        if extra:
            lines.append("      " + ", ".join(extra))
        if "valu_busy_cycles" in r and "GRBM_GUI_ACTIVE" in r:
            # GRBM_GUI_ACTIVE is summed over the 8 XCDs; 1024 SIMDs
            busy = r["valu_busy_cycles"] / 1024.0 / (r["GRBM_GUI_ACTIVE"] / 8.0)
            lines.append(f"      vector ALUs busy {busy:.3f} of the launch's cycles")
        if "valu_insts_per_elt_iter" in r:
            lines.append(f"      {r['valu_insts_per_elt_iter']:.1f} vector instructions per timestep-channel and iteration, "
                         f"{r['trans_insts_per_elt_iter']:.1f} of them transcendental")
        if r.get("SQ_VALU_MFMA_BUSY_CYCLES", 0) > 0 and "GRBM_GUI_ACTIVE" in r:
            busy = r["SQ_VALU_MFMA_BUSY_CYCLES"] / 1024.0 / (r["GRBM_GUI_ACTIVE"] / 8.0)
            lines.append(f"      matrix pipes busy {busy:.3f} of the launch's cycles")
    lines.append("")
    lines.append("Kernel trace of the profile run (us): name | dispatches | avg | min | max")
    for k, v in sorted(dur.items(), key=lambda kv: -sum(kv[1])):
        if sum(v) < 50 or re.search(r"at::|elementwise|distribution", k):
            continue
        lines.append(f"  {k:96s} {len(v):5d} {mean(v):10.1f} {min(v):10.1f} {max(v):10.1f}")
    fname = PROFILE_NAMES.get(cfg, cfg) + ".txt"
    # beside the tracked copy, one in the scratch folder of the raw output
    for path in (os.path.join(ROOT, "profiles", fname), os.path.join(outdir, fname)):
        open(path, "w").write("\n".join(lines) + "\n")
        print(f"[profile] wrote {path}", flush=True)
    return rec


def main():
    cfgs = sys.argv[1:] or ["C5", "C2", "C3", "C4"]
    outdir = RAW_OUT
    import ctypes
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2510_21450_amd", "libpararnn.so"))
    path = bench.COUNTERS_JSON
    stamp = {"source_hash": bench.source_hash(), "pararnn_version": lib.pararnn_version()}
    out = {"configs": {}}
    try:
        old = json.load(open(path))
        if all(old.get(k) == v for k, v in stamp.items()):
            out = old                     # same build: keep the workloads that are not re-profiled now
    except (OSError, ValueError):
        pass
    out.update(stamp)
    out["written_by"] = "python3 bench_profile.py " + " ".join(cfgs)
    for cfg in cfgs:
        out["configs"][cfg] = profile_config(cfg, outdir)
        json.dump(out, open(path, "w"), indent=1, sort_keys=True)
        # a copy comes back from the GPU machine with the raw output
        json.dump(out, open(os.path.join(outdir, "counters.json"), "w"), indent=1, sort_keys=True)
    print(f"[profile] wrote {path}", flush=True)


if __name__ == "__main__":
    main()
