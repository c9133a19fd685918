#!/usr/bin/env python3
"""Benchmark of the Soft-DTW hot path on one MI355X.

One "step" is one pass of the whole hot path over one synthetic batch that is already resident in
device memory: row norms and split operand copies, the forward sweep, the reverse sweep with the
alignment matrix, the input gradients.  The headline workload is the largest single-GPU
configuration at B = 32: N = M = 8192, D = 128, gamma = 0.01, fused mode (the only mode that
configuration lists).  The value is DP cells per second for forward+backward, cells = B*N*M.

The same JSON line carries, under `other_workloads`, the B = 32 configurations with N = M = 256 and
1024 (both modes each) and the barycenter configuration, every one with its own timings, peak
bytes, `roofline` and `cpu_baseline`; `--headline-only` leaves them out, and with them the two extra legs
of the headline shape (its unfused mode, for the memory comparison, and float16 inputs): a profiling run
then sees the kernels of the configuration's own step alone.

`roofline` describes the kernel that took the most time in the step, timed with HIP events on the
launch stream (per-kernel events are recorded in a second, identical loop so that they do not
perturb the headline timing); `cpu_baseline` is the float64 CPU oracle timed on this host.

Other legs (each prints one JSON line and exits):
  --calibrate-copy   a plain device copy of known size, the reference for the rocprofv3 HBM counters
  --calibrate-valu   the vector-ALU rates and the bare DP step (sdtw_debug_rate_probe)
  --ingest-pmc DIR   no GPU: turns the counter CSVs of four rocprofv3 --pmc runs under DIR
                     (cal_fetch, cal_write, fetch, write) into profiles/hbm_traffic.json / .md
"""
import argparse
import csv
import glob
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# Published MI355X peaks used for the roofline fractions.
PEAK_HBM_GBS = 8000.0
PEAK_MFMA_F32_TFLOPS = 157.3
PEAK_MFMA_F16_TFLOPS = 2500.0  # dense; the cost and gradient contractions run there for D <= 128 (split operands)
# Vector-ALU ceiling of the DP recurrence, in float64-rate lane operations: 256 CUs x 4 SIMDs x 16
# lanes x 2.4 GHz = 39.3e12/s (the published 78.6 TFLOP/s float64 vector peak counts an FMA as two).
# At the published rates a float64 add/min/max/fma/convert costs 1 such slot per lane, a float32
# add 0.5, a lane-shift move 1, an exp2/log2 (quarter of the float32 rate) 2.
PEAK_VALU_TOPS = 256 * 64 * 2.4e9 / 1e12

# Work per DP cell and sweep in those slots, from the instruction mix of the recurrence (Sec. 2
# Eq. 1-2 with the max-shift of Sec. 4.2): 11 float64 operations (3 min/max, 3 subtractions, 1 fma,
# 4 conversions), 2 lane-shift moves, 2 float32 additions, 3 transcendentals = 11 + 2 + 1 + 6 = 20
# (the micro-benchmark of the bare step measures 82 cycles per 64 cells per SIMD = 20.5).
# The reverse sweep that also forms E adds one exp2, one float64 subtraction, one conversion and one
# float32 addition: 24.5.  (Recomputing R in the backward of large problems is this library's
# choice, not algorithmic work: it is not counted.)
SLOTS_SWEEP_CELL = 20.0
SLOTS_BWD_E_CELL = 24.5
MODE_NAMES = {0: "unfused", 1: "fused"}
HEADLINE = "c4_b32_l8192"
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "hbm_traffic.json")
TRAFFIC_MD = os.path.join(ROOT, "profiles", "hbm_traffic.md")


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--modes", default="", help="comma list of unfused,fused (default: the workload's modes)")
    ap.add_argument("--headline-only", action="store_true", help="leave out the other configurations")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true")
    ap.add_argument("--calibrate-valu", action="store_true")
    ap.add_argument("--ingest-pmc", default="", metavar="DIR")
    ap.add_argument("--pmc-workload", default="", help="with --ingest-pmc: the workload the runs under DIR measured")
    return ap.parse_args()


# ------------------------------------------------------------------------------------------------
# rooflines
# ------------------------------------------------------------------------------------------------
def contraction_name(D):
    return "f16x3-split (float32 operands as two float16 halves, 3 fp16 MFMA products, float32 accumulate)" \
        if D <= 128 else "f32 MFMA"


def kernel_table(prof, steps):
    """[(label, ms)] of many steps -> {label: launches per step, mean ms per launch, ms per step}."""
    agg = {}
    for name, ms in prof:
        c, t = agg.get(name, (0, 0.0))
        agg[name] = (c + 1, t + ms)
    return {k: {"launches_per_step": c / steps, "ms_per_launch": t / c, "ms_per_step": t / steps} for k, (c, t) in agg.items()}


def roofline_for(name, ms_per_launch, wl_cells, D, traffic=None):
    """Roofline object for one kernel launch covering wl_cells DP cells."""
    sec = ms_per_launch * 1e-3
    if name.startswith("forward_dp") or name.startswith("backward_dp") or name.startswith("both_sweeps"):
        both = name.startswith("both_sweeps")
        slots = 2 * SLOTS_SWEEP_CELL if both else (SLOTS_SWEEP_CELL if name.startswith("forward") else SLOTS_BWD_E_CELL)
        achieved = slots * wl_cells / sec / 1e12
        out = {"kernel": name, "bound": "alu", "achieved": achieved, "peak": PEAK_VALU_TOPS,
               "unit": "Tlane-op/s", "frac": achieved / PEAK_VALU_TOPS, "traffic": traffic,
               "ms_per_launch": ms_per_launch, "per_cell": {"valu_slots": slots}}
        if name.endswith("_fused"):
            fl = (2 if both else 1) * 2.0 * D * wl_cells / sec / 1e12
            pk = PEAK_MFMA_F16_TFLOPS if D <= 128 else PEAK_MFMA_F32_TFLOPS
            out["mfma"] = {"achieved": fl, "peak": pk, "unit": "TFLOP/s", "frac": fl / pk, "dtype": contraction_name(D)}
        # table traffic: 8 B per cell and sweep where the table is stored (small problems); unfused reads the cost
        nbytes = (16.0 if both else 0.5) + ((8.0 if both else 4.0) if name.endswith("_unfused") else 0.0)
        bw = nbytes * wl_cells / sec / 1e9
        out["hbm"] = {"achieved": bw, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": bw / PEAK_HBM_GBS, "bytes_per_cell": nbytes}
        return out
    per_cell = {"cost_tensor": 4.0,    # the stored tensor
                "alignment": 20.0,     # reads both float64 tables, writes float32 E
                "input_grad": 8.0}     # E is read once per side
    if name in per_cell:
        bw = per_cell[name] * wl_cells / sec / 1e9
        return {"kernel": name, "bound": "hbm", "achieved": bw, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": bw / PEAK_HBM_GBS, "traffic": traffic, "ms_per_launch": ms_per_launch}
    return {"kernel": name, "bound": "hbm", "achieved": None, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": None,
            "traffic": traffic, "ms_per_launch": ms_per_launch}


def kernel_source_hash():
    """Hash of the sources the library is built from: ties counter figures to the kernels they measured."""
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(ROOT, "paper_2602_17206_amd", "csrc", "*"))):
        if path.endswith((".h", ".hip")):
            h.update(os.path.basename(path).encode())
            with open(path, "rb") as f:
                h.update(f.read())
    return h.hexdigest()[:16]


def load_traffic(workload):
    """HBM bytes per launch measured with rocprofv3 --pmc (profiles/hbm_traffic.json).  The figures are
    only used if they were taken with the kernels as they are now; otherwise (None, reason)."""
    try:
        with open(TRAFFIC_JSON) as f:
            data = json.load(f)
    except Exception as e:  # noqa: BLE001
        return None, "profiles/hbm_traffic.json not readable: %s" % e
    entry = data.get("workloads", {}).get(workload)
    if entry is None:
        return None, "profiles/hbm_traffic.json has no counters for %s" % workload
    now = kernel_source_hash()
    if entry.get("source_hash") != now:
        return None, ("counters in profiles/hbm_traffic.json were taken at kernel sources %s (commit %s); the sources are "
                      "now %s" % (entry.get("source_hash"), entry.get("commit"), now))
    return entry, None


def attach_traffic(roof, workload):
    entry, why = load_traffic(workload)
    if entry is None:
        roof["traffic"] = None
        roof["traffic_note"] = why
        return roof
    k = entry["kernels"].get(roof["kernel"])
    if k is None:
        roof["traffic"] = None
        roof["traffic_note"] = "no counters for kernel %s" % roof["kernel"]
        return roof
    roof["traffic"] = k["total_bytes"]
    roof["traffic_detail"] = dict(k, commit=entry.get("commit"), source_hash=entry.get("source_hash"))
    return roof


# ------------------------------------------------------------------------------------------------
# GPU legs
# ------------------------------------------------------------------------------------------------
def bench_pairs(wl, modes, steps, warmup, with_kernels=True, flags=0):
    """Forward+backward of a pair workload, one mode after the other per step."""
    import torch

    import paper_2602_17206_amd as pkg
    from paper_2602_17206_amd import binding

    xd = torch.from_numpy(wl.x).cuda()
    yd = torch.from_numpy(wl.y).cuda()
    torch.cuda.reset_peak_memory_stats()
    base_alloc = torch.cuda.memory_allocated()
    state = {}
    dx, dy = torch.empty_like(xd), torch.empty_like(yd)
    value = torch.empty(wl.B, dtype=torch.float32, device="cuda")
    for m in modes:
        desc = binding.make_desc(wl.B, wl.N, wl.M, wl.D, wl.gamma, m, flags=flags)
        nbytes = pkg.sdtw_workspace_bytes(desc)
        state[m] = dict(desc=desc, ws=binding.Workspace(nbytes), ws_bytes=nbytes)

    def fwd(m):
        s = state[m]
        binding.sdtw_forward_desc(s["desc"], xd, yd, s["ws"], value)

    def fwd_bwd(m):
        s = state[m]
        binding.sdtw_forward_desc(s["desc"], xd, yd, s["ws"], value)
        pkg.sdtw_backward(s["desc"], xd, yd, s["ws"], dx=dx, dy=dy)

    def timed(fn, n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n

    def step():
        for m in modes:
            fwd_bwd(m)

    for _ in range(warmup):
        step()
    sec_step = timed(step, steps)
    cells = wl.B * wl.N * wl.M
    per_mode = {}
    for m in modes:
        s = state[m]
        t_fb = timed(lambda: fwd_bwd(m), steps) if len(modes) > 1 else sec_step
        t_f = timed(lambda: fwd(m), steps)
        tensors = (xd.numel() + yd.numel() + dx.numel() + dy.numel() + value.numel()) * 4
        per_mode[MODE_NAMES[m]] = {
            "fwd_bwd_ms": t_fb * 1e3, "fwd_ms": t_f * 1e3,
            "fwd_bwd_cells_per_s": cells / t_fb, "fwd_cells_per_s": cells / t_f,
            "workspace_bytes": s["ws_bytes"], "peak_bytes": s["ws_bytes"] + tensors,
            "workspace_bytes_per_cell": s["ws_bytes"] / cells,
        }
    kernels = {}
    if with_kernels:
        binding.debug_profile(True)
        torch.cuda.synchronize()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        prof = binding.debug_profile_read(max_entries=steps * 64)
        binding.debug_profile(False)
        kernels = kernel_table(prof, steps)
    for m in modes:
        assert binding.workspace_status(state[m]["ws"]) == 0, "device reported an error"
    peak_alloc = torch.cuda.max_memory_allocated() - base_alloc
    return dict(sec_step=sec_step, cells_per_step=cells * len(modes), per_mode=per_mode, kernels=kernels,
                torch_peak_bytes=peak_alloc)


def peak_memory(per_mode):
    if "unfused" in per_mode and "fused" in per_mode:
        u, f = per_mode["unfused"], per_mode["fused"]
        return {"unfused_bytes": u["peak_bytes"], "fused_bytes": f["peak_bytes"],
                "fused_saving": 1.0 - f["peak_bytes"] / u["peak_bytes"]}
    return None


def dominant_roofline(kernels, cells, D, workload):
    dom = max(kernels.items(), key=lambda kv: kv[1]["ms_per_step"])
    roof = attach_traffic(roofline_for(dom[0], dom[1]["ms_per_launch"], cells, D), workload)
    roof["kernels_ms_per_step"] = {k: round(v["ms_per_step"], 5) for k, v in sorted(kernels.items())}
    return roof


def bench_barycenter(with_cpu):
    """The barycenter configuration: 50 Adam steps per mode, each forward+backward against all K."""
    import numpy as np
    import torch

    import paper_2602_17206_amd as pkg
    from paper_2602_17206_amd import binding, workloads

    bw = workloads.barycenter_workload()
    X = torch.from_numpy(bw.X).cuda()
    cells = bw.K * bw.L * bw.L
    out = {"config": {"workload": bw.name, "K": bw.K, "L": bw.L, "D": bw.D, "gamma": bw.gamma, "steps": bw.steps,
                      "lr": bw.lr, "cells_per_step": cells, "contraction": contraction_name(bw.D)}, "modes": {}}
    warmup = 3
    for mode in (pkg.UNFUSED, pkg.FUSED):
        z = torch.from_numpy(bw.z0.copy()).cuda()
        m = torch.zeros_like(z)
        v = torch.zeros_like(z)
        ws = None
        loss = torch.empty(1, dtype=torch.float32, device="cuda")
        losses = []
        for step in range(1, warmup + 1):
            _, _, ws = pkg.sdtw_barycenter_step(z, X, m, v, bw.gamma, step, bw.lr, mode=mode, workspace=ws, loss=loss)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for step in range(warmup + 1, warmup + bw.steps + 1):
            pkg.sdtw_barycenter_step(z, X, m, v, bw.gamma, step, bw.lr, mode=mode, workspace=ws, loss=loss)
            if step in (warmup + 1, warmup + bw.steps):
                losses.append(loss.item())
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        # per-kernel times of ten more steps
        binding.debug_profile(True)
        for step in range(warmup + bw.steps + 1, warmup + bw.steps + 11):
            pkg.sdtw_barycenter_step(z, X, m, v, bw.gamma, step, bw.lr, mode=mode, workspace=ws, loss=loss)
        torch.cuda.synchronize()
        kernels = kernel_table(binding.debug_profile_read(max_entries=1024), 10)
        binding.debug_profile(False)
        tensors = (X.numel() + 3 * z.numel() + 1) * 4
        out["modes"][MODE_NAMES[mode]] = {
            "steps": bw.steps, "ms_per_step": dt / bw.steps * 1e3, "fwd_bwd_cells_per_s": cells * bw.steps / dt,
            "loss_first": losses[0], "loss_last": losses[-1], "workspace_bytes": ws.nbytes,
            "peak_bytes": ws.nbytes + tensors, "roofline": dominant_roofline(kernels, cells, bw.D, bw.name)}
        assert binding.workspace_status(ws) == 0, "device reported an error"
    u, f = out["modes"]["unfused"], out["modes"]["fused"]
    out["peak_memory"] = {"unfused_bytes": u["peak_bytes"], "fused_bytes": f["peak_bytes"],
                          "fused_saving": 1.0 - f["peak_bytes"] / u["peak_bytes"]}
    # fused with SDTW_FLAG_MIN_MEMORY: 20 steps
    z = torch.from_numpy(bw.z0.copy()).cuda()
    m, v, ws = torch.zeros_like(z), torch.zeros_like(z), None
    loss = torch.empty(1, dtype=torch.float32, device="cuda")
    for step in range(1, 4):
        _, _, ws = pkg.sdtw_barycenter_step(z, X, m, v, bw.gamma, step, bw.lr, mode=pkg.FUSED, workspace=ws, loss=loss, min_memory=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for step in range(4, 24):
        pkg.sdtw_barycenter_step(z, X, m, v, bw.gamma, step, bw.lr, mode=pkg.FUSED, workspace=ws, loss=loss, min_memory=True)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    out["min_memory"] = {"flag": "SDTW_FLAG_MIN_MEMORY", "mode": "fused", "ms_per_step": dt / 20 * 1e3,
                         "workspace_bytes": ws.nbytes, "peak_bytes": ws.nbytes + (X.numel() + 3 * z.numel() + 1) * 4}
    if with_cpu:
        import oracle

        threads = host_threads()
        z = bw.z0.astype(np.float64)
        m, v = np.zeros_like(z), np.zeros_like(z)
        oracle.barycenter_step(z.copy(), bw.X[:2], bw.gamma, bw.lr, 0.9, 0.999, 1e-8, 1, m.copy(), v.copy())
        n, t0 = 0, time.perf_counter()
        while n < 3:
            oracle.barycenter_step(z, bw.X, bw.gamma, bw.lr, 0.9, 0.999, 1e-8, n + 1, m, v, nthreads=threads)
            n += 1
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": cells * n / dt, "unit": "DP cells/s (forward+backward)", "cores": threads,
                               "kind": "oracle", "sample": "%d barycenter steps on all K = %d sequences, %.1f s wall, float64"
                               % (n, bw.K, dt)}
    return out


_HOST_THREADS = None


def host_threads():
    """Threads the oracle may use, read once (a call with an explicit thread count changes OpenMP's default)."""
    global _HOST_THREADS
    if _HOST_THREADS is None:
        import oracle

        _HOST_THREADS = oracle.max_threads()
    return _HOST_THREADS


def cpu_baseline(wl, max_pairs=None, target_wall_s=2.0):
    """The CPU oracle as it stands, forward+backward, all host threads.  Small workloads: whole batches
    repeated for about target_wall_s.  max_pairs: one pass over the first max_pairs pairs of the batch
    (a pair of the N = M = 8192 configuration keeps about 2.1 GB of float64 tables in flight)."""
    import oracle

    threads = host_threads()
    oracle.batch(wl.x[:1, :64], wl.y[:1, :64], wl.gamma)  # load the library, touch memory
    if max_pairs is not None:
        nb = min(wl.B, max_pairs)
        t0 = time.perf_counter()
        oracle.batch(wl.x[:nb], wl.y[:nb], wl.gamma, nthreads=min(threads, nb))
        dt = time.perf_counter() - t0
        gb = (3 * (wl.N + 2) * (wl.M + 2) + wl.N * wl.M) * 8 / 1e9
        return {"value": nb * wl.N * wl.M / dt, "unit": "DP cells/s (forward+backward)", "cores": min(threads, nb),
                "kind": "oracle",
                "sample": "pairs 0..%d of the %s batch (B=%d), one pass, one pair per thread, %.1f s wall, float64, "
                          "%.1f GB of tables per in-flight pair" % (nb - 1, wl.name, wl.B, dt, gb)}
    reps, t0 = 0, time.perf_counter()
    while True:
        oracle.batch(wl.x, wl.y, wl.gamma, nthreads=threads)
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= target_wall_s or reps >= 200:
            break
    cells = wl.B * wl.N * wl.M * reps
    # ... and on one thread, on a few pairs of the same batch, for about a second
    nb = min(wl.B, 4)
    reps1, t1 = 0, time.perf_counter()
    while True:
        oracle.batch(wl.x[:nb], wl.y[:nb], wl.gamma, nthreads=1)
        reps1 += 1
        dt1 = time.perf_counter() - t1
        if dt1 >= 1.0 or reps1 >= 200:
            break
    return {"value": cells / dt, "unit": "DP cells/s (forward+backward)", "cores": threads, "kind": "oracle",
            "sample": "%d repetitions of the full %s batch (B=%d), %.1f s wall, float64" % (reps, wl.name, wl.B, dt),
            "value_one_core": nb * wl.N * wl.M * reps1 / dt1,
            "sample_one_core": "%d repetitions of %d pairs of the same batch on one thread, %.1f s" % (reps1, nb, dt1)}


def bench_half_inputs(wl, steps, warmup):
    """The workload's shape with float16 sequences (sdtw_forward_half / sdtw_backward_half), fused."""
    import torch

    import paper_2602_17206_amd as pkg
    from paper_2602_17206_amd import binding

    xh, yh = torch.from_numpy(wl.x).cuda().half(), torch.from_numpy(wl.y).cuda().half()
    value, desc, ws = pkg.sdtw_forward_half(xh, yh, wl.gamma, pkg.FUSED)

    def step():
        pkg.sdtw_forward_half(xh, yh, wl.gamma, pkg.FUSED, workspace=ws, value=value)
        return pkg.sdtw_backward_half(desc, ws)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        out = step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    del out
    assert binding.workspace_status(ws) == 0, "device reported an error"
    cells = wl.B * wl.N * wl.M
    return {"input_dtype": "f16", "mode": "fused", "contraction": "f16x1 (one fp16 MFMA product per 16 features, float32 accumulate)",
            "fwd_bwd_ms": dt * 1e3, "fwd_bwd_cells_per_s": cells / dt, "workspace_bytes": ws.nbytes,
            "note": "values and gradients of the sequences rounded to float16; includes allocating dx, dy per step"}


def pair_record(name, steps, warmup, with_cpu, mode_ids, extra_modes=(), min_memory=False, half_inputs=False):
    """Everything reported for one pair configuration: per-mode timings and bytes, roofline of the
    slowest kernel, CPU baseline.  extra_modes: modes that are not part of the configuration's step
    but are measured beside it for the memory comparison (fewer steps)."""
    import torch

    from paper_2602_17206_amd import workloads

    wl = workloads.pair_workload(name)
    modes = [mode_ids[m] for m in wl.modes]
    r = bench_pairs(wl, modes, steps, warmup)
    cells = wl.B * wl.N * wl.M
    rec = {"config": {"workload": wl.name, "B": wl.B, "N": wl.N, "M": wl.M, "D": wl.D, "gamma": wl.gamma,
                      "modes_per_step": list(wl.modes), "table_carry": "f64", "contraction": contraction_name(wl.D),
                      "cells_per_step": r["cells_per_step"]},
           "ms_per_step": r["sec_step"] * 1e3, "fwd_bwd_cells_per_s": r["cells_per_step"] / r["sec_step"],
           "modes": r["per_mode"], "torch_peak_bytes": r["torch_peak_bytes"],
           "roofline": dominant_roofline(r["kernels"], cells, wl.D, wl.name)}
    for em in extra_modes:
        torch.cuda.empty_cache()
        r2 = bench_pairs(wl, [mode_ids[em]], max(2, steps // 4), 1, with_kernels=False)
        rec["modes"][em] = dict(r2["per_mode"][em], note="not part of this configuration's step; measured for the memory comparison")
    pm = peak_memory(rec["modes"])
    if pm:
        rec["peak_memory"] = pm
    if min_memory:
        # the same configuration with SDTW_FLAG_MIN_MEMORY (checkpoints and a compact E instead of both
        # tables and a dense E): what the smaller workspace costs in time
        from paper_2602_17206_amd import binding

        torch.cuda.empty_cache()
        r3 = bench_pairs(wl, modes, max(5, steps // 2), 2, with_kernels=False, flags=binding.FLAG_MIN_MEMORY)
        rec["min_memory"] = {"flag": "SDTW_FLAG_MIN_MEMORY", "modes": r3["per_mode"], "peak_memory": peak_memory(r3["per_mode"])}
    if half_inputs:
        torch.cuda.empty_cache()
        rec["half_inputs"] = bench_half_inputs(wl, max(3, steps // 2), 2)
    if with_cpu:
        rec["cpu_baseline"] = cpu_baseline(wl, max_pairs=8 if wl.N * wl.M >= 4096 * 4096 else None)
    return rec, r


# ------------------------------------------------------------------------------------------------
# calibration legs
# ------------------------------------------------------------------------------------------------
def calibrate_valu():
    """Vector-ALU rates and the bare DP step, through sdtw_debug_rate_probe.  Cycles are wall time x
    2.4 GHz (the nominal clock; the ratios are what matters)."""
    from paper_2602_17206_amd import binding

    ghz, iters = 2.4, 2000
    scratch = binding.Workspace(binding.RATE_PROBE_SCRATCH_BYTES)
    names = ["v_add_f32", "v_fma_f32", "v_add_f64", "v_min_f64", "v_fma_f64", "v_exp_f32", "v_log_f32",
             "v_cvt_f32_f64", "v_cvt_f64_f32", "v_mov_b32_dpp"]

    def cyc(probe, variant, w, n, per):
        return binding.debug_rate_probe(probe, variant, w, n, scratch) * 1e-3 * ghz * 1e9 / (n * 32.0 * per)

    out = {"calibrate_valu": True, "clock_ghz_assumed": ghz, "instructions": {}, "dp_step": {}, "dp_step_two_rows": {},
           "dp_step_beside_mfma": {}, "dp_step_two_rows_beside_mfma": {}, "dp_step_with_memory_traffic": {}}
    for v, name in enumerate(names):
        row = {"w%d" % w: round(cyc(0, v, w, iters, w), 2) for w in (1, 2, 4)}
        if v not in (7, 8):
            row["dependent"] = round(cyc(1, v, 1, iters, 1), 2)
        out["instructions"][name] = row
    for w in (1, 2, 4):
        c1 = cyc(2, 0, w, iters, 1)
        c2 = cyc(3, 0, w, iters, 1)
        out["dp_step"]["w%d" % w] = {"cycles_per_step_of_a_wavefront": round(c1, 1), "cycles_per_64_cells_per_simd": round(c1 / w, 1)}
        out["dp_step_two_rows"]["w%d" % w] = {"cycles_per_step_of_a_wavefront": round(c2, 1),
                                             "cycles_per_64_cells_per_simd": round(c2 / w / 2, 1)}
    for mf in (0, 12, 24, 48, 96):
        out["dp_step_beside_mfma"]["%d_mfma_per_32_steps" % mf] = round(cyc(4, mf, 1, iters // 4, 1), 1)
        out["dp_step_two_rows_beside_mfma"]["%d_mfma_per_32_steps" % mf] = round(cyc(4, 1000 + mf, 1, iters // 4, 1), 1)
    for label, v in (("arithmetic only", 0), ("+ cost from LDS", 1), ("+ edge value to LDS", 3), ("+ table store to HBM", 7),
                     ("+ barrier per 32 steps", 15), ("table store only", 4), ("barrier only", 8)):
        out["dp_step_with_memory_traffic"][label] = round(cyc(5, v, 1, iters // 8, 1), 1)
    return out


def ingest_pmc(base, workload):
    """profiles/hbm_traffic.json / .md from the CSVs of four `rocprofv3 --pmc` runs under `base`:
    cal_fetch, cal_write (bench.py --calibrate-copy) and fetch, write (bench.py --workload W
    --headline-only --no-cpu-baseline).  Counters are KiB per dispatch, scaled by what the same counter
    reads for the 256 MiB copy."""
    import collections
    import subprocess

    def per_kernel(sub):
        files = glob.glob(os.path.join(base, sub, "**", "*counter_collection.csv"), recursive=True)
        assert files, "no counter CSV under %s/%s" % (base, sub)
        agg = collections.defaultdict(list)
        for path in files:
            with open(path) as f:
                for r in csv.DictReader(f):
                    agg[r["Kernel_Name"]].append(float(r["Counter_Value"]))
        return agg

    def short(n):
        return n.replace("void ", "").replace("sdtw::", "").split("(")[0]

    def cal(agg):  # the copy kernel: at least 10 dispatches, the largest counter
        k = max((k for k in agg if len(agg[k]) >= 10), key=lambda k: sum(agg[k]) / len(agg[k]))
        return k, sorted(agg[k])[len(agg[k]) // 2]

    labels = [(", true>", "second_sweep_dp"),  # backward_dp_kernel<..., true>: the contracting sweep (a no-op unless the pool overflowed)
              ("both_sweeps_kernel<-1", "both_sweeps_unfused"), ("both_sweeps_kernel<", "both_sweeps_fused"),
              ("forward_dp_kernel<-1", "forward_dp_unfused"), ("backward_dp_kernel<-1", "backward_dp_unfused"),
              ("forward_dp_kernel<", "forward_dp_fused"), ("backward_dp_kernel<", "backward_dp_fused"),
              ("cost_tensor", "cost_tensor"), ("input_grad", "input_grad"), ("alignment", "alignment"),
              ("forward_prep_kernel", "forward_prep"), ("backward_prep_kernel", "backward_prep"),
              ("gradient_finish", "gradient_finish")]
    kf, vf = cal(per_kernel("cal_fetch"))
    kw, vw = cal(per_kernel("cal_write"))
    nbytes = 256 * 1024 * 1024
    ff, fw = nbytes / (vf * 1024.0), nbytes / (vw * 1024.0)
    f, w = per_kernel("fetch"), per_kernel("write")
    try:
        commit = subprocess.check_output(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], text=True).strip()
    except Exception:  # noqa: BLE001
        commit = None
    entry = {"source_hash": kernel_source_hash(), "commit": commit,
             "calibration": {"copy_kernel": short(kf), "fetch_kib_per_copy": vf, "fetch_factor": ff,
                             "write_kib_per_copy": vw, "write_factor": fw}, "kernels": {}, "rows": []}
    for k in sorted(f):
        if "sdtw::" not in k:
            continue
        fb = sum(f[k]) / len(f[k]) * 1024 * ff
        wb = sum(w[k]) / len(w[k]) * 1024 * fw if k in w else 0.0
        entry["rows"].append({"kernel": short(k), "dispatches": len(f[k]), "fetch_bytes": fb, "write_bytes": wb})
        for pat, lab in labels:
            if pat in k:
                entry["kernels"][lab] = {"fetch_bytes": fb, "write_bytes": wb, "total_bytes": fb + wb}
                break
    try:
        with open(TRAFFIC_JSON) as fh:
            data = json.load(fh)
        if "workloads" not in data:
            data = {"workloads": {}}
    except Exception:  # noqa: BLE001
        data = {"workloads": {}}
    data["workloads"][workload] = entry
    with open(TRAFFIC_JSON, "w") as fh:
        json.dump(data, fh, indent=1, sort_keys=True)
    md = ["# HBM traffic per kernel launch (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)", "",
          "Commands, per workload W (from the repository root, after `cd /tmp && export TMPDIR=/tmp && cd <repo>`; one counter per run),",
          "then `python3 bench.py --ingest-pmc out --pmc-workload W` (no GPU) writes this file and `hbm_traffic.json`:", "",
          "    rocprofv3 --pmc FETCH_SIZE -d out/cal_fetch -o p --output-format csv -- python3 bench.py --calibrate-copy",
          "    rocprofv3 --pmc WRITE_SIZE -d out/cal_write -o p --output-format csv -- python3 bench.py --calibrate-copy",
          "    rocprofv3 --pmc FETCH_SIZE -d out/fetch -o p --output-format csv -- python3 bench.py --workload W --headline-only --no-cpu-baseline --steps 5 --warmup 1",
          "    rocprofv3 --pmc WRITE_SIZE -d out/write -o p --output-format csv -- python3 bench.py --workload W --headline-only --no-cpu-baseline --steps 5 --warmup 1", "",
          "The counters are in KiB per dispatch; they are scaled by what the same counter reads for a plain copy of known size",
          "(true bytes = counter KiB x 1024 x factor).  The numbers are means over all dispatches of a run.  `bench.py` uses a",
          "workload's figures only while the kernel sources still hash to the value noted here.", ""]
    for W in sorted(data["workloads"]):
        e = data["workloads"][W]
        c = e["calibration"]
        md += ["## %s" % W, "",
               "Kernel sources %s, commit %s.  Calibration (256 MiB device-to-device copy, kernel `%s`): FETCH_SIZE reads %.0f KiB per "
               "copy -> factor %.3f; WRITE_SIZE reads %.0f KiB -> factor %.3f." % (
                   e["source_hash"], e["commit"], c["copy_kernel"], c["fetch_kib_per_copy"], c["fetch_factor"],
                   c["write_kib_per_copy"], c["write_factor"]), "",
               "| kernel | dispatches | fetch MB/launch | write MB/launch |", "|---|---|---|---|"]
        md += ["| `%s` | %d | %.3f | %.3f |" % (r["kernel"], r["dispatches"], r["fetch_bytes"] / 1e6, r["write_bytes"] / 1e6)
               for r in e["rows"]]
        md.append("")
    with open(TRAFFIC_MD, "w") as fh:
        fh.write("\n".join(md))
    return {"ingest_pmc": True, "workload": workload, "kernels": entry["kernels"], "source_hash": entry["source_hash"]}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: every pair is independent, so more GPUs only shard the batch; "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.ingest_pmc:
        print(json.dumps(ingest_pmc(args.ingest_pmc, args.pmc_workload or args.workload)))
        return
    import torch

    import paper_2602_17206_amd as pkg

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    if args.calibrate_copy:
        n = 256 * 1024 * 1024  # bytes per buffer
        src = torch.empty(n // 4, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": True, "bytes_read_per_copy": n, "bytes_written_per_copy": n, "copies": 10}))
        return
    pkg.load_library()
    if args.calibrate_valu:
        print(json.dumps(calibrate_valu()))
        return
    mode_ids = {"unfused": pkg.UNFUSED, "fused": pkg.FUSED}
    with_cpu = not args.no_cpu_baseline

    if args.modes:  # a profiling run of chosen modes: the headline record alone
        from paper_2602_17206_amd import workloads

        wl = workloads.pair_workload(args.workload)
        r = bench_pairs(wl, [mode_ids[m] for m in args.modes.split(",")], args.steps, args.warmup)
        rec = {"config": {"workload": wl.name, "modes_per_step": args.modes.split(","), "cells_per_step": r["cells_per_step"]},
               "ms_per_step": r["sec_step"] * 1e3, "modes": r["per_mode"],
               "roofline": dominant_roofline(r["kernels"], wl.B * wl.N * wl.M, wl.D, wl.name)}
    else:
        # beside the configuration's own step: the unfused mode of the same shape (memory comparison) and
        # float16 inputs - not in a --headline-only run, whose kernel statistics are then the step's alone
        full = args.workload == HEADLINE and not args.headline_only
        rec, r = pair_record(args.workload, args.steps, args.warmup, with_cpu, mode_ids,
                             extra_modes=("unfused",) if full else (), half_inputs=full)

    line = {
        "metric": "Soft-DTW fwd+bwd DP cells/sec (B*N*M/s) at B=32",
        "value": r["cells_per_step"] / r["sec_step"], "unit": "cells/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": r["sec_step"] * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
    }
    line.update({k: rec[k] for k in ("config", "modes", "roofline") if k in rec})
    for k in ("torch_peak_bytes", "peak_memory", "half_inputs", "cpu_baseline"):
        if k in rec:
            line[k] = rec[k]
    if not args.headline_only and not args.modes:
        others = {}
        for name, steps in (("c2_b32_l256", 50), ("c3_b32_l1024_walk", 20)):
            if name == args.workload:
                continue
            torch.cuda.empty_cache()
            others[name], _ = pair_record(name, steps, 3, with_cpu, mode_ids, min_memory=True)
        torch.cuda.empty_cache()
        others["c5_barycenter"] = bench_barycenter(with_cpu)
        line["other_workloads"] = others
    print(json.dumps(line))


if __name__ == "__main__":
    main()
