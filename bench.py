#!/usr/bin/env python3
"""Benchmark of the Soft-DTW hot path on one MI355X.

One "step" is one pass of the whole hot path over one synthetic batch: row norms, then forward
+ backward in unfused mode (cost tensor materialised) and forward + backward in fused mode (cost
recomputed per tile), i.e. every DP cell is visited once per mode.  The headline value is DP
cells per second for forward+backward, cells = modes * B * N * M per step, with the inputs
already resident in device memory.  The default workload is the B=32, N=M=256, D=128, gamma=0.1
configuration; `--workload` selects another, `--all` appends a short report for every
configuration (including the barycenter step) to the same JSON line.

Prints ONE JSON line.  `roofline` describes the kernel that took the most time in the step,
timed with HIP events (per-kernel events are recorded in a second, identical loop so that they do
not perturb the headline timing); `cpu_baseline` is the float64 CPU oracle timed on this host.
"""
import argparse
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
# add or lane shift 0.5 to 1, an exp2/log2 (quarter of the float32 rate) 2.
PEAK_VALU_TOPS = 256 * 64 * 2.4e9 / 1e12

# Work per DP cell and sweep in those slots, from the instruction mix of the recurrence (Sec. 2
# Eq. 1-2 with the max-shift of Sec. 4.2): 11 float64 operations (3 min/max, 3 subtractions, 1 fma,
# 4 conversions), 2 lane-shift moves, 2 float32 additions, 3 transcendentals = 11 + 2 + 1 + 6 = 20
# (the stand-alone micro-benchmark of the step measures 82 cycles per 64 cells per SIMD = 20.5).
# The reverse sweep that also forms E adds one exp2, one float64 subtraction, one conversion and one
# float32 addition: 24.5.  (Recomputing R in the fused backward of large problems is this library's
# choice, not algorithmic work: it is not counted.)
SLOTS_SWEEP_CELL = 20.0
SLOTS_BWD_E_CELL = 24.5
MODE_NAMES = {0: "unfused", 1: "fused"}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2_b32_l256")
    ap.add_argument("--modes", default="", help="comma list of unfused,fused (default: the workload's modes)")
    ap.add_argument("--all", action="store_true", help="also report the other configurations")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device copy of known size (reference for the rocprofv3 HBM counters)")
    return ap.parse_args()


def kernel_table(prof, steps):
    """[(label, ms)] of many steps -> {label: (launches per step, mean ms per launch, ms per step)}."""
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
               "per_cell": {"valu_slots": slots}}
        if name.endswith("_fused"):
            fl = (2 if both else 1) * 2.0 * D * wl_cells / sec / 1e12
            pk = PEAK_MFMA_F16_TFLOPS if D <= 128 else PEAK_MFMA_F32_TFLOPS
            out["mfma"] = {"achieved": fl, "peak": pk, "unit": "TFLOP/s", "frac": fl / pk,
                           "dtype": "f16 x3 (split operands)" if D <= 128 else "f32"}
        # table traffic: 8 B per cell and sweep; the E-forming reverse sweep also writes E; unfused reads the cost
        nbytes = (16.0 if both else 8.0) + (4.0 if name.startswith("backward") else 0.0) + \
                 ((8.0 if both else 4.0) if name.endswith("_unfused") else 0.0)
        bw = nbytes * wl_cells / sec / 1e9
        out["hbm"] = {"achieved": bw, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": bw / PEAK_HBM_GBS, "bytes_per_cell": nbytes}
        return out
    if name == "cost_tensor":
        bw = 4.0 * wl_cells / sec / 1e9  # the stored tensor
        return {"kernel": name, "bound": "hbm", "achieved": bw, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": bw / PEAK_HBM_GBS, "traffic": traffic}
    if name == "alignment":
        bw = 20.0 * wl_cells / sec / 1e9  # reads both float64 tables, writes float32 E
        return {"kernel": name, "bound": "hbm", "achieved": bw, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": bw / PEAK_HBM_GBS, "traffic": traffic}
    if name == "input_grad":
        bw = 8.0 * wl_cells / sec / 1e9  # E is read once per side
        return {"kernel": name, "bound": "hbm", "achieved": bw, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": bw / PEAK_HBM_GBS, "traffic": traffic}
    return {"kernel": name, "bound": "hbm", "achieved": None, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": None,
            "traffic": traffic}


def load_traffic(workload):
    """HBM bytes per launch measured with rocprofv3 --pmc (committed under profiles/), if present."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            return json.load(f).get(workload, {})
    except Exception:
        return {}


def bench_pairs(wl, modes, steps, warmup, with_kernels=True):
    import torch

    import paper_2602_17206_amd as pkg
    from paper_2602_17206_amd import binding

    xd = torch.from_numpy(wl.x).cuda()
    yd = torch.from_numpy(wl.y).cuda()
    torch.cuda.reset_peak_memory_stats()
    base_alloc = torch.cuda.memory_allocated()
    state = {}
    for m in modes:
        desc = binding.make_desc(wl.B, wl.N, wl.M, wl.D, wl.gamma, m)
        nbytes = pkg.sdtw_workspace_bytes(desc)
        state[m] = dict(desc=desc, ws=binding.Workspace(nbytes), ws_bytes=nbytes,
                        value=torch.empty(wl.B, dtype=torch.float32, device="cuda"),
                        dx=torch.empty_like(xd), dy=torch.empty_like(yd))

    def fwd(m):
        s = state[m]
        pkg.sdtw_forward(xd, yd, wl.gamma, m, workspace=s["ws"], value=s["value"])

    def fwd_bwd(m):
        s = state[m]
        pkg.sdtw_forward(xd, yd, wl.gamma, m, workspace=s["ws"], value=s["value"])
        pkg.sdtw_backward(s["desc"], xd, yd, s["ws"], dx=s["dx"], dy=s["dy"])

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
        t_fb = timed(lambda: fwd_bwd(m), steps)
        t_f = timed(lambda: fwd(m), steps)
        tensors = (xd.numel() + yd.numel() + s["dx"].numel() + s["dy"].numel() + s["value"].numel()) * 4
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
        # split by mode: labels of mode-specific kernels carry the mode name; shared labels are pooled
        kernels = kernel_table(prof, steps)
    for m in modes:
        assert binding.workspace_status(state[m]["ws"]) == 0, "device reported an error"
    peak_alloc = torch.cuda.max_memory_allocated() - base_alloc
    return dict(sec_step=sec_step, cells_per_step=cells * len(modes), per_mode=per_mode, kernels=kernels,
                torch_peak_bytes=peak_alloc)


def bench_barycenter(steps, warmup):
    import torch

    import paper_2602_17206_amd as pkg
    from paper_2602_17206_amd import workloads

    bw = workloads.barycenter_workload()
    X = torch.from_numpy(bw.X).cuda()
    out = {}
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
        cells = bw.K * bw.L * bw.L
        out[MODE_NAMES[mode]] = {"steps": bw.steps, "ms_per_step": dt / bw.steps * 1e3,
                                 "fwd_bwd_cells_per_s": cells * bw.steps / dt, "loss_first": losses[0],
                                 "loss_last": losses[-1], "workspace_bytes": ws.nbytes}
    return out


def bench_normalized(wl, steps, warmup):
    """Normalised Soft-DTW (cross term + two self terms), fused, forward+backward."""
    import torch

    import paper_2602_17206_amd as pkg

    xd = torch.from_numpy(wl.x).cuda()
    yd = torch.from_numpy(wl.y).cuda()
    value, desc, ws = pkg.sdtw_normalized_forward(xd, yd, wl.gamma, pkg.FUSED)
    dx, dy = torch.empty_like(xd), torch.empty_like(yd)

    def step():
        pkg.sdtw_normalized_forward(xd, yd, wl.gamma, pkg.FUSED, workspace=ws, value=value)
        pkg.sdtw_normalized_backward(desc, xd, yd, ws, dx=dx, dy=dy)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    cells = wl.B * (wl.N * wl.M + wl.N * wl.N + wl.M * wl.M)
    return {"workload": wl.name, "mode": "fused", "ms_per_step": dt * 1e3, "cells_per_step_three_terms": cells,
            "fwd_bwd_cells_per_s": cells / dt, "workspace_bytes": ws.nbytes}


def bench_band(wl, w, steps, warmup):
    """Band constraint |i-j| <= w on a pair workload, forward+backward per mode; cells counted are
    those inside the band."""
    import torch

    import paper_2602_17206_amd as pkg

    xd = torch.from_numpy(wl.x).cuda()
    yd = torch.from_numpy(wl.y).cuda()
    dx, dy = torch.empty_like(xd), torch.empty_like(yd)
    inside = sum(max(0, min(wl.M - 1, i + w) - max(0, i - w) + 1) for i in range(wl.N))
    out = {"workload": wl.name, "bandwidth": w, "cells_inside_band": wl.B * inside}
    for name, mode in (("unfused", pkg.UNFUSED), ("fused", pkg.FUSED)):
        value, desc, ws = pkg.sdtw_forward(xd, yd, wl.gamma, mode, bandwidth=w)

        def step():
            pkg.sdtw_forward(xd, yd, wl.gamma, mode, workspace=ws, value=value, bandwidth=w)
            pkg.sdtw_backward(desc, xd, yd, ws, dx=dx, dy=dy)

        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        out[name] = {"fwd_bwd_ms": dt * 1e3, "fwd_bwd_band_cells_per_s": wl.B * inside / dt}
        del ws
        torch.cuda.empty_cache()
    return out


def cpu_baseline(wl, target_wall_s=2.0):
    """The CPU oracle as it stands, forward+backward, all host threads, on whole batches of the
    workload repeated until about target_wall_s has passed."""
    import oracle

    threads = oracle.max_threads()
    oracle.batch(wl.x[:1], wl.y[:1], wl.gamma)  # load the library, touch memory
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


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: every pair is independent, so more GPUs only shard the batch; "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2602_17206_amd as pkg
    from paper_2602_17206_amd import workloads

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
    wl = workloads.pair_workload(args.workload)
    mode_ids = {"unfused": pkg.UNFUSED, "fused": pkg.FUSED}
    modes = [mode_ids[m] for m in (args.modes.split(",") if args.modes else wl.modes)]

    r = bench_pairs(wl, modes, args.steps, args.warmup)
    cells = wl.B * wl.N * wl.M
    value = r["cells_per_step"] / r["sec_step"]
    traffic = load_traffic(wl.name)
    dom = max(r["kernels"].items(), key=lambda kv: kv[1]["ms_per_step"])
    roof = roofline_for(dom[0], dom[1]["ms_per_launch"], cells, wl.D, traffic.get(dom[0]))
    if isinstance(roof.get("traffic"), dict):  # HBM bytes per launch (rocprofv3 counters), split kept beside the total
        roof["traffic_detail"] = roof["traffic"]
        roof["traffic"] = roof["traffic"]["total_bytes"]
    roof["kernels_ms_per_step"] = {k: round(v["ms_per_step"], 5) for k, v in sorted(r["kernels"].items())}

    line = {
        "metric": "Soft-DTW fwd+bwd DP cells/sec (B*N*M/s) at B=32",
        "value": value, "unit": "cells/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r["sec_step"] * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "B": wl.B, "N": wl.N, "M": wl.M, "D": wl.D, "gamma": wl.gamma,
                   "modes_per_step": [MODE_NAMES[m] for m in modes],
                   "table_carry": "f64", "cells_per_step": r["cells_per_step"]},
        "modes": r["per_mode"],
        "torch_peak_bytes": r["torch_peak_bytes"],
        "roofline": roof,
    }
    if "unfused" in r["per_mode"] and "fused" in r["per_mode"]:
        u, f = r["per_mode"]["unfused"], r["per_mode"]["fused"]
        line["peak_memory"] = {"unfused_bytes": u["peak_bytes"], "fused_bytes": f["peak_bytes"],
                               "fused_saving": 1.0 - f["peak_bytes"] / u["peak_bytes"]}
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(wl)
    if args.all:
        others = {}
        for name in workloads.CONFIG_SHAPES:
            if name == wl.name:
                continue
            w2 = workloads.pair_workload(name)
            n2 = 5 if w2.N >= 4096 else 20
            r2 = bench_pairs(w2, [mode_ids[m] for m in w2.modes], n2, 2)
            c2 = w2.B * w2.N * w2.M
            d2 = max(r2["kernels"].items(), key=lambda kv: kv[1]["ms_per_step"])
            others[name] = {"modes": r2["per_mode"], "roofline": roofline_for(d2[0], d2[1]["ms_per_launch"], c2, w2.D),
                            "kernels_ms_per_step": {k: round(v["ms_per_step"], 5) for k, v in sorted(r2["kernels"].items())}}
            del r2
            torch.cuda.empty_cache()
        others["c5_barycenter"] = bench_barycenter(50, 3)
        others["normalized_c2"] = bench_normalized(wl, 20, 3)
        others["band_c3_w64"] = bench_band(workloads.pair_workload("c3_b32_l1024_walk"), 64, 20, 3)
        others["band_c4_w128"] = bench_band(workloads.pair_workload("c4_b32_l8192"), 128, 5, 2)
        line["other_workloads"] = others
    print(json.dumps(line))


if __name__ == "__main__":
    main()
