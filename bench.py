#!/usr/bin/env python3
"""Benchmark of the DropCompute step-time simulator on one MI355X.

One "step" is one whole pass of the hot path over a latency tensor already resident in HBM:
dc_simulate_async (thresholds sorted, the streaming scan over lat, reductions, finalize), the
copy of the 2*K result sums to the host, and dc_select_tau.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]
                  [--rows M] [--workers N] [--thresholds K] [--grid recipe|dense|upper-half]
                  [--path sums|per-step|analytic|worker-moments]

The result sums are written by the library's last kernel straight into pinned host memory (the output pointers of
dc_simulate_async may be any memory the device can write), so a step has no separate copy.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

HBM_PEAK_GBPS = 8000.0            # MI355X published HBM3E bandwidth
METRIC = "worker*microbatch*tau evals/s at N=2048; achieved HBM GB/s vs MI355X peak"
SCAN_KERNEL = "dc_scan_vec4_kernel"


def ensure_built() -> None:
    import paper_2306_10598_amd as dc
    from dc_workloads import device as gen_device
    if not dc.LIB_PATH.exists() or not gen_device._LIB_PATH.exists():
        import __graft_entry__
        __graft_entry__.build()


def kernel_source_hash() -> str:
    h = hashlib.sha256()
    for path in sorted((ROOT / "paper_2306_10598_amd" / "csrc").iterdir()):        # every source of the library
        if path.suffix in (".hip", ".h", ".inl"):
            h.update(path.read_bytes())
    return h.hexdigest()[:16]


def recorded_traffic(workload: str):
    """(HBM bytes per launch of the scan kernel, where the figure comes from): the committed rocprofv3 counter summary
    for this workload, or (None, why not) when there is none or the kernel sources changed since it was taken."""
    path = ROOT / "profiles" / f"{SCAN_KERNEL}_{workload}_pmc.txt"
    if not path.exists():
        return None, "no counter summary for this workload under profiles/"
    fields = {}
    for line in path.read_text().splitlines():
        if ":" in line and not line.startswith("#"):
            k, v = line.split(":", 1)
            fields[k.strip()] = v.strip()
    if fields.get("kernel_source_hash") != kernel_source_hash():
        return None, f"profiles/{path.name} was recorded for other kernel sources"
    try:
        return float(fields["hbm_bytes_per_launch"]), (f"profiles/{path.name}: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this "
                                                        "command, recorded earlier (not read in this run); kernel source hash matches")
    except (KeyError, ValueError):
        return None, f"profiles/{path.name} holds no hbm_bytes_per_launch"


def host_core_report():
    """How many cores the host has, how many this process may use, and how many threads the oracle gets."""
    from dc_workloads import host
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count() or 1
    return {"host_cores": os.cpu_count() or 1, "usable_cores": usable, "threads_used": host.cpu_threads(),
            "thread_cap": "16: the share of the host that one GPU's job may use on the benchmark machines"}


def literal_oracle_full(names=("tiny", "lognormal64")):
    """The four-loop oracle (the definition, O(K) work per element) on the two smallest workloads at full size."""
    import oracle
    from dc_workloads import config, host
    threads = host.cpu_threads()
    rows = []
    for name in names:
        r = config(name)
        lat = host.generate(r, 0, r.T, threads)
        taus = host.tau_grid(r, threads)
        t0 = time.perf_counter()
        oracle.simulate_threaded(lat, taus, r.comm, "literal", threads)
        dt = time.perf_counter() - t0
        rows.append({"workload": f"{name}: T={r.T} N={r.N} M={r.M} K={taus.size}", "seconds": dt,
                     "value": r.elements * taus.size / dt, "unit": "evals/s", "threads": threads})
    return rows


def cpu_baseline(r, taus, target_seconds: float = 12.0):
    """The CPU oracle, as it stands, on the first trials of the same workload."""
    import oracle
    from dc_workloads import host
    threads = host.cpu_threads()
    per_trial = r.N * r.M
    # calibrate on a small slab, then size the sample for about target_seconds
    t_small = max(threads, min(r.T, (32 << 20) // per_trial))
    lat = host.generate(r, 0, t_small, threads)
    t0 = time.perf_counter()
    oracle.simulate_threaded(lat, taus, r.comm, "sorted", threads)
    dt = max(time.perf_counter() - t0, 1e-4)
    trials = int(min(r.T, max(t_small, t_small * target_seconds / dt), (4 << 30) // (4 * per_trial)))
    lat = host.generate(r, 0, trials, threads)
    reps, dt = 0, 0.0
    t0 = time.perf_counter()
    while dt < target_seconds:                                 # repeat the same sample until the clock is long enough
        oracle.simulate_threaded(lat, taus, r.comm, "sorted", threads)
        reps += 1
        dt = time.perf_counter() - t0
    sorted_rate = reps * trials * per_trial * taus.size / dt
    # one thread, on a slab sized for a couple of seconds
    t_one = max(1, min(trials, int(trials * 2.0 * reps / (dt * threads)) if dt > 0 else 1))
    t0 = time.perf_counter()
    oracle.simulate(lat[:t_one], taus, r.comm, "sorted")
    d1 = time.perf_counter() - t0
    # the four-loop form on a slab of this workload small enough to finish in a few seconds
    t_lit = max(1, min(trials, int(2.0e10 // (per_trial * taus.size))))
    t0 = time.perf_counter()
    oracle.simulate_threaded(lat[:t_lit], taus, r.comm, "literal", threads)
    dl = time.perf_counter() - t0
    cores = host_core_report()
    return {
        "value": sorted_rate, "unit": "evals/s", "cores": threads, "kind": "oracle",
        "sample": f"first {trials} of {r.T} trials of {r.name} (N={r.N}, M={r.M}, K={taus.size}), "
                  f"sorted-threshold oracle, {reps} passes in {dt:.2f} s; input generation not timed",
        **cores,
        "value_1_thread": t_one * per_trial * taus.size / d1,
        "literal_value": t_lit * per_trial * taus.size / dl,
        "literal_sample": f"first {t_lit} trials of this workload, four-loop oracle, {dl:.2f} s",
        "literal_full": literal_oracle_full(),
    }


def trial_kernel_name(r, K: int) -> str:
    """The streaming kernel of the per-iteration pass for this shape (16-byte aligned, contiguous tensor)."""
    whole_rows = r.M % 4 == 0 and (r.M <= 128 or r.M == 256)
    if r.N * r.M <= 16384 and K <= 511:                                # every wave owns a trial
        return "dc_trial_scan_wave_kernel" if whole_rows else "dc_trial_scan_wave_flat_kernel"
    return "dc_trial_scan_vec4_kernel" if whole_rows else "dc_trial_scan_flat_kernel"


def bench_per_step(args, r, lat, taus, taus_dev, stream) -> int:
    """Same contract for the second entry point: S_eff as the mean of per-iteration speedups."""
    import numpy as np
    import torch

    import paper_2306_10598_amd as dc
    K = taus.size
    host_out = torch.zeros(K, dtype=torch.float64).pin_memory()       # written by the library's last kernel
    ws = torch.empty(dc.dc_speedup_workspace_bytes(r.T, r.N, r.M, K), dtype=torch.uint8, device=lat.device)
    torch.cuda.synchronize()

    call = dc.PreparedSpeedup(lat, taus_dev, r.comm, None, host_out, ws, stream, taus_host=taus)   # arguments marshalled once

    def step():
        call.enqueue()
        stream.synchronize()
        return call.select()                                           # Algorithm 2's final argmax

    dc.dc_set_kernel_timing(True)
    for _ in range(args.warmup):
        step()
    if dc.dc_workspace_status(ws, stream) != dc.DC_OK:
        print("device reported a value error", file=sys.stderr)
        return 1
    scan_ms = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        best = step()
        scan_ms.append(dc.dc_last_kernel_ms()[0])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    dc.dc_set_kernel_timing(False)
    scan_avg_ms = float(np.mean(scan_ms))
    algo_bytes = 4.0 * r.elements
    achieved = algo_bytes / (scan_avg_ms * 1e-3) / 1e9
    line = {
        "metric": METRIC, "value": float(r.elements) * K / (wall / args.steps), "unit": "evals/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": 1e3 * wall / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int32", "data": "synthetic",
        "config": {"workload": f"{r.name}: T={r.T} N={r.N} M={r.M} K={K} comm={r.comm}us, {r.description}",
                   "path": "per-step speedup (Algorithm 2 as printed)", "tensor_bytes": r.nbytes,
                   "best_tau_us": int(taus[best]), "best_seff": float(host_out[best])},
        "roofline": {"bound": "hbm", "kernel": trial_kernel_name(r, K), "achieved": achieved,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": None,
                     "kernel_ms": scan_avg_ms, "kernel_ms_min": float(np.min(scan_ms)),
                     "algorithmic_bytes": algo_bytes},
    }
    if not args.no_cpu_baseline:
        import oracle
        from dc_workloads import host
        trials = max(1, min(r.T, int(3.0e9 // (r.N * r.M * K))))
        sample = host.generate(r, 0, trials)
        t0 = time.perf_counter()
        oracle.per_step_speedup(sample, taus, r.comm)
        dt = time.perf_counter() - t0
        line["cpu_baseline"] = {"value": trials * r.N * r.M * K / dt, "unit": "evals/s", "cores": 1, "kind": "oracle",
                                "sample": f"first {trials} trials, Algorithm 2 as printed (float64, one thread), {dt:.2f} s"}
    print(json.dumps(line))
    return 0


def bench_analytic(args, r, lat, taus) -> int:
    """Moments pass + closed-form curves; the roofline is the moments kernel's (one read of lat)."""
    import numpy as np
    import torch

    import paper_2306_10598_amd as dc
    K = taus.size

    def step():
        _, _, mean, var = dc.dc_moments(lat)
        return dc.dc_analytic_curves(mean, var, r.N, r.M, taus, r.comm)

    dc.dc_set_kernel_timing(True)
    for _ in range(args.warmup):
        step()
    kernel_ms = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        dc.dc_moments(lat)
        kernel_ms.append(dc.dc_last_kernel_ms()[0])
        _, _, mean, var = dc.dc_moments(lat)
        e_done, e_t, s_eff, best = dc.dc_analytic_curves(mean, var, r.N, r.M, taus, r.comm)
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / 2.0                     # two moments passes per loop turn
    dc.dc_set_kernel_timing(False)
    ms = float(np.mean(kernel_ms))
    achieved = 4.0 * r.elements / (ms * 1e-3) / 1e9
    print(json.dumps({
        "metric": METRIC, "value": float(r.elements) * K / (wall / args.steps), "unit": "evals/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": 1e3 * wall / args.steps, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "int32", "data": "synthetic",
        "config": {"workload": f"{r.name}: T={r.T} N={r.N} M={r.M} K={K}", "path": "moments + closed-form curves",
                   "mu_us": mean, "sigma_us": var ** 0.5, "modelled_iteration_time_us": e_t,
                   "best_tau_us": int(taus[best])},
        "roofline": {"bound": "hbm", "kernel": "dc_moments_kernel", "achieved": achieved, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": None, "kernel_ms": ms,
                     "algorithmic_bytes": 4.0 * r.elements}}))
    return 0


def bench_worker_moments(args, r, lat) -> int:
    """Per-worker statistics (dc_worker_moments): one read of lat; the roofline is that of its streaming kernel."""
    import numpy as np
    import torch

    import paper_2306_10598_amd as dc
    dc.dc_set_kernel_timing(True)
    for _ in range(args.warmup):
        dc.dc_worker_moments(lat)
    kernel_ms = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        sums, squares, mean, var = dc.dc_worker_moments(lat)
        kernel_ms.append(dc.dc_last_kernel_ms()[0])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    dc.dc_set_kernel_timing(False)
    ms = float(np.mean(kernel_ms))
    achieved = 4.0 * r.elements / (ms * 1e-3) / 1e9
    print(json.dumps({
        "metric": "latencies/s through the per-worker statistics; achieved HBM GB/s vs MI355X peak",
        "value": float(r.elements) / (wall / args.steps), "unit": "latencies/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": 1e3 * wall / args.steps, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "int32", "data": "synthetic",
        "config": {"workload": f"{r.name}: T={r.T} N={r.N} M={r.M}", "path": "per-worker sums and sums of squares of the row totals",
                   "mean_of_worker_means_us": float(mean.mean()), "variance_between_worker_means_us2": float(mean.var())},
        "roofline": {"bound": "hbm", "kernel": "dc_worker_totals_vec4_kernel" if r.M % 4 == 0 and (r.M <= 128 or r.M == 256)
                     else "dc_worker_totals_flat_kernel", "achieved": achieved, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": None, "kernel_ms": ms,
                     "algorithmic_bytes": 4.0 * r.elements}}))
    return 0


def scan_kernel_name(M: int, grid: str = "recipe", N: int = 0, T: int = 0, K: int = 1) -> str:
    """The streaming kernel the library runs for N rows of M elements per trial and K thresholds (16-byte aligned,
    contiguous tensor), as a profile names it."""
    p2 = 4
    while p2 <= min(K, 4095):
        p2 *= 2
    two_blocks = lambda stage_bytes: 16 * p2 + stage_bytes + 1024 <= (80 if p2 <= 1024 else 160) * 1024   # two blocks per compute unit, one with large tables
    per_lane = M // 2 if M > 16 and M % 4 == 2 else M                  # 16-byte vectors of a lane's rows
    rows_fit = two_blocks(0 if 4 % M == 0 else 4 * 64 * (per_lane | 1) * 16)
    several = (M <= 15 and M != 12) or M == 17 or (M % 4 == 2 and M <= 30)         # row lengths of which a lane holds several
    if several and rows_fit and N % (2 if M > 16 and M % 2 == 0 else 4) == 0 and N >= 256:
        return f"dc_scan_rows_kernel<{M}, false>"
    if M <= 16 and rows_fit and N >= 4 and (T * N) % 4 == 0 and M not in (1, 2, 4):
        per_load = 64 // (M // 4) if M % 4 == 0 else 0                 # the same over trials of any worker count, unless
        if per_load == 0 or (N * 100 < -(-N // per_load) * per_load * 85 and T * N * M >= 1 << 22):   # whole rows per load fill their loads well
            return f"dc_scan_rows_kernel<{M}, true>"
    inside = (N * M) % 4 == 0 and N >= 32 and N * 100 >= -(-N // 64) * 64 * 85      # chunks of 64 rows inside the trials,
    over = 4 <= N < 64 and (T * N * M) % 4 == 0                                    # or over small trials of a contiguous tensor
    if 17 <= M <= 63 and M % 4 != 0 and (M >= 25 or N < 256) and (inside or over) and two_blocks(1024 * M):
        return f"dc_scan_row_lane_kernel<{8 if M <= 32 else 12 if M <= 48 else 16}>"          # one row per lane
    if M % 4 == 0 and (M <= 128 or M == 256):
        lanes = M // 4
        known = lanes if lanes & (lanes - 1) == 0 else 0              # one instantiation serves every other lane count
        two = M in (128, 256) or (M in (32, 64) and T * N * M >= 1 << 28)   # two launch shapes; the smaller M only from 1 GiB on
        shape = 0 if not two else (1 if grid == "recipe" else 2)     # <L, 1> works on narrow grids, <L, 2> on dense ones
        return f"{SCAN_KERNEL}<{known}, {shape}>"
    return f"dc_scan_flat_kernel<{M if M < 4 else 0}>"


def time_sums_path(r, lat, taus, taus_dev, stream, steps, warmup, timing: int = 1):
    """`warmup` untimed and `steps` timed passes of the whole path (dc_simulate_async writing its 2 K sums into pinned
    host memory, the wait for the stream, dc_select_tau) on `stream`.  timing: 0 = no events in the passes, 1 = the
    library brackets its streaming kernel with HIP events, 2 = also the whole enqueued sequence.
    Returns (wall seconds, per-step ms, scan-kernel ms per step, sequence ms per step, thr, best), or None if the device
    flagged a value error."""
    import numpy as np
    import torch

    import paper_2306_10598_amd as dc
    K = taus.size
    host_out = torch.zeros((2, K), dtype=torch.int64).pin_memory()      # out_step, out_done: written by the device
    host_step, host_done = host_out[0].numpy(), host_out[1].numpy()
    ws = torch.empty(dc.dc_workspace_bytes(r.T, r.N, r.M, K), dtype=torch.uint8, device=lat.device)

    # the same call on the same tensors every step: its arguments are marshalled once (the binding's prepared calls)
    simulation = dc.PreparedSimulation(lat, taus_dev, r.comm, host_out[0], host_out[1], ws, stream)
    selection = dc.PreparedSelection(host_step, host_done, taus, r.T, r.N, r.M, 0)

    def step():
        simulation.enqueue()
        stream.synchronize()
        return selection.select()

    dc.dc_set_kernel_timing(timing)
    try:
        for _ in range(warmup):
            step()
        if dc.dc_workspace_status(ws, stream) != dc.DC_OK:
            return None
        scan_ms, seq_ms, step_ms = [], [], []
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            ts = time.perf_counter()
            thr, _, best = step()
            step_ms.append(1e3 * (time.perf_counter() - ts))
            if timing:
                a, b = dc.dc_last_kernel_ms(whole=timing >= 2)   # HIP events on the stream the kernels ran on
                scan_ms.append(a)
                if b is not None:
                    seq_ms.append(b)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    finally:
        dc.dc_set_kernel_timing(False)
    return wall, step_ms, scan_ms, seq_ms, thr, best


def other_workloads(headline: str, stream, steps: int = 10, warmup: int = 3):
    """Short runs of the same path on the remaining workloads (reported beside the headline, not part of `value`)."""
    import numpy as np
    import torch

    from dc_workloads import config, device, spec
    rows = []
    for name in spec.CONFIG_NAMES:
        if name == headline:
            continue
        r = config(name)
        lat = device.generate(r)
        taus = device.tau_grid(r, lat)
        taus_dev = torch.from_numpy(taus).to(lat.device)
        m = time_sums_path(r, lat, taus, taus_dev, stream, steps, warmup, timing=0)     # the step as a caller sees it
        e = time_sums_path(r, lat, taus, taus_dev, stream, steps, 1, timing=2) if m else None   # device-side times
        del lat
        torch.cuda.empty_cache()
        if m is None or e is None:
            rows.append({"workload": name, "error": "device reported a value error"})
            continue
        wall = m[0]
        scan_ms, seq_ms = e[2], e[3]
        rows.append({"workload": f"{name}: T={r.T} N={r.N} M={r.M} K={taus.size}", "tensor_bytes": r.nbytes,
                     "value": float(r.elements) * taus.size / (wall / steps), "unit": "evals/s",
                     "ms_per_step": 1e3 * wall / steps, "kernel_ms": float(np.mean(scan_ms)),
                     "sequence_ms": float(np.mean(seq_ms)),
                     "achieved_GBps": 4.0 * r.elements / (float(np.mean(scan_ms)) * 1e-3) / 1e9, "steps": steps})
    return rows


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="heterogeneous2048")
    ap.add_argument("--path", choices=("sums", "per-step", "analytic", "worker-moments"), default="sums",
                    help="sums: dc_simulate_async + dc_select_tau (the headline path); "
                         "per-step: dc_speedup_per_step_async, Algorithm 2's mean of per-iteration speedups; "
                         "analytic: dc_moments + dc_analytic_curves, the closed-form curves; "
                         "worker-moments: dc_worker_moments, per-worker statistics of the iteration time")
    ap.add_argument("--rows", type=int, default=0,
                    help="run the workload with this many accumulations per worker instead of its own M, the number of "
                         "trials rescaled to keep the tensor's size (not a bench line: for timing other row lengths)")
    ap.add_argument("--workers", type=int, default=0,
                    help="run the workload with this many workers instead of its own N, the number of trials rescaled to "
                         "keep the tensor's size (not a bench line: for timing small trials)")
    ap.add_argument("--thresholds", type=int, default=0,
                    help="run the workload with this many thresholds on its grid rule instead of its own K (not a bench line)")
    ap.add_argument("--grid", choices=("recipe", "dense", "upper-half"), default="recipe",
                    help="recipe: the workload's own threshold grid; dense: K thresholds from 0 to the largest worker total "
                         "(every completion time falls inside the grid); upper-half: from half the largest total to it "
                         "(not a bench line: for timing grids that cover much of the data)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true",
                    help="skip the short runs on the other workloads that are reported in `per_config`")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run a plain 4 GiB device-to-device copy instead (scale factor for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU; the library has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    ensure_built()
    import numpy as np
    import torch

    import paper_2306_10598_amd as dc
    from dc_workloads import config, device

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    if args.calibrate_copy:
        src = torch.ones(1 << 30, dtype=torch.int32, device=dev)          # 4 GiB read + 4 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": 4 << 30, "calibrate_copy_bytes_written": 4 << 30, "copies": 3}))
        return 0
    r = config(args.workload)
    if args.rows > 0 and args.rows != r.M:
        r = r.with_shape(T=max(1, r.T * r.M // args.rows), M=args.rows)
    if args.workers > 0 and args.workers != r.N:
        r = r.with_shape(T=max(1, r.T * r.N // args.workers), N=args.workers)
    if args.thresholds > 0:
        r = r.with_shape(K=args.thresholds)

    lat = device.generate(r)                                   # resident in HBM before timing starts
    taus = device.tau_grid(r, lat)
    if args.grid != "recipe":
        top = int(device.worker_totals(lat).max().item())
        taus = np.linspace(0 if args.grid == "dense" else top // 2, top, taus.size).astype(np.int64)
    K = taus.size
    taus_dev = torch.from_numpy(taus).to(dev)
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()

    if args.path == "per-step":
        return bench_per_step(args, r, lat, taus, taus_dev, stream)
    if args.path == "analytic":
        return bench_analytic(args, r, lat, taus)
    if args.path == "worker-moments":
        return bench_worker_moments(args, r, lat)

    m = time_sums_path(r, lat, taus, taus_dev, stream, args.steps, args.warmup, timing=2)
    if m is None:
        print("device reported a value error", file=sys.stderr)
        return 1
    wall, step_ms, scan_ms, seq_ms, thr, best = m

    ms_per_step = 1e3 * wall / args.steps
    evals = float(r.elements) * K
    scan_avg_ms = float(np.mean(scan_ms))
    algo_bytes = 4.0 * r.elements                              # every latency read once, nothing written back
    achieved = algo_bytes / (scan_avg_ms * 1e-3) / 1e9
    plain = args.rows <= 0 and args.workers <= 0 and args.thresholds <= 0 and args.grid == "recipe"
    traffic, traffic_source = recorded_traffic(r.name) if plain else (None, "not the workload's own shape or grid")
    line = {
        "metric": METRIC, "value": evals / (wall / args.steps), "unit": "evals/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "ms_per_step_median": float(np.median(step_ms)), "ms_per_step_min": float(np.min(step_ms)),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": f"{r.name}: T={r.T} N={r.N} M={r.M} K={K} comm={r.comm}us, {r.description}",
                   "grid": args.grid, "tensor_bytes": r.nbytes, "best_tau_us": int(taus[best]),
                   "best_thr_per_us": float(thr[best])},
        "roofline": {"bound": "hbm", "kernel": scan_kernel_name(r.M, args.grid, r.N, r.T, K), "achieved": achieved,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": traffic, "traffic_source": traffic_source,
                     "kernel_ms": scan_avg_ms, "kernel_ms_min": float(np.min(scan_ms)),
                     "sequence_ms": float(np.mean(seq_ms)),     # all kernels of a call, first to last, on the device
                     "algorithmic_bytes": algo_bytes,
                     "peak_source": "MI355X published HBM3E bandwidth; `device` holds what this GPU reports about its memory"},
        "device": {"name": torch.cuda.get_device_name(dev), **dc.dc_device_info()},
    }
    del lat
    torch.cuda.empty_cache()
    if not args.no_per_config and plain:
        line["per_config"] = other_workloads(r.name, stream)
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(r, taus)
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
