#!/usr/bin/env python3
"""Scale sweep with the paper's additive-noise models (Appendix B.1 and C.3) on one GPU.

For each noise family it generates ONE tensor of synthetic latencies in HBM with the largest worker count, and for
each worker count N simulates the first N workers of it in place (dc_simulate's worker range: no copy), runs
dc_worker_moments, dc_select_tau and dc_analytic_curves and prints
  E[T]/E[T_i]   mean iteration time of N workers over the mean time of one worker (the ratio the appendix tabulates;
                the appendix does not state its N, so the sweep shows where each tabulated value would fall),
  tau*, S_eff(tau*), the completed fraction at tau*, and the closed-form S_eff at the same tau.

With --local-sgd it sweeps the synchronisation period of Local-SGD with random stragglers (Appendix B.3): throughput of
Local-SGD, and of Local-SGD with the best drop threshold, relative to synchronising at every step.

  python -m paper_2306_10598_amd.examples.noise_study [--families lognormal normal ...] [--workers 8 64 512 2048] [--variance 0.05 | --variances 0.05 0.1 0.2 0.3] [--delay]
  python -m paper_2306_10598_amd.examples.noise_study --local-sgd [--periods 1 2 4 8 16 32]

With --surrogate it repeats the check of the paper's iteration-time figure: measure every worker's mean and variance
of its iteration time (dc_worker_moments), redraw each T_n from a normal distribution with those moments, and compare
the mean iteration time and the speedup curve of the surrogate with those of the original latencies.

  python -m paper_2306_10598_amd.examples.noise_study --surrogate [--workers 200]
"""
from __future__ import annotations

import argparse
import sys
from pathlib import Path

ROOT = Path(__file__).resolve().parents[2]
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

PAPER_RATIO = {"lognormal": 1.496, "normal": 1.302, "bernoulli": 1.283, "exponential": 1.386, "gamma": 1.39}
BIG = 1 << 40


def sweep(recipe, workers):
    """One tensor with recipe.N workers in HBM; for each n in `workers` (n <= recipe.N) the first n workers of every
    iteration are simulated in place.  Returns one dict per n:
      ratio          E[T]/E[T_i]: mean iteration time of n workers over the mean iteration time of one worker
      tau, seff      the best threshold of the workload's grid rule applied to these n workers, and S_eff there
      completed      completed fraction of micro-batches at tau
      analytic_seff  the closed-form S_eff at tau, given the measured mean iteration time"""
    import numpy as np

    import paper_2306_10598_amd as dc
    from dc_workloads import device, spec
    lat = device.generate(recipe)
    T, M = recipe.T, recipe.M
    _, _, mean, var = dc.dc_moments(lat)                         # one micro-batch, all workers alike
    rows = []
    for n in workers:
        totals = lat[:, :n, :].sum(dim=2, dtype=__import__("torch").int64).reshape(-1)     # grid placement only
        i_lo, i_hi = spec.grid_rank_indices(totals.numel(), recipe.grid)
        ordered = totals.sort().values
        taus = np.append(spec.tau_grid((int(ordered[i_lo].item()), int(ordered[i_hi].item())), recipe.K), BIG)
        step, done = dc.dc_simulate(lat, taus, recipe.comm, workers=(0, n))
        sums, _, _, _ = dc.dc_worker_moments(lat, workers=(0, n))
        base = int(step[-1])
        thr, seff, best = dc.dc_select_tau(step, done, taus, T, n, M, base)
        mean_tmax = (base - T * recipe.comm) / T
        one_worker = sum(sums) / (T * n)
        ana = dc.dc_analytic_curves(mean, var, max(n, 2), M, taus, recipe.comm, mean_tmax)[2]
        rows.append({"workers": n, "ratio": mean_tmax / one_worker, "tau": int(taus[best]), "seff": float(seff[best]),
                     "completed": float(done[best]) / (T * n * M), "analytic_seff": float(ana[best])})
    return rows


def local_sgd_study(periods, trials: int) -> None:
    import numpy as np

    import paper_2306_10598_amd as dc
    from dc_workloads import device, noise
    print(f"{'scenario':<15}{'period':>7}{'local-SGD':>11}{'+ threshold':>13}{'tau* us':>10}{'dropped':>9}")
    for scenario in ("uniform", "single_server"):
        sync = None
        for H in periods:
            r = noise.local_sgd(trials, H, scenario)
            lat = device.generate(r)
            taus = np.append(device.tau_grid(r, lat), BIG)
            step, done = dc.dc_simulate(lat, taus, r.comm)
            thr, _, best = dc.dc_select_tau(step, done, taus, r.T, r.N, r.M, int(step[-1]))
            if sync is None:                                     # period 1, no threshold: synchronous training
                one = noise.local_sgd(trials, 1, scenario)
                s1, d1 = dc.dc_simulate(device.generate(one), [BIG], one.comm)
                sync = float(d1[0]) / float(s1[0])
            print(f"{scenario:<15}{H:>7}{thr[-1] / sync:>11.3f}{thr[best] / sync:>13.3f}{int(taus[best]):>10}"
                  f"{1 - float(done[best]) / (r.T * r.N * r.M):>9.3f}")


def surrogate_study(N: int, trials: int) -> None:
    import numpy as np

    import paper_2306_10598_amd as dc
    from dc_workloads import config, device, noise
    r = config("heterogeneous2048").with_shape(T=trials, N=N, M=64, K=16)
    lat = device.generate(r)
    taus = np.append(device.tau_grid(r, lat), BIG)
    step, done = dc.dc_simulate(lat, taus, r.comm)
    _, _, mean, var = dc.dc_worker_moments(lat)
    s = noise.per_worker_normal(trials, mean, np.sqrt(var), comm_us=r.comm)
    s_step, _ = dc.dc_simulate(device.generate(s), taus, r.comm)
    print(f"workers {N}, {trials} iterations, worker means {mean.min() / 1e6:.2f}..{mean.max() / 1e6:.2f} s")
    print(f"mean iteration time: measured {(step[-1] / trials - r.comm) / 1e6:.4f} s, "
          f"per-worker normal surrogate {(s_step[-1] / trials - r.comm) / 1e6:.4f} s")
    print(f"{'tau us':>10}{'step speedup':>14}{'surrogate':>11}{'completed':>11}")
    for k in range(taus.size - 1):
        print(f"{int(taus[k]):>10}{step[-1] / step[k]:>14.4f}{s_step[-1] / s_step[k]:>11.4f}"
              f"{done[k] / (trials * N * r.M):>11.4f}")


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--families", nargs="*", default=["lognormal", "normal", "bernoulli", "exponential", "gamma"])
    ap.add_argument("--workers", nargs="*", type=int, default=[8, 32, 128, 512, 2048])
    ap.add_argument("--variance", type=float, default=0.05)
    ap.add_argument("--variances", nargs="*", type=float, default=None,
                    help="sweep the noise variance (s^2) as well, as the appendix's second table does (overrides --variance)")
    ap.add_argument("--elements", type=int, default=1 << 28, help="approximate T*N*M of the tensor (N = the largest worker count)")
    ap.add_argument("--delay", action="store_true", help="also sweep the simulated-delay model of Appendix B.1")
    ap.add_argument("--local-sgd", action="store_true", help="sweep Local-SGD's synchronisation period instead")
    ap.add_argument("--surrogate", action="store_true", help="per-worker normal surrogate of the iteration time")
    ap.add_argument("--periods", nargs="*", type=int, default=[1, 2, 4, 8, 16, 32])
    args = ap.parse_args()
    if args.surrogate:
        surrogate_study(args.workers[0] if len(args.workers) == 1 else 200, trials=4000)
        return 0
    if args.local_sgd:
        local_sgd_study(args.periods, trials=20000)
        return 0
    from dc_workloads import noise
    print(f"{'noise':<16}{'var s^2':>8}{'N':>6}{'T':>8}{'E[T]/E[T_i]':>13}{'paper':>8}{'tau* us':>12}{'S_eff':>8}{'done':>8}{'closed form':>13}")
    top = max(args.workers)
    T = max(16, args.elements // (top * 12))
    for family in args.families + (["delay"] if args.delay else []):
        for variance in ([args.variance] if args.variances is None or family == "delay" else args.variances):
            r = noise.simulated_delay(T, top) if family == "delay" else noise.additive_noise(family, T, top, variance)
            ref = PAPER_RATIO.get(family) if abs(variance - 0.05) < 1e-12 else None
            shown = "-" if family == "delay" else f"{variance:g}"
            for row in sweep(r, sorted(args.workers)):
                print(f"{family:<16}{shown:>8}{row['workers']:>6}{T:>8}{row['ratio']:>13.3f}{(f'{ref:.3f}' if ref else '-'):>8}"
                      f"{row['tau']:>12}{row['seff']:>8.3f}{row['completed']:>8.3f}{row['analytic_seff']:>13.3f}", flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
