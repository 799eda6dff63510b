"""Workloads with the paper's own additive-noise models (synthetic; same integer generator as spec.py).

  simulated_delay(...)   Appendix B.1: every accumulation takes t + mu*eps, eps = min(Z/alpha, beta),
                         Z ~ LogNormal(4, 1), alpha = 2 e^4.5, beta = 5.5 (mean x1.5, at most x6.5).
                         The undisturbed compute time t is taken constant (= mu); the appendix does not give
                         its distribution.
  local_sgd(...)         Appendix B.3: Local-SGD with periodic synchronisation; the threshold is checked at each local
                         step, so a "micro-batch" is one local step and M is the synchronisation period.  At each
                         local step a worker is a straggler with a 4% chance and then waits 1 s; either every worker
                         can straggle ("uniform") or only the workers of one server ("single_server").  The
                         undisturbed local-step time is not given in the appendix; 0.25 s is assumed.
  per_worker_normal(...) Section 4.3 (iteration-time figure, "simulation" curve): every worker's iteration time T_n is
                         drawn from a normal distribution with that worker's own mean and standard deviation; one
                         "micro-batch" per worker (M = 1).
  additive_noise(...)    Appendix C.3: 12 accumulations of 0.45 s + eps, eps of mean 0.225 s and a chosen
                         variance from one of five families (lognormal, normal, bernoulli, exponential, gamma),
                         parameters derived from (mean, variance) as in the appendix's tables.
Input preparation only; nothing of the simulated method is computed here.
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import gammaincinv, ndtri

from .spec import Recipe, prob_to_thresh, quantile_tables

FAMILIES = ("lognormal", "normal", "bernoulli", "exponential", "gamma")


def simulated_delay(T: int, N: int, M: int = 12, base_us: int = 450_000, K: int = 128, comm_us: int = 100_000,
                    seed: int = 0) -> Recipe:
    alpha, beta = 2.0 * math.exp(4.5), 5.5

    def q(u):
        eps = np.minimum(np.exp(4.0 + ndtri(u)) / alpha, beta)
        return base_us * (1.0 + eps)

    return Recipe("simulated_delay", T=T, N=N, M=M, K=K, comm=comm_us, grid="pct", value=quantile_tables(q), seed=seed,
                  description=f"round({base_us} * (1 + min(LogNormal(4,1)/(2e^4.5), 5.5))) us")


def noise_parameters(family: str, mean: float, variance: float) -> dict:
    """Distribution parameters (seconds) that give the requested mean and variance."""
    if family == "lognormal":
        s2 = math.log(1.0 + variance / mean ** 2)
        return {"mu_log": math.log(mean) - s2 / 2.0, "sigma_log": math.sqrt(s2)}
    if family == "normal":
        return {"mu": mean, "sigma": math.sqrt(variance)}
    if family == "bernoulli":                       # a * Br(p): mean a p, variance a^2 p (1-p)
        p = mean ** 2 / (variance + mean ** 2)
        return {"amplitude": mean / p, "p": p}
    if family == "exponential":                     # one parameter: the appendix matches the variance (rate 1/sqrt(var))
        return {"rate": 1.0 / math.sqrt(variance)}
    if family == "gamma":
        return {"shape": mean ** 2 / variance, "rate": mean / variance}
    raise ValueError(family)


def additive_noise(family: str, T: int, N: int, variance: float = 0.05, mean: float = 0.225, M: int = 12,
                   base_s: float = 0.45, K: int = 128, comm_us: int = 100_000, seed: int = 0) -> Recipe:
    """Accumulations of base_s + eps seconds, in integer microseconds; eps >= -base_s (latencies stay >= 0)."""
    prm = noise_parameters(family, mean, variance)
    base_us = base_s * 1e6
    kw = {}
    if family == "lognormal":
        q = lambda u: base_us + 1e6 * np.exp(prm["mu_log"] + prm["sigma_log"] * ndtri(u))
    elif family == "normal":
        q = lambda u: base_us + 1e6 * (prm["mu"] + prm["sigma"] * ndtri(u))
    elif family == "bernoulli":                     # exact two-point law through the spike mechanism
        q = lambda u: np.full_like(u, base_us)
        kw = {"spike_thresh": prob_to_thresh(prm["p"]), "spike_add": int(round(prm["amplitude"] * 1e6))}
    elif family == "exponential":
        q = lambda u: base_us - 1e6 * np.log1p(-u) / prm["rate"]
    else:
        q = lambda u: base_us + 1e6 * gammaincinv(prm["shape"], u) / prm["rate"]
    # a worker's total must stay below 2^31 us: the far tail of the widest log-normal (beyond 1 - 1e-9) is cut there
    cap = float((2**31 - 1) // M - kw.get("spike_add", 0) - 1)
    return Recipe(f"additive_{family}", T=T, N=N, M=M, K=K, comm=comm_us, grid="pct",
                  value=quantile_tables(lambda u: np.minimum(q(u), cap)), seed=seed,
                  description=f"{base_s} s + {family} noise (mean {mean} s, variance {variance} s^2), us", **kw)


def local_sgd(T: int, period: int, scenario: str = "uniform", N: int = 32, step_us: int = 250_000,
              straggler_p: float = 0.04, wait_us: int = 1_000_000, server_workers: int = 8, K: int = 64,
              comm_us: int = 50_000, seed: int = 0) -> Recipe:
    if scenario not in ("uniform", "single_server"):
        raise ValueError(scenario)
    return Recipe(f"local_sgd_{scenario}", T=T, N=N, M=period, K=K, comm=comm_us, grid="minmax",
                  value=quantile_tables(lambda u: np.full_like(u, float(step_us))), seed=seed,
                  spike_thresh=prob_to_thresh(straggler_p), spike_add=wait_us,
                  spike_workers=server_workers if scenario == "single_server" else 0,
                  description=f"{step_us} us per local step, +{wait_us} us w.p. {straggler_p} "
                              f"({'workers of one server' if scenario == 'single_server' else 'any worker'})")


def per_worker_normal(T: int, mean_us, sd_us, K: int = 128, comm_us: int = 0, seed: int = 0) -> Recipe:
    """T_n ~ Normal(mean_us[n], sd_us[n]^2), clipped at 0, M = 1.  The shared table holds (z + 8) * 1024 and each
    worker scales it by sd/1024 and shifts it by mean - 8 sd, all in integers."""
    mean_us = np.asarray(mean_us, dtype=np.float64)
    sd_us = np.asarray(sd_us, dtype=np.float64)
    if mean_us.shape != sd_us.shape or mean_us.ndim != 1 or (sd_us < 0).any() or (sd_us * 64 >= 2**32).any():
        raise ValueError("mean_us and sd_us must be vectors of equal length, 0 <= sd < 2^26 us")
    scale = np.rint(sd_us * 64.0).astype(np.uint32)                       # q16 of sd/1024
    shift = np.rint(mean_us - 8.0 * scale.astype(np.float64) / 64.0).astype(np.int64)
    return Recipe("per_worker_normal", T=T, N=mean_us.size, M=1, K=K, comm=comm_us, grid="pct",
                  value=quantile_tables(lambda u: (ndtri(u) + 8.0) * 1024.0), seed=seed,
                  worker_scale_values=tuple(int(v) for v in scale), worker_add=tuple(int(v) for v in shift),
                  description="T_n ~ Normal(mean_n, sd_n^2) per worker, us")
