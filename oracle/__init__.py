"""CPU oracle for the DropCompute batched step-time computation (Python face of dc_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by the tests, the smoke check and the benchmark's
CPU-baseline leg.  The GPU library never imports, links or calls anything here, and this
package imports nothing of the GPU library.

  simulate(lat, taus, comm, method)  -> (step_sum[K], done_sum[K])  exact int64 sums over trials
      method="literal": the four nested loops of Appendix C.1 / Algorithm 2
      method="sorted" : same numbers via one walk over sorted thresholds (for large inputs)
  select_tau(step_sum, done_sum, taus, T, N, M, base_step_sum) -> (thr[K], s_eff[K], best_k)
      throughput N*M~/(min{tau,T}+T^c) and S_eff (Section 4.4), argmax (Algorithm 2, last line)
  per_step_speedup(lat, taus, comm) -> S_eff[K] as the mean over iterations of the per-iteration speedup
      S_i(tau) (Section 4.4's ratio taken iteration by iteration, then averaged: Algorithm 2; float64)
  per_step_best(s_eff, taus) -> index of the threshold with the largest S_eff (Algorithm 2, its final argmax)
"""
from __future__ import annotations

import ctypes
import subprocess
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_LIB_PATH = _HERE / "libdc_oracle.so"
_lib = None

OK, ERR_INVALID_ARG, ERR_NEGATIVE_LATENCY = 0, 1, 2


class OracleError(ValueError):
    def __init__(self, code: int):
        super().__init__({1: "invalid argument", 2: "negative latency"}.get(code, f"error {code}"))
        self.code = code


def build(verbose: bool = False) -> Path:
    """Compile dc_oracle.c with gcc into oracle/libdc_oracle.so."""
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", str(_LIB_PATH), str(_HERE / "dc_oracle.c")]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    global _lib
    _lib = None
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not _LIB_PATH.exists():
            build()
        lib = ctypes.CDLL(str(_LIB_PATH))
        sig = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
               ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
        for name in ("dc_oracle_simulate_literal", "dc_oracle_simulate_sorted"):
            fn = getattr(lib, name)
            fn.argtypes = sig
            fn.restype = ctypes.c_int
        lib.dc_oracle_per_step_speedup_sums.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                                        ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
        lib.dc_oracle_per_step_speedup_sums.restype = ctypes.c_int
        _lib = lib
    return _lib


def simulate(lat: np.ndarray, taus, comm: int, method: str = "literal"):
    """Exact step-time and completed-micro-batch sums per threshold.

    lat: int32 [T][N][M] microseconds.  Returns (step_sum, done_sum), int64 [K] each.
    """
    lat = np.ascontiguousarray(lat, dtype=np.int32)
    if lat.ndim != 3:
        raise OracleError(ERR_INVALID_ARG)
    T, N, M = lat.shape
    taus = np.ascontiguousarray(taus, dtype=np.int64)
    K = taus.size
    step = np.zeros(K, dtype=np.int64)
    done = np.zeros(K, dtype=np.int64)
    fn = getattr(_load(), {"literal": "dc_oracle_simulate_literal", "sorted": "dc_oracle_simulate_sorted"}[method])
    rc = fn(lat.ctypes.data, T, N, M, taus.ctypes.data, K, int(comm), step.ctypes.data, done.ctypes.data)
    if rc != OK:
        raise OracleError(rc)
    return step, done


def simulate_threaded(lat: np.ndarray, taus, comm: int, method: str = "sorted", threads: int = 1):
    """simulate() with the trials split over threads; the per-trial sums simply add."""
    T = lat.shape[0]
    threads = max(1, min(threads, T))
    if threads == 1:
        return simulate(lat, taus, comm, method)
    bounds = [T * i // threads for i in range(threads + 1)]
    with ThreadPoolExecutor(threads) as ex:
        parts = list(ex.map(lambda i: simulate(lat[bounds[i]:bounds[i + 1]], taus, comm, method), range(threads)))
    return sum(p[0] for p in parts), sum(p[1] for p in parts)


def select_tau(step_sum, done_sum, taus, T: int, N: int, M: int, base_step_sum: int = 0):
    """Throughput, effective speedup and the best threshold.

    thr[k]   = done_sum[k] / step_sum[k]         micro-batches per microsecond, all workers (Section 4.4)
    s_eff[k] = thr[k] / (T*N*M / base_step_sum)  ratio to the no-drop throughput (Section 4.4, S_eff),
               with base_step_sum = sum_i (T_i + T^c); NaN when base_step_sum == 0
    best_k   = argmax_k thr[k], compared exactly as integer cross-products; among exact
               ties the largest tau wins (fewest dropped micro-batches), then the lowest index.
    """
    step = [int(x) for x in step_sum]
    done = [int(x) for x in done_sum]
    tau = [int(x) for x in taus]
    K = len(tau)
    if K == 0 or any(s <= 0 for s in step):
        raise OracleError(ERR_INVALID_ARG)
    thr = np.array([d / s for d, s in zip(done, step)], dtype=np.float64)
    if base_step_sum > 0:
        seff = np.array([(d / s) * float(base_step_sum) / (float(T) * float(N) * float(M)) for d, s in zip(done, step)])
    else:
        seff = np.full(K, np.nan)
    best = 0
    for k in range(1, K):
        lhs, rhs = done[k] * step[best], done[best] * step[k]      # Python ints: exact
        if lhs > rhs or (lhs == rhs and tau[k] > tau[best]):
            best = k
    return thr, seff, best


def per_step_speedup(lat: np.ndarray, taus, comm, threads: int = 1):
    """Mean over iterations of the per-iteration effective speedup S_i(tau) (Section 4.4 per iteration,
    averaged as in Algorithm 2; float64).

    comm may be a scalar or one value per iteration (T_i^c).  threads > 1 splits the iterations into that many
    contiguous runs whose sums are added in order (the float additions are then grouped by run).
    """
    lat = np.ascontiguousarray(lat, dtype=np.int32)
    if lat.ndim != 3:
        raise OracleError(ERR_INVALID_ARG)
    T, N, M = lat.shape
    taus = np.ascontiguousarray(taus, dtype=np.int64)
    comm = np.ascontiguousarray(np.broadcast_to(np.asarray(comm, dtype=np.int64), (T,)))
    fn = _load().dc_oracle_per_step_speedup_sums

    def run(t0: int, t1: int) -> np.ndarray:
        part, c, out = lat[t0:t1], comm[t0:t1], np.zeros(taus.size, dtype=np.float64)
        rc = fn(part.ctypes.data, t1 - t0, N, M, taus.ctypes.data, taus.size, c.ctypes.data, out.ctypes.data)
        if rc != OK:
            raise OracleError(rc)
        return out

    threads = max(1, min(int(threads), T))
    bounds = [T * i // threads for i in range(threads + 1)]
    if threads == 1:
        sums = [run(0, T)]
    else:
        with ThreadPoolExecutor(threads) as ex:
            sums = list(ex.map(lambda i: run(bounds[i], bounds[i + 1]), range(threads)))
    total = np.zeros(taus.size, dtype=np.float64)
    for part in sums:
        total += part
    return total / float(T)


def per_step_best(s_eff, taus) -> int:
    """tau* = argmax_tau S_eff(tau), the last step of Algorithm 2, as an index into taus.

    The paper does not say which of several equal maxima is meant; as in select_tau the largest tau wins
    (fewest dropped micro-batches), then the lowest index.
    """
    s_eff = [float(x) for x in s_eff]
    tau = [int(x) for x in taus]
    if not tau or len(s_eff) != len(tau) or any(x != x for x in s_eff):
        raise OracleError(ERR_INVALID_ARG)
    best = 0
    for k in range(1, len(tau)):
        if s_eff[k] > s_eff[best] or (s_eff[k] == s_eff[best] and tau[k] > tau[best]):
            best = k
    return best


# ---- analytical model (Sections 4.2-4.4, Appendix C.2) ---------------------------------------------------

EULER_GAMMA = 0.5772156649015329


def moments(lat: np.ndarray):
    """Exact (count, sum, sum of squares) of all latencies as Python ints, and (mean, variance) as floats.

    mu and sigma^2 are the single-micro-batch statistics that the closed forms of Section 4.2-4.3 take
    (population variance, one distribution for all workers: Appendix C.2, first assumption).
    """
    flat = np.ascontiguousarray(lat, dtype=np.int64).reshape(-1)
    if flat.size == 0 or (flat < 0).any():
        raise OracleError(ERR_INVALID_ARG if flat.size == 0 else ERR_NEGATIVE_LATENCY)
    n, s, q = int(flat.size), 0, 0
    for start in range(0, n, 1 << 20):                      # chunks small enough that int64 squares cannot overflow a sum
        part = flat[start:start + (1 << 20)]
        s += int(part.sum())
        hi, lo = part >> 16, part & 0xFFFF                  # x^2 = hi^2*2^32 + 2*hi*lo*2^16 + lo^2, each sum < 2^63
        q += (int((hi * hi).sum()) << 32) + (int((hi * lo).sum()) << 17) + int((lo * lo).sum())
    mean = s / n
    variance = (q * n - s * s) / (n * n)
    return n, s, q, mean, variance


def analytic_curves(mu: float, sigma2: float, N: int, M: int, taus, comm: int, mean_tmax: float | None = None):
    """Closed-form estimates from (mu, sigma^2) of one micro-batch latency.

    e_done[k] = sum_{m=1..M} Phi((tau_k - m mu) / sqrt(m sigma^2))        expected completed micro-batches per
                                                                          worker (Section 4.3, CLT estimate of M~)
    e_t       = sqrt(M sigma^2) ((1-g) PhiInv(1 - 1/N) + g PhiInv(1 - 1/(e N))) + M mu
                                                                          expected compute time of the slowest of N
                                                                          workers (Section 4.2; compute only, N >= 2)
    s_eff[k]  = e_done[k]/M * (ET + T^c) / (min(tau_k, ET) + T^c)         Section 4.4's S_eff with the estimates plugged
                in; ET = mean_tmax when given ("analytical given E[T]", Appendix C.2), else e_t.  T^c is added
                to ET in the numerator because T = max_n T_n excludes T^c in Sections 4.2-4.4.
    best_k    = argmax_k e_done[k] / (tau_k + T^c)                        Appendix C.2, "Finding tau*"; ties: largest tau
    """
    from scipy.special import ndtr, ndtri
    taus = np.asarray(taus, dtype=np.int64)
    if N < 2 or M < 1 or sigma2 < 0 or comm < 0 or (taus < 0).any():
        raise OracleError(ERR_INVALID_ARG)
    m = np.arange(1, M + 1, dtype=np.float64)
    e_done = np.empty(taus.size, dtype=np.float64)
    for k, tau in enumerate(taus):
        if sigma2 > 0:
            e_done[k] = ndtr((float(tau) - m * mu) / np.sqrt(m * sigma2)).sum()
        else:
            e_done[k] = float(np.count_nonzero(m * mu < float(tau)))
    z = (1 - EULER_GAMMA) * ndtri(1 - 1 / N) + EULER_GAMMA * ndtri(1 - 1 / (np.e * N))
    e_t = float(np.sqrt(M * sigma2) * z + M * mu)
    et = e_t if mean_tmax is None else float(mean_tmax)
    tau_f = taus.astype(np.float64)
    s_eff = e_done / M * (et + comm) / (np.minimum(tau_f, et) + comm)
    score = e_done / (tau_f + comm)
    best = 0
    for k in range(1, taus.size):
        if score[k] > score[best] or (score[k] == score[best] and taus[k] > taus[best]):
            best = k
    return e_done, e_t, s_eff, best


def worker_moments(lat: np.ndarray):
    """Per worker n: exact sum and sum of squares over iterations of its compute time T_n = sum_m t_n^(m)
    (Python ints), and mean / population variance as float arrays.  These are the per-worker statistics behind
    the "simulation" curve of the paper's iteration-time figure (each worker's T_n redrawn from a normal
    distribution with that worker's empirical mean and variance; Section 4.3).
    """
    lat = np.ascontiguousarray(lat, dtype=np.int64)
    if lat.ndim != 3 or lat.size == 0:
        raise OracleError(ERR_INVALID_ARG)
    if (lat < 0).any():
        raise OracleError(ERR_NEGATIVE_LATENCY)
    T, N, _ = lat.shape
    totals = lat.sum(axis=2)                                   # [T][N], each < 2^63
    sums = [int(x) for x in totals.sum(axis=0)]
    if int(totals.max()) < (1 << 32) and T < (1 << 30):
        # x^2 = hi^2 2^32 + 2 hi lo 2^16 + lo^2 with 16-bit halves: every column sum stays below 2^63, so the
        # int64 sums are exact and the squares are assembled as Python ints
        hi, lo = totals >> 16, totals & 0xFFFF
        hh, hl, ll = (hi * hi).sum(axis=0), (hi * lo).sum(axis=0), (lo * lo).sum(axis=0)
        squares = [(int(a) << 32) + (int(b) << 17) + int(c) for a, b, c in zip(hh, hl, ll)]
    else:
        squares = [sum(int(v) * int(v) for v in totals[:, n]) for n in range(N)]
    mean = np.array([s / T for s in sums], dtype=np.float64)
    var = np.array([(q * T - s * s) / (T * T) for s, q in zip(sums, squares)], dtype=np.float64)
    return sums, squares, mean, var
