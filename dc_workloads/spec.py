"""Seeded synthetic micro-batch latency workloads: the specification.

This module defines WHAT the synthetic latency tensors are; `host.py` and
`device.py` produce them (on CPU and in HBM).  It holds none of the simulated
method's arithmetic: no prefix sums, no threshold counting, no step times.

The paper's recorded per-micro-batch timings t_{i,n}^{(m)} (Appendix C.1,
Algorithm 2 inputs) are not public, so every tensor here is a synthetic
stand-in with the paper's shapes: I iterations x N workers x M accumulations,
noise families as in Appendix B.1 / C.3 (log-normal, normal, exponential,
Bernoulli stragglers).

Generator definition (integer-only, so a CPU and a GPU implementation can be
bit-identical):

  mix64(z)         : z ^= z>>30; z *= 0xBF58476D1CE4E5B9; z ^= z>>27;
                     z *= 0x94D049BB133111EB; z ^= z>>31       (mod 2^64)
  key(seed,stream) = mix64(seed + GOLDEN*(stream+1))
  h(seed,stream,i) = mix64(key(seed,stream) + GOLDEN*(i+1))     GOLDEN=0x9E3779B97F4A7C15

  A distribution is a quantile function tabulated in fixed point (8 fractional
  bits, "q8") at three knot sets:
    main[c], c=0..65536          at u = c/2^16
    lo[j],   j=0..4096           at u = j/2^24                  (cells 0..15 refined)
    hi[j],   j=0..4096           at u = (65520*256 + j)/2^24    (cells 65520..65535 refined)
  with u=0 and u=1 replaced by 2^-30 and 1-2^-30.  A 64-bit hash h draws
    cell = h>>48, f = (h>>16) & 0xFFFFFFFF
    16 <= cell < 65520 : q = main[cell] + ((main[cell+1]-main[cell])*f >> 32)
    cell < 16          : j = cell*256 + (f>>24), g = f & 0xFFFFFF
                         q = lo[j] + ((lo[j+1]-lo[j])*g >> 24)
    cell >= 65520      : j = (cell-65520)*256 + (f>>24), g likewise, table hi.

  Element i = (t*N + n)*M + m of a workload:
    q      = draw(h(seed, 0, i))                                  (q8 microseconds)
    spike  = (h(seed, 1, i) >> 32) < spike_thresh   and, when spike_workers > 0, only for workers n < spike_workers
    mul    = spike ? spike_mul : 1
    v      = ((q * scale_q16[n] * mul + 2^23) >> 24) + worker_add[n]   (round half up; worker_add defaults to 0)
    lat[i] = max(clip_min, v) + add + (spike ? spike_add : 0)
  scale_q16[n] = 65536 (no per-worker slowdown) or
                 65536 + ((draw_scale(h(seed, 2, n)) + 128) >> 8), or explicit per-worker values.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Optional

import numpy as np
from scipy.special import ndtri

GOLDEN = 0x9E3779B97F4A7C15
MIX_A = 0xBF58476D1CE4E5B9
MIX_B = 0x94D049BB133111EB
MASK64 = (1 << 64) - 1

MAIN_CELLS = 1 << 16
TAIL_CELLS = 16            # refined cells at each end of the main table
TAIL_SUB = 256             # sub-cells per refined cell
TAIL_KNOTS = TAIL_CELLS * TAIL_SUB + 1
U_EPS = 2.0 ** -30

STREAM_VALUE = 0
STREAM_SPIKE = 1
STREAM_WORKER = 2


def mix64_int(z: int) -> int:
    """mix64 on a Python int (reference for scalars)."""
    z &= MASK64
    z ^= z >> 30
    z = (z * MIX_A) & MASK64
    z ^= z >> 27
    z = (z * MIX_B) & MASK64
    z ^= z >> 31
    return z


def stream_key(seed: int, stream: int) -> int:
    return mix64_int(seed + GOLDEN * (stream + 1))


@dataclass(frozen=True)
class QuantileTables:
    """Fixed-point (q8) quantile knots of one distribution."""
    main: np.ndarray   # int64 [65537]
    lo: np.ndarray     # int64 [4097]
    hi: np.ndarray     # int64 [4097]


def quantile_tables(qfun: Callable[[np.ndarray], np.ndarray]) -> QuantileTables:
    """Tabulate `qfun` (u in (0,1) -> value, float64) into q8 integer knots.

    Knots are clamped to >= 0 and made non-decreasing, so every interpolated
    draw is a non-negative integer and all generator arithmetic is unsigned.
    """
    def knots(u: np.ndarray) -> np.ndarray:
        u = np.clip(u, U_EPS, 1.0 - U_EPS)
        q = np.rint(np.asarray(qfun(u), dtype=np.float64) * 256.0)
        q = np.maximum(q, 0.0).astype(np.int64)
        return np.maximum.accumulate(q)

    c = np.arange(MAIN_CELLS + 1, dtype=np.float64)
    j = np.arange(TAIL_KNOTS, dtype=np.float64)
    main = knots(c / MAIN_CELLS)
    lo = knots(j / (MAIN_CELLS * TAIL_SUB))
    hi = knots(((MAIN_CELLS - TAIL_CELLS) * TAIL_SUB + j) / (MAIN_CELLS * TAIL_SUB))
    # the refined tables meet the main table at the same knot values
    lo[-1] = main[TAIL_CELLS]
    hi[0] = main[MAIN_CELLS - TAIL_CELLS]
    lo = np.maximum.accumulate(np.minimum(lo, lo[-1]))
    hi = np.maximum.accumulate(np.maximum(hi, hi[0]))
    # difference * fraction stays below 2^63 (the main table is only used in cells 16 .. 65519)
    used = main[TAIL_CELLS:MAIN_CELLS - TAIL_CELLS + 1]
    for tab, frac_bits in ((used, 32), (lo, 24), (hi, 24)):
        assert tab.min() >= 0 and tab.max() < (1 << 38)
        assert np.diff(tab).max(initial=0) < (1 << (63 - frac_bits))
    return QuantileTables(main=main, lo=lo, hi=hi)


# ---- quantile functions of the families the workloads use -------------------------------

def q_exponential(mean: float):
    return lambda u: -mean * np.log1p(-u)


def q_normal(mu: float, sigma: float):
    return lambda u: mu + sigma * ndtri(u)


def q_lognormal(mu_log: float, sigma_log: float):
    return lambda u: np.exp(mu_log + sigma_log * ndtri(u))


def q_uniform(a: float, b: float):
    return lambda u: a + (b - a) * u


def prob_to_thresh(p: float) -> int:
    """Bernoulli(p) as a 32-bit threshold on the top half of the spike hash."""
    return int(round(p * 4294967296.0))


@dataclass(frozen=True)
class Recipe:
    """Everything that fixes one latency tensor and its threshold grid."""
    name: str
    T: int
    N: int
    M: int
    K: int
    comm: int                      # fixed all-reduce / serial time T^c, microseconds
    grid: str                      # "minmax" or "pct" (see tau_grid)
    value: QuantileTables
    seed: int = 0
    add: int = 0
    clip_min: int = 0
    spike_thresh: int = 0
    spike_mul: int = 1
    spike_add: int = 0
    spike_workers: int = 0         # > 0: only the first spike_workers workers can spike (stragglers of one server)
    worker_scale: Optional[QuantileTables] = None   # q8 tables of 65536*(s_n - 1)
    worker_scale_values: Optional[tuple] = None     # explicit scale_q16[n] (uint32) instead of drawn ones
    worker_add: Optional[tuple] = None              # explicit per-worker offsets in microseconds (may be negative)
    description: str = ""

    @property
    def elements(self) -> int:
        return self.T * self.N * self.M

    @property
    def nbytes(self) -> int:
        return 4 * self.elements

    def with_shape(self, T=None, N=None, M=None, K=None, seed=None) -> "Recipe":
        """Same distribution, different sizes (for small parity cases)."""
        from dataclasses import replace
        return replace(self,
                       T=self.T if T is None else T, N=self.N if N is None else N,
                       M=self.M if M is None else M, K=self.K if K is None else K,
                       seed=self.seed if seed is None else seed)


def tau_grid(totals_sorted_lo_hi: tuple[int, int], K: int) -> np.ndarray:
    """K thresholds evenly spaced over [lo, hi]: tau_k = lo + floor((hi-lo)*k/(K-1))."""
    lo, hi = int(totals_sorted_lo_hi[0]), int(totals_sorted_lo_hi[1])
    if K == 1:
        return np.array([hi], dtype=np.int64)
    return np.array([lo + ((hi - lo) * k) // (K - 1) for k in range(K)], dtype=np.int64)


def grid_rank_indices(count: int, rule: str) -> tuple[int, int]:
    """Positions, in the ascending-sorted per-worker totals, of the grid's ends.

    "minmax": smallest and largest total.  "pct": nearest-rank 1st and 99.9th
    percentile, sorted[floor((count-1)/100)] and sorted[floor((count-1)*999/1000)].
    """
    if rule == "minmax":
        return 0, count - 1
    if rule == "pct":
        return (count - 1) // 100, ((count - 1) * 999) // 1000
    raise ValueError(f"unknown grid rule {rule!r}")


# ---- the five workloads ----------------------------------------------------------------

_cache: dict[str, Recipe] = {}


def _build(name: str) -> Recipe:
    import math
    if name == "tiny":
        return Recipe(name, T=1000, N=8, M=16, K=64, comm=20000, grid="minmax",
                      value=quantile_tables(q_exponential(10000.0)), add=100000,
                      description="100000 + round(Exp(mean 10000)) us")
    if name == "lognormal64":
        return Recipe(name, T=10000, N=64, M=32, K=128, comm=30000, grid="pct",
                      value=quantile_tables(q_lognormal(math.log(120000.0), 0.1)),
                      description="round(LogNormal(ln 120000, 0.1)) us, iid")
    if name == "additive200":
        return Recipe(name, T=10000, N=200, M=64, K=128, comm=50000, grid="pct",
                      value=quantile_tables(q_normal(150000.0, 15000.0)), clip_min=1,
                      spike_thresh=prob_to_thresh(0.01), spike_add=600000,
                      description="max(1, 150000 + round(N(0,15000^2))) us, +600000 us w.p. 0.01")
    if name == "extrapolation2048":
        return Recipe(name, T=4096, N=2048, M=128, K=256, comm=80000, grid="pct",
                      value=quantile_tables(q_normal(100000.0, 10000.0)), clip_min=1,
                      description="max(1, round(N(100000,10000^2))) us")
    if name == "heterogeneous2048":
        return Recipe(name, T=16384, N=2048, M=256, K=512, comm=80000, grid="pct",
                      value=quantile_tables(q_lognormal(math.log(100000.0), 0.15)),
                      spike_thresh=prob_to_thresh(0.005), spike_mul=5,
                      worker_scale=quantile_tables(q_exponential(0.05 * 65536.0)),
                      description="round(s_n * LogNormal(ln 100000, 0.15) * (5 w.p. 0.005)) us, "
                                  "s_n = 1 + Exp(mean 0.05) per worker")
    raise KeyError(name)


CONFIG_NAMES = ("tiny", "lognormal64", "additive200", "extrapolation2048", "heterogeneous2048")


def config(name: str) -> Recipe:
    if name not in _cache:
        _cache[name] = _build(name)
    return _cache[name]
