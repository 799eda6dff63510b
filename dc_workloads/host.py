"""CPU generation of the synthetic latency workloads (see spec.py for the definition).

Two implementations of the same integer recipe: a vectorised NumPy one (the readable
reference, slow) and a C one (fast, called through ctypes, threaded over chunks here).
Input preparation only: the per-worker totals computed here exist solely to place the
threshold grid the way each workload's recipe says (percentiles of those totals).
"""
from __future__ import annotations

import ctypes
import os
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

import numpy as np

from . import spec
from .spec import GOLDEN, MIX_A, MIX_B, Recipe, QuantileTables

_HERE = Path(__file__).resolve().parent
_LIB_PATH = _HERE / "libdcgen_host.so"
_lib = None


def build(verbose: bool = False) -> Path:
    """Compile the C generator with gcc into dc_workloads/libdcgen_host.so."""
    import subprocess
    src = _HERE / "csrc" / "gen_host.c"
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", str(_LIB_PATH), str(src)]
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
        p = ctypes.c_void_p
        lib.dcgen_fill_host.argtypes = [p, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64,
                                        ctypes.c_int64, ctypes.c_int64, p, p, p, p, p,
                                        ctypes.c_int64, ctypes.c_int64,
                                        ctypes.c_uint32, ctypes.c_uint32, ctypes.c_int64, ctypes.c_int64]
        lib.dcgen_fill_host.restype = None
        lib.dcgen_draw_host.argtypes = [p, p, ctypes.c_uint64, ctypes.c_uint64, p, p, p]
        lib.dcgen_draw_host.restype = None
        _lib = lib
    return _lib


def cpu_threads() -> int:
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = os.cpu_count() or 1
    return max(1, min(16, n))


# ---- NumPy reference -------------------------------------------------------------------

def mix64(z: np.ndarray) -> np.ndarray:
    z = z.astype(np.uint64, copy=True)
    z ^= z >> np.uint64(30)
    z *= np.uint64(MIX_A)
    z ^= z >> np.uint64(27)
    z *= np.uint64(MIX_B)
    z ^= z >> np.uint64(31)
    return z


def hash_counters(seed: int, stream: int, counters: np.ndarray) -> np.ndarray:
    key = np.uint64(spec.stream_key(seed, stream))
    with np.errstate(over="ignore"):
        return mix64(key + np.uint64(GOLDEN) * (counters.astype(np.uint64) + np.uint64(1)))


def draw_q8(h: np.ndarray, tab: QuantileTables) -> np.ndarray:
    """Table-interpolated quantile draw, q8 fixed point, from 64-bit hashes."""
    h = h.astype(np.uint64)
    cell = (h >> np.uint64(48)).astype(np.int64)
    f = (h >> np.uint64(16)) & np.uint64(0xFFFFFFFF)
    out = np.empty(h.shape, dtype=np.uint64)
    mid = (cell >= 16) & (cell < 65520)
    main = tab.main.astype(np.uint64)
    a, b = main[cell[mid]], main[cell[mid] + 1]
    out[mid] = a + (((b - a) * f[mid]) >> np.uint64(32))
    for sel, table, base in ((cell < 16, tab.lo, 0), (cell >= 65520, tab.hi, 65520)):
        if not sel.any():
            continue
        t = table.astype(np.uint64)
        j = (cell[sel] - base) * 256 + (f[sel] >> np.uint64(24)).astype(np.int64)
        g = f[sel] & np.uint64(0xFFFFFF)
        a, b = t[j], t[j + 1]
        out[sel] = a + (((b - a) * g) >> np.uint64(24))
    return out


def worker_scale_q16(r: Recipe) -> np.ndarray | None:
    """Per-worker slowdown s_n in q16 fixed point, or None when every s_n = 1."""
    if r.worker_scale_values is not None:
        return np.asarray(r.worker_scale_values, dtype=np.uint32)
    if r.worker_scale is None:
        return None
    q = draw_q8(hash_counters(r.seed, spec.STREAM_WORKER, np.arange(r.N, dtype=np.uint64)), r.worker_scale)
    return (np.uint64(65536) + ((q + np.uint64(128)) >> np.uint64(8))).astype(np.uint32)


def generate_numpy(r: Recipe, idx0: int = 0, count: int | None = None) -> np.ndarray:
    """Elements idx0..idx0+count of the flat [T][N][M] tensor, NumPy reference."""
    count = r.elements - idx0 if count is None else count
    i = np.arange(idx0, idx0 + count, dtype=np.uint64)
    q = draw_q8(hash_counters(r.seed, spec.STREAM_VALUE, i), r.value)
    scale = worker_scale_q16(r)
    s = np.uint64(65536) if scale is None else scale[((i // np.uint64(r.M)) % np.uint64(r.N)).astype(np.int64)].astype(np.uint64)
    if r.spike_thresh:
        spike = (hash_counters(r.seed, spec.STREAM_SPIKE, i) >> np.uint64(32)) < np.uint64(r.spike_thresh)
        if r.spike_workers:
            spike &= ((i // np.uint64(r.M)) % np.uint64(r.N)) < np.uint64(r.spike_workers)
    else:
        spike = np.zeros(count, dtype=bool)
    mul = np.where(spike, np.uint64(r.spike_mul), np.uint64(1))
    v = ((q * s * mul + np.uint64(1 << 23)) >> np.uint64(24)).astype(np.int64)
    if r.worker_add is not None:
        v = v + np.asarray(r.worker_add, dtype=np.int64)[((i // np.uint64(r.M)) % np.uint64(r.N)).astype(np.int64)]
    v = np.maximum(v, r.clip_min) + r.add + np.where(spike, r.spike_add, 0)
    assert v.max(initial=0) < (1 << 31)
    return v.astype(np.int32)


# ---- C generator -----------------------------------------------------------------------

class _Args:
    """ctypes views of a recipe's tables (kept alive for the duration of a fill)."""
    def __init__(self, r: Recipe):
        self.main = np.ascontiguousarray(r.value.main, dtype=np.int64)
        self.lo = np.ascontiguousarray(r.value.lo, dtype=np.int64)
        self.hi = np.ascontiguousarray(r.value.hi, dtype=np.int64)
        self.scale = worker_scale_q16(r)
        self.worker_add = None if r.worker_add is None else np.ascontiguousarray(r.worker_add, dtype=np.int64)
        self.key_value = spec.stream_key(r.seed, spec.STREAM_VALUE)
        self.key_spike = spec.stream_key(r.seed, spec.STREAM_SPIKE)


def fill(r: Recipe, out: np.ndarray, idx0: int, args: _Args | None = None) -> None:
    """Fill the flat int32 array `out` with elements idx0..idx0+len(out) (C, one thread)."""
    assert out.dtype == np.int32 and out.flags.c_contiguous
    a = args or _Args(r)
    _load().dcgen_fill_host(out.ctypes.data, idx0, out.size, a.key_value, a.key_spike, r.N, r.M,
                            a.main.ctypes.data, a.lo.ctypes.data, a.hi.ctypes.data,
                            None if a.scale is None else a.scale.ctypes.data,
                            None if a.worker_add is None else a.worker_add.ctypes.data,
                            r.add, r.clip_min, r.spike_thresh, r.spike_mul, r.spike_add, r.spike_workers)


def generate(r: Recipe, t0: int = 0, t1: int | None = None, threads: int | None = None) -> np.ndarray:
    """Trials t0..t1 of the workload as an int32 array [t1-t0][N][M] (C, threaded)."""
    t1 = r.T if t1 is None else t1
    per_trial = r.N * r.M
    out = np.empty((t1 - t0) * per_trial, dtype=np.int32)
    a = _Args(r)
    threads = threads or cpu_threads()
    n = out.size
    step = max(1 << 16, -(-n // (threads * 4)))
    spans = [(s, min(n, s + step)) for s in range(0, n, step)]

    def work(span):
        s, e = span
        fill(r, out[s:e], t0 * per_trial + s, a)

    if len(spans) == 1 or threads == 1:
        for sp in spans:
            work(sp)
    else:
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(work, spans))
    return out.reshape(t1 - t0, r.N, r.M)


def trial_chunks(r: Recipe, max_bytes: int = 256 << 20):
    """Yield (t0, t1) ranges whose tensors stay under max_bytes."""
    per = r.N * r.M * 4
    step = max(1, max_bytes // per)
    for t0 in range(0, r.T, step):
        yield t0, min(r.T, t0 + step)


def worker_totals(lat: np.ndarray) -> np.ndarray:
    """Sum of each worker's M latencies, int64, flattened over (trial, worker)."""
    return lat.reshape(-1, lat.shape[-1]).sum(axis=1, dtype=np.int64)


def tau_grid(r: Recipe, threads: int | None = None) -> np.ndarray:
    """The workload's K candidate thresholds (int64 microseconds), from CPU-generated data."""
    totals = np.empty(r.T * r.N, dtype=np.int64)
    for t0, t1 in trial_chunks(r):
        totals[t0 * r.N:t1 * r.N] = worker_totals(generate(r, t0, t1, threads))
    return tau_grid_from_totals(r, totals)


def tau_grid_from_totals(r: Recipe, totals: np.ndarray) -> np.ndarray:
    i_lo, i_hi = spec.grid_rank_indices(totals.size, r.grid)
    part = np.partition(totals, (i_lo, i_hi))
    return spec.tau_grid((int(part[i_lo]), int(part[i_hi])), r.K)
