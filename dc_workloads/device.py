"""GPU generation of the synthetic latency workloads (see spec.py for the definition).

The tensors of the two largest workloads (4.3 GB and 34 GB) are written straight into HBM by a
small HIP kernel that repeats the integer recipe of host.py; tests compare the two bit for bit.
The threshold grid is placed from per-worker totals computed with ordinary torch reductions.
Input preparation only: nothing here is part of the simulator library.
"""
from __future__ import annotations

import ctypes
import subprocess
from pathlib import Path

import numpy as np

from . import host, spec
from .spec import Recipe

_HERE = Path(__file__).resolve().parent
_LIB_PATH = _HERE / "libdcgen_hip.so"
_lib = None


def build(verbose: bool = False) -> Path:
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-o", str(_LIB_PATH), str(_HERE / "csrc" / "gen_device.hip")]
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
            raise ImportError(f"{_LIB_PATH} is missing: build it first")
        lib = ctypes.CDLL(str(_LIB_PATH))
        p, u64, i64, u32 = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int64, ctypes.c_uint32
        lib.dcgen_fill_device.argtypes = [p, u64, u64, u64, u64, i64, i64, p, p, p, p, p, i64, i64, u32, u32, i64, i64, p]
        lib.dcgen_fill_device.restype = ctypes.c_int
        _lib = lib
    return _lib


def generate(r: Recipe, t0: int = 0, t1: int | None = None, device: str = "cuda:0"):
    """Trials t0..t1 of the workload as a GPU int32 tensor [t1-t0][N][M]."""
    import torch
    t1 = r.T if t1 is None else t1
    dev = torch.device(device)
    out = torch.empty((t1 - t0, r.N, r.M), dtype=torch.int32, device=dev)
    tables = [torch.from_numpy(np.ascontiguousarray(t, dtype=np.int64)).to(dev)
              for t in (r.value.main, r.value.lo, r.value.hi)]
    scale_np = host.worker_scale_q16(r)
    scale = None if scale_np is None else torch.from_numpy(scale_np.view(np.int32).copy()).to(dev)
    wadd = None if r.worker_add is None else torch.from_numpy(np.ascontiguousarray(r.worker_add, dtype=np.int64)).to(dev)
    with torch.cuda.device(dev):
        stream = torch.cuda.current_stream()
        rc = _load().dcgen_fill_device(
            out.data_ptr(), t0 * r.N * r.M, out.numel(),
            spec.stream_key(r.seed, spec.STREAM_VALUE), spec.stream_key(r.seed, spec.STREAM_SPIKE),
            r.N, r.M, tables[0].data_ptr(), tables[1].data_ptr(), tables[2].data_ptr(),
            None if scale is None else scale.data_ptr(), None if wadd is None else wadd.data_ptr(),
            r.add, r.clip_min, r.spike_thresh, r.spike_mul, r.spike_add, r.spike_workers, int(stream.cuda_stream))
        if rc != 0:
            raise RuntimeError(f"dcgen_fill_device: hipError {rc}")
        stream.synchronize()          # the tables may be released once the kernel has run
    return out


def worker_totals(lat):
    """Sum of each worker's M latencies (int64, flattened over trial and worker), on the GPU."""
    import torch
    return lat.reshape(-1, lat.shape[-1]).sum(dim=1, dtype=torch.int64)


def tau_grid(r: Recipe, lat) -> np.ndarray:
    """The workload's K candidate thresholds from a GPU tensor holding all T trials."""
    import torch
    totals = worker_totals(lat)
    i_lo, i_hi = spec.grid_rank_indices(totals.numel(), r.grid)
    ordered = torch.sort(totals).values
    lo, hi = int(ordered[i_lo].item()), int(ordered[i_hi].item())
    return spec.tau_grid((lo, hi), r.K)
