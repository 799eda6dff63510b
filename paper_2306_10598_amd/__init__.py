"""Python binding of libdc (include/dc.h): argument marshalling only.

Every step of the computation runs in the HIP kernels of libdc.so; nothing here computes on
latencies, and there is no CPU fallback: importing works without the library (so that build
tooling can import the package), but every call raises if libdc.so cannot be loaded.

PyTorch is used only to hold device memory (`tensor.data_ptr()`) and to name a stream.
"""
from __future__ import annotations

import ctypes
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
LIB_PATH = _HERE / "libdc.so"

DC_OK, DC_ERR_INVALID_ARG, DC_ERR_NEGATIVE_LATENCY, DC_ERR_RANGE, DC_ERR_DEVICE, DC_ERR_NOMEM = range(6)
DC_MAX_THRESHOLDS = 65536

EXPORTS = (
    "dc_simulate", "dc_workspace_bytes", "dc_simulate_async", "dc_simulate_static", "dc_workspace_status", "dc_select_tau",
    "dc_simulate_strided", "dc_simulate_strided_async", "dc_worker_moments_strided", "dc_workspace_kernel_ms",
    "dc_speedup_per_step", "dc_speedup_workspace_bytes", "dc_speedup_per_step_async", "dc_select_tau_per_step",
    "dc_moments", "dc_worker_moments", "dc_analytic_curves",
    "dc_set_kernel_timing", "dc_last_kernel_ms", "dc_status_string", "dc_last_device_error", "dc_device_info", "dc_shutdown",
)

_lib = None


class DcError(RuntimeError):
    """A libdc call returned a status other than DC_OK."""

    def __init__(self, status: int, where: str):
        lib = _load()
        text = lib.dc_status_string(status).decode()
        detail = lib.dc_last_device_error().decode()
        super().__init__(f"{where}: {text}" + (f" ({detail})" if detail and status >= DC_ERR_DEVICE else ""))
        self.status = status


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not LIB_PATH.exists():
        raise ImportError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    lib = ctypes.CDLL(str(LIB_PATH))
    i64, p, sz = ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t
    lib.dc_simulate.argtypes = [p, i64, i64, i64, p, i64, i64, p, p]
    lib.dc_simulate.restype = ctypes.c_int
    lib.dc_workspace_bytes.argtypes = [i64, i64, i64, i64]
    lib.dc_workspace_bytes.restype = sz
    lib.dc_simulate_async.argtypes = [p, i64, i64, i64, p, i64, i64, p, p, p, sz, p]
    lib.dc_simulate_async.restype = ctypes.c_int
    lib.dc_simulate_static.argtypes = [p, i64, i64, i64, p, i64, i64, p, p, p, p]
    lib.dc_simulate_static.restype = ctypes.c_int
    lib.dc_simulate_strided.argtypes = [p, i64, i64, i64, i64, p, i64, i64, p, p]
    lib.dc_simulate_strided.restype = ctypes.c_int
    lib.dc_simulate_strided_async.argtypes = [p, i64, i64, i64, i64, p, i64, i64, p, p, p, sz, p]
    lib.dc_simulate_strided_async.restype = ctypes.c_int
    lib.dc_worker_moments_strided.argtypes = [p, i64, i64, i64, i64, p, p, p, p]
    lib.dc_worker_moments_strided.restype = ctypes.c_int
    lib.dc_workspace_kernel_ms.argtypes = [p, p, p]
    lib.dc_workspace_kernel_ms.restype = ctypes.c_int
    lib.dc_workspace_status.argtypes = [p, p]
    lib.dc_workspace_status.restype = ctypes.c_int
    lib.dc_select_tau.argtypes = [p, p, p, i64, i64, i64, i64, i64, p, p, p]
    lib.dc_select_tau.restype = ctypes.c_int
    lib.dc_select_tau_per_step.argtypes = [p, p, i64, p]
    lib.dc_select_tau_per_step.restype = ctypes.c_int
    lib.dc_speedup_per_step.argtypes = [p, i64, i64, i64, p, i64, i64, p, p]
    lib.dc_speedup_per_step.restype = ctypes.c_int
    lib.dc_speedup_workspace_bytes.argtypes = [i64, i64, i64, i64]
    lib.dc_speedup_workspace_bytes.restype = sz
    lib.dc_speedup_per_step_async.argtypes = [p, i64, i64, i64, p, i64, i64, p, p, p, sz, p]
    lib.dc_speedup_per_step_async.restype = ctypes.c_int
    lib.dc_moments.argtypes = [p, i64, i64, i64, p, p, p, p]
    lib.dc_moments.restype = ctypes.c_int
    lib.dc_worker_moments.argtypes = [p, i64, i64, i64, p, p, p, p]
    lib.dc_worker_moments.restype = ctypes.c_int
    lib.dc_analytic_curves.argtypes = [ctypes.c_double, ctypes.c_double, i64, i64, p, i64, i64, ctypes.c_double, p, p, p, p]
    lib.dc_analytic_curves.restype = ctypes.c_int
    lib.dc_set_kernel_timing.argtypes = [ctypes.c_int]
    lib.dc_set_kernel_timing.restype = ctypes.c_int
    lib.dc_last_kernel_ms.argtypes = [p, p]
    lib.dc_last_kernel_ms.restype = ctypes.c_int
    lib.dc_status_string.argtypes = [ctypes.c_int]
    lib.dc_status_string.restype = ctypes.c_char_p
    lib.dc_last_device_error.argtypes = []
    lib.dc_last_device_error.restype = ctypes.c_char_p
    lib.dc_device_info.argtypes = [p, p, p, p]
    lib.dc_device_info.restype = ctypes.c_int
    lib.dc_shutdown.argtypes = []
    lib.dc_shutdown.restype = None
    _lib = lib
    return lib


def _check(status: int, where: str) -> None:
    if status != DC_OK:
        raise DcError(status, where)


def _device_tensor(t, dtype_name: str, what: str):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{what} must be a GPU tensor")
    if t.dtype != getattr(torch, dtype_name) or not t.is_contiguous():
        raise TypeError(f"{what} must be a contiguous {dtype_name} tensor")
    return t


def _device_writable(t, dtype_name: str, what: str):
    """A contiguous tensor the device can write: device memory, or pinned host memory (mapped at the same address)."""
    import torch
    if not isinstance(t, torch.Tensor) or not (t.is_cuda or t.is_pinned()):
        raise TypeError(f"{what} must be a GPU tensor or a pinned host tensor")
    if t.dtype != getattr(torch, dtype_name) or not t.is_contiguous():
        raise TypeError(f"{what} must be a contiguous {dtype_name} tensor")
    return t


def _slab(lat, workers):
    """(pointer, T, N', M, trial stride in elements) of a contiguous GPU tensor [T][N][M], or of the workers
    workers[0] .. workers[1]-1 of it when `workers` = (n0, n1) is given: no copy is made."""
    lat = _device_tensor(lat, "int32", "lat")
    if lat.dim() != 3:
        raise TypeError("lat must have shape [T][N][M]")
    T, N, M = lat.shape
    if workers is None:
        return lat.data_ptr(), T, N, M, N * M
    n0, n1 = int(workers[0]), int(workers[1])
    if not 0 <= n0 < n1 <= N:
        raise ValueError("workers must be a range (n0, n1) with 0 <= n0 < n1 <= N")
    return lat.data_ptr() + 4 * n0 * M, T, n1 - n0, M, N * M


def dc_status_string(status: int) -> str:
    return _load().dc_status_string(int(status)).decode()


def dc_workspace_bytes(T: int, N: int, M: int, K: int) -> int:
    return int(_load().dc_workspace_bytes(T, N, M, K))


def dc_simulate(lat, taus, comm: int, workers=None):
    """out_step[K], out_done[K] (NumPy int64) for a GPU int32 tensor lat[T][N][M] and host thresholds.
    workers = (n0, n1): only those workers of every trial (dc_simulate_strided, the tensor is not copied)."""
    ptr, T, N, M, stride = _slab(lat, workers)
    taus = np.ascontiguousarray(taus, dtype=np.int64)
    K = taus.size
    out_step = np.empty(K, dtype=np.int64)
    out_done = np.empty(K, dtype=np.int64)
    if workers is None:
        rc = _load().dc_simulate(ptr, T, N, M, taus.ctypes.data, K, int(comm), out_step.ctypes.data, out_done.ctypes.data)
    else:
        rc = _load().dc_simulate_strided(ptr, T, N, M, stride, taus.ctypes.data, K, int(comm),
                                         out_step.ctypes.data, out_done.ctypes.data)
    _check(rc, "dc_simulate")
    return out_step, out_done


def dc_simulate_async(lat, taus_dev, comm: int, out_step_dev, out_done_dev, workspace, stream=None, workers=None) -> None:
    """Enqueue the computation on `stream` (a torch.cuda.Stream, or None for the null stream).
    workers = (n0, n1): only those workers of every trial (dc_simulate_strided_async)."""
    ptr, T, N, M, stride = _slab(lat, workers)
    taus_dev = _device_tensor(taus_dev, "int64", "taus_dev")
    K = taus_dev.numel()
    out_step_dev = _device_writable(out_step_dev, "int64", "out_step_dev")
    out_done_dev = _device_writable(out_done_dev, "int64", "out_done_dev")
    workspace = _device_tensor(workspace, "uint8", "workspace")
    if out_step_dev.numel() < K or out_done_dev.numel() < K:
        raise ValueError("output tensors are shorter than the threshold list")
    handle = 0 if stream is None else int(stream.cuda_stream)
    if workers is None:
        rc = _load().dc_simulate_async(ptr, T, N, M, taus_dev.data_ptr(), K, int(comm),
                                       out_step_dev.data_ptr(), out_done_dev.data_ptr(),
                                       workspace.data_ptr(), workspace.numel(), handle)
    else:
        rc = _load().dc_simulate_strided_async(ptr, T, N, M, stride, taus_dev.data_ptr(), K, int(comm),
                                               out_step_dev.data_ptr(), out_done_dev.data_ptr(),
                                               workspace.data_ptr(), workspace.numel(), handle)
    _check(rc, "dc_simulate_async")


class PreparedSimulation:
    """dc_simulate_async with its arguments marshalled once, for callers that repeat the call on the same tensors and
    stream (a tuning loop, a benchmark): enqueue() is the one C call, 5 us less of Python than dc_simulate_async."""

    def __init__(self, lat, taus_dev, comm: int, out_step_dev, out_done_dev, workspace, stream=None, workers=None):
        ptr, T, N, M, stride = _slab(lat, workers)
        taus_dev = _device_tensor(taus_dev, "int64", "taus_dev")
        K = taus_dev.numel()
        out_step_dev = _device_writable(out_step_dev, "int64", "out_step_dev")
        out_done_dev = _device_writable(out_done_dev, "int64", "out_done_dev")
        workspace = _device_tensor(workspace, "uint8", "workspace")
        if out_step_dev.numel() < K or out_done_dev.numel() < K:
            raise ValueError("output tensors are shorter than the threshold list")
        handle = 0 if stream is None else int(stream.cuda_stream)
        self._keep = (lat, taus_dev, out_step_dev, out_done_dev, workspace, stream)     # the call holds their addresses
        self._fn = _load().dc_simulate_strided_async
        self._args = (ptr, T, N, M, stride, taus_dev.data_ptr(), K, int(comm), out_step_dev.data_ptr(),
                      out_done_dev.data_ptr(), workspace.data_ptr(), workspace.numel(), handle)

    def enqueue(self) -> None:
        rc = self._fn(*self._args)
        if rc != DC_OK:
            raise DcError(rc, "dc_simulate_strided_async")


class PreparedSelection:
    """dc_select_tau on fixed host arrays (the pinned arrays that a PreparedSimulation writes, say): select() is the
    one C call; thr and s_eff are arrays of this object, overwritten by every call."""

    def __init__(self, step_sum, done_sum, taus, T: int, N: int, M: int, base_step_sum: int = 0):
        for a, what in ((step_sum, "step_sum"), (done_sum, "done_sum"), (taus, "taus")):
            if not isinstance(a, np.ndarray) or a.dtype != np.int64 or not a.flags.c_contiguous:
                raise TypeError(f"{what} must be a contiguous NumPy int64 array (it is read in place on every call)")
        K = taus.size
        if step_sum.size != K or done_sum.size != K:
            raise ValueError("step_sum, done_sum and taus must have the same length")
        self.thr = np.empty(K, dtype=np.float64)
        self.seff = np.empty(K, dtype=np.float64)
        self._best = ctypes.c_int64(-1)
        self._keep = (step_sum, done_sum, taus)
        self._fn = _load().dc_select_tau
        self._args = (step_sum.ctypes.data, done_sum.ctypes.data, taus.ctypes.data, K, int(T), int(N), int(M),
                      int(base_step_sum), self.thr.ctypes.data, self.seff.ctypes.data, ctypes.addressof(self._best))

    def select(self):
        rc = self._fn(*self._args)
        if rc != DC_OK:
            raise DcError(rc, "dc_select_tau")
        return self.thr, self.seff, self._best.value


class PreparedSpeedup:
    """dc_speedup_per_step_async with its arguments marshalled once (see PreparedSimulation); select() is Algorithm 2's
    final argmax on the result, which must then be a pinned host tensor."""

    def __init__(self, lat, taus_dev, comm: int, comm_per_trial_dev, out_seff, workspace, stream=None, taus_host=None):
        lat = _device_tensor(lat, "int32", "lat")
        if lat.dim() != 3:
            raise TypeError("lat must have shape [T][N][M]")
        T, N, M = lat.shape
        taus_dev = _device_tensor(taus_dev, "int64", "taus_dev")
        K = taus_dev.numel()
        out_seff = _device_writable(out_seff, "float64", "out_seff")
        workspace = _device_tensor(workspace, "uint8", "workspace")
        per_ptr = None
        if comm_per_trial_dev is not None:
            per = _device_tensor(comm_per_trial_dev, "int64", "comm_per_trial_dev")
            if per.numel() != T:
                raise ValueError("comm_per_trial_dev needs one value per trial")
            per_ptr = per.data_ptr()
        if out_seff.numel() < K:
            raise ValueError("output tensor is shorter than the threshold list")
        handle = 0 if stream is None else int(stream.cuda_stream)
        self._keep = (lat, taus_dev, comm_per_trial_dev, out_seff, workspace, stream, taus_host)
        self._fn = _load().dc_speedup_per_step_async
        self._args = (lat.data_ptr(), T, N, M, taus_dev.data_ptr(), K, int(comm), per_ptr, out_seff.data_ptr(),
                      workspace.data_ptr(), workspace.numel(), handle)
        self._select = None
        if taus_host is not None:
            if out_seff.is_cuda:
                raise TypeError("select() reads the result on the host: out_seff must be a pinned host tensor")
            if not isinstance(taus_host, np.ndarray) or taus_host.dtype != np.int64 or not taus_host.flags.c_contiguous \
                    or taus_host.size != K:
                raise TypeError("taus_host must be the K thresholds as a contiguous NumPy int64 array")
            self._best = ctypes.c_int64(-1)
            self._select = (out_seff.data_ptr(), taus_host.ctypes.data, K, ctypes.addressof(self._best))

    def enqueue(self) -> None:
        rc = self._fn(*self._args)
        if rc != DC_OK:
            raise DcError(rc, "dc_speedup_per_step_async")

    def select(self) -> int:
        if self._select is None:
            raise ValueError("prepared without the host copy of the thresholds")
        rc = _load().dc_select_tau_per_step(*self._select)
        if rc != DC_OK:
            raise DcError(rc, "dc_select_tau_per_step")
        return self._best.value


DC_STATIC_SCRATCH_BYTES = 16 << 20


def dc_simulate_static(lat, taus_dev, comm: int, out_step_dev, out_done_dev, status_dev=None, stream=None) -> None:
    """dc_simulate_async without a workspace: the library's fixed device array serves instead (nothing is allocated)."""
    lat = _device_tensor(lat, "int32", "lat")
    if lat.dim() != 3:
        raise TypeError("lat must have shape [T][N][M]")
    T, N, M = lat.shape
    taus_dev = _device_tensor(taus_dev, "int64", "taus_dev")
    K = taus_dev.numel()
    out_step_dev = _device_tensor(out_step_dev, "int64", "out_step_dev")
    out_done_dev = _device_tensor(out_done_dev, "int64", "out_done_dev")
    if out_step_dev.numel() < K or out_done_dev.numel() < K:
        raise ValueError("output tensors are shorter than the threshold list")
    status_ptr = None if status_dev is None else _device_tensor(status_dev, "int32", "status_dev").data_ptr()
    handle = 0 if stream is None else int(stream.cuda_stream)
    rc = _load().dc_simulate_static(lat.data_ptr(), T, N, M, taus_dev.data_ptr(), K, int(comm),
                                    out_step_dev.data_ptr(), out_done_dev.data_ptr(), status_ptr, handle)
    _check(rc, "dc_simulate_static")


def dc_workspace_status(workspace, stream=None) -> int:
    """Wait for the stream; return the status the device recorded in the workspace (no exception)."""
    workspace = _device_tensor(workspace, "uint8", "workspace")
    handle = 0 if stream is None else int(stream.cuda_stream)
    return int(_load().dc_workspace_status(workspace.data_ptr(), handle))


def dc_select_tau(step_sum, done_sum, taus, T: int, N: int, M: int, base_step_sum: int = 0):
    """(thr[K], s_eff[K], best_k) from dc_simulate's outputs; host only."""
    step_sum = np.ascontiguousarray(step_sum, dtype=np.int64)
    done_sum = np.ascontiguousarray(done_sum, dtype=np.int64)
    taus = np.ascontiguousarray(taus, dtype=np.int64)
    K = taus.size
    if step_sum.size != K or done_sum.size != K:
        raise ValueError("step_sum, done_sum and taus must have the same length")
    thr = np.empty(K, dtype=np.float64)
    seff = np.empty(K, dtype=np.float64)
    best = ctypes.c_int64(-1)
    rc = _load().dc_select_tau(step_sum.ctypes.data, done_sum.ctypes.data, taus.ctypes.data, K, T, N, M,
                               int(base_step_sum), thr.ctypes.data, seff.ctypes.data, ctypes.byref(best))
    _check(rc, "dc_select_tau")
    return thr, seff, int(best.value)


def dc_select_tau_per_step(seff, taus) -> int:
    """Index of the best threshold for dc_speedup_per_step's output (Algorithm 2's final argmax); host only."""
    seff = np.ascontiguousarray(seff, dtype=np.float64)
    taus = np.ascontiguousarray(taus, dtype=np.int64)
    if seff.size != taus.size:
        raise ValueError("seff and taus must have the same length")
    best = ctypes.c_int64(-1)
    _check(_load().dc_select_tau_per_step(seff.ctypes.data, taus.ctypes.data, taus.size, ctypes.byref(best)),
           "dc_select_tau_per_step")
    return int(best.value)


def dc_speedup_workspace_bytes(T: int, N: int, M: int, K: int) -> int:
    return int(_load().dc_speedup_workspace_bytes(T, N, M, K))


def dc_speedup_per_step(lat, taus, comm: int = 0, comm_per_trial=None):
    """S_eff[K] (NumPy float64) as the mean of per-iteration speedups; comm_per_trial: T host values or None."""
    lat = _device_tensor(lat, "int32", "lat")
    if lat.dim() != 3:
        raise TypeError("lat must have shape [T][N][M]")
    T, N, M = lat.shape
    taus = np.ascontiguousarray(taus, dtype=np.int64)
    per = None
    if comm_per_trial is not None:
        per = np.ascontiguousarray(comm_per_trial, dtype=np.int64)
        if per.size != T:
            raise ValueError("comm_per_trial needs one value per trial")
    out = np.empty(taus.size, dtype=np.float64)
    rc = _load().dc_speedup_per_step(lat.data_ptr(), T, N, M, taus.ctypes.data, taus.size, int(comm),
                                     None if per is None else per.ctypes.data, out.ctypes.data)
    _check(rc, "dc_speedup_per_step")
    return out


def dc_speedup_per_step_async(lat, taus_dev, comm: int, comm_per_trial_dev, out_seff_dev, workspace, stream=None) -> None:
    lat = _device_tensor(lat, "int32", "lat")
    if lat.dim() != 3:
        raise TypeError("lat must have shape [T][N][M]")
    T, N, M = lat.shape
    taus_dev = _device_tensor(taus_dev, "int64", "taus_dev")
    out_seff_dev = _device_writable(out_seff_dev, "float64", "out_seff_dev")
    workspace = _device_tensor(workspace, "uint8", "workspace")
    per_ptr = None
    if comm_per_trial_dev is not None:
        per = _device_tensor(comm_per_trial_dev, "int64", "comm_per_trial_dev")
        if per.numel() != T:
            raise ValueError("comm_per_trial_dev needs one value per trial")
        per_ptr = per.data_ptr()
    if out_seff_dev.numel() < taus_dev.numel():
        raise ValueError("output tensor is shorter than the threshold list")
    handle = 0 if stream is None else int(stream.cuda_stream)
    rc = _load().dc_speedup_per_step_async(lat.data_ptr(), T, N, M, taus_dev.data_ptr(), taus_dev.numel(), int(comm),
                                           per_ptr, out_seff_dev.data_ptr(), workspace.data_ptr(), workspace.numel(),
                                           handle)
    _check(rc, "dc_speedup_per_step_async")


def dc_moments(lat):
    """(sum, sum of squares) as exact Python ints and (mean, variance) as floats of a GPU int32 tensor."""
    lat = _device_tensor(lat, "int32", "lat")
    if lat.dim() != 3:
        raise TypeError("lat must have shape [T][N][M]")
    T, N, M = lat.shape
    total = ctypes.c_int64(0)
    sq = (ctypes.c_uint64 * 2)(0, 0)
    mean, var = ctypes.c_double(0), ctypes.c_double(0)
    rc = _load().dc_moments(lat.data_ptr(), T, N, M, ctypes.byref(total), sq, ctypes.byref(mean), ctypes.byref(var))
    _check(rc, "dc_moments")
    return int(total.value), (int(sq[1]) << 64) | int(sq[0]), float(mean.value), float(var.value)


def dc_worker_moments(lat, workers=None):
    """Per worker: (sums, sums of squares) of its iteration time as lists of exact Python ints, and (mean[N],
    variance[N]) as NumPy float64 arrays.  workers = (n0, n1): only those workers (dc_worker_moments_strided)."""
    ptr, T, N, M, stride = _slab(lat, workers)
    sums = np.empty(N, dtype=np.int64)
    sq = np.empty(2 * N, dtype=np.uint64)
    mean = np.empty(N, dtype=np.float64)
    var = np.empty(N, dtype=np.float64)
    rc = _load().dc_worker_moments_strided(ptr, T, N, M, stride, sums.ctypes.data, sq.ctypes.data, mean.ctypes.data,
                                           var.ctypes.data)
    _check(rc, "dc_worker_moments")
    low, high = sq[0::2].tolist(), sq[1::2].tolist()           # the 128-bit sums of squares as Python ints
    return (sums.tolist(), [(h << 64) | l for l, h in zip(low, high)], mean, var)


def dc_analytic_curves(mu: float, sigma2: float, N: int, M: int, taus, comm: int, mean_tmax=None):
    """(e_done[K], e_t, s_eff[K], best_k): the closed-form estimates; mean_tmax=None uses the modelled E[T]."""
    taus = np.ascontiguousarray(taus, dtype=np.int64)
    K = taus.size
    e_done = np.empty(K, dtype=np.float64)
    s_eff = np.empty(K, dtype=np.float64)
    e_t = ctypes.c_double(0)
    best = ctypes.c_int64(-1)
    rc = _load().dc_analytic_curves(float(mu), float(sigma2), N, M, taus.ctypes.data, K, int(comm),
                                    -1.0 if mean_tmax is None else float(mean_tmax),
                                    e_done.ctypes.data, s_eff.ctypes.data, ctypes.byref(e_t), ctypes.byref(best))
    _check(rc, "dc_analytic_curves")
    return e_done, float(e_t.value), s_eff, int(best.value)


def dc_set_kernel_timing(enable) -> None:
    """False/0: off; True/1: time the streaming kernel; 2: also the whole enqueued sequence."""
    _check(_load().dc_set_kernel_timing(int(enable)), "dc_set_kernel_timing")


def dc_last_kernel_ms(whole: bool = False):
    """(scan_ms, total_ms) of the last timed call; total_ms is None unless whole=True (timing level 2)."""
    a, b = ctypes.c_float(0), ctypes.c_float(0)
    _check(_load().dc_last_kernel_ms(ctypes.byref(a), ctypes.byref(b) if whole else None), "dc_last_kernel_ms")
    return float(a.value), (float(b.value) if whole else None)


def dc_workspace_kernel_ms(workspace, whole: bool = False):
    """(scan_ms, total_ms) of the last timed call that ran in `workspace`; total_ms is None unless whole=True."""
    workspace = _device_tensor(workspace, "uint8", "workspace")
    a, b = ctypes.c_float(0), ctypes.c_float(0)
    _check(_load().dc_workspace_kernel_ms(workspace.data_ptr(), ctypes.byref(a), ctypes.byref(b) if whole else None),
           "dc_workspace_kernel_ms")
    return float(a.value), (float(b.value) if whole else None)


def dc_device_info() -> dict:
    """Compute units, memory clock (kHz), memory bus width (bits) and L2 size (bytes) of the current device."""
    v = [ctypes.c_int32(0) for _ in range(4)]
    _check(_load().dc_device_info(*[ctypes.byref(x) for x in v]), "dc_device_info")
    return {"compute_units": v[0].value, "memory_clock_khz": v[1].value, "memory_bus_bits": v[2].value, "l2_bytes": v[3].value}


def dc_shutdown() -> None:
    _load().dc_shutdown()
