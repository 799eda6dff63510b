"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element.

Integer outputs must be bit-exact; the float ratios of dc_select_tau within 1e-6 relative.
Inputs are seeded and synthetic; the oracle always gets CPU-generated tensors and grids.
"""
import sys
import time

import numpy as np
import pytest

import oracle
import paper_2306_10598_amd as dc
from dc_workloads import config, host, spec

pytestmark = pytest.mark.gpu

SPEEDUP_RTOL = 1e-6        # stated bar for float ratios; the two sides differ only in rounding order (~1e-15)

torch = pytest.importorskip("torch")
BIG = 1 << 40


def progress(msg: str) -> None:
    """Progress lines of the long tests (shown by pytest -s, or with the captured output of a failure)."""
    print(f"{time.strftime('%H:%M:%S')} {msg}", file=sys.stderr, flush=True)


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    dc._load()
    return torch.device("cuda:0")


def to_dev(lat: np.ndarray, dev):
    return torch.from_numpy(np.ascontiguousarray(lat)).to(dev)


def extra_thresholds(taus: np.ndarray, rng) -> np.ndarray:
    """The workload's grid plus edge thresholds, duplicated and shuffled (any order is legal)."""
    t = np.concatenate([taus, [0, 1, BIG, (1 << 31) - 1, 1 << 31, int(taus[len(taus) // 2])]]).astype(np.int64)
    return t[rng.permutation(t.size)]


def check(lat: np.ndarray, taus, comm, dev, method="sorted"):
    step, done = dc.dc_simulate(to_dev(lat, dev), taus, comm)
    ref_step, ref_done = oracle.simulate(lat, taus, comm, method)
    assert np.array_equal(done, ref_done), (np.flatnonzero(done != ref_done)[:5], done[:5], ref_done[:5])
    assert np.array_equal(step, ref_step), (np.flatnonzero(step != ref_step)[:5], step[:5], ref_step[:5])
    return step, done


# ---- inputs: the GPU generator writes the same integers as the CPU generator --------------------

@pytest.mark.parametrize("name", spec.CONFIG_NAMES)
def test_device_generator_equals_host_generator(name, dev):
    from dc_workloads import device
    r = config(name)
    r = r.with_shape(T=max(2, min(r.T, (8 << 20) // (r.N * r.M * 4))))
    a = device.generate(r, 1, r.T).cpu().numpy()
    b = host.generate(r, 1, r.T)
    assert np.array_equal(a, b)
    if r.T * r.N >= 1000:
        assert np.array_equal(device.tau_grid(r, device.generate(r)), host.tau_grid(r))


# ---- hand-worked example and tiny cases ------------------------------------------------------------

def test_hand_worked_example(dev, golden_dir):
    from tests.test_oracle_pins import read_golden
    g = read_golden(golden_dir / "hand_example.txt")
    lat = np.array(g["lat"], dtype=np.int32).reshape(g["T"][0], g["N"][0], g["M"][0])
    step, done = dc.dc_simulate(to_dev(lat, dev), g["taus"], g["comm"][0])
    assert done.tolist() == g["done"] and step.tolist() == g["step"]


def test_tie_and_single_element(dev):
    lat = np.array([[[10, 20, 30, 40]]], dtype=np.int32)
    step, done = dc.dc_simulate(to_dev(lat, dev), [60, 61, 100, 101], 0)
    assert done.tolist() == [2, 3, 3, 4] and step.tolist() == [60, 61, 100, 100]
    one = np.array([[[7]]], dtype=np.int32)
    step, done = dc.dc_simulate(to_dev(one, dev), [7, 8, 0], 3)
    assert done.tolist() == [0, 1, 0] and step.tolist() == [10, 10, 3]


# ---- the five workloads at sizes the literal oracle finishes in seconds ----------------------------

@pytest.mark.parametrize("name,shape", [
    ("tiny", {}),                                           # full size: 1000 x 8 x 16
    ("lognormal64", {"T": 300}),
    ("lognormal64", {"T": 37, "N": 61}),                   # ragged: 61 workers, 8 per load
    ("additive200", {"T": 40}),
    ("additive200", {"T": 9, "N": 203}),                   # ragged tail of 3 workers
    ("extrapolation2048", {"T": 5}),
    ("extrapolation2048", {"T": 3, "N": 2047}),
    ("heterogeneous2048", {"T": 3}),
    ("heterogeneous2048", {"T": 2, "N": 1000}),
])
def test_workload_parity_literal(name, shape, dev):
    r = config(name).with_shape(**shape, K=min(config(name).K, 48))
    lat = host.generate(r)
    rng = np.random.default_rng(1)
    taus = extra_thresholds(host.tau_grid(r), rng)
    step, done = check(lat, taus, r.comm, dev, "literal")
    # select_tau on the GPU results against the oracle's
    base = int(step[np.argmax(taus)])
    thr, seff, best = dc.dc_select_tau(step, done, taus, r.T, r.N, r.M, base)
    othr, oseff, obest = oracle.select_tau(step, done, taus, r.T, r.N, r.M, base)
    assert best == obest
    assert np.allclose(thr, othr, rtol=1e-6, atol=0) and np.allclose(seff, oseff, rtol=1e-6, atol=0)
    assert seff[np.argmax(taus)] == pytest.approx(1.0, abs=1e-12)


@pytest.mark.parametrize("name,T", [("lognormal64", 4000), ("additive200", 1500), ("extrapolation2048", 96),
                                    ("heterogeneous2048", 40)])
def test_workload_parity_full_grid(name, T, dev):
    """Many units per wave and the workload's full threshold grid (sorted-walk oracle)."""
    r = config(name).with_shape(T=T)
    lat = host.generate(r)
    taus = host.tau_grid(r)
    ref = oracle.simulate_threaded(lat, taus, r.comm, "sorted", threads=host.cpu_threads())
    step, done = dc.dc_simulate(to_dev(lat, dev), taus, r.comm)
    assert np.array_equal(done, ref[1]) and np.array_equal(step, ref[0])


# ---- every vectorised row length, and the general kernel ------------------------------------------

@pytest.mark.parametrize("M", [4, 8, 16, 32, 64, 128, 256, 12, 20, 24, 44, 100, 132, 252])
@pytest.mark.parametrize("N", [1, 7, 64, 130])
def test_vector_kernel_shapes(M, N, dev):
    rng = np.random.default_rng(M * 1000 + N)
    lat = rng.integers(0, 5000, size=(11, N, M), dtype=np.int32)
    totals = lat.sum(axis=2, dtype=np.int64)
    taus = np.sort(rng.integers(0, int(totals.max()) + 50, size=33))
    check(lat, taus, 17, dev, "literal")


@pytest.mark.parametrize("M", [1, 2, 3, 5, 12, 63, 65, 100, 257, 300, 512, 1000])
def test_general_kernel_shapes(M, dev):
    rng = np.random.default_rng(M)
    lat = rng.integers(0, 3000, size=(6, 9, M), dtype=np.int32)
    totals = lat.sum(axis=2, dtype=np.int64)
    taus = rng.integers(0, int(totals.max()) + 50, size=21)
    check(lat, taus, 5, dev, "literal")


@pytest.mark.parametrize("words", [1, 2, 3])
@pytest.mark.parametrize("M", [1, 2, 3, 5, 8, 13, 64, 257, 700])
def test_any_alignment_any_row_length(words, M, dev):
    """Tensors that start 4, 8 or 12 bytes past a 16-byte boundary and end inside a vector, through all three
    entry points that stream them; the last latency is the largest legal one, so a read of the wrong element shows."""
    rng = np.random.default_rng(1000 * words + M)
    T, N = 5, int(rng.integers(3, 40))
    top = (2**31 - 1) // M
    lat = rng.integers(0, min(top, 4000) + 1, size=(T, N, M), dtype=np.int32)
    lat[0, 0, 0] = lat[-1, -1, -1] = min(top, 50000)
    flat = torch.full((lat.size + words + 4,), -7, dtype=torch.int32, device=dev)     # negative guard values around it
    view = flat[words:words + lat.size].view(T, N, M)
    view.copy_(torch.from_numpy(lat))
    assert view.data_ptr() % 16 == 4 * words
    totals = lat.sum(axis=2, dtype=np.int64)
    taus = rng.integers(0, int(totals.max()) + 50, size=33)
    step, done = dc.dc_simulate(view, taus, 3)
    ref = oracle.simulate(lat, taus, 3, "literal")
    assert np.array_equal(step, ref[0]) and np.array_equal(done, ref[1])
    taus1 = np.maximum(taus, 1)
    assert np.allclose(dc.dc_speedup_per_step(view, taus1, 3), oracle.per_step_speedup(lat, taus1, 3), rtol=SPEEDUP_RTOL, atol=0)
    gs, gq, _, _ = dc.dc_worker_moments(view)
    sums, squares, _, _ = oracle.worker_moments(lat)
    assert gs == sums and gq == squares


@pytest.mark.parametrize("N", [256, 260, 1024, 2052, 5000])
@pytest.mark.parametrize("M", list(range(1, 17)) + [17, 18, 19, 21, 22, 23, 25, 26, 30, 34])
def test_short_rows_held_whole_by_a_lane(M, N, dev):
    """Rows of up to 16 elements with at least 256 workers, a multiple of 4, on an aligned
    tensor go through the kernel in which every lane owns whole rows: full and partial chunks, one and several units
    per trial, a narrow grid near the row totals, a grid over every completion time (with 0, repeats and values no
    completion time reaches), and a worker range of the resident tensor (trials further apart than they are long)."""
    rng = np.random.default_rng(100 * M + N)
    T = 3
    top = min((2**31 - 1) // M, 6000)
    lat = rng.integers(0, top + 1, size=(T, N, M), dtype=np.int32)
    lat[0, 0, :] = top                                    # the largest legal row, and the row of trial 1 that decides its maximum
    lat[1, N - 1, :] = top // 2 + 1
    lat[1, :N - 1, :] //= 4
    totals = lat.sum(axis=2, dtype=np.int64)
    narrow = np.quantile(totals, np.linspace(0.6, 1.0, 33)).astype(np.int64)
    wide = np.concatenate([[0, 0, 1], rng.integers(0, int(totals.max()) + 50, size=60), [int(totals.max())] * 2, [BIG]])
    lat_dev = to_dev(lat, dev)
    for taus in (narrow, wide):
        step, done = dc.dc_simulate(lat_dev, taus, 9)
        ref = oracle.simulate(lat, taus, 9, "literal")
        assert np.array_equal(done, ref[1]) and np.array_equal(step, ref[0]), (M, N, taus[:4])
    if N >= 260:
        a = 4 * int(rng.integers(0, (N - 256) // 4 + 1))
        step, done = dc.dc_simulate(lat_dev, narrow, 2, workers=(a, a + 256))
        ref = oracle.simulate(np.ascontiguousarray(lat[:, a:a + 256]), narrow, 2, "literal")
        assert np.array_equal(done, ref[1]) and np.array_equal(step, ref[0]), (M, N, a)


@pytest.mark.parametrize("N", [4, 5, 6, 8, 10, 30, 64, 150, 200, 250, 252, 257, 1022])
@pytest.mark.parametrize("M", [3, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 16])
def test_short_rows_of_few_workers(M, N, dev):
    """Worker counts that are below 256 or no multiple of 4, short rows, contiguous tensor with a multiple of 4 rows in
    all: the lanes of a wave then hold rows of several trials, a trial boundary may fall inside a lane, and the trial
    maxima are built with atomic maxima.  Trials whose maximum sits in their first or last worker, a trial of zeros, a
    partial last chunk, narrow and all-covering grids."""
    rng = np.random.default_rng(1000 * M + N)
    T = 40
    top = min((2**31 - 1) // M, 6000)
    lat = rng.integers(0, top + 1, size=(T, N, M), dtype=np.int32)
    lat[::3] //= 3                                          # neighbouring trials with different maxima
    lat[1, 0, :] = top
    lat[2, N - 1, :] = top
    lat[5] = 0
    totals = lat.sum(axis=2, dtype=np.int64)
    narrow = np.quantile(totals, np.linspace(0.6, 1.0, 33)).astype(np.int64)
    wide = np.concatenate([[0, 0, 1], rng.integers(0, int(totals.max()) + 50, size=60), [int(totals.max())] * 2, [BIG]])
    lat_dev = to_dev(lat, dev)
    for taus in (narrow, wide):
        step, done = dc.dc_simulate(lat_dev, taus, 9)
        ref = oracle.simulate(lat, taus, 9, "literal")
        assert np.array_equal(done, ref[1]) and np.array_equal(step, ref[0]), (M, N, taus[:4])


@pytest.mark.parametrize("M,N", [(4, 64), (16, 16), (16, 48), (20, 12), (20, 36), (32, 8), (32, 24), (64, 4), (64, 12),
                                 (100, 2), (100, 6), (128, 2), (128, 8), (256, 1), (256, 4),          # whole loads per trial
                                 (20, 8), (20, 16), (24, 8), (28, 8), (32, 4), (36, 8), (44, 12), (48, 8), (64, 2), (64, 6),
                                 (20, 4), (24, 4), (36, 32), (20, 64), (20, 100)])
def test_small_trials_streamed_several_per_unit(M, N, dev):
    """Many trials of a few KiB on a contiguous tensor: a wave streams several consecutive trials as one run and keeps
    a maximum per trial.  Worker counts that are a whole number of 1 KiB loads, and worker counts that are not (a load
    then holds fewer rows than fit: 8 of 20 elements instead of 12).  A trial count that leaves the last unit short,
    trials whose maximum is their first or their last worker's next to trials of small values, a trial of zeros,
    narrow and all-covering grids; the same tensor through a worker range (trials apart: a unit per trial)."""
    rng = np.random.default_rng(1000 * M + N)
    T = 2 * 8192 * int(rng.integers(1, 3)) + int(rng.integers(1, 300))       # enough trials for units of several
    top = min((2**31 - 1) // M, 5000)
    lat = rng.integers(0, top + 1, size=(T, N, M), dtype=np.int32)
    lat[::3] //= 3                                          # neighbouring trials with different maxima
    lat[1, 0, :] = top
    lat[2, N - 1, :] = top
    lat[T - 1, N - 1, :] = top
    lat[5] = 0
    totals = lat.sum(axis=2, dtype=np.int64)
    narrow = np.quantile(totals, np.linspace(0.6, 1.0, 33)).astype(np.int64)
    wide = np.concatenate([[0, 0, 1], rng.integers(0, int(totals.max()) + 50, size=60), [int(totals.max())] * 2, [BIG]])
    lat_dev = to_dev(lat, dev)
    for taus in (narrow, wide):
        step, done = dc.dc_simulate(lat_dev, taus, 9)
        ref = oracle.simulate(lat, taus, 9, "sorted")
        assert np.array_equal(done, ref[1]) and np.array_equal(step, ref[0]), (M, N, T, taus[:4])
    if N >= 2:
        step, done = dc.dc_simulate(lat_dev, narrow, 2, workers=(0, N // 2))
        ref = oracle.simulate(np.ascontiguousarray(lat[:, :N // 2]), narrow, 2, "sorted")
        assert np.array_equal(done, ref[1]) and np.array_equal(step, ref[0]), (M, N, T)


@pytest.mark.parametrize("N", [32, 36, 64, 100, 120, 128, 192, 256, 1000, 2052])
@pytest.mark.parametrize("M", [17, 18, 21, 22, 25, 26, 27, 29, 30, 31, 33, 34, 35, 38, 42, 45, 47, 49, 50, 55, 62, 63])
def test_rows_of_a_few_dozen_elements_one_per_lane(M, N, dev):
    """Rows of 25 to 63 elements that are no multiple of 4 (nor 26, 30), and from 17 on with fewer than 256 workers, N*M a multiple of 4, at least 32 workers, aligned tensor:
    the kernel in which a lane owns one row and reads it word by word from the wave's copy of the chunk.  Full and
    partial chunks of 64 rows, one and several units per trial, a narrow grid near the row totals, a grid over every
    completion time (with 0, repeats and values no completion time reaches), 700 thresholds (tables that leave the
    kernel two blocks per compute unit for all but the longest rows), a threshold list of two passes (whose tables
    send every row length to the kernel for arbitrary rows), and a worker range of the resident tensor."""
    rng = np.random.default_rng(100 * M + N)
    T = 5
    top = min((2**31 - 1) // M, 6000)
    lat = rng.integers(0, top + 1, size=(T, N, M), dtype=np.int32)
    lat[0, 0, :] = top                                    # the largest legal row, and the row of trial 1 that decides its maximum
    lat[1, N - 1, :] = top // 2 + 1
    lat[1, :N - 1, :] //= 4
    lat[3] = 0
    totals = lat.sum(axis=2, dtype=np.int64)
    narrow = np.quantile(totals, np.linspace(0.6, 1.0, 33)).astype(np.int64)
    wide = np.concatenate([[0, 0, 1], rng.integers(0, int(totals.max()) + 50, size=60), [int(totals.max())] * 2, [BIG]])
    lat_dev = to_dev(lat, dev)
    for taus in (narrow, wide):
        step, done = dc.dc_simulate(lat_dev, taus, 9)
        ref = oracle.simulate(lat, taus, 9, "literal")
        assert np.array_equal(done, ref[1]) and np.array_equal(step, ref[0]), (M, N, taus[:4])
    if N == 256:
        for count in (700, 5000):
            many = rng.integers(int(totals.min()) // 2, int(totals.max()) + 10, size=count)
            step, done = dc.dc_simulate(lat_dev, many, 3)
            ref = oracle.simulate(lat, many, 3, "sorted")
            assert np.array_equal(done, ref[1]) and np.array_equal(step, ref[0]), (M, N, count)
    if N >= 100:
        a = 4 * int(rng.integers(0, (N - 64) // 4 + 1))
        step, done = dc.dc_simulate(lat_dev, narrow, 2, workers=(a, a + 64))
        ref = oracle.simulate(np.ascontiguousarray(lat[:, a:a + 64]), narrow, 2, "literal")
        assert np.array_equal(done, ref[1]) and np.array_equal(step, ref[0]), (M, N, a)


@pytest.mark.parametrize("N", [4, 5, 6, 10, 30, 50, 63, 100, 200, 250, 264])
@pytest.mark.parametrize("M", [17, 18, 21, 26, 33, 45, 50, 63])
def test_rows_of_a_few_dozen_elements_of_few_workers(M, N, dev):
    """Worker counts that fill the chunks of 64 rows badly, or not at all: on a contiguous tensor whose size is a
    multiple of 4 elements the kernel with one row per lane runs its chunks over the trials, a lane finds its row's
    trial by division and the trials' maxima are built with atomic maxima (otherwise the kernel for arbitrary rows
    takes the tensor).  Trials whose maximum sits in their first or last worker, a trial of zeros, a partial last
    chunk, narrow and all-covering grids, twice on one workspace."""
    rng = np.random.default_rng(1000 * M + N)
    T = 41 if (N * M) % 4 == 0 else 40
    top = min((2**31 - 1) // M, 6000)
    lat = rng.integers(0, top + 1, size=(T, N, M), dtype=np.int32)
    lat[::3] //= 3                                          # neighbouring trials with different maxima
    lat[1, 0, :] = top
    lat[2, N - 1, :] = top
    lat[5] = 0
    totals = lat.sum(axis=2, dtype=np.int64)
    narrow = np.quantile(totals, np.linspace(0.6, 1.0, 33)).astype(np.int64)
    wide = np.concatenate([[0, 0, 1], rng.integers(0, int(totals.max()) + 50, size=60), [int(totals.max())] * 2, [BIG]])
    lat_dev = to_dev(lat, dev)
    for taus in (narrow, wide, narrow):
        step, done = dc.dc_simulate(lat_dev, taus, 9)
        ref = oracle.simulate(lat, taus, 9, "literal")
        assert np.array_equal(done, ref[1]) and np.array_equal(step, ref[0]), (M, N, taus[:4])


@pytest.mark.parametrize("M", [15, 16, 17, 25, 30, 34, 62, 63])
def test_longest_rows_held_by_a_lane_with_a_full_pass_of_thresholds(M, dev):
    """Row lengths with the largest staging areas of the kernels with whole rows per lane, with the largest threshold
    tables (4095 per pass, two passes) and with tables of 600 thresholds: plans that would leave a compute unit room for
    one block only go to the other kernels, the rest stays."""
    rng = np.random.default_rng(M)
    lat = rng.integers(0, 5000, size=(6, 512, M), dtype=np.int32)
    totals = lat.sum(axis=2, dtype=np.int64)
    for count in (5000, 600):
        taus = rng.integers(int(totals.min()) // 2, int(totals.max()) + 10, size=count)
        check(lat, taus, 7, dev)
    check(lat, taus[:2500], 7, dev)


def test_short_rows_of_few_workers_many_trials_and_passes(dev):
    """The same path over many units and blocks, with more thresholds than one pass holds (every pass repeats the
    atomic maxima), twice on one workspace (the maxima are cleared per call), then through the entry point without
    a workspace."""
    rng = np.random.default_rng(4242)
    for T, N, M in ((30000, 20, 8), (25000, 12, 16), (600000, 4, 5)):   # rows of 8 and 16 elements take this path from 16 MB on; very many tiny trials
        lat = rng.integers(0, 5000, size=(T, N, M), dtype=np.int32)
        lat[rng.integers(0, T, 50), rng.integers(0, N, 50), :] = 30000
        totals = lat.sum(axis=2, dtype=np.int64)
        check(lat, rng.integers(int(totals.min()), int(totals.max()) + 10, size=200), 3, dev)
    T, N, M = 50000, 8, 12
    lat = rng.integers(0, 5000, size=(T, N, M), dtype=np.int32)
    lat[rng.integers(0, T, 50), rng.integers(0, N, 50), :] = 30000
    totals = lat.sum(axis=2, dtype=np.int64)
    taus = rng.integers(int(totals.min()), int(totals.max()) + 10, size=5000)
    lat_dev = to_dev(lat, dev)
    ref = oracle.simulate(lat, taus, 11)
    for scale in (1, 2):                                    # second call: smaller maxima on the same workspace
        step, done = dc.dc_simulate(lat_dev // (scale * scale) if scale > 1 else lat_dev, taus, 11)
        if scale == 1:
            assert np.array_equal(done, ref[1]) and np.array_equal(step, ref[0])
        else:
            ref2 = oracle.simulate(lat // 4, taus, 11)
            assert np.array_equal(done, ref2[1]) and np.array_equal(step, ref2[0])
    few = np.sort(taus[:100])
    taus_dev = torch.from_numpy(few).to(dev)
    out = torch.zeros((2, few.size), dtype=torch.int64, device=dev)
    flags = torch.zeros(1, dtype=torch.int32, device=dev)
    dc.dc_simulate_static(lat_dev, taus_dev, 11, out[0], out[1], flags)
    torch.cuda.synchronize()
    ref3 = oracle.simulate(lat, few, 11)
    assert int(flags.item()) == 0
    assert np.array_equal(out[0].cpu().numpy(), ref3[0]) and np.array_equal(out[1].cpu().numpy(), ref3[1])


def test_long_rows_and_many_rows_per_unit(dev):
    """Rows longer than a unit (one row per unit, carries across dozens of loads) and units of thousands of short rows."""
    rng = np.random.default_rng(12)
    for shape, top in (((3, 5, 20011), 100000), ((2, 3, 65536), 30000), ((3, 9001, 1), 10**9), ((2, 5000, 3), 10**8)):
        lat = rng.integers(0, min(top, (2**31 - 1) // shape[2]) + 1, size=shape, dtype=np.int32)
        totals = lat.sum(axis=2, dtype=np.int64)
        taus = np.concatenate([rng.integers(0, int(totals.max()) + 2, size=40), [int(totals.max()), int(totals.min())]])
        check(lat, taus, 2, dev)
        gs, gq, _, _ = dc.dc_worker_moments(to_dev(lat, dev)) if shape[1] <= 2560 else (None, None, None, None)
        if gs is not None:
            sums, squares, _, _ = oracle.worker_moments(lat)
            assert gs == sums and gq == squares


def test_unaligned_tensor(dev):
    rng = np.random.default_rng(77)
    lat = rng.integers(0, 3000, size=(5, 6, 64), dtype=np.int32)
    flat = torch.empty(lat.size + 1, dtype=torch.int32, device=dev)
    view = flat[1:].view(5, 6, 64)                         # 4-byte aligned, not 16-byte aligned
    view.copy_(torch.from_numpy(lat))
    assert view.data_ptr() % 16 == 4
    taus = np.sort(rng.integers(0, 64 * 3000, size=15))
    step, done = dc.dc_simulate(view, taus, 1)
    ref = oracle.simulate(lat, taus, 1, "literal")
    assert np.array_equal(step, ref[0]) and np.array_equal(done, ref[1])


# ---- random shapes, distributions and threshold lists -----------------------------------------------------------

@pytest.mark.parametrize("seed", range(40))
def test_random_cases_against_the_literal_oracle(seed, dev):
    rng = np.random.default_rng(1000 + seed)
    M = int(rng.choice([1, 2, 4, 7, 8, 12, 16, 20, 32, 48, 64, 96, 128, 200, 256, 260, 384]))
    N = int(rng.integers(1, 300))
    T = int(rng.integers(1, max(2, 60000 // (N * M) + 2)))
    top = min((2**31 - 1) // M, int(rng.choice([1, 10, 1000, 10**6, 10**9])))
    kind = rng.integers(0, 4)
    if kind == 0:
        lat = rng.integers(0, top + 1, size=(T, N, M))
    elif kind == 1:                                              # mostly equal rows: many ties with the thresholds
        lat = np.full((T, N, M), top // 2) + rng.integers(0, 2, size=(T, N, M))
    elif kind == 2:                                              # sparse: long runs of zero latency
        lat = rng.integers(0, top + 1, size=(T, N, M)) * (rng.random((T, N, M)) < 0.1)
    else:                                                        # heavy tail
        lat = np.minimum(top, (top / 50 * rng.pareto(1.5, size=(T, N, M))).astype(np.int64))
    lat = lat.astype(np.int32)
    P = np.cumsum(lat.astype(np.int64), axis=2)
    K = int(rng.choice([1, 2, 3, 17, 64, 300]))
    pool = np.concatenate([P.reshape(-1), P.reshape(-1) + 1, [0, 1, int(P.max()) + 5, BIG, 1 << 31]])
    taus = rng.choice(pool, size=K).astype(np.int64)             # thresholds on and next to completion times
    if K > 3 and rng.random() < 0.5:
        taus[rng.integers(0, K)] = int(P.max()) * 1000 + 7      # a far outlier
    comm = int(rng.integers(0, 1000))
    check(lat, taus, comm, dev, "literal")


def test_randomised_entry_points(dev):
    """A bounded, seeded sweep of random shapes, alignments, value ranges and threshold lists through the four entry
    points that stream the tensor (sums, per-iteration speedup, moments, per-worker statistics) and through a random
    range of workers, each against the oracle; stops at the first mismatch."""
    rng = np.random.default_rng(20260)
    for case in range(1500):
        M = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 13, 16, 24, 31, 32, 63, 64, 65, 100, 128, 132, 256, 257, 600]))
        N = int(rng.integers(1, 120)) if rng.random() < 0.85 else int(rng.choice([256, 257, 260, 512, 1022]))
        T = int(rng.integers(1, max(2, 40000 // (N * M) + 2)))
        if rng.random() < 0.3:
            T = (T + 3) // 4 * 4                                     # a multiple of 4 rows in all, whatever N
        top = min((2**31 - 1) // M, int(rng.choice([3, 100, 10**4, 10**6, 10**9])))
        lat = rng.integers(0, top + 1, size=(T, N, M), dtype=np.int64)
        if rng.random() < 0.3:
            lat *= rng.random((T, N, M)) < 0.2                       # long runs of zero latency
        lat = lat.astype(np.int32)
        words = int(rng.choice([0, 0, 0, 1, 2, 3]))                  # 0 (half of the cases), 4, 8 or 12 bytes past a 16-byte boundary
        flat = torch.full((lat.size + words + 4,), -3, dtype=torch.int32, device=dev)
        view = flat[words:words + lat.size].view(T, N, M)
        view.copy_(torch.from_numpy(lat))
        P = np.cumsum(lat.astype(np.int64), axis=2)
        K = int(rng.choice([1, 2, 5, 33, 130]))
        pool = np.concatenate([P.reshape(-1), P.reshape(-1) + 1, [1, int(P.max()) + 3, BIG]])
        taus = np.maximum(rng.choice(pool, size=K), 1).astype(np.int64)
        comm = int(rng.integers(0, 500))
        tag = (case, T, N, M, words, K)
        step, done = dc.dc_simulate(view, taus, comm)
        ref_step, ref_done = oracle.simulate(lat, taus, comm, "literal")
        assert np.array_equal(step, ref_step) and np.array_equal(done, ref_done), tag
        assert np.allclose(dc.dc_speedup_per_step(view, taus, comm), oracle.per_step_speedup(lat, taus, comm),
                           rtol=SPEEDUP_RTOL, atol=0), tag
        assert dc.dc_moments(view)[:2] == oracle.moments(lat)[1:3], tag
        assert dc.dc_worker_moments(view)[:2] == oracle.worker_moments(lat)[:2], tag
        n0 = int(rng.integers(0, N))
        n1 = int(rng.integers(n0 + 1, N + 1))
        part = np.ascontiguousarray(lat[:, n0:n1, :])
        step, done = dc.dc_simulate(view, taus, comm, workers=(n0, n1))
        ref_step, ref_done = oracle.simulate(part, taus, comm, "literal")
        assert np.array_equal(step, ref_step) and np.array_equal(done, ref_done), tag + (n0, n1)
        assert dc.dc_worker_moments(view, workers=(n0, n1))[:2] == oracle.worker_moments(part)[:2], tag + (n0, n1)


# ---- degenerate and adversarial inputs --------------------------------------------------------------

def test_thresholds_spanning_every_completion_time(dev):
    """Every element lies inside the grid: the histogram path handles all of them."""
    rng = np.random.default_rng(5)
    lat = rng.integers(0, 2000, size=(20, 96, 128), dtype=np.int32)
    taus = np.linspace(0, 128 * 2000, 300).astype(np.int64)
    check(lat, taus, 9, dev)


@pytest.mark.parametrize("M", [128, 256, 64, 100, 63])
def test_dense_grids_with_and_without_repeated_thresholds(M, dev):
    """Grids that cover most completion times, through both ways of finding a bin: evenly spaced thresholds (at
    most one per lookup cell), the same with repeats, with two far outliers, and an irregular list."""
    rng = np.random.default_rng(300 + M)
    lat = rng.integers(500, 1500, size=(24, 70, M), dtype=np.int32)
    top = int(lat.sum(axis=2, dtype=np.int64).max())
    even = np.linspace(0, top, 257).astype(np.int64)
    check(lat, even, 7, dev)
    check(lat, np.concatenate([even, even[::3]]), 7, dev)
    check(lat, np.concatenate([even, [BIG, top * 50]]), 7, dev)
    check(lat, np.concatenate([even[:100], rng.integers(0, top, size=300)]), 7, dev)
    check(lat, np.linspace(top // 2, top, 100).astype(np.int64), 7, dev)


def test_zero_latencies_and_constant_rows(dev):
    lat = np.zeros((4, 10, 32), dtype=np.int32)
    check(lat, [0, 1, 2], 4, dev, "literal")
    lat[:] = 5
    check(lat, [0, 5, 6, 160, 161, 159], 4, dev, "literal")


def test_single_threshold_and_no_thresholds(dev):
    rng = np.random.default_rng(6)
    lat = rng.integers(1, 100, size=(3, 5, 16), dtype=np.int32)
    check(lat, [400], 2, dev, "literal")
    step, done = dc.dc_simulate(to_dev(lat, dev), [], 2)
    assert step.size == 0 and done.size == 0


def test_more_thresholds_than_one_pass_holds(dev):
    rng = np.random.default_rng(8)
    lat = rng.integers(0, 4000, size=(6, 40, 64), dtype=np.int32)
    taus = rng.integers(0, 64 * 4000, size=9000)
    check(lat, taus, 3, dev)


def test_many_trials_with_scattered_maxima(dev):
    """Tens of thousands of trials whose maxima fall in every bin of the grid, and a trial count that is no multiple of 256."""
    rng = np.random.default_rng(9)
    T, N, M = 70001, 3, 8
    lat = (rng.integers(0, 500, size=(T, 1, 1)) + rng.integers(0, 20, size=(T, N, M))).astype(np.int32)
    taus = rng.integers(0, 8 * 520 + 2, size=700)
    check(lat, taus, 11, dev)
    check(np.ascontiguousarray(lat[:, :2, :7]), taus[:5], 0, dev)                      # odd row length, few thresholds


def test_largest_threshold_count(dev):
    rng = np.random.default_rng(10)
    lat = rng.integers(0, 3000, size=(5, 30, 32), dtype=np.int32)
    taus = rng.integers(0, 32 * 3000, size=dc.DC_MAX_THRESHOLDS)
    check(lat, taus, 3, dev)
    with pytest.raises(dc.DcError) as e:
        dc.dc_simulate(to_dev(lat, dev), np.zeros(dc.DC_MAX_THRESHOLDS + 1, dtype=np.int64), 0)
    assert e.value.status == dc.DC_ERR_INVALID_ARG


def test_largest_legal_latency(dev):
    M = 16
    top = (2**31 - 1) // M
    lat = np.full((2, 3, M), top, dtype=np.int32)
    taus = [top, top + 1, top * M, top * M + 1, 1 << 31, BIG]
    check(lat, taus, 0, dev, "literal")


def test_value_errors(dev):
    lat = np.ones((2, 4, 16), dtype=np.int32)
    bad = lat.copy(); bad[1, 2, 3] = -1
    with pytest.raises(dc.DcError) as e:
        dc.dc_simulate(to_dev(bad, dev), [5], 0)
    assert e.value.status == dc.DC_ERR_NEGATIVE_LATENCY
    big = lat.copy(); big[0, 0, 0] = (2**31 - 1) // 16 + 1
    with pytest.raises(dc.DcError) as e:
        dc.dc_simulate(to_dev(big, dev), [5], 0)
    assert e.value.status == dc.DC_ERR_RANGE
    for taus, comm in (([-1], 0), ([1], -1)):
        with pytest.raises(dc.DcError) as e:
            dc.dc_simulate(to_dev(lat, dev), taus, comm)
        assert e.value.status == dc.DC_ERR_INVALID_ARG
    with pytest.raises(oracle.OracleError):
        oracle.simulate(bad, [5], 0)
    # the library still works after an error
    check(lat, [5, 17], 1, dev, "literal")


# ---- the stream-ordered entry point ------------------------------------------------------------------

def test_async_entry_point_on_a_side_stream(dev):
    r = config("extrapolation2048").with_shape(T=12, K=100)
    lat = host.generate(r)
    taus = host.tau_grid(r)
    ref = oracle.simulate(lat, taus, r.comm, "sorted")
    lat_d = to_dev(lat, dev)
    taus_d = torch.from_numpy(taus).to(dev)
    out_step = torch.zeros(taus.size, dtype=torch.int64, device=dev)
    out_done = torch.zeros(taus.size, dtype=torch.int64, device=dev)
    ws = torch.empty(dc.dc_workspace_bytes(r.T, r.N, r.M, taus.size), dtype=torch.uint8, device=dev)
    ws.fill_(0xAB)                                          # contents on entry are irrelevant
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    for _ in range(3):                                      # reuse of the workspace
        dc.dc_simulate_async(lat_d, taus_d, r.comm, out_step, out_done, ws, stream)
        assert dc.dc_workspace_status(ws, stream) == dc.DC_OK
        assert np.array_equal(out_step.cpu().numpy(), ref[0]) and np.array_equal(out_done.cpu().numpy(), ref[1])
    pinned = torch.zeros((2, taus.size), dtype=torch.int64).pin_memory()   # outputs straight into host memory, no copy
    for _ in range(3):
        pinned.zero_()
        dc.dc_simulate_async(lat_d, taus_d, r.comm, pinned[0], pinned[1], ws, stream)
        stream.synchronize()
        assert np.array_equal(pinned[0].numpy(), ref[0]) and np.array_equal(pinned[1].numpy(), ref[1])
    with pytest.raises(TypeError):
        dc.dc_simulate_async(lat_d, taus_d, r.comm, torch.zeros(taus.size, dtype=torch.int64), pinned[1], ws, stream)
    taus_d[3] = -5
    dc.dc_simulate_async(lat_d, taus_d, r.comm, out_step, out_done, ws, stream)
    assert dc.dc_workspace_status(ws, stream) == dc.DC_ERR_INVALID_ARG
    taus_d[3] = 5
    for _ in range(20):                                     # a negative threshold far from the head of the list
        taus_d[77] = -1
        dc.dc_simulate_async(lat_d, taus_d, r.comm, out_step, out_done, ws, stream)
        assert dc.dc_workspace_status(ws, stream) == dc.DC_ERR_INVALID_ARG
        taus_d[77] = int(taus[77])
        dc.dc_simulate_async(lat_d, taus_d, r.comm, out_step, out_done, ws, stream)
        assert dc.dc_workspace_status(ws, stream) == dc.DC_OK
    small = torch.empty(256, dtype=torch.uint8, device=dev)
    with pytest.raises(dc.DcError):
        dc.dc_simulate_async(lat_d, taus_d, r.comm, out_step, out_done, small, stream)


def test_prepared_calls_of_the_binding(dev):
    """The binding's prepared calls (arguments marshalled once) give what the plain wrappers give, call after call,
    also on a range of workers, and follow the contents of the tensors they were prepared on."""
    r = config("lognormal64").with_shape(T=300)
    lat = host.generate(r)
    taus = host.tau_grid(r)
    lat_d, taus_d = to_dev(lat, dev), torch.from_numpy(taus).to(dev)
    out = torch.zeros((2, taus.size), dtype=torch.int64).pin_memory()
    step_h, done_h = out[0].numpy(), out[1].numpy()
    ws = torch.empty(dc.dc_workspace_bytes(r.T, r.N, r.M, taus.size), dtype=torch.uint8, device=dev)
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()
    sim = dc.PreparedSimulation(lat_d, taus_d, r.comm, out[0], out[1], ws, stream)
    sel = dc.PreparedSelection(step_h, done_h, taus, r.T, r.N, r.M)
    for scale in (1, 2, 1):
        lat_d.copy_(torch.from_numpy(lat // scale))
        torch.cuda.synchronize()
        sim.enqueue()
        stream.synchronize()
        ref_step, ref_done = oracle.simulate(lat // scale, taus, r.comm)
        assert np.array_equal(step_h, ref_step) and np.array_equal(done_h, ref_done)
        thr, seff, best = sel.select()
        othr, oseff, obest = oracle.select_tau(ref_step, ref_done, taus, r.T, r.N, r.M)
        assert best == obest and np.allclose(thr, othr, rtol=1e-6, atol=0)
        assert np.allclose(seff, oseff, rtol=1e-6, atol=0, equal_nan=True)      # no no-drop baseline given: not a number on both sides
    part = dc.PreparedSimulation(lat_d, taus_d, r.comm, out[0], out[1], ws, stream, workers=(8, 40))
    part.enqueue()
    stream.synchronize()
    ref_step, ref_done = oracle.simulate(np.ascontiguousarray(lat[:, 8:40]), taus, r.comm)
    assert np.array_equal(step_h, ref_step) and np.array_equal(done_h, ref_done)
    with pytest.raises(TypeError):
        dc.PreparedSelection(list(step_h), done_h, taus, r.T, r.N, r.M)


def test_async_entry_point_replays_from_a_graph(dev):
    """The enqueued sequence uses no memset and no allocation, so it can be captured; every replay must
    reproduce the eager result, with other work and synchronisations in between."""
    r = config("lognormal64").with_shape(T=500)
    lat = host.generate(r)
    taus = host.tau_grid(r)
    ref = oracle.simulate(lat, taus, r.comm, "sorted")
    lat_d, taus_d = to_dev(lat, dev), torch.from_numpy(taus).to(dev)
    out = torch.zeros((2, taus.size), dtype=torch.int64, device=dev)
    ws = torch.empty(dc.dc_workspace_bytes(r.T, r.N, r.M, taus.size), dtype=torch.uint8, device=dev)
    side = torch.cuda.Stream()
    dc.dc_simulate_async(lat_d, taus_d, r.comm, out[0], out[1], ws, side)        # eager once (warms caches of the plan)
    assert dc.dc_workspace_status(ws, side) == dc.DC_OK
    eager = out.cpu().numpy().copy()
    assert np.array_equal(eager[0], ref[0]) and np.array_equal(eager[1], ref[1])
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        dc.dc_simulate_async(lat_d, taus_d, r.comm, out[0], out[1], ws, torch.cuda.current_stream())
    for i in range(4):
        out.zero_()
        ws.fill_(i)                                          # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), eager), i


def test_kernel_timing_reports_positive_times(dev):
    r = config("extrapolation2048").with_shape(T=16)
    from dc_workloads import device
    lat_d = device.generate(r)
    taus = host.tau_grid(r)
    try:
        dc.dc_set_kernel_timing(2)
        dc.dc_simulate(lat_d, taus, r.comm)
        scan_ms, total_ms = dc.dc_last_kernel_ms(whole=True)
        assert 0 < scan_ms <= total_ms
        dc.dc_set_kernel_timing(1)
        dc.dc_simulate(lat_d, taus, r.comm)
        assert dc.dc_last_kernel_ms()[0] > 0
        with pytest.raises(dc.DcError):
            dc.dc_last_kernel_ms(whole=True)
    finally:
        dc.dc_set_kernel_timing(False)


# ---- Algorithm 2 as printed: mean over iterations of the per-iteration speedup -------------------------



@pytest.mark.parametrize("name,shape", [
    ("tiny", {"T": 200}),
    ("lognormal64", {"T": 60}),
    ("lognormal64", {"T": 9, "N": 61}),
    ("additive200", {"T": 12, "N": 203}),
    ("extrapolation2048", {"T": 5}),
    ("heterogeneous2048", {"T": 3, "N": 1000}),
])
def test_per_step_speedup_parity(name, shape, dev):
    r = config(name).with_shape(**shape, K=24)
    lat = host.generate(r)
    rng = np.random.default_rng(2)
    taus = extra_thresholds(host.tau_grid(r), rng)
    taus = taus[taus > 0]                                       # tau = 0 with comm = 0 would divide by zero
    got = dc.dc_speedup_per_step(to_dev(lat, dev), taus, r.comm)
    ref = oracle.per_step_speedup(lat, taus, r.comm)
    assert np.allclose(got, ref, rtol=SPEEDUP_RTOL, atol=0)
    assert np.allclose(got, ref, rtol=1e-11, atol=0)            # what the arithmetic actually delivers
    comm_t = rng.integers(0, 2 * r.comm + 1, size=r.T)
    got = dc.dc_speedup_per_step(to_dev(lat, dev), taus, 0, comm_t)
    ref = oracle.per_step_speedup(lat, taus, comm_t)
    assert np.allclose(got, ref, rtol=SPEEDUP_RTOL, atol=0)
    again = dc.dc_speedup_per_step(to_dev(lat, dev), taus, 0, comm_t)
    assert np.array_equal(got, again)                           # fixed summation order


@pytest.mark.parametrize("M", [1, 3, 12, 100, 300, 8, 64, 20, 252])
def test_per_step_speedup_shapes(M, dev):
    rng = np.random.default_rng(100 + M)
    lat = rng.integers(1, 3000, size=(7, 9, M), dtype=np.int32)
    totals = lat.sum(axis=2, dtype=np.int64)
    taus = rng.integers(1, int(totals.max()) + 50, size=19)
    got = dc.dc_speedup_per_step(to_dev(lat, dev), taus, 11)
    assert np.allclose(got, oracle.per_step_speedup(lat, taus, 11), rtol=SPEEDUP_RTOL, atol=0)


@pytest.mark.parametrize("N,M,K", [(8, 16, 40), (64, 12, 100), (64, 32, 511), (200, 64, 128), (7, 256, 33), (33, 4, 512),
                                   (64, 13, 100), (200, 5, 64), (9, 1, 20), (40, 3, 511), (17, 257, 50), (30, 2, 77)])
def test_per_step_speedup_small_trials(N, M, K, dev):
    """Trials of a few KiB: every wave owns a trial (up to 511 thresholds; 512 go the other way).  More trials than
    the grid has waves, a trial of zeros, one of the largest legal rows, per-iteration communication times."""
    rng = np.random.default_rng(N * 1000 + M)
    T = 9000
    top = min((2**31 - 1) // M, 5000)
    lat = rng.integers(0, top + 1, size=(T, N, M), dtype=np.int32)
    lat[3] = 0
    lat[T - 1, N - 1, :] = (2**31 - 1) // M
    totals = lat.sum(axis=2, dtype=np.int64)
    taus = np.concatenate([[1, BIG], rng.integers(1, int(np.quantile(totals, 0.999)) + 50, size=K - 2)])
    comm_t = rng.integers(1, 4000, size=T)
    lat_dev = to_dev(lat, dev)
    got = dc.dc_speedup_per_step(lat_dev, taus, 0, comm_t)
    ref = oracle.per_step_speedup(lat, taus, comm_t, threads=8)
    assert np.allclose(got, ref, rtol=SPEEDUP_RTOL, atol=0)
    assert np.allclose(got, ref, rtol=1e-11, atol=0)
    assert np.array_equal(got, dc.dc_speedup_per_step(lat_dev, taus, 0, comm_t))       # fixed summation order
    got = dc.dc_speedup_per_step(lat_dev, taus, 17)
    assert np.allclose(got, oracle.per_step_speedup(lat, taus, 17, threads=8), rtol=SPEEDUP_RTOL, atol=0)


@pytest.mark.parametrize("N,M,K", [(8, 32, 40), (16, 32, 33), (24, 32, 20), (32, 32, 25), (4, 256, 64), (3, 256, 30),
                                   (64, 4, 30), (12, 20, 25), (2, 128, 50), (128, 8, 20)])
def test_per_step_speedup_trials_of_a_few_loads(N, M, K, dev):
    """Trials of one to four 1 KiB loads, many more than the grid has waves: a wave requests the loads of its next
    few trials together and finishes the trials one after the other.  A trial count that leaves the last batch short,
    a trial of zeros, one of the largest legal rows, per-iteration communication times, identical bits on a repeat."""
    rng = np.random.default_rng(N * 1000 + M)
    T = 8 * 8192 + int(rng.integers(5000, 9000))
    top = min((2**31 - 1) // M, 5000)
    lat = rng.integers(0, top + 1, size=(T, N, M), dtype=np.int32)
    lat[3] = 0
    lat[T - 1, N - 1, :] = (2**31 - 1) // M
    totals = lat.sum(axis=2, dtype=np.int64)
    taus = np.concatenate([[1, BIG], rng.integers(1, int(np.quantile(totals, 0.999)) + 50, size=K - 2)])
    comm_t = rng.integers(1, 4000, size=T)
    lat_dev = to_dev(lat, dev)
    got = dc.dc_speedup_per_step(lat_dev, taus, 0, comm_t)
    ref = oracle.per_step_speedup(lat, taus, comm_t, threads=8)
    assert np.allclose(got, ref, rtol=1e-11, atol=0)
    assert np.array_equal(got, dc.dc_speedup_per_step(lat_dev, taus, 0, comm_t))       # fixed summation order
    got = dc.dc_speedup_per_step(lat_dev, taus, 17)
    assert np.allclose(got, oracle.per_step_speedup(lat, taus, 17, threads=8), rtol=SPEEDUP_RTOL, atol=0)


def test_per_step_speedup_many_trials_and_thresholds(dev):
    """More trials than blocks, more thresholds than one pass holds."""
    rng = np.random.default_rng(9)
    lat = rng.integers(0, 4000, size=(1500, 24, 16), dtype=np.int32)
    taus = rng.integers(1, 16 * 4000, size=2500)
    got = dc.dc_speedup_per_step(to_dev(lat, dev), taus, 40)
    ref = oracle.per_step_speedup(lat, taus, 40)
    assert np.allclose(got, ref, rtol=SPEEDUP_RTOL, atol=0)
    assert dc.dc_speedup_per_step(to_dev(lat, dev), [BIG], 40)[0] == pytest.approx(1.0, abs=1e-12)


def test_per_step_speedup_errors_and_async(dev):
    lat = np.ones((3, 4, 16), dtype=np.int32)
    with pytest.raises(dc.DcError) as e:                        # tau = 0 and comm = 0: step time 0
        dc.dc_speedup_per_step(to_dev(lat, dev), [0, 5], 0)
    assert e.value.status == dc.DC_ERR_INVALID_ARG
    with pytest.raises(dc.DcError):
        dc.dc_speedup_per_step(to_dev(lat, dev), [5], 0, [1, -1, 1])
    bad = lat.copy(); bad[2, 1, 5] = -3
    with pytest.raises(dc.DcError) as e:
        dc.dc_speedup_per_step(to_dev(bad, dev), [5], 1)
    assert e.value.status == dc.DC_ERR_NEGATIVE_LATENCY
    r = config("extrapolation2048").with_shape(T=6, K=40)
    lat = host.generate(r)
    taus = host.tau_grid(r)
    lat_d, taus_d = to_dev(lat, dev), torch.from_numpy(taus).to(dev)
    out = torch.zeros(taus.size, dtype=torch.float64, device=dev)
    ws = torch.empty(dc.dc_speedup_workspace_bytes(r.T, r.N, r.M, taus.size), dtype=torch.uint8, device=dev)
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()
    dc.dc_speedup_per_step_async(lat_d, taus_d, r.comm, None, out, ws, stream)
    assert dc.dc_workspace_status(ws, stream) == dc.DC_OK
    ref = oracle.per_step_speedup(lat, taus, r.comm)
    assert np.allclose(out.cpu().numpy(), ref, rtol=SPEEDUP_RTOL, atol=0)
    pinned = torch.zeros(taus.size, dtype=torch.float64).pin_memory()      # the result written straight to the host
    dc.dc_speedup_per_step_async(lat_d, taus_d, r.comm, None, pinned, ws, stream)
    assert dc.dc_workspace_status(ws, stream) == dc.DC_OK
    assert np.array_equal(pinned.numpy(), out.cpu().numpy())
    pinned.zero_()                                                         # the same through the binding's prepared call
    call = dc.PreparedSpeedup(lat_d, taus_d, r.comm, None, pinned, ws, stream, taus_host=taus)
    for _ in range(2):
        call.enqueue()
        stream.synchronize()
        assert np.array_equal(pinned.numpy(), out.cpu().numpy())
        assert call.select() == oracle.per_step_best(ref, taus)


# ---- analytical side: exact moments, closed-form curves ----------------------------------------------------

@pytest.mark.parametrize("shape", [(3, 5, 7), (40, 64, 128), (9, 200, 64), (2, 2048, 256), (1, 1, 1), (5, 33, 1000)])
def test_moments_are_exact(shape, dev):
    rng = np.random.default_rng(sum(shape))
    top = (2**31 - 1) // shape[2]
    lat = rng.integers(0, top + 1, size=shape, dtype=np.int32)
    n, s, q, mean, var = oracle.moments(lat)
    gs, gq, gmean, gvar = dc.dc_moments(to_dev(lat, dev))
    assert (gs, gq) == (s, q)
    assert gmean == pytest.approx(mean, rel=1e-14) and gvar == pytest.approx(var, rel=1e-12)


def test_moments_of_a_workload_and_errors(dev):
    from dc_workloads import device
    r = config("heterogeneous2048").with_shape(T=24)
    gs, gq, gmean, gvar = dc.dc_moments(device.generate(r))
    n, s, q, mean, var = oracle.moments(host.generate(r))
    assert (gs, gq) == (s, q) and gvar == pytest.approx(var, rel=1e-12)
    big = np.full((2, 3, 4), 2**31 - 1, dtype=np.int32)                    # squares overflow 64 bits
    assert dc.dc_moments(to_dev(big, dev))[:2] == (24 * (2**31 - 1), 24 * (2**31 - 1) ** 2)
    bad = np.ones((2, 3, 4), dtype=np.int32); bad[1, 1, 1] = -7
    with pytest.raises(dc.DcError) as e:
        dc.dc_moments(to_dev(bad, dev))
    assert e.value.status == dc.DC_ERR_NEGATIVE_LATENCY
    flat = torch.ones(4 * 5 * 64 + 1, dtype=torch.int32, device=dev)       # unaligned tensor
    assert dc.dc_moments(flat[1:].view(4, 5, 64))[:2] == (1280, 1280)


@pytest.mark.parametrize("shape", [(30, 64, 32), (7, 200, 64), (3, 2048, 256), (5, 2047, 128), (40, 33, 12),
                                   (9, 10, 100), (6, 9, 300), (11, 5, 1), (4, 2560, 16), (11, 50, 7), (20, 100, 3),
                                   (6, 170, 2), (4, 9, 257), (3, 2, 5000),
                                   # trials of one to three whole loads (a wave takes whole trials), few and many trials
                                   (3, 8, 32), (5000, 8, 32), (4099, 16, 32), (3001, 24, 32), (2500, 4, 64), (2222, 2, 128),
                                   (2601, 12, 20), (2048, 3, 256), (1234, 64, 4), (700, 96, 8),
                                   # worker counts that are no whole number of full loads: shorter loads
                                   (3000, 32, 20), (2000, 8, 20), (1500, 16, 24), (1800, 4, 32), (900, 40, 36), (1100, 6, 64)])
def test_worker_moments_are_exact(shape, dev):
    rng = np.random.default_rng(sum(shape))
    top = (2**31 - 1) // shape[2]
    lat = rng.integers(0, top + 1, size=shape, dtype=np.int32)
    sums, squares, mean, var = oracle.worker_moments(lat)
    gs, gq, gmean, gvar = dc.dc_worker_moments(to_dev(lat, dev))
    assert gs == sums and gq == squares
    assert np.allclose(gmean, mean, rtol=1e-14) and np.allclose(gvar, var, rtol=1e-12, atol=0)


def test_worker_moments_of_a_workload_and_errors(dev):
    r = config("heterogeneous2048").with_shape(T=20)
    lat = host.generate(r)
    sums, squares, mean, var = oracle.worker_moments(lat)
    gs, gq, gmean, gvar = dc.dc_worker_moments(to_dev(lat, dev))
    assert gs == sums and gq == squares
    bad = np.ones((2, 3, 8), dtype=np.int32); bad[1, 2, 7] = -1
    with pytest.raises(dc.DcError) as e:
        dc.dc_worker_moments(to_dev(bad, dev))
    assert e.value.status == dc.DC_ERR_NEGATIVE_LATENCY


def test_worker_moments_of_more_workers_than_one_pass_holds(dev):
    """The accumulators of 2560 workers fill the LDS; more workers take several passes over their rows."""
    rng = np.random.default_rng(44)
    for shape in ((5, 6000, 4), (3, 2561, 7), (2, 5121, 1)):
        lat = rng.integers(0, (2**31 - 1) // shape[2] + 1, size=shape, dtype=np.int32)
        sums, squares, mean, var = oracle.worker_moments(lat)
        gs, gq, gmean, gvar = dc.dc_worker_moments(to_dev(lat, dev))
        assert gs == sums and gq == squares, shape
        assert np.allclose(gmean, mean, rtol=1e-14) and np.allclose(gvar, var, rtol=1e-12, atol=0)


# ---- a range of workers of a resident tensor, without a copy (trial stride) -----------------------------------

@pytest.mark.parametrize("shape,ranges", [
    ((9, 64, 32), [(0, 64), (0, 17), (5, 40), (63, 64)]),          # whole rows per load; every start is 16-byte aligned
    ((7, 50, 128), [(0, 8), (3, 50)]),                             # long rows, two launch shapes
    ((6, 40, 12), [(0, 9), (7, 33)]),                              # three lanes per row
    ((8, 33, 7), [(0, 33), (0, 5), (2, 30), (32, 33)]),            # odd rows, odd stride: the kernel for any alignment
    ((5, 21, 1), [(0, 8), (1, 20)]),
    ((4, 10, 257), [(0, 3), (4, 9)]),
    ((3, 2100, 256), [(0, 2048), (52, 2100)]),
    ((400, 40, 13), [(0, 8), (4, 24), (0, 40)]),                   # short rows: another kernel than the contiguous tensor of that shape takes
    ((64, 600, 6), [(0, 256), (8, 520), (3, 259)]),
])
def test_worker_ranges_of_a_resident_tensor(shape, ranges, dev):
    rng = np.random.default_rng(sum(shape))
    lat = rng.integers(0, 4000, size=shape, dtype=np.int32)
    lat_d = to_dev(lat, dev)
    T, N, M = shape
    for n0, n1 in ranges:
        part = np.ascontiguousarray(lat[:, n0:n1, :])
        top = int(part.sum(axis=2, dtype=np.int64).max())
        taus = np.concatenate([rng.integers(0, top + 9, size=30), [0, BIG, top]]).astype(np.int64)
        step, done = dc.dc_simulate(lat_d, taus, 11, workers=(n0, n1))
        ref_step, ref_done = oracle.simulate(part, taus, 11, "literal")
        assert np.array_equal(step, ref_step) and np.array_equal(done, ref_done), (shape, n0, n1)
        sums, squares, _, _ = oracle.worker_moments(part)
        gs, gq, _, _ = dc.dc_worker_moments(lat_d, workers=(n0, n1))
        assert gs == sums and gq == squares, (shape, n0, n1)
        # the stream-ordered form, with negative guard values around the slab's rows to show a stray read
        taus_d = torch.from_numpy(taus).to(dev)
        out = torch.zeros((2, taus.size), dtype=torch.int64, device=dev)
        ws = torch.empty(dc.dc_workspace_bytes(T, n1 - n0, M, taus.size), dtype=torch.uint8, device=dev)
        guarded = torch.full((T, N, M), -9, dtype=torch.int32, device=dev)
        guarded[:, n0:n1, :] = lat_d[:, n0:n1, :]
        dc.dc_simulate_async(guarded, taus_d, 11, out[0], out[1], ws, None, workers=(n0, n1))
        assert dc.dc_workspace_status(ws, None) == dc.DC_OK
        assert np.array_equal(out[0].cpu().numpy(), ref_step) and np.array_equal(out[1].cpu().numpy(), ref_done)
    with pytest.raises(dc.DcError) as e:                          # a stride shorter than a trial
        dc._check(dc._load().dc_simulate_strided(lat_d.data_ptr(), T, N, M, N * M - 1, None, 0, 0, None, None), "strided")
    assert e.value.status == dc.DC_ERR_INVALID_ARG


@pytest.mark.parametrize("family", ["normal", "lognormal"])
def test_noise_study_sweep_against_the_oracle(family, dev):
    """The scale sweep of paper_2306_10598_amd/examples/noise_study.py (first n workers of one resident tensor, n = 4
    and 16) against the same quantities from the oracle's outputs on the sliced CPU tensor: E[T]/E[T_i] (Appendix
    C.3's ratio) and S_eff at the chosen threshold."""
    from dc_workloads import noise, spec
    from paper_2306_10598_amd.examples import noise_study
    r = noise.additive_noise(family, 200, 16, K=24)
    rows = noise_study.sweep(r, [4, 16])
    lat = host.generate(r)
    for row in rows:
        n = row["workers"]
        part = np.ascontiguousarray(lat[:, :n, :])
        totals = host.worker_totals(part)
        i_lo, i_hi = spec.grid_rank_indices(totals.size, r.grid)
        ordered = np.sort(totals)
        taus = np.append(spec.tau_grid((int(ordered[i_lo]), int(ordered[i_hi])), r.K), BIG)
        step, done = oracle.simulate(part, taus, r.comm, "sorted")
        _, seff, best = oracle.select_tau(step, done, taus, r.T, n, r.M, int(step[-1]))
        sums, _, _, _ = oracle.worker_moments(part)
        mean_tmax = (int(step[-1]) - r.T * r.comm) / r.T
        assert row["tau"] == int(taus[best])
        assert row["seff"] == pytest.approx(float(seff[best]), rel=1e-9)
        assert row["ratio"] == pytest.approx(mean_tmax / (sum(sums) / (r.T * n)), rel=1e-12)
        assert row["completed"] == pytest.approx(int(done[best]) / (r.T * n * r.M), rel=1e-12)
    assert rows[1]["ratio"] > rows[0]["ratio"] > 1.0            # the slowest of more workers takes longer (Section 4.2)


def test_two_streams_with_their_own_workspaces(dev):
    """Calls enqueued alternately on two streams, each with its own workspace: both results against the oracle, and
    each workspace's kernel times read back separately."""
    ra = config("extrapolation2048").with_shape(T=64, K=100)
    rb = config("lognormal64").with_shape(T=3000, K=60)
    cases = []
    for r in (ra, rb):
        lat = host.generate(r)
        taus = host.tau_grid(r)
        cases.append({"r": r, "ref": oracle.simulate_threaded(lat, taus, r.comm, "sorted", host.cpu_threads()),
                      "lat": to_dev(lat, dev), "taus": torch.from_numpy(taus).to(dev),
                      "out": torch.zeros((2, taus.size), dtype=torch.int64, device=dev),
                      "ws": torch.empty(dc.dc_workspace_bytes(r.T, r.N, r.M, taus.size), dtype=torch.uint8, device=dev),
                      "stream": torch.cuda.Stream()})
    torch.cuda.synchronize()
    try:
        dc.dc_set_kernel_timing(2)
        for _ in range(5):
            for c in cases:
                dc.dc_simulate_async(c["lat"], c["taus"], c["r"].comm, c["out"][0], c["out"][1], c["ws"], c["stream"])
        times = []
        for c in cases:
            assert dc.dc_workspace_status(c["ws"], c["stream"]) == dc.DC_OK
            got = c["out"].cpu().numpy()
            assert np.array_equal(got[0], c["ref"][0]) and np.array_equal(got[1], c["ref"][1]), c["r"].name
            scan_ms, total_ms = dc.dc_workspace_kernel_ms(c["ws"], whole=True)
            assert 0 < scan_ms <= total_ms
            times.append(scan_ms)
        assert times[0] != times[1]                                # two tensors of different size: two different clocks
    finally:
        dc.dc_set_kernel_timing(False)


def test_moments_sum_range(dev):
    """2^32 latencies of 2^31 - 1: the largest sum that is still shown to fit 63 bits; one trial more is refused."""
    top = 2**31 - 1
    lat = torch.full(((1 << 16) + 1, 1 << 8, 1 << 8), top, dtype=torch.int32, device=dev)      # 17 GB
    n = 1 << 32
    total, squares, mean, var = dc.dc_moments(lat[: 1 << 16])
    assert (total, squares) == (n * top, n * top * top) and mean == float(top) and var == 0.0
    with pytest.raises(dc.DcError) as e:
        dc.dc_moments(lat)
    assert e.value.status == dc.DC_ERR_RANGE
    del lat
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name", ["lognormal64", "extrapolation2048", "heterogeneous2048"])
def test_analytic_curves_parity(name, dev):
    r = config(name).with_shape(T=6)
    lat = host.generate(r)
    n, s, q, mean, var = oracle.moments(lat)
    taus = np.concatenate([host.tau_grid(r), [0, BIG, int(r.M * mean / 2)]]).astype(np.int64)
    for mean_tmax in (None, 1.01 * r.M * mean):
        e_done, e_t, s_eff, best = dc.dc_analytic_curves(mean, var, r.N, r.M, taus, r.comm, mean_tmax)
        o_done, o_t, o_seff, o_best = oracle.analytic_curves(mean, var, r.N, r.M, taus, r.comm, mean_tmax)
        assert np.allclose(e_done, o_done, rtol=1e-6, atol=0) and np.allclose(e_done, o_done, rtol=1e-11, atol=1e-13)
        assert e_t == pytest.approx(o_t, rel=1e-12)
        assert np.allclose(s_eff, o_seff, rtol=1e-6, atol=0)
        assert best == o_best
    e_done, _, _, _ = dc.dc_analytic_curves(10.0, 0.0, 4, 5, [10, 11, 30, 31, 1000], 1)
    assert e_done.tolist() == [0.0, 1.0, 2.0, 3.0, 5.0]


# ---- the paper's own noise models as workloads ----------------------------------------------------------------

@pytest.mark.parametrize("family", ["delay", "lognormal", "normal", "bernoulli", "exponential", "gamma"])
def test_noise_model_workloads_parity(family, dev):
    from dc_workloads import device, noise
    r = noise.simulated_delay(300, 64) if family == "delay" else noise.additive_noise(family, 300, 64)
    lat = host.generate(r)
    assert np.array_equal(device.generate(r).cpu().numpy(), lat)
    taus = np.append(host.tau_grid(r), BIG)
    assert np.array_equal(device.tau_grid(r, device.generate(r)), taus[:-1])
    step, done = check(lat, taus, r.comm, dev)                  # M = 12: three lanes per row
    assert np.allclose(dc.dc_speedup_per_step(to_dev(lat, dev), taus, r.comm),
                       oracle.per_step_speedup(lat, taus, r.comm), rtol=SPEEDUP_RTOL, atol=0)
    assert dc.dc_moments(to_dev(lat, dev))[:2] == oracle.moments(lat)[1:3]


@pytest.mark.parametrize("scenario,period", [("uniform", 1), ("uniform", 8), ("single_server", 16), ("single_server", 5)])
def test_local_sgd_workloads_parity(scenario, period, dev):
    from dc_workloads import device, noise
    r = noise.local_sgd(700, period, scenario)
    lat = host.generate(r)
    assert np.array_equal(device.generate(r).cpu().numpy(), lat)
    taus = np.append(host.tau_grid(r), BIG)
    check(lat, taus, r.comm, dev, "literal")


def test_per_worker_normal_surrogate_parity(dev):
    from dc_workloads import device, noise
    r0 = config("heterogeneous2048").with_shape(T=60, N=96, M=64)
    _, _, mean, var = dc.dc_worker_moments(device.generate(r0))
    r = noise.per_worker_normal(3000, mean, np.sqrt(var), comm_us=r0.comm)
    lat = host.generate(r)
    assert np.array_equal(device.generate(r).cpu().numpy(), lat)
    taus = np.append(host.tau_grid(r), BIG)
    check(lat, taus, r.comm, dev)                                # M = 1


# ---- full sizes of the two 2048-worker workloads, as the benchmark launches them -----------------------

LITERAL_FULL_EVALS = 2.0e10      # the four-loop oracle runs on the whole tensor up to this many (t, n, m, tau) combinations


@pytest.mark.parametrize("name,rows", [("tiny", 0), ("lognormal64", 0), ("additive200", 0), ("extrapolation2048", 0),
                                       ("heterogeneous2048", 0), ("heterogeneous2048", 65), ("heterogeneous2048", 63),
                                       ("extrapolation2048", 5),
                                       ("extrapolation2048", 16), ("additive200", 13), ("lognormal64", 12),
                                       ("heterogeneous2048", 5)])
def test_full_size_parity(name, rows, dev):
    """All five workloads at their stated size, in the launch configuration the benchmark times, against the
    sorted-walk oracle on the whole tensor; the three smaller ones also against the four-loop oracle on the whole
    tensor (the two 2048-worker ones on a sampled slab).  The largest runs once more with 65 accumulations per worker
    (same bytes, more than 2^32 elements through the kernel for arbitrary row lengths), with 63 (the kernel with one
    row per lane) and with 5 (the kernel in which every lane holds several whole rows); the 4.3 GB one with 5 and 16, the two middle ones with 13 and 12 (the same over trials of few workers)."""
    from dc_workloads import device
    r = config(name)
    if rows:
        r = r.with_shape(T=r.T * r.M // rows, M=rows)
    threads = host.cpu_threads()
    progress(f"{name}: generating {r.nbytes / 1e9:.1f} GB on the GPU")
    lat_d = device.generate(r)
    grid_dev = device.tau_grid(r, lat_d)

    # CPU side, streamed in chunks: totals for the grid, then the oracle's sums
    totals = np.empty(r.T * r.N, dtype=np.int64)
    chunks = list(host.trial_chunks(r, 512 << 20))
    import psutil
    keep = psutil.virtual_memory().available > r.nbytes + (16 << 30)   # hold the CPU tensor if RAM allows
    kept = {}
    for i, (t0, t1) in enumerate(chunks):
        lat = host.generate(r, t0, t1, threads)
        if keep:
            kept[t0] = lat
        totals[t0 * r.N:t1 * r.N] = host.worker_totals(lat)
        if i % 8 == 0:                                       # sampled chunks: the tensors themselves agree
            assert np.array_equal(lat_d[t0:t1].cpu().numpy(), lat), (name, t0)
        progress(f"{name}: totals chunk {i + 1}/{len(chunks)}")
    taus = host.tau_grid_from_totals(r, totals)
    assert np.array_equal(taus, grid_dev)
    taus = np.concatenate([taus, [BIG, 0, int(taus[taus.size // 3])]])      # edge thresholds and a repeat

    step, done = dc.dc_simulate(lat_d, taus, r.comm)
    literal_full = r.elements * taus.size <= LITERAL_FULL_EVALS
    ref_step = np.zeros(taus.size, dtype=np.int64)
    ref_done = np.zeros(taus.size, dtype=np.int64)
    lit_step, lit_done = ref_step.copy(), ref_done.copy()
    for i, (t0, t1) in enumerate(chunks):
        lat = kept.pop(t0) if keep else host.generate(r, t0, t1, threads)
        s, d = oracle.simulate_threaded(lat, taus, r.comm, "sorted", threads)
        ref_step += s
        ref_done += d
        if literal_full:
            s, d = oracle.simulate_threaded(lat, taus, r.comm, "literal", threads)
            lit_step += s
            lit_done += d
        progress(f"{name}: oracle chunk {i + 1}/{len(chunks)}")
    assert np.array_equal(done, ref_done) and np.array_equal(step, ref_step)
    assert done[-3] == r.elements and done[-2] == 0
    if literal_full:
        assert np.array_equal(done, lit_done) and np.array_equal(step, lit_step)
    else:                                                    # four-loop oracle on a few trials, same slab through the library
        sample = slice(r.T // 2, r.T // 2 + 2)
        some = taus[:: max(1, taus.size // 16)]
        s, d = dc.dc_simulate(lat_d[sample], some, r.comm)
        rs, rd = oracle.simulate(host.generate(r, sample.start, sample.stop), some, r.comm, "literal")
        assert np.array_equal(s, rs) and np.array_equal(d, rd)
    # the choice of the threshold from the full-size sums
    base = int(step[-3])
    thr, seff, best = dc.dc_select_tau(step, done, taus, r.T, r.N, r.M, base)
    _, oseff, obest = oracle.select_tau(ref_step, ref_done, taus, r.T, r.N, r.M, base)
    assert best == obest and np.allclose(seff, oseff, rtol=1e-6, atol=0)
    del lat_d
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name,per_trial_comm", [("extrapolation2048", True), ("heterogeneous2048", False)])
def test_full_size_widened_entry_points(name, per_trial_comm, dev):
    """The two 2048-worker workloads in full through the per-iteration speedup, the moments and the per-worker
    statistics, each against the oracle on the whole CPU tensor, streamed in chunks: per-iteration speedups add up
    over iterations (16 thresholds of the workload's grid keep the oracle's O(K) work per element to seconds),
    moments and per-worker sums are exact integers that add."""
    from concurrent.futures import ThreadPoolExecutor
    from dc_workloads import device
    r = config(name)
    threads = host.cpu_threads()
    lat_d = device.generate(r)
    grid = device.tau_grid(r, lat_d)
    taus = np.concatenate([grid[:: grid.size // 14], [BIG, int(grid[-1])]]).astype(np.int64)[:16]
    rng = np.random.default_rng(7)
    comm_t = rng.integers(0, 2 * r.comm + 1, size=r.T) if per_trial_comm else None

    got_seff = dc.dc_speedup_per_step(lat_d, taus, r.comm, comm_t)
    got_sum, got_sq, got_mean, got_var = dc.dc_moments(lat_d)
    got_wsum, got_wsq, got_wmean, got_wvar = dc.dc_worker_moments(lat_d)
    progress(f"{name}: library done on {r.nbytes / 1e9:.1f} GB")

    seff_sum = np.zeros(taus.size)
    n_all = s_all = q_all = 0
    wsum, wsq = [0] * r.N, [0] * r.N
    chunks = list(host.trial_chunks(r, 512 << 20))
    with ThreadPoolExecutor(threads) as pool:
        for i, (t0, t1) in enumerate(chunks):
            lat = host.generate(r, t0, t1, threads)
            comm = r.comm if comm_t is None else comm_t[t0:t1]
            seff_sum += oracle.per_step_speedup(lat, taus, comm, threads=threads) * (t1 - t0)
            cuts = [(t1 - t0) * j // threads for j in range(threads + 1)]
            parts = [lat[a:b] for a, b in zip(cuts, cuts[1:]) if b > a]
            for n, s_, q, _, _ in pool.map(oracle.moments, parts):
                n_all, s_all, q_all = n_all + n, s_all + s_, q_all + q
            for s_, q, _, _ in pool.map(oracle.worker_moments, parts):
                wsum = [a + b for a, b in zip(wsum, s_)]
                wsq = [a + b for a, b in zip(wsq, q)]
            progress(f"{name}: oracle chunk {i + 1}/{len(chunks)}")
    assert n_all == r.elements
    assert np.allclose(got_seff, seff_sum / r.T, rtol=SPEEDUP_RTOL, atol=0)
    assert np.allclose(got_seff, seff_sum / r.T, rtol=1e-10, atol=0)          # what the arithmetic delivers
    assert (got_sum, got_sq) == (s_all, q_all)
    assert got_mean == pytest.approx(s_all / n_all, rel=1e-14)
    assert got_var == pytest.approx((q_all * n_all - s_all * s_all) / (n_all * n_all), rel=1e-12)
    assert got_wsum == wsum and got_wsq == wsq
    assert np.allclose(got_wmean, [a / r.T for a in wsum], rtol=1e-14)
    assert np.allclose(got_wvar, [(q * r.T - a * a) / (r.T * r.T) for a, q in zip(wsum, wsq)], rtol=1e-12, atol=0)
    assert dc.dc_select_tau_per_step(got_seff, taus) == oracle.per_step_best(seff_sum / r.T, taus)
    del lat_d
    torch.cuda.empty_cache()


# ---- tau* under both conventions: ratio of iteration means (Section 4.4) and mean of iteration ratios (Algorithm 2) ----

@pytest.mark.parametrize("name,T", [("tiny", 1000), ("lognormal64", 400), ("additive200", 100),
                                    ("extrapolation2048", 16), ("heterogeneous2048", 8)])
def test_best_threshold_under_both_conventions(name, T, dev):
    """S_eff as the ratio of iteration means (dc_simulate + dc_select_tau) and as the mean of per-iteration ratios
    (dc_speedup_per_step + dc_select_tau_per_step, Algorithm 2 to its last line) on each workload: both against the
    oracle, and the gap between them against Appendix C.2's argument.  With R = (T + T^c) / (M (min{tau, T} + T^c))
    per iteration, the mean of ratios is E[M~ R] = E[M~] E[R] + cov(M~, R), and the appendix bounds the covariance by
    Cauchy-Schwarz: |cov| <= sqrt(E[R^2] var(M~_n) / N), the O(N^-1/2) term.  The ratio of means replaces E[R] by
    E[T + T^c] / (M E[min{tau, T} + T^c]); that second difference J does not shrink with N (it comes from the
    spread of T alone, and dominates for the workload with rare long delays).  Asserted: |gap - J| within the
    covariance bound.  J and the moments in the bound are taken from the CPU tensor."""
    r = config(name).with_shape(T=T, K=16)
    lat = host.generate(r)
    taus = np.append(host.tau_grid(r), BIG).astype(np.int64)
    lat_d = to_dev(lat, dev)
    step, done = dc.dc_simulate(lat_d, taus, r.comm)
    _, ratio_of_means, best_a = dc.dc_select_tau(step, done, taus, r.T, r.N, r.M, int(step[-1]))
    mean_of_ratios = dc.dc_speedup_per_step(lat_d, taus, r.comm)
    best_b = dc.dc_select_tau_per_step(mean_of_ratios, taus)

    ref_step, ref_done = oracle.simulate(lat, taus, r.comm, "sorted")
    _, ref_a, ref_best_a = oracle.select_tau(ref_step, ref_done, taus, r.T, r.N, r.M, int(ref_step[-1]))
    ref_b = oracle.per_step_speedup(lat, taus, r.comm, threads=host.cpu_threads())
    assert best_a == ref_best_a and np.allclose(ratio_of_means, ref_a, rtol=1e-6, atol=0)
    assert np.allclose(mean_of_ratios, ref_b, rtol=SPEEDUP_RTOL, atol=0)
    # the float sums differ in rounding order, so two almost equal maxima may swap: the chosen threshold must
    # reach the oracle's maximum to within that rounding, and be the same index when the maximum is clear
    ref_best_b = oracle.per_step_best(ref_b, taus)
    assert ref_b[best_b] >= ref_b[ref_best_b] * (1 - 1e-12)
    runner_up = np.max(np.delete(ref_b, ref_best_b))
    if ref_b[ref_best_b] - runner_up > 1e-9:
        assert best_b == ref_best_b

    P = np.cumsum(lat.astype(np.int64), axis=2)
    t_iter = P[:, :, -1].max(axis=1).astype(np.float64)
    worst = 0.0
    for k, tau in enumerate(taus):
        completed = (P < tau).sum(axis=2).astype(np.float64)                  # M~_n per iteration and worker
        capped = np.minimum(float(tau), t_iter) + r.comm
        ratio = (t_iter + r.comm) / (r.M * capped)                             # R per iteration
        spread = completed.mean() * (ratio.mean() - (t_iter + r.comm).mean() / (r.M * capped.mean()))      # J
        bound = np.sqrt((ratio ** 2).mean() * completed.var() / r.N)
        gap = mean_of_ratios[k] - ratio_of_means[k]
        assert abs(gap - spread) <= bound + 1e-12, (name, int(tau), gap, spread, bound)
        worst = max(worst, abs(gap))
    progress(f"{name}: tau* {int(taus[best_a])} us (ratio of means, S_eff {ratio_of_means[best_a]:.6f}), "
             f"{int(taus[best_b])} us (mean of ratios, S_eff {mean_of_ratios[best_b]:.6f}), largest gap {worst:.2e}")


def test_plain_c_caller_of_the_abi(dev, golden_dir):
    """paper_2306_10598_amd/examples/dc_from_c (C, no Python, no torch) on the hand-worked example and on a random problem."""
    import subprocess
    from tests.conftest import ROOT
    from tests.test_oracle_pins import read_golden
    exe = ROOT / "paper_2306_10598_amd" / "examples" / "dc_from_c"
    if not exe.exists():
        import __graft_entry__
        __graft_entry__.build_c_example()

    def run(lat, taus, comm):
        T, N, M = lat.shape
        text = f"{T} {N} {M} {len(taus)} {comm}\n" + " ".join(map(str, lat.reshape(-1))) + "\n" + " ".join(map(str, taus)) + "\n"
        res = subprocess.run([str(exe)], input=text, capture_output=True, text=True, timeout=100)
        assert res.returncode == 0, res.stderr
        lines = dict(line.split(" ", 1) for line in res.stdout.strip().splitlines())
        return (np.array(lines["step"].split(), dtype=np.int64), np.array(lines["done"].split(), dtype=np.int64),
                int(lines["best"]))

    g = read_golden(golden_dir / "hand_example.txt")
    lat = np.array(g["lat"], dtype=np.int32).reshape(g["T"][0], g["N"][0], g["M"][0])
    step, done, _ = run(lat, g["taus"], g["comm"][0])
    assert step.tolist() == g["step"] and done.tolist() == g["done"]

    rng = np.random.default_rng(21)
    lat = rng.integers(0, 5000, size=(7, 19, 12), dtype=np.int32)
    taus = rng.integers(0, 12 * 5000, size=40).astype(np.int64)
    step, done, best = run(lat, taus.tolist(), 9)
    ref_step, ref_done = oracle.simulate(lat, taus, 9, "literal")
    assert np.array_equal(step, ref_step) and np.array_equal(done, ref_done)
    assert best == oracle.select_tau(ref_step, ref_done, taus, 7, 19, 12, 0)[2]


def test_launch_shape_follows_the_threshold_grid(dev):
    """Long rows on one workspace with threshold grids that cover almost nothing, everything, and almost nothing
    again: the device-side choice between the two launch shapes must never leave stale partial histograms behind."""
    r = config("heterogeneous2048").with_shape(T=700)                    # enough units for the larger grid
    lat = host.generate(r)
    lat_d = to_dev(lat, dev)
    top = int(host.worker_totals(lat).max())
    grids = [np.linspace(top - top // 50, top, 64).astype(np.int64), np.linspace(0, top, 200).astype(np.int64),
             np.array([top + 5], dtype=np.int64), np.linspace(top // 3, top, 90).astype(np.int64),
             np.linspace(top - top // 40, top + 9, 64).astype(np.int64)]
    K = max(g.size for g in grids)
    ws = torch.empty(dc.dc_workspace_bytes(r.T, r.N, r.M, K), dtype=torch.uint8, device=dev)
    out = torch.zeros((2, K), dtype=torch.int64, device=dev)
    for taus in grids + grids[::-1]:
        k = taus.size
        dc.dc_simulate_async(lat_d, torch.from_numpy(taus).to(dev), r.comm, out[0, :k], out[1, :k], ws, None)
        torch.cuda.synchronize()
        assert dc.dc_workspace_status(ws, None) == dc.DC_OK
        ref_step, ref_done = oracle.simulate_threaded(lat, taus, r.comm, "sorted", host.cpu_threads())
        assert np.array_equal(out[0, :k].cpu().numpy(), ref_step) and np.array_equal(out[1, :k].cpu().numpy(), ref_done)


def test_long_rows_with_more_thresholds_than_one_pass_holds(dev):
    """Long rows, enough units for both launch shapes, and more thresholds than one pass holds (a full pass's grid
    leaves room for two blocks per compute unit only, so there is one launch shape): the first pass starts at 0, the
    later ones ever higher.  Both entry points, against the oracle."""
    r = config("heterogeneous2048").with_shape(T=700)
    lat = host.generate(r)
    lat_d = to_dev(lat, dev)
    top = int(host.worker_totals(lat).max())
    rng = np.random.default_rng(31)
    taus = np.linspace(0, top + 3, 9001).astype(np.int64)[rng.permutation(9001)]
    step, done = dc.dc_simulate(lat_d, taus, r.comm)
    ref_step, ref_done = oracle.simulate_threaded(lat, taus, r.comm, "sorted", host.cpu_threads())
    assert np.array_equal(step, ref_step) and np.array_equal(done, ref_done)
    few = r.with_shape(T=40)
    lat_few = np.ascontiguousarray(lat[:40])
    taus1 = np.maximum(np.linspace(0, top + 3, 4500).astype(np.int64), 1)       # three passes of 2047 thresholds
    got = dc.dc_speedup_per_step(to_dev(lat_few, dev), taus1, few.comm)
    assert np.allclose(got, oracle.per_step_speedup(lat_few, taus1, few.comm, threads=host.cpu_threads()), rtol=SPEEDUP_RTOL, atol=0)


def test_graph_replay_picks_the_launch_shape_from_the_data(dev):
    """A captured sequence for long rows holds both launch shapes; each replay chooses on the device.  The graph is
    replayed on a tensor whose contents change between replays (scaled so that the same thresholds cover almost
    nothing, then everything), and must match the oracle each time."""
    r = config("extrapolation2048").with_shape(T=300)
    base = host.generate(r)
    top = int(host.worker_totals(base).max())
    taus = np.linspace(top - top // 40, top, 128).astype(np.int64)
    taus_d = torch.from_numpy(taus).to(dev)
    lat_d = to_dev(base, dev)
    out = torch.zeros((2, taus.size), dtype=torch.int64, device=dev)
    ws = torch.empty(dc.dc_workspace_bytes(r.T, r.N, r.M, taus.size), dtype=torch.uint8, device=dev)
    side = torch.cuda.Stream()
    dc.dc_simulate_async(lat_d, taus_d, r.comm, out[0], out[1], ws, side)
    assert dc.dc_workspace_status(ws, side) == dc.DC_OK
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        dc.dc_simulate_async(lat_d, taus_d, r.comm, out[0], out[1], ws, torch.cuda.current_stream())
    for factor in (1, 3, 1, 2, 3, 1):                            # x3: every completion time passes the smallest threshold early
        lat = base * factor
        lat_d.copy_(torch.from_numpy(lat))
        out.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ref_step, ref_done = oracle.simulate_threaded(lat, taus, r.comm, "sorted", host.cpu_threads())
        got = out.cpu().numpy()
        assert np.array_equal(got[0], ref_step) and np.array_equal(got[1], ref_done), factor


def test_per_step_speedup_launch_shapes(dev):
    """The per-iteration speedup of long rows over more trials than the narrow launch has blocks, with threshold
    grids that cover almost nothing and almost everything (the two launch shapes): the result must equal the
    trial-weighted combination of slabs small enough to take the single-shape path, and a slab must match the oracle."""
    r = config("extrapolation2048").with_shape(T=900)
    from dc_workloads import device
    lat_d = device.generate(r)
    top = int(lat_d.sum(dim=2, dtype=torch.int64).max().item())
    grids = [np.linspace(top - top // 40, top, 48).astype(np.int64), np.linspace(1, top, 96).astype(np.int64),
             np.linspace(top - top // 30, top + 3, 20).astype(np.int64)]
    for taus in grids + grids[::-1]:
        whole = dc.dc_speedup_per_step(lat_d, taus, r.comm)
        parts = np.zeros(taus.size)
        for t0 in range(0, r.T, 300):
            parts += dc.dc_speedup_per_step(lat_d[t0:t0 + 300], taus, r.comm) * (300 / r.T)
        assert np.allclose(whole, parts, rtol=1e-10, atol=0)
        assert np.array_equal(whole, dc.dc_speedup_per_step(lat_d, taus, r.comm))     # same launch shape, same bits
    lat = host.generate(r, 450, 454)
    for taus in grids[:2]:
        assert np.allclose(dc.dc_speedup_per_step(lat_d[450:454], taus[::4], r.comm),
                           oracle.per_step_speedup(lat, taus[::4], r.comm), rtol=SPEEDUP_RTOL, atol=0)
