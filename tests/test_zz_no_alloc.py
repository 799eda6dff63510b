"""The entry point that allocates nothing (dc_simulate_static: the library's fixed device array instead of a
workspace) against the workspace entry point and the CPU oracle, through the C ABI.

Two calls in a row on the same GPU, the second on a smaller input, so that what the first call left in the
array must not show in the second; then the size limit, the device-side value checks, and a side stream.
"""
import numpy as np
import pytest

import oracle
import paper_2306_10598_amd as dc
from dc_workloads import config, host

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
BIG = 1 << 40


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    dc._load()
    return torch.device("cuda:0")


def both_entry_points(lat, taus, comm, dev, stream=None):
    """(step, done) from dc_simulate_async with a workspace and from dc_simulate_static, as NumPy arrays."""
    T, N, M = lat.shape
    lat_d = torch.from_numpy(np.ascontiguousarray(lat)).to(dev)
    taus_d = torch.from_numpy(np.ascontiguousarray(taus, dtype=np.int64)).to(dev)
    K = taus_d.numel()
    ws = torch.empty(dc.dc_workspace_bytes(T, N, M, K), dtype=torch.uint8, device=dev)
    with_ws = torch.zeros((2, K), dtype=torch.int64, device=dev)
    static = torch.full((2, K), -1, dtype=torch.int64, device=dev)
    status = torch.full((1,), -1, dtype=torch.int32, device=dev)
    torch.cuda.synchronize()
    dc.dc_simulate_async(lat_d, taus_d, comm, with_ws[0], with_ws[1], ws, stream)
    assert dc.dc_workspace_status(ws, stream) == dc.DC_OK
    dc.dc_simulate_static(lat_d, taus_d, comm, static[0], static[1], status, stream)
    (stream.synchronize() if stream is not None else torch.cuda.synchronize())
    assert int(status.item()) == dc.DC_OK
    return with_ws.cpu().numpy(), static.cpu().numpy()


def test_static_scratch_entry_point_two_calls_in_a_row(dev):
    big = config("extrapolation2048").with_shape(T=48, K=256)        # 50 MB, long rows, two launch shapes
    small = config("lognormal64").with_shape(T=200, N=61, K=40)      # 1.6 MB, ragged worker count, fewer thresholds
    for r in (big, small):
        lat = host.generate(r)
        taus = np.concatenate([host.tau_grid(r), [0, BIG]]).astype(np.int64)
        with_ws, static = both_entry_points(lat, taus, r.comm, dev)
        assert np.array_equal(static, with_ws), r.name
        ref_step, ref_done = oracle.simulate_threaded(lat, taus, r.comm, "sorted", host.cpu_threads())
        assert np.array_equal(static[0], ref_step) and np.array_equal(static[1], ref_done), r.name


def test_static_scratch_other_row_lengths_and_a_side_stream(dev):
    rng = np.random.default_rng(3)
    stream = torch.cuda.Stream()
    for shape in ((40, 9, 63), (3, 700, 256), (500, 3, 1), (7, 33, 12)):
        lat = rng.integers(0, 4000, size=shape, dtype=np.int32)
        top = int(lat.sum(axis=2, dtype=np.int64).max())
        taus = rng.integers(0, top + 9, size=int(rng.integers(1, 90)))
        with_ws, static = both_entry_points(lat, taus, 5, dev, stream)
        assert np.array_equal(static, with_ws), shape
        ref_step, ref_done = oracle.simulate(lat, taus, 5, "literal")
        assert np.array_equal(static[0], ref_step) and np.array_equal(static[1], ref_done), shape


def test_static_scratch_limit_and_value_checks(dev):
    out = torch.zeros((2, 4095), dtype=torch.int64, device=dev)
    wide = torch.ones((4096, 256, 64), dtype=torch.int32, device=dev)      # 1024 blocks x 4096 bins of partial histograms
    assert dc.dc_workspace_bytes(4096, 256, 64, 4095) > dc.DC_STATIC_SCRATCH_BYTES
    with pytest.raises(dc.DcError) as e:                          # refused on the host, nothing enqueued
        dc.dc_simulate_static(wide, torch.zeros(4095, dtype=torch.int64, device=dev), 0, out[0], out[1])
    assert e.value.status == dc.DC_ERR_INVALID_ARG and b"scratch" in dc._load().dc_last_device_error()
    del wide
    lat = torch.ones((4, 64, 64), dtype=torch.int32, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    taus = torch.tensor([5, 70, 3], dtype=torch.int64, device=dev)
    bad = lat.clone()
    bad[2, 5, 9] = -4
    dc.dc_simulate_static(bad, taus, 1, out[0, :3], out[1, :3], status)
    torch.cuda.synchronize()
    assert int(status.item()) == dc.DC_ERR_NEGATIVE_LATENCY
    taus[1] = -70
    dc.dc_simulate_static(lat, taus, 1, out[0, :3], out[1, :3], status)
    torch.cuda.synchronize()
    assert int(status.item()) == dc.DC_ERR_INVALID_ARG
    taus[1] = 70                                                  # and the array is usable again afterwards
    dc.dc_simulate_static(lat, taus, 1, out[0, :3], out[1, :3], status)
    torch.cuda.synchronize()
    assert int(status.item()) == dc.DC_OK
    assert out[1, :3].tolist() == [4 * 64 * 4, 4 * 64 * 64, 4 * 64 * 2] and out[0, :3].tolist() == [24, 260, 16]
