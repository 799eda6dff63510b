"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol that
include/dc.h declares, and the host-only threshold selection agrees with the oracle."""
import re

import numpy as np
import pytest

import oracle
import paper_2306_10598_amd as dc
from tests.conftest import ROOT


def declared_functions():
    text = (ROOT / "include" / "dc.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dc_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = dc._load()
    names = declared_functions()
    assert len(names) >= 10
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(dc.EXPORTS) == names


def test_status_strings():
    assert dc.dc_status_string(dc.DC_OK) == "ok"
    assert "negative" in dc.dc_status_string(dc.DC_ERR_NEGATIVE_LATENCY)
    assert dc.dc_status_string(99) == "unknown status"


def test_workspace_bytes_is_pure_arithmetic():
    assert dc.dc_workspace_bytes(0, 1, 1, 1) == 0
    assert dc.dc_workspace_bytes(1, 1, 1, dc.DC_MAX_THRESHOLDS + 1) == 0
    small = dc.dc_workspace_bytes(10, 8, 16, 64)
    big = dc.dc_workspace_bytes(16384, 2048, 256, 512)
    assert 0 < small < big < (64 << 20)
    assert small % 256 == 0


def test_select_tau_matches_oracle_and_breaks_ties_exactly():
    rng = np.random.default_rng(0)
    K, T, N, M = 200, 50, 16, 32
    step = rng.integers(10**9, 10**12, size=K)
    done = rng.integers(0, T * N * M + 1, size=K)
    taus = rng.integers(0, 10**7, size=K)
    step[17], done[17], taus[17] = step[3], done[3], taus[3] + 5          # exact tie, larger tau
    thr, seff, best = dc.dc_select_tau(step, done, taus, T, N, M, int(step.max()))
    othr, oseff, obest = oracle.select_tau(step, done, taus, T, N, M, int(step.max()))
    assert best == obest
    assert np.allclose(thr, othr, rtol=1e-6, atol=0) and np.allclose(seff, oseff, rtol=1e-6, atol=0)
    # ordering that float64 cannot resolve
    big = 3 * 10**18
    _, _, b = dc.dc_select_tau([big, big - 1], [big - 1, big - 2], [1, 2], 1, 1, 1)
    assert b == oracle.select_tau([big, big - 1], [big - 1, big - 2], [1, 2], 1, 1, 1)[2] == 0
    _, _, b = dc.dc_select_tau([4, 8, 16, 2], [2, 4, 8, 1], [10, 30, 40, 20], 1, 1, 8)
    assert b == 2
    _, seff, _ = dc.dc_select_tau([5], [3], [7], 1, 1, 3)
    assert np.isnan(seff[0])


def test_select_tau_per_step_matches_oracle_and_breaks_ties():
    rng = np.random.default_rng(5)
    for K in (1, 2, 7, 300):
        seff = rng.random(K)
        taus = rng.integers(0, 10**7, size=K)
        if K > 5:
            seff[4] = seff[1] = seff.max() + 0.25                      # equal maxima: the larger tau wins
            taus[4] = taus[1] + 3
        assert dc.dc_select_tau_per_step(seff, taus) == oracle.per_step_best(seff, taus)
    assert dc.dc_select_tau_per_step([3 / 7, 3 / 4, 9 / 11, 3 / 4, 1.0, 1.0], [5, 6, 9, 10, 11, 50]) == 5
    assert dc.dc_select_tau_per_step([0.5, 0.7, 0.7, 0.2], [10, 30, 30, 40]) == 1
    for seff, taus in (([], []), ([float("nan")], [1]), ([1.0], [-1])):
        with pytest.raises(dc.DcError) as e:
            dc.dc_select_tau_per_step(seff, taus)
        assert e.value.status == dc.DC_ERR_INVALID_ARG


def test_select_tau_rejects_bad_input():
    with pytest.raises(dc.DcError) as e:
        dc.dc_select_tau([0], [1], [1], 1, 1, 1)
    assert e.value.status == dc.DC_ERR_INVALID_ARG
    with pytest.raises(dc.DcError):
        dc.dc_select_tau([], [], [], 1, 1, 1)


def test_modelled_iteration_time_needs_no_gpu_and_matches_oracle():
    """With K = 0 dc_analytic_curves only evaluates the normal-maximum formula (host arithmetic)."""
    for N in (2, 3, 64, 200, 2048, 10**6):
        for M, mu, s2 in ((1, 0.0, 1.0), (32, 100000.0, 1.0e8), (256, 108000.0, 1.2e9)):
            _, e_t, _, _ = dc.dc_analytic_curves(mu, s2, N, M, [], 0)
            _, ref, _, _ = oracle.analytic_curves(mu, s2, N, M, [1], 0)
            assert e_t == pytest.approx(ref, rel=1e-13, abs=1e-12), (N, M)
    with pytest.raises(dc.DcError):
        dc.dc_analytic_curves(1.0, 1.0, 1, 4, [], 0)
    with pytest.raises(dc.DcError):
        dc.dc_analytic_curves(1.0, -1.0, 8, 4, [], 0)
