"""The synthetic latency generator: hash vectors, NumPy vs C agreement, distribution sanity."""
import math

import numpy as np
import pytest

from dc_workloads import CONFIG_NAMES, config, host, spec


def test_mix64_matches_published_splitmix64_outputs():
    # first three outputs of SplitMix64 seeded with 0 (Steele, Lea & Flood; Vigna's reference code)
    got = [spec.mix64_int(spec.GOLDEN * i) for i in (1, 2, 3)]
    assert got == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    arr = host.mix64(np.array([spec.GOLDEN, (2 * spec.GOLDEN) & spec.MASK64], dtype=np.uint64))
    assert [int(x) for x in arr] == got[:2]


@pytest.mark.parametrize("name", CONFIG_NAMES)
def test_c_generator_equals_numpy_reference(name):
    r = config(name).with_shape(T=3)
    n = min(r.elements, 150_000)
    ref = host.generate_numpy(r, 0, n)
    fast = host.generate(r).reshape(-1)[:n]
    assert np.array_equal(ref, fast)
    # an offset window equals the same window of the whole
    off = 12_345 % max(1, n - 100)
    assert np.array_equal(host.generate_numpy(r, off, 100), ref[off:off + 100])


def test_tail_cells_are_exercised_and_agree():
    # hashes whose top 16 bits fall in the refined cells at both ends
    r = config("extrapolation2048")
    h = np.array([0, 1 << 40, (15 << 48) | 0xFFFFFFFF0000, (16 << 48), (65519 << 48) | 0xFFFFFFFF0000,
                  (65520 << 48), (65535 << 48), spec.MASK64], dtype=np.uint64)
    q = host.draw_q8(h, r.value)
    assert np.all(np.diff(q.astype(np.int64)) >= 0)
    assert q[0] == r.value.lo[0] and q[3] == r.value.main[16] and q[5] == r.value.main[65520]
    assert q[7] <= r.value.hi[-1]


def test_generation_is_seeded_and_windowed():
    r = config("tiny")
    a = host.generate(r, 10, 20)
    b = host.generate(r, 0, 30)[10:20]
    assert np.array_equal(a, b)
    assert not np.array_equal(host.generate(r.with_shape(seed=1), 0, 2), host.generate(r, 0, 2))


@pytest.mark.parametrize("name,mean,sd", [
    ("tiny", 110000.0, 10000.0),
    ("lognormal64", 120000.0 * math.exp(0.005), 120000.0 * math.exp(0.005) * math.sqrt(math.exp(0.01) - 1)),
    ("extrapolation2048", 100000.0, 10000.0),
])
def test_moments_of_iid_workloads(name, mean, sd):
    r = config(name)
    r = r.with_shape(T=max(1, 2_000_000 // (r.N * r.M)))
    x = host.generate(r).astype(np.float64).reshape(-1)
    assert abs(x.mean() - mean) <= 5 * sd / math.sqrt(x.size) + 0.5
    assert abs(x.std() - sd) <= 0.01 * sd
    assert x.min() >= 1


def test_straggler_rate_and_size():
    r = config("additive200").with_shape(T=100)
    x = host.generate(r).reshape(-1)
    frac = np.mean(x > 450000)
    assert abs(frac - 0.01) <= 5 * math.sqrt(0.01 * 0.99 / x.size)
    assert abs(np.median(x[x > 450000]) - 750000) < 2000


def test_heterogeneous_workers_have_persistent_slowdown():
    r = config("heterogeneous2048").with_shape(T=4)
    s = host.worker_scale_q16(r).astype(np.float64) / 65536.0
    assert s.min() >= 1.0 and abs(s.mean() - 1.05) < 5 * 0.05 / math.sqrt(r.N)
    x = host.generate(r).astype(np.float64)
    per_worker = np.median(x, axis=(0, 2))
    assert np.corrcoef(per_worker, s)[0, 1] > 0.99


def test_tau_grid_rules():
    r = config("tiny")
    lat = host.generate(r)
    totals = host.worker_totals(lat)
    g = host.tau_grid(r)
    assert g.size == r.K and g[0] == totals.min() and g[-1] == totals.max()
    assert np.all(np.diff(g) >= 0)
    r2 = config("lognormal64").with_shape(T=200)
    totals = np.sort(host.worker_totals(host.generate(r2)))
    g2 = host.tau_grid(r2)
    n = totals.size
    assert g2[0] == totals[(n - 1) // 100] and g2[-1] == totals[(n - 1) * 999 // 1000]
    k = 37
    assert g2[k] == g2[0] + (int(g2[-1] - g2[0]) * k) // (r2.K - 1)


def test_largest_latency_leaves_room_for_int32_worker_totals():
    for name in CONFIG_NAMES:
        r = config(name)
        scale = host.worker_scale_q16(r)
        smax = 65536 if scale is None else int(scale.max())
        top = ((int(r.value.hi[-1]) * smax * r.spike_mul + (1 << 23)) >> 24) + r.add + r.spike_add
        assert max(top, r.clip_min) <= (2 ** 31 - 1) // r.M, name


# ---- the paper's own noise models (Appendix B.1, C.3) ---------------------------------------------------

def test_simulated_delay_scales_mean_and_bounds_the_tail():
    from dc_workloads import noise
    r = noise.simulated_delay(T=40, N=64, M=12, base_us=450_000)
    x = host.generate(r).astype(np.float64).reshape(-1) / 450_000
    assert x.min() >= 1.0 and x.max() <= 6.5 + 1e-6
    # eps = min(Z/alpha, 5.5): E[Z/alpha] = 0.5, the bound removes a little of it
    assert 1.45 < x.mean() < 1.5
    assert np.mean(x > 6.49) < 0.01


@pytest.mark.parametrize("family", ["lognormal", "normal", "bernoulli", "exponential", "gamma"])
def test_additive_noise_families_have_the_requested_moments(family):
    from dc_workloads import noise
    r = noise.additive_noise(family, T=60, N=64, variance=0.05)
    eps = host.generate(r).astype(np.float64).reshape(-1) / 1e6 - 0.45
    n = eps.size
    want_mean = math.sqrt(0.05) if family == "exponential" else 0.225     # one-parameter family: rate 1/sqrt(var)
    assert abs(eps.mean() - want_mean) < 5 * math.sqrt(0.05 / n) + 2e-3
    assert abs(eps.var() - 0.05) < 0.004
    prm = noise.noise_parameters(family, 0.225, 0.05)
    if family == "lognormal":                      # the appendix quotes LN(-1.84, 0.83)
        assert abs(prm["mu_log"] + 1.84) < 0.01 and abs(prm["sigma_log"] - 0.83) < 0.005
    if family == "gamma":                          # gamma(alpha = 1, beta = 4.5)
        assert abs(prm["shape"] - 1.0) < 0.02 and abs(prm["rate"] - 4.5) < 0.01
    if family == "bernoulli":                      # 0.45 Br(0.5)
        assert abs(prm["amplitude"] - 0.45) < 0.003 and abs(prm["p"] - 0.5) < 0.01
        assert set(np.unique(np.round(eps, 3))) <= {0.0, round(prm["amplitude"], 3)}


def test_local_sgd_stragglers_by_scenario():
    from dc_workloads import noise
    for scenario, eligible in (("uniform", 32), ("single_server", 8)):
        r = noise.local_sgd(T=400, period=16, scenario=scenario)
        x = host.generate(r)
        assert np.array_equal(host.generate_numpy(r).reshape(x.shape), x)
        slow = x > 250_000
        assert set(np.unique(x)) == {250_000, 1_250_000}
        per_worker = slow.mean(axis=(0, 2))
        assert np.all(per_worker[eligible:] == 0)
        assert abs(per_worker[:eligible].mean() - 0.04) < 5 * math.sqrt(0.04 * 0.96 / (400 * 16 * eligible))


def test_per_worker_normal_reproduces_each_workers_moments():
    from dc_workloads import noise
    rng = np.random.default_rng(3)
    mean = rng.uniform(2.0e6, 4.0e6, size=24)
    sd = rng.uniform(1.0e4, 3.0e5, size=24)
    sd[5] = 0.0
    r = noise.per_worker_normal(20000, mean, sd)
    x = host.generate(r)
    assert np.array_equal(host.generate_numpy(r, 0, 5000), x.reshape(-1)[:5000])
    got_mean, got_sd = x[:, :, 0].mean(axis=0), x[:, :, 0].std(axis=0)
    assert np.all(np.abs(got_mean - mean) <= 5 * sd / math.sqrt(20000) + 1.0)
    assert np.allclose(got_sd, sd, rtol=0.03, atol=1.0)
