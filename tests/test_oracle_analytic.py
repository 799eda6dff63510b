"""Pins for the oracle's analytical side (moments and the closed forms of Sections 4.2-4.4 / Appendix C.2)."""
import math

import numpy as np
import pytest
from scipy import integrate
from scipy.stats import norm

import oracle
from dc_workloads import host, spec
from tests.test_oracle_pins import iid_recipe

BIG = 1 << 40


def test_moments_against_python_integers():
    rng = np.random.default_rng(1)
    lat = rng.integers(0, 2**31 - 1, size=(3, 5, 7), dtype=np.int32)         # squares need more than 64 bits in total
    n, s, q, mean, var = oracle.moments(lat)
    vals = [int(v) for v in lat.reshape(-1)]
    assert (n, s, q) == (len(vals), sum(vals), sum(v * v for v in vals))
    assert mean == pytest.approx(np.mean(lat.astype(np.float64)), rel=1e-12)
    assert var == pytest.approx(np.var(lat.astype(np.float64)), rel=1e-9)
    assert oracle.moments(np.full((2, 2, 2), 9, dtype=np.int32))[3:] == (9.0, 0.0)
    with pytest.raises(oracle.OracleError):
        oracle.moments(np.array([[[1, -2]]], dtype=np.int32))


def test_completed_estimate_limits_and_single_microbatch():
    mu, s2 = 100.0, 25.0
    e_done, _, _, _ = oracle.analytic_curves(mu, s2, 8, 1, [90, 100, 110, 10**6], 0)
    assert np.allclose(e_done, [norm.cdf(-2), 0.5, norm.cdf(2), 1.0], atol=1e-14)      # M = 1: one normal CDF
    e_done, _, _, _ = oracle.analytic_curves(mu, s2, 8, 12, [0, BIG], 1)
    assert e_done[0] == pytest.approx(0.0, abs=1e-12) and e_done[1] == pytest.approx(12.0, abs=1e-12)
    # deterministic latencies: a step function, strict at ties
    e_done, _, _, _ = oracle.analytic_curves(10.0, 0.0, 4, 5, [10, 11, 30, 31, 1000], 1)
    assert e_done.tolist() == [0.0, 1.0, 2.0, 3.0, 5.0]


def test_slowest_worker_estimate_against_exact_order_statistics():
    """E[max of N iid normals] by quadrature of x N phi(x) Phi(x)^(N-1) (the iid-max density of Section 4.2)."""
    # the approximation overestimates slightly and tightens with N; swapping its two weights, or dropping
    # the factor e, moves it by more than these margins
    for N, margin in ((16, 0.025), (64, 0.013), (200, 0.009), (2048, 0.0045)):
        exact, _ = integrate.quad(lambda x: x * N * norm.pdf(x) * norm.cdf(x) ** (N - 1), -10, 12, limit=400)
        _, e_t, _, _ = oracle.analytic_curves(0.0, 1.0, N, 1, [1], 0)
        assert 0 < e_t / exact - 1 < margin, (N, e_t, exact)
    _, e_t, _, _ = oracle.analytic_curves(7.0, 4.0, 64, 9, [1], 0)
    _, z, _, _ = oracle.analytic_curves(0.0, 1.0, 64, 1, [1], 0)
    assert e_t == pytest.approx(math.sqrt(9 * 4.0) * z + 9 * 7.0, rel=1e-14)            # scaling by sqrt(M sigma^2), shift M mu


def test_speedup_estimate_identities():
    mu, s2, N, M, comm = 100000.0, 1.0e8, 200, 32, 50000
    taus = np.array([int(0.9 * M * mu), int(M * mu), int(1.02 * M * mu), BIG])
    e_done, e_t, s_eff, best = oracle.analytic_curves(mu, s2, N, M, taus, comm)
    assert s_eff[-1] == pytest.approx(1.0, abs=1e-12)                                   # no drops
    assert np.allclose(s_eff, e_done / M * (e_t + comm) / (np.minimum(taus, e_t) + comm), rtol=1e-15)
    assert best == int(np.argmax(e_done / (taus + comm)))
    _, _, given, _ = oracle.analytic_curves(mu, s2, N, M, taus, comm, mean_tmax=3.3e6)
    assert np.allclose(given, e_done / M * (3.3e6 + comm) / (np.minimum(taus, 3.3e6) + comm), rtol=1e-15)
    with pytest.raises(oracle.OracleError):
        oracle.analytic_curves(mu, s2, 1, M, taus, comm)                                # the estimate needs N >= 2


def test_analytic_best_threshold_worked_by_hand():
    """Appendix C.2, "Finding tau*": tau* = argmax (1/(tau + T^c)) sum_m Phi((tau - m mu)/sqrt(m sigma^2)).

    One micro-batch per worker (M = 1), mu = 100, sigma = 10, so the sum is one normal CDF at a whole number of
    standard deviations; Phi(0), Phi(2), Phi(3) from a table: 0.5, 0.97725, 0.99865.
      T^c = 0:     tau 100: 0.5/100 = 0.00500   tau 120: 0.97725/120 = 0.008144   tau 130: 0.99865/130 = 0.007682
      T^c = 1000:  tau 100: 0.5/1100 = 0.000455 tau 120: 0.97725/1120 = 0.000873  tau 130: 0.99865/1130 = 0.000884
    A long serial part moves the best threshold up: with T^c = 0 it is 120, with T^c = 1000 it is 130."""
    taus = [100, 120, 130]
    e_done, _, _, best = oracle.analytic_curves(100.0, 100.0, 4, 1, taus, 0)
    assert np.allclose(e_done, [0.5, 0.97725, 0.99865], atol=5e-6) and best == 1
    assert oracle.analytic_curves(100.0, 100.0, 4, 1, taus, 1000)[3] == 2
    assert oracle.analytic_curves(100.0, 100.0, 4, 1, [130, 100, 120], 0)[3] == 2        # any order of the list
    assert oracle.analytic_curves(100.0, 100.0, 4, 1, taus, 0, mean_tmax=105.0)[3] == 1  # no estimate of T enters
    assert oracle.analytic_curves(100.0, 100.0, 4, 1, [120, 100, 120], 0)[3] == 0        # equal thresholds: lowest index
    # deterministic latencies of 10 with M = 3 (sigma = 0): completed = #{m : 10 m < tau}; T^c = 5
    #   tau 10: 0/15   tau 11: 1/16 = 0.0625   tau 21: 2/26 = 0.0769   tau 31: 3/36 = 0.0833   tau 60: 3/65 = 0.046
    assert oracle.analytic_curves(10.0, 0.0, 2, 3, [10, 11, 21, 31, 60], 5)[3] == 3


def test_worker_moments_squares_against_python_integers():
    rng = np.random.default_rng(8)
    lat = rng.integers(0, (2**31 - 1) // 4, size=(300, 5, 4), dtype=np.int32)              # totals up to 2^31
    sums, squares, _, _ = oracle.worker_moments(lat)
    for n in range(5):
        totals = [sum(int(v) for v in lat[t, n]) for t in range(300)]
        assert sums[n] == sum(totals) and squares[n] == sum(v * v for v in totals)


def test_estimates_track_the_simulation_for_normal_latencies():
    """Normal samples: the analytical S_eff follows the simulated one (the paper's Figure 3a claim)."""
    T, N, M, mu, sigma, comm = 3000, 64, 32, 100000.0, 10000.0, 30000
    lat = host.generate(iid_recipe(spec.q_normal(mu, sigma), T, N, M, clip_min=1))
    n, s, q, mean, var = oracle.moments(lat)
    assert mean == pytest.approx(mu, rel=2e-3) and math.sqrt(var) == pytest.approx(sigma, rel=1e-2)
    taus = np.array([int(M * mu * f) for f in (0.97, 0.99, 1.0, 1.01, 1.02, 1.04)] + [BIG])
    step, done = oracle.simulate(lat, taus, comm, "sorted")
    _, sim, _ = oracle.select_tau(step, done, taus, T, N, M, int(step[-1]))
    e_done, e_t, ana, _ = oracle.analytic_curves(mean, var, N, M, taus, comm)
    assert np.allclose(e_done, done / (T * N), atol=0.03)
    assert e_t == pytest.approx((step[-1] - T * comm) / T, rel=2e-3)
    assert np.allclose(ana, sim, rtol=0.01)


def test_worker_moments(golden_dir):
    from tests.test_oracle_pins import read_golden
    g = read_golden(golden_dir / "hand_example.txt")
    lat = np.array(g["lat"], dtype=np.int32).reshape(1, 2, 3)
    sums, squares, mean, var = oracle.worker_moments(lat)
    assert sums == [12, 13] and squares == [144, 169] and var.tolist() == [0.0, 0.0]      # worker totals 12 and 13
    rng = np.random.default_rng(4)
    lat = rng.integers(0, 2**31 // 16, size=(50, 7, 16), dtype=np.int32)
    sums, squares, mean, var = oracle.worker_moments(lat)
    totals = lat.astype(np.float64).sum(axis=2)
    assert np.allclose(mean, totals.mean(axis=0), rtol=1e-13) and np.allclose(var, totals.var(axis=0), rtol=1e-9)
    assert sum(sums) == int(lat.astype(np.int64).sum())
    # permuting iterations changes nothing; permuting workers permutes the result
    perm = rng.permutation(7)
    s2, q2, _, _ = oracle.worker_moments(lat[::-1][:, perm])
    assert s2 == [sums[p] for p in perm] and q2 == [squares[p] for p in perm]
