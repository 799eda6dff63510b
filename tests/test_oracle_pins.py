"""Pins for the CPU oracle: what the paper's definitions and plain mathematics fix.

None of these compares the oracle with itself: each expected value is a hand computation,
a closed form, an independent formulation (sort + binary search) or an invariant that
follows from the definitions in Sections 4.2-4.4 / Appendix C.1.
"""
import itertools
import math

import numpy as np
import pytest
from scipy.special import ndtr, ndtri

import oracle
from dc_workloads import host, spec

METHODS = ("literal", "sorted")
BIG = 1 << 40


def read_golden(path):
    out = {}
    for line in path.read_text().splitlines():
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *vals = line.split()
        out[key] = [int(v) for v in vals]
    return out


def independent_counts(lat, taus, comm):
    """Sort every completion time once, then count by binary search (strictly below tau)."""
    P = np.cumsum(lat.astype(np.int64), axis=2)
    flat = np.sort(P.reshape(-1))
    done = np.searchsorted(flat, np.asarray(taus, dtype=np.int64), side="left")
    tmax = P[:, :, -1].max(axis=1)
    step = np.array([np.minimum(tmax, t).sum() + comm * lat.shape[0] for t in taus], dtype=np.int64)
    return step, done.astype(np.int64)


def iid_recipe(qfun, T, N, M, seed=1, clip_min=0):
    return spec.Recipe("pin", T=T, N=N, M=M, K=1, comm=0, grid="minmax",
                       value=spec.quantile_tables(qfun), seed=seed, clip_min=clip_min)


# --- p5: hand-worked example --------------------------------------------------------------

@pytest.mark.parametrize("method", METHODS)
def test_hand_worked_example(golden_dir, method):
    g = read_golden(golden_dir / "hand_example.txt")
    T, N, M = g["T"][0], g["N"][0], g["M"][0]
    lat = np.array(g["lat"], dtype=np.int32).reshape(T, N, M)
    step, done = oracle.simulate(lat, g["taus"], g["comm"][0], method)
    assert done.tolist() == g["done"]
    assert step.tolist() == g["step"]


# --- p1 / p2 / p3: limits and the strict inequality ---------------------------------------

@pytest.mark.parametrize("method", METHODS)
def test_threshold_above_everything(method):
    rng = np.random.default_rng(3)
    lat = rng.integers(0, 1000, size=(7, 5, 9), dtype=np.int32)
    step, done = oracle.simulate(lat, [BIG], 17, method)
    assert done[0] == 7 * 5 * 9
    assert step[0] == int(lat.astype(np.int64).sum(axis=2).max(axis=1).sum()) + 7 * 17


@pytest.mark.parametrize("method", METHODS)
def test_threshold_below_everything(method):
    rng = np.random.default_rng(4)
    lat = rng.integers(50, 1000, size=(6, 4, 8), dtype=np.int32)
    tau = int(lat[:, :, 0].min())
    step, done = oracle.simulate(lat, [tau, 0], 11, method)
    assert done.tolist() == [0, 0]
    assert step.tolist() == [6 * (tau + 11), 6 * 11]


@pytest.mark.parametrize("method", METHODS)
def test_tie_is_not_completed(method):
    lat = np.array([[[10, 20, 30, 40]]], dtype=np.int32)       # completion times 10 30 60 100
    step, done = oracle.simulate(lat, [60, 61, 100, 101], 0, method)
    assert done.tolist() == [2, 3, 3, 4]
    assert step.tolist() == [60, 61, 100, 100]


# --- p4: brute force on tiny inputs -------------------------------------------------------

@pytest.mark.parametrize("method", METHODS)
def test_exhaustive_small_alphabet(method):
    taus = list(range(0, 8))
    for vals in itertools.product((0, 1, 2), repeat=6):
        lat = np.array(vals, dtype=np.int32).reshape(1, 2, 3)
        step, done = oracle.simulate(lat, taus, 1, method)
        estep, edone = independent_counts(lat, taus, 1)
        assert done.tolist() == edone.tolist(), vals
        assert step.tolist() == estep.tolist(), vals


@pytest.mark.parametrize("method", METHODS)
@pytest.mark.parametrize("shape", [(3, 4, 5), (2, 1, 7), (5, 3, 1), (1, 6, 2)])
def test_random_small_vs_sort_and_search(method, shape):
    rng = np.random.default_rng(hash(shape) % 1000)
    lat = rng.integers(0, 50, size=shape, dtype=np.int32)
    lat[rng.random(shape) < 0.2] = 0                       # zero latencies are legal
    taus = rng.integers(0, 50 * shape[2] + 5, size=7)
    taus[3] = taus[1]                                      # duplicate, unsorted thresholds
    step, done = oracle.simulate(lat, taus, 9, method)
    estep, edone = independent_counts(lat, taus, 9)
    assert done.tolist() == edone.tolist()
    assert step.tolist() == estep.tolist()


def test_sorted_walk_equals_literal_loops():
    rng = np.random.default_rng(11)
    for T, N, M, K in [(4, 3, 16, 33), (9, 17, 5, 8), (2, 2, 64, 100)]:
        lat = rng.integers(0, 2000, size=(T, N, M), dtype=np.int32)
        totals = lat.sum(axis=2, dtype=np.int64)
        taus = rng.integers(0, int(totals.max()) + 10, size=K)
        a = oracle.simulate(lat, taus, 5, "literal")
        b = oracle.simulate(lat, taus, 5, "sorted")
        c = oracle.simulate_threaded(lat, taus, 5, "sorted", threads=3)
        assert a[0].tolist() == b[0].tolist() == c[0].tolist()
        assert a[1].tolist() == b[1].tolist() == c[1].tolist()


# --- p6: M = 1, maximum of iid workers (order statistics of the iid-max density, Section 4.2) --

def test_exponential_max_matches_harmonic_number():
    T, N, mean = 40000, 16, 10000.0
    lat = host.generate(iid_recipe(spec.q_exponential(mean), T, N, 1))
    step, done = oracle.simulate(lat, [BIG], 0, "sorted")
    H = sum(1.0 / j for j in range(1, N + 1))
    sd = mean * math.sqrt(sum(1.0 / j ** 2 for j in range(1, N + 1)))
    assert done[0] == T * N
    assert abs(step[0] / T - mean * H) <= 4 * sd / math.sqrt(T) + 1.0


def test_uniform_max_matches_closed_form():
    T, N, a, b = 40000, 16, 50000.0, 150000.0
    lat = host.generate(iid_recipe(spec.q_uniform(a, b), T, N, 1))
    step, _ = oracle.simulate(lat, [BIG], 0, "literal")
    sd = (b - a) * math.sqrt(N / ((N + 1) ** 2 * (N + 2)))
    assert abs(step[0] / T - (a + (b - a) * N / (N + 1))) <= 4 * sd / math.sqrt(T) + 1.0


# --- p7 / p8: normal latencies against the closed forms of Section 4.2-4.3 ----------------

def test_completed_count_matches_normal_cdf_sum():
    T, N, M, mu, sigma = 2000, 8, 32, 100000.0, 10000.0
    lat = host.generate(iid_recipe(spec.q_normal(mu, sigma), T, N, M, clip_min=1))
    taus = [int(mu * M * f) for f in (0.55, 0.8, 0.95, 0.99, 1.0, 1.01, 1.05)]
    _, done = oracle.simulate(lat, taus, 0, "sorted")
    m = np.arange(1, M + 1)
    for tau, d in zip(taus, done):
        expected = ndtr((tau - m * mu) / (sigma * np.sqrt(m))).sum()
        assert abs(d / (T * N) - expected) <= 0.03, (tau, d / (T * N), expected)


def test_mean_iteration_time_near_normal_max_approximation():
    T, N, M, mu, sigma = 4000, 64, 32, 100000.0, 10000.0
    lat = host.generate(iid_recipe(spec.q_normal(mu, sigma), T, N, M, clip_min=1))
    step, _ = oracle.simulate(lat, [BIG], 0, "sorted")
    gamma = 0.5772156649015329
    z = (1 - gamma) * ndtri(1 - 1 / N) + gamma * ndtri(1 - 1 / (math.e * N))
    measured = (step[0] / T - M * mu) / (sigma * math.sqrt(M))
    assert abs(measured - z) <= 0.05, (measured, z)
    # the slowest of more workers takes longer
    fewer, _ = oracle.simulate(lat[:, :8, :], [BIG], 0, "sorted")
    assert fewer[0] < step[0]


# --- p9 - p12: invariants -----------------------------------------------------------------

@pytest.fixture(scope="module")
def sample():
    rng = np.random.default_rng(21)
    lat = rng.integers(0, 3000, size=(12, 10, 24), dtype=np.int32)
    totals = lat.sum(axis=2, dtype=np.int64)
    taus = np.sort(rng.integers(0, int(totals.max()) + 100, size=40))
    return lat, taus


@pytest.mark.parametrize("method", METHODS)
def test_monotone_and_bounded(sample, method):
    lat, taus = sample
    T, N, M = lat.shape
    step, done = oracle.simulate(lat, taus, 7, method)
    assert np.all(np.diff(step) >= 0) and np.all(np.diff(done) >= 0)
    assert np.all(step <= T * (taus + 7))
    assert np.all(done <= T * N * M) and np.all(done >= 0)


@pytest.mark.parametrize("method", METHODS)
def test_additivity_and_permutations(sample, method):
    lat, taus = sample
    step, done = oracle.simulate(lat, taus, 7, method)
    a = oracle.simulate(lat[:5], taus, 7, method)
    b = oracle.simulate(lat[5:], taus, 7, method)
    assert (a[0] + b[0]).tolist() == step.tolist() and (a[1] + b[1]).tolist() == done.tolist()
    # splitting the workers: completed counts add
    l = oracle.simulate(lat[:, :4], taus, 7, method)
    r = oracle.simulate(lat[:, 4:], taus, 7, method)
    assert (l[1] + r[1]).tolist() == done.tolist()
    rng = np.random.default_rng(5)
    shuffled = lat[rng.permutation(lat.shape[0])][:, rng.permutation(lat.shape[1])]
    s2, d2 = oracle.simulate(shuffled, taus, 7, method)
    assert s2.tolist() == step.tolist() and d2.tolist() == done.tolist()
    # reversing the micro-batch order keeps every worker's total, hence the step times
    s3, _ = oracle.simulate(lat[:, :, ::-1], taus, 7, method)
    assert s3.tolist() == step.tolist()


@pytest.mark.parametrize("method", METHODS)
def test_comm_only_shifts_step_time(sample, method):
    lat, taus = sample
    s0, d0 = oracle.simulate(lat, taus, 0, method)
    s1, d1 = oracle.simulate(lat, taus, 123, method)
    assert (s1 - s0).tolist() == [123 * lat.shape[0]] * len(taus)
    assert d0.tolist() == d1.tolist()


def test_select_tau_identities(sample):
    lat, taus = sample
    T, N, M = lat.shape
    taus = np.append(taus, BIG)
    step, done = oracle.simulate(lat, taus, 50, "sorted")
    thr, seff, best = oracle.select_tau(step, done, taus, T, N, M, base_step_sum=int(step[-1]))
    assert seff[-1] == pytest.approx(1.0, abs=1e-12)             # no drops: speedup 1
    assert np.allclose(thr, done / step, rtol=1e-15)
    assert thr[best] == thr.max()
    extra = M / (done / (T * N)) - 1                             # compensation factor R = M/M~ - 1
    assert np.all(extra[done > 0] >= -1e-12)


def test_select_tau_tie_prefers_largest_threshold():
    # identical throughput 1/2 everywhere -> the largest tau (index 2) is chosen
    thr, _, best = oracle.select_tau([4, 8, 16, 2], [2, 4, 8, 1], [10, 30, 40, 20], 1, 1, 8)
    assert best == 2 and np.allclose(thr, 0.5)
    # cross-products that differ only beyond float64 resolution are still ordered exactly
    big = 3 * 10 ** 18
    _, _, best = oracle.select_tau([big, big - 1], [big - 1, big - 2], [1, 2], 1, 1, 1)
    assert best == 0


def test_per_step_speedup_matches_hand_example(golden_dir):
    g = read_golden(golden_dir / "hand_example.txt")
    lat = np.array(g["lat"], dtype=np.int32).reshape(1, 2, 3)
    s = oracle.per_step_speedup(lat, g["taus"], g["comm"][0])
    # S_i = (T_i + T^c)/(min(tau,T_i) + T^c) * (completed/N)/M with T_i = 13, N*M = 6
    expected = [14 / 6 * 3 / 6, 14 / 9 * 4 / 6, 14 / 14 * 5 / 6, 1.0]
    assert np.allclose(s, expected, rtol=1e-14)


def test_per_step_speedup_pins():
    rng = np.random.default_rng(31)
    lat = rng.integers(1, 3000, size=(9, 6, 12), dtype=np.int32)
    totals = lat.sum(axis=2, dtype=np.int64)
    taus = np.sort(rng.integers(1, int(totals.max()) + 100, size=25))
    taus = np.append(taus, BIG)
    # one iteration: the mean of ratios is the ratio itself, i.e. select_tau's S_eff from the integer sums
    one = lat[:1]
    step, done = oracle.simulate(one, taus, 70, "literal")
    _, seff, _ = oracle.select_tau(step, done, taus, 1, 6, 12, int(step[-1]))
    assert np.allclose(oracle.per_step_speedup(one, taus, 70), seff, rtol=1e-12)
    # no drops: every iteration's speedup is exactly 1
    assert oracle.per_step_speedup(lat, [BIG], 70)[0] == pytest.approx(1.0, abs=1e-12)
    # mean over iterations = mean of the single-iteration values, also with per-iteration T^c
    comm = rng.integers(0, 500, size=9)
    whole = oracle.per_step_speedup(lat, taus, comm)
    parts = np.mean([oracle.per_step_speedup(lat[i:i + 1], taus, comm[i:i + 1]) for i in range(9)], axis=0)
    assert np.allclose(whole, parts, rtol=1e-12)
    # S_i <= (T_i + c)/(min(tau,T_i) + c) and >= 0
    assert np.all(whole >= 0) and np.all(whole[:-1] <= (totals.max() + comm.max()) / taus[:-1].clip(1))
    with pytest.raises(oracle.OracleError):
        oracle.per_step_speedup(np.zeros((1, 1, 2), dtype=np.int32), [5], 0)      # 0/0 step time


def test_threaded_forms_agree_with_the_single_threaded_ones():
    """The oracle's helpers that spread trials over threads (used for the large comparisons) return what one thread
    returns: exactly for the integer sums, to rounding for the float mean over iterations."""
    rng = np.random.default_rng(77)
    lat = rng.integers(0, 4000, size=(53, 7, 9), dtype=np.int32)
    totals = lat.sum(axis=2, dtype=np.int64)
    taus = np.maximum(rng.integers(0, int(totals.max()) + 9, size=31), 1)
    comm = rng.integers(0, 300, size=53)
    for method in ("sorted", "literal"):
        one = oracle.simulate(lat, taus, 40, method)
        many = oracle.simulate_threaded(lat, taus, 40, method, 5)
        assert np.array_equal(one[0], many[0]) and np.array_equal(one[1], many[1])
    assert np.allclose(oracle.per_step_speedup(lat, taus, comm, threads=5), oracle.per_step_speedup(lat, taus, comm), rtol=1e-13)
    assert np.allclose(oracle.per_step_speedup(lat, taus, 12, threads=64), oracle.per_step_speedup(lat, taus, 12), rtol=1e-13)


def test_per_step_best_on_hand_worked_values(golden_dir):
    """The final argmax of Algorithm 2 on speedups worked by hand from Section 4.4's ratio.

    One iteration, two workers with completion times {4, 8} and {5, 10}, T = 10, T^c = 2, N*M = 4:
      tau  completed  S = completed/4 * (10 + 2)/(min(tau, 10) + 2)
        5      1      1/4 * 12/7  = 3/7   ~ 0.4286
        6      2      2/4 * 12/8  = 3/4
        9      3      3/4 * 12/11 = 9/11  ~ 0.8182      <- largest
       10      3      3/4 * 12/12 = 3/4                  (10 is not < 10)
       11      4      1
       50      4      1
    so S_eff peaks at 1 for tau = 11 and tau = 50: the tie goes to the larger threshold."""
    lat = np.array([[[4, 4], [5, 5]]], dtype=np.int32)
    taus = [5, 6, 9, 10, 11, 50]
    s = oracle.per_step_speedup(lat, taus, 2)
    assert np.allclose(s, [3 / 7, 3 / 4, 9 / 11, 3 / 4, 1.0, 1.0], rtol=1e-15)
    assert oracle.per_step_best(s, taus) == 5
    assert oracle.per_step_best(s[:4], taus[:4]) == 2                     # without the no-drop thresholds: tau = 9
    assert oracle.per_step_best(s[[5, 4, 2]], [50, 11, 9]) == 0           # any order of the list
    assert oracle.per_step_best([0.5, 0.7, 0.7, 0.2], [10, 30, 30, 40]) == 1    # equal tau too: the lowest index
    # two iterations: the mean of the two ratios, not the ratio of the means.  Second iteration: completion
    # times {1, 2} and {12, 20}, T = 20; at tau = 9: 2 completed, S = 2/4 * 22/11 = 1; mean (9/11 + 1)/2 = 10/11
    two = np.array([[[4, 4], [5, 5]], [[1, 1], [12, 8]]], dtype=np.int32)
    s2 = oracle.per_step_speedup(two, [9, 50], 2)
    assert np.allclose(s2, [10 / 11, 1.0], rtol=1e-15)
    assert oracle.per_step_best(s2, [9, 50]) == 1
    step, done = oracle.simulate(two, [9, 50], 2, "literal")             # ratio of means: 5/8 * (30+4)/(18+4) = 85/88
    _, ratio_of_means, _ = oracle.select_tau(step, done, [9, 50], 2, 2, 2, int(step[1]))
    assert ratio_of_means[0] == pytest.approx(85 / 88, rel=1e-15) and s2[0] < 0.95 < ratio_of_means[0]
    with pytest.raises(oracle.OracleError):
        oracle.per_step_best([], [])
    assert np.allclose(oracle.per_step_speedup(two, [9, 50], 2, threads=2), s2, rtol=1e-15)


# --- error behaviour ------------------------------------------------------------------------

@pytest.mark.parametrize("method", METHODS)
def test_negative_latency_is_rejected(method):
    lat = np.array([[[5, -1, 3]]], dtype=np.int32)
    with pytest.raises(oracle.OracleError) as e:
        oracle.simulate(lat, [4], 0, method)
    assert e.value.code == oracle.ERR_NEGATIVE_LATENCY


@pytest.mark.parametrize("method", METHODS)
def test_invalid_arguments(method):
    lat = np.ones((1, 1, 2), dtype=np.int32)
    with pytest.raises(oracle.OracleError):
        oracle.simulate(lat, [-1], 0, method)
    with pytest.raises(oracle.OracleError):
        oracle.simulate(lat, [1], -5, method)
    step, done = oracle.simulate(lat, [], 0, method)
    assert step.size == 0 and done.size == 0
