"""The lane bookkeeping of the kernel in which every lane holds whole rows, modelled in NumPy.

`dc_scan_rows_kernel` reads a chunk of 64 V vectors with coalesced loads (lane l takes vectors l, l + 64, ...),
passes them through a padded stretch of LDS so that lane l ends up with vectors l V ... l V + V - 1, meets the
thresholds from each row's end backwards, and, when a chunk may hold rows of several trials, finds every lane's trial
with a fixed-point quotient and the trials' maxima with a running maximum over lanes that restarts where the trial
changes.  This file writes those steps out for 64 "lanes" and checks them against their plain definitions; the kernel
itself is compared with the oracle in test_gpu_parity.py.
"""
import numpy as np
import pytest

LANES = np.arange(64)


def staged_shape(M: int):
    """(V vectors per lane and chunk, R rows per lane and chunk, vectors between two lanes' stretches in LDS)."""
    staged = 4 % M != 0
    V = M if staged else 4
    return V, 4 * V // M, (V | 1) if staged else 0


@pytest.mark.parametrize("M", [3, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 16])
def test_staging_gives_every_lane_its_own_rows(M):
    V, R, span = staged_shape(M)
    assert R == 4 and span % 2 == 1
    chunk = np.arange(64 * V)                                   # vector numbers of a chunk stand in for their contents
    lds = np.full(64 * span, -1)
    for j in range(V):                                          # write: the vector a lane loaded with instruction j
        i = 64 * j + LANES
        at = i if span == V else i + i // V
        assert np.all(lds[at] == -1)                            # no two vectors share a slot
        lds[at] = chunk[i]
    for j in range(V):                                          # read: lane l's j-th vector
        got = lds[LANES * span + j]
        assert np.array_equal(got, LANES * V + j)
    # eight consecutive lanes read 16 bytes each from eight different groups of four banks (32 banks of 4 bytes)
    for j in range(V):
        for l0 in range(0, 64, 8):
            banks = ((np.arange(l0, l0 + 8) * span + j) * 4) % 32
            assert len(set(banks.tolist())) == 8


@pytest.mark.parametrize("M", [1, 2, 3, 5, 8, 13, 16])
def test_backward_steps_count_what_a_search_over_every_element_counts(M):
    """Binning the (M-1-s)-th completion time of every row for s = 0, 1, ... until no row of the wave reaches the
    smallest threshold gives the histogram of all completion times at or above it."""
    rng = np.random.default_rng(M)
    for trial in range(20):
        rows = rng.integers(0, 300, size=(256, M))
        if trial % 4 == 0:
            rows[rng.integers(0, 256, 40)] = 0                  # rows of zeros: equal completion times
        p = np.cumsum(rows, axis=1)
        taus = np.sort(rng.integers(int(p.max() * rng.uniform(0, 1)), int(p.max()) + 2, size=17))
        want = np.bincount(np.searchsorted(taus, p.ravel(), side="right"), minlength=18)
        hist = np.zeros(18, dtype=np.int64)
        steps = 0
        for s in range(M):
            val = p[:, M - 1 - s]
            if not np.any(val >= taus[0]):
                break                                           # completion times do not decrease along a row
            steps += 1
            hist += np.bincount(np.searchsorted(taus, val, side="right"), minlength=18)
        assert np.array_equal(hist[1:], want[1:])               # bin 0 (below every threshold) is never read
        assert steps == int(np.max(np.sum(p >= taus[0], axis=1)))   # as many steps as the fullest row has entries in the grid


def test_fixed_point_quotient_finds_the_trial_of_every_row():
    """trial offset = (x * ceil(2^20 / N)) >> 20 must equal x // N for every worker count below 256 and every row
    x = within + 4 lane + 0..3 of a chunk counted from the head of the trial of the chunk's first row; from 256
    workers on the offset is 0 or 1."""
    for N in range(4, 256):
        recip = ((1 << 20) + N - 1) // N
        x = np.arange(0, N + 4 * 63 + 3 + 1)
        assert x.max() < 512 and int(x.max()) * recip < 2**32
        assert np.array_equal((x * recip) >> 20, x // N), N
    for N in (256, 257, 1000, 5001):
        x = np.arange(0, N + 4 * 63 + 3 + 1)
        assert np.array_equal((x >= N).astype(np.int64), x // N)


def test_chunk_to_chunk_update_of_the_first_rows_trial():
    for N in list(range(4, 256)) + [256, 257, 1000]:
        for row0 in (0, 256 * 7, 256 * 1000 + 0):
            trial, within = divmod(row0, N)
            for c in range(40):
                assert (trial, within) == divmod(row0 + 256 * c, N)
                trial += 256 // N
                within += 256 % N
                if within >= N:
                    within -= N
                    trial += 1


@pytest.mark.parametrize("N", [4, 5, 6, 7, 8, 10, 12, 30, 64, 100, 150, 200, 250, 252, 257, 1001])
def test_running_maximum_restarts_where_the_trial_changes(N):
    """A lane's four rows lie in one trial or in two.  Key = trial of the lane's last row, value = maximum over its rows
    in that trial; steps of 1, 2, 4, ... lanes, as many as a trial can span, leave each trial's maximum in the last
    lane with its key; a lane with a boundary inside adds its rows before the boundary to the previous trial itself."""
    rng = np.random.default_rng(N)
    trial_lanes = (N + 3) // 4 + 1
    for case in range(50):
        within = int(rng.integers(0, N))
        valid_lanes = 64 if case % 3 else int(rng.integers(1, 65))
        totals = rng.integers(1, 1000, size=(64, 4))
        totals[LANES >= valid_lanes] = 0
        rows = within + 4 * LANES[:, None] + np.arange(4)[None, :]           # counted from the head of the first row's trial
        trial_of = rows // N
        want = {}
        for lane in range(valid_lanes):
            for q in range(4):
                k = int(trial_of[lane, q])
                want[k] = max(want.get(k, 0), int(totals[lane, q]))
        t = trial_of[:, 3]
        before = np.where(trial_of[:, 0] != t, t * N - rows[:, 0], 0)
        assert np.all((before >= 0) & (before <= 3))
        q = np.arange(4)[None, :]
        m_before = np.where(q < before[:, None], totals, 0).max(axis=1)
        m = np.where(q < before[:, None], 0, totals).max(axis=1)
        key = np.where(LANES < valid_lanes, t, 0xFFFFFFFF)
        run = m.copy()
        d = 1
        while d < 64 and d < trial_lanes:
            up = np.concatenate([np.zeros(d, dtype=run.dtype), run[:-d]])
            up_key = np.concatenate([np.full(d, -1, dtype=np.int64), key[:-d].astype(np.int64)])
            take = (LANES >= d) & (up_key == key)
            run = np.where(take, np.maximum(run, up), run)
            d <<= 1
        nxt = np.concatenate([key[1:], [-2]])
        last = (LANES < valid_lanes) & ((LANES == 63) | (nxt != key))
        got = {}
        for lane in np.flatnonzero(last):
            assert int(key[lane]) not in got                    # one addition per key and chunk
            got[int(key[lane])] = int(run[lane])
        for lane in np.flatnonzero((LANES < valid_lanes) & (m_before > 0)):
            k = int(t[lane]) - 1
            got[k] = max(got.get(k, 0), int(m_before[lane]))
        assert got == want


# ---------------------------------------------------------------------------------------------
# dc_scan_row_lane_kernel: one row per lane, read word by word from the wave's copy of a chunk of 64 rows
# ---------------------------------------------------------------------------------------------
ROW_LANE_LENGTHS = [25, 27, 29, 31, 33, 34, 35, 37, 38, 39, 41, 42, 43, 45, 46, 47, 49, 50, 51, 53, 54, 55, 57, 58, 59,
                    61, 62, 63]


@pytest.mark.parametrize("M", ROW_LANE_LENGTHS)
def test_row_lane_chunks_are_whole_vectors_and_lanes_read_distinct_banks(M):
    """A chunk starts at a multiple of 64 rows, so its first element is a multiple of 4 whatever M; the last chunk of
    a trial holds N mod 64 rows, whole vectors iff N*M is a multiple of 4.  NB vectors per lane hold a chunk.  Lane l
    reads word l*M + m: 32 different banks per half wave for odd M, pairs of lanes for M = 2 mod 4."""
    nb = 8 if M <= 32 else 12 if M <= 48 else 16
    assert 64 * M % 4 == 0 and 64 * M // 4 <= 64 * nb
    for N in range(32, 200):
        if N * M % 4:
            continue
        for c0 in range(0, N, 64):
            here = min(64, N - c0)
            assert (c0 * M) % 4 == 0 and (here * M) % 4 == 0
    for m in (0, 1, M - 1):
        for half in (LANES[:32], LANES[32:]):
            banks = (half * M + m) % 32
            distinct = len(set(banks.tolist()))
            assert distinct == (32 if M % 2 else 16)


@pytest.mark.parametrize("M", [25, 27, 38, 45, 63])
def test_row_lane_backward_walk_counts_every_completion_time_in_the_grid(M):
    """total = sum of the row; val starts at the total and loses the row's elements from the end, one step at a time or
    four at once when 48 lanes are inside the grid or two steps have been taken; the walk stops at the first step in which no lane reaches the
    smallest threshold.  What it bins equals the histogram of all completion times at or above that threshold."""
    rng = np.random.default_rng(M)
    for trial in range(12):
        here = 64 if trial % 3 else int(rng.integers(1, 64))          # a partial chunk: lanes beyond it own no row
        rows = rng.integers(0, 300, size=(64, M))
        if trial % 4 == 0:
            rows[rng.integers(0, 64, 10)] = 0
        mine = LANES < here
        p = np.cumsum(rows, axis=1)
        top = int(p[mine].max())
        taus = np.sort(rng.integers(int(top * rng.choice([0.0, 0.3, 0.9])), top + 2, size=17))
        if trial == 5:
            taus[0] = 0                                                # every completion time is inside the grid
        want = np.bincount(np.searchsorted(taus, p[mine].ravel(), side="right"), minlength=18)
        hist = np.zeros(18, dtype=np.int64)
        val = np.where(mine, rows.sum(axis=1), 0)
        s = 0
        while s < M:
            reach = mine & (val >= taus[0])
            if not reach.any():
                break
            width = 4 if s + 4 <= M and (reach.sum() >= 48 or s >= 2) else 1
            for k in range(width):
                b = np.searchsorted(taus, val, side="right")
                np.add.at(hist, b[mine], 1)
                val = np.where(mine, val - rows[:, M - 1 - s - k], val)
            s += width
        assert np.array_equal(hist[1:], want[1:])                      # bin 0 (below every threshold) is never read


@pytest.mark.parametrize("N", [4, 5, 7, 8, 13, 31, 32, 50, 63])
def test_row_lane_maxima_over_small_trials(N):
    """The kernel with one row per lane over trials of fewer than 64 workers: lane l of a chunk holds row first + l of
    the whole run, its trial is that row number divided by N, and a running maximum over lanes that restarts where the
    trial changes (steps of 1, 2, 4, ... lanes below N) leaves each trial's maximum in the last lane of the trial."""
    rng = np.random.default_rng(N)
    for case in range(60):
        first = 64 * int(rng.integers(0, 1000))                 # chunks start at multiples of 64 rows
        here = 64 if case % 3 else int(rng.integers(1, 65))
        totals = rng.integers(0, 1000, size=64)
        valid = LANES < here
        trial = (first + LANES) // N
        want = {}
        for lane in range(here):
            want[int(trial[lane])] = max(want.get(int(trial[lane]), 0), int(totals[lane]))
        key = np.where(valid, trial, -1)
        run = totals.copy()
        d = 1
        while d < 64 and d < N:
            up = np.concatenate([np.zeros(d, dtype=run.dtype), run[:-d]])
            up_key = np.concatenate([np.full(d, -2, dtype=np.int64), key[:-d]])
            run = np.where((LANES >= d) & (up_key == key), np.maximum(run, up), run)
            d <<= 1
        nxt = np.concatenate([key[1:], [-3]])
        last = valid & ((LANES == 63) | (nxt != key))
        got = {int(key[lane]): int(run[lane]) for lane in np.flatnonzero(last)}
        assert len(got) == int(np.count_nonzero(last)) and got == want
