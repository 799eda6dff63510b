"""The index algebra of the kernel for arbitrary row lengths, modelled lane by lane in NumPy.

`dc_scan_flat_kernel` reads the tensor as one run of 16-byte vectors; every lane works out from its
position alone where the row heads fall inside its four elements, fetches one running sum from the
lane that holds the previous row end, and takes a wave-uniform carry for a row that began in an
earlier load.  This file writes that arithmetic out for 64 "lanes" of a NumPy array (sums modulo
2^32 as on the GPU) and checks it against plain cumulative sums over many row lengths, unit sizes,
alignments and value ranges, including loads past the end of a unit.  It pins the algebra on the
CPU; the kernel itself is compared with the oracle in test_gpu_parity.py.
"""
import numpy as np
import pytest

MASK = 0xFFFFFFFF
LANES = np.arange(64)


def stream_unit(vec_space: np.ndarray, start: int, length: int, M: int, loads_per_batch: int = 4):
    """Completion times of the `length` elements (whole rows of M) that begin at element `start` of
    vector space, the largest of them, and each row's total as found at the lane holding its last
    element.  Loads past the unit's last one (a batch may reach there) must yield zeros only."""
    v0, k = start >> 2, start & 3                       # first vector; components of it before the unit
    nv = (k + length + 3) >> 2
    nloads = (nv + 63) // 64
    q0 = 4 * LANES - k                                   # unit-relative element of each lane's first component
    pos0 = np.where(q0 >= 0, q0 % M, (M - ((-q0) % M)) % M).astype(np.int64)
    row = np.where(q0 >= 0, q0 // M, -((-q0 + M - 1) // M)).astype(np.int64)    # floor(q0 / M)
    pos_last = (252 - k) % M
    step, row_step = 256 % M, 256 // M
    out = np.full(length, -1, dtype=np.int64)
    totals = {}
    carry = prev2 = prev3 = 0
    top = 0
    for i in range(-(-nloads // loads_per_batch) * loads_per_batch):
        first = k if i == 0 else 0
        limit = max(0, min(length + k - 256 * i, 256))
        x = np.zeros((64, 4), dtype=np.int64)
        valid = np.zeros((64, 4), dtype=bool)
        for c in range(4):
            e = 4 * LANES + c
            valid[:, c] = (e >= first) & (e < limit)
            loaded = ((64 * i + LANES) < nv) & (i < nloads)
            assert not np.any(valid[:, c] & ~loaded)    # every valid component lies in a vector that is read
            idx = 4 * (v0 + 64 * i + LANES) + c
            x[valid[:, c], c] = vec_space[idx[valid[:, c]]]
        if M >= 4:
            s = np.cumsum(x, axis=1) & MASK
            before = (np.cumsum(s[:, 3]) - s[:, 3]) & MASK
            ce = M - pos0                                # components 0..ce-1 continue the first element's row
            se = np.where(ce > 3, s[:, 3], np.where(ce > 2, s[:, 2], np.where(ce > 1, s[:, 1], s[:, 0])))
            back = 4 * LANES - 1 - pos0                  # 4 * lane + component of the previous row end
            src = np.maximum(back, 0) >> 2
            assert np.all((ce <= 4)[src[back >= 0]])     # the lane asked holds a row end
            prev_end = ((before + se) & MASK)[src]
            a = (before - np.where(back >= 0, prev_end, (-carry) & MASK)) & MASK
            b = (-se) & MASK
            p = np.stack([(s[:, c] + np.where(ce > c, a, b)) & MASK for c in range(4)], axis=1)
            carry = int(p[63, 3]) if M - pos_last != 4 else 0
        else:
            y = np.zeros((64, 6), dtype=np.int64)
            y[:, 2:] = x
            y[1:, 0], y[1:, 1] = x[:-1, 2], x[:-1, 3]
            y[0, 0], y[0, 1] = prev2, prev3
            p = np.zeros((64, 4), dtype=np.int64)
            for c in range(4):
                pc = (pos0 + c) % M
                p[:, c] = (y[:, c + 2] + np.where(pc >= 1, y[:, c + 1], 0) + np.where(pc >= 2, y[:, c], 0)) & MASK
            prev2, prev3 = int(x[63, 2]), int(x[63, 3])
        assert np.all(p[~valid] == 0)                    # masked components never disturb a maximum
        top = max(top, int(p.max()))
        for c in range(4):
            q = 256 * i + 4 * LANES + c - k
            out[q[valid[:, c]]] = p[valid[:, c], c]
        for lane in range(64):                           # row ends, as the per-worker totals kernel finds them
            if M >= 4:
                end = M - pos0[lane]
                if end <= 4 and valid[lane, end - 1]:
                    assert int(row[lane]) not in totals
                    totals[int(row[lane])] = int(p[lane, end - 1])
            else:
                for c in range(4):
                    e = pos0[lane] + c
                    if valid[lane, c] and e % M == M - 1:
                        r = int(row[lane] + e // M)
                        assert r not in totals
                        totals[r] = int(p[lane, c])
        pos0 = pos0 + step
        wrapped = pos0 >= M
        pos0 = np.where(wrapped, pos0 - M, pos0)
        row = row + row_step + wrapped
        pos_last = (pos_last + step) % M
    return out, top, totals


ROW_LENGTHS = [1, 2, 3, 4, 5, 6, 7, 9, 13, 31, 63, 64, 65, 100, 127, 255, 256, 257, 260, 300, 511, 700, 1001]


@pytest.mark.parametrize("M", ROW_LENGTHS)
def test_lane_arithmetic_gives_the_prefix_sums(M):
    rng = np.random.default_rng(M)
    for case in range(30):
        rows = int(rng.integers(1, max(2, 3000 // M)))
        off = int(rng.integers(0, 4))                    # 4-byte words between the 16-byte boundary and the tensor
        before_rows = int(rng.integers(0, 3)) * M        # rows of a neighbouring unit in front
        top = int(rng.choice([1, 5, 1000, (2**31 - 1) // M]))
        total = before_rows + rows * M + int(rng.integers(0, 3)) * M
        lat = rng.integers(0, top + 1, size=total).astype(np.int64)
        vec_space = np.concatenate([np.full(off, 777777), lat, np.full(8, 999999)])     # junk outside the tensor
        got, biggest, totals = stream_unit(vec_space, before_rows + off, rows * M, M)
        ref = np.cumsum(lat[before_rows:before_rows + rows * M].reshape(rows, M), axis=1)
        assert np.array_equal(got, ref.reshape(-1)), (M, rows, off, before_rows)
        assert biggest == ref.max()
        assert sorted(totals) == list(range(rows)) and all(totals[r] == ref[r, -1] for r in range(rows))


def test_sums_may_wrap_but_differences_stay_exact():
    M, rows = 5, 200                                     # 1000 elements near the largest legal latency: the load-wide sums wrap
    top = (2**31 - 1) // M
    lat = np.full(rows * M, top, dtype=np.int64)
    got, biggest, _ = stream_unit(np.concatenate([lat, np.zeros(8, dtype=np.int64)]), 0, rows * M, M)
    assert biggest == top * M and np.array_equal(got.reshape(rows, M), np.cumsum(lat.reshape(rows, M), axis=1))
