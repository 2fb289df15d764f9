"""Pins of the oracle's slice table (a derived index of the format of Sec. 3.3: the value array is read sequentially,
so where the values of a column range start is a count of set bits).  The table is checked against loops over single
bits written here, against the row offsets it has to start from and arrive at, and against the decoded matrix."""
import numpy as np
import pytest

import oracle
import salr_workloads as wl


def _pruned(rows, cols, density, seed):
    rng = np.random.default_rng(seed)
    w = wl.gaussian_bf16((rows, cols), 0.05, seed)
    keep = rng.random((rows, cols)) < density
    return np.where(keep, w, np.uint16(0)).astype(np.uint16)


def _bit(bitmap, n, k):
    return (int(bitmap[n, k // 32]) >> (k % 32)) & 1


@pytest.mark.parametrize("rows,cols,density", [(5, 128, 0.5), (3, 1024, 0.3), (4, 1056, 0.7), (2, 96, 1.0), (3, 4096, 0.5),
                                               (2, 2080, 0.05)])
def test_slice_table_against_bit_loops(rows, cols, density):
    w_hat = _pruned(rows, cols, density, 77 + rows + cols)
    bitmap, values, ro = oracle.encode(w_hat)
    table = oracle.slice_table(bitmap, ro, cols)
    chunks = (cols + 127) // 128
    for n in range(rows):
        for w in range(8):
            c0, c1 = chunks * w // 8, chunks * (w + 1) // 8
            before = sum(_bit(bitmap, n, k) for k in range(min(128 * c0, cols)))
            assert int(table[n, w, 0]) == int(ro[n]) + before
            longest = 0
            for c in range(c0, c1):
                longest = max(longest, sum(_bit(bitmap, n, k) for k in range(128 * c, min(128 * (c + 1), cols))))
            assert int(table[n, w, 1]) == longest


def test_slice_table_starts_at_the_row_offset_and_arrives_at_the_next():
    rows, cols = 9, 3200
    w_hat = _pruned(rows, cols, 0.4, 5)
    w_hat[4, :] = 0   # an empty row
    bitmap, values, ro = oracle.encode(w_hat)
    table = oracle.slice_table(bitmap, ro, cols)
    dense = oracle.decode(bitmap, values, ro, rows, cols)
    nz = (dense & 0x7FFF) != 0
    chunks = (cols + 127) // 128
    for n in range(rows):
        assert int(table[n, 0, 0]) == int(ro[n])
        for w in range(8):
            c0, c1 = chunks * w // 8, chunks * (w + 1) // 8
            in_slice = int(nz[n, 128 * c0:128 * c1].sum())
            nxt = int(table[n, w + 1, 0]) if w < 7 else int(ro[n + 1])
            assert int(table[n, w, 0]) + in_slice == nxt
            # the value the first entry points at is the first nonzero of the slice in the decoded row
            if in_slice:
                first = 128 * c0 + int(np.argmax(nz[n, 128 * c0:128 * c1]))
                assert int(values[int(table[n, w, 0])]) == int(dense[n, first])
            assert 0 <= int(table[n, w, 1]) <= 128
    assert np.all(table[4, :, 1] == 0) and np.all(table[4, :, 0] == ro[4])


def test_slice_table_of_a_full_and_of_a_short_row():
    # every bit set: offsets advance by 128 per chunk, every chunk holds 128 (the last, ragged one fewer)
    rows, cols = 2, 1120   # 8.75 chunks -> 9 chunks, the last of 96 columns
    w_hat = np.full((rows, cols), 0x3F80, dtype=np.uint16)
    bitmap, values, ro = oracle.encode(w_hat)
    table = oracle.slice_table(bitmap, ro, cols)
    chunks = 9
    for w in range(8):
        c0, c1 = chunks * w // 8, chunks * (w + 1) // 8
        assert int(table[1, w, 0]) == cols + 128 * c0
        assert int(table[1, w, 1]) == (0 if c1 == c0 else (96 if c0 == 8 else 128))
