"""Pins for the segmented side of the oracle (rows of different lengths, each scanned on its own)."""
import numpy as np
import pytest

import oracle


def offsets_from(lengths, start=0):
    return np.concatenate([[start], start + np.cumsum(lengths)]).astype(np.int64)


def test_rows_restart_and_gaps_stay_zero():
    x = np.ones(20, np.int32)
    off = np.array([2, 5, 5, 11, 18], np.int64)                 # rows [2,5) [5,5) [5,11) [11,18); 0..1 and 18..19 outside
    got = oracle.scan_segments(x, "i32", off)
    want = np.array([0, 0, 1, 2, 3, 1, 2, 3, 4, 5, 6, 1, 2, 3, 4, 5, 6, 7, 0, 0])
    assert np.array_equal(got, want)
    assert np.array_equal(oracle.scan_segments(x, "i32", off, exclusive=True), np.maximum(want - 1, 0))
    rev = np.array([0, 0, 3, 2, 1, 6, 5, 4, 3, 2, 1, 7, 6, 5, 4, 3, 2, 1, 0, 0])
    assert np.array_equal(oracle.scan_segments(x, "i32", off, reverse=True), rev)


@pytest.mark.parametrize("reverse", [False, True])
@pytest.mark.parametrize("excl", [False, True])
def test_brute_force_against_numpy_per_row(excl, reverse):
    rng = np.random.default_rng(5)
    lengths = rng.integers(0, 40, size=30)
    off = offsets_from(lengths, start=3)
    x = rng.integers(-50, 50, size=int(off[-1]) + 4).astype(np.int32)
    got = oracle.scan_segments(x, "i32", off, exclusive=excl, reverse=reverse)
    for r in range(30):
        a, b = int(off[r]), int(off[r + 1])
        row = x[a:b].astype(np.int64)
        if reverse:
            inc = np.cumsum(row[::-1])[::-1]
        else:
            inc = np.cumsum(row)
        want = inc - row if excl else inc
        assert np.array_equal(got[a:b], want)
    assert not got[:3].any() and not got[int(off[-1]):].any()


def test_equal_rows_agree_with_the_batched_oracle():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((7, 300)).astype(np.float32)
    off = np.arange(8, dtype=np.int64) * 300
    assert np.array_equal(oracle.scan_segments(x, "f32", off), oracle.scan(x, "f32").reshape(-1))
    assert np.array_equal(oracle.scan_segments(x, "f32", off, exclusive=True, reverse=True),
                          oracle.scan_reverse(x, "f32", exclusive=True).reshape(-1))


def test_comparator_catches_planted_mistakes():
    rng = np.random.default_rng(4)
    lengths = np.array([5, 0, 100, 1, 33, 700])
    off = offsets_from(lengths)
    x = rng.integers(-9, 10, size=int(off[-1])).astype(np.int32)
    good = oracle.scan_segments(x, "i32", off)
    assert oracle.compare_segments(x, "i32", off, good) == (0, -1)
    leaked = oracle.scan(x, "i32")                                # the carry was not reset at the row starts
    nb, first = oracle.compare_segments(x, "i32", off, leaked)
    assert nb > 0 and first == 2
    bad = good.copy(); bad[int(off[5])] += 1                      # first element of the last row
    assert oracle.compare_segments(x, "i32", off, bad) == (1, 5)
    assert oracle.compare_segments(x, "i32", off, good, reverse=True)[0] > 0
    xf = rng.standard_normal(int(off[-1])).astype(np.float32)
    gf = oracle.scan_segments(xf, "f32", off).astype(np.float32)
    assert oracle.compare_segments(xf, "f32", off, gf).ok(1e-6)
    gf[int(off[4]) + 2] += 1e-2
    rep = oracle.compare_segments(xf, "f32", off, gf)
    assert not rep.ok(1e-5) and rep.worst_index == int(off[4]) + 2
