"""Pins for the reverse-scan side of the oracle (suffix sums = the scan of the reversed row, reversed).

The forward oracle is pinned in test_oracle_pins.py; here the reversal wrappers are pinned to things that do not
go through them: closed forms, brute force, numpy on the un-flipped data, and planted mistakes."""
import numpy as np
import pytest

import oracle


def test_closed_forms():
    n = 1000
    ones = np.ones(n, np.int32)
    assert np.array_equal(oracle.scan_reverse(ones, "i32"), np.arange(n, 0, -1))            # n - i
    assert np.array_equal(oracle.scan_reverse(ones, "i32", exclusive=True), np.arange(n - 1, -1, -1))
    ar = np.arange(1, n + 1, dtype=np.int32)                                                  # sum_{j>=i} (j+1)
    i = np.arange(n, dtype=np.int64)
    assert np.array_equal(oracle.scan_reverse(ar, "i32").astype(np.int64), n * (n + 1) // 2 - i * (i + 1) // 2)
    f = np.ones(n, np.float32)
    assert np.array_equal(oracle.scan_reverse(f, "f32"), np.arange(n, 0, -1, dtype=np.float64))


@pytest.mark.parametrize("excl", [False, True])
def test_brute_force_and_numpy_on_unflipped_data(excl):
    rng = np.random.default_rng(7)
    x = rng.integers(-100, 100, size=(5, 37)).astype(np.int32)
    got = oracle.scan_reverse(x, "i32", exclusive=excl)
    for r in range(5):
        for i in range(37):
            want = int(x[r, i + 1:].sum()) if excl else int(x[r, i:].sum())
            assert got[r, i] == want
    xf = rng.standard_normal((3, 501)).astype(np.float32)
    gf = oracle.scan_reverse(xf, "f32", exclusive=excl)
    suffix = np.cumsum(xf[:, ::-1].astype(np.float64), axis=1)[:, ::-1]
    want = suffix - xf if excl else suffix
    assert np.allclose(gf, want, rtol=0, atol=1e-12)
    assert gf.shape == xf.shape


def test_relation_to_the_forward_scan_and_the_total():
    rng = np.random.default_rng(8)
    x = rng.integers(-5, 6, size=4096).astype(np.int32)
    fwd = oracle.scan(x, "i32").astype(np.int64)
    rev = oracle.scan_reverse(x, "i32").astype(np.int64)
    # inclusive prefix + inclusive suffix = total + the element itself
    assert np.array_equal(fwd + rev, fwd[-1] + x)
    assert oracle.scan_reverse(x, "i32", exclusive=True)[-1] == 0


def test_comparators_catch_planted_mistakes():
    rng = np.random.default_rng(9)
    x = rng.integers(-9, 10, size=(4, 300)).astype(np.int32)
    good = oracle.scan_reverse(x, "i32")
    assert oracle.compare_int_reverse(x, "i32", good) == (0, -1)
    assert oracle.compare_int_reverse(x, "i32", oracle.scan(x, "i32"))[0] > 0                # forward instead of reverse
    assert oracle.compare_int_reverse(x, "i32", oracle.scan_reverse(x, "i32", exclusive=True))[0] > 0
    bad = good.copy(); bad[2, 0] += 1                                                          # one wrong carry at a row start
    assert oracle.compare_int_reverse(x, "i32", bad)[0] == 1
    shifted = np.roll(good, 1, axis=1)                                                         # off by one element
    assert oracle.compare_int_reverse(x, "i32", shifted)[0] > 0
    xf = rng.standard_normal((2, 1000)).astype(np.float32)
    gf = oracle.scan_reverse(xf, "f32").astype(np.float32)
    assert oracle.compare_float_reverse(xf, "f32", gf).ok(1e-6)
    gf2 = gf.copy(); gf2[1, 999] *= 1.01                                                       # the last element: its norm is tiny
    assert not oracle.compare_float_reverse(xf, "f32", gf2).ok(1e-6)
    assert not oracle.compare_float_reverse(xf, "f32", oracle.scan(xf, "f32").astype(np.float32)).ok(1e-3)
    xi = rng.integers(-3, 4, size=700).astype(np.float32)
    assert oracle.compare_float_exact_reverse(xi, "f32", oracle.scan_reverse(xi, "f32").astype(np.float32)) == (0, -1)
