"""Pins for the CPU replay of the paper's schedule (oracle/matmulscan_model.py).

Checked against: the state rows printed in Figure 1(a); Lemma 1's depth and product bound
(tests/golden/lemma1_counts.txt holds the lemma's formulas evaluated, nothing else); the
block-sum invariant that defines what the up-sweep must leave behind; the displayed
definition of B_s; the plain sequential oracle; and the depth / size statements of
Section 2.2 for n that is not a power of s.
"""
import os

import numpy as np
import pytest

import oracle
from oracle import matmulscan_model as mm

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_rows(name):
    rows = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append([int(t) for t in line.split()])
    return rows


def test_constant_matrices_match_their_definitions():
    w = np.array([3, -1, 4, 1, -5], dtype=np.int64)
    assert np.array_equal(mm.L(5) @ w, np.cumsum(w))                       # L_s w = prefix sum of w
    a, q = 7, np.array([10, 20, 30, 40], dtype=np.int64)
    assert np.array_equal(mm.B(5) @ np.concatenate([[a], q]), np.concatenate([[a], q + a]))   # B_s [a; q] = [a; q + a 1]
    Bs = mm.B(4)
    assert Bs.tolist() == [[1, 0, 0, 0], [1, 1, 0, 0], [1, 0, 1, 0], [1, 0, 0, 1]]      # the displayed matrix
    assert mm.L(3).tolist() == [[1, 0, 0], [1, 1, 0], [1, 1, 1]]


def test_figure_1a_state_rows():
    rows = read_rows("fig1a_s4_states.txt")
    tr = mm.Trace()
    out = mm.matmul_scan(np.array(rows[0], dtype=np.int64), 4, tr)
    assert tr.depth == 3                                                   # 2k-1 with k = 2
    assert [s.tolist() for s in tr.states] == rows[1:]
    assert out.tolist() == rows[3]


def test_batch_matmul_reads_runs_of_s_as_columns():
    """Figure 2's setting (y = 1..16, A = L_2): each run of s entries is one column, so L_2 turns
    every aligned pair (a, b) into (a, a + b); with s = 4 every aligned quadruple gets its local scan."""
    y = np.arange(1, 17, dtype=np.int64)
    z = mm.batch_matmul(y, mm.L(2))
    assert z.tolist() == [1, 3, 3, 7, 5, 11, 7, 15, 9, 19, 11, 23, 13, 27, 15, 31]
    z4 = mm.batch_matmul(y, mm.L(4))
    assert z4.tolist() == np.concatenate([np.cumsum(y[i:i + 4]) for i in range(0, 16, 4)]).tolist()
    # zero-padding is dropped again: a length that is not a multiple of s^2 or of s
    y7 = np.arange(1, 8, dtype=np.int64)
    assert mm.batch_matmul(y7, mm.L(4)).tolist() == [1, 3, 6, 10, 5, 11, 18]
    # an asymmetric operand shows the operand order and the column orientation are right
    A = np.array([[1, 0], [5, 1]], dtype=np.int64)                          # (a, b) -> (a, 5a + b)
    assert mm.batch_matmul(np.array([1, 2, 3, 4], dtype=np.int64), A).tolist() == [1, 7, 3, 19]


@pytest.mark.parametrize("s,k", [(2, 4), (4, 2), (4, 5), (16, 1), (16, 2), (16, 3)])
def test_up_sweep_leaves_block_sums(s, k):
    """After up-sweep round t every index congruent to -1 mod s^(t+1) holds the sum of its aligned
    block of s^(t+1) inputs (what 'prefix sums correct on an exponentially increasing set' means)."""
    n = s ** k
    rng = np.random.default_rng(s * 100 + k)
    x = rng.integers(-50, 50, n).astype(np.int64)
    tr = mm.Trace()
    mm.matmul_scan(x, s, tr)
    for t in range(k):
        blk = s ** (t + 1)
        st = tr.states[t]
        sums = x.reshape(-1, blk).sum(axis=1)
        assert np.array_equal(st[blk - 1::blk], sums)
    # the last up-sweep state already has the grand total in place
    assert tr.states[k - 1][-1] == x.sum()


def lemma_rows():
    return [tuple(r) for r in read_rows("lemma1_counts.txt")]


@pytest.mark.parametrize("s,k,n,depth,bound", [r for r in lemma_rows() if r[2] <= 65536])
def test_lemma1_depth_and_product_bound(s, k, n, depth, bound):
    rng = np.random.default_rng(n)
    x = rng.integers(-100, 100, n).astype(np.int64)
    tr = mm.Trace()
    out = mm.matmul_scan(x, s, tr)
    assert np.array_equal(out, np.cumsum(x))
    assert tr.depth == depth == 2 * k - 1
    assert tr.matmuls <= bound
    # per-round bounds used in the lemma's proof: ceil(n / s^(t+2)) up, ceil(n / s^(t+1)) down
    ups, downs = tr.matmuls_per_round[:k], tr.matmuls_per_round[k:]
    for t, c in enumerate(ups):
        assert c <= -(-n // s ** (t + 2))
    for c, t in zip(downs, range(k - 1, 0, -1)):
        assert c <= -(-n // s ** (t + 1))


def closed_form_matmuls(n, s, k):
    """Products Algorithm 1 issues for n = s^k, from the gathered lengths alone."""
    total = 0
    for t in range(k):
        m = (n - s ** t) // s ** t + 1
        total += -(-m // (s * s))
    for t in range(k - 1, 0, -1):
        m = (n - s ** t) // s ** (t - 1) + 1
        total += -(-m // (s * s))
    return total


def test_product_counts_at_benchmark_sizes():
    """Counts at sizes too large to replay are taken from the gathered-vector lengths; the formula is first
    validated against the replay at sizes that can be run, then compared with the lemma's bound."""
    for s, k in [(2, 4), (4, 5), (4, 6), (16, 2), (16, 3), (16, 4), (32, 2), (32, 3)]:
        n = s ** k
        tr = mm.Trace()
        mm.matmul_scan(np.ones(n, dtype=np.int64), s, tr)
        assert tr.matmuls == closed_form_matmuls(n, s, k)
        ks = list(range(k)) + list(range(k - 1, 0, -1))
        lens = [(n - s ** t) // s ** t + 1 for t in range(k)] + [(n - s ** t) // s ** (t - 1) + 1 for t in range(k - 1, 0, -1)]
        assert tr.gathered_len_per_round == lens and len(ks) == tr.depth
    for s, k, n, depth, bound in lemma_rows():
        assert closed_form_matmuls(n, s, k) == mm.product_count(n, s) <= bound
        assert len(mm.gathered_lengths(n, s)) == depth
    # the counts the GPU tests expect at full size
    assert mm.product_count(16 ** 7, 16) == 2236963 and mm.product_count(4 ** 14, 4) == 44739243
    assert mm.product_count(32 ** 5, 32) == 67651


@pytest.mark.parametrize("s,k", [(2, 5), (3, 4), (4, 3), (16, 2), (16, 3)])
def test_recursive_form_equals_iterative_and_oracle(s, k):
    n = s ** k
    rng = np.random.default_rng(k * 31 + s)
    x = rng.integers(-128, 128, n).astype(np.int64)
    a = mm.matmul_scan(x, s)
    b = mm.matmul_scan_recursive(x, s)
    ref = oracle.scan_int64(x.astype(np.int32), "i32")
    assert np.array_equal(a, ref) and np.array_equal(b, ref)
    xf = rng.standard_normal(n)
    yf = mm.matmul_scan(xf, s)
    ref_f = oracle.scan(xf.astype(np.float32), "f32")
    yf32 = mm.matmul_scan(xf.astype(np.float32).astype(np.float64), s)
    assert np.max(np.abs(yf32 - ref_f)) < 1e-9
    assert np.max(np.abs(yf - np.cumsum(xf))) < 1e-9


def test_recurse_postcondition_from_its_precondition():
    """Appendix: given local prefix sums on every aligned run of s, Recurse returns the full prefix sums."""
    s, n = 4, 64
    rng = np.random.default_rng(1)
    x = rng.integers(-9, 9, n).astype(np.int64)
    z = np.concatenate([np.cumsum(x[i:i + s]) for i in range(0, n, s)])
    out = mm._recurse(z.copy(), s, mm.L(s), mm.B(s), None)
    assert np.array_equal(out, np.cumsum(x))


def test_algorithm_1_rejects_lengths_that_are_not_powers():
    with pytest.raises(ValueError):
        mm.matmul_scan(np.ones(48, dtype=np.int64), 4)


def test_base_s_digits():
    assert mm.base_s_digits(100_000_007, 16) == [(5, 6), (15, 5), (5, 4), (14, 3), (1, 2), (7, 0)]
    assert sum(mu * 16 ** k for mu, k in mm.base_s_digits(100_000_007, 16)) == 100_000_007
    assert sum(mu for mu, _ in mm.base_s_digits(100_000_007, 16)) == 47      # segments
    assert mm.base_s_digits(4096, 16) == [(1, 3)]


@pytest.mark.parametrize("s,n", [(4, 1), (4, 3), (4, 23), (4, 255), (4, 1000), (16, 17), (16, 4097), (16, 70000), (2, 77)])
def test_any_length_extension(s, n):
    rng = np.random.default_rng(n + s)
    x = rng.integers(-100, 100, n).astype(np.int64)
    out, info = mm.matmul_scan_any_length(x, s)
    assert np.array_equal(out, np.cumsum(x))
    k1 = 0
    while s ** (k1 + 1) <= n:
        k1 += 1
    # Section 2.2, depth paragraph: step 1 has depth at most 2 k1 - 1, step 4 adds one round
    assert info["step1_depth"] <= max(2 * k1 - 1, 0)
    assert max(info["step1_depth"], 0) + 1 <= max(2 * k1, 1)
    # one total per segment, fewer than s segments per power, k1 + 1 powers at most
    assert info["w_len"] == len(info["segments"]) <= (k1 + 1) * (s - 1)
    # matrix-multiplication paragraph: O(n / s^2) products overall
    total = info["step1_matmuls"] + info["step3_matmuls"] + info["step4_matmuls"]
    assert total <= -(-4 * n // (s * (s - 1))) + 4 * s * (k1 + 1) ** 2
