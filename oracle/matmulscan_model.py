"""The paper's schedule replayed on the CPU -- TEST INFRASTRUCTURE ONLY.

Where ``scan_oracle.c`` is the *definition* of the result, this module walks the
paper's own steps in the paper's order and notation, so that tests can show the
schedule (a) reproduces the states printed in Figure 1(a), (b) needs the number
of s x s products and rounds that Lemma 1 states, and (c) ends in the plain
prefix sum.  It is deliberately slow and literal: one numpy product per
BatchMatMul call, strided gathers and scatters exactly as Algorithm 1 names
them, no fusion of levels.

  * ``L(s)``, ``B(s)``            -- Section 2: the two constant left operands.
  * ``batch_matmul``              -- Algorithm 1, procedure BatchMatMul.
  * ``matmul_scan``               -- Algorithm 1, procedure MatMulScan (n = s^k).
  * ``matmul_scan_recursive``     -- Algorithm 2 (appendix, correctness proof).
  * ``matmul_scan_any_length``    -- Section 2.2, the four steps for arbitrary n.

All arithmetic is done in the dtype of the input array (use int64 / float64).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


def L(s: int, dtype=np.int64) -> np.ndarray:
    """Section 2: lower-triangular all-ones matrix, diagonal included -- entry (i, j) is 1 exactly when j <= i -- so
    that L_s w is the prefix sum of w."""
    i = np.arange(s)
    return (i[None, :] <= i[:, None]).astype(dtype)


def B(s: int, dtype=np.int64) -> np.ndarray:
    """Section 2, displayed equation: ones on the diagonal and down the first column, zeros elsewhere, so that
    B_s [a; q] = [a; q + a 1]  (the scalar a is added to every other entry)."""
    i = np.arange(s)
    return ((i[None, :] == i[:, None]) | (i[None, :] == 0)).astype(dtype)


@dataclass
class Trace:
    """Bookkeeping for Lemma 1: products issued per round and the vector after each round."""
    matmuls_per_round: list = field(default_factory=list)
    gathered_len_per_round: list = field(default_factory=list)
    states: list = field(default_factory=list)
    _pending: int = 0

    def count(self, k: int) -> None:
        self._pending += k

    def end_round(self, x: np.ndarray, gathered: int) -> None:
        self.matmuls_per_round.append(self._pending)
        self.gathered_len_per_round.append(gathered)
        self.states.append(x.copy())
        self._pending = 0

    @property
    def depth(self) -> int:
        return len(self.matmuls_per_round)

    @property
    def matmuls(self) -> int:
        return sum(self.matmuls_per_round)


def batch_matmul(y: np.ndarray, A: np.ndarray, trace: Trace | None = None) -> np.ndarray:
    """Algorithm 1, BatchMatMul: zero-pad y to a multiple of s^2, read every run of s^2
    entries as an s x s matrix in column-major order (so every run of s consecutive
    entries is one column), left-multiply each by A, write the products back in the same
    order and drop the padding."""
    s = A.shape[0]
    m = y.shape[0]
    nchunks = -(-m // (s * s))
    padded = np.zeros(nchunks * s * s, dtype=y.dtype)
    padded[:m] = y
    cols = padded.reshape(nchunks, s, s)          # cols[b, c, :] is column c of matrix b
    out = np.empty_like(cols)
    for b in range(nchunks):                       # one s x s product per chunk
        T = cols[b].T                              # T[:, c] = column c
        W = A @ T
        out[b] = W.T
    if trace is not None:
        trace.count(nchunks)
    return out.reshape(-1)[:m]


def _exact_log(n: int, s: int) -> int:
    k, p = 0, 1
    while p < n:
        p *= s
        k += 1
    if p != n:
        raise ValueError(f"Algorithm 1 is defined for n = s^k only (n={n}, s={s})")
    return k


@dataclass(frozen=True)
class Round:
    """One round of Algorithm 1: which entries of x it touches and which constant matrix multiplies them."""
    phase: str          # "up": first phase, operand L_s;  "down": second phase, operand B_s
    t: int              # the level
    first: int          # index of the first entry touched
    stride: int         # distance between touched entries

    def touched(self, n: int) -> np.ndarray:
        return np.arange(self.first, n, self.stride)


def schedule(n: int, s: int) -> list:
    """Algorithm 1 as a table of rounds, in execution order, for n = s^k.  First phase, levels t = 0 .. k-1: the
    entries s^t - 1, 2 s^t - 1, ... (the last entry of every block of s^t) are scanned in runs of s.  Second phase,
    levels t = k-1 down to 1: starting from the same entry s^t - 1 but with the finer stride s^(t-1), every run of s
    gets its first entry (a finished prefix) added to the s - 1 partial sums behind it."""
    k = _exact_log(n, s)
    first_phase = [Round("up", t, s ** t - 1, s ** t) for t in range(k)]
    second_phase = [Round("down", t, s ** t - 1, s ** (t - 1)) for t in reversed(range(1, k))]
    return first_phase + second_phase


def matmul_scan(x: np.ndarray, s: int, trace: Trace | None = None) -> np.ndarray:
    """Algorithm 1, MatMulScan, round by round from `schedule`: gather the touched entries, BatchMatMul them with
    the round's matrix, scatter them back.  Returns a new array; n must be s^k."""
    x = np.array(x, copy=True)
    n = x.shape[0]
    operand = {"up": L(s, x.dtype), "down": B(s, x.dtype)}
    for rnd in schedule(n, s):
        where = rnd.touched(n)
        x[where] = batch_matmul(x[where], operand[rnd.phase], trace)
        if trace is not None:
            trace.end_round(x, where.size)
    return x


def gathered_lengths(n: int, s: int):
    """Lengths of the subvectors Algorithm 1 gathers, round by round, for n = s^k (how many entries each round of
    `schedule` touches)."""
    return [rnd.touched(n).size for rnd in schedule(n, s)]


def product_count(n: int, s: int) -> int:
    """Number of s x s products Algorithm 1 issues for n = s^k: BatchMatMul pads every gathered vector
    to a multiple of s^2 and multiplies chunk by chunk (the quantity Lemma 1 bounds)."""
    return sum(-(-m // (s * s)) for m in gathered_lengths(n, s))


def _recurse(z: np.ndarray, s: int, Ls, Bs, trace) -> np.ndarray:
    """Algorithm 2, Recurse.  Precondition: every aligned run of s entries of z already holds
    its local prefix sums.  Postcondition: z holds the prefix sums of the whole vector."""
    if z.shape[0] <= s:
        return z
    start = s - 1
    z[start::s] = batch_matmul(z[start::s].copy(), Ls, trace)
    z[start::s] = _recurse(z[start::s].copy(), s, Ls, Bs, trace)
    z[start:] = batch_matmul(z[start:].copy(), Bs, trace)
    return z


def matmul_scan_recursive(x: np.ndarray, s: int, trace: Trace | None = None) -> np.ndarray:
    """Algorithm 2, MatMulScanRecursive: local scans of every s-run, then Recurse."""
    x = np.array(x, copy=True)
    Ls, Bs = L(s, x.dtype), B(s, x.dtype)
    z = batch_matmul(x, Ls, trace)
    return _recurse(z, s, Ls, Bs, trace)


def base_s_digits(n: int, s: int):
    """Section 2.2: n = sum_i mu_i s^(k_i), k_1 = floor(log_s n) > k_2 > ... >= 0, 0 <= mu_i < s.
    Returns [(mu_i, k_i)] for the non-zero digits, highest power first."""
    digs, k = [], 0
    while n:
        n, d = divmod(n, s)
        if d:
            digs.append((d, k))
        k += 1
    return digs[::-1]


def _broadcast_add(seg: np.ndarray, alpha, s: int, trace: Trace | None) -> np.ndarray:
    """Section 2.2 step 4 (and its time analysis): view the segment as an (s-1) x ceil(m/(s-1))
    column-major matrix, put a constant row holding alpha on top, left-multiply by B_s, and
    read the segment back from rows 1..s-1."""
    m = seg.shape[0]
    ncols = -(-m // (s - 1))
    body = np.zeros(ncols * (s - 1), dtype=seg.dtype)
    body[:m] = seg
    M = np.empty((s, ncols), dtype=seg.dtype)
    M[0, :] = alpha
    M[1:, :] = body.reshape(ncols, s - 1).T
    W = B(s, seg.dtype) @ M
    if trace is not None:
        trace.count(-(-ncols // s))                       # s columns per s x s product
    return W[1:, :].T.reshape(-1)[:m]


def matmul_scan_any_length(x: np.ndarray, s: int):
    """Section 2.2: (1) Algorithm 1 on each base-s segment, (2) gather the last entry (the
    total) of every segment into w, (3) zero-pad w to a power of s and scan it with
    Algorithm 1, (4) broadcast-add w_i onto segment i+1.  Returns (result, info) where info
    holds the per-step product counts and depths."""
    x = np.array(x, copy=True)
    n = x.shape[0]
    info = {"segments": [], "step1_depth": 0, "step1_matmuls": 0, "w_len": 0, "step3_depth": 0,
            "step3_matmuls": 0, "step4_matmuls": 0}
    if n == 0:
        return x, info
    pos, bounds = 0, []
    for mu, k in base_s_digits(n, s):
        for _ in range(mu):
            bounds.append((pos, pos + s ** k, k))
            pos += s ** k
    assert pos == n
    info["segments"] = bounds
    for a, b, k in bounds:                                 # step 1
        tr = Trace()
        x[a:b] = matmul_scan(x[a:b], s, tr)
        info["step1_depth"] = max(info["step1_depth"], tr.depth)
        info["step1_matmuls"] += tr.matmuls
    w = np.array([x[b - 1] for _, b, _ in bounds], dtype=x.dtype)   # step 2
    info["w_len"] = int(w.shape[0])
    q, p = 0, 1                                            # step 3
    while p < w.shape[0]:
        p *= s
        q += 1
    wpad = np.zeros(p, dtype=x.dtype)
    wpad[: w.shape[0]] = w
    tr = Trace()
    w = matmul_scan(wpad, s, tr)[: w.shape[0]]
    info["step3_depth"], info["step3_matmuls"] = tr.depth, tr.matmuls
    tr4 = Trace()
    for i in range(len(bounds) - 1):                       # step 4
        a, b, _ = bounds[i + 1]
        x[a:b] = _broadcast_add(x[a:b], w[i], s, tr4)
    info["step4_matmuls"] = tr4._pending
    return x, info
