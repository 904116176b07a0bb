"""CPU oracle for the two scan applications -- TEST INFRASTRUCTURE ONLY.

The paper's introduction motivates the scan with stream compaction / splitting and with Blelloch's
reduction of radix sort to prefix sums.  These functions follow that reduction step by step on top of
the plain sequential scan of ``scan_oracle.c`` (so they check the *reduction*, not just the result); the
tests pin them against the things they must equal by definition: a boolean filter, a stable sort,
brute-force selection on tiny inputs, and the permutation / order invariants.
"""
from __future__ import annotations

import numpy as np

import oracle


def compact(values: np.ndarray, mask: np.ndarray):
    """Keep values[i] where mask[i] != 0, in order: destination index = exclusive scan of the 0/1 mask.
    Returns (kept values, positions)."""
    mask = np.ascontiguousarray(mask, dtype=np.int8)
    pos = oracle.scan(mask, "i8", exclusive=True)
    count = int(pos[-1]) + int(mask[-1]) if mask.size else 0
    out = np.empty(count, dtype=values.dtype)
    for i in np.nonzero(mask)[0]:                 # the scatter, element by element
        out[pos[i]] = values[i]
    return out, pos


def split(keys: np.ndarray, vals, bit: int):
    """One split pass: keys whose `bit` is 0 move to the front, the others behind them, both in their old
    order.  f = (bit is 0); pos = exclusive_scan(f); Z = total zeros; destination = pos if f else Z + (i - pos)."""
    n = keys.size
    f = (((keys >> np.uint32(bit)) & np.uint32(1)) ^ np.uint32(1)).astype(np.int8)
    pos = oracle.scan(f, "i8", exclusive=True).astype(np.int64)
    zeros = int(pos[-1]) + int(f[-1])
    idx = np.arange(n, dtype=np.int64)
    dst = np.where(f != 0, pos, zeros + (idx - pos))
    out_k = np.empty_like(keys)
    out_k[dst] = keys
    out_v = None
    if vals is not None:
        out_v = np.empty_like(vals)
        out_v[dst] = vals
    return out_k, out_v


def split_radix_sort(keys: np.ndarray, vals=None, bits: int = 32):
    """`bits` split passes, least significant bit first (stable)."""
    keys = np.array(keys, dtype=np.uint32, copy=True)
    vals = None if vals is None else np.array(vals, copy=True)
    if keys.size > 1:
        for b in range(bits):
            keys, vals = split(keys, vals, b)
    return keys, vals
