"""Pins for oracle/apps.py (compaction and split radix sort built on the sequential scan)."""
import numpy as np
import pytest

from oracle import apps
from paper_2411_17887_amd import inputs


def keys_u32(n, seed):
    return inputs.int32_full(n, seed).view(np.uint32)


@pytest.mark.parametrize("n", [1, 2, 17, 1000, 40000])
def test_compact_equals_boolean_filter(n):
    v = keys_u32(n, n)
    m = inputs.mask_i8(n, n + 1)
    out, pos = apps.compact(v, m)
    assert np.array_equal(out, v[m != 0])
    assert np.array_equal(pos, np.concatenate([[0], np.cumsum(m.astype(np.int64))[:-1]]))
    for mm in (np.zeros(n, np.int8), np.ones(n, np.int8)):
        assert np.array_equal(apps.compact(v, mm)[0], v[mm != 0])


def test_split_is_a_stable_partition_by_one_bit():
    k = keys_u32(5000, 3)
    tagged = np.arange(k.size, dtype=np.uint32)
    out_k, out_v = apps.split(k, tagged, 5)
    bit = (out_k >> np.uint32(5)) & np.uint32(1)
    z = int((bit == 0).sum())
    assert np.all(bit[:z] == 0) and np.all(bit[z:] == 1)
    assert np.all(np.diff(out_v[:z].astype(np.int64)) > 0) and np.all(np.diff(out_v[z:].astype(np.int64)) > 0)   # old order kept
    assert np.array_equal(k[out_v], out_k)                                                                      # a permutation


def brute_force_sorted(keys):
    rest, out = list(int(k) for k in keys), []
    while rest:                               # selection sort: the definition of "sorted", O(n^2)
        m = min(rest)
        out.append(m)
        rest.remove(m)
    return out


@pytest.mark.parametrize("n", [0, 1, 2, 3, 16, 33, 64])
def test_sort_bruteforce_tiny(n):
    k = keys_u32(n, 7 + n)
    assert apps.split_radix_sort(k)[0].tolist() == brute_force_sorted(k)


@pytest.mark.parametrize("n", [1000, 30011])
def test_sort_equals_library_stable_sort(n):
    k = keys_u32(n, n)
    s, _ = apps.split_radix_sort(k)
    assert np.array_equal(s, np.sort(k))
    small = k & np.uint32(0xFF)                         # many duplicates: stability is observable through the payload
    payload = np.arange(n, dtype=np.uint32)
    s2, p2 = apps.split_radix_sort(small, payload, bits=8)
    order = np.argsort(small, kind="stable")
    assert np.array_equal(s2, small[order]) and np.array_equal(p2, payload[order])


def test_sort_by_low_bits_only_orders_those_bits():
    k = keys_u32(4000, 1)
    s, _ = apps.split_radix_sort(k, bits=12)
    low = s & np.uint32(0xFFF)
    assert np.all(np.diff(low.astype(np.int64)) >= 0)
    assert np.array_equal(np.sort(s), np.sort(k))
    order = np.argsort(k & np.uint32(0xFFF), kind="stable")
    assert np.array_equal(s, k[order])
