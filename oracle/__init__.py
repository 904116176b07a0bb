"""CPU oracle for prefix sums -- TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes front end over ``scan_oracle.c`` (the plain sequential
definition of the inclusive / exclusive / row-wise prefix sum; paper Section 1
notation paragraph and Section 2) plus ``matmulscan_model`` (the paper's
Algorithm 1 / Algorithm 2 / Section 2.2 replayed step by step on the CPU).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares no code with the HIP path and
never imports it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "scan_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

# input kinds, the oracle's own numbering (see scan_oracle.c)
K_I32, K_F16, K_I8, K_F32, K_BF16 = 0, 1, 2, 3, 4
KIND_NAMES = {"i32": K_I32, "f16": K_F16, "i8": K_I8, "f32": K_F32, "bf16": K_BF16}
_INT_KINDS = (K_I32, K_I8)
_IN_DTYPE = {K_I32: np.int32, K_F16: np.uint16, K_I8: np.int8, K_F32: np.float32, K_BF16: np.uint16}


def build(force: bool = False) -> str:
    """Compile scan_oracle.c with gcc (strict IEEE: no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fno-fast-math", "-ffp-contract=off", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _FCmp(ctypes.Structure):
    _fields_ = [("e1", ctypes.c_double), ("max_abs_err", ctypes.c_double), ("max_abs_ref", ctypes.c_double),
                ("worst_index", ctypes.c_uint64), ("zero_norm_bad", ctypes.c_uint64), ("nonfinite", ctypes.c_uint64)]


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        vp, sz, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        L.oracle_scan_int.argtypes = [vp, ci, vp, sz, sz, ci]
        L.oracle_scan_int64.argtypes = [vp, ci, vp, sz, sz, ci]
        L.oracle_scan_float.argtypes = [vp, ci, vp, vp, sz, sz, ci]
        L.oracle_scan_to_f32.argtypes = [vp, ci, vp, sz, sz, ci]
        L.oracle_compare_float.argtypes = [vp, ci, vp, sz, sz, ci, ctypes.POINTER(_FCmp)]
        L.oracle_compare_int.argtypes = [vp, ci, vp, sz, sz, ci, ctypes.POINTER(ctypes.c_uint64),
                                         ctypes.POINTER(ctypes.c_int64)]
        L.oracle_compare_float_exact.argtypes = L.oracle_compare_int.argtypes
        L.oracle_half_to_double.argtypes = [ctypes.c_uint16]
        L.oracle_half_to_double.restype = ctypes.c_double
        L.oracle_bf16_to_double.argtypes = [ctypes.c_uint16]
        L.oracle_bf16_to_double.restype = ctypes.c_double
        _lib = L
    return _lib


def _kind(kind) -> int:
    return KIND_NAMES[kind] if isinstance(kind, str) else int(kind)


def _prep(x: np.ndarray, kind: int, rows, cols):
    """Check the storage type (f16 / bf16 travel as uint16 bit patterns) and the shape."""
    x = np.ascontiguousarray(x)
    want = _IN_DTYPE[kind]
    if kind == K_F16 and x.dtype == np.float16:
        x = x.view(np.uint16)
    if x.dtype != want:
        raise TypeError(f"kind {kind} wants storage {want}, got {x.dtype}")
    if rows is None:
        if x.ndim == 2:
            rows, cols = x.shape
        else:
            rows, cols = 1, x.size
    if rows * cols != x.size:
        raise ValueError("rows*cols != size")
    return x, int(rows), int(cols)


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def scan(x: np.ndarray, kind, exclusive: bool = False, rows=None, cols=None, with_l1: bool = False):
    """Sequential prefix sum.  Integer kinds -> int32 (sum mod 2^32); float kinds -> float64.

    With ``with_l1`` (floats) also returns the running L1 norm S_i used by the E1 metric."""
    kind = _kind(kind)
    x, rows, cols = _prep(x, kind, rows, cols)
    if kind in _INT_KINDS:
        y = np.empty(x.size, np.int32)
        rc = lib().oracle_scan_int(_ptr(x), kind, _ptr(y), rows, cols, int(exclusive))
        assert rc == 0
        return y.reshape(x.shape)
    y = np.empty(x.size, np.float64)
    l1 = np.empty(x.size, np.float64) if with_l1 else None
    rc = lib().oracle_scan_float(_ptr(x), kind, _ptr(y), _ptr(l1) if with_l1 else None, rows, cols, int(exclusive))
    assert rc == 0
    return (y.reshape(x.shape), l1.reshape(x.shape)) if with_l1 else y.reshape(x.shape)


def scan_int64(x: np.ndarray, kind, exclusive: bool = False, rows=None, cols=None) -> np.ndarray:
    """Integer prefix sums kept in 64 bits (to show that a configuration never wraps)."""
    kind = _kind(kind)
    x, rows, cols = _prep(x, kind, rows, cols)
    y = np.empty(x.size, np.int64)
    rc = lib().oracle_scan_int64(_ptr(x), kind, _ptr(y), rows, cols, int(exclusive))
    assert rc == 0
    return y.reshape(x.shape)


def scan_to_f32(x: np.ndarray, kind, out: np.ndarray, exclusive: bool = False, rows=None, cols=None) -> None:
    """The float oracle writing fp32 into a caller-provided buffer (host-baseline timing)."""
    kind = _kind(kind)
    x, rows, cols = _prep(x, kind, rows, cols)
    assert out.dtype == np.float32 and out.size == x.size and out.flags.c_contiguous
    rc = lib().oracle_scan_to_f32(_ptr(x), kind, _ptr(out), rows, cols, int(exclusive))
    assert rc == 0


def scan_int_into(x: np.ndarray, kind, out: np.ndarray, exclusive: bool = False, rows=None, cols=None) -> None:
    """The integer oracle writing int32 into a caller-provided buffer (host-baseline timing)."""
    kind = _kind(kind)
    x, rows, cols = _prep(x, kind, rows, cols)
    assert out.dtype == np.int32 and out.size == x.size and out.flags.c_contiguous
    rc = lib().oracle_scan_int(_ptr(x), kind, _ptr(out), rows, cols, int(exclusive))
    assert rc == 0


@dataclass
class FloatReport:
    e1: float
    max_abs_err: float
    max_abs_ref: float
    worst_index: int
    zero_norm_bad: int
    nonfinite: int

    @property
    def einf(self) -> float:
        return self.max_abs_err / self.max_abs_ref if self.max_abs_ref > 0 else 0.0

    def ok(self, tol: float) -> bool:
        return self.nonfinite == 0 and self.zero_norm_bad == 0 and self.e1 <= tol


def compare_float(x: np.ndarray, kind, got: np.ndarray, exclusive: bool = False, rows=None, cols=None) -> FloatReport:
    """Stream the oracle over x and measure a candidate fp32 output against it (E1 metric)."""
    kind = _kind(kind)
    x, rows, cols = _prep(x, kind, rows, cols)
    got = np.ascontiguousarray(got)
    assert got.dtype == np.float32 and got.size == x.size
    r = _FCmp()
    rc = lib().oracle_compare_float(_ptr(x), kind, _ptr(got), rows, cols, int(exclusive), ctypes.byref(r))
    assert rc == 0
    return FloatReport(r.e1, r.max_abs_err, r.max_abs_ref, int(r.worst_index), int(r.zero_norm_bad), int(r.nonfinite))


def compare_int(x: np.ndarray, kind, got: np.ndarray, exclusive: bool = False, rows=None, cols=None):
    """(number of mismatching int32 outputs, first mismatching flat index or -1)."""
    kind = _kind(kind)
    x, rows, cols = _prep(x, kind, rows, cols)
    got = np.ascontiguousarray(got)
    assert got.dtype == np.int32 and got.size == x.size
    nb, fb = ctypes.c_uint64(), ctypes.c_int64()
    rc = lib().oracle_compare_int(_ptr(x), kind, _ptr(got), rows, cols, int(exclusive), ctypes.byref(nb), ctypes.byref(fb))
    assert rc == 0
    return int(nb.value), int(fb.value)


def compare_float_exact(x: np.ndarray, kind, got: np.ndarray, exclusive: bool = False, rows=None, cols=None):
    """Bit-exact check for integer-valued float inputs: (mismatches, first index or -1)."""
    kind = _kind(kind)
    x, rows, cols = _prep(x, kind, rows, cols)
    got = np.ascontiguousarray(got)
    assert got.dtype == np.float32 and got.size == x.size
    nb, fb = ctypes.c_uint64(), ctypes.c_int64()
    rc = lib().oracle_compare_float_exact(_ptr(x), kind, _ptr(got), rows, cols, int(exclusive), ctypes.byref(nb),
                                          ctypes.byref(fb))
    assert rc == 0
    return int(nb.value), int(fb.value)


# ---- reverse scans (suffix sums): by definition the scan of the reversed row, reversed.  Nothing new is
# computed here: rows are flipped on the way in and on the way out of the functions above.

def _flip_rows(a: np.ndarray, rows: int, cols: int) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a).reshape(rows, cols)[:, ::-1])


def scan_reverse(x: np.ndarray, kind, exclusive: bool = False, rows=None, cols=None, with_l1: bool = False):
    """Suffix sums: y[i] = x[i] + ... + x[cols-1] (inclusive) or x[i+1] + ... + x[cols-1] (exclusive), per row."""
    k = _kind(kind)
    xx, rows, cols = _prep(x, k, rows, cols)
    r = scan(_flip_rows(xx, rows, cols), k, exclusive, rows, cols, with_l1)
    if with_l1:
        return _flip_rows(r[0], rows, cols).reshape(xx.shape), _flip_rows(r[1], rows, cols).reshape(xx.shape)
    return _flip_rows(r, rows, cols).reshape(xx.shape)


def compare_float_reverse(x, kind, got, exclusive: bool = False, rows=None, cols=None) -> FloatReport:
    k = _kind(kind)
    xx, rows, cols = _prep(x, k, rows, cols)
    return compare_float(_flip_rows(xx, rows, cols), k, _flip_rows(got, rows, cols), exclusive, rows, cols)


def compare_int_reverse(x, kind, got, exclusive: bool = False, rows=None, cols=None):
    """(mismatches, first mismatching index in the flipped order or -1)."""
    k = _kind(kind)
    xx, rows, cols = _prep(x, k, rows, cols)
    return compare_int(_flip_rows(xx, rows, cols), k, _flip_rows(got, rows, cols), exclusive, rows, cols)


def compare_float_exact_reverse(x, kind, got, exclusive: bool = False, rows=None, cols=None):
    k = _kind(kind)
    xx, rows, cols = _prep(x, k, rows, cols)
    return compare_float_exact(_flip_rows(xx, rows, cols), k, _flip_rows(got, rows, cols), exclusive, rows, cols)


# ---- segmented scans: rows of different lengths stored back to back.  By definition every row is scanned on its
# own, so the functions below only slice the flat arrays at the offsets and hand each row to the functions above.

def _rows_of(offsets):
    off = np.asarray(offsets, dtype=np.int64)
    assert off.ndim == 1 and off.size >= 1 and np.all(np.diff(off) >= 0) and off[0] >= 0
    return [(int(off[r]), int(off[r + 1])) for r in range(off.size - 1)]


def scan_segments(x: np.ndarray, kind, offsets, exclusive: bool = False, reverse: bool = False) -> np.ndarray:
    """Flat output (int32 or float64) with every row [offsets[r], offsets[r+1]) scanned separately; elements of x
    outside all rows are returned as 0."""
    k = _kind(kind)
    x = np.ascontiguousarray(x).reshape(-1)
    out = np.zeros(x.size, np.int32 if k in _INT_KINDS else np.float64)
    f = scan_reverse if reverse else scan
    for a, b in _rows_of(offsets):
        if b > a:
            out[a:b] = f(x[a:b], k, exclusive)
    return out


def compare_segments(x: np.ndarray, kind, offsets, got: np.ndarray, exclusive: bool = False, reverse: bool = False,
                     exact_float: bool = False):
    """Integers / exact floats: (mismatches, first bad row or -1).  Floats: the worst FloatReport over the rows
    (largest E1; non-finite and zero-norm counts summed)."""
    k = _kind(kind)
    x = np.ascontiguousarray(x).reshape(-1)
    got = np.ascontiguousarray(got).reshape(-1)
    ints = k in _INT_KINDS
    if ints or exact_float:
        cmp = (compare_int_reverse if reverse else compare_int) if ints else \
              (compare_float_exact_reverse if reverse else compare_float_exact)
        bad, first = 0, -1
        for r, (a, b) in enumerate(_rows_of(offsets)):
            if b > a:
                nb, _ = cmp(x[a:b], k, got[a:b], exclusive)
                if nb and first < 0:
                    first = r
                bad += nb
        return bad, first
    cmp = compare_float_reverse if reverse else compare_float
    worst = FloatReport(0.0, 0.0, 0.0, -1, 0, 0)
    for a, b in _rows_of(offsets):
        if b > a:
            rep = cmp(x[a:b], k, got[a:b], exclusive)
            zero_bad, nonfin = worst.zero_norm_bad + rep.zero_norm_bad, worst.nonfinite + rep.nonfinite
            if rep.e1 >= worst.e1:
                worst = FloatReport(rep.e1, rep.max_abs_err, rep.max_abs_ref, a + rep.worst_index, 0, 0)
            worst.zero_norm_bad, worst.nonfinite = zero_bad, nonfin
    return worst


def half_to_double(bits: int) -> float:
    return float(lib().oracle_half_to_double(int(bits)))


def bf16_to_double(bits: int) -> float:
    return float(lib().oracle_bf16_to_double(int(bits)))
