"""
ctypes front end of ``host_threads.c``: the all-core host baseline that the benchmark times next to the GPU path.

Measurement infrastructure only, and not the oracle: the oracle is the sequential definition in
``oracle/scan_oracle.c``; this is the usual chunked multi-thread scan, kept in a folder of its own because it has a
blocking (chunks per thread) that the yardstick must not have.  It is checked against the oracle in
``tests/test_host_threads.py`` and again in every benchmark run.  The product path never imports it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "host_threads.c")
_LIB = os.path.join(_HERE, "libhostthreads.so")
_KINDS = {"i32": 0, "f16": 1, "i8": 2, "f32": 3, "bf16": 4}
_IN_DTYPE = {"i32": np.int32, "f16": np.uint16, "i8": np.int8, "f32": np.float32, "bf16": np.uint16}


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.run(["gcc", "-O2", "-std=gnu11", "-fno-fast-math", "-ffp-contract=off", "-fPIC", "-shared", "-pthread",
                        "-Wall", "-Wextra", "-o", _LIB, _SRC], check=True)
    return _LIB


_lib = None


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.host_threads_scan.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_size_t,
                                        ctypes.c_int, ctypes.c_int]
        L.host_threads_available.restype = ctypes.c_int
        _lib = L
    return _lib


def available() -> int:
    """Cores this process may run on (its affinity mask)."""
    return int(_load().host_threads_available())


def scan_into(x: np.ndarray, kind: str, out: np.ndarray, exclusive: bool = False, rows: int | None = None,
              cols: int | None = None, threads: int = 0) -> None:
    """out (int32 for integer kinds, float32 otherwise) <- scan of x, rows x cols, on `threads` threads (0: all cores)."""
    x = np.ascontiguousarray(x)
    if kind == "f16" and x.dtype == np.float16:
        x = x.view(np.uint16)                       # the bit patterns
    if x.dtype != _IN_DTYPE[kind]:
        raise TypeError(f"{kind} input must be {_IN_DTYPE[kind]}, got {x.dtype}")
    if rows is None:
        rows, cols = (1, x.size) if x.size else (0, 0)
    want = np.int32 if kind in ("i32", "i8") else np.float32
    if out.dtype != want or out.size != rows * cols or not out.flags.c_contiguous or x.size != rows * cols:
        raise ValueError("output must be a contiguous array of rows * cols elements of the output type")
    rc = _load().host_threads_scan(x.ctypes.data_as(ctypes.c_void_p), _KINDS[kind], out.ctypes.data_as(ctypes.c_void_p),
                                   rows, cols, int(exclusive), int(threads))
    if rc != 0:
        raise RuntimeError(f"host_threads_scan failed with {rc}")
