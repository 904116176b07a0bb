"""The all-core host baseline of the benchmark against the sequential oracle (CPU only)."""
import numpy as np
import pytest

import oracle
import hostbaseline as host_threads
from paper_2411_17887_amd import inputs


def make(kind, n, seed):
    if kind == "i32":
        return inputs.int32_small(n, seed)
    if kind == "i8":
        return inputs.mask_i8(n, seed)
    if kind == "f16":
        return inputs.f16_uniform01(n, seed)
    if kind == "bf16":
        return inputs.bf16_uniform_pm1(n, seed)
    return inputs.f32_normal(n, seed)


@pytest.mark.parametrize("kind", ["i32", "i8", "f16", "bf16", "f32"])
@pytest.mark.parametrize("threads", [1, 3, 8])
@pytest.mark.parametrize("exclusive", [False, True])
def test_one_row_in_chunks(kind, threads, exclusive):
    n = 100003
    x = make(kind, n, 77)
    is_int = kind in ("i32", "i8")
    out = np.full(n, -9, dtype=np.int32 if is_int else np.float32)
    host_threads.scan_into(x, kind, out, exclusive=exclusive, threads=threads)
    if is_int:
        assert oracle.compare_int(x, kind, out, exclusive=exclusive) == (0, -1)
    else:
        assert oracle.compare_float(x, kind, out, exclusive=exclusive).ok(1e-6)


@pytest.mark.parametrize("kind", ["i8", "bf16"])
@pytest.mark.parametrize("rows,cols,threads", [(37, 1001, 4), (3, 50001, 4), (4, 7, 4), (1, 5, 8), (9, 1, 2)])
def test_rows(kind, rows, cols, threads):
    x = make(kind, rows * cols, 5)
    is_int = kind == "i8"
    out = np.full(rows * cols, -9, dtype=np.int32 if is_int else np.float32)
    host_threads.scan_into(x, kind, out, rows=rows, cols=cols, threads=threads)
    if is_int:
        assert oracle.compare_int(x, kind, out, rows=rows, cols=cols) == (0, -1)
    else:
        assert oracle.compare_float(x, kind, out, rows=rows, cols=cols).ok(1e-6)


def test_wraps_like_the_oracle_and_counts_cores():
    x = np.full(70000, 2**31 - 1, dtype=np.int32)
    out = np.empty(x.size, dtype=np.int32)
    host_threads.scan_into(x, "i32", out, threads=5)
    assert oracle.compare_int(x, "i32", out) == (0, -1)
    assert host_threads.available() >= 1
    host_threads.scan_into(np.empty(0, np.int8), "i8", np.empty(0, np.int32))
    with pytest.raises(TypeError):
        host_threads.scan_into(np.zeros(4, np.float64), "f32", np.zeros(4, np.float32))
