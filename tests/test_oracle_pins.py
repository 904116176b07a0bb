"""Pins for the CPU oracle (oracle/scan_oracle.c).

The oracle is checked against things that are NOT itself: closed forms, exact rational
arithmetic, the O(n^2) definition, a library cumulative sum, math.fsum, the values the paper
prints in Figure 1(a), and planted mistakes that the comparators must catch.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2411_17887_amd import inputs

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_rows(name):
    rows = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append([int(t) for t in line.split()])
    return rows


# ------------------------------------------------------------------ closed forms

@pytest.mark.parametrize("kind,dt", [("i32", np.int32), ("i8", np.int8)])
@pytest.mark.parametrize("n", [1, 2, 15, 16, 17, 255, 4096, 100003])
def test_all_ones_int(kind, dt, n):
    y = oracle.scan(np.ones(n, dt), kind)
    assert np.array_equal(y, np.arange(1, n + 1, dtype=np.int64).astype(np.int32))
    ye = oracle.scan(np.ones(n, dt), kind, exclusive=True)
    assert np.array_equal(ye, np.arange(0, n, dtype=np.int32))


@pytest.mark.parametrize("n", [1, 7, 16, 1000, 65536])
def test_arange_gives_triangular_numbers(n):
    x = np.arange(1, n + 1, dtype=np.int32)
    i = np.arange(1, n + 1, dtype=np.int64)
    assert np.array_equal(oracle.scan_int64(x, "i32"), i * (i + 1) // 2)
    # the int32 result is the same thing modulo 2^32
    assert np.array_equal(oracle.scan(x, "i32"), ((i * (i + 1) // 2) & 0xFFFFFFFF).astype(np.uint32).view(np.int32))


@pytest.mark.parametrize("kind", ["i32", "i8", "f32", "f16", "bf16"])
def test_alternating_signs(kind):
    n = 1001
    v = np.where(np.arange(n) % 2 == 0, 1, -1)
    x = {"i32": v.astype(np.int32), "i8": v.astype(np.int8), "f32": v.astype(np.float32),
         "f16": v.astype(np.float16), "bf16": inputs.f32_to_bf16_bits(v.astype(np.float32))}[kind]
    y = oracle.scan(x, kind)
    assert np.array_equal(np.asarray(y, dtype=np.int64), (np.arange(n) % 2 == 0).astype(np.int64))


def test_figure_1a_final_row():
    """Figure 1(a): input 1..16 -> last printed row."""
    rows = read_rows("fig1a_s4_states.txt")
    x = np.array(rows[0], dtype=np.int32)
    assert np.array_equal(oracle.scan(x, "i32"), np.array(rows[3], dtype=np.int32))
    assert np.array_equal(oracle.scan(x.astype(np.float32), "f32"), np.array(rows[3], dtype=np.float64))


# ------------------------------------------------------- brute force / exact rationals

def brute_inclusive(vals):
    return [sum(vals[: i + 1]) for i in range(len(vals))]


@pytest.mark.parametrize("n", [1, 2, 3, 16, 33, 64])
@pytest.mark.parametrize("kind,gen", [("i32", inputs.int32_small), ("i32", inputs.int32_full), ("i8", inputs.int8_full)])
def test_bruteforce_int(n, kind, gen):
    x = gen(n, 7 + n)
    want = np.array([((v + 2 ** 31) % 2 ** 32) - 2 ** 31 for v in brute_inclusive([int(v) for v in x])], dtype=np.int64)
    assert np.array_equal(oracle.scan(x, kind).astype(np.int64), want)
    want_ex = np.concatenate([[0], want[:-1]])
    assert np.array_equal(oracle.scan(x, kind, exclusive=True).astype(np.int64), want_ex)


def to_fraction(x, kind):
    if kind == "f16":
        return [Fraction(float(v)) for v in x.astype(np.float64)]
    if kind == "bf16":
        f = (x.astype(np.uint32) << 16).view(np.float32)
        return [Fraction(float(v)) for v in f]
    return [Fraction(float(v)) for v in x]


@pytest.mark.parametrize("n", [1, 5, 16, 64, 300])
@pytest.mark.parametrize("kind,gen", [("f32", inputs.f32_normal), ("f16", inputs.f16_uniform01),
                                      ("bf16", inputs.bf16_uniform_pm1)])
def test_exact_rational_float(n, kind, gen):
    """The fp64 compensated oracle agrees with exact rational prefix sums to 2 ulp of the running L1 norm."""
    x = gen(n, 99 + n)
    fr = to_fraction(x, kind)
    y, l1 = oracle.scan(x, kind, with_l1=True)
    acc, nrm = Fraction(0), Fraction(0)
    for i, v in enumerate(fr):
        acc += v
        nrm += abs(v)
        assert abs(Fraction(float(y[i])) - acc) <= nrm * Fraction(1, 2 ** 51)
        assert abs(Fraction(float(l1[i])) - nrm) <= nrm * Fraction(1, 2 ** 51)
    ye, l1e = oracle.scan(x, kind, exclusive=True, with_l1=True)
    assert ye[0] == 0.0 and l1e[0] == 0.0
    assert np.array_equal(ye[1:], y[:-1]) and np.array_equal(l1e[1:], l1[:-1])


def test_f16_uniform01_oracle_is_exact():
    """Every half in [0,1) is a multiple of 2^-24 and every partial sum stays below 2^24, so fp64 never rounds."""
    n = 1 << 14
    x = inputs.f16_uniform01(n, 5)
    y = oracle.scan(x, "f16")
    ints = (x.astype(np.float64) * 2.0 ** 24)
    assert np.all(ints == np.round(ints))
    want = np.cumsum(ints.astype(np.int64))             # exact integer arithmetic in units of 2^-24
    assert np.array_equal(y * 2.0 ** 24, want.astype(np.float64))


# --------------------------------------------------------- library cross-checks

@pytest.mark.parametrize("n", [1000, 65537])
def test_against_numpy_cumsum(n):
    xi = inputs.int32_small(n, 3)
    assert np.array_equal(oracle.scan_int64(xi, "i32"), np.cumsum(xi.astype(np.int64)))
    x8 = inputs.mask_i8(n, 4)
    assert np.array_equal(oracle.scan(x8, "i8").astype(np.int64), np.cumsum(x8.astype(np.int64)))
    xf = inputs.f32_normal(n, 5)
    y = oracle.scan(xf, "f32")
    ref = np.cumsum(xf.astype(np.float64))
    l1 = np.cumsum(np.abs(xf.astype(np.float64)))
    assert np.max(np.abs(y - ref) / l1) < 1e-13          # cumsum in fp64 is itself only ~n*2^-53 accurate


@pytest.mark.parametrize("kind,gen", [("f32", inputs.f32_normal), ("f16", inputs.f16_uniform01)])
def test_last_element_is_the_exactly_rounded_total(kind, gen):
    n = 200001
    x = gen(n, 11)
    total = math.fsum(float(v) for v in x.astype(np.float64))
    y = oracle.scan(x, kind)
    assert abs(y[-1] - total) <= 2 * math.ulp(max(abs(total), 1.0))


def test_int32_wraps_modulo_2_32():
    x = np.full(5, 2 ** 31 - 1, dtype=np.int32)
    y = oracle.scan(x, "i32")
    want = [((k * (2 ** 31 - 1) + 2 ** 31) % 2 ** 32) - 2 ** 31 for k in range(1, 6)]
    assert y.tolist() == want
    big = inputs.int32_full(100000, 17)
    u = np.cumsum(big.astype(np.int64)) & 0xFFFFFFFF
    assert np.array_equal(oracle.scan(big, "i32").view(np.uint32).astype(np.int64), u)


# ------------------------------------------------------------------ invariants

@pytest.mark.parametrize("kind,gen", [("i32", inputs.int32_small), ("i8", inputs.mask_i8), ("f32", inputs.f32_normal),
                                      ("f16", inputs.f16_uniform01), ("bf16", inputs.bf16_uniform_pm1)])
def test_exclusive_is_inclusive_shifted(kind, gen):
    x = gen(5000, 23)
    yi, ye = oracle.scan(x, kind), oracle.scan(x, kind, exclusive=True)
    assert ye[0] == 0
    assert np.array_equal(ye[1:], yi[:-1])


def test_int_differences_return_the_input():
    x = inputs.int32_small(4096, inputs.BASE_SEED)
    y = oracle.scan_int64(x, "i32")
    assert y[0] == x[0] and np.array_equal(np.diff(y), x[1:].astype(np.int64))
    e = oracle.scan_int64(x, "i32", exclusive=True)
    assert np.array_equal(y - e, x.astype(np.int64))


@pytest.mark.parametrize("kind,gen", [("i32", inputs.int32_small), ("bf16", inputs.bf16_uniform_pm1), ("f32", inputs.f32_normal)])
@pytest.mark.parametrize("exclusive", [False, True])
def test_batched_rows_are_independent(kind, gen, exclusive):
    rows, cols = 7, 333
    x = gen(rows * cols, 31)
    yb = oracle.scan(x, kind, exclusive=exclusive, rows=rows, cols=cols).reshape(rows, cols)
    for r in range(rows):
        assert np.array_equal(yb[r], oracle.scan(x[r * cols:(r + 1) * cols], kind, exclusive=exclusive))


def test_zero_extension_does_not_change_kept_outputs():
    """BatchMatMul zero-pads and drops the padding: the first n outputs of a zero-extended input are unchanged."""
    x = inputs.f32_normal(1000, 41)
    xp = np.concatenate([x, np.zeros(4096 - 1000, np.float32)])
    assert np.array_equal(oracle.scan(xp, "f32")[:1000], oracle.scan(x, "f32"))
    assert np.all(oracle.scan(xp, "f32")[1000:] == oracle.scan(x, "f32")[-1])


def test_configs_never_overflow_int32():
    x1 = inputs.make_config("C1")
    assert np.abs(oracle.scan_int64(x1, "i32")).max() < 2 ** 31
    assert x1.min() >= -128 and x1.max() <= 127
    x3 = inputs.mask_i8(1 << 20, inputs.CONFIGS["C3"]["seed"])
    assert set(np.unique(x3).tolist()) == {0, 1}
    assert abs(float(x3.mean()) - 0.5) < 2e-3           # P(1) = 1/2


# ------------------------------------------------------------- number formats

def test_half_conversion_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    for b in range(0, 65536, 1):
        r = ref[b]
        if np.isnan(r):
            continue
        v = oracle.half_to_double(b)
        assert v == r and math.copysign(1.0, v) == math.copysign(1.0, r)


def test_bf16_conversion():
    bits = np.arange(65536, dtype=np.uint16)
    with np.errstate(invalid="ignore"):
        ref = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    for b in range(0, 65536, 7):
        if np.isnan(ref[b]):
            continue
        assert oracle.bf16_to_double(b) == ref[b]


# -------------------------------------------- comparators catch planted mistakes

def test_float_comparator_accepts_rounded_oracle_and_catches_errors():
    n = 50000
    x = inputs.f32_normal(n, 77)
    ref = oracle.scan(x, "f32")
    good = ref.astype(np.float32)
    rep = oracle.compare_float(x, "f32", good)
    assert rep.ok(1e-6) and rep.e1 < 2 ** -23
    # dropped term: one input skipped
    bad = oracle.scan(np.concatenate([x[:100], [0], x[101:]]).astype(np.float32), "f32").astype(np.float32)
    assert not oracle.compare_float(x, "f32", bad).ok(1e-5)
    # off-by-one (exclusive handed in as inclusive)
    ex = oracle.scan(x, "f32", exclusive=True).astype(np.float32)
    assert not oracle.compare_float(x, "f32", ex).ok(1e-3)
    assert oracle.compare_float(x, "f32", ex, exclusive=True).ok(1e-6)
    # wrong sign on a segment carry
    sg = good.copy(); sg[4096:] -= 2 * good[4095]
    assert not oracle.compare_float(x, "f32", sg).ok(1e-3)
    # NaN
    nn = good.copy(); nn[7] = np.nan
    assert oracle.compare_float(x, "f32", nn).nonfinite == 1 and not oracle.compare_float(x, "f32", nn).ok(1.0)
    # exclusive output 0 must be exactly zero
    e0 = ex.copy(); e0[0] = 1e-30
    assert oracle.compare_float(x, "f32", e0, exclusive=True).zero_norm_bad == 1


def test_float_comparator_e1_equals_relative_error_for_nonnegative_data():
    n = 20000
    x = inputs.f16_uniform01(n, 3)
    ref = oracle.scan(x, "f16")
    cand = (ref * (1 + 3e-4)).astype(np.float32)
    rep = oracle.compare_float(x, "f16", cand)
    rel = np.max(np.abs(cand.astype(np.float64) - ref)[ref > 0] / ref[ref > 0])
    assert abs(rep.e1 - rel) < 1e-12 and 2e-4 < rep.e1 < 4e-4


def test_int_comparator():
    x = inputs.mask_i8(30000, 9)
    ref = oracle.scan(x, "i8", exclusive=True)
    assert oracle.compare_int(x, "i8", ref, exclusive=True) == (0, -1)
    bad = ref.copy(); bad[12345] += 1; bad[20000] -= 1
    assert oracle.compare_int(x, "i8", bad, exclusive=True) == (2, 12345)
    # a transposed pair of inputs changes exactly one output when the two values differ
    j = int(np.nonzero(x[:-1] != x[1:])[0][10])
    xs = x.copy(); xs[j], xs[j + 1] = x[j + 1], x[j]
    nb, fb = oracle.compare_int(x, "i8", oracle.scan(xs, "i8"), exclusive=False)
    assert nb == 1 and fb == j


def test_exact_float_comparator_on_integer_valued_floats():
    n = 100000
    for kind, x in [("f32", inputs.tri_f32(n, 5)), ("f16", inputs.tri_f16(n, 6)), ("bf16", inputs.tri_bf16_bits(n, 7))]:
        ref = oracle.scan(x, kind)
        assert np.all(ref == np.round(ref)) and np.abs(ref).max() < 2 ** 24
        assert oracle.compare_float_exact(x, kind, ref.astype(np.float32)) == (0, -1)
        bad = ref.astype(np.float32); bad[777] += 1
        assert oracle.compare_float_exact(x, kind, bad) == (1, 777)
