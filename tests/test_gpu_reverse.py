"""GPU parity for reverse scans (suffix sums, tcuscan_scan with TCUSCAN_REVERSE) against the CPU oracle.

Same bars as the forward suite: integers bit-exact, integer-valued floats bit-exact, random floats by the E1 metric
(here the running L1 norm runs from the end of the row) <= 1e-3 for f16 / bf16 and <= 1e-5 for f32 inputs."""
import numpy as np
import pytest

import oracle
from paper_2411_17887_amd import inputs, tcuscan
from gpu_util import run_scan

pytestmark = pytest.mark.gpu

TOL = {"f16": 1e-3, "bf16": 1e-3, "f32": 1e-5}
INT_GEN = {"i32": inputs.int32_full, "i8": inputs.int8_full}
TRI_GEN = {"f32": inputs.tri_f32, "f16": inputs.tri_f16, "bf16": inputs.tri_bf16_bits}
RND_GEN = {"f32": inputs.f32_normal, "f16": inputs.f16_uniform01, "bf16": inputs.bf16_uniform_pm1}
KINDS = ["i32", "f16", "i8", "f32", "bf16"]


@pytest.fixture
def tile_policy():
    yield tcuscan.set_tile_policy
    tcuscan.set_tile_policy(tcuscan.TILE_AUTO)


def check(x, kind, got, exclusive, rows, cols, exact_float=False):
    if kind in INT_GEN:
        nb, fb = oracle.compare_int_reverse(x, kind, got, exclusive=exclusive, rows=rows, cols=cols)
        assert nb == 0, f"{kind}: {nb} mismatches, first (flipped index) at {fb}"
    elif exact_float:
        nb, fb = oracle.compare_float_exact_reverse(x, kind, got, exclusive=exclusive, rows=rows, cols=cols)
        assert nb == 0, f"{kind}: {nb} mismatches, first (flipped index) at {fb}"
    else:
        rep = oracle.compare_float_reverse(x, kind, got, exclusive=exclusive, rows=rows, cols=cols)
        assert rep.ok(TOL[kind]), f"{kind}: {rep}"


def run_and_check(kind, rows, cols, excl, seed, random_floats=True):
    call = "reverse_exclusive" if excl else "reverse"
    n = rows * cols
    if kind in INT_GEN:
        x = INT_GEN[kind](n, seed)
        check(x, kind, run_scan(x, kind, call, rows=rows, cols=cols), excl, rows, cols)
    else:
        x = TRI_GEN[kind](n, seed + 1)
        check(x, kind, run_scan(x, kind, call, rows=rows, cols=cols), excl, rows, cols, exact_float=True)
        if random_floats:
            x = RND_GEN[kind](n, seed + 2)
            check(x, kind, run_scan(x, kind, call, rows=rows, cols=cols), excl, rows, cols)


@pytest.mark.parametrize("excl", [False, True])
@pytest.mark.parametrize("kind", KINDS)
def test_edge_sizes(kind, excl):
    tile = tcuscan.tile_elems(kind)
    for n in [1, 2, 15, 16, 17, 63, 64, 65, 255, 256, 257, 1023, 1024, 1025, 4095, 4097, tile - 1, tile, tile + 1,
              2 * tile + 3, 65 * tile + 11, (1 << 20) + 7]:
        print("n =", n, flush=True)
        run_and_check(kind, 1, n, excl, 500 + n)


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("rows,cols", [(7, 333), (3, 8192), (5, 8193), (64, 20000), (33, 16385), (1000, 16), (2, 70001),
                                       (4096, 256), (513, 2048), (77, 2047), (100, 300), (50, 2815), (31, 2600), (64, 512), (30, 1536), (19, 2560), (17, 2561)])
def test_batched_shapes_including_short_rows_and_unaligned_rows(kind, rows, cols):
    run_and_check(kind, rows, cols, False, 900 + rows + cols, random_floats=False)
    run_and_check(kind, rows, cols, True, 901 + rows + cols)


@pytest.mark.parametrize("policy", [1, 2, 3])
@pytest.mark.parametrize("kind", KINDS)
def test_every_tile_size(kind, policy, tile_policy):
    tile_policy(policy)
    big = tcuscan.huge_tile_elems(kind)
    for rows, cols in [(1, 5 * big + 77), (3, 2 * big + 1), (2, big)]:
        run_and_check(kind, rows, cols, False, 40 + policy, random_floats=False)
        run_and_check(kind, rows, cols, True, 41 + policy)


def test_full_size_configurations_in_reverse():
    x = inputs.make_config("C3")
    check(x, "i8", run_scan(x, "i8", "reverse_exclusive", rows=1, cols=x.size), True, 1, x.size)
    x = inputs.make_config("C5")
    r, c = inputs.CONFIGS["C5"]["rows"], inputs.CONFIGS["C5"]["cols"]
    check(x, "bf16", run_scan(x, "bf16", "reverse", rows=r, cols=c), False, r, c)
    x = inputs.f32_normal(10_000_019, 77)
    check(x, "f32", run_scan(x, "f32", "reverse", rows=1, cols=x.size), False, 1, x.size)


def test_flags_zero_is_the_plain_inclusive_scan_and_unknown_flags_are_refused():
    import torch
    x = inputs.int32_full(50_000, 3)
    got = run_scan(x, "i32", "scan_flags0", rows=5, cols=10_000)
    assert oracle.compare_int(x, "i32", got, rows=5, cols=10_000) == (0, -1)
    t = torch.zeros(64, dtype=torch.int32, device="cuda")
    with pytest.raises(tcuscan.TcuscanError) as e:
        tcuscan.scan(t, t, 1, 64, "i32", flags=4)
    assert e.value.code == tcuscan.ERR_INVALID_ARG


def test_reverse_in_place_and_unaligned_pointers():
    x = inputs.int32_full(3 * 8192 + 5, 11)
    got = run_scan(x, "i32", "reverse", rows=1, cols=x.size, inplace=True)
    assert oracle.compare_int_reverse(x, "i32", got) == (0, -1)
    for kind in KINDS:
        gen = INT_GEN.get(kind) or TRI_GEN[kind]
        x = gen(40_003, 12)
        got = run_scan(x, kind, "reverse", rows=1, cols=x.size, in_offset=1, out_offset=3)
        check(x, kind, got, False, 1, x.size, exact_float=True)
