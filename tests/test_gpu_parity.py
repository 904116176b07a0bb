"""GPU parity: the HIP path (through the C-ABI) against the CPU oracle, element by element.

Bars: integers bit-exact; floats by the E1 metric (max |got - ref| / running L1 norm against the
compensated fp64 oracle) <= 1e-3 for f16 / bf16 inputs and <= 1e-5 for f32 inputs at every size
used here, including n = 100,000,007; integer-valued float inputs bit-exact at any size (every
partial sum is exactly representable in fp32, so no summation order can change a bit).
"""
import numpy as np
import pytest

import oracle
from paper_2411_17887_amd import inputs, tcuscan
from gpu_util import run_scan, to_device

pytestmark = pytest.mark.gpu

TOL = {"f16": 1e-3, "bf16": 1e-3, "f32": 1e-5}
INT_GEN = {"i32": inputs.int32_full, "i8": inputs.int8_full}
TRI_GEN = {"f32": inputs.tri_f32, "f16": inputs.tri_f16, "bf16": inputs.tri_bf16_bits}
RND_GEN = {"f32": inputs.f32_normal, "f16": inputs.f16_uniform01, "bf16": inputs.bf16_uniform_pm1}
KINDS = ["i32", "f16", "i8", "f32", "bf16"]


def check(x, kind, got, exclusive=False, rows=None, cols=None, exact_float=False, tol=None):
    if kind in INT_GEN:
        nb, fb = oracle.compare_int(x, kind, got, exclusive=exclusive, rows=rows, cols=cols)
        assert nb == 0, f"{kind}: {nb} mismatches, first at {fb}"
    elif exact_float:
        nb, fb = oracle.compare_float_exact(x, kind, got, exclusive=exclusive, rows=rows, cols=cols)
        assert nb == 0, f"{kind}: {nb} mismatches, first at {fb}"
    else:
        rep = oracle.compare_float(x, kind, got, exclusive=exclusive, rows=rows, cols=cols)
        assert rep.ok(tol or TOL[kind]), f"{kind}: {rep}"
        return rep


def edge_sizes():
    tile = tcuscan.tile_elems("f32")
    return [1, 2, 15, 16, 17, 63, 64, 65, 255, 256, 257, 511, 512, 513, 1023, 1024, 1025, 2047, 2049, 4095, 4096, 4097,
            tile - 1, tile, tile + 1, 2 * tile + 3, 65 * tile + 11, (1 << 20) + 7]


@pytest.mark.parametrize("call", ["inclusive", "exclusive"])
@pytest.mark.parametrize("kind", KINDS)
def test_edge_sizes(kind, call):
    ex = call == "exclusive"
    for n in edge_sizes():
        print("n =", n, flush=True)
        if kind in INT_GEN:
            x = INT_GEN[kind](n, 1000 + n)
            check(x, kind, run_scan(x, kind, call), exclusive=ex)
        else:
            x = TRI_GEN[kind](n, 2000 + n)
            check(x, kind, run_scan(x, kind, call), exclusive=ex, exact_float=True)
            x = RND_GEN[kind](n, 3000 + n)
            check(x, kind, run_scan(x, kind, call), exclusive=ex)


def test_empty_input_enqueues_nothing():
    import torch
    out = torch.full((4,), 5, dtype=torch.int32, device="cuda")
    tcuscan.inclusive(out, out, "i32", n=0)
    tcuscan.batched(out, out, 0, 7, "i32")
    torch.cuda.synchronize()
    assert out.tolist() == [5, 5, 5, 5]


# ----------------------------------------------------------------- the five configurations

def test_config_C1_int32_4096():
    x = inputs.make_config("C1")
    got = run_scan(x, "i32", "inclusive")
    assert np.array_equal(got, oracle.scan(x, "i32"))


def test_config_C2_f16_2p24():
    x = inputs.make_config("C2")
    rep = check(x, "f16", run_scan(x, "f16", "inclusive"), tol=1e-3)
    print("C2", rep, flush=True)


def test_config_C3_mask_exclusive_2p28():
    x = inputs.make_config("C3")
    got = run_scan(x, "i8", "exclusive")
    check(x, "i8", got, exclusive=True)
    assert got[0] == 0 and int(got[-1]) + int(x[-1]) == int(x.astype(np.int64).sum())


def test_config_C4_f32_normal_100000007():
    x = inputs.make_config("C4")
    rep = check(x, "f32", run_scan(x, "f32", "inclusive"), tol=1e-5)
    print("C4", rep, "Einf", rep.einf, flush=True)


def test_config_C5_batched_bf16_4096x65536():
    c = inputs.CONFIGS["C5"]
    x = inputs.make_config("C5")
    got = run_scan(x, "bf16", "batched", rows=c["rows"], cols=c["cols"])
    rep = check(x, "bf16", got, rows=c["rows"], cols=c["cols"], tol=1e-3)
    print("C5", rep, flush=True)


# ------------------------------------------------- structure checks at full size (bit-exact floats)

@pytest.mark.parametrize("kind", ["f32", "f16", "bf16"])
def test_integer_valued_floats_are_bit_exact_at_scale(kind):
    n = (1 << 26) + 5
    x = TRI_GEN[kind](n, 77)
    check(x, kind, run_scan(x, kind, "inclusive"), exact_float=True)
    check(x, kind, run_scan(x, kind, "exclusive"), exclusive=True, exact_float=True)


def test_int32_full_range_wraps_modulo_2_32_at_scale():
    n = (1 << 25) + 3
    x = inputs.int32_full(n, 5)
    check(x, "i32", run_scan(x, "i32", "inclusive"))
    x = np.full(100000, 2 ** 31 - 1, dtype=np.int32)
    check(x, "i32", run_scan(x, "i32", "exclusive"), exclusive=True)
    x = np.full(100000, -2 ** 31, dtype=np.int32)
    check(x, "i32", run_scan(x, "i32", "inclusive"))


def test_int8_extremes():
    for v in (-128, 127):
        x = np.full(3 * 8192 + 5, v, dtype=np.int8)
        check(x, "i8", run_scan(x, "i8", "inclusive"))
        check(x, "i8", run_scan(x, "i8", "exclusive"), exclusive=True)


def test_f16_subnormal_inputs_are_summed_not_flushed():
    n = 50000
    x = np.full(n, 1, dtype=np.uint16).view(np.float16)          # 2^-24, the smallest subnormal half
    got = run_scan(x, "f16", "inclusive")
    check(x, "f16", got, exact_float=True)


# ------------------------------------------------------------------------------- batched

@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("rows,cols", [(7, 333), (3, 8192), (5, 8193), (64, 20000), (33, 16385), (1000, 16), (2, 70001)])
def test_batched_shapes(kind, rows, cols):
    for call in ("batched", "batched_exclusive"):
        ex = call.endswith("exclusive")
        if kind in INT_GEN:
            x = INT_GEN[kind](rows * cols, rows + cols)
            check(x, kind, run_scan(x, kind, call, rows=rows, cols=cols), exclusive=ex, rows=rows, cols=cols)
        else:
            x = TRI_GEN[kind](rows * cols, rows + cols)
            check(x, kind, run_scan(x, kind, call, rows=rows, cols=cols), exclusive=ex, rows=rows, cols=cols, exact_float=True)
            x = RND_GEN[kind](rows * cols, rows * cols)
            check(x, kind, run_scan(x, kind, call, rows=rows, cols=cols), exclusive=ex, rows=rows, cols=cols)


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("rows,cols", [(4096, 256), (1000, 1024), (513, 2048), (77, 2047), (9, 1), (100, 300), (8, 2048),
                                       (4099, 64), (33, 513), (65537, 16), (50, 2815), (31, 2600), (12, 2816), (9, 2817), (64, 512), (30, 1536), (21, 2304), (19, 2560), (17, 2561)])
def test_short_rows_one_per_wavefront(kind, rows, cols):
    """Many short rows (histogram-like shapes): each wavefront scans whole rows; includes row lengths that
    leave rows unaligned, a ragged last workgroup and exclusive scans."""
    for call in ("batched", "batched_exclusive"):
        ex = call.endswith("exclusive")
        if kind in INT_GEN:
            x = INT_GEN[kind](rows * cols, rows + 3 * cols)
            check(x, kind, run_scan(x, kind, call, rows=rows, cols=cols), exclusive=ex, rows=rows, cols=cols)
        else:
            x = TRI_GEN[kind](rows * cols, rows + 3 * cols)
            check(x, kind, run_scan(x, kind, call, rows=rows, cols=cols), exclusive=ex, rows=rows, cols=cols, exact_float=True)
            x = RND_GEN[kind](rows * cols, rows * cols + 1)
            check(x, kind, run_scan(x, kind, call, rows=rows, cols=cols), exclusive=ex, rows=rows, cols=cols)


@pytest.mark.parametrize("kind", KINDS)
def test_batched_rows_that_are_exact_multiples_of_the_tiles(kind):
    """Row lengths that are whole numbers of small / large tiles, on either side of the policy's switch points."""
    for rows, cols in [(3, 16384), (64, 16384), (40, 32768), (17, 65536), (5, (1 << 18)), (3, (1 << 18) + 8192), (2, 1 << 20)]:
        x = (INT_GEN.get(kind) or TRI_GEN[kind])(rows * cols, rows)
        check(x, kind, run_scan(x, kind, "batched", rows=rows, cols=cols), rows=rows, cols=cols, exact_float=kind not in INT_GEN)


def test_batched_row_equals_unbatched_scan_of_that_row():
    rows, cols = 6, 30011
    x = inputs.int32_small(rows * cols, 9)
    got = run_scan(x, "i32", "batched", rows=rows, cols=cols).reshape(rows, cols)
    for r in range(rows):
        assert np.array_equal(got[r], run_scan(x[r * cols:(r + 1) * cols].copy(), "i32", "inclusive"))


# ------------------------------------------------------------------ pointers and buffers

@pytest.mark.parametrize("kind", KINDS)
def test_unaligned_pointers(kind):
    n = 3 * 8192 + 77
    for in_off, out_off in [(1, 0), (0, 1), (3, 2), (5, 3)]:
        if kind in INT_GEN:
            x = INT_GEN[kind](n, in_off * 10 + out_off)
            check(x, kind, run_scan(x, kind, "inclusive", in_offset=in_off, out_offset=out_off))
        else:
            x = TRI_GEN[kind](n, in_off * 10 + out_off)
            check(x, kind, run_scan(x, kind, "exclusive", in_offset=in_off, out_offset=out_off), exclusive=True, exact_float=True)


@pytest.mark.parametrize("kind", ["i32", "f32"])
def test_in_place(kind):
    n = 40 * 8192 + 123
    x = (inputs.int32_full if kind == "i32" else inputs.tri_f32)(n, 3)
    got = run_scan(x, kind, "inclusive", inplace=True)
    check(x, kind, got, exact_float=(kind == "f32"))


@pytest.mark.parametrize("kind", ["i32", "f32"])
def test_in_place_rows_that_share_granules(kind):
    """Short rows of odd lengths, in place: a 16-byte granule at a row boundary belongs to two rows, which two
    wavefronts scan at the same time; each must write its own elements only."""
    for rows, cols, call in [(3001, 333, "batched"), (257, 2815, "batched_exclusive"), (1000, 7, "reverse")]:
        x = (inputs.int32_full if kind == "i32" else inputs.tri_f32)(rows * cols, rows + cols)
        got = run_scan(x, kind, call, rows=rows, cols=cols, inplace=True)
        if "reverse" in call:
            assert (oracle.compare_int_reverse if kind == "i32" else oracle.compare_float_exact_reverse)(x, kind, got, rows=rows, cols=cols) == (0, -1)
        else:
            check(x, kind, got, exclusive=call.endswith("exclusive"), rows=rows, cols=cols, exact_float=(kind == "f32"))


@pytest.mark.parametrize("kind", KINDS)
def test_long_rows_that_do_not_start_at_16_byte_boundaries(kind):
    """Odd row lengths and shifted base pointers with rows too long for one wavefront: tiled from the boundary below the
    row start (the descriptor-free form of the segmented kernel), forward and reverse; lengths that fill their last
    tile to the end need one tile more than the workspace promises and take the element-wise path -- same results."""
    cases = [(7, 8191, 0), (3, 3 * 8192 - 1, 0), (5, 2 * 8192 - 2, 0), (9, 65537, 0), (1, 300001, 1), (2, 600001, 3), (3, 40000, 2)]
    for rows, cols, shift in cases:
        for call in ("batched", "batched_exclusive", "reverse", "reverse_exclusive"):
            ex, rev = call.endswith("exclusive"), call.startswith("reverse")
            x = (INT_GEN.get(kind) or TRI_GEN[kind])(rows * cols, rows + cols + shift)
            got = run_scan(x, kind, call, rows=rows, cols=cols, in_offset=shift, out_offset=shift)
            if rev:
                cmp = oracle.compare_int_reverse if kind in INT_GEN else oracle.compare_float_exact_reverse
                assert cmp(x, kind, got, exclusive=ex, rows=rows, cols=cols) == (0, -1), (rows, cols, shift, call)
            else:
                check(x, kind, got, exclusive=ex, rows=rows, cols=cols, exact_float=kind not in INT_GEN)


def test_workspace_is_reusable_across_calls_shapes_and_dtypes():
    import torch
    big = tcuscan.new_workspace(1, 1 << 22, "i8")
    for rep in range(3):
        for kind, n, call in [("i8", (1 << 22) - 5, "exclusive"), ("f16", 100000, "inclusive"), ("i32", 8193, "inclusive"),
                              ("bf16", 1 << 21, "exclusive"), ("f32", 65536 * 3 + 1, "inclusive")]:
            x = (INT_GEN.get(kind) or TRI_GEN[kind])(n, rep * 100 + n)
            got = run_scan(x, kind, call, ws=big)
            check(x, kind, got, exclusive=(call == "exclusive"), exact_float=kind not in INT_GEN)
    x = inputs.int32_small(5 * 20000, 1)
    check(x, "i32", run_scan(x, "i32", "batched", rows=5, cols=20000, ws=big), rows=5, cols=20000)
    assert tcuscan.workspace_fault(big) == 0
    torch.cuda.synchronize()


def test_carry_chain_stress_repeated_calls_are_identical():
    """Many tiles, many repetitions, one workspace: the look-back must give the same integers every time."""
    import torch
    n = 300 * 8192 + 1
    for kind, gen in [("i8", inputs.mask_i8), ("i32", inputs.int32_full)]:
        x = gen(n, 42)
        ref = oracle.scan(x, kind)
        d_in = to_device(x, kind)
        d_ref = torch.from_numpy(ref).cuda()
        ws = tcuscan.new_workspace(1, n, kind)
        out = torch.empty(n, dtype=torch.int32, device="cuda")
        for rep in range(120):
            out.fill_(-1)
            tcuscan.inclusive(d_in, out, kind, ws=ws)
            assert torch.equal(out, d_ref), f"{kind}: repetition {rep} differs"
        assert tcuscan.workspace_fault(ws) == 0


def test_two_streams_with_their_own_workspaces():
    import torch
    n = 200 * 8192 + 9
    xa, xb = inputs.mask_i8(n, 1), inputs.int8_full(n, 2)
    da, db = to_device(xa, "i8"), to_device(xb, "i8")
    oa, ob = torch.empty(n, dtype=torch.int32, device="cuda"), torch.empty(n, dtype=torch.int32, device="cuda")
    wa, wb = tcuscan.new_workspace(1, n, "i8"), tcuscan.new_workspace(1, n, "i8")
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for _ in range(10):
        tcuscan.exclusive(da, oa, "i8", ws=wa, stream=sa)
        tcuscan.inclusive(db, ob, "i8", ws=wb, stream=sb)
    torch.cuda.synchronize()
    check(xa, "i8", oa.cpu().numpy(), exclusive=True)
    check(xb, "i8", ob.cpu().numpy())


def test_workspace_init_kernel_zeroes_the_buffer():
    import torch
    ws = torch.full((1000,), -1, dtype=torch.int64, device="cuda")
    tcuscan.workspace_init(ws)
    torch.cuda.synchronize()
    assert int(ws.abs().sum()) == 0
    n = 20 * 8192
    x = inputs.mask_i8(n, 8)
    check(x, "i8", run_scan(x, "i8", "inclusive", ws=ws))


# ------------------------------------------------------------ both tile sizes, forced

@pytest.fixture
def tile_policy():
    yield tcuscan.set_tile_policy
    tcuscan.set_tile_policy(tcuscan.TILE_AUTO)


@pytest.mark.parametrize("size", ["large", "huge"])
@pytest.mark.parametrize("kind", KINDS)
def test_large_tile_edges(kind, size, tile_policy):
    """Sizes around multiples of the large / huge tile, with that tile forced, inclusive and exclusive."""
    tile_policy(tcuscan.TILE_LARGE if size == "large" else tcuscan.TILE_HUGE)
    lt = tcuscan.large_tile_elems(kind) if size == "large" else tcuscan.huge_tile_elems(kind)
    assert lt % 8192 == 0 and lt > 8192
    for n in [8193, lt - 1, lt, lt + 1, 2 * lt - 3, 3 * lt + lt // 2 + 5, 70 * lt + 4097]:
        print("n =", n, flush=True)
        for call in ("inclusive", "exclusive"):
            ex = call == "exclusive"
            if kind in INT_GEN:
                x = INT_GEN[kind](n, n + 1)
                check(x, kind, run_scan(x, kind, call), exclusive=ex)
            else:
                x = TRI_GEN[kind](n, n + 2)
                check(x, kind, run_scan(x, kind, call), exclusive=ex, exact_float=True)
                x = RND_GEN[kind](n, n + 3)
                check(x, kind, run_scan(x, kind, call), exclusive=ex)


@pytest.mark.parametrize("policy", [1, 2, 3])
@pytest.mark.parametrize("kind", KINDS)
def test_tile_policies_give_the_same_integers(kind, policy, tile_policy):
    tile_policy(policy)
    rows, cols = 5, 3 * tcuscan.huge_tile_elems(kind) + 777
    if kind in INT_GEN:
        x = INT_GEN[kind](rows * cols, policy)
        check(x, kind, run_scan(x, kind, "batched", rows=rows, cols=cols), rows=rows, cols=cols)
    else:
        x = TRI_GEN[kind](rows * cols, policy)
        check(x, kind, run_scan(x, kind, "batched_exclusive", rows=rows, cols=cols), exclusive=True, rows=rows, cols=cols,
              exact_float=True)


def test_auto_policy_picks_the_large_tile_only_for_long_inputs():
    # observable through results only: both must be right; the sizes sit on either side of the switches (128 large
    # tiles in a row, 256 huge tiles of 8- and 16-bit inputs, 512 huge 32-bit tiles)
    for kind in ("i8", "f32", "bf16"):
        lt, ht = tcuscan.large_tile_elems(kind), tcuscan.huge_tile_elems(kind)
        for n in (127 * lt, 127 * lt + 1, 128 * lt + 1, 512 * lt - 1, 512 * lt + 1, 256 * ht - 1, 256 * ht + 1, 512 * ht - ht + 1,
                  512 * ht + 1):
            x = (INT_GEN.get(kind) or TRI_GEN[kind])(n, 7)
            check(x, kind, run_scan(x, kind, "inclusive"), exact_float=kind not in INT_GEN)


@pytest.mark.parametrize("kind", ["i8", "f16", "f32"])
def test_auto_policy_switches_in_batched_calls(kind):
    """Row lengths on either side of the small / large switch (2^17 for 8- and 32-bit inputs, 2^18 for 16-bit), with row
    counts on either side of 256 large tiles in the call."""
    lt = tcuscan.large_tile_elems(kind)
    edge = (1 << 18) if kind in ("f16", "bf16") else (1 << 17)
    for cols in (edge, edge + 8):
        per_row = -(-cols // lt)
        for rows in (1, 255 // per_row, 255 // per_row + 1, 256 // per_row + 2):
            x = (INT_GEN.get(kind) or TRI_GEN[kind])(rows * cols, rows + cols)
            check(x, kind, run_scan(x, kind, "batched", rows=rows, cols=cols), rows=rows, cols=cols, exact_float=kind not in INT_GEN)


# ------------------------------------------------------------------------ graph capture

def test_graph_capture_replays_match_eager():
    """A captured call is replayed with its recorded tag; the library records a fill kernel in front of it
    so stale status words of the previous replay cannot be mistaken for fresh ones."""
    import torch
    n = 100 * 8192 + 321
    kind = "i8"
    ws = tcuscan.new_workspace(1, n, kind)
    d_in = torch.zeros(n, dtype=torch.int8, device="cuda")
    d_out = torch.empty(n, dtype=torch.int32, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        tcuscan.inclusive(d_in, d_out, kind, ws=ws, stream=side)          # warm-up outside capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        tcuscan.inclusive(d_in, d_out, kind, ws=ws, stream=side)
    eager_out = torch.empty_like(d_out)
    for rep in range(5):
        x = inputs.int8_full(n, 100 + rep)
        d_in.copy_(torch.from_numpy(x).cuda())
        d_out.fill_(-1)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        check(x, kind, d_out.cpu().numpy())
        # eager work on the same workspace between the replays
        tcuscan.exclusive(d_in, eager_out, kind, ws=ws)
        torch.cuda.synchronize()
        check(x, kind, eager_out.cpu().numpy(), exclusive=True)
    assert tcuscan.workspace_fault(ws) == 0


def test_graph_capture_of_rows_that_are_not_aligned():
    """The two forms for rows that do not start at 16-byte boundaries (one per wavefront; chained tiles without
    descriptors), recorded into one graph and replayed with new data, eager calls on the same workspace in between."""
    import torch
    kind = "f32"
    rows_a, cols_a = 300, 1001                       # one row per wavefront, tiled from the boundary below the row start
    rows_b, cols_b = 5, 50001                        # chained tiles, status words cleared by a recorded fill kernel
    ws = tcuscan.new_workspace(rows_b, cols_b, kind)
    a_in = torch.zeros(rows_a * cols_a, dtype=torch.float32, device="cuda")
    b_in = torch.zeros(rows_b * cols_b, dtype=torch.float32, device="cuda")
    a_out, b_out = torch.empty_like(a_in), torch.empty_like(b_in)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                     # warm-up outside capture
        tcuscan.batched(a_in, a_out, rows_a, cols_a, kind, stream=side)
        tcuscan.batched(b_in, b_out, rows_b, cols_b, kind, ws=ws, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        tcuscan.batched(a_in, a_out, rows_a, cols_a, kind, stream=side)
        tcuscan.batched(b_in, b_out, rows_b, cols_b, kind, exclusive_scan=True, ws=ws, stream=side)
    eager = torch.empty_like(b_out)
    for rep in range(4):
        xa, xb = inputs.tri_f32(rows_a * cols_a, 70 + rep), inputs.tri_f32(rows_b * cols_b, 80 + rep)
        a_in.copy_(torch.from_numpy(xa).cuda()); b_in.copy_(torch.from_numpy(xb).cuda())
        a_out.fill_(-1); b_out.fill_(-1)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        check(xa, kind, a_out.cpu().numpy(), rows=rows_a, cols=cols_a, exact_float=True)
        check(xb, kind, b_out.cpu().numpy(), exclusive=True, rows=rows_b, cols=cols_b, exact_float=True)
        tcuscan.scan(b_in, eager, rows_b, cols_b, kind, flags=tcuscan.REVERSE, ws=ws)      # eager, same workspace
        torch.cuda.synchronize()
        assert oracle.compare_float_exact_reverse(xb, kind, eager.cpu().numpy(), rows=rows_b, cols=cols_b) == (0, -1)
    assert tcuscan.workspace_fault(ws) == 0


# ------------------------------------------------------------------ seeded random shapes

def test_random_shapes_dtypes_and_offsets(tile_policy):
    """300 seeded random calls: dtype, inclusive / exclusive, rows x cols (log-uniform), tile policy, pointer offsets."""
    rng = np.random.default_rng(20241127)
    for case in range(300):
        kind = KINDS[int(rng.integers(0, 5))]
        ex = bool(rng.integers(0, 2))
        total = int(2 ** rng.uniform(0, 21))
        rows = int(2 ** rng.uniform(0, np.log2(total) + 1e-9)) if rng.integers(0, 3) else 1
        rows = max(1, min(rows, total))
        cols = max(1, total // rows)
        pol = int(rng.integers(0, 4))
        in_off = int(rng.integers(0, 4)) if rng.integers(0, 4) == 0 else 0
        out_off = int(rng.integers(0, 4)) if rng.integers(0, 4) == 0 else 0
        tile_policy(pol)
        call = ("batched_exclusive" if ex else "batched") if rows > 1 else ("exclusive" if ex else "inclusive")
        print(f"case {case}: {kind} {call} {rows}x{cols} policy {pol} offsets {in_off},{out_off}", flush=True)
        n = rows * cols
        if kind in INT_GEN:
            x = INT_GEN[kind](n, case)
            got = run_scan(x, kind, call, rows=rows, cols=cols, in_offset=in_off, out_offset=out_off)
            check(x, kind, got, exclusive=ex, rows=rows, cols=cols)
        else:
            x = TRI_GEN[kind](n, case)
            got = run_scan(x, kind, call, rows=rows, cols=cols, in_offset=in_off, out_offset=out_off)
            check(x, kind, got, exclusive=ex, rows=rows, cols=cols, exact_float=True)


def test_more_than_2_to_the_31_elements():
    """Element indices beyond 31 and 32 bits: n = 2^32 + 2^31 + 12345 int8 {0,1} values (6 GiB in, 24 GiB out on the
    device), checked on sampled windows -- the first and last 2^24 elements and one window across 2^32 -- whose
    carries-in come from a popcount of everything before the window (exact, no scan involved)."""
    import torch
    n = (1 << 32) + (1 << 31) + 12345
    g = torch.Generator(device="cuda").manual_seed(1234)
    d_in = torch.randint(0, 2, (n,), dtype=torch.int8, device="cuda", generator=g)
    d_out = torch.empty(n, dtype=torch.int32, device="cuda")
    ws = tcuscan.new_workspace(1, n, "i8")
    tcuscan.exclusive(d_in, d_out, "i8", ws=ws, n=n)
    torch.cuda.synchronize()
    assert tcuscan.workspace_fault(ws) == 0
    w = 1 << 24
    for start in (0, (1 << 32) - w // 2, n - w):
        # carry into the window: number of ones before it, counted in int64 chunks (a reduction, not a scan)
        before = 0
        for a in range(0, start, 1 << 30):
            before += int(d_in[a:min(a + (1 << 30), start)].sum(dtype=torch.int64).item())
        x = d_in[start:start + w].cpu().numpy()
        got = d_out[start:start + w].cpu().numpy()
        want = oracle.scan_int64(x, "i8", exclusive=True) + before
        assert np.array_equal(got.astype(np.int64) & 0xFFFFFFFF, want & 0xFFFFFFFF), f"window at {start}"
    del d_in, d_out
