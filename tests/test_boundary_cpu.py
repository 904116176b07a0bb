"""Host-side checks of the C-ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments with status codes before anything is enqueued."""
import ctypes
import os
import re

import pytest

from paper_2411_17887_amd import tcuscan

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "tcuscan.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tcuscan_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = tcuscan.load()
    names = declared_symbols()
    assert set(names) == set(tcuscan.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_status_strings():
    assert tcuscan.status_string(tcuscan.OK) == "ok"
    seen = {tcuscan.status_string(c) for c in range(5)}
    assert len(seen) == 5 and "unknown status" not in seen
    assert tcuscan.status_string(99) == "unknown status"


def test_workspace_sizing():
    for kind in tcuscan.DTYPES:
        tile = tcuscan.tile_elems(kind)
        assert tile >= 4096 and tile % 4096 == 0
        assert tcuscan.workspace_bytes(1, tile, kind) == 0            # one tile per row: no carry chain
        assert tcuscan.workspace_bytes(1000, tile, kind) == 0
        assert tcuscan.workspace_bytes(1, tile + 1, kind) == 256 + 64 * 2
        # a row and the part of a 16-byte granule in front of it: one more tile when the length is within a granule
        # of a multiple of the tile
        granule = 16 // {"i8": 1, "f16": 2, "bf16": 2}.get(kind, 4)
        assert tcuscan.workspace_bytes(3, 5 * tile - granule + 1, kind) == 256 + 64 * 15
        assert tcuscan.workspace_bytes(3, 5 * tile - granule + 2, kind) == 256 + 64 * 18
        assert tcuscan.workspace_bytes(3, 5 * tile, kind) == 256 + 64 * 18
        assert tcuscan.workspace_bytes(0, 100, kind) == 0 and tcuscan.workspace_bytes(4, 0, kind) == 0
    assert tcuscan.workspace_bytes(1, 1 << 20, 9) == 0 and tcuscan.tile_elems(9) == 0


FAKE = 0x10000      # a non-null, 16-byte aligned address that is never dereferenced on these paths


def call(fn, *a):
    return getattr(tcuscan.load(), fn)(*a)


def test_empty_inputs_are_ok_and_touch_nothing():
    assert call("tcuscan_inclusive", 0, 0, 0, tcuscan.F16_F32, 0, 0, 0) == tcuscan.OK
    assert call("tcuscan_exclusive", 0, 0, 0, tcuscan.I8_I32, 0, 0, 0) == tcuscan.OK
    assert call("tcuscan_batched", 0, 0, 0, 128, tcuscan.F32_F32, 0, 0, 0, 0) == tcuscan.OK
    assert call("tcuscan_batched", 0, 0, 128, 0, tcuscan.F32_F32, 1, 0, 0, 0) == tcuscan.OK
    assert call("tcuscan_workspace_init", 0, 0, 0) == tcuscan.OK


def test_bad_arguments_are_rejected_before_any_launch():
    tile = tcuscan.tile_elems("f32")
    # null pointers with work to do
    assert call("tcuscan_inclusive", 0, FAKE, 10, tcuscan.F32_F32, 0, 0, 0) == tcuscan.ERR_INVALID_ARG
    assert call("tcuscan_inclusive", FAKE, 0, 10, tcuscan.F32_F32, 0, 0, 0) == tcuscan.ERR_INVALID_ARG
    # unknown dtype
    assert call("tcuscan_inclusive", FAKE, FAKE, 10, 5, 0, 0, 0) == tcuscan.ERR_UNSUPPORTED
    assert call("tcuscan_exclusive", FAKE, FAKE, 10, -1, 0, 0, 0) == tcuscan.ERR_UNSUPPORTED
    # pointers not aligned to their element size
    assert call("tcuscan_inclusive", FAKE + 2, FAKE + 64, 10, tcuscan.F32_F32, 0, 0, 0) == tcuscan.ERR_INVALID_ARG
    assert call("tcuscan_inclusive", FAKE + 1, FAKE + 64, 10, tcuscan.F16_F32, 0, 0, 0) == tcuscan.ERR_INVALID_ARG
    assert call("tcuscan_inclusive", FAKE, FAKE + 66, 10, tcuscan.I8_I32, 0, 0, 0) == tcuscan.ERR_INVALID_ARG
    # in place only when element sizes match
    assert call("tcuscan_inclusive", FAKE, FAKE, 10, tcuscan.F16_F32, 0, 0, 0) == tcuscan.ERR_INVALID_ARG
    assert call("tcuscan_inclusive", FAKE, FAKE, 10, tcuscan.I8_I32, 0, 0, 0) == tcuscan.ERR_INVALID_ARG
    # workspace missing / too small / misaligned when the row spans several tiles
    n = 3 * tile - 100            # (not within a granule of a multiple of the tile: the size query is the exact minimum)
    need = tcuscan.workspace_bytes(1, n, "f32")
    assert need == 256 + 64 * 3
    assert call("tcuscan_inclusive", FAKE, FAKE + (1 << 30), n, tcuscan.F32_F32, 0, 0, 0) == tcuscan.ERR_WORKSPACE
    assert call("tcuscan_inclusive", FAKE, FAKE + (1 << 30), n, tcuscan.F32_F32, FAKE, need - 1, 0) == tcuscan.ERR_WORKSPACE
    assert call("tcuscan_inclusive", FAKE, FAKE + (1 << 30), n, tcuscan.F32_F32, FAKE + 4, need, 0) == tcuscan.ERR_WORKSPACE
    assert call("tcuscan_batched", FAKE, FAKE + (1 << 30), 2, n, tcuscan.F32_F32, 0, FAKE, need, 0) == tcuscan.ERR_WORKSPACE
    # more tiles than the 31-bit tile index can name
    assert call("tcuscan_batched", FAKE, FAKE + (1 << 30), 1 << 33, 16, tcuscan.I8_I32, 0, 0, 0, 0) == tcuscan.ERR_UNSUPPORTED
    # workspace_init / workspace_fault argument checks
    assert call("tcuscan_workspace_init", 0, 64, 0) == tcuscan.ERR_INVALID_ARG
    assert call("tcuscan_workspace_init", FAKE + 4, 64, 0) == tcuscan.ERR_INVALID_ARG
    assert call("tcuscan_workspace_fault", 0, 0, ctypes.byref(ctypes.c_uint(0))) == tcuscan.ERR_INVALID_ARG
    assert call("tcuscan_workspace_fault", FAKE, 0, None) == tcuscan.ERR_INVALID_ARG


def test_binding_raises_with_the_status_text():
    with pytest.raises(tcuscan.TcuscanError) as e:
        class T:                      # stands in for a tensor: only data_ptr / numel / element_size are marshalled
            def data_ptr(self): return 0
            def numel(self): return 5
            def element_size(self): return 4
        tcuscan.inclusive(T(), T(), "f32", stream=0)
    assert e.value.code == tcuscan.ERR_INVALID_ARG and "invalid argument" in str(e.value)


def test_new_entry_points_reject_bad_arguments_on_the_host():
    """tcuscan_scan (flags), tcuscan_segmented and the radix executor: everything the host can refuse, it refuses
    before a launch (these calls return without touching the fake pointers)."""
    # unknown flag bits; empty shapes are fine whatever the flags
    assert call("tcuscan_scan", FAKE, FAKE + (1 << 30), 1, 10, tcuscan.F32_F32, 4, 0, 0, 0) == tcuscan.ERR_INVALID_ARG
    assert call("tcuscan_scan", 0, 0, 0, 10, tcuscan.F32_F32, 3, 0, 0, 0) == tcuscan.OK
    assert call("tcuscan_scan", FAKE, 0, 1, 10, tcuscan.F32_F32, 2, 0, 0, 0) == tcuscan.ERR_INVALID_ARG
    # segmented: sizing is monotone in both arguments, zero for nothing to do, and the call checks its arguments
    assert tcuscan.segmented_workspace_bytes(0, 100, "f32") == 0 and tcuscan.segmented_workspace_bytes(5, 0, "f32") == 0
    assert tcuscan.segmented_workspace_bytes(5, 100, 9) == 0
    a = tcuscan.segmented_workspace_bytes(10, 1000, "i8")
    assert 0 < a <= tcuscan.segmented_workspace_bytes(20, 1000, "i8") <= tcuscan.segmented_workspace_bytes(20, 100000, "i8")
    assert call("tcuscan_segmented", 0, 0, 0, 0, 100, tcuscan.F32_F32, 0, 0, 0, 0) == tcuscan.OK          # no rows
    assert call("tcuscan_segmented", FAKE, FAKE + (1 << 30), 0, 2, 100, tcuscan.F32_F32, 0, FAKE, 1 << 20, 0) == tcuscan.ERR_INVALID_ARG
    assert call("tcuscan_segmented", FAKE, FAKE + (1 << 30), FAKE + 4, 2, 100, tcuscan.F32_F32, 0, FAKE, 1 << 20, 0) == tcuscan.ERR_INVALID_ARG
    assert call("tcuscan_segmented", FAKE, FAKE + (1 << 30), FAKE, 2, 100, tcuscan.F32_F32, 8, FAKE, 1 << 20, 0) == tcuscan.ERR_INVALID_ARG
    assert call("tcuscan_segmented", FAKE, FAKE + (1 << 30), FAKE, 2, 100, tcuscan.F32_F32, 0, 0, 0, 0) == tcuscan.ERR_WORKSPACE
    need = tcuscan.segmented_workspace_bytes(2, 100, "f32")
    assert call("tcuscan_segmented", FAKE, FAKE + (1 << 30), FAKE, 2, 100, tcuscan.F32_F32, 0, FAKE, need - 1, 0) == tcuscan.ERR_WORKSPACE
    assert call("tcuscan_segmented", FAKE, FAKE, FAKE, 2, 100, tcuscan.F16_F32, 0, FAKE, need, 0) == tcuscan.ERR_INVALID_ARG   # in place, 16-bit
    assert call("tcuscan_segmented", FAKE, FAKE + (1 << 30), FAKE, 2, 100, 7, 0, FAKE, need, 0) == tcuscan.ERR_UNSUPPORTED
    # radix executor: only s = 4, 16, 32 and n = s^k
    for s, n in [(2, 16), (8, 64), (4, 5), (32, 1000), (16, 0)]:
        assert call("tcuscan_matmulscan_levels_radix", FAKE, FAKE + (1 << 30), n, tcuscan.I32_I32, s, -1, 0, 0) == tcuscan.ERR_UNSUPPORTED
    assert call("tcuscan_matmulscan_levels_radix", 0, FAKE, 16, tcuscan.I32_I32, 4, -1, 0, 0) == tcuscan.ERR_INVALID_ARG


def test_process_wide_knobs():
    """The measurement / test knobs are host-side settings: valid values are accepted, anything else is refused, and
    the defaults are put back."""
    try:
        for form in (0, 1, 2):
            assert call("tcuscan_set_sort_fusion", form) == tcuscan.OK
        for form in (-1, 3, 100):
            assert call("tcuscan_set_sort_fusion", form) == tcuscan.ERR_INVALID_ARG
        with pytest.raises(tcuscan.TcuscanError):
            tcuscan.set_sort_fusion(7)
        for flat in (0, 1, 5):                                   # any non-zero value means "on"
            assert call("tcuscan_set_segmented_form", flat) == tcuscan.OK
        for policy in (0, 1, 2, 3):
            assert call("tcuscan_set_tile_policy", policy) == tcuscan.OK
        assert call("tcuscan_set_tile_policy", 4) == tcuscan.ERR_INVALID_ARG
    finally:
        tcuscan.set_sort_fusion(1)
        tcuscan.set_segmented_form(True)
        call("tcuscan_set_tile_policy", 0)


def test_path_query_and_workspace_promise():
    """tcuscan_path_for is the host-side decision run() itself follows.  With a workspace of tcuscan_workspace_bytes()
    no shape is left to the element-wise path."""
    A, U = 0x10000, 0x10004            # a 16-byte aligned address and one that is not
    for kind, esz in (("i8", 1), ("f16", 2), ("bf16", 2), ("f32", 4), ("i32", 4)):
        tile, large = tcuscan.tile_elems(kind), tcuscan.large_tile_elems(kind)
        g = 16 // esz
        assert tcuscan.path_for(A, 100, 512, kind, 0) == tcuscan.PATH_ROWS
        assert tcuscan.path_for(U, 100, 513, kind, 0) == tcuscan.PATH_ROWS           # short rows handle their own alignment
        assert tcuscan.path_for(A, 1, 10 * tile + 3, kind, 1 << 20) == tcuscan.PATH_TILES
        assert tcuscan.path_for(A, 4, 10 * tile, kind, 1 << 20) == tcuscan.PATH_TILES
        for rows, cols in ((1, 10 * tile), (3, 10 * tile + 1), (5, 3 * tile), (7, 2 * large), (2, 64 * large), (3, 64 * large - 1),
                           (1000, tile), (9, 2 * tile - 1)):
            ptr = U if rows == 1 or (cols * esz) % 16 == 0 else A
            new = tcuscan.workspace_bytes(rows, cols, kind)
            assert tcuscan.path_for(ptr, rows, cols, kind, new) == tcuscan.PATH_TILES_FROM_BOUNDARY, (kind, rows, cols)
            # a workspace sized by the older rule (tiles of the rows alone) is still enough for one of the two tile sizes
            old_tiles = -(-cols // tile)
            old = 256 + 64 * rows * old_tiles if old_tiles > 1 else 0
            assert old <= new and tcuscan.path_for(ptr, rows, cols, kind, old) == tcuscan.PATH_TILES_FROM_BOUNDARY
    assert tcuscan.path_for(A, 0, 5, "f32", 0) == -1 and tcuscan.path_for(A, 5, 5, 9, 0) == -1


def test_chain_knobs_static_entry_and_stream_kernel_reject_bad_arguments():
    try:
        assert call("tcuscan_set_chain_policy", 1) == tcuscan.OK
        for bad in (-1, 2):
            assert call("tcuscan_set_chain_policy", bad) == tcuscan.ERR_INVALID_ARG
    finally:
        assert call("tcuscan_set_chain_policy", 0) == tcuscan.OK
    assert call("tcuscan_test_chain_fault", 0, 1 << 40) == tcuscan.ERR_INVALID_ARG
    assert call("tcuscan_test_chain_fault", 0, -1) == tcuscan.OK
    assert tcuscan.test_tag_period() == (1 << 30) - 2
    # the entry point without a workspace argument: same host-side checks, and a clear refusal beyond its fixed scratch
    assert call("tcuscan_scan_static", 0, 0, 0, 10, tcuscan.F32_F32, 0, 0) == tcuscan.OK
    assert call("tcuscan_scan_static", FAKE, FAKE + (1 << 30), 1, 10, tcuscan.F32_F32, 4, 0) == tcuscan.ERR_INVALID_ARG
    assert call("tcuscan_scan_static", FAKE, FAKE + (1 << 30), 1, 10, 9, 0, 0) == tcuscan.ERR_UNSUPPORTED
    tile = tcuscan.tile_elems("i8")
    assert tcuscan.workspace_bytes(1, 65535 * tile, "i8") <= tcuscan.STATIC_SCRATCH_BYTES < tcuscan.workspace_bytes(1, 65536 * tile + 1, "i8")
    assert call("tcuscan_scan_static", FAKE, FAKE + (1 << 34), 1, 65536 * tile + 1, tcuscan.I8_I32, 0, 0) == tcuscan.ERR_WORKSPACE
    assert call("tcuscan_scan_static", FAKE, FAKE + (1 << 34), 70000, 2 * tile, tcuscan.I8_I32, 0, 0) == tcuscan.ERR_WORKSPACE
    # streaming yardstick: mixes 0, 1, 2, 4 only; aligned pointers; whole 64-byte groups
    assert call("tcuscan_measure_stream", FAKE, FAKE, 0, 1, 0, 0) == tcuscan.OK
    assert call("tcuscan_measure_stream", FAKE, FAKE, 64, 3, 0, 0) == tcuscan.ERR_INVALID_ARG
    assert call("tcuscan_measure_stream", FAKE, FAKE, 64, 1, 6, 0) == tcuscan.ERR_INVALID_ARG
    assert call("tcuscan_measure_stream", FAKE, FAKE, 64, 1, 8, 0) == tcuscan.ERR_INVALID_ARG
    assert call("tcuscan_measure_stream", FAKE, FAKE, 64, 1, 0x2000, 0) == tcuscan.ERR_INVALID_ARG
    assert call("tcuscan_measure_stream", FAKE, FAKE, 64, 1, 0x1800, 0) == tcuscan.ERR_INVALID_ARG      # pause: 0, 1 or 2
    assert call("tcuscan_measure_stream", FAKE, FAKE, 64, 1, 0x802, 0) == tcuscan.ERR_INVALID_ARG       # ... with 1 or 2 loads per lane
    assert call("tcuscan_measure_stream", FAKE, FAKE, 64, 0, 0x800, 0) == tcuscan.ERR_INVALID_ARG       # ... and an input
    assert call("tcuscan_measure_stream", FAKE, FAKE + 4, 64, 1, 0, 0) == tcuscan.ERR_INVALID_ARG
    assert call("tcuscan_measure_stream", 0, FAKE, 64, 2, 0, 0) == tcuscan.ERR_INVALID_ARG
    assert call("tcuscan_measure_stream", FAKE, FAKE, 48, 4, 0, 0) == tcuscan.ERR_INVALID_ARG
