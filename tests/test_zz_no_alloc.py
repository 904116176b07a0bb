"""The entry point that allocates nothing (tcuscan_scan_static: the carry chain's status words live in a fixed device
array inside the library) against tcuscan_scan with a caller's workspace: same inputs, two calls in a row, the second
on a smaller input.  Integers must agree bit for bit; floats are compared with the oracle at the usual bar and with
each other within twice that bar (the two calls may group their partial sums differently)."""
import numpy as np
import pytest

import oracle
from paper_2411_17887_amd import inputs, tcuscan
from gpu_util import to_device, out_dtype

pytestmark = pytest.mark.gpu

TOL = {"f16": 1e-3, "bf16": 1e-3, "f32": 1e-5}
GEN = {"i32": inputs.int32_full, "i8": inputs.int8_full, "f32": inputs.f32_normal, "f16": inputs.f16_uniform01,
       "bf16": inputs.bf16_uniform_pm1}


def both(kind, rows, cols, flags, seed):
    import torch
    n = rows * cols
    x = GEN[kind](n, seed)
    d_in = to_device(x, kind)
    ref_out = torch.full((n + 8,), -77, dtype=out_dtype(kind), device="cuda")
    new_out = torch.full((n + 8,), -77, dtype=out_dtype(kind), device="cuda")
    ws = tcuscan.new_workspace(rows, cols, kind)
    tcuscan.scan(d_in, ref_out, rows, cols, kind, flags=flags, ws=ws)
    before = torch.cuda.memory_allocated()
    tcuscan.scan_static(d_in, new_out, rows, cols, kind, flags=flags)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    assert tcuscan.workspace_fault(tcuscan.STATIC_SCRATCH) == 0
    a, b = ref_out.cpu().numpy(), new_out.cpu().numpy()
    assert np.all(b[n:] == -77)
    a, b = a[:n], b[:n]
    excl, rev = bool(flags & tcuscan.EXCLUSIVE), bool(flags & tcuscan.REVERSE)
    if kind in ("i32", "i8"):
        assert np.array_equal(a, b), f"{kind} {rows}x{cols} flags {flags}: static entry differs from tcuscan_scan"
    else:
        fn = oracle.scan_reverse if rev else oracle.scan
        ref, l1 = fn(x, kind, exclusive=excl, rows=rows, cols=cols, with_l1=True)
        ref, l1 = ref.reshape(-1), l1.reshape(-1)
        where = l1 > 0
        e1_new = np.max(np.abs(b.astype(np.float64) - ref)[where] / l1[where], initial=0.0)
        assert e1_new <= TOL[kind] and np.all(b[~where] == 0), (kind, rows, cols, flags, e1_new)
        gap = np.max(np.abs(a.astype(np.float64) - b.astype(np.float64))[where] / l1[where], initial=0.0)
        assert gap <= 2 * TOL[kind], (kind, rows, cols, flags, gap)


@pytest.mark.parametrize("kind", ["i32", "i8", "f32", "f16", "bf16"])
def test_static_entry_matches_the_workspace_entry_on_two_calls_in_a_row(kind):
    tile = tcuscan.tile_elems(kind)
    both(kind, 1, 150 * tile + 37, 0, 11)                       # a long chain ...
    both(kind, 1, 20 * tile + 5, 0, 12)                         # ... then a smaller input over the same scratch
    both(kind, 6, 9 * tile + 3, tcuscan.EXCLUSIVE, 13)          # rows (and rows that do not start at 16-byte boundaries)
    both(kind, 2, 3 * tile, tcuscan.REVERSE, 14)
    both(kind, 1, 100, 0, 15)                                   # no chain at all
    both(kind, 100, 700, tcuscan.EXCLUSIVE | tcuscan.REVERSE, 16)


def test_static_entry_at_the_full_batched_configuration():
    both("bf16", 4096, 65536, 0, 5)
    both("i8", 1, 1 << 28, tcuscan.EXCLUSIVE, 3)
    both("i8", 1, 1 << 20, tcuscan.EXCLUSIVE, 4)


def test_static_entry_recorded_into_a_graph():
    """What the entry point is for: a call under stream capture, where nothing may be allocated.  (Its first call on
    the device was made outside capture by the tests above or by the warm-up here.)  Replayed with new data, eager
    calls on the same scratch between the replays."""
    import torch
    n = 60 * tcuscan.tile_elems("i32") + 9
    d_in = torch.zeros(n, dtype=torch.int32, device="cuda")
    d_out = torch.empty(n, dtype=torch.int32, device="cuda")
    eager_out = torch.empty_like(d_out)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        tcuscan.scan_static(d_in, d_out, 1, n, "i32", stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        tcuscan.scan_static(d_in, d_out, 1, n, "i32", stream=side)
    for rep in range(4):
        x = inputs.int32_full(n, 900 + rep)
        d_in.copy_(torch.from_numpy(x).cuda())
        d_out.fill_(-1)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert oracle.compare_int(x, "i32", d_out.cpu().numpy())[0] == 0
        tcuscan.scan_static(d_in, eager_out, 1, n // 2, "i32", flags=tcuscan.EXCLUSIVE)
        torch.cuda.synchronize()
        assert oracle.compare_int(x[: n // 2], "i32", eager_out.cpu().numpy()[: n // 2], exclusive=True)[0] == 0
    assert tcuscan.workspace_fault(tcuscan.STATIC_SCRATCH) == 0


def test_static_entry_refuses_what_its_scratch_cannot_hold():
    import torch
    t = torch.zeros(16, dtype=torch.int8, device="cuda")
    o = torch.zeros(16, dtype=torch.int32, device="cuda")
    with pytest.raises(tcuscan.TcuscanError) as e:
        tcuscan.scan_static(t, o, 1, (1 << 29) + (1 << 20), "i8")      # rejected on the host, nothing is enqueued
    assert e.value.code == tcuscan.ERR_WORKSPACE
