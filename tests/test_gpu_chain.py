"""GPU tests of the carry chain's protocol around its edges: status-word tags that come round again, the ticket
policy (tiles drawn from a counter instead of taken in workgroup-index order), and a wait that is made to give up
from the host -- which must end in a fault word, with every kernel exiting normally, and never in a hang."""
import numpy as np
import pytest

import oracle
from oracle import apps
from paper_2411_17887_amd import inputs, tcuscan
from gpu_util import run_scan, to_device, out_dtype
from test_gpu_parity import check, INT_GEN, RND_GEN, KINDS
import test_gpu_segmented as seg

pytestmark = pytest.mark.gpu


def test_tags_that_come_round_do_not_resurrect_old_status_words():
    """Call A leaves finished-prefix words with tag T in every slot.  Exactly one tag period later call B draws T
    again: without the library's own clearing B's tiles would take A's words for their predecessors' prefixes."""
    import torch
    tile = tcuscan.tile_elems("i32")
    n = 300 * tile + 11
    period = tcuscan.test_tag_period()
    ws = tcuscan.new_workspace(1, n, "i32")
    xa, xb = inputs.int32_full(n, 51), inputs.int32_full(n, 52)
    d_a, d_b = to_device(xa, "i32"), to_device(xb, "i32")
    out = torch.empty(n, dtype=torch.int32, device="cuda")
    tcuscan.inclusive(d_a, out, "i32", ws=ws)
    torch.cuda.synchronize()
    assert oracle.compare_int(xa, "i32", out.cpu().numpy())[0] == 0
    tcuscan.test_advance_calls(period - 1)                    # the next call's tag is A's tag, one generation on
    tcuscan.inclusive(d_b, out, "i32", ws=ws)
    torch.cuda.synchronize()
    assert oracle.compare_int(xb, "i32", out.cpu().numpy())[0] == 0
    # later calls of the new generation, a smaller and then a larger one on a workspace that is larger still
    big = tcuscan.new_workspace(1, 2 * n, "i32")
    for m, seed in ((n // 3, 53), (2 * n, 54)):
        x = inputs.int32_full(m, seed)
        o = torch.empty(m, dtype=torch.int32, device="cuda")
        tcuscan.exclusive(to_device(x, "i32"), o, "i32", ws=big)
        torch.cuda.synchronize()
        assert oracle.compare_int(x, "i32", o.cpu().numpy(), exclusive=True)[0] == 0
    tcuscan.test_advance_calls(period - 2)                    # ... and round once more, on the same workspaces
    for w in (ws, big):
        tcuscan.inclusive(d_a, out, "i32", ws=w)
        torch.cuda.synchronize()
        assert oracle.compare_int(xa, "i32", out.cpu().numpy())[0] == 0
        assert tcuscan.workspace_fault(w) == 0


@pytest.fixture
def ticket_policy():
    tcuscan.set_chain_policy(1)
    yield
    tcuscan.set_chain_policy(0)


@pytest.mark.parametrize("kind", KINDS)
def test_ticket_policy_gives_the_same_results(kind, ticket_policy):
    tile = tcuscan.tile_elems(kind)
    for call, rows, cols in (("inclusive", 1, 70 * tile + 13), ("exclusive", 1, 33 * tile), ("batched", 5, 9 * tile + 1),
                             ("batched_exclusive", 3, 4 * tile - 1), ("reverse", 2, 11 * tile + 5), ("inclusive", 1, (1 << 23) + 3)):
        n = rows * cols
        x = INT_GEN[kind](n, 700 + cols % 1000) if kind in INT_GEN else RND_GEN[kind](n, 700 + cols % 1000)
        got = run_scan(x, kind, call, rows=rows, cols=cols)
        if call.startswith("reverse"):
            ref_in = x.reshape(rows, cols)[:, ::-1].copy().reshape(-1)
            got = got.reshape(rows, cols)[:, ::-1].copy().reshape(-1)
            check(ref_in, kind, got, rows=rows, cols=cols)
        else:
            check(x, kind, got, exclusive=call.endswith("exclusive"), rows=rows, cols=cols)
    # rows that do not start at 16-byte boundaries (tiles from the boundary below)
    rows, cols = 3, 5 * tile + 1
    x = INT_GEN[kind](rows * cols, 9) if kind in INT_GEN else RND_GEN[kind](rows * cols, 9)
    check(x, kind, run_scan(x, kind, "batched", rows=rows, cols=cols), rows=rows, cols=cols)


@pytest.mark.parametrize("kind", ["f32", "i8", "bf16"])
def test_ticket_policy_segmented(kind, ticket_policy):
    rng = np.random.default_rng(5)
    for lengths in (rng.geometric(1 / 150, size=3000) - 1, np.array([40000, 0, 3, 100001, 8192, 1]), rng.integers(0, 30000, size=40)):
        off = seg.offsets_from(lengths)
        n = int(off[-1])
        x = INT_GEN[kind](n, 31) if kind in INT_GEN else RND_GEN[kind](n, 31)
        for flat in seg.forms():
            for flags in (0, tcuscan.EXCLUSIVE | tcuscan.REVERSE):
                got, fault = seg.run_segmented(x, kind, off, flags=flags)
                assert fault == 0
                seg.check(x, kind, off, got, bool(flags & tcuscan.EXCLUSIVE), bool(flags & tcuscan.REVERSE))


def test_ticket_policy_compaction_and_sort(ticket_policy):
    import torch
    from test_gpu_apps import gpu_compact, keys_u32
    n = 8192 * 40 + 77
    v, m = keys_u32(n, 3), inputs.mask_i8(n, 4)
    for fused in (False, True):
        got, _, cnt = gpu_compact(v, m, fused=fused)
        ref = apps.compact(v, m)[0]
        assert cnt == ref.size and np.array_equal(got, ref)
    n = (1 << 20) + 5
    k = keys_u32(n, 8)
    for form in (1, 2, 0):
        tcuscan.set_sort_fusion(form)
        try:
            d_k = torch.from_numpy(k.view(np.int32)).cuda()
            tmp, flags, pos = torch.empty_like(d_k), torch.empty(n, dtype=torch.int8, device="cuda"), torch.empty_like(d_k)
            ws = tcuscan.new_workspace(1, n, "i8")
            tcuscan.split_radix_sort_u32(d_k, tmp, flags, pos, bits=32, ws=ws)
            torch.cuda.synchronize()
            assert tcuscan.workspace_fault(ws) == 0
            assert np.array_equal(d_k.cpu().numpy().view(np.uint32), np.sort(k, kind="stable"))
        finally:
            tcuscan.set_sort_fusion(1)


def test_ticket_policy_recorded_into_a_graph(ticket_policy):
    """The ticket counter is cleared by a kernel in front of the scan, so a recorded call draws its tickets from zero
    on every replay; eager calls (also ticketed) run on the same workspace between the replays."""
    import torch
    n = 90 * tcuscan.tile_elems("i8") + 17
    ws = tcuscan.new_workspace(1, n, "i8")
    d_in = torch.zeros(n, dtype=torch.int8, device="cuda")
    d_out = torch.empty(n, dtype=torch.int32, device="cuda")
    eager_out = torch.empty_like(d_out)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        tcuscan.inclusive(d_in, d_out, "i8", ws=ws, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        tcuscan.inclusive(d_in, d_out, "i8", ws=ws, stream=side)
    for rep in range(4):
        x = inputs.int8_full(n, 300 + rep)
        d_in.copy_(torch.from_numpy(x).cuda())
        d_out.fill_(-1)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        check(x, "i8", d_out.cpu().numpy())
        tcuscan.exclusive(d_in, eager_out, "i8", ws=ws)
        torch.cuda.synchronize()
        check(x, "i8", eager_out.cpu().numpy(), exclusive=True)
    assert tcuscan.workspace_fault(ws) == 0


def test_a_tile_that_never_publishes_ends_in_a_fault_word_not_in_a_hang():
    """Forced from the host: tile 3 keeps silent and the wait's poll limit is tiny, so every later tile gives up,
    publishes a (wrong) prefix and goes on; the kernel ends normally and the sticky fault word reads 1."""
    import torch
    tile = tcuscan.tile_elems("i32")
    n = 40 * tile
    x = inputs.int32_full(n, 77)
    d_in = to_device(x, "i32")
    out = torch.empty(n, dtype=torch.int32, device="cuda")
    ws = tcuscan.new_workspace(1, n, "i32")
    tcuscan.set_tile_policy(tcuscan.TILE_SMALL)
    try:
        tcuscan.test_chain_fault(spin_limit=64, mute_tile=3)
        tcuscan.inclusive(d_in, out, "i32", ws=ws)
        torch.cuda.synchronize()
        assert tcuscan.workspace_fault(ws) == 1
        got = out.cpu().numpy()
        ref = oracle.scan(x, "i32")
        assert np.array_equal(got[: 4 * tile], ref[: 4 * tile])        # tiles 0..3 never waited for the silent one
    finally:
        tcuscan.test_chain_fault(0, -1)
        tcuscan.set_tile_policy(tcuscan.TILE_AUTO)
    # the fault word is sticky until the workspace is initialised again; after that the same call is right
    tcuscan.inclusive(d_in, out, "i32", ws=ws)
    torch.cuda.synchronize()
    assert tcuscan.workspace_fault(ws) == 1
    tcuscan.workspace_init(ws)
    tcuscan.inclusive(d_in, out, "i32", ws=ws)
    torch.cuda.synchronize()
    assert tcuscan.workspace_fault(ws) == 0
    assert oracle.compare_int(x, "i32", out.cpu().numpy())[0] == 0


def test_plain_call_after_segmented_calls_on_the_same_workspace():
    """A segmented call keeps row maps where a plain call of another shape expects status words; the library clears
    them itself before the plain call."""
    import torch
    n = 1 << 22
    lengths = np.full(2000, n // 2000)
    off = seg.offsets_from(lengths)
    total = int(off[-1])
    x = inputs.int32_full(total, 5)
    ws = tcuscan.new_segmented_workspace(len(lengths), total, "i32")
    assert ws.numel() * 8 >= tcuscan.workspace_bytes(1, total, "i32")
    for rep in range(2):
        got, fault = seg.run_segmented(x, "i32", off, ws=ws)
        assert fault == 0
        seg.check(x, "i32", off, got, False, False)
        check(x, "i32", run_scan(x, "i32", "inclusive", ws=ws))


@pytest.mark.parametrize("mix", [0, 1, 2, 4])
def test_streaming_yardstick_writes_what_it_says(mix):
    """Measurement kernel: output granule R*i + k of a wavefront's R KiB is input granule i plus k in every word
    (write-only: a pattern of the output index); every byte of the output is written, nothing beyond it."""
    import torch
    out_bytes = 1 << 20
    R = 4 // mix if mix else 0
    n_out = out_bytes // 16
    x = np.arange(4 * (n_out // max(R, 1)), dtype=np.uint32) * 7 + 1
    d_in = torch.from_numpy(x.view(np.int32)).cuda()
    pauses = (0x800, 0x1001, 0x900, 0x1300) if mix else ()          # a pause between loads and stores: kernels with input only
    for variant in (0, 1, 2, 3, 0x100, 0x103, 0x200, 0x203, 0x302, 0x401, 0x703, 0x204, 0x205, 0x705) + pauses:
        d_out = torch.full((n_out * 4 + 64,), -1, dtype=torch.int32, device="cuda")
        tcuscan.measure_stream(d_in, d_out, out_bytes, mix, variant)
        torch.cuda.synchronize()
        got = d_out.cpu().numpy().view(np.uint32)
        assert np.all(got[n_out * 4:] == 0xFFFFFFFF)
        g = got[: n_out * 4].reshape(n_out, 4)
        if R == 0:
            assert np.array_equal(g[:, :3], np.tile(np.array([1, 2, 3], np.uint32), (n_out, 1)))
            assert np.array_equal(g[:, 3], np.arange(n_out, dtype=np.uint32))
        else:
            i = np.arange(n_out // R)
            src = x.reshape(-1, 4)
            for k in range(R):
                o = (i & ~63) * R + 64 * k + (i & 63)
                assert np.array_equal(g[o], src + np.uint32(k))
