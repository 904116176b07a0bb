"""GPU parity for stream compaction and the split radix sort (through the C ABI) against oracle/apps.py.
Integer and index work: everything is compared bit for bit."""
import numpy as np
import pytest

from oracle import apps
from paper_2411_17887_amd import inputs, tcuscan

pytestmark = pytest.mark.gpu


def keys_u32(n, seed):
    return inputs.int32_full(n, seed).view(np.uint32)


def gpu_compact(v, m, fused=False, offset=0):
    """fused: no positions buffer, the scatter happens inside the scan kernel.  offset: shift the value / mask pointers
    by that many elements (pointers that are not 16-byte aligned)."""
    import torch
    n = v.size
    d_v = torch.from_numpy(np.concatenate([np.zeros(offset, np.int32), v.view(np.int32)])).cuda()[offset:]
    d_m = torch.from_numpy(np.concatenate([np.zeros(offset, np.int8), m])).cuda()[offset:]
    d_out = torch.full((n + 2,), -5, dtype=torch.int32, device="cuda")
    d_pos = None if fused else torch.empty(n, dtype=torch.int32, device="cuda")
    d_cnt = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    ws = tcuscan.new_workspace(1, n, "i8")
    tcuscan.compact_u32(d_v, d_m, d_out, d_pos, count=d_cnt, ws=ws)
    torch.cuda.synchronize()
    assert ws is None or tcuscan.workspace_fault(ws) == 0
    cnt = int(d_cnt.item())
    out = d_out.cpu().numpy()
    assert np.all(out[cnt:] == -5)                      # nothing written past the kept elements
    return out[:cnt].view(np.uint32), (None if fused else d_pos.cpu().numpy()), cnt


@pytest.mark.parametrize("n", [1, 15, 4097, 8192 * 3 + 5, (1 << 22) + 9, 1 << 26])
def test_compaction(n):
    v, m = keys_u32(n, n), inputs.mask_i8(n, n + 1)
    got, pos, cnt = gpu_compact(v, m)
    ref, ref_pos = apps.compact(v, m) if n <= (1 << 22) + 9 else (v[m != 0], None)
    assert cnt == ref.size and np.array_equal(got, ref)
    if ref_pos is not None:
        assert np.array_equal(pos, ref_pos)
    for mm in (np.zeros(min(n, 100000), np.int8), np.ones(min(n, 100000), np.int8)):
        g, _, c = gpu_compact(v[: mm.size], mm)
        assert c == int(mm.sum()) and np.array_equal(g, v[: mm.size][mm != 0])


@pytest.mark.parametrize("n", [1, 3, 15, 16, 17, 255, 257, 4097, 8191, 8192, 8193, 8192 * 3 + 5, 65536 * 5 + 77, (1 << 22) + 9, 1 << 26,
                               (1 << 28) + 3])
def test_fused_compaction_without_a_positions_buffer(n):
    v, m = keys_u32(n, n + 7), inputs.mask_i8(n, n + 8)
    got, _, cnt = gpu_compact(v, m, fused=True)
    ref = apps.compact(v, m)[0] if n <= (1 << 22) + 9 else v[m != 0]
    assert cnt == ref.size and np.array_equal(got, ref)
    if n <= (1 << 22) + 9:
        for off in (1, 3):                                  # unaligned values and mask
            g, _, c = gpu_compact(v, m, fused=True, offset=off)
            assert c == ref.size and np.array_equal(g, ref)
        for mm in (np.zeros(n, np.int8), np.ones(n, np.int8)):
            g, _, c = gpu_compact(v, mm, fused=True)
            assert c == int(mm.sum()) and np.array_equal(g, v[mm != 0])


def test_fused_compaction_whatever_the_tile_policy():
    try:
        for policy in (1, 2, 3):
            tcuscan.set_tile_policy(policy)
            n = 7 * 65536 + 4321
            v, m = keys_u32(n, 90 + policy), inputs.mask_i8(n, 91 + policy)
            got, _, cnt = gpu_compact(v, m, fused=True)
            ref = apps.compact(v, m)[0]
            assert cnt == ref.size and np.array_equal(got, ref)
    finally:
        tcuscan.set_tile_policy(tcuscan.TILE_AUTO)


def gpu_sort(k, vals=None, bits=32):
    import torch
    n = k.size
    d_k = torch.from_numpy(k.view(np.int32).copy()).cuda()
    d_kt = torch.empty_like(d_k)
    d_v = torch.from_numpy(vals.view(np.int32).copy()).cuda() if vals is not None else None
    d_vt = torch.empty_like(d_v) if vals is not None else None
    d_f = torch.empty(max(n, 16), dtype=torch.int8, device="cuda")
    d_p = torch.empty(max(n, 1), dtype=torch.int32, device="cuda")
    ws = tcuscan.new_workspace(1, max(n, 1), "i8")
    tcuscan.split_radix_sort_u32(d_k, d_kt, d_f, d_p, vals=d_v, vals_tmp=d_vt, bits=bits, ws=ws)
    torch.cuda.synchronize()
    return d_k.cpu().numpy().view(np.uint32), (d_v.cpu().numpy().view(np.uint32) if vals is not None else None)


@pytest.fixture(params=[1, 2, 0], ids=["fused_two_bits", "fused_one_bit", "three_kernels"])
def sort_form(request):
    """The forms of a split pass: the fused kernels (two bits per pass, the default; one bit per pass) and mask kernel +
    scan + scatter kernel."""
    tcuscan.set_sort_fusion(request.param)
    yield request.param
    tcuscan.set_sort_fusion(1)


@pytest.mark.parametrize("n", [1, 2, 17, 31, 32, 33, 95, 96, 97, 255, 257, 1000, 8192 * 5 + 3, 32768, 32769, 5 * 32768 - 1, (1 << 20) + 1])
def test_sort_full_keys(n, sort_form):
    k = keys_u32(n, 2 * n + 1)
    got, _ = gpu_sort(k)
    ref, _ = apps.split_radix_sort(k) if n <= 50000 else (np.sort(k), None)
    assert np.array_equal(got, ref)


def test_sort_large_and_unaligned(sort_form):
    k = keys_u32((1 << 24) + 12345, 99)
    got, _ = gpu_sort(k, bits=32)
    assert np.array_equal(got, np.sort(k))


def test_sort_is_stable_and_moves_payloads(sort_form):
    n = 300007
    k = keys_u32(n, 5) & np.uint32(0x3FF)
    payload = np.arange(n, dtype=np.uint32)
    gk, gv = gpu_sort(k, payload, bits=10)
    order = np.argsort(k, kind="stable")
    assert np.array_equal(gk, k[order]) and np.array_equal(gv, payload[order])
    # an odd number of passes ends in the scratch buffer and is copied home
    gk, gv = gpu_sort(k, payload, bits=7)
    order = np.argsort(k & np.uint32(0x7F), kind="stable")
    assert np.array_equal(gk, k[order]) and np.array_equal(gv, payload[order])


def test_sort_special_inputs(sort_form):
    n = 70001
    for k in (np.arange(n, dtype=np.uint32), np.arange(n, dtype=np.uint32)[::-1].copy(), np.full(n, 0xDEADBEEF, np.uint32),
              np.where(np.arange(n) % 2 == 0, np.uint32(0xFFFFFFFF), np.uint32(0))):
        got, _ = gpu_sort(k)
        assert np.array_equal(got, np.sort(k))
    g, _ = gpu_sort(keys_u32(1000, 1), bits=0)
    assert np.array_equal(g, keys_u32(1000, 1))              # zero passes: untouched


def test_sort_random_sizes_bits_and_forms():
    """Seeded random cases: sizes around the tile sizes, 1 .. 32 bits (odd counts end with a one-bit pass), keys with few
    distinct values, with and without payloads, both fused forms; against numpy's stable sort."""
    rng = np.random.default_rng(1711)
    try:
        for case in range(40):
            n = int(rng.choice([97, 1000, 16383, 16384, 16385, 100000, (1 << 20) + 7])) + int(rng.integers(0, 50))
            bits = int(rng.integers(1, 33))
            k = keys_u32(n, 3000 + case)
            if rng.random() < 0.3:
                k = k & np.uint32(rng.integers(1, 1 << 16))
            payload = np.arange(n, dtype=np.uint32) if rng.random() < 0.5 else None
            tcuscan.set_sort_fusion(1 + case % 2)
            gk, gv = gpu_sort(k, payload, bits=bits)
            mask = np.uint32((1 << bits) - 1) if bits < 32 else np.uint32(0xFFFFFFFF)
            order = np.argsort(k & mask, kind="stable")
            assert np.array_equal(gk, k[order]), f"case {case}: n {n}, {bits} bits"
            assert payload is None or np.array_equal(gv, payload[order]), f"case {case}: payloads"
    finally:
        tcuscan.set_sort_fusion(1)


def test_graph_capture_of_compaction_and_sort(sort_form):
    """A fused compaction and a sort with payloads recorded into one graph; replays with new data, with eager calls on
    the same workspaces in between, must match the stable reference every time (recorded calls clear their status
    words with fill kernels, and the fused kernels' look-back polls words of the same replay only)."""
    import torch
    n, m = (1 << 20) + 333, (1 << 19) + 77
    d_v = torch.zeros(n, dtype=torch.int32, device="cuda")
    d_m = torch.zeros(n, dtype=torch.int8, device="cuda")
    d_out = torch.empty(n + 2, dtype=torch.int32, device="cuda")
    d_cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    d_k, d_p = torch.zeros(m, dtype=torch.int32, device="cuda"), torch.zeros(m, dtype=torch.int32, device="cuda")
    d_kt, d_pt = torch.empty_like(d_k), torch.empty_like(d_p)
    d_f, d_pos = torch.empty(m, dtype=torch.int8, device="cuda"), torch.empty(m, dtype=torch.int32, device="cuda")
    ws_c, ws_s = tcuscan.new_workspace(1, n, "i8"), tcuscan.new_workspace(1, m, "i8")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                                             # warm-up outside capture
        tcuscan.compact_u32(d_v, d_m, d_out, None, count=d_cnt, ws=ws_c, stream=side)
        tcuscan.split_radix_sort_u32(d_k, d_kt, d_f, d_pos, vals=d_p, vals_tmp=d_pt, bits=32, ws=ws_s, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        tcuscan.compact_u32(d_v, d_m, d_out, None, count=d_cnt, ws=ws_c, stream=side)
        tcuscan.split_radix_sort_u32(d_k, d_kt, d_f, d_pos, vals=d_p, vals_tmp=d_pt, bits=32, ws=ws_s, stream=side)
    for rep in range(3):
        v, msk = keys_u32(n, 70 + rep), inputs.mask_i8(n, 80 + rep)
        k = keys_u32(m, 90 + rep) & np.uint32(0xFFFF if rep == 1 else 0xFFFFFFFF)      # once with many equal keys
        d_v.copy_(torch.from_numpy(v.view(np.int32)).cuda()); d_m.copy_(torch.from_numpy(msk).cuda())
        d_k.copy_(torch.from_numpy(k.view(np.int32)).cuda()); d_p.copy_(torch.arange(m, dtype=torch.int32, device="cuda"))
        d_out.fill_(-5)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        ref = v[msk != 0]
        cnt = int(d_cnt.item())
        out = d_out.cpu().numpy()
        assert cnt == ref.size and np.array_equal(out[:cnt].view(np.uint32), ref) and np.all(out[cnt:] == -5), f"replay {rep}: compaction"
        order = np.argsort(k, kind="stable")
        assert np.array_equal(d_k.cpu().numpy().view(np.uint32), k[order]), f"replay {rep}: keys"
        assert np.array_equal(d_p.cpu().numpy().view(np.uint32), order.astype(np.uint32)), f"replay {rep}: payloads"
        # eager calls on the same workspaces between the replays
        got, _, c = gpu_compact(v[: 100001], msk[: 100001], fused=True)
        assert c == int((msk[: 100001] != 0).sum()) and np.array_equal(got, v[: 100001][msk[: 100001] != 0])
        d_k.copy_(torch.from_numpy(k.view(np.int32)).cuda())
        tcuscan.split_radix_sort_u32(d_k, d_kt, d_f, d_pos, bits=32, ws=ws_s)
        torch.cuda.synchronize()
        assert np.array_equal(d_k.cpu().numpy().view(np.uint32), np.sort(k))
    assert tcuscan.workspace_fault(ws_c) == 0 and tcuscan.workspace_fault(ws_s) == 0
