"""GPU parity for stream compaction and the split radix sort (through the C ABI) against oracle/apps.py.
Integer and index work: everything is compared bit for bit."""
import numpy as np
import pytest

from oracle import apps
from paper_2411_17887_amd import inputs, tcuscan

pytestmark = pytest.mark.gpu


def keys_u32(n, seed):
    return inputs.int32_full(n, seed).view(np.uint32)


def gpu_compact(v, m):
    import torch
    n = v.size
    d_v = torch.from_numpy(v.view(np.int32)).cuda()
    d_m = torch.from_numpy(m).cuda()
    d_out = torch.full((n + 2,), -5, dtype=torch.int32, device="cuda")
    d_pos = torch.empty(n, dtype=torch.int32, device="cuda")
    d_cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    ws = tcuscan.new_workspace(1, n, "i8")
    tcuscan.compact_u32(d_v, d_m, d_out, d_pos, count=d_cnt, ws=ws)
    torch.cuda.synchronize()
    cnt = int(d_cnt.item())
    out = d_out.cpu().numpy()
    assert np.all(out[cnt:] == -5)                      # nothing written past the kept elements
    return out[:cnt].view(np.uint32), d_pos.cpu().numpy(), cnt


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


@pytest.mark.parametrize("n", [1, 2, 17, 1000, 8192 * 5 + 3, (1 << 20) + 1])
def test_sort_full_keys(n):
    k = keys_u32(n, 2 * n + 1)
    got, _ = gpu_sort(k)
    ref, _ = apps.split_radix_sort(k) if n <= 50000 else (np.sort(k), None)
    assert np.array_equal(got, ref)


def test_sort_is_stable_and_moves_payloads():
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


def test_sort_special_inputs():
    n = 70001
    for k in (np.arange(n, dtype=np.uint32), np.arange(n, dtype=np.uint32)[::-1].copy(), np.full(n, 0xDEADBEEF, np.uint32),
              np.where(np.arange(n) % 2 == 0, np.uint32(0xFFFFFFFF), np.uint32(0))):
        got, _ = gpu_sort(k)
        assert np.array_equal(got, np.sort(k))
    g, _ = gpu_sort(keys_u32(1000, 1), bits=0)
    assert np.array_equal(g, keys_u32(1000, 1))              # zero passes: untouched
