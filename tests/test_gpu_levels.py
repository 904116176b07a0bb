"""GPU parity for the round-by-round executor of Algorithm 1 (tcuscan_matmulscan_levels).

Final results against the sequential oracle; intermediate states after every round against the CPU
replay of the paper's schedule (which is itself pinned to Figure 1(a)); the number of s x s products
against the replay's count and Lemma 1's bound (tests/golden/lemma1_counts.txt)."""
import os

import numpy as np
import pytest

import oracle
from oracle import matmulscan_model as mm
from paper_2411_17887_amd import inputs, tcuscan
from gpu_util import to_device, out_dtype

pytestmark = pytest.mark.gpu
GOLD = os.path.join(os.path.dirname(__file__), "golden")


def run_levels(x, kind, rounds=-1, count=False, inplace=False, s=16):
    import torch
    d_in = to_device(x, kind)
    d_out = d_in if inplace else torch.full((x.size + 4,), -7, dtype=out_dtype(kind), device="cuda")
    cnt = torch.zeros(1, dtype=torch.int64, device="cuda") if count else None
    tcuscan.matmulscan_levels(d_in, d_out, kind, rounds=rounds, matmuls=cnt, n=x.size, s=s)
    torch.cuda.synchronize()
    if not inplace:
        assert int((d_out[x.size:] != -7).sum()) == 0
    got = d_out[: x.size].cpu().numpy().copy()
    return (got, int(cnt.item())) if count else got


def lemma_rows():
    rows = []
    with open(os.path.join(GOLD, "lemma1_counts.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append(tuple(int(t) for t in line.split()))
    return {r[2]: r for r in rows if r[0] == 16}


def lemma_row(s, n):
    with open(os.path.join(GOLD, "lemma1_counts.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                r = tuple(int(t) for t in line.split())
                if r[0] == s and r[2] == n:
                    return r
    raise KeyError((s, n))


@pytest.mark.parametrize("k", [1, 2, 3, 4])
@pytest.mark.parametrize("kind", ["i32", "i8", "f32", "f16", "bf16"])
def test_final_result_and_product_count(kind, k):
    n = 16 ** k
    ints = kind in ("i32", "i8")
    gen = {"i32": inputs.int32_full, "i8": inputs.int8_full, "f32": inputs.tri_f32, "f16": inputs.tri_f16,
           "bf16": inputs.tri_bf16_bits}[kind]
    x = gen(n, 50 + k)
    got, cnt = run_levels(x, kind, count=True)
    if ints:
        assert oracle.compare_int(x, kind, got) == (0, -1)
    else:
        assert oracle.compare_float_exact(x, kind, got) == (0, -1)
    tr = mm.Trace()
    mm.matmul_scan(np.zeros(n, dtype=np.int64), 16, tr)
    s, kk, nn, depth, bound = lemma_rows()[n]
    assert cnt == tr.matmuls <= bound and tr.depth == depth == 2 * k - 1


@pytest.mark.parametrize("kind", ["i32", "f32"])
def test_every_intermediate_state_matches_the_cpu_replay(kind):
    n, k = 4096, 3
    x = inputs.int32_small(n, inputs.BASE_SEED)           # the C1 input; as floats every partial sum is exact
    tr = mm.Trace()
    mm.matmul_scan(x.astype(np.int64), 16, tr)
    xin = x if kind == "i32" else x.astype(np.float32)
    for r in range(1, 2 * k):
        got = run_levels(xin, kind, rounds=r)
        assert np.array_equal(got.astype(np.int64), tr.states[r - 1]), f"state after round {r}"
    assert np.array_equal(run_levels(xin, kind, rounds=0, inplace=True).astype(np.int64), x.astype(np.int64))


def test_random_floats_within_tolerance_and_large_sizes():
    for kind, gen, tol in [("f32", inputs.f32_normal, 1e-5), ("f16", inputs.f16_uniform01, 1e-3), ("bf16", inputs.bf16_uniform_pm1, 1e-3)]:
        x = gen(16 ** 5, 9)
        rep = oracle.compare_float(x, kind, run_levels(x, kind))
        assert rep.ok(tol), rep
    x = inputs.mask_i8(16 ** 6, 3)
    got, cnt = run_levels(x, "i8", count=True)
    assert oracle.compare_int(x, "i8", got) == (0, -1)
    assert cnt == 139811 <= lemma_rows()[16 ** 6][4]
    x = inputs.int32_full(16 ** 5, 4)
    assert oracle.compare_int(x, "i32", run_levels(x, "i32", inplace=True)) == (0, -1)


def test_full_size_2p28_result_and_lemma1_count():
    x = inputs.mask_i8(16 ** 7, inputs.CONFIGS["C3"]["seed"])
    got, cnt = run_levels(x, "i8", count=True)
    assert oracle.compare_int(x, "i8", got) == (0, -1)
    assert cnt == 2236963 <= lemma_rows()[16 ** 7][4]          # 13 rounds


def test_lengths_that_are_not_powers_of_16_are_refused():
    import torch
    t = torch.zeros(48, dtype=torch.int32, device="cuda")
    for n in (0, 15, 17, 48, 4095):
        with pytest.raises(tcuscan.TcuscanError) as e:
            tcuscan.matmulscan_levels(t, t, "i32", n=n)
        assert e.value.code == tcuscan.ERR_UNSUPPORTED


# ---------------------------------------------------------------- other radices: s = 4 and s = 32

@pytest.mark.parametrize("s,k", [(4, 1), (4, 2), (4, 3), (4, 6), (32, 1), (32, 2), (32, 3)])
@pytest.mark.parametrize("kind", ["i32", "i8", "f32", "f16", "bf16"])
def test_radix_final_result_and_product_count(kind, s, k):
    n = s ** k
    gen = {"i32": inputs.int32_full, "i8": inputs.int8_full, "f32": inputs.tri_f32, "f16": inputs.tri_f16,
           "bf16": inputs.tri_bf16_bits}[kind]
    x = gen(n, 70 + s + k)
    got, cnt = run_levels(x, kind, count=True, s=s)
    if kind in ("i32", "i8"):
        assert oracle.compare_int(x, kind, got) == (0, -1)
    else:
        assert oracle.compare_float_exact(x, kind, got) == (0, -1)
    tr = mm.Trace()
    mm.matmul_scan(np.zeros(n, dtype=np.int64), s, tr)
    _, kk, _, depth, bound = lemma_row(s, n)
    assert cnt == tr.matmuls == mm.product_count(n, s) <= bound and tr.depth == depth == 2 * k - 1


@pytest.mark.parametrize("s,k", [(4, 6), (32, 3)])
@pytest.mark.parametrize("kind", ["i32", "f32"])
def test_radix_every_intermediate_state_matches_the_cpu_replay(kind, s, k):
    n = s ** k
    x = inputs.int32_small(n, inputs.BASE_SEED + s)       # small integers: as floats every partial sum is exact
    tr = mm.Trace()
    mm.matmul_scan(x.astype(np.int64), s, tr)
    xin = x if kind == "i32" else x.astype(np.float32)
    for r in range(1, 2 * k):
        got = run_levels(xin, kind, rounds=r, s=s)
        assert np.array_equal(got.astype(np.int64), tr.states[r - 1]), f"s={s}: state after round {r}"


def test_radix_large_sizes():
    # s = 4, n = 4^12 = 2^24 (23 rounds); s = 32, n = 32^5 = 2^25 (9 rounds); full-range integers wrap mod 2^32
    for s, k in [(4, 12), (32, 5)]:
        n = s ** k
        x = inputs.mask_i8(n, 5 + s)
        got, cnt = run_levels(x, "i8", count=True, s=s)
        assert oracle.compare_int(x, "i8", got) == (0, -1)
        assert cnt == mm.product_count(n, s)
        x = inputs.int32_full(n, 6 + s)
        assert oracle.compare_int(x, "i32", run_levels(x, "i32", inplace=True, s=s)) == (0, -1)
        x = inputs.f32_normal(n, 7 + s)
        rep = oracle.compare_float(x, "f32", run_levels(x, "f32", s=s))
        assert rep.ok(1e-5), rep
    assert mm.product_count(32 ** 5, 32) == 67651 <= lemma_row(32, 32 ** 5)[4]


def test_radix_full_size_2p28_with_s4():
    n = 4 ** 14
    x = inputs.mask_i8(n, inputs.CONFIGS["C3"]["seed"])
    got, cnt = run_levels(x, "i8", count=True, s=4)
    assert oracle.compare_int(x, "i8", got) == (0, -1)
    assert cnt == mm.product_count(n, 4) == 44739243 <= lemma_row(4, n)[4]      # 27 rounds


def test_radix_refusals():
    import torch
    t = torch.zeros(1100, dtype=torch.int32, device="cuda")
    for s, n in [(4, 0), (4, 5), (4, 48), (32, 16), (32, 1000), (32, 1025)]:
        with pytest.raises(tcuscan.TcuscanError) as e:
            tcuscan.matmulscan_levels(t, t, "i32", n=n, s=s)
        assert e.value.code == tcuscan.ERR_UNSUPPORTED
    for s in (2, 8, 64):
        with pytest.raises(tcuscan.TcuscanError) as e:
            tcuscan.matmulscan_levels(t, t, "i32", n=64, s=s)
        assert e.value.code == tcuscan.ERR_UNSUPPORTED
