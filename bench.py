#!/usr/bin/env python3
"""Benchmark of the MatMulScan hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C5] [--no-others] [--no-cpu] [--apps-only]

A step is one pass of the whole hot path (tile load, MFMA local scans, in-workgroup up-sweep,
carry chain between workgroups, down-sweep add, store) over one batch of seeded synthetic
input that is already resident in HBM.  Prints ONE JSON line.  `value` is G elements/s of the
headline workload; `roofline` prices the scan kernel against the 8 TB/s HBM peak using
algorithmic bytes (input read once + output written once) and, beside it, against the best
plain streaming kernel of the same read : write mix and size measured in the same run
(`ceiling_GBps`, `frac_of_ceiling`: tcuscan_measure_stream, 128-bit loads, non-temporal stores,
no dependencies); `cpu_baseline` is the sequential CPU oracle timed on this host in the same
run, `cpu_all_cores` a chunked scan on one thread per available core (a second host figure,
checked against the oracle here); `others` holds the remaining benchmark configurations, the
five single-row scans of 2^28 elements, the latency of the smallest configuration and the
shapes beyond the hot path, all measured the same way.

Cold inputs: the device has a 256 MB memory-side cache, and an input that is read again before a few times that many
bytes of other data have been READ is served from it in part (the kernels' non-temporal stores do not displace it:
an int8 input of 256 MiB scanned over and over on one buffer runs 10-35 % faster than on rotated buffers).  Every
timed loop here therefore cycles over copies of its input (and as many output buffers) that hold at least
ROTATE_INPUT_BYTES together, so each launch reads its input from HBM; `buffer_pairs` says how many.

Timing: `kernel_ms` is the mean over back-to-back launches between two HIP events on the launch
stream; `kernel_ms_median` / `kernel_ms_min` come from an event pair around every single launch
(the events add a gap, so for kernels of a few microseconds they can exceed the mean).
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2411_17887_amd import inputs, tcuscan  # noqa: E402

PEAK_HBM_GBPS = 8000.0
ROTATE_INPUT_BYTES = 1 << 30          # distinct input bytes a timed loop cycles over: 4 x the memory-side cache
IN_BYTES = {"i32": 4, "f16": 2, "i8": 1, "f32": 4, "bf16": 2}
DESCR = {
    "C2": "C2: inclusive scan, n=2^24, fp16 U[0,1) -> fp32",
    "C3": "C3: exclusive scan, n=2^28, int8 {0,1} mask -> int32",
    "C4": "C4: inclusive scan, n=100,000,007, fp32 N(0,1) -> fp32",
    "C5": "C5: batched row-wise inclusive scan, 4096 x 65536 (2^28 elements), bf16 U[-1,1] -> fp32",
}
# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), scaled by the same counters on a plain
# 1 GiB device copy; the table and the commands are in TRAFFIC_SOURCE.  The figures belong to the kernels they were
# measured on: TRAFFIC_KERNEL_SHA is the hash of the kernel source at that time, and a run on any other source
# reports `traffic: null` instead of a stale number.
MEASURED_TRAFFIC_BYTES = {"C5": 1626986407, "C3": 1358250200, "C4": 805081780, "C2": 101634492}
TRAFFIC_SOURCE = "profiles/scan_kernel_bench_default.md"
TRAFFIC_KERNEL_SHA = "07d2bc2ca91d1b91"
KERNEL_SOURCE = os.path.join(ROOT, "paper_2411_17887_amd", "csrc", "tcuscan.hip")


def kernel_source_sha() -> str:
    with open(KERNEL_SOURCE, "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()[:16]


def pairs_for(input_bytes: int) -> int:
    """Copies of an input a timed loop rotates over so that the copies hold ROTATE_INPUT_BYTES together (at most 32)."""
    return int(max(1, min(32, -(-ROTATE_INPUT_BYTES // max(1, input_bytes)))))


def timed_mean(fn, steps: int, warmup: int = 2) -> float:
    """ms per call: `steps` calls back to back between two events on the current stream."""
    import torch
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def timed_each(fn, m: int):
    """Sorted ms of m single calls, an event pair around each."""
    import torch
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(m + 1)]
    evs[0].record()
    for i in range(m):
        fn(i)
        evs[i + 1].record()
    torch.cuda.synchronize()
    return sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(m))


STREAM_VARIANTS = [u | ntl | runs | res for u in range(6) for ntl in (0, 0x100) for runs in (0, 0x200) for res in (0, 0x400)]
STREAM_VARIANTS += [u | ntl | runs | res | pause for u in (0, 1) for ntl in (0, 0x100) for runs in (0, 0x200) for res in (0, 0x400)
                    for pause in (0x800, 0x1000)]          # a pause of 512 / 2048 cycles between loads and stores
_ceiling_cache = {}


def stream_ceiling(d_ins, d_outs, n: int, in_bytes: int):
    """The best plain streaming kernel with this read : write mix on the same buffers: 4 n bytes written, in_bytes * n
    read (tcuscan_measure_stream, every variant tried).  GB/s counts both directions."""
    out_bytes = (4 * n) // 64 * 64
    key = (out_bytes, in_bytes)
    if key in _ceiling_cache:
        return _ceiling_cache[key]
    pairs = len(d_ins)
    # enough launches per variant for about a millisecond of run time (small configurations would otherwise be noise)
    reps = int(min(200, max(6, 1.0e-3 / (out_bytes * (1 + in_bytes / 4) / 6.0e12))))
    best = None
    for v in STREAM_VARIANTS:
        if in_bytes == 0 and (v & 0x1900):
            continue
        ms = timed_mean(lambda i: tcuscan.measure_stream(d_ins[i % pairs], d_outs[i % pairs], out_bytes, in_bytes, v), reps, 2)
        if best is None or ms < best[0]:
            best = (ms, v)
    ms = timed_mean(lambda i: tcuscan.measure_stream(d_ins[i % pairs], d_outs[i % pairs], out_bytes, in_bytes, best[1]), 3 * reps, 2)
    ms = min(ms, best[0])
    res = {"GBps": out_bytes * (1 + in_bytes / 4) / (ms * 1e-3) / 1e9, "ms": ms, "variant": "0x%03x" % best[1]}
    _ceiling_cache[key] = res
    return res


def device_input(x: np.ndarray, kind: str):
    import torch
    if kind == "bf16":
        return torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(x).cuda()


def launch(cfg, d_in, d_out, ws):
    kind = cfg["kind"]
    if cfg["call"] == "inclusive":
        tcuscan.inclusive(d_in, d_out, kind, ws=ws)
    elif cfg["call"] == "exclusive":
        tcuscan.exclusive(d_in, d_out, kind, ws=ws)
    else:
        tcuscan.batched(d_in, d_out, cfg["rows"], cfg["cols"], kind, ws=ws)


def figures(n: int, kind: str, ms: float, ceiling=None) -> dict:
    nbytes = n * (IN_BYTES[kind] + 4)
    res = {"kernel_ms": ms, "gelems_per_s": n / (ms * 1e-3) / 1e9, "achieved_GBps": nbytes / (ms * 1e-3) / 1e9}
    res["frac_of_peak"] = res["achieved_GBps"] / PEAK_HBM_GBPS
    if ceiling is not None:
        res["ceiling_GBps"] = ceiling["GBps"]
        res["frac_of_ceiling"] = res["achieved_GBps"] / ceiling["GBps"]
        res["ceiling_variant"] = ceiling["variant"]
    return res


def measure(name: str, steps: int, warmup: int, keep_host: bool = False):
    """Times `steps` launches of workload `name`; returns a dict of figures (and the host input)."""
    import torch
    cfg = inputs.CONFIGS[name]
    kind, n = cfg["kind"], cfg["rows"] * cfg["cols"]
    x = inputs.make_config(name)
    out_dt = torch.int32 if kind in ("i32", "i8") else torch.float32
    bytes_per_elem = IN_BYTES[kind] + 4
    pairs = pairs_for(n * IN_BYTES[kind])          # every launch reads its input from HBM, not from the memory-side cache
    d_in0 = device_input(x, kind)
    d_ins = [d_in0] + [d_in0.clone() for _ in range(pairs - 1)]
    d_outs = [torch.empty(n, dtype=out_dt, device="cuda") for _ in range(pairs)]
    ws = tcuscan.new_workspace(cfg["rows"], cfg["cols"], kind)
    for i in range(warmup):
        launch(cfg, d_ins[i % pairs], d_outs[i % pairs], ws)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()                                   # same (current) stream the kernels are launched on
    for i in range(steps):
        launch(cfg, d_ins[i % pairs], d_outs[i % pairs], ws)
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps          # exactly `steps` steps between two synchronisations
    kern_ms = ev0.elapsed_time(ev1) / steps
    if ws is not None and tcuscan.workspace_fault(ws) != 0:
        raise RuntimeError("carry chain fault flag set")
    last = d_outs[(steps - 1) % pairs].cpu().numpy() if keep_host else None
    each = timed_each(lambda i: launch(cfg, d_ins[i % pairs], d_outs[i % pairs], ws), min(steps, 30))
    ceiling = stream_ceiling(d_ins, d_outs, n, IN_BYTES[kind])
    res = {"workload": DESCR.get(name, name), "n": n, "dtype": kind, "bytes_per_elem": bytes_per_elem,
           "ms_per_step": wall_ms, "kernel_ms_median": each[len(each) // 2], "kernel_ms_min": each[0], "buffer_pairs": pairs}
    res.update(figures(n, kind, kern_ms, ceiling))
    res["gelems_per_s"] = n / (wall_ms * 1e-3) / 1e9           # whole-job throughput by the host clock; the roofline uses kernel_ms
    if pairs > 1:
        # for comparison with figures taken the usual way (the same buffers over and over; for C2 eight pairs): part of
        # the input then comes from the memory-side cache, so this is NOT an HBM figure and no headline uses it
        few = 8 if name == "C2" else 1
        warm_ms = timed_mean(lambda i: launch(cfg, d_ins[i % few], d_outs[i % few], ws), steps)
        res["warm_inputs"] = {"buffer_pairs": few, "kernel_ms": warm_ms, "frac_of_peak": n * bytes_per_elem / (warm_ms * 1e-3) / 1e9 / PEAK_HBM_GBPS,
                              "note": "input re-read from the same buffers: partly served by the 256 MB memory-side cache"}
    del d_ins, d_outs, d_in0
    torch.cuda.empty_cache()
    return res, x, last


def measure_shapes(steps: int):
    """Timing-only entries (device-generated seeded data; parity of these shapes is the tests' business): the five
    single-row inclusive scans of 2^28 elements, shapes without a carry chain, short rows, the smallest
    configuration's latency, and the ticket policy's price."""
    import torch
    torch.manual_seed(241117887)
    n = 1 << 28
    raw = torch.randint(0, 2 ** 31 - 1, (n,), dtype=torch.int32, device="cuda")          # 1 GiB of seeded bits
    outs = [torch.empty(n, dtype=torch.int32, device="cuda") for _ in range(2)]

    def views(kind, count):
        """Inputs of `count` elements of `kind` over successive parts of the random bits (as many as fit, see pairs_for),
        made harmless for floating point (no Inf / NaN), and an output buffer for each."""
        k = min(pairs_for(count * IN_BYTES[kind]), (4 * n) // (count * IN_BYTES[kind]))
        xs = []
        for j in range(k):
            if kind == "i8":
                xs.append(raw.view(torch.int8)[j * count:(j + 1) * count])
            elif kind == "i32":
                xs.append(raw[j * count:(j + 1) * count])
            elif kind == "f32":
                xs.append((raw[j * count:(j + 1) * count] & 0x3FFFFFFF | 0x30000000).view(torch.float32))   # exponents 96 .. 127: |x| < 2
            else:
                w = raw.view(torch.int16)[j * count:(j + 1) * count]
                xs.append((w & 0x3FFF | 0x3000).view(torch.float16 if kind == "f16" else torch.bfloat16))
        os_ = [(outs[j % 2] if kind in ("i8", "i32") else outs[j % 2].view(torch.float32))[:count] for j in range(k)]
        return xs, os_

    res = {}
    rows_1 = {}
    for kind in ("f32", "i32", "bf16", "f16", "i8"):
        xs, os_ = views(kind, n)
        ws = tcuscan.new_workspace(1, n, kind)
        ms = timed_mean(lambda i: tcuscan.inclusive(xs[i % len(xs)], os_[i % len(xs)], kind, ws=ws), steps)
        assert tcuscan.workspace_fault(ws) == 0
        rows_1[kind] = figures(n, kind, ms, stream_ceiling(xs, os_, n, IN_BYTES[kind]))
        rows_1[kind]["buffer_pairs"] = len(xs)
        del xs, os_
    res["single_row_2p28"] = {"workload": "inclusive scan of ONE row of 2^28 elements (one carry chain through the whole input)", **rows_1}

    shapes = {}
    for label, kind, rows, cols in (("no_chain_i8_32768x8192", "i8", 32768, 8192), ("no_chain_bf16_32768x8192", "bf16", 32768, 8192),
                                    ("no_chain_f32_16384x8192", "f32", 16384, 8192), ("short_rows_f32_1048576x256", "f32", 1048576, 256),
                                    ("short_rows_i8_262144x1024", "i8", 262144, 1024), ("short_rows_f16_524288x512", "f16", 524288, 512)):
        m = rows * cols
        xs, os_ = views(kind, m)
        ws = tcuscan.new_workspace(rows, cols, kind)
        ms = timed_mean(lambda i: tcuscan.batched(xs[i % len(xs)], os_[i % len(xs)], rows, cols, kind, ws=ws), steps)
        shapes[label] = figures(m, kind, ms, stream_ceiling(xs, os_, m, IN_BYTES[kind]))
        shapes[label]["buffer_pairs"] = len(xs)
        del xs, os_
    res["rows_without_a_chain"] = {"workload": "batched inclusive scans whose rows fit one workgroup tile (8192) or one wavefront", **shapes}

    # C1: n = 4096 int32, one workgroup, no carry chain -- launch latency, not bandwidth
    x, o = raw[:4096], outs[0][:4096]
    each = timed_each(lambda i: tcuscan.inclusive(x, o, "i32"), 200)
    mean_ms = timed_mean(lambda i: tcuscan.inclusive(x, o, "i32"), 1000, 10)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        tcuscan.inclusive(x, o, "i32", stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        tcuscan.inclusive(x, o, "i32", stream=side)
    for _ in range(5):
        g.replay()
    torch.cuda.synchronize()
    replay = timed_each(lambda i: g.replay(), 200)
    g100 = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g100, stream=side):
        for _ in range(100):
            tcuscan.inclusive(x, o, "i32", stream=side)
    g100.replay()
    torch.cuda.synchronize()
    chain = timed_each(lambda i: g100.replay(), 20)
    res["C1_latency"] = {"workload": "C1: inclusive scan, n=4096 int32 (one workgroup, no carry chain): launch latency in microseconds",
                         "us_median_of_200_launches": each[100] * 1e3, "us_min": each[0] * 1e3,
                         "us_mean_back_to_back_1000": mean_ms * 1e3,
                         "us_median_graph_replay_of_one_launch": replay[100] * 1e3,
                         "us_per_launch_in_a_graph_of_100": chain[10] * 1e3 / 100}

    # the ticket policy (tiles drawn from a counter: no reliance on dispatch order) on the C5 shape and one long row
    rows, cols = 4096, 65536
    xs, os_ = views("bf16", n)
    k = len(xs)
    ws = tcuscan.new_workspace(rows, cols, "bf16")
    ws1 = tcuscan.new_workspace(1, n, "bf16")
    tick = {}
    for policy in (0, 1):
        tcuscan.set_chain_policy(policy)
        try:
            tick["index_order" if policy == 0 else "ticket"] = {
                "C5_shape_ms": timed_mean(lambda i: tcuscan.batched(xs[i % k], os_[i % k], rows, cols, "bf16", ws=ws), max(3, steps // 4)),
                "single_row_2p28_bf16_ms": timed_mean(lambda i: tcuscan.inclusive(xs[i % k], os_[i % k], "bf16", ws=ws1), max(3, steps // 4))}
        finally:
            tcuscan.set_chain_policy(0)
    res["chain_policy"] = {"workload": "how tiles are handed to workgroups: by workgroup index (default) or from a ticket counter", **tick}
    # the entry point that allocates nothing (status words in the library's fixed device array) beside the one with a workspace
    res["static_entry"] = {
        "workload": "C5 shape and one bf16 row of 2^28 through tcuscan_scan_static (no workspace argument) and through tcuscan_scan",
        "C5_shape_ms": {"scan_static": timed_mean(lambda i: tcuscan.scan_static(xs[i % k], os_[i % k], rows, cols, "bf16"), max(3, steps // 4)),
                        "scan": timed_mean(lambda i: tcuscan.scan(xs[i % k], os_[i % k], rows, cols, "bf16", ws=ws), max(3, steps // 4))},
        "single_row_2p28_bf16_ms": {"scan_static": timed_mean(lambda i: tcuscan.scan_static(xs[i % k], os_[i % k], 1, n, "bf16"), max(3, steps // 4)),
                                    "scan": timed_mean(lambda i: tcuscan.scan(xs[i % k], os_[i % k], 1, n, "bf16", ws=ws1), max(3, steps // 4))}}
    assert tcuscan.workspace_fault(tcuscan.STATIC_SCRATCH) == 0
    del raw, outs, xs, os_
    torch.cuda.empty_cache()
    return res


def measure_levels(steps: int):
    """Algorithm 1 run literally (one launch per round, 13 rounds at n = 16^7) against the fused kernel, same input."""
    import torch
    n = 1 << 28
    x = inputs.mask_i8(n, inputs.CONFIGS["C3"]["seed"])
    d_in = torch.from_numpy(x).cuda()
    np_ = pairs_for(n)
    d_ins = [d_in] + [d_in.clone() for _ in range(np_ - 1)]         # cold inputs (see the module's note)
    d_out = torch.empty(n, dtype=torch.int32, device="cuda")
    ws = tcuscan.new_workspace(1, n, "i8")
    res = {}
    for name, fn in (("levels", lambda i: tcuscan.matmulscan_levels(d_ins[i % np_], d_out, "i8")),
                     ("fused", lambda i: tcuscan.inclusive(d_ins[i % np_], d_out, "i8", ws=ws))):
        ms = timed_mean(fn, steps)
        res[name] = {"ms": ms, "gelems_per_s": n / (ms * 1e-3) / 1e9}
    res["workload"] = "inclusive scan, n=2^28=16^7, int8 {0,1} -> int32; 'levels' = 13 launches of Algorithm 1's rounds"
    res["fused_speedup"] = res["levels"]["ms"] / res["fused"]["ms"]
    # The fan-in against depth trade-off (Lemma 1: 2 log_s n - 1 rounds): the same executor with s = 4, 16, 32 on the
    # one length all three divide (2^20 = 4^10 = 16^5 = 32^4, where the launches dominate) and on their largest
    # power below 2^28 + 1 (where the strided gathers dominate).
    radices = []
    for s, k in ((4, 10), (16, 5), (32, 4), (4, 14), (16, 7), (32, 5)):
        m = s ** k
        ms = timed_mean(lambda i: tcuscan.matmulscan_levels(d_ins[i % np_], d_out, "i8", n=m, s=s), steps)
        radices.append({"s": s, "n": m, "rounds": 2 * k - 1, "ms": ms, "gelems_per_s": m / (ms * 1e-3) / 1e9})
    res["radices"] = radices
    return res


def measure_variants(steps: int):
    """Reverse scans on the C3 / C5 shapes and segmented scans on two ragged layouts (seeded geometric row lengths)."""
    import torch

    def copies(t):
        """The input and enough copies of it that a timed loop reads cold data (see the module's note)."""
        return [t] + [t.clone() for _ in range(pairs_for(t.numel() * t.element_size()) - 1)]

    def timed(fn):
        return timed_mean(fn, steps)

    res = {}
    n = 1 << 28
    d_in = copies(torch.from_numpy(inputs.mask_i8(n, inputs.CONFIGS["C3"]["seed"])).cuda())
    d_out = torch.empty(n, dtype=torch.int32, device="cuda")
    ws = tcuscan.new_workspace(1, n, "i8")
    ms = timed(lambda i: tcuscan.scan(d_in[i % len(d_in)], d_out, 1, n, "i8", flags=tcuscan.REVERSE | tcuscan.EXCLUSIVE, ws=ws))
    res["reverse_C3_shape"] = {"workload": "exclusive suffix sums, n=2^28, int8 {0,1} -> int32", "ms": ms,
                               "gelems_per_s": n / ms / 1e6, "frac_of_peak": n * 5 / ms / 1e6 / PEAK_HBM_GBPS}
    del d_in, ws
    rows, cols = 4096, 65536
    xb = copies(torch.from_numpy(inputs.bf16_uniform_pm1(rows * cols, 5).view(np.int16)).cuda().view(torch.bfloat16))
    d_of = d_out.view(torch.float32)
    ws = tcuscan.new_workspace(rows, cols, "bf16")
    ms = timed(lambda i: tcuscan.scan(xb[i % len(xb)], d_of, rows, cols, "bf16", flags=tcuscan.REVERSE, ws=ws))
    res["reverse_C5_shape"] = {"workload": "inclusive suffix sums, 4096 x 65536, bf16 -> fp32", "ms": ms,
                               "gelems_per_s": rows * cols / ms / 1e6, "frac_of_peak": rows * cols * 6 / ms / 1e6 / PEAK_HBM_GBPS}
    # segmented: (a) 2^27 bf16 elements in 64 rows cut at seeded random places; (b) 2^26 fp32 elements in rows of
    # geometric length, mean 200 (the length mix of a sparse matrix / a ragged batch), a few empty and a few long ones
    rng = np.random.default_rng(241117887)
    m = 1 << 27
    off = np.concatenate([[0], np.sort(rng.integers(0, m, size=63)), [m]]).astype(np.int64)
    d_off = torch.from_numpy(off).cuda()
    ws = tcuscan.new_segmented_workspace(64, m, "bf16")
    xh = copies(xb[0][:m])                                      # 2^27 elements: 256 MiB, four copies
    ms = timed(lambda i: tcuscan.segmented(xh[i % len(xh)], d_of, d_off, 64, m, "bf16", ws=ws))
    res["segmented_long_rows"] = {"workload": "2^27 bf16 -> fp32 in 64 rows of random lengths", "ms": ms,
                                  "gelems_per_s": m / ms / 1e6, "frac_of_peak": m * 6 / ms / 1e6 / PEAK_HBM_GBPS}
    del xb, xh, ws
    m = 1 << 26
    lens = rng.geometric(1.0 / 200, size=int(m / 199)) - 1
    lens[:: 97] = 0
    lens[:: 1009] = 8000 + 13
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    off = off[off <= m]
    nrows = off.size - 1
    xf = copies(torch.from_numpy(inputs.f32_normal(m, 6)).cuda())
    d_off = torch.from_numpy(off).cuda()
    ws = tcuscan.new_segmented_workspace(nrows, m, "f32")
    ms = timed(lambda i: tcuscan.segmented(xf[i % len(xf)], d_of, d_off, nrows, m, "f32", ws=ws))
    covered = int(off[-1])
    res["segmented_short_rows"] = {"workload": f"{covered} fp32 elements in {nrows} rows, geometric lengths (mean 200), some empty, some of 8013; "
                                               "the range scanned as one row with row-start bits",
                                   "ms": ms, "gelems_per_s": covered / ms / 1e6, "frac_of_peak": covered * 8 / ms / 1e6 / PEAK_HBM_GBPS}
    tcuscan.set_segmented_form(False)
    try:
        ms = timed(lambda i: tcuscan.segmented(xf[i % len(xf)], d_of, d_off, nrows, m, "f32", ws=ws))
        res["segmented_short_rows_own_tiles"] = {"workload": "the same with tiles of its own for every row", "ms": ms,
                                                 "gelems_per_s": covered / ms / 1e6, "frac_of_peak": covered * 8 / ms / 1e6 / PEAK_HBM_GBPS}
    finally:
        tcuscan.set_segmented_form(True)
    # the same length mix on 2^27 bf16 elements (level 0 of the row-start-bits form runs in the lane for 8/16-bit inputs)
    del xf, ws
    m = 1 << 27
    lens = rng.geometric(1.0 / 200, size=int(m / 199)) - 1
    lens[:: 97] = 0
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    off = off[off <= m]
    nrows = off.size - 1
    covered = int(off[-1])
    xb = copies(torch.from_numpy(inputs.bf16_uniform_pm1(m, 7).view(np.int16)).cuda())
    d_ob = torch.empty(m, dtype=torch.float32, device="cuda")
    d_off = torch.from_numpy(off).cuda()
    ws = tcuscan.new_segmented_workspace(nrows, m, "bf16")
    for name, flat in (("segmented_short_rows_bf16", True), ("segmented_short_rows_bf16_own_tiles", False)):
        tcuscan.set_segmented_form(flat)
        try:
            ms = timed(lambda i: tcuscan.segmented(xb[i % len(xb)], d_ob, d_off, nrows, m, "bf16", ws=ws))
        finally:
            tcuscan.set_segmented_form(True)
        res[name] = {"workload": f"{covered} bf16 -> fp32 elements in {nrows} rows, geometric lengths (mean 200), "
                                 + ("one range with row-start bits" if flat else "tiles of its own for every row"),
                     "ms": ms, "gelems_per_s": covered / ms / 1e6, "frac_of_peak": covered * 6 / ms / 1e6 / PEAK_HBM_GBPS}
    return res


def measure_apps(steps: int):
    """Stream compaction on the C3 mask (n = 2^28) and the 32-pass split radix sort (n = 2^26 random 32-bit keys)."""
    import torch

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    n = 1 << 28
    mask = torch.from_numpy(inputs.mask_i8(n, inputs.CONFIGS["C3"]["seed"])).cuda()
    vals = torch.arange(n, dtype=torch.int32, device="cuda")
    out = torch.empty(n, dtype=torch.int32, device="cuda")
    pos = torch.empty(n, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    ws = tcuscan.new_workspace(1, n, "i8")
    ms = timed(lambda: tcuscan.compact_u32(vals, mask, out, pos, count=cnt, ws=ws), steps)
    kept = int(cnt.item())
    # scan: n + 4n; pack: mask n + positions 4n + values 4n read, 4 * kept written
    nbytes = 5 * n + 9 * n + 4 * kept
    res = {"compaction": {"workload": "n=2^28 int8 {0,1} mask, 32-bit values", "ms": ms, "gelems_per_s": n / (ms * 1e-3) / 1e9,
                          "kept": kept, "algorithmic_GBps": nbytes / (ms * 1e-3) / 1e9}}
    # the same without a positions buffer: the scatter is fused into the scan kernel (mask n + values 4n read, 4 * kept written)
    ms_f = timed(lambda: tcuscan.compact_u32(vals, mask, out, None, count=cnt, ws=ws), steps)
    res["compaction_fused"] = {"workload": "n=2^28 int8 {0,1} mask, 32-bit values, no positions buffer (one kernel)", "ms": ms_f,
                               "gelems_per_s": n / (ms_f * 1e-3) / 1e9, "kept": int(cnt.item()),
                               "algorithmic_GBps": (5 * n + 4 * kept) / (ms_f * 1e-3) / 1e9}
    del vals, out, pos, mask
    torch.cuda.empty_cache()
    m = 1 << 26
    keys0 = torch.from_numpy(inputs.int32_full(m, 12345)).cuda()
    keys = torch.empty_like(keys0)
    tmp, flags, p2 = torch.empty_like(keys0), torch.empty(m, dtype=torch.int8, device="cuda"), torch.empty_like(keys0)
    ws2 = tcuscan.new_workspace(1, m, "i8")

    def sort_once():
        keys.copy_(keys0)
        tcuscan.split_radix_sort_u32(keys, tmp, flags, p2, bits=32, ws=ws2)
    def is_sorted():
        k = keys.view(torch.int32).to(torch.int64) & 0xFFFFFFFF
        return bool((k[1:] >= k[:-1]).all().item())

    ms2 = timed(sort_once, max(2, steps // 2))
    res["split_radix_sort"] = {"workload": "n=2^26 random 32-bit keys, 16 fused split passes on two bits each (flags from the keys, MFMA "
                                           "scans, scatter: one kernel per pass), includes one 256 MiB copy per run",
                               "ms": ms2, "mkeys_per_s": m / (ms2 * 1e-3) / 1e6, "sorted": is_sorted()}
    try:
        tcuscan.set_sort_fusion(2)
        ms1 = timed(sort_once, max(2, steps // 2))
        res["split_radix_sort_one_bit"] = {"workload": "the same with 32 fused split passes on one bit each",
                                           "ms": ms1, "mkeys_per_s": m / (ms1 * 1e-3) / 1e6, "sorted": is_sorted()}
        tcuscan.set_sort_fusion(0)
        ms3 = timed(sort_once, max(2, steps // 2))
        res["split_radix_sort_three_kernels"] = {"workload": "the same with mask kernel + tcuscan_exclusive + scatter kernel per bit",
                                                 "ms": ms3, "mkeys_per_s": m / (ms3 * 1e-3) / 1e6, "sorted": is_sorted()}
    finally:
        tcuscan.set_sort_fusion(1)
    return res


def copy_ceiling_gbps() -> float:
    """A plain device-to-device copy of 1 GiB (read + write counted): calibrates the HBM byte counters of rocprofv3."""
    import torch
    a = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    b = torch.empty_like(a)
    for _ in range(3):
        b.copy_(a)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        b.copy_(a)
    e1.record()
    torch.cuda.synchronize()
    return 2 * a.numel() * 4 / (e0.elapsed_time(e1) / 10 * 1e-3) / 1e9


def cpu_baseline(name: str, x: np.ndarray, gpu_out):
    """The sequential oracle as it stands, one core, on the same workload; also used to check the GPU output."""
    import oracle
    cfg = inputs.CONFIGS[name]
    kind, rows, cols = cfg["kind"], cfg["rows"], cfg["cols"]
    excl = cfg["call"] == "exclusive"
    n = rows * cols
    is_int = kind in ("i32", "i8")
    out = np.zeros(n, dtype=np.int32 if is_int else np.float32)      # pre-faulted
    best = float("inf")
    for _ in range(3):
        t0 = time.perf_counter()
        if is_int:
            oracle.scan_int_into(x, kind, out, exclusive=excl, rows=rows, cols=cols)
        else:
            oracle.scan_to_f32(x, kind, out, exclusive=excl, rows=rows, cols=cols)
        best = min(best, time.perf_counter() - t0)
    parity = None
    if gpu_out is not None:
        if is_int:
            nb, _ = oracle.compare_int(x, kind, gpu_out, exclusive=excl, rows=rows, cols=cols)
            parity = {"bit_exact": nb == 0}
        else:
            rep = oracle.compare_float(x, kind, gpu_out, exclusive=excl, rows=rows, cols=cols)
            parity = {"E1": rep.e1, "tol": cfg["tol"], "ok": rep.ok(cfg["tol"])}
    return {"value": n / best / 1e9, "unit": "G elements/s", "cores": 1, "kind": "oracle",
            "sample": f"full workload ({n} elements), best of 3 passes, {best * 1e3:.0f} ms per pass",
            "ms": best * 1e3}, parity


def cpu_all_cores(name: str, x: np.ndarray):
    """The usual multi-thread host scan (rows dealt to threads, or chunk sums / offsets / chunk scans), one thread per
    available core, on the same workload; its output is checked against the oracle."""
    import oracle
    import hostbaseline as host_threads
    cfg = inputs.CONFIGS[name]
    kind, rows, cols = cfg["kind"], cfg["rows"], cfg["cols"]
    excl = cfg["call"] == "exclusive"
    n = rows * cols
    is_int = kind in ("i32", "i8")
    out = np.zeros(n, dtype=np.int32 if is_int else np.float32)      # pre-faulted
    cores = host_threads.available()
    best = float("inf")
    for _ in range(3):
        t0 = time.perf_counter()
        host_threads.scan_into(x, kind, out, exclusive=excl, rows=rows, cols=cols, threads=cores)
        best = min(best, time.perf_counter() - t0)
    if is_int:
        ok = oracle.compare_int(x, kind, out, exclusive=excl, rows=rows, cols=cols)[0] == 0
    else:
        ok = oracle.compare_float(x, kind, out, exclusive=excl, rows=rows, cols=cols).ok(cfg["tol"])
    return {"value": n / best / 1e9, "unit": "G elements/s", "cores": cores, "kind": "chunked scan, one thread per core",
            "sample": f"full workload ({n} elements), best of 3 passes, {best * 1e3:.0f} ms per pass", "matches_oracle": bool(ok)}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C5", choices=["C2", "C3", "C4", "C5"])
    ap.add_argument("--no-others", action="store_true", help="measure only the headline workload")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--copy-only", action="store_true",
                    help="run only the plain 1 GiB device copy (calibrates the HBM byte counters of rocprofv3 --pmc)")
    ap.add_argument("--apps-only", action="store_true",
                    help="run only the compaction and split-radix-sort measurements (for rocprofv3 counter passes over their kernels)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU by design (the scan shards with one 8-byte exchange per GPU, "
              "which is not built); run with --gpus 1", file=sys.stderr)
        return 2
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    tcuscan.load()
    if args.copy_only:
        print(json.dumps({"copy_GBps": copy_ceiling_gbps(), "bytes_read": 1 << 30, "bytes_written": 1 << 30}))
        return 0

    if args.apps_only:
        print(json.dumps(measure_apps(8)))
        return 0

    head, x, last = measure(args.workload, args.steps, args.warmup, keep_host=not args.no_cpu)
    cpu, parity = (None, None) if args.no_cpu else cpu_baseline(args.workload, x, last)
    cpu_all = None if args.no_cpu else cpu_all_cores(args.workload, x)
    del x, last
    others = {}
    if not args.no_others:
        keep = ("workload", "kernel_ms", "kernel_ms_median", "kernel_ms_min", "gelems_per_s", "achieved_GBps", "frac_of_peak",
                "ceiling_GBps", "frac_of_ceiling", "ceiling_variant", "buffer_pairs")
        for name in ["C2", "C3", "C4", "C5"]:
            if name == args.workload:
                continue
            r, _, _ = measure(name, max(10, args.steps // 2), args.warmup)
            others[name] = {k: r[k] for k in keep + ("warm_inputs",) if k in r}
        others.update(measure_shapes(max(10, args.steps // 2)))
        others["algorithm1_round_by_round"] = measure_levels(5)
        others.update(measure_apps(5))
        others.update(measure_variants(10))

    sha = kernel_source_sha()
    traffic = MEASURED_TRAFFIC_BYTES.get(args.workload) if sha == TRAFFIC_KERNEL_SHA else None
    line = {
        "metric": "G elements/s (and fraction of peak HBM bandwidth in roofline.frac), inclusive scan of 2^28 elements, 1x MI355X",
        "value": head["gelems_per_s"], "unit": "G elements/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"bf16": "bf16->f32", "f16": "f16->f32", "i8": "i8->i32", "f32": "f32", "i32": "i32"}[head["dtype"]],
        "data": "synthetic (seeded SplitMix64 streams, resident in HBM before timing)",
        "config": {"workload": head["workload"], "n": head["n"], "buffer_pairs_rotated": head["buffer_pairs"]},
        "roofline": {"bound": "hbm", "achieved": head["achieved_GBps"], "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                     "frac": head["frac_of_peak"], "traffic": traffic,
                     "traffic_source": (f"{TRAFFIC_SOURCE} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, measured on kernel source {TRAFFIC_KERNEL_SHA})"
                                        if traffic is not None else
                                        f"none for kernel source {sha}: the stored figures were measured on {TRAFFIC_KERNEL_SHA} ({TRAFFIC_SOURCE})"),
                     "kernel": "scan_kernel", "kernel_ms": head["kernel_ms"],
                     "kernel_ms_median": head["kernel_ms_median"], "kernel_ms_min": head["kernel_ms_min"],
                     "timing": "kernel_ms: mean of back-to-back launches between two HIP events on the launch stream; median / min: an "
                               "event pair around every launch",
                     "algorithmic_bytes_per_elem": head["bytes_per_elem"],
                     "ceiling_GBps": head["ceiling_GBps"], "frac_of_ceiling": head["frac_of_ceiling"],
                     "ceiling": "best tcuscan_measure_stream variant (" + head["ceiling_variant"] + ") with the same read:write mix, "
                                "byte count and buffers, same run",
                     "cold_inputs": "every launch of the timed loop reads another copy of the input (config.buffer_pairs_rotated), so "
                                    "none of it comes from the 256 MB memory-side cache",
                     **({"warm_inputs": head["warm_inputs"]} if "warm_inputs" in head else {})},
        "cpu_baseline": cpu,
        "cpu_all_cores": cpu_all,
        "parity_of_timed_output": parity,
        "others": others,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
