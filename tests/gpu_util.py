"""Helpers for the GPU parity tests: move seeded host inputs to the GPU, call the C-ABI through
the binding, bring the result back.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np


def to_device(x: np.ndarray, kind: str):
    import torch
    if kind == "bf16":
        return torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def out_dtype(kind: str):
    import torch
    return torch.int32 if kind in ("i32", "i8") else torch.float32


def run_scan(x: np.ndarray, kind: str, call: str = "inclusive", rows: int | None = None, cols: int | None = None,
             ws=None, in_offset: int = 0, out_offset: int = 0, inplace: bool = False):
    """Run one library call and return the output as a numpy array (int32 or float32).

    in_offset / out_offset shift the device pointers by that many ELEMENTS to produce
    buffers that are not 16-byte aligned."""
    import torch
    from paper_2411_17887_amd import tcuscan
    n = x.size
    if rows is None:
        rows, cols = 1, n
    if in_offset:
        pad = np.zeros(in_offset, dtype=x.dtype)
        d_in_full = to_device(np.concatenate([pad, x.reshape(-1)]), kind)
        d_in = d_in_full[in_offset:]
    else:
        d_in = to_device(x.reshape(-1), kind)
    if inplace:
        d_out = d_in.view(out_dtype(kind)) if kind == "i32" else d_in
    else:
        d_out_full = torch.full((n + out_offset + 8,), -77, dtype=out_dtype(kind), device="cuda")
        d_out = d_out_full[out_offset:out_offset + n]
    own_ws = ws is None
    if own_ws:
        ws = tcuscan.new_workspace(rows, cols, kind)
    if call == "inclusive":
        tcuscan.inclusive(d_in, d_out, kind, ws=ws, n=n)
    elif call == "exclusive":
        tcuscan.exclusive(d_in, d_out, kind, ws=ws, n=n)
    elif call == "batched":
        tcuscan.batched(d_in, d_out, rows, cols, kind, exclusive_scan=False, ws=ws)
    elif call == "batched_exclusive":
        tcuscan.batched(d_in, d_out, rows, cols, kind, exclusive_scan=True, ws=ws)
    elif call == "reverse":
        tcuscan.scan(d_in, d_out, rows, cols, kind, flags=tcuscan.REVERSE, ws=ws)
    elif call == "reverse_exclusive":
        tcuscan.scan(d_in, d_out, rows, cols, kind, flags=tcuscan.REVERSE | tcuscan.EXCLUSIVE, ws=ws)
    elif call == "scan_flags0":
        tcuscan.scan(d_in, d_out, rows, cols, kind, flags=0, ws=ws)
    else:
        raise ValueError(call)
    torch.cuda.synchronize()
    if ws is not None:
        assert tcuscan.workspace_fault(ws) == 0, "carry chain hit its spin bound"
    if not inplace:
        # guard words around the output must be untouched
        assert int((d_out_full[:out_offset] != -77).sum()) == 0 and int((d_out_full[out_offset + n:] != -77).sum()) == 0
    return d_out.cpu().numpy().copy()
