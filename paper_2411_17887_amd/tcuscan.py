"""ctypes binding of libtcuscan.so -- argument marshalling only.

Same names as the C entry points in ``include/tcuscan.h``.  Tensors are torch CUDA tensors
(PyTorch is used for device memory and streams, nothing else); every step of the scan runs in
the HIP kernels.  There is no CPU fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtcuscan.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = 0, 1, 2, 3, 4
I32_I32, F16_F32, I8_I32, F32_F32, BF16_F32 = 0, 1, 2, 3, 4
DTYPES = {"i32": I32_I32, "f16": F16_F32, "i8": I8_I32, "f32": F32_F32, "bf16": BF16_F32}

EXPORTS = ["tcuscan_workspace_bytes", "tcuscan_workspace_init", "tcuscan_inclusive", "tcuscan_exclusive",
           "tcuscan_batched", "tcuscan_scan", "tcuscan_segmented_workspace_bytes", "tcuscan_segmented", "tcuscan_tile_elems", "tcuscan_large_tile_elems", "tcuscan_huge_tile_elems",
           "tcuscan_set_tile_policy", "tcuscan_set_segmented_form",
           "tcuscan_workspace_fault", "tcuscan_matmulscan_levels", "tcuscan_matmulscan_levels_radix", "tcuscan_compact_u32",
           "tcuscan_split_radix_sort_u32", "tcuscan_set_sort_fusion", "tcuscan_status_string",
           "tcuscan_set_chain_policy", "tcuscan_scan_static", "tcuscan_path_for", "tcuscan_measure_stream",
           "tcuscan_test_advance_calls", "tcuscan_test_tag_period", "tcuscan_test_chain_fault"]

_lib = None


class TcuscanError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {status_string(code)} (status {code})")


def load() -> ctypes.CDLL:
    """Load the built library.  Building is a separate step (``python -m paper_2411_17887_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} not built; run `python -m paper_2411_17887_amd.build` (hipcc, gfx950)")
        # PyTorch ships its own HIP runtime; it must be the one already mapped when this library's
        # dependency on libamdhip64 is resolved, or the process ends up with two runtimes that do not
        # know each other's streams and allocations.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        L.tcuscan_workspace_bytes.argtypes = [sz, sz, ci]
        L.tcuscan_workspace_bytes.restype = sz
        L.tcuscan_tile_elems.argtypes = [ci]
        L.tcuscan_tile_elems.restype = sz
        L.tcuscan_large_tile_elems.argtypes = [ci]
        L.tcuscan_large_tile_elems.restype = sz
        L.tcuscan_huge_tile_elems.argtypes = [ci]
        L.tcuscan_huge_tile_elems.restype = sz
        L.tcuscan_set_tile_policy.argtypes = [ci]
        L.tcuscan_set_tile_policy.restype = ci
        L.tcuscan_set_sort_fusion.argtypes = [ci]
        L.tcuscan_set_sort_fusion.restype = ci
        L.tcuscan_set_segmented_form.argtypes = [ci]
        L.tcuscan_set_segmented_form.restype = ci
        L.tcuscan_workspace_init.argtypes = [vp, sz, vp]
        L.tcuscan_inclusive.argtypes = [vp, vp, sz, ci, vp, sz, vp]
        L.tcuscan_exclusive.argtypes = [vp, vp, sz, ci, vp, sz, vp]
        L.tcuscan_batched.argtypes = [vp, vp, sz, sz, ci, ci, vp, sz, vp]
        L.tcuscan_scan.argtypes = [vp, vp, sz, sz, ci, ctypes.c_uint, vp, sz, vp]
        L.tcuscan_segmented_workspace_bytes.argtypes = [sz, sz, ci]
        L.tcuscan_segmented_workspace_bytes.restype = sz
        L.tcuscan_segmented.argtypes = [vp, vp, vp, sz, sz, ci, ctypes.c_uint, vp, sz, vp]
        L.tcuscan_workspace_fault.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_uint)]
        L.tcuscan_matmulscan_levels.argtypes = [vp, vp, sz, ci, ci, vp, vp]
        L.tcuscan_matmulscan_levels_radix.argtypes = [vp, vp, sz, ci, ci, ci, vp, vp]
        L.tcuscan_compact_u32.argtypes = [vp, vp, vp, sz, vp, vp, vp, sz, vp]
        L.tcuscan_split_radix_sort_u32.argtypes = [vp, vp, sz, ci, vp, vp, vp, vp, vp, sz, vp]
        L.tcuscan_set_chain_policy.argtypes = [ci]
        L.tcuscan_set_chain_policy.restype = ci
        L.tcuscan_scan_static.argtypes = [vp, vp, sz, sz, ci, ctypes.c_uint, vp]
        L.tcuscan_scan_static.restype = ci
        L.tcuscan_path_for.argtypes = [vp, sz, sz, ci, sz]
        L.tcuscan_path_for.restype = ci
        L.tcuscan_measure_stream.argtypes = [vp, vp, sz, ci, ctypes.c_uint, vp]
        L.tcuscan_measure_stream.restype = ci
        L.tcuscan_test_advance_calls.argtypes = [ctypes.c_ulonglong]
        L.tcuscan_test_advance_calls.restype = ci
        L.tcuscan_test_tag_period.argtypes = []
        L.tcuscan_test_tag_period.restype = ctypes.c_ulonglong
        L.tcuscan_test_chain_fault.argtypes = [ctypes.c_uint, ctypes.c_longlong]
        L.tcuscan_test_chain_fault.restype = ci
        L.tcuscan_status_string.argtypes = [ci]
        L.tcuscan_status_string.restype = ctypes.c_char_p
        for f in ("tcuscan_workspace_init", "tcuscan_inclusive", "tcuscan_exclusive", "tcuscan_batched", "tcuscan_scan", "tcuscan_segmented",
                  "tcuscan_workspace_fault", "tcuscan_matmulscan_levels", "tcuscan_matmulscan_levels_radix",
                  "tcuscan_compact_u32", "tcuscan_split_radix_sort_u32"):
            getattr(L, f).restype = ci
        _lib = L
    return _lib


def status_string(code: int) -> str:
    return load().tcuscan_status_string(int(code)).decode()


def _dt(dt) -> int:
    return DTYPES[dt] if isinstance(dt, str) else int(dt)


def workspace_bytes(rows: int, cols: int, dt) -> int:
    return int(load().tcuscan_workspace_bytes(rows, cols, _dt(dt)))


def tile_elems(dt) -> int:
    return int(load().tcuscan_tile_elems(_dt(dt)))


def large_tile_elems(dt) -> int:
    return int(load().tcuscan_large_tile_elems(_dt(dt)))


def huge_tile_elems(dt) -> int:
    return int(load().tcuscan_huge_tile_elems(_dt(dt)))


TILE_AUTO, TILE_SMALL, TILE_LARGE, TILE_HUGE = 0, 1, 2, 3


def set_tile_policy(policy: int) -> None:
    rc = load().tcuscan_set_tile_policy(int(policy))
    if rc != OK:
        raise TcuscanError(rc, "tcuscan_set_tile_policy")


def _stream(stream) -> int:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return int(getattr(stream, "cuda_stream", stream))


def _ptr(t) -> int:
    return 0 if t is None else int(t.data_ptr())


def _ws_args(ws):
    return (_ptr(ws), 0 if ws is None else ws.numel() * ws.element_size())


def new_workspace(rows: int, cols: int, dt, device="cuda"):
    """Allocate and zero a workspace tensor (None when the shape needs none)."""
    import torch
    nbytes = workspace_bytes(rows, cols, dt)
    if nbytes == 0:
        return None
    return torch.zeros((nbytes + 7) // 8, dtype=torch.int64, device=device)


def workspace_init(ws, stream=None) -> None:
    p, nb = _ws_args(ws)
    rc = load().tcuscan_workspace_init(p, nb, _stream(stream))
    if rc != OK:
        raise TcuscanError(rc, "tcuscan_workspace_init")


def inclusive(x, out, dt, ws=None, stream=None, n=None) -> None:
    rc = load().tcuscan_inclusive(_ptr(x), _ptr(out), x.numel() if n is None else n, _dt(dt), *_ws_args(ws), _stream(stream))
    if rc != OK:
        raise TcuscanError(rc, "tcuscan_inclusive")


def exclusive(x, out, dt, ws=None, stream=None, n=None) -> None:
    rc = load().tcuscan_exclusive(_ptr(x), _ptr(out), x.numel() if n is None else n, _dt(dt), *_ws_args(ws), _stream(stream))
    if rc != OK:
        raise TcuscanError(rc, "tcuscan_exclusive")


def batched(x, out, rows: int, cols: int, dt, exclusive_scan: bool = False, ws=None, stream=None) -> None:
    rc = load().tcuscan_batched(_ptr(x), _ptr(out), rows, cols, _dt(dt), int(bool(exclusive_scan)), *_ws_args(ws),
                                _stream(stream))
    if rc != OK:
        raise TcuscanError(rc, "tcuscan_batched")


EXCLUSIVE, REVERSE = 1, 2      # flag bits of tcuscan_scan


def scan(x, out, rows: int, cols: int, dt, flags: int = 0, ws=None, stream=None) -> None:
    """Row-wise scans with option flags (EXCLUSIVE, REVERSE = suffix sums)."""
    rc = load().tcuscan_scan(_ptr(x), _ptr(out), rows, cols, _dt(dt), int(flags), *_ws_args(ws), _stream(stream))
    if rc != OK:
        raise TcuscanError(rc, "tcuscan_scan")


def segmented_workspace_bytes(rows: int, total: int, dt) -> int:
    return int(load().tcuscan_segmented_workspace_bytes(rows, total, _dt(dt)))


def new_segmented_workspace(rows: int, total: int, dt):
    """A zero-filled workspace for tcuscan_segmented (None when nothing is to be done)."""
    import torch
    nbytes = segmented_workspace_bytes(rows, total, dt)
    return torch.zeros(nbytes // 8 + 1, dtype=torch.int64, device="cuda") if nbytes else None


def segmented(x, out, offsets, rows: int, total: int, dt, flags: int = 0, ws=None, stream=None) -> None:
    """Row-wise scans of rows stored back to back; `offsets`: int64 device tensor of rows + 1 element offsets."""
    rc = load().tcuscan_segmented(_ptr(x), _ptr(out), _ptr(offsets), rows, total, _dt(dt), int(flags), *_ws_args(ws),
                                  _stream(stream))
    if rc != OK:
        raise TcuscanError(rc, "tcuscan_segmented")


def matmulscan_levels(x, out, dt, rounds: int = -1, matmuls=None, stream=None, n=None, s: int = 16) -> None:
    """Algorithm 1 round by round (n = s^k; s = 16 by default, 4 and 32 as well).  `matmuls`: optional int64
    device tensor of one element."""
    n = x.numel() if n is None else n
    if s == 16:
        rc = load().tcuscan_matmulscan_levels(_ptr(x), _ptr(out), n, _dt(dt), int(rounds), _ptr(matmuls), _stream(stream))
    else:
        rc = load().tcuscan_matmulscan_levels_radix(_ptr(x), _ptr(out), n, _dt(dt), int(s), int(rounds), _ptr(matmuls),
                                                    _stream(stream))
    if rc != OK:
        raise TcuscanError(rc, "tcuscan_matmulscan_levels")


def compact_u32(values, mask, out, positions, count=None, ws=None, stream=None) -> None:
    """out <- values[mask != 0] in order; positions (int32, n) is scratch; count: optional 1-element int32 tensor."""
    rc = load().tcuscan_compact_u32(_ptr(values), _ptr(mask), _ptr(out), values.numel(), _ptr(positions), _ptr(count),
                                    *_ws_args(ws), _stream(stream))
    if rc != OK:
        raise TcuscanError(rc, "tcuscan_compact_u32")


def set_segmented_form(flat: bool) -> None:
    load().tcuscan_set_segmented_form(int(bool(flat)))


def set_sort_fusion(form: int) -> None:
    """1: fused split passes on two bits (default); 2: fused passes on one bit; 0: mask kernel + scan + scatter kernel."""
    rc = load().tcuscan_set_sort_fusion(int(form))
    if rc != OK:
        raise TcuscanError(rc, "tcuscan_set_sort_fusion")


def split_radix_sort_u32(keys, keys_tmp, flags, positions, vals=None, vals_tmp=None, bits: int = 32, ws=None, stream=None) -> None:
    """Stable LSD radix sort of 32-bit keys (and optional payloads) by `bits` split passes, one mask scan each."""
    rc = load().tcuscan_split_radix_sort_u32(_ptr(keys), _ptr(vals), keys.numel(), int(bits), _ptr(keys_tmp), _ptr(vals_tmp),
                                             _ptr(flags), _ptr(positions), *_ws_args(ws), _stream(stream))
    if rc != OK:
        raise TcuscanError(rc, "tcuscan_split_radix_sort_u32")


STATIC_SCRATCH = "static"      # workspace_fault(STATIC_SCRATCH): the fixed scratch of scan_static on the current GPU
STATIC_SCRATCH_BYTES = 4194560
PATH_ROWS, PATH_TILES, PATH_TILES_FROM_BOUNDARY, PATH_ELEMENTWISE = 0, 1, 2, 3


def scan_static(x, out, rows: int, cols: int, dt, flags: int = 0, stream=None) -> None:
    """tcuscan_scan without a workspace argument: the library's fixed device scratch is used; allocates nothing."""
    rc = load().tcuscan_scan_static(_ptr(x), _ptr(out), rows, cols, _dt(dt), int(flags), _stream(stream))
    if rc != OK:
        raise TcuscanError(rc, "tcuscan_scan_static")


def path_for(in_ptr: int, rows: int, cols: int, dt, ws_bytes: int) -> int:
    return int(load().tcuscan_path_for(int(in_ptr), rows, cols, _dt(dt), ws_bytes))


def set_chain_policy(policy: int) -> None:
    """0: tiles in workgroup-index order (default); 1: tiles drawn from a ticket counter."""
    rc = load().tcuscan_set_chain_policy(int(policy))
    if rc != OK:
        raise TcuscanError(rc, "tcuscan_set_chain_policy")


def measure_stream(x, out, out_bytes: int, in_bytes_per_out_word: int, variant: int = 0, stream=None) -> None:
    """The streaming yardstick kernel (measurement only)."""
    rc = load().tcuscan_measure_stream(_ptr(x), _ptr(out), out_bytes, int(in_bytes_per_out_word), int(variant), _stream(stream))
    if rc != OK:
        raise TcuscanError(rc, "tcuscan_measure_stream")


def test_advance_calls(calls: int) -> None:
    load().tcuscan_test_advance_calls(int(calls))


def test_tag_period() -> int:
    return int(load().tcuscan_test_tag_period())


def test_chain_fault(spin_limit: int = 0, mute_tile: int = -1) -> None:
    rc = load().tcuscan_test_chain_fault(int(spin_limit), int(mute_tile))
    if rc != OK:
        raise TcuscanError(rc, "tcuscan_test_chain_fault")


def workspace_fault(ws, stream=None) -> int:
    v = ctypes.c_uint(0)
    rc = load().tcuscan_workspace_fault(1 if isinstance(ws, str) and ws == STATIC_SCRATCH else _ptr(ws), _stream(stream), ctypes.byref(v))
    if rc != OK:
        raise TcuscanError(rc, "tcuscan_workspace_fault")
    return int(v.value)
