"""ctypes binding of libdct.so: same names as the C ABI, argument marshalling only.

Tensors must be CUDA (HIP) tensors; kernels are enqueued on torch's current
stream.  There is no CPU fallback: if the library is missing or cannot be
loaded, importing a symbol from it raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import NamedTuple

import torch

from . import build as _build

DCT_OK, DCT_ERR_INVALID, DCT_ERR_WORKSPACE, DCT_ERR_OVERFLOW, DCT_ERR_HIP = range(5)
DCT_F32, DCT_BF16 = 0, 1
DCT_GE_TAU, DCT_EXACT_K = 0, 1
DCT_TAU_KEY_ERROR = 0xFFFFFFFF
DCT_SCATTER_ASSIGN, DCT_SCATTER_ADD = 0, 1
COUNT_WORKSPACE_ERROR = (1 << 64) - 1

_EXPORTS = {
    # name: (restype, argtypes)
    "dct_select_threshold_workspace_bytes": (ctypes.c_size_t, [ctypes.c_int, ctypes.c_uint64]),
    "dct_select_threshold_workspace_bytes_for": (ctypes.c_size_t, [ctypes.c_int, ctypes.c_uint64, ctypes.c_uint64]),
    "dct_select_threshold": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint64,
                                            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "dct_threshold_compact_workspace_bytes": (ctypes.c_size_t, [ctypes.c_int, ctypes.c_uint64]),
    "dct_threshold_compact_workspace_init": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "dct_threshold_compact": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_void_p,
                                             ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64,
                                             ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "dct_threshold_compact_static_scratch_bytes": (ctypes.c_size_t, []),
    "dct_threshold_compact_static": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_void_p,
                                                    ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64,
                                                    ctypes.c_void_p, ctypes.c_void_p]),
    "dct_ef_select_threshold": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64,
                                               ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                               ctypes.c_void_p]),
    "dct_ef_threshold_compact": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                                ctypes.c_uint64, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p,
                                                ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p,
                                                ctypes.c_size_t, ctypes.c_void_p]),
    "dct_rowtopk_fwd": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint32, ctypes.c_uint32,
                                       ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p,
                                       ctypes.c_void_p, ctypes.c_void_p]),
    "dct_rowtopk_bwd": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint32, ctypes.c_uint32,
                                       ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p,
                                       ctypes.c_void_p]),
    "dct_rowtopk_fwd_bitmask": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint32, ctypes.c_uint32,
                                               ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p,
                                               ctypes.c_void_p, ctypes.c_void_p]),
    "dct_rowtopk_bwd_bitmask": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint32, ctypes.c_uint32,
                                               ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p,
                                               ctypes.c_void_p]),
    "dct_rowtopk_scatter_bitmask": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_uint32,
                                                   ctypes.c_uint32, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_uint64,
                                                   ctypes.c_void_p]),
    "dct_rowtopk_fwd_idx16": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint32, ctypes.c_uint32,
                                             ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p,
                                             ctypes.c_void_p, ctypes.c_void_p]),
    "dct_rowtopk_bwd_idx16": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint32, ctypes.c_uint32,
                                             ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p,
                                             ctypes.c_void_p]),
    "dct_rowtopk_scatter_idx16": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_uint32,
                                                 ctypes.c_uint32, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_uint64,
                                                 ctypes.c_void_p]),
    "dct_batched_workspace_bytes": (ctypes.c_size_t, [ctypes.c_int, ctypes.c_void_p, ctypes.c_uint32]),
    "dct_select_threshold_batched": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_uint32,
                                                    ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                                    ctypes.c_void_p]),
    "dct_threshold_compact_batched": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_uint32,
                                                     ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                                     ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                                     ctypes.c_void_p]),
    "dct_scatter": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int,
                                   ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int, ctypes.c_void_p]),
    "dct_rowtopk_scatter": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_uint32,
                                           ctypes.c_uint32, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_uint64,
                                           ctypes.c_void_p]),
    "dct_status_string": (ctypes.c_char_p, [ctypes.c_int]),
    "dct_set_wait_limit": (None, [ctypes.c_uint32]),
}

_lib = None


class DctError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {dct_status_string(status)}")


def lib() -> ctypes.CDLL:
    """Load libdct.so (building it only if no built library is present)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB):
            _build.build_library(force=True)
        handle = ctypes.CDLL(_build.LIB)
        for name, (res, args) in _EXPORTS.items():
            fn = getattr(handle, name)  # AttributeError if the library lacks an entry point
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def dct_status_string(status: int) -> str:
    return lib().dct_status_string(int(status)).decode()


class Threshold(NamedTuple):
    tau_key: int
    n_gt: int
    n_eq: int
    tie_quota: int


def _check(status: int, where: str):
    if status != DCT_OK:
        raise DctError(status, where)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return DCT_F32
    if t.dtype == torch.bfloat16:
        return DCT_BF16
    raise TypeError(f"libdct takes float32 or bfloat16 tensors, got {t.dtype}")


def _dev(t: torch.Tensor, name: str) -> int:
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    return t.data_ptr()


def _flat(t: torch.Tensor, name: str) -> int:
    if t.dim() != 1 or (t.numel() > 1 and t.stride(0) != 1):
        raise ValueError(f"{name} must be a contiguous 1-D tensor")
    return _dev(t, name)


def _rows(t: torch.Tensor, name: str):
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError(f"{name} must be 2-D with unit column stride")
    stride = t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1])
    return _dev(t, name), t.shape[0], t.shape[1], stride


# ------------------------------------------------------------------ workspaces
def dct_select_threshold_workspace_bytes(dt: int, n: int) -> int:
    return lib().dct_select_threshold_workspace_bytes(dt, n)


def dct_threshold_compact_workspace_bytes(dt: int, n: int) -> int:
    return lib().dct_threshold_compact_workspace_bytes(dt, n)


def dct_select_threshold_workspace_bytes_for(dt: int, n: int, k: int) -> int:
    return lib().dct_select_threshold_workspace_bytes_for(dt, n, k)


def new_select_workspace(g: torch.Tensor, k: int | None = None) -> torch.Tensor:
    """Workspace for selections on vectors of g's size: for any k, or (smaller) for this k."""
    nbytes = dct_select_threshold_workspace_bytes(_dt(g), g.numel()) if k is None else \
        dct_select_threshold_workspace_bytes_for(_dt(g), g.numel(), int(k))
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=g.device)


def dct_threshold_compact_workspace_init(ws: torch.Tensor) -> None:
    _check(lib().dct_threshold_compact_workspace_init(_dev(ws, "ws"), ws.numel() * ws.element_size(), _stream()),
           "dct_threshold_compact_workspace_init")


def new_compact_workspace(g: torch.Tensor) -> torch.Tensor:
    nbytes = dct_threshold_compact_workspace_bytes(_dt(g), g.numel())
    ws = torch.empty(max(nbytes, 512), dtype=torch.uint8, device=g.device)
    dct_threshold_compact_workspace_init(ws)
    return ws


# ------------------------------------------------------------------ DCT-DP
def dct_select_threshold(g: torch.Tensor, k: int, thr_out: torch.Tensor, ws: torch.Tensor) -> None:
    """thr_out: int32[4] device tensor receiving {tau_key, n_gt, n_eq, tie_quota}."""
    _check(lib().dct_select_threshold(_flat(g, "g"), _dt(g), g.numel(), int(k), _dev(thr_out, "thr_out"),
                                      _dev(ws, "ws"), ws.numel() * ws.element_size(), _stream()),
           "dct_select_threshold")


def dct_threshold_compact(g: torch.Tensor, thr: torch.Tensor, mode: int, idx_out: torch.Tensor,
                          val_out: torch.Tensor, count_out: torch.Tensor, ws: torch.Tensor,
                          capacity: int | None = None) -> None:
    """idx_out int32[capacity], val_out g.dtype[capacity], count_out int64[1]; all device tensors."""
    cap = min(idx_out.numel(), val_out.numel()) if capacity is None else int(capacity)
    if cap > min(idx_out.numel(), val_out.numel()):
        raise ValueError("capacity exceeds the output tensors")
    if idx_out.dtype != torch.int32 or val_out.dtype != g.dtype or count_out.dtype != torch.int64:
        raise TypeError("idx_out must be int32, val_out must match g, count_out must be int64")
    _check(lib().dct_threshold_compact(_flat(g, "g"), _dt(g), g.numel(), _dev(thr, "thr"), int(mode),
                                       _flat(idx_out, "idx_out") if cap else None,
                                       _flat(val_out, "val_out") if cap else None, cap,
                                       _dev(count_out, "count_out"), _dev(ws, "ws"),
                                       ws.numel() * ws.element_size(), _stream()),
           "dct_threshold_compact")


def dct_threshold_compact_static_scratch_bytes() -> int:
    return lib().dct_threshold_compact_static_scratch_bytes()


def dct_threshold_compact_static(g: torch.Tensor, thr: torch.Tensor, mode: int, idx_out: torch.Tensor,
                                 val_out: torch.Tensor, count_out: torch.Tensor, capacity: int | None = None) -> None:
    """dct_threshold_compact without a workspace argument (the library's static device array serves)."""
    cap = min(idx_out.numel(), val_out.numel()) if capacity is None else int(capacity)
    if cap > min(idx_out.numel(), val_out.numel()):
        raise ValueError("capacity exceeds the output tensors")
    if idx_out.dtype != torch.int32 or val_out.dtype != g.dtype or count_out.dtype != torch.int64:
        raise TypeError("idx_out must be int32, val_out must match g, count_out must be int64")
    _check(lib().dct_threshold_compact_static(_flat(g, "g"), _dt(g), g.numel(), _dev(thr, "thr"), int(mode),
                                              _flat(idx_out, "idx_out") if cap else None,
                                              _flat(val_out, "val_out") if cap else None, cap,
                                              _dev(count_out, "count_out"), _stream()),
           "dct_threshold_compact_static")


def dct_ef_select_threshold(g: torch.Tensor, e: torch.Tensor, k: int, thr_out: torch.Tensor,
                            ws: torch.Tensor) -> None:
    """Threshold of the corrected gradient g + e (float32 tensors of equal length)."""
    if e.dtype != g.dtype or e.numel() != g.numel():
        raise ValueError("e must have the dtype and length of g")
    _check(lib().dct_ef_select_threshold(_flat(g, "g"), _flat(e, "e"), _dt(g), g.numel(), int(k),
                                         _dev(thr_out, "thr_out"), _dev(ws, "ws"), ws.numel() * ws.element_size(),
                                         _stream()),
           "dct_ef_select_threshold")


def dct_ef_threshold_compact(g: torch.Tensor, e_in: torch.Tensor, e_out: torch.Tensor, thr: torch.Tensor, mode: int,
                             idx_out: torch.Tensor, val_out: torch.Tensor, count_out: torch.Tensor,
                             ws: torch.Tensor, capacity: int | None = None) -> None:
    """Survivors of g + e_in and the new residual e_out (which may be e_in itself)."""
    cap = min(idx_out.numel(), val_out.numel()) if capacity is None else int(capacity)
    if cap > min(idx_out.numel(), val_out.numel()):
        raise ValueError("capacity exceeds the output tensors")
    if idx_out.dtype != torch.int32 or val_out.dtype != g.dtype or count_out.dtype != torch.int64:
        raise TypeError("idx_out must be int32, val_out must match g, count_out must be int64")
    if e_in.dtype != g.dtype or e_out.dtype != g.dtype or e_in.numel() != g.numel() or e_out.numel() != g.numel():
        raise ValueError("e_in and e_out must have the dtype and length of g")
    _check(lib().dct_ef_threshold_compact(_flat(g, "g"), _flat(e_in, "e_in"), _flat(e_out, "e_out"), _dt(g),
                                          g.numel(), _dev(thr, "thr"), int(mode),
                                          _flat(idx_out, "idx_out") if cap else None,
                                          _flat(val_out, "val_out") if cap else None, cap,
                                          _dev(count_out, "count_out"), _dev(ws, "ws"),
                                          ws.numel() * ws.element_size(), _stream()),
           "dct_ef_threshold_compact")


def read_threshold(thr: torch.Tensor) -> Threshold:
    """Synchronising host copy of a device dct_threshold; raises if the selection gave up."""
    v = [x & 0xFFFFFFFF for x in thr.cpu().tolist()]
    if v[0] == DCT_TAU_KEY_ERROR:
        raise DctError(DCT_ERR_HIP, "dct_select_threshold (its workgroups did not become resident together: "
                                    "select again)")
    return Threshold(*v)


def read_count(count_out: torch.Tensor, capacity: int | None = None) -> int:
    """Synchronising read of the survivor count; raises on a workspace error or,
    when `capacity` is given, on overflow."""
    c = int(count_out.cpu().item()) & ((1 << 64) - 1)
    if c == COUNT_WORKSPACE_ERROR:
        raise DctError(DCT_ERR_WORKSPACE, "dct_threshold_compact")
    if capacity is not None and c > capacity:
        raise DctError(DCT_ERR_OVERFLOW, f"dct_threshold_compact (count {c} > capacity {capacity})")
    return c


# ------------------------------------------------------------------ DCT-MP
def dct_rowtopk_fwd(x: torch.Tensor, k: int, idx_out: torch.Tensor, val_out: torch.Tensor,
                    tau_out: torch.Tensor | None = None) -> None:
    ptr, B, D, stride = _rows(x, "x")
    if idx_out.dtype != torch.int32 or val_out.dtype != x.dtype or not idx_out.is_contiguous() \
            or not val_out.is_contiguous() or idx_out.numel() != B * k or val_out.numel() != B * k:
        raise ValueError("idx_out / val_out must be contiguous [B, k] int32 / x.dtype tensors")
    if tau_out is not None and (tau_out.dtype != x.dtype or tau_out.numel() != B or not tau_out.is_contiguous()):
        raise ValueError("tau_out must be a contiguous [B] tensor of x.dtype")
    _check(lib().dct_rowtopk_fwd(ptr, _dt(x), B, D, stride, int(k), _dev(idx_out, "idx_out"),
                                 _dev(val_out, "val_out"), _dev(tau_out, "tau_out") if tau_out is not None else None,
                                 _stream()), "dct_rowtopk_fwd")


def dct_rowtopk_bwd(dy: torch.Tensor, idx: torch.Tensor, dval_out: torch.Tensor) -> None:
    ptr, B, D, stride = _rows(dy, "dy")
    if idx.dtype != torch.int32 or idx.dim() != 2 or idx.shape[0] != B or not idx.is_contiguous():
        raise ValueError("idx must be a contiguous int32 [B, k] tensor")
    k = idx.shape[1]
    if dval_out.dtype != dy.dtype or dval_out.numel() != B * k or not dval_out.is_contiguous():
        raise ValueError("dval_out must be a contiguous [B, k] tensor of dy.dtype")
    _check(lib().dct_rowtopk_bwd(ptr, _dt(dy), B, D, stride, k, _dev(idx, "idx"), _dev(dval_out, "dval_out"),
                                 _stream()), "dct_rowtopk_bwd")


# ------------------------------------------------------------------ DCT-MP, the mask as a bitmap
def _mask_ok(mask: torch.Tensor, B: int, D: int) -> None:
    if mask.dtype != torch.int32 or mask.numel() != B * ((D + 31) // 32) or not mask.is_contiguous():
        raise ValueError("mask must be a contiguous int32 [B, ceil(D/32)] tensor")


def dct_rowtopk_fwd_bitmask(x: torch.Tensor, k: int, mask_out: torch.Tensor, val_out: torch.Tensor,
                            tau_out: torch.Tensor | None = None) -> None:
    ptr, B, D, stride = _rows(x, "x")
    _mask_ok(mask_out, B, D)
    if val_out.dtype != x.dtype or not val_out.is_contiguous() or val_out.numel() != B * k:
        raise ValueError("val_out must be a contiguous [B, k] tensor of x.dtype")
    if tau_out is not None and (tau_out.dtype != x.dtype or tau_out.numel() != B or not tau_out.is_contiguous()):
        raise ValueError("tau_out must be a contiguous [B] tensor of x.dtype")
    _check(lib().dct_rowtopk_fwd_bitmask(ptr, _dt(x), B, D, stride, int(k), _dev(mask_out, "mask_out"),
                                         _dev(val_out, "val_out"),
                                         _dev(tau_out, "tau_out") if tau_out is not None else None, _stream()),
           "dct_rowtopk_fwd_bitmask")


def dct_rowtopk_bwd_bitmask(dy: torch.Tensor, mask: torch.Tensor, dval_out: torch.Tensor) -> None:
    ptr, B, D, stride = _rows(dy, "dy")
    _mask_ok(mask, B, D)
    if dval_out.dtype != dy.dtype or dval_out.dim() != 2 or dval_out.shape[0] != B or not dval_out.is_contiguous():
        raise ValueError("dval_out must be a contiguous [B, k] tensor of dy.dtype")
    _check(lib().dct_rowtopk_bwd_bitmask(ptr, _dt(dy), B, D, stride, dval_out.shape[1], _dev(mask, "mask"),
                                         _dev(dval_out, "dval_out"), _stream()), "dct_rowtopk_bwd_bitmask")


def dct_rowtopk_scatter_bitmask(mask: torch.Tensor, val: torch.Tensor, out: torch.Tensor) -> None:
    ptr, B, D, stride = _rows(out, "out")
    _mask_ok(mask, B, D)
    if val.dtype != out.dtype or val.dim() != 2 or val.shape[0] != B or not val.is_contiguous():
        raise ValueError("val must be a contiguous [B, k] tensor of out.dtype")
    _check(lib().dct_rowtopk_scatter_bitmask(_dev(mask, "mask"), _dev(val, "val"), _dt(out), B, D, val.shape[1],
                                             ptr, stride, _stream()), "dct_rowtopk_scatter_bitmask")


# ------------------------------------------------------------------ DCT-DP, many tensors
class Segment(ctypes.Structure):
    """One tensor of a batched call (dct_segment): all fields in elements / slots."""
    _fields_ = [("offset", ctypes.c_uint64), ("n", ctypes.c_uint64), ("k", ctypes.c_uint64),
                ("out_offset", ctypes.c_uint64), ("capacity", ctypes.c_uint64)]


def segment_table(segments):
    """ctypes array of dct_segment from (offset, n, k, out_offset, capacity) tuples."""
    arr = (Segment * len(segments))()
    for i, sgm in enumerate(segments):
        arr[i] = Segment(*(int(v) for v in sgm))
    return arr


def dct_batched_workspace_bytes(dt: int, table) -> int:
    return lib().dct_batched_workspace_bytes(dt, ctypes.cast(table, ctypes.c_void_p), len(table))


def new_batched_workspace(g: torch.Tensor, table) -> torch.Tensor:
    nbytes = dct_batched_workspace_bytes(_dt(g), table)
    if nbytes == 0:
        raise DctError(DCT_ERR_INVALID, "dct_batched_workspace_bytes")
    return torch.empty(nbytes, dtype=torch.uint8, device=g.device)


def dct_select_threshold_batched(g: torch.Tensor, table, thr_out: torch.Tensor, ws: torch.Tensor) -> None:
    """thr_out: int32[n_seg, 4] device tensor; `table` from segment_table()."""
    if thr_out.dtype != torch.int32 or thr_out.numel() != 4 * len(table) or not thr_out.is_contiguous():
        raise ValueError("thr_out must be a contiguous int32 [n_seg, 4] tensor")
    for sgm in table:
        if sgm.offset + sgm.n > g.numel():
            raise ValueError("a segment exceeds g")
    _check(lib().dct_select_threshold_batched(_flat(g, "g"), _dt(g), ctypes.cast(table, ctypes.c_void_p), len(table),
                                              _dev(thr_out, "thr_out"), _dev(ws, "ws"),
                                              ws.numel() * ws.element_size(), _stream()),
           "dct_select_threshold_batched")


def dct_threshold_compact_batched(g: torch.Tensor, table, thr: torch.Tensor, mode: int, idx_out: torch.Tensor,
                                  val_out: torch.Tensor, count_out: torch.Tensor, ws: torch.Tensor) -> None:
    """count_out: int64[n_seg]; every segment's out_offset + capacity must lie inside idx_out / val_out."""
    if idx_out.dtype != torch.int32 or val_out.dtype != g.dtype or count_out.dtype != torch.int64:
        raise TypeError("idx_out must be int32, val_out must match g, count_out must be int64")
    if count_out.numel() != len(table) or thr.numel() != 4 * len(table):
        raise ValueError("count_out / thr must have one entry per segment")
    room = min(idx_out.numel(), val_out.numel())
    for sgm in table:
        if sgm.out_offset + sgm.capacity > room:
            raise ValueError("a segment's output range exceeds the output tensors")
        if sgm.offset + sgm.n > g.numel():
            raise ValueError("a segment exceeds g")
    _check(lib().dct_threshold_compact_batched(_flat(g, "g"), _dt(g), ctypes.cast(table, ctypes.c_void_p), len(table),
                                               _dev(thr, "thr"), int(mode), _flat(idx_out, "idx_out"),
                                               _flat(val_out, "val_out"), _dev(count_out, "count_out"),
                                               _dev(ws, "ws"), ws.numel() * ws.element_size(), _stream()),
           "dct_threshold_compact_batched")


# ------------------------------------------------------------------ receiver side
def dct_scatter(idx: torch.Tensor, val: torch.Tensor, count: torch.Tensor | None, out: torch.Tensor,
                mode: int = DCT_SCATTER_ASSIGN, capacity: int | None = None) -> None:
    """Pairs -> dense vector `out`; `count` is the device int64[1] written by the compaction (or None)."""
    cap = min(idx.numel(), val.numel()) if capacity is None else int(capacity)
    if cap > min(idx.numel(), val.numel()):
        raise ValueError("capacity exceeds the pair tensors")
    if idx.dtype != torch.int32 or val.dtype != out.dtype or (count is not None and count.dtype != torch.int64):
        raise TypeError("idx must be int32, val must match out, count must be int64")
    _check(lib().dct_scatter(_flat(idx, "idx") if cap else None, _flat(val, "val") if cap else None,
                             _dev(count, "count") if count is not None else None, cap, _dt(out),
                             _flat(out, "out"), out.numel(), int(mode), _stream()), "dct_scatter")


def dct_rowtopk_scatter(idx: torch.Tensor, val: torch.Tensor, out: torch.Tensor) -> None:
    """Per-row lists [B, k] -> dense rows of `out` ([B, D], unit column stride)."""
    ptr, B, D, stride = _rows(out, "out")
    if idx.dtype != torch.int32 or idx.dim() != 2 or idx.shape[0] != B or not idx.is_contiguous():
        raise ValueError("idx must be a contiguous int32 [B, k] tensor")
    if val.dtype != out.dtype or val.shape != idx.shape or not val.is_contiguous():
        raise ValueError("val must be a contiguous [B, k] tensor of out.dtype")
    _check(lib().dct_rowtopk_scatter(_dev(idx, "idx"), _dev(val, "val"), _dt(out), B, D, idx.shape[1], ptr, stride,
                                     _stream()), "dct_rowtopk_scatter")


# ------------------------------------------------------------------ DCT-MP, the mask as 16-bit indices
_IDX16 = (torch.uint16, torch.int16)  # both hold the same 16 bits; the library reads them unsigned


def dct_rowtopk_fwd_idx16(x: torch.Tensor, k: int, idx_out: torch.Tensor, val_out: torch.Tensor,
                          tau_out: torch.Tensor | None = None) -> None:
    ptr, B, D, stride = _rows(x, "x")
    if idx_out.dtype not in _IDX16 or val_out.dtype != x.dtype or not idx_out.is_contiguous() \
            or not val_out.is_contiguous() or idx_out.numel() != B * k or val_out.numel() != B * k:
        raise ValueError("idx_out / val_out must be contiguous [B, k] uint16 / x.dtype tensors")
    if tau_out is not None and (tau_out.dtype != x.dtype or tau_out.numel() != B or not tau_out.is_contiguous()):
        raise ValueError("tau_out must be a contiguous [B] tensor of x.dtype")
    _check(lib().dct_rowtopk_fwd_idx16(ptr, _dt(x), B, D, stride, int(k), _dev(idx_out, "idx_out"),
                                       _dev(val_out, "val_out"),
                                       _dev(tau_out, "tau_out") if tau_out is not None else None, _stream()),
           "dct_rowtopk_fwd_idx16")


def dct_rowtopk_bwd_idx16(dy: torch.Tensor, idx: torch.Tensor, dval_out: torch.Tensor) -> None:
    ptr, B, D, stride = _rows(dy, "dy")
    if idx.dtype not in _IDX16 or idx.dim() != 2 or idx.shape[0] != B or not idx.is_contiguous():
        raise ValueError("idx must be a contiguous uint16 [B, k] tensor")
    k = idx.shape[1]
    if dval_out.dtype != dy.dtype or dval_out.numel() != B * k or not dval_out.is_contiguous():
        raise ValueError("dval_out must be a contiguous [B, k] tensor of dy.dtype")
    _check(lib().dct_rowtopk_bwd_idx16(ptr, _dt(dy), B, D, stride, k, _dev(idx, "idx"), _dev(dval_out, "dval_out"),
                                       _stream()), "dct_rowtopk_bwd_idx16")


def dct_rowtopk_scatter_idx16(idx: torch.Tensor, val: torch.Tensor, out: torch.Tensor) -> None:
    ptr, B, D, stride = _rows(out, "out")
    if idx.dtype not in _IDX16 or idx.dim() != 2 or idx.shape[0] != B or not idx.is_contiguous():
        raise ValueError("idx must be a contiguous uint16 [B, k] tensor")
    if val.dtype != out.dtype or val.shape != idx.shape or not val.is_contiguous():
        raise ValueError("val must be a contiguous [B, k] tensor of out.dtype")
    _check(lib().dct_rowtopk_scatter_idx16(_dev(idx, "idx"), _dev(val, "val"), _dt(out), B, D, idx.shape[1], ptr,
                                           stride, _stream()), "dct_rowtopk_scatter_idx16")


# ------------------------------------------------------------------ service
def dct_set_wait_limit(polls: int) -> None:
    """Polls after which a device-side wait gives up (0: the default); for tests of the give-up paths."""
    lib().dct_set_wait_limit(int(polls))
