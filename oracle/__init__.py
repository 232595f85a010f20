"""ctypes front end of the CPU oracle (oracle/dct_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The HIP library and its Python binding never
import this package, and this package never imports them.

Arrays are numpy: float32 for fp32 data, uint16 bit patterns for bf16 data
(`as_numpy` converts a CPU torch tensor without changing a bit).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import NamedTuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dct_oracle.cpp")
_LIB = os.path.join(_HERE, "libdct_oracle.so")

F32, BF16 = 0, 1
GE_TAU, EXACT_K = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (host code only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def build_sanitized(path: str) -> str:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (errors abort), written to `path`.
    A process loads it instead of the plain build when DCT_ORACLE_LIB names it; it needs gcc's libasan
    preloaded (the interpreter is not instrumented)."""
    cmd = ["g++", "-O1", "-g", "-std=c++17", "-shared", "-fPIC", "-Wall", "-Wextra", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-o", path, _SRC]
    subprocess.run(cmd, check=True)
    return path


_lib = None


def _load():
    global _lib
    if _lib is None:
        override = os.environ.get("DCT_ORACLE_LIB")
        if not override:
            build()
        lib = ctypes.CDLL(override or _LIB)
        vp, u64, u32, i32 = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int
        lib.oracle_select_threshold.argtypes = [vp, i32, u64, u64, vp]
        lib.oracle_select_threshold_nth.argtypes = [vp, i32, u64, u64, vp]
        lib.oracle_threshold_compact.argtypes = [vp, i32, u64, vp, i32, vp, vp, u64, vp]
        lib.oracle_rowtopk_fwd.argtypes = [vp, i32, u32, u32, u64, u32, vp, vp, vp]
        lib.oracle_rowtopk_bwd.argtypes = [vp, i32, u32, u32, u64, u32, vp, vp]
        lib.oracle_ef_accumulate.argtypes = [vp, vp, u64, vp]
        lib.oracle_ef_select_threshold.argtypes = [vp, vp, u64, u64, vp]
        lib.oracle_ef_threshold_compact.argtypes = [vp, vp, u64, vp, i32, vp, vp, u64, vp, vp]
        lib.oracle_scatter.argtypes = [vp, vp, u64, i32, u64, vp, i32]
        lib.oracle_rowscatter.argtypes = [vp, vp, i32, u32, u32, u32, vp, u64]
        lib.oracle_scatter.restype = lib.oracle_rowscatter.restype = ctypes.c_int
        lib.oracle_rowtopk_fwd_bitmask.argtypes = [vp, i32, u32, u32, u64, u32, vp, vp, vp]
        lib.oracle_rowtopk_bwd_bitmask.argtypes = [vp, i32, u32, u32, u64, u32, vp, vp]
        lib.oracle_rowscatter_bitmask.argtypes = [vp, vp, i32, u32, u32, u32, vp, u64]
        for f in (lib.oracle_rowtopk_fwd_bitmask, lib.oracle_rowtopk_bwd_bitmask, lib.oracle_rowscatter_bitmask):
            f.restype = ctypes.c_int
        lib.oracle_rowtopk_fwd_idx16.argtypes = [vp, i32, u32, u32, u64, u32, vp, vp, vp]
        lib.oracle_rowtopk_bwd_idx16.argtypes = [vp, i32, u32, u32, u64, u32, vp, vp]
        lib.oracle_rowscatter_idx16.argtypes = [vp, vp, i32, u32, u32, u32, vp, u64]
        for f in (lib.oracle_rowtopk_fwd_idx16, lib.oracle_rowtopk_bwd_idx16, lib.oracle_rowscatter_idx16):
            f.restype = ctypes.c_int
        for f in (lib.oracle_ef_accumulate, lib.oracle_ef_select_threshold, lib.oracle_ef_threshold_compact):
            f.restype = ctypes.c_int
        for f in (lib.oracle_select_threshold, lib.oracle_select_threshold_nth, lib.oracle_threshold_compact,
                  lib.oracle_rowtopk_fwd, lib.oracle_rowtopk_bwd):
            f.restype = ctypes.c_int
        _lib = lib
    return _lib


class Threshold(NamedTuple):
    tau_key: int
    n_gt: int
    n_eq: int
    tie_quota: int


def as_numpy(t):
    """CPU torch tensor (float32 or bfloat16) -> numpy array of the same bits."""
    import torch
    t = t.detach()
    assert t.device.type == "cpu"
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"oracle takes float32 or uint16 (bf16 bits), got {a.dtype}")


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def select_threshold(g: np.ndarray, k: int, method: str = "sort") -> Threshold:
    g = np.ascontiguousarray(g)
    assert g.ndim == 1
    out = np.zeros(4, dtype=np.uint32)
    fn = _load().oracle_select_threshold if method == "sort" else _load().oracle_select_threshold_nth
    rc = fn(_ptr(g), _dtype_code(g), g.size, int(k), _ptr(out))
    if rc != 0:
        raise ValueError("oracle_select_threshold: invalid arguments")
    return Threshold(*(int(v) for v in out))


def threshold_compact(g: np.ndarray, thr: Threshold, mode: int, capacity: int | None = None):
    """Returns (idx int32[min(count, capacity)], val[same], count)."""
    g = np.ascontiguousarray(g)
    assert g.ndim == 1
    cap = g.size if capacity is None else int(capacity)
    idx = np.full(cap, -1, dtype=np.int32)
    val = np.zeros(cap, dtype=g.dtype)
    count = np.zeros(1, dtype=np.uint64)
    t = np.array(list(thr), dtype=np.uint32)
    rc = _load().oracle_threshold_compact(_ptr(g), _dtype_code(g), g.size, _ptr(t), int(mode),
                                          _ptr(idx), _ptr(val), cap, _ptr(count))
    if rc != 0:
        raise ValueError("oracle_threshold_compact: invalid arguments")
    c = int(count[0])
    m = min(c, cap)
    return idx[:m], val[:m], c


def _row_stride(x: np.ndarray) -> int:
    assert x.ndim == 2 and x.strides[1] == x.itemsize and x.strides[0] % x.itemsize == 0
    return x.strides[0] // x.itemsize


def rowtopk_fwd(x: np.ndarray, k: int):
    """x: [B, D] with unit column stride (row stride may exceed D).
    Returns (idx int32[B,k], val[B,k], tau[B])."""
    B, D = x.shape
    idx = np.zeros((B, k), dtype=np.int32)
    val = np.zeros((B, k), dtype=x.dtype)
    tau = np.zeros(B, dtype=x.dtype)
    rc = _load().oracle_rowtopk_fwd(_ptr(x), _dtype_code(x), B, D, _row_stride(x), int(k),
                                    _ptr(idx), _ptr(val), _ptr(tau))
    if rc != 0:
        raise ValueError("oracle_rowtopk_fwd: invalid arguments")
    return idx, val, tau


def rowtopk_bwd(dy: np.ndarray, idx: np.ndarray):
    B, D = dy.shape
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    assert idx.shape[0] == B
    k = idx.shape[1]
    dval = np.zeros((B, k), dtype=dy.dtype)
    rc = _load().oracle_rowtopk_bwd(_ptr(dy), _dtype_code(dy), B, D, _row_stride(dy), k, _ptr(idx), _ptr(dval))
    if rc != 0:
        raise ValueError(f"oracle_rowtopk_bwd: error {rc}")
    return dval


# ---- Algorithm 1 with error feedback (fp32 only) ----------------------------
def _f32_pair(g: np.ndarray, e: np.ndarray):
    g = np.ascontiguousarray(g)
    e = np.ascontiguousarray(e)
    if g.dtype != np.float32 or e.dtype != np.float32:
        raise TypeError("error feedback is defined for float32")
    assert g.ndim == 1 and g.shape == e.shape
    return g, e


def ef_accumulate(g: np.ndarray, e: np.ndarray) -> np.ndarray:
    """w = g + e, one binary32 addition per element."""
    g, e = _f32_pair(g, e)
    w = np.zeros_like(g)
    if _load().oracle_ef_accumulate(_ptr(g), _ptr(e), g.size, _ptr(w)) != 0:
        raise ValueError("oracle_ef_accumulate: invalid arguments")
    return w


def ef_select_threshold(g: np.ndarray, e: np.ndarray, k: int) -> Threshold:
    g, e = _f32_pair(g, e)
    out = np.zeros(4, dtype=np.uint32)
    if _load().oracle_ef_select_threshold(_ptr(g), _ptr(e), g.size, int(k), _ptr(out)) != 0:
        raise ValueError("oracle_ef_select_threshold: invalid arguments")
    return Threshold(*(int(v) for v in out))


def ef_threshold_compact(g: np.ndarray, e: np.ndarray, thr: Threshold, mode: int, capacity: int | None = None):
    """Returns (idx, val, count, e_out): survivors of w = g + e and the new residual."""
    g, e = _f32_pair(g, e)
    cap = g.size if capacity is None else int(capacity)
    idx = np.full(cap, -1, dtype=np.int32)
    val = np.zeros(cap, dtype=np.float32)
    e_out = np.zeros_like(g)
    count = np.zeros(1, dtype=np.uint64)
    t = np.array(list(thr), dtype=np.uint32)
    rc = _load().oracle_ef_threshold_compact(_ptr(g), _ptr(e), g.size, _ptr(t), int(mode), _ptr(idx), _ptr(val),
                                             cap, _ptr(count), _ptr(e_out))
    if rc != 0:
        raise ValueError("oracle_ef_threshold_compact: invalid arguments")
    c = int(count[0])
    m = min(c, cap)
    return idx[:m], val[:m], c, e_out


# ---- receiver side: decompression --------------------------------------------
SCATTER_ASSIGN, SCATTER_ADD = 0, 1


def scatter(idx: np.ndarray, val: np.ndarray, n: int, out: np.ndarray | None = None, mode: int = SCATTER_ASSIGN):
    """Dense vector of n elements from (idx, val) pairs.  ASSIGN ignores the
    contents of `out` (a fresh array if None); ADD updates `out` (float32)."""
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    val = np.ascontiguousarray(val)
    assert idx.shape == val.shape and idx.ndim == 1
    if out is None:
        out = np.full(n, 7, dtype=val.dtype)  # ASSIGN must overwrite every element
    assert out.dtype == val.dtype and out.size == n and out.flags.c_contiguous
    rc = _load().oracle_scatter(_ptr(idx), _ptr(val), idx.size, _dtype_code(val), n, _ptr(out), int(mode))
    if rc != 0:
        raise ValueError("oracle_scatter: invalid arguments")
    return out


def rowscatter(idx: np.ndarray, val: np.ndarray, D: int, out: np.ndarray | None = None):
    """Dense [B, D] matrix from per-row (idx, val) lists; `out` may have a row stride above D."""
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    val = np.ascontiguousarray(val)
    B, k = idx.shape
    assert val.shape == idx.shape
    if out is None:
        out = np.full((B, D), 7, dtype=val.dtype)
    assert out.dtype == val.dtype and out.shape == (B, D)
    rc = _load().oracle_rowscatter(_ptr(idx), _ptr(val), _dtype_code(val), B, D, k, _ptr(out), _row_stride(out))
    if rc != 0:
        raise ValueError("oracle_rowscatter: invalid arguments")
    return out


# ---- Algorithm 2 with the mask as a bitmap ------------------------------------
def rowtopk_fwd_bitmask(x: np.ndarray, k: int):
    """Returns (mask uint32[B, ceil(D/32)], val[B,k], tau[B]); bit c%32 of word c//32 = column c kept."""
    B, D = x.shape
    mask = np.zeros((B, (D + 31) // 32), dtype=np.uint32)
    val = np.zeros((B, k), dtype=x.dtype)
    tau = np.zeros(B, dtype=x.dtype)
    rc = _load().oracle_rowtopk_fwd_bitmask(_ptr(x), _dtype_code(x), B, D, _row_stride(x), int(k),
                                            _ptr(mask), _ptr(val), _ptr(tau))
    if rc != 0:
        raise ValueError("oracle_rowtopk_fwd_bitmask: invalid arguments")
    return mask, val, tau


def rowtopk_bwd_bitmask(dy: np.ndarray, mask: np.ndarray, k: int):
    B, D = dy.shape
    mask = np.ascontiguousarray(mask, dtype=np.uint32)
    assert mask.shape == (B, (D + 31) // 32)
    dval = np.zeros((B, k), dtype=dy.dtype)
    rc = _load().oracle_rowtopk_bwd_bitmask(_ptr(dy), _dtype_code(dy), B, D, _row_stride(dy), int(k), _ptr(mask),
                                            _ptr(dval))
    if rc != 0:
        raise ValueError("oracle_rowtopk_bwd_bitmask: invalid arguments")
    return dval


def rowscatter_bitmask(mask: np.ndarray, val: np.ndarray, D: int):
    mask = np.ascontiguousarray(mask, dtype=np.uint32)
    val = np.ascontiguousarray(val)
    B, k = val.shape
    assert mask.shape == (B, (D + 31) // 32)
    out = np.full((B, D), 7, dtype=val.dtype)
    rc = _load().oracle_rowscatter_bitmask(_ptr(mask), _ptr(val), _dtype_code(val), B, D, k, _ptr(out), D)
    if rc != 0:
        raise ValueError("oracle_rowscatter_bitmask: invalid arguments")
    return out


# ---- Algorithm 2 with the mask as 16-bit column indices -------------------------
def rowtopk_fwd_idx16(x: np.ndarray, k: int):
    """Returns (idx uint16[B,k], val[B,k], tau[B]); rows of at most 65536 columns."""
    B, D = x.shape
    idx = np.zeros((B, k), dtype=np.uint16)
    val = np.zeros((B, k), dtype=x.dtype)
    tau = np.zeros(B, dtype=x.dtype)
    rc = _load().oracle_rowtopk_fwd_idx16(_ptr(x), _dtype_code(x), B, D, _row_stride(x), int(k),
                                          _ptr(idx), _ptr(val), _ptr(tau))
    if rc != 0:
        raise ValueError(f"oracle_rowtopk_fwd_idx16: error {rc}")
    return idx, val, tau


def rowtopk_bwd_idx16(dy: np.ndarray, idx: np.ndarray):
    B, D = dy.shape
    idx = np.ascontiguousarray(idx)
    assert idx.dtype == np.uint16 and idx.shape[0] == B
    k = idx.shape[1]
    dval = np.zeros((B, k), dtype=dy.dtype)
    rc = _load().oracle_rowtopk_bwd_idx16(_ptr(dy), _dtype_code(dy), B, D, _row_stride(dy), k, _ptr(idx), _ptr(dval))
    if rc != 0:
        raise ValueError(f"oracle_rowtopk_bwd_idx16: error {rc}")
    return dval


def rowscatter_idx16(idx: np.ndarray, val: np.ndarray, D: int):
    idx = np.ascontiguousarray(idx)
    val = np.ascontiguousarray(val)
    assert idx.dtype == np.uint16 and val.shape == idx.shape
    B, k = idx.shape
    out = np.full((B, D), 7, dtype=val.dtype)
    rc = _load().oracle_rowscatter_idx16(_ptr(idx), _ptr(val), _dtype_code(val), B, D, k, _ptr(out), D)
    if rc != 0:
        raise ValueError("oracle_rowscatter_idx16: invalid arguments")
    return out
