"""ctypes binding of libdct_bench.so: plain streaming kernels that bench.py uses to measure the
achievable HBM rate next to the DCT kernels.  Not part of the method; nothing else loads it."""
from __future__ import annotations

import ctypes
import os

import torch

from . import build as _build

_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(_build.BENCH_LIB):
            _build.build_library(force=False)
        handle = ctypes.CDLL(_build.BENCH_LIB)
        handle.dct_bench_probe_read.restype = ctypes.c_int
        handle.dct_bench_probe_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
        handle.dct_bench_probe_copy.restype = ctypes.c_int
        handle.dct_bench_probe_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        handle.dct_bench_probe_rows.restype = ctypes.c_int
        handle.dct_bench_probe_rows.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p,
                                                ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p]
        _lib = handle
    return _lib


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def probe_read(src: torch.Tensor, sink: torch.Tensor) -> None:
    """Sum `src` (a multiple of 16 bytes) into `sink` (>= 16384 bytes): a read-only pass over src."""
    rc = lib().dct_bench_probe_read(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(), _stream())
    if rc != 0:
        raise RuntimeError(f"dct_bench_probe_read: status {rc}")


def probe_copy(dst: torch.Tensor, src: torch.Tensor) -> None:
    rc = lib().dct_bench_probe_copy(dst.data_ptr(), src.data_ptr(), src.numel() * src.element_size(), _stream())
    if rc != 0:
        raise RuntimeError(f"dct_bench_probe_copy: status {rc}")


def probe_rows(src: torch.Tensor, chunk_bytes: int, dst: torch.Tensor, out_bytes: int, sink: torch.Tensor) -> None:
    """Read `src` in chunks of `chunk_bytes` (one wavefront per chunk, next chunk in flight) and write
    `out_bytes` per chunk to consecutive places of `dst`: the traffic of a row kernel without its work."""
    nbytes = src.numel() * src.element_size()
    chunks = nbytes // chunk_bytes
    if chunks * out_bytes > dst.numel() * dst.element_size():
        raise ValueError("dst too small")
    rc = lib().dct_bench_probe_rows(src.data_ptr(), chunks, chunk_bytes, dst.data_ptr(), out_bytes, sink.data_ptr(),
                                    _stream())
    if rc != 0:
        raise RuntimeError(f"dct_bench_probe_rows: status {rc}")
