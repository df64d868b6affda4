"""Binding of libdlrm_ceilings.so: plain memory kernels of known traffic that a benchmark times to
learn what the board sustains per access pattern (include/dlrm_ceilings.h).  Not part of the method."""
from __future__ import annotations

import ctypes as C
import os

import torch

from . import build as _build
from .binding import _check, _ptr, _stream

_lib = None


def lib() -> C.CDLL:
    """Loads the built library; builds it only if nothing is built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.CEIL_LIB):
            _build.build(force=True)
        L = C.CDLL(_build.CEIL_LIB)
        vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        L.dlrm_ceiling_sink_floats.restype = i32
        L.dlrm_ceiling_sink_floats.argtypes = []
        L.dlrm_ceiling_copy.restype = i32
        L.dlrm_ceiling_copy.argtypes = [vp, vp, sz, vp]
        L.dlrm_ceiling_read.restype = i32
        L.dlrm_ceiling_read.argtypes = [vp, sz, vp, vp]
        L.dlrm_ceiling_gather.restype = i32
        L.dlrm_ceiling_gather.argtypes = [vp, vp, i64, i32, vp, vp]
        L.dlrm_ceiling_rmw.restype = i32
        L.dlrm_ceiling_rmw.argtypes = [vp, vp, i64, i32, vp]
        _lib = L
    return _lib


def _nbytes(t: torch.Tensor) -> int:
    assert t.is_contiguous()
    return t.numel() * t.element_size()


def ceiling_sink() -> torch.Tensor:
    """Scratch output of the read-only measurement kernels."""
    return torch.empty(int(lib().dlrm_ceiling_sink_floats()), dtype=torch.float32, device="cuda")


def dlrm_ceiling_copy(src: torch.Tensor, dst: torch.Tensor):
    assert _nbytes(src) == _nbytes(dst)
    _check("dlrm_ceiling_copy", lib().dlrm_ceiling_copy(_ptr(src), _ptr(dst), _nbytes(src), _stream()))


def dlrm_ceiling_read(src: torch.Tensor, sink: torch.Tensor):
    assert sink.dtype == torch.float32 and sink.numel() >= int(lib().dlrm_ceiling_sink_floats())
    _check("dlrm_ceiling_read", lib().dlrm_ceiling_read(_ptr(src), _nbytes(src), _ptr(sink), _stream()))


def _rows_arg(table: torch.Tensor, rows: torch.Tensor, row_bytes: int) -> int:
    # row numbers as uint32 bit patterns in an int32 tensor; the caller keeps them below the row count
    assert rows.dtype == torch.int32 and rows.is_contiguous() and rows.numel() >= 1
    assert _nbytes(table) % row_bytes == 0
    return rows.numel()


def dlrm_ceiling_gather(table: torch.Tensor, rows: torch.Tensor, row_bytes: int, sink: torch.Tensor):
    assert sink.dtype == torch.float32 and sink.numel() >= int(lib().dlrm_ceiling_sink_floats())
    n = _rows_arg(table, rows, row_bytes)
    _check("dlrm_ceiling_gather",
           lib().dlrm_ceiling_gather(_ptr(table), _ptr(rows), n, row_bytes, _ptr(sink), _stream()))


def dlrm_ceiling_rmw(table: torch.Tensor, rows: torch.Tensor, row_bytes: int):
    """Scales the fp32 elements of the listed (distinct) rows by 1 + 2^-10 in place."""
    n = _rows_arg(table, rows, row_bytes)
    _check("dlrm_ceiling_rmw", lib().dlrm_ceiling_rmw(_ptr(table), _ptr(rows), n, row_bytes, _stream()))
