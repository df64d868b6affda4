"""Thin ctypes binding of libdlrm_hot.so: same names as the C ABI, argument
marshalling only.  torch supplies device memory and the current HIP stream;
every step of the path runs in the library's kernels.  There is no fallback:
if the library is missing or a call fails, an exception is raised."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import torch

from . import build as _build

F32, F16, BF16 = 0, 1, 2
I64, I32 = 0, 1
BWD_AUTO, BWD_SORT, BWD_ATOMIC, BWD_SORT_PREPARED, BWD_SORT_PREPARED_FLAT = 0, 1, 2, 3, 4
FWD_AUTO, FWD_FUSED, FWD_SPLIT = 0, 1, 2
_TORCH_DTYPE = {F32: torch.float32, F16: torch.float16, BF16: torch.bfloat16}
_ELEM = {F32: 4, F16: 2, BF16: 2}


class DlrmError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        super().__init__("%s failed: status %d (%s)" % (fn, status, status_string(status)))


class _BwdTimingC(C.Structure):
    _fields_ = [("ev_start", C.c_void_p), ("ev_stop", C.c_void_p)]


class _SparseBatchC(C.Structure):
    _fields_ = [
        ("K", C.c_int32), ("B", C.c_int32), ("d", C.c_int32), ("table_dtype", C.c_int32),
        ("nnz_total", C.c_int64), ("max_rows", C.c_int64),
        ("tables", C.c_void_p), ("rows", C.c_void_p), ("indices", C.c_void_p),
        ("offsets", C.c_void_p), ("tbl_off", C.c_void_p), ("weights", C.c_void_p),
        ("index_dtype", C.c_int32),
    ]


_lib = None


def lib() -> C.CDLL:
    """Loads the built library; builds it only if nothing is built."""
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build(force=True)
        L = C.CDLL(path)
        vp, i32, i64, f32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_size_t
        sb = C.POINTER(_SparseBatchC)
        L.dlrm_version.restype = i32
        L.dlrm_version.argtypes = []
        L.dlrm_status_string.restype = C.c_char_p
        L.dlrm_status_string.argtypes = [i32]
        L.dlrm_lengths_to_offsets.restype = i32
        L.dlrm_lengths_to_offsets.argtypes = [vp, i32, i32, vp, vp, vp]
        L.dlrm_validate_csr.restype = i32
        L.dlrm_validate_csr.argtypes = [sb, vp, vp]
        L.dlrm_emb_bag_fwd.restype = i32
        L.dlrm_emb_bag_fwd.argtypes = [sb, vp, i64, i64, vp]
        L.dlrm_place_dense.restype = i32
        L.dlrm_place_dense.argtypes = [vp, i32, i32, vp, i32, vp]
        L.dlrm_interact_dot_fwd.restype = i32
        L.dlrm_interact_dot_fwd.argtypes = [vp, i32, i32, i32, vp, vp]
        L.dlrm_emb_interact_fwd.restype = i32
        L.dlrm_emb_interact_fwd.argtypes = [sb, vp, vp, vp, i32, vp]
        L.dlrm_emb_interact_fwd_stamped.restype = i32
        L.dlrm_emb_interact_fwd_stamped.argtypes = [sb, vp, vp, vp, i32, vp, C.c_uint32, vp]
        L.dlrm_emb_interact_bwd.restype = i32
        L.dlrm_emb_interact_bwd.argtypes = [sb, vp, vp, vp, vp]
        L.dlrm_interact_dot_bwd.restype = i32
        L.dlrm_interact_dot_bwd.argtypes = [vp, vp, i32, i32, i32, vp, vp]
        L.dlrm_emb_bag_bwd_workspace_bytes.restype = sz
        L.dlrm_emb_bag_bwd_workspace_bytes.argtypes = [i32, i32, i32, i64, i64, i32]
        L.dlrm_emb_bag_bwd_sgd.restype = i32
        L.dlrm_emb_bag_bwd_sgd.argtypes = [sb, vp, i64, i64, f32, vp, sz, i32, vp]
        L.dlrm_emb_bag_bwd_sgd_noalloc.restype = i32
        L.dlrm_emb_bag_bwd_sgd_noalloc.argtypes = [sb, vp, i64, i64, f32, vp]
        L.dlrm_emb_bag_bwd_adagrad.restype = i32
        L.dlrm_emb_bag_bwd_adagrad.argtypes = [sb, vp, vp, i64, i64, f32, f32, vp, sz, i32, vp]
        L.dlrm_emb_bag_bwd_prepare.restype = i32
        L.dlrm_emb_bag_bwd_prepare.argtypes = [sb, vp, sz, vp]
        L.dlrm_emb_bag_bwd_prepared_oversized.restype = i32
        L.dlrm_emb_bag_bwd_prepared_oversized.argtypes = [sb, vp, sz, vp, vp]
        L.dlrm_emb_bag_bwd_route_counts.restype = i32
        L.dlrm_emb_bag_bwd_route_counts.argtypes = [sb, vp, sz, vp, vp]
        L.dlrm_emb_bag_bwd_export_groups.restype = i32
        L.dlrm_emb_bag_bwd_export_groups.argtypes = [sb, vp, sz, vp, vp, vp, vp, vp]
        L.dlrm_table_init_hash.restype = i32
        L.dlrm_table_init_hash.argtypes = [vp, i64, i32, i32, C.c_uint64, f32, vp]
        tm = C.POINTER(_BwdTimingC)
        L.dlrm_emb_bag_bwd_sgd_timed.restype = i32
        L.dlrm_emb_bag_bwd_sgd_timed.argtypes = [sb, vp, i64, i64, f32, vp, sz, i32, tm, vp]
        L.dlrm_emb_bag_bwd_adagrad_timed.restype = i32
        L.dlrm_emb_bag_bwd_adagrad_timed.argtypes = [sb, vp, vp, i64, i64, f32, f32, vp, sz, i32, tm, vp]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().dlrm_status_string(int(status)).decode()


def version() -> int:
    return int(lib().dlrm_version())


def _check(fn: str, status: int) -> None:
    if status != 0:
        raise DlrmError(fn, status)


def _stream() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


class SparseBatch:
    """Device-side sparse batch: owns the pointer array and keeps the tensors alive."""

    def __init__(self, tables: Sequence[torch.Tensor], table_dtype: int, indices: torch.Tensor,
                 offsets: torch.Tensor, tbl_off: torch.Tensor, nnz_total: int,
                 max_rows: Optional[int] = None, weights: Optional[torch.Tensor] = None):
        self.tables = list(tables)
        K = len(self.tables)
        d = int(self.tables[0].shape[1])
        dev = indices.device if indices.numel() else offsets.device
        for t in self.tables:
            assert t.is_contiguous() and t.dtype == _TORCH_DTYPE[table_dtype] and t.shape[1] == d
        assert offsets.dtype == torch.int64 and offsets.is_contiguous() and offsets.shape[0] == K
        assert indices.dtype in (torch.int64, torch.int32) and tbl_off.dtype == torch.int64
        assert indices.is_contiguous()
        self.K, self.B, self.d = K, int(offsets.shape[1]) - 1, d
        self.table_dtype = table_dtype
        self.indices, self.offsets, self.tbl_off = indices, offsets, tbl_off
        if weights is not None:
            assert weights.dtype == torch.float32 and weights.is_contiguous() and weights.shape == indices.shape
        self.weights = weights
        rows_host = [int(t.shape[0]) for t in self.tables]
        self.rows = torch.tensor(rows_host, dtype=torch.int64, device=dev)
        self.table_ptrs = torch.tensor([t.data_ptr() for t in self.tables], dtype=torch.int64,
                                       device=dev)
        self.nnz_total = int(nnz_total)
        self.max_rows = int(max(rows_host) if max_rows is None else max_rows)
        self.c = _SparseBatchC(K, self.B, d, table_dtype, self.nnz_total, self.max_rows,
                               _ptr(self.table_ptrs), _ptr(self.rows),
                               _ptr(indices) if indices.numel() else None,
                               _ptr(offsets), _ptr(tbl_off),
                               _ptr(weights) if weights is not None and weights.numel() else None,
                               I32 if indices.dtype == torch.int32 else I64)

    def ref(self):
        return C.byref(self.c)


# ------------------------------------------------------------------ the C ABI, one to one
def dlrm_lengths_to_offsets(lengths: torch.Tensor, offsets: torch.Tensor, tbl_off: torch.Tensor):
    K, B = lengths.shape
    assert lengths.dtype == torch.int32 and lengths.is_contiguous()
    _check("dlrm_lengths_to_offsets",
           lib().dlrm_lengths_to_offsets(_ptr(lengths), K, B, _ptr(offsets), _ptr(tbl_off), _stream()))


def dlrm_validate_csr(batch: SparseBatch, n_bad: torch.Tensor):
    _check("dlrm_validate_csr", lib().dlrm_validate_csr(batch.ref(), _ptr(n_bad), _stream()))


def dlrm_emb_bag_fwd(batch: SparseBatch, out: torch.Tensor, stride_b: int, stride_k: int,
                     out_offset: int = 0):
    """out_offset: element offset into `out` (e.g. d, to write rows 1..K of T[B,F,d])."""
    _check("dlrm_emb_bag_fwd",
           lib().dlrm_emb_bag_fwd(batch.ref(), _ptr(out) + 4 * out_offset, stride_b, stride_k,
                                  _stream()))


def dlrm_place_dense(x: torch.Tensor, T: torch.Tensor):
    B, F, d = T.shape
    _check("dlrm_place_dense", lib().dlrm_place_dense(_ptr(x), B, d, _ptr(T), F, _stream()))


def dlrm_interact_dot_fwd(T: torch.Tensor, R: torch.Tensor):
    B, F, d = T.shape
    _check("dlrm_interact_dot_fwd", lib().dlrm_interact_dot_fwd(_ptr(T), B, F, d, _ptr(R), _stream()))


def dlrm_emb_interact_fwd(batch: SparseBatch, x: torch.Tensor, T: torch.Tensor, R: torch.Tensor,
                          algo: int = FWD_AUTO):
    _check("dlrm_emb_interact_fwd",
           lib().dlrm_emb_interact_fwd(batch.ref(), _ptr(x), _ptr(T), _ptr(R), algo, _stream()))


def dlrm_emb_interact_fwd_stamped(batch: SparseBatch, x: torch.Tensor, T: torch.Tensor, R: torch.Tensor,
                                  algo: int, stamp: torch.Tensor, stamp_value: int, index: int = 0):
    """stamp: int32 tensor the device can write (device memory, or host memory allocated pinned);
    element `index` receives stamp_value when the call's first kernel starts."""
    assert stamp.dtype == torch.int32 and (stamp.is_cuda or stamp.is_pinned()) and 0 <= index < stamp.numel()
    _check("dlrm_emb_interact_fwd_stamped",
           lib().dlrm_emb_interact_fwd_stamped(batch.ref(), _ptr(x), _ptr(T), _ptr(R), algo,
                                               _ptr(stamp) + 4 * index, stamp_value & 0xFFFFFFFF, _stream()))


def dlrm_emb_interact_bwd(batch: SparseBatch, x: torch.Tensor, dR: torch.Tensor, dT: torch.Tensor):
    """dT of the interaction with the pooled vectors formed again from the tables (no T)."""
    assert x.dtype == torch.float32 and x.is_contiguous() and x.shape == (batch.B, batch.d)
    F = batch.K + 1
    assert dR.dtype == torch.float32 and dR.is_contiguous() and dR.shape == (batch.B, batch.d + F * (F - 1) // 2)
    assert dT.dtype == torch.float32 and dT.is_contiguous() and dT.shape == (batch.B, F, batch.d)
    _check("dlrm_emb_interact_bwd", lib().dlrm_emb_interact_bwd(batch.ref(), _ptr(x), _ptr(dR), _ptr(dT), _stream()))


def dlrm_interact_dot_bwd(T: torch.Tensor, dR: torch.Tensor, dT: torch.Tensor):
    B, F, d = T.shape
    _check("dlrm_interact_dot_bwd",
           lib().dlrm_interact_dot_bwd(_ptr(T), _ptr(dR), B, F, d, _ptr(dT), _stream()))


def dlrm_emb_bag_bwd_workspace_bytes(K: int, B: int, d: int, nnz_total: int, max_rows: int,
                                     table_dtype: int) -> int:
    return int(lib().dlrm_emb_bag_bwd_workspace_bytes(K, B, d, nnz_total, max_rows, table_dtype))


def dlrm_emb_bag_bwd_sgd(batch: SparseBatch, dS: torch.Tensor, stride_b: int, stride_k: int,
                         lr: float, workspace: Optional[torch.Tensor], algo: int = BWD_AUTO,
                         dS_offset: int = 0):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check("dlrm_emb_bag_bwd_sgd",
           lib().dlrm_emb_bag_bwd_sgd(batch.ref(), _ptr(dS) + 4 * dS_offset, stride_b, stride_k,
                                      C.c_float(lr), _ptr(workspace), ws_bytes, algo, _stream()))


def _timing(ev_start, ev_stop):
    """ev_start / ev_stop: raw hipEvent_t handles (ints or c_void_p)."""
    val = lambda e: e.value if isinstance(e, C.c_void_p) else e
    return _BwdTimingC(val(ev_start), val(ev_stop))


def dlrm_emb_bag_bwd_sgd_timed(batch: SparseBatch, dS: torch.Tensor, stride_b: int, stride_k: int,
                               lr: float, workspace: Optional[torch.Tensor], ev_start, ev_stop,
                               algo: int = BWD_AUTO, dS_offset: int = 0):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    tm = _timing(ev_start, ev_stop)
    _check("dlrm_emb_bag_bwd_sgd_timed",
           lib().dlrm_emb_bag_bwd_sgd_timed(batch.ref(), _ptr(dS) + 4 * dS_offset, stride_b, stride_k,
                                            C.c_float(lr), _ptr(workspace), ws_bytes, algo, C.byref(tm), _stream()))


def dlrm_emb_bag_bwd_adagrad_timed(batch: SparseBatch, state_ptrs: torch.Tensor, dS: torch.Tensor, stride_b: int,
                                   stride_k: int, lr: float, eps: float, workspace: Optional[torch.Tensor],
                                   ev_start, ev_stop, algo: int = BWD_AUTO, dS_offset: int = 0):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    tm = _timing(ev_start, ev_stop)
    _check("dlrm_emb_bag_bwd_adagrad_timed",
           lib().dlrm_emb_bag_bwd_adagrad_timed(batch.ref(), _ptr(state_ptrs), _ptr(dS) + 4 * dS_offset, stride_b,
                                                stride_k, C.c_float(lr), C.c_float(eps), _ptr(workspace), ws_bytes,
                                                algo, C.byref(tm), _stream()))


NOALLOC_SCRATCH_BYTES = 64 << 20


def dlrm_emb_bag_bwd_sgd_noalloc(batch: SparseBatch, dS: torch.Tensor, stride_b: int, stride_k: int, lr: float,
                                 dS_offset: int = 0):
    """The update on the library's own per-GPU scratch array (no workspace argument, no allocation)."""
    _check("dlrm_emb_bag_bwd_sgd_noalloc",
           lib().dlrm_emb_bag_bwd_sgd_noalloc(batch.ref(), _ptr(dS) + 4 * dS_offset, stride_b, stride_k,
                                              C.c_float(lr), _stream()))


def dlrm_emb_bag_bwd_adagrad(batch: SparseBatch, state_ptrs: torch.Tensor, dS: torch.Tensor, stride_b: int,
                             stride_k: int, lr: float, eps: float, workspace: Optional[torch.Tensor],
                             algo: int = BWD_AUTO, dS_offset: int = 0):
    """state_ptrs: int64 device tensor [K] of the accumulators' addresses (see state_pointers)."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check("dlrm_emb_bag_bwd_adagrad",
           lib().dlrm_emb_bag_bwd_adagrad(batch.ref(), _ptr(state_ptrs), _ptr(dS) + 4 * dS_offset, stride_b,
                                          stride_k, C.c_float(lr), C.c_float(eps), _ptr(workspace), ws_bytes,
                                          algo, _stream()))


def state_pointers(state: Sequence[torch.Tensor]) -> torch.Tensor:
    """Device array of the K accumulators' base addresses; the caller keeps `state` alive."""
    for h in state:
        assert h.dtype == torch.float32 and h.is_contiguous()
    return torch.tensor([h.data_ptr() for h in state], dtype=torch.int64, device=state[0].device)


def dlrm_emb_bag_bwd_prepare(batch: SparseBatch, workspace: torch.Tensor,
                             stream: Optional[torch.cuda.Stream] = None):
    """Enqueued on `stream`, or like every other call on torch's current stream."""
    ws_bytes = workspace.numel() * workspace.element_size()
    _check("dlrm_emb_bag_bwd_prepare",
           lib().dlrm_emb_bag_bwd_prepare(batch.ref(), _ptr(workspace), ws_bytes,
                                          _stream() if stream is None else int(stream.cuda_stream)))


def dlrm_emb_bag_bwd_prepared_oversized(batch: SparseBatch, workspace: torch.Tensor, out: torch.Tensor,
                                        index: int = 0, stream: Optional[torch.cuda.Stream] = None):
    """out: int32 tensor the device can write (device memory, or host memory allocated pinned);
    element `index` receives the count once the stream has passed this call."""
    assert out.dtype == torch.int32 and (out.is_cuda or out.is_pinned()) and 0 <= index < out.numel()
    ws_bytes = workspace.numel() * workspace.element_size()
    _check("dlrm_emb_bag_bwd_prepared_oversized",
           lib().dlrm_emb_bag_bwd_prepared_oversized(batch.ref(), _ptr(workspace), ws_bytes,
                                                     _ptr(out) + 4 * index,
                                                     _stream() if stream is None else int(stream.cuda_stream)))


ROUTE_NAMES = ("heavy_ranges", "oversized_ranges", "segments", "segment_tiles", "dominant_row_splits",
               "global_sorts", "one_row_ranges", "huge_runs_in_place", "hot_rows", "dense_hot_tables")


def dlrm_emb_bag_bwd_route_counts(batch: SparseBatch, workspace: torch.Tensor, counts: torch.Tensor):
    """counts: int32 device tensor of >= 10 elements (see ROUTE_NAMES)."""
    assert counts.dtype == torch.int32 and counts.is_cuda and counts.numel() >= 10
    ws_bytes = workspace.numel() * workspace.element_size()
    _check("dlrm_emb_bag_bwd_route_counts",
           lib().dlrm_emb_bag_bwd_route_counts(batch.ref(), _ptr(workspace), ws_bytes, _ptr(counts), _stream()))


def dlrm_emb_bag_bwd_export_groups(batch: SparseBatch, workspace: torch.Tensor,
                                   uniq_rows: torch.Tensor, seg_start: torch.Tensor,
                                   sorted_bag: torch.Tensor, n_uniq: torch.Tensor):
    ws_bytes = workspace.numel() * workspace.element_size()
    _check("dlrm_emb_bag_bwd_export_groups",
           lib().dlrm_emb_bag_bwd_export_groups(batch.ref(), _ptr(workspace), ws_bytes,
                                                _ptr(uniq_rows), _ptr(seg_start), _ptr(sorted_bag),
                                                _ptr(n_uniq), _stream()))


def dlrm_table_init_hash(table: torch.Tensor, table_dtype: int, key: int, scale: float):
    rows, d = table.shape
    _check("dlrm_table_init_hash",
           lib().dlrm_table_init_hash(_ptr(table), rows, d, table_dtype, C.c_uint64(key),
                                      C.c_float(scale), _stream()))


def alloc_workspace(batch: SparseBatch) -> torch.Tensor:
    n = dlrm_emb_bag_bwd_workspace_bytes(batch.K, batch.B, batch.d, batch.nnz_total, batch.max_rows,
                                         batch.table_dtype)
    if n == 0:
        raise DlrmError("dlrm_emb_bag_bwd_workspace_bytes", -2)
    # torch's caching allocator returns 512-byte aligned blocks
    return torch.empty(n, dtype=torch.uint8, device=batch.offsets.device)
