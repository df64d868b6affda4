"""ctypes front end of the CPU oracle (oracle/dlrm_oracle.c).

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg; never by the product package.  Host numpy arrays
in, host numpy arrays (float64 results) out.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dlrm_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

F32, F16, BF16 = 0, 1, 2
_NP_OF = {F32: np.float32, F16: np.uint16, BF16: np.uint16}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP, no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.oracle_half_to_double.restype = C.c_double
        L.oracle_half_to_double.argtypes = [C.c_uint16]
        L.oracle_double_to_half.restype = C.c_uint16
        L.oracle_double_to_half.argtypes = [C.c_double]
        L.oracle_bf16_to_double.restype = C.c_double
        L.oracle_bf16_to_double.argtypes = [C.c_uint16]
        L.oracle_double_to_bf16.restype = C.c_uint16
        L.oracle_double_to_bf16.argtypes = [C.c_double]
        L.oracle_validate_csr.restype = C.c_int64
        L.oracle_get_threads.restype = C.c_int
        _lib = L
    return _lib


def set_threads(n: int) -> None:
    lib().oracle_set_threads(C.c_int(int(n)))


def get_threads() -> int:
    return int(lib().oracle_get_threads())


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _i64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int64)


def _table_ptrs(tables: Sequence[np.ndarray], dtype: int):
    want = _NP_OF[dtype]
    keep = []
    for t in tables:
        if dtype == F16 and t.dtype == np.float16:
            t = t.view(np.uint16)
        if t.dtype != want or not t.flags["C_CONTIGUOUS"]:
            raise TypeError("table must be C-contiguous %s, got %s" % (want, t.dtype))
        keep.append(t)
    arr = (C.c_void_p * len(keep))(*[t.ctypes.data for t in keep])
    return arr, keep


def half_to_double(bits: np.ndarray) -> np.ndarray:
    L = lib()
    return np.array([L.oracle_half_to_double(int(b)) for b in np.asarray(bits).ravel()])


def double_to_half(vals: np.ndarray) -> np.ndarray:
    L = lib()
    return np.array([L.oracle_double_to_half(float(v)) for v in np.asarray(vals).ravel()],
                    dtype=np.uint16)


def bf16_to_double(bits: np.ndarray) -> np.ndarray:
    L = lib()
    return np.array([L.oracle_bf16_to_double(int(b)) for b in np.asarray(bits).ravel()])


def double_to_bf16(vals: np.ndarray) -> np.ndarray:
    L = lib()
    return np.array([L.oracle_double_to_bf16(float(v)) for v in np.asarray(vals).ravel()],
                    dtype=np.uint16)


def lengths_to_offsets(lengths: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """lengths int32 [K,B] -> (offsets int64 [K,B+1], tbl_off int64 [K+1])."""
    lengths = np.ascontiguousarray(lengths, dtype=np.int32)
    K, B = lengths.shape
    offsets = np.empty((K, B + 1), dtype=np.int64)
    tbl_off = np.empty(K + 1, dtype=np.int64)
    st = lib().oracle_lengths_to_offsets(_p(lengths), C.c_int32(K), C.c_int32(B), _p(offsets),
                                         _p(tbl_off))
    if st != 0:
        raise ValueError("oracle_lengths_to_offsets status %d" % st)
    return offsets, tbl_off


def validate_csr(rows, indices, offsets, tbl_off) -> int:
    rows, indices, offsets, tbl_off = _i64(rows), _i64(indices), _i64(offsets), _i64(tbl_off)
    K, B1 = offsets.shape
    return int(lib().oracle_validate_csr(C.c_int32(K), C.c_int32(B1 - 1), _p(rows), _p(indices),
                                         _p(offsets), _p(tbl_off)))


def emb_bag_fwd(tables: Sequence[np.ndarray], dtype: int, indices, offsets, tbl_off) -> np.ndarray:
    """Pooled vectors as float64 [B, K, d]."""
    indices, offsets, tbl_off = _i64(indices), _i64(offsets), _i64(tbl_off)
    K, B1 = offsets.shape
    B = B1 - 1
    d = tables[0].shape[1]
    rows = _i64([t.shape[0] for t in tables])
    ptrs, keep = _table_ptrs(tables, dtype)
    out = np.empty((B, K, d), dtype=np.float64)
    st = lib().oracle_emb_bag_fwd(C.c_int32(K), C.c_int32(B), C.c_int32(d), C.c_int32(dtype), ptrs,
                                  _p(rows), _p(indices), _p(offsets), _p(tbl_off), _p(out),
                                  C.c_int64(K * d), C.c_int64(d))
    if st != 0:
        raise ValueError("oracle_emb_bag_fwd status %d" % st)
    return out


def interact_dot_fwd(T: np.ndarray) -> np.ndarray:
    """T float32 [B,F,d] -> R float64 [B, d + F(F-1)/2]."""
    T = np.ascontiguousarray(T, dtype=np.float32)
    B, F, d = T.shape
    R = np.empty((B, d + F * (F - 1) // 2), dtype=np.float64)
    st = lib().oracle_interact_dot_fwd(_p(T), C.c_int32(B), C.c_int32(F), C.c_int32(d), _p(R))
    if st != 0:
        raise ValueError("oracle_interact_dot_fwd status %d" % st)
    return R


def emb_interact_fwd(tables: Sequence[np.ndarray], dtype: int, indices, offsets, tbl_off,
                     x: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """The forward of the sparse side in one call (Sec. 2.2: the processed dense vector and the
    pooled vectors of Eq. (2) are the F = K + 1 inputs of the dot interaction).
    x float32 [B,d] -> (T float32 [B,F,d], R float64 [B, d + F(F-1)/2]); T[:,0] = x,
    T[:,k+1] = the pooled vectors of table k rounded to fp32 (the type T is handed over in)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    S = emb_bag_fwd(tables, dtype, indices, offsets, tbl_off)
    B, K, d = S.shape
    T = np.empty((B, K + 1, d), dtype=np.float32)
    T[:, 0] = x
    T[:, 1:] = S.astype(np.float32)
    return T, interact_dot_fwd(T)


def emb_interact_bwd(tables: Sequence[np.ndarray], dtype: int, indices, offsets, tbl_off, x: np.ndarray,
                     dR: np.ndarray) -> np.ndarray:
    """Backward of emb_interact_fwd with respect to its F vectors, composed of the functions above:
    T as emb_interact_fwd hands it over (pooled vectors of Eq. (2) rounded to fp32, x in row 0), then the
    chain rule of the interaction (Sec. 2.2).  -> dT float64 [B,F,d]."""
    T, _ = emb_interact_fwd(tables, dtype, indices, offsets, tbl_off, x)
    return interact_dot_bwd(T, dR)


def interact_dot_bwd(T: np.ndarray, dR: np.ndarray) -> np.ndarray:
    """-> dT float64 [B,F,d]."""
    T = np.ascontiguousarray(T, dtype=np.float32)
    dR = np.ascontiguousarray(dR, dtype=np.float32)
    B, F, d = T.shape
    assert dR.shape == (B, d + F * (F - 1) // 2)
    dT = np.empty((B, F, d), dtype=np.float64)
    st = lib().oracle_interact_dot_bwd(_p(T), _p(dR), C.c_int32(B), C.c_int32(F), C.c_int32(d),
                                       _p(dT))
    if st != 0:
        raise ValueError("oracle_interact_dot_bwd status %d" % st)
    return dT


def group_rows(indices, offsets, tbl_off):
    """Per table: (uniq_rows, seg_start, sorted_pos, sorted_bag) lists of arrays."""
    indices, offsets, tbl_off = _i64(indices), _i64(offsets), _i64(tbl_off)
    K, B1 = offsets.shape
    n = max(int(tbl_off[-1]), 1)
    sorted_pos = np.zeros(n, dtype=np.int64)
    sorted_bag = np.zeros(n, dtype=np.int32)
    uniq = np.zeros(n, dtype=np.int64)
    seg = np.zeros(n, dtype=np.int64)
    nu = np.zeros(K, dtype=np.int64)
    st = lib().oracle_group_rows(C.c_int32(K), C.c_int32(B1 - 1), _p(indices), _p(offsets),
                                 _p(tbl_off), _p(sorted_pos), _p(sorted_bag), _p(uniq), _p(seg),
                                 _p(nu))
    if st != 0:
        raise ValueError("oracle_group_rows status %d" % st)
    out = []
    for k in range(K):
        a, b = int(tbl_off[k]), int(tbl_off[k + 1])
        u = int(nu[k])
        out.append((uniq[a:a + u].copy(), seg[a:a + u].copy(), sorted_pos[a:b].copy(),
                    sorted_bag[a:b].copy()))
    return out


def emb_bag_bwd_sgd(tables: Sequence[np.ndarray], dtype: int, indices, offsets, tbl_off,
                    dS: np.ndarray, lr: float, apply: bool = True, want_grad: bool = False):
    """Updates ``tables`` in place (if apply).  dS float32 [B,K,d].
    Returns (uniq_rows per table, row_grad per table or None)."""
    indices, offsets, tbl_off = _i64(indices), _i64(offsets), _i64(tbl_off)
    dS = np.ascontiguousarray(dS, dtype=np.float32)
    K, B1 = offsets.shape
    B = B1 - 1
    d = tables[0].shape[1]
    assert dS.shape == (B, K, d)
    rows = _i64([t.shape[0] for t in tables])
    ptrs, keep = _table_ptrs(tables, dtype)
    n = max(int(tbl_off[-1]), 1)
    uniq = np.zeros(n, dtype=np.int64)
    nu = np.zeros(K, dtype=np.int64)
    grad = np.zeros((n, d), dtype=np.float64) if want_grad else None
    st = lib().oracle_emb_bag_bwd_sgd(
        C.c_int32(K), C.c_int32(B), C.c_int32(d), C.c_int32(dtype), ptrs, _p(rows), _p(indices),
        _p(offsets), _p(tbl_off), _p(dS), C.c_int64(K * d), C.c_int64(d), C.c_double(float(lr)),
        C.c_int32(1 if apply else 0), _p(grad) if want_grad else None, _p(uniq), _p(nu))
    if st != 0:
        raise ValueError("oracle_emb_bag_bwd_sgd status %d" % st)
    uniq_l, grad_l = [], []
    for k in range(K):
        a = int(tbl_off[k])
        u = int(nu[k])
        uniq_l.append(uniq[a:a + u].copy())
        if want_grad:
            grad_l.append(grad[a:a + u].copy())
    return uniq_l, (grad_l if want_grad else None)


def emb_bag_bwd_adagrad(tables: Sequence[np.ndarray], state: Sequence[np.ndarray], dtype: int, indices,
                        offsets, tbl_off, dS: np.ndarray, lr: float, eps: float):
    """Updates ``tables`` and the float32 accumulators ``state`` in place.  dS float32 [B,K,d]."""
    indices, offsets, tbl_off = _i64(indices), _i64(offsets), _i64(tbl_off)
    dS = np.ascontiguousarray(dS, dtype=np.float32)
    K, B1 = offsets.shape
    B = B1 - 1
    d = tables[0].shape[1]
    assert dS.shape == (B, K, d)
    for t, h in zip(tables, state):
        assert h.dtype == np.float32 and h.shape == t.shape and h.flags["C_CONTIGUOUS"]
    rows = _i64([t.shape[0] for t in tables])
    ptrs, keep = _table_ptrs(tables, dtype)
    sptrs = (C.c_void_p * K)(*[h.ctypes.data for h in state])
    st = lib().oracle_emb_bag_bwd_adagrad(
        C.c_int32(K), C.c_int32(B), C.c_int32(d), C.c_int32(dtype), ptrs, sptrs, _p(rows), _p(indices),
        _p(offsets), _p(tbl_off), _p(dS), C.c_int64(K * d), C.c_int64(d), C.c_double(float(lr)),
        C.c_double(float(eps)))
    if st != 0:
        raise ValueError("oracle_emb_bag_bwd_adagrad status %d" % st)


def emb_bag_fwd_weighted(tables: Sequence[np.ndarray], dtype: int, indices, offsets, tbl_off,
                         weights: np.ndarray) -> np.ndarray:
    """Eq. (2) with its weights: float64 [B,K,d]; weights float32 parallel to indices."""
    indices, offsets, tbl_off = _i64(indices), _i64(offsets), _i64(tbl_off)
    weights = np.ascontiguousarray(weights, dtype=np.float32)
    assert weights.shape == indices.shape
    K, B1 = offsets.shape
    B = B1 - 1
    d = tables[0].shape[1]
    rows = _i64([t.shape[0] for t in tables])
    ptrs, keep = _table_ptrs(tables, dtype)
    out = np.empty((B, K, d), dtype=np.float64)
    st = lib().oracle_emb_bag_fwd_weighted(C.c_int32(K), C.c_int32(B), C.c_int32(d), C.c_int32(dtype), ptrs,
                                           _p(rows), _p(indices), _p(offsets), _p(tbl_off), _p(weights),
                                           _p(out), C.c_int64(K * d), C.c_int64(d))
    if st != 0:
        raise ValueError("oracle_emb_bag_fwd_weighted status %d" % st)
    return out


def emb_bag_bwd_weighted(tables: Sequence[np.ndarray], dtype: int, indices, offsets, tbl_off, weights,
                         dS: np.ndarray, lr: float, state: Optional[Sequence[np.ndarray]] = None,
                         eps: float = 0.0):
    """Backward of the weighted lookup, tables (and Adagrad state, if given) updated in place."""
    indices, offsets, tbl_off = _i64(indices), _i64(offsets), _i64(tbl_off)
    weights = np.ascontiguousarray(weights, dtype=np.float32)
    dS = np.ascontiguousarray(dS, dtype=np.float32)
    K, B1 = offsets.shape
    B = B1 - 1
    d = tables[0].shape[1]
    assert dS.shape == (B, K, d) and weights.shape == indices.shape
    rows = _i64([t.shape[0] for t in tables])
    ptrs, keep = _table_ptrs(tables, dtype)
    sptrs = None
    if state is not None:
        for t, h in zip(tables, state):
            assert h.dtype == np.float32 and h.shape == t.shape and h.flags["C_CONTIGUOUS"]
        sptrs = (C.c_void_p * K)(*[h.ctypes.data for h in state])
    st = lib().oracle_emb_bag_bwd_weighted(
        C.c_int32(K), C.c_int32(B), C.c_int32(d), C.c_int32(dtype), ptrs, sptrs, _p(rows), _p(indices),
        _p(offsets), _p(tbl_off), _p(weights), _p(dS), C.c_int64(K * d), C.c_int64(d), C.c_double(float(lr)),
        C.c_double(float(eps)), C.c_int32(0 if state is None else 1))
    if st != 0:
        raise ValueError("oracle_emb_bag_bwd_weighted status %d" % st)
