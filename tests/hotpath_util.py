"""Test plumbing shared by the GPU parity tests: moving a generated batch onto the
device, building tables there (uploaded, or hash-initialised in place), running
the oracle on the touched rows only, and the error metric.  No method arithmetic."""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

import paper_1906_00091_amd as hot
from workloads import gen

DEV = "cuda:0"
_TORCH_DT = {gen.F32: torch.float32, gen.F16: torch.float16, gen.BF16: torch.bfloat16}

# Tolerances of the parity gate.  "Relative error" of an output element is its absolute
# error divided by the magnitude scale of the sum that produced it, S_i = sum_j |term_ij|
# (the same computation applied to absolute values; S_i = |ref_i| whenever no cancellation
# occurs, e.g. for one-hot lookups).  fp32 summation of n terms in any order satisfies
# |err_i| <= n * 2^-24 * S_i, so this is the quantity the arithmetic bounds; dividing by
# |ref_i| instead would blow up on elements that cancel to nearly zero.
TOL = {gen.F32: 1e-5, gen.F16: 1e-2, gen.BF16: 1e-2}


# Below the smallest normal number of the storage type a rounding is an absolute, not a
# relative, perturbation: the scale of a stored low-precision value is floored there.
SCALE_FLOOR = {gen.F32: 0.0, gen.F16: 2.0 ** -14, gen.BF16: 2.0 ** -126}


def rel_err(got: np.ndarray, ref: np.ndarray, scale: np.ndarray, floor: float = 0.0) -> float:
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    scale = np.maximum(np.asarray(scale, dtype=np.float64), floor)
    assert got.shape == ref.shape == scale.shape
    if ref.size == 0:
        return 0.0
    assert np.all(scale * 1.01 >= np.abs(ref))   # sanity: |ref| never exceeds its own magnitude scale
    err = np.abs(got - ref)
    tiny = np.finfo(np.float64).tiny
    return float(np.max(np.where(err == 0.0, 0.0, err / np.maximum(scale, tiny))))


def plain_metrics(got: np.ndarray, ref: np.ndarray):
    """The two plain figures beside the gate (reported, not gated): max |got - ref| / max(|ref|, tau) with the
    floor tau = 1e-3 * max|ref| per tensor, and the infinity-norm ratio max|got - ref| / max|ref|."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0, 0.0
    err = np.abs(got - ref)
    top = float(np.abs(ref).max())
    if top == 0.0:
        return float(err.max()), float(err.max())
    return float((err / np.maximum(np.abs(ref), 1e-3 * top)).max()), float(err.max() / top)


def abs_f32_tables(host_tables, dtype):
    """|W| as fp32 arrays (exact for every storage type)."""
    return [np.abs(widen_host(t, dtype)).astype(np.float32) for t in host_tables]


def scale_emb_fwd(host_tables, dtype, indices, offsets, tbl_off):
    from oracle import oracle
    return oracle.emb_bag_fwd(abs_f32_tables(host_tables, dtype), gen.F32, indices, offsets, tbl_off)


def scale_interact_fwd(T):
    from oracle import oracle
    return oracle.interact_dot_fwd(np.abs(T))


def scale_interact_bwd(T, dR):
    from oracle import oracle
    return oracle.interact_dot_bwd(np.abs(T), np.abs(dR))


def scale_sgd(host_tables, dtype, indices, offsets, tbl_off, dS, lr):
    """|W| + lr * sum |dS| per table (fp32 arrays; untouched rows = |W|)."""
    from oracle import oracle
    t = abs_f32_tables(host_tables, dtype)
    oracle.emb_bag_bwd_sgd(t, gen.F32, indices, offsets, tbl_off, -np.abs(dS), lr)
    return t


def table_to_numpy(t: torch.Tensor, dtype: int) -> np.ndarray:
    """Device table (or rows of it) -> host array in the oracle's storage convention."""
    if dtype == gen.BF16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def numpy_to_table(a: np.ndarray, dtype: int) -> torch.Tensor:
    if dtype == gen.BF16:
        return torch.from_numpy(a.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(a).to(DEV)


def upload_tables(host_tables: Sequence[np.ndarray], dtype: int) -> List[torch.Tensor]:
    return [numpy_to_table(np.ascontiguousarray(t), dtype).contiguous() for t in host_tables]


def device_hash_tables(batch: gen.Batch) -> List[torch.Tensor]:
    """Allocate every table on the device and fill it with the counter-based initialiser."""
    w = batch.workload
    out = []
    for k in range(w.K):
        m = int(batch.rows[k])
        t = torch.empty((m, w.d), dtype=_TORCH_DT[w.dtype], device=DEV)
        hot.dlrm_table_init_hash(t, w.dtype, gen.table_key(batch.seed, k), float(gen.table_scale(m)))
        out.append(t)
    return out


def make_sparse_batch(batch: gen.Batch, tables: Sequence[torch.Tensor], weights=None,
                      index32: bool = False) -> hot.SparseBatch:
    idx = torch.from_numpy(batch.indices.astype(np.int32) if index32 else batch.indices).to(DEV)
    off = torch.from_numpy(np.ascontiguousarray(batch.offsets)).to(DEV)
    tbl = torch.from_numpy(batch.tbl_off).to(DEV)
    wts = None if weights is None else torch.from_numpy(np.ascontiguousarray(weights, dtype=np.float32)).to(DEV)
    return hot.SparseBatch(tables, batch.workload.dtype, idx, off, tbl, batch.nnz, weights=wts)


class Compact:
    """The touched rows of every table, for running the oracle without the full tables."""

    def __init__(self, batch: gen.Batch, host_rows_of=None):
        w = batch.workload
        self.uniq = []
        self.tables = []
        self.indices = np.empty_like(batch.indices)
        for k in range(w.K):
            idx = batch.indices_of(k)
            u = np.unique(idx)
            self.uniq.append(u)
            if host_rows_of is None:
                rows = gen.init_rows(batch.seed, k, int(batch.rows[k]), w.d, w.dtype, u)
            else:
                rows = host_rows_of(k, u)
            self.tables.append(np.ascontiguousarray(rows))
            self.indices[batch.tbl_off[k]:batch.tbl_off[k + 1]] = np.searchsorted(u, idx)

    def gather_device(self, tables: Sequence[torch.Tensor], dtype: int) -> List[np.ndarray]:
        out = []
        for k, u in enumerate(self.uniq):
            sel = torch.from_numpy(u).to(DEV)
            out.append(table_to_numpy(tables[k].index_select(0, sel), dtype))
        return out


def widen_host(a: np.ndarray, dtype: int) -> np.ndarray:
    if dtype == gen.BF16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)
