"""Seeded synthetic inputs for the DLRM sparse hot path.

This module only *draws inputs*: table shapes, CSR index lists, dense vectors,
upstream gradients and the counter-based table initialiser.  It holds none of
the method's arithmetic (no pooling, no interaction, no update), so both the
CPU oracle's tests and the HIP path's tests/bench may use it.

The five workloads mirror the shapes of the paper's experiments:
  * the random generator of Sec. 4.1 (uniform indices, a fixed or uniformly
    random number of indices per lookup, lengths/offsets CSR encoding),
  * the click-log shape of Sec. 4.3 (13 dense + 26 one-hot categorical
    features, embedding dimension 16 in Sec. 5.1),
  * the single-device profile shape of Sec. 5.2 (8 tables x 1M rows x dim 64,
    mini-batch 2048).
The public click logs themselves are not used; Zipf-distributed indices stand
in for their skew.

Draw order for a workload (fixed, so every consumer sees the same arrays):
table row counts -> rank->row bijection constants  (stream ``[seed, 0]``)
lengths -> indices -> x -> dR -> dS               (stream ``[seed, 1 + batch_id]``)
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

F32, F16, BF16 = 0, 1, 2
DTYPE_NAMES = {F32: "f32", F16: "f16", BF16: "bf16"}
ELEM_BYTES = {F32: 4, F16: 2, BF16: 2}


@dataclass
class Workload:
    """Shape of one workload (no data)."""
    name: str
    K: int                       # number of tables (categorical features)
    B: int                       # mini-batch size
    d: int                       # embedding dimension
    dtype: int                   # table storage type
    rows: Tuple                  # ("fixed", m) | ("loguniform", lo, hi, cap_total or None, min_rows)
    bag: Tuple                   # ("fixed", L) | ("uniform", lo, hi)  inclusive
    dist: Tuple                  # ("uniform",) | ("zipf", alpha) | ("trace", alpha): Sec. 4.2 generator
    lr: float = 0.01
    seed: int = 0

    @property
    def F(self) -> int:
        return self.K + 1

    @property
    def P(self) -> int:
        return self.F * (self.F - 1) // 2


WORKLOADS: Dict[int, Workload] = {
    1: Workload("tiny", K=8, B=128, d=16, dtype=F32, rows=("fixed", 1000),
                bag=("uniform", 1, 4), dist=("uniform",)),
    2: Workload("clicklog_onehot", K=26, B=2048, d=16, dtype=F32,
                rows=("loguniform", 3, 10_000_000, None, 3),
                bag=("fixed", 1), dist=("zipf", 1.05)),
    3: Workload("multihot_bandwidth", K=8, B=2048, d=64, dtype=F32, rows=("fixed", 1_000_000),
                bag=("uniform", 1, 200), dist=("uniform",)),
    4: Workload("large_onehot", K=26, B=8192, d=128, dtype=F32,
                rows=("loguniform", 1000, 40_000_000, 180_000_000, 1000),
                bag=("fixed", 1), dist=("zipf", 1.05)),
    5: Workload("hotrow_stress", K=64, B=16384, d=128, dtype=F16, rows=("fixed", 2_000_000),
                bag=("fixed", 32), dist=("zipf", 1.2)),
}


# --------------------------------------------------------------------------
# Counter-based table initialiser: value(seed, k, row, col) without any state,
# so a 90 GB table never has to exist on the host.  The device library fills
# tables with the same function; both sides implement it independently.
#
#   key_k = mix(seed ^ mix(k))                       (64-bit, wrap-around)
#   h     = mix(key_k + row*d + col)
#   u     = h >> 40                                  (24 bits)
#   x     = (2u + 1 - 2^24) / 2^24                   (odd/2^24: exact in fp32, in (-1,1))
#   W     = fp32(x) * fp32(1/sqrt(m))                (one fp32 multiply), then
#           one round-to-nearest-even to fp16/bf16 for low-precision tables
#
# mix() is the splitmix64 output function (Steele, Lea, Flood 2014).
# --------------------------------------------------------------------------
_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLD = np.uint64(0x9E3779B97F4A7C15)
_C1 = np.uint64(0xBF58476D1CE4E5B9)
_C2 = np.uint64(0x94D049BB133111EB)


def _mix64(z: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        z = (z + _GOLD).astype(np.uint64)
        z = ((z ^ (z >> np.uint64(30))) * _C1).astype(np.uint64)
        z = ((z ^ (z >> np.uint64(27))) * _C2).astype(np.uint64)
        return z ^ (z >> np.uint64(31))


def table_key(seed: int, k: int) -> int:
    """64-bit stream key of table k (passed to the device fill as a scalar)."""
    a = _mix64(np.array([k], dtype=np.uint64))
    b = _mix64(np.array([seed], dtype=np.uint64) ^ a)
    return int(b[0])


def table_scale(m: int) -> np.float32:
    """fp32(1/sqrt(m)): the half-width of the uniform init range."""
    return np.float32(1.0 / math.sqrt(float(m)))


def _to_bf16_bits(x32: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit pattern, round-to-nearest-even (inputs are finite)."""
    u = x32.astype(np.float32).view(np.uint32).astype(np.uint64)
    rnd = ((u >> np.uint64(16)) & np.uint64(1)) + np.uint64(0x7FFF)
    return ((u + rnd) >> np.uint64(16)).astype(np.uint16)


def init_rows(seed: int, k: int, m: int, d: int, dtype: int, row_ids: np.ndarray) -> np.ndarray:
    """Materialise rows ``row_ids`` of table k.  Returns [len(row_ids), d] as
    float32 (F32), float16 (F16) or uint16 bf16 bit patterns (BF16)."""
    row_ids = np.asarray(row_ids, dtype=np.int64)
    key = np.uint64(table_key(seed, k))
    e = (row_ids[:, None].astype(np.uint64) * np.uint64(d)
         + np.arange(d, dtype=np.uint64)[None, :])
    with np.errstate(over="ignore"):
        h = _mix64((e + key).astype(np.uint64))
    u = (h >> np.uint64(40)).astype(np.int64)
    x = ((2 * u + 1 - (1 << 24)).astype(np.float32)) / np.float32(1 << 24)
    w = (x * table_scale(m)).astype(np.float32)
    if dtype == F32:
        return w
    if dtype == F16:
        return w.astype(np.float16)
    if dtype == BF16:
        return _to_bf16_bits(w)
    raise ValueError("dtype")


def init_table(seed: int, k: int, m: int, d: int, dtype: int, chunk: int = 1 << 18) -> np.ndarray:
    """Whole table k on the host (only sensible for small/medium tables)."""
    out = np.empty((m, d), dtype={F32: np.float32, F16: np.float16, BF16: np.uint16}[dtype])
    for r0 in range(0, m, chunk):
        r1 = min(m, r0 + chunk)
        out[r0:r1] = init_rows(seed, k, m, d, dtype, np.arange(r0, r1, dtype=np.int64))
    return out


# --------------------------------------------------------------------------
# Shapes
# --------------------------------------------------------------------------
def table_rows(w: Workload, seed: Optional[int] = None) -> np.ndarray:
    """Row count m_k of every table (int64[K])."""
    seed = w.seed if seed is None else seed
    rng = np.random.default_rng([seed, 0])
    kind = w.rows[0]
    if kind == "fixed":
        return np.full(w.K, int(w.rows[1]), dtype=np.int64)
    if kind == "loguniform":
        _, lo, hi, cap, min_rows = w.rows
        m = np.floor(np.exp(rng.uniform(math.log(lo), math.log(hi), size=w.K))).astype(np.int64)
        m = np.clip(m, lo, hi)
        if cap is not None and int(m.sum()) > cap:
            m = np.maximum(np.floor(m * (cap / float(m.sum()))).astype(np.int64), min_rows)
        return m
    raise ValueError(kind)


def _bijection_constants(w: Workload, rows: np.ndarray, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """Per-table (A, C) with gcd(A, m) = 1 so rank -> (rank*A + C) mod m is a
    bijection that scatters the popular ranks over the table."""
    rng = np.random.default_rng([seed, 0])
    # burn the draws table_rows() made so the constants follow them in the stream
    if w.rows[0] == "loguniform":
        rng.uniform(0.0, 1.0, size=w.K)
    A = np.empty(w.K, dtype=np.int64)
    C = np.empty(w.K, dtype=np.int64)
    for k in range(w.K):
        m = int(rows[k])
        a = int(rng.integers(1, max(m, 2)))
        while math.gcd(a, m) != 1:
            a += 1
            if a >= m:
                a = 1
        A[k] = a if m > 1 else 0
        C[k] = int(rng.integers(0, m))
    return A, C


_ZIPF_CDF_CACHE: Dict[Tuple[int, float], np.ndarray] = {}


def _zipf_cdf(m: int, alpha: float) -> np.ndarray:
    key = (m, alpha)
    cdf = _ZIPF_CDF_CACHE.get(key)
    if cdf is None:
        p = np.arange(1, m + 1, dtype=np.float64) ** (-alpha)
        cdf = np.cumsum(p)
        cdf /= cdf[-1]
        if len(_ZIPF_CDF_CACHE) > 2:
            _ZIPF_CDF_CACHE.clear()
        _ZIPF_CDF_CACHE[key] = cdf
    return cdf


def _draw_indices(rng, dist: Tuple, m: int, n: int, A: int, C: int) -> np.ndarray:
    if dist[0] == "uniform":
        return rng.integers(0, m, size=n, dtype=np.int64)
    if dist[0] == "zipf":
        cdf = _zipf_cdf(m, float(dist[1]))
        rank = np.searchsorted(cdf, rng.random(n), side="left").astype(np.int64)  # 0-based rank
        rank = np.minimum(rank, m - 1)
        return (rank * np.int64(A) + np.int64(C)) % np.int64(m)
    if dist[0] == "trace":
        # Sec. 4.2: a synthetic trace with the locality of an original one.  The original here is a
        # bounded-Zipf draw (alpha = dist[1]) four times as long as the batch; Alg. 1 profiles it into its
        # unique ids u and stack-distance distribution p, Alg. 2 emits n lookups from (u, p) (first-time
        # accesses at no less than 10 % while unseen ids remain, the section's adjustment).
        from workloads import trace
        original = _draw_indices(rng, ("zipf", float(dist[1])), m, 4 * n, A, C)
        u, p = trace.profile_trace(original, m)
        return trace.generate_trace(u, p, rng.random(n), min_new=0.1)
    raise ValueError(dist)


def locality_workload(base: int, alpha: float) -> "Workload":
    """Workload `base` with its indices drawn by the stack-distance generator of Sec. 4.2 from the profile
    of a Zipf(alpha) trace: alpha moves the temporal locality (how soon an id comes back)."""
    import dataclasses
    w = WORKLOADS[base]
    return dataclasses.replace(w, name="%s_trace_a%g" % (w.name, alpha), dist=("trace", float(alpha)))


@dataclass
class Batch:
    """One mini-batch of inputs (host arrays)."""
    workload: Workload
    rows: np.ndarray             # int64 [K]
    lengths: np.ndarray          # int32 [K, B]
    offsets: np.ndarray          # int64 [K, B+1]  per-table local offsets
    tbl_off: np.ndarray          # int64 [K+1]
    indices: np.ndarray          # int64 [nnz_total], table-major
    x: np.ndarray                # float32 [B, d]
    dR: np.ndarray               # float32 [B, d+P]
    seed: int = 0
    batch_id: int = 0
    _dS: Optional[np.ndarray] = field(default=None, repr=False)

    @property
    def nnz(self) -> int:
        return int(self.tbl_off[-1])

    def dS(self) -> np.ndarray:
        """Direct upstream gradient of the pooled vectors, float32 [B, K, d]
        (for exercising the embedding backward without the interaction)."""
        if self._dS is None:
            w = self.workload
            rng = np.random.default_rng([self.seed, 1 + self.batch_id, 7])
            self._dS = rng.standard_normal((w.B, w.K, w.d), dtype=np.float32)
        return self._dS

    def indices_of(self, k: int) -> np.ndarray:
        return self.indices[self.tbl_off[k]:self.tbl_off[k + 1]]


def make_batch(w: Workload, seed: Optional[int] = None, batch_id: int = 0,
               rows: Optional[np.ndarray] = None) -> Batch:
    seed = w.seed if seed is None else seed
    rows = table_rows(w, seed) if rows is None else np.asarray(rows, dtype=np.int64)
    A, C = _bijection_constants(w, rows, seed)
    rng = np.random.default_rng([seed, 1 + batch_id])
    if w.bag[0] == "fixed":
        lengths = np.full((w.K, w.B), int(w.bag[1]), dtype=np.int32)
    elif w.bag[0] == "uniform":
        lengths = rng.integers(int(w.bag[1]), int(w.bag[2]) + 1, size=(w.K, w.B)).astype(np.int32)
    else:
        raise ValueError(w.bag)
    offsets = np.zeros((w.K, w.B + 1), dtype=np.int64)
    np.cumsum(lengths, axis=1, out=offsets[:, 1:])
    nnz_k = offsets[:, -1]
    tbl_off = np.zeros(w.K + 1, dtype=np.int64)
    np.cumsum(nnz_k, out=tbl_off[1:])
    indices = np.empty(int(tbl_off[-1]), dtype=np.int64)
    for k in range(w.K):
        indices[tbl_off[k]:tbl_off[k + 1]] = _draw_indices(
            rng, w.dist, int(rows[k]), int(nnz_k[k]), int(A[k]), int(C[k]))
    x = rng.standard_normal((w.B, w.d), dtype=np.float32)
    dR = rng.standard_normal((w.B, w.d + w.P), dtype=np.float32)
    return Batch(w, rows, lengths, offsets, tbl_off, indices, x, dR, seed=seed, batch_id=batch_id)


def custom_workload(name: str, K: int, B: int, d: int, dtype: int = F32, rows=1000,
                    bag=("uniform", 1, 4), dist=("uniform",), lr: float = 0.01,
                    seed: int = 0) -> Workload:
    rows_spec = ("fixed", int(rows)) if not isinstance(rows, tuple) else rows
    return Workload(name, K=K, B=B, d=d, dtype=dtype, rows=rows_spec, bag=bag, dist=dist,
                    lr=lr, seed=seed)


def batch_from_lists(rows: List[int], bags: List[List[List[int]]], d: int, dtype: int = F32,
                     seed: int = 0) -> Batch:
    """Hand-written index lists: ``bags[k][b]`` is the list of row ids of bag b
    of table k (may be empty, may repeat).  Used by edge-case tests."""
    K = len(bags)
    B = len(bags[0])
    w = Workload("handmade", K=K, B=B, d=d, dtype=dtype, rows=("fixed", 0),
                 bag=("fixed", 0), dist=("uniform",), seed=seed)
    lengths = np.array([[len(b) for b in t] for t in bags], dtype=np.int32).reshape(K, B)
    offsets = np.zeros((K, B + 1), dtype=np.int64)
    np.cumsum(lengths, axis=1, out=offsets[:, 1:])
    tbl_off = np.zeros(K + 1, dtype=np.int64)
    np.cumsum(offsets[:, -1], out=tbl_off[1:])
    flat = [i for t in bags for b in t for i in b]
    indices = np.array(flat, dtype=np.int64).reshape(-1)
    rng = np.random.default_rng([seed, 1])
    x = rng.standard_normal((B, d), dtype=np.float32)
    dR = rng.standard_normal((B, d + w.P), dtype=np.float32)
    return Batch(w, np.asarray(rows, dtype=np.int64), lengths, offsets, tbl_off, indices, x, dR,
                 seed=seed)


def make_weights(batch: "Batch", seed: int = 0) -> np.ndarray:
    """Per-lookup weights for Eq. (2), parallel to ``batch.indices``: float32 uniform in [0.5, 1.5)."""
    rng = np.random.default_rng([seed, 77, batch.nnz])
    return rng.uniform(0.5, 1.5, size=batch.indices.shape).astype(np.float32)
