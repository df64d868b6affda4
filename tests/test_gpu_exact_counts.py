"""Index handling of the UPDATE itself, bit for bit (transpose of Eq. (2): the gradient of a row is
the sum of the pooled-vector gradients of every lookup of it -- "count x upstream gradient").

The exported grouping is checked elsewhere; the update takes other routes for heavy rows (dominant
rows split off unsorted, lists sorted by many workgroups or through global memory, hot rows summed
per bag group, entry by entry or as a dense contraction).  A float tolerance cannot see one lookup
dropped or doubled in a run of 10^5, so here every quantity is an exactly representable number:
gradients are small integers, tables hold small integers, lr is a power of two, weights are powers
of two.  Every partial sum, in any order, is then exact in fp32, the fp64 oracle is exact too, and
the updated rows must be EQUAL.  One miscounted lookup changes a sum by at least one unit.

Each case also reads back which routes the update took (dlrm_emb_bag_bwd_route_counts) and requires
the routes it was written for."""
import numpy as np
import pytest
import torch

import paper_1906_00091_amd as hot
from oracle import oracle
from workloads import gen

from hotpath_util import DEV, Compact, make_sparse_batch, table_to_numpy

pytestmark = pytest.mark.gpu

_TORCH_DT = {gen.F32: torch.float32, gen.F16: torch.float16, gen.BF16: torch.bfloat16}

# name, K, B, d, dtype, rows, bag, dist, routes that the SORT update must have taken
CASES = [
    # 19 K lookups: no tail launches; the hottest row's run (> 2048) is split off and summed in place
    ("hot-rows", 2, 600, 32, gen.F32, 50000, ("fixed", 16), ("zipf", 1.4),
     ("oversized_ranges", "dominant_row_splits", "huge_runs_in_place")),
    # 5 rows per table above 2048 lookups: the entry-by-entry hot-row kernel (fewer than 8 per table)
    ("hot-rows-large", 2, 4096, 32, gen.F32, 50000, ("fixed", 16), ("zipf", 1.4),
     ("oversized_ranges", "dominant_row_splits", "hot_rows")),
    # 40 single-row ranges of ~4096 lookups per table: more hot rows than one pass of the dense kernel holds
    ("many-hot-rows", 2, 4096, 32, gen.F32, 40, ("fixed", 40), ("uniform",),
     ("one_row_ranges", "hot_rows", "dense_hot_tables")),
    ("dense-hot-rows-d64", 2, 2500, 64, gen.F32, 20, ("fixed", 40), ("uniform",),
     ("one_row_ranges", "hot_rows", "dense_hot_tables")),
    ("dense-hot-rows-d256-f16", 1, 1100, 256, gen.F16, 12, ("fixed", 70), ("uniform",),
     ("one_row_ranges", "hot_rows", "dense_hot_tables")),
    # every range too large for the LDS sort, nothing dominant, 12 unsorted bits: segment kernels
    ("segments-no-dominant-row", 1, 32768, 8, gen.F32, 1 << 22, ("fixed", 96), ("uniform",),
     ("oversized_ranges", "segments", "segment_tiles")),
    # dominant rows split off AND a remainder that is still too large
    ("dominant-rows-large-rest", 1, 32768, 16, gen.F32, 1 << 22, ("fixed", 200), ("zipf", 1.1),
     ("oversized_ranges", "dominant_row_splits", "segments", "hot_rows")),
    # the same with 15 unsorted bits: the remainder is sorted through global memory
    ("dominant-rows-large-rest-many-bits", 1, 65536, 4, gen.F32, 1 << 25, ("fixed", 96), ("zipf", 1.05),
     ("oversized_ranges", "dominant_row_splits", "global_sorts", "hot_rows")),
    # 15 unsorted bits: a workgroup streams its range through global memory
    ("large-buckets-many-bits", 1, 65536, 4, gen.F32, 1 << 25, ("fixed", 64), ("uniform",),
     ("oversized_ranges", "global_sorts")),
    # one table of the hot-row stress workload at its real size: fp16, 2 M rows, 32 lookups per bag, Zipf 1.2
    ("zipf12-fixed32-2Mrows-f16", 1, 16384, 128, gen.F16, 2000000, ("fixed", 32), ("zipf", 1.2),
     ("heavy_ranges", "oversized_ranges", "dominant_row_splits", "hot_rows", "dense_hot_tables")),
    ("bf16-zipf-d64", 3, 8192, 64, gen.BF16, 30000, ("fixed", 12), ("zipf", 1.3),
     ("oversized_ranges", "dominant_row_splits", "hot_rows")),
    # a gradient slice of 6.3 MB per table: the update deals its row ranges to the dies by table; nine tables, so
    # that eight go through that mapping and the ninth keeps the plain order
    ("nine-tables-by-die", 9, 16384, 96, gen.F32, 20000, ("fixed", 3), ("zipf", 1.1),
     ("oversized_ranges", "dominant_row_splits", "hot_rows")),
]

MODES = ["sort", "prepared", "flat"]


def _say(msg):
    print("[case] " + msg, flush=True)


def _integer_tables(rows, d, dtype, seed):
    g = torch.Generator(device=DEV).manual_seed(seed)
    return [torch.randint(-8, 9, (int(m), d), generator=g, device=DEV, dtype=torch.int32).to(_TORCH_DT[dtype])
            for m in rows]


def _max_run(batch):
    return max(int(np.bincount(batch.indices_of(k)).max()) if len(batch.indices_of(k)) else 0
               for k in range(batch.workload.K))


def _integer_dS(B, K, d, max_run, wmax=1.0):
    """Small signed integers: column 0 = 1 (the row's sum is its lookup count), column 1 = parity of the
    bag, the others a pattern in bag, table and column.  Magnitudes are bounded so that
    max_run * wmax * max|dS| < 2^22: every partial sum is an integer (or a multiple of the smallest
    weight) that fp32 holds exactly."""
    M = int(min(256, max(2, (1 << 22) // max(1, int(max_run * wmax)))))
    b = np.arange(B, dtype=np.int64)[:, None, None]
    k = np.arange(K, dtype=np.int64)[None, :, None]
    c = np.arange(d, dtype=np.int64)[None, None, :]
    v = (b * (c + 1) + 3 * k + c) % M - M // 2
    dS = v.astype(np.float32)
    dS[:, :, 0] = 1.0
    if d > 1:
        dS[:, :, 1] = (np.arange(B) & 1)[:, None]
    assert max_run * wmax * max(M // 2, 1) < (1 << 22)
    return dS


def _pow2_weights(batch, seed=3):
    rng = np.random.default_rng([seed, batch.nnz])
    return np.array([0.5, 1.0, 2.0], dtype=np.float32)[rng.integers(0, 3, size=batch.indices.shape)]


def _run_update(b, tables, dT, lr, mode, weights=None, state=None, eps=0.0):
    w = b.workload
    F = w.K + 1
    sb = make_sparse_batch(b, tables, weights=weights)
    ws = hot.alloc_workspace(sb)
    if mode == "sort":
        code = hot.BWD_SORT
    else:
        hot.dlrm_emb_bag_bwd_prepare(sb, ws)
        code = hot.BWD_SORT_PREPARED if mode == "prepared" else hot.BWD_SORT_PREPARED_FLAT
    if state is None:
        hot.dlrm_emb_bag_bwd_sgd(sb, dT, F * w.d, w.d, lr, ws, algo=code, dS_offset=w.d)
    else:
        hot.dlrm_emb_bag_bwd_adagrad(sb, hot.state_pointers(state), dT, F * w.d, w.d, lr, eps, ws, algo=code,
                                     dS_offset=w.d)
    counts = torch.zeros(10, dtype=torch.int32, device=DEV)
    hot.dlrm_emb_bag_bwd_route_counts(sb, ws, counts)
    torch.cuda.synchronize()
    return dict(zip(hot.ROUTE_NAMES, counts.cpu().tolist()))


def _assert_only_touched_rows_changed(before, after, uniq):
    changed = (before.view(torch.uint8).reshape(before.shape[0], -1) !=
               after.view(torch.uint8).reshape(after.shape[0], -1)).any(dim=1)
    rows = torch.nonzero(changed).flatten().cpu().numpy()
    assert np.isin(rows, uniq).all()


@pytest.mark.parametrize("weighted", [False, True], ids=["sum", "pow2-weights"])
@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_sgd_update_equals_the_oracle_on_exact_inputs(case, weighted):
    name, K, B, d, dtype, rows, bag, dist, routes = case
    w = gen.custom_workload(name, K=K, B=B, d=d, dtype=dtype, rows=rows, bag=bag, dist=dist, seed=21)
    b = gen.make_batch(w)
    wts = _pow2_weights(b) if weighted else None
    dS = _integer_dS(B, K, d, _max_run(b), 2.0 if weighted else 1.0)
    lr = 0.5 if dtype == gen.F32 else 2.0 ** -8
    start = _integer_tables(b.rows, d, dtype, seed=5)
    comp = Compact(b, host_rows_of=lambda k, u: table_to_numpy(
        start[k].index_select(0, torch.from_numpy(u).to(DEV)), dtype))
    ref = [t.copy() for t in comp.tables]
    if weighted:
        oracle.emb_bag_bwd_weighted(ref, dtype, comp.indices, b.offsets, b.tbl_off, wts, dS, lr)
    else:
        oracle.emb_bag_bwd_sgd(ref, dtype, comp.indices, b.offsets, b.tbl_off, dS, lr)
    F = K + 1
    dT = torch.zeros((B, F, d), dtype=torch.float32, device=DEV)
    dT[:, 1:, :] = torch.from_numpy(dS).to(DEV)
    for mode in MODES:
        _say("exact sgd %s weighted=%s %s" % (name, weighted, mode))
        tables = [t.clone() for t in start]
        counts = _run_update(b, tables, dT, lr, mode, weights=wts)
        print("        routes: " + ", ".join("%s=%d" % kv for kv in counts.items() if kv[1]), flush=True)
        for k in range(K):
            got = table_to_numpy(tables[k].index_select(0, torch.from_numpy(comp.uniq[k]).to(DEV)), dtype)
            assert np.array_equal(got.view(np.uint8), ref[k].view(np.uint8)), (name, mode, k)
            _assert_only_touched_rows_changed(start[k], tables[k], comp.uniq[k])
        if mode == "sort":
            for r in routes:
                if weighted and r == "dense_hot_tables":
                    assert counts[r] == 0      # weighted batches keep the entry-by-entry kernel
                else:
                    assert counts[r] > 0, (name, r, counts)
        if mode == "flat":
            assert counts["segments"] == 0 and counts["hot_rows"] == 0


@pytest.mark.parametrize("case", [c for c in CASES if c[0] in (
    "hot-rows", "hot-rows-large", "many-hot-rows", "dense-hot-rows-d256-f16", "segments-no-dominant-row",
    "dominant-rows-large-rest", "zipf12-fixed32-2Mrows-f16")], ids=lambda c: c[0])
def test_adagrad_state_equals_the_oracle_on_exact_inputs(case):
    """h <- h + g*g with integer g and a small integer h: the exact value rounded once, on both sides
    (fp32 fused multiply-add here, fp64 there), so the accumulators must be EQUAL -- a sum off by one
    lookup moves g*g by more than an fp32 unit in the last place at any run length.  W follows within the
    usual tolerance (its step divides by a square root)."""
    name, K, B, d, dtype, rows, bag, dist, _ = case
    w = gen.custom_workload(name, K=K, B=B, d=d, dtype=dtype, rows=rows, bag=bag, dist=dist, seed=22)
    b = gen.make_batch(w)
    dS = _integer_dS(B, K, d, _max_run(b))
    lr, eps = float(np.float32(0.05)), float(np.float32(1e-8))
    start = _integer_tables(b.rows, d, dtype, seed=6)
    g = torch.Generator(device=DEV).manual_seed(7)
    h_start = [torch.randint(1, 5, (int(m), d), generator=g, device=DEV, dtype=torch.int32).to(torch.float32)
               for m in b.rows]
    rows_of = lambda ts, dt: (lambda k, u: table_to_numpy(ts[k].index_select(0, torch.from_numpy(u).to(DEV)), dt))
    comp = Compact(b, host_rows_of=rows_of(start, dtype))
    h0 = [rows_of(h_start, gen.F32)(k, comp.uniq[k]) for k in range(K)]
    ref_w = [t.copy() for t in comp.tables]
    ref_h = [np.ascontiguousarray(h.copy()) for h in h0]
    oracle.emb_bag_bwd_adagrad(ref_w, ref_h, dtype, comp.indices, b.offsets, b.tbl_off, dS, lr, eps)
    sg = [np.zeros(t.shape, dtype=np.float32) for t in comp.tables]
    oracle.emb_bag_bwd_sgd(sg, gen.F32, comp.indices, b.offsets, b.tbl_off, np.abs(dS), -1.0)
    F = K + 1
    dT = torch.zeros((B, F, d), dtype=torch.float32, device=DEV)
    dT[:, 1:, :] = torch.from_numpy(dS).to(DEV)
    from hotpath_util import SCALE_FLOOR, TOL, rel_err, widen_host
    for mode in ("sort", "prepared"):
        _say("exact adagrad %s %s" % (name, mode))
        tables = [t.clone() for t in start]
        state = [h.clone() for h in h_start]
        counts = _run_update(b, tables, dT, lr, mode, state=state, eps=eps)
        print("        routes: " + ", ".join("%s=%d" % kv for kv in counts.items() if kv[1]), flush=True)
        for k in range(K):
            sel = torch.from_numpy(comp.uniq[k]).to(DEV)
            got_h = state[k].index_select(0, sel).cpu().numpy()
            assert np.array_equal(got_h.view(np.uint32), ref_h[k].view(np.uint32)), (name, mode, k)
            _assert_only_touched_rows_changed(h_start[k], state[k], comp.uniq[k])
            _assert_only_touched_rows_changed(start[k], tables[k], comp.uniq[k])
            got_w = widen_host(table_to_numpy(tables[k].index_select(0, sel), dtype), dtype)
            w0 = np.abs(widen_host(comp.tables[k], dtype))
            scale = w0 + lr * sg[k].astype(np.float64) / (np.sqrt(h0[k].astype(np.float64)) + eps)
            assert rel_err(got_w, widen_host(ref_w[k], dtype), scale, SCALE_FLOOR[dtype]) <= TOL[dtype]


def _random_shape(seed):
    """A small seeded shape off the beaten track: row widths of any multiple of 4, tables from one row to a few
    thousand, empty / one-hot / ragged / fixed bags, uniform or skewed indices, any of the three table types."""
    rng = np.random.default_rng([1906, seed])
    d = int(rng.choice([4, 8, 12, 16, 24, 32, 48, 64, 96, 128, 160, 256]))
    K = int(rng.integers(1, 7))
    B = int(rng.choice([1, 3, 17, 64, 257, 1000, 2048, 5000]))
    rows = int(rng.choice([1, 2, 7, 100, 1000, 4096, 30000]))
    bag = [("fixed", 1), ("fixed", int(rng.integers(2, 40))), ("uniform", 0, int(rng.integers(1, 60))),
           ("uniform", 1, 3)][int(rng.integers(0, 4))]
    dist = [("uniform",), ("zipf", 1.05), ("zipf", 1.4)][int(rng.integers(0, 3))]
    dtype = [gen.F32, gen.F16, gen.BF16][int(rng.integers(0, 3))]
    if dtype != gen.F32 and d % 8:
        d *= 2          # a 16-bit row is whole 16-byte pieces
    return K, B, d, dtype, rows, bag, dist


@pytest.mark.parametrize("seed", range(32))
def test_random_shapes_sgd_update_equals_the_oracle_on_exact_inputs(seed):
    """Thirty-two seeded random shapes through the same exact-arithmetic comparison, sum and weighted pooling,
    the complete call and the prepared one: whichever way the sorted entries fall into the lane groups' slabs
    (empty slabs, a run across several slabs, a run that ends on a slab boundary, a bucket smaller than the
    number of lane groups), every touched row must equal the oracle's and no other row may change."""
    K, B, d, dtype, rows, bag, dist = _random_shape(seed)
    name = "random-%d" % seed
    w = gen.custom_workload(name, K=K, B=B, d=d, dtype=dtype, rows=rows, bag=bag, dist=dist, seed=100 + seed)
    b = gen.make_batch(w)
    _say("exact sgd %s K=%d B=%d d=%d dtype=%s rows=%d bag=%s dist=%s nnz=%d" % (name, K, B, d, dtype, rows, bag, dist, b.nnz))
    lr = 0.5 if dtype == gen.F32 else 2.0 ** -8
    start = _integer_tables(b.rows, d, dtype, seed=5)
    comp = Compact(b, host_rows_of=lambda k, u: table_to_numpy(
        start[k].index_select(0, torch.from_numpy(u).to(DEV)), dtype))
    F = K + 1
    for weighted in (False, True):
        wts = _pow2_weights(b) if weighted else None
        dS = _integer_dS(B, K, d, max(_max_run(b), 1), 2.0 if weighted else 1.0)
        ref = [t.copy() for t in comp.tables]
        if weighted:
            oracle.emb_bag_bwd_weighted(ref, dtype, comp.indices, b.offsets, b.tbl_off, wts, dS, lr)
        else:
            oracle.emb_bag_bwd_sgd(ref, dtype, comp.indices, b.offsets, b.tbl_off, dS, lr)
        dT = torch.zeros((B, F, d), dtype=torch.float32, device=DEV)
        dT[:, 1:, :] = torch.from_numpy(dS).to(DEV)
        for mode in ("sort", "prepared"):
            tables = [t.clone() for t in start]
            _run_update(b, tables, dT, lr, mode, weights=wts)
            for k in range(K):
                got = table_to_numpy(tables[k].index_select(0, torch.from_numpy(comp.uniq[k]).to(DEV)), dtype)
                assert np.array_equal(got.view(np.uint8), ref[k].view(np.uint8)), (name, weighted, mode, k)
                _assert_only_touched_rows_changed(start[k], tables[k], comp.uniq[k])


def _random_hot_shape(seed):
    """Few rows, thousands of lookups each: every row is a hot row, and a table with at least 8 of them goes
    through the matrix-core kernel -- with bag counts that leave a last bag group, a last wavefront quarter and a
    last 64-bag tile partly empty, row widths of one, two and four 64-column pieces, and more hot rows than one
    pass holds."""
    rng = np.random.default_rng([5, seed])
    d = int(rng.choice([8, 32, 64, 96, 128, 160, 256]))
    K = int(rng.integers(1, 4))
    B = int(rng.choice([2500, 3000, 4096, 4099]))
    rows = int(rng.choice([3, 9, 20, 33, 40]))
    bag = ("fixed", int(rng.integers(25, 41)))
    rows = max(1, min(rows, B * bag[1] // 3000))   # about 3000 lookups a row or more
    dtype = [gen.F32, gen.F16][seed % 2]
    return K, B, d, dtype, rows, bag, ("uniform",)


@pytest.mark.parametrize("seed", range(10))
def test_random_hot_row_shapes_sgd_update_equals_the_oracle_on_exact_inputs(seed):
    K, B, d, dtype, rows, bag, dist = _random_hot_shape(seed)
    name = "random-hot-%d" % seed
    w = gen.custom_workload(name, K=K, B=B, d=d, dtype=dtype, rows=rows, bag=bag, dist=dist, seed=200 + seed)
    b = gen.make_batch(w)
    _say("exact sgd %s K=%d B=%d d=%d dtype=%s rows=%d bag=%s nnz=%d" % (name, K, B, d, dtype, rows, bag, b.nnz))
    lr = 0.5 if dtype == gen.F32 else 2.0 ** -8
    start = _integer_tables(b.rows, d, dtype, seed=5)
    comp = Compact(b, host_rows_of=lambda k, u: table_to_numpy(
        start[k].index_select(0, torch.from_numpy(u).to(DEV)), dtype))
    dS = _integer_dS(B, K, d, _max_run(b))
    ref = [t.copy() for t in comp.tables]
    oracle.emb_bag_bwd_sgd(ref, dtype, comp.indices, b.offsets, b.tbl_off, dS, lr)
    F = K + 1
    dT = torch.zeros((B, F, d), dtype=torch.float32, device=DEV)
    dT[:, 1:, :] = torch.from_numpy(dS).to(DEV)
    tables = [t.clone() for t in start]
    counts = _run_update(b, tables, dT, lr, "sort")
    print("        routes: " + ", ".join("%s=%d" % kv for kv in counts.items() if kv[1]), flush=True)
    hot_per_table = [int((np.bincount(b.indices_of(k)) > 2048).sum()) for k in range(K)]
    assert counts["hot_rows"] == sum(hot_per_table) > 0
    assert counts["dense_hot_tables"] == sum(1 for n in hot_per_table if n >= 8)
    for k in range(K):
        got = table_to_numpy(tables[k].index_select(0, torch.from_numpy(comp.uniq[k]).to(DEV)), dtype)
        assert np.array_equal(got.view(np.uint8), ref[k].view(np.uint8)), (name, k)
        _assert_only_touched_rows_changed(start[k], tables[k], comp.uniq[k])
