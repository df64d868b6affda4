"""The seeded input generators: deterministic, shaped as stated, no method arithmetic."""
import math

import numpy as np

from workloads import gen


def test_tiny_shapes_and_determinism():
    w = gen.WORKLOADS[1]
    a = gen.make_batch(w)
    b = gen.make_batch(w)
    assert np.array_equal(a.indices, b.indices) and np.array_equal(a.dR, b.dR)
    assert a.lengths.shape == (8, 128) and a.lengths.min() >= 1 and a.lengths.max() <= 4
    assert a.offsets.shape == (8, 129) and a.tbl_off[-1] == a.lengths.sum() == len(a.indices)
    assert a.x.shape == (128, 16) and a.dR.shape == (128, 16 + 36)
    assert a.indices.min() >= 0 and a.indices.max() < 1000
    c = gen.make_batch(w, batch_id=1)
    assert not np.array_equal(a.indices[:100], c.indices[:100])


def test_clicklog_shape_rows_and_zipf_skew():
    w = gen.WORKLOADS[2]
    rows = gen.table_rows(w)
    assert rows.shape == (26,) and rows.min() >= 3 and rows.max() <= 10_000_000
    b = gen.make_batch(w)
    assert np.all(b.lengths == 1) and b.nnz == 26 * 2048
    for k in range(w.K):
        idx = b.indices_of(k)
        assert idx.min() >= 0 and idx.max() < rows[k]
    big = int(np.argmax(rows))
    _, cnt = np.unique(b.indices_of(big), return_counts=True)
    assert cnt.max() > 20          # a heavy head: uniform draws over millions of rows would not repeat


def test_large_onehot_row_cap():
    w = gen.WORKLOADS[4]
    rows = gen.table_rows(w)
    assert rows.sum() <= 180_000_000 and rows.min() >= 1000


def test_hash_init_range_reproducibility_and_dtype():
    m, d = 1000, 16
    full = gen.init_table(0, 3, m, d, gen.F32)
    s = 1.0 / math.sqrt(m)
    assert full.dtype == np.float32 and np.abs(full).max() < s * 1.0000001
    assert abs(float(full.mean())) < 0.05 * s and float(full.std()) > 0.5 * s
    some = np.array([7, 999, 0, 512], dtype=np.int64)
    assert np.array_equal(gen.init_rows(0, 3, m, d, gen.F32, some), full[some])
    assert not np.array_equal(gen.init_table(0, 4, m, d, gen.F32), full)
    h = gen.init_rows(0, 3, m, d, gen.F16, some)
    assert h.dtype == np.float16 and np.array_equal(h, full[some].astype(np.float16))
    bf = gen.init_rows(0, 3, m, d, gen.BF16, some)
    back = (bf.astype(np.uint32) << 16).view(np.float32)
    assert np.all(np.abs(back - full[some]) <= np.abs(full[some]) * 2.0 ** -8)


def test_rank_to_row_map_is_a_bijection():
    w = gen.WORKLOADS[2]
    rows = gen.table_rows(w)
    A, C = gen._bijection_constants(w, rows, w.seed)
    for k in range(w.K):
        m = int(rows[k])
        if m > 200_000:
            continue
        img = (np.arange(m, dtype=np.int64) * A[k] + C[k]) % m
        assert len(np.unique(img)) == m


def test_batch_from_lists():
    b = gen.batch_from_lists([6], [[[0, 2], [0, 1, 5], [3]]], d=4)
    assert b.offsets.tolist() == [[0, 2, 5, 6]] and b.indices.tolist() == [0, 2, 0, 1, 5, 3]
