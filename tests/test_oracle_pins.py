"""Pins for the CPU oracle: every oracle function is checked against something
other than itself -- the example the paper prints, closed forms, library
routines (numpy matmul / unique / float16 casts), brute force on tiny inputs
and finite differences -- chosen so that a dropped term, a wrong sign or index,
or a transposed operand fails at least one of them.  No GPU needed."""
import os

import numpy as np
import pytest

from oracle import oracle
from workloads import gen

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            out[parts[0]] = [int(v) for v in parts[1:]]
    return out


def _rand_tables(rng, rows, d, dtype=gen.F32):
    ts = []
    for m in rows:
        w = rng.standard_normal((m, d)).astype(np.float32)
        if dtype == gen.F16:
            w = w.astype(np.float16)
        ts.append(w)
    return ts


def _dense_A(batch, k, m):
    """m x B multiplicity matrix of table k (the A of Eq. (2))."""
    A = np.zeros((m, batch.workload.B), dtype=np.float64)
    off = batch.offsets[k]
    idx = batch.indices_of(k)
    for b in range(batch.workload.B):
        for p in range(off[b], off[b + 1]):
            A[idx[p], b] += 1.0
    return A


# ---------------------------------------------------------------- CSR (Sec. 4.1)
def test_csr_example_lengths_to_offsets():
    g = _read_golden("csr_example.txt")
    lengths = np.array([g["lengths"]], dtype=np.int32)
    offsets, tbl_off = oracle.lengths_to_offsets(lengths)
    # the paper prints offsets without the terminator; ours appends nnz
    assert offsets[0, :-1].tolist() == g["offsets"]
    assert offsets[0, -1] == len(g["indices"])
    assert tbl_off.tolist() == [0, len(g["indices"])]


def test_csr_example_pooling_and_backward():
    g = _read_golden("csr_example.txt")
    d = 4
    W = (np.arange(6 * d, dtype=np.float32).reshape(6, d) + 1.0) * np.float32(0.25)
    lengths = np.array([g["lengths"]], dtype=np.int32)
    offsets, tbl_off = oracle.lengths_to_offsets(lengths)
    idx = np.array(g["indices"], dtype=np.int64)
    S = oracle.emb_bag_fwd([W], gen.F32, idx, offsets, tbl_off)
    W64 = W.astype(np.float64)
    assert np.array_equal(S[0, 0], W64[0] + W64[2])
    assert np.array_equal(S[1, 0], W64[0] + W64[1] + W64[5])
    assert np.array_equal(S[2, 0], W64[3])
    # backward: row 0 is looked up by bags 0 and 1, row 4 by nobody
    dS = np.array([[[1, 2, 3, 4]], [[10, 20, 30, 40]], [[100, 200, 300, 400]]], dtype=np.float32)
    uniq, grad = oracle.emb_bag_bwd_sgd([W.copy()], gen.F32, idx, offsets, tbl_off, dS, 0.5,
                                        apply=False, want_grad=True)
    assert uniq[0].tolist() == [0, 1, 2, 3, 5]
    assert np.array_equal(grad[0][0], dS[0, 0].astype(np.float64) + dS[1, 0])
    assert np.array_equal(grad[0][1], dS[1, 0])
    assert np.array_equal(grad[0][2], dS[0, 0])
    assert np.array_equal(grad[0][3], dS[2, 0])
    assert np.array_equal(grad[0][4], dS[1, 0])
    W2 = W.copy()
    oracle.emb_bag_bwd_sgd([W2], gen.F32, idx, offsets, tbl_off, dS, 0.5)
    assert np.array_equal(W2[4], W[4])
    assert np.array_equal(W2[0], (W64[0] - 0.5 * (dS[0, 0].astype(np.float64) + dS[1, 0])).astype(np.float32))


def test_lengths_to_offsets_matches_cumsum():
    rng = np.random.default_rng(1)
    lengths = rng.integers(0, 7, size=(5, 33)).astype(np.int32)
    offsets, tbl_off = oracle.lengths_to_offsets(lengths)
    assert np.array_equal(offsets[:, 0], np.zeros(5))
    assert np.array_equal(offsets[:, 1:], np.cumsum(lengths, axis=1))
    assert np.array_equal(tbl_off[1:], np.cumsum(lengths.sum(axis=1)))


def test_validate_csr_counts_violations():
    b = gen.make_batch(gen.WORKLOADS[1])
    assert oracle.validate_csr(b.rows, b.indices, b.offsets, b.tbl_off) == 0
    idx = b.indices.copy()
    idx[3] = -1
    idx[10] = b.rows[0]
    assert oracle.validate_csr(b.rows, idx, b.offsets, b.tbl_off) == 2
    off = b.offsets.copy()
    off[2, 5], off[2, 6] = off[2, 6] + 1, off[2, 5]
    assert oracle.validate_csr(b.rows, b.indices, off, b.tbl_off) >= 1


# ---------------------------------------------------------------- forward, Eq. (1)-(2)
def test_one_hot_lookup_is_row_gather_bitwise():
    rng = np.random.default_rng(2)
    w = gen.custom_workload("oh", K=3, B=50, d=8, rows=40, bag=("fixed", 1))
    b = gen.make_batch(w)
    tables = _rand_tables(rng, b.rows, w.d)
    S = oracle.emb_bag_fwd(tables, gen.F32, b.indices, b.offsets, b.tbl_off)
    for k in range(w.K):
        got = S[:, k, :].astype(np.float32)
        want = tables[k][b.indices_of(k)]
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("dtype", [gen.F32, gen.F16])
def test_multi_hot_equals_dense_AtW(dtype):
    rng = np.random.default_rng(3)
    w = gen.custom_workload("mh", K=3, B=17, d=12, rows=23, bag=("uniform", 0, 9), dtype=dtype)
    b = gen.make_batch(w)
    tables = _rand_tables(rng, b.rows, w.d, dtype)
    S = oracle.emb_bag_fwd(tables, dtype, b.indices, b.offsets, b.tbl_off)
    assert (b.lengths == 0).any()          # empty bags are in the draw
    for k in range(w.K):
        A = _dense_A(b, k, int(b.rows[k]))
        assert A.max() >= 2.0 or k > 0     # a repeated index inside a bag occurs
        want = A.T @ tables[k].astype(np.float64)
        np.testing.assert_allclose(S[:, k, :], want, rtol=1e-13, atol=1e-13)
    empty = np.argwhere(b.lengths == 0)
    for k, bb in empty:
        assert np.all(S[bb, k, :] == 0.0)


def test_pooling_is_linear_and_order_free():
    rng = np.random.default_rng(4)
    w = gen.custom_workload("lin", K=2, B=9, d=4, rows=30, bag=("uniform", 1, 6))
    b = gen.make_batch(w)
    W1 = _rand_tables(rng, b.rows, w.d)
    W2 = _rand_tables(rng, b.rows, w.d)
    # pick values that add exactly in fp32 so that W1 + W2 is formed without rounding
    W1 = [np.round(t * 64) / 64 for t in W1]
    W2 = [np.round(t * 64) / 64 for t in W2]
    f = lambda ts: oracle.emb_bag_fwd([t.astype(np.float32) for t in ts], gen.F32, b.indices,
                                      b.offsets, b.tbl_off)
    np.testing.assert_allclose(f([a + c for a, c in zip(W1, W2)]), f(W1) + f(W2), rtol=0, atol=1e-12)
    np.testing.assert_allclose(f([4 * a for a in W1]), 4 * f(W1), rtol=0, atol=0)
    # permuting the indices inside each bag does not change the sums (to rounding)
    idx = b.indices.copy()
    for k in range(w.K):
        for bb in range(w.B):
            lo, hi = b.tbl_off[k] + b.offsets[k, bb], b.tbl_off[k] + b.offsets[k, bb + 1]
            idx[lo:hi] = idx[lo:hi][::-1]
    S2 = oracle.emb_bag_fwd([t.astype(np.float32) for t in W1], gen.F32, idx, b.offsets, b.tbl_off)
    np.testing.assert_allclose(S2, f(W1), rtol=0, atol=1e-12)


def test_out_of_range_index_is_an_error():
    w = gen.custom_workload("bad", K=1, B=4, d=4, rows=10, bag=("fixed", 2))
    b = gen.make_batch(w)
    tables = [np.zeros((10, 4), dtype=np.float32)]
    idx = b.indices.copy()
    idx[0] = 10
    with pytest.raises(ValueError):
        oracle.emb_bag_fwd(tables, gen.F32, idx, b.offsets, b.tbl_off)


# ---------------------------------------------------------------- interaction (Sec. 2.2)
def test_pair_counts_match_stated_shapes():
    g = _read_golden("pair_counts.txt")
    for F, (P,) in ((int(k), v) for k, v in g.items()):
        T = np.zeros((1, F, 4), dtype=np.float32)
        assert oracle.interact_dot_fwd(T).shape[1] == 4 + P


def test_interaction_forward_is_strict_lower_triangle_of_gram():
    rng = np.random.default_rng(5)
    B, F, d = 6, 7, 10
    T = rng.standard_normal((B, F, d)).astype(np.float32)
    R = oracle.interact_dot_fwd(T)
    il, jl = np.tril_indices(F, -1)             # row-major order of the strict lower triangle
    assert il[:3].tolist() == [1, 2, 2] and jl[:3].tolist() == [0, 0, 1]
    for b in range(B):
        Z = T[b].astype(np.float64) @ T[b].astype(np.float64).T
        assert np.array_equal(R[b, :d].astype(np.float32).view(np.uint32), T[b, 0].view(np.uint32))
        np.testing.assert_allclose(R[b, d:], Z[il, jl], rtol=1e-13, atol=1e-13)
    # brute-force single entries, including which two vectors each column pairs
    b, i, j = 3, 5, 2
    q = d + i * (i - 1) // 2 + j
    want = sum(float(T[b, i, c]) * float(T[b, j, c]) for c in range(d))
    assert abs(R[b, q] - want) < 1e-12


def test_interaction_F2_closed_forms():
    rng = np.random.default_rng(6)
    B, d = 4, 5
    T = rng.standard_normal((B, 2, d)).astype(np.float32)
    dR = rng.standard_normal((B, d + 1)).astype(np.float32)
    R = oracle.interact_dot_fwd(T)
    T64 = T.astype(np.float64)
    np.testing.assert_allclose(R[:, d], np.einsum("bc,bc->b", T64[:, 0], T64[:, 1]), rtol=1e-14)
    dT = oracle.interact_dot_bwd(T, dR)
    g = dR[:, d].astype(np.float64)[:, None]
    np.testing.assert_allclose(dT[:, 0], g * T64[:, 1] + dR[:, :d], rtol=1e-14, atol=1e-14)
    np.testing.assert_allclose(dT[:, 1], g * T64[:, 0], rtol=1e-14, atol=1e-14)


def test_pooled_interaction_is_the_gram_of_dense_AtW_and_x():
    # the one-call forward against dense linear algebra: T_b = [x_b; (A_k^t W_k)_b], R = its Gram
    rng = np.random.default_rng(61)
    wl = gen.custom_workload("pi", K=3, B=5, d=8, rows=9, bag=("uniform", 0, 3))
    batch = gen.make_batch(wl)
    tables = _rand_tables(rng, batch.rows, wl.d)
    x = rng.standard_normal((wl.B, wl.d)).astype(np.float32)
    T, R = oracle.emb_interact_fwd(tables, gen.F32, batch.indices, batch.offsets, batch.tbl_off, x)
    assert T.dtype == np.float32 and np.array_equal(T[:, 0].view(np.uint32), x.view(np.uint32))
    il, jl = np.tril_indices(wl.K + 1, -1)
    for b in range(wl.B):
        rows = [x[b].astype(np.float64)]
        for k in range(wl.K):
            rows.append((_dense_A(batch, k, int(batch.rows[k])).T @ tables[k].astype(np.float64))[b])
        V = np.stack(rows)
        np.testing.assert_allclose(T[b], V, rtol=2e-7, atol=1e-7)
        np.testing.assert_allclose(R[b, wl.d:], (V @ V.T)[il, jl], rtol=2e-6, atol=2e-6)
        assert np.array_equal(R[b, :wl.d].astype(np.float32).view(np.uint32), x[b].view(np.uint32))


def test_interaction_backward_matches_finite_differences():
    rng = np.random.default_rng(7)
    B, F, d = 3, 5, 6
    # values on a 2^-10 grid, so that T +/- h is formed exactly in fp32
    T = (np.round(rng.standard_normal((B, F, d)) * 1024) / 1024).astype(np.float32)
    U = rng.standard_normal((B, d + F * (F - 1) // 2)).astype(np.float32)
    dT = oracle.interact_dot_bwd(T, U)
    loss = lambda Tx: float(np.sum(oracle.interact_dot_fwd(Tx) * U.astype(np.float64)))
    h = 2.0 ** -10
    num = np.zeros_like(dT)
    for idx in np.ndindex(B, F, d):
        Tp, Tm = T.copy(), T.copy()
        Tp[idx] += np.float32(h)
        Tm[idx] -= np.float32(h)
        num[idx] = (loss(Tp) - loss(Tm)) / (2 * h)
    # L is quadratic in T, so central differences are exact up to rounding
    np.testing.assert_allclose(dT, num, rtol=1e-8, atol=1e-8)


def test_interaction_backward_is_symmetric_product():
    rng = np.random.default_rng(8)
    B, F, d = 2, 6, 4
    T = rng.standard_normal((B, F, d)).astype(np.float32)
    dR = rng.standard_normal((B, d + F * (F - 1) // 2)).astype(np.float32)
    dT = oracle.interact_dot_bwd(T, dR)
    il, jl = np.tril_indices(F, -1)
    for b in range(B):
        G = np.zeros((F, F))
        G[il, jl] = dR[b, d:]
        want = (G + G.T) @ T[b].astype(np.float64)
        want[0] += dR[b, :d]
        np.testing.assert_allclose(dT[b], want, rtol=1e-13, atol=1e-13)


# ---------------------------------------------------------------- grouping
def test_grouping_matches_numpy_unique():
    w = gen.custom_workload("grp", K=4, B=64, d=4, rows=37, bag=("uniform", 0, 5))
    b = gen.make_batch(w)
    groups = oracle.group_rows(b.indices, b.offsets, b.tbl_off)
    for k, (uniq, seg, spos, sbag) in enumerate(groups):
        idx = b.indices_of(k)
        u, cnt = np.unique(idx, return_counts=True)
        assert np.array_equal(uniq, u)
        assert np.all(np.diff(uniq) > 0)
        ends = np.append(seg[1:], len(idx))
        assert np.array_equal(ends - seg, cnt)
        assert int(cnt.sum()) == len(idx)
        assert np.array_equal(np.sort(spos), np.arange(len(idx)))
        assert np.array_equal(idx[spos], np.repeat(u, cnt))
        for s, e in zip(seg, ends):                      # ascending position inside a row's run
            assert np.all(np.diff(spos[s:e]) > 0)
        bag_of = np.repeat(np.arange(w.B), b.lengths[k])
        assert np.array_equal(sbag, bag_of[spos])


# ---------------------------------------------------------------- embedding backward + SGD
def test_embedding_backward_equals_dense_A_dS():
    w = gen.custom_workload("bwd", K=3, B=21, d=6, rows=19, bag=("uniform", 0, 7))
    b = gen.make_batch(w)
    rng = np.random.default_rng(9)
    tables = _rand_tables(rng, b.rows, w.d)
    dS = b.dS()
    uniq, grad = oracle.emb_bag_bwd_sgd([t.copy() for t in tables], gen.F32, b.indices, b.offsets,
                                        b.tbl_off, dS, 0.1, apply=False, want_grad=True)
    for k in range(w.K):
        A = _dense_A(b, k, int(b.rows[k]))
        dW = A @ dS[:, k, :].astype(np.float64)
        touched = np.flatnonzero(A.sum(axis=1) > 0)
        assert np.array_equal(uniq[k], touched)
        np.testing.assert_allclose(grad[k], dW[touched], rtol=1e-13, atol=1e-13)


def test_same_gradient_everywhere_gives_count_times_g():
    w = gen.custom_workload("cnt", K=2, B=32, d=4, rows=8, bag=("fixed", 4))
    b = gen.make_batch(w)
    g = np.array([1.0, -2.0, 0.5, 3.0], dtype=np.float32)
    dS = np.broadcast_to(g, (w.B, w.K, w.d)).copy()
    tables = [np.zeros((8, 4), dtype=np.float32) for _ in range(w.K)]
    oracle.emb_bag_bwd_sgd(tables, gen.F32, b.indices, b.offsets, b.tbl_off, dS, 1.0)
    for k in range(w.K):
        cnt = np.bincount(b.indices_of(k), minlength=8).astype(np.float32)
        assert np.array_equal(tables[k], -cnt[:, None] * g[None, :])


def test_sgd_lr_zero_linearity_and_untouched_rows():
    w = gen.custom_workload("sgd", K=2, B=16, d=8, rows=50, bag=("uniform", 1, 3))
    b = gen.make_batch(w)
    rng = np.random.default_rng(10)
    tables = _rand_tables(rng, b.rows, w.d)
    dS = b.dS()
    t0 = [t.copy() for t in tables]
    oracle.emb_bag_bwd_sgd(t0, gen.F32, b.indices, b.offsets, b.tbl_off, dS, 0.0)
    for a, c in zip(t0, tables):
        assert np.array_equal(a.view(np.uint32), c.view(np.uint32))
    # exact-arithmetic check of linearity in lr on a grid of representable values
    tg = [(np.round(t * 256) / 256).astype(np.float32) for t in tables]
    dSg = (np.round(dS * 256) / 256).astype(np.float32)
    t1 = [t.copy() for t in tg]
    t2 = [t.copy() for t in tg]
    oracle.emb_bag_bwd_sgd(t1, gen.F32, b.indices, b.offsets, b.tbl_off, dSg, 0.25)
    oracle.emb_bag_bwd_sgd(t2, gen.F32, b.indices, b.offsets, b.tbl_off, dSg, 0.5)
    for k in range(w.K):
        np.testing.assert_array_equal((t2[k] - tg[k]), 2 * (t1[k] - tg[k]))
        touched = np.unique(b.indices_of(k))
        mask = np.ones(int(b.rows[k]), dtype=bool)
        mask[touched] = False
        assert np.array_equal(t1[k][mask], tg[k][mask])
        assert np.all(np.any(t1[k][touched] != tg[k][touched], axis=1))


def test_whole_chain_gradient_matches_finite_differences():
    """d/dW of L = sum(R * U) through pooling and interaction, against central
    differences on the table entries (fp64 oracle outputs; the tables live on a
    2^-8 grid so W +/- h is exact in fp32)."""
    w = gen.custom_workload("fd", K=2, B=5, d=4, rows=6, bag=("uniform", 1, 3))
    b = gen.make_batch(w)
    rng = np.random.default_rng(11)
    tables = [(np.round(rng.standard_normal((6, 4)) * 256) / 256).astype(np.float32) for _ in range(2)]
    U = b.dR

    def fwd(ts):
        S = oracle.emb_bag_fwd(ts, gen.F32, b.indices, b.offsets, b.tbl_off)
        T = np.concatenate([b.x[:, None, :].astype(np.float64), S], axis=1)
        # the pooled sums of grid values are exact in fp32, so this cast loses nothing
        T32 = T.astype(np.float32)
        assert np.array_equal(T32.astype(np.float64), T)
        return T32

    T = fwd(tables)
    dT = oracle.interact_dot_bwd(T, U)
    dS = dT[:, 1:, :]
    dS32 = dS.astype(np.float32)
    uniq, grad = oracle.emb_bag_bwd_sgd([t.copy() for t in tables], gen.F32, b.indices, b.offsets,
                                        b.tbl_off, dS32, 1.0, apply=False, want_grad=True)
    loss = lambda ts: float(np.sum(oracle.interact_dot_fwd(fwd(ts)) * U.astype(np.float64)))
    h = 2.0 ** -8
    for k in range(2):
        for ui, r in enumerate(uniq[k]):
            for c in range(4):
                tp = [t.copy() for t in tables]
                tm = [t.copy() for t in tables]
                tp[k][r, c] += np.float32(h)
                tm[k][r, c] -= np.float32(h)
                num = (loss(tp) - loss(tm)) / (2 * h)
                # dS was rounded to fp32 before the scatter: allow that much
                assert abs(num - grad[k][ui, c]) <= 1e-5 * max(1.0, abs(num))


# ---------------------------------------------------------------- fp16 / bf16 storage
def test_half_widening_exhaustive_against_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = oracle.half_to_double(bits)
    both_nan = np.isnan(want) & np.isnan(got)
    assert np.array_equal(got[~both_nan], want[~both_nan])
    assert both_nan.sum() == np.isnan(want).sum()


def test_half_narrowing_rne_against_numpy_including_ties():
    bits = np.arange(0, 0x7C00, dtype=np.uint16)          # all non-negative finite halves
    v = bits.view(np.float16).astype(np.float64)
    mid = (v[:-1] + v[1:]) / 2                            # exact ties between neighbours
    eps = np.abs(mid) * 2.0 ** -30 + 2.0 ** -60
    cases = np.concatenate([v, mid, mid + eps, mid - eps, -v, -mid, [65519.9, 65520.0, 1e-9, 7e4]])
    with np.errstate(over="ignore"):
        want = cases.astype(np.float16).view(np.uint16)
    got = oracle.double_to_half(cases)
    assert np.array_equal(got, want)


def test_bf16_roundtrip_and_rne():
    rng = np.random.default_rng(12)
    bits = rng.integers(0, 0x7F80, size=4000).astype(np.uint16)
    v = oracle.bf16_to_double(bits)
    want = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert np.array_equal(v, want)
    assert np.array_equal(oracle.double_to_bf16(v), bits)
    nxt = ((bits + 1).astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    ok = np.isfinite(nxt)
    mid = (v + nxt) / 2
    even = np.where(bits % 2 == 0, bits, bits + 1).astype(np.uint16)
    assert np.array_equal(oracle.double_to_bf16(mid[ok]), even[ok])
    assert np.array_equal(oracle.double_to_bf16(mid[ok] * (1 + 2.0 ** -40)), (bits + 1)[ok])


def test_fp16_tables_update_rounds_once():
    w = gen.custom_workload("h", K=1, B=8, d=8, rows=12, bag=("fixed", 3), dtype=gen.F16)
    b = gen.make_batch(w)
    rng = np.random.default_rng(13)
    W = (rng.standard_normal((12, 8)) * 0.03).astype(np.float16)
    dS = b.dS()
    W2 = W.copy()
    uniq, grad = oracle.emb_bag_bwd_sgd([W2], gen.F16, b.indices, b.offsets, b.tbl_off, dS, 0.01,
                                        want_grad=True)
    lr = 0.01
    for ui, r in enumerate(uniq[0]):
        want = (W[r].astype(np.float64) - lr * grad[0][ui]).astype(np.float16)
        assert np.array_equal(W2[r].view(np.uint16), want.view(np.uint16))


# ------------------------------------------------------------------ sparse Adagrad (Sec. 5.1)
def _one_table_batch(rows, lists, d):
    return gen.batch_from_lists([rows], [lists], d=d)


def test_adagrad_closed_forms_single_row():
    # one row, one lookup, g = 2, h0 = 0, eps = 0: h = 4, W = 1 - 0.1 * 2 / 2 = 0.9 (to fp32)
    b = _one_table_batch(3, [[1]], d=2)
    dS = np.array([[[2.0, -4.0]]], dtype=np.float32)
    W = [np.ones((3, 2), dtype=np.float32)]
    h = [np.zeros((3, 2), dtype=np.float32)]
    oracle.emb_bag_bwd_adagrad(W, h, gen.F32, b.indices, b.offsets, b.tbl_off, dS, 0.1, 0.0)
    assert np.array_equal(h[0][1], np.array([4.0, 16.0], dtype=np.float32))
    assert np.array_equal(W[0][1], np.array([np.float32(1.0 - 0.1), np.float32(1.0 + 0.1)]))
    # from h = 0 with eps = 0 the first step is lr * sign(g) whatever |g| is
    assert np.array_equal(W[0][[0, 2]], np.ones((2, 2), dtype=np.float32))
    assert np.array_equal(h[0][[0, 2]], np.zeros((2, 2), dtype=np.float32))
    # n steps with the same gradient: h = n g^2, W = 1 - lr * sum_{i<=n} 1/sqrt(i)
    W = [np.ones((3, 2), dtype=np.float64).astype(np.float32)]
    h = [np.zeros((3, 2), dtype=np.float32)]
    dS = np.array([[[0.5, 0.5]]], dtype=np.float32)
    for _ in range(9):
        oracle.emb_bag_bwd_adagrad(W, h, gen.F32, b.indices, b.offsets, b.tbl_off, dS, 0.01, 0.0)
    assert np.array_equal(h[0][1], np.full(2, 9 * 0.25, dtype=np.float32))
    want = 1.0 - 0.01 * sum(1.0 / np.sqrt(i) for i in range(1, 10))
    assert np.allclose(W[0][1], want, rtol=0, atol=5e-7)
    # eps enters outside the square root: g = 3, h0 = 16 -> h = 25, W = 1 - 1 * 3 / (5 + 1)
    W = [np.ones((3, 2), dtype=np.float32)]
    h = [np.full((3, 2), 16.0, dtype=np.float32)]
    dS = np.array([[[3.0, -3.0]]], dtype=np.float32)
    oracle.emb_bag_bwd_adagrad(W, h, gen.F32, b.indices, b.offsets, b.tbl_off, dS, 1.0, 1.0)
    assert np.array_equal(W[0][1], np.array([0.5, 1.5], dtype=np.float32))


def test_adagrad_sums_duplicates_before_squaring():
    # row 2 is looked up by three bags with gradients 1, 2, -0.5: h = (2.5)^2, not 1 + 4 + 0.25
    b = _one_table_batch(4, [[2], [2, 0], [2]], d=1)
    dS = np.array([[[1.0]], [[2.0]], [[-0.5]]], dtype=np.float32)
    W = [np.zeros((4, 1), dtype=np.float32)]
    h = [np.zeros((4, 1), dtype=np.float32)]
    oracle.emb_bag_bwd_adagrad(W, h, gen.F32, b.indices, b.offsets, b.tbl_off, dS, 1.0, 0.0)
    assert h[0][2, 0] == np.float32(6.25) and W[0][2, 0] == np.float32(-1.0)
    assert h[0][0, 0] == np.float32(4.0) and W[0][0, 0] == np.float32(-1.0)
    assert np.all(h[0][[1, 3]] == 0) and np.all(W[0][[1, 3]] == 0)


def test_adagrad_matches_the_library_optimizer_on_dense_gradients():
    torch = pytest.importorskip("torch")
    w = gen.custom_workload("ada", K=2, B=40, d=8, rows=30, bag=("uniform", 0, 5))
    b = gen.make_batch(w)
    rng = np.random.default_rng(3)
    tables = _rand_tables(rng, b.rows, w.d)
    state = [np.zeros_like(t) for t in tables]
    params = [torch.nn.Parameter(torch.from_numpy(t.copy())) for t in tables]
    opt = torch.optim.Adagrad(params, lr=0.05, eps=1e-10, initial_accumulator_value=0.0)
    for step in range(3):
        dS = rng.standard_normal((w.B, w.K, w.d)).astype(np.float32)
        # the dense gradient of every table by the library's scatter-add; untouched rows get 0,
        # for which the dense optimizer changes nothing either
        for k in range(w.K):
            dense = torch.zeros(int(b.rows[k]), w.d, dtype=torch.float64)
            off = b.offsets[k]
            bag_of = np.repeat(np.arange(w.B), np.diff(off))
            dense.index_add_(0, torch.from_numpy(b.indices_of(k)),
                             torch.from_numpy(dS[bag_of, k, :].astype(np.float64)))
            params[k].grad = dense.to(torch.float32)
        opt.step()
        oracle.emb_bag_bwd_adagrad(tables, state, gen.F32, b.indices, b.offsets, b.tbl_off, dS, 0.05, 1e-10)
        for k in range(w.K):
            touched = np.unique(b.indices_of(k))
            lib_w = params[k].detach().numpy()
            lib_h = opt.state[params[k]]["sum"].numpy()
            # the library works in fp32 throughout, the oracle in fp64 with one rounding
            assert np.allclose(tables[k], lib_w, rtol=2e-6, atol=1e-7), (step, k)
            assert np.allclose(state[k], lib_h, rtol=2e-6, atol=1e-9), (step, k)
            mask = np.ones(int(b.rows[k]), dtype=bool)
            mask[touched] = False
            assert np.all(state[k][mask] == 0)


def test_adagrad_fp16_tables_round_once_and_keep_untouched_rows():
    b = _one_table_batch(5, [[4], [1, 4]], d=2)
    dS = np.array([[[1.0, 1.0]], [[1.0, 3.0]]], dtype=np.float32)
    W16 = np.full((5, 2), 0.1, dtype=np.float16)
    W = [W16.copy()]
    h = [np.full((5, 2), 5.0, dtype=np.float32)]
    oracle.emb_bag_bwd_adagrad(W, h, gen.F16, b.indices, b.offsets, b.tbl_off, dS, 0.01, 1e-10)
    w0 = float(np.float16(0.1))
    # row 4: g = (2, 4) -> h = (9, 21); row 1: g = (1, 3) -> h = (6, 14)
    assert np.array_equal(h[0][4], np.array([9.0, 21.0], dtype=np.float32))
    assert np.array_equal(h[0][1], np.array([6.0, 14.0], dtype=np.float32))
    want4 = np.array([w0 - 0.01 * 2 / 3.0, w0 - 0.01 * 4 / np.sqrt(21.0)]).astype(np.float16)
    want1 = np.array([w0 - 0.01 * 1 / np.sqrt(6.0), w0 - 0.01 * 3 / np.sqrt(14.0)]).astype(np.float16)
    assert np.array_equal(W[0][4].view(np.uint16), want4.view(np.uint16))
    assert np.array_equal(W[0][1].view(np.uint16), want1.view(np.uint16))
    assert np.array_equal(W[0][[0, 2, 3]].view(np.uint16), W16[[0, 2, 3]].view(np.uint16))
    assert np.all(h[0][[0, 2, 3]] == 5.0)


# ------------------------------------------------------------------ weighted pooling, Eq. (2) in full
def test_weighted_pooling_is_the_dense_weighted_matrix_product():
    w = gen.custom_workload("wp", K=3, B=20, d=6, rows=15, bag=("uniform", 0, 6))
    b = gen.make_batch(w)
    rng = np.random.default_rng(5)
    tables = _rand_tables(rng, b.rows, w.d)
    a = rng.uniform(-2, 2, size=b.indices.shape).astype(np.float32)
    S = oracle.emb_bag_fwd_weighted(tables, gen.F32, b.indices, b.offsets, b.tbl_off, a)
    dS = rng.standard_normal((w.B, w.K, w.d)).astype(np.float32)
    upd = [t.copy() for t in tables]
    oracle.emb_bag_bwd_weighted(upd, gen.F32, b.indices, b.offsets, b.tbl_off, a, dS, 1.0)
    for k in range(w.K):
        # A[i, b] = sum of the weights with which bag b looks row i up (Eq. (2): S = A^T W)
        A = np.zeros((int(b.rows[k]), w.B))
        off = b.offsets[k]
        bag_of = np.repeat(np.arange(w.B), np.diff(off))
        np.add.at(A, (b.indices_of(k), bag_of), a[b.tbl_off[k]:b.tbl_off[k + 1]].astype(np.float64))
        assert np.allclose(S[:, k, :], A.T @ tables[k].astype(np.float64), rtol=1e-12, atol=1e-12)
        want = tables[k].astype(np.float64) - A @ dS[:, k, :].astype(np.float64)
        assert np.allclose(upd[k], want.astype(np.float32), rtol=0, atol=1e-6)


def test_unit_weights_are_the_unweighted_functions_and_repeats_add_their_weights():
    w = gen.custom_workload("wu", K=2, B=16, d=4, rows=9, bag=("uniform", 0, 5))
    b = gen.make_batch(w)
    rng = np.random.default_rng(6)
    tables = _rand_tables(rng, b.rows, w.d)
    ones = np.ones(b.indices.shape, dtype=np.float32)
    assert np.array_equal(oracle.emb_bag_fwd_weighted(tables, gen.F32, b.indices, b.offsets, b.tbl_off, ones),
                          oracle.emb_bag_fwd(tables, gen.F32, b.indices, b.offsets, b.tbl_off))
    dS = b.dS()
    t1 = [t.copy() for t in tables]
    t2 = [t.copy() for t in tables]
    oracle.emb_bag_bwd_sgd(t1, gen.F32, b.indices, b.offsets, b.tbl_off, dS, 0.1)
    oracle.emb_bag_bwd_weighted(t2, gen.F32, b.indices, b.offsets, b.tbl_off, ones, dS, 0.1)
    for x, y in zip(t1, t2):
        assert np.array_equal(x.view(np.uint32), y.view(np.uint32))
    h1 = [np.zeros_like(t) for t in tables]
    h2 = [np.zeros_like(t) for t in tables]
    oracle.emb_bag_bwd_adagrad(t1, h1, gen.F32, b.indices, b.offsets, b.tbl_off, dS, 0.1, 1e-8)
    oracle.emb_bag_bwd_weighted(t2, gen.F32, b.indices, b.offsets, b.tbl_off, ones, dS, 0.1, state=h2, eps=1e-8)
    for x, y in zip(t1 + h1, t2 + h2):
        assert np.array_equal(x.view(np.uint32), y.view(np.uint32))
    # one bag looks row 3 up twice, with weights 0.25 and -2: the row counts (0.25 - 2) times
    bb = gen.batch_from_lists([5], [[[3, 1, 3]]], d=2)
    W = [np.arange(10, dtype=np.float32).reshape(5, 2)]
    a = np.array([0.25, 1.0, -2.0], dtype=np.float32)
    S = oracle.emb_bag_fwd_weighted(W, gen.F32, bb.indices, bb.offsets, bb.tbl_off, a)
    assert np.array_equal(S[0, 0], -1.75 * W[0][3].astype(np.float64) + W[0][1])
    dS1 = np.array([[[1.0, 2.0]]], dtype=np.float32)
    oracle.emb_bag_bwd_weighted(W, gen.F32, bb.indices, bb.offsets, bb.tbl_off, a, dS1, 1.0)
    assert np.array_equal(W[0][3], np.array([6.0 + 1.75, 7.0 + 3.5], dtype=np.float32))
    assert np.array_equal(W[0][1], np.array([2.0 - 1.0, 3.0 - 2.0], dtype=np.float32))


def test_emb_interact_bwd_is_the_chain_rule_through_pooling_and_interaction():
    """The composed backward against central finite differences of L = sum(R * U) with respect to the
    dense vector and to the pooled vectors (moved through one table row of a one-index bag)."""
    rng = np.random.default_rng(31)
    K, B, d, m = 3, 4, 8, 6
    tables = [rng.standard_normal((m, d)).astype(np.float32) for _ in range(K)]
    bags = [[[int(rng.integers(0, m))] for _ in range(B)] for _ in range(K)]
    bags[1][2] = [1, 4, 4]          # one multi-index bag with a repeat
    b = gen.batch_from_lists([m] * K, bags, d)
    x = rng.standard_normal((B, d)).astype(np.float32)
    F = K + 1
    U = rng.standard_normal((B, d + F * (F - 1) // 2)).astype(np.float32)
    dT = oracle.emb_interact_bwd(tables, gen.F32, b.indices, b.offsets, b.tbl_off, x, U)

    def loss(tabs, xx):
        _, R = oracle.emb_interact_fwd(tabs, gen.F32, b.indices, b.offsets, b.tbl_off, xx)
        return float((R * U).sum())
    eps = 1e-3
    for (bb, c) in ((0, 0), (3, 5)):                      # dense vector
        xp, xm = x.copy(), x.copy()
        xp[bb, c] += eps
        xm[bb, c] -= eps
        fd = (loss(tables, xp) - loss(tables, xm)) / (2 * eps)
        assert abs(fd - dT[bb, 0, c]) <= 2e-3 * max(1.0, abs(fd))
    # a table row looked up once, by bag (k=0, b=1) only: dL/dW = dT[b, k+1]
    k, bb = 0, 1
    r = bags[k][bb][0]
    others = sum(1 for q in range(B) for i in bags[k][q] if i == r)
    if others == 1:
        for c in (2, 7):
            tp = [t.copy() for t in tables]
            tm = [t.copy() for t in tables]
            tp[k][r, c] += eps
            tm[k][r, c] -= eps
            fd = (loss(tp, x) - loss(tm, x)) / (2 * eps)
            assert abs(fd - dT[bb, k + 1, c]) <= 2e-3 * max(1.0, abs(fd))
