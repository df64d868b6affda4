"""GPU parity on seeded random shapes: table count, batch size, row width, storage type, table
size, bag-length mix, index distribution, weights, index type and optimizer are all drawn per case,
so that combinations nobody listed by hand are compared with the oracle too.  Same bar as the
hand-written cases: fp32 sums within 1e-5, fp16/bf16 tables within 1e-2, relative to the magnitude
of the sum behind the element; rows nobody looked up keep their bits."""
import numpy as np
import pytest
import torch

import paper_1906_00091_amd as hot
from oracle import oracle
from workloads import gen

from hotpath_util import (DEV, SCALE_FLOOR, TOL, abs_f32_tables, make_sparse_batch, rel_err, table_to_numpy,
                          upload_tables, widen_host)

pytestmark = pytest.mark.gpu

N_CASES = 40


def _draw_case(i):
    rng = np.random.default_rng(7000 + i)
    K = int(rng.integers(1, 7))
    d = 4 * int(rng.integers(1, 65))
    dtype = [gen.F32, gen.F32, gen.F16, gen.BF16][int(rng.integers(0, 4))]
    if dtype != gen.F32:
        d = (d + 7) // 8 * 8  # a table row is a whole number of 16-byte pieces
    rows = int(np.exp(rng.uniform(0.0, np.log(min(2.0e6, 6.0e6 / d)))))
    if rng.random() < 0.5:
        bag = ("fixed", int(rng.integers(1, 41)))
        mean = bag[1]
    else:
        hi = int(rng.integers(1, 80))
        bag = ("uniform", 0, hi)
        mean = hi / 2.0
    dist = ("uniform",) if rng.random() < 0.5 else ("zipf", float(rng.uniform(1.05, 1.5)))
    # lookups per case: up to ~250 K, so that the partition has many tiles and the oracle stays quick
    bmax = max(1, int(250000 / (K * max(mean, 1.0))))
    bmax = min(bmax, 20000)
    if rng.random() < 0.5:  # half of the cases near the cap, the rest anywhere below (log-uniform)
        B = int(rng.integers(max(1, bmax // 2), bmax + 1))
    else:
        B = int(np.exp(rng.uniform(0.0, np.log(bmax))))
    weighted = bool(rng.random() < 0.4)
    index32 = bool(rng.random() < 0.4)
    opt = "adagrad" if rng.random() < 0.4 else "sgd"
    return dict(K=K, B=B, d=d, dtype=dtype, rows=rows, bag=bag, dist=dist, weighted=weighted, index32=index32,
                opt=opt)


def _draw_large_case(i):
    """Millions of lookups on narrow rows: many partition tiles, the separate scan, buckets past the LDS
    sort, with whatever the draw makes of hot rows."""
    rng = np.random.default_rng(8000 + i)
    K = int(rng.integers(1, 4))
    d = 4 * int(rng.integers(1, 5))
    dtype = gen.F32 if d % 8 else [gen.F32, gen.F16, gen.BF16][int(rng.integers(0, 3))]
    rows = int(np.exp(rng.uniform(np.log(1000.0), np.log(4.0e6))))
    n = int(rng.integers(24, 100))
    bag = ("fixed", n) if rng.random() < 0.5 else ("uniform", 0, 2 * n)
    dist = ("uniform",) if rng.random() < 0.5 else ("zipf", float(rng.uniform(1.05, 1.3)))
    B = int(rng.uniform(1.0e6, 3.5e6) / (K * n))
    return dict(K=K, B=B, d=d, dtype=dtype, rows=rows, bag=bag, dist=dist, weighted=bool(rng.random() < 0.5),
                index32=bool(rng.random() < 0.5), opt="adagrad" if rng.random() < 0.5 else "sgd")


# hundreds of tables with enough lookups for the separate scan (one workgroup per table there)
MANY_TABLES = [
    dict(K=600, B=1000, d=8, dtype=gen.F32, rows=3000, bag=("fixed", 8), dist=("zipf", 1.2), weighted=False,
         index32=False, opt="sgd"),
    dict(K=700, B=900, d=16, dtype=gen.F16, rows=50, bag=("uniform", 0, 20), dist=("uniform",), weighted=True,
         index32=True, opt="adagrad"),
]

CASES = [_draw_case(i) for i in range(N_CASES)] + [_draw_large_case(i) for i in range(6)] + MANY_TABLES


def _id(c):
    return "K%d-B%d-d%d-t%d-m%d-%s%s-%s%s%s-%s" % (
        c["K"], c["B"], c["d"], c["dtype"], c["rows"], c["bag"][0], c["bag"][-1], c["dist"][0],
        "-wt" if c["weighted"] else "", "-i32" if c["index32"] else "", c["opt"])


@pytest.mark.parametrize("c", CASES, ids=[_id(c) for c in CASES])
def test_random_shape_forward_and_update_match_oracle(c):
    print("[case] random shape " + _id(c), flush=True)
    K, B, d, dtype = c["K"], c["B"], c["d"], c["dtype"]
    w = gen.custom_workload("random", K=K, B=B, d=d, dtype=dtype, rows=c["rows"], bag=c["bag"], dist=c["dist"],
                            seed=11)
    b = gen.make_batch(w)
    ones = np.ones(b.nnz, dtype=np.float32)
    wts = (gen.make_weights(b) * np.where(np.arange(b.nnz) % 4 == 0, -1.0, 1.0).astype(np.float32)
           if c["weighted"] else ones)
    host = [gen.init_table(b.seed, k, int(b.rows[k]), d, dtype) for k in range(K)]
    tables = upload_tables(host, dtype)
    sb = make_sparse_batch(b, tables, weights=wts if c["weighted"] else None, index32=c["index32"])
    F = K + 1

    # ---- forward (Eq. (2)), written into rows 1.. of T
    T = torch.full((B, F, d), 123.0, dtype=torch.float32, device=DEV)
    hot.dlrm_emb_bag_fwd(sb, T, F * d, d, out_offset=d)
    torch.cuda.synchronize()
    got = T.cpu().numpy()
    want = oracle.emb_bag_fwd_weighted(host, dtype, b.indices, b.offsets, b.tbl_off, wts)
    scale = oracle.emb_bag_fwd_weighted(abs_f32_tables(host, dtype), gen.F32, b.indices, b.offsets, b.tbl_off,
                                        np.abs(wts))
    assert np.all(got[:, 0, :] == 123.0)
    assert rel_err(got[:, 1:, :], want, scale) <= 1e-5

    # ---- the one-call forward gives the same pooled bits and the interaction of them
    if not c["weighted"] and K <= 64:
        x = np.random.default_rng(5).standard_normal((B, d)).astype(np.float32)
        T1 = torch.zeros((B, F, d), dtype=torch.float32, device=DEV)
        R1 = torch.zeros((B, d + F * (F - 1) // 2), dtype=torch.float32, device=DEV)
        hot.dlrm_emb_interact_fwd(sb, torch.from_numpy(x).to(DEV), T1, R1)
        torch.cuda.synchronize()
        assert torch.equal(T1[:, 1:, :], T[:, 1:, :])
        t1 = T1.cpu().numpy()
        assert np.array_equal(t1[:, 0, :].view(np.uint32), x.view(np.uint32))
        assert rel_err(R1.cpu().numpy(), oracle.interact_dot_fwd(t1), oracle.interact_dot_fwd(np.abs(t1))) <= 1e-5

    # ---- the grouping of the lookups by row (index work: bit-exact)
    ws = hot.alloc_workspace(sb)
    n = max(b.nnz, 1)
    uniq = torch.full((n,), -1, dtype=torch.int64, device=DEV)
    seg = torch.full((n,), -1, dtype=torch.int64, device=DEV)
    sbag = torch.full((n,), -1, dtype=torch.int32, device=DEV)
    nu = torch.full((K,), -1, dtype=torch.int64, device=DEV)
    hot.dlrm_emb_bag_bwd_export_groups(sb, ws, uniq, seg, sbag, nu)
    torch.cuda.synchronize()
    uniq, seg, sbag, nu = uniq.cpu().numpy(), seg.cpu().numpy(), sbag.cpu().numpy(), nu.cpu().numpy()
    groups = oracle.group_rows(b.indices, b.offsets, b.tbl_off)
    for k in range(K):
        a0, a1 = int(b.tbl_off[k]), int(b.tbl_off[k + 1])
        wu, wseg, wpos, wbag = groups[k]
        assert int(nu[k]) == len(wu)
        assert np.array_equal(uniq[a0:a0 + len(wu)], wu)
        assert np.array_equal(seg[a0:a0 + len(wu)], wseg)
        assert np.array_equal(sbag[a0:a1], wbag)

    # ---- backward fused with the row update (Sec. 5.1: SGD or Adagrad)
    dS = b.dS()
    dT = torch.zeros((B, F, d), dtype=torch.float32, device=DEV)
    dT[:, 1:, :] = torch.from_numpy(dS).to(DEV)
    lr, eps = float(np.float32(0.05)), float(np.float32(1e-8))
    ref_w = [t.copy() for t in host]
    sg = [np.zeros((int(r), d), dtype=np.float32) for r in b.rows]  # sum of the terms' magnitudes per row
    oracle.emb_bag_bwd_weighted(sg, gen.F32, b.indices, b.offsets, b.tbl_off, np.abs(wts), np.abs(dS), -1.0)
    h0 = [np.random.default_rng(13 + k).uniform(0.01, 1.0, size=(int(r), d)).astype(np.float32)
          for k, r in enumerate(b.rows)]
    if c["opt"] == "sgd":
        hot.dlrm_emb_bag_bwd_sgd(sb, dT, F * d, d, lr, ws, algo=hot.BWD_SORT, dS_offset=d)
        oracle.emb_bag_bwd_weighted(ref_w, dtype, b.indices, b.offsets, b.tbl_off, wts, dS, lr)
    else:
        state = [torch.from_numpy(h.copy()).to(DEV) for h in h0]
        hot.dlrm_emb_bag_bwd_adagrad(sb, hot.state_pointers(state), dT, F * d, d, lr, eps, ws, dS_offset=d)
        ref_h = [h.copy() for h in h0]
        oracle.emb_bag_bwd_weighted(ref_w, dtype, b.indices, b.offsets, b.tbl_off, wts, dS, lr, state=ref_h,
                                    eps=eps)
    torch.cuda.synchronize()
    for k in range(K):
        u = np.unique(b.indices_of(k))
        got_w = table_to_numpy(tables[k], dtype)
        mask = np.ones(int(b.rows[k]), dtype=bool)
        mask[u] = False
        assert np.array_equal(got_w[mask].view(np.uint8), host[k][mask].view(np.uint8))
        if len(u) == 0:
            continue
        S = sg[k][u].astype(np.float64)
        w0 = np.abs(widen_host(host[k][u], dtype)).astype(np.float64)
        gw, rw = widen_host(got_w[u], dtype), widen_host(ref_w[k][u], dtype)
        if c["opt"] == "sgd":
            assert rel_err(gw, rw, w0 + lr * S, SCALE_FLOOR[dtype]) <= TOL[dtype]
        else:
            got_h = state[k].cpu().numpy()
            assert np.array_equal(got_h[mask].view(np.uint32), h0[k][mask].view(np.uint32))
            assert rel_err(got_h[u], ref_h[k][u], h0[k][u] + S * S) <= 1e-5
            assert rel_err(gw, rw, w0 + lr * S / (np.sqrt(h0[k][u].astype(np.float64)) + eps),
                           SCALE_FLOOR[dtype]) <= TOL[dtype]


def _draw_interaction(i):
    rng = np.random.default_rng(9000 + i)
    F = int(rng.integers(1, 129))
    d = 4 * int(rng.integers(1, 65))
    B = int(np.exp(rng.uniform(0.0, np.log(max(2.0, 2.0e7 / (F * d))))))
    return B, F, d


INTERACTIONS = [_draw_interaction(i) for i in range(24)]


@pytest.mark.parametrize("B,F,d", INTERACTIONS)
def test_random_shape_interaction_matches_oracle(B, F, d):
    """Sec. 2.2: dots of all distinct pairs of the F vectors, the dense vector copied in front; and the
    transpose of that map applied to an upstream gradient."""
    print("[case] random interaction B=%d F=%d d=%d" % (B, F, d), flush=True)
    rng = np.random.default_rng(B * 1000 + F)
    P = F * (F - 1) // 2
    T = rng.standard_normal((B, F, d)).astype(np.float32)
    dR = rng.standard_normal((B, d + P)).astype(np.float32)
    Td = torch.from_numpy(T).to(DEV)
    R = torch.full((B, d + P), -5.0, dtype=torch.float32, device=DEV)
    hot.dlrm_interact_dot_fwd(Td, R)
    got = R.cpu().numpy()
    assert np.array_equal(got[:, :d].view(np.uint32), T[:, 0, :].view(np.uint32))
    assert rel_err(got, oracle.interact_dot_fwd(T), oracle.interact_dot_fwd(np.abs(T))) <= 1e-5
    dT = torch.full((B, F, d), -5.0, dtype=torch.float32, device=DEV)
    hot.dlrm_interact_dot_bwd(Td, torch.from_numpy(dR).to(DEV), dT)
    assert rel_err(dT.cpu().numpy(), oracle.interact_dot_bwd(T, dR),
                   oracle.interact_dot_bwd(np.abs(T), np.abs(dR))) <= 1e-5
