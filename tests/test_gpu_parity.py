"""GPU parity: every C-ABI entry point against the CPU oracle on the same seeded
inputs.  Integer / index work must match bit for bit; floating point within
1e-5 (fp32 tables) or 1e-2 (fp16/bf16 tables) max error relative to the magnitude
of the sum that produced the element, sum_j |term_j| (the oracle run on absolute
values; equal to |reference| where nothing cancels)."""
import numpy as np
import pytest
import torch

import paper_1906_00091_amd as hot
from paper_1906_00091_amd import ceilings
from oracle import oracle
from workloads import gen

from hotpath_util import (DEV, SCALE_FLOOR, TOL, make_sparse_batch, rel_err, scale_emb_fwd, scale_interact_bwd,
                          scale_interact_fwd, scale_sgd, table_to_numpy, upload_tables, widen_host)

pytestmark = pytest.mark.gpu


def _say(msg):
    print("[case] " + msg, flush=True)


def _host_tables(batch, scale=1.0):
    w = batch.workload
    return [gen.init_table(batch.seed, k, int(batch.rows[k]), w.d, w.dtype) for k in range(w.K)]


# ------------------------------------------------------------------ helpers around the path
def test_lengths_to_offsets_bit_exact():
    rng = np.random.default_rng(0)
    for K, B, hi in [(1, 3, 4), (8, 128, 5), (3, 5000, 300), (26, 2048, 2)]:
        _say("lengths_to_offsets K=%d B=%d" % (K, B))
        lengths = rng.integers(0, hi, size=(K, B)).astype(np.int32)
        if K == 1:
            lengths = np.array([[2, 3, 1]], dtype=np.int32)       # the example of Sec. 4.1
        want_off, want_tbl = oracle.lengths_to_offsets(lengths)
        off = torch.full((K, B + 1), -7, dtype=torch.int64, device=DEV)
        tbl = torch.full((K + 1,), -7, dtype=torch.int64, device=DEV)
        hot.dlrm_lengths_to_offsets(torch.from_numpy(lengths).to(DEV), off, tbl)
        assert np.array_equal(off.cpu().numpy(), want_off)
        assert np.array_equal(tbl.cpu().numpy(), want_tbl)


def test_validate_csr_counts_like_the_oracle():
    b = gen.make_batch(gen.WORKLOADS[1])
    tables = upload_tables(_host_tables(b), gen.F32)
    n_bad = torch.zeros(1, dtype=torch.int64, device=DEV)
    sb = make_sparse_batch(b, tables)
    hot.dlrm_validate_csr(sb, n_bad)
    assert int(n_bad.item()) == 0
    idx = b.indices.copy()
    idx[[3, 500, 900]] = [-1, 1000, 1 << 40]
    off = b.offsets.copy()
    off[2, 5], off[2, 6] = off[2, 6] + 1, off[2, 5]
    want = oracle.validate_csr(b.rows, idx, off, b.tbl_off)
    bad = gen.Batch(b.workload, b.rows, b.lengths, off, b.tbl_off, idx, b.x, b.dR)
    hot.dlrm_validate_csr(make_sparse_batch(bad, tables), n_bad)
    assert int(n_bad.item()) == want and want >= 4


@pytest.mark.parametrize("dtype", [gen.F32, gen.F16, gen.BF16])
def test_table_init_hash_matches_host_generator_bitwise(dtype):
    m, d = 3001, 24
    t = torch.empty((m, d), dtype={0: torch.float32, 1: torch.float16, 2: torch.bfloat16}[dtype],
                    device=DEV)
    hot.dlrm_table_init_hash(t, dtype, gen.table_key(5, 3), float(gen.table_scale(m)))
    got = table_to_numpy(t, dtype)
    want = gen.init_table(5, 3, m, d, dtype)
    assert np.array_equal(got.view(np.uint8), want.view(np.uint8))


# ------------------------------------------------------------------ embedding forward
FWD_CASES = [
    # name, K, B, d, dtype, rows, bag, dist
    ("tiny-shape", 8, 128, 16, gen.F32, 1000, ("uniform", 1, 4), ("uniform",)),
    ("d4-group", 3, 70, 4, gen.F32, 50, ("uniform", 0, 3), ("uniform",)),
    ("d4-wave", 2, 33, 4, gen.F32, 50, ("uniform", 0, 150), ("uniform",)),
    ("d64-long-bags", 3, 67, 64, gen.F32, 5000, ("uniform", 0, 300), ("uniform",)),
    ("d64-short-bags", 3, 67, 64, gen.F32, 5000, ("uniform", 0, 5), ("uniform",)),
    ("d128-onehot", 5, 257, 128, gen.F32, 3000, ("fixed", 1), ("zipf", 1.05)),
    ("d128-medium", 2, 40, 128, gen.F32, 3000, ("uniform", 0, 40), ("zipf", 1.05)),
    ("d48-nonpow2", 2, 31, 48, gen.F32, 100, ("uniform", 0, 40), ("uniform",)),
    ("d256-fullwave", 2, 19, 256, gen.F32, 100, ("uniform", 0, 9), ("uniform",)),
    ("f16-d128-fixed32", 4, 200, 128, gen.F16, 20000, ("fixed", 32), ("zipf", 1.2)),
    ("f16-d8", 2, 50, 8, gen.F16, 64, ("uniform", 0, 6), ("uniform",)),
    # the widest low-precision rows (1024 bytes): short and long bags
    ("f16-d512", 3, 70, 512, gen.F16, 500, ("uniform", 0, 12), ("uniform",)),
    ("bf16-d384-long-bags", 2, 9, 384, gen.BF16, 500, ("uniform", 0, 300), ("uniform",)),
    ("bf16-d64", 3, 90, 64, gen.BF16, 700, ("uniform", 0, 70), ("uniform",)),
    ("one-row-table", 2, 20, 16, gen.F32, 1, ("uniform", 0, 5), ("uniform",)),
    ("300-tables", 300, 40, 8, gen.F32, 60, ("uniform", 0, 6), ("zipf", 1.1)),
    ("single-table-single-bag", 1, 1, 32, gen.F32, 500, ("fixed", 700), ("uniform",)),
    ("single-bag", 1, 1, 32, gen.F32, 10, ("fixed", 7), ("uniform",)),
]


@pytest.mark.parametrize("case", FWD_CASES, ids=[c[0] for c in FWD_CASES])
def test_emb_bag_fwd_matches_oracle(case):
    name, K, B, d, dtype, rows, bag, dist = case
    _say("emb_bag_fwd " + name)
    w = gen.custom_workload(name, K=K, B=B, d=d, dtype=dtype, rows=rows, bag=bag, dist=dist, seed=3)
    b = gen.make_batch(w)
    host = _host_tables(b)
    tables = upload_tables(host, dtype)
    sb = make_sparse_batch(b, tables)
    F = K + 1
    T = torch.full((B, F, d), 123.0, dtype=torch.float32, device=DEV)
    hot.dlrm_emb_bag_fwd(sb, T, F * d, d, out_offset=d)
    torch.cuda.synchronize()
    got = T.cpu().numpy()
    want = oracle.emb_bag_fwd(host, dtype, b.indices, b.offsets, b.tbl_off)
    assert np.all(got[:, 0, :] == 123.0)                 # row 0 belongs to the dense vector
    scale = scale_emb_fwd(host, dtype, b.indices, b.offsets, b.tbl_off)
    assert rel_err(got[:, 1:, :], want, scale) <= 1e-5   # the sums are fp32 whatever the storage type
    if bag == ("fixed", 1):
        assert np.array_equal(got[:, 1:, :].view(np.uint32), want.astype(np.float32).view(np.uint32))
    empty = np.argwhere(b.lengths == 0)
    for k, bb in empty:
        assert np.all(got[bb, k + 1, :].view(np.uint32) == 0)     # +0.0 exactly


def test_emb_bag_fwd_single_index_bags_copy_rows_bitwise_even_in_the_long_bag_kernel():
    # mean bag length is large (wavefront-per-bag kernel) but some bags hold one index
    lists = [[[5], list(range(40)) * 8, [], [7], [7, 7, 7]], ]
    b = gen.batch_from_lists([64], lists, d=16)
    host = [gen.init_table(0, 0, 64, 16, gen.F32)]
    host[0][5, 3] = -0.0
    tables = upload_tables(host, gen.F32)
    out = torch.empty((5, 1, 16), dtype=torch.float32, device=DEV)
    hot.dlrm_emb_bag_fwd(make_sparse_batch(b, tables), out, 16, 16)
    got = out.cpu().numpy()
    assert np.array_equal(got[0, 0].view(np.uint32), host[0][5].view(np.uint32))
    assert np.array_equal(got[3, 0].view(np.uint32), host[0][7].view(np.uint32))
    assert np.all(got[2, 0].view(np.uint32) == 0)
    want = oracle.emb_bag_fwd(host, gen.F32, b.indices, b.offsets, b.tbl_off)
    assert rel_err(got, want, scale_emb_fwd(host, gen.F32, b.indices, b.offsets, b.tbl_off)) <= 1e-5


# ------------------------------------------------------------------ interaction
INT_CASES = [(1, 2, 4), (37, 2, 16), (128, 9, 16), (300, 9, 64), (77, 27, 16), (41, 27, 128),
             (19, 65, 128), (5, 3, 256), (1030, 5, 8),
             # every count of 16-row blocks (1..8), F = 1, block boundaries (17, 18, 33, 34), the largest
             # F and d, and d that is no multiple of 16 / 64
             (3, 1, 8), (9, 17, 12), (9, 18, 20), (7, 33, 16), (6, 34, 36), (4, 50, 72), (3, 66, 64),
             (3, 90, 24), (2, 100, 40), (2, 113, 4), (2, 128, 256)]


@pytest.mark.parametrize("B,F,d", INT_CASES)
def test_interact_dot_fwd_bwd_match_oracle(B, F, d):
    _say("interact B=%d F=%d d=%d" % (B, F, d))
    rng = np.random.default_rng(B * 1000 + F)
    P = F * (F - 1) // 2
    T = rng.standard_normal((B, F, d)).astype(np.float32)
    dR = rng.standard_normal((B, d + P)).astype(np.float32)
    Td = torch.from_numpy(T).to(DEV)
    R = torch.full((B, d + P), -5.0, dtype=torch.float32, device=DEV)
    hot.dlrm_interact_dot_fwd(Td, R)
    got = R.cpu().numpy()
    want = oracle.interact_dot_fwd(T)
    assert np.array_equal(got[:, :d].view(np.uint32), T[:, 0, :].view(np.uint32))   # exact copy of x
    assert rel_err(got, want, scale_interact_fwd(T)) <= 1e-5
    dT = torch.full((B, F, d), -5.0, dtype=torch.float32, device=DEV)
    hot.dlrm_interact_dot_bwd(Td, torch.from_numpy(dR).to(DEV), dT)
    assert rel_err(dT.cpu().numpy(), oracle.interact_dot_bwd(T, dR), scale_interact_bwd(T, dR)) <= 1e-5


# ------------------------------------------------------------------ pooled lookup + interaction in one call
PI_CASES = [
    # name, K, B, d, dtype, rows, bag, dist, index32
    ("tiny-shape", 8, 128, 16, gen.F32, 1000, ("uniform", 1, 4), ("uniform",), False),
    ("onehot-26x16", 26, 300, 16, gen.F32, 500, ("fixed", 1), ("zipf", 1.05), False),
    ("onehot-26x128", 26, 131, 128, gen.F32, 3000, ("fixed", 1), ("zipf", 1.05), True),
    ("k16-d20", 16, 45, 20, gen.F32, 90, ("uniform", 0, 3), ("uniform",), False),
    ("k17-d12", 17, 33, 12, gen.F32, 90, ("uniform", 0, 3), ("uniform",), False),
    ("k33-f16-d40", 33, 21, 40, gen.F16, 70, ("uniform", 0, 4), ("uniform",), False),
    ("k64-bf16-d8", 64, 18, 8, gen.BF16, 70, ("uniform", 0, 2), ("uniform",), True),
    ("k48-d256", 48, 9, 256, gen.F32, 40, ("fixed", 1), ("uniform",), False),
    ("k1-b1-d4", 1, 1, 4, gen.F32, 3, ("fixed", 2), ("uniform",), False),
    ("mostly-empty", 5, 66, 32, gen.F32, 30, ("uniform", 0, 1), ("uniform",), False),
    ("long-bags-forced", 3, 20, 64, gen.F32, 400, ("uniform", 0, 40), ("uniform",), False),
    # four-row bags of 104 floats: the three-call path pools them with a wavefront per bag
    ("fixed4-d104", 17, 48, 104, gen.F32, 146, ("fixed", 4), ("zipf", 1.1), False),
    ("f16-d512", 5, 40, 512, gen.F16, 300, ("uniform", 0, 3), ("uniform",), False),
]


@pytest.mark.parametrize("case", PI_CASES, ids=[c[0] for c in PI_CASES])
def test_emb_interact_fwd_fused_matches_oracle_and_the_separate_calls(case):
    name, K, B, d, dtype, rows, bag, dist, index32 = case
    _say("emb_interact_fwd " + name)
    w = gen.custom_workload(name, K=K, B=B, d=d, dtype=dtype, rows=rows, bag=bag, dist=dist, seed=5)
    b = gen.make_batch(w)
    host = _host_tables(b)
    tables = upload_tables(host, dtype)
    sb = make_sparse_batch(b, tables, index32=index32)
    F, P = K + 1, (K + 1) * K // 2
    x = np.random.default_rng(K * 100 + d).standard_normal((B, d)).astype(np.float32)
    xd = torch.from_numpy(x).to(DEV)
    got = {}
    for algo in (hot.FWD_FUSED, hot.FWD_SPLIT, hot.FWD_AUTO):
        T = torch.full((B, F, d), 123.0, dtype=torch.float32, device=DEV)
        R = torch.full((B, d + P), -5.0, dtype=torch.float32, device=DEV)
        hot.dlrm_emb_interact_fwd(sb, xd, T, R, algo)
        torch.cuda.synchronize()
        got[algo] = (T.cpu().numpy(), R.cpu().numpy())
    wantT, wantR = oracle.emb_interact_fwd(host, dtype, b.indices, b.offsets, b.tbl_off, x)
    scaleT = scale_emb_fwd(host, dtype, b.indices, b.offsets, b.tbl_off)
    for algo, (T, R) in got.items():
        assert np.array_equal(T[:, 0].view(np.uint32), x.view(np.uint32))          # the dense vector, bit for bit
        assert np.array_equal(R[:, :d].view(np.uint32), x.view(np.uint32))
        assert rel_err(T[:, 1:], wantT[:, 1:].astype(np.float64), scaleT) <= 1e-5
        # the pairs are products of the fp32 T this path wrote
        assert rel_err(R, oracle.interact_dot_fwd(T), scale_interact_fwd(T)) <= 1e-5
        assert rel_err(R, wantR, scale_interact_fwd(scaleT_pad(scaleT, x))) <= 1e-5
    # short bags: both paths add a bag's rows one by one in position order, unless the three-call path
    # gives every bag a whole wavefront (mean bag >= twice the lane groups a wavefront holds), where
    # the lane groups' partial sums meet in a butterfly
    groups = 64 // min(64, 1 << int(np.ceil(np.log2(d * gen.ELEM_BYTES[dtype] / 16.0))))
    wavefront_per_bag = groups > 1 and b.nnz / float(K * B) >= 2 * groups
    if bag[-1] <= 4 and not wavefront_per_bag:
        assert np.array_equal(got[hot.FWD_FUSED][0].view(np.uint32), got[hot.FWD_SPLIT][0].view(np.uint32))
    for k, bb in np.argwhere(b.lengths == 0):
        assert np.all(got[hot.FWD_FUSED][0][bb, k + 1].view(np.uint32) == 0)     # +0.0 exactly


@pytest.mark.parametrize("case", PI_CASES, ids=[c[0] for c in PI_CASES])
def test_emb_interact_bwd_without_T_gives_the_bits_of_the_backward_on_T(case):
    """dlrm_emb_interact_fwd(T = NULL) + dlrm_emb_interact_bwd: the forward leaves T alone and gives the same
    R; the backward pools the bags again and gives, bit for bit, what dlrm_interact_dot_bwd gives on the T of
    the one-launch forward -- and matches the oracle's composed backward."""
    name, K, B, d, dtype, rows, bag, dist, index32 = case
    _say("emb_interact_bwd " + name)
    w = gen.custom_workload(name, K=K, B=B, d=d, dtype=dtype, rows=rows, bag=bag, dist=dist, seed=5)
    b = gen.make_batch(w)
    host = _host_tables(b)
    tables = upload_tables(host, dtype)
    sb = make_sparse_batch(b, tables, index32=index32)
    F, P = K + 1, (K + 1) * K // 2
    rng = np.random.default_rng(K * 100 + d)
    x = rng.standard_normal((B, d)).astype(np.float32)
    dR = rng.standard_normal((B, d + P)).astype(np.float32)
    xd, dRd = torch.from_numpy(x).to(DEV), torch.from_numpy(dR).to(DEV)
    T = torch.empty((B, F, d), dtype=torch.float32, device=DEV)
    R = torch.empty((B, d + P), dtype=torch.float32, device=DEV)
    hot.dlrm_emb_interact_fwd(sb, xd, T, R, hot.FWD_FUSED)
    R2 = torch.full((B, d + P), -5.0, dtype=torch.float32, device=DEV)
    hot.dlrm_emb_interact_fwd(sb, xd, None, R2, hot.FWD_FUSED)
    dT_ref = torch.empty((B, F, d), dtype=torch.float32, device=DEV)
    hot.dlrm_interact_dot_bwd(T, dRd, dT_ref)
    dT = torch.full((B, F, d), 7.0, dtype=torch.float32, device=DEV)
    hot.dlrm_emb_interact_bwd(sb, xd, dRd, dT)
    torch.cuda.synchronize()
    assert torch.equal(R.view(torch.int32), R2.view(torch.int32))
    assert torch.equal(dT.view(torch.int32), dT_ref.view(torch.int32))
    want = oracle.emb_interact_bwd(host, dtype, b.indices, b.offsets, b.tbl_off, x, dR)
    Th = T.cpu().numpy()
    assert rel_err(dT.cpu().numpy(), oracle.interact_dot_bwd(Th, dR), scale_interact_bwd(Th, dR)) <= 1e-5
    scaleT = scaleT_pad(scale_emb_fwd(host, dtype, b.indices, b.offsets, b.tbl_off), x)
    assert rel_err(dT.cpu().numpy(), want, scale_interact_bwd(scaleT, dR)) <= 2e-5


def test_emb_interact_fwd_without_T_needs_the_one_launch_path():
    w = gen.custom_workload("long-bags", K=3, B=20, d=64, dtype=gen.F32, rows=400, bag=("uniform", 0, 40), seed=5)
    b = gen.make_batch(w)
    sb = make_sparse_batch(b, upload_tables(_host_tables(b), gen.F32))
    x = torch.zeros((20, 64), dtype=torch.float32, device=DEV)
    R = torch.zeros((20, 64 + 6), dtype=torch.float32, device=DEV)
    for algo in (hot.FWD_SPLIT, hot.FWD_AUTO):      # AUTO takes the separate calls for bags this long
        with pytest.raises(hot.DlrmError) as e:
            hot.dlrm_emb_interact_fwd(sb, x, None, R, algo)
        assert e.value.status == -1


def scaleT_pad(scaleT, x):
    """|x| and the pooled magnitude scales laid out like T."""
    return np.concatenate([np.abs(x)[:, None, :].astype(np.float64), scaleT], axis=1).astype(np.float32)


@pytest.mark.parametrize("algo", ["fused", "split"])
def test_emb_interact_fwd_start_stamp_arrives_and_changes_nothing(algo):
    _say("emb_interact_fwd stamped " + algo)
    code = hot.FWD_FUSED if algo == "fused" else hot.FWD_SPLIT
    w = gen.custom_workload("st", K=5, B=300, d=32, rows=400, bag=("uniform", 0, 3), seed=9)
    b = gen.make_batch(w)
    tables = upload_tables(_host_tables(b), gen.F32)
    sb = make_sparse_batch(b, tables)
    F, P = 6, 15
    x = torch.from_numpy(np.random.default_rng(1).standard_normal((300, 32)).astype(np.float32)).to(DEV)
    T0, R0 = torch.empty((300, F, 32), device=DEV), torch.empty((300, 32 + P), device=DEV)
    hot.dlrm_emb_interact_fwd(sb, x, T0, R0, code)
    for stamp in (torch.full((3,), -1, dtype=torch.int32).pin_memory(),
                  torch.full((3,), -1, dtype=torch.int32, device=DEV)):
        T1, R1 = torch.full_like(T0, 7.0), torch.full_like(R0, 7.0)
        hot.dlrm_emb_interact_fwd_stamped(sb, x, T1, R1, code, stamp, 123456, index=1)
        torch.cuda.synchronize()
        assert stamp.cpu().tolist() == [-1, 123456, -1]
        assert torch.equal(T1.view(torch.int32), T0.view(torch.int32))
        assert torch.equal(R1.view(torch.int32), R0.view(torch.int32))


def test_emb_interact_fwd_fused_refuses_what_it_cannot_do_and_auto_takes_the_separate_calls():
    _say("emb_interact_fwd refusals")
    for K, weighted in ((65, False), (4, True)):
        w = gen.custom_workload("r", K=K, B=6, d=8, rows=20, bag=("uniform", 0, 3), seed=2)
        b = gen.make_batch(w)
        host = _host_tables(b)
        tables = upload_tables(host, gen.F32)
        wts = gen.make_weights(b, seed=1) if weighted else None
        sb = make_sparse_batch(b, tables, weights=wts)
        F, P = K + 1, (K + 1) * K // 2
        x = np.random.default_rng(K).standard_normal((6, 8)).astype(np.float32)
        xd = torch.from_numpy(x).to(DEV)
        T = torch.empty((6, F, 8), dtype=torch.float32, device=DEV)
        R = torch.empty((6, 8 + P), dtype=torch.float32, device=DEV)
        with pytest.raises(hot.DlrmError):
            hot.dlrm_emb_interact_fwd(sb, xd, T, R, hot.FWD_FUSED)
        hot.dlrm_emb_interact_fwd(sb, xd, T, R, hot.FWD_AUTO)
        torch.cuda.synchronize()
        if weighted:
            S = oracle.emb_bag_fwd_weighted(host, gen.F32, b.indices, b.offsets, b.tbl_off, wts)
        else:
            S = oracle.emb_bag_fwd(host, gen.F32, b.indices, b.offsets, b.tbl_off)
        Tw = np.concatenate([x[:, None, :], S.astype(np.float32)], axis=1)
        assert rel_err(R.cpu().numpy(), oracle.interact_dot_fwd(Tw), scale_interact_fwd(Tw) + 1e-30) <= 2e-5


def test_place_dense_is_an_exact_copy():
    rng = np.random.default_rng(1)
    B, F, d = 333, 9, 64
    x = rng.standard_normal((B, d)).astype(np.float32)
    T = torch.full((B, F, d), 9.0, dtype=torch.float32, device=DEV)
    hot.dlrm_place_dense(torch.from_numpy(x).to(DEV), T)
    got = T.cpu().numpy()
    assert np.array_equal(got[:, 0, :].view(np.uint32), x.view(np.uint32))
    assert np.all(got[:, 1:, :] == 9.0)


# ------------------------------------------------------------------ grouping + backward
BWD_CASES = [
    ("tiny-shape", 8, 128, 16, gen.F32, 1000, ("uniform", 1, 4), ("uniform",)),
    ("multi-tile-ragged", 3, 700, 64, gen.F32, 100000, ("uniform", 0, 40), ("uniform",)),
    ("hot-rows", 2, 600, 32, gen.F32, 50000, ("fixed", 16), ("zipf", 1.4)),
    ("onehot-zipf", 5, 2048, 16, gen.F32, 3000000, ("fixed", 1), ("zipf", 1.05)),
    ("d128-onehot", 3, 999, 128, gen.F32, 70000, ("fixed", 1), ("zipf", 1.05)),
    ("d4", 2, 100, 4, gen.F32, 37, ("uniform", 0, 6), ("uniform",)),
    ("d48-nonpow2", 2, 64, 48, gen.F32, 300, ("uniform", 0, 10), ("uniform",)),
    ("f16-d128-fixed32", 4, 300, 128, gen.F16, 20000, ("fixed", 32), ("zipf", 1.2)),
    ("bf16-d64", 3, 90, 64, gen.BF16, 700, ("uniform", 0, 70), ("uniform",)),
    ("one-row-table", 2, 5000, 16, gen.F32, 1, ("fixed", 1), ("uniform",)),
    # more tables than a workgroup has threads (the tile map and the hot-row lists walk them in chunks)
    ("300-tables", 300, 40, 8, gen.F32, 60, ("uniform", 0, 6), ("zipf", 1.1)),
    ("single-table-single-bag", 1, 1, 32, gen.F32, 500, ("fixed", 700), ("uniform",)),
    # rarely taken routes of the sort path
    # 40 rows x ~4096 lookups each: more hot rows per table than one pass of the hot-row kernel holds
    ("many-hot-rows", 2, 4096, 32, gen.F32, 40, ("fixed", 40), ("uniform",)),
    # 20 hot rows per table, rows of 64 and 256 floats: the dense hot-row kernel with one and four
    # 16-column blocks per wavefront, a last bag group that is not full, a last tile that is not full
    ("dense-hot-rows-d64", 2, 2500, 64, gen.F32, 20, ("fixed", 40), ("uniform",)),
    ("dense-hot-rows-d256-f16", 1, 1100, 256, gen.F16, 12, ("fixed", 70), ("uniform",)),
    # every bucket too large for the LDS sort, nothing dominant, few unsorted bits: segment kernels
    ("segments-no-dominant-row", 1, 32768, 8, gen.F32, 1 << 22, ("fixed", 96), ("uniform",)),
    # dominant rows split off AND a remainder that is still too large
    ("dominant-rows-large-rest", 1, 32768, 16, gen.F32, 1 << 22, ("fixed", 96), ("zipf", 1.1)),
    # too many unsorted bits for per-row counters: a workgroup streams its bucket through global memory
    ("large-buckets-many-bits", 1, 65536, 4, gen.F32, 1 << 25, ("fixed", 64), ("uniform",)),
]


def _run_export(sb, nnz, K):
    ws = hot.alloc_workspace(sb)
    n = max(nnz, 1)
    uniq = torch.full((n,), -1, dtype=torch.int64, device=DEV)
    seg = torch.full((n,), -1, dtype=torch.int64, device=DEV)
    sbag = torch.full((n,), -1, dtype=torch.int32, device=DEV)
    nu = torch.full((K,), -1, dtype=torch.int64, device=DEV)
    hot.dlrm_emb_bag_bwd_export_groups(sb, ws, uniq, seg, sbag, nu)
    torch.cuda.synchronize()
    return uniq.cpu().numpy(), seg.cpu().numpy(), sbag.cpu().numpy(), nu.cpu().numpy()


@pytest.mark.parametrize("case", BWD_CASES, ids=[c[0] for c in BWD_CASES])
def test_grouping_is_bit_exact(case):
    name, K, B, d, dtype, rows, bag, dist = case
    _say("export_groups " + name)
    w = gen.custom_workload(name, K=K, B=B, d=d, dtype=dtype, rows=rows, bag=bag, dist=dist, seed=4)
    b = gen.make_batch(w)
    tables = [torch.zeros((int(m), d), dtype=torch.float32, device=DEV) for m in b.rows[:1]] * K
    sb = hot.SparseBatch(tables, gen.F32, torch.from_numpy(b.indices).to(DEV),
                         torch.from_numpy(b.offsets).to(DEV), torch.from_numpy(b.tbl_off).to(DEV),
                         b.nnz, max_rows=int(b.rows.max()))
    uniq, seg, sbag, nu = _run_export(sb, b.nnz, K)
    want = oracle.group_rows(b.indices, b.offsets, b.tbl_off)
    for k in range(K):
        a0, a1 = int(b.tbl_off[k]), int(b.tbl_off[k + 1])
        wu, wseg, wpos, wbag = want[k]
        assert int(nu[k]) == len(wu)
        assert np.array_equal(uniq[a0:a0 + len(wu)], wu)
        assert np.array_equal(seg[a0:a0 + len(wu)], wseg)
        assert np.array_equal(sbag[a0:a1], wbag)


@pytest.mark.parametrize("algo", ["sort", "atomic"])
@pytest.mark.parametrize("case", BWD_CASES, ids=[c[0] for c in BWD_CASES])
def test_emb_bag_bwd_sgd_matches_oracle(case, algo):
    name, K, B, d, dtype, rows, bag, dist = case
    if algo == "atomic" and dtype != gen.F32:
        pytest.skip("atomic path is defined for fp32 tables only")
    _say("emb_bag_bwd_sgd %s %s" % (name, algo))
    w = gen.custom_workload(name, K=K, B=B, d=d, dtype=dtype, rows=rows, bag=bag, dist=dist, seed=4)
    b = gen.make_batch(w)
    host = _host_tables(b)
    tables = upload_tables(host, dtype)
    before = [t.clone() for t in tables]
    sb = make_sparse_batch(b, tables)
    F = K + 1
    dS = b.dS()
    dT = torch.zeros((B, F, d), dtype=torch.float32, device=DEV)
    dT[:, 1:, :] = torch.from_numpy(dS).to(DEV)
    ws = hot.alloc_workspace(sb)
    lr = float(np.float32(w.lr))
    code = hot.BWD_SORT if algo == "sort" else hot.BWD_ATOMIC
    hot.dlrm_emb_bag_bwd_sgd(sb, dT, F * d, d, lr, ws, algo=code, dS_offset=d)
    torch.cuda.synchronize()
    ref = [t.copy() for t in host]
    uniq, grad = oracle.emb_bag_bwd_sgd(ref, dtype, b.indices, b.offsets, b.tbl_off, dS,
                                        float(np.float32(lr)), want_grad=True)
    scale = scale_sgd(host, dtype, b.indices, b.offsets, b.tbl_off, dS, float(np.float32(lr)))
    for k in range(K):
        got = table_to_numpy(tables[k], dtype)
        # rows nobody looked up keep their bits
        mask = np.ones(int(b.rows[k]), dtype=bool)
        mask[uniq[k]] = False
        assert np.array_equal(got[mask].view(np.uint8), host[k][mask].view(np.uint8))
        if len(uniq[k]) == 0:
            continue
        g_rows, r_rows, h_rows = got[uniq[k]], ref[k][uniq[k]], host[k][uniq[k]]
        assert rel_err(widen_host(g_rows, dtype), widen_host(r_rows, dtype), scale[k][uniq[k]],
                       SCALE_FLOOR[dtype]) <= TOL[dtype]
        if dtype == gen.F32:
            # the applied step W_before - W_after against lr*g, allowing the rounding of W:
            # once per row for the sort path, once per occurrence for the atomic path
            step_got = h_rows.astype(np.float64) - g_rows.astype(np.float64)
            ulp = max(np.abs(h_rows).max(), np.abs(g_rows).max()) * 2.0 ** -23
            n_round = 2 if algo == "sort" else 2 + int(np.bincount(b.indices_of(k)).max())
            bound = 1e-5 * np.abs(lr * grad[k]).max() + n_round * ulp
            assert np.max(np.abs(step_got - lr * grad[k])) <= bound
        else:
            # low-precision tables: fp32 arithmetic + one rounding lands within one unit in the
            # last place of the fp64-then-rounded reference, give or take the fp32 error of the value
            # that was rounded (1e-5 of its magnitude scale: it matters where thousands of gradient rows
            # are summed and the result cancels against the row)
            a, r = widen_host(g_rows, dtype), widen_host(r_rows, dtype)
            mant = 10 if dtype == gen.F16 else 7
            emin = -14 if dtype == gen.F16 else -126
            expo = np.maximum(np.floor(np.log2(np.maximum(np.abs(r), 2.0 ** emin))), emin)
            assert np.all(np.abs(a - r) <= 2.0 ** (expo - mant) + 1e-5 * scale[k][uniq[k]])
    if algo == "sort":
        # bitwise reproducible: same inputs, same bits
        tables2 = [t.clone() for t in before]
        sb2 = make_sparse_batch(b, tables2)
        hot.dlrm_emb_bag_bwd_sgd(sb2, dT, F * d, d, lr, ws, algo=code, dS_offset=d)
        torch.cuda.synchronize()
        for k in range(K):
            assert torch.equal(tables2[k].view(torch.uint8), tables[k].view(torch.uint8))


@pytest.mark.parametrize("case", [c for c in BWD_CASES if c[0] in ("multi-tile-ragged", "hot-rows",
                                                                   "f16-d128-fixed32")], ids=lambda c: c[0])
def test_prepare_on_a_second_stream_then_update_gives_the_same_bits(case):
    """dlrm_emb_bag_bwd_prepare on a side stream (while other work runs on the main one), then
    the update with DLRM_BWD_SORT_PREPARED, against the single-call sort path."""
    name, K, B, d, dtype, rows, bag, dist = case
    _say("emb_bag_bwd prepare/update %s" % name)
    w = gen.custom_workload(name, K=K, B=B, d=d, dtype=dtype, rows=rows, bag=bag, dist=dist, seed=6)
    b = gen.make_batch(w)
    host = _host_tables(b)
    one = upload_tables(host, dtype)
    two = upload_tables(host, dtype)
    F = K + 1
    dT = torch.zeros((B, F, d), dtype=torch.float32, device=DEV)
    dT[:, 1:, :] = torch.from_numpy(b.dS()).to(DEV)
    lr = float(np.float32(w.lr))
    sb1 = make_sparse_batch(b, one)
    ws1 = hot.alloc_workspace(sb1)
    hot.dlrm_emb_bag_bwd_sgd(sb1, dT, F * d, d, lr, ws1, algo=hot.BWD_SORT, dS_offset=d)
    sb2 = make_sparse_batch(b, two)
    ws2 = hot.alloc_workspace(sb2)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    done = torch.cuda.Event()
    with torch.cuda.stream(side):
        hot.dlrm_emb_bag_bwd_prepare(sb2, ws2)
        done.record(side)
    pooled = torch.empty((B, F, d), dtype=torch.float32, device=DEV)
    hot.dlrm_emb_bag_fwd(sb2, pooled, F * d, d, out_offset=d)   # the main stream is busy meanwhile
    torch.cuda.current_stream().wait_event(done)
    hot.dlrm_emb_bag_bwd_sgd(sb2, dT, F * d, d, lr, ws2, algo=hot.BWD_SORT_PREPARED, dS_offset=d)
    torch.cuda.synchronize()
    for k in range(K):
        assert torch.equal(one[k].view(torch.uint8), two[k].view(torch.uint8))


FLAT_CASES = [
    # name, K, B, d, dtype, rows, bag, dist, any oversized row group?
    ("uniform-large", 2, 1500, 16, gen.F32, 1000000, ("fixed", 40), ("uniform",), False),
    ("onehot-zipf-large", 26, 4096, 32, gen.F32, 3000000, ("fixed", 1), ("zipf", 1.05), False),
    ("hot-rows-large", 2, 4096, 32, gen.F32, 50000, ("fixed", 16), ("zipf", 1.4), True),
    ("many-hot-rows", 2, 4096, 32, gen.F32, 40, ("fixed", 40), ("uniform",), True),
    ("small-batch", 3, 100, 16, gen.F16, 500, ("uniform", 0, 6), ("uniform",), False),
]


@pytest.mark.parametrize("case", FLAT_CASES, ids=lambda c: c[0])
def test_oversized_count_and_the_reduce_launch_alone(case):
    """dlrm_emb_bag_bwd_prepared_oversized into pinned host memory; DLRM_BWD_SORT_PREPARED_FLAT gives the
    bits of DLRM_BWD_SORT_PREPARED when the count is zero and the oracle's result (other summation
    order) when it is not."""
    name, K, B, d, dtype, rows, bag, dist, oversized = case
    _say("emb_bag_bwd flat %s" % name)
    w = gen.custom_workload(name, K=K, B=B, d=d, dtype=dtype, rows=rows, bag=bag, dist=dist, seed=8)
    b = gen.make_batch(w)
    host = _host_tables(b)
    one, two = upload_tables(host, dtype), upload_tables(host, dtype)
    F = K + 1
    dS = b.dS()
    dT = torch.zeros((B, F, d), dtype=torch.float32, device=DEV)
    dT[:, 1:, :] = torch.from_numpy(dS).to(DEV)
    lr = float(np.float32(w.lr))
    sb1, sb2 = make_sparse_batch(b, one), make_sparse_batch(b, two)
    ws = hot.alloc_workspace(sb1)
    count = torch.full((3,), -1, dtype=torch.int32).pin_memory()
    hot.dlrm_emb_bag_bwd_prepare(sb1, ws)
    hot.dlrm_emb_bag_bwd_prepared_oversized(sb1, ws, count, index=1)
    hot.dlrm_emb_bag_bwd_sgd(sb1, dT, F * d, d, lr, ws, algo=hot.BWD_SORT_PREPARED, dS_offset=d)
    torch.cuda.synchronize()
    assert count[0] == -1 and count[2] == -1
    assert (int(count[1]) > 0) == oversized
    hot.dlrm_emb_bag_bwd_prepare(sb2, ws)
    hot.dlrm_emb_bag_bwd_sgd(sb2, dT, F * d, d, lr, ws, algo=hot.BWD_SORT_PREPARED_FLAT, dS_offset=d)
    torch.cuda.synchronize()
    if not oversized:
        for k in range(K):
            assert torch.equal(one[k].view(torch.uint8), two[k].view(torch.uint8))
    ref = [t.copy() for t in host]
    uniq, _ = oracle.emb_bag_bwd_sgd(ref, dtype, b.indices, b.offsets, b.tbl_off, dS, lr, want_grad=True)
    scale = scale_sgd(host, dtype, b.indices, b.offsets, b.tbl_off, dS, lr)
    for k in range(K):
        got = table_to_numpy(two[k], dtype)
        mask = np.ones(int(b.rows[k]), dtype=bool)
        mask[uniq[k]] = False
        assert np.array_equal(got[mask].view(np.uint8), host[k][mask].view(np.uint8))
        assert rel_err(widen_host(got[uniq[k]], dtype), widen_host(ref[k][uniq[k]], dtype), scale[k][uniq[k]],
                       SCALE_FLOOR[dtype]) <= TOL[dtype]


ADAGRAD_CASES = [c for c in BWD_CASES if c[0] in (
    "tiny-shape", "multi-tile-ragged", "hot-rows", "d48-nonpow2", "f16-d128-fixed32", "bf16-d64",
    "many-hot-rows", "dominant-rows-large-rest", "dense-hot-rows-d64", "one-row-table")]


@pytest.mark.parametrize("fresh", [False, True], ids=["warm-state", "fresh-state"])
@pytest.mark.parametrize("case", ADAGRAD_CASES, ids=lambda c: c[0])
def test_emb_bag_bwd_adagrad_matches_oracle(case, fresh):
    """h <- h + g^2, W <- W - lr g / (sqrt(h) + eps) on the touched rows (Sec. 5.1's second optimizer).
    Error model: the fp32 sum g carries |dg| <= n 2^-24 S_g (S_g = sum of |terms|); h + g^2 has only
    positive terms, so h is compared relative to h0 + S_g^2; d(step)/dg is at most lr / (sqrt(h0) + eps),
    so W is compared relative to |W| + lr S_g / (sqrt(h0) + eps).  With a fresh state (h0 = 0) that bound is
    vacuous where g cancels to ~0 (the step is lr*sign(g) there): those elements are held to |dW| <= lr and
    to the comparison of h, which carries g."""
    name, K, B, d, dtype, rows, bag, dist = case
    _say("emb_bag_bwd_adagrad %s fresh=%s" % (name, fresh))
    w = gen.custom_workload(name, K=K, B=B, d=d, dtype=dtype, rows=rows, bag=bag, dist=dist, seed=8)
    b = gen.make_batch(w)
    host = _host_tables(b)
    rng = np.random.default_rng(12)
    h0 = [np.zeros((int(r), d), dtype=np.float32) if fresh
          else rng.uniform(0.01, 1.0, size=(int(r), d)).astype(np.float32) for r in b.rows]
    tables = upload_tables(host, dtype)
    state = [torch.from_numpy(h.copy()).to(DEV) for h in h0]
    sptr = hot.state_pointers(state)
    sb = make_sparse_batch(b, tables)
    F = K + 1
    dS = b.dS()
    dT = torch.zeros((B, F, d), dtype=torch.float32, device=DEV)
    dT[:, 1:, :] = torch.from_numpy(dS).to(DEV)
    ws = hot.alloc_workspace(sb)
    lr, eps = float(np.float32(0.05)), float(np.float32(1e-8))
    hot.dlrm_emb_bag_bwd_adagrad(sb, sptr, dT, F * d, d, lr, eps, ws, dS_offset=d)
    torch.cuda.synchronize()
    ref_w = [t.copy() for t in host]
    ref_h = [h.copy() for h in h0]
    oracle.emb_bag_bwd_adagrad(ref_w, ref_h, dtype, b.indices, b.offsets, b.tbl_off, dS, lr, eps)
    # S_g per touched row: the oracle's SGD on zero tables with |dS| and lr = -1
    sg = [np.zeros((int(r), d), dtype=np.float32) for r in b.rows]
    uniq, _ = oracle.emb_bag_bwd_sgd(sg, gen.F32, b.indices, b.offsets, b.tbl_off, np.abs(dS), -1.0)
    for k in range(K):
        got_w = table_to_numpy(tables[k], dtype)
        got_h = state[k].cpu().numpy()
        mask = np.ones(int(b.rows[k]), dtype=bool)
        mask[uniq[k]] = False
        assert np.array_equal(got_w[mask].view(np.uint8), host[k][mask].view(np.uint8))
        assert np.array_equal(got_h[mask].view(np.uint32), h0[k][mask].view(np.uint32))
        if len(uniq[k]) == 0:
            continue
        u = uniq[k]
        S = sg[k][u].astype(np.float64)
        assert rel_err(got_h[u], ref_h[k][u], h0[k][u] + S * S) <= 1e-5
        gw, rw = widen_host(got_w[u], dtype), widen_host(ref_w[k][u], dtype)
        w0 = np.abs(widen_host(host[k][u], dtype)).astype(np.float64)
        if fresh:
            g_ref = np.sqrt(ref_h[k][u].astype(np.float64))      # |g| (h0 = 0)
            ok = g_ref >= 1e-3 * S
            scale = w0 + lr
            err = np.abs(gw.astype(np.float64) - rw.astype(np.float64)) / np.maximum(scale, SCALE_FLOOR[dtype])
            if ok.any():
                assert err[ok].max() <= TOL[dtype]
            # where g cancels to ~0 the step lr*g/(|g| + eps) may take either sign: no element-wise comparison,
            # but the step is at most lr in size on both sides (plus one rounding of the stored type), and h,
            # which carries g, has been compared above
            ulp = np.abs(gw) * (2.0 ** -23 if dtype == gen.F32 else 2.0 ** -10 if dtype == gen.F16 else 2.0 ** -7)
            w_before = widen_host(host[k][u], dtype)
            assert np.all(np.abs(gw - w_before) <= lr * (1 + 1e-6) + ulp + SCALE_FLOOR[dtype])
            assert np.all(np.abs(rw - w_before) <= lr * (1 + 1e-6) + ulp + SCALE_FLOOR[dtype])
        else:
            scale = w0 + lr * S / (np.sqrt(h0[k][u].astype(np.float64)) + eps)
            assert rel_err(gw, rw, scale, SCALE_FLOOR[dtype]) <= TOL[dtype]
    # bitwise reproducible, and the same bits when the grouping was prepared on another stream
    tables2 = upload_tables(host, dtype)
    state2 = [torch.from_numpy(h.copy()).to(DEV) for h in h0]
    sb2 = make_sparse_batch(b, tables2)
    side = torch.cuda.Stream()
    done = torch.cuda.Event()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        hot.dlrm_emb_bag_bwd_prepare(sb2, ws)
        done.record(side)
    torch.cuda.current_stream().wait_event(done)
    hot.dlrm_emb_bag_bwd_adagrad(sb2, hot.state_pointers(state2), dT, F * d, d, lr, eps, ws,
                                 algo=hot.BWD_SORT_PREPARED, dS_offset=d)
    torch.cuda.synchronize()
    for k in range(K):
        assert torch.equal(tables2[k].view(torch.uint8), tables[k].view(torch.uint8))
        assert torch.equal(state2[k], state[k])


# ------------------------------------------------------------------ weighted pooling (Eq. (2) in full)
def _abs_tables(host, dtype):
    return [np.abs(widen_host(t, dtype)).astype(np.float32) for t in host]


@pytest.mark.parametrize("case", [c for c in FWD_CASES if c[0] in (
    "tiny-shape", "d4-wave", "d64-long-bags", "d64-short-bags", "d128-onehot", "d48-nonpow2",
    "f16-d128-fixed32", "bf16-d64")], ids=lambda c: c[0])
def test_weighted_emb_bag_fwd_matches_oracle(case):
    name, K, B, d, dtype, rows, bag, dist = case
    _say("weighted emb_bag_fwd " + name)
    w = gen.custom_workload(name, K=K, B=B, d=d, dtype=dtype, rows=rows, bag=bag, dist=dist, seed=3)
    b = gen.make_batch(w)
    wts = gen.make_weights(b) * np.where(np.arange(b.nnz) % 3 == 0, -1.0, 1.0).astype(np.float32)
    host = _host_tables(b)
    tables = upload_tables(host, dtype)
    sb = make_sparse_batch(b, tables, weights=wts)
    F = K + 1
    T = torch.full((B, F, d), 123.0, dtype=torch.float32, device=DEV)
    hot.dlrm_emb_bag_fwd(sb, T, F * d, d, out_offset=d)
    torch.cuda.synchronize()
    got = T.cpu().numpy()
    want = oracle.emb_bag_fwd_weighted(host, dtype, b.indices, b.offsets, b.tbl_off, wts)
    scale = oracle.emb_bag_fwd_weighted(_abs_tables(host, dtype), gen.F32, b.indices, b.offsets, b.tbl_off,
                                        np.abs(wts))
    assert np.all(got[:, 0, :] == 123.0)
    assert rel_err(got[:, 1:, :], want, scale) <= 1e-5
    # weights of one give the bits of the unweighted call
    ones = make_sparse_batch(b, tables, weights=np.ones_like(wts))
    T1 = torch.zeros_like(T)
    T2 = torch.zeros_like(T)
    hot.dlrm_emb_bag_fwd(ones, T1, F * d, d, out_offset=d)
    hot.dlrm_emb_bag_fwd(make_sparse_batch(b, tables), T2, F * d, d, out_offset=d)
    assert torch.equal(T1, T2)


@pytest.mark.parametrize("opt", ["sgd", "adagrad"])
@pytest.mark.parametrize("case", [c for c in BWD_CASES if c[0] in (
    "tiny-shape", "multi-tile-ragged", "hot-rows", "d48-nonpow2", "f16-d128-fixed32", "many-hot-rows",
    "dominant-rows-large-rest")], ids=lambda c: c[0])
def test_weighted_emb_bag_bwd_matches_oracle(case, opt):
    """g_r = sum_p a_p dS[bag(p)] followed by either row update; compared relative to the sum of the
    terms' magnitudes, sum_p |a_p| |dS[bag(p)]| (and as in the Adagrad test for h and W there)."""
    name, K, B, d, dtype, rows, bag, dist = case
    _say("weighted emb_bag_bwd %s %s" % (name, opt))
    w = gen.custom_workload(name, K=K, B=B, d=d, dtype=dtype, rows=rows, bag=bag, dist=dist, seed=9)
    b = gen.make_batch(w)
    wts = gen.make_weights(b) * np.where(np.arange(b.nnz) % 5 == 0, -1.0, 1.0).astype(np.float32)
    host = _host_tables(b)
    tables = upload_tables(host, dtype)
    sb = make_sparse_batch(b, tables, weights=wts)
    F = K + 1
    dS = b.dS()
    dT = torch.zeros((B, F, d), dtype=torch.float32, device=DEV)
    dT[:, 1:, :] = torch.from_numpy(dS).to(DEV)
    ws = hot.alloc_workspace(sb)
    lr, eps = float(np.float32(0.05)), float(np.float32(1e-8))
    rng = np.random.default_rng(13)
    h0 = [rng.uniform(0.01, 1.0, size=(int(r), d)).astype(np.float32) for r in b.rows]
    ref_w = [t.copy() for t in host]
    sg = [np.zeros((int(r), d), dtype=np.float32) for r in b.rows]       # S_g per row
    oracle.emb_bag_bwd_weighted(sg, gen.F32, b.indices, b.offsets, b.tbl_off, np.abs(wts), np.abs(dS), -1.0)
    uniq = [np.unique(b.indices_of(k)) for k in range(K)]
    if opt == "sgd":
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
        got_w = table_to_numpy(tables[k], dtype)
        mask = np.ones(int(b.rows[k]), dtype=bool)
        mask[uniq[k]] = False
        assert np.array_equal(got_w[mask].view(np.uint8), host[k][mask].view(np.uint8))
        if len(uniq[k]) == 0:
            continue
        u = uniq[k]
        S = sg[k][u].astype(np.float64)
        w0 = np.abs(widen_host(host[k][u], dtype)).astype(np.float64)
        gw, rw = widen_host(got_w[u], dtype), widen_host(ref_w[k][u], dtype)
        if opt == "sgd":
            assert rel_err(gw, rw, w0 + lr * S, SCALE_FLOOR[dtype]) <= TOL[dtype]
        else:
            got_h = state[k].cpu().numpy()
            assert np.array_equal(got_h[mask].view(np.uint32), h0[k][mask].view(np.uint32))
            assert rel_err(got_h[u], ref_h[k][u], h0[k][u] + S * S) <= 1e-5
            scale = w0 + lr * S / (np.sqrt(h0[k][u].astype(np.float64)) + eps)
            assert rel_err(gw, rw, scale, SCALE_FLOOR[dtype]) <= TOL[dtype]
    if opt == "sgd" and dtype == gen.F32:
        # the atomic path honours the weights too
        tables3 = upload_tables(host, dtype)
        hot.dlrm_emb_bag_bwd_sgd(make_sparse_batch(b, tables3, weights=wts), dT, F * d, d, lr, None,
                                 algo=hot.BWD_ATOMIC, dS_offset=d)
        torch.cuda.synchronize()
        for k in range(K):
            if len(uniq[k]):
                u = uniq[k]
                scale = np.abs(host[k][u]).astype(np.float64) + lr * sg[k][u]
                assert rel_err(tables3[k].cpu().numpy()[u], ref_w[k][u], scale) <= 1e-5
    if opt == "sgd":
        # same bits again, also with the grouping prepared ahead
        tables2 = upload_tables(host, dtype)
        sb2 = make_sparse_batch(b, tables2, weights=wts)
        hot.dlrm_emb_bag_bwd_prepare(sb2, ws)
        hot.dlrm_emb_bag_bwd_sgd(sb2, dT, F * d, d, lr, ws, algo=hot.BWD_SORT_PREPARED, dS_offset=d)
        # and the grouping exported from a weighted batch is the unweighted one
        uq, seg, sbag, nu = _run_export(sb2, b.nnz, K)
        want = oracle.group_rows(b.indices, b.offsets, b.tbl_off)
        torch.cuda.synchronize()
        for k in range(K):
            assert torch.equal(tables2[k].view(torch.uint8), tables[k].view(torch.uint8))
            a0, a1 = int(b.tbl_off[k]), int(b.tbl_off[k + 1])
            assert np.array_equal(sbag[a0:a1], want[k][3])


# ------------------------------------------------------------------ int32 indices
@pytest.mark.parametrize("case", [c for c in BWD_CASES if c[0] in (
    "tiny-shape", "multi-tile-ragged", "hot-rows", "onehot-zipf", "f16-d128-fixed32", "many-hot-rows")],
    ids=lambda c: c[0])
def test_int32_indices_give_the_bits_of_int64_indices(case):
    """Forward, validator, sort and atomic backward, grouping export: a batch whose index array is
    int32 must give, bit for bit, what the same batch with int64 indices gives (itself checked against
    the oracle by the other tests)."""
    name, K, B, d, dtype, rows, bag, dist = case
    _say("int32 indices " + name)
    w = gen.custom_workload(name, K=K, B=B, d=d, dtype=dtype, rows=rows, bag=bag, dist=dist, seed=10)
    b = gen.make_batch(w)
    wts = gen.make_weights(b)
    host = _host_tables(b)
    F = K + 1
    dT = torch.zeros((B, F, d), dtype=torch.float32, device=DEV)
    dT[:, 1:, :] = torch.from_numpy(b.dS()).to(DEV)
    lr = float(np.float32(w.lr))
    results = []
    for index32 in (False, True):
        out = {}
        for weights in (None, wts):
            tables = upload_tables(host, dtype)
            sb = make_sparse_batch(b, tables, weights=weights, index32=index32)
            n_bad = torch.zeros(1, dtype=torch.int64, device=DEV)
            hot.dlrm_validate_csr(sb, n_bad)
            assert int(n_bad.item()) == 0
            T = torch.zeros((B, F, d), dtype=torch.float32, device=DEV)
            hot.dlrm_emb_bag_fwd(sb, T, F * d, d, out_offset=d)
            ws = hot.alloc_workspace(sb)
            hot.dlrm_emb_bag_bwd_sgd(sb, dT, F * d, d, lr, ws, algo=hot.BWD_SORT, dS_offset=d)
            tag = "w" if weights is not None else "u"
            out["T" + tag] = T
            out["W" + tag] = tables
        sb = make_sparse_batch(b, upload_tables(host, dtype), index32=index32)
        out["export"] = _run_export(sb, b.nnz, K)
        results.append(out)
    torch.cuda.synchronize()
    a64, a32 = results
    for tag in ("u", "w"):
        assert torch.equal(a64["T" + tag], a32["T" + tag])
        for k in range(K):
            assert torch.equal(a64["W" + tag][k].view(torch.uint8), a32["W" + tag][k].view(torch.uint8))
    for x, y in zip(a64["export"], a32["export"]):
        assert np.array_equal(x, y)
    # a bad int32 index is counted like a bad int64 one
    bad_idx = b.indices.copy()
    bad_idx[0] = -1
    bad = gen.Batch(b.workload, b.rows, b.lengths, b.offsets, b.tbl_off, bad_idx, b.x, b.dR)
    n_bad = torch.zeros(1, dtype=torch.int64, device=DEV)
    hot.dlrm_validate_csr(make_sparse_batch(bad, upload_tables(host, dtype), index32=True), n_bad)
    assert int(n_bad.item()) == 1
    if dtype == gen.F32:   # atomic path with int32 indices against the oracle
        tables = upload_tables(host, dtype)
        hot.dlrm_emb_bag_bwd_sgd(make_sparse_batch(b, tables, index32=True), dT, F * d, d, lr, None,
                                 algo=hot.BWD_ATOMIC, dS_offset=d)
        ref = [t.copy() for t in host]
        oracle.emb_bag_bwd_sgd(ref, dtype, b.indices, b.offsets, b.tbl_off, b.dS(), lr)
        scale = scale_sgd(host, dtype, b.indices, b.offsets, b.tbl_off, b.dS(), lr)
        for k in range(K):
            assert rel_err(tables[k].cpu().numpy(), ref[k], scale[k]) <= 1e-5


def test_a_captured_step_replays_to_the_eager_bits():
    """The library only enqueues kernels (no allocation, no memset, no synchronisation), so a caller can
    capture a whole step in a HIP graph.  Three replays, with eager work and synchronisations in
    between, each against the eager step's bits (sort path: bitwise reproducible)."""
    w = gen.custom_workload("graph", K=4, B=300, d=32, dtype=gen.F32, rows=20000, bag=("uniform", 0, 30),
                            dist=("zipf", 1.2), seed=11)
    b = gen.make_batch(w)
    K, B, d, F, P = w.K, w.B, w.d, w.F, w.P
    host = _host_tables(b)
    x = torch.from_numpy(b.x).to(DEV)
    dR = torch.from_numpy(b.dR).to(DEV)
    lr = float(np.float32(w.lr))

    def buffers():
        return (torch.zeros((B, F, d), dtype=torch.float32, device=DEV),
                torch.zeros((B, d + P), dtype=torch.float32, device=DEV),
                torch.zeros((B, F, d), dtype=torch.float32, device=DEV))

    def step(sb, ws, T, R, dT, side=None):
        if side is not None:
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                hot.dlrm_emb_bag_bwd_prepare(sb, ws)
        hot.dlrm_place_dense(x, T)
        hot.dlrm_emb_bag_fwd(sb, T, F * d, d, out_offset=d)
        hot.dlrm_interact_dot_fwd(T, R)
        hot.dlrm_interact_dot_bwd(T, dR, dT)
        if side is not None:
            torch.cuda.current_stream().wait_stream(side)
            hot.dlrm_emb_bag_bwd_sgd(sb, dT, F * d, d, lr, ws, algo=hot.BWD_SORT_PREPARED, dS_offset=d)
        else:
            hot.dlrm_emb_bag_bwd_sgd(sb, dT, F * d, d, lr, ws, algo=hot.BWD_SORT, dS_offset=d)

    # eager: three consecutive steps, the tables after each
    tables_e = upload_tables(host, gen.F32)
    sb_e = make_sparse_batch(b, tables_e)
    ws_e = hot.alloc_workspace(sb_e)
    Te, Re, dTe = buffers()
    eager = []
    for _ in range(3):
        step(sb_e, ws_e, Te, Re, dTe)
        torch.cuda.synchronize()
        eager.append(([t.clone() for t in tables_e], Re.clone(), dTe.clone()))
    # captured once, replayed three times on tables of its own
    tables_g = upload_tables(host, gen.F32)
    sb_g = make_sparse_batch(b, tables_g)
    ws_g = hot.alloc_workspace(sb_g)
    Tg, Rg, dTg = buffers()
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(sb_g, ws_g, Tg, Rg, dTg, side=side)
    torch.cuda.synchronize()
    for t, h in zip(tables_g, host):        # the capture itself ran nothing
        assert np.array_equal(t.cpu().numpy(), h)
    for r in range(3):
        graph.replay()
        torch.cuda.synchronize()
        want_tables, want_R, want_dT = eager[r]
        assert torch.equal(Rg, want_R) and torch.equal(dTg, want_dT), "replay %d" % r
        for k in range(K):
            assert torch.equal(tables_g[k], want_tables[k]), "replay %d table %d" % (r, k)
        # the program's own eager work between replays
        scratch = torch.empty((B, F, d), dtype=torch.float32, device=DEV)
        hot.dlrm_emb_bag_fwd(sb_e, scratch, F * d, d, out_offset=d)
        torch.cuda.synchronize()


def test_backward_with_a_table_nobody_looks_up_and_lr_zero():
    lists = [[[1, 1, 3], [], [3]], [[], [], []], [[0], [0], [0]]]
    b = gen.batch_from_lists([8, 8, 8], lists, d=8)
    host = [gen.init_table(1, k, 8, 8, gen.F32) for k in range(3)]
    for algo in (hot.BWD_SORT, hot.BWD_ATOMIC):
        tables = upload_tables(host, gen.F32)
        sb = make_sparse_batch(b, tables)
        dS = torch.from_numpy(b.dS()).to(DEV)
        ws = hot.alloc_workspace(sb)
        hot.dlrm_emb_bag_bwd_sgd(sb, dS, 3 * 8, 8, 0.0, ws, algo=algo)
        for k in range(3):
            assert np.array_equal(tables[k].cpu().numpy().view(np.uint32), host[k].view(np.uint32))
        hot.dlrm_emb_bag_bwd_sgd(sb, dS, 3 * 8, 8, 0.5, ws, algo=algo)
        ref = [t.copy() for t in host]
        oracle.emb_bag_bwd_sgd(ref, gen.F32, b.indices, b.offsets, b.tbl_off, b.dS(), 0.5)
        scale = scale_sgd(host, gen.F32, b.indices, b.offsets, b.tbl_off, b.dS(), 0.5)
        for k in range(3):
            assert rel_err(tables[k].cpu().numpy(), ref[k], scale[k]) <= 1e-5
        assert np.array_equal(tables[1].cpu().numpy(), host[1])
    uniq, seg, sbag, nu = _run_export(sb, b.nnz, 3)
    assert nu.tolist() == [2, 0, 1]


def test_empty_batch_is_a_no_op():
    lists = [[[], []], [[], []]]
    b = gen.batch_from_lists([4, 4], lists, d=4)
    host = [gen.init_table(1, k, 4, 4, gen.F32) for k in range(2)]
    tables = upload_tables(host, gen.F32)
    sb = make_sparse_batch(b, tables)
    out = torch.full((2, 2, 4), 3.0, dtype=torch.float32, device=DEV)
    hot.dlrm_emb_bag_fwd(sb, out, 8, 4)
    assert np.all(out.cpu().numpy() == 0.0)
    ws = hot.alloc_workspace(sb)
    hot.dlrm_emb_bag_bwd_sgd(sb, out, 8, 4, 0.1, ws, algo=hot.BWD_SORT)
    hot.dlrm_emb_bag_bwd_sgd(sb, out, 8, 4, 0.1, ws, algo=hot.BWD_ATOMIC)
    for k in range(2):
        assert np.array_equal(tables[k].cpu().numpy(), host[k])


# ------------------------------------------------------------------ measurement kernels
@pytest.mark.parametrize("row_bytes", [64, 128, 256, 512])
def test_measurement_kernels_move_the_bytes_they_claim(row_bytes):
    """The kernels a benchmark times for the board's ceilings: the copy copies, the row update touches
    exactly the listed rows (one fp32 multiply by 1 + 2^-10 each), the read-only ones change nothing."""
    _say("ceiling kernels, rows of %d bytes" % row_bytes)
    g = torch.Generator(device="cpu").manual_seed(row_bytes)
    nrows, w = 5003, row_bytes // 4
    table = torch.randn((nrows, w), generator=g).to(DEV)
    before = table.clone()
    rows = torch.randperm(nrows, generator=g)[:3001].to(torch.int32).to(DEV)   # distinct, ragged count
    sink = ceilings.ceiling_sink()
    ceilings.dlrm_ceiling_gather(table, rows, row_bytes, sink)
    ceilings.dlrm_ceiling_read(table, sink)
    assert torch.equal(table, before)
    ceilings.dlrm_ceiling_rmw(table, rows, row_bytes)
    want = before.clone()
    sel = rows.long()
    want[sel] = before[sel] * torch.tensor(1.0 + 2.0 ** -10, dtype=torch.float32, device=DEV)
    assert torch.equal(table, want)
    dst = torch.zeros_like(table)
    ceilings.dlrm_ceiling_copy(table, dst)
    assert torch.equal(dst, table)
