"""dlrm_emb_bag_bwd_sgd_noalloc (the update on the library's own per-GPU scratch array, for callers
that cannot allocate) against dlrm_emb_bag_bwd_sgd on a caller-owned workspace: same bits, on two
calls in a row, the second with a smaller batch (the array then still holds the first call's pairs,
lists and counters)."""
import numpy as np
import pytest
import torch

import paper_1906_00091_amd as hot
from workloads import gen

from hotpath_util import DEV, make_sparse_batch, upload_tables

pytestmark = pytest.mark.gpu


def _tables(batch):
    w = batch.workload
    return [gen.init_table(batch.seed, k, int(batch.rows[k]), w.d, w.dtype) for k in range(w.K)]


# first call, then a smaller one: (K, B, d, dtype, rows, bag, dist)
PAIRS = [
    # hot rows in both (tail launches, hot-row lists and partial sums live in the array), then fewer lookups
    (("first", 2, 4096, 32, gen.F32, 50000, ("fixed", 16), ("zipf", 1.4)),
     ("second", 2, 700, 32, gen.F32, 50000, ("fixed", 16), ("zipf", 1.4))),
    # multi-hot, ragged bags, fp16 rows; then a tiny batch of another shape
    (("first", 3, 2048, 64, gen.F16, 100000, ("uniform", 0, 60), ("uniform",)),
     ("second", 5, 100, 16, gen.F16, 900, ("uniform", 0, 4), ("zipf", 1.1))),
]


@pytest.mark.parametrize("pair", PAIRS, ids=["hot-rows-then-fewer", "multihot-f16-then-tiny"])
def test_noalloc_update_gives_the_bits_of_the_workspace_update_twice_in_a_row(pair):
    for i, (name, K, B, d, dtype, rows, bag, dist) in enumerate(pair):
        print("[case] noalloc call %d: K=%d B=%d d=%d" % (i, K, B, d), flush=True)
        w = gen.custom_workload(name, K=K, B=B, d=d, dtype=dtype, rows=rows, bag=bag, dist=dist, seed=31 + i)
        b = gen.make_batch(w)
        host = _tables(b)
        one, two = upload_tables(host, dtype), upload_tables(host, dtype)
        F = K + 1
        dT = torch.zeros((B, F, d), dtype=torch.float32, device=DEV)
        dT[:, 1:, :] = torch.from_numpy(b.dS()).to(DEV)
        lr = float(np.float32(w.lr))
        sb1 = make_sparse_batch(b, one)
        ws = hot.alloc_workspace(sb1)
        assert ws.numel() <= hot.NOALLOC_SCRATCH_BYTES
        hot.dlrm_emb_bag_bwd_sgd(sb1, dT, F * d, d, lr, ws, algo=hot.BWD_SORT, dS_offset=d)
        sb2 = make_sparse_batch(b, two)
        torch.cuda.synchronize()
        hot.dlrm_emb_bag_bwd_sgd_noalloc(sb2, dT, F * d, d, lr, dS_offset=d)
        torch.cuda.synchronize()
        changed = 0
        for k in range(K):
            assert torch.equal(one[k].view(torch.uint8), two[k].view(torch.uint8)), (i, k)
            changed += int((two[k] != torch.from_numpy(host[k]).to(DEV)).any(dim=1).sum())
        assert changed > 0   # the call did update rows


def test_noalloc_update_rejects_a_batch_beyond_its_array_before_touching_anything():
    w = gen.custom_workload("too-large", K=1, B=30000, d=16, dtype=gen.F32, rows=1000, bag=("fixed", 100),
                            dist=("uniform",), seed=33)
    b = gen.make_batch(w)
    tables = upload_tables(_tables(b), gen.F32)
    before = [t.clone() for t in tables]
    sb = make_sparse_batch(b, tables)
    assert hot.dlrm_emb_bag_bwd_workspace_bytes(1, 30000, 16, b.nnz, 1000, gen.F32) > hot.NOALLOC_SCRATCH_BYTES
    dT = torch.ones((30000, 2, 16), dtype=torch.float32, device=DEV)
    with pytest.raises(hot.DlrmError) as e:
        hot.dlrm_emb_bag_bwd_sgd_noalloc(sb, dT, 32, 16, 0.5, dS_offset=16)
    assert e.value.status == -4   # DLRM_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert torch.equal(before[0], tables[0])
