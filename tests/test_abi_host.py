"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the header declares, and rejects bad arguments before launching anything."""
import ctypes as C
import os
import re

import pytest

import paper_1906_00091_amd as hot
from paper_1906_00091_amd import binding, ceilings

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dlrm_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared("dlrm_hot.h")
    assert len(names) >= 20
    L = hot.lib()
    for n in names:
        assert hasattr(L, n), n
    assert hot.version() >= 100
    assert hot.status_string(0) == "ok" and "NULL" in hot.status_string(-1)


def test_measurement_library_is_separate_and_exports_its_header():
    """The plain memory kernels a benchmark times live in a library of their own: the method's
    header declares none of them and the method's library exports none."""
    names = _declared("dlrm_ceilings.h")
    assert len(names) == 5
    L = ceilings.lib()
    for n in names:
        assert hasattr(L, n), n
        assert not hasattr(hot.lib(), n), n
    assert not [n for n in _declared("dlrm_hot.h") if "ceiling" in n or "profile" in n]


def _batch(**kw):
    base = dict(K=2, B=4, d=16, table_dtype=0, nnz_total=8, max_rows=100, tables=0x1000,
                rows=0x1000, indices=0x1000, offsets=0x1000, tbl_off=0x1000)
    base.update(kw)
    return binding._SparseBatchC(**base)


def test_forward_rejects_bad_arguments_on_the_host():
    L = hot.lib()
    out = C.c_void_p(0x1000)
    call = lambda b, o=out, sb=64, sk=16: L.dlrm_emb_bag_fwd(C.byref(b), o, sb, sk, None)
    assert call(_batch(tables=None)) == -1
    assert call(_batch(), o=None) == -1
    assert call(_batch(K=0)) == -2
    assert call(_batch(d=6)) == -2                  # 24-byte rows: not a multiple of 16
    assert call(_batch(d=512)) == -2                # 2 KB rows: above the supported row size
    assert call(_batch(table_dtype=7)) == -3
    assert call(_batch(max_rows=1 << 31)) == -2
    assert call(_batch(nnz_total=-1)) == -2
    assert call(_batch(), sk=8) == -2               # stride_k < d
    assert call(_batch(), o=C.c_void_p(0x1004)) == -2
    assert L.dlrm_emb_bag_fwd(None, out, 64, 16, None) == -1


def test_one_call_forward_rejects_bad_arguments_on_the_host():
    L = hot.lib()
    p = C.c_void_p(0x1000)
    call = lambda b, x=p, T=p, R=p, algo=0: L.dlrm_emb_interact_fwd(C.byref(b), x, T, R, algo, None)
    assert call(_batch(tables=None)) == -1
    assert call(_batch(), x=None) == -1
    assert call(_batch(), T=None, algo=2) == -1        # only the one-launch path can do without T
    assert call(_batch(nnz_total=800), T=None) == -1   # AUTO with long bags takes the separate calls
    assert call(_batch(), R=None) == -1
    assert call(_batch(K=128)) == -2                  # F = 129 vectors
    assert call(_batch(), x=C.c_void_p(0x1004)) == -2
    assert call(_batch(), T=C.c_void_p(0x1008)) == -2
    assert call(_batch(), algo=3) == -5
    assert call(_batch(K=65), algo=1) == -5           # the one-launch kernel takes up to 64 tables
    assert call(_batch(weights=0x1000), algo=1) == -5  # and no pooling weights
    bwd = lambda b, x=p, dR=p, dT=p: L.dlrm_emb_interact_bwd(C.byref(b), x, dR, dT, None)
    assert bwd(_batch(tables=None)) == -1
    assert bwd(_batch(), x=None) == -1 and bwd(_batch(), dR=None) == -1 and bwd(_batch(), dT=None) == -1
    assert bwd(_batch(), dT=C.c_void_p(0x1008)) == -2
    assert bwd(_batch(K=65)) == -5 and bwd(_batch(weights=0x1000)) == -5
    st = lambda b, x=p, stamp=None: L.dlrm_emb_interact_fwd_stamped(C.byref(b), x, p, p, 0, stamp, 5, None)
    assert st(_batch(tables=None)) == -1                # the stamped call checks the same things first
    assert st(_batch(), x=None, stamp=C.c_void_p(0x1000)) == -1


def test_more_bags_than_32_bits_number_is_rejected():
    L = hot.lib()
    p = C.c_void_p(0x1000)
    assert L.dlrm_emb_bag_fwd(C.byref(_batch(K=64, B=(1 << 25))), p, 64 * 16, 16, None) == -2
    assert L.dlrm_emb_bag_fwd(C.byref(_batch(K=1 << 20, B=1 << 12)), p, 64 * 16, 16, None) == -2


def test_unknown_index_dtype_is_rejected():
    L = hot.lib()
    # (no output pointer: a known index type gets as far as that check, nothing is launched)
    assert L.dlrm_emb_bag_fwd(C.byref(_batch(index_dtype=1)), None, 64, 16, None) == -1
    assert L.dlrm_emb_bag_fwd(C.byref(_batch(index_dtype=2)), None, 64, 16, None) == -3


def test_backward_rejects_bad_arguments_on_the_host():
    L = hot.lib()
    ds = C.c_void_p(0x1000)
    need = hot.dlrm_emb_bag_bwd_workspace_bytes(2, 4, 16, 8, 100, 0)
    assert need > 0 and need % 256 == 0
    call = lambda b, ws, n, algo: L.dlrm_emb_bag_bwd_sgd(C.byref(b), ds, 64, 16, C.c_float(0.01), ws,
                                                         n, algo, None)
    assert call(_batch(), None, 0, hot.BWD_SORT) == -4
    assert call(_batch(), C.c_void_p(0x1000), need - 1, hot.BWD_SORT) == -4
    assert call(_batch(), C.c_void_p(0x1010), need, hot.BWD_SORT) == -4      # misaligned
    assert call(_batch(), C.c_void_p(0x1000), need, 9) == -5
    assert call(_batch(), None, 0, hot.BWD_SORT_PREPARED) == -4
    assert call(_batch(K=65536, B=1), C.c_void_p(0x1000), 1 << 40, hot.BWD_SORT) == -2   # K is a grid dimension
    assert call(_batch(K=65536, B=1), C.c_void_p(0x1000), 1 << 40, hot.BWD_ATOMIC) == -2
    # the timed call: both events or none
    tm = binding._BwdTimingC(0x10, None)
    assert L.dlrm_emb_bag_bwd_sgd_timed(C.byref(_batch()), ds, 64, 16, C.c_float(0.01), C.c_void_p(0x1000), need,
                                        hot.BWD_SORT, C.byref(tm), None) == -1
    assert L.dlrm_emb_bag_bwd_adagrad_timed(C.byref(_batch()), C.c_void_p(0x1000), ds, 64, 16, C.c_float(0.01),
                                            C.c_float(1e-8), C.c_void_p(0x1000), need, hot.BWD_SORT, C.byref(tm),
                                            None) == -1
    prep = lambda b, ws, n: L.dlrm_emb_bag_bwd_prepare(C.byref(b), ws, n, None)
    over = lambda b, ws, n, o: L.dlrm_emb_bag_bwd_prepared_oversized(C.byref(b), ws, n, o, None)
    assert over(_batch(), C.c_void_p(0x1000), 1 << 30, None) == -1
    assert over(_batch(), None, 1 << 30, C.c_void_p(0x1000)) == -4
    assert over(_batch(d=6), C.c_void_p(0x1000), 1 << 30, C.c_void_p(0x1000)) == -2
    assert prep(_batch(), None, 0) == -4
    assert prep(_batch(), C.c_void_p(0x1000), need - 1) == -4
    assert prep(_batch(K=0), C.c_void_p(0x1000), need) != 0
    ada = lambda b, st, eps, algo: L.dlrm_emb_bag_bwd_adagrad(C.byref(b), st, ds, 64, 16, C.c_float(0.01),
                                                              C.c_float(eps), C.c_void_p(0x1000), need, algo, None)
    assert ada(_batch(), None, 1e-8, hot.BWD_SORT) == -1            # no state
    assert ada(_batch(), C.c_void_p(0x1000), 0.0, hot.BWD_SORT) == -2   # eps must be positive
    assert ada(_batch(), C.c_void_p(0x1000), 1e-8, hot.BWD_ATOMIC) == -5
    assert call(_batch(table_dtype=1), C.c_void_p(0x1000), need, hot.BWD_ATOMIC) == -3
    # a gradient row is d fp32 values and one wavefront wide at most: fp16 rows of 512 elements can be
    # pooled but not updated
    wide = lambda: _batch(d=512, table_dtype=1)
    assert L.dlrm_emb_bag_bwd_sgd(C.byref(wide()), ds, 3 * 512, 512, C.c_float(0.01), C.c_void_p(0x1000),
                                  1 << 30, hot.BWD_SORT, None) == -2
    assert prep(wide(), C.c_void_p(0x1000), 1 << 30) == -2
    assert hot.dlrm_emb_bag_bwd_workspace_bytes(0, 4, 16, 8, 100, 0) == 0
    assert hot.dlrm_emb_bag_bwd_workspace_bytes(2, 4, 16, 8, 100, 5) == 0
    # workspace grows with the number of lookups
    assert hot.dlrm_emb_bag_bwd_workspace_bytes(2, 4, 16, 1 << 20, 100, 0) > need


def test_interaction_and_helpers_reject_bad_arguments_on_the_host():
    L = hot.lib()
    p = C.c_void_p(0x1000)
    assert L.dlrm_interact_dot_fwd(None, 4, 3, 16, p, None) == -1
    assert L.dlrm_interact_dot_fwd(p, 4, 3, 6, p, None) == -2
    assert L.dlrm_interact_dot_fwd(p, 0, 3, 16, p, None) == -2
    assert L.dlrm_interact_dot_fwd(p, 4, 500, 16, p, None) == -2
    assert L.dlrm_interact_dot_bwd(p, p, 4, 3, 16, None, None) == -1
    assert L.dlrm_place_dense(p, 4, 16, None, 3, None) == -1
    assert L.dlrm_lengths_to_offsets(p, 0, 4, p, p, None) == -2
    assert L.dlrm_validate_csr(C.byref(_batch()), None, None) == -1
    assert L.dlrm_table_init_hash(p, 10, 6, 0, C.c_uint64(1), C.c_float(1.0), None) == -2


def test_measurement_kernels_reject_bad_arguments_on_the_host():
    L = ceilings.lib()
    p = C.c_void_p(0x1000)
    assert L.dlrm_ceiling_sink_floats() >= 4096
    assert L.dlrm_ceiling_copy(None, p, 64, None) == -1
    assert L.dlrm_ceiling_copy(p, p, 0, None) == -2
    assert L.dlrm_ceiling_copy(p, p, 24, None) == -2
    assert L.dlrm_ceiling_copy(C.c_void_p(0x1004), p, 64, None) == -2
    assert L.dlrm_ceiling_read(p, 64, None, None) == -1
    assert L.dlrm_ceiling_read(p, 8, p, None) == -2
    assert L.dlrm_ceiling_gather(p, None, 4, 256, p, None) == -1
    assert L.dlrm_ceiling_gather(p, p, 0, 256, p, None) == -2
    assert L.dlrm_ceiling_gather(p, p, 4, 100, p, None) == -2
    assert L.dlrm_ceiling_rmw(None, p, 4, 256, None) == -1
    assert L.dlrm_ceiling_rmw(p, p, 4, 1024, None) == -2


def test_binding_raises_instead_of_falling_back():
    with pytest.raises(hot.DlrmError):
        binding._check("dlrm_emb_bag_fwd", -2)
    src = open(os.path.join(ROOT, "paper_1906_00091_amd", "binding.py")).read()
    assert "oracle" not in src.replace("no fallback", "")
