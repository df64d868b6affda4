"""DLRM sparse hot path on one MI355X: pooled embedding lookup, dot interaction,
their backward and the fused sparse SGD update, as hand-written HIP kernels
behind a C ABI (include/dlrm_hot.h).  This package is the thin binding."""
from .binding import (  # noqa: F401
    BF16, BWD_ATOMIC, BWD_AUTO, BWD_SORT, BWD_SORT_PREPARED, BWD_SORT_PREPARED_FLAT, F16, F32, FWD_AUTO, FWD_FUSED, FWD_SPLIT, DlrmError, SparseBatch, alloc_workspace,
    dlrm_emb_bag_bwd_adagrad, dlrm_emb_bag_bwd_export_groups, dlrm_emb_bag_bwd_route_counts, ROUTE_NAMES, dlrm_emb_bag_bwd_prepare, dlrm_emb_bag_bwd_prepared_oversized, dlrm_emb_bag_bwd_sgd, dlrm_emb_bag_bwd_sgd_noalloc, NOALLOC_SCRATCH_BYTES,
    state_pointers, dlrm_emb_bag_bwd_workspace_bytes,
    dlrm_emb_bag_fwd, dlrm_emb_interact_fwd, dlrm_emb_interact_bwd, dlrm_emb_interact_fwd_stamped, dlrm_interact_dot_bwd, dlrm_interact_dot_fwd, dlrm_lengths_to_offsets,
    dlrm_place_dense, dlrm_emb_bag_bwd_sgd_timed, dlrm_emb_bag_bwd_adagrad_timed, dlrm_table_init_hash, dlrm_validate_csr, lib, status_string, version,
)
