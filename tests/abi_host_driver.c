/*
 * Host-side checks of the C ABI as a stand-alone C program (TEST INFRASTRUCTURE): every entry point is
 * called with arguments that must be rejected on the host, before anything is launched, so the program
 * needs no GPU.  The CPU tests build the library with AddressSanitizer and UndefinedBehaviorSanitizer on
 * its host code, build this file the same way, link the two and run it.
 */
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "dlrm_hot.h"

static int fails = 0;
#define EXPECT(call, want)                                                              \
  do {                                                                                  \
    const long got_ = (long)(call);                                                     \
    if (got_ != (long)(want)) {                                                         \
      fprintf(stderr, "abi_host_driver: %s = %ld, expected %ld\n", #call, got_, (long)(want)); \
      ++fails;                                                                          \
    }                                                                                   \
  } while (0)

static dlrm_sparse_batch batch(void) {
  dlrm_sparse_batch b;
  memset(&b, 0, sizeof(b));
  b.K = 2;
  b.B = 4;
  b.d = 16;
  b.table_dtype = DLRM_F32;
  b.nnz_total = 8;
  b.max_rows = 100;
  b.tables = (void* const*)0x1000;
  b.rows = (const int64_t*)0x1000;
  b.indices = (const void*)0x1000;
  b.offsets = (const int64_t*)0x1000;
  b.tbl_off = (const int64_t*)0x1000;
  b.weights = NULL;
  b.index_dtype = DLRM_I64;
  return b;
}

int main(void) {
  float* p = (float*)0x1000;
  dlrm_sparse_batch b = batch(), t;
  EXPECT(dlrm_version() >= 100, 1);
  EXPECT(strcmp(dlrm_status_string(0), "ok"), 0);
  EXPECT(dlrm_status_string(-99) != NULL, 1);
  /* forward */
  EXPECT(dlrm_emb_bag_fwd(NULL, p, 64, 16, NULL), DLRM_ERR_NULL);
  EXPECT(dlrm_emb_bag_fwd(&b, NULL, 64, 16, NULL), DLRM_ERR_NULL);
  t = b; t.K = 0;
  EXPECT(dlrm_emb_bag_fwd(&t, p, 64, 16, NULL), DLRM_ERR_BAD_SHAPE);
  t = b; t.d = 6;
  EXPECT(dlrm_emb_bag_fwd(&t, p, 64, 16, NULL), DLRM_ERR_BAD_SHAPE);
  t = b; t.table_dtype = 7;
  EXPECT(dlrm_emb_bag_fwd(&t, p, 64, 16, NULL), DLRM_ERR_BAD_DTYPE);
  t = b; t.nnz_total = -1;
  EXPECT(dlrm_emb_bag_fwd(&t, p, 64, 16, NULL), DLRM_ERR_BAD_SHAPE);
  t = b; t.max_rows = 1ll << 31;
  EXPECT(dlrm_emb_bag_fwd(&t, p, 64, 16, NULL), DLRM_ERR_BAD_SHAPE);
  t = b; t.K = 1 << 20; t.B = 1 << 12;
  EXPECT(dlrm_emb_bag_fwd(&t, p, 64, 16, NULL), DLRM_ERR_BAD_SHAPE);
  t = b; t.index_dtype = 2;
  EXPECT(dlrm_emb_bag_fwd(&t, p, 64, 16, NULL), DLRM_ERR_BAD_DTYPE);
  EXPECT(dlrm_emb_bag_fwd(&b, p, 64, 8, NULL), DLRM_ERR_BAD_SHAPE);
  EXPECT(dlrm_emb_bag_fwd(&b, (float*)0x1004, 64, 16, NULL), DLRM_ERR_BAD_SHAPE);
  /* one-call forward and its backward */
  EXPECT(dlrm_emb_interact_fwd(&b, NULL, p, p, DLRM_FWD_AUTO, NULL), DLRM_ERR_NULL);
  EXPECT(dlrm_emb_interact_fwd(&b, p, NULL, p, DLRM_FWD_SPLIT, NULL), DLRM_ERR_NULL);
  EXPECT(dlrm_emb_interact_fwd(&b, p, p, p, 3, NULL), DLRM_ERR_BAD_ALGO);
  t = b; t.K = 65;
  EXPECT(dlrm_emb_interact_fwd(&t, p, p, p, DLRM_FWD_FUSED, NULL), DLRM_ERR_BAD_ALGO);
  EXPECT(dlrm_emb_interact_bwd(&t, p, p, p, NULL), DLRM_ERR_BAD_ALGO);
  EXPECT(dlrm_emb_interact_bwd(&b, p, NULL, p, NULL), DLRM_ERR_NULL);
  EXPECT(dlrm_emb_interact_fwd_stamped(&b, NULL, p, p, DLRM_FWD_AUTO, (uint32_t*)0x1000, 5, NULL), DLRM_ERR_NULL);
  /* interaction, helpers */
  EXPECT(dlrm_interact_dot_fwd(NULL, 4, 3, 16, p, NULL), DLRM_ERR_NULL);
  EXPECT(dlrm_interact_dot_fwd(p, 4, 500, 16, p, NULL), DLRM_ERR_BAD_SHAPE);
  EXPECT(dlrm_interact_dot_bwd(p, p, 4, 3, 16, NULL, NULL), DLRM_ERR_NULL);
  EXPECT(dlrm_place_dense(p, 4, 16, NULL, 3, NULL), DLRM_ERR_NULL);
  EXPECT(dlrm_lengths_to_offsets((const int32_t*)p, 0, 4, (int64_t*)p, (int64_t*)p, NULL), DLRM_ERR_BAD_SHAPE);
  EXPECT(dlrm_validate_csr(&b, NULL, NULL), DLRM_ERR_NULL);
  EXPECT(dlrm_table_init_hash(p, 10, 6, DLRM_F32, 1, 1.0f, NULL), DLRM_ERR_BAD_SHAPE);
  /* backward: workspace query and checks */
  const size_t need = dlrm_emb_bag_bwd_workspace_bytes(2, 4, 16, 8, 100, DLRM_F32);
  EXPECT(need > 0 && need % 256 == 0, 1);
  EXPECT(dlrm_emb_bag_bwd_workspace_bytes(0, 4, 16, 8, 100, DLRM_F32), 0);
  EXPECT(dlrm_emb_bag_bwd_workspace_bytes(2, 4, 16, 8, 100, 5), 0);
  EXPECT(dlrm_emb_bag_bwd_workspace_bytes(64, 16384, 128, 33554432, 2000000, DLRM_F16) > (size_t)33554432 * 16, 1);
  EXPECT(dlrm_emb_bag_bwd_workspace_bytes(2, 4, 16, DLRM_MAX_NNZ, 100, DLRM_F32) > (size_t)DLRM_MAX_NNZ * 16, 1);
  EXPECT(dlrm_emb_bag_bwd_sgd(&b, p, 64, 16, 0.01f, NULL, 0, DLRM_BWD_SORT, NULL), DLRM_ERR_WORKSPACE);
  EXPECT(dlrm_emb_bag_bwd_sgd(&b, p, 64, 16, 0.01f, (void*)0x1000, need - 1, DLRM_BWD_SORT, NULL), DLRM_ERR_WORKSPACE);
  EXPECT(dlrm_emb_bag_bwd_sgd(&b, p, 64, 16, 0.01f, (void*)0x1010, need, DLRM_BWD_SORT, NULL), DLRM_ERR_WORKSPACE);
  EXPECT(dlrm_emb_bag_bwd_sgd(&b, p, 64, 16, 0.01f, (void*)0x1000, need, 9, NULL), DLRM_ERR_BAD_ALGO);
  t = b; t.table_dtype = DLRM_F16;
  EXPECT(dlrm_emb_bag_bwd_sgd(&t, p, 64, 16, 0.01f, (void*)0x1000, need, DLRM_BWD_ATOMIC, NULL), DLRM_ERR_BAD_DTYPE);
  t = b; t.K = 65536; t.B = 1;
  EXPECT(dlrm_emb_bag_bwd_sgd(&t, p, 64, 16, 0.01f, (void*)0x1000, (size_t)1 << 40, DLRM_BWD_SORT, NULL), DLRM_ERR_BAD_SHAPE);
  dlrm_bwd_timing tm = {(void*)0x10, NULL};
  EXPECT(dlrm_emb_bag_bwd_sgd_timed(&b, p, 64, 16, 0.01f, (void*)0x1000, need, DLRM_BWD_SORT, &tm, NULL), DLRM_ERR_NULL);
  EXPECT(dlrm_emb_bag_bwd_adagrad(&b, NULL, p, 64, 16, 0.01f, 1e-8f, (void*)0x1000, need, DLRM_BWD_SORT, NULL), DLRM_ERR_NULL);
  EXPECT(dlrm_emb_bag_bwd_adagrad(&b, (void* const*)0x1000, p, 64, 16, 0.01f, 0.0f, (void*)0x1000, need, DLRM_BWD_SORT, NULL),
         DLRM_ERR_BAD_SHAPE);
  EXPECT(dlrm_emb_bag_bwd_adagrad(&b, (void* const*)0x1000, p, 64, 16, 0.01f, 1e-8f, (void*)0x1000, need, DLRM_BWD_ATOMIC, NULL),
         DLRM_ERR_BAD_ALGO);
  EXPECT(dlrm_emb_bag_bwd_prepare(&b, NULL, 0, NULL), DLRM_ERR_WORKSPACE);
  EXPECT(dlrm_emb_bag_bwd_prepared_oversized(&b, (void*)0x1000, need, NULL, NULL), DLRM_ERR_NULL);
  EXPECT(dlrm_emb_bag_bwd_route_counts(&b, (void*)0x1000, need, NULL, NULL), DLRM_ERR_NULL);
  EXPECT(dlrm_emb_bag_bwd_export_groups(&b, NULL, 0, (int64_t*)p, (int64_t*)p, (int32_t*)p, (int64_t*)p, NULL) != DLRM_OK, 1);
  /* the update on the library's own scratch: a batch beyond the array is refused before anything is touched */
  t = b; t.B = 30000; t.nnz_total = 3000000;
  EXPECT(dlrm_emb_bag_bwd_sgd_noalloc(&t, p, 64, 16, 0.01f, NULL), DLRM_ERR_WORKSPACE);
  EXPECT(dlrm_emb_bag_bwd_sgd_noalloc(NULL, p, 64, 16, 0.01f, NULL), DLRM_ERR_NULL);
  if (fails) return 1;
  printf("abi_host_driver ok\n");
  return 0;
}
