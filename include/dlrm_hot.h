/*
 * dlrm_hot -- the sparse-feature hot path of DLRM on one MI355X (gfx950).
 *
 * C ABI.  Every pointer is a DEVICE pointer owned by the caller unless a
 * comment says "host".  The library allocates nothing, keeps no state between
 * calls (one exception, stated at dlrm_emb_bag_bwd_sgd_noalloc), and only enqueues work on the
 * HIP stream passed as `stream` (a hipStream_t cast to void*; NULL = the default stream).  No call
 * synchronises with the host.
 *
 * Every function returns a status: DLRM_OK, or a negative DLRM_ERR_* value.
 * Argument errors are detected on the host BEFORE anything is launched; a
 * failed launch is reported as DLRM_ERR_HIP.
 *
 * Notation (follows the paper): K embedding tables, table k is
 * W_k in R^{m_k x d} stored row-major and contiguous; mini-batch size B; the
 * lookups of table k form B "bags" given in the CSR-like encoding of Sec. 4.1
 * (indices + offsets); F = K + 1 vectors enter the interaction (the processed
 * dense vector x and the K pooled vectors); P = F(F-1)/2 distinct pairs.
 */
#ifndef DLRM_HOT_H_
#define DLRM_HOT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* status codes */
#define DLRM_OK 0
#define DLRM_ERR_NULL (-1)      /* a required pointer is NULL */
#define DLRM_ERR_BAD_SHAPE (-2) /* K, B, d, F, strides, nnz or max_rows outside the supported range */
#define DLRM_ERR_BAD_DTYPE (-3) /* unknown table dtype, or dtype not supported by the chosen algo */
#define DLRM_ERR_WORKSPACE (-4) /* workspace NULL, misaligned or smaller than the query says */
#define DLRM_ERR_BAD_ALGO (-5)  /* unknown algorithm, or one that cannot take this batch */
#define DLRM_ERR_HIP (-6)       /* a HIP call / kernel launch failed */

/* table storage types.  The paper uses fp32 parameters (Sec. 5); fp16/bf16
 * storage is an extension: rows are widened exactly, all sums are fp32, and a
 * row is rounded to nearest-even once when it is written back. */
#define DLRM_F32 0
#define DLRM_F16 1
#define DLRM_BF16 2

/* element type of a batch's index array (Sec. 5, opening paragraph: the framework operators take
 * int64 or int32 indices) */
#define DLRM_I64 0 /* int64 (what the five workloads use) */
#define DLRM_I32 1 /* int32: 4 bytes less traffic per lookup */

/* backward algorithms */
#define DLRM_BWD_AUTO 0   /* library's measured choice for the shape */
#define DLRM_BWD_SORT 1   /* group (row, bag) pairs by row, reduce, one update per row; deterministic */
#define DLRM_BWD_ATOMIC 2 /* fp32 tables only: one hardware fp32 atomic add per looked-up element */
#define DLRM_BWD_SORT_PREPARED 3 /* DLRM_BWD_SORT whose grouping dlrm_emb_bag_bwd_prepare already did */
#define DLRM_BWD_SORT_PREPARED_FLAT 4 /* ... for a prepared batch without oversized buckets: the reduce launch
                                         alone (see dlrm_emb_bag_bwd_prepared_oversized) */

/* forward paths of dlrm_emb_interact_fwd */
#define DLRM_FWD_AUTO 0  /* fused for short bags (mean <= 4 rows) without weights and K <= 64, else split */
#define DLRM_FWD_FUSED 1 /* one launch: a wavefront pools a sample's K bags and multiplies them */
#define DLRM_FWD_SPLIT 2 /* dlrm_place_dense, dlrm_emb_bag_fwd, dlrm_interact_dot_fwd in turn */

/* supported ranges */
#define DLRM_MAX_ROW_BYTES 1024         /* d * sizeof(element) <= 1024, multiple of 16 */
#define DLRM_MAX_ROWS 2147483647LL      /* m_k < 2^31 */
#define DLRM_MAX_NNZ 2147483647LL       /* total lookups per batch < 2^31 */
#define DLRM_MAX_INTERACT_F 128         /* F <= 128 */
#define DLRM_MAX_BWD_TABLES 65535        /* the backward takes K <= 65535 (tables are a grid dimension) */
/* also: K * (B + 1) <= DLRM_MAX_NNZ (bags are numbered in 32 bits); the backward needs d <= 256 */

/*
 * One mini-batch of sparse lookups for all K tables (Sec. 2.1.1, Eq. (2);
 * encoding of Sec. 4.1: concatenated indices delineated by offsets).
 * The struct itself lives in HOST memory; the arrays it points to are DEVICE
 * arrays.  Indices are 0-based, 0 <= index < rows[k] (the paper's example uses
 * index 0).  The hot calls do NOT range-check indices: an out-of-range index is
 * undefined behaviour; dlrm_validate_csr is the checked path.
 */
typedef struct dlrm_sparse_batch {
  int32_t K;               /* number of tables, >= 1 */
  int32_t B;               /* bags per table (mini-batch size), >= 1 */
  int32_t d;               /* embedding dimension; d*elem_size a multiple of 16, <= DLRM_MAX_ROW_BYTES */
  int32_t table_dtype;     /* DLRM_F32 | DLRM_F16 | DLRM_BF16 */
  int64_t nnz_total;       /* host copy of tbl_off[K]: total lookups, 0 <= nnz_total <= DLRM_MAX_NNZ */
  int64_t max_rows;        /* host upper bound on rows[k] over all k, 1 <= max_rows <= DLRM_MAX_ROWS */
  void* const* tables;     /* [K] base pointer of table k: [rows[k], d] row-major, 16-byte aligned */
  const int64_t* rows;     /* [K] m_k */
  const void* indices;     /* [nnz_total] int64 (or int32, see index_dtype), table-major: table k owns
                              [tbl_off[k], tbl_off[k+1]) */
  const int64_t* offsets;  /* [K*(B+1)] per-table local offsets; bag b of table k = positions
                              [offsets[k*(B+1)+b], offsets[k*(B+1)+b+1]); offsets[k*(B+1)+B] = nnz_k */
  const int64_t* tbl_off;  /* [K+1] start of table k's slice in `indices` */
  const float* weights;    /* NULL, or [nnz_total] fp32 parallel to `indices`: the weight a of every
                              lookup in Eq. (2).  NULL = all ones (sum pooling, what the five workloads
                              use).  With weights, bag b of table k pools sum_p weights[p] * W_k[indices[p],:]
                              and the backward sums weights[p] * dS[bag(p)]; the weights get no gradient. */
  int32_t index_dtype;     /* DLRM_I64 (0) or DLRM_I32: element type of `indices` */
} dlrm_sparse_batch;

/* Library version (major*10000 + minor*100 + patch). */
int32_t dlrm_version(void);

/* Static, host-side text for a status code. */
const char* dlrm_status_string(int32_t status);

/*
 * CSR helper (Sec. 4.1 footnote: lengths, as SparseLengthsSum takes them, vs
 * offsets, as EmbeddingBag takes them).  Exclusive scan per table:
 *   offsets[k*(B+1)+0] = 0, offsets[k*(B+1)+b+1] = offsets[k*(B+1)+b] + lengths[k*B+b]
 *   tbl_off[0] = 0, tbl_off[k+1] = tbl_off[k] + offsets[k*(B+1)+B]
 * lengths: [K*B] int32, each >= 0.  Integer work, exact.
 */
int32_t dlrm_lengths_to_offsets(const int32_t* lengths, int32_t K, int32_t B, int64_t* offsets,
                                int64_t* tbl_off, void* stream);

/*
 * Checked path for a batch: writes to *n_bad (device int64 scalar) the number of
 * violations: offsets[k][0] != 0, decreasing offsets, offsets[k][B] != nnz_k,
 * tbl_off not matching, index < 0 or >= rows[k].  Reads only inside the arrays'
 * stated extents whatever their contents.
 */
int32_t dlrm_validate_csr(const dlrm_sparse_batch* batch, int64_t* n_bad, void* stream);

/*
 * Pooled embedding lookup, Eq. (2) (Eq. (1) when a bag has one index):
 * out[b*stride_b + k*stride_k + c] = sum over the bag's positions p of
 * a_p * W_k[indices[p], c], c < d, with a_p = batch->weights[p], or 1 when the batch
 * has no weights (sum pooling).  An index repeated inside a bag counts once per
 * occurrence; an empty bag gives zeros.  Sums are fp32, positions in ascending
 * order per lane group; a one-index bag is an exact copy of the row (widened).
 * out: fp32, strides in elements, stride_k >= d, 16-byte aligned rows
 * (stride_b, stride_k multiples of 4).  Writing straight into rows 1..K of the
 * interaction input T[B,F,d] is: out = T + d, stride_b = F*d, stride_k = d.
 */
int32_t dlrm_emb_bag_fwd(const dlrm_sparse_batch* batch, float* out, int64_t stride_b,
                         int64_t stride_k, void* stream);

/*
 * Places the processed dense vector (the bottom MLP's output, same length as the
 * embedding vectors, Sec. 2.2) as row 0 of the interaction input:
 * T[b,0,:] = x[b,:].  x: [B,d] fp32; T: [B,F,d] fp32.  Exact copy.  d multiple of 4.
 */
int32_t dlrm_place_dense(const float* x, int32_t B, int32_t d, float* T, int32_t F, void* stream);

/*
 * Dot-product feature interaction (Sec. 2.2: dot products between all pairs of
 * the F vectors, concatenated with the processed dense vector; distinct pairs
 * only, as the strict triangle in Eq. (4)).
 *   R[b, 0:d]                    = T[b,0,:]                       (exact copy)
 *   R[b, d + i(i-1)/2 + j]       = <T[b,i,:], T[b,j,:]>,  1 <= i < F, 0 <= j < i
 * T: [B,F,d] fp32 contiguous; R: [B, d + P] fp32 contiguous.  fp32 FMA.
 * Requires d a multiple of 4, 1 <= F <= DLRM_MAX_INTERACT_F.
 */
int32_t dlrm_interact_dot_fwd(const float* T, int32_t B, int32_t F, int32_t d, float* R,
                              void* stream);

/*
 * The forward of the sparse side in one call (Sec. 2.2: the processed dense vector and the
 * pooled vectors of Eq. (2) are the F = K + 1 vectors the dot interaction pairs up):
 *   T[b,0,:] = x[b,:];  T[b,k+1,:] = pooled vector of bag (k,b);  R = interaction of T
 * with the values dlrm_place_dense, dlrm_emb_bag_fwd(out = T + d, stride_b = F*d,
 * stride_k = d) and dlrm_interact_dot_fwd define; T is written because the backward reads it.
 * x: [B,d] fp32, T: [B,F,d] fp32, R: [B, d + F(F-1)/2] fp32, all device, contiguous, x and T
 * 16-byte aligned.  Requires K + 1 <= DLRM_MAX_INTERACT_F and d a multiple of 4.
 * T may be NULL where the one-launch path runs (DLRM_FWD_FUSED, or DLRM_FWD_AUTO choosing it): T is
 * then never written, for a caller whose backward is dlrm_emb_interact_bwd; elsewhere a NULL T is
 * DLRM_ERR_NULL.
 * algo: DLRM_FWD_FUSED needs a batch without weights and K <= 64 (else DLRM_ERR_BAD_ALGO); it
 * adds a bag's rows one by one in ascending position order (a one-index bag is an exact copy
 * of its row), each lane walking one bag, so it is meant for bags of a few rows;
 * DLRM_FWD_AUTO takes it up to a mean bag length of 4.  The paths differ in rounding order only.
 */
int32_t dlrm_emb_interact_fwd(const dlrm_sparse_batch* batch, const float* x, float* T, float* R,
                              int32_t algo, void* stream);

/*
 * The same call with a start stamp.  stamp: one uint32 the device can write (e.g. pinned host
 * memory), or NULL for none.  The first kernel of the call stores stamp_value there as it
 * begins to execute (a system-scope store: it does not wait for the end of the kernel).
 * By stream order everything enqueued on `stream` before this call has completed by then, so
 * a host that polls the word learns it without an event on the stream -- e.g. that the
 * previous step's update is done with its backward workspace, which may now be prepared
 * for another batch on a second stream.  (An event record costs the stream about 6 us on
 * MI355X; the stamp rides in a kernel that runs anyway.)
 */
int32_t dlrm_emb_interact_fwd_stamped(const dlrm_sparse_batch* batch, const float* x, float* T, float* R,
                                      int32_t algo, uint32_t* stamp, uint32_t stamp_value, void* stream);

/*
 * Backward of the above by the chain rule (the paper prints none).  With
 * g_ij = dR[b, d + i(i-1)/2 + j]:
 *   dT[b,i,:] = sum_{j<i} g_ij T[b,j,:] + sum_{j>i} g_ji T[b,j,:]  (+ dR[b,0:d] for i = 0)
 * dT: [B,F,d] fp32; row 0 is the gradient of the dense vector, rows 1..K are dS,
 * the gradients of the pooled vectors.
 */
int32_t dlrm_interact_dot_bwd(const float* T, const float* dR, int32_t B, int32_t F, int32_t d,
                              float* dT, void* stream);

/*
 * Backward of dlrm_emb_interact_fwd without T (Sec. 2.2 by the chain rule, with the pooled vectors of
 * Eq. (2) formed again on the way): dT as dlrm_interact_dot_bwd(T, dR, ...) defines it, for the T that
 * dlrm_emb_interact_fwd(DLRM_FWD_FUSED) defines -- T[b,0,:] = x[b,:], T[b,k+1,:] = the bag's rows added
 * one by one in ascending position order -- bit for bit, but T is not an argument: a wavefront pools a
 * sample's K bags from the tables again while it multiplies.  A training step made of
 * dlrm_emb_interact_fwd(T = NULL), this call and the update never writes or reads T (per sample
 * 2*F*d floats of traffic less, the bags' rows read a second time instead).
 * The tables must still hold the values the forward pass read: call it BEFORE the update of the step.
 * x: [B,d] fp32, dR: [B, d + F(F-1)/2] fp32, dT: [B,F,d] fp32 (row 0: gradient of the dense vector,
 * rows 1..K: dS), device, contiguous, x and dT 16-byte aligned.  A batch without pooling weights and
 * K <= 64 (else DLRM_ERR_BAD_ALGO); each lane walks a bag, so it is meant for bags of a few rows.
 */
int32_t dlrm_emb_interact_bwd(const dlrm_sparse_batch* batch, const float* x, const float* dR, float* dT,
                              void* stream);

/*
 * Bytes of workspace dlrm_emb_bag_bwd_sgd / dlrm_emb_bag_bwd_export_groups need
 * for this shape (enough for every algo).  Returns 0 for an unsupported shape.
 */
size_t dlrm_emb_bag_bwd_workspace_bytes(int32_t K, int32_t B, int32_t d, int64_t nnz_total,
                                        int64_t max_rows, int32_t table_dtype);

/*
 * Embedding backward fused with the sparse SGD update (transpose of Eq. (2);
 * SGD without regularisation, Sec. 5.1).  For every distinct row r that table k
 * looks up in this batch:
 *   g = sum over positions p with indices[p] == r of dS[bag(p)*stride_b + k*stride_k + :]
 *   W_k[r,:] <- W_k[r,:] - lr * g
 * Rows that are not looked up keep their bits.  Tables are updated in place.
 * DLRM_BWD_SORT: duplicates are summed first (fp32, ascending position) and
 * the row is written once (one rounding for fp16/bf16); bitwise reproducible.
 * DLRM_BWD_ATOMIC: fp32 tables only; each occurrence is applied with a hardware
 * fp32 atomic add of -lr*dS, so the rounding order varies from run to run.
 * dS: fp32, strides in elements (rows 1..K of dT: dS = dT + d, stride_b = F*d,
 * stride_k = d); 16-byte aligned rows.
 * workspace: device memory, 256-byte aligned, at least
 * dlrm_emb_bag_bwd_workspace_bytes(...) bytes; contents are scratch.
 * d <= 256 (a gradient row of d fp32 values is at most one wavefront of 16-byte pieces): fp16/bf16
 * tables with 256 < d <= 512 can be pooled but not updated (DLRM_ERR_BAD_SHAPE, here and in
 * dlrm_emb_bag_bwd_adagrad and dlrm_emb_bag_bwd_prepare).  K <= DLRM_MAX_BWD_TABLES (else
 * DLRM_ERR_BAD_SHAPE, before anything is launched).
 */
int32_t dlrm_emb_bag_bwd_sgd(const dlrm_sparse_batch* batch, const float* dS, int64_t stride_b,
                             int64_t stride_k, float lr, void* workspace, size_t workspace_bytes,
                             int32_t algo, void* stream);

/*
 * For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): dlrm_emb_bag_bwd_sgd with algo = DLRM_BWD_SORT, its
 * workspace being an array of DLRM_NOALLOC_SCRATCH_BYTES that the library holds on every GPU it
 * runs on from the moment it is loaded until the process ends.  Allocates nothing, frees nothing.
 * Same arguments, same launches, same bits as dlrm_emb_bag_bwd_sgd on a caller-owned workspace.
 * DLRM_ERR_WORKSPACE if dlrm_emb_bag_bwd_workspace_bytes(...) of this batch exceeds
 * DLRM_NOALLOC_SCRATCH_BYTES (about 24 bytes per lookup plus 4 KB per 4096 lookups and per table:
 * batches up to ~2.5 M lookups fit); nothing is launched then.
 * All calls on one GPU share that GPU's array: two calls that overlap in time (different streams,
 * or different host threads without stream order between them) race on it -- the caller orders
 * them.  The array keeps the previous call's contents; the first kernel of every call resets the
 * counters the later ones read, nothing else needs to start at zero.
 * The per-GPU address of the array is looked up on the first call on that GPU and kept (the one piece
 * of state the library holds).
 */
#define DLRM_NOALLOC_SCRATCH_BYTES (64u << 20)
int32_t dlrm_emb_bag_bwd_sgd_noalloc(const dlrm_sparse_batch* batch, const float* dS, int64_t stride_b,
                                     int64_t stride_k, float lr, void* stream);

/*
 * The same backward with sparse Adagrad in place of the SGD step (Sec. 5.1 trains with "SGD
 * and Adagrad"; the paper prints no formula: this is the standard element-wise rule applied
 * to the rows a batch touches, duplicates summed first as for SGD).  For every distinct row r
 * of table k, with g as in dlrm_emb_bag_bwd_sgd:
 *   h_k[r,:] <- h_k[r,:] + g*g
 *   W_k[r,:] <- W_k[r,:] - lr * g / (sqrt(h_k[r,:]) + eps)        (the updated h)
 * state: device array of K device pointers; state[k] is the fp32 accumulator h_k, row-major
 * [rows[k], d], 16-byte aligned, owned and initialised by the caller (zeros for a fresh
 * optimizer), updated in place.  Rows that are not looked up keep W and h bit for bit.
 * Arithmetic is fp32; fp16/bf16 tables are widened, updated and rounded once.
 * eps must be > 0 (else DLRM_ERR_BAD_SHAPE).  algo: DLRM_BWD_AUTO, DLRM_BWD_SORT,
 * DLRM_BWD_SORT_PREPARED or DLRM_BWD_SORT_PREPARED_FLAT (else DLRM_ERR_BAD_ALGO); bitwise reproducible.  Everything else
 * as for dlrm_emb_bag_bwd_sgd.
 */
int32_t dlrm_emb_bag_bwd_adagrad(const dlrm_sparse_batch* batch, void* const* state, const float* dS,
                                 int64_t stride_b, int64_t stride_k, float lr, float eps,
                                 void* workspace, size_t workspace_bytes, int32_t algo, void* stream);

/*
 * The index-only half of DLRM_BWD_SORT (Sec. 4.1: the indices of a batch are known
 * before its forward pass): partitions the batch's (row, bag) pairs by row inside
 * `workspace`.  It reads indices, offsets, tbl_off, rows and, if the batch has them, the
 * weights (copied beside the bag of every lookup) -- no table, no
 * gradient -- so a caller may enqueue it on a second stream while the forward pass
 * and the interaction run, then call dlrm_emb_bag_bwd_sgd with
 * algo = DLRM_BWD_SORT_PREPARED, the same batch and the same workspace once both
 * streams have met (the caller orders the two calls, e.g. with an event; nothing
 * else may touch the workspace in between).  Prepare + prepared update perform the
 * same launches as one DLRM_BWD_SORT call and give the same bits.
 * An update with DLRM_BWD_SORT_PREPARED on a workspace that was not prepared for
 * this batch is undefined (it is not detected).
 */
int32_t dlrm_emb_bag_bwd_prepare(const dlrm_sparse_batch* batch, void* workspace,
                                 size_t workspace_bytes, void* stream);

/*
 * After dlrm_emb_bag_bwd_prepare (same batch, same workspace, same stream or ordered after
 * it): writes to *n_oversized the number of row groups of the batch that are too large for
 * one workgroup's sort in LDS (more than 2048 lookups falling into one of the row ranges the
 * grouping cuts a table into: heavy-hitter rows, or tables much smaller than the batch).
 * n_oversized: one uint32 the device can write, e.g. pinned host memory, which the caller
 * reads once the stream has passed this call.
 * Zero means the update needs none of its segment / hot-row launches (launches that
 * would find nothing to do): DLRM_BWD_SORT_PREPARED_FLAT then enqueues the reduce kernel
 * alone and gives the same bits as DLRM_BWD_SORT_PREPARED.  With oversized groups FLAT is
 * still correct, but each is handled by a single workgroup (slow for heavy hitters) and long
 * runs are summed in another order; a caller that picks FLAT exactly when the count is zero
 * keeps results a function of the batch alone.
 */
int32_t dlrm_emb_bag_bwd_prepared_oversized(const dlrm_sparse_batch* batch, void* workspace,
                                            size_t workspace_bytes, uint32_t* n_oversized, void* stream);

/*
 * Diagnostic (for tests of the update's rarely taken routes; not part of the method).  After a
 * DLRM_BWD_SORT* update (dlrm_emb_bag_bwd_sgd or _adagrad) of `batch` with `workspace`, same stream
 * or ordered after it: copies to counts[0..9] (device, uint32) how the update handled the row
 * groups of this batch (transpose of Eq. (2): every lookup of a row must reach that row's sum once):
 *   [0] heavy row ranges handed to the first workgroups   [1] of them too large for one LDS sort
 *   [2] lists sorted by many workgroups ("segments")      [3] their 2048-pair tiles
 *   [4] oversized ranges that split off dominant rows     [5] lists one workgroup sorted through memory
 *   [6] oversized ranges holding a single row             [7] runs > 2048 summed by one workgroup
 *   [8] hot rows (runs > 2048) summed by the bag-group kernels, all tables
 *   [9] tables whose hot rows took the dense (matrix core) kernel
 * DLRM_ERR_BAD_SHAPE for an empty batch (nothing ran).
 */
int32_t dlrm_emb_bag_bwd_route_counts(const dlrm_sparse_batch* batch, void* workspace,
                                      size_t workspace_bytes, uint32_t* counts, void* stream);

/*
 * Runs only the grouping stage of DLRM_BWD_SORT and exports it in canonical
 * form, for checking index handling bit for bit.  Per table k, in that table's
 * slice [tbl_off[k], tbl_off[k+1]) of each output array:
 *   uniq_rows  (int64) : distinct rows ascending, first n_uniq[k] entries
 *   seg_start  (int64) : start of each row's run in sorted_bag, local to the slice
 *   sorted_bag (int32) : bag of every position, ordered by (row asc, position asc)
 *   n_uniq     (int64) : [K]
 * Entries of uniq_rows / seg_start past n_uniq[k] are left untouched.
 */
int32_t dlrm_emb_bag_bwd_export_groups(const dlrm_sparse_batch* batch, void* workspace,
                                       size_t workspace_bytes, int64_t* uniq_rows,
                                       int64_t* seg_start, int32_t* sorted_bag, int64_t* n_uniq,
                                       void* stream);

/*
 * Synthetic-input helper (not part of the method): fills a table with the
 * counter-based uniform initialiser U(-scale, scale):
 *   h = mix(key + row*d + col); u = h >> 40; x = (2u + 1 - 2^24) / 2^24;
 *   W[row,col] = fp32(x) * scale, rounded once to the table dtype,
 * mix = the splitmix64 output function.  Lets a table of tens of GB be created
 * on the device and any row be re-derived on the host.
 */
int32_t dlrm_table_init_hash(void* table, int64_t rows, int32_t d, int32_t table_dtype,
                             uint64_t key, float scale, void* stream);

/*
 * Timing aid (not part of the method): dlrm_emb_bag_bwd_sgd / dlrm_emb_bag_bwd_adagrad with a pair of
 * caller-owned HIP events for THIS call.  On the sort path ev_start is recorded on `stream`
 * immediately before and ev_stop immediately after the launch of the call's dominant kernel (the
 * bucket sort + row reduce + row update), so a benchmark can time that one kernel with HIP events
 * on the stream it runs on.  timing == NULL, or both events NULL: exactly the plain call.  One event
 * NULL and the other not: DLRM_ERR_NULL.  With DLRM_BWD_ATOMIC the events bracket its one launch.
 */
typedef struct dlrm_bwd_timing {
  void* ev_start; /* hipEvent_t */
  void* ev_stop;  /* hipEvent_t */
} dlrm_bwd_timing;
int32_t dlrm_emb_bag_bwd_sgd_timed(const dlrm_sparse_batch* batch, const float* dS, int64_t stride_b,
                                   int64_t stride_k, float lr, void* workspace, size_t workspace_bytes,
                                   int32_t algo, const dlrm_bwd_timing* timing, void* stream);
int32_t dlrm_emb_bag_bwd_adagrad_timed(const dlrm_sparse_batch* batch, void* const* state, const float* dS,
                                       int64_t stride_b, int64_t stride_k, float lr, float eps,
                                       void* workspace, size_t workspace_bytes, int32_t algo,
                                       const dlrm_bwd_timing* timing, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DLRM_HOT_H_ */
