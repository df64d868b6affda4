// Entry points of the embedding backward (transpose of Eq. (2) fused with the row update of
// Sec. 5.1) and the ATOMIC path.  The SORT path is described in bwd_common.h.
// ATOMIC path (fp32 tables): a lane group per bag adds -lr*dS[b,k,:] to every row of the bag
// with hardware fp32 atomics; no workspace, one launch.  Measured 6x slower than SORT on the
// 8 x 1M x 64 multi-hot workload, so AUTO always takes SORT.
#include "bwd_common.h"

#include <mutex>

namespace dlrm {

// Backward workspace of dlrm_emb_bag_bwd_sgd_noalloc: one array per GPU, held until the process
// ends.  The name below is a host-side stand-in; host code only ever uses the per-device address
// that hipGetSymbolAddress returns (scratch_base).
static __device__ __align__(256) unsigned char scratch[DLRM_NOALLOC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mu;

// Address of the current device's copy of `scratch` (looked up once per device).
static int scratch_base(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return DLRM_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return DLRM_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return DLRM_OK;
}

// --- ATOMIC path --------------------------------------------------------------------
struct AtomArgs {
  void* const* tables;
  const void* indices;
  int32_t idx32;
  const int64_t* offsets;
  const int64_t* tbl_off;
  const float* weights;  // NULL = sum pooling
  const float* dS;
  int64_t stride_b, stride_k;
  float lr;
  int32_t K, B, d;
};

template <int G>
__global__ __launch_bounds__(256) void atomic_update_kernel(AtomArgs a) {
  constexpr int S = DLRM_WAVE / G;
  const int lane = lane_id();
  const int slot = lane / G, chunk = lane % G;
  const uint32_t bag = (blockIdx.x * (blockDim.x >> 6) + wave_id()) * S + slot;
  if (bag >= (uint32_t)a.K * (uint32_t)a.B || chunk * 4 >= a.d) return;
  const int k = (int)(bag / (uint32_t)a.B), b = (int)(bag - (uint32_t)k * (uint32_t)a.B);
  const int64_t* off = a.offsets + (int64_t)k * (a.B + 1);
  const int64_t p0 = off[b], p1 = off[b + 1];
  if (p1 <= p0) return;
  const int64_t tbl = a.tbl_off[k];
  const float* wts = a.weights ? a.weights + tbl : nullptr;
  float* W = static_cast<float*>(a.tables[k]) + chunk * 4;
  f32x4 g = loadf4(a.dS + (int64_t)b * a.stride_b + (int64_t)k * a.stride_k + chunk * 4);
  g *= -a.lr;
  for (int64_t p = p0; p < p1; ++p) {
    float* w = W + index_at(a.indices, a.idx32, tbl + p) * a.d;
    const float ap = wts ? wts[p] : 1.0f;  // the lookup's weight in Eq. (2)
    unsafeAtomicAdd(w + 0, ap * g.x);
    unsafeAtomicAdd(w + 1, ap * g.y);
    unsafeAtomicAdd(w + 2, ap * g.z);
    unsafeAtomicAdd(w + 3, ap * g.w);
  }
}


// The sort path behind both optimizers' entry points: grouping (unless prepared), then the
// reduce launches with the row update OPT.
__global__ void copy_u32_kernel(const uint32_t* src, uint32_t* dst) { *dst = src ? *src : 0u; }

// One thread copies the counters an update left in the workspace (dlrm_emb_bag_bwd_route_counts).
__global__ void route_counts_kernel(GroupArgs a, uint32_t* out) {
  uint32_t hot = 0, dense = 0;
  for (int k = 0; k < a.K; ++k) {
    const uint32_t c = a.hot_cnt[k];
    hot += c;
    dense += (a.weights == nullptr && c >= (uint32_t)kDenseFrom) ? 1u : 0u;
  }
  out[0] = *a.list_cnt;
  out[1] = *a.over_cnt;
  out[2] = a.seg_meta[1];
  out[3] = a.seg_meta[0];
  out[4] = a.seg_meta[kRouteSplit];
  out[5] = a.seg_meta[kRouteGlobalSort];
  out[6] = a.seg_meta[kRouteOneRow];
  out[7] = a.seg_meta[kRouteHugeInPlace];
  out[8] = hot;
  out[9] = dense;
}

template <int OPT>
static int run_sort_path(const dlrm_sparse_batch* s, const UpdArgs& u, void* workspace, size_t workspace_bytes,
                         int algo, const dlrm_bwd_timing* tm, hipStream_t hs) {
  const bool prepared = algo == DLRM_BWD_SORT_PREPARED || algo == DLRM_BWD_SORT_PREPARED_FLAT;
  const int G = pow2_ceil(s->d / 4);  // lanes per fp32 gradient row
  if (G > DLRM_WAVE) return DLRM_ERR_BAD_SHAPE;
  WsLayout L;
  int st = check_ws(s, workspace, workspace_bytes, &L);
  if (st != DLRM_OK) return st;
  if (s->nnz_total == 0) return DLRM_OK;
  GroupArgs g;
  fill_group_args(g, s, L, workspace);
  if (!prepared) {
    st = enqueue_partition(s, g, hs);
    if (st != DLRM_OK) return st;
  }
  if (algo == DLRM_BWD_SORT_PREPARED_FLAT) g.no_tail = 1;  // the grouping itself does not depend on it
  if (g.weights != nullptr)
    return OPT == kAdagrad ? run_reduce_adagrad_weighted(g, u, s->table_dtype, G, s->K, tm, hs)
                           : run_reduce_sgd_weighted(g, u, s->table_dtype, G, s->K, tm, hs);
  return OPT == kAdagrad ? run_reduce_adagrad(g, u, s->table_dtype, G, s->K, tm, hs)
                         : run_reduce_sgd(g, u, s->table_dtype, G, s->K, tm, hs);
}

template <int G>
static int launch_atomic(const AtomArgs& a, const dlrm_bwd_timing* tm, hipStream_t st) {
  constexpr int S = DLRM_WAVE / G;
  if (tm && tm->ev_start && hipEventRecord(static_cast<hipEvent_t>(tm->ev_start), st) != hipSuccess) return DLRM_ERR_HIP;
  hipLaunchKernelGGL((atomic_update_kernel<G>), dim3(div_up((int64_t)a.K * a.B, 4 * S)), dim3(256), 0,
                     st, a);
  DLRM_CHECK_LAUNCH();
  if (tm && tm->ev_stop && hipEventRecord(static_cast<hipEvent_t>(tm->ev_stop), st) != hipSuccess) return DLRM_ERR_HIP;
  return DLRM_OK;
}

static bool timing_ok(const dlrm_bwd_timing* tm) { return !tm || ((tm->ev_start == nullptr) == (tm->ev_stop == nullptr)); }


}  // namespace dlrm

using namespace dlrm;

extern "C" size_t dlrm_emb_bag_bwd_workspace_bytes(int32_t K, int32_t B, int32_t d, int64_t nnz_total,
                                                   int64_t max_rows, int32_t table_dtype) {
  if (K < 1 || B < 1 || d < 1 || nnz_total < 0 || nnz_total > DLRM_MAX_NNZ || max_rows < 1 ||
      max_rows > DLRM_MAX_ROWS || !dtype_ok(table_dtype))
    return 0;
  return ws_layout(K, B, d, nnz_total).total;
}

extern "C" int32_t dlrm_emb_bag_bwd_sgd(const dlrm_sparse_batch* s, const float* dS, int64_t stride_b,
                                        int64_t stride_k, float lr, void* workspace,
                                        size_t workspace_bytes, int32_t algo, void* stream) {
  return dlrm_emb_bag_bwd_sgd_timed(s, dS, stride_b, stride_k, lr, workspace, workspace_bytes, algo, nullptr, stream);
}

extern "C" int32_t dlrm_emb_bag_bwd_sgd_timed(const dlrm_sparse_batch* s, const float* dS, int64_t stride_b,
                                              int64_t stride_k, float lr, void* workspace,
                                              size_t workspace_bytes, int32_t algo, const dlrm_bwd_timing* tm,
                                              void* stream) {
  int st = check_batch(s);
  if (st != DLRM_OK) return st;
  if (!dS || !timing_ok(tm)) return DLRM_ERR_NULL;
  if (s->K > DLRM_MAX_BWD_TABLES) return DLRM_ERR_BAD_SHAPE;
  if ((s->d & 3) || stride_k < s->d || (stride_k & 3) || (stride_b & 3) || stride_b < 0)
    return DLRM_ERR_BAD_SHAPE;
  if (reinterpret_cast<uintptr_t>(dS) & 15) return DLRM_ERR_BAD_SHAPE;
  if (algo != DLRM_BWD_AUTO && algo != DLRM_BWD_SORT && algo != DLRM_BWD_ATOMIC && algo != DLRM_BWD_SORT_PREPARED &&
      algo != DLRM_BWD_SORT_PREPARED_FLAT)
    return DLRM_ERR_BAD_ALGO;
  if (algo == DLRM_BWD_ATOMIC && s->table_dtype != DLRM_F32) return DLRM_ERR_BAD_DTYPE;
  if (algo == DLRM_BWD_AUTO) algo = DLRM_BWD_SORT;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const int G = pow2_ceil(s->d / 4);  // lanes per fp32 gradient row
  if (G > DLRM_WAVE) return DLRM_ERR_BAD_SHAPE;

  if (algo == DLRM_BWD_ATOMIC) {
    if (s->nnz_total == 0) return DLRM_OK;
    AtomArgs a;
    a.tables = s->tables;
    a.indices = s->indices;
    a.idx32 = s->index_dtype == DLRM_I32;
    a.offsets = s->offsets;
    a.tbl_off = s->tbl_off;
    a.weights = s->weights;
    a.dS = dS;
    a.stride_b = stride_b;
    a.stride_k = stride_k;
    a.lr = lr;
    a.K = s->K;
    a.B = s->B;
    a.d = s->d;
    switch (G) {
      case 1: return launch_atomic<1>(a, tm, hs);
      case 2: return launch_atomic<2>(a, tm, hs);
      case 4: return launch_atomic<4>(a, tm, hs);
      case 8: return launch_atomic<8>(a, tm, hs);
      case 16: return launch_atomic<16>(a, tm, hs);
      case 32: return launch_atomic<32>(a, tm, hs);
      case 64: return launch_atomic<64>(a, tm, hs);
    }
    return DLRM_ERR_BAD_SHAPE;
  }

  UpdArgs u;
  u.tables = s->tables;
  u.state = nullptr;
  u.dS = dS;
  u.stride_b = stride_b;
  u.stride_k = stride_k;
  u.lr = lr;
  u.eps = 0.0f;
  u.d = s->d;
  return run_sort_path<kSgd>(s, u, workspace, workspace_bytes, algo, tm, hs);
}

extern "C" int32_t dlrm_emb_bag_bwd_sgd_noalloc(const dlrm_sparse_batch* s, const float* dS, int64_t stride_b,
                                                int64_t stride_k, float lr, void* stream) {
  int st = check_batch(s);
  if (st != DLRM_OK) return st;
  // the size is checked before the address is looked up: a batch that does not fit touches nothing
  if (ws_layout(s->K, s->B, s->d, s->nnz_total).total > (size_t)DLRM_NOALLOC_SCRATCH_BYTES) return DLRM_ERR_WORKSPACE;
  void* ws = nullptr;
  st = scratch_base(&ws);
  if (st != DLRM_OK) return st;
  // every counter the update reads is zeroed by the first kernel of the grouping: nothing to clear here
  return dlrm_emb_bag_bwd_sgd(s, dS, stride_b, stride_k, lr, ws, (size_t)DLRM_NOALLOC_SCRATCH_BYTES, DLRM_BWD_SORT,
                              stream);
}

extern "C" int32_t dlrm_emb_bag_bwd_adagrad(const dlrm_sparse_batch* s, void* const* state, const float* dS,
                                            int64_t stride_b, int64_t stride_k, float lr, float eps,
                                            void* workspace, size_t workspace_bytes, int32_t algo,
                                            void* stream) {
  return dlrm_emb_bag_bwd_adagrad_timed(s, state, dS, stride_b, stride_k, lr, eps, workspace, workspace_bytes, algo,
                                        nullptr, stream);
}

extern "C" int32_t dlrm_emb_bag_bwd_adagrad_timed(const dlrm_sparse_batch* s, void* const* state, const float* dS,
                                                  int64_t stride_b, int64_t stride_k, float lr, float eps,
                                                  void* workspace, size_t workspace_bytes, int32_t algo,
                                                  const dlrm_bwd_timing* tm, void* stream) {
  int st = check_batch(s);
  if (st != DLRM_OK) return st;
  if (!dS || !state || !timing_ok(tm)) return DLRM_ERR_NULL;
  if ((s->d & 3) || stride_k < s->d || (stride_k & 3) || (stride_b & 3) || stride_b < 0)
    return DLRM_ERR_BAD_SHAPE;
  if (reinterpret_cast<uintptr_t>(dS) & 15) return DLRM_ERR_BAD_SHAPE;
  if (!(eps > 0.0f)) return DLRM_ERR_BAD_SHAPE;  // h = 0 and g = 0 would divide 0 by 0
  if (algo != DLRM_BWD_AUTO && algo != DLRM_BWD_SORT && algo != DLRM_BWD_SORT_PREPARED &&
      algo != DLRM_BWD_SORT_PREPARED_FLAT)
    return DLRM_ERR_BAD_ALGO;
  if (algo == DLRM_BWD_AUTO) algo = DLRM_BWD_SORT;
  UpdArgs u;
  u.tables = s->tables;
  u.state = state;
  u.dS = dS;
  u.stride_b = stride_b;
  u.stride_k = stride_k;
  u.lr = lr;
  u.eps = eps;
  u.d = s->d;
  return run_sort_path<kAdagrad>(s, u, workspace, workspace_bytes, algo, tm, static_cast<hipStream_t>(stream));
}

extern "C" int32_t dlrm_emb_bag_bwd_prepare(const dlrm_sparse_batch* s, void* workspace,
                                            size_t workspace_bytes, void* stream) {
  int st = check_batch(s);
  if (st != DLRM_OK) return st;
  if ((s->d & 3) || pow2_ceil(s->d / 4) > DLRM_WAVE) return DLRM_ERR_BAD_SHAPE;
  WsLayout L;
  st = check_ws(s, workspace, workspace_bytes, &L);
  if (st != DLRM_OK) return st;
  if (s->nnz_total == 0) return DLRM_OK;
  GroupArgs g;
  fill_group_args(g, s, L, workspace);
  return enqueue_partition(s, g, static_cast<hipStream_t>(stream));
}

extern "C" int32_t dlrm_emb_bag_bwd_route_counts(const dlrm_sparse_batch* s, void* workspace,
                                                 size_t workspace_bytes, uint32_t* counts, void* stream) {
  int st = check_batch(s);
  if (st != DLRM_OK) return st;
  if (!counts) return DLRM_ERR_NULL;
  if ((s->d & 3) || pow2_ceil(s->d / 4) > DLRM_WAVE) return DLRM_ERR_BAD_SHAPE;
  WsLayout L;
  st = check_ws(s, workspace, workspace_bytes, &L);
  if (st != DLRM_OK) return st;
  if (s->nnz_total == 0) return DLRM_ERR_BAD_SHAPE;  // an empty batch never wrote the counters
  GroupArgs g;
  fill_group_args(g, s, L, workspace);
  hipLaunchKernelGGL(route_counts_kernel, dim3(1), dim3(1), 0, static_cast<hipStream_t>(stream), g, counts);
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}

extern "C" int32_t dlrm_emb_bag_bwd_prepared_oversized(const dlrm_sparse_batch* s, void* workspace,
                                                       size_t workspace_bytes, uint32_t* n_oversized,
                                                       void* stream) {
  int st = check_batch(s);
  if (st != DLRM_OK) return st;
  if (!n_oversized) return DLRM_ERR_NULL;
  if ((s->d & 3) || pow2_ceil(s->d / 4) > DLRM_WAVE) return DLRM_ERR_BAD_SHAPE;
  WsLayout L;
  st = check_ws(s, workspace, workspace_bytes, &L);
  if (st != DLRM_OK) return st;
  GroupArgs g;
  fill_group_args(g, s, L, workspace);
  // (an empty batch was never partitioned: the counter may hold anything, and nothing is oversized)
  if (s->nnz_total == 0) g.over_cnt = nullptr;
  hipLaunchKernelGGL(copy_u32_kernel, dim3(1), dim3(1), 0, static_cast<hipStream_t>(stream), g.over_cnt,
                     n_oversized);
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}
