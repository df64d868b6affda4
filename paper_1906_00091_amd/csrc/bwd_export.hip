// dlrm_emb_bag_bwd_export_groups: the grouping stage alone, exported in canonical form so that
// index handling can be checked bit for bit.
#include "bwd_sort.h"

namespace dlrm {

// --- export (debug / parity): bucket sort written back, then canonical run lists --------------
__global__ __launch_bounds__(kThreads) void bucket_sort_only_kernel(GroupArgs a) {
  __shared__ SortLds s;
  if (blockIdx.x == 0) prepare_segments(a, s.smem);
  const Bucket b = bucket_of_block(a, blockIdx.x);
  if (b.n == 0) return;
  if (b.n > (uint32_t)kBktCap && b.low_bits >= 1 && b.low_bits <= kSegMaxBits) return;  // a segment
  uint32_t* kout = a.keys[0] + b.start;
  uint32_t* vout = a.vals[0] + b.start;
  if (b.n <= (uint32_t)kBktCap) {
    sort_bucket_lds(a, b, s);
    for (uint32_t i = threadIdx.x; i < b.n; i += kThreads) {
      kout[i] = s.skey[i];
      vout[i] = s.sval[i];
    }
    return;
  }
  const int src = sort_bucket_global(a, b, s);
  __syncthreads();
  if (src != 0) {
    for (uint32_t i = threadIdx.x; i < b.n; i += kThreads) {
      kout[i] = a.keys[1][b.start + i];
      vout[i] = a.vals[1][b.start + i];
    }
  }
}

__device__ inline bool is_head(const uint32_t* keys, int64_t pos, int64_t tbl_start) {
  return pos == tbl_start || keys[pos] != keys[pos - 1];
}

__global__ __launch_bounds__(kThreads) void heads_count_kernel(GroupArgs a) {
  __shared__ uint32_t smem[kNW + 1];
  TileInfo ti;
  uint32_t cnt = 0;
  const bool live = find_tile(a, blockIdx.x, ti, smem);
  if (live) {
    const uint32_t* keys = a.keys[0];
    for (int i = threadIdx.x; i < ti.count; i += kThreads)
      cnt += is_head(keys, ti.start + i, ti.tbl_start) ? 1u : 0u;
  }
  uint32_t total;
  block_exclusive_scan<kThreads>(cnt, smem, &total);
  if (threadIdx.x == 0) a.tile_heads[blockIdx.x] = total;  // dead tiles write 0
}

__global__ __launch_bounds__(1024) void heads_scan_kernel(GroupArgs a, int64_t nnz) {
  __shared__ uint32_t smem[1024 / DLRM_WAVE + 1];
  uint32_t carry = 0;
  for (int t0 = 0; t0 < a.nt_max; t0 += 1024) {
    const int t = t0 + threadIdx.x;
    const uint32_t v = t < a.nt_max ? a.tile_heads[t] : 0u;
    uint32_t total;
    const uint32_t ex = block_exclusive_scan<1024>(v, smem, &total);
    if (t < a.nt_max) a.tile_heads[t] = carry + ex;
    carry += total;
  }
  if (threadIdx.x == 0) {
    a.n_seg[0] = carry;
    a.seg_start[carry] = (uint32_t)nnz;  // sentinel: the last run ends at nnz
  }
}

__global__ __launch_bounds__(kThreads) void heads_write_kernel(GroupArgs a) {
  __shared__ uint32_t smem[kNW + 1];
  TileInfo ti;
  if (!find_tile(a, blockIdx.x, ti, smem)) return;
  const uint32_t* keys = a.keys[0];
  const uint32_t base = a.tile_heads[blockIdx.x];
  // thread t owns the contiguous positions [t*per, (t+1)*per) so that heads keep their order
  const int per = 1 << (a.tile_shift - 8);   // positions per thread: tile / kThreads
  uint32_t flags = 0, cnt = 0;
#pragma unroll
  for (int j = 0; j < kItems; ++j) {
    const int li = threadIdx.x * per + j;
    if (j < per && li < ti.count && is_head(keys, ti.start + li, ti.tbl_start)) {
      flags |= 1u << j;
      ++cnt;
    }
  }
  uint32_t total;
  uint32_t pos = base + block_exclusive_scan<kThreads>(cnt, smem, &total);
#pragma unroll
  for (int j = 0; j < kItems; ++j) {
    if (flags & (1u << j)) {
      a.seg_start[pos] = (uint32_t)(ti.start + threadIdx.x * per + j);
      a.seg_tbl[pos] = (uint32_t)ti.k;
      ++pos;
    }
  }
}

struct ExportArgs {
  int64_t* uniq_rows;
  int64_t* seg_start_out;
  int32_t* sorted_bag;
  int64_t* n_uniq;
  int64_t nnz;
};

__global__ __launch_bounds__(256) void export_kernel(GroupArgs a, ExportArgs e) {
  const uint32_t nseg = a.n_seg[0];
  const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t nth = (int64_t)gridDim.x * blockDim.x;
  for (int64_t p = tid; p < e.nnz; p += nth) e.sorted_bag[p] = (int32_t)a.vals[0][p];
  for (int64_t u = tid; u < nseg; u += nth) {
    const uint32_t k = a.seg_tbl[u];
    const int64_t tstart = a.tbl_off[k];
    // first run of table k: lower bound of tstart among the run heads
    int64_t lo = 0, hi = u;  // seg_start[hi] >= tstart
    while (lo < hi) {
      const int64_t mid = (lo + hi) >> 1;
      if ((int64_t)a.seg_start[mid] < tstart) lo = mid + 1; else hi = mid;
    }
    const int64_t local_u = u - lo;
    const uint32_t pos = a.seg_start[u];
    e.uniq_rows[tstart + local_u] = (int64_t)a.keys[0][pos];
    e.seg_start_out[tstart + local_u] = (int64_t)pos - tstart;
    const bool last_of_table = (u + 1 == nseg) || a.seg_tbl[u + 1] != k;
    if (last_of_table) e.n_uniq[k] = local_u + 1;
  }
}

__global__ void zero_i64_kernel(int64_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

}  // namespace dlrm

using namespace dlrm;

extern "C" int32_t dlrm_emb_bag_bwd_export_groups(const dlrm_sparse_batch* s, void* workspace,
                                                  size_t workspace_bytes, int64_t* uniq_rows,
                                                  int64_t* seg_start, int32_t* sorted_bag,
                                                  int64_t* n_uniq, void* stream) {
  int st = check_batch(s);
  if (st != DLRM_OK) return st;
  if (!uniq_rows || !seg_start || !sorted_bag || !n_uniq) return DLRM_ERR_NULL;
  WsLayout L;
  st = check_ws(s, workspace, workspace_bytes, &L);
  if (st != DLRM_OK) return st;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(zero_i64_kernel, dim3(div_up(s->K, 256)), dim3(256), 0, hs, n_uniq, s->K);
  DLRM_CHECK_LAUNCH();
  if (s->nnz_total == 0) return DLRM_OK;
  GroupArgs g;
  fill_group_args(g, s, L, workspace);
  g.weights = nullptr;  // the export is about rows and bags; (row, bag) pairs whatever the batch carries
  st = enqueue_partition(s, g, hs);
  if (st != DLRM_OK) return st;
  hipLaunchKernelGGL(bucket_sort_only_kernel, dim3((unsigned)s->K << g.top_bits), dim3(kThreads), 0, hs, g);
  DLRM_CHECK_LAUNCH();
  st = launch_segment_sort(g, hs);
  if (st != DLRM_OK) return st;
  hipLaunchKernelGGL(heads_count_kernel, dim3(g.nt_max), dim3(kThreads), 0, hs, g);
  DLRM_CHECK_LAUNCH();
  hipLaunchKernelGGL(heads_scan_kernel, dim3(1), dim3(1024), 0, hs, g, s->nnz_total);
  DLRM_CHECK_LAUNCH();
  hipLaunchKernelGGL(heads_write_kernel, dim3(g.nt_max), dim3(kThreads), 0, hs, g);
  DLRM_CHECK_LAUNCH();
  ExportArgs e;
  e.uniq_rows = uniq_rows;
  e.seg_start_out = seg_start;
  e.sorted_bag = sorted_bag;
  e.n_uniq = n_uniq;
  e.nnz = s->nnz_total;
  unsigned grid = div_up(s->nnz_total, 256);
  if (grid > 2048) grid = 2048;
  hipLaunchKernelGGL(export_kernel, dim3(grid), dim3(256), 0, hs, g, e);
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}
