// Backward grouping, steps 1-3: most-significant-digit partition of the (row, bag) pairs.
#include "bwd_common.h"

namespace dlrm {

// --- 1. per-tile histogram of the partition digit ----------------------------------
template <typename IT>
__global__ __launch_bounds__(kThreads) void bucket_hist_kernel(GroupArgs a) {
  __shared__ uint32_t h[kMaxBuckets];
  __shared__ uint32_t smem[kNW + 1];
  TileInfo ti;
  if (!find_tile(a, blockIdx.x, ti, smem)) return;
  const int nb = 1 << a.top_bits;
  for (int i = threadIdx.x; i < nb; i += kThreads) h[i] = 0;
  __syncthreads();
  const IT* idx = static_cast<const IT*>(a.indices) + ti.start;
  const int shift = top_shift(a, ti.k);
  const uint32_t mask = (uint32_t)nb - 1;
  for (int i = threadIdx.x; i < ti.count; i += kThreads)
    atomicAdd(&h[((uint32_t)idx[i] >> shift) & mask], 1u);
  __syncthreads();
  for (int i = threadIdx.x; i < nb; i += kThreads) a.hist[(size_t)i * a.nt_max + blockIdx.x] = h[i];
  if (blockIdx.x == 0 && threadIdx.x == 0) {  // consumed by later launches of the same call
    *a.over_cnt = 0u;
    *a.list_cnt = 0u;
    for (int k = 0; k < a.K; ++k) a.hot_cnt[k] = 0u;
    for (int i = 0; i < 8; ++i) a.seg_meta[i] = 0u;
  }
}

// --- 2. per-table scan (large batches only): counts -> destination offsets ------------
// One workgroup per table walks (digit, tile) in digit-major order with a running carry
// that starts at the table's slice, so every table is scattered inside its own slice.
// (256 threads: a 1024-thread workgroup is not placed on a compute unit while the forward kernel,
// which runs beside this one, keeps filling every freed slot with its own 256-thread workgroups --
// measured: the scan then only starts when the forward kernel drains)
__global__ __launch_bounds__(kThreads) void bucket_scan_kernel(GroupArgs a) {
  __shared__ uint32_t smem[kThreads / DLRM_WAVE + 1];
  const int k = blockIdx.x;
  // first tile of table k = tiles of all earlier tables
  uint32_t t0 = 0;
  const int64_t tile = (int64_t)1 << a.tile_shift;
  for (int j = 0; j < k; ++j) t0 += (uint32_t)((a.tbl_off[j + 1] - a.tbl_off[j] + tile - 1) >> a.tile_shift);
  const int nt = (int)((a.tbl_off[k + 1] - a.tbl_off[k] + tile - 1) >> a.tile_shift);
  const int nb = 1 << a.top_bits;
  uint32_t carry = (uint32_t)a.tbl_off[k];
  if (nt <= 0) {
    for (int i = threadIdx.x; i < nb; i += kThreads) a.bucket_start[(size_t)k * nb + i] = carry;
    return;
  }
  // kScanItems consecutive entries per thread and round: their loads are in flight together and a
  // round costs one workgroup scan (the kernel shares the machine with the forward pass, where every
  // dependent round trip to memory is several microseconds)
  constexpr int kScanItems = 16;
  const uint32_t n = (uint32_t)nt * (uint32_t)nb;   // < 2^31: nt <= nnz / tile + 1 (<= 1024 + 1 with small tiles), nb <= 1024
  for (uint32_t e0 = 0; e0 < n; e0 += kThreads * kScanItems) {
    uint32_t v[kScanItems], digit[kScanItems], t[kScanItems];
    size_t addr[kScanItems];
    uint32_t sum = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
      const uint32_t e = e0 + threadIdx.x * kScanItems + j;
      v[j] = 0;
      digit[j] = t[j] = 0;
      addr[j] = 0;
      if (e < n) {
        digit[j] = e / (uint32_t)nt;
        t[j] = e - digit[j] * (uint32_t)nt;
        addr[j] = (size_t)digit[j] * a.nt_max + t0 + t[j];
        v[j] = a.hist[addr[j]];
      }
    }
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) sum += v[j];
    uint32_t total;
    uint32_t run = carry + block_exclusive_scan<kThreads>(sum, smem, &total);
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
      const uint32_t e = e0 + threadIdx.x * kScanItems + j;
      if (e < n) {
        a.hist[addr[j]] = run;
        if (t[j] == 0) a.bucket_start[(size_t)k * nb + digit[j]] = run;
        run += v[j];
      }
    }
    carry += total;
  }
  __syncthreads();  // this workgroup's bucket_start writes are visible to it
  for (int dg = threadIdx.x; dg < nb; dg += kThreads) {
    const uint32_t st = a.bucket_start[(size_t)k * nb + dg];
    const uint32_t en = dg + 1 < nb ? a.bucket_start[(size_t)k * nb + dg + 1] : (uint32_t)a.tbl_off[k + 1];
    if (en - st > a.big) a.over_list[atomicAdd(a.list_cnt, 1u)] = (uint32_t)(k * nb + dg);
    if (en - st > (uint32_t)kBktCap) atomicAdd(a.over_cnt, 1u);
  }
}


// --- 3. stable scatter into buckets ---------------------------------------------------
// ITEMS positions per thread: the tile holds kThreads * ITEMS positions (GroupArgs::tile_shift agrees)
template <typename IT, int ITEMS>
__global__ __launch_bounds__(kThreads) void bucket_scatter_kernel(GroupArgs a) {
  constexpr int TILE = kThreads * ITEMS;
  __shared__ uint32_t wcnt[kNW][kMaxBuckets];
  __shared__ uint32_t gofs[kMaxBuckets];
  __shared__ uint32_t skey[TILE];
  __shared__ uint32_t sval[TILE];
  __shared__ uint32_t smem[kNW + 1];
  __shared__ int sflag[1];
  TileInfo ti;
  if (!find_tile(a, blockIdx.x, ti, smem)) return;
  const int nb = 1 << a.top_bits;
  const uint32_t mask = (uint32_t)nb - 1;
  const int lane = lane_id(), w = wave_id();
  const int tid = threadIdx.x;

  // ---- requested first so that their latency hides behind the bag search: the tile's row ids
  // (wave-striped) and, for small batches, this digit's counts in all tiles of the table
  const IT* kin = static_cast<const IT*>(a.indices) + ti.start;
  const int shift = top_shift(a, ti.k);
  uint32_t key[ITEMS], val[ITEMS], dg[ITEMS], rnk[ITEMS];
  bool ok[ITEMS];
#pragma unroll
  for (int j = 0; j < ITEMS; ++j) {
    const int li = w * (DLRM_WAVE * ITEMS) + j * DLRM_WAVE + lane;
    ok[j] = li < ti.count;
    key[j] = ok[j] ? (uint32_t)kin[li] : 0xFFFFFFFFu;
    dg[j] = (key[j] >> shift) & mask;
  }
  // thread t owns the partition digits t*kDPT .. t*kDPT + kDPT-1
  uint32_t goff[kDPT], before[kDPT], total[kDPT];
#pragma unroll
  for (int q = 0; q < kDPT; ++q) {
    const int dgt = tid * kDPT + q;
    goff[q] = before[q] = total[q] = 0;
    if (dgt >= nb) continue;
    if (a.fused_scan) {
      const uint32_t* hrow = a.hist + (size_t)dgt * a.nt_max + ti.t0;
      int t = 0;
      for (; t + 8 <= ti.nt; t += 8) {
        uint32_t c[8];
#pragma unroll
        for (int z = 0; z < 8; ++z) c[z] = hrow[t + z];
#pragma unroll
        for (int z = 0; z < 8; ++z) {
          total[q] += c[z];
          before[q] += t + z < ti.t ? c[z] : 0u;
        }
      }
      for (; t < ti.nt; ++t) {
        const uint32_t c = hrow[t];
        total[q] += c;
        before[q] += t < ti.t ? c : 0u;
      }
    } else {
      goff[q] = a.hist[(size_t)dgt * a.nt_max + blockIdx.x];
    }
  }

  // ---- bag of every position of the tile, from the offsets
  // b0 = the bag holding the tile's first position: last b with off[b] <= P0.
  const int64_t* off = a.offsets + (int64_t)ti.k * (a.B + 1);
  const int64_t P0 = ti.start - ti.tbl_start;
  int lo = 0, hi = a.B;  // off[lo] <= P0 (off[0] = 0); the answer lies in [lo, hi)
  while (hi - lo > 1) {   // 256-ary search, uniform
    const int step = (hi - lo + kThreads - 1) / kThreads;
    const int q = lo + (tid + 1) * step;
    const int pred = (q < hi && off[q] <= P0) ? 1 : 0;
    const int cnt = __syncthreads_count(pred);   // offsets are monotone: the first cnt probes pass
    const int nlo = lo + cnt * step;
    const int nhi = nlo + step < hi ? nlo + step : hi;
    lo = nlo;
    hi = nhi;
  }
  const int b0 = lo;
  for (int i = tid; i < TILE; i += kThreads) skey[i] = 0;  // skey doubles as the bag-start counters
  for (int i = tid; i < kNW * kMaxBuckets; i += kThreads) (&wcnt[0][0])[i] = 0;
  __syncthreads();
  for (int base = b0 + 1;; base += kThreads) {  // bags that start inside the tile (after P0)
    const int b = base + tid;
    if (tid == 0) sflag[0] = (b >= a.B || off[b] >= P0 + ti.count) ? 1 : 0;
    if (b < a.B) {
      const int64_t ob = off[b];
      if (ob < P0 + ti.count) atomicAdd(&skey[(int)(ob - P0)], 1u);
    }
    __syncthreads();
    const int done = sflag[0];
    __syncthreads();
    // monotone offsets: once this round's first bag starts past the tile, every later one does;
    // a round whose first bag is inside may still have later bags inside, so go on
    if (done) break;
  }
  {  // inclusive prefix of the start counters, thread t owning positions [t*ITEMS, (t+1)*ITEMS)
    uint32_t c[ITEMS], s = 0;
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
      c[j] = skey[tid * ITEMS + j];
      s += c[j];
    }
    uint32_t total;
    uint32_t run = block_exclusive_scan<kThreads>(s, smem, &total);
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
      run += c[j];
      sval[tid * ITEMS + j] = (uint32_t)b0 + run;
    }
  }
  __syncthreads();

  // ---- bags of this thread's (wave-striped) positions, then rank by partition digit
#pragma unroll
  for (int j = 0; j < ITEMS; ++j) {
    const int li = w * (DLRM_WAVE * ITEMS) + j * DLRM_WAVE + lane;
    val[j] = ok[j] ? sval[li] : 0u;
    if (a.weights != nullptr && ok[j]) {  // uniform branch: weighted batch
      PosEntry pe;
      pe.bag = val[j];
      pe.w = a.weights[ti.start + li];
      a.pos_entry[ti.start + li] = pe;
      val[j] = (uint32_t)(P0 + li);       // position inside the table
    }
  }
  rank_items<ITEMS, kMaxBuckets>(dg, ok, a.top_bits, wcnt, rnk);
  __syncthreads();

  // ---- destination offsets of this tile's digits
  if (a.fused_scan) {
    // few tiles: the raw counts of the table's tiles were summed above instead of a separate scan
    uint32_t sum = 0, all;
#pragma unroll
    for (int q = 0; q < kDPT; ++q) sum += total[q];
    uint32_t base = block_exclusive_scan<kThreads>(sum, smem, &all);
#pragma unroll
    for (int q = 0; q < kDPT; ++q) {
      const int dgt = tid * kDPT + q;
      goff[q] = (uint32_t)ti.tbl_start + base + before[q];
      if (ti.t == 0 && dgt < nb) {
        a.bucket_start[(size_t)ti.k * nb + dgt] = (uint32_t)ti.tbl_start + base;
        if (total[q] > a.big) a.over_list[atomicAdd(a.list_cnt, 1u)] = (uint32_t)(ti.k * nb + dgt);
        if (total[q] > (uint32_t)kBktCap) atomicAdd(a.over_cnt, 1u);
      }
      base += total[q];
    }
  }
  uint32_t lofs[kDPT], tot[kDPT];
  digit_offsets<kMaxBuckets>(nb, wcnt, smem, lofs, tot);
#pragma unroll
  for (int q = 0; q < kDPT; ++q) {
    const int dgt = tid * kDPT + q;
    if (dgt < nb) gofs[dgt] = goff[q] - lofs[q];
  }
  __syncthreads();

  // ---- stage in LDS in sorted order so that one digit's global writes are contiguous
#pragma unroll
  for (int j = 0; j < ITEMS; ++j) {
    if (ok[j]) {
      const uint32_t lp = wcnt[w][dg[j]] + rnk[j];
      skey[lp] = key[j];
      sval[lp] = val[j];
    }
  }
  __syncthreads();
  uint32_t* kout = a.keys[1];
  uint32_t* vout = a.vals[1];
  for (int lp = tid; lp < ti.count; lp += kThreads) {
    const uint32_t kk = skey[lp];
    const uint32_t dst = gofs[(kk >> shift) & mask] + (uint32_t)lp;
    kout[dst] = kk;
    vout[dst] = sval[lp];
  }
}


int enqueue_partition(const dlrm_sparse_batch* s, const GroupArgs& g, hipStream_t st) {
  if (g.idx32)
    hipLaunchKernelGGL(bucket_hist_kernel<int32_t>, dim3(g.nt_max), dim3(kThreads), 0, st, g);
  else
    hipLaunchKernelGGL(bucket_hist_kernel<int64_t>, dim3(g.nt_max), dim3(kThreads), 0, st, g);
  DLRM_CHECK_LAUNCH();
  if (!g.fused_scan) {
    hipLaunchKernelGGL(bucket_scan_kernel, dim3(s->K), dim3(kThreads), 0, st, g);
    DLRM_CHECK_LAUNCH();
  }
  const bool small = g.tile_shift == 10;
  if (g.idx32) {
    if (small)
      hipLaunchKernelGGL((bucket_scatter_kernel<int32_t, kSmallItems>), dim3(g.nt_max), dim3(kThreads), 0, st, g);
    else
      hipLaunchKernelGGL((bucket_scatter_kernel<int32_t, kItems>), dim3(g.nt_max), dim3(kThreads), 0, st, g);
  } else {
    if (small)
      hipLaunchKernelGGL((bucket_scatter_kernel<int64_t, kSmallItems>), dim3(g.nt_max), dim3(kThreads), 0, st, g);
    else
      hipLaunchKernelGGL((bucket_scatter_kernel<int64_t, kItems>), dim3(g.nt_max), dim3(kThreads), 0, st, g);
  }
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}

}  // namespace dlrm
