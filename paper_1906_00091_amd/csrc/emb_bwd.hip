// Embedding backward fused with the sparse SGD row update (transpose of Eq. (2);
// SGD of Sec. 5.1):  for every distinct row r looked up in table k,
//   g = sum_{p : idx_k[p] = r} dS[bag(p), k, :],   W_k[r,:] <- W_k[r,:] - lr * g.
//
// SORT path (deterministic, any table dtype):
//   1. expand      : (row, bag) pair for every lookup position
//   2. radix sort  : least-significant-digit passes over the row id, per table
//                    (tiles never straddle two tables, so every table is sorted
//                    inside its own slice); each pass = tile histograms, a scan
//                    per table, and a stable scatter staged through LDS
//   3. run heads   : positions where the row changes -> one segment per distinct row
//   4. reduce+SGD  : a lane group per segment sums its dS rows in ascending
//                    position order (fp32) and read-modify-writes the table row once
// ATOMIC path (fp32 tables): a lane group per bag adds -lr*dS[b,k,:] to every row
// of the bag with hardware fp32 atomics; no workspace, one launch.
#include "common.h"

namespace dlrm {

constexpr int kTileThreads = 256;
constexpr int kItems = 16;                       // items per thread in a sort tile
constexpr int kTile = kTileThreads * kItems;     // 4096 positions per tile
constexpr int kMaxDigitBits = 8;
constexpr int kMaxBuckets = 1 << kMaxDigitBits;

// ---------------------------------------------------------------------------
// Workspace layout (all offsets 256-byte aligned)
struct WsLayout {
  size_t keys[2], vals[2];   // uint32[nnz] ping-pong: row ids / bag ids
  size_t tile_prefix;        // int32[K+1]: first tile of every table
  size_t hist;               // uint32[kMaxBuckets * nt_max]: per-tile digit counts, then offsets
  size_t tile_heads;         // uint32[nt_max + 1]: run heads per tile, then exclusive prefix
  size_t seg_start;          // uint32[nnz + 1]: position of every run head (+ sentinel)
  size_t seg_tbl;            // uint32[nnz]: table of every run
  size_t n_seg;              // uint32[4]: total number of runs
  size_t total;
  int64_t nt_max;            // upper bound on the number of tiles
};

static inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

static WsLayout ws_layout(int32_t K, int64_t nnz) {
  WsLayout L;
  size_t o = 0;
  const size_t n = (size_t)(nnz > 0 ? nnz : 1);
  L.nt_max = nnz / kTile + K;
  for (int i = 0; i < 2; ++i) { L.keys[i] = o; o = align256(o + n * 4); }
  for (int i = 0; i < 2; ++i) { L.vals[i] = o; o = align256(o + n * 4); }
  L.tile_prefix = o; o = align256(o + (size_t)(K + 1) * 4);
  L.hist = o;        o = align256(o + (size_t)kMaxBuckets * (size_t)L.nt_max * 4);
  L.tile_heads = o;  o = align256(o + (size_t)(L.nt_max + 1) * 4);
  L.seg_start = o;   o = align256(o + (n + 1) * 4);
  L.seg_tbl = o;     o = align256(o + n * 4);
  L.n_seg = o;       o = align256(o + 16);
  L.total = o;
  return L;
}

// ---------------------------------------------------------------------------
struct GroupArgs {            // everything the grouping kernels need
  const int64_t* indices;
  const int64_t* offsets;
  const int64_t* tbl_off;
  int32_t K, B;
  int32_t nt_max;
  uint32_t* keys[2];
  uint32_t* vals[2];
  int32_t* tile_prefix;
  uint32_t* hist;
  uint32_t* tile_heads;
  uint32_t* seg_start;
  uint32_t* seg_tbl;
  uint32_t* n_seg;
};

// Which table and which positions a tile covers.  Wave-uniform.
struct TileInfo {
  int k;
  int64_t start;   // global position of the tile's first item
  int count;       // items in the tile (1..kTile)
  int64_t tbl_start;
};

__device__ inline bool find_tile(const GroupArgs& a, int tile, TileInfo& ti) {
  if (tile >= a.tile_prefix[a.K]) return false;
  int lo = 0, hi = a.K;  // tile_prefix[lo] <= tile < tile_prefix[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (a.tile_prefix[mid] <= tile) lo = mid; else hi = mid;
  }
  // tables without lookups own no tiles: tile_prefix[lo] == tile_prefix[lo+1] is skipped by
  // the search because it keeps the LAST k with tile_prefix[k] <= tile
  ti.k = lo;
  ti.tbl_start = a.tbl_off[lo];
  const int64_t tbl_end = a.tbl_off[lo + 1];
  ti.start = ti.tbl_start + (int64_t)(tile - a.tile_prefix[lo]) * kTile;
  const int64_t rem = tbl_end - ti.start;
  ti.count = (int)(rem < kTile ? rem : kTile);
  return ti.count > 0;
}

// --- 0. tile map -------------------------------------------------------------
__global__ __launch_bounds__(256) void tile_map_kernel(GroupArgs a) {
  __shared__ uint32_t smem[256 / DLRM_WAVE + 1];
  uint32_t carry = 0;
  if (threadIdx.x == 0) a.tile_prefix[0] = 0;
  for (int k0 = 0; k0 < a.K; k0 += 256) {
    const int k = k0 + threadIdx.x;
    uint32_t nt = 0;
    if (k < a.K) nt = (uint32_t)((a.tbl_off[k + 1] - a.tbl_off[k] + kTile - 1) / kTile);
    uint32_t total;
    const uint32_t ex = block_exclusive_scan<256>(nt, smem, &total);
    if (k < a.K) a.tile_prefix[k + 1] = (int32_t)(carry + ex + nt);
    carry += total;
  }
}

// --- 1. expand ----------------------------------------------------------------
// 2^lg lanes per bag walk the bag's positions; writes the 32-bit row id and the bag id.
__global__ __launch_bounds__(256) void expand_kernel(GroupArgs a, int lg) {
  const int64_t gid = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> lg;
  const int sub = threadIdx.x & ((1 << lg) - 1);
  if (gid >= (int64_t)a.K * a.B) return;
  const int k = (int)(gid / a.B), b = (int)(gid - (int64_t)k * a.B);
  const int64_t* off = a.offsets + (int64_t)k * (a.B + 1);
  const int64_t base = a.tbl_off[k];
  const int64_t p1 = base + off[b + 1];
  for (int64_t p = base + off[b] + sub; p < p1; p += (1 << lg)) {
    a.keys[0][p] = (uint32_t)a.indices[p];
    a.vals[0][p] = (uint32_t)b;
  }
}

// --- 2a. per-tile digit histogram ----------------------------------------------
__global__ __launch_bounds__(kTileThreads) void sort_hist_kernel(GroupArgs a, int src, int shift,
                                                                  int bits) {
  __shared__ uint32_t h[kMaxBuckets];
  TileInfo ti;
  if (!find_tile(a, blockIdx.x, ti)) return;
  const int nb = 1 << bits;
  for (int i = threadIdx.x; i < nb; i += kTileThreads) h[i] = 0;
  __syncthreads();
  const uint32_t* keys = a.keys[src] + ti.start;
  const uint32_t mask = (uint32_t)nb - 1;
  for (int i = threadIdx.x; i < ti.count; i += kTileThreads)
    atomicAdd(&h[(keys[i] >> shift) & mask], 1u);
  __syncthreads();
  for (int i = threadIdx.x; i < nb; i += kTileThreads)
    a.hist[(size_t)i * a.nt_max + blockIdx.x] = h[i];
}

// --- 2b. per-table scan: counts -> destination offsets ---------------------------
// One workgroup per table walks (digit, tile) in digit-major order with a running carry
// that starts at the table's slice, so every table is scattered inside its own slice.
__global__ __launch_bounds__(1024) void sort_scan_kernel(GroupArgs a, int bits) {
  __shared__ uint32_t smem[1024 / DLRM_WAVE + 1];
  const int k = blockIdx.x;
  const int t0 = a.tile_prefix[k], nt = a.tile_prefix[k + 1] - t0;
  if (nt <= 0) return;
  const int64_t n = (int64_t)nt << bits;
  uint32_t carry = (uint32_t)a.tbl_off[k];
  for (int64_t e0 = 0; e0 < n; e0 += 1024) {
    const int64_t e = e0 + threadIdx.x;
    uint32_t v = 0;
    size_t addr = 0;
    if (e < n) {
      const int digit = (int)(e / nt), t = (int)(e - (int64_t)digit * nt);
      addr = (size_t)digit * a.nt_max + t0 + t;
      v = a.hist[addr];
    }
    uint32_t total;
    const uint32_t ex = block_exclusive_scan<1024>(v, smem, &total);
    if (e < n) a.hist[addr] = carry + ex;
    carry += total;
  }
}

// --- 2c. stable scatter ---------------------------------------------------------
// Wave w of the workgroup owns the contiguous positions [w*64*kItems, (w+1)*64*kItems)
// of the tile, item j of lane l being position w*64*kItems + j*64 + l.  Ranks inside a
// wave come from ballot matching; per-wave digit counters in LDS give the order across
// waves.  Items are first placed in LDS in sorted order so that the global writes of
// one digit are contiguous.
__global__ __launch_bounds__(kTileThreads) void sort_scatter_kernel(GroupArgs a, int src, int shift,
                                                                     int bits) {
  constexpr int NW = kTileThreads / DLRM_WAVE;
  __shared__ uint32_t wcnt[NW][kMaxBuckets];
  __shared__ uint32_t gofs[kMaxBuckets];
  __shared__ uint32_t skey[kTile];
  __shared__ uint32_t sval[kTile];
  __shared__ uint32_t scan_smem[kTileThreads / DLRM_WAVE + 1];
  TileInfo ti;
  if (!find_tile(a, blockIdx.x, ti)) return;
  const int nb = 1 << bits;
  const uint32_t mask = (uint32_t)nb - 1;
  const int lane = lane_id(), w = wave_id();
  for (int i = threadIdx.x; i < NW * kMaxBuckets; i += kTileThreads) (&wcnt[0][0])[i] = 0;
  __syncthreads();

  const uint32_t* kin = a.keys[src] + ti.start;
  const uint32_t* vin = a.vals[src] + ti.start;
  uint32_t key[kItems], val[kItems], rnk[kItems];
#pragma unroll
  for (int j = 0; j < kItems; ++j) {
    const int li = w * (DLRM_WAVE * kItems) + j * DLRM_WAVE + lane;
    const bool ok = li < ti.count;
    key[j] = ok ? kin[li] : 0xFFFFFFFFu;
    val[j] = ok ? vin[li] : 0u;
  }
  const unsigned long long lt = (1ull << lane) - 1ull;
#pragma unroll
  for (int j = 0; j < kItems; ++j) {
    const int li = w * (DLRM_WAVE * kItems) + j * DLRM_WAVE + lane;
    const bool ok = li < ti.count;
    const uint32_t dg = (key[j] >> shift) & mask;
    unsigned long long m = __ballot(ok);
    for (int bit = 0; bit < bits; ++bit) {
      const bool one = (dg >> bit) & 1u;
      const unsigned long long bal = __ballot(one);
      m &= one ? bal : ~bal;
    }
    // m: valid lanes of this wave holding the same digit in item j (meaningful where ok)
    uint32_t prev = 0;
    const int leader = ok ? (__ffsll((long long)m) - 1) : lane;
    if (ok && lane == leader) prev = atomicAdd(&wcnt[w][dg], (uint32_t)__popcll(m));
    prev = __shfl(prev, leader, DLRM_WAVE);
    rnk[j] = prev + (uint32_t)__popcll(m & lt);
  }
  __syncthreads();
  // per digit: totals, exclusive prefix over waves, exclusive prefix over digits
  {
    uint32_t c[NW], tot = 0;
    const int dg = threadIdx.x;  // kTileThreads >= kMaxBuckets
#pragma unroll
    for (int i = 0; i < NW; ++i) {
      c[i] = dg < nb ? wcnt[i][dg] : 0u;
      tot += c[i];
    }
    uint32_t total_all;
    const uint32_t lofs = block_exclusive_scan<kTileThreads>(tot, scan_smem, &total_all);
    if (dg < nb) {
      uint32_t run = lofs;
#pragma unroll
      for (int i = 0; i < NW; ++i) {
        wcnt[i][dg] = run;  // local sorted position of wave i's first item with this digit
        run += c[i];
      }
      gofs[dg] = a.hist[(size_t)dg * a.nt_max + blockIdx.x] - lofs;
    }
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < kItems; ++j) {
    const int li = w * (DLRM_WAVE * kItems) + j * DLRM_WAVE + lane;
    if (li < ti.count) {
      const uint32_t dg = (key[j] >> shift) & mask;
      const uint32_t lp = wcnt[w][dg] + rnk[j];
      skey[lp] = key[j];
      sval[lp] = val[j];
    }
  }
  __syncthreads();
  uint32_t* kout = a.keys[src ^ 1];
  uint32_t* vout = a.vals[src ^ 1];
  for (int lp = threadIdx.x; lp < ti.count; lp += kTileThreads) {
    const uint32_t kk = skey[lp];
    const uint32_t dst = gofs[(kk >> shift) & mask] + (uint32_t)lp;
    kout[dst] = kk;
    vout[dst] = sval[lp];
  }
}

// --- 3. run heads ----------------------------------------------------------------
__device__ inline bool is_head(const uint32_t* keys, int64_t pos, int64_t tbl_start) {
  return pos == tbl_start || keys[pos] != keys[pos - 1];
}

__global__ __launch_bounds__(kTileThreads) void heads_count_kernel(GroupArgs a, int src) {
  __shared__ uint32_t smem[kTileThreads / DLRM_WAVE + 1];
  TileInfo ti;
  uint32_t cnt = 0;
  const bool live = find_tile(a, blockIdx.x, ti);
  if (live) {
    const uint32_t* keys = a.keys[src];
    for (int i = threadIdx.x; i < ti.count; i += kTileThreads)
      cnt += is_head(keys, ti.start + i, ti.tbl_start) ? 1u : 0u;
  }
  uint32_t total;
  block_exclusive_scan<kTileThreads>(cnt, smem, &total);
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

__global__ __launch_bounds__(kTileThreads) void heads_write_kernel(GroupArgs a, int src) {
  __shared__ uint32_t smem[kTileThreads / DLRM_WAVE + 1];
  TileInfo ti;
  if (!find_tile(a, blockIdx.x, ti)) return;
  const uint32_t* keys = a.keys[src];
  uint32_t base = a.tile_heads[blockIdx.x];
  // thread t owns the contiguous positions [t*kItems, (t+1)*kItems) so that heads keep their order
  uint32_t flags = 0, cnt = 0;
#pragma unroll
  for (int j = 0; j < kItems; ++j) {
    const int li = threadIdx.x * kItems + j;
    if (li < ti.count && is_head(keys, ti.start + li, ti.tbl_start)) {
      flags |= 1u << j;
      ++cnt;
    }
  }
  uint32_t total;
  uint32_t pos = base + block_exclusive_scan<kTileThreads>(cnt, smem, &total);
#pragma unroll
  for (int j = 0; j < kItems; ++j) {
    if (flags & (1u << j)) {
      a.seg_start[pos] = (uint32_t)(ti.start + threadIdx.x * kItems + j);
      a.seg_tbl[pos] = (uint32_t)ti.k;
      ++pos;
    }
  }
}

// --- 4. segment reduce + SGD row update ---------------------------------------------
struct UpdArgs {
  void* const* tables;
  const float* dS;
  int64_t stride_b, stride_k;
  float lr;
  int32_t d;
  const uint32_t* keys;     // sorted row ids
  const uint32_t* bags;     // sorted bag ids
  const uint32_t* seg_start;
  const uint32_t* seg_tbl;
  const uint32_t* n_seg;
};

// G lanes per segment, each lane owns 4 consecutive columns (16 bytes of fp32 gradient).
template <int DT, int G, int U>
__global__ __launch_bounds__(256) void reduce_update_kernel(UpdArgs a) {
  constexpr int S = DLRM_WAVE / G;
  const int lane = lane_id();
  const int slot = lane / G, chunk = lane % G;
  const bool col_ok = chunk * 4 < a.d;
  const uint32_t nseg = a.n_seg[0];
  const uint32_t ngroups = gridDim.x * (blockDim.x >> 6) * S;
  for (uint32_t u = (blockIdx.x * (blockDim.x >> 6) + wave_id()) * S + slot; u < nseg; u += ngroups) {
    const uint32_t i0 = a.seg_start[u], i1 = a.seg_start[u + 1];
    const uint32_t k = a.seg_tbl[u];
    // lanes past the last column shadow column group 0 (same addresses) and never write
    const float* g = a.dS + (int64_t)k * a.stride_k + (col_ok ? chunk : 0) * 4;
    f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
    for (uint32_t i = i0; i < i1; i += U) {
      // branch-free: U bag ids, then U gradient rows, in flight together; the tail re-reads
      // the run's last entry and is dropped
      uint32_t bg[U];
      f32x4 v[U];
#pragma unroll
      for (int t = 0; t < U; ++t) bg[t] = a.bags[i + t < i1 ? i + t : i1 - 1];
#pragma unroll
      for (int t = 0; t < U; ++t) v[t] = loadf4(g + (int64_t)bg[t] * a.stride_b);
#pragma unroll
      for (int t = 0; t < U; ++t) {
        const float m = i + t < i1 ? 1.0f : 0.0f;
        if (m != 0.0f) acc += v[t];
      }
    }
    if (!col_ok) continue;
    const int64_t r = a.keys[i0];
    char* W = static_cast<char*>(a.tables[k]);
    if constexpr (DT == DLRM_F32) {
      float* w = reinterpret_cast<float*>(W) + r * a.d + chunk * 4;
      f32x4 x = loadf4(w);
      x.x = fmaf(-a.lr, acc.x, x.x);
      x.y = fmaf(-a.lr, acc.y, x.y);
      x.z = fmaf(-a.lr, acc.z, x.z);
      x.w = fmaf(-a.lr, acc.w, x.w);
      storef4(w, x);
    } else {
      u32x2* w = reinterpret_cast<u32x2*>(W + (r * a.d + chunk * 4) * 2);
      u32x2 bits = *w;
      float x0, x1, x2, x3;
      if constexpr (DT == DLRM_F16) {
        half2_to_float2(bits.x, x0, x1);
        half2_to_float2(bits.y, x2, x3);
      } else {
        bf162_to_float2(bits.x, x0, x1);
        bf162_to_float2(bits.y, x2, x3);
      }
      x0 = fmaf(-a.lr, acc.x, x0);
      x1 = fmaf(-a.lr, acc.y, x1);
      x2 = fmaf(-a.lr, acc.z, x2);
      x3 = fmaf(-a.lr, acc.w, x3);
      if constexpr (DT == DLRM_F16) {
        bits.x = float2_to_half2(x0, x1);
        bits.y = float2_to_half2(x2, x3);
      } else {
        bits.x = float2_to_bf162(x0, x1);
        bits.y = float2_to_bf162(x2, x3);
      }
      *w = bits;
    }
  }
}

// --- ATOMIC path --------------------------------------------------------------------
struct AtomArgs {
  void* const* tables;
  const int64_t* indices;
  const int64_t* offsets;
  const int64_t* tbl_off;
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
  const int64_t bag = ((int64_t)blockIdx.x * (blockDim.x >> 6) + wave_id()) * S + slot;
  if (bag >= (int64_t)a.K * a.B || chunk * 4 >= a.d) return;
  const int k = (int)(bag / a.B), b = (int)(bag - (int64_t)k * a.B);
  const int64_t* off = a.offsets + (int64_t)k * (a.B + 1);
  const int64_t p0 = off[b], p1 = off[b + 1];
  if (p1 <= p0) return;
  const int64_t* idx = a.indices + a.tbl_off[k];
  float* W = static_cast<float*>(a.tables[k]) + chunk * 4;
  f32x4 g = loadf4(a.dS + (int64_t)b * a.stride_b + (int64_t)k * a.stride_k + chunk * 4);
  g *= -a.lr;
  for (int64_t p = p0; p < p1; ++p) {
    float* w = W + idx[p] * a.d;
    unsafeAtomicAdd(w + 0, g.x);
    unsafeAtomicAdd(w + 1, g.y);
    unsafeAtomicAdd(w + 2, g.z);
    unsafeAtomicAdd(w + 3, g.w);
  }
}

// --- export (debug / parity) ---------------------------------------------------------
struct ExportArgs {
  int64_t* uniq_rows;
  int64_t* seg_start_out;
  int32_t* sorted_bag;
  int64_t* n_uniq;
  int64_t nnz;
};

__global__ __launch_bounds__(256) void export_kernel(GroupArgs a, int src, ExportArgs e) {
  const uint32_t nseg = a.n_seg[0];
  const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t nth = (int64_t)gridDim.x * blockDim.x;
  for (int64_t p = tid; p < e.nnz; p += nth) e.sorted_bag[p] = (int32_t)a.vals[src][p];
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
    e.uniq_rows[tstart + local_u] = (int64_t)a.keys[src][pos];
    e.seg_start_out[tstart + local_u] = (int64_t)pos - tstart;
    const bool last_of_table = (u + 1 == nseg) || a.seg_tbl[u + 1] != k;
    if (last_of_table) e.n_uniq[k] = local_u + 1;
  }
}

__global__ void zero_i64_kernel(int64_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

// ---------------------------------------------------------------------------
int check_batch(const dlrm_sparse_batch* s);  // util.hip

static void fill_group_args(GroupArgs& g, const dlrm_sparse_batch* s, const WsLayout& L, void* ws) {
  char* base = static_cast<char*>(ws);
  g.indices = s->indices;
  g.offsets = s->offsets;
  g.tbl_off = s->tbl_off;
  g.K = s->K;
  g.B = s->B;
  g.nt_max = (int32_t)L.nt_max;
  for (int i = 0; i < 2; ++i) {
    g.keys[i] = reinterpret_cast<uint32_t*>(base + L.keys[i]);
    g.vals[i] = reinterpret_cast<uint32_t*>(base + L.vals[i]);
  }
  g.tile_prefix = reinterpret_cast<int32_t*>(base + L.tile_prefix);
  g.hist = reinterpret_cast<uint32_t*>(base + L.hist);
  g.tile_heads = reinterpret_cast<uint32_t*>(base + L.tile_heads);
  g.seg_start = reinterpret_cast<uint32_t*>(base + L.seg_start);
  g.seg_tbl = reinterpret_cast<uint32_t*>(base + L.seg_tbl);
  g.n_seg = reinterpret_cast<uint32_t*>(base + L.n_seg);
}

// Enqueues stages 1-3; *final_src receives the index of the ping-pong buffer holding the
// sorted pairs.
static int enqueue_grouping(const dlrm_sparse_batch* s, const GroupArgs& g, int* final_src,
                            hipStream_t st) {
  const int64_t bags = (int64_t)s->K * s->B;
  hipLaunchKernelGGL(tile_map_kernel, dim3(1), dim3(256), 0, st, g);
  DLRM_CHECK_LAUNCH();
  {
    const double mean_len = (double)s->nnz_total / (double)bags;
    int lg = 0;
    while (lg < 6 && (double)(1 << (lg + 1)) <= mean_len) ++lg;
    hipLaunchKernelGGL(expand_kernel, dim3(div_up(bags << lg, 256)), dim3(256), 0, st, g, lg);
    DLRM_CHECK_LAUNCH();
  }
  const int key_bits = ilog2_ceil(s->max_rows) > 0 ? ilog2_ceil(s->max_rows) : 1;
  const int passes = (key_bits + kMaxDigitBits - 1) / kMaxDigitBits;
  int src = 0, shift = 0;
  for (int p = 0; p < passes; ++p) {
    const int left = key_bits - shift;
    const int bits = (left + (passes - p) - 1) / (passes - p);
    hipLaunchKernelGGL(sort_hist_kernel, dim3(g.nt_max), dim3(kTileThreads), 0, st, g, src, shift, bits);
    DLRM_CHECK_LAUNCH();
    hipLaunchKernelGGL(sort_scan_kernel, dim3(s->K), dim3(1024), 0, st, g, bits);
    DLRM_CHECK_LAUNCH();
    hipLaunchKernelGGL(sort_scatter_kernel, dim3(g.nt_max), dim3(kTileThreads), 0, st, g, src, shift, bits);
    DLRM_CHECK_LAUNCH();
    src ^= 1;
    shift += bits;
  }
  hipLaunchKernelGGL(heads_count_kernel, dim3(g.nt_max), dim3(kTileThreads), 0, st, g, src);
  DLRM_CHECK_LAUNCH();
  hipLaunchKernelGGL(heads_scan_kernel, dim3(1), dim3(1024), 0, st, g, s->nnz_total);
  DLRM_CHECK_LAUNCH();
  hipLaunchKernelGGL(heads_write_kernel, dim3(g.nt_max), dim3(kTileThreads), 0, st, g, src);
  DLRM_CHECK_LAUNCH();
  *final_src = src;
  return DLRM_OK;
}

template <int DT, int G>
static int launch_update(const UpdArgs& u, int64_t nnz, hipStream_t st) {
  constexpr int S = DLRM_WAVE / G;
  // persistent grid: enough lane groups to cover the machine several times over, never more
  // than one group per possible segment
  int64_t blocks = (nnz + 4 * S - 1) / (4 * S);
  if (blocks > 256 * 16) blocks = 256 * 16;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL((reduce_update_kernel<DT, G, 4>), dim3((unsigned)blocks), dim3(256), 0, st, u);
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}

template <int DT>
static int dispatch_update(const UpdArgs& u, int G, int64_t nnz, hipStream_t st) {
  switch (G) {
    case 1: return launch_update<DT, 1>(u, nnz, st);
    case 2: return launch_update<DT, 2>(u, nnz, st);
    case 4: return launch_update<DT, 4>(u, nnz, st);
    case 8: return launch_update<DT, 8>(u, nnz, st);
    case 16: return launch_update<DT, 16>(u, nnz, st);
    case 32: return launch_update<DT, 32>(u, nnz, st);
    case 64: return launch_update<DT, 64>(u, nnz, st);
  }
  return DLRM_ERR_BAD_SHAPE;
}

template <int G>
static int launch_atomic(const AtomArgs& a, hipStream_t st) {
  constexpr int S = DLRM_WAVE / G;
  hipLaunchKernelGGL((atomic_update_kernel<G>), dim3(div_up((int64_t)a.K * a.B, 4 * S)), dim3(256), 0,
                     st, a);
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}

static int check_ws(const dlrm_sparse_batch* s, void* ws, size_t bytes, WsLayout* L) {
  *L = ws_layout(s->K, s->nnz_total);
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255) || bytes < L->total) return DLRM_ERR_WORKSPACE;
  if (L->nt_max > 0x7FFFFFFF) return DLRM_ERR_BAD_SHAPE;
  return DLRM_OK;
}

}  // namespace dlrm

using namespace dlrm;

extern "C" size_t dlrm_emb_bag_bwd_workspace_bytes(int32_t K, int32_t B, int32_t d, int64_t nnz_total,
                                                   int64_t max_rows, int32_t table_dtype) {
  if (K < 1 || B < 1 || d < 1 || nnz_total < 0 || nnz_total > DLRM_MAX_NNZ || max_rows < 1 ||
      max_rows > DLRM_MAX_ROWS || !dtype_ok(table_dtype))
    return 0;
  return ws_layout(K, nnz_total).total;
}

extern "C" int32_t dlrm_emb_bag_bwd_sgd(const dlrm_sparse_batch* s, const float* dS, int64_t stride_b,
                                        int64_t stride_k, float lr, void* workspace,
                                        size_t workspace_bytes, int32_t algo, void* stream) {
  int st = check_batch(s);
  if (st != DLRM_OK) return st;
  if (!dS) return DLRM_ERR_NULL;
  if ((s->d & 3) || stride_k < s->d || (stride_k & 3) || (stride_b & 3) || stride_b < 0)
    return DLRM_ERR_BAD_SHAPE;
  if (reinterpret_cast<uintptr_t>(dS) & 15) return DLRM_ERR_BAD_SHAPE;
  if (algo != DLRM_BWD_AUTO && algo != DLRM_BWD_SORT && algo != DLRM_BWD_ATOMIC) return DLRM_ERR_BAD_ALGO;
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
    a.offsets = s->offsets;
    a.tbl_off = s->tbl_off;
    a.dS = dS;
    a.stride_b = stride_b;
    a.stride_k = stride_k;
    a.lr = lr;
    a.K = s->K;
    a.B = s->B;
    a.d = s->d;
    switch (G) {
      case 1: return launch_atomic<1>(a, hs);
      case 2: return launch_atomic<2>(a, hs);
      case 4: return launch_atomic<4>(a, hs);
      case 8: return launch_atomic<8>(a, hs);
      case 16: return launch_atomic<16>(a, hs);
      case 32: return launch_atomic<32>(a, hs);
      case 64: return launch_atomic<64>(a, hs);
    }
    return DLRM_ERR_BAD_SHAPE;
  }

  WsLayout L;
  st = check_ws(s, workspace, workspace_bytes, &L);
  if (st != DLRM_OK) return st;
  if (s->nnz_total == 0) return DLRM_OK;
  GroupArgs g;
  fill_group_args(g, s, L, workspace);
  int src = 0;
  st = enqueue_grouping(s, g, &src, hs);
  if (st != DLRM_OK) return st;
  UpdArgs u;
  u.tables = s->tables;
  u.dS = dS;
  u.stride_b = stride_b;
  u.stride_k = stride_k;
  u.lr = lr;
  u.d = s->d;
  u.keys = g.keys[src];
  u.bags = g.vals[src];
  u.seg_start = g.seg_start;
  u.seg_tbl = g.seg_tbl;
  u.n_seg = g.n_seg;
  switch (s->table_dtype) {
    case DLRM_F32: return dispatch_update<DLRM_F32>(u, G, s->nnz_total, hs);
    case DLRM_F16: return dispatch_update<DLRM_F16>(u, G, s->nnz_total, hs);
    case DLRM_BF16: return dispatch_update<DLRM_BF16>(u, G, s->nnz_total, hs);
  }
  return DLRM_ERR_BAD_DTYPE;
}

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
  int src = 0;
  st = enqueue_grouping(s, g, &src, hs);
  if (st != DLRM_OK) return st;
  ExportArgs e;
  e.uniq_rows = uniq_rows;
  e.seg_start_out = seg_start;
  e.sorted_bag = sorted_bag;
  e.n_uniq = n_uniq;
  e.nnz = s->nnz_total;
  unsigned grid = div_up(s->nnz_total, 256);
  if (grid > 2048) grid = 2048;
  hipLaunchKernelGGL(export_kernel, dim3(grid), dim3(256), 0, hs, g, src, e);
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}
