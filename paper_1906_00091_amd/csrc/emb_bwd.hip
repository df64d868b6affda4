// Embedding backward fused with the sparse SGD row update (transpose of Eq. (2);
// SGD of Sec. 5.1):  for every distinct row r looked up in table k,
//   g = sum_{p : idx_k[p] = r} dS[bag(p), k, :],   W_k[r,:] <- W_k[r,:] - lr * g.
//
// SORT path (deterministic, any table dtype) -- a most-significant-digit partition
// followed by a bucket-local sort, so that one workgroup owns all lookups of a row:
//   1. bucket_hist    : per 4096-position tile, histogram of the top digit of the row id
//                       (tiles never straddle two tables)
//   2. scan           : (digit, tile) counts -> destination offsets inside the table's slice
//                       (folded into step 3 when the batch has few tiles)
//   3. bucket_scatter : derives the bag of every position from the offsets, then moves the
//                       (row, bag) pairs to their bucket, stably, staged through LDS
//   4. bucket_reduce  : one workgroup per (table, top digit): stable LSD radix sort of the
//                       bucket on the remaining low bits (in LDS when it fits), run heads,
//                       then a lane group per run sums its dS rows in ascending position
//                       order (fp32) and read-modify-writes the table row once.  Runs longer
//                       than 32 are summed by the whole workgroup; runs longer than 2048 are
//                       queued per table as hot rows.  Buckets too large for LDS first split
//                       off their dominant rows unsorted (4a); what still does not fit goes to
//   4b. segment_sort / segment_reduce : a large list sorted by one workgroup per 2048 pairs
//                       with per-row counters in LDS, then reduced window by window.
//   5. hot_rows       : workgroup (bag group, table) streams the gradient rows of its bags
//                       through LDS once and adds them into every hot row that names them;
//      hot_finish     : adds a hot row's partial sums in bag-group order and updates the row.
// Steps 1-3 read indices and offsets only; dlrm_emb_bag_bwd_prepare enqueues just them.
// ATOMIC path (fp32 tables): a lane group per bag adds -lr*dS[b,k,:] to every row of the bag
// with hardware fp32 atomics; no workspace, one launch.  Measured 6x slower than SORT on the
// 8 x 1M x 64 multi-hot workload, so AUTO always takes SORT.
#include "common.h"

namespace dlrm {

constexpr int kThreads = 256;
constexpr int kNW = kThreads / DLRM_WAVE;       // wavefronts per workgroup
constexpr int kItems = 16;                      // positions per thread in a partition tile
constexpr int kTile = kThreads * kItems;        // 4096 positions per tile
constexpr int kMaxTopBits = 10;                 // partition digit: up to 1024 buckets per table
constexpr int kMaxBuckets = 1 << kMaxTopBits;
constexpr int kDPT = kMaxBuckets / kThreads;    // partition digits owned by one thread
constexpr int kSortBits = 8;                    // digit of the bucket-local LSD passes
constexpr int kSortBuckets = 1 << kSortBits;
constexpr int kBktItems = 8;                    // positions per thread in a bucket-sort tile
constexpr int kBktCap = kThreads * kBktItems;   // 2048: buckets up to this size are sorted in LDS
constexpr int kLongRun = 32;                    // longer runs are summed by the whole workgroup
constexpr int kHugeRun = 2048;                  // longer runs are split over workgroups
constexpr int kHotTileFloats = 16384;            // 64 KB of LDS: gradient rows of one bag tile
constexpr int kHotZeroRow = 256;                // floats of the widest gradient row
constexpr int kHotStagePasses = 16;             // float4 registers per thread holding the next tile
constexpr int kHotTilesPerGroup = 8;            // bag tiles streamed by one workgroup
constexpr int kHotRunsPerWave = 8;              // hot runs a wavefront accumulates at once
constexpr int kFusedScanMaxTiles = 512;         // fold the scan into the scatter below this
constexpr int kSegMaxBits = 13;                 // oversized buckets with at most this many low bits are
                                                // sorted by many workgroups (per-row counters in LDS)
constexpr int kSegKeys = 1 << kSegMaxBits;
constexpr int kSmallBatch = 65536;              // up to this many lookups the four launches that only
                                                // serve oversized buckets and hot rows cost more (~16 us)
                                                // than one workgroup doing that work in place ever could
constexpr int kCandMin = 128;                   // a row with this many of an oversized bucket's first
                                                // kBktCap pairs is split off before any sorting
constexpr int kCand = kBktCap / kCandMin;       // at most this many such rows

// ---------------------------------------------------------------------------
// Workspace layout (all offsets 256-byte aligned)
struct WsLayout {
  size_t keys[2], vals[2];   // uint32[nnz] ping-pong: row ids / bag ids
  size_t hist;               // uint32[kMaxBuckets * nt_max]: per-tile digit counts / offsets
  size_t bucket_start;       // uint32[K * kMaxBuckets + 1]
  size_t tile_heads;         // uint32[nt_max + 1]   (export only)
  size_t seg_start;          // uint32[nnz + 1]      (export only)
  size_t seg_tbl;            // uint32[nnz]          (export only)
  size_t n_seg;              // uint32[4]            (export only)
  size_t huge_ctr;           // uint32[4]: [2] = oversized-bucket count
  size_t hot_cnt;            // uint32[K]: queued hot runs per table
  size_t over_list;          // uint32[nnz / kBktCap + 1]: buckets too large for the LDS sort
  size_t segs;               // SegInfo[nnz / kBktCap + 2]: those of them sorted by many workgroups
  size_t seg_meta;           // uint32[8]: segment tiles, segments
  size_t huge_runs;          // HugeRun[nnz / kHugeRun + K]: table k's list starts at sum_{j<k}(nnz_j/kHugeRun + 1)
  size_t huge_part;          // float[max_runs * bag groups * d]
  size_t total;
  int64_t nt_max;            // upper bound on the number of tiles
  int64_t max_huge;          // upper bound on the number of queued runs
};

struct SegInfo {
  uint32_t start, n, k, low_bits;   // an oversized bucket: global position, pairs, table, unsorted bits
  uint32_t tile0, src, pad1, pad2;   // index of its first kBktCap-position tile among all segments;
                                     // pair buffer holding the unsorted pairs
};

struct HugeRun {
  uint32_t k, row, start, len;   // start: global position of the run's first sorted entry
  uint32_t pad0, src, pad1, pad2; // src: pair buffer holding the run
};

static inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// bags whose gradient rows one hot-row workgroup streams: kHotTilesPerGroup tiles of
// kHotStagePasses passes of kThreads / G rows (G lanes per row)
static inline int hot_group_bags(int d) { return kThreads / pow2_ceil(d / 4) * kHotStagePasses * kHotTilesPerGroup; }
static inline int hot_groups(int B, int d) {
  const int gb = hot_group_bags(d);
  return (B + gb - 1) / gb;
}

static WsLayout ws_layout(int32_t K, int32_t B, int32_t d, int64_t nnz) {
  WsLayout L;
  size_t o = 0;
  const size_t n = (size_t)(nnz > 0 ? nnz : 1);
  L.nt_max = nnz / kTile + K;
  L.max_huge = nnz / kHugeRun + K;
  for (int i = 0; i < 2; ++i) { L.keys[i] = o; o = align256(o + n * 4); }
  for (int i = 0; i < 2; ++i) { L.vals[i] = o; o = align256(o + n * 4); }
  L.hist = o;         o = align256(o + (size_t)kMaxBuckets * (size_t)L.nt_max * 4);
  L.bucket_start = o; o = align256(o + ((size_t)K * kMaxBuckets + 1) * 4);
  L.tile_heads = o;   o = align256(o + (size_t)(L.nt_max + 1) * 4);
  L.seg_start = o;    o = align256(o + (n + 1) * 4);
  L.seg_tbl = o;      o = align256(o + n * 4);
  L.n_seg = o;        o = align256(o + 16);
  L.huge_ctr = o;     o = align256(o + 16);
  L.hot_cnt = o;      o = align256(o + (size_t)K * 4);
  L.over_list = o;    o = align256(o + ((size_t)(nnz / kBktCap) + 1) * 4);
  L.segs = o;         o = align256(o + ((size_t)(nnz / kBktCap) + 2) * sizeof(SegInfo));
  L.seg_meta = o;     o = align256(o + 32);
  L.huge_runs = o;    o = align256(o + (size_t)L.max_huge * sizeof(HugeRun));
  L.huge_part = o;    o = align256(o + (size_t)L.max_huge * (size_t)hot_groups(B, d) * (size_t)d * 4);
  L.total = o;
  return L;
}

// ---------------------------------------------------------------------------
struct GroupArgs {            // everything the grouping kernels need
  const int64_t* indices;
  const int64_t* offsets;
  const int64_t* tbl_off;
  const int64_t* rows;
  int32_t K, B;
  int32_t nt_max;
  int32_t top_bits;           // bits of the partition digit (0..kMaxTopBits)
  int32_t fused_scan;         // 1: the scatter derives its offsets from the raw tile counts
  int32_t no_tail;            // 1: small batch, the segment and hot-row launches are left out and
                              //    bucket_reduce handles whatever they would have taken
  uint32_t* keys[2];
  uint32_t* vals[2];
  uint32_t* hist;
  uint32_t* bucket_start;
  uint32_t* tile_heads;
  uint32_t* seg_start;
  uint32_t* seg_tbl;
  uint32_t* n_seg;
  uint32_t* hot_cnt;
  uint32_t* over_cnt;
  uint32_t* over_list;
  int32_t max_over;           // workgroups reserved at the front of the bucket grid for oversized buckets
  SegInfo* segs;
  int32_t seg_tiles_max;      // upper bound on the number of segment tiles
  uint32_t* seg_meta;         // [0] segment tiles, [1] segments (one 64-bit counter)
  HugeRun* huge_runs;
  float* huge_part;
};

// start of table k's hot-run list: every table may queue at most nnz_k / kHugeRun runs
__device__ inline uint32_t hot_list_base(const GroupArgs& a, int k) {
  uint32_t base = 0;
  for (int j = 0; j < k; ++j) base += (uint32_t)((a.tbl_off[j + 1] - a.tbl_off[j]) / kHugeRun) + 1u;
  return base;
}

// bits needed to index m rows; the partition digit of table k is row >> top_shift(k)
__device__ inline int key_bits(int64_t m) { return m <= 1 ? 0 : 64 - __clzll((unsigned long long)(m - 1)); }
__device__ inline int top_shift(const GroupArgs& a, int k) {
  const int s = key_bits(a.rows[k]) - a.top_bits;
  return s > 0 ? s : 0;
}

// Which table and which positions a tile covers.  Workgroup-uniform.
struct TileInfo {
  int k;
  int t;           // tile index inside the table
  int t0;          // global index of the table's first tile
  int nt;          // tiles of the table
  int64_t start;   // global position of the tile's first item
  int count;       // items in the tile (1..kTile)
  int64_t tbl_start;
  int total_tiles; // tiles of all tables
};

// Every workgroup rebuilds the tile map from tbl_off (K is small): tables own
// ceil(nnz_k / kTile) consecutive tiles.  All threads must call this (it synchronises).
__device__ inline bool find_tile(const GroupArgs& a, int tile, TileInfo& ti, uint32_t* smem) {
  __shared__ int res[4];
  if (threadIdx.x == 0) res[0] = -1;
  uint32_t carry = 0;
  for (int k0 = 0; k0 < a.K; k0 += kThreads) {
    const int k = k0 + threadIdx.x;
    uint32_t nt = 0;
    if (k < a.K) nt = (uint32_t)((a.tbl_off[k + 1] - a.tbl_off[k] + kTile - 1) / kTile);
    uint32_t total;
    const uint32_t first = carry + block_exclusive_scan<kThreads>(nt, smem, &total);
    if (k < a.K && (uint32_t)tile >= first && (uint32_t)tile < first + nt) {
      res[0] = k;
      res[1] = (int)first;
      res[2] = (int)nt;
    }
    carry += total;
  }
  __syncthreads();
  ti.total_tiles = (int)carry;
  if (res[0] < 0) return false;
  ti.k = res[0];
  ti.t0 = res[1];
  ti.nt = res[2];
  ti.t = tile - ti.t0;
  ti.tbl_start = a.tbl_off[ti.k];
  ti.start = ti.tbl_start + (int64_t)ti.t * kTile;
  const int64_t rem = a.tbl_off[ti.k + 1] - ti.start;
  ti.count = (int)(rem < kTile ? rem : kTile);
  return true;
}

// --- 1. per-tile histogram of the partition digit ----------------------------------
__global__ __launch_bounds__(kThreads) void bucket_hist_kernel(GroupArgs a) {
  __shared__ uint32_t h[kMaxBuckets];
  __shared__ uint32_t smem[kNW + 1];
  TileInfo ti;
  if (!find_tile(a, blockIdx.x, ti, smem)) return;
  const int nb = 1 << a.top_bits;
  for (int i = threadIdx.x; i < nb; i += kThreads) h[i] = 0;
  __syncthreads();
  const int64_t* idx = a.indices + ti.start;
  const int shift = top_shift(a, ti.k);
  const uint32_t mask = (uint32_t)nb - 1;
  for (int i = threadIdx.x; i < ti.count; i += kThreads)
    atomicAdd(&h[((uint32_t)idx[i] >> shift) & mask], 1u);
  __syncthreads();
  for (int i = threadIdx.x; i < nb; i += kThreads) a.hist[(size_t)i * a.nt_max + blockIdx.x] = h[i];
  if (blockIdx.x == 0 && threadIdx.x == 0) {  // consumed by later launches of the same call
    *a.over_cnt = 0u;
    for (int k = 0; k < a.K; ++k) a.hot_cnt[k] = 0u;
    a.seg_meta[0] = 0u;
    a.seg_meta[1] = 0u;
    a.seg_meta[2] = 0u;
  }
}

// --- 2. per-table scan (large batches only): counts -> destination offsets ------------
// One workgroup per table walks (digit, tile) in digit-major order with a running carry
// that starts at the table's slice, so every table is scattered inside its own slice.
__global__ __launch_bounds__(1024) void bucket_scan_kernel(GroupArgs a) {
  __shared__ uint32_t smem[1024 / DLRM_WAVE + 1];
  const int k = blockIdx.x;
  // first tile of table k = tiles of all earlier tables
  uint32_t t0 = 0;
  for (int j = 0; j < k; ++j) t0 += (uint32_t)((a.tbl_off[j + 1] - a.tbl_off[j] + kTile - 1) / kTile);
  const int nt = (int)((a.tbl_off[k + 1] - a.tbl_off[k] + kTile - 1) / kTile);
  const int nb = 1 << a.top_bits;
  uint32_t carry = (uint32_t)a.tbl_off[k];
  if (nt <= 0) {
    for (int i = threadIdx.x; i < nb; i += 1024) a.bucket_start[(size_t)k * nb + i] = carry;
    return;
  }
  const int64_t n = (int64_t)nt * nb;
  for (int64_t e0 = 0; e0 < n; e0 += 1024) {
    const int64_t e = e0 + threadIdx.x;
    uint32_t v = 0;
    size_t addr = 0;
    int digit = 0, t = 0;
    if (e < n) {
      digit = (int)(e / nt);
      t = (int)(e - (int64_t)digit * nt);
      addr = (size_t)digit * a.nt_max + t0 + t;
      v = a.hist[addr];
    }
    uint32_t total;
    const uint32_t ex = block_exclusive_scan<1024>(v, smem, &total);
    if (e < n) {
      a.hist[addr] = carry + ex;
      if (t == 0) a.bucket_start[(size_t)k * nb + digit] = carry + ex;
    }
    carry += total;
  }
  __syncthreads();  // this workgroup's bucket_start writes are visible to it
  for (int dg = threadIdx.x; dg < nb; dg += 1024) {
    const uint32_t st = a.bucket_start[(size_t)k * nb + dg];
    const uint32_t en = dg + 1 < nb ? a.bucket_start[(size_t)k * nb + dg + 1] : (uint32_t)a.tbl_off[k + 1];
    if (en - st > (uint32_t)kBktCap) a.over_list[atomicAdd(a.over_cnt, 1u)] = (uint32_t)(k * nb + dg);
  }
}

// --- shared by steps 3 and 4: stable ranking of a tile by a digit ---------------------
// Wave w of the workgroup owns the contiguous positions [w*64*ITEMS, (w+1)*64*ITEMS) of
// the tile, item j of lane l being position w*64*ITEMS + j*64 + l.  Ranks inside a wave
// come from ballot matching; per-wave digit counters in LDS give the order across waves.
// On return rnk[j] is the item's rank among the items of its wave with the same digit that
// precede it, and wcnt[w][digit] the wave's count.  wcnt must be zero on entry.
template <int ITEMS, int NBK>
__device__ inline void rank_items(const uint32_t* dg, const bool* ok, int bits,
                                  uint32_t (*wcnt)[NBK], uint32_t* rnk) {
  const int lane = lane_id(), w = wave_id();
  const unsigned long long lt = (1ull << lane) - 1ull;
#pragma unroll
  for (int j = 0; j < ITEMS; ++j) {
    unsigned long long m = __ballot(ok[j]);
    for (int bit = 0; bit < bits; ++bit) {
      const bool one = (dg[j] >> bit) & 1u;
      const unsigned long long bal = __ballot(one);
      m &= one ? bal : ~bal;
    }
    // m: valid lanes of this wave holding the same digit in item j (meaningful where ok)
    uint32_t prev = 0;
    const int leader = ok[j] ? (__ffsll((long long)m) - 1) : lane;
    if (ok[j] && lane == leader) prev = atomicAdd(&wcnt[w][dg[j]], (uint32_t)__popcll(m));
    prev = __shfl(prev, leader, DLRM_WAVE);
    rnk[j] = prev + (uint32_t)__popcll(m & lt);
  }
}

// After rank_items + a barrier: turns wcnt[w][digit] into the tile-local sorted position of
// wave w's first item with that digit.  Thread t owns the DPT = NBK/256 consecutive digits
// t*DPT .. t*DPT+DPT-1 and gets their tile-local offsets and counts.  All threads must call it.
template <int NBK>
__device__ inline void digit_offsets(int nb, uint32_t (*wcnt)[NBK], uint32_t* scan_smem,
                                     uint32_t* lofs_out, uint32_t* tot_out) {
  constexpr int DPT = NBK / kThreads;
  uint32_t c[DPT][kNW], tot[DPT], sum = 0;
#pragma unroll
  for (int q = 0; q < DPT; ++q) {
    const int dg = threadIdx.x * DPT + q;
    tot[q] = 0;
#pragma unroll
    for (int i = 0; i < kNW; ++i) {
      c[q][i] = dg < nb ? wcnt[i][dg] : 0u;
      tot[q] += c[q][i];
    }
    sum += tot[q];
  }
  uint32_t total_all;
  uint32_t run = block_exclusive_scan<kThreads>(sum, scan_smem, &total_all);
#pragma unroll
  for (int q = 0; q < DPT; ++q) {
    const int dg = threadIdx.x * DPT + q;
    lofs_out[q] = run;
    tot_out[q] = tot[q];
    if (dg < nb) {
#pragma unroll
      for (int i = 0; i < kNW; ++i) {
        wcnt[i][dg] = run;
        run += c[q][i];
      }
    }
  }
}

// Oversized buckets whose unsorted low bits fit per-row counters in LDS become "segments",
// sorted by one workgroup per kBktCap-position tile (segment_sort_kernel).  One workgroup builds
// the segment list and its tile map.  All threads call it.
__device__ inline void prepare_segments(const GroupArgs& a, uint32_t* smem) {
  const int nb = 1 << a.top_bits;
  const uint32_t n_over = atomicAdd(a.over_cnt, 0u);
  uint32_t nseg = 0, ntiles = 0;
  for (uint32_t e0 = 0; e0 < n_over; e0 += kThreads) {
    const uint32_t e = e0 + threadIdx.x;
    SegInfo sg;
    uint32_t ok = 0, nt = 0;
    if (e < n_over) {
      const uint32_t id = a.over_list[e];
      const int k = (int)(id >> a.top_bits), dg = (int)(id & (uint32_t)(nb - 1));
      sg.start = a.bucket_start[(size_t)k * nb + dg];
      const uint32_t end = dg + 1 < nb ? a.bucket_start[(size_t)k * nb + dg + 1] : (uint32_t)a.tbl_off[k + 1];
      sg.n = end - sg.start;
      sg.k = (uint32_t)k;
      sg.low_bits = (uint32_t)top_shift(a, k);
      ok = sg.low_bits >= 1 && sg.low_bits <= (uint32_t)kSegMaxBits ? 1u : 0u;
      nt = ok ? (sg.n + kBktCap - 1) / kBktCap : 0u;
    }
    uint32_t tot_s, tot_t;
    const uint32_t slot = block_exclusive_scan<kThreads>(ok, smem, &tot_s);
    const uint32_t tpos = block_exclusive_scan<kThreads>(nt, smem, &tot_t);
    if (ok) {
      sg.tile0 = ntiles + tpos;
      sg.src = 1;
      sg.pad1 = sg.pad2 = 0;
      a.segs[nseg + slot] = sg;
    }
    nseg += tot_s;
    ntiles += tot_t;
  }
  if (threadIdx.x == 0) {
    a.seg_meta[0] = ntiles;
    a.seg_meta[1] = nseg;
  }
}

// --- 3. stable scatter into buckets ---------------------------------------------------
__global__ __launch_bounds__(kThreads) void bucket_scatter_kernel(GroupArgs a) {
  __shared__ uint32_t wcnt[kNW][kMaxBuckets];
  __shared__ uint32_t gofs[kMaxBuckets];
  __shared__ uint32_t skey[kTile];
  __shared__ uint32_t sval[kTile];
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
  const int64_t* kin = a.indices + ti.start;
  const int shift = top_shift(a, ti.k);
  uint32_t key[kItems], val[kItems], dg[kItems], rnk[kItems];
  bool ok[kItems];
#pragma unroll
  for (int j = 0; j < kItems; ++j) {
    const int li = w * (DLRM_WAVE * kItems) + j * DLRM_WAVE + lane;
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
  for (int i = tid; i < kTile; i += kThreads) skey[i] = 0;  // skey doubles as the bag-start counters
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
  {  // inclusive prefix of the start counters, thread t owning positions [t*kItems, (t+1)*kItems)
    uint32_t c[kItems], s = 0;
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
      c[j] = skey[tid * kItems + j];
      s += c[j];
    }
    uint32_t total;
    uint32_t run = block_exclusive_scan<kThreads>(s, smem, &total);
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
      run += c[j];
      sval[tid * kItems + j] = (uint32_t)b0 + run;
    }
  }
  __syncthreads();

  // ---- bags of this thread's (wave-striped) positions, then rank by partition digit
#pragma unroll
  for (int j = 0; j < kItems; ++j) {
    const int li = w * (DLRM_WAVE * kItems) + j * DLRM_WAVE + lane;
    val[j] = ok[j] ? sval[li] : 0u;
  }
  rank_items<kItems, kMaxBuckets>(dg, ok, a.top_bits, wcnt, rnk);
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
        if (total[q] > (uint32_t)kBktCap) a.over_list[atomicAdd(a.over_cnt, 1u)] = (uint32_t)(ti.k * nb + dgt);
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
  for (int j = 0; j < kItems; ++j) {
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

// --- 4. bucket-local sort ----------------------------------------------------------------
struct Bucket {
  int k;
  uint32_t start, n;   // global position of the bucket's first pair, pairs in the bucket
  int low_bits;        // row-id bits below the partition digit
};

// Buckets larger than the LDS sort take much longer than the rest: they are listed during the
// partition and handed to the FIRST workgroups of the grid, so that they start early and run
// beside everything else.  Returns false if this workgroup has nothing to do.
__device__ inline bool bucket_id_of_block(const GroupArgs& a, uint32_t* id, bool* oversized) {
  if (blockIdx.x < (uint32_t)a.max_over) {
    if (blockIdx.x >= *a.over_cnt) return false;
    *id = a.over_list[blockIdx.x];
    *oversized = true;
    return true;
  }
  *id = blockIdx.x - (uint32_t)a.max_over;
  *oversized = false;
  return true;
}

__device__ inline Bucket bucket_of_block(const GroupArgs& a, uint32_t id) {
  const int nb = 1 << a.top_bits;
  Bucket b;
  b.k = (int)(id >> a.top_bits);
  const int dg = (int)(id & (uint32_t)(nb - 1));
  b.start = 0;
  b.n = 0;
  b.low_bits = 0;
  if (a.tbl_off[b.k + 1] == a.tbl_off[b.k]) return b;  // no lookups: its bucket_start is never written
  b.start = a.bucket_start[(size_t)b.k * nb + dg];
  const uint32_t end = dg + 1 < nb ? a.bucket_start[(size_t)b.k * nb + dg + 1] : (uint32_t)a.tbl_off[b.k + 1];
  b.n = end - b.start;
  b.low_bits = top_shift(a, b.k);
  return b;
}

struct SortLds {
  uint32_t wcnt[kNW][kSortBuckets];
  uint32_t skey[kBktCap];
  uint32_t sval[kBktCap];
  uint32_t heads[kBktCap + 1];
  uint32_t base[kSortBuckets];
  uint32_t smem[kNW + 1];
  uint32_t longs[kBktCap / kLongRun + 2];   // runs longer than kLongRun among the current heads
  uint32_t nlong;
};

__device__ inline int pass_bits(int left, int passes_left) { return (left + passes_left - 1) / passes_left; }

// Buckets of at most kBktCap pairs (read from pair buffer src): stable LSD passes entirely in
// LDS.  The pairs end up in s.skey / s.sval in (row, position) order.
__device__ inline void sort_bucket_lds(const GroupArgs& a, const Bucket& b, SortLds& s, int src = 1) {
  const int lane = lane_id(), w = wave_id(), tid = threadIdx.x;
  const uint32_t* kin = a.keys[src] + b.start;
  const uint32_t* vin = a.vals[src] + b.start;
  const int n = (int)b.n;
  uint32_t key[kBktItems], val[kBktItems], dg[kBktItems], rnk[kBktItems];
  bool ok[kBktItems];
#pragma unroll
  for (int j = 0; j < kBktItems; ++j) {
    const int li = w * (DLRM_WAVE * kBktItems) + j * DLRM_WAVE + lane;
    ok[j] = li < n;
    key[j] = ok[j] ? kin[li] : 0xFFFFFFFFu;
    val[j] = ok[j] ? vin[li] : 0u;
  }
  const int passes = (b.low_bits + kSortBits - 1) / kSortBits;
  if (passes == 0) {  // a single row per bucket: already in position order
#pragma unroll
    for (int j = 0; j < kBktItems; ++j) {
      const int li = w * (DLRM_WAVE * kBktItems) + j * DLRM_WAVE + lane;
      if (ok[j]) {
        s.skey[li] = key[j];
        s.sval[li] = val[j];
      }
    }
    __syncthreads();
    return;
  }
  int shift = 0;
  for (int p = 0; p < passes; ++p) {
    const int bits = pass_bits(b.low_bits - shift, passes - p);
    const int nb = 1 << bits;
    const uint32_t mask = (uint32_t)nb - 1;
    for (int i = tid; i < kNW * kSortBuckets; i += kThreads) (&s.wcnt[0][0])[i] = 0;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kBktItems; ++j) dg[j] = (key[j] >> shift) & mask;
    rank_items<kBktItems, kSortBuckets>(dg, ok, bits, s.wcnt, rnk);
    __syncthreads();
    uint32_t lofs, tot;
    digit_offsets<kSortBuckets>(nb, s.wcnt, s.smem, &lofs, &tot);
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kBktItems; ++j) {
      if (ok[j]) {
        const uint32_t lp = s.wcnt[w][dg[j]] + rnk[j];
        s.skey[lp] = key[j];
        s.sval[lp] = val[j];
      }
    }
    __syncthreads();
    shift += bits;
    if (p + 1 < passes) {
#pragma unroll
      for (int j = 0; j < kBktItems; ++j) {
        const int li = w * (DLRM_WAVE * kBktItems) + j * DLRM_WAVE + lane;
        if (ok[j]) {
          key[j] = s.skey[li];
          val[j] = s.sval[li];
        }
      }
      __syncthreads();
    }
  }
}

// Larger buckets: the same stable passes, one workgroup streaming its bucket through global
// memory (ping-pong between the two pair buffers, starting in buffer src).  Returns the buffer
// holding the result.
__device__ inline int sort_bucket_global(const GroupArgs& a, const Bucket& b, SortLds& s, int src = 1) {
  const int lane = lane_id(), w = wave_id(), tid = threadIdx.x;
  const int passes = (b.low_bits + kSortBits - 1) / kSortBits;
  int shift = 0;
  for (int p = 0; p < passes; ++p) {
    const int bits = pass_bits(b.low_bits - shift, passes - p);
    const int nb = 1 << bits;
    const uint32_t mask = (uint32_t)nb - 1;
    const uint32_t* kin = a.keys[src] + b.start;
    const uint32_t* vin = a.vals[src] + b.start;
    uint32_t* kout = a.keys[src ^ 1] + b.start;
    uint32_t* vout = a.vals[src ^ 1] + b.start;
    // digit totals over the whole bucket -> running destination of every digit
    if (tid < kSortBuckets) s.base[tid] = 0;
    __syncthreads();
    for (uint32_t i = tid; i < b.n; i += kThreads) atomicAdd(&s.base[(kin[i] >> shift) & mask], 1u);
    __syncthreads();
    {
      const uint32_t c = tid < nb ? s.base[tid] : 0u;
      uint32_t all;
      const uint32_t ex = block_exclusive_scan<kThreads>(c, s.smem, &all);
      __syncthreads();
      if (tid < nb) s.base[tid] = ex;
    }
    __syncthreads();
    for (uint32_t t0 = 0; t0 < b.n; t0 += kBktCap) {  // tiles in order: stable
      const int cnt = (int)(b.n - t0 < (uint32_t)kBktCap ? b.n - t0 : (uint32_t)kBktCap);
      uint32_t key[kBktItems], val[kBktItems], dg[kBktItems], rnk[kBktItems];
      bool ok[kBktItems];
      for (int i = tid; i < kNW * kSortBuckets; i += kThreads) (&s.wcnt[0][0])[i] = 0;
#pragma unroll
      for (int j = 0; j < kBktItems; ++j) {
        const int li = w * (DLRM_WAVE * kBktItems) + j * DLRM_WAVE + lane;
        ok[j] = li < cnt;
        key[j] = ok[j] ? kin[t0 + li] : 0xFFFFFFFFu;
        val[j] = ok[j] ? vin[t0 + li] : 0u;
        dg[j] = (key[j] >> shift) & mask;
      }
      __syncthreads();
      rank_items<kBktItems, kSortBuckets>(dg, ok, bits, s.wcnt, rnk);
      __syncthreads();
      uint32_t lofs, tot;
      digit_offsets<kSortBuckets>(nb, s.wcnt, s.smem, &lofs, &tot);
      if (tid < nb) s.heads[tid] = lofs;  // s.heads is free during the sort: tile-local digit offsets
      __syncthreads();
#pragma unroll
      for (int j = 0; j < kBktItems; ++j) {
        if (ok[j]) {
          // wcnt[w][dg] = tile-local sorted position of the wave's first item of the digit;
          // minus the digit's tile-local offset = rank inside the digit within this tile
          const uint32_t dst = s.base[dg[j]] + (s.wcnt[w][dg[j]] - s.heads[dg[j]]) + rnk[j];
          kout[dst] = key[j];
          vout[dst] = val[j];
        }
      }
      __syncthreads();
      if (tid < nb) s.base[tid] += tot;
      __syncthreads();
    }
    src ^= 1;
    shift += bits;
  }
  return src;
}

// --- 4b. runs -> row updates ------------------------------------------------------------------
struct UpdArgs {
  void* const* tables;
  void* const* state;   // Adagrad: K fp32 accumulators shaped like the tables; else unused
  const float* dS;
  int64_t stride_b, stride_k;
  float lr, eps;
  int32_t d;
};

// What is done to a row once its gradient g is summed (Sec. 5.1 names both optimizers):
//   kSgd     : W <- W - lr * g
//   kAdagrad : h <- h + g*g (fp32 state), W <- W - lr * g / (sqrt(h) + eps), element-wise
constexpr int kSgd = 0, kAdagrad = 1;

// The 4 columns [chunk*4, chunk*4+4) of a table row: raw load, and update + store
// (fp32: W - lr*g; fp16/bf16: widen, update in fp32, one round-to-nearest-even).
// W: base of the table, read from the pointer array ONCE per workgroup -- the row stores below
// may alias anything as far as the compiler knows, so a per-row read of tables[k] would be
// re-issued (and waited for) before every row.
template <int DT>
__device__ inline char* row_chunk_ptr(char* W, int d, uint32_t row, int chunk) {
  return W + ((int64_t)row * d + chunk * 4) * Tab<DT>::EB;
}
template <int DT>
__device__ inline u32x4 row_chunk_load(const char* p) {
  if constexpr (DT == DLRM_F32) {
    return load16(p);
  } else {
    const u32x2 b = *reinterpret_cast<const u32x2*>(p);
    return u32x4{b.x, b.y, 0u, 0u};
  }
}
template <int DT>
__device__ inline void row_chunk_update_store(char* p, u32x4 raw, f32x4 g, float lr) {
  if constexpr (DT == DLRM_F32) {
    f32x4 x;
    x.x = fmaf(-lr, g.x, u2f(raw.x));
    x.y = fmaf(-lr, g.y, u2f(raw.y));
    x.z = fmaf(-lr, g.z, u2f(raw.z));
    x.w = fmaf(-lr, g.w, u2f(raw.w));
    storef4(reinterpret_cast<float*>(p), x);
  } else {
    float x0, x1, x2, x3;
    if constexpr (DT == DLRM_F16) {
      half2_to_float2(raw.x, x0, x1);
      half2_to_float2(raw.y, x2, x3);
    } else {
      bf162_to_float2(raw.x, x0, x1);
      bf162_to_float2(raw.y, x2, x3);
    }
    x0 = fmaf(-lr, g.x, x0);
    x1 = fmaf(-lr, g.y, x1);
    x2 = fmaf(-lr, g.z, x2);
    x3 = fmaf(-lr, g.w, x3);
    u32x2 b;
    if constexpr (DT == DLRM_F16) {
      b.x = float2_to_half2(x0, x1);
      b.y = float2_to_half2(x2, x3);
    } else {
      b.x = float2_to_bf162(x0, x1);
      b.y = float2_to_bf162(x2, x3);
    }
    *reinterpret_cast<u32x2*>(p) = b;
  }
}
// The same 4 columns of a row together with their optimizer state (none for SGD).
struct RowRef {
  char* w;
  float* h;
};
struct RowVal {
  u32x4 w;
  f32x4 h;
};
template <int DT, int OPT>
__device__ inline RowRef row_ref(char* W, float* H, int d, uint32_t row, int chunk) {
  const int64_t e = (int64_t)row * d + chunk * 4;
  RowRef r;
  r.w = W + e * Tab<DT>::EB;
  r.h = OPT == kAdagrad ? H + e : nullptr;
  return r;
}
template <int DT, int OPT>
__device__ inline RowVal row_load(const RowRef& r) {
  RowVal v;
  v.w = row_chunk_load<DT>(r.w);
  v.h = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
  if constexpr (OPT == kAdagrad) v.h = loadf4(r.h);
  return v;
}
template <int DT, int OPT>
__device__ inline void row_update_store(const RowRef& r, const RowVal& v, f32x4 g, const UpdArgs& u) {
  if constexpr (OPT == kAdagrad) {
    f32x4 h, step;
    h.x = fmaf(g.x, g.x, v.h.x);
    h.y = fmaf(g.y, g.y, v.h.y);
    h.z = fmaf(g.z, g.z, v.h.z);
    h.w = fmaf(g.w, g.w, v.h.w);
    storef4(r.h, h);
    step.x = u.lr * g.x / (sqrtf(h.x) + u.eps);
    step.y = u.lr * g.y / (sqrtf(h.y) + u.eps);
    step.z = u.lr * g.z / (sqrtf(h.z) + u.eps);
    step.w = u.lr * g.w / (sqrtf(h.w) + u.eps);
    row_chunk_update_store<DT>(r.w, v.w, step, 1.0f);  // W - 1 * step, one rounding
  } else {
    row_chunk_update_store<DT>(r.w, v.w, g, u.lr);
  }
}
template <int DT, int OPT>
__device__ inline void row_update(char* W, float* H, const UpdArgs& u, uint32_t row, int chunk, f32x4 g) {
  const RowRef r = row_ref<DT, OPT>(W, H, u.d, row, chunk);
  row_update_store<DT, OPT>(r, row_load<DT, OPT>(r), g, u);
}
// base of table k's optimizer state (read once per workgroup, like the table base)
template <int OPT>
__device__ inline float* state_base(const UpdArgs& u, int k) {
  if constexpr (OPT == kAdagrad) return static_cast<float*>(u.state[k]);
  return nullptr;
}

// Sum dS rows of the sorted entries [i0, i1) taking every `stride`-th entry from i0 + first;
// U loads in flight, ascending order.  bags: LDS or global.
template <int U>
__device__ inline f32x4 sum_entries(const float* g, int64_t stride_b, const uint32_t* bags, uint32_t i0,
                                    uint32_t i1, uint32_t first, uint32_t stride) {
  f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
  for (uint32_t i = i0 + first; i < i1; i += U * stride) {
    uint32_t bg[U];
    f32x4 v[U];
#pragma unroll
    for (int t = 0; t < U; ++t) bg[t] = bags[i + t * stride < i1 ? i + t * stride : i];
#pragma unroll
    for (int t = 0; t < U; ++t) v[t] = loadf4(g + (int64_t)bg[t] * stride_b);
#pragma unroll
    for (int t = 0; t < U; ++t)
      if (i + t * stride < i1) acc += v[t];
  }
  return acc;
}

// keys/bags: the bucket's sorted pairs (n of them; LDS or global), heads: LDS list of run starts
// with heads[nruns] = n.  gpos0: global position of the bucket's first pair.
template <int DT, int G, int OPT>
__device__ inline void reduce_runs(const GroupArgs& a, const UpdArgs& u, const Bucket& b, char* W,
                                   const uint32_t* keys, const uint32_t* bags, const uint32_t* heads,
                                   uint32_t h0, uint32_t nruns, const uint32_t* longs, uint32_t nlong,
                                   int src, float* part) {
  constexpr int NG = kThreads / G;
  const int grp = threadIdx.x / G, chunk = threadIdx.x % G;
  const bool col_ok = chunk * 4 < u.d;
  // lanes past the last column shadow column group 0 (same addresses) and never write
  const float* g = u.dS + (int64_t)b.k * u.stride_k + (col_ok ? chunk : 0) * 4;
  // short runs: a lane group takes RU runs per round; the table rows and the first gradient
  // row of all RU runs are requested before any of them is consumed
  constexpr int RU = OPT == kAdagrad ? 2 : 4;  // Adagrad also holds the state rows
  const int cchunk = col_ok ? chunk : 0;
  float* H = state_base<OPT>(u, b.k);
  for (uint32_t r0 = (uint32_t)grp * RU; r0 < nruns; r0 += NG * RU) {
    uint32_t i0[RU], i1[RU];
    RowRef wp[RU];
    RowVal wv[RU];
    f32x4 acc[RU];
#pragma unroll
    for (int t = 0; t < RU; ++t) {
      const uint32_t rr = r0 + t < nruns ? r0 + t : nruns - 1;  // the tail repeats the last run
      i0[t] = heads[rr] - h0;
      i1[t] = heads[rr + 1] - h0;
      wp[t] = row_ref<DT, OPT>(W, H, u.d, keys[i0[t]], cchunk);
    }
#pragma unroll
    for (int t = 0; t < RU; ++t) acc[t] = loadf4(g + (int64_t)bags[i0[t]] * u.stride_b);
#pragma unroll
    for (int t = 0; t < RU; ++t) wv[t] = row_load<DT, OPT>(wp[t]);
#pragma unroll
    for (int t = 0; t < RU; ++t) {
      const uint32_t len = i1[t] - i0[t];
      if (r0 + t >= nruns || len > (uint32_t)kLongRun) continue;
      if (len > 1) acc[t] += sum_entries<4>(g, u.stride_b, bags, i0[t] + 1, i1[t], 0, 1);
      if (col_ok) row_update_store<DT, OPT>(wp[t], wv[t], acc[t], u);
    }
  }
  // long runs: the whole workgroup per run, lane group s taking entries s, s+NG, ...; the NG
  // partial sums are added in group order
  for (uint32_t q = 0; q < nlong; ++q) {  // uniform
    const uint32_t r = longs[q];
    const uint32_t i0 = heads[r] - h0, i1 = heads[r + 1] - h0;
    const uint32_t len = i1 - i0;
    if (len > (uint32_t)kHugeRun && !a.no_tail) {  // queue for the multi-workgroup pass
      if (threadIdx.x == 0) {
        HugeRun hr;
        hr.k = (uint32_t)b.k;
        hr.row = keys[i0];
        hr.start = b.start + h0 + i0;
        hr.len = len;
        hr.src = (uint32_t)src;
        hr.pad0 = hr.pad1 = hr.pad2 = 0;
        a.huge_runs[hot_list_base(a, b.k) + atomicAdd(&a.hot_cnt[b.k], 1u)] = hr;
      }
      continue;
    }
    const f32x4 acc = sum_entries<4>(g, u.stride_b, bags, i0, i1, (uint32_t)grp, (uint32_t)NG);
    __syncthreads();
    if (col_ok) storef4(part + grp * (G * 4) + chunk * 4, acc);
    __syncthreads();
    if (grp == 0 && col_ok) {
      f32x4 tot = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int s = 0; s < NG; ++s) tot += loadf4(part + s * (G * 4) + chunk * 4);
      row_update<DT, OPT>(W, H, u, keys[i0], chunk, tot);
    }
  }
}

// Run heads of sorted keys[0..n) (LDS) into s.heads (positions, ascending) with the sentinel
// heads[nruns] = n.  Returns nruns.  All threads call it.
__device__ inline uint32_t compact_heads_lds(SortLds& s, int n) {
  const int tid = threadIdx.x;
  uint32_t flags = 0, cnt = 0;
#pragma unroll
  for (int j = 0; j < kBktItems; ++j) {
    const int li = tid * kBktItems + j;
    if (li < n && (li == 0 || s.skey[li] != s.skey[li - 1])) {
      flags |= 1u << j;
      ++cnt;
    }
  }
  uint32_t total;
  uint32_t pos = block_exclusive_scan<kThreads>(cnt, s.smem, &total);
#pragma unroll
  for (int j = 0; j < kBktItems; ++j) {
    if (flags & (1u << j)) s.heads[pos++] = (uint32_t)(tid * kBktItems + j);
  }
  if (tid == 0) s.heads[total] = (uint32_t)n;
  __syncthreads();
  return total;
}

// Lists the runs longer than kLongRun among s.heads[0..nruns] (any order: each is a different
// row).  At most kBktCap/kLongRun + 1 of them have their head inside a window of kBktCap positions.
__device__ inline uint32_t collect_long_runs(SortLds& s, uint32_t nruns) {
  if (threadIdx.x == 0) s.nlong = 0;
  __syncthreads();
  for (uint32_t r = threadIdx.x; r < nruns; r += kThreads) {
    if (s.heads[r + 1] - s.heads[r] > (uint32_t)kLongRun) s.longs[atomicAdd(&s.nlong, 1u)] = r;
  }
  __syncthreads();
  return s.nlong;
}

// First position in [lo, n) whose key differs from `key`, given that keys are sorted and every
// position in [.., lo) of the run equals it: 256-ary search, workgroup-uniform.
__device__ inline uint32_t run_end_search(const uint32_t* keys, uint32_t lo, uint32_t n, uint32_t key) {
  uint32_t hi = n;  // the answer lies in [lo, hi]
  while (lo < hi) {
    const uint32_t step = (hi - lo + kThreads - 1) / kThreads;
    const uint32_t q = lo + threadIdx.x * step;
    const int same = (q < hi && keys[q] == key) ? 1 : 0;
    const uint32_t cnt = (uint32_t)__syncthreads_count(same);  // sorted: the first cnt probes match
    if (cnt == 0) break;
    const uint32_t nhi = lo + cnt * step < hi ? lo + cnt * step : hi;
    lo = lo + (cnt - 1) * step + 1;
    hi = nhi;
  }
  return lo;
}

// One window of kBktCap positions of a sorted pair list (global memory): the runs whose head
// lies in the window are reduced and applied; a run may extend past the window.
template <int DT, int G, int OPT>
__device__ inline void reduce_window(const GroupArgs& a, const UpdArgs& u, const Bucket& b, char* W,
                                     const uint32_t* keys, const uint32_t* bags, uint32_t w0, int src,
                                     SortLds& s, float* part) {
  const int cnt = (int)(b.n - w0 < (uint32_t)kBktCap ? b.n - w0 : (uint32_t)kBktCap);
  const int tid = threadIdx.x;
  uint32_t flags = 0, c = 0;
#pragma unroll
  for (int j = 0; j < kBktItems; ++j) {
    const int li = tid * kBktItems + j;
    if (li < cnt && (w0 + li == 0 || keys[w0 + li] != keys[w0 + li - 1])) {
      flags |= 1u << j;
      ++c;
    }
  }
  uint32_t total;
  uint32_t pos = block_exclusive_scan<kThreads>(c, s.smem, &total);
#pragma unroll
  for (int j = 0; j < kBktItems; ++j) {
    if (flags & (1u << j)) s.heads[pos++] = w0 + (uint32_t)(tid * kBktItems + j);
  }
  __syncthreads();
  if (total > 0) {  // uniform
    const uint32_t e = run_end_search(keys, w0 + (uint32_t)cnt, b.n, keys[s.heads[total - 1]]);
    if (tid == 0) s.heads[total] = e;
    __syncthreads();
    const uint32_t nlong = collect_long_runs(s, total);
    reduce_runs<DT, G, OPT>(a, u, b, W, keys, bags, s.heads, 0u, total, s.longs, nlong, src, part);
  }
  __syncthreads();
}

// --- 4a. oversized buckets: dominant rows split off first ------------------------------------------
// A bucket outgrows the LDS sort almost always because a few hot rows own most of its pairs.
// Rows holding at least kCandMin of the bucket's first kBktCap pairs become candidates (at most
// kCand = kBktCap / kCandMin of them).  One count pass and one stable partition pass over the
// bucket then give every candidate its own list (position order is kept, so its bags ascend) and
// collect the rest behind them; no pair of a candidate is ever sorted.  The rest usually fits
// the LDS sort; if not, it alone goes to the segment kernels or the streaming sort.
struct SplitLds {
  uint32_t cand[kCand];       // candidate row ids, in row order; unused slots 0xFFFFFFFF
  uint32_t cnt[kCand + 1];    // pairs per class; class kCand = every other row
  uint32_t wcnt[kNW][kCand + 1];   // the same per wavefront (each streams a quarter of the bucket)
  uint32_t wbase[kNW][kCand + 1];  // running destination of every (wavefront, class)
  uint32_t cbase[kCand + 2];  // exclusive prefix of cnt
  uint32_t nc;
};

__device__ inline uint32_t class_of(uint32_t key, const uint32_t* cd) {
  uint32_t cls = (uint32_t)kCand;
#pragma unroll
  for (int c = 0; c < kCand; ++c) cls = key == cd[c] ? (uint32_t)c : cls;
  return cls;
}

// Pairs [bk.start, bk.start + bk.n) of pair buffer src, more than kBktCap of them, that no
// shortcut applies to: queued as a segment when per-row counters fit LDS, else sorted here.
template <int DT, int G, int OPT>
__device__ inline void sort_reduce_large(const GroupArgs& a, const UpdArgs& u, const Bucket& bk, char* W,
                                         int src, SortLds& s, float* part) {
  if (bk.low_bits <= kSegMaxBits && !a.no_tail) {
    if (threadIdx.x == 0) {
      const uint32_t nt = (bk.n + kBktCap - 1) / kBktCap;
      // one 64-bit counter hands out the slot and the first tile together, so that the list is
      // ordered by first tile
      const unsigned long long old =
          atomicAdd(reinterpret_cast<unsigned long long*>(a.seg_meta), (1ull << 32) | (unsigned long long)nt);
      SegInfo sg;
      sg.start = bk.start;
      sg.n = bk.n;
      sg.k = (uint32_t)bk.k;
      sg.low_bits = (uint32_t)bk.low_bits;
      sg.tile0 = (uint32_t)old;
      sg.src = (uint32_t)src;
      sg.pad1 = sg.pad2 = 0;
      a.segs[(uint32_t)(old >> 32)] = sg;
    }
    return;
  }
  const int res = sort_bucket_global(a, bk, s, src);
  __syncthreads();
  const uint32_t* keys = a.keys[res] + bk.start;
  const uint32_t* bags = a.vals[res] + bk.start;
  for (uint32_t w0 = 0; w0 < bk.n; w0 += kBktCap) reduce_window<DT, G, OPT>(a, u, bk, W, keys, bags, w0, res, s, part);
}

template <int DT, int G, int OPT>
__device__ inline void reduce_oversized(const GroupArgs& a, const UpdArgs& u, const Bucket& b, char* W,
                                        SortLds& s, SplitLds& sp, float* part) {
  const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
  // ---- candidates: long runs among the first kBktCap pairs
  if (tid < kCand) sp.cand[tid] = 0xFFFFFFFFu;
  if (tid < kNW * (kCand + 1)) (&sp.wcnt[0][0])[tid] = 0;
  {
    Bucket head = b;
    head.n = (uint32_t)kBktCap;
    sort_bucket_lds(a, head, s, 1);
    const uint32_t nruns = compact_heads_lds(s, kBktCap);
    uint32_t flags = 0, c = 0;
#pragma unroll
    for (int j = 0; j < kBktItems; ++j) {  // thread t owns runs [t*kBktItems, (t+1)*kBktItems): row order
      const uint32_t r = (uint32_t)(tid * kBktItems + j);
      if (r < nruns && s.heads[r + 1] - s.heads[r] >= (uint32_t)kCandMin) {
        flags |= 1u << j;
        ++c;
      }
    }
    uint32_t total;
    uint32_t pos = block_exclusive_scan<kThreads>(c, s.smem, &total);
#pragma unroll
    for (int j = 0; j < kBktItems; ++j)
      if (flags & (1u << j)) sp.cand[pos++] = s.skey[s.heads[tid * kBktItems + j]];
    if (tid == 0) sp.nc = total;
  }
  __syncthreads();
  const uint32_t nc = sp.nc;
  if (nc == 0) {  // uniform
    sort_reduce_large<DT, G, OPT>(a, u, b, W, 1, s, part);
    return;
  }
  uint32_t cd[kCand];
#pragma unroll
  for (int c = 0; c < kCand; ++c) cd[c] = sp.cand[c];
  const uint32_t* kin = a.keys[1] + b.start;
  const uint32_t* vin = a.vals[1] + b.start;
  // Both passes: wavefront w streams its own quarter [q0, q1) of the bucket, no barriers inside.
  const uint32_t span = (b.n + kNW * DLRM_WAVE - 1) / (kNW * DLRM_WAVE) * DLRM_WAVE;
  const uint32_t q0 = (uint32_t)w * span < b.n ? (uint32_t)w * span : b.n;
  const uint32_t q1 = q0 + span < b.n ? q0 + span : b.n;
  // ---- pass 1: pairs per (wavefront, class).  A wavefront's lanes mostly agree (the dominant
  // row): those that agree with the first valid lane are counted with one LDS atomic
  // (the next 8 steps of 64 pairs are in flight while the current 8 are processed)
  uint32_t kk[8];
  if (q0 < q1) {
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const uint32_t i = q0 + q * DLRM_WAVE + lane;
      kk[q] = kin[i < q1 ? i : q1 - 1];
    }
  }
  for (uint32_t i0 = q0; i0 < q1; i0 += DLRM_WAVE * 8) {
    uint32_t nk[8];
    if (i0 + DLRM_WAVE * 8 < q1) {  // uniform
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const uint32_t i = i0 + DLRM_WAVE * 8 + q * DLRM_WAVE + lane;
        nk[q] = kin[i < q1 ? i : q1 - 1];
      }
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const uint32_t i = i0 + q * DLRM_WAVE + lane;
      const bool valid = i < q1;
      const uint32_t cls = class_of(kk[q], cd);
      const unsigned long long vm = __ballot(valid);
      if (vm == 0ull) continue;  // wave-uniform
      const int first = __ffsll((long long)vm) - 1;
      const uint32_t c0 = (uint32_t)__builtin_amdgcn_readlane((int)cls, first);
      const unsigned long long same = __ballot(valid && cls == c0);
      if (lane == first) atomicAdd(&sp.wcnt[w][c0], (uint32_t)__popcll(same));
      if (valid && cls != c0) atomicAdd(&sp.wcnt[w][cls], 1u);
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) kk[q] = nk[q];
  }
  __syncthreads();
  if (tid <= kCand) {
    uint32_t tot = 0;
    for (int i = 0; i < kNW; ++i) tot += sp.wcnt[i][tid];
    sp.cnt[tid] = tot;
  }
  __syncthreads();
  if (tid == 0) {
    uint32_t run = 0;
    for (int c = 0; c <= kCand; ++c) {
      sp.cbase[c] = run;
      run += sp.cnt[c];
    }
    sp.cbase[kCand + 1] = run;
  }
  __syncthreads();
  if (tid <= kCand) {  // where wavefront i's first pair of the class goes
    uint32_t run = sp.cbase[tid];
    for (int i = 0; i < kNW; ++i) {
      sp.wbase[i][tid] = run;
      run += sp.wcnt[i][tid];
    }
  }
  __syncthreads();
  // ---- pass 2: stable partition by class into pair buffer 0.  Candidate lists keep only the
  // bags (plus the row id at their first position); the rest keeps (row, bag).  Within a step
  // of 64 pairs the lanes of one class rank themselves by ballot; the wavefront's running
  // destination per class lives in its own LDS row.
  uint32_t* kout = a.keys[0] + b.start;
  uint32_t* vout = a.vals[0] + b.start;
  const unsigned long long lt = (1ull << lane) - 1ull;
  uint32_t key[8], val[8];
  if (q0 < q1) {
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const uint32_t i = q0 + q * DLRM_WAVE + lane;
      key[q] = kin[i < q1 ? i : q1 - 1];
      val[q] = vin[i < q1 ? i : q1 - 1];
    }
  }
  for (uint32_t i0 = q0; i0 < q1; i0 += DLRM_WAVE * 8) {
    uint32_t nk[8], nv[8];
    if (i0 + DLRM_WAVE * 8 < q1) {  // uniform
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const uint32_t i = i0 + DLRM_WAVE * 8 + q * DLRM_WAVE + lane;
        nk[q] = kin[i < q1 ? i : q1 - 1];
        nv[q] = vin[i < q1 ? i : q1 - 1];
      }
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const uint32_t i = i0 + q * DLRM_WAVE + lane;
      const bool valid = i < q1;
      const uint32_t cls = class_of(key[q], cd);
      unsigned long long rem = __ballot(valid);
      uint32_t dst = 0;
      while (rem != 0ull) {  // wave-uniform: one round per class present in the step
        const int f = __ffsll((long long)rem) - 1;
        const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)cls, f);
        const unsigned long long m = __ballot(valid && cls == c);
        const uint32_t bs = sp.wbase[w][c];
        if (valid && cls == c) dst = bs + (uint32_t)__popcll(m & lt);
        if (lane == f) sp.wbase[w][c] = bs + (uint32_t)__popcll(m);
        rem &= ~m;
      }
      if (valid) {
        vout[dst] = val[q];
        if (cls == (uint32_t)kCand) kout[dst] = key[q];
      }
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      key[q] = nk[q];
      val[q] = nv[q];
    }
  }
  __syncthreads();
  if ((uint32_t)tid < nc) kout[sp.cbase[tid]] = sp.cand[tid];
  if ((uint32_t)tid <= nc) s.heads[tid] = sp.cbase[tid];
  __syncthreads();
  // ---- candidate lists are runs: short ones summed here, those above kHugeRun queued as hot rows
  {
    const uint32_t nlong = collect_long_runs(s, nc);
    reduce_runs<DT, G, OPT>(a, u, b, W, kout, vout, s.heads, 0u, nc, s.longs, nlong, 0, part);
  }
  // ---- the rest
  Bucket rest = b;
  rest.start = b.start + sp.cbase[kCand];
  rest.n = sp.cnt[kCand];
  __syncthreads();
  if (rest.n == 0) return;  // uniform
  if (rest.n > (uint32_t)kBktCap) {
    sort_reduce_large<DT, G, OPT>(a, u, rest, W, 0, s, part);
    return;
  }
  sort_bucket_lds(a, rest, s, 0);
  const uint32_t nruns = compact_heads_lds(s, (int)rest.n);
  const uint32_t nlong = collect_long_runs(s, nruns);
  reduce_runs<DT, G, OPT>(a, u, rest, W, s.skey, s.sval, s.heads, 0u, nruns, s.longs, nlong, 0, part);
}

template <int DT, int G, int OPT>
__global__ __launch_bounds__(kThreads, OPT == kAdagrad ? 3 : 4) void bucket_reduce_kernel(GroupArgs a, UpdArgs u) {
  __shared__ SortLds s;
  __shared__ SplitLds sp;
  __shared__ float part[kThreads * 4];
  uint32_t bid;
  bool oversized;
  if (!bucket_id_of_block(a, &bid, &oversized)) return;
  const Bucket b = bucket_of_block(a, bid);
  if (b.n == 0 || (!oversized && b.n > (uint32_t)kBktCap)) return;
  char* W = static_cast<char*>(u.tables[b.k]);
  if (b.n <= (uint32_t)kBktCap) {
    sort_bucket_lds(a, b, s);
    const uint32_t nruns = compact_heads_lds(s, (int)b.n);
    const uint32_t nlong = collect_long_runs(s, nruns);
    reduce_runs<DT, G, OPT>(a, u, b, W, s.skey, s.sval, s.heads, 0u, nruns, s.longs, nlong, 1, part);
    return;
  }
  if (b.low_bits == 0) {  // the bucket holds one row: a single run, already in position order
    if (threadIdx.x == 0) {
      s.heads[0] = 0;
      s.heads[1] = b.n;
    }
    __syncthreads();
    const uint32_t nlong = collect_long_runs(s, 1);
    reduce_runs<DT, G, OPT>(a, u, b, W, a.keys[1] + b.start, a.vals[1] + b.start, s.heads, 0u, 1, s.longs, nlong, 1,
                       part);
    return;
  }
  reduce_oversized<DT, G, OPT>(a, u, b, W, s, sp, part);
}

// --- 4c. oversized buckets ("segments") sorted by one workgroup per tile ------------------------
__device__ inline bool find_segment_tile(const GroupArgs& a, SegInfo* sg, uint32_t* t) {
  const uint32_t ntiles = a.seg_meta[0], nseg = a.seg_meta[1];
  if (blockIdx.x >= ntiles) return false;
  uint32_t lo = 0, hi = nseg;  // segs[lo].tile0 <= tile < segs[hi].tile0
  while (hi - lo > 1) {
    const uint32_t mid = (lo + hi) >> 1;
    if (a.segs[mid].tile0 <= blockIdx.x) lo = mid; else hi = mid;
  }
  *sg = a.segs[lo];
  *t = blockIdx.x - sg->tile0;
  return true;
}

// Every workgroup counts, per row of the segment, the pairs in the tiles before its own and in
// the whole segment (the segment's keys stream through L2), sorts its own tile in LDS, and
// writes each pair to  segment start + rows before + same row in earlier tiles + rank in tile:
// the segment ends up fully sorted by (row, position) in the other pair buffer.
__global__ __launch_bounds__(kThreads) void segment_sort_kernel(GroupArgs a) {
  __shared__ SortLds s;
  __shared__ uint32_t before[kSegKeys];
  __shared__ uint32_t base[kSegKeys];
  SegInfo sg;
  uint32_t t;
  if (!find_segment_tile(a, &sg, &t)) return;
  const int tid = threadIdx.x;
  const uint32_t nkeys = 1u << sg.low_bits, mask = nkeys - 1u;
  const uint32_t tstart = t * kBktCap;
  const uint32_t cnt = sg.n - tstart < (uint32_t)kBktCap ? sg.n - tstart : (uint32_t)kBktCap;
  for (uint32_t i = tid; i < nkeys; i += kThreads) {
    before[i] = 0;
    base[i] = 0;
  }
  __syncthreads();
  const uint32_t* kin = a.keys[sg.src] + sg.start;
  for (uint32_t i0 = 0; i0 < sg.n; i0 += kThreads * 8) {  // 8 loads in flight per thread
    uint32_t kk[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const uint32_t i = i0 + q * kThreads + tid;
      kk[q] = kin[i < sg.n ? i : sg.n - 1];
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      // a wavefront covers 64 consecutive positions, all on one side of tstart (a multiple of 64).
      // Segments are dominated by a few rows: the lanes that agree with the first valid lane
      // are counted with ONE LDS atomic instead of a 64-way conflict on the same counter.
      const uint32_t i = i0 + q * kThreads + tid;
      const bool valid = i < sg.n;
      uint32_t* ctr = i < tstart ? before : base;
      const uint32_t r = kk[q] & mask;
      const unsigned long long vm = __ballot(valid);
      if (vm == 0ull) continue;  // wave-uniform
      const int first = __ffsll((long long)vm) - 1;
      const uint32_t r0 = __shfl(r, first, DLRM_WAVE);
      const unsigned long long same = __ballot(valid && r == r0);
      if (lane_id() == first) atomicAdd(&ctr[r0], (uint32_t)__popcll(same));
      if (valid && r != r0) atomicAdd(&ctr[r], 1u);
    }
  }
  __syncthreads();
  {  // base[r] <- number of pairs of the segment with a smaller row (exclusive scan of the totals)
    const uint32_t per = (nkeys + kThreads - 1) / kThreads;
    uint32_t sum = 0;
    for (uint32_t j = 0; j < per; ++j) {
      const uint32_t r = tid * per + j;
      if (r < nkeys) sum += before[r] + base[r];
    }
    uint32_t all;
    uint32_t run = block_exclusive_scan<kThreads>(sum, s.smem, &all);
    for (uint32_t j = 0; j < per; ++j) {
      const uint32_t r = tid * per + j;
      if (r < nkeys) {
        const uint32_t c = before[r] + base[r];
        base[r] = run;
        run += c;
      }
    }
  }
  __syncthreads();
  Bucket tb;
  tb.k = (int)sg.k;
  tb.start = sg.start + tstart;
  tb.n = cnt;
  tb.low_bits = (int)sg.low_bits;
  sort_bucket_lds(a, tb, s, (int)sg.src);
  uint32_t* kout = a.keys[sg.src ^ 1u] + sg.start;
  uint32_t* vout = a.vals[sg.src ^ 1u] + sg.start;
  for (uint32_t p = tid; p < cnt; p += kThreads) {
    const uint32_t key = s.skey[p];
    uint32_t lo = 0, hi = p;  // first position of this key in the sorted tile
    while (lo < hi) {
      const uint32_t mid = (lo + hi) >> 1;
      if (s.skey[mid] < key) lo = mid + 1; else hi = mid;
    }
    const uint32_t r = key & mask;
    const uint32_t dst = base[r] + before[r] + (p - lo);
    kout[dst] = key;
    vout[dst] = s.sval[p];
  }
}

template <int DT, int G, int OPT>
__global__ __launch_bounds__(kThreads) void segment_reduce_kernel(GroupArgs a, UpdArgs u) {
  __shared__ SortLds s;
  __shared__ float part[kThreads * 4];
  SegInfo sg;
  uint32_t t;
  if (!find_segment_tile(a, &sg, &t)) return;
  Bucket b;
  b.k = (int)sg.k;
  b.start = sg.start;
  b.n = sg.n;
  b.low_bits = 0;
  char* W = static_cast<char*>(u.tables[b.k]);
  const int dst = (int)(sg.src ^ 1u);
  reduce_window<DT, G, OPT>(a, u, b, W, a.keys[dst] + sg.start, a.vals[dst] + sg.start, t * kBktCap, dst, s, part);
}

// --- 5. hot rows: runs too long for one workgroup -------------------------------------------------
// A hot row is looked up by a large share of the bags, so summing its run entry by entry would
// fetch nearly the whole gradient slice dS[:, k, :] once per hot row.  Instead workgroup (g, k)
// streams the gradient rows of bag group g of table k through LDS ONCE, tile by tile (the next
// tile travels in registers while the current one is consumed), and every wavefront adds, for
// each of its hot runs, the rows of the run's entries whose bag lies in the tile.  A run's bags
// ascend, so binary searches give its entry range per tile, and equal neighbours (a bag that
// looks the row up several times) are folded into one LDS read times a multiplicity.  Partial
// sums per (run, bag group) go to global memory; hot_finish_kernel adds them in group order.

// Entry e + slot of the 64 values the lanes hold in `v` (e: uniform).  Few slots: scalar lane
// reads and selects, no LDS round trip; many slots: a lane permute.
template <int S>
__device__ inline uint32_t lane_entry(uint32_t v, uint32_t e, int slot) {
  if constexpr (S <= 4) {
    uint32_t r = (uint32_t)__builtin_amdgcn_readlane((int)v, (int)(e & 63u));
#pragma unroll
    for (int sl = 1; sl < S; ++sl) {
      const uint32_t o = (uint32_t)__builtin_amdgcn_readlane((int)v, (int)((e + sl) & 63u));
      r = slot == sl ? o : r;
    }
    return r;
  } else {
    return (uint32_t)__shfl((int)v, (int)((e + (uint32_t)slot) & 63u), DLRM_WAVE);
  }
}

template <int DT, int G>
__global__ __launch_bounds__(kThreads) void hot_rows_kernel(GroupArgs a, UpdArgs u, int ngroups) {
  constexpr int S = DLRM_WAVE / G;
  constexpr int MR = kHotRunsPerWave;
  constexpr int NT = kHotTilesPerGroup;
  constexpr int HU = S <= 8 ? 8 : DLRM_WAVE / S;  // HU * S entries per round, never past the 64 held
  constexpr int NG = kThreads / G;                // gradient rows staged per pass of the workgroup
  constexpr int NP = kHotStagePasses;
  constexpr int TB = NG * NP;                     // bags per tile: TB * d <= kHotTileFloats
  constexpr int GB = TB * NT;                     // bags per workgroup
  __shared__ float tile[kHotTileFloats + kHotZeroRow];  // gradient rows of a bag tile, then a row of zeros
  __shared__ uint32_t cursor[kNW * MR][NT + 1];  // first entry of a run at or after every tile boundary
  __shared__ uint32_t rsrc[kNW * MR];            // pair buffer holding the run
  __shared__ uint32_t wsc[kNW][DLRM_WAVE];       // per wavefront: compacted (offset, multiplicity) words
  const int k = blockIdx.y, g = blockIdx.x;
  const uint32_t nruns = a.hot_cnt[k];
  if (nruns == 0) return;  // uniform
  const uint32_t base = hot_list_base(a, k);
  const int lane = lane_id(), w = wave_id(), tid = threadIdx.x;
  const int slot = lane / G, chunk = lane % G;
  const int grp = tid / G;
  const bool col_ok = chunk * 4 < u.d;
  const int cchunk = col_ok ? chunk : 0;  // lanes past the last column shadow column group 0, never store
  const unsigned long long lt = (1ull << lane) - 1ull;
  const int bag_lo = g * GB;
  const int bag_hi = bag_lo + GB < a.B ? bag_lo + GB : a.B;
  const float* gk = u.dS + (int64_t)k * u.stride_k + cchunk * 4;
  for (int i = tid; i < kHotZeroRow; i += kThreads) tile[kHotTileFloats + i] = 0.0f;
  for (uint32_t r0 = 0; r0 < nruns; r0 += kNW * MR) {  // uniform
    __syncthreads();
    for (int task = tid; task < kNW * MR * (NT + 1); task += kThreads) {
      const int rl = task / (NT + 1), tb = task - rl * (NT + 1);
      const uint32_t r = r0 + (uint32_t)rl;
      uint32_t c = 0;
      if (r < nruns) {
        const HugeRun hr = a.huge_runs[base + r];
        const uint32_t* bags = (hr.src ? a.vals[1] : a.vals[0]) + hr.start;
        const int bnd = bag_lo + tb * TB;
        const uint32_t bound = (uint32_t)(bnd < bag_hi ? bnd : bag_hi);
        uint32_t lo = 0, hi = hr.len;
        while (lo < hi) {
          const uint32_t mid = (lo + hi) >> 1;
          if (bags[mid] < bound) lo = mid + 1; else hi = mid;
        }
        c = hr.start + lo;
        if (tb == 0) rsrc[rl] = hr.src;
      }
      cursor[rl][tb] = c;
    }
    __syncthreads();
    const uint32_t* bags[MR];
    f32x4 acc[MR];
#pragma unroll
    for (int i = 0; i < MR; ++i) {
      const int rl = w + kNW * i;
      acc[i] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
      bags[i] = (r0 + (uint32_t)rl < nruns && rsrc[rl]) ? a.vals[1] : a.vals[0];
    }
    // staging registers: row p*NG + grp of a tile, this lane's 4 columns (rows past the tile's
    // end repeat its last row and are never stored)
    f32x4 stage[NP];
    {
      const int nb = bag_hi - bag_lo < TB ? bag_hi - bag_lo : TB;
#pragma unroll
      for (int p = 0; p < NP; ++p) {
        const int bb = p * NG + grp < nb ? p * NG + grp : nb - 1;
        stage[p] = loadf4(gk + (int64_t)(bag_lo + bb) * u.stride_b);
      }
    }
    int t = 0;
    for (int tb0 = bag_lo; tb0 < bag_hi; tb0 += TB, ++t) {  // uniform
      const int nb = bag_hi - tb0 < TB ? bag_hi - tb0 : TB;
      // the first 64 bags of every run of this wave are requested before the tile is stored
      uint32_t first[MR];
#pragma unroll
      for (int i = 0; i < MR; ++i) {
        const uint32_t c0 = cursor[w + kNW * i][t], c1 = cursor[w + kNW * i][t + 1];
        first[i] = 0;
        if (c0 + (uint32_t)lane < c1) first[i] = bags[i][c0 + lane];
      }
      __syncthreads();  // the previous tile has been consumed
#pragma unroll
      for (int p = 0; p < NP; ++p) {
        const int bb = p * NG + grp;
        if (bb < nb && col_ok) storef4(tile + bb * u.d + chunk * 4, stage[p]);
      }
      __syncthreads();
      if (tb0 + TB < bag_hi) {  // uniform: the next tile travels while this one is summed
        const int nn = bag_hi - (tb0 + TB) < TB ? bag_hi - (tb0 + TB) : TB;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
          const int bb = p * NG + grp < nn ? p * NG + grp : nn - 1;
          stage[p] = loadf4(gk + (int64_t)(tb0 + TB + bb) * u.stride_b);
        }
      }
#pragma unroll
      for (int i = 0; i < MR; ++i) {
        // the cursors are the same in every lane: scalar loop control
        const uint32_t c0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)cursor[w + kNW * i][t]);
        const uint32_t c1 = (uint32_t)__builtin_amdgcn_readfirstlane((int)cursor[w + kNW * i][t + 1]);
        uint32_t cur = first[i];
        for (uint32_t e0 = c0; e0 < c1; e0 += DLRM_WAVE) {
          uint32_t nxt = 0;  // the next 64 bags travel while these are summed
          if (e0 + DLRM_WAVE + (uint32_t)lane < c1) nxt = bags[i][e0 + DLRM_WAVE + lane];
          const uint32_t cnt = c1 - e0 < (uint32_t)DLRM_WAVE ? c1 - e0 : (uint32_t)DLRM_WAVE;
          // fold equal neighbours: the first entry of each distinct bag carries how many follow
          const uint32_t prev = (uint32_t)__shfl_up((int)cur, 1, DLRM_WAVE);
          const bool head = (uint32_t)lane < cnt && (lane == 0 || cur != prev);
          const unsigned long long hm = __ballot(head);
          const uint32_t nh = (uint32_t)__popcll(hm);
          const unsigned long long rest = (hm >> lane) >> 1;
          const uint32_t nextp = rest ? (uint32_t)lane + (uint32_t)__ffsll((long long)rest) : cnt;
          // LDS offset of the bag's gradient row (< 2^16) | multiplicity << 16
          if (head) wsc[w][__popcll(hm & lt)] = ((nextp - (uint32_t)lane) << 16) | ((cur - (uint32_t)tb0) * (uint32_t)u.d);
          uint32_t mine = wsc[w][lane];
          mine = (uint32_t)lane < nh ? mine : (uint32_t)kHotTileFloats;  // the row of zeros, zero times
          for (uint32_t e = 0; e < nh; e += HU * S) {
            f32x4 v[HU];
            float m[HU];
#pragma unroll
            for (int q = 0; q < HU; ++q) {  // HU independent LDS reads in flight
              const uint32_t pk = lane_entry<S>(mine, e + (uint32_t)(q * S), slot);
              v[q] = loadf4(tile + (pk & 0xFFFFu) + cchunk * 4);
              m[q] = (float)(pk >> 16);
            }
#pragma unroll
            for (int q = 0; q < HU; ++q) {
              acc[i].x = fmaf(m[q], v[q].x, acc[i].x);
              acc[i].y = fmaf(m[q], v[q].y, acc[i].y);
              acc[i].z = fmaf(m[q], v[q].z, acc[i].z);
              acc[i].w = fmaf(m[q], v[q].w, acc[i].w);
            }
          }
          cur = nxt;
        }
      }
    }
#pragma unroll
    for (int i = 0; i < MR; ++i) {
      const uint32_t r = r0 + w + kNW * i;
      if (r >= nruns) continue;  // wave-uniform
      f32x4 tot = acc[i];
#pragma unroll
      for (int o = G; o < DLRM_WAVE; o <<= 1) {
        tot.x += __shfl_xor(tot.x, o, DLRM_WAVE);
        tot.y += __shfl_xor(tot.y, o, DLRM_WAVE);
        tot.z += __shfl_xor(tot.z, o, DLRM_WAVE);
        tot.w += __shfl_xor(tot.w, o, DLRM_WAVE);
      }
      float* part = a.huge_part + ((size_t)(base + r) * ngroups) * u.d;
      if (slot == 0 && col_ok) storef4(part + (size_t)g * u.d + chunk * 4, tot);
    }
  }
}

// A lane group per hot run adds the run's partial sums in bag-group order and updates the row.
// A launch of its own: the kernel boundary orders it after every partial, at no fence.
template <int DT, int G, int OPT>
__global__ __launch_bounds__(kThreads) void hot_finish_kernel(GroupArgs a, UpdArgs u, int ngroups) {
  constexpr int S = DLRM_WAVE / G;
  const int k = blockIdx.y;
  const uint32_t nruns = a.hot_cnt[k];
  if (nruns == 0) return;
  const uint32_t base = hot_list_base(a, k);
  const int lane = lane_id();
  const int chunk = lane % G;
  if (chunk * 4 >= u.d) return;
  char* W = static_cast<char*>(u.tables[k]);
  float* H = state_base<OPT>(u, k);
  for (uint32_t r = (blockIdx.x * kNW + wave_id()) * S + lane / G; r < nruns; r += gridDim.x * kNW * S) {
    const float* part = a.huge_part + ((size_t)(base + r) * ngroups) * u.d + chunk * 4;
    f32x4 sum = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int g0 = 0; g0 < ngroups; g0 += 8) {
      f32x4 v[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) v[q] = loadf4(part + (size_t)(g0 + q < ngroups ? g0 + q : g0) * u.d);
#pragma unroll
      for (int q = 0; q < 8; ++q)
        if (g0 + q < ngroups) sum += v[q];
    }
    row_update<DT, OPT>(W, H, u, a.huge_runs[base + r].row, chunk, sum);
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
  const uint32_t bag = (blockIdx.x * (blockDim.x >> 6) + wave_id()) * S + slot;
  if (bag >= (uint32_t)a.K * (uint32_t)a.B || chunk * 4 >= a.d) return;
  const int k = (int)(bag / (uint32_t)a.B), b = (int)(bag - (uint32_t)k * (uint32_t)a.B);
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
  uint32_t pos = base + block_exclusive_scan<kThreads>(cnt, smem, &total);
#pragma unroll
  for (int j = 0; j < kItems; ++j) {
    if (flags & (1u << j)) {
      a.seg_start[pos] = (uint32_t)(ti.start + threadIdx.x * kItems + j);
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

// ---------------------------------------------------------------------------
int check_batch(const dlrm_sparse_batch* s);  // util.hip

static void fill_group_args(GroupArgs& g, const dlrm_sparse_batch* s, const WsLayout& L, void* ws) {
  char* base = static_cast<char*>(ws);
  g.indices = s->indices;
  g.offsets = s->offsets;
  g.tbl_off = s->tbl_off;
  g.rows = s->rows;
  g.K = s->K;
  g.B = s->B;
  g.nt_max = (int32_t)L.nt_max;
  // partition digit: one workgroup per bucket, so aim at >= ~1536 buckets when the batch is
  // large enough, with 128..1024 pairs per bucket (measured on the 8 x 1M x 64 multi-hot batch:
  // 800 pairs per bucket beat 200 by 8%); never more digits than the row ids have
  double target = (double)s->nnz_total / 1536.0;
  if (target < 128.0) target = 128.0;
  if (target > 1024.0) target = 1024.0;
  const double per_table = (double)s->nnz_total / (double)s->K;
  int tb = 0;
  while (tb < kMaxTopBits && per_table / (double)(1 << tb) > target) ++tb;
  const int kb = ilog2_ceil(s->max_rows);
  if (tb > kb) tb = kb;
  g.top_bits = tb;
  g.fused_scan = L.nt_max <= kFusedScanMaxTiles ? 1 : 0;
  g.no_tail = s->nnz_total <= kSmallBatch ? 1 : 0;
  for (int i = 0; i < 2; ++i) {
    g.keys[i] = reinterpret_cast<uint32_t*>(base + L.keys[i]);
    g.vals[i] = reinterpret_cast<uint32_t*>(base + L.vals[i]);
  }
  g.hist = reinterpret_cast<uint32_t*>(base + L.hist);
  g.bucket_start = reinterpret_cast<uint32_t*>(base + L.bucket_start);
  g.tile_heads = reinterpret_cast<uint32_t*>(base + L.tile_heads);
  g.seg_start = reinterpret_cast<uint32_t*>(base + L.seg_start);
  g.seg_tbl = reinterpret_cast<uint32_t*>(base + L.seg_tbl);
  g.n_seg = reinterpret_cast<uint32_t*>(base + L.n_seg);
  g.hot_cnt = reinterpret_cast<uint32_t*>(base + L.hot_cnt);
  g.over_cnt = reinterpret_cast<uint32_t*>(base + L.huge_ctr + 8);
  g.over_list = reinterpret_cast<uint32_t*>(base + L.over_list);
  g.segs = reinterpret_cast<SegInfo*>(base + L.segs);
  g.seg_meta = reinterpret_cast<uint32_t*>(base + L.seg_meta);
  {
    const int64_t nbk = (int64_t)s->K << tb, cap = s->nnz_total / kBktCap + 1;
    g.max_over = (int32_t)(nbk < cap ? nbk : cap);
    g.seg_tiles_max = (int32_t)(s->nnz_total / kBktCap + g.max_over);
  }
  g.huge_runs = reinterpret_cast<HugeRun*>(base + L.huge_runs);
  g.huge_part = reinterpret_cast<float*>(base + L.huge_part);
}

// Enqueues steps 1-3: afterwards keys[1]/vals[1] hold the pairs partitioned into buckets and
// bucket_start the bucket boundaries.
static int enqueue_partition(const dlrm_sparse_batch* s, const GroupArgs& g, hipStream_t st) {
  hipLaunchKernelGGL(bucket_hist_kernel, dim3(g.nt_max), dim3(kThreads), 0, st, g);
  DLRM_CHECK_LAUNCH();
  if (!g.fused_scan) {
    hipLaunchKernelGGL(bucket_scan_kernel, dim3(s->K), dim3(1024), 0, st, g);
    DLRM_CHECK_LAUNCH();
  }
  hipLaunchKernelGGL(bucket_scatter_kernel, dim3(g.nt_max), dim3(kThreads), 0, st, g);
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}

// optional pair of caller-owned HIP events recorded around the bucket_reduce launch
static hipEvent_t g_ev_start = nullptr, g_ev_stop = nullptr;

template <int DT, int G, int OPT>
static int launch_reduce(const GroupArgs& g, const UpdArgs& u, int K, hipStream_t st) {
  const unsigned blocks = ((unsigned)K << g.top_bits) + (unsigned)g.max_over;
  if (g_ev_start && hipEventRecord(g_ev_start, st) != hipSuccess) return DLRM_ERR_HIP;
  hipLaunchKernelGGL((bucket_reduce_kernel<DT, G, OPT>), dim3(blocks), dim3(kThreads), 0, st, g, u);
  DLRM_CHECK_LAUNCH();
  if (g_ev_stop && hipEventRecord(g_ev_stop, st) != hipSuccess) return DLRM_ERR_HIP;
  if (g.no_tail) return DLRM_OK;
  const unsigned seg_tiles = (unsigned)(g.seg_tiles_max);
  hipLaunchKernelGGL(segment_sort_kernel, dim3(seg_tiles), dim3(kThreads), 0, st, g);
  DLRM_CHECK_LAUNCH();
  hipLaunchKernelGGL((segment_reduce_kernel<DT, G, OPT>), dim3(seg_tiles), dim3(kThreads), 0, st, g, u);
  DLRM_CHECK_LAUNCH();
  const int ng = hot_groups(g.B, u.d);
  hipLaunchKernelGGL((hot_rows_kernel<DT, G>), dim3(ng, K), dim3(kThreads), 0, st, g, u, ng);
  DLRM_CHECK_LAUNCH();
  hipLaunchKernelGGL((hot_finish_kernel<DT, G, OPT>), dim3(4, K), dim3(kThreads), 0, st, g, u, ng);
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}

template <int DT, int OPT>
static int dispatch_reduce(const GroupArgs& g, const UpdArgs& u, int G, int K, hipStream_t st) {
  switch (G) {
    case 1: return launch_reduce<DT, 1, OPT>(g, u, K, st);
    case 2: return launch_reduce<DT, 2, OPT>(g, u, K, st);
    case 4: return launch_reduce<DT, 4, OPT>(g, u, K, st);
    case 8: return launch_reduce<DT, 8, OPT>(g, u, K, st);
    case 16: return launch_reduce<DT, 16, OPT>(g, u, K, st);
    case 32: return launch_reduce<DT, 32, OPT>(g, u, K, st);
    case 64: return launch_reduce<DT, 64, OPT>(g, u, K, st);
  }
  return DLRM_ERR_BAD_SHAPE;
}

static int check_ws(const dlrm_sparse_batch* s, void* ws, size_t bytes, WsLayout* L);

// The sort path behind both optimizers' entry points: grouping (unless prepared), then the
// reduce launches with the row update OPT.
template <int OPT>
static int run_sort_path(const dlrm_sparse_batch* s, const UpdArgs& u, void* workspace, size_t workspace_bytes,
                         bool prepared, hipStream_t hs) {
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
  switch (s->table_dtype) {
    case DLRM_F32: return dispatch_reduce<DLRM_F32, OPT>(g, u, G, s->K, hs);
    case DLRM_F16: return dispatch_reduce<DLRM_F16, OPT>(g, u, G, s->K, hs);
    case DLRM_BF16: return dispatch_reduce<DLRM_BF16, OPT>(g, u, G, s->K, hs);
  }
  return DLRM_ERR_BAD_DTYPE;
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
  *L = ws_layout(s->K, s->B, s->d, s->nnz_total);
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255) || bytes < L->total) return DLRM_ERR_WORKSPACE;
  if (L->nt_max > 0x7FFFFFFF || ((int64_t)s->K << kMaxTopBits) > 0x7FFFFFFF) return DLRM_ERR_BAD_SHAPE;
  return DLRM_OK;
}

}  // namespace dlrm

using namespace dlrm;

extern "C" int32_t dlrm_profile_reduce_kernel(void* ev_start, void* ev_stop) {
  if ((ev_start == nullptr) != (ev_stop == nullptr)) return DLRM_ERR_NULL;
  g_ev_start = static_cast<hipEvent_t>(ev_start);
  g_ev_stop = static_cast<hipEvent_t>(ev_stop);
  return DLRM_OK;
}

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
  int st = check_batch(s);
  if (st != DLRM_OK) return st;
  if (!dS) return DLRM_ERR_NULL;
  if ((s->d & 3) || stride_k < s->d || (stride_k & 3) || (stride_b & 3) || stride_b < 0)
    return DLRM_ERR_BAD_SHAPE;
  if (reinterpret_cast<uintptr_t>(dS) & 15) return DLRM_ERR_BAD_SHAPE;
  if (algo != DLRM_BWD_AUTO && algo != DLRM_BWD_SORT && algo != DLRM_BWD_ATOMIC && algo != DLRM_BWD_SORT_PREPARED)
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

  UpdArgs u;
  u.tables = s->tables;
  u.state = nullptr;
  u.dS = dS;
  u.stride_b = stride_b;
  u.stride_k = stride_k;
  u.lr = lr;
  u.eps = 0.0f;
  u.d = s->d;
  return run_sort_path<kSgd>(s, u, workspace, workspace_bytes, algo == DLRM_BWD_SORT_PREPARED, hs);
}

extern "C" int32_t dlrm_emb_bag_bwd_adagrad(const dlrm_sparse_batch* s, void* const* state, const float* dS,
                                            int64_t stride_b, int64_t stride_k, float lr, float eps,
                                            void* workspace, size_t workspace_bytes, int32_t algo,
                                            void* stream) {
  int st = check_batch(s);
  if (st != DLRM_OK) return st;
  if (!dS || !state) return DLRM_ERR_NULL;
  if ((s->d & 3) || stride_k < s->d || (stride_k & 3) || (stride_b & 3) || stride_b < 0)
    return DLRM_ERR_BAD_SHAPE;
  if (reinterpret_cast<uintptr_t>(dS) & 15) return DLRM_ERR_BAD_SHAPE;
  if (!(eps > 0.0f)) return DLRM_ERR_BAD_SHAPE;  // h = 0 and g = 0 would divide 0 by 0
  if (algo != DLRM_BWD_AUTO && algo != DLRM_BWD_SORT && algo != DLRM_BWD_SORT_PREPARED) return DLRM_ERR_BAD_ALGO;
  UpdArgs u;
  u.tables = s->tables;
  u.state = state;
  u.dS = dS;
  u.stride_b = stride_b;
  u.stride_k = stride_k;
  u.lr = lr;
  u.eps = eps;
  u.d = s->d;
  return run_sort_path<kAdagrad>(s, u, workspace, workspace_bytes, algo == DLRM_BWD_SORT_PREPARED,
                                 static_cast<hipStream_t>(stream));
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
  st = enqueue_partition(s, g, hs);
  if (st != DLRM_OK) return st;
  hipLaunchKernelGGL(bucket_sort_only_kernel, dim3((unsigned)s->K << g.top_bits), dim3(kThreads), 0, hs, g);
  DLRM_CHECK_LAUNCH();
  hipLaunchKernelGGL(segment_sort_kernel, dim3((unsigned)g.seg_tiles_max), dim3(kThreads), 0, hs, g);
  DLRM_CHECK_LAUNCH();
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
