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
//                       (row, bag) pairs to their bucket, stably, staged through LDS.
//                       Weighted batches (Eq. (2) with its weights) move (row, position) pairs
//                       instead and keep (bag, weight) records in a side array in the original
//                       order: nothing downstream looks inside the second member until a gradient
//                       row is fetched, where bag and weight are looked up by position.
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
//      hot_rows_dense : the same for tables with many hot rows, as a dense contraction on the
//                       matrix cores (multiplicity matrix [bag][hot row] times gradient tile);
//      hot_finish     : adds a hot row's partial sums in bag-group order and updates the row.
// Steps 1-3 read indices and offsets only; dlrm_emb_bag_bwd_prepare enqueues just them.
// ATOMIC path (fp32 tables): a lane group per bag adds -lr*dS[b,k,:] to every row of the bag
// with hardware fp32 atomics; no workspace, one launch.  Measured 6x slower than SORT on the
// 8 x 1M x 64 multi-hot workload, so AUTO always takes SORT.
//
// Files: bwd_common.h (this: constants, workspace, arguments, shared device helpers),
// bwd_partition.hip (steps 1-3), bwd_sort.h (bucket and segment sorts), bwd_reduce.h (steps 4, 4a and
// the row updates; instantiated per optimizer in bwd_reduce_sgd.hip / bwd_reduce_adagrad.hip),
// bwd_tail.hip (segment sort, hot rows), bwd_export.hip (grouping exported for tests),
// emb_bwd.hip (entry points, ATOMIC path).
#pragma once
#include "common.h"

namespace dlrm {

constexpr int kThreads = 256;
constexpr int kNW = kThreads / DLRM_WAVE;       // wavefronts per workgroup
constexpr int kItems = 16;                      // positions per thread in a (large) partition tile
constexpr int kTile = kThreads * kItems;        // 4096 positions per tile; batches below kSmallTileNnz lookups
constexpr int kSmallItems = 4;                  // use tiles of 1024: four times the workgroups, a quarter of the
constexpr int64_t kSmallTileNnz = 1 << 20;      // dependent steps each (the partition of a small batch is a chain
                                                // of latencies on a mostly idle machine)
// log2 of the partition tile for a batch of nnz lookups (host and device agree through GroupArgs::tile_shift)
inline int tile_shift_for(int64_t nnz) { return nnz < kSmallTileNnz ? 10 : 12; }
constexpr int kMaxTopBits = 10;                 // partition digit: up to 1024 buckets per table
constexpr int kMaxBuckets = 1 << kMaxTopBits;
constexpr int kDPT = kMaxBuckets / kThreads;    // partition digits owned by one thread
constexpr int kSortBits = 8;                    // digit of the bucket-local LSD passes
constexpr int kSortBuckets = 1 << kSortBits;
constexpr int kBktItems = 8;                    // positions per thread in a bucket-sort tile
constexpr int kBktCap = kThreads * kBktItems;   // 2048: buckets up to this size are sorted in LDS
constexpr int kLongRun = 32;                    // longer runs are summed by the whole workgroup
constexpr int kBigMin = 256;                     // smallest bucket size that can count as heavy (see GroupArgs::big)
constexpr int kLongRunMin = 16;                 // ... 16 where a workgroup has >= 32 lane groups
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
constexpr int kDenseFrom = 8;                   // tables with at least this many hot rows (unweighted batch)
                                                // have them summed as a dense contraction on the matrix cores
// Route counters of an update, kept behind the two segment counters in seg_meta (zeroed by the
// partition, read back by dlrm_emb_bag_bwd_route_counts): how often each rarely taken route ran.
constexpr int kRouteSplit = 4;                  // oversized buckets that split off dominant rows
constexpr int kRouteGlobalSort = 5;             // lists sorted by one workgroup through global memory
constexpr int kRouteOneRow = 6;                 // oversized buckets holding a single row
constexpr int kRouteHugeInPlace = 7;            // runs above kHugeRun summed by one workgroup (no tail launches)

// ---------------------------------------------------------------------------
// Workspace layout (all offsets 256-byte aligned)
struct WsLayout {
  size_t keys[2], vals[2];   // uint32[nnz] ping-pong: row ids / bag ids
  size_t hist;               // uint32[kMaxBuckets * nt_max]: per-tile digit counts / offsets
  size_t bucket_start;       // uint32[K * kMaxBuckets + 1]
  size_t tile_heads;         // uint32[nt_max + 1]   (export only)
  size_t seg_start;          // uint32[nnz + 1]      (export only; a weighted update keeps its nnz
  size_t seg_tbl;            // uint32[nnz]           8-byte PosEntry records across these two)
  size_t n_seg;              // uint32[4]            (export only)
  size_t huge_ctr;           // uint32[4]: [2] = listed (heavy) buckets, [3] = oversized buckets among them
  size_t hot_cnt;            // uint32[K]: queued hot runs per table
  size_t over_list;          // uint32[nnz / kBigMin + 1]: heavy buckets, handed to the first workgroups
  size_t segs;               // SegInfo[nnz / kBktCap + 2]: those of them sorted by many workgroups
  size_t seg_meta;           // uint32[8]: segment tiles, segments, -, -, route counters (kRoute*)
  size_t huge_runs;          // HugeRun[nnz / kHugeRun + K]: table k's list starts at sum_{j<k}(nnz_j/kHugeRun + 1)
  size_t huge_part;          // float[max_runs * bag groups * d]
  size_t total;
  int64_t nt_max;            // upper bound on the number of tiles
  int64_t max_huge;          // upper bound on the number of queued runs
};

// Weighted batches: what one lookup contributes besides its row, found by its position with one
// 8-byte load.
struct alignas(8) PosEntry {
  uint32_t bag;
  float w;  // the weight a of Eq. (2)
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

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// bags whose gradient rows one hot-row workgroup streams: kHotTilesPerGroup tiles of
// kHotStagePasses passes of kThreads / G rows (G lanes per row)
inline int hot_group_bags(int d) { return kThreads / pow2_ceil(d / 4) * kHotStagePasses * kHotTilesPerGroup; }
inline int hot_groups(int B, int d) {
  const int gb = hot_group_bags(d);
  return (B + gb - 1) / gb;
}

inline WsLayout ws_layout(int32_t K, int32_t B, int32_t d, int64_t nnz) {
  WsLayout L;
  size_t o = 0;
  const size_t n = (size_t)(nnz > 0 ? nnz : 1);
  L.nt_max = (nnz >> tile_shift_for(nnz)) + K;
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
  L.over_list = o;    o = align256(o + ((size_t)(nnz / kBigMin) + 1) * 4);
  L.segs = o;         o = align256(o + ((size_t)(nnz / kBktCap) + 2) * sizeof(SegInfo));
  L.seg_meta = o;     o = align256(o + 32);
  L.huge_runs = o;    o = align256(o + (size_t)L.max_huge * sizeof(HugeRun));
  L.huge_part = o;    o = align256(o + (size_t)L.max_huge * (size_t)hot_groups(B, d) * (size_t)d * 4);
  L.total = o;
  return L;
}

// ---------------------------------------------------------------------------
struct GroupArgs {            // everything the grouping kernels need
  const void* indices;        // int64 or int32 (idx32)
  const int64_t* offsets;
  const int64_t* tbl_off;
  const int64_t* rows;
  int32_t idx32;
  const float* weights;       // NULL, or the weight of every lookup (parallel to indices)
  PosEntry* pos_entry;        // weighted batches: bag and weight of every position, in the original order
  int32_t K, B;
  int32_t nt_max;
  int32_t tile_shift;         // log2 of the positions per partition tile (10 or 12)
  int32_t top_bits;           // bits of the partition digit (0..kMaxTopBits)
  int32_t by_die;             // buckets dealt to the dies by table (bucket_id_of_block)
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
  uint32_t* list_cnt;         // heavy buckets listed by the partition (more than `big` pairs)
  uint32_t* over_cnt;         // those of them with more than kBktCap pairs (oversized)
  uint32_t* over_list;
  int32_t max_over;           // workgroups reserved at the front of the bucket grid for the listed buckets
  uint32_t big;               // a bucket with more pairs is heavy: 4 x the mean bucket, within [kBigMin, kBktCap]
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
  int count;       // items in the tile (1 .. tile size)
  int64_t tbl_start;
  int total_tiles; // tiles of all tables
};

// Every workgroup rebuilds the tile map from tbl_off (K is small): tables own
// ceil(nnz_k / tile) consecutive tiles.  All threads must call this (it synchronises).
__device__ inline bool find_tile(const GroupArgs& a, int tile, TileInfo& ti, uint32_t* smem) {
  __shared__ int res[4];
  const int64_t tsize = (int64_t)1 << a.tile_shift;
  if (threadIdx.x == 0) res[0] = -1;
  uint32_t carry = 0;
  for (int k0 = 0; k0 < a.K; k0 += kThreads) {
    const int k = k0 + threadIdx.x;
    uint32_t nt = 0;
    if (k < a.K) nt = (uint32_t)((a.tbl_off[k + 1] - a.tbl_off[k] + tsize - 1) >> a.tile_shift);
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
  ti.start = ti.tbl_start + ((int64_t)ti.t << a.tile_shift);
  const int64_t rem = a.tbl_off[ti.k + 1] - ti.start;
  ti.count = (int)(rem < tsize ? rem : tsize);
  return true;
}

// --- shared by steps 3 and 4: stable ranking of a tile by a digit ---------------------
// Wave w of the workgroup owns the contiguous positions [w*64*items, (w+1)*64*items) of
// the tile, item j < items of lane l being position w*64*items + j*64 + l (items <= ITEMS is
// workgroup-uniform: a tile that is not full is dealt evenly to the wavefronts, and nobody ranks
// items that do not exist).  Ranks inside a wave come from ballot matching; per-wave digit counters
// in LDS give the order across waves.
// On return rnk[j] is the item's rank among the items of its wave with the same digit that
// precede it, and wcnt[w][digit] the wave's count.  wcnt must be zero on entry.
template <int ITEMS, int NBK>
__device__ inline void rank_items(const uint32_t* dg, const bool* ok, int bits,
                                  uint32_t (*wcnt)[NBK], uint32_t* rnk, int items = ITEMS) {
  const int lane = lane_id(), w = wave_id();
  const unsigned long long lt = (1ull << lane) - 1ull;
#pragma unroll
  for (int j = 0; j < ITEMS; ++j) {
    if (j >= items) break;  // uniform
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

struct Bucket {
  int k;
  uint32_t start, n;   // global position of the bucket's first pair, pairs in the bucket
  int low_bits;        // row-id bits below the partition digit
};

// Heavy buckets (hot rows: long runs, or more pairs than the LDS sort holds) take much longer than
// the rest: they are listed during the partition and handed to the FIRST workgroups of the grid, so
// that they start at once and run beside everything else; the workgroup a heavy bucket would get by
// its index leaves it alone.  Returns false if this workgroup has nothing to do.
__device__ inline bool bucket_id_of_block(const GroupArgs& a, uint32_t* id, bool* listed) {
  if (blockIdx.x < (uint32_t)a.max_over) {
    if (blockIdx.x >= *a.list_cnt) return false;
    *id = a.over_list[blockIdx.x];
    *listed = true;
    return true;
  }
  // Workgroups go to the eight accelerator dies round-robin by their index, and every die has an L2 of
  // its own.  The gradient rows a bucket gathers belong to its table alone, so with large gradient
  // slices (by_die) a die works through whole tables (die x: tables x, x + 8, ...) and its L2 holds one
  // table's slice at a time, not an eighth of the buckets of every table.  Tables past the last
  // multiple of 8 keep the plain order.
  const uint32_t j = blockIdx.x - (uint32_t)a.max_over;
  const uint32_t k8 = (uint32_t)a.K & ~7u;
  if (a.by_die && j < (k8 << a.top_bits)) {
    const uint32_t die = blockIdx.x & 7u, q = j >> 3;
    *id = ((((q >> a.top_bits) << 3) + die) << a.top_bits) | (q & ((1u << a.top_bits) - 1u));
  } else {
    *id = j;
  }
  *listed = false;
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
    return load16_stream(p);
  } else {
    const u32x2 b = load8_stream(p);
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
    store16_stream(p, u32x4{f2u(x.x), f2u(x.y), f2u(x.z), f2u(x.w)});
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
    store8_stream(p, b);
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
  if constexpr (OPT == kAdagrad) {
    const u32x4 hb = load16_stream(r.h);
    v.h = f32x4{u2f(hb.x), u2f(hb.y), u2f(hb.z), u2f(hb.w)};
  }
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
    store16_stream(r.h, u32x4{f2u(h.x), f2u(h.y), f2u(h.z), f2u(h.w)});
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


// ---------------------------------------------------------------------------
int check_batch(const dlrm_sparse_batch* s);  // util.hip

inline void fill_group_args(GroupArgs& g, const dlrm_sparse_batch* s, const WsLayout& L, void* ws) {
  char* base = static_cast<char*>(ws);
  g.indices = s->indices;
  g.idx32 = s->index_dtype == DLRM_I32;
  g.offsets = s->offsets;
  g.tbl_off = s->tbl_off;
  g.rows = s->rows;
  g.weights = s->weights;
  g.K = s->K;
  g.B = s->B;
  g.nt_max = (int32_t)L.nt_max;
  g.tile_shift = tile_shift_for(s->nnz_total);
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
  // Only for slices well above a die's 4 MB of L2 (measured: the hot-row workload's 8.4 MB slices -3.5 %
  // time and -21 % fetched bytes; 0.5 MB slices +8 % time), because a die then has whole tables and tables
  // differ in work: with 4 MB slices and tables of 100 to 10 M rows the kernel lost 15 %.
  g.by_die = (int64_t)s->B * s->d * 4 >= (6 << 20) ? 1 : 0;
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
  // the two export arrays, idle during an update and adjacent in the layout, hold the nnz records
  g.pos_entry = reinterpret_cast<PosEntry*>(base + L.seg_start);
  g.seg_tbl = reinterpret_cast<uint32_t*>(base + L.seg_tbl);
  g.n_seg = reinterpret_cast<uint32_t*>(base + L.n_seg);
  g.hot_cnt = reinterpret_cast<uint32_t*>(base + L.hot_cnt);
  g.list_cnt = reinterpret_cast<uint32_t*>(base + L.huge_ctr + 8);
  g.over_cnt = reinterpret_cast<uint32_t*>(base + L.huge_ctr + 12);
  g.over_list = reinterpret_cast<uint32_t*>(base + L.over_list);
  g.segs = reinterpret_cast<SegInfo*>(base + L.segs);
  g.seg_meta = reinterpret_cast<uint32_t*>(base + L.seg_meta);
  {
    const int64_t nbk = (int64_t)s->K << tb;
    int64_t big = 4 * (s->nnz_total / nbk);
    if (big < kBigMin) big = kBigMin;
    if (big > kBktCap) big = kBktCap;
    g.big = (uint32_t)big;
    const int64_t cap = s->nnz_total / big + 1, cap_over = s->nnz_total / kBktCap + 1;
    g.max_over = (int32_t)(nbk < cap ? nbk : cap);
    g.seg_tiles_max = (int32_t)(s->nnz_total / kBktCap + (nbk < cap_over ? nbk : cap_over));
  }
  g.huge_runs = reinterpret_cast<HugeRun*>(base + L.huge_runs);
  g.huge_part = reinterpret_cast<float*>(base + L.huge_part);
}

// Enqueues steps 1-3: afterwards keys[1]/vals[1] hold the pairs partitioned into buckets and

inline int check_ws(const dlrm_sparse_batch* s, void* ws, size_t bytes, WsLayout* L) {
  *L = ws_layout(s->K, s->B, s->d, s->nnz_total);
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255) || bytes < L->total) return DLRM_ERR_WORKSPACE;
  if (L->nt_max > 0x7FFFFFFF || ((int64_t)s->K << kMaxTopBits) > 0x7FFFFFFF) return DLRM_ERR_BAD_SHAPE;
  if (s->K > DLRM_MAX_BWD_TABLES) return DLRM_ERR_BAD_SHAPE;  // the hot-row launches put the table in grid.y
  return DLRM_OK;
}

// steps 1-3 (bwd_partition.hip): afterwards keys[1]/vals[1] hold the pairs partitioned into buckets
// and bucket_start the bucket boundaries
int enqueue_partition(const dlrm_sparse_batch* s, const GroupArgs& g, hipStream_t st);
// step 4 onwards with the SGD / Adagrad row update (bwd_reduce_sgd.hip, bwd_reduce_adagrad.hip)
// (one translation unit per optimizer and per weighted / unweighted pooling)
// tm: NULL, or the caller's event pair recorded around the bucket_reduce launch of this call
int run_reduce_sgd(const GroupArgs& g, const UpdArgs& u, int dtype, int G, int K, const dlrm_bwd_timing* tm,
                   hipStream_t st);
int run_reduce_adagrad(const GroupArgs& g, const UpdArgs& u, int dtype, int G, int K, const dlrm_bwd_timing* tm,
                       hipStream_t st);
int run_reduce_sgd_weighted(const GroupArgs& g, const UpdArgs& u, int dtype, int G, int K, const dlrm_bwd_timing* tm,
                            hipStream_t st);
int run_reduce_adagrad_weighted(const GroupArgs& g, const UpdArgs& u, int dtype, int G, int K,
                                const dlrm_bwd_timing* tm, hipStream_t st);
// bwd_tail.hip
int launch_segment_sort(const GroupArgs& g, hipStream_t st);
// *dense_groups_used: bag groups the dense kernel wrote partial sums for (tables it took; the others: ngroups)
int launch_hot_rows(const GroupArgs& g, const UpdArgs& u, int G, int K, int ngroups, int* dense_groups_used,
                    hipStream_t st);

}  // namespace dlrm
