// Bucket-local sorts of the backward (LDS, streaming through global memory) and the list of
// oversized buckets ("segments"); shared by the reduce, tail and export translation units.
#pragma once
#include "bwd_common.h"

namespace dlrm {

__device__ inline void prepare_segments(const GroupArgs& a, uint32_t* smem) {
  const int nb = 1 << a.top_bits;
  const uint32_t n_over = atomicAdd(a.list_cnt, 0u);   // heavy buckets; the oversized ones are among them
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
      ok = sg.n > (uint32_t)kBktCap && sg.low_bits >= 1 && sg.low_bits <= (uint32_t)kSegMaxBits ? 1u : 0u;
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


struct SortLds {
  uint32_t wcnt[kNW][kSortBuckets];
  uint32_t skey[kBktCap];
  uint32_t sval[kBktCap];
  uint32_t heads[kBktCap + 1];
  uint32_t base[kSortBuckets];
  uint32_t smem[kNW + 1];
  uint32_t longs[kBktCap / kLongRunMin + 2];   // runs longer than the threshold among the current heads
  uint32_t nlong;
};

__device__ inline int pass_bits(int left, int passes_left) { return (left + passes_left - 1) / passes_left; }

// Buckets of at most kBktCap pairs (read from pair buffer src): stable LSD passes entirely in
// LDS.  The pairs end up in s.skey / s.sval in (row, position) order.  The bucket is dealt evenly to
// the wavefronts, `per` = ceil(n / 256) items a lane (see rank_items).
__device__ inline void sort_bucket_lds(const GroupArgs& a, const Bucket& b, SortLds& s, int src = 1) {
  const int lane = lane_id(), w = wave_id(), tid = threadIdx.x;
  const uint32_t* kin = a.keys[src] + b.start;
  const uint32_t* vin = a.vals[src] + b.start;
  const int n = (int)b.n;
  const int per = (n + kThreads - 1) / kThreads;   // 1..kBktItems, uniform
  uint32_t key[kBktItems], val[kBktItems], dg[kBktItems], rnk[kBktItems];
  bool ok[kBktItems];
#pragma unroll
  for (int j = 0; j < kBktItems; ++j) {
    const int li = w * (DLRM_WAVE * per) + j * DLRM_WAVE + lane;
    ok[j] = j < per && li < n;
    key[j] = ok[j] ? kin[li] : 0xFFFFFFFFu;
    val[j] = ok[j] ? vin[li] : 0u;
    dg[j] = 0;
    rnk[j] = 0;
  }
  const int passes = (b.low_bits + kSortBits - 1) / kSortBits;
  if (passes == 0) {  // a single row per bucket: already in position order
#pragma unroll
    for (int j = 0; j < kBktItems; ++j) {
      const int li = w * (DLRM_WAVE * per) + j * DLRM_WAVE + lane;
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
    rank_items<kBktItems, kSortBuckets>(dg, ok, bits, s.wcnt, rnk, per);
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
        const int li = w * (DLRM_WAVE * per) + j * DLRM_WAVE + lane;
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

}  // namespace dlrm
