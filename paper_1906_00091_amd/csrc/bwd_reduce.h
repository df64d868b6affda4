// Backward steps 4 / 4a and the row updates: sorted runs -> one read-modify-write per row.
// Template code; bwd_reduce_{sgd,adagrad}[_weighted].hip instantiate it per optimizer and per
// unweighted / weighted pooling.
#pragma once
#include "bwd_sort.h"

namespace dlrm {

// The second member of a sorted pair is the bag itself (sum pooling) or, for a weighted batch,
// the position inside the table, by which the bag and the weight a of Eq. (2) are looked up.
struct Entry {
  uint32_t bag;
  float w;
};
template <bool WT>
__device__ inline Entry entry_of(const GroupArgs& a, int64_t tbl, uint32_t val) {
  Entry e;
  if constexpr (WT) {
    const PosEntry pe = a.pos_entry[tbl + val];
    e.bag = pe.bag;
    e.w = pe.w;
  } else {
    e.bag = val;
    e.w = 1.0f;
  }
  return e;
}

// A weighted bucket sorted in LDS has its entries resolved once, by all threads at the same time,
// before any run is summed: the bag replaces the position in the sorted values and the weight goes to
// LDS beside it, in two pieces (the sort's per-wavefront counters, dead once the sort is done, and
// an extension for the rest), which keeps four workgroups per compute unit.  Without this every
// gradient row load waits for two dependent gathers of its own.
constexpr int kResolvedLo = kNW * kSortBuckets;
struct ResolvedW {
  float* lo;  // entries [0, kResolvedLo)
  float* hi;  // entries [kResolvedLo, kBktCap)
  __device__ float& at(uint32_t i) const { return i < (uint32_t)kResolvedLo ? lo[i] : hi[i - kResolvedLo]; }
};
// Runs longer than this are summed by the whole workgroup.  With many lane groups per workgroup
// (narrow rows) a medium run left to one lane group is the critical path of the bucket sooner.
template <int G>
__device__ constexpr uint32_t long_run() {
  return kThreads / G >= 32 ? (uint32_t)kLongRunMin : (uint32_t)kLongRun;
}

// Sum (weight times) dS rows of the sorted entries [i0, i1) taking every `stride`-th entry from
// i0 + first; U loads in flight, ascending order.  vals: LDS or global.  tbl: start of the table
// in the batch's index array.
template <int U, bool WT>
__device__ inline f32x4 sum_entries(const GroupArgs& a, int64_t tbl, const float* g, int64_t stride_b,
                                    const uint32_t* vals, uint32_t i0, uint32_t i1,
                                    uint32_t first, uint32_t stride) {
  f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
  for (uint32_t i = i0 + first; i < i1; i += U * stride) {
    Entry e[U];
    f32x4 v[U];
#pragma unroll
    for (int t = 0; t < U; ++t) e[t] = entry_of<WT>(a, tbl, vals[i + t * stride < i1 ? i + t * stride : i]);
#pragma unroll
    for (int t = 0; t < U; ++t) v[t] = loadf4(g + (int64_t)e[t].bag * stride_b);
#pragma unroll
    for (int t = 0; t < U; ++t) {
      if (i + t * stride < i1) {
        if constexpr (WT) {
          acc.x = fmaf(e[t].w, v[t].x, acc.x);
          acc.y = fmaf(e[t].w, v[t].y, acc.y);
          acc.z = fmaf(e[t].w, v[t].z, acc.z);
          acc.w = fmaf(e[t].w, v[t].w, acc.w);
        } else {
          acc += v[t];
        }
      }
    }
  }
  return acc;
}

// keys/bags: the bucket's sorted pairs (n of them; LDS or global), heads: LDS list of run starts
// with heads[nruns] = n.  gpos0: global position of the bucket's first pair.
template <int DT, int G, int OPT, bool WT>
__device__ inline void reduce_runs(const GroupArgs& a, const UpdArgs& u, const Bucket& b, char* W,
                                   const uint32_t* keys, const uint32_t* bags, const uint32_t* heads,
                                   uint32_t h0, uint32_t nruns, const uint32_t* longs, uint32_t nlong,
                                   int src, float* part) {
  constexpr int NG = kThreads / G;
  // gradient rows a lane group keeps in flight while the workgroup sums a long run: few lane groups
  // (wide rows) need more each to keep the same number of bytes in flight
  constexpr int kLongU = (NG >= 32 || WT) ? 4 : 8;
  const int grp = threadIdx.x / G, chunk = threadIdx.x % G;
  const bool col_ok = chunk * 4 < u.d;
  // lanes past the last column shadow column group 0 (same addresses) and never write
  const float* g = u.dS + (int64_t)b.k * u.stride_k + (col_ok ? chunk : 0) * 4;
  // short runs: a lane group takes RU runs per round; the table rows and the first gradient
  // row of all RU runs are requested before any of them is consumed
  constexpr int RU = OPT == kAdagrad ? 2 : 4;  // Adagrad also holds the state rows
  const int cchunk = col_ok ? chunk : 0;
  float* H = state_base<OPT>(u, b.k);
  const int64_t tbl = WT ? a.tbl_off[b.k] : 0;
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
    Entry e0[RU];
#pragma unroll
    for (int t = 0; t < RU; ++t) e0[t] = entry_of<WT>(a, tbl, bags[i0[t]]);
#pragma unroll
    for (int t = 0; t < RU; ++t) acc[t] = loadf4(g + (int64_t)e0[t].bag * u.stride_b);
#pragma unroll
    for (int t = 0; t < RU; ++t) wv[t] = row_load<DT, OPT>(wp[t]);
    if constexpr (WT) {
#pragma unroll
      for (int t = 0; t < RU; ++t) acc[t] *= e0[t].w;
    }
#pragma unroll
    for (int t = 0; t < RU; ++t) {
      const uint32_t len = i1[t] - i0[t];
      if (r0 + t >= nruns || len > long_run<G>()) continue;
      if (len > 1) acc[t] += sum_entries<4, WT>(a, tbl, g, u.stride_b, bags, i0[t] + 1, i1[t], 0, 1);
      if (col_ok) row_update_store<DT, OPT>(wp[t], wv[t], acc[t], u);
    }
  }
  // long runs: the whole workgroup per run, lane group s taking entries s, s+NG, ...; the NG
  // partial sums are added in group order (in two levels of fixed shape when NG > 16)
  for (uint32_t q = 0; q < nlong; ++q) {  // uniform
    const uint32_t r = longs[q];
    const uint32_t i0 = heads[r] - h0, i1 = heads[r + 1] - h0;
    const uint32_t len = i1 - i0;
    if (len > (uint32_t)kHugeRun && a.no_tail && threadIdx.x == 0) atomicAdd(&a.seg_meta[kRouteHugeInPlace], 1u);
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
    // the row is requested first: its latency hides behind the gather
    const bool upd = grp == 0 && col_ok;
    RowRef wr = row_ref<DT, OPT>(W, H, u.d, keys[i0], cchunk);
    RowVal wv{};
    if (upd) wv = row_load<DT, OPT>(wr);
    const f32x4 acc = sum_entries<kLongU, WT>(a, tbl, g, u.stride_b, bags, i0, i1, (uint32_t)grp, (uint32_t)NG);
    __syncthreads();
    if (col_ok) storef4(part + grp * (G * 4) + chunk * 4, acc);
    __syncthreads();
    constexpr int L1 = NG > 16 ? 8 : 1;  // many lane groups: sums of L1 consecutive partials first
    if constexpr (L1 > 1) {
      if (grp < NG / L1 && col_ok) {
        f32x4 t = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int s = 0; s < L1; ++s) t += loadf4(part + (grp * L1 + s) * (G * 4) + chunk * 4);
        storef4(part + grp * L1 * (G * 4) + chunk * 4, t);  // a slot only this lane reads above
      }
      __syncthreads();
    }
    if (upd) {
      f32x4 tot = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int s = 0; s < NG / L1; ++s) tot += loadf4(part + s * L1 * (G * 4) + chunk * 4);
      row_update_store<DT, OPT>(wr, wv, tot, u);
    }
  }
}

// A bucket sorted in LDS (unweighted batch), reduced with the WORK, not the runs, dealt evenly: lane
// group g takes the sorted entries [g*E, (g+1)*E), E = ceil(n / groups), whatever runs they belong
// to, U gradient rows in flight from the first entry to the last.  An entry whose row differs from
// its predecessor's starts a run (its table row is requested with the gradient rows of its round);
// a run that ends inside the slab is applied at once.  What a slab holds of a run that began in an
// earlier slab goes to LDS, and after one barrier the group where a run began adds the later slabs'
// pieces in slab order and applies the row.  Within a run the entries are added in position order
// inside each slab and the slabs in order: a fixed order, the same on every call.  No list of run
// heads is needed, and a run of any length inside the bucket is covered.
// WT: sval holds the resolved bags and rw the weights a of Eq. (2) of the sorted entries.
template <int DT, int G, int OPT, bool WT = false>
__device__ inline void reduce_slabs(const UpdArgs& u, const Bucket& b, char* W, const uint32_t* skey,
                                    const uint32_t* sval, uint32_t n, float* part, uint32_t* flags,
                                    const ResolvedW& rw = ResolvedW{nullptr, nullptr}) {
  constexpr int NG = kThreads / G;
  // Gradient rows in flight per lane group, each measured with whole libraries on one box.  16-bit tables, SGD (128
  // registers): 3 / 4 / 6 / 8 / 10 -> 1.154 / 1.178 / 1.140 / 1.123 / 1.240 ms per launch on the hot-row workload.
  // fp32, SGD (168 registers): 4 / 8 / 12 -> 165 / 162 / 160 us on the multi-hot workload, step 135.8 / 134.3 /
  // 132.5 us on the large one-hot one (12 spills 120 bytes; 16 spills 300).  Adagrad: 4 / 6 / 8 -> 325 / 317 / 324 us
  // (multi-hot), 2.66 / 2.40 / 2.57 ms (hot-row).
  constexpr int U = OPT == kAdagrad ? 6 : DT == DLRM_F32 ? 12 : 8;
  const int grp = threadIdx.x / G, chunk = threadIdx.x % G;
  const bool col_ok = chunk * 4 < u.d;
  const int cchunk = col_ok ? chunk : 0;  // lanes past the last column shadow column group 0 and never write
  const float* g = u.dS + (int64_t)b.k * u.stride_k + cchunk * 4;
  float* H = state_base<OPT>(u, b.k);
  const uint32_t E = (n + NG - 1) / NG;
  const uint32_t p0 = (uint32_t)grp * E < n ? (uint32_t)grp * E : n;
  const uint32_t p1 = p0 + E < n ? p0 + E : n;
  const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
  f32x4 acc = zero, headp = zero;
  bool have = false;   // a run has begun in this slab
  RowRef cur{nullptr, nullptr};
  RowVal curv{};
  for (uint32_t c0 = p0; c0 < p1; c0 += U) {
    uint32_t key[U];
    bool hd[U];
    f32x4 v[U];
    float wt[WT ? U : 1];
    // the table rows of the runs that begin in this round (16-bit tables: 8 bytes per lane)
    u32x2 wlo[U], whi[DT == DLRM_F32 ? U : 1];
    f32x4 wh[OPT == kAdagrad ? U : 1];
#pragma unroll
    for (int j = 0; j < U; ++j) {
      const uint32_t p = c0 + j < p1 ? c0 + j : p1 - 1;
      key[j] = skey[p];
      const uint32_t prev = skey[p > 0 ? p - 1 : 0];
      hd[j] = c0 + j < p1 && (p == 0 || key[j] != prev);
      v[j] = loadf4(g + (int64_t)sval[p] * u.stride_b);
      if constexpr (WT) wt[j] = rw.at(p);
    }
#pragma unroll
    for (int j = 0; j < U; ++j) {
      wlo[j] = u32x2{0u, 0u};
      if constexpr (DT == DLRM_F32) whi[j] = u32x2{0u, 0u};
      if constexpr (OPT == kAdagrad) wh[j] = zero;
      if (hd[j]) {
        const RowVal t = row_load<DT, OPT>(row_ref<DT, OPT>(W, H, u.d, key[j], cchunk));
        wlo[j] = u32x2{t.w.x, t.w.y};
        if constexpr (DT == DLRM_F32) whi[j] = u32x2{t.w.z, t.w.w};
        if constexpr (OPT == kAdagrad) wh[j] = t.h;
      }
    }
#pragma unroll
    for (int j = 0; j < U; ++j) {
      if (hd[j]) {
        if (have) {
          if (col_ok) row_update_store<DT, OPT>(cur, curv, acc, u);
        } else {
          headp = acc;
        }
        acc = zero;
        cur = row_ref<DT, OPT>(W, H, u.d, key[j], cchunk);
        curv.w = u32x4{wlo[j].x, wlo[j].y, 0u, 0u};
        if constexpr (DT == DLRM_F32) {
          curv.w.z = whi[j].x;
          curv.w.w = whi[j].y;
        }
        if constexpr (OPT == kAdagrad) curv.h = wh[j];
        have = true;
      }
      if (c0 + j < p1) {
        if constexpr (WT) {
          acc.x = fmaf(wt[j], v[j].x, acc.x);
          acc.y = fmaf(wt[j], v[j].y, acc.y);
          acc.z = fmaf(wt[j], v[j].z, acc.z);
          acc.w = fmaf(wt[j], v[j].w, acc.w);
        } else {
          acc += v[j];
        }
      }
    }
  }
  if (!have) headp = acc;   // the whole slab continues an earlier run (an empty slab: zero)
  if (col_ok) storef4(part + grp * (G * 4) + chunk * 4, headp);
  if (chunk == 0) flags[grp] = p0 < p1 ? (have ? 1u : 2u) : 0u;   // empty / a run begins here / all continuation
  __syncthreads();
  if (have) {
    f32x4 tot = acc;
    for (int g2 = grp + 1; g2 < NG; ++g2) {
      const uint32_t f = flags[g2];
      if (f == 0u) break;
      tot += loadf4(part + g2 * (G * 4) + cchunk * 4);
      if (f == 1u) break;
    }
    if (col_ok) row_update_store<DT, OPT>(cur, curv, tot, u);
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

// Lists the runs longer than `longer_than` (>= kLongRunMin) among s.heads[0..nruns] (any order: each is a
// different row).  At most kBktCap/kLongRunMin + 1 of them have their head inside a window of kBktCap
// positions.
__device__ inline uint32_t collect_long_runs(SortLds& s, uint32_t nruns, uint32_t longer_than) {
  if (threadIdx.x == 0) s.nlong = 0;
  __syncthreads();
  for (uint32_t r = threadIdx.x; r < nruns; r += kThreads) {
    if (s.heads[r + 1] - s.heads[r] > longer_than) s.longs[atomicAdd(&s.nlong, 1u)] = r;
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
template <int DT, int G, int OPT, bool WT>
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
    const uint32_t nlong = collect_long_runs(s, total, long_run<G>());
    reduce_runs<DT, G, OPT, WT>(a, u, b, W, keys, bags, s.heads, 0u, total, s.longs, nlong, src, part);
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

// nc: number of candidates (uniform); most oversized buckets have one or two
__device__ inline uint32_t class_of(uint32_t key, const uint32_t* cd, uint32_t nc) {
  uint32_t cls = (uint32_t)kCand;
#pragma unroll
  for (int c = 0; c < kCand; ++c) {
    if ((uint32_t)c >= nc) break;  // uniform
    cls = key == cd[c] ? (uint32_t)c : cls;
  }
  return cls;
}

// Pairs [bk.start, bk.start + bk.n) of pair buffer src, more than kBktCap of them, that no
// shortcut applies to: queued as a segment when per-row counters fit LDS, else sorted here.
template <int DT, int G, int OPT, bool WT>
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
  if (threadIdx.x == 0) atomicAdd(&a.seg_meta[kRouteGlobalSort], 1u);
  const int res = sort_bucket_global(a, bk, s, src);
  __syncthreads();
  const uint32_t* keys = a.keys[res] + bk.start;
  const uint32_t* bags = a.vals[res] + bk.start;
  for (uint32_t w0 = 0; w0 < bk.n; w0 += kBktCap) reduce_window<DT, G, OPT, WT>(a, u, bk, W, keys, bags, w0, res, s, part);
}

template <int DT, int G, int OPT, bool WT>
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
    sort_reduce_large<DT, G, OPT, WT>(a, u, b, W, 1, s, part);
    return;
  }
  if (tid == 0) atomicAdd(&a.seg_meta[kRouteSplit], 1u);
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
      const uint32_t cls = class_of(kk[q], cd, nc);
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
      const uint32_t cls = class_of(key[q], cd, nc);
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
    const uint32_t nlong = collect_long_runs(s, nc, long_run<G>());
    reduce_runs<DT, G, OPT, WT>(a, u, b, W, kout, vout, s.heads, 0u, nc, s.longs, nlong, 0, part);
  }
  // ---- the rest
  Bucket rest = b;
  rest.start = b.start + sp.cbase[kCand];
  rest.n = sp.cnt[kCand];
  __syncthreads();
  if (rest.n == 0) return;  // uniform
  if (rest.n > (uint32_t)kBktCap) {
    sort_reduce_large<DT, G, OPT, WT>(a, u, rest, W, 0, s, part);
    return;
  }
  sort_bucket_lds(a, rest, s, 0);
  if constexpr (!WT) {
    reduce_slabs<DT, G, OPT>(u, rest, W, s.skey, s.sval, rest.n, part, s.heads);
    return;
  }
  const uint32_t nruns = compact_heads_lds(s, (int)rest.n);
  const uint32_t nlong = collect_long_runs(s, nruns, long_run<G>());
  reduce_runs<DT, G, OPT, WT>(a, u, rest, W, s.skey, s.sval, s.heads, 0u, nruns, s.longs, nlong, 0, part);
}

template <int DT, int G, int OPT, bool WT>
// register budget: 4 wavefronts per SIMD for 16-bit tables with SGD, 3 (168 registers) otherwise -- measured both ways
// on the multi-hot and one-hot workloads (fp32: 3 is 2 % ahead) and on the hot-row one (fp16: 4 is 12 % ahead)
__global__ __launch_bounds__(kThreads, (OPT == kAdagrad || DT == DLRM_F32) ? 3 : 4) void bucket_reduce_kernel(GroupArgs a, UpdArgs u) {
  __shared__ SortLds s;
  __shared__ SplitLds sp;
  __shared__ float part[kThreads * 4];
  __shared__ float wext[WT ? kBktCap - kResolvedLo : 1];
  uint32_t bid;
  bool listed;
  if (!bucket_id_of_block(a, &bid, &listed)) return;
  const Bucket b = bucket_of_block(a, bid);
  if (b.n == 0 || (!listed && b.n > a.big)) return;   // a heavy bucket belongs to one of the first workgroups
  char* W = static_cast<char*>(u.tables[b.k]);
  if (b.n <= (uint32_t)kBktCap) {
    sort_bucket_lds(a, b, s);
    if constexpr (!WT) {
      reduce_slabs<DT, G, OPT>(u, b, W, s.skey, s.sval, b.n, part, s.heads);
      return;
    }
    // weighted: every sorted entry is resolved (position -> bag, weight) once, by all threads at the same time
    uint32_t ebag[WT ? kBktItems : 1];
    float ew[WT ? kBktItems : 1];
    if constexpr (WT) {
      const int64_t tbl = a.tbl_off[b.k];
#pragma unroll
      for (int j = 0; j < kBktItems; ++j) {
        const uint32_t li = threadIdx.x + j * kThreads;
        const uint32_t pos = li < b.n ? s.sval[li] : s.sval[0];
        const PosEntry pe = a.pos_entry[tbl + pos];
        ebag[j] = pe.bag;
        ew[j] = pe.w;
      }
    }
    const ResolvedW rw{reinterpret_cast<float*>(&s.wcnt[0][0]), wext};
    if constexpr (WT) {
#pragma unroll
      for (int j = 0; j < kBktItems; ++j) {  // a thread rewrites only the slots it read
        const uint32_t li = threadIdx.x + j * kThreads;
        if (li < b.n) {
          s.sval[li] = ebag[j];
          rw.at(li) = ew[j];
        }
      }
      __syncthreads();
    }
    reduce_slabs<DT, G, OPT, WT>(u, b, W, s.skey, s.sval, b.n, part, s.heads, rw);
    return;
  }
  if (b.low_bits == 0) {  // the bucket holds one row: a single run, already in position order
    if (threadIdx.x == 0) {
      s.heads[0] = 0;
      s.heads[1] = b.n;
      atomicAdd(&a.seg_meta[kRouteOneRow], 1u);
    }
    __syncthreads();
    const uint32_t nlong = collect_long_runs(s, 1, long_run<G>());
    reduce_runs<DT, G, OPT, WT>(a, u, b, W, a.keys[1] + b.start, a.vals[1] + b.start, s.heads, 0u, 1, s.longs, nlong, 1,
                       part);
    return;
  }
  reduce_oversized<DT, G, OPT, WT>(a, u, b, W, s, sp, part);
}


template <int DT, int G, int OPT, bool WT>
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
  reduce_window<DT, G, OPT, WT>(a, u, b, W, a.keys[dst] + sg.start, a.vals[dst] + sg.start, t * kBktCap, dst, s, part);
}


// A lane group per hot run adds the run's partial sums in bag-group order and updates the row.
// A launch of its own: the kernel boundary orders it after every partial, at no fence.
template <int DT, int G, int OPT, bool WT>
__global__ __launch_bounds__(kThreads) void hot_finish_kernel(GroupArgs a, UpdArgs u, int ngroups, int ngd) {
  constexpr int S = DLRM_WAVE / G;
  const int k = blockIdx.y;
  const uint32_t nruns = a.hot_cnt[k];
  if (nruns == 0) return;
  const uint32_t base = hot_list_base(a, k);
  const int lane = lane_id();
  const int chunk = lane % G;
  if (chunk * 4 >= u.d) return;
  // a table the dense kernel took has partial sums for its own (fewer) bag groups, in the same layout
  const int nsum = (!WT && nruns >= (uint32_t)kDenseFrom) ? ngd : ngroups;
  char* W = static_cast<char*>(u.tables[k]);
  float* H = state_base<OPT>(u, k);
  for (uint32_t r = (blockIdx.x * kNW + wave_id()) * S + lane / G; r < nruns; r += gridDim.x * kNW * S) {
    const float* part = a.huge_part + ((size_t)(base + r) * ngroups) * u.d + chunk * 4;
    f32x4 sum = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int g0 = 0; g0 < nsum; g0 += 8) {
      f32x4 v[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) v[q] = loadf4(part + (size_t)(g0 + q < nsum ? g0 + q : g0) * u.d);
#pragma unroll
      for (int q = 0; q < 8; ++q)
        if (g0 + q < nsum) sum += v[q];
    }
    row_update<DT, OPT>(W, H, u, a.huge_runs[base + r].row, chunk, sum);
  }
}


template <int DT, int G, int OPT, bool WT>
static int launch_reduce(const GroupArgs& g, const UpdArgs& u, int K, const dlrm_bwd_timing* tm, hipStream_t st) {
  const unsigned blocks = ((unsigned)K << g.top_bits) + (unsigned)g.max_over;
  if (tm && tm->ev_start && hipEventRecord(static_cast<hipEvent_t>(tm->ev_start), st) != hipSuccess) return DLRM_ERR_HIP;
  hipLaunchKernelGGL((bucket_reduce_kernel<DT, G, OPT, WT>), dim3(blocks), dim3(kThreads), 0, st, g, u);
  DLRM_CHECK_LAUNCH();
  if (tm && tm->ev_stop && hipEventRecord(static_cast<hipEvent_t>(tm->ev_stop), st) != hipSuccess) return DLRM_ERR_HIP;
  if (g.no_tail) return DLRM_OK;
  const unsigned seg_tiles = (unsigned)(g.seg_tiles_max);
  int rc = launch_segment_sort(g, st);
  if (rc != DLRM_OK) return rc;
  hipLaunchKernelGGL((segment_reduce_kernel<DT, G, OPT, WT>), dim3(seg_tiles), dim3(kThreads), 0, st, g, u);
  DLRM_CHECK_LAUNCH();
  const int ng = hot_groups(g.B, u.d);
  int ngd = ng;
  rc = launch_hot_rows(g, u, G, K, ng, &ngd, st);
  if (rc != DLRM_OK) return rc;
  hipLaunchKernelGGL((hot_finish_kernel<DT, G, OPT, WT>), dim3(4, K), dim3(kThreads), 0, st, g, u, ng, ngd);
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}

template <int DT, int OPT, bool WT>
static int dispatch_reduce(const GroupArgs& g, const UpdArgs& u, int G, int K, const dlrm_bwd_timing* tm, hipStream_t st) {
  switch (G) {
    case 1: return launch_reduce<DT, 1, OPT, WT>(g, u, K, tm, st);
    case 2: return launch_reduce<DT, 2, OPT, WT>(g, u, K, tm, st);
    case 4: return launch_reduce<DT, 4, OPT, WT>(g, u, K, tm, st);
    case 8: return launch_reduce<DT, 8, OPT, WT>(g, u, K, tm, st);
    case 16: return launch_reduce<DT, 16, OPT, WT>(g, u, K, tm, st);
    case 32: return launch_reduce<DT, 32, OPT, WT>(g, u, K, tm, st);
    case 64: return launch_reduce<DT, 64, OPT, WT>(g, u, K, tm, st);
  }
  return DLRM_ERR_BAD_SHAPE;
}


template <int OPT, bool WT>
inline int run_reduce(const GroupArgs& g, const UpdArgs& u, int dtype, int G, int K, const dlrm_bwd_timing* tm, hipStream_t st) {
  switch (dtype) {
    case DLRM_F32: return dispatch_reduce<DLRM_F32, OPT, WT>(g, u, G, K, tm, st);
    case DLRM_F16: return dispatch_reduce<DLRM_F16, OPT, WT>(g, u, G, K, tm, st);
    case DLRM_BF16: return dispatch_reduce<DLRM_BF16, OPT, WT>(g, u, G, K, tm, st);
  }
  return DLRM_ERR_BAD_DTYPE;
}

}  // namespace dlrm
