// Backward tail: the segment sort (oversized lists the bucket kernel could not take) and the hot
// rows kernel.  Neither updates a row, so neither depends on the optimizer.
#include "bwd_sort.h"

namespace dlrm {

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

template <int G, bool WT>
__global__ __launch_bounds__(kThreads) void hot_rows_kernel(GroupArgs a, UpdArgs u, int ngroups, int dense_from) {
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
  // weighted batches: a run lists positions; bag and weight are looked up by position
  const int64_t tbl = WT ? a.tbl_off[blockIdx.y] : 0;
  const int k = blockIdx.y, g = blockIdx.x;
  const uint32_t nruns = a.hot_cnt[k];
  if (nruns == 0) return;  // uniform
  if (dense_from > 0 && nruns >= (uint32_t)dense_from) return;  // hot_rows_dense_kernel has this table
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
          const uint32_t bm = WT ? a.pos_entry[tbl + bags[mid]].bag : bags[mid];
          if (bm < bound) lo = mid + 1; else hi = mid;
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
          if constexpr (WT) {
            // every entry on its own: LDS offset of its bag's gradient row and its weight
            uint32_t moff = (uint32_t)kHotTileFloats;  // entries past the end: the row of zeros, weight 0
            float mw = 0.0f;
            if ((uint32_t)lane < cnt) {
              const PosEntry pe = a.pos_entry[tbl + cur];
              moff = (pe.bag - (uint32_t)tb0) * (uint32_t)u.d;
              mw = pe.w;
            }
            for (uint32_t e = 0; e < cnt; e += HU * S) {
              f32x4 v[HU];
              float m[HU];
#pragma unroll
              for (int q = 0; q < HU; ++q) {
                v[q] = loadf4(tile + lane_entry<S>(moff, e + (uint32_t)(q * S), slot) + cchunk * 4);
                m[q] = u2f(lane_entry<S>(f2u(mw), e + (uint32_t)(q * S), slot));
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
            continue;
          }
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


// --- 5b. many hot rows in one table: the same pass as a dense product on the matrix cores -----------
// With many hot rows per table (a skewed table: the hottest few are in nearly every bag) the kernel
// above reads a gradient row from LDS once per (hot row, bag) that meets, and LDS reads are what it
// spends its time on.  Here the multiplicities of kDenseRuns hot rows against the bags of a tile
// are first counted into a small matrix C[bag][run] in LDS (integer atomics: exact, order-free);
// then G_hot[run][col] += sum_bag C[bag][run] * dS[bag][col] is a dense contraction over the bags
// of the tile, done with v_mfma_f32_16x16x4_f32: runs are the M index (two blocks of 16), columns
// the N index (blocks of 16, dealt to the wavefronts), four bags per instruction.  Every gradient
// row is read from LDS once per tile, and the accumulators are the instruction's result registers.
// The same workgroup grid, bag groups, run lists and partial-sum layout as hot_rows_kernel (which
// keeps the tables with few hot rows and the weighted batches); hot_finish_kernel follows.
//   16x16x4 layout: lane l supplies A[m = l%16][k = l/16] and B[k = l/16][n = l%16] and holds
//   D[m = 4*(l/16) + v][n = l%16] in element v of its accumulator.
constexpr int kDenseRuns = 32;     // hot rows per pass of a workgroup
constexpr int kDenseStage = 8;     // float4 registers per thread holding the next tile
constexpr int kDenseTileFloats = 8192;
constexpr int kDenseDeep = 4;      // 64-entry chunks of one run's list in flight while counting

template <int G>
__global__ __launch_bounds__(kThreads) void hot_rows_dense_kernel(GroupArgs a, UpdArgs u, int ngroups) {
  constexpr int R = kDenseRuns;
  constexpr int NG = kThreads / G;                 // lane groups = gradient rows staged per pass
  constexpr int NP = G < kDenseStage ? G : kDenseStage;   // float4 staging registers: tiles of at most 256 bags
  constexpr int TB = NG * NP;                      // bags per tile: TB * d <= kDenseTileFloats
  constexpr int GB = NG * kHotStagePasses * kHotTilesPerGroup;  // bags per workgroup, as in hot_rows_kernel
  constexpr int RW = R / kNW;                      // runs whose entries one wavefront counts
  constexpr int NBLK = (G * 4 + 15) / 16;          // 16-column blocks of a gradient row (d <= 4G)
  constexpr int NBW = (NBLK + kNW - 1) / kNW;      // of which a wavefront takes blocks w, w + kNW, ...
  static_assert(TB * G * 4 <= kDenseTileFloats, "tile");
  __shared__ float tile[kDenseTileFloats];
  __shared__ uint32_t cmat[TB][R];                 // multiplicity of run r in bag tb0 + b
  __shared__ uint32_t rpos[R], rend[R], rsrc[R];   // first entry of a run for this workgroup's bags, its end, its pair buffer
  const int k = blockIdx.y, g = blockIdx.x;
  const uint32_t nruns = a.hot_cnt[k];
  if (nruns < (uint32_t)kDenseFrom) return;  // uniform: hot_rows_kernel has this table
  const uint32_t base = hot_list_base(a, k);
  const int lane = lane_id(), w = wave_id(), tid = threadIdx.x;
  const int chunk = lane % G;
  const int grp = tid / G;
  const bool col_ok = chunk * 4 < u.d;
  const int cchunk = col_ok ? chunk : 0;  // lanes past the last column shadow column group 0, never store
  const int bag_lo = g * GB;
  const int bag_hi = bag_lo + GB < a.B ? bag_lo + GB : a.B;
  if (bag_lo >= bag_hi) return;  // uniform
  const float* gk = u.dS + (int64_t)k * u.stride_k + cchunk * 4;
  const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
  for (uint32_t r0 = 0; r0 < nruns; r0 += R) {  // uniform
    __syncthreads();
    // where each run's entries for this workgroup's bags begin (one binary search per run; the tile
    // boundaries are found on the way, a run's bags ascend) and where the run ends
    for (int rl = tid; rl < R; rl += kThreads) {
      const uint32_t r = r0 + (uint32_t)rl;
      uint32_t c = 0, e = 0, src = 0;
      if (r < nruns) {
        const HugeRun hr = a.huge_runs[base + r];
        const uint32_t* bags = (hr.src ? a.vals[1] : a.vals[0]) + hr.start;
        uint32_t lo = 0, hi = hr.len;
        while (lo < hi) {
          const uint32_t mid = (lo + hi) >> 1;
          if (bags[mid] < (uint32_t)bag_lo) lo = mid + 1; else hi = mid;
        }
        c = hr.start + lo;
        e = hr.start + hr.len;
        src = hr.src;
      }
      rpos[rl] = c;   // runs past the last one: empty
      rend[rl] = e;
      rsrc[rl] = src;
    }
    __syncthreads();
    uint32_t pos[RW], end[RW];   // wave-uniform: next entry / end of the runs this wavefront counts
    int want[RW];                // wave-uniform: list chunks to request for the next tile
    const uint32_t* rb[RW];
#pragma unroll
    for (int i = 0; i < RW; ++i) {
      const int rl = w + kNW * i;
      pos[i] = rpos[rl];
      end[i] = rend[rl];
      want[i] = 1;
      rb[i] = rsrc[rl] ? a.vals[1] : a.vals[0];
    }
    f32x4 acc[2][NBW];   // [run block][column block of this wavefront]
#pragma unroll
    for (int j = 0; j < NBW; ++j) acc[0][j] = acc[1][j] = zero;
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
      __syncthreads();  // the previous tile and its counts have been consumed
#pragma unroll
      for (int p = 0; p < NP; ++p) {
        const int bb = p * NG + grp;
        if (col_ok) storef4(tile + bb * u.d + chunk * 4, bb < nb ? stage[p] : zero);  // no stale rows
      }
      for (int i = tid; i < TB * R; i += kThreads) (&cmat[0][0])[i] = 0u;
      __syncthreads();
      if (tb0 + TB < bag_hi) {  // uniform: the next tile travels while this one is used
        const int nn = bag_hi - (tb0 + TB) < TB ? bag_hi - (tb0 + TB) : TB;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
          const int bb = p * NG + grp < nn ? p * NG + grp : nn - 1;
          stage[p] = loadf4(gk + (int64_t)(tb0 + TB + bb) * u.stride_b);
        }
      }
      // count: wavefront w takes the entries of runs w, w + 4, ... that fall into this tile (a prefix
      // of what is left of the run).  All its runs' list chunks are requested together: per run as
      // many 64-entry chunks as the previous tile used, plus one (a run's share of a tile changes
      // little from tile to tile), so that a tile usually costs one round trip to memory.
      {
        const uint32_t bound = (uint32_t)(tb0 + nb);
        uint32_t ent[RW][kDenseDeep];
#pragma unroll
        for (int i = 0; i < RW; ++i) {
#pragma unroll
          for (int q = 0; q < kDenseDeep; ++q) {
            ent[i][q] = 0xFFFFFFFFu;
            const uint32_t e = pos[i] + (uint32_t)(q * DLRM_WAVE + lane);
            if (q < want[i] && e < end[i]) ent[i][q] = rb[i][e];   // q < want[i]: wave-uniform
          }
        }
#pragma unroll
        for (int i = 0; i < RW; ++i) {
          const int rl = w + kNW * i;
          uint32_t n = 0;
#pragma unroll
          for (int q = 0; q < kDenseDeep; ++q) {   // ascending bags: those inside the tile are a prefix
            const bool in = ent[i][q] < bound;
            if (in) atomicAdd(&cmat[ent[i][q] - (uint32_t)tb0][rl], 1u);
            n += (uint32_t)__popcll(__ballot(in));
          }
          pos[i] += n;
          uint32_t used = n;
          while (n == (uint32_t)(want[i] * DLRM_WAVE)) {   // wave-uniform: every requested entry was inside
            want[i] = kDenseDeep;
            uint32_t bag[kDenseDeep];
#pragma unroll
            for (int q = 0; q < kDenseDeep; ++q) {
              const uint32_t e = pos[i] + (uint32_t)(q * DLRM_WAVE + lane);
              bag[q] = 0xFFFFFFFFu;
              if (e < end[i]) bag[q] = rb[i][e];
            }
            n = 0;
#pragma unroll
            for (int q = 0; q < kDenseDeep; ++q) {
              const bool in = bag[q] < bound;
              if (in) atomicAdd(&cmat[bag[q] - (uint32_t)tb0][rl], 1u);
              n += (uint32_t)__popcll(__ballot(in));
            }
            pos[i] += n;
            used += n;
          }
          const int w1 = (int)(used / DLRM_WAVE) + 1;
          want[i] = w1 < kDenseDeep ? w1 : kDenseDeep;
        }
      }
      __syncthreads();
      // contract over the bags of the tile, four per instruction
      {
        const int m = lane & 15, kk = lane >> 4;
#pragma unroll 2
        for (int k0 = 0; k0 < TB; k0 += 4) {
          const float a0 = (float)cmat[k0 + kk][m];
          const float a1 = (float)cmat[k0 + kk][16 + m];
          const float* trow = tile + (k0 + kk) * u.d;
#pragma unroll
          for (int j = 0; j < NBW; ++j) {
            const int col = (w + kNW * j) * 16 + m;
            if ((w + kNW * j) * 16 < u.d) {  // wave-uniform
              const float b = col < u.d ? trow[col] : 0.0f;
              acc[0][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, b, acc[0][j], 0, 0, 0);
              acc[1][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, b, acc[1][j], 0, 0, 0);
            }
          }
        }
      }
    }
    // D[m = 4*(l/16) + v][n = l%16]: run r0 + 16*mb + m, column 16*(w + kNW*j) + n
    {
      const int n = lane & 15, mq = (lane >> 4) * 4;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
#pragma unroll
        for (int j = 0; j < NBW; ++j) {
          const int col = (w + kNW * j) * 16 + n;
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const uint32_t run = r0 + (uint32_t)(mb * 16 + mq + v);
            if (run < nruns && col < u.d)
              a.huge_part[((size_t)(base + run) * ngroups + g) * u.d + col] = acc[mb][j][v];
          }
        }
      }
    }
  }
}


int launch_segment_sort(const GroupArgs& g, hipStream_t st) {
  hipLaunchKernelGGL(segment_sort_kernel, dim3((unsigned)g.seg_tiles_max), dim3(kThreads), 0, st, g);
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}

template <int G>
static int launch_hot(const GroupArgs& g, const UpdArgs& u, int K, int ngroups, hipStream_t st) {
  if (g.weights != nullptr) {
    hipLaunchKernelGGL((hot_rows_kernel<G, true>), dim3(ngroups, K), dim3(kThreads), 0, st, g, u, ngroups, 0);
  } else {
    // tables with many hot rows go through the dense kernel, the others through the entry-by-entry one
    hipLaunchKernelGGL((hot_rows_dense_kernel<G>), dim3(ngroups, K), dim3(kThreads), 0, st, g, u, ngroups);
    DLRM_CHECK_LAUNCH();
    hipLaunchKernelGGL((hot_rows_kernel<G, false>), dim3(ngroups, K), dim3(kThreads), 0, st, g, u, ngroups,
                       kDenseFrom);
  }
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}

int launch_hot_rows(const GroupArgs& g, const UpdArgs& u, int G, int K, int ngroups, hipStream_t st) {
  switch (G) {
    case 1: return launch_hot<1>(g, u, K, ngroups, st);
    case 2: return launch_hot<2>(g, u, K, ngroups, st);
    case 4: return launch_hot<4>(g, u, K, ngroups, st);
    case 8: return launch_hot<8>(g, u, K, ngroups, st);
    case 16: return launch_hot<16>(g, u, K, ngroups, st);
    case 32: return launch_hot<32>(g, u, K, ngroups, st);
    case 64: return launch_hot<64>(g, u, K, ngroups, st);
  }
  return DLRM_ERR_BAD_SHAPE;
}

}  // namespace dlrm
