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
// spends its time on.  Here the multiplicities of kDenseRuns hot rows against a tile of bags are
// first counted into a small matrix C[run][bag] in LDS (integer atomics: exact, order-free); then
// G_hot[run][col] += sum_bag C[run][bag] * dS[bag][col] is a dense contraction over the bags of the
// tile, done with v_mfma_f32_16x16x4_f32: runs are the M index (two blocks of 16), four bags per
// instruction.
//
// Every wavefront works alone: it owns a quarter of the workgroup's bags, its own count matrix and
// accumulators for all runs and columns, and takes its gradient rows straight from global memory,
// so there is no barrier anywhere in the streaming loop and wavefronts in different phases
// (list reads, counting, contraction) fill each other's gaps.  The four partial results are added
// in bag order at the end.
//   16x16x4 layout: lane l supplies A[m = l%16][k = l/16] and B[k = l/16][n = l%16] and holds
//   D[m = 4*(l/16) + v][n = l%16] in element v of its accumulator.
//   Which column the N index n stands for is free as long as B and D agree: lane l loads the 16 bytes
//   dS[bag k][64h + 4n .. 64h + 4n + 3] with one instruction (a bag row is read as contiguous 256-byte
//   pieces) and component c of that load is the B operand of contraction (h, c), whose result
//   column n is gradient column 64h + 4n + c.
// The same bag groups, run lists and partial-sum layout as hot_rows_kernel (which keeps the
// tables with few hot rows and the weighted batches); hot_finish_kernel follows.
// A count of zero still multiplies the bag's gradient: a non-finite gradient entry of a bag reaches
// every hot row of this pass, not only the rows the bag looked up.
constexpr int kDenseRuns = 32;      // hot rows per pass of a workgroup
constexpr int kDenseTile = 64;      // bags per tile of a wavefront
constexpr int kDenseCStride = 68;   // words per run of the count matrix: 4m + k is a different bank for all 64 lanes
constexpr int kDensePre = 4;        // 4-bag steps of gradient rows in flight
constexpr int kDenseHeavy = 4;      // the longest runs of a pass: 256 list entries per request instead of 64

template <int NH>   // 64-column pieces of a gradient row
__global__ __launch_bounds__(kThreads, NH <= 2 ? 3 : 2) void hot_rows_dense_kernel(GroupArgs a, UpdArgs u, int ngroups,
                                                                                   int group_bags) {
  constexpr int R = kDenseRuns, TB = kDenseTile, CS = kDenseCStride, PRE = NH <= 2 ? kDensePre : kDensePre / 2;
  static_assert(R * CS * kNW >= R * 64 * NH, "the reduction buffer aliases the count matrices");
  __shared__ __align__(16) uint32_t cmat[kNW][R * CS];   // per wavefront: multiplicity of run r in bag tb0 + b at [r * CS + b]
  const int k = blockIdx.y, g = blockIdx.x;
  const uint32_t nruns = a.hot_cnt[k];
  if (nruns < (uint32_t)kDenseFrom) return;  // uniform: hot_rows_kernel has this table
  const uint32_t base = hot_list_base(a, k);
  const int lane = lane_id(), w = wave_id();
  const int m = lane & 15, kk = lane >> 4;
  // this wavefront's bags
  const int quarter = group_bags / kNW;
  int wb_lo = g * group_bags + w * quarter;
  wb_lo = wb_lo < a.B ? wb_lo : a.B;
  const int wb_hi = wb_lo + quarter < a.B ? wb_lo + quarter : a.B;
  const float* gk = u.dS + (int64_t)k * u.stride_k + 4 * m;
  // lanes whose columns lie past the row's end load piece 0 again (no branch around a load) and never store
  bool col_ok[NH];
  int hoff[NH];
#pragma unroll
  for (int h = 0; h < NH; ++h) {
    col_ok[h] = 64 * h + 4 * m < u.d;
    hoff[h] = col_ok[h] ? 64 * h : 0;
  }
  uint32_t* cm = cmat[w];
  float* red = reinterpret_cast<float*>(&cmat[0][0]);
  const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
  for (uint32_t r0 = 0; r0 < nruns; r0 += R) {  // uniform
    // lane r keeps the state of one run of this pass: next entry for this wavefront's bags (a binary
    // search: a run's bags ascend), end of the run, pair buffer that holds it.  The runs are dealt to
    // the lanes by length, longest first: the first kDenseHeavy get the wide list requests.
    uint32_t pos = 0, end = 0, src = 0, ridx = 0xFFFFFFFFu;
    {
      uint32_t len = 0;
      HugeRun hr;
      hr.start = hr.len = hr.src = 0;
      if (lane < R && r0 + (uint32_t)lane < nruns) {
        hr = a.huge_runs[base + r0 + (uint32_t)lane];
        len = hr.len;
      }
      uint32_t rank = 0;
#pragma unroll
      for (int j = 0; j < R; ++j) {
        const uint32_t lj = (uint32_t)__builtin_amdgcn_readlane((int)len, j);
        rank += (lj > len || (lj == len && j < lane)) ? 1u : 0u;
      }
      rank = lane < R ? rank : (uint32_t)lane;
      uint32_t lo = 0;
      if (len != 0 && wb_lo < wb_hi) {
        const uint32_t* bags = (hr.src ? a.vals[1] : a.vals[0]) + hr.start;
        uint32_t hi = hr.len;
        while (lo < hi) {
          const uint32_t mid = (lo + hi) >> 1;
          if (bags[mid] < (uint32_t)wb_lo) lo = mid + 1; else hi = mid;
        }
      }
      const bool live = len != 0 && wb_lo < wb_hi;
      pos = (uint32_t)__builtin_amdgcn_ds_permute((int)(rank * 4), (int)(live ? hr.start + lo : 0u));
      end = (uint32_t)__builtin_amdgcn_ds_permute((int)(rank * 4), (int)(live ? hr.start + hr.len : 0u));
      src = (uint32_t)__builtin_amdgcn_ds_permute((int)(rank * 4), (int)hr.src);
      ridx = (uint32_t)__builtin_amdgcn_ds_permute((int)(rank * 4), (int)(len != 0 ? r0 + (uint32_t)lane : 0xFFFFFFFFu));
    }
    const int nr = nruns - r0 < (uint32_t)R ? (int)(nruns - r0) : R;  // uniform; the absent runs are the last lanes
    f32x4 acc[2][NH][4];   // [run block][column piece][component of the 16-byte load]
#pragma unroll
    for (int h = 0; h < NH; ++h)
#pragma unroll
      for (int c = 0; c < 4; ++c) acc[0][h][c] = acc[1][h][c] = zero;
#pragma unroll 1
    for (int tb0 = wb_lo; tb0 < wb_hi; tb0 += TB) {  // wave-uniform
      const int nb = wb_hi - tb0 < TB ? wb_hi - tb0 : TB;
      const uint32_t bound = (uint32_t)(tb0 + nb);
      f32x4 bq[PRE][NH];
      for (int i = lane; i < R * CS / 4; i += DLRM_WAVE) reinterpret_cast<u32x4*>(cm)[i] = u32x4{0u, 0u, 0u, 0u};
      // count: the entries of every run that fall into this tile are a prefix of what is left of it
      {
        constexpr int HV = kDenseHeavy;
        // every run's request goes out before the first answer is used: 256 entries of each of the
        // longest runs, 64 of the others (requests past a run's end repeat its last entry and are
        // masked afterwards; an absent run has pos = end = 0)
        u32x4 hent[HV];
        uint32_t ent[R - HV];
#pragma unroll
        for (int q = 0; q < R; ++q) {
          const uint32_t pq = (uint32_t)__builtin_amdgcn_readlane((int)pos, q);
          const uint32_t eq = (uint32_t)__builtin_amdgcn_readlane((int)end, q);
          const uint32_t* lq = __builtin_amdgcn_readlane((int)src, q) ? a.vals[1] : a.vals[0];
          const uint32_t last = eq ? eq - 1u : 0u;
          if (q < HV) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
              const uint32_t x = pq + (uint32_t)(4 * lane + t);
              hent[q < HV ? q : 0][t] = lq[x < last ? x : last];
            }
          } else {
            const uint32_t x = pq + (uint32_t)lane;
            ent[q >= HV ? q - HV : 0] = lq[x < last ? x : last];
          }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < R; ++q) {
          if (q == R / 2) {
            // the first gradient rows travel while the second half of the runs is counted (bags past
            // the end repeat the last one; their counts stay zero)
#pragma unroll
            for (int s = 0; s < PRE; ++s) {
              const int bag = tb0 + 4 * s + kk < wb_hi ? tb0 + 4 * s + kk : wb_hi - 1;
#pragma unroll
              for (int h = 0; h < NH; ++h) bq[s][h] = loadf4(gk + (int64_t)bag * u.stride_b + hoff[h]);
            }
            __builtin_amdgcn_sched_barrier(0);
          }
          if (q >= nr) continue;  // uniform (the gradient requests above are not skipped)
          uint32_t pq = (uint32_t)__builtin_amdgcn_readlane((int)pos, q);
          const uint32_t eq = (uint32_t)__builtin_amdgcn_readlane((int)end, q);
          uint32_t* crow = cm + q * CS - tb0;
          uint32_t n = 0, full;
          if (q < HV) {
            full = 4u * DLRM_WAVE;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
              const uint32_t x = pq + (uint32_t)(4 * lane + t);
              const uint32_t bag = hent[q < HV ? q : 0][t];
              const bool in = x < eq && bag < bound;
              if (in) atomicAdd(crow + bag, 1u);
              n += (uint32_t)__popcll(__ballot(in));
            }
          } else {
            full = (uint32_t)DLRM_WAVE;
            const uint32_t x = pq + (uint32_t)lane;
            const uint32_t bag = ent[q >= HV ? q - HV : 0];
            const bool in = x < eq && bag < bound;
            if (in) atomicAdd(crow + bag, 1u);
            n = (uint32_t)__popcll(__ballot(in));
          }
          pq += n;
          while (n == full) {   // wave-uniform: every requested entry was inside the tile
            const uint32_t* lq = __builtin_amdgcn_readlane((int)src, q) ? a.vals[1] : a.vals[0];
            full = 4u * DLRM_WAVE;
            uint32_t bag[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
              const uint32_t x = pq + (uint32_t)(t * DLRM_WAVE + lane);
              bag[t] = 0xFFFFFFFFu;
              if (x < eq) bag[t] = lq[x];
            }
            n = 0;
#pragma unroll
            for (int t = 0; t < 4; ++t) {   // ascending bags: those inside are a prefix
              const bool in = bag[t] < bound;
              if (in) atomicAdd(crow + bag[t], 1u);
              n += (uint32_t)__popcll(__ballot(in));
            }
            pq += n;
          }
          pos = lane == q ? pq : pos;
        }
      }
      // contract over the bags of the tile, four per step
#pragma unroll
      for (int s = 0; s < TB / 4; ++s) {
        const float a0 = (float)cm[m * CS + 4 * s + kk];
        const float a1 = (float)cm[(16 + m) * CS + 4 * s + kk];
        f32x4 cur[NH];
#pragma unroll
        for (int h = 0; h < NH; ++h) cur[h] = bq[s % PRE][h];
        if (s + PRE < TB / 4) {
          const int bag = tb0 + 4 * (s + PRE) + kk < wb_hi ? tb0 + 4 * (s + PRE) + kk : wb_hi - 1;
#pragma unroll
          for (int h = 0; h < NH; ++h) bq[s % PRE][h] = loadf4(gk + (int64_t)bag * u.stride_b + hoff[h]);
        }
        __builtin_amdgcn_sched_barrier(0);   // the request stays PRE steps ahead of its use
#pragma unroll
        for (int h = 0; h < NH; ++h) {
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            acc[0][h][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, cur[h][c], acc[0][h][c], 0, 0, 0);
            acc[1][h][c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, cur[h][c], acc[1][h][c], 0, 0, 0);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // the four wavefronts' results added in bag order: wavefront 0 takes in 1, 2, 3 through LDS
    // (run slot r, column j at red[r * d + j]).  out[mb][h][v]: run slot 16*mb + 4*(l/16) + v, the four
    // columns 64h + 4*(l%16) + c.
    f32x4 out[2][NH][4];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int h = 0; h < NH; ++h)
#pragma unroll
        for (int v = 0; v < 4; ++v)
          out[mb][h][v] = f32x4{acc[mb][h][0][v], acc[mb][h][1][v], acc[mb][h][2][v], acc[mb][h][3][v]};
    __syncthreads();   // every count matrix has been consumed
    for (int from = 1; from < kNW; ++from) {  // uniform
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int h = 0; h < NH; ++h)
#pragma unroll
          for (int v = 0; v < 4; ++v)
            if (w == from && col_ok[h]) storef4(red + (mb * 16 + kk * 4 + v) * u.d + 64 * h + 4 * m, out[mb][h][v]);
      __syncthreads();
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int h = 0; h < NH; ++h)
#pragma unroll
          for (int v = 0; v < 4; ++v)
            if (w == 0 && col_ok[h]) out[mb][h][v] += loadf4(red + (mb * 16 + kk * 4 + v) * u.d + 64 * h + 4 * m);
      __syncthreads();
    }
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        // the run that was dealt to accumulator row mb*16 + kk*4 + v
        const uint32_t run = (uint32_t)__shfl((int)ridx, mb * 16 + kk * 4 + v, DLRM_WAVE);
#pragma unroll
        for (int h = 0; h < NH; ++h)
          if (w == 0 && run != 0xFFFFFFFFu && col_ok[h])
            storef4(a.huge_part + ((size_t)(base + run) * ngroups + g) * u.d + 64 * h + 4 * m, out[mb][h][v]);
      }
  }
}


int launch_segment_sort(const GroupArgs& g, hipStream_t st) {
  hipLaunchKernelGGL(segment_sort_kernel, dim3((unsigned)g.seg_tiles_max), dim3(kThreads), 0, st, g);
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}

// Bag groups of the dense kernel: as few as fill the machine once (gfx950: 256 compute units, three
// resident workgroups each, two for rows above 128 columns), never more than the partial-sum layout
// has room for; a wavefront's quarter of a group is whole tiles.
static void dense_groups(int B, int K, int nh, int ngroups, int* group_bags, int* ngd) {
  const int slots = 256 * (nh <= 2 ? 3 : 2);
  int n = slots / (K > 0 ? K : 1);
  n = n < 1 ? 1 : (n > ngroups ? ngroups : n);
  const int unit = kNW * kDenseTile;
  int gb = ((B + n - 1) / n + unit - 1) / unit * unit;
  if (gb < unit) gb = unit;
  *group_bags = gb;
  *ngd = (B + gb - 1) / gb;
}

template <int G>
static int launch_hot(const GroupArgs& g, const UpdArgs& u, int K, int ngroups, int* ngd, hipStream_t st) {
  *ngd = ngroups;
  if (g.weights != nullptr) {
    hipLaunchKernelGGL((hot_rows_kernel<G, true>), dim3(ngroups, K), dim3(kThreads), 0, st, g, u, ngroups, 0);
  } else {
    // tables with many hot rows go through the dense kernel, the others through the entry-by-entry one
    constexpr int NH = G <= 16 ? 1 : G == 32 ? 2 : 4;
    int group_bags;
    dense_groups(g.B, K, NH, ngroups, &group_bags, ngd);
    hipLaunchKernelGGL((hot_rows_dense_kernel<NH>), dim3(*ngd, K), dim3(kThreads), 0, st, g, u, ngroups, group_bags);
    DLRM_CHECK_LAUNCH();
    hipLaunchKernelGGL((hot_rows_kernel<G, false>), dim3(ngroups, K), dim3(kThreads), 0, st, g, u, ngroups,
                       kDenseFrom);
  }
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}

int launch_hot_rows(const GroupArgs& g, const UpdArgs& u, int G, int K, int ngroups, int* dense_groups_used,
                    hipStream_t st) {
  switch (G) {
    case 1: return launch_hot<1>(g, u, K, ngroups, dense_groups_used, st);
    case 2: return launch_hot<2>(g, u, K, ngroups, dense_groups_used, st);
    case 4: return launch_hot<4>(g, u, K, ngroups, dense_groups_used, st);
    case 8: return launch_hot<8>(g, u, K, ngroups, dense_groups_used, st);
    case 16: return launch_hot<16>(g, u, K, ngroups, dense_groups_used, st);
    case 32: return launch_hot<32>(g, u, K, ngroups, dense_groups_used, st);
    case 64: return launch_hot<64>(g, u, K, ngroups, dense_groups_used, st);
  }
  return DLRM_ERR_BAD_SHAPE;
}

}  // namespace dlrm
