// Pooled embedding lookup (Sec. 2.1.1, Eq. (1)-(2)):
// S_k[b,:] = sum over the positions p of bag (k,b) of a_p W_k[idx_p,:]; the weights a are all
// ones unless the batch brings them (WT kernels: one fused multiply-add per element instead
// of an add).
//
// HBM-bound gather.  A table row is d*e bytes; a lane moves 16 bytes
// (global_load_dwordx4), so a row occupies a "lane group" of G = pow2(d*e/16)
// lanes and a 64-wide wavefront carries S = 64/G rows per load instruction.
//   * short kernel: every lane group owns 4 consecutive one-row bags (one-hot batches:
//     a pure gather whose only parallelism is across bags).
//   * group kernel: every lane group owns one bag and walks it with U loads in
//     flight (short bags).
//   * wave kernel : the whole wavefront owns one bag; its 64 indices per chunk are
//     fetched with one coalesced load and handed to the lane groups through
//     cross-lane reads; group s takes positions s, s+S, ...; the S partial sums
//     meet in an xor butterfly over the lane groups.
// All K tables go in one launch (grid over table x bag).
#include "common.h"

namespace dlrm {

struct FwdArgs {
  void* const* tables;
  const void* indices;   // int64 or int32: the kernels are compiled per index type IT
  const int64_t* offsets;
  const int64_t* tbl_off;
  const float* weights;  // NULL or parallel to indices
  float* out;
  int64_t stride_b, stride_k;
  int32_t K, B, d;
  int32_t chunks;  // 16-byte chunks per table row
  // optional rider: workgroups past bag_blocks copy the dense vectors x[B,d] to dense_out + b*stride_b
  // (row 0 of the interaction input), which saves the launch of its own that copy would take
  const float* dense;
  float* dense_out;
  uint32_t bag_blocks;
  uint32_t* stamp;       // optional: see stamp_start
  uint32_t stamp_value;
};

// true for the rider workgroups, after they have done their copy
__device__ inline bool dense_rider(const FwdArgs& a) {
  if (a.dense == nullptr || blockIdx.x < a.bag_blocks) return false;
  const int d4 = a.d / 4;
  const int64_t n4 = (int64_t)a.B * d4;
  const int64_t nthreads = (int64_t)(gridDim.x - a.bag_blocks) * blockDim.x;
  for (int64_t i = (int64_t)(blockIdx.x - a.bag_blocks) * blockDim.x + threadIdx.x; i < n4; i += nthreads) {
    const int64_t b = i / d4, c4 = i - b * d4;
    storef4(a.dense_out + b * a.stride_b + c4 * 4, loadf4(a.dense + i * 4));
  }
  return true;
}

// acc += w * widen(v): the 16 bytes of a row held by this lane.  fp16 rows: fma(x, 1, acc) is the
// same single rounding as acc + x and lets the conversion fold into a mixed-precision multiply-add
// (one instruction per element instead of two; the pooling of fp16 tables is bound by the vector ALUs).
template <int DT, bool WT>
__device__ inline void add_row(float* acc, u32x4 v, float w) {
  constexpr int E = Tab<DT>::ELEMS;
  if constexpr (DT == DLRM_F16) {
    // v_fma_mix_f32: fp32 result of a * b + c where a is the low or high fp16 half of a register, widened
    // exactly; b = w (fp32), c = acc (fp32): one rounding, the same value as acc + w * (float)a computed
    // with a fused multiply-add.  (The compiler turns fma(x, 1, acc) back into convert + add.)
    const uint32_t q[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      asm("v_fma_mix_f32 %0, %1, %2, %0 op_sel_hi:[1,0,0]" : "+v"(acc[2 * i]) : "v"(q[i]), "v"(w));
      asm("v_fma_mix_f32 %0, %1, %2, %0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "+v"(acc[2 * i + 1]) : "v"(q[i]), "v"(w));
    }
  } else {
    float f[E];
    Tab<DT>::widen(v, f);
    if constexpr (WT) {
#pragma unroll
      for (int i = 0; i < E; ++i) acc[i] = fmaf(w, f[i], acc[i]);
    } else {
#pragma unroll
      for (int i = 0; i < E; ++i) acc[i] += f[i];
    }
  }
}

// Rows [0, n) of an index chunk held one per lane in `rows` (weights in `wts`): lane group `slot` adds the
// rows at positions slot, slot + S, ... in ascending order, U row loads in flight.  Wbase: address of this
// lane's 16 bytes of row 0.  Rounds that lie entirely inside the chunk carry no per-lane bounds logic.
template <int DT, int G, int U, bool WT>
__device__ inline void gather_chunk(float* acc, uint64_t Wbase, uint32_t row_bytes, uint32_t rows, float wts, int n,
                                    int slot) {
  constexpr int S = DLRM_WAVE / G;
  const int iters = (n + S - 1) / S;
  const int full = n / S;  // rounds in which every lane group has a row
  int q = 0;
  for (; q + U <= full; q += U) {
    u32x4 v[U];
    float wt[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int e = (q + u) * S + slot;
      const uint32_t r = (uint32_t)__shfl((int)rows, e, DLRM_WAVE);
      wt[u] = 1.0f;
      if constexpr (WT) wt[u] = __shfl(wts, e, DLRM_WAVE);
      v[u] = load16_global(Wbase + (uint64_t)r * row_bytes);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) add_row<DT, WT>(acc, v[u], wt[u]);
  }
  for (; q < iters; q += U) {   // the tail: branch-free, positions past the end re-read n - 1 and add the identity
    u32x4 v[U];
    float wt[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int e = (q + u) * S + slot;
      const uint32_t r = (uint32_t)__shfl((int)rows, e < n ? e : n - 1, DLRM_WAVE);
      wt[u] = 1.0f;
      if constexpr (WT) wt[u] = __shfl(wts, e < n ? e : n - 1, DLRM_WAVE);
      v[u] = load16_global(Wbase + (uint64_t)r * row_bytes);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool past = (q + u) * S + slot >= n;
      if (past) {
        v[u] = Tab<DT>::ident();
        wt[u] = 1.0f;   // 1 * (-0) leaves the sum alone
      }
      add_row<DT, WT>(acc, v[u], wt[u]);
    }
  }
}

template <int DT>
__device__ inline void write_pooled(float* o, const float* acc) {
  constexpr int E = Tab<DT>::ELEMS;
#pragma unroll
  for (int i = 0; i < E; i += 4) storef4(o + i, f32x4{acc[i], acc[i + 1], acc[i + 2], acc[i + 3]});
}

// ---------------------------------------------------------------------------
template <int DT, int G, int U, bool WT, typename IT>
__global__ __launch_bounds__(256) void emb_fwd_group_kernel(FwdArgs a) {
  stamp_start(a.stamp, a.stamp_value);
  if (dense_rider(a)) return;  // workgroup-uniform
  constexpr int E = Tab<DT>::ELEMS;
  constexpr int S = DLRM_WAVE / G;
  const int lane = lane_id();
  const int slot = lane / G, chunk = lane % G;
  // K*(B+1) < 2^31 is checked on the host, so 32-bit bag arithmetic is exact
  const uint32_t bag = (blockIdx.x * (blockDim.x >> 6) + wave_id()) * S + slot;
  if (bag >= (uint32_t)a.K * (uint32_t)a.B || chunk >= a.chunks) return;  // no cross-lane ops below
  const int k = (int)(bag / (uint32_t)a.B), b = (int)(bag - (uint32_t)k * (uint32_t)a.B);
  const int64_t* off = a.offsets + (int64_t)k * (a.B + 1);
  const int64_t p0 = off[b], p1 = off[b + 1];
  const IT* idx = static_cast<const IT*>(a.indices) + a.tbl_off[k];
  const float* wts = WT ? a.weights + a.tbl_off[k] : nullptr;
  const char* W = static_cast<const char*>(a.tables[k]) + chunk * 16;
  const int64_t row_bytes = (int64_t)a.chunks * 16;

  float acc[E];
#pragma unroll
  for (int i = 0; i < E; ++i) acc[i] = -0.0f;

  for (int64_t p = p0; p < p1; p += U) {
    // all U index loads, then all U row loads, are issued before anything is consumed; the
    // tail re-reads the bag's last position (in cache) and is replaced by the identity
    int64_t r[U];
    u32x4 v[U];
    float wt[U];
#pragma unroll
    for (int u = 0; u < U; ++u) r[u] = idx[p + u < p1 ? p + u : p1 - 1];
    if constexpr (WT) {
#pragma unroll
      for (int u = 0; u < U; ++u) wt[u] = wts[p + u < p1 ? p + u : p1 - 1];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = load16(W + r[u] * row_bytes);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (p + u >= p1) v[u] = Tab<DT>::ident();
      float f[E];
      Tab<DT>::widen(v[u], f);
      if constexpr (WT) {
        const float w1 = p + u >= p1 ? 1.0f : wt[u];  // 1 * (-0) leaves the sum alone
#pragma unroll
        for (int i = 0; i < E; ++i) acc[i] = fmaf(w1, f[i], acc[i]);
      } else {
#pragma unroll
        for (int i = 0; i < E; ++i) acc[i] += f[i];
      }
    }
  }
  if (p1 <= p0) {
#pragma unroll
    for (int i = 0; i < E; ++i) acc[i] = 0.0f;
  }
  write_pooled<DT>(a.out + (int64_t)b * a.stride_b + (int64_t)k * a.stride_k + chunk * E, acc);
}

// ---------------------------------------------------------------------------
// One-hot and near one-hot batches: a bag is one row, so a lane group that owns a single bag
// has one dependent chain (offsets -> index -> row) and nothing else in flight.  Here it owns
// NB consecutive bags and walks their chains side by side.
template <int DT, int G, int NB, bool WT, typename IT>
__global__ __launch_bounds__(256) void emb_fwd_short_kernel(FwdArgs a) {
  stamp_start(a.stamp, a.stamp_value);
  if (dense_rider(a)) return;  // workgroup-uniform
  constexpr int E = Tab<DT>::ELEMS;
  constexpr int S = DLRM_WAVE / G;
  const int lane = lane_id();
  const int slot = lane / G, chunk = lane % G;
  const uint32_t nbags = (uint32_t)a.K * (uint32_t)a.B;
  const uint32_t bag0 = ((blockIdx.x * (blockDim.x >> 6) + wave_id()) * S + slot) * NB;
  if (bag0 >= nbags || chunk >= a.chunks) return;  // no cross-lane ops below
  const int64_t row_bytes = (int64_t)a.chunks * 16;
  int k[NB], b[NB];
  int64_t p0[NB], p1[NB];
  const IT* idx[NB];
  int64_t tb[NB];
  const char* W[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    const uint32_t bag = bag0 + j < nbags ? bag0 + j : nbags - 1;  // the tail repeats the last bag
    k[j] = (int)(bag / (uint32_t)a.B);
    b[j] = (int)(bag - (uint32_t)k[j] * (uint32_t)a.B);
    const int64_t* off = a.offsets + (int64_t)k[j] * (a.B + 1);
    p0[j] = off[b[j]];
    p1[j] = off[b[j] + 1];
    tb[j] = a.tbl_off[k[j]];
    idx[j] = static_cast<const IT*>(a.indices) + tb[j];
    W[j] = static_cast<const char*>(a.tables[k[j]]) + chunk * 16;
  }
  int64_t r[NB];
  float w0[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    r[j] = 0;  // an empty bag fetches row 0 (every table has one) and drops it
    w0[j] = 1.0f;
    if (p1[j] > p0[j]) {
      r[j] = idx[j][p0[j]];
      if constexpr (WT) w0[j] = a.weights[tb[j] + p0[j]];
    }
  }
  u32x4 v[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j) v[j] = load16(W[j] + r[j] * row_bytes);
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    if (bag0 + j >= nbags) continue;
    float acc[E];
    Tab<DT>::widen(v[j], acc);  // a one-index bag is a bit copy of its row
    if constexpr (WT) {
#pragma unroll
      for (int i = 0; i < E; ++i) acc[i] *= w0[j];
    }
    if (p1[j] <= p0[j]) {
#pragma unroll
      for (int i = 0; i < E; ++i) acc[i] = 0.0f;
    }
    for (int64_t p = p0[j] + 1; p < p1[j]; ++p) {  // the occasional longer bag
      float f[E];
      Tab<DT>::widen(load16(W[j] + (int64_t)idx[j][p] * row_bytes), f);
      const float w1 = WT ? a.weights[tb[j] + p] : 1.0f;
#pragma unroll
      for (int i = 0; i < E; ++i) acc[i] = WT ? fmaf(w1, f[i], acc[i]) : acc[i] + f[i];
    }
    write_pooled<DT>(a.out + (int64_t)b[j] * a.stride_b + (int64_t)k[j] * a.stride_k + chunk * E, acc);
  }
}

// ---------------------------------------------------------------------------
template <int DT, int G, int U, bool WT, typename IT>
__global__ __launch_bounds__(256) void emb_fwd_wave_kernel(FwdArgs a) {
  stamp_start(a.stamp, a.stamp_value);
  if (dense_rider(a)) return;  // workgroup-uniform
  constexpr int E = Tab<DT>::ELEMS;
  constexpr int S = DLRM_WAVE / G;
  const int lane = lane_id();
  const int slot = lane / G, chunk = lane % G;
  const uint32_t bag = blockIdx.x * (blockDim.x >> 6) + wave_id();
  if (bag >= (uint32_t)a.K * (uint32_t)a.B) return;  // wave-uniform
  const int k = (int)(bag / (uint32_t)a.B), b = (int)(bag - (uint32_t)k * (uint32_t)a.B);
  const int64_t* off = a.offsets + (int64_t)k * (a.B + 1);
  const int64_t p0 = off[b], p1 = off[b + 1];
  const int64_t pos0 = a.tbl_off[k] + p0;
  const IT* idx = static_cast<const IT*>(a.indices) + pos0;
  const bool col_ok = chunk < a.chunks;
  // lanes past the row's last chunk shadow chunk 0 (same address, no extra traffic) and never write
  const char* W = static_cast<const char*>(a.tables[k]) + (col_ok ? chunk : 0) * 16;
  const int64_t row_bytes = (int64_t)a.chunks * 16;
  const int64_t len = p1 - p0;

  float acc[E];
#pragma unroll
  for (int i = 0; i < E; ++i) acc[i] = -0.0f;

  for (int64_t base = 0; base < len; base += DLRM_WAVE) {
    const int n = (int)((len - base) < DLRM_WAVE ? (len - base) : DLRM_WAVE);
    // one coalesced fetch of this chunk's indices; rows are < 2^31
    const uint32_t my_row = (uint32_t)idx[base + (lane < n ? lane : n - 1)];
    float my_wt = 1.0f;
    if constexpr (WT) my_wt = a.weights[pos0 + base + (lane < n ? lane : n - 1)];
    gather_chunk<DT, G, U, WT>(acc, reinterpret_cast<uint64_t>(W), (uint32_t)row_bytes, my_row, my_wt, n, slot);
  }
  // combine the S lane groups: xor butterfly, identical result in every group
#pragma unroll
  for (int o = G; o < DLRM_WAVE; o <<= 1) {
#pragma unroll
    for (int i = 0; i < E; ++i) acc[i] += __shfl_xor(acc[i], o, DLRM_WAVE);
  }
  if (slot != 0 || !col_ok) return;
  if (len <= 0) {
#pragma unroll
    for (int i = 0; i < E; ++i) acc[i] = 0.0f;
  }
  write_pooled<DT>(a.out + (int64_t)b * a.stride_b + (int64_t)k * a.stride_k + chunk * E, acc);
}

// ---------------------------------------------------------------------------
// A wavefront per bag as above, but the wavefront walks NBW consecutive bags and keeps the index
// chunk of the NEXT bag (or of the next 64 positions of a long bag) in flight while it gathers the
// rows of the current one.  With one bag per wavefront a bag of a few dozen rows is a chain of
// dependent round trips (offsets -> indices -> rows) with little to overlap; here the offsets and
// table bases of all NBW bags are fetched up front by the lanes (lane j holds bag j), and per bag
// only the row gathers remain on the critical path.  Same additions in the same order as
// emb_fwd_wave_kernel: the results are identical bit for bit.
template <int DT, int G, int U, bool WT, typename IT>
__global__ __launch_bounds__(256) void emb_fwd_wave_seq_kernel(FwdArgs a, int nbw) {
  stamp_start(a.stamp, a.stamp_value);
  if (dense_rider(a)) return;  // workgroup-uniform
  constexpr int E = Tab<DT>::ELEMS;
  constexpr int S = DLRM_WAVE / G;
  const int lane = lane_id();
  const int slot = lane / G, chunk = lane % G;
  const uint32_t nbags = (uint32_t)a.K * (uint32_t)a.B;
  const uint32_t bag0 = (blockIdx.x * (blockDim.x >> 6) + wave_id()) * (uint32_t)nbw;
  if (bag0 >= nbags) return;  // wave-uniform
  const int nb = (int)(nbags - bag0 < (uint32_t)nbw ? nbags - bag0 : (uint32_t)nbw);
  const bool col_ok = chunk < a.chunks;
  const int64_t row_bytes = (int64_t)a.chunks * 16;
  // lane j describes bag bag0 + j: table, sample, first position (global), length, table base
  const uint32_t my_bag = bag0 + (uint32_t)(lane < nb ? lane : nb - 1);
  const int my_k = (int)(my_bag / (uint32_t)a.B), my_b = (int)(my_bag - (uint32_t)my_k * (uint32_t)a.B);
  const int64_t* off = a.offsets + (int64_t)my_k * (a.B + 1);
  const int64_t my_p0 = off[my_b], my_p1 = off[my_b + 1];
  const uint64_t my_pos = (uint64_t)(a.tbl_off[my_k] + my_p0);
  const uint32_t my_len = (uint32_t)(my_p1 - my_p0);
  const uint64_t my_W = reinterpret_cast<uint64_t>(a.tables[my_k]);
  auto bcast64 = [](uint64_t v, int j) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, j);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), j);
    return ((uint64_t)hi << 32) | lo;
  };
  // the index chunk [base, base + 64) of bag j: one coalesced fetch; rows are < 2^31
  auto fetch = [&](int j, uint32_t base, uint32_t& row, float& wt) {
    const uint32_t len = (uint32_t)__builtin_amdgcn_readlane((int)my_len, j);
    if (base >= len) return;  // wave-uniform (an empty bag)
    const uint32_t n = len - base < (uint32_t)DLRM_WAVE ? len - base : (uint32_t)DLRM_WAVE;
    const uint64_t pos = bcast64(my_pos, j) + base + ((uint32_t)lane < n ? (uint32_t)lane : n - 1);
    row = (uint32_t)static_cast<const IT*>(a.indices)[pos];
    if constexpr (WT) wt = a.weights[pos];
  };
  uint32_t cur_row = 0, nxt_row = 0;
  float cur_wt = 1.0f, nxt_wt = 1.0f;
  fetch(0, 0u, cur_row, cur_wt);
  float acc[E];
  int j = 0;
  uint32_t base = 0;
  while (j < nb) {  // wave-uniform
    const uint32_t len = (uint32_t)__builtin_amdgcn_readlane((int)my_len, j);
    int nj = j;
    uint32_t nbase = base + DLRM_WAVE;
    if (nbase >= len) {
      nj = j + 1;
      nbase = 0;
    }
    if (nj < nb) fetch(nj, nbase, nxt_row, nxt_wt);   // in flight while this chunk's rows are gathered
    if (base == 0) {
#pragma unroll
      for (int i = 0; i < E; ++i) acc[i] = -0.0f;
    }
    if (base < len) {
      const int n = (int)(len - base < (uint32_t)DLRM_WAVE ? len - base : (uint32_t)DLRM_WAVE);
      const uint64_t W = bcast64(my_W, j) + (uint64_t)((col_ok ? chunk : 0) * 16);
      gather_chunk<DT, G, U, WT>(acc, W, (uint32_t)row_bytes, cur_row, cur_wt, n, slot);
    }
    if (nbase == 0) {  // the bag is complete: combine the S lane groups (xor butterfly) and store
      float tot[E];
#pragma unroll
      for (int i = 0; i < E; ++i) tot[i] = acc[i];
#pragma unroll
      for (int o = G; o < DLRM_WAVE; o <<= 1) {
#pragma unroll
        for (int i = 0; i < E; ++i) tot[i] += __shfl_xor(tot[i], o, DLRM_WAVE);
      }
      if (len == 0) {
#pragma unroll
        for (int i = 0; i < E; ++i) tot[i] = 0.0f;
      }
      const uint32_t bag = bag0 + (uint32_t)j;
      const int k = (int)(bag / (uint32_t)a.B), b = (int)(bag - (uint32_t)k * (uint32_t)a.B);
      if (slot == 0 && col_ok)
        write_pooled<DT>(a.out + (int64_t)b * a.stride_b + (int64_t)k * a.stride_k + chunk * E, tot);
    }
    j = nj;
    base = nbase;
    cur_row = nxt_row;
    cur_wt = nxt_wt;
  }
}

// ---------------------------------------------------------------------------
constexpr int kShortBags = 4;  // bags per lane group of the short-bag kernel
constexpr int kSeqMaxMeanLen = 64;  // mean bag length below which a wavefront walks several bags

template <int DT, int G, bool WT, typename IT>
static int launch_fwd(const FwdArgs& a_in, int mode, hipStream_t st) {
  constexpr int S = DLRM_WAVE / G;
  const int64_t bags = (int64_t)a_in.K * a_in.B;
  const bool wave_mode = mode == 2;
  FwdArgs a = a_in;
  unsigned riders = 0;
  if (a.dense != nullptr) {
    riders = div_up((int64_t)a.B * (a.d / 4), 256);
    if (riders > 1024) riders = 1024;
  }
  if (mode == 0) {
    a.bag_blocks = div_up(bags, 4 * S * kShortBags);
    hipLaunchKernelGGL((emb_fwd_short_kernel<DT, G, kShortBags, WT, IT>), dim3(a.bag_blocks + riders), dim3(256), 0,
                       st, a);
  } else if (mode == 3) {
    // several bags per wavefront, as many as leaves every compute unit a few dozen wavefronts
    int nbw = (int)(bags / 16384);
    nbw = nbw < 1 ? 1 : nbw > 16 ? 16 : nbw;
    a.bag_blocks = div_up(bags, 4 * nbw);
    hipLaunchKernelGGL((emb_fwd_wave_seq_kernel<DT, G, 8, WT, IT>), dim3(a.bag_blocks + riders), dim3(256), 0, st, a, nbw);
  } else if (wave_mode) {
    // in-flight depth (2..16 rows per lane group; 8 measured 2% ahead of 4) and workgroup size (64 or 256) were swept on the
    // 8 x 1M x 64 multi-hot workload: all within 3% -- the kernel runs at the gather rate of HBM
    a.bag_blocks = div_up(bags, 4);
    hipLaunchKernelGGL((emb_fwd_wave_kernel<DT, G, 8, WT, IT>), dim3(a.bag_blocks + riders), dim3(256), 0, st, a);
  } else {
    a.bag_blocks = div_up(bags, 4 * S);
    hipLaunchKernelGGL((emb_fwd_group_kernel<DT, G, 4, WT, IT>), dim3(a.bag_blocks + riders), dim3(256), 0, st, a);
  }
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}

template <int DT, int G>
static int pick_fwd(const FwdArgs& a, bool idx32, int mode, hipStream_t st) {
  if (a.weights)
    return idx32 ? launch_fwd<DT, G, true, int32_t>(a, mode, st) : launch_fwd<DT, G, true, int64_t>(a, mode, st);
  return idx32 ? launch_fwd<DT, G, false, int32_t>(a, mode, st) : launch_fwd<DT, G, false, int64_t>(a, mode, st);
}

template <int DT>
static int dispatch_g(const FwdArgs& a, int G, bool idx32, int wave_mode, hipStream_t st) {
  switch (G) {
    case 1: return pick_fwd<DT, 1>(a, idx32, wave_mode, st);
    case 2: return pick_fwd<DT, 2>(a, idx32, wave_mode, st);
    case 4: return pick_fwd<DT, 4>(a, idx32, wave_mode, st);
    case 8: return pick_fwd<DT, 8>(a, idx32, wave_mode, st);
    case 16: return pick_fwd<DT, 16>(a, idx32, wave_mode, st);
    case 32: return pick_fwd<DT, 32>(a, idx32, wave_mode, st);
    case 64: return pick_fwd<DT, 64>(a, idx32, wave_mode, st);
  }
  return DLRM_ERR_BAD_SHAPE;
}

int check_batch(const dlrm_sparse_batch* s);  // util.hip

}  // namespace dlrm

namespace dlrm {
// The pooled lookup; with x != NULL the same launch also copies x[B,d] to out - d + b*stride_b
// (the dense vector into row 0 of an interaction input whose rows 1..K are `out`).
int emb_fwd_enqueue(const dlrm_sparse_batch* s, float* out, int64_t stride_b, int64_t stride_k, const float* x,
                    uint32_t* stamp, uint32_t stamp_value, void* stream) {
  int st = check_batch(s);
  if (st != DLRM_OK) return st;
  if (!out) return DLRM_ERR_NULL;
  if (stride_k < s->d || (stride_k & 3) || (stride_b & 3) || stride_b < 0) return DLRM_ERR_BAD_SHAPE;
  if ((reinterpret_cast<uintptr_t>(out) & 15) != 0) return DLRM_ERR_BAD_SHAPE;
  FwdArgs a;
  a.tables = s->tables;
  a.indices = s->indices;
  a.offsets = s->offsets;
  a.tbl_off = s->tbl_off;
  a.weights = s->weights;
  a.out = out;
  a.stride_b = stride_b;
  a.stride_k = stride_k;
  a.K = s->K;
  a.B = s->B;
  a.d = s->d;
  a.chunks = s->d * elem_bytes(s->table_dtype) / 16;
  a.dense = x;
  a.dense_out = x ? out - s->d : nullptr;
  a.bag_blocks = 0;
  a.stamp = stamp;
  a.stamp_value = stamp_value;
  const int G = pow2_ceil(a.chunks);
  const int S = DLRM_WAVE / G;
  // a wavefront per bag pays off once a bag keeps all S lane groups busy for a few rounds
  const double mean_len = (double)s->nnz_total / ((double)s->K * s->B);
  // mode 0: several bags per lane group (mean bag <= 2), 1: a lane group per bag, 2: a wavefront per bag,
  // 3: a wavefront per bag walking several bags with the next bag's indices in flight (bags of up to a
  // few dozen rows, where a bag is a chain of round trips rather than a stream)
  int wave_mode = mean_len <= 2.0 ? 0 : (S > 1 && mean_len >= 2.0 * S) ? 2 : 1;
  if (wave_mode == 2 && mean_len < (double)kSeqMaxMeanLen) wave_mode = 3;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const bool idx32 = s->index_dtype == DLRM_I32;
  switch (s->table_dtype) {
    case DLRM_F32: return dispatch_g<DLRM_F32>(a, G, idx32, wave_mode, hs);
    case DLRM_F16: return dispatch_g<DLRM_F16>(a, G, idx32, wave_mode, hs);
    case DLRM_BF16: return dispatch_g<DLRM_BF16>(a, G, idx32, wave_mode, hs);
  }
  return DLRM_ERR_BAD_DTYPE;
}
}  // namespace dlrm

extern "C" int32_t dlrm_emb_bag_fwd(const dlrm_sparse_batch* s, float* out, int64_t stride_b,
                                    int64_t stride_k, void* stream) {
  return dlrm::emb_fwd_enqueue(s, out, stride_b, stride_k, nullptr, nullptr, 0u, stream);
}
