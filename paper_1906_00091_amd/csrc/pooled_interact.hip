// The forward of the sparse side in one launch: pooled lookups (Sec. 2.1.1, Eq. (1)-(2)), the
// dense vector placed beside them and the dot interaction over the F = K + 1 vectors (Sec. 2.2).
//
// For one-hot and other short-bag batches the three separate launches are latency-bound and
// the interaction re-reads the T it has just been handed.  Here one wavefront owns a sample:
// lane (i = l%16, h = l/16) pools, for every block of 16 tables, the 4 columns 16q + 4h of
// table 16*rb + i's bag straight into the register layout v_mfma_f32_16x16x4_f32 wants (the
// layout of the interaction kernel in interact.hip), writes them to T (the backward reads T),
// and multiplies.  Each lane walks its own bag, so a wavefront takes as long as its longest
// bag: meant for mean bag lengths of a few rows; longer bags go through the separate kernels.
#include "common.h"

namespace dlrm {

constexpr int kPiThreads = 256;
constexpr int kPiWaves = kPiThreads / DLRM_WAVE;  // samples per workgroup
constexpr int kPiMaxNB = 4;                       // blocks of 16 tables: K <= 64
constexpr double kPiMaxMeanBag = 4.0;             // AUTO fuses up to this mean bag length

struct PiArgs {
  void* const* tables;
  const void* indices;
  const int64_t* offsets;
  const int64_t* tbl_off;
  const float* x;
  float* T;
  float* R;
  int32_t K, B, d, pstride;
  uint32_t* stamp;       // optional: see stamp_start
  uint32_t stamp_value;
};

// table elements col .. col+3 of the row at `row`, widened to fp32 (col a multiple of 4)
template <int DT>
__device__ inline f32x4 load_row4(const char* row, int col) {
  if constexpr (DT == DLRM_F32) {
    return loadf4(reinterpret_cast<const float*>(row) + col);
  } else {
    const u32x2 v = *reinterpret_cast<const u32x2*>(row + col * 2);
    f32x4 f;
    float a, b, c, e;
    if constexpr (DT == DLRM_F16) {
      half2_to_float2(v.x, a, b);
      half2_to_float2(v.y, c, e);
    } else {
      bf162_to_float2(v.x, a, b);
      bf162_to_float2(v.y, c, e);
    }
    f.x = a;
    f.y = b;
    f.z = c;
    f.w = e;
    return f;
  }
}

template <int NB, int DT, typename IT>
__global__ __launch_bounds__(kPiThreads, NB <= 2 ? 4 : 2) void pooled_interact_fwd_kernel(PiArgs a) {
  constexpr int QC = NB <= 2 ? 4 : 2;  // 16-column chunks per round
  constexpr int NTILE = NB * (NB + 1) / 2;
  constexpr int EB = Tab<DT>::EB;
  extern __shared__ float lds[];
  stamp_start(a.stamp, a.stamp_value);
  const int lane = lane_id();
  const int b = blockIdx.x * kPiWaves + wave_id();
  if (b >= a.B) return;  // wavefronts are independent: no barriers below
  const int i = lane & 15, h = lane >> 4;
  const int K = a.K, F = K + 1, d = a.d;
  const int P = F * (F - 1) / 2;
  const float* xb = a.x + (int64_t)b * d;
  float* Tb = a.T ? a.T + (int64_t)b * F * d : nullptr;  // NULL: the caller's backward pools again
  float* Rb = a.R + (int64_t)b * ((int64_t)d + P);
  const int64_t row_bytes = (int64_t)d * EB;

  // this lane's bag in every block of 16 tables; lanes past the last table own an empty bag,
  // whose zero vector only meets interaction entries that are never stored
  const char* W[NB];
  const IT* idx[NB];
  int64_t p0[NB], p1[NB], r0[NB];
#pragma unroll
  for (int rb = 0; rb < NB; ++rb) {
    const int e = rb * 16 + i;
    const int ec = e < K ? e : K - 1;
    const int64_t* off = a.offsets + (int64_t)ec * (a.B + 1);
    p0[rb] = off[b];
    p1[rb] = e < K ? off[b + 1] : p0[rb];
    idx[rb] = static_cast<const IT*>(a.indices) + a.tbl_off[ec];
    W[rb] = static_cast<const char*>(a.tables[ec]);
  }
#pragma unroll
  for (int rb = 0; rb < NB; ++rb) r0[rb] = p1[rb] > p0[rb] ? (int64_t)idx[rb][p0[rb]] : 0;  // row 0 exists, dropped

  f32x4 acc[NTILE];
#pragma unroll
  for (int t = 0; t < NTILE; ++t) acc[t] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
  float pd[NB];  // partial products with the dense vector
#pragma unroll
  for (int rb = 0; rb < NB; ++rb) pd[rb] = 0.0f;

  for (int k0 = 0; k0 < d; k0 += 16 * QC) {
    f32x4 x0[QC], x[NB][QC];
    const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
    // first position of every bag: all loads of the round in flight together (a one-index bag,
    // the common case, is done after this and is a bit copy of its row)
#pragma unroll
    for (int q = 0; q < QC; ++q) {
      const int col = k0 + 16 * q + 4 * h;
      const int ccol = col < d ? col : 0;
      const f32x4 v0 = loadf4(xb + ccol);
      x0[q] = col < d ? v0 : zero;
#pragma unroll
      for (int rb = 0; rb < NB; ++rb) {
        const f32x4 v = load_row4<DT>(W[rb] + r0[rb] * row_bytes, ccol);
        x[rb][q] = (col < d && p1[rb] > p0[rb]) ? v : zero;  // columns past d contribute 0 * 0
      }
    }
    // the rest of the bag, positions in ascending order
#pragma unroll
    for (int rb = 0; rb < NB; ++rb) {
      for (int64_t p = p0[rb] + 1; p < p1[rb]; ++p) {
        const char* row = W[rb] + (int64_t)idx[rb][p] * row_bytes;
#pragma unroll
        for (int q = 0; q < QC; ++q) {
          const int col = k0 + 16 * q + 4 * h;
          const f32x4 v = load_row4<DT>(row, col < d ? col : 0);
          if (col < d) x[rb][q] += v;
        }
      }
    }
    // T_b: the dense vector (lanes i == 0) and the pooled vectors
#pragma unroll
    for (int q = 0; q < QC; ++q) {
      const int col = k0 + 16 * q + 4 * h;
      if (col >= d || Tb == nullptr) continue;
      if (i == 0) storef4(Tb + col, x0[q]);
#pragma unroll
      for (int rb = 0; rb < NB; ++rb) {
        const int e = rb * 16 + i;
        if (e < K) storef4(Tb + (int64_t)(e + 1) * d + col, x[rb][q]);
      }
    }
#pragma unroll
    for (int q = 0; q < QC; ++q) {
      if (k0 + 16 * q < d) {  // uniform
#pragma unroll
        for (int rb = 0; rb < NB; ++rb) {
          pd[rb] = fmaf(x[rb][q].x, x0[q].x, pd[rb]);
          pd[rb] = fmaf(x[rb][q].y, x0[q].y, pd[rb]);
          pd[rb] = fmaf(x[rb][q].z, x0[q].z, pd[rb]);
          pd[rb] = fmaf(x[rb][q].w, x0[q].w, pd[rb]);
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          int tile = 0;
#pragma unroll
          for (int ib = 0; ib < NB; ++ib) {
#pragma unroll
            for (int jb = 0; jb <= ib; ++jb, ++tile)
              acc[tile] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[ib][q][t], x[jb][q][t], acc[tile], 0, 0, 0);
          }
        }
      }
    }
  }
  // pairs gathered in this wavefront's LDS so that they leave as whole contiguous lines;
  // pair (gi, gj), gi > gj, sits at gi(gi-1)/2 + gj, table e being vector e + 1
  float* Rp = lds + wave_id() * a.pstride;
#pragma unroll
  for (int rb = 0; rb < NB; ++rb) {
    float v = pd[rb];
    v += __shfl_xor(v, 16, DLRM_WAVE);
    v += __shfl_xor(v, 32, DLRM_WAVE);
    const int e = rb * 16 + i;
    if (h == 0 && e < K) Rp[(e + 1) * e / 2] = v;
  }
  int tile = 0;
#pragma unroll
  for (int ib = 0; ib < NB; ++ib) {
#pragma unroll
    for (int jb = 0; jb <= ib; ++jb, ++tile) {
      const int ej = jb * 16 + i;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int ei = ib * 16 + 4 * h + v;
        if (ej < ei && ei < K) Rp[(ei + 1) * ei / 2 + ej + 1] = acc[tile][v];
      }
    }
  }
  for (int c = lane; c < d; c += DLRM_WAVE) Rb[c] = xb[c];  // dense part: exact copy
  for (int c = lane; c < P; c += DLRM_WAVE) Rb[d + c] = Rp[c];
}

template <int NB, int DT, typename IT>
static int launch_pi(const PiArgs& a, hipStream_t st) {
  const size_t lds = (size_t)kPiWaves * a.pstride * 4;  // <= 4 * 2080 * 4 bytes
  hipLaunchKernelGGL((pooled_interact_fwd_kernel<NB, DT, IT>), dim3(div_up(a.B, kPiWaves)), dim3(kPiThreads), lds,
                     st, a);
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}

template <int DT, typename IT>
static int dispatch_nb(const PiArgs& a, hipStream_t st) {
  switch (a.K <= 16 ? 1 : (a.K + 15) / 16) {
    case 1: return launch_pi<1, DT, IT>(a, st);
    case 2: return launch_pi<2, DT, IT>(a, st);
    case 3: return launch_pi<3, DT, IT>(a, st);
    case 4: return launch_pi<4, DT, IT>(a, st);
  }
  return DLRM_ERR_BAD_SHAPE;
}

template <int DT>
static int dispatch_it(const PiArgs& a, bool idx32, hipStream_t st) {
  return idx32 ? dispatch_nb<DT, int32_t>(a, st) : dispatch_nb<DT, int64_t>(a, st);
}

// CW consecutive floats (CW = 2 or 4, address CW*4-byte aligned) <-> registers; zeros if !ok
typedef float f32x2 __attribute__((ext_vector_type(2)));
template <int CW>
__device__ inline void load_cols(const float* p, bool ok, float* out) {
  if constexpr (CW == 4) {
    const f32x4 v = loadf4(p);
    out[0] = ok ? v.x : 0.0f;
    out[1] = ok ? v.y : 0.0f;
    out[2] = ok ? v.z : 0.0f;
    out[3] = ok ? v.w : 0.0f;
  } else {
    const f32x2 v = *reinterpret_cast<const f32x2*>(p);
    out[0] = ok ? v.x : 0.0f;
    out[1] = ok ? v.y : 0.0f;
  }
}
template <int CW>
__device__ inline void store_cols(float* p, const float* v) {
  if constexpr (CW == 4) {
    storef4(p, f32x4{v[0], v[1], v[2], v[3]});
  } else {
    *reinterpret_cast<f32x2*>(p) = f32x2{v[0], v[1]};
  }
}

// --- backward without T ---------------------------------------------------------------------
// dT_b = G T_b as in interact_bwd_kernel (interact.hip: same operand layout, same instructions in the
// same order), but the rows of T_b are not read from memory: the B operand of contraction step s,
// embedding row e = 4s + l/16, is pooled again from table e's bag of this sample (rows added one by
// one in ascending position order, exactly as the forward kernel above forms T), and row 0 is the
// dense vector x_b.  A training step that uses this pair never writes or reads T: per sample F*d
// floats less written by the forward and F*d less read here, against the bag's rows read twice
// (the second time mostly from cache).  Meant for the same short-bag batches as the forward kernel.
struct PbArgs {
  void* const* tables;
  const void* indices;
  const int64_t* offsets;
  const int64_t* tbl_off;
  const float* x;
  const float* dR;
  float* dT;
  int32_t K, B, d, gstride;
};

constexpr int kPbInfoWords = 4;  // per bag in LDS: length, first position (global), table base lo / hi

// CW (4 or 2) consecutive table elements from a device address held as an integer, widened to fp32
template <int DT, int CW>
__device__ inline void gload_cols(uint64_t addr, float* out) {
  typedef const __attribute__((address_space(1))) f32x4* g16;
  typedef const __attribute__((address_space(1))) u32x2* g8;
  typedef const __attribute__((address_space(1))) uint32_t* g4;
  if constexpr (DT == DLRM_F32) {
    if constexpr (CW == 4) {
      const f32x4 v = *(g16)addr;
      out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
    } else {
      const u32x2 v = *(g8)addr;
      out[0] = u2f(v.x); out[1] = u2f(v.y);
    }
  } else {
    uint32_t w0, w1 = 0;
    if constexpr (CW == 4) {
      const u32x2 v = *(g8)addr;
      w0 = v.x;
      w1 = v.y;
    } else {
      w0 = *(g4)addr;
    }
    if constexpr (DT == DLRM_F16) {
      half2_to_float2(w0, out[0], out[1]);
      if constexpr (CW == 4) half2_to_float2(w1, out[2], out[3]);
    } else {
      bf162_to_float2(w0, out[0], out[1]);
      if constexpr (CW == 4) bf162_to_float2(w1, out[2], out[3]);
    }
  }
}

template <int NB, int DT, typename IT>
__global__ __launch_bounds__(kPiThreads) void pooled_interact_bwd_kernel(PbArgs a) {
  constexpr int JS = 4 * NB;  // contraction steps of 4 embedding rows
  constexpr int CW = NB <= 2 ? 4 : 2;
  constexpr int EB = Tab<DT>::EB;
  extern __shared__ float lds[];
  const int lane = lane_id();
  const int b = blockIdx.x * kPiWaves + wave_id();
  if (b >= a.B) return;  // wavefronts are independent: no barriers below
  const int x_ = lane & 15, h_ = lane >> 4;
  const int K = a.K, F = K + 1, d = a.d;
  const int P = F * (F - 1) / 2;
  const float* xb = a.x + (int64_t)b * d;
  const float* gR = a.dR + (int64_t)b * ((int64_t)d + P);
  float* dTb = a.dT + (int64_t)b * F * d;
  float* gs = lds + wave_id() * a.gstride;
  uint32_t* binfo = reinterpret_cast<uint32_t*>(lds + kPiWaves * a.gstride) + wave_id() * (16 * kPiMaxNB * kPbInfoWords);
  const uint32_t row_bytes = (uint32_t)d * EB;
  // bag (e, b) of every table e, described once per wavefront by lane e
  for (int e = lane; e < K; e += DLRM_WAVE) {
    const int64_t* off = a.offsets + (int64_t)e * (a.B + 1);
    const int64_t p0 = off[b], p1 = off[b + 1];
    const uint64_t W = reinterpret_cast<uint64_t>(a.tables[e]);
    binfo[e * kPbInfoWords + 0] = (uint32_t)(p1 - p0);
    binfo[e * kPbInfoWords + 1] = (uint32_t)(a.tbl_off[e] + p0);   // < 2^31
    binfo[e * kPbInfoWords + 2] = (uint32_t)W;
    binfo[e * kPbInfoWords + 3] = (uint32_t)(W >> 32);
  }
  for (int t0 = 0; t0 < P; t0 += DLRM_WAVE * 16) {  // the sample's pair gradients: 16 loads in flight per lane
    float v[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int idx = t0 + q * DLRM_WAVE + lane;
      v[q] = gR[d + (idx < P ? idx : P - 1)];
    }
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int idx = t0 + q * DLRM_WAVE + lane;
      if (idx < P) gs[idx] = v[q];
    }
  }
  __builtin_amdgcn_wave_barrier();  // the LDS writes above are read by other lanes of this wavefront below
  const IT* indices = static_cast<const IT*>(a.indices);
  for (int g0 = 0; g0 < d; g0 += 16 * CW) {
    int x = x_, h = h_;
    asm volatile("" : "+v"(x), "+v"(h));   // (see interact_bwd_kernel: keeps per-round values out of registers)
    const int col = g0 + CW * x;
    const bool cok = col < d;
    const int ccol = cok ? col : 0;
    float tb[JS][CW], t0v[CW];
    load_cols<CW>(xb + ccol, cok, t0v);
    // first row of every bag: all in flight together (a one-index bag is done after this)
    uint32_t len[JS], pos[JS];
    uint64_t Wc[JS];
#pragma unroll
    for (int s = 0; s < JS; ++s) {
      const int e = 4 * s + h;
      const int ec = e < K ? e : K - 1;
      len[s] = e < K ? binfo[ec * kPbInfoWords + 0] : 0u;
      pos[s] = binfo[ec * kPbInfoWords + 1];
      Wc[s] = (((uint64_t)binfo[ec * kPbInfoWords + 3] << 32) | binfo[ec * kPbInfoWords + 2]) + (uint64_t)ccol * EB;
    }
    uint32_t r0[JS];
#pragma unroll
    for (int s = 0; s < JS; ++s) r0[s] = len[s] > 0 ? (uint32_t)indices[pos[s]] : 0u;   // row 0 exists, dropped
#pragma unroll
    for (int s = 0; s < JS; ++s) {
      float v[CW];
      gload_cols<DT, CW>(Wc[s] + (uint64_t)r0[s] * row_bytes, v);
#pragma unroll
      for (int c = 0; c < CW; ++c) tb[s][c] = (len[s] > 0 && cok) ? v[c] : 0.0f;
    }
    // the rest of each bag, positions in ascending order
#pragma unroll
    for (int s = 0; s < JS; ++s) {
      for (uint32_t p = 1; p < len[s]; ++p) {
        float v[CW];
        gload_cols<DT, CW>(Wc[s] + (uint64_t)(uint32_t)indices[pos[s] + p] * row_bytes, v);
#pragma unroll
        for (int c = 0; c < CW; ++c)
          if (cok) tb[s][c] += v[c];
      }
    }
    // gradient of the dense row: dR[0:d] + sum_e g(e+1, 0) S_e; g(e+1, 0) sits at (e+1)e/2
    {
      float a0[CW];
#pragma unroll
      for (int c = 0; c < CW; ++c) a0[c] = 0.0f;
#pragma unroll
      for (int s = 0; s < JS; ++s) {
        const int e = 4 * s + h;
        const float gv = gs[e < K ? (e + 1) * e / 2 : 0];
        const float g0e = e < K ? gv : 0.0f;
#pragma unroll
        for (int c = 0; c < CW; ++c) a0[c] = fmaf(g0e, tb[s][c], a0[c]);
      }
#pragma unroll
      for (int c = 0; c < CW; ++c) {
        a0[c] += __shfl_xor(a0[c], 16, DLRM_WAVE);
        a0[c] += __shfl_xor(a0[c], 32, DLRM_WAVE);
      }
      if (h == 0 && cok) {
#pragma unroll
        for (int c = 0; c < CW; ++c) a0[c] += gR[col + c];
        store_cols<CW>(dTb + col, a0);
      }
    }
#pragma unroll(NB <= 2 ? NB : 1)
    for (int ib = 0; ib < NB; ++ib) {
      if (ib * 16 >= K) break;  // uniform
      const int m = ib * 16 + x;
      float ga[JS];
#pragma unroll
      for (int s = 0; s < JS; ++s) {
        const int e = 4 * s + h;
        const int hi = m > e ? m : e, lo = m > e ? e : m;
        const bool ok = hi < K && hi != lo;
        const float gv = gs[ok ? (hi + 1) * hi / 2 + lo + 1 : 0];
        ga[s] = ok ? gv : 0.0f;
      }
      float gd[4];  // g(row, 0) of this lane's 4 output rows
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int ei = ib * 16 + 4 * h + v;
        const float gv = gs[ei < K ? (ei + 1) * ei / 2 : 0];
        gd[v] = ei < K ? gv : 0.0f;
      }
      f32x4 acc[CW];
#pragma unroll
      for (int u = 0; u < CW; ++u) acc[u] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int s = 0; s < JS; ++s) {
        if (4 * s < K) {  // uniform
#pragma unroll
          for (int u = 0; u < CW; ++u) acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(ga[s], tb[s][u], acc[u], 0, 0, 0);
        }
      }
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int ei = ib * 16 + 4 * h + v;
        if (ei < K && cok) {
          float o[CW];
#pragma unroll
          for (int u = 0; u < CW; ++u) o[u] = fmaf(gd[v], t0v[u], acc[u][v]);
          store_cols<CW>(dTb + (int64_t)(ei + 1) * d + col, o);
        }
      }
    }
  }
}

template <int NB, int DT, typename IT>
static int launch_pb(const PbArgs& a, hipStream_t st) {
  const size_t lds = (size_t)kPiWaves * a.gstride * 4 + (size_t)kPiWaves * 16 * kPiMaxNB * kPbInfoWords * 4;
  hipLaunchKernelGGL((pooled_interact_bwd_kernel<NB, DT, IT>), dim3(div_up(a.B, kPiWaves)), dim3(kPiThreads), lds,
                     st, a);
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}

template <int DT, typename IT>
static int dispatch_pb(const PbArgs& a, hipStream_t st) {
  switch (a.K <= 16 ? 1 : (a.K + 15) / 16) {
    case 1: return launch_pb<1, DT, IT>(a, st);
    case 2: return launch_pb<2, DT, IT>(a, st);
    case 3: return launch_pb<3, DT, IT>(a, st);
    case 4: return launch_pb<4, DT, IT>(a, st);
  }
  return DLRM_ERR_BAD_SHAPE;
}

int check_batch(const dlrm_sparse_batch* s);  // util.hip
int emb_fwd_enqueue(const dlrm_sparse_batch* s, float* out, int64_t stride_b, int64_t stride_k, const float* x,
                    uint32_t* stamp, uint32_t stamp_value, void* stream);   // emb_fwd.hip

}  // namespace dlrm

extern "C" int32_t dlrm_emb_interact_fwd(const dlrm_sparse_batch* s, const float* x, float* T, float* R,
                                         int32_t algo, void* stream) {
  return dlrm_emb_interact_fwd_stamped(s, x, T, R, algo, nullptr, 0u, stream);
}

extern "C" int32_t dlrm_emb_interact_fwd_stamped(const dlrm_sparse_batch* s, const float* x, float* T, float* R,
                                                 int32_t algo, uint32_t* stamp, uint32_t stamp_value,
                                                 void* stream) {
  using namespace dlrm;
  int st = check_batch(s);
  if (st != DLRM_OK) return st;
  if (!x || !R) return DLRM_ERR_NULL;
  if (s->K + 1 > DLRM_MAX_INTERACT_F || (s->d & 3)) return DLRM_ERR_BAD_SHAPE;
  if ((reinterpret_cast<uintptr_t>(x) & 15) || (reinterpret_cast<uintptr_t>(T) & 15)) return DLRM_ERR_BAD_SHAPE;
  if (algo != DLRM_FWD_AUTO && algo != DLRM_FWD_FUSED && algo != DLRM_FWD_SPLIT) return DLRM_ERR_BAD_ALGO;
  const int F = s->K + 1;
  const bool can_fuse = s->weights == nullptr && s->K <= 16 * kPiMaxNB;
  if (algo == DLRM_FWD_FUSED && !can_fuse) return DLRM_ERR_BAD_ALGO;
  if (algo == DLRM_FWD_AUTO) {
    const double mean_len = (double)s->nnz_total / ((double)s->K * s->B);
    algo = can_fuse && mean_len <= kPiMaxMeanBag ? DLRM_FWD_FUSED : DLRM_FWD_SPLIT;
  }
  if (!T && algo != DLRM_FWD_FUSED) return DLRM_ERR_NULL;  // only the one-launch kernel can do without T
  if (algo == DLRM_FWD_SPLIT) {
    // the dense vectors ride along in the pooling launch
    st = emb_fwd_enqueue(s, T + s->d, (int64_t)F * s->d, s->d, x, stamp, stamp_value, stream);
    if (st != DLRM_OK) return st;
    return dlrm_interact_dot_fwd(T, s->B, F, s->d, R, stream);
  }
  PiArgs a;
  a.tables = s->tables;
  a.indices = s->indices;
  a.offsets = s->offsets;
  a.tbl_off = s->tbl_off;
  a.x = x;
  a.T = T;
  a.R = R;
  a.K = s->K;
  a.B = s->B;
  a.d = s->d;
  a.stamp = stamp;
  a.stamp_value = stamp_value;
  const int P = F * (F - 1) / 2;
  a.pstride = P < 4 ? 4 : ((P + 3) & ~3);
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const bool idx32 = s->index_dtype == DLRM_I32;
  switch (s->table_dtype) {
    case DLRM_F32: return dispatch_it<DLRM_F32>(a, idx32, hs);
    case DLRM_F16: return dispatch_it<DLRM_F16>(a, idx32, hs);
    case DLRM_BF16: return dispatch_it<DLRM_BF16>(a, idx32, hs);
  }
  return DLRM_ERR_BAD_DTYPE;
}

extern "C" int32_t dlrm_emb_interact_bwd(const dlrm_sparse_batch* s, const float* x, const float* dR, float* dT,
                                         void* stream) {
  using namespace dlrm;
  int st = check_batch(s);
  if (st != DLRM_OK) return st;
  if (!x || !dR || !dT) return DLRM_ERR_NULL;
  if (s->K + 1 > DLRM_MAX_INTERACT_F || (s->d & 3)) return DLRM_ERR_BAD_SHAPE;
  if ((reinterpret_cast<uintptr_t>(x) & 15) || (reinterpret_cast<uintptr_t>(dT) & 15)) return DLRM_ERR_BAD_SHAPE;
  if (s->weights != nullptr || s->K > 16 * kPiMaxNB) return DLRM_ERR_BAD_ALGO;
  const int F = s->K + 1;
  PbArgs a;
  a.tables = s->tables;
  a.indices = s->indices;
  a.offsets = s->offsets;
  a.tbl_off = s->tbl_off;
  a.x = x;
  a.dR = dR;
  a.dT = dT;
  a.K = s->K;
  a.B = s->B;
  a.d = s->d;
  const int P = F * (F - 1) / 2;
  a.gstride = P < 4 ? 4 : ((P + 3) & ~3);
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const bool idx32 = s->index_dtype == DLRM_I32;
  switch (s->table_dtype) {
    case DLRM_F32: return idx32 ? dispatch_pb<DLRM_F32, int32_t>(a, hs) : dispatch_pb<DLRM_F32, int64_t>(a, hs);
    case DLRM_F16: return idx32 ? dispatch_pb<DLRM_F16, int32_t>(a, hs) : dispatch_pb<DLRM_F16, int64_t>(a, hs);
    case DLRM_BF16: return idx32 ? dispatch_pb<DLRM_BF16, int32_t>(a, hs) : dispatch_pb<DLRM_BF16, int64_t>(a, hs);
  }
  return DLRM_ERR_BAD_DTYPE;
}
