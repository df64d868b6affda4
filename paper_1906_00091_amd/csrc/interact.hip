// Dot-product feature interaction (Sec. 2.2) and its backward.
//   fwd: R[b] = [ T[b,0,:] | <T[b,i,:],T[b,j,:]> for 1 <= i < F, 0 <= j < i ]
//   bwd: dT[b,i,:] = sum_{j != i} g(i,j) T[b,j,:]  (+ dR[b,0:d] on row 0),
//        g(i,j) = dR[b, d + pair(max(i,j), min(i,j))]
// Both are small dense contractions per sample (Z = T T^t, dT = G T with G symmetric), run on
// the matrix cores in fp32: v_mfma_f32_16x16x4_f32, one wavefront per sample, operands loaded
// straight from global memory into the register layout the instruction wants (no LDS staging
// of T, no workgroup barriers), so HBM sees each input and output once.
//   16x16x4 layout: lane l supplies A[m = l%16][k = l/16] and B[k = l/16][n = l%16] and holds
//   D[m = 4*(l/16) + v][n = l%16] in element v of its accumulator.
// The contraction index may be visited in any order as long as A and B agree on it, which is
// what lets every lane fetch 16 contiguous bytes and use them in 4 consecutive instructions.
#include "common.h"

namespace dlrm {

constexpr int kIntThreads = 256;
constexpr int kIntWaves = kIntThreads / DLRM_WAVE;   // samples per workgroup

__device__ inline f32x4 mfma16(float a, float b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// --- forward --------------------------------------------------------------------------------
// Row 0 of T_b (the dense vector) is kept apart; the K = F-1 embedding rows form NB blocks of
// 16.  Lane (i = l%16, h = l/16) fetches, for every row block, the 4 floats at columns 16q + 4h
// of embedding row 16*rb + i.  Element t of that float4 is at once the A operand of the row
// block and the B operand of the column block for the 4 columns {16q + 4h' + t : h' = 0..3},
// so a tile (ib, jb) of Z = S S^t takes one instruction per 4 columns; only tiles on or below
// the diagonal are computed.  The K products with the dense row are plain FMAs on the same
// registers (a 17th row would cost a whole extra row and column of tiles).
template <int NB>
__global__ __launch_bounds__(kIntThreads) void interact_fwd_kernel(const float* __restrict__ T,
                                                                    float* __restrict__ R, int B, int F,
                                                                    int d, int pstride) {
  constexpr int QC = NB <= 2 ? 4 : 2;  // 16-column chunks fetched per round
  constexpr int NTILE = NB * (NB + 1) / 2;
  extern __shared__ float lds[];
  const int lane = lane_id();
  const int b = blockIdx.x * kIntWaves + wave_id();
  if (b >= B) return;  // wavefronts are independent: no barriers below
  const int i = lane & 15, h = lane >> 4;
  const int K = F - 1;
  const int P = F * (F - 1) / 2;
  const float* Tb = T + (int64_t)b * F * d;
  float* Rb = R + (int64_t)b * ((int64_t)d + P);
  f32x4 acc[NTILE];
#pragma unroll
  for (int t = 0; t < NTILE; ++t) acc[t] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
  const float* rowp[NB];
  float pd[NB];  // partial products with the dense row
#pragma unroll
  for (int rb = 0; rb < NB; ++rb) {
    // rows past the last one repeat it (the dense row if there is none): their products land in
    // entries that are never stored
    const int e = rb * 16 + i < K ? rb * 16 + i : K - 1;
    rowp[rb] = Tb + (int64_t)(e + 1) * d;
    pd[rb] = 0.0f;
  }
  for (int k0 = 0; k0 < d; k0 += 16 * QC) {
    f32x4 x0[QC], x[NB][QC];
#pragma unroll
    for (int q = 0; q < QC; ++q) {
      const int col = k0 + 16 * q + 4 * h;
      const int ccol = col < d ? col : 0;
      const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
      const f32x4 v0 = loadf4(Tb + ccol);
      x0[q] = col < d ? v0 : zero;
#pragma unroll
      for (int rb = 0; rb < NB; ++rb) {
        const f32x4 v = loadf4(rowp[rb] + ccol);
        x[rb][q] = col < d ? v : zero;  // columns past d contribute 0 * 0
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
            for (int jb = 0; jb <= ib; ++jb, ++tile) acc[tile] = mfma16(x[ib][q][t], x[jb][q][t], acc[tile]);
          }
        }
      }
    }
  }
  // The accumulator layout scatters the pairs; they are gathered in this wavefront's LDS and
  // leave as whole contiguous lines (partial-line writes cost a fill read each).
  float* Rp = lds + wave_id() * pstride;
  // pair (gi, gj), gi > gj, sits at gi(gi-1)/2 + gj; embedding row e is row e + 1 of T
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
  for (int c = lane; c < d; c += DLRM_WAVE) Rb[c] = Tb[c];  // dense part: exact copy of row 0
  for (int c = lane; c < P; c += DLRM_WAVE) Rb[d + c] = Rp[c];
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

// --- backward -------------------------------------------------------------------------------
// dT_b = G T_b with G the symmetric F x F matrix of pair gradients (zero diagonal), held per
// wavefront in LDS as the lower triangle exactly as dR stores it.  For the K embedding rows,
// row block ib of G is the A operand (lane: embedding row 16*ib + l%16, column 4s + l/16 in
// step s); the B operand of step s is embedding row 4s + l/16, of which lane x = l%16 fetches
// CW = 4 (or 2) floats at columns 16*CW*g + CW*x: element u of them belongs to the output tile
// whose 16 columns are {16*CW*g + CW*x' + u}, so that after the contraction every lane owns CW
// consecutive columns of 4 rows and stores them as one vector.  The dense row enters and leaves through plain FMAs: a rank-1
// update of every tile, and one matrix-vector product for its own gradient.
template <int NB>
__global__ __launch_bounds__(kIntThreads) void interact_bwd_kernel(const float* __restrict__ T,
                                                                    const float* __restrict__ dR,
                                                                    float* __restrict__ dT, int B, int F,
                                                                    int d, int gstride) {
  constexpr int JS = 4 * NB;  // contraction steps of 4 embedding rows
  // columns per lane and round: 4 (64-column groups) while the operand registers allow three
  // wavefronts per SIMD (up to 4 row blocks: 144 registers; measured on 65 rows of 128 columns, batch 16384:
  // 0.348 ms with 2 columns, 0.317 ms with 4), else 2 -- a lane then owns CW consecutive columns of 4 rows
  constexpr int CW = NB <= 4 ? 4 : 2;
  extern __shared__ float lds[];
  const int lane = lane_id();
  const int b = blockIdx.x * kIntWaves + wave_id();
  if (b >= B) return;  // wavefronts are independent: no barriers below
  const int x_ = lane & 15, h_ = lane >> 4;
  const int K = F - 1;
  const int P = F * (F - 1) / 2;
  const float* Tb = T + (int64_t)b * F * d;
  const float* gR = dR + (int64_t)b * ((int64_t)d + P);
  float* dTb = dT + (int64_t)b * F * d;
  float* gs = lds + wave_id() * gstride;
  for (int t0 = 0; t0 < P; t0 += DLRM_WAVE * 16) {  // 16 loads in flight per lane
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
  for (int g0 = 0; g0 < d; g0 += 16 * CW) {
    // opaque copies: without them every row offset, LDS index and validity mask below is
    // hoisted out of this loop and held in registers, which halves the occupancy
    int x = x_, h = h_;
    asm volatile("" : "+v"(x), "+v"(h));
    const int col = g0 + CW * x;
    const bool cok = col < d;
    const int ccol = cok ? col : 0;
    float tb[JS][CW], t0v[CW];
    load_cols<CW>(Tb + ccol, cok, t0v);
#pragma unroll
    for (int s = 0; s < JS; ++s) {
      const int e = 4 * s + h;
      load_cols<CW>(Tb + (int64_t)((e < K ? e : K - 1) + 1) * d + ccol, e < K && cok, tb[s]);
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
    for (int ib = 0; ib < NB; ++ib) {  // many row blocks: one at a time keeps the register count down
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
          for (int u = 0; u < CW; ++u) acc[u] = mfma16(ga[s], tb[s][u], acc[u]);
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

static int check_interact(const void* a, const void* b, int B, int F, int d) {
  if (!a || !b) return DLRM_ERR_NULL;
  if (B < 1 || F < 1 || F > DLRM_MAX_INTERACT_F || d < 4 || (d & 3)) return DLRM_ERR_BAD_SHAPE;
  if ((int64_t)B * F * d > ((int64_t)1 << 40)) return DLRM_ERR_BAD_SHAPE;
  return DLRM_OK;
}

// floats of LDS per wavefront: the P pair values of one sample
static int pair_stride(int F) {
  const int P = F * (F - 1) / 2;
  return P < 4 ? 4 : ((P + 3) & ~3);
}

template <int NB>
static int launch_fwd(const float* T, float* R, int B, int F, int d, hipStream_t st) {
  const int pstride = pair_stride(F);
  const size_t lds = (size_t)kIntWaves * pstride * 4;
  if (lds > 64 * 1024) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(interact_fwd_kernel<NB>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return DLRM_ERR_HIP;
  }
  hipLaunchKernelGGL((interact_fwd_kernel<NB>), dim3(div_up(B, kIntWaves)), dim3(kIntThreads), lds, st, T, R,
                     B, F, d, pstride);
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}

template <int NB>
static int launch_bwd(const float* T, const float* dR, float* dT, int B, int F, int d, hipStream_t st) {
  const int gstride = pair_stride(F);
  const size_t lds = (size_t)kIntWaves * gstride * 4;
  if (lds > 64 * 1024) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(interact_bwd_kernel<NB>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return DLRM_ERR_HIP;
  }
  hipLaunchKernelGGL((interact_bwd_kernel<NB>), dim3(div_up(B, kIntWaves)), dim3(kIntThreads), lds, st, T, dR,
                     dT, B, F, d, gstride);
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}

}  // namespace dlrm

using namespace dlrm;

extern "C" int32_t dlrm_interact_dot_fwd(const float* T, int32_t B, int32_t F, int32_t d, float* R,
                                         void* stream) {
  int st = check_interact(T, R, B, F, d);
  if (st != DLRM_OK) return st;
  if (reinterpret_cast<uintptr_t>(T) & 15) return DLRM_ERR_BAD_SHAPE;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  switch (F <= 17 ? 1 : (F + 14) / 16) {  // blocks of 16 embedding rows (all rows but the dense one)
    case 1: return launch_fwd<1>(T, R, B, F, d, hs);
    case 2: return launch_fwd<2>(T, R, B, F, d, hs);
    case 3: return launch_fwd<3>(T, R, B, F, d, hs);
    case 4: return launch_fwd<4>(T, R, B, F, d, hs);
    case 5: return launch_fwd<5>(T, R, B, F, d, hs);
    case 6: return launch_fwd<6>(T, R, B, F, d, hs);
    case 7: return launch_fwd<7>(T, R, B, F, d, hs);
    case 8: return launch_fwd<8>(T, R, B, F, d, hs);
  }
  return DLRM_ERR_BAD_SHAPE;
}

extern "C" int32_t dlrm_interact_dot_bwd(const float* T, const float* dR, int32_t B, int32_t F,
                                         int32_t d, float* dT, void* stream) {
  int st = check_interact(T, dR, B, F, d);
  if (st != DLRM_OK) return st;
  if (!dT) return DLRM_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(T) & 15) || (reinterpret_cast<uintptr_t>(dT) & 15))
    return DLRM_ERR_BAD_SHAPE;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  switch (F <= 17 ? 1 : (F + 14) / 16) {
    case 1: return launch_bwd<1>(T, dR, dT, B, F, d, hs);
    case 2: return launch_bwd<2>(T, dR, dT, B, F, d, hs);
    case 3: return launch_bwd<3>(T, dR, dT, B, F, d, hs);
    case 4: return launch_bwd<4>(T, dR, dT, B, F, d, hs);
    case 5: return launch_bwd<5>(T, dR, dT, B, F, d, hs);
    case 6: return launch_bwd<6>(T, dR, dT, B, F, d, hs);
    case 7: return launch_bwd<7>(T, dR, dT, B, F, d, hs);
    case 8: return launch_bwd<8>(T, dR, dT, B, F, d, hs);
  }
  return DLRM_ERR_BAD_SHAPE;
}
