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
// Rows of T_b in NB blocks of 16; lane (i = l%16, h = l/16) fetches, for every row block, the 4
// floats at columns 16q + 4h of row 16*rb + i.  Element t of that float4 is at once the A
// operand of the row block and the B operand of the column block for the 4 columns
// {16q + 4h' + t : h' = 0..3}, so a tile (ib, jb) of Z = T T^t takes one instruction per 4
// columns.  Only tiles on or below the diagonal are computed.
template <int NB>
__global__ __launch_bounds__(kIntThreads) void interact_fwd_kernel(const float* __restrict__ T,
                                                                    float* __restrict__ R, int B, int F,
                                                                    int d) {
  constexpr int QC = NB <= 5 ? 4 : 2;  // 16-column chunks fetched per round
  constexpr int NTILE = NB * (NB + 1) / 2;
  const int lane = lane_id();
  const int b = blockIdx.x * kIntWaves + wave_id();
  if (b >= B) return;  // wavefronts are independent: no barriers below
  const int i = lane & 15, h = lane >> 4;
  const int P = F * (F - 1) / 2;
  const float* Tb = T + (int64_t)b * F * d;
  float* Rb = R + (int64_t)b * ((int64_t)d + P);
  for (int c = lane; c < d; c += DLRM_WAVE) Rb[c] = Tb[c];  // dense part: exact copy of row 0
  f32x4 acc[NTILE];
#pragma unroll
  for (int t = 0; t < NTILE; ++t) acc[t] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
  const float* rowp[NB];
#pragma unroll
  for (int rb = 0; rb < NB; ++rb) {
    const int row = rb * 16 + i < F ? rb * 16 + i : F - 1;  // rows past F repeat the last one; their
    rowp[rb] = Tb + (int64_t)row * d;                        // products land in entries never stored
  }
  for (int k0 = 0; k0 < d; k0 += 16 * QC) {
    f32x4 x[NB][QC];
#pragma unroll
    for (int q = 0; q < QC; ++q) {
      const int col = k0 + 16 * q + 4 * h;
      const int ccol = col < d ? col : 0;
#pragma unroll
      for (int rb = 0; rb < NB; ++rb) {
        const f32x4 v = loadf4(rowp[rb] + ccol);
        x[rb][q] = col < d ? v : f32x4{0.0f, 0.0f, 0.0f, 0.0f};  // columns past d contribute 0 * 0
      }
    }
#pragma unroll
    for (int q = 0; q < QC; ++q) {
      if (k0 + 16 * q < d) {  // uniform
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
  float* Rp = Rb + d;
  int tile = 0;
#pragma unroll
  for (int ib = 0; ib < NB; ++ib) {
#pragma unroll
    for (int jb = 0; jb <= ib; ++jb, ++tile) {
      const int gj = jb * 16 + i;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int gi = ib * 16 + 4 * h + v;
        if (gj < gi && gi < F) Rp[gi * (gi - 1) / 2 + gj] = acc[tile][v];
      }
    }
  }
}

// --- backward -------------------------------------------------------------------------------
// dT_b = G T_b with G the symmetric F x F matrix of pair gradients (zero diagonal), held per
// wavefront in LDS as the lower triangle exactly as dR stores it.  Row block ib of G is the A
// operand (lane: row 16*ib + l%16, column 4s + l/16 in step s); the B operand of step s is row
// 4s + l/16 of T, of which lane x = l%16 fetches the float4 at columns 64g + 4x: element u of
// it belongs to the output tile whose 16 columns are {64g + 4x' + u}, so that after the
// contraction every lane owns 4 consecutive columns of 4 rows and stores float4s.
template <int NB>
__global__ __launch_bounds__(kIntThreads) void interact_bwd_kernel(const float* __restrict__ T,
                                                                    const float* __restrict__ dR,
                                                                    float* __restrict__ dT, int B, int F,
                                                                    int d, int gstride) {
  constexpr int JS = 4 * NB;  // contraction steps of 4 rows
  extern __shared__ float lds[];
  const int lane = lane_id();
  const int b = blockIdx.x * kIntWaves + wave_id();
  if (b >= B) return;  // wavefronts are independent: no barriers below
  const int x = lane & 15, h = lane >> 4;
  const int P = F * (F - 1) / 2;
  const float* Tb = T + (int64_t)b * F * d;
  const float* gR = dR + (int64_t)b * ((int64_t)d + P);
  float* dTb = dT + (int64_t)b * F * d;
  float* gs = lds + wave_id() * gstride;
  for (int t = lane; t < P; t += DLRM_WAVE) gs[t] = gR[d + t];
  for (int g0 = 0; g0 < d; g0 += 64) {
    const int col = g0 + 4 * x;
    const bool cok = col < d;
    const int ccol = cok ? col : 0;
    f32x4 tb[JS];
#pragma unroll
    for (int s = 0; s < JS; ++s) {
      const int j = 4 * s + h;
      const f32x4 v = loadf4(Tb + (int64_t)(j < F ? j : F - 1) * d + ccol);
      tb[s] = (j < F && cok) ? v : f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    }
    for (int ib = 0; ib < NB; ++ib) {
      if (ib * 16 >= F) break;  // uniform
      const int m = ib * 16 + x;
      float ga[JS];
#pragma unroll
      for (int s = 0; s < JS; ++s) {
        const int j = 4 * s + h;
        const int hi = m > j ? m : j, lo = m > j ? j : m;
        const int q = hi * (hi - 1) / 2 + lo;
        const float gv = gs[(hi < F && hi != lo) ? q : 0];
        ga[s] = (hi < F && hi != lo) ? gv : 0.0f;
      }
      f32x4 acc[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) acc[u] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int s = 0; s < JS; ++s) {
        if (4 * s < F) {  // uniform
#pragma unroll
          for (int u = 0; u < 4; ++u) acc[u] = mfma16(ga[s], tb[s][u], acc[u]);
        }
      }
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int gi = ib * 16 + 4 * h + v;
        if (gi < F && cok) {
          f32x4 o = {acc[0][v], acc[1][v], acc[2][v], acc[3][v]};
          if (gi == 0) {  // the dense part of dR flows straight into row 0
            o.x += gR[col];
            o.y += gR[col + 1];
            o.z += gR[col + 2];
            o.w += gR[col + 3];
          }
          storef4(dTb + (int64_t)gi * d + col, o);
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

template <int NB>
static int launch_fwd(const float* T, float* R, int B, int F, int d, hipStream_t st) {
  hipLaunchKernelGGL((interact_fwd_kernel<NB>), dim3(div_up(B, kIntWaves)), dim3(kIntThreads), 0, st, T, R, B,
                     F, d);
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}

template <int NB>
static int launch_bwd(const float* T, const float* dR, float* dT, int B, int F, int d, hipStream_t st) {
  const int P = F * (F - 1) / 2;
  const int gstride = P < 4 ? 4 : ((P + 3) & ~3);  // floats of LDS per wavefront: the pair gradients
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
  switch ((F + 15) / 16) {  // row blocks of 16
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
  switch ((F + 15) / 16) {
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
