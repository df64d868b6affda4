// Dot-product feature interaction (Sec. 2.2) and its backward.
//   fwd: R[b] = [ T[b,0,:] | <T[b,i,:],T[b,j,:]> for 1 <= i < F, 0 <= j < i ]
//   bwd: dT[b,i,:] = sum_{j != i} g(i,j) T[b,j,:]  (+ dR[b,0:d] on row 0),
//        g(i,j) = dR[b, d + pair(max(i,j), min(i,j))]
// Per sample the operand T_b is F x d fp32 (2 KB .. 33 KB): it is staged once in
// LDS and every output of the sample is produced from there, so HBM sees each
// input and output exactly once.  Rows in LDS are padded by 4 floats so that
// lanes reading different rows at the same column hit different banks.
#include "common.h"

namespace dlrm {

constexpr int kIntThreads = 256;
constexpr int kPad = 4;
constexpr int kIntLdsBytes = 64 * 1024;  // LDS budget per workgroup for the staged tiles

__device__ inline void pair_from_index(int q, int& i, int& j) {
  // q = i(i-1)/2 + j with 0 <= j < i: invert the triangular number, then fix rounding
  int t = (int)((1.0f + sqrtf(1.0f + 8.0f * (float)q)) * 0.5f);
  while (t * (t - 1) / 2 > q) --t;
  while ((t + 1) * t / 2 <= q) ++t;
  i = t;
  j = q - t * (t - 1) / 2;
}

// stage NS samples' T tiles: global [ns][F][d] contiguous -> LDS [ns][F][d+kPad]
__device__ inline void stage_T(const float* __restrict__ Tg, float* Ts, int ns, int F, int d) {
  const int d4 = d >> 2, dp = d + kPad;
  const int n4 = ns * F * d4;
  for (int t = threadIdx.x; t < n4; t += kIntThreads) {
    const int row = t / d4, c4 = t - row * d4;
    storef4(Ts + row * dp + c4 * 4, loadf4(Tg + (int64_t)t * 4));
  }
}

__global__ __launch_bounds__(kIntThreads) void interact_fwd_kernel(const float* __restrict__ T,
                                                                    float* __restrict__ R, int B, int F,
                                                                    int d, int NS) {
  extern __shared__ float lds[];
  const int dp = d + kPad, d4 = d >> 2;
  const int P = F * (F - 1) / 2;
  const int b0 = blockIdx.x * NS;
  const int ns = (B - b0) < NS ? (B - b0) : NS;
  stage_T(T + (int64_t)b0 * F * d, lds, ns, F, d);
  __syncthreads();
  const int64_t W = (int64_t)d + P;
  // dense part: exact copy of row 0
  for (int t = threadIdx.x; t < ns * d4; t += kIntThreads) {
    const int s = t / d4, c4 = t - s * d4;
    // R rows are d+P floats wide: only 4-byte alignment is guaranteed
    const float* src = lds + (s * F) * dp + c4 * 4;
    float* dst = R + (b0 + s) * W + c4 * 4;
    dst[0] = src[0];
    dst[1] = src[1];
    dst[2] = src[2];
    dst[3] = src[3];
  }
  // pair part
  for (int t = threadIdx.x; t < ns * P; t += kIntThreads) {
    const int s = t / P, q = t - s * P;
    int i, j;
    pair_from_index(q, i, j);
    const float* a = lds + (s * F + i) * dp;
    const float* c = lds + (s * F + j) * dp;
    float acc = 0.0f;
    for (int c4 = 0; c4 < d4; ++c4) {
      const f32x4 x = loadf4(a + c4 * 4), y = loadf4(c + c4 * 4);
      acc = fmaf(x.x, y.x, acc);
      acc = fmaf(x.y, y.y, acc);
      acc = fmaf(x.z, y.z, acc);
      acc = fmaf(x.w, y.w, acc);
    }
    R[(b0 + s) * W + d + q] = acc;
  }
}

__global__ __launch_bounds__(kIntThreads) void interact_bwd_kernel(const float* __restrict__ T,
                                                                    const float* __restrict__ dR,
                                                                    float* __restrict__ dT, int B, int F,
                                                                    int d, int NS) {
  extern __shared__ float lds[];
  const int dp = d + kPad, d4 = d >> 2;
  const int P = F * (F - 1) / 2;
  const int b0 = blockIdx.x * NS;
  const int ns = (B - b0) < NS ? (B - b0) : NS;
  float* Ts = lds;                 // [NS][F][dp]
  float* Gs = lds + NS * F * dp;   // [NS][d + P]  (the whole dR row)
  const int64_t W = (int64_t)d + P;
  stage_T(T + (int64_t)b0 * F * d, Ts, ns, F, d);
  for (int t = threadIdx.x; t < ns * (int)W; t += kIntThreads) Gs[t] = dR[(int64_t)b0 * W + t];
  __syncthreads();
  const int per = F * d4;
  for (int t = threadIdx.x; t < ns * per; t += kIntThreads) {
    const int s = t / per, rem = t - s * per;
    const int i = rem / d4, c4 = rem - i * d4;
    const float* g = Gs + s * (int)W;
    const float* Tb = Ts + s * F * dp + c4 * 4;
    f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
    if (i == 0) acc = f32x4{g[c4 * 4], g[c4 * 4 + 1], g[c4 * 4 + 2], g[c4 * 4 + 3]};
    const float* grow = g + d + i * (i - 1) / 2;  // g(i, j) for j < i is contiguous
    for (int j = 0; j < i; ++j) {
      const float gij = grow[j];
      const f32x4 v = loadf4(Tb + j * dp);
      acc.x = fmaf(gij, v.x, acc.x);
      acc.y = fmaf(gij, v.y, acc.y);
      acc.z = fmaf(gij, v.z, acc.z);
      acc.w = fmaf(gij, v.w, acc.w);
    }
    for (int j = i + 1; j < F; ++j) {
      const float gji = g[d + j * (j - 1) / 2 + i];
      const f32x4 v = loadf4(Tb + j * dp);
      acc.x = fmaf(gji, v.x, acc.x);
      acc.y = fmaf(gji, v.y, acc.y);
      acc.z = fmaf(gji, v.z, acc.z);
      acc.w = fmaf(gji, v.w, acc.w);
    }
    storef4(dT + ((int64_t)(b0 + s) * F + i) * d + c4 * 4, acc);
  }
}

static int pick_ns(int B, int F, int d, bool bwd) {
  const int64_t per = (int64_t)F * (d + kPad) * 4 + (bwd ? ((int64_t)d + (int64_t)F * (F - 1) / 2) * 4 : 0);
  int ns = (int)(kIntLdsBytes / per);
  if (ns < 1) ns = 1;
  if (ns > 16) ns = 16;
  // keep at least ~4 workgroups per compute unit when the batch allows it
  while (ns > 1 && (B + ns - 1) / ns < 1024) ns >>= 1;
  return ns;
}

static int check_interact(const void* a, const void* b, int B, int F, int d) {
  if (!a || !b) return DLRM_ERR_NULL;
  if (B < 1 || F < 1 || F > DLRM_MAX_INTERACT_F || d < 4 || (d & 3)) return DLRM_ERR_BAD_SHAPE;
  if ((int64_t)F * (d + kPad) * 4 + ((int64_t)d + (int64_t)F * (F - 1) / 2) * 4 > 160 * 1024 - 1024)
    return DLRM_ERR_BAD_SHAPE;
  if ((int64_t)B * F * d > ((int64_t)1 << 40)) return DLRM_ERR_BAD_SHAPE;
  return DLRM_OK;
}

}  // namespace dlrm

using namespace dlrm;

extern "C" int32_t dlrm_interact_dot_fwd(const float* T, int32_t B, int32_t F, int32_t d, float* R,
                                         void* stream) {
  int st = check_interact(T, R, B, F, d);
  if (st != DLRM_OK) return st;
  if (reinterpret_cast<uintptr_t>(T) & 15) return DLRM_ERR_BAD_SHAPE;
  const int NS = pick_ns(B, F, d, false);
  const size_t lds = (size_t)NS * F * (d + kPad) * 4;
  if (lds > 64 * 1024) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(interact_fwd_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return DLRM_ERR_HIP;
  }
  hipLaunchKernelGGL(interact_fwd_kernel, dim3(div_up(B, NS)), dim3(kIntThreads), lds,
                     static_cast<hipStream_t>(stream), T, R, B, F, d, NS);
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}

extern "C" int32_t dlrm_interact_dot_bwd(const float* T, const float* dR, int32_t B, int32_t F,
                                         int32_t d, float* dT, void* stream) {
  int st = check_interact(T, dR, B, F, d);
  if (st != DLRM_OK) return st;
  if (!dT) return DLRM_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(T) & 15) || (reinterpret_cast<uintptr_t>(dT) & 15))
    return DLRM_ERR_BAD_SHAPE;
  const int NS = pick_ns(B, F, d, true);
  const int P = F * (F - 1) / 2;
  const size_t lds = ((size_t)NS * F * (d + kPad) + (size_t)NS * (d + P)) * 4;
  if (lds > 64 * 1024) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(interact_bwd_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return DLRM_ERR_HIP;
  }
  hipLaunchKernelGGL(interact_bwd_kernel, dim3(div_up(B, NS)), dim3(kIntThreads), lds,
                     static_cast<hipStream_t>(stream), T, dR, dT, B, F, d, NS);
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}
