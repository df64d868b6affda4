// Measurement aid: memory-bound kernels of known traffic and no arithmetic to speak of, in the access
// patterns of the path (stream, whole-row gather, whole-row read-modify-write).  A benchmark times
// them to learn what the board in front of it sustains for each pattern, which is what a kernel of
// the path can be held against besides the nominal HBM peak.
#include "common.h"
#include "dlrm_ceilings.h"

namespace dlrm {

constexpr int kCeilThreads = 256;
constexpr int kCeilStreamBlocks = 8192;  // grid-stride loops: enough workgroups to fill every compute unit
constexpr int kCeilRowBlocks = 4096;     // several times over
constexpr int kCeilRowsInFlight = 4;     // rows a lane group requests before it consumes any

__global__ __launch_bounds__(kCeilThreads) void ceiling_copy_kernel(const f32x4* __restrict__ src,
                                                                    f32x4* __restrict__ dst, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * kCeilThreads + threadIdx.x; i < n16; i += (size_t)gridDim.x * kCeilThreads)
    dst[i] = src[i];
}

__global__ __launch_bounds__(kCeilThreads) void ceiling_read_kernel(const f32x4* __restrict__ src, size_t n16,
                                                                    float* __restrict__ sink) {
  f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
  for (size_t i = (size_t)blockIdx.x * kCeilThreads + threadIdx.x; i < n16; i += (size_t)gridDim.x * kCeilThreads)
    acc += src[i];
  // keeps the loads alive; a block writes its lane-0 sum (the value means nothing)
  if (threadIdx.x == 0) sink[blockIdx.x] = acc.x + acc.y + acc.z + acc.w;
}

// LANES lanes per row of LANES * 16 bytes; a lane group takes kCeilRowsInFlight listed rows per round.
template <int LANES, bool WRITE>
__global__ __launch_bounds__(kCeilThreads) void ceiling_rows_kernel(char* __restrict__ table,
                                                                    const uint32_t* __restrict__ rows, size_t n,
                                                                    float* __restrict__ sink) {
  constexpr int U = kCeilRowsInFlight;
  const int lane = threadIdx.x % LANES;
  const size_t g = ((size_t)blockIdx.x * kCeilThreads + threadIdx.x) / LANES;
  const size_t ng = (size_t)gridDim.x * kCeilThreads / LANES;
  f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
  for (size_t i = g * U; i < n; i += ng * U) {
    uint32_t r[U];
    f32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) r[u] = rows[i + u < n ? i + u : n - 1];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = *reinterpret_cast<const f32x4*>(table + (size_t)r[u] * (LANES * 16) + lane * 16);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if constexpr (WRITE) {
        if (i + u < n) *reinterpret_cast<f32x4*>(table + (size_t)r[u] * (LANES * 16) + lane * 16) = v[u] * 1.0009765625f;
      } else {
        acc += v[u];
      }
    }
  }
  if constexpr (!WRITE) {
    if (threadIdx.x == 0) sink[blockIdx.x] = acc.x + acc.y + acc.z + acc.w;
  }
}

template <bool WRITE>
static int launch_rows(void* table, const uint32_t* rows, int64_t n, int row_bytes, float* sink, hipStream_t st) {
  const dim3 grid(kCeilRowBlocks), block(kCeilThreads);
  char* t = static_cast<char*>(table);
  switch (row_bytes) {
    case 64: hipLaunchKernelGGL((ceiling_rows_kernel<4, WRITE>), grid, block, 0, st, t, rows, (size_t)n, sink); break;
    case 128: hipLaunchKernelGGL((ceiling_rows_kernel<8, WRITE>), grid, block, 0, st, t, rows, (size_t)n, sink); break;
    case 256: hipLaunchKernelGGL((ceiling_rows_kernel<16, WRITE>), grid, block, 0, st, t, rows, (size_t)n, sink); break;
    case 512: hipLaunchKernelGGL((ceiling_rows_kernel<32, WRITE>), grid, block, 0, st, t, rows, (size_t)n, sink); break;
    default: return DLRM_ERR_BAD_SHAPE;
  }
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}

}  // namespace dlrm

using namespace dlrm;

extern "C" int32_t dlrm_ceiling_sink_floats(void) { return kCeilStreamBlocks; }

extern "C" int32_t dlrm_ceiling_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (!src || !dst) return DLRM_ERR_NULL;
  if (bytes == 0 || (bytes & 15) || ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15))
    return DLRM_ERR_BAD_SHAPE;
  hipLaunchKernelGGL(ceiling_copy_kernel, dim3(kCeilStreamBlocks), dim3(kCeilThreads), 0,
                     static_cast<hipStream_t>(stream), static_cast<const f32x4*>(src), static_cast<f32x4*>(dst),
                     bytes / 16);
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}

extern "C" int32_t dlrm_ceiling_read(const void* src, size_t bytes, float* sink, void* stream) {
  if (!src || !sink) return DLRM_ERR_NULL;
  if (bytes == 0 || (bytes & 15) || (reinterpret_cast<uintptr_t>(src) & 15)) return DLRM_ERR_BAD_SHAPE;
  hipLaunchKernelGGL(ceiling_read_kernel, dim3(kCeilStreamBlocks), dim3(kCeilThreads), 0,
                     static_cast<hipStream_t>(stream), static_cast<const f32x4*>(src), bytes / 16, sink);
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}

extern "C" int32_t dlrm_ceiling_gather(const void* table, const uint32_t* rows, int64_t n, int32_t row_bytes,
                                       float* sink, void* stream) {
  if (!table || !rows || !sink) return DLRM_ERR_NULL;
  if (n < 1 || (reinterpret_cast<uintptr_t>(table) & 15)) return DLRM_ERR_BAD_SHAPE;
  return launch_rows<false>(const_cast<void*>(table), rows, n, row_bytes, sink, static_cast<hipStream_t>(stream));
}

extern "C" int32_t dlrm_ceiling_rmw(void* table, const uint32_t* rows, int64_t n, int32_t row_bytes, void* stream) {
  if (!table || !rows) return DLRM_ERR_NULL;
  if (n < 1 || (reinterpret_cast<uintptr_t>(table) & 15)) return DLRM_ERR_BAD_SHAPE;
  return launch_rows<true>(table, rows, n, row_bytes, nullptr, static_cast<hipStream_t>(stream));
}
