// Internal helpers shared by the HIP translation units of libdlrm_hot.
// gfx950 only: 64-wide wavefronts, 16-byte (dwordx4) global accesses per lane.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dlrm_hot.h"

#define DLRM_WAVE 64

#define DLRM_CHECK_LAUNCH()                          \
  do {                                               \
    if (hipGetLastError() != hipSuccess) return DLRM_ERR_HIP; \
  } while (0)

namespace dlrm {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

// Bit casts by value.  (__builtin_bit_cast applied directly to an element of an
// ext_vector_type lvalue reads element 0 whatever the element: always go through these.)
__device__ inline float u2f(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ inline uint32_t f2u(float f) { return __builtin_bit_cast(uint32_t, f); }

__host__ __device__ inline int elem_bytes(int dtype) { return dtype == DLRM_F32 ? 4 : 2; }

__host__ inline bool dtype_ok(int dtype) {
  return dtype == DLRM_F32 || dtype == DLRM_F16 || dtype == DLRM_BF16;
}

// smallest power of two >= v (v >= 1)
__host__ __device__ inline int pow2_ceil(int v) {
  int p = 1;
  while (p < v) p <<= 1;
  return p;
}

__host__ inline int ilog2_ceil(int64_t v) {  // number of bits needed to index v values
  int b = 0;
  while (((int64_t)1 << b) < v) ++b;
  return b;
}

// ---- storage-type traits: a 16-byte chunk of a table row <-> fp32 lanes ----

// fp16 pair <-> fp32 pair (v_cvt_f32_f16 / v_cvt_f16_f32: exact widening,
// round-to-nearest-even narrowing, subnormals honoured)
__device__ inline void half2_to_float2(uint32_t bits, float& a, float& b) {
  f16x2 h = __builtin_bit_cast(f16x2, bits);
  a = (float)h.x;
  b = (float)h.y;
}
__device__ inline uint32_t float2_to_half2(float a, float b) {
  f16x2 h;
  h.x = (_Float16)a;
  h.y = (_Float16)b;
  return __builtin_bit_cast(uint32_t, h);
}
// bf16 = upper half of fp32
__device__ inline void bf162_to_float2(uint32_t bits, float& a, float& b) {
  a = u2f(bits << 16);
  b = u2f(bits & 0xFFFF0000u);
}
__device__ inline uint32_t float_to_bf16_rne(float f) {
  const uint32_t u = f2u(f);
  const uint32_t nan = (u >> 16) | 0x40u;  // NaN stays NaN (quiet)
  const uint32_t rne = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
  return (u & 0x7FFFFFFFu) > 0x7F800000u ? nan : rne;
}
__device__ inline uint32_t float2_to_bf162(float a, float b) {
  return float_to_bf16_rne(a) | (float_to_bf16_rne(b) << 16);
}

template <int DT>
struct Tab;  // ELEMS = table elements per 16-byte chunk

template <>
struct Tab<DLRM_F32> {
  static constexpr int ELEMS = 4;
  static constexpr int EB = 4;
  __device__ static inline u32x4 ident() {  // -0.0f: x + (-0) == x for every x, bit for bit
    return u32x4{0x80000000u, 0x80000000u, 0x80000000u, 0x80000000u};
  }
  __device__ static inline void widen(u32x4 v, float* f) {
    f[0] = u2f(v.x);
    f[1] = u2f(v.y);
    f[2] = u2f(v.z);
    f[3] = u2f(v.w);
  }
};
template <>
struct Tab<DLRM_F16> {
  static constexpr int ELEMS = 8;
  static constexpr int EB = 2;
  __device__ static inline u32x4 ident() {
    return u32x4{0x80008000u, 0x80008000u, 0x80008000u, 0x80008000u};
  }
  __device__ static inline void widen(u32x4 v, float* f) {
    half2_to_float2(v.x, f[0], f[1]);
    half2_to_float2(v.y, f[2], f[3]);
    half2_to_float2(v.z, f[4], f[5]);
    half2_to_float2(v.w, f[6], f[7]);
  }
};
template <>
struct Tab<DLRM_BF16> {
  static constexpr int ELEMS = 8;
  static constexpr int EB = 2;
  __device__ static inline u32x4 ident() {
    return u32x4{0x80008000u, 0x80008000u, 0x80008000u, 0x80008000u};
  }
  __device__ static inline void widen(u32x4 v, float* f) {
    bf162_to_float2(v.x, f[0], f[1]);
    bf162_to_float2(v.y, f[2], f[3]);
    bf162_to_float2(v.z, f[4], f[5]);
    bf162_to_float2(v.w, f[6], f[7]);
  }
};

__device__ inline u32x4 load16(const void* p) { return *reinterpret_cast<const u32x4*>(p); }
// 16 bytes from a device address held as an integer (e.g. a table base that travelled through a
// cross-lane read): the pointer is built in the global address space, so the load is a global one.  A
// pointer made from an integer is otherwise a flat pointer, and flat loads also count as LDS-type
// operations, so that every wait for a cross-lane permute would wait for the rows in flight too.
__device__ inline u32x4 load16_global(uint64_t addr) {
  return *(const __attribute__((address_space(1))) u32x4*)addr;
}
__device__ inline void store16(void* p, u32x4 v) { *reinterpret_cast<u32x4*>(p) = v; }
__device__ inline f32x4 loadf4(const float* p) { return *reinterpret_cast<const f32x4*>(p); }
// Element i of a batch's index array, whose element type is a run-time property of the batch
// (cold paths only; the hot kernels are compiled per index type).
__device__ inline int64_t index_at(const void* indices, int is32, int64_t i) {
  return is32 ? (int64_t)static_cast<const int32_t*>(indices)[i] : static_cast<const int64_t*>(indices)[i];
}

// Streaming accesses: data touched once per launch (table rows) should not push reusable data
// (gradient rows, pair lists) out of the L2.  (Flat accesses on purpose: the same helpers through
// global-address-space pointers measured 2-3 % slower in the update kernels.)
__device__ inline u32x4 load16_stream(const void* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}
__device__ inline void store16_stream(void* p, u32x4 v) {
  __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(p));
}
__device__ inline u32x2 load8_stream(const void* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p));
}
__device__ inline void store8_stream(void* p, u32x2 v) {
  __builtin_nontemporal_store(v, reinterpret_cast<u32x2*>(p));
}
__device__ inline void storef4(float* p, f32x4 v) { *reinterpret_cast<f32x4*>(p) = v; }

// The first thread of a launch tells a polling host that the launch has begun (and so, by stream
// order, that everything enqueued before it on its stream is done): a system-scope store that
// leaves the device at once instead of waiting in a cache for the end of the kernel.
__device__ inline void stamp_start(uint32_t* stamp, uint32_t value) {
  if (stamp != nullptr && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0)
    __hip_atomic_store(stamp, value, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

__device__ inline int lane_id() { return threadIdx.x & (DLRM_WAVE - 1); }
__device__ inline int wave_id() { return threadIdx.x >> 6; }

// ---- block-wide exclusive scan of one uint32 per thread (THREADS multiple of 64) ----
// smem: at least THREADS/64 + 1 words.  Returns the exclusive prefix; *total = block sum.
template <int THREADS>
__device__ inline uint32_t block_exclusive_scan(uint32_t v, uint32_t* smem, uint32_t* total) {
  constexpr int NW = THREADS / DLRM_WAVE;
  const int lane = lane_id(), w = wave_id();
  uint32_t inc = v;
#pragma unroll
  for (int o = 1; o < DLRM_WAVE; o <<= 1) {
    uint32_t t = __shfl_up(inc, o, DLRM_WAVE);
    if (lane >= o) inc += t;
  }
  __syncthreads();  // smem may still be read from a previous call
  if (lane == DLRM_WAVE - 1) smem[w] = inc;
  __syncthreads();
  uint32_t base = 0, sum = 0;
#pragma unroll
  for (int i = 0; i < NW; ++i) {
    uint32_t c = smem[i];
    if (i < w) base += c;
    sum += c;
  }
  *total = sum;
  return base + inc - v;
}

// host-side launch geometry helpers
__host__ inline unsigned div_up(int64_t a, int64_t b) { return (unsigned)((a + b - 1) / b); }

}  // namespace dlrm
