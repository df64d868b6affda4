// Host-side argument checks and the small helper kernels around the hot path:
// CSR lengths -> offsets (Sec. 4.1 footnote), the checked CSR validator, the
// dense-vector placement (Sec. 2.2) and the counter-based table initialiser
// used to create synthetic tables on the device.
#include "common.h"

namespace dlrm {

int check_batch(const dlrm_sparse_batch* s) {
  if (!s) return DLRM_ERR_NULL;
  if (!dtype_ok(s->table_dtype)) return DLRM_ERR_BAD_DTYPE;
  if (s->K < 1 || s->B < 1 || s->d < 1) return DLRM_ERR_BAD_SHAPE;
  const int64_t row_bytes = (int64_t)s->d * elem_bytes(s->table_dtype);
  if ((row_bytes & 15) != 0 || row_bytes > DLRM_MAX_ROW_BYTES) return DLRM_ERR_BAD_SHAPE;
  if (s->nnz_total < 0 || s->nnz_total > DLRM_MAX_NNZ) return DLRM_ERR_BAD_SHAPE;
  if (s->max_rows < 1 || s->max_rows > DLRM_MAX_ROWS) return DLRM_ERR_BAD_SHAPE;
  if ((int64_t)s->K * (s->B + 1) > DLRM_MAX_NNZ) return DLRM_ERR_BAD_SHAPE;
  if (!s->tables || !s->rows || !s->offsets || !s->tbl_off) return DLRM_ERR_NULL;
  if (s->nnz_total > 0 && !s->indices) return DLRM_ERR_NULL;
  if (s->index_dtype != DLRM_I64 && s->index_dtype != DLRM_I32) return DLRM_ERR_BAD_DTYPE;
  return DLRM_OK;
}

// ---------------------------------------------------------------------------
// lengths -> offsets: one workgroup per table scans its B lengths in chunks of
// 1024 with a running carry (64-bit), then one workgroup scans the K totals.
__global__ __launch_bounds__(1024) void lengths_scan_kernel(const int32_t* __restrict__ lengths,
                                                            int32_t B, int64_t* __restrict__ offsets) {
  __shared__ uint32_t smem[1024 / DLRM_WAVE + 1];
  const int k = blockIdx.x;
  const int32_t* len = lengths + (int64_t)k * B;
  int64_t* off = offsets + (int64_t)k * (B + 1);
  int64_t carry = 0;
  if (threadIdx.x == 0) off[0] = 0;
  for (int32_t b0 = 0; b0 < B; b0 += 1024) {
    const int32_t b = b0 + threadIdx.x;
    const uint32_t v = b < B ? (uint32_t)len[b] : 0u;
    uint32_t total;
    const uint32_t ex = block_exclusive_scan<1024>(v, smem, &total);
    if (b < B) off[b + 1] = carry + ex + v;
    carry += total;
  }
}

__global__ __launch_bounds__(256) void tbl_off_kernel(const int64_t* __restrict__ offsets, int32_t K,
                                                      int32_t B, int64_t* __restrict__ tbl_off) {
  // K is small (tens): a serial walk by one lane is enough and trivially exact
  if (threadIdx.x == 0) {
    int64_t run = 0;
    tbl_off[0] = 0;
    for (int32_t k = 0; k < K; ++k) {
      run += offsets[(int64_t)k * (B + 1) + B];
      tbl_off[k + 1] = run;
    }
  }
}

// ---------------------------------------------------------------------------
struct ValArgs {
  const int64_t* rows;
  const void* indices;
  const int64_t* offsets;
  const int64_t* tbl_off;
  int64_t nnz_total;
  int32_t K, B, idx32;
  unsigned long long* n_bad;
};

__global__ __launch_bounds__(256) void validate_kernel(ValArgs a) {
  const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t nthreads = (int64_t)gridDim.x * blockDim.x;
  unsigned long long bad = 0;
  // offsets: K*(B+1) entries
  const int64_t noff = (int64_t)a.K * (a.B + 1);
  for (int64_t i = tid; i < noff; i += nthreads) {
    const int k = (int)(i / (a.B + 1)), b = (int)(i - (int64_t)k * (a.B + 1));
    const int64_t o = a.offsets[i];
    if (b == 0) {
      if (o != 0) ++bad;
    } else if (o < a.offsets[i - 1]) {
      ++bad;
    }
    if (b == a.B && o != a.tbl_off[k + 1] - a.tbl_off[k]) ++bad;
  }
  // tbl_off: K+1 entries
  for (int64_t k = tid; k <= a.K; k += nthreads) {
    const int64_t t = a.tbl_off[k];
    if (k == 0 && t != 0) ++bad;
    if (k > 0 && t < a.tbl_off[k - 1]) ++bad;
    if (k == a.K && t != a.nnz_total) ++bad;
  }
  // indices: position p belongs to the table whose slice holds it (clamped search, so a
  // broken tbl_off cannot send a read outside [0, K])
  for (int64_t p = tid; p < a.nnz_total; p += nthreads) {
    int lo = 0, hi = a.K;  // find k with tbl_off[k] <= p < tbl_off[k+1]
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (a.tbl_off[mid] <= p) lo = mid; else hi = mid;
    }
    const int64_t r = index_at(a.indices, a.idx32, p);
    if (r < 0 || r >= a.rows[lo]) ++bad;
  }
  // wave reduction, one atomic per wavefront
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) bad += __shfl_xor(bad, o, DLRM_WAVE);
  if (lane_id() == 0 && bad) atomicAdd(a.n_bad, bad);
}

__global__ void zero_u64_kernel(unsigned long long* p) { *p = 0; }

// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void place_dense_kernel(const float* __restrict__ x, int64_t n4,
                                                          int32_t d4, float* __restrict__ T,
                                                          int64_t row_stride) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4;
       i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t b = i / d4, c4 = i - b * d4;
    storef4(T + b * row_stride + c4 * 4, loadf4(x + i * 4));
  }
}

// ---------------------------------------------------------------------------
__device__ inline uint64_t mix64(uint64_t z) {  // splitmix64 output function
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

__device__ inline float hash_value(uint64_t key, uint64_t e, float scale) {
  const uint32_t u = (uint32_t)(mix64(key + e) >> 40);                 // 24 bits
  const float x = (float)((int32_t)(2u * u + 1u) - (1 << 24)) * (1.0f / 16777216.0f);  // exact
  return __fmul_rn(x, scale);
}

// each thread produces one 16-byte chunk of the table
template <int DT>
__global__ __launch_bounds__(256) void table_init_kernel(void* table, int64_t nchunks, uint64_t key,
                                                         float scale) {
  constexpr int E = Tab<DT>::ELEMS;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nchunks;
       i += (int64_t)gridDim.x * blockDim.x) {
    float f[E];
#pragma unroll
    for (int j = 0; j < E; ++j) f[j] = hash_value(key, (uint64_t)(i * E + j), scale);
    u32x4 v;
    if constexpr (DT == DLRM_F32) {
      v = u32x4{f2u(f[0]), f2u(f[1]), f2u(f[2]), f2u(f[3])};
    } else if constexpr (DT == DLRM_F16) {
      v = u32x4{float2_to_half2(f[0], f[1]), float2_to_half2(f[2], f[3]),
                float2_to_half2(f[4], f[5]), float2_to_half2(f[6], f[7])};
    } else {
      v = u32x4{float2_to_bf162(f[0], f[1]), float2_to_bf162(f[2], f[3]),
                float2_to_bf162(f[4], f[5]), float2_to_bf162(f[6], f[7])};
    }
    store16(static_cast<char*>(table) + i * 16, v);
  }
}

}  // namespace dlrm

using namespace dlrm;

extern "C" int32_t dlrm_version(void) { return 100; }

extern "C" const char* dlrm_status_string(int32_t status) {
  switch (status) {
    case DLRM_OK: return "ok";
    case DLRM_ERR_NULL: return "a required pointer is NULL";
    case DLRM_ERR_BAD_SHAPE: return "shape, stride, alignment or size outside the supported range";
    case DLRM_ERR_BAD_DTYPE: return "unknown or unsupported table dtype";
    case DLRM_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case DLRM_ERR_BAD_ALGO: return "unknown backward algorithm";
    case DLRM_ERR_HIP: return "HIP launch failed";
  }
  return "unknown status";
}

extern "C" int32_t dlrm_lengths_to_offsets(const int32_t* lengths, int32_t K, int32_t B,
                                           int64_t* offsets, int64_t* tbl_off, void* stream) {
  if (!lengths || !offsets || !tbl_off) return DLRM_ERR_NULL;
  if (K < 1 || B < 1 || (int64_t)K * (B + 1) > DLRM_MAX_NNZ) return DLRM_ERR_BAD_SHAPE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(lengths_scan_kernel, dim3(K), dim3(1024), 0, st, lengths, B, offsets);
  DLRM_CHECK_LAUNCH();
  hipLaunchKernelGGL(tbl_off_kernel, dim3(1), dim3(64), 0, st, offsets, K, B, tbl_off);
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}

extern "C" int32_t dlrm_validate_csr(const dlrm_sparse_batch* s, int64_t* n_bad, void* stream) {
  int st = check_batch(s);
  if (st != DLRM_OK) return st;
  if (!n_bad) return DLRM_ERR_NULL;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  ValArgs a;
  a.rows = s->rows;
  a.indices = s->indices;
  a.idx32 = s->index_dtype == DLRM_I32;
  a.offsets = s->offsets;
  a.tbl_off = s->tbl_off;
  a.nnz_total = s->nnz_total;
  a.K = s->K;
  a.B = s->B;
  a.n_bad = reinterpret_cast<unsigned long long*>(n_bad);
  hipLaunchKernelGGL(zero_u64_kernel, dim3(1), dim3(1), 0, hs, a.n_bad);
  DLRM_CHECK_LAUNCH();
  const int64_t work = s->nnz_total > (int64_t)s->K * (s->B + 1) ? s->nnz_total
                                                                  : (int64_t)s->K * (s->B + 1);
  unsigned grid = div_up(work, 256);
  if (grid > 4096) grid = 4096;
  hipLaunchKernelGGL(validate_kernel, dim3(grid), dim3(256), 0, hs, a);
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}

extern "C" int32_t dlrm_place_dense(const float* x, int32_t B, int32_t d, float* T, int32_t F,
                                    void* stream) {
  if (!x || !T) return DLRM_ERR_NULL;
  if (B < 1 || d < 4 || (d & 3) || F < 1) return DLRM_ERR_BAD_SHAPE;
  if ((reinterpret_cast<uintptr_t>(x) & 15) || (reinterpret_cast<uintptr_t>(T) & 15))
    return DLRM_ERR_BAD_SHAPE;
  const int64_t n4 = (int64_t)B * (d / 4);
  unsigned grid = div_up(n4, 256);
  if (grid > 8192) grid = 8192;
  hipLaunchKernelGGL(place_dense_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream),
                     x, n4, d / 4, T, (int64_t)F * d);
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}

extern "C" int32_t dlrm_table_init_hash(void* table, int64_t rows, int32_t d, int32_t table_dtype,
                                        uint64_t key, float scale, void* stream) {
  if (!table) return DLRM_ERR_NULL;
  if (!dtype_ok(table_dtype)) return DLRM_ERR_BAD_DTYPE;
  if (rows < 1 || d < 1) return DLRM_ERR_BAD_SHAPE;
  const int64_t row_bytes = (int64_t)d * elem_bytes(table_dtype);
  if (row_bytes & 15) return DLRM_ERR_BAD_SHAPE;
  if (reinterpret_cast<uintptr_t>(table) & 15) return DLRM_ERR_BAD_SHAPE;
  const int64_t nchunks = rows * (row_bytes / 16);
  unsigned grid = div_up(nchunks, 256);
  if (grid > 65536) grid = 65536;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  switch (table_dtype) {
    case DLRM_F32:
      hipLaunchKernelGGL(table_init_kernel<DLRM_F32>, dim3(grid), dim3(256), 0, hs, table, nchunks, key, scale);
      break;
    case DLRM_F16:
      hipLaunchKernelGGL(table_init_kernel<DLRM_F16>, dim3(grid), dim3(256), 0, hs, table, nchunks, key, scale);
      break;
    default:
      hipLaunchKernelGGL(table_init_kernel<DLRM_BF16>, dim3(grid), dim3(256), 0, hs, table, nchunks, key, scale);
      break;
  }
  DLRM_CHECK_LAUNCH();
  return DLRM_OK;
}
