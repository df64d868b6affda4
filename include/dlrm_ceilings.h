/*
 * dlrm_ceilings -- measurement kernels for a benchmark of libdlrm_hot (a library of its own:
 * nothing of the method is in here, and the method's library holds none of this).
 *
 * C ABI; all pointers are DEVICE pointers, 16-byte aligned; each call enqueues one launch on
 * `stream` (hipStream_t as void*).  Status codes are those of dlrm_hot.h.
 */
#ifndef DLRM_CEILINGS_H_
#define DLRM_CEILINGS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Memory-bound kernels of known traffic in the access
 * patterns of the path, for a benchmark to time, so that a kernel of the path can be held against
 * what the board sustains for its pattern as well as against the nominal HBM peak.  Each call
 * enqueues one launch on `stream`; all pointers are device pointers, 16-byte aligned.
 *   copy   : dst[0:bytes] = src[0:bytes]; bytes a multiple of 16.  Traffic: bytes read + bytes written.
 *   read   : reads src[0:bytes]; `sink` receives dlrm_ceiling_sink_floats() meaningless floats.
 *   gather : reads the n listed rows (row r = table[r*row_bytes : (r+1)*row_bytes], row_bytes one of
 *            64, 128, 256, 512; `rows` uint32 [n]) whole, four rows in flight per lane group, like the
 *            pooled lookup of Eq. (2) with nothing to add them to.  Traffic: n*row_bytes read.
 *   rmw    : multiplies every fp32 element of the n listed rows by 1 + 2^-10 in place: each row is
 *            read once and written once, like the row update of Sec. 5.1 without its gradient.  The
 *            listed rows must be distinct (else the result depends on the order).  Traffic:
 *            n*row_bytes read + n*row_bytes written.
 * Out-of-range row numbers are undefined behaviour.  Errors: DLRM_ERR_NULL, DLRM_ERR_BAD_SHAPE
 * (size 0, misaligned, unsupported row_bytes).
 */
int32_t dlrm_ceiling_sink_floats(void);
int32_t dlrm_ceiling_copy(const void* src, void* dst, size_t bytes, void* stream);
int32_t dlrm_ceiling_read(const void* src, size_t bytes, float* sink, void* stream);
int32_t dlrm_ceiling_gather(const void* table, const uint32_t* rows, int64_t n, int32_t row_bytes, float* sink,
                            void* stream);
int32_t dlrm_ceiling_rmw(void* table, const uint32_t* rows, int64_t n, int32_t row_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DLRM_CEILINGS_H_ */
