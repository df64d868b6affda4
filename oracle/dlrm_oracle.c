/*
 * CPU oracle for the DLRM sparse hot path.  TEST INFRASTRUCTURE ONLY: it is
 * what the HIP kernels are checked against and what the benchmark times as the
 * CPU baseline.  It shares no code with the HIP library and the product path
 * never calls it.
 *
 * Everything here is the plain definition written out as nested loops, with
 * fp64 accumulation:
 *   - pooled lookup           S = A^T W                     (Sec. 2.1.1, Eq. (1)-(2))
 *   - CSR batch encoding      lengths <-> offsets, indices  (Sec. 4.1, footnote example)
 *   - dot interaction         all distinct pairs of {x, s_1..s_K}, concatenated
 *                             after x                       (Sec. 2.2; strict triangle
 *                             as in Eq. (4)'s upper(V V^T))
 *   - backward of the two, by the chain rule (the paper prints no backward)
 *   - sparse SGD              W <- W - lr * dW on touched rows (Sec. 5.1: SGD,
 *                             no regularisation)
 *   - weighted pooling        Eq. (2) in full, s = sum_p a_p W[idx_p], and its backward
 *                             g_r = sum_{p: idx_p = r} a_p dS[bag(p)]
 *   - sparse Adagrad          the other optimizer Sec. 5.1 names, element-wise:
 *                             h <- h + dW^2, W <- W - lr * dW / (sqrt(h) + eps)
 *                             on touched rows
 * Table storage is fp32 (Sec. 5: fp32 parameters) or fp16/bf16 (widened exactly,
 * narrowed once with round-to-nearest-even).
 *
 * Parity pins: every function below is pinned by tests/test_oracle_*.py
 * (the printed CSR example, one-hot == row gather, dense A^T W by a library
 * matmul, tril(T T^T), closed forms for F = 2, finite differences, count x g,
 * numpy.unique, exhaustive fp16 widening / RNE narrowing against numpy; Adagrad:
 * closed forms, the coalescing of duplicates, torch.optim.Adagrad on the CPU;
 * weighted pooling: the dense weighted matrix A through a library matmul, unit
 * weights == the unweighted functions, a repeated index adds its weights).
 *
 * Optional OpenMP `parallel for` over the outermost independent loop is the only
 * concession to speed; oracle_set_threads(1) gives the single-thread run.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F32 = 0, ORC_F16 = 1, ORC_BF16 = 2 };
enum { ORC_OK = 0, ORC_ERR_INDEX = -1, ORC_ERR_CSR = -2, ORC_ERR_ARG = -3, ORC_ERR_MEM = -4 };

static int g_threads = 0; /* 0 = leave OpenMP's default */

void oracle_set_threads(int n) { g_threads = n; }

int oracle_get_threads(void) {
#ifdef _OPENMP
  return g_threads > 0 ? g_threads : omp_get_max_threads();
#else
  return 1;
#endif
}

#ifdef _OPENMP
#define ORC_NT (g_threads > 0 ? g_threads : omp_get_max_threads())
#endif

/* ---------------- storage formats ---------------- */

/* binary16 -> double, exact (1 sign, 5 exponent bits bias 15, 10 fraction bits). */
double oracle_half_to_double(uint16_t h) {
  int sign = (h >> 15) & 1;
  int ex = (h >> 10) & 0x1F;
  int fr = h & 0x3FF;
  double v;
  if (ex == 0)
    v = ldexp((double)fr, -24); /* subnormal: fr * 2^-10 * 2^-14 */
  else if (ex == 31)
    v = fr ? NAN : INFINITY;
  else
    v = ldexp((double)(fr + 1024), ex - 25); /* (1 + fr/1024) * 2^(ex-15) */
  return sign ? -v : v;
}

/* double -> binary16, one rounding, ties to even. */
uint16_t oracle_double_to_half(double v) {
  uint16_t sign = signbit(v) ? 0x8000u : 0u;
  double a = fabs(v);
  if (isnan(v)) return (uint16_t)(sign | 0x7E00u);
  if (a >= 65520.0) return (uint16_t)(sign | 0x7C00u); /* >= max + half ulp -> inf */
  if (a == 0.0) return sign;
  int e;
  (void)frexp(a, &e); /* a = f * 2^e, f in [0.5,1) -> exponent of leading bit is e-1 */
  int lead = e - 1;
  if (lead < -14) lead = -14;              /* subnormal range shares the spacing 2^-24 */
  double q = ldexp(a, 10 - lead);          /* a in units of the local spacing; exact scaling */
  double r = nearbyint(q);                 /* default rounding mode: ties to even; exact ints */
  /* r is in [0, 2048]; r == 2048 means the round carried into the next binade */
  int64_t n = (int64_t)r;
  int64_t bits;
  if (lead == -14 && n < 1024) {
    bits = n; /* subnormal (or zero) */
  } else {
    if (n == 2048) { n = 1024; lead += 1; }
    bits = ((int64_t)(lead + 15) << 10) + (n - 1024);
  }
  return (uint16_t)(sign | (uint16_t)bits);
}

/* bfloat16 = the upper 16 bits of binary32. */
double oracle_bf16_to_double(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}

uint16_t oracle_double_to_bf16(double v) {
  uint16_t sign = signbit(v) ? 0x8000u : 0u;
  double a = fabs(v);
  if (isnan(v)) return (uint16_t)(sign | 0x7FC0u);
  if (a == 0.0) return sign;
  int e;
  (void)frexp(a, &e);
  int lead = e - 1;
  if (lead > 127) return (uint16_t)(sign | 0x7F80u);
  if (lead < -126) lead = -126;
  double q = ldexp(a, 7 - lead); /* 8-bit significand: units of 2^(lead-7) */
  double r = nearbyint(q);
  int64_t n = (int64_t)r;
  int64_t bits;
  if (lead == -126 && n < 128) {
    bits = n;
  } else {
    if (n == 256) { n = 128; lead += 1; }
    if (lead > 127) return (uint16_t)(sign | 0x7F80u);
    bits = ((int64_t)(lead + 127) << 7) + (n - 128);
  }
  return (uint16_t)(sign | (uint16_t)bits);
}

static inline double widen(const void* base, int dtype, int64_t i) {
  if (dtype == ORC_F32) return (double)((const float*)base)[i];
  if (dtype == ORC_F16) return oracle_half_to_double(((const uint16_t*)base)[i]);
  return oracle_bf16_to_double(((const uint16_t*)base)[i]);
}

static inline void narrow_store(void* base, int dtype, int64_t i, double v) {
  if (dtype == ORC_F32)
    ((float*)base)[i] = (float)v; /* one RNE rounding */
  else if (dtype == ORC_F16)
    ((uint16_t*)base)[i] = oracle_double_to_half(v);
  else
    ((uint16_t*)base)[i] = oracle_double_to_bf16(v);
}

/* ---------------- CSR encoding (Sec. 4.1 footnote) ---------------- */

/* lengths[K*B] -> offsets[K*(B+1)] (per-table, offsets[k][0] = 0, offsets[k][B] = nnz_k)
 * and tbl_off[K+1] (start of table k's slice in the concatenated index array). */
int oracle_lengths_to_offsets(const int32_t* lengths, int32_t K, int32_t B, int64_t* offsets,
                              int64_t* tbl_off) {
  if (!lengths || !offsets || !tbl_off || K <= 0 || B <= 0) return ORC_ERR_ARG;
  tbl_off[0] = 0;
  for (int32_t k = 0; k < K; ++k) {
    int64_t* off = offsets + (int64_t)k * (B + 1);
    off[0] = 0;
    for (int32_t b = 0; b < B; ++b) {
      if (lengths[(int64_t)k * B + b] < 0) return ORC_ERR_CSR;
      off[b + 1] = off[b] + lengths[(int64_t)k * B + b];
    }
    tbl_off[k + 1] = tbl_off[k] + off[B];
  }
  return ORC_OK;
}

/* Counts violations: non-monotone offsets, offsets[k][0] != 0, offsets[k][B] != nnz_k,
 * index outside [0, m_k). */
int64_t oracle_validate_csr(int32_t K, int32_t B, const int64_t* rows, const int64_t* indices,
                            const int64_t* offsets, const int64_t* tbl_off) {
  int64_t bad = 0;
  for (int32_t k = 0; k < K; ++k) {
    const int64_t* off = offsets + (int64_t)k * (B + 1);
    int64_t nnz = tbl_off[k + 1] - tbl_off[k];
    if (off[0] != 0) ++bad;
    if (off[B] != nnz) ++bad;
    for (int32_t b = 0; b < B; ++b)
      if (off[b + 1] < off[b]) ++bad;
    for (int64_t p = 0; p < nnz; ++p) {
      int64_t r = indices[tbl_off[k] + p];
      if (r < 0 || r >= rows[k]) ++bad;
    }
  }
  return bad;
}

/* ---------------- pooled lookup, Eq. (2) with unit weights ---------------- */

/* S[b,k,:] = sum over the bag's positions of W_k[idx,:]; an index repeated in a
 * bag counts once per occurrence; an empty bag gives zeros.
 * out is double, addressed out[b*stride_b + k*stride_k + c]. */
int oracle_emb_bag_fwd(int32_t K, int32_t B, int32_t d, int32_t dtype, const void* const* tables,
                       const int64_t* rows, const int64_t* indices, const int64_t* offsets,
                       const int64_t* tbl_off, double* out, int64_t stride_b, int64_t stride_k) {
  if (!tables || !rows || !offsets || !tbl_off || !out || K <= 0 || B <= 0 || d <= 0)
    return ORC_ERR_ARG;
  int status = ORC_OK;
#ifdef _OPENMP
#pragma omp parallel for collapse(2) schedule(static) num_threads(ORC_NT)
#endif
  for (int32_t k = 0; k < K; ++k) {
    for (int32_t b = 0; b < B; ++b) {
      const int64_t* off = offsets + (int64_t)k * (B + 1);
      const int64_t* idx = indices + tbl_off[k];
      double* o = out + (int64_t)b * stride_b + (int64_t)k * stride_k;
      for (int32_t c = 0; c < d; ++c) o[c] = 0.0;
      for (int64_t p = off[b]; p < off[b + 1]; ++p) {
        int64_t r = idx[p];
        if (r < 0 || r >= rows[k]) {
          status = ORC_ERR_INDEX;
          continue;
        }
        for (int32_t c = 0; c < d; ++c) o[c] += widen(tables[k], dtype, r * d + c);
      }
    }
  }
  return status;
}

/* ---------------- dot interaction, Sec. 2.2 ---------------- */

/* T[B,F,d] (row 0 = processed dense vector, row k+1 = pooled vector of table k).
 * R[b] = [ T[b,0,:] | <T[b,i],T[b,j]> for i = 1..F-1, j = 0..i-1 ]  (width d + F(F-1)/2). */
int oracle_interact_dot_fwd(const float* T, int32_t B, int32_t F, int32_t d, double* R) {
  if (!T || !R || B <= 0 || F <= 0 || d <= 0) return ORC_ERR_ARG;
  int64_t P = (int64_t)F * (F - 1) / 2;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(ORC_NT)
#endif
  for (int32_t b = 0; b < B; ++b) {
    const float* Tb = T + (int64_t)b * F * d;
    double* Rb = R + (int64_t)b * (d + P);
    for (int32_t c = 0; c < d; ++c) Rb[c] = (double)Tb[c];
    int64_t q = d;
    for (int32_t i = 1; i < F; ++i)
      for (int32_t j = 0; j < i; ++j) {
        double acc = 0.0;
        for (int32_t c = 0; c < d; ++c)
          acc += (double)Tb[(int64_t)i * d + c] * (double)Tb[(int64_t)j * d + c];
        Rb[q++] = acc;
      }
  }
  return ORC_OK;
}

/* Chain rule through the above: with g_ij = dR[b, d + pair(i,j)],
 * dT[b,i,:] += g_ij T[b,j,:], dT[b,j,:] += g_ij T[b,i,:], and dT[b,0,:] += dR[b,0:d]. */
int oracle_interact_dot_bwd(const float* T, const float* dR, int32_t B, int32_t F, int32_t d,
                            double* dT) {
  if (!T || !dR || !dT || B <= 0 || F <= 0 || d <= 0) return ORC_ERR_ARG;
  int64_t P = (int64_t)F * (F - 1) / 2;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(ORC_NT)
#endif
  for (int32_t b = 0; b < B; ++b) {
    const float* Tb = T + (int64_t)b * F * d;
    const float* gb = dR + (int64_t)b * (d + P);
    double* o = dT + (int64_t)b * F * d;
    for (int64_t t = 0; t < (int64_t)F * d; ++t) o[t] = 0.0;
    for (int32_t c = 0; c < d; ++c) o[c] += (double)gb[c];
    int64_t q = d;
    for (int32_t i = 1; i < F; ++i)
      for (int32_t j = 0; j < i; ++j) {
        double g = (double)gb[q++];
        for (int32_t c = 0; c < d; ++c) {
          o[(int64_t)i * d + c] += g * (double)Tb[(int64_t)j * d + c];
          o[(int64_t)j * d + c] += g * (double)Tb[(int64_t)i * d + c];
        }
      }
  }
  return ORC_OK;
}

/* ---------------- backward grouping ---------------- */

typedef struct {
  int64_t row;
  int64_t pos;
} orc_pair;

static int pair_cmp(const void* a, const void* b) {
  const orc_pair* x = (const orc_pair*)a;
  const orc_pair* y = (const orc_pair*)b;
  if (x->row != y->row) return x->row < y->row ? -1 : 1;
  if (x->pos != y->pos) return x->pos < y->pos ? -1 : 1;
  return 0;
}

/* Group the positions of every table by row id.  Per table k, writes into the
 * table's slice [tbl_off[k], tbl_off[k+1]) of the output arrays:
 *   sorted_pos : local positions ordered by (row asc, position asc)
 *   sorted_bag : the bag each of those positions belongs to
 *   uniq_rows  : the distinct rows ascending   (first n_uniq[k] entries of the slice)
 *   seg_start  : start of each row's run in sorted_pos, local to the slice
 *                (first n_uniq[k] entries; a run ends where the next starts or at nnz_k)
 */
int oracle_group_rows(int32_t K, int32_t B, const int64_t* indices, const int64_t* offsets,
                      const int64_t* tbl_off, int64_t* sorted_pos, int32_t* sorted_bag,
                      int64_t* uniq_rows, int64_t* seg_start, int64_t* n_uniq) {
  if (!offsets || !tbl_off || !n_uniq || K <= 0 || B <= 0) return ORC_ERR_ARG;
  int status = ORC_OK;
  for (int32_t k = 0; k < K; ++k) {
    int64_t base = tbl_off[k], nnz = tbl_off[k + 1] - tbl_off[k];
    const int64_t* off = offsets + (int64_t)k * (B + 1);
    orc_pair* pr = (orc_pair*)malloc(sizeof(orc_pair) * (size_t)(nnz > 0 ? nnz : 1));
    int32_t* bag_of = (int32_t*)malloc(sizeof(int32_t) * (size_t)(nnz > 0 ? nnz : 1));
    if (!pr || !bag_of) {
      free(pr);
      free(bag_of);
      return ORC_ERR_MEM;
    }
    for (int32_t b = 0; b < B; ++b)
      for (int64_t p = off[b]; p < off[b + 1]; ++p) bag_of[p] = b;
    for (int64_t p = 0; p < nnz; ++p) {
      pr[p].row = indices[base + p];
      pr[p].pos = p;
    }
    qsort(pr, (size_t)nnz, sizeof(orc_pair), pair_cmp);
    int64_t u = 0;
    for (int64_t t = 0; t < nnz; ++t) {
      sorted_pos[base + t] = pr[t].pos;
      sorted_bag[base + t] = bag_of[pr[t].pos];
      if (t == 0 || pr[t].row != pr[t - 1].row) {
        uniq_rows[base + u] = pr[t].row;
        seg_start[base + u] = t;
        ++u;
      }
    }
    n_uniq[k] = u;
    free(pr);
    free(bag_of);
  }
  return status;
}

/* ---------------- embedding backward + sparse SGD ---------------- */

/* For every distinct row r of table k:  g = sum over the positions p that look
 * r up of dS[bag(p), k, :]  (transpose of Eq. (2));  W_k[r,:] <- W_k[r,:] - lr*g,
 * duplicates summed first and applied once, one rounding to the storage type.
 * If row_grad != NULL it receives g (double), laid out like uniq_rows x d per
 * table slice: row_grad[(tbl_off[k] + u) * d + c].  apply = 0 leaves tables alone. */
int oracle_emb_bag_bwd_sgd(int32_t K, int32_t B, int32_t d, int32_t dtype, void* const* tables,
                           const int64_t* rows, const int64_t* indices, const int64_t* offsets,
                           const int64_t* tbl_off, const float* dS, int64_t stride_b,
                           int64_t stride_k, double lr, int32_t apply, double* row_grad,
                           int64_t* uniq_rows_out, int64_t* n_uniq_out) {
  if (!tables || !rows || !offsets || !tbl_off || !dS || K <= 0 || B <= 0 || d <= 0)
    return ORC_ERR_ARG;
  int64_t nnz_total = tbl_off[K];
  size_t n = (size_t)(nnz_total > 0 ? nnz_total : 1);
  int64_t* sorted_pos = (int64_t*)malloc(sizeof(int64_t) * n);
  int32_t* sorted_bag = (int32_t*)malloc(sizeof(int32_t) * n);
  int64_t* uniq = (int64_t*)malloc(sizeof(int64_t) * n);
  int64_t* seg = (int64_t*)malloc(sizeof(int64_t) * n);
  int64_t* nu = (int64_t*)malloc(sizeof(int64_t) * (size_t)K);
  int status = ORC_ERR_MEM;
  if (sorted_pos && sorted_bag && uniq && seg && nu) {
    status = oracle_group_rows(K, B, indices, offsets, tbl_off, sorted_pos, sorted_bag, uniq, seg,
                               nu);
  }
  if (status == ORC_OK) {
    for (int32_t k = 0; k < K; ++k) {
      int64_t base = tbl_off[k], nnz = tbl_off[k + 1] - tbl_off[k];
      int64_t U = nu[k];
      int bad = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 64) num_threads(ORC_NT)
#endif
      for (int64_t u = 0; u < U; ++u) {
        int64_t r = uniq[base + u];
        if (r < 0 || r >= rows[k]) {
          bad = 1;
          continue;
        }
        int64_t t0 = seg[base + u], t1 = (u + 1 < U) ? seg[base + u + 1] : nnz;
        for (int32_t c = 0; c < d; ++c) {
          double g = 0.0;
          for (int64_t t = t0; t < t1; ++t)
            g += (double)dS[(int64_t)sorted_bag[base + t] * stride_b + (int64_t)k * stride_k + c];
          if (row_grad) row_grad[(base + u) * d + c] = g;
          if (apply) {
            double w = widen(tables[k], dtype, r * d + c);
            narrow_store(tables[k], dtype, r * d + c, w - lr * g);
          }
        }
      }
      if (bad) status = ORC_ERR_INDEX;
      if (uniq_rows_out)
        for (int64_t u = 0; u < U; ++u) uniq_rows_out[base + u] = uniq[base + u];
      if (n_uniq_out) n_uniq_out[k] = U;
    }
  }
  free(sorted_pos);
  free(sorted_bag);
  free(uniq);
  free(seg);
  free(nu);
  return status;
}

/* Sparse Adagrad in place of the SGD step (Sec. 5.1 names both optimizers; the paper prints no
 * formula, this is the standard element-wise one).  For every distinct row r of table k, with
 * g the row's batch gradient as in oracle_emb_bag_bwd_sgd (duplicates summed first):
 *   h_k[r,:] <- h_k[r,:] + g*g            (fp32 state, one rounding)
 *   W_k[r,:] <- W_k[r,:] - lr * g / (sqrt(h_k[r,:]) + eps)   with the updated h, one rounding
 * Rows nobody looks up keep W and h. */
int oracle_emb_bag_bwd_adagrad(int32_t K, int32_t B, int32_t d, int32_t dtype, void* const* tables,
                               float* const* state, const int64_t* rows, const int64_t* indices,
                               const int64_t* offsets, const int64_t* tbl_off, const float* dS,
                               int64_t stride_b, int64_t stride_k, double lr, double eps) {
  if (!tables || !state || !rows || !offsets || !tbl_off || !dS || K <= 0 || B <= 0 || d <= 0)
    return ORC_ERR_ARG;
  int64_t nnz_total = tbl_off[K];
  size_t n = (size_t)(nnz_total > 0 ? nnz_total : 1);
  int64_t* sorted_pos = (int64_t*)malloc(sizeof(int64_t) * n);
  int32_t* sorted_bag = (int32_t*)malloc(sizeof(int32_t) * n);
  int64_t* uniq = (int64_t*)malloc(sizeof(int64_t) * n);
  int64_t* seg = (int64_t*)malloc(sizeof(int64_t) * n);
  int64_t* nu = (int64_t*)malloc(sizeof(int64_t) * (size_t)K);
  int status = ORC_ERR_MEM;
  if (sorted_pos && sorted_bag && uniq && seg && nu)
    status = oracle_group_rows(K, B, indices, offsets, tbl_off, sorted_pos, sorted_bag, uniq, seg, nu);
  if (status == ORC_OK) {
    for (int32_t k = 0; k < K; ++k) {
      int64_t base = tbl_off[k], nnz = tbl_off[k + 1] - tbl_off[k];
      int64_t U = nu[k];
      int bad = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 64) num_threads(ORC_NT)
#endif
      for (int64_t u = 0; u < U; ++u) {
        int64_t r = uniq[base + u];
        if (r < 0 || r >= rows[k]) {
          bad = 1;
          continue;
        }
        int64_t t0 = seg[base + u], t1 = (u + 1 < U) ? seg[base + u + 1] : nnz;
        for (int32_t c = 0; c < d; ++c) {
          double g = 0.0;
          for (int64_t t = t0; t < t1; ++t)
            g += (double)dS[(int64_t)sorted_bag[base + t] * stride_b + (int64_t)k * stride_k + c];
          double h = (double)state[k][r * d + c] + g * g;
          state[k][r * d + c] = (float)h;
          double w = widen(tables[k], dtype, r * d + c);
          narrow_store(tables[k], dtype, r * d + c, w - lr * g / (sqrt(h) + eps));
        }
      }
      if (bad) status = ORC_ERR_INDEX;
    }
  }
  free(sorted_pos);
  free(sorted_bag);
  free(uniq);
  free(seg);
  free(nu);
  return status;
}

/* ---------------- weighted pooling: Eq. (2) with its weights a ---------------- */

/* S[b,k,:] = sum over the bag's positions p of weights[tbl_off[k] + p] * W_k[idx_p,:]
 * (weights: fp32, parallel to indices).  Everything else as oracle_emb_bag_fwd. */
int oracle_emb_bag_fwd_weighted(int32_t K, int32_t B, int32_t d, int32_t dtype, const void* const* tables,
                                const int64_t* rows, const int64_t* indices, const int64_t* offsets,
                                const int64_t* tbl_off, const float* weights, double* out,
                                int64_t stride_b, int64_t stride_k) {
  if (!tables || !rows || !offsets || !tbl_off || !weights || !out || K <= 0 || B <= 0 || d <= 0)
    return ORC_ERR_ARG;
  int status = ORC_OK;
#ifdef _OPENMP
#pragma omp parallel for collapse(2) schedule(static) num_threads(ORC_NT)
#endif
  for (int32_t k = 0; k < K; ++k) {
    for (int32_t b = 0; b < B; ++b) {
      const int64_t* off = offsets + (int64_t)k * (B + 1);
      const int64_t* idx = indices + tbl_off[k];
      const float* a = weights + tbl_off[k];
      double* o = out + (int64_t)b * stride_b + (int64_t)k * stride_k;
      for (int32_t c = 0; c < d; ++c) o[c] = 0.0;
      for (int64_t p = off[b]; p < off[b + 1]; ++p) {
        int64_t r = idx[p];
        if (r < 0 || r >= rows[k]) {
          status = ORC_ERR_INDEX;
          continue;
        }
        for (int32_t c = 0; c < d; ++c) o[c] += (double)a[p] * widen(tables[k], dtype, r * d + c);
      }
    }
  }
  return status;
}

/* Backward of the weighted lookup with the row update: for every distinct row r of table k
 *   g = sum over the positions p that look r up of weights[tbl_off[k] + p] * dS[bag(p), k, :]
 * then, optimizer 0: W <- W - lr*g;  optimizer 1 (state != NULL): h <- h + g*g,
 * W <- W - lr*g / (sqrt(h) + eps).  The weights themselves receive no gradient here. */
int oracle_emb_bag_bwd_weighted(int32_t K, int32_t B, int32_t d, int32_t dtype, void* const* tables,
                                float* const* state, const int64_t* rows, const int64_t* indices,
                                const int64_t* offsets, const int64_t* tbl_off, const float* weights,
                                const float* dS, int64_t stride_b, int64_t stride_k, double lr,
                                double eps, int32_t optimizer) {
  if (!tables || !rows || !offsets || !tbl_off || !weights || !dS || K <= 0 || B <= 0 || d <= 0 ||
      (optimizer != 0 && optimizer != 1) || (optimizer == 1 && !state))
    return ORC_ERR_ARG;
  int64_t nnz_total = tbl_off[K];
  size_t n = (size_t)(nnz_total > 0 ? nnz_total : 1);
  int64_t* sorted_pos = (int64_t*)malloc(sizeof(int64_t) * n);
  int32_t* sorted_bag = (int32_t*)malloc(sizeof(int32_t) * n);
  int64_t* uniq = (int64_t*)malloc(sizeof(int64_t) * n);
  int64_t* seg = (int64_t*)malloc(sizeof(int64_t) * n);
  int64_t* nu = (int64_t*)malloc(sizeof(int64_t) * (size_t)K);
  int status = ORC_ERR_MEM;
  if (sorted_pos && sorted_bag && uniq && seg && nu)
    status = oracle_group_rows(K, B, indices, offsets, tbl_off, sorted_pos, sorted_bag, uniq, seg, nu);
  if (status == ORC_OK) {
    for (int32_t k = 0; k < K; ++k) {
      int64_t base = tbl_off[k], nnz = tbl_off[k + 1] - tbl_off[k];
      int64_t U = nu[k];
      int bad = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 64) num_threads(ORC_NT)
#endif
      for (int64_t u = 0; u < U; ++u) {
        int64_t r = uniq[base + u];
        if (r < 0 || r >= rows[k]) {
          bad = 1;
          continue;
        }
        int64_t t0 = seg[base + u], t1 = (u + 1 < U) ? seg[base + u + 1] : nnz;
        for (int32_t c = 0; c < d; ++c) {
          double g = 0.0;
          for (int64_t t = t0; t < t1; ++t)
            g += (double)weights[base + sorted_pos[base + t]] *
                 (double)dS[(int64_t)sorted_bag[base + t] * stride_b + (int64_t)k * stride_k + c];
          double w = widen(tables[k], dtype, r * d + c);
          if (optimizer == 1) {
            double h = (double)state[k][r * d + c] + g * g;
            state[k][r * d + c] = (float)h;
            narrow_store(tables[k], dtype, r * d + c, w - lr * g / (sqrt(h) + eps));
          } else {
            narrow_store(tables[k], dtype, r * d + c, w - lr * g);
          }
        }
      }
      if (bad) status = ORC_ERR_INDEX;
    }
  }
  free(sorted_pos);
  free(sorted_bag);
  free(uniq);
  free(seg);
  free(nu);
  return status;
}
