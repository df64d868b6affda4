/*
 * Sanitizer driver (TEST INFRASTRUCTURE): runs every entry point of the CPU oracle (dlrm_oracle.c) and of
 * the trace tools (workloads/trace_tools.c) on small seeded inputs with edge cases (empty bags, repeated
 * indices, a table nobody looks up, one-row tables, fp16 and bf16 storage).  Built by the CPU tests with
 * gcc -fsanitize=address,undefined -fno-sanitize-recover together with both sources: any out-of-bounds
 * access, use of uninitialised heap, signed overflow or misaligned access ends the run with a report.
 * Prints a checksum so that the optimiser cannot drop the calls.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_lengths_to_offsets(const int32_t*, int32_t, int32_t, int64_t*, int64_t*);
int64_t oracle_validate_csr(int32_t, int32_t, const int64_t*, const int64_t*, const int64_t*, const int64_t*);
int oracle_emb_bag_fwd(int32_t, int32_t, int32_t, int32_t, const void* const*, const int64_t*, const int64_t*,
                       const int64_t*, const int64_t*, double*, int64_t, int64_t);
int oracle_interact_dot_fwd(const float*, int32_t, int32_t, int32_t, double*);
int oracle_interact_dot_bwd(const float*, const float*, int32_t, int32_t, int32_t, double*);
int oracle_group_rows(int32_t, int32_t, const int64_t*, const int64_t*, const int64_t*, int64_t*, int32_t*, int64_t*,
                      int64_t*, int64_t*);
int oracle_emb_bag_bwd_sgd(int32_t, int32_t, int32_t, int32_t, void* const*, const int64_t*, const int64_t*,
                           const int64_t*, const int64_t*, const float*, int64_t, int64_t, double, int32_t, double*,
                           int64_t*, int64_t*);
int oracle_emb_bag_bwd_adagrad(int32_t, int32_t, int32_t, int32_t, void* const*, float* const*, const int64_t*,
                               const int64_t*, const int64_t*, const int64_t*, const float*, int64_t, int64_t, double,
                               double);
int oracle_emb_bag_fwd_weighted(int32_t, int32_t, int32_t, int32_t, const void* const*, const int64_t*, const int64_t*,
                                const int64_t*, const int64_t*, const float*, double*, int64_t, int64_t);
int oracle_emb_bag_bwd_weighted(int32_t, int32_t, int32_t, int32_t, void* const*, float* const*, const int64_t*,
                                const int64_t*, const int64_t*, const int64_t*, const float*, const float*, int64_t,
                                int64_t, double, double, int32_t);
uint16_t oracle_double_to_half(double);
uint16_t oracle_double_to_bf16(double);
double oracle_half_to_double(uint16_t);
double oracle_bf16_to_double(uint16_t);
void oracle_set_threads(int);
int trace_profile(const int64_t*, int64_t, int64_t, int64_t*, int64_t*, int64_t*, int64_t*);
int trace_generate(const int64_t*, int64_t, const double*, int64_t, const double*, int64_t, double, int64_t*);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint64_t next_u64(void) { /* splitmix64 */
  uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
static double next_unit(void) { return (double)(next_u64() >> 11) / 9007199254740992.0; }

#define CHECK(x)                                                   \
  do {                                                             \
    if ((x) != 0) {                                                \
      fprintf(stderr, "sanitize_driver: %s failed\n", #x);         \
      return 1;                                                    \
    }                                                              \
  } while (0)

static int run_shape(int K, int B, int d, int dtype, const int64_t* rows, int max_len, double* checksum) {
  const int F = K + 1, P = F * (F - 1) / 2;
  int32_t* lengths = (int32_t*)malloc(sizeof(int32_t) * (size_t)K * B);
  int64_t* offsets = (int64_t*)malloc(sizeof(int64_t) * (size_t)K * (B + 1));
  int64_t* tbl_off = (int64_t*)malloc(sizeof(int64_t) * (size_t)(K + 1));
  for (int i = 0; i < K * B; ++i) lengths[i] = (int32_t)(next_u64() % (uint64_t)(max_len + 1));
  for (int b = 0; b < B && K > 1; ++b) lengths[(K - 1) * B + b] = 0; /* a table nobody looks up */
  CHECK(oracle_lengths_to_offsets(lengths, K, B, offsets, tbl_off));
  const int64_t nnz = tbl_off[K];
  int64_t* idx = (int64_t*)malloc(sizeof(int64_t) * (size_t)(nnz > 0 ? nnz : 1));
  float* wts = (float*)malloc(sizeof(float) * (size_t)(nnz > 0 ? nnz : 1));
  for (int k = 0; k < K; ++k)
    for (int64_t p = tbl_off[k]; p < tbl_off[k + 1]; ++p) {
      idx[p] = (int64_t)(next_u64() % (uint64_t)rows[k]);
      if (p > tbl_off[k] && (next_u64() & 3) == 0) idx[p] = idx[p - 1]; /* repeats */
      wts[p] = (float)(0.5 + next_unit());
    }
  if (oracle_validate_csr(K, B, rows, idx, offsets, tbl_off) != 0) return 1;
  const size_t eb = dtype == 0 ? 4 : 2;
  void** tables = (void**)malloc(sizeof(void*) * (size_t)K);
  float** state = (float**)malloc(sizeof(float*) * (size_t)K);
  for (int k = 0; k < K; ++k) {
    const size_t n = (size_t)rows[k] * d;
    tables[k] = malloc(n * eb);
    state[k] = (float*)malloc(n * sizeof(float));
    for (size_t i = 0; i < n; ++i) {
      const double v = next_unit() - 0.5;
      if (dtype == 0) ((float*)tables[k])[i] = (float)v;
      else if (dtype == 1) ((uint16_t*)tables[k])[i] = oracle_double_to_half(v);
      else ((uint16_t*)tables[k])[i] = oracle_double_to_bf16(v);
      state[k][i] = (float)(0.1 + next_unit());
    }
  }
  double* S = (double*)malloc(sizeof(double) * (size_t)B * K * d);
  CHECK(oracle_emb_bag_fwd(K, B, d, dtype, (const void* const*)tables, rows, idx, offsets, tbl_off, S, (int64_t)K * d, d));
  CHECK(oracle_emb_bag_fwd_weighted(K, B, d, dtype, (const void* const*)tables, rows, idx, offsets, tbl_off, wts, S,
                                    (int64_t)K * d, d));
  float* T = (float*)malloc(sizeof(float) * (size_t)B * F * d);
  for (int b = 0; b < B; ++b)
    for (int f = 0; f < F; ++f)
      for (int c = 0; c < d; ++c)
        T[((size_t)b * F + f) * d + c] = f == 0 ? (float)(next_unit() - 0.5) : (float)S[((size_t)b * K + (f - 1)) * d + c];
  double* R = (double*)malloc(sizeof(double) * (size_t)B * (d + P));
  CHECK(oracle_interact_dot_fwd(T, B, F, d, R));
  float* dR = (float*)malloc(sizeof(float) * (size_t)B * (d + P));
  for (size_t i = 0; i < (size_t)B * (d + P); ++i) dR[i] = (float)(next_unit() - 0.5);
  double* dT = (double*)malloc(sizeof(double) * (size_t)B * F * d);
  CHECK(oracle_interact_dot_bwd(T, dR, B, F, d, dT));
  float* dS = (float*)malloc(sizeof(float) * (size_t)B * K * d);
  for (int b = 0; b < B; ++b)
    for (int k = 0; k < K; ++k)
      for (int c = 0; c < d; ++c) dS[((size_t)b * K + k) * d + c] = (float)dT[((size_t)b * F + k + 1) * d + c];
  const size_t n1 = (size_t)(nnz > 0 ? nnz : 1);
  int64_t* spos = (int64_t*)malloc(sizeof(int64_t) * n1);
  int32_t* sbag = (int32_t*)malloc(sizeof(int32_t) * n1);
  int64_t* uniq = (int64_t*)malloc(sizeof(int64_t) * n1);
  int64_t* seg = (int64_t*)malloc(sizeof(int64_t) * n1);
  int64_t* nu = (int64_t*)malloc(sizeof(int64_t) * (size_t)K);
  CHECK(oracle_group_rows(K, B, idx, offsets, tbl_off, spos, sbag, uniq, seg, nu));
  double* grad = (double*)malloc(sizeof(double) * n1 * d);
  CHECK(oracle_emb_bag_bwd_sgd(K, B, d, dtype, tables, rows, idx, offsets, tbl_off, dS, (int64_t)K * d, d, 0.01, 1, grad,
                               uniq, nu));
  CHECK(oracle_emb_bag_bwd_sgd(K, B, d, dtype, tables, rows, idx, offsets, tbl_off, dS, (int64_t)K * d, d, 0.01, 0, NULL,
                               uniq, nu));
  CHECK(oracle_emb_bag_bwd_adagrad(K, B, d, dtype, tables, state, rows, idx, offsets, tbl_off, dS, (int64_t)K * d, d, 0.05,
                                   1e-8));
  CHECK(oracle_emb_bag_bwd_weighted(K, B, d, dtype, tables, NULL, rows, idx, offsets, tbl_off, wts, dS, (int64_t)K * d, d,
                                    0.01, 0.0, 0));
  CHECK(oracle_emb_bag_bwd_weighted(K, B, d, dtype, tables, state, rows, idx, offsets, tbl_off, wts, dS, (int64_t)K * d, d,
                                    0.05, 1e-8, 1));
  for (size_t i = 0; i < (size_t)B * (d + P); ++i) *checksum += R[i];
  for (int k = 0; k < K; ++k) {
    *checksum += dtype == 0 ? ((float*)tables[k])[0]
                            : (dtype == 1 ? oracle_half_to_double(((uint16_t*)tables[k])[0])
                                          : oracle_bf16_to_double(((uint16_t*)tables[k])[0]));
    free(tables[k]);
    free(state[k]);
  }
  free(lengths); free(offsets); free(tbl_off); free(idx); free(wts); free(tables); free(state); free(S); free(T);
  free(R); free(dR); free(dT); free(dS); free(spos); free(sbag); free(uniq); free(seg); free(nu); free(grad);
  return 0;
}

static int run_trace(int64_t m, int64_t n, double* checksum) {
  int64_t* tr = (int64_t*)malloc(sizeof(int64_t) * (size_t)n);
  for (int64_t i = 0; i < n; ++i) { /* skewed ids */
    const double r = next_unit();
    tr[i] = (int64_t)((double)m * r * r * r);
    if (tr[i] >= m) tr[i] = m - 1;
  }
  int64_t* u = (int64_t*)malloc(sizeof(int64_t) * (size_t)n);
  int64_t* cnt = (int64_t*)calloc((size_t)n + 1, sizeof(int64_t));
  int64_t n_u = 0, max_d = 0;
  CHECK(trace_profile(tr, n, m, u, &n_u, cnt, &max_d));
  double* cum = (double*)malloc(sizeof(double) * (size_t)(max_d + 1));
  double run = 0.0;
  for (int64_t d = 0; d <= max_d; ++d) {
    run += (double)cnt[d] / (double)n;
    cum[d] = run;
  }
  const int64_t len = 2 * n;
  double* r = (double*)malloc(sizeof(double) * (size_t)len);
  for (int64_t i = 0; i < len; ++i) r[i] = next_unit();
  int64_t* out = (int64_t*)malloc(sizeof(int64_t) * (size_t)len);
  CHECK(trace_generate(u, n_u, cum, max_d + 1, r, len, 0.0, out));
  CHECK(trace_generate(u, n_u, cum, max_d + 1, r, len, 0.2, out));
  for (int64_t i = 0; i < len; ++i) *checksum += (double)out[i];
  free(tr); free(u); free(cnt); free(cum); free(r); free(out);
  return 0;
}

int main(void) {
  double checksum = 0.0;
  oracle_set_threads(2);
  const int64_t rows_a[3] = {7, 1, 5};
  const int64_t rows_b[5] = {300, 2, 41, 1, 64};
  for (int dtype = 0; dtype < 3; ++dtype) {
    if (run_shape(3, 5, 8, dtype, rows_a, 4, &checksum)) return 1;
    if (run_shape(5, 33, 16, dtype, rows_b, 9, &checksum)) return 1;
    if (run_shape(1, 1, 8, dtype, rows_a, 0, &checksum)) return 1; /* one empty bag: nnz = 0 */
  }
  if (run_trace(50, 2000, &checksum)) return 1;
  if (run_trace(1, 10, &checksum)) return 1;
  if (run_trace(4000, 3000, &checksum)) return 1;
  printf("sanitize_driver ok, checksum %.6f\n", checksum);
  return 0;
}
