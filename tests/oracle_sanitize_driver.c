/* Drives the CPU oracle through exact-size heap buffers; built by tests/test_oracle_sanitizers.py
 * together with oracle/sa_oracle.c under AddressSanitizer and UndefinedBehaviorSanitizer.  Any read
 * or write outside a buffer, and any undefined arithmetic, aborts the run.  TEST INFRASTRUCTURE. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_dense_rows(const uint16_t *, const uint16_t *, const uint16_t *, int, int, int, int, double,
                      const int32_t *, int, double *, double *);
int oracle_estimate(const uint16_t *, const uint16_t *, int, int, int, int, int, int, double, double *,
                    double *, double *);
int oracle_default_budgets(int, int, double, int32_t[5]);
int64_t oracle_triangular_count(int, int, int);
int oracle_build_index(const float *, const float *, const float *, int, int, int, int, int, int, int, int,
                       int, int, int, int, int, const int32_t *, int, int32_t *, int32_t *, int32_t *,
                       int32_t *, int32_t *, int32_t *, int32_t *, int, int);
int oracle_masked_rows(const uint16_t *, const uint16_t *, const uint16_t *, int, int, int, int, int, double,
                       int, int, int, const int32_t *, const int32_t *, const int32_t *, const int32_t *,
                       const int32_t *, const int32_t *, const int32_t *, int, double *, double *, int64_t *);
int64_t oracle_mask_count(int, int, int, int, int, int, const int32_t *, const int32_t *, const int32_t *,
                          const int32_t *, const int32_t *, const int32_t *);

static uint32_t rng = 12345u;
static float unif(void) { rng = rng * 1664525u + 1013904223u; return (float)((rng >> 8) & 0xFFFF) / 65536.0f; }
static uint16_t bf16(float x) { union { float f; uint32_t u; } c; c.f = x; return (uint16_t)((c.u + 0x7FFFu + ((c.u >> 16) & 1u)) >> 16); }

static int run(int Hq, int Hkv, int N, int b, int w, double rho, int block_select, int diagonal_select) {
  const int d = 128, nb = N / b;
  const size_t nq = (size_t)Hq * N * d, nk = (size_t)Hkv * N * d;
  uint16_t *Q = malloc(nq * 2), *K = malloc(nk * 2), *V = malloc(nk * 2);
  for (size_t i = 0; i < nq; ++i) Q[i] = bf16(2.f * unif() - 1.f);
  for (size_t i = 0; i < nk; ++i) { K[i] = bf16(2.f * unif() - 1.f); V[i] = bf16(2.f * unif() - 1.f); }
  const double scale = 1.0 / sqrt((double)d);
  double *v = malloc(sizeof(double) * Hq * N), *s = malloc(sizeof(double) * Hq * N);
  double *blk = malloc(sizeof(double) * Hq * nb * nb);
  if (oracle_estimate(Q, K, Hq, Hkv, N, d, b, w, scale, v, s, blk)) return 1;
  float *vf = malloc(4 * (size_t)Hq * N), *sf = malloc(4 * (size_t)Hq * N), *bf = malloc(4 * (size_t)Hq * nb * nb);
  for (size_t i = 0; i < (size_t)Hq * N; ++i) { vf[i] = (float)v[i]; sf[i] = (float)s[i]; }
  for (size_t i = 0; i < (size_t)Hq * nb * nb; ++i) bf[i] = (float)blk[i];
  int32_t bud[5];
  if (oracle_default_budgets(N, b, rho, bud)) return 2;
  const int sink = bud[0], local = bud[1], kv = bud[2], ks = bud[3], kb = bud[4];
  int64_t cap = oracle_triangular_count(nb, sink, local);
  int64_t kcap = kb + (block_select == 1 ? nb : 0);
  if (kcap > cap) cap = kcap;
  if (diagonal_select) {
    int64_t dc = 0, m = 2 * (int64_t)(ks < N ? ks : N) + 1;
    for (int R = 0; R < nb; ++R) dc += (R + 1 < m ? R + 1 : m);
    if (dc > cap) cap = dc;
  }
  for (int ov = -1; ov < 3; ++ov) {   /* run-time rule, then every head forced to each pattern */
    int32_t *override = NULL;
    if (ov >= 0) { override = malloc(4 * (size_t)Hq); for (int h = 0; h < Hq; ++h) override[h] = ov; }
    int32_t *pattern = malloc(4 * (size_t)Hq), *n_cols = malloc(4 * (size_t)Hq), *n_offs = malloc(4 * (size_t)Hq);
    int32_t *cols = malloc(4 * (size_t)Hq * kv), *offs = malloc(4 * (size_t)Hq * ks);
    int32_t *rowptr = malloc(4 * (size_t)Hq * (nb + 1)), *blkcols = malloc(4 * (size_t)Hq * cap);
    if (oracle_build_index(vf, sf, bf, Hq, N, b, w, sink, local, kv, ks, kb, 4, 4, 4, 1, override, (int)cap,
                           pattern, n_cols, cols, n_offs, offs, rowptr, blkcols, block_select, diagonal_select))
      return 3;
    const int nrows = 5;
    int32_t rows[5] = {0, 1, N / 2, N - 2, N - 1};
    double *O = malloc(sizeof(double) * Hq * nrows * d), *ws = malloc(sizeof(double) * Hq * nrows);
    int64_t *kept = malloc(sizeof(int64_t) * Hq * nrows);
    if (oracle_masked_rows(Q, K, V, Hq, Hkv, N, d, b, scale, kv, ks, (int)cap, n_cols, cols, n_offs, offs, rowptr,
                           blkcols, rows, nrows, O, ws, kept))
      return 4;
    for (int i = 0; i < Hq * nrows; ++i)
      if (fabs(ws[i] - 1.0) > 1e-9) return 5;
    int64_t total = 0;
    for (int h = 0; h < Hq; ++h) total += oracle_mask_count(N, b, h, kv, ks, (int)cap, n_cols, cols, n_offs, offs, rowptr, blkcols);
    if (total <= 0) return 6;
    double *Od = malloc(sizeof(double) * Hq * nrows * d), *wd = malloc(sizeof(double) * Hq * nrows);
    if (oracle_dense_rows(Q, K, V, Hq, Hkv, N, d, scale, rows, nrows, Od, wd)) return 7;
    free(Od); free(wd); free(O); free(ws); free(kept); free(pattern); free(n_cols); free(n_offs); free(cols);
    free(offs); free(rowptr); free(blkcols); free(override);
  }
  free(Q); free(K); free(V); free(v); free(s); free(blk); free(vf); free(sf); free(bf);
  return 0;
}

int main(void) {
  const int cases[][8] = {/* Hq Hkv N b w rho% block_select diagonal_select */
                          {4, 2, 512, 64, 64, 20, 0, 0}, {3, 1, 384, 128, 32, 30, 1, 0}, {2, 2, 256, 64, 16, 50, 2, 1},
                          {2, 1, 64, 64, 64, 100, 0, 1}, {4, 4, 640, 128, 64, 10, 1, 1}};
  for (unsigned c = 0; c < sizeof(cases) / sizeof(cases[0]); ++c) {
    const int *p = cases[c];
    const int rc = run(p[0], p[1], p[2], p[3], p[4], p[5] / 100.0, p[6], p[7]);
    if (rc) { printf("case %u failed with %d\n", c, rc); return 1; }
  }
  printf("oracle sanitizer run ok\n");
  return 0;
}
