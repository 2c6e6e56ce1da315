/*
 * CPU oracle for dynamic sparse prefill attention.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 implementation of what the GPU path computes, written
 * from the paper's algorithms and used only by the tests, the smoke check and
 * the benchmark's cpu_baseline leg.  It shares no code with the HIP library
 * and must never be reached from the product path.
 *
 * Inputs are raw bf16 bit patterns (uint16); bf16 -> double is exact.  No
 * blocking, fusion or reordering beyond the definitions: every function is a
 * direct loop nest.  OpenMP only splits independent (head,row) work items.
 *
 * Passages followed:
 *   dense causal attention   - Alg. 1 "Evaluate Patterns" (A_dense) with the
 *                              causal mask of Alg. 2 "Compute Dense Attention
 *                              Scores";
 *   window estimator         - Alg. 2 "Compute Dense Attention Scores" and
 *                              "Select Top Indices" (SumRows, SumDiagonals),
 *                              restricted to the last w query rows (the "fast
 *                              approximation" of Main Idea / Dynamic Sparse
 *                              Masking);
 *   block map                - Alg. 3 "Compute Blocked Representation";
 *   index                    - Alg. 2 TopK / CombineIndices, Alg. 3 TopKBlocks,
 *                              Main Idea "Categorization of Attention Heads";
 *   masked attention         - Alg. 2 / Alg. 3 "Compute Sparse Attention"
 *                              (scale read inside the softmax, as in the dense
 *                              line of both algorithms).
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py (library
 * fp64 attention, closed forms, brute force, invariants).  None is unpinned.
 */
#include <math.h>
#include <omp.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define PAT_TRIANGULAR 0
#define PAT_INTERVAL_SLASH 1
#define PAT_BLOCK_CLUSTER 2

static inline double bf16_to_f64(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}

static double dot_bf16(const uint16_t *a, const uint16_t *b, int d) {
  double acc = 0.0;
  for (int t = 0; t < d; ++t) acc += bf16_to_f64(a[t]) * bf16_to_f64(b[t]);
  return acc;
}

/* OpenMP threads the loops below will use. */
int oracle_num_threads(void) { return omp_get_max_threads(); }

/* ------------------------------------------------------------------ dense */

/* O[h][r][:] = sum_{j<=i} softmax_j(scale * Q_h[i].K_kv[j]) V_kv[j], i = rows[r]
 * (rows == NULL: r = i over all N rows, nrows must equal N).
 * wsum[h][r] = sum of the normalised weights of that row (should be 1). */
int oracle_dense_rows(const uint16_t *Q, const uint16_t *K, const uint16_t *V, int Hq, int Hkv,
                      int N, int d, double scale, const int32_t *rows, int nrows, double *O,
                      double *wsum) {
  if (Hq % Hkv) return 1;
  const int g = Hq / Hkv;
  int err = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 4)
  for (int h = 0; h < Hq; ++h) {
    for (int r = 0; r < nrows; ++r) {
      const int i = rows ? rows[r] : r;
      if (i < 0 || i >= N) { err = 1; continue; }
      const uint16_t *q = Q + ((size_t)h * N + i) * d;
      const uint16_t *Kh = K + (size_t)(h / g) * N * d;
      const uint16_t *Vh = V + (size_t)(h / g) * N * d;
      double *p = (double *)malloc(sizeof(double) * (size_t)(i + 1));
      double m = -INFINITY;
      for (int j = 0; j <= i; ++j) {
        p[j] = scale * dot_bf16(q, Kh + (size_t)j * d, d);
        if (p[j] > m) m = p[j];
      }
      double Z = 0.0;
      for (int j = 0; j <= i; ++j) { p[j] = exp(p[j] - m); Z += p[j]; }
      double *o = O + ((size_t)h * nrows + r) * d;
      for (int t = 0; t < d; ++t) o[t] = 0.0;
      double ws = 0.0;
      for (int j = 0; j <= i; ++j) {
        const double wgt = p[j] / Z;
        ws += wgt;
        const uint16_t *vr = Vh + (size_t)j * d;
        for (int t = 0; t < d; ++t) o[t] += wgt * bf16_to_f64(vr[t]);
      }
      if (wsum) wsum[(size_t)h * nrows + r] = ws;
      free(p);
    }
  }
  return err;
}

/* A[i][j] = causal softmax weights of one head, all N x N (small N only). */
int oracle_dense_weights(const uint16_t *Q, const uint16_t *K, int Hq, int Hkv, int N, int d,
                         double scale, int h, double *A) {
  const int g = Hq / Hkv;
  const uint16_t *Kh = K + (size_t)(h / g) * N * d;
  for (int i = 0; i < N; ++i) {
    const uint16_t *q = Q + ((size_t)h * N + i) * d;
    double *a = A + (size_t)i * N;
    double m = -INFINITY;
    for (int j = 0; j <= i; ++j) {
      a[j] = scale * dot_bf16(q, Kh + (size_t)j * d, d);
      if (a[j] > m) m = a[j];
    }
    double Z = 0.0;
    for (int j = 0; j <= i; ++j) { a[j] = exp(a[j] - m); Z += a[j]; }
    for (int j = 0; j <= i; ++j) a[j] /= Z;
    for (int j = i + 1; j < N; ++j) a[j] = 0.0;
  }
  return 0;
}

/* -------------------------------------------------------------- estimator */

/* Window weights Ahat[h][i][j], i in [0,w): row N-w+i of the causal softmax. */
int oracle_window_weights(const uint16_t *Q, const uint16_t *K, int Hq, int Hkv, int N, int d,
                          int w, double scale, double *Ahat) {
  if (Hq % Hkv || w > N) return 1;
  const int g = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int h = 0; h < Hq; ++h) {
    for (int i = 0; i < w; ++i) {
      const int qi = N - w + i;
      const uint16_t *q = Q + ((size_t)h * N + qi) * d;
      const uint16_t *Kh = K + (size_t)(h / g) * N * d;
      double *a = Ahat + ((size_t)h * w + i) * N;
      double m = -INFINITY;
      for (int j = 0; j <= qi; ++j) {
        a[j] = scale * dot_bf16(q, Kh + (size_t)j * d, d);
        if (a[j] > m) m = a[j];
      }
      double Z = 0.0;
      for (int j = 0; j <= qi; ++j) { a[j] = exp(a[j] - m); Z += a[j]; }
      for (int j = 0; j <= qi; ++j) a[j] /= Z;
      for (int j = qi + 1; j < N; ++j) a[j] = 0.0;
    }
  }
  return 0;
}

/* v[h][j]   = sum_i Ahat[h][i][j]                          (vertical score)
 * s[h][o]   = sum_{i : N-w+i-o >= 0} Ahat[h][i][N-w+i-o]   (slash score)
 * blk[h][R][C] = softmax_{C<=R}(scale * mean(Q_h rows of R) . mean(K rows of C)),
 *                entries with C > R are 0. */
int oracle_estimate(const uint16_t *Q, const uint16_t *K, int Hq, int Hkv, int N, int d, int b,
                    int w, double scale, double *v, double *s, double *blk) {
  if (Hq % Hkv || N % b || w > N) return 1;
  const int g = Hq / Hkv;
  const int nb = N / b;
  /* vertical and slash scores: one window row at a time */
#pragma omp parallel for schedule(dynamic, 1)
  for (int h = 0; h < Hq; ++h) {
    const uint16_t *Kh = K + (size_t)(h / g) * N * d;
    double *vh = v + (size_t)h * N, *sh = s + (size_t)h * N;
    double *a = (double *)malloc(sizeof(double) * (size_t)N);
    for (int j = 0; j < N; ++j) { vh[j] = 0.0; sh[j] = 0.0; }
    for (int i = 0; i < w; ++i) {
      const int qi = N - w + i;
      const uint16_t *q = Q + ((size_t)h * N + qi) * d;
      double m = -INFINITY;
      for (int j = 0; j <= qi; ++j) {
        a[j] = scale * dot_bf16(q, Kh + (size_t)j * d, d);
        if (a[j] > m) m = a[j];
      }
      double Z = 0.0;
      for (int j = 0; j <= qi; ++j) { a[j] = exp(a[j] - m); Z += a[j]; }
      for (int j = 0; j <= qi; ++j) {
        const double p = a[j] / Z;
        vh[j] += p;
        sh[qi - j] += p;
      }
    }
    free(a);
  }
  /* block means */
  double *Qm = (double *)malloc(sizeof(double) * (size_t)Hq * nb * d);
  double *Km = (double *)malloc(sizeof(double) * (size_t)Hkv * nb * d);
#pragma omp parallel for collapse(2)
  for (int h = 0; h < Hq; ++h)
    for (int R = 0; R < nb; ++R) {
      double *o = Qm + ((size_t)h * nb + R) * d;
      for (int t = 0; t < d; ++t) o[t] = 0.0;
      for (int r = 0; r < b; ++r) {
        const uint16_t *q = Q + ((size_t)h * N + (size_t)R * b + r) * d;
        for (int t = 0; t < d; ++t) o[t] += bf16_to_f64(q[t]);
      }
      for (int t = 0; t < d; ++t) o[t] /= (double)b;
    }
#pragma omp parallel for collapse(2)
  for (int h = 0; h < Hkv; ++h)
    for (int C = 0; C < nb; ++C) {
      double *o = Km + ((size_t)h * nb + C) * d;
      for (int t = 0; t < d; ++t) o[t] = 0.0;
      for (int r = 0; r < b; ++r) {
        const uint16_t *k = K + ((size_t)h * N + (size_t)C * b + r) * d;
        for (int t = 0; t < d; ++t) o[t] += bf16_to_f64(k[t]);
      }
      for (int t = 0; t < d; ++t) o[t] /= (double)b;
    }
  /* block-level causal softmax */
#pragma omp parallel for collapse(2) schedule(dynamic, 8)
  for (int h = 0; h < Hq; ++h)
    for (int R = 0; R < nb; ++R) {
      const double *qm = Qm + ((size_t)h * nb + R) * d;
      double *row = blk + ((size_t)h * nb + R) * nb;
      double m = -INFINITY;
      for (int C = 0; C <= R; ++C) {
        const double *km = Km + ((size_t)(h / g) * nb + C) * d;
        double acc = 0.0;
        for (int t = 0; t < d; ++t) acc += qm[t] * km[t];
        row[C] = scale * acc;
        if (row[C] > m) m = row[C];
      }
      double Z = 0.0;
      for (int C = 0; C <= R; ++C) { row[C] = exp(row[C] - m); Z += row[C]; }
      for (int C = 0; C <= R; ++C) row[C] /= Z;
      for (int C = R + 1; C < nb; ++C) row[C] = 0.0;
    }
  free(Qm);
  free(Km);
  return 0;
}

/* ---------------------------------------------------------------- budgets */

/* Number of kept blocks of the Triangular pattern: key blocks C <= R with
 * C < sink_blocks or R - C < local_blocks, over all row blocks R. */
int64_t oracle_triangular_count(int nb, int sink_blocks, int local_blocks) {
  int64_t n = 0;
  for (int R = 0; R < nb; ++R)
    for (int C = 0; C <= R; ++C)
      if (C < sink_blocks || R - C < local_blocks) ++n;
  return n;
}

/* Default budgets from a keep fraction rho (our reading; the paper leaves
 * k_v, k_s, k_b and the FLOPs target as inputs).  out = {sink_blocks,
 * local_blocks, k_vertical, k_slash, k_blocks}. */
int oracle_default_budgets(int N, int b, double rho, int32_t out[5]) {
  if (N % b || rho <= 0.0 || rho > 1.0) return 1;
  const int64_t nb = N / b;
  const int64_t causal = nb * (nb + 1) / 2;
  int64_t T = (int64_t)floor(rho * (double)causal + 0.5);
  if (T < nb) T = nb;
  const int sink = 1;
  int L = 1;
  for (int cand = 1; cand <= nb; ++cand) {
    const int64_t cost = (int64_t)cand * nb - (int64_t)cand * (cand - 1) / 2 + (nb - cand) * sink;
    if (cost <= T) L = cand;
  }
  int64_t ks = (int64_t)floor(rho * (double)N / 128.0 + 0.5);
  if (ks < 1) ks = 1;
  int64_t kv = (int64_t)floor(rho * (double)N / 256.0 + 0.5);
  if (kv < 1) kv = 1;
  kv *= 64;
  if (kv > N) kv = N;
  if (ks > N) ks = N;
  out[0] = sink;
  out[1] = L;
  out[2] = (int32_t)kv;
  out[3] = (int32_t)ks;
  out[4] = (int32_t)T;
  return 0;
}

/* ------------------------------------------------------------------ index */

typedef struct { uint32_t key; int32_t idx; } keyidx;

static int cmp_keyidx(const void *pa, const void *pb) {
  const keyidx *a = (const keyidx *)pa, *b = (const keyidx *)pb;
  if (a->key != b->key) return a->key > b->key ? -1 : 1; /* larger score first */
  return a->idx < b->idx ? -1 : (a->idx > b->idx ? 1 : 0); /* ties: lower index first */
}

static int cmp_i32(const void *pa, const void *pb) {
  const int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
  return a < b ? -1 : (a > b ? 1 : 0);
}

static uint32_t f32_bits(float x) { uint32_t u; memcpy(&u, &x, 4); return u; }

/* floor(x * 2^30) for a finite fp32 x >= 0 (exact: a power-of-two scaling). */
static uint64_t fx30(float x) { return (uint64_t)floor((double)x * 1073741824.0); }

/* The k candidates with the largest score (fp32 bit pattern compared as an
 * unsigned integer; equal scores: lower index wins), written ascending by
 * index into out[0..k'), k' = min(k, n); returns k'.  idx_of maps candidate
 * position -> reported index (NULL: identity).  topsum (optional) receives
 * sum fx30 over the `probe` best. */
static int topk_full_sort(const float *score, const int32_t *idx_of, int n, int k, int32_t *out,
                          int probe, uint64_t *topsum) {
  keyidx *a = (keyidx *)malloc(sizeof(keyidx) * (size_t)(n > 0 ? n : 1));
  for (int t = 0; t < n; ++t) { a[t].key = f32_bits(score[t]); a[t].idx = idx_of ? idx_of[t] : t; }
  qsort(a, (size_t)n, sizeof(keyidx), cmp_keyidx);
  if (k > n) k = n;
  for (int t = 0; t < k; ++t) out[t] = a[t].idx;
  qsort(out, (size_t)k, sizeof(int32_t), cmp_i32);
  if (topsum) {
    uint64_t acc = 0;
    for (int t = 0; t < probe && t < n; ++t) {
      float f; uint32_t u = a[t].key; memcpy(&f, &u, 4);
      acc += fx30(f);
    }
    *topsum = acc;
  }
  free(a);
  return k;
}

/* Per-head pattern rule (our reading; the paper only says heads are categorised
 * at run time).  Integer arithmetic on fx30 of the fp32 scores:
 *   Triangular     if lift_den*C_T*E >= lift_num*Vtot*E_T
 *   Interval-Slash elif lift_den*(sumVtop+sumStop)*E >= lift_num*Vtot*(probe_v+probe_s)*w
 *   Block-Cluster  otherwise
 * with E the number of causal window entries, C_T / E_T the vertical mass /
 * entry count inside the Triangular region of the window rows. */
static int choose_pattern(const float *v, const float *s, int N, int b, int w, int sink_blocks,
                          int local_blocks, int probe_v, int probe_s, int lift_num, int lift_den) {
  const int nb = N / b;
  int64_t sb = (int64_t)sink_blocks * b;
  if (sb > N) sb = N;
  int64_t lb0 = (int64_t)(nb - local_blocks) * b;
  if (lb0 < sb) lb0 = sb;
  uint64_t Vtot = 0, CT = 0;
  for (int j = 0; j < N; ++j) {
    const uint64_t f = fx30(v[j]);
    Vtot += f;
    if (j < sb || j >= lb0) CT += f;
  }
  uint64_t E = 0, ET = 0;
  for (int i = 0; i < w; ++i) {
    const int64_t qi = (int64_t)N - w + i;
    E += (uint64_t)(qi + 1);
    ET += (uint64_t)(qi + 1 < sb ? qi + 1 : sb);
    if (qi + 1 > lb0) ET += (uint64_t)(qi + 1 - lb0);
  }
  typedef unsigned __int128 u128;
  if ((u128)lift_den * CT * E >= (u128)lift_num * Vtot * ET) return PAT_TRIANGULAR;
  uint64_t sumV = 0, sumS = 0;
  int32_t *tmp = (int32_t *)malloc(sizeof(int32_t) * (size_t)(probe_v > probe_s ? probe_v : probe_s) + 4);
  topk_full_sort(v, NULL, N, probe_v, tmp, probe_v, &sumV);
  topk_full_sort(s, NULL, N, probe_s, tmp, probe_s, &sumS);
  free(tmp);
  if ((u128)lift_den * (sumV + sumS) * E >=
      (u128)lift_num * Vtot * (uint64_t)(probe_v + probe_s) * (uint64_t)w)
    return PAT_INTERVAL_SLASH;
  return PAT_BLOCK_CLUSTER;
}

/* Index of every head from fp32 scores.  Layout (all int32, canonical):
 *   pattern[Hq]; n_cols[Hq]; cols[Hq][k_vertical] ascending, -1 padded;
 *   n_offs[Hq]; offs[Hq][k_slash] ascending, -1 padded;
 *   rowptr[Hq][nb+1]; blkcols[Hq][cap_b] ascending within a row, -1 padded.
 * Every head keeps the diagonal blocks (R,R).  Triangular: C < sink_blocks or
 * R-C < local_blocks.  Interval-Slash: top-k_vertical columns of v, top-k_slash
 * offsets of s.  Block-Cluster, block_select 0 (Alg. 3 TopKBlocks read
 * literally): the k_blocks-nb largest blk[R][C], C<R, one global top-k over the
 * flattened causal off-diagonal entries.  block_select 1 (the per-row reading of
 * the same step): row R keeps keep(R) = min(R+1, ceil(k_blocks (R+1) / (nb (nb+1)/2)))
 * blocks: its diagonal block and the keep(R)-1 largest blk[R][C], C<R (ties to
 * the lower C), i.e. every row block gets the same fraction of its causal blocks.
 * block_select 2: the global top-k again, on the row-normalised key blk[R][C] * (R+1).
 * diagonal_select 1 (diagonals at block granularity instead of element-exact):
 * an Interval-Slash head keeps, for every selected offset o and every query i >= o,
 * the whole block pair (i / b, (i - o) / b); the offsets are then part of the CSR
 * and the offs list is returned empty (n_offs = 0). */
int oracle_build_index(const float *v, const float *s, const float *blk, int Hq, int N, int b,
                       int w, int sink_blocks, int local_blocks, int k_vertical, int k_slash,
                       int k_blocks, int probe_v, int probe_s, int lift_num, int lift_den,
                       const int32_t *override, int cap_b, int32_t *pattern, int32_t *n_cols,
                       int32_t *cols, int32_t *n_offs, int32_t *offs, int32_t *rowptr,
                       int32_t *blkcols, int block_select, int diagonal_select) {
  if (N % b) return 1;
  if (block_select < 0 || block_select > 2) return 1;
  if (diagonal_select != 0 && diagonal_select != 1) return 1;
  const int nb = N / b;
  int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int h = 0; h < Hq; ++h) {
    const float *vh = v + (size_t)h * N, *sh = s + (size_t)h * N;
    const float *bh = blk + (size_t)h * nb * nb;
    int32_t *ch = cols + (size_t)h * k_vertical, *oh = offs + (size_t)h * k_slash;
    int32_t *rp = rowptr + (size_t)h * (nb + 1), *bc = blkcols + (size_t)h * cap_b;
    int pat = (override && override[h] >= 0)
                  ? override[h]
                  : choose_pattern(vh, sh, N, b, w, sink_blocks, local_blocks, probe_v, probe_s,
                                   lift_num, lift_den);
    pattern[h] = pat;
    for (int t = 0; t < k_vertical; ++t) ch[t] = -1;
    for (int t = 0; t < k_slash; ++t) oh[t] = -1;
    for (int t = 0; t < cap_b; ++t) bc[t] = -1;
    n_cols[h] = 0;
    n_offs[h] = 0;
    if (pat == PAT_INTERVAL_SLASH) {
      n_cols[h] = topk_full_sort(vh, NULL, N, k_vertical, ch, 0, NULL);
      n_offs[h] = topk_full_sort(sh, NULL, N, k_slash, oh, 0, NULL);
    }
    /* block CSR */
    unsigned char *keep = (unsigned char *)calloc((size_t)nb * nb, 1);
    for (int R = 0; R < nb; ++R) keep[(size_t)R * nb + R] = 1;
    if (pat == PAT_INTERVAL_SLASH && diagonal_select == 1) {
      for (int t = 0; t < n_offs[h]; ++t)
        for (int i = oh[t]; i < N; ++i) keep[(size_t)(i / b) * nb + (i - oh[t]) / b] = 1;
      for (int t = 0; t < k_slash; ++t) oh[t] = -1;
      n_offs[h] = 0;
    }
    if (pat == PAT_TRIANGULAR) {
      for (int R = 0; R < nb; ++R)
        for (int C = 0; C <= R; ++C)
          if (C < sink_blocks || R - C < local_blocks) keep[(size_t)R * nb + C] = 1;
    } else if (pat == PAT_BLOCK_CLUSTER && block_select == 1) {
      const int64_t all = (int64_t)nb * (nb + 1) / 2;
      int32_t *sel = (int32_t *)malloc(sizeof(int32_t) * (size_t)nb);
      for (int R = 1; R < nb; ++R) {
        int64_t keep_r = ((int64_t)k_blocks * (R + 1) + all - 1) / all;
        if (keep_r > R + 1) keep_r = R + 1;
        const int k = topk_full_sort(bh + (size_t)R * nb, NULL, R, (int)keep_r - 1, sel, 0, NULL);
        for (int u = 0; u < k; ++u) keep[(size_t)R * nb + sel[u]] = 1;
      }
      free(sel);
    } else if (pat == PAT_BLOCK_CLUSTER) {
      const int ncand = nb * (nb - 1) / 2;
      float *sc = (float *)malloc(sizeof(float) * (size_t)(ncand > 0 ? ncand : 1));
      int32_t *ix = (int32_t *)malloc(sizeof(int32_t) * (size_t)(ncand > 0 ? ncand : 1));
      int t = 0;
      for (int R = 0; R < nb; ++R)
        for (int C = 0; C < R; ++C) {
          /* block_select 2: the key is the entry times the length R+1 of its softmax row (one
           * fp32 multiplication), so that short early rows do not outrank long ones by construction */
          sc[t] = block_select == 2 ? bh[(size_t)R * nb + C] * (float)(R + 1) : bh[(size_t)R * nb + C];
          ix[t] = R * nb + C;
          ++t;
        }
      int k = k_blocks - nb;
      if (k < 0) k = 0;
      int32_t *sel = (int32_t *)malloc(sizeof(int32_t) * (size_t)(k > 0 ? k : 1));
      k = topk_full_sort(sc, ix, ncand, k, sel, 0, NULL);
      for (int u = 0; u < k; ++u) keep[sel[u]] = 1;
      free(sc); free(ix); free(sel);
    } else if (pat != PAT_INTERVAL_SLASH) {
      err = 1;
    }
    int n = 0;
    for (int R = 0; R < nb; ++R) {
      rp[R] = n;
      for (int C = 0; C <= R; ++C)
        if (keep[(size_t)R * nb + C]) {
          if (n < cap_b) bc[n] = C; else err = 1;
          ++n;
        }
    }
    rp[nb] = n;
    free(keep);
  }
  return err;
}

/* Exposed for the pattern-rule pin. */
int oracle_choose_pattern(const float *v, const float *s, int N, int b, int w, int sink_blocks,
                          int local_blocks, int probe_v, int probe_s, int lift_num, int lift_den) {
  return choose_pattern(v, s, N, b, w, sink_blocks, local_blocks, probe_v, probe_s, lift_num,
                        lift_den);
}

/* ------------------------------------------------------- masked attention */

/* O[h][r][:] over the keys j <= i (i = rows[r]) with
 *   (blk(i), blk(j)) in CSR_h  or  j in cols_h  or  (i - j) in offs_h,
 * each kept key counted once.  wsum = sum of normalised weights (1 for every
 * row, since the diagonal block is always kept); kept = number of kept keys. */
int oracle_masked_rows(const uint16_t *Q, const uint16_t *K, const uint16_t *V, int Hq, int Hkv,
                       int N, int d, int b, double scale, int k_vertical, int k_slash, int cap_b,
                       const int32_t *n_cols, const int32_t *cols, const int32_t *n_offs,
                       const int32_t *offs, const int32_t *rowptr, const int32_t *blkcols,
                       const int32_t *rows, int nrows, double *O, double *wsum, int64_t *kept) {
  if (Hq % Hkv || N % b) return 1;
  const int g = Hq / Hkv;
  const int nb = N / b;
  int err = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 4)
  for (int h = 0; h < Hq; ++h) {
    for (int r = 0; r < nrows; ++r) {
      const int i = rows ? rows[r] : r;
      if (i < 0 || i >= N) { err = 1; continue; }
      const uint16_t *q = Q + ((size_t)h * N + i) * d;
      const uint16_t *Kh = K + (size_t)(h / g) * N * d;
      const uint16_t *Vh = V + (size_t)(h / g) * N * d;
      unsigned char *mask = (unsigned char *)calloc((size_t)(i + 1), 1);
      const int R = i / b;
      const int32_t *rp = rowptr + (size_t)h * (nb + 1);
      for (int t = rp[R]; t < rp[R + 1]; ++t) {
        const int C = blkcols[(size_t)h * cap_b + t];
        for (int j = C * b; j < (C + 1) * b && j <= i; ++j) mask[j] = 1;
      }
      for (int t = 0; t < n_cols[h]; ++t) {
        const int j = cols[(size_t)h * k_vertical + t];
        if (j >= 0 && j <= i) mask[j] = 1;
      }
      for (int t = 0; t < n_offs[h]; ++t) {
        const int o = offs[(size_t)h * k_slash + t];
        if (o >= 0 && i - o >= 0) mask[i - o] = 1;
      }
      double *p = (double *)malloc(sizeof(double) * (size_t)(i + 1));
      double m = -INFINITY;
      int64_t cnt = 0;
      for (int j = 0; j <= i; ++j)
        if (mask[j]) {
          p[j] = scale * dot_bf16(q, Kh + (size_t)j * d, d);
          if (p[j] > m) m = p[j];
          ++cnt;
        }
      double Z = 0.0;
      for (int j = 0; j <= i; ++j)
        if (mask[j]) { p[j] = exp(p[j] - m); Z += p[j]; }
      double *o = O + ((size_t)h * nrows + r) * d;
      for (int t = 0; t < d; ++t) o[t] = 0.0;
      double ws = 0.0;
      for (int j = 0; j <= i; ++j)
        if (mask[j]) {
          const double wgt = p[j] / Z;
          ws += wgt;
          const uint16_t *vr = Vh + (size_t)j * d;
          for (int t = 0; t < d; ++t) o[t] += wgt * bf16_to_f64(vr[t]);
        }
      if (wsum) wsum[(size_t)h * nrows + r] = ws;
      if (kept) kept[(size_t)h * nrows + r] = cnt;
      free(p);
      free(mask);
    }
  }
  return err;
}

/* Number of kept (query,key) pairs of one head: |M_h|, exact, by rows. */
int64_t oracle_mask_count(int N, int b, int h, int k_vertical, int k_slash, int cap_b,
                          const int32_t *n_cols, const int32_t *cols, const int32_t *n_offs,
                          const int32_t *offs, const int32_t *rowptr, const int32_t *blkcols) {
  const int nb = N / b;
  int64_t total = 0;
  unsigned char *colset = (unsigned char *)calloc((size_t)N, 1);
  unsigned char *offset = (unsigned char *)calloc((size_t)N, 1);
  for (int t = 0; t < n_cols[h]; ++t) colset[cols[(size_t)h * k_vertical + t]] = 1;
  for (int t = 0; t < n_offs[h]; ++t) offset[offs[(size_t)h * k_slash + t]] = 1;
  unsigned char *bset = (unsigned char *)malloc((size_t)nb);
  const int32_t *rp = rowptr + (size_t)h * (nb + 1);
  for (int R = 0; R < nb; ++R) {
    memset(bset, 0, (size_t)nb);
    for (int t = rp[R]; t < rp[R + 1]; ++t) bset[blkcols[(size_t)h * cap_b + t]] = 1;
    for (int i = R * b; i < (R + 1) * b; ++i)
      for (int j = 0; j <= i; ++j)
        if (bset[j / b] || colset[j] || offset[i - j]) ++total;
  }
  free(colset); free(offset); free(bset);
  return total;
}
