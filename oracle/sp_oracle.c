/*
 * CPU oracle for the SharePrefill prefill hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct C: fp32 inputs (bf16 values widened exactly),
 * fp64 arithmetic inside, fp32 / int32 results.  Nothing here is blocked, fused
 * or reordered beyond what the definitions state; the only parallelism is an
 * OpenMP loop over independent query rows.  This file shares no code, header,
 * table or helper with the HIP path and is never loaded by the product path.
 *
 * What is computed (per attention head; Q, K, V are [N][d] row-major float):
 *
 *   logits      x[t][s] = scale * sum_e Q[t][e] K[s][e],  only s <= t exists
 *               (Sec. 5.1, the argument of the softmax in A(Q,K,V); causal
 *               because this is decoder prefill).
 *   dense       P[t][s] = exp(x[t][s] - max_s x[t][.]) / sum_s exp(.),
 *               O[t] = sum_s P[t][s] V[s]              (Sec. 5.1, A(Q,K,V)).
 *   scores      S[i][j] = (1/B) sum_{t in block i} sum_{s in block j, s<=t} P[t][s]
 *               for j <= i, else 0: the exact attention mass of each
 *               (query-block, key-block) pair, every row of S sums to 1.
 *               (Alg. 1 line 8 returns a block-level score map next to O; the
 *               per-block *mass* reading is the one this build is specified on.)
 *   mask rows   Alg. 2 (argsort, minimal prefix whose cumulative score reaches
 *               gamma) applied per query-block row in exact fixed point, then
 *               the sink block 0 and the diagonal block i are added.
 *   masked      Sec. 5.1, A(Q,K,V,M): softmax restricted to the key blocks with
 *               M = 1 (excluded entries get weight exactly 0), renormalised.
 *
 * All functions take a list of query-block rows so that long sequences can be
 * checked on a sample of rows: row i only needs Q block i and K/V[0 .. (i+1)B).
 *
 * The second half of the file holds the pattern construction exactly as the
 * paper prints it (block-mean logits, row softmax, one selection over the
 * flattened map); see the comment there.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int spo_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* scaled logits of query t against keys [0, t] into x[0..t]; returns the max */
static double logits_row(const float *q, const float *k, int t, int d, double scale, double *x) {
  double mx = -INFINITY;
  const float *qt = q + (size_t)t * d;
  for (int s = 0; s <= t; ++s) {
    const float *ks = k + (size_t)s * d;
    double acc = 0.0;
#pragma omp simd reduction(+ : acc)
    for (int e = 0; e < d; ++e) acc += (double)qt[e] * (double)ks[e];
    x[s] = acc * scale;
    if (x[s] > mx) mx = x[s];
  }
  return mx;
}

/*
 * Dense causal attention for the query blocks listed in rows[0..nrows).
 *   o      [nrows][B][d]   attention output of those query blocks (may be NULL)
 *   scores [nrows][nkb]    block-mass map rows (may be NULL), nkb = N / B
 *   lse    [nrows][B]      natural-log sum-exp of each query row (may be NULL)
 */
int spo_dense_rows(const float *q, const float *k, const float *v, int N, int d, int B, double scale,
                   const int *rows, int nrows, float *o, float *scores, float *lse) {
  if (N <= 0 || d <= 0 || B <= 0 || N % B) return 1;
  const int nkb = N / B;
  for (int r = 0; r < nrows; ++r)
    if (rows[r] < 0 || rows[r] >= nkb) return 1;
  int fail = 0;
#pragma omp parallel
  {
    double *x = (double *)malloc(sizeof(double) * (size_t)N);
    double *acc = (double *)malloc(sizeof(double) * (size_t)d);
    double *mass = (double *)malloc(sizeof(double) * (size_t)nkb);
    if (!x || !acc || !mass) {
#pragma omp atomic write
      fail = 1;
    } else {
#pragma omp for schedule(dynamic, 1)
      for (int r = 0; r < nrows; ++r) {
        const int i = rows[r];
        for (int j = 0; j < nkb; ++j) mass[j] = 0.0;
        for (int tt = 0; tt < B; ++tt) {
          const int t = i * B + tt;
          const double mx = logits_row(q, k, t, d, scale, x);
          double den = 0.0;
          for (int s = 0; s <= t; ++s) {
            x[s] = exp(x[s] - mx);
            den += x[s];
          }
          for (int e = 0; e < d; ++e) acc[e] = 0.0;
          for (int s = 0; s <= t; ++s) {
            const double p = x[s] / den;
            mass[s / B] += p;
            const float *vs = v + (size_t)s * d;
            for (int e = 0; e < d; ++e) acc[e] += p * (double)vs[e];
          }
          if (o)
            for (int e = 0; e < d; ++e) o[((size_t)r * B + tt) * d + e] = (float)acc[e];
          if (lse) lse[(size_t)r * B + tt] = (float)(mx + log(den));
        }
        if (scores)
          for (int j = 0; j < nkb; ++j) scores[(size_t)r * nkb + j] = (j <= i) ? (float)(mass[j] / B) : 0.0f;
      }
    }
    free(x);
    free(acc);
    free(mass);
  }
  return fail ? 2 : 0;
}

/* ---- Alg. 2, per query-block row, in exact fixed point ------------------- */

typedef struct {
  uint32_t u;
  int32_t j;
} spo_key;

static int key_cmp(const void *a, const void *b) {
  const spo_key *x = (const spo_key *)a, *y = (const spo_key *)b;
  if (x->u != y->u) return (x->u > y->u) ? -1 : 1; /* score descending */
  return (x->j < y->j) ? -1 : (x->j > y->j);       /* ties: lower key block first */
}

static int int_cmp(const void *a, const void *b) {
  const int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
  return (x < y) ? -1 : (x > y);
}

/* quantise a block score to 24 fractional bits: rint(clamp(s,0,1) * 2^24), NaN -> 0 */
static uint32_t quantise(float s) {
  if (!(s > 0.0f)) return 0u; /* also catches NaN */
  if (s > 1.0f) s = 1.0f;
  return (uint32_t)rintf(s * 16777216.0f);
}

/*
 * scores  [nrows][nkb] block-score rows; row r describes query block row_ids[r]
 * kb_idx  [nrows][nkb] selected key blocks, ascending, tail filled with -1
 * kb_cnt  [nrows]
 * k_star  [nrows] (may be NULL): size of the thresholded set before the forced
 *         sink / diagonal blocks are added (for tests of minimality).
 */
int spo_build_mask_rows(const float *scores, const int *row_ids, int nrows, int nkb, float gamma,
                        int32_t *kb_idx, int32_t *kb_cnt, int32_t *k_star) {
  if (nkb <= 0 || nkb > 32768 || !(gamma > 0.0f) || gamma > 1.0f) return 1;
  const uint64_t gq = (uint64_t)rintf(gamma * 16777216.0f);
  spo_key *keys = (spo_key *)malloc(sizeof(spo_key) * (size_t)nkb);
  int32_t *sel = (int32_t *)malloc(sizeof(int32_t) * ((size_t)nkb + 2));
  if (!keys || !sel) {
    free(keys);
    free(sel);
    return 2;
  }
  for (int r = 0; r < nrows; ++r) {
    const int i = row_ids[r];
    if (i < 0 || i >= nkb) {
      free(keys);
      free(sel);
      return 1;
    }
    const float *row = scores + (size_t)r * nkb;
    uint64_t tot = 0;
    for (int j = 0; j <= i; ++j) {
      keys[j].u = quantise(row[j]);
      keys[j].j = j;
      tot += keys[j].u;
    }
    qsort(keys, (size_t)i + 1, sizeof(spo_key), key_cmp);
    int kstar = 0;
    if (tot > 0) {
      uint64_t cum = 0;
      for (int kk = 0; kk <= i; ++kk) {
        cum += keys[kk].u;
        if ((cum << 24) >= gq * tot) { /* cum/tot >= gamma, exactly */
          kstar = kk + 1;
          break;
        }
      }
    }
    int n = 0, has0 = 0, hasi = 0;
    for (int kk = 0; kk < kstar; ++kk) {
      sel[n++] = keys[kk].j;
      if (keys[kk].j == 0) has0 = 1;
      if (keys[kk].j == i) hasi = 1;
    }
    if (!has0) {
      sel[n++] = 0;
      if (i == 0) hasi = 1;
    }
    if (!hasi) sel[n++] = i;
    qsort(sel, (size_t)n, sizeof(int32_t), int_cmp);
    int32_t *out = kb_idx + (size_t)r * nkb;
    for (int j = 0; j < nkb; ++j) out[j] = (j < n) ? sel[j] : -1;
    kb_cnt[r] = n;
    if (k_star) k_star[r] = kstar;
  }
  free(keys);
  free(sel);
  return 0;
}

/*
 * Masked (block-sparse) causal attention for the query blocks in rows[].
 *   kb_idx [nrows][nkb], kb_cnt [nrows]: key blocks with M = 1 for each listed row
 *   o      [nrows][B][d]
 * A listed key block beyond the diagonal contributes nothing (causal).  A query
 * with no admissible key yields a zero output row.
 */
int spo_masked_rows(const float *q, const float *k, const float *v, int N, int d, int B, double scale,
                    const int *rows, int nrows, const int32_t *kb_idx, const int32_t *kb_cnt, float *o) {
  if (N <= 0 || d <= 0 || B <= 0 || N % B) return 1;
  const int nkb = N / B;
  for (int r = 0; r < nrows; ++r) {
    if (rows[r] < 0 || rows[r] >= nkb || kb_cnt[r] < 0 || kb_cnt[r] > nkb) return 1;
    for (int c = 0; c < kb_cnt[r]; ++c) {
      const int j = kb_idx[(size_t)r * nkb + c];
      if (j < 0 || j >= nkb) return 1;
    }
  }
  int fail = 0;
#pragma omp parallel
  {
    double *x = (double *)malloc(sizeof(double) * (size_t)N);
    double *acc = (double *)malloc(sizeof(double) * (size_t)d);
    unsigned char *on = (unsigned char *)malloc((size_t)nkb);
    if (!x || !acc || !on) {
#pragma omp atomic write
      fail = 1;
    } else {
#pragma omp for schedule(dynamic, 1)
      for (int r = 0; r < nrows; ++r) {
        const int i = rows[r];
        memset(on, 0, (size_t)nkb);
        for (int c = 0; c < kb_cnt[r]; ++c) on[kb_idx[(size_t)r * nkb + c]] = 1;
        for (int tt = 0; tt < B; ++tt) {
          const int t = i * B + tt;
          const float *qt = q + (size_t)t * d;
          double mx = -INFINITY;
          for (int s = 0; s <= t; ++s) {
            if (!on[s / B]) continue;
            const float *ks = k + (size_t)s * d;
            double a = 0.0;
#pragma omp simd reduction(+ : a)
            for (int e = 0; e < d; ++e) a += (double)qt[e] * (double)ks[e];
            x[s] = a * scale;
            if (x[s] > mx) mx = x[s];
          }
          double den = 0.0;
          for (int s = 0; s <= t; ++s) {
            if (!on[s / B]) continue;
            x[s] = exp(x[s] - mx);
            den += x[s];
          }
          for (int e = 0; e < d; ++e) acc[e] = 0.0;
          if (den > 0.0) {
            for (int s = 0; s <= t; ++s) {
              if (!on[s / B]) continue;
              const double p = x[s] / den;
              const float *vs = v + (size_t)s * d;
              for (int e = 0; e < d; ++e) acc[e] += p * (double)vs[e];
            }
          }
          for (int e = 0; e < d; ++e) o[((size_t)r * B + tt) * d + e] = (float)acc[e];
        }
      }
    }
    free(x);
    free(acc);
    free(on);
  }
  return fail ? 2 : 0;
}

/* ==== paper-literal pattern construction (Sec. 5.2, Alg. 2 as printed) ======
 *
 *   mean logits  Abar[i][j] = average of the scaled logits x[t][s] over the
 *                entries of block (i, j) that exist (s <= t): B*B entries for
 *                j < i, B(B+1)/2 on the diagonal block, none for j > i, which
 *                gets -inf ("blocks not computed are assigned -inf").
 *                (Sec. 5.2 "Sparse Attention Computation": block-wise average
 *                of the QK values.)
 *   row softmax  Atil[i][.] = softmax(Abar[i][.])        (Alg. 2, first step)
 *   selection    the whole map is normalised by its total, flattened row-major,
 *                sorted descending, and the shortest prefix whose sum reaches
 *                gamma is kept (Alg. 2, remaining steps).  Ties: lower flat
 *                index first.  Evaluated in exact 24-bit fixed point like the
 *                per-row variant above.
 */

int spo_mean_logit_rows(const float *q, const float *k, int N, int d, int B, double scale, const int *rows,
                        int nrows, float *abar) {
  if (N <= 0 || d <= 0 || B <= 0 || N % B) return 1;
  const int nkb = N / B;
  for (int r = 0; r < nrows; ++r)
    if (rows[r] < 0 || rows[r] >= nkb) return 1;
  int fail = 0;
#pragma omp parallel
  {
    double *x = (double *)malloc(sizeof(double) * (size_t)N);
    double *sum = (double *)malloc(sizeof(double) * (size_t)nkb);
    long *num = (long *)malloc(sizeof(long) * (size_t)nkb);
    if (!x || !sum || !num) {
#pragma omp atomic write
      fail = 1;
    } else {
#pragma omp for schedule(dynamic, 1)
      for (int r = 0; r < nrows; ++r) {
        const int i = rows[r];
        for (int j = 0; j < nkb; ++j) {
          sum[j] = 0.0;
          num[j] = 0;
        }
        for (int tt = 0; tt < B; ++tt) {
          const int t = i * B + tt;
          logits_row(q, k, t, d, scale, x);
          for (int s = 0; s <= t; ++s) {
            sum[s / B] += x[s];
            num[s / B] += 1;
          }
        }
        for (int j = 0; j < nkb; ++j)
          abar[(size_t)r * nkb + j] = (num[j] > 0) ? (float)(sum[j] / (double)num[j]) : -INFINITY;
      }
    }
    free(x);
    free(sum);
    free(num);
  }
  return fail ? 2 : 0;
}

/* softmax of each row; -inf entries get exactly 0; a row of only -inf becomes all 0 */
int spo_softmax_rows(const float *a, int nrows, int n, float *out) {
  if (nrows < 0 || n <= 0) return 1;
  for (int r = 0; r < nrows; ++r) {
    const float *row = a + (size_t)r * n;
    double mx = -INFINITY;
    for (int j = 0; j < n; ++j)
      if ((double)row[j] > mx) mx = row[j];
    double den = 0.0;
    if (mx > -INFINITY)
      for (int j = 0; j < n; ++j) den += exp((double)row[j] - mx);
    for (int j = 0; j < n; ++j)
      out[(size_t)r * n + j] = (den > 0.0) ? (float)(exp((double)row[j] - mx) / den) : 0.0f;
  }
  return 0;
}

typedef struct {
  uint32_t u;
  int64_t f; /* flat index i * nkb + j */
} spo_gkey;

static int gkey_cmp(const void *a, const void *b) {
  const spo_gkey *x = (const spo_gkey *)a, *y = (const spo_gkey *)b;
  if (x->u != y->u) return (x->u > y->u) ? -1 : 1;
  return (x->f < y->f) ? -1 : (x->f > y->f);
}

/*
 * Alg. 2 on the whole map.  scores [nkb][nkb] (row i = query block i; entries
 * with j > i are ignored: they do not exist under causality).
 *   forced   nonzero: every row additionally receives the sink block 0 and its
 *            diagonal block (not in the paper; keeps every query row non-empty)
 *   kb_idx   [nkb][nkb] ascending, -1 tail;  kb_cnt [nkb]
 *   k_star   (may be NULL) the global K before forced blocks
 */
int spo_build_mask_global(const float *scores, int nkb, float gamma, int forced, int32_t *kb_idx,
                          int32_t *kb_cnt, int64_t *k_star) {
  if (nkb <= 0 || nkb > 32768 || !(gamma > 0.0f) || gamma > 1.0f) return 1;
  const uint64_t gq = (uint64_t)rintf(gamma * 16777216.0f);
  const size_t n = (size_t)nkb * ((size_t)nkb + 1) / 2;
  spo_gkey *keys = (spo_gkey *)malloc(sizeof(spo_gkey) * n);
  unsigned char *on = (unsigned char *)calloc((size_t)nkb * (size_t)nkb, 1);
  if (!keys || !on) {
    free(keys);
    free(on);
    return 2;
  }
  size_t m = 0;
  unsigned __int128 tot = 0;
  for (int i = 0; i < nkb; ++i)
    for (int j = 0; j <= i; ++j) {
      keys[m].u = quantise(scores[(size_t)i * nkb + j]);
      keys[m].f = (int64_t)i * nkb + j;
      tot += keys[m].u;
      ++m;
    }
  qsort(keys, n, sizeof(spo_gkey), gkey_cmp);
  int64_t K = 0;
  if (tot > 0) {
    unsigned __int128 cum = 0;
    for (size_t kk = 0; kk < n; ++kk) {
      cum += keys[kk].u;
      if ((cum << 24) >= (unsigned __int128)gq * tot) { /* cum / tot >= gamma, exactly */
        K = (int64_t)kk + 1;
        break;
      }
    }
  }
  for (int64_t kk = 0; kk < K; ++kk) on[keys[kk].f] = 1;
  for (int i = 0; i < nkb; ++i) {
    if (forced) {
      on[(size_t)i * nkb] = 1;
      on[(size_t)i * nkb + i] = 1;
    }
    int c = 0;
    for (int j = 0; j < nkb; ++j)
      if (j <= i && on[(size_t)i * nkb + j]) kb_idx[(size_t)i * nkb + c++] = j;
    kb_cnt[i] = c;
    for (; c < nkb; ++c) kb_idx[(size_t)i * nkb + c] = -1;
  }
  if (k_star) *k_star = K;
  free(keys);
  free(on);
  return 0;
}

/* ==== Determine Sparse Pattern (Alg. 3) =====================================
 *
 *   a_hat    the block-averaged attention estimate of the last query block:
 *            softmax over key blocks of the pooled, scaled logits of the last
 *            B queries -- i.e. row nkb-1 of the map spo_mean_logit_rows /
 *            spo_softmax_rows give (the caller composes those two).
 *   distance sqrt(JSD(p || q)), JSD(p||q) = KL(p||m)/2 + KL(q||m)/2 with
 *            m = (p+q)/2, natural logarithm, 0*log(0) = 0.
 *   decision shared_pivot iff d(a_hat, uniform) < delta and
 *            d(a_hat, a_tilde) < tau; otherwise the fallback pattern.
 */
int spo_js_distance(const float *p, const float *q, int n, double *out) {
  if (n <= 0 || !p || !q || !out) return 1;
  double a = 0.0, b = 0.0;
  for (int j = 0; j < n; ++j) {
    const double pj = p[j], qj = q[j];
    if (pj < 0.0 || qj < 0.0) return 1;
    const double m = 0.5 * (pj + qj);
    if (pj > 0.0) a += pj * log(pj / m);
    if (qj > 0.0) b += qj * log(qj / m);
  }
  const double jsd = 0.5 * a + 0.5 * b;
  *out = sqrt(jsd > 0.0 ? jsd : 0.0);
  return 0;
}

/* ==== Search Vertical Slash Pattern (Alg. 5) ================================
 *
 *   A_hat    = causal softmax of the scaled logits of the last n_hat queries
 *              (the representative subset Q_hat) against every key.
 *   a_v[s]   = sum over those queries of A_hat[t][s]          ("vertical" sums)
 *   a_s[o]   = sum over those queries of A_hat[t][t - o]      ("slash" sums, o = t - s >= 0)
 *              both divided by the total of A_hat (= n_hat: every row sums to 1).
 *   select   each vector is sorted descending (ties: lower index first) and the
 *              shortest prefix whose sum reaches gamma of the vector's total is kept,
 *              in the same exact 24-bit fixed point as the block selections above.
 *   pattern  token (t, s), s <= t, is attended iff key s is a kept vertical or
 *              offset t - s a kept slash.  A key block j of query block i is kept
 *              iff it contains at least one such (t, s); attention then runs over
 *              whole blocks (a superset of the token pattern).
 */
int spo_vertical_slash_sums(const float *q, const float *k, int N, int d, int n_hat, double scale, float *a_v,
                            float *a_s) {
  if (N <= 0 || d <= 0 || n_hat <= 0 || n_hat > N) return 1;
  double *av = (double *)calloc((size_t)N, sizeof(double));
  double *as = (double *)calloc((size_t)N, sizeof(double));
  double *x = (double *)malloc(sizeof(double) * (size_t)N);
  if (!av || !as || !x) {
    free(av);
    free(as);
    free(x);
    return 2;
  }
  for (int t = N - n_hat; t < N; ++t) {
    const double mx = logits_row(q, k, t, d, scale, x);
    double den = 0.0;
    for (int s = 0; s <= t; ++s) {
      x[s] = exp(x[s] - mx);
      den += x[s];
    }
    for (int s = 0; s <= t; ++s) {
      const double p = x[s] / den;
      av[s] += p;
      as[t - s] += p;
    }
  }
  for (int s = 0; s < N; ++s) {
    a_v[s] = (float)(av[s] / (double)n_hat);
    a_s[s] = (float)(as[s] / (double)n_hat);
  }
  free(av);
  free(as);
  free(x);
  return 0;
}

typedef struct {
  uint32_t u;
  int64_t f;
} spo_vkey;
static int vkey_cmp(const void *a, const void *b) {
  const spo_vkey *x = (const spo_vkey *)a, *y = (const spo_vkey *)b;
  if (x->u != y->u) return (x->u > y->u) ? -1 : 1;
  return (x->f < y->f) ? -1 : (x->f > y->f);
}

/* keep[j] = 1 for the shortest descending prefix of v[0..n) whose sum reaches gamma of the total */
int spo_select_cumulative(const float *v, int64_t n, float gamma, unsigned char *keep, int64_t *K_out) {
  if (n <= 0 || !(gamma > 0.0f) || gamma > 1.0f) return 1;
  const uint64_t gq = (uint64_t)rintf(gamma * 16777216.0f);
  spo_vkey *keys = (spo_vkey *)malloc(sizeof(spo_vkey) * (size_t)n);
  if (!keys) return 2;
  unsigned __int128 tot = 0;
  for (int64_t j = 0; j < n; ++j) {
    keys[j].u = quantise(v[j]);
    keys[j].f = j;
    tot += keys[j].u;
    keep[j] = 0;
  }
  qsort(keys, (size_t)n, sizeof(spo_vkey), vkey_cmp);
  int64_t K = 0;
  if (tot > 0) {
    unsigned __int128 cum = 0;
    for (int64_t kk = 0; kk < n; ++kk) {
      cum += keys[kk].u;
      if ((cum << 24) >= (unsigned __int128)gq * tot) {
        K = kk + 1;
        break;
      }
    }
  }
  for (int64_t kk = 0; kk < K; ++kk) keep[keys[kk].f] = 1;
  if (K_out) *K_out = K;
  free(keys);
  return 0;
}

/*
 * Block lists of a vertical-slash pattern.  keep_v / keep_s [N]: kept keys / kept offsets.
 * Block (i, j), j <= i, is kept iff some token pair (t, s) inside it with s <= t has
 * keep_v[s] or keep_s[t - s]: any kept key in block j, or any kept offset among the
 * offsets the block's pairs realise, max(0, (i-j)B - (B-1)) .. (i-j)B + (B-1).
 * forced != 0 adds the sink block 0 and the diagonal block i to every row.
 */
int spo_vs_block_lists(const unsigned char *keep_v, const unsigned char *keep_s, int N, int B, int forced,
                       int32_t *kb_idx, int32_t *kb_cnt) {
  if (N <= 0 || B <= 0 || N % B) return 1;
  const int nkb = N / B;
  for (int i = 0; i < nkb; ++i) {
    int c = 0;
    for (int j = 0; j <= i; ++j) {
      int on = forced && (j == 0 || j == i);
      for (int s = j * B; s < (j + 1) * B && !on; ++s) on = keep_v[s];
      const int lo = (i - j) * B - (B - 1) < 0 ? 0 : (i - j) * B - (B - 1);
      const int hi = (i - j) * B + (B - 1);
      for (int o = lo; o <= hi && o < N && !on; ++o) on = keep_s[o];
      if (on) kb_idx[(size_t)i * nkb + c++] = j;
    }
    kb_cnt[i] = c;
    for (; c < nkb; ++c) kb_idx[(size_t)i * nkb + c] = -1;
  }
  return 0;
}

/*
 * Attention over the vertical-slash pattern of Alg. 5 at token granularity (the mask M the algorithm builds from
 * S = S_v U S_s): query t attends to key s <= t iff key s is kept (a vertical line), or offset t - s is kept
 * (a slash line), or -- forced != 0 -- s lies in the first block or in t's own block (the sink and diagonal
 * blocks every pattern of this library carries).  Excluded pairs get weight exactly 0 and the softmax is
 * renormalised (Sec. 5.1); a query with no allowed key gets zeros.  rows: query-block rows to evaluate;
 * o: [nrows * B][d].
 */
int spo_vs_token_rows(const float *q, const float *k, const float *v, int N, int d, int B, double scale,
                      const int *rows, int nrows, const unsigned char *keep_v, const unsigned char *keep_s, int forced,
                      float *o) {
  if (N <= 0 || d <= 0 || B <= 0 || N % B) return 1;
  const int nkb = N / B;
  for (int r = 0; r < nrows; ++r)
    if (rows[r] < 0 || rows[r] >= nkb) return 1;
  int fail = 0;
#pragma omp parallel
  {
    double *x = (double *)malloc(sizeof(double) * (size_t)N);
    double *acc = (double *)malloc(sizeof(double) * (size_t)d);
    unsigned char *on = (unsigned char *)malloc((size_t)N);
    if (!x || !acc || !on) {
#pragma omp atomic write
      fail = 1;
    } else {
#pragma omp for schedule(dynamic, 1)
      for (int r = 0; r < nrows; ++r) {
        const int i = rows[r];
        for (int tt = 0; tt < B; ++tt) {
          const int t = i * B + tt;
          const float *qt = q + (size_t)t * d;
          double mx = -INFINITY;
          for (int s = 0; s <= t; ++s) {
            on[s] = keep_v[s] || keep_s[t - s] || (forced && (s / B == 0 || s / B == i));
            if (!on[s]) continue;
            const float *ks = k + (size_t)s * d;
            double a = 0.0;
#pragma omp simd reduction(+ : a)
            for (int e = 0; e < d; ++e) a += (double)qt[e] * (double)ks[e];
            x[s] = a * scale;
            if (x[s] > mx) mx = x[s];
          }
          double den = 0.0;
          for (int s = 0; s <= t; ++s) {
            if (!on[s]) continue;
            x[s] = exp(x[s] - mx);
            den += x[s];
          }
          for (int e = 0; e < d; ++e) acc[e] = 0.0;
          if (den > 0.0) {
            for (int s = 0; s <= t; ++s) {
              if (!on[s]) continue;
              const double p = x[s] / den;
              const float *vs = v + (size_t)s * d;
              for (int e = 0; e < d; ++e) acc[e] += p * (double)vs[e];
            }
          }
          float *ot = o + ((size_t)r * B + tt) * d;
          for (int e = 0; e < d; ++e) ot[e] = (float)acc[e];
        }
      }
    }
    free(x);
    free(acc);
    free(on);
  }
  return fail;
}
