/*
 * sts_oracle.c -- CPU oracle for the STS hot path. TEST INFRASTRUCTURE ONLY.
 * See sts_oracle.h for the contract of every function and the list of pins.
 * Plain loops, fp64 accumulation, OpenMP over independent (batch, head) pairs only.
 */
#include "sts_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* bf16 is the upper half of an IEEE fp32 word: widening is exact. */
static inline float bf16_to_float(uint16_t h) {
  uint32_t w = (uint32_t)h << 16;
  float f;
  memcpy(&f, &w, sizeof f);
  return f;
}

/* ---------------------------------------------------------------- aggregation */

int oracle_aggregate(const float *scores, const float *lse, int B, int Hd, int Tq, int N,
                     int kind, int reduce, float *A) {
  if (!scores || !A || B < 0 || Hd < 0 || Tq < 1 || N < 0) return -1;
  if (kind == ORACLE_SCORES_LOGITS_LSE && !lse) return -1;
  if (kind != ORACLE_SCORES_PROBS && kind != ORACLE_SCORES_LOGITS_LSE) return -1;
  if (reduce != ORACLE_REDUCE_SUM && reduce != ORACLE_REDUCE_MAX) return -1;
  const long rows = (long)B * Hd;
#pragma omp parallel for schedule(static)
  for (long r = 0; r < rows; ++r) {
    const float *P = scores + (size_t)r * Tq * N;
    float *out = A + (size_t)r * N;
    for (int n = 0; n < N; ++n) {
      float acc = 0.0f;
      for (int i = 0; i < Tq; ++i) {
        float p = P[(size_t)i * N + n];
        if (kind == ORACLE_SCORES_LOGITS_LSE) p = expf(p - lse[(size_t)r * Tq + i]);
        if (i == 0) {
          acc = p;
        } else if (reduce == ORACLE_REDUCE_SUM) {
          /* volatile keeps the single-rounding fp32 add from being widened or fused */
          volatile float s = acc + p;
          acc = s;
        } else {
          acc = (p > acc) ? p : acc;
        }
      }
      out[n] = acc;
    }
  }
  return 0;
}

/* ------------------------------------------------------------------ selection */

typedef struct {
  float a;
  int32_t n;
} scored_t;

/* (A descending, n ascending): a strict total order on distinct n, so qsort's lack of
 * stability cannot matter. +0 and -0 compare equal under the C comparison operators. */
static int by_score_then_index(const void *x, const void *y) {
  const scored_t *p = (const scored_t *)x, *q = (const scored_t *)y;
  if (p->a > q->a) return -1;
  if (p->a < q->a) return 1;
  return (p->n > q->n) - (p->n < q->n);
}

static int by_int(const void *x, const void *y) {
  const int32_t a = *(const int32_t *)x, b = *(const int32_t *)y;
  return (a > b) - (a < b);
}

/* top-c of one score row; writes c ascending indices; returns -2 on NaN */
static int topk_row(const float *a, int nb, int c, int32_t *out, scored_t *tmp) {
  for (int n = 0; n < nb; ++n) {
    if (isnan(a[n])) return -2;
    tmp[n].a = a[n];
    tmp[n].n = n;
  }
  qsort(tmp, (size_t)nb, sizeof(scored_t), by_score_then_index);
  for (int i = 0; i < c; ++i) out[i] = tmp[i].n;
  qsort(out, (size_t)c, sizeof(int32_t), by_int);
  return 0;
}

int oracle_select(const float *A, int B, int Hd, int N, const int32_t *seq_lens, int k,
                  int32_t *sel, int32_t *cnt) {
  if (!A || !sel || !cnt || B < 0 || Hd < 0 || N < 0 || k < 1) return -1;
  if (seq_lens)
    for (int b = 0; b < B; ++b)
      if (seq_lens[b] < 0 || seq_lens[b] > N) return -1;
  int status = 0;
  const long rows = (long)B * Hd;
#pragma omp parallel for schedule(dynamic, 1)
  for (long r = 0; r < rows; ++r) {
    const int b = (int)(r / Hd);
    const int nb = seq_lens ? seq_lens[b] : N;
    const int c = k < nb ? k : nb;
    int32_t *out = sel + (size_t)r * k;
    for (int i = 0; i < k; ++i) out[i] = -1;
    cnt[r] = c;
    if (c == 0) continue;
    scored_t *tmp = (scored_t *)malloc((size_t)nb * sizeof(scored_t));
    int rc = tmp ? topk_row(A + (size_t)r * N, nb, c, out, tmp) : -4;
    free(tmp);
    if (rc != 0) {
#pragma omp critical
      status = rc;
    }
  }
  return status;
}

int oracle_block_scores(const float *A, int B, int Hd, int N, const int32_t *seq_lens, int page,
                        float *blk) {
  if (!A || !blk || B < 0 || Hd < 0 || N < 0 || page < 1) return -1;
  const int NB = (N + page - 1) / page;
  for (int b = 0; b < B; ++b) {
    const int nb = seq_lens ? seq_lens[b] : N;
    if (nb < 0 || nb > N) return -1;
    for (int j = 0; j < Hd; ++j) {
      const float *a = A + ((size_t)b * Hd + j) * N;
      float *o = blk + ((size_t)b * Hd + j) * NB;
      for (int m = 0; m < NB; ++m) {
        float acc = 0.0f;
        int first = 1;
        for (int n = m * page; n < (m + 1) * page && n < nb; ++n) {
          if (first) {
            acc = a[n];
            first = 0;
          } else {
            volatile float s = acc + a[n];   /* one fp32 rounding per add */
            acc = s;
          }
        }
        o[m] = acc;
      }
    }
  }
  return 0;
}

int oracle_remap(const int32_t *sel, const int32_t *cnt, int B, int Hd, int Hq, int k,
                 const int32_t *head_map, int32_t *indices, int32_t *counts) {
  if (!sel || !cnt || !head_map || !indices || B < 0 || Hd < 1 || Hq < 0 || k < 1) return -1;
  for (int t = 0; t < Hq; ++t)
    if (head_map[t] < 0 || head_map[t] >= Hd) return -1;
  for (int b = 0; b < B; ++b)
    for (int t = 0; t < Hq; ++t) {
      const int j = head_map[t];
      memcpy(indices + ((size_t)b * Hq + t) * k, sel + ((size_t)b * Hd + j) * k,
             (size_t)k * sizeof(int32_t));
      if (counts) counts[(size_t)b * Hq + t] = cnt[(size_t)b * Hd + j];
    }
  return 0;
}

/* ------------------------------------------------------------------ attention */

int oracle_attn(const uint16_t *q, const uint16_t *k, const uint16_t *v, int B, int Tq, int Hq,
                int Hkv, int d, int N, int64_t stride_b, int64_t stride_h, int64_t stride_n,
                const int32_t *indices, const int32_t *counts, int kmax,
                const int32_t *seq_lens, float scale, float *out, float *lse_out,
                float *logits_out, int batch_begin, int batch_end, int head_begin,
                int head_end, const uint16_t *k_new, const uint16_t *v_new, int causal) {
  if (!q || !out) return -1;
  if (N > 0 && (!k || !v)) return -1;
  if ((k_new == NULL) != (v_new == NULL)) return -1;
  if (B < 0 || Tq < 1 || Hq < 1 || Hkv < 1 || d < 1 || N < 0 || Hq % Hkv != 0) return -1;
  if (indices && kmax < 0) return -1;
  if (indices && logits_out) return -1;
  if (batch_begin < 0 || batch_end > B || head_begin < 0 || head_end > Hq) return -1;
  const int G = Hq / Hkv;
  const int nbatch = batch_end - batch_begin, nhead = head_end - head_begin;
  if (nbatch <= 0 || nhead <= 0) return 0;
  int status = 0;
  const long units = (long)nbatch * nhead;
#pragma omp parallel for schedule(dynamic, 1)
  for (long u = 0; u < units; ++u) {
    const int b = batch_begin + (int)(u / nhead);
    const int t = head_begin + (int)(u % nhead);
    const int g = t / G;
    int c;
    const int32_t *idx = NULL;
    if (indices) {
      idx = indices + ((size_t)b * Hq + t) * kmax;
      c = counts ? counts[(size_t)b * Hq + t] : kmax;
      if (c < 0 || c > kmax) {
#pragma omp critical
        status = -3;
        continue;
      }
    } else {
      c = seq_lens ? seq_lens[b] : N;
      if (c < 0 || c > N) {
#pragma omp critical
        status = -3;
        continue;
      }
    }
    int bad = 0;
    for (int j = 0; j < c && idx; ++j)
      if (idx[j] < 0 || idx[j] >= N) bad = 1;
    if (bad) {
#pragma omp critical
      status = -3;
      continue;
    }
    const uint16_t *Kg = k + (size_t)b * stride_b + (size_t)g * stride_h;
    const uint16_t *Vg = v + (size_t)b * stride_b + (size_t)g * stride_h;
    double *s = (double *)malloc(((size_t)c + (size_t)Tq + 1) * sizeof(double));
    double *acc = (double *)malloc((size_t)d * sizeof(double));
    if (!s || !acc) {
      free(s);
      free(acc);
#pragma omp critical
      status = -4;
      continue;
    }
    for (int i = 0; i < Tq; ++i) {
      const uint16_t *qr = q + (((size_t)b * Tq + i) * Hq + t) * d;
      float *o = out + (((size_t)b * Tq + i) * Hq + t) * d;
      double m = -INFINITY;
      for (int j = 0; j < c; ++j) {
        const size_t row = idx ? (size_t)idx[j] : (size_t)j;
        const uint16_t *kr = Kg + row * stride_n;
        double dot = 0.0;
        for (int e = 0; e < d; ++e) dot += (double)bf16_to_float(qr[e]) * (double)bf16_to_float(kr[e]);
        s[j] = (double)scale * dot;
        if (s[j] > m) m = s[j];
        if (logits_out) logits_out[(((size_t)b * Hq + t) * Tq + i) * N + j] = (float)s[j];
      }
      /* the block's own tokens, appended after the cached keys */
      const int nnew = k_new ? (causal ? i + 1 : Tq) : 0;
      for (int j = 0; j < nnew; ++j) {
        const uint16_t *kr = k_new + (((size_t)b * Tq + j) * Hkv + g) * d;
        double dot = 0.0;
        for (int e = 0; e < d; ++e) dot += (double)bf16_to_float(qr[e]) * (double)bf16_to_float(kr[e]);
        s[c + j] = (double)scale * dot;
        if (s[c + j] > m) m = s[c + j];
      }
      for (int e = 0; e < d; ++e) acc[e] = 0.0;
      double l = 0.0;
      for (int j = 0; j < c + nnew; ++j) {
        const uint16_t *vr;
        if (j < c) {
          const size_t row = idx ? (size_t)idx[j] : (size_t)j;
          vr = Vg + row * stride_n;
        } else {
          vr = v_new + (((size_t)b * Tq + (j - c)) * Hkv + g) * d;
        }
        const double p = exp(s[j] - m);
        l += p;
        for (int e = 0; e < d; ++e) acc[e] += p * (double)bf16_to_float(vr[e]);
      }
      const int total = c + nnew;
      for (int e = 0; e < d; ++e) o[e] = (total > 0) ? (float)(acc[e] / l) : 0.0f;
      if (lse_out) lse_out[((size_t)b * Hq + t) * Tq + i] = (total > 0) ? (float)(m + log(l)) : -INFINITY;
    }
    free(s);
    free(acc);
  }
  return status;
}

/* ------------------------------------------------- Algorithm 1: head mapping */

/* Tokens that the top-k sets of target head ht and draft head hd have in common, summed over
 * every query row of every sample (membership bitmaps, one byte per token). */
static int64_t shared_topk_total(const unsigned char *mt, const unsigned char *md, int S, int Ht, int Hd, int R,
                                 int N, int ht, int hd) {
  int64_t shared = 0;
  for (int s = 0; s < S; ++s)
    for (int r = 0; r < R; ++r) {
      const unsigned char *in_t = mt + (((size_t)s * Ht + ht) * R + r) * (size_t)N;
      const unsigned char *in_d = md + (((size_t)s * Hd + hd) * R + r) * (size_t)N;
      for (int n = 0; n < N; ++n) shared += (in_t[n] & in_d[n]);
    }
  return shared;
}

/* Position of the largest entry; among equal entries the first one (so an all-zero row gives 0:
 * a target head that shares nothing with any draft head maps to draft head 0). */
static int32_t first_largest(const int64_t *row, int n) {
  int32_t where = 0;
  for (int i = 1; i < n; ++i)
    if (row[i] > row[where]) where = i;
  return where;
}

int oracle_head_mapping(const float *a_d, const float *a_t, int S, int Hd, int Ht, int R,
                        int N, int k, int32_t *map, int64_t *overlap) {
  if (!a_d || !a_t || !map || S < 1 || Hd < 1 || Ht < 1 || R < 1 || N < 1 || k < 1) return -1;
  const int c = k < N ? k : N;
  /* top-k membership bitmaps for every (sample, head, row) of both models */
  const size_t nd = (size_t)S * Hd * R, nt = (size_t)S * Ht * R;
  unsigned char *md = (unsigned char *)calloc(nd * (size_t)N, 1);
  unsigned char *mt = (unsigned char *)calloc(nt * (size_t)N, 1);
  int64_t *ov = (int64_t *)calloc((size_t)Ht * Hd, sizeof(int64_t));
  if (!md || !mt || !ov) {
    free(md);
    free(mt);
    free(ov);
    return -4;
  }
  int status = 0;
#pragma omp parallel
  {
    scored_t *tmp = (scored_t *)malloc((size_t)N * sizeof(scored_t));
    int32_t *top = (int32_t *)malloc((size_t)c * sizeof(int32_t));
#pragma omp for schedule(static)
    for (long r = 0; r < (long)(nd + nt); ++r) {
      const int is_t = (size_t)r >= nd;
      const size_t row = is_t ? (size_t)r - nd : (size_t)r;
      const float *a = (is_t ? a_t : a_d) + row * (size_t)N;
      unsigned char *mask = (is_t ? mt : md) + row * (size_t)N;
      int rc = (tmp && top) ? topk_row(a, N, c, top, tmp) : -4;
      if (rc != 0) {
#pragma omp critical
        status = rc;
        continue;
      }
      for (int i = 0; i < c; ++i) mask[top[i]] = 1;
    }
    free(tmp);
    free(top);
  }
  if (status == 0) {
    /* the whole matrix of summed intersection sizes first, then one arg-max per target head */
    for (int ht = 0; ht < Ht; ++ht)
      for (int hd = 0; hd < Hd; ++hd) ov[(size_t)ht * Hd + hd] = shared_topk_total(mt, md, S, Ht, Hd, R, N, ht, hd);
    for (int ht = 0; ht < Ht; ++ht) map[ht] = first_largest(ov + (size_t)ht * Hd, Hd);
    if (overlap) memcpy(overlap, ov, (size_t)Ht * Hd * sizeof(int64_t));
  }
  free(md);
  free(mt);
  free(ov);
  return status;
}
