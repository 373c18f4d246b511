/*
 * zeppelin_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain, slow, fp64 CPU statement of what the packed variable-length attention engine computes.
 * Only tests, the smoke check and the bench's cpu_baseline leg may call this; it shares no code
 * with the HIP library and the HIP library never calls it.
 *
 * What is computed (paper sections in brackets):
 *  - causal softmax attention per sequence of a packed batch [Sec. 2.1: lower-triangular mask;
 *    Sec. 3.2: local sequences run a standard variable-length attention, no token ever attends
 *    outside its own sequence -- cross-sequence attention is the waste Sec. 2.3 describes];
 *  - the same restricted to the keys of one KV chunk, for a Q chunk of the same sequence
 *    [Sec. 3.2: a ring of size G cuts a sequence into 2G equal-length chunks and each round
 *    computes the chunks in hand against the KV in hand];
 *  - the combination of such per-round partial results by their softmax statistics
 *    [Sec. 3.2, "standard ring attention pattern"; the paper does not print the formula, the
 *    log-sum-exp identity used here is the textbook one];
 *  - the backward of the whole-sequence attention [Sec. 5.4: backward reverses the forward];
 *  - the remapping layer's token move as a row gather / scatter [Sec. 3.4].
 *
 * Conventions (the paper is silent on all of them; these are the build's readings):
 *  scale multiplies q.k before the softmax; key j is visible to query i iff pos(j) <= pos(i);
 *  LSE is the natural-log log-sum-exp of the scaled scores; a row with no visible key has
 *  LSE = -inf and O = 0; Q head h reads KV head h / (Hq/Hkv).
 *
 * Layouts: q,o,dout,dq [T][Hq][d]; k,v,dk,dv [T][Hkv][d]; lse [Hq][T]; all contiguous doubles.
 * Every function returns 0, or -1 on an invalid argument.
 *
 * Parallelism: OpenMP over independent output rows/columns only. No blocking, no fusion.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double dotd(const double *a, const double *b, int d) {
  double s = 0.0;
  for (int c = 0; c < d; c++) s += a[c] * b[c];
  return s;
}

/* One softmax-attention row over the first n_vis keys of a key/value run.
 * qrow[d]; keys at kbase + j*kv_stride, values at vbase + j*kv_stride, j = 0..n_vis-1.
 * Writes o_row[d] (if non-null) and returns LSE (natural log). */
static double attn_row(const double *qrow, const double *kbase, const double *vbase, int64_t kv_stride,
                       int64_t n_vis, int d, double scale, double *o_row) {
  if (n_vis <= 0) {
    if (o_row) for (int c = 0; c < d; c++) o_row[c] = 0.0;
    return -INFINITY;
  }
  double *s = (double *)malloc(sizeof(double) * (size_t)n_vis);
  double m = -INFINITY;
  for (int64_t j = 0; j < n_vis; j++) {
    s[j] = scale * dotd(qrow, kbase + j * kv_stride, d);
    if (s[j] > m) m = s[j];
  }
  double l = 0.0;
  for (int64_t j = 0; j < n_vis; j++) l += exp(s[j] - m);
  double lse = m + log(l);
  if (o_row) {
    for (int c = 0; c < d; c++) o_row[c] = 0.0;
    for (int64_t j = 0; j < n_vis; j++) {
      double p = exp(s[j] - lse);
      const double *vj = vbase + j * kv_stride;
      for (int c = 0; c < d; c++) o_row[c] += p * vj[c];
    }
  }
  free(s);
  return lse;
}

static int check_cu(const int32_t *cu, int S, int64_t T) {
  if (!cu || S < 0 || cu[0] != 0) return -1;
  for (int s = 0; s < S; s++) if (cu[s + 1] < cu[s]) return -1;
  if (cu[S] != T) return -1;
  return 0;
}

static int seq_of_token(const int32_t *cu, int S, int64_t t) {
  for (int s = 0; s < S; s++) if (t >= cu[s] && t < cu[s + 1]) return s;
  return -1;
}

/* O = softmax(scale Q K^T + causal mask) V per sequence and head; LSE per row. */
int zo_varlen_attn_fwd(const double *q, const double *k, const double *v, int64_t T, int Hq, int Hkv, int d,
                       const int32_t *cu, int S, double scale, double *o, double *lse) {
  if (!q || !k || !v || !o || !lse || Hq <= 0 || Hkv <= 0 || d <= 0 || Hq % Hkv) return -1;
  if (check_cu(cu, S, T)) return -1;
  const int grp = Hq / Hkv;
  const int64_t kvs = (int64_t)Hkv * d;
#pragma omp parallel for collapse(2) schedule(dynamic, 16)
  for (int h = 0; h < Hq; h++) {
    for (int64_t t = 0; t < T; t++) {
      int s = seq_of_token(cu, S, t);
      int64_t t0 = cu[s], i = t - t0;
      int g = h / grp;
      lse[(int64_t)h * T + t] = attn_row(q + (t * Hq + h) * d, k + (t0 * Hkv + g) * d, v + (t0 * Hkv + g) * d, kvs,
                                         i + 1, d, scale, o + (t * Hq + h) * d);
    }
  }
  return 0;
}

/* A (Q chunk, KV chunk) pair of one sequence. Token offsets index the packed buffers; positions are
 * the offsets of the first query / first key inside their sequence; out_row0 is the pair's first row
 * in o_part / lse_part. */
typedef struct {
  int32_t q_tok0, q_len, k_tok0, k_len, q_pos0, k_pos0, out_row0;
} zo_pair;

/* Partial attention of each pair: softmax over only the pair's keys that are causally visible,
 * normalised by its own sum, with its own LSE. o_part [part_rows][Hq][d], lse_part [Hq][part_rows]. */
int zo_chunk_attn_partial(const double *q, const double *k, const double *v, int64_t T, int Hq, int Hkv, int d,
                          const zo_pair *pairs, int n_pairs, double scale, double *o_part, double *lse_part,
                          int64_t part_rows) {
  if (!q || !k || !v || !o_part || !lse_part || Hq <= 0 || Hkv <= 0 || d <= 0 || Hq % Hkv) return -1;
  const int grp = Hq / Hkv;
  const int64_t kvs = (int64_t)Hkv * d;
  for (int p = 0; p < n_pairs; p++) {
    const zo_pair *pr = &pairs[p];
    if (pr->q_len < 0 || pr->k_len < 0 || pr->q_tok0 < 0 || pr->k_tok0 < 0 || pr->q_tok0 + (int64_t)pr->q_len > T ||
        pr->k_tok0 + (int64_t)pr->k_len > T || pr->out_row0 < 0 || pr->out_row0 + (int64_t)pr->q_len > part_rows)
      return -1;
  }
  for (int p = 0; p < n_pairs; p++) {
    const zo_pair *pr = &pairs[p];
#pragma omp parallel for collapse(2) schedule(dynamic, 16)
    for (int h = 0; h < Hq; h++) {
      for (int ii = 0; ii < pr->q_len; ii++) {
        int g = h / grp;
        int64_t tq = pr->q_tok0 + ii;
        int64_t q_pos = (int64_t)pr->q_pos0 + ii;
        int64_t n_vis = q_pos - pr->k_pos0 + 1; /* keys with position <= q_pos */
        if (n_vis > pr->k_len) n_vis = pr->k_len;
        int64_t row = pr->out_row0 + ii;
        lse_part[(int64_t)h * part_rows + row] =
            attn_row(q + (tq * Hq + h) * d, k + ((int64_t)pr->k_tok0 * Hkv + g) * d,
                     v + ((int64_t)pr->k_tok0 * Hkv + g) * d, kvs, n_vis, d, scale, o_part + (row * Hq + h) * d);
      }
    }
  }
  return 0;
}

#define ZO_MAX_PARTS 16
/* One run of `len` output tokens starting at out_tok0, each the combination of n_parts partial rows:
 * part p contributes rows part_row0[p] .. part_row0[p]+len-1 of o_part / lse_part. */
typedef struct {
  int32_t out_tok0, len, n_parts;
  int32_t part_row0[ZO_MAX_PARTS];
} zo_merge;

/* LSE = log sum_p exp(LSE_p);  O = sum_p exp(LSE_p - LSE) O_p.  Parts with LSE_p = -inf weigh 0;
 * if all are -inf the row is LSE = -inf, O = 0. o [T][Hq][d], lse [Hq][T]. */
int zo_lse_merge(const double *o_part, const double *lse_part, int64_t part_rows, const zo_merge *merges,
                 int n_merges, int64_t T, int Hq, int d, double *o, double *lse) {
  if (!o_part || !lse_part || !o || !lse) return -1;
  for (int m = 0; m < n_merges; m++) {
    const zo_merge *mg = &merges[m];
    if (mg->n_parts < 1 || mg->n_parts > ZO_MAX_PARTS || mg->len < 0 || mg->out_tok0 < 0 ||
        mg->out_tok0 + (int64_t)mg->len > T)
      return -1;
    for (int p = 0; p < mg->n_parts; p++)
      if (mg->part_row0[p] < 0 || mg->part_row0[p] + (int64_t)mg->len > part_rows) return -1;
  }
  for (int m = 0; m < n_merges; m++) {
    const zo_merge *mg = &merges[m];
#pragma omp parallel for collapse(2) schedule(static)
    for (int h = 0; h < Hq; h++) {
      for (int r = 0; r < mg->len; r++) {
        double mx = -INFINITY;
        for (int p = 0; p < mg->n_parts; p++) {
          double lp = lse_part[(int64_t)h * part_rows + mg->part_row0[p] + r];
          if (lp > mx) mx = lp;
        }
        int64_t t = (int64_t)mg->out_tok0 + r;
        double *orow = o + (t * Hq + h) * d;
        for (int c = 0; c < d; c++) orow[c] = 0.0;
        if (mx == -INFINITY) {
          lse[(int64_t)h * T + t] = -INFINITY;
          continue;
        }
        double sum = 0.0;
        for (int p = 0; p < mg->n_parts; p++) sum += exp(lse_part[(int64_t)h * part_rows + mg->part_row0[p] + r] - mx);
        double L = mx + log(sum);
        lse[(int64_t)h * T + t] = L;
        for (int p = 0; p < mg->n_parts; p++) {
          int64_t prow = (int64_t)mg->part_row0[p] + r;
          double lp = lse_part[(int64_t)h * part_rows + prow];
          if (lp == -INFINITY) continue;
          double w = exp(lp - L);
          const double *op = o_part + (prow * Hq + h) * d;
          for (int c = 0; c < d; c++) orow[c] += w * op[c];
        }
      }
    }
  }
  return 0;
}

/* ---- backward ------------------------------------------------------------------------------
 * With P_ij = exp(S_ij - LSE_i), D_i = dO_i . O_i, dP_ij = dO_i . V_j, dS_ij = P_ij (dP_ij - D_i):
 *   dQ_i = scale sum_{j<=i} dS_ij K_j
 *   dK_j = scale sum_{h in group} sum_{i>=j} dS_ij Q_i      dV_j = sum_{h in group} sum_{i>=j} P_ij dO_i
 * O and LSE are the oracle's own fp64 forward values. */

static void dq_row(const double *q, const double *k, const double *v, const double *dout, int Hq, int Hkv, int d,
                   int64_t t0, int64_t i, int h, double scale, double lse_i, double D_i, double *dq_out) {
  const int g = h / (Hq / Hkv);
  const double *qi = q + ((t0 + i) * Hq + h) * d;
  const double *doi = dout + ((t0 + i) * Hq + h) * d;
  for (int c = 0; c < d; c++) dq_out[c] = 0.0;
  for (int64_t j = 0; j <= i; j++) {
    const double *kj = k + ((t0 + j) * Hkv + g) * d;
    const double *vj = v + ((t0 + j) * Hkv + g) * d;
    double p = exp(scale * dotd(qi, kj, d) - lse_i);
    double ds = p * (dotd(doi, vj, d) - D_i);
    for (int c = 0; c < d; c++) dq_out[c] += scale * ds * kj[c];
  }
}

static void dkdv_col(const double *q, const double *k, const double *v, const double *dout, int Hq, int Hkv, int d,
                     int64_t T, int64_t t0, int64_t L, int64_t j, int g, double scale, const double *lse,
                     const double *D, double *dk_out, double *dv_out) {
  const int grp = Hq / Hkv;
  const double *kj = k + ((t0 + j) * Hkv + g) * d;
  const double *vj = v + ((t0 + j) * Hkv + g) * d;
  for (int c = 0; c < d; c++) dk_out[c] = dv_out[c] = 0.0;
  for (int h = g * grp; h < (g + 1) * grp; h++) {
    for (int64_t i = j; i < L; i++) {
      const double *qi = q + ((t0 + i) * Hq + h) * d;
      const double *doi = dout + ((t0 + i) * Hq + h) * d;
      double p = exp(scale * dotd(qi, kj, d) - lse[(int64_t)h * T + t0 + i]);
      double ds = p * (dotd(doi, vj, d) - D[(int64_t)h * T + t0 + i]);
      for (int c = 0; c < d; c++) {
        dk_out[c] += scale * ds * qi[c];
        dv_out[c] += p * doi[c];
      }
    }
  }
}

/* LSE_i and D_i for one (token, head), from the oracle's own forward row. */
static void row_stats(const double *q, const double *k, const double *v, const double *dout, int Hq, int Hkv, int d,
                      int64_t t0, int64_t i, int h, double scale, double *lse_out, double *D_out) {
  const int g = h / (Hq / Hkv);
  double *orow = (double *)malloc(sizeof(double) * (size_t)d);
  *lse_out = attn_row(q + ((t0 + i) * Hq + h) * d, k + (t0 * Hkv + g) * d, v + (t0 * Hkv + g) * d, (int64_t)Hkv * d,
                      i + 1, d, scale, orow);
  *D_out = dotd(dout + ((t0 + i) * Hq + h) * d, orow, d);
  free(orow);
}

int zo_varlen_attn_bwd(const double *dout, const double *q, const double *k, const double *v, int64_t T, int Hq,
                       int Hkv, int d, const int32_t *cu, int S, double scale, double *dq, double *dk, double *dv) {
  if (!dout || !q || !k || !v || !dq || !dk || !dv || Hq <= 0 || Hkv <= 0 || d <= 0 || Hq % Hkv) return -1;
  if (check_cu(cu, S, T)) return -1;
  double *lse = (double *)malloc(sizeof(double) * (size_t)(Hq * T + 1));
  double *D = (double *)malloc(sizeof(double) * (size_t)(Hq * T + 1));
#pragma omp parallel for collapse(2) schedule(dynamic, 16)
  for (int h = 0; h < Hq; h++) {
    for (int64_t t = 0; t < T; t++) {
      int s = seq_of_token(cu, S, t);
      int64_t t0 = cu[s];
      row_stats(q, k, v, dout, Hq, Hkv, d, t0, t - t0, h, scale, &lse[(int64_t)h * T + t], &D[(int64_t)h * T + t]);
      dq_row(q, k, v, dout, Hq, Hkv, d, t0, t - t0, h, scale, lse[(int64_t)h * T + t], D[(int64_t)h * T + t],
             dq + (t * Hq + h) * d);
    }
  }
#pragma omp parallel for collapse(2) schedule(dynamic, 16)
  for (int g = 0; g < Hkv; g++) {
    for (int64_t t = 0; t < T; t++) {
      int s = seq_of_token(cu, S, t);
      int64_t t0 = cu[s], L = cu[s + 1] - cu[s];
      dkdv_col(q, k, v, dout, Hq, Hkv, d, T, t0, L, t - t0, g, scale, lse, D, dk + (t * Hkv + g) * d,
               dv + (t * Hkv + g) * d);
    }
  }
  free(lse);
  free(D);
  return 0;
}

/* Sampled backward for sizes where the full one takes too long: dQ rows for n_q (token, Q head) samples
 * -> dq_out[n_q][d]; dK, dV rows for n_k (token, KV head) samples -> dk_out, dv_out [n_k][d].
 * Same row/column formulas as the full function. */
int zo_varlen_attn_bwd_sample(const double *dout, const double *q, const double *k, const double *v, int64_t T,
                              int Hq, int Hkv, int d, const int32_t *cu, int S, double scale, const int32_t *q_tok,
                              const int32_t *q_head, int n_q, double *dq_out, const int32_t *k_tok,
                              const int32_t *k_head, int n_k, double *dk_out, double *dv_out) {
  if (!dout || !q || !k || !v || Hq <= 0 || Hkv <= 0 || d <= 0 || Hq % Hkv) return -1;
  if (check_cu(cu, S, T)) return -1;
  const int grp = Hq / Hkv;
  for (int n = 0; n < n_q; n++) if (q_tok[n] < 0 || q_tok[n] >= T || q_head[n] < 0 || q_head[n] >= Hq) return -1;
  for (int n = 0; n < n_k; n++) if (k_tok[n] < 0 || k_tok[n] >= T || k_head[n] < 0 || k_head[n] >= Hkv) return -1;
#pragma omp parallel for schedule(dynamic, 1)
  for (int n = 0; n < n_q; n++) {
    int s = seq_of_token(cu, S, q_tok[n]);
    int64_t t0 = cu[s], i = q_tok[n] - t0;
    double l, Dv;
    row_stats(q, k, v, dout, Hq, Hkv, d, t0, i, q_head[n], scale, &l, &Dv);
    dq_row(q, k, v, dout, Hq, Hkv, d, t0, i, q_head[n], scale, l, Dv, dq_out + (int64_t)n * d);
  }
  if (n_k > 0) {
    /* statistics of every row a sampled column needs: rows at or after it, same sequence, heads of its group */
    unsigned char *need = (unsigned char *)calloc((size_t)(Hq * T + 1), 1);
    double *lse = (double *)malloc(sizeof(double) * (size_t)(Hq * T + 1));
    double *D = (double *)malloc(sizeof(double) * (size_t)(Hq * T + 1));
    for (int n = 0; n < n_k; n++) {
      int s = seq_of_token(cu, S, k_tok[n]);
      for (int h = k_head[n] * grp; h < (k_head[n] + 1) * grp; h++)
        for (int64_t t = k_tok[n]; t < cu[s + 1]; t++) need[(int64_t)h * T + t] = 1;
    }
#pragma omp parallel for collapse(2) schedule(dynamic, 16)
    for (int h = 0; h < Hq; h++) {
      for (int64_t t = 0; t < T; t++) {
        if (!need[(int64_t)h * T + t]) continue;
        int s = seq_of_token(cu, S, t);
        int64_t t0 = cu[s];
        row_stats(q, k, v, dout, Hq, Hkv, d, t0, t - t0, h, scale, &lse[(int64_t)h * T + t], &D[(int64_t)h * T + t]);
      }
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int n = 0; n < n_k; n++) {
      int s = seq_of_token(cu, S, k_tok[n]);
      int64_t t0 = cu[s], L = cu[s + 1] - cu[s];
      dkdv_col(q, k, v, dout, Hq, Hkv, d, T, t0, L, k_tok[n] - t0, k_head[n], scale, lse, D, dk_out + (int64_t)n * d,
               dv_out + (int64_t)n * d);
    }
    free(need);
    free(lse);
    free(D);
  }
  return 0;
}

/* Backward contribution of (Q chunk, KV chunk) pairs, ADDED to dq/dk/dv: the sums of the whole-sequence backward
 * restricted to the pair's causally visible (i, j). lse [Hq][T] and D [Hq][T] are the statistics of the WHOLE rows
 * (merged over all KV chunks): what a ring rank holds after the forward rounds (Sec. 3.2, Sec. 5.4). */
int zo_chunk_attn_partial_bwd(const double *dout, const double *q, const double *k, const double *v, int64_t T,
                              int Hq, int Hkv, int d, const zo_pair *pairs, int n_pairs, double scale,
                              const double *lse, const double *D, double *dq, double *dk, double *dv) {
  if (!dout || !q || !k || !v || !lse || !D || !dq || !dk || !dv || Hq <= 0 || Hkv <= 0 || d <= 0 || Hq % Hkv) return -1;
  const int grp = Hq / Hkv;
  for (int p = 0; p < n_pairs; p++) {
    const zo_pair *pr = &pairs[p];
    if (pr->q_len < 0 || pr->k_len < 0 || pr->q_tok0 < 0 || pr->k_tok0 < 0 || pr->q_tok0 + (int64_t)pr->q_len > T ||
        pr->k_tok0 + (int64_t)pr->k_len > T)
      return -1;
  }
  for (int p = 0; p < n_pairs; p++) {
    const zo_pair *pr = &pairs[p];
    for (int h = 0; h < Hq; h++) {
      const int g = h / grp;
      for (int ii = 0; ii < pr->q_len; ii++) {
        const int64_t ti = (int64_t)pr->q_tok0 + ii;
        const double *qi = q + (ti * Hq + h) * d, *doi = dout + (ti * Hq + h) * d;
        const double lse_i = lse[(int64_t)h * T + ti], D_i = D[(int64_t)h * T + ti];
        for (int jj = 0; jj < pr->k_len; jj++) {
          if ((int64_t)pr->k_pos0 + jj > (int64_t)pr->q_pos0 + ii) break; /* not visible */
          const int64_t tj = (int64_t)pr->k_tok0 + jj;
          const double *kj = k + (tj * Hkv + g) * d, *vj = v + (tj * Hkv + g) * d;
          const double pij = exp(scale * dotd(qi, kj, d) - lse_i);
          const double ds = pij * (dotd(doi, vj, d) - D_i);
          for (int c = 0; c < d; c++) {
            dq[(ti * Hq + h) * d + c] += scale * ds * kj[c];
            dk[(tj * Hkv + g) * d + c] += scale * ds * qi[c];
            dv[(tj * Hkv + g) * d + c] += pij * doi[c];
          }
        }
      }
    }
  }
  return 0;
}

/* Token move of the remapping layer: mode 0 gathers dst[i] = src[idx[i]], mode 1 scatters
 * dst[idx[i]] = src[i]; rows are raw bytes. */
int zo_remap_tokens(const void *src, void *dst, int64_t row_bytes, const int32_t *idx, int64_t n_rows, int mode) {
  if (!src || !dst || !idx || row_bytes <= 0 || n_rows < 0 || (mode != 0 && mode != 1)) return -1;
  for (int64_t i = 0; i < n_rows; i++) if (idx[i] < 0 || idx[i] >= n_rows) return -1;
  const char *s = (const char *)src;
  char *t = (char *)dst;
  for (int64_t i = 0; i < n_rows; i++) {
    if (mode == 0) memcpy(t + i * row_bytes, s + (int64_t)idx[i] * row_bytes, (size_t)row_bytes);
    else memcpy(t + (int64_t)idx[i] * row_bytes, s + i * row_bytes, (size_t)row_bytes);
  }
  return 0;
}

int zo_num_threads(void) {
  int n = 1;
#ifdef _OPENMP
#pragma omp parallel
  {
#pragma omp master
    n = omp_get_num_threads();
  }
#endif
  return n;
}
