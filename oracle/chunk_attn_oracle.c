/*
 * CPU fp64 oracle for chunk attention (forward and gradients).  TEST INFRASTRUCTURE ONLY:
 * it exists to check the GPU library and is never part of the product path.
 *
 * What it computes is the plain definition of masked softmax attention.  A chunk is a set
 * of segments (paper section 3.1, "Definition of Chunk": a chunk {C, S} is a context
 * length C for the first slice plus the slice lengths S).  Segment t has q_len = s query
 * rows and kv_len = C + s key/value rows.  Query i of the segment sits at absolute position
 * C + i of its sequence and, because of the causal mask, sees keys j = 0 .. C + i of the
 * segment's own key range and nothing else (section 2.1, pipeline-parallelism paragraph: a
 * query accesses only preceding tokens' keys and values; section 2.2, sequence packing:
 * packed sequences stay independent).  For query head h (KV head g = h / (Hq/Hkv)):
 *
 *     S_ij  = scale * <Q_i, K_j>                 j < n_i = C + i + 1
 *     LSE_i = log sum_j exp(S_ij)
 *     P_ij  = exp(S_ij - LSE_i)
 *     O_i   = sum_j P_ij V_j
 *
 * and, for the scalar loss L = sum O .* dO, the exact gradients
 *
 *     D_i   = <dO_i, O_i>
 *     dP_ij = <dO_i, V_j>          dS_ij = P_ij (dP_ij - D_i)
 *     dQ_i  = scale * sum_j dS_ij K_j
 *     dK_j  = scale * sum_{h in g} sum_{i sees j} dS_ij Q_i
 *     dV_j  =         sum_{h in g} sum_{i sees j} P_ij  dO_i
 *
 * (section 2.1: the key/value gradients of a token depend on the tokens after it; section
 * 3.2.2: key/value gradients of a split sequence collect contributions of all its slices).
 *
 * Everything is float64, written as loops over (head, row, key) with no tiling and no
 * running softmax.  Inputs are either float64 arrays or bf16 bit patterns (uint16), which
 * widen exactly.  Layouts: Q, dO, O, dQ are [rows][Hq][d]; K, V, dK, dV are [rows][Hkv][d].
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  int32_t q_start, q_len, kv_start, kv_len;
} oracle_seg;

typedef struct {
  int32_t num_q_heads, num_kv_heads, head_dim;
  int32_t num_segments;
  const oracle_seg *segments;
  double scale;
  int32_t is_bf16; /* 1: inputs are uint16 bf16 bit patterns, 0: inputs are double */
} oracle_problem;

static inline double ld(const void *base, int64_t idx, int is_bf16) {
  if (is_bf16) {
    uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
    float f;
    memcpy(&f, &bits, 4);
    return (double)f;
  }
  return ((const double *)base)[idx];
}

/* segment that owns query row `row`, or -1 */
static int find_seg(const oracle_problem *p, int64_t row) {
  for (int t = 0; t < p->num_segments; ++t) {
    const oracle_seg *s = &p->segments[t];
    if (row >= s->q_start && row < (int64_t)s->q_start + s->q_len) return t;
  }
  return -1;
}

/* Scores of one query against its visible keys; returns n_i, fills sc[0..n_i) and *lse. */
static int64_t row_scores(const oracle_problem *p, const void *q, const void *k, int h, int64_t row,
                          const oracle_seg *s, double *sc, double *lse) {
  const int d = p->head_dim, Hq = p->num_q_heads, Hkv = p->num_kv_heads;
  const int g = h / (Hq / Hkv);
  const int64_t i = row - s->q_start;
  const int64_t n = (int64_t)(s->kv_len - s->q_len) + i + 1;
  double mx = -INFINITY;
  for (int64_t j = 0; j < n; ++j) {
    double acc = 0.0;
    for (int c = 0; c < d; ++c)
      acc += ld(q, (row * Hq + h) * d + c, p->is_bf16) *
             ld(k, (((int64_t)s->kv_start + j) * Hkv + g) * d + c, p->is_bf16);
    sc[j] = acc * p->scale;
    if (sc[j] > mx) mx = sc[j];
  }
  double sum = 0.0;
  for (int64_t j = 0; j < n; ++j) sum += exp(sc[j] - mx);
  *lse = mx + log(sum);
  return n;
}

static int64_t max_kv_len(const oracle_problem *p) {
  int64_t m = 1;
  for (int t = 0; t < p->num_segments; ++t)
    if (p->segments[t].kv_len > m) m = p->segments[t].kv_len;
  return m;
}

/*
 * Forward for a list of (head, row) pairs: out_o[n][d], out_lse[n].
 * Returns 0, or -1 if a row belongs to no segment.
 */
int oracle_fwd_rows(const oracle_problem *p, const void *q, const void *k, const void *v, int64_t n_pairs,
                    const int32_t *heads, const int32_t *rows, double *out_o, double *out_lse) {
  const int d = p->head_dim, Hq = p->num_q_heads, Hkv = p->num_kv_heads;
  const int64_t cap = max_kv_len(p);
  int bad = 0;
#pragma omp parallel
  {
    double *sc = (double *)malloc(sizeof(double) * (size_t)cap);
#pragma omp for schedule(dynamic, 1)
    for (int64_t r = 0; r < n_pairs; ++r) {
      const int h = heads[r];
      const int64_t row = rows[r];
      const int t = find_seg(p, row);
      if (t < 0 || h < 0 || h >= Hq) {
#pragma omp atomic write
        bad = 1;
        continue;
      }
      const oracle_seg *s = &p->segments[t];
      const int g = h / (Hq / Hkv);
      double lse;
      const int64_t n = row_scores(p, q, k, h, row, s, sc, &lse);
      for (int c = 0; c < d; ++c) out_o[r * d + c] = 0.0;
      for (int64_t j = 0; j < n; ++j) {
        const double pij = exp(sc[j] - lse);
        for (int c = 0; c < d; ++c)
          out_o[r * d + c] += pij * ld(v, (((int64_t)s->kv_start + j) * Hkv + g) * d + c, p->is_bf16);
      }
      out_lse[r] = lse;
    }
    free(sc);
  }
  return bad ? -1 : 0;
}

/*
 * Query-side backward for a list of (head, row) pairs:
 * out_dq[n][d], out_lse[n], out_dsum[n] (= D_i).  The oracle uses its own fp64 O for D.
 */
int oracle_dq_rows(const oracle_problem *p, const void *q, const void *k, const void *v, const void *d_o,
                   int64_t n_pairs, const int32_t *heads, const int32_t *rows, double *out_dq, double *out_lse,
                   double *out_dsum) {
  const int d = p->head_dim, Hq = p->num_q_heads, Hkv = p->num_kv_heads;
  const int64_t cap = max_kv_len(p);
  int bad = 0;
#pragma omp parallel
  {
    double *sc = (double *)malloc(sizeof(double) * (size_t)cap);
    double *o = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 1)
    for (int64_t r = 0; r < n_pairs; ++r) {
      const int h = heads[r];
      const int64_t row = rows[r];
      const int t = find_seg(p, row);
      if (t < 0 || h < 0 || h >= Hq) {
#pragma omp atomic write
        bad = 1;
        continue;
      }
      const oracle_seg *s = &p->segments[t];
      const int g = h / (Hq / Hkv);
      double lse;
      const int64_t n = row_scores(p, q, k, h, row, s, sc, &lse);
      for (int c = 0; c < d; ++c) o[c] = 0.0;
      for (int64_t j = 0; j < n; ++j) {
        const double pij = exp(sc[j] - lse);
        for (int c = 0; c < d; ++c) o[c] += pij * ld(v, (((int64_t)s->kv_start + j) * Hkv + g) * d + c, p->is_bf16);
      }
      double dsum = 0.0;
      for (int c = 0; c < d; ++c) dsum += ld(d_o, (row * Hq + h) * d + c, p->is_bf16) * o[c];
      for (int c = 0; c < d; ++c) out_dq[r * d + c] = 0.0;
      for (int64_t j = 0; j < n; ++j) {
        const int64_t kv = (((int64_t)s->kv_start + j) * Hkv + g) * d;
        double dp = 0.0;
        for (int c = 0; c < d; ++c) dp += ld(d_o, (row * Hq + h) * d + c, p->is_bf16) * ld(v, kv + c, p->is_bf16);
        const double ds = exp(sc[j] - lse) * (dp - dsum);
        for (int c = 0; c < d; ++c) out_dq[r * d + c] += p->scale * ds * ld(k, kv + c, p->is_bf16);
      }
      out_lse[r] = lse;
      out_dsum[r] = dsum;
    }
    free(sc);
    free(o);
  }
  return bad ? -1 : 0;
}

/*
 * Key/value-side backward for a list of (kv_head, kv_row) pairs: out_dk[n][d], out_dv[n][d].
 * lse and dsum are [Hq][total_q] tables of LSE_i and D_i (from oracle_dq_rows) and must be
 * filled for every query that sees a requested key row.  A key row outside every segment
 * gets zeros (no query sees it).
 */
int oracle_dkv_rows(const oracle_problem *p, const void *q, const void *k, const void *v, const void *d_o,
                    int64_t total_q, const double *lse, const double *dsum, int64_t n_pairs,
                    const int32_t *kv_heads, const int32_t *kv_rows, double *out_dk, double *out_dv) {
  const int d = p->head_dim, Hq = p->num_q_heads, Hkv = p->num_kv_heads;
  const int G = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t r = 0; r < n_pairs; ++r) {
    const int g = kv_heads[r];
    const int64_t kvrow = kv_rows[r];
    for (int c = 0; c < d; ++c) out_dk[r * d + c] = out_dv[r * d + c] = 0.0;
    for (int t = 0; t < p->num_segments; ++t) {
      const oracle_seg *s = &p->segments[t];
      if (kvrow < s->kv_start || kvrow >= (int64_t)s->kv_start + s->kv_len) continue;
      const int64_t j = kvrow - s->kv_start;
      const int64_t C = s->kv_len - s->q_len;
      /* query i sees key j iff j <= C + i */
      int64_t i0 = j - C;
      if (i0 < 0) i0 = 0;
      for (int h = g * G; h < (g + 1) * G; ++h) {
        for (int64_t i = i0; i < s->q_len; ++i) {
          const int64_t row = (int64_t)s->q_start + i;
          const int64_t qo = (row * Hq + h) * d, ko = (kvrow * Hkv + g) * d;
          double sij = 0.0, dp = 0.0;
          for (int c = 0; c < d; ++c) sij += ld(q, qo + c, p->is_bf16) * ld(k, ko + c, p->is_bf16);
          for (int c = 0; c < d; ++c) dp += ld(d_o, qo + c, p->is_bf16) * ld(v, ko + c, p->is_bf16);
          const double pij = exp(sij * p->scale - lse[(int64_t)h * total_q + row]);
          const double ds = pij * (dp - dsum[(int64_t)h * total_q + row]);
          for (int c = 0; c < d; ++c) {
            out_dk[r * d + c] += p->scale * ds * ld(q, qo + c, p->is_bf16);
            out_dv[r * d + c] += pij * ld(d_o, qo + c, p->is_bf16);
          }
        }
      }
    }
  }
  return 0;
}

/* Number of (query, key) pairs the loops above visit for one query head. */
int64_t oracle_pair_count(const oracle_problem *p) {
  int64_t n = 0;
  for (int t = 0; t < p->num_segments; ++t) {
    const oracle_seg *s = &p->segments[t];
    for (int64_t i = 0; i < s->q_len; ++i) n += (int64_t)(s->kv_len - s->q_len) + i + 1;
  }
  return n;
}
