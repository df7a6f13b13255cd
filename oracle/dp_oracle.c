/*
 * Double-P decode attention: plain fp64 CPU oracle (test infrastructure only;
 * see dp_oracle.h).  Scalar loops, no blocking, no fusion: each function is
 * one equation or one selection rule of the paper, in the paper's order.
 */
#include "dp_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* bf16 is the upper half of an IEEE float: widening is exact. */
static double bf16_to_double(uint16_t bits) {
  uint32_t u = (uint32_t)bits << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

static double scale_of(const dpo_cache *c) {
  return c->sm_scale != 0.0 ? c->sm_scale : 1.0 / sqrt((double)c->head_dim);
}

static int32_t seg_of(const dpo_cache *c, int32_t b, int32_t h) {
  int32_t group = c->n_q_heads / c->n_kv_heads;
  return b * c->n_kv_heads + h / group;
}

/* (q . row) * scale, with row a bf16 row of length d */
static double scaled_dot(const uint16_t *q, const uint16_t *row, int32_t d, double scale) {
  double acc = 0.0;
  for (int32_t t = 0; t < d; ++t) acc += bf16_to_double(q[t]) * bf16_to_double(row[t]);
  return acc * scale;
}

int32_t dpo_num_clusters(const dpo_cache *c, int32_t b, int32_t h) {
  int32_t seg = seg_of(c, b, h);
  return c->seg_cluster_ptr[seg + 1] - c->seg_cluster_ptr[seg];
}

/* ---- Sec. 4.2, Eq. 3 (centroid logit) and Eq. 5 (log of the estimated mass) ---- */
void dpo_centroid_logits(const dpo_cache *c, int32_t b, int32_t h, double *logit) {
  const int32_t d = c->head_dim, seg = seg_of(c, b, h);
  const int32_t c0 = c->seg_cluster_ptr[seg], n = c->seg_cluster_ptr[seg + 1] - c0;
  const uint16_t *q = c->q + ((int64_t)b * c->n_q_heads + h) * d;
  const double scale = scale_of(c);
  for (int32_t i = 0; i < n; ++i) {
    int32_t s = c->cluster_sizes[c0 + i];
    if (s <= 0) {
      logit[i] = -INFINITY;
      continue;
    }
    double xbar = scaled_dot(q, c->k_centroids + (int64_t)(c0 + i) * d, d, scale);
    logit[i] = xbar + log((double)s);
  }
}

/* ---- Eq. 6: softmax over clusters ---- */
void dpo_cluster_distribution(const double *logit, int32_t n, double *a_hat) {
  double mx = -INFINITY, sum = 0.0;
  for (int32_t i = 0; i < n; ++i)
    if (logit[i] > mx) mx = logit[i];
  for (int32_t i = 0; i < n; ++i) {
    a_hat[i] = (logit[i] == -INFINITY) ? 0.0 : exp(logit[i] - mx);
    sum += a_hat[i];
  }
  for (int32_t i = 0; i < n; ++i) a_hat[i] = (sum > 0.0) ? a_hat[i] / sum : 0.0;
}

/* ---- order of Eq. 7: descending score, lower index first among equals ---- */
typedef struct {
  double key;
  int32_t idx;
} keyed;

static int by_key_desc_then_index(const void *pa, const void *pb) {
  const keyed *a = (const keyed *)pa, *b = (const keyed *)pb;
  if (a->key > b->key) return -1;
  if (a->key < b->key) return 1;
  return (a->idx > b->idx) - (a->idx < b->idx);
}

int32_t dpo_sorted_order(const double *logit, int32_t n, int32_t *order) {
  keyed *tmp = (keyed *)malloc(sizeof(keyed) * (size_t)(n > 0 ? n : 1));
  int32_t m = 0;
  for (int32_t i = 0; i < n; ++i)
    if (logit[i] != -INFINITY) {
      tmp[m].key = logit[i];
      tmp[m].idx = i;
      ++m;
    }
  qsort(tmp, (size_t)m, sizeof(keyed), by_key_desc_then_index);
  for (int32_t i = 0; i < m; ++i) order[i] = tmp[i].idx;
  free(tmp);
  return m;
}

/* ---- Eq. 7 (first top-p) and Sec. 4.3 (second top-p on the same order) ---- */
void dpo_double_top_p(const double *a_hat, const int32_t *order, int32_t n_nonempty, double p1, double p2,
                      uint32_t flags, double *cum, int32_t *k1_out, int32_t *k2_out, double *m1_out) {
  double run = 0.0;
  for (int32_t r = 0; r < n_nonempty; ++r) {
    run += a_hat[order[r]];
    cum[r] = run;
  }
  /* smallest prefix whose mass reaches p1; everything if p1 >= 1 or never reached */
  int32_t k1 = n_nonempty;
  if (p1 < 1.0)
    for (int32_t r = 0; r < n_nonempty; ++r)
      if (cum[r] >= p1) {
        k1 = r + 1;
        break;
      }
  double m1 = (k1 > 0) ? cum[k1 - 1] : 0.0;
  /* second threshold: a fraction p2 of the retained mass (default), or p2 of the whole */
  int32_t k2;
  if (p2 >= 1.0) {
    k2 = k1;
  } else {
    double tau2 = (flags & DPO_P2_ABSOLUTE) ? (p2 < m1 ? p2 : m1) : p2 * m1;
    k2 = k1;
    if (tau2 <= 0.0) {
      k2 = 0;
    } else {
      for (int32_t r = 0; r < k1; ++r)
        if (cum[r] >= tau2) {
          k2 = r + 1;
          break;
        }
    }
  }
  *k1_out = k1;
  *k2_out = k2;
  *m1_out = m1;
}

/* ---- Eq. 8 (shared normaliser) and Eq. 9 (mixed output) ---- */
void dpo_mixed_attention(const dpo_cache *c, int32_t b, int32_t h, const int32_t *exact_ids, int32_t n_exact,
                         const int32_t *approx_ids, int32_t n_approx, double *out, double *lse) {
  const int32_t d = c->head_dim, seg = seg_of(c, b, h);
  const int32_t c0 = c->seg_cluster_ptr[seg];
  const int64_t row0 = c->seg_row_base[seg];
  const uint16_t *q = c->q + ((int64_t)b * c->n_q_heads + h) * d;
  const double scale = scale_of(c);

  /* pass 1: the largest exponent, so that exp() below cannot overflow */
  double mx = -INFINITY;
  for (int32_t e = 0; e < n_exact; ++e) {
    int32_t ci = c0 + exact_ids[e];
    for (int32_t j = 0; j < c->cluster_sizes[ci]; ++j) {
      double x = scaled_dot(q, c->k_cache + (row0 + c->cluster_offsets[ci] + j) * d, d, scale);
      if (x > mx) mx = x;
    }
  }
  for (int32_t a = 0; a < n_approx; ++a) {
    int32_t ci = c0 + approx_ids[a];
    if (c->cluster_sizes[ci] <= 0) continue;
    double lz = scaled_dot(q, c->k_centroids + (int64_t)ci * d, d, scale) + log((double)c->cluster_sizes[ci]);
    if (lz > mx) mx = lz;
  }
  for (int32_t t = 0; t < d; ++t) out[t] = 0.0;
  if (mx == -INFINITY) {
    *lse = -INFINITY;
    return;
  }
  /* pass 2: Z~ * exp(-mx) and the unnormalised output */
  double z = 0.0;
  for (int32_t e = 0; e < n_exact; ++e) {
    int32_t ci = c0 + exact_ids[e];
    for (int32_t j = 0; j < c->cluster_sizes[ci]; ++j) {
      int64_t row = row0 + c->cluster_offsets[ci] + j;
      double w = exp(scaled_dot(q, c->k_cache + row * d, d, scale) - mx); /* exp(x_ij) */
      z += w;
      for (int32_t t = 0; t < d; ++t) out[t] += w * bf16_to_double(c->v_cache[row * d + t]);
    }
  }
  for (int32_t a = 0; a < n_approx; ++a) {
    int32_t ci = c0 + approx_ids[a];
    int32_t s = c->cluster_sizes[ci];
    if (s <= 0) continue;
    double xbar = scaled_dot(q, c->k_centroids + (int64_t)ci * d, d, scale);
    double w = (double)s * exp(xbar - mx); /* Zhat_i = s_i exp(xbar_i) */
    z += w;
    for (int32_t t = 0; t < d; ++t) out[t] += w * bf16_to_double(c->v_centroids[(int64_t)ci * d + t]);
  }
  for (int32_t t = 0; t < d; ++t) out[t] /= z;
  *lse = mx + log(z);
}

/* ---- Eq. 1: dense softmax attention over all tokens of the segment ---- */
void dpo_dense_attention(const dpo_cache *c, int32_t b, int32_t h, double *out, double *lse) {
  const int32_t d = c->head_dim, seg = seg_of(c, b, h);
  const int32_t c0 = c->seg_cluster_ptr[seg], n = c->seg_cluster_ptr[seg + 1] - c0;
  const int64_t row0 = c->seg_row_base[seg];
  const uint16_t *q = c->q + ((int64_t)b * c->n_q_heads + h) * d;
  const double scale = scale_of(c);
  double mx = -INFINITY;
  for (int32_t i = 0; i < n; ++i)
    for (int32_t j = 0; j < c->cluster_sizes[c0 + i]; ++j) {
      double x = scaled_dot(q, c->k_cache + (row0 + c->cluster_offsets[c0 + i] + j) * d, d, scale);
      if (x > mx) mx = x;
    }
  for (int32_t t = 0; t < d; ++t) out[t] = 0.0;
  if (mx == -INFINITY) {
    *lse = -INFINITY;
    return;
  }
  double z = 0.0;
  for (int32_t i = 0; i < n; ++i)
    for (int32_t j = 0; j < c->cluster_sizes[c0 + i]; ++j) {
      int64_t row = row0 + c->cluster_offsets[c0 + i] + j;
      double w = exp(scaled_dot(q, c->k_cache + row * d, d, scale) - mx);
      z += w;
      for (int32_t t = 0; t < d; ++t) out[t] += w * bf16_to_double(c->v_cache[row * d + t]);
    }
  for (int32_t t = 0; t < d; ++t) out[t] /= z;
  *lse = mx + log(z);
}

/* ---- Eq. 4: exact cluster mass, as a logarithm ---- */
void dpo_exact_cluster_log_mass(const dpo_cache *c, int32_t b, int32_t h, double *log_z) {
  const int32_t d = c->head_dim, seg = seg_of(c, b, h);
  const int32_t c0 = c->seg_cluster_ptr[seg], n = c->seg_cluster_ptr[seg + 1] - c0;
  const int64_t row0 = c->seg_row_base[seg];
  const uint16_t *q = c->q + ((int64_t)b * c->n_q_heads + h) * d;
  const double scale = scale_of(c);
  for (int32_t i = 0; i < n; ++i) {
    int32_t s = c->cluster_sizes[c0 + i];
    double mx = -INFINITY, z = 0.0;
    for (int32_t j = 0; j < s; ++j) {
      double x = scaled_dot(q, c->k_cache + (row0 + c->cluster_offsets[c0 + i] + j) * d, d, scale);
      if (x > mx) mx = x;
    }
    for (int32_t j = 0; j < s; ++j)
      z += exp(scaled_dot(q, c->k_cache + (row0 + c->cluster_offsets[c0 + i] + j) * d, d, scale) - mx);
    log_z[i] = (s > 0) ? mx + log(z) : -INFINITY;
  }
}

/* ---- pinned clusters (Sec. 5.1: sink and window tokens stay dense, the selection sees the rest) ---- */
static int is_pinned(const dpo_cache *c, int32_t cluster) {
  return c->cluster_flags && (c->cluster_flags[cluster] & DPO_CLUSTER_PINNED);
}

void dpo_candidate_logits(const dpo_cache *c, int32_t b, int32_t h, double *logit) {
  const int32_t seg = seg_of(c, b, h);
  const int32_t c0 = c->seg_cluster_ptr[seg], n = c->seg_cluster_ptr[seg + 1] - c0;
  dpo_centroid_logits(c, b, h, logit);
  for (int32_t i = 0; i < n; ++i)
    if (is_pinned(c, c0 + i)) logit[i] = -INFINITY;
}

int32_t dpo_pinned_clusters(const dpo_cache *c, int32_t b, int32_t h, int32_t *ids) {
  const int32_t seg = seg_of(c, b, h);
  const int32_t c0 = c->seg_cluster_ptr[seg], n = c->seg_cluster_ptr[seg + 1] - c0;
  int32_t m = 0;
  for (int32_t i = 0; i < n; ++i)
    if (is_pinned(c, c0 + i) && c->cluster_sizes[c0 + i] > 0) ids[m++] = i;
  return m;
}

/* exact set of a head = the pinned clusters, then the first k2 clusters of the order */
static int32_t exact_with_pinned(const dpo_cache *c, int32_t b, int32_t h, const int32_t *order, int32_t k2,
                                 int32_t *exact) {
  int32_t m = dpo_pinned_clusters(c, b, h, exact);
  for (int32_t r = 0; r < k2; ++r) exact[m++] = order[r];
  return m;
}

/* ---- one head of the decode step: the stages chained in the paper's order ---- */
static void decode_head(const dpo_cache *c, int32_t b, int32_t h, double p1, double p2, uint32_t flags, double *out,
                        double *lse, int32_t *k1, int32_t *k2, int32_t *order_out) {
  int32_t n = dpo_num_clusters(c, b, h);
  size_t m = (size_t)(n > 0 ? n : 1);
  double *logit = (double *)malloc(sizeof(double) * m);
  double *a_hat = (double *)malloc(sizeof(double) * m);
  double *cum = (double *)malloc(sizeof(double) * m);
  int32_t *order = (int32_t *)malloc(sizeof(int32_t) * m);
  double m1;
  int32_t *exact = (int32_t *)malloc(sizeof(int32_t) * m);
  dpo_candidate_logits(c, b, h, logit);
  dpo_cluster_distribution(logit, n, a_hat);
  int32_t nn = dpo_sorted_order(logit, n, order);
  dpo_double_top_p(a_hat, order, nn, p1, p2, flags, cum, k1, k2, &m1);
  int32_t ne = exact_with_pinned(c, b, h, order, *k2, exact);
  dpo_mixed_attention(c, b, h, exact, ne, order + *k2, *k1 - *k2, out, lse);
  if (order_out) memcpy(order_out, order, sizeof(int32_t) * (size_t)nn);
  free(exact);
  free(logit);
  free(a_hat);
  free(cum);
  free(order);
}

int32_t dpo_decode_step(const dpo_cache *c, double p1, double p2, uint32_t flags, double *out, double *lse,
                        int32_t *k1, int32_t *k2, int32_t *order, int64_t order_stride, int32_t n_threads) {
  const int32_t nh = c->batch * c->n_q_heads, d = c->head_dim;
  int32_t used = 1;
#ifdef _OPENMP
  if (n_threads > 1) {
    used = n_threads < nh ? n_threads : (nh > 0 ? nh : 1);
#pragma omp parallel for schedule(dynamic, 1) num_threads(used)
    for (int32_t i = 0; i < nh; ++i)
      decode_head(c, i / c->n_q_heads, i % c->n_q_heads, p1, p2, flags, out + (int64_t)i * d, lse + i, k1 + i,
                  k2 + i, order ? order + i * order_stride : 0);
    return used;
  }
#endif
  (void)n_threads;
  for (int32_t i = 0; i < nh; ++i)
    decode_head(c, i / c->n_q_heads, i % c->n_q_heads, p1, p2, flags, out + (int64_t)i * d, lse + i, k1 + i, k2 + i,
                order ? order + i * order_stride : 0);
  return used;
}

/* ---- fixed budget instead of the two top-p thresholds (Sec. 5.1, cluster-based baseline) ---- */
void dpo_fixed_budget(int32_t n_nonempty, int32_t k_retained, int32_t k_exact, int32_t *k1_out, int32_t *k2_out) {
  int32_t k1 = k_retained < 0 ? 0 : k_retained;
  if (k1 > n_nonempty) k1 = n_nonempty;
  int32_t k2 = k_exact < 0 ? 0 : k_exact;
  if (k2 > k1) k2 = k1;
  *k1_out = k1;
  *k2_out = k2;
}

static void budget_head(const dpo_cache *c, int32_t b, int32_t h, int32_t k_retained, int32_t k_exact, double *out,
                        double *lse, int32_t *k1, int32_t *k2, int32_t *order_out) {
  int32_t n = dpo_num_clusters(c, b, h);
  size_t m = (size_t)(n > 0 ? n : 1);
  double *logit = (double *)malloc(sizeof(double) * m);
  int32_t *order = (int32_t *)malloc(sizeof(int32_t) * m);
  int32_t *exact = (int32_t *)malloc(sizeof(int32_t) * m);
  dpo_candidate_logits(c, b, h, logit);
  int32_t nn = dpo_sorted_order(logit, n, order);
  dpo_fixed_budget(nn, k_retained, k_exact, k1, k2);
  int32_t ne = exact_with_pinned(c, b, h, order, *k2, exact);
  dpo_mixed_attention(c, b, h, exact, ne, order + *k2, *k1 - *k2, out, lse);
  if (order_out) memcpy(order_out, order, sizeof(int32_t) * (size_t)nn);
  free(exact);
  free(logit);
  free(order);
}

int32_t dpo_budget_step(const dpo_cache *c, int32_t k_retained, int32_t k_exact, double *out, double *lse,
                        int32_t *k1, int32_t *k2, int32_t *order, int64_t order_stride, int32_t n_threads) {
  const int32_t nh = c->batch * c->n_q_heads, d = c->head_dim;
  int32_t used = 1;
#ifdef _OPENMP
  if (n_threads > 1) {
    used = n_threads < nh ? n_threads : (nh > 0 ? nh : 1);
#pragma omp parallel for schedule(dynamic, 1) num_threads(used)
    for (int32_t i = 0; i < nh; ++i)
      budget_head(c, i / c->n_q_heads, i % c->n_q_heads, k_retained, k_exact, out + (int64_t)i * d, lse + i, k1 + i,
                  k2 + i, order ? order + i * order_stride : 0);
    return used;
  }
#endif
  (void)n_threads;
  for (int32_t i = 0; i < nh; ++i)
    budget_head(c, i / c->n_q_heads, i % c->n_q_heads, k_retained, k_exact, out + (int64_t)i * d, lse + i, k1 + i,
                k2 + i, order ? order + i * order_stride : 0);
  return used;
}

int32_t dpo_dense_step(const dpo_cache *c, double *out, double *lse, int32_t n_threads) {
  const int32_t nh = c->batch * c->n_q_heads, d = c->head_dim;
  int32_t used = 1;
#ifdef _OPENMP
  if (n_threads > 1) {
    used = n_threads < nh ? n_threads : (nh > 0 ? nh : 1);
#pragma omp parallel for schedule(dynamic, 1) num_threads(used)
    for (int32_t i = 0; i < nh; ++i)
      dpo_dense_attention(c, i / c->n_q_heads, i % c->n_q_heads, out + (int64_t)i * d, lse + i);
    return used;
  }
#endif
  (void)n_threads;
  for (int32_t i = 0; i < nh; ++i)
    dpo_dense_attention(c, i / c->n_q_heads, i % c->n_q_heads, out + (int64_t)i * d, lse + i);
  return used;
}

/* ---- prefill side (Sec. 4.1): cluster-contiguous cache and cluster metadata from token-order K/V ---- */

/* double -> bf16 bits, one rounding to 8 significant bits, ties to even (finite, normal values) */
static uint16_t double_to_bf16(double x) {
  if (x == 0.0) return (uint16_t)(signbit(x) ? 0x8000u : 0u);
  int e;
  double m = frexp(x, &e);                  /* x = m * 2^e, 0.5 <= |m| < 1 */
  double r = nearbyint(ldexp(m, 8));        /* default rounding mode: ties to even */
  float f = (float)ldexp(r, e - 8);         /* exactly representable */
  uint32_t u;
  memcpy(&u, &f, sizeof u);
  return (uint16_t)(u >> 16);
}

void dpo_build_cluster_cache(int32_t n_seg, int32_t d, const uint16_t *k_tokens, const uint16_t *v_tokens,
                             const int32_t *assignment, const int64_t *seg_row_base, const int32_t *seg_rows,
                             const int32_t *seg_cluster_ptr, uint16_t *k_cache, uint16_t *v_cache,
                             int32_t *cluster_offsets, int32_t *cluster_sizes, uint16_t *k_centroids,
                             uint16_t *v_centroids, double *v_sums, int32_t *token_row) {
  for (int32_t seg = 0; seg < n_seg; ++seg) {
    const int64_t r0 = seg_row_base[seg];
    const int32_t n = seg_rows[seg], c0 = seg_cluster_ptr[seg], kc = seg_cluster_ptr[seg + 1] - c0;
    /* s_i = |T_i| */
    for (int32_t i = 0; i < kc; ++i) cluster_sizes[c0 + i] = 0;
    for (int32_t t = 0; t < n; ++t) {
      int32_t a = assignment[r0 + t];
      if (a >= 0 && a < kc) cluster_sizes[c0 + a] += 1;
    }
    /* clusters are laid out one after the other, in index order */
    int32_t run = 0;
    for (int32_t i = 0; i < kc; ++i) {
      cluster_offsets[c0 + i] = run;
      run += cluster_sizes[c0 + i];
    }
    /* tokens of a cluster keep their token order */
    int32_t *cursor = (int32_t *)malloc(sizeof(int32_t) * (size_t)(kc > 0 ? kc : 1));
    for (int32_t i = 0; i < kc; ++i) cursor[i] = cluster_offsets[c0 + i];
    for (int32_t t = 0; t < n; ++t) {
      int32_t a = assignment[r0 + t];
      int32_t row = -1;
      if (a >= 0 && a < kc) {
        row = cursor[a]++;
        memcpy(k_cache + (r0 + row) * d, k_tokens + (r0 + t) * d, sizeof(uint16_t) * (size_t)d);
        memcpy(v_cache + (r0 + row) * d, v_tokens + (r0 + t) * d, sizeof(uint16_t) * (size_t)d);
      }
      if (token_row) token_row[r0 + t] = row;
    }
    free(cursor);
    /* C_i = mean key, Eq. 2: V^Sigma_i = sum of values, V-bar_i = V^Sigma_i / s_i */
    for (int32_t i = 0; i < kc; ++i) {
      const int32_t s = cluster_sizes[c0 + i];
      for (int32_t j = 0; j < d; ++j) {
        double ks = 0.0, vs = 0.0;
        for (int32_t r = 0; r < s; ++r) {
          const int64_t row = r0 + cluster_offsets[c0 + i] + r;
          ks += bf16_to_double(k_cache[row * d + j]);
          vs += bf16_to_double(v_cache[row * d + j]);
        }
        k_centroids[(int64_t)(c0 + i) * d + j] = s > 0 ? double_to_bf16(ks / s) : 0;
        v_centroids[(int64_t)(c0 + i) * d + j] = s > 0 ? double_to_bf16(vs / s) : 0;
        if (v_sums) v_sums[(int64_t)(c0 + i) * d + j] = vs;
      }
    }
  }
}

/* ---- k-means assignment step (Sec. 4.1): nearest centroid of every key ---- */
void dpo_kmeans_assign(int32_t n_seg, int32_t d, const uint16_t *k_tokens, const uint16_t *centroids,
                       const int64_t *seg_row_base, const int32_t *seg_rows, const int32_t *seg_cluster_ptr,
                       int32_t *assignment, double *best_score, double *runner_up) {
  for (int32_t seg = 0; seg < n_seg; ++seg) {
    const int64_t r0 = seg_row_base[seg];
    const int32_t n = seg_rows[seg], c0 = seg_cluster_ptr[seg], kc = seg_cluster_ptr[seg + 1] - c0;
    for (int32_t t = 0; t < n; ++t) {
      /* |x - c|^2 = |x|^2 - 2 (x.c - |c|^2 / 2): the nearest centroid maximises x.c - |c|^2 / 2 */
      double best = -INFINITY, second = -INFINITY;
      int32_t arg = -1;
      for (int32_t c = 0; c < kc; ++c) {
        double dot = 0.0, nrm = 0.0;
        for (int32_t j = 0; j < d; ++j) {
          const double cj = bf16_to_double(centroids[(int64_t)(c0 + c) * d + j]);
          dot += bf16_to_double(k_tokens[(r0 + t) * d + j]) * cj;
          nrm += cj * cj;
        }
        const double s = dot - 0.5 * nrm;
        if (s > best) { /* strict: the lower index keeps a tie */
          second = best;
          best = s;
          arg = c;
        } else if (s > second) {
          second = s;
        }
      }
      assignment[r0 + t] = arg;
      if (best_score) best_score[r0 + t] = best;
      if (runner_up) runner_up[r0 + t] = second;
    }
  }
}
