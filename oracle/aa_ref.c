/*
 * aa_ref.c -- CPU oracle for the AutoAssist shrink + SGD path (arXiv 1905.03381).
 *
 * TEST INFRASTRUCTURE ONLY: plain single-threaded C, double accumulation in
 * index order, no blocking, fusion or reordering.  Shares nothing with the HIP
 * path.  See aa_ref.h for the contract of every function.
 */
#include "aa_ref.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* Philox4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies
 * with a Weyl key schedule.                                                  */

void aa_ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
  const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    uint64_t p0 = M0 * (uint64_t)c0;
    uint64_t p1 = M1 * (uint64_t)c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += W0;
    k1 += W1;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

float aa_ref_uniform(uint64_t seed, uint64_t step, uint32_t j) {
  uint32_t ctr[4] = {j, 0u, (uint32_t)(step & 0xFFFFFFFFu), (uint32_t)(step >> 32)};
  uint32_t key[2] = {(uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32)};
  uint32_t out[4];
  aa_ref_philox4x32_10(ctr, key, out);
  /* 24 high bits -> multiples of 2^-24 in [0, 1): exact in float. */
  return (float)(out[0] >> 8) * (1.0f / 16777216.0f);
}

/* ------------------------------------------------------------------------- */
/* Row access helpers (oracle-local).                                         */

static int features_ok(const aa_ref_features *F) {
  if (!F) return 0;
  if (F->d <= 0 || F->n < 0) return 0;
  if (F->layout == AA_REF_DENSE) return F->x != NULL && F->ld >= F->d;
  if (F->layout == AA_REF_CSR) return F->rowptr != NULL && (F->col != NULL || F->rowptr[F->n] == 0);
  return 0;
}

/* v . x_row in double, stored entries in stored order. */
static double row_dot(const aa_ref_features *F, int64_t row, const float *v) {
  double acc = 0.0;
  if (F->layout == AA_REF_DENSE) {
    const float *x = F->x + row * F->ld;
    for (int32_t k = 0; k < F->d; ++k) acc += (double)v[k] * (double)x[k];
  } else {
    for (int64_t e = F->rowptr[row]; e < F->rowptr[row + 1]; ++e) {
      double xv = F->val ? (double)F->val[e] : 1.0;
      acc += (double)v[F->col[e]] * xv;
    }
  }
  return acc;
}

/* acc[:] += a * x_row */
static void row_axpy(const aa_ref_features *F, int64_t row, double a, double *acc) {
  if (F->layout == AA_REF_DENSE) {
    const float *x = F->x + row * F->ld;
    for (int32_t k = 0; k < F->d; ++k) acc[k] += a * (double)x[k];
  } else {
    for (int64_t e = F->rowptr[row]; e < F->rowptr[row + 1]; ++e) {
      double xv = F->val ? (double)F->val[e] : 1.0;
      acc[F->col[e]] += a * xv;
    }
  }
}

static double sigmoid_d(double s) { return 1.0 / (1.0 + exp(-s)); }

/* ------------------------------------------------------------------------- */

int32_t aa_ref_assistant_score(const aa_ref_features *F, const int32_t *idx, int32_t P,
                               const float *phi, const float *bias, float *logit, float *prob) {
  if (P < 0) return -2;
  if (P == 0) return 0;
  if (!features_ok(F)) return F ? -2 : -1;
  if (!phi || !prob) return -1;
  double b = bias ? (double)bias[0] : 0.0;
  for (int32_t j = 0; j < P; ++j) {
    int64_t row = idx ? (int64_t)idx[j] : (int64_t)j;
    if (row < 0 || row >= F->n) return -2;
    float s = (float)(row_dot(F, row, phi) + b);
    if (logit) logit[j] = s;
    prob[j] = (float)sigmoid_d((double)s);
  }
  return 0;
}

int32_t aa_ref_shrink(const float *prob, int32_t P, float gamma, uint64_t seed, uint64_t step,
                      uint8_t *keep, int32_t *kept_pos, int32_t *kept_count) {
  if (P < 0) return -2;
  if (!kept_count) return -1;
  if (P > 0 && (!prob || !kept_pos)) return -1;
  int32_t m = 0;
  const float one_minus_gamma = 1.0f - gamma;
  for (int32_t j = 0; j < P; ++j) {
    float u = aa_ref_uniform(seed, step, (uint32_t)j);
    float p = fmaf(one_minus_gamma, prob[j], gamma); /* gamma + (1-gamma) g, one rounding */
    int k = u < p;
    if (keep) keep[j] = (uint8_t)k;
    if (k) kept_pos[m++] = j;
  }
  *kept_count = m;
  return 0;
}

int32_t aa_ref_shrink_threshold(const float *crit, int32_t P, float T, uint8_t *keep,
                                int32_t *kept_pos, int32_t *kept_count) {
  if (P < 0) return -2;
  if (!kept_count) return -1;
  if (P > 0 && (!crit || !kept_pos)) return -1;
  int32_t m = 0;
  for (int32_t j = 0; j < P; ++j) {
    int k = crit[j] > T;
    if (keep) keep[j] = (uint8_t)k;
    if (k) kept_pos[m++] = j;
  }
  *kept_count = m;
  return 0;
}

/* Keep decision of the sequential generator (Algorithm 1) for one candidate, in double.
 * The unit interval of the draw c is split at gamma: the mass below gamma is the smoothing
 * term and keeps any candidate; the mass above it, stretched back onto [0,1), is a uniform
 * independent of that event and is compared with the Assistant's score g.  Together:
 * P(keep) = gamma + (1 - gamma) g.  gamma == 1 always takes the first case, so the
 * stretch never divides by zero. */
static int sequential_keep(double c, double gamma, double g) {
  if (c < gamma) return 1;
  const double stretched = (c - gamma) / (1.0 - gamma);
  return stretched < g;
}

int32_t aa_ref_sample_batch(const float *prob, int32_t P, float gamma, uint64_t seed,
                            uint64_t step, int32_t batch_size, int32_t *B, int32_t *B_size,
                            int32_t *consumed) {
  if (P < 0 || batch_size < 0) return -2;
  if (!B_size || !consumed) return -1;
  if (P > 0 && batch_size > 0 && (!prob || !B)) return -1;
  /* candidates are visited in pool order until the batch is full or the pool runs out */
  int32_t size = 0, j = 0;
  for (; j < P && size < batch_size; ++j) {
    const double c = (double)aa_ref_uniform(seed, step, (uint32_t)j);
    if (sequential_keep(c, (double)gamma, (double)prob[j])) B[size++] = j;
  }
  *B_size = size;
  *consumed = j;
  return 0;
}

int32_t aa_ref_gather(const void *src, int64_t row_bytes, const int32_t *idx,
                      const int32_t *kept_pos, int32_t m, void *dst, int32_t *kept_ids) {
  if (m < 0 || row_bytes < 0) return -2;
  if (m == 0) return 0;
  if (!kept_pos) return -1;
  if ((src == NULL) != (dst == NULL)) return -1;
  for (int32_t r = 0; r < m; ++r) {
    int64_t id = idx ? (int64_t)idx[kept_pos[r]] : (int64_t)kept_pos[r];
    if (kept_ids) kept_ids[r] = (int32_t)id;
    if (src && row_bytes > 0)
      memcpy((char *)dst + (int64_t)r * row_bytes, (const char *)src + id * row_bytes,
             (size_t)row_bytes);
  }
  return 0;
}

int32_t aa_ref_gather_csr(const aa_ref_features *F, const int32_t *idx, const int32_t *kept_pos,
                          int32_t m, int64_t *out_rowptr, int32_t *out_col, float *out_val,
                          int64_t out_nnz_cap) {
  if (m < 0) return -2;
  if (!F || F->layout != AA_REF_CSR || !F->rowptr) return -2;
  if (!out_rowptr) return -1;
  if (m > 0 && !kept_pos) return -1;
  int64_t fill = 0;
  out_rowptr[0] = 0;
  for (int32_t r = 0; r < m; ++r) {
    int64_t id = idx ? (int64_t)idx[kept_pos[r]] : (int64_t)kept_pos[r];
    if (id < 0 || id >= F->n) return -2;
    for (int64_t e = F->rowptr[id]; e < F->rowptr[id + 1]; ++e) {
      if (fill >= out_nnz_cap) return -2;
      out_col[fill] = F->col[e];
      if (F->val && out_val) out_val[fill] = F->val[e];
      ++fill;
    }
    out_rowptr[r + 1] = fill;
  }
  return 0;
}

int32_t aa_ref_svm_sgd_step(const aa_ref_features *F, const float *y, const int32_t *rows,
                            int32_t m, float *w, float lambda, float lr, float radius,
                            float *loss) {
  if (m < 0) return -2;
  if (m == 0) return 0; /* nothing kept: no update at all, regulariser included */
  if (!features_ok(F)) return F ? -2 : -1;
  if (!y || !w) return -1;
  const int32_t d = F->d;
  double *G = (double *)calloc((size_t)d, sizeof(double));
  if (!G) return -2;
  for (int32_t r = 0; r < m; ++r) {
    int64_t row = rows ? (int64_t)rows[r] : (int64_t)r;
    if (row < 0 || row >= F->n) { free(G); return -2; }
    float margin = (float)((double)y[row] * row_dot(F, row, w)); /* y w.x at the pre-update w */
    if (loss) loss[r] = (float)fmax(0.0, 1.0 - (double)margin);
    if (margin < 1.0f) row_axpy(F, row, (double)y[row], G); /* -subgradient of the hinge */
  }
  const double shrink = 1.0 - (double)lr * (double)lambda;
  const double scale = (double)lr / (double)m;
  for (int32_t k = 0; k < d; ++k) w[k] = (float)(shrink * (double)w[k] + scale * G[k]);
  free(G);
  if (radius > 0.0f) {
    double nrm2 = 0.0;
    for (int32_t k = 0; k < d; ++k) nrm2 += (double)w[k] * (double)w[k];
    double nrm = sqrt(nrm2);
    if (nrm > (double)radius) {
      double f = (double)radius / nrm;
      for (int32_t k = 0; k < d; ++k) w[k] = (float)(f * (double)w[k]);
    }
  }
  return 0;
}

int32_t aa_ref_vanilla_minibatch_sgd(const aa_ref_features *F, const float *y,
                                     const int32_t *idx, int32_t P, float *w, float lambda,
                                     float lr) {
  /* Pegasos mini-batch iteration: A+ = {i in batch : y_i <w, x_i> < 1};
   * w <- (1 - lr*lambda) w + (lr/|batch|) sum_{A+} y_i x_i. */
  if (P < 0) return -2;
  if (P == 0) return 0;
  if (!features_ok(F)) return F ? -2 : -1;
  if (!y || !w) return -1;
  const int32_t d = F->d;
  double *sum = (double *)calloc((size_t)d, sizeof(double));
  if (!sum) return -2;
  for (int32_t j = 0; j < P; ++j) {
    int64_t i = idx ? (int64_t)idx[j] : (int64_t)j;
    double wx = 0.0;
    if (F->layout == AA_REF_DENSE) {
      for (int32_t k = 0; k < d; ++k) wx += (double)w[k] * (double)F->x[i * F->ld + k];
    } else {
      for (int64_t e = F->rowptr[i]; e < F->rowptr[i + 1]; ++e)
        wx += (double)w[F->col[e]] * (F->val ? (double)F->val[e] : 1.0);
    }
    float yi_wx = (float)((double)y[i] * wx);
    if (yi_wx < 1.0f) {
      if (F->layout == AA_REF_DENSE) {
        for (int32_t k = 0; k < d; ++k) sum[k] += (double)y[i] * (double)F->x[i * F->ld + k];
      } else {
        for (int64_t e = F->rowptr[i]; e < F->rowptr[i + 1]; ++e)
          sum[F->col[e]] += (double)y[i] * (F->val ? (double)F->val[e] : 1.0);
      }
    }
  }
  for (int32_t k = 0; k < d; ++k)
    w[k] = (float)((1.0 - (double)lr * (double)lambda) * (double)w[k] +
                   ((double)lr / (double)P) * sum[k]);
  free(sum);
  return 0;
}

int32_t aa_ref_assistant_update(const aa_ref_features *F, const int32_t *rows, int32_t m,
                                const float *loss, float T, float *phi, float *bias,
                                float lr_a, float l2_a) {
  if (m < 0) return -2;
  if (m == 0) return 0;
  if (!features_ok(F)) return F ? -2 : -1;
  if (!loss || !phi) return -1;
  const int32_t d = F->d;
  double *G = (double *)calloc((size_t)d, sizeof(double));
  if (!G) return -2;
  double gb = 0.0;
  const double b = bias ? (double)bias[0] : 0.0;
  for (int32_t r = 0; r < m; ++r) {
    int64_t row = rows ? (int64_t)rows[r] : (int64_t)r;
    if (row < 0 || row >= F->n) { free(G); return -2; }
    double z = loss[r] > T ? 1.0 : 0.0;       /* label: Boss loss above the threshold */
    float s = (float)(row_dot(F, row, phi) + b);
    double q = sigmoid_d((double)s);          /* g at the current phi */
    double resid = q - z;                     /* d(cross-entropy)/d(logit) */
    row_axpy(F, row, resid, G);
    gb += resid;
  }
  for (int32_t k = 0; k < d; ++k)
    phi[k] = (float)((double)phi[k] -
                     (double)lr_a * (G[k] / (double)m + (double)l2_a * (double)phi[k]));
  if (bias) bias[0] = (float)(b - (double)lr_a * gb / (double)m);
  free(G);
  return 0;
}

double aa_ref_primal_objective(const aa_ref_features *F, const float *y, const int32_t *rows,
                               int64_t count, const float *w, float lambda) {
  double nrm2 = 0.0;
  for (int32_t k = 0; k < F->d; ++k) nrm2 += (double)w[k] * (double)w[k];
  double hinge = 0.0;
  for (int64_t r = 0; r < count; ++r) {
    int64_t row = rows ? (int64_t)rows[r] : r;
    hinge += fmax(0.0, 1.0 - (double)y[row] * row_dot(F, row, w));
  }
  return 0.5 * (double)lambda * nrm2 + (count > 0 ? hinge / (double)count : 0.0);
}

double aa_ref_assistant_objective(const aa_ref_features *F, const int32_t *rows, int32_t m,
                                  const uint8_t *z, const float *phi, const float *bias) {
  double total = 0.0;
  const double b = bias ? (double)bias[0] : 0.0;
  for (int32_t r = 0; r < m; ++r) {
    int64_t row = rows ? (int64_t)rows[r] : (int64_t)r;
    double s = row_dot(F, row, phi) + b;
    /* -[z log g + (1-z) log(1-g)] with g = sigmoid(s), written stably:
     * softplus(s) - z s. */
    double softplus = s > 0 ? s + log1p(exp(-s)) : log1p(exp(s));
    total += softplus - (z[r] ? s : 0.0);
  }
  return m > 0 ? total / (double)m : 0.0;
}

int32_t aa_ref_step(const aa_ref_features *F, const float *y, const int32_t *idx, int32_t P,
                    float *w, float *phi, float *bias, float gamma, uint64_t seed,
                    uint64_t step, float lambda, float lr, float T, float lr_a, float l2_a,
                    float *logit, float *prob, uint8_t *keep, int32_t *kept_pos,
                    int32_t *kept_ids, float *loss, int32_t *kept_count) {
  if (P < 0) return -2;
  if (!kept_count) return -1;
  *kept_count = 0;
  if (P == 0) return 0;
  float *prob_l = prob ? prob : (float *)malloc((size_t)P * sizeof(float));
  int32_t *pos_l = kept_pos ? kept_pos : (int32_t *)malloc((size_t)P * sizeof(int32_t));
  int32_t *ids_l = kept_ids ? kept_ids : (int32_t *)malloc((size_t)P * sizeof(int32_t));
  float *loss_l = loss ? loss : (float *)malloc((size_t)P * sizeof(float));
  int32_t rc = -2, m = 0;
  if (!prob_l || !pos_l || !ids_l || !loss_l) goto done;
  rc = aa_ref_assistant_score(F, idx, P, phi, bias, logit, prob_l);
  if (rc) goto done;
  rc = aa_ref_shrink(prob_l, P, gamma, seed, step, keep, pos_l, &m);
  if (rc) goto done;
  rc = aa_ref_gather(NULL, 0, idx, pos_l, m, NULL, ids_l);
  if (rc) goto done;
  /* Boss: forward (losses at the pre-update w), then update. */
  rc = aa_ref_svm_sgd_step(F, y, ids_l, m, w, lambda, lr, 0.0f, loss_l);
  if (rc) goto done;
  /* Assistant learns from the (index, loss) pairs the Boss just produced. */
  rc = aa_ref_assistant_update(F, ids_l, m, loss_l, T, phi, bias, lr_a, l2_a);
  *kept_count = m;
done:
  if (!prob) free(prob_l);
  if (!kept_pos) free(pos_l);
  if (!kept_ids) free(ids_l);
  if (!loss) free(loss_l);
  return rc;
}

int32_t aa_ref_sk_step(const aa_ref_features *F, const float *y, const int32_t *idx, int32_t P,
                       float *w, float lambda, float lr, float T, float *loss_pool,
                       uint8_t *keep, int32_t *kept_pos, int32_t *kept_ids, float *loss,
                       int32_t *kept_count) {
  if (P < 0) return -2;
  if (!kept_count) return -1;
  *kept_count = 0;
  if (P == 0) return 0;
  if (!features_ok(F)) return F ? -2 : -1;
  if (!y || !w) return -1;
  float *crit = loss_pool ? loss_pool : (float *)malloc((size_t)P * sizeof(float));
  int32_t *pos_l = kept_pos ? kept_pos : (int32_t *)malloc((size_t)P * sizeof(int32_t));
  int32_t *ids_l = kept_ids ? kept_ids : (int32_t *)malloc((size_t)P * sizeof(int32_t));
  int32_t rc = -2, m = 0;
  if (!crit || !pos_l || !ids_l) goto done;
  /* the criterion: every candidate's objective value at the current w */
  for (int32_t j = 0; j < P; ++j) {
    int64_t row = idx ? (int64_t)idx[j] : (int64_t)j;
    if (row < 0 || row >= F->n) goto done;
    float margin = (float)((double)y[row] * row_dot(F, row, w));
    crit[j] = (float)fmax(0.0, 1.0 - (double)margin);
  }
  rc = aa_ref_shrink_threshold(crit, P, T, keep, pos_l, &m);
  if (rc) goto done;
  rc = aa_ref_gather(NULL, 0, idx, pos_l, m, NULL, ids_l);
  if (rc) goto done;
  rc = aa_ref_svm_sgd_step(F, y, ids_l, m, w, lambda, lr, 0.0f, loss);
  *kept_count = m;
done:
  if (!loss_pool) free(crit);
  if (!kept_pos) free(pos_l);
  if (!kept_ids) free(ids_l);
  return rc;
}

int32_t aa_ref_sk_sgd(const aa_ref_features *F, const float *y, double *w, double mu, double G,
                      double D, uint64_t seed, int32_t K, const double *w_star, double *dist2,
                      int32_t *picked, int32_t *dropped) {
  if (K < 0) return -2;
  if (!features_ok(F) || F->n <= 0 || F->n > 0x7fffffff) return F ? -2 : -1;
  if (!y || !w) return -1;
  if (!(mu > 0.0)) return -2;
  const int32_t d = F->d;
  double *g = (double *)malloc((size_t)d * sizeof(double));
  if (!g) return -2;
  int32_t n_dropped = 0;
  for (int32_t k = 1; k <= K; ++k) {
    if (w_star && dist2) {
      double s = 0.0;
      for (int32_t c = 0; c < d; ++c) s += (w[c] - w_star[c]) * (w[c] - w_star[c]);
      dist2[k - 1] = s;
    }
    /* i ~ uniform{0..N-1}: second Philox word of counter (k, 0, 0, 0), scaled by N */
    uint32_t ctr[4] = {(uint32_t)k, 0u, 0u, 0u}, out[4];
    uint32_t key[2] = {(uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32)};
    aa_ref_philox4x32_10(ctr, key, out);
    int64_t i = (int64_t)(((uint64_t)out[1] * (uint64_t)F->n) >> 32);
    if (picked) picked[k - 1] = (int32_t)i;
    /* grad f_i(w) with f_i(w) = (mu/2)|w|^2 + max(0, 1 - y_i w.x_i) */
    double wx = 0.0;
    if (F->layout == AA_REF_DENSE) {
      for (int32_t c = 0; c < d; ++c) wx += w[c] * (double)F->x[i * F->ld + c];
    } else {
      for (int64_t e = F->rowptr[i]; e < F->rowptr[i + 1]; ++e)
        wx += w[F->col[e]] * (F->val ? (double)F->val[e] : 1.0);
    }
    for (int32_t c = 0; c < d; ++c) g[c] = mu * w[c];
    if ((double)y[i] * wx < 1.0) row_axpy(F, i, -(double)y[i], g);
    double nrm2 = 0.0;
    for (int32_t c = 0; c < d; ++c) nrm2 += g[c] * g[c];
    if (sqrt(nrm2) <= G / (double)k) { /* epsilon_k = grad f_i: the step is dropped */
      ++n_dropped;
      continue;
    }
    const double eta = 1.0 / (mu * (double)k);
    for (int32_t c = 0; c < d; ++c) w[c] -= eta * g[c];
    if (D > 0.0) {
      double wn2 = 0.0;
      for (int32_t c = 0; c < d; ++c) wn2 += w[c] * w[c];
      if (sqrt(wn2) > D) {
        const double f = D / sqrt(wn2);
        for (int32_t c = 0; c < d; ++c) w[c] *= f;
      }
    }
  }
  if (w_star && dist2) {
    double s = 0.0;
    for (int32_t c = 0; c < d; ++c) s += (w[c] - w_star[c]) * (w[c] - w_star[c]);
    dist2[K] = s;
  }
  if (dropped) *dropped = n_dropped;
  free(g);
  return 0;
}

static int cmp_float(const void *a, const void *b) {
  const float x = *(const float *)a, y = *(const float *)b;
  return (x > y) - (x < y);
}

int32_t aa_ref_threshold_update(const float *loss, int32_t m, float momentum, float *T,
                                int32_t *initialised) {
  if (m < 0) return -2;
  if (!T || !initialised) return -1;
  if (m == 0) return 0;
  if (!loss) return -1;
  for (int32_t i = 0; i < m; ++i) {
    if (loss[i] != loss[i]) { /* a NaN loss has no rank: the threshold becomes NaN, visibly */
      *T = NAN;
      *initialised = 1;
      return 0;
    }
  }
  float *sorted = (float *)malloc((size_t)m * sizeof(float));
  if (!sorted) return -2;
  memcpy(sorted, loss, (size_t)m * sizeof(float));
  qsort(sorted, (size_t)m, sizeof(float), cmp_float);
  float med;
  if (m % 2) {
    med = sorted[m / 2];
  } else {
    const float sum = sorted[m / 2 - 1] + sorted[m / 2];
    med = sum * 0.5f;
  }
  free(sorted);
  if (!*initialised) {
    *T = med;
    *initialised = 1;
  } else {
    const float keep_part = momentum * *T;
    const float one_minus = 1.0f - momentum;
    const float new_part = one_minus * med;
    *T = keep_part + new_part;
  }
  return 0;
}

int32_t aa_ref_bucket_batches(const int32_t *len_s, const int32_t *len_t, int32_t m,
                              int32_t width, int32_t n_buckets, int32_t token_budget,
                              int32_t *order, int32_t *bucket_start, int32_t *batch_of) {
  if (m < 0 || width <= 0 || n_buckets <= 0 || token_budget <= 0) return -2;
  if (!bucket_start) return -1;
  if (m > 0 && (!len_s || !len_t || !order || !batch_of)) return -1;
  for (int32_t b = 0; b <= n_buckets; ++b) bucket_start[b] = 0;
  for (int32_t r = 0; r < m; ++r) {
    int32_t L = len_s[r] > len_t[r] ? len_s[r] : len_t[r];
    int32_t b = (L - 1) / width;
    if (b < 0) b = 0;
    if (b > n_buckets - 1) b = n_buckets - 1;
    bucket_start[b + 1] += 1;
  }
  for (int32_t b = 0; b < n_buckets; ++b) bucket_start[b + 1] += bucket_start[b];
  int32_t *fill = (int32_t *)calloc((size_t)n_buckets, sizeof(int32_t));
  if (!fill) return -2;
  for (int32_t r = 0; r < m; ++r) {
    int32_t L = len_s[r] > len_t[r] ? len_s[r] : len_t[r];
    int32_t b = (L - 1) / width;
    if (b < 0) b = 0;
    if (b > n_buckets - 1) b = n_buckets - 1;
    order[bucket_start[b] + fill[b]++] = r;
  }
  free(fill);
  int32_t batches = 0;
  for (int32_t b = 0; b < n_buckets; ++b) {
    int32_t cap = token_budget / (2 * width * (b + 1));
    if (cap < 1) cap = 1;
    int32_t count = bucket_start[b + 1] - bucket_start[b];
    for (int32_t q = 0; q < count; ++q) batch_of[bucket_start[b] + q] = batches + q / cap;
    batches += (count + cap - 1) / cap;
  }
  return batches;
}
