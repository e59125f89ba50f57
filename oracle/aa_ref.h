/*
 * aa_ref.h -- CPU oracle for the AutoAssist shrink + SGD path (arXiv 1905.03381).
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, single-threaded reference
 * that defines what the GPU library must compute.  It shares no code, header,
 * table or helper with the HIP path; only tests, the smoke check and the
 * benchmark's cpu_baseline leg may load it.  Never route product calls here.
 *
 * All pointers are HOST pointers owned by the caller.  Floating-point sums are
 * accumulated in double, in index order, and rounded once to float where a
 * float is stored.  Functions return 0 on success, a negative code on a bad
 * argument (-1 null pointer, -2 bad shape).
 *
 * Parity status: every function below is pinned by tests against something
 * other than itself (published Philox known-answer vectors, closed forms,
 * library routines, brute force).  Two helpers are not in the paper and are
 * this build's definitions: aa_ref_bucket_batches (parity unpinned beyond
 * brute force of its own definition) and aa_ref_threshold_update (its median is
 * pinned against numpy's; the momentum rule is parity unpinned).
 */
#ifndef AA_REF_H
#define AA_REF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AA_REF_DENSE 0
#define AA_REF_CSR 1

/* Feature matrix of the data set D = {x_i, y_i} (Section 5.2, Algorithm 1 input).
 * Dense: row-major x[n, ld], ld >= d.  CSR: rowptr[n+1], col[nnz], val[nnz];
 * val == NULL means every stored entry is 1 (bag-of-tokens lists). */
typedef struct {
  int32_t layout;
  int32_t d;
  int64_t n;
  const float *x;
  int64_t ld;
  const int64_t *rowptr;
  const int32_t *col;
  const float *val;
} aa_ref_features;

/* Philox4x32-10 block function (Salmon, Moraes, Dror, Shaw, SC'11). */
void aa_ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* The uniform c ~ U[0,1) of Algorithm 1 for pool position j at step `step`:
 * counter (j, 0, lo(step), hi(step)), key (lo(seed), hi(seed)),
 * u = (out[0] >> 8) * 2^-24. */
float aa_ref_uniform(uint64_t seed, uint64_t step, uint32_t j);

/* Assistant g(x; phi) = sigmoid(phi . x + b) on P candidates (objective of
 * Section 5.2; Algorithm 1 evaluates g per drawn candidate).
 * idx == NULL means rows 0..P-1.  bias == NULL means 0.  logit may be NULL. */
int32_t aa_ref_assistant_score(const aa_ref_features *F, const int32_t *idx, int32_t P,
                               const float *phi, const float *bias, float *logit, float *prob);

/* Bernoulli keep with smoothing term gamma and stable compaction
 * (Algorithm 1): p = fmaf(1-gamma, g, gamma) in float, keep = (u < p).
 * keep may be NULL.  kept_pos has capacity P. */
int32_t aa_ref_shrink(const float *prob, int32_t P, float gamma, uint64_t seed, uint64_t step,
                      uint8_t *keep, int32_t *kept_pos, int32_t *kept_count);

/* Hard-threshold shrinking (eq. "shrinking_grad", SK in Section 3.4 with the
 * objective value as criterion): keep_j = (crit_j > T). */
int32_t aa_ref_shrink_threshold(const float *crit, int32_t P, float T, uint8_t *keep,
                                int32_t *kept_pos, int32_t *kept_count);

/* The sequential batch generator of Algorithm 1 over a candidate sequence of
 * length P: candidates are visited in order and the batch is full after
 * batch_size keeps.  A candidate is kept when its draw c falls into the smoothing
 * mass [0, gamma), or when the rest of the draw, stretched from [gamma, 1) onto
 * [0, 1), falls below the Assistant's score g.  Double arithmetic.  B receives
 * pool positions; *consumed the number of candidates looked at. */
int32_t aa_ref_sample_batch(const float *prob, int32_t P, float gamma, uint64_t seed,
                            uint64_t step, int32_t batch_size, int32_t *B, int32_t *B_size,
                            int32_t *consumed);

/* Batch assembly: dst[r,:] = src[id_r,:], id_r = idx[kept_pos[r]] (idx NULL:
 * id_r = kept_pos[r]).  kept_ids may be NULL, dst/src may be NULL together. */
int32_t aa_ref_gather(const void *src, int64_t row_bytes, const int32_t *idx,
                      const int32_t *kept_pos, int32_t m, void *dst, int32_t *kept_ids);

/* CSR batch assembly.  out_rowptr[m+1]; out_col/out_val capacity out_nnz_cap.
 * Returns -2 if the kept rows do not fit.  out_val may be NULL iff F->val is. */
int32_t aa_ref_gather_csr(const aa_ref_features *F, const int32_t *idx, const int32_t *kept_pos,
                          int32_t m, int64_t *out_rowptr, int32_t *out_col, float *out_val,
                          int64_t out_nnz_cap);

/* One mini-batch SGD step of the L2-regularised hinge objective
 * (lambda/2)|w|^2 + mean hinge (Section 3.1 loss, Pegasos scaling) on the m
 * kept rows.  rows == NULL: rows 0..m-1.  y is indexed like the rows.
 * loss[r] is the hinge loss at the PRE-update w (Algorithm 3 order).
 * m == 0: nothing changes.  radius > 0: project onto the ball afterwards. */
int32_t aa_ref_svm_sgd_step(const aa_ref_features *F, const float *y, const int32_t *rows,
                            int32_t m, float *w, float lambda, float lr, float radius,
                            float *loss);

/* Plain Pegasos-style mini-batch SGD over rows idx[0..P-1] with no shrinking,
 * written separately from aa_ref_svm_sgd_step (the baseline of Section 3.4). */
int32_t aa_ref_vanilla_minibatch_sgd(const aa_ref_features *F, const float *y,
                                     const int32_t *idx, int32_t P, float *w, float lambda,
                                     float lr);

/* Assistant SGD step on mean cross-entropy with labels z_r = (loss_r > T)
 * (objective and label definition of Section 5.2). */
int32_t aa_ref_assistant_update(const aa_ref_features *F, const int32_t *rows, int32_t m,
                                const float *loss, float T, float *phi, float *bias,
                                float lr_a, float l2_a);

/* (lambda/2)|w|^2 + (1/count) sum hinge over rows (NULL: 0..count-1). */
double aa_ref_primal_objective(const aa_ref_features *F, const float *y, const int32_t *rows,
                               int64_t count, const float *w, float lambda);

/* Mean cross-entropy of the Assistant on rows with labels z (0/1). */
double aa_ref_assistant_objective(const aa_ref_features *F, const int32_t *rows, int32_t m,
                                  const uint8_t *z, const float *phi, const float *bias);

/* One synchronous step of the whole path on pool idx[0..P-1]:
 * score -> keep -> compact -> gather ids -> SVM step on kept rows -> Assistant
 * update labelled by the pre-update losses.  Outputs (any may be NULL except
 * kept_count): logit[P], prob[P], keep[P], kept_pos[P], kept_ids[P], loss[P]. */
int32_t aa_ref_step(const aa_ref_features *F, const float *y, const int32_t *idx, int32_t P,
                    float *w, float *phi, float *bias, float gamma, uint64_t seed,
                    uint64_t step, float lambda, float lr, float T, float lr_a, float l2_a,
                    float *logit, float *prob, uint8_t *keep, int32_t *kept_pos,
                    int32_t *kept_ids, float *loss, int32_t *kept_count);

/* One step of hard-threshold shrinking (SK of Section 3.4; the update of eq.
 * "shrinking_grad" with the objective value as the criterion) on pool
 * idx[0..P-1]: crit_j = hinge loss of candidate j at the current w,
 * keep_j = (crit_j > T), stable compaction, then the SVM step on the kept rows.
 * Outputs (any may be NULL except kept_count): loss_pool[P] = crit, keep[P],
 * kept_pos[P], kept_ids[P], loss[P] (kept rows, pre-update). */
int32_t aa_ref_sk_step(const aa_ref_features *F, const float *y, const int32_t *idx, int32_t P,
                       float *w, float lambda, float lr, float T, float *loss_pool,
                       uint8_t *keep, int32_t *kept_pos, int32_t *kept_ids, float *loss,
                       int32_t *kept_count);

/* The iteration Theorem 1 (Section 4) is stated for, in double: K single-instance
 * steps on f_i(w) = (mu/2)|w|^2 + max(0, 1 - y_i w.x_i), step size 1/(mu k),
 * i_k uniform on the rows; step k is dropped when |grad f_i(w_k)| <= G/k.
 * D > 0 projects onto the ball of radius D after every step (the boundedness
 * assumption of the theorem, as in Pegasos); D = 0: no projection.
 * i_k = (word 1 of Philox(counter (k,0,0,0), key seed) * N) >> 32, k = 1..K.
 * Optional outputs: dist2[K+1] (|w_k - w_star|^2 for k = 1..K+1, needs
 * w_star), picked[K] (the i_k), *dropped (number of dropped steps). */
int32_t aa_ref_sk_sgd(const aa_ref_features *F, const float *y, double *w, double mu, double G,
                      double D, uint64_t seed, int32_t K, const double *w_star, double *dist2,
                      int32_t *picked, int32_t *dropped);

/* Running-median shrinking threshold for the image batch generator ("loss above
 * the running median"): med = median of loss[0..m-1] (mean of the two middle
 * values for even m, in float); the first call sets *T = med, later calls
 * *T = momentum * *T + (1 - momentum) * med, each product and the sum rounded
 * to float.  m == 0 changes nothing.  This estimator is this build's reading
 * (the paper gives no estimator); it is pinned against numpy's median.  A batch that holds a NaN loss sets *T to NaN
 * (and *initialised to 1). */
int32_t aa_ref_threshold_update(const float *loss, int32_t m, float momentum, float *T,
                                int32_t *initialised);

/* Length-bucketed batching of kept sentence pairs (translation batch
 * generator).  bucket_r = min(n_buckets-1, (max(len_s,len_t)-1)/width);
 * within a bucket, pairs keep arrival order and batch number = rank / cap_b
 * with cap_b = max(1, token_budget / (2*width*(b+1))).  Output: order[m] lists r
 * grouped by bucket then rank; bucket_start[n_buckets+1]; batch_of[m] is the
 * global batch number of order[q].  Returns number of batches (>= 0). */
int32_t aa_ref_bucket_batches(const int32_t *len_s, const int32_t *len_t, int32_t m,
                              int32_t width, int32_t n_buckets, int32_t token_budget,
                              int32_t *order, int32_t *bucket_start, int32_t *batch_of);

#ifdef __cplusplus
}
#endif
#endif
