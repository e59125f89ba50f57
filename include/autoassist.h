/*
 * autoassist.h -- C ABI of the MI355X (gfx950) AutoAssist hot path.
 *
 * Method: "AutoAssist: A Framework to Accelerate Training of Deep Neural
 * Networks" (arXiv 1905.03381).  A light Assistant g(x; phi) (logistic
 * regression) scores a pool of candidate instances, each candidate is kept by
 * a Bernoulli draw with probability gamma + (1-gamma) g (Algorithm 1), the
 * survivors are compacted in arrival order and gathered, the Boss (here the
 * hinge-loss linear SVM of Section 3) takes its SGD step on the kept rows only
 * (eq. "shrinking_grad"), and the Boss's per-instance losses label the
 * Assistant's own SGD update (Section 5.2 objective, Algorithms 2 and 3).
 *
 * Conventions
 *  - Every function returns an int32_t status (AA_OK or a negative AA_ERR_*).
 *    Argument errors are reported synchronously; nothing is launched then.
 *  - Unless said otherwise every data pointer is a DEVICE pointer owned by the
 *    caller; the library never allocates, frees or keeps them.
 *  - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All
 *    calls are asynchronous on it and never synchronise with the host.
 *  - Counts produced on the device (the kept count m) are passed on as device
 *    pointers plus a host upper bound.
 *  - `ws` is caller-provided device scratch of at least
 *    aa_workspace_bytes(P_max, d_max) bytes, 256-byte aligned, prepared once
 *    with aa_workspace_init().  A workspace must not be used by two calls that
 *    may overlap in time (different streams).  Keep flags are bytes 0 or 1.
 *  - Row ids are int32, CSR row pointers int64, column ids int32, values fp32.
 *    PRECONDITION: every row id handed over (idx, perm, rows, kept_pos) lies in
 *    [0, n) of the data it indexes and every CSR column id in [0, d).  Ids are
 *    not checked on the device: an id outside the range reads (or, for column
 *    ids of a gradient pass, writes) outside the caller's buffers.
 *  - P == 0 and *m == 0 are valid and leave the model state untouched.
 *  - Reproducibility: the same call on the same inputs gives the same bits.  The
 *    register-resident dense kernels add in a fixed order.  The CSR / general
 *    kernels add the fp32 terms of a column in doubles and round the total
 *    once, so the order in which waves arrive does not show -- unless the terms
 *    of one column span more than about 2^17 in magnitude, where a double sum
 *    can round and the last fp32 bit may then differ from run to run.
 */
#ifndef AUTOASSIST_H
#define AUTOASSIST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AA_OK 0
#define AA_ERR_NULL (-1)      /* a required pointer is NULL */
#define AA_ERR_SHAPE (-2)     /* negative size, ld < d, unknown layout, ... */
#define AA_ERR_ALIGN (-3)     /* a pointer that must be aligned is not */
#define AA_ERR_WORKSPACE (-4) /* ws is NULL, misaligned or too small */
#define AA_ERR_HIP (-5)       /* the HIP runtime reported a launch error */

#define AA_DENSE 0
#define AA_CSR 1

/* The feature side of the training set D = {x_i, y_i} (Algorithm 1, input).
 * Dense: x is row-major [n, ld] with ld >= d (elements).  The fast kernels need
 * x 16-byte aligned, ld % 4 == 0, d % 4 == 0 and d <= 2048; anything else runs
 * on slower general kernels, not an error.
 * CSR: rowptr[n+1], col[nnz], val[nnz]; val == NULL means every stored entry
 * is 1 (token lists).  Duplicate column ids within a row are allowed and add.
 * Exactly one of the two layouts is read, chosen by `layout`. */
typedef struct aa_features {
  int32_t layout; /* AA_DENSE or AA_CSR */
  int32_t d;      /* feature dimension */
  int64_t n;      /* rows in the data set */
  const float *x; /* dense values (device) */
  int64_t ld;     /* dense leading dimension in elements */
  const int64_t *rowptr;
  const int32_t *col;
  const float *val;
} aa_features;

/* Scalars of one whole step (see aa_fused_step). */
typedef struct aa_step_config {
  float gamma;     /* smoothing term / base probability of Algorithm 1 */
  float lambda;    /* L2 regularisation of the SVM objective */
  float lr;        /* Boss step size eta for this step */
  float lr_a;      /* Assistant step size */
  float l2_a;      /* Assistant L2 regularisation (0 in the paper) */
  int32_t reserved;
  uint64_t seed;   /* Philox key */
  uint64_t step;   /* Philox counter high words: one value per pool */
  const float *T;  /* device scalar: shrinking threshold on the Boss loss */
} aa_step_config;

int32_t aa_version(void);
const char *aa_status_string(int32_t status);

/* Bytes of scratch needed by any call with pool size <= P_max and feature
 * dimension <= d_max: a few MB for the dense layouts; for CSR rows (and dense
 * rows with d > 2048) about 24 d + 790 P_max bytes plus 16 MB (gradient
 * accumulators, model pairs, per-block partial sums and the bins that sort sparse
 * gradient terms by column, at most 2 GiB of those). */
size_t aa_workspace_bytes(int32_t P_max, int32_t d_max);

/* Zero the control words of a fresh workspace (one small fill kernel). */
int32_t aa_workspace_init(void *ws, size_t ws_bytes, void *stream);

/* Measurement aid: arm a one-shot hook so that the NEXT row-pass kernel launched by
 * this library (the kernel that streams the feature rows, in whichever entry
 * point launches it) hands its own start and stop time stamps to the two events
 * (hipExtLaunchKernel with start and stop events, on the call's stream), so that
 * hipEventElapsedTime(event_before, event_after) is the kernel's duration.  Both
 * are hipEvent_t handles created with timing enabled, owned by the caller, passed
 * as void*.  Two NULLs disarm.  Not for calls under stream capture.  Host state
 * only, not thread safe. */
int32_t aa_profile_hook(void *event_before, void *event_after);

/* The same for the next `count` row-pass launches, pair i around the i-th of
 * them (e.g. every step of one aa_train_epoch call).  The two arrays are host
 * arrays of hipEvent_t handles that must stay valid until those launches have
 * been issued.  count == 0 disarms. */
int32_t aa_profile_hooks(void *const *events_before, void *const *events_after, int32_t count);

/* ---- a1: Assistant score (Section 5.2: g(x_i; phi); Algorithm 1 evaluates it
 * once per drawn candidate).  For pool position j in [0, P):
 *   logit[j] = phi . x_{idx[j]} + *bias,   prob[j] = 1 / (1 + exp(-logit[j])).
 * idx == NULL means rows 0..P-1.  bias == NULL means 0.  logit may be NULL.
 * Reads: F, idx[P], phi[d], bias[1].  Writes: logit[P], prob[P]. */
int32_t aa_assistant_score(const aa_features *F, const int32_t *idx, int32_t P,
                           const float *phi, const float *bias, float *logit, float *prob,
                           void *stream);

/* ---- a2 + a3: Bernoulli keep and stable compaction (Algorithm 1).
 *   u_j  = Philox4x32-10(counter = (j, 0, lo32(step), hi32(step)),
 *                        key = (lo32(seed), hi32(seed)))[0] >> 8, times 2^-24
 *   keep[j] = u_j < fmaf(1 - gamma, prob[j], gamma)
 *   kept_pos = positions j with keep[j], increasing; *kept_count = their number.
 * keep may be NULL.  kept_pos must hold P entries; entries past *kept_count
 * are left untouched. */
int32_t aa_shrink(const float *prob, int32_t P, float gamma, uint64_t seed, uint64_t step,
                  uint8_t *keep, int32_t *kept_pos, int32_t *kept_count, void *ws,
                  size_t ws_bytes, void *stream);

/* ---- a7: a1 + a2 fused in the row pass (score and keep draw from registers, so
 * each feature row crosses HBM once), then the compaction of a3 over the flags.
 * Same outputs as aa_assistant_score followed by aa_shrink. */
int32_t aa_score_shrink(const aa_features *F, const int32_t *idx, int32_t P, const float *phi,
                        const float *bias, float gamma, uint64_t seed, uint64_t step,
                        float *logit, float *prob, uint8_t *keep, int32_t *kept_pos,
                        int32_t *kept_count, void *ws, size_t ws_bytes, void *stream);

/* Hard-threshold shrinking (eq. "shrinking_grad"; SK of Section 3.4 with the
 * objective value as criterion): keep[j] = crit[j] > *T, then the same stable
 * compaction.  T is a device scalar. */
int32_t aa_shrink_threshold(const float *crit, int32_t P, const float *T, uint8_t *keep,
                            int32_t *kept_pos, int32_t *kept_count, void *ws, size_t ws_bytes,
                            void *stream);

/* ---- a4: batch assembly (the BossQueue holds {x_i, y_i} of the batch,
 * Section 5.3).  For r < *kept_count (at most max_rows):
 *   id_r = idx[kept_pos[r]]  (idx == NULL: id_r = kept_pos[r])
 *   dst[r, 0:row_bytes] = src[id_r, 0:row_bytes],   kept_ids[r] = id_r.
 * row_bytes is arbitrary; 16-byte aligned rows take a 128-bit path.  src and
 * dst may both be NULL (ids only); kept_ids may be NULL.  kept_pos == NULL
 * means kept_pos[r] = r. */
int32_t aa_gather(const void *src, int64_t row_bytes, const int32_t *idx,
                  const int32_t *kept_pos, const int32_t *kept_count, int32_t max_rows,
                  void *dst, int32_t *kept_ids, void *stream);

/* CSR batch assembly: out_rowptr[0..m], out_col/out_val hold the kept rows in
 * order.  Rows that would not fit in out_nnz_cap entries are not copied, but
 * out_rowptr is always complete: the caller checks out_rowptr[m] <= cap.
 * out_val may be NULL iff F->val is NULL.  ws (sized for P_max >= max_rows) is
 * needed when max_rows > 1024: AA_ERR_WORKSPACE otherwise. */
int32_t aa_gather_csr(const aa_features *F, const int32_t *idx, const int32_t *kept_pos,
                      const int32_t *kept_count, int32_t max_rows, int64_t *out_rowptr,
                      int32_t *out_col, float *out_val, int64_t out_nnz_cap, void *ws,
                      size_t ws_bytes, void *stream);

/* ---- a5: one mini-batch SGD step of the L2-regularised hinge objective
 *   (lambda/2)|w|^2 + (1/N) sum max(0, 1 - y_i w.x_i)     (Section 3.1 loss,
 * Pegasos scaling) on the m = *m_dev kept rows (m <= m_max):
 *   loss[r] = max(0, 1 - y w.x) at the PRE-update w (Algorithm 3: forward,
 *             send losses, then update);
 *   w <- (1 - lr*lambda) w + (lr/m) sum_{r: y w.x < 1} y_r x_r;
 *   radius > 0: afterwards w <- w * min(1, radius/|w|).
 * rows[r] are data-set row ids (rows == NULL: row r); y is indexed like the
 * rows.  m == 0: w is left as it is.  loss may be NULL. */
int32_t aa_svm_sgd_step(const aa_features *F, const float *y, const int32_t *rows,
                        const int32_t *m_dev, int32_t m_max, float *w, float lambda, float lr,
                        float radius, float *loss, void *ws, size_t ws_bytes, void *stream);

/* ---- a6: Assistant SGD step on the mean cross-entropy with labels
 *   z_r = loss[r] > *T        (Section 5.2: z_i = 1 iff f(x_i, y_i, theta) > T)
 *   q_r = sigmoid(phi . x_r + b) at the current phi
 *   phi <- phi - lr_a ((1/m) sum (q_r - z_r) x_r + l2_a phi)
 *   b   <- b   - lr_a  (1/m) sum (q_r - z_r)            (bias may be NULL)
 * T is a device scalar.  m == 0: nothing changes. */
int32_t aa_assistant_update(const aa_features *F, const int32_t *rows, const int32_t *m_dev,
                            int32_t m_max, const float *loss, const float *T, float *phi,
                            float *bias, float lr_a, float l2_a, void *ws, size_t ws_bytes,
                            void *stream);

/* a5 + a6 in one pass over the kept rows (the Assistant shares the Boss's
 * features): same results as aa_svm_sgd_step followed by aa_assistant_update
 * with the losses it wrote. */
int32_t aa_boss_assistant_step(const aa_features *F, const float *y, const int32_t *rows,
                               const int32_t *m_dev, int32_t m_max, float *w, float *phi,
                               float *bias, const aa_step_config *cfg, float *loss, void *ws,
                               size_t ws_bytes, void *stream);

/* ---- Batch-generator helpers (neither is in the paper; both are this
 * library's definitions, mirrored by the CPU reference used in the tests).
 *
 * Running-median shrinking threshold ("Boss loss above the running median" as
 * the label of the image batch generator): med = median of loss[0..m-1]
 * (m = min(*m_dev, m_max) <= 16384; mean of the two middle values for even m);
 * the first call (*initialised == 0) sets *T = med and *initialised = 1, later
 * calls *T = momentum * *T + (1 - momentum) * med, every operation rounded to
 * fp32.  m == 0 changes nothing.  A batch that holds a NaN loss sets *T to NaN
 * (and *initialised to 1).  T and initialised are device scalars. */
int32_t aa_threshold_update(const float *loss, const int32_t *m_dev, int32_t m_max, float momentum,
                            float *T, int32_t *initialised, void *stream);

/* The per-batch Assistant step of that generator (Sec. 5.2: the label of a kept
 * instance is "Boss loss above the threshold", here the running median) in one
 * call: the same results, bit for bit, as aa_threshold_update(loss, m_dev,
 * m_max, momentum, T, initialised) followed by aa_assistant_update(F, rows,
 * m_dev, m_max, loss, T, phi, bias, lr_a, l2_a), i.e. the labels are taken
 * against the threshold AFTER this batch's median went into it.  Dense rows in a
 * register layout and m_max <= 512 run as one pass and one update launch (every
 * block of the pass works the new threshold out for itself); anything else
 * runs the two calls it stands for.  T and initialised are device scalars,
 * read during the pass and written by the update launch; workspace as for
 * aa_assistant_update.  Errors: AA_ERR_SHAPE (m_max < 0 or > 16384, momentum
 * outside [0, 1]), AA_ERR_NULL, AA_ERR_WORKSPACE, AA_ERR_HIP. */
int32_t aa_threshold_assistant_update(const aa_features *F, const int32_t *rows, const int32_t *m_dev,
                                      int32_t m_max, const float *loss, float momentum, float *T,
                                      int32_t *initialised, float *phi, float *bias, float lr_a,
                                      float l2_a, void *ws, size_t ws_bytes, void *stream);

/* Length-bucketed batching of m kept sentence pairs (translation batch
 * generator): bucket(r) = min(n_buckets - 1, (max(len_s[r], len_t[r]) - 1) / width),
 * n_buckets <= 32.  order[] lists r grouped by bucket, arrival order kept inside
 * a bucket (stable); bucket_start[n_buckets + 1] are the group boundaries;
 * batch_of[q] is the batch number of order[q], batches being consecutive runs of
 * cap_b = max(1, token_budget / (2 * width * (b + 1))) pairs inside bucket b
 * (padded-token budget), numbered bucket after bucket; *n_batches their count.
 * len_s / len_t are indexed by r (gather them with aa_gather first). */
int32_t aa_bucket_batches(const int32_t *len_s, const int32_t *len_t, const int32_t *m_dev,
                          int32_t m_max, int32_t width, int32_t n_buckets, int32_t token_budget,
                          int32_t *order, int32_t *bucket_start, int32_t *batch_of,
                          int32_t *n_batches, void *ws, size_t ws_bytes, void *stream);

/* ---- The whole step a1..a6 with every feature row read once: score, keep,
 * compact, gather ids, SVM step on the kept rows, Assistant update labelled
 * by the pre-update losses.  Outputs as in the staged calls: logit[P],
 * prob[P], keep[P], kept_pos[<=P], kept_ids[<=P], loss[<=P] (loss[r] belongs
 * to kept_ids[r]), *kept_count.  logit, prob, keep, kept_pos, kept_ids and loss
 * may be NULL. */
int32_t aa_fused_step(const aa_features *F, const float *y, const int32_t *idx, int32_t P,
                      float *w, float *phi, float *bias, const aa_step_config *cfg,
                      float *logit, float *prob, uint8_t *keep, int32_t *kept_pos,
                      int32_t *kept_ids, float *loss, int32_t *kept_count, void *ws,
                      size_t ws_bytes, void *stream);

/* ---- aa_fused_step for callers that cannot allocate device memory or carry a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, outputs and errors as aa_fused_step minus
 * `ws` / `ws_bytes`: the scratch (block partials of the gradient sums, per-block
 * kept counts, keep flags and per-position losses when the caller passes none)
 * lives in a static device array of AA_STATIC_SCRATCH_BYTES inside the library,
 * one copy per GPU, held until the process ends.  The call allocates nothing and
 * frees nothing.  A step that needs more scratch than the array holds
 * (aa_workspace_bytes-sized needs of large CSR problems, say) is refused with
 * AA_ERR_WORKSPACE and launches nothing; the register-resident dense layouts fit
 * for any d <= 2048 and P <= 131072.  The first call on a device looks up that
 * device's copy of the array (make it outside stream capture).  All calls on one
 * GPU share the array: two calls that may overlap in time on one GPU (different
 * streams) race; calls on one stream are ordered and safe.  Nothing in the array
 * has to survive between calls. */
#define AA_STATIC_SCRATCH_BYTES (8u << 20)
size_t aa_static_scratch_bytes(void);
int32_t aa_fused_step_static(const aa_features *F, const float *y, const int32_t *idx, int32_t P,
                             float *w, float *phi, float *bias, const aa_step_config *cfg,
                             float *logit, float *prob, uint8_t *keep, int32_t *kept_pos,
                             int32_t *kept_ids, float *loss, int32_t *kept_count, void *stream);

/* ---- Hard-threshold shrinking (SK of Section 3.4; the update of eq.
 * "shrinking_grad" with the objective value as the criterion), one step on the
 * pool idx[0..P-1] with every feature row read once: crit_j = max(0, 1 - y w.x)
 * of candidate j at the current w; keep_j = (crit_j > *T); stable compaction;
 * w <- (1 - lr*lambda) w + (lr/m) sum over kept rows with margin < 1 of y x;
 * m == 0 changes nothing.  No Assistant takes part.  T: device scalar.
 * Outputs: loss_pool[P] = crit (may be NULL), keep[P] (may be NULL),
 * kept_pos[<=P], kept_ids[<=P], loss[<=P] = crit of the kept rows in kept order
 * (each may be NULL), *kept_count (device, required).  Errors as aa_fused_step. */
int32_t aa_sk_step(const aa_features *F, const float *y, const int32_t *idx, int32_t P, float *w,
                   const float *T, float lambda, float lr, float *loss_pool, uint8_t *keep,
                   int32_t *kept_pos, int32_t *kept_ids, float *loss, int32_t *kept_count,
                   void *ws, size_t ws_bytes, void *stream);

/* One epoch of fused steps: pool t is perm[t*P : min((t+1)*P, n_perm)] (the
 * shuffled index list that replaces uniform sampling, Section 5.2), Philox
 * step = cfg->step + t, Boss step size lr_t = cfg->lr / sqrt(t_upd) where
 * *t_upd (device counter, incremented by each step with m > 0) counts the
 * updates made so far including this one; t_upd == NULL keeps lr constant.
 * kept_hist[t] (device, may be NULL) receives each step's kept count.  Each
 * step assembles its batch (keep probabilities, keep flags, kept positions,
 * kept ids, per-instance losses): the kept ids of step t go to
 * kept_ids_hist[t*P ..] and their losses to loss_hist[t*P ..] (kept_hist[t]
 * entries each; either may be NULL: the batch then lives in ws until the next
 * step replaces it).  With the fast dense layout the compaction of step t is
 * carried by the row pass of step t+1 (every output is complete when the
 * call's work has drained).  Every layout takes t_upd. */
int32_t aa_train_epoch(const aa_features *F, const float *y, const int32_t *perm,
                       int64_t n_perm, int32_t P, float *w, float *phi, float *bias,
                       const aa_step_config *cfg, int32_t *t_upd, int32_t *kept_hist,
                       int32_t *kept_ids_hist, float *loss_hist, void *ws, size_t ws_bytes,
                       void *stream);

/* One epoch of hard-threshold shrinking steps: aa_sk_step on pool t =
 * perm[t*P : min((t+1)*P, n_perm)] for every t, with the step size
 * lr_t = lr0 / sqrt(t_upd) kept on the device as in aa_train_epoch (t_upd ==
 * NULL: lr0 throughout), kept counts in kept_hist[t], and the kept ids and
 * losses of step t in kept_ids_hist[t*P ..] / loss_hist[t*P ..] (each may be
 * NULL).  T: device scalar. */
int32_t aa_sk_epoch(const aa_features *F, const float *y, const int32_t *perm, int64_t n_perm,
                    int32_t P, float *w, const float *T, float lambda, float lr0, int32_t *t_upd,
                    int32_t *kept_hist, int32_t *kept_ids_hist, float *loss_hist, void *ws,
                    size_t ws_bytes, void *stream);

/* ---- The asynchronous Boss / Assistant schedule of Section 5.3 in a deterministic
 * form, on two streams.  Pool s is perm[s*P : min((s+1)*P, n_perm)].  The
 * generator (stream_gen) makes batch s -- score, keep draw with Philox step
 * cfg->step + s, stable compaction to kept ids -- with the Assistant as it stood
 * after max(0, s - staleness) updates, so `staleness` batches wait in the Boss
 * queue while the Assistant keeps learning.  The Boss (stream_boss), tick s: SVM
 * step on batch s (losses at the pre-update w, lr_t = cfg->lr / sqrt(t_upd) as in
 * aa_train_epoch), then the Assistant update from those losses at its current
 * parameters.  Generation of batch s + staleness overlaps Boss tick s; events
 * order the two streams, the result does not depend on timing.  staleness = 0 is
 * the synchronous schedule (the generator then waits for every Boss tick).
 * On return all work is enqueued; the last Boss tick waits for every generator
 * launch, so synchronising stream_boss is enough.  The caller makes its inputs
 * visible to stream_boss; stream_gen must be a different stream with no
 * unrelated work pending.  0 <= staleness <= 15.
 * kept_hist[steps] (may be NULL): kept count of each tick.  kept_ids_hist
 * [steps][P] (may be NULL): the kept ids of each batch, row s holding
 * kept_hist[s] entries.  ws must hold aa_pipeline_workspace_bytes(P, d,
 * staleness) bytes. */
size_t aa_pipeline_workspace_bytes(int32_t P_max, int32_t d_max, int32_t staleness);
int32_t aa_train_epoch_stale(const aa_features *F, const float *y, const int32_t *perm,
                             int64_t n_perm, int32_t P, int32_t staleness, float *w, float *phi,
                             float *bias, const aa_step_config *cfg, int32_t *t_upd,
                             int32_t *kept_hist, int32_t *kept_ids_hist, void *ws,
                             size_t ws_bytes, void *stream_boss, void *stream_gen);

#ifdef __cplusplus
}
#endif
#endif
