// Host-side launch interface of the dense register-resident row passes.
#pragma once

#include "aa_common.hpp"
#include "aa_compact.hpp"

namespace aa {

enum : int { kSvm = 1, kAssist = 2, kPool = 4, kHard = 8 };

// One pass over feature rows.  In pool mode (kPool) the pass walks the candidate
// pool: score, keep draw and -- with kSvm|kAssist -- both gradient sums of the
// kept rows.  Without kPool it walks rows already chosen (kept ids).
// kPool|kSvm|kHard is the hard-threshold pool pass: no Assistant, a candidate is
// kept when its own hinge loss at the current w exceeds *T.
struct PassArgs {
  const float *x;
  int64_t ld;
  int32_t d4;             // d / 4
  const float *y;         // labels indexed by data-set row (kSvm)
  const int32_t *rows;    // pool ids idx[P] or kept ids rows[m]; NULL = 0..count-1
  int32_t count_max;      // P (pool) or m_max (kept)
  const int32_t *m_dev;   // device row count for kept mode (NULL in pool mode)
  const float *w;
  const float *phi;
  const float *bias;      // device scalar or NULL
  const float *T;         // device scalar (kAssist, kHard)
  float gamma, one_minus_gamma;
  DrawKey key;
  int32_t do_keep;        // pool mode: draw keep flags
  float *logit;           // pool outputs (may be NULL)
  float *prob;
  uint8_t *flags;         // pool: keep flags [P]
  float *loss_out;        // kSvm: loss per position (pool) or per row (kept); may be NULL
  const float *loss_in;   // kAssist without kSvm: Boss losses per row
  float *partial;         // [nblk][nvec][d_pad]
  int32_t *blk_cnt;       // [nblk] kept count per block (pool mode)
  float *blk_gb;          // [nblk] bias-gradient partial (kAssist)
  const int32_t *t_upd;   // optional update counter; block 0 snapshots it into *t_snap
  int32_t *t_snap;
  // kAssist alone, at most kRankSelectMax rows: with med_init the labels are taken against
  // the running threshold AFTER this batch (first batch: the median of loss_in; later:
  // momentum * *T + (1 - momentum) * median) instead of *T.  Every block works it out for
  // itself from *T and *med_init, which stay untouched during the pass; block 0 leaves the value
  // in *T_next, and the update kernel stores it to *T and sets the flag.
  const int32_t *med_init;
  float med_momentum;
  float *T_next;
  // Compaction of the pool before this one, carried by a pool pass with gradient sums
  // (prev.flags == NULL: none): block b compacts positions [64 b, 64 b + 64) of that pool
  // while its own rows are in flight.  Needs ceil(prev.P / 64) <= blocks of this launch and
  // 16-byte aligned prev.flags; prev.tile_off is not used.
  CompactArgs prev;
  // Measurement builds only (AA_PHASE_TRACE): per-wave phase time stamps of k_step_pass,
  // trace[(block * waves + wave) * kTraceStamps + k] in 10 ns ticks; NULL = none.
  unsigned long long *trace;
};

constexpr int kTraceStamps = 8;

// Largest pool whose compaction a pass of `nblk` blocks can carry.
inline int64_t dense_carry_capacity(int32_t nblk) { return (int64_t)nblk * kWave; }

struct FinalizeArgs {
  const float *partial;
  int32_t nblk, nvec, d, d_pad;
  const int32_t *blk_cnt;  // pool mode: m = sum
  const float *blk_gb;
  const int32_t *m_dev;    // kept mode: m = min(*m_dev, m_max)
  int32_t m_max;
  float *w;                // updated if non-NULL (vector 0)
  float *phi;              // updated if non-NULL (next vector)
  float *bias;
  float *phi_copy;         // optional: the Assistant after this update is also stored here
  float *bias_copy;        //   (even when m == 0 and nothing changed)
  float lambda, lr, lr_a, l2_a;
  int32_t *t_upd;          // optional device update counter driving lr/sqrt(t)
  const int32_t *t_snap;   // its value before this step (written by the pass kernel)
  int32_t *kept_hist;      // optional: receives m
  // optional: the threshold a pass has worked out (see PassArgs::med_init) becomes the running
  // threshold, and its flag is set, when the batch is not empty
  const float *T_next;
  float *T_out;
  int32_t *T_init;
  // optional compaction blocks (pool mode), one per tile of flags
  const uint8_t *flags;
  int32_t P;
  const int32_t *idx;
  int32_t *kept_pos;
  int32_t *kept_ids;
  const float *loss_pool;
  float *loss;
  int32_t *kept_count;
};

// True if the register-resident kernels can take this feature matrix.
bool dense_fast_ok(const aa_features *F);

// Padded width (floats) of one gradient partial for dimension d.
int32_t dense_d_pad(int32_t d);

// Number of blocks the pass will use for `count` rows of dimension d.
int32_t dense_pass_blocks(int32_t d, int32_t count, int mode);

// started / stopped: optional events that receive the kernel's own time stamps (both or none)
hipError_t launch_dense_pass(const PassArgs &a, int mode, int32_t d, int32_t nblk,
                             hipStream_t stream, hipEvent_t started = nullptr,
                             hipEvent_t stopped = nullptr);
hipError_t launch_dense_finalize(const FinalizeArgs &a, hipStream_t stream);

}  // namespace aa
