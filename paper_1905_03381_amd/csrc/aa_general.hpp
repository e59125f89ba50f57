// Host-side launch interface of the general (CSR / any dense) row passes.
#pragma once

#include "aa_common.hpp"
#include "aa_dense.hpp"

namespace aa {

struct GenArgs {
  // features
  const float *x;
  int64_t ld;
  int32_t d;
  const int64_t *rowptr;
  const int32_t *col;
  const float *val;
  const float *y;
  const int32_t *rows;
  int32_t count_max;
  const int32_t *m_dev;
  const float *w;
  const float *phi;
  const float *bias;
  const float *T;
  float gamma, one_minus_gamma;
  DrawKey key;
  int32_t do_keep;
  float *logit;
  float *prob;
  uint8_t *flags;
  float *loss_out;
  const float *loss_in;
  // atomic accumulators (zeroed before the pass)
  float *acc_w;      // [d]
  float *acc_p;      // [d]
  int32_t *acc_cnt;  // kept count
  float *acc_gb;     // bias gradient
  // per-block sums of the first `head` columns: part[(block * nvec + vec) * head + column],
  // written whole by every block of a gradient pass (no clearing needed)
  float *part;
  int32_t head;
};

// Columns whose gradient sums leave a block as plain stores instead of atomics, for a pass
// that updates nvec vectors over d columns; blocks of a gradient pass at most.
int32_t general_head_columns(int32_t d, int nvec);
constexpr int kGeneralGradBlocks = 256;
inline size_t general_part_floats(int32_t d) {
  const size_t per_block = 2 * (size_t)d < 16384 ? 2 * (size_t)d : 16384;
  return kGeneralGradBlocks * per_block;
}

struct ApplyArgs {
  int32_t d;
  const float *acc_w;
  const float *acc_p;
  const int32_t *acc_cnt;
  const float *acc_gb;
  const int32_t *m_dev;
  int32_t m_max;
  float *w;
  float *phi;
  float *bias;
  float *phi_copy;   // optional second destination of the updated Assistant (written even if m == 0)
  float *bias_copy;
  const float *part;  // per-block sums of the first `head` columns (see GenArgs)
  int32_t head, nvec, nblk_pass;
  float lambda, lr, lr_a, l2_a;
  int32_t *kept_hist;
  const uint8_t *flags;
  int32_t P;
  const int32_t *idx;
  int32_t *kept_pos;
  int32_t *kept_ids;
  const float *loss_pool;
  float *loss;
  int32_t *kept_count;
};

int32_t general_pass_blocks(int32_t count, bool csr, int mode);
hipError_t launch_general_pass(const GenArgs &a, int mode, bool csr, int32_t nblk,
                               hipStream_t stream);
hipError_t launch_zero_f32(float *p, size_t count, hipStream_t stream);
hipError_t launch_general_apply(const ApplyArgs &a, hipStream_t stream);

}  // namespace aa
