// Host-side launch interface of the general (CSR / any dense) row passes.
#pragma once

#include "aa_common.hpp"
#include "aa_dense.hpp"

namespace aa {

// What leaves a block of a gradient pass for a column without a slot in its LDS table.
// kind 0: one stored entry of a kept row -- a and b hold, as float bits, its terms of the (up
// to two) gradient sums (two updated vectors: a -> w, b -> phi; one: a -> that vector).
// kind 1, 2: the sum a hashed slot collected for the first / second updated vector -- a and b
// hold the low and high word of the double.
struct __attribute__((aligned(16))) TailRecord {
  int32_t col;
  int32_t a, b;
  int32_t kind;
};

// Columns from `head` on are dealt to nb bins (a power of two, 0: no binning) in groups of
// 2^group_log2: group g = (col - head) >> group_log2 goes to bin g % nb, where it is group
// g / nb; a bin spans `cols` columns in all and holds up to `cap` records.  A group is 16
// columns (one 64-byte line of a model vector) when there are many columns, so that the
// owners read and write the model in whole lines; with fewer columns that traffic is small
// beside the records', and groups of 4 spread a run of frequent neighbouring columns (the
// head of a vocabulary, say) over four times as many bins -- the bin with the most records
// sets the update kernel's time.
struct BinPlan {
  int32_t nb, nb_log2, cols, cap, group_log2;
};
constexpr int kMaxBins = 256;
constexpr int kBinGroupLog2 = 4, kBinFineGroupLog2 = 2;
constexpr int64_t kBinFineColsMax = 1 << 18;  // groups of 4 up to this many binned columns
constexpr int kBinColsMax = 8192;  // LDS floats of a bin's owner in the update kernel
// Records the bins hold in all: 48 per candidate (the sparse configuration needs about 26),
// at least 65,536, at most 2^27 (2 GiB); what does not fit goes to the accumulators.
inline size_t general_record_capacity(int32_t count_max) {
  const size_t want = 48 * (size_t)(count_max > 0 ? count_max : 0);
  return want < 65536 ? 65536 : (want > ((size_t)1 << 27) ? ((size_t)1 << 27) : want);
}
inline BinPlan general_bin_plan(int32_t d, int32_t head, int nvec, int32_t count_max) {
  BinPlan p{0, 0, 0, 0, kBinGroupLog2};
  const int gl = (int64_t)d - head <= kBinFineColsMax ? kBinFineGroupLog2 : kBinGroupLog2;
  const int64_t group = (int64_t)1 << gl;
  const int64_t groups = ((int64_t)d - head + group - 1) / group;
  if (groups <= 0 || nvec < 1) return p;
  int nb = 1, lg = 0;
  while (nb * 2 <= kMaxBins && nb * 2 <= groups) {
    nb *= 2;
    ++lg;
  }
  const int64_t cols = group * ((groups + nb - 1) / nb);
  if (cols * nvec > kBinColsMax) return p;  // too many columns for the owners' LDS: atomics instead
  p.nb = nb;
  p.nb_log2 = lg;
  p.group_log2 = gl;
  p.cols = (int32_t)cols;
  p.cap = (int32_t)(general_record_capacity(count_max) / nb);
  return p;
}

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
  // (w[c], phi[c]) side by side for the columns past `head`, indexed by column: one gather
  // brings both values of a column that is not in LDS (written before the pass; NULL unless
  // the pass updates both vectors)
  const float2 *wp;
  // atomic accumulators (zeroed before the pass); with bins, acc_used[bin] (zeroed too) is set
  // by whoever adds to a column of that bin
  double *acc_w;     // [d]
  double *acc_p;     // [d]
  int32_t *acc_used; // [kMaxBins]
  // per-block kept count and bias-gradient sum of a gradient pass (plain stores)
  int32_t *blk_cnt;  // [blocks of the pass]
  float *blk_gb;     // [blocks of the pass]
  // per-block sums of the first `head` columns: part[(block * nvec + vec) * head + column],
  // written whole by every block of a gradient pass (no clearing needed)
  float *part;
  int32_t head;
  // entries of the other columns leave a block as records, sorted into bins by column
  // (see BinPlan); fill[bin] counts the records offered to a bin, zeroed before the pass
  TailRecord *bins;
  unsigned long long *bin_fill;
  BinPlan plan;
  // optional device-side update counter (step size lr / sqrt(t)): block 0 of a gradient pass
  // copies it to *t_snap, which the update kernel reads (the counter itself changes there)
  const int32_t *t_upd;
  int32_t *t_snap;
};

// Columns whose gradient sums leave a block as plain stores instead of atomics, for a pass
// that updates nvec vectors over d columns; blocks of a gradient pass at most.
int32_t general_head_columns(int32_t d, int nvec, bool csr);
// Whether the update kernel can leave the workspace ready for the next pass (see ApplyArgs).
bool general_keeps_ready(int32_t d, int nvec, bool csr);
constexpr int kGeneralGradBlocks = 256;
// floats ahead of the accumulators: 16 scalars, the 64-bit fill counts of the bins, then one
// flag per bin (an even count in all: the accumulators behind it are doubles)
constexpr int kGeneralHeader = 16 + 3 * kMaxBins;
// floats the header and the two accumulators of d doubles take
inline size_t general_clear_floats(int32_t d) { return kGeneralHeader + 4 * (size_t)d; }
inline size_t general_part_floats(int32_t d) {
  const size_t per_block = 2 * (size_t)d < 16384 ? 2 * (size_t)d : 16384;
  return kGeneralGradBlocks * per_block;
}

struct ApplyArgs {
  int32_t d;
  double *acc_w;
  double *acc_p;
  int32_t *acc_used;  // [bin] 0: the pass added nothing to the accumulators of the bin's columns
  // Leave the workspace as the next pass of the same call needs it, so that no preparing
  // launch has to run in between (bins only): every bin owner clears its fill count, its flag
  // and whatever it read from the accumulators, and with two updated vectors writes the new
  // (w[c], phi[c]) pairs of its columns.
  int32_t keep_ready;
  float2 *wp_out;     // pairs, indexed by column (NULL: none)
  const int32_t *blk_cnt;  // per-block kept counts and bias-gradient sums of the pass
  const float *blk_gb;
  const int32_t *m_dev;
  int32_t m_max;
  float *w;
  float *phi;
  float *bias;
  float *phi_copy;   // optional second destination of the updated Assistant (written even if m == 0)
  float *bias_copy;
  const float *part;  // per-block sums of the first `head` columns (see GenArgs)
  int32_t head, nvec, nblk_pass;
  const TailRecord *bins;  // records of the other columns (see GenArgs)
  unsigned long long *bin_fill;
  BinPlan plan;
  float lambda, lr, lr_a, l2_a;
  int32_t *t_upd;          // optional update counter: the Boss step size is lr / sqrt(updates so far)
  const int32_t *t_snap;   // its value before this step (written by the pass kernel)
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
                               hipStream_t stream, hipEvent_t started = nullptr,
                               hipEvent_t stopped = nullptr);
hipError_t launch_zero_f32(float *p, size_t count, hipStream_t stream);
// Zeroes p[0, count) and writes wp[c] = (w[c], phi[c]) for head <= c < d (one launch).
hipError_t launch_prepare_general(float *p, size_t count, const float *w, const float *phi,
                                  float2 *wp, int32_t head, int32_t d, hipStream_t stream);
hipError_t launch_general_apply(const ApplyArgs &a, hipStream_t stream);

}  // namespace aa
