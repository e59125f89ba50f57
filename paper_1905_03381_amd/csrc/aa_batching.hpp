// Host-side launch interface of the batch-generator helpers: running-median
// threshold and length-bucketed batching of kept sentence pairs.
#pragma once

#include "aa_common.hpp"

namespace aa {

constexpr int kMaxBuckets = 32;
constexpr int kMedianMax = 16384;  // losses sorted in LDS by one block
constexpr int kBucketTile = 2048;  // kept pairs ranked by one block of the bucket partition

// int32 entries of the bucket table for up to m_max pairs: one row of kMaxBuckets counts per
// tile, then the bucket starts and the batch bases (the kernels index rows with the call's
// n_buckets <= kMaxBuckets, so this covers every bucket count).
inline size_t bucket_table_ints(int64_t m_max) {
  const size_t tiles = (size_t)((m_max > 0 ? m_max : 0) + kBucketTile - 1) / kBucketTile;
  return (tiles + 2) * kMaxBuckets;
}

struct ThresholdArgs {
  const float *loss;
  const int32_t *m_dev;
  int32_t m_max;
  float momentum;
  float *T;
  int32_t *initialised;
};

struct BucketArgs {
  const int32_t *len_s;
  const int32_t *len_t;
  const int32_t *m_dev;
  int32_t m_max;
  int32_t width, n_buckets, token_budget;
  int32_t *order;         // [m] row numbers grouped by bucket, arrival order inside
  int32_t *bucket_start;  // [n_buckets + 1]
  int32_t *batch_of;      // [m] batch number of order[q]
  int32_t *n_batches;     // device scalar
  int32_t *tile_base;     // workspace [ntiles][n_buckets], then [2 * n_buckets]
};

hipError_t launch_threshold_update(const ThresholdArgs &a, hipStream_t stream);
hipError_t launch_bucket_batches(const BucketArgs &a, hipStream_t stream);

}  // namespace aa
