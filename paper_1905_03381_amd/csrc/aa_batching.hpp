// Host-side launch interface of the batch-generator helpers: running-median
// threshold and length-bucketed batching of kept sentence pairs.
#pragma once

#include "aa_common.hpp"

namespace aa {

constexpr int kMaxBuckets = 32;
constexpr int kMedianMax = 16384;  // losses sorted in LDS by one block
constexpr int kBucketTile = 2048;  // kept pairs ranked by one block of the bucket partition
// Batches up to this size find their two middle losses by rank counting (every thread ranks
// its losses against all others, read as LDS broadcasts); larger ones are sorted.
constexpr int kRankSelectMax = 512;

#ifdef __HIPCC__
// The running threshold after a batch whose sorted losses have the middle values lo_mid
// (index (m-1)/2) and hi_mid (index m/2): the first batch sets it to the median, later ones move
// it by T <- momentum T + (1 - momentum) med.  Every product and sum is rounded to fp32 on its
// own (no fused multiply-add), so every caller gets the same bits.
__device__ __forceinline__ float running_threshold(float lo_mid, float hi_mid, int m, int init_old,
                                                   float T_old, float momentum) {
#pragma clang fp contract(off)
  float med;
  if (m & 1) {
    med = hi_mid;
  } else {
    const float sum = lo_mid + hi_mid;
    med = sum * 0.5f;
  }
  if (init_old == 0) return med;
  const float keep_part = momentum * T_old;
  const float one_minus = 1.0f - momentum;
  const float new_part = one_minus * med;
  return keep_part + new_part;
}

// The two middle values of loss[0..m), 1 <= m <= kRankSelectMax, by rank counting.  Whole block
// (any size); s holds kRankSelectMax + 2 floats, 16-byte aligned.  False when a loss is NaN (no rank).
__device__ __forceinline__ bool block_middle_values(const float *loss, int m, float *s, float *lo_mid,
                                                    float *hi_mid) {
  int has_nan = 0;
  for (int i = threadIdx.x; i < m; i += blockDim.x) {
    const float v = loss[i];
    s[i] = v;
    has_nan |= v != v;
  }
  if (__syncthreads_or(has_nan)) return false;
  for (int i = threadIdx.x; i < m; i += blockDim.x) {
    const float x = s[i];
    int rank = 0;  // position of x in the stable sorted order
    const int m4 = m & ~3;
#pragma unroll 4
    for (int j = 0; j < m4; j += 4) {  // 128-bit LDS broadcasts, several in flight
      const float4 v = *reinterpret_cast<const float4 *>(s + j);
      rank += (v.x < x || (v.x == x && j < i)) ? 1 : 0;
      rank += (v.y < x || (v.y == x && j + 1 < i)) ? 1 : 0;
      rank += (v.z < x || (v.z == x && j + 2 < i)) ? 1 : 0;
      rank += (v.w < x || (v.w == x && j + 3 < i)) ? 1 : 0;
    }
    for (int j = m4; j < m; ++j) {
      const float v = s[j];
      rank += (v < x || (v == x && j < i)) ? 1 : 0;
    }
    if (rank == (m - 1) / 2) s[kRankSelectMax] = x;
    if (rank == m / 2) s[kRankSelectMax + 1] = x;
  }
  __syncthreads();
  *lo_mid = s[kRankSelectMax];
  *hi_mid = s[kRankSelectMax + 1];
  return true;
}
#endif

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
