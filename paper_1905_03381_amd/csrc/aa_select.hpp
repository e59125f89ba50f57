// Host-side launch interface of keep/compact and gather kernels.
#pragma once

#include "aa_common.hpp"

namespace aa {

enum KeepSource : int { kFromProb = 0, kFromCrit = 1, kFromFlags = 2 };

struct KeepArgs {
  const float *src;     // prob[P] (kFromProb) or crit[P] (kFromCrit)
  const float *T;       // device scalar (kFromCrit)
  int32_t P;
  float gamma, one_minus_gamma;
  DrawKey key;
  uint8_t *flags;       // [P] written (read for kFromFlags)
  int32_t *blk_off;     // [nblk] per-block counts, then exclusive offsets
  int32_t *kept_count;
  int32_t *ticket;
};

struct ScatterArgs {
  const uint8_t *flags;
  int32_t P;
  const int32_t *blk_off;
  int32_t *kept_pos;
};

struct GatherArgs {
  const char *src;
  char *dst;
  int64_t row_bytes;
  const int32_t *idx;
  const int32_t *kept_pos;
  const int32_t *kept_count;
  int32_t max_rows;
  int32_t *kept_ids;
};

struct GatherCsrArgs {
  const int64_t *rowptr;
  const int32_t *col;
  const float *val;
  const int32_t *idx;
  const int32_t *kept_pos;
  const int32_t *kept_count;
  int32_t max_rows;
  int64_t *out_rowptr;
  int32_t *out_col;
  float *out_val;
  int64_t out_nnz_cap;
};

constexpr int kKeepBlock = 256;  // candidates per block of the keep/scatter kernels

hipError_t launch_keep_count(const KeepArgs &a, int source, hipStream_t stream);
hipError_t launch_scatter(const ScatterArgs &a, hipStream_t stream);
hipError_t launch_gather(const GatherArgs &a, hipStream_t stream);
hipError_t launch_gather_csr(const GatherCsrArgs &a, hipStream_t stream);

}  // namespace aa
