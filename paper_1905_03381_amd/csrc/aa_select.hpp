// Host-side launch interface of keep/compact and gather kernels.
#pragma once

#include "aa_common.hpp"
#include "aa_compact.hpp"

namespace aa {

enum KeepSource : int { kFromProb = 0, kFromCrit = 1 };

struct KeepArgs {
  const float *src;     // prob[P] (kFromProb) or crit[P] (kFromCrit)
  const float *T;       // device scalar (kFromCrit)
  int32_t P;
  float gamma, one_minus_gamma;
  DrawKey key;
  uint8_t *flags;       // [P] written
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

// Pools up to this size let every compaction tile count the flags before it directly.
constexpr int kDirectCountMax = 1 << 18;

hipError_t launch_keep_flags(const KeepArgs &a, int source, hipStream_t stream);
// Compact c.flags (c.tile_off is set here).  tile_off_scratch: P/2048 + 1 ints of workspace.
hipError_t launch_compact(CompactArgs c, int32_t *tile_off_scratch, hipStream_t stream);
hipError_t launch_gather(const GatherArgs &a, hipStream_t stream);
// tile_scratch: max_rows / 1024 + 1 64-bit words of workspace (NULL: one block scans all rows).
hipError_t launch_gather_csr(const GatherCsrArgs &a, long long *tile_scratch, hipStream_t stream);

}  // namespace aa
