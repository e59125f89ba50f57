// Stable stream compaction of keep flags (the append order of Algorithm 1:
// kept candidates stay in arrival order).
#pragma once

#include "aa_common.hpp"

namespace aa {

struct CompactArgs {
  const uint8_t *flags;     // [P] one byte per pool position, 0 or 1
  int32_t P;
  const int32_t *idx;       // pool ids (may be NULL)
  int32_t *kept_pos;        // out, may be NULL
  int32_t *kept_ids;        // out, may be NULL
  const float *loss_pool;   // per-position loss (may be NULL)
  float *loss;              // out: loss[r] = loss_pool[kept_pos[r]] (may be NULL)
  int32_t *kept_count;      // out, may be NULL
};

// Whole compaction done by ONE block (any multiple of 64 threads).  Each thread
// owns kTailFlagsPerThread consecutive flags of a tile; a wave-shuffle scan and an
// LDS scan over the waves give its output offset.  `smem` >= 32 ints.
__device__ inline void block_compact(const CompactArgs &c, int *smem) {
  const int nt = blockDim.x;
  const int tile = nt * kTailFlagsPerThread;
  const bool aligned = (((uintptr_t)c.flags) & 15) == 0;
  int running = 0;
  for (int t0 = 0; t0 < c.P; t0 += tile) {
    const int j0 = t0 + (int)threadIdx.x * kTailFlagsPerThread;
    uint64_t mask = 0;  // bit i = flag of position j0 + i
    if (j0 < c.P) {
      if (aligned && j0 + kTailFlagsPerThread <= c.P) {
        const uint4 *p = reinterpret_cast<const uint4 *>(c.flags + j0);
#pragma unroll
        for (int q = 0; q < kTailFlagsPerThread / 16; ++q) {
          const uint4 v = p[q];
          const uint32_t wds[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
          for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int b = 0; b < 4; ++b)
              if ((wds[k] >> (8 * b)) & 0xFFu) mask |= 1ull << (q * 16 + k * 4 + b);
        }
      } else {
        for (int i = 0; i < kTailFlagsPerThread && j0 + i < c.P; ++i)
          if (c.flags[j0 + i]) mask |= 1ull << i;
      }
    }
    const int cnt = __popcll(mask);
    int total;
    int off = running + block_exclusive_scan(cnt, smem, &total);
    while (mask) {
      const int i = __ffsll((long long)mask) - 1;
      mask &= mask - 1;
      const int j = j0 + i;
      if (c.kept_pos) c.kept_pos[off] = j;
      if (c.kept_ids) c.kept_ids[off] = c.idx ? c.idx[j] : j;
      if (c.loss) c.loss[off] = c.loss_pool[j];
      ++off;
    }
    running += total;
  }
  if (threadIdx.x == 0 && c.kept_count) *c.kept_count = running;
}

}  // namespace aa
