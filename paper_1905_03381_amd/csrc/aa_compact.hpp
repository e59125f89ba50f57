// Stable stream compaction of keep flags (the append order of Algorithm 1:
// kept candidates stay in arrival order).
//
// A block compacts one tile of kCompactTile flags.  Each of its four waves owns
// a contiguous 512-flag segment and walks it in eight 64-lane rounds: a wavefront
// ballot turns the round's flags into a 64-bit mask, mbcnt on the mask ranks a
// lane among the survivors of its round, popcounts of the masks give the wave's
// total, and an LDS exchange of the four wave totals gives each wave its base.
// The tile's own base is the number of flags set before it: either read from a
// table of tile offsets or counted directly (popcount over the 0/1 bytes).
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
  const int32_t *tile_off;  // exclusive tile offsets, or NULL: count the flags before the tile
};

// Number of set flags in [0, j0) (j0 a multiple of 16), whole block cooperates.
__device__ inline int count_flags_before(const uint8_t *flags, int j0, int *smem) {
  int cnt = 0;
  if ((reinterpret_cast<uintptr_t>(flags) & 15) == 0) {
    const uint4 *p = reinterpret_cast<const uint4 *>(flags);
    const int n16 = j0 >> 4, stride = blockDim.x;
    int q = threadIdx.x;
    for (; q + 3 * stride < n16; q += 4 * stride) {  // four loads in flight per thread
      const uint4 v0 = p[q], v1 = p[q + stride], v2 = p[q + 2 * stride], v3 = p[q + 3 * stride];
      cnt += __popc(v0.x) + __popc(v0.y) + __popc(v0.z) + __popc(v0.w);  // bytes are 0 or 1
      cnt += __popc(v1.x) + __popc(v1.y) + __popc(v1.z) + __popc(v1.w);
      cnt += __popc(v2.x) + __popc(v2.y) + __popc(v2.z) + __popc(v2.w);
      cnt += __popc(v3.x) + __popc(v3.y) + __popc(v3.z) + __popc(v3.w);
    }
    for (; q < n16; q += stride) {
      const uint4 v = p[q];
      cnt += __popc(v.x) + __popc(v.y) + __popc(v.z) + __popc(v.w);
    }
  } else {
    for (int j = threadIdx.x; j < j0; j += blockDim.x) cnt += flags[j] != 0;
  }
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) cnt += __shfl_xor(cnt, off, kWave);
  const int nw = blockDim.x >> 6;
  if ((threadIdx.x & 63) == 0) smem[threadIdx.x >> 6] = cnt;
  __syncthreads();
  int total = 0;
  for (int i = 0; i < nw; ++i) total += smem[i];
  __syncthreads();
  return total;
}

// Compact tile `tile` with a 256-thread block.  `smem` holds at least 8 ints.
__device__ inline void tile_compact(const CompactArgs &c, int tile, int *smem) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j0 = tile * kCompactTile;
  const int seg = j0 + wave * (kCompactTile / 4);
  // The tile's own loads go out first, then the count of the flags before the tile.  No load
  // sits under a per-element condition (the compiler would wait for each before requesting
  // the next): a position past the pool reads the pool's last element instead, and whether
  // an array takes part at all is decided once, around its eight loads.
  uint8_t fl[8];
  int ids[8];
  float ls[8];
  const int last = c.P - 1;  // (a tile exists: P > 0)
#pragma unroll
  for (int r = 0; r < 8; ++r) fl[r] = c.flags[min(seg + r * kWave + lane, last)];
  if (c.kept_ids && c.idx) {
#pragma unroll
    for (int r = 0; r < 8; ++r) ids[r] = c.idx[min(seg + r * kWave + lane, last)];
  } else {
#pragma unroll
    for (int r = 0; r < 8; ++r) ids[r] = seg + r * kWave + lane;
  }
  if (c.loss) {
#pragma unroll
    for (int r = 0; r < 8; ++r) ls[r] = c.loss_pool[min(seg + r * kWave + lane, last)];
  } else {
#pragma unroll
    for (int r = 0; r < 8; ++r) ls[r] = 0.f;
  }
  const int prefix = c.tile_off ? c.tile_off[tile] : count_flags_before(c.flags, j0, smem);
#pragma unroll
  for (int r = 0; r < 8; ++r)
    if (seg + r * kWave + lane > last) fl[r] = 0;
  unsigned long long masks[8];
  int wave_total = 0;
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    masks[r] = __ballot(fl[r] != 0);
    wave_total += __popcll(masks[r]);
  }
  if (lane == 0) smem[wave] = wave_total;
  __syncthreads();
  int running = prefix, total = 0;
  for (int i = 0; i < 4; ++i) {
    const int t = smem[i];
    if (i < wave) running += t;
    total += t;
  }
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const unsigned long long m = masks[r];
    if ((m >> lane) & 1ull) {
      const int pos = running + __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32),
                                                          __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
      const int j = seg + r * kWave + lane;
      if (c.kept_pos) c.kept_pos[pos] = j;
      if (c.kept_ids) c.kept_ids[pos] = ids[r];
      if (c.loss) c.loss[pos] = ls[r];
    }
    running += __popcll(m);
  }
  if (threadIdx.x == 0 && c.kept_count && j0 + kCompactTile >= c.P) *c.kept_count = prefix + total;
}

__host__ __device__ inline int compact_tiles(int P) { return (P + kCompactTile - 1) / kCompactTile; }

}  // namespace aa
