// Device helpers shared by the gfx950 kernels: counter-based uniforms, wave64
// reductions and scans, workspace layout.  CDNA4 only (wave64).
#pragma once

#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/autoassist.h"

namespace aa {

constexpr int kWave = 64;
constexpr int kMaxBlocks = 1024;       // upper bound on persistent blocks of a row pass
constexpr int kFastDenseMaxD = 2048;   // register-resident model vectors up to this d
constexpr int kCompactTile = 2048;     // keep flags compacted by one block

// ---- workspace layout (byte offsets from ws) ------------------------------
// [0, 256)            int32 control words (word 0: snapshot of the update counter)
// [256, +4K)          int32 blk_cnt[kMaxBlocks]
// [.., +4K)           float blk_gb[kMaxBlocks]
// [.., +8)            scalars
// then a region sized by the call: gradient partials / accumulators, pool
// scratch (flags, per-position losses), block offsets.
constexpr size_t kWsControl = 0;
constexpr size_t kWsBlkCnt = 256;
constexpr size_t kWsBlkGb = kWsBlkCnt + sizeof(int32_t) * kMaxBlocks;
constexpr size_t kWsScalars = kWsBlkGb + sizeof(float) * kMaxBlocks;
constexpr size_t kWsBody = kWsScalars + 256;

__host__ __device__ inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// A kernel launch whose own start and stop time stamps go to a pair of caller events when
// both are given (a measurement aid: not for use under stream capture).
template <typename Kernel, typename Args>
inline void launch_stamped(Kernel kernel, dim3 grid, dim3 block, hipStream_t stream,
                           hipEvent_t started, hipEvent_t stopped, const Args &args) {
  if (started && stopped)
    hipExtLaunchKernelGGL(kernel, grid, block, 0, stream, started, stopped, 0, args);
  else
    hipLaunchKernelGGL(kernel, grid, block, 0, stream, args);
}

// ---- Philox4x32-10 (Salmon et al., SC'11) ---------------------------------
// Counter (j, 0, step_lo, step_hi), key (seed_lo, seed_hi); returns word 0.
__device__ __forceinline__ uint32_t philox_word0(uint32_t j, uint32_t step_lo, uint32_t step_hi,
                                                 uint32_t k0, uint32_t k1) {
  uint32_t c0 = j, c1 = 0u, c2 = step_lo, c3 = step_hi;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    const uint32_t n0 = hi1 ^ c1 ^ k0;
    const uint32_t n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return c0;
}

struct DrawKey {
  uint32_t k0, k1, s0, s1;
};

__host__ inline DrawKey make_draw_key(uint64_t seed, uint64_t step) {
  DrawKey k;
  k.k0 = (uint32_t)(seed & 0xFFFFFFFFull);
  k.k1 = (uint32_t)(seed >> 32);
  k.s0 = (uint32_t)(step & 0xFFFFFFFFull);
  k.s1 = (uint32_t)(step >> 32);
  return k;
}

// c ~ U[0,1) of Algorithm 1 on the 2^-24 grid (exact in fp32).
__device__ __forceinline__ float keep_uniform(const DrawKey &k, uint32_t j) {
  return (float)(philox_word0(j, k.s0, k.s1, k.k0, k.k1) >> 8) * 0x1p-24f;
}

// keep iff c < gamma + (1 - gamma) g, as one fused multiply-add in fp32.
__device__ __forceinline__ bool keep_decision(float u, float g, float gamma, float one_minus_gamma) {
  return u < __fmaf_rn(one_minus_gamma, g, gamma);
}

__device__ __forceinline__ float sigmoidf_(float s) { return 1.0f / (1.0f + expf(-s)); }

// ---- wave64 primitives -----------------------------------------------------
// Butterfly sum over aligned groups of WIDTH lanes; every lane gets the total.
template <int WIDTH>
__device__ __forceinline__ float group_sum(float v) {
#pragma unroll
  for (int off = WIDTH / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

// Sum of the values held by lanes (sub, sub+LPR, sub+2*LPR, ...): folds the
// row groups of one wave onto each other.
template <int LPR>
__device__ __forceinline__ float fold_groups(float v) {
#pragma unroll
  for (int off = kWave / 2; off >= LPR; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

__device__ __forceinline__ int wave_inclusive_scan(int v, int lane) {
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const int t = __shfl_up(v, off, kWave);
    if (lane >= off) v += t;
  }
  return v;
}

// Exclusive scan of one int per thread over the block.  `smem` holds at least
// blockDim.x/64 + 1 ints.  Returns the exclusive prefix; *total gets the sum.
__device__ __forceinline__ int block_exclusive_scan(int v, int *smem, int *total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  const int incl = wave_inclusive_scan(v, lane);
  if (lane == 63) smem[wave] = incl;
  __syncthreads();
  int base = 0, sum = 0;
  for (int i = 0; i < nw; ++i) {
    const int t = smem[i];
    if (i < wave) base += t;
    sum += t;
  }
  __syncthreads();
  *total = sum;
  return base + incl - v;
}

}  // namespace aa
