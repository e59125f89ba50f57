// Batch-generator helpers around the shrink path.
//
// Running-median threshold: one block sorts the batch's losses in LDS (bitonic
// network, padded with +inf) and folds the median into the threshold.
//
// Length-bucketed batching: a stable multi-way partition of the kept pairs by
// length bucket, three launches: per-tile bucket histograms (LDS integer
// atomics), one block that turns them into per-tile, per-bucket offsets, bucket
// starts and batch numbers, and a scatter in which a wave ranks each pair among
// the earlier pairs of its bucket with one ballot per bucket and mbcnt.
#include "aa_batching.hpp"

namespace aa {

namespace {

__global__ __launch_bounds__(1024) void k_threshold_update(const ThresholdArgs a) {
  __shared__ __attribute__((aligned(16))) float s[kMedianMax];
  __shared__ float s_mid[2];
  // every load that does not depend on another leaves at once: the count, the first losses,
  // the state (one memory round trip for a small batch instead of three)
  const int i0 = threadIdx.x;
  const float x0 = i0 < a.m_max ? a.loss[i0] : 0.f;
  const float T_old = *a.T;
  const int init_old = *a.initialised;
  const int m = min(max(*a.m_dev, 0), a.m_max);
  if (m == 0) return;
  // a NaN loss has no rank: the threshold becomes NaN, visibly (the whole block agrees)
  int has_nan = 0;
  for (int i = threadIdx.x; i < m; i += blockDim.x) {
    const float v = i == i0 ? x0 : a.loss[i];
    has_nan |= v != v;
  }
  if (__syncthreads_or(has_nan)) {
    if (threadIdx.x == 0) {
      *a.T = __builtin_nanf("");
      *a.initialised = 1;
    }
    return;
  }
  float lo_mid, hi_mid;  // sorted[(m-1)/2] and sorted[m/2]
  if (m <= kRankSelectMax) {
    const int i = i0;
    const float x = x0;
    if (i < m) s[i] = x;
    __syncthreads();
    if (i < m) {
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
      if (rank == (m - 1) / 2) s_mid[0] = x;
      if (rank == m / 2) s_mid[1] = x;
    }
    __syncthreads();
    lo_mid = s_mid[0];
    hi_mid = s_mid[1];
  } else {
    int n = 1;
    while (n < m) n <<= 1;
    for (int i = threadIdx.x; i < n; i += blockDim.x) s[i] = i < m ? a.loss[i] : __builtin_inff();
    __syncthreads();
    for (int k = 2; k <= n; k <<= 1) {
      for (int j = k >> 1; j > 0; j >>= 1) {
        for (int i = threadIdx.x; i < n; i += blockDim.x) {
          const int p = i ^ j;
          if (p > i) {
            const float x = s[i], y = s[p];
            const bool up = (i & k) == 0;
            if (up ? (x > y) : (x < y)) {
              s[i] = y;
              s[p] = x;
            }
          }
        }
        __syncthreads();
      }
    }
    lo_mid = s[(m - 1) / 2];
    hi_mid = s[m / 2];
  }
  if (threadIdx.x == 0) {
    *a.T = running_threshold(lo_mid, hi_mid, m, init_old, T_old, a.momentum);
    if (init_old == 0) *a.initialised = 1;
  }
}

__device__ __forceinline__ int bucket_of(int ls, int lt, int width, int nb) {
  const int L = max(ls, lt);
  int b = (L - 1) / width;
  b = max(b, 0);
  return min(b, nb - 1);
}

__global__ __launch_bounds__(256) void k_bucket_counts(const BucketArgs a) {
  __shared__ int hist[kMaxBuckets];
  const int m = min(max(*a.m_dev, 0), a.m_max);
  if (threadIdx.x < kMaxBuckets) hist[threadIdx.x] = 0;
  __syncthreads();
  // all sixteen loads of a thread first, none under a condition of its own (a row past the
  // end reads the last kept row instead and is not counted): one memory round trip, not eight
  const int r0 = blockIdx.x * kBucketTile, last = m - 1;
  if (m > 0) {
    int ls[kBucketTile / 256], lt[kBucketTile / 256];
#pragma unroll
    for (int q = 0; q < kBucketTile / 256; ++q) {
      const int r = min(r0 + q * 256 + (int)threadIdx.x, last);
      ls[q] = a.len_s[r];
      lt[q] = a.len_t[r];
    }
#pragma unroll
    for (int q = 0; q < kBucketTile / 256; ++q)
      if (r0 + q * 256 + (int)threadIdx.x < m)
        atomicAdd(&hist[bucket_of(ls[q], lt[q], a.width, a.n_buckets)], 1);
  }
  __syncthreads();
  if ((int)threadIdx.x < a.n_buckets) a.tile_base[blockIdx.x * a.n_buckets + threadIdx.x] = hist[threadIdx.x];
}

// One block, one wave per bucket (16 waves, each taking buckets w, w + 16): per-bucket totals over
// the tiles, then the bucket starts and batch bases, then each tile's count becomes the position
// where that tile's share of the bucket begins.
__global__ __launch_bounds__(1024) void k_bucket_scan(const BucketArgs a, int ntiles_max) {
  __shared__ int total[kMaxBuckets], start[kMaxBuckets + 1], batch_base[kMaxBuckets + 1];
  const int m = min(max(*a.m_dev, 0), a.m_max);
  const int ntiles = (m + kBucketTile - 1) / kBucketTile;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int nb = a.n_buckets;
  for (int b = wave; b < nb; b += nw) {
    int sum = 0;
    for (int t = lane; t < ntiles; t += kWave) sum += a.tile_base[t * nb + b];
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) sum += __shfl_xor(sum, off, kWave);
    if (lane == 0) total[b] = sum;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int s = 0, batches = 0;
    for (int q = 0; q < nb; ++q) {
      start[q] = s;
      batch_base[q] = batches;
      const int cap = max(1, a.token_budget / (2 * a.width * (q + 1)));
      batches += (total[q] + cap - 1) / cap;
      s += total[q];
    }
    start[nb] = s;
    batch_base[nb] = batches;
    *a.n_batches = batches;
  }
  __syncthreads();
  const int tid = threadIdx.x;
  if (tid <= nb) a.bucket_start[tid] = start[tid];
  int *tail = a.tile_base + (size_t)ntiles_max * nb;  // [nb] starts, [nb] batch bases
  if (tid < nb) {
    tail[tid] = start[tid];
    tail[nb + tid] = batch_base[tid];
  }
  for (int b = wave; b < nb; b += nw) {
    int run = start[b];
    for (int t0 = 0; t0 < ntiles; t0 += kWave) {
      const int t = t0 + lane;
      const int c = t < ntiles ? a.tile_base[t * nb + b] : 0;
      int incl = c;
#pragma unroll
      for (int off = 1; off < kWave; off <<= 1) {
        const int up = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += up;
      }
      if (t < ntiles) a.tile_base[t * nb + b] = run + incl - c;
      run += __shfl(incl, kWave - 1, kWave);
    }
  }
}

__global__ __launch_bounds__(256) void k_bucket_scatter(const BucketArgs a, int ntiles_max) {
  __shared__ int wave_tot[4][kMaxBuckets];
  const int m = min(max(*a.m_dev, 0), a.m_max);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nb = a.n_buckets;
  const int seg = blockIdx.x * kBucketTile + wave * (kBucketTile / 4);
  if (m <= 0) return;  // (the whole block: nothing is kept)
  int bk[8];
  {  // (loads first and without conditions of their own, as in k_bucket_counts)
    int ls[8], lt[8];
    const int last = m - 1;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const int row = min(seg + r * kWave + lane, last);
      ls[r] = a.len_s[row];
      lt[r] = a.len_t[row];
    }
#pragma unroll
    for (int r = 0; r < 8; ++r)
      bk[r] = seg + r * kWave + lane < m ? bucket_of(ls[r], lt[r], a.width, nb) : -1;
  }
  // Lane b keeps what belongs to bucket b (there are at most 32): the wave's count, then its
  // running position, the bucket's start, first batch and batch size.  A round of 64 rows is
  // taken bucket by bucket over the buckets that occur in it (the leader lane's, then the
  // next one still open), not over all of them.
  auto for_each_bucket = [&](int bucket, auto &&body) __attribute__((always_inline)) {
    unsigned long long todo = __ballot(bucket >= 0);
    while (todo != 0ull) {
      const int b = __shfl(bucket, __ffsll((long long)todo) - 1, kWave);
      const unsigned long long mask = __ballot(bucket == b);
      body(b, mask);
      todo &= ~mask;
    }
  };
  int mine = 0;
#pragma unroll
  for (int r = 0; r < 8; ++r)
    for_each_bucket(bk[r], [&](int b, unsigned long long mask) {
      if (lane == b) mine += __popcll(mask);
    });
  if (lane < nb) wave_tot[wave][lane] = mine;
  const int *tail = a.tile_base + (size_t)ntiles_max * nb;
  const int lb = min(lane, nb - 1);
  int run = a.tile_base[blockIdx.x * nb + lb];  // where this tile's share of bucket `lane` begins
  const int first = tail[lb], first_batch = tail[nb + lb];
  const int cap = max(1, a.token_budget / (2 * a.width * (lb + 1)));
  __syncthreads();
  for (int w = 0; w < wave; ++w) run += wave_tot[w][lb];
#pragma unroll
  for (int r = 0; r < 8; ++r)
    for_each_bucket(bk[r], [&](int b, unsigned long long mask) {
      const int base = __shfl(run, b, kWave), b_first = __shfl(first, b, kWave);
      const int b_batch = __shfl(first_batch, b, kWave), b_cap = __shfl(cap, b, kWave);
      if (bk[r] == b) {
        const int pos = base + __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                                         __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
        a.order[pos] = seg + r * kWave + lane;
        a.batch_of[pos] = b_batch + (pos - b_first) / b_cap;
      }
      if (lane == b) run += __popcll(mask);
    });
}

}  // namespace

hipError_t launch_threshold_update(const ThresholdArgs &a, hipStream_t st) {
  hipLaunchKernelGGL(k_threshold_update, dim3(1), dim3(1024), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_bucket_batches(const BucketArgs &a, hipStream_t st) {
  const int ntiles = (a.m_max + kBucketTile - 1) / kBucketTile;
  if (ntiles > 0) {
    hipLaunchKernelGGL(k_bucket_counts, dim3(ntiles), dim3(256), 0, st, a);
    if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
  }
  hipLaunchKernelGGL(k_bucket_scan, dim3(1), dim3(1024), 0, st, a, ntiles);
  if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
  if (ntiles > 0) hipLaunchKernelGGL(k_bucket_scatter, dim3(ntiles), dim3(256), 0, st, a, ntiles);
  return hipGetLastError();
}

}  // namespace aa
