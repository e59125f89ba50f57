// Keep draw + stable compaction (Algorithm 1) and batch assembly (gather).
//
// aa_shrink is two launches: one thread per candidate draws (or thresholds) the
// keep flag, then one block per 2048-flag tile compacts (ballot + mbcnt + LDS
// prefix, see aa_compact.hpp).  Up to kDirectCountMax candidates every tile
// counts the flags before it by itself; larger pools insert a per-tile count
// and a one-block scan of the tile counts.
#include "aa_compact.hpp"
#include "aa_select.hpp"

namespace aa {

namespace {

typedef unsigned int u4 __attribute__((ext_vector_type(4)));

// One thread per candidate: the keep flag from a Philox draw against the keep
// probability, or from a threshold on a criterion.
template <int SRC>
__global__ __launch_bounds__(256) void k_keep_flags(const KeepArgs a) {
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= a.P) return;
  bool keep;
  if (SRC == kFromProb) {
    const float u = keep_uniform(a.key, (uint32_t)j);
    keep = keep_decision(u, a.src[j], a.gamma, a.one_minus_gamma);
  } else {
    keep = a.src[j] > *a.T;
  }
  a.flags[j] = keep ? 1 : 0;
}

// Compaction of the flags, one block per tile.
__global__ __launch_bounds__(256) void k_compact(const CompactArgs c) {
  __shared__ int s_int[8];
  tile_compact(c, blockIdx.x, s_int);
}

// Large pools: per-tile counts, then one block turns them into exclusive offsets.
__global__ __launch_bounds__(256) void k_tile_counts(const uint8_t *flags, int P, int32_t *tile_off) {
  __shared__ int s_int[8];
  const int j0 = blockIdx.x * kCompactTile;
  int cnt = 0;
  for (int j = j0 + threadIdx.x; j < min(P, j0 + kCompactTile); j += 256) cnt += flags[j] != 0;
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) cnt += __shfl_xor(cnt, off, kWave);
  if ((threadIdx.x & 63) == 0) s_int[threadIdx.x >> 6] = cnt;
  __syncthreads();
  if (threadIdx.x == 0) tile_off[blockIdx.x] = s_int[0] + s_int[1] + s_int[2] + s_int[3];
}

__global__ __launch_bounds__(1024) void k_scan_tiles(int32_t *tile_off, int ntiles) {
  __shared__ int s_int[40];
  int running = 0;
  for (int t0 = 0; t0 < ntiles; t0 += 1024) {
    const int i = t0 + threadIdx.x;
    const int v = i < ntiles ? tile_off[i] : 0;
    int total;
    const int excl = block_exclusive_scan(v, s_int, &total);
    if (i < ntiles) tile_off[i] = running + excl;
    running += total;
  }
}

__global__ void k_set_i32(int32_t *p, int32_t v) { *p = v; }

// Copy rows chunk by chunk; a block owns one chunk of one kept row at a time.
template <int VEC, int UNROLL>
__global__ __launch_bounds__(256) void k_gather_rows(const GatherArgs a, int cpr,
                                                     long long chunk_bytes) {
  const int m = min(max(*a.kept_count, 0), a.max_rows);
  const long long total = (long long)m * cpr;
  for (long long wi = blockIdx.x; wi < total; wi += gridDim.x) {
    const int r = (int)(wi / cpr), ch = (int)(wi % cpr);
    const int pos = a.kept_pos ? a.kept_pos[r] : r;
    const long long id = a.idx ? a.idx[pos] : pos;
    if (ch == 0 && threadIdx.x == 0 && a.kept_ids) a.kept_ids[r] = (int32_t)id;
    const long long off = (long long)ch * chunk_bytes;
    const long long nbytes = min(chunk_bytes, a.row_bytes - off);
    const char *s = a.src + id * a.row_bytes + off;
    char *d = a.dst + (long long)r * a.row_bytes + off;
    if (VEC == 16) {
      const int n = (int)(nbytes >> 4);
      const u4 *s4 = reinterpret_cast<const u4 *>(s);
      u4 *d4 = reinterpret_cast<u4 *>(d);
      u4 v[UNROLL];
#pragma unroll
      for (int q = 0; q < UNROLL; ++q) {
        const int i = q * 256 + threadIdx.x;
        if (i < n) v[q] = __builtin_nontemporal_load(s4 + i);
      }
#pragma unroll
      for (int q = 0; q < UNROLL; ++q) {
        const int i = q * 256 + threadIdx.x;
        if (i < n) __builtin_nontemporal_store(v[q], d4 + i);
      }
    } else if (VEC == 4) {
      const int n = (int)(nbytes >> 2);
      const uint32_t *s1 = reinterpret_cast<const uint32_t *>(s);
      uint32_t *d1 = reinterpret_cast<uint32_t *>(d);
      for (int i = threadIdx.x; i < n; i += 256) d1[i] = s1[i];
    } else {
      for (int i = threadIdx.x; i < (int)nbytes; i += 256) d[i] = s[i];
    }
  }
}

// Short rows (labels, lengths, a few words): one thread per 32-bit word.
__global__ __launch_bounds__(256) void k_gather_words(const GatherArgs a, int words_per_row) {
  const int m = min(max(*a.kept_count, 0), a.max_rows);
  const long long total = (long long)m * words_per_row;
  const uint32_t *src = reinterpret_cast<const uint32_t *>(a.src);
  uint32_t *dst = reinterpret_cast<uint32_t *>(a.dst);
  for (long long t = (long long)blockIdx.x * 256 + threadIdx.x; t < total;
       t += (long long)gridDim.x * 256) {
    const int r = (int)(t / words_per_row), k = (int)(t % words_per_row);
    const int pos = a.kept_pos ? a.kept_pos[r] : r;
    const long long id = a.idx ? a.idx[pos] : pos;
    if (k == 0 && a.kept_ids) a.kept_ids[r] = (int32_t)id;
    dst[t] = src[id * words_per_row + k];
  }
}

__global__ __launch_bounds__(256) void k_gather_ids(const GatherArgs a) {
  const int m = min(max(*a.kept_count, 0), a.max_rows);
  for (int r = blockIdx.x * 256 + threadIdx.x; r < m; r += gridDim.x * 256) {
    const int pos = a.kept_pos ? a.kept_pos[r] : r;
    a.kept_ids[r] = a.idx ? a.idx[pos] : pos;
  }
}

// Row lengths of the kept CSR rows -> out_rowptr (one block, running scan).
__global__ __launch_bounds__(1024) void k_csr_rowptr(const GatherCsrArgs a) {
  __shared__ int s_int[40];
  const int m = min(max(*a.kept_count, 0), a.max_rows);
  const int tid = threadIdx.x;
  long long running = 0;
  if (tid == 0) a.out_rowptr[0] = 0;
  for (int t0 = 0; t0 < m; t0 += 1024) {
    const int r = t0 + tid;
    int len = 0;
    if (r < m) {
      const int pos = a.kept_pos ? a.kept_pos[r] : r;
      const long long id = a.idx ? a.idx[pos] : pos;
      len = (int)(a.rowptr[id + 1] - a.rowptr[id]);
    }
    int total;
    const int excl = block_exclusive_scan(len, s_int, &total);
    if (r < m) a.out_rowptr[r + 1] = running + excl + len;
    running += total;
  }
}

// Row pointers of many kept rows in three launches: entry count of every tile of 1024 rows,
// exclusive scan of the tile counts (one block), then the scan inside each tile.
constexpr int kCsrTile = 1024;

__device__ __forceinline__ int kept_row_len(const GatherCsrArgs &a, int r, int m) {
  if (r >= m) return 0;
  const int pos = a.kept_pos ? a.kept_pos[r] : r;
  const long long id = a.idx ? a.idx[pos] : pos;
  return (int)(a.rowptr[id + 1] - a.rowptr[id]);
}

__global__ __launch_bounds__(kCsrTile) void k_csr_tile_sums(const GatherCsrArgs a,
                                                            long long *tile_sum) {
  __shared__ int s_int[40];
  const int m = min(max(*a.kept_count, 0), a.max_rows);
  int total;
  (void)block_exclusive_scan(kept_row_len(a, blockIdx.x * kCsrTile + threadIdx.x, m), s_int, &total);
  if (threadIdx.x == 0) tile_sum[blockIdx.x] = total;
}

__global__ __launch_bounds__(1024) void k_csr_scan_tiles(long long *tile_sum, int ntiles) {
  __shared__ long long s_part[16];
  long long running = 0;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int t0 = 0; t0 < ntiles; t0 += 1024) {
    const int t = t0 + threadIdx.x;
    const long long v = t < ntiles ? tile_sum[t] : 0;
    long long incl = v;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
      const long long up = __shfl_up(incl, off, kWave);
      if (lane >= off) incl += up;
    }
    if (lane == 63) s_part[wave] = incl;
    __syncthreads();
    long long base = 0, sum = 0;
    for (int i = 0; i < 16; ++i) {
      if (i < wave) base += s_part[i];
      sum += s_part[i];
    }
    __syncthreads();
    if (t < ntiles) tile_sum[t] = running + base + incl - v;
    running += sum;
  }
}

__global__ __launch_bounds__(kCsrTile) void k_csr_rowptr_tiles(const GatherCsrArgs a,
                                                               const long long *tile_off) {
  __shared__ int s_int[40];
  const int m = min(max(*a.kept_count, 0), a.max_rows);
  const int r = blockIdx.x * kCsrTile + threadIdx.x;
  const int len = kept_row_len(a, r, m);
  int total;
  const int excl = block_exclusive_scan(len, s_int, &total);
  if (r == 0) a.out_rowptr[0] = 0;
  if (r < m) a.out_rowptr[r + 1] = tile_off[blockIdx.x] + excl + len;
}

// A wave takes 64 kept rows at a time: every lane fetches the extent of one row (position, id,
// row pointers, output offset: one dependent chain for all 64), then groups of 16 lanes copy the
// rows four at a time.  A lane moves four consecutive entries with one 128-bit load and one
// 128-bit store per array (dword-aligned: rows start anywhere), so a row of up to 64 entries
// is one instruction per array and direction; its last one to three entries go singly.  The
// loads of the next four rows leave before the stores of these four.
typedef int i4v __attribute__((ext_vector_type(4), aligned(4)));
typedef float f4v __attribute__((ext_vector_type(4), aligned(4)));

__global__ __launch_bounds__(256) void k_csr_copy(const GatherCsrArgs a) {
  const int m = min(max(*a.kept_count, 0), a.max_rows);
  const int lane = threadIdx.x & 63, grp = lane >> 4, sub = lane & 15;
  const int wave = (blockIdx.x * 256 + threadIdx.x) >> 6, nwaves = (gridDim.x * 256) >> 6;
  const bool with_val = a.val && a.out_val;
  struct Piece {  // up to four entries of one row, in registers between their load and their store
    i4v c;
    f4v v;
    long long o;  // where they go
    int n;        // how many there are (0: none)
  };
  auto fetch = [&](long long e0, long long o0, int len, int e, Piece &p) __attribute__((always_inline)) {
    p.n = min(4, len - e);
    p.o = o0 + e;
    if (p.n == 4) {
      p.c = *reinterpret_cast<const i4v *>(a.col + e0 + e);
      if (with_val) p.v = *reinterpret_cast<const f4v *>(a.val + e0 + e);
    } else {
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        if (k < p.n) {
          p.c[k] = a.col[e0 + e + k];
          if (with_val) p.v[k] = a.val[e0 + e + k];
        }
      }
    }
  };
  auto put = [&](const Piece &p) __attribute__((always_inline)) {
    if (p.n == 4) {
      *reinterpret_cast<i4v *>(a.out_col + p.o) = p.c;
      if (with_val) *reinterpret_cast<f4v *>(a.out_val + p.o) = p.v;
    } else {
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        if (k < p.n) {
          a.out_col[p.o + k] = p.c[k];
          if (with_val) a.out_val[p.o + k] = p.v[k];
        }
      }
    }
  };
  for (int base = wave * kWave; base < m; base += nwaves * kWave) {
    const int r = base + lane;
    long long e0_l = 0, o0_l = 0;
    int len_l = 0;
    if (r < m) {
      const int pos = a.kept_pos ? a.kept_pos[r] : r;
      const long long id = a.idx ? a.idx[pos] : pos;
      e0_l = a.rowptr[id];
      len_l = (int)(a.rowptr[id + 1] - e0_l);
      o0_l = a.out_rowptr[r];
      if (o0_l + len_l > a.out_nnz_cap) len_l = 0;  // a row that does not fit is not copied
    }
    const int cnt = min(kWave, m - base);
    const int iters = (cnt + 3) / 4;
    Piece next;
    fetch(__shfl(e0_l, grp, kWave), __shfl(o0_l, grp, kWave), __shfl(len_l, grp, kWave), sub * 4, next);
    for (int it = 0; it < iters; ++it) {
      const int li = it * 4 + grp;
      const long long e0 = __shfl(e0_l, li, kWave), o0 = __shfl(o0_l, li, kWave);
      const int len = __shfl(len_l, li, kWave);  // rows past the batch's end have length 0
      const Piece now = next;
      const int ln = min(li + 4, kWave - 1);
      const int len_n = it + 1 < iters ? __shfl(len_l, ln, kWave) : 0;
      fetch(__shfl(e0_l, ln, kWave), __shfl(o0_l, ln, kWave), len_n, sub * 4, next);
      put(now);
      for (int e = 64 + sub * 4; e < len; e += 64) {  // rows of more than 64 entries
        Piece more;
        fetch(e0, o0, len, e, more);
        put(more);
      }
    }
  }
}

}  // namespace

hipError_t launch_keep_flags(const KeepArgs &a, int source, hipStream_t st) {
  if (a.P <= 0) return hipSuccess;
  const dim3 grid((a.P + 255) / 256), block(256);
  if (source == kFromProb)
    hipLaunchKernelGGL((k_keep_flags<kFromProb>), grid, block, 0, st, a);
  else
    hipLaunchKernelGGL((k_keep_flags<kFromCrit>), grid, block, 0, st, a);
  return hipGetLastError();
}

hipError_t launch_compact(CompactArgs c, int32_t *tile_off_scratch, hipStream_t st) {
  if (c.P <= 0) {
    if (c.kept_count) hipLaunchKernelGGL(k_set_i32, dim3(1), dim3(1), 0, st, c.kept_count, 0);
    return hipGetLastError();
  }
  const int ntiles = compact_tiles(c.P);
  c.tile_off = nullptr;
  if (c.P > kDirectCountMax) {
    hipLaunchKernelGGL(k_tile_counts, dim3(ntiles), dim3(256), 0, st, c.flags, c.P,
                       tile_off_scratch);
    hipLaunchKernelGGL(k_scan_tiles, dim3(1), dim3(1024), 0, st, tile_off_scratch, ntiles);
    c.tile_off = tile_off_scratch;
  }
  hipLaunchKernelGGL(k_compact, dim3(ntiles), dim3(256), 0, st, c);
  return hipGetLastError();
}

hipError_t launch_gather(const GatherArgs &a, hipStream_t st) {
  if (a.max_rows <= 0) return hipSuccess;
  if (a.src == nullptr || a.row_bytes == 0) {
    if (!a.kept_ids) return hipSuccess;
    int nb = (a.max_rows + 255) / 256;
    if (nb > 1024) nb = 1024;
    hipLaunchKernelGGL(k_gather_ids, dim3(nb), dim3(256), 0, st, a);
    return hipGetLastError();
  }
  const uintptr_t bits = reinterpret_cast<uintptr_t>(a.src) | reinterpret_cast<uintptr_t>(a.dst) |
                         (uintptr_t)a.row_bytes;
  if ((bits & 3) == 0 && a.row_bytes <= 256) {
    const int words = (int)(a.row_bytes / 4);
    long long nb = ((long long)a.max_rows * words + 255) / 256;
    if (nb > 256 * 16) nb = 256 * 16;
    hipLaunchKernelGGL(k_gather_words, dim3((unsigned)nb), dim3(256), 0, st, a, words);
    return hipGetLastError();
  }
  const int vec = (bits & 15) == 0 ? 16 : ((bits & 3) == 0 ? 4 : 1);
  const int unroll = (vec == 16 && a.row_bytes > 8192) ? 4 : 1;
  const long long chunk = vec == 16 ? 4096ll * unroll : 4096ll;
  const long long cpr = (a.row_bytes + chunk - 1) / chunk;
  long long want = (long long)a.max_rows * cpr;
  if (want > 256 * 16) want = 256 * 16;
  const dim3 grid((unsigned)want), block(256);
  if (vec == 16 && unroll == 4)
    hipLaunchKernelGGL((k_gather_rows<16, 4>), grid, block, 0, st, a, (int)cpr, chunk);
  else if (vec == 16)
    hipLaunchKernelGGL((k_gather_rows<16, 1>), grid, block, 0, st, a, (int)cpr, chunk);
  else if (vec == 4)
    hipLaunchKernelGGL((k_gather_rows<4, 1>), grid, block, 0, st, a, (int)cpr, chunk);
  else
    hipLaunchKernelGGL((k_gather_rows<1, 1>), grid, block, 0, st, a, (int)cpr, chunk);
  return hipGetLastError();
}

hipError_t launch_gather_csr(const GatherCsrArgs &a, long long *tile_scratch, hipStream_t st) {
  if (a.max_rows <= kCsrTile || !tile_scratch) {
    hipLaunchKernelGGL(k_csr_rowptr, dim3(1), dim3(1024), 0, st, a);
  } else {
    const int ntiles = (a.max_rows + kCsrTile - 1) / kCsrTile;
    hipLaunchKernelGGL(k_csr_tile_sums, dim3(ntiles), dim3(kCsrTile), 0, st, a, tile_scratch);
    hipLaunchKernelGGL(k_csr_scan_tiles, dim3(1), dim3(1024), 0, st, tile_scratch, ntiles);
    hipLaunchKernelGGL(k_csr_rowptr_tiles, dim3(ntiles), dim3(kCsrTile), 0, st, a, tile_scratch);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || a.max_rows <= 0) return e;
  int nb = (a.max_rows + 255) / 256;   // 64 rows per wave, four waves per block
  if (nb > 256 * 8) nb = 256 * 8;
  hipLaunchKernelGGL(k_csr_copy, dim3(nb), dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace aa
