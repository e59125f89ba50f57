// General row passes: CSR rows, and dense rows the register-resident kernels
// cannot take (d > 2048, d % 4 != 0, unaligned).  A group of GL lanes walks the
// stored entries of a row; phi and w are read through the caches (they are the
// only reused data); gradient sums go into dense fp32 accumulators that a second
// kernel folds into the model.  Every block first sums what it can in an LDS table
// of its own -- the first columns have a slot each (frequency-ranked column ids,
// the usual layout of bag-of-words data, put the hot columns there), any other
// column claims a slot by hash, first come first served.  At the end the first
// columns leave the block as plain stores into a per-block array that the second
// kernel sums (nearly every block touches nearly every one of them, so atomics
// would buy nothing), the hashed slots as one atomic each.
// In bag-of-words data a few hot columns take most of the entries, and device-wide
// atomics on one address run one after the other, about 13 ns each on MI355X: the
// table turns the thousands of adds a block would send to a hot column into one.
// Columns that find their slots taken add to HBM directly, which the chip
// sustains at about 20 G atomics/s on scattered addresses.
#include "aa_compact.hpp"
#include "aa_general.hpp"

namespace aa {

namespace {

template <int WIDTH>
__device__ __forceinline__ float gsum(float v) {
#pragma unroll
  for (int off = WIDTH / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

// Per-block LDS table: kDirect* slots for columns 0..kDirect*-1, then kHashed* slots
// claimed by hash (a column tag each); one sum per slot and updated vector.
// 112 KB with both vectors, 128 KB with one: one block of 16 waves per compute unit.
constexpr int kDirectTwoVec = 8192, kHashedTwoVec = 4096;
constexpr int kDirectOneVec = 16384, kHashedOneVec = 8192;
constexpr int kGradThreads = 1024, kPoolThreads = 256;

template <int GL, int MODE, bool CSR>
__global__ __launch_bounds__(1024) void k_rows_general(const GenArgs a) {
  constexpr bool POOL = (MODE & kPool) != 0;
  constexpr bool SVM = (MODE & kSvm) != 0;
  constexpr bool ASSIST = (MODE & kAssist) != 0;
  constexpr bool HARD = (MODE & kHard) != 0;  // keep by the row's own loss, no Assistant
  constexpr bool GRAD = SVM || ASSIST;
  constexpr bool NEED_PHI = (POOL && !HARD) || ASSIST;
  constexpr int G = kWave / GL;
  constexpr int NVEC = (SVM ? 1 : 0) + (ASSIST ? 1 : 0);
  constexpr int D = NVEC == 2 ? kDirectTwoVec : kDirectOneVec;  // slots 0..D-1: column = slot
  constexpr int H = NVEC == 2 ? kHashedTwoVec : kHashedOneVec;  // slots D..D+H-1: by hash
  __shared__ int s_tag[GRAD ? H : 1];
  __shared__ float s_sum[GRAD ? NVEC * (D + H) : 1];
  float *const s_w = s_sum, *const s_p = s_sum + (SVM ? D + H : 0);
  const int salt = (int)((blockIdx.x * 0x9E3779B1u) >> 19) & (H - 1);
  if (GRAD) {
    for (int k = threadIdx.x; k < H; k += blockDim.x) s_tag[k] = -1;
    for (int k = threadIdx.x; k < NVEC * (D + H); k += blockDim.x) s_sum[k] = 0.f;
    __syncthreads();
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int grp = lane / GL, sub = lane % GL;

  int total = a.count_max;
  if (!POOL && a.m_dev) total = min(max(*a.m_dev, 0), a.count_max);
  const int nwaves = gridDim.x * nw, gwave = blockIdx.x * nw + wave;
  const int per = total / nwaves, rem = total % nwaves;
  const int lo = gwave * per + min(gwave, rem);
  const int hi = lo + per + (gwave < rem ? 1 : 0);

  const float b = (NEED_PHI && a.bias) ? *a.bias : 0.f;
  const float T = (ASSIST || HARD) ? *a.T : 0.f;
  float gb = 0.f;
  int kept = 0;

  for (int base = lo; base < hi; base += kWave) {
    const int cnt = min(kWave, hi - base);
    const int j_l = base + lane;
    int row_l = 0;
    long long e0_l = 0;
    int len_l = 0;
    float y_l = 0.f, u_l = 2.f, lin_l = 0.f;
    if (lane < cnt) {
      row_l = a.rows ? a.rows[j_l] : j_l;
      if (CSR) {
        e0_l = a.rowptr[row_l];
        len_l = (int)(a.rowptr[row_l + 1] - e0_l);
      } else {
        e0_l = (long long)row_l * a.ld;
        len_l = a.d;
      }
      if (SVM) y_l = a.y[row_l];
      if (POOL && a.do_keep) u_l = keep_uniform(a.key, (uint32_t)j_l);
      if (ASSIST && !SVM) lin_l = a.loss_in[j_l];
    }
    const int iters = (cnt + G - 1) / G;
    for (int it = 0; it < iters; ++it) {
      const int li = it * G + grp;
      const bool live = li < cnt;
      const int j = base + li;
      const long long e0 = __shfl(e0_l, li, kWave);
      const int len_any = __shfl(len_l, li, kWave);  // every lane takes part in the shuffle
      const int len = live ? len_any : 0;
      const float u = __shfl(u_l, li, kWave);
      const float yy = __shfl(y_l, li, kWave);
      const float lin = __shfl(lin_l, li, kWave);
      float dp = 0.f, dw = 0.f;
      // kUnroll entries per lane at a time: their column and value loads leave together, then
      // the model gathers that depend on the columns (the chain that bounds this loop)
      constexpr int kUnroll = 8;
      for (int e = sub; e < len; e += GL * kUnroll) {
        int c[kUnroll];
        float xv[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
          const int eu = e + u * GL;
          const bool in = eu < len;
          c[u] = CSR ? (in ? a.col[e0 + eu] : 0) : (in ? eu : 0);
          xv[u] = in ? (CSR ? (a.val ? a.val[e0 + eu] : 1.f) : a.x[e0 + eu]) : 0.f;
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
          if (NEED_PHI) dp = __fmaf_rn(a.phi[c[u]], xv[u], dp);
          if (SVM) dw = __fmaf_rn(a.w[c[u]], xv[u], dw);
        }
      }
      float g = 0.f;
      bool keep = live;
      if (NEED_PHI) {
        dp = gsum<GL>(dp);
        const float s = dp + b;
        g = sigmoidf_(s);
        if (POOL) {
          if (a.do_keep) keep = live && keep_decision(u, g, a.gamma, a.one_minus_gamma);
          if (sub == 0 && live) {
            if (a.logit) a.logit[j] = s;
            if (a.prob) a.prob[j] = g;
            if (a.flags) a.flags[j] = keep ? 1 : 0;
          }
        }
      }
      if (GRAD) {
        float loss = lin;
        float cw = 0.f, resid = 0.f;
        if (SVM) {
          dw = gsum<GL>(dw);
          const float marg = yy * dw;
          loss = fmaxf(0.f, 1.f - marg);
          if (HARD) {  // shrinking by the objective value itself
            keep = live && loss > T;
            if (sub == 0 && live && a.flags) a.flags[j] = keep ? 1 : 0;
          }
          if (sub == 0 && (HARD ? live : keep) && a.loss_out) a.loss_out[j] = loss;
          cw = (keep && marg < 1.f) ? yy : 0.f;
        }
        if (ASSIST) {
          const float z = loss > T ? 1.f : 0.f;
          resid = keep ? g - z : 0.f;
          if (sub == 0) gb += resid;
        }
        if (sub == 0 && keep) kept += 1;
        if (cw != 0.f || resid != 0.f) {
          for (int e = sub; e < len; e += GL) {
            const int c = CSR ? a.col[e0 + e] : e;
            const float xv = CSR ? (a.val ? a.val[e0 + e] : 1.f) : a.x[e0 + e];
            int slot = -1;
            if (c < D) {
              slot = c;
            } else {  // claim a slot for this column, or find the one it already holds
              int h = (c ^ (c >> 13) ^ salt) & (H - 1);
              int old = atomicCAS(s_tag + h, -1, c);
              if (old == -1 || old == c) {
                slot = D + h;
              } else {
                h = (h + 1) & (H - 1);
                old = atomicCAS(s_tag + h, -1, c);
                if (old == -1 || old == c) slot = D + h;
              }
            }
            if (slot >= 0) {  // LDS and HBM atomics are different instructions: branch, not select
              if (SVM && cw != 0.f) unsafeAtomicAdd(s_w + slot, cw * xv);
              if (ASSIST && resid != 0.f) unsafeAtomicAdd(s_p + slot, resid * xv);
            } else {
              if (SVM && cw != 0.f) unsafeAtomicAdd(a.acc_w + c, cw * xv);
              if (ASSIST && resid != 0.f) unsafeAtomicAdd(a.acc_p + c, resid * xv);
            }
          }
        }
      }
    }
  }

  if (GRAD) {
    __syncthreads();
    // the first columns: this block's sums, zeros included, as plain stores
    float *const mine = a.part + (size_t)blockIdx.x * NVEC * a.head;
    for (int k = threadIdx.x; k < a.head; k += blockDim.x) {
      if (SVM) mine[k] = s_w[k];
      if (ASSIST) mine[(SVM ? a.head : 0) + k] = s_p[k];
    }
    for (int k = D + threadIdx.x; k < D + H; k += blockDim.x) {
      const int c = s_tag[k - D];
      if (c < 0) continue;
      if (SVM) {
        const float v = s_w[k];
        if (v != 0.f) unsafeAtomicAdd(a.acc_w + c, v);
      }
      if (ASSIST) {
        const float v = s_p[k];
        if (v != 0.f) unsafeAtomicAdd(a.acc_p + c, v);
      }
    }
    // scalars[0] = kept count (int), scalars[1] = bias gradient (float bits via atomics)
    int kw = kept;
    float gbw = gb;
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
      kw += __shfl_xor(kw, off, kWave);
      gbw += __shfl_xor(gbw, off, kWave);
    }
    if (lane == 0) {
      if (kw) atomicAdd(a.acc_cnt, kw);
      if (ASSIST && gbw != 0.f) unsafeAtomicAdd(a.acc_gb, gbw);
    }
  }
}

__global__ __launch_bounds__(256) void k_zero_f32(float *p, size_t count) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count;
       i += (size_t)gridDim.x * blockDim.x)
    p[i] = 0.f;
}

// Folds the gradient sums into the model.  Blocks [0, nh): 16 of the first `head` columns each,
// 16 threads per column adding the per-block sums of the pass in a fixed order; blocks after
// them: the other columns, whose sums are the atomic accumulators; then one block per
// compaction tile.
constexpr int kHeadCols = 16;

__global__ __launch_bounds__(256) void k_apply_general(const ApplyArgs a, int nh, int nrest) {
  __shared__ int s_int[40];
  __shared__ float s_part[2][16][kHeadCols];
  if ((int)blockIdx.x >= nh + nrest) {
    CompactArgs c;
    c.flags = a.flags;
    c.P = a.P;
    c.idx = a.idx;
    c.kept_pos = a.kept_pos;
    c.kept_ids = a.kept_ids;
    c.loss_pool = a.loss_pool;
    c.loss = a.loss;
    c.kept_count = a.kept_count;
    c.tile_off = nullptr;
    tile_compact(c, (int)blockIdx.x - nh - nrest, s_int);
    return;
  }
  const int m = a.m_dev ? min(max(*a.m_dev, 0), a.m_max) : *a.acc_cnt;
  if (blockIdx.x == 0 && threadIdx.x == 0 && a.kept_hist) *a.kept_hist = m;
  const float inv_m = m > 0 ? 1.f / (float)m : 0.f;
  const float shrink = 1.f - a.lr * a.lambda, scale = a.lr * inv_m;
  // one column: sums gw / gp -> new w, new phi (m == 0: the model stays, its copy is still due)
  auto fold = [&](int k, float gw, float gp) {
    if (m <= 0) {
      if (a.phi && a.phi_copy) a.phi_copy[k] = a.phi[k];
      return;
    }
    if (a.w) a.w[k] = __fmaf_rn(scale, gw, shrink * a.w[k]);
    if (a.phi) {
      const float ph = a.phi[k];
      const float pn = ph - a.lr_a * __fmaf_rn(a.l2_a, ph, gp * inv_m);
      a.phi[k] = pn;
      if (a.phi_copy) a.phi_copy[k] = pn;
    }
  };
  if ((int)blockIdx.x < nh) {
    const int cl = threadIdx.x & (kHeadCols - 1), q = threadIdx.x >> 4;
    const int k = blockIdx.x * kHeadCols + cl;
    float sw = 0.f, sp = 0.f;
    if (k < a.head && m > 0) {
      const size_t stride = (size_t)a.nvec * a.head;
      const float *pw = a.part + k, *pp = a.part + (a.w ? a.head : 0) + k;
#pragma unroll 4
      for (int b = q; b < a.nblk_pass; b += 16) {
        if (a.w) sw += pw[b * stride];
        if (a.phi) sp += pp[b * stride];
      }
    }
    s_part[0][q][cl] = sw;
    s_part[1][q][cl] = sp;
    __syncthreads();
    if (q == 0 && k < a.head) {
      float gw = a.w ? a.acc_w[k] : 0.f, gp = a.phi ? a.acc_p[k] : 0.f;
      for (int i = 0; i < 16; ++i) {
        gw += s_part[0][i][cl];
        gp += s_part[1][i][cl];
      }
      fold(k, gw, gp);
    }
  } else {
    for (int k = a.head + ((int)blockIdx.x - nh) * blockDim.x + threadIdx.x; k < a.d;
         k += nrest * blockDim.x)
      fold(k, a.w ? a.acc_w[k] : 0.f, a.phi ? a.acc_p[k] : 0.f);
  }
  if (blockIdx.x == 0 && threadIdx.x == 0 && a.phi && a.bias) {
    const float bn = m > 0 ? *a.bias - a.lr_a * (*a.acc_gb * inv_m) : *a.bias;
    if (m > 0) *a.bias = bn;
    if (a.bias_copy) *a.bias_copy = bn;
  }
}

template <int GL, bool CSR>
hipError_t launch_gl(const GenArgs &a, int mode, int nblk, hipStream_t st) {
  const dim3 grid(nblk), block(mode == kPool ? kPoolThreads : kGradThreads);
  switch (mode) {
    case kPool:
      hipLaunchKernelGGL((k_rows_general<GL, kPool, CSR>), grid, block, 0, st, a);
      break;
    case kSvm:
      hipLaunchKernelGGL((k_rows_general<GL, kSvm, CSR>), grid, block, 0, st, a);
      break;
    case kAssist:
      hipLaunchKernelGGL((k_rows_general<GL, kAssist, CSR>), grid, block, 0, st, a);
      break;
    case kSvm | kAssist:
      hipLaunchKernelGGL((k_rows_general<GL, kSvm | kAssist, CSR>), grid, block, 0, st, a);
      break;
    case kPool | kSvm | kAssist:
      hipLaunchKernelGGL((k_rows_general<GL, kPool | kSvm | kAssist, CSR>), grid, block, 0, st, a);
      break;
    case kPool | kSvm | kHard:
      hipLaunchKernelGGL((k_rows_general<GL, kPool | kSvm | kHard, CSR>), grid, block, 0, st, a);
      break;
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace

int32_t general_pass_blocks(int32_t count, bool csr, int mode) {
  // Gradient passes flush a private LDS table per block, so they take few, fat blocks (one
  // per compute unit); the scoring pass has no such cost and takes many thin ones.
  const bool grad = (mode & (kSvm | kAssist)) != 0;
  const int waves = (grad ? kGradThreads : kPoolThreads) / kWave;
  const int rows_per_block = waves * (csr ? 4 : 1);
  const int cap = grad ? kGeneralGradBlocks : 256 * 16;
  int64_t want = ((int64_t)count + rows_per_block - 1) / rows_per_block;
  if (want > cap) want = cap;
  if (want < 1) want = 1;
  return (int32_t)want;
}

hipError_t launch_general_pass(const GenArgs &a, int mode, bool csr, int32_t nblk,
                               hipStream_t st) {
  if (csr) return launch_gl<16, true>(a, mode, nblk, st);
  return launch_gl<64, false>(a, mode, nblk, st);
}

hipError_t launch_zero_f32(float *p, size_t count, hipStream_t st) {
  if (count == 0) return hipSuccess;
  size_t blocks = (count + 1023) / 1024;
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(k_zero_f32, dim3((unsigned)blocks), dim3(256), 0, st, p, count);
  return hipGetLastError();
}

int32_t general_head_columns(int32_t d, int nvec) {
  const int direct = nvec == 2 ? kDirectTwoVec : kDirectOneVec;
  return d < direct ? d : direct;
}

hipError_t launch_general_apply(const ApplyArgs &a, hipStream_t st) {
  const int nh = (a.head + kHeadCols - 1) / kHeadCols;
  int nrest = (a.d - a.head + 1023) / 1024;
  if (nrest > 1024) nrest = 1024;
  if (nrest < 0) nrest = 0;
  if (nh + nrest < 1) nrest = 1;
  hipLaunchKernelGGL(k_apply_general, dim3(nh + nrest + (a.flags ? compact_tiles(a.P) : 0)), dim3(256),
                     0, st, a, nh, nrest);
  return hipGetLastError();
}

}  // namespace aa
