// General row passes: CSR rows, and dense rows the register-resident kernels
// cannot take (d > 2048, d % 4 != 0, unaligned).  A group of GL lanes walks the
// stored entries of a row; phi and w are read through the caches (they are the
// only reused data; a gradient pass keeps their first entries in LDS); a second
// kernel folds the gradient sums into the model.
// Device-wide fp32 atomics are what such a pass must avoid on MI355X: about 20 G/s
// on scattered addresses, and adds to one address run one after the other, about
// 13 ns each, while bag-of-words data puts most entries on a few hot columns.  So:
//  * the first columns (frequency-ranked column ids, the usual layout of such data,
//    put the hot ones there) have a slot each in an LDS table of the block and leave
//    it as plain stores into a per-block array that the second kernel sums;
//  * any other column may claim one of a few thousand hashed LDS slots, first come
//    first served (a hot column outside the first ones -- a bias-like feature at the
//    end, the head of a second vocabulary -- comes early and keeps its slot);
//  * entries that find their slot taken are collected as records in LDS and written,
//    sorted by column bin, into per-bin arrays, and so are the hashed slots at the
//    end; the block that owns a bin in the second kernel sums its records in LDS.
//    One integer atomic per block, bin and flush reserves the space.  The buffer is
//    emptied whenever the block finds it half full after 8 rows per wave;
//  * only what does not fit (records beyond the LDS buffer or a bin's capacity, or
//    more columns than the bins can cover) is added to dense accumulators in HBM.
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

// Per-block LDS: kDirect* slots for columns 0..kDirect*-1 (one sum per updated vector) and as
// many entries of the model vectors themselves, kHashed* slots with a column tag each, and a
// buffer of kRecords* records.  About 154 KB: one block of 16 waves per compute unit.
// The sums are doubles: on MI355X `ds_add_f32` retires about one lane every three cycles,
// `ds_add_f64` three lanes a cycle (measured, scattered addresses), and the sums come out
// closer to exact.
constexpr int kDirectTwoVec = 3072, kHashedTwoVec = 1024, kRecordsTwoVec = 5120;
// (dense rows keep the older split: with the sizes above their kernels need more registers
// than a block of 1024 threads has, and a dense row fills the table before anything else)
constexpr int kDirectTwoVecDense = 4096, kRecordsTwoVecDense = 3072;
constexpr int kDirectOneVec = 8192, kHashedOneVec = 2048, kRecordsOneVec = 4096;
constexpr int kGradThreads = 1024, kPoolThreads = 256;
constexpr int kCheckRows = 8;  // rows per wave between two looks at the record buffer (4: 2 to 4 % slower, 16: the buffer overflows)

__device__ __forceinline__ int bin_of(int c, int head, const BinPlan &p) {
  return ((c - head) >> p.group_log2) & (p.nb - 1);
}

// Adds one entry's terms to the dense accumulators in HBM (the path of last resort).  They
// are doubles like every other sum of entries: which entries end up here depends on timing,
// so their sum must not round before it meets the rest of the column's total.
template <bool SVM, bool ASSIST>
__device__ __forceinline__ void add_global(const GenArgs &a, int c, double ta, double tb) {
  // tells the owner of the column's bin to read its columns' accumulators at all (an entry
  // that goes this way must not make every owner read every accumulator)
  if (a.plan.nb > 0) a.acc_used[bin_of(c, a.head, a.plan)] = 1;
  if (SVM && ta != 0.0) unsafeAtomicAdd(a.acc_w + c, ta);
  if (ASSIST) {
    const double t = SVM ? tb : ta;
    if (t != 0.0) unsafeAtomicAdd(a.acc_p + c, t);
  }
}

// Empties the block's record buffer -- and with HASHED its hashed slots -- into the bins.
// Whole block; the caller has put a barrier between the last append and this call.
// Which columns win a hashed slot depends on the order in which the waves arrive, so a slot's
// sum must leave the block without rounding: it goes out as a record of its own kind that
// carries the double itself (one per updated vector).  The bin owner adds every record of a
// column in doubles, so a column's total does not depend on how its entries were split
// between slots and records.
template <int R, int H, bool SVM, bool ASSIST, bool HASHED>
__device__ __forceinline__ void flush_records(const GenArgs &a, int head, const int *s_rc,
                                              const float *s_ra, const float *s_rb, int *s_nrec,
                                              const int *s_tag, const double *s_ha,
                                              const double *s_hb, int *s_hist, int *s_base) {
  constexpr int kVec = (SVM && ASSIST) ? 2 : 1;
  constexpr int kPerR = R / kGradThreads, kPerH = HASHED ? kVec * H / kGradThreads : 0;
  constexpr int kPer = kPerR + kPerH;
  // the kind of the q-th record of a thread: 0 two float terms, 1 + v the double of vector v
  auto kind_of = [](int q) { return q < kPerR ? 0 : 1 + ((q - kPerR) * kGradThreads) / H; };
  static_assert(R % kGradThreads == 0 && H % kGradThreads == 0, "whole turns of the block");
  const int n = min(*s_nrec, R);
  const int nb = a.plan.nb;
  for (int t = threadIdx.x; t < nb; t += blockDim.x) s_hist[t] = 0;
  __syncthreads();
  // The q-th record of this thread: its column (-1: none) and its second and third words.
  // (Read from LDS again after the places are known rather than kept in registers across the
  // two barriers: only the ranks stay.)
  auto record = [&](int q, int &wa, int &wb) __attribute__((always_inline)) {
    const int i = threadIdx.x + q * kGradThreads;
    int c = -1;
    wa = wb = 0;
    if (q < kPerR) {
      if (i < n) {
        c = s_rc[i];
        wa = __float_as_int(s_ra[i]);
        if (SVM && ASSIST) wb = __float_as_int(s_rb[i]);
      }
    } else {
      const int slot = (i - R) & (H - 1);
      c = s_tag[slot];
      if (c >= 0) {
        const double v = kind_of(q) == 1 ? s_ha[slot] : s_hb[slot];
        wa = __double2loint(v);
        wb = __double2hiint(v);
        if (v == 0.0) c = -1;
      }
    }
    return c;
  };
  int rank[kPer];
#pragma unroll
  for (int q = 0; q < kPer; ++q) {
    int wa, wb;
    const int c = record(q, wa, wb);
    rank[q] = c >= 0 ? atomicAdd(s_hist + bin_of(c, head, a.plan), 1) : 0;
  }
  __syncthreads();
  for (int t = threadIdx.x; t < nb; t += blockDim.x) {
    const int h = s_hist[t];
    // (64-bit fill counts: they keep counting past the capacity; the base is clamped to it)
    s_base[t] = h > 0 ? (int)min(atomicAdd(a.bin_fill + t, (unsigned long long)h),
                                 (unsigned long long)a.plan.cap)
                      : 0;
  }
  __syncthreads();
#pragma unroll
  for (int q = 0; q < kPer; ++q) {
    int wa, wb;
    const int c = record(q, wa, wb);
    if (c < 0) continue;
    const int bin = bin_of(c, head, a.plan);
    const int pos = s_base[bin] + rank[q];
    const int kind = kind_of(q);
    if (pos < a.plan.cap) {
      TailRecord r;
      r.col = c;
      r.a = wa;
      r.b = wb;
      r.kind = kind;
      a.bins[(size_t)bin * a.plan.cap + pos] = r;
    } else if (kind == 0) {
      add_global<SVM, ASSIST>(a, c, __int_as_float(wa), __int_as_float(wb));
    } else {
      const double v = __hiloint2double(wb, wa);
      add_global<SVM, ASSIST>(a, c, kind == 1 ? v : 0.0, kind == 1 ? 0.0 : v);
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) *s_nrec = 0;
  __syncthreads();
}

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
  constexpr int D = NVEC == 2 ? (CSR ? kDirectTwoVec : kDirectTwoVecDense) : kDirectOneVec;  // slots 0..D-1: column = slot
  constexpr int H = NVEC == 2 ? kHashedTwoVec : kHashedOneVec;  // hashed slots
  constexpr int R = NVEC == 2 ? (CSR ? kRecordsTwoVec : kRecordsTwoVecDense) : kRecordsOneVec;  // record buffer
  __shared__ double s_sum[GRAD ? NVEC * D : 1];
  __shared__ float s_model[GRAD ? NVEC * D : 1];  // the first D entries of w and / or phi
  __shared__ int s_tag[GRAD ? H : 1];
  __shared__ double s_hs[GRAD ? NVEC * H : 1];
  __shared__ int s_rc[GRAD ? R : 1];
  __shared__ float s_rt[GRAD ? NVEC * R : 1];
  __shared__ int s_hist[GRAD ? kMaxBins : 1], s_base[GRAD ? kMaxBins : 1];
  __shared__ int s_nrec;
  __shared__ int s_cnt[16];
  __shared__ float s_gb[16];
  double *const s_w = s_sum, *const s_p = s_sum + (SVM ? D : 0);
  const float *const s_mw = s_model, *const s_mp = s_model + (SVM ? D : 0);
  float *const s_ra = s_rt, *const s_rb = s_rt + (NVEC == 2 ? R : 0);
  double *const s_ha = s_hs, *const s_hb = s_hs + (NVEC == 2 ? H : 0);
  const bool binned = GRAD && a.plan.nb > 0;
  const int salt = (int)((blockIdx.x * 0x9E3779B1u) >> 19) & (H - 1);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int grp = lane / GL, sub = lane % GL;

  int total = a.count_max;
  if (!POOL && a.m_dev) total = min(max(*a.m_dev, 0), a.count_max);
  const int nwaves = gridDim.x * nw, gwave = blockIdx.x * nw + wave;
  const int per = total / nwaves, rem = total % nwaves;
  const int lo = gwave * per + min(gwave, rem);
  const int hi = lo + per + (gwave < rem ? 1 : 0);

  // One row per lane, 64 rows per round: id, extent, label, draw, incoming loss.
  struct RowInfo {
    long long e0;
    int len;
    float y, u, lin;
  };
  auto load_rows = [&](int round) {
    RowInfo r{0, 0, 0.f, 2.f, 0.f};
    const int base = lo + round * kWave;
    const int j_l = base + lane;
    if (j_l < hi) {
      const int row_l = a.rows ? a.rows[j_l] : j_l;
      if (CSR) {
        r.e0 = a.rowptr[row_l];
        r.len = (int)(a.rowptr[row_l + 1] - r.e0);
      } else {
        r.e0 = (long long)row_l * a.ld;
        r.len = a.d;
      }
      if (SVM) r.y = a.y[row_l];
      if (POOL && a.do_keep) r.u = keep_uniform(a.key, (uint32_t)j_l);
      if (ASSIST && !SVM) r.lin = a.loss_in[j_l];
    }
    return r;
  };
  if (GRAD) {
    for (int k = threadIdx.x; k < NVEC * D; k += blockDim.x) s_sum[k] = 0.0;
    for (int k = threadIdx.x; k < min(D, a.d); k += blockDim.x) {
      if (SVM) s_model[k] = a.w[k];
      if (ASSIST) s_model[(SVM ? D : 0) + k] = a.phi[k];
    }
    for (int k = threadIdx.x; k < H; k += blockDim.x) s_tag[k] = -1;
    for (int k = threadIdx.x; k < NVEC * H; k += blockDim.x) s_hs[k] = 0.0;
    if (threadIdx.x == 0) s_nrec = 0;
    __syncthreads();
  }
  if (GRAD && a.t_upd && blockIdx.x == 0 && threadIdx.x == 0) *a.t_snap = *a.t_upd;

  const float b = (NEED_PHI && a.bias) ? *a.bias : 0.f;
  const float T = (ASSIST || HARD) ? *a.T : 0.f;
  float gb = 0.f;
  int kept = 0;

  // every wave of the grid makes the same number of rounds, so that a block can meet between them
  const int rows_max = per + (rem > 0 ? 1 : 0);
  const int rounds = (rows_max + kWave - 1) / kWave;
  for (int round = 0; round < rounds; ++round) {
    const int base = lo + round * kWave;
    const int cnt = max(0, min(kWave, hi - base));
    const RowInfo ri = load_rows(round);  // (ahead of the LDS set-up these loads only delay it: measured)
    const long long e0_l = ri.e0;
    const int len_l = ri.len;
    const float y_l = ri.y, u_l = ri.u, lin_l = ri.lin;
    // the same trip count in every wave of the block (rows past a wave's own count are idle)
    const int iters = (max(0, min(kWave, rows_max - round * kWave)) + G - 1) / G;
    constexpr int kUnroll = 8;
    constexpr bool KEEP = GRAD && CSR;  // (dense rows here are long: nothing worth keeping)
    // entries e, e + GL, ... of the row that starts at entry e0 and has len entries
    auto load_entries_at = [&](long long e0, int len, int e, int *c, float *xv) {
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const int eu = e + u * GL;
        const bool in = eu < len;
        c[u] = CSR ? (in ? a.col[e0 + eu] : 0) : (in ? eu : 0);
        xv[u] = in ? (CSR ? (a.val ? a.val[e0 + eu] : 1.f) : a.x[e0 + eu]) : 0.f;
      }
    };
    // The first kUnroll entries per lane of the NEXT group of rows are requested while this
    // group's terms are scattered, so that a group's walk starts with its entries at hand.
    int cn[KEEP ? kUnroll : 1];
    float xn[KEEP ? kUnroll : 1];
    auto prefetch_group = [&](int it) {
      const int li = min(it * G + grp, kWave - 1);
      const long long e0 = __shfl(e0_l, li, kWave);
      const int len = __shfl(len_l, li, kWave);
      load_entries_at(e0, it * G + grp < cnt ? len : 0, sub, cn, xn);
    };
    if (KEEP && iters > 0) prefetch_group(0);
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
      int c0[kUnroll];  // the first kUnroll entries of the lane stay in registers for the second walk
      float x0[kUnroll];
      auto load_entries = [&](int e, int *c, float *xv) { load_entries_at(e0, len, e, c, xv); };
      auto dot_entries = [&](const int *c, const float *xv) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
          if (GRAD) {  // the first columns of the model are in LDS
            const bool near = c[u] < D;
            if (SVM && ASSIST) {  // past the table: both values of the column with one gather
              float2 far = make_float2(0.f, 0.f);
              if (!near) far = a.wp[c[u]];
              dw = __fmaf_rn(near ? s_mw[c[u]] : far.x, xv[u], dw);
              dp = __fmaf_rn(near ? s_mp[c[u]] : far.y, xv[u], dp);
            } else {
              if (NEED_PHI) {
                const float pv = ASSIST ? (near ? s_mp[c[u]] : a.phi[c[u]]) : a.phi[c[u]];
                dp = __fmaf_rn(pv, xv[u], dp);
              }
              if (SVM) dw = __fmaf_rn(near ? s_mw[c[u]] : a.w[c[u]], xv[u], dw);
            }
          } else {
            if (NEED_PHI) dp = __fmaf_rn(a.phi[c[u]], xv[u], dp);
          }
        }
      };
      if (KEEP) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
          c0[u] = cn[u];
          x0[u] = xn[u];
        }
        dot_entries(c0, x0);
      }
      for (int e = sub + (KEEP ? GL * kUnroll : 0); e < len; e += GL * kUnroll) {
        int c[kUnroll];
        float xv[kUnroll];
        load_entries(e, c, xv);
        dot_entries(c, xv);
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
        if (KEEP && it + 1 < iters) prefetch_group(it + 1);
        // second walk: the wave's groups step together, so that lanes with an entry outside the
        // table can reserve their places in the record buffer with one LDS atomic per step
        const bool contrib = cw != 0.f || resid != 0.f;
        int steps_len = contrib ? len : 0;
#pragma unroll
        for (int off = GL; off < kWave; off <<= 1)
          steps_len = max(steps_len, __shfl_xor(steps_len, off, kWave));
        auto scatter = [&](bool active, int c, float xv) {
          const float ta = SVM ? cw * xv : resid * xv, tb = resid * xv;
          if (active && c < D) {
            if (SVM && cw != 0.f) unsafeAtomicAdd(s_w + c, (double)(cw * xv));
            if (ASSIST && resid != 0.f) unsafeAtomicAdd(s_p + c, (double)(resid * xv));
          }
          bool tail = active && c >= D;
          if (tail) {  // the column's hashed slot, if it is free or already the column's
            // (a tag changes once, from -1 to its column: a plain read settles most cases)
            auto owner_of = [&](int slot) {
              int t = s_tag[slot];
              if (t == -1) {
                const int old = atomicCAS(s_tag + slot, -1, c);
                t = old == -1 ? c : old;
              }
              return t;
            };
            int h = (c ^ (c >> 11) ^ salt) & (H - 1);
            int owner = owner_of(h);
            if (owner != c) {  // second try, elsewhere in the table
              h = (h ^ (H / 2) ^ (c >> 5)) & (H - 1);
              owner = owner_of(h);
            }
            if (owner == c) {
              if (SVM && cw != 0.f) unsafeAtomicAdd(s_ha + h, (double)ta);
              if (ASSIST && resid != 0.f) unsafeAtomicAdd((SVM ? s_hb : s_ha) + h, (double)tb);
              tail = false;
            }
          }
          if (binned) {
            const unsigned long long mask = __ballot(tail);
            if (mask != 0ull) {
              const int leader = __ffsll((long long)mask) - 1;
              int first = 0;
              if (lane == leader) first = atomicAdd(&s_nrec, __popcll(mask));
              first = __shfl(first, leader, kWave);
              if (tail) {
                const int pos = first + (int)__builtin_amdgcn_mbcnt_hi(
                                            (uint32_t)(mask >> 32),
                                            __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
                if ((unsigned)pos < (unsigned)R) {
                  s_rc[pos] = c;
                  s_ra[pos] = ta;
                  if (NVEC == 2) s_rb[pos] = tb;
                } else {
                  add_global<SVM, ASSIST>(a, c, ta, tb);
                }
              }
            }
          } else if (tail) {
            add_global<SVM, ASSIST>(a, c, ta, tb);
          }
                };
        if (KEEP) {
          // The entries held in registers go through the same stations as `scatter` above, but
          // kBatch of a lane together: their tag reads are in flight at once, then the claims,
          // then the second probes, and the wave reserves its places in the record buffer once
          // -- a handful of LDS round trips per batch, not per entry.  (All kUnroll together
          // cost more registers than there are.)
          constexpr int kBatch = 4;
#pragma unroll
          for (int u0 = 0; u0 < kUnroll; u0 += kBatch) {
            if (u0 * GL >= steps_len) break;  // (no row of the wave reaches this far)
            bool tl[kBatch];    // entry still on its way to a hashed slot or a record
            int slot[kBatch];   // hashed slot it is looking at
            int seen[kBatch];   // the tag found there
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {
              const int u = u0 + k;
              const bool active = contrib && sub + u * GL < len;
              const int c = c0[u];
              if (active && c < D) {
                if (SVM && cw != 0.f) unsafeAtomicAdd(s_w + c, (double)(cw * x0[u]));
                if (ASSIST && resid != 0.f) unsafeAtomicAdd(s_p + c, (double)(resid * x0[u]));
              }
              tl[k] = active && c >= D;
              slot[k] = (c ^ (c >> 11) ^ salt) & (H - 1);
              seen[k] = tl[k] ? s_tag[slot[k]] : 0;
            }
            auto claim = [&](int k) {  // (a tag changes once, from -1 to its column)
              if (tl[k] && seen[k] == -1) {
                const int old = atomicCAS(s_tag + slot[k], -1, c0[u0 + k]);
                seen[k] = old == -1 ? c0[u0 + k] : old;
              }
            };
#pragma unroll
            for (int k = 0; k < kBatch; ++k) claim(k);
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {  // second try, elsewhere in the table
              if (tl[k] && seen[k] != c0[u0 + k]) {
                slot[k] = (slot[k] ^ (H / 2) ^ (c0[u0 + k] >> 5)) & (H - 1);
                seen[k] = s_tag[slot[k]];
              }
            }
#pragma unroll
            for (int k = 0; k < kBatch; ++k) claim(k);
            int n_tail = 0;
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {
              const int u = u0 + k;
              if (tl[k] && seen[k] == c0[u]) {
                const float ta = SVM ? cw * x0[u] : resid * x0[u], tb = resid * x0[u];
                if (SVM && cw != 0.f) unsafeAtomicAdd(s_ha + slot[k], (double)ta);
                if (ASSIST && resid != 0.f) unsafeAtomicAdd((SVM ? s_hb : s_ha) + slot[k], (double)tb);
                tl[k] = false;
              }
              n_tail += __popcll(__ballot(tl[k]));
            }
            if (n_tail > 0) {  // (the same in every lane)
              int first = 0;
              if (binned) {
                if (lane == 0) first = atomicAdd(&s_nrec, n_tail);
                first = __shfl(first, 0, kWave);
              }
#pragma unroll
              for (int k = 0; k < kBatch; ++k) {
                const int u = u0 + k;
                const unsigned long long mask = __ballot(tl[k]);
                if (tl[k]) {
                  const float ta = SVM ? cw * x0[u] : resid * x0[u], tb = resid * x0[u];
                  const int pos = first + (int)__builtin_amdgcn_mbcnt_hi(
                                              (uint32_t)(mask >> 32),
                                              __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
                  if (binned && (unsigned)pos < (unsigned)R) {
                    s_rc[pos] = c0[u];
                    s_ra[pos] = ta;
                    if (NVEC == 2) s_rb[pos] = tb;
                  } else {
                    add_global<SVM, ASSIST>(a, c0[u], ta, tb);
                  }
                }
                first += __popcll(mask);
              }
            }
          }
        }
        for (int eb = KEEP ? GL * kUnroll : 0; eb < steps_len; eb += GL) {
          const int e = eb + sub;
          const bool active = contrib && e < len;
          int c = 0;
          float xv = 0.f;
          if (active) {
            c = CSR ? a.col[e0 + e] : e;
            xv = CSR ? (a.val ? a.val[e0 + e] : 1.f) : a.x[e0 + e];
          }
          scatter(active, c, xv);
        }
        // every kCheckRows rows per wave the block looks at its record buffer together
        if (binned && ((it + 1) * G) % kCheckRows == 0 && (it + 1 < iters || round + 1 < rounds)) {
          __syncthreads();
          const int fill = s_nrec;
          __syncthreads();
          if (fill > R / 2)
            flush_records<R, H, SVM, ASSIST, false>(a, D, s_rc, s_ra, s_rb, &s_nrec, s_tag, s_ha,
                                                    s_hb, s_hist, s_base);
        }
      }
    }
  }

  if (GRAD) {
    // kept count and bias-gradient sum of the block: wave sums, then wave order (one store per
    // block; thousands of waves adding to one address would run one after the other)
    int kw = kept;
    float gbw = gb;
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
      kw += __shfl_xor(kw, off, kWave);
      gbw += __shfl_xor(gbw, off, kWave);
    }
    if (lane == 0) {
      s_cnt[wave] = kw;
      s_gb[wave] = gbw;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      int kb = 0;
      float gbb = 0.f;
      for (int i = 0; i < nw; ++i) {
        kb += s_cnt[i];
        gbb += s_gb[i];
      }
      a.blk_cnt[blockIdx.x] = kb;
      a.blk_gb[blockIdx.x] = gbb;
    }
    if (binned) {
      flush_records<R, H, SVM, ASSIST, true>(a, D, s_rc, s_ra, s_rb, &s_nrec, s_tag, s_ha, s_hb,
                                             s_hist, s_base);
    } else {
      for (int k = threadIdx.x; k < H; k += blockDim.x) {
        const int c = s_tag[k];
        if (c >= 0)
          add_global<SVM, ASSIST>(a, c, s_ha[k], (SVM && ASSIST) ? s_hb[k] : 0.0);
      }
    }
    // the first columns: this block's sums, zeros included, as plain stores -- the last thing a
    // wave does, so that nothing waits for them (a barrier after them would)
    float *const mine = a.part + (size_t)blockIdx.x * NVEC * a.head;
    for (int k = threadIdx.x; k < a.head; k += blockDim.x) {
      if (SVM) mine[k] = (float)s_w[k];
      if (ASSIST) mine[(SVM ? a.head : 0) + k] = (float)s_p[k];
    }
  }
}

// p is 16-byte aligned: 128-bit stores, then the few floats left over.
__global__ __launch_bounds__(256) void k_zero_f32(float *p, size_t count) {
  const size_t n4 = count / 4, tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  float4 *p4 = reinterpret_cast<float4 *>(p);
  for (size_t i = tid; i < n4; i += stride) p4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  if (tid < count - 4 * n4) p[4 * n4 + tid] = 0.f;
}

// Scoring pass over CSR rows with the first kScoreTableCols entries of phi in LDS: one block of
// 16 waves per compute unit loads them once and then walks its rows; only columns past the
// table are gathered through the caches.  Pays when phi is too large for the vector L1 (a few
// thousand floats) and the rows are many: the gathers of k_rows_general then miss the L1 and
// pull a line from L2 for four bytes each.  Same outputs and the same order of additions per
// row as k_rows_general<16, kPool, true>, so the two give the same bits.
#ifndef AA_SCORE_TABLE_COLS
#define AA_SCORE_TABLE_COLS 39936
#endif
constexpr int kScoreTableCols = AA_SCORE_TABLE_COLS;  // 156 KB of the 160 KB
constexpr int kScoreTableThreads = 1024;
// Taken for pools of at least kScoreTableMinRows rows when phi is too large for the vector L1
// to serve (more than kScoreTableMinCols columns) and the table holds at least half of it:
// measured on 1,000,000 token-list rows over 64,002 columns 236 -> 161 us per launch; on
// 65,536 rows of about 100 entries over 2^20 Zipf-distributed columns, where a quarter of the
// entries lie past the table, k_rows_general stays ahead (34 us against 48).
#ifndef AA_SCORE_TABLE_MIN_COLS
#define AA_SCORE_TABLE_MIN_COLS 16384
#endif
constexpr int kScoreTableMinCols = AA_SCORE_TABLE_MIN_COLS, kScoreTableMinRows = 16384;
constexpr int kScoreTableMaxCols = 2 * kScoreTableCols;

// No load of the main loop sits behind a branch (a lane with nothing to read asks for an
// offset outside its buffer resource, which costs no memory access and reads as zero), so the
// waits the compiler places count the loads in flight exactly and never drain them: the
// entries of the row groups one and two steps ahead and the cold-column gathers of the next
// group stay outstanding while the current group is added up, and the row extents arrive a
// round (64 rows) ahead, the row ids two rounds.  Rows longer than one chunk (128 entries) are
// rare in data this kernel is for; they are skipped in the loop and walked afterwards.
template <bool VAL>
__global__ __launch_bounds__(kScoreTableThreads) void k_score_table(const GenArgs a) {
  constexpr int GL = 16, G = kWave / GL, kUnroll = 8, kChunk = GL * kUnroll;
  __shared__ float s_phi[kScoreTableCols];
  const int D = min(kScoreTableCols, a.d);
  for (int k = threadIdx.x; k < D; k += kScoreTableThreads) s_phi[k] = a.phi[k];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = kScoreTableThreads >> 6;
  const int grp = lane / GL, sub = lane % GL;
  const int total = a.count_max;
  const int nwaves = gridDim.x * nw, gwave = blockIdx.x * nw + wave;
  const int per = total / nwaves, rem = total % nwaves;
  const int lo = gwave * per + min(gwave, rem);
  const int hi = lo + per + (gwave < rem ? 1 : 0);
  const float b = a.bias ? *a.bias : 0.f;
  // an address that is always readable, for lanes with nothing to load
  const int *const nowhere = reinterpret_cast<const int *>(a.rowptr);
  __syncthreads();

  // Entries and cold columns are read through buffer resources: a lane with nothing to read
  // gives an offset past the resource's range, for which the hardware returns zero without a
  // memory access -- no stand-in addresses, no masks where the values are used (a missing entry
  // is column 0 with value 0, as in k_rows_general).  Offsets are 32 bits: rows whose entries
  // lie beyond kSpan bytes of the arrays take the walk after the loop.
  constexpr int kNone = (int)0x80000000;         // out of every resource's range
  constexpr long long kSpan = 0x7fffffffll / 4;  // entries within reach of a 32-bit byte offset
  const __amdgpu_buffer_rsrc_t r_col = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<int32_t *>(a.col), 0, kNone, 0x00020000);
  const __amdgpu_buffer_rsrc_t r_val = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<float *>(VAL ? a.val : a.phi), 0, kNone, 0x00020000);
  const __amdgpu_buffer_rsrc_t r_phi = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<float *>(a.phi), 0, a.d * 4, 0x00020000);
  struct Slot {  // one chunk per lane group
    int c[kUnroll];
    float x[kUnroll];
    float far[kUnroll];
  };
  // One half of a slot: the kHalf turns from turn u0 on hold entries [e, e + kHalfChunk) of the
  // row that starts at entry e0 and has len entries.
  constexpr int kHalf = kUnroll / 2, kHalfChunk = GL * kHalf;
  auto request_half = [&](int e0, int len, int e, int u0, Slot &t) __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < kHalf; ++u) {
      const int eu = e + sub + u * GL;
      const int off = eu < len ? (e0 + eu) * 4 : kNone;
      t.c[u0 + u] = __builtin_amdgcn_raw_buffer_load_b32(r_col, off, 0, 0);
      if (VAL)
        t.x[u0 + u] = __int_as_float(__builtin_amdgcn_raw_buffer_load_b32(r_val, off, 0, 0));
      else
        t.x[u0 + u] = eu < len ? 1.f : 0.f;
    }
  };
  auto gather = [&](Slot &t) __attribute__((always_inline)) {  // columns past the table
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
      t.far[u] = __int_as_float(
          __builtin_amdgcn_raw_buffer_load_b32(r_phi, t.c[u] >= D ? t.c[u] * 4 : kNone, 0, 0));
  };
  auto dot_half = [&](const Slot &t, int u0, float dp) __attribute__((always_inline)) {
    float near[kHalf];
#pragma unroll
    for (int u = 0; u < kHalf; ++u) near[u] = s_phi[min(t.c[u0 + u], D - 1)];
#pragma unroll
    for (int u = 0; u < kHalf; ++u)
      dp = __fmaf_rn(t.c[u0 + u] >= D ? t.far[u0 + u] : near[u], t.x[u0 + u], dp);
    return dp;
  };
  auto emit = [&](int j, float dp, float u) __attribute__((always_inline)) {
    const float s = dp + b;
    const float g = sigmoidf_(s);
    if (a.logit) a.logit[j] = s;
    if (a.prob) a.prob[j] = g;
    if (a.flags)
      a.flags[j] = (!a.do_keep || keep_decision(u, g, a.gamma, a.one_minus_gamma)) ? 1 : 0;
  };

  // raw loads of the row id of pool position j and of the extent of a row
  auto row_id = [&](int j) __attribute__((always_inline)) {
    return *((j < hi && a.rows) ? a.rows + j : nowhere);
  };
  struct Extent {
    int64_t lo, hi;
  };
  auto extent = [&](int j, int raw_id) __attribute__((always_inline)) {
    const int row = j < hi ? (a.rows ? raw_id : j) : 0;
    Extent e;
    e.lo = a.rowptr[row];
    e.hi = a.rowptr[row + 1];
    return e;
  };
  Extent cur = extent(lo + lane, row_id(lo + lane));
  Extent next = extent(lo + kWave + lane, row_id(lo + kWave + lane));
  int id_after = row_id(lo + 2 * kWave + lane);
  bool any_longer = false;

  // A step gives every group of 16 lanes two half slots of 64 entries: both chunks of one row of
  // 65 to 128 entries, or the only chunks of two rows of up to 64.  Per round the wave's 64 rows
  // are put in that order -- the longer rows, then the shorter ones, each class in pool order --
  // with one ds_permute per value, so half slot h belongs to sorted row h / 2 (chunk h % 2) while
  // h < 2 M and to sorted row h - M after that (M = number of longer rows).
  constexpr int kAhead = 3;  // steps in flight; slot (it % kAhead) holds step it of a round
  Slot t[kAhead];
  for (int base = lo; base < hi; base += kWave) {
    const float u_l = a.do_keep ? keep_uniform(a.key, (uint32_t)(base + lane)) : 2.f;
    const bool valid = base + lane < hi;
    int len_cur = valid ? (int)(cur.hi - cur.lo) : 0;
    if (cur.hi > kSpan) len_cur = kChunk + 1;  // (out of reach: a row for the walk after the loop)
    any_longer = any_longer || (valid && len_cur > kChunk);
    const bool two = valid && len_cur > kHalfChunk && len_cur <= kChunk;
    const bool one = valid && len_cur <= kHalfChunk;
    const unsigned long long m_two = __ballot(two), m_one = __ballot(one);
    const int M = __popcll(m_two), S = __popcll(m_one), H = 2 * M + S;
    auto rank_in = [&](unsigned long long mask) __attribute__((always_inline)) {
      return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                            __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
    };
    const int dest = two ? rank_in(m_two) : one ? M + rank_in(m_one) : M + S + rank_in(~(m_two | m_one));
    const int e0_s = __builtin_amdgcn_ds_permute(dest * 4, (int)cur.lo);
    const int len_s = __builtin_amdgcn_ds_permute(dest * 4, len_cur);
    const int src_s = __builtin_amdgcn_ds_permute(dest * 4, lane);
    const float u_s = __int_as_float(__builtin_amdgcn_ds_permute(dest * 4, __float_as_int(u_l)));
    const int nsteps = (H + 2 * G - 1) / (2 * G);
    // half slots (A, B) of this lane's group in step `it`: sorted row and first entry of each
    auto halves = [&](int it, int *rowA, int *rowB, bool *same) __attribute__((always_inline)) {
      const int hA = 2 * (it * G + grp), hB = hA + 1;
      *same = hB < 2 * M;
      *rowA = hA < 2 * M ? (hA >> 1) : hA - M;
      *rowB = *same ? *rowA : hB - M;
      if (hA >= H) *rowA = -1;
      if (hB >= H) *rowB = -1;
    };
    auto request_step = [&](int it, Slot &s) __attribute__((always_inline)) {
      int rowA, rowB;
      bool same;
      halves(it, &rowA, &rowB, &same);
      const int e0A = __shfl(e0_s, max(rowA, 0), kWave), lenA = __shfl(len_s, max(rowA, 0), kWave);
      const int e0B = __shfl(e0_s, max(rowB, 0), kWave), lenB = __shfl(len_s, max(rowB, 0), kWave);
      request_half(e0A, rowA >= 0 ? min(lenA, kHalfChunk) : 0, 0, 0, s);
      request_half(e0B, rowB >= 0 ? (same ? lenB : min(lenB, kHalfChunk)) : 0, same ? kHalfChunk : 0,
                   kHalf, s);
    };
    auto finish_step = [&](int it, float dpA, float dpB) __attribute__((always_inline)) {
      int rowA, rowB;
      bool same;
      halves(it, &rowA, &rowB, &same);
      dpA = gsum<GL>(dpA);
      dpB = gsum<GL>(dpB);
      const int jA = base + __shfl(src_s, max(rowA, 0), kWave), jB = base + __shfl(src_s, max(rowB, 0), kWave);
      const float uA = __shfl(u_s, max(rowA, 0), kWave), uB = __shfl(u_s, max(rowB, 0), kWave);
      if (sub == 0 && rowA >= 0 && !same) emit(jA, dpA, uA);
      if (sub == 0 && rowB >= 0) emit(jB, dpB, uB);
    };
    // the extents of the next round and the row ids of the one after go out ahead of this
    // round's entries: the only loads of a round that wait for nothing
    const Extent coming = extent(base + 2 * kWave + lane, id_after);
    id_after = row_id(base + 3 * kWave + lane);
#pragma unroll
    for (int p = 0; p < kAhead; ++p) request_step(p, t[p]);
    gather(t[0]);
    // (whole turns of the three slots: the steps past the last one hold nothing and load nothing)
#pragma unroll 1
    for (int it0 = 0; it0 < nsteps; it0 += kAhead) {
#pragma unroll
      for (int p = 0; p < kAhead; ++p) {
        gather(t[(p + 1) % kAhead]);  // step it + 1: its entries were requested two steps ago
        const int hB = 2 * ((it0 + p) * G + grp) + 1;
        const float dpA = dot_half(t[p], 0, 0.f);
        const float dpB = dot_half(t[p], kHalf, hB < 2 * M ? dpA : 0.f);  // (one row: its sum goes on)
        request_step(it0 + p + kAhead, t[p]);
        finish_step(it0 + p, dpA, dpB);
      }
    }
    cur = next;
    next = coming;
  }
  if (__ballot(any_longer) == 0ull) return;
  // rows of more than one chunk, one after the other in the wave's first lane group
  for (int base = lo; base < hi; base += kWave) {
    const int j_l = base + lane;
    const Extent e_l = extent(j_l, row_id(j_l));
    const int len_l = j_l < hi ? (int)(e_l.hi - e_l.lo) : 0;
    const float u_l = a.do_keep ? keep_uniform(a.key, (uint32_t)j_l) : 2.f;
    unsigned long long longer = __ballot(len_l > kChunk || (j_l < hi && e_l.hi > kSpan));
    while (longer != 0ull) {
      const int li = __ffsll((long long)longer) - 1;
      longer &= longer - 1;
      const long long e0 = __shfl((long long)e_l.lo, li, kWave);
      const int len = grp == 0 ? __shfl(len_l, li, kWave) : 0;
      const float u = __shfl(u_l, li, kWave);
      float dp = 0.f;
      for (int e = sub; e < len; e += GL) {  // (the order of a lane's additions is the loop's)
        const int c = a.col[e0 + e];
        const float xv = VAL ? a.val[e0 + e] : 1.f;
        dp = __fmaf_rn(c < D ? s_phi[c] : a.phi[c], xv, dp);
      }
      dp = gsum<GL>(dp);
      if (lane == 0) emit(base + li, dp, u);
    }
  }
}

// What a pass that updates both vectors needs beforehand, in one launch: the accumulators and
// the header cleared, and the two model vectors side by side for the columns past the LDS table.
__global__ __launch_bounds__(256) void k_prepare_general(float *p, size_t count, const float *w,
                                                         const float *phi, float2 *wp, int head,
                                                         int d) {
  const size_t n4 = count / 4, tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  float4 *p4 = reinterpret_cast<float4 *>(p);
  for (size_t i = tid; i < n4; i += stride) p4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  if (tid < count - 4 * n4) p[4 * n4 + tid] = 0.f;
  for (size_t c = head + tid; c < (size_t)d; c += stride) wp[c] = make_float2(w[c], phi[c]);
}

// Folds the gradient sums into the model.  Blocks [0, nh): 16 of the first `head` columns each,
// 16 threads per column adding the per-block sums of the pass in a fixed order; blocks after
// them: the other columns -- one block per bin, which adds the bin's records up in LDS (plus
// whatever overflowed into the dense accumulators), or with no bins a strided share of the
// accumulators; then one block per compaction tile.  Every block adds up the per-block kept
// counts of the pass for itself.
constexpr int kHeadCols = 16;
constexpr int kApplyThreads = 256;
static_assert(kGeneralGradBlocks <= kApplyThreads, "one per-block count of the pass per thread");

typedef float f4v __attribute__((ext_vector_type(4), aligned(4)));  // (any float address)

// The update of one column from its gradient sums (m == 0: the model stays, its copy is still due).
struct Fold {
  const ApplyArgs &a;
  int m;
  float inv_m, shrink, scale;
  __device__ Fold(const ApplyArgs &args, int m_) : a(args), m(m_), inv_m(m_ > 0 ? 1.f / (float)m_ : 0.f) {
    // step size: constant, or lr / sqrt(number of updates made, this one included)
    float lr = args.lr;
    if (args.t_upd && m_ > 0) lr = args.lr / sqrtf((float)(*args.t_snap + 1));
    shrink = 1.f - lr * args.lambda;
    scale = lr * inv_m;
  }
  // w_old, ph: the column's current values, loaded by the caller
  __device__ __forceinline__ void loaded(int k, float gw, float gp, float w_old, float ph) const {
    if (m <= 0) {
      if (a.phi && a.phi_copy) a.phi_copy[k] = ph;
      return;
    }
    const float wn = __fmaf_rn(scale, gw, shrink * w_old);
    const float pn = ph - a.lr_a * __fmaf_rn(a.l2_a, ph, gp * inv_m);
    if (a.w) a.w[k] = wn;
    if (a.phi) {
      a.phi[k] = pn;
      if (a.phi_copy) a.phi_copy[k] = pn;
    }
    if (a.wp_out) a.wp_out[k] = make_float2(wn, pn);  // (both vectors are updated then)
  }
  __device__ __forceinline__ void column(int k, float gw, float gp) const {
    loaded(k, gw, gp, a.w ? a.w[k] : 0.f, a.phi ? a.phi[k] : 0.f);
  }
  // four columns from k on (the same arithmetic per column), as 128-bit stores
  __device__ __forceinline__ void loaded4(int k, f4v gw, f4v gp, f4v w_old, f4v ph) const {
    if (m <= 0) {
      if (a.phi && a.phi_copy) *reinterpret_cast<f4v *>(a.phi_copy + k) = ph;
      return;
    }
    f4v wn, pn;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      wn[i] = __fmaf_rn(scale, gw[i], shrink * w_old[i]);
      pn[i] = ph[i] - a.lr_a * __fmaf_rn(a.l2_a, ph[i], gp[i] * inv_m);
    }
    if (a.w) *reinterpret_cast<f4v *>(a.w + k) = wn;
    if (a.phi) {
      *reinterpret_cast<f4v *>(a.phi + k) = pn;
      if (a.phi_copy) *reinterpret_cast<f4v *>(a.phi_copy + k) = pn;
    }
    if (a.wp_out) {  // (both vectors are updated then)
      const f4v lo = {wn[0], pn[0], wn[1], pn[1]}, hi = {wn[2], pn[2], wn[3], pn[3]};
      f4v *const dst = reinterpret_cast<f4v *>(a.wp_out + k);
      dst[0] = lo;
      dst[1] = hi;
    }
  }
};

// Kept count of the pass (and the sum of its bias gradients): one per-block value per thread.
__device__ __forceinline__ int pass_totals(const ApplyArgs &a, int cnt, float gbs, int *s_m,
                                           float *s_g, float *gb_out) {
  const int t = threadIdx.x;
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) {
    cnt += __shfl_xor(cnt, off, kWave);
    gbs += __shfl_xor(gbs, off, kWave);
  }
  if ((t & 63) == 0) {
    s_m[t >> 6] = cnt;
    s_g[t >> 6] = gbs;
  }
  __syncthreads();
  *gb_out = (s_g[0] + s_g[1]) + (s_g[2] + s_g[3]);
  const int m_pass = s_m[0] + s_m[1] + s_m[2] + s_m[3];
  return a.m_dev ? min(max(*a.m_dev, 0), a.m_max) : m_pass;
}

__device__ __forceinline__ int bin_local(int col, const ApplyArgs &a) {
  const int rel = col - a.head, gl = a.plan.group_log2;
  return (((rel >> gl) >> a.plan.nb_log2) << gl) | (rel & ((1 << gl) - 1));
}

__device__ __forceinline__ int bin_column(int k, int bin, const ApplyArgs &a) {
  const int gl = a.plan.group_log2;
  return a.head + (((((k >> gl) << a.plan.nb_log2) | bin) << gl) | (k & ((1 << gl) - 1)));
}

// The block that owns a bin.  Everything it needs from memory (the first records and columns
// per thread, in registers) is requested before anything is used: one round trip, not five.
__device__ __forceinline__ void apply_bin(const ApplyArgs &a, int bin, double *s_bin, int *s_m,
                                          float *s_g) {
  // per thread: kRec records per batch; kCol runs of four columns (a bin's columns come in
  // groups of at least four neighbours) -- 4 * kCol * kApplyThreads covers any bin of a pass
  // that updates two vectors, and half of the largest bin of one that updates one
  constexpr int kRec = 16, kCol = 4;
  const int tid = threadIdx.x, cols = a.plan.cols, cap = a.plan.cap;
  const int cnt = tid < a.nblk_pass ? a.blk_cnt[tid] : 0;
  const int fill = (int)min(a.bin_fill[bin], (unsigned long long)cap);
  const int acc_used = a.acc_used[bin];
  const TailRecord *rec = a.bins + (size_t)bin * cap;
  // records, four words each; two register sets, so that the loads of the next batch are in
  // flight while this one is added up
  int4 r0[kRec], r1[kRec];
  constexpr int kBatch = kRec * kApplyThreads;
  // (Every load below is unconditional: a load under a condition makes the compiler wait for
  // all loads in flight where the paths join, and the requests would go out one at a time.
  // An index past the end is clamped to the last record, whose value is then not used.)
  auto load_batch = [&](int4 *__restrict__ r, int base, int last) __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < kRec; ++u)
      r[u] = *reinterpret_cast<const int4 *>(rec + min(base + tid + u * kApplyThreads, last));
  };
  load_batch(r0, 0, cap - 1);  // past the fill count: stale, in bounds, not used
  int col[kCol];   // first column of the run, -1: none, or not all four exist (the model's end)
  f4v wo[kCol], po[kCol];
  const float *const w_src = a.w ? a.w : a.phi, *const p_src = a.phi ? a.phi : a.w;
#pragma unroll
  for (int u = 0; u < kCol; ++u) {
    const int k = 4 * (tid + u * kApplyThreads);
    int c = bin_column(k, bin, a);
    if (k >= cols || c + 4 > a.d) c = -1;
    col[u] = c;
    const int c_safe = c >= 0 ? c : a.d - 4;  // (bins exist: so do more than four columns)
    wo[u] = *reinterpret_cast<const f4v *>(w_src + c_safe);
    po[u] = *reinterpret_cast<const f4v *>(p_src + c_safe);
  }
  // A bin of few columns keeps several copies of its sums, one per lane residue, so that the
  // lanes of a wave that meet on a hot column add to different addresses (an odd stride puts
  // the copies of a column into different LDS banks).
  const int span = a.nvec * cols + 1;
  int copies = 1;
  while (copies < 16 && 2 * copies * span <= kBinColsMax) copies *= 2;
  double *const s_mine = s_bin + (tid & (copies - 1)) * span;
  for (int k = tid; k < copies * span; k += kApplyThreads) s_bin[k] = 0.0;
  float gb_unused;
  const int m = pass_totals(a, cnt, 0.f, s_m, s_g, &gb_unused);  // barrier: the sums are zero
  const Fold fold(a, m);
  const int n = min(fill, cap);
  auto add = [&](const int4 &r) {  // (x: column, y and z: the terms, w: the record's kind)
    const int k = bin_local(r.x, a);
    if (r.w == 0) {
      const float ta = __int_as_float(r.y), tb = __int_as_float(r.z);
      if (ta != 0.f) unsafeAtomicAdd(s_mine + k, (double)ta);
      if (a.nvec == 2 && tb != 0.f) unsafeAtomicAdd(s_mine + cols + k, (double)tb);
    } else {  // a hashed slot's sum: the double of one vector
      unsafeAtomicAdd(s_mine + (r.w == 2 ? cols : 0) + k, __hiloint2double(r.z, r.y));
    }
  };
  auto add_batch = [&](const int4 *r, int base) __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < kRec; ++u)
      if (base + tid + u * kApplyThreads < n) add(r[u]);
  };
  for (int base = 0; base < n; base += 2 * kBatch) {
    load_batch(r1, base + kBatch, n - 1);
    add_batch(r0, base);
    load_batch(r0, base + 2 * kBatch, n - 1);
    add_batch(r1, base + kBatch);
  }
  __syncthreads();
  auto sum_of = [&](int k) {  // over the copies, in order
    double v = 0.0;
    for (int c = 0; c < copies; ++c) v += s_bin[c * span + k];
    return v;
  };
  // (the dense accumulators hold something only if an entry found no room in LDS or in a bin);
  // a column's total is rounded to fp32 once, after everything has been added in doubles
  auto acc_w_of = [&](int c) { return (acc_used && a.w) ? a.acc_w[c] : 0.0; };
  auto acc_p_of = [&](int c) { return (acc_used && a.phi) ? a.acc_p[c] : 0.0; };
  // The runs held in registers, in three sweeps -- sums out of LDS, then (rarely) the
  // accumulators, then nothing but stores: a load between two stores would make every store
  // wait for the one before it to be acknowledged.
  double ga[kCol][4], gp[kCol][4];
#pragma unroll
  for (int u = 0; u < kCol; ++u) {
    if (4 * u * kApplyThreads >= cols) break;  // (no thread has a run this far out)
    const int k = min(4 * (tid + u * kApplyThreads), cols - 4);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const double va = sum_of(k + i), vb = a.nvec == 2 ? sum_of(cols + k + i) : va;
      ga[u][i] = a.w ? va : 0.0;
      gp[u][i] = vb;
    }
  }
  if (acc_used) {
    double *const w_acc = a.w ? a.acc_w : a.acc_p, *const p_acc = a.phi ? a.acc_p : a.acc_w;
    double xa[kCol][4], xp[kCol][4];
#pragma unroll
    for (int u = 0; u < kCol; ++u) {
      const int c_safe = col[u] >= 0 ? col[u] : a.d - 4;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        xa[u][i] = w_acc[c_safe + i];
        xp[u][i] = p_acc[c_safe + i];
      }
    }
#pragma unroll
    for (int u = 0; u < kCol; ++u) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        ga[u][i] += a.w ? xa[u][i] : 0.0;
        gp[u][i] += a.phi ? xp[u][i] : 0.0;
      }
    }
    if (a.keep_ready) {  // what was read is cleared for the next pass (this bin's columns only)
#pragma unroll
      for (int u = 0; u < kCol; ++u) {
        if (col[u] < 0) continue;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          w_acc[col[u] + i] = 0.0;
          p_acc[col[u] + i] = 0.0;
        }
      }
    }
  }
#pragma unroll
  for (int u = 0; u < kCol; ++u) {
    if (4 * u * kApplyThreads >= cols) break;
    if (col[u] < 0) continue;
    f4v fa, fp;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      fa[i] = (float)ga[u][i];
      fp[i] = (float)gp[u][i];
    }
    fold.loaded4(col[u], fa, fp, wo[u], po[u]);
  }
  // what is left: runs past the registers' reach, and the model's last columns where fewer
  // than four exist
  for (int k = tid; k < cols; k += kApplyThreads) {
    const int c = bin_column(k, bin, a);
    if (c >= a.d || (k < 4 * kCol * kApplyThreads && (c & ~3) + 4 <= a.d)) continue;
    const double va = sum_of(k), vb = a.nvec == 2 ? sum_of(cols + k) : va;
    fold.column(c, (float)(acc_w_of(c) + (a.w ? va : 0.0)), (float)(acc_p_of(c) + vb));
    if (acc_used && a.keep_ready) {
      if (a.w) a.acc_w[c] = 0.0;
      if (a.phi) a.acc_p[c] = 0.0;
    }
  }
  if (a.keep_ready && tid == 0) {  // (read at the top; the next pass counts from zero)
    a.bin_fill[bin] = 0ull;
    a.acc_used[bin] = 0;
  }
}

__global__ __launch_bounds__(kApplyThreads) void k_apply_general(const ApplyArgs a, int nh, int nrest) {
  __shared__ int s_int[40];
  __shared__ float s_part[2][16][kHeadCols];
  __shared__ int s_m[4];
  __shared__ float s_g[4];
  __shared__ double s_bin[kBinColsMax + 1];  // (+1: the odd stride of a single copy)
  // roles by block number: the other columns first (the bin owners have the longest way to
  // go), then the first columns, then the compaction tiles
  const int bid = (int)blockIdx.x, hb = bid - nrest;
  if (bid >= nh + nrest) {
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
    tile_compact(c, bid - nh - nrest, s_int);
    return;
  }
  if (bid < nrest && a.plan.nb > 0) {  // nrest == nb
    apply_bin(a, bid, s_bin, s_m, s_g);
    return;
  }
  const int t = threadIdx.x;
  const int cnt = t < a.nblk_pass ? a.blk_cnt[t] : 0;
  const float gbs = (t < a.nblk_pass && a.phi && a.bias) ? a.blk_gb[t] : 0.f;
  if (hb >= 0) {
    const int cl = t & (kHeadCols - 1), q = t >> 4;
    const int k = hb * kHeadCols + cl;
    float sw = 0.f, sp = 0.f;
    // (loads without conditions, so that they are all in flight together; with one updated
    // vector both pointers name the same sums and one of the two results is dropped)
    const int k_safe = min(k, a.head - 1);
    {  // (all zeros when nothing was kept)
      const size_t stride = (size_t)a.nvec * a.head;
      const float *pw = a.part + k_safe, *pp = a.part + (a.w ? a.head : 0) + k_safe;
#pragma unroll 8
      for (int b = q; b < a.nblk_pass; b += 16) {
        sw += pw[b * stride];
        sp += pp[b * stride];
      }
    }
    if (!a.w || k >= a.head) sw = 0.f;
    if (!a.phi || k >= a.head) sp = 0.f;
    // (the accumulators take entries of the other columns only)
    float gw = 0.f, gp = 0.f;
    const float wo = (a.w ? a.w : a.phi)[k_safe], po = (a.phi ? a.phi : a.w)[k_safe];
    s_part[0][q][cl] = sw;
    s_part[1][q][cl] = sp;
    float gb_pass;
    const int m = pass_totals(a, cnt, gbs, s_m, s_g, &gb_pass);  // barrier
    const Fold fold(a, m);
    if (hb == 0 && t == 0 && a.kept_hist) *a.kept_hist = m;
    if (hb == 0 && t == 0 && a.t_upd && m > 0) *a.t_upd = *a.t_snap + 1;
    if (q == 0 && k < a.head) {
      for (int i = 0; i < 16; ++i) {
        gw += s_part[0][i][cl];
        gp += s_part[1][i][cl];
      }
      fold.loaded(k, gw, gp, wo, po);
    }
    if (hb == 0 && t == 0 && a.phi && a.bias) {
      const float bn = m > 0 ? *a.bias - a.lr_a * (gb_pass * fold.inv_m) : *a.bias;
      if (m > 0) *a.bias = bn;
      if (a.bias_copy) *a.bias_copy = bn;
    }
  } else {
    float gb_pass;
    const int m = pass_totals(a, cnt, gbs, s_m, s_g, &gb_pass);
    const Fold fold(a, m);
    for (int k = a.head + bid * blockDim.x + t; k < a.d; k += nrest * blockDim.x)
      fold.column(k, a.w ? (float)a.acc_w[k] : 0.f, a.phi ? (float)a.acc_p[k] : 0.f);
  }
}

template <int GL, bool CSR>
hipError_t launch_gl(const GenArgs &a, int mode, int nblk, hipStream_t st, hipEvent_t e0,
                     hipEvent_t e1) {
  const dim3 grid(nblk), block(mode == kPool ? kPoolThreads : kGradThreads);
  switch (mode) {
    case kPool:
      launch_stamped((k_rows_general<GL, kPool, CSR>), grid, block, st, e0, e1, a);
      break;
    case kSvm:
      launch_stamped((k_rows_general<GL, kSvm, CSR>), grid, block, st, e0, e1, a);
      break;
    case kAssist:
      launch_stamped((k_rows_general<GL, kAssist, CSR>), grid, block, st, e0, e1, a);
      break;
    case kSvm | kAssist:
      launch_stamped((k_rows_general<GL, kSvm | kAssist, CSR>), grid, block, st, e0, e1, a);
      break;
    case kPool | kSvm | kAssist:
      launch_stamped((k_rows_general<GL, kPool | kSvm | kAssist, CSR>), grid, block, st, e0, e1, a);
      break;
    case kPool | kSvm | kHard:
      launch_stamped((k_rows_general<GL, kPool | kSvm | kHard, CSR>), grid, block, st, e0, e1, a);
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
                               hipStream_t st, hipEvent_t e0, hipEvent_t e1) {
  if (csr && mode == kPool && a.d > kScoreTableMinCols && a.d <= kScoreTableMaxCols &&
      a.count_max >= kScoreTableMinRows) {
    if (a.val)
      launch_stamped(k_score_table<true>, dim3(kGeneralGradBlocks), dim3(kScoreTableThreads), st, e0, e1, a);
    else
      launch_stamped(k_score_table<false>, dim3(kGeneralGradBlocks), dim3(kScoreTableThreads), st, e0, e1, a);
    return hipGetLastError();
  }
  if (csr) return launch_gl<16, true>(a, mode, nblk, st, e0, e1);
  return launch_gl<64, false>(a, mode, nblk, st, e0, e1);
}

hipError_t launch_prepare_general(float *p, size_t count, const float *w, const float *phi,
                                  float2 *wp, int32_t head, int32_t d, hipStream_t st) {
  if ((reinterpret_cast<uintptr_t>(p) & 15) != 0 || (reinterpret_cast<uintptr_t>(wp) & 7) != 0)
    return hipErrorInvalidValue;
  const size_t work = count / 4 > (size_t)d ? count / 4 : (size_t)d;
  size_t blocks = (work + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(k_prepare_general, dim3((unsigned)blocks), dim3(256), 0, st, p, count, w, phi,
                     wp, head, d);
  return hipGetLastError();
}

hipError_t launch_zero_f32(float *p, size_t count, hipStream_t st) {
  if (count == 0) return hipSuccess;
  if ((reinterpret_cast<uintptr_t>(p) & 15) != 0) return hipErrorInvalidValue;
  size_t blocks = (count / 4 + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(k_zero_f32, dim3((unsigned)blocks), dim3(256), 0, st, p, count);
  return hipGetLastError();
}

bool general_keeps_ready(int32_t d, int nvec, bool csr) {
  return general_bin_plan(d, general_head_columns(d, nvec, csr), nvec, 1).nb > 0;
}

int32_t general_head_columns(int32_t d, int nvec, bool csr) {
  const int direct = nvec == 2 ? (csr ? kDirectTwoVec : kDirectTwoVecDense) : kDirectOneVec;
  return d < direct ? d : direct;
}

hipError_t launch_general_apply(const ApplyArgs &a, hipStream_t st) {
  const int nh = (a.head + kHeadCols - 1) / kHeadCols;
  int nrest = (a.d - a.head + 1023) / 1024;
  if (nrest > 1024) nrest = 1024;
  if (nrest < 0) nrest = 0;
  if (a.plan.nb > 0) nrest = a.plan.nb;
  if (nh + nrest < 1) nrest = 1;
  hipLaunchKernelGGL(k_apply_general, dim3(nh + nrest + (a.flags ? compact_tiles(a.P) : 0)), dim3(kApplyThreads),
                     0, st, a, nh, nrest);
  return hipGetLastError();
}

}  // namespace aa
