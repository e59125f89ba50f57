// Dense row passes for gfx950.
//
// One wave64 (or an aligned group of LPR lanes for short rows) owns a feature
// row: each lane loads VPL 128-bit pieces, so a wave-wide load instruction
// covers 1 KiB of contiguous row.  A wave owns a contiguous chunk of the pool,
// so row ids, labels and the Philox draws are produced 64 at a time, one per
// lane, and broadcast per row.  All loads of up to RIF rows are issued before
// the first is consumed (at the dense configuration a wave's whole share of the
// pool is in flight at once); phi and w are staged in LDS once per block; dot
// products are folded with DPP row operations and lane reads (no LDS traffic);
// the gradient sums of the kept rows accumulate per lane in registers and are
// combined per block in LDS in a fixed order.
#include "aa_batching.hpp"
#include "aa_compact.hpp"
#include "aa_dense.hpp"

#ifndef AA_NW_D1024
#define AA_NW_D1024 16   // waves per block of the gradient passes at 512 < d <= 1024
#endif
#ifndef AA_RIF_D1024
#define AA_RIF_D1024 1   // rows in flight per wave there
#endif
#ifndef AA_STEP_NW_D1024
#define AA_STEP_NW_D1024 8   // whole-step pass at d = 1024: waves per block (one block per CU)
#endif
#ifndef AA_STEP_RIF_D1024
#define AA_STEP_RIF_D1024 2  // and rows requested at once per wave
#endif
#ifndef AA_STEP_ROLL
#define AA_STEP_ROLL 0       // 1: a consumed row's slot is refilled at once instead of batch-wise
#endif

// Feature rows are read once per step: non-temporal loads keep them from displacing the
// model vectors and block partials in L2.
#ifndef AA_ROW_LOAD
#define AA_ROW_LOAD(p) __builtin_nontemporal_load(p)
#endif

namespace aa {

typedef float f4 __attribute__((ext_vector_type(4)));

namespace {

__device__ __forceinline__ float dot4(const f4 a, const f4 b, float acc) {
  acc = __fmaf_rn(a.x, b.x, acc);
  acc = __fmaf_rn(a.y, b.y, acc);
  acc = __fmaf_rn(a.z, b.z, acc);
  acc = __fmaf_rn(a.w, b.w, acc);
  return acc;
}

__device__ __forceinline__ f4 axpy4(const float s, const f4 x, f4 acc) {
  acc.x = __fmaf_rn(s, x.x, acc.x);
  acc.y = __fmaf_rn(s, x.y, acc.y);
  acc.z = __fmaf_rn(s, x.z, acc.z);
  acc.w = __fmaf_rn(s, x.w, acc.w);
  return acc;
}

__device__ __forceinline__ int wave_sum_int(int v) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

// v + (v moved by a DPP control): one VALU instruction, no LDS.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
  const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true);
  return v + __int_as_float(moved);
}

__device__ __forceinline__ float lane_read(float v, int lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

// Sum over aligned groups of LPR lanes (16, 32 or 64); every lane of a group
// gets the same bits.  Inside a 16-lane row: quad swaps, half mirror, mirror.
template <int LPR>
__device__ __forceinline__ float row_group_sum(float v, int lane) {
  v = dpp_add<0xB1>(v);   // quad_perm [1,0,3,2]
  v = dpp_add<0x4E>(v);   // quad_perm [2,3,0,1]
  v = dpp_add<0x141>(v);  // row_half_mirror
  v = dpp_add<0x140>(v);  // row_mirror
  if (LPR == 16) return v;
  const float s0 = lane_read(v, 0), s1 = lane_read(v, 16), s2 = lane_read(v, 32),
              s3 = lane_read(v, 48);
  if (LPR == 32) return lane < 32 ? s0 + s1 : s2 + s3;
  return (s0 + s1) + (s2 + s3);
}

// Phase time stamps of measurement builds (compiled out otherwise).
#ifdef AA_PHASE_TRACE
#define AA_STAMP(k) (t_stamp[k] = (unsigned long long)wall_clock64())
#else
#define AA_STAMP(k) ((void)0)
#endif

// Marks a loaded value as used at this point of the program: the wait for its load is placed
// here and cannot sink below later memory requests.
__device__ __forceinline__ void arrived(int &v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ void arrived(float &v) { asm volatile("" : "+v"(v)); }

// Per-lane sums of one wave into its own LDS slot (row groups folded first).
// Slot layout: red[(wave * NVEC + vec) * ROW4 + column].
template <int LPR, int VPL>
__device__ __forceinline__ void wave_slot_store(f4 (&acc)[VPL], f4 *slot, int lane) {
  if (LPR < kWave) {
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
      acc[v].x = fold_groups<LPR>(acc[v].x);
      acc[v].y = fold_groups<LPR>(acc[v].y);
      acc[v].z = fold_groups<LPR>(acc[v].z);
      acc[v].w = fold_groups<LPR>(acc[v].w);
    }
  }
  if (lane < LPR) {
#pragma unroll
    for (int v = 0; v < VPL; ++v) slot[v * LPR + lane] = acc[v];
  }
}

template <int LPR, int VPL, int MODE, int NW, int RIF>
__global__ __launch_bounds__(NW * 64)
    __attribute__((amdgpu_waves_per_eu((MODE & 3) ? (VPL == 8 ? 2 : 4) : 1,
                                       (MODE & 3) ? (VPL == 8 ? 2 : 4) : 8))) void k_rows_pass(const PassArgs a) {
  constexpr bool POOL = (MODE & kPool) != 0;
  constexpr bool SVM = (MODE & kSvm) != 0;
  constexpr bool ASSIST = (MODE & kAssist) != 0;
  constexpr bool HARD = (MODE & kHard) != 0;  // keep by the row's own loss, no Assistant
  constexpr bool GRAD = SVM || ASSIST;
  constexpr bool NEED_PHI = (POOL && !HARD) || ASSIST;
  constexpr int G = kWave / LPR;  // rows per wave iteration
  constexpr int ROW4 = LPR * VPL;
  constexpr int NVEC = (SVM ? 1 : 0) + (ASSIST ? 1 : 0);
  constexpr int NT = NW * 64;
  constexpr int STG = (ROW4 + NT - 1) / NT;  // staged 128-bit pieces per thread and vector

  __shared__ int s_int[20];
  __shared__ float s_flt[20];
  __shared__ int s_carry[NW];
  __shared__ f4 s_w[SVM ? ROW4 : 1];
  __shared__ f4 s_phi[NEED_PHI ? ROW4 : 1];
  __shared__ f4 s_red[GRAD ? NW * NVEC * ROW4 : 1];  // one slot per wave and vector
  constexpr bool MEDIAN = ASSIST && !SVM && !POOL;   // may take its threshold from the batch itself
  __shared__ __attribute__((aligned(16))) float s_med[MEDIAN ? kRankSelectMax + 2 : 1];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int grp = lane / LPR, sub = lane % LPR;
  const f4 zero4 = {0.f, 0.f, 0.f, 0.f};

  int total = a.count_max;
  if (!POOL && a.m_dev) total = min(max(*a.m_dev, 0), a.count_max);

  // balanced contiguous chunk of rows for this wave
  const int nwaves = gridDim.x * NW, gwave = blockIdx.x * NW + wave;
  const int per = total / nwaves, rem = total % nwaves;
  const int lo = gwave * per + min(gwave, rem);
  const int hi = lo + per + (gwave < rem ? 1 : 0);

  // ---- start-up, ordered so that the row loads leave as early as possible:
  // row ids of the first 64 rows, model vectors into registers, first rows,
  // labels and draws, then the model vectors into LDS behind one barrier.
  int base = lo;
  int cnt = min(kWave, hi - base);  // rows of the current group of up to 64 (<= 0: none)
  int row_l = 0;
  if (lane < cnt) row_l = a.rows ? a.rows[base + lane] : base + lane;

  f4 st_w[STG], st_p[STG];
#pragma unroll
  for (int q = 0; q < STG; ++q) {
    const int c = q * NT + threadIdx.x;
    st_w[q] = (SVM && c < a.d4) ? reinterpret_cast<const f4 *>(a.w)[c] : zero4;
    st_p[q] = (NEED_PHI && c < a.d4) ? reinterpret_cast<const f4 *>(a.phi)[c] : zero4;
  }
  const float b = (NEED_PHI && a.bias) ? *a.bias : 0.f;
  float T = (ASSIST || HARD) ? *a.T : 0.f;
  const int med_init_old = (MEDIAN && a.med_init) ? *a.med_init : 0;

  f4 x[RIF][VPL];
  // Every load of the next RIF rows, before any is used.  When the row fills the lane layout
  // (d4 == ROW4) the loads are unconditional: a slot past the end of the group re-reads the
  // group's last row (a cache hit) and is never consumed, so the loads carry no branches.
  const bool full = a.d4 == ROW4;
  // (The two cases are two loops, not one loop with a case inside: the compiler would share
  // code between them, and with it the waits that the conditional loads need.)
  auto issue_rows = [&](int it0) {
    if (full) {
#pragma unroll
      for (int r = 0; r < RIF; ++r) {
        const int li = (it0 + r) * G + grp;
        const int row = __shfl(row_l, min(li, cnt - 1), kWave);
        const f4 *xr = reinterpret_cast<const f4 *>(a.x + (int64_t)row * a.ld);
#pragma unroll
        for (int v = 0; v < VPL; ++v) x[r][v] = AA_ROW_LOAD(xr + v * LPR + sub);
      }
    } else {
#pragma unroll
      for (int r = 0; r < RIF; ++r) {
        const int li = (it0 + r) * G + grp;
        const int row = __shfl(row_l, li & 63, kWave);
        const f4 *xr = reinterpret_cast<const f4 *>(a.x + (int64_t)row * a.ld);
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
          const int c = v * LPR + sub;
          x[r][v] = (li < cnt && c < a.d4) ? AA_ROW_LOAD(xr + c) : zero4;
        }
      }
    }
  };
  float y_l = 0.f, u_l = 2.f, lin_l = 0.f;
  auto lane_inputs = [&]() {  // one row per lane: label, draw, incoming loss
    y_l = 0.f;
    u_l = 2.f;
    lin_l = 0.f;
    if (lane < cnt) {
      if (SVM) y_l = a.y[row_l];
      if (POOL && a.do_keep) u_l = keep_uniform(a.key, (uint32_t)(base + lane));
      if (ASSIST && !SVM) lin_l = a.loss_in[base + lane];
    }
  };
  if (cnt > 0) {
    issue_rows(0);
    lane_inputs();
  }
  // Carried compaction of the previous pool: its loads leave behind the first rows, the
  // count of the flags before this block's 64 positions rides on the start-up barrier,
  // and the last wave places the survivors while the rows are still arriving.
  const bool carry = POOL && GRAD && a.prev.flags != nullptr && (int)blockIdx.x * kWave < a.prev.P;
  int carry_cnt = 0, carry_id = 0;
  uint8_t carry_flag = 0;
  float carry_loss = 0.f;
  if (POOL && GRAD && carry) {
    const int j0 = blockIdx.x * kWave;
    const uint4 *p16 = reinterpret_cast<const uint4 *>(a.prev.flags);
    for (int q = threadIdx.x; q < (j0 >> 4); q += NT) {
      const uint4 v = p16[q];
      carry_cnt += __popc(v.x) + __popc(v.y) + __popc(v.z) + __popc(v.w);  // bytes are 0 or 1
    }
    if (wave == NW - 1 && j0 + lane < a.prev.P) {
      carry_flag = a.prev.flags[j0 + lane];
      carry_id = a.prev.idx ? a.prev.idx[j0 + lane] : j0 + lane;
      if (a.prev.loss) carry_loss = a.prev.loss_pool[j0 + lane];
    }
  }
#pragma unroll
  for (int q = 0; q < STG; ++q) {
    const int c = q * NT + threadIdx.x;
    if (c < ROW4) {
      if (SVM) s_w[c] = st_w[q];
      if (NEED_PHI) s_phi[c] = st_p[q];
    }
  }
  if (POOL && GRAD && carry) {
    carry_cnt = wave_sum_int(carry_cnt);
    if (lane == 0) s_carry[wave] = carry_cnt;
  }
  __syncthreads();
  if (MEDIAN && a.med_init && total > 0) {  // (the same in every thread of the grid)
    float lo_mid, hi_mid;
    if (block_middle_values(a.loss_in, total, s_med, &lo_mid, &hi_mid))
      T = running_threshold(lo_mid, hi_mid, total, med_init_old, T, a.med_momentum);
    else
      T = __builtin_nanf("");  // a NaN loss has no rank: the threshold becomes NaN, visibly
    if (blockIdx.x == 0 && threadIdx.x == 0) *a.T_next = T;
  }
  if (POOL && GRAD && carry && wave == NW - 1) {
    int before = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) before += s_carry[i];
    const unsigned long long mask = __ballot(carry_flag != 0);
    if (carry_flag != 0) {
      const int pos = before + __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                                         __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
      if (a.prev.kept_pos) a.prev.kept_pos[pos] = blockIdx.x * kWave + lane;
      if (a.prev.kept_ids) a.prev.kept_ids[pos] = carry_id;
      if (a.prev.loss) a.prev.loss[pos] = carry_loss;
    }
    if (lane == 0 && a.prev.kept_count && (int)(blockIdx.x + 1) * kWave >= a.prev.P)
      *a.prev.kept_count = before + __popcll(mask);
  }

  f4 gw[VPL], gp[VPL];
#pragma unroll
  for (int v = 0; v < VPL; ++v) {
    gw[v] = zero4;
    gp[v] = zero4;
  }
  float gb = 0.f;
  int kept = 0;
  int it0 = 0;

  while (cnt > 0) {
    const int iters = (cnt + G - 1) / G;
#pragma unroll
    for (int r = 0; r < RIF; ++r) {
      const int it = it0 + r;
      if (it >= iters) break;
      const int li = it * G + grp;
      const bool live = li < cnt;
      const int j = base + li;
      float g = 0.f;
      bool keep = live;
      if (NEED_PHI) {
        float dp = 0.f;
#pragma unroll
        for (int v = 0; v < VPL; ++v) dp = dot4(x[r][v], s_phi[v * LPR + sub], dp);
        dp = row_group_sum<LPR>(dp, lane);
        const float s = dp + b;
        g = sigmoidf_(s);
        if (POOL) {
          const float u = __shfl(u_l, li & 63, kWave);
          if (a.do_keep) keep = live && keep_decision(u, g, a.gamma, a.one_minus_gamma);
          if (sub == 0 && live) {
            if (a.logit) a.logit[j] = s;
            if (a.prob) a.prob[j] = g;
            if (a.flags) a.flags[j] = keep ? 1 : 0;
          }
        }
      }
      if (GRAD) {
        const float yy = SVM ? __shfl(y_l, li & 63, kWave) : 0.f;
        const float lin = (ASSIST && !SVM) ? __shfl(lin_l, li & 63, kWave) : 0.f;
        bool any = true;
        if (LPR == kWave) any = __builtin_amdgcn_readfirstlane((int)keep) != 0;
        if (any) {
          float loss = lin;
          if (SVM) {
            float dw = 0.f;
#pragma unroll
            for (int v = 0; v < VPL; ++v) dw = dot4(x[r][v], s_w[v * LPR + sub], dw);
            dw = row_group_sum<LPR>(dw, lane);
            const float marg = yy * dw;
            loss = fmaxf(0.f, 1.f - marg);
            if (HARD) {  // shrinking by the objective value itself
              keep = live && loss > T;
              if (sub == 0 && live && a.flags) a.flags[j] = keep ? 1 : 0;
            }
            if (sub == 0 && (HARD ? live : keep) && a.loss_out) a.loss_out[j] = loss;
            const float cw = (keep && marg < 1.f) ? yy : 0.f;  // -d hinge / d margin, times y
#pragma unroll
            for (int v = 0; v < VPL; ++v) gw[v] = axpy4(cw, x[r][v], gw[v]);
          }
          if (ASSIST) {
            const float z = loss > T ? 1.f : 0.f;       // label: Boss loss above the threshold
            const float resid = keep ? g - z : 0.f;     // d cross-entropy / d logit
#pragma unroll
            for (int v = 0; v < VPL; ++v) gp[v] = axpy4(resid, x[r][v], gp[v]);
            if (sub == 0) gb += resid;
          }
          if (sub == 0 && keep) kept += 1;
        }
      }
    }
    // next rows: the same group of 64, or the next group
    it0 += RIF;
    if (it0 >= iters) {
      it0 = 0;
      base += kWave;
      cnt = min(kWave, hi - base);
      if (cnt > 0) {
        row_l = lane < cnt ? (a.rows ? a.rows[base + lane] : base + lane) : 0;
        issue_rows(0);
        lane_inputs();
      }
    } else {
      issue_rows(it0);
    }
  }

  if (GRAD) {
    // Block reduction behind a single barrier: every wave drops its sums into its own LDS
    // slot as soon as its rows are done, then one thread per 128-bit column adds the
    // slots in wave order and stores the block's partial vectors.
    f4 *slot = s_red + wave * NVEC * ROW4;
    if (SVM) wave_slot_store<LPR, VPL>(gw, slot, lane);
    if (ASSIST) wave_slot_store<LPR, VPL>(gp, slot + (SVM ? ROW4 : 0), lane);
    const int kw = wave_sum_int(kept);
    const float gbw = group_sum<kWave>(gb);
    if (lane == 0) {
      s_int[wave] = kw;
      s_flt[wave] = gbw;
    }
    __syncthreads();
    f4 *part = reinterpret_cast<f4 *>(a.partial) + (size_t)blockIdx.x * NVEC * ROW4;
    for (int c = threadIdx.x; c < NVEC * ROW4; c += NT) {
      f4 t = s_red[c];
#pragma unroll
      for (int q = 1; q < NW; ++q) t += s_red[q * NVEC * ROW4 + c];
      part[c] = t;
    }
    if (threadIdx.x == 0) {
      int ks = 0;
      float gs = 0.f;
      for (int i = 0; i < NW; ++i) {
        ks += s_int[i];
        gs += s_flt[i];
      }
      a.blk_cnt[blockIdx.x] = ks;
      a.blk_gb[blockIdx.x] = gs;
    }
  }
  if (GRAD && a.t_upd && blockIdx.x == 0 && threadIdx.x == 0) *a.t_snap = *a.t_upd;
}

// The whole-step pool pass (score, keep, both gradient sums; or the hard-threshold variant)
// for rows that fill the 64-lane layout exactly (d == 256 VPL).  Same arithmetic and the same
// summation order as k_rows_pass; the schedule differs.  A wave requests RIF rows at once and
// nothing sits between those requests and their use that the memory pipeline would have to
// finish first: every small load that does not depend on the row ids (model vectors,
// scalars, the flags of the carried compaction) is requested before the ids are waited for,
// the labels right behind the ids, the rows last; the per-row outputs (logit, probability,
// keep flag, loss) are collected one per lane and stored once per group of 64 rows, so no
// store is pending while rows arrive.  Loads return in request order, so row r of a batch
// is consumed as soon as it is there while rows r+1.. are still on their way.
template <int VPL, bool HARD, int NW, int RIF>
__global__ __launch_bounds__(NW * 64)
    __attribute__((amdgpu_waves_per_eu(NW / 4, NW / 4))) void k_step_pass(const PassArgs a) {
  constexpr bool ASSIST = !HARD;
  constexpr int ROW4 = kWave * VPL;
  constexpr int NVEC = ASSIST ? 2 : 1;
  constexpr int NT = NW * 64;
  constexpr int STG = (ROW4 + NT - 1) / NT;

  __shared__ int s_int[NW];
  __shared__ float s_flt[NW];
  __shared__ int s_carry[NW];
  __shared__ f4 s_w[ROW4];
  __shared__ f4 s_phi[ASSIST ? ROW4 : 1];
  __shared__ f4 s_red[NW * NVEC * ROW4];  // one slot per wave and vector

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const f4 zero4 = {0.f, 0.f, 0.f, 0.f};
#ifdef AA_PHASE_TRACE
  unsigned long long t_stamp[kTraceStamps] = {};
#endif
  AA_STAMP(0);  // entry

  // balanced contiguous chunk of pool positions for this wave
  const int total = a.count_max;
  const int nwaves = gridDim.x * NW, gwave = blockIdx.x * NW + wave;
  const int per = total / nwaves, rem = total % nwaves;
  const int lo = gwave * per + min(gwave, rem);
  const int hi = lo + per + (gwave < rem ? 1 : 0);

  int base = lo;
  int cnt = min(kWave, hi - base);  // rows of the current group of up to 64 (<= 0: none)

  // ---- Requests that depend on nothing, all unconditional: a load under a condition would
  // make every later wait for an older load a wait for everything (the pending counts of the
  // two paths are merged pessimistically), so absent inputs read a stand-in address (the
  // start of w, which always holds at least 1 KiB) and indices are clamped; what was read for
  // nothing is dropped by a select.
  const int32_t *stand_in = reinterpret_cast<const int32_t *>(a.w);
  const int32_t *rows_p = a.rows ? a.rows : stand_in;
  const int in_group = min(lane, max(cnt, 1) - 1);
  int row_l = rows_p[a.rows && cnt > 0 ? base + in_group : 0];
  if (!a.rows) row_l = base + in_group;

  const bool carry = a.prev.flags != nullptr && (int)blockIdx.x * kWave < a.prev.P;
  const int cj0 = blockIdx.x * kWave;     // this block places positions [cj0, cj0 + 64)
  const int n16 = carry ? (cj0 >> 4) : 0;  // 16-byte pieces of flags before them
  const uint4 *p16 = n16 > 0 ? reinterpret_cast<const uint4 *>(a.prev.flags)
                             : reinterpret_cast<const uint4 *>(a.w);
  uint4 carry_v = p16[min((int)threadIdx.x, max(n16, 1) - 1)];
  const int cpos = carry ? min(cj0 + lane, a.prev.P - 1) : 0;
  uint8_t carry_flag = (carry ? a.prev.flags : reinterpret_cast<const uint8_t *>(a.w))[cpos];
  int carry_id = ((carry && a.prev.idx) ? a.prev.idx : stand_in)[cpos];
  float carry_loss = ((carry && a.prev.loss) ? a.prev.loss_pool : a.w)[cpos];
  f4 st_w[STG], st_p[STG];
#pragma unroll
  for (int q = 0; q < STG; ++q) {
    const int c = min(q * NT + (int)threadIdx.x, ROW4 - 1);
    st_w[q] = reinterpret_cast<const f4 *>(a.w)[c];
    st_p[q] = reinterpret_cast<const f4 *>(ASSIST ? a.phi : a.w)[c];
  }
  float b = (ASSIST && a.bias ? a.bias : a.w)[0];
  if (!(ASSIST && a.bias)) b = 0.f;
  float T = *a.T;

  // Everything above is there after one memory round trip.  It is all consumed here, before
  // the rows are requested: the model vectors go to LDS, the carried flags are counted, and
  // values only needed later are pinned (arrived()) so that no wait for them can end up
  // behind the row requests, where it would be a wait for the rows.
  arrived(row_l);
  arrived(carry_id);
  arrived(carry_loss);
  arrived(b);
  arrived(T);
  AA_STAMP(1);  // ids, model, scalars, carried flags are there
  int carry_cnt = 0;
  if ((int)threadIdx.x < n16)
    carry_cnt = __popc(carry_v.x) + __popc(carry_v.y) + __popc(carry_v.z) + __popc(carry_v.w);
  if (!carry || cj0 + lane >= a.prev.P || wave != NW - 1) carry_flag = 0;
  if (carry && !a.prev.idx) carry_id = cj0 + lane;
  const unsigned long long carry_mask = __ballot(carry_flag != 0);
  for (int q = threadIdx.x + NT; q < n16; q += NT) {  // previous pools above 16 NT positions
    const uint4 v = p16[q];
    carry_cnt += __popc(v.x) + __popc(v.y) + __popc(v.z) + __popc(v.w);
  }
#pragma unroll
  for (int q = 0; q < STG; ++q) {
    const int c = q * NT + threadIdx.x;
    if (c < ROW4) {
      s_w[c] = st_w[q];
      if (ASSIST) s_phi[c] = st_p[q];
    }
  }
  if (carry) {
    carry_cnt = wave_sum_int(carry_cnt);
    if (lane == 0) s_carry[wave] = carry_cnt;
  }

  // ---- requests that need the ids: the labels, then the rows; nothing is requested after
  // them until they are consumed
  f4 x[RIF][VPL];
  auto issue_rows = [&](int it0) {
#pragma unroll
    for (int r = 0; r < RIF; ++r) {
      // a slot past the end of the group re-reads the group's last row and is never consumed
      const int li = min(it0 + r, cnt - 1);
      const int row = __builtin_amdgcn_readlane(row_l, li);
      const f4 *xr = reinterpret_cast<const f4 *>(a.x + (int64_t)row * a.ld) + lane;
#pragma unroll
      for (int v = 0; v < VPL; ++v) x[r][v] = AA_ROW_LOAD(xr + v * kWave);
    }
  };
  // The barrier that publishes the model vectors comes before the row requests: the memory
  // pipeline accepts a compute unit's requests only as fast as earlier ones complete, so a
  // barrier behind them would hold every wave until the last wave's requests were accepted.
  __syncthreads();
  AA_STAMP(2);  // past the start-up barrier
  float y_l = 0.f, u_l = 2.f;
  if (cnt > 0) {
    y_l = a.y[row_l];
    issue_rows(0);
    if (!HARD) u_l = keep_uniform(a.key, (uint32_t)(base + in_group));
  }
  AA_STAMP(3);  // rows requested, draws made
  if (carry && wave == NW - 1) {
    int before = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) before += s_carry[i];
    const unsigned long long mask = carry_mask;
    if (carry_flag != 0) {
      const int pos = before + __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                                         __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
      if (a.prev.kept_pos) a.prev.kept_pos[pos] = cj0 + lane;
      if (a.prev.kept_ids) a.prev.kept_ids[pos] = carry_id;
      if (a.prev.loss) a.prev.loss[pos] = carry_loss;
    }
    if (lane == 0 && a.prev.kept_count && cj0 + kWave >= a.prev.P)
      *a.prev.kept_count = before + __popcll(mask);
  }

  f4 gw[VPL], gp[VPL];
#pragma unroll
  for (int v = 0; v < VPL; ++v) {
    gw[v] = zero4;
    gp[v] = zero4;
  }
  float gb = 0.f;
  int kept = 0;

  while (cnt > 0) {
    // outputs of the group, one row per lane, stored after its last batch
    float o_logit = 0.f, o_prob = 0.f, o_loss = 0.f;
    int o_keep = 0;
    for (int it0 = 0; it0 < cnt; it0 += RIF) {
#pragma unroll
      for (int r = 0; r < RIF; ++r) {
        const int li = it0 + r;        // wave-uniform
        const bool live = li < cnt;
        const int src = li & 63;
        float g = 0.f, s = 0.f, loss = 0.f;
        bool keep = live;
        if (ASSIST) {
          float dp = 0.f;
#pragma unroll
          for (int v = 0; v < VPL; ++v) dp = dot4(x[r][v], s_phi[v * kWave + lane], dp);
          dp = row_group_sum<kWave>(dp, lane);
          s = dp + b;
          g = sigmoidf_(s);
          const float u = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(u_l), src));
          keep = live && keep_decision(u, g, a.gamma, a.one_minus_gamma);
        }
        const float yy = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(y_l), src));
        if (HARD || keep) {
          float dw = 0.f;
#pragma unroll
          for (int v = 0; v < VPL; ++v) dw = dot4(x[r][v], s_w[v * kWave + lane], dw);
          dw = row_group_sum<kWave>(dw, lane);
          const float marg = yy * dw;
          loss = fmaxf(0.f, 1.f - marg);
          if (HARD) keep = live && loss > T;  // shrinking by the objective value itself
          const float cw = (keep && marg < 1.f) ? yy : 0.f;  // -d hinge / d margin, times y
#pragma unroll
          for (int v = 0; v < VPL; ++v) gw[v] = axpy4(cw, x[r][v], gw[v]);
          if (ASSIST) {
            const float z = loss > T ? 1.f : 0.f;    // label: Boss loss above the threshold
            const float resid = g - z;               // d cross-entropy / d logit (kept rows only)
#pragma unroll
            for (int v = 0; v < VPL; ++v) gp[v] = axpy4(resid, x[r][v], gp[v]);
            gb += resid;
          }
          if (keep) kept += 1;
        }
        if (lane == li) {
          o_logit = s;
          o_prob = g;
          o_loss = loss;
          o_keep = keep ? 1 : 0;
        }
#ifdef AA_PHASE_TRACE
        if (t_stamp[4] == 0) AA_STAMP(4);  // first row arrived and used
#endif
        if (AA_STEP_ROLL && li + RIF < cnt) {  // the freed slot takes the row RIF further on
          const int row = __builtin_amdgcn_readlane(row_l, (li + RIF) & 63);
          const f4 *xr = reinterpret_cast<const f4 *>(a.x + (int64_t)row * a.ld) + lane;
#pragma unroll
          for (int v = 0; v < VPL; ++v) x[r][v] = AA_ROW_LOAD(xr + v * kWave);
        }
      }
      if (!AA_STEP_ROLL && it0 + RIF < cnt) issue_rows(it0 + RIF);
    }
    if (lane < cnt) {
      const int j = base + lane;
      if (ASSIST && a.logit) a.logit[j] = o_logit;
      if (ASSIST && a.prob) a.prob[j] = o_prob;
      if (a.flags) a.flags[j] = (uint8_t)o_keep;
      if ((HARD || o_keep) && a.loss_out) a.loss_out[j] = o_loss;
    }
    base += kWave;
    cnt = min(kWave, hi - base);
    if (cnt > 0) {
      const int in_next = min(lane, cnt - 1);
      row_l = a.rows ? a.rows[base + in_next] : base + in_next;
      y_l = a.y[row_l];
      issue_rows(0);
      if (!HARD) u_l = keep_uniform(a.key, (uint32_t)(base + in_next));
    }
  }

  AA_STAMP(5);  // all rows of this wave consumed
  // Block reduction behind a single barrier: every wave drops its sums into its own LDS
  // slot, then one thread per 128-bit column adds the slots in wave order and stores the
  // block's partial vectors.
  f4 *slot = s_red + wave * NVEC * ROW4;
#pragma unroll
  for (int v = 0; v < VPL; ++v) slot[v * kWave + lane] = gw[v];
  if (ASSIST) {
#pragma unroll
    for (int v = 0; v < VPL; ++v) slot[ROW4 + v * kWave + lane] = gp[v];
  }
  if (lane == 0) {
    s_int[wave] = kept;
    s_flt[wave] = gb;
  }
  __syncthreads();
  AA_STAMP(6);  // past the reduction barrier
  f4 *part = reinterpret_cast<f4 *>(a.partial) + (size_t)blockIdx.x * NVEC * ROW4;
  for (int c = threadIdx.x; c < NVEC * ROW4; c += NT) {
    f4 t = s_red[c];
#pragma unroll
    for (int q = 1; q < NW; ++q) t += s_red[q * NVEC * ROW4 + c];
    part[c] = t;
  }
  if (threadIdx.x == 0) {
    int ks = 0;
    float gs = 0.f;
    for (int i = 0; i < NW; ++i) {
      ks += s_int[i];
      gs += s_flt[i];
    }
    a.blk_cnt[blockIdx.x] = ks;
    a.blk_gb[blockIdx.x] = gs;
  }
  if (a.t_upd && blockIdx.x == 0 && threadIdx.x == 0) *a.t_snap = *a.t_upd;
#ifdef AA_PHASE_TRACE
  AA_STAMP(7);  // partials stored
  if (a.trace && lane == 0) {
    unsigned long long *tr = a.trace + ((size_t)blockIdx.x * NW + wave) * kTraceStamps;
    for (int k = 0; k < kTraceStamps; ++k) tr[k] = t_stamp[k];
  }
#endif
}

#ifndef AA_FIN_COLS4
#define AA_FIN_COLS4 8
#endif
constexpr int kFinCols4 = AA_FIN_COLS4;        // 128-bit columns reduced by one finalize block
constexpr int kFinGroups = 256 / kFinCols4;    // partial groups per column (256 threads)

// Sum the block partials in a fixed order and apply the SGD updates; extra blocks compact
// the keep flags of a pool pass, one tile each.  A reduce block owns kFinCols4 128-bit
// columns of one gradient vector: thread (group g, column c) adds the partials of blocks
// g, g + kFinGroups, ... in that order, the groups of a wave are folded with a fixed
// butterfly, the four wave sums are added in wave order.  One memory round trip (every
// load is requested before any is used) and one barrier.
__global__ __launch_bounds__(256) void k_finalize(const FinalizeArgs a) {
  __shared__ f4 s_acc[4][kFinCols4];
  __shared__ int s_int[40];
  __shared__ float s_flt[8];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row4 = a.d_pad / 4;
  const int per_vec = row4 / kFinCols4;  // reduce blocks per gradient vector
  const int nred = per_vec * a.nvec;

  if ((int)blockIdx.x >= nred) {
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
    tile_compact(c, (int)blockIdx.x - nred, s_int);
    return;
  }

  // vector 0 is the Boss gradient when w is updated, the Assistant's otherwise
  const int vec = blockIdx.x / per_vec;
  const bool boss = a.w != nullptr && vec == 0;
  float *model = boss ? a.w : a.phi;
  const bool bias_block = !boss && (int)blockIdx.x % per_vec == 0 && a.phi && a.bias;
  const int c4 = tid % kFinCols4, pg = tid / kFinCols4;
  const int col4 = ((int)blockIdx.x % per_vec) * kFinCols4 + c4;
  const int k0 = col4 * 4;

  // Every first load is requested before any is used and none sits under a condition (absent
  // inputs read a stand-in address, indices are clamped, what was read for nothing is
  // dropped): the block pays one memory round trip for counts, scalars, model slice and
  // its first eight partials per thread.
  const int nb = a.nblk;
  const int32_t *ints = a.blk_cnt;                       // always present: the stand-in address
  const int ci = min(tid, nb - 1);
  int cnt_part = a.blk_cnt[ci];
  float gb_part = a.blk_gb[ci];
  const int m_given = *(a.m_dev ? a.m_dev : ints);
  int t_old = *(a.t_upd ? a.t_snap : ints);
  float b_new = *(bias_block ? a.bias : a.blk_gb);       // the bias before this update
  const float t_next = *(a.T_next ? a.T_next : a.blk_gb);
  float old[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) old[i] = model[min(k0 + i, a.d - 1)];
  const f4 zero = {0.f, 0.f, 0.f, 0.f};
  f4 acc = zero;
  const f4 *p = reinterpret_cast<const f4 *>(a.partial) + (size_t)vec * row4 + col4;
  const size_t stride = (size_t)a.nvec * row4;
  for (int base = pg; base < nb; base += 8 * kFinGroups) {
    f4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = p[(size_t)min(base + j * kFinGroups, nb - 1) * stride];
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (base + j * kFinGroups < nb) acc += v[j];       // block order within the group
  }
  if (a.m_dev || tid >= nb) cnt_part = 0;
  if (!bias_block || tid >= nb) gb_part = 0.f;
  if (!a.t_upd) t_old = 0;
  if (pg != 0) old[0] = old[1] = old[2] = old[3] = 0.f;
  for (int i = tid + blockDim.x; i < nb; i += blockDim.x) {  // more than 256 partials
    if (!a.m_dev) cnt_part += a.blk_cnt[i];
    if (bias_block) gb_part += a.blk_gb[i];
  }

  // fold the groups of this wave (lanes that share a column), then the four waves
#pragma unroll
  for (int off = kFinCols4; off < kWave; off <<= 1) {
    acc.x += __shfl_xor(acc.x, off, kWave);
    acc.y += __shfl_xor(acc.y, off, kWave);
    acc.z += __shfl_xor(acc.z, off, kWave);
    acc.w += __shfl_xor(acc.w, off, kWave);
  }
  if (lane < kFinCols4) s_acc[wave][lane] = acc;
  cnt_part = wave_sum_int(cnt_part);
  gb_part = group_sum<kWave>(gb_part);
  if (lane == 0) {
    s_int[wave] = cnt_part;
    s_flt[wave] = gb_part;
  }
  __syncthreads();
  const int m = a.m_dev ? min(max(m_given, 0), a.m_max) : (s_int[0] + s_int[1]) + (s_int[2] + s_int[3]);

  // step size: constant, or lr / sqrt(number of updates made so far)
  const int t_new = t_old + (m > 0 ? 1 : 0);
  float lr = a.lr;
  if (a.t_upd && m > 0) lr = a.lr / sqrtf((float)t_new);

  float now[4] = {old[0], old[1], old[2], old[3]};
  const bool bias_thread = bias_block && tid == 0;
  if (m > 0) {
    const float inv_m = 1.f / (float)m;
    if (pg == 0) {
      const f4 g = (s_acc[0][c4] + s_acc[1][c4]) + (s_acc[2][c4] + s_acc[3][c4]);
      const float gv[4] = {g.x, g.y, g.z, g.w};
      if (boss) {
        const float shrink = 1.f - lr * a.lambda;
        const float scale = lr * inv_m;
#pragma unroll
        for (int i = 0; i < 4; ++i) now[i] = __fmaf_rn(scale, gv[i], shrink * old[i]);
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          now[i] = old[i] - a.lr_a * __fmaf_rn(a.l2_a, old[i], gv[i] * inv_m);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (k0 + i < a.d) model[k0 + i] = now[i];
    }
    if (bias_thread) {
      // bias gradient: per-wave sums of the block partials, added in wave order
      const float gb = (s_flt[0] + s_flt[1]) + (s_flt[2] + s_flt[3]);
      b_new = b_new - a.lr_a * (gb * inv_m);
      *a.bias = b_new;
    }
  }
  if (a.phi_copy && !boss && pg == 0) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (k0 + i < a.d) a.phi_copy[k0 + i] = now[i];
  }
  if (a.bias_copy && bias_thread) *a.bias_copy = b_new;
  if (blockIdx.x == 0 && tid == 0 && a.kept_hist) *a.kept_hist = m;
  if (blockIdx.x == 0 && tid == 0 && a.T_next && m > 0) {
    *a.T_out = t_next;
    *a.T_init = 1;
  }
  if (blockIdx.x == 0 && tid == 0 && a.t_upd) *a.t_upd = t_new;
}

int g_num_cu = 0;

int num_cu() {
  if (g_num_cu == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
      g_num_cu = prop.multiProcessorCount;
    if (g_num_cu <= 0) g_num_cu = 256;
  }
  return g_num_cu;
}

struct Shape {
  int lpr, vpl;
};

Shape pick_shape(int32_t d) {
  const int d4 = (d + 3) / 4;
  if (d4 <= 16) return {16, 1};
  if (d4 <= 32) return {32, 1};
  if (d4 <= 64) return {64, 1};
  if (d4 <= 128) return {64, 2};
  if (d4 <= 256) return {64, 4};
  return {64, 8};
}

// The whole-step pool passes take k_step_pass when the row fills the 64-lane layout exactly.
bool step_pass_ok(const Shape &s, int32_t d, int mode) {
  const bool whole = mode == (kPool | kSvm | kAssist) || mode == (kPool | kSvm | kHard);
  return whole && s.lpr == kWave && d == 4 * kWave * s.vpl;
}

// Waves per block: passes with gradient sums use one fat block per CU (few block
// partials); the general 1024-wide pass runs 16 waves of 128 registers, everything else 8.
int waves_per_block(const Shape &s, int32_t d, int mode) {
  const bool grad = (mode & (kSvm | kAssist)) != 0;
  if (!grad) return 4;
  if (step_pass_ok(s, d, mode)) return s.vpl == 4 ? AA_STEP_NW_D1024 : 8;
  return s.vpl == 4 ? AA_NW_D1024 : 8;
}

template <int LPR, int VPL, int NW, int RIF>
hipError_t launch_grad(const PassArgs &a, int mode, int nblk, hipStream_t st, hipEvent_t e0,
                       hipEvent_t e1) {
  const dim3 grid(nblk), block(NW * 64);
  switch (mode) {
    case kSvm:
      launch_stamped((k_rows_pass<LPR, VPL, kSvm, NW, RIF>), grid, block, st, e0, e1, a);
      break;
    case kAssist:
      launch_stamped((k_rows_pass<LPR, VPL, kAssist, NW, RIF>), grid, block, st, e0, e1, a);
      break;
    case kSvm | kAssist:
      launch_stamped((k_rows_pass<LPR, VPL, kSvm | kAssist, NW, RIF>), grid, block, st, e0, e1, a);
      break;
    case kPool | kSvm | kAssist:
      launch_stamped((k_rows_pass<LPR, VPL, kPool | kSvm | kAssist, NW, RIF>), grid, block, st, e0, e1, a);
      break;
    case kPool | kSvm | kHard:
      launch_stamped((k_rows_pass<LPR, VPL, kPool | kSvm | kHard, NW, RIF>), grid, block, st, e0, e1, a);
      break;
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <int VPL, int NW, int RIF>
hipError_t launch_step(const PassArgs &a, bool hard, int nblk, hipStream_t st, hipEvent_t e0,
                       hipEvent_t e1) {
  const dim3 grid(nblk), block(NW * 64);
  if (hard)
    launch_stamped((k_step_pass<VPL, true, NW, RIF>), grid, block, st, e0, e1, a);
  else
    launch_stamped((k_step_pass<VPL, false, NW, RIF>), grid, block, st, e0, e1, a);
  return hipGetLastError();
}

template <int LPR, int VPL, int RIF>
hipError_t launch_pool(const PassArgs &a, int nblk, hipStream_t st, hipEvent_t e0, hipEvent_t e1) {
  launch_stamped((k_rows_pass<LPR, VPL, kPool, 4, RIF>), dim3(nblk), dim3(256), st, e0, e1, a);
  return hipGetLastError();
}

}  // namespace

bool dense_fast_ok(const aa_features *F) {
  return F->layout == AA_DENSE && F->d % 4 == 0 && F->d <= kFastDenseMaxD && F->ld % 4 == 0 &&
         (reinterpret_cast<uintptr_t>(F->x) & 15) == 0;
}

int32_t dense_d_pad(int32_t d) {
  const Shape s = pick_shape(d);
  return s.lpr * s.vpl * 4;
}

int32_t dense_pass_blocks(int32_t d, int32_t count, int mode) {
  const Shape s = pick_shape(d);
  const int nw = waves_per_block(s, d, mode);
  const int rows_per_block = nw * (kWave / s.lpr);
  const bool grad = (mode & (kSvm | kAssist)) != 0;
  int64_t want = ((int64_t)count + rows_per_block - 1) / rows_per_block;
  // 16 waves per CU: one block of 16 waves, two of 8 or four of 4; the wide whole-step passes
  // hold several rows per wave in registers and fit one block per CU
  const bool one_per_cu = s.vpl == 8 || (step_pass_ok(s, d, mode) && s.vpl >= 4);
  const int64_t cap = grad ? (int64_t)num_cu() * (one_per_cu ? 1 : 16 / nw) : (int64_t)num_cu() * 8;
  if (want > cap) want = cap;
  if (want > kMaxBlocks) want = kMaxBlocks;
  if (want < 1) want = 1;
  return (int32_t)want;
}

hipError_t launch_dense_pass(const PassArgs &a, int mode, int32_t d, int32_t nblk,
                             hipStream_t st, hipEvent_t e0, hipEvent_t e1) {
  const Shape s = pick_shape(d);
  if (mode == kPool) {
    if (s.lpr == 16) return launch_pool<16, 1, 4>(a, nblk, st, e0, e1);
    if (s.lpr == 32) return launch_pool<32, 1, 4>(a, nblk, st, e0, e1);
    switch (s.vpl) {
      case 1: return launch_pool<64, 1, 4>(a, nblk, st, e0, e1);
      case 2: return launch_pool<64, 2, 4>(a, nblk, st, e0, e1);
      case 4: return launch_pool<64, 4, 2>(a, nblk, st, e0, e1);
      default: return launch_pool<64, 8, 2>(a, nblk, st, e0, e1);
    }
  }
  if (step_pass_ok(s, d, mode)) {
    const bool hard = (mode & kHard) != 0;
    switch (s.vpl) {
      case 1: return launch_step<1, 8, 8>(a, hard, nblk, st, e0, e1);
      case 2: return launch_step<2, 8, 8>(a, hard, nblk, st, e0, e1);
      case 4: return launch_step<4, AA_STEP_NW_D1024, AA_STEP_RIF_D1024>(a, hard, nblk, st, e0, e1);
      // (two rows of 8 KB in flight per wave: with four the hard-threshold variant does not fit
      // its registers -- the compiler then parks every arriving row in scratch, one load at a
      // time, 67 us per step instead of 30 -- and the other is 4 % slower at the register limit)
      default: return launch_step<8, 8, 2>(a, hard, nblk, st, e0, e1);
    }
  }
  if (s.lpr == 16) return launch_grad<16, 1, 8, 8>(a, mode, nblk, st, e0, e1);
  if (s.lpr == 32) return launch_grad<32, 1, 8, 8>(a, mode, nblk, st, e0, e1);
  switch (s.vpl) {
    case 1: return launch_grad<64, 1, 8, 8>(a, mode, nblk, st, e0, e1);
    case 2: return launch_grad<64, 2, 8, 8>(a, mode, nblk, st, e0, e1);
    case 4: return launch_grad<64, 4, AA_NW_D1024, AA_RIF_D1024>(a, mode, nblk, st, e0, e1);
    default: return launch_grad<64, 8, 8, 2>(a, mode, nblk, st, e0, e1);
  }
}

hipError_t launch_dense_finalize(const FinalizeArgs &a, hipStream_t st) {
  const int nred = a.d_pad / (4 * kFinCols4) * a.nvec;
  const int extra = a.flags ? compact_tiles(a.P) : 0;
  hipLaunchKernelGGL(k_finalize, dim3(nred + extra), dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace aa
