// C ABI of the AutoAssist hot path: argument checks, workspace carving and the
// choice between the register-resident dense kernels and the general ones.
// Every step of the path runs in the HIP kernels; there is no host fallback.
#include "../../include/autoassist.h"

#include "aa_common.hpp"
#include "aa_dense.hpp"
#include "aa_general.hpp"
#include "aa_batching.hpp"
#include "aa_select.hpp"

#include <mutex>

using namespace aa;

// Scratch of aa_fused_step_static: one copy per GPU the library runs on, held until the
// process ends.  In host code the name below is only a stand-in for the device array; its
// device address is looked up once per device (static_scratch()) and only that address is
// handed to kernels.  The compiler gives the device-side symbol external linkage because
// host code refers to it; that is what lets the runtime find it by name (an attribute that
// pins the symbol, such as `used`, keeps it local and the lookup then aborts the process).
constexpr size_t kStaticScratchBytes = AA_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kCtlUpdateSnapshot = 0;  // control word: update counter before the running step
constexpr int kCtlThresholdNext = 1;   // control word: the running threshold a pass worked out (a float)

struct Ws {
  char *base;
  int32_t *ctl;
  int32_t *blk_cnt;
  float *blk_gb;
  char *grad;         // gradient partials / accumulators
  uint8_t *flags;     // [P]
  float *loss_pool;   // [P]
  int32_t *tile_off;  // [ceil(P/2048) + 2]
  int32_t *bucket_tiles;  // [bucket_table_ints(P)]
  float *prob;        // [P]   per-step outputs of the epoch driver
  int32_t *kept_pos;  // [P]
  int32_t *kept_ids;  // [P]
  float *loss;        // [P]
  uint8_t *flags_odd;    // [P]   second keep-flag / loss buffers of the epoch driver: a step's
  float *loss_pool_odd;  // [P]   flags stay valid while the next step compacts them
  size_t total;
};

// General kernels: a header (scalars, bin fill counts), the two dense accumulators, the
// model vectors as (w, phi) pairs, the per-block sums of the first columns, then the record
// bins of the other columns.
size_t general_pairs_offset(int32_t d) {  // (w, phi) pairs of the columns, indexed by column
  return align_up(general_clear_floats(d) * sizeof(float), 256);
}
size_t general_part_offset(int32_t d) {
  return general_pairs_offset(d) + align_up(2 * (size_t)d * sizeof(float), 256);
}
size_t general_bins_offset(int32_t d) {
  return general_part_offset(d) + align_up(general_part_floats(d) * sizeof(float), 256);
}
size_t general_acc_bytes(int32_t d, int32_t count_max) {
  return general_bins_offset(d) + general_record_capacity(count_max) * sizeof(TailRecord);
}

Ws carve(void *ws, size_t grad_bytes, int32_t P, bool epoch_outputs = false) {
  Ws w;
  w.base = static_cast<char *>(ws);
  w.ctl = reinterpret_cast<int32_t *>(w.base + kWsControl);
  w.blk_cnt = reinterpret_cast<int32_t *>(w.base + kWsBlkCnt);
  w.blk_gb = reinterpret_cast<float *>(w.base + kWsBlkGb);
  size_t off = kWsBody;
  w.grad = w.base + off;
  off += align_up(grad_bytes, 256);
  w.flags = reinterpret_cast<uint8_t *>(w.base + off);
  off += align_up((size_t)(P > 0 ? P : 0), 256);
  w.loss_pool = reinterpret_cast<float *>(w.base + off);
  off += align_up(sizeof(float) * (size_t)(P > 0 ? P : 0), 256);
  w.tile_off = reinterpret_cast<int32_t *>(w.base + off);
  const size_t tiles = ((size_t)(P > 0 ? P : 0) + kCompactTile - 1) / kCompactTile;
  off += align_up(sizeof(int32_t) * (tiles + 2), 256);
  w.bucket_tiles = reinterpret_cast<int32_t *>(w.base + off);
  off += align_up(sizeof(int32_t) * bucket_table_ints(P), 256);
  const size_t per = align_up(sizeof(float) * (size_t)(P > 0 ? P : 0), 256);
  w.prob = reinterpret_cast<float *>(w.base + off);
  w.kept_pos = reinterpret_cast<int32_t *>(w.base + off + per);
  w.kept_ids = reinterpret_cast<int32_t *>(w.base + off + 2 * per);
  w.loss = reinterpret_cast<float *>(w.base + off + 3 * per);
  w.flags_odd = reinterpret_cast<uint8_t *>(w.base + off + 4 * per);
  w.loss_pool_odd = reinterpret_cast<float *>(w.base + off + 5 * per);
  if (epoch_outputs) off += 6 * per;
  w.total = off;
  return w;
}

int32_t check_ws(const void *ws, size_t ws_bytes, size_t need) {
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255) != 0 || ws_bytes < need)
    return AA_ERR_WORKSPACE;
  return AA_OK;
}

int32_t check_features(const aa_features *F) {
  if (!F) return AA_ERR_NULL;
  if (F->d <= 0 || F->n < 0) return AA_ERR_SHAPE;
  if (F->layout == AA_DENSE) {
    if (!F->x) return AA_ERR_NULL;
    if (F->ld < F->d) return AA_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(F->x) & 3) != 0) return AA_ERR_ALIGN;
    return AA_OK;
  }
  if (F->layout == AA_CSR) {
    if (!F->rowptr || !F->col) return AA_ERR_NULL;
    return AA_OK;
  }
  return AA_ERR_SHAPE;
}

int32_t hip_status(hipError_t e) { return e == hipSuccess ? AA_OK : AA_ERR_HIP; }

bool vec_ok(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

hipStream_t as_stream(void *s) { return static_cast<hipStream_t>(s); }

// Timing hook: the next row-pass launches hand their own start and stop time stamps to caller
// events, one pair each (the caller's arrays must outlive the launches they arm).
void *const *g_hook_before = nullptr, *const *g_hook_after = nullptr;
void *g_hook_single[2] = {nullptr, nullptr};
int32_t g_hook_left = 0;

struct Hook {
  hipEvent_t started = nullptr, stopped = nullptr;
  Hook() {
    if (g_hook_left > 0) {
      --g_hook_left;
      started = static_cast<hipEvent_t>(*g_hook_before++);
      stopped = static_cast<hipEvent_t>(*g_hook_after++);
    }
  }
};

#ifdef AA_PHASE_TRACE
// Measurement builds only: where the next whole-step passes write their per-wave phase stamps.
unsigned long long *g_phase_trace = nullptr;
#endif

// Common description of one row pass, lowered to either kernel family.
struct PassSpec {
  const aa_features *F;
  int mode;
  const float *y;
  const int32_t *rows;
  int32_t count_max;
  const int32_t *m_dev;
  float *w;
  float *phi;
  float *bias;
  const float *T;
  float gamma;
  uint64_t seed, step;
  int do_keep;
  float *logit;
  float *prob;
  uint8_t *flags;
  float *loss_out;
  const float *loss_in;
  const int32_t *t_upd;
  CompactArgs prev;  // compaction of the previous pool carried by this pass (fast dense pool pass only)
  // kAssist alone on the fast dense path: take the threshold from the batch's own losses
  // (running median with this momentum; *T and *med_init are rewritten by the update kernel)
  int32_t *med_init;
  float med_momentum;
  // general path: the update kernel of the previous step of this call has left the workspace
  // ready (cleared counts and accumulators, current model pairs): no preparing launch
  bool ws_ready;
};

bool use_fast(const PassSpec &s) {
  if (!dense_fast_ok(s.F)) return false;
  if ((s.mode & kSvm) && !vec_ok(s.w)) return false;
  if ((s.mode & (kPool | kAssist)) && !vec_ok(s.phi)) return false;
  return true;
}

size_t grad_bytes_for(const PassSpec &s) {
  const int nvec = ((s.mode & kSvm) ? 1 : 0) + ((s.mode & kAssist) ? 1 : 0);
  if (nvec == 0) return 0;
  if (use_fast(s))
    return (size_t)dense_pass_blocks(s.F->d, s.count_max, s.mode) * nvec *
           dense_d_pad(s.F->d) * sizeof(float);
  return general_acc_bytes(s.F->d, s.count_max);
}

// Launch the pass (and, for the general family, the accumulator clear before it).
hipError_t run_pass(const PassSpec &s, const Ws &ws, int32_t *nblk_out, hipStream_t st) {
  const float omg = 1.0f - s.gamma;
  if (use_fast(s)) {
    PassArgs a{};
    a.x = s.F->x;
    a.ld = s.F->ld;
    a.d4 = s.F->d / 4;
    a.y = s.y;
    a.rows = s.rows;
    a.count_max = s.count_max;
    a.m_dev = s.m_dev;
    a.w = s.w;
    a.phi = s.phi;
    a.bias = s.bias;
    a.T = s.T;
    a.gamma = s.gamma;
    a.one_minus_gamma = omg;
    a.key = make_draw_key(s.seed, s.step);
    a.do_keep = s.do_keep;
    a.logit = s.logit;
    a.prob = s.prob;
    a.flags = s.flags;
    a.loss_out = s.loss_out;
    a.loss_in = s.loss_in;
    a.partial = reinterpret_cast<float *>(ws.grad);
    a.blk_cnt = ws.blk_cnt;
    a.blk_gb = ws.blk_gb;
    a.t_upd = s.t_upd;
    a.t_snap = ws.ctl + kCtlUpdateSnapshot;
    a.prev = s.prev;
    a.med_init = s.med_init;
    a.med_momentum = s.med_momentum;
    a.T_next = reinterpret_cast<float *>(ws.ctl + kCtlThresholdNext);
#ifdef AA_PHASE_TRACE
    a.trace = g_phase_trace;
#endif
    const int32_t nblk = dense_pass_blocks(s.F->d, s.count_max, s.mode);
    if (a.prev.flags && (a.prev.P > dense_carry_capacity(nblk) ||
                         (reinterpret_cast<uintptr_t>(a.prev.flags) & 15) != 0))
      return hipErrorInvalidValue;  // the caller plans carried compactions within capacity
    *nblk_out = nblk;
    const Hook hook;
    return launch_dense_pass(a, s.mode, s.F->d, nblk, st, hook.started, hook.stopped);
  }
  const bool csr = s.F->layout == AA_CSR;
  float *acc = reinterpret_cast<float *>(ws.grad);
  if ((s.mode & (kSvm | kAssist)) && !s.ws_ready) {
    const size_t clear = general_clear_floats(s.F->d);
    const bool both = (s.mode & kSvm) && (s.mode & kAssist);
    const int32_t head = general_head_columns(s.F->d, 2, csr);
    float2 *pairs = reinterpret_cast<float2 *>(ws.grad + general_pairs_offset(s.F->d));
    hipError_t e = (both && s.F->d > head)
                       ? launch_prepare_general(acc, clear, s.w, s.phi, pairs, head, s.F->d, st)
                       : launch_zero_f32(acc, clear, st);
    if (e != hipSuccess) return e;
  }
  GenArgs a{};
  a.x = s.F->x;
  a.ld = s.F->ld;
  a.d = s.F->d;
  a.rowptr = s.F->rowptr;
  a.col = s.F->col;
  a.val = s.F->val;
  a.y = s.y;
  a.rows = s.rows;
  a.count_max = s.count_max;
  a.m_dev = s.m_dev;
  a.w = s.w;
  a.phi = s.phi;
  a.bias = s.bias;
  a.T = s.T;
  a.gamma = s.gamma;
  a.one_minus_gamma = omg;
  a.key = make_draw_key(s.seed, s.step);
  a.do_keep = s.do_keep;
  a.logit = s.logit;
  a.prob = s.prob;
  a.flags = s.flags;
  a.loss_out = s.loss_out;
  a.loss_in = s.loss_in;
  a.blk_cnt = ws.blk_cnt;
  a.blk_gb = ws.blk_gb;
  const int nvec = ((s.mode & kSvm) ? 1 : 0) + ((s.mode & kAssist) ? 1 : 0);
  a.acc_w = reinterpret_cast<double *>(acc + kGeneralHeader);
  a.acc_used = reinterpret_cast<int32_t *>(acc) + 16 + 2 * kMaxBins;
  a.acc_p = a.acc_w + s.F->d;
  a.part = reinterpret_cast<float *>(ws.grad + general_part_offset(s.F->d));
  a.head = general_head_columns(s.F->d, nvec, csr);
  a.wp = (nvec == 2 && s.F->d > a.head)
             ? reinterpret_cast<const float2 *>(ws.grad + general_pairs_offset(s.F->d))
             : nullptr;
  a.bin_fill = reinterpret_cast<unsigned long long *>(acc + 16);
  a.bins = reinterpret_cast<TailRecord *>(ws.grad + general_bins_offset(s.F->d));
  a.plan = general_bin_plan(s.F->d, a.head, nvec, s.count_max);
  a.t_upd = s.t_upd;
  a.t_snap = ws.ctl + kCtlUpdateSnapshot;
  const int32_t nblk = general_pass_blocks(s.count_max, csr, s.mode);
  *nblk_out = nblk;
  const Hook hook;
  return launch_general_pass(a, s.mode, csr, nblk, st, hook.started, hook.stopped);
}

struct UpdateSpec {
  float lambda, lr, lr_a, l2_a;
  int32_t *t_upd;
  int32_t *kept_hist;
  float *phi_copy;   // optional second destination of the updated Assistant
  float *bias_copy;
  // compaction of a pool pass (flags == NULL: none)
  const uint8_t *flags;
  int32_t P;
  const int32_t *idx;
  int32_t *kept_pos;
  int32_t *kept_ids;
  const float *loss_pool;
  float *loss;
  int32_t *kept_count;
  bool keep_ready;  // general path: leave the workspace ready for the next pass of this call
};

// Fold the gradient sums of the pass into the model.
hipError_t run_update(const PassSpec &s, const UpdateSpec &u, const Ws &ws, int32_t nblk,
                      hipStream_t st) {
  const bool pool = (s.mode & kPool) != 0;
  if (use_fast(s)) {
    FinalizeArgs f{};
    f.partial = reinterpret_cast<const float *>(ws.grad);
    f.nblk = nblk;
    f.nvec = ((s.mode & kSvm) ? 1 : 0) + ((s.mode & kAssist) ? 1 : 0);
    f.d = s.F->d;
    f.d_pad = dense_d_pad(s.F->d);
    f.blk_cnt = ws.blk_cnt;
    f.blk_gb = ws.blk_gb;
    f.m_dev = pool ? nullptr : s.m_dev;
    f.m_max = s.count_max;
    f.w = (s.mode & kSvm) ? s.w : nullptr;
    f.phi = (s.mode & kAssist) ? s.phi : nullptr;
    f.bias = (s.mode & kAssist) ? s.bias : nullptr;
    f.lambda = u.lambda;
    f.lr = u.lr;
    f.lr_a = u.lr_a;
    f.l2_a = u.l2_a;
    f.t_upd = u.t_upd;
    f.kept_hist = u.kept_hist;
    f.phi_copy = u.phi_copy;
    f.bias_copy = u.bias_copy;
    f.t_snap = ws.ctl + kCtlUpdateSnapshot;
    if (s.med_init) {
      f.T_next = reinterpret_cast<const float *>(ws.ctl + kCtlThresholdNext);
      f.T_out = const_cast<float *>(s.T);
      f.T_init = s.med_init;
    }
    f.flags = u.flags;
    f.P = u.P;
    f.idx = u.idx;
    f.kept_pos = u.kept_pos;
    f.kept_ids = u.kept_ids;
    f.loss_pool = u.loss_pool;
    f.loss = u.loss;
    f.kept_count = u.kept_count;
    return launch_dense_finalize(f, st);
  }
  float *acc = reinterpret_cast<float *>(ws.grad);
  ApplyArgs p{};
  p.d = s.F->d;
  p.blk_cnt = ws.blk_cnt;
  p.blk_gb = ws.blk_gb;
  p.acc_w = reinterpret_cast<double *>(acc + kGeneralHeader);
  p.acc_used = reinterpret_cast<int32_t *>(acc) + 16 + 2 * kMaxBins;
  p.acc_p = p.acc_w + s.F->d;
  p.part = reinterpret_cast<const float *>(ws.grad + general_part_offset(s.F->d));
  p.nvec = ((s.mode & kSvm) ? 1 : 0) + ((s.mode & kAssist) ? 1 : 0);
  p.head = general_head_columns(s.F->d, p.nvec, s.F->layout == AA_CSR);
  p.bin_fill = reinterpret_cast<unsigned long long *>(acc + 16);
  p.bins = reinterpret_cast<const TailRecord *>(ws.grad + general_bins_offset(s.F->d));
  p.plan = general_bin_plan(s.F->d, p.head, p.nvec, s.count_max);
  p.t_upd = u.t_upd;
  p.t_snap = ws.ctl + kCtlUpdateSnapshot;
  p.keep_ready = (u.keep_ready && p.plan.nb > 0) ? 1 : 0;
  p.wp_out = (p.keep_ready && p.nvec == 2 && s.F->d > p.head)
                 ? reinterpret_cast<float2 *>(ws.grad + general_pairs_offset(s.F->d))
                 : nullptr;
  p.nblk_pass = nblk;
  p.m_dev = pool ? nullptr : s.m_dev;
  p.m_max = s.count_max;
  p.w = (s.mode & kSvm) ? s.w : nullptr;
  p.phi = (s.mode & kAssist) ? s.phi : nullptr;
  p.bias = (s.mode & kAssist) ? s.bias : nullptr;
  p.lambda = u.lambda;
  p.lr = u.lr;
  p.lr_a = u.lr_a;
  p.l2_a = u.l2_a;
  p.kept_hist = u.kept_hist;
  p.phi_copy = u.phi_copy;
  p.bias_copy = u.bias_copy;
  p.flags = u.flags;
  p.P = u.P;
  p.idx = u.idx;
  p.kept_pos = u.kept_pos;
  p.kept_ids = u.kept_ids;
  p.loss_pool = u.loss_pool;
  p.loss = u.loss;
  p.kept_count = u.kept_count;
  return launch_general_apply(p, st);
}

__global__ __launch_bounds__(1024) void k_project(float *w, int32_t d, float radius,
                                                  const int32_t *m_dev) {
  __shared__ float s_part[16];
  __shared__ float s_scale;
  if (m_dev && *m_dev <= 0) return;
  float ss = 0.f;
  for (int k = threadIdx.x; k < d; k += blockDim.x) ss = __fmaf_rn(w[k], w[k], ss);
  ss = group_sum<kWave>(ss);
  if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = ss;
  __syncthreads();
  if (threadIdx.x == 0) {
    float tot = 0.f;
    for (int i = 0; i < (int)(blockDim.x >> 6); ++i) tot += s_part[i];
    const float nrm = sqrtf(tot);
    s_scale = nrm > radius ? radius / nrm : 1.f;
  }
  __syncthreads();
  const float f = s_scale;
  if (f != 1.f)
    for (int k = threadIdx.x; k < d; k += blockDim.x) w[k] *= f;
}

__global__ void k_zero_i32(int32_t *p, int n) {
  for (int i = threadIdx.x; i < n; i += blockDim.x) p[i] = 0;
}

// Epoch driver state handed to a step: where its batch goes, which of the two flag buffers
// it uses, the compaction it carries for the step before, and whether its own compaction
// may be left to the next step's pass.
struct EpochCtl {
  int32_t P_layout;          // pool size the workspace is laid out for (the epoch's P)
  int parity;
  int32_t *ids_dst;
  float *loss_dst;
  const CompactArgs *carry;  // NULL: nothing to carry
  bool may_defer;
  CompactArgs *deferred;     // out: filled when this step's compaction was left to the next pass
  bool did_defer;
  bool ws_ready;             // in: the previous step of this call left the general workspace ready
  bool left_ready;           // out: this step did
};

int32_t fused_step_impl(const aa_features *F, const float *y, const int32_t *idx, int32_t P,
                        float *w, float *phi, float *bias, const aa_step_config *cfg,
                        uint64_t step, float *logit, float *prob, uint8_t *keep,
                        int32_t *kept_pos, int32_t *kept_ids, float *loss, int32_t *kept_count,
                        int32_t *t_upd, int32_t *kept_hist, EpochCtl *ep, void *ws_ptr,
                        size_t ws_bytes, hipStream_t st, bool hard = false) {
  // hard: keep by the candidate's own loss against *cfg->T, no Assistant (phi, bias unused)
  PassSpec s{};
  s.F = F;
  s.mode = hard ? (kPool | kSvm | kHard) : (kPool | kSvm | kAssist);
  s.y = y;
  s.rows = idx;
  s.count_max = ep ? ep->P_layout : P;  // sizes the gradient partials for the whole epoch
  s.w = w;
  s.phi = phi;
  s.bias = bias;
  s.T = cfg->T;
  s.gamma = cfg->gamma;
  s.seed = cfg->seed;
  s.step = step;
  s.do_keep = hard ? 0 : 1;
  s.logit = logit;
  s.prob = prob;
  s.t_upd = t_upd;
  const bool fast = use_fast(s);
  const size_t gbytes = grad_bytes_for(s);
  Ws ws = carve(ws_ptr, gbytes, s.count_max, ep != nullptr);
  if (int32_t rc = check_ws(ws_ptr, ws_bytes, ws.total)) return rc;
  s.count_max = P;
  float *loss_pool = ws.loss_pool;
  s.flags = keep ? keep : ws.flags;
  if (ep) {  // the batch of each step is assembled in the workspace (or the caller's history)
    s.prob = hard ? nullptr : ws.prob;
    kept_pos = ws.kept_pos;
    kept_ids = ep->ids_dst ? ep->ids_dst : ws.kept_ids;
    loss = ep->loss_dst ? ep->loss_dst : ws.loss;
    if (ep->parity & 1) {
      s.flags = ws.flags_odd;
      loss_pool = ws.loss_pool_odd;
    }
    if (ep->carry && fast) s.prev = *ep->carry;
    ep->did_defer = false;
    s.ws_ready = !fast && ep->ws_ready;
    ep->left_ready = false;
  }
  s.loss_out = loss_pool;
  int32_t nblk = 0;
  hipError_t e = run_pass(s, ws, &nblk, st);
  if (e != hipSuccess) return AA_ERR_HIP;
  UpdateSpec u{};
  u.lambda = cfg->lambda;
  u.lr = cfg->lr;
  u.lr_a = cfg->lr_a;
  u.l2_a = cfg->l2_a;
  u.t_upd = t_upd;
  u.kept_hist = kept_hist;
  u.keep_ready = ep && !fast && general_keeps_ready(F->d, hard ? 1 : 2, F->layout == AA_CSR);
  if (kept_pos || kept_ids || loss || kept_count) {
    CompactArgs c{};
    c.flags = s.flags;
    c.P = P;
    c.idx = idx;
    c.kept_pos = kept_pos;
    c.kept_ids = kept_ids;
    c.loss_pool = loss_pool;
    c.loss = loss;
    c.kept_count = kept_count;
    if (ep && ep->may_defer && fast) {  // the next step's pass compacts this pool
      *ep->deferred = c;
      ep->did_defer = true;
    } else {
      u.flags = c.flags;
      u.P = c.P;
      u.idx = c.idx;
      u.kept_pos = c.kept_pos;
      u.kept_ids = c.kept_ids;
      u.loss_pool = c.loss_pool;
      u.loss = c.loss;
      u.kept_count = c.kept_count;
    }
  }
  const int32_t rc = hip_status(run_update(s, u, ws, nblk, st));
  if (ep && rc == AA_OK) ep->left_ready = u.keep_ready;
  return rc;
}

// Extra workspace of the two-stream pipeline behind the common layout: `ring` batch slots
// (kept ids + kept count) and `ring` Assistant snapshots (phi, then the bias).
struct PipeWs {
  size_t ids_stride, slot_stride, snap_stride;
  char *slots, *snaps;
  size_t total;
  int32_t *ids(int r) const { return reinterpret_cast<int32_t *>(slots + r * slot_stride); }
  int32_t *count(int r) const { return reinterpret_cast<int32_t *>(slots + r * slot_stride + ids_stride); }
  float *phi(int r) const { return reinterpret_cast<float *>(snaps + r * snap_stride); }
};

PipeWs carve_pipeline(char *base, size_t off, int32_t P, int32_t d, int32_t ring) {
  PipeWs p;
  p.ids_stride = align_up(sizeof(int32_t) * (size_t)(P > 0 ? P : 0), 256);
  p.slot_stride = p.ids_stride + 256;
  p.snap_stride = align_up(sizeof(float) * ((size_t)d + 4), 256);
  p.slots = base + off;
  p.snaps = p.slots + (size_t)ring * p.slot_stride;
  p.total = off + (size_t)ring * (p.slot_stride + p.snap_stride);
  return p;
}

__global__ void k_copy_model(const float *phi, const float *bias, int32_t d, float *phi_out,
                             float *bias_out) {
  for (int k = blockIdx.x * blockDim.x + threadIdx.x; k < d; k += gridDim.x * blockDim.x)
    phi_out[k] = phi[k];
  if (blockIdx.x == 0 && threadIdx.x == 0 && bias) *bias_out = *bias;
}

constexpr int kMaxStaleness = 15;

// Device address of this GPU's copy of `scratch`, resolved on the first call per device.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

int32_t static_scratch(void **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return AA_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return AA_ERR_HIP;
    if ((reinterpret_cast<uintptr_t>(p) & 255) != 0) return AA_ERR_ALIGN;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return AA_OK;
}

}  // namespace

extern "C" {

int32_t aa_version(void) { return 100; }

const char *aa_status_string(int32_t status) {
  switch (status) {
    case AA_OK: return "ok";
    case AA_ERR_NULL: return "a required pointer is NULL";
    case AA_ERR_SHAPE: return "bad shape or size";
    case AA_ERR_ALIGN: return "pointer not aligned as required";
    case AA_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case AA_ERR_HIP: return "HIP launch error";
    default: return "unknown status";
  }
}

size_t aa_workspace_bytes(int32_t P_max, int32_t d_max) {
  if (P_max < 0) P_max = 0;
  if (d_max < 1) d_max = 1;
  // any d up to d_max may be used: the register-resident kernels need block partials for
  // d <= 2048, the general kernels dense accumulators
  const int32_t d_fast = d_max < kFastDenseMaxD ? d_max : kFastDenseMaxD;
  size_t grad = (size_t)kMaxBlocks * 2 * dense_d_pad(d_fast) * sizeof(float);
  if (general_acc_bytes(d_max, P_max) > grad) grad = general_acc_bytes(d_max, P_max);
  return carve(nullptr, grad, P_max, true).total;
}

int32_t aa_profile_hook(void *event_before, void *event_after) {
  g_hook_left = 0;
  if (!event_before || !event_after) return event_before || event_after ? AA_ERR_NULL : AA_OK;
  g_hook_single[0] = event_before;
  g_hook_single[1] = event_after;
  g_hook_before = &g_hook_single[0];
  g_hook_after = &g_hook_single[1];
  g_hook_left = 1;
  return AA_OK;
}

int32_t aa_profile_hooks(void *const *events_before, void *const *events_after, int32_t count) {
  g_hook_left = 0;
  if (count < 0) return AA_ERR_SHAPE;
  if (count == 0) return AA_OK;
  if (!events_before || !events_after) return AA_ERR_NULL;
  for (int32_t i = 0; i < count; ++i)
    if (!events_before[i] || !events_after[i]) return AA_ERR_NULL;
  g_hook_before = events_before;
  g_hook_after = events_after;
  g_hook_left = count;
  return AA_OK;
}

int32_t aa_workspace_init(void *ws, size_t ws_bytes, void *stream) {
  if (int32_t rc = check_ws(ws, ws_bytes, kWsBody)) return rc;
  hipLaunchKernelGGL(k_zero_i32, dim3(1), dim3(64), 0, as_stream(stream),
                     reinterpret_cast<int32_t *>(ws), 64);
  return hip_status(hipGetLastError());
}

int32_t aa_assistant_score(const aa_features *F, const int32_t *idx, int32_t P, const float *phi,
                           const float *bias, float *logit, float *prob, void *stream) {
  if (P < 0) return AA_ERR_SHAPE;
  if (P == 0) return AA_OK;
  if (int32_t rc = check_features(F)) return rc;
  if (!phi || !prob) return AA_ERR_NULL;
  PassSpec s{};
  s.F = F;
  s.mode = kPool;
  s.rows = idx;
  s.count_max = P;
  s.phi = const_cast<float *>(phi);
  s.bias = const_cast<float *>(bias);
  s.logit = logit;
  s.prob = prob;
  Ws none{};
  int32_t nblk = 0;
  return hip_status(run_pass(s, none, &nblk, as_stream(stream)));
}

// Compact `flags` into kept_pos / kept_count (shared tail of the shrink entry points).
static int32_t compact_flags(const uint8_t *flags, int32_t P, int32_t *kept_pos,
                             int32_t *kept_count, const Ws &ws, hipStream_t st) {
  CompactArgs c{};
  c.flags = flags;
  c.P = P;
  c.kept_pos = kept_pos;
  c.kept_count = kept_count;
  return hip_status(launch_compact(c, ws.tile_off, st));
}

int32_t aa_shrink(const float *prob, int32_t P, float gamma, uint64_t seed, uint64_t step,
                  uint8_t *keep, int32_t *kept_pos, int32_t *kept_count, void *ws_ptr,
                  size_t ws_bytes, void *stream) {
  if (P < 0) return AA_ERR_SHAPE;
  if (!kept_count) return AA_ERR_NULL;
  if (P > 0 && (!prob || !kept_pos)) return AA_ERR_NULL;
  Ws ws = carve(ws_ptr, 0, P);
  if (int32_t rc = check_ws(ws_ptr, ws_bytes, ws.total)) return rc;
  KeepArgs k{};
  k.src = prob;
  k.P = P;
  k.gamma = gamma;
  k.one_minus_gamma = 1.0f - gamma;
  k.key = make_draw_key(seed, step);
  k.flags = keep ? keep : ws.flags;
  if (launch_keep_flags(k, kFromProb, as_stream(stream)) != hipSuccess) return AA_ERR_HIP;
  return compact_flags(k.flags, P, kept_pos, kept_count, ws, as_stream(stream));
}

int32_t aa_shrink_threshold(const float *crit, int32_t P, const float *T, uint8_t *keep,
                            int32_t *kept_pos, int32_t *kept_count, void *ws_ptr,
                            size_t ws_bytes, void *stream) {
  if (P < 0) return AA_ERR_SHAPE;
  if (!kept_count || !T) return AA_ERR_NULL;
  if (P > 0 && (!crit || !kept_pos)) return AA_ERR_NULL;
  Ws ws = carve(ws_ptr, 0, P);
  if (int32_t rc = check_ws(ws_ptr, ws_bytes, ws.total)) return rc;
  KeepArgs k{};
  k.src = crit;
  k.T = T;
  k.P = P;
  k.flags = keep ? keep : ws.flags;
  if (launch_keep_flags(k, kFromCrit, as_stream(stream)) != hipSuccess) return AA_ERR_HIP;
  return compact_flags(k.flags, P, kept_pos, kept_count, ws, as_stream(stream));
}

int32_t aa_score_shrink(const aa_features *F, const int32_t *idx, int32_t P, const float *phi,
                        const float *bias, float gamma, uint64_t seed, uint64_t step,
                        float *logit, float *prob, uint8_t *keep, int32_t *kept_pos,
                        int32_t *kept_count, void *ws_ptr, size_t ws_bytes, void *stream) {
  if (P < 0) return AA_ERR_SHAPE;
  if (!kept_count) return AA_ERR_NULL;
  Ws ws = carve(ws_ptr, 0, P);
  if (int32_t rc = check_ws(ws_ptr, ws_bytes, ws.total)) return rc;
  if (P == 0) return compact_flags(nullptr, 0, nullptr, kept_count, ws, as_stream(stream));
  if (int32_t rc = check_features(F)) return rc;
  if (!phi || !kept_pos) return AA_ERR_NULL;
  PassSpec s{};
  s.F = F;
  s.mode = kPool;
  s.rows = idx;
  s.count_max = P;
  s.phi = const_cast<float *>(phi);
  s.bias = const_cast<float *>(bias);
  s.gamma = gamma;
  s.seed = seed;
  s.step = step;
  s.do_keep = 1;
  s.logit = logit;
  s.prob = prob;
  s.flags = keep ? keep : ws.flags;
  int32_t nblk = 0;
  if (run_pass(s, ws, &nblk, as_stream(stream)) != hipSuccess) return AA_ERR_HIP;
  return compact_flags(s.flags, P, kept_pos, kept_count, ws, as_stream(stream));
}

int32_t aa_gather(const void *src, int64_t row_bytes, const int32_t *idx, const int32_t *kept_pos,
                  const int32_t *kept_count, int32_t max_rows, void *dst, int32_t *kept_ids,
                  void *stream) {
  if (max_rows < 0 || row_bytes < 0) return AA_ERR_SHAPE;
  if (!kept_count) return AA_ERR_NULL;
  if ((src == nullptr) != (dst == nullptr)) return AA_ERR_NULL;
  GatherArgs g{};
  g.src = static_cast<const char *>(src);
  g.dst = static_cast<char *>(dst);
  g.row_bytes = row_bytes;
  g.idx = idx;
  g.kept_pos = kept_pos;
  g.kept_count = kept_count;
  g.max_rows = max_rows;
  g.kept_ids = kept_ids;
  return hip_status(launch_gather(g, as_stream(stream)));
}

int32_t aa_gather_csr(const aa_features *F, const int32_t *idx, const int32_t *kept_pos,
                      const int32_t *kept_count, int32_t max_rows, int64_t *out_rowptr,
                      int32_t *out_col, float *out_val, int64_t out_nnz_cap, void *ws_ptr,
                      size_t ws_bytes, void *stream) {
  if (max_rows < 0 || out_nnz_cap < 0) return AA_ERR_SHAPE;
  if (int32_t rc = check_features(F)) return rc;
  if (F->layout != AA_CSR) return AA_ERR_SHAPE;
  if (!kept_count || !out_rowptr) return AA_ERR_NULL;
  if (out_nnz_cap > 0 && !out_col) return AA_ERR_NULL;
  if (F->val && out_nnz_cap > 0 && !out_val) return AA_ERR_NULL;
  GatherCsrArgs g{};
  g.rowptr = F->rowptr;
  g.col = F->col;
  g.val = F->val;
  g.idx = idx;
  g.kept_pos = kept_pos;
  g.kept_count = kept_count;
  g.max_rows = max_rows;
  g.out_rowptr = out_rowptr;
  g.out_col = out_col;
  g.out_val = out_val;
  g.out_nnz_cap = out_nnz_cap;
  // many rows: the row-pointer scan runs tile by tile and keeps its tile offsets in the workspace
  long long *tiles = nullptr;
  if (max_rows > 1024) {
    Ws ws = carve(ws_ptr, 0, max_rows);
    if (int32_t rc = check_ws(ws_ptr, ws_bytes, ws.total)) return rc;
    tiles = reinterpret_cast<long long *>(ws.bucket_tiles);
  }
  return hip_status(launch_gather_csr(g, tiles, as_stream(stream)));
}

int32_t aa_svm_sgd_step(const aa_features *F, const float *y, const int32_t *rows,
                        const int32_t *m_dev, int32_t m_max, float *w, float lambda, float lr,
                        float radius, float *loss, void *ws_ptr, size_t ws_bytes, void *stream) {
  if (m_max < 0) return AA_ERR_SHAPE;
  if (m_max == 0) return AA_OK;
  if (int32_t rc = check_features(F)) return rc;
  if (!y || !w || !m_dev) return AA_ERR_NULL;
  PassSpec s{};
  s.F = F;
  s.mode = kSvm;
  s.y = y;
  s.rows = rows;
  s.count_max = m_max;
  s.m_dev = m_dev;
  s.w = w;
  s.loss_out = loss;
  Ws ws = carve(ws_ptr, grad_bytes_for(s), 0);
  if (int32_t rc = check_ws(ws_ptr, ws_bytes, ws.total)) return rc;
  int32_t nblk = 0;
  hipStream_t st = as_stream(stream);
  if (run_pass(s, ws, &nblk, st) != hipSuccess) return AA_ERR_HIP;
  UpdateSpec u{};
  u.lambda = lambda;
  u.lr = lr;
  if (run_update(s, u, ws, nblk, st) != hipSuccess) return AA_ERR_HIP;
  if (radius > 0.f) {
    hipLaunchKernelGGL(k_project, dim3(1), dim3(1024), 0, st, w, F->d, radius, m_dev);
    return hip_status(hipGetLastError());
  }
  return AA_OK;
}

int32_t aa_assistant_update(const aa_features *F, const int32_t *rows, const int32_t *m_dev,
                            int32_t m_max, const float *loss, const float *T, float *phi,
                            float *bias, float lr_a, float l2_a, void *ws_ptr, size_t ws_bytes,
                            void *stream) {
  if (m_max < 0) return AA_ERR_SHAPE;
  if (m_max == 0) return AA_OK;
  if (int32_t rc = check_features(F)) return rc;
  if (!loss || !T || !phi || !m_dev) return AA_ERR_NULL;
  PassSpec s{};
  s.F = F;
  s.mode = kAssist;
  s.rows = rows;
  s.count_max = m_max;
  s.m_dev = m_dev;
  s.phi = phi;
  s.bias = bias;
  s.T = T;
  s.loss_in = loss;
  Ws ws = carve(ws_ptr, grad_bytes_for(s), 0);
  if (int32_t rc = check_ws(ws_ptr, ws_bytes, ws.total)) return rc;
  int32_t nblk = 0;
  hipStream_t st = as_stream(stream);
  if (run_pass(s, ws, &nblk, st) != hipSuccess) return AA_ERR_HIP;
  UpdateSpec u{};
  u.lr_a = lr_a;
  u.l2_a = l2_a;
  return hip_status(run_update(s, u, ws, nblk, st));
}

int32_t aa_threshold_assistant_update(const aa_features *F, const int32_t *rows, const int32_t *m_dev,
                                      int32_t m_max, const float *loss, float momentum, float *T,
                                      int32_t *initialised, float *phi, float *bias, float lr_a,
                                      float l2_a, void *ws_ptr, size_t ws_bytes, void *stream) {
  if (m_max < 0 || m_max > kMedianMax) return AA_ERR_SHAPE;
  if (!(momentum >= 0.f && momentum <= 1.f)) return AA_ERR_SHAPE;
  if (m_max == 0) return AA_OK;
  if (int32_t rc = check_features(F)) return rc;
  if (!loss || !T || !initialised || !phi || !m_dev) return AA_ERR_NULL;
  PassSpec s{};
  s.F = F;
  s.mode = kAssist;
  s.rows = rows;
  s.count_max = m_max;
  s.m_dev = m_dev;
  s.phi = phi;
  s.bias = bias;
  s.T = T;
  s.loss_in = loss;
  if (!use_fast(s) || m_max > kRankSelectMax) {  // no room in that pass: the two calls it stands for
    if (int32_t rc = aa_threshold_update(loss, m_dev, m_max, momentum, T, initialised, stream)) return rc;
    return aa_assistant_update(F, rows, m_dev, m_max, loss, T, phi, bias, lr_a, l2_a, ws_ptr, ws_bytes,
                               stream);
  }
  s.med_init = initialised;
  s.med_momentum = momentum;
  Ws ws = carve(ws_ptr, grad_bytes_for(s), 0);
  if (int32_t rc = check_ws(ws_ptr, ws_bytes, ws.total)) return rc;
  int32_t nblk = 0;
  hipStream_t st = as_stream(stream);
  if (run_pass(s, ws, &nblk, st) != hipSuccess) return AA_ERR_HIP;
  UpdateSpec u{};
  u.lr_a = lr_a;
  u.l2_a = l2_a;
  return hip_status(run_update(s, u, ws, nblk, st));
}

int32_t aa_boss_assistant_step(const aa_features *F, const float *y, const int32_t *rows,
                               const int32_t *m_dev, int32_t m_max, float *w, float *phi,
                               float *bias, const aa_step_config *cfg, float *loss, void *ws_ptr,
                               size_t ws_bytes, void *stream) {
  if (m_max < 0) return AA_ERR_SHAPE;
  if (m_max == 0) return AA_OK;
  if (int32_t rc = check_features(F)) return rc;
  if (!y || !w || !phi || !cfg || !cfg->T || !m_dev) return AA_ERR_NULL;
  PassSpec s{};
  s.F = F;
  s.mode = kSvm | kAssist;
  s.y = y;
  s.rows = rows;
  s.count_max = m_max;
  s.m_dev = m_dev;
  s.w = w;
  s.phi = phi;
  s.bias = bias;
  s.T = cfg->T;
  s.loss_out = loss;
  Ws ws = carve(ws_ptr, grad_bytes_for(s), 0);
  if (int32_t rc = check_ws(ws_ptr, ws_bytes, ws.total)) return rc;
  int32_t nblk = 0;
  hipStream_t st = as_stream(stream);
  if (run_pass(s, ws, &nblk, st) != hipSuccess) return AA_ERR_HIP;
  UpdateSpec u{};
  u.lambda = cfg->lambda;
  u.lr = cfg->lr;
  u.lr_a = cfg->lr_a;
  u.l2_a = cfg->l2_a;
  return hip_status(run_update(s, u, ws, nblk, st));
}

int32_t aa_fused_step(const aa_features *F, const float *y, const int32_t *idx, int32_t P,
                      float *w, float *phi, float *bias, const aa_step_config *cfg, float *logit,
                      float *prob, uint8_t *keep, int32_t *kept_pos, int32_t *kept_ids,
                      float *loss, int32_t *kept_count, void *ws, size_t ws_bytes, void *stream) {
  if (P < 0) return AA_ERR_SHAPE;
  if (!kept_count) return AA_ERR_NULL;
  if (P == 0) {
    CompactArgs c{};
    c.kept_count = kept_count;
    return hip_status(launch_compact(c, nullptr, as_stream(stream)));
  }
  if (int32_t rc = check_features(F)) return rc;
  if (!y || !w || !phi || !cfg || !cfg->T) return AA_ERR_NULL;
  return fused_step_impl(F, y, idx, P, w, phi, bias, cfg, cfg->step, logit, prob, keep, kept_pos,
                         kept_ids, loss, kept_count, nullptr, nullptr, nullptr, ws, ws_bytes,
                         as_stream(stream));
}

#ifdef AA_PHASE_TRACE
// Measurement builds only (not part of the product ABI): the whole-step dense passes launched
// from now on write kTraceStamps 64-bit time stamps (10 ns ticks) per wave into `buf`
// (device memory, blocks x waves x kTraceStamps entries); NULL stops it.
int32_t aa_phase_trace_buffer(void *buf) {
  g_phase_trace = static_cast<unsigned long long *>(buf);
  return AA_OK;
}
#endif

size_t aa_static_scratch_bytes(void) { return kStaticScratchBytes; }

int32_t aa_fused_step_static(const aa_features *F, const float *y, const int32_t *idx, int32_t P,
                             float *w, float *phi, float *bias, const aa_step_config *cfg,
                             float *logit, float *prob, uint8_t *keep, int32_t *kept_pos,
                             int32_t *kept_ids, float *loss, int32_t *kept_count, void *stream) {
  if (P < 0) return AA_ERR_SHAPE;
  if (!kept_count) return AA_ERR_NULL;
  if (P == 0) {
    CompactArgs c{};
    c.kept_count = kept_count;
    return hip_status(launch_compact(c, nullptr, as_stream(stream)));
  }
  if (int32_t rc = check_features(F)) return rc;
  if (!y || !w || !phi || !cfg || !cfg->T) return AA_ERR_NULL;
  void *ws = nullptr;
  if (int32_t rc = static_scratch(&ws)) return rc;
  // Every word of the scratch this step reads it has written before in the same call (block
  // partials, per-block counts, flags, per-position losses), so nothing needs clearing; a
  // step that needs more than the array holds is refused with AA_ERR_WORKSPACE.
  return fused_step_impl(F, y, idx, P, w, phi, bias, cfg, cfg->step, logit, prob, keep, kept_pos,
                         kept_ids, loss, kept_count, nullptr, nullptr, nullptr, ws,
                         kStaticScratchBytes, as_stream(stream));
}

int32_t aa_sk_step(const aa_features *F, const float *y, const int32_t *idx, int32_t P, float *w,
                   const float *T, float lambda, float lr, float *loss_pool, uint8_t *keep,
                   int32_t *kept_pos, int32_t *kept_ids, float *loss, int32_t *kept_count,
                   void *ws_ptr, size_t ws_bytes, void *stream) {
  if (P < 0) return AA_ERR_SHAPE;
  if (!kept_count) return AA_ERR_NULL;
  hipStream_t st = as_stream(stream);
  if (P == 0) {
    CompactArgs c{};
    c.kept_count = kept_count;
    return hip_status(launch_compact(c, nullptr, st));
  }
  if (int32_t rc = check_features(F)) return rc;
  if (!y || !w || !T) return AA_ERR_NULL;
  PassSpec s{};
  s.F = F;
  s.mode = kPool | kSvm | kHard;
  s.y = y;
  s.rows = idx;
  s.count_max = P;
  s.w = w;
  s.T = T;
  Ws ws = carve(ws_ptr, grad_bytes_for(s), P);
  if (int32_t rc = check_ws(ws_ptr, ws_bytes, ws.total)) return rc;
  s.flags = keep ? keep : ws.flags;
  s.loss_out = loss_pool ? loss_pool : ws.loss_pool;
  int32_t nblk = 0;
  if (run_pass(s, ws, &nblk, st) != hipSuccess) return AA_ERR_HIP;
  UpdateSpec u{};
  u.lambda = lambda;
  u.lr = lr;
  u.flags = s.flags;
  u.P = P;
  u.idx = idx;
  u.kept_pos = kept_pos;
  u.kept_ids = kept_ids;
  u.loss_pool = s.loss_out;
  u.loss = loss;
  u.kept_count = kept_count;
  return hip_status(run_update(s, u, ws, nblk, st));
}

int32_t aa_threshold_update(const float *loss, const int32_t *m_dev, int32_t m_max, float momentum,
                            float *T, int32_t *initialised, void *stream) {
  if (m_max < 0 || m_max > kMedianMax) return AA_ERR_SHAPE;
  if (!(momentum >= 0.f && momentum <= 1.f)) return AA_ERR_SHAPE;
  if (m_max == 0) return AA_OK;
  if (!loss || !m_dev || !T || !initialised) return AA_ERR_NULL;
  ThresholdArgs a{loss, m_dev, m_max, momentum, T, initialised};
  return hip_status(launch_threshold_update(a, as_stream(stream)));
}

int32_t aa_bucket_batches(const int32_t *len_s, const int32_t *len_t, const int32_t *m_dev,
                          int32_t m_max, int32_t width, int32_t n_buckets, int32_t token_budget,
                          int32_t *order, int32_t *bucket_start, int32_t *batch_of,
                          int32_t *n_batches, void *ws_ptr, size_t ws_bytes, void *stream) {
  if (m_max < 0 || width <= 0 || n_buckets <= 0 || n_buckets > kMaxBuckets || token_budget <= 0)
    return AA_ERR_SHAPE;
  if (!m_dev || !bucket_start || !n_batches) return AA_ERR_NULL;
  if (m_max > 0 && (!len_s || !len_t || !order || !batch_of)) return AA_ERR_NULL;
  Ws ws = carve(ws_ptr, 0, m_max);
  if (int32_t rc = check_ws(ws_ptr, ws_bytes, ws.total)) return rc;
  // what the three kernels index: one row of n_buckets counts per tile, then two tail rows
  const size_t tiles = ((size_t)m_max + kBucketTile - 1) / kBucketTile;
  if ((tiles + 2) * (size_t)n_buckets > bucket_table_ints(m_max)) return AA_ERR_WORKSPACE;
  BucketArgs a{};
  a.len_s = len_s;
  a.len_t = len_t;
  a.m_dev = m_dev;
  a.m_max = m_max;
  a.width = width;
  a.n_buckets = n_buckets;
  a.token_budget = token_budget;
  a.order = order;
  a.bucket_start = bucket_start;
  a.batch_of = batch_of;
  a.n_batches = n_batches;
  a.tile_base = ws.bucket_tiles;
  return hip_status(launch_bucket_batches(a, as_stream(stream)));
}

// The epoch loop of aa_train_epoch and aa_sk_epoch (hard: no Assistant, keep by own loss).
static int32_t epoch_impl(const aa_features *F, const float *y, const int32_t *perm, int64_t n_perm,
                          int32_t P, float *w, float *phi, float *bias, const aa_step_config *cfg,
                          int32_t *t_upd, int32_t *kept_hist, int32_t *kept_ids_hist,
                          float *loss_hist, void *ws, size_t ws_bytes, void *stream, bool hard) {
  if (P <= 0 || n_perm < 0) return AA_ERR_SHAPE;
  if (n_perm == 0) return AA_OK;
  if (int32_t rc = check_features(F)) return rc;
  if (!y || !w || (!hard && !phi) || !cfg || !cfg->T || !perm) return AA_ERR_NULL;
  const int64_t steps = (n_perm + P - 1) / P;
  const int mode = hard ? (kPool | kSvm | kHard) : (kPool | kSvm | kAssist);
  CompactArgs pending{};
  bool have_pending = false;
  bool ws_ready = false;  // (the first step of a call always prepares the workspace itself)
  for (int64_t t = 0; t < steps; ++t) {
    const int64_t lo = t * P;
    const int32_t Pt = (int32_t)((n_perm - lo) < P ? (n_perm - lo) : P);
    EpochCtl ep{};
    ep.P_layout = P;
    ep.parity = (int)(t & 1);
    ep.ids_dst = kept_ids_hist ? kept_ids_hist + t * (int64_t)P : nullptr;
    ep.loss_dst = loss_hist ? loss_hist + t * (int64_t)P : nullptr;
    ep.carry = have_pending ? &pending : nullptr;
    ep.ws_ready = ws_ready;
    CompactArgs mine{};
    ep.deferred = &mine;
    // This pool's compaction rides on the next step's pass when that pass has a block for
    // every 64 positions of this pool; the last step compacts in its own update kernel.
    if (t + 1 < steps) {
      const int64_t left = n_perm - (lo + P);
      const int32_t P_next = (int32_t)(left < P ? left : P);
      ep.may_defer = Pt <= dense_carry_capacity(dense_pass_blocks(F->d, P_next, mode));
    }
    const int32_t rc = fused_step_impl(F, y, perm + lo, Pt, w, phi, bias, cfg, cfg->step + t,
                                       nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                                       nullptr, t_upd, kept_hist ? kept_hist + t : nullptr, &ep, ws,
                                       ws_bytes, as_stream(stream), hard);
    if (rc != AA_OK) return rc;
    have_pending = ep.did_defer;
    pending = mine;
    ws_ready = ep.left_ready;
  }
  return AA_OK;
}

int32_t aa_train_epoch(const aa_features *F, const float *y, const int32_t *perm, int64_t n_perm,
                       int32_t P, float *w, float *phi, float *bias, const aa_step_config *cfg,
                       int32_t *t_upd, int32_t *kept_hist, int32_t *kept_ids_hist,
                       float *loss_hist, void *ws, size_t ws_bytes, void *stream) {
  return epoch_impl(F, y, perm, n_perm, P, w, phi, bias, cfg, t_upd, kept_hist, kept_ids_hist,
                    loss_hist, ws, ws_bytes, stream, false);
}

int32_t aa_sk_epoch(const aa_features *F, const float *y, const int32_t *perm, int64_t n_perm,
                    int32_t P, float *w, const float *T, float lambda, float lr0, int32_t *t_upd,
                    int32_t *kept_hist, int32_t *kept_ids_hist, float *loss_hist, void *ws,
                    size_t ws_bytes, void *stream) {
  aa_step_config cfg{};
  cfg.lambda = lambda;
  cfg.lr = lr0;
  cfg.T = T;
  return epoch_impl(F, y, perm, n_perm, P, w, nullptr, nullptr, &cfg, t_upd, kept_hist, kept_ids_hist,
                    loss_hist, ws, ws_bytes, stream, true);
}

size_t aa_pipeline_workspace_bytes(int32_t P_max, int32_t d_max, int32_t staleness) {
  if (staleness < 0) staleness = 0;
  if (staleness > kMaxStaleness) staleness = kMaxStaleness;
  const size_t base = aa_workspace_bytes(P_max, d_max);
  return carve_pipeline(nullptr, base, P_max, d_max < 1 ? 1 : d_max, staleness + 1).total;
}

int32_t aa_train_epoch_stale(const aa_features *F, const float *y, const int32_t *perm,
                             int64_t n_perm, int32_t P, int32_t staleness, float *w, float *phi,
                             float *bias, const aa_step_config *cfg, int32_t *t_upd,
                             int32_t *kept_hist, int32_t *kept_ids_hist, void *ws_ptr,
                             size_t ws_bytes, void *stream_boss, void *stream_gen) {
  if (P <= 0 || n_perm < 0 || staleness < 0 || staleness > kMaxStaleness) return AA_ERR_SHAPE;
  if (n_perm == 0) return AA_OK;
  if (int32_t rc = check_features(F)) return rc;
  if (!y || !w || !phi || !cfg || !cfg->T || !perm) return AA_ERR_NULL;
  hipStream_t sb = as_stream(stream_boss), sg = as_stream(stream_gen);
  if (sb == sg) return AA_ERR_SHAPE;  // the generator needs a stream of its own
  const int ring = staleness + 1;
  const int64_t steps = (n_perm + P - 1) / P;

  // Boss pass over kept rows: the description every tick shares
  PassSpec boss{};
  boss.F = F;
  boss.mode = kSvm | kAssist;
  boss.y = y;
  boss.count_max = P;
  boss.w = w;
  boss.phi = phi;
  boss.bias = bias;
  boss.T = cfg->T;
  boss.t_upd = t_upd;
  const size_t need_common = aa_workspace_bytes(P, F->d);
  Ws ws = carve(ws_ptr, grad_bytes_for(boss), P, true);
  if (ws.total > need_common) return AA_ERR_WORKSPACE;
  PipeWs pw = carve_pipeline(static_cast<char *>(ws_ptr), need_common, P, F->d, ring);
  if (int32_t rc = check_ws(ws_ptr, ws_bytes, pw.total)) return rc;
  boss.loss_out = ws.loss;

  hipEvent_t ev_boss[kMaxStaleness + 1], ev_gen[kMaxStaleness + 1], ev_start;
  if (hipEventCreateWithFlags(&ev_start, hipEventDisableTiming) != hipSuccess) return AA_ERR_HIP;
  int made = 0;  // complete (Boss, generator) event pairs
  int32_t rc = AA_OK;
  while (made < ring) {
    if (hipEventCreateWithFlags(&ev_boss[made], hipEventDisableTiming) != hipSuccess) break;
    if (hipEventCreateWithFlags(&ev_gen[made], hipEventDisableTiming) != hipSuccess) {
      (void)hipEventDestroy(ev_boss[made]);
      break;
    }
    ++made;
  }
  if (made < ring) rc = AA_ERR_HIP;
  auto hip_ok = [&rc](hipError_t e) {
    if (e != hipSuccess && rc == AA_OK) rc = AA_ERR_HIP;
    return rc == AA_OK;
  };

  if (rc == AA_OK) {
    // version 0 of the Assistant: what every batch made before the first feedback is drawn with
    hipLaunchKernelGGL(k_copy_model, dim3((F->d + 1023) / 1024 > 64 ? 64 : (F->d + 1023) / 1024),
                       dim3(1024), 0, sb, phi, bias, F->d, pw.phi(0), pw.phi(0) + F->d);
    hip_ok(hipGetLastError());
    hip_ok(hipEventRecord(ev_start, sb));
    hip_ok(hipStreamWaitEvent(sg, ev_start, 0));
  }
  for (int64_t s = 0; s < steps && rc == AA_OK; ++s) {
    const int64_t lo = s * P;
    const int32_t Ps = (int32_t)((n_perm - lo) < P ? (n_perm - lo) : P);
    const int slot = (int)(s % ring);
    int32_t *ids = kept_ids_hist ? kept_ids_hist + s * (int64_t)P : pw.ids(slot);
    int32_t *count = pw.count(slot);

    // ---- generator: batch s from the Assistant as it stood after s - staleness updates
    const int64_t version = s > staleness ? s - staleness : 0;
    // that version is written by the Boss tick before it, which also is the last reader of
    // the batch slot and the writer of the snapshot slot reused here
    if (version > 0) hip_ok(hipStreamWaitEvent(sg, ev_boss[(version - 1) % ring], 0));
    PassSpec g{};
    g.F = F;
    g.mode = kPool;
    g.rows = perm + lo;
    g.count_max = Ps;
    g.phi = pw.phi((int)(version % ring));
    g.bias = bias ? g.phi + F->d : nullptr;
    g.gamma = cfg->gamma;
    g.seed = cfg->seed;
    g.step = cfg->step + (uint64_t)s;
    g.do_keep = 1;
    g.flags = ws.flags;
    int32_t nblk = 0;
    if (rc == AA_OK) hip_ok(run_pass(g, ws, &nblk, sg));
    CompactArgs c{};
    c.flags = ws.flags;
    c.P = Ps;
    c.idx = perm + lo;
    c.kept_ids = ids;
    c.kept_count = count;
    if (rc == AA_OK) hip_ok(launch_compact(c, ws.tile_off, sg));
    if (rc == AA_OK) hip_ok(hipEventRecord(ev_gen[slot], sg));

    // ---- Boss tick s, then the Assistant update from its losses; the updated Assistant is
    // also stored as version s + 1
    if (rc == AA_OK) hip_ok(hipStreamWaitEvent(sb, ev_gen[slot], 0));
    boss.rows = ids;
    boss.count_max = Ps;
    boss.m_dev = count;
    if (rc == AA_OK) hip_ok(run_pass(boss, ws, &nblk, sb));
    UpdateSpec u{};
    u.lambda = cfg->lambda;
    u.lr = cfg->lr;
    u.lr_a = cfg->lr_a;
    u.l2_a = cfg->l2_a;
    u.t_upd = t_upd;
    u.kept_hist = kept_hist ? kept_hist + s : nullptr;
    u.phi_copy = pw.phi((int)((s + 1) % ring));
    u.bias_copy = u.phi_copy + F->d;
    if (rc == AA_OK) hip_ok(run_update(boss, u, ws, nblk, sb));
    if (rc == AA_OK) hip_ok(hipEventRecord(ev_boss[slot], sb));
  }
  // every generator launch is waited for by a Boss tick, so the Boss stream ends the epoch
  (void)hipEventDestroy(ev_start);
  for (int i = 0; i < made; ++i) {
    (void)hipEventDestroy(ev_boss[i]);
    (void)hipEventDestroy(ev_gen[i]);
  }
  return rc;
}

}  // extern "C"
