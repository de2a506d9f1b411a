// Host side of the C ABI declared in include/maaso.h: argument validation, the context, launch
// shapes.  Every step of the scoring path runs in the kernels of sweep_kernels.hpp and
// assign_kernels.hpp; nothing here computes on the CPU beyond table validation and the reciprocals
// of the class deadlines.
#include "../../include/maaso.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <new>

#include "assign_kernels.hpp"
#include "sweep_kernels.hpp"
#include "partition_kernels.hpp"
#include "probe_kernels.hpp"
#include "profile_fit_kernels.hpp"
#include "sweep_window_kernels.hpp"
#include "sweep_seq_kernels.hpp"
#include "window_kernels.hpp"

using namespace maaso;

static_assert(MAASO_MAX_SLO == kMaxSlo, "header and kernels disagree on the class limit");

constexpr uint32_t kMaxTimed = 256;
constexpr size_t kSmallBytes = 256;

// Workspace of maaso_placement_sweep_noalloc: device memory that exists from the moment the library
// is loaded, one copy per GPU, so that the call has nothing to allocate.  In host code the array's
// name is only a handle for hipGetSymbolAddress; kernels are given the address resolved per device.
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[MAASO_NOALLOC_SCRATCH_BYTES];
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

struct maaso_ctx {
  int device;
  uint32_t n_tp, b_cap, cells, n_slo;
  float d_ttft[kMaxSlo], d_tbt[kMaxSlo], i_ttft[kMaxSlo], i_tbt[kMaxSlo];
  float* tab;           // device: three tables back to back, then tp_degree [n_tp] as uint32
  bool has_degree;      // the profile came with GPUs-per-instance figures
  uint32_t* status;     // device status word
  uint32_t* cls_count;  // device [kMaxSlo]
  void* scratch_ptr;    // this device's copy of the static scratch array
  void* ws;             // device workspace: sized at load, resized only by maaso_ctx_reserve
  size_t ws_bytes;
  uint32_t ws_allocations;  // how often the workspace has been allocated (load counts as one)
  // one call at a time: the host part of a call is exclusive, and a call on another stream than the
  // context's previous call is ordered behind it with an event
  std::atomic<int> in_call;
  hipEvent_t order_ev;
  hipStream_t last_stream;
  bool has_last;
  uint32_t sweep_q;      // 0 = automatic
  uint32_t sweep_group;  // 0 = automatic
  uint32_t sweep_blocks_per_queue;  // 0 = automatic
  unsigned long long* last_evaluated;  // device word written by the last sweep, or null
  bool counters_dirty;   // class counters may be non-zero (a call failed between its launches)
  uint32_t window_blocks;  // 0 = automatic
  uint32_t spin_limit;     // polls of the inter-window barrier before a block gives up
  bool window_profile;     // the windowed distributor records where block 0 spends its cycles
  bool window_profiled;    // ... and the last windowed call did
  int n_cu;
  int cooperative;      // the device launches cooperative grids (all blocks resident, or refused)
  int sweep_resident[4];  // blocks of sweep_kernel<2|4|8|16> one compute unit holds at once
  size_t lds_per_block;
  // optional timing of the dominant kernel of each call (HIP events on the call's stream)
  bool timing;
  uint32_t n_timed;
  hipEvent_t ev_start[kMaxTimed], ev_stop[kMaxTimed];
};

namespace {

struct DeviceGuard {
  int prev = -1;
  bool ok = true;
  explicit DeviceGuard(int dev) {
    if (hipGetDevice(&prev) != hipSuccess) { ok = false; (void)hipGetLastError(); return; }
    if (prev != dev && hipSetDevice(dev) != hipSuccess) { ok = false; (void)hipGetLastError(); }
  }
  ~DeviceGuard() {
    int cur = -1;
    if (prev >= 0 && hipGetDevice(&cur) == hipSuccess && cur != prev) (void)hipSetDevice(prev);
  }
};

inline bool hip_ok(hipError_t e) {
  if (e == hipSuccess) return true;
  (void)hipGetLastError();
  return false;
}

// Event pair around the dominant kernel of a call, when timing is on and slots are left.
struct TimedRegion {
  maaso_ctx* ctx;
  hipStream_t s;
  bool on;
  TimedRegion(maaso_ctx* c, hipStream_t st) : ctx(c), s(st), on(c->timing && c->n_timed < kMaxTimed) {
    if (on) on = hipEventRecord(ctx->ev_start[ctx->n_timed], s) == hipSuccess;
  }
  ~TimedRegion() {
    if (on && hipEventRecord(ctx->ev_stop[ctx->n_timed], s) == hipSuccess) ctx->n_timed += 1;
  }
};

// Compute calls never allocate: a call whose shape needs more than the context holds is refused.
int need_workspace(const maaso_ctx* ctx, size_t bytes) {
  return bytes <= ctx->ws_bytes ? MAASO_OK : MAASO_E_WORKSPACE;
}

// Set-up only (load, maaso_ctx_reserve): (re)allocates the workspace when it is too small.
int alloc_workspace(maaso_ctx* ctx, size_t bytes) {
  if (bytes <= ctx->ws_bytes) return MAASO_OK;
  if (ctx->ws) {
    if (!hip_ok(hipDeviceSynchronize())) return MAASO_E_HIP;
    (void)hipFree(ctx->ws);
    ctx->ws = nullptr;
    ctx->ws_bytes = 0;
  }
  const size_t want = (bytes + (size_t(1) << 20) - 1) & ~((size_t(1) << 20) - 1);
  if (!hip_ok(hipMalloc(&ctx->ws, want))) { ctx->ws = nullptr; return MAASO_E_NOMEM; }
  ctx->ws_bytes = want;
  ctx->ws_allocations += 1;
  return MAASO_OK;
}

// Exclusive use of a context by one call, and stream order between consecutive calls.  The context's
// workspace, class counters and accumulators are shared by all its calls; calls issued on one stream
// are ordered by the stream, and a call issued on another stream than the previous one is made to
// wait for it: an event is recorded on the previous stream at that moment (it covers everything
// issued there so far) and the new stream waits for it - no host synchronisation.  Should the
// previous stream no longer exist, the device is synchronised instead.
struct CallGuard {
  maaso_ctx* ctx;
  int rc;
  CallGuard(maaso_ctx* c, hipStream_t s) : ctx(c), rc(MAASO_OK) {
    int idle = 0;
    if (!ctx->in_call.compare_exchange_strong(idle, 1, std::memory_order_acquire)) {
      ctx = nullptr;
      rc = MAASO_E_BUSY;
      return;
    }
    if (ctx->has_last && ctx->last_stream != s) {
      const bool ordered = hipEventRecord(ctx->order_ev, ctx->last_stream) == hipSuccess &&
                           hipStreamWaitEvent(s, ctx->order_ev, 0) == hipSuccess;
      if (!ordered) {
        (void)hipGetLastError();
        if (!hip_ok(hipDeviceSynchronize())) rc = MAASO_E_HIP;
      }
    }
    ctx->last_stream = s;
    ctx->has_last = true;
  }
  ~CallGuard() {
    if (ctx) ctx->in_call.store(0, std::memory_order_release);
  }
  CallGuard(const CallGuard&) = delete;
  CallGuard& operator=(const CallGuard&) = delete;
};

int check_common(const maaso_ctx* ctx, const maaso_placements* pl, const maaso_requests* rq,
                 const maaso_params* prm) {
  if (!ctx || !pl || !rq || !prm) return MAASO_E_INVALID_ARG;
  if (pl->n_cand == 0 || !pl->n_inst || !pl->tp_idx || !pl->max_batch || !pl->occ || !pl->q_ticks)
    return MAASO_E_INVALID_ARG;
  if (pl->i_pad == 0 || pl->i_pad > MAASO_MAX_INSTANCES) return MAASO_E_SHAPE;
  if (rq->n_req != 0 && (!rq->prompt_len || !rq->out_len || !rq->slo_class))
    return MAASO_E_INVALID_ARG;
  if (rq->n_req > MAASO_MAX_REQUESTS) return MAASO_E_SHAPE;
  if (!(prm->s_bar > 0.0f) || !std::isfinite(prm->s_bar)) return MAASO_E_INVALID_ARG;
  if (!(prm->pen_kappa >= 0.0f) || !std::isfinite(prm->pen_kappa)) return MAASO_E_INVALID_ARG;
  if (prm->tbt_mode > 1u || prm->policy > 1u) return MAASO_E_INVALID_ARG;
  return MAASO_OK;
}

ModelParams model_params(const maaso_ctx* ctx, const maaso_params* prm) {
  ModelParams mp;
  mp.s_bar = prm->s_bar;
  mp.pen_kappa = prm->pen_kappa;
  mp.tbt_mode = prm->tbt_mode;
  mp.n_tp = ctx->n_tp;
  mp.b_cap = ctx->b_cap;
  return mp;
}

template <int Q>
int launch_sweep(const SweepArgs& a, uint32_t blocks, hipStream_t s) {
  hipLaunchKernelGGL(sweep_kernel<Q>, dim3(blocks), dim3(kSweepThreads), 0, s, a);
  return hip_ok(hipGetLastError()) ? MAASO_OK : MAASO_E_HIP;
}

int score_assign_impl(maaso_ctx* ctx, const maaso_placements* pl, const uint32_t* cand_sel,
                      const maaso_requests* rq, const maaso_params* prm, const maaso_assign_out* out,
                      void* hip_stream);

int placement_sweep_impl(maaso_ctx* ctx, const maaso_placements* pl, const maaso_requests* rq,
                         const maaso_params* prm, uint32_t* sat_count, float* sat_ratio,
                         uint32_t* best_cand, void* hip_stream, bool static_scratch);

void fill_assign_args(AssignArgs& a, const maaso_ctx* ctx, const maaso_placements* pl,
                      const maaso_requests* rq, const maaso_params* prm,
                      const maaso_assign_out* out) {
  a.tab = ctx->tab;
  a.cells = ctx->cells;
  a.mp = model_params(ctx, prm);
  a.n_slo = ctx->n_slo;
  std::memcpy(a.d_ttft, ctx->d_ttft, sizeof(a.d_ttft));
  std::memcpy(a.d_tbt, ctx->d_tbt, sizeof(a.d_tbt));
  std::memcpy(a.i_ttft, ctx->i_ttft, sizeof(a.i_ttft));
  std::memcpy(a.i_tbt, ctx->i_tbt, sizeof(a.i_tbt));
  a.i_pad = pl->i_pad;
  a.n_cand = pl->n_cand;
  a.cand_sel = nullptr;
  a.n_inst = pl->n_inst;
  a.tp_idx = pl->tp_idx;
  a.max_batch = pl->max_batch;
  a.occ = pl->occ;
  a.q_ticks = reinterpret_cast<uint64_t*>(pl->q_ticks);
  a.n_req = rq->n_req;
  a.prompt_len = rq->prompt_len;
  a.out_len = rq->out_len;
  a.slo_class = rq->slo_class;
  a.arrival_ticks = rq->arrival_ticks;
  a.chosen = out->chosen;
  a.slack = out->slack;
  a.ttft = out->ttft;
  a.tbt = out->tbt;
  a.e2e = out->e2e;
  a.n_satisfied = reinterpret_cast<unsigned long long*>(out->n_satisfied);
  a.status = ctx->status;
  a.sat_acc = reinterpret_cast<unsigned long long*>(ctx->status + 36);
}

// One block per (request set, candidate); requests per lane chosen so that a window keeps the lanes
// busy (by the set with the longest windows: the choice never changes a result).
template <bool kScore, bool kSQ>
int launch_sweep_window_v(const SweepWindowArgs& a, size_t lds, hipStream_t s) {
  uint64_t per_window = 0;
  for (uint32_t k = 0; k < a.n_sets; ++k) {
    const uint64_t pw = a.sets[k].window < a.sets[k].n_req ? a.sets[k].window : a.sets[k].n_req;
    if (pw > per_window) per_window = pw;
  }
  const uint64_t blocks = (uint64_t)a.n_cand * a.n_sets;
  if (blocks == 0 || blocks > 0x7fffffffull) return MAASO_E_SHAPE;
  // Short windows go to the kernel that gives a wavefront to each (set, candidate) and its lanes to
  // the instances.  Measured crossover with the lanes-are-requests kernel (2048-8192 candidates): up to
  // 32 slots a window of 4 (6.2 against 7.6 ms; 8: 5.7 against 3.8), 128 slots 16 (6.6 against 9.4; 32:
  // 6.4 against 4.8), 256 slots 32 (7.7 against 8.9; 64: 7.6 against 4.5).
  const uint32_t short_window = a.i_pad / 8u > 4u ? a.i_pad / 8u : 4u;
  bool one_by_one = !kSQ;
  for (uint32_t k = 0; k < a.n_sets; ++k) one_by_one = one_by_one && a.sets[k].window <= short_window;
  if (one_by_one) {
    const dim3 g((uint32_t)((blocks + kSeqThreads / 64 - 1) / (kSeqThreads / 64)));
    bool one = true;  // every set request by request
    for (uint32_t k = 0; k < a.n_sets; ++k) one = one && a.sets[k].window == 1u;
    if (!kSQ) {
      const dim3 b(kSeqThreads);
      if (a.i_pad <= 64u) {
        if (one) hipLaunchKernelGGL((sweep_seq_kernel<kScore, 1, true>), g, b, lds, s, a);
        else hipLaunchKernelGGL((sweep_seq_kernel<kScore, 1>), g, b, lds, s, a);
      } else if (a.i_pad <= 128u) {
        if (one) hipLaunchKernelGGL((sweep_seq_kernel<kScore, 2, true>), g, b, lds, s, a);
        else hipLaunchKernelGGL((sweep_seq_kernel<kScore, 2>), g, b, lds, s, a);
      } else {
        if (one) hipLaunchKernelGGL((sweep_seq_kernel<kScore, 4, true>), g, b, lds, s, a);
        else hipLaunchKernelGGL((sweep_seq_kernel<kScore, 4>), g, b, lds, s, a);
      }
    }
    return hip_ok(hipGetLastError()) ? MAASO_OK : MAASO_E_HIP;
  }
  const dim3 grid((uint32_t)blocks);
  if (per_window > 2u * kAssignThreads)
    hipLaunchKernelGGL((sweep_window_kernel<kScore, 4, kSQ>), grid, dim3(kAssignThreads), lds, s, a);
  else if (per_window > kAssignThreads)
    hipLaunchKernelGGL((sweep_window_kernel<kScore, 2, kSQ>), grid, dim3(kAssignThreads), lds, s, a);
  else
    hipLaunchKernelGGL((sweep_window_kernel<kScore, 1, kSQ>), grid, dim3(kAssignThreads), lds, s, a);
  return hip_ok(hipGetLastError()) ? MAASO_OK : MAASO_E_HIP;
}

template <bool kScore>
int launch_sweep_window(const SweepWindowArgs& a, uint32_t policy, size_t lds, hipStream_t s) {
  return policy ? launch_sweep_window_v<kScore, true>(a, lds, s)
                : launch_sweep_window_v<kScore, false>(a, lds, s);
}

// Everything but the request sets.
void fill_sweep_window_args(SweepWindowArgs& a, const maaso_ctx* ctx, const maaso_placements* pl,
                            const maaso_params* prm) {
  a.tab = ctx->tab;
  a.cells = ctx->cells;
  a.mp = model_params(ctx, prm);
  a.n_slo = ctx->n_slo;
  std::memcpy(a.d_ttft, ctx->d_ttft, sizeof(a.d_ttft));
  std::memcpy(a.d_tbt, ctx->d_tbt, sizeof(a.d_tbt));
  std::memcpy(a.i_ttft, ctx->i_ttft, sizeof(a.i_ttft));
  std::memcpy(a.i_tbt, ctx->i_tbt, sizeof(a.i_tbt));
  a.n_cand = pl->n_cand;
  a.i_pad = pl->i_pad;
  a.n_inst = pl->n_inst;
  a.tp_idx = pl->tp_idx;
  a.max_batch = pl->max_batch;
  a.occ = pl->occ;
  a.q_ticks = reinterpret_cast<const uint64_t*>(pl->q_ticks);
  a.n_sets = 0;
  std::memset(a.sets, 0, sizeof(a.sets));
  a.status = ctx->status;
  a.alpha = a.beta = 0.0f;
  a.gamma_t = a.gamma_l = 1.0f;
}

// Appends a request set.  prm->window == 0 (static) = one window over everything: the state update is
// never reached.
void add_sweep_window_set(SweepWindowArgs& a, const maaso_requests* rq, const maaso_params* prm,
                          uint32_t* sat_count, const maaso_score_out* out) {
  SweepWindowSet& t = a.sets[a.n_sets++];
  t.n_req = rq->n_req;
  t.window = prm->window ? prm->window : (rq->n_req ? rq->n_req : 1u);
  t.prompt_len = rq->prompt_len;
  t.out_len = rq->out_len;
  t.slo_class = rq->slo_class;
  t.arrival_ticks = rq->arrival_ticks;
  t.sat_count = sat_count;
  t.phi_s = out ? out->phi_s : nullptr;
  t.phi_t = out ? out->phi_t : nullptr;
  t.phi_l = out ? out->phi_l : nullptr;
  t.score = out ? out->score : nullptr;
}

// Launch shape and workspace layout of the static sweep.
struct SweepPlan {
  uint32_t Q;         // requests per lane: a block owns 256*Q requests of one class
  uint32_t G;         // candidates per work item
  uint32_t n_items;   // ceil(C / G)
  uint32_t nrb_max;   // request-tile slots of the grid (>= tiles that exist)
  uint32_t blocks;    // 8 * nrb_max * blocks per (request tile, XCD) queue
  uint32_t static_blocks;  // of them resident at the kernel's start
  size_t lbuf_bytes, recs_bytes, queue_words;
  size_t bytes;       // class-bucketed prompt lengths | staged records | queue heads and pair counts
};

inline size_t up256(size_t x) { return (x + 255) & ~size_t(255); }

int plan_static_sweep(const maaso_ctx* ctx, uint32_t C, uint32_t I, uint32_t R, SweepPlan& p) {
  const uint32_t K = ctx->n_slo;
  uint32_t Q = ctx->sweep_q;
  // measured: 16 pays from 2^17 requests on (fewer trips to LDS per request; below that the lower
  // occupancy of its 102 registers costs more than it saves)
  if (Q == 0) Q = R >= (1u << 17) ? 16u : (R >= (1u << 14) ? 8u : (R >= (1u << 12) ? 4u : 2u));
  uint32_t G = (uint32_t)kGroupSlots / I;
  if (G > (uint32_t)kMaxGroup) G = kMaxGroup;
  // measured: items of about 256 instance slots (8 candidates of 32 slots a third full: 105 us against
  // 110 with 4 or 16; full slots: 4 and 8 equal; 128 slots: 1, 2 equal) balance the per-item
  // barrier against the tail of the dynamic queues
  uint32_t g_want = ctx->sweep_group ? ctx->sweep_group : (256u / I ? 256u / I : 1u);
  if (g_want < G) G = g_want;
  const uint32_t n_items = (C + G - 1) / G;
  const uint32_t tile = (uint32_t)kSweepThreads * Q;
  const uint32_t nrb_max = (uint32_t)(((uint64_t)R + tile - 1) / tile) + K;  // >= tiles that exist
  // Blocks: every (request tile, XCD) queue is served by bq persistent blocks.
  const uint32_t per_queue = (n_items + 7u) / 8u;
  uint32_t bq = ctx->sweep_blocks_per_queue;
  if (bq == 0) {
    // measured: about twice as many blocks as can be resident (8 per compute unit) - a block that
    // leaves makes room for one that has not started, so the compute units stay full while the
    // queues of small request tiles run dry
    bq = ((uint32_t)ctx->n_cu * 18u + 4u * nrb_max) / (8u * nrb_max);
    if (bq == 0) bq = 1;
  }
  if (bq > per_queue) bq = per_queue ? per_queue : 1u;
  const uint64_t blocks64 = (uint64_t)8 * nrb_max * bq;
  if (blocks64 > 0x7fffffffull) return MAASO_E_SHAPE;
  // the blocks the device holds at once start together: they take their first items without a trip
  // to the queue
  const int qi = Q == 2 ? 0 : (Q == 4 ? 1 : (Q == 8 ? 2 : 3));
  uint64_t resident = (uint64_t)ctx->n_cu * (uint64_t)ctx->sweep_resident[qi];
  if (resident > blocks64) resident = blocks64;
  p.static_blocks = (uint32_t)(resident & ~7ull);
  p.Q = Q;
  p.G = G;
  p.n_items = n_items;
  p.nrb_max = nrb_max;
  p.blocks = (uint32_t)blocks64;
  p.lbuf_bytes = up256((size_t)K * (R ? R : 1u) * sizeof(float));
  p.recs_bytes = up256((size_t)C * I * sizeof(float4));
  // queue heads, then two 8-byte evaluated-pairs words per sweep block
  p.queue_words = (size_t)nrb_max * 8u + 4u * (size_t)blocks64;
  p.bytes = p.lbuf_bytes + p.recs_bytes + up256(p.queue_words * sizeof(uint32_t));
  return MAASO_OK;
}

// Workspace that no call with at most C candidates of I slots and R requests exceeds, whatever launch
// shape it takes with the context's current knobs: the static sweep (its queue part bounded at two
// requests per lane, where the grid has the most request tiles), the windowed distributor's
// accumulators, the split's per-block counts.
size_t workspace_bound(const maaso_ctx* ctx, uint32_t C, uint32_t I, uint32_t R) {
  const uint64_t K = ctx->n_slo;
  const size_t lbuf = up256((size_t)K * (R ? R : 1u) * sizeof(float));
  const size_t recs = up256((size_t)C * I * sizeof(float4));
  const uint64_t nrb = ((uint64_t)R + 2u * kSweepThreads - 1) / (2u * kSweepThreads) + K;
  // blocks = 8 * nrb * bq with bq = floor((18 n_cu + 4 nrb) / (8 nrb)), at least 1
  const uint64_t blocks = ctx->sweep_blocks_per_queue ? 8u * nrb * ctx->sweep_blocks_per_queue
                                                      : (uint64_t)ctx->n_cu * 18u + 12u * nrb;
  const size_t queue = up256((size_t)(nrb * 8u + 4u * blocks) * sizeof(uint32_t));
  size_t need = lbuf + recs + queue;
  if (need < sizeof(WindowWs)) need = sizeof(WindowWs);
  const size_t split = (size_t)(((uint64_t)R + kSplitPerBlock - 1) / kSplitPerBlock + 1u) * sizeof(uint32_t);
  return need < split ? split : need;
}

// The three launches of the static sweep on workspace `ws` (at least plan.bytes, 256-byte aligned).
// Everything in the workspace that must start at zero is cleared by the first launch.
int launch_static_sweep(maaso_ctx* ctx, const maaso_placements* pl, const maaso_requests* rq,
                        const maaso_params* prm, const SweepPlan& plan, void* ws, uint32_t* sat_count,
                        float* sat_ratio, uint32_t* best_cand, hipStream_t s) {
  const uint32_t C = pl->n_cand, I = pl->i_pad, K = ctx->n_slo, R = rq->n_req;
  unsigned char* wsb = static_cast<unsigned char*>(ws);
  float* lbuf = reinterpret_cast<float*>(wsb);
  float4* recs = reinterpret_cast<float4*>(wsb + plan.lbuf_bytes);
  uint32_t* queues = reinterpret_cast<uint32_t*>(wsb + plan.lbuf_bytes + plan.recs_bytes);
  int rc = MAASO_OK;

  if (ctx->counters_dirty) {  // an earlier call failed between its launches
    hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(64), 0, s, ctx->cls_count, (uint32_t)kMaxSlo, 0u);
    if (!hip_ok(hipGetLastError())) return MAASO_E_HIP;
    ctx->counters_dirty = false;
  }
  ctx->counters_dirty = true;
  {
    PrepArgs p;
    p.prompt_len = rq->prompt_len;
    p.slo_class = rq->slo_class;
    p.n_req = R;
    p.n_slo = K;
    p.lbuf = lbuf;
    p.cls_count = ctx->cls_count;
    p.n_bucket_blocks = (uint32_t)(((uint64_t)R + kBucketPerBlock - 1) / kBucketPerBlock);
    p.tab = ctx->tab;
    p.cells = ctx->cells;
    p.mp = model_params(ctx, prm);
    p.n_cand = C;
    p.i_pad = I;
    p.n_inst = pl->n_inst;
    p.tp_idx = pl->tp_idx;
    p.max_batch = pl->max_batch;
    p.occ = pl->occ;
    p.q_ticks = reinterpret_cast<const uint64_t*>(pl->q_ticks);
    p.recs = recs;
    p.sat_count = sat_count;
    p.queues = queues;
    p.n_queues = (uint32_t)plan.queue_words;
    p.status = ctx->status;
    const uint64_t n_stage = ((uint64_t)C * I + kStageSlotsPerBlock - 1) / kStageSlotsPerBlock;
    const uint64_t n_prep = (uint64_t)p.n_bucket_blocks + n_stage;
    if (n_prep > 0x7fffffffull) return MAASO_E_SHAPE;
    size_t lds = (size_t)3 * ctx->cells * sizeof(float);
    if (lds < 2 * kMaxSlo * sizeof(uint32_t)) lds = 2 * kMaxSlo * sizeof(uint32_t);
    hipLaunchKernelGGL(sweep_prep_kernel, dim3((uint32_t)n_prep), dim3(256), lds, s, p);
    if (!hip_ok(hipGetLastError())) return MAASO_E_HIP;
  }
  if (R != 0) {
    SweepArgs a;
    a.n_slo = K;
    std::memcpy(a.d_ttft, ctx->d_ttft, sizeof(a.d_ttft));
    std::memcpy(a.d_tbt, ctx->d_tbt, sizeof(a.d_tbt));
    a.n_cand = C;
    a.i_pad = I;
    a.recs = recs;
    a.lbuf = lbuf;
    a.cls_count = ctx->cls_count;
    a.n_req = R;
    a.group = plan.G;
    a.n_items = plan.n_items;
    a.nrb_max = plan.nrb_max;
    a.queues = queues;
    a.static_blocks = plan.static_blocks;
    a.sat_count = sat_count;
    a.evaluated = reinterpret_cast<unsigned long long*>(queues + (size_t)plan.nrb_max * 8u);
    {
      TimedRegion timed(ctx, s);
      switch (plan.Q) {
        case 2: rc = launch_sweep<2>(a, plan.blocks, s); break;
        case 4: rc = launch_sweep<4>(a, plan.blocks, s); break;
        case 8: rc = launch_sweep<8>(a, plan.blocks, s); break;
        default: rc = launch_sweep<16>(a, plan.blocks, s); break;
      }
    }
    if (rc != MAASO_OK) return rc;
  }
  // evaluated-pairs total lands in the context's small device block, next to the class counters
  unsigned long long* eval_total = reinterpret_cast<unsigned long long*>(ctx->status + 32);
  hipLaunchKernelGGL(sweep_finalize_kernel, dim3(1), dim3(1024), 0, s, sat_count, C, R, sat_ratio,
                     best_cand, ctx->cls_count,
                     reinterpret_cast<const unsigned long long*>(queues + (size_t)plan.nrb_max * 8u),
                     R != 0 ? plan.blocks : 0u, eval_total);
  ctx->last_evaluated = eval_total;
  if (!hip_ok(hipGetLastError())) return MAASO_E_HIP;
  ctx->counters_dirty = false;
  return MAASO_OK;
}

bool score_weights_ok(const maaso_score_weights* wts) {
  return wts && std::isfinite(wts->alpha) && std::isfinite(wts->beta) && wts->gamma_t > 0.0f &&
         wts->gamma_l > 0.0f && std::isfinite(wts->gamma_t) && std::isfinite(wts->gamma_l);
}

// One request set of a scoring launch: where it comes from, where its results go, and - for a side
// of a split that only the device knows - the word holding the split position and which side.
struct ScoreSet {
  const maaso_requests* rq;
  const maaso_score_out* out;
  const uint32_t* split_at;
  uint32_t side;
};

int check_score_sets(const maaso_ctx* ctx, const maaso_placements* pl, uint32_t n_sets,
                     const ScoreSet* sets, const maaso_params* prm, const maaso_score_weights* wts) {
  for (uint32_t k = 0; k < n_sets; ++k) {
    const int rc = check_common(ctx, pl, sets[k].rq, prm);
    if (rc != MAASO_OK) return rc;
    if (!sets[k].out->sat_count || !sets[k].out->score) return MAASO_E_INVALID_ARG;
    if (prm->window != 0u && sets[k].rq->n_req != 0 && !sets[k].rq->arrival_ticks)
      return MAASO_E_INVALID_ARG;
  }
  return score_weights_ok(wts) ? MAASO_OK : MAASO_E_INVALID_ARG;
}

// Scores every candidate against every set in one launch (arguments checked, call guarded).
int launch_score_sets(maaso_ctx* ctx, const maaso_placements* pl, uint32_t n_sets,
                      const ScoreSet* sets, const maaso_params* prm, const maaso_score_weights* wts,
                      hipStream_t s) {
  SweepWindowArgs a;
  fill_sweep_window_args(a, ctx, pl, prm);
  // longest set first: its blocks run longest, so they should start first (a side of a device-side
  // split counts with the size of the whole, its upper bound)
  uint32_t order[MAASO_MAX_REQUEST_SETS];
  for (uint32_t k = 0; k < n_sets; ++k) order[k] = k;
  std::stable_sort(order, order + n_sets,
                   [&](uint32_t x, uint32_t y) { return sets[x].rq->n_req > sets[y].rq->n_req; });
  for (uint32_t k = 0; k < n_sets; ++k) {
    const ScoreSet& t = sets[order[k]];
    add_sweep_window_set(a, t.rq, prm, t.out->sat_count, t.out);
    a.sets[a.n_sets - 1].split_at = t.split_at;
    a.sets[a.n_sets - 1].side = t.side;
  }
  a.alpha = wts->alpha;
  a.beta = wts->beta;
  a.gamma_t = wts->gamma_t;
  a.gamma_l = wts->gamma_l;
  {
    TimedRegion timed(ctx, s);
    const int rc = launch_sweep_window<true>(a, prm->policy, (size_t)3 * ctx->cells * sizeof(float), s);
    if (rc != MAASO_OK) return rc;
  }
  for (uint32_t k = 0; k < n_sets; ++k)
    if (sets[k].out->best_cand) {
      hipLaunchKernelGGL(score_argmax_kernel, dim3(1), dim3(1024), 0, s, sets[k].out->score,
                         pl->n_cand, sets[k].out->best_cand);
      if (!hip_ok(hipGetLastError())) return MAASO_E_HIP;
    }
  return MAASO_OK;
}

int check_split(const maaso_ctx* ctx, const maaso_requests* rq, const uint32_t* prompt_len_out,
                const uint32_t* out_len_out, const uint8_t* slo_class_out,
                const uint32_t* arrival_ticks_out, const uint32_t* n_tight) {
  if (!ctx || !rq || !n_tight) return MAASO_E_INVALID_ARG;
  if (rq->n_req > MAASO_MAX_REQUESTS) return MAASO_E_SHAPE;
  if (rq->n_req != 0 && (!rq->prompt_len || !rq->out_len || !rq->slo_class || !prompt_len_out ||
                         !out_len_out || !slo_class_out))
    return MAASO_E_INVALID_ARG;
  if (rq->n_req != 0 && rq->arrival_ticks && !arrival_ticks_out) return MAASO_E_INVALID_ARG;
  const uint32_t n_blocks = (uint32_t)(((uint64_t)rq->n_req + kSplitPerBlock - 1) / kSplitPerBlock);
  return need_workspace(ctx, (size_t)(n_blocks ? n_blocks : 1u) * sizeof(uint32_t));
}

// Per-block counts, their scan, the scatter: three launches (arguments checked, call guarded).
int launch_split(maaso_ctx* ctx, const maaso_requests* rq, uint32_t tight_classes,
                 uint32_t* prompt_len_out, uint32_t* out_len_out, uint8_t* slo_class_out,
                 uint32_t* arrival_ticks_out, uint32_t* n_tight, hipStream_t s) {
  const uint32_t n_blocks = (uint32_t)(((uint64_t)rq->n_req + kSplitPerBlock - 1) / kSplitPerBlock);
  SplitArgs a;
  a.n_req = rq->n_req;
  a.prompt_len = rq->prompt_len;
  a.out_len = rq->out_len;
  a.slo_class = rq->slo_class;
  a.arrival_ticks = rq->arrival_ticks;
  a.tight_classes = tight_classes;
  a.n_slo = ctx->n_slo;
  a.block_tight = static_cast<uint32_t*>(ctx->ws);
  a.n_tight = n_tight;
  a.prompt_out = prompt_len_out;
  a.out_len_out = out_len_out;
  a.class_out = slo_class_out;
  a.arrival_out = arrival_ticks_out;
  a.status = ctx->status;
  if (n_blocks) hipLaunchKernelGGL(split_count_kernel, dim3(n_blocks), dim3(kPartitionThreads), 0, s, a);
  hipLaunchKernelGGL(split_scan_kernel, dim3(1), dim3(kPartitionThreads), 0, s, a.block_tight, n_blocks,
                     n_tight);
  if (n_blocks) hipLaunchKernelGGL(split_scatter_kernel, dim3(n_blocks), dim3(kPartitionThreads), 0, s, a);
  return hip_ok(hipGetLastError()) ? MAASO_OK : MAASO_E_HIP;
}

int check_select(const maaso_ctx* ctx, const maaso_placements* pl, const float* score, uint32_t n_gpus,
                 const float* phi_star, const int32_t* cand_star) {
  if (!ctx || !pl || !score || !phi_star || !cand_star) return MAASO_E_INVALID_ARG;
  if (pl->n_cand == 0 || !pl->n_inst || !pl->tp_idx) return MAASO_E_INVALID_ARG;
  if (!ctx->has_degree) return MAASO_E_INVALID_ARG;
  if (pl->i_pad == 0 || pl->i_pad > MAASO_MAX_INSTANCES || n_gpus > MAASO_MAX_GPUS) return MAASO_E_SHAPE;
  return MAASO_OK;
}

// Alg. 1's selection over n_lists score lists of the same deployments, one block each.
int launch_select(maaso_ctx* ctx, const maaso_placements* pl, uint32_t n_lists, const float* const* score,
                  const uint32_t* chain_offsets, uint32_t n_chains, uint32_t n_gpus,
                  float* const* phi_star, int32_t* const* cand_star, hipStream_t s) {
  SelectArgs a;
  a.n_lists = n_lists;
  for (uint32_t l = 0; l < (uint32_t)kMaxSelectLists; ++l) {
    a.score[l] = l < n_lists ? score[l] : nullptr;
    a.phi_star[l] = l < n_lists ? phi_star[l] : nullptr;
    a.cand_star[l] = l < n_lists ? cand_star[l] : nullptr;
  }
  a.n_cand = pl->n_cand;
  a.i_pad = pl->i_pad;
  a.n_inst = pl->n_inst;
  a.tp_idx = pl->tp_idx;
  a.tp_degree = reinterpret_cast<const uint32_t*>(ctx->tab + (size_t)3 * ctx->cells);
  a.n_tp = ctx->n_tp;
  a.chain_offsets = chain_offsets;
  a.n_chains = chain_offsets ? n_chains : 0u;
  a.n_gpus = n_gpus;
  a.status = ctx->status;
  hipLaunchKernelGGL(ins_deploy_select_kernel, dim3(n_lists), dim3(kPartitionThreads),
                     ((size_t)n_gpus + 1) * sizeof(unsigned long long), s, a);
  return hip_ok(hipGetLastError()) ? MAASO_OK : MAASO_E_HIP;
}

}  // namespace

extern "C" {

const char* maaso_strerror(int status) {
  switch (status) {
    case MAASO_OK: return "ok";
    case MAASO_E_INVALID_ARG: return "invalid argument";
    case MAASO_E_SHAPE: return "size beyond the library's limits";
    case MAASO_E_TABLE: return "profile table or deadline entry not finite and positive";
    case MAASO_E_HIP: return "HIP runtime error";
    case MAASO_E_NOMEM: return "out of memory";
    case MAASO_E_TIMEOUT: return "inter-window wait timed out on the device";
    case MAASO_E_WORKSPACE: return "workspace too small for this shape: call maaso_ctx_reserve first";
    case MAASO_E_BUSY: return "the context is in use by another call";
    case MAASO_E_RESIDENCY: return "the windowed distributor's blocks cannot all be resident on the device";
    default: return "unknown status";
  }
}

int maaso_profile_tables_load(const maaso_profile_desc* d, int device, maaso_ctx** out_ctx) {
  if (out_ctx) *out_ctx = nullptr;
  if (!d || !out_ctx || !d->prefill_a || !d->prefill_p || !d->tbt || !d->d_ttft || !d->d_tbt)
    return MAASO_E_INVALID_ARG;
  if (d->n_tp == 0 || d->b_cap == 0 || d->n_slo == 0) return MAASO_E_INVALID_ARG;
  if (d->n_slo > MAASO_MAX_SLO || d->b_cap > 65535u) return MAASO_E_SHAPE;
  const uint64_t cells64 = (uint64_t)d->n_tp * ((uint64_t)d->b_cap + 1u);
  if (cells64 > MAASO_MAX_TABLE_CELLS) return MAASO_E_SHAPE;
  const uint32_t cells = (uint32_t)cells64;
  for (uint32_t t = 0; t < d->n_tp; ++t)
    for (uint32_t b = 1; b <= d->b_cap; ++b) {
      const size_t i = (size_t)t * (d->b_cap + 1u) + b;
      const float v[3] = {d->prefill_a[i], d->prefill_p[i], d->tbt[i]};
      for (float x : v)
        if (!(x > 0.0f) || !std::isfinite(x)) return MAASO_E_TABLE;
    }
  for (uint32_t k = 0; k < d->n_slo; ++k) {
    const float v[2] = {d->d_ttft[k], d->d_tbt[k]};
    for (float x : v)
      if (!(x >= 0x1p-20f) || !(x <= 0x1p20f)) return MAASO_E_TABLE;
  }

  int n_dev = 0;
  if (!hip_ok(hipGetDeviceCount(&n_dev)) || device < 0 || device >= n_dev) return MAASO_E_HIP;
  DeviceGuard guard(device);
  if (!guard.ok) return MAASO_E_HIP;

  maaso_ctx* ctx = new (std::nothrow) maaso_ctx();  // value-initialised: every member starts at zero
  if (!ctx) return MAASO_E_NOMEM;
  ctx->device = device;
  ctx->n_tp = d->n_tp;
  ctx->b_cap = d->b_cap;
  ctx->cells = cells;
  ctx->n_slo = d->n_slo;
  ctx->spin_limit = 1u << 22;
  for (uint32_t k = 0; k < kMaxSlo; ++k) {
    const bool live = k < d->n_slo;
    ctx->d_ttft[k] = live ? d->d_ttft[k] : 1.0f;
    ctx->d_tbt[k] = live ? d->d_tbt[k] : 1.0f;
    // reciprocal of a deadline: evaluated in double, rounded once to binary32
    ctx->i_ttft[k] = (float)(1.0 / (double)ctx->d_ttft[k]);
    ctx->i_tbt[k] = (float)(1.0 / (double)ctx->d_tbt[k]);
  }
  hipDeviceProp_t prop;
  if (!hip_ok(hipGetDeviceProperties(&prop, device))) { delete ctx; return MAASO_E_HIP; }
  // address of this device's copy of the static scratch array (resolved once per device, with that
  // device current)
  if (device < kMaxDevices) {
    void* sp = g_scratch_ptr[device].load(std::memory_order_acquire);
    if (!sp) {
      if (!hip_ok(hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch))) || !sp) { delete ctx; return MAASO_E_HIP; }
      g_scratch_ptr[device].store(sp, std::memory_order_release);
    }
    ctx->scratch_ptr = sp;
  }
  ctx->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  ctx->lds_per_block = prop.sharedMemPerBlock;
  if (!hip_ok(hipDeviceGetAttribute(&ctx->cooperative, hipDeviceAttributeCooperativeLaunch, device)))
    ctx->cooperative = 0;
  {
    const void* fn[4] = {reinterpret_cast<const void*>(&sweep_kernel<2>), reinterpret_cast<const void*>(&sweep_kernel<4>),
                         reinterpret_cast<const void*>(&sweep_kernel<8>), reinterpret_cast<const void*>(&sweep_kernel<16>)};
    for (int i = 0; i < 4; ++i) {
      int n = 0;
      if (!hip_ok(hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, fn[i], kSweepThreads, 0)) || n < 1) n = 4;
      ctx->sweep_resident[i] = n;
    }
  }

  float* host = static_cast<float*>(std::malloc((size_t)3 * cells * sizeof(float)));
  if (!host) { delete ctx; return MAASO_E_NOMEM; }
  std::memcpy(host, d->prefill_a, (size_t)cells * 4);
  std::memcpy(host + cells, d->prefill_p, (size_t)cells * 4);
  std::memcpy(host + 2 * (size_t)cells, d->tbt, (size_t)cells * 4);
  int rc = MAASO_OK;
  if (!hip_ok(hipMalloc(reinterpret_cast<void**>(&ctx->tab), ((size_t)3 * cells + d->n_tp) * 4)))
    rc = MAASO_E_NOMEM;
  if (rc == MAASO_OK && !hip_ok(hipMalloc(reinterpret_cast<void**>(&ctx->status), kSmallBytes))) rc = MAASO_E_NOMEM;
  // the workspace is sized here, once: compute calls never allocate
  if (rc == MAASO_OK) rc = alloc_workspace(ctx, (size_t)MAASO_DEFAULT_WORKSPACE_BYTES);
  if (rc == MAASO_OK && !hip_ok(hipEventCreateWithFlags(&ctx->order_ev, hipEventDisableTiming))) rc = MAASO_E_HIP;
  if (rc == MAASO_OK) {
    // one small allocation, in 32-bit words: [0] status, [16..31] class counts, [32..35] evaluated
    // pairs of the last sweep (all; those without a wait), [36..37] admitted-count accumulator and
    // delivered-blocks ticket of the static distributor
    ctx->cls_count = ctx->status + 16;
    if (!hip_ok(hipMemcpy(ctx->tab, host, (size_t)3 * cells * 4, hipMemcpyHostToDevice)) ||
        !hip_ok(hipMemset(ctx->status, 0, kSmallBytes)))
      rc = MAASO_E_HIP;
    ctx->has_degree = d->tp_degree != nullptr;
    if (rc == MAASO_OK && ctx->has_degree &&
        !hip_ok(hipMemcpy(ctx->tab + (size_t)3 * cells, d->tp_degree, (size_t)d->n_tp * 4,
                          hipMemcpyHostToDevice)))
      rc = MAASO_E_HIP;
  }
  std::free(host);
  if (rc != MAASO_OK) {
    if (ctx->order_ev) (void)hipEventDestroy(ctx->order_ev);
    if (ctx->ws) (void)hipFree(ctx->ws);
    if (ctx->tab) (void)hipFree(ctx->tab);
    if (ctx->status) (void)hipFree(ctx->status);
    (void)hipGetLastError();
    delete ctx;
    return rc;
  }
  *out_ctx = ctx;
  return MAASO_OK;
}

void maaso_ctx_destroy(maaso_ctx* ctx) {
  if (!ctx) return;
  DeviceGuard guard(ctx->device);
  (void)hipDeviceSynchronize();
  for (uint32_t i = 0; i < kMaxTimed; ++i) {
    if (ctx->ev_start[i]) (void)hipEventDestroy(ctx->ev_start[i]);
    if (ctx->ev_stop[i]) (void)hipEventDestroy(ctx->ev_stop[i]);
  }
  if (ctx->order_ev) (void)hipEventDestroy(ctx->order_ev);
  if (ctx->ws) (void)hipFree(ctx->ws);
  if (ctx->tab) (void)hipFree(ctx->tab);
  if (ctx->status) (void)hipFree(ctx->status);
  (void)hipGetLastError();
  delete ctx;
}

int maaso_ctx_device_status(maaso_ctx* ctx, uint32_t* bits) {
  if (bits) *bits = 0;
  if (!ctx) return MAASO_E_INVALID_ARG;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return MAASO_E_HIP;
  uint32_t v = 0;
  if (!hip_ok(hipDeviceSynchronize())) return MAASO_E_HIP;
  if (!hip_ok(hipMemcpy(&v, ctx->status, 4, hipMemcpyDeviceToHost))) return MAASO_E_HIP;
  if (v != 0 && !hip_ok(hipMemset(ctx->status, 0, 4))) return MAASO_E_HIP;
  if (bits) *bits = v;
  if (v & MAASO_DEV_WAIT_TIMEOUT) return MAASO_E_TIMEOUT;
  return v ? MAASO_E_INVALID_ARG : MAASO_OK;
}

int maaso_ctx_set_launch_shape(maaso_ctx* ctx, uint32_t sweep_requests_per_lane,
                               uint32_t sweep_group, uint32_t sweep_blocks_per_queue,
                               uint32_t window_blocks) {
  if (!ctx) return MAASO_E_INVALID_ARG;
  const uint32_t q = sweep_requests_per_lane;
  if (q != 0 && q != 2 && q != 4 && q != 8 && q != 16) return MAASO_E_INVALID_ARG;
  ctx->sweep_q = q;
  ctx->sweep_group = sweep_group;
  ctx->sweep_blocks_per_queue = sweep_blocks_per_queue;
  ctx->window_blocks = window_blocks;
  return MAASO_OK;
}

int maaso_ctx_reserve(maaso_ctx* ctx, uint32_t max_cand, uint32_t i_pad, uint32_t max_req) {
  if (!ctx) return MAASO_E_INVALID_ARG;
  if (i_pad == 0 || i_pad > MAASO_MAX_INSTANCES || max_req > MAASO_MAX_REQUESTS) return MAASO_E_SHAPE;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return MAASO_E_HIP;
  int idle = 0;
  if (!ctx->in_call.compare_exchange_strong(idle, 1, std::memory_order_acquire)) return MAASO_E_BUSY;
  const int rc = alloc_workspace(ctx, workspace_bound(ctx, max_cand ? max_cand : 1u, i_pad, max_req));
  ctx->in_call.store(0, std::memory_order_release);
  return rc;
}

int maaso_ctx_workspace(maaso_ctx* ctx, uint64_t* bytes, uint32_t* allocations) {
  if (!ctx) return MAASO_E_INVALID_ARG;
  if (bytes) *bytes = ctx->ws_bytes;
  if (allocations) *allocations = ctx->ws_allocations;
  return MAASO_OK;
}

int maaso_placement_sweep(maaso_ctx* ctx, const maaso_placements* pl, const maaso_requests* rq,
                          const maaso_params* prm, uint32_t* sat_count, float* sat_ratio,
                          uint32_t* best_cand, void* hip_stream) {
  return placement_sweep_impl(ctx, pl, rq, prm, sat_count, sat_ratio, best_cand, hip_stream, false);
}

int maaso_placement_sweep_noalloc(maaso_ctx* ctx, const maaso_placements* pl, const maaso_requests* rq,
                                  const maaso_params* prm, uint32_t* sat_count, float* sat_ratio,
                                  uint32_t* best_cand, void* hip_stream) {
  return placement_sweep_impl(ctx, pl, rq, prm, sat_count, sat_ratio, best_cand, hip_stream, true);
}

}  // extern "C"

namespace {

// static_scratch: the static sweep works in the library's static device array instead of the
// context's workspace and refuses what does not fit; nothing is allocated on that path.
int placement_sweep_impl(maaso_ctx* ctx, const maaso_placements* pl, const maaso_requests* rq,
                         const maaso_params* prm, uint32_t* sat_count, float* sat_ratio,
                         uint32_t* best_cand, void* hip_stream, bool static_scratch) {
  int rc = check_common(ctx, pl, rq, prm);
  if (rc != MAASO_OK) return rc;
  if (!sat_count) return MAASO_E_INVALID_ARG;
  if (prm->window != 0u && rq->n_req != 0 && !rq->arrival_ticks) return MAASO_E_INVALID_ARG;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return MAASO_E_HIP;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  CallGuard call(ctx, s);
  if (call.rc != MAASO_OK) return call.rc;

  const uint32_t C = pl->n_cand, I = pl->i_pad, R = rq->n_req;

  if (prm->window != 0u && R != 0) {
    // Capacity-aware form: one block per candidate walks the request windows on its own state copy.
    SweepWindowArgs a;
    fill_sweep_window_args(a, ctx, pl, prm);
    add_sweep_window_set(a, rq, prm, sat_count, nullptr);
    {
      TimedRegion timed(ctx, s);
      rc = launch_sweep_window<false>(a, prm->policy, (size_t)3 * ctx->cells * sizeof(float), s);
      if (rc != MAASO_OK) return rc;
    }
    unsigned long long* eval_total = reinterpret_cast<unsigned long long*>(ctx->status + 32);
    hipLaunchKernelGGL(sweep_finalize_kernel, dim3(1), dim3(1024), 0, s, sat_count, C, R, sat_ratio,
                       best_cand, ctx->cls_count, static_cast<const unsigned long long*>(nullptr), 0u,
                       eval_total);
    if (!hip_ok(hipGetLastError())) return MAASO_E_HIP;
    ctx->last_evaluated = nullptr;
    return MAASO_OK;
  }

  SweepPlan plan;
  rc = plan_static_sweep(ctx, C, I, R, plan);
  if (rc != MAASO_OK) return rc;
  if (static_scratch) {
    if (!ctx->scratch_ptr) return MAASO_E_HIP;
    if (plan.bytes > (size_t)MAASO_NOALLOC_SCRATCH_BYTES) return MAASO_E_SHAPE;
    return launch_static_sweep(ctx, pl, rq, prm, plan, ctx->scratch_ptr, sat_count, sat_ratio,
                               best_cand, s);
  }
  rc = need_workspace(ctx, plan.bytes);
  if (rc != MAASO_OK) return rc;
  return launch_static_sweep(ctx, pl, rq, prm, plan, ctx->ws, sat_count, sat_ratio, best_cand, s);
}

}  // namespace

extern "C" {

int maaso_placement_score(maaso_ctx* ctx, const maaso_placements* pl, const maaso_requests* rq,
                          const maaso_params* prm, const maaso_score_weights* wts,
                          const maaso_score_out* out, void* hip_stream) {
  return maaso_placement_score_sets(ctx, pl, 1u, rq, prm, wts, out, hip_stream);
}

int maaso_placement_score_sets(maaso_ctx* ctx, const maaso_placements* pl, uint32_t n_sets,
                               const maaso_requests* rq, const maaso_params* prm,
                               const maaso_score_weights* wts, const maaso_score_out* out,
                               void* hip_stream) {
  if (!rq || !out || n_sets == 0u || n_sets > MAASO_MAX_REQUEST_SETS) return MAASO_E_INVALID_ARG;
  ScoreSet sets[MAASO_MAX_REQUEST_SETS];
  for (uint32_t k = 0; k < n_sets; ++k) sets[k] = ScoreSet{&rq[k], &out[k], nullptr, 0u};
  const int rc = check_score_sets(ctx, pl, n_sets, sets, prm, wts);
  if (rc != MAASO_OK) return rc;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return MAASO_E_HIP;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  CallGuard call(ctx, s);
  if (call.rc != MAASO_OK) return call.rc;
  return launch_score_sets(ctx, pl, n_sets, sets, prm, wts, s);
}

int maaso_profile_fit(int device, uint32_t n_tp, const uint32_t* offsets, const float* level,
                      const float* thr, uint32_t b_cap, float eps_lo, float eps_hi, double* params,
                      float* tbt) {
  if (!offsets || !level || !thr || !params || !tbt) return MAASO_E_INVALID_ARG;
  if (n_tp == 0 || b_cap == 0 || !(eps_lo > 0.0f) || !(eps_hi > eps_lo) || !std::isfinite(eps_hi))
    return MAASO_E_INVALID_ARG;
  if ((uint64_t)n_tp * ((uint64_t)b_cap + 1u) > MAASO_MAX_TABLE_CELLS) return MAASO_E_SHAPE;
  for (uint32_t t = 0; t < n_tp; ++t)
    if (offsets[t] > offsets[t + 1]) return MAASO_E_INVALID_ARG;
  const size_t n_samples = offsets[n_tp];
  for (size_t i = offsets[0]; i < n_samples; ++i)
    if (!(level[i] >= 1.0f) || !std::isfinite(level[i]) || !(thr[i] > 0.0f) || !std::isfinite(thr[i]))
      return MAASO_E_TABLE;
  int n_dev = 0;
  if (!hip_ok(hipGetDeviceCount(&n_dev)) || device < 0 || device >= n_dev) return MAASO_E_HIP;
  DeviceGuard guard(device);
  if (!guard.ok) return MAASO_E_HIP;
  // one device block: offsets | level | thr | params | tbt | flag
  const size_t cells = (size_t)n_tp * (b_cap + 1u);
  const size_t b_off = 0, b_par = (((size_t)n_tp + 1u) * 4u + 7u) & ~(size_t)7u;
  const size_t b_lvl = b_par + (size_t)n_tp * 4u * sizeof(double);
  const size_t b_thr = b_lvl + (n_samples ? n_samples : 1u) * 4u;
  const size_t b_tbt = b_thr + (n_samples ? n_samples : 1u) * 4u;
  const size_t b_bad = b_tbt + cells * 4u;
  unsigned char* dev = nullptr;
  if (!hip_ok(hipMalloc(reinterpret_cast<void**>(&dev), b_bad + 4u))) return MAASO_E_NOMEM;
  int rc = MAASO_OK;
  uint32_t bad = 0;
  if (!hip_ok(hipMemcpy(dev + b_off, offsets, ((size_t)n_tp + 1u) * 4u, hipMemcpyHostToDevice)) ||
      (n_samples && !hip_ok(hipMemcpy(dev + b_lvl, level, n_samples * 4u, hipMemcpyHostToDevice))) ||
      (n_samples && !hip_ok(hipMemcpy(dev + b_thr, thr, n_samples * 4u, hipMemcpyHostToDevice))) ||
      !hip_ok(hipMemset(dev + b_bad, 0, 4u)))
    rc = MAASO_E_HIP;
  if (rc == MAASO_OK) {
    FitArgs a;
    a.offsets = reinterpret_cast<const uint32_t*>(dev + b_off);
    a.level = reinterpret_cast<const float*>(dev + b_lvl);
    a.thr = reinterpret_cast<const float*>(dev + b_thr);
    a.b_cap = b_cap;
    a.log_eps_lo = std::log((double)eps_lo);
    a.log_eps_hi = std::log((double)eps_hi);
    a.params = reinterpret_cast<double*>(dev + b_par);
    a.tbt = reinterpret_cast<float*>(dev + b_tbt);
    a.bad = reinterpret_cast<uint32_t*>(dev + b_bad);
    hipLaunchKernelGGL(profile_fit_kernel, dim3(n_tp), dim3(kFitGrid), 0, nullptr, a);
    if (!hip_ok(hipGetLastError()) ||
        !hip_ok(hipMemcpy(params, dev + b_par, (size_t)n_tp * 4u * sizeof(double), hipMemcpyDeviceToHost)) ||
        !hip_ok(hipMemcpy(tbt, dev + b_tbt, cells * 4u, hipMemcpyDeviceToHost)) ||
        !hip_ok(hipMemcpy(&bad, dev + b_bad, 4u, hipMemcpyDeviceToHost)))
      rc = MAASO_E_HIP;
  }
  (void)hipFree(dev);
  if (rc == MAASO_OK && bad) rc = MAASO_E_TABLE;
  return rc;
}

int maaso_probe_valu(int device, uint32_t pattern, uint32_t trips, double* lane_ops_per_s,
                     uint32_t* instructions_per_trip) {
  static const uint32_t per_trip[5] = {24u, 40u, 96u, 16u, 8u};
  if (pattern > 4u || trips == 0u || !lane_ops_per_s) return MAASO_E_INVALID_ARG;
  int n_dev = 0;
  if (!hip_ok(hipGetDeviceCount(&n_dev)) || device < 0 || device >= n_dev) return MAASO_E_HIP;
  DeviceGuard guard(device);
  if (!guard.ok) return MAASO_E_HIP;
  hipDeviceProp_t prop;
  if (!hip_ok(hipGetDeviceProperties(&prop, device))) return MAASO_E_HIP;
  const uint32_t blocks = 8u * (uint32_t)(prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256);
  float* out = nullptr;
  if (!hip_ok(hipMalloc(reinterpret_cast<void**>(&out), (size_t)blocks * kProbeThreads * sizeof(float))))
    return MAASO_E_NOMEM;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  int rc = MAASO_OK;
  if (!hip_ok(hipEventCreate(&e0)) || !hip_ok(hipEventCreate(&e1))) rc = MAASO_E_HIP;
  float ms = 0.0f;
  for (int pass = 0; pass < 3 && rc == MAASO_OK; ++pass) {  // the first passes let the clock rise; the last is reported
    if (!hip_ok(hipEventRecord(e0, nullptr))) { rc = MAASO_E_HIP; break; }
    const dim3 g(blocks), b(kProbeThreads);
    switch (pattern) {
      case 0: hipLaunchKernelGGL(valu_probe_kernel<0>, g, b, 0, nullptr, out, trips, 1.0f); break;
      case 1: hipLaunchKernelGGL(valu_probe_kernel<1>, g, b, 0, nullptr, out, trips, 1.0f); break;
      case 2: hipLaunchKernelGGL(valu_probe_kernel<2>, g, b, 0, nullptr, out, trips, 1.0f); break;
      case 3: hipLaunchKernelGGL(valu_probe_kernel<3>, g, b, 0, nullptr, out, trips, 1.0f); break;
      default: hipLaunchKernelGGL(valu_probe_kernel<4>, g, b, 0, nullptr, out, trips, 1.0f); break;
    }
    if (!hip_ok(hipGetLastError()) || !hip_ok(hipEventRecord(e1, nullptr)) ||
        !hip_ok(hipEventSynchronize(e1)) || !hip_ok(hipEventElapsedTime(&ms, e0, e1)))
      rc = MAASO_E_HIP;
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  (void)hipFree(out);
  if (rc != MAASO_OK) return rc;
  if (instructions_per_trip) *instructions_per_trip = per_trip[pattern];
  *lane_ops_per_s = (double)blocks * kProbeThreads * (double)trips * per_trip[pattern] / ((double)ms * 1e-3);
  return MAASO_OK;
}

int maaso_split_by_slo(maaso_ctx* ctx, const maaso_requests* rq, uint32_t tight_classes,
                       uint32_t* prompt_len_out, uint32_t* out_len_out, uint8_t* slo_class_out,
                       uint32_t* arrival_ticks_out, uint32_t* n_tight, void* hip_stream) {
  int rc = check_split(ctx, rq, prompt_len_out, out_len_out, slo_class_out, arrival_ticks_out, n_tight);
  if (rc != MAASO_OK) return rc;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return MAASO_E_HIP;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  CallGuard call(ctx, s);
  if (call.rc != MAASO_OK) return call.rc;
  return launch_split(ctx, rq, tight_classes, prompt_len_out, out_len_out, slo_class_out,
                      arrival_ticks_out, n_tight, s);
}

int maaso_ins_deploy_select(maaso_ctx* ctx, const maaso_placements* pl, const float* score,
                            const uint32_t* chain_offsets, uint32_t n_chains, uint32_t n_gpus,
                            float* phi_star, int32_t* cand_star, void* hip_stream) {
  const int rc = check_select(ctx, pl, score, n_gpus, phi_star, cand_star);
  if (rc != MAASO_OK) return rc;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return MAASO_E_HIP;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  CallGuard call(ctx, s);
  if (call.rc != MAASO_OK) return call.rc;
  return launch_select(ctx, pl, 1u, &score, chain_offsets, n_chains, n_gpus, &phi_star, &cand_star, s);
}

int maaso_resource_partition(maaso_ctx* ctx, uint32_t n_gpus, const float* phi_t_star,
                             const float* phi_l_star, const float* phi_h_star,
                             const int32_t* cand_t_star, const int32_t* cand_l_star,
                             const int32_t* cand_h_star, uint64_t n_req_l, uint64_t n_req,
                             uint32_t* partition, float* phi_opt, void* hip_stream) {
  if (!ctx || !phi_t_star || !phi_l_star || !partition || !phi_opt) return MAASO_E_INVALID_ARG;
  if (n_req_l > n_req) return MAASO_E_INVALID_ARG;
  if (n_gpus > MAASO_MAX_GPUS) return MAASO_E_SHAPE;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return MAASO_E_HIP;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  CallGuard call(ctx, s);
  if (call.rc != MAASO_OK) return call.rc;
  PartitionArgs a;
  a.n_gpus = n_gpus;
  // initial share of the relaxed sub-cluster: floor(|R_l| / |R| * |G|), from the exact quotient
  a.g_l_cap = n_req == 0 ? 0u : (uint32_t)(((unsigned __int128)n_req_l * n_gpus) / n_req);
  a.n_tight = nullptr;
  a.n_req = 0u;
  a.phi_t_star = phi_t_star;
  a.phi_l_star = phi_l_star;
  a.phi_h_star = phi_h_star;
  a.cand_t_star = cand_t_star;
  a.cand_l_star = cand_l_star;
  a.cand_h_star = cand_h_star;
  a.out = partition;
  a.phi_opt = phi_opt;
  hipLaunchKernelGGL(resource_partition_kernel, dim3(1), dim3(kPartitionThreads), 0, s, a);
  return hip_ok(hipGetLastError()) ? MAASO_OK : MAASO_E_HIP;
}

int maaso_batch_size_prune(maaso_ctx* ctx, uint32_t n_cand, const uint32_t* group_offsets,
                           uint32_t n_groups, const uint32_t* sat_count, const float* latency,
                           uint8_t* keep, uint32_t* n_kept, void* hip_stream) {
  if (!ctx || !group_offsets || !n_kept) return MAASO_E_INVALID_ARG;
  if (n_cand != 0u && (!sat_count || !latency || !keep)) return MAASO_E_INVALID_ARG;
  if (n_groups > 0x7fffffffu) return MAASO_E_SHAPE;
  if (n_groups == 0u) return MAASO_OK;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return MAASO_E_HIP;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  CallGuard call(ctx, s);
  if (call.rc != MAASO_OK) return call.rc;
  PruneArgs a;
  a.n_cand = n_cand;
  a.group_offsets = group_offsets;
  a.n_groups = n_groups;
  a.sat_count = sat_count;
  a.latency = latency;
  a.keep = keep;
  a.n_kept = n_kept;
  a.status = ctx->status;
  hipLaunchKernelGGL(batch_prune_kernel, dim3(n_groups), dim3(kPruneTile), 0, s, a);
  return hip_ok(hipGetLastError()) ? MAASO_OK : MAASO_E_HIP;
}

int maaso_resource_partition_requests(maaso_ctx* ctx, const maaso_placements* pl,
                                      const uint32_t* chain_offsets, uint32_t n_chains,
                                      uint32_t n_gpus, const maaso_requests* rq,
                                      uint32_t tight_classes, const maaso_params* prm,
                                      const maaso_score_weights* wts,
                                      const maaso_partition_work* wk, void* hip_stream) {
  if (!wk || !rq) return MAASO_E_INVALID_ARG;
  if (!wk->score_t || !wk->score_l || !wk->sat_t || !wk->sat_l || !wk->phi_t_star ||
      !wk->phi_l_star || !wk->cand_t_star || !wk->cand_l_star || !wk->partition || !wk->phi_opt)
    return MAASO_E_INVALID_ARG;
  const bool homogeneous = wk->score_h != nullptr;
  if (homogeneous && (!wk->sat_h || !wk->phi_h_star || !wk->cand_h_star)) return MAASO_E_INVALID_ARG;
  int rc = check_split(ctx, rq, wk->prompt_len_split, wk->out_len_split, wk->slo_class_split,
                       wk->arrival_ticks_split, wk->n_tight);
  if (rc != MAASO_OK) return rc;
  // the split arrays as one request set of n_req requests; its two sides are cut on the device
  maaso_requests whole = *rq;
  whole.prompt_len = wk->prompt_len_split;
  whole.out_len = wk->out_len_split;
  whole.slo_class = wk->slo_class_split;
  whole.arrival_ticks = rq->arrival_ticks ? wk->arrival_ticks_split : nullptr;
  const maaso_score_out out_t = {wk->sat_t, nullptr, nullptr, nullptr, wk->score_t, nullptr};
  const maaso_score_out out_l = {wk->sat_l, nullptr, nullptr, nullptr, wk->score_l, nullptr};
  const maaso_score_out out_h = {wk->sat_h, nullptr, nullptr, nullptr, wk->score_h, nullptr};
  ScoreSet sets[3];
  uint32_t n_sets = 0;
  if (homogeneous) sets[n_sets++] = ScoreSet{rq, &out_h, nullptr, 0u};
  sets[n_sets++] = ScoreSet{&whole, &out_t, wk->n_tight, 1u};
  sets[n_sets++] = ScoreSet{&whole, &out_l, wk->n_tight, 2u};
  rc = check_score_sets(ctx, pl, n_sets, sets, prm, wts);
  if (rc != MAASO_OK) return rc;
  rc = check_select(ctx, pl, wk->score_t, n_gpus, wk->phi_t_star, wk->cand_t_star);
  if (rc != MAASO_OK) return rc;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return MAASO_E_HIP;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  CallGuard call(ctx, s);
  if (call.rc != MAASO_OK) return call.rc;
  rc = launch_split(ctx, rq, tight_classes, wk->prompt_len_split, wk->out_len_split,
                    wk->slo_class_split, wk->arrival_ticks_split, wk->n_tight, s);
  if (rc != MAASO_OK) return rc;
  rc = launch_score_sets(ctx, pl, n_sets, sets, prm, wts, s);
  if (rc != MAASO_OK) return rc;
  {
    const float* scores[3] = {wk->score_t, wk->score_l, wk->score_h};
    float* phis[3] = {wk->phi_t_star, wk->phi_l_star, wk->phi_h_star};
    int32_t* cands[3] = {wk->cand_t_star, wk->cand_l_star, wk->cand_h_star};
    rc = launch_select(ctx, pl, homogeneous ? 3u : 2u, scores, chain_offsets, n_chains, n_gpus, phis,
                       cands, s);
  }
  if (rc != MAASO_OK) return rc;
  PartitionArgs a;
  a.n_gpus = n_gpus;
  a.g_l_cap = 0u;
  a.n_tight = wk->n_tight;  // G'_l = floor(|R_l| * |G| / |R|) from the device's |R_t|
  a.n_req = rq->n_req;
  a.phi_t_star = wk->phi_t_star;
  a.phi_l_star = wk->phi_l_star;
  a.phi_h_star = homogeneous ? wk->phi_h_star : nullptr;
  a.cand_t_star = wk->cand_t_star;
  a.cand_l_star = wk->cand_l_star;
  a.cand_h_star = homogeneous ? wk->cand_h_star : nullptr;
  a.out = wk->partition;
  a.phi_opt = wk->phi_opt;
  hipLaunchKernelGGL(resource_partition_kernel, dim3(1), dim3(kPartitionThreads), 0, s, a);
  return hip_ok(hipGetLastError()) ? MAASO_OK : MAASO_E_HIP;
}

int maaso_score_assign(maaso_ctx* ctx, const maaso_placements* pl, const maaso_requests* rq,
                       const maaso_params* prm, const maaso_assign_out* out, void* hip_stream) {
  if (pl && pl->n_cand != 1u) return MAASO_E_INVALID_ARG;
  return score_assign_impl(ctx, pl, nullptr, rq, prm, out, hip_stream);
}

int maaso_score_assign_selected(maaso_ctx* ctx, const maaso_placements* pl, const uint32_t* cand,
                                const maaso_requests* rq, const maaso_params* prm,
                                const maaso_assign_out* out, void* hip_stream) {
  if (!cand) return MAASO_E_INVALID_ARG;
  return score_assign_impl(ctx, pl, cand, rq, prm, out, hip_stream);
}

}  // extern "C"

namespace {

int score_assign_impl(maaso_ctx* ctx, const maaso_placements* pl, const uint32_t* cand_sel,
                      const maaso_requests* rq, const maaso_params* prm, const maaso_assign_out* out,
                      void* hip_stream) {
  int rc = check_common(ctx, pl, rq, prm);
  if (rc != MAASO_OK) return rc;
  if (!out || (!out->chosen && !out->n_satisfied)) return MAASO_E_INVALID_ARG;
  const uint32_t R = rq->n_req;
  if (prm->window != 0u && R != 0 && !rq->arrival_ticks) return MAASO_E_INVALID_ARG;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return MAASO_E_HIP;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  CallGuard call(ctx, s);
  if (call.rc != MAASO_OK) return call.rc;

  AssignArgs a;
  fill_assign_args(a, ctx, pl, rq, prm, out);
  a.cand_sel = cand_sel;
  const bool lat = out->ttft || out->tbt || out->e2e;
  if (R == 0) {
    hipLaunchKernelGGL(assign_init_kernel, dim3(1), dim3(64), 0, s, a.n_satisfied);
    return hip_ok(hipGetLastError()) ? MAASO_OK : MAASO_E_HIP;
  }
  if (prm->window == 0u) {
    // 16-byte accesses, four requests per thread, when every array allows it
    auto al = [](const void* p, uintptr_t m) { return (reinterpret_cast<uintptr_t>(p) & m) == 0; };
    const bool vec = al(rq->prompt_len, 15) && al(rq->out_len, 15) && al(rq->slo_class, 3) &&
                     al(out->chosen, 15) && al(out->slack, 15) && al(out->ttft, 15) &&
                     al(out->tbt, 15) && al(out->e2e, 15);
    const uint32_t per_block = kAssignThreads * (vec ? 4u : 1u);
    uint32_t blocks = (uint32_t)(((uint64_t)R + per_block - 1) / per_block);
    // few instance slots: records live in registers and the loop needs no LDS (HBM-bound shape)
    const bool few = pl->i_pad <= 8u;
    // persistent blocks; measured on the HBM-bound shape: 3 per compute unit (all resident, 213 us)
    // beat 2 (228), 4 (219), 5 (254) and 8 (222)
    const uint32_t cap = (uint32_t)ctx->n_cu * (few ? 3u : 8u);
    if (blocks > cap) blocks = cap;
    TimedRegion timed(ctx, s);
#define MAASO_LAUNCH_STATIC(LAT, V, NREG)                                                          \
  do {                                                                                             \
    if (prm->policy)                                                                               \
      hipLaunchKernelGGL((assign_static_kernel<LAT, V, NREG, true>), dim3(blocks),                 \
                         dim3(kAssignThreads), 0, s, a);                                           \
    else                                                                                           \
      hipLaunchKernelGGL((assign_static_kernel<LAT, V, NREG, false>), dim3(blocks),                \
                         dim3(kAssignThreads), 0, s, a);                                           \
  } while (0)
    if (vec) {
      if (few) { if (lat) MAASO_LAUNCH_STATIC(true, 4, 8); else MAASO_LAUNCH_STATIC(false, 4, 8); }
      else     { if (lat) MAASO_LAUNCH_STATIC(true, 4, 0); else MAASO_LAUNCH_STATIC(false, 4, 0); }
    } else {
      if (few) { if (lat) MAASO_LAUNCH_STATIC(true, 1, 8); else MAASO_LAUNCH_STATIC(false, 1, 8); }
      else     { if (lat) MAASO_LAUNCH_STATIC(true, 1, 0); else MAASO_LAUNCH_STATIC(false, 1, 0); }
    }
#undef MAASO_LAUNCH_STATIC
    return hip_ok(hipGetLastError()) ? MAASO_OK : MAASO_E_HIP;
  }

  // Short windows (down to one request per window, the online distributor taken literally): one
  // wavefront with the instances in its lanes and no device-wide barrier.  Measured per request, one
  // wavefront against the persistent kernel: window 1: 0.88 against 2.72 us (64 slots), 1.72 against
  // 2.86 (256); window 4: 0.59 against 0.68 (64), 0.94 against 0.75 (256).  The window_blocks knob set
  // to a value asks for the persistent kernel below whatever the window.
  const uint32_t short_window = pl->i_pad <= 128u ? 4u : 2u;
  if (prm->policy == 0u && prm->window <= short_window && ctx->window_blocks == 0u) {
    const size_t lds = (size_t)3 * ctx->cells * sizeof(float);
    TimedRegion timed(ctx, s);
    if (pl->i_pad <= 64u) {
      if (lat) hipLaunchKernelGGL((assign_seq_kernel<true, 1>), dim3(1), dim3(64), lds, s, a, prm->window);
      else hipLaunchKernelGGL((assign_seq_kernel<false, 1>), dim3(1), dim3(64), lds, s, a, prm->window);
    } else if (pl->i_pad <= 128u) {
      if (lat) hipLaunchKernelGGL((assign_seq_kernel<true, 2>), dim3(1), dim3(64), lds, s, a, prm->window);
      else hipLaunchKernelGGL((assign_seq_kernel<false, 2>), dim3(1), dim3(64), lds, s, a, prm->window);
    } else {
      if (lat) hipLaunchKernelGGL((assign_seq_kernel<true, 4>), dim3(1), dim3(64), lds, s, a, prm->window);
      else hipLaunchKernelGGL((assign_seq_kernel<false, 4>), dim3(1), dim3(64), lds, s, a, prm->window);
    }
    return hip_ok(hipGetLastError()) ? MAASO_OK : MAASO_E_HIP;
  }

  // Windowed: one persistent kernel; all blocks must be resident at once (one per compute unit at
  // most).  Each request is spread over LPR lanes so that a window fills the blocks.
  rc = need_workspace(ctx, sizeof(WindowWs));
  if (rc != MAASO_OK) return rc;
  WindowWs* ws = static_cast<WindowWs*>(ctx->ws);
  const uint32_t per_window = prm->window < R ? prm->window : R;
  // More blocks shorten a window's scoring (more lanes per request, shorter instance walks) and
  // lengthen the window boundary, where every block adds to every instance's accumulators and the
  // owners of the instances read them until all blocks are counted in.  Measured per window
  // (16 / 32 / 64 / 128 blocks): 64 instances, windows of 4096: 3.63 / 3.15 / 3.81 / 5.77 us;
  // 256 instances, 4096: 7.2 / 5.4 / 5.7 / 7.6; 64 instances, 32768: 13.0 / 8.0 / 6.2 / 6.9;
  // 256 instances, 32768: 39.9 / 22.0 / 13.5 / 11.5.  Lanes per request are then chosen so that a
  // window is scored in one pass.
  const uint64_t window_triples = (uint64_t)per_window * pl->i_pad;
  uint32_t nb = ctx->window_blocks ? ctx->window_blocks
                                   : (window_triples < (1ull << 21) ? 32u : (window_triples < (1ull << 23) ? 64u : 128u));
  if (nb > (uint32_t)ctx->n_cu) nb = (uint32_t)ctx->n_cu;
  if (nb == 0) nb = 1;
  uint32_t lpr = 1;
  while (lpr < 64u && lpr * 2u <= pl->i_pad &&
         (uint64_t)per_window * (lpr * 2u) <= (uint64_t)nb * kWindowThreads)
    lpr *= 2u;
  const uint64_t need = ((uint64_t)per_window * lpr + kWindowThreads - 1) / kWindowThreads;
  if (need < nb) nb = (uint32_t)(need ? need : 1);
  hipLaunchKernelGGL(window_init_kernel, dim3(1), dim3(256), 0, s, ws, a.n_satisfied);
  if (!hip_ok(hipGetLastError())) return MAASO_E_HIP;
  uint32_t spin = ctx->spin_limit;
  uint32_t window_v = prm->window;
  const size_t wlds = (size_t)3 * ctx->cells * sizeof(float);  // profile tables in LDS
  TimedRegion timed(ctx, s);
  // The kernel's device-wide barrier needs every block resident at once.  A cooperative launch
  // guarantees that or is refused; where the device has none, the occupancy of the kernel decides on
  // the host (and the bounded spin remains the net under other work on the device).
  void* kargs[] = {&a, &window_v, &ws, &spin};
  hipError_t launched = hipSuccess;
  auto launch = [&](const void* fn) {
    if (ctx->cooperative) {
      launched = hipLaunchCooperativeKernel(fn, dim3(nb), dim3(kWindowThreads), kargs, (unsigned)wlds, s);
    } else {
      int per_cu = 0;
      launched = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kWindowThreads, wlds);
      if (launched == hipSuccess && (uint64_t)per_cu * (uint64_t)ctx->n_cu < nb)
        launched = hipErrorCooperativeLaunchTooLarge;
      if (launched == hipSuccess)
        launched = hipLaunchKernel(fn, dim3(nb), dim3(kWindowThreads), kargs, wlds, s);
    }
  };
  ctx->window_profiled = ctx->window_profile && !prm->policy && !lat;
#define MAASO_LAUNCH_WINDOW(LPR)                                                                  \
  do {                                                                                            \
    if (prm->policy) /* latency outputs are null-checked in the kernel: one variant serves both */ \
      launch(reinterpret_cast<const void*>(&assign_window_kernel<LPR, true, true>));               \
    else if (lat)                                                                                  \
      launch(reinterpret_cast<const void*>(&assign_window_kernel<LPR, true, false>));              \
    else if (ctx->window_profiled)                                                                 \
      launch(reinterpret_cast<const void*>(&assign_window_kernel<LPR, false, false, true>));       \
    else                                                                                           \
      launch(reinterpret_cast<const void*>(&assign_window_kernel<LPR, false, false>));             \
  } while (0)
  switch (lpr) {
    case 1: MAASO_LAUNCH_WINDOW(1); break;
    case 2: MAASO_LAUNCH_WINDOW(2); break;
    case 4: MAASO_LAUNCH_WINDOW(4); break;
    case 8: MAASO_LAUNCH_WINDOW(8); break;
    case 16: MAASO_LAUNCH_WINDOW(16); break;
    case 32: MAASO_LAUNCH_WINDOW(32); break;
    default: MAASO_LAUNCH_WINDOW(64); break;
  }
#undef MAASO_LAUNCH_WINDOW
  if (launched == hipErrorCooperativeLaunchTooLarge) {
    (void)hipGetLastError();
    return MAASO_E_RESIDENCY;
  }
  return hip_ok(launched) && hip_ok(hipGetLastError()) ? MAASO_OK : MAASO_E_HIP;
}

}  // namespace

extern "C" {

int maaso_ctx_kernel_timing(maaso_ctx* ctx, int enable) {
  if (!ctx) return MAASO_E_INVALID_ARG;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return MAASO_E_HIP;
  if (enable && !ctx->ev_start[0]) {
    for (uint32_t i = 0; i < kMaxTimed; ++i)
      if (!hip_ok(hipEventCreate(&ctx->ev_start[i])) || !hip_ok(hipEventCreate(&ctx->ev_stop[i])))
        return MAASO_E_HIP;
  }
  ctx->timing = enable != 0;
  ctx->n_timed = 0;
  return MAASO_OK;
}

int maaso_ctx_kernel_elapsed(maaso_ctx* ctx, float* total_ms, uint32_t* launches) {
  if (!ctx || !total_ms || !launches) return MAASO_E_INVALID_ARG;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return MAASO_E_HIP;
  float sum = 0.0f;
  for (uint32_t i = 0; i < ctx->n_timed; ++i) {
    float ms = 0.0f;
    if (!hip_ok(hipEventSynchronize(ctx->ev_stop[i])) ||
        !hip_ok(hipEventElapsedTime(&ms, ctx->ev_start[i], ctx->ev_stop[i])))
      return MAASO_E_HIP;
    sum += ms;
  }
  *total_ms = sum;
  *launches = ctx->n_timed;
  ctx->n_timed = 0;
  return MAASO_OK;
}

int maaso_ctx_kernel_durations(maaso_ctx* ctx, float* durations_ms, uint32_t cap, uint32_t* launches) {
  if (!ctx || !durations_ms || !launches) return MAASO_E_INVALID_ARG;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return MAASO_E_HIP;
  const uint32_t n = ctx->n_timed < cap ? ctx->n_timed : cap;
  for (uint32_t i = 0; i < n; ++i) {
    float ms = 0.0f;
    if (!hip_ok(hipEventSynchronize(ctx->ev_stop[i])) ||
        !hip_ok(hipEventElapsedTime(&ms, ctx->ev_start[i], ctx->ev_stop[i])))
      return MAASO_E_HIP;
    durations_ms[i] = ms;
  }
  *launches = n;
  ctx->n_timed = 0;
  return MAASO_OK;
}

int maaso_ctx_sweep_evaluated(maaso_ctx* ctx, uint64_t* pairs, uint64_t* pairs_without_wait) {
  if (!ctx || !pairs) return MAASO_E_INVALID_ARG;
  *pairs = 0;
  if (pairs_without_wait) *pairs_without_wait = 0;
  if (!ctx->last_evaluated) return MAASO_OK;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return MAASO_E_HIP;
  unsigned long long v[2] = {0, 0};
  if (!hip_ok(hipDeviceSynchronize())) return MAASO_E_HIP;
  if (!hip_ok(hipMemcpy(v, ctx->last_evaluated, sizeof(v), hipMemcpyDeviceToHost))) return MAASO_E_HIP;
  *pairs = v[0];
  if (pairs_without_wait) *pairs_without_wait = v[1];
  return MAASO_OK;
}

int maaso_ctx_window_profile(maaso_ctx* ctx, int enable) {
  if (!ctx) return MAASO_E_INVALID_ARG;
  ctx->window_profile = enable != 0;
  ctx->window_profiled = false;
  return MAASO_OK;
}

int maaso_ctx_window_phases(maaso_ctx* ctx, uint64_t cycles[6]) {
  if (!ctx || !cycles) return MAASO_E_INVALID_ARG;
  for (int i = 0; i < 6; ++i) cycles[i] = 0;
  if (!ctx->window_profiled) return MAASO_OK;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return MAASO_E_HIP;
  if (!hip_ok(hipDeviceSynchronize())) return MAASO_E_HIP;
  const WindowWs* ws = static_cast<const WindowWs*>(ctx->ws);
  unsigned long long v[6];
  if (!hip_ok(hipMemcpy(v, ws->phase, sizeof(v), hipMemcpyDeviceToHost))) return MAASO_E_HIP;
  for (int i = 0; i < 6; ++i) cycles[i] = v[i];
  return MAASO_OK;
}

int maaso_ctx_set_cooperative(maaso_ctx* ctx, int enable) {
  if (!ctx) return MAASO_E_INVALID_ARG;
  DeviceGuard guard(ctx->device);
  if (!guard.ok) return MAASO_E_HIP;
  int can = 0;
  if (enable && !hip_ok(hipDeviceGetAttribute(&can, hipDeviceAttributeCooperativeLaunch, ctx->device))) can = 0;
  ctx->cooperative = enable ? can : 0;
  return MAASO_OK;
}

int maaso_ctx_set_wait_limit(maaso_ctx* ctx, uint32_t polls) {
  if (!ctx) return MAASO_E_INVALID_ARG;
  ctx->spin_limit = polls;
  return MAASO_OK;
}

}  // extern "C"
