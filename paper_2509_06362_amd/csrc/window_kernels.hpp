// Distributor over an online request stream: requests are taken in windows; all requests of a window
// are scored in parallel against the instance state at the window's start, then the state advances
// (the simulator's clock-advance step, Sec. V-A "Simulator Implementation"; admission and blocking
// as in Sec. IV-F).  The window loop is sequential, so it lives inside ONE persistent kernel: no
// host round trip and no launch per window.
//
// Layout.  The work of a window is small (window x instances triples), so it is spread thin: each
// request is scored by LPR neighbouring lanes, each lane walking every LPR-th instance, followed by
// a cross-lane arg-max with lowest-index tie-break (DPP row operations inside a 16-lane row,
// ds_bpermute across rows).  Admitted load is summed with integer atomics - first in LDS per block,
// then once per block and instance into a small ring of global accumulators - so the sums do not
// depend on the order of arrival.  The accumulators count their own contributions: every block adds
// to every instance's words at every window (zero included), each addition carrying a one in the
// word's top bits, so the thread that owns instance j knows the sums are complete when the count
// equals the number of blocks.  That is the whole window boundary: one round of additions and one
// round of reads across the device, no separate arrival counter (bounded spin).  After it every
// block holds the same sums and advances its private copy of the state with the same integer /
// binary32 operations, so all copies stay identical.
#pragma once

#include "assign_kernels.hpp"
#include "lane_ops.hpp"

#pragma clang fp contract(off)

namespace maaso {

constexpr int kRing = 4;
constexpr int kWindowThreads = 1024;  // 16 wavefronts: four per SIMD hide the LDS latency of the instance loop

// Global scratch of the windowed kernel (zeroed by window_init_kernel before each call).
// Accumulator words: the low 40 bits hold a sum, the bits above how many blocks have added to it.
constexpr int kSumBits = 40;
constexpr unsigned long long kSumMask = (1ull << kSumBits) - 1ull;
constexpr unsigned long long kOneArrival = 1ull << kSumBits;

// Sleep between two looks at the accumulators, in units of 64 cycles (measured on config 2: 3 and 6
// are equal, 10 costs 0.5 %, 16 more than the second look gains).
constexpr int kLookGap = 6;

struct WindowWs {
  uint32_t abort_flag;                           // set when a wait gave up; every block then leaves
  uint32_t pad[3];
  // per instance, window w -> slot w % kRing: admitted requests (at most a window's 2^31), and the
  // admitted prefill ticks as the sums of the low and of the high 32-bit halves of the blocks'
  // 64-bit partial sums (each below 2^32 * 256 blocks = 2^40)
  unsigned long long ring_n[kRing][256];
  unsigned long long ring_tl[kRing][256];
  unsigned long long ring_th[kRing][256];
  // where block 0 spent its time, in shader clock cycles summed over the windows (written only by
  // the profiling variant of the kernel): stage, score, exchange, update; then the whole loop and
  // the number of windows
  unsigned long long phase[8];
};

__global__ void window_init_kernel(WindowWs* ws, unsigned long long* n_satisfied) {
  uint32_t* p = reinterpret_cast<uint32_t*>(ws);
  for (uint32_t i = threadIdx.x; i < sizeof(WindowWs) / 4u; i += blockDim.x) p[i] = 0u;
  if (threadIdx.x == 0 && n_satisfied) *n_satisfied = 0ull;
}

// kSQ: shortest-queue rule (see queue_rank_value); the rank values are rebuilt at every window from
// the queue lengths the window starts with.
// kProf: block 0 also sums the shader clock cycles it spends in each phase of a window into ws->phase.
template <int LPR, bool kLat, bool kSQ, bool kProf = false>
__global__ __launch_bounds__(kWindowThreads) void assign_window_kernel(const AssignArgs a,
                                                                       uint32_t window,
                                                                       WindowWs* ws,
                                                                       uint32_t spin_limit) {
  extern __shared__ __align__(16) unsigned char smem[];  // profile tables, read at every window's stage
  float* tab = reinterpret_cast<float*>(smem);
  __shared__ float4 recs[256];
  __shared__ ClassRow cls[kMaxSlo];
  __shared__ uint32_t n_blk[256];
  __shared__ unsigned long long t_blk[256];
  __shared__ uint32_t wave_sat[kWindowThreads / 64];
  __shared__ int32_t occ_s[kSQ ? 256 : 1];
  __shared__ float rankv[kSQ ? 256 : 1];
  __shared__ uint32_t gave_up_blk;  // a thread of this block gave up waiting at a window boundary

  const uint32_t tid = threadIdx.x;
  const PlacementRow row = select_row(a);
  const uint32_t n = row.n;
  // thread j owns instance j: configuration and live state stay in its registers
  uint32_t tp = 0, B = 1;
  int32_t occ = 0;
  uint64_t q = 0;
  if (tid < n) { tp = row.tp_idx[tid]; B = row.max_batch[tid]; occ = row.occ[tid]; q = row.q_ticks[tid]; }
  if (tid < a.n_slo) cls[tid] = ClassRow{a.d_ttft[tid], a.d_tbt[tid], a.i_ttft[tid], a.i_tbt[tid]};
  for (uint32_t i = tid; i < 3u * a.cells; i += kWindowThreads) tab[i] = a.tab[i];
  if (tid == 0u) gave_up_blk = 0u;
  __syncthreads();

  constexpr uint32_t kReqPerBlock = kWindowThreads / LPR;
  const uint32_t sl = tid % LPR;   // which slice of the instances this lane walks
  const uint32_t rq_in_blk = tid / LPR;
  const uint64_t R = a.n_req;
  const uint64_t n_windows = (R + window - 1) / window;
  uint32_t sat = 0;
  bool alive = true;

  // The request a lane scores first in a window is fetched one window ahead, and everything that
  // depends on the request alone - its class row, the end-to-end deadline and its reciprocal (a
  // division) - is worked out while the block waits for the other blocks at the window boundary, so
  // that neither the load nor that arithmetic follows the barrier.
  // The same goes for the arrival time that passes until the window after it opens (thread j needs
  // it when it advances instance j): fetched a window ahead, it is not waited for at a window's start.
  uint32_t pf_pl = 0, pf_ol = 0, pf_k = 0, pf_t0 = 0, pf_t1 = 0;
  auto prefetch = [&](uint64_t wn) {
    if (wn >= n_windows) return;
    const uint64_t s = wn * window;
    const uint64_t e = (s + window < R) ? s + window : R;
    const uint64_t r = s + (uint64_t)blockIdx.x * kReqPerBlock + rq_in_blk;
    if (r < e) { pf_pl = a.prompt_len[r]; pf_ol = a.out_len[r]; pf_k = a.slo_class[r]; }
    pf_t0 = 0u;
    pf_t1 = 0u;
    if (tid < n && e < R) { pf_t0 = a.arrival_ticks[s]; pf_t1 = a.arrival_ticks[e]; }
  };
  float pre_L = 0.0f, pre_S = 0.0f;
  Deadlines pre_d{};
  bool pre_ok = false;
  auto request_side = [&](uint32_t pl, uint32_t ol, uint32_t k, float& L, float& S, Deadlines& d) {
    L = (float)pl;
    S = (float)ol;
    if (k >= a.n_slo) return false;
    const ClassRow c = cls[k];
    d.Dt = c.Dt; d.Db = c.Db; d.iDt = c.iDt; d.iDb = c.iDb;
    d.De = fmaf(S, c.Db, c.Dt);
    d.iDe = 1.0f / d.De;
    return true;
  };
  prefetch(0);
  pre_ok = request_side(pf_pl, pf_ol, pf_k, pre_L, pre_S, pre_d);

  unsigned long long t_phase[4] = {0ull, 0ull, 0ull, 0ull};
  const long long t_loop = kProf ? clock64() : 0ll;

  for (uint64_t w = 0; w < n_windows; ++w) {
    const long long t0 = kProf ? clock64() : 0ll;
    const uint64_t s0 = w * window;
    const uint64_t e0 = (s0 + window < R) ? s0 + window : R;
    const uint32_t delta = pf_t1 - pf_t0;  // arrival time that passes until the next window opens
    float svc = 1.0f;
    if (tid < n) {
      Staged st;
      if (stage_instance(tab, a.cells, a.mp, tp, B, occ, q, st)) {
        recs[tid] = make_float4(st.a, st.p, st.tbt, st.wait);
        svc = st.svc;
      } else {
        raise_status(a.status, 2u);
        recs[tid] = make_float4(1.0f, 1.0f, 1.0f, INFINITY);
      }
      n_blk[tid] = 0u;
      t_blk[tid] = 0ull;
      if (kSQ) occ_s[tid] = occ;
    }
    __syncthreads();
    // A wait of the previous window's boundary gave up, here or (seen through the abort flag) in
    // another block: every block leaves before it scores anything of this window.  The verdict rides
    // on the barrier that publishes the staged records; the state advanced above from sums that
    // never arrived is not used and not written back.
    if (gave_up_blk != 0u) {
      alive = false;
      break;
    }
    if (kSQ) {
      if (tid < n) rankv[tid] = queue_rank_value(occ_s, n, tid);
      __syncthreads();
    }
    const long long t1 = kProf ? clock64() : 0ll;
    // what a triple competes with: its slack, or under the shortest-queue rule its instance's rank
    // value once the slack is non-negative
    auto value = [&](float slack, uint32_t j) { return (kSQ && slack >= 0.0f) ? rankv[j] : slack; };

    const uint64_t base0 = s0 + (uint64_t)blockIdx.x * kReqPerBlock;
    for (uint64_t base = base0; base < e0; base += (uint64_t)gridDim.x * kReqPerBlock) {
      const uint64_t r = base + rq_in_blk;
      const bool live = r < e0;
      const bool first = base == base0;
      float best = -INFINITY;
      int32_t idx = -1;
      float L = 0.0f, S = 0.0f;
      Deadlines d{};
      bool class_ok = false;
      if (live) {
        if (first) {
          L = pre_L; S = pre_S; d = pre_d; class_ok = pre_ok;
        } else {
          class_ok = request_side(a.prompt_len[r], a.out_len[r], a.slo_class[r], L, S, d);
        }
        if (class_ok) {
          uint32_t j = sl;
          for (; j + 3u * LPR < n; j += 4u * LPR) {  // four records per trip: one LDS wait for four reads
            const float4 r0 = recs[j], r1 = recs[j + LPR], r2 = recs[j + 2u * LPR], r3 = recs[j + 3u * LPR];
            const float s0 = value(score_triple(r0.x, r0.y, r0.z, r0.w, L, S, d).slack, j);
            const float s1 = value(score_triple(r1.x, r1.y, r1.z, r1.w, L, S, d).slack, j + LPR);
            const float s2 = value(score_triple(r2.x, r2.y, r2.z, r2.w, L, S, d).slack, j + 2u * LPR);
            const float s3 = value(score_triple(r3.x, r3.y, r3.z, r3.w, L, S, d).slack, j + 3u * LPR);
            if (s0 > best) { best = s0; idx = (int32_t)j; }
            if (s1 > best) { best = s1; idx = (int32_t)(j + LPR); }
            if (s2 > best) { best = s2; idx = (int32_t)(j + 2u * LPR); }
            if (s3 > best) { best = s3; idx = (int32_t)(j + 3u * LPR); }
          }
          for (; j < n; j += LPR) {
            const float4 rc = recs[j];
            const float sv = value(score_triple(rc.x, rc.y, rc.z, rc.w, L, S, d).slack, j);
            if (sv > best) { best = sv; idx = (int32_t)j; }
          }
        } else if (sl == 0) {
          raise_status(a.status, 1u);
        }
      }
      argmax_lanes<LPR>(best, idx);
      if (live && sl == 0) {
        float o_ttft = __builtin_nanf(""), o_tbt = o_ttft, o_e2e = o_ttft;
        float o_slack = best;
        if (idx >= 0) {
          const float4 rc = recs[idx];
          const Margins m = score_triple(rc.x, rc.y, rc.z, rc.w, L, S, d);
          o_ttft = m.ttft; o_tbt = rc.z; o_e2e = m.e2e;
          if (kSQ) o_slack = m.slack;  // `best` may be a rank value; report the instance's own slack
          if (best >= 0.0f) {  // admitted: it loads the instance; a blocked request does not
            ++sat;
            atomicAdd(&n_blk[idx], 1u);
            atomicAdd(&t_blk[idx], (unsigned long long)__float2ll_rn(m.pre * 1048576.0f));
          }
        }
        if (a.chosen) a.chosen[r] = idx;
        if (a.slack) a.slack[r] = o_slack;
        if (kLat) {
          if (a.ttft) a.ttft[r] = o_ttft;
          if (a.tbt) a.tbt[r] = o_tbt;
          if (a.e2e) a.e2e[r] = o_e2e;
        }
      }
    }
    prefetch(w + 1);
    lds_atomics_barrier();
    const long long t2 = kProf ? clock64() : 0ll;
    // Window boundary.  Thread j adds the block's sums for instance j, each with a one in the count
    // field, then reads the three words until all blocks are counted in.  Block 0 also recycles the
    // slot that window w + 2 will use: every block has read it (they all contributed to window w - 1
    // after doing so), and the stores complete before block 0's wait below ends (the wait's loads are
    // issued after them and the wait is for the thread's memory operations in full), hence before
    // block 0 contributes to window w + 1, without which nobody reaches window w + 2.
    unsigned long long sum_n = 0ull, sum_t = 0ull;
    bool gave_up = false;
    if (tid < n) {
      const uint32_t slot = (uint32_t)(w % kRing);
      const unsigned long long tb = t_blk[tid];
      atomicAdd(&ws->ring_n[slot][tid], kOneArrival | (unsigned long long)n_blk[tid]);
      atomicAdd(&ws->ring_tl[slot][tid], kOneArrival | (tb & 0xffffffffull));
      atomicAdd(&ws->ring_th[slot][tid], kOneArrival | (tb >> 32));
      if (blockIdx.x == 0) {
        const uint32_t recycle = (uint32_t)((w + 2) % kRing);
        __hip_atomic_store(&ws->ring_n[recycle][tid], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&ws->ring_tl[recycle][tid], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&ws->ring_th[recycle][tid], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    // the next window's request has been requested: what depends on it alone is done while the sums
    // of this window travel
    pre_ok = request_side(pf_pl, pf_ol, pf_k, pre_L, pre_S, pre_d);
    if (tid < n) {
      const uint32_t slot = (uint32_t)(w % kRing);
      const unsigned long long all_in = (unsigned long long)gridDim.x;
      uint32_t spins = 0;
      const unsigned long long* wn = &ws->ring_n[slot][tid];
      const unsigned long long* wl = &ws->ring_tl[slot][tid];
      const unsigned long long* wh = &ws->ring_th[slot][tid];
      auto look = [&](unsigned long long& v0, unsigned long long& v1, unsigned long long& v2) {
        v0 = __hip_atomic_load(wn, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        v1 = __hip_atomic_load(wl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        v2 = __hip_atomic_load(wh, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      };
      auto complete = [&](unsigned long long v0, unsigned long long v1, unsigned long long v2) {
        if ((v0 >> kSumBits) != all_in || (v1 >> kSumBits) != all_in || (v2 >> kSumBits) != all_in) return false;
        sum_n = v0 & kSumMask;
        sum_t = (v1 & kSumMask) + ((v2 & kSumMask) << 32);
        return true;
      };
      auto give_up_now = [&]() {
        if (spins < spin_limit &&
            __hip_atomic_load(&ws->abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u)
          return false;
        gave_up = true;
        __hip_atomic_store(&ws->abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        raise_status(a.status, 4u);
        return true;
      };
      // The first look also waits for everything this thread issued before it (vmcnt(0)).  After
      // that two looks are kept in flight, half a trip apart: how long a block takes to see the last
      // block's additions after they have landed is the time between two looks plus the way back.
      unsigned long long a0, a1, a2, b0, b1, b2;
      look(a0, a1, a2);
      __builtin_amdgcn_s_waitcnt(0x0f70);
      if (!complete(a0, a1, a2) && !(spins >= spin_limit && give_up_now())) {
        look(a0, a1, a2);
        for (;;) {
          __builtin_amdgcn_s_sleep(kLookGap);
          look(b0, b1, b2);
          if (complete(a0, a1, a2)) break;  // waits for the older look only
          ++spins;
          if ((spins & 15u) == 0u && give_up_now()) break;
          __builtin_amdgcn_s_sleep(kLookGap);
          look(a0, a1, a2);
          if (complete(b0, b1, b2)) break;
          ++spins;
          if (spins >= spin_limit && give_up_now()) break;
        }
      }
    }
    if (gave_up) gave_up_blk = 1u;
    const long long t3 = kProf ? clock64() : 0ll;

    if (tid < n) {
      occ += (int32_t)(uint32_t)sum_n;
      q += sum_t;
      if (e0 < R) {  // time passes until the next window opens
        q -= (q < (uint64_t)delta) ? q : (uint64_t)delta;
        const int32_t run = min(occ, (int32_t)B);
        const float x = ((float)run * ((float)delta * 0x1p-20f)) / svc;
        const int32_t done = min(occ, (int32_t)floorf(fminf(x, 2147483520.0f)));
        occ -= done;
      }
    }
    if (kProf) {
      const long long t4 = clock64();
      t_phase[0] += (unsigned long long)(t1 - t0);
      t_phase[1] += (unsigned long long)(t2 - t1);
      t_phase[2] += (unsigned long long)(t3 - t2);
      t_phase[3] += (unsigned long long)(t4 - t3);
    }
  }
  __syncthreads();  // the last boundary's verdict
  if (gave_up_blk != 0u) alive = false;
  if (kProf && blockIdx.x == 0 && tid == 0) {
    for (int i = 0; i < 4; ++i) ws->phase[i] = t_phase[i];
    ws->phase[4] = (unsigned long long)(clock64() - t_loop);
    ws->phase[5] = n_windows;
  }

  if (alive && blockIdx.x == 0 && tid < n) { row.occ[tid] = occ; row.q_ticks[tid] = q; }
  for (int dlt = 32; dlt >= 1; dlt >>= 1) sat += __shfl_xor(sat, dlt);
  if ((tid & 63u) == 0u) wave_sat[tid >> 6] = sat;
  __syncthreads();
  if (tid == 0 && a.n_satisfied) {
    uint32_t t = 0;
    for (int wv = 0; wv < kWindowThreads / 64; ++wv) t += wave_sat[wv];
    if (t) atomicAdd(a.n_satisfied, (unsigned long long)t);
    // a call that gave up marks its count as incomplete: the top bit survives every addition
    if (!alive) atomicOr(a.n_satisfied, 1ull << 63);
  }
}

}  // namespace maaso
