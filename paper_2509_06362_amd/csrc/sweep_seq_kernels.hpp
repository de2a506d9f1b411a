// Capacity-aware evaluation of candidate deployments with SHORT windows, down to one request per
// window - where every request meets the state left by all earlier ones, the paper's simulator taken
// literally (Sec. V-A: requests are mapped to slots one after the other and instance clocks advance
// in between).
//
// With a handful of requests per window the lanes of sweep_window_kernel (lanes = requests) are
// mostly idle and its block-wide barriers per window dominate.  Here a candidate belongs to ONE
// wavefront and the lanes are its INSTANCES (S slots per lane, instance j = s * 64 + lane): state,
// profile evaluation, triple, and the drain between two windows all stay in the lane's registers,
// the best instance of a request is a DPP arg-max over the wavefront, and nothing crosses a barrier.
// Requests are fetched 64 at a time (one per lane) and handed out lane by lane with v_readlane.
//
// The arithmetic is the windowed kernel's, operation by operation, so the two agree bit for bit and
// with the oracle's windowed distributor.  The shortest-queue rule is not offered here (its ranks
// need every instance's queue length); the windowed kernel serves it.
#pragma once

#include "sweep_window_kernels.hpp"
#include "window_kernels.hpp"

#pragma clang fp contract(off)

namespace maaso {

constexpr int kSeqThreads = 256;  // four wavefronts = four (request set, candidate) units per block

__device__ __forceinline__ float lane_value(float v, int l) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
}

// Arg-max of (slack, index) over the whole wavefront, lowest index among equals, as uniform values.
// The largest slack: four DPP steps settle each row of 16 lanes, two row broadcasts carry the rows'
// maxima into lane 63, one v_readlane fetches it.  The lowest index among the lanes that hold it:
// a lane's index is slot * 64 + lane (S slots per lane; -1 while it has seen nothing above -inf), so
// the lowest slot with a holder, and the first holder among its lanes, found on the scalar unit from
// one lane mask per slot - no trip through LDS and no per-lane compare chain on the per-request path.
template <int S>
__device__ __forceinline__ void argmax_wave(float s, int32_t i, uint32_t lane, float& ws, int32_t& wi) {
  float m = max_lanes<16>(s);
  MAASO_DPP_FOLD_ROWS("v_max_f32_dpp", m, "row_bcast:15", "0xa");
  MAASO_DPP_FOLD_ROWS("v_max_f32_dpp", m, "row_bcast:31", "0xc");
  ws = lane_value(m, 63);
  wi = -1;
#pragma unroll
  for (int sl = S - 1; sl >= 0; --sl) {
    const unsigned long long held = __ballot((s == ws) & (i == (int32_t)((uint32_t)sl * 64u + lane)));
    if (held != 0ull) wi = sl * 64 + (int32_t)__builtin_ctzll(held);
  }
}

// kOne: every set's window is one request (the window length is then a constant: the window loop and
// the per-window sums of admitted load fold away).
template <bool kScore, int S, bool kOne = false>
__global__ __launch_bounds__(kSeqThreads) void sweep_seq_kernel(const SweepWindowArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  float* tab = reinterpret_cast<float*>(smem);
  __shared__ ClassRow cls[kMaxSlo];

  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & 63u;
  if (tid < a.n_slo) cls[tid] = ClassRow{a.d_ttft[tid], a.d_tbt[tid], a.i_ttft[tid], a.i_tbt[tid]};
  for (uint32_t i = tid; i < 3u * a.cells; i += kSeqThreads) tab[i] = a.tab[i];
  __syncthreads();  // the only barrier: from here on a wavefront works alone

  // the wavefront's number within the block, as a scalar: what follows from it (the request set,
  // its pointers and size) then stays in scalar registers
  const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid >> 6));
  const uint64_t unit = (uint64_t)blockIdx.x * (kSeqThreads / 64) + wave;
  if (unit >= (uint64_t)a.n_sets * a.n_cand) return;
  const uint32_t set = (uint32_t)(unit / a.n_cand);
  const uint32_t c = (uint32_t)(unit - (uint64_t)set * a.n_cand);
  const SweepWindowSet rs = resolve_set(a.sets[set]);
  const size_t base = (size_t)c * a.i_pad;
  const uint32_t n = min(a.n_inst[c], a.i_pad);

  // instance state, S slots per lane
  uint32_t tp[S], B[S], served[S];
  int32_t occ[S];
  uint64_t q[S];
  float inv_tbt_first[S];
  bool valid[S];
#pragma unroll
  for (int s = 0; s < S; ++s) {
    const uint32_t j = (uint32_t)s * 64u + lane;
    valid[s] = j < n;
    tp[s] = 0; B[s] = 1; occ[s] = 0; q[s] = 0; served[s] = 0; inv_tbt_first[s] = 0.0f;
    if (valid[s]) {
      tp[s] = a.tp_idx[base + j]; B[s] = a.max_batch[base + j];
      occ[s] = a.occ[base + j]; q[s] = a.q_ticks[base + j];
    }
  }
  unsigned long long wait_sum = 0ull;  // queue waits of the requests this lane's instances admitted, ticks
  uint32_t sat = 0;                    // uniform
  bool bad_slot = false;               // a slot of this lane was outside the tables at some window

  const uint64_t R = rs.n_req;
  const uint64_t W = kOne ? 1ull : rs.window;
  // requests are fetched 64 at a time, one per lane, and handed out with v_readlane
  // what depends on the request alone (its deadlines, the reciprocal of the end-to-end one) is
  // worked out for the 64 requests of a batch at once, off the per-request chain
  uint64_t batch0 = ~0ull;  // first request of the batch held in the vectors below
  float Lv = 0.0f, Sv = 0.0f, Dtv = 1.0f, iDtv = 1.0f, Dbv = 1.0f, iDbv = 1.0f, Dev = 1.0f, iDev = 1.0f;
  uint32_t livev = 0;
  for (uint64_t s0 = 0; s0 < R; s0 += W) {
    const uint64_t e0 = (s0 + W < R) ? s0 + W : R;
    // stage this lane's instances against the state the window starts with
    float ra[S], rp[S], rt[S], rw[S], svc[S];
    unsigned long long wait_ticks[S];
    uint32_t n_add[S];
    unsigned long long t_add[S];
#pragma unroll
    for (int s = 0; s < S; ++s) {
      // every lane stages (an absent slot holds a harmless configuration) and the result is selected:
      // no divergent branch on the per-window chain
      n_add[s] = 0u; t_add[s] = 0ull;
      Staged st{1.0f, 1.0f, 1.0f, 1.0f, INFINITY};
      const bool ok = stage_instance(tab, a.cells, a.mp, tp[s], B[s], occ[s], q[s], st);
      const bool use = valid[s] & ok;
      bad_slot |= valid[s] & !ok;  // reported once, when the wavefront is done
      // an unused slot keeps whatever finite record came out (an absent slot holds a configuration
      // inside the tables, a rejected one the defaults above): its infinite wait alone keeps it from
      // ever being the best, and its occupancy of zero from ever draining
      ra[s] = st.a; rp[s] = st.p; rt[s] = st.tbt;
      rw[s] = use ? st.wait : INFINITY;
      svc[s] = st.svc;
      wait_ticks[s] = 0ull;
      if (kScore) {
        wait_ticks[s] = use ? (unsigned long long)__float2ll_rn(st.wait * 1048576.0f) : 0ull;
        if (s0 == 0u) inv_tbt_first[s] = use ? 1.0f / st.tbt : inv_tbt_first[s];
      }
    }
    for (uint64_t r = s0; r < e0; ++r) {
      if ((r & ~63ull) != batch0) {
        batch0 = r & ~63ull;
        const uint64_t mine = batch0 + lane;
        uint32_t pl = 0, ol = 0, kk = 0;
        if (mine < R) { pl = rs.prompt_len[mine]; ol = rs.out_len[mine]; kk = rs.slo_class[mine]; }
        livev = 1u;
        if (kk >= a.n_slo) { raise_status(a.status, 1u); livev = 0u; kk = 0; }
        Lv = (float)pl; Sv = (float)ol;
        const ClassRow cr = cls[kk];
        Dtv = cr.Dt; iDtv = cr.iDt; Dbv = cr.Db; iDbv = cr.iDb;
        Dev = fmaf(Sv, cr.Db, cr.Dt);
        iDev = 1.0f / Dev;
      }
      const int i = (int)(r & 63ull);
      const float L = lane_value(Lv, i), So = lane_value(Sv, i);
      const bool live = __builtin_amdgcn_readlane((int)livev, i) != 0;
      Deadlines d;
      d.Dt = lane_value(Dtv, i); d.iDt = lane_value(iDtv, i);
      d.Db = lane_value(Dbv, i); d.iDb = lane_value(iDbv, i);
      d.De = lane_value(Dev, i); d.iDe = lane_value(iDev, i);
      float best = -INFINITY, bpre = 0.0f;
      int32_t idx = -1;
#pragma unroll
      for (int s = 0; s < S; ++s) {  // an absent slot holds a record with an infinite wait: never the best
        const Margins m = score_triple(ra[s], rp[s], rt[s], rw[s], L, So, d);
        if (m.slack > best) { best = m.slack; idx = (int32_t)((uint32_t)s * 64u + lane); bpre = m.pre; }
      }
      if (!live) { best = -INFINITY; idx = -1; }
      float wbest;
      int32_t widx;
      argmax_wave<S>(best, idx, lane, wbest, widx);  // the wavefront's winner, uniform
      if (live && wbest >= 0.0f) {    // admitted: the chosen instance takes the load at the window's end
        sat += 1u;
#pragma unroll
        for (int s = 0; s < S; ++s)
          if (widx == (int32_t)((uint32_t)s * 64u + lane)) {
            n_add[s] += 1u;
            t_add[s] += (unsigned long long)__float2ll_rn(bpre * 1048576.0f);
          }
      }
    }
    // the window's load, then the time that passes until the next window opens
    uint32_t delta = 0;
    if (e0 < R) delta = rs.arrival_ticks[e0] - rs.arrival_ticks[s0];
#pragma unroll
    for (int s = 0; s < S; ++s) {  // an absent slot is empty and stays so
      if (kScore) {
        served[s] += n_add[s];
        wait_sum += (unsigned long long)n_add[s] * wait_ticks[s];
      }
      occ[s] += (int32_t)n_add[s];
      q[s] += t_add[s];
      if (e0 < R) {
        q[s] -= (q[s] < (uint64_t)delta) ? q[s] : (uint64_t)delta;
        const int32_t run = min(occ[s], (int32_t)B[s]);
        const float x = ((float)run * ((float)delta * 0x1p-20f)) / svc[s];
        const int32_t done = min(occ[s], (int32_t)floorf(fminf(x, 2147483520.0f)));
        occ[s] -= done;
      }
    }
  }

  if (bad_slot) raise_status(a.status, 2u);
  // results of this (set, candidate): lane 0 writes them
  if (kScore) wait_sum = wave_sum_u64(wait_sum);
  float pt = 0.0f;
  if (kScore) {
    // Phi_T: 1 / tbt of the serving instances, added in index order
#pragma unroll
    for (int s = 0; s < S; ++s) {
      const float inv = (valid[s] && served[s] != 0u) ? inv_tbt_first[s] : -1.0f;
      const uint32_t upto = n > (uint32_t)s * 64u ? min(n - (uint32_t)s * 64u, 64u) : 0u;
      for (uint32_t l = 0; l < upto; ++l) {
        const float v = lane_value(inv, (int)l);
        if (v >= 0.0f) pt = pt + v;
      }
    }
  }
  if (lane == 0u) {
    rs.sat_count[c] = sat;
    if (kScore) {
      const float ps = (rs.n_req == 0u) ? 0.0f : (float)sat / (float)rs.n_req;
      const float plat = (sat == 0u) ? 0.0f : ((float)wait_sum * 0x1p-20f) / (float)sat;
      const float ptn = fminf(pt, a.gamma_t) / a.gamma_t;
      const float pln = fmaxf(a.gamma_l - plat, 0.0f) / a.gamma_l;
      const float sc = fmaf(a.alpha, ps, fmaf(a.beta, ptn, (1.0f - a.beta) * pln));
      if (rs.phi_s) rs.phi_s[c] = ps;
      if (rs.phi_t) rs.phi_t[c] = pt;
      if (rs.phi_l) rs.phi_l[c] = plat;
      if (rs.score) rs.score[c] = sc;
    }
  }
}

// The distributor itself on short windows (one placement, requests in arrival order, down to one
// request per window - the online distributor of Sec. IV-F taken literally): the same wavefront
// scheme, plus the per-request outputs.  One wavefront does all the work - the method is sequential
// here - so this is about latency: no device-wide barrier per window.  The outputs of 64 requests are
// collected one lane each and stored together.
template <bool kLat, int S>
__global__ __launch_bounds__(64) void assign_seq_kernel(const AssignArgs a, uint32_t window) {
  extern __shared__ __align__(16) unsigned char smem[];
  float* tab = reinterpret_cast<float*>(smem);
  __shared__ ClassRow cls[kMaxSlo];
  const uint32_t lane = threadIdx.x;
  if (lane < a.n_slo) cls[lane] = ClassRow{a.d_ttft[lane], a.d_tbt[lane], a.i_ttft[lane], a.i_tbt[lane]};
  for (uint32_t i = lane; i < 3u * a.cells; i += 64u) tab[i] = a.tab[i];
  __syncthreads();

  const PlacementRow row = select_row(a);
  const uint32_t n = row.n;
  uint32_t tp[S], B[S];
  int32_t occ[S];
  uint64_t q[S];
  bool valid[S];
#pragma unroll
  for (int s = 0; s < S; ++s) {
    const uint32_t j = (uint32_t)s * 64u + lane;
    valid[s] = j < n;
    tp[s] = 0; B[s] = 1; occ[s] = 0; q[s] = 0;
    if (valid[s]) { tp[s] = row.tp_idx[j]; B[s] = row.max_batch[j]; occ[s] = row.occ[j]; q[s] = row.q_ticks[j]; }
  }
  unsigned long long sat = 0ull;  // uniform
  bool bad_slot = false;          // a slot of this lane was outside the tables at some window

  const uint64_t R = a.n_req;
  const uint64_t W = window;
  uint64_t batch0 = ~0ull;
  float Lv = 0.0f, Sv = 0.0f, Dtv = 1.0f, iDtv = 1.0f, Dbv = 1.0f, iDbv = 1.0f, Dev = 1.0f, iDev = 1.0f;
  uint32_t livev = 0;
  // outputs of the batch, request batch0 + lane in this lane
  int32_t o_idx = -1;
  float o_slack = -INFINITY, o_ttft = 0.0f, o_tbt = 0.0f, o_e2e = 0.0f;
  auto flush = [&]() {
    const uint64_t mine = batch0 + lane;
    if (batch0 == ~0ull || mine >= R) return;
    if (a.chosen) a.chosen[mine] = o_idx;
    if (a.slack) a.slack[mine] = o_slack;
    if (kLat) {
      if (a.ttft) a.ttft[mine] = o_ttft;
      if (a.tbt) a.tbt[mine] = o_tbt;
      if (a.e2e) a.e2e[mine] = o_e2e;
    }
  };
  for (uint64_t s0 = 0; s0 < R; s0 += W) {
    const uint64_t e0 = (s0 + W < R) ? s0 + W : R;
    float ra[S], rp[S], rt[S], rw[S], svc[S];
    uint32_t n_add[S];
    unsigned long long t_add[S];
#pragma unroll
    for (int s = 0; s < S; ++s) {  // every lane stages and the result is selected: no divergent branch
      n_add[s] = 0u; t_add[s] = 0ull;
      Staged st{1.0f, 1.0f, 1.0f, 1.0f, INFINITY};
      const bool ok = stage_instance(tab, a.cells, a.mp, tp[s], B[s], occ[s], q[s], st);
      const bool use = valid[s] & ok;
      bad_slot |= valid[s] & !ok;  // reported once, when the wavefront is done
      // an unused slot keeps whatever finite record came out (an absent slot holds a configuration
      // inside the tables, a rejected one the defaults above): its infinite wait alone keeps it from
      // ever being the best, and its occupancy of zero from ever draining
      ra[s] = st.a; rp[s] = st.p; rt[s] = st.tbt;
      rw[s] = use ? st.wait : INFINITY;
      svc[s] = st.svc;
    }
    for (uint64_t r = s0; r < e0; ++r) {
      if ((r & ~63ull) != batch0) {
        flush();
        batch0 = r & ~63ull;
        const uint64_t mine = batch0 + lane;
        uint32_t pl = 0, ol = 0, kk = 0;
        if (mine < R) { pl = a.prompt_len[mine]; ol = a.out_len[mine]; kk = a.slo_class[mine]; }
        livev = 1u;
        if (kk >= a.n_slo) { raise_status(a.status, 1u); livev = 0u; kk = 0; }
        Lv = (float)pl; Sv = (float)ol;
        const ClassRow cr = cls[kk];
        Dtv = cr.Dt; iDtv = cr.iDt; Dbv = cr.Db; iDbv = cr.iDb;
        Dev = fmaf(Sv, cr.Db, cr.Dt);
        iDev = 1.0f / Dev;
      }
      const int i = (int)(r & 63ull);
      const float L = lane_value(Lv, i), So = lane_value(Sv, i);
      const bool live = __builtin_amdgcn_readlane((int)livev, i) != 0;
      Deadlines d;
      d.Dt = lane_value(Dtv, i); d.iDt = lane_value(iDtv, i);
      d.Db = lane_value(Dbv, i); d.iDb = lane_value(iDbv, i);
      d.De = lane_value(Dev, i); d.iDe = lane_value(iDev, i);
      float best = -INFINITY, bpre = 0.0f, bttft = 0.0f, btbt = 0.0f, be2e = 0.0f;
      int32_t idx = -1;
#pragma unroll
      for (int s = 0; s < S; ++s) {  // an absent slot holds a record with an infinite wait: never the best
        const Margins m = score_triple(ra[s], rp[s], rt[s], rw[s], L, So, d);
        if (m.slack > best) {
          best = m.slack; idx = (int32_t)((uint32_t)s * 64u + lane); bpre = m.pre;
          bttft = m.ttft; btbt = rt[s]; be2e = m.e2e;
        }
      }
      if (!live) { best = -INFINITY; idx = -1; }
      float wbest;
      int32_t widx;
      argmax_wave<S>(best, idx, lane, wbest, widx);
      // what is reported about the chosen instance comes from the lane that holds it
      const float nanv = __builtin_nanf("");
      float w_ttft = nanv, w_tbt = nanv, w_e2e = nanv;
      if (widx >= 0) {
        const int owner = widx & 63;
        if (kLat) { w_ttft = lane_value(bttft, owner); w_tbt = lane_value(btbt, owner); w_e2e = lane_value(be2e, owner); }
        if (wbest >= 0.0f) {  // admitted: it loads the instance; a blocked request does not
          sat += 1ull;
#pragma unroll
          for (int s = 0; s < S; ++s)
            if (widx == (int32_t)((uint32_t)s * 64u + lane)) {
              n_add[s] += 1u;
              t_add[s] += (unsigned long long)__float2ll_rn(bpre * 1048576.0f);
            }
        }
      }
      if ((int)lane == i) { o_idx = widx; o_slack = wbest; o_ttft = w_ttft; o_tbt = w_tbt; o_e2e = w_e2e; }
    }
    uint32_t delta = 0;
    if (e0 < R) delta = a.arrival_ticks[e0] - a.arrival_ticks[s0];
#pragma unroll
    for (int s = 0; s < S; ++s) {  // an absent slot is empty and stays so
      occ[s] += (int32_t)n_add[s];
      q[s] += t_add[s];
      if (e0 < R) {  // time passes until the next window opens
        q[s] -= (q[s] < (uint64_t)delta) ? q[s] : (uint64_t)delta;
        const int32_t run = min(occ[s], (int32_t)B[s]);
        const float x = ((float)run * ((float)delta * 0x1p-20f)) / svc[s];
        const int32_t done = min(occ[s], (int32_t)floorf(fminf(x, 2147483520.0f)));
        occ[s] -= done;
      }
    }
  }
  flush();
  if (bad_slot) raise_status(a.status, 2u);
#pragma unroll
  for (int s = 0; s < S; ++s)
    if (valid[s]) { row.occ[(uint32_t)s * 64u + lane] = occ[s]; row.q_ticks[(uint32_t)s * 64u + lane] = q[s]; }
  if (lane == 0u && a.n_satisfied) *a.n_satisfied = sat;
}

}  // namespace maaso
