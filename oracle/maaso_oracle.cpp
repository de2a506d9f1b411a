// CPU oracle for the MaaSO scoring path.  TEST INFRASTRUCTURE ONLY.
//
// A plain, single-threaded, obviously-correct statement of what the scoring path computes, written
// from the paper's definitions.  It exists so that the GPU library can be checked against it; it is
// never part of the product path, shares no code with the HIP sources, and is linked only by the
// tests, the smoke check and the benchmark's CPU-baseline leg.
//
// Build: g++ -O2 -std=c++17 -ffp-contract=off -fno-fast-math -shared -fPIC (no contraction: every
// float operation below is one IEEE-754 binary32 operation, rounded to nearest even; fmaf is the
// only fused one).
//
// What is modelled, and where the paper defines it:
//   * An instance i has a parallelism strategy P_i, an inference batch size B_i and a live workload
//     level W_i.  Its decode speed follows the throughput-decay function F(M,P,B,W), which depends on
//     min(B, W): the decay is truncated once the workload reaches the batch size (Sec. IV-B, Eq. 1).
//     Profiles arrive already tabulated per (strategy, effective batch): seconds per output token
//     (= 1/F), and a linear prefill cost a + p * prompt_len.
//   * A request's latency is queuing latency plus decoding latency, L_r = L_q + L_d (Sec. IV-C,
//     Eq. 2).  Queuing occurs when W_i exceeds B_i; its per-instance size is W_i * E[L_d] / B_i
//     (Eq. 5), here applied to the requests beyond the batch cap, plus prefill work already queued
//     (the pending time p_r that shifts an instance's performance boundary, Sec. III-C).
//   * A request is served iff latency <= deadline, with equality counting as served (Eq. 3); the
//     distributor blocks a request only when latency > deadline on every instance (Sec. IV-F step 3)
//     and one request goes to at most one instance (constraint (b)).
//   * A deployment's SLO score is the satisfied fraction of its requests (Sec. IV-D, "SLO satisfaction
//     ratio"); the placer keeps the best-scoring deployment (Alg. 1).
//   * Requests carry three deadlines: first token (TTFT), between tokens (TBT) and end to end, the
//     last being TTFT deadline + out_len * TBT deadline.  Slack is the smallest of the three relative
//     margins; the chosen instance maximises slack, lowest index on ties.
//   * Between windows of an online request stream the instances' workload level and queued prefill
//     time are advanced from the assignments (the simulator's "advance instance clocks" step,
//     Sec. V-A "Simulator Implementation"): admitted requests add load, the prefill queue drains in
//     real time, and running requests complete at the fluid rate min(W,B) / (E[S] * tbt).
//
// Pins (tests/test_oracle_*.py): brute-force enumeration of assignments and of placements, closed
// forms in double for single-instance cases, printed values of the synthetic profile, an independent
// prompt-length-threshold count (oracle_threshold_sweep below, a different algorithm for the same
// counts), monotonicity and permutation invariants, equality-at-deadline.  Parity unpinned: absolute
// SLO-attainment figures of the paper (its traces and profiles are not public).

#include <cmath>
#include <cstdint>
#include <cstring>
#include <algorithm>
#include <limits>
#include <vector>

namespace {

struct Profile {
  uint32_t n_tp, b_cap;
  const float* prefill_a;  // [n_tp][b_cap+1]
  const float* prefill_p;
  const float* tbt;
  uint32_t n_slo;
  const float* d_ttft;  // [n_slo]
  const float* d_tbt;
};

struct Staged {  // one instance, after profile evaluation
  float a, p, tbt, svc, wait;
};

// Reciprocal of a deadline: computed in double, rounded once to float.
inline float recip_deadline(float d) { return (float)(1.0 / (double)d); }

// Profile evaluation for one instance: effective batch, table row, occupancy penalty, queue wait.
Staged stage_instance(const Profile& pf, uint32_t tp_idx, uint32_t B, int32_t occ, uint64_t q_ticks,
                      float s_bar, float pen_kappa, uint32_t tbt_mode) {
  Staged s;
  // Eq. 1: the arriving request joins the batch, so the workload level is occ + 1, capped at B.
  int64_t w = (tbt_mode == 1) ? (int64_t)B : std::min<int64_t>((int64_t)occ + 1, (int64_t)B);
  size_t row = (size_t)tp_idx * (pf.b_cap + 1) + (size_t)w;
  s.a = pf.prefill_a[row];
  s.p = pf.prefill_p[row];
  float tb = pf.tbt[row];
  float invB = 1.0f / (float)B;
  int64_t over = std::max<int64_t>(4 * w - 3 * (int64_t)B, 0);  // > 0 iff fill above 75 %
  float pen = fmaf(pen_kappa, (float)over * invB, 1.0f);
  s.tbt = tb * pen;
  s.svc = s_bar * s.tbt;  // expected decode latency E[L_d] on this instance
  int64_t ov = std::max<int64_t>((int64_t)occ + 1 - (int64_t)B, 0);  // requests beyond the cap
  float slot = ((float)ov * invB) * s.svc;  // W * E[L_d] / B form of Eq. 5
  s.wait = (float)q_ticks * 0x1p-20f + slot;
  return s;
}

struct Triple {
  float pre, ttft, e2e, s1, s2, s3, slack;
};

// One (request, instance) evaluation: latency (Eq. 2) and the three relative margins (Eq. 3).
inline Triple score_triple(const Staged& in, float L, float S, float Dt, float Db, float De,
                           float iDt, float iDb, float iDe) {
  Triple t;
  t.pre = fmaf(in.p, L, in.a);
  t.ttft = in.wait + t.pre;
  t.e2e = fmaf(S, in.tbt, t.ttft);
  t.s1 = (Dt - t.ttft) * iDt;
  t.s2 = (Db - in.tbt) * iDb;
  t.s3 = (De - t.e2e) * iDe;
  t.slack = fminf(fminf(t.s1, t.s2), t.s3);
  return t;
}

bool profile_ok(const Profile& pf) {
  if (pf.n_tp == 0 || pf.b_cap == 0 || pf.n_slo == 0) return false;
  for (uint32_t t = 0; t < pf.n_tp; ++t)
    for (uint32_t b = 1; b <= pf.b_cap; ++b) {
      size_t i = (size_t)t * (pf.b_cap + 1) + b;
      const float v[3] = {pf.prefill_a[i], pf.prefill_p[i], pf.tbt[i]};
      for (float x : v)
        if (!(x > 0.0f) || !std::isfinite(x)) return false;
    }
  for (uint32_t k = 0; k < pf.n_slo; ++k) {
    if (!(pf.d_ttft[k] > 0.0f) || !std::isfinite(pf.d_ttft[k])) return false;
    if (!(pf.d_tbt[k] > 0.0f) || !std::isfinite(pf.d_tbt[k])) return false;
  }
  return true;
}

}  // namespace

extern "C" {

// Stage n instances; every output array has n entries.  Returns 0, or -1 on a bad profile.
int oracle_stage(uint32_t n_tp, uint32_t b_cap, const float* prefill_a, const float* prefill_p,
                 const float* tbt, uint32_t n, const uint8_t* tp_idx, const uint16_t* max_batch,
                 const int32_t* occ, const uint64_t* q_ticks, float s_bar, float pen_kappa,
                 uint32_t tbt_mode, float* out_a, float* out_p, float* out_tbt, float* out_svc,
                 float* out_wait) {
  Profile pf{n_tp, b_cap, prefill_a, prefill_p, tbt, 1, nullptr, nullptr};
  for (uint32_t j = 0; j < n; ++j) {
    Staged s = stage_instance(pf, tp_idx[j], max_batch[j], occ[j], q_ticks[j], s_bar, pen_kappa,
                              tbt_mode);
    out_a[j] = s.a; out_p[j] = s.p; out_tbt[j] = s.tbt; out_svc[j] = s.svc; out_wait[j] = s.wait;
  }
  return 0;
}

// One triple from already-staged instance values.  out[7] = pre, ttft, e2e, s1, s2, s3, slack.
void oracle_triple(float a, float p, float tbt_j, float wait, uint32_t prompt_len, uint32_t out_len,
                   float d_ttft, float d_tbt, float* out) {
  Staged in{a, p, tbt_j, 0.0f, wait};
  float L = (float)prompt_len, S = (float)out_len;
  float De = fmaf(S, d_tbt, d_ttft);
  Triple t = score_triple(in, L, S, d_ttft, d_tbt, De, recip_deadline(d_ttft),
                          recip_deadline(d_tbt), 1.0f / De);
  out[0] = t.pre; out[1] = t.ttft; out[2] = t.e2e; out[3] = t.s1; out[4] = t.s2; out[5] = t.s3;
  out[6] = t.slack;
}

}  // extern "C"

namespace {

// What the serving score needs to know about a run of the distributor, beyond the admitted count.
struct RunStats {
  std::vector<uint64_t> admitted_per_inst;  // requests admitted to each instance, all windows
  std::vector<float> tbt_first;             // per-token latency of each instance in the first window
  uint64_t wait_ticks = 0;                  // sum over admitted requests of their instance's queue
                                            // wait at admission, in ticks of 2^-20 s (lrintf)
};

// The distributor proper; see oracle_score_assign for the contract.  `stats` may be null.
int distributor(uint32_t n_tp, uint32_t b_cap, const float* prefill_a, const float* prefill_p,
                const float* tbt, uint32_t n_slo, const float* d_ttft, const float* d_tbt,
                uint32_t n_inst, const uint8_t* tp_idx, const uint16_t* max_batch, int32_t* occ,
                uint64_t* q_ticks, uint32_t n_req, const uint32_t* prompt_len,
                const uint32_t* out_len, const uint8_t* slo_class, const uint32_t* arrival_ticks,
                float s_bar, float pen_kappa, uint32_t tbt_mode, uint32_t window, uint32_t policy,
                int32_t* chosen,
                float* slack, float* lat_ttft, float* lat_tbt, float* lat_e2e, uint64_t* n_satisfied,
                RunStats* stats) {
  Profile pf{n_tp, b_cap, prefill_a, prefill_p, tbt, n_slo, d_ttft, d_tbt};
  if (!profile_ok(pf) || policy > 1u) return -1;
  if (stats) {
    stats->admitted_per_inst.assign(n_inst, 0);
    stats->tbt_first.assign(n_inst, 0.0f);
    stats->wait_ticks = 0;
  }
  std::vector<float> iDt(n_slo), iDb(n_slo);
  for (uint32_t k = 0; k < n_slo; ++k) {
    iDt[k] = recip_deadline(d_ttft[k]);
    iDb[k] = recip_deadline(d_tbt[k]);
  }
  const float nan = std::numeric_limits<float>::quiet_NaN();
  std::vector<Staged> st(n_inst);
  std::vector<uint32_t> n_new(n_inst);
  std::vector<uint64_t> t_new(n_inst);
  uint64_t sat = 0;
  const uint32_t step = (window == 0) ? std::max<uint32_t>(n_req, 1u) : window;
  for (uint64_t s = 0; s < n_req; s += step) {
    const uint32_t e = (uint32_t)std::min<uint64_t>(s + step, n_req);
    for (uint32_t j = 0; j < n_inst; ++j)
      st[j] = stage_instance(pf, tp_idx[j], max_batch[j], occ[j], q_ticks[j], s_bar, pen_kappa,
                             tbt_mode);
    std::fill(n_new.begin(), n_new.end(), 0u);
    std::fill(t_new.begin(), t_new.end(), (uint64_t)0);
    if (stats && s == 0)
      for (uint32_t j = 0; j < n_inst; ++j) stats->tbt_first[j] = st[j].tbt;
    for (uint32_t r = (uint32_t)s; r < e; ++r) {
      const float L = (float)prompt_len[r], S = (float)out_len[r];
      const uint32_t k = slo_class[r];
      const float Dt = d_ttft[k], Db = d_tbt[k];
      const float De = fmaf(S, Db, Dt);
      const float iDe = 1.0f / De;
      float best = -INFINITY;
      int32_t idx = -1;
      Triple bt{nan, nan, nan, nan, nan, nan, nan};
      for (uint32_t j = 0; j < n_inst; ++j) {
        Triple t = score_triple(st[j], L, S, Dt, Db, De, iDt[k], iDb[k], iDe);
        if (t.slack > best) { best = t.slack; idx = (int32_t)j; bt = t; }
      }
      if (policy == 1) {
        // Sec. IV-F step 2 as the paper words it: among the instances able to meet the request's
        // SLO (slack >= 0) the one with the shortest request queue - the fewest requests on it at
        // the start of the window - and the lowest index among those.  Without a capable instance
        // the request is blocked and the largest-slack instance found above is reported.
        int32_t pick = -1;
        Triple pt{nan, nan, nan, nan, nan, nan, nan};
        for (uint32_t j = 0; j < n_inst; ++j) {
          Triple t = score_triple(st[j], L, S, Dt, Db, De, iDt[k], iDb[k], iDe);
          if (!(t.slack >= 0.0f)) continue;
          if (pick < 0 || occ[j] < occ[pick]) { pick = (int32_t)j; pt = t; }
        }
        if (pick >= 0) { idx = pick; best = pt.slack; bt = pt; }
      }
      const bool admitted = best >= 0.0f;
      if (admitted) {
        ++sat;
        if (stats) {
          stats->admitted_per_inst[idx] += 1;
          stats->wait_ticks += (uint64_t)lrintf(st[idx].wait * 1048576.0f);
        }
        if (window != 0) {
          n_new[idx] += 1;
          t_new[idx] += (uint64_t)lrintf(bt.pre * 1048576.0f);
        }
      }
      if (chosen) chosen[r] = idx;
      if (slack) slack[r] = best;
      if (lat_ttft) lat_ttft[r] = bt.ttft;
      if (lat_tbt) lat_tbt[r] = (idx >= 0) ? st[idx].tbt : nan;
      if (lat_e2e) lat_e2e[r] = bt.e2e;
    }
    if (window != 0) {
      const bool more = e < n_req;
      const uint32_t delta = more ? (arrival_ticks[e] - arrival_ticks[s]) : 0u;
      for (uint32_t j = 0; j < n_inst; ++j) {
        occ[j] += (int32_t)n_new[j];
        q_ticks[j] += t_new[j];
        if (!more) continue;  // after the last window: loaded, not drained
        q_ticks[j] -= std::min<uint64_t>(q_ticks[j], (uint64_t)delta);
        const int32_t run = std::min<int32_t>(occ[j], (int32_t)max_batch[j]);
        const float x = ((float)run * ((float)delta * 0x1p-20f)) / st[j].svc;
        const int32_t done = std::min<int32_t>(occ[j], (int32_t)floorf(fminf(x, 2147483520.0f)));
        occ[j] -= done;
      }
    }
  }
  if (n_satisfied) *n_satisfied = sat;
  return 0;
}

struct RequestSet {
  uint32_t n_req;
  const uint32_t* prompt_len;
  const uint32_t* out_len;
  const uint8_t* slo_class;
  const uint32_t* arrival_ticks;
};

struct ScoreSetup {
  float s_bar, pen_kappa;
  uint32_t tbt_mode, window, policy;
  float alpha, beta, gamma_t, gamma_l;
};

struct DeploymentScore {
  uint64_t sat = 0;
  float phi_s = 0, phi_t = 0, phi_l = 0, score = 0;
};

// Composite serving score of one deployment (Sec. IV-D, Eq. 3-8): run the distributor over all of
// R_x on a private copy of the instances' state, then
//   Phi_S^n = admitted / |R_x|;  Phi_T = sum over instances that served a request of 1 / tbt_j
//   (index order, tbt_j of the first window);  Phi_L = mean over admitted requests of their
//   instance's queue wait at admission;  Phi = alpha Phi_S^n + beta min(Phi_T, gamma_T) / gamma_T +
//   (1 - beta) max(gamma_L - Phi_L, 0) / gamma_L.
int score_deployment(const Profile& pf, const RequestSet& rs, const ScoreSetup& su, uint32_t ni,
                     const uint8_t* tp_idx, const uint16_t* max_batch, const int32_t* occ,
                     const uint64_t* q_ticks, DeploymentScore& d) {
  std::vector<int32_t> occ_c(occ, occ + ni);
  std::vector<uint64_t> q_c(q_ticks, q_ticks + ni);
  RunStats st;
  // one window over everything never reaches the state update, which is what "static" means
  const uint32_t win = su.window ? su.window : std::max<uint32_t>(rs.n_req, 1u);
  uint64_t sat = 0;
  const int rc = distributor(pf.n_tp, pf.b_cap, pf.prefill_a, pf.prefill_p, pf.tbt, pf.n_slo,
                             pf.d_ttft, pf.d_tbt, ni, tp_idx, max_batch, occ_c.data(), q_c.data(),
                             rs.n_req, rs.prompt_len, rs.out_len, rs.slo_class, rs.arrival_ticks,
                             su.s_bar, su.pen_kappa, su.tbt_mode, win, su.policy, nullptr, nullptr, nullptr,
                             nullptr, nullptr, &sat, &st);
  if (rc != 0) return rc;
  const float ps = (rs.n_req == 0) ? 0.0f : (float)sat / (float)rs.n_req;
  float pt = 0.0f;
  for (uint32_t j = 0; j < ni; ++j)
    if (st.admitted_per_inst[j] != 0) pt = pt + 1.0f / st.tbt_first[j];
  const float pl = (sat == 0) ? 0.0f : ((float)st.wait_ticks * 0x1p-20f) / (float)sat;
  const float ptn = fminf(pt, su.gamma_t) / su.gamma_t;
  const float pln = fmaxf(su.gamma_l - pl, 0.0f) / su.gamma_l;
  d.sat = sat;
  d.phi_s = ps; d.phi_t = pt; d.phi_l = pl;
  d.score = fmaf(su.alpha, ps, fmaf(su.beta, ptn, (1.0f - su.beta) * pln));
  return 0;
}

}  // namespace

extern "C" {

// Distributor over one placement (the first n_inst slots of the arrays given).
//   window == 0 : every request scores against the given state; the state is left untouched.
//   window  > 0 : requests are taken in windows of that many; all requests of a window see the state
//                 at the window's start; after each window the state is advanced (occ, q_ticks are
//                 updated in place).
// Per-request outputs (each may be NULL): chosen instance (-1 if there is none), its slack, and the
// chosen instance's ttft / tbt / e2e latencies (NaN if there is none).  Returns 0, -1 bad profile.
int oracle_score_assign(uint32_t n_tp, uint32_t b_cap, const float* prefill_a,
                        const float* prefill_p, const float* tbt, uint32_t n_slo,
                        const float* d_ttft, const float* d_tbt, uint32_t n_inst,
                        const uint8_t* tp_idx, const uint16_t* max_batch, int32_t* occ,
                        uint64_t* q_ticks, uint32_t n_req, const uint32_t* prompt_len,
                        const uint32_t* out_len, const uint8_t* slo_class,
                        const uint32_t* arrival_ticks, float s_bar, float pen_kappa,
                        uint32_t tbt_mode, uint32_t window, uint32_t policy, int32_t* chosen,
                        float* slack,
                        float* lat_ttft, float* lat_tbt, float* lat_e2e, uint64_t* n_satisfied) {
  return distributor(n_tp, b_cap, prefill_a, prefill_p, tbt, n_slo, d_ttft, d_tbt, n_inst, tp_idx,
                     max_batch, occ, q_ticks, n_req, prompt_len, out_len, slo_class, arrival_ticks,
                     s_bar, pen_kappa, tbt_mode, window, policy, chosen, slack, lat_ttft, lat_tbt,
                     lat_e2e,
                     n_satisfied, nullptr);
}

// Placer: static score of candidates [c_begin, c_end) of a [n_cand][i_pad] placement table against
// all requests.  sat_count / sat_ratio (count / R; 0 for R == 0) are indexed by absolute candidate; best_cand is the lowest
// candidate of the range with the largest count.  Returns 0, -1 bad profile.
int oracle_placement_sweep(uint32_t n_tp, uint32_t b_cap, const float* prefill_a,
                           const float* prefill_p, const float* tbt, uint32_t n_slo,
                           const float* d_ttft, const float* d_tbt, uint32_t n_cand, uint32_t i_pad,
                           const uint32_t* n_inst, const uint8_t* tp_idx, const uint16_t* max_batch,
                           const int32_t* occ, const uint64_t* q_ticks, uint32_t n_req,
                           const uint32_t* prompt_len, const uint32_t* out_len,
                           const uint8_t* slo_class, float s_bar, float pen_kappa,
                           uint32_t tbt_mode, uint32_t c_begin, uint32_t c_end, uint32_t* sat_count,
                           float* sat_ratio, uint32_t* best_cand) {
  Profile pf{n_tp, b_cap, prefill_a, prefill_p, tbt, n_slo, d_ttft, d_tbt};
  if (!profile_ok(pf) || c_end > n_cand) return -1;
  std::vector<float> iDt(n_slo), iDb(n_slo);
  for (uint32_t k = 0; k < n_slo; ++k) {
    iDt[k] = recip_deadline(d_ttft[k]);
    iDb[k] = recip_deadline(d_tbt[k]);
  }
  std::vector<Staged> st(i_pad);
  uint32_t best_c = c_begin, best_n = 0;
  bool have = false;
  for (uint32_t c = c_begin; c < c_end; ++c) {
    const size_t base = (size_t)c * i_pad;
    const uint32_t ni = n_inst[c];
    for (uint32_t j = 0; j < ni; ++j)
      st[j] = stage_instance(pf, tp_idx[base + j], max_batch[base + j], occ[base + j],
                             q_ticks[base + j], s_bar, pen_kappa, tbt_mode);
    uint32_t cnt = 0;
    for (uint32_t r = 0; r < n_req; ++r) {
      const float L = (float)prompt_len[r], S = (float)out_len[r];
      const uint32_t k = slo_class[r];
      const float Dt = d_ttft[k], Db = d_tbt[k];
      const float De = fmaf(S, Db, Dt);
      const float iDe = 1.0f / De;
      float best = -INFINITY;
      for (uint32_t j = 0; j < ni; ++j) {
        Triple t = score_triple(st[j], L, S, Dt, Db, De, iDt[k], iDb[k], iDe);
        if (t.slack > best) best = t.slack;
      }
      if (best >= 0.0f) ++cnt;
    }
    sat_count[c] = cnt;
    sat_ratio[c] = (n_req == 0) ? 0.0f : (float)cnt / (float)n_req;  // empty request set: 0
    if (!have || cnt > best_n) { best_n = cnt; best_c = c; have = true; }
  }
  if (best_cand) *best_cand = best_c;
  return 0;
}

// Placer with capacity-aware scoring: every candidate of [c_begin, c_end) is run through the windowed
// distributor above, on its own copy of its instance state (the candidates do not interact and the
// caller's state is not modified).  sat_count[c] is the number of requests admitted over all
// windows; ratio and best candidate as in the static sweep.  Returns 0, -1 bad arguments.
int oracle_placement_sweep_windowed(uint32_t n_tp, uint32_t b_cap, const float* prefill_a,
                                    const float* prefill_p, const float* tbt, uint32_t n_slo,
                                    const float* d_ttft, const float* d_tbt, uint32_t n_cand,
                                    uint32_t i_pad, const uint32_t* n_inst, const uint8_t* tp_idx,
                                    const uint16_t* max_batch, const int32_t* occ,
                                    const uint64_t* q_ticks, uint32_t n_req,
                                    const uint32_t* prompt_len, const uint32_t* out_len,
                                    const uint8_t* slo_class, const uint32_t* arrival_ticks,
                                    float s_bar, float pen_kappa, uint32_t tbt_mode, uint32_t window,
                                    uint32_t policy,
                                    uint32_t c_begin, uint32_t c_end, uint32_t* sat_count,
                                    float* sat_ratio, uint32_t* best_cand) {
  if (c_end > n_cand || window == 0) return -1;
  std::vector<int32_t> occ_c(i_pad);
  std::vector<uint64_t> q_c(i_pad);
  uint32_t best_c = c_begin, best_n = 0;
  bool have = false;
  for (uint32_t c = c_begin; c < c_end; ++c) {
    const size_t base = (size_t)c * i_pad;
    std::copy(occ + base, occ + base + i_pad, occ_c.begin());
    std::copy(q_ticks + base, q_ticks + base + i_pad, q_c.begin());
    uint64_t sat = 0;
    const int rc = oracle_score_assign(n_tp, b_cap, prefill_a, prefill_p, tbt, n_slo, d_ttft, d_tbt,
                                       std::min(n_inst[c], i_pad), tp_idx + base, max_batch + base,
                                       occ_c.data(), q_c.data(), n_req, prompt_len, out_len, slo_class,
                                       arrival_ticks, s_bar, pen_kappa, tbt_mode, window, policy,
                                       nullptr,
                                       nullptr, nullptr, nullptr, nullptr, &sat);
    if (rc != 0) return rc;
    sat_count[c] = (uint32_t)sat;
    sat_ratio[c] = (n_req == 0) ? 0.0f : (float)sat / (float)n_req;
    if (!have || (uint32_t)sat > best_n) { best_n = (uint32_t)sat; best_c = c; have = true; }
  }
  if (best_cand) *best_cand = best_c;
  return 0;
}

// Composite serving score of every candidate of [c_begin, c_end) (Sec. IV-D, Eq. 6-8):
//   Phi = alpha * Phi_S^n + beta * min(Phi_T, gamma_T) / gamma_T + (1 - beta) * max(gamma_L - Phi_L, 0) / gamma_L
// observed from a run of the distributor over the candidate (window == 0: one pass against the state
// as given; window > 0: capacity-aware, on a copy of the state):
//   Phi_S^n = admitted / R                                             (SLO satisfaction ratio, Eq. 3)
//   Phi_T   = sum over the instances that served at least one request, in index order, of
//             1 / tbt_j, tbt_j taken at the first window                (decoding throughput, Eq. 4)
//   Phi_L   = mean over the admitted requests of their instance's queue wait at admission, from the
//             exact integer sum of lrintf(wait * 2^20) ticks            (queuing latency, Eq. 5)
// All float operations are single binary32 operations in the order written below.
// Outputs are indexed by absolute candidate; best_cand is the lowest candidate of the range with the
// largest score.  Returns 0, -1 bad arguments.
int oracle_placement_score(uint32_t n_tp, uint32_t b_cap, const float* prefill_a,
                           const float* prefill_p, const float* tbt, uint32_t n_slo,
                           const float* d_ttft, const float* d_tbt, uint32_t n_cand, uint32_t i_pad,
                           const uint32_t* n_inst, const uint8_t* tp_idx, const uint16_t* max_batch,
                           const int32_t* occ, const uint64_t* q_ticks, uint32_t n_req,
                           const uint32_t* prompt_len, const uint32_t* out_len,
                           const uint8_t* slo_class, const uint32_t* arrival_ticks, float s_bar,
                           float pen_kappa, uint32_t tbt_mode, uint32_t window, uint32_t policy,
                           float alpha,
                           float beta, float gamma_t, float gamma_l, uint32_t c_begin, uint32_t c_end,
                           uint32_t* sat_count, float* phi_s, float* phi_t, float* phi_l,
                           float* score, uint32_t* best_cand) {
  if (c_end > n_cand || !(gamma_t > 0.0f) || !(gamma_l > 0.0f)) return -1;
  const Profile pf{n_tp, b_cap, prefill_a, prefill_p, tbt, n_slo, d_ttft, d_tbt};
  const RequestSet rs{n_req, prompt_len, out_len, slo_class, arrival_ticks};
  const ScoreSetup su{s_bar, pen_kappa, tbt_mode, window, policy, alpha, beta, gamma_t, gamma_l};
  uint32_t best_c = c_begin;
  float best_s = -INFINITY;
  for (uint32_t c = c_begin; c < c_end; ++c) {
    const size_t base = (size_t)c * i_pad;
    const uint32_t ni = std::min(n_inst[c], i_pad);
    DeploymentScore d;
    const int rc = score_deployment(pf, rs, su, ni, tp_idx + base, max_batch + base, occ + base,
                                    q_ticks + base, d);
    if (rc != 0) return rc;
    sat_count[c] = (uint32_t)d.sat;
    phi_s[c] = d.phi_s; phi_t[c] = d.phi_t; phi_l[c] = d.phi_l; score[c] = d.score;
    if (d.score > best_s) { best_s = d.score; best_c = c; }
  }
  if (best_cand) *best_cand = best_c;
  return 0;
}

// Alg. 1 (simulator-based instance configuration, Sec. IV-E) for a single model.
//
// With one model the set M has one element, so "the model with most unserved requests" is always that
// model and the first rejected instance saturates it, which ends the inner loop.  For every
// configuration (P_i, B_i) in the given order the deployment grows by one fresh instance (empty, no
// queued work) at a time; the grown deployment I' is scored against all of R_x with the composite
// score (the distributor run of oracle_placement_score); it replaces I when its score is strictly
// larger than I's (the empty deployment scores 0), and otherwise the configuration is finished.
// Phi*[k] / I*[k] keep, per GPU count k = gpuCount(I) of the accepted deployment, the best score seen
// (strictly larger replaces, so the earliest configuration wins ties); I*[k] is reported as
// (configuration index, instance count), cfg_star[k] = -1 where nothing was stored (Phi*[k] = 0).
// Readings: k is taken after acceptance; a grown deployment that would not fit in n_gpus GPUs, or
// would have more than max_inst instances, is not evaluated and finishes the configuration.
// n_evaluated (may be null) receives the number of deployments scored.
// Returns 0, -1 bad arguments, -2 invalid profile or configuration.
int oracle_ins_deploy(uint32_t n_tp, uint32_t b_cap, const float* prefill_a, const float* prefill_p,
                      const float* tbt, uint32_t n_slo, const float* d_ttft, const float* d_tbt,
                      const uint32_t* tp_degree, uint32_t n_req, const uint32_t* prompt_len,
                      const uint32_t* out_len, const uint8_t* slo_class,
                      const uint32_t* arrival_ticks, float s_bar, float pen_kappa, uint32_t tbt_mode,
                      uint32_t window, uint32_t policy, float alpha, float beta, float gamma_t,
                      float gamma_l, uint32_t n_gpus, uint32_t n_cfg, const uint8_t* cfg_tp, const uint16_t* cfg_b,
                      uint32_t max_inst, float* phi_star, int32_t* cfg_star, uint32_t* cnt_star,
                      uint64_t* n_evaluated) {
  if (!tp_degree || !(gamma_t > 0.0f) || !(gamma_l > 0.0f)) return -1;
  const Profile pf{n_tp, b_cap, prefill_a, prefill_p, tbt, n_slo, d_ttft, d_tbt};
  const RequestSet rs{n_req, prompt_len, out_len, slo_class, arrival_ticks};
  const ScoreSetup su{s_bar, pen_kappa, tbt_mode, window, policy, alpha, beta, gamma_t, gamma_l};
  for (uint32_t k = 0; k <= n_gpus; ++k) { phi_star[k] = 0.0f; cfg_star[k] = -1; cnt_star[k] = 0; }
  uint64_t evaluated = 0;
  for (uint32_t i = 0; i < n_cfg; ++i) {
    if (cfg_tp[i] >= n_tp || tp_degree[cfg_tp[i]] == 0) return -2;
    const uint32_t deg = tp_degree[cfg_tp[i]];
    std::vector<uint8_t> tp;       // the accepted deployment I: identical fresh instances
    std::vector<uint16_t> mb;
    float phi = 0.0f;
    while ((uint64_t)tp.size() * deg < n_gpus) {
      const size_t grown = tp.size() + 1;
      if (grown * deg > n_gpus || grown > max_inst) break;
      std::vector<uint8_t> tp2(tp);
      std::vector<uint16_t> mb2(mb);
      tp2.push_back(cfg_tp[i]);
      mb2.push_back(cfg_b[i]);
      const std::vector<int32_t> occ2(grown, 0);
      const std::vector<uint64_t> q2(grown, 0);
      DeploymentScore d;
      const int rc = score_deployment(pf, rs, su, (uint32_t)grown, tp2.data(), mb2.data(),
                                      occ2.data(), q2.data(), d);
      if (rc != 0) return -2;
      ++evaluated;
      if (!(d.score > phi)) break;  // the model is saturated under this configuration
      phi = d.score;
      tp.swap(tp2);
      mb.swap(mb2);
      const size_t k = tp.size() * deg;
      if (phi > phi_star[k]) {
        phi_star[k] = phi;
        cfg_star[k] = (int32_t)i;
        cnt_star[k] = (uint32_t)tp.size();
      }
    }
  }
  if (n_evaluated) *n_evaluated = evaluated;
  return 0;
}

// Alg. 2's scan over the two-way GPU partitions (dynamic resource partition, Sec. IV-E).
//
// phi_t_star / phi_l_star are Alg. 1's score lists (index = GPU count, 0..n_gpus) for the strict and
// the relaxed request sets.  The relaxed sub-cluster may take g_l = 1 .. G'_l GPUs with
// G'_l = floor(|R_l| / |R| * |G|) (taken as the floor of the exact quotient |R_l| * |G| / |R|; 0 when
// R is empty), the strict one gets the rest, and the pair with the largest phi_t + phi_l (one binary32
// addition) wins if it is strictly larger than the starting value; ascending g_l with a strict
// comparison, so the smallest such g_l.  The starting value is the largest entry of phi_h_star
// (Alg. 1 on all of R and all GPUs: the homogeneous fallback; its lowest index on ties) or 0 when
// phi_h_star is null.  out[0..4] = g_t, g_l, heterogeneous (1/0), k_h (GPU count of the homogeneous
// deployment, 0 without one); when the fallback stands, g_t = k_h and g_l = 0.
int oracle_resource_partition(uint32_t n_gpus, const float* phi_t_star, const float* phi_l_star,
                              const float* phi_h_star, uint64_t n_req_l, uint64_t n_req,
                              uint32_t* out, float* phi_opt) {
  if (n_req_l > n_req) return -1;
  const uint32_t g_l_cap =
      n_req == 0 ? 0u : (uint32_t)(((unsigned __int128)n_req_l * n_gpus) / n_req);
  float opt = 0.0f;
  uint32_t k_h = 0;
  if (phi_h_star)
    for (uint32_t k = 0; k <= n_gpus; ++k)
      if (phi_h_star[k] > opt) { opt = phi_h_star[k]; k_h = k; }
  uint32_t g_t = k_h, g_l = 0, hetero = 0;
  for (uint32_t gl = 1; gl <= g_l_cap && gl <= n_gpus; ++gl) {
    const uint32_t gt = n_gpus - gl;
    const float sum = phi_t_star[gt] + phi_l_star[gl];
    if (sum > opt) { opt = sum; g_t = gt; g_l = gl; hetero = 1; }
  }
  out[0] = g_t; out[1] = g_l; out[2] = hetero; out[3] = k_h;
  *phi_opt = opt;
  return 0;
}

// Independent second route to the static sweep's counts.  For a fixed (instance, class) the first-
// token latency is non-decreasing in prompt length and the end-to-end margin is implied by the other
// two, so feasibility reduces to "tbt within its deadline and prompt_len <= Lmax"; Lmax is found by
// bisection over integers with the same float operations, the per-class threshold is the largest
// Lmax over the candidate's instances, and the count comes from sorted per-class prompt lengths.
int oracle_threshold_sweep(uint32_t n_tp, uint32_t b_cap, const float* prefill_a,
                           const float* prefill_p, const float* tbt, uint32_t n_slo,
                           const float* d_ttft, const float* d_tbt, uint32_t n_cand, uint32_t i_pad,
                           const uint32_t* n_inst, const uint8_t* tp_idx, const uint16_t* max_batch,
                           const int32_t* occ, const uint64_t* q_ticks, uint32_t n_req,
                           const uint32_t* prompt_len, const uint8_t* slo_class, float s_bar,
                           float pen_kappa, uint32_t tbt_mode, uint32_t* sat_count) {
  Profile pf{n_tp, b_cap, prefill_a, prefill_p, tbt, n_slo, d_ttft, d_tbt};
  if (!profile_ok(pf)) return -1;
  std::vector<std::vector<uint32_t>> lens(n_slo);
  for (uint32_t r = 0; r < n_req; ++r) lens[slo_class[r]].push_back(prompt_len[r]);
  for (auto& v : lens) std::sort(v.begin(), v.end());
  const int64_t L_TOP = (1 << 24) - 1;
  for (uint32_t c = 0; c < n_cand; ++c) {
    const size_t base = (size_t)c * i_pad;
    uint32_t cnt = 0;
    for (uint32_t k = 0; k < n_slo; ++k) {
      int64_t theta = -1;  // largest servable prompt length of this class; -1: none
      for (uint32_t j = 0; j < n_inst[c]; ++j) {
        Staged s = stage_instance(pf, tp_idx[base + j], max_batch[base + j], occ[base + j],
                                  q_ticks[base + j], s_bar, pen_kappa, tbt_mode);
        if (!(s.tbt <= d_tbt[k])) continue;
        auto ok = [&](int64_t L) { return s.wait + fmaf(s.p, (float)L, s.a) <= d_ttft[k]; };
        if (!ok(0)) continue;
        int64_t lo = 0, hi = L_TOP + 1;  // ok(lo) true, ok(hi) treated as false
        if (ok(L_TOP)) lo = L_TOP;
        else {
          hi = L_TOP;
          while (hi - lo > 1) {
            int64_t mid = (lo + hi) / 2;
            if (ok(mid)) lo = mid; else hi = mid;
          }
        }
        theta = std::max(theta, lo);
      }
      if (theta < 0) continue;
      const auto& v = lens[k];
      cnt += (uint32_t)(std::upper_bound(v.begin(), v.end(), (uint32_t)theta) - v.begin());
    }
    sat_count[c] = cnt;
  }
  return 0;
}

}  // extern "C"
