// Per-instance profile evaluation and per-triple latency/margin arithmetic, device side (gfx950).
//
// Every float operation is a single IEEE-754 binary32 operation (round to nearest even); the only
// fused ones are the explicit fmaf calls.  The translation unit is compiled with contraction off, so
// the results do not depend on how a kernel tiles or orders the work.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#pragma clang fp contract(off)

namespace maaso {

struct ModelParams {
  float s_bar;
  float pen_kappa;
  uint32_t tbt_mode;
  uint32_t n_tp;
  uint32_t b_cap;
};

// One instance after profile evaluation.
struct Staged {
  float a;     // prefill intercept, seconds
  float p;     // prefill seconds per prompt token
  float tbt;   // seconds per output token, occupancy penalty applied
  float svc;   // expected decode latency E[L_d] = s_bar * tbt
  float wait;  // queue wait seen by an arriving request, seconds
};

// Profile evaluation of one instance (Sec. IV-B Eq. 1: the profile row depends on min(B, W), the
// arriving request included; Sec. IV-C Eq. 5: W * E[L_d] / B queue wait for the requests past the
// batch cap; queued prefill time is added).  `tab` holds the three tables back to back, `cells`
// entries each.  Returns false, leaving `s` untouched, when the slot's configuration is outside the
// tables (the caller treats such an instance as absent).
template <class TablePtr>
__device__ __forceinline__ bool stage_instance(TablePtr tab, uint32_t cells, const ModelParams& mp,
                                               uint32_t tp, uint32_t B, int32_t occ, uint64_t q_ticks,
                                               Staged& s) {
  if (tp >= mp.n_tp || B == 0u || B > mp.b_cap || occ < 0) return false;
  const uint32_t w = (mp.tbt_mode == 1u) ? B : min((uint32_t)occ + 1u, B);
  const uint32_t row = tp * (mp.b_cap + 1u) + w;
  s.a = tab[row];
  s.p = tab[cells + row];
  const float tb = tab[2u * cells + row];
  const float invB = 1.0f / (float)B;
  const int32_t over = max(4 * (int32_t)w - 3 * (int32_t)B, 0);  // > 0 iff the batch is > 75 % full
  const float pen = fmaf(mp.pen_kappa, (float)over * invB, 1.0f);
  s.tbt = tb * pen;
  s.svc = mp.s_bar * s.tbt;
  const uint32_t arriving = (uint32_t)occ + 1u;
  const uint32_t ov = arriving > B ? arriving - B : 0u;  // requests beyond the batch cap
  const float slot = ((float)ov * invB) * s.svc;
  s.wait = (float)q_ticks * 0x1p-20f + slot;
  return true;
}

// Per-request deadline values derived from its class and output length.
struct Deadlines {
  float Dt, Db, De;     // first-token, between-token, end-to-end deadlines (seconds)
  float iDt, iDb, iDe;  // their reciprocals
};

struct Margins {
  float pre, ttft, e2e, slack;
};

// One (request, instance) evaluation: L_r = L_q + L_d against the deadlines (Eq. 2, Eq. 3).
__device__ __forceinline__ Margins score_triple(float a, float p, float tbt, float wait, float L,
                                                float S, const Deadlines& d) {
  Margins m;
  m.pre = fmaf(p, L, a);
  m.ttft = wait + m.pre;
  m.e2e = fmaf(S, tbt, m.ttft);
  const float s1 = (d.Dt - m.ttft) * d.iDt;
  const float s2 = (d.Db - tbt) * d.iDb;
  const float s3 = (d.De - m.e2e) * d.iDe;
  m.slack = fminf(fminf(s1, s2), s3);
  return m;
}

}  // namespace maaso
