// Distributor: instance assignment with overflow protection (Sec. IV-F steps 2 and 3) for one
// placement.  Static form: every request is scored against the state as given.
//
// Layout: lanes = requests (coalesced structure-of-arrays reads of prompt_len / out_len / slo_class,
// coalesced writes of chosen / slack / latencies).  The placement's instances are evaluated once per
// block ("stage": Eq. 1 profile row, occupancy penalty, queue wait) into LDS records that every lane
// then reads with broadcast LDS loads; the per-class deadline table also sits in LDS.  Blocks are
// persistent over a grid-stride loop of request tiles, so staging is paid once per block.
#pragma once

#include "device_model.hpp"
#include "sweep_kernels.hpp"

#pragma clang fp contract(off)

namespace maaso {

constexpr int kAssignThreads = 256;

struct AssignArgs {
  const float* tab;
  uint32_t cells;
  ModelParams mp;
  uint32_t n_slo;
  float d_ttft[kMaxSlo], d_tbt[kMaxSlo], i_ttft[kMaxSlo], i_tbt[kMaxSlo];
  uint32_t i_pad;
  const uint32_t* n_inst;  // [1]
  const uint8_t* tp_idx;
  const uint16_t* max_batch;
  int32_t* occ;
  uint64_t* q_ticks;
  uint32_t n_req;
  const uint32_t* prompt_len;
  const uint32_t* out_len;
  const uint8_t* slo_class;
  const uint32_t* arrival_ticks;
  int32_t* chosen;
  float* slack;
  float* ttft;
  float* tbt;
  float* e2e;
  unsigned long long* n_satisfied;
  uint32_t* status;
};

__global__ void assign_init_kernel(unsigned long long* n_satisfied) {
  if (n_satisfied && threadIdx.x == 0 && blockIdx.x == 0) *n_satisfied = 0ull;
}

struct ClassRow {
  float Dt, Db, iDt, iDb;
};

// Scores one request against n staged instances held in LDS; j ascending and a strict '>' give the
// lowest index among equal slacks.
template <bool kLat>
__device__ __forceinline__ void best_instance(const float4* __restrict__ recs, uint32_t n, float L,
                                              float S, const Deadlines& d, float& best, int32_t& idx,
                                              float& b_ttft, float& b_tbt, float& b_e2e) {
  best = -INFINITY;
  idx = -1;
  b_ttft = b_tbt = b_e2e = __builtin_nanf("");
  for (uint32_t j = 0; j < n; ++j) {
    const float4 r = recs[j];  // a, p, tbt, wait
    const Margins m = score_triple(r.x, r.y, r.z, r.w, L, S, d);
    if (m.slack > best) {
      best = m.slack;
      idx = (int32_t)j;
      if (kLat) { b_ttft = m.ttft; b_tbt = r.z; b_e2e = m.e2e; }
    }
  }
}

// Stage the placement's instances into LDS records {a, p, tbt, wait}; invalid slots are compacted
// out would change indices, so an instance outside the tables keeps its slot with a record that can
// never win (wait = +inf gives slack = -inf, which a strict '>' against -inf never takes).
__device__ __forceinline__ void stage_placement(const AssignArgs& a, uint32_t n, float4* recs,
                                                float* svc) {
  for (uint32_t j = threadIdx.x; j < n; j += blockDim.x) {
    Staged s;
    if (stage_instance(a.tab, a.cells, a.mp, a.tp_idx[j], a.max_batch[j], a.occ[j], a.q_ticks[j], s)) {
      recs[j] = make_float4(s.a, s.p, s.tbt, s.wait);
      if (svc) svc[j] = s.svc;
    } else {
      raise_status(a.status, 2u);
      recs[j] = make_float4(1.0f, 1.0f, 1.0f, INFINITY);
      if (svc) svc[j] = 1.0f;
    }
  }
}

template <bool kLat>
__global__ __launch_bounds__(kAssignThreads) void assign_static_kernel(const AssignArgs a) {
  __shared__ float4 recs[256];
  __shared__ ClassRow cls[kMaxSlo];
  __shared__ uint32_t wave_sat[kAssignThreads / 64];
  const uint32_t n = min(a.n_inst[0], a.i_pad);
  stage_placement(a, n, recs, nullptr);
  if (threadIdx.x < a.n_slo) {
    const uint32_t k = threadIdx.x;
    cls[k] = ClassRow{a.d_ttft[k], a.d_tbt[k], a.i_ttft[k], a.i_tbt[k]};
  }
  __syncthreads();

  uint32_t sat = 0;
  for (uint64_t base = (uint64_t)blockIdx.x * kAssignThreads; base < a.n_req;
       base += (uint64_t)gridDim.x * kAssignThreads) {
    const uint64_t r = base + threadIdx.x;
    if (r < a.n_req) {
      const float L = (float)a.prompt_len[r];
      const float S = (float)a.out_len[r];
      const uint32_t k = a.slo_class[r];
      float best = -INFINITY, b_ttft, b_tbt, b_e2e;
      int32_t idx = -1;
      b_ttft = b_tbt = b_e2e = __builtin_nanf("");
      if (k < a.n_slo) {
        const ClassRow c = cls[k];
        Deadlines d;
        d.Dt = c.Dt; d.Db = c.Db; d.iDt = c.iDt; d.iDb = c.iDb;
        d.De = fmaf(S, c.Db, c.Dt);
        d.iDe = 1.0f / d.De;
        best_instance<kLat>(recs, n, L, S, d, best, idx, b_ttft, b_tbt, b_e2e);
      } else {
        raise_status(a.status, 1u);
      }
      if (a.chosen) a.chosen[r] = idx;
      if (a.slack) a.slack[r] = best;
      if (kLat) {
        if (a.ttft) a.ttft[r] = b_ttft;
        if (a.tbt) a.tbt[r] = b_tbt;
        if (a.e2e) a.e2e[r] = b_e2e;
      }
      sat += (best >= 0.0f) ? 1u : 0u;
    }
  }
  // block-then-atomic reduction of the admitted count
  for (int d = 32; d >= 1; d >>= 1) sat += __shfl_xor(sat, d);
  if ((threadIdx.x & 63u) == 0u) wave_sat[threadIdx.x >> 6] = sat;
  __syncthreads();
  if (threadIdx.x == 0 && a.n_satisfied) {
    uint32_t t = 0;
    for (int w = 0; w < kAssignThreads / 64; ++w) t += wave_sat[w];
    if (t) atomicAdd(a.n_satisfied, (unsigned long long)t);
  }
}

}  // namespace maaso
