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
  uint32_t n_cand;           // rows in the placement arrays
  const uint32_t* cand_sel;  // [1] device word naming the row to distribute over; null = row 0
  const uint32_t* n_inst;    // [n_cand]
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
  unsigned long long* sat_acc;  // [1] admitted count and delivered-blocks counter of the static kernel; zero between calls
};

__global__ void assign_init_kernel(unsigned long long* n_satisfied) {
  if (n_satisfied && threadIdx.x == 0 && blockIdx.x == 0) *n_satisfied = 0ull;
}

struct ClassRow {
  float Dt, Db, iDt, iDb;
};

// The placement row a call works on.  The row index may live on the device (the best candidate of a
// sweep that ran just before on the same stream), so that no host round trip separates the two.
struct PlacementRow {
  uint32_t n;  // valid instances, already clamped to i_pad; 0 when the index is out of range
  const uint8_t* tp_idx;
  const uint16_t* max_batch;
  int32_t* occ;
  uint64_t* q_ticks;
};
__device__ __forceinline__ PlacementRow select_row(const AssignArgs& a) {
  uint32_t c = a.cand_sel ? *a.cand_sel : 0u;
  PlacementRow r;
  if (c >= a.n_cand) {
    raise_status(a.status, 2u);
    c = 0u;
    r.n = 0u;
  } else {
    r.n = min(a.n_inst[c], a.i_pad);
  }
  const size_t off = (size_t)c * a.i_pad;
  r.tp_idx = a.tp_idx + off;
  r.max_batch = a.max_batch + off;
  r.occ = a.occ + off;
  r.q_ticks = a.q_ticks + off;
  return r;
}

// Stage the placement's instances into LDS records {a, p, tbt, wait}.  An instance outside the
// tables keeps its slot (dropping it would shift the indices) with a record that can never win:
// wait = +inf gives slack = -inf, which a strict '>' against -inf never takes.
__device__ __forceinline__ void stage_placement(const AssignArgs& a, const PlacementRow& row, uint32_t n,
                                                float4* recs, float* svc) {
  for (uint32_t j = threadIdx.x; j < n; j += blockDim.x) {
    Staged s;
    if (stage_instance(a.tab, a.cells, a.mp, row.tp_idx[j], row.max_batch[j], row.occ[j], row.q_ticks[j], s)) {
      recs[j] = make_float4(s.a, s.p, s.tbt, s.wait);
      if (svc) svc[j] = s.svc;
    } else {
      raise_status(a.status, 2u);
      recs[j] = make_float4(1.0f, 1.0f, 1.0f, INFINITY);
      if (svc) svc[j] = 1.0f;
    }
  }
}

// Shortest-queue rule (Sec. IV-F step 2 as worded in the paper: among the instances able to meet the
// request's SLO, the one with the shortest request queue, lowest index on ties).  Every instance gets
// a value from its place in the order of (requests on it, index): 512 - place, in [257, 512].  A
// triple whose slack is non-negative competes with that value instead of its slack; slacks never
// exceed 1, so capable instances beat incapable ones, the shortest queue beats the longer one, and
// the values being distinct, no ties arise.  With no capable instance the comparison is the ordinary
// one on (negative) slacks, and the request is blocked as before.
__device__ __forceinline__ float queue_rank_value(const int32_t* occ_s, uint32_t n, uint32_t j) {
  const int32_t mine = occ_s[j];
  uint32_t place = 0;
  for (uint32_t i = 0; i < n; ++i) {
    const int32_t o = occ_s[i];
    place += (o < mine || (o == mine && i < j)) ? 1u : 0u;
  }
  return (float)(512u - place);
}

constexpr int kS2Stride = 257;  // odd: the per-class rows of the margin table fall on different banks

// V consecutive requests starting at r0 (V = 4: 16-byte loads and stores; V = 1: any alignment).
// The instance loop is outermost so that one broadcast LDS read of a record serves all V requests;
// j ascending and a strict '>' give the lowest index among equal slacks.  The between-token margin
// (D_tbt - tbt_j) / D_tbt depends on (class, instance) only and is read from an LDS table.
//
// NREG = 0: records and between-token margins are read from LDS (any number of instances).
// NREG > 0: the placement has at most NREG instances and the caller holds their records in
// registers (`rreg`); the margin is recomputed from the class row, so the loop touches no LDS - the
// form used when there are so few instances that the request stream from HBM is the bound.
//
// Four consecutive requests as they come from memory: two 16-byte loads and one 4-byte load.
struct RequestVec {
  uint4 pl, ol;
  uint32_t kk;
};
// The request streams are read once and the outputs written once: both go past the caches as
// non-temporal accesses (measured on the HBM-bound shape: 218.7 -> 201 us).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store_stream(int32_t* p, int32_t x, int32_t y, int32_t z, int32_t w) {
  const i32x4 t = {x, y, z, w};
  __builtin_nontemporal_store(t, reinterpret_cast<i32x4*>(p));
}
__device__ __forceinline__ void store_stream(float* p, float x, float y, float z, float w) {
  const f32x4 t = {x, y, z, w};
  __builtin_nontemporal_store(t, reinterpret_cast<f32x4*>(p));
}
__device__ __forceinline__ RequestVec load_request_vec(const AssignArgs& a, uint64_t r0) {
  RequestVec v;
  const u32x4 pl = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(a.prompt_len + r0));
  const u32x4 ol = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(a.out_len + r0));
  v.pl = make_uint4(pl.x, pl.y, pl.z, pl.w);
  v.ol = make_uint4(ol.x, ol.y, ol.z, ol.w);
  v.kk = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(a.slo_class + r0));
  return v;
}

// kSQ: shortest-queue rule; `rankv` (LDS) or `rrank` (registers, with NREG) hold the instances'
// queue_rank_value, and the slack written out is the chosen instance's own.
template <bool kLat, int V, int NREG, bool kSQ>
__device__ __forceinline__ uint32_t assign_requests(const AssignArgs& a, uint64_t r0, uint32_t n,
                                                    const float4* __restrict__ recs,
                                                    const ClassRow* __restrict__ cls,
                                                    const float* __restrict__ s2tab,
                                                    const float4* rreg,
                                                    const float* __restrict__ rankv,
                                                    const float* rrank,
                                                    const RequestVec* pre = nullptr) {
  float L[V], S[V], best[V], De[V], iDe[V], Dt[V], iDt[V], Db[V], iDb[V];
  float b_slack[V];
  float b_ttft[V], b_tbt[V], b_e2e[V];
  uint32_t k[V];
  int32_t idx[V];
  if (V == 4) {
    const RequestVec rv = pre ? *pre : load_request_vec(a, r0);
    const uint4 pl = rv.pl, ol = rv.ol;
    const uint32_t kk = rv.kk;
    const uint32_t p4[4] = {pl.x, pl.y, pl.z, pl.w}, o4[4] = {ol.x, ol.y, ol.z, ol.w};
#pragma unroll
    for (int v = 0; v < V; ++v) {
      L[v] = (float)p4[v]; S[v] = (float)o4[v]; k[v] = (kk >> (8 * v)) & 0xffu;
    }
  } else {
#pragma unroll
    for (int v = 0; v < V; ++v) {
      L[v] = (float)a.prompt_len[r0 + v]; S[v] = (float)a.out_len[r0 + v]; k[v] = a.slo_class[r0 + v];
    }
  }
  bool ok[V];
#pragma unroll
  for (int v = 0; v < V; ++v) {
    ok[v] = k[v] < a.n_slo;
    if (!ok[v]) { raise_status(a.status, 1u); k[v] = 0u; }
    const ClassRow c = cls[k[v]];
    Dt[v] = c.Dt; iDt[v] = c.iDt; Db[v] = c.Db; iDb[v] = c.iDb;
    De[v] = fmaf(S[v], c.Db, c.Dt);
    iDe[v] = 1.0f / De[v];
    best[v] = -INFINITY;
    b_slack[v] = -INFINITY;
    idx[v] = -1;
    b_ttft[v] = b_tbt[v] = b_e2e[v] = __builtin_nanf("");
  }
  // r = {a, p, tbt, wait}; m2 = the between-token margins of the V requests when they come from the table
  auto score = [&](const float4 r, const float (&m2)[V], uint32_t j, float rank) {
#pragma unroll
    for (int v = 0; v < V; ++v) {
      const float pre = fmaf(r.y, L[v], r.x);
      const float ttft = r.w + pre;
      const float e2e = fmaf(S[v], r.z, ttft);
      const float s1 = (Dt[v] - ttft) * iDt[v];
      const float s2 = NREG ? (Db[v] - r.z) * iDb[v] : m2[v];
      const float s3 = (De[v] - e2e) * iDe[v];
      const float slack = fminf(fminf(s1, s2), s3);
      const float val = (kSQ && slack >= 0.0f) ? rank : slack;
      if (NREG || (!kLat && !kSQ)) {  // nothing but (best, idx) to carry, or records in registers
        if (val > best[v]) {
          best[v] = val;
          idx[v] = (int32_t)j;
          if (kSQ) b_slack[v] = slack;
          if (kLat) { b_ttft[v] = ttft; b_tbt[v] = r.z; b_e2e[v] = e2e; }
        }
      } else {
        // one compare, one select, one max per triple instead of a select per reported quantity: what
        // else is reported about the winner is worked out again after the loop from its record (the
        // same operations, so the same bits)
        idx[v] = (val > best[v]) ? (int32_t)j : idx[v];
        best[v] = max_no_nan(best[v], val);
      }
    }
  };
  if (NREG) {
    const float none[V] = {};
#pragma unroll
    for (int j = 0; j < (NREG ? NREG : 1); ++j)
      if ((uint32_t)j < n) score(rreg[j], none, (uint32_t)j, kSQ ? rrank[j] : 0.0f);
  } else {
    // four records and their margins are fetched per trip before any is used: one LDS wait and one
    // round of address arithmetic for sixteen triples
    constexpr uint32_t U = 4;
    uint32_t j = 0;
    for (; j + U <= n; j += U) {
      float4 r[U];
      float m2[U][V], rk[U];
#pragma unroll
      for (uint32_t u = 0; u < U; ++u) {
        r[u] = recs[j + u];
        rk[u] = kSQ ? rankv[j + u] : 0.0f;
#pragma unroll
        for (int v = 0; v < V; ++v) m2[u][v] = s2tab[k[v] * kS2Stride + j + u];
      }
#pragma unroll
      for (uint32_t u = 0; u < U; ++u) score(r[u], m2[u], j + u, rk[u]);
    }
    for (; j < n; ++j) {
      float m2[V];
#pragma unroll
      for (int v = 0; v < V; ++v) m2[v] = s2tab[k[v] * kS2Stride + j];
      score(recs[j], m2, j, kSQ ? rankv[j] : 0.0f);
    }
    if (kLat || kSQ) {
#pragma unroll
      for (int v = 0; v < V; ++v) {
        if (idx[v] < 0) continue;
        const float4 r = recs[idx[v]];
        const float pre = fmaf(r.y, L[v], r.x);
        const float ttft = r.w + pre;
        const float e2e = fmaf(S[v], r.z, ttft);
        if (kLat) { b_ttft[v] = ttft; b_tbt[v] = r.z; b_e2e[v] = e2e; }
        if (kSQ) {
          const float s1 = (Dt[v] - ttft) * iDt[v];
          const float s2 = s2tab[k[v] * kS2Stride + idx[v]];
          const float s3 = (De[v] - e2e) * iDe[v];
          b_slack[v] = fminf(fminf(s1, s2), s3);
        }
      }
    }
  }
  uint32_t sat = 0;
#pragma unroll
  for (int v = 0; v < V; ++v) {
    if (!ok[v]) { best[v] = -INFINITY; idx[v] = -1; b_ttft[v] = b_tbt[v] = b_e2e[v] = __builtin_nanf(""); }
    sat += (best[v] >= 0.0f) ? 1u : 0u;   // a rank value is positive: some instance can serve
    if (kSQ && ok[v]) best[v] = b_slack[v];  // what is written out is the chosen instance's slack
  }
  if (V == 4) {
    if (a.chosen) store_stream(a.chosen + r0, idx[0], idx[1], idx[2], idx[3]);
    if (a.slack) store_stream(a.slack + r0, best[0], best[1], best[2], best[3]);
    if (kLat) {
      if (a.ttft) store_stream(a.ttft + r0, b_ttft[0], b_ttft[1], b_ttft[2], b_ttft[3]);
      if (a.tbt) store_stream(a.tbt + r0, b_tbt[0], b_tbt[1], b_tbt[2], b_tbt[3]);
      if (a.e2e) store_stream(a.e2e + r0, b_e2e[0], b_e2e[1], b_e2e[2], b_e2e[3]);
    }
  } else {
#pragma unroll
    for (int v = 0; v < V; ++v) {
      if (a.chosen) a.chosen[r0 + v] = idx[v];
      if (a.slack) a.slack[r0 + v] = best[v];
      if (kLat) {
        if (a.ttft) a.ttft[r0 + v] = b_ttft[v];
        if (a.tbt) a.tbt[r0 + v] = b_tbt[v];
        if (a.e2e) a.e2e[r0 + v] = b_e2e[v];
      }
    }
  }
  return sat;
}

// Per-block set-up shared by the static and the windowed kernel: class rows and the table of
// between-token margins s2[k][j] = (D_tbt[k] - tbt_j) * (1 / D_tbt[k]).
__device__ __forceinline__ void fill_class_tables(const AssignArgs& a, uint32_t n, const float4* recs,
                                                  ClassRow* cls, float* s2tab) {
  if (threadIdx.x < a.n_slo) {
    const uint32_t k = threadIdx.x;
    cls[k] = ClassRow{a.d_ttft[k], a.d_tbt[k], a.i_ttft[k], a.i_tbt[k]};
  }
  for (uint32_t i = threadIdx.x; i < a.n_slo * n; i += blockDim.x) {
    const uint32_t k = i / n, j = i - k * n;
    s2tab[k * kS2Stride + j] = (a.d_tbt[k] - recs[j].z) * a.i_tbt[k];
  }
}

// V = 4 needs 16-byte aligned request and output arrays (slo_class 4-byte aligned); the host checks.
// NREG > 0 requires n_inst <= NREG (the host checks against the i_pad it was given).
template <bool kLat, int V, int NREG, bool kSQ>
__global__ __launch_bounds__(kAssignThreads) void assign_static_kernel(const AssignArgs a) {
  __shared__ float4 recs[256];
  __shared__ ClassRow cls[kMaxSlo];
  __shared__ float s2tab[NREG ? 1 : kMaxSlo * kS2Stride];
  __shared__ uint32_t wave_sat[kAssignThreads / 64];
  __shared__ int32_t occ_s[kSQ ? 256 : 1];
  __shared__ float rankv[kSQ ? 256 : 1];
  // the block's first requests are asked for before anything else: their latency then overlaps the
  // staging of the instances below
  const uint64_t n_vec = (uint64_t)a.n_req / V;  // groups of V requests
  const uint64_t g0 = (uint64_t)blockIdx.x * kAssignThreads + threadIdx.x;
  const uint64_t stride = (uint64_t)gridDim.x * kAssignThreads;
  RequestVec cur{}, nxt{};
  if (V == 4 && g0 < n_vec) cur = load_request_vec(a, g0 * V);
  const PlacementRow row = select_row(a);
  const uint32_t n = min(row.n, NREG ? (uint32_t)NREG : 256u);
  stage_placement(a, row, n, recs, nullptr);
  if (kSQ)
    for (uint32_t j = threadIdx.x; j < n; j += blockDim.x) occ_s[j] = row.occ[j];
  __syncthreads();
  if (kSQ)
    for (uint32_t j = threadIdx.x; j < n; j += blockDim.x) rankv[j] = queue_rank_value(occ_s, n, j);
  if (NREG) {
    if (threadIdx.x < a.n_slo) {
      const uint32_t k = threadIdx.x;
      cls[k] = ClassRow{a.d_ttft[k], a.d_tbt[k], a.i_ttft[k], a.i_tbt[k]};
    }
  } else {
    fill_class_tables(a, n, recs, cls, s2tab);
  }
  __syncthreads();
  float4 rreg[NREG ? NREG : 1];
  float rrank[NREG ? NREG : 1];
#pragma unroll
  for (int j = 0; j < (NREG ? NREG : 1); ++j) {
    rreg[j] = (NREG && (uint32_t)j < n) ? recs[j] : make_float4(1.0f, 1.0f, 1.0f, INFINITY);
    rrank[j] = (kSQ && NREG && (uint32_t)j < n) ? rankv[j] : 0.0f;
  }

  uint32_t sat = 0;
  if (V == 4) {
    // the next group's requests are loaded before the current group is scored, so that a thread
    // always has loads in flight (the loop is otherwise load -> wait -> compute -> store)
    for (uint64_t g = g0; g < n_vec; g += stride) {
      if (g + stride < n_vec) nxt = load_request_vec(a, (g + stride) * V);
      sat += assign_requests<kLat, V, NREG, kSQ>(a, g * V, n, recs, cls, s2tab, rreg, rankv, rrank, &cur);
      cur = nxt;
    }
  } else {
    for (uint64_t g = g0; g < n_vec; g += stride)
      sat += assign_requests<kLat, V, NREG, kSQ>(a, g * V, n, recs, cls, s2tab, rreg, rankv, rrank);
  }
  if (V > 1 && blockIdx.x == 0) {  // the ragged tail, one request per thread
    const uint64_t r = n_vec * V + threadIdx.x;
    if (r < a.n_req) sat += assign_requests<kLat, 1, NREG, kSQ>(a, r, n, recs, cls, s2tab, rreg, rankv, rrank);
  }
  // Admitted count: wavefront shuffle, block sum in LDS, then ONE returning device-scope atomic per
  // block on a 64-bit word the library owns and keeps at zero between calls: the block's count goes
  // into the low 40 bits and a 1 into the bits above, so the returned value tells the block how many
  // blocks delivered before it.  The last one knows the total, writes the output and zeroes the word:
  // no clearing launch, no fence (a write-back fence here would flush the kernel's per-request
  // outputs out of the L2), and a single same-address atomic per block (they serialise device-wide:
  // thousands of them at the kernel's end are measurable).
  for (int d = 32; d >= 1; d >>= 1) sat += __shfl_xor(sat, d);
  if ((threadIdx.x & 63u) == 0u) wave_sat[threadIdx.x >> 6] = sat;
  __syncthreads();
  if (threadIdx.x == 0 && a.n_satisfied) {
    unsigned long long t = 0;
    for (int w = 0; w < kAssignThreads / 64; ++w) t += wave_sat[w];
    // one word carries both: the admitted count in its low 40 bits, the blocks delivered above them
    const unsigned long long before = atomicAdd(a.sat_acc, (1ull << 40) | t);
    if ((before >> 40) == (unsigned long long)gridDim.x - 1ull) {
      *a.n_satisfied = (before & ((1ull << 40) - 1ull)) + t;
      atomicExch(a.sat_acc, 0ull);
    }
  }
}

}  // namespace maaso
