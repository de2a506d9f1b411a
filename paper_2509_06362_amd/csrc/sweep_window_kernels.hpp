// Placer with capacity-aware scoring: every candidate deployment is run through the windowed
// distributor on its own copy of its instance state - the stand-in for the paper's virtual-slot
// simulator (Sec. V-A "Simulator Implementation") inside the evaluation of a candidate (Alg. 1).
//
// Candidates do not interact, so one block owns one candidate and walks the windows by itself: no
// device-wide barrier.  Thread j keeps instance j's live state (occupancy, queued prefill ticks) in
// registers; per window the block stages its instances into LDS records, fills the per-(class,
// instance) between-token margins, scores the window's requests (lanes = requests, four in flight
// per lane, broadcast LDS reads of the records), adds the admitted load with integer LDS atomics
// (aggregated per wavefront when all its admitted requests chose the same instance, the common case
// when a window herds onto the instance with the most slack), and advances the state exactly as the
// distributor does.
#pragma once

#include "assign_kernels.hpp"
#include "lane_ops.hpp"

#pragma clang fp contract(off)

namespace maaso {

// One request set and the outputs of scoring every candidate against it.
struct SweepWindowSet {
  uint32_t n_req;
  uint32_t window;  // requests per window (>= 1)
  const uint32_t* prompt_len;
  const uint32_t* out_len;
  const uint8_t* slo_class;
  const uint32_t* arrival_ticks;
  uint32_t* sat_count;
  // composite serving score (kScore kernels only); every output may be null
  float* phi_s;
  float* phi_t;
  float* phi_l;
  float* score;
  // One side of a split whose position only the device knows (Alg. 2 scores R_t and R_l straight
  // after the split, without the host reading |R_t| back): with split_at set, the pointers above
  // address the whole split array of n_req requests and the set is its first *split_at requests
  // (side == 1) or the rest (side == 2).
  const uint32_t* split_at;
  uint32_t side;
};

constexpr int kMaxSweepSets = 4;

// The set a block works on, with a device-side split applied.
__device__ __forceinline__ SweepWindowSet resolve_set(const SweepWindowSet& in) {
  SweepWindowSet rs = in;
  if (in.split_at) {
    const uint32_t at = min(*in.split_at, in.n_req);
    const uint32_t off = in.side == 1u ? 0u : at;
    rs.n_req = in.side == 1u ? at : in.n_req - at;
    rs.prompt_len += off;
    rs.out_len += off;
    rs.slo_class += off;
    if (rs.arrival_ticks) rs.arrival_ticks += off;
  }
  return rs;
}

struct SweepWindowArgs {
  const float* tab;
  uint32_t cells;
  ModelParams mp;
  uint32_t n_slo;
  float d_ttft[kMaxSlo], d_tbt[kMaxSlo], i_ttft[kMaxSlo], i_tbt[kMaxSlo];
  uint32_t n_cand, i_pad;
  const uint32_t* n_inst;
  const uint8_t* tp_idx;
  const uint16_t* max_batch;
  const int32_t* occ;
  const uint64_t* q_ticks;
  // Block b scores candidate b % n_cand against set b / n_cand: the sets are independent runs over
  // the same candidates (Alg. 2 scores every deployment against R_t, R_l and all of R), listed
  // longest first so that the blocks that run longest start first.
  uint32_t n_sets;
  SweepWindowSet sets[kMaxSweepSets];
  uint32_t* status;
  float alpha, beta, gamma_t, gamma_l;
};

__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v) {
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
  return v;
}

// kScore: also observe what the composite serving score needs (Sec. IV-D, Eq. 6-8) - which instances
// served a request, and the exact integer sum of the admitted requests' queue waits - and finish the
// candidate's score in the block: Phi = alpha * Phi_S^n + beta * min(Phi_T, gamma_T) / gamma_T +
// (1 - beta) * max(gamma_L - Phi_L, 0) / gamma_L with Phi_T = sum of 1 / tbt_j over the serving
// instances in index order (tbt_j of the first window) and Phi_L = mean wait of the admitted requests.
// V: requests a lane scores at a time (4 for windows of a thousand requests or more; smaller windows
// leave most of those idle, so they run with 2 or 1).
// kSQ: the distributor's shortest-queue rule (see queue_rank_value) instead of the largest slack.
template <bool kScore, int V, bool kSQ>
__global__ __launch_bounds__(kAssignThreads) void sweep_window_kernel(const SweepWindowArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  float* tab = reinterpret_cast<float*>(smem);
  __shared__ float4 recs[256];
  __shared__ ClassRow cls[kMaxSlo];
  __shared__ float s2tab[kMaxSlo * kS2Stride];
  __shared__ uint32_t n_blk[256];
  __shared__ unsigned long long t_blk[256];
  __shared__ uint32_t wave_sat[kAssignThreads / 64];
  __shared__ int32_t occ_s[kSQ ? 256 : 1];
  __shared__ float rankv[kSQ ? 256 : 1];

  const uint32_t tid = threadIdx.x;
  const uint32_t set = blockIdx.x / a.n_cand;
  const uint32_t c = blockIdx.x - set * a.n_cand;
  const SweepWindowSet rs = resolve_set(a.sets[set]);
  const size_t base = (size_t)c * a.i_pad;
  const uint32_t n = min(a.n_inst[c], a.i_pad);
  uint32_t tp = 0, B = 1;
  int32_t occ = 0;
  uint64_t q = 0;
  if (tid < n) {
    tp = a.tp_idx[base + tid]; B = a.max_batch[base + tid];
    occ = a.occ[base + tid]; q = a.q_ticks[base + tid];
  }
  if (tid < a.n_slo) cls[tid] = ClassRow{a.d_ttft[tid], a.d_tbt[tid], a.i_ttft[tid], a.i_tbt[tid]};
  for (uint32_t i = tid; i < 3u * a.cells; i += kAssignThreads) tab[i] = a.tab[i];
  __syncthreads();

  const uint64_t R = rs.n_req;
  const uint64_t n_windows = (R + rs.window - 1) / rs.window;
  uint32_t sat = 0;
  uint32_t served = 0;                // requests admitted to instance tid over all windows
  unsigned long long wait_sum = 0ull; // their queue waits at admission, in ticks
  unsigned long long wait_ticks = 0ull;
  float inv_tbt_first = 0.0f;

  for (uint64_t w = 0; w < n_windows; ++w) {
    const uint64_t s0 = w * rs.window;
    const uint64_t e0 = (s0 + rs.window < R) ? s0 + rs.window : R;
    uint32_t delta = 0;
    if (tid < n && e0 < R) delta = rs.arrival_ticks[e0] - rs.arrival_ticks[s0];
    float svc = 1.0f;
    if (tid < n) {
      Staged st;
      if (stage_instance(tab, a.cells, a.mp, tp, B, occ, q, st)) {
        recs[tid] = make_float4(st.a, st.p, st.tbt, st.wait);
        svc = st.svc;
        if (kScore) {
          wait_ticks = (unsigned long long)__float2ll_rn(st.wait * 1048576.0f);
          if (w == 0) inv_tbt_first = 1.0f / st.tbt;
        }
      } else {
        raise_status(a.status, 2u);
        recs[tid] = make_float4(1.0f, 1.0f, 1.0f, INFINITY);
      }
      n_blk[tid] = 0u;
      t_blk[tid] = 0ull;
      if (kSQ) occ_s[tid] = occ;
      // the instance's between-token margins against every class, while its tbt is at hand
      const float tbt_j = recs[tid].z;
      for (uint32_t k = 0; k < a.n_slo; ++k) s2tab[k * kS2Stride + tid] = (cls[k].Db - tbt_j) * cls[k].iDb;
    }
    __syncthreads();
    if (kSQ) {
      if (tid < n) rankv[tid] = queue_rank_value(occ_s, n, tid);
      __syncthreads();
    }

    for (uint64_t b0 = s0; b0 < e0; b0 += (uint64_t)V * kAssignThreads) {
      float L[V], S[V], Dt[V], iDt[V], De[V], iDe[V], best[V], bpre[V];
      uint32_t k[V];
      int32_t idx[V];
      bool live[V];
#pragma unroll
      for (int v = 0; v < V; ++v) {
        const uint64_t r = b0 + (uint64_t)v * kAssignThreads + tid;
        live[v] = r < e0;
        uint32_t pl = 0, ol = 0;
        k[v] = 0;
        if (live[v]) { pl = rs.prompt_len[r]; ol = rs.out_len[r]; k[v] = rs.slo_class[r]; }
        if (k[v] >= a.n_slo) { raise_status(a.status, 1u); live[v] = false; k[v] = 0; }
        L[v] = (float)pl; S[v] = (float)ol;
        const ClassRow cr = cls[k[v]];
        Dt[v] = cr.Dt; iDt[v] = cr.iDt;
        De[v] = fmaf(S[v], cr.Db, cr.Dt);
        iDe[v] = 1.0f / De[v];
        best[v] = -INFINITY; idx[v] = -1; bpre[v] = 0.0f;
      }
      // one (request v, instance j) triple; r = {a, p, tbt, wait}, s2 = the between-token margin
      auto score_one = [&](const float4 r, float s2, uint32_t j, int v) {
        const float pre = fmaf(r.y, L[v], r.x);
        const float ttft = r.w + pre;
        const float e2e = fmaf(S[v], r.z, ttft);
        const float s1 = (Dt[v] - ttft) * iDt[v];
        const float s3 = (De[v] - e2e) * iDe[v];
        const float slack = fminf(fminf(s1, s2), s3);
        const float val = (kSQ && slack >= 0.0f) ? rankv[j] : slack;
        // one compare, one select, one max: the winner's prefill time is recomputed after the loop
        idx[v] = (val > best[v]) ? (int32_t)j : idx[v];
        best[v] = max_no_nan(best[v], val);
      };
      // U records are fetched per trip before any is used.  With one request per lane a wavefront has
      // little else to overlap an LDS read with (short windows leave a SIMD a few wavefronts);
      // with four, a longer trip also spreads the address bookkeeping of the per-class margin reads
      // over more triples.  Measured: V = 1: U = 4 beats 1 and 8; V = 4: U = 4 beats 1 and 2
      // (128 registers, still four wavefronts per SIMD).
      constexpr uint32_t U = (V == 2) ? 2u : 4u;
      uint32_t j = 0;
      for (; j + U <= n; j += U) {
        float4 r[U];
        float s2[U][V];
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
          r[u] = recs[j + u];
#pragma unroll
          for (int v = 0; v < V; ++v) s2[u][v] = s2tab[k[v] * kS2Stride + j + u];
        }
#pragma unroll
        for (uint32_t u = 0; u < U; ++u)
#pragma unroll
          for (int v = 0; v < V; ++v) score_one(r[u], s2[u][v], j + u, v);
      }
      for (; j < n; ++j) {
        const float4 r = recs[j];
#pragma unroll
        for (int v = 0; v < V; ++v) score_one(r, s2tab[k[v] * kS2Stride + j], j, v);
      }
#pragma unroll
      for (int v = 0; v < V; ++v)
        if (idx[v] >= 0) { const float4 r = recs[idx[v]]; bpre[v] = fmaf(r.y, L[v], r.x); }
#pragma unroll
      for (int v = 0; v < V; ++v) {
        const bool adm = live[v] && best[v] >= 0.0f;  // admitted requests load their instance
        const uint64_t am = __ballot(adm);
        if (am == 0ull) continue;
        sat += adm ? 1u : 0u;
        const unsigned long long ticks = adm ? (unsigned long long)__float2ll_rn(bpre[v] * 1048576.0f) : 0ull;
        const int32_t first = __builtin_amdgcn_readlane(idx[v], __builtin_ctzll(am));
        if (__ballot(adm && idx[v] == first) == am) {  // the whole wavefront chose one instance
          // prefill times below 64 s each (2^26 ticks) add up in 32 bits: the usual case
          const unsigned long long tsum = __ballot((ticks >> 26) != 0ull) == 0ull
                                              ? (unsigned long long)wave_sum_u32((uint32_t)ticks)
                                              : wave_sum_u64(ticks);
          if ((tid & 63u) == 0u) {
            atomicAdd(&n_blk[first], (uint32_t)__popcll(am));
            atomicAdd(&t_blk[first], tsum);
          }
        } else if (adm) {
          atomicAdd(&n_blk[idx[v]], 1u);
          atomicAdd(&t_blk[idx[v]], ticks);
        }
      }
    }
    lds_atomics_barrier();

    if (tid < n) {
      if (kScore) {
        served += n_blk[tid];
        wait_sum += (unsigned long long)n_blk[tid] * wait_ticks;
      }
      occ += (int32_t)n_blk[tid];
      q += t_blk[tid];
      if (e0 < R) {  // time passes until the next window opens
        q -= (q < (uint64_t)delta) ? q : (uint64_t)delta;
        const int32_t run = min(occ, (int32_t)B);
        const float x = ((float)run * ((float)delta * 0x1p-20f)) / svc;
        const int32_t done = min(occ, (int32_t)floorf(fminf(x, 2147483520.0f)));
        occ -= done;
      }
    }
    // No barrier before the next stage: it rewrites recs and the margin table, which every thread
    // finished reading before the barrier above, and n_blk / t_blk entries that only their own thread
    // reads; the next window's atomics on them come after the stage's barrier.
  }

  __syncthreads();  // the last update has read n_blk / t_blk, which are reused below
  for (int d = 32; d >= 1; d >>= 1) sat += __shfl_xor(sat, d);
  if ((tid & 63u) == 0u) wave_sat[tid >> 6] = sat;
  if (kScore) {
    // reuse the LDS arrays of the window loop (all threads are past its last barrier):
    // s2tab[j] = 1 / tbt_j of a serving instance, or -1; t_blk[wave] = wait ticks of the wavefront
    s2tab[tid] = (tid < n && served != 0u) ? inv_tbt_first : -1.0f;
    wait_sum = wave_sum_u64(wait_sum);
    if ((tid & 63u) == 0u) t_blk[tid >> 6] = wait_sum;
  }
  __syncthreads();
  if (tid == 0) {
    uint32_t t = 0;
    for (int wv = 0; wv < kAssignThreads / 64; ++wv) t += wave_sat[wv];
    rs.sat_count[c] = t;
    if (kScore) {
      unsigned long long ticks = 0ull;
      for (int wv = 0; wv < kAssignThreads / 64; ++wv) ticks += t_blk[wv];
      const float ps = (rs.n_req == 0u) ? 0.0f : (float)t / (float)rs.n_req;
      float pt = 0.0f;
      for (uint32_t j = 0; j < n; ++j) {
        const float inv = s2tab[j];
        if (inv >= 0.0f) pt = pt + inv;
      }
      const float pl = (t == 0u) ? 0.0f : ((float)ticks * 0x1p-20f) / (float)t;
      const float ptn = fminf(pt, a.gamma_t) / a.gamma_t;
      const float pln = fmaxf(a.gamma_l - pl, 0.0f) / a.gamma_l;
      const float sc = fmaf(a.alpha, ps, fmaf(a.beta, ptn, (1.0f - a.beta) * pln));
      if (rs.phi_s) rs.phi_s[c] = ps;
      if (rs.phi_t) rs.phi_t[c] = pt;
      if (rs.phi_l) rs.phi_l[c] = pl;
      if (rs.score) rs.score[c] = sc;
    }
  }
}

// Best candidate by score: largest score, lowest index on ties.  One block.
__global__ __launch_bounds__(1024) void score_argmax_kernel(const float* __restrict__ score,
                                                            uint32_t n_cand,
                                                            uint32_t* __restrict__ best_cand) {
  __shared__ unsigned long long best[16];
  unsigned long long key = 0ull;  // (order-preserving bits of the score << 32) | ~index
  for (uint32_t c = threadIdx.x; c < n_cand; c += blockDim.x) {
    const uint32_t b = __float_as_uint(score[c]);
    const uint32_t ord = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
    const unsigned long long kc = ((unsigned long long)ord << 32) | (unsigned long long)(~c);
    key = kc > key ? kc : key;
  }
  for (int d = 32; d >= 1; d >>= 1) {
    const unsigned long long o = __shfl_xor(key, d);
    key = o > key ? o : key;
  }
  if ((threadIdx.x & 63u) == 0u) best[threadIdx.x >> 6] = key;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (uint32_t w = 1; w < (blockDim.x >> 6); ++w) key = best[w] > key ? best[w] : key;
    *best_cand = ~(uint32_t)(key & 0xffffffffull);
  }
}

}  // namespace maaso
