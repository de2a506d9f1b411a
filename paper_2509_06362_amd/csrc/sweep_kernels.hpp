// Placer sweep: SLO-satisfaction count of every candidate deployment over the whole request set
// (the evaluation of Phi_S(I', R_x) inside Alg. 1; Eq. 3).
//
// Work decomposition (gfx950, wave64):
//   * bucket_requests_kernel groups the prompt lengths by SLO class, so that every wavefront of the
//     sweep holds requests of ONE class and its per-class deadline is a scalar.
//   * sweep_kernel: a block owns a tile of requests (lanes = requests, Q requests per lane, kept in
//     registers) and walks a chunk of candidates.  For each candidate the block evaluates the
//     profile of its instances once ("stage") and leaves, per SLO class present in the block (at
//     most one per wavefront), a compact list of the instances whose between-token latency meets
//     that class's deadline in LDS.  Each wavefront then streams its class's list with broadcast
//     LDS reads: per (request, instance) one fused multiply-add (prefill), one add (queue wait)
//     and one min.
//   * A request is satisfied iff min_j ttft_j <= D_ttft over the listed instances.  This is the same
//     predicate as "largest slack >= 0": the between-token margin depends only on (class, instance)
//     and is what the list filters on; the first-token margin is >= 0 iff ttft <= D_ttft; and the
//     end-to-end margin is implied by the other two, because S*tbt + ttft <= S*D_tbt + D_ttft holds
//     in exact arithmetic and a correctly rounded fma is monotone.
//   * Counts: wave ballot + popcount, parked in one lane per candidate, flushed with one coalesced
//     integer atomic per 64 candidates per wavefront; integer sums are order-independent.
//   * sweep_finalize_kernel: ratio = count / R and the best candidate (lowest index on ties).
#pragma once

#include "device_model.hpp"

#pragma clang fp contract(off)

namespace maaso {

constexpr int kSweepThreads = 256;  // 4 wavefronts
constexpr int kWave = 64;
constexpr int kMaxSlo = 16;
constexpr int kSweepWaves = kSweepThreads / kWave;  // a block meets at most this many classes

__device__ __forceinline__ void raise_status(uint32_t* status, uint32_t bit) {
  if ((__hip_atomic_load(status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & bit) == 0u)
    atomicOr(status, bit);
}

// ---------------------------------------------------------------------------------------------
// zero the per-call accumulators
__global__ void sweep_init_kernel(uint32_t* __restrict__ sat_count, uint32_t n_cand,
                                  uint32_t* __restrict__ cls_count, uint32_t n_slo) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_cand) sat_count[i] = 0u;
  if (i < n_slo) cls_count[i] = 0u;
}

// ---------------------------------------------------------------------------------------------
// Group prompt lengths by class: lbuf[k * n_req + pos] = (float)prompt_len, pos < cls_count[k].
// The order inside a class is arbitrary (it does not affect any count).
__global__ __launch_bounds__(256) void bucket_requests_kernel(
    const uint32_t* __restrict__ prompt_len, const uint8_t* __restrict__ slo_class, uint32_t n_req,
    uint32_t n_slo, float* __restrict__ lbuf, uint32_t* __restrict__ cls_count,
    uint32_t* __restrict__ status) {
  __shared__ uint32_t blk_cnt[kMaxSlo];
  __shared__ uint32_t blk_base[kMaxSlo];
  constexpr int kPer = 4;
  const uint32_t tile = blockIdx.x * (256u * kPer);
  if (threadIdx.x < kMaxSlo) blk_cnt[threadIdx.x] = 0u;
  __syncthreads();
  uint32_t k[kPer], rank[kPer];
  float L[kPer];
#pragma unroll
  for (int u = 0; u < kPer; ++u) {
    const uint32_t r = tile + u * 256u + threadIdx.x;
    k[u] = 0xffffffffu;
    if (r < n_req) {
      const uint32_t c = slo_class[r];
      L[u] = (float)prompt_len[r];
      if (c < n_slo) {
        k[u] = c;
        rank[u] = atomicAdd(&blk_cnt[c], 1u);
      } else {
        raise_status(status, 1u);
      }
    }
  }
  __syncthreads();
  if (threadIdx.x < n_slo) {
    const uint32_t n = blk_cnt[threadIdx.x];
    blk_base[threadIdx.x] = n ? atomicAdd(&cls_count[threadIdx.x], n) : 0u;
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < kPer; ++u)
    if (k[u] != 0xffffffffu) lbuf[(size_t)k[u] * n_req + blk_base[k[u]] + rank[u]] = L[u];
}

// ---------------------------------------------------------------------------------------------
struct SweepArgs {
  const float* tab;  // three tables back to back, `cells` entries each
  uint32_t cells;
  ModelParams mp;
  uint32_t n_slo;
  float d_ttft[kMaxSlo];
  float d_tbt[kMaxSlo];
  uint32_t n_cand, i_pad;
  const uint32_t* n_inst;
  const uint8_t* tp_idx;
  const uint16_t* max_batch;
  const int32_t* occ;
  const uint64_t* q_ticks;
  const float* lbuf;          // [n_slo][n_req] prompt lengths grouped by class
  const uint32_t* cls_count;  // [n_slo]
  uint32_t n_req;
  uint32_t group;         // G: candidates staged together (G * i_pad <= 256)
  uint32_t chunk;         // candidates per block, a multiple of G
  uint32_t n_req_blocks;  // request tiles of 4 wavefronts
  uint32_t n_chunks;
  uint32_t* sat_count;
  uint32_t* status;
};

struct RawInstance {
  uint32_t tp, B;
  int32_t occ;
  uint64_t q;
  bool valid;
};

template <int Q>
__global__ __launch_bounds__(kSweepThreads) void sweep_kernel(const SweepArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ int wave_class[kSweepWaves];
  // LDS: tables | instance lists [2][G][4][i_pad] float4 | list lengths [3][G][4]
  // (4 = class slots: one per wavefront of the block at most)
  float* tab = reinterpret_cast<float*>(smem);
  const uint32_t tab_bytes = (3u * a.cells * 4u + 15u) & ~15u;
  float4* lists = reinterpret_cast<float4*>(smem + tab_bytes);
  const uint32_t K = a.n_slo, G = a.group, I = a.i_pad;
  constexpr uint32_t NS = kSweepWaves;
  const uint32_t list_stride = G * NS * I;  // float4 per buffer
  uint32_t* lens = reinterpret_cast<uint32_t*>(lists + 2u * list_stride);
  const uint32_t lens_stride = G * NS;

  // XCD-aware block mapping: hardware deals consecutive blocks round-robin to the 8 XCDs, so the
  // blocks that share one chunk of candidates are given ids that are congruent modulo 8 and meet in
  // one XCD's L2.
  const uint32_t bid = blockIdx.x;
  const uint32_t xcd = bid & 7u, slot = bid >> 3;
  const uint32_t chunk_id = xcd + 8u * (slot / a.n_req_blocks);
  const uint32_t req_block = slot % a.n_req_blocks;
  if (chunk_id >= a.n_chunks) return;

  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & 63u;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  // Which class tile does this wavefront own?  Tiles of 64*Q requests, class after class.
  constexpr uint32_t kTile = kWave * Q;
  const uint32_t my_tile = req_block * 4u + wave;
  uint32_t k_w = 0, off = 0, n_k = 0;
  bool active = false;
  {
    uint32_t first = 0;
    for (uint32_t k = 0; k < K; ++k) {
      const uint32_t n = a.cls_count[k];
      const uint32_t tiles = (n + kTile - 1u) / kTile;
      if (!active && my_tile < first + tiles) {
        active = true; k_w = k; off = (my_tile - first) * kTile; n_k = n;
      }
      first += tiles;
    }
    if (req_block * 4u >= first) return;  // the whole block lies past the last tile
  }

  for (uint32_t i = tid; i < 3u * a.cells; i += kSweepThreads) tab[i] = a.tab[i];
  for (uint32_t i = tid; i < 3u * lens_stride; i += kSweepThreads) lens[i] = 0u;
  if (lane == 0u) wave_class[wave] = active ? (int)k_w : -1;
  __syncthreads();
  // the distinct classes of the block's wavefronts, and this wavefront's slot among them
  uint32_t n_slots = 0, my_slot = 0;
  uint32_t slot_class[NS];
#pragma unroll
  for (uint32_t wv = 0; wv < NS; ++wv) {
    slot_class[wv] = 0u;
  }
#pragma unroll
  for (uint32_t wv = 0; wv < NS; ++wv) {
    const int kk = wave_class[wv];
    if (kk < 0) continue;
    bool found = false;
#pragma unroll
    for (uint32_t sidx = 0; sidx < NS; ++sidx)
      if (sidx < n_slots && slot_class[sidx] == (uint32_t)kk) {
        found = true;
        if (wv == wave) my_slot = sidx;
      }
    if (!found) {
#pragma unroll
      for (uint32_t sidx = 0; sidx < NS; ++sidx)
        if (sidx == n_slots) slot_class[sidx] = (uint32_t)kk;
      if (wv == wave) my_slot = n_slots;
      ++n_slots;
    }
  }

  float L[Q];
  uint64_t vmask[Q];
#pragma unroll
  for (int q = 0; q < Q; ++q) {
    const uint32_t idx = off + q * kWave + lane;
    const bool ok = active && idx < n_k;
    L[q] = ok ? a.lbuf[(size_t)k_w * a.n_req + idx] : 0.0f;
    vmask[q] = __ballot(ok);
  }
  const float Dt = a.d_ttft[k_w];

  const uint32_t c_begin = chunk_id * a.chunk;
  const uint32_t c_end = min(c_begin + a.chunk, a.n_cand);
  const uint32_t n_groups = (c_end - c_begin + G - 1u) / G;
  const uint32_t cl = tid / I, j = tid - cl * I;  // staging slot of this thread

  auto load_raw = [&](uint32_t gi) {
    RawInstance r;
    const uint32_t c = c_begin + gi * G + cl;
    r.valid = cl < G && c < c_end;
    if (r.valid) r.valid = j < a.n_inst[c];
    if (r.valid) {
      const size_t s = (size_t)c * I + j;
      r.tp = a.tp_idx[s]; r.B = a.max_batch[s]; r.occ = a.occ[s]; r.q = a.q_ticks[s];
    }
    return r;
  };
  auto commit = [&](const RawInstance& r, uint32_t gi) {
    if (!r.valid) return;
    Staged s;
    if (!stage_instance(tab, a.cells, a.mp, r.tp, r.B, r.occ, r.q, s)) {
      raise_status(a.status, 2u);
      return;
    }
    float4* lst = lists + (gi & 1u) * list_stride + cl * NS * I;
    uint32_t* len = lens + (gi % 3u) * lens_stride + cl * NS;
    const float4 rec = make_float4(s.p, s.a, s.wait, 0.0f);
#pragma unroll
    for (uint32_t sidx = 0; sidx < NS; ++sidx)
      if (sidx < n_slots && s.tbt <= a.d_tbt[slot_class[sidx]])
        lst[sidx * I + atomicAdd(&len[sidx], 1u)] = rec;
  };

  __syncthreads();
  commit(load_raw(0), 0);
  __syncthreads();

  uint32_t acc = 0;  // lane l holds the count of candidate (flush base + l)
  uint32_t flush_base = c_begin;
  for (uint32_t gi = 0; gi < n_groups; ++gi) {
    RawInstance nxt;
    nxt.valid = false;
    if (gi + 1u < n_groups) nxt = load_raw(gi + 1u);

    if (active) {
      const float4* gl = lists + (gi & 1u) * list_stride;
      const uint32_t* glen = lens + (gi % 3u) * lens_stride;
      const uint32_t g_cands = min(G, c_end - (c_begin + gi * G));
      for (uint32_t g = 0; g < g_cands; ++g) {
        const uint32_t n = __builtin_amdgcn_readfirstlane(glen[g * NS + my_slot]);
        const float4* lst = gl + (g * NS + my_slot) * I;
        float m[Q];
#pragma unroll
        for (int q = 0; q < Q; ++q) m[q] = INFINITY;
        for (uint32_t i = 0; i < n; ++i) {
          const float4 r = lst[i];
#pragma unroll
          for (int q = 0; q < Q; ++q) m[q] = fminf(m[q], r.z + fmaf(r.x, L[q], r.y));
        }
        uint32_t cnt = 0;
#pragma unroll
        for (int q = 0; q < Q; ++q) cnt += (uint32_t)__popcll(__ballot(m[q] <= Dt) & vmask[q]);
        const uint32_t c = c_begin + gi * G + g;
        acc = (lane == c - flush_base) ? cnt : acc;
        if (c - flush_base == 63u) {
          atomicAdd(&a.sat_count[flush_base + lane], acc);
          flush_base += 64u;
          acc = 0;
        }
      }
    }

    if (gi + 1u < n_groups) commit(nxt, gi + 1u);
    // the length slots of group gi+2 were last read while scoring group gi-1
    for (uint32_t i = tid; i < lens_stride; i += kSweepThreads) lens[((gi + 2u) % 3u) * lens_stride + i] = 0u;
    __syncthreads();
  }
  if (active && flush_base + lane < c_end) atomicAdd(&a.sat_count[flush_base + lane], acc);
}

// ---------------------------------------------------------------------------------------------
// ratio[c] = count[c] / R and the best candidate: largest count, lowest index on ties (Alg. 1 keeps
// the best-scoring deployment).  One block.
__global__ __launch_bounds__(1024) void sweep_finalize_kernel(const uint32_t* __restrict__ sat_count,
                                                              uint32_t n_cand, uint32_t n_req,
                                                              float* __restrict__ sat_ratio,
                                                              uint32_t* __restrict__ best_cand) {
  __shared__ unsigned long long best[16];
  const float fr = (float)n_req;
  unsigned long long key = 0ull;  // (count << 32) | ~index: max key = max count, then min index
  for (uint32_t c = threadIdx.x; c < n_cand; c += blockDim.x) {
    const uint32_t n = sat_count[c];
    if (sat_ratio) sat_ratio[c] = n_req ? (float)n / fr : 0.0f;
    const unsigned long long kc = ((unsigned long long)n << 32) | (unsigned long long)(~c);
    key = kc > key ? kc : key;
  }
  for (int d = 32; d >= 1; d >>= 1) {
    const unsigned long long o = __shfl_xor(key, d);
    key = o > key ? o : key;
  }
  if ((threadIdx.x & 63u) == 0u) best[threadIdx.x >> 6] = key;
  __syncthreads();
  if (threadIdx.x == 0 && best_cand) {
    for (uint32_t w = 1; w < (blockDim.x >> 6); ++w) key = best[w] > key ? best[w] : key;
    *best_cand = ~(uint32_t)(key & 0xffffffffull);
  }
}

}  // namespace maaso
