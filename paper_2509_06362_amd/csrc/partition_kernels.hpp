// Kernels of the placer's outer algorithms (Sec. IV-E): the request split by SLO that opens Alg. 2,
// the bookkeeping of Alg. 1 (best score and deployment per GPU count, with its accept-while-improving
// rule along each configuration's growth path) and Alg. 2's scan over the two-way GPU partitions.
// The scoring of the deployments themselves is the sweep kernels' work; everything here is small,
// integer or comparison-only, and deterministic (maxima are taken on order-preserving integer keys).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sweep_kernels.hpp"

namespace maaso {

constexpr uint32_t kMaxGpus = 4096;       // per-GPU-count table of 64-bit keys lives in LDS
constexpr int kPartitionThreads = 1024;
constexpr uint32_t kSplitPerBlock = 4096;  // requests per block of the split kernels (4 per thread)

// binary32 -> uint32 such that a < b  <=>  order(a) < order(b) (no NaNs expected)
__device__ inline uint32_t float_order(float x) {
  const uint32_t b = __float_as_uint(x);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ inline float order_float(uint32_t o) {
  return __uint_as_float((o & 0x80000000u) ? (o & 0x7fffffffu) : ~o);
}

__device__ inline unsigned long long wave_max_u64(unsigned long long v) {
  for (int d = 32; d >= 1; d >>= 1) {
    const unsigned long long o = __shfl_xor(v, d);
    v = o > v ? o : v;
  }
  return v;
}

// Block-wide maximum of a 64-bit key, returned to every thread.  `slots` holds 16 words.
__device__ inline unsigned long long block_max_u64(unsigned long long v, unsigned long long* slots) {
  v = wave_max_u64(v);
  __syncthreads();  // slots may still be read from an earlier call
  if ((threadIdx.x & 63u) == 0u) slots[threadIdx.x >> 6] = v;
  __syncthreads();
  unsigned long long m = slots[0];
  for (uint32_t w = 1; w < (blockDim.x >> 6); ++w) m = slots[w] > m ? slots[w] : m;
  return m;
}

// ------------------------------------------------------------------------------------------------
// Alg. 1 bookkeeping
// ------------------------------------------------------------------------------------------------
constexpr int kMaxSelectLists = 4;

// Block b works on score list b: the same deployments scored against several request sets (Alg. 2
// runs Alg. 1 on R_t, on R_l and on all of R) are selected in one launch.
struct SelectArgs {
  uint32_t n_lists;
  const float* score[kMaxSelectLists];  // [n_cand] composite score of every candidate deployment
  uint32_t n_cand, i_pad;
  const uint32_t* n_inst;   // [n_cand]
  const uint8_t* tp_idx;    // [n_cand][i_pad]
  const uint32_t* tp_degree;  // [n_tp] GPUs per instance of a strategy
  uint32_t n_tp;
  const uint32_t* chain_offsets;  // [n_chains + 1] or null (every candidate on its own)
  uint32_t n_chains;
  uint32_t n_gpus;
  float* phi_star[kMaxSelectLists];     // [n_gpus + 1]
  int32_t* cand_star[kMaxSelectLists];  // [n_gpus + 1]
  uint32_t* status;
};

// GPUs a candidate occupies; 0xffffffff when one of its instances names no strategy.
__device__ inline uint32_t gpu_count(const SelectArgs& a, uint32_t c) {
  const uint32_t n = min(a.n_inst[c], a.i_pad);
  const uint8_t* tp = a.tp_idx + (size_t)c * a.i_pad;
  uint64_t k = 0;
  bool bad = false;
  for (uint32_t j = 0; j < n; ++j) {
    const uint32_t t = tp[j];
    if (t >= a.n_tp) { bad = true; continue; }
    k += a.tp_degree[t];
  }
  if (bad) { raise_status(a.status, 2u); return 0xffffffffu; }
  return k > 0xfffffffeull ? 0xfffffffeu : (uint32_t)k;
}

// One block per score list.  A chain is the growth path of one configuration in Alg. 1: its m-th candidate is the
// deployment after m + 1 additions.  A candidate is accepted when every candidate before it in the
// chain was accepted, it fits into n_gpus GPUs and its score is strictly larger than that of the
// candidate before it (0 for the first): the first failure ends the chain, as the saturated model ends
// Alg. 1's inner loop.  Phi*[k] is the largest accepted score among the deployments on exactly k GPUs,
// I*[k] its candidate (lowest index on ties: the earliest configuration keeps the entry), 0 and -1
// where nothing was accepted.
__global__ __launch_bounds__(kPartitionThreads) void ins_deploy_select_kernel(const SelectArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned long long* keys = reinterpret_cast<unsigned long long*>(smem);  // [n_gpus + 1]
  const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  const float* score = a.score[blockIdx.x];
  float* phi_star = a.phi_star[blockIdx.x];
  int32_t* cand_star = a.cand_star[blockIdx.x];
  for (uint32_t k = tid; k <= a.n_gpus; k += kPartitionThreads) keys[k] = 0ull;
  __syncthreads();

  if (a.chain_offsets == nullptr) {
    for (uint32_t c = tid; c < a.n_cand; c += kPartitionThreads) {
      const float s = score[c];
      const uint32_t k = gpu_count(a, c);
      if (s > 0.0f && k <= a.n_gpus)
        atomicMax(&keys[k], ((unsigned long long)float_order(s) << 32) | (unsigned long long)(~c));
    }
  } else {
    for (uint32_t ch = wave; ch < a.n_chains; ch += kPartitionThreads / 64) {
      const uint32_t o0 = a.chain_offsets[ch], o1 = a.chain_offsets[ch + 1];
      if (o0 > o1 || o1 > a.n_cand) {  // not a chain: flagged, ignored
        if (lane == 0) raise_status(a.status, 8u);
        continue;
      }
      bool alive = true;  // uniform over the wavefront
      for (uint32_t base = o0; base < o1 && alive; base += 64u) {
        const uint32_t c = base + lane;
        const bool in = c < o1;
        float s = 0.0f, prev = 0.0f;
        uint32_t k = 0;
        if (in) {
          s = score[c];
          prev = (c == o0) ? 0.0f : score[c - 1];
          k = gpu_count(a, c);
        }
        const bool ok = in && s > prev && k <= a.n_gpus;
        const unsigned long long bad = __ballot(in && !ok);
        const uint32_t first_bad = bad ? (uint32_t)__builtin_ctzll(bad) : 64u;
        if (in && lane < first_bad)
          atomicMax(&keys[k], ((unsigned long long)float_order(s) << 32) | (unsigned long long)(~c));
        alive = bad == 0ull;
      }
    }
  }
  lds_atomics_barrier();
  for (uint32_t k = tid; k <= a.n_gpus; k += kPartitionThreads) {
    const unsigned long long key = keys[k];
    phi_star[k] = key ? order_float((uint32_t)(key >> 32)) : 0.0f;
    cand_star[k] = key ? (int32_t)(~(uint32_t)(key & 0xffffffffull)) : -1;
  }
}

// ------------------------------------------------------------------------------------------------
// Alg. 2: scan over the partitions (g_t, g_l), g_t + g_l = n_gpus, g_l = 1 .. g_l_cap
// ------------------------------------------------------------------------------------------------
struct PartitionArgs {
  uint32_t n_gpus, g_l_cap;
  // with n_tight set (|R_t| as the split left it on the device) the cap is worked out here from
  // n_req instead: floor((n_req - *n_tight) * n_gpus / n_req), exact in 64-bit integers
  const uint32_t* n_tight;
  uint32_t n_req;
  const float* phi_t_star;     // [n_gpus + 1]
  const float* phi_l_star;     // [n_gpus + 1]
  const float* phi_h_star;     // [n_gpus + 1] or null: homogeneous deployment of all requests
  const int32_t* cand_t_star;  // [n_gpus + 1] or null
  const int32_t* cand_l_star;
  const int32_t* cand_h_star;
  uint32_t* out;    // [6] g_t, g_l, heterogeneous, k_h, cand_t, cand_l
  float* phi_opt;   // [1]
};

// One block.  The starting value is the best homogeneous score (lowest GPU count on ties; 0 without
// phi_h_star); a partition replaces it only with a strictly larger phi_t*[g_t] + phi_l*[g_l] (one
// binary32 addition), and among equal sums the smallest g_l stands, as in an ascending scan.
__global__ __launch_bounds__(kPartitionThreads) void resource_partition_kernel(const PartitionArgs a) {
  __shared__ unsigned long long slots[kPartitionThreads / 64];
  const uint32_t tid = threadIdx.x;
  unsigned long long hk = 0ull;
  if (a.phi_h_star)
    for (uint32_t k = tid; k <= a.n_gpus; k += kPartitionThreads) {
      const float v = a.phi_h_star[k];
      if (v > 0.0f) {
        const unsigned long long key = ((unsigned long long)float_order(v) << 32) | (unsigned long long)(~k);
        hk = key > hk ? key : hk;
      }
    }
  hk = block_max_u64(hk, slots);
  const float opt0 = hk ? order_float((uint32_t)(hk >> 32)) : 0.0f;
  const uint32_t k_h = hk ? ~(uint32_t)(hk & 0xffffffffull) : 0u;

  unsigned long long pk = 0ull;
  uint32_t g_l_cap = a.g_l_cap;
  if (a.n_tight) {
    const uint32_t n_t = min(*a.n_tight, a.n_req);
    g_l_cap = a.n_req == 0u ? 0u
                            : (uint32_t)(((unsigned long long)(a.n_req - n_t) * a.n_gpus) / a.n_req);
  }
  const uint32_t cap = min(g_l_cap, a.n_gpus);
  for (uint32_t gl = 1u + tid; gl <= cap; gl += kPartitionThreads) {
    const float sum = a.phi_t_star[a.n_gpus - gl] + a.phi_l_star[gl];
    if (sum > opt0) {
      const unsigned long long key = ((unsigned long long)float_order(sum) << 32) | (unsigned long long)(~gl);
      pk = key > pk ? key : pk;
    }
  }
  pk = block_max_u64(pk, slots);
  if (tid == 0) {
    if (pk) {
      const uint32_t gl = ~(uint32_t)(pk & 0xffffffffull), gt = a.n_gpus - gl;
      a.out[0] = gt; a.out[1] = gl; a.out[2] = 1u; a.out[3] = k_h;
      a.out[4] = a.cand_t_star ? (uint32_t)a.cand_t_star[gt] : 0xffffffffu;
      a.out[5] = a.cand_l_star ? (uint32_t)a.cand_l_star[gl] : 0xffffffffu;
      *a.phi_opt = order_float((uint32_t)(pk >> 32));
    } else {
      a.out[0] = k_h; a.out[1] = 0u; a.out[2] = 0u; a.out[3] = k_h;
      a.out[4] = (hk && a.cand_h_star) ? (uint32_t)a.cand_h_star[k_h] : 0xffffffffu;
      a.out[5] = 0xffffffffu;
      *a.phi_opt = opt0;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Batch-size pruning (Sec. IV-E, "Inference Batch Size Pruning"): of the batch sizes of one
// parallelism configuration keep those that are Pareto-optimal in (SLO satisfaction, latency)
// ------------------------------------------------------------------------------------------------
struct PruneArgs {
  uint32_t n_cand;
  const uint32_t* group_offsets;  // [n_groups + 1] group g = candidates [offsets[g], offsets[g + 1])
  uint32_t n_groups;
  const uint32_t* sat_count;      // [n_cand] requests whose SLO the candidate meets (more is better)
  const float* latency;           // [n_cand] its response latency (less is better)
  uint8_t* keep;                  // [n_cand] 1: retained
  uint32_t* n_kept;               // [n_groups] retained candidates of the group
  uint32_t* status;
};

constexpr int kPruneTile = 256;

// One block per group.  Candidate i goes when it meets no request's SLO, or when another candidate
// of its group is at least as good in both respects and better in one: sat_j >= sat_i and
// lat_j <= lat_i with one of them strict.  Equal candidates keep each other; a NaN latency compares
// false either way, so such a candidate neither removes another nor is removed by one.
__global__ __launch_bounds__(kPruneTile) void batch_prune_kernel(const PruneArgs a) {
  __shared__ uint32_t t_sat[kPruneTile];
  __shared__ float t_lat[kPruneTile];
  __shared__ uint32_t wave_kept[kPruneTile / 64];
  const uint32_t g = blockIdx.x, tid = threadIdx.x;
  const uint32_t o0 = a.group_offsets[g], o1 = a.group_offsets[g + 1];
  if (o0 > o1 || o1 > a.n_cand) {  // not a group: flagged, nothing written but its count
    if (tid == 0u) { raise_status(a.status, 8u); a.n_kept[g] = 0u; }
    return;
  }
  uint32_t kept = 0;
  for (uint32_t base = o0; base < o1; base += kPruneTile) {  // uniform trip count: barriers inside
    const uint32_t i = base + tid;
    const bool mine = i < o1;
    const uint32_t sat_i = mine ? a.sat_count[i] : 0u;
    const float lat_i = mine ? a.latency[i] : 0.0f;
    bool dominated = false;
    for (uint32_t jb = o0; jb < o1; jb += kPruneTile) {
      __syncthreads();
      if (jb + tid < o1) { t_sat[tid] = a.sat_count[jb + tid]; t_lat[tid] = a.latency[jb + tid]; }
      __syncthreads();
      const uint32_t n = min((uint32_t)kPruneTile, o1 - jb);
      for (uint32_t j = 0; j < n; ++j) {
        const uint32_t sat_j = t_sat[j];
        const float lat_j = t_lat[j];
        dominated |= (sat_j >= sat_i) & (lat_j <= lat_i) & ((sat_j > sat_i) | (lat_j < lat_i));
      }
    }
    const bool k = mine && sat_i != 0u && !dominated;
    if (mine) a.keep[i] = k ? 1u : 0u;
    kept += k ? 1u : 0u;
  }
  for (int d = 32; d >= 1; d >>= 1) kept += __shfl_xor(kept, d);
  if ((tid & 63u) == 0u) wave_kept[tid >> 6] = kept;
  __syncthreads();
  if (tid == 0u) {
    uint32_t t = 0;
    for (int w = 0; w < kPruneTile / 64; ++w) t += wave_kept[w];
    a.n_kept[g] = t;
  }
}

// ------------------------------------------------------------------------------------------------
// Alg. 2's first step: split the request streams by SLO class, keeping arrival order on both sides
// ------------------------------------------------------------------------------------------------
struct SplitArgs {
  uint32_t n_req;
  const uint32_t* prompt_len;
  const uint32_t* out_len;
  const uint8_t* slo_class;
  const uint32_t* arrival_ticks;  // may be null (then arrival_out is not written)
  uint32_t tight_classes;         // bit k set: class k belongs to the strict set R_t
  uint32_t n_slo;
  uint32_t* block_tight;  // [n_blocks] scratch: strict requests per block, then their exclusive prefix
  uint32_t* n_tight;      // [1]
  uint32_t* prompt_out;   // [n_req] strict requests first, relaxed ones from index *n_tight on
  uint32_t* out_len_out;
  uint8_t* class_out;
  uint32_t* arrival_out;
  uint32_t* status;
};

__device__ inline bool split_is_tight(const SplitArgs& a, uint32_t r) {
  const uint32_t k = a.slo_class[r];
  if (k >= a.n_slo) { raise_status(a.status, 1u); return false; }  // flagged; stays with the relaxed set
  return ((a.tight_classes >> k) & 1u) != 0u;
}

__global__ __launch_bounds__(kPartitionThreads) void split_count_kernel(const SplitArgs a) {
  __shared__ uint32_t wave_cnt[kPartitionThreads / 64];
  const uint32_t tid = threadIdx.x;
  const uint64_t base = (uint64_t)blockIdx.x * kSplitPerBlock;
  uint32_t cnt = 0;
#pragma unroll
  for (uint32_t i = 0; i < kSplitPerBlock / kPartitionThreads; ++i) {
    const uint64_t r = base + (uint64_t)i * kPartitionThreads + tid;
    const bool t = r < a.n_req && split_is_tight(a, (uint32_t)r);
    cnt += (uint32_t)__popcll(__ballot(t));
  }
  if ((tid & 63u) == 0u) wave_cnt[tid >> 6] = cnt;
  __syncthreads();
  if (tid == 0) {
    uint32_t s = 0;
    for (int w = 0; w < kPartitionThreads / 64; ++w) s += wave_cnt[w];
    a.block_tight[blockIdx.x] = s;
  }
}

// One block: exclusive prefix of the per-block counts in place, total to *n_tight.
__global__ __launch_bounds__(kPartitionThreads) void split_scan_kernel(uint32_t* __restrict__ block_tight,
                                                                      uint32_t n_blocks,
                                                                      uint32_t* __restrict__ n_tight) {
  __shared__ uint32_t wave_sum[kPartitionThreads / 64];
  __shared__ uint32_t carry_s;
  const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  if (tid == 0) carry_s = 0u;
  __syncthreads();
  for (uint32_t b0 = 0; b0 < n_blocks; b0 += kPartitionThreads) {
    const uint32_t b = b0 + tid;
    const uint32_t v = b < n_blocks ? block_tight[b] : 0u;
    uint32_t inc = v;  // inclusive prefix inside the wavefront
    for (int d = 1; d < 64; d <<= 1) {
      const uint32_t o = __shfl_up(inc, d);
      if (lane >= (uint32_t)d) inc += o;
    }
    if (lane == 63u) wave_sum[wave] = inc;
    __syncthreads();
    uint32_t before = carry_s;
    for (uint32_t w = 0; w < wave; ++w) before += wave_sum[w];
    if (b < n_blocks) block_tight[b] = before + inc - v;
    __syncthreads();
    if (tid == kPartitionThreads - 1) carry_s = before + inc;
    __syncthreads();
  }
  if (tid == 0) *n_tight = carry_s;
}

__global__ __launch_bounds__(kPartitionThreads) void split_scatter_kernel(const SplitArgs a) {
  constexpr uint32_t kItems = kSplitPerBlock / kPartitionThreads;  // 4
  constexpr uint32_t kGroups = kItems * (kPartitionThreads / 64);  // 64 (item, wavefront) groups
  __shared__ uint32_t grp[kGroups];  // strict requests per group, then their exclusive prefix
  const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  const uint64_t base = (uint64_t)blockIdx.x * kSplitPerBlock;
  bool tight[kItems];
  uint32_t before_in_wave[kItems];
#pragma unroll
  for (uint32_t i = 0; i < kItems; ++i) {
    const uint64_t r = base + (uint64_t)i * kPartitionThreads + tid;
    tight[i] = r < a.n_req && split_is_tight(a, (uint32_t)r);
    const unsigned long long m = __ballot(tight[i]);
    before_in_wave[i] = (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
    if (lane == 0) grp[i * (kPartitionThreads / 64) + wave] = (uint32_t)__popcll(m);
  }
  __syncthreads();
  if (wave == 0) {  // groups are in request order: item-major, wavefront-minor
    const uint32_t v = grp[lane];
    uint32_t inc = v;
    for (int d = 1; d < 64; d <<= 1) {
      const uint32_t o = __shfl_up(inc, d);
      if (lane >= (uint32_t)d) inc += o;
    }
    grp[lane] = inc - v;
  }
  __syncthreads();
  const uint32_t block_before = a.block_tight[blockIdx.x];
  const uint32_t total_tight = *a.n_tight;
#pragma unroll
  for (uint32_t i = 0; i < kItems; ++i) {
    const uint64_t r = base + (uint64_t)i * kPartitionThreads + tid;
    if (r >= a.n_req) continue;
    const uint32_t tight_before = block_before + grp[i * (kPartitionThreads / 64) + wave] + before_in_wave[i];
    const uint32_t dst = tight[i] ? tight_before : total_tight + ((uint32_t)r - tight_before);
    a.prompt_out[dst] = a.prompt_len[r];
    a.out_len_out[dst] = a.out_len[r];
    a.class_out[dst] = a.slo_class[r];
    if (a.arrival_ticks) a.arrival_out[dst] = a.arrival_ticks[r];
  }
}

}  // namespace maaso
