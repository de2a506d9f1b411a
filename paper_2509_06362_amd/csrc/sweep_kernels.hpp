// Placer sweep: SLO-satisfaction count of every candidate deployment over the whole request set
// (the evaluation of Phi_S(I', R_x) inside Alg. 1; Eq. 3).
//
// Three launches (gfx950, wave64):
//   1. sweep_prep_kernel - two jobs in one grid.  "bucket" blocks group the prompt lengths by SLO
//      class, so that every block of the sweep holds requests of ONE class and its deadlines are
//      scalars.  "stage" blocks evaluate the profile of every instance slot once (tables staged in
//      LDS; Eq. 1 row, occupancy penalty, queue wait) and leave a 16-byte record {p, a, wait, tbt}
//      per slot; padding slots and slots outside the tables get tbt = +inf and are never listed.
//   2. sweep_kernel - persistent blocks.  A block owns a tile of 256*Q requests of one class (lanes =
//      requests, Q per lane, in registers) and pulls work items - groups of G candidates - from a
//      queue.  For each group the block filters the records on the between-token deadline of its
//      class into compact per-candidate lists in LDS (double-buffered, loads for the next group are
//      issued before the current group is scored, one barrier per group), then every wavefront
//      streams the lists with broadcast LDS reads, two records per trip: per (request, instance) one
//      fused multiply-add (prefill), one add (queue wait) and half of a three-input min.  Records
//      whose queue wait is exactly zero are listed apart and walked without the add (0 + x = x).
//   3. sweep_finalize_kernel - ratio = count / R and the best candidate (lowest index on ties).
//
// A request is satisfied iff min_j ttft_j <= D_ttft over the listed instances.  This is the same
// predicate as "largest slack >= 0": the between-token margin depends only on (class, instance) and
// is what the list filters on; the first-token margin is >= 0 iff ttft <= D_ttft; and the end-to-end
// margin is implied by the other two, because S*tbt + ttft <= S*D_tbt + D_ttft holds in exact
// arithmetic and a correctly rounded fma is monotone.
//
// Counts: wave ballot + popcount (scalar unit), parked in one lane per candidate, summed over the
// block's four wavefronts in LDS, then one integer atomic per candidate per block; integer sums are
// order-independent, so the result does not depend on scheduling.
//
// Queues are XCD-aware: hardware deals consecutive blocks round-robin to the 8 XCDs, and the queue of
// a block with id b only holds the groups g with g % 8 == b % 8, so a group's records are read into
// one XCD's L2 only and are shared there by the blocks of all request tiles.
#pragma once

#include "device_model.hpp"

#pragma clang fp contract(off)

namespace maaso {

constexpr int kSweepThreads = 256;  // 4 wavefronts
constexpr int kWave = 64;
constexpr int kMaxSlo = 16;
constexpr int kSweepWaves = kSweepThreads / kWave;
constexpr int kSlotsPerThread = 2;                            // instance slots a thread files per group
constexpr int kGroupSlots = kSweepThreads * kSlotsPerThread;  // 512 records per LDS buffer
constexpr int kMaxGroup = 64;                                 // candidates per group (one lane each)
constexpr int kStageSlotsPerBlock = 512;   // two per thread: short blocks, their loads overlap
constexpr int kBucketPerBlock = 1024;

// Barrier that publishes LDS atomics.  For atomics whose result is unused the compiler emits no wait
// on the LDS counter before the s_barrier of __syncthreads(), and on gfx950 a wavefront reading behind
// that barrier can then see the location without some of the additions (observed as run-to-run
// differences in the per-window admission counts).  Waiting for this wavefront's outstanding LDS
// operations (s_waitcnt lgkmcnt(0), all other counters left at their maxima) before the barrier
// closes that window.  Atomics whose result is used need nothing: the use already waits.
__device__ __forceinline__ void lds_atomics_barrier() {
  __builtin_amdgcn_s_waitcnt(0xc07f);
  __syncthreads();
}

__device__ __forceinline__ void raise_status(uint32_t* status, uint32_t bit) {
  if ((__hip_atomic_load(status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & bit) == 0u)
    atomicOr(status, bit);
}

// Fill of a few 32-bit words (a kernel, not a memset node, so that a caller may capture the call in a
// HIP graph).
__global__ void fill_u32_kernel(uint32_t* p, uint32_t n, uint32_t v) {
  for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = v;
}

// v_min_f32 on values that are never NaN (the compiler's fminf adds a canonicalising v_max first).
__device__ __forceinline__ float min_no_nan(float x, float y) {
  float r;
  asm("v_min_f32 %0, %1, %2" : "=v"(r) : "v"(x), "v"(y));
  return r;
}

// min(x, y, z) in one instruction slot.
__device__ __forceinline__ float min3_no_nan(float x, float y, float z) {
  float r;
  asm("v_min3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "v"(y), "v"(z));
  return r;
}

// v[lane] = value for a uniform value and lane index (both scalar).  The instruction reads one scalar
// register beside M0, so the lane index travels through M0, whose content is put back afterwards
// (the compiler does not track M0 across an asm statement).
__device__ __forceinline__ void write_lane(uint32_t& v, uint32_t value, uint32_t lane_index) {
  uint32_t keep;
  asm("s_mov_b32 %1, m0\n\ts_mov_b32 m0, %3\n\tv_writelane_b32 %0, %2, m0\n\ts_mov_b32 m0, %1"
      : "+v"(v), "=&s"(keep)
      : "s"(value), "s"(lane_index));
}

__device__ __forceinline__ float max_no_nan(float x, float y) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(x), "v"(y));
  return r;
}

// First-token latency of a lane's Q requests on one listed instance: prefill (fused), plus the queue
// wait where the instance has one.  A record is {p, a, wait, tbt}.
template <int Q, bool kWait>
__device__ __forceinline__ void fold_first(float (&m)[Q], const float (&L)[Q], const float4* p) {
  const float4 r = p[0];
#pragma unroll
  for (int q = 0; q < Q; ++q) m[q] = kWait ? r.z + fmaf(r.x, L[q], r.y) : fmaf(r.x, L[q], r.y);
}

template <int Q, bool kWait>
__device__ __forceinline__ void fold_one(float (&m)[Q], const float (&L)[Q], const float4* p) {
  const float4 r = p[0];
#pragma unroll
  for (int q = 0; q < Q; ++q)
    m[q] = min_no_nan(m[q], kWait ? r.z + fmaf(r.x, L[q], r.y) : fmaf(r.x, L[q], r.y));
}

// Two records folded into the running minimum with ONE three-input minimum per request: per request
// fma, fma (each followed by the add of the queue wait where there is one), min3.  The sequence is
// fixed here instead of being left to the compiler's scheduler: two requests are interleaved so that
// no instruction reads the result of the one just before it, and four temporaries serve all requests
// (scheduled freely, the 2*Q products of a pair were all formed first, and with several pairs
// unrolled the kernel spilled).  v_fma_f32 / v_add_f32 / v_min3_f32 are the instructions the compiler
// emits for fmaf, + and a NaN-free minimum, so the values are the same bit for bit.
// Operands: %0-%(N-1) running minima, then 4 temporaries, then N prompt lengths, then p, a of the two
// records (and their waits).
#define MAASO_FOLD2(MA, MB, LA, LB, T0, T1, T2, T3, RX, RY, UX, UY)                                  \
  "v_fma_f32 " T0 ", " RX ", " LA ", " RY "\n\t" "v_fma_f32 " T1 ", " UX ", " LA ", " UY "\n\t"        \
  "v_fma_f32 " T2 ", " RX ", " LB ", " RY "\n\t" "v_fma_f32 " T3 ", " UX ", " LB ", " UY "\n\t"        \
  "v_min3_f32 " MA ", " MA ", " T0 ", " T1 "\n\t" "v_min3_f32 " MB ", " MB ", " T2 ", " T3 "\n\t"
#define MAASO_FOLD2W(MA, MB, LA, LB, T0, T1, T2, T3, RX, RY, UX, UY, RZ, UZ)                         \
  "v_fma_f32 " T0 ", " RX ", " LA ", " RY "\n\t" "v_fma_f32 " T1 ", " UX ", " LA ", " UY "\n\t"        \
  "v_fma_f32 " T2 ", " RX ", " LB ", " RY "\n\t" "v_fma_f32 " T3 ", " UX ", " LB ", " UY "\n\t"        \
  "v_add_f32 " T0 ", " RZ ", " T0 "\n\t" "v_add_f32 " T1 ", " UZ ", " T1 "\n\t"                       \
  "v_add_f32 " T2 ", " RZ ", " T2 "\n\t" "v_add_f32 " T3 ", " UZ ", " T3 "\n\t"                       \
  "v_min3_f32 " MA ", " MA ", " T0 ", " T1 "\n\t" "v_min3_f32 " MB ", " MB ", " T2 ", " T3 "\n\t"

template <bool kWait>
__device__ __forceinline__ void fold_pair_n(float (&m)[2], const float (&L)[2], const float4& r,
                                            const float4& u) {
  float t0, t1, t2, t3;
  if (kWait)
    asm(MAASO_FOLD2W("%0", "%1", "%6", "%7", "%2", "%3", "%4", "%5", "%8", "%9", "%10", "%11", "%12", "%13")
        : "+v"(m[0]), "+v"(m[1]), "=&v"(t0), "=&v"(t1), "=&v"(t2), "=&v"(t3)
        : "v"(L[0]), "v"(L[1]), "v"(r.x), "v"(r.y), "v"(u.x), "v"(u.y), "v"(r.z), "v"(u.z));
  else
    asm(MAASO_FOLD2("%0", "%1", "%6", "%7", "%2", "%3", "%4", "%5", "%8", "%9", "%10", "%11")
        : "+v"(m[0]), "+v"(m[1]), "=&v"(t0), "=&v"(t1), "=&v"(t2), "=&v"(t3)
        : "v"(L[0]), "v"(L[1]), "v"(r.x), "v"(r.y), "v"(u.x), "v"(u.y));
}

template <bool kWait>
__device__ __forceinline__ void fold_pair_n(float (&m)[4], const float (&L)[4], const float4& r,
                                            const float4& u) {
  float t0, t1, t2, t3;
  if (kWait)
    asm(MAASO_FOLD2W("%0", "%1", "%8", "%9", "%4", "%5", "%6", "%7", "%12", "%13", "%14", "%15", "%16", "%17")
        MAASO_FOLD2W("%2", "%3", "%10", "%11", "%4", "%5", "%6", "%7", "%12", "%13", "%14", "%15", "%16", "%17")
        : "+v"(m[0]), "+v"(m[1]), "+v"(m[2]), "+v"(m[3]), "=&v"(t0), "=&v"(t1), "=&v"(t2), "=&v"(t3)
        : "v"(L[0]), "v"(L[1]), "v"(L[2]), "v"(L[3]), "v"(r.x), "v"(r.y), "v"(u.x), "v"(u.y), "v"(r.z),
          "v"(u.z));
  else
    asm(MAASO_FOLD2("%0", "%1", "%8", "%9", "%4", "%5", "%6", "%7", "%12", "%13", "%14", "%15")
        MAASO_FOLD2("%2", "%3", "%10", "%11", "%4", "%5", "%6", "%7", "%12", "%13", "%14", "%15")
        : "+v"(m[0]), "+v"(m[1]), "+v"(m[2]), "+v"(m[3]), "=&v"(t0), "=&v"(t1), "=&v"(t2), "=&v"(t3)
        : "v"(L[0]), "v"(L[1]), "v"(L[2]), "v"(L[3]), "v"(r.x), "v"(r.y), "v"(u.x), "v"(u.y));
}

template <bool kWait>
__device__ __forceinline__ void fold_pair_n(float (&m)[8], const float (&L)[8], const float4& r,
                                            const float4& u) {
  float t0, t1, t2, t3;
  if (kWait)
    asm(MAASO_FOLD2W("%0", "%1", "%12", "%13", "%8", "%9", "%10", "%11", "%20", "%21", "%22", "%23", "%24", "%25")
        MAASO_FOLD2W("%2", "%3", "%14", "%15", "%8", "%9", "%10", "%11", "%20", "%21", "%22", "%23", "%24", "%25")
        MAASO_FOLD2W("%4", "%5", "%16", "%17", "%8", "%9", "%10", "%11", "%20", "%21", "%22", "%23", "%24", "%25")
        MAASO_FOLD2W("%6", "%7", "%18", "%19", "%8", "%9", "%10", "%11", "%20", "%21", "%22", "%23", "%24", "%25")
        : "+v"(m[0]), "+v"(m[1]), "+v"(m[2]), "+v"(m[3]), "+v"(m[4]), "+v"(m[5]), "+v"(m[6]), "+v"(m[7]),
          "=&v"(t0), "=&v"(t1), "=&v"(t2), "=&v"(t3)
        : "v"(L[0]), "v"(L[1]), "v"(L[2]), "v"(L[3]), "v"(L[4]), "v"(L[5]), "v"(L[6]), "v"(L[7]), "v"(r.x),
          "v"(r.y), "v"(u.x), "v"(u.y), "v"(r.z), "v"(u.z));
  else
    asm(MAASO_FOLD2("%0", "%1", "%12", "%13", "%8", "%9", "%10", "%11", "%20", "%21", "%22", "%23")
        MAASO_FOLD2("%2", "%3", "%14", "%15", "%8", "%9", "%10", "%11", "%20", "%21", "%22", "%23")
        MAASO_FOLD2("%4", "%5", "%16", "%17", "%8", "%9", "%10", "%11", "%20", "%21", "%22", "%23")
        MAASO_FOLD2("%6", "%7", "%18", "%19", "%8", "%9", "%10", "%11", "%20", "%21", "%22", "%23")
        : "+v"(m[0]), "+v"(m[1]), "+v"(m[2]), "+v"(m[3]), "+v"(m[4]), "+v"(m[5]), "+v"(m[6]), "+v"(m[7]),
          "=&v"(t0), "=&v"(t1), "=&v"(t2), "=&v"(t3)
        : "v"(L[0]), "v"(L[1]), "v"(L[2]), "v"(L[3]), "v"(L[4]), "v"(L[5]), "v"(L[6]), "v"(L[7]), "v"(r.x),
          "v"(r.y), "v"(u.x), "v"(u.y));
}

template <int Q, bool kWait>
__device__ __forceinline__ void fold_pair(float (&m)[Q], const float (&L)[Q], const float4* p) {
  static_assert(Q == 2 || Q == 4 || Q == 8 || Q == 16, "requests per lane");
  const float4 r = p[0];
  const float4 u = p[1];
  if constexpr (Q == 16) {  // an asm statement takes at most 30 operands: two halves of eight requests
    fold_pair_n<kWait>(reinterpret_cast<float (&)[8]>(m[0]), reinterpret_cast<const float (&)[8]>(L[0]), r, u);
    fold_pair_n<kWait>(reinterpret_cast<float (&)[8]>(m[8]), reinterpret_cast<const float (&)[8]>(L[8]), r, u);
  } else {
    fold_pair_n<kWait>(m, L, r, u);
  }
}

// Smallest first-token latency over a list of n > 0 records (uniform n, LDS list).  `fresh`: m holds
// nothing yet and is initialised from the list's first record(s).  After an odd record (or the
// initialising one or two) the list is walked in pairs: blocks of eight pairs (four with 16 requests
// per lane) in a loop, then the rest in straight-line pieces of four, two and one pairs - constant
// LDS offsets inside a piece, so its reads are issued ahead of the arithmetic, and next to nothing is
// spent on loop control for the short lists of typical candidate deployments.
template <int Q, bool kWait>
__device__ __forceinline__ void walk_list(float (&m)[Q], const float (&L)[Q], const float4* p,
                                          uint32_t n, bool fresh) {
  if (fresh) {
    if (n & 1u) {
      fold_first<Q, kWait>(m, L, p);
      p += 1;
    } else {
      fold_first<Q, kWait>(m, L, p);
      fold_one<Q, kWait>(m, L, p + 1);
      p += 2;
    }
    n = (n - 1u) >> 1;
  } else {
    if (n & 1u) {
      fold_one<Q, kWait>(m, L, p);
      p += 1;
    }
    n >>= 1;
  }
  // pairs per block of the loop: the records of a block are all in flight at once (three registers
  // each), so with 16 requests per lane a block is four pairs
  constexpr uint32_t kBlock = Q <= 8 ? 8u : 4u;
  for (; n >= kBlock; n -= kBlock, p += 2u * kBlock) {
#pragma unroll
    for (uint32_t k = 0; k < kBlock; ++k) fold_pair<Q, kWait>(m, L, p + 2u * k);
  }
  // what is left of a block, by the binary digits of its pair count: straight-line pieces of four,
  // two and one pairs behind plain uniform branches
  if (kBlock > 4u && (n & 4u)) {
#pragma unroll
    for (uint32_t k = 0; k < 4u; ++k) fold_pair<Q, kWait>(m, L, p + 2u * k);
    p += 8;
  }
  if (n & 2u) {
    fold_pair<Q, kWait>(m, L, p);
    fold_pair<Q, kWait>(m, L, p + 2);
    p += 4;
  }
  if (n & 1u) fold_pair<Q, kWait>(m, L, p);
}

// ---------------------------------------------------------------------------------------------
struct PrepArgs {
  // bucket job
  const uint32_t* prompt_len;
  const uint8_t* slo_class;
  uint32_t n_req, n_slo;
  float* lbuf;          // [n_slo][n_req] prompt lengths (as float) grouped by class, any order inside
  uint32_t* cls_count;  // [n_slo], zero on entry
  uint32_t n_bucket_blocks;
  // stage job
  const float* tab;  // three tables back to back, `cells` entries each
  uint32_t cells;
  ModelParams mp;
  uint32_t n_cand, i_pad;
  const uint32_t* n_inst;
  const uint8_t* tp_idx;
  const uint16_t* max_batch;
  const int32_t* occ;
  const uint64_t* q_ticks;
  float4* recs;  // [n_cand * i_pad] {p, a, wait, tbt}
  // per-call accumulators to clear
  uint32_t* sat_count;  // [n_cand]
  uint32_t* queues;     // [n_queues]
  uint32_t n_queues;  // words to clear: queue heads and evaluated-pair words
  uint32_t* status;
};

__global__ __launch_bounds__(256) void sweep_prep_kernel(const PrepArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  const uint32_t tid = threadIdx.x;
  if (blockIdx.x < a.n_bucket_blocks) {
    // ---- bucket: lbuf[k * n_req + pos] = (float)prompt_len, pos < cls_count[k]
    uint32_t* blk_cnt = reinterpret_cast<uint32_t*>(smem);
    uint32_t* blk_base = blk_cnt + kMaxSlo;
    constexpr int kPer = kBucketPerBlock / 256;
    const uint32_t tile = blockIdx.x * (uint32_t)kBucketPerBlock;
    if (tid < kMaxSlo) blk_cnt[tid] = 0u;
    __syncthreads();
    uint32_t k[kPer], rank[kPer];
    float L[kPer];
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
      const uint32_t r = tile + u * 256u + tid;
      k[u] = 0xffffffffu;
      rank[u] = 0u;
      L[u] = 0.0f;
      if (r < a.n_req) {
        const uint32_t c = a.slo_class[r];
        L[u] = (float)a.prompt_len[r];
        if (c < a.n_slo) {
          k[u] = c;
          rank[u] = atomicAdd(&blk_cnt[c], 1u);
        } else {
          raise_status(a.status, 1u);
        }
      }
    }
    __syncthreads();
    if (tid < a.n_slo) {
      const uint32_t n = blk_cnt[tid];
      blk_base[tid] = n ? atomicAdd(&a.cls_count[tid], n) : 0u;
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kPer; ++u)
      if (k[u] != 0xffffffffu) a.lbuf[(size_t)k[u] * a.n_req + blk_base[k[u]] + rank[u]] = L[u];
    return;
  }
  // ---- stage: one record per instance slot, tables read from LDS
  float* tab = reinterpret_cast<float*>(smem);
  for (uint32_t i = tid; i < 3u * a.cells; i += 256u) tab[i] = a.tab[i];
  const uint32_t sb = blockIdx.x - a.n_bucket_blocks;
  {  // queue heads, then the per-block words that count evaluated pairs: every stage block clears a slice
    const uint32_t n_stage = gridDim.x - a.n_bucket_blocks;
    for (uint32_t i = sb * 256u + tid; i < a.n_queues; i += n_stage * 256u) a.queues[i] = 0u;
  }
  __syncthreads();
  const uint64_t n_slots = (uint64_t)a.n_cand * a.i_pad;
  const uint64_t base = (uint64_t)sb * kStageSlotsPerBlock;
  constexpr int kPerThread = kStageSlotsPerBlock / 256;
  // all loads first, so that their latencies overlap
  uint32_t tp[kPerThread], B[kPerThread], c_of[kPerThread];
  int32_t occ[kPerThread];
  uint64_t q[kPerThread];
  bool live[kPerThread], valid[kPerThread];
#pragma unroll
  for (int u = 0; u < kPerThread; ++u) {
    const uint64_t s = base + (uint64_t)u * 256u + tid;
    live[u] = s < n_slots;
    valid[u] = false;
    tp[u] = 0; B[u] = 1; occ[u] = 0; q[u] = 0; c_of[u] = 0;
    if (live[u]) {
      const uint32_t c = (uint32_t)(s / a.i_pad);
      const uint32_t j = (uint32_t)(s - (uint64_t)c * a.i_pad);
      c_of[u] = c;
      if (j == 0u) a.sat_count[c] = 0u;
      valid[u] = j < a.n_inst[c];
      tp[u] = a.tp_idx[s]; B[u] = a.max_batch[s]; occ[u] = a.occ[s]; q[u] = a.q_ticks[s];
    }
  }
#pragma unroll
  for (int u = 0; u < kPerThread; ++u) {
    if (!live[u]) continue;
    const uint64_t s = base + (uint64_t)u * 256u + tid;
    float4 rec = make_float4(0.0f, 0.0f, INFINITY, INFINITY);  // absent: never listed
    if (valid[u]) {
      Staged st;
      if (stage_instance(tab, a.cells, a.mp, tp[u], B[u], occ[u], q[u], st))
        rec = make_float4(st.p, st.a, st.wait, st.tbt);
      else
        raise_status(a.status, 2u);
    }
    a.recs[s] = rec;
  }
}

// ---------------------------------------------------------------------------------------------
struct SweepArgs {
  uint32_t n_slo;
  float d_ttft[kMaxSlo];
  float d_tbt[kMaxSlo];
  uint32_t n_cand, i_pad;
  const float4* recs;         // [n_cand * i_pad] staged records
  const float* lbuf;          // [n_slo][n_req]
  const uint32_t* cls_count;  // [n_slo]
  uint32_t n_req;
  uint32_t group;    // G: candidates per work item, G * i_pad <= kGroupSlots, G <= kMaxGroup
  uint32_t n_items;  // ceil(n_cand / G)
  uint32_t nrb_max;  // request-tile slots of the grid (>= tiles that exist)
  uint32_t* queues;  // [nrb_max][8] next position of each (request tile, XCD) queue
  uint32_t static_blocks;  // blocks (a multiple of 8) resident at the kernel's start: they take their
                           // first two items by rank instead of from the queue
  uint32_t* sat_count;
  unsigned long long* evaluated;  // [2][gridDim.x] per block: (request, instance) pairs that reached
                                  // the latency loop (zero on entry; summed by the finalize kernel)
};

template <int Q>
__device__ __forceinline__ void sweep_body(const SweepArgs& a) {
  __shared__ float4 lists[2][kGroupSlots];
  __shared__ uint32_t lens[3][2][kMaxGroup];  // [buffer][0: records without a wait, 1: with][candidate]
  __shared__ uint32_t blk_cnt[2][kSweepWaves][kMaxGroup];
  __shared__ uint32_t items[2];

  const uint32_t tid = threadIdx.x;
  const uint32_t lane = tid & 63u;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t xcd = blockIdx.x & 7u;
  const uint32_t slot = blockIdx.x >> 3;  // this block's place among the blocks of its XCD
  const uint32_t rb = slot % a.nrb_max;
  const uint32_t G = a.group, I = a.i_pad;

  // Work items of this block.  Its (request tile, XCD) queue holds the groups xcd, xcd + 8, ...  The
  // blocks that are resident when the kernel starts (the first a.static_blocks of the grid) take
  // their first two items by their rank among the queue's blocks - no memory access, so the records
  // of the first item are requested before anything else; every further item, and every item of a
  // block that starts later, comes from the queue's counter.
  uint32_t* queue = a.queues + (size_t)rb * 8u + xcd;
  const uint32_t rank = slot / a.nrb_max;
  const uint32_t static_slots = a.static_blocks >> 3;
  const uint32_t n_static = static_slots > rb ? (static_slots - 1u - rb) / a.nrb_max + 1u : 0u;  // on this queue
  const uint32_t dynamic_base = 2u * n_static;
  uint32_t cur, nxt;
  if (rank < n_static) {
    cur = xcd + 8u * rank;
    nxt = xcd + 8u * (rank + n_static);
  } else {
    if (tid == 0u) {
      items[0] = xcd + 8u * (dynamic_base + atomicAdd(queue, 1u));
      items[1] = xcd + 8u * (dynamic_base + atomicAdd(queue, 1u));
    }
    __syncthreads();
    cur = __builtin_amdgcn_readfirstlane(items[0]);
    nxt = __builtin_amdgcn_readfirstlane(items[1]);
    __syncthreads();  // items[] is written again in the loop
  }
  if (cur >= a.n_items) return;

  // staging slot(s) of this thread inside a group
  uint32_t s_cl[kSlotsPerThread], s_j[kSlotsPerThread];
#pragma unroll
  for (int u = 0; u < kSlotsPerThread; ++u) {
    const uint32_t s = u * kSweepThreads + tid;
    s_cl[u] = s / I;
    s_j[u] = s - s_cl[u] * I;
  }
  auto load_group = [&](uint32_t item, float4 (&rec)[kSlotsPerThread]) {
#pragma unroll
    for (int u = 0; u < kSlotsPerThread; ++u) {
      const uint32_t c = item * G + s_cl[u];
      rec[u] = make_float4(0.0f, 0.0f, INFINITY, INFINITY);
      if (item < a.n_items && s_cl[u] < G && c < a.n_cand) rec[u] = a.recs[(size_t)c * I + s_j[u]];
    }
  };
  float4 rec0[kSlotsPerThread];
  load_group(cur, rec0);  // in flight while the tile is looked up

  // The request tile of this block: tiles of 256*Q requests, class after class.
  constexpr uint32_t kTile = kSweepThreads * Q;
  uint32_t k_b = 0, off = 0, n_k = 0;
  {
    uint32_t first = 0;
    bool found = false;
    for (uint32_t k = 0; k < a.n_slo; ++k) {
      const uint32_t n = a.cls_count[k];
      const uint32_t tiles = (n + kTile - 1u) / kTile;
      if (!found && rb < first + tiles) {
        found = true; k_b = k; off = (rb - first) * kTile; n_k = n;
      }
      first += tiles;
    }
    if (!found) return;  // no such tile: the whole block leaves
  }
  const float Dt = a.d_ttft[k_b];
  const float Db = a.d_tbt[k_b];

  // A lane without a request carries an infinite prompt length: its latency on every instance is
  // +inf (the per-token prefill cost is positive), so it never counts and needs no mask.
  float L[Q];
  uint32_t wave_reqs = 0;  // valid requests held by this wavefront
#pragma unroll
  for (int q = 0; q < Q; ++q) {
    const uint32_t idx = off + wave * (kWave * Q) + q * kWave + lane;
    const bool ok = idx < n_k;
    L[q] = ok ? a.lbuf[(size_t)k_b * a.n_req + idx] : INFINITY;
    wave_reqs += (uint32_t)__popcll(__ballot(ok));
  }
  const bool any_req = wave_reqs != 0u;

  for (uint32_t i = tid; i < 6u * kMaxGroup; i += kSweepThreads) (&lens[0][0][0])[i] = 0u;
  __syncthreads();

  auto file_group = [&](const float4 (&rec)[kSlotsPerThread], uint32_t it) {
#pragma unroll
    for (int u = 0; u < kSlotsPerThread; ++u)
      if (rec[u].w <= Db) {  // between-token deadline of the block's class
        // records whose queue wait is exactly zero (fresh instances: the placer's usual candidates)
        // fill the candidate's segment from the front, the others from the back
        const bool nowait = rec[u].z == 0.0f;
        const uint32_t pos = atomicAdd(&lens[it % 3u][nowait ? 0 : 1][s_cl[u]], 1u);
        lists[it & 1u][s_cl[u] * I + (nowait ? pos : I - 1u - pos)] = rec[u];
      }
  };
  file_group(rec0, 0u);
  __syncthreads();

  unsigned long long evaluated = 0ull, evaluated_nowait = 0ull;

  uint32_t prev_c0 = 0, prev_n = 0;
  for (uint32_t it = 0;; ++it) {
    uint32_t after_next = 0xffffffffu;
    if (tid == 0u && nxt < a.n_items) after_next = xcd + 8u * (dynamic_base + atomicAdd(queue, 1u));
    float4 rec[kSlotsPerThread];
    load_group(nxt, rec);

    // counts of the previous group: sum over the block's wavefronts, one atomic per candidate
    if (it > 0u && tid < prev_n) {
      const uint32_t b = (it - 1u) & 1u;
      const uint32_t t = blk_cnt[b][0][tid] + blk_cnt[b][1][tid] + blk_cnt[b][2][tid] + blk_cnt[b][3][tid];
      if (t) atomicAdd(&a.sat_count[prev_c0 + tid], t);
    }

    const uint32_t c0 = cur * G;
    const uint32_t g_cands = min(G, a.n_cand - c0);
    uint32_t acc = 0;  // lane g holds this wavefront's count for candidate c0 + g
    if (any_req) {
      const float4* gl = lists[it & 1u];
      const uint32_t* glen0 = lens[it % 3u][0];
      const uint32_t* glen1 = lens[it % 3u][1];
      // lane g fetches the list lengths of candidate g once; the loop reads them lane by lane
      const uint32_t len0 = glen0[lane], len1 = glen1[lane];
      uint32_t n_sum = 0, n0_sum = 0;  // records this wavefront walks in this group
      for (uint32_t g = 0; g < g_cands; ++g) {
        const uint32_t n0 = (uint32_t)__builtin_amdgcn_readlane((int)len0, (int)g);
        const uint32_t n1 = (uint32_t)__builtin_amdgcn_readlane((int)len1, (int)g);
        n_sum += n0 + n1;
        n0_sum += n0;
        const float4* lst = gl + g * I;
        const float4* wlst = lst + (I - n1);  // the records with a wait sit at the segment's end
        uint32_t cnt = 0;
        if (n0 + n1 != 0u) {
          float m[Q];  // smallest first-token latency so far
          // wait == +0: ttft = 0 + prefill = prefill exactly (the prefill time is positive), so the
          // add is left out for those records
          if (n0 != 0u) walk_list<Q, false>(m, L, lst, n0, true);
          if (n1 != 0u) walk_list<Q, true>(m, L, wlst, n1, n0 == 0u);
#pragma unroll
          for (int q = 0; q < Q; ++q) cnt += (uint32_t)__popcll(__ballot(m[q] <= Dt));
        }
        write_lane(acc, cnt, g);
      }
      evaluated += (unsigned long long)n_sum * wave_reqs;
      evaluated_nowait += (unsigned long long)n0_sum * wave_reqs;
    }
    blk_cnt[it & 1u][wave][lane] = acc;

    file_group(rec, it + 1u);
    if (tid < 2u * kMaxGroup) (&lens[(it + 2u) % 3u][0][0])[tid] = 0u;  // last read while scoring group it-1
    if (tid == 0u) items[it & 1u] = after_next;
    __syncthreads();
    prev_c0 = c0;
    prev_n = g_cands;
    cur = nxt;
    nxt = __builtin_amdgcn_readfirstlane(items[it & 1u]);
    if (cur >= a.n_items) {
      if (tid < prev_n) {
        const uint32_t b = it & 1u;
        const uint32_t t = blk_cnt[b][0][tid] + blk_cnt[b][1][tid] + blk_cnt[b][2][tid] + blk_cnt[b][3][tid];
        if (t) atomicAdd(&a.sat_count[prev_c0 + tid], t);
      }
      break;
    }
  }
  // one word per block, no atomics: thousands of same-address atomics at the kernel's end are slow
  __shared__ unsigned long long wave_eval[2][kSweepWaves];
  if (lane == 0u) { wave_eval[0][wave] = evaluated; wave_eval[1][wave] = evaluated_nowait; }
  __syncthreads();
  if (tid < 2u)  // all pairs, then those of them whose instance has no wait
    a.evaluated[(size_t)tid * gridDim.x + blockIdx.x] =
        wave_eval[tid][0] + wave_eval[tid][1] + wave_eval[tid][2] + wave_eval[tid][3];
}

// Wavefronts per SIMD the register allocation must leave room for: eight with up to 8 requests per
// lane, five with 16 (measured: one wavefront fewer costs more than the registers buy).
template <int Q>
__global__ __launch_bounds__(kSweepThreads, (Q <= 8 ? 8 : 5)) void sweep_kernel(const SweepArgs a) {
  sweep_body<Q>(a);
}

// ---------------------------------------------------------------------------------------------
// ratio[c] = count[c] / R and the best candidate: largest count, lowest index on ties (Alg. 1 keeps
// the best-scoring deployment).  One block.  Also clears the class counters for the next call.
__global__ __launch_bounds__(1024) void sweep_finalize_kernel(const uint32_t* __restrict__ sat_count,
                                                              uint32_t n_cand, uint32_t n_req,
                                                              float* __restrict__ sat_ratio,
                                                              uint32_t* __restrict__ best_cand,
                                                              uint32_t* __restrict__ cls_count,
                                                              const unsigned long long* __restrict__ eval_parts,
                                                              uint32_t n_parts,
                                                              unsigned long long* __restrict__ eval_total) {
  __shared__ unsigned long long best[16];
  __shared__ unsigned long long esum[2][16];
  if (threadIdx.x < kMaxSlo) cls_count[threadIdx.x] = 0u;
  // The kernel is one block, so its duration is the number of dependent trips to memory: the first
  // batch of every array (eight elements per thread each) is requested before anything is used.
  constexpr uint32_t kBatch = 8;
  const uint32_t stride = kBatch * blockDim.x;
  unsigned long long v0[kBatch], v1[kBatch];
  uint32_t n[kBatch];
#pragma unroll
  for (uint32_t u = 0; u < kBatch; ++u) {
    const uint32_t i = threadIdx.x + u * blockDim.x;
    v0[u] = i < n_parts ? eval_parts[i] : 0ull;
    v1[u] = i < n_parts ? eval_parts[(size_t)n_parts + i] : 0ull;
    n[u] = i < n_cand ? sat_count[i] : 0u;
  }
  for (uint32_t half = 0; half < 2u; ++half) {  // all pairs, then the pairs without a wait
    const unsigned long long* parts = eval_parts + (size_t)half * n_parts;
    unsigned long long e = 0ull;
#pragma unroll
    for (uint32_t u = 0; u < kBatch; ++u) e += half ? v1[u] : v0[u];
    for (uint32_t i0 = threadIdx.x + stride; i0 < n_parts; i0 += stride) {
      unsigned long long v[kBatch];
#pragma unroll
      for (uint32_t u = 0; u < kBatch; ++u) {
        const uint32_t i = i0 + u * blockDim.x;
        v[u] = i < n_parts ? parts[i] : 0ull;
      }
#pragma unroll
      for (uint32_t u = 0; u < kBatch; ++u) e += v[u];
    }
    for (int d = 32; d >= 1; d >>= 1) e += __shfl_xor(e, d);
    if ((threadIdx.x & 63u) == 0u) esum[half][threadIdx.x >> 6] = e;
  }
  const float fr = (float)n_req;
  unsigned long long key = 0ull;  // (count << 32) | ~index: max key = max count, then min index
  for (uint32_t c0 = threadIdx.x; c0 < n_cand; c0 += stride) {
    if (c0 != threadIdx.x) {
#pragma unroll
      for (uint32_t u = 0; u < kBatch; ++u) {
        const uint32_t c = c0 + u * blockDim.x;
        n[u] = c < n_cand ? sat_count[c] : 0u;
      }
    }
#pragma unroll
    for (uint32_t u = 0; u < kBatch; ++u) {
      const uint32_t c = c0 + u * blockDim.x;
      if (c >= n_cand) continue;
      if (sat_ratio) sat_ratio[c] = n_req ? (float)n[u] / fr : 0.0f;
      const unsigned long long kc = ((unsigned long long)n[u] << 32) | (unsigned long long)(~c);
      key = kc > key ? kc : key;
    }
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
  if (threadIdx.x < 2u) {
    unsigned long long e = 0ull;
    for (uint32_t w = 0; w < (blockDim.x >> 6); ++w) e += esum[threadIdx.x][w];
    eval_total[threadIdx.x] = e;
  }
}

}  // namespace maaso
