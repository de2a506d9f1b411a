// Sustained vector-ALU rate of the sweep's instruction mix, measured on the device the library runs
// on: the same fixed instruction sequences as the sweep's pair body (sweep_kernels.hpp), in a loop
// with nothing else - no LDS, no memory, no branches beyond the loop's own.  What these kernels reach
// is the practical ceiling for the sweep on this chip; the nominal peak (one instruction per SIMD
// every two cycles) is what the roofline fractions are quoted against.  Instrumentation only: no
// entry point of the scoring path uses them.
#pragma once

#include "sweep_kernels.hpp"

namespace maaso {

constexpr int kProbeThreads = 256;

// pattern 0: pair body without a queue wait (two fma, one three-input minimum per request), 24
//            instructions per trip;  1: with the wait's add, 40 per trip;  2: pattern 0 four times
//            per trip (96);  3: eight compares that write a lane mask, each followed by an add that
//            keeps it alive (16 per trip);  4: eight fma with a scalar-register operand.
template <int kPattern>
__global__ __launch_bounds__(kProbeThreads, 8) void valu_probe_kernel(float* out, uint32_t trips, float seed) {
  float m[8], L[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) { m[q] = 1.0e30f; L[q] = seed + (float)(threadIdx.x + q); }
  float4 r = make_float4(seed * 1.0e-5f, seed * 1.0e-2f, seed * 1.0e-3f, 0.0f);
  float4 u = make_float4(seed * 2.0e-5f, seed * 2.0e-2f, seed * 2.0e-3f, 0.0f);
  uint32_t hits = 0;
  for (uint32_t t = 0; t < trips; ++t) {
    if (kPattern == 0) fold_pair_n<false>(m, L, r, u);
    if (kPattern == 1) fold_pair_n<true>(m, L, r, u);
    if (kPattern == 2) {
      fold_pair_n<false>(m, L, r, u);
      fold_pair_n<false>(m, L, u, r);
      fold_pair_n<false>(m, L, r, u);
      fold_pair_n<false>(m, L, u, r);
    }
    if (kPattern == 3) {
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        uint32_t h;
        asm volatile("v_cmp_le_f32 vcc, %1, %2\n\tv_addc_co_u32 %0, vcc, 0, %3, vcc"
                     : "=v"(h) : "v"(L[q]), "v"(m[q]), "v"(hits) : "vcc");
        hits = h;
      }
    }
    if (kPattern == 4) {
      const float k = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, r.x)));
#pragma unroll
      for (int q = 0; q < 8; ++q) asm volatile("v_fma_f32 %0, %1, %2, %0" : "+v"(m[q]) : "s"(k), "v"(L[q]));
    }
    asm volatile("" : "+v"(r.x), "+v"(u.x));  // the records are not loop constants to the compiler
  }
  float s = (float)hits;
#pragma unroll
  for (int q = 0; q < 8; ++q) s += m[q];
  out[(size_t)blockIdx.x * kProbeThreads + threadIdx.x] = s;
}

}  // namespace maaso
