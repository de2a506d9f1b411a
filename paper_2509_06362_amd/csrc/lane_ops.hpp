// Exchanges between the lanes of a wavefront with DPP: what the windowed kernels use to settle a
// request that is spread over several lanes, and to add up what a wavefront admits.
#pragma once

#include "assign_kernels.hpp"

namespace maaso {

// (slack, index) of the better of two candidates: larger slack, lower index among equals.
__device__ __forceinline__ void take_better(float& s, int32_t& i, float os, int32_t oi) {
  const bool take = (os > s) | ((os == s) & (oi < i));  // no short circuit: three compares, no branches
  s = take ? os : s;
  i = take ? oi : i;
}

// x = OP(x, x of the lane that the DPP control CTRL names), one instruction.  A DPP operand written by
// the vector instruction just before needs two wait states, which the assembler does not add inside
// an asm statement: hence the s_nop.
// ROWS: mask of the 16-lane rows that are written; the others keep their value.
#define MAASO_DPP_FOLD_ROWS(OP, X, CTRL, ROWS) \
  asm("s_nop 1\n\t" OP " %0, %0, %0 " CTRL " row_mask:" ROWS " bank_mask:0xf" : "+v"(X))
#define MAASO_DPP_FOLD(OP, X, CTRL) MAASO_DPP_FOLD_ROWS(OP, X, CTRL, "0xf")

// Maximum (v_max_f32: a NaN operand loses) / unsigned minimum over groups of LPR consecutive lanes
// (a power of two up to 64); every lane ends with the group's value.  Up to 16 lanes the partner
// lanes are reached with DPP controls - lane ^ 1, lane ^ 2, then the mirrored quad of the 8 and the
// mirrored half of the 16-lane row - beyond that through LDS permutes.
template <int LPR>
__device__ __forceinline__ float max_lanes(float m) {
  if (LPR >= 2) MAASO_DPP_FOLD("v_max_f32_dpp", m, "quad_perm:[1,0,3,2]");
  if (LPR >= 4) MAASO_DPP_FOLD("v_max_f32_dpp", m, "quad_perm:[2,3,0,1]");
  if (LPR >= 8) MAASO_DPP_FOLD("v_max_f32_dpp", m, "row_half_mirror");
  if (LPR >= 16) MAASO_DPP_FOLD("v_max_f32_dpp", m, "row_mirror");
  if (LPR >= 32) m = max_no_nan(m, __shfl_xor(m, 16));
  if (LPR >= 64) m = max_no_nan(m, __shfl_xor(m, 32));
  return m;
}

template <int LPR>
__device__ __forceinline__ uint32_t min_lanes(uint32_t c) {
  if (LPR >= 2) MAASO_DPP_FOLD("v_min_u32_dpp", c, "quad_perm:[1,0,3,2]");
  if (LPR >= 4) MAASO_DPP_FOLD("v_min_u32_dpp", c, "quad_perm:[2,3,0,1]");
  if (LPR >= 8) MAASO_DPP_FOLD("v_min_u32_dpp", c, "row_half_mirror");
  if (LPR >= 16) MAASO_DPP_FOLD("v_min_u32_dpp", c, "row_mirror");
  if (LPR >= 32) c = min(c, (uint32_t)__shfl_xor((int)c, 16));
  if (LPR >= 64) c = min(c, (uint32_t)__shfl_xor((int)c, 32));
  return c;
}

// Arg-max of (slack, index) over groups of LPR consecutive lanes, lowest index among equal slacks;
// every lane ends with the winner.  Two reductions of one instruction per step: the largest slack,
// then the lowest index among the lanes that hold it.  A lane that has seen no slack above -inf
// carries index -1; when the maximum is -inf every lane of the group does, and -1 (the largest
// unsigned value) is what comes out.
template <int LPR>
__device__ __forceinline__ void argmax_lanes(float& s, int32_t& i) {
  const float m = max_lanes<LPR>(s);
  const uint32_t c = (s == m) ? (uint32_t)i : 0xffffffffu;
  i = (int32_t)min_lanes<LPR>(c);
  s = m;
}

// Sum of a 32-bit value over the wavefront (the caller makes sure it cannot overflow), as a uniform
// value: four DPP steps give every lane its row's sum, two row broadcasts carry the rows' sums into
// lane 63.  Six dependent vector additions instead of six trips through the LDS permute network.
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
  MAASO_DPP_FOLD("v_add_u32_dpp", v, "quad_perm:[1,0,3,2]");
  MAASO_DPP_FOLD("v_add_u32_dpp", v, "quad_perm:[2,3,0,1]");
  MAASO_DPP_FOLD("v_add_u32_dpp", v, "row_half_mirror");
  MAASO_DPP_FOLD("v_add_u32_dpp", v, "row_mirror");
  MAASO_DPP_FOLD_ROWS("v_add_u32_dpp", v, "row_bcast:15", "0xa");
  MAASO_DPP_FOLD_ROWS("v_add_u32_dpp", v, "row_bcast:31", "0xc");
  return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

}  // namespace maaso
