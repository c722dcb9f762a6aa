// Cross-lane reductions of a 64-lane wave built from DPP moves (one VALU instruction each)
// instead of LDS-routed lane permutes.
#pragma once
#include <hip/hip_runtime.h>

namespace nnc {

// v as seen through a DPP control word (all rows and banks enabled).
template <int CTRL>
__device__ __forceinline__ float dpp_get(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

constexpr int DPP_QUAD_XOR1 = 0xB1;         // quad_perm [1, 0, 3, 2]
constexpr int DPP_QUAD_XOR2 = 0x4E;         // quad_perm [2, 3, 0, 1]
constexpr int DPP_ROW_HALF_MIRROR = 0x141;  // lane i <-> 7 - i inside each group of 8
constexpr int DPP_ROW_MIRROR = 0x140;       // lane i <-> 15 - i inside each row of 16

// Sum / maximum over each row of 16 lanes, returned in every lane of the row.
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_get<DPP_QUAD_XOR1>(v);
  v += dpp_get<DPP_QUAD_XOR2>(v);
  v += dpp_get<DPP_ROW_HALF_MIRROR>(v);  // the other quad of the half holds the other quad's total
  v += dpp_get<DPP_ROW_MIRROR>(v);       // the other half of the row
  return v;
}
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, dpp_get<DPP_QUAD_XOR1>(v));
  v = fmaxf(v, dpp_get<DPP_QUAD_XOR2>(v));
  v = fmaxf(v, dpp_get<DPP_ROW_HALF_MIRROR>(v));
  v = fmaxf(v, dpp_get<DPP_ROW_MIRROR>(v));
  return v;
}

__device__ __forceinline__ float lane_get(float v, int lane) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

// Sum / maximum over the four lanes that share lane % 16 (one per row of 16 lanes), returned
// in all four, with the two row-swap instructions of gfx950 (no LDS).  v_permlane16_swap
// exchanges row 1 of its first register with row 0 of its second, and row 3 with row 2: from
// two copies of v it leaves rows [0,0,2,2] in the first and [1,1,3,3] in the second.
// v_permlane32_swap exchanges the upper half of the first with the lower half of the second:
// rows [0,1,0,1] and [2,3,2,3].  Written as inline assembly with both registers as in/out
// operands: the compiler's builtin folds the two results into one when its inputs are equal.
// The leading s_nop covers the wait states the instruction needs after a vector write of its
// operands.
__device__ __forceinline__ void row_swap16(float& a, float& b) {
  asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ void row_swap32(float& a, float& b) {
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ float col4_max(float v) {
  float a = v, b = v;
  row_swap16(a, b);
  a = fmaxf(a, b);
  b = a;
  row_swap32(a, b);
  return fmaxf(a, b);
}
__device__ __forceinline__ float col4_sum(float v) {
  float a = v, b = v;
  row_swap16(a, b);
  a = a + b;
  b = a;
  row_swap32(a, b);
  return a + b;
}

// Sum / maximum over the whole wave, returned in every lane (wave-uniform).
__device__ __forceinline__ float wave_sum(float v) {
  v = row16_sum(v);
  return (lane_get(v, 0) + lane_get(v, 16)) + (lane_get(v, 32) + lane_get(v, 48));
}
__device__ __forceinline__ float wave_max(float v) {
  v = row16_max(v);
  return fmaxf(fmaxf(lane_get(v, 0), lane_get(v, 16)), fmaxf(lane_get(v, 32), lane_get(v, 48)));
}

}  // namespace nnc
