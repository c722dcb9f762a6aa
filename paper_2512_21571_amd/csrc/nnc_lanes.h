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
