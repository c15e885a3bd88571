// Lane-level helpers shared by the kernels (wave64, gfx950).
#pragma once

#include <hip/hip_runtime.h>

namespace linear {

__device__ __forceinline__ float ninf() { return -__builtin_inff(); }
__device__ __forceinline__ float ex2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int CTRL>
__device__ __forceinline__ float dpp(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false));
}
constexpr int kXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kHalfMirror = 0x141; // lane i <- lane 7-i of its 8-lane half row
constexpr int kMirror = 0x140;     // lane i <- lane 15-i of its 16-lane row

// Sum over the aligned group of W adjacent lanes, result in every lane of the group.
template <int W>
__device__ __forceinline__ float sum_within(float x) {
  x += dpp<kXor1>(x);
  x += dpp<kXor2>(x);
  if (W >= 8) x += dpp<kHalfMirror>(x);
  if (W >= 16) x += dpp<kMirror>(x);
  if (W >= 32) x += __shfl_xor(x, 16);
  return x;
}
// Maximum over each 16-lane row, result in every lane of the row.
__device__ __forceinline__ float max_within_row(float x) {
  x = fmaxf(x, dpp<kXor1>(x));
  x = fmaxf(x, dpp<kXor2>(x));
  x = fmaxf(x, dpp<kHalfMirror>(x));
  x = fmaxf(x, dpp<kMirror>(x));
  return x;
}
__device__ __forceinline__ float lane_bcast(float x, int lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), lane));
}
__device__ __forceinline__ float wave_max(float x) {
  x = max_within_row(x);
  return fmaxf(fmaxf(lane_bcast(x, 0), lane_bcast(x, 16)), fmaxf(lane_bcast(x, 32), lane_bcast(x, 48)));
}

}  // namespace linear
