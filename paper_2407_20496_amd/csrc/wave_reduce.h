// Wave-wide reductions built from data-parallel-primitive moves (gfx9 family: row shifts and row
// broadcasts), which cost a few vector instructions and no LDS traffic.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hinm {

// Wave-wide minimum with data-parallel-primitive moves instead of LDS shuffles: four shifts inside
// every row of 16 lanes, then lane 15 of a row into the next row, then lane 31 into the upper half;
// lane 63 ends up with the minimum of all 64 lanes and is read back as a wave-uniform value.  Lanes
// that a step does not write keep their own value, which is harmless for a minimum.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_move(int own) {
  return __builtin_amdgcn_update_dpp(own, own, CTRL, ROW_MASK, 0xf, false);
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_move(double own) {
  const int lo = dpp_move<CTRL, ROW_MASK>(__double2loint(own));
  const int hi = dpp_move<CTRL, ROW_MASK>(__double2hiint(own));
  return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double wave_min(double v) {
  v = __builtin_fmin(v, dpp_move<0x111, 0xf>(v));  // row_shr:1
  v = __builtin_fmin(v, dpp_move<0x112, 0xf>(v));  // row_shr:2
  v = __builtin_fmin(v, dpp_move<0x114, 0xf>(v));  // row_shr:4
  v = __builtin_fmin(v, dpp_move<0x118, 0xf>(v));  // row_shr:8
  v = __builtin_fmin(v, dpp_move<0x142, 0xa>(v));  // row_bcast:15 into rows 1 and 3
  v = __builtin_fmin(v, dpp_move<0x143, 0xc>(v));  // row_bcast:31 into rows 2 and 3
  return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), 63),
                          __builtin_amdgcn_readlane(__double2loint(v), 63));
}
__device__ __forceinline__ int wave_min(int v) {
  v = min(v, dpp_move<0x111, 0xf>(v));
  v = min(v, dpp_move<0x112, 0xf>(v));
  v = min(v, dpp_move<0x114, 0xf>(v));
  v = min(v, dpp_move<0x118, 0xf>(v));
  v = min(v, dpp_move<0x142, 0xa>(v));
  v = min(v, dpp_move<0x143, 0xc>(v));
  return __builtin_amdgcn_readlane(v, 63);
}
// (smallest value, lowest index among the lanes that hold it) over the wave, wave-uniform
__device__ __forceinline__ void wave_argmin(double& best, int& best_j, int none) {
  const double lo = wave_min(best);
  best_j = wave_min(best == lo ? best_j : none);
  best = lo;
}

// Sum of one int per lane, wave-uniform.  Lanes a step does not write receive 0 for that step.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_move_or_zero(int own) {
  return __builtin_amdgcn_update_dpp(0, own, CTRL, ROW_MASK, 0xf, false);
}
__device__ __forceinline__ int wave_sum(int v) {
  v += dpp_move_or_zero<0x111, 0xf>(v);  // after the four shifts lane i of a row holds the sum of lanes 0..i of that row
  v += dpp_move_or_zero<0x112, 0xf>(v);
  v += dpp_move_or_zero<0x114, 0xf>(v);
  v += dpp_move_or_zero<0x118, 0xf>(v);
  v += dpp_move_or_zero<0x142, 0xa>(v);  // rows 1 and 3 add the total of the row before
  v += dpp_move_or_zero<0x143, 0xc>(v);  // rows 2 and 3 add the total of rows 0 and 1
  return __builtin_amdgcn_readlane(v, 63);
}

}  // namespace hinm
