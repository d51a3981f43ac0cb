// Scans over the 64 lanes of a wave in registers.
#pragma once
#include "common.hpp"
#include "segreduce.hpp"

namespace spt {

// Lane movement through the data-parallel-primitive path of the vector ALU (a few clocks,
// against a trip through the LDS crossbar for a shuffle). A lane without a source (first
// lanes of a row for row_shr, rows outside ROWS for row_bcast) receives `idle`.
template <int CTRL, int ROWS>
__device__ __forceinline__ int dpp_move(int idle, int v) {
  return __builtin_amdgcn_update_dpp(idle, v, CTRL, ROWS, 0xf, false);
}
template <int CTRL, int ROWS>
__device__ __forceinline__ float dpp_move(float idle, float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(idle), __float_as_int(v), CTRL, ROWS, 0xf, false));
}
template <int CTRL, int ROWS>
__device__ __forceinline__ double dpp_move(double idle, double v) {
  const int lo = __builtin_amdgcn_update_dpp(__double2loint(idle), __double2loint(v), CTRL, ROWS, 0xf, false);
  const int hi = __builtin_amdgcn_update_dpp(__double2hiint(idle), __double2hiint(v), CTRL, ROWS, 0xf, false);
  return __hiloint2double(hi, lo);
}

// One step of the wave's inclusive segmented scan: combine with the summary that the lane
// movement CTRL delivers (the identity where nothing arrives).
template <int CTRL, int ROWS, typename T>
__device__ __forceinline__ void wave_seg_step(SegSum<T>& me) {
  SegSum<T> up;
  up.f = dpp_move<CTRL, ROWS>(0, me.f);
  up.v = dpp_move<CTRL, ROWS>(T(0), me.v);
  up.k = dpp_move<CTRL, ROWS>(-1, me.k);
  me = seg_combine(up, me);
}

template <int CTRL, int ROWS>
__device__ __forceinline__ void wave_sum_step(int& v) {
  v += dpp_move<CTRL, ROWS>(0, v);
}

// Inclusive sum over the wave's lanes.
__device__ __forceinline__ int wave_inclusive_sum(int v) {
  wave_sum_step<0x111, 0xf>(v);
  wave_sum_step<0x112, 0xf>(v);
  wave_sum_step<0x114, 0xf>(v);
  wave_sum_step<0x118, 0xf>(v);
  wave_sum_step<0x142, 0xa>(v);
  wave_sum_step<0x143, 0xc>(v);
  return v;
}

// Sum over the wave's lanes, the same value in every lane.
template <typename T>
__device__ __forceinline__ T wave_total(T v) {
  v += dpp_move<0x111, 0xf>(T(0), v);
  v += dpp_move<0x112, 0xf>(T(0), v);
  v += dpp_move<0x114, 0xf>(T(0), v);
  v += dpp_move<0x118, 0xf>(T(0), v);
  v += dpp_move<0x142, 0xa>(T(0), v);
  v += dpp_move<0x143, 0xc>(T(0), v);
  return __shfl(v, kWave - 1);
}

}  // namespace spt
