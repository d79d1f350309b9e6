// Wavefront-wide sums of doubles by lane permutations (DPP): vector-ALU work only, no LDS traffic.
#pragma once
#include <hip/hip_runtime.h>

// One DPP step of a wavefront reduction on a double: both halves take the same lane permutation (old = 0 where the
// row mask keeps a row out, so that row adds zero).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_add(double v) {
  const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, ROW_MASK, 0xF, false);
  const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, ROW_MASK, 0xF, false);
  return v + __hiloint2double(hi, lo);
}

// The same for the permutations inside a row of 16 lanes, where every lane has a source lane and no row is masked out:
// nothing has to be written to the destination beforehand (three instructions instead of five).
template <int CTRL>
__device__ __forceinline__ double dpp_add_in_row(double v) {
  const int lo = __builtin_amdgcn_mov_dpp(__double2loint(v), CTRL, 0xF, 0xF, true);
  const int hi = __builtin_amdgcn_mov_dpp(__double2hiint(v), CTRL, 0xF, 0xF, true);
  return v + __hiloint2double(hi, lo);
}

// Sum over the wavefront in a fixed order, valid in lane 63: inside quads, quad pairs, halves of a row of 16 and
// rows by lane permutations, then row 0 into row 1 and row 2 into row 3 (lane 15 of a row to the next row), then
// rows 0-1 into rows 2-3 (lane 31 to the upper half).  Pure vector-ALU work, no LDS traffic.
__device__ __forceinline__ double wave_sum_lane63(double v) {
  v = dpp_add_in_row<0xB1>(v);   // quad_perm [1,0,3,2]
  v = dpp_add_in_row<0x4E>(v);   // quad_perm [2,3,0,1]
  v = dpp_add_in_row<0x141>(v);  // row_half_mirror
  v = dpp_add_in_row<0x140>(v);  // row_mirror
  v = dpp_add<0x142, 0xA>(v);  // row_bcast:15 into rows 1 and 3
  v = dpp_add<0x143, 0xC>(v);  // row_bcast:31 into rows 2 and 3
  return v;
}

// The same sum, with identical bits in every lane (lane 63's total through a scalar register).
__device__ __forceinline__ double wave_sum_all(double v) {
  const double t = wave_sum_lane63(v);
  const int lo = __builtin_amdgcn_readlane(__double2loint(t), 63);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(t), 63);
  return __hiloint2double(hi, lo);
}

// N sums at once over the lanes of the first `rows` rows of 16 lanes (rows = 1, 2 or 4, wave-uniform; the other lanes are
// ignored), identical bits in every lane.  The N reductions go through each permutation step together, so that their
// dependent chains hide one another's latency: a lone wavefront sum is latency-bound, N of them cost little more.
template <int N>
__device__ __forceinline__ void wave_sums(double (&v)[N], int rows) {
#pragma unroll
  for (int i = 0; i < N; ++i) v[i] = dpp_add_in_row<0xB1>(v[i]);
#pragma unroll
  for (int i = 0; i < N; ++i) v[i] = dpp_add_in_row<0x4E>(v[i]);
#pragma unroll
  for (int i = 0; i < N; ++i) v[i] = dpp_add_in_row<0x141>(v[i]);
#pragma unroll
  for (int i = 0; i < N; ++i) v[i] = dpp_add_in_row<0x140>(v[i]);
  if (rows > 1) {
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = dpp_add<0x142, 0xA>(v[i]);
  }
  if (rows > 2) {
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = dpp_add<0x143, 0xC>(v[i]);
  }
  const int src = __builtin_amdgcn_readfirstlane(rows * 16 - 1);
#pragma unroll
  for (int i = 0; i < N; ++i) {
    const int lo = __builtin_amdgcn_readlane(__double2loint(v[i]), src);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v[i]), src);
    v[i] = __hiloint2double(hi, lo);
  }
}
__device__ __forceinline__ double wave_sum_rows(double x, int rows) {
  double v[1] = {x};
  wave_sums<1>(v, rows);
  return v[0];
}
