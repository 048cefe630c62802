// Cross-lane sums for 64-wide wavefronts on gfx950.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tuner {

// The swap instructions exchange halves (or rows) of TWO registers.  Handing the
// builtin one value twice lets the compiler conclude that both results are equal and
// fold r[0] + r[1] into 2 * r[0]; the second operand therefore goes through an empty
// asm statement, which makes it a value of its own.
__device__ __forceinline__ uint32_t opaque_copy(uint32_t v) {
  asm volatile("" : "+v"(v));
  return v;
}

// x[lane] + x[lane ^ 32] in every lane (v_permlane32_swap exchanges the upper 32 lanes
// of its first operand with the lower 32 lanes of its second)
__device__ __forceinline__ float pair_sum(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), opaque_copy(__float_as_uint(x)), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ int pair_sum(int x) {
  const auto r = __builtin_amdgcn_permlane32_swap((unsigned)x, opaque_copy((unsigned)x), false, false);
  return (int)(r[0] + r[1]);
}

// x[lane] + x[lane ^ 16] in every lane (v_permlane16_swap exchanges the odd 16-lane
// rows of its first operand with the even rows of its second)
__device__ __forceinline__ float row_pair_sum(float x) {
  const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), opaque_copy(__float_as_uint(x)), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Sum over each 16-lane row, left in every lane of the row: quad_perm [1,0,3,2],
// quad_perm [2,3,0,1], row_half_mirror, row_mirror.
__device__ __forceinline__ float row_sum(float x) {
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xf, 0xf, false));
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x4E, 0xf, 0xf, false));
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x141, 0xf, 0xf, false));
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x140, 0xf, 0xf, false));
  return x;
}

// Sum over the lanes of a group, left in every lane: GROUP = 32 (each half wave) or 64.
template <int GROUP>
__device__ __forceinline__ float group_sum(float x) {
  static_assert(GROUP == 32 || GROUP == 64, "group of 32 or 64 lanes");
  x = row_pair_sum(row_sum(x));
  if constexpr (GROUP == 64) x = pair_sum(x);
  return x;
}

}  // namespace tuner
