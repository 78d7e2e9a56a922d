// Reductions over the four lanes l % 16 + 16 q of a wavefront (one lane of each 16-lane row), for
// kernels that keep a matrix row in those four lanes (16 rows per wave).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sea {

// all-reduce over the four lanes l % 16 + 16 q of a wave (one lane of each 16-lane row): the
// row-swap instructions hand every lane the value of its partner row, two steps cover all four
__device__ __forceinline__ uint32_t rows_sum_u(uint32_t x) {
  const auto a = __builtin_amdgcn_permlane16_swap(x, x, false, false);
  const uint32_t y = a[0] + a[1];
  const auto b = __builtin_amdgcn_permlane32_swap(y, y, false, false);
  return b[0] + b[1];
}
__device__ __forceinline__ uint32_t rows_or_u(uint32_t x) {
  const auto a = __builtin_amdgcn_permlane16_swap(x, x, false, false);
  const uint32_t y = a[0] | a[1];
  const auto b = __builtin_amdgcn_permlane32_swap(y, y, false, false);
  return b[0] | b[1];
}
__device__ __forceinline__ uint32_t rows_max_u(uint32_t x) {
  const auto a = __builtin_amdgcn_permlane16_swap(x, x, false, false);
  const uint32_t y = max(a[0], a[1]);
  const auto b = __builtin_amdgcn_permlane32_swap(y, y, false, false);
  return max(b[0], b[1]);
}
__device__ __forceinline__ float rows_sum(float x) {
  const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  const float y = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(y), __float_as_uint(y), false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}
// sum over the rows and, for each lane, the sum over the rows below its own (rows in order 0..3)
__device__ __forceinline__ uint32_t rows_sum_prefix_u(uint32_t x, int lg, uint32_t* below) {
  const auto a = __builtin_amdgcn_permlane16_swap(x, x, false, false);   // a[0]: even row of the pair, a[1]: odd
  const uint32_t pair = a[0] + a[1];
  const auto b = __builtin_amdgcn_permlane32_swap(pair, pair, false, false);  // b[0]: rows 0,1; b[1]: rows 2,3
  *below = ((lg & 1) ? a[0] : 0u) + ((lg & 2) ? b[0] : 0u);
  return b[0] + b[1];
}

}  // namespace sea
