// Reductions over the four lanes l, l ^ 16, l ^ 32, l ^ 48 of a wave with the
// two lane swaps of gfx950.  They are vector ALU instructions; a shuffle across
// 16-lane rows goes through the LDS crossbar and is waited for.
//   permlane32_swap(a, b) exchanges the upper half of a with the lower half of b,
//   permlane16_swap(a, b) the odd 16-lane rows of a with the even rows of b;
// fed the same value twice, the two results hold x and x[l ^ 32] (x and
// x[l ^ 16]) in every lane, in an order that does not matter to a commutative
// reduction (layout checked on the device).
#pragma once

#include <hip/hip_runtime.h>

namespace taskkv {

__device__ __forceinline__ float sum_lanes_16_32(float x) {
  const unsigned u = __float_as_uint(x);
  const auto h = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  const float y = __uint_as_float(h[0]) + __uint_as_float(h[1]);
  const unsigned v = __float_as_uint(y);
  const auto q = __builtin_amdgcn_permlane16_swap(v, v, false, false);
  return __uint_as_float(q[0]) + __uint_as_float(q[1]);
}

__device__ __forceinline__ float max_lanes_16_32(float x) {
  const unsigned u = __float_as_uint(x);
  const auto h = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  const float y = fmaxf(__uint_as_float(h[0]), __uint_as_float(h[1]));
  const unsigned v = __float_as_uint(y);
  const auto q = __builtin_amdgcn_permlane16_swap(v, v, false, false);
  return fmaxf(__uint_as_float(q[0]), __uint_as_float(q[1]));
}

}  // namespace taskkv
