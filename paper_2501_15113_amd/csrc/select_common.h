// Radix select on the bit patterns of non-negative fp64 scores (shared by the
// selection kernels): unsigned integer order equals numeric order.
#pragma once

#include "taskkv_internal.h"

namespace taskkv {

__device__ __forceinline__ uint64_t score_key(double x) { return (uint64_t)__double_as_longlong(x); }

// Add one count per active lane to hist[digit].  Lanes that share a digit are
// merged into one LDS atomic (the leading bytes of scores take only a handful of
// values, and same-address atomics of a wave serialise).
__device__ __forceinline__ void hist_add_merged(unsigned *hist, bool active, unsigned digit) {
  const int lane = threadIdx.x & 63;
  uint64_t todo = __ballot(active);
  while (todo) {
    const int leader = __ffsll((unsigned long long)todo) - 1;
    const unsigned d0 = __shfl(digit, leader);
    const uint64_t same = __ballot(active && digit == d0);
    if (lane == leader) atomicAdd(&hist[d0], (unsigned)__popcll(same));
    todo &= ~same;
  }
}

// Bit pattern of the count-th largest score inside [lo, hi), and how many of
// the entries equal to it belong to the top `count` (lowest index first).
// 8-bit digits, most significant first.  Called by all 1024 threads of a block;
// hist[256], s_bin, s_rem are block-shared scratch.
__device__ __forceinline__ uint64_t radix_threshold(const double *__restrict__ sc, int lo, int hi, int count,
                                                    unsigned *hist, int *s_bin, int *s_rem, int &take_equal) {
  const int tid = threadIdx.x;
  uint64_t pat = 0, known = 0;
  int remaining = count;
  for (int pass = 7; pass >= 0; --pass) {
    const int shift = pass * 8;
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int j0 = lo; j0 < hi; j0 += 4096) {
      uint64_t key[4];
      bool ok[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int j = j0 + r * 1024 + tid;
        ok[r] = j < hi;
        key[r] = ok[r] ? score_key(sc[j]) : 0;
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const bool hit = ok[r] && (key[r] & known) == pat;
        const unsigned digit = (unsigned)(key[r] >> shift) & 255u;
        if (pass == 7) hist_add_merged(hist, hit, digit);
        else if (hit) atomicAdd(&hist[digit], 1u);
      }
    }
    __syncthreads();
    if (tid == 0) {
      int cum = 0, b = 255;
      for (; b > 0; --b) {
        const int c = (int)hist[b];
        if (cum + c >= remaining) break;
        cum += c;
      }
      *s_bin = b;
      *s_rem = remaining - cum;
    }
    __syncthreads();
    pat |= (uint64_t)(*s_bin) << shift;
    known |= 0xffull << shift;
    remaining = *s_rem;
    __syncthreads();
  }
  take_equal = remaining;
  return pat;
}

}  // namespace taskkv
