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

// Candidates the radix select keeps in LDS once few enough remain.
constexpr int RADIX_CAND = 4096;
struct RadixScratch {
  unsigned hist[256];
  int bin, rem, n;
  uint64_t cand[RADIX_CAND];
};

// Bit pattern of the count-th largest score inside [lo, hi), and how many of
// the entries equal to it belong to the top `count` (lowest index first).
// 8-bit digits, most significant first.  Every digit costs a sweep over the
// scores (L2 latency bound: one block per unit), so as soon as the entries
// that still share the threshold's known digits fit RADIX_CAND, one more sweep
// copies their bit patterns to LDS and the remaining digits are settled there:
// typically three sweeps plus the copy instead of eight.  Called by all 1024
// threads of a block.
__device__ __forceinline__ uint64_t radix_threshold(const double *__restrict__ sc, int lo, int hi, int count,
                                                    RadixScratch &rs, int &take_equal) {
  const int tid = threadIdx.x, lane = tid & 63;
  uint64_t pat = 0, known = 0;
  int remaining = count;
  bool in_lds = false;
  int n_cand = 0;
  for (int pass = 7; pass >= 0; --pass) {
    const int shift = pass * 8;
    if (tid < 256) rs.hist[tid] = 0;
    __syncthreads();
    if (in_lds) {
      for (int i = tid; i < n_cand; i += 1024) {
        const uint64_t key = rs.cand[i];
        if ((key & known) == pat) atomicAdd(&rs.hist[(unsigned)(key >> shift) & 255u], 1u);
      }
    } else {
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
          if (pass == 7) hist_add_merged(rs.hist, hit, digit);
          else if (hit) atomicAdd(&rs.hist[digit], 1u);
        }
      }
    }
    __syncthreads();
    if (tid < 64) {
      // the bin that holds the remaining-th largest entry: lane i owns bins
      // 255 - 4 i ... 252 - 4 i, a wave scan gives the count above each lane's bins
      int c[4], own = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        c[q] = (int)rs.hist[255 - 4 * tid - q];
        own += c[q];
      }
      int incl = own;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const int t = __shfl_up(incl, off);
        if (tid >= off) incl += t;
      }
      int cum = incl - own;   // entries in bins above mine
      const uint64_t reach = __ballot(incl >= remaining);
      const int owner = reach ? __ffsll((unsigned long long)reach) - 1 : 63;   // else bin 0 takes what is left
      if (tid == owner) {
        int q = 0;   // the lane's fourth bin is taken when the first three do not reach
        for (; q < 3; ++q) {
          if (cum + c[q] >= remaining) break;
          cum += c[q];
        }
        rs.bin = 255 - 4 * tid - q;
        rs.rem = remaining - cum;
        rs.n = 0;
      }
    }
    __syncthreads();
    const int n_match = (int)rs.hist[rs.bin];   // entries that share all digits known after this pass
    pat |= (uint64_t)rs.bin << shift;
    known |= 0xffull << shift;
    remaining = rs.rem;
    __syncthreads();
    if (!in_lds && pass >= 2 && n_match <= RADIX_CAND) {
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
          const uint64_t bal = __ballot(hit);
          if (bal) {
            const int leader = __ffsll((unsigned long long)bal) - 1;
            int base = 0;
            if (lane == leader) base = atomicAdd(&rs.n, __popcll(bal));
            base = __shfl(base, leader);
            if (hit) rs.cand[base + __popcll(bal & ((1ull << lane) - 1ull))] = key[r];
          }
        }
      }
      __syncthreads();
      n_cand = rs.n;
      in_lds = true;
    }
  }
  take_equal = remaining;
  return pat;
}

}  // namespace taskkv
