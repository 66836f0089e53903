// Radix select on the bit patterns of non-negative fp64 scores (shared by the
// selection kernels): unsigned integer order equals numeric order.
#pragma once

#include "taskkv_internal.h"

namespace taskkv {

__device__ __forceinline__ uint64_t score_key(double x) { return (uint64_t)__double_as_longlong(x); }

// Add one count per active lane to hist[digit].  Lanes that share a digit are
// merged into one LDS atomic (same-address atomics of a wave serialise); pays
// when the digit takes only a handful of values.
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

// Scores a thread has in flight per step of a sweep: a sweep is bound by the
// latency of its loads (one block per unit), not by their number.
constexpr int SWEEP_U = 8;

// Candidates the radix select keeps in LDS once few enough remain.
constexpr int RADIX_CAND = 4096;
struct RadixScratch {
  unsigned hist[256];
  int bin, rem, n;
  unsigned top_and, top_or;   // bits 60-63 of every key, and-ed / or-ed
  int wsum[16];
  unsigned hist12[4096];
  uint64_t cand[RADIX_CAND];
};

// Bit pattern of the count-th largest score inside [lo, hi), and how many of
// the entries equal to it belong to the top `count` (lowest index first).
// Radix select, most significant digit first.  Every digit costs a sweep over
// the scores (one block per unit: about 60 GB/s), so
//  - the first sweep takes a 12-bit digit, bits 48-59 (the low eight exponent
//    bits and four of the fraction): scores are means of softmax weights, their
//    leading byte is the same for all of them and says nothing, while this
//    digit spreads them over a few hundred bins.  The sweep also checks that
//    bits 60-63 are indeed common to all keys; if not, it is discarded and the
//    plain 8-bit passes run from the top;
//  - as soon as the entries that still share the threshold's known digits fit
//    RADIX_CAND, one more sweep copies their bit patterns to LDS and the
//    remaining digits are settled there.
// Typically two sweeps instead of eight.  Called by all 1024 threads of a block.
__device__ __forceinline__ uint64_t radix_threshold(const double *__restrict__ sc, int lo, int hi, int count,
                                                    RadixScratch &rs, int &take_equal) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  uint64_t pat = 0, known = 0;
  int remaining = count;
  bool in_lds = false;
  int n_cand = 0;
  int first_pass = 7;
  int n_match0 = hi - lo;
  {
    for (int i = tid; i < 4096; i += 1024) rs.hist12[i] = 0;
    if (tid == 0) rs.top_and = 15u, rs.top_or = 0u, rs.n = 0;
    __syncthreads();
    unsigned t_and = 15u, t_or = 0u;
    for (int j0 = lo; j0 < hi; j0 += SWEEP_U * 1024) {
      uint64_t key[SWEEP_U];
#pragma unroll
      for (int r = 0; r < SWEEP_U; ++r) key[r] = score_key(sc[min(j0 + r * 1024 + tid, hi - 1)]);
#pragma unroll
      for (int r = 0; r < SWEEP_U; ++r) {
        if (j0 + r * 1024 + tid < hi) {
          atomicAdd(&rs.hist12[(unsigned)(key[r] >> 48) & 4095u], 1u);
          const unsigned top = (unsigned)(key[r] >> 60);
          t_and &= top;
          t_or |= top;
        }
      }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      t_and &= __shfl_xor(t_and, off);
      t_or |= __shfl_xor(t_or, off);
    }
    if (lane == 0) {
      atomicAnd(&rs.top_and, t_and);
      atomicOr(&rs.top_or, t_or);
    }
    __syncthreads();
    if (rs.top_and == rs.top_or) {
      // thread i owns bins 4095 - 4 i ... 4092 - 4 i; a block scan gives the count above them
      int c[4], own = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        c[q] = (int)rs.hist12[4095 - 4 * tid - q];
        own += c[q];
      }
      int incl = own;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const int t = __shfl_up(incl, off);
        if (lane >= off) incl += t;
      }
      if (lane == 63) rs.wsum[wv] = incl;
      __syncthreads();
      for (int w = 0; w < wv; ++w) incl += rs.wsum[w];
      int cum = incl - own;
      // the one thread whose bins hold the remaining-th largest entry; the last
      // thread takes what is left when there are fewer entries than asked for
      if ((cum < remaining && remaining <= incl) || (tid == 1023 && incl < remaining)) {
        int q = 0;
        for (; q < 3; ++q) {
          if (cum + c[q] >= remaining) break;
          cum += c[q];
        }
        rs.bin = 4095 - 4 * tid - q;
        rs.rem = remaining - cum;
      }
      __syncthreads();
      pat = ((uint64_t)rs.top_and << 60) | ((uint64_t)rs.bin << 48);
      known = 0xffffull << 48;
      remaining = rs.rem;
      n_match0 = (int)rs.hist12[rs.bin];
      first_pass = 5;
    }
    __syncthreads();
  }
  for (int pass = first_pass; pass >= 0; --pass) {
    // entries that share all known digits, before this pass
    if (!in_lds && pass >= 1 && pass < 7 && n_match0 <= RADIX_CAND) {
      for (int j0 = lo; j0 < hi; j0 += SWEEP_U * 1024) {
        uint64_t key[SWEEP_U];
#pragma unroll
        for (int r = 0; r < SWEEP_U; ++r) key[r] = score_key(sc[min(j0 + r * 1024 + tid, hi - 1)]);
#pragma unroll
        for (int r = 0; r < SWEEP_U; ++r) {
          const bool hit = j0 + r * 1024 + tid < hi && (key[r] & known) == pat;
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
    const int shift = pass * 8;
    // The leading byte takes a handful of values, and so does every digit while
    // more than half of the entries still share all digits known so far (many
    // equal scores): lanes with equal digits are then merged into one atomic.
    const bool concentrated = pass == 7 || 2 * (int64_t)n_match0 > hi - lo;
    if (tid < 256) rs.hist[tid] = 0;
    __syncthreads();
    if (in_lds) {
      for (int i = tid; i < n_cand; i += 1024) {
        const uint64_t key = rs.cand[i];
        if ((key & known) == pat) atomicAdd(&rs.hist[(unsigned)(key >> shift) & 255u], 1u);
      }
    } else {
      for (int j0 = lo; j0 < hi; j0 += SWEEP_U * 1024) {
        uint64_t key[SWEEP_U];
        bool ok[SWEEP_U];
#pragma unroll
        for (int r = 0; r < SWEEP_U; ++r) {
          const int j = j0 + r * 1024 + tid;
          ok[r] = j < hi;
          key[r] = ok[r] ? score_key(sc[j]) : 0;
        }
#pragma unroll
        for (int r = 0; r < SWEEP_U; ++r) {
          const bool hit = ok[r] && (key[r] & known) == pat;
          const unsigned digit = (unsigned)(key[r] >> shift) & 255u;
          if (concentrated) hist_add_merged(rs.hist, hit, digit);
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
    n_match0 = n_match;
  }
  take_equal = remaining;
  return pat;
}

// Ascending list of the indices j in [lo, hi) that `classify(j, sc[j])` marks: 1 = listed,
// 2 = listed while fewer than take_equal entries of class 2 precede it (ties of
// a threshold go to the lower index), 0 = not listed.  Returns the list's
// length.  Every wave of the 1024-thread block owns a contiguous sixteenth of
// the range: one sweep counts, a block-wide exchange of the sixteen totals
// gives every wave its place, a second sweep writes -- no barrier inside the
// sweeps.  s_cnt: 32 ints of LDS.
template <typename F>
__device__ __forceinline__ int list_ascending(const double *__restrict__ sc, int lo, int hi, int take_equal,
                                              int32_t *__restrict__ out, int *s_cnt, F classify) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int seg = (((hi - lo + 15) / 16) + 63) & ~63;
  const int a = min(hi, lo + wv * seg), b = min(hi, a + seg);
  const uint64_t below = (1ull << lane) - 1ull;
  int n1 = 0, n2 = 0;
  for (int j0 = a; j0 < b; j0 += 64 * SWEEP_U) {
    double x[SWEEP_U];   // all loads first, unconditional: a load under a branch is waited for at once
#pragma unroll
    for (int r = 0; r < SWEEP_U; ++r) x[r] = sc[min(j0 + 64 * r + lane, b - 1)];
    int cls[SWEEP_U];
#pragma unroll
    for (int r = 0; r < SWEEP_U; ++r) {
      const int j = j0 + 64 * r + lane;
      cls[r] = j < b ? classify(j, x[r]) : 0;
    }
#pragma unroll
    for (int r = 0; r < SWEEP_U; ++r) {
      n1 += __popcll(__ballot(cls[r] == 1));
      n2 += __popcll(__ballot(cls[r] == 2));
    }
  }
  __syncthreads();   // s_cnt may still be read from an earlier call
  if (lane == 0) {
    s_cnt[wv] = n1;
    s_cnt[16 + wv] = n2;
  }
  __syncthreads();
  int run1 = 0, run2 = 0, tot1 = 0, tot2 = 0;
#pragma unroll
  for (int w = 0; w < 16; ++w) {
    const int c1 = s_cnt[w], c2 = s_cnt[16 + w];
    if (w < wv) run1 += c1, run2 += c2;
    tot1 += c1;
    tot2 += c2;
  }
  for (int j0 = a; j0 < b; j0 += 64 * SWEEP_U) {
    double x[SWEEP_U];   // all loads first, unconditional: a load under a branch is waited for at once
#pragma unroll
    for (int r = 0; r < SWEEP_U; ++r) x[r] = sc[min(j0 + 64 * r + lane, b - 1)];
    int cls[SWEEP_U];
#pragma unroll
    for (int r = 0; r < SWEEP_U; ++r) {
      const int j = j0 + 64 * r + lane;
      cls[r] = j < b ? classify(j, x[r]) : 0;
    }
#pragma unroll
    for (int r = 0; r < SWEEP_U; ++r) {
      const uint64_t b1 = __ballot(cls[r] == 1), b2 = __ballot(cls[r] == 2);
      const int before1 = run1 + __popcll(b1 & below), before2 = run2 + __popcll(b2 & below);
      if (cls[r] == 1 || (cls[r] == 2 && before2 < take_equal))
        out[before1 + min(before2, take_equal)] = j0 + 64 * r + lane;
      run1 += __popcll(b1);
      run2 += __popcll(b2);
    }
  }
  return tot1 + min(tot2, take_equal);
}

}  // namespace taskkv
