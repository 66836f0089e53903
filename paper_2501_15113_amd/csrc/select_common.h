// Radix select on the bit patterns of non-negative fp64 scores (shared by the
// selection kernels): unsigned integer order equals numeric order.
#pragma once

#include <type_traits>

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

// Views of a unit's scores.  A plain pointer is a view of all columns in
// place; ListedScores is the view of the columns an ascending index list
// names: entry j is the score of column list[j], and that column is what a
// selection reports for it.
struct ListedScores {
  const double *sc;
  const int32_t *list;
  __device__ __forceinline__ double operator[](int j) const { return sc[list[j]]; }
};
__device__ __forceinline__ int position_of(const double *, int j) { return j; }
__device__ __forceinline__ int position_of(const ListedScores &v, int j) { return v.list[j]; }

// Scores a thread has in flight per step of a sweep: a sweep is bound by the
// latency of its loads (one block per unit), not by their number.
constexpr int SWEEP_U = 8;

// Candidates the radix select keeps in LDS once few enough remain.
constexpr int RADIX_CAND = 8192;
struct RadixScratch {
  uint64_t found;
  int bin, rem, n_bin, n;
  unsigned top_and, top_or;   // bits 60-63 of every key, and-ed / or-ed
  int wsum[16];
  alignas(16) unsigned hist12[4096];   // read four bins at a time
  uint64_t cand[RADIX_CAND];
};

// The bin of `hist` (4096 bins of a 12-bit digit, in LDS or in global memory)
// that holds the remaining-th largest entry -> rs.bin, its rank inside the bin
// -> rs.rem, the bin's count -> rs.n_bin.  Thread i owns bins 4095 - 4 i ...
// 4092 - 4 i; a block scan gives the count above them.  Called by all 1024
// threads; ends with a barrier.
template <typename RS>
__device__ __forceinline__ void pick_bin12(const unsigned *hist, RS &rs, int remaining) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const uint4 mine = *reinterpret_cast<const uint4 *>(hist + 4092 - 4 * tid);
  const int c[4] = {(int)mine.w, (int)mine.z, (int)mine.y, (int)mine.x};   // highest bin first
  const int own = c[0] + c[1] + c[2] + c[3];
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
    rs.n_bin = c[q];
  }
  __syncthreads();
}

// The digits of a radix select from `shift` down: `pat` holds the digits
// settled so far (`known` masks them), n_match entries of [lo, hi) share them
// and the wanted one is the remaining-th largest of those.  All 1024 threads.
template <typename SC>
__device__ __forceinline__ uint64_t radix_finish(SC sc, int lo, int hi, RadixScratch &rs, uint64_t pat, uint64_t known,
                                                 int shift, int remaining, int n_match, int &take_equal,
                                                 int n_in_lds = 0) {
  const int tid = threadIdx.x, lane = tid & 63;
  // n_in_lds > 0: the caller has put all hi - lo keys into rs.cand already
  bool in_lds = n_in_lds > 0;
  int n_cand = n_in_lds;
  if (tid == 0) rs.n = 0;
  __syncthreads();
  for (; shift >= 0; shift -= 12) {
    if (!in_lds && n_match <= RADIX_CAND) {
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
    if (in_lds && n_match == 1) {
      // one entry shares the known digits: it is the wanted one
      for (int i = tid; i < n_cand; i += 1024)
        if ((rs.cand[i] & known) == pat) rs.found = rs.cand[i];
      __syncthreads();
      pat = rs.found;
      __syncthreads();
      take_equal = 1;
      return pat;
    }
    // many equal scores: more than half of the entries still share all digits
    // known so far, and lanes with equal digits are merged into one atomic
    const bool concentrated = 2 * (int64_t)n_match > hi - lo;
    for (int i = tid; i < 4096; i += 1024) rs.hist12[i] = 0;
    __syncthreads();
    if (in_lds) {
      for (int i = tid; i < n_cand; i += 1024) {
        const uint64_t key = rs.cand[i];
        if ((key & known) == pat) atomicAdd(&rs.hist12[(unsigned)(key >> shift) & 4095u], 1u);
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
          const unsigned digit = (unsigned)(key[r] >> shift) & 4095u;
          if (concentrated) hist_add_merged(rs.hist12, hit, digit);
          else if (hit) atomicAdd(&rs.hist12[digit], 1u);
        }
      }
    }
    __syncthreads();
    pick_bin12(rs.hist12, rs, remaining);
    n_match = rs.n_bin;   // entries that share all digits known after this pass
    pat |= (uint64_t)rs.bin << shift;
    known |= 0xfffull << shift;
    remaining = rs.rem;
    __syncthreads();
  }
  take_equal = remaining;
  return pat;
}

// Bit pattern of the count-th largest score inside [lo, hi), and how many of
// the entries equal to it belong to the top `count` (lowest index first).
// Radix select on 12-bit digits, most significant first.  Every digit costs a
// sweep over the scores, so
//  - the first sweep takes bits 48-59 (the low eight exponent bits and four of
//    the fraction): scores are means of softmax weights, their leading four
//    bits are the same for all of them and say nothing, while this digit
//    spreads them over sixteen bins per octave.  The sweep also checks that
//    bits 60-63 are indeed common to all keys; if not, it is discarded and a
//    sweep on those four bits comes first;
//  - as soon as the entries that still share the threshold's known digits fit
//    RADIX_CAND, one more sweep copies their bit patterns to LDS and the
//    remaining digits are settled there; when a single entry is left, it is
//    the answer.
// Typically two or three sweeps.  Called by all 1024 threads of a block.
// The scores are read through `sc`, anything indexable that yields the double
// at a position (an array, or a view of listed columns).
template <typename SC>
__device__ __forceinline__ uint64_t radix_threshold(SC sc, int lo, int hi, int count,
                                                    RadixScratch &rs, int &take_equal) {
  const int tid = threadIdx.x, lane = tid & 63;
  uint64_t pat = 0, known = 0;
  int remaining = count;
  int n_match = hi - lo;   // entries that share all known digits
  int shift = 36;
  // a range that fits the candidate buffer is read from memory once: its keys
  // stay in LDS for all the digits
  const bool keep = hi - lo <= RADIX_CAND;
  {
    for (int i = tid; i < 4096; i += 1024) rs.hist12[i] = 0;
    if (tid == 0) rs.top_and = 15u, rs.top_or = 0u;
    __syncthreads();
    unsigned t_and = 15u, t_or = 0u;
    for (int j0 = lo; j0 < hi; j0 += SWEEP_U * 1024) {
      uint64_t key[SWEEP_U];
#pragma unroll
      for (int r = 0; r < SWEEP_U; ++r) key[r] = score_key(sc[min(j0 + r * 1024 + tid, hi - 1)]);
#pragma unroll
      for (int r = 0; r < SWEEP_U; ++r) {
        if (j0 + r * 1024 + tid < hi) {
          if (keep) rs.cand[j0 + r * 1024 + tid - lo] = key[r];
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
    const bool common = rs.top_and == rs.top_or;
    if (common) {
      pick_bin12(rs.hist12, rs, remaining);
      pat = ((uint64_t)rs.top_and << 60) | ((uint64_t)rs.bin << 48);
      known = 0xffffull << 48;
    } else {
      // the leading four bits differ: settle them first (a handful of values:
      // lanes with equal digits are merged into one atomic)
      __syncthreads();
      for (int i = tid; i < 4096; i += 1024) rs.hist12[i] = 0;
      __syncthreads();
      for (int j0 = lo; j0 < hi; j0 += SWEEP_U * 1024) {
        uint64_t key[SWEEP_U];
#pragma unroll
        for (int r = 0; r < SWEEP_U; ++r) key[r] = score_key(sc[min(j0 + r * 1024 + tid, hi - 1)]);
#pragma unroll
        for (int r = 0; r < SWEEP_U; ++r)
          hist_add_merged(rs.hist12, j0 + r * 1024 + tid < hi, (unsigned)(key[r] >> 60));
      }
      __syncthreads();
      pick_bin12(rs.hist12, rs, remaining);
      pat = (uint64_t)rs.bin << 60;
      known = 0xfull << 60;
      shift = 48;
    }
    remaining = rs.rem;
    n_match = rs.n_bin;
    __syncthreads();
  }
  return radix_finish(sc, lo, hi, rs, pat, known, shift, remaining, n_match, take_equal, keep ? hi - lo : 0);
}

// Ascending list of the indices j in [lo, hi) that `classify(j, sc[j])` marks: 1 = listed,
// 2 = listed while fewer than take_equal entries of class 2 precede it (ties of
// a threshold go to the lower index), 0 = not listed.  Returns the list's
// length.  Every wave of the 1024-thread block owns a contiguous sixteenth of
// the range: one sweep counts, a block-wide exchange of the sixteen totals
// gives every wave its place, a second sweep writes -- no barrier inside the
// sweeps.  s_cnt: 32 ints of LDS.
// When [lo, hi) is one slice of a longer range that several blocks list
// together, base1 / base2 are the class-1 / class-2 entries of the slices
// before it: they shift the output position and use up the take_equal quota.
template <typename SC, typename F>
__device__ __forceinline__ int list_ascending(SC sc, int lo, int hi, int take_equal,
                                              int32_t *__restrict__ out, int *s_cnt, F classify,
                                              int base1 = 0, int base2 = 0) {
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
  int run1 = base1, run2 = base2, tot1 = 0, tot2 = 0;
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
        out[before1 + min(before2, take_equal)] = position_of(sc, j0 + 64 * r + lane);
      run1 += __popcll(b1);
      run2 += __popcll(b2);
    }
  }
  return tot1 + min(base2 + tot2, take_equal) - min(base2, take_equal);
}

// A classifier may class the SWEEP_U x 64 consecutive entries a wave holds at
// once -- wave_masks(first entry, lane, the lane's scores, hi, class-1 masks,
// class-2 masks), one mask per run of 64 -- instead of entry by entry: for
// tests that look at an entry's neighbours.
template <typename F, typename = void>
struct classifies_by_wave : std::false_type {};
template <typename F>
struct classifies_by_wave<F, std::void_t<decltype(F::BY_WAVE)>> : std::true_type {};

// list_ascending with every score read once: the range is taken in chunks of
// 1024 * SWEEP_U entries that the block holds in registers between counting
// and writing (two barriers per chunk; every wave owns a contiguous sixteenth
// of the chunk).  For blocks that list one slice of a unit.  Returns the number
// of entries this call listed; n_class2: the class-2 entries it met.  Nothing is
// written at or past out[limit], whatever the bases claim.
template <typename SC, typename F>
__device__ __forceinline__ int list_chunked(SC sc, int lo, int hi, int take_equal, int32_t *__restrict__ out,
                                            int limit, int *s_cnt, F classify, int base1, int base2,
                                            int &n_class2) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const uint64_t below = (1ull << lane) - 1ull;
  int run1 = base1, run2 = base2;   // the same in every thread
  for (int j0 = lo; j0 < hi; j0 += 1024 * SWEEP_U) {
    const int jw = j0 + wv * 64 * SWEEP_U;
    double x[SWEEP_U];
#pragma unroll
    for (int r = 0; r < SWEEP_U; ++r) x[r] = sc[min(jw + 64 * r + lane, hi - 1)];
    uint64_t b1[SWEEP_U], b2[SWEEP_U];
    int n1 = 0, n2 = 0;
    if constexpr (classifies_by_wave<F>::value) {
      classify.wave_masks(jw, lane, x, hi, b1, b2);
    } else {
#pragma unroll
      for (int r = 0; r < SWEEP_U; ++r) {
        const int j = jw + 64 * r + lane;
        const int cls = j < hi ? classify(j, x[r]) : 0;
        b1[r] = __ballot(cls == 1);
        b2[r] = __ballot(cls == 2);
      }
    }
#pragma unroll
    for (int r = 0; r < SWEEP_U; ++r) {
      n1 += __popcll(b1[r]);
      n2 += __popcll(b2[r]);
    }
    __syncthreads();   // s_cnt may still be read from the chunk before
    if (lane == 0) {
      s_cnt[wv] = n1;
      s_cnt[16 + wv] = n2;
    }
    __syncthreads();
    int w1 = run1, w2 = run2;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
      const int c1 = s_cnt[w], c2 = s_cnt[16 + w];
      if (w < wv) w1 += c1, w2 += c2;
      run1 += c1;
      run2 += c2;
    }
#pragma unroll
    for (int r = 0; r < SWEEP_U; ++r) {
      const bool m1 = (b1[r] >> lane) & 1ull, m2 = (b2[r] >> lane) & 1ull;
      const int before1 = w1 + __popcll(b1[r] & below), before2 = w2 + __popcll(b2[r] & below);
      const int at = before1 + min(before2, take_equal);
      if ((m1 || (m2 && before2 < take_equal)) && at < limit) out[at] = position_of(sc, jw + 64 * r + lane);
      w1 += __popcll(b1[r]);
      w2 += __popcll(b2[r]);
    }
  }
  n_class2 = run2 - base2;
  return (run1 - base1) + min(run2, take_equal) - min(base2, take_equal);
}

// The two class counts of list_ascending over [lo, hi), without listing
// anything (all 1024 threads; the counts are returned to every thread).
template <typename SC, typename F>
__device__ __forceinline__ void count_classes(SC sc, int lo, int hi, int *s_cnt, F classify, int &n1, int &n2) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  int c1 = 0, c2 = 0;
  for (int j0 = lo + wv * 64 * SWEEP_U; j0 < hi; j0 += 16 * 64 * SWEEP_U) {
    double x[SWEEP_U];
#pragma unroll
    for (int r = 0; r < SWEEP_U; ++r) x[r] = sc[min(j0 + 64 * r + lane, hi - 1)];
#pragma unroll
    for (int r = 0; r < SWEEP_U; ++r) {
      const int j = j0 + 64 * r + lane;
      const int cls = j < hi ? classify(j, x[r]) : 0;
      c1 += __popcll(__ballot(cls == 1));
      c2 += __popcll(__ballot(cls == 2));
    }
  }
  __syncthreads();
  if (lane == 0) {
    s_cnt[wv] = c1;
    s_cnt[16 + wv] = c2;
  }
  __syncthreads();
  n1 = n2 = 0;
#pragma unroll
  for (int w = 0; w < 16; ++w) {
    n1 += s_cnt[w];
    n2 += s_cnt[16 + w];
  }
}

// 1 = above the threshold, 2 = equal to it.
struct AboveOrAt {
  uint64_t pat;
  __device__ __forceinline__ int operator()(int, double x) const {
    const uint64_t key = score_key(x);
    return key > pat ? 1 : (key == pat ? 2 : 0);
  }
};

// One block selects for one unit: the `count` largest scores inside [lo, hi) by
// (score desc, index asc), written as  [0, prefix) ++ picks ascending ++ (gap
// slots left for the caller) ++ [N - suffix, N)  with the rest of the row -1.
// With a list of columns (`listed`, n_listed of them, ascending) the picks are
// taken among the listed columns only: [lo, hi) is ignored.  All 1024 threads;
// s_cnt: 32 ints of LDS.
__device__ __forceinline__ void select_of_unit(const double *__restrict__ sc, int32_t *__restrict__ orow, int N, int lo,
                                               int hi, int count, int prefix, int gap, int suffix, int out_stride,
                                               const int32_t *__restrict__ listed, int n_listed, RadixScratch &rs,
                                               int *s_cnt) {
  const int tid = threadIdx.x;
  if (count > 0) {
    // pat = the count-th largest score; `remaining` of the entries equal to it
    // are taken, lowest index first.
    auto pick = [&](auto view, int a, int b) {
      int remaining;
      const uint64_t pat = radix_threshold(view, a, b, count, rs, remaining);
      list_ascending(view, a, b, remaining, orow + prefix, s_cnt, AboveOrAt{pat});
    };
    if (listed != nullptr) pick(ListedScores{sc, listed}, 0, n_listed);
    else pick(sc, lo, hi);
  }
  for (int i = tid; i < prefix; i += 1024) orow[i] = i;
  for (int i = tid; i < suffix; i += 1024) orow[prefix + count + gap + i] = N - suffix + i;
  for (int i = prefix + count + gap + suffix + tid; i < out_stride; i += 1024) orow[i] = -1;
}

}  // namespace taskkv
