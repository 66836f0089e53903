// The selections of select.hip and the band of score_screen.hip with a unit's
// scores cut into slices that several blocks sweep at once.
//
// A sweep over the scores of all units is a pass over up to 64 MB; with one
// block per unit a selection takes six to eight of them, each at the speed of
// 8-64 blocks.  Here every phase is a kernel of S blocks per unit and the
// scores are read three or four times:
//   clear    the per-unit histograms and counters;
//   hist1    12-bit digit histogram (bits 48-59 of the fp64 pattern: sixteen
//            bins per octave over [2^-255, 2), anything smaller in bin 0,
//            anything larger in bin 4095) of a slice, added to the unit's;
//   hist2    histogram of the next twelve bits of the entries in the bin that
//            holds the wanted rank.
// A selection (top-t of unscreened scores, the middle pick) skips hist2 unless
// the wanted bin has more entries than the candidate list takes, and goes on:
//   gather   every block finds the wanted bin from the unit's histograms,
//            appends its slice's entries of that bin (pattern and position) to
//            the unit's candidate list and counts its entries in higher bins;
//   settle   one block per unit settles the remaining digits on the candidate
//            list -> threshold pattern and how many entries equal to it are
//            taken; the candidates' positions give every slice's share;
//   write    every block lists its slice's picks behind those of the slices
//            before it (ascending positions, ties to the lower index).
// The band of the screening pass wants two thresholds at once (top-t and the
// middle pick, from the same reads) but only to within a fraction of its own
// width: the two digits bracket each to 2^-16 of itself, so it goes on with
//   brackets the wanted bins of both levels -> the brackets, and the largest
//            window-row norm for the error bound;
//   write    every block lists its slice's band columns from the slice's first
//            slot of the row and counts the middle columns above the band;
//   close    one block per unit closes the gaps between the slices' lists.
// The compressor's middle pick on screened scores then needs no sweep to find
// its threshold: every middle column the band leaves out is above it (counted)
// or below it, so the threshold is the (k - columns above)-th largest listed
// score (mlist_settle), and `write` lists the picks.
// Results do not depend on the order in which blocks run: histograms and
// candidate lists are only counted, never read in order.  A unit whose wanted
// rank falls into one of the two mixed end bins, or whose wanted bin still
// holds too many entries after the second digit (thousands of equal scores),
// is flagged and left to one block, as in the one-block kernels.
#include <math.h>

#include "band_common.h"
#include "select_common.h"

namespace taskkv {

// View of a list of fp64 bit patterns as scores.
struct KeyArray {
  const unsigned long long *k;
  __device__ __forceinline__ double operator[](int j) const { return __longlong_as_double((long long)k[j]); }
};
__device__ __forceinline__ int position_of(const KeyArray &, int j) { return j; }

// Entries per slice when [0, N) is cut into S slices (whole rounds of 64).
__host__ __device__ __forceinline__ int slice_len(int N, int S) { return (((N + S - 1) / S) + 63) & ~63; }
__device__ __forceinline__ void slice_of(int N, int s, int S, int &a, int &b) {
  const int seg = slice_len(N, S);
  a = min(N, s * seg);
  b = min(N, a + seg);
}

__device__ __forceinline__ size_t counts_at(int unit, int s) { return ((size_t)unit * MSEL_MAX_SLICES + s) * 2; }
__device__ __forceinline__ size_t hist_at(int level, int sel, int unit, int units) {
  return ((size_t)(level * 2 + sel) * units + unit) * 4096;
}

// Scores a thread holds per round of a slice's sweep (sixteen measured slower
// than eight: 18.9 against 16.5 us for the first histogram of the largest
// workload, 8.4 against 5.9 us where a slice is 2048 entries); the first
// round's loads are issued before the block's preparations (clearing LDS,
// looking up the wanted bin) so that both overlap.
constexpr int SLICE_U = 8;

constexpr unsigned long long DIGIT1_BASE = 0x3000ull;   // leading 16 bits of 2^-255
__device__ __forceinline__ int digit1(uint64_t key) {
  const long long d = (long long)(key >> 48) - (long long)DIGIT1_BASE;
  return d < 0 ? 0 : (d > 4095 ? 4095 : (int)d);
}
__device__ __forceinline__ int digit2(uint64_t key) { return (int)(key >> 36) & 4095; }

// LDS of a block that looks up a wanted bin.
struct PickScratch {
  int wsum[16];
  int bin, rem, n_bin;
};

// What a unit's histograms say about one selection: the digits of the wanted
// entry known so far, its rank among the entries that share them and how many
// those are.  Every block of the unit derives the same answer.
struct Wanted {
  uint64_t pat, known;
  int rem, n;
  bool redo;     // leave the unit to the one-block kernel
  bool level2;   // the second digit is needed (and, after hist2, known)
};

// Level 1 only.  All 1024 threads; ps is overwritten.
__device__ __forceinline__ Wanted wanted_level1(const MSelBufs &mb, int sel, int unit, int units, PickScratch &ps) {
  __syncthreads();   // ps may still be read from the call before
  pick_bin12(mb.hist + hist_at(0, sel, unit, units), ps, mb.count[sel]);
  Wanted w;
  const int bin = ps.bin;
  w.n = ps.n_bin;
  w.rem = ps.rem;
  w.pat = (DIGIT1_BASE + (unsigned long long)bin) << 48;
  w.known = 0xffffull << 48;
  w.redo = bin == 0 || bin == 4095 || w.n == 0;
  w.level2 = !w.redo && (w.n > MSEL_CAND || mb.bracket);
  return w;
}

// Both levels.
__device__ __forceinline__ Wanted wanted_bin(const MSelBufs &mb, int sel, int unit, int units, PickScratch &ps) {
  Wanted w = wanted_level1(mb, sel, unit, units, ps);
  if (!w.level2) return w;   // the same in every thread
  __syncthreads();
  pick_bin12(mb.hist + hist_at(1, sel, unit, units), ps, w.rem);
  w.n = ps.n_bin;
  w.rem = ps.rem;
  w.pat |= (unsigned long long)ps.bin << 36;
  w.known |= 0xfffull << 36;
  w.redo = w.n == 0 || (w.n > MSEL_CAND && !mb.bracket);
  return w;
}

__global__ void msel_clear_kernel(MSelBufs mb, int units) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < (size_t)4 * units * 4096) mb.hist[i] = 0u;
  if (i < (size_t)2 * units) mb.n_cand[i] = 0;
  if (i < (size_t)units) mb.flag[i] = 0;
}

// scores1: what the second threshold ranks by when that is not `scores` (the
// pooled scores of a middle pick that pools), else null.
__global__ __launch_bounds__(1024) void msel_hist1_kernel(const double *__restrict__ scores,
                                                          const double *__restrict__ scores1,
                                                          const uint8_t *__restrict__ skip, MSelBufs mb, int N) {
  const int s = blockIdx.x, unit = blockIdx.y, units = gridDim.y, tid = threadIdx.x;
  if (skip && skip[unit]) return;
  const double *sc = scores + (size_t)unit * N;
  int a, b;
  slice_of(N, s, mb.S, a, b);
  if (a >= b) return;
  // Two thresholds on the same scores: the second one's range lies inside the
  // first one's (the middle of the context inside the whole of it), so an entry
  // is counted once, in the lower half if only the first range holds it, else
  // in the upper half, and the first threshold's histogram is the sum of the
  // two.  On different scores each half is a histogram of its own.
  __shared__ unsigned h[2 * 4096];
  const bool two = mb.nsel > 1, split = two && scores1 != nullptr;
  const double *sc1 = split ? scores1 + (size_t)unit * N : sc;
  for (int j0 = a; j0 < b; j0 += SLICE_U * 1024) {
    uint64_t key[SLICE_U], key1[SLICE_U];
#pragma unroll
    for (int r = 0; r < SLICE_U; ++r) key[r] = score_key(sc[min(j0 + r * 1024 + tid, b - 1)]);
    if (split) {
#pragma unroll
      for (int r = 0; r < SLICE_U; ++r) key1[r] = score_key(sc1[min(j0 + r * 1024 + tid, b - 1)]);
    }
    if (j0 == a) {   // with the first loads in flight
      for (int i = tid; i < 2 * 4096; i += 1024) h[i] = 0;
      __syncthreads();
    }
#pragma unroll
    for (int r = 0; r < SLICE_U; ++r) {
      const int j = j0 + r * 1024 + tid;
      if (j < b) {
        const int d = digit1(key[r]);
        const bool in1 = two && j >= mb.lo[1] && j < mb.hi[1], in0 = j >= mb.lo[0] && j < mb.hi[0];
        if (split) {
          if (in1) atomicAdd(&h[4096 + digit1(key1[r])], 1u);
          if (in0) atomicAdd(&h[d], 1u);
        } else if (in1) {
          atomicAdd(&h[4096 + d], 1u);
        } else if (in0) {
          atomicAdd(&h[d], 1u);
        }
      }
    }
  }
  __syncthreads();
  unsigned *g0 = mb.hist + hist_at(0, 0, unit, units), *g1 = mb.hist + hist_at(0, 1, unit, units);
  for (int i = tid; i < 4096; i += 1024) {
    const unsigned inner = h[4096 + i], all = split ? h[i] : h[i] + inner;
    if (all) atomicAdd(&g0[i], all);
    if (inner) atomicAdd(&g1[i], inner);   // only with two thresholds
  }
}

__global__ __launch_bounds__(1024) void msel_hist2_kernel(const double *__restrict__ scores,
                                                          const double *__restrict__ scores1,
                                                          const uint8_t *__restrict__ skip, MSelBufs mb, int N) {
  const int s = blockIdx.x, unit = blockIdx.y, units = gridDim.y, tid = threadIdx.x;
  if (skip && skip[unit]) return;
  __shared__ PickScratch ps;
  __shared__ unsigned h[2 * 4096];
  Wanted w[2];
  w[0] = wanted_level1(mb, 0, unit, units, ps);
  w[1] = w[0];
  w[1].level2 = false;
  if (mb.nsel > 1) w[1] = wanted_level1(mb, 1, unit, units, ps);
  // a unit that will be redone anyway needs no second digit
  if (w[0].redo || (mb.nsel > 1 && w[1].redo) || (!w[0].level2 && !w[1].level2)) return;
  const double *sc = scores + (size_t)unit * N;
  int a, b;
  slice_of(N, s, mb.S, a, b);
  if (a >= b) return;
  for (int i = tid; i < 2 * 4096; i += 1024) h[i] = 0;
  __syncthreads();
  const bool split = mb.nsel > 1 && scores1 != nullptr;
  const double *sc1 = split ? scores1 + (size_t)unit * N : sc;
  for (int j0 = a; j0 < b; j0 += SWEEP_U * 1024) {
    uint64_t key[2][SWEEP_U];
#pragma unroll
    for (int r = 0; r < SWEEP_U; ++r) key[0][r] = score_key(sc[min(j0 + r * 1024 + tid, b - 1)]);
#pragma unroll
    for (int r = 0; r < SWEEP_U; ++r) key[1][r] = split ? score_key(sc1[min(j0 + r * 1024 + tid, b - 1)]) : key[0][r];
#pragma unroll
    for (int r = 0; r < SWEEP_U; ++r) {
      const int j = j0 + r * 1024 + tid;
      if (j < b) {
#pragma unroll
        for (int sel = 0; sel < 2; ++sel)
          if (w[sel].level2 && j >= mb.lo[sel] && j < mb.hi[sel] && (key[sel][r] & w[sel].known) == w[sel].pat)
            atomicAdd(&h[sel * 4096 + digit2(key[sel][r])], 1u);
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int sel = 0; sel < 2; ++sel) {
    if (sel >= mb.nsel || !w[sel].level2) continue;
    unsigned *g = mb.hist + hist_at(1, sel, unit, units);
    for (int i = tid; i < 4096; i += 1024)
      if (h[sel * 4096 + i]) atomicAdd(&g[i], h[sel * 4096 + i]);
  }
}

__global__ __launch_bounds__(1024) void msel_gather_kernel(const double *__restrict__ scores,
                                                           const uint8_t *__restrict__ skip, MSelBufs mb, int N) {
  const int s = blockIdx.x, unit = blockIdx.y, units = gridDim.y, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  if (skip && skip[unit]) return;
  __shared__ PickScratch ps;
  __shared__ int s_w[16];
  __shared__ int s_base;
  const double *sc = scores + (size_t)unit * N;
  const uint64_t below = (1ull << lane) - 1ull;
  int a, b;
  slice_of(N, s, mb.S, a, b);
  Wanted w[2];
  int above = 0;   // entries of selection 0 in higher bins, counted per wave
  for (int j0 = a; j0 < b; j0 += SLICE_U * 1024) {
    const int jw = j0 + wv * 64 * SLICE_U;
    uint64_t key[SLICE_U];
#pragma unroll
    for (int r = 0; r < SLICE_U; ++r) key[r] = score_key(sc[min(jw + 64 * r + lane, b - 1)]);
    if (j0 == a) {   // with the first loads in flight
      w[0] = wanted_bin(mb, 0, unit, units, ps);
      w[1] = w[0];
      if (mb.nsel > 1) w[1] = wanted_bin(mb, 1, unit, units, ps);
      if (w[0].redo || w[1].redo) {   // the same for every block of the unit
        if (s == 0 && tid == 0) mb.flag[unit] = 1;
        return;
      }
      if (s == 0 && tid == 0) {
#pragma unroll
        for (int sel = 0; sel < 2; ++sel) {
          if (sel >= mb.nsel) break;
          mb.take[sel * units + unit] = w[sel].rem;
          mb.wpat[sel * units + unit] = w[sel].pat;
          mb.wshift[sel * units + unit] = w[sel].level2 ? 24 : 36;
        }
      }
    }
#pragma unroll
    for (int sel = 0; sel < 2; ++sel) {
      if (sel >= mb.nsel) break;
      const size_t su = (size_t)sel * units + unit;
      uint64_t hit[SLICE_U];
      int n_hit = 0;
#pragma unroll
      for (int r = 0; r < SLICE_U; ++r) {
        const int j = jw + 64 * r + lane;
        const bool in = j < b && j >= mb.lo[sel] && j < mb.hi[sel];
        const uint64_t part = key[r] & w[sel].known;
        hit[r] = __ballot(in && part == w[sel].pat);
        n_hit += __popcll(hit[r]);
        if (sel == 0) above += __popcll(__ballot(in && part > w[0].pat));
      }
      __syncthreads();   // s_w, s_base may still be read from the round before
      if (lane == 0) s_w[wv] = n_hit;
      __syncthreads();
      if (tid == 0) {
        int tot = 0;
        for (int i = 0; i < 16; ++i) tot += s_w[i];
        s_base = tot ? atomicAdd(&mb.n_cand[su], tot) : 0;   // one atomic per block and round
      }
      __syncthreads();
      int at = s_base;
      for (int i = 0; i < wv; ++i) at += s_w[i];
#pragma unroll
      for (int r = 0; r < SLICE_U; ++r) {
        if ((hit[r] >> lane) & 1ull) {
          const size_t p = su * MSEL_CAND + at + __popcll(hit[r] & below);
          mb.cand_key[p] = key[r];
          mb.cand_idx[p] = jw + 64 * r + lane;
        }
        at += __popcll(hit[r]);
      }
    }
  }
  __syncthreads();
  if (lane == 0) s_w[wv] = above;
  __syncthreads();
  if (tid == 0) {
    int tot = 0;
    for (int i = 0; i < 16; ++i) tot += s_w[i];
    mb.n_above[(size_t)unit * MSEL_MAX_SLICES + s] = tot;
  }
}

// Threshold of one selection of a unit from its candidate list: the pattern of
// the wanted entry and how many entries equal to it are taken.  The list's
// entries share their leading digits; the others are settled in LDS.  All 1024
// threads.
__device__ __forceinline__ uint64_t settle(const MSelBufs &mb, size_t su, RadixScratch &rs, int &take_equal) {
  const KeyArray view{mb.cand_key + su * MSEL_CAND};
  const int shift = mb.wshift[su], n = mb.n_cand[su];
  return radix_finish(view, 0, n, rs, mb.wpat[su], ~0ull << (shift + 12), shift, mb.take[su], n, take_equal);
}

// One block per unit: the threshold, and the picks of every slice (entries in
// higher bins + candidates above / at the threshold).
__global__ __launch_bounds__(1024) void msel_settle_kernel(const uint8_t *__restrict__ skip, MSelBufs mb, Dims dm) {
  const int unit = blockIdx.x, tid = threadIdx.x;
  if ((skip && skip[unit]) || mb.flag[unit]) return;
  __shared__ RadixScratch rs;
  __shared__ int c[2 * MSEL_MAX_SLICES];
  int take_equal;
  const uint64_t pat = settle(mb, unit, rs, take_equal);
  if (tid < 2 * MSEL_MAX_SLICES) c[tid] = 0;
  __syncthreads();
  const int seg = slice_len(dm.N, mb.S), n = mb.n_cand[unit];
  for (int i = tid; i < n; i += 1024) {
    const uint64_t key = mb.cand_key[(size_t)unit * MSEL_CAND + i];
    const int sl = mb.cand_idx[(size_t)unit * MSEL_CAND + i] / seg;
    if (key > pat) atomicAdd(&c[sl], 1);
    else if (key == pat) atomicAdd(&c[MSEL_MAX_SLICES + sl], 1);
  }
  __syncthreads();
  if (tid < mb.S) {
    mb.counts[counts_at(unit, tid)] = mb.n_above[(size_t)unit * MSEL_MAX_SLICES + tid] + c[tid];
    mb.counts[counts_at(unit, tid) + 1] = c[MSEL_MAX_SLICES + tid];
  }
  if (tid == 0) {
    mb.pat[unit] = pat;
    mb.take_final[unit] = take_equal;
  }
}

// The band needs no exact thresholds of the fp32 scores, only brackets: the
// two digits of the histograms place each within 2^-16 of itself, less than
// the band's own width.  Three blocks per unit: the two brackets and the largest
// squared norm of a window row.
__global__ __launch_bounds__(1024) void mband_brackets_kernel(MSelBufs mb, Dims dm, const double *__restrict__ qd) {
  const int unit = blockIdx.x, units = gridDim.x, what = blockIdx.y, tid = threadIdx.x;
  if (what == 2) {
    __shared__ double s_q[16];
    const double qmax = max_row_norm2(qd, unit, dm, s_q);
    if (tid == 0) mb.band[(size_t)2 * units + unit] = qmax;
    return;
  }
  if (what >= mb.nsel) return;
  __shared__ PickScratch ps;
  const Wanted w = wanted_bin(mb, what, unit, units, ps);
  if (tid == 0) {
    if (w.redo) mb.flag[unit] = 1;
    mb.band[(size_t)what * units + unit] = __longlong_as_double((long long)w.pat);   // the bracket's lower end
  }
}

// Row layout as select_kernel writes it: [0, prefix) ++ picks ++ gap ++ [N - suffix, N) ++ -1 padding.
__global__ __launch_bounds__(1024) void msel_write_kernel(const double *__restrict__ scores,
                                                          const uint8_t *__restrict__ skip, MSelBufs mb, int N,
                                                          int prefix, int gap, int suffix, int32_t *__restrict__ out,
                                                          int out_stride) {
  const int s = blockIdx.x, unit = blockIdx.y, tid = threadIdx.x;
  int32_t *orow = out + (size_t)unit * out_stride;
  if (skip && skip[unit]) {
    if (s == 0)
      for (int i = tid; i < out_stride; i += 1024) orow[i] = -1;
    return;
  }
  __shared__ int s_cnt[32];
  if (mb.flag[unit]) {   // the sliced kernels gave up on this unit: its first block selects alone
    __shared__ RadixScratch rs;
    if (s == 0)
      select_of_unit(scores + (size_t)unit * N, orow, N, mb.lo[0], mb.hi[0], mb.count[0], prefix, gap, suffix,
                     out_stride, nullptr, 0, rs, s_cnt);
    return;
  }
  // picks of the slices before mine: all counts in one trip to memory
  __shared__ int s_n[2 * MSEL_MAX_SLICES];
  if (tid < 2 * s) s_n[tid] = mb.counts[counts_at(unit, tid >> 1) + (tid & 1)];
  __syncthreads();
  int base1 = 0, base2 = 0;
  for (int x = 0; x < s; ++x) {
    base1 += s_n[2 * x];
    base2 += s_n[2 * x + 1];
  }
  int a, b;
  slice_of(N, s, mb.S, a, b);
  a = max(a, mb.lo[0]);
  b = min(b, mb.hi[0]);
  int unused;
  list_chunked(scores + (size_t)unit * N, a, b, mb.take_final[unit], orow + prefix, mb.count[0], s_cnt,
               AboveOrAt{mb.pat[unit]}, base1, base2, unused);
  if (s == 0) {
    const int count = mb.count[0];
    for (int i = tid; i < prefix; i += 1024) orow[i] = i;
    for (int i = tid; i < suffix; i += 1024) orow[prefix + count + gap + i] = N - suffix + i;
    for (int i = prefix + count + gap + suffix + tid; i < out_stride; i += 1024) orow[i] = -1;
  }
}

// The band of a middle pick that pools: its threshold is one of the pooled
// scores, and a pooled score that has to be decided exactly needs the exact
// scores of all the columns under its pooling window.  Lists the columns at or
// above lo_t and those within `radius` of a middle column whose pooled score
// lies inside [lo_k, hi_k] (1); 2 = a middle column that is not listed and
// whose pooled score is above the band.  (A listed column outside the band
// keeps a pooled score that is only fp32-accurate, and still on the same side
// of the middle threshold as its exact value.)
struct InBandPooled {
  InBand b;
  const double *pooled;   // the unit's row
  int radius;
  __device__ __forceinline__ int operator()(int j, double x) const {
    int hit = x >= b.lo_t ? 1 : 0, above = 0;
    const int i0 = max(j - radius, b.m0), i1 = min(j + radius, b.m1 - 1);
    for (int i = i0; i <= i1; ++i) {
      const double p = pooled[i];
      hit |= (p >= b.lo_k && p <= b.hi_k) ? 1 : 0;
      above |= (i == j && p > b.hi_k) ? 1 : 0;
    }
    return hit ? 1 : (above ? 2 : 0);
  }
};

// The same test for a whole wave's SWEEP_U x 64 consecutive columns: every
// column's own pooled score gives one bit (in the band or not), and "within
// `radius` of a set bit" is shifts and ors of the 64-bit masks, with the
// neighbouring runs' bits carried in and `radius` columns of halo on either
// side of the wave's span -- one read of the pooled scores per column, all of
// them in flight together, where the test column by column makes 2 radius + 1
// dependent trips.  radius <= 31.
struct InBandPooledWave {
  static constexpr bool BY_WAVE = true;
  InBand b;
  const double *pooled;   // the unit's row
  int radius;
  __device__ __forceinline__ void wave_masks(int jw, int lane, const double (&x)[SWEEP_U], int hi,
                                             uint64_t (&b1)[SWEEP_U], uint64_t (&b2)[SWEEP_U]) const {
    uint64_t kb[SWEEP_U], live[SWEEP_U];
    double p[SWEEP_U];
#pragma unroll
    for (int r = 0; r < SWEEP_U; ++r) {
      const int j = jw + 64 * r + lane;
      p[r] = pooled[min(max(j, b.m0), b.m1 - 1)];
    }
    // halo, one load: lanes [0, radius) take the columns before the span, lanes
    // [32, 32 + radius) those behind it; bit u of `left` is column
    // jw - radius + u, bit u of `right` column jw + 64 SWEEP_U + u
    const int hl = lane & 31, hcol = lane < 32 ? jw - radius + hl : jw + 64 * SWEEP_U + hl;
    const double hp = pooled[min(max(hcol, b.m0), b.m1 - 1)];   // (no branch around it: it travels with the loads above)
    const uint64_t halo = __ballot(hl < radius && hcol >= b.m0 && hcol < b.m1 && hp >= b.lo_k && hp <= b.hi_k);
    const uint64_t left = halo & 0xffffffffull, right = halo >> 32;
#pragma unroll
    for (int r = 0; r < SWEEP_U; ++r) {
      const int j = jw + 64 * r + lane;
      const bool mid = j >= b.m0 && j < b.m1;
      live[r] = __ballot(j < hi);
      kb[r] = __ballot(mid && p[r] >= b.lo_k && p[r] <= b.hi_k);
      b1[r] = __ballot(x[r] >= b.lo_t);
      b2[r] = __ballot(mid && p[r] > b.hi_k);
    }
#pragma unroll
    for (int r = 0; r < SWEEP_U; ++r) {
      const uint64_t prev = r > 0 ? kb[r - 1] : left << (64 - radius);
      const uint64_t next = r < SWEEP_U - 1 ? kb[r + 1] : right;
      uint64_t d = kb[r];
      for (int u = 1; u <= radius; ++u) d |= (kb[r] << u) | (kb[r] >> u) | (prev >> (64 - u)) | (next << (64 - u));
      b1[r] = (b1[r] | d) & live[r];
      b2[r] = b2[r] & ~b1[r] & live[r];
    }
  }
};

// The band's columns of a slice, listed from the slice's first slot of the row.
__global__ __launch_bounds__(1024) void mband_write_kernel(const double *__restrict__ scores,
                                                           const double *__restrict__ pooled,
                                                           const unsigned long long *__restrict__ knorm, MSelBufs mb,
                                                           Dims dm, int32_t *__restrict__ band_idx,
                                                           int *__restrict__ above_band) {
  const int s = blockIdx.x, unit = blockIdx.y, units = gridDim.y, tid = threadIdx.x;
  if (mb.flag[unit]) return;
  __shared__ int s_cnt[32];
  const uint64_t rest = (1ull << 36) - 1ull;   // the digits the brackets leave open
  const double tau_k = mb.nsel > 1 ? mb.band[(size_t)units + unit] : 0.0;
  const InBand band =
      band_limits(dm, mb.band[(size_t)2 * units + unit], __longlong_as_double((long long)knorm[unit]), mb.band[unit],
                  tau_k, __longlong_as_double((long long)(score_key(tau_k) | rest)));
  int a, b;
  slice_of(dm.N, s, mb.S, a, b);
  int n_above = 0, n;
  const double *sc = scores + (size_t)unit * dm.N;
  int32_t *out = band_idx + (size_t)unit * dm.N + a;
  if (pooled != nullptr && mb.nsel > 1 && dm.pool / 2 <= 31)
    n = list_chunked(sc, a, b, 0, out, b - a, s_cnt, InBandPooledWave{band, pooled + (size_t)unit * dm.N, dm.pool / 2},
                     0, 0, n_above);
  else if (pooled != nullptr && mb.nsel > 1)
    n = list_chunked(sc, a, b, 0, out, b - a, s_cnt, InBandPooled{band, pooled + (size_t)unit * dm.N, dm.pool / 2}, 0,
                     0, n_above);
  else
    n = list_chunked(sc, a, b, 0, out, b - a, s_cnt, band, 0, 0, n_above);
  if (tid == 0) {
    mb.counts[counts_at(unit, s)] = n;
    above_band[(size_t)unit * MSEL_MAX_SLICES + s] = n_above;
  }
}

// Closes the gaps between the slices' lists of a row (a list only ever moves
// towards the row's start, chunk by chunk through registers).
__global__ __launch_bounds__(1024) void mband_close_kernel(const double *__restrict__ scores,
                                                           const double *__restrict__ qd,
                                                           const unsigned long long *__restrict__ knorm, MSelBufs mb,
                                                           Dims dm, int32_t *__restrict__ band_idx,
                                                           int32_t *__restrict__ band_cnt, int *__restrict__ list_ok,
                                                           int pooled) {
  const int unit = blockIdx.x, tid = threadIdx.x, N = dm.N;
  if (tid == 0) list_ok[unit] = mb.flag[unit] ? 0 : 1;
  if (mb.flag[unit]) {   // the sliced kernels gave up on this unit: one block lists its band, without slice counts
    __shared__ RadixScratch rs;
    __shared__ int s_cnt[32];
    __shared__ double s_q[16];
    if (pooled) {
      // with pooling the one-block band has no list of neighbours to offer:
      // every column of such a unit (degenerate scores) is recomputed
      for (int i = tid; i < N; i += 1024) band_idx[(size_t)unit * N + i] = i;
      if (tid == 0) band_cnt[unit] = N;
      return;
    }
    band_of_unit(scores + (size_t)unit * N, qd, __longlong_as_double((long long)knorm[unit]), unit, dm,
                 band_idx + (size_t)unit * N, band_cnt + unit, rs, s_cnt, s_q);
    return;
  }
  int32_t *row = band_idx + (size_t)unit * N;
  const int seg = slice_len(N, mb.S);
  __shared__ int s_n[MSEL_MAX_SLICES];   // one trip to memory for all counts
  if (tid < mb.S) s_n[tid] = mb.counts[counts_at(unit, tid)];
  __syncthreads();
  int total = 0;
  for (int s = 0; s < mb.S; ++s) total += s_n[s];
  constexpr int CLOSE_U = 8;
  if (total <= 1024 * CLOSE_U) {
    // the usual case, a few thousand columns: every thread reads its entries of
    // the closed list from wherever their slices put them, then all write
    int32_t v[CLOSE_U];
    int s = 0, before = 0;   // slice of the thread's current entry (its entries ascend)
#pragma unroll
    for (int i = 0; i < CLOSE_U; ++i) {
      const int p = tid + 1024 * i;
      while (s < mb.S - 1 && p >= before + s_n[s]) before += s_n[s++];
      v[i] = p < total ? row[min(N, s * seg) + (p - before)] : 0;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < CLOSE_U; ++i)
      if (tid + 1024 * i < total) row[tid + 1024 * i] = v[i];
  } else {
    total = s_n[0];
    for (int s = 1; s < mb.S; ++s) {
      const int c = s_n[s];
      const int32_t *src = row + min(N, s * seg);
      int32_t *dst = row + total;
      if (dst != src) {
        for (int off = 0; off < c; off += 1024) {
          const int32_t v = off + tid < c ? src[off + tid] : 0;
          __syncthreads();
          if (off + tid < c) dst[off + tid] = v;
          __syncthreads();
        }
      }
      total += c;
    }
  }
  if (tid == 0) band_cnt[unit] = total;
}

// ---- launchers
// The sliced kernels hold one 1024-thread block per compute unit at a time
// (registers), and a block's fixed costs -- a few dependent trips to memory,
// two barriers -- are most of what it takes on a slice of a few thousand
// scores: one block per compute unit in all, two where a slice would otherwise
// exceed two sweeps of a block (32 units of 32768 scores: the band and the
// selections together 20 us faster with 8 slices than with 16).
static int msel_slices(const Dims &dm, int n_cu) {
  int S = n_cu / dm.units;
  if (S >= 1 && dm.N / S > 2 * 1024 * SWEEP_U) S *= 2;
  return S < 1 ? 1 : (S > MSEL_MAX_SLICES ? MSEL_MAX_SLICES : S);
}
static bool msel_sized(const Dims &dm) { return dm.N >= MSEL_MIN_RANGE && dm.units <= MSEL_MAX_UNITS; }

// Long ranges on few units; elsewhere the extra launches cost more than the
// idle compute units.  Measured on 8 and 32 units, separator and compressor
// together: sliced 7-36 us slower at 8192 scores, 4-5 us faster at 12288, 7-16 us
// at 16384, 14-19 us at 24000.
bool msel_pays(const Dims &dm, int n_cu, int lo, int hi, int count) {
  return msel_sized(dm) && hi - lo >= MSEL_MIN_RANGE && count > 0 && count < hi - lo && msel_slices(dm, n_cu) >= 2;
}

static size_t al256(size_t b) { return (b + 255) & ~size_t(255); }

size_t msel_workspace_bytes(const Dims &dm) {
  if (!msel_sized(dm)) return 0;
  const size_t u = dm.units;
  return al256(4 * u * 4096 * 4) + al256(2 * u * MSEL_CAND * 8) + al256(2 * u * MSEL_CAND * 4) + 3 * al256(2 * u * 4) + al256(2 * u * 8) +
         al256(u * 4) + al256(u * MSEL_MAX_SLICES * 4) + al256(u * 8) + al256(u * 4) +
         al256(u * MSEL_MAX_SLICES * 2 * 4) + al256(u * 3 * 8);
}

bool msel_carve(Carver &cv, const Dims &dm, MSelBufs &mb) {
  mb.hist = nullptr;
  if (!msel_sized(dm)) return false;
  const size_t u = dm.units;
  mb.hist = cv.take<unsigned>(4 * u * 4096);
  mb.cand_key = cv.take<unsigned long long>(2 * u * MSEL_CAND);
  mb.cand_idx = cv.take<int32_t>(2 * u * MSEL_CAND);
  mb.n_cand = cv.take<int>(2 * u);
  mb.take = cv.take<int>(2 * u);
  mb.wpat = cv.take<unsigned long long>(2 * u);
  mb.wshift = cv.take<int>(2 * u);
  mb.flag = cv.take<int>(u);
  mb.n_above = cv.take<int>(u * MSEL_MAX_SLICES);
  mb.pat = cv.take<unsigned long long>(u);
  mb.take_final = cv.take<int>(u);
  mb.counts = cv.take<int>(u * MSEL_MAX_SLICES * 2);
  mb.band = cv.take<double>(u * 3);
  return cv.ok;
}

// What msel_clear_kernel clears.
void msel_zero_words(const Dims &dm, const MSelBufs &mb, ZeroList &z) {
  z.add(mb.hist, (size_t)4 * dm.units * 4096);
  z.add(mb.n_cand, (size_t)2 * dm.units);
  z.add(mb.flag, (size_t)dm.units);
}

static void msel_histograms(const Dims &dm, const double *scores, const uint8_t *skip, const MSelBufs &mb,
                            hipStream_t s, bool cleared = false, const double *scores1 = nullptr) {
  const size_t n = (size_t)4 * dm.units * 4096;
  if (!cleared) msel_clear_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(mb, dm.units);
  const dim3 grid(mb.S, dm.units), block(1024);
  msel_hist1_kernel<<<grid, block, 0, s>>>(scores, scores1, skip, mb, dm.N);
  msel_hist2_kernel<<<grid, block, 0, s>>>(scores, scores1, skip, mb, dm.N);
}
static void msel_candidates(const Dims &dm, const double *scores, const uint8_t *skip, const MSelBufs &mb,
                            hipStream_t s) {
  msel_histograms(dm, scores, skip, mb, s);
  msel_gather_kernel<<<dim3(mb.S, dm.units), dim3(1024), 0, s>>>(scores, skip, mb, dm.N);
}

int launch_select_sliced(const Dims &dm, int n_cu, MSelBufs mb, const double *scores, const uint8_t *skip_mask, int lo,
                         int hi, int count, int prefix, int gap, int suffix, int32_t *out, int out_stride,
                         hipStream_t s) {
  mb.S = msel_slices(dm, n_cu);
  mb.nsel = 1;
  mb.bracket = 0;
  mb.lo[0] = lo; mb.hi[0] = hi; mb.count[0] = count;
  mb.lo[1] = mb.hi[1] = mb.count[1] = 0;
  msel_candidates(dm, scores, skip_mask, mb, s);
  msel_settle_kernel<<<dim3(dm.units), dim3(1024), 0, s>>>(skip_mask, mb, dm);
  msel_write_kernel<<<dim3(mb.S, dm.units), dim3(1024), 0, s>>>(scores, skip_mask, mb, dm.N, prefix, gap, suffix, out,
                                                             out_stride);
  return hip_ok(hipGetLastError());
}

int launch_band_sliced(const Dims &dm, int n_cu, MSelBufs mb, const double *scores, const double *pooled,
                       const double *qd, const unsigned long long *knorm, int32_t *band_idx, int32_t *band_cnt, int *above_band,
                       int *list_ok, bool cleared, hipStream_t s) {
  mb.S = msel_slices(dm, n_cu);
  mb.nsel = band_has_middle(dm) ? 2 : 1;
  mb.lo[0] = 0; mb.hi[0] = dm.N; mb.count[0] = dm.T;
  mb.lo[1] = dm.s1; mb.hi[1] = dm.N - dm.s2; mb.count[1] = dm.k;
  mb.bracket = 1;
  if (mb.nsel < 2) pooled = nullptr;   // pooling only concerns the middle pick
  msel_histograms(dm, scores, nullptr, mb, s, cleared, pooled);
  mband_brackets_kernel<<<dim3(dm.units, 3), dim3(1024), 0, s>>>(mb, dm, qd);
  mband_write_kernel<<<dim3(mb.S, dm.units), dim3(1024), 0, s>>>(scores, pooled, knorm, mb, dm, band_idx, above_band);
  mband_close_kernel<<<dim3(dm.units), dim3(1024), 0, s>>>(scores, qd, knorm, mb, dm, band_idx, band_cnt, list_ok,
                                                         pooled != nullptr ? 1 : 0);
  return hip_ok(hipGetLastError());
}

// One block per unit: the middle threshold from the band's list.  The columns
// of the middle that the list leaves out are either above the band (counted
// per slice when the list was written) or below it, so the k-th largest score
// of the middle is the (k - columns above)-th largest of the listed ones.
__global__ __launch_bounds__(1024) void mlist_settle_kernel(const double *__restrict__ scores,
                                                            const uint8_t *__restrict__ skip, MSelBufs mb, Dims dm,
                                                            const int32_t *__restrict__ band_idx,
                                                            const int32_t *__restrict__ band_cnt,
                                                            const int *__restrict__ above_band,
                                                            const int *__restrict__ list_ok) {
  const int unit = blockIdx.x, tid = threadIdx.x;
  if (skip && skip[unit]) {
    if (tid == 0) mb.flag[unit] = 0;
    return;
  }
  if (!list_ok[unit]) {
    if (tid == 0) mb.flag[unit] = 1;
    return;
  }
  const int N = dm.N;
  const double *sc = scores + (size_t)unit * N;
  const int32_t *list = band_idx + (size_t)unit * N;
  const int n = band_cnt[unit];
  // The list indexes the scores: it has to be what the band kernels write
  // (ascending columns inside the row), or the full selection decides.  The
  // same pass counts the entries before the middle and before its end: the
  // listed columns of the middle are entries [ia, ib) of the ascending list
  // (a binary search would be two dozen dependent trips to memory).
  __shared__ int s_below[2];
  if (tid < 2) s_below[tid] = 0;
  __syncthreads();
  {
    bool bad = n < 0 || n > N;
    int b1 = 0, b2 = 0;
    // (SWEEP_U entries of a thread in flight at once: a loop that looks at one
    // entry per trip is a chain of memory latencies, eight of them for a list
    // of 8192 columns)
    for (int i0 = tid; i0 < n && !bad; i0 += 1024 * SWEEP_U) {
      int v[SWEEP_U], before[SWEEP_U];
#pragma unroll
      for (int r = 0; r < SWEEP_U; ++r) {
        const int i = min(i0 + 1024 * r, n - 1);
        v[r] = list[i];
        before[r] = i > 0 ? list[i - 1] : -1;
      }
#pragma unroll
      for (int r = 0; r < SWEEP_U; ++r) {
        if (i0 + 1024 * r >= n) continue;
        bad = bad || v[r] < 0 || v[r] >= N || before[r] >= v[r];
        b1 += v[r] < dm.s1 ? 1 : 0;
        b2 += v[r] < N - dm.s2 ? 1 : 0;
      }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      b1 += __shfl_xor(b1, off);
      b2 += __shfl_xor(b2, off);
    }
    if ((tid & 63) == 0 && (b1 | b2)) {
      atomicAdd(&s_below[0], b1);
      atomicAdd(&s_below[1], b2);
    }
    if (__syncthreads_or(bad)) {
      if (tid == 0) mb.flag[unit] = 1;
      return;
    }
  }
  const int ia = s_below[0], ib = s_below[1];
  // the slices' counts of middle columns above the band: one lane each (a loop
  // over them in every thread is a chain of up to 64 memory latencies)
  static_assert(MSEL_MAX_SLICES <= 64, "one wave adds up the slices' counts");
  __shared__ int s_above;
  if (tid < 64) {
    int a = tid < mb.S ? above_band[(size_t)unit * MSEL_MAX_SLICES + tid] : 0;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) a += __shfl_xor(a, off);
    if (tid == 0) s_above = a;
  }
  __syncthreads();
  const int need = dm.k - s_above;
  if (need < 1 || need > ib - ia) {   // not while the band's bound holds; the full selection decides then
    if (tid == 0) mb.flag[unit] = 1;
    return;
  }
  __shared__ RadixScratch rs;
  __shared__ int c[2 * MSEL_MAX_SLICES];
  int take_equal;
  const ListedScores view{sc, list};
  const uint64_t pat = radix_threshold(view, ia, ib, need, rs, take_equal);
  if (tid < 2 * MSEL_MAX_SLICES) c[tid] = 0;
  __syncthreads();
  const int seg = slice_len(N, mb.S);
  for (int i0 = ia + tid; i0 < ib; i0 += 1024 * SWEEP_U) {
    int j[SWEEP_U];
    uint64_t key[SWEEP_U];
#pragma unroll
    for (int r = 0; r < SWEEP_U; ++r) j[r] = list[min(i0 + 1024 * r, ib - 1)];
#pragma unroll
    for (int r = 0; r < SWEEP_U; ++r) key[r] = score_key(sc[j[r]]);
#pragma unroll
    for (int r = 0; r < SWEEP_U; ++r) {
      if (i0 + 1024 * r >= ib) continue;
      if (key[r] > pat) atomicAdd(&c[j[r] / seg], 1);
      else if (key[r] == pat) atomicAdd(&c[MSEL_MAX_SLICES + j[r] / seg], 1);
    }
  }
  __syncthreads();
  if (tid < mb.S) {
    mb.counts[counts_at(unit, tid)] = above_band[(size_t)unit * MSEL_MAX_SLICES + tid] + c[tid];
    mb.counts[counts_at(unit, tid) + 1] = c[MSEL_MAX_SLICES + tid];
  }
  if (tid == 0) {
    mb.pat[unit] = pat;
    mb.take_final[unit] = take_equal;
    mb.flag[unit] = 0;
  }
}

int launch_select_from_band(const Dims &dm, int n_cu, MSelBufs mb, const double *scores, const uint8_t *skip_mask,
                            const int32_t *band_idx, const int32_t *band_cnt, const int *above_band,
                            const int *list_ok, int32_t *out, hipStream_t s) {
  mb.S = msel_slices(dm, n_cu);
  mb.nsel = 1;
  mb.bracket = 0;
  mb.lo[0] = dm.s1; mb.hi[0] = dm.N - dm.s2; mb.count[0] = dm.k;
  mb.lo[1] = mb.hi[1] = mb.count[1] = 0;
  mlist_settle_kernel<<<dim3(dm.units), dim3(1024), 0, s>>>(scores, skip_mask, mb, dm, band_idx, band_cnt, above_band,
                                                           list_ok);
  msel_write_kernel<<<dim3(mb.S, dm.units), dim3(1024), 0, s>>>(scores, skip_mask, mb, dm.N, dm.s1, 0, dm.s2, out,
                                                             dm.row_stride);
  return hip_ok(hipGetLastError());
}

}  // namespace taskkv
