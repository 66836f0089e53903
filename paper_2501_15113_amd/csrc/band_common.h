// Pieces the one-block and the sliced band kernels of the screening pass share:
// the error bound of the fp32 scores and the test that lists a column.
#pragma once

#include <math.h>

#include "select_common.h"
#include "taskkv_internal.h"

namespace taskkv {

// Largest squared norm of a unit's window rows (fp64 rows of the separator).
// All 1024 threads; s_q: 16 doubles of LDS; ends with a barrier.
__device__ __forceinline__ double max_row_norm2(const double *__restrict__ qd, int unit, const Dims &dm, double *s_q) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, D = dm.D;
  double qmax = 0.0;
  for (int r0 = wv; r0 < dm.R; r0 += 16 * 8) {
    // eight rows of the wave at a time: sixteen loads in flight, not two
    double e[8][2];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = r0 + 16 * i;
      const double *row = qd + ((size_t)unit * dm.Rpad + (r < dm.R ? r : r0)) * D;
      e[i][0] = row[lane];
      e[i][1] = D > 64 ? row[64 + lane] : 0.0;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      double ss = fma(e[i][0], e[i][0], e[i][1] * e[i][1]);
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
      qmax = fmax(qmax, ss);   // a row past R repeats row r0
    }
  }
  if (lane == 0) s_q[wv] = qmax;
  __syncthreads();
  qmax = 0.0;
  for (int i = 0; i < 16; ++i) qmax = fmax(qmax, s_q[i]);
  __syncthreads();
  return qmax;
}

// 1 = in the band: columns at or above lo_t, and middle columns inside
// [lo_k, hi_k].  2 = a middle column outside the band and above it: not listed,
// and certainly above the middle threshold.
struct InBand {
  double lo_t, lo_k, hi_k;
  int m0, m1;   // the middle [m0, m1); empty when no middle threshold is wanted
  __device__ __forceinline__ int operator()(int j, double x) const {
    if (x >= lo_t) return 1;
    if (j >= m0 && j < m1) return x > hi_k ? 2 : (x >= lo_k ? 1 : 0);
    return 0;
  }
};

__host__ __device__ __forceinline__ bool band_has_middle(const Dims &dm) {
  return dm.pack_mode == TASKKV_PACK_SELECTIVE && !dm.keep_all && dm.k > 0 && dm.k < dm.N - dm.s1 - dm.s2;
}

// The band around the two thresholds: three times the relative error bound of
// the fp32 scores, from the measured norms (qmax, kmax: largest squared norms
// of a window row and of a key).  The thresholds of the fp32 scores may be
// given as brackets: tau_t is any value at or below the top-t threshold, and
// the middle threshold lies in [tau_k_lo, tau_k_hi]; a wider bracket lists more
// columns and loses nothing.
__device__ __forceinline__ InBand band_limits(const Dims &dm, double qmax, double kmax, double tau_t, double tau_k_lo,
                                              double tau_k_hi) {
  const double gamma = 4.0 * dm.D * 5.9604644775390625e-08;   // 4 d 2^-24
  const double eps = dm.scale * gamma * sqrt(qmax) * sqrt(kmax) + 2e-5 + dm.R * 1.2e-7;
  const double w3 = 3.0 * eps;
  const bool middle = band_has_middle(dm);
  InBand b;
  // values below 1e-30 may have been flushed to zero by the fp32 pass: treat them as ties
  b.lo_t = w3 >= 1.0 ? -1.0 : tau_t * (1.0 - w3) - 1e-30;
  b.lo_k = w3 >= 1.0 ? -1.0 : tau_k_lo * (1.0 - w3) - 1e-30;
  b.hi_k = w3 >= 1.0 ? INFINITY : tau_k_hi * (1.0 + w3) + 1e-30;
  b.m0 = middle ? dm.s1 : 0;
  b.m1 = middle ? dm.N - dm.s2 : 0;
  return b;
}

// One block lists the band of one unit: error bound, the two thresholds of the
// fp32 scores, the columns to recompute (ascending) and their number.  All
// 1024 threads; s_cnt: 32 ints, s_q: 16 doubles of LDS.
__device__ __forceinline__ void band_of_unit(const double *__restrict__ sc, const double *__restrict__ qd, double kmax,
                                             int unit, const Dims &dm, int32_t *__restrict__ list,
                                             int32_t *__restrict__ count, RadixScratch &rs, int *s_cnt, double *s_q) {
  const int N = dm.N;
  const double qmax = max_row_norm2(qd, unit, dm, s_q);
  int unused;
  const double tau_t = __longlong_as_double((long long)radix_threshold(sc, 0, N, dm.T, rs, unused));
  double tau_k = 0.0;
  if (band_has_middle(dm))
    tau_k = __longlong_as_double((long long)radix_threshold(sc, dm.s1, N - dm.s2, dm.k, rs, unused));
  const InBand band = band_limits(dm, qmax, kmax, tau_t, tau_k, tau_k);
  const int listed = list_ascending(sc, 0, N, 0, list, s_cnt, band);
  if (threadIdx.x == 0) *count = listed;
}

}  // namespace taskkv
