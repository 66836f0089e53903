// Window scores in fp64 on the vector ALUs (paper Sec. 4.1, Eq. 12-13): the
// fallback for window/group sizes the matrix-core scorer does not cover.
//
// Two passes over K.  Pass "stats" finds, for every window row, the row maximum
// and the softmax denominator; pass "mean" recomputes the logits and
// accumulates the column mean C.  Re-reading K (2*d bytes per key) is cheaper
// than spilling the G*L logits per key.  Every product and sum is fp64 on the
// vector ALUs; one thread owns one key column and keeps its K row in registers,
// the window rows arrive as wave-uniform loads.
#include <math.h>

#include "taskkv_internal.h"

namespace taskkv {

__device__ __forceinline__ float elem_to_float(float x) { return x; }
__device__ __forceinline__ float elem_to_float(uint16_t x) { return __uint_as_float(uint32_t(x) << 16); }

// q_win [B, Hq, L, D] -> qd [unit][Rpad][D] fp64, rows r = g*L + i, zero padded.
template <typename T>
__global__ void q_to_f64_kernel(const T *__restrict__ q, double *__restrict__ qd, Dims dm) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t total = (size_t)dm.units * dm.Rpad * dm.D;
  if (idx >= total) return;
  int c = idx % dm.D;
  size_t rest = idx / dm.D;
  int r = rest % dm.Rpad;
  int unit = rest / dm.Rpad;
  double val = 0.0;
  if (r < dm.R) {
    int b = unit / dm.Hkv, h = unit % dm.Hkv, g = r / dm.L, i = r % dm.L;
    size_t src = (((size_t)b * dm.Hq + h * dm.G + g) * dm.L + i) * dm.D + c;
    val = (double)elem_to_float(q[src]);
  }
  qd[idx] = val;
}

template <int D>
__device__ __forceinline__ void load_row(const float *p, float (&kr)[D]) {
  const float4 *p4 = reinterpret_cast<const float4 *>(p);
#pragma unroll
  for (int i = 0; i < D / 4; ++i) {
    float4 x = p4[i];
    kr[4 * i] = x.x; kr[4 * i + 1] = x.y; kr[4 * i + 2] = x.z; kr[4 * i + 3] = x.w;
  }
}
template <int D>
__device__ __forceinline__ void load_row(const uint16_t *p, float (&kr)[D]) {
  const uint4 *p4 = reinterpret_cast<const uint4 *>(p);
#pragma unroll
  for (int i = 0; i < D / 8; ++i) {
    uint4 x = p4[i];
    uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      kr[8 * i + 2 * e] = __uint_as_float(w[e] << 16);
      kr[8 * i + 2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
    }
  }
}

constexpr int MAX_R = 1024;

// MODE 0: per-(unit, chunk) row statistics -> part[unit][chunk][Rpad][2].
// MODE 1: column mean -> scores[unit][N], using stats[unit][Rpad][2].
template <typename T, int D, int MODE>
__global__ __launch_bounds__(256) void score_f64_kernel(const T *__restrict__ k,
                                                        const double *__restrict__ qd,
                                                        const double *__restrict__ stats,
                                                        double *__restrict__ part,
                                                        double *__restrict__ scores, Dims dm,
                                                        int tiles_per_wg, int n_chunks) {
  const int unit = blockIdx.y, chunk = blockIdx.x, tid = threadIdx.x;
  const int N = dm.N, L = dm.L, R = dm.R, Rpad = dm.Rpad;
  const T *kb = k + (size_t)unit * N * D;
  const double *qb = qd + (size_t)unit * Rpad * D;
  const double *st = stats + (size_t)unit * Rpad * 2;

  __shared__ double sl[MODE == 0 ? ROW_BLK : 1][SCORE_TILE];
  __shared__ double run_m[MODE == 0 ? MAX_R : 1], run_l[MODE == 0 ? MAX_R : 1];
  if (MODE == 0) {
    for (int r = tid; r < Rpad; r += 256) { run_m[r] = -INFINITY; run_l[r] = 0.0; }
    __syncthreads();
  }

  for (int tile = 0; tile < tiles_per_wg; ++tile) {
    const int jb = (chunk * tiles_per_wg + tile) * SCORE_TILE;
    if (jb >= N) break;
    const int j = jb + tid;
    const bool valid = j < N;
    float kr[D];
    if (valid) {
      load_row<D>(kb + (size_t)j * D, kr);
    } else {
#pragma unroll
      for (int c = 0; c < D; ++c) kr[c] = 0.f;
    }
    double cacc = 0.0;
    for (int r0 = 0; r0 < Rpad; r0 += ROW_BLK) {
      double acc[ROW_BLK];
#pragma unroll
      for (int r = 0; r < ROW_BLK; ++r) acc[r] = 0.0;
      const double *qr = qb + (size_t)r0 * D;
#pragma unroll
      for (int c = 0; c < D; ++c) {
        const double kc = (double)kr[c];
#pragma unroll
        for (int r = 0; r < ROW_BLK; ++r) acc[r] = fma(qr[r * D + c], kc, acc[r]);
      }
#pragma unroll
      for (int r = 0; r < ROW_BLK; ++r) {
        const int row = r0 + r;
        const int i = row % L;
        const bool vis = valid && row < R && j <= N - L + i;
        const double s = acc[r] * dm.scale;
        if (MODE == 0) {
          sl[r][tid] = vis ? s : -INFINITY;
        } else if (vis) {
          cacc += exp(s - st[2 * row]) / st[2 * row + 1];
        }
      }
      if (MODE == 0) {
        __syncthreads();
        const int row = tid >> 5, ln = tid & 31;
        double mx = -INFINITY;
#pragma unroll
        for (int e = 0; e < SCORE_TILE / 32; ++e) mx = fmax(mx, sl[row][ln + 32 * e]);
#pragma unroll
        for (int off = 16; off >= 1; off >>= 1) mx = fmax(mx, __shfl_xor(mx, off));
        double sm = 0.0;
        if (mx > -INFINITY) {
#pragma unroll
          for (int e = 0; e < SCORE_TILE / 32; ++e) sm += exp(sl[row][ln + 32 * e] - mx);
        }
#pragma unroll
        for (int off = 16; off >= 1; off >>= 1) sm += __shfl_xor(sm, off);
        if (ln == 0 && mx > -INFINITY) {
          const int rr = r0 + row;
          const double m0 = run_m[rr];
          const double mn = fmax(m0, mx);
          run_l[rr] = run_l[rr] * exp(m0 - mn) + sm * exp(mx - mn);
          run_m[rr] = mn;
        }
        __syncthreads();
      }
    }
    if (MODE == 1 && valid) scores[(size_t)unit * N + j] = cacc / (double)R;
  }
  if (MODE == 0) {
    __syncthreads();
    double *pp = part + ((size_t)unit * n_chunks + chunk) * Rpad * 2;
    for (int r = tid; r < Rpad; r += 256) { pp[2 * r] = run_m[r]; pp[2 * r + 1] = run_l[r]; }
  }
}

// Fixed-order merge of the per-chunk row statistics.
__global__ void merge_stats_kernel(const double *__restrict__ part, double *__restrict__ stats,
                                   int Rpad, int n_chunks) {
  const int unit = blockIdx.x;
  for (int r = threadIdx.x; r < Rpad; r += blockDim.x) {
    double m = -INFINITY, l = 0.0;
    for (int c = 0; c < n_chunks; ++c) {
      const double *pp = part + (((size_t)unit * n_chunks + c) * Rpad + r) * 2;
      const double mc = pp[0], lc = pp[1];
      if (mc > -INFINITY) {
        const double mn = fmax(m, mc);
        l = l * exp(m - mn) + lc * exp(mc - mn);
        m = mn;
      }
    }
    stats[((size_t)unit * Rpad + r) * 2] = m;
    stats[((size_t)unit * Rpad + r) * 2 + 1] = l;
  }
}

template <typename T, int D>
static int run_scores(const Dims &dm, const T *k, double *qd, double *part, double *stats,
                      double *scores, int tiles_per_wg, hipStream_t s) {
  const int n_tiles = (dm.N + SCORE_TILE - 1) / SCORE_TILE;
  const int n_chunks = (n_tiles + tiles_per_wg - 1) / tiles_per_wg;
  dim3 grid(n_chunks, dm.units);
  score_f64_kernel<T, D, 0><<<grid, dim3(256), 0, s>>>(k, qd, stats, part, scores, dm, tiles_per_wg, n_chunks);
  merge_stats_kernel<<<dim3(dm.units), dim3(256), 0, s>>>(part, stats, dm.Rpad, n_chunks);
  score_f64_kernel<T, D, 1><<<grid, dim3(256), 0, s>>>(k, qd, stats, part, scores, dm, tiles_per_wg, n_chunks);
  return hip_ok(hipGetLastError());
}

int launch_q_to_f64(const Dims &dm, int dtype, const void *q_win, double *qd, hipStream_t s) {
  const size_t total = (size_t)dm.units * dm.Rpad * dm.D;
  const dim3 grid((unsigned)((total + 255) / 256)), block(256);
  if (dtype == TASKKV_F32)
    q_to_f64_kernel<float><<<grid, block, 0, s>>>(static_cast<const float *>(q_win), qd, dm);
  else
    q_to_f64_kernel<uint16_t><<<grid, block, 0, s>>>(static_cast<const uint16_t *>(q_win), qd, dm);
  return hip_ok(hipGetLastError());
}

int launch_merge_stats(const double *part, double *stats, int units, int Rpad, int n_parts, hipStream_t s) {
  merge_stats_kernel<<<dim3(units), dim3(256), 0, s>>>(part, stats, Rpad, n_parts);
  return hip_ok(hipGetLastError());
}

int launch_scores_f64(const Dims &dm, int dtype, const void *k, double *qd, double *stat_part,
                      double *stats, double *scores, int tiles_per_wg, hipStream_t s) {
  if (dtype == TASKKV_F32) {
    auto kk = static_cast<const float *>(k);
    return dm.D == 64 ? run_scores<float, 64>(dm, kk, qd, stat_part, stats, scores, tiles_per_wg, s)
                      : run_scores<float, 128>(dm, kk, qd, stat_part, stats, scores, tiles_per_wg, s);
  }
  auto kk = static_cast<const uint16_t *>(k);
  return dm.D == 64 ? run_scores<uint16_t, 64>(dm, kk, qd, stat_part, stats, scores, tiles_per_wg, s)
                    : run_scores<uint16_t, 128>(dm, kk, qd, stat_part, stats, scores, tiles_per_wg, s);
}

}  // namespace taskkv
