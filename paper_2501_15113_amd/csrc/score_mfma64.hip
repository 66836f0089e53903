// Window scores in fp64 on the matrix cores (paper Sec. 4.1, Eq. 12-13).
//
// Same two passes as the vector-ALU scorer (row statistics, then column mean),
// same arithmetic (every product, sum and exponential in fp64), but the
// Q.K^T contraction runs on v_mfma_f64_16x16x4_f64: a wave keeps two 16-row
// blocks of the window in registers as A operands (fp64, 2 * d/4 values per
// lane) and streams 16-key tiles of K as B operand, converting bf16/fp32 to
// fp64 on the fly.  The contraction index is permuted so that every lane reads
// one contiguous d/4-element piece of its key row.
//
// Lane layout of the instruction (l = lane): A[i][k] in lane i + 16 k,
// B[k][j] in lane j + 16 k, D[4 v + l / 16][l % 16] in register v (checked on
// the device with distinct-valued operands).
//
// Pass 0 keeps per-lane online softmax statistics for the lane's 8 rows (one
// exponential per logit), merges the 16 key lanes at the end of the wave's key
// range and writes one partial per (block, key slice, row); pass 1 writes each
// (row pair, key) column sum to LDS exactly once and adds the row pairs in index
// order, so the result does not depend on scheduling.
#include <math.h>

#include "taskkv_internal.h"

namespace taskkv {

typedef double f64x4 __attribute__((ext_vector_type(4)));

constexpr int SKC = 256;   // keys per chunk
constexpr int SNW = 8;     // waves per block: with <= 8 row pairs every pair streams the same K tiles
                           // at the same time, so K comes from HBM once per pass
constexpr int MAXP = 16;   // row pairs (32 rows each) one block can hold column sums for

template <int NKK>
__device__ __forceinline__ void fetch_piece(const uint16_t *p, bool ok, uint4 (&raw)[NKK / 8]) {
#pragma unroll
  for (int i = 0; i < NKK / 8; ++i)
    raw[i] = ok ? reinterpret_cast<const uint4 *>(p)[i] : make_uint4(0, 0, 0, 0);
}
template <int NKK>
__device__ __forceinline__ void fetch_piece(const float *p, bool ok, uint4 (&raw)[NKK / 4]) {
#pragma unroll
  for (int i = 0; i < NKK / 4; ++i)
    raw[i] = ok ? reinterpret_cast<const uint4 *>(p)[i] : make_uint4(0, 0, 0, 0);
}
template <int NKK>
__device__ __forceinline__ void widen_piece(const uint4 (&raw)[NKK / 8], double (&b)[NKK], const uint16_t *) {
#pragma unroll
  for (int i = 0; i < NKK / 8; ++i) {
    const uint32_t w[4] = {raw[i].x, raw[i].y, raw[i].z, raw[i].w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      b[8 * i + 2 * e] = (double)__uint_as_float(w[e] << 16);
      b[8 * i + 2 * e + 1] = (double)__uint_as_float(w[e] & 0xffff0000u);
    }
  }
}
template <int NKK>
__device__ __forceinline__ void widen_piece(const uint4 (&raw)[NKK / 4], double (&b)[NKK], const float *) {
#pragma unroll
  for (int i = 0; i < NKK / 4; ++i) {
    b[4 * i] = (double)__uint_as_float(raw[i].x);
    b[4 * i + 1] = (double)__uint_as_float(raw[i].y);
    b[4 * i + 2] = (double)__uint_as_float(raw[i].z);
    b[4 * i + 3] = (double)__uint_as_float(raw[i].w);
  }
}

template <typename T> struct RawCount;
template <> struct RawCount<uint16_t> { static constexpr int per16B = 8; };
template <> struct RawCount<float> { static constexpr int per16B = 4; };

// MODE 0: row statistics -> part[unit][n_parts][Rpad][2], n_parts = gridDim.x * ksplit.
// MODE 1: column mean -> scores[unit][N] from stats[unit][Rpad][2].
template <typename T, int D, int MODE>
__global__ __launch_bounds__(64 * SNW) void score_mfma64_kernel(const T *__restrict__ k,
                                                           const double *__restrict__ qd,
                                                           const double *__restrict__ stats,
                                                           double *__restrict__ part,
                                                           double *__restrict__ scores, Dims dm,
                                                           int chunks_per_wg) {
  constexpr int NKK = D / 4;
  constexpr int NRAW = NKK / RawCount<T>::per16B;
  const int unit = blockIdx.y, tid = threadIdx.x, w = tid >> 6, l = tid & 63, c = l & 15, kq = l >> 4;
  const int N = dm.N, L = dm.L, R = dm.R, Rpad = dm.Rpad;
  const int n_pairs = Rpad / 32;
  const int ksplit = n_pairs >= SNW ? 1 : SNW / n_pairs;
  const int n_items = n_pairs * ksplit;
  const int sub = SKC / ksplit;  // keys per slice of a chunk
  const T *kb = k + (size_t)unit * N * D;
  const double *qb = qd + (size_t)unit * Rpad * D;
  const double *st = stats + (size_t)unit * Rpad * 2;
  const double scale = dm.scale;

  __shared__ double cs[MODE == 1 ? MAXP : 1][SKC];

  double a[2][NKK];
  int cur_pair = -1;
  auto load_a = [&](int pair) {
    if (pair == cur_pair) return;
    cur_pair = pair;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
      const double *row = qb + (size_t)(32 * pair + 16 * rb + c) * D + NKK * kq;
#pragma unroll
      for (int kk = 0; kk < NKK; ++kk) a[rb][kk] = row[kk];
    }
  };

  // logits of one 16-key tile for the wave's two row blocks
  auto tile_logits = [&](int j0, bool &valid, f64x4 (&acc)[2]) {
    const int j = j0 + c;
    valid = j < N;
    uint4 raw[NRAW];
    fetch_piece<NKK>(kb + (size_t)(valid ? j : 0) * D + NKK * kq, valid, raw);
    double b[NKK];
    widen_piece<NKK>(raw, b, (const T *)nullptr);
    acc[0] = f64x4{0., 0., 0., 0.};
    acc[1] = f64x4{0., 0., 0., 0.};
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
      acc[0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[0][kk], b[kk], acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[1][kk], b[kk], acc[1], 0, 0, 0);
    }
  };

  if (MODE == 0) {
    const int n_parts = gridDim.x * ksplit;
    for (int item = w; item < n_items; item += SNW) {
      const int pair = item % n_pairs, ks = item / n_pairs;
      load_a(pair);
      double m[8], ls[8];
#pragma unroll
      for (int s = 0; s < 8; ++s) { m[s] = -INFINITY; ls[s] = 0.0; }
      for (int ch = 0; ch < chunks_per_wg; ++ch) {
        const int jc = (blockIdx.x * chunks_per_wg + ch) * SKC + ks * sub;
        if (jc >= N) break;
        for (int j0 = jc; j0 < jc + sub && j0 < N; j0 += 16) {
          bool valid;
          f64x4 acc[2];
          tile_logits(j0, valid, acc);
          const int j = j0 + c;
#pragma unroll
          for (int s = 0; s < 8; ++s) {
            const int row = 32 * pair + 16 * (s >> 2) + 4 * (s & 3) + kq;
            const bool vis = valid && row < R && j <= N - L + row % L;
            if (vis) {
              // one exponential per logit, no divergent branch: e = exp(-|t - m|)
              const double t = acc[s >> 2][s & 3] * scale;
              const bool up = t > m[s];
              const double e = exp(up ? m[s] - t : t - m[s]);
              ls[s] = up ? ls[s] * e + 1.0 : ls[s] + e;
              m[s] = up ? t : m[s];
            }
          }
        }
      }
      // merge the 16 key lanes of every row slot
#pragma unroll
      for (int s = 0; s < 8; ++s) {
#pragma unroll
        for (int off = 1; off < 16; off <<= 1) {
          const double mo = __shfl_xor(m[s], off), lo = __shfl_xor(ls[s], off);
          const double mn = fmax(m[s], mo);
          if (mn > -INFINITY) ls[s] = ls[s] * exp(m[s] - mn) + lo * exp(mo - mn);
          m[s] = mn;
        }
      }
      if (c == 0) {
        double *pp = part + ((size_t)unit * n_parts + (size_t)blockIdx.x * ksplit + ks) * Rpad * 2;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          const int row = 32 * pair + 16 * (s >> 2) + 4 * (s & 3) + kq;
          pp[2 * row] = m[s];
          pp[2 * row + 1] = ls[s];
        }
      }
    }
  } else {
    for (int ch = 0; ch < chunks_per_wg; ++ch) {
      const int jchunk = (blockIdx.x * chunks_per_wg + ch) * SKC;
      if (jchunk >= N) break;
      for (int item = w; item < n_items; item += SNW) {
        const int pair = item % n_pairs, ks = item / n_pairs;
        load_a(pair);
        double mr[8], inv[8];
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          const int row = 32 * pair + 16 * (s >> 2) + 4 * (s & 3) + kq;
          mr[s] = st[2 * row];
          inv[s] = 1.0 / st[2 * row + 1];
        }
        const int jc = jchunk + ks * sub;
        for (int j0 = jc; j0 < jc + sub && j0 < N; j0 += 16) {
          bool valid;
          f64x4 acc[2];
          tile_logits(j0, valid, acc);
          const int j = j0 + c;
          double colsum = 0.0;
#pragma unroll
          for (int s = 0; s < 8; ++s) {
            const int row = 32 * pair + 16 * (s >> 2) + 4 * (s & 3) + kq;
            const bool vis = valid && row < R && j <= N - L + row % L;
            if (vis) colsum += exp(acc[s >> 2][s & 3] * scale - mr[s]) * inv[s];
          }
          colsum += __shfl_xor(colsum, 16);
          colsum += __shfl_xor(colsum, 32);
          if (kq == 0) cs[pair][j - jchunk] = colsum;
        }
      }
      __syncthreads();
      {
        const int j = jchunk + tid;
        if (tid < SKC && j < N) {
          double sum = 0.0;
          for (int p = 0; p < n_pairs; ++p) sum += cs[p][tid];
          scores[(size_t)unit * N + j] = sum / (double)R;
        }
      }
      __syncthreads();
    }
  }
}

int score_mfma64_parts(const Dims &dm, int chunks_per_wg) {
  const int n_chunks = (dm.N + SKC - 1) / SKC;
  const int n_wg = (n_chunks + chunks_per_wg - 1) / chunks_per_wg;
  const int n_pairs = dm.Rpad / 32;
  return n_wg * (n_pairs >= SNW ? 1 : SNW / n_pairs);
}

bool score_mfma64_supported(const Dims &dm) { return dm.Rpad % 32 == 0 && dm.Rpad / 32 <= MAXP; }

template <typename T, int D>
static int run_mfma64(const Dims &dm, const T *k, const double *qd, double *part, double *stats,
                      double *scores, int chunks_per_wg, hipStream_t s) {
  const int n_chunks = (dm.N + SKC - 1) / SKC;
  const dim3 grid((n_chunks + chunks_per_wg - 1) / chunks_per_wg, dm.units), block(64 * SNW);
  score_mfma64_kernel<T, D, 0><<<grid, block, 0, s>>>(k, qd, stats, part, scores, dm, chunks_per_wg);
  launch_merge_stats(part, stats, dm.units, dm.Rpad, score_mfma64_parts(dm, chunks_per_wg), s);
  score_mfma64_kernel<T, D, 1><<<grid, block, 0, s>>>(k, qd, stats, part, scores, dm, chunks_per_wg);
  return hip_ok(hipGetLastError());
}

int launch_scores_mfma64(const Dims &dm, int dtype, const void *k, const double *qd, double *part,
                         double *stats, double *scores, int chunks_per_wg, hipStream_t s) {
  if (dtype == TASKKV_F32) {
    auto kk = static_cast<const float *>(k);
    return dm.D == 64 ? run_mfma64<float, 64>(dm, kk, qd, part, stats, scores, chunks_per_wg, s)
                      : run_mfma64<float, 128>(dm, kk, qd, part, stats, scores, chunks_per_wg, s);
  }
  auto kk = static_cast<const uint16_t *>(k);
  return dm.D == 64 ? run_mfma64<uint16_t, 64>(dm, kk, qd, part, stats, scores, chunks_per_wg, s)
                    : run_mfma64<uint16_t, 128>(dm, kk, qd, part, stats, scores, chunks_per_wg, s);
}

}  // namespace taskkv
