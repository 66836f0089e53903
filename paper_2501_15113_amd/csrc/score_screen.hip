// Screening pass for the column mean C of Eq. 13 (paper Sec. 4.1), bf16 inputs.
//
// Selections must be decided on fp64 scores, but only a few hundred of the N
// columns of a unit can take part in a decision: the top-t tokens of Eq. 14 and
// the tokens whose score lies next to the middle-activation threshold of
// Sec. 4.2.  So, after the exact fp64 row statistics (m_i, l_i):
//   1. score_screen_kernel computes every column in fp32 on the bf16 matrix
//      cores (v_mfma_f32_16x16x32_bf16, exp2 on the vector ALUs);
//   2. band_kernel bounds the relative error eps of those values, finds the two
//      thresholds among them and lists the columns that could matter -- every
//      column at or above (1 - 3 eps) x the top-t threshold, and every middle
//      column within 3 eps of the middle threshold;
//      (on long contexts the same list comes from the sliced kernels of
//      select_multi.hip, which bracket the thresholds instead of finding them);
//   3. the fp64 scorer recomputes exactly the listed columns.
// Unlisted columns keep their fp32 value; each is provably on the same side of
// both thresholds as its exact value.
//
// Error bound.  bf16 products are exact in fp32, so a logit differs from its
// exact value by at most the accumulation error, gamma * |q_i|.|k_j| with
// gamma <= 4 d 2^-24 (factor 4 covers any summation order and truncating adds).
// Through exp this is a relative error of scale * gamma * max|q_i| * max|k_j| per
// term; converting m_i, 1/l_i to fp32, exp2 and the fp32 row sum add
// 2e-5 + R * 1.2e-7.  band_kernel evaluates the bound from the measured norms.
#include <math.h>

#include "band_common.h"
#include "lane_ops.h"
#include "select_common.h"

namespace taskkv {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;

constexpr int QKC = 256;   // keys per chunk
constexpr int MAXQ = 8;    // row quads (64 rows each) per unit: windows up to 512 rows

union Frag16 {
  uint4 u;
  bf16x8 b;
};

// Softmax weights of one 16-key tile summed over the RB 16-row blocks a wave
// holds (A operands a, row statistics m2 / inv in accumulator layout): the
// 16 RB x 16 logits with RB x d/32 matrix instructions, issued together ahead
// of the exponentials; returns the lane's share of its key's column sum (lane
// (c, kg): key j0 + c, rows 4 kg .. 4 kg + 3 of every block), to be added over kg.
template <int D, int RB>
__device__ __forceinline__ float tile_column_sums(const Frag16 (&a)[RB][D / 32], const Frag16 (&bk)[D / 32],
                                                  const float (&m2)[RB][4], const float (&inv)[RB][4],
                                                  float scale_log2, int j0, int c, int kg, int rq, const Dims &dm) {
  constexpr int KS = D / 32;
  const int N = dm.N, L = dm.L, R = dm.R;
  floatx4 acc[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) acc[rb] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int kk = 0; kk < KS; ++kk)
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
      acc[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[rb][kk].b, bk[kk].b, acc[rb], 0, 0, 0);
  float colsum = 0.f;
  if (j0 + 15 <= N - L) {
    // before the window: no causal mask inside the tile.  Rows past R have
    // inv = 0; keys past N are dropped when the sums are stored
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int v = 0; v < 4; ++v)
        colsum = fmaf(__builtin_amdgcn_exp2f(fmaf(acc[rb][v], scale_log2, -m2[rb][v])), inv[rb][v], colsum);
  } else {
    const int j = j0 + c;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int r2 = 64 * rq + 16 * rb + 4 * kg + v;
        const bool vis = j < N && r2 < R && j <= N - L + r2 % L;
        const float p = __builtin_amdgcn_exp2f(fmaf(acc[rb][v], scale_log2, -m2[rb][v])) * inv[rb][v];
        colsum += vis ? p : 0.f;
      }
  }
  return colsum;
}

// A operands and row statistics of the 16-row blocks [64 rq + 16 rb, + 16),
// rb < RB, of a unit's window: lane (c, kg) holds Q[row 64 rq + 16 rb + c][(d/4) kg + 8 kk .. +8]
// and, in accumulator layout, m (in units of ln 2) and 1 / l of rows 4 kg .. 4 kg + 3.
template <int D, int RB>
__device__ __forceinline__ void load_window_rows(const uint16_t *__restrict__ q_win, const double *__restrict__ st,
                                                 int unit, int rq, int c, int kg, const Dims &dm,
                                                 Frag16 (&a)[RB][D / 32], float (&m2)[RB][4], float (&inv)[RB][4]) {
  constexpr int KS = D / 32;
  const int b = unit / dm.Hkv, h = unit % dm.Hkv, L = dm.L, R = dm.R;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int row = 64 * rq + 16 * rb + c;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) a[rb][kk].u = make_uint4(0, 0, 0, 0);
    if (row < R) {
      const int g = row / L, i = row % L;
      const uint16_t *qp = q_win + (((size_t)b * dm.Hq + (size_t)h * dm.G + g) * L + i) * D + (D / 4) * kg;
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) a[rb][kk].u = *reinterpret_cast<const uint4 *>(qp + 8 * kk);
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int r2 = 64 * rq + 16 * rb + 4 * kg + v;   // row of accumulator register v
      const bool ok = r2 < R;
      m2[rb][v] = ok ? (float)(st[2 * r2] * 1.4426950408889634) : 0.f;
      inv[rb][v] = ok ? (float)(1.0 / st[2 * r2 + 1]) : 0.f;
    }
  }
}

// One block = 4 waves.  A wave owns a quad of four 16-row blocks of the window
// (A operands in registers) and a slice of the chunk's keys; for every 16-key
// tile it forms the 64 x 16 logits with 4 x d/32 MFMAs, turns them into softmax
// weights with the exact row statistics and adds the 64 rows per key.  Row
// quads are added per key in index order through LDS.
template <int D>
__global__ __launch_bounds__(256) void score_screen_kernel(const uint16_t *__restrict__ q_win,
                                                           const uint16_t *__restrict__ k,
                                                           const double *__restrict__ stats,
                                                           double *__restrict__ scores, Dims dm,
                                                           int chunks_per_wg) {
  constexpr int KS = D / 32;
  const int unit = blockIdx.y, tid = threadIdx.x, w = tid >> 6, l = tid & 63, c = l & 15, kg = l >> 4;
  const int N = dm.N, L = dm.L, R = dm.R;
  const int n_rq = (dm.Rpad + 63) / 64;
  const int ksplit = n_rq >= 4 ? 1 : 4 / n_rq;
  const int n_items = n_rq * ksplit;
  const int sub = QKC / ksplit;
  const int b = unit / dm.Hkv, h = unit % dm.Hkv;
  const uint16_t *kb = k + (size_t)unit * N * D;
  const double *st = stats + (size_t)unit * dm.Rpad * 2;
  const float scale_log2 = (float)(dm.scale * 1.4426950408889634);

  __shared__ float cs[MAXQ][QKC];
  // the chunk's keys, read from memory once per block and shared by the four
  // waves (each would otherwise fetch every key itself); rows padded by 16 bytes
  // so that the sixteen keys of a tile fall into different banks
  constexpr int KROW = D * 2 + 16;
  __shared__ __attribute__((aligned(16))) unsigned char s_keys[QKC * KROW];

  // A operands: lane (c, kg) holds Q[row 64 rq + 16 rb + c][(d/4) kg + 8 kk .. +8].
  // They and the rows' statistics are loaded when the wave's row quad changes:
  // once per block when there are at most four quad-slice items.
  Frag16 a[4][KS];
  float m2[4][4], inv[4][4];
  int cur_rq = -1;
  auto load_rows = [&](int rq) {
    if (rq == cur_rq) return;
    cur_rq = rq;
    load_window_rows<D, 4>(q_win, st, unit, rq, c, kg, dm, a, m2, inv);
  };

  for (int ch = 0; ch < chunks_per_wg; ++ch) {
    const int jchunk = (blockIdx.x * chunks_per_wg + ch) * QKC;
    if (jchunk >= N) break;
    {
      // in rounds of eight 16-byte pieces per thread: few registers, so that the
      // window rows can stay in registers across chunks
      constexpr int PARTS = D / 8;   // 16-byte pieces per key
      constexpr int ROUND = 8, N_ROUNDS = QKC * PARTS / 256 / ROUND;
#pragma unroll 1
      for (int rd = 0; rd < N_ROUNDS; ++rd) {
        uint4 piece[ROUND];
#pragma unroll
        for (int i = 0; i < ROUND; ++i) {
          const int idx = (rd * ROUND + i) * 256 + tid, key = idx / PARTS, part = idx % PARTS;
          const int j = jchunk + key;
          piece[i] = j < N ? *reinterpret_cast<const uint4 *>(kb + (size_t)j * D + part * 8) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < ROUND; ++i) {
          const int idx = (rd * ROUND + i) * 256 + tid, key = idx / PARTS, part = idx % PARTS;
          *reinterpret_cast<uint4 *>(s_keys + key * KROW + part * 16) = piece[i];
        }
      }
    }
    __syncthreads();
    for (int item = w; item < n_items; item += 4) {
      const int rq = item % n_rq, ks = item / n_rq;
      load_rows(rq);
      const int jc = jchunk + ks * sub;
      // K tiles of the next step are read from LDS before this step's work, and
      // the sixteen matrix instructions of a tile (four accumulators, one per row
      // block) are issued together, ahead of the exponentials
      auto read_tile = [&](int j0, Frag16 (&bk)[KS]) {
        const int key = min(j0 + c - jchunk, QKC - 1);
#pragma unroll
        for (int kk = 0; kk < KS; ++kk)
          bk[kk].u = *reinterpret_cast<const uint4 *>(s_keys + key * KROW + ((D / 4) * kg + 8 * kk) * 2);
      };
      const int jend = min(jc + sub, N);
      Frag16 bk[KS], bk_next[KS];
      if (jc < jend) read_tile(jc, bk);
      for (int j0 = jc; j0 < jend; j0 += 16) {
        const int j = j0 + c;
        if (j0 + 16 < jend) read_tile(j0 + 16, bk_next);
        float colsum = tile_column_sums<D, 4>(a, bk, m2, inv, scale_log2, j0, c, kg, rq, dm);
        colsum = sum_lanes_16_32(colsum);
        if (kg == 0) cs[rq][j - jchunk] = colsum;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) bk[kk] = bk_next[kk];
      }
    }
    __syncthreads();
    {
      const int j = jchunk + tid;
      if (j < N) {
        float sum = 0.f;
        for (int p = 0; p < n_rq; ++p) sum += cs[p][tid];
        scores[(size_t)unit * N + j] = (double)(sum / (float)dm.Rtot);
      }
    }
    __syncthreads();
  }
}

// Windows of at most 64 rows are one row quad: a key's column sum is complete
// inside one wave, and a chunk of keys staged for four waves would be used by
// one.  Every wave streams a run of keys of its own straight from memory into
// operand layout (lane (c, kg) holds key c's channels (d/4) kg .. + d/4: four
// lanes read a key's row between them), two tiles ahead of the one it works on,
// and writes its sums itself: no LDS, no barriers.  RB: 16-row blocks in use.
template <int D, int RB>
__global__ __launch_bounds__(256) void score_screen_direct_kernel(const uint16_t *__restrict__ q_win,
                                                                  const uint16_t *__restrict__ k,
                                                                  const double *__restrict__ stats,
                                                                  double *__restrict__ scores, Dims dm,
                                                                  int keys_per_wave) {
  constexpr int KS = D / 32;
  const int unit = blockIdx.y, tid = threadIdx.x, w = tid >> 6, l = tid & 63, c = l & 15, kg = l >> 4;
  const int N = dm.N;
  const uint16_t *kb = k + (size_t)unit * N * D;
  const float scale_log2 = (float)(dm.scale * 1.4426950408889634);
  const float inv_rows = 1.f / (float)dm.Rtot;
  Frag16 a[RB][KS];
  float m2[RB][4], inv[RB][4];
  load_window_rows<D, RB>(q_win, stats + (size_t)unit * dm.Rpad * 2, unit, 0, c, kg, dm, a, m2, inv);
  const int jbeg = (blockIdx.x * 4 + w) * keys_per_wave, jend = min(jbeg + keys_per_wave, N);
  auto read_tile = [&](int j0, Frag16 (&bk)[KS]) {
    const int j = min(j0 + c, N - 1);
#pragma unroll
    for (int kk = 0; kk < KS; ++kk)
      bk[kk].u = *reinterpret_cast<const uint4 *>(kb + (size_t)j * D + (D / 4) * kg + 8 * kk);
  };
  Frag16 bk[3][KS];
  if (jbeg < jend) read_tile(jbeg, bk[0]);
  if (jbeg + 16 < jend) read_tile(jbeg + 16, bk[1]);
  for (int j0 = jbeg; j0 < jend; j0 += 16) {
    if (j0 + 32 < jend) read_tile(j0 + 32, bk[2]);
    float colsum = tile_column_sums<D, RB>(a, bk[0], m2, inv, scale_log2, j0, c, kg, 0, dm);
    colsum = sum_lanes_16_32(colsum);
    const int j = j0 + c;
    if (kg == 0 && j < N) scores[(size_t)unit * N + j] = (double)(colsum * inv_rows);
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      bk[0][kk] = bk[1][kk];
      bk[1][kk] = bk[2][kk];
    }
  }
}

// One block per unit: error bound, thresholds, list of the columns to recompute.
__global__ __launch_bounds__(1024) void band_kernel(const double *__restrict__ scores,
                                                    const double *__restrict__ qd,
                                                    const unsigned long long *__restrict__ knorm,
                                                    int32_t *__restrict__ band_idx,
                                                    int32_t *__restrict__ band_cnt, Dims dm) {
  const int unit = blockIdx.x;
  __shared__ RadixScratch rs;
  __shared__ int s_cnt[32];
  __shared__ double s_q[16];
  band_of_unit(scores + (size_t)unit * dm.N, qd, __longlong_as_double((long long)knorm[unit]), unit, dm,
               band_idx + (size_t)unit * dm.N, band_cnt + unit, rs, s_cnt, s_q);
}

__global__ void zero_u64_kernel(unsigned long long *p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0ull;
}

// Per-unit maximum of ||k_j||^2 (bf16 rows), slightly over-estimated: fp32 sums
// scaled by 1.001.  Stored as the bit pattern of a non-negative double, so the
// integer atomic max is the numeric max and the result is order independent.
template <int D>
__global__ __launch_bounds__(256) void key_norm_kernel(const uint16_t *__restrict__ k,
                                                       unsigned long long *__restrict__ knorm, int N) {
  const int unit = blockIdx.y;
  const uint16_t *kb = k + (size_t)unit * N * D;
  float best = 0.f;
  for (int j = blockIdx.x * 256 + threadIdx.x; j < N; j += gridDim.x * 256) {
    const uint4 *row = reinterpret_cast<const uint4 *>(kb + (size_t)j * D);
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < D / 8; ++i) {
      const uint4 x = row[i];
      const uint32_t wd[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float lo = __uint_as_float(wd[e] << 16), hi = __uint_as_float(wd[e] & 0xffff0000u);
        ss = fmaf(lo, lo, ss);
        ss = fmaf(hi, hi, ss);
      }
    }
    best = fmaxf(best, ss);
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) best = fmaxf(best, __shfl_xor(best, off));
  if ((threadIdx.x & 63) == 0 && best > 0.f)
    atomicMax(knorm + unit, (unsigned long long)__double_as_longlong((double)best * 1.001));
}

bool screen_supported(const Dims &dm, int dtype) {
  return dtype == TASKKV_BF16 && dm.Rtot <= 64 * MAXQ;
}

int launch_zero_u64(unsigned long long *p, int n, hipStream_t s) {
  zero_u64_kernel<<<dim3((n + 255) / 256), dim3(256), 0, s>>>(p, n);
  return hip_ok(hipGetLastError());
}

int launch_key_norms(const Dims &dm, const void *k, unsigned long long *knorm, hipStream_t s) {
  zero_u64_kernel<<<dim3((dm.units + 255) / 256), dim3(256), 0, s>>>(knorm, dm.units);
  int gx = (dm.N + 255) / 256;
  if (gx > 64) gx = 64;
  const dim3 grid(gx, dm.units), block(256);
  auto kk = static_cast<const uint16_t *>(k);
  if (dm.D == 64) key_norm_kernel<64><<<grid, block, 0, s>>>(kk, knorm, dm.N);
  else key_norm_kernel<128><<<grid, block, 0, s>>>(kk, knorm, dm.N);
  return hip_ok(hipGetLastError());
}

int launch_screen(const Dims &dm, const void *q_win, const void *k, const double *stats, double *scores,
                  int chunks_per_wg, int n_cu, hipStream_t s) {
  auto qq = static_cast<const uint16_t *>(q_win), kk = static_cast<const uint16_t *>(k);
  if (dm.Rpad <= 64) {
    // one row quad: runs of keys per wave, some sixteen waves per compute unit in all
    const int tiles = (dm.N + 15) / 16;
    int per_wave = (int)(((int64_t)tiles * dm.units + n_cu * 16 - 1) / (n_cu * 16));
    per_wave = per_wave < 8 ? 8 : per_wave;
    const int keys_per_wave = per_wave * 16;
    const dim3 grid((dm.N + 4 * keys_per_wave - 1) / (4 * keys_per_wave), dm.units), block(256);
    if (dm.D == 64) {
      if (dm.Rpad <= 32) score_screen_direct_kernel<64, 2><<<grid, block, 0, s>>>(qq, kk, stats, scores, dm, keys_per_wave);
      else score_screen_direct_kernel<64, 4><<<grid, block, 0, s>>>(qq, kk, stats, scores, dm, keys_per_wave);
    } else {
      if (dm.Rpad <= 32) score_screen_direct_kernel<128, 2><<<grid, block, 0, s>>>(qq, kk, stats, scores, dm, keys_per_wave);
      else score_screen_direct_kernel<128, 4><<<grid, block, 0, s>>>(qq, kk, stats, scores, dm, keys_per_wave);
    }
    return hip_ok(hipGetLastError());
  }
  const int n_chunks = (dm.N + QKC - 1) / QKC;
  while ((int64_t)((n_chunks + 2 * chunks_per_wg - 1) / (2 * chunks_per_wg)) * dm.units >= 2 * n_cu && chunks_per_wg < 16)
    chunks_per_wg *= 2;
  const dim3 grid((n_chunks + chunks_per_wg - 1) / chunks_per_wg, dm.units), block(256);
  if (dm.D == 64) score_screen_kernel<64><<<grid, block, 0, s>>>(qq, kk, stats, scores, dm, chunks_per_wg);
  else score_screen_kernel<128><<<grid, block, 0, s>>>(qq, kk, stats, scores, dm, chunks_per_wg);
  return hip_ok(hipGetLastError());
}

int launch_band(const Dims &dm, const double *scores, const double *qd, const unsigned long long *knorm,
                int32_t *band_idx, int32_t *band_cnt, hipStream_t s) {
  band_kernel<<<dim3(dm.units), dim3(1024), 0, s>>>(scores, qd, knorm, band_idx, band_cnt, dm);
  return hip_ok(hipGetLastError());
}

}  // namespace taskkv
