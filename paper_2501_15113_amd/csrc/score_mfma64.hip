// Window scores in fp64 on the matrix cores (paper Sec. 4.1, Eq. 12-13).
//
// Two passes over K.  Pass 0 finds, for every window row, the row maximum and
// the softmax denominator; pass 1 recomputes the logits and accumulates the
// column mean C.  Re-reading K (2*d bytes per key) is cheaper than spilling the
// G*L logits per key.  Every product, sum and exponential is fp64; the
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
//
// Windows of more than 512 rows per KV head (G*L; the whole prompt when L = N,
// which turns Eq. 12-13 into the full attention matrix of Eq. 1-2) are handled
// in groups of 512 rows: each group runs both passes over the keys its rows can
// see and adds its share to C.
#include <math.h>

#include "band_common.h"
#include "taskkv_internal.h"

namespace taskkv {

typedef double f64x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float elem_to_float(float x) { return x; }
__device__ __forceinline__ float elem_to_float(uint16_t x) { return __uint_as_float(uint32_t(x) << 16); }

// Rows [row0, row0 + R) of the flattened window (row = g*L + i) of every unit
// -> qd [unit][Rpad][D] fp64, zero padded.
// Also clears the words of `zeros` (counters and histograms of the kernels
// that follow on the stream).
template <typename T>
__global__ void q_to_f64_kernel(const T *__restrict__ q, double *__restrict__ qd, Dims dm, ZeroList zeros) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (int z = 0; z < zeros.count; ++z)
    for (size_t i = idx; i < zeros.n[z]; i += (size_t)gridDim.x * blockDim.x) zeros.p[z][i] = 0u;
  size_t total = (size_t)dm.units * dm.Rpad * dm.D;
  if (idx >= total) return;
  int c = idx % dm.D;
  size_t rest = idx / dm.D;
  int r = rest % dm.Rpad;
  int unit = rest / dm.Rpad;
  double val = 0.0;
  if (r < dm.R) {
    const int rg = dm.row0 + r;
    int b = unit / dm.Hkv, h = unit % dm.Hkv, g = rg / dm.L, i = rg % dm.L;
    size_t src = (((size_t)b * dm.Hq + h * dm.G + g) * dm.L + i) * dm.D + c;
    val = (double)elem_to_float(q[src]);
  }
  qd[idx] = val;
}

// Fixed-order merge of the per-part row statistics.  A wave shares a row: lane
// i merges the parts i, i + 64, ... (records requested four at a time: the loop
// is bound by memory latency), then the 64 results are merged in a fixed tree.
// Launched with 1024 threads: 16 rows per block.
__global__ __launch_bounds__(1024) void merge_stats_kernel(const double *__restrict__ part,
                                                           double *__restrict__ stats, int Rpad, int n_parts) {
  const int unit = blockIdx.x, sub = threadIdx.x & 63;
  const int r = blockIdx.y * 16 + (threadIdx.x >> 6);
  if (r >= Rpad) return;   // whole waves
  double m = -INFINITY, l = 0.0;
  for (int c0 = sub; c0 < n_parts; c0 += 256) {
    double mc[4], lc[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const bool ok = c0 + 64 * u < n_parts;
      const double *pp = part + (((size_t)unit * n_parts + (ok ? c0 + 64 * u : 0)) * Rpad + r) * 2;
      mc[u] = ok ? pp[0] : -INFINITY;
      lc[u] = ok ? pp[1] : 0.0;
    }
    double mn = m;
#pragma unroll
    for (int u = 0; u < 4; ++u) mn = fmax(mn, mc[u]);
    if (mn > -INFINITY) {
      double sum = l * exp(m - mn);
#pragma unroll
      for (int u = 0; u < 4; ++u) sum += lc[u] * exp(mc[u] - mn);
      l = sum;
      m = mn;
    }
  }
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const double mo = __shfl_xor(m, off), lo = __shfl_xor(l, off);
    const double mn = fmax(m, mo);
    // both partners form the same sum: the lower lane's term first
    const bool low = (sub & off) == 0;
    const double a = low ? l : lo, am = low ? m : mo, b = low ? lo : l, bm = low ? mo : m;
    if (mn > -INFINITY) l = a * exp(am - mn) + b * exp(bm - mn);
    m = mn;
  }
  if (sub == 0) {
    stats[((size_t)unit * Rpad + r) * 2] = m;
    stats[((size_t)unit * Rpad + r) * 2 + 1] = l;
  }
}

__global__ void zero_f64_kernel(double *p, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0.0;
}

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
// GATHER (MODE 1 only): score just the keys listed in band_idx[unit][0 .. band_cnt[unit]).
template <typename T, int D, int MODE, bool GATHER>
__global__ __launch_bounds__(64 * SNW) void score_mfma64_kernel(const T *__restrict__ k,
                                                           const double *__restrict__ qd,
                                                           const double *__restrict__ stats,
                                                           double *__restrict__ part,
                                                           double *__restrict__ scores, Dims dm,
                                                           int chunks_per_wg,
                                                           const int32_t *__restrict__ band_idx,
                                                           const int32_t *__restrict__ band_cnt) {
  constexpr int NKK = D / 4;
  constexpr int NRAW = NKK / RawCount<T>::per16B;
  const int unit = blockIdx.y, tid = threadIdx.x, w = tid >> 6, l = tid & 63, c = l & 15, kq = l >> 4;
  const int N = dm.N, NK = GATHER ? band_cnt[unit] : dm.n_keys, L = dm.L, R = dm.R, Rpad = dm.Rpad,
            row0 = dm.row0;
  const int32_t *gidx = GATHER ? band_idx + (size_t)unit * N : nullptr;
  const int n_pairs = Rpad / 32;
  const int ksplit = n_pairs >= SNW ? 1 : SNW / n_pairs;
  const int n_items = n_pairs * ksplit;
  // keys per chunk and per key slice; the gathered pass uses the smallest chunk
  // (one 16-key tile per wave) so that a few hundred listed keys spread over
  // many blocks
  const int ckeys = GATHER ? 16 * ksplit : SKC;
  const int sub = ckeys / ksplit;
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
  auto tile_logits = [&](int j0, bool &valid, int &j, f64x4 (&acc)[2]) {
    const int pos = j0 + c;
    valid = pos < NK;
    j = GATHER ? (valid ? gidx[pos] : 0) : pos;
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
        if (jc >= NK) break;
        for (int j0 = jc; j0 < jc + sub && j0 < NK; j0 += 16) {
          bool valid;
          int j;
          f64x4 acc[2];
          tile_logits(j0, valid, j, acc);
#pragma unroll
          for (int s = 0; s < 8; ++s) {
            const int row = 32 * pair + 16 * (s >> 2) + 4 * (s & 3) + kq;
            const bool vis = valid && row < R && j <= N - L + (row0 + row) % L;
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
    for (int it = 0; GATHER || it < chunks_per_wg; ++it) {
      // plain pass: chunks_per_wg consecutive chunks; gathered pass: grid-stride
      const int chunk = GATHER ? blockIdx.x + it * gridDim.x : blockIdx.x * chunks_per_wg + it;
      const int jchunk = chunk * ckeys;
      if (jchunk >= NK) break;
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
        for (int j0 = jc; j0 < jc + sub && j0 < NK; j0 += 16) {
          bool valid;
          int j;
          f64x4 acc[2];
          tile_logits(j0, valid, j, acc);
          double colsum = 0.0;
#pragma unroll
          for (int s = 0; s < 8; ++s) {
            const int row = 32 * pair + 16 * (s >> 2) + 4 * (s & 3) + kq;
            const bool vis = valid && row < R && j <= N - L + (row0 + row) % L;
            if (vis) colsum += exp(acc[s >> 2][s & 3] * scale - mr[s]) * inv[s];
          }
          colsum += __shfl_xor(colsum, 16);
          colsum += __shfl_xor(colsum, 32);
          if (kq == 0) cs[pair][j0 + c - jchunk] = colsum;
        }
      }
      __syncthreads();
      {
        const int pos = jchunk + tid;
        if (tid < ckeys && pos < NK) {
          double sum = 0.0;
          for (int p = 0; p < n_pairs; ++p) sum += cs[p][tid];
          double *dst = scores + (size_t)unit * N + (GATHER ? gidx[pos] : pos);
          *dst = dm.accumulate ? *dst + sum / (double)dm.Rtot : sum / (double)dm.Rtot;
        }
      }
      __syncthreads();
    }
  }
}

constexpr int ROW_GROUP = 32 * MAXP;  // window rows scored per launch pair

static int chunks_per_wg_for(const Dims &dm) {
  const int64_t n_chunks = (dm.N + SKC - 1) / SKC;
  int64_t t = (n_chunks * dm.units + 4095) / 4096;
  if (t < 1) t = 1;
  if (t > 16) t = 16;
  return (int)t;
}

// Row-statistics partial records per unit (for the workspace size).
int score_parts(const Dims &dm) {
  const int cpw = chunks_per_wg_for(dm);
  const int n_chunks = (dm.N + SKC - 1) / SKC;
  const int n_wg = (n_chunks + cpw - 1) / cpw;
  const int rpad = dm.Rtot < ROW_GROUP ? (dm.Rtot + 31) / 32 * 32 : ROW_GROUP;
  const int n_pairs = rpad / 32;
  return n_wg * (n_pairs >= SNW ? 1 : SNW / n_pairs);
}

int score_rows_padded(const Dims &dm) { return dm.Rtot < ROW_GROUP ? (dm.Rtot + 31) / 32 * 32 : ROW_GROUP; }

template <typename T, int D>
static int run_scores(const Dims &dm_all, int dtype, const T *q_win, const T *k, double *qd, double *part,
                      double *stats, double *scores, const ScreenBufs *scr, const I8Bufs *i8b, hipStream_t s) {
  const int cpw = chunks_per_wg_for(dm_all);
  const int n_groups = (dm_all.Rtot + ROW_GROUP - 1) / ROW_GROUP;
  const bool screen = scores_screened(dm_all, dtype, scr);
  if (n_groups > 1) {
    const size_t n = (size_t)dm_all.units * dm_all.N;
    zero_f64_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(scores, n);
  }
  // the int8 statistics pass reads every key anyway and leaves the key norms
  // the screening pass needs; otherwise they get a pass of their own
  const bool i8 = i8b != nullptr && i8_stats_supported(dm_all, dtype);
  // counters and histograms of the kernels below are cleared by the first
  // kernel of the sequence instead of by launches of their own
  ZeroList zeros;
  if (i8) zeros.add(i8b->qcnt, (size_t)dm_all.units);
  if (screen && i8) zeros.add(scr->knorm, (size_t)2 * dm_all.units);
  const bool sliced_band = screen && band_is_sliced(dm_all, scr);
  if (sliced_band) msel_zero_words(dm_all, *scr->msel, zeros);
  if (screen && !i8) {
    int rc = launch_key_norms(dm_all, k, scr->knorm, s);
    if (rc) return rc;
  }
  for (int grp = 0; grp < n_groups; ++grp) {
    Dims dm = dm_all;
    dm.row0 = grp * ROW_GROUP;
    dm.R = dm_all.Rtot - dm.row0 < ROW_GROUP ? dm_all.Rtot - dm.row0 : ROW_GROUP;
    dm.Rpad = (dm.R + 31) / 32 * 32;
    dm.accumulate = n_groups > 1 ? 1 : 0;
    // keys the rows of this group can see: all of them unless the group lies
    // inside one query head's window, where the last row bounds it
    const int last = dm.row0 + dm.R - 1;
    dm.n_keys = dm.N;
    if (dm.row0 / dm.L == last / dm.L) {
      const int64_t vis = (int64_t)dm.N - dm.L + last % dm.L + 1;
      dm.n_keys = (int)(vis < dm.N ? vis : dm.N);
    }
    const size_t total = (size_t)dm.units * dm.Rpad * dm.D;
    q_to_f64_kernel<T><<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s>>>(q_win, qd, dm,
                                                                                    grp == 0 ? zeros : ZeroList());
    const int n_chunks = (dm.n_keys + SKC - 1) / SKC;
    const int n_wg = (n_chunks + cpw - 1) / cpw;
    const int n_pairs = dm.Rpad / 32;
    const int n_parts = n_wg * (n_pairs >= SNW ? 1 : SNW / n_pairs);
    const dim3 grid(n_wg, dm.units), block(64 * SNW);
    if (i8) {
      // bf16 inputs: exact integer dot products on the int8 matrix cores
      int n_recs = n_wg;
      int rc = launch_i8_stats(dm, q_win, k, qd, *i8b, part, screen ? scr->knorm : nullptr, n_wg, cpw * SKC, grp == 0,
                               &n_recs, s);
      if (rc) return rc;
      merge_stats_kernel<<<dim3(dm.units, (dm.Rpad + 15) / 16), dim3(1024), 0, s>>>(part, stats, dm.Rpad, n_recs);
    } else {
      score_mfma64_kernel<T, D, 0, false><<<grid, block, 0, s>>>(k, qd, stats, part, scores, dm, cpw, nullptr,
                                                                nullptr);
      merge_stats_kernel<<<dim3(dm.units, (dm.Rpad + 15) / 16), dim3(1024), 0, s>>>(part, stats, dm.Rpad, n_parts);
    }
    if (!screen) {
      if (i8) {
        // bf16 inputs: all columns from the integer contraction, a tile of 32
        // columns per wave (8 units x 128 rows x 8192 keys: 61 us as the fp64
        // column pass)
        const int n_cu = i8b->prof ? i8b->prof->n_cu : 256;
        int per_unit = 2 * n_cu / dm.units;
        per_unit = per_unit < 1 ? 1 : (per_unit > 256 ? 256 : per_unit);
        const int rc = launch_i8_columns(dm, k, qd, *i8b, stats, nullptr, nullptr, scores, per_unit, s);
        if (rc) return rc;
        continue;
      }
      score_mfma64_kernel<T, D, 1, false><<<grid, block, 0, s>>>(k, qd, stats, part, scores, dm, cpw, nullptr,
                                                                nullptr);
      continue;
    }
    // fp32 screening of every column, then fp64 for the columns that can take
    // part in a decision (any number of them: the grid covers all N)
    int rc = launch_screen(dm, q_win, k, stats, scores, cpw, scr->n_cu, s);
    if (rc) return rc;
    // a middle pick that pools ranks by the pooled scores: the band follows it
    const double *pooled = nullptr;
    if (dm.pool > 1 && band_has_middle(dm)) {
      rc = launch_pool(dm, scores, scr->pooled, s);
      if (rc) return rc;
      pooled = scr->pooled;
    }
    if (sliced_band)
      rc = launch_band_sliced(dm, scr->n_cu, *scr->msel, scores, pooled, qd, scr->knorm, scr->band_idx, scr->band_cnt,
                              scr->above_band, scr->list_ok, true, s);
    else
      rc = launch_band(dm, scores, qd, scr->knorm, scr->band_idx, scr->band_cnt, s);
    if (rc) return rc;
    // The listed columns of a unit make about twenty 16-key tasks of some ten
    // microseconds each (a chain of dependent loads, 64 fp64 matrix instructions,
    // eight exponentials); a block that takes several of them in turn loads its
    // window rows once, and one block per compute unit in all keeps the tasks
    // from queueing: measured 134 -> 60 us at 64 units, 69 -> 35 us at 32.
    int band_grid = scr->n_cu / dm.units;
    band_grid = band_grid < 1 ? 1 : (band_grid > 64 ? 64 : band_grid);
    if (i8) {
      // bf16 inputs: the listed columns from the integer contraction too (the
      // fp64 matrix instruction makes 6 us of a 16-key task's 11)
      rc = launch_i8_columns(dm, k, qd, *i8b, stats, scr->band_idx, scr->band_cnt, scores, 2 * band_grid, s);
      if (rc) return rc;
      continue;
    }
    score_mfma64_kernel<T, D, 1, true><<<dim3(band_grid, dm.units), block, 0, s>>>(k, qd, stats, part, scores, dm,
                                                                           cpw, scr->band_idx, scr->band_cnt);
  }
  return hip_ok(hipGetLastError());
}

// Whether the column means of this layer go through the fp32 screening pass:
// it pays once the fp64 column pass is large compared with the extra launches
// (mode 1 = decide here, 2 = whenever possible).
bool band_is_sliced(const Dims &dm, const ScreenBufs *scr) {
  return scr != nullptr && scr->msel != nullptr && msel_pays(dm, scr->n_cu, 0, dm.N, dm.T);
}

bool scores_screened(const Dims &dm, int dtype, const ScreenBufs *scr) {
  const int n_groups = (dm.Rtot + ROW_GROUP - 1) / ROW_GROUP;
  // Measured against the integer form of the full column pass, separator and
  // compressor together, W = units x rows x keys: below 12288 keys the band is
  // one block per unit and screening wins only on large layers (32 units x 128
  // rows x 8192 keys, W = 3.4e7: 22 us faster; 16 x 128 x 8192, 1.7e7: 12 us
  // slower); from 12288 keys on it wins from W = 1.26e7 for windows of 32 rows
  // (16 us) and from 1.7e7 for 128 rows (5 us; 11 us slower at 1.26e7).
  const double W = (double)dm.units * dm.Rtot * dm.N;
  const bool big = W >= 3e7 || (dm.N >= MSEL_MIN_RANGE && W >= (dm.Rtot <= 32 ? 1.2e7 : 1.6e7));
  // with pooling only the sliced band kernels list the neighbours a pooled score needs
  const bool pool_ok = dm.pool == 1 || (band_is_sliced(dm, scr) && scr->pooled != nullptr);
  return scr != nullptr && scr->mode != 0 && n_groups == 1 && screen_supported(dm, dtype) && pool_ok &&
         (scr->mode == 2 || big);
}

int launch_scores(const Dims &dm, int dtype, const void *q_win, const void *k, double *qd, double *part,
                  double *stats, double *scores, const ScreenBufs *scr, const I8Bufs *i8, hipStream_t s) {
  if (dtype == TASKKV_F32) {
    auto qq = static_cast<const float *>(q_win), kk = static_cast<const float *>(k);
    return dm.D == 64 ? run_scores<float, 64>(dm, dtype, qq, kk, qd, part, stats, scores, scr, i8, s)
                      : run_scores<float, 128>(dm, dtype, qq, kk, qd, part, stats, scores, scr, i8, s);
  }
  auto qq = static_cast<const uint16_t *>(q_win), kk = static_cast<const uint16_t *>(k);
  return dm.D == 64 ? run_scores<uint16_t, 64>(dm, dtype, qq, kk, qd, part, stats, scores, scr, i8, s)
                    : run_scores<uint16_t, 128>(dm, dtype, qq, kk, qd, part, stats, scores, scr, i8, s);
}

}  // namespace taskkv
