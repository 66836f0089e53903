// int8 scoring kernels in which every wave converts its own tiles of 32 keys
// (paper Sec. 4.1, Eq. 12-13; the arithmetic is described in score_i8_common.h):
// the row statistics of windows of at most 32 rows, and the exact scores of the
// columns a screening separator lists.
#include "score_i8_common.h"

namespace taskkv {

// Lanes of one wave hand data to each other through LDS without a block
// barrier: the wave's LDS operations execute in program order, so all it takes
// is that the compiler keeps them in that order, for memory (the fence) and in
// its instruction schedule (the barrier).
__device__ __forceinline__ void wave_lds_handover() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// ---- a wave that converts its own tile of 32 keys (the two kernels below)

// The pieces of a key's row that lane (key, half) holds of the operand: the two
// 16-channel segments [32 ks + 16 half, + 16) of every 32-channel block; zeros
// without a row.
template <int D>
__device__ __forceinline__ void fetch_key_pieces(const uint16_t *__restrict__ key_row, int half,
                                                 uint32_t (&raw)[D / 32][8]) {
  constexpr int KS = D / 32;
  if (key_row != nullptr) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const uint4 lo = *reinterpret_cast<const uint4 *>(key_row + ks * 32 + half * 16);
      const uint4 hi = *reinterpret_cast<const uint4 *>(key_row + ks * 32 + half * 16 + 8);
      raw[ks][0] = lo.x; raw[ks][1] = lo.y; raw[ks][2] = lo.z; raw[ks][3] = lo.w;
      raw[ks][4] = hi.x; raw[ks][5] = hi.y; raw[ks][6] = hi.z; raw[ks][7] = hi.w;
    }
  } else {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int x = 0; x < 8; ++x) raw[ks][x] = 0u;
  }
}

// The tile's digits in operand layout into the wave's LDS (dig), the keys'
// factors (ek[key] with f_k = 2^ek, the row factor's grid folded in) and the
// remainders of the elements that do not fit on the wave's short list, filled
// lane by lane (.row = key of the tile); returns their number: above I8_KCAP
// the tile takes the plain route.  key_row: the lane's key in memory (its
// elements are read again for the list: indexing the registers by a loop
// counter would move them to scratch memory).  norm_best (or null): running
// maximum of the keys' squared norms.
template <int D>
__device__ __forceinline__ int convert_own_tile(const uint32_t (&raw)[D / 32][8], const uint16_t *__restrict__ key_row,
                                                int l, v4i (&dig_out)[D / 32][4][64], int (&ek)[32],
                                                QTiny (&list)[I8_KCAP], bool &k_low_zero, float *norm_best) {
  constexpr int KS = D / 32;
  const int c32 = l & 31, half = l >> 5;
  int E = 1;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) E = max(E, row_exponent_of(raw[ks]));
  E = max(E, __shfl_xor(E, 32));
  if (norm_best != nullptr) {
    float ss = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int x = 0; x < 8; ++x) {
        const float lo = __uint_as_float(raw[ks][x] << 16), hi = __uint_as_float(raw[ks][x] & 0xffff0000u);
        ss = fmaf(lo, lo, ss);
        ss = fmaf(hi, hi, ss);
      }
    ss += __shfl_xor(ss, 32);
    *norm_best = fmaxf(*norm_best, ss);
  }
  bool ok = true, k_low = false;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    v4i dig[4];
    ok = digits_of(raw[ks], E, dig) && ok;
    k_low = k_low || (dig[0][0] | dig[0][1] | dig[0][2] | dig[0][3]) != 0;
#pragma unroll
    for (int t = 0; t < 4; ++t) dig_out[ks][t][l] = dig[t];
  }
  k_low_zero = __ballot(k_low) == 0ull;
  int cnt = 0;
  unsigned long long bad = __ballot(!ok);
  while (bad) {
    const int src = __ffsll((long long)bad) - 1;
    bad &= bad - 1;
    if (l == src) {
#pragma unroll 1
      for (int i = 0; i < 16 * KS; ++i) {
        const int c = (i >> 4) * 32 + half * 16 + (i & 15);
        double rem;
        if (!remainder_of(key_row[c], E, rem)) continue;
        if (cnt < I8_KCAP) {
          QTiny ent;
          ent.row = c32;
          ent.c = c;
          ent.r = rem;
          list[cnt] = ent;
        }
        ++cnt;
      }
    }
    cnt = __shfl(cnt, src);
  }
  if (half == 0) ek[c32] = E - (2 * I8_GRID - 126);   // with the row factor: 2^(Eq - I8_GRID) 2^(Ek - I8_GRID)
  return cnt;
}

// Class sums -> logits in table units: the row's factor and the factors of the
// lane's sixteen keys.
__device__ __forceinline__ void scale_logits(double (&t16)[16], double gqr, const int (&ek)[32], int half) {
#pragma unroll
  for (int v4 = 0; v4 < 4; ++v4) {
    const v4i e4 = *reinterpret_cast<const v4i *>(&ek[8 * v4 + 4 * half]);
#pragma unroll
    for (int x = 0; x < 4; ++x) t16[4 * v4 + x] = ldexp(t16[4 * v4 + x] * gqr, e4[x]);
  }
}

// Windows of at most 32 rows (one query head per KV head with the usual window
// of 32): the key digits of a tile are used by one wave only, so there is
// nothing to share.  Every wave converts its own tiles straight into operand
// layout -- lane (key c32, half) loads and converts the 16-channel segments
// [32 ks + 16 half, + 16) of its key, which is what it holds of the operand --
// with no staging through other waves and no barrier between the waves; the
// staged kernel's 64 KB of double-buffered digits would leave such a block's two
// waves alone on their SIMDs.
// grid = (key ranges, units); wave w of a block takes the tiles w, w + NW, ...
// of the block's range and writes a partial record of its own:
// part[unit][range][w][32][2].
template <int D, int NW>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2))) void score_i8_direct_kernel(
    const uint16_t *__restrict__ k, const v4i *__restrict__ qdig, const double *__restrict__ gq,
    const double *__restrict__ qd, const QTiny *__restrict__ qtiny, const int32_t *__restrict__ qcnt,
    double *__restrict__ part, unsigned long long *__restrict__ knorm, Dims dm, int keys_per_wg) {
  constexpr int KS = D / 32, THREADS = 64 * NW;
  const int unit = blockIdx.y, tid = threadIdx.x, w = tid >> 6, l = tid & 63, c32 = l & 31, half = l >> 5;
  const int N = dm.N, NK = dm.n_keys;
  const double unit_scale = dm.scale * EXP_UNITS;   // logits are kept in units of ln 2 / 256
  const uint16_t *kb = k + (size_t)unit * N * D;
  const double *qdu = qd + (size_t)unit * 32 * D;
  const int n_tiny_all = qcnt[unit];
  const bool q_overflow = n_tiny_all > I8_QCAP;   // then every logit takes the plain fp64 route
  const int n_tiny = q_overflow ? 0 : n_tiny_all;
  const QTiny *tiny = qtiny + (size_t)unit * I8_QCAP;

  __shared__ double s_pow[EXP_TAB];         // 2^(j/256)
  __shared__ QTiny s_ktiny[NW][I8_KCAP];    // a wave's listed key remainders of its tile; .row = key of the tile
  __shared__ int s_ek[NW][32];              // key factors of a wave's tile
  // A wave's digits wait in LDS of its own for the matrix instructions that
  // use them: held in registers (64 of them) they push others into scratch
  // memory, and a reload from there waits, in order, for the key loads of the
  // next tile that are meant to stay in flight behind the arithmetic.
  __shared__ v4i s_dig[NW][KS][4][64];
  for (int i = tid; i < EXP_TAB; i += THREADS) s_pow[i] = exp2((double)i * (1.0 / EXP_TAB));
  __syncthreads();

  const int row = c32;
  v4i qv[KS][4];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
#pragma unroll
    for (int t = 0; t < 4; ++t) qv[ks][t] = qdig[((((size_t)unit) * KS + ks) * 4 + t) * 64 + l];
  const double gqr = gq[(size_t)unit * 32 + row];
  double m = -INFINITY, ls = 0.0;
  bool q_low = false;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) q_low = q_low || (qv[ks][0][0] | qv[ks][0][1] | qv[ks][0][2] | qv[ks][0][3]) != 0;
  const bool q_low_zero = __ballot(q_low) == 0ull;

  const int kbase = blockIdx.x * keys_per_wg;
  const int kend = min(kbase + keys_per_wg, NK);
  const int n_tiles = kend > kbase ? (kend - kbase + 31) / 32 : 0;
  uint32_t raw[KS][8];
  auto fetch = [&](int tile) {
    const int j = kbase + tile * 32 + c32;
    fetch_key_pieces<D>(tile < n_tiles && j < kend ? kb + (size_t)j * D : nullptr, half, raw);
  };
  const bool want_norm = knorm != nullptr;   // the screening pass wants the largest squared key norm (over-estimated)
  float norm_best = 0.f;

  fetch(w);
  for (int tile = w; tile < n_tiles; tile += NW) {
    const int j0 = kbase + tile * 32;
    // the tile's digits, in operand layout as they are converted
    bool k_low_zero;
    const int cnt = convert_own_tile<D>(raw, kb + (size_t)min(j0 + c32, NK - 1) * D, l, s_dig[w], s_ek[w], s_ktiny[w],
                                        k_low_zero, want_norm ? &norm_best : nullptr);
    fetch(tile + NW);   // the next tile's keys travel during this tile's arithmetic
    wave_lds_handover();   // the wave's own LDS writes above are read below, in program order

    double t16[16];
    if (!q_overflow && cnt <= I8_KCAP) {
      contract_tile<KS>([&](int ks, int a) { return s_dig[w][ks][a][l]; }, qv, k_low_zero, q_low_zero, t16);
      scale_logits(t16, gqr, s_ek[w], half);
      add_row_remainders<D>(tiny, n_tiny, row, ConsecutiveKeys{j0, half, NK}, unit_scale, kb, t16);
      for (int e = 0; e < cnt; ++e) {
        const QTiny ent = s_ktiny[w][e];
        add_key_remainder<D>(ent, ent.row, half, row, qdu, tiny, n_tiny, unit_scale, t16);
      }
    } else {
      plain_logits<D>(qdu + (size_t)row * D, kb, ConsecutiveKeys{j0, half, NK}, unit_scale, t16);
    }
    join_statistics(t16, j0, half, row, dm, s_pow, m, ls);
    wave_lds_handover();   // the lists are rewritten by the next tile
  }

  if (want_norm) {
#pragma unroll
    for (int off = 16; off >= 1; off >>= 1) norm_best = fmaxf(norm_best, __shfl_xor(norm_best, off));
    if (l == 0 && norm_best > 0.f)
      atomicMax(knorm + unit, (unsigned long long)__double_as_longlong((double)norm_best * 1.001));
  }
  write_partial(m, ls, half, row, part + (((size_t)unit * gridDim.x + blockIdx.x) * NW + w) * 32 * 2);
}

// Exact column means (Eq. 13) of the columns a unit's list names, after the
// screening pass: score[j] = (1 / rows) sum_i exp(x_ij - m_i) / l_i with the
// logits of the integer contraction above and the row statistics it produced.
// A tile is 32 listed keys; every wave converts its own tiles as in
// score_i8_direct_kernel, then goes through the window's 32-row blocks with
// the tile's digits in LDS of its own: logits, exponentials against the rows'
// maxima, a running sum per key and lane.  The lanes of a key half hold the
// same sixteen keys for 32 different rows: their sums meet in LDS, one lane per
// key adds the rows up and writes the score.  grid = (blocks per unit, units);
// tiles are dealt to the waves of a unit's blocks in turn.
template <int D, int NW>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2))) void score_i8_columns_kernel(
    const uint16_t *__restrict__ k, const v4i *__restrict__ qdig, const double *__restrict__ gq,
    const double *__restrict__ qd, const QTiny *__restrict__ qtiny, const int32_t *__restrict__ qcnt,
    const double *__restrict__ stats, const int32_t *__restrict__ band_idx, const int32_t *__restrict__ band_cnt,
    double *__restrict__ scores, Dims dm) {
  constexpr int KS = D / 32, THREADS = 64 * NW;
  const int unit = blockIdx.y, tid = threadIdx.x, w = tid >> 6, l = tid & 63, c32 = l & 31, half = l >> 5;
  const int N = dm.N, L = dm.L, R = dm.R, Rpad = dm.Rpad, n_rb = Rpad / 32;
  // without a list: every column of the unit
  const int n_listed = band_idx != nullptr ? band_cnt[unit] : N;
  const int32_t *cols = band_idx != nullptr ? band_idx + (size_t)unit * N : nullptr;
  const double unit_scale = dm.scale * EXP_UNITS;
  const uint16_t *kb = k + (size_t)unit * N * D;
  const double *qdu = qd + (size_t)unit * Rpad * D;
  const double *st = stats + (size_t)unit * Rpad * 2;
  const int n_tiny_all = qcnt[unit];
  const bool q_overflow = n_tiny_all > I8_QCAP;
  const int n_tiny = q_overflow ? 0 : n_tiny_all;
  const QTiny *tiny = qtiny + (size_t)unit * I8_QCAP;

  __shared__ double s_pow[EXP_TAB];
  __shared__ QTiny s_ktiny[NW][I8_KCAP];
  __shared__ int s_ek[NW][32];
  __shared__ int s_col[NW][32];              // columns of the tile's keys, -1 past the list's end
  // a wave's digits, and in their place, when they are done with, a lane's sums
  // of its sixteen keys over the row blocks
  union TileLds {
    v4i dig[KS][4][64];
    double sum[16][64];
  };
  static_assert(sizeof(v4i) * KS * 4 * 64 >= sizeof(double) * 16 * 64, "the sums fit the digits' place");
  __shared__ TileLds s_tile[NW];
  auto &s_dig_w = s_tile[w].dig;
  auto &s_sum = s_tile[w].sum;
  for (int i = tid; i < EXP_TAB; i += THREADS) s_pow[i] = exp2((double)i * (1.0 / EXP_TAB));
  __syncthreads();

  const int n_tiles = (n_listed + 31) / 32;
  for (int tile = blockIdx.x * NW + w; tile < n_tiles; tile += gridDim.x * NW) {
    const int pos = tile * 32 + c32;
    const int col = pos < n_listed ? (cols != nullptr ? cols[pos] : pos) : -1;
    uint32_t raw[KS][8];
    const uint16_t *key_row = kb + (size_t)max(col, 0) * D;
    fetch_key_pieces<D>(col >= 0 ? key_row : nullptr, half, raw);
    bool k_low_zero;
    const int cnt = convert_own_tile<D>(raw, key_row, l, s_dig_w, s_ek[w], s_ktiny[w], k_low_zero, nullptr);
    if (half == 0) s_col[w][c32] = col;
    wave_lds_handover();   // the wave's own LDS writes above are read below, in program order

    // the lane's sixteen keys: their columns (and factors) are read from the
    // wave's LDS where they are used, not held in registers across the row blocks
    const auto key_at = [&](int v) { return s_col[w][tile_key(v, half)]; };
    const bool plain = q_overflow || cnt > I8_KCAP;
    double sum16[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) sum16[v] = 0.0;
#pragma unroll 1
    for (int rb = 0; rb < n_rb; ++rb) {
      const int row = rb * 32 + c32;
      double t16[16];
      if (!plain) {
        v4i qv[KS][4];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
          for (int t = 0; t < 4; ++t) qv[ks][t] = qdig[((((size_t)unit * n_rb + rb) * KS + ks) * 4 + t) * 64 + l];
        bool q_low = false;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) q_low = q_low || (qv[ks][0][0] | qv[ks][0][1] | qv[ks][0][2] | qv[ks][0][3]) != 0;
        contract_tile<KS>([&](int ks, int a) { return s_dig_w[ks][a][l]; }, qv, k_low_zero, __ballot(q_low) == 0ull, t16);
        scale_logits(t16, gq[(size_t)unit * Rpad + row], s_ek[w], half);
        add_row_remainders<D>(tiny, n_tiny, row, key_at, unit_scale, kb, t16);
        for (int e = 0; e < cnt; ++e) {
          const QTiny ent = s_ktiny[w][e];
          add_key_remainder<D>(ent, ent.row, half, row, qdu, tiny, n_tiny, unit_scale, t16);
        }
      } else {
        plain_logits<D>(qdu + (size_t)row * D, kb, key_at, unit_scale, t16);
      }
      // weights against the row's statistics (in table units), masked where the
      // key lies behind the row's own position or there is no row or key
      const bool row_ok = row < R;
      const double m_units = row_ok ? st[2 * row] * EXP_UNITS : 0.0;
      const double inv = row_ok ? 1.0 / st[2 * row + 1] : 0.0;
      const int last_visible = N - L + (dm.row0 + row) % L;
#pragma unroll
      for (int h8 = 0; h8 < 2; ++h8) {
        double x[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] = fmin(t16[8 * h8 + i] - m_units, 0.0);
        exp_each<8>(x, s_pow);
#pragma unroll
        for (int v4 = 0; v4 < 2; ++v4) {
          const v4i c4 = *reinterpret_cast<const v4i *>(&s_col[w][8 * (2 * h8 + v4) + 4 * half]);
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const bool vis = c4[i] >= 0 && c4[i] <= last_visible;
            sum16[8 * h8 + 4 * v4 + i] += vis ? x[4 * v4 + i] * inv : 0.0;
          }
        }
      }
    }
    // rows of a key half meet in LDS; lane t < 32 adds up key t
    wave_lds_handover();   // (all reads of the digits come before)
#pragma unroll
    for (int v = 0; v < 16; ++v) s_sum[v][l] = sum16[v];
    wave_lds_handover();
    if (l < 32) {
      const int v = 4 * (l >> 3) + (l & 3), hf = (l >> 2) & 1;
      double total = 0.0;
#pragma unroll 8
      for (int r = 0; r < 32; ++r) total += s_sum[v][32 * hf + r];
      const int out_col = s_col[w][l];
      // (a window of several row groups, all columns: the groups' launches add
      // up in the scores, which were cleared before the first)
      if (out_col >= 0) {
        double *dst = scores + (size_t)unit * N + out_col;
        const double part_mean = total / (double)dm.Rtot;
        *dst = cols == nullptr && dm.R != dm.Rtot ? *dst + part_mean : part_mean;
      }
    }
    wave_lds_handover();   // the wave's LDS is rewritten by its next tile
  }
}

// The same for windows of several 32-row blocks, where a wave that went through
// all row blocks of a tile of its own would take as many microseconds as there
// are blocks, one after the other, with most of the chip waiting for the longest
// list: here the NW waves of a block share a tile.  Wave w converts the 32-channel
// block w of the tile's keys (the keys' common exponents meet in LDS first),
// takes the row blocks w, w + NW, ... against the digits of all waves, and the
// waves' sums meet in LDS, where lane t of wave 0 adds up key t in a fixed
// order.  grid = (blocks per unit, units); tiles are dealt to a unit's blocks
// in turn.
template <int D, int NW>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2))) void score_i8_columns_shared_kernel(
    const uint16_t *__restrict__ k, const v4i *__restrict__ qdig, const double *__restrict__ gq,
    const double *__restrict__ qd, const QTiny *__restrict__ qtiny, const int32_t *__restrict__ qcnt,
    const double *__restrict__ stats, const int32_t *__restrict__ band_idx, const int32_t *__restrict__ band_cnt,
    double *__restrict__ scores, Dims dm) {
  constexpr int KS = D / 32, THREADS = 64 * NW;
  static_assert(KS <= NW, "one converting wave per 32-channel block");
  const int unit = blockIdx.y, tid = threadIdx.x, w = tid >> 6, l = tid & 63, c32 = l & 31, half = l >> 5;
  const int N = dm.N, L = dm.L, R = dm.R, Rpad = dm.Rpad, n_rb = Rpad / 32;
  const int n_listed = band_cnt[unit];
  const int32_t *cols = band_idx + (size_t)unit * N;
  const double unit_scale = dm.scale * EXP_UNITS;
  const uint16_t *kb = k + (size_t)unit * N * D;
  const double *qdu = qd + (size_t)unit * Rpad * D;
  const double *st = stats + (size_t)unit * Rpad * 2;
  const int n_tiny_all = qcnt[unit];
  const bool q_overflow = n_tiny_all > I8_QCAP;
  const int n_tiny = q_overflow ? 0 : n_tiny_all;
  const QTiny *tiny = qtiny + (size_t)unit * I8_QCAP;

  __shared__ double s_pow[EXP_TAB];
  __shared__ QTiny s_ktiny[KS][I8_KCAP];     // remainders of the elements a converting wave could not fit
  __shared__ int s_kcnt[KS];
  __shared__ int s_low[KS];                  // a converting wave met a non-zero lowest digit
  __shared__ int s_E[KS][32];                // largest exponent field of a key's channel block
  __shared__ int s_ek[32];
  __shared__ int s_col[32];                  // columns of the tile's keys, -1 past the list's end
  __shared__ v4i s_dig[KS][4][64];
  __shared__ double s_sum[NW][16][64];       // a wave's lanes' sums of their sixteen keys over its row blocks
  for (int i = tid; i < EXP_TAB; i += THREADS) s_pow[i] = exp2((double)i * (1.0 / EXP_TAB));

  v4i qv[KS][4];
  const auto load_q = [&](int rb) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int t = 0; t < 4; ++t) qv[ks][t] = qdig[((((size_t)unit * n_rb + rb) * KS + ks) * 4 + t) * 64 + l];
  };

  const int n_tiles = (n_listed + 31) / 32;
  for (int tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
    const int pos = tile * 32 + c32;
    const int col = pos < n_listed ? cols[pos] : -1;
    const uint16_t *key_row = kb + (size_t)max(col, 0) * D;
    uint32_t raw[8];
#pragma unroll
    for (int x = 0; x < 8; ++x) raw[x] = 0u;
    if (w < KS && col >= 0) {
      const uint4 lo = *reinterpret_cast<const uint4 *>(key_row + w * 32 + half * 16);
      const uint4 hi = *reinterpret_cast<const uint4 *>(key_row + w * 32 + half * 16 + 8);
      raw[0] = lo.x; raw[1] = lo.y; raw[2] = lo.z; raw[3] = lo.w;
      raw[4] = hi.x; raw[5] = hi.y; raw[6] = hi.z; raw[7] = hi.w;
    }
    if (w < KS) {
      int Ew = row_exponent_of(raw);
      Ew = max(Ew, __shfl_xor(Ew, 32));
      if (half == 0) s_E[w][c32] = Ew;
    }
    if (w == 0 && half == 0) s_col[c32] = col;
    __syncthreads();   // (also: the table, and the previous tile's readers are done)
    int E = 1;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) E = max(E, s_E[ks][c32]);
    if (w < KS) {
      v4i dig[4];
      const bool ok = digits_of(raw, E, dig);
      const bool k_low = (dig[0][0] | dig[0][1] | dig[0][2] | dig[0][3]) != 0;
#pragma unroll
      for (int t = 0; t < 4; ++t) s_dig[w][t][l] = dig[t];
      int cnt = 0;
      unsigned long long bad = __ballot(!ok);
      while (bad) {
        const int src = __ffsll((long long)bad) - 1;
        bad &= bad - 1;
        if (l == src) {
#pragma unroll 1
          for (int i = 0; i < 16; ++i) {
            const int c = w * 32 + half * 16 + i;
            double rem;
            if (!remainder_of(key_row[c], E, rem)) continue;
            if (cnt < I8_KCAP) {
              QTiny ent;
              ent.row = c32;
              ent.c = c;
              ent.r = rem;
              s_ktiny[w][cnt] = ent;
            }
            ++cnt;
          }
        }
        cnt = __shfl(cnt, src);
      }
      const bool any_low = __ballot(k_low) != 0ull;
      if (l == 0) {
        s_kcnt[w] = cnt;
        s_low[w] = any_low ? 1 : 0;
      }
      if (w == 0 && half == 0) s_ek[c32] = E - (2 * I8_GRID - 126);
    }
    __syncthreads();
    bool k_low_zero = true, plain = q_overflow;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      k_low_zero = k_low_zero && s_low[ks] == 0;
      plain = plain || s_kcnt[ks] > I8_KCAP;
    }

    const auto key_at = [&](int v) { return s_col[tile_key(v, half)]; };
    double sum16[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) sum16[v] = 0.0;
#pragma unroll 1
    for (int rb = w; rb < n_rb; rb += NW) {
      const int row = rb * 32 + c32;
      double t16[16];
      if (!plain) {
        // (requested earlier -- before the conversion, or during the exponentials
        // of the row block before -- the 64 registers push a hundred others into
        // scratch memory)
        load_q(rb);
        bool q_low = false;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) q_low = q_low || (qv[ks][0][0] | qv[ks][0][1] | qv[ks][0][2] | qv[ks][0][3]) != 0;
        contract_tile<KS>([&](int ks, int a) { return s_dig[ks][a][l]; }, qv, k_low_zero, __ballot(q_low) == 0ull, t16);
        scale_logits(t16, gq[(size_t)unit * Rpad + row], s_ek, half);
        add_row_remainders<D>(tiny, n_tiny, row, key_at, unit_scale, kb, t16);
        for (int ks = 0; ks < KS; ++ks)
          for (int e = 0; e < s_kcnt[ks]; ++e) {
            const QTiny ent = s_ktiny[ks][e];
            add_key_remainder<D>(ent, ent.row, half, row, qdu, tiny, n_tiny, unit_scale, t16);
          }
      } else {
        plain_logits<D>(qdu + (size_t)row * D, kb, key_at, unit_scale, t16);
      }
      // weights against the row's statistics (in table units), masked where the
      // key lies behind the row's own position or there is no row or key
      const bool row_ok = row < R;
      const double m_units = row_ok ? st[2 * row] * EXP_UNITS : 0.0;
      const double inv = row_ok ? 1.0 / st[2 * row + 1] : 0.0;
      const int last_visible = N - L + (dm.row0 + row) % L;
#pragma unroll
      for (int h8 = 0; h8 < 2; ++h8) {
        double x[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] = fmin(t16[8 * h8 + i] - m_units, 0.0);
        exp_each<8>(x, s_pow);
#pragma unroll
        for (int v4 = 0; v4 < 2; ++v4) {
          const v4i c4 = *reinterpret_cast<const v4i *>(&s_col[8 * (2 * h8 + v4) + 4 * half]);
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const bool vis = c4[i] >= 0 && c4[i] <= last_visible;
            sum16[8 * h8 + 4 * v4 + i] += vis ? x[4 * v4 + i] * inv : 0.0;
          }
        }
      }
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) s_sum[w][v][l] = sum16[v];
    __syncthreads();
    if (tid < 32) {
      const int v = 4 * (l >> 3) + (l & 3), hf = (l >> 2) & 1;
      double total = 0.0;
      for (int ww = 0; ww < NW; ++ww)
#pragma unroll 8
        for (int r = 0; r < 32; ++r) total += s_sum[ww][v][32 * hf + r];
      const int out_col = s_col[l];
      if (out_col >= 0) scores[(size_t)unit * N + out_col] = total / (double)dm.Rtot;
    }
    // (the next tile's first barrier comes after its writes of s_E and s_col only:
    // s_col is read by wave 0 above, so that barrier alone does not protect it)
    __syncthreads();
  }
}

// Row statistics of a window of at most 32 rows (see score_i8_direct_kernel);
// the window rows' digits are in `bufs`.  max_parts: partial records per unit
// that `part` has room for; *n_parts: records written.
int launch_i8_direct(const Dims &dm, const void *k, const double *qd, const I8Bufs &bufs, double *part,
                     unsigned long long *knorm, int max_parts, int *n_parts, hipStream_t s) {
  auto kk = static_cast<const uint16_t *>(k);
  auto qdig = static_cast<const v4i *>(bufs.qdig);
  // Enough tiles per wave to pay for its set-up (the row block's operands, the
  // table), few enough for two waves on every SIMD, and no more partial records
  // than there is room for.
  constexpr int DNW = 4;
  const int tiles = (dm.n_keys + 31) / 32, n_cu = bufs.prof ? bufs.prof->n_cu : 256;
  int per_wave = (int)(((int64_t)tiles * dm.units + n_cu * 8 - 1) / (n_cu * 8));
  per_wave = per_wave < 4 ? 4 : per_wave;
  int n_blk = (tiles + DNW * per_wave - 1) / (DNW * per_wave);
  while (n_blk * DNW > max_parts && n_blk > 1) n_blk = (n_blk + 1) / 2;
  const int keys_per_blk = ((tiles + n_blk - 1) / n_blk) * 32;
  n_blk = (dm.n_keys + keys_per_blk - 1) / keys_per_blk;
  *n_parts = n_blk * DNW;
  const dim3 grid(n_blk, dm.units), block(64 * DNW);
  if (dm.D == 64)
    launch_profiled(bufs.prof, 2, score_i8_direct_kernel<64, DNW>, grid, block, s, kk, qdig, bufs.gq, qd, bufs.qtiny,
                    bufs.qcnt, part, knorm, dm, keys_per_blk);
  else
    launch_profiled(bufs.prof, 2, score_i8_direct_kernel<128, DNW>, grid, block, s, kk, qdig, bufs.gq, qd, bufs.qtiny,
                    bufs.qcnt, part, knorm, dm, keys_per_blk);
  return hip_ok(hipGetLastError());
}

// Exact scores of the listed columns of every unit (see score_i8_columns_kernel);
// band_idx == nullptr: of all columns (the pass of a layer that does not screen).
// The window rows' digits, factors and remainder lists are those launch_i8_stats
// left in `bufs` for the same rows.
int launch_i8_columns(const Dims &dm, const void *k, const double *qd, const I8Bufs &bufs, const double *stats,
                      const int32_t *band_idx, const int32_t *band_cnt, double *scores, int blocks_per_unit,
                      hipStream_t s) {
  auto kk = static_cast<const uint16_t *>(k);
  auto qdig = static_cast<const v4i *>(bufs.qdig);
  constexpr int CNW = 4;
  const dim3 grid(blocks_per_unit < 1 ? 1 : blocks_per_unit, dm.units), block(64 * CNW);
  // Several row blocks and short lists: the waves of a block share a tile.  A
  // block then takes one tile at a time where its waves would take one each, so
  // it pays up to about two tiles per block (a few hundred listed columns per
  // unit: 32 units of 128 rows 27 -> 21 us, 8 units of 128 rows 22 -> 12 us,
  // 64 units of 256 rows 43 -> 42 us); the lists of a
  // pooled middle pick carry the neighbours of every band column, several
  // thousand columns per unit, and stay with the kernel of a tile per wave
  // (8-head stack at 60 %: 0.305 against 0.311 ms per layer).
  if (dm.Rpad > 32 && dm.pool == 1 && band_idx != nullptr) {
    if (dm.D == 64)
      score_i8_columns_shared_kernel<64, CNW><<<grid, block, 0, s>>>(kk, qdig, bufs.gq, qd, bufs.qtiny, bufs.qcnt, stats,
                                                                    band_idx, band_cnt, scores, dm);
    else
      score_i8_columns_shared_kernel<128, CNW><<<grid, block, 0, s>>>(kk, qdig, bufs.gq, qd, bufs.qtiny, bufs.qcnt, stats,
                                                                     band_idx, band_cnt, scores, dm);
    return hip_ok(hipGetLastError());
  }
  if (dm.D == 64)
    score_i8_columns_kernel<64, CNW><<<grid, block, 0, s>>>(kk, qdig, bufs.gq, qd, bufs.qtiny, bufs.qcnt, stats, band_idx,
                                                            band_cnt, scores, dm);
  else
    score_i8_columns_kernel<128, CNW><<<grid, block, 0, s>>>(kk, qdig, bufs.gq, qd, bufs.qtiny, bufs.qcnt, stats, band_idx,
                                                             band_cnt, scores, dm);
  return hip_ok(hipGetLastError());
}

}  // namespace taskkv
