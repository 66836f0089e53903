// Row statistics of the window scores (paper Sec. 4.1, Eq. 12) for bf16 inputs on
// the int8 matrix cores: the window rows' digits, and the kernel whose blocks
// convert a step of keys once for all their row blocks (windows above 32 rows).
// The arithmetic is described in score_i8_common.h; windows of at most 32 rows
// and the listed columns of a screening separator are in score_i8_own.hip.
#include "score_i8_common.h"

namespace taskkv {

// Window rows [row0, row0 + R) of every unit -> digit vectors in operand
// layout qdig[unit][rb][ks][t][lane] (rb: 32-row block, ks: 32 channels), the
// row factors gq = (256 / ln 2) * scale * 2^(E - 126) (logits come out in units of ln 2 / 256),
// and the list of remainders.  One wave per (unit, 32-row block).
template <int D>
__global__ __launch_bounds__(64) void q_digits_kernel(const uint16_t *__restrict__ q, v4i *__restrict__ qdig,
                                                      double *__restrict__ gq, QTiny *__restrict__ qtiny,
                                                      int32_t *__restrict__ qcnt, Dims dm) {
  constexpr int KS = D / 32;
  const int n_rb = dm.Rpad / 32;
  const int unit = blockIdx.x / n_rb, rb = blockIdx.x % n_rb, l = threadIdx.x;
  const int r = rb * 32 + (l & 31), half = l >> 5;
  uint32_t w[KS][8];
  const bool live = r < dm.R;
  if (live) {
    const int rg = dm.row0 + r;
    const int b = unit / dm.Hkv, h = unit % dm.Hkv, g = rg / dm.L, i = rg % dm.L;
    const uint16_t *src = q + (((size_t)b * dm.Hq + h * dm.G + g) * dm.L + i) * D;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const uint4 lo = *reinterpret_cast<const uint4 *>(src + ks * 32 + half * 16);
      const uint4 hi = *reinterpret_cast<const uint4 *>(src + ks * 32 + half * 16 + 8);
      w[ks][0] = lo.x; w[ks][1] = lo.y; w[ks][2] = lo.z; w[ks][3] = lo.w;
      w[ks][4] = hi.x; w[ks][5] = hi.y; w[ks][6] = hi.z; w[ks][7] = hi.w;
    }
  } else {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int x = 0; x < 8; ++x) w[ks][x] = 0u;
  }
  int E = 1;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    const int e = row_exponent_of(w[ks]);
    E = e > E ? e : E;
  }
  E = max(E, __shfl_xor(E, 32));
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    v4i dig[4];
    const bool ok = digits_of(w[ks], E, dig);
#pragma unroll
    for (int t = 0; t < 4; ++t)
      qdig[((((size_t)unit * n_rb + rb) * KS + ks) * 4 + t) * 64 + l] = dig[t];
    if (!ok) {
      // the remainders of the elements that do not fit go on the unit's list
      for (int x = 0; x < 16; ++x) {
        double rem;
        if (!remainder_of((x & 1) ? (w[ks][x >> 1] >> 16) : (w[ks][x >> 1] & 0xffffu), E, rem)) continue;
        const int at = atomicAdd(qcnt + unit, 1);
        if (at < I8_QCAP) {
          QTiny ent;
          ent.row = r;
          ent.c = ks * 32 + half * 16 + x;
          ent.r = rem;
          qtiny[(size_t)unit * I8_QCAP + at] = ent;
        }
      }
    }
  }
  if (half == 0) gq[(size_t)unit * dm.Rpad + r] = ldexp(dm.scale * EXP_UNITS, E - 126);
}

__global__ void zero_i32_kernel(int32_t *p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

// part[unit][n_parts][Rpad][2] <- (row maximum, denominator) over the keys of
// this block; grid = (key ranges, units, groups of 32 NW / WPR window rows).  NW
// waves per block, one 32-row block each: 8, or 4 when the window has at most
// 128 rows (two such blocks share a compute unit, so that every SIMD still
// holds two waves with rows to work on).
// Windows of 64 rows have fewer 32-row blocks than a block has waves: there
// WPR = 2 waves share a row block and take one of the two 32-key tiles of a
// step each, and each writes a partial record of its own.  (Windows of at most
// 32 rows: score_i8_direct_kernel.)
template <int D, int NW, int WPR>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2))) void score_i8_stats_kernel(
    const uint16_t *__restrict__ k, const v4i *__restrict__ qdig, const double *__restrict__ gq,
    const double *__restrict__ qd, const QTiny *__restrict__ qtiny, const int32_t *__restrict__ qcnt,
    double *__restrict__ part, unsigned long long *__restrict__ knorm, Dims dm, int keys_per_wg) {
  constexpr int KS = D / 32, SEGS = D / 16, THREADS = 64 * NW;
  const int unit = blockIdx.y, tid = threadIdx.x, w = tid >> 6, l = tid & 63, c32 = l & 31, half = l >> 5;
  const int N = dm.N, NK = dm.n_keys, L = dm.L, R = dm.R, Rpad = dm.Rpad, row0 = dm.row0;
  const int n_rb = Rpad / 32;
  const double unit_scale = dm.scale * EXP_UNITS;   // logits are kept in units of ln 2 / 256
  const uint16_t *kb = k + (size_t)unit * N * D;
  const double *qdu = qd + (size_t)unit * Rpad * D;
  const int n_tiny_all = qcnt[unit];
  const bool q_overflow = n_tiny_all > I8_QCAP;   // then every logit takes the plain fp64 route
  const int n_tiny = q_overflow ? 0 : n_tiny_all;
  const QTiny *tiny = qtiny + (size_t)unit * I8_QCAP;

  __shared__ v4i s_dig[2][I8_KEYS / 32][KS][4][64];
  __shared__ int s_ek[2][I8_KEYS];                   // key factor f_k = 2^s_ek
  __shared__ QTiny s_ktiny[2][NW][I8_KCAP];   // .row = key of the step
  __shared__ int s_kcnt[2][NW];
  __shared__ int s_knz[2][NW];                       // bit t: tile t of the step has a non-zero lowest key digit
  __shared__ double s_pow[EXP_TAB];                  // 2^(j/256)
  for (int i = tid; i < EXP_TAB; i += THREADS) s_pow[i] = exp2((double)i * (1.0 / EXP_TAB));

  // my 32-row block: operands, factor, statistics (lane: row c32)
  constexpr int RBB = NW / WPR;   // row blocks per block
  const int rb = blockIdx.z * RBB + w % RBB, sub = w / RBB;
  const bool have = rb < n_rb;
  const int row = (have ? rb : 0) * 32 + c32;
  v4i qv[KS][4];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
#pragma unroll
    for (int t = 0; t < 4; ++t)
      qv[ks][t] = qdig[((((size_t)unit * n_rb + (have ? rb : 0)) * KS + ks) * 4 + t) * 64 + l];
  const double gqr = gq[(size_t)unit * Rpad + row];
  double m = -INFINITY, ls = 0.0;
  // The lowest digit of an element is non-zero only if the element is 2^14 times
  // smaller than the largest of its row, so the lowest digits of a whole 32-row
  // block (all channels) are often all zero: the products with them are left out.
  bool q_low = false;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) q_low = q_low || (qv[ks][0][0] | qv[ks][0][1] | qv[ks][0][2] | qv[ks][0][3]) != 0;
  const bool q_low_zero = __ballot(q_low) == 0ull;

  const int kbase = blockIdx.x * keys_per_wg;
  const int kend = min(kbase + keys_per_wg, NK);
  const int n_steps = kend > kbase ? (kend - kbase + I8_KEYS - 1) / I8_KEYS : 0;

  // converter role: thread -> ITEMS (key of the step, 16-channel segment)
  // pairs; the SEGS threads of a key sit in adjacent lanes, and the keys of a
  // wave's item all lie in one tile
  constexpr int ITEMS = (I8_KEYS * SEGS + THREADS - 1) / THREADS;
  uint32_t raw[ITEMS][8];
  auto fetch = [&](int step) {
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
      const int item = tid + it * THREADS, ck = item / SEGS, cseg = item % SEGS;
      const int j = kbase + step * I8_KEYS + ck;
      if (item < I8_KEYS * SEGS && step < n_steps && j < NK) {
        const uint4 lo = *reinterpret_cast<const uint4 *>(kb + (size_t)j * D + cseg * 16);
        const uint4 hi = *reinterpret_cast<const uint4 *>(kb + (size_t)j * D + cseg * 16 + 8);
        raw[it][0] = lo.x; raw[it][1] = lo.y; raw[it][2] = lo.z; raw[it][3] = lo.w;
        raw[it][4] = hi.x; raw[it][5] = hi.y; raw[it][6] = hi.z; raw[it][7] = hi.w;
      } else {
#pragma unroll
        for (int x = 0; x < 8; ++x) raw[it][x] = 0u;
      }
    }
  };
  // the screening pass wants the largest squared key norm of the unit (slightly
  // over-estimated): the converters see every key once
  const bool want_norm = knorm != nullptr && blockIdx.z == 0;
  float norm_best = 0.f;
  auto convert = [&](int buf) {
    int cnt = 0;   // entries on this wave's list of key remainders
    int low_tiles = 0;   // tiles in which one of this wave's keys has a non-zero lowest digit
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
      const int item = tid + it * THREADS, ck = item / SEGS, cseg = item % SEGS;
      const bool converter = item < I8_KEYS * SEGS;
      if (want_norm) {
        float ss = 0.f;
#pragma unroll
        for (int x = 0; x < 8; ++x) {
          const float lo = __uint_as_float(raw[it][x] << 16), hi = __uint_as_float(raw[it][x] & 0xffff0000u);
          ss = fmaf(lo, lo, ss);
          ss = fmaf(hi, hi, ss);
        }
#pragma unroll
        for (int off = 1; off < SEGS; off <<= 1) ss += __shfl_xor(ss, off);
        norm_best = fmaxf(norm_best, ss);
      }
      int E = row_exponent_of(raw[it]);
#pragma unroll
      for (int off = 1; off < SEGS; off <<= 1) E = max(E, __shfl_xor(E, off));
      v4i dig[4];
      const bool ok = digits_of(raw[it], E, dig);
      if (__ballot(converter && (dig[0][0] | dig[0][1] | dig[0][2] | dig[0][3]) != 0) != 0ull)
        low_tiles |= 1 << ((((w + it * NW) * 64) / SEGS) >> 5);   // the keys of a wave's item lie in one tile
      if (converter) {
        const int tile = ck >> 5, ks = cseg >> 1, lane = (ck & 31) + 32 * (cseg & 1);
#pragma unroll
        for (int t = 0; t < 4; ++t) s_dig[buf][tile][ks][t][lane] = dig[t];
        if (cseg == 0) s_ek[buf][ck] = E - (2 * I8_GRID - 126);   // with the row factor: 2^(Eq - I8_GRID) 2^(Ek - I8_GRID)
      }
      // remainders of the elements that do not fit: the wave's own short list,
      // filled lane by lane (no atomics, nothing to reset); a count above the
      // capacity tells the readers to take the plain route for this step
      unsigned long long bad = __ballot(converter && !ok);
      while (bad) {
        const int src = __ffsll((long long)bad) - 1;
        bad &= bad - 1;
        if (l == src) {
          for (int x = 0; x < 16; ++x) {
            double rem;
            if (!remainder_of((x & 1) ? (raw[it][x >> 1] >> 16) : (raw[it][x >> 1] & 0xffffu), E, rem)) continue;
            if (cnt < I8_KCAP) {
              QTiny ent;
              ent.row = ck;
              ent.c = cseg * 16 + x;
              ent.r = rem;
              s_ktiny[buf][w][cnt] = ent;
            }
            ++cnt;
          }
        }
        cnt = __shfl(cnt, src);
      }
    }
    if (l == 0) {
      s_kcnt[buf][w] = cnt;
      s_knz[buf][w] = low_tiles;
    }
  };

  fetch(0);
  if (n_steps > 0) convert(0);
  fetch(1);
  __syncthreads();

  for (int step = 0; step < n_steps; ++step) {
    const int buf = step & 1;
    // All waves leave the barrier together and would run the same phases at the
    // same time, the matrix pipe idle during every conversion and every
    // exponential phase: half of the waves convert after their tiles instead of
    // before them.  (Which half hardly matters: odd waves, the upper four, or
    // pairs measured within 1 % of each other; all waves on one side: 2-3 % slower.)
    const bool convert_first = (w & 1) == 0;
    if (convert_first) {
      if (step + 1 < n_steps) convert(buf ^ 1);
      fetch(step + 2);
    }
    const int jstep = kbase + step * I8_KEYS;
    int k_listed = 0, knz = 0;
    bool plain = q_overflow;
#pragma unroll
    for (int ww = 0; ww < NW; ++ww) {
      const int cw = s_kcnt[buf][ww];
      k_listed += cw;
      plain = plain || cw > I8_KCAP;
      knz |= s_knz[buf][ww];
    }
    knz = __builtin_amdgcn_readfirstlane(knz);
    if (have) {
#pragma unroll 1
      for (int tile = 0; tile < I8_KEYS / 32; ++tile) {
        const int j0 = jstep + tile * 32;
        if (j0 >= kend) break;
        if (WPR == 2 && tile != sub) continue;
        double t16[16];
        if (!plain) {
          // The tile's key digits are named where they are used: the compiler
          // then reads each from LDS once per variant and places the reads
          // itself, which leaves it fewer registers to spill than sixteen vectors
          // read up front (1-2 % of the whole compression for every block shape).
          const bool k_low_zero = !((knz >> tile) & 1);
          contract_tile<KS>([&](int ks, int a) { return s_dig[buf][tile][ks][a][l]; }, qv, k_low_zero, q_low_zero, t16);
          {
            // exponents of the lane's sixteen keys (read late: sixteen registers
            // fewer across the matrix phase keep most temporaries out of scratch memory)
            int ek[16];
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
              const v4i e4 = *reinterpret_cast<const v4i *>(&s_ek[buf][tile * 32 + 8 * v4 + 4 * half]);
#pragma unroll
              for (int x = 0; x < 4; ++x) ek[4 * v4 + x] = e4[x];
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) t16[v] = ldexp(t16[v] * gqr, ek[v]);
          }
          add_row_remainders<D>(tiny, n_tiny, row, ConsecutiveKeys{j0, half, NK}, unit_scale, kb, t16);
          // remainders of key elements that did not fit: qh[c] * r
          if (k_listed) {
            for (int ww = 0; ww < NW; ++ww) {
              const int cw = s_kcnt[buf][ww];
              for (int e = 0; e < cw; ++e) {
                const QTiny ent = s_ktiny[buf][ww][e];
                add_key_remainder<D>(ent, ent.row - tile * 32, half, row, qdu, tiny, n_tiny, unit_scale, t16);
              }
            }
          }
        } else {
          plain_logits<D>(qdu + (size_t)row * D, kb, ConsecutiveKeys{j0, half, NK}, unit_scale, t16);
        }
        join_statistics(t16, j0, half, row, dm, s_pow, m, ls);
      }
    }
    if (!convert_first) {
      if (step + 1 < n_steps) convert(buf ^ 1);
      fetch(step + 2);
    }
    __syncthreads();
  }

  if (want_norm) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) norm_best = fmaxf(norm_best, __shfl_xor(norm_best, off));
    if (l == 0 && norm_best > 0.f)
      atomicMax(knorm + unit, (unsigned long long)__double_as_longlong((double)norm_best * 1.001));
  }
  if (have) write_partial(m, ls, half, row, part + (((size_t)unit * gridDim.x + blockIdx.x) * WPR + sub) * Rpad * 2);
}

bool i8_stats_supported(const Dims &dm, int dtype) {
  return dtype == TASKKV_BF16 && (dm.D == 64 || dm.D == 128);
}

// Row statistics of one row group: digits of the window rows, then the
// statistics partials; n_wg key ranges of keys_per_wg keys each.
int launch_i8_stats(const Dims &dm, const void *q_win, const void *k, const double *qd, const I8Bufs &bufs,
                    double *part, unsigned long long *knorm, int n_wg, int keys_per_wg, bool qcnt_zeroed,
                    int *n_parts, hipStream_t s) {
  const int n_rb = dm.Rpad / 32;
  auto qq = static_cast<const uint16_t *>(q_win), kk = static_cast<const uint16_t *>(k);
  auto qdig = static_cast<v4i *>(bufs.qdig);
  if (!qcnt_zeroed) zero_i32_kernel<<<dim3((dm.units + 255) / 256), dim3(256), 0, s>>>(bufs.qcnt, dm.units);
  // waves per block, waves per row block: 8 x 1 for windows above 128 rows, 4 x 1
  // down to 96 rows (8 x 2 on few keys), 4 x 2 for 64 rows
  if (n_rb == 1) {
    // one row block: every wave for itself (score_i8_own.hip)
    if (dm.D == 64) q_digits_kernel<64><<<dim3(dm.units), dim3(64), 0, s>>>(qq, qdig, bufs.gq, bufs.qtiny, bufs.qcnt, dm);
    else q_digits_kernel<128><<<dim3(dm.units), dim3(64), 0, s>>>(qq, qdig, bufs.gq, bufs.qtiny, bufs.qcnt, dm);
    return launch_i8_direct(dm, k, qd, bufs, part, knorm, n_wg * 8, n_parts, s);
  }
  // (96- and 128-row windows on few keys in all -- a layer of 8 units x 8192
  // keys -- leave most of the chip idle as blocks of four waves: there eight
  // waves, two per row block, measured 164 -> 159 us for the whole compression;
  // from 8 units x 32768 keys on, the same shape is 3-8 % slower than 4 x 1)
  const bool few_keys = n_rb > 2 && n_rb <= 4 && (int64_t)dm.units * dm.n_keys <= 131072;
  const int nw = n_rb > 4 || few_keys ? 8 : 4, wpr = n_rb <= 2 || few_keys ? 2 : 1;
  const int rows_per_block = 32 * nw / wpr;
  const int nz = (dm.Rpad + rows_per_block - 1) / rows_per_block;
  // A block's set-up (operands of its row blocks, the table, filling the key
  // pipeline) is worth several 64-key steps: ranges of up to 1024 keys while
  // the blocks still fill the chip once (measured on 8 and 32 units of 128 rows
  // x 32768 and 65536 keys: 3-5 % of the whole compression against ranges of
  // 256 keys, 2048 keys a little slower again)
  const int slots = (bufs.prof ? bufs.prof->n_cu : 256) * (nw == 8 ? 1 : 2);
  while ((int64_t)((n_wg + 1) / 2) * dm.units * nz >= slots && keys_per_wg < 1024) {
    keys_per_wg *= 2;
    n_wg = (dm.n_keys + keys_per_wg - 1) / keys_per_wg;
  }
  const dim3 grid(n_wg, dm.units, nz);
  *n_parts = n_wg * wpr;
  auto launch = [&](auto kernel) {
    launch_profiled(bufs.prof, 2, kernel, grid, dim3(64 * nw), s, kk, qdig, bufs.gq, qd, bufs.qtiny, bufs.qcnt, part,
                    knorm, dm, keys_per_wg);
  };
  auto pick = [&](auto d) {
    constexpr int DD = decltype(d)::value;
    q_digits_kernel<DD><<<dim3(dm.units * n_rb), dim3(64), 0, s>>>(qq, qdig, bufs.gq, bufs.qtiny, bufs.qcnt, dm);
    if (nw == 8 && wpr == 1) launch(score_i8_stats_kernel<DD, 8, 1>);
    else if (nw == 8) launch(score_i8_stats_kernel<DD, 8, 2>);
    else if (wpr == 1) launch(score_i8_stats_kernel<DD, 4, 1>);
    else launch(score_i8_stats_kernel<DD, 4, 2>);
  };
  if (dm.D == 64) pick(std::integral_constant<int, 64>{});
  else pick(std::integral_constant<int, 128>{});
  return hip_ok(hipGetLastError());
}

}  // namespace taskkv
