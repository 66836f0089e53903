// Shared by the int8 scoring kernels (score_i8.hip, score_i8_own.hip): the row
// statistics of the window scores (paper Sec. 4.1, Eq. 12: the maximum and the
// softmax denominator of every window row) for bf16 inputs, on the int8 matrix
// cores, with fp64 accuracy.
//
// The decisions downstream (Eq. 14 top-t, the middle-activation pick of
// Sec. 4.2) need the denominators to about 1e-10, which fp32 logits cannot
// give, and the fp64 matrix instruction of this part sustains only 45 TFLOP/s.
// bf16 operands, however, make the dot products exactly computable in
// integers: an element is +-M * 2^(e - 134) with an 8-bit M.  Every row (of
// the window and of K) gets its own exponent E = the largest e of the row, and
// an element is placed on the row's grid as H = M << (e - E + 22), a number
// below 2^30.  The signed value S = +-H is cut into four balanced base-256
// digits, d0 ... d2 in -128 ... 127 and d3 in -64 ... 64 with
// S = d0 + 256 d1 + 256^2 d2 + 256^3 d3: they are the bytes of
// (S + 0x00808080) xor 0x00808080 -- two integer instructions per element for
// all four digits, where shifting and masking each digit out took twelve -- and
//
//   sum_c Sq[c] Sk[c] = sum_{a,b} 256^(a+b) sum_c dq_a[c] dk_b[c],
//
// where each inner sum is a v_mfma_i32_32x32x32_i8 contraction with exact
// int32 accumulation (a class a+b sums at most four digit pairs over d <= 128
// channels: below 2^23, and 256 x a class plus the next one stays below 2^31
// because the top digits are at most 64; the 32x32x32
// shape issues at twice the rate of 16x16x64 on this part: 4.8 against 2.7
// POP/s measured).  The seven class sums are combined in fp64 by Horner's rule
// from the top class down (rounding 1e-16) and scaled by the two row factors
// 2^(E - 156): the logit is then the exact dot product, rounded a few times in
// fp64, like the plain fp64 definition.
//
// Elements more than 22 binary orders below their row's largest do not fit the
// window.  They are rare (Gaussian bf16 data has them at a rate of about 1e-6
// per element) and handled without approximation.  With x = xh + r (the part
// inside the window and the remainder),
//
//   q . k = qh . kh  +  sum_c rq[c] k[c]  +  sum_c qh[c] rk[c]:
//
// the first term is the integer contraction, the second runs over a short
// per-unit list of window-row remainders, the third over a short per-step list
// of key remainders, both in fp64.  Should a list overflow (data with a huge
// dynamic range inside most rows), the logits concerned come from plain fp64
// dot products instead.
//
// Lane layout of the instruction (checked on the device): A[i][k] in lane
// i + 32 (k / 16), bytes k % 16; B[j][k] likewise; D[8 (v / 4) + 4 (l / 32) +
// v % 4][l % 32] in register v.  Keys are the A rows, window rows the B rows.
#pragma once

#include <math.h>

#include <type_traits>

#include "taskkv_internal.h"

namespace taskkv {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int I8_WAVES = 8;                 // waves per block at most, one 32-row block each
constexpr int I8_KEYS = 64;                 // keys converted per step (2 tiles of 32)
constexpr int I8_KCAP = 8;                  // listed key remainders per converting wave and step

__device__ __forceinline__ void bf16_fields(uint32_t b, int &e, int &M, bool &neg) {
  const int ef = (b >> 7) & 0xff, fr = b & 0x7f;
  M = ef ? (0x80 | fr) : fr;   // subnormals: no hidden bit, exponent field 1
  e = ef ? ef : 1;
  neg = (b & 0x8000u) != 0;
}
constexpr int I8_SHIFT = 22;               // the largest element of a row has its top bit at bit 29
constexpr int I8_GRID = 134 + I8_SHIFT;     // an element times 2^(I8_GRID - E) is its integer on the row's grid
// Part of an element inside the 30-bit window of a row with exponent E.
__device__ __forceinline__ uint32_t window_part(int M, int e, int E) {
  const int sh = e - E + I8_SHIFT;   // <= I8_SHIFT
  const uint32_t up = (uint32_t)M << (sh & 31), down = (uint32_t)M >> min(-sh, 31);
  return sh >= 0 ? up : down;   // both computed: no branch per element
}
__device__ __forceinline__ bool fits_window(int M, int e, int E) {
  const int sh = e - E + I8_SHIFT;
  const int back = min(-sh, 31);
  return sh >= 0 || (((uint32_t)M >> back) << back) == (uint32_t)M;
}
__device__ __forceinline__ double bf16_to_double(uint32_t b) { return (double)__uint_as_float(b << 16); }
// The bf16 element b in a row with exponent E: false if it fits the row's
// window, else its remainder (the element minus the part inside the window).
__device__ __forceinline__ bool remainder_of(uint32_t b, int E, double &rem) {
  int e, M;
  bool neg;
  bf16_fields(b, e, M, neg);
  if (fits_window(M, e, E)) return false;
  const double kept = ldexp((double)window_part(M, e, E), E - I8_GRID);
  rem = bf16_to_double(b) - (neg ? -kept : kept);
  return true;
}

// Exponentials of the row statistics.  Logits are kept in units of ln 2 / 256
// (the factor is folded into the rows' scale factors), so that for an argument
// x <= 0 in those units  2^(x / 256) = 2^n * 2^(j / 256) * e^(r ln2 / 256)  with
// 256 n + j = rint(x) and r = x - rint(x), |r| <= 1/2, exact: 2^(j/256) from a
// table of 256 doubles, e^(r ln2/256) - 1 from three terms (the fourth is below
// 1.5e-13).  Nine fp64 operations where the library routine takes about twice
// as many; the row statistics need one exponential per logit, which is what
// bounds the kernel.  Arguments known to be finite need no clamp (any size: a
// huge negative one ends as 2^(-large) = 0); -inf does.
constexpr int EXP_TAB = 256;
constexpr double EXP_UNITS = 369.3299304675746322841407;   // 256 / ln 2: units per natural unit

// carry * 2^(x0/256) + sum of 2^(x[v]/256) over sixteen arguments, all <= 0, in
// three sweeps -- range reduction, table reads, polynomial -- so that the
// seventeen table reads are in flight together instead of each being waited
// for where it is used.  x0 may be -inf (clamped); CLAMP says whether x[] may be.
template <bool CLAMP>
__device__ __forceinline__ double exp_sum17(double carry, double x0, const double (&x)[16], const double *tab) {
  double r[17];
  int ki[17];
#pragma unroll
  for (int v = 0; v < 17; ++v) {
    double xv = v == 16 ? x0 : x[v];
    if (CLAMP || v == 16) xv = fmax(xv, -300000.0);   // 2^-1171 = 0
    const double kf = rint(xv);
    r[v] = xv - kf;
    ki[v] = (int)kf;
  }
  double y[17];
#pragma unroll
  for (int v = 0; v < 17; ++v) y[v] = tab[ki[v] & (EXP_TAB - 1)];
  __builtin_amdgcn_sched_barrier(0);   // the compiler would otherwise move every read down to its use
#pragma unroll
  for (int v = 0; v < 17; ++v) {
    // e^(r c) - 1 with c = ln2 / 256: r (c + r (c^2/2 + r c^3/6))
    const double q = fma(r[v], 3.308302680541371e-09, 3.665565596910106e-06);
    r[v] = fma(q, r[v], 0.0027076061740622863) * r[v];
  }
  __builtin_amdgcn_sched_barrier(0);
  double sum = 0.0;
#pragma unroll
  for (int v = 0; v < 17; ++v) {
    const double e = ldexp(fma(y[v], r[v], y[v]), ki[v] >> 8);
    sum = v == 16 ? fma(carry, e, sum) : sum + e;
  }
  return sum;
}

// The same exponential for N finite arguments one by one, in place: x[v] <- 2^(x[v] / 256).
template <int N>
__device__ __forceinline__ void exp_each(double (&x)[N], const double *tab) {
  double y[N];
  int ki[N];
#pragma unroll
  for (int v = 0; v < N; ++v) {
    const double kf = rint(x[v]);
    x[v] -= kf;
    ki[v] = (int)kf;
  }
#pragma unroll
  for (int v = 0; v < N; ++v) y[v] = tab[ki[v] & (EXP_TAB - 1)];
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int v = 0; v < N; ++v) {
    const double q = fma(x[v], 3.308302680541371e-09, 3.665565596910106e-06);
    const double p = fma(q, x[v], 0.0027076061740622863) * x[v];
    x[v] = ldexp(fma(y[v], p, y[v]), ki[v] >> 8);
  }
}

// 16 elements (8 dwords of bf16 pairs) -> four 16-byte digit vectors; returns
// whether every element fits the window.  An element times 2^(I8_GRID - E) is
// below 2^30 in magnitude, so the scaling and the conversion to an integer S
// (towards zero: the magnitude keeps window_part's bits) are exact float
// operations, and the element fits when converting back returns the scaled
// value.  That test is only made when the quick one fails: a scaled magnitude
// of 128 or more has all eight mantissa bits on the grid, so if the smallest of
// the sixteen is that large everything fits (a zero, or an element 2^22 below
// its row's largest, sends the sixteen through the exact test).  The four
// balanced digits of S are the bytes of
// (S + 0x00808080) ^ 0x00808080; two rounds of byte permutes turn the four
// elements' digit bytes into one dword per digit.
__device__ __forceinline__ float scaled_element(const uint32_t (&w)[8], int x, int E) {
  const float val = __uint_as_float((x & 1) ? (w[x >> 1] & 0xffff0000u) : (w[x >> 1] << 16));
  return ldexpf(val, I8_GRID - E);
}
__device__ __forceinline__ bool digits_of(const uint32_t (&w)[8], int E, v4i (&dig)[4]) {
  float smallest = INFINITY;
#pragma unroll
  for (int x4 = 0; x4 < 4; ++x4) {
    uint32_t dd[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float scaled = scaled_element(w, 4 * x4 + i, E);
      smallest = __builtin_fminf(smallest, __builtin_fabsf(scaled));
      dd[i] = (uint32_t)((int)scaled + 0x00808080) ^ 0x00808080u;
    }
    // byte t of dd[i] -> byte i of digit t (v_perm_b32: selectors 0-3 take bytes of the second operand, 4-7 of the first)
    const uint32_t a01 = __builtin_amdgcn_perm(dd[1], dd[0], 0x05010400u), b01 = __builtin_amdgcn_perm(dd[1], dd[0], 0x07030602u);
    const uint32_t a23 = __builtin_amdgcn_perm(dd[3], dd[2], 0x05010400u), b23 = __builtin_amdgcn_perm(dd[3], dd[2], 0x07030602u);
    dig[0][x4] = (int)__builtin_amdgcn_perm(a23, a01, 0x05040100u);
    dig[1][x4] = (int)__builtin_amdgcn_perm(a23, a01, 0x07060302u);
    dig[2][x4] = (int)__builtin_amdgcn_perm(b23, b01, 0x05040100u);
    dig[3][x4] = (int)__builtin_amdgcn_perm(b23, b01, 0x07060302u);
  }
  if (smallest >= 128.f) return true;
  bool all_fit = true;
#pragma unroll
  for (int x = 0; x < 16; ++x) {
    const float scaled = scaled_element(w, x, E);
    all_fit = all_fit && (float)(int)scaled == scaled;
  }
  return all_fit;
}
// Largest exponent field (at least 1) among the non-zero elements: the field
// sits above the fraction, so it is that of the largest magnitude pattern.
__device__ __forceinline__ int row_exponent_of(const uint32_t (&w)[8]) {
  uint32_t best = 0;
#pragma unroll
  for (int x = 0; x < 8; ++x) {
    const uint32_t mag = w[x] & 0x7fff7fffu;
    best = max(best, max(mag & 0xffffu, mag >> 16));
  }
  return max((int)(best >> 7), 1);
}

// ---- pieces of a 32-key x 32-row tile that the kernels below share

// t16[v] <- sum_{a,b} 256^(a+b) sum_c dk_a[c] dq_b[c] for the lane's sixteen
// (key, row) pairs; ka(ks, a) gives the key digits a of channel block ks.
// Classes a + b = 6 ... 0: Horner from the top class down, two classes
// joined in int32 (256 x a class sum plus the next stays below 2^31) before every fp64 step.
// (Interleaving the instructions of two classes, so that no two
// consecutive ones accumulate into the same registers, was measured
// 4 % slower: the second register block costs more than it hides.)
// KZ / QZ: the tile's lowest key digits / the row block's lowest
// digits are all zero, so the products with digit 0 on that side drop out.
template <int KS, bool KZ, bool QZ, typename KA>
__device__ __forceinline__ void digit_classes(KA ka, const v4i (&qv)[KS][4], double (&t16)[16]) {
  // (the scheduler's pattern for small matrix kernels, LDS operand reads slotted between the matrix
  // instructions: 2.4 % of the whole compression at 256-row windows, 1.4 % at 128)
  __builtin_amdgcn_iglp_opt(0);
  // acc += the digit products of class cls
  auto class_sum = [&](int cls, v16i acc) {
#pragma unroll
    for (int a = KZ ? 1 : 0; a < 4; ++a) {
      const int b = cls - a;
      if (b < (QZ ? 1 : 0) || b > 3) continue;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(ka(ks, a), qv[ks][b], acc, 0, 0, 0);
    }
    return acc;
  };
  v16i zero;
#pragma unroll
  for (int v = 0; v < 16; ++v) zero[v] = 0;
  {
    const v16i top = class_sum(6, zero);
#pragma unroll
    for (int v = 0; v < 16; ++v) t16[v] = (double)top[v];
  }
#pragma unroll
  for (int cls = 5; cls >= 1; cls -= 2) {
    if (KZ && QZ && cls == 1) {
      // classes 1 and 0 are empty
#pragma unroll
      for (int v = 0; v < 16; ++v) t16[v] *= 65536.0;
    } else if ((KZ || QZ) && cls == 1) {
      const v16i hi = class_sum(1, zero);   // class 0 is empty
#pragma unroll
      for (int v = 0; v < 16; ++v) t16[v] = fma(t16[v], 65536.0, (double)(hi[v] * 256));
    } else {
      // the lower class is accumulated on top of 256 x the upper one: one
      // accumulator block instead of two
      v16i acc = class_sum(cls, zero);
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] *= 256;
      acc = class_sum(cls - 1, acc);
#pragma unroll
      for (int v = 0; v < 16; ++v) t16[v] = fma(t16[v], 65536.0, (double)acc[v]);
    }
  }
}

// Four straight-line variants of digit_classes, chosen once per tile.  The
// matrix phase runs at raised priority: when both waves of a SIMD are ready,
// the one with matrix instructions to issue goes first and the other one's
// vector work fills the gaps behind them (-2.5 %).
template <int KS, typename KA>
__device__ __forceinline__ void contract_tile(KA ka, const v4i (&qv)[KS][4], bool k_low_zero, bool q_low_zero,
                                              double (&t16)[16]) {
  __builtin_amdgcn_s_setprio(1);
  if (k_low_zero) {
    if (q_low_zero) digit_classes<KS, true, true>(ka, qv, t16);
    else digit_classes<KS, true, false>(ka, qv, t16);
  } else {
    if (q_low_zero) digit_classes<KS, false, true>(ka, qv, t16);
    else digit_classes<KS, false, false>(ka, qv, t16);
  }
  __builtin_amdgcn_s_setprio(0);
}

// Key of the tile that register v of a lane in key half `half` belongs to.
__device__ __forceinline__ int tile_key(int v, int half) { return 8 * (v >> 2) + 4 * half + (v & 3); }

// Remainders of this row's elements that did not fit: t16 += r * scale * k[c].
// key_at(v): the key of register v, or a negative number for none.
template <int D, typename KEY>
__device__ __forceinline__ void add_row_remainders(const QTiny *__restrict__ tiny, int n_tiny, int row, KEY key_at,
                                                   double unit_scale, const uint16_t *__restrict__ kb,
                                                   double (&t16)[16]) {
  for (int e = 0; e < n_tiny; ++e) {
    const QTiny ent = tiny[e];
    if (ent.row != row) continue;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int j = key_at(v);
      if (j >= 0) t16[v] += ent.r * unit_scale * bf16_to_double(kb[(size_t)j * D + ent.c]);
    }
  }
}
// The keys of a tile of 32 consecutive ones from j0 on, for a lane in key half
// `half`.  (The indices are formed where they are used on purpose: hoisted,
// their sixteen addresses and compares would be paid by every tile.)
struct ConsecutiveKeys {
  int j0, half, n_keys;
  __device__ __forceinline__ int operator()(int v) const {
    int jl = j0 + 4 * half;
    asm volatile("" : "+v"(jl));
    const int j = jl + 8 * (v >> 2) + (v & 3);
    return j < n_keys ? j : -1;
  }
};

// Remainder of one key element that did not fit (ent.c: channel, ent.r: the
// remainder; kk: the key within the tile): t16 += qh[c] * r * scale, with qh
// the part of the row's element inside its window.
template <int D>
__device__ __forceinline__ void add_key_remainder(const QTiny &ent, int kk, int half, int row,
                                                  const double *__restrict__ qdu, const QTiny *__restrict__ tiny,
                                                  int n_tiny, double unit_scale, double (&t16)[16]) {
  if (kk < 0 || kk >= 32 || ((kk >> 2) & 1) != half) return;
  double qh = qdu[(size_t)row * D + ent.c];
  for (int e2 = 0; e2 < n_tiny; ++e2) {
    const QTiny q2 = tiny[e2];
    if (q2.row == row && q2.c == ent.c) qh -= q2.r;
  }
  const int vv = 4 * (kk >> 3) + (kk & 3);
  const double add = qh * ent.r * unit_scale;
#pragma unroll
  for (int v = 0; v < 16; ++v)
    if (v == vv) t16[v] += add;
}

// Plain fp64 dot products for the lane's sixteen keys (key_at as above; a
// register without a key gets the first key's product, which nobody reads).
template <int D, typename KEY>
__device__ __forceinline__ void plain_logits(const double *__restrict__ q_row, const uint16_t *__restrict__ kb,
                                             KEY key_at, double unit_scale, double (&t16)[16]) {
#pragma unroll
  for (int v = 0; v < 16; ++v) t16[v] = 0.0;
  for (int cc = 0; cc < D; ++cc) {
    const double qe = q_row[cc];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int j = key_at(v);
      t16[v] += qe * bf16_to_double(kb[(size_t)(j >= 0 ? j : 0) * D + cc]);
    }
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) t16[v] *= unit_scale;
}

// The tile's visible logits join the running statistics (m, ls) of the lane's
// row at once: seventeen exponentials for sixteen logits, no per-logit selects.
__device__ __forceinline__ void join_statistics(double (&t16)[16], int j0, int half, int row, const Dims &dm,
                                                const double *pow_tab, double &m, double &ls) {
  const int N = dm.N, NK = dm.n_keys, L = dm.L;
  double mx = m;
  if (j0 + 31 < NK && j0 + 31 <= N - L) {
    // a tile before the window: every key is visible to every row (rows
    // past R carry zero digits; their statistics are never read), so the
    // maximum and all sixteen arguments are finite
#pragma unroll
    for (int v = 0; v < 16; ++v) mx = fmax(mx, t16[v]);
#pragma unroll
    for (int v = 0; v < 16; ++v) t16[v] -= mx;
    ls = exp_sum17<false>(ls, m - mx, t16, pow_tab);
    m = mx;
  } else {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int j = j0 + tile_key(v, half);
      const bool vis = j < NK && row < dm.R && j <= N - L + (dm.row0 + row) % L;
      t16[v] = vis ? t16[v] : -INFINITY;
      mx = fmax(mx, t16[v]);
    }
    if (mx > -INFINITY) {
#pragma unroll
      for (int v = 0; v < 16; ++v) t16[v] -= mx;
      ls = exp_sum17<true>(ls, m - mx, t16, pow_tab);
      m = mx;
    }
  }
}

// Merges the two key halves of every row (lanes l and l ^ 32) and writes the
// wave's partial record.
__device__ __forceinline__ void write_partial(double m, double ls, int half, int row, double *__restrict__ pp) {
  const double mo = __shfl_xor(m, 32), lo = __shfl_xor(ls, 32);
  const double mn = fmax(m, mo);
  if (mn > -INFINITY) ls = ls * exp2((m - mn) * (1.0 / 256)) + lo * exp2((mo - mn) * (1.0 / 256));
  if (half == 0) {
    pp[2 * row] = mn * (1.0 / EXP_UNITS);   // back to natural units
    pp[2 * row + 1] = ls;
  }
}

}  // namespace taskkv
