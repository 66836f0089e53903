// Row statistics of the window scores (paper Sec. 4.1, Eq. 12: the maximum and
// the softmax denominator of every window row) for bf16 inputs, on the int8
// matrix cores, with fp64 accuracy.
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
    __builtin_amdgcn_wave_barrier();   // the wave's own LDS writes above are read below, in program order

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
    __builtin_amdgcn_wave_barrier();   // the lists are rewritten by the next tile
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
  __shared__ QTiny s_ktiny[NW][I8_KCAP];
  __shared__ int s_ek[NW][32];
  __shared__ int s_col[NW][32];              // columns of the tile's keys, -1 past the list's end
  __shared__ v4i s_dig[NW][KS][4][64];
  // a lane's sums of its sixteen keys over the row blocks, [16][64] doubles in
  // the place of the wave's digits, which are done with by then
  static_assert(sizeof(v4i) * KS * 4 * 64 >= sizeof(double) * 16 * 64, "the sums fit the digits' place");
  double(*s_sum)[64] = reinterpret_cast<double(*)[64]>(&s_dig[w][0][0][0]);
  for (int i = tid; i < EXP_TAB; i += THREADS) s_pow[i] = exp2((double)i * (1.0 / EXP_TAB));
  __syncthreads();

  const int n_tiles = (n_listed + 31) / 32;
  for (int tile = blockIdx.x * NW + w; tile < n_tiles; tile += gridDim.x * NW) {
    const int pos = tile * 32 + c32;
    const int col = pos < n_listed ? cols[pos] : -1;
    uint32_t raw[KS][8];
    const uint16_t *key_row = kb + (size_t)max(col, 0) * D;
    fetch_key_pieces<D>(col >= 0 ? key_row : nullptr, half, raw);
    bool k_low_zero;
    const int cnt = convert_own_tile<D>(raw, key_row, l, s_dig[w], s_ek[w], s_ktiny[w], k_low_zero, nullptr);
    if (half == 0) s_col[w][c32] = col;
    __builtin_amdgcn_wave_barrier();   // the wave's own LDS writes above are read below, in program order

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
        contract_tile<KS>([&](int ks, int a) { return s_dig[w][ks][a][l]; }, qv, k_low_zero, __ballot(q_low) == 0ull, t16);
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
    __builtin_amdgcn_wave_barrier();   // (all reads of the digits come before)
#pragma unroll
    for (int v = 0; v < 16; ++v) s_sum[v][l] = sum16[v];
    __builtin_amdgcn_wave_barrier();
    if (l < 32) {
      const int v = 4 * (l >> 3) + (l & 3), hf = (l >> 2) & 1;
      double total = 0.0;
#pragma unroll 8
      for (int r = 0; r < 32; ++r) total += s_sum[v][32 * hf + r];
      const int out_col = s_col[w][l];
      if (out_col >= 0) scores[(size_t)unit * N + out_col] = total / (double)dm.Rtot;
    }
    __builtin_amdgcn_wave_barrier();   // the wave's LDS is rewritten by its next tile
  }
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
  // down to 96 rows, 4 x 2 for 64 rows
  if (n_rb == 1) {
    // one row block: every wave for itself.  Enough tiles per wave to pay for
    // its set-up (the row block's operands, the table), few enough for two
    // waves on every SIMD, and no more partial records than the caller's
    // split allows for (n_wg x 8 for one row block).
    constexpr int DNW = 4;
    const int tiles = (dm.n_keys + 31) / 32, n_cu = bufs.prof ? bufs.prof->n_cu : 256;
    int per_wave = (int)(((int64_t)tiles * dm.units + n_cu * 8 - 1) / (n_cu * 8));
    per_wave = per_wave < 4 ? 4 : per_wave;
    int n_blk = (tiles + DNW * per_wave - 1) / (DNW * per_wave);
    while (n_blk * DNW > n_wg * 8 && n_blk > 1) n_blk = (n_blk + 1) / 2;
    const int keys_per_blk = ((tiles + n_blk - 1) / n_blk) * 32;
    n_blk = (dm.n_keys + keys_per_blk - 1) / keys_per_blk;
    *n_parts = n_blk * DNW;
    auto go = [&](auto d) {
      constexpr int DD = decltype(d)::value;
      q_digits_kernel<DD><<<dim3(dm.units), dim3(64), 0, s>>>(qq, qdig, bufs.gq, bufs.qtiny, bufs.qcnt, dm);
      launch_profiled(bufs.prof, 2, score_i8_direct_kernel<DD, DNW>, dim3(n_blk, dm.units), dim3(64 * DNW), s, kk, qdig,
                      bufs.gq, qd, bufs.qtiny, bufs.qcnt, part, knorm, dm, keys_per_blk);
    };
    if (dm.D == 64) go(std::integral_constant<int, 64>{});
    else go(std::integral_constant<int, 128>{});
    return hip_ok(hipGetLastError());
  }
  const int nw = n_rb > 4 ? 8 : 4, wpr = n_rb <= 2 ? 2 : 1;
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
    if (nw == 8) launch(score_i8_stats_kernel<DD, 8, 1>);
    else if (wpr == 1) launch(score_i8_stats_kernel<DD, 4, 1>);
    else launch(score_i8_stats_kernel<DD, 4, 2>);
  };
  if (dm.D == 64) pick(std::integral_constant<int, 64>{});
  else pick(std::integral_constant<int, 128>{});
  return hip_ok(hipGetLastError());
}

// Exact scores of the listed columns of every unit (see score_i8_columns_kernel).
// The window rows' digits, factors and remainder lists are those launch_i8_stats
// left in `bufs` for the same rows.
int launch_i8_columns(const Dims &dm, const void *k, const double *qd, const I8Bufs &bufs, const double *stats,
                      const int32_t *band_idx, const int32_t *band_cnt, double *scores, int blocks_per_unit,
                      hipStream_t s) {
  auto kk = static_cast<const uint16_t *>(k);
  auto qdig = static_cast<const v4i *>(bufs.qdig);
  constexpr int CNW = 4;
  const dim3 grid(blocks_per_unit < 1 ? 1 : blocks_per_unit, dm.units), block(64 * CNW);
  if (dm.D == 64)
    score_i8_columns_kernel<64, CNW><<<grid, block, 0, s>>>(kk, qdig, bufs.gq, qd, bufs.qtiny, bufs.qcnt, stats, band_idx,
                                                            band_cnt, scores, dm);
  else
    score_i8_columns_kernel<128, CNW><<<grid, block, 0, s>>>(kk, qdig, bufs.gq, qd, bufs.qtiny, bufs.qcnt, stats, band_idx,
                                                             band_cnt, scores, dm);
  return hip_ok(hipGetLastError());
}

}  // namespace taskkv
