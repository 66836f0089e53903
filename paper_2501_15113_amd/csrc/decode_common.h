// Device helpers shared by the decode attention kernels (bf16 matrix-core path).
#pragma once

#include <math.h>

#include "lane_ops.h"
#include "taskkv_internal.h"

namespace taskkv {

// Launch of a decode attention kernel (timed when profiling mode 1 is on).
template <typename... P, typename... A>
inline void launch_attention(taskkv_ctx *ctx, void (*kernel)(P...), dim3 grid, dim3 block, hipStream_t s,
                             A... args) {
  launch_profiled(ctx, 1, kernel, grid, block, s, args...);
}

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

union Frag {
  uint4 u;
  u32x4 v;
  bf16x8 b;
};

// K/V rows are read once per step and never reused by the step.  When the
// cache is larger than the L2 caches together (NT = true) nontemporal loads keep
// the stream from displacing useful lines and run measurably faster than
// ordinary loads on this part (7.5 against 6.1 TB/s from HBM; 71 MB that stay
// in the last-level cache between steps: 22.4 against 23.7 us per step); smaller
// caches use ordinary loads (9.6 MB: 12.9 against 14.7 us with nontemporal ones).
template <bool NT>
__device__ __forceinline__ u32x4 stream_load(const uint4 *p) {
  if (NT) return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
  return *reinterpret_cast<const u32x4 *>(p);
}

// Caches above this many bytes (K plus V) are streamed with nontemporal loads:
// 8 XCDs x 4 MB of L2.
constexpr size_t NT_THRESHOLD_BYTES = size_t(32) << 20;

// Unit owning token slot `tok` (largest u with offsets[u] <= tok), or -1 past
// the last region.  Few units (the common case): every lane loads its share of
// offsets at once and a ballot counts the entries <= tok -- one memory latency
// instead of a dependent binary-search chain.
__device__ __forceinline__ int find_unit_fast(const int64_t *__restrict__ offsets, int n_units,
                                              int64_t tok, int lane) {
  if (n_units > 256) return find_unit(offsets, n_units, tok);
  int64_t v[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int idx = lane + 64 * r;
    v[r] = idx <= n_units ? offsets[idx] : INT64_MAX;
  }
  int cnt = 0;
#pragma unroll
  for (int r = 0; r < 4; ++r) cnt += __popcll(__ballot(v[r] <= tok));
  // cnt entries of offsets[0..n_units] are <= tok; the last region ends at offsets[n_units]
  return cnt > n_units ? -1 : cnt - 1;
}

template <int D>
struct PageRegs {
  Frag kr[2][D / 32];
  Frag vr[D / 16];
};

template <int D, bool NT>
__device__ __forceinline__ void load_page(const uint4 *kp, const uint4 *vp, int l, PageRegs<D> &r) {
#pragma unroll
  for (int sb = 0; sb < 2; ++sb)
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk) r.kr[sb][kk].v = stream_load<NT>(kp + sb * 2 * D + kk * 64 + l);
#pragma unroll
  for (int mb = 0; mb < D / 16; ++mb) r.vr[mb].v = stream_load<NT>(vp + mb * 64 + l);
}

// One 32-token page: S^T = K q^T, online softmax (exp2 domain), O^T += V^T P^T,
// in two halves, so that a caller can request the next K tiles as soon as the
// QK^T MFMAs have consumed the current ones.
template <int D>
__device__ __forceinline__ void page_scores(const PageRegs<D> &r, const Frag (&qv)[D / 32], floatx4 (&s)[2]) {
#pragma unroll
  for (int sb = 0; sb < 2; ++sb) {
    s[sb] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk)
      s[sb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(r.kr[sb][kk].b, qv[kk].b, s[sb], 0, 0, 0);
  }
}

template <int D>
__device__ __forceinline__ void page_values(const PageRegs<D> &r, const floatx4 (&s)[2], int tok_base,
                                            int n_tok, int g, float scale_log2, float &m_run,
                                            float &l_run, floatx4 (&acc)[D / 16]) {
  float sv[8];
  float mloc = -INFINITY;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int t = tok_base + 16 * (e >> 2) + 4 * g + (e & 3);
    sv[e] = t < n_tok ? s[e >> 2][e & 3] * scale_log2 : -INFINITY;
    mloc = fmaxf(mloc, sv[e]);
  }
  mloc = max_lanes_16_32(mloc);
  const float m_new = fmaxf(m_run, mloc);  // finite: the page holds >= 1 token
  const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
  float lsum = 0.f;
  Frag ph, plo;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float p = __builtin_amdgcn_exp2f(sv[e] - m_new);
    lsum += p;
    const __bf16 hi = (__bf16)p;
    ph.b[e] = hi;
    plo.b[e] = (__bf16)(p - (float)hi);
  }
  l_run = l_run * alpha + lsum;
  m_run = m_new;
#pragma unroll
  for (int mb = 0; mb < D / 16; ++mb) {
    acc[mb] *= alpha;
    acc[mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(r.vr[mb].b, ph.b, acc[mb], 0, 0, 0);
    acc[mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(r.vr[mb].b, plo.b, acc[mb], 0, 0, 0);
  }
}

template <int D>
__device__ __forceinline__ void attend_page(const PageRegs<D> &r, const Frag (&qv)[D / 32], int tok_base,
                                            int n_tok, int g, float scale_log2, float &m_run,
                                            float &l_run, floatx4 (&acc)[D / 16]) {
  floatx4 s[2];
  page_scores<D>(r, qv, s);
  page_values<D>(r, s, tok_base, n_tok, g, scale_log2, m_run, l_run, acc);
}

template <int D, bool NT>
__device__ __forceinline__ void load_page_k(const uint4 *kp, int l, PageRegs<D> &r) {
#pragma unroll
  for (int sb = 0; sb < 2; ++sb)
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk) r.kr[sb][kk].v = stream_load<NT>(kp + sb * 2 * D + kk * 64 + l);
}
template <int D, bool NT>
__device__ __forceinline__ void load_page_v(const uint4 *vp, int l, PageRegs<D> &r) {
#pragma unroll
  for (int mb = 0; mb < D / 16; ++mb) r.vr[mb].v = stream_load<NT>(vp + mb * 64 + l);
}

}  // namespace taskkv
