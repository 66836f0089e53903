// Decode attention over the ragged cache: split-K partial kernels + fixed-order
// combine.  The workload is HBM-bound (each kept K and V row is read once per
// step and shared by the G query heads of the group); the matrix cores are
// used because q.K^T and p.V are contractions and G*d FMAs per token would
// saturate the vector ALUs long before HBM.
//
// Work decomposition: the token space of the cache is cut into CHUNK-token
// pieces; regions are CHUNK aligned, so piece c belongs to exactly one unit
// (binary search in offsets).  A 131072-token heterogeneous unit becomes 256
// work items, a 1028-token unit 3: load balance comes from the grid, not from
// a scheduler.  Each work item writes an online-softmax partial (m, l, o) per
// query head; the combine kernel merges a unit's partials in ascending chunk
// order, so the result does not depend on execution order.
#include <math.h>

#include "taskkv_internal.h"

namespace taskkv {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;

__device__ __forceinline__ int find_unit_d(const int64_t *__restrict__ offsets, int n_units, int64_t tok) {
  if (tok >= offsets[n_units]) return -1;
  int lo = 0, hi = n_units - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (offsets[mid] <= tok) lo = mid; else hi = mid - 1;
  }
  return lo;
}

union Frag {
  uint4 u;
  bf16x8 b;
};

// bf16 cache, matrix-core path.  Block = 4 waves; wave w takes pages w, w+4, ...
// of its chunk.  Per 32-token page and wave: 2*D/32 MFMAs for S^T = K q^T
// (rows = tokens, columns = the <=16 query heads of the group), online softmax
// in the exp2 domain, then 2*D/16 MFMAs for O^T += V^T P^T with P split into
// bf16 high and low parts so the probabilities keep ~16 bits.
template <int D>
__global__ __launch_bounds__(256) void decode_bf16_kernel(
    const uint16_t *__restrict__ q, const uint4 *__restrict__ kc, const uint4 *__restrict__ vc,
    const int64_t *__restrict__ offsets, const int32_t *__restrict__ lens, float *__restrict__ pm,
    float *__restrict__ pl, float *__restrict__ po, int n_units, int Hq, int Hkv, int G,
    float scale_log2) {
  constexpr int KK = D / 32, MB = D / 16;
  const int chunk = blockIdx.x, hg = blockIdx.y;
  const int64_t tok0 = (int64_t)chunk * CHUNK;
  const int u = find_unit_d(offsets, n_units, tok0);
  if (u < 0) return;
  const int local0 = (int)(tok0 - offsets[u]);
  const int len = lens[u];
  if (local0 >= len) return;
  const int n_tok = min(CHUNK, len - local0);
  const int n_pages = (n_tok + PAGE - 1) / PAGE;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, g = l >> 4, c = l & 15;
  const int b = u / Hkv, h = u % Hkv;
  const int slot = hg * 16 + c;

  Frag qv[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) qv[kk].u = make_uint4(0, 0, 0, 0);
  if (slot < G) {
    const uint16_t *qp = q + ((size_t)b * Hq + (size_t)h * G + slot) * D;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qv[kk].u = *reinterpret_cast<const uint4 *>(qp + 32 * kk + 8 * g);
  }

  float m_run = -INFINITY, l_run = 0.f;
  floatx4 acc[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) acc[mb] = floatx4{0.f, 0.f, 0.f, 0.f};

  for (int pg = w; pg < n_pages; pg += 4) {
    const uint4 *kp = kc + ((size_t)tok0 + (size_t)pg * PAGE) * (D / 8);
    const uint4 *vp = vc + ((size_t)tok0 + (size_t)pg * PAGE) * (D / 8);
    Frag kr[2][KK], vr[MB];
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) kr[sb][kk].u = kp[sb * 2 * D + kk * 64 + l];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) vr[mb].u = vp[mb * 64 + l];

    floatx4 s[2];
#pragma unroll
    for (int sb = 0; sb < 2; ++sb) {
      s[sb] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < KK; ++kk)
        s[sb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kr[sb][kk].b, qv[kk].b, s[sb], 0, 0, 0);
    }
    float sv[8];
    float mloc = -INFINITY;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int t = pg * PAGE + 16 * (e >> 2) + 4 * g + (e & 3);
      sv[e] = t < n_tok ? s[e >> 2][e & 3] * scale_log2 : -INFINITY;
      mloc = fmaxf(mloc, sv[e]);
    }
    mloc = fmaxf(mloc, __shfl_xor(mloc, 16));
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
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
    for (int mb = 0; mb < MB; ++mb) {
      acc[mb] *= alpha;
      acc[mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vr[mb].b, ph.b, acc[mb], 0, 0, 0);
      acc[mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vr[mb].b, plo.b, acc[mb], 0, 0, 0);
    }
  }

  // merge the four waves (fixed order) and write the chunk's partial
  __shared__ float sm[4][16], sl[4][16];
  __shared__ float so[4][16][D + 1];
  float l_tot = l_run + __shfl_xor(l_run, 16);
  l_tot += __shfl_xor(l_tot, 32);
  if (g == 0) { sm[w][c] = m_run; sl[w][c] = l_tot; }
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int i = 0; i < 4; ++i) so[w][c][16 * mb + 4 * g + i] = acc[mb][i];
  __syncthreads();
  const int nh = min(16, G - hg * 16);
  for (int idx = tid; idx < nh * D; idx += 256) {
    const int cc = idx / D, dd = idx % D;
    float M = sm[0][cc];
#pragma unroll
    for (int ww = 1; ww < 4; ++ww) M = fmaxf(M, sm[ww][cc]);
    float o = 0.f, L = 0.f;
#pragma unroll
    for (int ww = 0; ww < 4; ++ww) {
      const float wgt = __builtin_amdgcn_exp2f(sm[ww][cc] - M);
      o += so[ww][cc][dd] * wgt;
      L += sl[ww][cc] * wgt;
    }
    const size_t pi = (size_t)chunk * G + hg * 16 + cc;
    po[pi * D + dd] = o;
    if (dd == 0) { pm[pi] = M; pl[pi] = L; }
  }
}

// fp32 cache, vector-ALU path (plain rows).  Small workloads only; accuracy
// first: fp32 FMA dot products, expf, fp32 accumulation.
template <int D>
__global__ __launch_bounds__(256) void decode_f32_kernel(
    const float *__restrict__ q, const float *__restrict__ kc, const float *__restrict__ vc,
    const int64_t *__restrict__ offsets, const int32_t *__restrict__ lens, float *__restrict__ pm,
    float *__restrict__ pl, float *__restrict__ po, int n_units, int Hq, int Hkv, int G, float scale) {
  const int chunk = blockIdx.x, hg = blockIdx.y;
  const int64_t tok0 = (int64_t)chunk * CHUNK;
  const int u = find_unit_d(offsets, n_units, tok0);
  if (u < 0) return;
  const int local0 = (int)(tok0 - offsets[u]);
  const int len = lens[u];
  if (local0 >= len) return;
  const int n_tok = min(CHUNK, len - local0);
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int b = u / Hkv, h = u % Hkv;
  const int nh = min(16, G - hg * 16);

  __shared__ float qs[16][D];
  __shared__ float ps[16][CHUNK];
  __shared__ float sm[16], sl[16];
  for (int idx = tid; idx < nh * D; idx += 256) {
    const int hh = idx / D, dd = idx % D;
    qs[hh][dd] = q[((size_t)b * Hq + (size_t)h * G + hg * 16 + hh) * D + dd];
  }
  __syncthreads();
  for (int t = tid; t < n_tok; t += 256) {
    const float4 *kr = reinterpret_cast<const float4 *>(kc + ((size_t)tok0 + t) * D);
    float dot[16];
#pragma unroll
    for (int hh = 0; hh < 16; ++hh) dot[hh] = 0.f;
    for (int c4 = 0; c4 < D / 4; ++c4) {
      const float4 kv = kr[c4];
#pragma unroll
      for (int hh = 0; hh < 16; ++hh) {
        if (hh < nh) {
          dot[hh] = fmaf(qs[hh][4 * c4], kv.x, dot[hh]);
          dot[hh] = fmaf(qs[hh][4 * c4 + 1], kv.y, dot[hh]);
          dot[hh] = fmaf(qs[hh][4 * c4 + 2], kv.z, dot[hh]);
          dot[hh] = fmaf(qs[hh][4 * c4 + 3], kv.w, dot[hh]);
        }
      }
    }
#pragma unroll
    for (int hh = 0; hh < 16; ++hh)
      if (hh < nh) ps[hh][t] = dot[hh] * scale;
  }
  __syncthreads();
  for (int hh = w; hh < nh; hh += 4) {
    float mx = -INFINITY;
    for (int t = lane; t < n_tok; t += 64) mx = fmaxf(mx, ps[hh][t]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    float sum = 0.f;
    for (int t = lane; t < n_tok; t += 64) {
      const float p = expf(ps[hh][t] - mx);
      ps[hh][t] = p;
      sum += p;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
    if (lane == 0) { sm[hh] = mx; sl[hh] = sum; }
  }
  __syncthreads();
  for (int idx = tid; idx < nh * D; idx += 256) {
    const int hh = idx / D, dd = idx % D;
    float o = 0.f;
    for (int t = 0; t < n_tok; ++t) o = fmaf(ps[hh][t], vc[((size_t)tok0 + t) * D + dd], o);
    const size_t pi = (size_t)chunk * G + hg * 16 + hh;
    po[pi * D + dd] = o;
    if (dd == 0) { pm[pi] = sm[hh]; pl[pi] = sl[hh]; }
  }
}

// Merge a unit's partials in ascending chunk order.  One block per (b, query
// head), one thread per output channel.
template <bool LOG2>
__global__ void combine_kernel(const float *__restrict__ pm, const float *__restrict__ pl,
                               const float *__restrict__ po, const int64_t *__restrict__ offsets,
                               const int32_t *__restrict__ lens, float *__restrict__ out, int Hq,
                               int Hkv, int G, int D) {
  const int bq = blockIdx.x, dd = threadIdx.x;
  const int b = bq / Hq, hq = bq % Hq, h = hq / G, slot = hq % G;
  const int u = b * Hkv + h;
  const int64_t chunk0 = offsets[u] / CHUNK;
  const int len = lens[u];
  const int nch = (len + CHUNK - 1) / CHUNK;
  float M = -INFINITY;
  for (int i = 0; i < nch; ++i) M = fmaxf(M, pm[(size_t)(chunk0 + i) * G + slot]);
  float L = 0.f, O = 0.f;
  for (int i = 0; i < nch; ++i) {
    const size_t pi = (size_t)(chunk0 + i) * G + slot;
    const float dlt = pm[pi] - M;
    const float wgt = LOG2 ? __builtin_amdgcn_exp2f(dlt) : expf(dlt);
    L += pl[pi] * wgt;
    O += po[pi * D + dd] * wgt;
  }
  out[(size_t)bq * D + dd] = nch > 0 ? O / L : 0.f;
}

int launch_decode(taskkv_ctx *ctx, const Dims &dm, int dtype, const void *q, const void *k_cache,
                  const void *v_cache, int64_t capacity, const int64_t *offsets, const int32_t *lens,
                  float *pm, float *pl, float *po, float *out, hipStream_t s) {
  const dim3 grid((unsigned)(capacity / CHUNK), (dm.G + 15) / 16), block(256);
  const bool prof = ctx->profiling && ctx->n_events < MAX_PROFILE_EVENTS;
  if (prof) hipEventRecord(ctx->ev_start[ctx->n_events], s);
  if (dtype == TASKKV_F32) {
    auto qq = static_cast<const float *>(q);
    auto kc = static_cast<const float *>(k_cache), vc = static_cast<const float *>(v_cache);
    const float scale = (float)dm.scale;
    if (dm.D == 64)
      decode_f32_kernel<64><<<grid, block, 0, s>>>(qq, kc, vc, offsets, lens, pm, pl, po, dm.units, dm.Hq, dm.Hkv, dm.G, scale);
    else
      decode_f32_kernel<128><<<grid, block, 0, s>>>(qq, kc, vc, offsets, lens, pm, pl, po, dm.units, dm.Hq, dm.Hkv, dm.G, scale);
  } else {
    auto qq = static_cast<const uint16_t *>(q);
    auto kc = static_cast<const uint4 *>(k_cache), vc = static_cast<const uint4 *>(v_cache);
    const float scale_log2 = (float)(dm.scale * 1.4426950408889634);
    if (dm.D == 64)
      decode_bf16_kernel<64><<<grid, block, 0, s>>>(qq, kc, vc, offsets, lens, pm, pl, po, dm.units, dm.Hq, dm.Hkv, dm.G, scale_log2);
    else
      decode_bf16_kernel<128><<<grid, block, 0, s>>>(qq, kc, vc, offsets, lens, pm, pl, po, dm.units, dm.Hq, dm.Hkv, dm.G, scale_log2);
  }
  if (prof) {
    hipEventRecord(ctx->ev_stop[ctx->n_events], s);
    ctx->n_events++;
  }
  const dim3 cgrid(dm.B * dm.Hq), cblock(dm.D);
  if (dtype == TASKKV_F32)
    combine_kernel<false><<<cgrid, cblock, 0, s>>>(pm, pl, po, offsets, lens, out, dm.Hq, dm.Hkv, dm.G, dm.D);
  else
    combine_kernel<true><<<cgrid, cblock, 0, s>>>(pm, pl, po, offsets, lens, out, dm.Hq, dm.Hkv, dm.G, dm.D);
  return hip_ok(hipGetLastError());
}

}  // namespace taskkv
