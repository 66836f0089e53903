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

#include "decode_common.h"

namespace taskkv {

// bf16 cache, matrix-core path.  Block = 4 waves; wave w takes pages w, w+4, ...
// of its chunk.  Per 32-token page and wave: 2*D/32 MFMAs for S^T = K q^T
// (rows = tokens, columns = the <=16 query heads of the group), online softmax
// in the exp2 domain, then 2*D/16 MFMAs for O^T += V^T P^T with P split into
// bf16 high and low parts so the probabilities keep ~16 bits.  K/V addresses
// depend only on the block index, so the first page is requested before the
// block knows which unit it serves; later pages are requested one iteration
// ahead of their use.
template <int D, bool NT>
__global__ __launch_bounds__(256) void decode_bf16_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ k_new,
    const uint16_t *__restrict__ v_new, uint4 *kc, uint4 *vc, const int64_t *__restrict__ offsets,
    const int32_t *__restrict__ lens, int32_t *__restrict__ eff_len, int *__restrict__ d_err,
    float *__restrict__ pm, float *__restrict__ pl, float *__restrict__ po, int n_units, int Hq,
    int Hkv, int G, float scale_log2) {
  constexpr int KK = D / 32, MB = D / 16, PSTRIDE = PAGE * (D / 8);  // uint4 per page
  const int chunk = blockIdx.x, hg = blockIdx.y;
  const int64_t tok0 = (int64_t)chunk * CHUNK;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, g = l >> 4, c = l & 15;
  const uint4 *kbase = kc + (size_t)tok0 * (D / 8);
  const uint4 *vbase = vc + (size_t)tok0 * (D / 8);
  PageRegs<D> ra, rb;
  load_page<D, NT>(kbase + (size_t)w * PSTRIDE, vbase + (size_t)w * PSTRIDE, l, ra);  // in bounds: whole chunks are allocated

  const int u = find_unit_fast(offsets, n_units, tok0, l);
  if (u < 0) return;
  const int64_t base = offsets[u];
  const int local0 = (int)(tok0 - base);
  const int len_old = lens[u];
  // Fused append (only when one head slice covers the group, so that this
  // block is the sole reader of the page it writes): the new token goes to
  // slot len_old of the unit; the block that owns that slot stores it, and the
  // wave that had already requested that page requests it again afterwards.
  const bool want_app = k_new != nullptr;
  const bool can_app = want_app && len_old < (int)(offsets[u + 1] - base);
  const int len = len_old + (can_app ? 1 : 0);
  if (local0 == 0 && hg == 0 && tid == 0) {
    eff_len[u] = len;
    if (want_app && !can_app) atomicOr(d_err, 1);
  }
  if (local0 >= len) return;
  if (can_app && len_old >= local0 && len_old < local0 + CHUNK) {
    if (tid < D) {
      uint16_t *kc16 = reinterpret_cast<uint16_t *>(kc), *vc16 = reinterpret_cast<uint16_t *>(vc);
      const int64_t page = base + (len_old / PAGE) * PAGE;
      const int t32 = len_old % PAGE, sb = t32 >> 4, r = t32 & 15;
      kc16[((size_t)page + sb * 16) * D + (size_t)((tid >> 3) * 16 + r) * 8 + (tid & 7)] = k_new[(size_t)u * D + tid];
      const int ga = (t32 & 15) >> 2, ea = 4 * (t32 >> 4) + (t32 & 3);
      vc16[(size_t)page * D + (size_t)((tid >> 4) * 64 + ga * 16 + (tid & 15)) * 8 + ea] = v_new[(size_t)u * D + tid];
    }
    __threadfence_block();
    __syncthreads();
    if ((len_old - local0) / PAGE == w)
      load_page<D, NT>(kbase + (size_t)w * PSTRIDE, vbase + (size_t)w * PSTRIDE, l, ra);
  }
  const int n_tok = min(CHUNK, len - local0);
  const int n_pages = (n_tok + PAGE - 1) / PAGE;
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

  for (int pg = w; pg < n_pages; pg += 8) {
    if (pg + 4 < n_pages)
      load_page<D, NT>(kbase + (size_t)(pg + 4) * PSTRIDE, vbase + (size_t)(pg + 4) * PSTRIDE, l, rb);
    attend_page<D>(ra, qv, pg * PAGE, n_tok, g, scale_log2, m_run, l_run, acc);
    if (pg + 4 < n_pages) {
      if (pg + 8 < n_pages)
        load_page<D, NT>(kbase + (size_t)(pg + 8) * PSTRIDE, vbase + (size_t)(pg + 8) * PSTRIDE, l, ra);
      attend_page<D>(rb, qv, (pg + 4) * PAGE, n_tok, g, scale_log2, m_run, l_run, acc);
    }
  }

  // merge the four waves (fixed order) and write the chunk's partial
  __shared__ float sm[4][16], sl[4][16];
  __shared__ float so[4][16][D + 1];
  const float l_tot = sum_lanes_16_32(l_run);
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

// fp32 cache, vector-ALU path (plain rows); accuracy first: fp32 FMA dot
// products, expf, fp32 accumulation.  With k_new given (only when one head
// slice covers the query group, so that this block is the sole reader of the
// row it writes) the block that owns slot len of its unit stores the new
// token before reading, and eff_len takes the length the step works with.
template <int D>
__global__ __launch_bounds__(256) void decode_f32_kernel(
    const float *__restrict__ q, const float *__restrict__ k_new, const float *__restrict__ v_new, float *kc,
    float *vc, const int64_t *__restrict__ offsets, const int32_t *__restrict__ lens,
    int32_t *__restrict__ eff_len, int *__restrict__ d_err, float *__restrict__ pm, float *__restrict__ pl,
    float *__restrict__ po, int n_units, int Hq, int Hkv, int G, float scale) {
  const int chunk = blockIdx.x, hg = blockIdx.y;
  const int64_t tok0 = (int64_t)chunk * CHUNK;
  const int u = find_unit(offsets, n_units, tok0);
  if (u < 0) return;
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int64_t base = offsets[u];
  const int local0 = (int)(tok0 - base);
  const int len_old = lens[u];
  const bool want_app = k_new != nullptr;
  const bool can_app = want_app && len_old < (int)(offsets[u + 1] - base);
  const int len = len_old + (can_app ? 1 : 0);
  if (want_app && local0 == 0 && hg == 0 && tid == 0) {
    eff_len[u] = len;
    if (!can_app) atomicOr(d_err, 1);
  }
  if (local0 >= len) return;
  if (can_app && len_old >= local0 && len_old < local0 + CHUNK) {
    if (tid < D) {
      kc[((size_t)base + len_old) * D + tid] = k_new[(size_t)u * D + tid];
      vc[((size_t)base + len_old) * D + tid] = v_new[(size_t)u * D + tid];
    }
    __threadfence_block();
    __syncthreads();
  }
  const int n_tok = min(CHUNK, len - local0);
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
  if (nh <= 4) {
    // few query heads per KV head (multi-head attention: one): D/4 lanes share a
    // token, one float4 of its row each, so that a wave's load covers whole rows
    // of 64/(D/4) consecutive tokens (fully coalesced, eight loads in flight);
    // the lanes' partial dot products are added across the token's lanes.
    constexpr int QL = D / 4, TPW = 64 / QL, U = 8;
    const int ql = lane % QL, tl = lane / QL;
    float4 qf[4];
#pragma unroll
    for (int hh = 0; hh < 4; ++hh)
      qf[hh] = hh < nh ? *reinterpret_cast<const float4 *>(&qs[hh][4 * ql]) : make_float4(0.f, 0.f, 0.f, 0.f);
    for (int t0 = w * TPW; t0 < n_tok; t0 += 4 * TPW * U) {
      float4 kv[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int t = t0 + u * 4 * TPW + tl;
        kv[u] = t < n_tok ? *reinterpret_cast<const float4 *>(kc + ((size_t)tok0 + t) * D + 4 * ql)
                          : make_float4(0.f, 0.f, 0.f, 0.f);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int t = t0 + u * 4 * TPW + tl;
#pragma unroll
        for (int hh = 0; hh < 4; ++hh) {
          if (hh < nh) {   // the same for all lanes
            float d = fmaf(qf[hh].x, kv[u].x, fmaf(qf[hh].y, kv[u].y, fmaf(qf[hh].z, kv[u].z, qf[hh].w * kv[u].w)));
#pragma unroll
            for (int off = QL / 2; off >= 1; off >>= 1) d += __shfl_xor(d, off);
            if (ql == 0 && t < n_tok) ps[hh][t] = d * scale;
          }
        }
      }
    }
  } else {
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
  }
  // p.V: NTL token lanes x D/4 channel lanes; every thread walks its tokens with
  // float4 loads of V (8 in flight), then the token lanes are added in lane order.
  // The first eight rows of every thread are requested here, ahead of the
  // softmax of the chunk, which needs no memory.
  constexpr int DL = D / 4, NTL = 256 / DL, PRE = 8;
  __shared__ float4 red[NTL][DL];
  const int dl = tid % DL, tl = tid / DL;
  float4 vpre[PRE];
#pragma unroll
  for (int i = 0; i < PRE; ++i) {
    const int t = tl + i * NTL;
    vpre[i] = t < n_tok ? *reinterpret_cast<const float4 *>(vc + ((size_t)tok0 + t) * D + 4 * dl)
                        : make_float4(0.f, 0.f, 0.f, 0.f);
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
  for (int hh = 0; hh < nh; ++hh) {
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int i = 0; i < PRE; ++i) {
      const int t = tl + i * NTL;
      const float p = t < n_tok ? ps[hh][t] : 0.f;
      acc.x = fmaf(p, vpre[i].x, acc.x); acc.y = fmaf(p, vpre[i].y, acc.y);
      acc.z = fmaf(p, vpre[i].z, acc.z); acc.w = fmaf(p, vpre[i].w, acc.w);
    }
#pragma unroll 8
    for (int t = tl + PRE * NTL; t < n_tok; t += NTL) {
      const float p = ps[hh][t];
      const float4 vv = *reinterpret_cast<const float4 *>(vc + ((size_t)tok0 + t) * D + 4 * dl);
      acc.x = fmaf(p, vv.x, acc.x); acc.y = fmaf(p, vv.y, acc.y);
      acc.z = fmaf(p, vv.z, acc.z); acc.w = fmaf(p, vv.w, acc.w);
    }
    red[tl][dl] = acc;
    __syncthreads();
    if (tid < DL) {
      float4 o = red[0][tid];
#pragma unroll
      for (int r = 1; r < NTL; ++r) {
        const float4 x = red[r][tid];
        o.x += x.x; o.y += x.y; o.z += x.z; o.w += x.w;
      }
      const size_t pi = (size_t)chunk * G + hg * 16 + hh;
      *reinterpret_cast<float4 *>(po + pi * D + 4 * tid) = o;
      if (tid == 0) { pm[pi] = sm[hh]; pl[pi] = sl[hh]; }
    }
    __syncthreads();
  }
}

// Merge a unit's partials.  One block of 1024 threads per (b, query head):
// NCL chunk lanes x D/4 channel lanes.  Chunk lane c owns chunks c, c+NCL, ...;
// it requests UN of them at once (the partials sit in L2, the loop is latency
// bound otherwise), accumulates them in ascending order, and the NCL lane sums
// are then added in lane order.  The summation order is fixed by indices
// alone, so the result is reproducible.  `len_src` holds the unit lengths valid
// for this step; when `lens_out` is given the block of the group's first head
// stores them there (this is how the fused append publishes the new length).
template <int D, bool LOG2>
__global__ __launch_bounds__(1024) void combine_kernel(const float *__restrict__ pm,
                                                       const float *__restrict__ pl,
                                                       const float *__restrict__ po,
                                                       const int64_t *__restrict__ offsets,
                                                       const int32_t *__restrict__ len_src,
                                                       int32_t *__restrict__ lens_out,
                                                       float *__restrict__ out, int Hq, int Hkv, int G) {
  constexpr int DL = D / 4, NCL = 1024 / DL, UN = 8;
  const int bq = blockIdx.x, tid = threadIdx.x;
  const int b = bq / Hq, hq = bq % Hq, h = hq / G, slot = hq % G;
  const int u = b * Hkv + h;
  const int64_t chunk0 = offsets[u] / CHUNK;
  // a unit without a region (left empty by an overflowing layout) has no
  // chunk and therefore no block that recorded its length
  const int len = offsets[u + 1] > offsets[u] ? len_src[u] : 0;
  if (lens_out != nullptr && slot == 0 && tid == 0) lens_out[u] = len;
  const int nch = (len + CHUNK - 1) / CHUNK;
  const int dl = tid % DL, cl = tid / DL;
  __shared__ float red_m[16];
  __shared__ float4 red_o[NCL][DL];
  __shared__ float red_l[NCL];
  if (nch == 0) {
    if (tid < D) out[(size_t)bq * D + tid] = 0.f;
    return;
  }
  float M = -INFINITY;
  for (int i = tid; i < nch; i += 1024) M = fmaxf(M, pm[(size_t)(chunk0 + i) * G + slot]);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
  if ((tid & 63) == 0) red_m[tid >> 6] = M;
  __syncthreads();
  M = red_m[0];
#pragma unroll
  for (int r = 1; r < 16; ++r) M = fmaxf(M, red_m[r]);
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  float lacc = 0.f;
  for (int i0 = cl; i0 < nch; i0 += NCL * UN) {
    float4 o[UN];
    float pmv[UN], plv[UN];
#pragma unroll
    for (int r = 0; r < UN; ++r) {
      const int i = i0 + r * NCL;
      const bool ok = i < nch;
      const size_t pi = (size_t)(chunk0 + (ok ? i : 0)) * G + slot;
      pmv[r] = ok ? pm[pi] : -INFINITY;
      plv[r] = ok ? pl[pi] : 0.f;
      o[r] = ok ? *reinterpret_cast<const float4 *>(po + pi * D + 4 * dl) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int r = 0; r < UN; ++r) {
      const float dlt = pmv[r] - M;
      const float wgt = LOG2 ? __builtin_amdgcn_exp2f(dlt) : expf(dlt);
      acc.x += o[r].x * wgt; acc.y += o[r].y * wgt; acc.z += o[r].z * wgt; acc.w += o[r].w * wgt;
      lacc += plv[r] * wgt;
    }
  }
  red_o[cl][dl] = acc;
  if (dl == 0) red_l[cl] = lacc;
  __syncthreads();
  if (tid < DL) {
    float4 o = red_o[0][tid];
    float L = red_l[0];
#pragma unroll
    for (int c = 1; c < NCL; ++c) {
      const float4 x = red_o[c][tid];
      o.x += x.x; o.y += x.y; o.z += x.z; o.w += x.w;
      L += red_l[c];
    }
    const float inv = 1.f / L;
    *reinterpret_cast<float4 *>(out + (size_t)bq * D + 4 * tid) = make_float4(o.x * inv, o.y * inv, o.z * inv, o.w * inv);
  }
}

int launch_decode(taskkv_ctx *ctx, const Dims &dm, int dtype, const void *q, const void *k_new,
                  const void *v_new, void *k_cache, void *v_cache, int64_t capacity,
                  const int64_t *offsets, int32_t *lens, int32_t *eff_len, float *pm, float *pl,
                  float *po, float *out, hipStream_t s) {
  const dim3 grid((unsigned)(capacity / CHUNK), (dm.G + 15) / 16), block(256);
  const dim3 cgrid(dm.B * dm.Hq), cblock(1024);
  if (dtype == TASKKV_F32) {
    // the append is fused into the attention kernel when one head slice covers
    // the query group; otherwise it runs as its own kernel first
    const bool fused = k_new != nullptr && grid.y == 1;
    if (k_new && !fused) {
      int rc = launch_append(dm, dtype, k_new, v_new, k_cache, v_cache, offsets, lens, ctx->d_err, s);
      if (rc) return rc;
    }
    auto qq = static_cast<const float *>(q);
    auto kn = fused ? static_cast<const float *>(k_new) : nullptr;
    auto vn = fused ? static_cast<const float *>(v_new) : nullptr;
    auto kc = static_cast<float *>(k_cache), vc = static_cast<float *>(v_cache);
    const float scale = (float)dm.scale;
    if (dm.D == 64)
      launch_attention(ctx, decode_f32_kernel<64>, grid, block, s, qq, kn, vn, kc, vc, offsets, lens, eff_len,
                       ctx->d_err, pm, pl, po, dm.units, dm.Hq, dm.Hkv, dm.G, scale);
    else
      launch_attention(ctx, decode_f32_kernel<128>, grid, block, s, qq, kn, vn, kc, vc, offsets, lens, eff_len,
                       ctx->d_err, pm, pl, po, dm.units, dm.Hq, dm.Hkv, dm.G, scale);
    const int32_t *len_src = fused ? eff_len : lens;
    if (dm.D == 64)
      combine_kernel<64, false><<<cgrid, cblock, 0, s>>>(pm, pl, po, offsets, len_src, fused ? lens : nullptr, out,
                                                        dm.Hq, dm.Hkv, dm.G);
    else
      combine_kernel<128, false><<<cgrid, cblock, 0, s>>>(pm, pl, po, offsets, len_src, fused ? lens : nullptr, out,
                                                         dm.Hq, dm.Hkv, dm.G);
    return hip_ok(hipGetLastError());
  }
  // bf16: the append is fused into the attention kernel when one head slice
  // covers the query group; otherwise it runs as its own kernel first.
  const bool fused = k_new != nullptr && grid.y == 1;
  if (k_new && !fused) {
    int rc = launch_append(dm, dtype, k_new, v_new, k_cache, v_cache, offsets, lens, ctx->d_err, s);
    if (rc) return rc;
  }
  auto qq = static_cast<const uint16_t *>(q);
  auto kn = fused ? static_cast<const uint16_t *>(k_new) : nullptr;
  auto vn = fused ? static_cast<const uint16_t *>(v_new) : nullptr;
  auto kc = static_cast<uint4 *>(k_cache), vc = static_cast<uint4 *>(v_cache);
  const float scale_log2 = (float)(dm.scale * 1.4426950408889634);
  const bool nt = (size_t)capacity * dm.D * 4 > NT_THRESHOLD_BYTES;
#define TASKKV_LAUNCH_CHUNK(DD, NTV)                                                                      \
  launch_attention(ctx, decode_bf16_kernel<DD, NTV>, grid, block, s, qq, kn, vn, kc, vc, offsets, lens, \
                   eff_len, ctx->d_err, pm, pl, po, dm.units, dm.Hq, dm.Hkv, dm.G, scale_log2)
  if (dm.D == 64) {
    if (nt) TASKKV_LAUNCH_CHUNK(64, true); else TASKKV_LAUNCH_CHUNK(64, false);
  } else {
    if (nt) TASKKV_LAUNCH_CHUNK(128, true); else TASKKV_LAUNCH_CHUNK(128, false);
  }
#undef TASKKV_LAUNCH_CHUNK
  if (dm.D == 64)
    combine_kernel<64, true><<<cgrid, cblock, 0, s>>>(pm, pl, po, offsets, eff_len, fused ? lens : nullptr, out, dm.Hq, dm.Hkv, dm.G);
  else
    combine_kernel<128, true><<<cgrid, cblock, 0, s>>>(pm, pl, po, offsets, eff_len, fused ? lens : nullptr, out, dm.Hq, dm.Hkv, dm.G);
  return hip_ok(hipGetLastError());
}

}  // namespace taskkv
