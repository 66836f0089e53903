// The ragged KV cache (paper Sec. 4.2): region layout, packing, export, append.
//
// Token space: unit u owns slots [offsets[u], offsets[u+1]), both multiples of
// CHUNK; lens[u] of them are filled, the rest are zero.
//
// fp32 cache: plain rows, slot p of the token space is row p.
//
// bf16 cache: laid out so that a wavefront loads matrix-core operands straight
// from HBM with one 16-byte read per lane and no shuffling:
//   K, per block of 16 tokens (16*D*2 bytes): 16-byte piece (kk, g, r) at index
//      kk*64 + g*16 + r holds K[token r][32*kk + 8*g .. +8]  -- lane g*16+r of
//      the QK^T MFMA reads piece kk*64 + lane.
//   V, per page of 32 tokens (32*D*2 bytes): 16-byte piece (mb, g, r) at index
//      mb*64 + g*16 + r holds, for e = 0..7, V[token tau(g,e)][16*mb + r] with
//      tau(g,e) = 16*(e/4) + 4*g + e%4 -- exactly the token order in which the
//      QK^T MFMA leaves its results in lane group g, so the probabilities feed
//      the PV MFMA without leaving their lane.
#include "taskkv_internal.h"

namespace taskkv {

__device__ __forceinline__ double elem_as_double(float x) { return (double)x; }
__device__ __forceinline__ double elem_as_double(uint16_t x) {
  return (double)__uint_as_float(uint32_t(x) << 16);
}

// lens / offsets from the mask (single block; units are few).  A mask that
// marks more keep-everything heads than the cfg's counts provide room for
// cannot be laid out in `capacity` tokens: the units that do not fit are left
// empty (no region, length 0), so that nothing downstream reads or writes past
// the buffer, and bit 2 of the sticky flag reports it.
// The usual case -- everything fits -- is a block-wide prefix sum of the units'
// regions (every thread takes a run of consecutive units); only a layout that
// overflows is walked unit by unit, by one thread.
__global__ __launch_bounds__(256) void layout_kernel(const uint8_t *__restrict__ mask, int64_t *__restrict__ offsets,
                                                     int32_t *__restrict__ lens, int *__restrict__ d_err, Dims dm,
                                                     int reserve, int64_t capacity) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int short_len = dm.s1 + dm.k + dm.s2;
  const auto len_of = [&](int u) { return (dm.keep_all || mask[u]) ? dm.N : short_len; };
  const auto region_of = [&](int len) {
    const int64_t cap = ((int64_t)len + reserve + CHUNK - 1) / CHUNK * CHUNK;
    return cap < CHUNK ? (int64_t)CHUNK : cap;   // every unit owns at least one chunk
  };
  const int upt = (dm.units + 255) / 256, first = tid * upt;
  int64_t own = 0;
  for (int i = 0; i < upt; ++i)
    if (first + i < dm.units) own += region_of(len_of(first + i));
  int64_t incl = own;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int64_t t = __shfl_up(incl, off);
    if (lane >= off) incl += t;
  }
  __shared__ int64_t s_wave[4];
  if (lane == 63) s_wave[wv] = incl;
  __syncthreads();
  int64_t run = incl - own;
  for (int w = 0; w < wv; ++w) run += s_wave[w];
  const int64_t total = s_wave[0] + s_wave[1] + s_wave[2] + s_wave[3];
  if (total <= capacity) {
    for (int i = 0; i < upt; ++i) {
      const int u = first + i;
      if (u >= dm.units) break;
      const int len = len_of(u);
      lens[u] = len;
      offsets[u] = run;
      run += region_of(len);
    }
    if (tid == 0) offsets[dm.units] = total;
    return;
  }
  if (tid == 0) {
    int64_t off = 0;
    for (int u = 0; u < dm.units; ++u) {
      offsets[u] = off;
      int len = len_of(u);
      int64_t cap = region_of(len);
      if (off + cap > capacity) {
        len = 0;
        cap = 0;
      }
      lens[u] = len;
      off += cap;
    }
    offsets[dm.units] = off;
    atomicOr(d_err, 2);
  }
}

__device__ __forceinline__ int tau_of(int g, int e) { return 16 * (e >> 2) + 4 * g + (e & 3); }

// Where slot p of a unit's region comes from: a source row index (>= 0), a
// compensation token (-2 - g, compressed-cache mode), or nothing (-1: zero fill).
__device__ __forceinline__ int source_of_slot(int p, int len, bool direct, const int32_t *kept_row,
                                              bool has_comp, const Dims &dm) {
  if (p >= len) return -1;
  if (direct) return p;
  if (has_comp && p >= dm.s1 && p < dm.s1 + dm.k) return -2 - (p - dm.s1);
  return kept_row[p];
}

// fp64 -> storage dtype, one rounding to nearest even.
__device__ __forceinline__ float round_store(double x, float) { return (float)x; }
__device__ __forceinline__ uint16_t round_store(double x, uint16_t) {
  const uint64_t u = (uint64_t)__double_as_longlong(x);
  const uint32_t sign = (uint32_t)(u >> 63) << 15;
  uint64_t mag = u & 0x7fffffffffffffffull;
  mag += ((mag >> 45) & 1ull) + ((1ull << 44) - 1ull);  // ties to even on the 45 dropped bits
  mag >>= 45;                                           // 11-bit exponent, 7-bit mantissa
  const uint32_t e64 = (uint32_t)(mag >> 7);
  if (e64 == 0) return (uint16_t)sign;                  // zero (subnormal doubles do not occur here)
  return (uint16_t)(sign | ((e64 - 896u) << 7) | (uint32_t)(mag & 0x7full));
}

// Compressed-cache mode (paper Sec. 6.2): one block per (group, unit); thread c
// averages channel c of the group's K rows and V rows in fp64.
template <typename T>
__global__ void group_mean_kernel(const T *__restrict__ k, const T *__restrict__ v,
                                  const uint8_t *__restrict__ mask, T *__restrict__ comp_k,
                                  T *__restrict__ comp_v, int32_t *__restrict__ kept, Dims dm) {
  const int g = blockIdx.x, u = blockIdx.y, c = threadIdx.x;
  if (dm.keep_all || mask[u]) return;
  const int64_t M = (int64_t)dm.N - dm.s1 - dm.s2;
  const int a = dm.s1 + (int)((int64_t)g * M / dm.k), b = dm.s1 + (int)((int64_t)(g + 1) * M / dm.k);
  if (c == 0) kept[(size_t)u * dm.row_stride + dm.s1 + g] = a;
  const T *kb = k + (size_t)u * dm.N * dm.D, *vb = v + (size_t)u * dm.N * dm.D;
  double sk = 0.0, sv = 0.0;
  for (int j = a; j < b; ++j) {
    sk += elem_as_double(kb[(size_t)j * dm.D + c]);
    sv += elem_as_double(vb[(size_t)j * dm.D + c]);
  }
  const double n = (double)(b - a);
  const size_t o = ((size_t)u * dm.k + g) * dm.D + c;
  comp_k[o] = round_store(sk / n, T());
  comp_v[o] = round_store(sv / n, T());
}

// One block per 32-token page of the token space.
template <int D>
__global__ __launch_bounds__(256) void pack_bf16_kernel(
    const uint16_t *__restrict__ k, const uint16_t *__restrict__ v, const int32_t *__restrict__ kept,
    const uint8_t *__restrict__ mask, const int64_t *__restrict__ offsets,
    const int32_t *__restrict__ lens, const uint16_t *__restrict__ comp_k,
    const uint16_t *__restrict__ comp_v, uint16_t *__restrict__ kc, uint16_t *__restrict__ vc, Dims dm) {
  constexpr int CH = D / 8;  // 16-byte pieces per row
  const int64_t tok0 = (int64_t)blockIdx.x * PAGE;
  const int u = find_unit(offsets, dm.units, tok0);
  if (u < 0) return;
  const int tid = threadIdx.x;
  const int local0 = (int)(tok0 - offsets[u]);
  const int len = lens[u];
  const bool direct = dm.keep_all || mask[u];
  __shared__ int src[PAGE];
  __shared__ __align__(16) uint16_t vt[PAGE][D + 8];
  if (tid < PAGE) {
    const int p = local0 + tid;
    src[tid] = source_of_slot(p, len, direct, kept + (size_t)u * dm.row_stride, comp_k != nullptr, dm);
  }
  __syncthreads();
  const size_t ubase = (size_t)u * dm.N * D;
  for (int idx = tid; idx < PAGE * CH; idx += 256) {
    const int row = idx / CH, ci = idx % CH;
    uint4 kv = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
    if (src[row] >= 0) {
      const size_t off = ubase + (size_t)src[row] * D + ci * 8;
      kv = *reinterpret_cast<const uint4 *>(k + off);
      vv = *reinterpret_cast<const uint4 *>(v + off);
    } else if (src[row] <= -2) {
      const size_t off = ((size_t)u * dm.k + (size_t)(-2 - src[row])) * D + ci * 8;
      kv = *reinterpret_cast<const uint4 *>(comp_k + off);
      vv = *reinterpret_cast<const uint4 *>(comp_v + off);
    }
    const int sb = row >> 4, r = row & 15;
    uint16_t *dst = kc + ((size_t)tok0 + sb * 16) * D + (size_t)(ci * 16 + r) * 8;
    *reinterpret_cast<uint4 *>(dst) = kv;
    *reinterpret_cast<uint4 *>(&vt[row][ci * 8]) = vv;
  }
  __syncthreads();
  for (int o = tid; o < (D / 16) * 64; o += 256) {
    const int mb = o >> 6, g = (o >> 4) & 3, r = o & 15;
    uint32_t w[4];
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      const uint32_t a = vt[tau_of(g, 2 * e2)][16 * mb + r];
      const uint32_t b = vt[tau_of(g, 2 * e2 + 1)][16 * mb + r];
      w[e2] = a | (b << 16);
    }
    *reinterpret_cast<uint4 *>(vc + (size_t)tok0 * D + (size_t)o * 8) = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

template <int D>
__global__ __launch_bounds__(256) void export_bf16_kernel(const uint16_t *__restrict__ kc,
                                                          const uint16_t *__restrict__ vc,
                                                          const int64_t *__restrict__ offsets,
                                                          uint16_t *__restrict__ k_rows,
                                                          uint16_t *__restrict__ v_rows, Dims dm) {
  constexpr int CH = D / 8;
  const int64_t tok0 = (int64_t)blockIdx.x * PAGE;
  if (tok0 >= offsets[dm.units]) return;
  const int tid = threadIdx.x;
  for (int idx = tid; idx < PAGE * CH; idx += 256) {
    const int row = idx / CH, ci = idx % CH;
    const int sb = row >> 4, r = row & 15;
    const uint16_t *srcp = kc + ((size_t)tok0 + sb * 16) * D + (size_t)(ci * 16 + r) * 8;
    *reinterpret_cast<uint4 *>(k_rows + ((size_t)tok0 + row) * D + ci * 8) =
        *reinterpret_cast<const uint4 *>(srcp);
  }
  for (int o = tid; o < (D / 16) * 64; o += 256) {
    const int mb = o >> 6, g = (o >> 4) & 3, r = o & 15;
    const uint16_t *srcp = vc + (size_t)tok0 * D + (size_t)o * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) v_rows[((size_t)tok0 + tau_of(g, e)) * D + 16 * mb + r] = srcp[e];
  }
}

// fp32 cache: plain rows.  One block per 32-token page.
template <int D>
__global__ __launch_bounds__(256) void pack_f32_kernel(
    const float *__restrict__ k, const float *__restrict__ v, const int32_t *__restrict__ kept,
    const uint8_t *__restrict__ mask, const int64_t *__restrict__ offsets,
    const int32_t *__restrict__ lens, const float *__restrict__ comp_k,
    const float *__restrict__ comp_v, float *__restrict__ kc, float *__restrict__ vc, Dims dm) {
  constexpr int CH = D / 4;
  const int64_t tok0 = (int64_t)blockIdx.x * PAGE;
  const int u = find_unit(offsets, dm.units, tok0);
  if (u < 0) return;
  const int tid = threadIdx.x;
  const int local0 = (int)(tok0 - offsets[u]);
  const int len = lens[u];
  const bool direct = dm.keep_all || mask[u];
  __shared__ int src[PAGE];
  if (tid < PAGE) {
    const int p = local0 + tid;
    src[tid] = source_of_slot(p, len, direct, kept + (size_t)u * dm.row_stride, comp_k != nullptr, dm);
  }
  __syncthreads();
  const size_t ubase = (size_t)u * dm.N * D;
  for (int idx = tid; idx < PAGE * CH; idx += 256) {
    const int row = idx / CH, ci = idx % CH;
    float4 kv = make_float4(0, 0, 0, 0), vv = kv;
    if (src[row] >= 0) {
      const size_t off = ubase + (size_t)src[row] * D + ci * 4;
      kv = *reinterpret_cast<const float4 *>(k + off);
      vv = *reinterpret_cast<const float4 *>(v + off);
    } else if (src[row] <= -2) {
      const size_t off = ((size_t)u * dm.k + (size_t)(-2 - src[row])) * D + ci * 4;
      kv = *reinterpret_cast<const float4 *>(comp_k + off);
      vv = *reinterpret_cast<const float4 *>(comp_v + off);
    }
    const size_t dst = ((size_t)tok0 + row) * D + ci * 4;
    *reinterpret_cast<float4 *>(kc + dst) = kv;
    *reinterpret_cast<float4 *>(vc + dst) = vv;
  }
}

// Append one token to every unit (paper is silent on decode-time policy; every
// head grows, as in the prefill-compression methods the paper builds on).
template <typename T, int D, bool TILED>
__global__ void append_kernel(const T *__restrict__ k_new, const T *__restrict__ v_new,
                              T *__restrict__ kc, T *__restrict__ vc,
                              const int64_t *__restrict__ offsets, int32_t *__restrict__ lens,
                              int *__restrict__ d_err) {
  const int u = blockIdx.x, c = threadIdx.x;
  const int p = lens[u];
  const int64_t base = offsets[u];
  const int64_t cap = offsets[u + 1] - base;
  __syncthreads();  // every thread has read lens[u] before it is bumped
  if (p >= cap) {
    if (c == 0) atomicOr(d_err, 1);
    return;
  }
  const T kval = k_new[(size_t)u * D + c], vval = v_new[(size_t)u * D + c];
  if (TILED) {
    const int64_t page = base + (p / PAGE) * PAGE;
    const int t32 = p % PAGE, sb = t32 >> 4, r = t32 & 15;
    kc[((size_t)page + sb * 16) * D + (size_t)((c >> 3) * 16 + r) * 8 + (c & 7)] = kval;
    const int g = (t32 & 15) >> 2, e = 4 * (t32 >> 4) + (t32 & 3);
    vc[(size_t)page * D + (size_t)((c >> 4) * 64 + g * 16 + (c & 15)) * 8 + e] = vval;
  } else {
    kc[((size_t)base + p) * D + c] = kval;
    vc[((size_t)base + p) * D + c] = vval;
  }
  if (c == 0) lens[u] = p + 1;
}

// Offsets of a stack of layers whose caches lie one after the other in one
// allocation: entry r * units + u = layer r's offsets[u] + the tokens of the
// layers before it; the last entry = all tokens.
struct StackBases {
  int64_t base[STACK_REBASE_LAYERS + 1];
};
__global__ void stack_rebase_kernel(const int64_t *__restrict__ layer_offsets, int64_t *__restrict__ stacked,
                                    StackBases bases, int layer0, int n_here, int units, int is_last) {
  const int r = blockIdx.y, u = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= n_here || u >= units) return;
  stacked[(size_t)(layer0 + r) * units + u] = layer_offsets[(size_t)(layer0 + r) * (units + 1) + u] + bases.base[r];
  if (is_last && r == n_here - 1 && u == 0) stacked[(size_t)(layer0 + n_here) * units] = bases.base[n_here];
}

int launch_stack_rebase(const int64_t *layer_offsets, const int64_t *layer_capacity, int n_layers, int units,
                        int64_t *stacked, hipStream_t s) {
  int64_t run = 0;
  for (int l0 = 0; l0 < n_layers; l0 += STACK_REBASE_LAYERS) {
    const int n_here = n_layers - l0 < STACK_REBASE_LAYERS ? n_layers - l0 : STACK_REBASE_LAYERS;
    StackBases b;
    for (int r = 0; r < n_here; ++r) {
      b.base[r] = run;
      run += layer_capacity[l0 + r];
    }
    b.base[n_here] = run;
    stack_rebase_kernel<<<dim3((units + 255) / 256, n_here), dim3(256), 0, s>>>(layer_offsets, stacked, b, l0, n_here,
                                                                              units, l0 + n_here == n_layers);
  }
  return hip_ok(hipGetLastError());
}

int launch_layout(const Dims &dm, const uint8_t *mask, int reserve, int64_t capacity, int64_t *offsets,
                  int32_t *lens, int *d_err, hipStream_t s) {
  layout_kernel<<<dim3(1), dim3(256), 0, s>>>(mask, offsets, lens, d_err, dm, reserve, capacity);
  return hip_ok(hipGetLastError());
}

int launch_group_means(const Dims &dm, int dtype, const void *k, const void *v, const uint8_t *mask,
                       void *comp_k, void *comp_v, int32_t *kept_idx, hipStream_t s) {
  const dim3 grid(dm.k, dm.units), block(dm.D);
  if (dtype == TASKKV_F32)
    group_mean_kernel<float><<<grid, block, 0, s>>>(static_cast<const float *>(k), static_cast<const float *>(v),
                                                   mask, static_cast<float *>(comp_k),
                                                   static_cast<float *>(comp_v), kept_idx, dm);
  else
    group_mean_kernel<uint16_t><<<grid, block, 0, s>>>(
        static_cast<const uint16_t *>(k), static_cast<const uint16_t *>(v), mask,
        static_cast<uint16_t *>(comp_k), static_cast<uint16_t *>(comp_v), kept_idx, dm);
  return hip_ok(hipGetLastError());
}

int launch_pack(const Dims &dm, int dtype, const void *k, const void *v, const int32_t *kept_idx,
                const uint8_t *mask, const int64_t *offsets, const int32_t *lens, const void *comp_k,
                const void *comp_v, void *k_cache, void *v_cache, int64_t capacity, hipStream_t s) {
  const dim3 grid((unsigned)(capacity / PAGE)), block(256);
  if (grid.x == 0) return TASKKV_OK;
  if (dtype == TASKKV_F32) {
    auto kk = static_cast<const float *>(k), vv = static_cast<const float *>(v);
    auto kc = static_cast<float *>(k_cache), vc = static_cast<float *>(v_cache);
    auto ck = static_cast<const float *>(comp_k), cv = static_cast<const float *>(comp_v);
    if (dm.D == 64) pack_f32_kernel<64><<<grid, block, 0, s>>>(kk, vv, kept_idx, mask, offsets, lens, ck, cv, kc, vc, dm);
    else pack_f32_kernel<128><<<grid, block, 0, s>>>(kk, vv, kept_idx, mask, offsets, lens, ck, cv, kc, vc, dm);
  } else {
    auto kk = static_cast<const uint16_t *>(k), vv = static_cast<const uint16_t *>(v);
    auto kc = static_cast<uint16_t *>(k_cache), vc = static_cast<uint16_t *>(v_cache);
    auto ck = static_cast<const uint16_t *>(comp_k), cv = static_cast<const uint16_t *>(comp_v);
    if (dm.D == 64) pack_bf16_kernel<64><<<grid, block, 0, s>>>(kk, vv, kept_idx, mask, offsets, lens, ck, cv, kc, vc, dm);
    else pack_bf16_kernel<128><<<grid, block, 0, s>>>(kk, vv, kept_idx, mask, offsets, lens, ck, cv, kc, vc, dm);
  }
  return hip_ok(hipGetLastError());
}

int launch_export(const Dims &dm, int dtype, const void *k_cache, const void *v_cache,
                  const int64_t *offsets, void *k_rows, void *v_rows, int64_t capacity, hipStream_t s) {
  if (capacity == 0) return TASKKV_OK;
  if (dtype == TASKKV_F32) {
    // plain rows already: two device-to-device copies
    const size_t bytes = (size_t)capacity * dm.D * sizeof(float);
    if (hipMemcpyAsync(k_rows, k_cache, bytes, hipMemcpyDeviceToDevice, s) != hipSuccess) return TASKKV_EHIP;
    if (hipMemcpyAsync(v_rows, v_cache, bytes, hipMemcpyDeviceToDevice, s) != hipSuccess) return TASKKV_EHIP;
    return TASKKV_OK;
  }
  const dim3 grid((unsigned)(capacity / PAGE)), block(256);
  auto kc = static_cast<const uint16_t *>(k_cache), vc = static_cast<const uint16_t *>(v_cache);
  auto kr = static_cast<uint16_t *>(k_rows), vr = static_cast<uint16_t *>(v_rows);
  if (dm.D == 64) export_bf16_kernel<64><<<grid, block, 0, s>>>(kc, vc, offsets, kr, vr, dm);
  else export_bf16_kernel<128><<<grid, block, 0, s>>>(kc, vc, offsets, kr, vr, dm);
  return hip_ok(hipGetLastError());
}

int launch_append(const Dims &dm, int dtype, const void *k_new, const void *v_new, void *k_cache,
                  void *v_cache, const int64_t *offsets, int32_t *lens, int *d_err, hipStream_t s) {
  const dim3 grid(dm.units), block(dm.D);
  if (dtype == TASKKV_F32) {
    auto kn = static_cast<const float *>(k_new), vn = static_cast<const float *>(v_new);
    auto kc = static_cast<float *>(k_cache), vc = static_cast<float *>(v_cache);
    if (dm.D == 64) append_kernel<float, 64, false><<<grid, block, 0, s>>>(kn, vn, kc, vc, offsets, lens, d_err);
    else append_kernel<float, 128, false><<<grid, block, 0, s>>>(kn, vn, kc, vc, offsets, lens, d_err);
  } else {
    auto kn = static_cast<const uint16_t *>(k_new), vn = static_cast<const uint16_t *>(v_new);
    auto kc = static_cast<uint16_t *>(k_cache), vc = static_cast<uint16_t *>(v_cache);
    if (dm.D == 64) append_kernel<uint16_t, 64, true><<<grid, block, 0, s>>>(kn, vn, kc, vc, offsets, lens, d_err);
    else append_kernel<uint16_t, 128, true><<<grid, block, 0, s>>>(kn, vn, kc, vc, offsets, lens, d_err);
  }
  return hip_ok(hipGetLastError());
}

}  // namespace taskkv
