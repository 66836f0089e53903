// Selection and ranking on fp64 scores: top-t of Eq. 14, the middle-activation
// pick of Sec. 4.2, the semantic vector of Eq. 15, centre / distance (Eq. 7-8)
// and the head ranking of Sec. 4.1.  All decisions are taken on the fp64 bit
// patterns (scores are >= 0, so unsigned integer order equals numeric order),
// ties go to the lower index.
#include <math.h>

#include "select_common.h"

namespace taskkv {

// Average pooling of the selection scores: stride 1, zero padding, fixed
// divisor (Sec. 5.4 names only the kernel size).
// A block of 256 threads stages 1024 scores and the halo on either side in LDS
// (coalesced loads, all in flight), then every thread adds up the windows of
// four outputs from there, left to right.
constexpr int POOL_SPAN = 1024, POOL_MAX_HALO = 64;
__global__ __launch_bounds__(256) void pool_kernel(const double *__restrict__ c, double *__restrict__ p, int N,
                                                   int width) {
  const int unit = blockIdx.y, tid = threadIdx.x;
  const int j0 = blockIdx.x * POOL_SPAN;
  const double *row = c + (size_t)unit * N;
  const int r = (width - 1) / 2;
  if (r > POOL_MAX_HALO) {   // windows wider than the staged halo: straight from memory
    for (int j = j0 + tid; j < min(j0 + POOL_SPAN, N); j += 256) {
      double acc = 0.0;
      for (int u = -r; u <= r; ++u) {
        const int jj = j + u;
        if (jj >= 0 && jj < N) acc += row[jj];
      }
      p[(size_t)unit * N + j] = acc / (double)width;
    }
    return;
  }
  __shared__ double s[POOL_SPAN + 2 * POOL_MAX_HALO];
  // s[i] = row[j0 - r + i], zero outside the row
  double x[5];
#pragma unroll
  for (int i = 0; i < 5; ++i) {
    const int at = tid + 256 * i, jj = j0 - r + at;
    x[i] = at < POOL_SPAN + 2 * r && jj >= 0 && jj < N ? row[jj] : 0.0;
  }
#pragma unroll
  for (int i = 0; i < 5; ++i) {
    const int at = tid + 256 * i;
    if (at < POOL_SPAN + 2 * r) s[at] = x[i];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int at = tid + 256 * i, j = j0 + at;
    if (j >= N) break;
    double acc = 0.0;
    for (int u = 0; u <= 2 * r; ++u) acc += s[at + u];
    p[(size_t)unit * N + j] = acc / (double)width;
  }
}

// One block per unit (see select_of_unit).  Units flagged in `skip` get an all
// -1 row.
__global__ __launch_bounds__(1024) void select_kernel(const double *__restrict__ scores,
                                                      const uint8_t *__restrict__ skip, int skip_all,
                                                      int N, int lo, int hi, int count, int prefix,
                                                      int gap, int suffix, int32_t *__restrict__ out,
                                                      int out_stride) {
  const int unit = blockIdx.x, tid = threadIdx.x;
  int32_t *orow = out + (size_t)unit * out_stride;
  if (skip_all || (skip && skip[unit])) {
    for (int i = tid; i < out_stride; i += 1024) orow[i] = -1;
    return;
  }
  __shared__ RadixScratch rs;
  __shared__ int s_cnt[32];
  select_of_unit(scores + (size_t)unit * N, orow, N, lo, hi, count, prefix, gap, suffix, out_stride, nullptr, 0, rs,
                 s_cnt);
}

__device__ __forceinline__ double elem_to_double(float x) { return (double)x; }
__device__ __forceinline__ double elem_to_double(uint16_t x) {
  return (double)__uint_as_float(uint32_t(x) << 16);
}

// Eq. 15: v' = sum over the t picked tokens of C_j v_j, all 1024 threads of a
// unit's block.  A wave takes sixteen picks at a time, a lane the channels c and
// c + 64 of every one of them: the sixteen index loads, then the sixteen score
// and value loads behind them, are in flight together, and a block's sixteen
// waves cover 256 picks per round -- the usual t in one.  Picks are added in
// index order inside a wave and the waves' partial vectors in wave order: the
// same sum every time.  idx: the unit's picks (-1 = none); red: LDS.
template <typename T>
__device__ __forceinline__ void semvec_of_unit(const double *__restrict__ sc, const T *__restrict__ vb,
                                               const int32_t *__restrict__ idx, double *__restrict__ sem_row,
                                               int n_picks, int D, double (&red)[16][128]) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  constexpr int U = 16;
  const bool second = D > 64;   // head sizes 64 and 128: one or two channels per lane
  double acc0 = 0.0, acc1 = 0.0;
  for (int n0 = wv * U; n0 < n_picks; n0 += 16 * U) {
    int j[U];
#pragma unroll
    for (int u = 0; u < U; ++u) j[u] = n0 + u < n_picks ? idx[n0 + u] : -1;
    // every load unconditional (a pick past the end reads token 0 with weight
    // zero) and converted only after all are requested: a load under a branch
    // is waited for where it stands, sixteen memory latencies one after the other
    double w[U];
    T r0[U], r1[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t row = (size_t)max(j[u], 0) * D;
      w[u] = sc[max(j[u], 0)];
      r0[u] = vb[row + lane];
      r1[u] = vb[row + (second ? 64 : 0) + lane];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool on = j[u] >= 0;
      const double wu = on ? w[u] : 0.0;
      acc0 += wu * (on ? elem_to_double(r0[u]) : 0.0);
      acc1 += wu * (on && second ? elem_to_double(r1[u]) : 0.0);
    }
  }
  red[wv][lane] = acc0;
  red[wv][64 + lane] = acc1;
  __syncthreads();
  if (threadIdx.x < D) {
    double sum = 0.0;
    for (int g = 0; g < 16; ++g) sum += red[g][threadIdx.x];
    sem_row[threadIdx.x] = sum;
  }
}

// One block per unit: the semantic vector from picks that are in memory.
template <typename T>
__global__ __launch_bounds__(1024) void semvec_kernel(const double *__restrict__ scores, const T *__restrict__ v,
                                                      const int32_t *__restrict__ top_idx,
                                                      double *__restrict__ sem, Dims dm) {
  const int unit = blockIdx.x;
  __shared__ double red[16][128];
  semvec_of_unit(scores + (size_t)unit * dm.N, v + (size_t)unit * dm.N * dm.D, top_idx + (size_t)unit * dm.T,
                 sem + (size_t)unit * dm.D, dm.T, dm.D, red);
}

// One block per unit: the top-t pick (Eq. 14; among all columns, or among the
// columns a list names) and the semantic vector of the picks behind it -- the
// two are a chain inside one unit, and as two kernels they paid two launches
// for it.  The picks go through memory (they are an output of their own); the
// barrier between the halves makes the block's writes visible to its readers.
template <typename T>
__global__ __launch_bounds__(1024) void topt_semvec_kernel(const double *__restrict__ scores,
                                                           const int32_t *__restrict__ listed,
                                                           const int32_t *__restrict__ n_listed,
                                                           const T *__restrict__ v, int32_t *__restrict__ top_idx,
                                                           double *__restrict__ sem, Dims dm) {
  const int unit = blockIdx.x;
  __shared__ RadixScratch rs;
  __shared__ int s_cnt[32];
  __shared__ double red[16][128];
  int32_t *picks = top_idx + (size_t)unit * dm.T;
  select_of_unit(scores + (size_t)unit * dm.N, picks, dm.N, 0, dm.N, dm.T, 0, 0, 0, dm.T,
                 listed ? listed + (size_t)unit * dm.N : nullptr, listed ? n_listed[unit] : 0, rs, s_cnt);
  __syncthreads();
  semvec_of_unit(scores + (size_t)unit * dm.N, v + (size_t)unit * dm.N * dm.D, picks, sem + (size_t)unit * dm.D,
                 dm.T, dm.D, red);
}

// Eq. 7-8 and the ranking rule: one block per batch element.
__global__ __launch_bounds__(1024) void dist_mask_kernel(const double *__restrict__ sem,
                                                        double *__restrict__ dist,
                                                        uint8_t *__restrict__ mask, Dims dm) {
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int H = dm.Hkv, D = dm.D;
  const double *sb = sem + (size_t)b * H * D;
  __shared__ double centre[128];
  __shared__ double part[8][128];
  __shared__ double sd[256];
  __shared__ uint8_t smask[256];
  // the centre: eight groups of threads take every eighth head each (their
  // loads are in flight together), the groups' sums are added in a fixed order
  {
    const int c = tid & 127, hg = tid >> 7;
    double acc = 0.0;
    if (c < D) {
#pragma unroll 4
      for (int h = hg; h < H; h += 8) acc += sb[(size_t)h * D + c];
    }
    part[hg][c] = acc;
  }
  __syncthreads();
  if (tid < D) {
    double acc = 0.0;
#pragma unroll
    for (int g = 0; g < 8; ++g) acc += part[g][tid];
    centre[tid] = acc / (double)H;
  }
  __syncthreads();
  for (int h = wv; h < H; h += 16) {
    double acc = 0.0;
    for (int c = lane; c < D; c += 64) {
      const double dl = sb[(size_t)h * D + c] - centre[c];
      acc += dl * dl;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
    if (lane == 0) sd[h] = sqrt(acc);
  }
  __syncthreads();
  if (tid < H) {
    const double mine = sd[tid];
    int rank = 0;
    for (int o = 0; o < H; ++o) {
      const double other = sd[o];
      rank += (other > mine) || (other == mine && o < tid);
    }
    smask[tid] = rank < dm.n_het ? 1 : 0;
  }
  __syncthreads();
  // the unmarked head nearest to the centre (lowest index among equals):
  // every unmarked head counts the unmarked ones that come before it
  bool nearest = false;
  if (dm.add_centre && tid < H) {
    const double mine = sd[tid];
    int before = 0;
    for (int o = 0; o < H; ++o) {
      const double other = sd[o];
      before += !smask[o] && ((other < mine) || (other == mine && o < tid));
    }
    nearest = !smask[tid] && before == 0;
  }
  __syncthreads();
  if (nearest) smask[tid] = 1;
  __syncthreads();
  if (tid < H) {
    dist[(size_t)b * H + tid] = sd[tid];
    mask[(size_t)b * H + tid] = smask[tid];
  }
}

int launch_select(const Dims &dm, const double *scores, const uint8_t *skip_mask, int lo, int hi,
                  int count, int prefix, int gap, int suffix, int32_t *out, int out_stride, int skip_all,
                  hipStream_t s) {
  select_kernel<<<dim3(dm.units), dim3(1024), 0, s>>>(scores, skip_mask, skip_all, dm.N, lo, hi, count, prefix, gap,
                                                     suffix, out, out_stride);
  return hip_ok(hipGetLastError());
}

int launch_pool(const Dims &dm, const double *scores, double *pooled, hipStream_t s) {
  pool_kernel<<<dim3((dm.N + POOL_SPAN - 1) / POOL_SPAN, dm.units), dim3(256), 0, s>>>(scores, pooled, dm.N, dm.pool);
  return hip_ok(hipGetLastError());
}

int launch_topt_semvec_mask(const Dims &dm, int dtype, const double *scores, const int32_t *listed,
                            const int32_t *n_listed, const void *v, int32_t *top_idx, double *sem_vec, double *dist,
                            uint8_t *mask, hipStream_t s) {
  if (dtype == TASKKV_F32)
    topt_semvec_kernel<float><<<dim3(dm.units), dim3(1024), 0, s>>>(scores, listed, n_listed,
                                                                  static_cast<const float *>(v), top_idx, sem_vec, dm);
  else
    topt_semvec_kernel<uint16_t><<<dim3(dm.units), dim3(1024), 0, s>>>(
        scores, listed, n_listed, static_cast<const uint16_t *>(v), top_idx, sem_vec, dm);
  dist_mask_kernel<<<dim3(dm.B), dim3(1024), 0, s>>>(sem_vec, dist, mask, dm);
  return hip_ok(hipGetLastError());
}

int launch_semvec_mask(const Dims &dm, int dtype, const double *scores, const void *v,
                       const int32_t *top_idx, double *sem_vec, double *dist, uint8_t *mask,
                       hipStream_t s) {
  if (dtype == TASKKV_F32)
    semvec_kernel<float><<<dim3(dm.units), dim3(1024), 0, s>>>(scores, static_cast<const float *>(v),
                                                             top_idx, sem_vec, dm);
  else
    semvec_kernel<uint16_t><<<dim3(dm.units), dim3(1024), 0, s>>>(
        scores, static_cast<const uint16_t *>(v), top_idx, sem_vec, dm);
  dist_mask_kernel<<<dim3(dm.B), dim3(1024), 0, s>>>(sem_vec, dist, mask, dm);
  return hip_ok(hipGetLastError());
}

}  // namespace taskkv
