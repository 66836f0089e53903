// Internal declarations shared by the HIP sources of libtaskkv (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "taskkv.h"

namespace taskkv {

constexpr int CHUNK = TASKKV_CHUNK_TOKENS;  // tokens per split-K work item / region alignment
constexpr int PAGE = 32;                    // tokens per matrix-core page of the bf16 cache
constexpr int MAX_PROFILE_EVENTS = 2048;  // event pairs in flight; a full record is summed up and reused
constexpr int STREAM_MAX_UNITS = 4096;  // units the streaming decode kernel can index in LDS
constexpr int STREAM_MAX_WG = 1024;     // workgroups (4 waves each) it is ever launched with
constexpr int STACK_REBASE_LAYERS = 64;  // layers one launch of the offset rebasing kernel covers
constexpr int STREAM_SKEW_DEFAULT = 56; // share moved from odd to even workgroups, in 1/1024ths (measured)

// Resolved problem sizes handed to kernels by value.
struct Dims {
  int B, Hq, Hkv, G, D, N, L, T;  // T = min(top_t, N)
  int s1, s2, k;                  // k already clipped to the middle
  int n_het, add_centre, pool;
  int pack_mode;                  // taskkv_pack_mode
  int Rtot;                       // window rows per unit, G*L
  int R, Rpad;                    // rows of the group being scored, and padded to 32
  int row0, n_keys, accumulate;   // first row of the group, keys it can see, add to C instead of storing
  int units;                      // B * Hkv
  int keep_all;                   // s1 + s2 >= N: every unit keeps everything
  int row_stride;                 // s1 + cfg.n_middle + s2: width of a kept_idx row
  double scale;                   // softmax scale
};

}  // namespace taskkv

struct taskkv_ctx {
  int device;
  char *ws;
  size_t ws_bytes;
  int *d_err;  // sticky device flag
  int profiling;
  int n_events;          // event pairs attached to launches and not yet summed up
  hipEvent_t ev_start[taskkv::MAX_PROFILE_EVENTS];
  hipEvent_t ev_stop[taskkv::MAX_PROFILE_EVENTS];
  int events_created;    // pairs that exist (all of them once profiling has been switched on)
  double prof_ms;        // durations summed up so far
  int64_t prof_launches; // launches they belong to
  int n_cu;           // compute units of the device
  int stream_skew;    // 1/1024ths of an equal share moved from the waves of odd workgroups to even ones
  int stats_engine;   // row statistics of bf16 inputs: 0 = fp64 matrix instruction, 1 = int8 digits
  int screening;      // fp32 screening + fp64 recompute of contested columns: 0 off, 1 auto, 2 always
  int stream_wg[4];   // cached launch width of the streaming decode kernel per (D, NT) variant, 0 = unknown
  // what the last taskkv_separate screened its scores for: off the listed
  // columns they are fp32 values, good only for this selection
  const double *screened_scores;
  int screened_list;     // the band lists of that call are still in the workspace, with per-slice counts
  unsigned long long screened_capture;   // id of the stream capture that call was recorded in, 0 = it ran at once
  int screened_sel[8];   // ctx_len, n_sink, n_recent, n_middle, pack_mode, pool_kernel, batch, n_kv_heads
};

namespace taskkv {

// Bump allocator over the ctx workspace (256-byte aligned pieces).
struct Carver {
  char *base;
  size_t cap, used;
  bool ok;
  Carver(char *b, size_t c) : base(b), cap(c), used(0), ok(true) {}
  template <typename T>
  T *take(size_t n) {
    size_t bytes = (n * sizeof(T) + 255) & ~size_t(255);
    if (used + bytes > cap) {
      ok = false;
      return nullptr;
    }
    T *p = reinterpret_cast<T *>(base + used);
    used += bytes;
    return p;
  }
};

// Unit that owns token slot `tok` of the ragged cache: the largest u with
// offsets[u] <= tok, or -1 if tok is past the last region.
__device__ __forceinline__ int find_unit(const int64_t *__restrict__ offsets, int n_units, int64_t tok) {
  if (tok >= offsets[n_units]) return -1;
  int lo = 0, hi = n_units - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (offsets[mid] <= tok) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// Words a kernel at the head of a sequence sets to zero for the kernels behind
// it (counters, histograms), which saves them a launch of their own.
struct ZeroList {
  uint32_t *p[6];
  size_t n[6];   // 32-bit words
  int count;
  ZeroList() : count(0) {}
  // at most five pieces are ever listed; a sixth would be refused rather than written past the arrays
  bool add(void *ptr, size_t words) {
    if (count >= 6) return false;
    p[count] = static_cast<uint32_t *>(ptr);
    n[count++] = words;
    return true;
  }
};

// ---- launchers (each validates nothing; api.hip has checked the arguments) ----
int score_parts(const Dims &dm);
int score_rows_padded(const Dims &dm);
// Buffers of the fp32 screening pass (see score_screen.hip).
struct ScreenBufs {
  int32_t *band_idx;           // [units][N] columns to recompute in fp64
  int32_t *band_cnt;           // [units]
  unsigned long long *knorm;   // [units] max squared key norm (bit pattern of a double)
  int mode;                    // 1 = when it pays, 2 = whenever the inputs allow
  int n_cu;                    // compute units of the device
  const struct MSelBufs *msel; // buffers of the sliced band kernels, or null
  // what the sliced band kernels leave for the middle pick of the compressor:
  int *above_band;             // [units][MSEL_MAX_SLICES] middle columns of a slice above the band
  int *list_ok;                // [units] 1 = the unit's list and counts come from the sliced kernels
  double *pooled;              // [units][N] pooled fp32 scores when the middle pick pools (else null)
};
// Buffers of the int8 row-statistics pass (see score_i8.hip).
constexpr int I8_QCAP = 4096;   // listed window-row remainders per unit
struct QTiny {
  int32_t row, c;   // window row and channel of an element that does not fit its row's window
  double r;         // its remainder
};
struct I8Bufs {
  void *qdig;       // [units][Rpad/16][D/64][4][64] 16-byte digit vectors of the window rows
  double *gq;       // [units][Rpad] row factors
  QTiny *qtiny;     // [units][I8_QCAP]
  int32_t *qcnt;    // [units]
  taskkv_ctx *prof; // ctx whose profiling hook may time the statistics kernel (or null)
};
bool i8_stats_supported(const Dims &dm, int dtype);
// qcnt_zeroed: bufs.qcnt has been set to zero by an earlier kernel on the stream
// n_parts: partial records per row the kernel leaves in `part` (n_wg or twice that)
int launch_i8_stats(const Dims &dm, const void *q_win, const void *k, const double *qd, const I8Bufs &bufs,
                    double *part, unsigned long long *knorm, int n_wg, int keys_per_wg, bool qcnt_zeroed,
                    int *n_parts, hipStream_t s);
// row statistics of a window of at most 32 rows from the digits in bufs (launch_i8_stats calls it)
int launch_i8_direct(const Dims &dm, const void *k, const double *qd, const I8Bufs &bufs, double *part,
                     unsigned long long *knorm, int max_parts, int *n_parts, hipStream_t s);
// exact scores of the listed columns from the digits launch_i8_stats left in bufs
int launch_i8_columns(const Dims &dm, const void *k, const double *qd, const I8Bufs &bufs, const double *stats,
                      const int32_t *band_idx, const int32_t *band_cnt, double *scores, int blocks_per_unit,
                      hipStream_t s);
int launch_zero_u64(unsigned long long *p, int n, hipStream_t s);
bool screen_supported(const Dims &dm, int dtype);
int launch_key_norms(const Dims &dm, const void *k, unsigned long long *knorm, hipStream_t s);
int launch_screen(const Dims &dm, const void *q_win, const void *k, const double *stats, double *scores,
                  int chunks_per_wg, int n_cu, hipStream_t s);
// Buffers of the selections whose sweeps are cut into slices (see select_multi.hip).
constexpr int MSEL_MAX_SLICES = 32;    // blocks that share a unit
constexpr int MSEL_MAX_UNITS = 256;    // beyond this one block per unit fills the chip anyway
constexpr int MSEL_MIN_RANGE = 12288;  // shorter ranges do not pay for the extra launches
constexpr int MSEL_CAND = 4096;        // entries of the wanted bin a unit's candidate list takes
struct MSelBufs {
  unsigned *hist;                // [2 levels][2][units][4096] digit histograms
  unsigned long long *cand_key;  // [2][units][MSEL_CAND] bit patterns in the wanted bin
  int32_t *cand_idx;             // [2][units][MSEL_CAND] and their positions
  int *n_cand, *take;            // [2][units] their number, rank of the wanted entry among them
  unsigned long long *wpat;      // [2][units] the digits they share
  int *wshift;                   // [2][units] position of the first digit they may differ in
  int *flag;                     // [units] 1 = redo this unit with one block
  int *n_above;                  // [units][MSEL_MAX_SLICES] entries of a slice in bins above the wanted one
  unsigned long long *pat;       // [units] threshold pattern
  int *take_final;               // [units] entries equal to it that are taken
  int *counts;                   // [units][MSEL_MAX_SLICES][2] picks of every slice: above / at the threshold
  double *band;                  // [3][units] band: brackets of the two thresholds, largest squared window-row norm
  int bracket;                   // 1 = the thresholds are wanted to their second digit only (the band's)
  int S, nsel;                   // slices per unit, thresholds wanted (1 or 2)
  int lo[2], hi[2], count[2];    // range and rank of each
};
size_t msel_workspace_bytes(const Dims &dm);
// false when the workspace was not sized for the sliced kernels
bool msel_carve(Carver &cv, const Dims &dm, MSelBufs &mb);
bool msel_pays(const Dims &dm, int n_cu, int lo, int hi, int count);
int launch_select_sliced(const Dims &dm, int n_cu, MSelBufs mb, const double *scores, const uint8_t *skip_mask, int lo,
                         int hi, int count, int prefix, int gap, int suffix, int32_t *out, int out_stride,
                         hipStream_t s);
// cleared: the words of msel_zero_words have been set to zero by an earlier kernel on the stream
// pooled: the pooled scores the middle pick ranks by when it pools (width dm.pool), else null
int launch_band_sliced(const Dims &dm, int n_cu, MSelBufs mb, const double *scores, const double *pooled,
                       const double *qd, const unsigned long long *knorm, int32_t *band_idx, int32_t *band_cnt, int *above_band,
                       int *list_ok, bool cleared, hipStream_t s);
void msel_zero_words(const Dims &dm, const MSelBufs &mb, ZeroList &z);
// The middle pick on screened scores whose band lists are still there: the
// threshold is one of the listed columns, so no sweep is needed to find it.
int launch_select_from_band(const Dims &dm, int n_cu, MSelBufs mb, const double *scores, const uint8_t *skip_mask,
                            const int32_t *band_idx, const int32_t *band_cnt, const int *above_band,
                            const int *list_ok, int32_t *out, hipStream_t s);
int launch_band(const Dims &dm, const double *scores, const double *qd, const unsigned long long *knorm,
                int32_t *band_idx, int32_t *band_cnt, hipStream_t s);
bool band_is_sliced(const Dims &dm, const struct ScreenBufs *scr);
bool scores_screened(const Dims &dm, int dtype, const ScreenBufs *scr);
int launch_scores(const Dims &dm, int dtype, const void *q_win, const void *k, double *qd, double *part,
                  double *stats, double *scores, const ScreenBufs *scr, const I8Bufs *i8, hipStream_t s);
int launch_select(const Dims &dm, const double *scores, const uint8_t *skip_mask, int lo, int hi,
                  int count, int prefix, int gap, int suffix, int32_t *out, int out_stride, int skip_all,
                  hipStream_t s);
int launch_pool(const Dims &dm, const double *scores, double *pooled, hipStream_t s);
// top-t pick (among the columns an ascending per-unit list names -- [units][N] entries, n_listed[unit] used -- or
// among all when listed is null), semantic vectors, distances, mask
int launch_topt_semvec_mask(const Dims &dm, int dtype, const double *scores, const int32_t *listed,
                            const int32_t *n_listed, const void *v, int32_t *top_idx, double *sem_vec, double *dist,
                            uint8_t *mask, hipStream_t s);
int launch_semvec_mask(const Dims &dm, int dtype, const double *scores, const void *v,
                       const int32_t *top_idx, double *sem_vec, double *dist, uint8_t *mask,
                       hipStream_t s);
int launch_layout(const Dims &dm, const uint8_t *mask, int reserve, int64_t capacity, int64_t *offsets,
                  int32_t *lens, int *d_err, hipStream_t s);
int launch_stack_rebase(const int64_t *layer_offsets, const int64_t *layer_capacity, int n_layers, int units,
                        int64_t *stacked, hipStream_t s);
int launch_pack(const Dims &dm, int dtype, const void *k, const void *v, const int32_t *kept_idx,
                const uint8_t *mask, const int64_t *offsets, const int32_t *lens, const void *comp_k,
                const void *comp_v, void *k_cache, void *v_cache, int64_t capacity, hipStream_t s);
int launch_group_means(const Dims &dm, int dtype, const void *k, const void *v, const uint8_t *mask,
                       void *comp_k, void *comp_v, int32_t *kept_idx, hipStream_t s);
int launch_export(const Dims &dm, int dtype, const void *k_cache, const void *v_cache,
                  const int64_t *offsets, void *k_rows, void *v_rows, int64_t capacity, hipStream_t s);
int launch_append(const Dims &dm, int dtype, const void *k_new, const void *v_new, void *k_cache,
                  void *v_cache, const int64_t *offsets, int32_t *lens, int *d_err, hipStream_t s);
int launch_decode(taskkv_ctx *ctx, const Dims &dm, int dtype, const void *q, const void *k_new,
                  const void *v_new, void *k_cache, void *v_cache, int64_t capacity,
                  const int64_t *offsets, int32_t *lens, int32_t *eff_len, float *pm, float *pl,
                  float *po, float *out, hipStream_t s);

int launch_decode_stream(taskkv_ctx *ctx, const Dims &dm, const void *q, const void *k_new,
                         const void *v_new, void *k_cache, void *v_cache, int64_t capacity,
                         const int64_t *offsets, int32_t *lens, int32_t *eff_len, int32_t *page_prefix,
                         float *pm, float *pl, float *po, float *out, hipStream_t s);

inline int hip_ok(hipError_t e) { return e == hipSuccess ? TASKKV_OK : TASKKV_EHIP; }

// Adds the durations of the recorded event pairs to the running totals and frees
// the pairs for reuse (waits for the launches they are attached to).
int profile_harvest(taskkv_ctx *ctx);

// Launch of a kernel that the profiling hook can time (mode: 1 = the decode
// attention kernel, 2 = the row-statistics kernel of the separator).  When the
// ctx profiles this mode, two events are attached to the launch itself: they
// take the kernel's own begin and end times from its completion signal, so the
// recorded duration holds no dispatch latency and the stream gets no extra
// packets (events recorded before and after the launch read 2-3 us more than
// the kernel runs).  When every pair is in use the recorded ones are summed up
// first (this waits for their launches: profiling is for measurement passes,
// not for the timed ones).  Arguments are converted to the kernel's parameter
// types before they are packed.
template <typename... P, typename... A>
inline void launch_profiled(taskkv_ctx *ctx, int mode, void (*kernel)(P...), dim3 grid, dim3 block,
                            hipStream_t s, A... args) {
  const bool timed = ctx != nullptr && ctx->profiling == mode;
  if (timed && ctx->n_events >= ctx->events_created) (void)profile_harvest(ctx);
  if (timed && ctx->n_events < ctx->events_created) {
    hipExtLaunchKernelGGL(kernel, grid, block, 0, s, ctx->ev_start[ctx->n_events], ctx->ev_stop[ctx->n_events], 0,
                          static_cast<P>(args)...);
    ++ctx->n_events;
  } else {
    kernel<<<grid, block, 0, s>>>(static_cast<P>(args)...);
  }
}

}  // namespace taskkv
