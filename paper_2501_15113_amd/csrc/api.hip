// C ABI entry points of libtaskkv: argument validation, workspace carving and
// kernel sequencing.  No entry point here synchronises the device or allocates,
// except create / destroy / last_async_error / profile_read.
#include <math.h>
#include <mutex>
#include <new>

#include "taskkv_internal.h"

namespace taskkv {

// Makes `device` current for the lifetime of the object and puts the caller's
// device back afterwards.
struct DeviceGuard {
  int prev;
  bool ok;
  explicit DeviceGuard(int device) : prev(-1), ok(false) {
    if (hipGetDevice(&prev) != hipSuccess) prev = -1;
    ok = hipSetDevice(device) == hipSuccess;
  }
  ~DeviceGuard() {
    if (prev >= 0) (void)hipSetDevice(prev);
  }
};

static bool resolve(const taskkv_layer_cfg *c, Dims &d) {
  if (!c) return false;
  if (c->batch < 1 || c->n_kv_heads < 1 || c->n_kv_heads > 256 || c->n_q_heads < 1) return false;
  if (c->n_q_heads % c->n_kv_heads) return false;
  if (c->head_dim != 64 && c->head_dim != 128) return false;
  if (c->ctx_len < 1 || c->obs_window < 1 || c->obs_window > c->ctx_len) return false;
  if (c->top_t < 1 || c->n_sink < 0 || c->n_recent < 0 || c->n_middle < 0 || c->n_hetero < 0) return false;
  if (c->pool_kernel < 1 || c->pool_kernel % 2 == 0) return false;
  if (c->dtype != TASKKV_F32 && c->dtype != TASKKV_BF16) return false;
  if (c->pack_mode < TASKKV_PACK_SELECTIVE || c->pack_mode > TASKKV_PACK_COMPRESSED) return false;
  if (!(c->softmax_scale >= 0.f)) return false;
  d.B = c->batch; d.Hq = c->n_q_heads; d.Hkv = c->n_kv_heads; d.G = d.Hq / d.Hkv;
  d.D = c->head_dim; d.N = c->ctx_len; d.L = c->obs_window;
  d.T = c->top_t < d.N ? c->top_t : d.N;
  d.s1 = c->n_sink; d.s2 = c->n_recent;
  d.pack_mode = c->pack_mode;
  if (d.pack_mode == TASKKV_PACK_NO_CACHE) {
    // the middle budget is spent on a longer recent window
    const int64_t recent = (int64_t)c->n_recent + c->n_middle;
    d.keep_all = ((int64_t)d.s1 + recent >= d.N) ? 1 : 0;
    d.s2 = d.keep_all ? c->n_recent : (int)recent;
    d.k = 0;
  } else {
    d.keep_all = ((int64_t)d.s1 + d.s2 >= d.N) ? 1 : 0;
    const int64_t middle = d.keep_all ? 0 : (int64_t)d.N - d.s1 - d.s2;
    d.k = (int)(c->n_middle < middle ? c->n_middle : middle);
  }
  d.n_het = c->n_hetero; d.add_centre = c->add_centre_head ? 1 : 0; d.pool = c->pool_kernel;
  if (d.G > 64 || (int64_t)d.G * d.L > (int64_t)1 << 30) return false;
  d.Rtot = d.G * d.L;
  d.R = d.Rtot;
  d.Rpad = score_rows_padded(d);
  d.row0 = 0; d.n_keys = d.N; d.accumulate = 0;
  if ((int64_t)d.B * d.Hkv > 65535) return false;
  d.units = d.B * d.Hkv;
  const int64_t stride = (int64_t)c->n_sink + c->n_middle + c->n_recent;
  if (stride > (int64_t)1 << 30) return false;
  d.row_stride = (int)stride;
  d.scale = c->softmax_scale > 0.f ? (double)c->softmax_scale : 1.0 / sqrt((double)d.D);
  return true;
}

static int64_t cache_tokens(const Dims &d, int reserve) {
  int n_long = d.n_het < d.Hkv ? d.n_het : d.Hkv;
  if (d.add_centre && n_long < d.Hkv) n_long += 1;
  if (d.keep_all) n_long = d.Hkv;
  auto cap = [&](int64_t len) {
    const int64_t c = (len + reserve + CHUNK - 1) / CHUNK * CHUNK;
    return c < CHUNK ? (int64_t)CHUNK : c;  // every unit owns at least one chunk
  };
  const int64_t short_len = (int64_t)d.s1 + d.k + d.s2;
  return (int64_t)d.B * (n_long * cap(d.N) + (int64_t)(d.Hkv - n_long) * cap(short_len));
}

static size_t al(size_t b) { return (b + 255) & ~size_t(255); }

// What the screening pass of the separator leaves for the compressor; both
// carve it first, so it sits at the start of the workspace.
static size_t ws_screen_state(const Dims &d) {
  return al((size_t)d.units * d.N * sizeof(int32_t)) +                 // columns to recompute
         al((size_t)d.units * 2 * sizeof(int32_t)) +                   // their count
         al((size_t)d.units * MSEL_MAX_SLICES * sizeof(int)) +         // middle columns above the band, per slice
         al((size_t)d.units * sizeof(int));                            // which units have those counts
}
static void carve_screen_state(Carver &cv, const Dims &d, ScreenBufs &scr) {
  scr.band_idx = cv.take<int32_t>((size_t)d.units * d.N);
  scr.band_cnt = cv.take<int32_t>((size_t)d.units * 2);
  scr.above_band = cv.take<int>((size_t)d.units * MSEL_MAX_SLICES);
  scr.list_ok = cv.take<int>((size_t)d.units);
  scr.pooled = nullptr;
}

// Id of the capture `s` is recording into, 0 when work on it runs at once.  What
// a call leaves in the workspace for the next one can only be relied on when
// both run at once or both are recorded into the same graph: a graph is
// replayed without the host-side bookkeeping of this file.
static unsigned long long capture_id(hipStream_t s) {
  hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
  unsigned long long id = 0;
  if (hipStreamGetCaptureInfo(s, &status, &id) != hipSuccess) {
    (void)hipGetLastError();
    return ~0ull;   // unknown: matches nothing
  }
  return status == hipStreamCaptureStatusActive ? id : 0ull;
}

static size_t ws_separate(const Dims &d) {
  const int n_chunks = score_parts(d);
  size_t b = ws_screen_state(d);
  b += al((size_t)d.units * d.Rpad * d.D * sizeof(double));           // window rows in fp64
  b += al((size_t)d.units * n_chunks * d.Rpad * 2 * sizeof(double));  // per-chunk row stats
  b += al((size_t)d.units * d.Rpad * 2 * sizeof(double));             // row stats
  b += al((size_t)d.units * d.T * sizeof(int32_t));                   // top-t picks
  b += al((size_t)d.units * sizeof(unsigned long long));              // key norms
  b += al((size_t)d.units * d.Rpad * d.D * 4);                        // int8 pass: digits of the window rows
  b += al((size_t)d.units * d.Rpad * sizeof(double));                 //   row factors
  b += al((size_t)d.units * I8_QCAP * sizeof(QTiny));                 //   remainders that do not fit
  b += al((size_t)d.units * sizeof(int32_t));                         //   their count
  b += msel_workspace_bytes(d);                                       // sliced selections
  if (d.pool > 1) b += al((size_t)d.units * d.N * sizeof(double));    // pooled scores of the screening pass
  return b;
}
static size_t ws_compress(const Dims &d, int dtype) {
  size_t b = ws_screen_state(d) + (d.pool > 1 ? al((size_t)d.units * d.N * sizeof(double)) : 0);
  if (d.pack_mode == TASKKV_PACK_COMPRESSED)
    b += 2 * al((size_t)d.units * d.k * d.D * (dtype == TASKKV_F32 ? 4 : 2));
  b += msel_workspace_bytes(d);
  return b;
}
// Partial slots a decode call needs: one per chunk for the chunk-grid kernels,
// one per (wave, unit) staircase step for the streaming kernel.
static size_t decode_slots(const Dims &d, int64_t capacity) {
  const size_t chunk_slots = (size_t)(capacity / CHUNK);
  const size_t stream_slots = (size_t)STREAM_MAX_WG * 4 + d.units;
  return chunk_slots > stream_slots ? chunk_slots : stream_slots;
}
static size_t stream_table_ints(const Dims &d) {
  return (size_t)d.units + 1 + STREAM_MAX_WG * 4 + 1 + 2 * (size_t)d.units;
}
static size_t ws_decode(const Dims &d, int64_t capacity) {
  const size_t n = decode_slots(d, capacity);
  return 2 * al(n * d.G * sizeof(float)) + al(n * d.G * d.D * sizeof(float)) +
         al(((size_t)d.units + 1) * sizeof(int32_t)) +
         al(stream_table_ints(d) * sizeof(int32_t));   // page prefix, wave range starts, first/last wave of each unit
}

static int decode_step(taskkv_ctx *ctx, const taskkv_layer_cfg *cfg, const void *q, const void *k_new,
                       const void *v_new, void *k_cache, void *v_cache, int64_t capacity_tokens,
                       const int64_t *offsets, int32_t *lens, float *out, void *hip_stream) {
  Dims d;
  if (!ctx || !resolve(cfg, d)) return TASKKV_EINVAL;
  if (!q || !k_cache || !v_cache || !offsets || !lens || !out) return TASKKV_EINVAL;
  if ((k_new == nullptr) != (v_new == nullptr)) return TASKKV_EINVAL;
  if (capacity_tokens <= 0 || capacity_tokens % CHUNK) return TASKKV_EINVAL;
  if (capacity_tokens / CHUNK > 0x7fffffff) return TASKKV_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (capacity_tokens / PAGE > 0x7fffffff) return TASKKV_EINVAL;
  const size_t n_slots = decode_slots(d, capacity_tokens);
  Carver cv(ctx->ws, ctx->ws_bytes);
  ctx->screened_list = 0;   // the workspace is reused
  float *pm = cv.take<float>(n_slots * d.G);
  float *pl = cv.take<float>(n_slots * d.G);
  float *po = cv.take<float>(n_slots * d.G * d.D);
  int32_t *eff_len = cv.take<int32_t>((size_t)d.units + 1);
  int32_t *page_prefix = cv.take<int32_t>(stream_table_ints(d));
  if (!cv.ok) return TASKKV_EWORKSPACE;
  if (cfg->dtype == TASKKV_BF16 && d.units <= STREAM_MAX_UNITS)
    return launch_decode_stream(ctx, d, q, k_new, v_new, k_cache, v_cache, capacity_tokens, offsets, lens,
                                eff_len, page_prefix, pm, pl, po, out, s);
  return launch_decode(ctx, d, cfg->dtype, q, k_new, v_new, k_cache, v_cache, capacity_tokens, offsets,
                       lens, eff_len, pm, pl, po, out, s);
}


// ---- state of the entry point that allocates nothing (taskkv_decode_attn_static)
// Its kernels' scratch -- partial results, per-step tables, the sticky flag --
// lives in a device array of fixed size that every GPU the library runs on
// holds from module load to process end.
constexpr size_t STATIC_SCRATCH_BYTES = TASKKV_STATIC_SCRATCH_BYTES;
constexpr size_t STATIC_FLAG_BYTES = 256;
constexpr int STATIC_MAX_DEVICES = 64;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
struct StaticState {
  bool ready;
  int *own_flag;     // flag word inside the device's scratch array
  taskkv_ctx ctx;    // a context whose workspace is the device's scratch array
};
static StaticState g_static[STATIC_MAX_DEVICES];
static std::mutex g_static_mutex;

int profile_harvest(taskkv_ctx *ctx) {
  for (int i = 0; i < ctx->n_events; ++i) {
    if (hipEventSynchronize(ctx->ev_stop[i]) != hipSuccess) return TASKKV_EHIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, ctx->ev_start[i], ctx->ev_stop[i]) != hipSuccess) return TASKKV_EHIP;
    ctx->prof_ms += ms;
  }
  ctx->prof_launches += ctx->n_events;
  ctx->n_events = 0;
  return TASKKV_OK;
}

}  // namespace taskkv

using namespace taskkv;

extern "C" {

const char *taskkv_strerror(int status) {
  switch (status) {
    case TASKKV_OK: return "ok";
    case TASKKV_EINVAL: return "invalid argument";
    case TASKKV_ECAPACITY: return "cache buffer too small";
    case TASKKV_EWORKSPACE: return "workspace too small";
    case TASKKV_EHIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

int taskkv_create(taskkv_ctx **out, int device_id, size_t workspace_bytes) {
  if (!out) return TASKKV_EINVAL;
  *out = nullptr;
  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess || device_id < 0 || device_id >= n_dev) return TASKKV_EHIP;
  DeviceGuard guard(device_id);   // the caller's current device is put back on return
  if (!guard.ok) return TASKKV_EHIP;
  taskkv_ctx *c = new (std::nothrow) taskkv_ctx();
  if (!c) return TASKKV_EHIP;
  c->device = device_id;
  c->ws = nullptr;
  c->ws_bytes = workspace_bytes;
  c->d_err = nullptr;
  c->profiling = 0;
  c->n_events = 0;
  c->events_created = 0;
  c->prof_ms = 0.0;
  c->prof_launches = 0;
  c->n_cu = 0;
  c->screening = 1;
  c->stats_engine = 1;
  c->stream_skew = STREAM_SKEW_DEFAULT;
  for (int i = 0; i < 4; ++i) c->stream_wg[i] = 0;
  c->screened_scores = nullptr;
  c->screened_list = 0;
  c->screened_capture = 0;
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, device_id) != hipSuccess) {
    delete c;
    return TASKKV_EHIP;
  }
  c->n_cu = prop.multiProcessorCount;
  if (workspace_bytes && hipMalloc((void **)&c->ws, workspace_bytes) != hipSuccess) {
    delete c;
    return TASKKV_EHIP;
  }
  if (hipMalloc((void **)&c->d_err, 256) != hipSuccess || hipMemset(c->d_err, 0, 256) != hipSuccess) {
    if (c->ws) (void)hipFree(c->ws);
    delete c;
    return TASKKV_EHIP;
  }
  *out = c;
  return TASKKV_OK;
}

void taskkv_destroy(taskkv_ctx *ctx) {
  if (!ctx) return;
  DeviceGuard guard(ctx->device);
  (void)hipDeviceSynchronize();
  for (int i = 0; i < ctx->events_created; ++i) {
    (void)hipEventDestroy(ctx->ev_start[i]);
    (void)hipEventDestroy(ctx->ev_stop[i]);
  }
  if (ctx->ws) (void)hipFree(ctx->ws);
  if (ctx->d_err) (void)hipFree(ctx->d_err);
  delete ctx;
}

size_t taskkv_workspace_bytes(const taskkv_layer_cfg *cfg, int32_t reserve_decode_tokens) {
  Dims d;
  if (!resolve(cfg, d) || reserve_decode_tokens < 0) return 0;
  size_t a = ws_separate(d), b = ws_compress(d, cfg->dtype), c = ws_decode(d, cache_tokens(d, reserve_decode_tokens));
  size_t m = a > b ? a : b;
  return (m > c ? m : c) + 4096;
}

int64_t taskkv_cache_tokens(const taskkv_layer_cfg *cfg, int32_t reserve_decode_tokens) {
  Dims d;
  if (!resolve(cfg, d) || reserve_decode_tokens < 0) return TASKKV_EINVAL;
  return cache_tokens(d, reserve_decode_tokens);
}

int32_t taskkv_hetero_head_count(int32_t n_heads, double beta, int32_t m_top, int32_t layer, int32_t n_layers) {
  double f = n_heads * beta;
  if (n_layers > 1) f -= (n_heads * beta - m_top) / (double)(n_layers - 1) * layer;
  double r = floor(f + 0.5);
  if (r < 0) r = 0;
  if (r > n_heads) r = n_heads;
  return (int32_t)r;
}

int32_t taskkv_middle_budget(int64_t layer_budget_tokens, int32_t ctx_len, int32_t n_heads,
                             int32_t n_hetero, int32_t n_sink, int32_t n_recent) {
  if (n_heads <= n_hetero) return 0;
  const int64_t num = layer_budget_tokens - (int64_t)ctx_len * n_hetero;
  const int64_t den = n_heads - n_hetero;
  int64_t q = num / den;
  if (num % den != 0 && num < 0) q -= 1;  // floor division
  q -= (int64_t)n_sink + n_recent;
  return (int32_t)(q < 0 ? 0 : q);
}

int taskkv_layer_plan(int32_t n_heads, double beta, int32_t m_top, int32_t n_layers, double budget_frac,
                      int32_t ctx_len, int32_t n_sink, int32_t n_recent, int32_t *n_hetero, int32_t *n_middle) {
  if (n_heads < 1 || n_layers < 1 || ctx_len < 1 || n_sink < 0 || n_recent < 0 || m_top < 0 || !n_hetero || !n_middle)
    return TASKKV_EINVAL;
  if (!(beta >= 0.0) || !(budget_frac >= 0.0) || !(budget_frac <= 1.0)) return TASKKV_EINVAL;
  const int64_t budget = (int64_t)floor(budget_frac * n_heads * ctx_len);
  for (int r = 0; r < n_layers; ++r) {
    n_hetero[r] = taskkv_hetero_head_count(n_heads, beta, m_top, r, n_layers);
    n_middle[r] = taskkv_middle_budget(budget, ctx_len, n_heads, n_hetero[r], n_sink, n_recent);
  }
  return TASKKV_OK;
}

int taskkv_separate(taskkv_ctx *ctx, const taskkv_layer_cfg *cfg, const void *q_win, const void *k,
                    const void *v, double *scores, double *sem_vec, double *dist,
                    uint8_t *hetero_mask, void *hip_stream) {
  Dims d;
  if (!ctx || !resolve(cfg, d)) return TASKKV_EINVAL;
  if (!q_win || !k || !v || !scores || !sem_vec || !dist || !hetero_mask) return TASKKV_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int n_parts = score_parts(d);
  Carver cv(ctx->ws, ctx->ws_bytes);
  ScreenBufs scr;
  carve_screen_state(cv, d, scr);
  double *qd = cv.take<double>((size_t)d.units * d.Rpad * d.D);
  double *part = cv.take<double>((size_t)d.units * n_parts * d.Rpad * 2);
  double *stats = cv.take<double>((size_t)d.units * d.Rpad * 2);
  int32_t *top_idx = cv.take<int32_t>((size_t)d.units * d.T);
  scr.knorm = cv.take<unsigned long long>((size_t)d.units);
  scr.mode = ctx->screening;
  scr.n_cu = ctx->n_cu;
  I8Bufs i8;
  i8.qdig = cv.take<char>((size_t)d.units * d.Rpad * d.D * 4);
  i8.gq = cv.take<double>((size_t)d.units * d.Rpad);
  i8.qtiny = cv.take<QTiny>((size_t)d.units * I8_QCAP);
  i8.qcnt = cv.take<int32_t>((size_t)d.units);
  i8.prof = ctx;
  MSelBufs mb;
  const bool sliced = msel_carve(cv, d, mb);
  scr.msel = sliced ? &mb : nullptr;
  scr.pooled = d.pool > 1 ? cv.take<double>((size_t)d.units * d.N) : nullptr;
  if (!cv.ok) return TASKKV_EWORKSPACE;
  ctx->screened_list = 0;
  if (scores_screened(d, cfg->dtype, &scr)) {
    ctx->screened_scores = scores;
    ctx->screened_list = band_is_sliced(d, &scr) ? 1 : 0;
    ctx->screened_capture = capture_id(s);
    const int sel[8] = {cfg->ctx_len, cfg->n_sink, cfg->n_recent, cfg->n_middle, cfg->pack_mode, cfg->pool_kernel,
                        cfg->batch, cfg->n_kv_heads};
    for (int i = 0; i < 8; ++i) ctx->screened_sel[i] = sel[i];
  } else if (ctx->screened_scores == scores) {
    ctx->screened_scores = nullptr;
  }
  int rc = launch_scores(d, cfg->dtype, q_win, k, qd, part, stats, scores, ctx->screening ? &scr : nullptr,
                         ctx->stats_engine ? &i8 : nullptr, s);
  if (rc) return rc;
  // Eq. 14.  After screening, the t best columns are among the listed ones (an
  // unlisted column is provably below the threshold): a few hundred candidates
  // instead of N.
  if (ctx->screening && scores_screened(d, cfg->dtype, &scr))
    return launch_topt_semvec_mask(d, cfg->dtype, scores, scr.band_idx, scr.band_cnt, v, top_idx, sem_vec, dist,
                                   hetero_mask, s);
  if (!(sliced && msel_pays(d, ctx->n_cu, 0, d.N, d.T)))
    return launch_topt_semvec_mask(d, cfg->dtype, scores, nullptr, nullptr, v, top_idx, sem_vec, dist, hetero_mask, s);
  rc = launch_select_sliced(d, ctx->n_cu, mb, scores, nullptr, 0, d.N, d.T, 0, 0, 0, top_idx, d.T, s);
  if (rc) return rc;
  return launch_semvec_mask(d, cfg->dtype, scores, v, top_idx, sem_vec, dist, hetero_mask, s);
}

int taskkv_compress(taskkv_ctx *ctx, const taskkv_layer_cfg *cfg, const void *k, const void *v,
                    const double *scores, const uint8_t *hetero_mask, void *k_cache, void *v_cache,
                    int64_t capacity_tokens, int32_t reserve_decode_tokens, int64_t *offsets,
                    int32_t *lens, int32_t *kept_idx, void *hip_stream) {
  Dims d;
  if (!ctx || !resolve(cfg, d) || reserve_decode_tokens < 0) return TASKKV_EINVAL;
  if (!k || !v || !scores || !hetero_mask || !k_cache || !v_cache || !offsets || !lens) return TASKKV_EINVAL;
  if (d.row_stride > 0 && !kept_idx) return TASKKV_EINVAL;
  if (capacity_tokens % CHUNK) return TASKKV_EINVAL;
  if (capacity_tokens < cache_tokens(d, reserve_decode_tokens)) return TASKKV_ECAPACITY;
  if (capacity_tokens / PAGE > 0x7fffffff) return TASKKV_EINVAL;
  if (scores == ctx->screened_scores) {
    // screened scores are exact only where the separator's own budget can decide
    const int sel[8] = {cfg->ctx_len, cfg->n_sink, cfg->n_recent, cfg->n_middle, cfg->pack_mode, cfg->pool_kernel,
                        cfg->batch, cfg->n_kv_heads};
    for (int i = 0; i < 8; ++i)
      if (sel[i] != ctx->screened_sel[i]) return TASKKV_EINVAL;
  }
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  Carver cv(ctx->ws, ctx->ws_bytes);
  ScreenBufs scr;
  carve_screen_state(cv, d, scr);   // still as the separator left it, if this call follows it
  const unsigned long long cap = capture_id(s);
  const bool from_band = scores == ctx->screened_scores && ctx->screened_list && cap != ~0ull &&
                         cap == ctx->screened_capture;
  ctx->screened_list = 0;           // the rest of the workspace is reused below
  const double *sel_scores = scores;
  int rc = TASKKV_OK;
  if (d.pool > 1 && d.pack_mode == TASKKV_PACK_SELECTIVE) {
    double *pooled = cv.take<double>((size_t)d.units * d.N);
    if (!cv.ok) return TASKKV_EWORKSPACE;
    rc = launch_pool(d, scores, pooled, s);
    if (rc) return rc;
    sel_scores = pooled;
  }
  void *comp_k = nullptr, *comp_v = nullptr;
  if (d.pack_mode == TASKKV_PACK_COMPRESSED && d.k > 0) {
    const size_t esz = cfg->dtype == TASKKV_F32 ? 4 : 2;
    comp_k = cv.take<char>((size_t)d.units * d.k * d.D * esz);
    comp_v = cv.take<char>((size_t)d.units * d.k * d.D * esz);
    if (!cv.ok) return TASKKV_EWORKSPACE;
  }
  if (d.row_stride > 0) {
    // selective: middle pick by score; the other modes take no middle token by
    // score (count 0) and get sinks + recent from the same kernel
    const int count = d.pack_mode == TASKKV_PACK_SELECTIVE ? d.k : 0;
    const int gap = d.pack_mode == TASKKV_PACK_COMPRESSED ? d.k : 0;  // filled with group positions below
    MSelBufs mb;
    const bool sliced = msel_carve(cv, d, mb);
    if (!cv.ok) return TASKKV_EWORKSPACE;
    if (sliced && from_band && !d.keep_all && count > 0 && count < d.N - d.s1 - d.s2)
      rc = launch_select_from_band(d, ctx->n_cu, mb, sel_scores, hetero_mask, scr.band_idx, scr.band_cnt,
                                   scr.above_band, scr.list_ok, kept_idx, s);
    else if (sliced && !d.keep_all && msel_pays(d, ctx->n_cu, d.s1, d.N - d.s2, count))
      rc = launch_select_sliced(d, ctx->n_cu, mb, sel_scores, hetero_mask, d.s1, d.N - d.s2, count, d.s1, gap, d.s2,
                                kept_idx, d.row_stride, s);
    else
      rc = launch_select(d, sel_scores, hetero_mask, d.s1, d.N - d.s2, count, d.s1, gap, d.s2, kept_idx,
                         d.row_stride, d.keep_all, s);
    if (rc) return rc;
  }
  if (comp_k) {
    rc = launch_group_means(d, cfg->dtype, k, v, hetero_mask, comp_k, comp_v, kept_idx, s);
    if (rc) return rc;
  }
  rc = launch_layout(d, hetero_mask, reserve_decode_tokens, capacity_tokens, offsets, lens, ctx->d_err, s);
  if (rc) return rc;
  return launch_pack(d, cfg->dtype, k, v, kept_idx, hetero_mask, offsets, lens, comp_k, comp_v, k_cache,
                     v_cache, capacity_tokens, s);
}

int taskkv_decode_attn(taskkv_ctx *ctx, const taskkv_layer_cfg *cfg, const void *q, const void *k_new,
                       const void *v_new, void *k_cache, void *v_cache, int64_t capacity_tokens,
                       const int64_t *offsets, int32_t *lens, float *out, void *hip_stream) {
  return decode_step(ctx, cfg, q, k_new, v_new, k_cache, v_cache, capacity_tokens, offsets, lens, out, hip_stream);
}

int taskkv_decode_attn_static(const taskkv_layer_cfg *cfg, const void *q, const void *k_new, const void *v_new,
                              void *k_cache, void *v_cache, int64_t capacity_tokens, const int64_t *offsets,
                              int32_t *lens, float *out, int32_t *async_flag, void *hip_stream) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= STATIC_MAX_DEVICES) return TASKKV_EHIP;
  // one call at a time builds and uses a device's state (calls that overlap on
  // one GPU would race on the scratch array anyway)
  std::lock_guard<std::mutex> lock(g_static_mutex);
  StaticState &st = g_static[dev];
  if (!st.ready) {
    // the array's name is a host-side stand-in: its device address on the
    // current GPU comes from the runtime, once per device
    unsigned char *ptr = nullptr;
    if (hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return TASKKV_EHIP;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return TASKKV_EHIP;
    taskkv_ctx &c = st.ctx;
    c.device = dev;
    c.ws = reinterpret_cast<char *>(ptr) + STATIC_FLAG_BYTES;
    c.ws_bytes = STATIC_SCRATCH_BYTES - STATIC_FLAG_BYTES;
    c.d_err = reinterpret_cast<int *>(ptr);   // zero when the module is loaded, like the whole array
    c.profiling = 0;
    c.n_events = c.events_created = 0;
    c.prof_ms = 0.0;
    c.prof_launches = 0;
    c.n_cu = prop.multiProcessorCount;
    c.screening = 1;
    c.stats_engine = 1;
    c.stream_skew = STREAM_SKEW_DEFAULT;
    for (int i = 0; i < 4; ++i) c.stream_wg[i] = 0;
    c.screened_scores = nullptr;
    c.screened_list = 0;
    c.screened_capture = 0;
    st.own_flag = c.d_err;
    st.ready = true;
  }
  st.ctx.d_err = async_flag ? reinterpret_cast<int *>(async_flag) : st.own_flag;
  return decode_step(&st.ctx, cfg, q, k_new, v_new, k_cache, v_cache, capacity_tokens, offsets, lens, out,
                     hip_stream);
}

int taskkv_stack_rebase(taskkv_ctx *ctx, int32_t n_layers, int32_t units_per_layer, const int64_t *layer_offsets,
                        const int64_t *layer_capacity_tokens, int64_t *stacked_offsets, void *hip_stream) {
  if (!ctx || n_layers < 1 || units_per_layer < 1 || !layer_offsets || !layer_capacity_tokens || !stacked_offsets)
    return TASKKV_EINVAL;
  if ((int64_t)n_layers * units_per_layer > 65535) return TASKKV_EINVAL;
  for (int r = 0; r < n_layers; ++r)
    if (layer_capacity_tokens[r] < 0 || layer_capacity_tokens[r] % CHUNK) return TASKKV_EINVAL;
  return launch_stack_rebase(layer_offsets, layer_capacity_tokens, n_layers, units_per_layer, stacked_offsets,
                             static_cast<hipStream_t>(hip_stream));
}

int taskkv_decode_attn_layers(taskkv_ctx *ctx, const taskkv_layer_cfg *cfg, int32_t n_layers, const void *q,
                              const void *k_new, const void *v_new, void *k_cache, void *v_cache,
                              int64_t capacity_tokens, const int64_t *offsets, int32_t *lens, float *out,
                              void *hip_stream) {
  if (!cfg || n_layers < 1 || (int64_t)cfg->batch * n_layers > 0x7fffffff) return TASKKV_EINVAL;
  taskkv_layer_cfg all = *cfg;
  all.batch = cfg->batch * n_layers;   // the step sees (layer, batch element) pairs as batch elements
  return taskkv_decode_attn(ctx, &all, q, k_new, v_new, k_cache, v_cache, capacity_tokens, offsets, lens, out,
                            hip_stream);
}

int taskkv_cache_export(taskkv_ctx *ctx, const taskkv_layer_cfg *cfg, const void *k_cache,
                        const void *v_cache, int64_t capacity_tokens, const int64_t *offsets,
                        void *k_rows, void *v_rows, void *hip_stream) {
  Dims d;
  if (!ctx || !resolve(cfg, d)) return TASKKV_EINVAL;
  if (!k_cache || !v_cache || !offsets || !k_rows || !v_rows) return TASKKV_EINVAL;
  if (capacity_tokens < 0 || capacity_tokens % CHUNK || capacity_tokens / PAGE > 0x7fffffff) return TASKKV_EINVAL;
  return launch_export(d, cfg->dtype, k_cache, v_cache, offsets, k_rows, v_rows, capacity_tokens,
                       static_cast<hipStream_t>(hip_stream));
}

int taskkv_last_async_error(taskkv_ctx *ctx, void *hip_stream) {
  if (!ctx) return TASKKV_EINVAL;
  DeviceGuard guard(ctx->device);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  int flag = 0;
  if (hipMemcpyAsync(&flag, ctx->d_err, sizeof(int), hipMemcpyDeviceToHost, s) != hipSuccess) return TASKKV_EHIP;
  if (hipStreamSynchronize(s) != hipSuccess) return TASKKV_EHIP;
  if (flag && hipMemsetAsync(ctx->d_err, 0, sizeof(int), s) != hipSuccess) return TASKKV_EHIP;
  return flag;
}

int taskkv_set_screening(taskkv_ctx *ctx, int mode) {
  if (!ctx || mode < 0 || mode > 2) return TASKKV_EINVAL;
  ctx->screening = mode;
  return TASKKV_OK;
}

int taskkv_set_stats_engine(taskkv_ctx *ctx, int engine) {
  if (!ctx || engine < 0 || engine > 1) return TASKKV_EINVAL;
  ctx->stats_engine = engine;
  return TASKKV_OK;
}

int taskkv_set_stream_skew(taskkv_ctx *ctx, int skew) {
  if (!ctx || skew < 0 || skew > 128) return TASKKV_EINVAL;
  ctx->stream_skew = skew;
  return TASKKV_OK;
}

int taskkv_profile_enable(taskkv_ctx *ctx, int on) {
  if (!ctx || on < 0 || on > 2) return TASKKV_EINVAL;
  if (on) {
    // the event pairs are made on first use; a failure leaves the pairs made so
    // far usable and no half-made pair behind
    while (ctx->events_created < MAX_PROFILE_EVENTS) {
      const int i = ctx->events_created;
      if (hipEventCreate(&ctx->ev_start[i]) != hipSuccess) break;
      if (hipEventCreate(&ctx->ev_stop[i]) != hipSuccess) {
        (void)hipEventDestroy(ctx->ev_start[i]);
        break;
      }
      ctx->events_created = i + 1;
    }
    if (ctx->events_created == 0) return TASKKV_EHIP;
  }
  ctx->profiling = on;
  return TASKKV_OK;
}

int taskkv_profile_read(taskkv_ctx *ctx, double *total_ms, int64_t *launches) {
  if (!ctx || !total_ms || !launches) return TASKKV_EINVAL;
  const int rc = profile_harvest(ctx);
  if (rc) return rc;
  *total_ms = ctx->prof_ms;
  *launches = ctx->prof_launches;
  ctx->prof_ms = 0.0;
  ctx->prof_launches = 0;
  return TASKKV_OK;
}

}  // extern "C"
