/*
 * taskkv.h -- C ABI of the Task-KV hot path on one AMD MI355X (gfx950).
 *
 * Task-KV (arXiv 2501.15113) compresses the KV cache of one transformer layer
 * at the end of prefill: a semantic separator (paper Sec. 4.1) marks the heads
 * far from the semantic centre as heterogeneous; those keep their full cache,
 * all other heads keep attention sinks, a recent window and the best-scored
 * middle tokens ("middle activations", paper Sec. 4.2).  Decoding then runs
 * attention over the resulting ragged, mixed-budget cache.
 *
 * Conventions for every entry point
 *   - Tensor arguments are DEVICE pointers owned by the caller, contiguous and
 *     row-major in the stated shape, 16-byte aligned.  Inputs are never
 *     written unless stated.  Scalars and the cfg struct are host values.
 *   - Work is enqueued on `hip_stream` (a hipStream_t, NULL = default stream);
 *     no entry point synchronises the device or allocates device memory,
 *     except taskkv_create / taskkv_destroy (both), taskkv_last_async_error and
 *     taskkv_profile_read (they wait for the stream / the recorded launches);
 *     taskkv_profile_enable creates HIP event objects on its first call.
 *   - Return value: TASKKV_OK or a negative taskkv_status.  Host-visible
 *     argument errors are reported before anything is enqueued.  Conditions
 *     only the device can see (appending to a full cache) set a sticky flag
 *     read by taskkv_last_async_error.
 *   - A "unit" is one (batch element, KV head) pair, unit = b * n_kv_heads + h.
 *   - One ctx serves one stream at a time; calls on one ctx must not overlap.
 */
#ifndef TASKKV_H
#define TASKKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Every unit's region of the ragged cache starts at a multiple of this many
 * tokens and is a multiple of it long; it is also the split-K granularity of
 * decode attention. */
#define TASKKV_CHUNK_TOKENS 512

typedef struct taskkv_ctx taskkv_ctx; /* opaque: workspace + error flag on one device */

typedef enum { TASKKV_F32 = 0, TASKKV_BF16 = 1 } taskkv_dtype;

/* How non-heterogeneous heads fill the part of their budget that lies between
 * sinks and recent window (the compensation methods compared in paper Sec. 6.2). */
typedef enum {
  TASKKV_PACK_SELECTIVE = 0,  /* the method: the n_middle best-scored middle tokens (Sec. 4.2) */
  TASKKV_PACK_NO_CACHE = 1,   /* nothing from the middle; the recent window grows by n_middle */
  TASKKV_PACK_COMPRESSED = 2  /* the middle is cut into n_middle contiguous groups of near-equal
                                 size, each replaced by the mean of its K rows and of its V rows */
} taskkv_pack_mode;

typedef enum {
  TASKKV_OK = 0,
  TASKKV_EINVAL = -1,     /* bad argument (shape, NULL pointer, unsupported size) */
  TASKKV_ECAPACITY = -2,  /* ragged cache buffer too small for this cfg */
  TASKKV_EWORKSPACE = -3, /* ctx workspace too small for this cfg */
  TASKKV_EHIP = -4        /* a HIP runtime call failed */
} taskkv_status;

/* One layer's problem statement (paper Sec. 4.1-4.2 notation in comments). */
typedef struct taskkv_layer_cfg {
  int32_t batch;           /* B */
  int32_t n_q_heads;       /* H_q; multiple of n_kv_heads, group G = H_q/H_kv <= 64 */
  int32_t n_kv_heads;      /* H_kv = n of the paper, <= 256 */
  int32_t head_dim;        /* d, 64 or 128 */
  int32_t ctx_len;         /* N, prompt length */
  int32_t obs_window;      /* L, observation window, 1 <= L <= N (paper: 32) */
  int32_t top_t;           /* t of Eq. 14 (paper: 256); clipped to N */
  int32_t n_sink;          /* s1 */
  int32_t n_recent;        /* s2 */
  int32_t n_middle;        /* k of Eq. 17; clipped to the size of the middle */
  int32_t n_hetero;        /* f(r): heads farthest from the centre that keep everything */
  int32_t add_centre_head; /* 1: the remaining head closest to the centre also keeps
                              everything (last rule of the ranking paragraph, Sec. 4.1) */
  int32_t pool_kernel;     /* odd width of the average pooling of selection scores
                              (paper Sec. 5.4 uses 7); 1 = none */
  int32_t pack_mode;       /* taskkv_pack_mode; 0 = the paper's method */
  int32_t dtype;           /* taskkv_dtype of Q/K/V and of the cache */
  float softmax_scale;     /* 0 => 1/sqrt(d) */
} taskkv_layer_cfg;

/*
 * Create a context on `device_id` with `workspace_bytes` of scratch (see
 * taskkv_workspace_bytes).  Allocates device memory; the only call that does
 * (the first taskkv_profile_enable creates HIP events, nothing else allocates). */
int taskkv_create(taskkv_ctx **out, int device_id, size_t workspace_bytes);
void taskkv_destroy(taskkv_ctx *ctx);
const char *taskkv_strerror(int status);

/* Host only.  Upper bound of the scratch any of the three hot-path calls needs
 * for this cfg with `reserve_decode_tokens` of append room per unit. */
size_t taskkv_workspace_bytes(const taskkv_layer_cfg *cfg, int32_t reserve_decode_tokens);

/* Host only.  Exact token capacity of the ragged cache this cfg produces: the
 * head counts are fixed by cfg (n_hetero is a count), so the size is known
 * without reading the mask back.  Each unit gets its kept tokens plus
 * `reserve_decode_tokens`, rounded up to TASKKV_CHUNK_TOKENS (at least one chunk).  Returns < 0 on
 * a bad cfg. */
int64_t taskkv_cache_tokens(const taskkv_layer_cfg *cfg, int32_t reserve_decode_tokens);

/* Host helpers for the budget arithmetic.
 * Eq. 16: heads marked heterogeneous in layer r of R: n*beta - (n*beta-m)/(R-1)*r,
 * rounded half up, clipped to [0, n].
 * Eq. 17: middle budget k = (B_layer - N*f)/(n-f) - s1 - s2, floored, clipped at 0. */
int32_t taskkv_hetero_head_count(int32_t n_heads, double beta, int32_t m_top, int32_t layer, int32_t n_layers);
int32_t taskkv_middle_budget(int64_t layer_budget_tokens, int32_t ctx_len, int32_t n_heads,
                             int32_t n_hetero, int32_t n_sink, int32_t n_recent);

/* Host only.  The plan of a stack of n_layers layers under one budget (Eq. 16 and
 * Eq. 17 together, the operating points "KV cache budget 40 % / 60 %" of
 * Sec. 5.4): every layer may hold B = floor(budget_frac * n_heads * ctx_len)
 * tokens; layer r marks n_hetero[r] = f(r) heads (Eq. 16 with beta, m_top) and
 * gives every other head n_middle[r] = k middle activations (Eq. 17 with B,
 * n_sink, n_recent).  n_heads is the number of heads that are ranked (the KV
 * heads).  n_hetero, n_middle: host arrays of n_layers entries.  The two
 * values go into the layers' taskkv_layer_cfg.  budget_frac in [0, 1]. */
int taskkv_layer_plan(int32_t n_heads, double beta, int32_t m_top, int32_t n_layers, double budget_frac,
                      int32_t ctx_len, int32_t n_sink, int32_t n_recent, int32_t *n_hetero, int32_t *n_middle);

/*
 * Semantic separator (paper Sec. 4.1, Eq. 12-15, Eq. 7-8, ranking paragraph).
 *   q_win   [B, H_q, L, d]  last L query rows of the prompt (dtype of cfg)
 *   k, v    [B, H_kv, N, d] key / value states (dtype of cfg)
 * out
 *   scores  [B, H_kv, N] f64  C of Eq. 13, averaged over the G*L window rows of
 *                             the KV head's query group.  fp64-exact for every
 *                             token that can take part in a decision (the top-t
 *                             tokens and all tokens whose score is next to the
 *                             top-t or middle-activation threshold); with bf16
 *                             inputs the remaining tokens carry an fp32 value
 *                             whose relative error is bounded by eps =
 *                             scale * 4 d 2^-24 * max|q_i| * max|k_j| + 2e-5 +
 *                             G L 1.2e-7 (about 1e-3 on the named workloads;
 *                             the tests check 5e-3) unless screening is
 *                             switched off (taskkv_set_screening).  Such scores
 *                             are good for the selections of this cfg only,
 *                             and taskkv_compress assumes that the array still
 *                             holds what this call wrote
 *   sem_vec [B, H_kv, d] f64  v' of Eq. 15 over the top-t tokens of Eq. 14
 *   dist    [B, H_kv]    f64  L2 distance of v' from the mean over heads (Eq. 7-8)
 *   hetero_mask [B, H_kv] u8  1 = heterogeneous (keeps its full cache)
 * Decisions (top-t membership, head ranking) are taken on the f64 values, ties
 * to the lower index.
 */
int taskkv_separate(taskkv_ctx *ctx, const taskkv_layer_cfg *cfg, const void *q_win, const void *k,
                    const void *v, double *scores, double *sem_vec, double *dist,
                    uint8_t *hetero_mask, void *hip_stream);

/*
 * KV cache allocation (paper Sec. 4.2): build the ragged cache.
 *   k, v        [B, H_kv, N, d]  as above
 *   scores      [B, H_kv, N] f64 from taskkv_separate
 *   hetero_mask [B, H_kv] u8
 * out
 *   k_cache, v_cache  capacity_tokens * d elements each (dtype of cfg), library
 *                     layout (bf16: tiled for the matrix cores; read it back
 *                     with taskkv_cache_export)
 *   offsets  [B*H_kv + 1] i64  first token slot of each unit, multiples of
 *                              TASKKV_CHUNK_TOKENS
 *   lens     [B*H_kv]     i32  tokens held per unit: N for heterogeneous units (and
 *                              when s1 + s2 >= N), else s1 + min(k, N-s1-s2) + s2
 *   kept_idx [B*H_kv, s1+k+s2] i32  original positions kept by each
 *                              non-heterogeneous unit, ascending, -1 padded;
 *                              rows of keep-everything units are all -1; in
 *                              TASKKV_PACK_COMPRESSED mode a compensation token is
 *                              listed by the first position of its group
 * capacity_tokens must be >= taskkv_cache_tokens(cfg, reserve_decode_tokens)
 * (else TASKKV_ECAPACITY).  cfg must name the same batch, n_kv_heads, ctx_len,
 * n_sink, n_recent, n_middle, pack_mode and pool_kernel as the taskkv_separate
 * call that produced `scores` whenever that call screened them (see
 * taskkv_set_screening): the fp32 values off the decision columns are good for
 * that selection only.  The library checks this for the scores buffer of the
 * ctx's last screening taskkv_separate and returns TASKKV_EINVAL on a mismatch;
 * switch screening off to compress one set of scores under several budgets, or
 * to edit them between the two calls (when no other call on the ctx came in
 * between, the middle pick reuses the column lists that call left in the
 * workspace and relies on `scores` being unchanged; under stream capture only
 * when both calls are recorded into the same graph, since a replay runs
 * without the library's host-side bookkeeping).
 * Middle tokens are the n_middle best of the pooled
 * scores inside [s1, N - s2), ties to the lower index; rows are copied
 * bit-for-bit; slots past a unit's length are zero-filled.  In
 * TASKKV_PACK_COMPRESSED mode group g of n covers middle offsets
 * [g*M/n, (g+1)*M/n) (M = N - s1 - s2, n = min(n_middle, M)); its token is the
 * fp64 mean of the group's rows rounded once (to nearest even) to the cache dtype.
 */
int taskkv_compress(taskkv_ctx *ctx, const taskkv_layer_cfg *cfg, const void *k, const void *v,
                    const double *scores, const uint8_t *hetero_mask, void *k_cache, void *v_cache,
                    int64_t capacity_tokens, int32_t reserve_decode_tokens, int64_t *offsets,
                    int32_t *lens, int32_t *kept_idx, void *hip_stream);

/*
 * One decode step of attention over the ragged cache (softmax attention of
 * Eq. 1 for a single new query row, restricted to each head's kept tokens;
 * the step the paper times in Sec. 5.5.3).
 *   q            [B, H_q, d]   query of the new token (dtype of cfg)
 *   k_new, v_new [B, H_kv, d]  its key / value, appended to EVERY unit before
 *                              attention (lens += 1); both NULL = no append
 *   k_cache, v_cache, offsets, lens  as produced by taskkv_compress
 *                              (cache and lens are updated by the append)
 * out
 *   out          [B, H_q, d] f32   softmax(scale * q K_c^T) V_c per query head;
 *                              the G query heads of a group share one read of K_c, V_c
 * A unit whose region is full cannot append: the token is dropped and the
 * sticky error flag is set.  The result is independent of launch order
 * (partials are merged in a fixed order).
 */
int taskkv_decode_attn(taskkv_ctx *ctx, const taskkv_layer_cfg *cfg, const void *q, const void *k_new,
                       const void *v_new, void *k_cache, void *v_cache, int64_t capacity_tokens,
                       const int64_t *offsets, int32_t *lens, float *out, void *hip_stream);

/*
 * taskkv_decode_attn for callers that cannot allocate and hold no context:
 * code whose stream is being captured into a HIP graph, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, results and append rule
 * as taskkv_decode_attn, without the ctx: the kernels' scratch memory is a
 * device array of TASKKV_STATIC_SCRATCH_BYTES that is part of the library's
 * code object (each GPU the library runs on holds it from module load until the
 * process ends).  The call allocates nothing and synchronises nothing; its
 * first call on a device looks up the array's address on that device and the
 * device's properties (make that call outside graph capture).
 *   async_flag  device pointer to an int32 that receives the sticky condition
 *               bits of taskkv_last_async_error (bit 1: append to a full unit),
 *               OR-ed in by the kernels; the caller clears and reads it.  NULL:
 *               the bits go to a word inside the scratch array and are lost.
 * Returns TASKKV_EWORKSPACE when the step needs more scratch than the array
 * holds (taskkv_workspace_bytes of a decode-only use: about
 * (4096 + B*H_kv) * G * (d + 2) * 4 bytes for bf16 caches), before anything is
 * enqueued.  The device that is current at the call is used.  All calls on one
 * GPU share that GPU's array, which keeps the previous call's contents: calls
 * that overlap in time on one GPU (two streams, two threads) race; calls on
 * one stream, or ordered by events, do not.
 */
#define TASKKV_STATIC_SCRATCH_BYTES (24u << 20)
int taskkv_decode_attn_static(const taskkv_layer_cfg *cfg, const void *q, const void *k_new, const void *v_new,
                              void *k_cache, void *v_cache, int64_t capacity_tokens, const int64_t *offsets,
                              int32_t *lens, float *out, int32_t *async_flag, void *hip_stream);

/*
 * A decode step of a whole stack of layers in one call (the step of Sec. 5.5.3
 * for every layer at once; it serves callers that have all layers' queries at
 * hand, e.g. a benchmark or speculative pipelines -- in an ordinary decoder
 * layer r+1's query depends on layer r's output).  The layers' ragged caches
 * lie one after the other in k_cache / v_cache: layer r was compressed into
 * the slice that starts at token sum(layer_capacity_tokens[0..r)), with its
 * own offsets / lens arrays.  All layers share B, H_q, H_kv, d, dtype and the
 * softmax scale (cfg: any layer's cfg; only these fields are read).
 *
 * taskkv_stack_rebase writes the offsets array of the stack:
 *   layer_offsets  [n_layers, units_per_layer + 1] i64 (device)  row r = the
 *                  offsets taskkv_compress wrote for layer r
 *   layer_capacity_tokens [n_layers] i64 (HOST)  capacity of each layer's slice
 *   stacked_offsets [n_layers * units_per_layer + 1] i64 (device, out)
 * n_layers * units_per_layer <= 65535.
 *
 * taskkv_decode_attn_layers is taskkv_decode_attn with (layer, batch element)
 * in place of the batch element:
 *   q [n_layers, B, H_q, d], k_new / v_new [n_layers, B, H_kv, d] or both NULL,
 *   lens [n_layers * B * H_kv] (the layers' lens arrays, contiguous, layer-major),
 *   offsets = stacked_offsets, capacity_tokens = the sum of the layers' capacities,
 *   out [n_layers, B, H_q, d] f32.
 */
int taskkv_stack_rebase(taskkv_ctx *ctx, int32_t n_layers, int32_t units_per_layer, const int64_t *layer_offsets,
                        const int64_t *layer_capacity_tokens, int64_t *stacked_offsets, void *hip_stream);
int taskkv_decode_attn_layers(taskkv_ctx *ctx, const taskkv_layer_cfg *cfg, int32_t n_layers, const void *q,
                              const void *k_new, const void *v_new, void *k_cache, void *v_cache,
                              int64_t capacity_tokens, const int64_t *offsets, int32_t *lens, float *out,
                              void *hip_stream);

/*
 * Inspection: copy the cache back to plain rows.  k_rows / v_rows are
 * [capacity_tokens, d] row-major (dtype of cfg); token p of unit u lands in row
 * offsets[u] + p.  Rows past a unit's length are written as stored (zeros).
 */
int taskkv_cache_export(taskkv_ctx *ctx, const taskkv_layer_cfg *cfg, const void *k_cache,
                        const void *v_cache, int64_t capacity_tokens, const int64_t *offsets,
                        void *k_rows, void *v_rows, void *hip_stream);

/* Synchronises `hip_stream`, returns and clears the sticky device-side flag (the
 * clearing store is enqueued on `hip_stream`).  Bits: 1 = a token was appended
 * to a full unit and dropped; 2 = taskkv_compress was given a hetero_mask that
 * marks more keep-everything heads than cfg's counts (n_hetero, plus one with
 * add_centre_head) leave room for in capacity_tokens: the units that did not
 * fit were left empty (length 0, no region), nothing was written out of bounds. */
int taskkv_last_async_error(taskkv_ctx *ctx, void *hip_stream);

/* Screening lets taskkv_separate score bf16 inputs on the bf16 matrix cores
 * first and recompute in fp64 only the columns that can matter; decisions are
 * identical either way.  mode 0: never (every score exact); 1 (default): when
 * the layer is large enough for it to pay; 2: whenever the inputs allow
 * (bf16, at most 512 window rows per KV head; with pool_kernel > 1 only
 * contexts of 12288 tokens and more, on at most 256 (batch, KV head) units). */
int taskkv_set_screening(taskkv_ctx *ctx, int mode);

/* Row maxima and softmax denominators of the window scores (Eq. 12) are needed
 * to fp64 accuracy.  For bf16 inputs they come from exact integer dot products
 * on the int8 matrix cores (engine 1, default), and so do the scores of the
 * columns that a screening separator recomputes, and of all columns of a layer
 * that does not screen (windows of at most 512 rows); engine 0 uses the fp64 matrix
 * instruction, as fp32 inputs always do.  Engine 1 evaluates its exponentials
 * from a table and a cubic (relative error 2e-13), so the two engines' scores
 * agree to about 1e-13 relative, not to the last bit; decisions (top-t, middle
 * pick, head ranking) are the same wherever the margin between the competing
 * values exceeds that (the parity tests demand 1e-9 of their inputs). */
int taskkv_set_stats_engine(taskkv_ctx *ctx, int engine);

/* Decode attention (Eq. 1 on the kept keys) deals the pages of a step to the
 * resident waves.  On MI355X the odd XCDs sustain less read bandwidth than the
 * even ones under a saturating stream, so waves of even workgroups take
 * (1024 + skew) / 1024 of an equal share and waves of odd workgroups
 * (1024 - skew) / 1024.  skew in [0, 128]; 0 deals equal shares; the default
 * (56) is the measured ratio.  Outputs stay within the stated tolerance for
 * any value; bit patterns depend on it (it moves the split points of the
 * partial sums).  Returns TASKKV_EINVAL for a value out of range. */
int taskkv_set_stream_skew(taskkv_ctx *ctx, int skew);

/*
 * Timing hooks for the benchmark.  on = 1: taskkv_decode_attn attaches two HIP
 * events to the launch of its attention kernel, on the launch stream; they
 * record when the kernel began and ended.  on = 2: taskkv_separate does the
 * same for its row-statistics kernel (Eq. 12, bf16 inputs).  on = 0: off.  2048 event pairs are
 * created by the first taskkv_profile_enable(ctx, 1); when all are in use the
 * next launch first waits for the recorded ones and adds their durations to a
 * running total, so every launch is counted however many there are (and the
 * host no longer runs ahead of the device: use it for measurement passes).
 * taskkv_profile_read waits for the recorded launches, returns the total in
 * *total_ms / *launches and clears it.  Keep profiling off while the stream is
 * being captured into a HIP graph.
 */
int taskkv_profile_enable(taskkv_ctx *ctx, int on);
int taskkv_profile_read(taskkv_ctx *ctx, double *total_ms, int64_t *launches);

#ifdef __cplusplus
}
#endif
#endif /* TASKKV_H */
