/*
 * A caller of the Task-KV library written in plain C (compiled with gcc, no
 * C++ and no Python): reads one layer's tensors from raw files, runs
 * separate -> compress -> one decode step with append through the C ABI and
 * writes the results back as raw files.  tests/test_gpu_c_caller.py prepares
 * the inputs with the seeded generators and checks the outputs against the
 * oracle.
 *
 * usage: taskkv_c_caller DIR [stack]
 *   DIR/cfg.txt    the sixteen fields of taskkv_layer_cfg in order, then the
 *                  number of tokens to reserve per unit for decoding
 *   DIR/q_win.bin  [B, Hq, L, d]   DIR/k.bin, DIR/v.bin  [B, Hkv, N, d]
 *   DIR/q.bin      [B, Hq, d]      DIR/k_new.bin, DIR/v_new.bin  [B, Hkv, d]
 * writes mask.bin (u8), dist.bin (f64), lens.bin (i32), offsets.bin (i64),
 * kept_idx.bin (i32), out.bin (f32).
 *
 * With `stack` it then treats the same tensors as a stack of two layers that
 * differ in their middle budget (layer 1 keeps half of layer 0's), compresses
 * both into one cache allocation, has taskkv_stack_rebase write the stack's
 * offsets and runs one taskkv_decode_attn_layers step for both layers; it
 * writes out_stack.bin (f32 [2, B, Hq, d]) and lens_stack.bin (i32 [2, B*Hkv]).
 */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "taskkv.h"

#define CHECK_HIP(x)                                                            \
  do {                                                                          \
    hipError_t e_ = (x);                                                        \
    if (e_ != hipSuccess) {                                                     \
      fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));                   \
      return 2;                                                                 \
    }                                                                           \
  } while (0)
#define CHECK_TK(x)                                                             \
  do {                                                                          \
    int r_ = (x);                                                               \
    if (r_ != TASKKV_OK) {                                                      \
      fprintf(stderr, "%s: %s\n", #x, taskkv_strerror(r_));                     \
      return 3;                                                                 \
    }                                                                           \
  } while (0)

static char path[4096];
static const char *in_dir(const char *dir, const char *name) {
  snprintf(path, sizeof path, "%s/%s", dir, name);
  return path;
}

/* file -> freshly allocated device buffer of exactly `bytes` bytes */
static int load(const char *dir, const char *name, size_t bytes, void **dev) {
  FILE *f = fopen(in_dir(dir, name), "rb");
  void *host = malloc(bytes);
  if (!f || !host || fread(host, 1, bytes, f) != bytes) {
    fprintf(stderr, "cannot read %zu bytes of %s\n", bytes, name);
    return 1;
  }
  fclose(f);
  if (hipMalloc(dev, bytes) != hipSuccess || hipMemcpy(*dev, host, bytes, hipMemcpyHostToDevice) != hipSuccess) {
    fprintf(stderr, "cannot place %s on the device\n", name);
    return 1;
  }
  free(host);
  return 0;
}

static int store(const char *dir, const char *name, const void *dev, size_t bytes) {
  void *host = malloc(bytes);
  FILE *f = fopen(in_dir(dir, name), "wb");
  if (!host || !f || hipMemcpy(host, dev, bytes, hipMemcpyDeviceToHost) != hipSuccess ||
      fwrite(host, 1, bytes, f) != bytes) {
    fprintf(stderr, "cannot write %s\n", name);
    return 1;
  }
  fclose(f);
  free(host);
  return 0;
}

int main(int argc, char **argv) {
  if (argc != 2 && !(argc == 3 && strcmp(argv[2], "stack") == 0)) {
    fprintf(stderr, "usage: %s DIR [stack]\n", argv[0]);
    return 1;
  }
  const int with_stack = argc == 3;
  const char *dir = argv[1];
  taskkv_layer_cfg cfg;
  int reserve = 0;
  FILE *f = fopen(in_dir(dir, "cfg.txt"), "r");
  if (!f || fscanf(f, "%d %d %d %d %d %d %d %d %d %d %d %d %d %d %d %f %d", &cfg.batch, &cfg.n_q_heads,
                   &cfg.n_kv_heads, &cfg.head_dim, &cfg.ctx_len, &cfg.obs_window, &cfg.top_t, &cfg.n_sink,
                   &cfg.n_recent, &cfg.n_middle, &cfg.n_hetero, &cfg.add_centre_head, &cfg.pool_kernel,
                   &cfg.pack_mode, &cfg.dtype, &cfg.softmax_scale, &reserve) != 17) {
    fprintf(stderr, "cannot read cfg.txt\n");
    return 1;
  }
  fclose(f);
  const size_t B = cfg.batch, Hq = cfg.n_q_heads, Hkv = cfg.n_kv_heads, d = cfg.head_dim, N = cfg.ctx_len,
               L = cfg.obs_window, esz = cfg.dtype == TASKKV_F32 ? 4 : 2, units = B * Hkv;
  const size_t row = (size_t)cfg.n_sink + cfg.n_middle + cfg.n_recent;

  const int64_t capacity = taskkv_cache_tokens(&cfg, reserve);
  size_t ws = taskkv_workspace_bytes(&cfg, reserve);
  /* the stacked decode step needs the workspace of a cfg with (layers x B) batch elements */
  taskkv_layer_cfg cfg_l1 = cfg, cfg_both = cfg;
  cfg_l1.n_middle = cfg.n_middle / 2;
  cfg_both.batch = 2 * cfg.batch;
  const int64_t cap_l1 = taskkv_cache_tokens(&cfg_l1, reserve);
  if (with_stack) {
    const size_t ws_both = taskkv_workspace_bytes(&cfg_both, reserve);
    if (cap_l1 <= 0 || ws_both == 0) {
      fprintf(stderr, "the library rejects the stacked cfg\n");
      return 1;
    }
    ws = ws_both > ws ? ws_both : ws;
  }
  if (capacity <= 0 || ws == 0) {
    fprintf(stderr, "the library rejects this cfg\n");
    return 1;
  }
  CHECK_HIP(hipSetDevice(0));
  void *q_win, *k, *v, *q, *k_new, *v_new;
  if (load(dir, "q_win.bin", B * Hq * L * d * esz, &q_win) || load(dir, "k.bin", units * N * d * esz, &k) ||
      load(dir, "v.bin", units * N * d * esz, &v) || load(dir, "q.bin", B * Hq * d * esz, &q) ||
      load(dir, "k_new.bin", units * d * esz, &k_new) || load(dir, "v_new.bin", units * d * esz, &v_new))
    return 1;
  double *scores, *sem_vec, *dist;
  uint8_t *mask;
  void *k_cache, *v_cache;
  int64_t *offsets;
  int32_t *lens, *kept_idx = NULL;
  float *out;
  CHECK_HIP(hipMalloc((void **)&scores, units * N * sizeof(double)));
  CHECK_HIP(hipMalloc((void **)&sem_vec, units * d * sizeof(double)));
  CHECK_HIP(hipMalloc((void **)&dist, units * sizeof(double)));
  CHECK_HIP(hipMalloc((void **)&mask, units));
  CHECK_HIP(hipMalloc(&k_cache, (size_t)capacity * d * esz));
  CHECK_HIP(hipMalloc(&v_cache, (size_t)capacity * d * esz));
  CHECK_HIP(hipMalloc((void **)&offsets, (units + 1) * sizeof(int64_t)));
  CHECK_HIP(hipMalloc((void **)&lens, units * sizeof(int32_t)));
  if (row) CHECK_HIP(hipMalloc((void **)&kept_idx, units * row * sizeof(int32_t)));
  CHECK_HIP(hipMalloc((void **)&out, B * Hq * d * sizeof(float)));

  taskkv_ctx *ctx = NULL;
  hipStream_t stream;
  CHECK_HIP(hipStreamCreate(&stream));
  CHECK_TK(taskkv_create(&ctx, 0, ws));
  CHECK_TK(taskkv_separate(ctx, &cfg, q_win, k, v, scores, sem_vec, dist, mask, stream));
  CHECK_TK(taskkv_compress(ctx, &cfg, k, v, scores, mask, k_cache, v_cache, capacity, reserve, offsets, lens,
                           kept_idx, stream));
  CHECK_TK(taskkv_decode_attn(ctx, &cfg, q, k_new, v_new, k_cache, v_cache, capacity, offsets, lens, out, stream));
  CHECK_HIP(hipStreamSynchronize(stream));
  if (taskkv_last_async_error(ctx, stream) != 0) {
    fprintf(stderr, "the device reported an error\n");
    return 4;
  }
  if (store(dir, "mask.bin", mask, units) || store(dir, "dist.bin", dist, units * sizeof(double)) ||
      store(dir, "lens.bin", lens, units * sizeof(int32_t)) ||
      store(dir, "offsets.bin", offsets, (units + 1) * sizeof(int64_t)) ||
      (row && store(dir, "kept_idx.bin", kept_idx, units * row * sizeof(int32_t))) ||
      store(dir, "out.bin", out, B * Hq * d * sizeof(float)))
    return 1;
  if (with_stack) {
    /* two layers in one allocation: layer 0 = cfg, layer 1 = cfg_l1, same input tensors */
    const int64_t caps[2] = {capacity, cap_l1};
    const int64_t cap_all = capacity + cap_l1;
    void *k_all, *v_all, *q2, *kn2, *vn2;
    int64_t *layer_off, *stack_off;
    int32_t *lens2, *kept2 = NULL;
    float *out2;
    CHECK_HIP(hipMalloc(&k_all, (size_t)cap_all * d * esz));
    CHECK_HIP(hipMalloc(&v_all, (size_t)cap_all * d * esz));
    CHECK_HIP(hipMalloc((void **)&layer_off, 2 * (units + 1) * sizeof(int64_t)));
    CHECK_HIP(hipMalloc((void **)&stack_off, (2 * units + 1) * sizeof(int64_t)));
    CHECK_HIP(hipMalloc((void **)&lens2, 2 * units * sizeof(int32_t)));
    if (row) CHECK_HIP(hipMalloc((void **)&kept2, units * row * sizeof(int32_t)));
    CHECK_HIP(hipMalloc((void **)&out2, 2 * B * Hq * d * sizeof(float)));
    CHECK_HIP(hipMalloc(&q2, 2 * B * Hq * d * esz));
    CHECK_HIP(hipMalloc(&kn2, 2 * units * d * esz));
    CHECK_HIP(hipMalloc(&vn2, 2 * units * d * esz));
    for (int r = 0; r < 2; ++r) {
      CHECK_HIP(hipMemcpy((char *)q2 + r * B * Hq * d * esz, q, B * Hq * d * esz, hipMemcpyDeviceToDevice));
      CHECK_HIP(hipMemcpy((char *)kn2 + r * units * d * esz, k_new, units * d * esz, hipMemcpyDeviceToDevice));
      CHECK_HIP(hipMemcpy((char *)vn2 + r * units * d * esz, v_new, units * d * esz, hipMemcpyDeviceToDevice));
    }
    CHECK_TK(taskkv_compress(ctx, &cfg, k, v, scores, mask, k_all, v_all, capacity, reserve, layer_off, lens2,
                             kept_idx, stream));
    CHECK_TK(taskkv_compress(ctx, &cfg_l1, k, v, scores, mask, (char *)k_all + (size_t)capacity * d * esz,
                             (char *)v_all + (size_t)capacity * d * esz, cap_l1, reserve, layer_off + units + 1,
                             lens2 + units, kept2, stream));
    CHECK_TK(taskkv_stack_rebase(ctx, 2, (int32_t)units, layer_off, caps, stack_off, stream));
    CHECK_TK(taskkv_decode_attn_layers(ctx, &cfg, 2, q2, kn2, vn2, k_all, v_all, cap_all, stack_off, lens2, out2,
                                       stream));
    CHECK_HIP(hipStreamSynchronize(stream));
    if (taskkv_last_async_error(ctx, stream) != 0) {
      fprintf(stderr, "the device reported an error in the stacked step\n");
      return 4;
    }
    if (store(dir, "out_stack.bin", out2, 2 * B * Hq * d * sizeof(float)) ||
        store(dir, "lens_stack.bin", lens2, 2 * units * sizeof(int32_t)))
      return 1;
  }
  taskkv_destroy(ctx);
  CHECK_HIP(hipStreamDestroy(stream));
  printf("ok: %zu units, cache of %lld tokens, workspace %zu bytes\n", units, (long long)capacity, ws);
  return 0;
}
