/* A plain C client of the library: no Python, no torch.  It builds a tiny float32 model with a
 * pinned host pool, runs two decode steps in each of the three modes plus a prefill pass, and checks
 * what must hold without any reference implementation: every call succeeds, outputs are finite,
 * the counters obey their identities (predictions = k*B*(L-1) per token, bytes = misses * block
 * size), two runs of one mode are bit-identical, and prefetch-hint mode reproduces on-demand
 * mode's outputs bit for bit (paper: Sec. 4 -- the hint policy executes the true experts).
 * Exit status 0 and a last line "abi demo ok" on success. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "../../include/moe_spec.h"

enum { L = 3, H = 64, E = 6, K = 2, I = 40, S = 3, B = 2, TOKENS = 2, P = 5 };

#define HIP_OK(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { \
  fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_)); return 1; } } while (0)
#define LIB_OK(ctx, call) do { int rc_ = (call); if (rc_ != MOE_SPEC_OK) { \
  fprintf(stderr, "%s returned %d: %s\n", #call, rc_, moe_spec_last_error(ctx)); return 1; } } while (0)

static unsigned long long rng_state = 0x9E3779B97F4A7C15ull;
static float draw(float scale) {                      /* uniform in [-scale, scale): enough for a demo */
  rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
  return scale * ((float)((rng_state >> 40) & 0xFFFFFF) / 8388608.0f - 1.0f);
}

static int run_mode(int mode, const moe_spec_config *base, void *const *router, void *const *gain,
                    void *const *dvec, const float *pool, size_t expert_bytes, const float *x_host,
                    float *out_host, moe_spec_stats_t *st) {
  moe_spec_config cfg = *base;
  cfg.mode = mode;
  moe_spec_ctx *ctx = NULL;
  if (moe_spec_create(&cfg, &ctx) != MOE_SPEC_OK) {
    fprintf(stderr, "moe_spec_create: %s\n", moe_spec_last_error(NULL));
    return 1;
  }
  for (int l = 0; l < L; ++l) {
    LIB_OK(ctx, moe_spec_set_layer_resident(ctx, l, router[l], gain[l], dvec[l]));
    LIB_OK(ctx, moe_spec_load_host_experts(ctx, l, 0, E, (const char *)pool + (size_t)l * E * expert_bytes,
                                            E * expert_bytes));
  }
  float *r_dev = NULL, *o_dev = NULL;
  HIP_OK(hipMalloc((void **)&r_dev, sizeof(float) * P * H));
  HIP_OK(hipMalloc((void **)&o_dev, sizeof(float) * P * H));
  hipStream_t compute = (hipStream_t)cfg.compute_stream;
  float r_host[B * H];
  for (int t = 0; t < TOKENS; ++t) {
    LIB_OK(ctx, moe_spec_begin_token(ctx));
    memcpy(r_host, x_host + (size_t)t * B * H, sizeof r_host);
    for (int l = 0; l < L; ++l) {
      HIP_OK(hipMemcpyAsync(r_dev, r_host, sizeof r_host, hipMemcpyHostToDevice, compute));
      LIB_OK(ctx, moe_spec_layer_step(ctx, l, r_dev, B, o_dev, NULL));
      float *o = out_host + ((size_t)t * L + l) * B * H;
      HIP_OK(hipMemcpyAsync(o, o_dev, sizeof r_host, hipMemcpyDeviceToHost, compute));
      HIP_OK(hipStreamSynchronize(compute));
      for (int i = 0; i < B * H; ++i) {
        if (!isfinite(o[i])) { fprintf(stderr, "non-finite output at token %d layer %d\n", t, l); return 1; }
        r_host[i] += o[i];                              /* the residual stream of a model without attention */
      }
    }
  }
  LIB_OK(ctx, moe_spec_stats(ctx, st));
  /* a prompt of P tokens through the prefill step of every layer */
  float p_host[P * H];
  for (int i = 0; i < P * H; ++i) p_host[i] = x_host[i % (TOKENS * B * H)];
  for (int l = 0; l < L; ++l) {
    HIP_OK(hipMemcpyAsync(r_dev, p_host, sizeof p_host, hipMemcpyHostToDevice, compute));
    LIB_OK(ctx, moe_spec_prefill_layer_step(ctx, l, r_dev, P, o_dev, NULL, NULL));
    float o[P * H];
    HIP_OK(hipMemcpyAsync(o, o_dev, sizeof o, hipMemcpyDeviceToHost, compute));
    HIP_OK(hipStreamSynchronize(compute));
    for (int i = 0; i < P * H; ++i) {
      if (!isfinite(o[i])) { fprintf(stderr, "non-finite prefill output at layer %d\n", l); return 1; }
      p_host[i] += o[i];
    }
  }
  moe_spec_stats_t after;
  LIB_OK(ctx, moe_spec_stats(ctx, &after));
  if (after.prefill_tokens != (int64_t)P * L || after.cache_misses - st->cache_misses != (int64_t)E * L) {
    fprintf(stderr, "prefill counters are off\n");
    return 1;
  }
  /* argument errors come back as codes, with a reason */
  if (moe_spec_layer_step(ctx, 0, r_dev, B, o_dev, NULL) != MOE_SPEC_ESTATE ||      /* no begin_token */
      moe_spec_prefill_layer_step(ctx, L, r_dev, P, o_dev, NULL, NULL) != MOE_SPEC_EINVAL) {
    fprintf(stderr, "expected error codes did not come back\n");
    return 1;
  }
  moe_spec_destroy(ctx);
  HIP_OK(hipFree(r_dev));
  HIP_OK(hipFree(o_dev));
  return 0;
}

int main(void) {
  moe_spec_config cfg;
  memset(&cfg, 0, sizeof cfg);
  cfg.n_layers = L; cfg.hidden = H; cfg.n_experts = E; cfg.top_k = K; cfg.inter = I;
  cfg.max_batch = B; cfg.slots_per_layer = S; cfg.dtype = MOE_SPEC_F32; cfg.rms_eps = 1e-6f;
  cfg.predict_in_on_demand = 1; cfg.copy_engine = MOE_SPEC_COPY_DMA2; cfg.max_prefill_tokens = P;
  const size_t expert_bytes = moe_spec_expert_bytes(&cfg), arena_bytes = moe_spec_arena_bytes(&cfg);
  if (expert_bytes != (size_t)3 * H * I * sizeof(float) || arena_bytes == 0) {
    fprintf(stderr, "sizing calls are off\n");
    return 1;
  }
  HIP_OK(hipMalloc(&cfg.device_arena, arena_bytes));
  cfg.device_arena_bytes = arena_bytes;
  hipStream_t compute, copy;
  HIP_OK(hipStreamCreateWithFlags(&compute, hipStreamNonBlocking));
  HIP_OK(hipStreamCreateWithFlags(&copy, hipStreamNonBlocking));
  cfg.compute_stream = compute;
  cfg.copy_stream = copy;

  /* resident tables on the device, expert pool in pinned host memory */
  void *router[L], *gain[L], *dvec[L];
  float tmp[E * H];
  for (int l = 0; l < L; ++l) {
    HIP_OK(hipMalloc(&router[l], sizeof tmp));
    HIP_OK(hipMalloc(&dvec[l], sizeof tmp));
    HIP_OK(hipMalloc(&gain[l], sizeof(float) * H));
    for (int i = 0; i < E * H; ++i) tmp[i] = draw(0.2f);
    HIP_OK(hipMemcpy(router[l], tmp, sizeof tmp, hipMemcpyHostToDevice));
    for (int i = 0; i < E * H; ++i) tmp[i] = draw(0.05f);
    HIP_OK(hipMemcpy(dvec[l], tmp, sizeof tmp, hipMemcpyHostToDevice));
    for (int i = 0; i < H; ++i) tmp[i] = 1.0f + draw(0.1f);
    HIP_OK(hipMemcpy(gain[l], tmp, sizeof(float) * H, hipMemcpyHostToDevice));
  }
  float *pool = NULL;
  HIP_OK(hipHostMalloc((void **)&pool, (size_t)L * E * expert_bytes, hipHostMallocDefault));
  for (size_t i = 0; i < (size_t)L * E * 3 * H * I; ++i) pool[i] = draw(0.1f);
  float x_host[TOKENS * B * H];
  for (int i = 0; i < TOKENS * B * H; ++i) x_host[i] = draw(1.0f);

  /* a pool that is not page-locked is refused */
  {
    moe_spec_ctx *ctx = NULL;
    cfg.mode = MOE_SPEC_MODE_ON_DEMAND;
    if (moe_spec_create(&cfg, &ctx) != MOE_SPEC_OK) { fprintf(stderr, "create: %s\n", moe_spec_last_error(NULL)); return 1; }
    void *pageable = malloc(E * expert_bytes);
    if (moe_spec_load_host_experts(ctx, 0, 0, E, pageable, E * expert_bytes) != MOE_SPEC_EINVAL) {
      fprintf(stderr, "a pageable pool was accepted\n");
      return 1;
    }
    free(pageable);
    moe_spec_destroy(ctx);
  }

  static float out[4][TOKENS * L * B * H];
  moe_spec_stats_t st[4];
  const int modes[4] = {MOE_SPEC_MODE_ON_DEMAND, MOE_SPEC_MODE_PREFETCH_HINT, MOE_SPEC_MODE_SPECULATIVE,
                        MOE_SPEC_MODE_SPECULATIVE};
  for (int m = 0; m < 4; ++m)
    if (run_mode(modes[m], &cfg, router, gain, dvec, pool, expert_bytes, x_host, out[m], &st[m])) return 1;

  if (memcmp(out[0], out[1], sizeof out[0]) != 0) { fprintf(stderr, "hint mode differs from on-demand mode\n"); return 1; }
  if (memcmp(out[2], out[3], sizeof out[2]) != 0) { fprintf(stderr, "two speculative runs differ\n"); return 1; }
  for (int m = 0; m < 4; ++m) {
    if (st[m].tokens != TOKENS || st[m].layer_steps != TOKENS * L ||
        st[m].predictions != (int64_t)K * B * (L - 1) * TOKENS || st[m].hits < 0 || st[m].hits > st[m].predictions ||
        st[m].h2d_bytes != st[m].cache_misses * (int64_t)expert_bytes) {
      fprintf(stderr, "counters of mode %d are off\n", modes[m]);
      return 1;
    }
  }
  printf("on-demand: %lld misses; hint: %lld misses; speculative: %lld misses, recall %lld / %lld\n",
         (long long)st[0].cache_misses, (long long)st[1].cache_misses, (long long)st[2].cache_misses,
         (long long)st[2].hits, (long long)st[2].predictions);
  printf("abi demo ok\n");
  return 0;
}
