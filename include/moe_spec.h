/* moe_spec -- decode-time Mixture-of-Experts layer step with speculative expert prefetch,
 * for one AMD MI355X (gfx950).  C ABI: plain pointers and sizes only.
 *
 * What one layer step computes (paper: Sec. 3.1-3.3 for the signals, Sec. 4 for the execution
 * policy, Algorithm 1 and the "Implementation Details" of Sec. 5.1 for the block and its ordering):
 *
 *   s_l = LN_l(r_l);  (E_l, G_l) = TopK(Gate_l(s_l))               true routing of layer l
 *   d_l = sum_{e in E_l} g_{l,e} d_{l,e};  q_l = LN_{l+1}(r_l + d_l)  quasi-hidden state
 *   (E^_{l+1}, G^_{l+1}) = TopK(Gate_{l+1}(q_l))                    prediction for layer l+1
 *   prefetch of E^_{l+1} from the pinned host pool into layer l+1's device slots (copy stream)
 *   O_l = sum_{e in X_l} g_e * W_down_e( silu(W_gate_e s_l) * (W_up_e s_l) )
 *
 * X_l (executed experts and their mixing weights) is the set predicted at layer l-1 in
 * speculative mode (layer 0 of a token is a cold start: true routing, blocking load), and the
 * true routing in on-demand mode, where the load of E_l blocks the expert computation.
 * Prefetch-hint mode is the policy of earlier work the paper compares against (Sec. 2, Sec. 4): the
 * predicted experts are prefetched as in speculative mode, but the true experts are executed, and
 * those the prefetch missed are loaded on demand; its outputs equal on-demand mode's.
 * LN is RMSNorm with gain; TopK breaks ties towards the lower expert index; the mixing weights
 * are a softmax over the k selected logits.  Norms, router logits, top-k and gates are evaluated
 * in double precision; expert products accumulate in float.  With bf16 weights, s_l, q_l and the
 * SwiGLU product are rounded to bf16 (nearest even) before they enter a matrix product.
 *
 * Memory: "dev" pointers are device memory, "host" pointers are host memory.  The library never
 * allocates device memory: the caller hands it an arena (see moe_spec_arena_bytes).  The host
 * expert pool, the resident tables, the arena and both streams are borrowed and must outlive the
 * context.  The library owns the context, its events and a small pinned mailbox through which
 * the routing kernels hand expert ids to the host.
 *
 * Every call returns a status; nothing throws or aborts; outputs are untouched on error and
 * moe_spec_last_error gives the reason.  Calls on one context are not thread-safe.
 */
#ifndef MOE_SPEC_H
#define MOE_SPEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct moe_spec_ctx moe_spec_ctx;   /* opaque, library-owned */

enum { MOE_SPEC_OK = 0, MOE_SPEC_EINVAL = -1, MOE_SPEC_ENOMEM = -2, MOE_SPEC_ESTATE = -3,
       MOE_SPEC_EHIP = -4 };
enum { MOE_SPEC_MODE_ON_DEMAND = 0, MOE_SPEC_MODE_SPECULATIVE = 1, MOE_SPEC_MODE_PREFETCH_HINT = 2 };
enum { MOE_SPEC_F32 = 0, MOE_SPEC_BF16 = 1 };   /* storage type of every weight table */
enum { MOE_SPEC_COPY_DMA = 0, MOE_SPEC_COPY_KERNEL = 1, MOE_SPEC_COPY_DMA2 = 2 };

/* limits checked by moe_spec_create */
#define MOE_SPEC_MAX_EXPERTS 256
#define MOE_SPEC_MAX_TOP_K   16
#define MOE_SPEC_MAX_BATCH   64
#define MOE_SPEC_MAX_HIDDEN  8192

typedef struct {
  int32_t n_layers, hidden, n_experts, top_k, inter;   /* L, H, E, k, I; H and I multiples of 8 */
  int32_t max_batch;                /* largest decode batch B a step may be called with */
  int32_t slots_per_layer;          /* S >= k: device cache slots per layer (the memory cap) */
  int32_t dtype;                    /* MOE_SPEC_F32 | MOE_SPEC_BF16 */
  int32_t mode;                     /* MOE_SPEC_MODE_* */
  float   rms_eps;                  /* added to the mean square under the root */
  int32_t q_from_normalized;        /* 0: q_l = LN_{l+1}(r_l + d_l) (Sec. 3.2 equation);
                                       1: LN_{l+1}(s_l + d_l) (reading of the caption of Fig. 1) */
  int32_t predict_in_on_demand;     /* on-demand mode only: 1 still runs the prediction so that
                                       hit statistics exist; 0 skips it (timing runs) */
  int32_t profile;                  /* 1: bracket copies and kernels with timing events and fill
                                       copy_ms / compute_ms / stall_ms (adds a sync per token) */
  int32_t copy_engine;              /* how experts travel host -> device on the copy stream:
                                       0: one hipMemcpyAsync per expert (DMA engine);
                                       1: one gather-copy kernel per request that reads the pinned
                                          pool directly (a few workgroups; keeps the link busier but
                                          slows kernels that run beside it);
                                       2: experts dealt alternately to two DMA queues (copy_stream and one
                                          stream the library creates), so that one transfer's set-up hides
                                          behind the other's data */
  int32_t predict_signal;           /* what layer l+1's router is run on to predict: 0 the quasi-hidden
                                       state q_l (the method); 1 the normalised residual s_l as it is
                                       (the baseline signal of Sec. 3.3) */
  int32_t diagnostics;              /* 1: per-layer rank agreement and cosine similarity are collected
                                       too (moe_spec_layer_diagnostics); recall per layer always is */
  int32_t accumulate_defaults;      /* 1: keep, per layer and expert, the running sum and count of the
                                       un-gated outputs of every executed expert (the offline statistic
                                       behind the default vectors, Sec. 3.1); costs L*E*H doubles of arena
                                       and disables the fused batch-1 down+combine kernel */
  int32_t max_prefill_tokens;       /* 0 <= P_max <= 32768: most prompt tokens one moe_spec_prefill_layer_step takes;
                                       0: no prefill path.  Costs about P_max*(k+2)*H floats of arena */
  int32_t wait_spin_limit;          /* kernels that wait for another workgroup's result poll at most this
                                       often before they give up and the call after reports MOE_SPEC_EHIP;
                                       0: the default (about two seconds).  Tests force tiny values */
  int32_t lookahead;                /* prefetching modes: 0 or 1: experts are prefetched one layer ahead (the method);
                                       2: layer l also applies layer l+2's router to LN_{l+2}(r_l + d_l) and requests
                                       the experts it selects into layer l+2's pool as a cache hint, one layer before
                                       the regular prefetch (a reading of the multi-layer prefetching the paper leaves
                                       to future work).  Executed experts and outputs do not change.  Needs the
                                       router-based prediction (no estimator, predict_signal = 0, diagnostics = 0) */
  int32_t est_latent, est_ffn;      /* sizes of the neural estimator (Appendix A): latent size H/m and
                                       feed-forward size n*H/m, multiples of 8; 0, 0: no estimator */
  void   *device_arena;             /* dev, 256-byte aligned, >= moe_spec_arena_bytes(cfg) */
  size_t  device_arena_bytes;
  void   *compute_stream;           /* hipStream_t, borrowed; kernels run here */
  void   *copy_stream;              /* hipStream_t, borrowed; host-to-device expert copies run here */
} moe_spec_config;

typedef struct {
  int64_t tokens, layer_steps;
  int64_t predictions, hits;        /* recall@k of Sec. 3.3: hits = sum |E^_l & E_l|, predictions = sum k */
  int64_t cache_hits, cache_misses; /* per requested expert */
  int64_t h2d_bytes;                /* cache_misses * bytes per expert */
  int64_t hbm_bytes_algorithmic;    /* weight bytes the kernels had to read: routers, default-vector
                                       rows, executed experts */
  double  copy_ms, compute_ms, stall_ms;   /* profile=1 only, else 0: copy-stream busy time, kernel
                                       time, time the compute stream spent waiting for a copy */
  double  wall_ms;                  /* host clock from the first begin_token after create/reset to
                                       the end of this call's synchronisation */
  double  expert_ms;                /* profile=1 only: summed duration of the expert FFN launches (gate/up
                                       and down), each cache wave bracketed by two events on the
                                       compute stream */
  int64_t expert_launches;          /* number of such brackets */
  int64_t prefill_tokens;           /* prompt tokens through moe_spec_prefill_layer_step, summed over layers */
  int64_t predictions2, hits2;      /* lookahead = 2: recall@k of the predictions made two layers ahead */
  int64_t cache_waves;              /* decode steps: chunks of at most S experts the executed unions were split
                                       into; each is one cache request followed by one pass of the expert kernels */
} moe_spec_stats_t;

/* Optional per-step outputs, each dev [B, k] or NULL.  ids are by descending logit. */
typedef struct {
  int32_t *true_ids;  float *true_gates;     /* (E_l, G_l) */
  int32_t *exec_ids;  float *exec_gates;     /* what the expert kernels executed at this layer */
  int32_t *next_ids;  float *next_gates;     /* (E^_{l+1}, G^_{l+1}); untouched when no prediction ran */
} moe_spec_step_outputs;

/* Bytes of device arena a context with this configuration needs (slot cache of
 * L*S expert blocks plus scratch).  Returns 0 if the configuration is invalid. */
size_t moe_spec_arena_bytes(const moe_spec_config *cfg);

/* Bytes of one expert block in the host pool and in a device slot:
 * W_gate [I,H] | W_up [I,H] | W_down [H,I], row-major, in the configured dtype. */
size_t moe_spec_expert_bytes(const moe_spec_config *cfg);

/* The set-up that Algorithm 1 takes as given ("Require": the model's shape, a GPU expert cache C_l per
 * layer, experts resident on the CPU; Sec. 5.1 "Implementation Details" for the streams): validates cfg
 * (MOE_SPEC_EINVAL), then sets up events, the pinned mailbox and the hand-over slots on the current
 * device (MOE_SPEC_EHIP if no usable GPU).  *out is written only on success. */
int moe_spec_create(const moe_spec_config *cfg, moe_spec_ctx **out);

/* Tables that stay on the device (Sec. 5.1: only experts are offloaded).  router_w dev [E,H] and
 * default_vecs dev [E,H] in the configured dtype, rms_gain dev [H] float.  Borrowed. */
int moe_spec_set_layer_resident(moe_spec_ctx *ctx, int layer, const void *router_w,
                                const void *rms_gain, const void *default_vecs);

/* Weights of the neural expert estimator (paper: Sec. 6, Appendix A), forward pass only.  Every
 * matrix is dev, row-major [out, in], in the configured dtype, 16-byte aligned: proj [dm, H] (the
 * paper's A), layer_emb [L, dm], ffn_in [F, dm] (B), ffn_out [dm, F] (C), head [E, dm] (W_head);
 * ln_gain, ln_bias dev [dm] float.  dm = est_latent, F = est_ffn of the configuration
 * (MOE_SPEC_ESTATE if they are 0).  Borrowed.  The estimator maps the predicting signal of layer l
 * to logits for layer l+1: latent = proj.q + emb_l; latent += ffn_out.silu(ffn_in.latent);
 * logits = head.LayerNorm(latent); all in double precision. */
int moe_spec_set_estimator(moe_spec_ctx *ctx, const void *proj, const void *layer_emb, const void *ffn_in,
                           const void *ffn_out, const float *ln_gain, const float *ln_bias,
                           const void *head, float ln_eps);

/* use[l] != 0 (host, n_layers entries): the prediction made at layer l for layer l+1 takes the
 * estimator's logits instead of layer l+1's router (all layers: the paper's Est-PF; the layers with
 * low router hit rates only: Hybrid-PF).  Needs moe_spec_set_estimator first. */
int moe_spec_set_estimator_layers(moe_spec_ctx *ctx, const uint8_t *use, int n_layers);

/* The CPU-resident expert weights {W_{l,e}} of Algorithm 1, kept in pinned host memory so that copies to
 * the GPU can run asynchronously (Sec. 5.1 "Implementation Details"; only experts are offloaded).
 * Registers n_experts consecutive expert blocks of `layer`, starting at first_expert, that live at
 * pinned_host (host, page-locked: MOE_SPEC_EINVAL otherwise).  bytes must equal
 * n_experts * moe_spec_expert_bytes.  Nothing is copied: the pool is read at prefetch time. */
int moe_spec_load_host_experts(moe_spec_ctx *ctx, int layer, int first_expert, int n_experts,
                               const void *pinned_host, size_t bytes);

/* Starts a decode step: drops the carried prediction, so layer 0 is a cold start (Algorithm 1). */
int moe_spec_begin_token(moe_spec_ctx *ctx);

/* One MoE block with expert prefetch, Algorithm 1 (decode): true routing TopK(Gate_l(X)), GetNextExperts
 * (Sec. 3.1-3.3: d_l, q_l, layer l+1's router), WaitAndPrefetch of the predicted experts, MoE_l on the
 * experts chosen by the mode (Sec. 4).  r_dev [batch,H] float (post-attention residual r_l), out_dev [batch,H] float
 * (O_l, valid in compute-stream order).  Layers must be stepped 0,1,...,L-1 after begin_token with
 * the same batch (MOE_SPEC_ESTATE otherwise, also when a layer's tables or experts were never
 * registered).  outs may be NULL.  Asynchronous except for the hand-over of expert ids to the host.
 * Non-finite activations do not fault: a logit that is not a number ranks as minus infinity, so the k
 * ids stay distinct and inside [0, E); the row's gates and outputs are NaN. */
int moe_spec_layer_step(moe_spec_ctx *ctx, int layer, const void *r_dev, int batch, void *out_dev,
                        const moe_spec_step_outputs *outs);

/* For callers that cannot allocate device memory and want the arena to hold nothing but state
 * (code that runs where hipMalloc is forbidden, tight serving loops that size the arena once for
 * the slot cache): the same layer step as moe_spec_layer_step, same arguments, same results bit for
 * bit, but the scratch of the step (normalised inputs, router logits, true ids and gates, SwiGLU
 * products, un-gated expert outputs, the estimator's intermediates: everything the kernels write
 * and read back within one call) lives in a static device array inside the library instead of in
 * the arena.  The array is MOE_SPEC_STATIC_SCRATCH_BYTES large, one copy per GPU, held until the
 * process ends; its device address is looked up once per device by moe_spec_create.  The call
 * allocates nothing on the device (no hipMalloc, no hipFree, no event creation).
 * MOE_SPEC_EINVAL if the configuration's step scratch exceeds the array (it grows with
 * max_batch * top_k * (inter + hidden)); MOE_SPEC_ESTATE for a context with profile = 1 (timing
 * events are created on demand there) or when the current device is not the context's.
 * Every context on a GPU shares that GPU's array, and the array keeps the previous call's
 * contents: nothing in it has to start at zero (every word is written before it is read within a
 * call), but two calls that overlap in time on one GPU (two contexts on different streams, or two
 * host threads) race.  Calls of the two entry points may be mixed freely on one context. */
#define MOE_SPEC_STATIC_SCRATCH_BYTES (8u << 20)
int moe_spec_layer_step_static(moe_spec_ctx *ctx, int layer, const void *r_dev, int batch, void *out_dev,
                               const moe_spec_step_outputs *outs);

/* Prefill (paper: Sec. 5.2, prefill phase): one MoE block over all n_tokens prompt tokens at once.
 * Nothing is predicted: a prompt activates (nearly) every expert, so every expert of `layer` is
 * streamed from the host pool through the layer's slots, half of the slots receiving the next group
 * of experts while the kernels run on the other half, and every token executes its true top-k
 * experts.  Copies depend on no routing result, so the copy stream runs ahead of the compute stream
 * into the following layers' calls (the layer-ahead loading of the paper).  The call returns when
 * all of the layer's copies and kernels are queued; with more than S experts it waits on the host
 * for the kernels of the group before last, so it returns about one group of copies before the
 * layer's last transfer ends.
 * r_dev [n_tokens,H] float, out_dev [n_tokens,H] float (valid in compute-stream order),
 * 1 <= n_tokens <= max_prefill_tokens (MOE_SPEC_EINVAL otherwise).  true_ids / true_gates: dev
 * [n_tokens,k] or NULL.  Any layer order; not between begin_token and a token's last layer_step
 * (MOE_SPEC_ESTATE).  Leaves the layer's slot cache empty.  Counts E cache misses and E expert
 * blocks of host-to-device traffic. */
int moe_spec_prefill_layer_step(moe_spec_ctx *ctx, int layer, const void *r_dev, int n_tokens,
                                void *out_dev, int32_t *true_ids, float *true_gates);

/* Statistics of the predictions made FOR one layer (at the layer before it): recall@k as in the
 * paper's per-layer hit-rate figure, agreement per routing-weight rank as in its rank-alignment
 * figure, and the cosine similarity between the predicting signal (q_{l-1} or s_{l-1}) and the true
 * router input s_l as in its similarity figure.  The last two need diagnostics = 1. */
typedef struct {
  int64_t predictions, hits;
  int64_t rank_match[MOE_SPEC_MAX_TOP_K];   /* tokens whose predicted expert at rank j is the true one */
  double  cos_sum;                          /* sum over tokens; divide by cos_count */
  int64_t cos_count;
} moe_spec_layer_diag_t;

/* Synchronises both streams, then copies layer `layer`'s statistics. */
int moe_spec_layer_diagnostics(moe_spec_ctx *ctx, int layer, moe_spec_layer_diag_t *out);

/* accumulate_defaults = 1 only (MOE_SPEC_ESTATE otherwise): writes the mean un-gated output of each
 * expert of `layer` over the steps that executed it to mean_dev (dev [E,H] float, zero rows for experts
 * never executed) and the number of executions to counts_host (host [E], may be NULL).  These means
 * are the per-expert default vectors d_{l,e} of Sec. 3.1.  Synchronises the compute stream. */
int moe_spec_read_default_vectors(moe_spec_ctx *ctx, int layer, float *mean_dev, int64_t *counts_host);

/* The figures the paper's evaluation reports (Sec. 3.3 recall@k; Sec. 5.1.2 time per output token and its
 * compute / copy / idle parts).  Synchronises both streams, then copies the counters. */
int moe_spec_stats(moe_spec_ctx *ctx, moe_spec_stats_t *out);

/* Empties the slot cache, drops the carried prediction and zeroes the statistics. */
int moe_spec_reset(moe_spec_ctx *ctx);

void moe_spec_destroy(moe_spec_ctx *ctx);

/* Text of the last error on this context (or of the last failed moe_spec_create when ctx is NULL). */
const char *moe_spec_last_error(const moe_spec_ctx *ctx);

/* Measurement aid: launches one of the weight-streaming kernels `reps` times back to back on the
 * compute stream between two timing events, each launch on the slots of the next layer in turn
 * (so that no launch finds its weights in a cache), executing k resident slots per launch for a
 * batch of one.  which: 0 = gate/up GEMV + SwiGLU, 1 = down GEMV + combine, 2 = router (true routing),
 * 3 = a kernel that only reads the gate/up bytes of the same slots (what streaming alone reaches),
 * 4 / 5 = the matrix-core gate/up / down kernels (bf16 only) on a batch of max_batch tokens whose
 * k*max_batch positions are dealt round-robin over min(S, E, k*max_batch) resident slots,
 * 6 = the fused routing kernel doing the true routing only, 7 = the same kernel doing the true routing and
 * the prediction for the next layer (both routers and k default-vector rows per token), both on a batch of
 * max_batch tokens,
 * 9 = a kernel that only reads the W_down bytes of the same slots (8 is not used).
 * Writes the mean milliseconds per launch and the weight bytes one launch reads.
 * The slot contents are whatever the cache holds; outputs go to scratch.  Not inside a decode step. */
int moe_spec_time_kernel(moe_spec_ctx *ctx, int which, int reps, double *ms_per_launch,
                         int64_t *bytes_per_launch);

#ifdef __cplusplus
}
#endif
#endif /* MOE_SPEC_H */
