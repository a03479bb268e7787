// Argument blocks and launchers of the device kernels.  Host code sees only this header.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moe_spec {

constexpr int kMaxExperts = 256;
constexpr int kMaxTopK = 16;
constexpr int kMaxBatch = 64;
constexpr int kRouteBlock = 256;        // threads per workgroup of the routing kernels
constexpr int kRouteRowsPerBlock = 4;   // one router row per wavefront
constexpr int kMailboxIds = kMaxBatch * kMaxTopK;

// Pinned host mailbox written by the reporting workgroups of a routing kernel.  Every id word is its own flag:
// the host sets the words it is about to wait for to -1 before the launch and spins until none is -1.
struct Mailbox {
  int32_t ids[kMailboxIds];   // [B, k] expert ids by descending logit
  uint32_t pad[16];
};

// Per-layer statistics of the predictions made for a layer, accumulated by the routing kernel
// that computes the layer's true routing (paper: Sec. 3.3 recall@k; the per-rank agreement and the
// cosine similarity of the figures in Sec. 3.3 and Sec. 4).
struct LayerDiag {
  unsigned long long hits, preds;
  unsigned long long rank_match[kMaxTopK];   // same expert at the same routing-weight rank
  double cos_sum;                            // sum over tokens of cos(predicting signal, s_l)
  unsigned long long cos_count;
};

// Routing kernel: RMSNorm -> router GEMV -> top-k -> softmax over the selected logits.
// spec = 0: input is r_l (true routing of layer l).
// spec = 1: input is r_l (or s_l) + sum_j g_j d_{l,e_j}, normalised with layer l+1's gain and
//           routed with layer l+1's router (the quasi-hidden state of Sec. 3.2).
// spec = 2: input is s_l as it is, routed with layer l+1's router (the baseline signal of Sec. 3.3).
// spec = 3: input is x_f64 [B,H] (the estimator's latent vector), LayerNorm with gain and bias,
//           then the estimator's head as the "router" (Appendix A); H is the latent size.
struct RouteArgs {
  const float *r;             // [B,H]
  const float *s_in;          // [B,H] s_l, read when spec && from_normalized
  const void *w;              // [E,H] router weights of the layer being routed
  const float *gain;          // [H] gain of that layer's norm
  const float *bias;          // [H] LayerNorm bias (spec = 3)
  const double *x_f64;        // [B,H] input of spec = 3
  const void *dvec;           // spec: [E,H] default vectors of layer l
  const int32_t *d_ids;       // spec: [B,k] true ids of layer l
  const double *d_gates;      // spec: [B,k] true gates of layer l
  unsigned long long *slots;  // [B,E] logit hand-over slots of this launch, armed (all ones)
  unsigned long long *arm_a, *arm_b;   // the two sets of slots the next routing launch may use, armed by this launch
  int arm_count;              // slots per set (largest batch * E)
  unsigned int spin_limit;    // bound of the finishing workgroup's wait for a logit
  unsigned int *status;       // pinned host word raised when that wait runs out
  float *vec_out;             // [B,H] normalised (and rounded) vector, or null
  uint16_t *vec_out_q;        // [B,H] the same as bf16 bit patterns (bf16 mode), or null
  int32_t *ids_out;           // [B,k]
  float *gates_out;           // [B,k]
  double *gates64_out;        // [B,k] or null
  const int32_t *cmp_ids;     // [B,k] prediction to score against this routing, or null
  LayerDiag *diag;            // statistics of the layer being routed (spec = 0)
  const float *prev_signal;   // [B,H] the vector that predicted this layer, for the cosine; or null
  int rank_stats;             // also count per-rank agreement
  int32_t *user_ids;          // optional copies for the caller
  float *user_gates;
  Mailbox *mailbox;           // pinned host, or null: ids[B*k] words the host set to -1 and waits for
  int B, H, E, k;
  float eps;
  int bf16, spec, from_normalized, tok_tile;
};

// True routing of layer l and the prediction for layer l+1 in one launch (route_pair_kernel).  Logits
// travel between the workgroups of a token through 8-byte slots that hold all ones until written; the
// two sets of slots are used by alternate launches, and a launch re-arms the other set.
struct RoutePairArgs {
  const float *r;                         // [B,H] r_l
  const void *w_true, *w_next;            // [E,H] routers of layers l and l+1; w_next null: no prediction
  const float *gain_true, *gain_next;     // [H] gains of LN_l and LN_{l+1}
  const void *dvec;                       // [E,H] default vectors d_{l,e}
  unsigned long long *z_true, *z_pred;    // [B,E] logit slots of this launch, armed
  unsigned long long *z_true_next, *z_pred_next;   // the other set, armed by this launch
  int arm_count;                          // slots per set (largest batch * E)
  float *s_out;                           // [B,H] s_l for the expert kernels
  uint16_t *s_out_q;                      // [B,H] the same as bf16 bit patterns, or null
  int32_t *true_ids;  float *true_gates;  // [B,k]
  double *true_gates64;                   // [B,k] the same gates unrounded, or null
  int32_t *next_ids;  float *next_gates;  // [B,k] the prediction carried to layer l+1
  const int32_t *cmp_ids;                 // [B,k] prediction to score against this routing, or null
  LayerDiag *diag;
  int32_t *user_true_ids;  float *user_true_gates;   // optional copies for the caller
  int32_t *user_next_ids;  float *user_next_gates;
  Mailbox *mb_true, *mb_next;             // pinned host, or null: ids[B*k] words the host set to -1 and waits for
  unsigned int *status;                   // raised when a bounded wait ran out
  int B, H, E, k;
  float eps;
  int bf16, from_normalized;
  unsigned int spin_limit;
  unsigned long long *stage_clock;        // development builds only (MOE_SPEC_STAGE_CLOCK): [12] stage times, or null
};
bool route_pair_supported(int H, int dtype);
hipError_t launch_route_pair(const RoutePairArgs &a, int dtype, hipStream_t st);

// Expert kernels read weights from the device slots of one layer.
struct ActiveList {           // experts executed by one launch and where they live
  int32_t n;
  int16_t expert[kMaxExperts];
  int16_t slot[kMaxExperts];
};

struct ExpertArgs {
  const char *pool;           // first slot of the layer's pool
  size_t slot_bytes;          // distance between slots (expert block bytes)
  const float *s;             // [B,H] router input s_l
  const int32_t *exec_ids;    // [B,k]
  const float *exec_gates;    // [B,k]
  float *h;                   // [B,k,I] SwiGLU products
  float *y;                   // [B,k,H] un-gated expert outputs
  float *out;                 // [B,H]
  int B, k, H, I, bf16;
  // matrix-core kernels over more than one decode batch (prefill): positions grouped by expert as
  // written by launch_expert_lists for list_tokens tokens; null: the [B,k] table exec_ids is searched
  const int32_t *pos_list;    // [E, list_stride]
  const int32_t *pos_count;   // [E]
  int list_stride, list_tokens;
};

// Host-to-device gather copy: each entry moves one expert block from the pinned pool to a slot.
constexpr int kCopyListMax = 32;
struct CopyList {
  const void *src[kCopyListMax];   // host (pinned, device-visible)
  void *dst[kCopyListMax];         // device slot
  int32_t n;
  uint32_t n16;                    // 16-byte units per block
};
hipError_t launch_gather_copy(const CopyList &cl, hipStream_t st);

// Double-precision GEMV used by the estimator: y = act(W x + add_w) + add_f64.
struct GemvArgs {
  const void *w;              // [rows, cols] in the weight dtype
  const float *x_f32;         // [B, cols], or null when x_f64 is given
  const double *x_f64;        // [B, cols]
  const void *add_w;          // [rows] in the weight dtype, added before the activation, or null
  const double *add_f64;      // [B, rows] added after the activation, or null
  double *y;                  // [B, rows]
  int B, rows, cols, silu;
};
hipError_t launch_gemv64(const GemvArgs &a, int dtype, hipStream_t st);

hipError_t launch_route(const RouteArgs &a, int dtype, hipStream_t st);
hipError_t launch_gateup(const ExpertArgs &a, const ActiveList &act, int dtype, hipStream_t st);
hipError_t launch_down(const ExpertArgs &a, const ActiveList &act, int dtype, hipStream_t st);
hipError_t launch_combine(const ExpertArgs &a, hipStream_t st);
// reads n16 16-byte units of every active slot, starting first16 units into the slot, and nothing else
hipError_t launch_stream_read(const ExpertArgs &a, const ActiveList &act, size_t first16, size_t n16, hipStream_t st);
hipError_t launch_gateup_mfma(const ExpertArgs &a, const ActiveList &act, const uint16_t *s_q, uint16_t *hq,
                              hipStream_t st);
hipError_t launch_down_mfma(const ExpertArgs &a, const ActiveList &act, const uint16_t *hq, hipStream_t st);
hipError_t launch_expert_lists(const int32_t *ids, int tokens, int k, int E, int32_t *pos, int32_t *count,
                               hipStream_t st);      // pos [E, tokens], count [E]
constexpr int kMfmaMinBatch = 2;      // bf16 decode batches from here on use the matrix-core expert kernels
// Running sums for the default vectors: sum[e,:] += y[f,:] and cnt[e] += 1 for every position f whose
// expert ids[f] is in the launch's active list; means = sum / max(cnt, 1).
hipError_t launch_accumulate_defaults(const ExpertArgs &a, const ActiveList &act, double *sum,
                                      unsigned long long *cnt, hipStream_t st);
hipError_t launch_default_means(const double *sum, const unsigned long long *cnt, float *mean, int E, int H,
                                hipStream_t st);
bool b1_supported(int H, int dtype);
hipError_t launch_gateup_b1(const ExpertArgs &a, const ActiveList &act, int dtype, hipStream_t st);
hipError_t launch_down_combine_b1(const ExpertArgs &a, const ActiveList &act, int dtype, hipStream_t st);
hipError_t init_kernels();     // one-time function attributes (dynamic LDS limits)

size_t route_lds_bytes(int H, int B, int *tok_tile);

}  // namespace moe_spec
