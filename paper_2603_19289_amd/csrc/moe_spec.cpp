// Host side of the library: context, slot cache, stream/event ordering, C ABI.
//
// Ordering of one layer step (paper: Algorithm 1 and the wait-and-prefetch description in
// Sec. 5.1 "Implementation Details"; here with per-layer slot pools instead of two buffers):
//   compute stream: route(l) -> predict(l+1) -> [wait ready(l)] -> gate/up -> down -> combine
//   copy stream   : [wait done(l+1) of the previous token] -> H2D of the missing experts of
//                   layer l+1 -> record ready(l+1)
// The host learns expert ids through a pinned mailbox the routing kernels write; it needs them
// to decide which slots to fill.  done(l) is recorded after the last kernel that reads pool l, and
// every copy into pool l waits for it, so a slot is never overwritten while it is being read.
#include "../../include/moe_spec.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <deque>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "kernels.h"

using namespace moe_spec;

// Scratch of moe_spec_layer_step_static, the entry point for callers that cannot allocate device
// memory: one array per GPU, held by every GPU the library runs on until the process ends.  Host code
// never uses this name as an address: the device address is asked for once per device
// (static_scratch_of_current_device) and handed to the kernels like any other pointer.
static __device__ __align__(256) unsigned char scratch[MOE_SPEC_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
char *g_scratch_ptr[kMaxDevices];        // device address of `scratch` on each GPU, null until asked for

// Device address of the scratch array on the current device (looked up once per device).
hipError_t static_scratch_of_current_device(int *device, char **ptr) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = static_cast<char *>(p);
  }
  *device = dev;
  *ptr = g_scratch_ptr[dev];
  return hipSuccess;
}

thread_local std::string g_create_error;

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Pool {                       // one layer's slot cache (least recently used replacement)
  std::vector<int> slot_expert, slot_stamp, where;   // where[e] = slot or -1
  long clock = 0;
};

constexpr int kDmaQueues = 2;        // copy_engine 2: the caller's copy stream plus one more

struct TimedSpan { hipEvent_t a, b; int kind; };   // kind 0 compute, 1 copy, 2 stall, 3 expert FFN of one cache wave

struct ArenaLayout {
  size_t slots, s_buf, true_ids, true_gates, true_gates64, pend_ids[2], pend_gates[2],
      diag, zslots, zslots_end, la_ids, la_gates, h, y, bench_ids, s_q, sig, est_u, est_t, est_v, dacc_sum, dacc_cnt, dacc_end, tr_begin, tr_end, pf_s, pf_sq, pf_ids, pf_gates, pf_y, pf_hq, pf_pos, pf_count, total;
};

const char *validate(const moe_spec_config *c) {
  if (!c) return "config is null";
  if (c->n_layers < 1) return "n_layers must be >= 1";
  if (c->hidden < 8 || c->hidden % 8) return "hidden must be a positive multiple of 8";
  if (c->hidden > MOE_SPEC_MAX_HIDDEN) return "hidden exceeds MOE_SPEC_MAX_HIDDEN";
  if (c->inter < 8 || c->inter % 8) return "inter must be a positive multiple of 8";
  if (c->inter > 32768) return "inter exceeds 32768";
  if (c->n_experts < 1 || c->n_experts > MOE_SPEC_MAX_EXPERTS) return "n_experts out of range";
  if (c->top_k < 1 || c->top_k > MOE_SPEC_MAX_TOP_K || c->top_k > c->n_experts) return "top_k out of range";
  if (c->max_batch < 1 || c->max_batch > MOE_SPEC_MAX_BATCH) return "max_batch out of range";
  if (c->slots_per_layer < c->top_k) return "slots_per_layer must be at least top_k";
  if (c->slots_per_layer > 32767) return "slots_per_layer too large";
  if (c->dtype != MOE_SPEC_F32 && c->dtype != MOE_SPEC_BF16) return "unknown dtype";
  if (c->mode < MOE_SPEC_MODE_ON_DEMAND || c->mode > MOE_SPEC_MODE_PREFETCH_HINT) return "unknown mode";
  if (!(c->rms_eps >= 0.f)) return "rms_eps must be >= 0";
  if (c->copy_engine < MOE_SPEC_COPY_DMA || c->copy_engine > MOE_SPEC_COPY_DMA2) return "unknown copy_engine";
  if (c->predict_signal != 0 && c->predict_signal != 1) return "unknown predict_signal";
  if (c->est_latent < 0 || c->est_ffn < 0 || (c->est_latent == 0) != (c->est_ffn == 0)) return "estimator sizes must both be set or both be 0";
  if (c->est_latent % 8 || c->est_ffn % 8) return "estimator sizes must be multiples of 8";
  if (c->max_prefill_tokens < 0 || c->max_prefill_tokens > 32768) return "max_prefill_tokens out of range";
  if (c->wait_spin_limit < 0) return "wait_spin_limit must be >= 0";
  if (c->lookahead < 0 || c->lookahead > 2) return "lookahead must be 0, 1 or 2";
  if (c->lookahead == 2 && (c->diagnostics || c->predict_signal != 0))
    return "lookahead = 2 needs the router-based prediction (predict_signal = 0, diagnostics = 0)";
  if (c->est_latent > MOE_SPEC_MAX_HIDDEN || c->est_ffn > 8 * MOE_SPEC_MAX_HIDDEN) return "estimator sizes too large";
  return nullptr;
}

size_t expert_bytes_of(const moe_spec_config *c) {
  return size_t(3) * c->hidden * c->inter * (c->dtype == MOE_SPEC_BF16 ? 2 : 4);
}

ArenaLayout layout_of(const moe_spec_config *c) {
  ArenaLayout a{};
  const size_t B = c->max_batch, k = c->top_k, H = c->hidden, I = c->inter, E = c->n_experts;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t at = off; off = align_up(off + bytes, 256); return at; };
  a.slots = take(size_t(c->n_layers) * c->slots_per_layer * align_up(expert_bytes_of(c), 256));
  // state that lives from call to call
  for (int i = 0; i < 2; ++i) { a.pend_ids[i] = take(B * k * 4); a.pend_gates[i] = take(B * k * 4); }
  a.diag = take(size_t(c->n_layers) * sizeof(LayerDiag));
  a.bench_ids = take(256);
  // hand-over slots of the fused routing kernel: two sets each of true and predicted logits [B,E], all
  // ones when armed
  a.zslots = take(size_t(4) * B * E * 8);
  a.zslots_end = off;
  a.dacc_sum = take(c->accumulate_defaults ? size_t(c->n_layers) * E * H * 8 : 0);
  a.dacc_cnt = take(c->accumulate_defaults ? size_t(c->n_layers) * E * 8 : 0);
  a.dacc_end = off;
  // scratch of one decode layer step: written before it is read within the call.  This is the part
  // that moe_spec_layer_step_static keeps in the library's static array instead.
  a.tr_begin = off;
  a.s_buf = take(B * H * 4);
  a.true_ids = take(B * k * 4);
  a.true_gates = take(B * k * 4);
  a.true_gates64 = take(B * k * 8);
  a.la_ids = take(B * k * 4);
  a.la_gates = take(B * k * 4);
  a.h = take(B * k * I * 4);
  a.y = take(B * k * H * 4);
  a.s_q = take(B * H * 2);
  a.sig = take(B * H * 4);
  a.est_u = take(B * size_t(c->est_latent) * 8);
  a.est_t = take(B * size_t(c->est_ffn) * 8);
  a.est_v = take(B * size_t(c->est_latent) * 8);
  a.tr_end = off;
  const size_t P = size_t(c->max_prefill_tokens);
  a.pf_s = take(P * H * 4);
  a.pf_sq = take(P * H * 2);
  a.pf_ids = take(P * k * 4);
  a.pf_gates = take(P * k * 4);
  a.pf_y = take(P * k * H * 4);
  a.pf_hq = take(c->dtype == MOE_SPEC_BF16 ? P * k * I * 2 : 0);
  a.pf_pos = take(c->dtype == MOE_SPEC_BF16 ? E * P * 4 : 0);
  a.pf_count = take(c->dtype == MOE_SPEC_BF16 && P ? E * 4 : 0);
  a.total = off;
  return a;
}

}  // namespace

struct moe_spec_ctx {
  moe_spec_config cfg{};
  size_t expert_bytes = 0, slot_stride = 0;
  ArenaLayout lay{};
  char *arena = nullptr;
  int device = -1;                               // the device that was current at create
  char *static_scratch = nullptr;                // this device's copy of the library's scratch array
  bool use_static = false;                       // the running call keeps its step scratch there
  hipStream_t compute = nullptr, copy = nullptr;
  std::vector<hipStream_t> copy_aux;             // owned; further DMA queues of copy_engine 2
  std::vector<hipEvent_t> aux_done;
  hipEvent_t pf_ready[2] = {nullptr, nullptr}, pf_done[2] = {nullptr, nullptr};   // prefill: one pair per half pool

  std::vector<const void *> router_w, gain, dvecs;
  struct { const void *proj, *layer_emb, *ffn_in, *ffn_out, *head; const float *ln_gain, *ln_bias; float ln_eps; bool set; } est{};
  std::vector<char> est_use;                    // [L] predict with the estimator at this layer
  std::vector<const char *> host_expert;        // [L*E]
  std::vector<Pool> pools;
  std::vector<hipEvent_t> ready, done;
  std::vector<char> done_recorded, ready_recorded;
  Mailbox *mb_true = nullptr, *mb_next = nullptr, *mb_look = nullptr;       // pinned host
  Mailbox *mb_true_dev = nullptr, *mb_next_dev = nullptr, *mb_look_dev = nullptr;
  volatile unsigned int *wait_status = nullptr;         // pinned host word after the mailboxes: a kernel's bounded wait ran out
  unsigned int *wait_status_dev = nullptr;
  unsigned int spin_limit = 1u << 21;
  uint32_t route_parity = 0;                            // which set of logit slots the next fused routing launch uses

  // token state
  bool token_open = false;
  int next_layer = 0, batch = 0;
  bool have_pending = false;                    // a prediction for next_layer sits on the device
  std::vector<int> pending_union;               // sorted union of predicted ids (host copy)
  std::vector<int> pending_ids;                 // the predicted ids [B,k] in position order (host copy)
  ActiveList pending_wave0{};                   // slots of its first wave (already requested)
  std::vector<int> look_ids[3];                 // lookahead = 2: ids predicted for layer l two layers earlier, at [l % 3]

  // statistics
  moe_spec_stats_t st{};
  bool clock_running = false;
  std::chrono::steady_clock::time_point t0;
  std::deque<TimedSpan> spans;     // addresses stay valid while a span is open
  std::vector<hipEvent_t> free_events;

  std::string err;

  int fail(int code, const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    err = buf;
    return code;
  }
  int hip_fail(hipError_t e, const char *what) {
    return fail(MOE_SPEC_EHIP, "%s: %s", what, hipGetErrorString(e));
  }

  // Arena offset -> pointer.  The scratch of a decode layer step moves to the static array for a
  // call of moe_spec_layer_step_static.
  template <typename T> T *at(size_t off) const {
    if (use_static && off >= lay.tr_begin && off < lay.tr_end)
      return reinterpret_cast<T *>(static_scratch + (off - lay.tr_begin));
    return reinterpret_cast<T *>(arena + off);
  }
  char *pool_base(int layer) const {
    return arena + lay.slots + size_t(layer) * cfg.slots_per_layer * slot_stride;
  }

  hipEvent_t timing_event() {
    if (!free_events.empty()) { hipEvent_t e = free_events.back(); free_events.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
  // record (a) now, return span whose (b) the caller records later
  TimedSpan *open_span(int kind, hipStream_t s) {
    if (!cfg.profile) return nullptr;
    TimedSpan sp{timing_event(), timing_event(), kind};
    if (!sp.a || !sp.b) return nullptr;
    (void)hipEventRecord(sp.a, s);
    spans.push_back(sp);
    return &spans.back();
  }
  void close_span(TimedSpan *sp, hipStream_t s) { if (sp) (void)hipEventRecord(sp->b, s); }
  int resolve_spans() {
    if (spans.empty()) return MOE_SPEC_OK;
    hipError_t e = sync_streams();
    if (e != hipSuccess) return hip_fail(e, "synchronize for timing");
    for (auto &sp : spans) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, sp.a, sp.b) == hipSuccess) {
        if (sp.kind == 0) st.compute_ms += ms;
        else if (sp.kind == 1) st.copy_ms += ms;
        else if (sp.kind == 2) st.stall_ms += ms;
        else { st.expert_ms += ms; st.expert_launches += 1; }
      }
      free_events.push_back(sp.a);
      free_events.push_back(sp.b);
    }
    spans.clear();
    return MOE_SPEC_OK;
  }

  // The routing kernels overwrite id words that the host armed with -1 (arm_ids): spin until all n are there.
  // Bounded; also notices a failed stream.
  int wait_ids(const Mailbox *mb, int n) {
    const volatile int32_t *ids = mb->ids;
    auto start = std::chrono::steady_clock::now();
    unsigned long spins = 0;
    for (int i = 0; i < n; ++i) {
      while (ids[i] == -1) {
        __builtin_ia32_pause();
        if ((++spins & 0xfffff) == 0) {
          hipError_t q = hipStreamQuery(compute);
          if (q != hipSuccess && q != hipErrorNotReady) return hip_fail(q, "compute stream failed while routing");
          if (q == hipSuccess && ids[i] == -1)
            return fail(MOE_SPEC_EHIP, "routing kernel finished without posting expert ids");
          if (std::chrono::steady_clock::now() - start > std::chrono::seconds(30))
            return fail(MOE_SPEC_EHIP, "timed out waiting for expert ids from the routing kernel");
        }
      }
    }
    __atomic_thread_fence(__ATOMIC_ACQUIRE);
    return MOE_SPEC_OK;
  }

  // One expert block host -> device by the configured engine; `index` counts the blocks of the
  // current group (it picks the queue).  copy_join ends the group: afterwards everything issued is
  // ordered before whatever is recorded next on the copy stream.
  int copy_expert(CopyList &cl, int index, char *dst, const char *src) {
    if (cfg.copy_engine == MOE_SPEC_COPY_KERNEL) {
      cl.src[cl.n] = src;
      cl.dst[cl.n] = dst;
      if (++cl.n == kCopyListMax) {
        hipError_t c = launch_gather_copy(cl, copy);
        if (c != hipSuccess) return hip_fail(c, "host-to-device gather copy");
        cl.n = 0;
      }
    } else if (cfg.copy_engine == MOE_SPEC_COPY_DMA2) {
      // whole experts, dealt round-robin over the queues (cutting every expert into one part per
      // queue moved no more bytes per second and made the timing erratic)
      const size_t q = size_t(index) % (1 + copy_aux.size());
      hipError_t c = hipMemcpyAsync(dst, src, expert_bytes, hipMemcpyHostToDevice, q == 0 ? copy : copy_aux[q - 1]);
      if (c != hipSuccess) return hip_fail(c, "host-to-device expert copy");
    } else {
      hipError_t c = hipMemcpyAsync(dst, src, expert_bytes, hipMemcpyHostToDevice, copy);
      if (c != hipSuccess) return hip_fail(c, "host-to-device expert copy");
    }
    return MOE_SPEC_OK;
  }
  int copy_join(CopyList &cl) {
    if (cl.n > 0) {
      hipError_t c = launch_gather_copy(cl, copy);
      if (c != hipSuccess) return hip_fail(c, "host-to-device gather copy");
      cl.n = 0;
    }
    for (size_t q = 0; q < copy_aux.size(); ++q) {
      hipError_t r = hipEventRecord(aux_done[q], copy_aux[q]);
      if (r == hipSuccess) r = hipStreamWaitEvent(copy, aux_done[q], 0);
      if (r != hipSuccess) return hip_fail(r, "join copy queues");
    }
    return MOE_SPEC_OK;
  }
  // Host waits for the compute stream and every copy queue.
  hipError_t sync_streams() {
    hipError_t e = hipStreamSynchronize(compute);
    if (e == hipSuccess) e = hipStreamSynchronize(copy);
    for (hipStream_t q : copy_aux) if (e == hipSuccess) e = hipStreamSynchronize(q);
    return e;
  }
  // Every copy queue waits for an event recorded on the compute stream.
  int copy_queues_wait(hipEvent_t ev) {
    hipError_t w = hipStreamWaitEvent(copy, ev, 0);
    for (hipStream_t q : copy_aux) if (w == hipSuccess) w = hipStreamWaitEvent(q, ev, 0);
    return w == hipSuccess ? MOE_SPEC_OK : hip_fail(w, "copy stream wait");
  }

  // Cache request for at most S experts (ascending ids): hits are stamped, each miss takes the
  // least recently used slot that holds no requested expert and is copied in on the copy stream.
  // Fills act with (expert, slot) of every requested expert.  Returns the number of copies issued.
  int request(int layer, const std::vector<int> &experts, ActiveList *act, int *n_copies) {
    Pool &p = pools[layer];
    const int S = cfg.slots_per_layer;
    std::vector<char> in_q(cfg.n_experts, 0);
    for (int e : experts) in_q[e] = 1;
    act->n = 0;
    int copies = 0;
    TimedSpan *span = nullptr;
    CopyList cl{};
    cl.n16 = uint32_t(expert_bytes / 16);
    for (int e : experts)                        // refuse before any state changes
      if (p.where[e] < 0 && !host_expert[size_t(layer) * cfg.n_experts + e])
        return fail(MOE_SPEC_ESTATE, "expert %d of layer %d was never registered", e, layer);
    p.clock += 1;
    for (int e : experts) {
      if (p.where[e] >= 0) { p.slot_stamp[p.where[e]] = int(p.clock); st.cache_hits += 1; }
    }
    for (int e : experts) {
      if (p.where[e] >= 0) continue;
      int victim = -1;
      for (int s = 0; s < S; ++s) {
        const int held = p.slot_expert[s];
        if (held >= 0 && in_q[held]) continue;
        if (victim < 0 || p.slot_stamp[s] < p.slot_stamp[victim]) victim = s;
      }
      if (victim < 0) return fail(MOE_SPEC_ESTATE, "no evictable slot (request larger than the pool)");
      const char *src = host_expert[size_t(layer) * cfg.n_experts + e];
      if (copies == 0) {
        if (done_recorded[layer]) {
          hipError_t w = hipStreamWaitEvent(copy, done[layer], 0);
          for (hipStream_t q : copy_aux) if (w == hipSuccess) w = hipStreamWaitEvent(q, done[layer], 0);
          if (w != hipSuccess) return hip_fail(w, "copy stream wait");
        }
        if (ready_recorded[layer]) {
          // further queues: also behind the previous request on this pool (its slots may be reused
          // by this one before any kernel ran, e.g. a true request right after a mispredicted prefetch)
          for (hipStream_t q : copy_aux) {
            hipError_t w = hipStreamWaitEvent(q, ready[layer], 0);
            if (w != hipSuccess) return hip_fail(w, "copy queue wait");
          }
        }
        span = open_span(1, copy);
      }
      if (p.slot_expert[victim] >= 0) p.where[p.slot_expert[victim]] = -1;
      p.slot_expert[victim] = e;
      p.slot_stamp[victim] = int(p.clock);
      p.where[e] = victim;
      char *dst = pool_base(layer) + size_t(victim) * slot_stride;
      if (int rc = copy_expert(cl, copies, dst, src)) return rc;
      copies += 1;
      st.cache_misses += 1;
      st.h2d_bytes += int64_t(expert_bytes);
    }
    if (copies > 0) {                            // the request is complete when every queue is
      if (int rc = copy_join(cl)) return rc;
    }
    if (copies > 0) {
      close_span(span, copy);
      hipError_t r = hipEventRecord(ready[layer], copy);
      if (r != hipSuccess) return hip_fail(r, "record ready event");
      ready_recorded[layer] = 1;
    }
    for (int e : experts) {
      act->expert[act->n] = int16_t(e);
      act->slot[act->n] = int16_t(p.where[e]);
      act->n += 1;
    }
    *n_copies = copies;
    return MOE_SPEC_OK;
  }

  // Expert ids handed over by a routing kernel index host tables: refuse anything outside [0, E).
  int check_ids(const int32_t *ids, int n) {
    for (int i = 0; i < n; ++i)
      if (ids[i] < 0 || ids[i] >= cfg.n_experts)
        return fail(MOE_SPEC_EHIP, "the routing kernel handed over expert id %d (position %d), outside [0, %d)",
                    ids[i], i, cfg.n_experts);
    return MOE_SPEC_OK;
  }

  // Hand-over slots, their bound and the status word of one launch of the one-routing kernel; the launch uses
  // the current set of logit slots and arms both sets of the other parity, like the fused kernel.
  void prep_route(RouteArgs &ra) {
    ra.slots = zslot_set(0, route_parity);
    ra.arm_a = zslot_set(0, route_parity ^ 1);
    ra.arm_b = zslot_set(1, route_parity ^ 1);
    ra.arm_count = cfg.max_batch * cfg.n_experts;
    ra.spin_limit = spin_limit;
    ra.status = wait_status_dev;
    route_parity ^= 1;
  }
  static void arm_ids(Mailbox *mb, int n) {
    std::memset(mb->ids, 0xff, size_t(n) * 4);
    __atomic_thread_fence(__ATOMIC_RELEASE);
  }

  // A waiter inside a fused kernel gave up: its results are not to be trusted, and the hand-over slots are
  // in an unknown state until moe_spec_reset re-arms them.
  int check_waits() {
    if (wait_status && *wait_status)
      return fail(MOE_SPEC_EHIP, "a kernel's bounded wait for another workgroup's result ran out; results since the "
                  "last successful moe_spec_stats are invalid (moe_spec_reset re-arms the context)");
    return MOE_SPEC_OK;
  }
  hipError_t arm_handover_slots() {
    hipError_t e = hipMemsetAsync(arena + lay.zslots, 0xff, lay.zslots_end - lay.zslots, compute);
    route_parity = 0;
    if (wait_status) *wait_status = 0;
    return e;
  }
  unsigned long long *zslot_set(int which /*0 true, 1 predicted*/, uint32_t parity) const {
    return at<unsigned long long>(lay.zslots) + (size_t(which) * 2 + parity) * cfg.max_batch * cfg.n_experts;
  }

  static std::vector<int> sorted_union(const int32_t *ids, int n) {
    std::vector<int> u(ids, ids + n);
    std::sort(u.begin(), u.end());
    u.erase(std::unique(u.begin(), u.end()), u.end());
    return u;
  }
};

extern "C" {

size_t moe_spec_expert_bytes(const moe_spec_config *cfg) {
  if (validate(cfg)) return 0;
  return expert_bytes_of(cfg);
}

size_t moe_spec_arena_bytes(const moe_spec_config *cfg) {
  if (validate(cfg)) return 0;
  return layout_of(cfg).total;
}

const char *moe_spec_last_error(const moe_spec_ctx *ctx) {
  return ctx ? ctx->err.c_str() : g_create_error.c_str();
}

int moe_spec_create(const moe_spec_config *cfg, moe_spec_ctx **out) {
  if (!out) { g_create_error = "out is null"; return MOE_SPEC_EINVAL; }
  if (const char *why = validate(cfg)) { g_create_error = why; return MOE_SPEC_EINVAL; }
  const ArenaLayout lay = layout_of(cfg);
  if (!cfg->device_arena || (reinterpret_cast<uintptr_t>(cfg->device_arena) & 255)) {
    g_create_error = "device_arena must be a 256-byte aligned device pointer";
    return MOE_SPEC_EINVAL;
  }
  if (cfg->device_arena_bytes < lay.total) {
    g_create_error = "device_arena_bytes is smaller than moe_spec_arena_bytes(cfg)";
    return MOE_SPEC_EINVAL;
  }
  int n_dev = 0;
  hipError_t e = hipGetDeviceCount(&n_dev);
  if (e != hipSuccess || n_dev < 1) {
    g_create_error = std::string("no usable GPU: ") + (e != hipSuccess ? hipGetErrorString(e) : "device count is 0");
    return MOE_SPEC_EHIP;
  }
  moe_spec_ctx *c = new (std::nothrow) moe_spec_ctx;
  if (!c) { g_create_error = "out of host memory"; return MOE_SPEC_ENOMEM; }
  c->cfg = *cfg;
  c->lay = lay;
  c->expert_bytes = expert_bytes_of(cfg);
  c->slot_stride = align_up(c->expert_bytes, 256);
  c->arena = static_cast<char *>(cfg->device_arena);
  c->compute = static_cast<hipStream_t>(cfg->compute_stream);
  c->copy = static_cast<hipStream_t>(cfg->copy_stream);
  const int L = cfg->n_layers, E = cfg->n_experts, S = cfg->slots_per_layer;
  c->router_w.assign(L, nullptr);
  c->gain.assign(L, nullptr);
  c->dvecs.assign(L, nullptr);
  c->host_expert.assign(size_t(L) * E, nullptr);
  c->pools.resize(L);
  for (auto &p : c->pools) { p.slot_expert.assign(S, -1); p.slot_stamp.assign(S, -1); p.where.assign(E, -1); }
  c->done_recorded.assign(L, 0);
  c->ready_recorded.assign(L, 0);

  auto bail = [&](hipError_t err, const char *what) {
    g_create_error = std::string(what) + ": " + hipGetErrorString(err);
    moe_spec_destroy(c);
    return MOE_SPEC_EHIP;
  };
  if ((e = init_kernels()) != hipSuccess) return bail(e, "kernel attributes");
  if ((e = static_scratch_of_current_device(&c->device, &c->static_scratch)) != hipSuccess)
    return bail(e, "address of the static scratch array");
  c->ready.assign(L, nullptr);
  c->done.assign(L, nullptr);
  for (int l = 0; l < L; ++l) {
    if ((e = hipEventCreateWithFlags(&c->ready[l], hipEventDisableTiming)) != hipSuccess) return bail(e, "event");
    if ((e = hipEventCreateWithFlags(&c->done[l], hipEventDisableTiming)) != hipSuccess) return bail(e, "event");
  }
  for (int h = 0; h < 2 && cfg->max_prefill_tokens > 0; ++h) {
    if ((e = hipEventCreateWithFlags(&c->pf_ready[h], hipEventDisableTiming)) != hipSuccess) return bail(e, "event");
    if ((e = hipEventCreateWithFlags(&c->pf_done[h], hipEventDisableTiming)) != hipSuccess) return bail(e, "event");
  }
  if (cfg->copy_engine == MOE_SPEC_COPY_DMA2) {
    for (int q = 1; q < kDmaQueues; ++q) {
      hipStream_t sq = nullptr;
      hipEvent_t ev = nullptr;
      if ((e = hipStreamCreateWithFlags(&sq, hipStreamNonBlocking)) != hipSuccess) return bail(e, "auxiliary copy stream");
      c->copy_aux.push_back(sq);
      if ((e = hipEventCreateWithFlags(&ev, hipEventDisableTiming)) != hipSuccess) return bail(e, "event");
      c->aux_done.push_back(ev);
    }
  }
  void *mb = nullptr;
  // fine-grained (coherent) pinned memory: device stores become visible to the spinning host
  if ((e = hipHostMalloc(&mb, 3 * sizeof(Mailbox) + 64, hipHostMallocMapped | hipHostMallocCoherent)) != hipSuccess)
    return bail(e, "pinned mailbox");
  std::memset(mb, 0, 3 * sizeof(Mailbox) + 64);
  c->mb_true = static_cast<Mailbox *>(mb);
  c->mb_next = c->mb_true + 1;
  void *mb_dev = nullptr;
  if ((e = hipHostGetDevicePointer(&mb_dev, mb, 0)) != hipSuccess) return bail(e, "mailbox device pointer");
  c->mb_true_dev = static_cast<Mailbox *>(mb_dev);
  c->mb_next_dev = c->mb_true_dev + 1;
  c->mb_look = c->mb_true + 2;
  c->mb_look_dev = c->mb_true_dev + 2;
  c->wait_status = reinterpret_cast<volatile unsigned int *>(c->mb_true + 3);
  c->wait_status_dev = reinterpret_cast<unsigned int *>(c->mb_true_dev + 3);
  if (cfg->wait_spin_limit > 0) c->spin_limit = unsigned(cfg->wait_spin_limit);
  if ((e = c->arm_handover_slots()) != hipSuccess) return bail(e, "arm hand-over slots");
  // counters start at zero
  if ((e = hipMemsetAsync(c->arena + lay.diag, 0, size_t(L) * sizeof(LayerDiag), c->compute)) != hipSuccess) return bail(e, "clear counters");
  if (cfg->accumulate_defaults) {
    if ((e = hipMemsetAsync(c->arena + lay.dacc_sum, 0, lay.dacc_end - lay.dacc_sum, c->compute)) != hipSuccess) return bail(e, "clear sums");
  }
  if ((e = hipStreamSynchronize(c->compute)) != hipSuccess) return bail(e, "synchronize");
  *out = c;
  return MOE_SPEC_OK;
}

void moe_spec_destroy(moe_spec_ctx *c) {
  if (!c) return;
  if (c->compute || c->copy || c->mb_true) {
    (void)hipStreamSynchronize(c->compute);
    (void)hipStreamSynchronize(c->copy);
    for (hipStream_t q : c->copy_aux) (void)hipStreamSynchronize(q);
  }
  for (hipStream_t q : c->copy_aux) (void)hipStreamDestroy(q);
  for (hipEvent_t ev : c->aux_done) (void)hipEventDestroy(ev);
  for (int h = 0; h < 2; ++h) {
    if (c->pf_ready[h]) (void)hipEventDestroy(c->pf_ready[h]);
    if (c->pf_done[h]) (void)hipEventDestroy(c->pf_done[h]);
  }
  for (auto ev : c->ready) if (ev) (void)hipEventDestroy(ev);
  for (auto ev : c->done) if (ev) (void)hipEventDestroy(ev);
  for (auto &sp : c->spans) { (void)hipEventDestroy(sp.a); (void)hipEventDestroy(sp.b); }
  for (auto ev : c->free_events) (void)hipEventDestroy(ev);
  if (c->mb_true) (void)hipHostFree(c->mb_true);
  delete c;
}

int moe_spec_set_layer_resident(moe_spec_ctx *c, int layer, const void *router_w, const void *rms_gain,
                                const void *default_vecs) {
  if (!c) return MOE_SPEC_EINVAL;
  if (layer < 0 || layer >= c->cfg.n_layers) return c->fail(MOE_SPEC_EINVAL, "layer %d out of range", layer);
  if (!router_w || !rms_gain || !default_vecs) return c->fail(MOE_SPEC_EINVAL, "null table pointer");
  if ((reinterpret_cast<uintptr_t>(router_w) | reinterpret_cast<uintptr_t>(default_vecs) |
       reinterpret_cast<uintptr_t>(rms_gain)) & 15)
    return c->fail(MOE_SPEC_EINVAL, "tables must be 16-byte aligned");
  c->router_w[layer] = router_w;
  c->gain[layer] = rms_gain;
  c->dvecs[layer] = default_vecs;
  return MOE_SPEC_OK;
}

int moe_spec_load_host_experts(moe_spec_ctx *c, int layer, int first_expert, int n_experts,
                               const void *pinned_host, size_t bytes) {
  if (!c) return MOE_SPEC_EINVAL;
  if (layer < 0 || layer >= c->cfg.n_layers) return c->fail(MOE_SPEC_EINVAL, "layer %d out of range", layer);
  if (first_expert < 0 || n_experts < 1 || first_expert + n_experts > c->cfg.n_experts)
    return c->fail(MOE_SPEC_EINVAL, "expert range [%d, %d) out of range", first_expert, first_expert + n_experts);
  if (!pinned_host) return c->fail(MOE_SPEC_EINVAL, "host pointer is null");
  if (bytes != size_t(n_experts) * c->expert_bytes)
    return c->fail(MOE_SPEC_EINVAL, "bytes must be n_experts * %zu", c->expert_bytes);
  hipPointerAttribute_t attr;
  hipError_t e = hipPointerGetAttributes(&attr, pinned_host);
  if (e != hipSuccess || attr.type != hipMemoryTypeHost) {
    (void)hipGetLastError();
    return c->fail(MOE_SPEC_EINVAL, "host pool must be page-locked (pinned) host memory");
  }
  const char *base = static_cast<const char *>(pinned_host);
  if (c->cfg.copy_engine == MOE_SPEC_COPY_KERNEL) {     // the address the copy kernel reads the pool at
    void *dev_view = nullptr;
    e = hipHostGetDevicePointer(&dev_view, const_cast<void *>(pinned_host), 0);
    if (e != hipSuccess || !dev_view) {
      (void)hipGetLastError();
      return c->fail(MOE_SPEC_EINVAL, "host pool is not mapped into the device address space");
    }
    base = static_cast<const char *>(dev_view);
  }
  for (int i = 0; i < n_experts; ++i)
    c->host_expert[size_t(layer) * c->cfg.n_experts + first_expert + i] = base + size_t(i) * c->expert_bytes;
  return MOE_SPEC_OK;
}

int moe_spec_set_estimator(moe_spec_ctx *c, const void *proj, const void *layer_emb, const void *ffn_in,
                           const void *ffn_out, const float *ln_gain, const float *ln_bias, const void *head,
                           float ln_eps) {
  if (!c) return MOE_SPEC_EINVAL;
  if (c->cfg.est_latent == 0) return c->fail(MOE_SPEC_ESTATE, "the configuration names no estimator sizes");
  if (!proj || !layer_emb || !ffn_in || !ffn_out || !ln_gain || !ln_bias || !head)
    return c->fail(MOE_SPEC_EINVAL, "null estimator pointer");
  const uintptr_t all = reinterpret_cast<uintptr_t>(proj) | reinterpret_cast<uintptr_t>(layer_emb) |
                        reinterpret_cast<uintptr_t>(ffn_in) | reinterpret_cast<uintptr_t>(ffn_out) |
                        reinterpret_cast<uintptr_t>(head);
  if (all & 15) return c->fail(MOE_SPEC_EINVAL, "estimator matrices must be 16-byte aligned");
  if (!(ln_eps >= 0.f)) return c->fail(MOE_SPEC_EINVAL, "ln_eps must be >= 0");
  c->est.proj = proj; c->est.layer_emb = layer_emb; c->est.ffn_in = ffn_in; c->est.ffn_out = ffn_out;
  c->est.head = head; c->est.ln_gain = ln_gain; c->est.ln_bias = ln_bias; c->est.ln_eps = ln_eps;
  c->est.set = true;
  return MOE_SPEC_OK;
}

int moe_spec_set_estimator_layers(moe_spec_ctx *c, const uint8_t *use, int n_layers) {
  if (!c) return MOE_SPEC_EINVAL;
  if (!use || n_layers != c->cfg.n_layers) return c->fail(MOE_SPEC_EINVAL, "need one flag per layer");
  if (!c->est.set) return c->fail(MOE_SPEC_ESTATE, "set the estimator's weights first");
  c->est_use.assign(use, use + n_layers);
  return MOE_SPEC_OK;
}

int moe_spec_begin_token(moe_spec_ctx *c) {
  if (!c) return MOE_SPEC_EINVAL;
  if (c->cfg.profile) { int rc = c->resolve_spans(); if (rc) return rc; }
  if (!c->clock_running) { c->clock_running = true; c->t0 = std::chrono::steady_clock::now(); }
  c->token_open = true;
  c->next_layer = 0;
  c->batch = 0;
  c->have_pending = false;
  c->pending_union.clear();
  for (auto &v : c->look_ids) v.clear();
  c->st.tokens += 1;
  return MOE_SPEC_OK;
}

}  // extern "C"

namespace {

int layer_step_impl(moe_spec_ctx *c, int layer, const void *r_dev, int batch, void *out_dev,
                    const moe_spec_step_outputs *outs) {
  const moe_spec_config &cfg = c->cfg;
  if (!r_dev || !out_dev) return c->fail(MOE_SPEC_EINVAL, "null activation pointer");
  if (batch < 1 || batch > cfg.max_batch) return c->fail(MOE_SPEC_EINVAL, "batch %d out of range", batch);
  if (!c->token_open) return c->fail(MOE_SPEC_ESTATE, "layer_step before begin_token");
  if (layer != c->next_layer) return c->fail(MOE_SPEC_ESTATE, "expected layer %d, got %d", c->next_layer, layer);
  if (layer > 0 && batch != c->batch) return c->fail(MOE_SPEC_ESTATE, "batch changed inside a token");
  const int L = cfg.n_layers, E = cfg.n_experts, k = cfg.top_k, H = cfg.hidden, I = cfg.inter, S = cfg.slots_per_layer;
  const bool last = layer == L - 1;
  if (!c->router_w[layer] || (!last && !c->router_w[layer + 1]))
    return c->fail(MOE_SPEC_ESTATE, "resident tables of layer %d (or %d) were never set", layer, layer + 1);
  const bool spec_mode = cfg.mode == MOE_SPEC_MODE_SPECULATIVE;
  const bool hint_mode = cfg.mode == MOE_SPEC_MODE_PREFETCH_HINT;
  const bool prefetching = spec_mode || hint_mode;
  const bool do_pred = !last && (prefetching || cfg.predict_in_on_demand);
  const bool exec_pred = spec_mode && c->have_pending;
  const bool hinted = hint_mode && c->have_pending;      // a prefetch for this layer may be in flight
  const size_t wbytes = cfg.dtype == MOE_SPEC_BF16 ? 2 : 4;
  hipError_t e;

  if (int rc = c->check_waits()) return rc;
  TimedSpan *sp_route = c->open_span(0, c->compute);

  const bool use_est = do_pred && c->est.set && !c->est_use.empty() && c->est_use[layer];
  // One launch for the true routing and the prediction, unless the prediction comes from the estimator or
  // from the baseline signal, or the per-layer figures' extra statistics are collected (those keep the
  // one-kernel-per-routing path below).
  const bool fused_route = !cfg.diagnostics && route_pair_supported(H, cfg.dtype) &&
                           !(do_pred && (use_est || cfg.predict_signal == 1));
  // lookahead = 2: a second prediction, for layer l+2, from the same quasi-hidden vector
  const bool look2 = cfg.lookahead == 2 && prefetching && do_pred && layer + 2 < L;
  if (cfg.lookahead == 2 && prefetching && !fused_route)
    return c->fail(MOE_SPEC_ESTATE, "lookahead = 2 needs the router-based prediction at every layer (no estimator layers)");
  if (look2 && !c->router_w[layer + 2]) return c->fail(MOE_SPEC_ESTATE, "resident tables of layer %d were never set", layer + 2);
  const bool score_look = cfg.lookahead == 2 && !c->look_ids[layer % 3].empty();
  const bool true_ids_to_host = !exec_pred || score_look;
  if (fused_route) {
    RoutePairArgs pa{};
    pa.r = static_cast<const float *>(r_dev);
    pa.w_true = c->router_w[layer];
    pa.gain_true = static_cast<const float *>(c->gain[layer]);
    if (do_pred) {
      pa.w_next = c->router_w[layer + 1];
      pa.gain_next = static_cast<const float *>(c->gain[layer + 1]);
      pa.dvec = c->dvecs[layer];
    }
    pa.z_true = c->zslot_set(0, c->route_parity);
    pa.z_pred = c->zslot_set(1, c->route_parity);
    pa.z_true_next = c->zslot_set(0, c->route_parity ^ 1);
    pa.z_pred_next = c->zslot_set(1, c->route_parity ^ 1);
    pa.arm_count = cfg.max_batch * E;
    c->route_parity ^= 1;
    pa.s_out = c->at<float>(c->lay.s_buf);
    pa.s_out_q = cfg.dtype == MOE_SPEC_BF16 && batch >= kMfmaMinBatch ? c->at<uint16_t>(c->lay.s_q) : nullptr;
    pa.true_ids = c->at<int32_t>(c->lay.true_ids);
    pa.true_gates = c->at<float>(c->lay.true_gates);
    pa.true_gates64 = look2 ? c->at<double>(c->lay.true_gates64) : nullptr;
    pa.next_ids = c->at<int32_t>(c->lay.pend_ids[(layer + 1) & 1]);
    pa.next_gates = c->at<float>(c->lay.pend_gates[(layer + 1) & 1]);
    pa.cmp_ids = c->have_pending ? c->at<int32_t>(c->lay.pend_ids[layer & 1]) : nullptr;
    pa.diag = c->at<LayerDiag>(c->lay.diag) + layer;
    if (outs) {
      pa.user_true_ids = outs->true_ids; pa.user_true_gates = outs->true_gates;
      pa.user_next_ids = outs->next_ids; pa.user_next_gates = outs->next_gates;
    }
    // the host arms the id words it will wait for; the kernel's workgroups overwrite them
    if (true_ids_to_host) { pa.mb_true = c->mb_true_dev; moe_spec_ctx::arm_ids(c->mb_true, batch * k); }
    if (do_pred && prefetching) { pa.mb_next = c->mb_next_dev; moe_spec_ctx::arm_ids(c->mb_next, batch * k); }
    pa.status = c->wait_status_dev;
    pa.B = batch; pa.H = H; pa.E = E; pa.k = k;
    pa.eps = cfg.rms_eps;
    pa.bf16 = cfg.dtype == MOE_SPEC_BF16;
    pa.from_normalized = cfg.q_from_normalized;
    pa.spin_limit = c->spin_limit;
    if ((e = launch_route_pair(pa, cfg.dtype, c->compute)) != hipSuccess) return c->hip_fail(e, "routing kernel");
    c->st.hbm_bytes_algorithmic += int64_t(E) * H * wbytes;
    if (do_pred) c->st.hbm_bytes_algorithmic += int64_t(E) * H * wbytes + int64_t(batch) * k * H * wbytes;
    if (look2) {
      // the same quasi-hidden vector under layer l+2's norm and router: one more launch of the one-routing kernel
      RouteArgs la{};
      la.r = static_cast<const float *>(r_dev);
      la.s_in = c->at<float>(c->lay.s_buf);
      la.w = c->router_w[layer + 2];
      la.gain = static_cast<const float *>(c->gain[layer + 2]);
      la.dvec = c->dvecs[layer];
      la.d_ids = c->at<int32_t>(c->lay.true_ids);
      la.d_gates = c->at<double>(c->lay.true_gates64);
      la.ids_out = c->at<int32_t>(c->lay.la_ids);
      la.gates_out = c->at<float>(c->lay.la_gates);
      la.diag = c->at<LayerDiag>(c->lay.diag) + layer;
      la.mailbox = c->mb_look_dev;
      moe_spec_ctx::arm_ids(c->mb_look, batch * k);
      la.B = batch; la.H = H; la.E = E; la.k = k;
      la.eps = cfg.rms_eps;
      la.bf16 = cfg.dtype == MOE_SPEC_BF16;
      la.spec = 1;
      la.from_normalized = cfg.q_from_normalized;
      c->prep_route(la);
      if ((e = launch_route(la, cfg.dtype, c->compute)) != hipSuccess) return c->hip_fail(e, "lookahead routing kernel");
      c->st.hbm_bytes_algorithmic += int64_t(E) * H * wbytes + int64_t(batch) * k * H * wbytes;
    }
  } else {
  // --- true routing of layer l (and scoring of the prediction made at l-1)
  RouteArgs ra{};
  ra.r = static_cast<const float *>(r_dev);
  ra.w = c->router_w[layer];
  ra.gain = static_cast<const float *>(c->gain[layer]);
  ra.vec_out = c->at<float>(c->lay.s_buf);
  ra.vec_out_q = cfg.dtype == MOE_SPEC_BF16 && batch >= kMfmaMinBatch ? c->at<uint16_t>(c->lay.s_q) : nullptr;
  ra.ids_out = c->at<int32_t>(c->lay.true_ids);
  ra.gates_out = c->at<float>(c->lay.true_gates);
  ra.gates64_out = c->at<double>(c->lay.true_gates64);
  ra.cmp_ids = c->have_pending ? c->at<int32_t>(c->lay.pend_ids[layer & 1]) : nullptr;
  ra.diag = c->at<LayerDiag>(c->lay.diag) + layer;
  ra.rank_stats = cfg.diagnostics;
  ra.prev_signal = cfg.diagnostics && c->have_pending ? c->at<float>(c->lay.sig) : nullptr;
  ra.user_ids = outs ? outs->true_ids : nullptr;
  ra.user_gates = outs ? outs->true_gates : nullptr;
  ra.mailbox = true_ids_to_host ? c->mb_true_dev : nullptr;
  if (ra.mailbox) moe_spec_ctx::arm_ids(c->mb_true, batch * k);
  ra.B = batch; ra.H = H; ra.E = E; ra.k = k;
  ra.eps = cfg.rms_eps;
  ra.bf16 = cfg.dtype == MOE_SPEC_BF16;
  ra.spec = 0;
  if (!cfg.diagnostics && route_pair_supported(H, cfg.dtype)) {
    // the fused kernel, asked for the true routing only (it is the faster of the two at that); the prediction
    // below comes from the estimator or the baseline signal and keeps its own launches
    RoutePairArgs ta{};
    ta.r = ra.r;
    ta.w_true = ra.w;
    ta.gain_true = ra.gain;
    ta.z_true = c->zslot_set(0, c->route_parity);
    ta.z_pred = c->zslot_set(1, c->route_parity);
    ta.z_true_next = c->zslot_set(0, c->route_parity ^ 1);
    ta.z_pred_next = c->zslot_set(1, c->route_parity ^ 1);
    ta.arm_count = cfg.max_batch * E;
    c->route_parity ^= 1;
    ta.s_out = ra.vec_out;
    ta.s_out_q = ra.vec_out_q;
    ta.true_ids = ra.ids_out;
    ta.true_gates = ra.gates_out;
    ta.true_gates64 = ra.gates64_out;
    ta.cmp_ids = ra.cmp_ids;
    ta.diag = ra.diag;
    ta.user_true_ids = ra.user_ids;
    ta.user_true_gates = ra.user_gates;
    ta.mb_true = ra.mailbox;
    ta.status = c->wait_status_dev;
    ta.B = batch; ta.H = H; ta.E = E; ta.k = k;
    ta.eps = cfg.rms_eps;
    ta.bf16 = ra.bf16;
    ta.spin_limit = c->spin_limit;
    if ((e = launch_route_pair(ta, cfg.dtype, c->compute)) != hipSuccess) return c->hip_fail(e, "routing kernel");
  } else {
    c->prep_route(ra);
    if ((e = launch_route(ra, cfg.dtype, c->compute)) != hipSuccess) return c->hip_fail(e, "routing kernel");
  }
  c->st.hbm_bytes_algorithmic += int64_t(E) * H * wbytes;

  // --- prediction for layer l+1 from the quasi-hidden state
  if (do_pred) {
    RouteArgs pa = ra;
    pa.s_in = c->at<float>(c->lay.s_buf);
    pa.w = c->router_w[layer + 1];
    pa.gain = static_cast<const float *>(c->gain[layer + 1]);
    pa.dvec = c->dvecs[layer];
    pa.d_ids = c->at<int32_t>(c->lay.true_ids);
    pa.d_gates = c->at<double>(c->lay.true_gates64);
    pa.vec_out = cfg.diagnostics ? c->at<float>(c->lay.sig) : nullptr;
    pa.vec_out_q = nullptr;
    pa.prev_signal = nullptr;
    pa.ids_out = c->at<int32_t>(c->lay.pend_ids[(layer + 1) & 1]);
    pa.gates_out = c->at<float>(c->lay.pend_gates[(layer + 1) & 1]);
    pa.gates64_out = nullptr;
    pa.cmp_ids = nullptr;
    pa.user_ids = outs ? outs->next_ids : nullptr;
    pa.user_gates = outs ? outs->next_gates : nullptr;
    pa.mailbox = prefetching ? c->mb_next_dev : nullptr;
    if (pa.mailbox) moe_spec_ctx::arm_ids(c->mb_next, batch * k);
    pa.spec = cfg.predict_signal == 1 ? 2 : 1;
    pa.from_normalized = cfg.q_from_normalized;
    if (use_est) {
      // The routing launch only produces the predicting signal; the estimator's four steps turn it
      // into logits, and its last step (the routing kernel in LayerNorm mode) selects and hands over.
      RouteArgs sa = pa;
      sa.vec_out = c->at<float>(c->lay.sig);
      sa.user_ids = nullptr;
      sa.user_gates = nullptr;
      sa.mailbox = nullptr;
      c->prep_route(sa);
      if ((e = launch_route(sa, cfg.dtype, c->compute)) != hipSuccess) return c->hip_fail(e, "signal kernel");
      const int dm = cfg.est_latent, F = cfg.est_ffn;
      GemvArgs g{};
      g.B = batch;
      g.w = c->est.proj; g.x_f32 = c->at<float>(c->lay.sig); g.rows = dm; g.cols = H;
      g.add_w = static_cast<const char *>(c->est.layer_emb) + size_t(layer) * dm * wbytes;
      g.y = c->at<double>(c->lay.est_u);
      if ((e = launch_gemv64(g, cfg.dtype, c->compute)) != hipSuccess) return c->hip_fail(e, "estimator projection");
      g = GemvArgs{};
      g.B = batch;
      g.w = c->est.ffn_in; g.x_f64 = c->at<double>(c->lay.est_u); g.rows = F; g.cols = dm; g.silu = 1;
      g.y = c->at<double>(c->lay.est_t);
      if ((e = launch_gemv64(g, cfg.dtype, c->compute)) != hipSuccess) return c->hip_fail(e, "estimator feed-forward");
      g = GemvArgs{};
      g.B = batch;
      g.w = c->est.ffn_out; g.x_f64 = c->at<double>(c->lay.est_t); g.rows = dm; g.cols = F;
      g.add_f64 = c->at<double>(c->lay.est_u);
      g.y = c->at<double>(c->lay.est_v);
      if ((e = launch_gemv64(g, cfg.dtype, c->compute)) != hipSuccess) return c->hip_fail(e, "estimator feed-forward");
      RouteArgs ha = pa;
      ha.spec = 3;
      ha.x_f64 = c->at<double>(c->lay.est_v);
      ha.w = c->est.head;
      ha.gain = c->est.ln_gain;
      ha.bias = c->est.ln_bias;
      ha.eps = c->est.ln_eps;
      ha.H = dm;
      ha.vec_out = nullptr;
      c->prep_route(ha);
      if ((e = launch_route(ha, cfg.dtype, c->compute)) != hipSuccess) return c->hip_fail(e, "estimator head");
      c->st.hbm_bytes_algorithmic += (int64_t(dm) * H + 2 * int64_t(F) * dm + int64_t(E) * dm + dm) * wbytes +
                                     int64_t(batch) * k * H * wbytes;
    } else {
      c->prep_route(pa);
      if ((e = launch_route(pa, cfg.dtype, c->compute)) != hipSuccess) return c->hip_fail(e, "prediction kernel");
      c->st.hbm_bytes_algorithmic += int64_t(E) * H * wbytes + int64_t(batch) * k * H * wbytes;
    }
  }
  }   // one kernel per routing
  c->close_span(sp_route, c->compute);

  // --- which experts run, and where their ids and gates live on the device
  std::vector<int> exec_union, exec_ids_host;
  const int32_t *exec_ids_dev;
  const float *exec_gates_dev;
  if (exec_pred) {
    exec_union = c->pending_union;
    exec_ids_host = c->pending_ids;
    exec_ids_dev = c->at<int32_t>(c->lay.pend_ids[layer & 1]);
    exec_gates_dev = c->at<float>(c->lay.pend_gates[layer & 1]);
  } else {
    int rc = c->wait_ids(c->mb_true, batch * k);
    if (rc) return rc;
    if ((rc = c->check_ids(c->mb_true->ids, batch * k))) return rc;
    exec_union = moe_spec_ctx::sorted_union(c->mb_true->ids, batch * k);
    exec_ids_host.assign(c->mb_true->ids, c->mb_true->ids + batch * k);
    exec_ids_dev = c->at<int32_t>(c->lay.true_ids);
    exec_gates_dev = c->at<float>(c->lay.true_gates);
  }
  if (outs && outs->exec_ids) {
    if ((e = hipMemcpyAsync(outs->exec_ids, exec_ids_dev, size_t(batch) * k * 4, hipMemcpyDeviceToDevice, c->compute)) != hipSuccess)
      return c->hip_fail(e, "copy exec ids");
  }
  if (outs && outs->exec_gates) {
    if ((e = hipMemcpyAsync(outs->exec_gates, exec_gates_dev, size_t(batch) * k * 4, hipMemcpyDeviceToDevice, c->compute)) != hipSuccess)
      return c->hip_fail(e, "copy exec gates");
  }

  ExpertArgs xa{};
  xa.pool = c->pool_base(layer);
  xa.slot_bytes = c->slot_stride;
  xa.s = c->at<float>(c->lay.s_buf);
  xa.exec_ids = exec_ids_dev;
  xa.exec_gates = exec_gates_dev;
  xa.h = c->at<float>(c->lay.h);
  xa.y = c->at<float>(c->lay.y);
  xa.out = static_cast<float *>(out_dev);
  xa.B = batch; xa.k = k; xa.H = H; xa.I = I;
  xa.bf16 = cfg.dtype == MOE_SPEC_BF16;

  const bool fast_b1 = batch == 1 && b1_supported(H, cfg.dtype) && !cfg.accumulate_defaults;
  const bool use_mfma = cfg.dtype == MOE_SPEC_BF16 && batch >= kMfmaMinBatch;

  // --- cache waves: make resident (unless prefetched), wait, run
  // profile = 1: every cache wave's wait for its copies is a stall span, its kernels a compute span
  for (size_t w0 = 0, wave = 0; w0 < exec_union.size(); w0 += S, ++wave) {
    ActiveList act{};
    int copies = 0;
    bool need_wait;
    if (exec_pred && wave == 0) {
      act = c->pending_wave0;
      need_wait = true;                         // the prefetch may still be in flight
    } else {
      std::vector<int> req(exec_union.begin() + w0, exec_union.begin() + std::min(exec_union.size(), w0 + S));
      int rc = c->request(layer, req, &act, &copies);
      if (rc) return rc;
      need_wait = copies > 0 || (hinted && wave == 0);
    }
    if (need_wait) {
      TimedSpan *sp_stall = c->open_span(2, c->compute);
      if ((e = hipStreamWaitEvent(c->compute, c->ready[layer], 0)) != hipSuccess) return c->hip_fail(e, "compute stream wait");
      c->close_span(sp_stall, c->compute);
    }
    c->st.cache_waves += 1;
    TimedSpan *sp_exec = c->open_span(0, c->compute);
    TimedSpan *sp_gu = c->open_span(3, c->compute);
    if (fast_b1) {
      // batch 1: the k executed experts are one wave; hand the kernels the slots in position order
      ActiveList by_pos{};
      by_pos.n = k;
      for (int j = 0; j < k; ++j) {
        by_pos.expert[j] = int16_t(exec_ids_host[j]);
        by_pos.slot[j] = int16_t(c->pools[layer].where[exec_ids_host[j]]);
      }
      if ((e = launch_gateup_b1(xa, by_pos, cfg.dtype, c->compute)) != hipSuccess) return c->hip_fail(e, "gate/up kernel");
      if ((e = launch_down_combine_b1(xa, by_pos, cfg.dtype, c->compute)) != hipSuccess) return c->hip_fail(e, "down kernel");
      c->close_span(sp_gu, c->compute);
    } else if (use_mfma) {
      uint16_t *hq = c->at<uint16_t>(c->lay.h);
      if ((e = launch_gateup_mfma(xa, act, c->at<uint16_t>(c->lay.s_q), hq, c->compute)) != hipSuccess)
        return c->hip_fail(e, "gate/up MFMA kernel");
      if ((e = launch_down_mfma(xa, act, hq, c->compute)) != hipSuccess) return c->hip_fail(e, "down MFMA kernel");
      c->close_span(sp_gu, c->compute);
    } else {
      if ((e = launch_gateup(xa, act, cfg.dtype, c->compute)) != hipSuccess) return c->hip_fail(e, "gate/up kernel");
      if ((e = launch_down(xa, act, cfg.dtype, c->compute)) != hipSuccess) return c->hip_fail(e, "down kernel");
      c->close_span(sp_gu, c->compute);
    }
    if (cfg.accumulate_defaults &&
        (e = launch_accumulate_defaults(xa, act, c->at<double>(c->lay.dacc_sum) + size_t(layer) * E * H,
                                        c->at<unsigned long long>(c->lay.dacc_cnt) + size_t(layer) * E,
                                        c->compute)) != hipSuccess)
      return c->hip_fail(e, "default-vector accumulation");
    if ((e = hipEventRecord(c->done[layer], c->compute)) != hipSuccess) return c->hip_fail(e, "record done event");
    c->done_recorded[layer] = 1;
    c->st.hbm_bytes_algorithmic += int64_t(act.n) * int64_t(c->expert_bytes);
    c->close_span(sp_exec, c->compute);
  }
  if (!fast_b1) {
    TimedSpan *sp_comb = c->open_span(0, c->compute);
    if ((e = launch_combine(xa, c->compute)) != hipSuccess) return c->hip_fail(e, "combine kernel");
    c->close_span(sp_comb, c->compute);
  }

  // --- prefetch the first wave of the predicted experts of layer l+1
  c->have_pending = do_pred;
  if (do_pred && prefetching) {
    int rc = c->wait_ids(c->mb_next, batch * k);
    if (rc) return rc;
    if ((rc = c->check_ids(c->mb_next->ids, batch * k))) return rc;
    c->pending_union = moe_spec_ctx::sorted_union(c->mb_next->ids, batch * k);
    c->pending_ids.assign(c->mb_next->ids, c->mb_next->ids + batch * k);
    std::vector<int> req(c->pending_union.begin(),
                         c->pending_union.begin() + std::min<size_t>(c->pending_union.size(), S));
    int copies = 0;
    rc = c->request(layer + 1, req, &c->pending_wave0, &copies);
    if (rc) return rc;
    if (copies == 0) {
      // nothing to copy: make the wait at the next step a no-op that is still well defined
      if ((e = hipEventRecord(c->ready[layer + 1], c->copy)) != hipSuccess) return c->hip_fail(e, "record ready event");
      c->ready_recorded[layer + 1] = 1;
    }
  }
  if (score_look) {
    // recall@k of what layer l-2 predicted for this layer; the true ids were posted before the predicted ones
    if (exec_pred) {
      int rc = c->wait_ids(c->mb_true, batch * k);
      if (rc) return rc;
      if ((rc = c->check_ids(c->mb_true->ids, batch * k))) return rc;
    }
    const std::vector<int> &look = c->look_ids[layer % 3];
    for (int b = 0; b < batch; ++b)
      for (int j = 0; j < k; ++j)
        for (int q = 0; q < k; ++q) c->st.hits2 += look[size_t(b) * k + j] == c->mb_true->ids[size_t(b) * k + q];
    c->st.predictions2 += int64_t(batch) * k;
    c->look_ids[layer % 3].clear();
  }
  if (look2) {
    int rc = c->wait_ids(c->mb_look, batch * k);
    if (rc) return rc;
    if ((rc = c->check_ids(c->mb_look->ids, batch * k))) return rc;
    std::vector<int> &look = c->look_ids[(layer + 2) % 3];
    look.assign(c->mb_look->ids, c->mb_look->ids + batch * k);
    std::vector<int> uni = moe_spec_ctx::sorted_union(c->mb_look->ids, batch * k);
    uni.resize(std::min<size_t>(uni.size(), S));
    ActiveList hinted_slots{};
    int copies = 0;
    if ((rc = c->request(layer + 2, uni, &hinted_slots, &copies))) return rc;
  }

  c->batch = batch;
  c->next_layer = layer + 1;
  if (last) c->token_open = false;
  c->st.layer_steps += 1;
  return MOE_SPEC_OK;
}

}  // namespace

extern "C" {

int moe_spec_layer_step(moe_spec_ctx *c, int layer, const void *r_dev, int batch, void *out_dev,
                        const moe_spec_step_outputs *outs) {
  if (!c) return MOE_SPEC_EINVAL;
  c->use_static = false;
  return layer_step_impl(c, layer, r_dev, batch, out_dev, outs);
}

int moe_spec_layer_step_static(moe_spec_ctx *c, int layer, const void *r_dev, int batch, void *out_dev,
                               const moe_spec_step_outputs *outs) {
  if (!c) return MOE_SPEC_EINVAL;
  const size_t need = c->lay.tr_end - c->lay.tr_begin;
  if (need > size_t(MOE_SPEC_STATIC_SCRATCH_BYTES))
    return c->fail(MOE_SPEC_EINVAL, "this configuration needs %zu bytes of step scratch, the static array holds %zu: "
                   "use moe_spec_layer_step (scratch in the arena) or a smaller max_batch", need,
                   size_t(MOE_SPEC_STATIC_SCRATCH_BYTES));
  if (c->cfg.profile) return c->fail(MOE_SPEC_ESTATE, "profile = 1 creates timing events; not available through the static entry point");
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != c->device)
    return c->fail(MOE_SPEC_ESTATE, "the current device is not the one the context was created on");
  c->use_static = true;
  const int rc = layer_step_impl(c, layer, r_dev, batch, out_dev, outs);
  c->use_static = false;
  return rc;
}

int moe_spec_prefill_layer_step(moe_spec_ctx *c, int layer, const void *r_dev, int n_tokens, void *out_dev,
                                int32_t *true_ids, float *true_gates) {
  if (!c) return MOE_SPEC_EINVAL;
  const moe_spec_config &cfg = c->cfg;
  if (!r_dev || !out_dev) return c->fail(MOE_SPEC_EINVAL, "null activation pointer");
  if (cfg.max_prefill_tokens < 1) return c->fail(MOE_SPEC_ESTATE, "context was created without a prefill path");
  if (n_tokens < 1 || n_tokens > cfg.max_prefill_tokens)
    return c->fail(MOE_SPEC_EINVAL, "n_tokens %d out of range", n_tokens);
  if (layer < 0 || layer >= cfg.n_layers) return c->fail(MOE_SPEC_EINVAL, "layer %d out of range", layer);
  if (c->token_open) return c->fail(MOE_SPEC_ESTATE, "prefill inside a decode step");
  if (!c->router_w[layer]) return c->fail(MOE_SPEC_ESTATE, "resident tables of layer %d were never set", layer);
  const int E = cfg.n_experts, k = cfg.top_k, H = cfg.hidden, I = cfg.inter, S = cfg.slots_per_layer;
  for (int x = 0; x < E; ++x)
    if (!c->host_expert[size_t(layer) * E + x])
      return c->fail(MOE_SPEC_ESTATE, "expert %d of layer %d was never registered", x, layer);
  const int P = n_tokens, MB = cfg.max_batch;
  const int halves = S >= 2 ? 2 : 1;
  const int group = std::min(S / halves, E);           // experts per group; group g lives in half g % halves
  const size_t wbytes = cfg.dtype == MOE_SPEC_BF16 ? 2 : 4;
  const float *r = static_cast<const float *>(r_dev);
  float *out = static_cast<float *>(out_dev);
  float *s_all = c->at<float>(c->lay.pf_s);
  uint16_t *sq_all = c->at<uint16_t>(c->lay.pf_sq);
  int32_t *ids_all = c->at<int32_t>(c->lay.pf_ids);
  float *gates_all = c->at<float>(c->lay.pf_gates);
  float *y_all = c->at<float>(c->lay.pf_y);
  hipError_t e;
  if (int rc = c->check_waits()) return rc;
  if (!c->clock_running) { c->clock_running = true; c->t0 = std::chrono::steady_clock::now(); }

  // --- true routing of every prompt token, one kernel per micro-batch of at most max_batch tokens
  TimedSpan *sp_route = c->open_span(0, c->compute);
  const bool pair_kernel = route_pair_supported(H, cfg.dtype);   // the fused kernel, asked for the true routing only
  for (int t0 = 0; t0 < P; t0 += MB) {
    const int nb = std::min(MB, P - t0);
    if (pair_kernel) {
      RoutePairArgs pa{};
      pa.r = r + size_t(t0) * H;
      pa.w_true = c->router_w[layer];
      pa.gain_true = static_cast<const float *>(c->gain[layer]);
      pa.z_true = c->zslot_set(0, c->route_parity);
      pa.z_pred = c->zslot_set(1, c->route_parity);
      pa.z_true_next = c->zslot_set(0, c->route_parity ^ 1);
      pa.z_pred_next = c->zslot_set(1, c->route_parity ^ 1);
      pa.arm_count = cfg.max_batch * E;
      c->route_parity ^= 1;
      pa.s_out = s_all + size_t(t0) * H;
      pa.s_out_q = cfg.dtype == MOE_SPEC_BF16 ? sq_all + size_t(t0) * H : nullptr;
      pa.true_ids = ids_all + size_t(t0) * k;
      pa.true_gates = gates_all + size_t(t0) * k;
      pa.diag = c->at<LayerDiag>(c->lay.diag) + layer;
      pa.user_true_ids = true_ids ? true_ids + size_t(t0) * k : nullptr;
      pa.user_true_gates = true_gates ? true_gates + size_t(t0) * k : nullptr;
      pa.status = c->wait_status_dev;
      pa.B = nb; pa.H = H; pa.E = E; pa.k = k;
      pa.eps = cfg.rms_eps;
      pa.bf16 = cfg.dtype == MOE_SPEC_BF16;
      pa.spin_limit = c->spin_limit;
      if ((e = launch_route_pair(pa, cfg.dtype, c->compute)) != hipSuccess) return c->hip_fail(e, "routing kernel");
      c->st.hbm_bytes_algorithmic += int64_t(E) * H * wbytes;
      continue;
    }
    RouteArgs ra{};
    ra.r = r + size_t(t0) * H;
    ra.w = c->router_w[layer];
    ra.gain = static_cast<const float *>(c->gain[layer]);
    ra.vec_out = s_all + size_t(t0) * H;
    ra.vec_out_q = cfg.dtype == MOE_SPEC_BF16 ? sq_all + size_t(t0) * H : nullptr;
    ra.ids_out = ids_all + size_t(t0) * k;
    ra.gates_out = gates_all + size_t(t0) * k;
    ra.diag = c->at<LayerDiag>(c->lay.diag) + layer;
    ra.user_ids = true_ids ? true_ids + size_t(t0) * k : nullptr;
    ra.user_gates = true_gates ? true_gates + size_t(t0) * k : nullptr;
    ra.B = nb; ra.H = H; ra.E = E; ra.k = k;
    ra.eps = cfg.rms_eps;
    ra.bf16 = cfg.dtype == MOE_SPEC_BF16;
    c->prep_route(ra);
    if ((e = launch_route(ra, cfg.dtype, c->compute)) != hipSuccess) return c->hip_fail(e, "routing kernel");
    c->st.hbm_bytes_algorithmic += int64_t(E) * H * wbytes;
  }
  const bool all_at_once = cfg.dtype == MOE_SPEC_BF16;   // matrix-core kernels over per-expert position lists
  if (all_at_once &&
      (e = launch_expert_lists(ids_all, P, k, E, c->at<int32_t>(c->lay.pf_pos), c->at<int32_t>(c->lay.pf_count),
                               c->compute)) != hipSuccess)
    return c->hip_fail(e, "expert list kernel");
  c->close_span(sp_route, c->compute);

  // --- the pool is taken over: whatever the decode cache held is dropped
  Pool &p = c->pools[layer];
  std::fill(p.slot_expert.begin(), p.slot_expert.end(), -1);
  std::fill(p.slot_stamp.begin(), p.slot_stamp.end(), -1);
  std::fill(p.where.begin(), p.where.end(), -1);
  p.clock = 0;
  if (c->done_recorded[layer]) { int rc = c->copy_queues_wait(c->done[layer]); if (rc) return rc; }
  if (c->ready_recorded[layer]) {
    for (hipStream_t q : c->copy_aux)
      if ((e = hipStreamWaitEvent(q, c->ready[layer], 0)) != hipSuccess) return c->hip_fail(e, "copy queue wait");
  }

  // --- stream every expert through the two halves of the pool
  for (int e0 = 0, g = 0; e0 < E; e0 += group, ++g) {
    const int half = g % halves, n_here = std::min(group, E - e0);
    if (g >= halves) {
      // The slots were last read by the kernels of group g - halves.  The host waits for them here
      // (the copy engines are then still busy with group g - 1, so they never run dry): a copy
      // queued behind an event that has already completed starts without a cross-queue barrier,
      // and such barriers cost the DMA queues about 0.1 ms each.
      if ((e = hipEventSynchronize(c->pf_done[half])) != hipSuccess) return c->hip_fail(e, "wait for the kernels of an earlier group");
      int rc = c->copy_queues_wait(c->pf_done[half]);
      if (rc) return rc;
    }
    TimedSpan *sp_copy = c->open_span(1, c->copy);
    CopyList cl{};
    cl.n16 = uint32_t(c->expert_bytes / 16);
    ActiveList act{};
    for (int x = 0; x < n_here; ++x) {
      const int slot = half * group + x;               // < halves * group <= S
      int rc = c->copy_expert(cl, x, c->pool_base(layer) + size_t(slot) * c->slot_stride,
                              c->host_expert[size_t(layer) * E + e0 + x]);
      if (rc) return rc;
      act.expert[x] = int16_t(e0 + x);
      act.slot[x] = int16_t(slot);
    }
    act.n = n_here;
    if (int rc = c->copy_join(cl)) return rc;
    c->close_span(sp_copy, c->copy);
    if ((e = hipEventRecord(c->pf_ready[half], c->copy)) != hipSuccess) return c->hip_fail(e, "record ready event");
    c->st.cache_misses += n_here;
    c->st.h2d_bytes += int64_t(n_here) * int64_t(c->expert_bytes);

    TimedSpan *sp_stall = c->open_span(2, c->compute);
    if ((e = hipStreamWaitEvent(c->compute, c->pf_ready[half], 0)) != hipSuccess) return c->hip_fail(e, "compute stream wait");
    c->close_span(sp_stall, c->compute);
    TimedSpan *sp_exec = c->open_span(0, c->compute);
    // bf16: the matrix-core kernels take all tokens of every expert in one launch, 64 per grid plane;
    // float32: the general kernels, one launch pair per micro-batch
    for (int t0 = 0; t0 < P; t0 += all_at_once ? P : MB) {
      const int nb = all_at_once ? std::min(MB, P) : std::min(MB, P - t0);
      ExpertArgs xa{};
      xa.pool = c->pool_base(layer);
      xa.slot_bytes = c->slot_stride;
      xa.s = s_all + size_t(t0) * H;
      xa.exec_ids = ids_all + size_t(t0) * k;
      xa.exec_gates = gates_all + size_t(t0) * k;
      xa.h = c->at<float>(c->lay.h);                   // [nb,k,I], reused by every micro-batch
      xa.y = y_all + size_t(t0) * k * H;
      xa.out = out + size_t(t0) * H;
      xa.B = nb; xa.k = k; xa.H = H; xa.I = I;
      xa.bf16 = cfg.dtype == MOE_SPEC_BF16;
      if (all_at_once) {
        uint16_t *hq = c->at<uint16_t>(c->lay.pf_hq);  // [P,k,I]
        xa.pos_list = c->at<int32_t>(c->lay.pf_pos);
        xa.pos_count = c->at<int32_t>(c->lay.pf_count);
        xa.list_stride = P;
        xa.list_tokens = P;
        if ((e = launch_gateup_mfma(xa, act, sq_all, hq, c->compute)) != hipSuccess)
          return c->hip_fail(e, "gate/up MFMA kernel");
        if ((e = launch_down_mfma(xa, act, hq, c->compute)) != hipSuccess) return c->hip_fail(e, "down MFMA kernel");
      } else {
        if ((e = launch_gateup(xa, act, cfg.dtype, c->compute)) != hipSuccess) return c->hip_fail(e, "gate/up kernel");
        if ((e = launch_down(xa, act, cfg.dtype, c->compute)) != hipSuccess) return c->hip_fail(e, "down kernel");
      }
      if (cfg.accumulate_defaults)
        for (int u0 = t0; u0 < (all_at_once ? P : t0 + nb); u0 += MB) {
          ExpertArgs ya = xa;                          // per micro-batch: the kernel indexes positions from 0
          ya.exec_ids = ids_all + size_t(u0) * k;
          ya.y = y_all + size_t(u0) * k * H;
          ya.B = std::min(MB, P - u0);
          if ((e = launch_accumulate_defaults(ya, act, c->at<double>(c->lay.dacc_sum) + size_t(layer) * E * H,
                                              c->at<unsigned long long>(c->lay.dacc_cnt) + size_t(layer) * E,
                                              c->compute)) != hipSuccess)
            return c->hip_fail(e, "default-vector accumulation");
        }
      c->st.hbm_bytes_algorithmic += int64_t(n_here) * int64_t(c->expert_bytes);
    }
    c->close_span(sp_exec, c->compute);
    if ((e = hipEventRecord(c->pf_done[half], c->compute)) != hipSuccess) return c->hip_fail(e, "record done event");
  }

  // --- gate-weighted sums
  TimedSpan *sp_comb = c->open_span(0, c->compute);
  {
    ExpertArgs xa{};                                   // one launch: a grid row per token
    xa.exec_gates = gates_all;
    xa.y = y_all;
    xa.out = out;
    xa.B = P; xa.k = k; xa.H = H; xa.I = I;
    if ((e = launch_combine(xa, c->compute)) != hipSuccess) return c->hip_fail(e, "combine kernel");
  }
  c->close_span(sp_comb, c->compute);
  // later copies into this pool wait for the kernels above
  if ((e = hipEventRecord(c->done[layer], c->compute)) != hipSuccess) return c->hip_fail(e, "record done event");
  c->done_recorded[layer] = 1;
  c->st.layer_steps += 1;
  c->st.prefill_tokens += P;
  return MOE_SPEC_OK;
}

int moe_spec_stats(moe_spec_ctx *c, moe_spec_stats_t *out) {
  if (!c) return MOE_SPEC_EINVAL;
  if (!out) return c->fail(MOE_SPEC_EINVAL, "out is null");
  hipError_t e = c->sync_streams();
  if (e != hipSuccess) return c->hip_fail(e, "synchronize");
  int rc = c->resolve_spans();
  if (rc) return rc;
  if ((rc = c->check_waits())) return rc;
  std::vector<LayerDiag> dg(c->cfg.n_layers);
  if ((e = hipMemcpy(dg.data(), c->arena + c->lay.diag, dg.size() * sizeof(LayerDiag), hipMemcpyDeviceToHost)) != hipSuccess)
    return c->hip_fail(e, "read hit counters");
  c->st.hits = c->st.predictions = 0;
  for (const LayerDiag &d : dg) { c->st.hits += int64_t(d.hits); c->st.predictions += int64_t(d.preds); }
  if (c->clock_running)
    c->st.wall_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - c->t0).count();
  *out = c->st;
  return MOE_SPEC_OK;
}

int moe_spec_layer_diagnostics(moe_spec_ctx *c, int layer, moe_spec_layer_diag_t *out) {
  if (!c) return MOE_SPEC_EINVAL;
  if (!out) return c->fail(MOE_SPEC_EINVAL, "out is null");
  if (layer < 0 || layer >= c->cfg.n_layers) return c->fail(MOE_SPEC_EINVAL, "layer %d out of range", layer);
  hipError_t e = c->sync_streams();
  if (e != hipSuccess) return c->hip_fail(e, "synchronize");
  LayerDiag d;
  if ((e = hipMemcpy(&d, c->arena + c->lay.diag + size_t(layer) * sizeof(LayerDiag), sizeof d, hipMemcpyDeviceToHost)) != hipSuccess)
    return c->hip_fail(e, "read layer statistics");
  out->predictions = int64_t(d.preds);
  out->hits = int64_t(d.hits);
  for (int j = 0; j < MOE_SPEC_MAX_TOP_K; ++j) out->rank_match[j] = int64_t(d.rank_match[j]);
  out->cos_sum = d.cos_sum;
  out->cos_count = int64_t(d.cos_count);
  return MOE_SPEC_OK;
}

int moe_spec_read_default_vectors(moe_spec_ctx *c, int layer, float *mean_dev, int64_t *counts_host) {
  if (!c) return MOE_SPEC_EINVAL;
  if (!c->cfg.accumulate_defaults) return c->fail(MOE_SPEC_ESTATE, "the context was created without accumulate_defaults");
  if (layer < 0 || layer >= c->cfg.n_layers) return c->fail(MOE_SPEC_EINVAL, "layer %d out of range", layer);
  if (!mean_dev) return c->fail(MOE_SPEC_EINVAL, "mean_dev is null");
  const int E = c->cfg.n_experts, H = c->cfg.hidden;
  const double *sum = c->at<double>(c->lay.dacc_sum) + size_t(layer) * E * H;
  const unsigned long long *cnt = c->at<unsigned long long>(c->lay.dacc_cnt) + size_t(layer) * E;
  hipError_t e = launch_default_means(sum, cnt, mean_dev, E, H, c->compute);
  if (e == hipSuccess) e = hipStreamSynchronize(c->compute);
  if (e != hipSuccess) return c->hip_fail(e, "default-vector means");
  if (counts_host) {
    static_assert(sizeof(unsigned long long) == sizeof(int64_t), "counter width");
    if ((e = hipMemcpy(counts_host, cnt, size_t(E) * 8, hipMemcpyDeviceToHost)) != hipSuccess)
      return c->hip_fail(e, "read counts");
  }
  return MOE_SPEC_OK;
}

int moe_spec_reset(moe_spec_ctx *c) {
  if (!c) return MOE_SPEC_EINVAL;
  hipError_t e = c->sync_streams();
  if (e != hipSuccess) return c->hip_fail(e, "synchronize");
  int rc = c->resolve_spans();
  if (rc) return rc;
  for (auto &p : c->pools) {
    std::fill(p.slot_expert.begin(), p.slot_expert.end(), -1);
    std::fill(p.slot_stamp.begin(), p.slot_stamp.end(), -1);
    std::fill(p.where.begin(), p.where.end(), -1);
    p.clock = 0;
  }
  if ((e = hipMemsetAsync(c->arena + c->lay.diag, 0, size_t(c->cfg.n_layers) * sizeof(LayerDiag), c->compute)) != hipSuccess)
    return c->hip_fail(e, "clear counters");
  if (c->cfg.accumulate_defaults &&
      (e = hipMemsetAsync(c->arena + c->lay.dacc_sum, 0, c->lay.dacc_end - c->lay.dacc_sum, c->compute)) != hipSuccess)
    return c->hip_fail(e, "clear sums");
  if ((e = c->arm_handover_slots()) != hipSuccess) return c->hip_fail(e, "arm hand-over slots");
  if ((e = hipStreamSynchronize(c->compute)) != hipSuccess) return c->hip_fail(e, "synchronize");
  c->st = moe_spec_stats_t{};
  c->clock_running = false;
  c->token_open = false;
  c->have_pending = false;
  c->next_layer = 0;
  c->pending_union.clear();
  return MOE_SPEC_OK;
}

int moe_spec_time_kernel(moe_spec_ctx *c, int which, int reps, double *ms_per_launch, int64_t *bytes_per_launch) {
  if (!c) return MOE_SPEC_EINVAL;
  if (which < 0 || which > 9 || which == 8 || reps < 1 || !ms_per_launch || !bytes_per_launch)
    return c->fail(MOE_SPEC_EINVAL, "bad arguments to time_kernel");
  if ((which == 4 || which == 5) && c->cfg.dtype != MOE_SPEC_BF16) return c->fail(MOE_SPEC_ESTATE, "the matrix-core kernels need bf16 weights");
  if (c->token_open) return c->fail(MOE_SPEC_ESTATE, "time_kernel inside a decode step");
  const moe_spec_config &cfg = c->cfg;
  const int L = cfg.n_layers, E = cfg.n_experts, k = cfg.top_k, H = cfg.hidden, I = cfg.inter;
  const size_t wbytes = cfg.dtype == MOE_SPEC_BF16 ? 2 : 4;
  if ((which == 6 || which == 7) && (!c->router_w[0] || !route_pair_supported(H, cfg.dtype)))
    return c->fail(MOE_SPEC_ESTATE, "the fused routing kernel does not apply to this configuration");
  if (which == 2 || which == 6 || which == 7) for (int l = 0; l < L; ++l) if (!c->router_w[l]) return c->fail(MOE_SPEC_ESTATE, "resident tables not set");
  hipError_t e;
  int32_t ids[kMaxTopK];
  ActiveList act{};
  act.n = k;
  for (int j = 0; j < k; ++j) { ids[j] = j; act.expert[j] = int16_t(j); act.slot[j] = int16_t(j); }
  if ((e = hipMemcpyAsync(c->arena + c->lay.bench_ids, ids, size_t(k) * 4, hipMemcpyHostToDevice, c->compute)) != hipSuccess)
    return c->hip_fail(e, "upload ids");
  // The activations the launches read: a bell-shaped draw per element (sum of four uniforms), so that logits are
  // distinct as they are in a decode step (equal logits, as zeros would give, send the top-k through its
  // tie-breaking path on every comparison).
  {
    std::vector<float> rin(size_t(cfg.max_batch) * H);
    uint32_t state = 0x9e3779b9u;
    for (float &v : rin) {
      float acc = 0.f;
      for (int u = 0; u < 4; ++u) { state = state * 1664525u + 1013904223u; acc += float(state >> 8) * (1.0f / 16777216.0f); }
      v = (acc - 2.0f) * 1.7320508f;
    }
    if ((e = hipMemcpyAsync(c->arena + c->lay.s_buf, rin.data(), rin.size() * 4, hipMemcpyHostToDevice, c->compute)) != hipSuccess ||
        (e = hipStreamSynchronize(c->compute)) != hipSuccess)
      return c->hip_fail(e, "upload activations");
  }
  hipEvent_t t0 = nullptr, t1 = nullptr;
  if ((e = hipEventCreate(&t0)) != hipSuccess) return c->hip_fail(e, "event");
  if ((e = hipEventCreate(&t1)) != hipSuccess) { (void)hipEventDestroy(t0); return c->hip_fail(e, "event"); }
  ExpertArgs xa{};
  xa.slot_bytes = c->slot_stride;
  xa.s = c->at<float>(c->lay.s_buf);
  xa.exec_ids = c->at<int32_t>(c->lay.bench_ids);
  xa.exec_gates = c->at<float>(c->lay.true_gates);
  xa.h = c->at<float>(c->lay.h);
  xa.y = c->at<float>(c->lay.y);
  xa.out = c->at<float>(c->lay.y);
  xa.B = 1; xa.k = k; xa.H = H; xa.I = I;
  xa.bf16 = cfg.dtype == MOE_SPEC_BF16;
  RouteArgs ra{};
  ra.r = c->at<float>(c->lay.s_buf);
  ra.ids_out = c->at<int32_t>(c->lay.true_ids);
  ra.gates_out = c->at<float>(c->lay.true_gates);
  ra.diag = c->at<LayerDiag>(c->lay.diag);
  ra.B = 1; ra.H = H; ra.E = E; ra.k = k; ra.eps = cfg.rms_eps; ra.bf16 = xa.bf16;
  const bool fast = b1_supported(H, cfg.dtype);
  // matrix-core kernels: a full batch whose positions are dealt round-robin over as many resident
  // slots as a cache wave can hold (a token's k experts stay distinct because n_act >= k)
  const int Bm = cfg.max_batch;
  const int n_act = std::min({cfg.slots_per_layer, E, Bm * k});
  ActiveList act_m{};
  ExpertArgs xm = xa;
  std::vector<int32_t> tab;                                        // outlives the launches that read its device copy
  if (which == 4 || which == 5) {
    tab.resize(size_t(Bm) * k);
    for (size_t f = 0; f < tab.size(); ++f) tab[f] = int32_t(f % n_act);
    act_m.n = n_act;
    for (int j = 0; j < n_act; ++j) { act_m.expert[j] = int16_t(j); act_m.slot[j] = int16_t(j); }
    // on the compute stream, like the launches that follow (the stream does not synchronise with the null stream)
    if ((e = hipMemcpyAsync(c->arena + c->lay.pend_ids[0], tab.data(), tab.size() * 4, hipMemcpyHostToDevice, c->compute)) != hipSuccess) {
      (void)hipEventDestroy(t0); (void)hipEventDestroy(t1);
      return c->hip_fail(e, "upload ids");
    }
    xm.exec_ids = c->at<int32_t>(c->lay.pend_ids[0]);
    xm.B = Bm;
  }
  hipError_t le = hipSuccess;
  for (int pass = 0; pass < 2 && le == hipSuccess; ++pass) {      // pass 0 warms up
    const int n = pass == 0 ? std::min(reps, 4) : reps;
    if (pass == 1) le = hipEventRecord(t0, c->compute);
    for (int i = 0; i < n && le == hipSuccess; ++i) {
      const int l = i % L;
      xa.pool = c->pool_base(l);
      if (which == 0) le = fast ? launch_gateup_b1(xa, act, cfg.dtype, c->compute) : launch_gateup(xa, act, cfg.dtype, c->compute);
      else if (which == 1) le = fast ? launch_down_combine_b1(xa, act, cfg.dtype, c->compute) : launch_down(xa, act, cfg.dtype, c->compute);
      else if (which == 3) le = launch_stream_read(xa, act, 0, size_t(2) * I * H * wbytes / 16, c->compute);
      else if (which == 9) le = launch_stream_read(xa, act, size_t(2) * I * H * wbytes / 16, size_t(I) * H * wbytes / 16, c->compute);
      else if (which == 6 || which == 7) {
        RoutePairArgs pa{};
        pa.r = c->at<float>(c->lay.s_buf);
        pa.w_true = c->router_w[l];
        pa.gain_true = static_cast<const float *>(c->gain[l]);
        if (which == 7) {
          pa.w_next = c->router_w[(l + 1) % L];
          pa.gain_next = static_cast<const float *>(c->gain[(l + 1) % L]);
          pa.dvec = c->dvecs[l];
        }
        pa.z_true = c->zslot_set(0, c->route_parity);
        pa.z_pred = c->zslot_set(1, c->route_parity);
        pa.z_true_next = c->zslot_set(0, c->route_parity ^ 1);
        pa.z_pred_next = c->zslot_set(1, c->route_parity ^ 1);
        pa.arm_count = cfg.max_batch * E;
        c->route_parity ^= 1;
        pa.s_out = c->at<float>(c->lay.sig);
        pa.true_ids = c->at<int32_t>(c->lay.true_ids);
        pa.true_gates = c->at<float>(c->lay.true_gates);
        pa.next_ids = c->at<int32_t>(c->lay.pend_ids[0]);
        pa.next_gates = c->at<float>(c->lay.pend_gates[0]);
        pa.diag = c->at<LayerDiag>(c->lay.diag);
        pa.status = c->wait_status_dev;
        pa.B = Bm; pa.H = H; pa.E = E; pa.k = k;
        pa.eps = cfg.rms_eps;
        pa.bf16 = xa.bf16;
        pa.spin_limit = c->spin_limit;
#ifdef MOE_SPEC_STAGE_CLOCK
        pa.mb_true = c->mb_true_dev; pa.mb_next = c->mb_next_dev;     // as in a prefetching decode step
        pa.stage_clock = c->at<unsigned long long>(c->lay.y);
#endif
        le = launch_route_pair(pa, cfg.dtype, c->compute);
      }
      else if (which == 4) { xm.pool = xa.pool; le = launch_gateup_mfma(xm, act_m, c->at<uint16_t>(c->lay.s_q), c->at<uint16_t>(c->lay.h), c->compute); }
      else if (which == 5) { xm.pool = xa.pool; le = launch_down_mfma(xm, act_m, c->at<uint16_t>(c->lay.h), c->compute); }
      else { ra.w = c->router_w[l]; ra.gain = static_cast<const float *>(c->gain[l]); c->prep_route(ra); le = launch_route(ra, cfg.dtype, c->compute); }
    }
    if (pass == 1 && le == hipSuccess) le = hipEventRecord(t1, c->compute);
  }
  e = hipStreamSynchronize(c->compute);
  float ms = 0.f;
  if (le == hipSuccess && e == hipSuccess) e = hipEventElapsedTime(&ms, t0, t1);
  (void)hipEventDestroy(t0);
  (void)hipEventDestroy(t1);
#ifdef MOE_SPEC_STAGE_CLOCK
  if (which == 7 && le == hipSuccess) {
    unsigned long long t[12];
    if (hipMemcpy(t, c->arena + c->lay.y, sizeof t, hipMemcpyDeviceToHost) == hipSuccess) {
      std::fprintf(stderr, "[stage clock, last launch, 10 ns ticks since kernel start]");
      for (int i = 1; i < 12; ++i) std::fprintf(stderr, " %llu", t[i] - t[0]);
      std::fprintf(stderr, "\n");
    }
  }
#endif
  if (le != hipSuccess) return c->hip_fail(le, "kernel launch");
  if (e != hipSuccess) return c->hip_fail(e, "timing");
  *ms_per_launch = double(ms) / reps;
  *bytes_per_launch = which == 0 || which == 3 ? int64_t(k) * 2 * I * H * wbytes
                    : which == 1 || which == 9 ? int64_t(k) * I * H * wbytes
                    : which == 7 ? 2 * int64_t(E) * H * wbytes + int64_t(Bm) * k * H * wbytes
                    : which == 4 ? int64_t(n_act) * 2 * I * H * wbytes
                    : which == 5 ? int64_t(n_act) * I * H * wbytes
                                 : int64_t(E) * H * wbytes;
  return MOE_SPEC_OK;
}

}  // extern "C"
