// One launch per dependent stage of a decode layer step:
//
//   route_pair_kernel   true routing of layer l AND the prediction for layer l+1 in one launch
//                       (paper: Sec. 3.1-3.3; Algorithm 1, TopK(Gate_l(X)) and GetNextExperts): RMSNorm,
//                       router l, top-k, gates, d_l, q_l, router l+1, top-k, gates.
//   expert_b1_kernel    the expert FFN of a batch of one in one launch (Algorithm 1, MoE_l(X, ids, g, C_l);
//                       Sec. 4 for whose gates): gate/up GEMV + SwiGLU, then down GEMV + gate-weighted combine.
//
// Both hand small results from the workgroups that compute them to the workgroups that need them inside
// the launch.  The hand-over is "the data is the flag": a slot of global memory holds a bit pattern that
// no result can have (all ones: a NaN) until its producer overwrites it with one relaxed device-scope
// atomic store; consumers read the slot with relaxed device-scope atomic loads until it no longer holds
// that pattern.  Each slot is a single atomic object, so nothing has to be ordered against anything
// else: no fence, no counter, no wait for a store's acknowledgement.  Slots come in two sets used by
// alternate launches; a launch re-arms the set the next launch will use (the previous launch, which
// read that set, has ended).  Every wait is bounded: after `spin_limit` polls a waiter gives up, raises
// the status word and finishes with whatever it has, so every wavefront reaches its end.
// Who may wait for whom: a consumer only waits for workgroups with lower block indices (dispatched no
// later than itself), or for the other workgroups of its own routing group, which the launcher checks
// to fit on the device together.
#include "device_utils.h"
#include "kernels.h"

namespace moe_spec {
namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / kWave;
constexpr unsigned long long kEmpty64 = ~0ull;
constexpr uint32_t kEmpty32 = ~0u;

__device__ __forceinline__ void raise_status(unsigned int *status) {      // a word in pinned host memory
  __hip_atomic_store(status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

__device__ __forceinline__ void publish64(unsigned long long *slot, double v) {
  if (!(v == v)) v = -INFINITY;                // a result that is not a number must not look like an empty slot
  __hip_atomic_store(slot, static_cast<unsigned long long>(__double_as_longlong(v)), __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void arm64(unsigned long long *slot) {
  __hip_atomic_store(slot, kEmpty64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ unsigned long long await64(const unsigned long long *slot, unsigned int limit,
                                                      unsigned int *status) {
  unsigned long long v = __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  for (unsigned int spins = 0; v == kEmpty64; ++spins) {
    if (spins >= limit) { raise_status(status); break; }
    __builtin_amdgcn_s_sleep(2);
    v = __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  return v;
}

__device__ __forceinline__ uint32_t await32(const uint32_t *slot, uint32_t first, unsigned int limit,
                                            unsigned int *status) {
  uint32_t v = first;
  for (unsigned int spins = 0; v == kEmpty32; ++spins) {
    if (spins >= limit) { raise_status(status); break; }
    __builtin_amdgcn_s_sleep(2);
    v = __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  return v;
}

// ---------------------------------------------------------------------------------------------
// Routing

struct SelectShared {
  int rank[kMaxExperts];
  double top_z[kMaxTopK];
  double top_e[kMaxTopK];
  double gate[kMaxTopK];
  int top_i[kMaxTopK];
  int hits;
};

struct RouteShared {
  double red[kWaves];
  double part[kWaves];
  SelectShared sel;
};

// Sum over the workgroup, the same value in every thread; red[] may be reused after the call.
__device__ __forceinline__ double block_sum(double v, double *red, int lane, int wave) {
  v = wave_sum(v);
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  double tot = 0.0;
#pragma unroll
  for (int x = 0; x < kWaves; ++x) tot += red[x];
  return tot;
}

// Top-k of one token's E logits (read from their slots as they arrive), ties to the lower index, and the
// softmax over the k selected: fills sel.top_i / top_z / gate, the same in every workgroup that calls it.
// Every wavefront holds all candidates in registers (element i = r*64 + lane); the four wavefronts split
// the source lanes of the rank count and add their counts in LDS.
template <int R>
__device__ void select_topk(const unsigned long long *slots, int E, int k, SelectShared &sel, int tid,
                            unsigned int limit, unsigned int *status) {
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  constexpr int kSrcPerWave = kWave / kWaves;
  double key[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int i = r * kWave + lane;
    double zi = -INFINITY;
    if (i < E) zi = __longlong_as_double(static_cast<long long>(await64(slots + i, limit, status)));
    key[r] = zi == zi ? zi : -INFINITY;          // total order whatever the input: ids stay distinct and in range
  }
  for (int i = tid; i < kMaxExperts; i += kBlock) sel.rank[i] = 0;
  if (tid == 0) sel.hits = 0;
  __syncthreads();
  int cnt[R];
  rank_counts<R>(key, lane, wave * kSrcPerWave, (wave + 1) * kSrcPerWave, cnt);
#pragma unroll
  for (int r = 0; r < R; ++r) atomicAdd(&sel.rank[r * kWave + lane], cnt[r]);
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int i = r * kWave + lane;
      const int rk = sel.rank[i];
      if (i < E && rk < k) { sel.top_z[rk] = key[r]; sel.top_i[rk] = i; }
    }
  }
  __syncthreads();
  if (tid < k) sel.top_e[tid] = exp(sel.top_z[tid] - sel.top_z[0]);
  __syncthreads();
  if (tid < k) {
    double denom = 0.0;
    for (int q = 0; q < k; ++q) denom += sel.top_e[q];
    sel.gate[tid] = sel.top_e[tid] / denom;
  }
  __syncthreads();
}

__device__ __forceinline__ void select_topk_any(const unsigned long long *slots, int E, int k, SelectShared &sel,
                                                int tid, unsigned int limit, unsigned int *status) {
  if (E <= kWave) select_topk<1>(slots, E, k, sel, tid, limit, status);
  else if (E <= 2 * kWave) select_topk<2>(slots, E, k, sel, tid, limit, status);
  else select_topk<4>(slots, E, k, sel, tid, limit, status);
}

// The mailbox is complete when every token group has written its ids: the last group to get here posts.
__device__ __forceinline__ void post_mailbox(Mailbox *mb, uint32_t seq, unsigned int *groups_done, int tid) {
  __threadfence_system();                        // this group's ids
  __syncthreads();
  if (tid == 0) {
    bool all_done = true;
    if (gridDim.y > 1) {
      __threadfence();
      all_done = atomicAdd(groups_done, 1u) == gridDim.y - 1;
      if (all_done) { __threadfence(); __hip_atomic_store(groups_done, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
    }
    if (all_done) __hip_atomic_store(&mb->seq, seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
  }
}

// SPLIT wavefronts share one router row (4 / SPLIT rows per workgroup); NCH 16-byte chunks of the row
// per lane, loaded into registers for both routers at the top of the kernel so that their latency
// overlaps the normalisation.  blockIdx.y is the token; the workgroups of a token form a group that
// exchanges logits through the token's slots and computes everything else redundantly (the norm, the
// top-k, the default-vector sum), so that nothing but the 8-byte logits crosses between workgroups.
template <typename WT, int SPLIT, int NCH>
__global__ __launch_bounds__(kBlock) void route_pair_kernel(const RoutePairArgs a) {
  extern __shared__ double vec[];              // [H] the router input being built, double precision
  __shared__ RouteShared sh;
  using P = Packed<WT>;
  using Raw = typename P::Raw;
  constexpr int VN = P::N;
  constexpr int RPW = kWaves / SPLIT;          // rows per workgroup

  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int wg = blockIdx.x, b = blockIdx.y;
  const int H = a.H, E = a.E, k = a.k;
  const int row = wg * RPW + wave / SPLIT, part = wave % SPLIT;
  const bool pred = a.w_next != nullptr;
  const WT *wt = static_cast<const WT *>(a.w_true);
  const WT *wn = static_cast<const WT *>(a.w_next);

  Raw rt[NCH], rn[NCH];
  if (row < E) {
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      const int c = ((ch * SPLIT + part) * kWave + lane) * VN;
      rt[ch] = *reinterpret_cast<const Raw *>(wt + size_t(row) * H + (c < H ? c : 0));
      if (pred) rn[ch] = *reinterpret_cast<const Raw *>(wn + size_t(row) * H + (c < H ? c : 0));
    }
  }
  // re-arm the whole set of slots the next launch will use (last read by the previous launch, which has
  // ended), for every token the context allows: the next launch may carry a larger batch than this one
  for (int i = (b * gridDim.x + wg) * kBlock + tid; i < a.arm_count; i += gridDim.x * gridDim.y * kBlock) {
    arm64(a.z_true_next + i);
    arm64(a.z_pred_next + i);
  }

  // ---- s_l = LN_l(r_l)
  const float *rrow = a.r + size_t(b) * H;
  {
    double ss = 0.0;
    for (int c = tid * VN; c < H; c += kBlock * VN) {
#pragma unroll
      for (int x = 0; x < VN; x += 4) {
        const float4 f = *reinterpret_cast<const float4 *>(rrow + c + x);
        const float4 g = *reinterpret_cast<const float4 *>(a.gain_true + c + x);
        vec[c + x] = double(f.x) * double(g.x); vec[c + x + 1] = double(f.y) * double(g.y);
        vec[c + x + 2] = double(f.z) * double(g.z); vec[c + x + 3] = double(f.w) * double(g.w);
        ss += double(f.x) * double(f.x) + double(f.y) * double(f.y) + double(f.z) * double(f.z) + double(f.w) * double(f.w);
      }
    }
    const double tot = block_sum(ss, sh.red, lane, wave);
    const double inv = 1.0 / sqrt(tot / double(H) + double(a.eps));
    for (int c = tid * VN; c < H; c += kBlock * VN) {
#pragma unroll
      for (int x = 0; x < VN; ++x) {
        double n = vec[c + x] * inv;
        if (a.bf16) n = round_to_bf16_fast(n);
        vec[c + x] = n;
        if (wg == 0) {
          a.s_out[size_t(b) * H + c + x] = static_cast<float>(n);
          if (a.s_out_q) a.s_out_q[size_t(b) * H + c + x] = uint16_t(__float_as_uint(static_cast<float>(n)) >> 16);
        }
      }
    }
    __syncthreads();
  }

  // ---- logits of router l; one row per SPLIT wavefronts
  auto row_logit = [&](const Raw (&w)[NCH]) {
    double acc = 0.0;
    if (row < E) {
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) {
        const int c = ((ch * SPLIT + part) * kWave + lane) * VN;
        if (c < H) {
          float wf[VN];
          P::unpack(w[ch], wf);
#pragma unroll
          for (int x = 0; x < VN; ++x) acc += double(wf[x]) * vec[c + x];
        }
      }
    }
    return wave_sum(acc);
  };
  auto publish_rows = [&](double acc, unsigned long long *slots) {
    if (SPLIT == 1) {
      if (lane == 0 && row < E) publish64(slots + size_t(b) * E + row, acc);
    } else {
      if (lane == 0) sh.part[wave] = acc;
      __syncthreads();
      if (tid < RPW && wg * RPW + tid < E) {
        double s = 0.0;
#pragma unroll
        for (int p = 0; p < SPLIT; ++p) s += sh.part[tid * SPLIT + p];
        publish64(slots + size_t(b) * E + wg * RPW + tid, s);
      }
    }
  };
  publish_rows(row_logit(rt), a.z_true);
  if (!pred && wg != 0) return;

  // ---- (E_l, G_l): every workgroup of the token selects for itself; workgroup 0 also reports
  select_topk_any(a.z_true + size_t(b) * E, E, k, sh.sel, tid, a.spin_limit, a.status);
  if (wg == 0) {
    if (tid < k) {
      const int id = sh.sel.top_i[tid];
      const double g = sh.sel.gate[tid];
      const size_t o = size_t(b) * k + tid;
      a.true_ids[o] = id;
      a.true_gates[o] = static_cast<float>(g);
      if (a.user_true_ids) a.user_true_ids[o] = id;
      if (a.user_true_gates) a.user_true_gates[o] = static_cast<float>(g);
      if (a.mb_true) a.mb_true->ids[o] = id;
      if (a.cmp_ids) {                           // recall@k of the prediction made one layer earlier (Sec. 3.3)
        int hit = 0;
        for (int j = 0; j < k; ++j) hit |= (a.cmp_ids[size_t(b) * k + j] == id);
        if (hit) atomicAdd(&sh.sel.hits, 1);
      }
    }
    __syncthreads();
    if (tid == 0 && a.cmp_ids) {
      atomicAdd(&a.diag->hits, static_cast<unsigned long long>(sh.sel.hits));
      atomicAdd(&a.diag->preds, static_cast<unsigned long long>(k));
    }
    if (a.mb_true) post_mailbox(a.mb_true, a.seq_true, a.groups_done, tid);
  }
  if (!pred) return;

  // ---- d_l = sum_j g_j d_{l,e_j};  q_l = LN_{l+1}(r_l + d_l)   (or s_l + d_l, the caption's reading)
  {
    const WT *dv = static_cast<const WT *>(a.dvec);
    double ss = 0.0;
    for (int c = tid * VN; c < H; c += kBlock * VN) {
      double u[VN];
      if (a.from_normalized) {
#pragma unroll
        for (int x = 0; x < VN; ++x) u[x] = vec[c + x];
      } else {
#pragma unroll
        for (int x = 0; x < VN; x += 4) {
          const float4 f = *reinterpret_cast<const float4 *>(rrow + c + x);
          u[x] = f.x; u[x + 1] = f.y; u[x + 2] = f.z; u[x + 3] = f.w;
        }
      }
      double d[VN];
#pragma unroll
      for (int x = 0; x < VN; ++x) d[x] = 0.0;
      for (int j0 = 0; j0 < k; j0 += 8) {              // eight default-vector rows in flight
        Raw dr[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const int j = min(j0 + q, k - 1);
          dr[q] = *reinterpret_cast<const Raw *>(dv + size_t(sh.sel.top_i[j]) * H + c);
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          if (j0 + q < k) {
            const double g = sh.sel.gate[j0 + q];
            float dvf[VN];
            P::unpack(dr[q], dvf);
#pragma unroll
            for (int x = 0; x < VN; ++x) d[x] += g * double(dvf[x]);
          }
        }
      }
      float gf[VN];
#pragma unroll
      for (int x = 0; x < VN; x += 4) {
        const float4 g = *reinterpret_cast<const float4 *>(a.gain_next + c + x);
        gf[x] = g.x; gf[x + 1] = g.y; gf[x + 2] = g.z; gf[x + 3] = g.w;
      }
#pragma unroll
      for (int x = 0; x < VN; ++x) {
        const double ux = u[x] + d[x];
        vec[c + x] = ux * double(gf[x]);
        ss += ux * ux;
      }
    }
    const double tot = block_sum(ss, sh.red, lane, wave);
    const double inv = 1.0 / sqrt(tot / double(H) + double(a.eps));
    for (int c = tid * VN; c < H; c += kBlock * VN) {
#pragma unroll
      for (int x = 0; x < VN; ++x) {
        double n = vec[c + x] * inv;
        if (a.bf16) n = round_to_bf16_fast(n);
        vec[c + x] = n;
      }
    }
    __syncthreads();
  }
  publish_rows(row_logit(rn), a.z_pred);
  if (wg != 0) return;

  // ---- (E^_{l+1}, G^_{l+1})
  select_topk_any(a.z_pred + size_t(b) * E, E, k, sh.sel, tid, a.spin_limit, a.status);
  if (tid < k) {
    const int id = sh.sel.top_i[tid];
    const float g = static_cast<float>(sh.sel.gate[tid]);
    const size_t o = size_t(b) * k + tid;
    a.next_ids[o] = id;
    a.next_gates[o] = g;
    if (a.user_next_ids) a.user_next_ids[o] = id;
    if (a.user_next_gates) a.user_next_gates[o] = g;
    if (a.mb_next) a.mb_next->ids[o] = id;
  }
  if (a.mb_next) post_mailbox(a.mb_next, a.seq_next, a.groups_done + 1, tid);
}

// ---------------------------------------------------------------------------------------------
// Expert FFN at batch 1, one launch

constexpr int kDownPre = 12;       // 16-byte weight chunks per lane a down-projection wavefront loads before it waits

// Workgroups [0, n_gateup_wg): hq[pos, row] = round(silu(W_gate[row,:] . s) * (W_up[row,:] . s)) for two rows per
// wavefront, all 4*NCH loads issued before anything is reduced; s_l in registers, no LDS, no barrier.
template <typename WT, int NCH>
__device__ __forceinline__ void gateup_role(const ExpertB1Args &a, int wg) {
  using R = Packed<WT>;
  constexpr int VN = R::N;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int H = a.H, I = a.I;
  const int pos = wg / a.gateup_wg_per_expert, blk = wg - pos * a.gateup_wg_per_expert;
  const int row0 = (blk * kWaves + wave) * 2;
  if (row0 >= I) return;
  const WT *wg_ = reinterpret_cast<const WT *>(a.pool + size_t(a.slot[pos]) * a.slot_bytes);
  const WT *wu = wg_ + size_t(I) * H;

  int col[NCH];
  bool live[NCH];
#pragma unroll
  for (int ch = 0; ch < NCH; ++ch) {
    col[ch] = (ch * kWave + lane) * VN;
    live[ch] = col[ch] < H;
    if (!live[ch]) col[ch] = 0;                // dead lanes re-read column 0 and multiply by zero
  }
  typename R::Raw rg[2][NCH], ru[2][NCH];
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    const int row = min(row0 + r, I - 1);
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      rg[r][ch] = load_stream<typename R::Raw>(wg_ + size_t(row) * H + col[ch]);
      ru[r][ch] = load_stream<typename R::Raw>(wu + size_t(row) * H + col[ch]);
    }
  }
  float sv[NCH][VN];
#pragma unroll
  for (int ch = 0; ch < NCH; ++ch) {
#pragma unroll
    for (int x = 0; x < VN; x += 4) {
      const float4 f = *reinterpret_cast<const float4 *>(a.s + col[ch] + x);
      const float m = live[ch] ? 1.f : 0.f;
      sv[ch][x] = f.x * m; sv[ch][x + 1] = f.y * m; sv[ch][x + 2] = f.z * m; sv[ch][x + 3] = f.w * m;
    }
  }
  float hv[2];
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    float ag = 0.f, au = 0.f;
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      float fg[VN], fu[VN];
      R::unpack(rg[r][ch], fg);
      R::unpack(ru[r][ch], fu);
#pragma unroll
      for (int x = 0; x < VN; ++x) { ag += fg[x] * sv[ch][x]; au += fu[x] * sv[ch][x]; }
    }
    const float g = wave_sum(ag);
    const float u = wave_sum(au);
    hv[r] = g / (1.f + expf(-g)) * u;
    if (a.bf16) hv[r] = round_to_bf16(hv[r]);
  }
  if (lane == 0) {
    // I is even and row0 is even: both rows exist.  One 4-byte word carries two bf16 values (or one float).
    const size_t e0 = size_t(pos) * I + row0;
    if (sizeof(WT) == 2) {
      uint32_t word = (__float_as_uint(hv[0]) >> 16) | (__float_as_uint(hv[1]) & 0xffff0000u);
      if (word == kEmpty32) word = 0x7fc07fc0u;            // two NaNs, but not the empty pattern
      __hip_atomic_store(a.hq + e0 / 2, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(a.hq_next + e0 / 2, kEmpty32, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        uint32_t word = __float_as_uint(hv[r]);
        if (word == kEmpty32) word = 0x7fc00000u;
        __hip_atomic_store(a.hq + e0 + r, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(a.hq_next + e0 + r, kEmpty32, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
}

// Workgroups [n_gateup_wg, ...): O[row] = sum_j gate_j * (W_down_{e_j}[row,:] . hq[j,:]), one output row per
// wavefront.  The k rows it needs are walked as one flat list of 16-byte chunks (chunk t belongs to expert
// t / chunks_per_expert).  A wavefront first issues the loads of its first kDownPre chunks per lane (the
// weights do not depend on hq), then the workgroup collects hq into LDS as the gate/up workgroups deliver
// it, then the chunks are multiplied; rows longer than 64 * kDownPre chunks stream the rest.
template <typename WT>
__device__ __forceinline__ void down_role(const ExpertB1Args &a, int wg, uint32_t *hq_lds) {
  using R = Packed<WT>;
  using Raw = typename R::Raw;
  constexpr int VN = R::N;
  __shared__ float gate_lds[kMaxTopK];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int H = a.H, I = a.I, k = a.k;
  const int row = wg * kWaves + wave;
  const bool valid = row < H;
  const int chunks = I / VN, total = chunks * k;
  const size_t down_off = (size_t(2) * I * H + size_t(valid ? row : 0) * I) * sizeof(WT);
  auto expert_of = [&](int t) {
    int j = int(float(t) * a.inv_chunks);      // t / chunks, fixed up (t < 2^24 is exact in float)
    j -= (j * chunks > t);
    j += ((j + 1) * chunks <= t);
    return j;
  };

  Raw w[kDownPre];
#pragma unroll
  for (int u = 0; u < kDownPre; ++u) {
    const int t = u * kWave + lane;
    if (valid && t < total) {
      const int j = expert_of(t);
      w[u] = load_stream<Raw>(a.pool + size_t(a.slot[j]) * a.slot_bytes + down_off + size_t(t - j * chunks) * 16);
    }
  }
  if (tid < k) gate_lds[tid] = a.gates[tid];
  const int n_words = total * 4;               // 4-byte words of hq
  for (int i0 = 0; i0 < n_words; i0 += kBlock * 8) {
    uint32_t v[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int i = i0 + q * kBlock + tid;
      v[q] = i < n_words ? __hip_atomic_load(a.hq + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int i = i0 + q * kBlock + tid;
      if (i < n_words) hq_lds[i] = await32(a.hq + i, v[q], a.spin_limit, a.status);
    }
  }
  __syncthreads();
  if (!valid) return;
  const uint4 *hq16 = reinterpret_cast<const uint4 *>(hq_lds);
  float acc = 0.f;
#pragma unroll
  for (int u = 0; u < kDownPre; ++u) {
    const int t = u * kWave + lane;
    if (t < total) {
      const int j = expert_of(t);
      const Raw hh = __builtin_bit_cast(Raw, hq16[t]);
      acc += gate_lds[j] * dot_chunk(w[u], hh, 0.f);
    }
  }
#pragma unroll 4
  for (int t = kDownPre * kWave + lane; t < total; t += kWave) {
    const int j = expert_of(t);
    const Raw ww = load_stream<Raw>(a.pool + size_t(a.slot[j]) * a.slot_bytes + down_off + size_t(t - j * chunks) * 16);
    const Raw hh = __builtin_bit_cast(Raw, hq16[t]);
    acc += gate_lds[j] * dot_chunk(ww, hh, 0.f);
  }
  const float v = wave_sum(acc);
  if (lane == 0) a.out[row] = v;
}

template <typename WT, int NCH>
__global__ __launch_bounds__(kBlock) void expert_b1_kernel(const ExpertB1Args a) {
  extern __shared__ __align__(16) uint32_t hq_lds[];
  const int wg = blockIdx.x;
  if (wg < a.n_gateup_wg) gateup_role<WT, NCH>(a, wg);
  else down_role<WT>(a, wg - a.n_gateup_wg, hq_lds);
}

// ---------------------------------------------------------------------------------------------
// Launchers

int g_compute_units = 0;

template <typename K>
hipError_t prepare_kernel(K kernel, size_t lds, int *blocks_per_cu) {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, 96 << 10);
  if (e != hipSuccess) return e;
  if (g_compute_units == 0) {
    int dev = 0;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
    if ((e = hipDeviceGetAttribute(&g_compute_units, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
  }
  return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, kernel, kBlock, lds);
}

template <typename WT, int SPLIT, int NCH>
hipError_t launch_route_pair_n(const RoutePairArgs &a, hipStream_t st) {
  constexpr int RPW = kWaves / SPLIT;
  const size_t lds = size_t(a.H) * sizeof(double);
  const int n_wg = (a.E + RPW - 1) / RPW;
  static int blocks_per_cu = -1;               // per instantiation
  static size_t checked_lds = 0;
  if (blocks_per_cu < 0 || lds > checked_lds) {
    int n = 0;
    hipError_t e = prepare_kernel(route_pair_kernel<WT, SPLIT, NCH>, lds, &n);
    if (e != hipSuccess) return e;
    blocks_per_cu = n;
    checked_lds = lds;
  }
  // the workgroups of a token wait for one another: they must fit on the device together
  if (long(n_wg) > long(blocks_per_cu) * g_compute_units) return hipErrorLaunchOutOfResources;
  hipLaunchKernelGGL((route_pair_kernel<WT, SPLIT, NCH>), dim3(n_wg, a.B), dim3(kBlock), lds, st, a);
  return hipGetLastError();
}

template <typename WT, int SPLIT>
hipError_t launch_route_pair_s(const RoutePairArgs &a, int need, hipStream_t st) {
  if (need <= 1) return launch_route_pair_n<WT, SPLIT, 1>(a, st);
  if (need <= 2) return launch_route_pair_n<WT, SPLIT, 2>(a, st);
  if (need <= 4) return launch_route_pair_n<WT, SPLIT, 4>(a, st);
  if (need <= 8) return launch_route_pair_n<WT, SPLIT, 8>(a, st);
  return hipErrorInvalidValue;
}

template <typename WT>
hipError_t launch_route_pair_t(const RoutePairArgs &a, hipStream_t st) {
  const int chunks = (a.H + Packed<WT>::N - 1) / Packed<WT>::N;
  const int need1 = (chunks + kWave - 1) / kWave;              // per lane, one wavefront per row
  const int need4 = (chunks + 4 * kWave - 1) / (4 * kWave);    // four wavefronts per row
  // one token: a workgroup per router row, so that E workgroups share the work; a batch: its tokens
  // already fill the device, four rows per workgroup keep the redundant normalisation down
  if (a.B > 1 && need1 <= 8) return launch_route_pair_s<WT, 1>(a, need1, st);
  return launch_route_pair_s<WT, 4>(a, need4, st);
}

template <typename WT, int NCH>
hipError_t launch_expert_b1_n(const ExpertB1Args &a, hipStream_t st) {
  const size_t lds = size_t(a.k) * a.I * sizeof(WT);
  static bool prepared = false;
  if (!prepared) {
    int n = 0;
    hipError_t e = prepare_kernel(expert_b1_kernel<WT, NCH>, 96 << 10, &n);
    if (e != hipSuccess) return e;
    prepared = true;
  }
  const int n_down = (a.H + kWaves - 1) / kWaves;
  hipLaunchKernelGGL((expert_b1_kernel<WT, NCH>), dim3(a.n_gateup_wg + n_down), dim3(kBlock), lds, st, a);
  return hipGetLastError();
}

template <typename WT>
hipError_t launch_expert_b1_t(const ExpertB1Args &a, hipStream_t st) {
  const int need = (a.H + kWave * Packed<WT>::N - 1) / (kWave * Packed<WT>::N);
  if (need <= 1) return launch_expert_b1_n<WT, 1>(a, st);
  if (need <= 2) return launch_expert_b1_n<WT, 2>(a, st);
  if (need <= 4) return launch_expert_b1_n<WT, 4>(a, st);
  return hipErrorInvalidValue;
}

}  // namespace

// H up to 64 * 4 * 8 chunks of 16 bytes per row (8192 columns of either dtype).
bool route_pair_supported(int H, int dtype) {
  const int vn = dtype == 1 ? 8 : 4;
  return (H + vn - 1) / vn <= 4 * kWave * 8;
}

hipError_t launch_route_pair(const RoutePairArgs &a, int dtype, hipStream_t st) {
  return dtype == 1 ? launch_route_pair_t<uint16_t>(a, st) : launch_route_pair_t<float>(a, st);
}

// Small launches only: every gate/up wavefront resident at once with its s_l in registers (at most
// four chunks per lane), and hq of all k experts in one workgroup's LDS.
bool expert_b1_fused_supported(int H, int I, int k, int dtype) {
  const int vn = dtype == 1 ? 8 : 4, wbytes = dtype == 1 ? 2 : 4;
  return (H + kWave * vn - 1) / (kWave * vn) <= 4 && long(I) * k <= 8192 && size_t(k) * I * wbytes <= kExpertB1MaxHqBytes;
}

hipError_t launch_expert_b1_fused(const ExpertB1Args &a, int dtype, hipStream_t st) {
  ExpertB1Args args = a;
  const int vn = dtype == 1 ? 8 : 4;
  args.gateup_wg_per_expert = (a.I + 2 * kWaves - 1) / (2 * kWaves);
  args.n_gateup_wg = args.gateup_wg_per_expert * a.k;
  args.inv_chunks = 1.0f / float(a.I / vn);
  return dtype == 1 ? launch_expert_b1_t<uint16_t>(args, st) : launch_expert_b1_t<float>(args, st);
}

}  // namespace moe_spec
