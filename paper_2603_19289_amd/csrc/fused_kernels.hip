// route_pair_kernel: the true routing of layer l AND the prediction for layer l+1 in one launch
// (paper: Sec. 3.1-3.3; Algorithm 1, TopK(Gate_l(X)) and GetNextExperts): RMSNorm, router l, top-k, gates,
// d_l, q_l, router l+1, top-k, gates.
//
// Logits are handed from the workgroups that compute them to the workgroups that need them inside
// the launch.  The hand-over is "the data is the flag": a slot of global memory holds a bit pattern that
// no result can have (all ones: a NaN) until its producer overwrites it with one relaxed device-scope
// atomic store; consumers read the slot with relaxed device-scope atomic loads until it no longer holds
// that pattern.  Each slot is a single atomic object, so nothing has to be ordered against anything
// else: no fence, no counter, no wait for a store's acknowledgement.  Slots come in two sets used by
// alternate launches; a launch re-arms the set the next launch will use (the previous launch, which
// read that set, has ended).  Every wait is bounded: after `spin_limit` polls a waiter gives up, raises
// the status word and finishes with whatever it has, so every wavefront reaches its end.
// Who may wait for whom: a workgroup only waits for the other workgroups of its own token, which the
// launcher checks to fit on the device together (groups are dispatched in order, so the earliest
// unfinished group always gets the next free compute units).
#include "device_utils.h"
#include "kernels.h"

namespace moe_spec {
namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / kWave;
// Development aid, compiled in with -DMOE_SPEC_STAGE_CLOCK only: workgroup 0 of token 0 notes the
// constant-rate clock (100 MHz) at the stages of the routing kernel.
#ifdef MOE_SPEC_STAGE_CLOCK
#define STAGE(i) do { if (a.stage_clock && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) a.stage_clock[i] = wall_clock64(); } while (0)
#else
#define STAGE(i) do { } while (0)
#endif

// ---------------------------------------------------------------------------------------------
// Routing

struct SelectShared {
  unsigned long long keys[kMaxExperts];   // the token's logits as order-preserving integers
  int cnt[kWaves][kMaxExperts];   // partial rank counts of the four wavefronts
  double top_z[kMaxTopK];
  double top_e[kMaxTopK];
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

// A double as an unsigned integer that orders the same way (the sign bit flipped for positive values, all
// bits for negative ones).  -0.0 never gets here: logits are published as v + 0.0.
__device__ __forceinline__ unsigned long long sortable(double v) {
  const unsigned long long u = static_cast<unsigned long long>(__double_as_longlong(v));
  return u ^ ((u >> 63) ? ~0ull : 0x8000000000000000ull);
}
__device__ __forceinline__ double unsortable(unsigned long long s) {
  const unsigned long long u = s ^ ((s >> 63) ? 0x8000000000000000ull : ~0ull);
  return __longlong_as_double(static_cast<long long>(u));
}
__device__ __forceinline__ unsigned long long readlane(unsigned long long v, int src_lane) {
  const unsigned int lo = __builtin_amdgcn_readlane(static_cast<unsigned int>(v), src_lane);
  const unsigned int hi = __builtin_amdgcn_readlane(static_cast<unsigned int>(v >> 32), src_lane);
  return (static_cast<unsigned long long>(hi) << 32) | lo;
}

// Top-k of one token's E logits, read from their slots as they arrive: larger logit first, equal logits by
// lower index.  Every wavefront holds all candidates in registers as order-preserving integers (element
// i = r*64 + lane, R per lane) and counts, for each of its candidates, how many candidates broadcast from
// source lanes [16 wave, 16 wave + 16) rank before it; the four partial counts of a candidate add up to
// its position in the sorted order.  Fills sel.top_i / sel.top_z (by descending logit), the same in every
// workgroup that calls it.
template <int R>
__device__ void select_ids(const RoutePairArgs &a, int stage, const unsigned long long *slots, int E, int k,
                           SelectShared &sel, int tid, int32_t *post) {
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  constexpr int kSrcPerWave = kWave / kWaves;
  // thread i waits for logit i (one look at every slot per workgroup, not one per wavefront) and shares it
  // through LDS; then every wavefront holds all candidates in registers
  static_assert(kMaxExperts == kBlock, "one thread per candidate");
  unsigned long long mine = 0ull;                // padding ranks below every logit, minus infinity included
  // A logit needs more than a microsecond to get from its producer to here, so the first look comes 0.4 us after
  // this workgroup's own logits went out.  Fewer polls in flight across the device let the stores themselves get
  // through sooner: both routings 12.9 -> 11.7 us on 128 experts (8 to 25 units of 64 cycles measure alike,
  // 45 units 12.7 us).
  __builtin_amdgcn_s_sleep(16);
  if (tid < E) {
    const double zi = __longlong_as_double(static_cast<long long>(await64(slots + tid, a.spin_limit, a.status)));
    // a logit that is not a number (an empty slot after a wait that ran out) sorts as minus infinity: the
    // order stays total whatever the input, so the k ids are distinct and inside [0, E)
    mine = sortable(zi == zi ? zi : -INFINITY);
  }
  sel.keys[tid] = mine;
  __syncthreads();
  unsigned long long key[R];
#pragma unroll
  for (int r = 0; r < R; ++r) key[r] = sel.keys[r * kWave + lane];
  STAGE(stage);
  int cnt[R];
#pragma unroll
  for (int r = 0; r < R; ++r) cnt[r] = 0;
  for (int j = wave * kSrcPerWave; j < (wave + 1) * kSrcPerWave; ++j) {
    const bool after = lane > j;                 // same register: the source has the lower index
#pragma unroll
    for (int r2 = 0; r2 < R; ++r2) {
      const unsigned long long sj = readlane(key[r2], j);
#pragma unroll
      for (int r = 0; r < R; ++r) {
        bool before;                             // does (r2, j) rank before (r, lane)?
        if (r2 < r) before = sj >= key[r];
        else if (r2 > r) before = sj > key[r];
        else before = sj > key[r] || (after && sj == key[r]);
        cnt[r] += before ? 1 : 0;
      }
    }
  }
#pragma unroll
  for (int r = 0; r < R; ++r) sel.cnt[wave][r * kWave + lane] = cnt[r];
  if (tid == 0) sel.hits = 0;
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int i = r * kWave + lane;
      const int rk = (sel.cnt[0][i] + sel.cnt[1][i]) + (sel.cnt[2][i] + sel.cnt[3][i]);
      if (i < E && rk < k) { sel.top_z[rk] = unsortable(key[r]); sel.top_i[rk] = i; }
    }
    // still in wavefront 0, whose own LDS writes it reads back in order: the ids go out to the host, if it waits
    // for them, and the numerators of the k gates are formed, before the other wavefronts are let go
    if (lane < k) {
      if (post) post[lane] = sel.top_i[lane];
      sel.top_e[lane] = exp(sel.top_z[lane] - sel.top_z[0]);
    }
  }
  __syncthreads();
}

__device__ __forceinline__ void select_ids_any(const RoutePairArgs &a, int stage, const unsigned long long *slots,
                                               int E, int k, SelectShared &sel, int tid, int32_t *post = nullptr) {
  if (E <= kWave) select_ids<1>(a, stage, slots, E, k, sel, tid, post);
  else if (E <= 2 * kWave) select_ids<2>(a, stage, slots, E, k, sel, tid, post);
  else select_ids<4>(a, stage, slots, E, k, sel, tid, post);
}

// Softmax over the k selected logits: select_ids left sel.top_e[j] = exp(z_j - z_0); returns their sum (the same
// in every thread), so that gate j is top_e[j] / sum.
__device__ __forceinline__ double select_gates(int k, SelectShared &sel, int tid) {
  (void)tid;
  double denom = 0.0;
  for (int q = 0; q < k; ++q) denom += sel.top_e[q];
  return denom;
}

// SPLIT wavefronts share one router row (4 / SPLIT rows per workgroup); NCH 16-byte chunks of the row
// per lane, loaded into registers for both routers at the top of the kernel so that their latency
// overlaps the normalisation.  blockIdx.y is the token; the workgroups of a token form a group that
// exchanges logits through the token's slots and computes everything else redundantly (the norm, the
// top-k, the default-vector sum), so that nothing but the 8-byte logits crosses between workgroups.
// Workgroup 0 of a token finishes the prediction; the last one reports the true routing, off the path
// that the prediction waits on.
template <typename WT, int SPLIT, int NCH, int ROWS>
__global__ __launch_bounds__(kBlock) void route_pair_kernel(const RoutePairArgs a) {
  static_assert(ROWS == 1 || SPLIT == 1, "several rows per wavefront only with one wavefront per row");
  // The router input being built, double precision, H values.  Threads own groups of VN consecutive columns (in
  // the norms: group tid, tid + 256, ...; in the products: the groups of the wavefront's chunks); column x of
  // group o lives at word x * G + o, so that the lanes of a wavefront, which hold consecutive groups, touch
  // consecutive words whatever x is (with the columns in their natural order every access of a wavefront fell
  // on a few banks)
  extern __shared__ double vec_lds[];
  __shared__ RouteShared sh;
  using P = Packed<WT>;
  using Raw = typename P::Raw;
  constexpr int VN = P::N;
  constexpr int RPW = kWaves / SPLIT * ROWS;   // rows per workgroup

  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int wg = blockIdx.x, b = blockIdx.y;
  const int H = a.H, E = a.E, k = a.k;
  const int G = H / VN;                        // column groups (H is a multiple of 8)
#define V(c, x) vec_lds[(x) * G + (c) / VN]
  const int row = wg * RPW + wave / SPLIT * ROWS, part = wave % SPLIT;   // this wavefront's (first) row
  const bool pred = a.w_next != nullptr;
  const WT *wt = static_cast<const WT *>(a.w_true);
  const WT *wn = static_cast<const WT *>(a.w_next);
  const float *rrow = a.r + size_t(b) * H;
  const int c0 = tid * VN;                     // this thread's columns of the first pass over the row
  STAGE(0);

  // ---- loads that depend on nothing, in the order they are needed: r_l and the gain first, then this
  // wavefront's part of its router rows (waited for at the products only)
  float r0[VN], g0[VN];
  if (c0 < H) {
#pragma unroll
    for (int x = 0; x < VN; x += 4) {
      const float4 f = *reinterpret_cast<const float4 *>(rrow + c0 + x);
      const float4 g = *reinterpret_cast<const float4 *>(a.gain_true + c0 + x);
      r0[x] = f.x; r0[x + 1] = f.y; r0[x + 2] = f.z; r0[x + 3] = f.w;
      g0[x] = g.x; g0[x + 1] = g.y; g0[x + 2] = g.z; g0[x + 3] = g.w;
    }
  }
  Raw rt[NCH], rn[NCH];                        // one row per wavefront: both routers' rows travel in registers
  if (ROWS == 1 && row < E) {
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
  {
    double ss = 0.0;
    double v0[VN];                               // this thread's first columns stay in registers until they are final
    if (c0 < H) {
#pragma unroll
      for (int x = 0; x < VN; ++x) { v0[x] = double(r0[x]) * double(g0[x]); ss += double(r0[x]) * double(r0[x]); }
    }
    for (int c = c0 + kBlock * VN; c < H; c += kBlock * VN) {
#pragma unroll
      for (int x = 0; x < VN; x += 4) {
        const float4 f = *reinterpret_cast<const float4 *>(rrow + c + x);
        const float4 g = *reinterpret_cast<const float4 *>(a.gain_true + c + x);
        V(c, x) = double(f.x) * double(g.x); V(c, x + 1) = double(f.y) * double(g.y);
        V(c, x + 2) = double(f.z) * double(g.z); V(c, x + 3) = double(f.w) * double(g.w);
        ss += double(f.x) * double(f.x) + double(f.y) * double(f.y) + double(f.z) * double(f.z) + double(f.w) * double(f.w);
      }
    }
    const double tot = block_sum(ss, sh.red, lane, wave);
    const double inv = 1.0 / sqrt(tot / double(H) + double(a.eps));
    for (int c = c0; c < H; c += kBlock * VN) {
#pragma unroll
      for (int x = 0; x < VN; ++x) {
        double n = (c == c0 ? v0[x] : V(c, x)) * inv;
        if (a.bf16) n = round_to_bf16_fast(n);
        V(c, x) = n;
      }
      if (wg == 0) {                             // s_l for the expert kernels, 16 bytes per store
#pragma unroll
        for (int x = 0; x < VN; x += 4)
          *reinterpret_cast<float4 *>(a.s_out + size_t(b) * H + c + x) =
              make_float4(float(V(c, x)), float(V(c, x + 1)), float(V(c, x + 2)), float(V(c, x + 3)));
        if (a.s_out_q) {
#pragma unroll
          for (int x = 0; x < VN; x += 2)
            *reinterpret_cast<uint32_t *>(a.s_out_q + size_t(b) * H + c + x) =
                (__float_as_uint(float(V(c, x))) >> 16) | (__float_as_uint(float(V(c, x + 1))) & 0xffff0000u);
        }
      }
    }
    __syncthreads();
  }
  STAGE(1);
  // ---- logits of a router: one row per SPLIT wavefronts from the registers loaded above, or (batches) ROWS
  //      rows per wavefront read where they are used, the router being in L2 after the first tokens
  auto dot_row = [&](const Raw (&w)[NCH]) {
    double acc = 0.0;
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      const int c = ((ch * SPLIT + part) * kWave + lane) * VN;
      if (c < H) {
        float wf[VN];
        P::unpack(w[ch], wf);
#pragma unroll
        for (int x = 0; x < VN; ++x) acc += double(wf[x]) * V(c, x);
      }
    }
    return wave_sum(acc);
  };
  auto publish_rows = [&](const Raw (&held)[NCH], const WT *wmat, unsigned long long *slots) {
    if (ROWS > 1) {
      Raw w[2][NCH];
      auto fetch = [&](int rr, Raw (&dst)[NCH]) {
        const int rclamped = min(row + rr, E - 1);
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
          const int c = (ch * kWave + lane) * VN;
          dst[ch] = *reinterpret_cast<const Raw *>(wmat + size_t(rclamped) * H + (c < H ? c : 0));
        }
      };
      fetch(0, w[0]);
#pragma unroll
      for (int rr = 0; rr < ROWS; ++rr) {
        if (rr + 1 < ROWS) fetch(rr + 1, w[(rr + 1) & 1]);
        const double acc = dot_row(w[rr & 1]);
        if (lane == 0 && row + rr < E) publish64(slots + size_t(b) * E + row + rr, acc);
      }
    } else if (SPLIT == 1) {
      const double acc = row < E ? dot_row(held) : 0.0;
      if (lane == 0 && row < E) publish64(slots + size_t(b) * E + row, acc);
    } else {
      const double acc = row < E ? dot_row(held) : 0.0;
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
  publish_rows(rt, wt, a.z_true);
  STAGE(2);
  const int reporter = gridDim.x - 1;
  if (!pred && wg != reporter) return;

  // ---- (E_l, G_l): every workgroup of the token selects for itself
  select_ids_any(a, 3, a.z_true + size_t(b) * E, E, k, sh.sel, tid);
  STAGE(4);
  // the first eight default-vector rows, asked for as soon as the ids are known; the gates follow meanwhile
  const WT *dv = static_cast<const WT *>(a.dvec);
  Raw dr0[8];
  if (pred && c0 < H) {
#pragma unroll
    for (int q = 0; q < 8; ++q) dr0[q] = *reinterpret_cast<const Raw *>(dv + size_t(sh.sel.top_i[min(q, k - 1)]) * H + c0);
  }
  float gn0[VN];
  if (pred && c0 < H) {
#pragma unroll
    for (int x = 0; x < VN; x += 4) {
      const float4 g = *reinterpret_cast<const float4 *>(a.gain_next + c0 + x);
      gn0[x] = g.x; gn0[x + 1] = g.y; gn0[x + 2] = g.z; gn0[x + 3] = g.w;
    }
  }
  const double denom = select_gates(k, sh.sel, tid);
  if (wg == reporter) {
    if (tid < k) {
      const int id = sh.sel.top_i[tid];
      const double g64 = sh.sel.top_e[tid] / denom;
      const float g = static_cast<float>(g64);
      const size_t o = size_t(b) * k + tid;
      if (a.mb_true) a.mb_true->ids[o] = id;     // the host waits for every word it armed
      a.true_ids[o] = id;
      a.true_gates[o] = g;
      if (a.true_gates64) a.true_gates64[o] = g64;
      if (a.user_true_ids) a.user_true_ids[o] = id;
      if (a.user_true_gates) a.user_true_gates[o] = g;
      if (a.cmp_ids) {                           // recall@k of the prediction made one layer earlier (Sec. 3.3)
        int hit = 0;
        for (int j = 0; j < k; ++j) hit |= (a.cmp_ids[size_t(b) * k + j] == id);
        if (hit) atomicAdd(&sh.sel.hits, 1);
      }
    }
    if (a.cmp_ids) {
      __syncthreads();
      if (tid == 0) {
        atomicAdd(&a.diag->hits, static_cast<unsigned long long>(sh.sel.hits));
        atomicAdd(&a.diag->preds, static_cast<unsigned long long>(k));
      }
    }
  }
  STAGE(5);
  if (!pred) return;

  // ---- d_l = sum_j g_j d_{l,e_j};  q_l = LN_{l+1}(r_l + d_l)   (or s_l + d_l, the caption's reading)
  {
    const double inv_denom = 1.0 / denom;
    double ss = 0.0;
    double q0[VN];                               // as in the first norm: the first columns stay in registers
    for (int c = c0; c < H; c += kBlock * VN) {
      const bool first = c == c0;
      double u[VN];
      if (a.from_normalized) {
#pragma unroll
        for (int x = 0; x < VN; ++x) u[x] = V(c, x);
      } else if (first) {
#pragma unroll
        for (int x = 0; x < VN; ++x) u[x] = r0[x];
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
          if (first && j0 == 0) dr[q] = dr0[q];
          else dr[q] = *reinterpret_cast<const Raw *>(dv + size_t(sh.sel.top_i[min(j0 + q, k - 1)]) * H + c);
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          if (j0 + q < k) {
            const double g = sh.sel.top_e[j0 + q] * inv_denom;
            float dvf[VN];
            P::unpack(dr[q], dvf);
#pragma unroll
            for (int x = 0; x < VN; ++x) d[x] += g * double(dvf[x]);
          }
        }
      }
      float gf[VN];
      if (first) {
#pragma unroll
        for (int x = 0; x < VN; ++x) gf[x] = gn0[x];
      } else {
#pragma unroll
        for (int x = 0; x < VN; x += 4) {
          const float4 g = *reinterpret_cast<const float4 *>(a.gain_next + c + x);
          gf[x] = g.x; gf[x + 1] = g.y; gf[x + 2] = g.z; gf[x + 3] = g.w;
        }
      }
#pragma unroll
      for (int x = 0; x < VN; ++x) {
        const double ux = u[x] + d[x];
        if (first) q0[x] = ux * double(gf[x]);
        else V(c, x) = ux * double(gf[x]);
        ss += ux * ux;
      }
    }
    STAGE(6);
    const double tot = block_sum(ss, sh.red, lane, wave);
    const double inv = 1.0 / sqrt(tot / double(H) + double(a.eps));
    for (int c = c0; c < H; c += kBlock * VN) {
#pragma unroll
      for (int x = 0; x < VN; ++x) {
        double n = (c == c0 ? q0[x] : V(c, x)) * inv;
        if (a.bf16) n = round_to_bf16_fast(n);
        V(c, x) = n;
      }
    }
    __syncthreads();
  }
  STAGE(7);
  publish_rows(rn, wn, a.z_pred);
  STAGE(8);
  if (wg != 0) return;

  // ---- (E^_{l+1}, G^_{l+1})
  select_ids_any(a, 9, a.z_pred + size_t(b) * E, E, k, sh.sel, tid,
                 a.mb_next ? a.mb_next->ids + size_t(b) * k : nullptr);                  // the host starts the prefetch on these
  const double denom_next = select_gates(k, sh.sel, tid);
  STAGE(10);
  if (tid < k) {
    const int id = sh.sel.top_i[tid];
    const float g = static_cast<float>(sh.sel.top_e[tid] / denom_next);
    const size_t o = size_t(b) * k + tid;
    a.next_ids[o] = id;
    a.next_gates[o] = g;
    if (a.user_next_ids) a.user_next_ids[o] = id;
    if (a.user_next_gates) a.user_next_gates[o] = g;
  }
  STAGE(11);
#undef V
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

template <typename WT, int SPLIT, int NCH, int ROWS>
hipError_t launch_route_pair_n(const RoutePairArgs &a, hipStream_t st) {
  constexpr int RPW = kWaves / SPLIT * ROWS;
  const size_t lds = size_t(a.H) * sizeof(double);
  const int n_wg = (a.E + RPW - 1) / RPW;
  static int blocks_per_cu = -1;               // per instantiation
  static size_t checked_lds = 0;
  if (blocks_per_cu < 0 || lds > checked_lds) {
    int n = 0;
    hipError_t e = prepare_kernel(route_pair_kernel<WT, SPLIT, NCH, ROWS>, lds, &n);
    if (e != hipSuccess) return e;
    blocks_per_cu = n;
    checked_lds = lds;
  }
  // the workgroups of a token wait for one another: they must fit on the device together
  if (long(n_wg) > long(blocks_per_cu) * g_compute_units) return hipErrorLaunchOutOfResources;
  hipLaunchKernelGGL((route_pair_kernel<WT, SPLIT, NCH, ROWS>), dim3(n_wg, a.B), dim3(kBlock), lds, st, a);
  return hipGetLastError();
}

template <typename WT, int SPLIT, int ROWS>
hipError_t launch_route_pair_s(const RoutePairArgs &a, int need, hipStream_t st) {
  if (need <= 1) return launch_route_pair_n<WT, SPLIT, 1, ROWS>(a, st);
  if (need <= 2) return launch_route_pair_n<WT, SPLIT, 2, ROWS>(a, st);
  if (need <= 4) return launch_route_pair_n<WT, SPLIT, 4, ROWS>(a, st);
  if (need <= 8) return launch_route_pair_n<WT, SPLIT, 8, ROWS>(a, st);
  return hipErrorInvalidValue;
}

template <typename WT>
hipError_t launch_route_pair_t(const RoutePairArgs &a, hipStream_t st) {
  const int chunks = (a.H + Packed<WT>::N - 1) / Packed<WT>::N;
  const int need1 = (chunks + kWave - 1) / kWave;              // per lane, one wavefront per row
  const int need4 = (chunks + 4 * kWave - 1) / (4 * kWave);    // four wavefronts per row
  // One token: a workgroup per router row, E workgroups (measured on 128 experts of 2048 columns: 11.4 us per
  // launch).  A batch: its tokens already fill the device, and every workgroup repeats its token's norm, top-k
  // and default-vector sum, so the more tokens, the more rows per workgroup: 4 up to about 512 workgroups per
  // launch, 16 beyond (measured before the polls were thinned out, which took about another
  // 0.5 us off each: 8 tokens x 128 experts: 13.5 us with 4 rows per workgroup, 14.4 with 8, 16.7 with 16;
  // 32 tokens: 28.6, 17.3, 17.3 us; 64 tokens: 53.8, 31.7, 21.2 us; 32 rows per workgroup: 21 to 22 us at all three).
  if (a.B > 1 && need1 <= 8) {
    const long wgs4 = long(a.B) * ((a.E + 3) / 4);
    if (wgs4 <= 512) return launch_route_pair_s<WT, 1, 1>(a, need1, st);
    return launch_route_pair_s<WT, 1, 4>(a, need1, st);
  }
  return launch_route_pair_s<WT, 4, 1>(a, need4, st);
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

}  // namespace moe_spec
