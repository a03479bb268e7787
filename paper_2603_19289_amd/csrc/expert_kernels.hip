// Expert kernels: SwiGLU expert GEMVs gathered over the device cache slots of one layer, and
// the gate-weighted combine (paper: Algorithm 1, O <- MoE_l(X, ids, g, C_l); Sec. 4 for which ids
// and gates are executed).
//
// A launch covers the experts of one cache wave.  blockIdx.y picks the expert, blockIdx.x a
// block of output rows.  Each workgroup finds the tokens routed to its expert by scanning the
// [B,k] id table, stages their activation vectors in LDS, and each wavefront streams whole
// weight rows with 16-byte loads per lane, reducing across the 64 lanes with shuffles.
// Weights are read once per token tile; at batch 1 that is exactly once.
#include "device_utils.h"
#include "kernels.h"

namespace moe_spec {
namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / kWave;

// Positions f = b*k + j of the id table that name expert e, in ascending order, by wavefront 0.
// All of the table's words a lane looks at are requested before the first is examined, so the
// scan costs one memory latency whatever the size of the table (at most 64 x 16 ids).
__device__ __forceinline__ void gather_tokens(const int32_t *ids, int n_ids, int e, int *list,
                                              int *n_list, int tid) {
  constexpr int kPerLane = kMaxBatch * kMaxTopK / kWave;
  if (tid < kWave) {
    int v[kPerLane];
#pragma unroll
    for (int i = 0; i < kPerLane; ++i) {
      const int f = i * kWave + tid;
      v[i] = f < n_ids ? ids[f] : -1;
    }
    int count = 0;
#pragma unroll
    for (int i = 0; i < kPerLane; ++i) {
      if (i * kWave < n_ids) {                 // uniform over the wavefront
        const bool match = v[i] == e;
        const unsigned long long mask = __ballot(match);
        if (match) list[count + __popcll(mask & ((1ull << tid) - 1ull))] = i * kWave + tid;
        count += __popcll(mask);
      }
    }
    if (tid == 0) *n_list = count;
  }
  __syncthreads();
}

// h[f, row] = silu(W_gate[row,:] . s_b) * (W_up[row,:] . s_b) for every position f routed to the expert.
template <typename WT, int TT>
__global__ __launch_bounds__(kBlock) void gateup_kernel(const ExpertArgs a, const ActiveList act,
                                                        const int rpw) {
  extern __shared__ float act_rows[];          // [TT][H]
  __shared__ int list[kMaxBatch];
  __shared__ int n_list;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int H = a.H, I = a.I;
  constexpr int VN = Packed<WT>::N;

  const int e = act.expert[blockIdx.y];
  const WT *wg = reinterpret_cast<const WT *>(a.pool + size_t(act.slot[blockIdx.y]) * a.slot_bytes);
  const WT *wu = wg + size_t(I) * H;
  gather_tokens(a.exec_ids, a.B * a.k, e, list, &n_list, tid);
  const int n = n_list;
  const int row0 = (blockIdx.x * kWaves + wave) * rpw;

  for (int t0 = 0; t0 < n; t0 += TT) {
    const int nt = min(TT, n - t0);
    for (int t = 0; t < nt; ++t) {
      const float *src = a.s + size_t(list[t0 + t] / a.k) * H;
      for (int i = tid * 4; i < H; i += kBlock * 4)
        *reinterpret_cast<float4 *>(act_rows + size_t(t) * H + i) = *reinterpret_cast<const float4 *>(src + i);
    }
    __syncthreads();
    for (int rr = 0; rr < rpw; ++rr) {
      const int row = row0 + rr;
      if (row >= I) break;
      float ag[TT], au[TT];
#pragma unroll
      for (int t = 0; t < TT; ++t) { ag[t] = 0.f; au[t] = 0.f; }
      const WT *pg = wg + size_t(row) * H;
      const WT *pu = wu + size_t(row) * H;
#pragma unroll 4
      for (int c = lane * VN; c < H; c += kWave * VN) {
        float fg[VN], fu[VN];
        Packed<WT>::unpack(load_stream<typename Packed<WT>::Raw>(pg + c), fg);
        Packed<WT>::unpack(load_stream<typename Packed<WT>::Raw>(pu + c), fu);
#pragma unroll
        for (int t = 0; t < TT; ++t) {
          if (t < nt) {
            const float *sv = act_rows + size_t(t) * H + c;
#pragma unroll
            for (int x = 0; x < VN; ++x) { ag[t] += fg[x] * sv[x]; au[t] += fu[x] * sv[x]; }
          }
        }
      }
#pragma unroll
      for (int t = 0; t < TT; ++t) {
        if (t < nt) {
          const float g = wave_sum(ag[t]);
          const float u = wave_sum(au[t]);
          if (lane == 0) {
            float hv = g / (1.f + expf(-g)) * u;
            if (a.bf16) hv = round_to_bf16(hv);
            a.h[size_t(list[t0 + t]) * I + row] = hv;
          }
        }
      }
    }
    __syncthreads();
  }
}

// y[f, row] = W_down[row,:] . h[f,:] for every position f routed to the expert.
template <typename WT, int TT>
__global__ __launch_bounds__(kBlock) void down_kernel(const ExpertArgs a, const ActiveList act,
                                                      const int rpw) {
  extern __shared__ float act_rows[];          // [TT][I]
  __shared__ int list[kMaxBatch];
  __shared__ int n_list;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int H = a.H, I = a.I;
  constexpr int VN = Packed<WT>::N;

  const int e = act.expert[blockIdx.y];
  const WT *wd = reinterpret_cast<const WT *>(a.pool + size_t(act.slot[blockIdx.y]) * a.slot_bytes) +
                 size_t(2) * I * H;
  gather_tokens(a.exec_ids, a.B * a.k, e, list, &n_list, tid);
  const int n = n_list;
  const int row0 = (blockIdx.x * kWaves + wave) * rpw;

  for (int t0 = 0; t0 < n; t0 += TT) {
    const int nt = min(TT, n - t0);
    for (int t = 0; t < nt; ++t) {
      const float *src = a.h + size_t(list[t0 + t]) * I;
      for (int i = tid * 4; i < I; i += kBlock * 4)
        *reinterpret_cast<float4 *>(act_rows + size_t(t) * I + i) = *reinterpret_cast<const float4 *>(src + i);
    }
    __syncthreads();
    for (int rr = 0; rr < rpw; ++rr) {
      const int row = row0 + rr;
      if (row >= H) break;
      float acc[TT];
#pragma unroll
      for (int t = 0; t < TT; ++t) acc[t] = 0.f;
      const WT *pw = wd + size_t(row) * I;
#pragma unroll 4
      for (int c = lane * VN; c < I; c += kWave * VN) {
        float fw[VN];
        Packed<WT>::unpack(load_stream<typename Packed<WT>::Raw>(pw + c), fw);
#pragma unroll
        for (int t = 0; t < TT; ++t) {
          if (t < nt) {
            const float *hv = act_rows + size_t(t) * I + c;
#pragma unroll
            for (int x = 0; x < VN; ++x) acc[t] += fw[x] * hv[x];
          }
        }
      }
#pragma unroll
      for (int t = 0; t < TT; ++t) {
        if (t < nt) {
          const float v = wave_sum(acc[t]);
          if (lane == 0) a.y[size_t(list[t0 + t]) * H + row] = v;
        }
      }
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------------
// Batch-1 kernels: no token lists, no staging barrier in the gate/up kernel, combine fused into
// the down kernel.  These are the kernels of the headline workload.

// hq[pos, row] for the one token of the batch, stored in the weight dtype for the down kernel.
// `act` is in execution-position order, so blockIdx.y is the position.  Each lane keeps its NCH
// chunks of s_l in registers; a wavefront owns `rpw` consecutive rows and keeps the 2*NCH
// 16-byte loads of the next row in flight while it reduces the current one.
template <typename WT, int NCH>
__global__ __launch_bounds__(kBlock) void gateup_b1_kernel(const ExpertArgs a, const ActiveList act,
                                                           const int rpw) {
  using R = Packed<WT>;
  constexpr int VN = R::N;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int H = a.H, I = a.I;
  const int row0 = (blockIdx.x * kWaves + wave) * rpw;
  if (row0 >= I) return;
  const int row_end = min(row0 + rpw, I);
  const int pos = blockIdx.y;
  const WT *wg = reinterpret_cast<const WT *>(a.pool + size_t(act.slot[pos]) * a.slot_bytes);
  const WT *wu = wg + size_t(I) * H;
  WT *hq = reinterpret_cast<WT *>(a.h) + size_t(pos) * I;

  int col[NCH];
  bool live[NCH];
#pragma unroll
  for (int ch = 0; ch < NCH; ++ch) {
    col[ch] = (ch * kWave + lane) * VN;
    live[ch] = col[ch] < H;
    if (!live[ch]) col[ch] = 0;                // dead lanes re-read column 0 and multiply by zero
  }
  typename R::Raw rg[NCH], ru[NCH];
#pragma unroll
  for (int ch = 0; ch < NCH; ++ch) {
    rg[ch] = load_stream<typename R::Raw>(wg + size_t(row0) * H + col[ch]);
    ru[ch] = load_stream<typename R::Raw>(wu + size_t(row0) * H + col[ch]);
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
  for (int row = row0; row < row_end; ++row) {
    float ag = 0.f, au = 0.f;
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      float fg[VN], fu[VN];
      R::unpack(rg[ch], fg);
      R::unpack(ru[ch], fu);
#pragma unroll
      for (int x = 0; x < VN; ++x) { ag += fg[x] * sv[ch][x]; au += fu[x] * sv[ch][x]; }
    }
    if (row + 1 < row_end) {
#pragma unroll
      for (int ch = 0; ch < NCH; ++ch) {
        rg[ch] = load_stream<typename R::Raw>(wg + size_t(row + 1) * H + col[ch]);
        ru[ch] = load_stream<typename R::Raw>(wu + size_t(row + 1) * H + col[ch]);
      }
    }
    const float g = wave_sum(ag);
    const float u = wave_sum(au);
    if (lane == 0) {
      float hv = g / (1.f + expf(-g)) * u;
      if (a.bf16) hv = round_to_bf16(hv);
      hq[row] = R::pack_one(hv);
    }
  }
}

// Small launches (all wavefronts resident at once): a wavefront owns two consecutive rows and
// issues the 4*NCH 16-byte loads of both before it reduces anything.
template <typename WT, int NCH>
__global__ __launch_bounds__(kBlock) void gateup_b1_pair_kernel(const ExpertArgs a, const ActiveList act) {
  using R = Packed<WT>;
  constexpr int VN = R::N;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int H = a.H, I = a.I;
  const int row0 = (blockIdx.x * kWaves + wave) * 2;
  if (row0 >= I) return;
  const int pos = blockIdx.y;
  const WT *wg = reinterpret_cast<const WT *>(a.pool + size_t(act.slot[pos]) * a.slot_bytes);
  const WT *wu = wg + size_t(I) * H;
  WT *hq = reinterpret_cast<WT *>(a.h) + size_t(pos) * I;

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
    const int row = min(row0 + r, I - 1);      // an odd last row is loaded twice and stored once
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      rg[r][ch] = load_stream<typename R::Raw>(wg + size_t(row) * H + col[ch]);
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
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    if (row0 + r >= I) break;
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
    if (lane == 0) {
      float hv = g / (1.f + expf(-g)) * u;
      if (a.bf16) hv = round_to_bf16(hv);
      hq[row0 + r] = R::pack_one(hv);
    }
  }
}

// O[row] = sum_j gate_j * (W_down_{e_j}[row,:] . hq[j,:]) for the one token of the batch: the down
// projection of all k executed experts and the gate-weighted combine in one pass.  SPLIT
// wavefronts share one output row.  The k rows it needs (one per expert, I values each) are
// walked as one flat list of 16-byte chunks so that all 64 lanes load on every iteration
// whatever I is; each lane folds the gate of its chunk's expert into its partial sum, one
// reduction per wavefront remains, and the SPLIT partial sums meet in LDS.  `act` is in
// execution-position order.
template <typename WT, int SPLIT, int UNROLL>
__global__ __launch_bounds__(kBlock) void down_combine_b1_kernel(const ExpertArgs a, const ActiveList act,
                                                                 const float inv_chunks) {
  using R = Packed<WT>;
  constexpr int VN = R::N;
  __shared__ float part_sum[kWaves];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int H = a.H, I = a.I, k = a.k;
  const int row = blockIdx.x * (kWaves / SPLIT) + wave / SPLIT;
  const int part = wave % SPLIT;
  const bool valid = row < H;
  const int chunks = I / VN;                   // per expert row
  const int total = chunks * k;
  const WT *hq = reinterpret_cast<const WT *>(a.h);
  const size_t down_off = (size_t(2) * I * H + size_t(valid ? row : 0) * I) * sizeof(WT);
  float acc = 0.f;
  if (valid) {
#pragma unroll UNROLL
    for (int t = part * kWave + lane; t < total; t += kWave * SPLIT) {
      int j = int(float(t) * inv_chunks);      // t / chunks, fixed up below (t < 2^24 is exact in float)
      j -= (j * chunks > t);
      j += ((j + 1) * chunks <= t);
      const int c = (t - j * chunks) * VN;
      const char *base = a.pool + size_t(act.slot[j]) * a.slot_bytes + down_off;
      const typename R::Raw w = load_stream<typename R::Raw>(base + size_t(c) * sizeof(WT));
      const typename R::Raw hh = *reinterpret_cast<const typename R::Raw *>(hq + size_t(j) * I + c);
      acc += a.exec_gates[j] * dot_chunk(w, hh, 0.f);
    }
  }
  const float v = wave_sum(acc);
  if (SPLIT == 1) {
    if (lane == 0 && valid) a.out[row] = v;
  } else {
    if (lane == 0) part_sum[wave] = v;
    __syncthreads();
    if (lane == 0 && part == 0 && valid) {
      float tot = 0.f;
#pragma unroll
      for (int p = 0; p < SPLIT; ++p) tot += part_sum[wave + p];
      a.out[row] = tot;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Matrix-core kernels for decode batches of two and more (bf16 weights) and for prefill: the
// expert FFN as 16x16x32 bf16 MFMA tiles.  The launches stay HBM-bound, but one weight fragment
// meets up to 16 tokens per instruction, where the general kernels above fetch every token's
// activations from LDS for every weight chunk and are LDS-bound from a few tokens on.  A operand = 16 weight rows, B operand = up to 16 tokens routed to the expert, K walks
// the reduction dimension 64 columns per step: lane (m, g) = (lane % 16, lane / 16) loads the 32
// contiguous bytes at column k0 + 16 g of row m (so four lanes cover one 128-byte line) and
// feeds the first 8 columns to one MFMA and the next 8 to a second one; the B operand is read
// with the same column assignment, which is all that the contraction needs.
// Accumulator layout: lane holds token column lane % 16, rows 4 (lane / 16) .. +3.

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

__device__ __forceinline__ bf16x8_t load_bf16x8(const uint16_t *p, bool valid) {
  uint4 v = make_uint4(0u, 0u, 0u, 0u);
  if (valid) v = *reinterpret_cast<const uint4 *>(p);
  return __builtin_bit_cast(bf16x8_t, v);
}

// One step of the reduction for one wavefront: the weight fragments of its 16 rows and the token
// fragments of up to NT tiles, each the 2 x 16 bytes a lane feeds to two MFMAs.
template <bool GATEUP, int NT>
struct MfmaStep {
  bf16x8_t w0[2], w1[2];       // rows of W_gate (or W_down), rows of W_up
  bf16x8_t x[NT][2];
};

// GATEUP: hq[f, row] = bf16(silu(W_gate[row,:] . s_b) * (W_up[row,:] . s_b)),  act_q = s_l as bf16 [tokens, K]
// else  : y[f, row]  = W_down[row,:] . hq[f,:],                                  act_q = hq [tokens*k, K]
// The positions f = b*k + j routed to the expert come either from the [B,k] id table of a decode
// batch (B <= 64, one grid plane) or, with a.pos_list, from per-expert lists over any number of
// tokens, 64 positions per grid plane blockIdx.z.  Weights are read with ordinary loads: a lane's
// two 16-byte loads of a step take alternate quarters of the same 128-byte lines, and the planes
// of an expert share its weights through the caches; streaming loads measured 8-10 % slower here.
template <bool GATEUP, int NT, int KSPLIT>
__global__ __launch_bounds__(kBlock) void expert_mfma_kernel(const ExpertArgs a, const ActiveList act,
                                                             const uint16_t *act_q, uint16_t *hq_out) {
  __shared__ int list[kMaxBatch];
  __shared__ int n_list;
  // partial accumulators of the wavefronts that share a tile: [wave][token tile][gate | up][register][lane]
  __shared__ float partial[KSPLIT > 1 ? kWaves : 1][NT][GATEUP ? 2 : 1][4][kWave];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int m = lane & 15, g = lane >> 4;
  const int K = GATEUP ? a.H : a.I;            // reduction length
  const int R = GATEUP ? a.I : a.H;            // output rows

  const int e = act.expert[blockIdx.y];
  const uint16_t *wbase = reinterpret_cast<const uint16_t *>(a.pool + size_t(act.slot[blockIdx.y]) * a.slot_bytes);
  // KSPLIT wavefronts share 16 output rows: they split the reduction dimension into equal parts
  // (whole 64-column steps) and add their partial tiles in LDS.  Many short chains of dependent
  // loads that start at different columns keep HBM busier than few long ones that walk their rows
  // in step: a read-only probe of this access pattern reaches 6.2 TB/s with four wavefronts per 16
  // rows against 4.6 TB/s with one.  Short reductions are not split: the launcher picks KSPLIT.
  const int row_base = (blockIdx.x * (kWaves / KSPLIT) + wave / KSPLIT) * 16;
  const int part = wave % KSPLIT;
  const bool rows_inside = row_base < R;       // a workgroup's last tiles may lie past the matrix
  const int k_part = (K + KSPLIT * 64 - 1) / (KSPLIT * 64) * 64;
  const int k_begin = part * k_part, k_end = rows_inside ? min(K, k_begin + k_part) : k_begin;
  const int my_row = min(row_base + m, R - 1);
  const uint16_t *p0 = wbase + (GATEUP ? size_t(0) : size_t(2) * a.I * a.H) + size_t(my_row) * K;
  const uint16_t *p1 = p0 + size_t(a.I) * a.H;             // W_up row (GATEUP only)

  // columns past the wavefront's part load nothing and contribute zeros, so the staged loop
  // below may run one step beyond the end
  auto fetch_w = [&](int k0, MfmaStep<GATEUP, NT> &st) {
    const int kk = k0 + 16 * g;
    const bool v0 = kk < k_end, v1 = kk + 8 < k_end;
    st.w0[0] = load_bf16x8(p0 + kk, v0);
    st.w0[1] = load_bf16x8(p0 + kk + 8, v1);
    if (GATEUP) { st.w1[0] = load_bf16x8(p1 + kk, v0); st.w1[1] = load_bf16x8(p1 + kk + 8, v1); }
  };
  MfmaStep<GATEUP, NT> even, odd;              // the loads of one step are in flight during the other's MFMAs
  // down projection with up to two token tiles: the first weights are on their way while the token list is
  // built (measured: 6 % faster there; 7 % slower in the gate/up kernel, which has twice the weight registers
  // per step, and 20 % slower with four token tiles, as in prefill)
  constexpr bool kEarlyWeights = !GATEUP && NT <= 2;
  if (kEarlyWeights) fetch_w(k_begin, even);

  int n;
  if (a.pos_list) {
    const int first = blockIdx.z * kMaxBatch;
    n = min(kMaxBatch, a.pos_count[e] - first);
    if (n <= 0) return;                        // the same for the whole workgroup
    if (tid < n) list[tid] = a.pos_list[size_t(e) * a.list_stride + first + tid];
    __syncthreads();
  } else {
    gather_tokens(a.exec_ids, a.B * a.k, e, list, &n_list, tid);
    n = n_list;
  }
  if (n == 0) return;                          // the same for the whole workgroup
  if (KSPLIT == 1 && !rows_inside) return;     // nothing to share, nobody waits for this wavefront
  const int ntiles = (n + 15) / 16;

  const uint16_t *bp[NT];
  bool bvalid[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int idx = t * 16 + m;
    bvalid[t] = idx < n;
    const int f = bvalid[t] ? list[idx] : 0;
    bp[t] = act_q + size_t(GATEUP ? f / a.k : f) * K;
  }
  f32x4_t acc0[NT], acc1[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) { acc0[t] = f32x4_t{0.f, 0.f, 0.f, 0.f}; acc1[t] = f32x4_t{0.f, 0.f, 0.f, 0.f}; }

  auto fetch_x = [&](int k0, MfmaStep<GATEUP, NT> &st) {
    const int kk = k0 + 16 * g;
    const bool v0 = kk < k_end, v1 = kk + 8 < k_end;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      if (t < ntiles) {
        st.x[t][0] = load_bf16x8(bp[t] + kk, v0 && bvalid[t]);
        st.x[t][1] = load_bf16x8(bp[t] + kk + 8, v1 && bvalid[t]);
      }
    }
  };
  auto fetch = [&](int k0, MfmaStep<GATEUP, NT> &st) { fetch_w(k0, st); fetch_x(k0, st); };
  auto multiply = [&](const MfmaStep<GATEUP, NT> &st) {
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      if (t < ntiles) {
        acc0[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(st.w0[0], st.x[t][0], acc0[t], 0, 0, 0);
        acc0[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(st.w0[1], st.x[t][1], acc0[t], 0, 0, 0);
        if (GATEUP) {
          acc1[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(st.w1[0], st.x[t][0], acc1[t], 0, 0, 0);
          acc1[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(st.w1[1], st.x[t][1], acc1[t], 0, 0, 0);
        }
      }
    }
  };
  if (kEarlyWeights) fetch_x(k_begin, even);
  else fetch(k_begin, even);
  for (int k0 = k_begin; k0 < k_end; k0 += 128) {
    fetch(k0 + 64, odd);
    multiply(even);
    fetch(k0 + 128, even);
    multiply(odd);
  }

  if (KSPLIT > 1) {
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      if (t < ntiles) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          partial[wave][t][0][i][lane] = acc0[t][i];
          if (GATEUP) partial[wave][t][GATEUP ? 1 : 0][i][lane] = acc1[t][i];
        }
      }
    }
    __syncthreads();
  }

  // Of the wavefronts that share a tile, number p finishes token tiles p, p + KSPLIT, ...  The
  // accumulator layout is as the MFMA left it: lane = token column lane % 16, rows 4 (lane / 16) .. + 3.
  const int r0 = row_base + 4 * g;             // this lane's four output rows, all inside or all outside
  if (r0 >= R) return;
  const int w0 = wave - part;                  // first of the wavefronts that share this tile
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    if (t % KSPLIT == part && t < ntiles && bvalid[t]) {
      float s0[4], s1[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (KSPLIT == 1) {
          s0[i] = acc0[t][i];
          s1[i] = acc1[t][i];
        } else {
          s0[i] = 0.f;
          s1[i] = 0.f;
#pragma unroll
          for (int p = 0; p < KSPLIT; ++p) {
            s0[i] += partial[w0 + p][t][0][i][lane];
            if (GATEUP) s1[i] += partial[w0 + p][t][GATEUP ? 1 : 0][i][lane];
          }
        }
      }
      const int f = list[t * 16 + m];
      if (GATEUP) {
        uint16_t q[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float hv = round_to_bf16(s0[i] / (1.f + expf(-s0[i])) * s1[i]);
          q[i] = uint16_t(__float_as_uint(hv) >> 16);
        }
        uint2 packed;
        packed.x = uint32_t(q[0]) | (uint32_t(q[1]) << 16);
        packed.y = uint32_t(q[2]) | (uint32_t(q[3]) << 16);
        *reinterpret_cast<uint2 *>(hq_out + size_t(f) * R + r0) = packed;
      } else {
        *reinterpret_cast<float4 *>(a.y + size_t(f) * R + r0) = make_float4(s0[0], s0[1], s0[2], s0[3]);
      }
    }
  }
}

// Positions f = b*k + j of an id table [tokens, k], grouped by expert, ascending inside a group:
// pos[e*stride + i] for i < count[e].  One workgroup per expert; each wavefront counts and then
// writes its own contiguous quarter of the table.
__global__ __launch_bounds__(kBlock) void expert_lists_kernel(const int32_t *ids, int n_ids, int stride,
                                                              int32_t *pos, int32_t *count) {
  __shared__ int wave_count[kWaves];
  const int e = blockIdx.x, tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int per_wave = (n_ids + kBlock - 1) / kBlock * kWave;
  const int lo = wave * per_wave, hi = min(n_ids, lo + per_wave);
  int c = 0;
  for (int base = lo; base < hi; base += kWave) {
    const int f = base + lane;
    c += __popcll(__ballot(f < hi && ids[f] == e));
  }
  if (lane == 0) wave_count[wave] = c;
  __syncthreads();
  int off = 0, total = 0;
  for (int w = 0; w < kWaves; ++w) { if (w < wave) off += wave_count[w]; total += wave_count[w]; }
  for (int base = lo; base < hi; base += kWave) {
    const int f = base + lane;
    const bool match = f < hi && ids[f] == e;
    const unsigned long long mask = __ballot(match);
    if (match) pos[size_t(e) * stride + off + __popcll(mask & ((1ull << lane) - 1ull))] = f;
    off += __popcll(mask);
  }
  if (tid == 0) count[e] = total;
}

// Default-vector statistics (paper: Sec. 3.1, the offline aggregation behind d_{l,e}): for every
// position f routed to an expert of this launch, sum[e,:] += y[f,:] and cnt[e] += 1.
__global__ __launch_bounds__(kBlock) void accumulate_defaults_kernel(const ExpertArgs a, const ActiveList act,
                                                                     double *sum, unsigned long long *cnt) {
  const int f = blockIdx.y;
  const int e = a.exec_ids[f];
  bool mine = false;
  for (int i = 0; i < act.n; ++i) mine |= act.expert[i] == e;
  if (!mine) return;
  const int i = blockIdx.x * kBlock + threadIdx.x;
  if (i < a.H) atomicAdd(sum + size_t(e) * a.H + i, double(a.y[size_t(f) * a.H + i]));
  if (i == 0) atomicAdd(cnt + e, 1ull);
}

__global__ __launch_bounds__(kBlock) void default_means_kernel(const double *sum, const unsigned long long *cnt,
                                                               float *mean, int H) {
  const int e = blockIdx.y, i = blockIdx.x * kBlock + threadIdx.x;
  if (i >= H) return;
  const unsigned long long n = cnt[e];
  mean[size_t(e) * H + i] = n ? float(sum[size_t(e) * H + i] / double(n)) : 0.f;
}

// Measurement aid: reads a range of 16-byte units of the launch's slots and does nothing else (the
// sum is never stored unless it hits an impossible value).  What a kernel can reach on these bytes.
__global__ __launch_bounds__(kBlock) void stream_read_kernel(const ExpertArgs a, const ActiveList act, size_t first16,
                                                             size_t n16, float *sink) {
  const uint4 *p = reinterpret_cast<const uint4 *>(a.pool + size_t(act.slot[blockIdx.y]) * a.slot_bytes) + first16;
  const size_t stride = size_t(gridDim.x) * kBlock;
  float acc = 0.f;
  for (size_t i = size_t(blockIdx.x) * kBlock + threadIdx.x; i < n16; i += stride) {
    const uint4 v = load_stream<uint4>(p + i);
    acc += __uint_as_float(v.x ^ v.y ^ v.z ^ v.w);
  }
  if (acc == 1.2345e-30f) *sink = acc;
}

// O[b, i] = sum_j gates[b, j] * y[b, j, i]
__global__ __launch_bounds__(kBlock) void combine_kernel(const ExpertArgs a) {
  const int i = blockIdx.x * kBlock + threadIdx.x;
  const int b = blockIdx.y;
  if (i >= a.H) return;
  float acc = 0.f;
  for (int j = 0; j < a.k; ++j)
    acc += a.exec_gates[b * a.k + j] * a.y[(size_t(b) * a.k + j) * a.H + i];
  a.out[size_t(b) * a.H + i] = acc;
}

// Host-to-device copy of whole expert blocks by a few workgroups that read the pinned pool
// directly.  blockIdx.y picks the block, the workgroups of a row share it in 16-byte units.
// kCopyUnroll loads are in flight per lane; the launch keeps the bytes in flight near the link's
// bandwidth-delay product, because host reads that queue up in the memory system delay the
// HBM requests of kernels running beside the copy.
constexpr int kCopyWorkgroups = 16, kCopyUnroll = 2;      // 16 x 256 lanes x 2 x 16 B = 128 KB in flight
__global__ __launch_bounds__(kBlock) void gather_copy_kernel(const CopyList cl) {
  const uint4 *src = static_cast<const uint4 *>(cl.src[blockIdx.y]);
  uint4 *dst = static_cast<uint4 *>(cl.dst[blockIdx.y]);
  const uint32_t n = cl.n16;
  const uint32_t stride = gridDim.x * kBlock;
  uint32_t i = blockIdx.x * kBlock + threadIdx.x;
  for (; i + (kCopyUnroll - 1) * stride < n; i += kCopyUnroll * stride) {
    uint4 v[kCopyUnroll];
#pragma unroll
    for (int u = 0; u < kCopyUnroll; ++u) v[u] = src[i + u * stride];
#pragma unroll
    for (int u = 0; u < kCopyUnroll; ++u) dst[i + u * stride] = v[u];
  }
  for (; i < n; i += stride) dst[i] = src[i];
}

int pick_tok_tile(int B, int row_len) {
  int tt = 1;
  while (tt < B && tt < 8) tt <<= 1;
  while (tt > 1 && size_t(tt) * row_len * sizeof(float) > (size_t(60) << 10)) tt >>= 1;
  return tt;
}

int pick_rows_per_wave(int rows, int n_active) {
  // aim for about 2048 workgroups so that all 256 compute units hold several
  const long total = long(rows) * n_active;
  long rpw = total / (long(kWaves) * 2048);
  if (rpw < 1) rpw = 1;
  if (rpw > 8) rpw = 8;
  return int(rpw);
}

template <typename WT>
hipError_t launch_gateup_t(const ExpertArgs &a, const ActiveList &act, hipStream_t st) {
  const int tt = pick_tok_tile(a.B, a.H);
  const int rpw = pick_rows_per_wave(a.I, act.n);
  const size_t lds = size_t(tt) * a.H * sizeof(float);
  const dim3 grid((a.I + kWaves * rpw - 1) / (kWaves * rpw), act.n), block(kBlock);
  switch (tt) {
    case 1: hipLaunchKernelGGL((gateup_kernel<WT, 1>), grid, block, lds, st, a, act, rpw); break;
    case 2: hipLaunchKernelGGL((gateup_kernel<WT, 2>), grid, block, lds, st, a, act, rpw); break;
    case 4: hipLaunchKernelGGL((gateup_kernel<WT, 4>), grid, block, lds, st, a, act, rpw); break;
    default: hipLaunchKernelGGL((gateup_kernel<WT, 8>), grid, block, lds, st, a, act, rpw); break;
  }
  return hipGetLastError();
}

template <typename WT>
hipError_t launch_down_t(const ExpertArgs &a, const ActiveList &act, hipStream_t st) {
  const int tt = pick_tok_tile(a.B, a.I);
  const int rpw = pick_rows_per_wave(a.H, act.n);
  const size_t lds = size_t(tt) * a.I * sizeof(float);
  const dim3 grid((a.H + kWaves * rpw - 1) / (kWaves * rpw), act.n), block(kBlock);
  switch (tt) {
    case 1: hipLaunchKernelGGL((down_kernel<WT, 1>), grid, block, lds, st, a, act, rpw); break;
    case 2: hipLaunchKernelGGL((down_kernel<WT, 2>), grid, block, lds, st, a, act, rpw); break;
    case 4: hipLaunchKernelGGL((down_kernel<WT, 4>), grid, block, lds, st, a, act, rpw); break;
    default: hipLaunchKernelGGL((down_kernel<WT, 8>), grid, block, lds, st, a, act, rpw); break;
  }
  return hipGetLastError();
}

template <typename WT, int NCH>
void launch_gateup_b1_n(const ExpertArgs &a, const ActiveList &act, hipStream_t st) {
  const dim3 block(kBlock);
  // up to 4096 wavefronts of two rows each are all resident at once (137 registers at NCH = 4)
  if (NCH <= 4 && long(a.I) * act.n <= 8192) {
    const dim3 grid((a.I + 2 * kWaves - 1) / (2 * kWaves), act.n);
    hipLaunchKernelGGL((gateup_b1_pair_kernel<WT, NCH>), grid, block, 0, st, a, act);
    return;
  }
  // one row per wavefront until that would exceed about 6144 wavefronts (24 per compute unit)
  long rpw = (long(a.I) * act.n + 6143) / 6144;
  if (rpw < 1) rpw = 1;
  const dim3 grid((a.I + kWaves * rpw - 1) / (kWaves * rpw), act.n);
  hipLaunchKernelGGL((gateup_b1_kernel<WT, NCH>), grid, block, 0, st, a, act, int(rpw));
}

// Returns false when H needs more register chunks than the batch-1 kernel is built for.
template <typename WT>
bool launch_gateup_b1(const ExpertArgs &a, const ActiveList &act, hipStream_t st) {
  constexpr int VN = Packed<WT>::N;
  const int need = (a.H + kWave * VN - 1) / (kWave * VN);
  if (need <= 1) launch_gateup_b1_n<WT, 1>(a, act, st);
  else if (need <= 2) launch_gateup_b1_n<WT, 2>(a, act, st);
  else if (need <= 4) launch_gateup_b1_n<WT, 4>(a, act, st);
  else if (need <= 6) launch_gateup_b1_n<WT, 6>(a, act, st);
  else if (need <= 8) launch_gateup_b1_n<WT, 8>(a, act, st);
  else if (need <= 16) launch_gateup_b1_n<WT, 16>(a, act, st);
  else return false;
  return true;
}

template <typename WT, int SPLIT, int UNROLL>
void launch_down_combine_b1_n(const ExpertArgs &a, const ActiveList &act, hipStream_t st) {
  const dim3 grid((a.H + kWaves / SPLIT - 1) / (kWaves / SPLIT)), block(kBlock);
  const float inv_chunks = 1.0f / float(a.I / Packed<WT>::N);
  hipLaunchKernelGGL((down_combine_b1_kernel<WT, SPLIT, UNROLL>), grid, block, 0, st, a, act, inv_chunks);
}

// The loop of a wavefront is unrolled UNROLL times, so that many loads per lane are in flight
// together; where a row's chunk list is short enough, SPLIT is chosen so that each wavefront's
// share is exactly one such batch (iterations beyond a multiple of UNROLL run one by one).
// Otherwise four wavefronts per row and batches of four, the best measured on the 1440- and
// 3584-chunk rows of the larger workloads.
template <typename WT>
void launch_down_combine_b1(const ExpertArgs &a, const ActiveList &act, hipStream_t st) {
  const long chunks = long(a.I / Packed<WT>::N) * a.k;
  const long iters = chunks % kWave == 0 ? chunks / kWave : 0;      // per row, for one wavefront
  if (iters == 4) launch_down_combine_b1_n<WT, 1, 4>(a, act, st);
  else if (iters == 6) launch_down_combine_b1_n<WT, 1, 6>(a, act, st);
  else if (iters == 8) launch_down_combine_b1_n<WT, 2, 4>(a, act, st);
  else if (iters == 12) launch_down_combine_b1_n<WT, 2, 6>(a, act, st);
  else launch_down_combine_b1_n<WT, 4, 4>(a, act, st);
}

template <bool GATEUP, int KSPLIT>
hipError_t launch_expert_mfma_k(const ExpertArgs &a, const ActiveList &act, const uint16_t *act_q, uint16_t *hq,
                                hipStream_t st) {
  const int rows = GATEUP ? a.I : a.H;
  const int rows_per_wg = 16 * kWaves / KSPLIT;
  const int planes = a.pos_list ? (a.list_tokens + kMaxBatch - 1) / kMaxBatch : 1;
  const dim3 grid((rows + rows_per_wg - 1) / rows_per_wg, act.n, planes), block(kBlock);
  const int nt = a.pos_list ? (std::min(a.list_tokens, kMaxBatch) + 15) / 16 : (a.B + 15) / 16;
  switch (nt) {
    case 1: hipLaunchKernelGGL((expert_mfma_kernel<GATEUP, 1, KSPLIT>), grid, block, 0, st, a, act, act_q, hq); break;
    case 2: hipLaunchKernelGGL((expert_mfma_kernel<GATEUP, 2, KSPLIT>), grid, block, 0, st, a, act, act_q, hq); break;
    case 3: hipLaunchKernelGGL((expert_mfma_kernel<GATEUP, 3, KSPLIT>), grid, block, 0, st, a, act, act_q, hq); break;
    default: hipLaunchKernelGGL((expert_mfma_kernel<GATEUP, 4, KSPLIT>), grid, block, 0, st, a, act, act_q, hq); break;
  }
  return hipGetLastError();
}

// Wavefronts per 16-row tile by the length of the reduction: each should still walk at least
// eight 64-column steps, below that the shared start-up (token lists, partial sums) outweighs
// what the extra parallelism wins.
template <bool GATEUP>
hipError_t launch_expert_mfma(const ExpertArgs &a, const ActiveList &act, const uint16_t *act_q, uint16_t *hq,
                              hipStream_t st) {
  const int steps = ((GATEUP ? a.H : a.I) + 63) / 64;
  if (steps >= 32) return launch_expert_mfma_k<GATEUP, 4>(a, act, act_q, hq, st);
  if (steps >= 16) return launch_expert_mfma_k<GATEUP, 2>(a, act, act_q, hq, st);
  return launch_expert_mfma_k<GATEUP, 1>(a, act, act_q, hq, st);
}

template <typename K>
hipError_t allow_big_lds(K kernel) {
  return hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                             hipFuncAttributeMaxDynamicSharedMemorySize, 128 << 10);
}

}  // namespace

hipError_t launch_gateup(const ExpertArgs &a, const ActiveList &act, int dtype, hipStream_t st) {
  if (act.n <= 0) return hipSuccess;
  return dtype == 1 ? launch_gateup_t<uint16_t>(a, act, st) : launch_gateup_t<float>(a, act, st);
}

// Batch 1, `act` in execution-position order.  H up to 64*16 chunks (8192 bf16 / 4096 float32 columns).
bool b1_supported(int H, int dtype) { return H <= kWave * 16 * (dtype == 1 ? 8 : 4); }

hipError_t launch_gateup_b1(const ExpertArgs &a, const ActiveList &act, int dtype, hipStream_t st) {
  const bool ok = dtype == 1 ? launch_gateup_b1<uint16_t>(a, act, st) : launch_gateup_b1<float>(a, act, st);
  return ok ? hipGetLastError() : hipErrorInvalidValue;
}

// Batch 1: down projection and combine in one kernel (the k executed experts are always one cache
// wave); reads the hq written by launch_gateup_b1.
hipError_t launch_down_combine_b1(const ExpertArgs &a, const ActiveList &act, int dtype, hipStream_t st) {
  if (dtype == 1) launch_down_combine_b1<uint16_t>(a, act, st);
  else launch_down_combine_b1<float>(a, act, st);
  return hipGetLastError();
}

hipError_t launch_down(const ExpertArgs &a, const ActiveList &act, int dtype, hipStream_t st) {
  if (act.n <= 0) return hipSuccess;
  return dtype == 1 ? launch_down_t<uint16_t>(a, act, st) : launch_down_t<float>(a, act, st);
}

// bf16 weights, batch >= kMfmaMinBatch: s_q is s_l as bf16 [B,H]; hq (bf16 [B,k,I]) is written by the gate/up
// launch and read by the down launch.
hipError_t launch_gateup_mfma(const ExpertArgs &a, const ActiveList &act, const uint16_t *s_q, uint16_t *hq,
                              hipStream_t st) {
  if (act.n <= 0) return hipSuccess;
  return launch_expert_mfma<true>(a, act, s_q, hq, st);
}

hipError_t launch_down_mfma(const ExpertArgs &a, const ActiveList &act, const uint16_t *hq, hipStream_t st) {
  if (act.n <= 0) return hipSuccess;
  return launch_expert_mfma<false>(a, act, hq, nullptr, st);
}

hipError_t launch_expert_lists(const int32_t *ids, int tokens, int k, int E, int32_t *pos, int32_t *count,
                               hipStream_t st) {
  hipLaunchKernelGGL(expert_lists_kernel, dim3(E), dim3(kBlock), 0, st, ids, tokens * k, tokens, pos, count);
  return hipGetLastError();
}

hipError_t launch_gather_copy(const CopyList &cl, hipStream_t st) {
  if (cl.n <= 0) return hipSuccess;
  const int wg_per_block = (kCopyWorkgroups + cl.n - 1) / cl.n;
  hipLaunchKernelGGL(gather_copy_kernel, dim3(wg_per_block, cl.n), dim3(kBlock), 0, st, cl);
  return hipGetLastError();
}

hipError_t launch_accumulate_defaults(const ExpertArgs &a, const ActiveList &act, double *sum,
                                      unsigned long long *cnt, hipStream_t st) {
  const dim3 grid((a.H + kBlock - 1) / kBlock, a.B * a.k), block(kBlock);
  hipLaunchKernelGGL(accumulate_defaults_kernel, grid, block, 0, st, a, act, sum, cnt);
  return hipGetLastError();
}

hipError_t launch_default_means(const double *sum, const unsigned long long *cnt, float *mean, int E, int H,
                                hipStream_t st) {
  const dim3 grid((H + kBlock - 1) / kBlock, E), block(kBlock);
  hipLaunchKernelGGL(default_means_kernel, grid, block, 0, st, sum, cnt, mean, H);
  return hipGetLastError();
}

hipError_t launch_stream_read(const ExpertArgs &a, const ActiveList &act, size_t first16, size_t n16, hipStream_t st) {
  hipLaunchKernelGGL(stream_read_kernel, dim3(768, act.n), dim3(kBlock), 0, st, a, act, first16, n16, a.out);
  return hipGetLastError();
}

hipError_t launch_combine(const ExpertArgs &a, hipStream_t st) {
  const dim3 grid((a.H + kBlock - 1) / kBlock, a.B), block(kBlock);
  hipLaunchKernelGGL(combine_kernel, grid, block, 0, st, a);
  return hipGetLastError();
}

hipError_t init_route_kernels();

hipError_t init_kernels() {
  hipError_t e = init_route_kernels();
#define MOE_SPEC_ALLOW(k) if (e == hipSuccess) e = allow_big_lds(k)
  MOE_SPEC_ALLOW((gateup_kernel<uint16_t, 1>)); MOE_SPEC_ALLOW((gateup_kernel<uint16_t, 2>));
  MOE_SPEC_ALLOW((gateup_kernel<uint16_t, 4>)); MOE_SPEC_ALLOW((gateup_kernel<uint16_t, 8>));
  MOE_SPEC_ALLOW((gateup_kernel<float, 1>)); MOE_SPEC_ALLOW((gateup_kernel<float, 2>));
  MOE_SPEC_ALLOW((gateup_kernel<float, 4>)); MOE_SPEC_ALLOW((gateup_kernel<float, 8>));
  MOE_SPEC_ALLOW((down_kernel<uint16_t, 1>)); MOE_SPEC_ALLOW((down_kernel<uint16_t, 2>));
  MOE_SPEC_ALLOW((down_kernel<uint16_t, 4>)); MOE_SPEC_ALLOW((down_kernel<uint16_t, 8>));
  MOE_SPEC_ALLOW((down_kernel<float, 1>)); MOE_SPEC_ALLOW((down_kernel<float, 2>));
  MOE_SPEC_ALLOW((down_kernel<float, 4>)); MOE_SPEC_ALLOW((down_kernel<float, 8>));
#undef MOE_SPEC_ALLOW
  return e;
}

}  // namespace moe_spec
