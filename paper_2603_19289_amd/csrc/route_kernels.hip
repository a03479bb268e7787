// Routing kernels: RMSNorm + router GEMV + top-k + softmax gates, for the true routing of a
// layer and for the prediction of the next layer's routing from the quasi-hidden state
// (paper: Sec. 3.1-3.3; Algorithm 1, TopK(Gate_l(X)) and GetNextExperts).
//
// One launch covers the whole batch: grid dimension y is the token, so tokens run side by side and a
// batch costs little more than its slowest token.  Every workgroup of a token normalises the token's input row itself (a few KB from L2),
// keeps it in LDS in double precision, and one wavefront per router row reads that row once
// with 16-byte loads.  Logits go to self-flagging slots in global memory; workgroup 0 of the token
// reads them as they arrive, rank-sorts them in registers (keys stay in VGPRs, broadcast lane
// by lane through scalar registers), writes ids and gates, scores the previous prediction and
// writes the ids to a pinned host mailbox.  Everything that decides an expert index is double precision.
// Layer order of the default-vector sum follows the id order (descending logit).
#include "device_utils.h"
#include "kernels.h"

namespace moe_spec {
namespace {

constexpr int kMaxTokTile = 1;     // tokens a workgroup handles (one: see route_lds_bytes)

struct FinishShared {
  double keys[kMaxExperts];          // the token's logits, one thread having waited for each
  int rank[kMaxExperts];
  double top_z[kMaxTopK];
  double top_e[kMaxTopK];
  int top_i[kMaxTopK];
  int hits;
};

// Top-k, gates and bookkeeping of the group's tokens by its workgroup 0, which reads the logits from their slots
// as the other workgroups deliver them.
template <int R>
__device__ void finish_tokens(const RouteArgs &a, FinishShared &sh, int tid, int b_begin, int b_end) {
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  constexpr int kSrcPerWave = kWave / (kRouteBlock / kWave);
  static_assert(kMaxExperts == kRouteBlock, "one thread per candidate");
  if (tid == 0) sh.hits = 0;
  // the other workgroups' logits need more than a microsecond to get here: no look before 0.4 us have passed
  // (polls in flight hold up the stores they are waiting for)
  __builtin_amdgcn_s_sleep(16);
  for (int b = b_begin; b < b_end; ++b) {
    // Thread i waits for logit i and shares it through LDS: one look at every slot per workgroup.
    // A logit that is not a number (a non-finite input row) sorts as minus infinity: comparisons
    // with NaN are all false, ranks would collide, and slots of the top-k table would keep whatever
    // the LDS held - ids far outside [0, E) that later kernels use as row indices.  With this the
    // order (logit descending, index ascending) is total whatever the input, and ids stay in range.
    double mine = -INFINITY;
    if (tid < a.E) {
      const double zi = __longlong_as_double(static_cast<long long>(await64(a.slots + size_t(b) * a.E + tid, a.spin_limit, a.status)));
      mine = zi == zi ? zi : -INFINITY;
    }
    sh.keys[tid] = mine;
    sh.rank[tid] = 0;
    __syncthreads();
    double key[R];
#pragma unroll
    for (int r = 0; r < R; ++r) key[r] = sh.keys[r * kWave + lane];
    int cnt[R];
    rank_counts<R>(key, lane, wave * kSrcPerWave, (wave + 1) * kSrcPerWave, cnt);
#pragma unroll
    for (int r = 0; r < R; ++r) atomicAdd(&sh.rank[r * kWave + lane], cnt[r]);
    __syncthreads();
    if (wave == 0) {
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const int i = r * kWave + lane;
        const int rk = sh.rank[i];
        if (i < a.E && rk < a.k) { sh.top_z[rk] = key[r]; sh.top_i[rk] = i; }
      }
    }
    __syncthreads();
    double my_exp = 0.0;
    if (tid < a.k) {
      my_exp = exp(sh.top_z[tid] - sh.top_z[0]);
      sh.top_e[tid] = my_exp;
    }
    __syncthreads();
    if (tid < a.k) {
      double denom = 0.0;
      for (int q = 0; q < a.k; ++q) denom += sh.top_e[q];
      const double g = my_exp / denom;
      const int id = sh.top_i[tid];
      const size_t o = size_t(b) * a.k + tid;
      a.ids_out[o] = id;
      a.gates_out[o] = static_cast<float>(g);
      if (a.gates64_out) a.gates64_out[o] = g;
      if (a.user_ids) a.user_ids[o] = id;
      if (a.user_gates) a.user_gates[o] = static_cast<float>(g);
      if (a.mailbox) a.mailbox->ids[o] = id;
      if (a.cmp_ids) {
        int hit = 0;
        for (int j = 0; j < a.k; ++j) hit |= (a.cmp_ids[size_t(b) * a.k + j] == id);
        if (hit) atomicAdd(&sh.hits, 1);
        if (a.rank_stats && a.cmp_ids[o] == id) atomicAdd(&a.diag->rank_match[tid], 1ull);
      }
    }
    __syncthreads();
  }
  if (tid == 0 && a.cmp_ids) {
    atomicAdd(&a.diag->hits, static_cast<unsigned long long>(sh.hits));
    atomicAdd(&a.diag->preds, static_cast<unsigned long long>(a.k) * (b_end - b_begin));
  }
}

// NCH > 0: the wavefront's router row (NCH 16-byte chunks per lane) is loaded into registers at
// the top of the kernel, so its HBM latency overlaps the normalisation; NCH = 0 streams the row
// in a loop for hidden sizes beyond 64*8 chunks.
template <typename WT, int NCH>
__global__ __launch_bounds__(kRouteBlock) void route_kernel(const RouteArgs a) {
  extern __shared__ double vec[];            // [tok_tile][H]
  __shared__ double red[kRouteBlock / kWave];
  __shared__ double red3[3][kRouteBlock / kWave];
  __shared__ FinishShared fin;

  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int row = blockIdx.x * kRouteRowsPerBlock + wave;
  const WT *w = static_cast<const WT *>(a.w);
  const WT *dv = static_cast<const WT *>(a.dvec);
  const int H = a.H;
  constexpr int VN = Packed<WT>::N;
  using Raw = typename Packed<WT>::Raw;

  constexpr int NREG = NCH > 0 ? NCH : 1;
  Raw wreg[NREG];
  if (NCH > 0 && row < a.E) {
#pragma unroll
    for (int ch = 0; ch < NREG; ++ch) {
      const int c = (ch * kWave + lane) * VN;
      wreg[ch] = *reinterpret_cast<const Raw *>(w + size_t(row) * H + (c < H ? c : 0));
    }
  }

  // re-arm both sets of slots the next routing launch may use (last read by the previous launch, which has ended)
  for (int i = (blockIdx.y * gridDim.x + blockIdx.x) * kRouteBlock + tid; i < a.arm_count; i += gridDim.x * gridDim.y * kRouteBlock) {
    arm64(a.arm_a + i);
    arm64(a.arm_b + i);
  }
  const int b_begin = blockIdx.y * a.tok_tile, b_end = min(a.B, b_begin + a.tok_tile);   // this group's tokens
  for (int b0 = b_begin; b0 < b_end; b0 += a.tok_tile) {
    const int nb = min(a.tok_tile, b_end - b0);
    for (int t = 0; t < nb; ++t) {
      const int b = b0 + t;
      double *v = vec + size_t(t) * H;
      if (a.spec == 3) {                          // LayerNorm of the estimator's latent vector
        double sum = 0.0;
        for (int i = tid; i < H; i += kRouteBlock) {
          const double x = a.x_f64[size_t(b) * H + i];
          v[i] = x;
          sum += x;
        }
        sum = wave_sum(sum);
        __syncthreads();
        if (lane == 0) red[wave] = sum;
        __syncthreads();
        const double mean = ((red[0] + red[1]) + (red[2] + red[3])) / double(H);
        double sq = 0.0;
        for (int i = tid; i < H; i += kRouteBlock) { const double d = v[i] - mean; sq += d * d; }
        sq = wave_sum(sq);
        __syncthreads();
        if (lane == 0) red[wave] = sq;
        __syncthreads();
        const double root = sqrt(((red[0] + red[1]) + (red[2] + red[3])) / double(H) + double(a.eps));
        for (int i = tid; i < H; i += kRouteBlock)
          v[i] = (v[i] - mean) / root * double(a.gain[i]) + double(a.bias[i]);
        continue;
      }
      if (a.spec == 2) {                          // s_l as it is: no default vector, no second norm
        for (int i = tid; i < H; i += kRouteBlock) {
          const float x = a.s_in[size_t(b) * H + i];
          v[i] = double(x);
          if (blockIdx.x == 0 && a.vec_out) a.vec_out[size_t(b) * H + i] = x;
        }
        continue;
      }
      double ss = 0.0;
      for (int c = tid * VN; c < H; c += kRouteBlock * VN) {     // VN consecutive elements per thread
        double u[VN];
        const float *base = (a.spec && a.from_normalized ? a.s_in : a.r) + size_t(b) * H + c;
#pragma unroll
        for (int x = 0; x < VN; x += 4) {
          const float4 f = *reinterpret_cast<const float4 *>(base + x);
          u[x] = f.x; u[x + 1] = f.y; u[x + 2] = f.z; u[x + 3] = f.w;
        }
        if (a.spec) {
          double d[VN];
#pragma unroll
          for (int x = 0; x < VN; ++x) d[x] = 0.0;
          for (int j0 = 0; j0 < a.k; j0 += 4) {            // four default-vector rows in flight
            Raw dr[4];
            double g[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const int j = min(j0 + q, a.k - 1);
              g[q] = j0 + q < a.k ? a.d_gates[b * a.k + j] : 0.0;
              dr[q] = *reinterpret_cast<const Raw *>(dv + size_t(a.d_ids[b * a.k + j]) * H + c);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              float dvf[VN];
              Packed<WT>::unpack(dr[q], dvf);
#pragma unroll
              for (int x = 0; x < VN; ++x) d[x] += g[q] * double(dvf[x]);
            }
          }
#pragma unroll
          for (int x = 0; x < VN; ++x) u[x] += d[x];
        }
        float gf[VN];                                    // gains now, so that no load follows the reduction
#pragma unroll
        for (int x = 0; x < VN; x += 4) {
          const float4 f = *reinterpret_cast<const float4 *>(a.gain + c + x);
          gf[x] = f.x; gf[x + 1] = f.y; gf[x + 2] = f.z; gf[x + 3] = f.w;
        }
#pragma unroll
        for (int x = 0; x < VN; ++x) { v[c + x] = u[x] * double(gf[x]); ss += u[x] * u[x]; }
      }
      ss = wave_sum(ss);
      __syncthreads();                       // red[] free again
      if (lane == 0) red[wave] = ss;
      __syncthreads();
      double tot = 0.0;
#pragma unroll
      for (int x = 0; x < kRouteBlock / kWave; ++x) tot += red[x];
      const double root = sqrt(tot / double(H) + double(a.eps));
      for (int i = tid; i < H; i += kRouteBlock) {
        double n = v[i] / root;                          // v holds x*gain
        if (a.bf16) n = round_to_bf16(n);
        v[i] = n;
        if (blockIdx.x == 0 && a.vec_out) a.vec_out[size_t(b) * H + i] = static_cast<float>(n);
        if (blockIdx.x == 0 && a.vec_out_q)
          a.vec_out_q[size_t(b) * H + i] = uint16_t(__float_as_uint(static_cast<float>(n)) >> 16);
      }
      if (blockIdx.x == 0 && a.prev_signal) {     // cosine between the predicting signal and s_l
        __syncthreads();
        double dot = 0.0, pp = 0.0, qq = 0.0;
        for (int i = tid; i < H; i += kRouteBlock) {
          const double p = double(a.prev_signal[size_t(b) * H + i]), q = v[i];
          dot += p * q; pp += p * p; qq += q * q;
        }
        dot = wave_sum(dot); pp = wave_sum(pp); qq = wave_sum(qq);
        if (lane == 0) { red3[0][wave] = dot; red3[1][wave] = pp; red3[2][wave] = qq; }
        __syncthreads();
        if (tid == 0) {
          double t[3];
          for (int x = 0; x < 3; ++x) t[x] = (red3[x][0] + red3[x][1]) + (red3[x][2] + red3[x][3]);
          atomicAdd(&a.diag->cos_sum, t[0] / sqrt(t[1] * t[2]));
          atomicAdd(&a.diag->cos_count, 1ull);
        }
      }
    }
    __syncthreads();

    if (row < a.E) {
      double acc[kMaxTokTile];
#pragma unroll
      for (int t = 0; t < kMaxTokTile; ++t) acc[t] = 0.0;
      if (NCH > 0) {
#pragma unroll
        for (int ch = 0; ch < NREG; ++ch) {
          const int c = (ch * kWave + lane) * VN;
          if (c < H) {
            float wf[VN];
            Packed<WT>::unpack(wreg[ch], wf);
#pragma unroll
            for (int t = 0; t < kMaxTokTile; ++t) {
              if (t < nb) {
                const double *v = vec + size_t(t) * H + c;
#pragma unroll
                for (int x = 0; x < VN; ++x) acc[t] += double(wf[x]) * v[x];
              }
            }
          }
        }
      } else {
        const WT *wr = w + size_t(row) * H;
        for (int c0 = lane * VN; c0 < H; c0 += 4 * kWave * VN) {     // four chunks in flight
          Raw wr4[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int c = c0 + u * kWave * VN;
            wr4[u] = *reinterpret_cast<const Raw *>(wr + (c < H ? c : 0));
          }
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int c = c0 + u * kWave * VN;
            if (c < H) {
              float wf[VN];
              Packed<WT>::unpack(wr4[u], wf);
#pragma unroll
              for (int t = 0; t < kMaxTokTile; ++t) {
                if (t < nb) {
                  const double *v = vec + size_t(t) * H + c;
#pragma unroll
                  for (int x = 0; x < VN; ++x) acc[t] += double(wf[x]) * v[x];
                }
              }
            }
          }
        }
      }
#pragma unroll
      for (int t = 0; t < kMaxTokTile; ++t) {
        if (t < nb) {
          const double s = wave_sum(acc[t]);
          if (lane == 0) publish64(a.slots + size_t(b0 + t) * a.E + row, s);
        }
      }
    }
    __syncthreads();                         // vec is rewritten by the next tile
  }

  // Workgroup 0 of the group collects the logits (it waits, boundedly, only for workgroups of its own group,
  // a few dozen at most, which fit on the device together), selects, reports and writes the ids to the host.
  if (blockIdx.x != 0) return;
  if (a.E <= kWave) finish_tokens<1>(a, fin, tid, b_begin, b_end);
  else if (a.E <= 2 * kWave) finish_tokens<2>(a, fin, tid, b_begin, b_end);
  else finish_tokens<4>(a, fin, tid, b_begin, b_end);
}

}  // namespace

// One token per group: the per-token chain (load, reduce, normalise, row products, hand-over, sort)
// is a sequence of dependent latencies, so tokens side by side in separate workgroups finish in
// the time of one, while tokens one after the other in one workgroup add about 10 us each.  The
// router rows are then read once per token, from L2 after the first.
size_t route_lds_bytes(int H, int B, int *tok_tile) {
  (void)B;
  *tok_tile = 1;
  return size_t(H) * sizeof(double);
}

template <typename WT, int NCH>
hipError_t launch_route_n(const RouteArgs &args, size_t lds, hipStream_t st) {
  static bool big_lds_allowed = false;       // dynamic LDS above the 64 KB default is opt-in
  if (!big_lds_allowed) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(route_kernel<WT, NCH>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 96 << 10);
    if (e != hipSuccess) return e;
    big_lds_allowed = true;
  }
  const dim3 grid((args.E + kRouteRowsPerBlock - 1) / kRouteRowsPerBlock,
                  (args.B + args.tok_tile - 1) / args.tok_tile), block(kRouteBlock);
  hipLaunchKernelGGL((route_kernel<WT, NCH>), grid, block, lds, st, args);
  return hipGetLastError();
}

template <typename WT>
hipError_t launch_route_t(const RouteArgs &args, size_t lds, hipStream_t st) {
  const int need = (args.H + kWave * Packed<WT>::N - 1) / (kWave * Packed<WT>::N);
  if (need <= 1) return launch_route_n<WT, 1>(args, lds, st);
  if (need <= 2) return launch_route_n<WT, 2>(args, lds, st);
  if (need <= 4) return launch_route_n<WT, 4>(args, lds, st);
  if (need <= 6) return launch_route_n<WT, 6>(args, lds, st);
  if (need <= 8) return launch_route_n<WT, 8>(args, lds, st);
  return launch_route_n<WT, 0>(args, lds, st);
}

hipError_t launch_route(const RouteArgs &a, int dtype, hipStream_t st) {
  RouteArgs args = a;
  const size_t lds = route_lds_bytes(a.H, a.B, &args.tok_tile);
  return dtype == 1 ? launch_route_t<uint16_t>(args, lds, st) : launch_route_t<float>(args, lds, st);
}

hipError_t init_route_kernels() { return hipSuccess; }

}  // namespace moe_spec
