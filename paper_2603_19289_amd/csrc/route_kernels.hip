// Routing kernels: RMSNorm + router GEMV + top-k + softmax gates, for the true routing of a
// layer and for the prediction of the next layer's routing from the quasi-hidden state
// (paper: Sec. 3.1-3.3; Algorithm 1, TopK(Gate_l(X)) and GetNextExperts).
//
// One launch covers the whole batch.  Every workgroup normalises the input rows itself (they
// are a few KB and sit in L2), keeps them in LDS in double precision, and one wavefront per
// router row streams that row once with 16-byte loads.  Logits go to global memory; the last
// workgroup to arrive (a ticket counter, no waiting) sorts them in registers, one wavefront per
// token, writes ids and gates, scores the previous prediction, and posts the ids to a pinned
// host mailbox.  Everything that decides an expert index is double precision.
#include "kernels.h"

namespace moe_spec {
namespace {

constexpr int kWave = 64;
constexpr int kMaxTokTile = 4;

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int m = 32; m > 0; m >>= 1) v += __shfl_xor(v, m);
  return v;
}

// Nearest bfloat16 (8 significant bits), ties to even, straight from the double.
__device__ __forceinline__ double round_to_bf16(double x) {
  if (x == 0.0) return x;
  int e;
  const double m = frexp(x, &e);
  return ldexp(rint(m * 256.0), e - 8);
}

// 16 bytes of weights -> floats.  bf16: 8 values, float: 4 values.
template <typename WT> struct Chunk;
template <> struct Chunk<uint16_t> {
  static constexpr int N = 8;
  __device__ static void load(const uint16_t *p, float (&f)[8]) {
    const uint4 v = *reinterpret_cast<const uint4 *>(p);
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
    f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
    f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
  }
  __device__ static float one(const uint16_t *p) { return __uint_as_float(uint32_t(*p) << 16); }
};
template <> struct Chunk<float> {
  static constexpr int N = 4;
  __device__ static void load(const float *p, float (&f)[4]) {
    const float4 v = *reinterpret_cast<const float4 *>(p);
    f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
  }
  __device__ static float one(const float *p) { return *p; }
};

__device__ __forceinline__ double load_coherent(const double *p) {
  const unsigned long long u = __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p),
                                                 __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return __longlong_as_double(static_cast<long long>(u));
}

// (za, ia) ranks before (zb, ib): larger logit first, equal logits by lower index.
__device__ __forceinline__ bool ranks_before(double za, int ia, double zb, int ib) {
  return za > zb || (za == zb && ia < ib);
}

// Bitonic sort of 64*R (logit, index) pairs held R per lane, element i = lane*R + r, into rank
// order.  Afterwards rank p sits in lane p / R, register p % R.
template <int R>
__device__ __forceinline__ void wave_rank_sort(double (&key)[R], int (&idx)[R], int lane) {
  constexpr int N = kWave * R;
#pragma unroll
  for (int k2 = 2; k2 <= N; k2 <<= 1) {
#pragma unroll
    for (int j = k2 >> 1; j > 0; j >>= 1) {
      if (j >= R) {
        const int lj = j / R;
        const bool lower = (lane & lj) == 0;
#pragma unroll
        for (int r = 0; r < R; ++r) {
          const int i = lane * R + r;
          const double ok = __shfl_xor(key[r], lj);
          const int oi = __shfl_xor(idx[r], lj);
          const bool up = (i & k2) == 0;
          const bool want_first = lower == up;
          const bool other_first = ranks_before(ok, oi, key[r], idx[r]);
          if (want_first == other_first) { key[r] = ok; idx[r] = oi; }
        }
      } else {
#pragma unroll
        for (int r = 0; r < R; ++r) {
          if ((r & j) == 0) {
            const int r2 = r | j;
            const bool up = ((lane * R + r) & k2) == 0;
            const bool second_first = ranks_before(key[r2], idx[r2], key[r], idx[r]);
            if (second_first == up) {
              const double tk = key[r]; key[r] = key[r2]; key[r2] = tk;
              const int ti = idx[r]; idx[r] = idx[r2]; idx[r2] = ti;
            }
          }
        }
      }
    }
  }
}

// Top-k, gates and bookkeeping for one token by one wavefront.
template <int R>
__device__ void finish_token(const RouteArgs &a, int b, int lane) {
  double key[R];
  int idx[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int i = lane * R + r;
    idx[r] = i;
    key[r] = i < a.E ? load_coherent(a.z + size_t(b) * a.E + i) : -INFINITY;
  }
  wave_rank_sort<R>(key, idx, lane);

  const double zmax = __shfl(key[0], 0);
  double ex[R];
  double part = 0.0;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int p = lane * R + r;
    ex[r] = p < a.k ? exp(key[r] - zmax) : 0.0;
    part += ex[r];
  }
  const double denom = wave_sum(part);

  int my_hits = 0;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int p = lane * R + r;
    if (p < a.k) {
      const double g = ex[r] / denom;
      const size_t o = size_t(b) * a.k + p;
      a.ids_out[o] = idx[r];
      a.gates_out[o] = static_cast<float>(g);
      if (a.gates64_out) a.gates64_out[o] = g;
      if (a.user_ids) a.user_ids[o] = idx[r];
      if (a.user_gates) a.user_gates[o] = static_cast<float>(g);
      if (a.mailbox) a.mailbox->ids[o] = idx[r];
      if (a.cmp_ids) {
        for (int j = 0; j < a.k; ++j) my_hits += (a.cmp_ids[size_t(b) * a.k + j] == idx[r]);
      }
    }
  }
  if (a.cmp_ids) {
    int h = my_hits;
#pragma unroll
    for (int m = 32; m > 0; m >>= 1) h += __shfl_xor(h, m);
    if (lane == 0) {
      atomicAdd(&a.hit_counters[0], static_cast<unsigned long long>(h));
      atomicAdd(&a.hit_counters[1], static_cast<unsigned long long>(a.k));
    }
  }
}

template <typename WT>
__global__ __launch_bounds__(kRouteBlock) void route_kernel(const RouteArgs a) {
  extern __shared__ double vec[];            // [tok_tile][H]
  __shared__ double red[kRouteBlock / kWave];
  __shared__ int last_flag;

  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int row = blockIdx.x * kRouteRowsPerBlock + wave;
  const WT *w = static_cast<const WT *>(a.w);
  const WT *dv = static_cast<const WT *>(a.dvec);
  const int H = a.H;
  constexpr int VN = Chunk<WT>::N;

  for (int b0 = 0; b0 < a.B; b0 += a.tok_tile) {
    const int nb = min(a.tok_tile, a.B - b0);
    for (int t = 0; t < nb; ++t) {
      const int b = b0 + t;
      double *v = vec + size_t(t) * H;
      double ss = 0.0;
      for (int i = tid; i < H; i += kRouteBlock) {
        double u;
        if (a.spec) {
          u = a.from_normalized ? double(a.s_in[size_t(b) * H + i]) : double(a.r[size_t(b) * H + i]);
          double d = 0.0;
          for (int j = 0; j < a.k; ++j) {
            const int e = a.d_ids[b * a.k + j];
            d += a.d_gates[b * a.k + j] * double(Chunk<WT>::one(dv + size_t(e) * H + i));
          }
          u += d;
        } else {
          u = double(a.r[size_t(b) * H + i]);
        }
        v[i] = u;
        ss += u * u;
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
        double n = v[i] * double(a.gain[i]) / root;
        if (a.bf16) n = round_to_bf16(n);
        v[i] = n;
        if (blockIdx.x == 0 && a.vec_out) a.vec_out[size_t(b) * H + i] = static_cast<float>(n);
      }
    }
    __syncthreads();

    if (row < a.E) {
      double acc[kMaxTokTile];
#pragma unroll
      for (int t = 0; t < kMaxTokTile; ++t) acc[t] = 0.0;
      const WT *wr = w + size_t(row) * H;
      for (int c = lane * VN; c < H; c += kWave * VN) {
        float wf[VN];
        Chunk<WT>::load(wr + c, wf);
#pragma unroll
        for (int t = 0; t < kMaxTokTile; ++t) {
          if (t < nb) {
            const double *v = vec + size_t(t) * H + c;
#pragma unroll
            for (int x = 0; x < VN; ++x) acc[t] += double(wf[x]) * v[x];
          }
        }
      }
#pragma unroll
      for (int t = 0; t < kMaxTokTile; ++t) {
        if (t < nb) {
          const double s = wave_sum(acc[t]);
          if (lane == 0) a.z[size_t(b0 + t) * a.E + row] = s;
        }
      }
    }
    __syncthreads();                         // vec is rewritten by the next tile
  }

  // Hand the logits to whichever workgroup arrives last.
  __threadfence();
  __syncthreads();
  if (tid == 0) {
    const unsigned int ticket = atomicAdd(a.counter, 1u);
    last_flag = (ticket == gridDim.x - 1);
  }
  __syncthreads();
  if (!last_flag) return;
  __threadfence();

  for (int b = wave; b < a.B; b += kRouteBlock / kWave) {
    if (a.E <= kWave) finish_token<1>(a, b, lane);
    else if (a.E <= 2 * kWave) finish_token<2>(a, b, lane);
    else finish_token<4>(a, b, lane);
  }
  __threadfence_system();
  __syncthreads();
  if (tid == 0) {
    *a.counter = 0u;
    if (a.mailbox)
      __hip_atomic_store(&a.mailbox->seq, a.seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
  }
}

}  // namespace

size_t route_lds_bytes(int H, int B, int *tok_tile) {
  int tt = int((size_t(48) << 10) / (size_t(H) * sizeof(double)));
  if (tt < 1) tt = 1;
  if (tt > kMaxTokTile) tt = kMaxTokTile;
  if (tt > B) tt = B;
  *tok_tile = tt;
  return size_t(tt) * H * sizeof(double);
}

hipError_t launch_route(const RouteArgs &a, int dtype, hipStream_t st) {
  RouteArgs args = a;
  const size_t lds = route_lds_bytes(a.H, a.B, &args.tok_tile);
  const dim3 grid((a.E + kRouteRowsPerBlock - 1) / kRouteRowsPerBlock), block(kRouteBlock);
  if (dtype == 1)
    hipLaunchKernelGGL(route_kernel<uint16_t>, grid, block, lds, st, args);
  else
    hipLaunchKernelGGL(route_kernel<float>, grid, block, lds, st, args);
  return hipGetLastError();
}

hipError_t init_route_kernels() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(route_kernel<uint16_t>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, 96 << 10);
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute(reinterpret_cast<const void *>(route_kernel<float>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, 96 << 10);
}

}  // namespace moe_spec
