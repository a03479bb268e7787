// Forward pass of the neural expert estimator (paper: Sec. 6 and Appendix A): project the
// predicting signal to a latent size, add the layer's embedding, feed forward with SiLU and a
// residual connection, LayerNorm, linear head to E logits.  The first three steps are the generic
// double-precision GEMV below, launched three times; LayerNorm, head, top-k and gates run in the
// routing kernel (its input mode 3), so the hand-over to the host is the same as for the router.
// Everything is double precision: these logits decide expert indices.
#include "device_utils.h"
#include "kernels.h"

namespace moe_spec {
namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / kWave;
constexpr int kTokTile = 4;

// y[b, row] = act( W[row,:] . x[b,:] + add_w[row] ) + add_f64[b, row]; one wavefront per row.
template <typename WT>
__global__ __launch_bounds__(kBlock) void gemv64_kernel(const GemvArgs a) {
  using P = Packed<WT>;
  constexpr int VN = P::N;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int row = blockIdx.x * kWaves + wave;
  if (row >= a.rows) return;
  const WT *w = static_cast<const WT *>(a.w) + size_t(row) * a.cols;
  double bias = 0.0;
  if (a.add_w) {
    float one[VN];
    const WT *src = static_cast<const WT *>(a.add_w) + (row / VN) * VN;
    load_chunk<WT>(src, one);
    bias = double(one[row % VN]);
  }
  for (int b0 = 0; b0 < a.B; b0 += kTokTile) {
    const int nb = min(kTokTile, a.B - b0);
    double acc[kTokTile];
#pragma unroll
    for (int t = 0; t < kTokTile; ++t) acc[t] = 0.0;
#pragma unroll 2
    for (int c = lane * VN; c < a.cols; c += kWave * VN) {
      float wf[VN];
      load_chunk<WT>(w + c, wf);
#pragma unroll
      for (int t = 0; t < kTokTile; ++t) {
        if (t < nb) {
          const size_t at = size_t(b0 + t) * a.cols + c;
#pragma unroll
          for (int x = 0; x < VN; ++x)
            acc[t] += double(wf[x]) * (a.x_f64 ? a.x_f64[at + x] : double(a.x_f32[at + x]));
        }
      }
    }
#pragma unroll
    for (int t = 0; t < kTokTile; ++t) {
      if (t < nb) {
        double v = wave_sum(acc[t]) + bias;
        if (a.silu) v = v / (1.0 + exp(-v));
        if (lane == 0) {
          const size_t o = size_t(b0 + t) * a.rows + row;
          if (a.add_f64) v += a.add_f64[o];
          a.y[o] = v;
        }
      }
    }
  }
}

}  // namespace

hipError_t launch_gemv64(const GemvArgs &a, int dtype, hipStream_t st) {
  const dim3 grid((a.rows + kWaves - 1) / kWaves), block(kBlock);
  if (dtype == 1) hipLaunchKernelGGL(gemv64_kernel<uint16_t>, grid, block, 0, st, a);
  else hipLaunchKernelGGL(gemv64_kernel<float>, grid, block, 0, st, a);
  return hipGetLastError();
}

}  // namespace moe_spec
