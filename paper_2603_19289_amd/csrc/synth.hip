// Synthetic residual driver used by the benchmark and the tests: the stand-in for everything
// that happens between two MoE blocks of a real model.  Not part of the method.
//   v = r + O;  r' = a*v + b*(|v|_2/sqrt(H))*eps      per row
#include "../../include/moe_spec_synth.h"

#include <hip/hip_runtime.h>

namespace {

__global__ __launch_bounds__(256) void advance_kernel(const float *r, const float *o, const float *eps,
                                                      double a, double b, int H, float *r_next) {
  __shared__ double red[4];
  const int row = blockIdx.x, tid = threadIdx.x;
  const float *rr = r + size_t(row) * H, *oo = o + size_t(row) * H, *ee = eps + size_t(row) * H;
  double ss = 0.0;
  for (int i = tid; i < H; i += 256) { const double v = double(rr[i]) + double(oo[i]); ss += v * v; }
  for (int m = 32; m > 0; m >>= 1) ss += __shfl_xor(ss, m);
  if ((tid & 63) == 0) red[tid >> 6] = ss;
  __syncthreads();
  const double scale = sqrt(red[0] + red[1] + red[2] + red[3]) / sqrt(double(H));
  for (int i = tid; i < H; i += 256) {
    const double v = double(rr[i]) + double(oo[i]);
    r_next[size_t(row) * H + i] = float(a * v + b * scale * double(ee[i]));
  }
}

}  // namespace

extern "C" int moe_spec_synth_advance(void *stream, const float *r_dev, const float *out_dev,
                                      const float *eps_dev, double a, double b, int batch, int hidden,
                                      float *r_next_dev) {
  if (!r_dev || !out_dev || !eps_dev || !r_next_dev || batch < 1 || hidden < 1) return -1;
  hipLaunchKernelGGL(advance_kernel, dim3(batch), dim3(256), 0, static_cast<hipStream_t>(stream), r_dev,
                     out_dev, eps_dev, a, b, hidden, r_next_dev);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}
