// Max-pooling, the subsampling layer between CONV / FC layers (Sec. 2.1), which the paper's
// hardware runs in its peripheral block on comparators (Sec. 4.2): O(n), no arithmetic.
//   y[n][c][ho][wo] = max_{a, b < window} x[n][c][ho*stride + a][wo*stride + b]
// NCHW, windows that lie entirely inside the image (no padding).
#pragma once

#include <hip/hip_runtime.h>

namespace circ {

// One thread per output value of one image plane (n, c) = blockIdx.y + 65535 * blockIdx.z;
// consecutive threads take consecutive wo, so the reads of a wave walk along image rows.
// mul_wo = ceil(2^32 / Wo) turns the division of the in-plane index into a multiply-high
// (exact while Ho*Wo*Wo < 2^32, checked on the host; 0 = Wo is 1).
__global__ __launch_bounds__(256) void maxpool_kernel(const float* __restrict__ x, float* __restrict__ y, unsigned planes,
                                                      int H, int W, int Ho, int Wo, int window, int stride, unsigned mul_wo) {
  const unsigned plane = blockIdx.y + 65535u * blockIdx.z;
  const unsigned idx = blockIdx.x * 256u + threadIdx.x;
  if (plane >= planes || idx >= unsigned(Ho) * unsigned(Wo)) return;
  const unsigned ho = mul_wo ? __umulhi(idx, mul_wo) : idx;   // idx / Wo
  const unsigned wo = idx - ho * unsigned(Wo);
  const float* src = x + (size_t(plane) * H + size_t(ho) * stride) * W + size_t(wo) * stride;
  float m = src[0];
  for (int a = 0; a < window; ++a)
    for (int b = 0; b < window; ++b) m = fmaxf(m, src[a * W + b]);
  y[size_t(plane) * Ho * Wo + idx] = m;
}

}  // namespace circ
