// Gradients of the block-circulant CONV layer and of the bias.
//
// Sec. 3.2 derives only the forward pass of CONV layers and notes that training follows the FC
// derivation (Algorithm 2).  With the channel FFT taken per pixel, the chain rule through Eq. 6
// gives, per frequency f,
//   dX^[f][j][n][hi][wi] = sum_{dh,dw,i} conj(W^[dh][dw][f][i][j]) dY^[f][i][n][hi-dh+pad][wi-dw+pad]
//   dW^[dh][dw][f][i][j] = sum_{n,ho,wo} dY^[f][i][n][ho][wo] conj(X^[f][j][n][ho+dh-pad][wo+dw-pad])
// (zero outside the image).  The first is the forward contraction with the conjugated,
// transposed operand, the offsets reflected and the padding r-1-pad, so it runs on
// conv_contract_kernel; the second is a reduction over all output pixels (kernel below).
// The bias gradient of Eq. 1 (a = Wx + theta) is dL/da summed over everything but the channel.
#pragma once

#include <hip/hip_runtime.h>

namespace circ {

// Sum `v` over the threads of a 256-thread block, in a fixed order: butterfly inside each wave,
// then the four wave sums in index order.  `red` holds 4 floats per call site in flight; the
// result is valid in thread 0.
__device__ __forceinline__ float block_sum_256(float v, float* red, int tid) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_down(v, off, 64);
  if ((tid & 63) == 0) red[tid >> 6] = v;
  __syncthreads();
  float s = 0.f;
  if (tid == 0) s = (red[0] + red[1]) + (red[2] + red[3]);
  __syncthreads();
  return s;
}

// Partial weight-gradient spectra.  Block (x = pixel chunk, y = frequency f,
// z = (offset group, tile of IT output blocks, tile of JT input blocks)) accumulates, over its
// chunk of output pixels, the IT x JT x NG products dY^ conj(X^) of NG consecutive offsets and
// writes part[chunk][f][(g*p + i)*q + j].  The chunks are added later in index order, so the
// result does not depend on scheduling.
//   dyh  [f][i][n][ho][wo]  spectrum of dy over the channel axis (NF frequencies)
//   xh   [f][j][n][h][w]    spectrum of x
template <int IT, int JT, int NG>
__global__ __launch_bounds__(256) void conv_dw_kernel(const float2* __restrict__ dyh, const float2* __restrict__ xh,
                                                      float2* __restrict__ part, int p, int q, int NF, int Nimg, int H,
                                                      int W, int Ho, int Wo, int r, int pad, long long pix_per_block,
                                                      long long part_stride) {
  const int tid = threadIdx.x, f = blockIdx.y;
  const int nit = (p + IT - 1) / IT, njt = (q + JT - 1) / JT;
  int z = blockIdx.z;
  const int jt = z % njt; z /= njt;
  const int it = z % nit;
  const int g0 = (z / nit) * NG;
  const int i0 = it * IT, j0 = jt * JT;
  const long long npix = (long long)Nimg * Ho * Wo;
  const long long pbeg = (long long)blockIdx.x * pix_per_block, pend = min(npix, pbeg + pix_per_block);
  // offsets inside one frequency of a spectrum fit 32 bits (host check)
  const unsigned HW = unsigned(H) * unsigned(W), HWo = unsigned(Ho) * unsigned(Wo);
  const float2* dyf = dyh + (long long)f * p * npix;
  const float2* xf = xh + (long long)f * q * Nimg * HW;

  float2 acc[NG][IT][JT];
#pragma unroll
  for (int g = 0; g < NG; ++g)
#pragma unroll
    for (int ii = 0; ii < IT; ++ii)
#pragma unroll
      for (int jj = 0; jj < JT; ++jj) acc[g][ii][jj] = make_float2(0.f, 0.f);

  for (long long pix64 = pbeg + tid; pix64 < pend; pix64 += 256) {
    const unsigned pix = unsigned(pix64);
    const unsigned n = pix / HWo, rem = pix - n * HWo;
    const int ho = int(rem / unsigned(Wo)), wo = int(rem - unsigned(ho) * unsigned(Wo));
    float2 dv[IT];
#pragma unroll
    for (int ii = 0; ii < IT; ++ii) {
      const unsigned i = unsigned(min(i0 + ii, p - 1));
      dv[ii] = dyf[i * unsigned(npix) + pix];
      if (i0 + ii >= p) dv[ii] = make_float2(0.f, 0.f);
    }
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const int gg = g0 + g;
      const int dh = gg / r, dw = gg % r;
      const int hi = ho + dh - pad, wi = wo + dw - pad;
      // positions outside the image (and offsets past r*r) read a clamped address and count as zero
      const bool inb = gg < r * r && hi >= 0 && hi < H && wi >= 0 && wi < W;
      const unsigned pos = n * HW + unsigned(min(max(hi, 0), H - 1)) * unsigned(W) + unsigned(min(max(wi, 0), W - 1));
#pragma unroll
      for (int jj = 0; jj < JT; ++jj) {
        const unsigned j = unsigned(min(j0 + jj, q - 1));
        float2 xv = xf[j * (unsigned(Nimg) * HW) + pos];
        if (!inb || j0 + jj >= q) xv = make_float2(0.f, 0.f);
#pragma unroll
        for (int ii = 0; ii < IT; ++ii) {
          // d * conj(x)
          acc[g][ii][jj].x += dv[ii].x * xv.x + dv[ii].y * xv.y;
          acc[g][ii][jj].y += dv[ii].y * xv.x - dv[ii].x * xv.y;
        }
      }
    }
  }

  // Block sum in a fixed order: butterfly inside each wave, the four wave sums through LDS,
  // then thread v adds the four partial sums of value v in wave order.
  constexpr int NV = NG * IT * JT * 2;
  __shared__ float wsum[4][NV];
  const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
  for (int g = 0; g < NG; ++g)
#pragma unroll
    for (int ii = 0; ii < IT; ++ii)
#pragma unroll
      for (int jj = 0; jj < JT; ++jj) {
        float vx = acc[g][ii][jj].x, vy = acc[g][ii][jj].y;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
          vx += __shfl_down(vx, off, 64);
          vy += __shfl_down(vy, off, 64);
        }
        if (lane == 0) {
          wsum[wave][((g * IT + ii) * JT + jj) * 2 + 0] = vx;
          wsum[wave][((g * IT + ii) * JT + jj) * 2 + 1] = vy;
        }
      }
  __syncthreads();
  const long long rows = (long long)r * r * p * q;
  float* out = reinterpret_cast<float*>(part + (long long)blockIdx.x * part_stride + (long long)f * rows);
  for (int v = tid; v < NV; v += 256) {
    const int c = v & 1, e = v >> 1;
    const int jj = e % JT, ii = (e / JT) % IT, g = e / (JT * IT);
    const int gg = g0 + g, i = i0 + ii, j = j0 + jj;
    if (gg < r * r && i < p && j < q)
      out[2 * (((long long)gg * p + i) * q + j) + c] = (wsum[0][v] + wsum[1][v]) + (wsum[2][v] + wsum[3][v]);
  }
}

// db[c] = sum_{o < outer, t < inner} dy[(o*channels + c)*inner + t], one block per channel
// (CONV: outer = images, inner = pixels per image).
__global__ __launch_bounds__(256) void bias_grad_channel_kernel(const float* __restrict__ dy, float* __restrict__ db,
                                                                long long outer, int channels, long long inner) {
  __shared__ float red[4];
  const int c = blockIdx.x, tid = threadIdx.x;
  float s = 0.f;
  const long long total = outer * inner;
  // flat element index e = o*inner + t of this channel; the loads of a thread are independent
#pragma unroll 8
  for (long long e = tid; e < total; e += 256) {
    const long long o = e / inner, t = e - o * inner;
    s += dy[(o * channels + c) * inner + t];
  }
  const float tot = block_sum_256(s, red, tid);
  if (tid == 0) db[c] = tot;
}

// inner == 1 (FC: dy[batch][m]): a block owns 64 consecutive columns; its four waves take the
// rows r = wave, wave + 4, ... and their sums are added in wave order.
__global__ __launch_bounds__(256) void bias_grad_column_kernel(const float* __restrict__ dy, float* __restrict__ db,
                                                               long long rows, int cols) {
  __shared__ float red[4][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + lane;
  float s = 0.f;
  if (c < cols)
    for (long long rr = wave; rr < rows; rr += 4) s += dy[rr * cols + c];
  red[wave][lane] = s;
  __syncthreads();
  if (wave == 0 && c < cols) db[c] = (red[0][lane] + red[1][lane]) + (red[2][lane] + red[3][lane]);
}

}  // namespace circ
