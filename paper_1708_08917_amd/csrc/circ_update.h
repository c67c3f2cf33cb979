// Operand sections of the spectra blob, and the gradient step applied to the cached spectra.
//
// Algorithm 2 ends in dL/dw_ij = IFFT(G_ij), G_ij the spectrum summed over the batch.  The
// update w_ij <- w_ij - lr dL/dw_ij is linear and so is the FFT, hence the cached spectra
// (Sec. 3.1: FFT(w_ij) is what is stored) can take the step directly,
//   FFT(w_ij)/k <- FFT(w_ij)/k - (lr/k) G_ij,
// without the inverse transform of G and the forward transform of the new w.
#pragma once

#include <hip/hip_runtime.h>

#include "circ_conv_fused.h"
#include "circ_fused.h"
#include "circ_gemv.h"

namespace circ {

// The operand sections of the blob that are rearrangements of the two spectrum sections, all
// written by one launch: section s owns the workgroups [first[s], first[s+1]) and every thread
// writes one element of it.  kind: 0 fused FC operands, 1 batch <= 2 operands, 2 fused CONV
// operands (a = ncombo, b = flip).
struct PackPlan {
  static constexpr int MAXS = 6;
  int n;
  unsigned first[MAXS + 1];
  int kind[MAXS], p[MAXS], q[MAXS], a[MAXS], b[MAXS];
  const float2* spec[MAXS];
  void* dst[MAXS];
};

__global__ __launch_bounds__(256) void pack_sections_kernel(PackPlan pl, int n_grids, int K) {
  int s = 0;
  while (s + 1 < pl.n && blockIdx.x >= pl.first[s + 1]) ++s;
  const long long idx = (long long)(blockIdx.x - pl.first[s]) * 256 + threadIdx.x;
  if (pl.kind[s] == 0)
    pack_fused_elem(idx, pl.spec[s], static_cast<float4*>(pl.dst[s]), pl.p[s], pl.q[s], K, pl.a[s], pl.b[s]);
  else if (pl.kind[s] == 1)
    pack_gemv_elem(idx, pl.spec[s], static_cast<float2*>(pl.dst[s]), pl.p[s], pl.q[s], K);
  else
    pack_conv_elem(idx, pl.spec[s], static_cast<float2*>(pl.dst[s]), n_grids, pl.p[s], pl.q[s], K, pl.a[s], pl.b[s]);
}

// G[g][f][i][j] = sum over the nparts partial spectra (in index order) of
//   src[s*part_stride + f*src_fstride + g*src_gstride + i*q + j].
// Block (x = 32x32 tile of (i, j), y = f, z = g) updates both spectrum sections of grid g:
//   bwd[(g*NF + f)*p*q + i*q + j] -= a * conj(G)      (read and written along j)
//   fwd[(g*NF + f)*p*q + j*p + i] -= a * G            (transposed through LDS, written along i)
// The DC bin and, for even K, the Nyquist bin of a real vector are real: the imaginary part of G
// is dropped there.
__global__ __launch_bounds__(256) void spectra_step_kernel(const float2* __restrict__ src, int nparts,
                                                           long long part_stride, long long src_fstride,
                                                           long long src_gstride, float2* __restrict__ fwd,
                                                           float2* __restrict__ bwd, int p, int q, int NF, int K, float a) {
  __shared__ float2 tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int tiles_j = (q + 31) / 32;
  const int i0 = (blockIdx.x / tiles_j) * 32, j0 = (blockIdx.x % tiles_j) * 32;
  const int f = blockIdx.y, g = blockIdx.z;
  const bool real_bin = f == 0 || 2 * f == K;
  const long long sec = ((long long)g * NF + f) * p * q;
  const float2* sp = src + (long long)f * src_fstride + (long long)g * src_gstride;
  // the four elements of a thread: their loads of one partial spectrum are issued together (one
  // wait per part, not per load); elements outside the grid reload element 0 and are dropped
  long long e[4];
  bool ok[4];
  float2 G[4];
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    const int i = i0 + ty + 8 * m, j = j0 + tx;
    ok[m] = i < p && j < q;
    e[m] = ok[m] ? (long long)i * q + j : 0;
  }
#pragma unroll
  for (int m = 0; m < 4; ++m) G[m] = sp[e[m]];
#pragma unroll 2
  for (int s = 1; s < nparts; ++s) {
    float2 v[4];
#pragma unroll
    for (int m = 0; m < 4; ++m) v[m] = sp[s * part_stride + e[m]];
#pragma unroll
    for (int m = 0; m < 4; ++m) { G[m].x += v[m].x; G[m].y += v[m].y; }
  }
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    if (ok[m]) {
      if (real_bin) G[m].y = 0.f;
      float2 b = bwd[sec + e[m]];
      b.x -= a * G[m].x;
      b.y += a * G[m].y;
      bwd[sec + e[m]] = b;
      tile[ty + 8 * m][tx] = G[m];
    }
  }
  __syncthreads();
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    const int j = j0 + ty + 8 * m, i = i0 + tx;
    if (i < p && j < q) {
      const float2 G = tile[tx][ty + 8 * m];
      const long long e = sec + (long long)j * p + i;
      float2 w = fwd[e];
      w.x -= a * G.x;
      w.y -= a * G.y;
      fwd[e] = w;
    }
  }
}

}  // namespace circ
