// Transforms for block sizes that are not powers of two.
//
// Sec. 3.1 only asks that the block size k divide the layer dimensions (the example of Fig. 1
// has k = 3); the radix-2 recursion of Sec. 4.1 covers powers of two.  Every other k takes the
// transform by its definition, X[f] = sum_t x[t] e^{-2 pi i f t / k}: O(k^2) per row instead of
// O(k log k), on the plain vector units, with the k roots of unity tabulated in LDS.  The
// contraction between the two transforms does not depend on how they are computed.
//
// Interfaces mirror rfft_kernel / irfft_kernel: rows are addressed through a RowMap, spectra are
// stored [f][row id] with f = 0..k/2 (for odd k the last bin is complex: there is no Nyquist bin).
#pragma once

#include <hip/hip_runtime.h>

#include "circ_fft.h"

namespace circ {

// LDS bytes of a tile of R rows (either direction): roots, row tile (odd pitch; K + 4 floats per
// row cover both the real rows and the half spectra), row bases, bias blocks.
inline size_t dft_tile_lds_bytes(int K, int R) {
  return size_t(K) * sizeof(float2) + size_t(R) * (K + 4) * sizeof(float) + size_t(R) * (sizeof(long long) + sizeof(int));
}

// Rows per workgroup: as many as fit 40 KB, at most 256; fewer when that leaves the launch with
// less than about four workgroups per CU (every row costs K^2/2 multiply-adds, so even a few
// rows are a workgroup's worth of work).
inline int dft_rows_per_block(int K, long long nrows) {
  int R = 256;
  while (R > 1 && dft_tile_lds_bytes(K, R) > 40 * 1024) R >>= 1;
  while (R > 4 && (nrows + R - 1) / R < 1024) R >>= 1;
  return R;
}

struct DftLds {
  float2* tw;        // K roots of unity
  long long* rbase;  // first element of each row (-1: past the end)
  int* rblk;         // bias block of each row
  float* tile;       // R rows
};

__device__ __forceinline__ DftLds carve_dft(float* smem, int K, int R) {
  DftLds L;
  L.rbase = reinterpret_cast<long long*>(smem);
  L.tw = reinterpret_cast<float2*>(L.rbase + R);
  L.tile = reinterpret_cast<float*>(L.tw + K);          // 8-byte aligned; R*(K + 4) floats
  L.rblk = reinterpret_cast<int*>(L.tile + size_t(R) * (K + 4));
  return L;
}

// tw[n] = e^{sign * 2 pi i n / K}, evaluated in double (n/K is exact enough there that the
// float results are correctly rounded to within one unit)
__device__ __forceinline__ void stage_roots(float2* tw, int K, int tid, int nt, double sign) {
  for (int n = tid; n < K; n += nt) {
    double s, c;
    sincospi(2.0 * double(n) / double(K), &s, &c);
    tw[n] = make_float2(float(c), float(sign * s));
  }
}

// Forward: real rows -> bins 0..K/2, out[g*out_gstride + f*out_fstride + rid] (scaled; imaginary
// part negated when conj).  Block (x = tile of R rows, y = grid g).  rows_fast: consecutive row
// ids are adjacent in memory and elements of a row are strided (NCHW channel axis); otherwise
// rows are contiguous.  Only the order of the staging loop depends on it.
__global__ __launch_bounds__(256) void dft_rows_kernel(const float* __restrict__ in, float2* __restrict__ out, RowMap map,
                                                       long long nrows, long long out_fstride, long long in_gstride,
                                                       long long out_gstride, int K, int R, float scale, int conj,
                                                       int rows_fast) {
  extern __shared__ float smem[];
  DftLds L = carve_dft(smem, K, R);
  const int tid = threadIdx.x, pitch = K | 1, NF = K / 2 + 1;
  const long long t0 = (long long)blockIdx.x * R;
  in += (long long)blockIdx.y * in_gstride;
  out += (long long)blockIdx.y * out_gstride;
  stage_roots(L.tw, K, tid, 256, -1.0);
  for (int r = tid; r < R; r += 256) L.rbase[r] = t0 + r < nrows ? row_base(map, t0 + r) : -1;
  __syncthreads();
  for (int idx = tid; idx < R * K; idx += 256) {
    int row, t;
    if (rows_fast) { t = idx / R; row = idx - t * R; }
    else { row = idx / K; t = idx - row * K; }
    const long long b = L.rbase[row];
    L.tile[row * pitch + t] = b >= 0 ? in[b + (long long)t * map.es] : 0.f;
  }
  __syncthreads();
  const float si = conj ? -scale : scale;
  // lanes run over the rows of the tile (adjacent row ids are adjacent in the output)
  for (int idx = tid; idx < R * NF; idx += 256) {
    const int f = idx / R, row = idx - f * R;
    if (L.rbase[row] < 0) continue;
    const float* xr = L.tile + row * pitch;
    float re = 0.f, im = 0.f;
    int m = 0;                                   // (f*t) mod K
    for (int t = 0; t < K; ++t) {
      const float2 w = L.tw[m];
      const float v = xr[t];
      re += v * w.x;
      im += v * w.y;
      m += f;
      if (m >= K) m -= K;
    }
    out[(long long)f * out_fstride + t0 + row] = make_float2(scale * re, si * im);
  }
}

// Inverse with epilogue: out_row[t] = psi(scale * sum_f Y[f] e^{+2 pi i f t / K} + bias[blk*K + t])
// over all K bins, the upper half taken from the Hermitian symmetry of a real signal.  The
// spectrum may come as nparts partial sums, part_stride elements apart, added in index order.
__global__ __launch_bounds__(256) void idft_rows_kernel(const float2* __restrict__ in, float* __restrict__ out, RowMap map,
                                                        long long nrows, long long in_fstride, int K, int R, float scale,
                                                        const float* __restrict__ bias, long long bias_div, int relu,
                                                        int nparts, long long part_stride, int rows_fast) {
  extern __shared__ float smem[];
  DftLds L = carve_dft(smem, K, R);
  const int tid = threadIdx.x, NF = K / 2 + 1, pitch = NF | 1;   // in float2 units
  float2* ys = reinterpret_cast<float2*>(L.tile);
  const long long t0 = (long long)blockIdx.x * R;
  stage_roots(L.tw, K, tid, 256, 1.0);
  for (int r = tid; r < R; r += 256) {
    const bool ok = t0 + r < nrows;
    L.rbase[r] = ok ? row_base(map, t0 + r) : -1;
    L.rblk[r] = ok ? int((unsigned)(t0 + r) / (unsigned)bias_div) : 0;
  }
  for (int idx = tid; idx < R * NF; idx += 256) {
    const int f = idx / R, row = idx - f * R;
    float2 y = make_float2(0.f, 0.f);
    if (t0 + row < nrows) {
      const float2* s = in + (long long)f * in_fstride + t0 + row;
      y = s[0];
      for (int part = 1; part < nparts; ++part) {
        const float2 v = s[part * part_stride];
        y.x += v.x;
        y.y += v.y;
      }
    }
    if (f == 0 || 2 * f == K) y.y = 0.f;         // DC and Nyquist bins of a real signal are real
    ys[row * pitch + f] = y;
  }
  __syncthreads();
  const int nmid = (K - 1) / 2;                  // bins with a mirror image in the upper half
  for (int idx = tid; idx < R * K; idx += 256) {
    int row, t;
    if (rows_fast) { t = idx / R; row = idx - t * R; }
    else { row = idx / K; t = idx - row * K; }
    const long long b = L.rbase[row];
    if (b < 0) continue;
    const float2* yr = ys + row * pitch;
    float acc = yr[0].x, mid = 0.f;
    int m = t;                                   // (f*t) mod K for f = 1
    for (int f = 1; f <= nmid; ++f) {
      const float2 w = L.tw[m], y = yr[f];
      mid += y.x * w.x - y.y * w.y;
      m += t;
      if (m >= K) m -= K;
    }
    acc += 2.f * mid;
    if ((K & 1) == 0) acc += (t & 1) ? -yr[K / 2].x : yr[K / 2].x;
    float v = scale * acc;
    if (bias) v += bias[(long long)L.rblk[row] * K + t];
    if (relu) v = fmaxf(v, 0.f);
    out[b + (long long)t * map.es] = v;
  }
}

}  // namespace circ
