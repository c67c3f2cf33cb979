// Transforms for block sizes without a fast transform.
//
// Sec. 3.1 only asks that the block size k divide the layer dimensions (the example of Fig. 1
// has k = 3); the radix-2 recursion of Sec. 4.1 covers powers of two, and its mixed-radix form
// (FftReg) the sizes 3 * 2^a, 5 * 2^a and 25 * 2^a.  Every other k takes the
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

// ---- composite block sizes: one Cooley-Tukey split K = K1 * K2 (K1 the largest divisor not above
// sqrt(K)), each factor by its definition.  With n = K2*n1 + n2 and f = f1 + K1*f2,
//   A[f1][n2] = (sum_n1 x[K2*n1 + n2] W_K1^(f1 n1)) * W_K^(f1 n2),   X[f] = sum_n2 A[f1][n2] W_K2^(f2 n2),
// K*(K1 + K2) terms per row instead of K^2 (K = 96: 20 against 96 per value, K = 384: 40 against
// 384).  All roots come from the one table of K roots: W_K1^m = W_K^(K2 m), W_K2^m = W_K^(K1 m).
// Prime K keeps the kernels above.
inline int dft_factor(int K) {
  int best = 1;
  for (int d = 2; d * d <= K; ++d)
    if (K % d == 0) best = d;
  return best;
}
// LDS of a tile of R rows: roots, two complex buffers of K + 1 values per row, row bases, bias blocks
inline size_t dft2_tile_lds_bytes(int K, int R) {
  return size_t(K) * sizeof(float2) + size_t(R) * (2 * size_t(K + 1) * sizeof(float2) + sizeof(long long) + sizeof(int));
}
inline int dft2_rows_per_block(int K, long long nrows) {
  int R = 32;
  while (R > 1 && dft2_tile_lds_bytes(K, R) > 48 * 1024) R >>= 1;
  while (R > 2 && (nrows + R - 1) / R < 1024) R >>= 1;
  return R;
}

struct Dft2Lds {
  long long* rbase;
  float2* tw;
  float2* b0;        // R rows of K + 1 complex values (forward: the real rows, as floats)
  float2* b1;
  int* rblk;
};
__device__ __forceinline__ Dft2Lds carve_dft2(float* smem, int K, int R) {
  Dft2Lds L;
  L.rbase = reinterpret_cast<long long*>(smem);
  L.tw = reinterpret_cast<float2*>(L.rbase + R);
  L.b0 = L.tw + K;
  L.b1 = L.b0 + size_t(R) * (K + 1);
  L.rblk = reinterpret_cast<int*>(L.b1 + size_t(R) * (K + 1));
  return L;
}

// Same interface as dft_rows_kernel, plus K1.
__global__ __launch_bounds__(256) void dft2_rows_kernel(const float* __restrict__ in, float2* __restrict__ out, RowMap map,
                                                        long long nrows, long long out_fstride, long long in_gstride,
                                                        long long out_gstride, int K, int K1, int R, float scale, int conj,
                                                        int rows_fast) {
  extern __shared__ float smem[];
  Dft2Lds L = carve_dft2(smem, K, R);
  const int tid = threadIdx.x, K2 = K / K1, NF = K / 2 + 1, pitch = K | 1, cp = K + 1;
  float* xs = reinterpret_cast<float*>(L.b0);
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
    xs[row * pitch + t] = b >= 0 ? in[b + (long long)t * map.es] : 0.f;
  }
  __syncthreads();
  // first factor and the twiddle between the factors; lanes run along n2
  for (int idx = tid; idx < R * K; idx += 256) {
    const int row = idx / K, rem = idx - row * K;
    const int f1 = rem / K2, n2 = rem - f1 * K2;
    const float* xr = xs + row * pitch + n2;
    float re = 0.f, im = 0.f;
    int m = 0;                                   // (f1*n1) mod K1
    for (int n1 = 0; n1 < K1; ++n1) {
      const float2 w = L.tw[m * K2];
      const float v = xr[K2 * n1];
      re += v * w.x;
      im += v * w.y;
      m += f1;
      if (m >= K1) m -= K1;
    }
    const float2 t = L.tw[f1 * n2];
    L.b1[row * cp + rem] = make_float2(re * t.x - im * t.y, re * t.y + im * t.x);
  }
  __syncthreads();
  const float si = conj ? -scale : scale;
  // second factor; lanes run over the rows of the tile (adjacent row ids are adjacent in the output)
  for (int idx = tid; idx < R * NF; idx += 256) {
    const int f = idx / R, row = idx - f * R;
    if (L.rbase[row] < 0) continue;
    const int f2 = f / K1, f1 = f - f2 * K1;
    const float2* ar = L.b1 + row * cp + f1 * K2;
    float re = 0.f, im = 0.f;
    int m = 0;                                   // (f2*n2) mod K2
    for (int n2 = 0; n2 < K2; ++n2) {
      const float2 w = L.tw[m * K1], a = ar[n2];
      re += a.x * w.x - a.y * w.y;
      im += a.x * w.y + a.y * w.x;
      m += f2;
      if (m >= K2) m -= K2;
    }
    out[(long long)f * out_fstride + t0 + row] = make_float2(scale * re, si * im);
  }
}

// Same interface as idft_rows_kernel, plus K1.  With f = K2*f1 + f2 and t = t1 + K1*t2,
//   B[t1][f2] = (sum_f1 Y[K2*f1 + f2] W_K1^(-t1 f1)) * W_K^(-t1 f2),   y[t] = Re sum_f2 B[t1][f2] W_K2^(-t2 f2)
// on the full spectrum (upper half from the Hermitian symmetry of a real signal).
__global__ __launch_bounds__(256) void idft2_rows_kernel(const float2* __restrict__ in, float* __restrict__ out, RowMap map,
                                                         long long nrows, long long in_fstride, int K, int K1, int R,
                                                         float scale, const float* __restrict__ bias, long long bias_div,
                                                         int relu, int nparts, long long part_stride, int rows_fast) {
  extern __shared__ float smem[];
  Dft2Lds L = carve_dft2(smem, K, R);
  const int tid = threadIdx.x, K2 = K / K1, NF = K / 2 + 1, cp = K + 1;
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
    L.b0[row * cp + f] = y;
    if (f > 0 && 2 * f != K) L.b0[row * cp + K - f] = make_float2(y.x, -y.y);
  }
  __syncthreads();
  for (int idx = tid; idx < R * K; idx += 256) {
    const int row = idx / K, rem = idx - row * K;
    const int t1 = rem / K2, f2 = rem - t1 * K2;
    const float2* yr = L.b0 + row * cp + f2;
    float re = 0.f, im = 0.f;
    int m = 0;                                   // (t1*f1) mod K1
    for (int f1 = 0; f1 < K1; ++f1) {
      const float2 w = L.tw[m * K2], y = yr[K2 * f1];
      re += y.x * w.x - y.y * w.y;
      im += y.x * w.y + y.y * w.x;
      m += t1;
      if (m >= K1) m -= K1;
    }
    const float2 t = L.tw[t1 * f2];
    L.b1[row * cp + rem] = make_float2(re * t.x - im * t.y, re * t.y + im * t.x);
  }
  __syncthreads();
  for (int idx = tid; idx < R * K; idx += 256) {
    int row, t;
    if (rows_fast) { t = idx / R; row = idx - t * R; }
    else { row = idx / K; t = idx - row * K; }
    const long long b = L.rbase[row];
    if (b < 0) continue;
    const int t2 = t / K1, t1 = t - t2 * K1;
    const float2* br = L.b1 + row * cp + t1 * K2;
    float acc = 0.f;
    int m = 0;                                   // (t2*f2) mod K2
    for (int f2 = 0; f2 < K2; ++f2) {
      const float2 w = L.tw[m * K1], bv = br[f2];
      acc += bv.x * w.x - bv.y * w.y;
      m += t2;
      if (m >= K2) m -= K2;
    }
    float v = scale * acc;
    if (bias) v += bias[(long long)L.rblk[row] * K + t];
    if (relu) v = fmaxf(v, 0.f);
    out[b + (long long)t * map.es] = v;
  }
}

}  // namespace circ
