// Gradients of the block-circulant CONV layer and of the bias.
//
// Sec. 3.2 derives only the forward pass of CONV layers and notes that training follows the FC
// derivation (Algorithm 2).  With the channel FFT taken per pixel, the chain rule through Eq. 6
// gives, per frequency f,
//   dX^[f][j][n][hi][wi] = sum_{dh,dw,i} conj(W^[dh][dw][f][i][j]) dY^[f][i][n][hi-dh+pad][wi-dw+pad]
//   dW^[dh][dw][f][i][j] = sum_{n,ho,wo} dY^[f][i][n][ho][wo] conj(X^[f][j][n][ho+dh-pad][wo+dw-pad])
// (zero outside the image; written for stride 1 - with stride s the output pixel (ho, wo) pairs
// with the input pixel (ho*s+dh-pad, wo*s+dw-pad)).  The first is the forward contraction with the
// conjugated, transposed operand, the offsets reflected and the padding r-1-pad (for s > 1 on the
// output gradient with s-1 zeros between its pixels), so it runs on conv_contract_kernel; the
// second is a reduction over all output pixels (kernels below).
// The bias gradient of Eq. 1 (a = Wx + theta) is dL/da summed over everything but the channel.
#pragma once

#include <hip/hip_runtime.h>

namespace circ {

// Partial weight-gradient spectra on the matrix cores.  Block (x = pixel chunk, y = frequency f,
// z = (offset group, tile of 4 output blocks, tile of 4 input blocks)) accumulates, over its
// chunk of output pixels, the 4 x 4 x NG products dY^ conj(X^) of NG consecutive offsets and
// writes part[chunk][f][(g*p + i)*q + j].  The chunks are added later in index order, so the
// result does not depend on scheduling.
//   dyh  [f][i][n][ho][wo]  spectrum of dy over the channel axis (NF frequencies)
//   xh   [f][j][n][h][w]    spectrum of x
// v_mfma_f32_4x4x1_16B_f32 runs 16 independent 4x4 outer products: block b of a wave takes output pixel pix0 + b, rows are
// the 4 output blocks i (operand A: dY^[f][i][pixel]), columns the 4 input blocks j (operand B:
// X^[f][j][shifted pixel]); a complex product d * conj(x) is four instructions on two
// accumulators.  Every block thus sums its own subset of the pixels; at the end the 16 blocks of
// a wave are added by a butterfly over the lanes (fixed order), then the four waves through LDS.
// mul_hwo, mul_wo: ceil(2^32 / (Ho*Wo)) and ceil(2^32 / Wo) when the pixel index can be divided
// exactly by a multiply-high with them (host check: pixels * divisor < 2^32), else 0 (plain
// division): one pixel per lane and step leaves little else to amortise the division over.
typedef float dw_floatx4 __attribute__((ext_vector_type(4)));

template <int NG>
__global__ __launch_bounds__(256) void conv_dw_mfma_kernel(const float2* __restrict__ dyh, const float2* __restrict__ xh,
                                                           float2* __restrict__ part, int p, int q, int NF, int Nimg,
                                                           int H, int W, int Ho, int Wo, int r, int pad,
                                                           long long pix_per_block, long long part_stride,
                                                           unsigned mul_hwo, unsigned mul_wo, int stride) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, f = blockIdx.y;
  const int blk = lane >> 2, sub = lane & 3;
  const int nit = (p + 3) / 4, njt = (q + 3) / 4;
  int z = blockIdx.z;
  const int jt = z % njt; z /= njt;
  const int it = z % nit;
  const int g0 = (z / nit) * NG;
  const int i0 = it * 4, j0 = jt * 4;
  const long long npix = (long long)Nimg * Ho * Wo;
  const long long pbeg = (long long)blockIdx.x * pix_per_block, pend = min(npix, pbeg + pix_per_block);
  // offsets inside one frequency of a spectrum fit 32 bits (host check)
  const unsigned HW = unsigned(H) * unsigned(W), HWo = unsigned(Ho) * unsigned(Wo);
  const float2* dyf = dyh + (long long)f * p * npix;
  const float2* xf = xh + (long long)f * q * Nimg * HW;
  const bool iok = i0 + sub < p, jok = j0 + sub < q;
  const unsigned irow = unsigned(min(i0 + sub, p - 1)) * unsigned(npix);
  const unsigned jrow = unsigned(min(j0 + sub, q - 1)) * (unsigned(Nimg) * HW);

  dw_floatx4 accR[NG], accI[NG];
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    accR[g] = dw_floatx4{0.f, 0.f, 0.f, 0.f};
    accI[g] = dw_floatx4{0.f, 0.f, 0.f, 0.f};
  }

  // A wave takes 16 consecutive pixels per step and UNR steps per iteration: all loads of an
  // iteration are issued before its first matrix instruction, so that several steps' worth of
  // memory latency overlap.  The trip count is the same for every lane of a wave.
  constexpr int UNR = NG >= 9 ? 2 : 4;
  int goff_h[NG], goff_w[NG];                     // wave-uniform: offset (dh, dw) minus the padding
  bool gok[NG];
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    const int gg = g0 + g;
    goff_h[g] = gg / r - pad;
    goff_w[g] = gg % r - pad;
    gok[g] = gg < r * r;
  }
  for (long long base = pbeg + wave * 16; base < pend; base += 64 * UNR) {
    float2 d[UNR], xv[UNR][NG];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const long long pix64 = base + 64 * u + blk;
      const bool valid = pix64 < pend;
      const unsigned pix = unsigned(min(pix64, pend - 1));
      const unsigned n = mul_hwo ? __umulhi(pix, mul_hwo) : pix / HWo;
      const unsigned rem = pix - n * HWo;
      const int ho = int(mul_wo ? __umulhi(rem, mul_wo) : rem / unsigned(Wo));
      const int wo = int(rem) - ho * Wo;
      d[u] = dyf[irow + pix];
      if (!valid || !iok) d[u] = make_float2(0.f, 0.f);
      const unsigned xbase = jrow + n * HW;
#pragma unroll
      for (int g = 0; g < NG; ++g) {
        const int hi = ho * stride + goff_h[g], wi = wo * stride + goff_w[g];
        // positions outside the image (and offsets past r*r) read a clamped address and count as zero
        const bool inb = gok[g] && unsigned(hi) < unsigned(H) && unsigned(wi) < unsigned(W);
        xv[u][g] = xf[xbase + unsigned(min(max(hi, 0), H - 1)) * unsigned(W) + unsigned(min(max(wi, 0), W - 1))];
        if (!inb || !jok) xv[u][g] = make_float2(0.f, 0.f);
      }
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u)
#pragma unroll
      for (int g = 0; g < NG; ++g) {
        // d * conj(x) = (dr xr + di xi) + i (di xr - dr xi)
        accR[g] = __builtin_amdgcn_mfma_f32_4x4x1f32(d[u].x, xv[u][g].x, accR[g], 0, 0, 0);
        accI[g] = __builtin_amdgcn_mfma_f32_4x4x1f32(d[u].y, xv[u][g].x, accI[g], 0, 0, 0);
        accR[g] = __builtin_amdgcn_mfma_f32_4x4x1f32(d[u].y, xv[u][g].y, accR[g], 0, 0, 0);
        accI[g] = __builtin_amdgcn_mfma_f32_4x4x1f32(-d[u].x, xv[u][g].y, accI[g], 0, 0, 0);
      }
  }

  // lane (blk, sub) holds, in register m, the sum over its block's pixels for (i = i0 + m, j = j0 + sub)
  constexpr int NV = NG * 4 * 2;                  // values per column j
  __shared__ float wsum[4][4][NV];                // [wave][j][value]
#pragma unroll
  for (int g = 0; g < NG; ++g)
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      float vx = accR[g][m], vy = accI[g][m];
#pragma unroll
      for (int off = 4; off <= 32; off <<= 1) {
        vx += __shfl_xor(vx, off, 64);
        vy += __shfl_xor(vy, off, 64);
      }
      if (blk == 0) {
        wsum[wave][sub][(g * 4 + m) * 2 + 0] = vx;
        wsum[wave][sub][(g * 4 + m) * 2 + 1] = vy;
      }
    }
  __syncthreads();
  const long long rows = (long long)r * r * p * q;
  float* out = reinterpret_cast<float*>(part + (long long)blockIdx.x * part_stride + (long long)f * rows);
  for (int v = tid; v < 4 * NV; v += 256) {
    const int j4 = v / NV, e = v % NV;
    const int c = e & 1, m = (e >> 1) & 3, g = e >> 3;
    const int gg = g0 + g, i = i0 + m, j = j0 + j4;
    if (gg < r * r && i < p && j < q)
      out[2 * (((long long)gg * p + i) * q + j) + c] =
          (wsum[0][j4][e] + wsum[1][j4][e]) + (wsum[2][j4][e] + wsum[3][j4][e]);
  }
}

// The same partial sums with both spectra staged in LDS and the 16 blocks of the matrix
// instruction spread over the filter offsets instead of over pixels.  For one output pixel,
// block b multiplies the 4 values dY^[i][pixel] (the same in every block) with the 4 values
// X^[j][pixel shifted by offset g0 + b]: lane (b, sub) accumulates, in its own registers, the
// complete sums for (offset g0 + b, i = i0 + 0..3, j = j0 + sub) over all pixels its wave sees,
// so nothing has to be added across lanes at the end, only across the four waves.
// A workgroup stages, for its 4 input blocks, the band of image rows that a band of BR output
// rows touches (`pad` zero columns on either side, rows outside the image as zeros: a tap is
// one LDS read at the pixel's address plus a per-lane constant) and the 4 x (BR*Wo) values of
// dY^, and walks over cpb consecutive (image, band) chunks with the same accumulators.
// Block (x = group of cpb chunks, y = frequency, z = (group of 16 offsets, tile of 4 i, tile of
// 4 j)); output part[x][f][(g*p + i)*q + j] as above.
// Dynamic LDS: 4 * (S(((BR - 1)*stride + r) * (W + 2*pad)) + S(BR*Wo)) float2, S() = dw_plane_stride
// (at least 2048 floats).
// mul_wo, mul_w: ceil(2^32 / Wo), ceil(2^32 / W): exact division of indices inside a band.
// Plane stride (in float2) for n elements per plane: the next value that is 4 modulo 16, so that the
// four planes a wave reads at once start 8 banks apart.
__host__ __device__ inline int dw_plane_stride(int n) { return n + (20 - n % 16) % 16; }

// PAIR: tiles of 2 x 2 channel blocks for layers with few of them.  The rows of the matrix
// instruction then are (output block, re / im of dY^) and its columns (input block, re / im of X^):
// one instruction per pixel yields all four real products of every one of the 4 block pairs (the
// 4 x 4 form spends four instructions per pixel on 16 pairs, most of them absent when p, q <= 2),
// and a lane reads 4 bytes per operand instead of 8.  Re = rr + ii and Im = ir - ri are put
// together from a lane and its neighbour (same input block, other component) at the end.
template <bool PAIR>
__global__ __launch_bounds__(256) void conv_dw_lds_kernel(const float2* __restrict__ dyh, const float2* __restrict__ xh,
                                                          float2* __restrict__ part, int p, int q, int NF, int Nimg,
                                                          int H, int W, int Ho, int Wo, int r, int pad, int BR,
                                                          int nbands, int cpb, long long part_stride, unsigned mul_wo,
                                                          unsigned mul_w, int stride) {
  extern __shared__ float2 xs[];                  // [4 input blocks][rows_in][Wp], then [4 output blocks][BR*Wo]
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), f = blockIdx.y;
  const int blk = lane >> 2, sub = lane & 3;
  constexpr int T = PAIR ? 2 : 4;                 // channel blocks per tile side
  const int nit = (p + T - 1) / T, njt = (q + T - 1) / T;
  int z = blockIdx.z;
  const int jt = z % njt; z /= njt;
  const int it = z % nit;
  const int g0 = (z / nit) * 16;
  const int i0 = it * T, j0 = jt * T;
  const int Wp = W + 2 * pad;
  const int rows_in = (BR - 1) * stride + r, plane = rows_in * W;   // input rows under a band of BR output rows
  const int planep = dw_plane_stride(rows_in * Wp), dplane = dw_plane_stride(BR * Wo);
  float2* dys = xs + 4 * planep;
  const unsigned HW = unsigned(H) * unsigned(W), HWo = unsigned(Ho) * unsigned(Wo);
  const long long npix = (long long)Nimg * HWo;
  const float2* dyf = dyh + (long long)f * p * npix;
  const float2* xf = xh + (long long)f * q * Nimg * HW;

  // this lane's offset (lanes past r*r repeat the last offset; their sums are never stored)
  const int gl = min(g0 + blk, r * r - 1);
  const float2* xsl = xs + (PAIR ? sub >> 1 : sub) * planep + (gl / r) * Wp + gl % r;   // staged column = wo + (gl % r - pad) + pad
  const float2* dsl = dys + (PAIR ? sub >> 1 : sub) * dplane;
  const float* xslf = reinterpret_cast<const float*>(xsl) + (sub & 1);   // PAIR: this lane's component of X^ ...
  const float* dslf = reinterpret_cast<const float*>(dsl) + (sub & 1);   // ... and of dY^
  dw_floatx4 accR[2], accI[2];                    // two independent chains (even / odd pixels of a step); PAIR uses accR only
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    accR[e] = dw_floatx4{0.f, 0.f, 0.f, 0.f};
    accI[e] = dw_floatx4{0.f, 0.f, 0.f, 0.f};
  }
  // the zero columns are written once; staging only ever writes the W image columns of a row
  for (int e = tid; e < 4 * planep; e += 256) xs[e] = make_float2(0.f, 0.f);
  const int total = Nimg * nbands;
  const int cend = min(total, (int(blockIdx.x) + 1) * cpb);
  for (int c = blockIdx.x * cpb; c < cend; ++c) {
    const int n = c / nbands, band = c - n * nbands;
    const int ho0 = band * BR, brc = min(BR, Ho - ho0), npx = brc * Wo;
    __syncthreads();                              // the previous chunk has been read by every wave (first pass: zeros written)
    // The staged rows are whole image rows, so the band of one input block is one contiguous run
    // of the image: staged element t = (row, column) is image element (ho0*stride - pad)*W + t, or zero
    // outside the image.  The four blocks are fetched together (four independent loads per step).
    {
      const int e0 = (ho0 * stride - pad) * W;
      const float2* src[T];
#pragma unroll
      for (int jj = 0; jj < T; ++jj)
        src[jj] = xf + (unsigned(min(j0 + jj, q - 1)) * unsigned(Nimg) + unsigned(n)) * HW;
#pragma unroll 2
      for (int t = tid; t < plane; t += 256) {
        const int e = e0 + t;
        const bool in_img = e >= 0 && e < int(HW);
        const int ec = min(max(e, 0), int(HW) - 1);
        const int row = int(__umulhi(unsigned(t), mul_w));
        const int dst = t + row * (2 * pad) + pad;   // row*Wp + pad + column
        float2 v[T];
#pragma unroll
        for (int jj = 0; jj < T; ++jj) v[jj] = src[jj][ec];
#pragma unroll
        for (int jj = 0; jj < T; ++jj)
          xs[jj * planep + dst] = (in_img && j0 + jj < q) ? v[jj] : make_float2(0.f, 0.f);
      }
      const float2* dsrc[T];
#pragma unroll
      for (int ii = 0; ii < T; ++ii)
        dsrc[ii] = dyf + unsigned(min(i0 + ii, p - 1)) * unsigned(npix) + unsigned(n) * HWo + unsigned(ho0) * unsigned(Wo);
#pragma unroll 2
      for (int t = tid; t < npx; t += 256) {
        float2 v[T];
#pragma unroll
        for (int ii = 0; ii < T; ++ii) v[ii] = dsrc[ii][t];
#pragma unroll
        for (int ii = 0; ii < T; ++ii) dys[ii * dplane + t] = i0 + ii < p ? v[ii] : make_float2(0.f, 0.f);
      }
    }
    __syncthreads();
    // wave w takes pixels w, w + 4, ...: four at a time (operands first, then 16 matrix instructions)
    auto mac = [&](int e, float2 dv, float2 xv) {
      accR[e] = __builtin_amdgcn_mfma_f32_4x4x1f32(dv.x, xv.x, accR[e], 0, 0, 0);
      accI[e] = __builtin_amdgcn_mfma_f32_4x4x1f32(dv.y, xv.x, accI[e], 0, 0, 0);
      accR[e] = __builtin_amdgcn_mfma_f32_4x4x1f32(dv.y, xv.y, accR[e], 0, 0, 0);
      accI[e] = __builtin_amdgcn_mfma_f32_4x4x1f32(-dv.x, xv.y, accI[e], 0, 0, 0);
    };
    auto tap = [&](int pix) -> int {              // staged element of output pixel pix, offset (0, 0): stride*(hl*Wp + wo)
      const int hl = int(__umulhi(unsigned(pix), mul_wo));
      return stride * (pix + hl * (Wp - Wo));
    };
    int pix = wave;
    if constexpr (PAIR) {
      for (; pix + 12 < npx; pix += 16) {
        float dv[4], xv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          dv[u] = dslf[2 * (pix + 4 * u)];
          xv[u] = xslf[2 * tap(pix + 4 * u)];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) accR[u & 1] = __builtin_amdgcn_mfma_f32_4x4x1f32(dv[u], xv[u], accR[u & 1], 0, 0, 0);
      }
      for (; pix < npx; pix += 4) accR[0] = __builtin_amdgcn_mfma_f32_4x4x1f32(dslf[2 * pix], xslf[2 * tap(pix)], accR[0], 0, 0, 0);
    } else {
      for (; pix + 12 < npx; pix += 16) {
        float2 dv[4], xv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          dv[u] = dsl[pix + 4 * u];
          xv[u] = xsl[tap(pix + 4 * u)];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) mac(u & 1, dv[u], xv[u]);
      }
      for (; pix < npx; pix += 4) mac(0, dsl[pix], xsl[tap(pix)]);
    }
  }

  // sums over the four waves: accumulators -> LDS (the staging area is free after the barrier)
  __syncthreads();
  float* wsum = reinterpret_cast<float*>(xs);    // [wave][value m*2 + c][lane]
  if constexpr (PAIR) {
    // register m = row (output block m / 2, component m % 2); this lane's column = (input block
    // sub / 2, component sub % 2).  Lanes of component 0 take the neighbour's sums:
    //   Re(i, j) = rr + ii = mine[2i] + other[2i + 1],  Im(i, j) = ir - ri = mine[2i + 1] - other[2i]
    float mine[4], other[4];
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      mine[m] = accR[0][m] + accR[1][m];
      other[m] = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(mine[m]), 0xB1 /* quad_perm [1,0,3,2] */, 0xF, 0xF, false));
    }
#pragma unroll
    for (int ii = 0; ii < 2; ++ii) {
      wsum[(wave * 8 + 2 * ii + 0) * 64 + lane] = mine[2 * ii] + other[2 * ii + 1];
      wsum[(wave * 8 + 2 * ii + 1) * 64 + lane] = mine[2 * ii + 1] - other[2 * ii];
    }
  } else {
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      wsum[(wave * 8 + 2 * m + 0) * 64 + lane] = accR[0][m] + accR[1][m];
      wsum[(wave * 8 + 2 * m + 1) * 64 + lane] = accI[0][m] + accI[1][m];
    }
  }
  __syncthreads();
  const long long rows = (long long)r * r * p * q;
  float* out = reinterpret_cast<float*>(part + (long long)blockIdx.x * part_stride + (long long)f * rows);
  for (int v = tid; v < (PAIR ? 4 : 8) * 64; v += 256) {
    const int ln = v & 63, e = v >> 6;           // e = m*2 + c (PAIR: m = output block of the pair, lanes of component 0 only)
    const int c = e & 1, m = e >> 1;
    const int gg = g0 + (ln >> 2), i = i0 + m, j = j0 + (PAIR ? (ln & 3) >> 1 : ln & 3);
    if (gg < r * r && i < p && j < q && !(PAIR && (ln & 1)))
      out[2 * (((long long)gg * p + i) * q + j) + c] =
          (wsum[(0 * 8 + e) * 64 + ln] + wsum[(1 * 8 + e) * 64 + ln]) + (wsum[(2 * 8 + e) * 64 + ln] + wsum[(3 * 8 + e) * 64 + ln]);
  }
}

// part[0][e] = sum over s < nparts of part[s][e], in index order (e < n floats): the partial
// spectra of the weight gradient folded into the first one, one thread per value.
__global__ __launch_bounds__(256) void sum_parts_kernel(float* __restrict__ part, int nparts, long long part_stride, long long n) {
  const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
  if (e >= n) return;
  float v[8];
  float acc = part[e];
  int s = 1;
  for (; s + 8 <= nparts; s += 8) {
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = part[(s + u) * part_stride + e];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += v[u];
  }
  for (; s < nparts; ++s) acc += part[s * part_stride + e];
  part[e] = acc;
}

// db[c] = sum_{o < outer, t < inner} dy[(o*channels + c)*inner + t], one block of 1024 threads per
// channel (CONV: outer = images, inner = pixels per image; with as many channels as CUs, the
// threads of a block are what keeps enough loads in flight).  Fixed order: each thread adds its
// strided elements in index order, a butterfly adds the lanes of a wave, one thread the 16 waves.
__global__ __launch_bounds__(1024) void bias_grad_channel_kernel(const float* __restrict__ dy, float* __restrict__ db,
                                                                 long long outer, int channels, long long inner, int vec4) {
  __shared__ float red[16];
  const int c = blockIdx.x, tid = threadIdx.x;
  float s = 0.f;
  const long long total = outer * inner;
  // flat element index e = o*inner + t of this channel; the loads of a thread are independent
  if (vec4) {
    // inner is a multiple of 4 (a 16-byte group never straddles two images), dy is 16-byte
    // aligned and total < 2^32 (host checks): 16-byte loads, 32-bit index arithmetic
    const unsigned ngroups = unsigned(total >> 2), inner4 = unsigned(inner >> 2);
    float s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll 4
    for (unsigned g = tid; g < ngroups; g += 1024) {
      const unsigned o = g / inner4, t4 = g - o * inner4;
      const float4 v = *reinterpret_cast<const float4*>(dy + ((long long)o * channels + c) * inner + 4 * t4);
      s += v.x; s1 += v.y; s2 += v.z; s3 += v.w;
    }
    s = (s + s1) + (s2 + s3);
  } else {
#pragma unroll 8
    for (long long e = tid; e < total; e += 1024) {
      const long long o = e / inner, t = e - o * inner;
      s += dy[(o * channels + c) * inner + t];
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) s += __shfl_down(s, off, 64);
  if ((tid & 63) == 0) red[tid >> 6] = s;
  __syncthreads();
  if (tid == 0) {
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < 16; ++w) tot += red[w];
    db[c] = tot;
  }
}

// inner == 1 (FC: dy[batch][m]): a block owns 64 consecutive columns; its 16 waves take the
// rows r = wave, wave + 16, ... and their sums are added in wave order.
__global__ __launch_bounds__(1024) void bias_grad_column_kernel(const float* __restrict__ dy, float* __restrict__ db,
                                                                long long rows, int cols) {
  // 64 columns per block, 16 waves: wave w adds rows w, w + 16, ... with four independent partial
  // sums (several loads in flight per lane); fixed order throughout
  __shared__ float red[16][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + lane;
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  if (c < cols) {
    const float* col = dy + c;
    long long rr = wave;
#pragma unroll 2
    for (; rr + 48 < rows; rr += 64) {
      s0 += col[rr * cols];
      s1 += col[(rr + 16) * cols];
      s2 += col[(rr + 32) * cols];
      s3 += col[(rr + 48) * cols];
    }
    for (; rr < rows; rr += 16) s0 += col[rr * cols];
  }
  red[wave][lane] = (s0 + s1) + (s2 + s3);
  __syncthreads();
  if (wave == 0 && c < cols) {
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < 16; ++w) tot += red[w][lane];
    db[c] = tot;
  }
}

}  // namespace circ
