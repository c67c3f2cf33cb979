// Fused FC forward: FFT -> per-frequency contraction -> IFFT -> bias/ReLU in ONE kernel
// (Algorithm 1 with the sum over j taken in the frequency domain, plus Eq. 1's epilogue).
//
// A workgroup owns IT output block rows and 2*NP batch rows and streams over the q input
// blocks in chunks.  Nothing but x, the cached weight spectra, the bias and y touches HBM.
//
// Real-input trick (Sec. 4.1: the symmetric half of the spectrum is redundant): two batch
// rows are packed as z = x_b0 + i*x_b1.  Because every block acts as a real linear
// operator, no separation of the two rows is needed: for bin f the two columns
//   U = Z[f]  and  V = conj(Z[K-f])
// are both multiplied by the same half-spectrum weight W^[f], and the results are
// Zy[f] and conj(Zy[K-f]) of the packed output pair, which one complex inverse FFT turns
// into (y_b0, y_b1).  DC and Nyquist bins (both real) share slot 0, so a block needs
// exactly K/2 complex slots = K floats, the size of w_ij itself.
//
// Contraction on the matrix cores: v_mfma_f32_4x4x1_16B_f32 runs 16 independent 4x4x1
// outer products.  Block = frequency slot, rows = 4 output block rows i, columns =
// (Re U, Im U, Re V, Im V) of one packed batch pair, k = one input block j.  Two
// instructions per (j, slot group): P += Re(W^) x cols, Q += Im(W^) x cols; the complex
// product is assembled once at the end:  Zy[f] = (P0 - Q1, P1 + Q0), Zy[K-f] = (P2 + Q3, P3 - Q2)
// (column 3 holds +Im Z[K-f]).  The x FFT output is written straight into this operand
// layout, and the accumulators feed the inverse FFT through LDS.
#pragma once

#include <hip/hip_runtime.h>

#include "circ_fft.h"
#include "circ_kernels.h"

namespace circ {

template <int K, int IT, int NP>
struct FusedShape {
  static constexpr int NT = 256;
  static constexpr int PT = 2048 / K;          // packed column pairs per chunk
  static constexpr int JC = PT / NP;           // input blocks j per chunk
  static constexpr int S = K / 2;              // complex slots per block
  static constexpr int FG = S / 16;            // slot groups (16 slots = one MFMA)
  static constexpr int IG = IT / 4;            // groups of 4 output block rows
  static constexpr int NCOMBO = FG * IG;
  static constexpr int CPW = NCOMBO / 4;       // (slot group, i group) combos per wave
  static constexpr int PP = PT + 1;
  static constexpr int OPROW = 2 * K + 2;      // floats per operand row (4 per slot, +2 pad)
  static constexpr int PTI = IT * NP;          // columns of the inverse transform
  static constexpr int PPI = PTI + 1;
  static constexpr int TILE_ELEMS = K * (PP > PPI ? PP : PPI);
  static constexpr size_t LDS_BYTES = size_t(TILE_ELEMS) * sizeof(float2) + size_t(PT) * OPROW * sizeof(float);
  static_assert(K >= 32 && PT >= 1 && JC >= 1 && JC * NP == PT, "bad chunk shape");
  static_assert(IT % 4 == 0 && NCOMBO % 4 == 0 && CPW >= 1, "combos must split over 4 waves");
  static_assert((PTI & (PTI - 1)) == 0 && PTI <= NT, "inverse columns must be a power of two");
  static_assert(2 * PT * (K / 4) == 4 * NT, "x staging assumes 4 float4 per thread");
};

// Weight spectra in the operand order of the fused kernel:
//   Wf[((ig*q + j)*FG + fg)*64 + 4*blk + m] = W^[i = 4*ig + m][j][slot = 16*fg + blk]
// slot 0 = (W^[0].re, W^[K/2].re); rows i >= p are zero.  `spec` is the [f][j][i] section.
__global__ void pack_fused_kernel(const float2* __restrict__ spec, float2* __restrict__ Wf, int p, int q, int K) {
  const int FG = K / 32;
  const long long total = (long long)((p + 3) / 4) * q * FG * 64;
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int l = int(idx & 63);
  long long r = idx >> 6;
  const int fg = int(r % FG); r /= FG;
  const int j = int(r % q);
  const int ig = int(r / q);
  const int i = 4 * ig + (l & 3), slot = 16 * fg + (l >> 2);
  float2 v = make_float2(0.f, 0.f);
  if (i < p) {
    const long long fs = (long long)p * q;
    if (slot == 0) v = make_float2(spec[(long long)j * p + i].x, spec[(K / 2) * fs + (long long)j * p + i].x);
    else v = spec[slot * fs + (long long)j * p + i];
  }
  Wf[idx] = v;
}

template <int K, int IT, int NP>
__global__ __launch_bounds__(256) void fc_fused_kernel(const float2* __restrict__ Wf, const float* __restrict__ x,
                                                       const float* __restrict__ bias, float* __restrict__ y,
                                                       int p, int q, int B, int n_it, int relu) {
  using Sh = FusedShape<K, IT, NP>;
  constexpr int PT = Sh::PT, JC = Sh::JC, S = Sh::S, FG = Sh::FG, IG = Sh::IG, CPW = Sh::CPW;
  constexpr int PP = Sh::PP, OPROW = Sh::OPROW, PTI = Sh::PTI, PPI = Sh::PPI;
  extern __shared__ float smem[];
  float2* z = reinterpret_cast<float2*>(smem);
  float* op = smem + 2 * Sh::TILE_ELEMS;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int it = blockIdx.x % n_it, bt = blockIdx.x / n_it;
  const int i0 = it * IT, b0 = bt * 2 * NP;
  const long long ldx = (long long)q * K, ldy = (long long)p * K;
  const int nchunks = (q + JC - 1) / JC;
  const int ig_max = (p + 3) / 4 - 1;

  floatx4 P[CPW][NP], Q[CPW][NP];
#pragma unroll
  for (int cc = 0; cc < CPW; ++cc)
#pragma unroll
    for (int u = 0; u < NP; ++u) {
      P[cc][u] = floatx4{0.f, 0.f, 0.f, 0.f};
      Q[cc][u] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

  // --- global loads: 4 float4 of x per thread and JC weight operands per combo, per chunk
  float4 xr[4];
  auto load_x = [&](int c) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int flat = e * 256 + tid;
      const int row = flat / (K / 4), n4 = flat % (K / 4);
      const int col = row >> 1, half = row & 1;
      const int j = c * JC + col / NP, b = b0 + 2 * (col % NP) + half;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (j < q && b < B) v = *reinterpret_cast<const float4*>(x + (long long)b * ldx + (long long)j * K + 4 * n4);
      xr[e] = v;
    }
  };
  auto store_x = [&]() {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int flat = e * 256 + tid;
      const int row = flat / (K / 4), n = 4 * (flat % (K / 4));
      const int col = row >> 1, half = row & 1;
      lds_put(z, (n + 0) * PP + col, half, xr[e].x);
      lds_put(z, (n + 1) * PP + col, half, xr[e].y);
      lds_put(z, (n + 2) * PP + col, half, xr[e].z);
      lds_put(z, (n + 3) * PP + col, half, xr[e].w);
    }
  };
  float2 a_cur[CPW][JC], a_nxt[CPW][JC];
  auto load_a = [&](int c, float2 (&a)[CPW][JC]) {
#pragma unroll
    for (int cc = 0; cc < CPW; ++cc) {
      const int combo = wave * CPW + cc;
      const int fg = combo / IG, ig = min(it * IG + combo % IG, ig_max);
#pragma unroll
      for (int jj = 0; jj < JC; ++jj) {
        const int j = min(c * JC + jj, q - 1);
        a[cc][jj] = Wf[(((long long)ig * q + j) * FG + fg) * 64 + lane];
      }
    }
  };

  load_x(0);
  load_a(0, a_cur);

  const int col = tid % PT, t = tid / PT;
  constexpr int TT = 256 / PT;

  for (int c = 0; c < nchunks; ++c) {
    store_x();
    __syncthreads();
    if (c + 1 < nchunks) load_x(c + 1);
    fft_lds_pass1<K, false>(z, PP, col, t, TT);
    __syncthreads();
    // pass 2 writes the spectrum of column `col` straight into MFMA operand order
    fft_lds_pass2<K, false>(z, PP, col, t, TT, [&](int f, float2 v) {
      int slot, h;
      if (f == 0) { slot = 0; h = 0; }
      else if (f == S) { slot = 0; h = 1; }
      else if (f < S) { slot = f; h = 0; }
      else { slot = K - f; h = 1; }
      *reinterpret_cast<float2*>(op + col * OPROW + 4 * slot + 2 * h) = v;
    });
    __syncthreads();
    if (c + 1 < nchunks) load_a(c + 1, a_nxt);
#pragma unroll
    for (int jj = 0; jj < JC; ++jj) {
#pragma unroll
      for (int u = 0; u < NP; ++u) {
#pragma unroll
        for (int cc = 0; cc < CPW; ++cc) {
          const int fg = (wave * CPW + cc) / IG;
          const float bv = op[(jj * NP + u) * OPROW + fg * 64 + lane];
          P[cc][u] = __builtin_amdgcn_mfma_f32_4x4x1f32(a_cur[cc][jj].x, bv, P[cc][u], 0, 0, 0);
          Q[cc][u] = __builtin_amdgcn_mfma_f32_4x4x1f32(a_cur[cc][jj].y, bv, Q[cc][u], 0, 0, 0);
        }
      }
    }
    if (c + 1 < nchunks) {
#pragma unroll
      for (int cc = 0; cc < CPW; ++cc)
#pragma unroll
        for (int jj = 0; jj < JC; ++jj) a_cur[cc][jj] = a_nxt[cc][jj];
    }
  }

  // --- assemble Zy of every (output block row, batch pair) into the inverse tile
  {
    const int n = lane & 3, blk = lane >> 2;
#pragma unroll
    for (int cc = 0; cc < CPW; ++cc) {
      const int combo = wave * CPW + cc;
      const int fg = combo / IG, ig = combo % IG;
      const int slot = 16 * fg + blk;
      const int fidx = (n < 2) ? slot : (slot == 0 ? S : K - slot);
#pragma unroll
      for (int u = 0; u < NP; ++u) {
#pragma unroll
        for (int m = 0; m < 4; ++m) {
          const float pv = P[cc][u][m], qv = Q[cc][u][m];
          const float qs = __shfl_xor(qv, 1, 64);
          float val;
          if (slot == 0) val = (n < 2) ? pv : qv;
          else val = (n == 0 || n == 3) ? pv - qs : pv + qs;
          lds_put(z, fidx * PPI + (4 * ig + m) * NP + u, n & 1, val);
        }
      }
    }
  }
  __syncthreads();
  {
    const int coli = tid % PTI, ti = tid / PTI;
    constexpr int TTI = 256 / PTI;
    fft_lds_pass1<K, true>(z, PPI, coli, ti, TTI);
    __syncthreads();
    fft_lds_pass2_inplace<K, true>(z, PPI, coli, ti, TTI);
    __syncthreads();
  }
#pragma unroll 4
  for (int idx = tid; idx < 2 * PTI * K; idx += 256) {
    const int row = idx / K, n = idx % K;
    const int coli = row >> 1, half = row & 1;
    const int i = i0 + coli / NP, b = b0 + 2 * (coli % NP) + half;
    if (i < p && b < B) {
      float v = lds_get(z, fft_pos<K>(n) * PPI + coli, half);
      if (bias) v += bias[(long long)i * K + n];
      if (relu) v = fmaxf(v, 0.f);
      y[(long long)b * ldy + (long long)i * K + n] = v;
    }
  }
}

}  // namespace circ
