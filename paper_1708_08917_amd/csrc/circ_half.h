// Half-width storage: 16-bit spectra and activations, fp32 accumulation.
//
// The hardware of Sec. 4.2 keeps inputs and weights in a 16-bit representation.  Its counterpart
// here is IEEE fp16 or bfloat16 in memory (activations, FFT(w_ij), and the spectra that travel
// between the three kernels of the unfused route), with every FFT butterfly and every accumulation
// in fp32.  The per-frequency contraction then runs on the 16-bit matrix instructions:
//   Y^[f][i][b] = (1/k) * sum_j W^[f][i][j] X^[f][b][j]
// with both operands stored j-fastest as (re, im) pairs.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include "circ_kernels.h"

namespace circ {

typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef __bf16 bfloatx8 __attribute__((ext_vector_type(8)));
typedef float hfloatx16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ halfx8 as_halfx8(uint4 v) {
  union { uint4 u; halfx8 h; } c;
  c.u = v;
  return c.h;
}
__device__ __forceinline__ bfloatx8 as_bfloatx8(uint4 v) {
  union { uint4 u; bfloatx8 h; } c;
  c.u = v;
  return c.h;
}
// acc += A (32 x 16) * B (16 x 32) on 16-bit operands (fp16, or bfloat16 when BF), fp32 accumulation
template <bool BF>
__device__ __forceinline__ hfloatx16 mfma16(uint4 a, uint4 b, hfloatx16 acc) {
  if constexpr (BF) return __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bfloatx8(a), as_bfloatx8(b), acc, 0, 0, 0);
  else return __builtin_amdgcn_mfma_f32_32x32x16_f16(as_halfx8(a), as_halfx8(b), acc, 0, 0, 0);
}

// One workgroup = 64 rows (m) x 128 columns (n) of one frequency; wave w owns columns
// [32w, 32w + 32) as two 32 x 32 tiles.  v_mfma_f32_32x32x16_f16 multiplies 16 real values per
// row and column and step; with the (re, im) pairs interleaved along the reduction index,
//   Re C = A . (br, -bi, ...)      Im C = A . (bi, br, ...)
// so the two real products per tile need only the B operand rewritten, lane-locally: a sign
// flip of the odd halves and a swap inside every 32-bit word.  Lane (h, r) = (lane / 32,
// lane % 32) takes complex elements [8s + 4h, 8s + 4h + 4) of its row in step s for both
// operands, so the operands pair up element by element whatever order the instruction sums them in.
// Accumulators: column = lane % 32, register t holds row 8*(t/4) + 4*(lane/32) + t%4.
//
// The reduction runs in chunks of 64 complex values.  A chunk of both operand tiles goes through
// LDS: the workgroup loads it with lanes running along the rows (every 128-byte line of the
// operands is fetched once, by one instruction), and the waves then read their fragments, 16 bytes
// per lane, from LDS rows padded to 68 words (consecutive rows start 4 banks apart).  Fetching
// the fragments straight from global memory makes every instruction touch 32 lines for 32 bytes
// each, and the same lines come back for the next steps; that version ran at the L2 line rate.
// VEC: Kd is a multiple of 4 (16-byte pieces are whole or entirely past the end of a row);
// otherwise the chunk is staged element by element.  Values past Kd are staged as zeros.
// TB: B is stored with n fastest, B[f][k][n] (row pitch N), and is transposed on its way into
// LDS: a wave-load takes 16 values of k times four 16-byte groups along n, so that the four
// 4-byte LDS stores of a lane fall on 16 consecutive banks per group and two groups 16 banks
// apart.  VEC then also requires N to be a multiple of 4.
constexpr int kHChunk = 64;                      // complex values of the reduction per chunk
constexpr int kHPitch = kHChunk + 4;             // LDS row pitch in complex values (272 bytes)

template <bool VEC, bool BF, bool TB = false>
__global__ __launch_bounds__(256) void cgemm_h_kernel(const __half2* __restrict__ A, const __half2* __restrict__ B,
                                                      __half2* __restrict__ C, int M, int N, int Kd, long long sA,
                                                      long long sB, long long sC, float scale) {
  __shared__ __attribute__((aligned(16))) __half2 lds[(64 + 128) * kHPitch];
  __half2* la = lds;
  __half2* lb = lds + 64 * kHPitch;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int f = blockIdx.z, m0 = blockIdx.y * 64, nb0 = blockIdx.x * 128;
  const int r = lane & 31, h = lane >> 5;
  const __half2* Af = A + f * sA;
  const __half2* Bf = B + f * sB;
  hfloatx16 cr0, ci0, cr1, ci1;
#pragma unroll
  for (int t = 0; t < 16; ++t) { cr0[t] = 0.f; ci0[t] = 0.f; cr1[t] = 0.f; ci1[t] = 0.f; }
  const bool wave_active = nb0 + 32 * wave < N;  // waves past N only help with the staging
  for (int kc = 0; kc < Kd; kc += kHChunk) {
    __syncthreads();                             // the previous chunk has been read
    if constexpr (VEC) {
      // piece e of the chunk: row e / 16, 16-byte piece e % 16 of the row's 256 bytes; rows of A
      // first, then rows of B (rows past M or N repeat the last one: their results are not stored)
      constexpr int NIT = TB ? 4 : 12;             // direct rows: A only, or A and B
      uint4 v[NIT];
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int e = it * 256 + tid, row = e >> 4, j = kc + 4 * (e & 15);
        const __half2* src = row < 64 ? Af + (long long)min(m0 + row, M - 1) * Kd : Bf + (long long)min(nb0 + row - 64, N - 1) * Kd;
        v[it] = *reinterpret_cast<const uint4*>(src + min(j, Kd - 4));
      }
      uint4 vt[TB ? 8 : 1];
      if constexpr (TB) {
#pragma unroll
        for (int it = 0; it < 8; ++it) {
          const int combo = it * 4 + wave, kk = kc + 16 * (combo & 3) + (lane & 15), n = nb0 + 4 * (4 * (combo >> 2) + (lane >> 4));
          vt[it] = *reinterpret_cast<const uint4*>(Bf + (long long)min(kk, Kd - 1) * N + min(n, N - 4));
        }
      }
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int e = it * 256 + tid, row = e >> 4, j = kc + 4 * (e & 15);
        *reinterpret_cast<uint4*>(lds + row * kHPitch + 4 * (e & 15)) = j < Kd ? v[it] : make_uint4(0u, 0u, 0u, 0u);
      }
      if constexpr (TB) {
#pragma unroll
        for (int it = 0; it < 8; ++it) {
          const int combo = it * 4 + wave, kl = 16 * (combo & 3) + (lane & 15), nl = 4 * (4 * (combo >> 2) + (lane >> 4));
          const uint4 w = kc + kl < Kd ? vt[it] : make_uint4(0u, 0u, 0u, 0u);
          unsigned* d = reinterpret_cast<unsigned*>(lb) + nl * kHPitch + kl;
          d[0] = w.x;
          d[kHPitch] = w.y;
          d[2 * kHPitch] = w.z;
          d[3 * kHPitch] = w.w;
        }
      }
    } else {
      for (int e = tid; e < (TB ? 64 : 64 + 128) * kHChunk; e += 256) {
        const int row = e >> 6, j = kc + (e & 63);
        const __half2* src = row < 64 ? Af + (long long)min(m0 + row, M - 1) * Kd : Bf + (long long)min(nb0 + row - 64, N - 1) * Kd;
        const unsigned v = reinterpret_cast<const unsigned*>(src)[min(j, Kd - 1)];
        reinterpret_cast<unsigned*>(lds)[row * kHPitch + (e & 63)] = j < Kd ? v : 0u;
      }
      if constexpr (TB) {
        for (int e = tid; e < 128 * kHChunk; e += 256) {
          const int nl = e & 127, kl = e >> 7;
          const unsigned v = reinterpret_cast<const unsigned*>(Bf)[(long long)min(kc + kl, Kd - 1) * N + min(nb0 + nl, N - 1)];
          reinterpret_cast<unsigned*>(lb)[nl * kHPitch + kl] = kc + kl < Kd ? v : 0u;
        }
      }
    }
    __syncthreads();
    if (wave_active) {
      const __half2* fa0 = la + r * kHPitch + 4 * h;
      const __half2* fa1 = la + (32 + r) * kHPitch + 4 * h;
      const __half2* fb = lb + (32 * wave + r) * kHPitch + 4 * h;
      const int nsteps = min(kHChunk, Kd - kc + 7) / 8;   // whole steps of 8 that hold anything
#pragma unroll
      for (int s = 0; s < kHChunk / 8; ++s) {
        if (s < nsteps) {                        // wave-uniform
          const uint4 va0 = *reinterpret_cast<const uint4*>(fa0 + 8 * s);
          const uint4 va1 = *reinterpret_cast<const uint4*>(fa1 + 8 * s);
          const uint4 vb = *reinterpret_cast<const uint4*>(fb + 8 * s);
          const uint4 vre = make_uint4(vb.x ^ 0x80000000u, vb.y ^ 0x80000000u, vb.z ^ 0x80000000u, vb.w ^ 0x80000000u);
          const uint4 vim = make_uint4(__builtin_amdgcn_alignbit(vb.x, vb.x, 16), __builtin_amdgcn_alignbit(vb.y, vb.y, 16),
                                       __builtin_amdgcn_alignbit(vb.z, vb.z, 16), __builtin_amdgcn_alignbit(vb.w, vb.w, 16));
          cr0 = mfma16<BF>(va0, vre, cr0);
          ci0 = mfma16<BF>(va0, vim, ci0);
          cr1 = mfma16<BF>(va1, vre, cr1);
          ci1 = mfma16<BF>(va1, vim, ci1);
        }
      }
    }
  }
  const int col = nb0 + 32 * wave + r;
  if (!wave_active || col >= N) return;
  unsigned* c = reinterpret_cast<unsigned*>(C) + f * sC + col;
#pragma unroll
  for (int t = 0; t < 16; ++t) {
    const int row = m0 + 8 * (t / 4) + 4 * h + (t % 4);
    if (row < M) c[(long long)row * N] = pack_pair16<BF>(scale * cr0[t], scale * ci0[t]);
    if (row + 32 < M) c[(long long)(row + 32) * N] = pack_pair16<BF>(scale * cr1[t], scale * ci1[t]);
  }
}

// Backward-weights (Algorithm 2: the spectrum of dL/dw_ij is the sum over the batch of
// FFT(dL/da_i) o conj(FFT(x_j))):
//   C[f][m][n] = scale * sum_k A[f][m][k] conj(B[f][n][k]),   k = the batch index,
// with Re C = A . (br, bi, ...) and Im C = A . (-bi, br, ...).  The output is narrow (p x q block
// pairs) and the reduction long, so a workgroup owns a 64 x 64 tile (wave w the 32 x 32 quadrant
// (w % 2, w / 2): every staged row feeds two waves) and the reduction is cut into slices of `klen`
// values (a multiple of 64): blockIdx.x = slice * ceil(N/64) + column tile, slice ks writes its
// partial sums to C + ks*part_stride, to be added later in index order.  C is fp32: a sum over a
// long batch leaves the fp16 range, and the output is small.
template <bool VEC, bool BF>
__global__ __launch_bounds__(256) void cgemm_h_dw_kernel(const __half2* __restrict__ A, const __half2* __restrict__ B,
                                                         float2* __restrict__ C, int M, int N, int Kd, long long sA,
                                                         long long sB, long long sC, float scale, int klen,
                                                         long long part_stride) {
  __shared__ __attribute__((aligned(16))) __half2 lds[(64 + 64) * kHPitch];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int ntn = (N + 63) / 64, ks = blockIdx.x / ntn;
  const int f = blockIdx.z, m0 = blockIdx.y * 64, nb0 = (blockIdx.x - ks * ntn) * 64;
  const int kbeg = ks * klen, kend = min(Kd, kbeg + klen);
  const int r = lane & 31, h = lane >> 5, wm = wave & 1, wn = wave >> 1;
  const __half2* Af = A + f * sA;
  const __half2* Bf = B + f * sB;
  hfloatx16 cr, ci;
#pragma unroll
  for (int t = 0; t < 16; ++t) { cr[t] = 0.f; ci[t] = 0.f; }
  const bool wave_active = m0 + 32 * wm < M && nb0 + 32 * wn < N;   // the others only help with the staging
  for (int kc = kbeg; kc < kend; kc += kHChunk) {
    __syncthreads();                             // the previous chunk has been read
    if constexpr (VEC) {
      uint4 v[8];
#pragma unroll
      for (int it = 0; it < 8; ++it) {
        const int e = it * 256 + tid, row = e >> 4, j = kc + 4 * (e & 15);
        const __half2* src = row < 64 ? Af + (long long)min(m0 + row, M - 1) * Kd : Bf + (long long)min(nb0 + row - 64, N - 1) * Kd;
        v[it] = *reinterpret_cast<const uint4*>(src + min(j, Kd - 4));
      }
#pragma unroll
      for (int it = 0; it < 8; ++it) {
        const int e = it * 256 + tid, row = e >> 4, j = kc + 4 * (e & 15);
        *reinterpret_cast<uint4*>(lds + row * kHPitch + 4 * (e & 15)) = j < kend ? v[it] : make_uint4(0u, 0u, 0u, 0u);
      }
    } else {
      for (int e = tid; e < (64 + 64) * kHChunk; e += 256) {
        const int row = e >> 6, j = kc + (e & 63);
        const __half2* src = row < 64 ? Af + (long long)min(m0 + row, M - 1) * Kd : Bf + (long long)min(nb0 + row - 64, N - 1) * Kd;
        const unsigned v = reinterpret_cast<const unsigned*>(src)[min(j, Kd - 1)];
        reinterpret_cast<unsigned*>(lds)[row * kHPitch + (e & 63)] = j < kend ? v : 0u;
      }
    }
    __syncthreads();
    if (wave_active) {
      const __half2* fa = lds + (32 * wm + r) * kHPitch + 4 * h;
      const __half2* fb = lds + (64 + 32 * wn + r) * kHPitch + 4 * h;
      const int nsteps = min(kHChunk, kend - kc + 7) / 8;   // whole steps of 8 that hold anything
#pragma unroll
      for (int s = 0; s < kHChunk / 8; ++s) {
        if (s < nsteps) {                        // wave-uniform
          const uint4 va = *reinterpret_cast<const uint4*>(fa + 8 * s);
          const uint4 vb = *reinterpret_cast<const uint4*>(fb + 8 * s);
          // (bi, br) after the swap inside each word; the sign goes to the half that now holds bi
          const uint4 vim = make_uint4(__builtin_amdgcn_alignbit(vb.x, vb.x, 16) ^ 0x8000u, __builtin_amdgcn_alignbit(vb.y, vb.y, 16) ^ 0x8000u,
                                       __builtin_amdgcn_alignbit(vb.z, vb.z, 16) ^ 0x8000u, __builtin_amdgcn_alignbit(vb.w, vb.w, 16) ^ 0x8000u);
          cr = mfma16<BF>(va, vb, cr);
          ci = mfma16<BF>(va, vim, ci);
        }
      }
    }
  }
  const int col = nb0 + 32 * wn + r;
  if (!wave_active || col >= N) return;
  float2* c = C + ks * part_stride + f * sC + col;
#pragma unroll
  for (int t = 0; t < 16; ++t) {
    const int row = m0 + 32 * wm + 8 * (t / 4) + 4 * h + (t % 4);
    if (row < M) c[(long long)row * N] = make_float2(scale * cr[t], scale * ci[t]);
  }
}

}  // namespace circ
