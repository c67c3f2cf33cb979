// Half-width storage: fp16 spectra and activations, fp32 accumulation.
//
// The hardware of Sec. 4.2 keeps inputs and weights in a 16-bit representation.  Its counterpart
// here is IEEE fp16 in memory (activations, FFT(w_ij), and the spectra that travel between the
// three kernels of the unfused route), with every FFT butterfly and every accumulation in fp32.
// The per-frequency contraction then runs on the fp16 matrix instructions:
//   Y^[f][i][b] = (1/k) * sum_j W^[f][i][j] X^[f][b][j]
// with both operands stored j-fastest as (re, im) pairs.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

namespace circ {

typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef float hfloatx16 __attribute__((ext_vector_type(16)));

// Eight consecutive fp16 values (four complex numbers) of a row starting at complex index j.
// VEC: rows are 16-byte aligned and Kd is a multiple of 4, so the group is inside the row or
// entirely past its end; otherwise element by element with a bounds test each.
template <bool VEC>
__device__ __forceinline__ uint4 load_complex4(const __half2* row, int j, int Kd) {
  uint4 v = make_uint4(0u, 0u, 0u, 0u);
  if constexpr (VEC) {
    if (j < Kd) v = *reinterpret_cast<const uint4*>(row + j);
  } else {
    const unsigned* r32 = reinterpret_cast<const unsigned*>(row);
    if (j + 0 < Kd) v.x = r32[j + 0];
    if (j + 1 < Kd) v.y = r32[j + 1];
    if (j + 2 < Kd) v.z = r32[j + 2];
    if (j + 3 < Kd) v.w = r32[j + 3];
  }
  return v;
}

__device__ __forceinline__ halfx8 as_halfx8(uint4 v) {
  union { uint4 u; halfx8 h; } c;
  c.u = v;
  return c.h;
}

// One workgroup = 64 rows (m) x 128 columns (n) of one frequency; wave w owns columns
// [32w, 32w + 32) as two 32 x 32 tiles.  v_mfma_f32_32x32x16_f16 multiplies 16 real values per
// row and column and step; with the (re, im) pairs interleaved along the reduction index,
//   Re C = A . (br, -bi, ...)      Im C = A . (bi, br, ...)
// so the two real products per tile need only the B operand rewritten, lane-locally: a sign
// flip of the odd halves and a swap inside every 32-bit word.  Lane (h, r) = (lane / 32,
// lane % 32) loads complex elements [k0 + 4h, k0 + 4h + 4) of its row for both operands, so the
// two operands pair up element by element whatever order the instruction sums them in.
// Accumulators: column = lane % 32, register t holds row 8*(t/4) + 4*(lane/32) + t%4.
// No LDS and no barriers: a wave whose columns lie past N leaves at once.
template <bool VEC>
__global__ __launch_bounds__(256) void cgemm_h_kernel(const __half2* __restrict__ A, const __half2* __restrict__ B,
                                                      __half2* __restrict__ C, int M, int N, int Kd, long long sA,
                                                      long long sB, long long sC, float scale) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int f = blockIdx.z, m0 = blockIdx.y * 64, n0 = blockIdx.x * 128 + 32 * wave;
  if (n0 >= N) return;
  const int r = lane & 31, h = lane >> 5;
  const __half2* a0 = A + f * sA + (long long)min(m0 + r, M - 1) * Kd;
  const __half2* a1 = A + f * sA + (long long)min(m0 + 32 + r, M - 1) * Kd;
  const __half2* b = B + f * sB + (long long)min(n0 + r, N - 1) * Kd;
  hfloatx16 cr0, ci0, cr1, ci1;
#pragma unroll
  for (int t = 0; t < 16; ++t) { cr0[t] = 0.f; ci0[t] = 0.f; cr1[t] = 0.f; ci1[t] = 0.f; }
#pragma unroll 2
  for (int k0 = 0; k0 < Kd; k0 += 8) {
    const int j = k0 + 4 * h;
    const uint4 va0 = load_complex4<VEC>(a0, j, Kd), va1 = load_complex4<VEC>(a1, j, Kd);
    const uint4 vb = load_complex4<VEC>(b, j, Kd);
    const uint4 vre = make_uint4(vb.x ^ 0x80000000u, vb.y ^ 0x80000000u, vb.z ^ 0x80000000u, vb.w ^ 0x80000000u);
    const uint4 vim = make_uint4(__builtin_amdgcn_alignbit(vb.x, vb.x, 16), __builtin_amdgcn_alignbit(vb.y, vb.y, 16),
                                 __builtin_amdgcn_alignbit(vb.z, vb.z, 16), __builtin_amdgcn_alignbit(vb.w, vb.w, 16));
    const halfx8 ha0 = as_halfx8(va0), ha1 = as_halfx8(va1), hre = as_halfx8(vre), him = as_halfx8(vim);
    cr0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(ha0, hre, cr0, 0, 0, 0);
    ci0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(ha0, him, ci0, 0, 0, 0);
    cr1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(ha1, hre, cr1, 0, 0, 0);
    ci1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(ha1, him, ci1, 0, 0, 0);
  }
  const int col = n0 + r;
  if (col >= N) return;
  __half2* c = C + f * sC + col;
#pragma unroll
  for (int t = 0; t < 16; ++t) {
    const int row = m0 + 8 * (t / 4) + 4 * h + (t % 4);
    if (row < M) c[(long long)row * N] = __floats2half2_rn(scale * cr0[t], scale * ci0[t]);
    if (row + 32 < M) c[(long long)(row + 32) * N] = __floats2half2_rn(scale * cr1[t], scale * ci1[t]);
  }
}

}  // namespace circ
