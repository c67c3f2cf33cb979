// Length-K complex FFT of a tile of column pairs held in LDS.
//
// The paper's FFT kernel is recursive radix-2: a size-n transform is two size-n/2
// transforms plus one butterfly level (Sec. 4.1).  On a wave64 machine the recursion
// is cut in two at K = R1 * R2: each lane runs whole radix-2 sub-transforms of R1 (then
// R2) points in registers with compile-time twiddles, and the two passes exchange
// data through LDS.  Real inputs are exploited (Sec. 4.1: the symmetric half of the
// spectrum is never computed or stored) by packing two real rows into one complex
// sequence z = row_a + i*row_b; the half spectra of both rows are separated from
// Z[f] and conj(Z[K-f]) when the tile is written out.
//
// LDS layout of a tile: complex (float2) values, element (n, column) at n*PP + column,
// with the column the fastest index so that lanes of a wave that work on the same n hit
// consecutive banks.
#pragma once

#include <hip/hip_runtime.h>

#include "circ_twiddle.h"
#include "circ_fftreg.h"

namespace circ {

__device__ const TwiddleTable kTw = TwiddleTable();
template <int K>
__device__ const RootsTable<K> kRoots = RootsTable<K>();

// ---- the two LDS passes ------------------------------------------------------------
// Index split: n = R2*n1 + n2 on the way in, f = f1 + R1*f2 on the way out:
//   pass 1: A[f1][n2] = sum_n1 z[R2*n1+n2] W_R1^(f1*n1), then times W_K^(f1*n2)
//   pass 2: Z[f1+R1*f2] = sum_n2 A[f1][n2] W_R2^(f2*n2)
// Both passes work in place; after pass 2 the value of index f sits at
// position fft_pos<K>(f) = R2*(f % R1) + f / R1.
template <int K>
__device__ __forceinline__ int fft_pos(int f) {
  constexpr int R2 = radix2_of(K), R1 = radix1_of(K);
  return R2 * (f % R1) + f / R1;
}

// Copy the K inter-pass twiddles (cos, sin)(2*pi*m/K), m < K, from the table in the code
// object into LDS; call at kernel start so that the global latency overlaps the data loads.
template <int K>
__device__ __forceinline__ void stage_twiddles(float2* twl, int tid, int nthreads) {
  if constexpr (kTwN % K == 0) {
    for (int m = tid; m < K; m += nthreads) twl[m] = make_float2(kTw.c[m * (kTwN / K)], kTw.s[m * (kTwN / K)]);
  } else {
    for (int m = tid; m < K; m += nthreads) twl[m] = reinterpret_cast<const float2*>(kRoots<K>.cs)[m];
  }
}

// The same in two steps, for kernels that have other loads to issue: memory returns loads in issue
// order, so the roots are requested first (into registers), the kernel's own loads go out behind
// them, and the roots are written to LDS later, when they have long arrived.  nthreads >= 64.
template <int K>
struct TwiddleStage {
  static constexpr int N = (K + 63) / 64;
  float2 v[N];
  __device__ __forceinline__ void request(int tid, int nthreads) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int m = tid + i * nthreads;
      v[i] = make_float2(0.f, 0.f);
      if (m < K) {
        if constexpr (kTwN % K == 0) v[i] = reinterpret_cast<const float2*>(kTw.cs)[m * (kTwN / K)];
        else v[i] = reinterpret_cast<const float2*>(kRoots<K>.cs)[m];
      }
    }
  }
  __device__ __forceinline__ void store(float2* twl, int tid, int nthreads) const {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int m = tid + i * nthreads;
      if (m < K) twl[m] = v[i];
    }
  }
};

// z: tile of complex values, element (n, col) at z[n*PP + col].
// col: column of this thread; t, TT: index and count of threads sharing a column.
// twl: LDS copy of the twiddles made by stage_twiddles<K>.
template <int K, bool INV>
__device__ __forceinline__ void fft_lds_pass1(float2* z, int PP, int col, int t, int TT, const float2* twl) {
  constexpr int R2 = radix2_of(K), R1 = radix1_of(K);
  for (int n2 = t; n2 < R2; n2 += TT) {
    float re[R1], im[R1];
#pragma unroll
    for (int n1 = 0; n1 < R1; ++n1) {
      float2 v = z[(R2 * n1 + n2) * PP + col];
      re[n1] = v.x;
      im[n1] = v.y;
    }
    FftReg<R1, INV>::run(re, im);
#pragma unroll
    for (int f1 = 0; f1 < R1; ++f1) {
      float vr = re[f1], vi = im[f1];
      if (f1 > 0 && R2 > 1) {
        float2 w = twl[f1 * n2];
        float c = w.x;
        float s = INV ? w.y : -w.y;
        float xr = c * vr - s * vi;
        vi = c * vi + s * vr;
        vr = xr;
      }
      z[(R2 * f1 + n2) * PP + col] = make_float2(vr, vi);
    }
  }
}

// The same with a compile-time count TT of threads per column: a thread's R2 / TT sub-transforms are
// unrolled, so that their loads, butterflies and stores interleave (a thread with two of them
// otherwise runs two dependent chains one after the other).
template <int K, bool INV, int TT>
__device__ __forceinline__ void fft_lds_pass1_unrolled(float2* z, int PP, int col, int t, const float2* twl) {
  constexpr int R2 = radix2_of(K), R1 = radix1_of(K), NI = (R2 + TT - 1) / TT;
  float re[NI][R1], im[NI][R1];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int n2 = min(t + i * TT, R2 - 1);
#pragma unroll
    for (int n1 = 0; n1 < R1; ++n1) {
      const float2 v = z[(R2 * n1 + n2) * PP + col];
      re[i][n1] = v.x;
      im[i][n1] = v.y;
    }
  }
#pragma unroll
  for (int i = 0; i < NI; ++i) FftReg<R1, INV>::run(re[i], im[i]);
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int n2 = t + i * TT;
    if (n2 < R2) {
#pragma unroll
      for (int f1 = 0; f1 < R1; ++f1) {
        float vr = re[i][f1], vi = im[i][f1];
        if (f1 > 0 && R2 > 1) {
          const float2 w = twl[f1 * n2];
          const float c = w.x, s = INV ? w.y : -w.y;
          const float xr = c * vr - s * vi;
          vi = c * vi + s * vr;
          vr = xr;
        }
        z[(R2 * f1 + n2) * PP + col] = make_float2(vr, vi);
      }
    }
  }
}

// Pass 2 hands every finished value to `sink(f, value)` with f = f1 + R1*f2 instead of
// storing it, so that callers choose where spectra (or time samples) go.
template <int K, bool INV, class Sink>
__device__ __forceinline__ void fft_lds_pass2(const float2* z, int PP, int col, int t, int TT, Sink&& sink) {
  constexpr int R2 = radix2_of(K), R1 = radix1_of(K);
  for (int f1 = t; f1 < R1; f1 += TT) {
    float re[R2], im[R2];
#pragma unroll
    for (int n2 = 0; n2 < R2; ++n2) {
      float2 v = z[(R2 * f1 + n2) * PP + col];
      re[n2] = v.x;
      im[n2] = v.y;
    }
    FftReg<R2, INV>::run(re, im);
#pragma unroll
    for (int f2 = 0; f2 < R2; ++f2) sink(f1 + R1 * f2, make_float2(re[f2], im[f2]));
  }
}

// In-place variant: the value of index f is left at position fft_pos<K>(f).
template <int K, bool INV>
__device__ __forceinline__ void fft_lds_pass2_inplace(float2* z, int PP, int col, int t, int TT) {
  fft_lds_pass2<K, INV>(z, PP, col, t, TT, [&](int f, float2 v) { z[fft_pos<K>(f) * PP + col] = v; });
}

// Whole transform of one column by one thread (small K): no exchange between passes, no
// twiddle table.  Every finished value goes to `sink(f, value)`.
template <int K, bool INV, class Sink>
__device__ __forceinline__ void fft_lds_single(const float2* z, int PP, int col, Sink&& sink) {
  float re[K], im[K];
#pragma unroll
  for (int n = 0; n < K; ++n) {
    float2 v = z[n * PP + col];
    re[n] = v.x;
    im[n] = v.y;
  }
  FftReg<K, INV>::run(re, im);
#pragma unroll
  for (int f = 0; f < K; ++f) sink(f, make_float2(re[f], im[f]));
}

// ---- an 8-point transform spread over 8 consecutive lanes ----------------------------
// For tiles with few columns (the inverse transform of the fused kernel: 8 columns) the
// lane-local sub-transforms above leave most of a workgroup idle, and the few lanes that work run
// a chain of ~100 dependent instructions per pass.  Here lane m (m = lane % 8) holds point m, the
// three radix-2 stages (decimation in frequency) exchange values with lanes m^4, m^2, m^1 through
// DPP moves, and the chain is ~30 instructions.  On return lane m holds output index bitrev3(m).
__device__ __forceinline__ int bitrev3(int m) { return ((m & 1) << 2) | (m & 2) | ((m >> 2) & 1); }

__device__ __forceinline__ float lane_xor4(float v) {
  // lanes with bit 2 clear (banks 0 and 2 of a row of 16) take lane + 4, the others lane - 4
  int t = __builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x104 /* row_shl:4 */, 0xF, 0x5, false);
  t = __builtin_amdgcn_update_dpp(t, __float_as_int(v), 0x114 /* row_shr:4 */, 0xF, 0xA, false);
  return __int_as_float(t);
}
__device__ __forceinline__ float lane_xor2(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E /* quad_perm [2,3,0,1] */, 0xF, 0xF, false));
}
__device__ __forceinline__ float lane_xor1(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1 /* quad_perm [1,0,3,2] */, 0xF, 0xF, false));
}

// Per-lane constants of the three stages: the sign that turns (mine, other) into a + b or a - b,
// and the twiddles of the upper halves, W8^(m & 3) after the first stage and W4^(m & 1) after
// the second (forward: e^{-2 pi i ./8}; INV: e^{+2 pi i ./8}).
template <bool INV>
struct Fft8Lanes {
  float s4, s2, s1;      // -1 in the upper half of the stage's pairs, +1 in the lower
  float c1, d1, c2, d2;  // twiddles (cos, signed sin) after stages 1 and 2; (1, 0) in the lower halves
  __device__ __forceinline__ explicit Fft8Lanes(int m) {
    constexpr float r = 0.70710678118654752440f;
    s4 = (m & 4) ? -1.f : 1.f;
    s2 = (m & 2) ? -1.f : 1.f;
    s1 = (m & 1) ? -1.f : 1.f;
    const int a = m & 3;
    float c = a == 0 ? 1.f : (a == 1 ? r : (a == 2 ? 0.f : -r));
    float d = a == 0 ? 0.f : (a == 2 ? 1.f : r);
    c1 = (m & 4) ? c : 1.f;
    d1 = (m & 4) ? (INV ? d : -d) : 0.f;
    c2 = ((m & 2) && (m & 1)) ? 0.f : 1.f;
    d2 = ((m & 2) && (m & 1)) ? (INV ? 1.f : -1.f) : 0.f;
  }
  __device__ __forceinline__ void run(float& re, float& im) const {
    // stage 1: pairs (m, m^4)
    float tr = fmaf(s4, re, lane_xor4(re)), ti = fmaf(s4, im, lane_xor4(im));
    re = tr * c1 - ti * d1;
    im = tr * d1 + ti * c1;
    // stage 2: pairs (m, m^2)
    tr = fmaf(s2, re, lane_xor2(re));
    ti = fmaf(s2, im, lane_xor2(im));
    re = tr * c2 - ti * d2;
    im = tr * d2 + ti * c2;
    // stage 3: pairs (m, m^1), no twiddle
    tr = fmaf(s1, re, lane_xor1(re));
    ti = fmaf(s1, im, lane_xor1(im));
    re = tr;
    im = ti;
  }
};

// The same for 16 points on 16 consecutive lanes (one DPP row): a first stage over the pairs
// (m, m^8) with twiddles W16^(m & 7), then the 8-point network on each half.  `w16` is that
// twiddle of the lane, (cos, sin)(2 pi (m & 7) / 16), e.g. from the LDS table of K roots at index
// (m & 7) * K / 16.  On return lane m holds output index bitrev4(m).
__device__ __forceinline__ int bitrev4(int m) { return ((m & 1) << 3) | ((m & 2) << 1) | ((m & 4) >> 1) | ((m >> 3) & 1); }
__device__ __forceinline__ float lane_xor8(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x128 /* row_ror:8 */, 0xF, 0xF, false));
}
template <bool INV>
struct Fft16Lanes {
  Fft8Lanes<INV> f8;
  float s8, c0, d0;
  __device__ __forceinline__ Fft16Lanes(int m, float2 w16) : f8(m & 7) {
    s8 = (m & 8) ? -1.f : 1.f;
    c0 = (m & 8) ? w16.x : 1.f;
    d0 = (m & 8) ? (INV ? w16.y : -w16.y) : 0.f;
  }
  __device__ __forceinline__ void run(float& re, float& im) const {
    const float tr = fmaf(s8, re, lane_xor8(re)), ti = fmaf(s8, im, lane_xor8(im));
    re = tr * c0 - ti * d0;
    im = tr * d0 + ti * c0;
    f8.run(re, im);
  }
};

// A transform of R points (8 or 16) on R consecutive lanes; lane m in, index lane_rev<R>(m) out.
template <int R>
__device__ __forceinline__ int lane_rev(int m) { return R == 8 ? bitrev3(m) : bitrev4(m); }
template <int R, int K, bool INV>
__device__ __forceinline__ void fft_lanes(float2& v, int m, const float2* twl) {
  static_assert(R == 8 || R == 16, "8 or 16 lanes");
  if constexpr (R == 8) {
    const Fft8Lanes<INV> F(m);
    F.run(v.x, v.y);
  } else {
    const Fft16Lanes<INV> F(m, twl[(m & 7) * (K / 16)]);
    F.run(v.x, v.y);
  }
}

// One column of K = R1*R2 points (both 8 or 16; element n at z[n*stride]) transformed by the
// first K threads of the workgroup, every sub-transform on R1 (then R2) lanes.  In place; index f
// ends at position fft_pos<K>(f), as with the lane-local passes.  Call with all threads (it
// holds the barrier between the passes); twl must be staged.
template <int K, bool INV>
__device__ __forceinline__ void fft_column_lanes(float2* z, int stride, int tid, const float2* twl) {
  constexpr int R2 = radix2_of(K), R1 = radix1_of(K);
  if (tid < K) {                                   // pass 1: lane = n1, task = n2
    const int m = tid % R1, n2 = tid / R1, fo = lane_rev<R1>(m);
    float2 v = z[(R2 * m + n2) * stride];
    const float2 w = twl[fo * n2];
    fft_lanes<R1, K, INV>(v, m, twl);
    const float s = INV ? w.y : -w.y;
    z[(R2 * fo + n2) * stride] = make_float2(w.x * v.x - s * v.y, w.x * v.y + s * v.x);
  }
  __syncthreads();
  if (tid < K) {                                   // pass 2: lane = n2, task = f1
    const int m = tid % R2, f1 = tid / R2;
    float2 v = z[(R2 * f1 + m) * stride];
    fft_lanes<R2, K, INV>(v, m, twl);
    z[(R2 * f1 + lane_rev<R2>(m)) * stride] = v;
  }
}

// ---- addressing of "rows" (the length-K vectors that are transformed) ----------------
// Row ids enumerate the rows in the order of the spectrum buffer:
// spectrum[f][rid].  A row id decomposes as rid = (a*n1 + b)*n0 + c and the first
// element of the row sits at c*s0 + b*s1 + a*s2; consecutive elements are `es` apart.
// quad: set when every aligned group of 4 consecutive row ids is 4 contiguous, 16-byte aligned
// floats at every element index (s0 == 1, n0 and the row count multiples of 4, s1, s2 and es
// multiples of 4): the kernels then move 4 rows per 16-byte access.
struct RowMap {
  int n0, n1;
  long long s0, s1, s2, es;
  int quad;
};

// Row ids fit 32 bits (checked on the host), so the decomposition uses 32-bit divisions.
__device__ __forceinline__ long long row_base(const RowMap& m, long long rid) {
  const unsigned r = (unsigned)rid, n0 = (unsigned)m.n0, n1 = (unsigned)m.n1;
  const unsigned ab = r / n0, c = r - ab * n0;
  const unsigned a = ab / n1, b = ab - a * n1;
  return (long long)c * m.s0 + (long long)b * m.s1 + (long long)a * m.s2;
}

}  // namespace circ
