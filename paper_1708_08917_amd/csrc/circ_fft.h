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

namespace circ {

__device__ const TwiddleTable kTw = TwiddleTable();
template <int K>
__device__ const RootsTable<K> kRoots = RootsTable<K>();

constexpr int ilog2(int v) { return v <= 1 ? 0 : 1 + ilog2(v >> 1); }
constexpr bool is_pow2_c(int v) { return v > 0 && (v & (v - 1)) == 0; }
// K = R1 * R2 with R1 <= R2.  Powers of two: R2 <= 2 * R1; for odd log2 K the longer sub-transform
// is the second one: the first pass then has R2 = 2*R1 short sub-transforms (plus the twiddles) per
// column, which keep every thread of a 16-threads-per-column kernel busy, and the second pass R1
// long ones without twiddles (fused kernel, K = 128: 1.25 + 0.47 us per chunk with the longer one
// first, about 0.4 us less this way).  Other sizes: the factor pair closest to the square root
// (96 = 8 * 12, 100 = 10 * 10, 384 = 16 * 24).
constexpr int radix1_of(int K) {
  if (is_pow2_c(K)) return K / (1 << ((ilog2(K) + 1) / 2));
  int best = 1;
  for (int d = 2; d * d <= K; ++d)
    if (K % d == 0) best = d;
  return best;
}
constexpr int radix2_of(int K) { return K / radix1_of(K); }
constexpr int smallest_odd_factor(int R) {
  for (int d = 3; d * d <= R; d += 2)
    if (R % d == 0) return d;
  return R;
}

// ---- in-register FFT of R points, natural order in and out ---------------------------
// Even R: the radix-2 recursion of Sec. 4.1 (two transforms of R/2 points and one butterfly
// level).  Odd R = p * M, p its smallest prime factor: p transforms of M points over the
// subsequences x[p*n + s], then X[f + M*m] = sum_s (E_s[f] W_R^(s f)) W_p^(s m): the same
// recursion with p-point butterflies.  The p-point butterfly pairs s with p - s:
// with a_s = T_s + T_(p-s), b_s = T_s - T_(p-s), X_m and X_(p-m) are
// (T_0 + sum_s cos(2 pi s m / p) a_s) -/+ i (sum_s sin(2 pi s m / p) b_s)  (forward; inverse: +/-).
// All twiddles are compile-time constants.
template <int R, bool INV>
struct FftReg {
  template <int M>
  static __device__ __forceinline__ void combine(float (&re)[R], float (&im)[R],
                                                 const float (&er)[R / 2], const float (&ei)[R / 2],
                                                 const float (&pr)[R / 2], const float (&pi)[R / 2]) {
    if constexpr (M < R / 2) {
      float tr, ti;
      if constexpr (M == 0) {
        tr = pr[M];
        ti = pi[M];
      } else if constexpr (4 * M == R) {           // twiddle = -i (forward) or +i (inverse)
        tr = INV ? -pi[M] : pi[M];
        ti = INV ? pr[M] : -pr[M];
      } else {
        constexpr float c = tw_cos(M, R);
        constexpr float s = INV ? tw_sin(M, R) : -tw_sin(M, R);   // twiddle = c + i*s
        tr = c * pr[M] - s * pi[M];
        ti = c * pi[M] + s * pr[M];
      }
      re[M] = er[M] + tr;
      im[M] = ei[M] + ti;
      re[M + R / 2] = er[M] - tr;
      im[M + R / 2] = ei[M] - ti;
      combine<M + 1>(re, im, er, ei, pr, pi);
    }
  }

  // odd R: outputs f, f + M, ..., f + (p-1)*M from the p sub-transforms' values at f
  template <int P, int M, int F>
  static __device__ __forceinline__ void combine_odd(float (&re)[R], float (&im)[R], const float (&sr)[P][M],
                                                     const float (&si)[P][M]) {
    if constexpr (F < M) {
      float tr[P], ti[P];
      tr[0] = sr[0][F];
      ti[0] = si[0][F];
      odd_twiddle<P, M, F, 1>(tr, ti, sr, si);
      constexpr int H = (P - 1) / 2;
      float ar[H + 1], ai[H + 1], br[H + 1], bi[H + 1];
#pragma unroll
      for (int s = 1; s <= H; ++s) {
        ar[s] = tr[s] + tr[P - s];
        ai[s] = ti[s] + ti[P - s];
        br[s] = tr[s] - tr[P - s];
        bi[s] = ti[s] - ti[P - s];
      }
      float x0r = tr[0], x0i = ti[0];
#pragma unroll
      for (int s = 1; s <= H; ++s) {
        x0r += ar[s];
        x0i += ai[s];
      }
      re[F] = x0r;
      im[F] = x0i;
      odd_outputs<P, M, F, 1>(re, im, tr[0], ti[0], ar, ai, br, bi);
      combine_odd<P, M, F + 1>(re, im, sr, si);
    }
  }
  template <int P, int M, int F, int S>
  static __device__ __forceinline__ void odd_twiddle(float (&tr)[P], float (&ti)[P], const float (&sr)[P][M],
                                                     const float (&si)[P][M]) {
    if constexpr (S < P) {
      if constexpr (F == 0) {
        tr[S] = sr[S][F];
        ti[S] = si[S][F];
      } else {
        constexpr float c = tw_cos(S * F, R);
        constexpr float s = INV ? tw_sin(S * F, R) : -tw_sin(S * F, R);
        tr[S] = c * sr[S][F] - s * si[S][F];
        ti[S] = c * si[S][F] + s * sr[S][F];
      }
      odd_twiddle<P, M, F, S + 1>(tr, ti, sr, si);
    }
  }
  template <int P, int M, int F, int MM>
  static __device__ __forceinline__ void odd_outputs(float (&re)[R], float (&im)[R], float t0r, float t0i,
                                                     const float (&ar)[(P - 1) / 2 + 1], const float (&ai)[(P - 1) / 2 + 1],
                                                     const float (&br)[(P - 1) / 2 + 1], const float (&bi)[(P - 1) / 2 + 1]) {
    constexpr int H = (P - 1) / 2;
    if constexpr (MM <= H) {
      float cr = t0r, ci = t0i, qr = 0.f, qi = 0.f;
      odd_terms<P, MM, 1>(cr, ci, qr, qi, ar, ai, br, bi);
      // forward: X_m = C - i Q, X_(p-m) = C + i Q; inverse: the other way round
      if constexpr (INV) {
        re[F + M * MM] = cr - qi;
        im[F + M * MM] = ci + qr;
        re[F + M * (P - MM)] = cr + qi;
        im[F + M * (P - MM)] = ci - qr;
      } else {
        re[F + M * MM] = cr + qi;
        im[F + M * MM] = ci - qr;
        re[F + M * (P - MM)] = cr - qi;
        im[F + M * (P - MM)] = ci + qr;
      }
      odd_outputs<P, M, F, MM + 1>(re, im, t0r, t0i, ar, ai, br, bi);
    }
  }
  template <int P, int MM, int S>
  static __device__ __forceinline__ void odd_terms(float& cr, float& ci, float& qr, float& qi,
                                                   const float (&ar)[(P - 1) / 2 + 1], const float (&ai)[(P - 1) / 2 + 1],
                                                   const float (&br)[(P - 1) / 2 + 1], const float (&bi)[(P - 1) / 2 + 1]) {
    if constexpr (S <= (P - 1) / 2) {
      constexpr float c = tw_cos((S * MM) % P, P), s = tw_sin((S * MM) % P, P);
      cr = fmaf(c, ar[S], cr);
      ci = fmaf(c, ai[S], ci);
      qr = fmaf(s, br[S], qr);
      qi = fmaf(s, bi[S], qi);
      odd_terms<P, MM, S + 1>(cr, ci, qr, qi, ar, ai, br, bi);
    }
  }

  static __device__ __forceinline__ void run(float (&re)[R], float (&im)[R]) {
    if constexpr (R % 2 == 0) {
      float er[R / 2], ei[R / 2], pr[R / 2], pi[R / 2];
#pragma unroll
      for (int i = 0; i < R / 2; ++i) {
        er[i] = re[2 * i];
        ei[i] = im[2 * i];
        pr[i] = re[2 * i + 1];
        pi[i] = im[2 * i + 1];
      }
      FftReg<R / 2, INV>::run(er, ei);
      FftReg<R / 2, INV>::run(pr, pi);
      combine<0>(re, im, er, ei, pr, pi);
    } else {
      constexpr int P = smallest_odd_factor(R), M = R / P;
      float sr[P][M], si[P][M];
#pragma unroll
      for (int s = 0; s < P; ++s) {
#pragma unroll
        for (int n = 0; n < M; ++n) {
          sr[s][n] = re[P * n + s];
          si[s][n] = im[P * n + s];
        }
        FftReg<M, INV>::run(sr[s], si[s]);
      }
      combine_odd<P, M, 0>(re, im, sr, si);
    }
  }
};

template <bool INV>
struct FftReg<1, INV> {
  static __device__ __forceinline__ void run(float (&)[1], float (&)[1]) {}
};

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
