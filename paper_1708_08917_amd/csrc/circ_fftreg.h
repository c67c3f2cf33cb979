// In-register FFT of R points (any R) and the split K = R1 * R2 of the two-pass transforms: the
// arithmetic core of every transform in the library.
// Plain C++ apart from the __device__ / __forceinline__ markers: tests/test_fftreg_host.py compiles
// it for the CPU and checks every size the kernels use against the definition of the transform.
#pragma once

#include <cmath>

#include "circ_twiddle.h"

namespace circ {

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

}  // namespace circ
