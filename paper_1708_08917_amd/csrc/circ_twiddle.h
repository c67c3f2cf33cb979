// Twiddle factors W_n^m = exp(-2*pi*i*m/n) as compile-time constants.
//
// The paper keeps the FFT coefficients (real and imaginary parts) in a ROM
// (Sec. 4.2).  Here they are evaluated in double precision at compile time and
// rounded once to fp32: small ones become immediates of the in-register
// butterflies, the inter-pass ones live in a 512-entry table in the code object.
#pragma once

namespace circ {

constexpr double kPi = 3.141592653589793238462643383279502884;

// Taylor series, used only for |x| <= pi/4 where 11 terms are exact to < 1e-17.
constexpr double sin_small(double x) {
  double x2 = x * x, term = x, sum = x;
  for (int n = 1; n <= 11; ++n) {
    term *= -x2 / double((2 * n) * (2 * n + 1));
    sum += term;
  }
  return sum;
}
constexpr double cos_small(double x) {
  double x2 = x * x, term = 1.0, sum = 1.0;
  for (int n = 1; n <= 11; ++n) {
    term *= -x2 / double((2 * n - 1) * (2 * n));
    sum += term;
  }
  return sum;
}

struct cpair { double c, s; };

// (cos, sin) of 2*pi*m/n, reduced to the first octant by exact symmetries.
constexpr cpair cos_sin_frac(int m, int n) {
  double fr = double(m % n) / double(n);   // exact for power-of-two n
  double sc = 1.0, ss = 1.0;
  if (fr > 0.5) { fr = 1.0 - fr; ss = -ss; }          // theta -> 2pi - theta
  if (fr > 0.25) { fr = 0.5 - fr; sc = -sc; }         // theta -> pi - theta
  bool swap = false;
  if (fr > 0.125) { fr = 0.25 - fr; swap = true; }    // theta -> pi/2 - theta
  double x = 2.0 * kPi * fr;
  double c = cos_small(x), s = sin_small(x);
  if (swap) { double t = c; c = s; s = t; }
  return cpair{sc * c, ss * s};
}

constexpr float tw_cos(int m, int n) { return float(cos_sin_frac(m, n).c); }
constexpr float tw_sin(int m, int n) { return float(cos_sin_frac(m, n).s); }

constexpr int kTwN = 512;   // largest supported block size

struct alignas(16) TwiddleTable {
  float c[kTwN];   // cos(2 pi m / 512)
  float s[kTwN];   // sin(2 pi m / 512)
  float cs[2 * kTwN];   // the same values as (cos, sin) pairs, for one 8-byte load per twiddle
  constexpr TwiddleTable() : c(), s(), cs() {
    for (int m = 0; m < kTwN; ++m) {
      cpair v = cos_sin_frac(m, kTwN);
      c[m] = float(v.c);
      s[m] = float(v.s);
      cs[2 * m] = float(v.c);
      cs[2 * m + 1] = float(v.s);
    }
  }
};

// The K roots of unity (cos, sin)(2 pi m / K) of a block size that does not divide 512.
template <int K>
struct alignas(8) RootsTable {
  float cs[2 * K];
  constexpr RootsTable() : cs() {
    for (int m = 0; m < K; ++m) {
      cpair v = cos_sin_frac(m, K);
      cs[2 * m] = float(v.c);
      cs[2 * m + 1] = float(v.s);
    }
  }
};

}  // namespace circ
