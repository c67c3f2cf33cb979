// CPU check of the in-register transforms (csrc/circ_fftreg.h) against the definition of the DFT,
//   X[f] = sum_n x[n] e^{-/+ 2 pi i f n / R}   (Sec. 4.1: the FFT computes exactly this sum),
// evaluated in double precision, for every sub-transform size the kernels instantiate; and of the
// two-pass split K = R1 * R2 (first pass over n1 with n = R2*n1 + n2, twiddle W_K^(f1*n2), second
// pass over n2, output index f = f1 + R1*f2) for every block size with a fast transform.
// Prints one line per case: name, size, max error relative to the largest output.
#define __device__
#define __forceinline__ inline
#include <cstdio>
#include <cstdlib>
#include <vector>
#include "circ_fftreg.h"

using namespace circ;

static double frand() { return 2.0 * (double(rand()) / RAND_MAX) - 1.0; }

static void naive(int R, bool inv, const std::vector<double>& xr, const std::vector<double>& xi, std::vector<double>& yr,
                  std::vector<double>& yi) {
  const double sg = inv ? 1.0 : -1.0;
  for (int f = 0; f < R; ++f) {
    double sr = 0, si = 0;
    for (int n = 0; n < R; ++n) {
      const double a = sg * 2.0 * kPi * double((long long)f * n % R) / R;
      sr += xr[n] * cos(a) - xi[n] * sin(a);
      si += xr[n] * sin(a) + xi[n] * cos(a);
    }
    yr[f] = sr;
    yi[f] = si;
  }
}

template <int R, bool INV>
static void check_reg() {
  std::vector<double> xr(R), xi(R), yr(R), yi(R);
  float re[R], im[R];
  for (int n = 0; n < R; ++n) { xr[n] = frand(); xi[n] = frand(); re[n] = float(xr[n]); im[n] = float(xi[n]); xr[n] = re[n]; xi[n] = im[n]; }
  naive(R, INV, xr, xi, yr, yi);
  FftReg<R, INV>::run(re, im);
  double err = 0, mx = 0;
  for (int f = 0; f < R; ++f) {
    err = fmax(err, fmax(fabs(re[f] - yr[f]), fabs(im[f] - yi[f])));
    mx = fmax(mx, fmax(fabs(yr[f]), fabs(yi[f])));
  }
  printf("reg %s %d %.3e\n", INV ? "inv" : "fwd", R, err / mx);
}

template <int K, bool INV>
static void check_two_pass() {
  constexpr int R1 = radix1_of(K), R2 = radix2_of(K);
  static_assert(R1 * R2 == K && R1 <= R2, "split");
  std::vector<double> xr(K), xi(K), yr(K), yi(K);
  std::vector<float> zr(K), zi(K), orr(K), oi(K);
  for (int n = 0; n < K; ++n) { zr[n] = float(frand()); zi[n] = float(frand()); xr[n] = zr[n]; xi[n] = zi[n]; }
  naive(K, INV, xr, xi, yr, yi);
  std::vector<float> ar(K), ai(K);                       // A[f1][n2] at R2*f1 + n2
  for (int n2 = 0; n2 < R2; ++n2) {
    float re[R1], im[R1];
    for (int n1 = 0; n1 < R1; ++n1) { re[n1] = zr[R2 * n1 + n2]; im[n1] = zi[R2 * n1 + n2]; }
    FftReg<R1, INV>::run(re, im);
    for (int f1 = 0; f1 < R1; ++f1) {
      const cpair w = cos_sin_frac((f1 * n2) % K, K);
      const float c = float(w.c), s = INV ? float(w.s) : -float(w.s);
      ar[R2 * f1 + n2] = c * re[f1] - s * im[f1];
      ai[R2 * f1 + n2] = c * im[f1] + s * re[f1];
    }
  }
  for (int f1 = 0; f1 < R1; ++f1) {
    float re[R2], im[R2];
    for (int n2 = 0; n2 < R2; ++n2) { re[n2] = ar[R2 * f1 + n2]; im[n2] = ai[R2 * f1 + n2]; }
    FftReg<R2, INV>::run(re, im);
    for (int f2 = 0; f2 < R2; ++f2) { orr[f1 + R1 * f2] = re[f2]; oi[f1 + R1 * f2] = im[f2]; }
  }
  double err = 0, mx = 0;
  for (int f = 0; f < K; ++f) {
    err = fmax(err, fmax(fabs(orr[f] - yr[f]), fabs(oi[f] - yi[f])));
    mx = fmax(mx, fmax(fabs(yr[f]), fabs(yi[f])));
  }
  printf("two-pass %s %d %.3e\n", INV ? "inv" : "fwd", K, err / mx);
}

template <int... Rs>
static void all_reg() { (check_reg<Rs, false>(), ...); (check_reg<Rs, true>(), ...); }
template <int... Ks>
static void all_two_pass() { (check_two_pass<Ks, false>(), ...); (check_two_pass<Ks, true>(), ...); }

int main() {
  srand(12345);
  all_reg<1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 12, 15, 16, 20, 24, 25, 32>();
  all_two_pass<2, 4, 8, 16, 32, 64, 128, 256, 512, 12, 24, 48, 96, 192, 384, 20, 40, 80, 160, 320, 100, 200, 400>();
  return 0;
}
