// Per-frequency complex GEMM on the fp32 matrix cores, LDS-tiled and persistent:
//   C[f][m][n] = sum_k A[f][k][m] * B[f][k][n]        (B conjugated if CONJ_B)
// This is the "o" of Algorithm 1 with the sum over j moved inside the IFFT (Eq. 3 is linear),
// and, with the batch as the reduction index, the accumulation of Algorithm 2's weight
// gradient in the frequency domain.
//
// A is stored with m fastest, B and C with n fastest, so a k-slab of either operand is a set
// of contiguous rows and goes to LDS as it is; v_mfma_f32_32x32x2_f32 then takes, per lane,
// element (k = lane/32, m or n = lane%32) of a slab, which is one 8-byte LDS read (re, im).
// A workgroup of four waves owns a (32*FM*WM) x (32*WN) tile of one frequency; every wave owns
// FM 32x32 sub-tiles.  A complex product is three real accumulations (Gauss, see multiply).
//
// The DC and the Nyquist bin of a real signal are real (Sec. 4.1: the spectrum of a real
// sequence is Hermitian), so these two frequencies share one tile: its operands carry
// (bin 0, bin K/2) in the (re, im) slots and only two of its four accumulations carry data.
//
// A workgroup walks a contiguous run of tiles.  The next k-slab - of the same tile or of the
// next one - is fetched into registers while the current one is multiplied, and the stores of a
// finished tile overlap the arithmetic of the next, so that the memory system and the matrix
// cores are busy at the same time.
#pragma once

#include <hip/hip_runtime.h>

#include "circ_kernels.h"

namespace circ {

template <int FM, int WM, int WN>
struct GemmShape {
  static constexpr int TM = 32 * FM * WM, TN = 32 * WN, KT = 16, NT = 64 * WM * WN;
  static constexpr int LA = KT * TM / NT, LB = KT * TN / NT;   // float2 loads per thread and slab
  static_assert(WM * WN == 4, "four waves per workgroup");
  static_assert(KT * TM % NT == 0 && KT * TN % NT == 0, "slab must split evenly over the threads");
};

// Grid: 1-D, a multiple of 8.  Tile index t = ((fi*ksplit + ks)*ntm + mt)*ntn + nt with
// fi = 0..NF-3 for frequency fi+1 and fi = NF-2 for the shared tile of bins 0 and NF-1.
// Workgroup v owns tiles [v*chunk, (v+1)*chunk); v is derived from blockIdx.x so that
// neighbouring runs (which share A or B) sit on the same XCD (workgroups go round-robin to
// the 8 XCDs, each with a private L2).  Split-K: slice ks reduces k in
// [ks*kchunk, (ks+1)*kchunk) and writes its partial sums to C + ks*part_stride (summed later
// in a fixed order).
// A_T: A is stored [f][m][k] (k fastest, row pitch Kd) instead of [f][k][m]: the slab is then
// fetched along k and kept in LDS as [m][KT+1]; the odd pitch makes the operand reads (32 lanes
// along m) hit every bank once.  This lets backward-weights take the spectrum of dy in the
// layout that backward-data needs, so that dy is transformed once.
template <int FM, int WM, int WN, bool CONJ_B, bool A_T>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void cgemm_tiled_kernel(const float2* __restrict__ A, const float2* __restrict__ B,
                                                          float2* __restrict__ C, int M, int N, int Kd, int NF,
                                                          long long sA, long long sB, long long sC, int ntm, int ntn,
                                                          int ksplit, int kchunk, long long part_stride,
                                                          unsigned ntiles, unsigned chunk) {
  using Sh = GemmShape<FM, WM, WN>;
  constexpr int TM = Sh::TM, TN = Sh::TN, KT = Sh::KT, NT = Sh::NT, LA = Sh::LA, LB = Sh::LB;
  constexpr int PA = KT + 1;                       // row pitch of the transposed A slab
  __shared__ float2 sa[A_T ? TM * PA : KT * TM];
  __shared__ float2 sb[KT * TN];

  const unsigned v = (blockIdx.x & 7u) * (gridDim.x >> 3) + (blockIdx.x >> 3);
  const unsigned first = v * chunk, last = min(ntiles, first + chunk);
  if (first >= last) return;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int nslab = (min(kchunk, Kd) + KT - 1) / KT;

  struct Tile {
    const float2 *a0, *a1, *b0, *b1;   // a1, b1: the Nyquist bin of the shared tile
    float2 *c0, *c1;
    int m0, n0, kbeg, kend;
    bool shared;
  };
  auto decode = [&](unsigned t) {
    Tile T;
    const int nt = int(t % unsigned(ntn));
    unsigned r = t / unsigned(ntn);
    const int mt = int(r % unsigned(ntm));
    r /= unsigned(ntm);
    const int ks = int(r % unsigned(ksplit)), fi = int(r / unsigned(ksplit));
    T.shared = fi == NF - 2;
    const int f = T.shared ? 0 : fi + 1;
    T.m0 = mt * TM;
    T.n0 = nt * TN;
    T.kbeg = ks * kchunk;
    T.kend = min(Kd, T.kbeg + kchunk);
    T.a0 = A + f * sA;
    T.b0 = B + f * sB;
    T.c0 = C + f * sC + ks * part_stride;
    T.a1 = A + (NF - 1) * sA;
    T.b1 = B + (NF - 1) * sB;
    T.c1 = C + (NF - 1) * sC + ks * part_stride;
    return T;
  };

  // global -> register staging of one k-slab.  Addresses are clamped so that the loads are
  // unconditional; rows past kend and columns past M / N are replaced by zeros only when the
  // registers are copied to LDS, so that nothing waits for a load before the slab that is
  // being multiplied is finished.
  float2 ra[LA], rb[LB];
  float ra1[LA], rb1[LB];          // bin K/2 of the shared tile
  unsigned keep_a = 0, keep_b = 0; // bit e: element e is inside the operand
  bool staged_shared = false;
  // Every thread keeps its column of the slab (TM and TN divide the thread count) and walks
  // down the rows; offsets inside one frequency of an operand fit 32 bits (host check).
  // (A_T: a thread keeps its k and walks down the m rows, NT/KT at a time.)
  const int col_a = A_T ? tid % KT : tid % TM, row_a = A_T ? tid / KT : tid / TM;
  const int col_b = tid % TN, row_b = tid / TN;
  auto fetch = [&](const Tile& T, int slab) {
    const int k0 = T.kbeg + slab * KT, klast = max(T.kend - 1, 0);
    keep_a = keep_b = 0;
    staged_shared = T.shared;
    const int nb = T.n0 + col_b;
    const unsigned cb = unsigned(min(nb, N - 1));
    unsigned offa[LA], offb[LB];
    if constexpr (A_T) {
      const int k = k0 + col_a;
      const unsigned ck = unsigned(min(k, klast));
#pragma unroll
      for (int e = 0; e < LA; ++e) {
        const int m = T.m0 + e * (NT / KT) + row_a;
        offa[e] = unsigned(min(m, M - 1)) * unsigned(Kd) + ck;
        ra[e] = T.a0[offa[e]];
        keep_a |= (k < T.kend && m < M) ? (1u << e) : 0u;
      }
    } else {
      const int ma = T.m0 + col_a;
      const unsigned ca = unsigned(min(ma, M - 1));
#pragma unroll
      for (int e = 0; e < LA; ++e) {
        const int k = k0 + e * (NT / TM) + row_a;
        offa[e] = unsigned(min(k, klast)) * unsigned(M) + ca;
        ra[e] = T.a0[offa[e]];
        keep_a |= (k < T.kend && ma < M) ? (1u << e) : 0u;
      }
    }
#pragma unroll
    for (int e = 0; e < LB; ++e) {
      const int k = k0 + e * (NT / TN) + row_b;
      offb[e] = unsigned(min(k, klast)) * unsigned(N) + cb;
      rb[e] = T.b0[offb[e]];
      keep_b |= (k < T.kend && nb < N) ? (1u << e) : 0u;
    }
    if (T.shared) {
#pragma unroll
      for (int e = 0; e < LA; ++e) ra1[e] = T.a1[offa[e]].x;
#pragma unroll
      for (int e = 0; e < LB; ++e) rb1[e] = T.b1[offb[e]].x;
    }
  };
  auto stage = [&]() {
#pragma unroll
    for (int e = 0; e < LA; ++e) {
      float2 val = ra[e];
      if (staged_shared) val.y = ra1[e];
      if (!((keep_a >> e) & 1u)) val = make_float2(0.f, 0.f);
      if constexpr (A_T) sa[(e * (NT / KT) + row_a) * PA + col_a] = val;
      else sa[e * NT + tid] = val;
    }
#pragma unroll
    for (int e = 0; e < LB; ++e) {
      float2 val = rb[e];
      if (staged_shared) val.y = rb1[e];
      if (!((keep_b >> e) & 1u)) val = make_float2(0.f, 0.f);
      sb[e * NT + tid] = val;
    }
  };

  // operand element (k = 2*kk + lane/32, m = lane%32 of sub-tile fm) sits at pa[kk*KSA + fm*FSA]
  const float2* pa = A_T ? sa + (wm * 32 * FM + (lane & 31)) * PA + (lane >> 5)
                         : sa + (lane >> 5) * TM + wm * 32 * FM + (lane & 31);
  constexpr int KSA = A_T ? 2 : 2 * TM, FSA = A_T ? 32 * PA : 32;
  const float2* pb = sb + (lane >> 5) * TN + wn * 32 + (lane & 31);

  // accumulator layout of a 32x32 tile: column = lane % 32; row = 8*(r/4) + 4*(lane/32) + r%4
  // o1, o2, o3: the three sums of products (see multiply)
  auto store_tile = [&](const Tile& T, const floatx16 (&o1)[FM], const floatx16 (&o2)[FM], const floatx16 (&o3)[FM]) {
    const int n = T.n0 + wn * 32 + (lane & 31);
    const int mb = T.m0 + wm * 32 * FM + 4 * (lane >> 5);
    const unsigned base = unsigned(mb) * unsigned(N) + unsigned(n);
#pragma unroll
    for (int fm = 0; fm < FM; ++fm)
#pragma unroll
      for (int rr = 0; rr < 16; ++rr) {
        const int dm = fm * 32 + 8 * (rr / 4) + (rr % 4);
        if (mb + dm < M && n < N) {
          const unsigned off = base + unsigned(dm) * unsigned(N);
          if (T.shared) {
            T.c0[off] = make_float2(o1[fm][rr], 0.f);
            T.c1[off] = make_float2(o3[fm][rr], 0.f);
          } else {
            T.c0[off] = make_float2(o1[fm][rr] - o3[fm][rr], o1[fm][rr] + o2[fm][rr]);
          }
        }
      }
  };

  // One k-slab of the current tile: registers -> LDS, prefetch of the next slab (of this tile or
  // of the next one), 8 k-steps on the matrix cores.
  floatx16 acc1[FM], acc2[FM], acc3[FM];
  auto zero_acc = [&]() {
#pragma unroll
    for (int fm = 0; fm < FM; ++fm)
#pragma unroll
      for (int i = 0; i < 16; ++i) { acc1[fm][i] = 0.f; acc2[fm][i] = 0.f; acc3[fm][i] = 0.f; }
  };
  auto multiply = [&](bool sh) {
    // Three real products per complex one (Gauss): with b.y already conjugated when CONJ_B,
    //   K1 += (ar + ai) br,  K2 += ar (bi - br),  K3 += ai (br + bi);  Re = K1 - K3,  Im = K1 + K2.
    // One instruction sequence for both kinds of tile (two would make the compiler move the
    // accumulators between register files around the branch): the shared tile holds two real
    // bins in (x, y) and multiplies (a.x, b.x) into K1 and (a.y, b.y) into K3, zeros into K2.
#pragma unroll
    for (int kk = 0; kk < KT / 2; ++kk) {
      float2 b = pb[2 * kk * TN];
      if (CONJ_B) b.y = -b.y;
      const float b2 = b.y - b.x, b3 = sh ? (CONJ_B ? -b.y : b.y) : b.x + b.y;
#pragma unroll
      for (int fm = 0; fm < FM; ++fm) {
        const float2 a = pa[kk * KSA + fm * FSA];
        const float a1 = sh ? a.x : a.x + a.y, a2 = sh ? 0.f : a.x;
        acc1[fm] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b.x, acc1[fm], 0, 0, 0);
        acc2[fm] = __builtin_amdgcn_mfma_f32_32x32x2f32(a2, b2, acc2[fm], 0, 0, 0);
        acc3[fm] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b3, acc3[fm], 0, 0, 0);
      }
    }
  };
  // slabs [from, nslab) of tile `cur`; after the last one the first slab of `nxt` is fetched
  auto run_slabs = [&](const Tile& cur, const Tile& nxt, bool more, int from) {
    for (int slab = from; slab < nslab; ++slab) {
      stage();
      __syncthreads();
      if (slab + 1 < nslab) fetch(cur, slab + 1);
      else if (more) fetch(nxt, 0);
      multiply(cur.shared);
      __syncthreads();
    }
  };

  Tile cur = decode(first);
  fetch(cur, 0);
  zero_acc();
  {
    const bool more = first + 1 < last;
    Tile nxt = cur;
    if (more) nxt = decode(first + 1);
    run_slabs(cur, nxt, more, 0);
    // A finished tile is copied to other registers and stored while the first slab of the next
    // tile is multiplied.  Stored right away, the wait for the prefetched operands of the next
    // tile would also wait for these stores (loads and stores complete in one order), and all
    // workgroups reach that point together.
    for (unsigned t = first + 1; t < last; ++t) {
      floatx16 out1[FM], out2[FM], out3[FM];
#pragma unroll
      for (int fm = 0; fm < FM; ++fm) { out1[fm] = acc1[fm]; out2[fm] = acc2[fm]; out3[fm] = acc3[fm]; }
      const Tile done = cur;
      cur = nxt;
      const bool more2 = t + 1 < last;
      if (more2) nxt = decode(t + 1);
      zero_acc();
      stage();
      __syncthreads();
      store_tile(done, out1, out2, out3);
      if (1 < nslab) fetch(cur, 1);
      else if (more2) fetch(nxt, 0);
      multiply(cur.shared);
      __syncthreads();
      run_slabs(cur, nxt, more2, 1);
    }
  }
  store_tile(cur, acc1, acc2, acc3);
}

}  // namespace circ
