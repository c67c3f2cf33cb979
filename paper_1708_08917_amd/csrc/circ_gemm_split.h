// Per-frequency complex GEMM with fp32 operands on the bfloat16 matrix instruction:
//   C[f][m][n] = sum_k A[f][k][m] * B[f][k][n]        (B conjugated if CONJ_B)
// - the "o" of Algorithm 1 summed over the input blocks j (Eq. 3 is linear, so the sum moves
// inside the IFFT) and, with the transposed, conjugated weights, the same step of Algorithm 2.
//
// The fp32 matrix instruction bounds the plain fp32 kernel (cgemm_kernel).  Here every fp32
// operand value x is written as the sum of three bfloat16 terms,
//   h = bf16(x),  m = bf16(x - h),  l = bf16(x - h - m)      (both differences are exact in fp32),
// which reproduce x to within 2^-24 |x|, and a product a*b is taken as the six partial products
// of combined order <= 2 (hh, hm, mh, hl, lh, mm); the three left out (ml, lm, ll) and the two
// residuals add up to at most 2^-22 |a b| (2^-24.5 over random operands: one rounding of an fp32
// product is 2^-24).  Partial products of bfloat16 values are exact in fp32 and the matrix cores
// accumulate in fp32, so the result carries the rounding errors of an fp32 sum of products (measured:
// no larger than those of the fp32 matrix instruction), at 6/16 of the matrix-core time of the fp32
// instruction (v_mfma_f32_32x32x16_bf16 multiplies 8 times as many values in half the cycles).
// bfloat16 has the exponent range of fp32, so no scaling is involved; the two ends of that range
// are the exceptions: |x| within 2^-8 of the largest finite fp32 value rounds to infinity in its
// first term, and the lower terms of |x| < 2^-110 fall below the smallest normal value.
//
// A complex product runs on the real instruction with the (re, im) pairs interleaved along the
// reduction index:   Re C = A' . (br, -bi, ...)      Im C = A' . (bi, br, ...),   A' = (ar, ai, ...)
// so only B is rewritten, lane-locally: a sign flip of one half and a swap inside each 32-bit word.
//
// A is stored with m fastest, B and C with n fastest.  A workgroup of four waves owns a 64 (m) x
// 128 (n) tile of one frequency, wave w the columns [32w, 32w + 32) as two 32 x 32 sub-tiles.
// Lane (h, r) = (lane / 32, lane % 32) of a matrix instruction supplies the complex elements
// k = 8*step + 4h .. + 3 of row (A) or column (B) r:
// - B: these are four loads straight from memory (two runs of 32 consecutive n per instruction);
//   every value of B is read by exactly one lane, split in registers and used for both sub-tiles.
//   The requests run RING = 4 steps (32 k) ahead of their use in a register ring (a scheduling
//   barrier keeps the compiler from sinking them to their first use).
// - A (the small operand: the weights of one frequency) is split once per workgroup and slab
//   and kept in LDS as planes [term][m][k] (row pitch 68 words: eight consecutive rows start at
//   eight different groups of four banks, for the 16-byte stores and for the 16-byte fragment
//   reads alike); consecutive tiles of a workgroup that share the slab do not stage it again.
// The waves of a workgroup meet at a barrier only when A is staged.
#pragma once

#include <hip/hip_runtime.h>

#include "circ_half.h"
#include "circ_kernels.h"
#include "circ_probe.h"

namespace circ {

struct SplitGemmShape {
  static constexpr int TM = 64, TN = 128, KA = 64, PITCH = KA + 4, NT = 256, NSTEP = KA / 8, RING = 4;
  static constexpr int PLANE = TM * PITCH;                                  // words per term
};

typedef __bf16 bfloatx2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

// (re, im) -> one word of two bfloat16 values (re in the low half), round to nearest even
__device__ __forceinline__ unsigned pack_bf16x2(float re, float im) {
  const floatx2 v = {re, im};
  union { bfloatx2 b; unsigned u; } c;
  c.b = __builtin_convertvector(v, bfloatx2);
  return c.u;
}
// v = h + m + l up to 2^-24 |v| per component
__device__ __forceinline__ void split_bf16x3(float2 v, unsigned& h, unsigned& m, unsigned& l) {
  h = pack_bf16x2(v.x, v.y);
  float2 r = make_float2(v.x - __uint_as_float(h << 16), v.y - __uint_as_float(h & 0xffff0000u));
  m = pack_bf16x2(r.x, r.y);
  r = make_float2(r.x - __uint_as_float(m << 16), r.y - __uint_as_float(m & 0xffff0000u));
  l = pack_bf16x2(r.x, r.y);
}

// Grid: 1-D, a multiple of 8.  Tile t = (f*ntm + mt)*ntn + nt; workgroup v owns `base` consecutive
// tiles, the first `rem` workgroups one more; v is taken from blockIdx.x so that neighbouring
// runs, which share the A operand of a frequency, sit on the same XCD (workgroups go round-robin
// to the 8 XCDs, each with a private L2).  Offsets inside one frequency of an operand fit 32 bits
// (host check).
template <bool CONJ_B>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void cgemm_split_kernel(const float2* __restrict__ A, const float2* __restrict__ B,
                                                          float2* __restrict__ C, int M, int N, int Kd, long long sA,
                                                          long long sB, long long sC, int ntm, int ntn, unsigned ntiles,
                                                          unsigned base, unsigned rem) {
  using Sh = SplitGemmShape;
  constexpr int TM = Sh::TM, TN = Sh::TN, KA = Sh::KA, PITCH = Sh::PITCH, NSTEP = Sh::NSTEP;
  __shared__ __attribute__((aligned(16))) unsigned la[3 * Sh::PLANE];      // [term][m][k]

  const unsigned v = (blockIdx.x & 7u) * (gridDim.x >> 3) + (blockIdx.x >> 3);
  const unsigned first = v * base + min(v, rem);
  if (first >= ntiles) return;                         // (the grid is rounded up to a multiple of 8)
  const unsigned count = min(base + (v < rem ? 1u : 0u), ntiles - first);
  CIRC_PROBE(0);
  const int nkc = (Kd + KA - 1) / KA;                  // slabs per tile
  const unsigned nslabs = count * unsigned(nkc);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r = lane & 31, h = lane >> 5;

  struct Slab {
    int f, m0, n0, kc;
    int last;                // 1: the last slab of its tile
  };
  auto slab_at = [&](unsigned i) {
    Slab S;
    const unsigned t = first + i / unsigned(nkc);
    const int ks = int(i % unsigned(nkc));
    S.kc = ks * KA;
    S.last = ks == nkc - 1 ? 1 : 0;
    S.n0 = int(t % unsigned(ntn)) * TN;
    S.m0 = int((t / unsigned(ntn)) % unsigned(ntm)) * TM;
    S.f = int(t / unsigned(ntn * ntm));
    return S;
  };

  // B of a slab: lane (h, r) of wave w takes column n0 + 32w + r (clamped: columns past N are
  // computed on copies and not stored), rows kc + 8*step + 4h + u (clamped; zeroed at the split)
  constexpr int RING = Sh::RING;                       // steps of B in flight
  float2 braw[RING][4];
  auto b_column = [&](const Slab& S) { return B + S.f * sB + min(S.n0 + 32 * wave + r, N - 1); };
  // (pitch: N, or 0 for the loads behind the last slab, which then all read one valid element: the
  // loads stay unconditional, so that no register copy - and with it a wait for the youngest
  // loads - appears at the head of the slab loop)
  auto fetch_b = [&](const float2* bcol, unsigned pitch, int kc, int step) {
    const unsigned row0 = unsigned(kc + 4 * h) * pitch;             // the rest of the offset is uniform
#pragma unroll
    for (int u = 0; u < 4; ++u)
      braw[step % RING][u] = bcol[kc + 8 * step + 4 * h + u < Kd ? row0 + unsigned(8 * step + u) * pitch : unsigned(Kd - 1) * pitch];
  };

  // A of a slab -> LDS planes: thread (row tid % 64, k-quads tid / 64 + 4e); rows past M and k past
  // Kd are staged as zeros
  const int ra = tid & 63, qa = tid >> 6;
  float2 va[4][4];
  auto load_a = [&](const Slab& S) {
    const float2* acol = A + S.f * sA + min(S.m0 + ra, M - 1);
    const unsigned row0 = unsigned(S.kc + 4 * qa) * unsigned(M);
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
      for (int u = 0; u < 4; ++u)
        va[e][u] = acol[S.kc + 4 * (qa + 4 * e) + u < Kd ? row0 + unsigned(16 * e + u) * unsigned(M) : unsigned(Kd - 1) * unsigned(M)];
  };
  auto put_a = [&](const Slab& S) {
    const bool oka = S.m0 + ra < M;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      uint4 th, tm, tl;
      unsigned* ph = reinterpret_cast<unsigned*>(&th);
      unsigned* pm = reinterpret_cast<unsigned*>(&tm);
      unsigned* pl = reinterpret_cast<unsigned*>(&tl);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const bool keep = oka && S.kc + 4 * (qa + 4 * e) + u < Kd;
        split_bf16x3(keep ? va[e][u] : make_float2(0.f, 0.f), ph[u], pm[u], pl[u]);
      }
      unsigned* d = la + ra * PITCH + 4 * (qa + 4 * e);
      *reinterpret_cast<uint4*>(d) = th;
      *reinterpret_cast<uint4*>(d + Sh::PLANE) = tm;
      *reinterpret_cast<uint4*>(d + 2 * Sh::PLANE) = tl;
    }
  };

  hfloatx16 cre[2], cim[2];
  auto zero_acc = [&]() {
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
      for (int i = 0; i < 16; ++i) { cre[s][i] = 0.f; cim[s][i] = 0.f; }
  };
  // accumulator layout of a 32 x 32 tile: column = lane % 32; register i holds row 8*(i/4) + 4*(lane/32) + i%4
  auto store_rows = [&](float2* c, int m0, const hfloatx16 (&vre)[2], const hfloatx16 (&vim)[2], int j0, int nj) {
#pragma unroll
    for (int j = j0; j < j0 + nj; ++j) {
      const int s = j >> 4, i = j & 15;
      const int row = m0 + 32 * s + 8 * (i / 4) + 4 * h + (i % 4);
      if (row < M) c[unsigned(row) * unsigned(N)] = make_float2(vre[s][i], vim[s][i]);
    }
  };
  auto c_column = [&](const Slab& S) -> float2* {
    const int col = S.n0 + 32 * wave + r;
    return col < N ? C + S.f * sC + col : nullptr;
  };

  // A fragment of lane (h, r): words [8*step + 4h, 8*step + 4h + 4) of row r (sub-tile 1: row 32 + r)
  const unsigned* fa = la + r * PITCH + 4 * h;

  // the first slab: A is requested ahead of B (loads return in issue order), so that its split
  // runs while B is still on its way
  Slab cur = slab_at(0);
  load_a(cur);
  {
    const float2* bcol = b_column(cur);
#pragma unroll
    for (int step = 0; step < RING; ++step) fetch_b(bcol, unsigned(N), cur.kc, step);
  }
  put_a(cur);
  __syncthreads();
  zero_acc();
  CIRC_PROBE(1);
  int f_staged = cur.f, m_staged = cur.m0, kc_staged = cur.kc;
  for (unsigned i = 0; i < nslabs; ++i) {
    const bool more = i + 1 < nslabs;
    Slab nxt = cur;
    if (more) nxt = slab_at(i + 1);
    const float2* bnext = more ? b_column(nxt) : B;
    const unsigned pnext = more ? unsigned(N) : 0u;
    const float2* bcur = b_column(cur);
    if (cur.f != f_staged || cur.m0 != m_staged || cur.kc != kc_staged) {     // uniform over the workgroup
      __syncthreads();                                  // every wave has finished with the planes
      load_a(cur);
      put_a(cur);
      __syncthreads();
      f_staged = cur.f;
      m_staged = cur.m0;
      kc_staged = cur.kc;
    }
    CIRC_PROBE(2 + 3 * i);
#pragma unroll
    for (int step = 0; step < NSTEP; ++step) {
      uint4 bt[3];
      {
        unsigned* ph = reinterpret_cast<unsigned*>(&bt[0]);
        unsigned* pm = reinterpret_cast<unsigned*>(&bt[1]);
        unsigned* pl = reinterpret_cast<unsigned*>(&bt[2]);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const bool keep = cur.kc + 8 * step + 4 * h + u < Kd;
          split_bf16x3(keep ? braw[step % RING][u] : make_float2(0.f, 0.f), ph[u], pm[u], pl[u]);
        }
      }
      // the registers are free again: RING steps ahead, in this slab or the next one
      if (step + RING < NSTEP) fetch_b(bcur, unsigned(N), cur.kc, step + RING);
      else fetch_b(bnext, pnext, nxt.kc, step + RING - NSTEP);
      __builtin_amdgcn_sched_barrier(0);                // the requests stay here, RING steps ahead of their use
      uint4 a[2][3], bre[3], bim[3];
#pragma unroll
      for (int term = 0; term < 3; ++term) {
        a[0][term] = *reinterpret_cast<const uint4*>(fa + term * Sh::PLANE + 8 * step);
        a[1][term] = *reinterpret_cast<const uint4*>(fa + term * Sh::PLANE + 32 * PITCH + 8 * step);
        const uint4 b = bt[term];
        // re form (br, -bi) and im form (bi, br); with conj(B): (br, bi) and (-bi, br)
        constexpr unsigned sre = CONJ_B ? 0u : 0x80000000u, sim = CONJ_B ? 0x8000u : 0u;
        bre[term] = make_uint4(b.x ^ sre, b.y ^ sre, b.z ^ sre, b.w ^ sre);
        bim[term] = make_uint4(__builtin_amdgcn_alignbit(b.x, b.x, 16) ^ sim, __builtin_amdgcn_alignbit(b.y, b.y, 16) ^ sim,
                               __builtin_amdgcn_alignbit(b.z, b.z, 16) ^ sim, __builtin_amdgcn_alignbit(b.w, b.w, 16) ^ sim);
      }
      // the six partial products, smallest first: (m,m), (l,h), (h,l), (m,h), (h,m), (h,h); no
      // branch around the matrix instructions, so that the accumulators stay in place
      constexpr int TA[6] = {1, 2, 0, 1, 0, 0}, TB[6] = {1, 0, 2, 0, 1, 0};
#pragma unroll
      for (int pp = 0; pp < 6; ++pp) {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
          cre[s] = mfma16<true>(a[s][TA[pp]], bre[TB[pp]], cre[s]);
          cim[s] = mfma16<true>(a[s][TA[pp]], bim[TB[pp]], cim[s]);
        }
      }
    }
    CIRC_PROBE(3 + 3 * i);
    if (cur.last) {
      float2* c = c_column(cur);
      if (c != nullptr) store_rows(c, cur.m0, cre, cim, 0, 32);
      zero_acc();
    }
    CIRC_PROBE(4 + 3 * i);
    cur = nxt;
  }
}


// Backward-weights (Algorithm 2: the spectrum of dL/dw_ij is the sum over the batch of
// FFT(dL/da_i) o conj(FFT(x_j))) on the same split arithmetic:
//   C[ks][f][m][n] = sum_{k in slice ks} A[f][m][k] * conj(B[f][k][n])
// A = the spectrum of dy stored [f][i][b] (k = the batch index fastest: the order backward-data
// needs it in, so dy is transformed once), B = the spectrum of x stored [f][b][j] (n fastest).
// The output is narrow (p x q block pairs) and the reduction long, so the reduction is cut into
// `ksplit` slices of `kchunk` values (a multiple of 64) whose partial sums go to
// C + ks*part_stride, to be added later in index order.
// A workgroup owns a 64 (m) x 64 (n) tile of one (frequency, slice): wave w takes the columns
// 32*(w % 2) .. + 31 and, of every slab of 64 k, the steps 4*(w / 2) .. + 3 - all four waves
// share the staged A slab, and the two halves of the reduction meet in LDS at the end of the tile.
// B goes from memory to the lanes as in cgemm_split_kernel; the A slab of the next 64 k is
// requested (lanes along k: runs of 512 bytes) while the current one is multiplied.
// Requires Kd to be a multiple of 4 (16-byte loads of whole quads along k); offsets inside one
// frequency fit 32 bits (host check).
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void cgemm_split_dw_kernel(
    const float2* __restrict__ A, const float2* __restrict__ B, float2* __restrict__ C, int M, int N, int Kd, long long sA,
    long long sB, long long sC, int ntm, int ntn, int ksplit, int kchunk, long long part_stride, unsigned ntiles, unsigned base,
    unsigned rem) {
  using Sh = SplitGemmShape;
  constexpr int TM = Sh::TM, TN = 64, KA = Sh::KA, PITCH = Sh::PITCH, WSTEP = Sh::NSTEP / 2;   // steps per wave and slab
  __shared__ __attribute__((aligned(16))) unsigned la[3 * Sh::PLANE];      // [term][m][k]; at a tile's end: partial sums

  const unsigned v = (blockIdx.x & 7u) * (gridDim.x >> 3) + (blockIdx.x >> 3);
  const unsigned first = v * base + min(v, rem);
  if (first >= ntiles) return;
  const unsigned count = min(base + (v < rem ? 1u : 0u), ntiles - first);
  const int nkc = kchunk / KA;                         // slabs per tile
  const unsigned nslabs = count * unsigned(nkc);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wn = wave & 1, kh = wave >> 1;
  const int r = lane & 31, h = lane >> 5;

  struct Slab {
    int f, m0, n0, ks, kc, kend;
    int last;                // 1: the last slab of its tile
  };
  auto slab_at = [&](unsigned i) {
    Slab S;
    unsigned t = first + i / unsigned(nkc);
    const int sl = int(i % unsigned(nkc));
    S.ks = int(t % unsigned(ksplit));
    t /= unsigned(ksplit);
    S.n0 = int(t % unsigned(ntn)) * TN;
    S.m0 = int((t / unsigned(ntn)) % unsigned(ntm)) * TM;
    S.f = int(t / unsigned(ntn * ntm));
    S.kc = S.ks * kchunk + sl * KA;
    S.kend = min(Kd, (S.ks + 1) * kchunk);
    S.last = sl == nkc - 1 ? 1 : 0;
    return S;
  };

  // B: lane (h, r) takes column n0 + 32*wn + r (clamped), rows kc + 8*(4*kh + j) + 4h + u of step j
  float2 braw[WSTEP][4];
  auto b_column = [&](const Slab& S) { return B + S.f * sB + min(S.n0 + 32 * wn + r, N - 1); };
  auto fetch_b = [&](const float2* bcol, unsigned pitch, int kc, int j) {
    const int k0 = kc + 8 * (WSTEP * kh + j) + 4 * h;
#pragma unroll
    for (int u = 0; u < 4; ++u) braw[j][u] = bcol[unsigned(min(k0 + u, Kd - 1)) * pitch];
  };

  // A slab -> LDS planes: thread (row tid / 16 + 16e, k-quad tid % 16): 16 lanes along k
  const int qa = tid & 15, ra = tid >> 4;
  float4 va[4][2];
  auto load_a = [&](const float2* abase, int m0, int kc) {
    const int k = min(kc + 4 * qa, Kd - 4);             // a quad inside the row (quads past Kd are zeroed at the split)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float2* src = abase + unsigned(min(m0 + ra + 16 * e, M - 1)) * unsigned(Kd) + k;
      va[e][0] = *reinterpret_cast<const float4*>(src);
      va[e][1] = *reinterpret_cast<const float4*>(src + 2);
    }
  };
  auto put_a = [&](int m0, int kc, int kend) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const bool okrow = m0 + ra + 16 * e < M;
      uint4 th, tm, tl;
      unsigned* ph = reinterpret_cast<unsigned*>(&th);
      unsigned* pm = reinterpret_cast<unsigned*>(&tm);
      unsigned* pl = reinterpret_cast<unsigned*>(&tl);
      const float2 x[4] = {make_float2(va[e][0].x, va[e][0].y), make_float2(va[e][0].z, va[e][0].w),
                           make_float2(va[e][1].x, va[e][1].y), make_float2(va[e][1].z, va[e][1].w)};
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const bool keep = okrow && kc + 4 * qa + u < kend;
        split_bf16x3(keep ? x[u] : make_float2(0.f, 0.f), ph[u], pm[u], pl[u]);
      }
      unsigned* d = la + (ra + 16 * e) * PITCH + 4 * qa;
      *reinterpret_cast<uint4*>(d) = th;
      *reinterpret_cast<uint4*>(d + Sh::PLANE) = tm;
      *reinterpret_cast<uint4*>(d + 2 * Sh::PLANE) = tl;
    }
  };

  hfloatx16 cre[2], cim[2];
  auto zero_acc = [&]() {
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
      for (int i = 0; i < 16; ++i) { cre[s][i] = 0.f; cim[s][i] = 0.f; }
  };
  const unsigned* fa = la + r * PITCH + 4 * h;
  float* red = reinterpret_cast<float*>(la) + (wn * 64) * 64 + lane;   // [wn][value 0..63][lane]

  Slab cur = slab_at(0);
  load_a(A + cur.f * sA, cur.m0, cur.kc);
  {
    const float2* bcol = b_column(cur);
#pragma unroll
    for (int j = 0; j < WSTEP; ++j) fetch_b(bcol, unsigned(N), cur.kc, j);
  }
  zero_acc();
  CIRC_PROBE(0);
  for (unsigned i = 0; i < nslabs; ++i) {
    const bool more = i + 1 < nslabs;
    Slab nxt = cur;
    if (more) nxt = slab_at(i + 1);
    const float2* bnext = more ? b_column(nxt) : B;
    const unsigned pnext = more ? unsigned(N) : 0u;
    __syncthreads();                                    // every wave has finished with the planes
    put_a(cur.m0, cur.kc, cur.kend);
    __syncthreads();
    // the next slab of A; behind the last slab the same one again (unconditional: see fetch_b of cgemm_split_kernel)
    load_a(A + nxt.f * sA, nxt.m0, nxt.kc);
    CIRC_PROBE(1 + 3 * i);
#pragma unroll
    for (int j = 0; j < WSTEP; ++j) {
      const int step = WSTEP * kh + j;                   // wave-uniform
      uint4 bt[3];
      {
        unsigned* ph = reinterpret_cast<unsigned*>(&bt[0]);
        unsigned* pm = reinterpret_cast<unsigned*>(&bt[1]);
        unsigned* pl = reinterpret_cast<unsigned*>(&bt[2]);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const bool keep = cur.kc + 8 * step + 4 * h + u < cur.kend;
          split_bf16x3(keep ? braw[j][u] : make_float2(0.f, 0.f), ph[u], pm[u], pl[u]);
        }
      }
      fetch_b(bnext, pnext, nxt.kc, j);                 // the registers are free again: next slab
      __builtin_amdgcn_sched_barrier(0);
      uint4 a[2][3], bre[3], bim[3];
#pragma unroll
      for (int term = 0; term < 3; ++term) {
        a[0][term] = *reinterpret_cast<const uint4*>(fa + term * Sh::PLANE + 8 * step);
        a[1][term] = *reinterpret_cast<const uint4*>(fa + term * Sh::PLANE + 32 * PITCH + 8 * step);
        const uint4 b = bt[term];
        // conj(B): re form (br, bi), im form (-bi, br)
        bre[term] = b;
        bim[term] = make_uint4(__builtin_amdgcn_alignbit(b.x, b.x, 16) ^ 0x8000u, __builtin_amdgcn_alignbit(b.y, b.y, 16) ^ 0x8000u,
                               __builtin_amdgcn_alignbit(b.z, b.z, 16) ^ 0x8000u, __builtin_amdgcn_alignbit(b.w, b.w, 16) ^ 0x8000u);
      }
      constexpr int TA[6] = {1, 2, 0, 1, 0, 0}, TB[6] = {1, 0, 2, 0, 1, 0};
#pragma unroll
      for (int pp = 0; pp < 6; ++pp) {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
          cre[s] = mfma16<true>(a[s][TA[pp]], bre[TB[pp]], cre[s]);
          cim[s] = mfma16<true>(a[s][TA[pp]], bim[TB[pp]], cim[s]);
        }
      }
    }
    CIRC_PROBE(2 + 3 * i);
    if (cur.last) {
      // the two halves of the reduction: waves 2, 3 hand their sums to waves 0, 1 through LDS
      __syncthreads();                                  // the planes are free
      if (kh == 1) {
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
          for (int q = 0; q < 16; ++q) {
            red[(32 * s + q) * 64] = cre[s][q];
            red[(32 * s + 16 + q) * 64] = cim[s][q];
          }
      }
      __syncthreads();
      const int col = cur.n0 + 32 * wn + r;
      if (kh == 0 && col < N) {
        float2* c = C + cur.ks * part_stride + cur.f * sC + col;
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
          for (int q = 0; q < 16; ++q) {
            const int row = cur.m0 + 32 * s + 8 * (q / 4) + 4 * h + (q % 4);
            if (row < M)
              c[unsigned(row) * unsigned(N)] = make_float2(cre[s][q] + red[(32 * s + q) * 64], cim[s][q] + red[(32 * s + 16 + q) * 64]);
          }
      }
      zero_acc();
    }
    CIRC_PROBE(3 + 3 * i);
    cur = nxt;
  }
}

}  // namespace circ
