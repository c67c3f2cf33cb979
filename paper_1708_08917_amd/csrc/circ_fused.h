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

#include <type_traits>

#include "circ_fft.h"
#include "circ_kernels.h"
#include "circ_probe.h"


namespace circ {

// K block size, IT output block rows per workgroup, NP packed batch pairs per workgroup,
// NT threads per workgroup (256 or 512).
template <int K, int IT, int NP, int NT>
struct FusedShape {
  static constexpr int NW = NT / 64;           // waves
  static constexpr int PT = 8 * NT / K;        // packed column pairs (complex FFTs) per chunk
  static constexpr int JC = PT / NP;           // input blocks j per chunk
  static constexpr int S = K / 2;              // complex slots per block
  static constexpr int FG = S / 16;            // slot groups (16 slots = one MFMA)
  static constexpr int IG = IT / 4;            // groups of 4 output block rows
  static constexpr int NCOMBO = FG * IG;       // (slot group, row group) pairs to accumulate
  static constexpr int JS = NCOMBO >= NW ? 1 : NW / NCOMBO;   // waves sharing a combo split the j range
  static constexpr int CPW = NCOMBO >= NW ? NCOMBO / NW : 1;  // combos per wave
  static constexpr int JW = JC / JS;           // input blocks per wave and chunk
  static constexpr int PP = PT + 1;
  static constexpr int OPROW = 2 * K + 2;      // floats per operand row (4 per slot, +2 pad)
  static constexpr int PTI = IT * NP;          // columns of the inverse transform
  static constexpr int PPI = PTI + 1;
  static constexpr int TILE_ELEMS = K * (PP > PPI ? PP : PPI);
  static constexpr int RED_FLOATS = (JS - 1) * NCOMBO * NP * 8 * 64;
  static constexpr size_t LDS_BYTES = size_t(TILE_ELEMS) * sizeof(float2) + size_t(PT) * OPROW * sizeof(float) +
                                      size_t(K) * sizeof(float2) + size_t(RED_FLOATS) * sizeof(float);
  static_assert(K >= 32 && PT >= 1 && JC >= 1 && JC * NP == PT, "bad chunk shape");
  static_assert(IT % 4 == 0 && (NCOMBO % NW == 0 || NW % NCOMBO == 0), "combos must split over the waves");
  static_assert(JW >= 2 && JW % 2 == 0 && JW * JS == JC, "each wave needs an even number of input blocks");
  static_assert((PTI & (PTI - 1)) == 0 && PTI <= NT, "inverse columns must be a power of two");
  static_assert(2 * PT * (K / 4) == 4 * NT, "x staging assumes 4 float4 per thread");
};

// Weight spectra in the operand order of the fused kernel, two input blocks per element:
//   Wf[((ig*q2p + j2)*FG + fg)*64 + 4*blk + m] = (W^[i][2*j2][slot], W^[i][2*j2+1][slot]),
//   i = 4*ig + m, slot = 16*fg + blk
// slot 0 = (W^[0].re, W^[K/2].re).  The section is padded with zeros to whole tiles:
// igp groups of 4 block rows (p rounded up to the kernel's IT), q2p pairs of block columns
// (q rounded up to the kernel's chunk).  `spec` is the [f][j][i] section.
// Element idx of the section (one call per element; see pack_sections_kernel).
__device__ __forceinline__ void pack_fused_elem(long long idx, const float2* __restrict__ spec, float4* __restrict__ Wf,
                                                int p, int q, int K, int igp, int q2p) {
  const int FG = K / 32;
  const long long total = (long long)igp * q2p * FG * 64;
  if (idx >= total) return;
  const int l = int(idx & 63);
  long long r = idx >> 6;
  const int fg = int(r % FG); r /= FG;
  const int j2 = int(r % q2p);
  const int ig = int(r / q2p);
  const int i = 4 * ig + (l & 3), slot = 16 * fg + (l >> 2);
  const long long fs = (long long)p * q;
  float2 v[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int j = 2 * j2 + h;
    v[h] = make_float2(0.f, 0.f);
    if (i < p && j < q) {
      if (slot == 0) v[h] = make_float2(spec[(long long)j * p + i].x, spec[(K / 2) * fs + (long long)j * p + i].x);
      else v[h] = spec[slot * fs + (long long)j * p + i];
    }
  }
  Wf[idx] = make_float4(v[0].x, v[0].y, v[1].x, v[1].y);
}

// The same operand order for 16-bit storage: element idx = two 32-bit words, each the (re, im)
// 16-bit pair of one input block; `spec` is the 16-bit section [f][i][j] (one word per value, not
// normalised), so packing only moves bits and works for fp16 and bfloat16 alike.
__device__ __forceinline__ void pack_fused_half_elem(long long idx, const unsigned* __restrict__ spec, uint2* __restrict__ Wf,
                                                     int p, int q, int K, int igp, int q2p) {
  const int FG = K / 32;
  const long long total = (long long)igp * q2p * FG * 64;
  if (idx >= total) return;
  const int l = int(idx & 63);
  long long r = idx >> 6;
  const int fg = int(r % FG); r /= FG;
  const int j2 = int(r % q2p);
  const int ig = int(r / q2p);
  const int i = 4 * ig + (l & 3), slot = 16 * fg + (l >> 2);
  const long long fs = (long long)p * q;
  unsigned v[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int j = 2 * j2 + h;
    v[h] = 0u;
    if (i < p && j < q) {
      const long long e = (long long)i * q + j;
      if (slot == 0) v[h] = (spec[e] & 0xffffu) | (spec[(K / 2) * fs + e] << 16);   // the two real bins
      else v[h] = spec[slot * fs + e];
    }
  }
  Wf[idx] = make_uint2(v[0], v[1]);
}
__global__ __launch_bounds__(256) void pack_fused_half_kernel(const unsigned* __restrict__ spec, uint2* __restrict__ Wf, int p,
                                                              int q, int K, int igp, int q2p) {
  pack_fused_half_elem((long long)blockIdx.x * 256 + threadIdx.x, spec, Wf, p, q, K, igp, q2p);
}

// Exchange each lane's value with its neighbour inside a quad: lanes (0,1) and (2,3) swap.
__device__ __forceinline__ float quad_swap_pairs(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1 /* quad_perm [1,0,3,2] */, 0xF, 0xF, false));
}

// ONE: all q input blocks fit one chunk, so the second (prefetch) set of weight operands is
// never needed.  With 512 threads that variant is held to 128 registers per lane: two
// workgroups then fit one CU (registers and LDS), and a launch on another stream can start on
// a CU while the previous one is still waiting for its operands or draining.  Kernels of
// independent batches overlap that way; a single launch is not slowed down.
// HM: 0 = fp32 operands; 1 (fp16) / 2 (bfloat16) = 16-bit storage: Wf then points to the packed
// 16-bit operands (pack_fused_half_elem: 8 bytes per element, not normalised), x and y to 16-bit
// values; everything between the loads and the final store is the same fp32 arithmetic, and the
// 1/k of the inverse transform is applied to the fp32 result.
template <int K, int IT, int NP, int NT, bool ONE = false, int HM = 0>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(ONE && NT == 512 ? 4 : 1, ONE && NT == 512 ? 4 : 8)))
void fc_fused_kernel(const float4* __restrict__ Wf, const float* __restrict__ x,
                                                      const float* __restrict__ bias, float* __restrict__ y,
                                                      int p, int q, int B, int n_it, int q2p, int xa, int relu) {
  constexpr bool BF = HM == 2;
  using AOp = typename std::conditional<HM != 0, uint2, float4>::type;   // weight operand of two input blocks
  using Sh = FusedShape<K, IT, NP, NT>;
  constexpr int PT = Sh::PT, JC = Sh::JC, S = Sh::S, FG = Sh::FG, IG = Sh::IG, CPW = Sh::CPW, JS = Sh::JS;
  constexpr int JW = Sh::JW, NW = Sh::NW, NCOMBO = Sh::NCOMBO;
  constexpr int PP = Sh::PP, OPROW = Sh::OPROW, PTI = Sh::PTI, PPI = Sh::PPI;
  constexpr int NFW = CPW > IG ? CPW / IG : 1;       // distinct slot groups per wave
  constexpr int JB = JW < 8 ? JW : 8;                // operand rows fetched from LDS per batch
  constexpr int NOUT4 = 2 * PTI * K / 4;             // float4 outputs of the tile
  constexpr int NV = (NOUT4 + NT - 1) / NT;          // ... per thread
  static_assert(JW % JB == 0, "batching of operand rows");
  extern __shared__ float smem[];
  float2* z = reinterpret_cast<float2*>(smem);
  float* op = smem + 2 * Sh::TILE_ELEMS;
  float2* twl = reinterpret_cast<float2*>(op + PT * OPROW);
  float* red = reinterpret_cast<float*>(twl + K);

  // the wave index is made explicitly wave-uniform, so that everything derived from it
  // (combo, slot group, operand addresses) lives in scalar registers and branches on it are scalar
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // Workgroups go round-robin to the 8 XCDs, each with its own L2 (not kept across
  // launches).  The tile grid (n_it x n_bt) is cut into xa x (8/xa) rectangles, one per XCD,
  // so that the weight tiles and x rows an XCD has to pull into its L2 are as few as possible.
  const int n_bt = (B + 2 * NP - 1) / (2 * NP);
  const int xb = 8 / xa, xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
  const int ni = (n_it + xa - 1) / xa, nb = (n_bt + xb - 1) / xb;
  const int it = (xcd % xa) * ni + local % ni, bt = (xcd / xa) * nb + local / ni;
  if (local >= ni * nb || it >= n_it || bt >= n_bt) return;
  const int i0 = it * IT, b0 = bt * 2 * NP;
  const long long ldx = (long long)q * K, ldy = (long long)p * K;
  const int nchunks = (q + JC - 1) / JC;
  // this wave's share of the contraction: CPW combos starting at combo0, input blocks
  // [js*JW, (js+1)*JW) of every chunk
  const int combo0 = (wave % (NW / JS)) * CPW, js = wave / (NW / JS);

  // NCH independent accumulation chains per result (consecutive input blocks alternate between
  // them), so that a matrix instruction never waits for the previous one on the same registers
  constexpr int NCH = (CPW * NP >= 2) ? 2 : 4;
  floatx4 P[NCH][CPW][NP], Q[NCH][CPW][NP];
#pragma unroll
  for (int h = 0; h < NCH; ++h)
#pragma unroll
    for (int cc = 0; cc < CPW; ++cc)
#pragma unroll
      for (int u = 0; u < NP; ++u) {
        P[h][cc][u] = floatx4{0.f, 0.f, 0.f, 0.f};
        Q[h][cc][u] = floatx4{0.f, 0.f, 0.f, 0.f};
      }

  // --- global loads: 4 float4 of x per thread and JW/2 weight operands per combo, per chunk.
  // Addresses are a wave-uniform base plus a 32-bit per-lane offset fixed for the whole
  // kernel, so that issuing a load costs no vector arithmetic.
  // Rows past the batch and input blocks past q are clamped to the last valid one instead of
  // being skipped (their products meet zero weights or are never stored), so that the loads
  // are unconditional and the number of loads in flight is known at compile time.
  float4 xr[4];
  unsigned xoff[4];
  int xjj[4];
  // A wave-load covers 8 rows x 8 float4 (128 contiguous bytes of each row): with the lanes of a
  // wave spread over rows as well as over n, the four LDS stores per float4 spread over all banks
  // (lanes that only differ in n are 8*PP floats apart, which is 8 banks modulo 32).
  constexpr int RB = 2 * PT / 8;                 // blocks of 8 rows per chunk
  auto x_elem = [&](int e, int& row, int& n4) {
    const int blk = e * NW + wave;               // NT/16 blocks of 8 x 8 float4, four per wave
    row = 8 * (blk % RB) + (lane >> 3);
    n4 = 8 * (blk / RB) + (lane & 7);
  };
  static_assert((2 * PT) % 8 == 0 && (K / 4) % 8 == 0 && RB * (K / 32) == NT / 16, "x staging blocks");
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    int row, n4;
    x_elem(e, row, n4);
    const int cl = row >> 1, half = row & 1;
    const int jj = cl / NP, brow = min(2 * (cl % NP) + half, B - 1 - b0);
    xjj[e] = jj;
    xoff[e] = unsigned(brow) * unsigned(ldx) + unsigned(4 * n4);
  }
  const float* xtile = x + (long long)b0 * ldx;
  const unsigned short* xtile16 = reinterpret_cast<const unsigned short*>(x) + (long long)b0 * ldx;
  auto load_x = [&](int c) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const unsigned j = unsigned(min(c * JC + xjj[e], q - 1));
      if constexpr (HM == 0) xr[e] = *reinterpret_cast<const float4*>(xtile + (xoff[e] + j * unsigned(K)));
      else xr[e] = load_half4<BF>(xtile16 + (xoff[e] + j * unsigned(K)));
    }
  };
  auto store_x = [&]() {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      int row, n4;
      x_elem(e, row, n4);
      const int n = 4 * n4, cl = row >> 1, half = row & 1;
      lds_put(z, (n + 0) * PP + cl, half, xr[e].x);
      lds_put(z, (n + 1) * PP + cl, half, xr[e].y);
      lds_put(z, (n + 2) * PP + cl, half, xr[e].z);
      lds_put(z, (n + 3) * PP + cl, half, xr[e].w);
    }
  };
  // weight operands: the packed section is zero-padded to whole tiles (q2p pairs of block
  // columns per row group), so no clamping is needed
  const AOp* wtile = reinterpret_cast<const AOp*>(Wf) + ((long long)it * IG * q2p + js * (JW / 2)) * FG * 64;
  unsigned aoff[CPW];
#pragma unroll
  for (int cc = 0; cc < CPW; ++cc) {
    const int combo = combo0 + cc;
    aoff[cc] = unsigned(((combo % IG) * q2p) * FG + combo / IG) * 64u + unsigned(lane);
  }
  AOp a_even[CPW][JW / 2], a_odd[ONE ? 1 : CPW][ONE ? 1 : JW / 2];
  // [lo, hi) selects a part of the chunk's operands: a workgroup can only push requests into
  // the memory pipeline at a bounded rate, so the loads of the next chunk are issued in
  // pieces between the phases of the current one instead of stalling one phase
  auto load_a = [&](int c, AOp (&a)[CPW][JW / 2], int lo, int hi) {
    const AOp* wc = wtile + (long long)c * (JC / 2) * FG * 64;
#pragma unroll
    for (int jh = 0; jh < JW / 2; ++jh)
#pragma unroll
      for (int cc = 0; cc < CPW; ++cc)
        if (jh >= lo && jh < hi) a[cc][jh] = wc[(long long)jh * FG * 64 + aoff[cc]];
  };
  constexpr int AH = JW / 2, AH1 = (AH + 2) / 3, AH2 = (2 * AH + 2) / 3;

  CIRC_PROBE(0);
  // memory returns loads in issue order: the twiddles go first because they are needed first,
  // so that waiting for them does not also wait for the weight operands
  float2 tw_stage[(K + NT - 1) / NT];
#pragma unroll
  for (int s = 0; s < (K + NT - 1) / NT; ++s) {
    const int m = min(s * NT + tid, K - 1);
    tw_stage[s] = make_float2(kTw.c[m * (kTwN / K)], kTw.s[m * (kTwN / K)]);
  }
  load_x(0);
  load_a(0, a_even, 0, AH);
#pragma unroll
  for (int s = 0; s < (K + NT - 1) / NT; ++s)
    if (s * NT + tid < K) twl[s * NT + tid] = tw_stage[s];

  // bias of the outputs this thread will store (fetched now, used at the very end)
  float4 bv4[NV];
#pragma unroll
  for (int s = 0; s < NV; ++s) {
    const int idx = s * NT + tid;
    const int row = idx / (K / 4), n = 4 * (idx % (K / 4));
    const int i = i0 + (row >> 1) / NP;
    bv4[s] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (bias && idx < NOUT4 && i < p) bv4[s] = *reinterpret_cast<const float4*>(bias + (long long)i * K + n);
  }

  const int col = tid % PT, t = tid / PT;
  constexpr int TT = NT / PT;

  // one chunk of JC input blocks: FFT of its 2*PT rows, then the contraction with `a_use`;
  // meanwhile the loads of the next chunk (x into xr, weights into `a_pref`) are in flight.
  // `more` (a compile-time tag): another chunk follows, so its loads are issued here.
  auto chunk = [&](int c, AOp (&a_use)[CPW][JW / 2], AOp (&a_pref)[CPW][JW / 2], auto more_tag) {
    constexpr bool more = decltype(more_tag)::value;
    store_x();
    __syncthreads();
    CIRC_PROBE(1 + 4 * c);
    if constexpr (more) {
      load_x(c + 1);
      load_a(c + 1, a_pref, 0, AH1);
    }
    fft_lds_pass1<K, false>(z, PP, col, t, TT, twl);
    __syncthreads();
    CIRC_PROBE(2 + 4 * c);
    if constexpr (more) load_a(c + 1, a_pref, AH1, AH2);
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
    CIRC_PROBE(3 + 4 * c);
    if constexpr (more) load_a(c + 1, a_pref, AH2, AH);
    // operand rows come from LDS one batch ahead of the matrix instructions that use them
    const float* opw = op + (js * JW * NP) * OPROW + lane;
    float bvv[2][JB][NP][NFW];
    auto fetch_b = [&](int jb, float (&dst)[JB][NP][NFW]) {
#pragma unroll
      for (int jj = 0; jj < JB; ++jj)
#pragma unroll
        for (int u = 0; u < NP; ++u)
#pragma unroll
          for (int fw = 0; fw < NFW; ++fw) {
            const int fg = (combo0 + fw * IG) / IG;
            dst[jj][u][fw] = opw[((jb + jj) * NP + u) * OPROW + fg * 64];
          }
    };
    fetch_b(0, bvv[0]);
#pragma unroll
    for (int jb = 0; jb < JW; jb += JB) {
      const int cur = (jb / JB) & 1;
      if (jb + JB < JW) fetch_b(jb + JB, bvv[cur ^ 1]);
#pragma unroll
      for (int jj = 0; jj < JB; ++jj)
#pragma unroll
        for (int u = 0; u < NP; ++u)
#pragma unroll
          for (int cc = 0; cc < CPW; ++cc) {
            const float bval = bvv[cur][jj][u][NFW > 1 ? cc / IG : 0];
            const AOp av = a_use[cc][(jb + jj) / 2];
            float ar, ai;
            if constexpr (HM == 0) {
              ar = ((jb + jj) & 1) ? av.z : av.x;
              ai = ((jb + jj) & 1) ? av.w : av.y;
            } else {
              const float2 cv = unpack_pair16<BF>(((jb + jj) & 1) ? av.y : av.x);
              ar = cv.x;
              ai = cv.y;
            }
            P[jj % NCH][cc][u] = __builtin_amdgcn_mfma_f32_4x4x1f32(ar, bval, P[jj % NCH][cc][u], 0, 0, 0);
            Q[jj % NCH][cc][u] = __builtin_amdgcn_mfma_f32_4x4x1f32(ai, bval, Q[jj % NCH][cc][u], 0, 0, 0);
          }
    }
    CIRC_PROBE(4 + 4 * c);
  };
  // steady state without conditionals around the loads (the compiler then waits for exactly the
  // operands a phase needs, not for everything in flight); the last one or two chunks are peeled
  {
    constexpr std::true_type yes{};
    constexpr std::false_type no{};
    int c = 0;
    if constexpr (ONE) {
      chunk(0, a_even, a_even, no);
    } else {
    for (; c + 2 < nchunks; c += 2) {
      chunk(c, a_even, a_odd, yes);
      chunk(c + 1, a_odd, a_even, yes);
    }
    if (c + 2 == nchunks) {
      chunk(c, a_even, a_odd, yes);
      chunk(c + 1, a_odd, a_even, no);
    } else {
      chunk(c, a_even, a_odd, no);
    }
    }
  }

  // --- sum the accumulation chains of this wave, in a fixed order
#pragma unroll
  for (int cc = 0; cc < CPW; ++cc)
#pragma unroll
    for (int u = 0; u < NP; ++u) {
      if constexpr (NCH == 4) {
        P[0][cc][u] = (P[0][cc][u] + P[1][cc][u]) + (P[2][cc][u] + P[3][cc][u]);
        Q[0][cc][u] = (Q[0][cc][u] + Q[1][cc][u]) + (Q[2][cc][u] + Q[3][cc][u]);
      } else {
        P[0][cc][u] += P[1][cc][u];
        Q[0][cc][u] += Q[1][cc][u];
      }
    }
  // Waves that split the j range (JS = 2) each assemble the output spectra of their share: the
  // first into the inverse tile, the second into a twin of it in `red`; the first pass of the
  // inverse transform adds the twin as it reads (first + second: a fixed order), which saves a
  // round trip through LDS and a barrier over summing the accumulators first.
  static_assert(JS <= 2 && (JS == 1 || K == 64), "the twin tile is added by the k = 64 inverse transform only");
  static_assert(JS == 1 || Sh::RED_FLOATS >= 2 * K * PPI, "the twin tile must fit the reduction buffer");
  // --- assemble Zy of every (output block row, batch pair) into the inverse tile
  {
    const int n = lane & 3, blk = lane >> 2;
#pragma unroll
    for (int cc = 0; cc < CPW; ++cc) {
      const int combo = combo0 + cc;
      const int fg = combo / IG, ig = combo % IG;
      const int slot = 16 * fg + blk;
      const int fidx = (n < 2) ? slot : (slot == 0 ? S : K - slot);
      // value = ca*P + cb*Q + cc*swap(Q) with per-lane constants (no divergent branches):
      // slot 0: (P, P, Q, Q) by column; other slots: (P - Qs, P + Qs, P + Qs, P - Qs)
      const float ca = (slot == 0 && n >= 2) ? 0.f : 1.f;
      const float cb = (slot == 0 && n >= 2) ? 1.f : 0.f;
      const float cs = slot == 0 ? 0.f : ((n == 0 || n == 3) ? -1.f : 1.f);
      float* zl = (js == 0 ? reinterpret_cast<float*>(z) : red) + 2 * (fidx * PPI + 4 * ig * NP) + (n & 1);
#pragma unroll
      for (int u = 0; u < NP; ++u) {
#pragma unroll
        for (int m = 0; m < 4; ++m) {
          const float pv = P[0][cc][u][m], qv = Q[0][cc][u][m];
          const float qs = quad_swap_pairs(qv);
          zl[2 * (m * NP + u)] = fmaf(cs, qs, fmaf(cb, qv, ca * pv));
        }
      }
    }
  }
  __syncthreads();
  CIRC_PROBE(60);
  if constexpr (K == 64) {
    // few columns (IT*NP), 8 x 8 points each: every 8-point sub-transform runs on 8 lanes
    // (Fft8Lanes), so that all waves take part and the dependent chain per pass is short
    const int m = tid & 7, fo = bitrev3(m);
    const Fft8Lanes<true> F(m);
    for (int task = tid >> 3; task < PTI * 8; task += NT / 8) {      // pass 1: (column, n2), lane = n1
      const int n2 = task & 7, coli = task >> 3;
      float2 v = z[(8 * m + n2) * PPI + coli];
      if constexpr (JS > 1) {                                        // the second wave's share of the j range
        const float2 v2 = reinterpret_cast<const float2*>(red)[(8 * m + n2) * PPI + coli];
        v.x += v2.x;
        v.y += v2.y;
      }
      const float2 w = twl[fo * n2];                                 // twiddle of output f1 = fo
      F.run(v.x, v.y);
      z[(8 * fo + n2) * PPI + coli] = make_float2(w.x * v.x - w.y * v.y, w.x * v.y + w.y * v.x);
    }
    __syncthreads();
    for (int task = tid >> 3; task < PTI * 8; task += NT / 8) {      // pass 2: (column, f1), lane = n2
      const int f1 = task & 7, coli = task >> 3;
      float2 v = z[(8 * f1 + m) * PPI + coli];
      F.run(v.x, v.y);
      z[(8 * f1 + fo) * PPI + coli] = v;                             // index f1 + 8*f2 at fft_pos = 8*f1 + f2
    }
    __syncthreads();
  } else {
    const int coli = tid % PTI, ti = tid / PTI;
    constexpr int TTI = NT / PTI;
    fft_lds_pass1<K, true>(z, PPI, coli, ti, TTI, twl);
    __syncthreads();
    fft_lds_pass2_inplace<K, true>(z, PPI, coli, ti, TTI);
    __syncthreads();
  }
  CIRC_PROBE(61);
#pragma unroll
  for (int s = 0; s < NV; ++s) {
    const int idx = s * NT + tid;
    const int row = idx / (K / 4), n = 4 * (idx % (K / 4));
    const int coli = row >> 1, half = row & 1;
    const int i = i0 + coli / NP, b = b0 + 2 * (coli % NP) + half;
    if (idx < NOUT4 && i < p && b < B) {
      constexpr float osc = HM == 0 ? 1.0f : 1.0f / float(K);   // fp32 operands carry the 1/k already
      float4 v;
      v.x = lds_get(z, fft_pos<K>(n + 0) * PPI + coli, half) * osc + bv4[s].x;
      v.y = lds_get(z, fft_pos<K>(n + 1) * PPI + coli, half) * osc + bv4[s].y;
      v.z = lds_get(z, fft_pos<K>(n + 2) * PPI + coli, half) * osc + bv4[s].z;
      v.w = lds_get(z, fft_pos<K>(n + 3) * PPI + coli, half) * osc + bv4[s].w;
      if (relu) { v.x = fmaxf(v.x, 0.f); v.y = fmaxf(v.y, 0.f); v.z = fmaxf(v.z, 0.f); v.w = fmaxf(v.w, 0.f); }
      const long long yo = (long long)b * ldy + (long long)i * K + n;
      if constexpr (HM == 0) *reinterpret_cast<float4*>(y + yo) = v;
      else store_half4<BF>(reinterpret_cast<unsigned short*>(y) + yo, v);
    }
  }
  CIRC_PROBE(62);
}

}  // namespace circ
