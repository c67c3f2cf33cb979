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

// Workgroup -> tile map of the fused kernel.  Workgroups go round-robin to the 8 XCDs, each
// with its own L2 (not kept across launches).  The tile grid (n_it tiles of output block rows x
// n_bt tiles of batch rows) is cut into 2^xa_shift x 2^(3 - xa_shift) rectangles of ni x nb
// tiles, one per XCD, chosen on the host so that the weight tiles and x rows an XCD has to pull
// into its L2 are as few as possible.  Everything the kernel needs to find its tile is worked
// out here, so that no integer division stands between the start of a workgroup and its first
// loads: local / ni is a multiply-high by ni_magic = ceil(2^32 / ni) (exact while
// local * ni < 2^32; ni = 1 is handled apart).
struct FusedTileMap {
  int n_it, n_bt, ni, nb, xa_shift;
  unsigned ni_magic;
  unsigned grid;       // workgroups to launch
};
inline FusedTileMap make_fused_tile_map(int p, int q, int K, int IT, int NP, int batch) {
  FusedTileMap m;
  m.n_it = (p + IT - 1) / IT;
  m.n_bt = (batch + 2 * NP - 1) / (2 * NP);
  int xa = 1;
  double best = 1e300;
  for (int cand = 1, sh = 0; cand <= 8; cand *= 2, ++sh) {
    const double wbytes = double((m.n_it + cand - 1) / cand) * IT * q * K * 4.0;
    const double xbytes = double((m.n_bt + 8 / cand - 1) / (8 / cand)) * 2 * NP * q * K * 4.0;
    if (wbytes + xbytes < best) { best = wbytes + xbytes; xa = cand; m.xa_shift = sh; }
  }
  m.ni = (m.n_it + xa - 1) / xa;
  m.nb = (m.n_bt + 8 / xa - 1) / (8 / xa);
  m.ni_magic = m.ni > 1 ? unsigned(((1ull << 32) + unsigned(m.ni) - 1) / unsigned(m.ni)) : 0u;
  m.grid = 8u * unsigned(m.ni) * unsigned(m.nb);
  return m;
}

// K block size, IT output block rows per workgroup, NP packed batch pairs per workgroup,
// NT threads per workgroup (256 or 512).
template <int K, int IT, int NP, int NT>
struct FusedShape {
  static constexpr int NW = NT / 64;           // waves
  static constexpr int R1 = radix1_of(K), R2 = radix2_of(K);   // K = R1 * R2, R1 <= R2 <= 16
  static constexpr int LC = R2;                // lanes that share a column of the forward transform
  static constexpr int PT = 8 * NT / K;        // packed column pairs (complex FFTs) per chunk
  static constexpr int CPR = NT / LC;          // columns the workgroup transforms at a time
  static constexpr int NR = PT >= CPR ? PT / CPR : 1;   // rounds of the forward transform per chunk
  static constexpr int JC = PT / NP;           // input blocks j per chunk
  static constexpr int S = K / 2;              // complex slots per block
  static constexpr int FG = S / 16;            // slot groups (16 slots = one MFMA)
  static constexpr int IG = IT / 4;            // groups of 4 output block rows
  static constexpr int NCOMBO = FG * IG;       // (slot group, row group) pairs to accumulate
  static constexpr int JS = NCOMBO >= NW ? 1 : NW / NCOMBO;   // waves sharing a combo split the j range
  static constexpr int CPW = NCOMBO >= NW ? NCOMBO / NW : 1;  // combos per wave
  static constexpr int JW = JC / JS;           // input blocks per wave and chunk
  // A column's LDS region serves twice: first the exchange between the two passes of its
  // transform, [f1][n2] with rows of R2 + 1 complex values, then its operand row (4 floats per
  // slot).  XCS: complex values of the exchange layout; OPROW: floats per region.
  static constexpr int XCS = R1 * (R2 + 1) + 1;
  static constexpr int OPROW = 2 * XCS > 2 * K + 2 ? 2 * XCS : 2 * K + 2;
  static constexpr int PTI = IT * NP;          // columns of the inverse transform
  static constexpr int PPI = PTI + 1;
  static constexpr int OP_FLOATS = PT * OPROW;               // one set of operand rows
  static constexpr int ZI_FLOATS = 2 * K * PPI;              // one tile of output spectra
  static_assert(K >= 32 && PT >= 1 && JC >= 1 && JC * NP == PT, "bad chunk shape");
  static_assert(IT % 4 == 0 && (NCOMBO % NW == 0 || NW % NCOMBO == 0), "combos must split over the waves");
  static_assert(JW >= 2 && JW % 2 == 0 && JW * JS == JC, "each wave needs an even number of input blocks");
  static_assert(JS == 1 || K == 64, "only the k = 64 inverse transform adds partial tiles");
  static_assert(LC <= 64 && 64 % LC == 0, "the lanes of a column lie in one wave");
  static_assert(NR * CPR == PT || (NR == 1 && PT < CPR), "rounds of the forward transform");
  static_assert((PTI & (PTI - 1)) == 0 && PTI <= NT, "inverse columns must be a power of two");
  static_assert(K != 64 || (PTI * 64) % NT == 0, "k = 64: one wave per column of the inverse transform");
  // LDS: operand rows (two sets when the input blocks take several chunks, so that one barrier
  // per chunk suffices), JS tiles of output spectra (one per share of the j range), the K roots
  static constexpr size_t lds_bytes(bool one) {
    return (size_t(one ? 1 : 2) * OP_FLOATS + size_t(JS) * ZI_FLOATS + 2 * K) * sizeof(float);
  }
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

// W_R2^f = e^{-2 pi i f / R2}, f < R2/2, as (cos, -sin) on the odd lane of a pair and (1, 0) on the even one.
template <int R2, int F = 1>
__device__ __forceinline__ void pair_twiddles(float (&c)[R2 / 2], float (&s)[R2 / 2], int odd) {
  if constexpr (F == 1) { c[0] = 1.f; s[0] = 0.f; }
  if constexpr (F < R2 / 2) {
    c[F] = odd ? tw_cos(F, R2) : 1.f;
    s[F] = odd ? -tw_sin(F, R2) : 0.f;
    pair_twiddles<R2, F + 1>(c, s, odd);
  }
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
//
// Phases of a workgroup (two barriers when all input blocks fit one chunk):
//   x (global, strided 4-byte loads straight into the order of the first pass) -> first pass in
//   registers -> exchange through the column's own LDS region, inside one wave (no barrier) ->
//   second pass in registers -> operand rows in LDS | barrier | contraction on the matrix cores,
//   weight operands in registers | assembly of the output spectra into LDS | barrier | inverse
//   transform (k = 64: one wave per column on the lane network, stores from registers) -> bias,
//   ReLU -> y.
template <int K, int IT, int NP, int NT, bool ONE = false, int HM = 0>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(ONE && NT == 512 ? 4 : 1, ONE && NT == 512 ? 4 : 8)))
void fc_fused_kernel(const float4* __restrict__ Wf, const float* __restrict__ x,
                                                      const float* __restrict__ bias, float* __restrict__ y,
                                                      int p, int q, int B, FusedTileMap tm, int q2p, int relu) {
  constexpr bool BF = HM == 2;
  using AOp = typename std::conditional<HM != 0, uint2, float4>::type;   // weight operand of two input blocks
  using Sh = FusedShape<K, IT, NP, NT>;
  constexpr int PT = Sh::PT, JC = Sh::JC, S = Sh::S, FG = Sh::FG, IG = Sh::IG, CPW = Sh::CPW, JS = Sh::JS;
  constexpr int JW = Sh::JW, NW = Sh::NW, R1 = Sh::R1, R2 = Sh::R2, LC = Sh::LC, CPR = Sh::CPR, NR = Sh::NR;
  constexpr int OPROW = Sh::OPROW, PTI = Sh::PTI, PPI = Sh::PPI;
  constexpr int NFW = CPW > IG ? CPW / IG : 1;       // distinct slot groups per wave
  constexpr int JB = JW < 8 ? JW : 8;                // operand rows fetched from LDS per batch
  static_assert(JW % JB == 0, "batching of operand rows");
  extern __shared__ float smem[];
  float* op0 = smem;                                                   // operand rows, set 0 (and 1)
  float* zi = smem + (ONE ? 1 : 2) * Sh::OP_FLOATS;                    // JS tiles of output spectra
  float2* twl = reinterpret_cast<float2*>(zi + JS * Sh::ZI_FLOATS);    // K roots, for the inverse transform

  // the wave index is made explicitly wave-uniform, so that everything derived from it
  // (combo, slot group, operand addresses) lives in scalar registers and branches on it are scalar
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // this workgroup's tile (see FusedTileMap)
  const unsigned xcd = blockIdx.x & 7u, local = blockIdx.x >> 3;
  const unsigned lq = tm.ni > 1 ? __umulhi(local, tm.ni_magic) : local;            // local / ni
  const int it = int(xcd & ((1u << tm.xa_shift) - 1u)) * tm.ni + int(local - lq * unsigned(tm.ni));
  const int bt = int(xcd >> tm.xa_shift) * tm.nb + int(lq);
  if (int(lq) >= tm.nb || it >= tm.n_it || bt >= tm.n_bt) return;
  const int i0 = it * IT, b0 = bt * 2 * NP;
  const long long ldx = (long long)q * K, ldy = (long long)p * K;
  const int nchunks = (q + JC - 1) / JC;
  // this wave's share of the contraction: CPW combos starting at combo0, input blocks
  // [js*JW, (js+1)*JW) of every chunk
  const int combo0 = (wave % (NW / JS)) * CPW, js = wave / (NW / JS);

  // NCH independent accumulation chains per result (consecutive input blocks alternate between
  // them), so that a matrix instruction never waits for the previous one on the same registers
  constexpr int NCH = (CPW * NP >= 4) ? 1 : ((CPW * NP >= 2) ? 2 : 4);
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

  // --- global loads.  x: the LC lanes of a column read the K values of its two batch rows in the
  // order of the first pass, lane n2 taking x[R2*n1 + n2], n1 < R1, so that the values go from
  // the load straight into the first butterflies (4-byte loads; a wave-load covers LC
  // consecutive values of each of its 64 / LC columns).  NR columns per thread and chunk.
  // Addresses are a wave-uniform base plus a 32-bit per-lane offset fixed for the whole
  // kernel, so that issuing a load costs no vector arithmetic.
  // Rows past the batch and input blocks past q are clamped to the last valid one instead of
  // being skipped (their products meet zero weights or are never stored), so that the loads
  // are unconditional and the number of loads in flight is known at compile time.
  const int fn2 = tid % LC, fc = tid / LC;           // lane of the column, column of the round
  const bool fwd_active = PT >= CPR || fc < PT;      // (fewer columns than the workgroup could take: K = 256)
  float xr[NR][2][R1];
  unsigned xoff[NR][2];
  int xjj[NR];
#pragma unroll
  for (int rd = 0; rd < NR; ++rd) {
    const int cl = min(rd * CPR + fc, PT - 1);
    xjj[rd] = cl / NP;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int brow = min(2 * (cl % NP) + h, B - 1 - b0);
      xoff[rd][h] = unsigned(brow) * unsigned(ldx) + unsigned(fn2);
    }
  }
  const float* xtile = x + (long long)b0 * ldx;
  const unsigned short* xtile16 = reinterpret_cast<const unsigned short*>(x) + (long long)b0 * ldx;
  auto load_x = [&](int c) {
#pragma unroll
    for (int rd = 0; rd < NR; ++rd) {
      const unsigned j = unsigned(min(c * JC + xjj[rd], q - 1));
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int n1 = 0; n1 < R1; ++n1) {
          const unsigned o = xoff[rd][h] + j * unsigned(K) + unsigned(R2 * n1);
          if constexpr (HM == 0) xr[rd][h][n1] = xtile[o];
          else if constexpr (BF) xr[rd][h][n1] = __uint_as_float(unsigned(xtile16[o]) << 16);
          else xr[rd][h][n1] = __half2float(__ushort_as_half(xtile16[o]));
        }
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
  constexpr int AH = JW / 2;
  // Where the weight operands of the next chunk are requested: in portions ahead of each batch of
  // matrix instructions (the requests queue while the matrix cores work), or, k = 128, all of
  // them behind the last matrix instruction.  Measured, warm, multi-chunk layers: k = 32 16.3 ->
  // 12.8 us (q = 300), k = 64 65.8 -> 58.7 us (q = 200, batch 512), k = 256 26.7 -> 25.6 us with
  // the first placement against half of the requests on either side of the barrier; k = 128
  // (9216 -> 4096, batch 256) 14.6 -> 15.1 us with the first, 13.8 us with the second.
  constexpr bool kWeightsLast = K == 128;
  // weight loads of the first chunk issued before x has arrived (see below); kernels that loop
  // over chunks keep a second set of operands in registers and issue all of the first set at once
  constexpr int AF0 = ONE ? (AH + 7) / 8 : AH;

  CIRC_PROBE(0);
  // memory returns loads in issue order: the twiddles go first because they are needed first,
  // so that waiting for them does not also wait for the weight operands
  // twiddles of the first pass for this lane, W_K^(f1*n2), straight from the table in the code object
  // k >= 128: x first (the twiddles, behind it, still precede every weight operand; 9216 -> 4096 at
  // k = 128 14.2 -> 13.5 us, k = 256 24.5 -> 24.3 us; at k = 64 the order above measured better)
  constexpr bool kXFirst = K >= 128;
  if constexpr (kXFirst) {
    load_x(0);
    __builtin_amdgcn_sched_barrier(0);
  }
  float2 ftw[R1];
#pragma unroll
  for (int f1 = 1; f1 < R1; ++f1) ftw[f1] = reinterpret_cast<const float2*>(kTw.cs)[((f1 * fn2) % K) * (kTwN / K)];
  // second pass shared by lane pairs (R2 = 2*R1, see below): which half this lane takes, the sign of
  // its own value in the final butterfly, and its twiddles W_R2^f (1 on the even lane)
  // (k = 128: 14.6 -> 14.0 us for 9216 -> 4096 at batch 256; k = 32, 4-point halves: slower, not used)
  constexpr bool kPairPass2 = R2 == 2 * R1 && R2 >= 16;
  const int p2h = fn2 & 1;
  const float p2sgn = p2h ? -1.f : 1.f;
  float p2c[kPairPass2 ? R2 / 2 : 1], p2s[kPairPass2 ? R2 / 2 : 1];
  if constexpr (kPairPass2) pair_twiddles<R2>(p2c, p2s, p2h);
  float2 tw_stage[(K + NT - 1) / NT];
#pragma unroll
  for (int s = 0; s < (K + NT - 1) / NT; ++s) {
    const int m = min(s * NT + tid, K - 1);
    tw_stage[s] = reinterpret_cast<const float2*>(kTw.cs)[m * (kTwN / K)];
  }
  if constexpr (!kXFirst) load_x(0);
  // A CU serves the loads of its waves in the order they were issued.  The barrier (no wait on
  // any counter: nothing has to have arrived) puts the x loads of all waves ahead of every weight
  // operand load, so that the last wave's x is not queued behind the 16 KB of weights of each
  // wave before it: the transforms start when the 32 KB of x have arrived, and the weights, which
  // are not needed before the contraction, stream in meanwhile.
  __builtin_amdgcn_s_barrier();
  // When one chunk holds all input blocks, an eighth of its weights goes out now, while x is on its
  // way, and the rest is issued between the passes of the first transform.  A CU takes load instructions at a
  // bounded rate (one 16-byte load of a wave per 16 cycles): with all of them ahead of the
  // transform, its first instruction would wait for the last load to be accepted.
  load_a(0, a_even, 0, AF0);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int s = 0; s < (K + NT - 1) / NT; ++s)
    if (s * NT + tid < K) twl[s * NT + tid] = tw_stage[s];

  // bias of the outputs this thread will store (fetched now, used at the very end)
  constexpr int NOUT4 = 2 * PTI * K / 4;             // float4 outputs of the tile (k != 64)
  constexpr int NV = (NOUT4 + NT - 1) / NT;          // ... per thread
  constexpr int NI64 = K == 64 ? PTI * 64 / NT : 1;  // k = 64: columns per wave of the inverse transform
  float4 bv4[K == 64 ? 1 : NV];
  float bv1[NI64];
  // k = 64: lane l of a wave ends the inverse transform holding sample (l >> 3) + 8 * bitrev3(l & 7)
  const int n64 = (lane >> 3) + 8 * bitrev3(lane & 7);
  if constexpr (K == 64) {
#pragma unroll
    for (int t = 0; t < NI64; ++t) {
      const int i = i0 + (wave + t * NW) / NP;
      bv1[t] = (bias && i < p) ? bias[(long long)i * K + n64] : 0.f;
    }
  } else {
#pragma unroll
    for (int s = 0; s < NV; ++s) {
      const int idx = s * NT + tid;
      const int row = idx / (K / 4), n = 4 * (idx % (K / 4));
      const int i = i0 + (row >> 1) / NP;
      bv4[s] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (bias && idx < NOUT4 && i < p) bv4[s] = *reinterpret_cast<const float4*>(bias + (long long)i * K + n);
    }
  }

  // one chunk of JC input blocks: transform of its 2*PT rows, then the contraction with `a_use`;
  // meanwhile the loads of the next chunk (x into xr, weights into `a_pref`) are in flight.
  // `more` (a compile-time tag): another chunk follows, so its loads are issued here.
  // `first`: the first chunk, whose own weights are not all on their way yet.
  // `ragged`: the last chunk of a q that is not a multiple of the chunk; the transforms and the
  // batches of matrix instructions that lie entirely past the last input block are skipped (a
  // separate instance, so that the branches do not disturb the schedule of whole chunks:
  // 9216 -> 4096 at k = 128, q = 72 = 4.5 chunks, 14.5 -> 13.3 us)
  auto chunk = [&](int c, float* op, AOp (&a_use)[CPW][JW / 2], AOp (&a_pref)[CPW][JW / 2], auto more_tag, auto first_tag,
                   auto ragged_tag) {
    constexpr bool more = decltype(more_tag)::value, first = decltype(first_tag)::value;
    constexpr bool ragged = decltype(ragged_tag)::value;
    static_assert(!ragged || (!more && !first), "only the last of several chunks");
    // forward transform of this thread's columns; everything a column touches in LDS belongs to
    // the LC lanes of one wave, whose LDS accesses execute in program order: no barrier
    constexpr int AQ = first ? (AH - AF0 + 4) / 5 : 0;   // weight loads issued at each of the five points below
    auto more_weights = [&](int step) {
      if constexpr (first) {
        const int lo = AF0 + step * AQ < AH ? AF0 + step * AQ : AH, hi = lo + AQ < AH ? lo + AQ : AH;
        __builtin_amdgcn_sched_barrier(0);
        load_a(c, a_use, lo, step == 4 ? AH : hi);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
#pragma unroll
    for (int rd = 0; rd < NR; ++rd) {
      float* creg = op + (rd * CPR + (PT >= CPR ? fc : min(fc, PT - 1))) * OPROW;   // region of this lane's column
      float2* xch = reinterpret_cast<float2*>(creg);
      if (rd == 0) more_weights(0);
      // last chunk of a ragged q: a wave whose columns all lie past the last input block has nothing
      // to transform (their operand rows meet zero weights and keep whatever finite values they hold)
      if constexpr (ragged) {
        const int jw0 = (rd * CPR + (wave * 64) / LC) / NP;       // first input block of this wave's columns
        if (c * JC + jw0 >= q) continue;
      }
      {
        float re[R1], im[R1];
#pragma unroll
        for (int n1 = 0; n1 < R1; ++n1) {
          re[n1] = xr[rd][0][n1];
          im[n1] = xr[rd][1][n1];
        }
        if (rd == 0) more_weights(1);
        FftReg<R1, false>::run(re, im);               // A[f1][n2] = sum_n1 z[R2*n1 + n2] W_R1^(f1*n1)
        if (fwd_active) {
#pragma unroll
          for (int f1 = 0; f1 < R1; ++f1) {
            float vr = re[f1], vi = im[f1];
            if (f1 > 0) {                              // times W_K^(f1*n2) = cos - i sin
              const float c = ftw[f1].x, sn = ftw[f1].y;
              vr = c * re[f1] + sn * im[f1];
              vi = c * im[f1] - sn * re[f1];
            }
            xch[f1 * (R2 + 1) + fn2] = make_float2(vr, vi);
          }
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      CIRC_PROBE(2 + 4 * c);
      if (rd == 0) more_weights(2);
      if constexpr (kPairPass2) {
        // R2 = 2*R1: with one lane per second-pass transform half of the column's lanes would idle.
        // A pair of lanes shares one instead: lane hh of the pair runs the R2/2-point transform
        // of the inputs n2 = 2m + hh, E_hh, the odd lane multiplies by W_R2^f', the two exchange
        // their values, and lane hh ends with Z[f1 + R1*(f' + hh*R2/2)] = E_0[f'] +/- W_R2^f' E_1[f'].
        if (fwd_active) {
          constexpr int H = R2 / 2;
          const int f1 = fn2 >> 1;
          float re[H], im[H];
#pragma unroll
          for (int m = 0; m < H; ++m) {
            const float2 v = xch[f1 * (R2 + 1) + 2 * m + p2h];
            re[m] = v.x;
            im[m] = v.y;
          }
          if (rd == 0) more_weights(3);
          FftReg<H, false>::run(re, im);
#pragma unroll
          for (int f = 1; f < H; ++f) {
            const float tr = p2c[f] * re[f] - p2s[f] * im[f];
            im[f] = p2c[f] * im[f] + p2s[f] * re[f];
            re[f] = tr;
          }
#pragma unroll
          for (int f = 0; f < H; ++f) {
            re[f] = fmaf(p2sgn, re[f], quad_swap_pairs(re[f]));
            im[f] = fmaf(p2sgn, im[f], quad_swap_pairs(im[f]));
          }
          __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
          __builtin_amdgcn_wave_barrier();            // every lane of the column has read its inputs
#pragma unroll
          for (int fp = 0; fp < H; ++fp) {
            const int f = f1 + R1 * (fp + H * p2h);
            int slot, h;
            if (f == 0) { slot = 0; h = 0; }
            else if (f == S) { slot = 0; h = 1; }
            else if (f < S) { slot = f; h = 0; }
            else { slot = K - f; h = 1; }
            *reinterpret_cast<float2*>(creg + 4 * slot + 2 * h) = make_float2(re[fp], im[fp]);
          }
        } else if (rd == 0) {
          more_weights(3);
        }
      } else if (fwd_active && fn2 < R1) {            // lane f1 = fn2: Z[f1 + R1*f2] = sum_n2 A[f1][n2] W_R2^(f2*n2)
        float re[R2], im[R2];
#pragma unroll
        for (int n2 = 0; n2 < R2; ++n2) {
          const float2 v = xch[fn2 * (R2 + 1) + n2];
          re[n2] = v.x;
          im[n2] = v.y;
        }
        if (rd == 0) more_weights(3);
        FftReg<R2, false>::run(re, im);
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();              // every lane of the column has read its inputs
#pragma unroll
        for (int f2 = 0; f2 < R2; ++f2) {
          const int f = fn2 + R1 * f2;
          int slot, h;
          if (f == 0) { slot = 0; h = 0; }
          else if (f == S) { slot = 0; h = 1; }
          else if (f < S) { slot = f; h = 0; }
          else { slot = K - f; h = 1; }
          *reinterpret_cast<float2*>(creg + 4 * slot + 2 * h) = make_float2(re[f2], im[f2]);
        }
      } else if (rd == 0) {
        more_weights(3);
      }
    }
    more_weights(4);
    CIRC_PROBE(3 + 4 * c);
    // The x of the next chunk goes out before the barrier: a CU takes load instructions at a bounded
    // rate, and a wave that has to wait for the others anyway is the one place where queueing behind
    // them costs nothing.  The next chunk's weights follow inside the contraction (below).
    if constexpr (more) load_x(c + 1);
    __syncthreads();
    CIRC_PROBE(1 + 4 * c);
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
      if constexpr (more && !kWeightsLast) {   // one portion ahead of each batch of matrix instructions
        constexpr int NB = JW / JB;
        __builtin_amdgcn_sched_barrier(0);
        load_a(c + 1, a_pref, (jb / JB) * AH / NB, (jb / JB + 1) * AH / NB);
        __builtin_amdgcn_sched_barrier(0);
      }
      if constexpr (ragged) {
        if (c * JC + js * JW + jb >= q) continue;     // a batch of input blocks past the last one: zero weights
      }
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
    if constexpr (more && kWeightsLast) {
      __builtin_amdgcn_sched_barrier(0);
      load_a(c + 1, a_pref, 0, AH);
      __builtin_amdgcn_sched_barrier(0);
    }
    CIRC_PROBE(4 + 4 * c);
  };
  // steady state without conditionals around the loads (the compiler then waits for exactly the
  // operands a phase needs, not for everything in flight); the last one or two chunks are peeled.
  // Chunks alternate between the two sets of operand rows: a wave that is done with chunk c may
  // write the rows of chunk c+1 while others still read those of chunk c.
  {
    constexpr std::true_type yes{};
    constexpr std::false_type no{};
    int c = 0;
    if constexpr (ONE) {
      chunk(0, op0, a_even, a_even, no, yes, no);
    } else {
    float* op1 = op0 + Sh::OP_FLOATS;
    const bool rag = q % JC != 0;
    for (; c + 2 < nchunks; c += 2) {
      chunk(c, op0, a_even, a_odd, yes, no, no);
      chunk(c + 1, op1, a_odd, a_even, yes, no, no);
    }
    if (c + 2 == nchunks) {
      chunk(c, op0, a_even, a_odd, yes, no, no);
      if (rag) chunk(c + 1, op1, a_odd, a_even, no, no, yes);
      else chunk(c + 1, op1, a_odd, a_even, no, no, no);
    } else {
      if (rag) chunk(c, op0, a_even, a_odd, no, no, yes);
      else chunk(c, op0, a_even, a_odd, no, no, no);
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
      } else if constexpr (NCH == 2) {
        P[0][cc][u] += P[1][cc][u];
        Q[0][cc][u] += Q[1][cc][u];
      }
    }
  // Waves that split the j range (JS > 1) each assemble the output spectra of their share into a
  // tile of their own; the inverse transform adds the tiles as it reads them (in share order: a
  // fixed order), which saves a round trip through LDS and a barrier over summing the
  // accumulators first.
  // --- assemble Zy of every (output block row, batch pair) into the tile of this wave's share
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
      float* zl = zi + js * Sh::ZI_FLOATS + 2 * (fidx * PPI + 4 * ig * NP) + (n & 1);
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
  constexpr float osc = HM == 0 ? 1.0f : 1.0f / float(K);   // fp32 operands carry the 1/k already
  if constexpr (K == 64) {
    // 8 x 8 points per column, one wave per column: both passes run on the lane network
    // (Fft8Lanes: 8 points on 8 lanes), the exchange between them stays inside the wave, and
    // every lane ends with one sample of the two batch rows, which it stores itself.
    float2* z = reinterpret_cast<float2*>(zi);
    const int m = lane & 7, g = lane >> 3, fo = bitrev3(m);
    const Fft8Lanes<true> F(m);
#pragma unroll
    for (int t = 0; t < NI64; ++t) {
      const int coli = wave + t * NW;
      float2 v = z[(8 * m + g) * PPI + coli];                          // pass 1: lane = n1, group = n2
#pragma unroll
      for (int sh = 1; sh < JS; ++sh) {                                // the other shares of the j range, in order
        const float2 v2 = z[sh * K * PPI + (8 * m + g) * PPI + coli];
        v.x += v2.x;
        v.y += v2.y;
      }
      const float2 w = twl[fo * g];                                    // twiddle of output f1 = fo
      F.run(v.x, v.y);
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      __builtin_amdgcn_wave_barrier();                                 // the column has been read
      z[(8 * fo + g) * PPI + coli] = make_float2(w.x * v.x - w.y * v.y, w.x * v.y + w.y * v.x);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      v = z[(8 * g + m) * PPI + coli];                                 // pass 2: lane = n2, group = f1
      F.run(v.x, v.y);                                                 // sample g + 8*fo of rows (re, im)
      const int i = i0 + coli / NP, b = b0 + 2 * (coli % NP);
      if (i < p) {
        float o0 = v.x * osc + bv1[t], o1 = v.y * osc + bv1[t];
        if (relu) { o0 = fmaxf(o0, 0.f); o1 = fmaxf(o1, 0.f); }
        const long long yo = (long long)b * ldy + (long long)i * K + n64;
        if constexpr (HM == 0) {
          if (b < B) y[yo] = o0;
          if (b + 1 < B) y[yo + ldy] = o1;
        } else {
          unsigned short* y16 = reinterpret_cast<unsigned short*>(y);
          if (b < B) y16[yo] = (unsigned short)(pack_pair16<BF>(o0, 0.f) & 0xffffu);
          if (b + 1 < B) y16[yo + ldy] = (unsigned short)(pack_pair16<BF>(o1, 0.f) & 0xffffu);
        }
      }
    }
    CIRC_PROBE(61);
  } else {
    float2* z = reinterpret_cast<float2*>(zi);
    const int coli = tid % PTI, ti = tid / PTI;
    constexpr int TTI = NT / PTI;
    fft_lds_pass1<K, true>(z, PPI, coli, ti, TTI, twl);
    __syncthreads();
    fft_lds_pass2_inplace<K, true>(z, PPI, coli, ti, TTI);
    __syncthreads();
    CIRC_PROBE(61);
#pragma unroll
    for (int s = 0; s < NV; ++s) {
      const int idx = s * NT + tid;
      const int row = idx / (K / 4), n = 4 * (idx % (K / 4));
      const int colo = row >> 1, half = row & 1;
      const int i = i0 + colo / NP, b = b0 + 2 * (colo % NP) + half;
      if (idx < NOUT4 && i < p && b < B) {
        float4 v;
        v.x = lds_get(z, fft_pos<K>(n + 0) * PPI + colo, half) * osc + bv4[s].x;
        v.y = lds_get(z, fft_pos<K>(n + 1) * PPI + colo, half) * osc + bv4[s].y;
        v.z = lds_get(z, fft_pos<K>(n + 2) * PPI + colo, half) * osc + bv4[s].z;
        v.w = lds_get(z, fft_pos<K>(n + 3) * PPI + colo, half) * osc + bv4[s].w;
        if (relu) { v.x = fmaxf(v.x, 0.f); v.y = fmaxf(v.y, 0.f); v.z = fmaxf(v.z, 0.f); v.w = fmaxf(v.w, 0.f); }
        const long long yo = (long long)b * ldy + (long long)i * K + n;
        if constexpr (HM == 0) *reinterpret_cast<float4*>(y + yo) = v;
        else store_half4<BF>(reinterpret_cast<unsigned short*>(y) + yo, v);
      }
    }
  }
  CIRC_PROBE(62);
}

}  // namespace circ
