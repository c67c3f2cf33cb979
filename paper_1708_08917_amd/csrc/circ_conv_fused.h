// Fused block-circulant CONV forward (Sec. 3.2, Eq. 6 with the weight structure of Eq. 7):
// channel FFT -> contraction over the r*r offsets and the input channel blocks -> channel
// IFFT -> bias/ReLU in ONE kernel; x, the cached weight spectra and y are the only HBM traffic.
//
// The FFT runs over the channel axis of every pixel, and a spatial shift commutes with it, so
// each input pixel of a tile (output tile + halo) is transformed once and the r*r taps only
// pick different rows of the transformed tile; pixels outside the image have a zero spectrum.
//
// As in the fused FC kernel two real vectors share one complex transform, here the same pixel
// of two consecutive images (z = x[n] + i*x[n+1]): offsets and borders act identically on
// both, so the pair never has to be separated.  The contraction uses
// v_mfma_f32_4x4x1_16B_f32: block = frequency slot, rows = 4 output channel blocks,
// columns = (Re U, Im U, Re V, Im V) of one pixel pair, k = one (offset, input block).
// The r*r*q weight operands of a wave stay in registers for the whole tile.
#pragma once

#include <hip/hip_runtime.h>

#include "circ_fft.h"
#include "circ_fused.h"
#include "circ_kernels.h"

namespace circ {

// source of the zero padding (one aligned group of 4 pixels)
// (not const: it then lives in the same address space as x, and the loads stay global loads)
__device__ float kZeroPixels[4] __attribute__((aligned(16))) = {0.f, 0.f, 0.f, 0.f};

template <int K, int NT>
struct ConvFusedShape {
  static constexpr int NW = NT / 64;
  static constexpr int PT = 8 * NT / K;        // FFT columns per chunk
  static constexpr int PP = PT + 1;
  static constexpr int S = K / 2;
  static constexpr int FG = S / 16;
  static constexpr int OPROW = 2 * K + 2;
  static constexpr int MAXT = 4096 / NT;       // output positions per wave (8 or 16)
  static_assert(K >= 32 && NT % PT == 0 && (2 * K * PT) % NT == 0, "bad chunk shape");
};

// LDS bytes of a tile with `nrows` operand rows held at a time (input positions * channel
// blocks per round) and `ncoli` inverse columns (p * output positions).
template <int K, int NT>
inline size_t conv_fused_lds_bytes(int nrows, int ncoli) {
  using Sh = ConvFusedShape<K, NT>;
  size_t fwd = size_t(K) * Sh::PP * sizeof(float2) + size_t(nrows) * Sh::OPROW * sizeof(float);
  size_t inv = size_t(K) * (ncoli + 1) * sizeof(float2);   // overlays the forward tile and the operand rows
  return size_t(K) * sizeof(float2) + (fwd > inv ? fwd : inv);
}

// Weight spectra in the operand order of the fused CONV kernel:
//   Wc[((g*q + j)*ncombo + combo)*64 + 4*blk + m] = W^[g][i = 4*ig + m][j][slot = 16*fg + blk]
// with combo = ig*FG + fg, slot 0 = (W^[0].re, W^[K/2].re), rows i >= p zero.
// `spec` is the [g][f][j][i] section.  flip: grid g takes the spectra of grid n_grids-1-g (the
// spatially reflected filter of backward-data, where `spec` is the conjugated, transposed
// section and p, q are the block counts of the transposed grids).
__device__ __forceinline__ void pack_conv_elem(long long idx, const float2* __restrict__ spec, float2* __restrict__ Wc,
                                               int n_grids, int p, int q, int K, int ncombo, int flip) {
  const int FG = K / 32;
  const long long total = (long long)n_grids * q * ncombo * 64;
  if (idx >= total) return;
  const int l = int(idx & 63);
  long long rr = idx >> 6;
  const int combo = int(rr % ncombo); rr /= ncombo;
  const int j = int(rr % q);
  const int g = int(rr / q);
  const int fg = combo % FG, ig = combo / FG;
  const int i = 4 * ig + (l & 3), slot = 16 * fg + (l >> 2);
  float2 v = make_float2(0.f, 0.f);
  if (i < p) {
    const long long fs = (long long)p * q;
    const float2* sg = spec + (long long)(flip ? n_grids - 1 - g : g) * (K / 2 + 1) * fs;
    const long long e = (long long)j * p + i;
    v = slot == 0 ? make_float2(sg[e].x, sg[(long long)(K / 2) * fs + e].x) : sg[(long long)slot * fs + e];
  }
  Wc[idx] = v;
}

// R: filter size r, Q: input channel blocks q, QH: input channel blocks whose spectra are held
// in LDS at a time (the contraction runs in Q/QH rounds over the same accumulators).  All are
// compile-time so that the weight operands live in registers.
// One workgroup = one tile of TH x TW output positions of one image pair.
// HM: 0 = fp32 activations; 1 (fp16) / 2 (bfloat16): x and y point to 16-bit values (the loads
// convert on the way into the tile, the stores round the finished outputs; the cached weight
// spectra, 0.1 % of the bytes of a layer, stay fp32).
template <int K, int NT, int R, int Q, int QH, int HM = 0, bool RAGGED = false>
__global__ __launch_bounds__(NT, 2) void conv_fused_kernel(const float2* __restrict__ Wc, const float* __restrict__ x,
                                                        const float* __restrict__ bias, float* __restrict__ y,
                                                        int N, int C_out, int H, int W, int Ho, int Wo, int pad,
                                                        int TH, int TW, int tiles_h, int tiles_w, int ncombo, int relu) {
  using Sh = ConvFusedShape<K, NT>;
  constexpr int PT = Sh::PT, PP = Sh::PP, S = Sh::S, FG = Sh::FG, OPROW = Sh::OPROW, NW = Sh::NW, MAXT = Sh::MAXT;
  constexpr int C_in = Q * K;
  constexpr int R2 = radix2_of(K), R1 = radix1_of(K);
  static_assert(Q % QH == 0, "rounds must cover the input channel blocks evenly");
  extern __shared__ float smem[];
  float2* twl = reinterpret_cast<float2*>(smem);
  float2* z = twl + K;
  float* op = reinterpret_cast<float*>(z + K * PP);
  float2* zi = z;                                   // inverse tile, reuses the forward tile and the operand rows

  // the wave index is made explicitly wave-uniform: combo, positions and row addresses derived
  // from it then live in scalar registers
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int p = C_out / K;
  int bid = blockIdx.x;
  const int tw_i = bid % tiles_w; bid /= tiles_w;
  const int th_i = bid % tiles_h; bid /= tiles_h;
  const int n0 = 2 * bid;                           // first image of the pair
  const int h0 = th_i * TH, w0 = tw_i * TW;         // output tile origin
  // input positions of the tile use a fixed row pitch of 16 (IW <= 16), so that the offset of a
  // tap (dh, dw) inside the operand buffer is a compile-time constant
  constexpr int IWP = 16;
  const int IH = TH + R - 1, IW = TW + R - 1, IPOS = IH * IWP, NPOS = TH * TW;
  const int cpj = (IPOS + PT - 1) / PT;             // chunks per input channel block
  const int HW = H * W, HWo = Ho * Wo;

  CIRC_PROBE(0);
  // x of one chunk (RPC input rows of the tile, one channel block, both images).  Image rows are
  // multiples of 4 pixels (checked on the host), so a tile row of 16 input positions lies inside
  // NG aligned groups of 4 pixels: a task is one such group of one (image, channel, row) and
  // costs one 16-byte load; the lanes of a wave run along groups, then rows, then channels.
  // A group is entirely inside or outside the image; outside groups and rows load nothing and
  // put zeros into the tile (the zero padding of the convolution).
  constexpr int RPC = PT / IWP;                     // tile rows per chunk
  constexpr int NG = IWP / 4 + 1;                   // aligned groups that can touch one tile row
  constexpr int NLD = 2 * K * RPC * NG / NT;        // tasks per thread and chunk
  static_assert(PT % IWP == 0 && (2 * K * RPC * NG) % NT == 0, "x tasks must split evenly over the threads");
  const int colc = tid % PT;
  constexpr bool BF = HM == 2;
  const float* ximg = x + (long long)n0 * C_in * HW;
  const unsigned short* ximg16 = reinterpret_cast<const unsigned short*>(x) + (long long)n0 * C_in * HW;
  const bool second = n0 + 1 < N;
  const int gx0 = w0 - pad, g0 = gx0 >> 2, gsh = gx0 - 4 * g0;   // arithmetic shift = floor division
  auto load_chunk = [&](int ch, float4 (&xr)[NLD]) {  // ch = global chunk index over (j, row chunk)
    const int j = ch / cpj, pc = ch % cpj;
    const float* pj = ximg + (long long)j * K * HW;        // wave-uniform part of the address
    const unsigned short* pj16 = ximg16 + (long long)j * K * HW;
#pragma unroll
    for (int it = 0; it < NLD; ++it) {
      const int task = it * NT + tid;
      const int g = task % NG, r1 = task / NG;
      const int row = r1 % RPC, r2 = r1 / RPC;
      const int chn = r2 % K, img = r2 / K;
      const int rowg = pc * RPC + row, gh = h0 - pad + rowg, px0 = 4 * (g0 + g);
      // bitwise on purpose: one mask, no short-circuit branches
      const bool ok = bool(int(rowg < IH) & int(gh >= 0) & int(gh < H) & int(px0 >= 0) & int(px0 < W) &
                           (int(img == 0) | int(second)));
      // padding is read from a block of zeros: the load itself is unconditional
      if constexpr (!RAGGED) {
        if constexpr (HM == 0) {
          const float* src = ok ? pj + ((img * C_in + chn) * HW + gh * W + px0) : kZeroPixels;
          xr[it] = *reinterpret_cast<const float4*>(src);
        } else {
          const unsigned short* src = ok ? pj16 + ((img * C_in + chn) * HW + gh * W + px0) : reinterpret_cast<const unsigned short*>(kZeroPixels);
          xr[it] = load_half4<BF>(src);
        }
      } else {
        // rows that are no multiple of 4 pixels: a group is neither aligned nor entirely inside
        // the row, so its pixels are fetched one by one, each with its own test
        float vals[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const bool oke = ok && px0 + e < W;
          const int off = oke ? (img * C_in + chn) * HW + gh * W + px0 + e : 0;
          if constexpr (HM == 0) {
            vals[e] = oke ? pj[off] : 0.f;
          } else {
            const unsigned short hv = oke ? pj16[off] : (unsigned short)0;
            vals[e] = unpack_pair16<BF>(unsigned(hv)).x;
          }
        }
        xr[it] = make_float4(vals[0], vals[1], vals[2], vals[3]);
      }
    }
  };
  auto store_chunk = [&](const float4 (&xr)[NLD]) {
    float* zf = reinterpret_cast<float*>(z);
#pragma unroll
    for (int it = 0; it < NLD; ++it) {
      const int task = it * NT + tid;
      const int g = task % NG, r1 = task / NG;
      const int row = r1 % RPC, r2 = r1 / RPC;
      const int chn = r2 % K, img = r2 / K;
      const int iw0 = 4 * g - gsh;                         // tile column of the group's first pixel
      // pixels that fall left or right of the tile row go to the spare column PT of the tile
      // (never transformed), so that every write is unconditional
      float* zrow = zf + 2 * (chn * PP) + img;
      const float vals[4] = {xr[it].x, xr[it].y, xr[it].z, xr[it].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int iw = iw0 + e;
        const int col = (iw >= 0 && iw < IWP) ? row * IWP + iw : PT;
        zrow[2 * col] = vals[e];
      }
    }
  };
  // Memory returns loads in issue order: the K roots (from the table in the code object, cached) are
  // requested first, so that writing them to LDS does not wait for the first chunk of x behind them.
  float2 tw_stage[(K + NT - 1) / NT];
#pragma unroll
  for (int s = 0; s < (K + NT - 1) / NT; ++s)
    tw_stage[s] = reinterpret_cast<const float2*>(kTw.cs)[min(s * NT + tid, K - 1) * (kTwN / K)];
  float4 xa[NLD];
  load_chunk(0, xa);
#pragma unroll
  for (int s = 0; s < (K + NT - 1) / NT; ++s)
    if (s * NT + tid < K) twl[s * NT + tid] = tw_stage[s];

  // weight operands of this wave's (slot group, row group), one round (R*R*QH values) at a time
  const int combo = wave % ncombo, fg = combo % FG, ig = combo / FG;
  float2 a[R * R * QH];
  auto load_a = [&](int round) {
#pragma unroll
    for (int g = 0; g < R * R; ++g)
#pragma unroll
      for (int jl = 0; jl < QH; ++jl)
        a[g * QH + jl] = Wc[((g * Q + round * QH + jl) * ncombo + combo) * 64 + lane];
  };

  // output positions of this wave and their first input position
  floatx4 P[MAXT], Qa[MAXT];
  const int pos_first = wave / ncombo, pos_step = NW / ncombo;
#pragma unroll
  for (int tk = 0; tk < MAXT; ++tk) {
    P[tk] = floatx4{0.f, 0.f, 0.f, 0.f};
    Qa[tk] = floatx4{0.f, 0.f, 0.f, 0.f};
  }
  // first input position (top-left tap) of each of this wave's output positions, wave-uniform:
  // row*IWP + column of the output position, stepped from one position to the next without a
  // division; positions past the end of the tile use row 0 (their results are never stored);
  // ntk = positions that count
  static_assert(MAXT % 2 == 0, "positions are taken in pairs");
  int ipos[MAXT];
  int ntk = 0;
  {
    int prow = 0, pcol = pos_first;                   // pos_first < pos_step <= 8
    while (pcol >= TW) { pcol -= TW; ++prow; }
#pragma unroll
    for (int tk = 0; tk < MAXT; ++tk) {
      const bool in = pos_first + tk * pos_step < NPOS;
      ipos[tk] = __builtin_amdgcn_readfirstlane(in ? prow * IWP + pcol : 0);
      ntk += in ? 1 : 0;
      pcol += pos_step;
      while (pcol >= TW) { pcol -= TW; ++prow; }
    }
  }
  CIRC_PROBE(2);

  const int nch_total = Q * cpj, nch_round = QH * cpj;

  // one chunk: registers -> z tile -> two FFT passes -> operand rows
  auto fft_chunk = [&](int ch, float4 (&xr)[NLD], float4 (&xnext)[NLD]) {
    CIRC_PROBE(9 + 4 * ch);
    store_chunk(xr);
    __syncthreads();
    CIRC_PROBE(10 + 4 * ch);
    if (ch + 1 < nch_total) load_chunk(ch + 1, xnext);
    const int t = tid / PT;
    fft_lds_pass1<K, false>(z, PP, colc, t, NT / PT, twl);
    __syncthreads();
    CIRC_PROBE(11 + 4 * ch);
    const int jl = (ch % nch_round) / cpj, pos = (ch % cpj) * PT + colc;
    float* orow = op + (jl * IPOS + pos) * OPROW;
    const bool keep = pos < IPOS;
    fft_lds_pass2<K, false>(z, PP, colc, t, NT / PT, [&](int f, float2 v) {
      int sl, h;
      if (f == 0) { sl = 0; h = 0; }
      else if (f == S) { sl = 0; h = 1; }
      else if (f < S) { sl = f; h = 0; }
      else { sl = K - f; h = 1; }
      if (keep) *reinterpret_cast<float2*>(orow + 4 * sl + 2 * h) = v;
    });
    __syncthreads();
    CIRC_PROBE(12 + 4 * ch);
  };

#pragma unroll 1
  for (int round = 0; round < Q / QH; ++round) {
    load_a(round);
    for (int cl = 0; cl < nch_round; ++cl) fft_chunk(round * nch_round + cl, xa, xa);
    CIRC_PROBE(44 + 3 * round);
    // ---- contraction of this round: every wave takes up to MAXT output positions for its combo,
    // two at a time (independent accumulators back to back).  Rows of positions outside the
    // image hold the spectrum of zeros, so the taps need no border test.  Row indices are
    // wave-uniform (scalar registers); only the lane offset is per thread.  All operand rows of
    // a pair of positions are fetched before its matrix instructions.
    const float* opw = op + fg * 64 + lane;
#pragma unroll
    for (int tk = 0; tk < MAXT; tk += 2) {
      if (tk < ntk) {                                       // wave-uniform
        const float* r0 = opw + ipos[tk] * OPROW;
        const float* r1 = opw + ipos[tk + 1] * OPROW;       // the row of position 0 if tk + 1 is past the end
        float b0[R * R * QH], b1[R * R * QH];
#pragma unroll
        for (int dh = 0; dh < R; ++dh)
#pragma unroll
          for (int dw = 0; dw < R; ++dw)
#pragma unroll
            for (int jl = 0; jl < QH; ++jl) {
              b0[(dh * R + dw) * QH + jl] = (r0 + jl * IPOS * OPROW)[(dh * IWP + dw) * OPROW];
              b1[(dh * R + dw) * QH + jl] = (r1 + jl * IPOS * OPROW)[(dh * IWP + dw) * OPROW];
            }
#pragma unroll
        for (int g = 0; g < R * R * QH; ++g) {
          const float2 av = a[g];
          P[tk] = __builtin_amdgcn_mfma_f32_4x4x1f32(av.x, b0[g], P[tk], 0, 0, 0);
          Qa[tk] = __builtin_amdgcn_mfma_f32_4x4x1f32(av.y, b0[g], Qa[tk], 0, 0, 0);
          P[tk + 1] = __builtin_amdgcn_mfma_f32_4x4x1f32(av.x, b1[g], P[tk + 1], 0, 0, 0);
          Qa[tk + 1] = __builtin_amdgcn_mfma_f32_4x4x1f32(av.y, b1[g], Qa[tk + 1], 0, 0, 0);
        }
      }
    }
    CIRC_PROBE(45 + 3 * round);
    __syncthreads();   // every wave is done with the operand rows of this round
    CIRC_PROBE(46 + 3 * round);
  }
  // ---- spectra of the output pairs -> inverse tile (reuses the operand buffer),
  // column = i*NPOS + position, padded to CP (a power of two) columns for the thread mapping
  const int NCOLI = p * NPOS, PPI = NCOLI + 1;
  {
    const int n = lane & 3, blk = lane >> 2;
    const int slot = 16 * fg + blk;
    const int fidx = (n < 2) ? slot : (slot == 0 ? S : K - slot);
    float* zl = reinterpret_cast<float*>(zi) + 2 * fidx * PPI + (n & 1);   // per-lane part of the address
    // value = ca*P + cb*Q + cs*swap(Q) with per-lane constants (no divergent branches)
    const float ca = (slot == 0 && n >= 2) ? 0.f : 1.f;
    const float cb = (slot == 0 && n >= 2) ? 1.f : 0.f;
    const float cs = slot == 0 ? 0.f : ((n == 0 || n == 3) ? -1.f : 1.f);
    // rows of output blocks that do not exist (the last group of a p that is no multiple of 4) go to
    // the spare column of the tile, so that no store needs a test of its own
    int rowoff[4], posmul[4];
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const bool have = 4 * ig + m < p;
      rowoff[m] = __builtin_amdgcn_readfirstlane(have ? 2 * (4 * ig + m) * NPOS : 2 * NCOLI);
      posmul[m] = __builtin_amdgcn_readfirstlane(have ? 2 : 0);
    }
#pragma unroll
    for (int tk = 0; tk < MAXT; ++tk) {
      const int pos = pos_first + tk * pos_step;
      if (pos < NPOS) {
#pragma unroll
        for (int m = 0; m < 4; ++m) {
          const float pv = P[tk][m], qv = Qa[tk][m];
          const float qs = quad_swap_pairs(qv);
          zl[rowoff[m] + posmul[m] * pos] = fmaf(cs, qs, fmaf(cb, qv, ca * pv));
        }
      }
    }
  }
  CIRC_PROBE(57);
  __syncthreads();
  CIRC_PROBE(58);
  // Inverse transform of the NCOLI columns.  Several independent sub-transforms per thread and pass
  // (the loops are unrolled) hide each other's LDS latency: cfg4 47.6 -> 45 us.  (Running the
  // transform and the stores in two stages over halves of the output blocks, so that the stores of
  // one half overlap the transform of the other, measured 0.8 us slower: two more barriers.)
  int lgcp = 6;
  while ((1 << lgcp) < NCOLI) ++lgcp;
  const int CP = 1 << lgcp;
#pragma unroll 4
  for (int wk = tid; wk < CP * R2; wk += NT) {
    const int col = wk & (CP - 1);
    if (col < NCOLI) fft_lds_pass1<K, true>(zi, PPI, col, wk >> lgcp, R2, twl);
  }
  __syncthreads();
  CIRC_PROBE(59);
#pragma unroll 4
  for (int wk = tid; wk < CP * R1; wk += NT) {
    const int col = wk & (CP - 1);
    if (col < NCOLI) fft_lds_pass2_inplace<K, true>(zi, PPI, col, wk >> lgcp, R1);
  }
  __syncthreads();
  CIRC_PROBE(60);
  {
    // ---- store: a task is one pair of neighbouring output positions of one output channel,
    // for both images (two 8-byte stores); tile origins and row lengths are even (checked on the
    // host), so a pair is aligned and entirely inside or outside the image.  A wave covers
    // 64 / (pairs per channel) channels at a time; a lane keeps its pair for the whole loop.
    const int NPAIR = TW / 2, per_ch = TH * NPAIR;          // per_ch <= 32
    const int cpl = 64 / per_ch;                            // channels per wave iteration
    const int c_sub = lane / per_ch, rem = lane - c_sub * per_ch;
    const int orow = rem / NPAIR, pr = rem - orow * NPAIR;
    const int oh = h0 + orow, ow = w0 + 2 * pr;
    const bool lane_ok = c_sub < cpl && oh < Ho && ow < Wo;
    const bool two = ow + 1 < Wo;                           // false only for the last column of an odd row length
    const int zoff = orow * TW + 2 * pr;
    float* yimg = y + (long long)n0 * C_out * HWo + oh * Wo + ow;
    unsigned short* yimg16 = reinterpret_cast<unsigned short*>(y) + (long long)n0 * C_out * HWo + oh * Wo + ow;
#pragma unroll 4
    for (int cb = wave * cpl; cb < C_out; cb += NW * cpl) {
      const int c = cb + c_sub;
      if (lane_ok && c < C_out) {
        const int i = c / K, t = c % K;
        const float2* zc = zi + fft_pos<K>(t) * PPI + i * NPOS + zoff;
        const float2 u0 = zc[0], u1 = zc[1];               // (image 0, image 1) of the two positions
        const float bv = bias ? bias[c] : 0.f;
        float2 o0 = make_float2(u0.x + bv, u1.x + bv), o1 = make_float2(u0.y + bv, u1.y + bv);
        if (relu) {
          o0.x = fmaxf(o0.x, 0.f); o0.y = fmaxf(o0.y, 0.f);
          o1.x = fmaxf(o1.x, 0.f); o1.y = fmaxf(o1.y, 0.f);
        }
        if constexpr (HM == 0) {
          float* yo = yimg + (long long)c * HWo;
          float* yo1 = yo + (long long)C_out * HWo;
          if constexpr (!RAGGED) {
            *reinterpret_cast<float2*>(yo) = o0;
            if (second) *reinterpret_cast<float2*>(yo1) = o1;
          } else {                                          // odd row length: pairs are not aligned
            yo[0] = o0.x;
            if (two) yo[1] = o0.y;
            if (second) {
              yo1[0] = o1.x;
              if (two) yo1[1] = o1.y;
            }
          }
        } else {
          unsigned short* yo = yimg16 + (long long)c * HWo;
          unsigned short* yo1 = yo + (long long)C_out * HWo;
          const unsigned w0p = pack_pair16<BF>(o0.x, o0.y), w1p = pack_pair16<BF>(o1.x, o1.y);
          if constexpr (!RAGGED) {
            *reinterpret_cast<unsigned*>(yo) = w0p;
            if (second) *reinterpret_cast<unsigned*>(yo1) = w1p;
          } else {
            yo[0] = (unsigned short)(w0p & 0xffffu);
            if (two) yo[1] = (unsigned short)(w0p >> 16);
            if (second) {
              yo1[0] = (unsigned short)(w1p & 0xffffu);
              if (two) yo1[1] = (unsigned short)(w1p >> 16);
            }
          }
        }
      }
    }
  }
  CIRC_PROBE(62);
}

}  // namespace circ
