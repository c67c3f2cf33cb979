// FC forward for batch <= 2 in one launch: a bandwidth-bound streaming reduction.
//
// With one or two input vectors the contraction  Y^[i,f] = sum_j W^[i,j,f] X^[j,f]  is a
// matrix-vector product per frequency: every weight is used once, so the kernel is bound by
// streaming the cached weight spectra and runs on the vector ALUs (no matrix cores).
// One workgroup per output block row i:
//   1. FFT of the packed pair z = x_b0 + i*x_b1 for all q input blocks (recomputed by every
//      workgroup: x is tiny compared with the weights), written as the four real columns
//      (Re U, Im U, Re V, Im V), U = Z[f], V = conj(Z[K-f]) (column 3 stores +Im Z[K-f]);
//   2. thread (j-group, slot) streams W^[i][j][slot] (fully coalesced) and accumulates
//      P += Re(W^) * cols, Q += Im(W^) * cols;
//   3. the j-groups are summed through LDS in a fixed order, Zy[f] = (P0-Q1, P1+Q0),
//      Zy[K-f] = (P2+Q3, P3-Q2), slot 0 holds the real DC and Nyquist bins;
//   4. one inverse FFT gives (y_b0, y_b1); bias and ReLU are applied on the way out.
// This is Algorithm 1 with the weights cached in the frequency domain (Sec. 3.1, Sec. 4.2)
// and the real-input symmetry of Sec. 4.1.
#pragma once

#include <hip/hip_runtime.h>

#include <type_traits>

#include "circ_fft.h"
#include "circ_kernels.h"
#include "circ_probe.h"


namespace circ {

template <int K>
struct GemvShape {
  // threads per workgroup: these launches have few workgroups (one per output block row, times the
  // splits of the j range), so a workgroup takes 512 threads for its transforms and its share of
  // the weights (k = 4, whose chunks hold 512 one-thread columns, measured faster with 256)
  static constexpr int NT = K >= 8 ? 512 : 256;
  static constexpr int S = K / 2;                       // complex slots per block
  // input blocks (FFT columns) per chunk: up to 128, for the shortest blocks up to 512 (a chunk costs
  // one round trip to memory for its x rows, and layers with k <= 8 have many blocks per row)
  static constexpr int PTMAX = K <= 8 ? 512 : 128;
  static constexpr int PT = 4096 / K < PTMAX ? 4096 / K : PTMAX;
  static constexpr int PP = PT + 1;
  static constexpr int OPROW = 2 * K + 2;
  static constexpr int JG = NT / S >= 1 ? NT / S : 1;   // threads sharing a slot split the j range
  static constexpr int ZELEMS = K * PP;
  // the sum over the JG j-groups runs in two stages when there are threads to spare: NV values
  // (8 per slot), each first summed over NR contiguous ranges of GL groups, then over the ranges
  static constexpr int NV = 8 * S;
  static constexpr int NR = NT / NV >= 1 ? (NT / NV < JG ? NT / NV : JG) : 1;
  static constexpr int GL = JG / NR;
  static constexpr size_t LDS_BYTES = size_t(ZELEMS) * sizeof(float2) + size_t(PT) * OPROW * sizeof(float) +
                                      size_t(K) * sizeof(float2) + size_t(NT) * 9 * sizeof(float);
  static_assert(K >= 4 && K <= 512 && S <= NT, "block size out of range for this kernel");
};

// Weight spectra for the batch <= 2 kernel: Wg[(i*q + j)*S + slot], slot 0 = (W^[0].re,
// W^[K/2].re), slot f = W^[f] otherwise.  `spec` is the [f][j][i] section.
__device__ __forceinline__ void pack_gemv_elem(long long idx, const float2* __restrict__ spec, float2* __restrict__ Wg,
                                               int p, int q, int K) {
  const int S = K / 2;
  const long long total = (long long)p * q * S;
  if (idx >= total) return;
  const int slot = int(idx % S);
  const long long ij = idx / S;
  const int j = int(ij % q), i = int(ij / q);
  const long long fs = (long long)p * q, e = (long long)j * p + i;
  Wg[idx] = slot == 0 ? make_float2(spec[e].x, spec[(long long)S * fs + e].x) : spec[(long long)slot * fs + e];
}

// The same order for 16-bit storage, one word per value; `spec` is the 16-bit section [f][i][j].
__device__ __forceinline__ void pack_gemv_half_elem(long long idx, const unsigned* __restrict__ spec, unsigned* __restrict__ Wg,
                                                    int p, int q, int K) {
  const int S = K / 2;
  const long long total = (long long)p * q * S;
  if (idx >= total) return;
  const int slot = int(idx % S);
  const long long e = idx / S, fs = (long long)p * q;   // e = i*q + j
  Wg[idx] = slot == 0 ? ((spec[e] & 0xffffu) | (spec[(long long)S * fs + e] << 16)) : spec[(long long)slot * fs + e];
}
__global__ __launch_bounds__(256) void pack_gemv_half_kernel(const unsigned* __restrict__ spec, unsigned* __restrict__ Wg, int p,
                                                             int q, int K) {
  pack_gemv_half_elem((long long)blockIdx.x * 256 + threadIdx.x, spec, Wg, p, q, K);
}

// MODE 0: the whole layer in one launch, one workgroup per output block row (grid p).
// Layers with few block rows and long rows leave most of the chip idle that way and make every
// workgroup transform all of x; they run as two launches instead:
// MODE 1 (grid p x nsplit): workgroup (i, js) transforms and contracts only the input blocks
//   [js*jper, (js+1)*jper) and writes the spectrum of its partial output pair to
//   part[(js*p + i)*K + f];
// MODE 2 (grid p): adds the nsplit partial spectra in index order, inverse transform, epilogue.
// HM: 0 = fp32; 1 (fp16) / 2 (bfloat16) = 16-bit storage: Wg then points to one 32-bit word per
// value (the 16-bit (re, im) pair, not normalised; pack_gemv_half_elem), x and y to 16-bit values;
// the arithmetic and the partial spectra of MODE 1 / 2 stay fp32, the 1/k goes onto the result.
template <int K, int MODE, int HM = 0>
__global__ __launch_bounds__(GemvShape<K>::NT) void fc_gemv_kernel(const float2* __restrict__ Wg, const float* __restrict__ x,
                                                      const float* __restrict__ bias, float* __restrict__ y,
                                                      int p, int q, int B, int relu, float2* __restrict__ part,
                                                      int nsplit, int jper) {
  using Sh = GemvShape<K>;
  constexpr int NT = Sh::NT, S = Sh::S, PT = Sh::PT, PP = Sh::PP, OPROW = Sh::OPROW, JG = Sh::JG;
  extern __shared__ float smem[];
  float2* z = reinterpret_cast<float2*>(smem);
  float* op = smem + 2 * Sh::ZELEMS;
  float2* twl = reinterpret_cast<float2*>(op + PT * OPROW);
  float* red = reinterpret_cast<float*>(twl + K);

  const int tid = threadIdx.x;
  const int i = blockIdx.x;
  const long long ldx = (long long)q * K, ldy = (long long)p * K;
  // input blocks of this workgroup: [jbeg, jend)
  const int jbeg = MODE == 1 ? blockIdx.y * jper : 0;
  const int jend = MODE == 1 ? min(q, jbeg + jper) : q;
  const int nchunks = MODE == 2 ? 0 : (jend - jbeg + PT - 1) / PT;
  // the K roots are requested first and written to LDS once the first x loads are out (memory
  // returns loads in issue order: nothing waits for the roots before x and the weights are requested)
  TwiddleStage<K> tws;
  tws.request(tid, NT);

  const int slot = tid % S, jg = tid / S;          // contraction role (threads beyond S*JG idle)
  const bool active = jg < JG;
  float P[4] = {0.f, 0.f, 0.f, 0.f}, Q[4] = {0.f, 0.f, 0.f, 0.f};
  constexpr bool BF = HM == 2;
  using WOp = typename std::conditional<HM != 0, unsigned, float2>::type;
  const WOp* wrow = reinterpret_cast<const WOp*>(Wg) + (long long)i * q * S + slot;
  // The weights of a chunk are fetched one chunk ahead (those of the first chunk before x is
  // even staged), so that their latency overlaps the FFT instead of following it.
  constexpr int NPF = (PT + JG - 1) / JG;          // weights per thread and chunk
  WOp wnext[NPF];
  auto fetch_w = [&](int c) {
#pragma unroll
    for (int u = 0; u < NPF; ++u) {
      const int jj = jg + u * JG, j = jbeg + c * PT + jj;
      wnext[u] = WOp{};                              // zero in either format
      if (active && jj < PT && j < jend) wnext[u] = wrow[(long long)j * S];
    }
  };
  if (MODE != 2) fetch_w(0);
  CIRC_PROBE(0);

  for (int c = 0; c < nchunks; ++c) {
    const int j0 = jbeg + c * PT;
    // rows b0 (real part) and b1 (imaginary part) of the chunk -> z[n][column j].  A step of one
    // float4 along n is 8*PP words in the tile (8 banks modulo 32, PP odd) and a step of one
    // column 2 words: GW lanes along n times 64/GW consecutive columns per wave spread the LDS
    // stores over 16 banks (all lanes along n would share 4).  A wave stays inside one row, so
    // that for batch 1 the waves of the absent row issue no loads.
    constexpr int GW = K / 4 < 8 ? K / 4 : 8;
    static_assert(PT % (64 / GW) == 0, "a wave-load must not straddle the two rows");
    for (int idx = tid; idx < 2 * PT * (K / 4); idx += NT) {
      const int gl = idx % GW, rest = idx / GW;
      const int col = rest % PT, half = (rest / PT) & 1, n = 4 * ((rest / (2 * PT)) * GW + gl);
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (half < B && j0 + col < jend) {
        const long long xo = (long long)half * ldx + (long long)(j0 + col) * K + n;
        if constexpr (HM == 0) v = *reinterpret_cast<const float4*>(x + xo);
        else v = load_half4<BF>(reinterpret_cast<const unsigned short*>(x) + xo);
      }
      lds_put(z, (n + 0) * PP + col, half, v.x);
      lds_put(z, (n + 1) * PP + col, half, v.y);
      lds_put(z, (n + 2) * PP + col, half, v.z);
      lds_put(z, (n + 3) * PP + col, half, v.w);
    }
    if (c == 0) tws.store(twl, tid, NT);
    __syncthreads();
    CIRC_PROBE(1 + 3 * c);
    auto sink = [&](int col) {
      return [=](int f, float2 v) {
        int sl, h;
        if (f == 0) { sl = 0; h = 0; }
        else if (f == S) { sl = 0; h = 1; }
        else if (f < S) { sl = f; h = 0; }
        else { sl = K - f; h = 1; }
        *reinterpret_cast<float2*>(op + col * OPROW + 4 * sl + 2 * h) = v;
      };
    };
    if constexpr (K <= 16) {
      // short blocks: one thread transforms a whole column in registers (no second pass)
      for (int col = tid; col < PT; col += NT) fft_lds_single<K, false>(z, PP, col, sink(col));
    } else {
      const int col = tid % PT, t = tid / PT;
      fft_lds_pass1_unrolled<K, false, NT / PT>(z, PP, col, t, twl);
      __syncthreads();
      fft_lds_pass2<K, false>(z, PP, col, t, NT / PT, sink(col));
    }
    __syncthreads();
    CIRC_PROBE(2 + 3 * c);
    WOp wcur[NPF];
#pragma unroll
    for (int u = 0; u < NPF; ++u) wcur[u] = wnext[u];
    if (c + 1 < nchunks) fetch_w(c + 1);
    if (active) {
      const int jlim = min(PT, jend - j0);
#pragma unroll
      for (int u = 0; u < NPF; ++u) {
        const int jj = jg + u * JG;
        if (jj < jlim) {     // (weights past the end were fetched as zeros; the operand row must exist)
          float2 w;
          if constexpr (HM == 0) w = wcur[u];
          else w = unpack_pair16<BF>(wcur[u]);
          const float4 cv = *reinterpret_cast<const float4*>(op + jj * OPROW + 4 * slot);
          P[0] += w.x * cv.x; P[1] += w.x * cv.y; P[2] += w.x * cv.z; P[3] += w.x * cv.w;
          Q[0] += w.y * cv.x; Q[1] += w.y * cv.y; Q[2] += w.y * cv.z; Q[3] += w.y * cv.w;
        }
      }
    }
    __syncthreads();   // z and op are rewritten by the next chunk
    CIRC_PROBE(3 + 3 * c);
  }

  if constexpr (MODE == 2) {
    tws.store(twl, tid, NT);
    // spectrum of the output pair = sum of the partial spectra, in index order
    for (int f = tid; f < K; f += NT) {
      float2 acc = make_float2(0.f, 0.f);
      const float2* src = part + (long long)i * K + f;
#pragma unroll 4
      for (int js = 0; js < nsplit; ++js) {
        const float2 v = src[(long long)js * p * K];
        acc.x += v.x;
        acc.y += v.y;
      }
      z[2 * f] = acc;
    }
  } else {
    // sum over the j-groups in a fixed order, then assemble the spectrum of the output pair
    if (active) {
  #pragma unroll
      for (int m = 0; m < 4; ++m) {
        red[(m * JG + jg) * S + slot] = P[m];
        red[((4 + m) * JG + jg) * S + slot] = Q[m];
      }
    }
    __syncthreads();
    constexpr int NV = Sh::NV, NR = Sh::NR, GL = Sh::GL;
    float* red2 = red + NT * 8;                    // [range][value]
    if constexpr (NR > 1) {
      // stage 1: thread (range r, value v = m8*S + slot) adds its GL groups in index order
      if (tid < NV * NR) {
        const int v = tid % NV, r = tid / NV, m8 = v / S, sl = v % S;
        float a = 0.f;
        for (int g = r * GL; g < (r + 1) * GL; ++g) a += red[(m8 * JG + g) * S + sl];
        red2[r * NV + v] = a;
      }
      __syncthreads();
    }
    if (tid < S) {
      float Ps[4], Qs[4];
  #pragma unroll
      for (int m = 0; m < 4; ++m) {
        float a = 0.f, b = 0.f;
        if constexpr (NR > 1) {
          for (int r = 0; r < NR; ++r) {             // stage 2: the ranges, in index order
            a += red2[r * NV + m * S + tid];
            b += red2[r * NV + (4 + m) * S + tid];
          }
        } else {
          for (int g = 0; g < JG; ++g) {
            a += red[(m * JG + g) * S + tid];
            b += red[((4 + m) * JG + g) * S + tid];
          }
        }
        Ps[m] = a;
        Qs[m] = b;
      }
      if (tid == 0) {
        z[0] = make_float2(Ps[0], Ps[1]);              // DC of (y_b0, y_b1)
        z[S * 2] = make_float2(Qs[2], Qs[3]);          // Nyquist
      } else {
        z[tid * 2] = make_float2(Ps[0] - Qs[1], Ps[1] + Qs[0]);
        z[(K - tid) * 2] = make_float2(Ps[2] + Qs[3], Ps[3] - Qs[2]);
      }
    }
  }
  __syncthreads();
  CIRC_PROBE(40);
  if constexpr (MODE == 1) {
    // partial spectrum of the output pair (column 0 of z, row stride 2) -> workspace
    float2* dst = part + ((long long)blockIdx.y * p + i) * K;
    for (int f = tid; f < K; f += NT) dst[f] = z[2 * f];
    return;
  }
  // inverse transform of the single column (row stride 2); afterwards sample n of the pair sits
  // at position opos(n)
  if constexpr (K == 8 || K == 16) {
    // one short column: its K points on K lanes (DPP exchanges) instead of one thread's ~170
    // dependent instructions
    float2* zo = z + 2 * K;                      // natural order, behind the input column
    if (tid < K) {
      float2 v = z[2 * tid];
      fft_lanes<K, K, true>(v, tid, twl);
      zo[2 * lane_rev<K>(tid)] = v;
    }
    __syncthreads();
  } else if constexpr (K <= 16) {
    float2* zo = z + 2 * K;                      // natural order, behind the input column
    if (tid == 0) fft_lds_single<K, true>(z, 2, 0, [&](int n, float2 v) { zo[2 * n] = v; });
    __syncthreads();
  } else if constexpr (K == 64 || K == 128 || K == 256) {
    fft_column_lanes<K, true>(z, 2, tid, twl);   // sub-transforms of 8 or 16 points, on as many lanes each
    __syncthreads();
  } else {
    fft_lds_pass1<K, true>(z, 2, 0, tid, NT, twl);
    __syncthreads();
    fft_lds_pass2_inplace<K, true>(z, 2, 0, tid, NT);
    __syncthreads();
  }
  CIRC_PROBE(41);
  auto opos = [](int n) { return K <= 16 ? K + n : fft_pos<K>(n); };
  for (int idx = tid; idx < 2 * K; idx += NT) {
    const int half = idx / K, n = idx % K;
    if (half < B) {
      constexpr float osc = HM == 0 ? 1.0f : 1.0f / float(K);   // fp32 operands carry the 1/k already
      float v = lds_get(z, opos(n) * 2, half) * osc;
      if (bias) v += bias[(long long)i * K + n];
      if (relu) v = fmaxf(v, 0.f);
      const long long yo = (long long)half * ldy + (long long)i * K + n;
      if constexpr (HM == 0) y[yo] = v;
      else reinterpret_cast<unsigned short*>(y)[yo] = (unsigned short)(pack_pair16<BF>(v, 0.f) & 0xffffu);
    }
  }
  CIRC_PROBE(42);
}

}  // namespace circ
