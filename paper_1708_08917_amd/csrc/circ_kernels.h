// HIP kernels (gfx950) of the block-circulant layer pipeline:
//   rfft_kernel      real rows -> half spectra            (FFT of Algorithm 1 / 2)
//   cgemm_kernel     per-frequency complex contraction on the fp32 matrix cores
//                    (the "o" of Algorithm 1 with the sum over j moved inside the IFFT,
//                    which Eq. 3 allows because the transform is linear)
//   conv_contract_kernel  the same contraction for CONV: sum over the r*r offsets and
//                    the input channel blocks (Eq. 6 / Eq. 7)
//   irfft_kernel     half spectra -> real rows, fused bias + ReLU (Eq. 1)
// The two transform kernels can also read or write 16-bit values (IEEE fp16 or bfloat16; rows and /
// or spectra, HMODE) for the half-width storage route; their arithmetic stays fp32.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include "circ_fft.h"

namespace circ {

// Half-width storage (16-bit values in memory, fp32 in registers and LDS): bit 0 of HMODE = the
// real rows are 16-bit, bit 1 = the spectra are 16-bit (re, im) pairs, bit 2 = the 16-bit format
// is bfloat16 (the upper half of an fp32, rounded to nearest even) instead of IEEE fp16.
constexpr int kHalfRows = 1, kHalfSpectra = 2, kHalfBf16 = 4;

template <bool BF>
__device__ __forceinline__ float2 unpack_pair16(unsigned w) {       // one 32-bit word = two 16-bit values
  if constexpr (BF) return make_float2(__uint_as_float(w << 16), __uint_as_float(w & 0xffff0000u));
  else return __half22float2(*reinterpret_cast<const __half2*>(&w));
}
__device__ __forceinline__ unsigned bf16_bits(float v) {            // round to nearest even; NaN stays NaN
  const unsigned u = __float_as_uint(v);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
template <bool BF>
__device__ __forceinline__ unsigned pack_pair16(float a, float b) {
  if constexpr (BF) return bf16_bits(a) | (bf16_bits(b) << 16);
  else {
    const __half2 h = __floats2half2_rn(a, b);
    return *reinterpret_cast<const unsigned*>(&h);
  }
}
template <bool BF>
__device__ __forceinline__ float4 load_half4(const void* p) {       // 4 consecutive 16-bit values, 8-byte aligned
  const uint2 raw = *reinterpret_cast<const uint2*>(p);
  const float2 a = unpack_pair16<BF>(raw.x), b = unpack_pair16<BF>(raw.y);
  return make_float4(a.x, a.y, b.x, b.y);
}
template <bool BF>
__device__ __forceinline__ void store_half4(void* p, float4 v) {
  *reinterpret_cast<uint2*>(p) = make_uint2(pack_pair16<BF>(v.x, v.y), pack_pair16<BF>(v.z, v.w));
}

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// LDS bytes of one FFT tile of P column pairs.
inline size_t fft_tile_lds_bytes(int K, int P) {
  return size_t(K) * (P + 1) * sizeof(float2) + size_t(K) * sizeof(float2) +
         size_t(2 * P) * (sizeof(long long) + sizeof(int));
}

struct TileLds {
  float2* z;
  float2* tw;
  long long* rbase;
  int* rblk;
};

template <int K>
__device__ __forceinline__ TileLds carve_tile(float* smem, int P) {
  TileLds t;
  t.z = reinterpret_cast<float2*>(smem);
  t.tw = t.z + K * (P + 1);
  t.rbase = reinterpret_cast<long long*>(t.tw + K);
  t.rblk = reinterpret_cast<int*>(t.rbase + 2 * P);
  return t;
}

__device__ __forceinline__ void lds_put(float2* z, int idx, int half, float v) {
  reinterpret_cast<float*>(z)[2 * idx + half] = v;
}
__device__ __forceinline__ float lds_get(const float2* z, int idx, int half) {
  return reinterpret_cast<const float*>(z)[2 * idx + half];
}

// Separates the two real rows of each column of a transformed tile (z, P column pairs starting at
// row id t0) and stores bins 0..K/2: out[f*out_fstride + rid], scaled, conjugated if `conj`.
template <int K, int HMODE>
__device__ __forceinline__ void rfft_store_tile(const float2* z, int P, int lgP, int tid, int NT, long long t0, long long nrows,
                                                float2* __restrict__ out, long long out_fstride, float scale, int conj) {
  const int PP = P + 1;
  // separate the two real rows of each column and store bins 0..K/2
  constexpr int NF = K / 2 + 1;
  const float h = 0.5f * scale, hc = conj ? -h : h;
  {
    // a thread keeps its column pair; its bin advances by NT/P per step
    const int pr = tid & (P - 1), fstep = NT >> lgP;
    const long long rid = t0 + 2 * pr;
    const bool ok0 = rid < nrows, ok1 = rid + 1 < nrows;
    static_assert(HMODE == 0 || K >= 4, "half-width storage: K >= 4 only");
    long long o = (long long)(tid >> lgP) * out_fstride + rid;
    const long long ostep = (long long)fstep * out_fstride;
    // whole tile inside the buffer and the pair (rid, rid + 1) aligned to its combined width:
    // one store per bin, no predicates (the loop body is then branch-free and several bins'
    // LDS reads are in flight at once)
    constexpr int PAIRB = (HMODE & kHalfSpectra) ? 8 : 16;
    const bool whole = t0 + 2 * P <= nrows && (out_fstride & 1) == 0 &&
                       (reinterpret_cast<unsigned long long>(out) & (PAIRB - 1)) == 0;
    if (whole) {
#pragma unroll 4
      for (int f = tid >> lgP; f < NF; f += fstep, o += ostep) {
        float2 u = z[fft_pos<K>(f) * PP + pr], w = z[fft_pos<K>(f == 0 ? 0 : K - f) * PP + pr];
        const float2 v0 = make_float2(h * (u.x + w.x), hc * (u.y - w.y));
        const float2 v1 = make_float2(h * (u.y + w.y), hc * (w.x - u.x));
        if constexpr (HMODE & kHalfSpectra) {
          *reinterpret_cast<uint2*>(reinterpret_cast<unsigned*>(out) + o) =
              make_uint2(pack_pair16<(HMODE & kHalfBf16) != 0>(v0.x, v0.y), pack_pair16<(HMODE & kHalfBf16) != 0>(v1.x, v1.y));
        } else {
          *reinterpret_cast<float4*>(out + o) = make_float4(v0.x, v0.y, v1.x, v1.y);
        }
      }
      return;
    }
#pragma unroll 2
    for (int f = tid >> lgP; f < NF; f += fstep, o += ostep) {
      float2 u = z[fft_pos<K>(f) * PP + pr], w = z[fft_pos<K>(f == 0 ? 0 : K - f) * PP + pr];
      const float2 v0 = make_float2(h * (u.x + w.x), hc * (u.y - w.y));
      const float2 v1 = make_float2(h * (u.y + w.y), hc * (w.x - u.x));
      if constexpr (HMODE & kHalfSpectra) {
        unsigned* oh = reinterpret_cast<unsigned*>(out) + o;
        if (ok0) oh[0] = pack_pair16<(HMODE & kHalfBf16) != 0>(v0.x, v0.y);
        if (ok1) oh[1] = pack_pair16<(HMODE & kHalfBf16) != 0>(v1.x, v1.y);
      } else {
        if (ok0) out[o] = v0;
        if (ok1) out[o + 1] = v1;
      }
    }
  }
}

// -------------------------------------------------------------------------------------
// Forward real FFT of rows.  Block b handles rows [2*P*b, 2*P*(b+1)); out[f*fstride + rid]
// holds bin f (0..K/2) of row rid, scaled by `scale`, conjugated if `conj`.
// blockIdx.y selects one of several independent grids (weight precompute for CONV).
// ROWS_FAST: consecutive rows are adjacent in memory (CONV, NCHW: the FFT axis is the
// channel axis and pixels are contiguous) — lanes then run along rows when loading.
// HMODE (see kHalfRows / kHalfSpectra / kHalfBf16): `in` then points to 16-bit rows and / or `out` to 16-bit pairs;
// offsets and strides keep their meaning in elements.  K >= 4 only.
template <int K, bool ROWS_FAST, int HMODE = 0>
__global__ void rfft_kernel(const float* __restrict__ in, float2* __restrict__ out, RowMap map,
                            long long nrows, long long out_fstride, long long in_gstride,
                            long long out_gstride, int P, float scale, int conj) {
  extern __shared__ float smem[];
  const int PP = P + 1;
  const int lgP = __ffs(P) - 1;
  TileLds L = carve_tile<K>(smem, P);
  in += (long long)blockIdx.y * in_gstride;
  out += (long long)blockIdx.y * out_gstride;
  const long long t0 = (long long)blockIdx.x * 2 * P;
  const int tid = threadIdx.x, NT = blockDim.x;

  TwiddleStage<K> tws;
  tws.request(tid, NT);
  // (groups of 4 adjacent rows, below, need no table of row addresses and no barrier before their loads)
  const bool quad_rows = ROWS_FAST && map.quad;
  if (!quad_rows) {
    for (int r = tid; r < 2 * P; r += NT) {
      long long rid = t0 + r;
      L.rbase[r] = rid < nrows ? row_base(map, rid) : -1;
    }
    __syncthreads();
  }

  // load: row 2u -> real part of column u, row 2u+1 -> imaginary part
  if constexpr (ROWS_FAST) {
    if (map.quad) {
      // 4 rows per 16-byte load; they are the (re, im) slots of two neighbouring columns, i.e.
      // 4 consecutive floats of the tile (8-byte aligned: two 8-byte LDS stores).  A thread keeps
      // its group of 4 rows (NT is a multiple of the P/2 groups of a tile) and works out their
      // address itself; its loads, one per element index, go out together.
      const int nq = P >> 1;                       // groups of 4 rows in the tile
      const int qd = tid & (nq - 1), nstep = NT >> (lgP - 1);
      const long long rid = t0 + 4 * qd;
      float2* zq = L.z + 2 * qd;
      if (rid < nrows) {
        const long long b = row_base(map, rid);
#pragma unroll 8
        for (int n = tid >> (lgP - 1); n < K; n += nstep) {
          float4 v;
          if constexpr (HMODE & kHalfRows) v = load_half4<(HMODE & kHalfBf16) != 0>(reinterpret_cast<const unsigned short*>(in) + b + n * map.es);
          else v = *reinterpret_cast<const float4*>(in + b + n * map.es);
          float2* zd = zq + n * PP;
          zd[0] = make_float2(v.x, v.y);
          zd[1] = make_float2(v.z, v.w);
        }
      } else {
        for (int n = tid >> (lgP - 1); n < K; n += nstep) {
          float2* zd = zq + n * PP;
          zd[0] = make_float2(0.f, 0.f);
          zd[1] = make_float2(0.f, 0.f);
        }
      }
    } else {
#pragma unroll 4
      for (int idx = tid; idx < 2 * P * K; idx += NT) {
        int row = idx & (2 * P - 1), n = idx >> (lgP + 1);
        long long b = L.rbase[row];
        float v = 0.f;
        if constexpr (HMODE & kHalfRows) {
          if (b >= 0) v = unpack_pair16<(HMODE & kHalfBf16) != 0>(reinterpret_cast<const unsigned short*>(in)[b + n * map.es]).x;
        } else {
          if (b >= 0) v = in[b + n * map.es];
        }
        lds_put(L.z, n * PP + (row >> 1), row & 1, v);
      }
    }
  } else if constexpr (K >= 4 && is_pow2_c(K)) {
    // rows are contiguous (element stride 1) and 16-byte aligned: vector loads along the row.
    // One wave-load covers 64/GW rows x GW*16 contiguous bytes.  A step of one float4 along the
    // row is 8*PP words in the tile, a multiple of 8 (PP is odd), so with all 64 lanes along one
    // row they would share 4 LDS banks; 8 lanes along the row (4 banks, twice) times 8 rows
    // (row r sits r words from row 0) give every bank exactly two lanes.
    constexpr int GW = K / 4 < 8 ? K / 4 : 8, NSEG = K / (4 * GW);
    const int gl = tid % GW, rstep = NT / GW;
    for (int row = tid / GW; row < 2 * P; row += rstep) {
      const long long b = L.rbase[row];
      float* zrow = reinterpret_cast<float*>(L.z) + row;      // 2*(row >> 1) + (row & 1) == row
#pragma unroll
      for (int seg = 0; seg < NSEG; ++seg) {
        const int n = 4 * (seg * GW + gl);
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if constexpr (HMODE & kHalfRows) {
          if (b >= 0) v = load_half4<(HMODE & kHalfBf16) != 0>(reinterpret_cast<const unsigned short*>(in) + b + n);
        } else {
          if (b >= 0) v = *reinterpret_cast<const float4*>(in + b + n);
        }
        float* zd = zrow + 2 * n * PP;
        zd[0] = v.x;
        zd[2 * PP] = v.y;
        zd[4 * PP] = v.z;
        zd[6 * PP] = v.w;
      }
    }
  } else if constexpr (K % 4 == 0) {
    // the same for block sizes that are not powers of two: one float4 per thread and step,
    // consecutive threads along the row
    constexpr int Q4 = K / 4;
    for (int idx = tid; idx < 2 * P * Q4; idx += NT) {
      const int row = idx / Q4, n = 4 * (idx - row * Q4);
      const long long b = L.rbase[row];
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if constexpr (HMODE & kHalfRows) {
        if (b >= 0) v = load_half4<(HMODE & kHalfBf16) != 0>(reinterpret_cast<const unsigned short*>(in) + b + n);
      } else {
        if (b >= 0) v = *reinterpret_cast<const float4*>(in + b + n);
      }
      float* zd = reinterpret_cast<float*>(L.z) + row + 2 * n * PP;
      zd[0] = v.x;
      zd[2 * PP] = v.y;
      zd[4 * PP] = v.z;
      zd[6 * PP] = v.w;
    }
  } else {
    for (int idx = tid; idx < 2 * P * K; idx += NT) {
      int row = idx / K, n = idx % K;
      long long b = L.rbase[row];
      float v = b >= 0 ? in[b + n] : 0.f;
      lds_put(L.z, n * PP + (row >> 1), row & 1, v);
    }
  }
  tws.store(L.tw, tid, NT);
  __syncthreads();

  const int col = tid & (P - 1), t = tid >> lgP, TT = NT >> lgP;
  fft_lds_pass1<K, false>(L.z, PP, col, t, TT, L.tw);
  __syncthreads();
  fft_lds_pass2_inplace<K, false>(L.z, PP, col, t, TT);
  __syncthreads();

  rfft_store_tile<K, HMODE>(L.z, P, lgP, tid, NT, t0, nrows, out, out_fstride, scale, conj);
}

// -------------------------------------------------------------------------------------
// The same transform for long runs of contiguous rows (the activations of a large FC layer):
// a workgroup walks over tiles of 4096 / K column pairs, blockIdx.x, blockIdx.x + gridDim.x, ..., and
// requests the rows of its next tile before it transforms the current one, so that a CU keeps
// loads in flight while its vector units work (in rfft_kernel a workgroup spends half of its time
// waiting for its 32 KB of rows: 10,500 of 21,900 cycles at 65,536 rows of 256).  Memory returns
// loads in issue order, so the K roots are requested ahead of the first rows, and a thread works
// out the addresses of its own rows instead of waiting for a table of them in LDS.
// 256 threads; rows contiguous (element stride 1) and 16-byte aligned; 32 <= K <= 256.
template <int K, int HMODE = 0>
__global__ __launch_bounds__(256) void rfft_stream_kernel(const float* __restrict__ in, float2* __restrict__ out, RowMap map,
                                                          long long nrows, long long out_fstride, int ntiles, float scale,
                                                          int conj) {
  static_assert(is_pow2_c(K) && K >= 32 && K <= 256, "block sizes of the streaming transform");
  constexpr int P = 4096 / K, PP = P + 1, NT = 256, lgP = ilog2(P);
  constexpr int GW = 8, NSEG = K / (4 * GW), RSTEP = NT / GW, NRI = 2 * P / RSTEP;   // NRI * NSEG = 8 loads per thread
  static_assert(NRI >= 1 && NRI * RSTEP == 2 * P, "rows of a tile split evenly over the threads");
  extern __shared__ float smem[];
  TileLds L = carve_tile<K>(smem, P);
  const int tid = threadIdx.x, gl = tid % GW, r0 = tid / GW;
  constexpr bool BF = (HMODE & kHalfBf16) != 0;

  TwiddleStage<K> tws;
  tws.request(tid, NT);

  float4 xr[NRI][NSEG];
  // rows past the end are read from the last row (a valid address) and zeroed
  auto request = [&](int tile) {
#pragma unroll
    for (int i = 0; i < NRI; ++i) {
      const long long rid = (long long)tile * 2 * P + r0 + i * RSTEP;
      const bool ok = rid < nrows;
      const long long b = row_base(map, ok ? rid : nrows - 1);
#pragma unroll
      for (int seg = 0; seg < NSEG; ++seg) {
        const int n = 4 * (seg * GW + gl);
        float4 v;
        if constexpr (HMODE & kHalfRows) v = load_half4<BF>(reinterpret_cast<const unsigned short*>(in) + b + n);
        else v = *reinterpret_cast<const float4*>(in + b + n);
        xr[i][seg] = ok ? v : make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
  };
  int tile = blockIdx.x;
  if (tile < ntiles) request(tile);
  tws.store(L.tw, tid, NT);

  for (; tile < ntiles; tile += gridDim.x) {
    // 8 lanes along the row times 8 rows per wave-store: every LDS bank gets exactly two lanes
    // (see the row loader of rfft_kernel)
#pragma unroll
    for (int i = 0; i < NRI; ++i) {
      float* zrow = reinterpret_cast<float*>(L.z) + r0 + i * RSTEP;
#pragma unroll
      for (int seg = 0; seg < NSEG; ++seg) {
        float* zd = zrow + 2 * (4 * (seg * GW + gl)) * PP;
        zd[0] = xr[i][seg].x;
        zd[2 * PP] = xr[i][seg].y;
        zd[4 * PP] = xr[i][seg].z;
        zd[6 * PP] = xr[i][seg].w;
      }
    }
    __syncthreads();
    if (tile + (int)gridDim.x < ntiles) request(tile + gridDim.x);
    const int col = tid & (P - 1), t = tid >> lgP, TT = NT >> lgP;
    fft_lds_pass1<K, false>(L.z, PP, col, t, TT, L.tw);
    __syncthreads();
    fft_lds_pass2_inplace<K, false>(L.z, PP, col, t, TT);
    __syncthreads();
    rfft_store_tile<K, HMODE>(L.z, P, lgP, tid, NT, (long long)tile * 2 * P, nrows, out, out_fstride, scale, conj);
    __syncthreads();   // the tile is free for the next rows
  }
}

// -------------------------------------------------------------------------------------
// Inverse real FFT of rows with epilogue:  out_row[n] = psi(scale * z[n] + bias[blk*K + n]),
// blk = rid / bias_div (the output block row / channel block of the row).
// The spectrum may come as `nparts` partial sums (split-K GEMM), `part_stride` elements apart;
// they are added in index order, so the result does not depend on scheduling.
template <int K, bool ROWS_FAST, int HMODE = 0>
__global__ void irfft_kernel(const float2* __restrict__ in, float* __restrict__ out, RowMap map,
                             long long nrows, long long in_fstride, int P, float scale,
                             const float* __restrict__ bias, long long bias_div, int relu,
                             int nparts, long long part_stride) {
  extern __shared__ float smem[];
  const int PP = P + 1;
  const int lgP = __ffs(P) - 1;
  TileLds L = carve_tile<K>(smem, P);
  const long long t0 = (long long)blockIdx.x * 2 * P;
  const int tid = threadIdx.x, NT = blockDim.x;

  TwiddleStage<K> tws;
  tws.request(tid, NT);
  // build Z = Ya + i*Yb on all K bins from the two half spectra (Hermitian symmetry)
  constexpr int NF = K / 2 + 1;
  {
    // a thread keeps its column pair; its bin advances by NT/P per step
    const int pr = tid & (P - 1), fstep = NT >> lgP;
    const long long rid = t0 + 2 * pr;
    const bool ok0 = rid < nrows, ok1 = rid + 1 < nrows;
    static_assert(HMODE == 0 || K >= 4, "half-width storage: K >= 4 only");
    long long s = (long long)(tid >> lgP) * in_fstride + rid;
    const long long sstep = (long long)fstep * in_fstride;
    auto bin = [&](long long e, bool ok) -> float2 {
      if (!ok) return make_float2(0.f, 0.f);
      if constexpr (HMODE & kHalfSpectra) return unpack_pair16<(HMODE & kHalfBf16) != 0>(reinterpret_cast<const unsigned*>(in)[e]);
      else return in[e];
    };
    // both bins of a column pair in one access (see the store of rfft_kernel)
    constexpr int PAIRB = (HMODE & kHalfSpectra) ? 8 : 16;
    const bool whole = t0 + 2 * P <= nrows && ((in_fstride | part_stride) & 1) == 0 &&
                       (reinterpret_cast<unsigned long long>(in) & (PAIRB - 1)) == 0;
    auto bin2 = [&](long long e) -> float4 {
      if constexpr (HMODE & kHalfSpectra) {
        const uint2 raw = *reinterpret_cast<const uint2*>(reinterpret_cast<const unsigned*>(in) + e);
        const float2 a = unpack_pair16<(HMODE & kHalfBf16) != 0>(raw.x), b = unpack_pair16<(HMODE & kHalfBf16) != 0>(raw.y);
        return make_float4(a.x, a.y, b.x, b.y);
      } else {
        return *reinterpret_cast<const float4*>(in + e);
      }
    };
    if (whole) {
      // GB bins at a time: their loads (and those of every further partial spectrum) are issued
      // together, so that a thread waits for memory once per group and part, not once per load.
      // Bins past the end reload the last one and are dropped.
      constexpr int GB = 8;
      for (int f0 = tid >> lgP; f0 < NF; f0 += GB * fstep) {
        long long e[GB];
        float4 y[GB];
#pragma unroll
        for (int g = 0; g < GB; ++g) e[g] = (long long)min(f0 + g * fstep, NF - 1) * in_fstride + rid;
#pragma unroll
        for (int g = 0; g < GB; ++g) y[g] = bin2(e[g]);
        for (int part = 1; part < nparts; ++part) {
          float4 v[GB];
#pragma unroll
          for (int g = 0; g < GB; ++g) v[g] = bin2(e[g] + part * part_stride);
#pragma unroll
          for (int g = 0; g < GB; ++g) { y[g].x += v[g].x; y[g].y += v[g].y; y[g].z += v[g].z; y[g].w += v[g].w; }
        }
#pragma unroll
        for (int g = 0; g < GB; ++g) {
          const int f = f0 + g * fstep;
          if (f >= NF) break;
          if (f == 0 || 2 * f == K) {
            L.z[f * PP + pr] = make_float2(y[g].x, y[g].z);
          } else {
            L.z[f * PP + pr] = make_float2(y[g].x - y[g].w, y[g].y + y[g].z);
            L.z[(K - f) * PP + pr] = make_float2(y[g].x + y[g].w, y[g].z - y[g].y);
          }
        }
      }
    } else {
#pragma unroll 4
      for (int f = tid >> lgP; f < NF; f += fstep, s += sstep) {
        float2 ya = bin(s, ok0);
        float2 yb = bin(s + 1, ok1);
        // partial sums: loads four parts ahead, additions in index order
#pragma unroll 4
        for (int part = 1; part < nparts; ++part) {
          const long long sp = s + part * part_stride;
          const float2 pa = bin(sp, ok0);
          const float2 pb = bin(sp + 1, ok1);
          ya.x += pa.x; ya.y += pa.y;
          yb.x += pb.x; yb.y += pb.y;
        }
        if (f == 0 || 2 * f == K) {            // DC and Nyquist bins of a real signal are real
          L.z[f * PP + pr] = make_float2(ya.x, yb.x);
        } else {
          L.z[f * PP + pr] = make_float2(ya.x - yb.y, ya.y + yb.x);
          L.z[(K - f) * PP + pr] = make_float2(ya.x + yb.y, yb.x - ya.y);
        }
      }
    }
  }
  for (int r = tid; r < 2 * P; r += NT) {
    long long rid = t0 + r;
    bool ok = rid < nrows;
    L.rbase[r] = ok ? row_base(map, rid) : -1;
    L.rblk[r] = ok ? int((unsigned)rid / (unsigned)bias_div) : 0;   // both fit 32 bits (host check)
  }
  tws.store(L.tw, tid, NT);
  __syncthreads();

  const int col = tid & (P - 1), t = tid >> lgP, TT = NT >> lgP;
  fft_lds_pass1<K, true>(L.z, PP, col, t, TT, L.tw);
  __syncthreads();
  fft_lds_pass2_inplace<K, true>(L.z, PP, col, t, TT);
  __syncthreads();

  if constexpr (!ROWS_FAST && K >= 4 && is_pow2_c(K)) {
    // contiguous rows: float4 stores; a thread keeps its position n in the row, its row index
    // advances by NT/(K/4) per step (NT is a multiple of K/4)
    const int n = 4 * (tid % (K / 4)), rstep = NT / (K / 4);
    const float* z0 = reinterpret_cast<const float*>(L.z) + 2 * fft_pos<K>(n + 0) * PP;
    const float* z1 = reinterpret_cast<const float*>(L.z) + 2 * fft_pos<K>(n + 1) * PP;
    const float* z2 = reinterpret_cast<const float*>(L.z) + 2 * fft_pos<K>(n + 2) * PP;
    const float* z3 = reinterpret_cast<const float*>(L.z) + 2 * fft_pos<K>(n + 3) * PP;
#pragma unroll 4
    for (int row = tid / (K / 4); row < 2 * P; row += rstep) {
      long long b = L.rbase[row];
      if (b < 0) continue;
      const int c = 2 * (row >> 1) + (row & 1);
      float4 v = make_float4(z0[c] * scale, z1[c] * scale, z2[c] * scale, z3[c] * scale);
      if (bias) {
        const float4 bb = *reinterpret_cast<const float4*>(bias + (long long)L.rblk[row] * K + n);
        v.x += bb.x; v.y += bb.y; v.z += bb.z; v.w += bb.w;
      }
      if (relu) { v.x = fmaxf(v.x, 0.f); v.y = fmaxf(v.y, 0.f); v.z = fmaxf(v.z, 0.f); v.w = fmaxf(v.w, 0.f); }
      if constexpr (HMODE & kHalfRows) store_half4<(HMODE & kHalfBf16) != 0>(reinterpret_cast<unsigned short*>(out) + b + n, v);
      else *reinterpret_cast<float4*>(out + b + n) = v;
    }
  } else if constexpr (!ROWS_FAST && K % 4 == 0) {
    // the same for block sizes that are not powers of two
    constexpr int Q4 = K / 4;
#pragma unroll 2
    for (int idx = tid; idx < 2 * P * Q4; idx += NT) {
      const int row = idx / Q4, n = 4 * (idx - row * Q4);
      const long long b = L.rbase[row];
      if (b < 0) continue;
      const float* zc = reinterpret_cast<const float*>(L.z) + row;
      float4 v = make_float4(zc[2 * fft_pos<K>(n + 0) * PP] * scale, zc[2 * fft_pos<K>(n + 1) * PP] * scale,
                             zc[2 * fft_pos<K>(n + 2) * PP] * scale, zc[2 * fft_pos<K>(n + 3) * PP] * scale);
      if (bias) {
        const float4 bb = *reinterpret_cast<const float4*>(bias + (long long)L.rblk[row] * K + n);
        v.x += bb.x; v.y += bb.y; v.z += bb.z; v.w += bb.w;
      }
      if (relu) { v.x = fmaxf(v.x, 0.f); v.y = fmaxf(v.y, 0.f); v.z = fmaxf(v.z, 0.f); v.w = fmaxf(v.w, 0.f); }
      if constexpr (HMODE & kHalfRows) store_half4<(HMODE & kHalfBf16) != 0>(reinterpret_cast<unsigned short*>(out) + b + n, v);
      else *reinterpret_cast<float4*>(out + b + n) = v;
    }
  } else if (ROWS_FAST && map.quad) {
    // 4 rows per 16-byte store (see the loader of rfft_kernel); a group of 4 rows lies inside
    // one bias block
    const int nq = P >> 1;
#pragma unroll 4
    for (int idx = tid; idx < nq * K; idx += NT) {
      const int qd = idx & (nq - 1), n = idx >> (lgP - 1);
      long long b = L.rbase[4 * qd];
      if (b < 0) continue;
      const float2* zs = L.z + fft_pos<K>(n) * PP + 2 * qd;
      const float2 u0 = zs[0], u1 = zs[1];
      float4 v = make_float4(u0.x * scale, u0.y * scale, u1.x * scale, u1.y * scale);
      if (bias) {
        const float bb = bias[(long long)L.rblk[4 * qd] * K + n];
        v.x += bb; v.y += bb; v.z += bb; v.w += bb;
      }
      if (relu) { v.x = fmaxf(v.x, 0.f); v.y = fmaxf(v.y, 0.f); v.z = fmaxf(v.z, 0.f); v.w = fmaxf(v.w, 0.f); }
      if constexpr (HMODE & kHalfRows) store_half4<(HMODE & kHalfBf16) != 0>(reinterpret_cast<unsigned short*>(out) + b + n * map.es, v);
      else *reinterpret_cast<float4*>(out + b + n * map.es) = v;
    }
  } else {
#pragma unroll 4
    for (int idx = tid; idx < 2 * P * K; idx += NT) {
      int row, n;
      if (ROWS_FAST) { row = idx & (2 * P - 1); n = idx >> (lgP + 1); }
      else { row = idx / K; n = idx % K; }
      long long b = L.rbase[row];
      if (b < 0) continue;
      float v = lds_get(L.z, fft_pos<K>(n) * PP + (row >> 1), row & 1) * scale;
      if (bias) v += bias[(long long)L.rblk[row] * K + n];
      if (relu) v = fmaxf(v, 0.f);
      if constexpr (HMODE & kHalfRows)
        reinterpret_cast<unsigned short*>(out)[b + n * map.es] = (unsigned short)(pack_pair16<(HMODE & kHalfBf16) != 0>(v, 0.f) & 0xffffu);
      else out[b + n * map.es] = v;
    }
  }
}

// -------------------------------------------------------------------------------------
// The inverse transform for long runs of contiguous rows (the outputs of a large FC layer), in
// the streaming form of rfft_stream_kernel: a workgroup walks over tiles of 4096 / K column pairs
// and requests the spectra of its next tile before it transforms the current one (in irfft_kernel
// a workgroup waits 9,500 of its 24,900 cycles for its spectra at 65,536 rows of 256, and for the
// roots before that).  A thread keeps its column pair and takes bins f0, f0 + K/16, ..., nine of
// them (the ninth, bin K/2, only for f0 = 0), both rows of the pair in one 16-byte load.
// 256 threads; one spectrum (no partial sums); an even number of rows, an even plane pitch and a
// 16-byte aligned input (whole pairs); contiguous 16-byte aligned output rows; 32 <= K <= 256.
// HMODE: 0, or 16-bit spectra and rows (kHalfSpectra | kHalfRows, with kHalfBf16 for bfloat16).
template <int K, int HMODE = 0>
__global__ __launch_bounds__(256) void irfft_stream_kernel(const float2* __restrict__ in, float* __restrict__ out, RowMap map,
                                                           long long nrows, long long in_fstride, int ntiles, float scale,
                                                           const float* __restrict__ bias, long long bias_div, int relu) {
  static_assert(is_pow2_c(K) && K >= 32 && K <= 256, "block sizes of the streaming transform");
  static_assert(HMODE == 0 || (HMODE & (kHalfSpectra | kHalfRows)) == (kHalfSpectra | kHalfRows), "16-bit spectra come with 16-bit rows");
  constexpr int P = 4096 / K, PP = P + 1, NT = 256, lgP = ilog2(P), NF = K / 2 + 1, FSTEP = NT / P, NG = 8;
  static_assert(NG * FSTEP == K / 2 && NF == K / 2 + 1, "eight bins per thread, and bin K/2 for the threads of bin 0");
  constexpr bool HALF = HMODE != 0, BF = (HMODE & kHalfBf16) != 0;
  extern __shared__ float smem[];
  TileLds L = carve_tile<K>(smem, P);
  const int tid = threadIdx.x, pr = tid & (P - 1), f0 = tid >> lgP;

  TwiddleStage<K> tws;
  tws.request(tid, NT);

  // the two rows of a pair at one bin: 16 bytes of fp32 spectra, 8 bytes of 16-bit ones
  using PairT = typename std::conditional<HALF, uint2, float4>::type;
  PairT y[NG + 1];
  auto pair_at = [&](long long e) -> PairT {
    if constexpr (HALF) return *reinterpret_cast<const uint2*>(reinterpret_cast<const unsigned*>(in) + e);
    else return *reinterpret_cast<const float4*>(in + e);
  };
  auto pair_values = [&](const PairT& v) -> float4 {
    if constexpr (HALF) {
      const float2 a = unpack_pair16<BF>(v.x), b = unpack_pair16<BF>(v.y);
      return make_float4(a.x, a.y, b.x, b.y);
    } else {
      return v;
    }
  };
  // pairs past the end reload the last pair (a valid address) and are zeroed when they are written to LDS
  auto request = [&](int tile) {
    const long long rid = (long long)tile * 2 * P + 2 * pr;
    const long long e0 = (rid < nrows ? rid : nrows - 2) + (long long)f0 * in_fstride;
#pragma unroll
    for (int g = 0; g < NG; ++g) y[g] = pair_at(e0 + (long long)(g * FSTEP) * in_fstride);
    y[NG] = PairT{};
    if (f0 == 0) y[NG] = pair_at(e0 + (long long)(K / 2) * in_fstride);
  };
  int tile = blockIdx.x;
  if (tile < ntiles) request(tile);
  tws.store(L.tw, tid, NT);

  for (; tile < ntiles; tile += gridDim.x) {
    const long long t0 = (long long)tile * 2 * P;
    if (tid < 2 * P) {
      const long long rid = t0 + tid;
      const bool ok = rid < nrows;
      L.rbase[tid] = ok ? row_base(map, rid) : -1;
      L.rblk[tid] = ok ? int((unsigned)rid / (unsigned)bias_div) : 0;   // both fit 32 bits (host check)
    }
    // Z = Ya + i*Yb on all K bins from the two half spectra (Hermitian symmetry; bins 0 and K/2 are real)
    const bool ok = t0 + 2 * pr < nrows;
#pragma unroll
    for (int g = 0; g <= NG; ++g) {
      const int f = f0 + g * FSTEP;
      const float4 v = ok ? pair_values(y[g]) : make_float4(0.f, 0.f, 0.f, 0.f);
      if (g == NG) {
        if (f0 == 0) L.z[(K / 2) * PP + pr] = make_float2(v.x, v.z);
      } else if (g == 0 && f0 == 0) {
        L.z[pr] = make_float2(v.x, v.z);
      } else {
        L.z[f * PP + pr] = make_float2(v.x - v.w, v.y + v.z);
        L.z[(K - f) * PP + pr] = make_float2(v.x + v.w, v.z - v.y);
      }
    }
    __syncthreads();
    if (tile + (int)gridDim.x < ntiles) request(tile + gridDim.x);
    const int col = tid & (P - 1), t = tid >> lgP, TT = NT >> lgP;
    fft_lds_pass1<K, true>(L.z, PP, col, t, TT, L.tw);
    __syncthreads();
    fft_lds_pass2_inplace<K, true>(L.z, PP, col, t, TT);
    __syncthreads();
    // float4 stores: a thread keeps its position n in the row, its row advances by NT/(K/4) per step
    {
      const int n = 4 * (tid % (K / 4)), rstep = NT / (K / 4);
      const float* z0 = reinterpret_cast<const float*>(L.z) + 2 * fft_pos<K>(n + 0) * PP;
      const float* z1 = reinterpret_cast<const float*>(L.z) + 2 * fft_pos<K>(n + 1) * PP;
      const float* z2 = reinterpret_cast<const float*>(L.z) + 2 * fft_pos<K>(n + 2) * PP;
      const float* z3 = reinterpret_cast<const float*>(L.z) + 2 * fft_pos<K>(n + 3) * PP;
#pragma unroll 4
      for (int row = tid / (K / 4); row < 2 * P; row += rstep) {
        const long long b = L.rbase[row];
        if (b < 0) continue;
        const int c = 2 * (row >> 1) + (row & 1);
        float4 v = make_float4(z0[c] * scale, z1[c] * scale, z2[c] * scale, z3[c] * scale);
        if (bias) {
          const float4 bb = *reinterpret_cast<const float4*>(bias + (long long)L.rblk[row] * K + n);
          v.x += bb.x; v.y += bb.y; v.z += bb.z; v.w += bb.w;
        }
        if (relu) { v.x = fmaxf(v.x, 0.f); v.y = fmaxf(v.y, 0.f); v.z = fmaxf(v.z, 0.f); v.w = fmaxf(v.w, 0.f); }
        if constexpr (HALF) store_half4<BF>(reinterpret_cast<unsigned short*>(out) + b + n, v);
        else *reinterpret_cast<float4*>(out + b + n) = v;
      }
    }
    __syncthreads();   // the tile and the row tables are free for the next spectra
  }
}

// -------------------------------------------------------------------------------------
// Per-frequency complex GEMM on the fp32 MFMA units, one wave per output tile:
//   C[f][m][n] = sum_k A[f][k][m] * B[f][k][n]        (B conjugated if CONJ_B)
// A is stored with m fastest, B and C with n fastest, so every operand load is one
// contiguous run per k.  A complex product is three real MFMA accumulations (see below).
// TILE = 32 uses v_mfma_f32_32x32x2_f32, TILE = 16 uses v_mfma_f32_16x16x4_f32.
// Operand loads run one group of U k-steps ahead of the matrix instructions.
// Split-K: blockIdx.x = ks*ntn + (tile along n); slice ks reduces k in [ks*kchunk, (ks+1)*kchunk)
// and writes its partial sums to C + ks*part_stride (summed later in a fixed order).
template <int TILE, bool CONJ_B>
__global__ __launch_bounds__(64) void cgemm_kernel(const float2* __restrict__ A,
                                                   const float2* __restrict__ B,
                                                   float2* __restrict__ C, int M, int N, int Kd,
                                                   long long sA, long long sB, long long sC,
                                                   int ntn, int kchunk, long long part_stride) {
  constexpr int KS = 64 / TILE;           // k values per MFMA: 2 or 4
  constexpr int NACC = TILE * TILE / 64;  // accumulator registers per lane: 16 or 4
  constexpr int U = 8;                    // k-steps per group
  typedef float accv __attribute__((ext_vector_type(NACC)));
  const int lane = threadIdx.x;
  const int ks = blockIdx.x / ntn;
  const int f = blockIdx.z, m0 = blockIdx.y * TILE, n0 = (blockIdx.x - ks * ntn) * TILE;
  const int kbeg = ks * kchunk, kend = min(Kd, kbeg + kchunk);
  A += f * sA;
  B += f * sB;
  C += f * sC + ks * part_stride;
  const int kk = lane / TILE, mm = lane % TILE;
  const int am = min(m0 + mm, M - 1);
  const int bn = min(n0 + mm, N - 1);
  // Three real products per complex one instead of four (Gauss):
  //   K1 = (ar + ai) br,  K2 = ar (bi - br),  K3 = ai (br + bi):  Re = K1 - K3,  Im = K1 + K2
  // (conj(b): bi -> -bi).  The three operand sums are vector additions per loaded value; the
  // matrix cores, which bound this kernel, do a quarter less work.
  accv acc1, acc2, acc3;
#pragma unroll
  for (int r = 0; r < NACC; ++r) { acc1[r] = 0.f; acc2[r] = 0.f; acc3[r] = 0.f; }

  float2 a[U], b[U], an[U], bn2[U];
  auto load_group = [&](int k0, float2 (&ga)[U], float2 (&gb)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int kidx = k0 + u * KS + kk;
      int kc = min(kidx, kend - 1);
      float2 va = A[(long long)kc * M + am];
      float2 vb = B[(long long)kc * N + bn];
      if (kidx >= kend) { va = make_float2(0.f, 0.f); vb = make_float2(0.f, 0.f); }
      ga[u] = va;
      gb[u] = vb;
    }
  };
  load_group(kbeg, a, b);
  for (int k0 = kbeg; k0 < kend; k0 += U * KS) {
    if (k0 + U * KS < kend) load_group(k0 + U * KS, an, bn2);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float bi = CONJ_B ? -b[u].y : b[u].y;
      const float a_s = a[u].x + a[u].y, b_d = bi - b[u].x, b_s = b[u].x + bi;
      if constexpr (TILE == 32) {
        acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a_s, b[u].x, acc1, 0, 0, 0);
        acc2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u].x, b_d, acc2, 0, 0, 0);
        acc3 = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u].y, b_s, acc3, 0, 0, 0);
      } else {
        acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a_s, b[u].x, acc1, 0, 0, 0);
        acc2 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u].x, b_d, acc2, 0, 0, 0);
        acc3 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u].y, b_s, acc3, 0, 0, 0);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) { a[u] = an[u]; b[u] = bn2[u]; }
  }

  // accumulator layout: column = lane % TILE; rows in groups of 4
  const int j = n0 + lane % TILE;
#pragma unroll
  for (int r = 0; r < NACC; ++r) {
    int i;
    if constexpr (TILE == 32) i = 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
    else i = 4 * (lane / 16) + r;
    i += m0;
    if (i < M && j < N) C[(long long)i * N + j] = make_float2(acc1[r] - acc3[r], acc1[r] + acc2[r]);
  }
}

// -------------------------------------------------------------------------------------
// CONV contraction, one thread per (frequency, image, output pixel), IT output channel
// blocks at a time:
//   Yh[f][i][n][ho][wo] = sum_{dh,dw,j} What[dh*r+dw][f][j][i] * Xh[f][j][n][ho*stride+dh-pad][wo*stride+dw-pad]
// with zero spectra outside the image (the channel FFT of a zero pixel is zero, so the
// spatial shift is taken after the transform and every input pixel is transformed once).
// flip: offset (dh, dw) takes the weights of offset (r-1-dh, r-1-dw) - the reflected filter of
// backward-data, whose operand is the conjugated, transposed section and whose padding is r-1-pad.
// stride: the filter moves `stride` input pixels per output pixel (tap = ho*stride + dh - pad).
// dil: the input grid is the H x W one with dil-1 zeros inserted between its pixels (a tap u
// reads input pixel u/dil when dil divides u, zero otherwise) - backward-data of a strided layer.
template <int IT>
__global__ void conv_contract_kernel(const float2* __restrict__ What, const float2* __restrict__ Xh,
                                     float2* __restrict__ Yh, int p, int q, int NF, int Nimg, int H,
                                     int W, int Ho, int Wo, int r, int pad, int flip, int stride, int dil) {
  const long long npix = (long long)Nimg * Ho * Wo;
  const long long opix = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (opix >= npix) return;
  const int f = blockIdx.y, i0 = blockIdx.z * IT;
  const int n = int(opix / (Ho * Wo)), rem = int(opix % (Ho * Wo));
  const int ho = rem / Wo, wo = rem % Wo;
  float2 acc[IT];
#pragma unroll
  for (int ii = 0; ii < IT; ++ii) acc[ii] = make_float2(0.f, 0.f);
  for (int dh = 0; dh < r; ++dh) {
    for (int dw = 0; dw < r; ++dw) {
      int hi = ho * stride + dh - pad, wi = wo * stride + dw - pad;
      bool inb = hi >= 0 && wi >= 0;
      if (dil > 1) {
        inb = inb && hi % dil == 0 && wi % dil == 0;
        hi /= dil;
        wi /= dil;
      }
      inb = inb && hi < H && wi < W;
      const int g = flip ? r * r - 1 - (dh * r + dw) : dh * r + dw;
      const float2* wg = What + ((long long)g * NF + f) * q * p;
      for (int j = 0; j < q; ++j) {
        float2 xv = make_float2(0.f, 0.f);
        if (inb) xv = Xh[(((long long)f * q + j) * Nimg + n) * H * W + hi * W + wi];
#pragma unroll
        for (int ii = 0; ii < IT; ++ii) {
          float2 wv = wg[j * p + min(i0 + ii, p - 1)];
          acc[ii].x += wv.x * xv.x - wv.y * xv.y;
          acc[ii].y += wv.x * xv.y + wv.y * xv.x;
        }
      }
    }
  }
#pragma unroll
  for (int ii = 0; ii < IT; ++ii)
    if (i0 + ii < p) Yh[(((long long)f * p + i0 + ii) * Nimg + n) * Ho * Wo + rem] = acc[ii];
}

}  // namespace circ
