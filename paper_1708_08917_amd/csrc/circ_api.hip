// C ABI of the block-circulant layer library: argument checks, workspace carving,
// launch planning.  Every operation of the layers runs in the kernels of circ_kernels.h.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>
#include <mutex>

#include "../../include/circ.h"
#include "circ_kernels.h"
#include "circ_dft.h"
#include "circ_gemm.h"
#include "circ_gemm_split.h"
#include "circ_fused.h"
#include "circ_gemv.h"
#include "circ_conv_fused.h"
#include "circ_conv_bwd.h"
#include "circ_update.h"
#include "circ_half.h"
#include "circ_pool.h"

namespace {

using namespace circ;

constexpr int kMinK = 1, kMaxK = 512;

inline bool is_pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }
inline bool valid_k(int k) { return k >= kMinK && k <= kMaxK; }
// Block sizes served by the radix-2 kernels.
inline bool radix2_k(int k) { return is_pow2(k) && k >= 2; }
// Block sizes 3 * 2^a, 5 * 2^a and 25 * 2^a (multiples of 4): the same kernels with mixed-radix
// sub-transforms in registers (96 and 384 are the channel counts of AlexNet-style CONV layers).
// Every other size takes the transforms by their definition.
inline bool mixed_k(int k) {
  switch (k) {
    case 12: case 24: case 48: case 96: case 192: case 384:
    case 20: case 40: case 80: case 160: case 320:
    case 100: case 200: case 400: return true;
    default: return false;
  }
}
// Block sizes served by the batch <= 2 streaming kernel.
inline bool gemv_k(int k) { return is_pow2(k) && k >= 4; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline long long cdiv(long long a, long long b) { return (a + b - 1) / b; }

inline size_t spectrum_elems(int k, long long rows) { return size_t(k / 2 + 1) * size_t(rows); }

// Activation spectra in the FC workspace are stored [f][row], densely.
inline long long ws_fstride(long long rows) { return rows; }
inline size_t ws_spectrum_elems(int k, long long rows) { return size_t(k / 2 + 1) * size_t(ws_fstride(rows)); }

// Spectra blob: section 0 = forward operand [g][f][j][i] (i fastest), section 1 =
// backward operand [g][f][i][j] (j fastest, conjugated).  Both carry the 1/k of the IFFT.
inline size_t spectra_section_elems(int n_grids, int p, int q, int k) {
  return size_t(n_grids) * spectrum_elems(k, (long long)p * q);
}

// Output block rows per workgroup of the fused kernel for block size k (0: not fused).
inline int fused_it(int k) { return (!is_pow2(k) || k < 32 || k > 256) ? 0 : (k == 32 ? 16 : 8); }
// Section 2 (FC only, 32 <= k <= 256): the operand order of the fused forward kernel,
// zero-padded to whole tiles: igp groups of 4 block rows, q2p pairs of block columns.
inline int fused_igp(int p, int k) { return int(cdiv(p, fused_it(k))) * fused_it(k) / 4; }
inline int fused_q2p(int q, int k) { const int jc = 4096 / k; return int(cdiv(q, jc)) * (jc / 2); }
inline size_t fused_section_elems(int n_grids, int p, int q, int k) {   // in float4 units
  if (n_grids != 1 || fused_it(k) == 0) return 0;
  return size_t(fused_igp(p, k)) * fused_q2p(q, k) * (k / 32) * 64;
}

// Section 3 (FC only, k >= 4): [i][j][slot] order of the batch <= 2 kernel.
inline size_t gemv_section_elems(int n_grids, int p, int q, int k) {      // in float2 units
  if (n_grids != 1 || !gemv_k(k)) return 0;
  return size_t(p) * q * (k / 2);
}

// Fused CONV kernel: built for k = 64, 3x3 filters, q in {1, 2, 3, 4, 6, 8} input channel blocks and
// up to 16 output channel blocks.  ncombo = (slot groups) x (groups of 4 output blocks, rounded
// up to a power of two) must divide the 8 waves of a workgroup.
inline int conv_fused_ncombo(int p, int q, int k, int r) {
  if (k != 64 || r != 3 || !(q == 1 || q == 2 || q == 3 || q == 4 || q == 6 || q == 8)) return 0;
  int ig = 1;
  while (ig * 4 < p) ig *= 2;
  const int ncombo = (k / 32) * ig;
  return ncombo <= 8 ? ncombo : 0;
}
// Section 2 of a CONV blob (n_grids = r*r > 1): operand order of the fused CONV kernel.
inline size_t conv_section_elems(int n_grids, int p, int q, int k) {      // in float2 units
  int r = 1;
  while (r * r < n_grids) ++r;
  if (n_grids == 1 || r * r != n_grids) return 0;
  return size_t(n_grids) * q * conv_fused_ncombo(p, q, k, r) * 64;
}

// Byte offsets of the sections of a spectra blob.  FC (n_grids == 1): unfused forward and
// backward operands, then the fused / batch<=2 operand orders for the forward pass (p x q grid)
// and for backward-data, which is the same computation on the transposed, conjugated grid
// (q x p).  CONV: unfused operands, then the fused CONV order.
struct BlobLayout {
  size_t fwd, bwd, fused_fwd, gemv_fwd, fused_bwd, gemv_bwd, conv, conv_bwd, total;
};
inline BlobLayout blob_layout(int n_grids, int p, int q, int k) {
  BlobLayout b;
  const size_t sec = align_up(spectra_section_elems(n_grids, p, q, k) * sizeof(float2), 256);
  size_t off = 0;
  b.fwd = off; off += sec;
  b.bwd = off; off += sec;
  b.fused_fwd = off; off += align_up(fused_section_elems(n_grids, p, q, k) * sizeof(float4), 256);
  b.gemv_fwd = off; off += align_up(gemv_section_elems(n_grids, p, q, k) * sizeof(float2), 256);
  b.fused_bwd = off; off += align_up(fused_section_elems(n_grids, q, p, k) * sizeof(float4), 256);
  b.gemv_bwd = off; off += align_up(gemv_section_elems(n_grids, q, p, k) * sizeof(float2), 256);
  b.conv = off; off += align_up(conv_section_elems(n_grids, p, q, k) * sizeof(float2), 256);
  b.conv_bwd = off; off += align_up(conv_section_elems(n_grids, q, p, k) * sizeof(float2), 256);
  b.total = off;
  return b;
}
template <class T>
inline T* blob_at(void* blob, size_t off) { return reinterpret_cast<T*>(static_cast<char*>(blob) + off); }
template <class T>
inline const T* blob_at(const void* blob, size_t off) { return reinterpret_cast<const T*>(static_cast<const char*>(blob) + off); }

struct FftPlan { int P, NT; size_t lds; };

// P column pairs per block, NT threads.  Small problems get small tiles so that the
// launch still covers the chip; the tile must fit comfortably in LDS.
constexpr size_t kFftMaxLdsBytes = 40 * 1024;   // LDS tile limit of the unfused transform kernels
FftPlan plan_fft(int K, long long nrows) {
  int R2 = radix2_of(K);
  int P = 64;
  while (P > 8 && fft_tile_lds_bytes(K, P) > kFftMaxLdsBytes) P >>= 1;
  long long pairs = cdiv(nrows, 2);
  while (P > 8 && cdiv(pairs, P) < 512) P >>= 1;
  int TT = R2;
  if (is_pow2(K)) {
    if (P * TT > 256) TT = 256 / P;
  } else {
    // a divisor of the R2 sub-transforms of the first pass, so that no round of it is half empty
    while (P * TT > 512 || R2 % TT != 0) --TT;
  }
  if (TT < 1) TT = 1;
  int NT = P * TT;
  if (NT < 64) NT = 64;
  // a launch that leaves CUs idle is bound by the latency of its loads and stores, which all
  // threads share (the butterflies occupy R2 threads per column, the others skip them)
  if (cdiv(pairs, P) <= 256 && NT < 256) NT = 256;
  if (is_pow2(K) && NT < K / 4) NT = K / 4;   // the row loaders keep one float4 column per thread
  return FftPlan{P, NT, fft_tile_lds_bytes(K, P)};
}

// Long runs of contiguous rows take the streaming form of the transform (rfft_stream_kernel: tiles of
// 4096 / K column pairs, at most four workgroups per CU walking over them) once there is at least
// one tile per CU; 65,536 rows of 256: 28.8 -> 23.7 us, 18,432 rows of 128: 7.4 -> 6.5 us.
constexpr long long kStreamMinTiles = 256, kStreamMaxWorkgroups = 1024;
template <int K>
constexpr bool stream_k() { return is_pow2_c(K) && K >= 32 && K <= 256; }
template <int K, int HMODE>
bool launch_rfft_stream(const float* in, float2* out, const RowMap& map, long long nrows, long long out_fstride, float scale,
                        int conj, hipStream_t s) {
  if constexpr (stream_k<K>()) {
    constexpr int P = 4096 / K;
    const long long ntiles = cdiv(nrows, 2 * P);
    if (ntiles < kStreamMinTiles || ntiles > (1ll << 31) - 1) return false;
    const unsigned grid = unsigned(ntiles < kStreamMaxWorkgroups ? ntiles : kStreamMaxWorkgroups);
    hipLaunchKernelGGL((rfft_stream_kernel<K, HMODE>), dim3(grid), dim3(256), fft_tile_lds_bytes(K, P), s, in, out, map, nrows,
                       out_fstride, int(ntiles), scale, conj);
    return true;
  } else {
    return false;
  }
}

template <int K>
hipError_t launch_rfft_k(bool rows_fast, const float* in, float2* out, const RowMap& map, long long nrows,
                         long long out_fstride, int n_grids, long long in_gstride, long long out_gstride,
                         float scale, int conj, hipStream_t s) {
  if (!rows_fast && n_grids == 1 && launch_rfft_stream<K, 0>(in, out, map, nrows, out_fstride, scale, conj, s))
    return hipGetLastError();
  FftPlan pl = plan_fft(K, nrows);
  dim3 grid((unsigned)cdiv(nrows, 2 * pl.P), (unsigned)n_grids);
  if (rows_fast)
    hipLaunchKernelGGL((rfft_kernel<K, true>), grid, dim3(pl.NT), pl.lds, s, in, out, map, nrows, out_fstride,
                       in_gstride, out_gstride, pl.P, scale, conj);
  else
    hipLaunchKernelGGL((rfft_kernel<K, false>), grid, dim3(pl.NT), pl.lds, s, in, out, map, nrows, out_fstride,
                       in_gstride, out_gstride, pl.P, scale, conj);
  return hipGetLastError();
}

template <int K>
hipError_t launch_irfft_k(bool rows_fast, const float2* in, float* out, const RowMap& map, long long nrows,
                          long long in_fstride, float scale, const float* bias, long long bias_div, int relu,
                          int nparts, long long part_stride, hipStream_t s) {
  if constexpr (stream_k<K>()) {
    // long runs of contiguous rows: the streaming form (65,536 rows of 256)
    constexpr int P = 4096 / K;
    const long long ntiles = cdiv(nrows, 2 * P);
    if (!rows_fast && nparts == 1 && ntiles >= kStreamMinTiles && ntiles <= (1ll << 31) - 1 && (nrows & 1) == 0 &&
        (in_fstride & 1) == 0 && aligned16(in)) {
      const unsigned grid = unsigned(ntiles < kStreamMaxWorkgroups ? ntiles : kStreamMaxWorkgroups);
      hipLaunchKernelGGL((irfft_stream_kernel<K>), dim3(grid), dim3(256), fft_tile_lds_bytes(K, P), s, in, out, map, nrows,
                         in_fstride, int(ntiles), scale, bias, bias_div, relu);
      return hipGetLastError();
    }
  }
  FftPlan pl = plan_fft(K, nrows);
  dim3 grid((unsigned)cdiv(nrows, 2 * pl.P));
  if (rows_fast)
    hipLaunchKernelGGL((irfft_kernel<K, true>), grid, dim3(pl.NT), pl.lds, s, in, out, map, nrows, in_fstride,
                       pl.P, scale, bias, bias_div, relu, nparts, part_stride);
  else
    hipLaunchKernelGGL((irfft_kernel<K, false>), grid, dim3(pl.NT), pl.lds, s, in, out, map, nrows, in_fstride,
                       pl.P, scale, bias, bias_div, relu, nparts, part_stride);
  return hipGetLastError();
}

#define CIRC_DISPATCH_K(k, CALL)                    \
  switch (k) {                                      \
    case 2: return CALL(2);                         \
    case 4: return CALL(4);                         \
    case 8: return CALL(8);                         \
    case 16: return CALL(16);                       \
    case 32: return CALL(32);                       \
    case 64: return CALL(64);                       \
    case 128: return CALL(128);                     \
    case 256: return CALL(256);                     \
    case 512: return CALL(512);                     \
    default: return hipErrorInvalidValue;           \
  }
#define CIRC_DISPATCH_MIXED_K(k, CALL)              \
  switch (k) {                                      \
    case 12: return CALL(12);                       \
    case 24: return CALL(24);                       \
    case 48: return CALL(48);                       \
    case 96: return CALL(96);                       \
    case 192: return CALL(192);                     \
    case 384: return CALL(384);                     \
    case 20: return CALL(20);                       \
    case 40: return CALL(40);                       \
    case 80: return CALL(80);                       \
    case 160: return CALL(160);                     \
    case 320: return CALL(320);                     \
    case 100: return CALL(100);                     \
    case 200: return CALL(200);                     \
    case 400: return CALL(400);                     \
    default: break;                                 \
  }

hipError_t launch_rfft(int k, bool rows_fast, const float* in, float2* out, const RowMap& map, long long nrows,
                       long long out_fstride, int n_grids, long long in_gstride, long long out_gstride,
                       float scale, int conj, hipStream_t s) {
#define CALL(KK) launch_rfft_k<KK>(rows_fast, in, out, map, nrows, out_fstride, n_grids, in_gstride, out_gstride, scale, conj, s)
  CIRC_DISPATCH_MIXED_K(k, CALL)
#undef CALL
  if (!radix2_k(k)) {
    if (const int k1 = dft_factor(k); k1 > 1) {   // composite: two factors
      const int R = dft2_rows_per_block(k, nrows);
      hipLaunchKernelGGL(dft2_rows_kernel, dim3((unsigned)cdiv(nrows, R), (unsigned)n_grids), dim3(256),
                         dft2_tile_lds_bytes(k, R), s, in, out, map, nrows, out_fstride, in_gstride, out_gstride, k, k1, R,
                         scale, conj, int(rows_fast));
      return hipGetLastError();
    }
    const int R = dft_rows_per_block(k, nrows);
    hipLaunchKernelGGL(dft_rows_kernel, dim3((unsigned)cdiv(nrows, R), (unsigned)n_grids), dim3(256),
                       dft_tile_lds_bytes(k, R), s, in, out, map, nrows, out_fstride, in_gstride, out_gstride, k, R, scale,
                       conj, int(rows_fast));
    return hipGetLastError();
  }
#define CALL(KK) launch_rfft_k<KK>(rows_fast, in, out, map, nrows, out_fstride, n_grids, in_gstride, out_gstride, scale, conj, s)
  CIRC_DISPATCH_K(k, CALL)
#undef CALL
}

hipError_t launch_irfft(int k, bool rows_fast, const float2* in, float* out, const RowMap& map, long long nrows,
                        long long in_fstride, float scale, const float* bias, long long bias_div, int relu,
                        hipStream_t s, int nparts = 1, long long part_stride = 0) {
#define CALL(KK) launch_irfft_k<KK>(rows_fast, in, out, map, nrows, in_fstride, scale, bias, bias_div, relu, nparts, part_stride, s)
  CIRC_DISPATCH_MIXED_K(k, CALL)
#undef CALL
  if (!radix2_k(k)) {
    if (const int k1 = dft_factor(k); k1 > 1) {
      const int R = dft2_rows_per_block(k, nrows);
      hipLaunchKernelGGL(idft2_rows_kernel, dim3((unsigned)cdiv(nrows, R)), dim3(256), dft2_tile_lds_bytes(k, R), s, in, out,
                         map, nrows, in_fstride, k, k1, R, scale, bias, bias_div, relu, nparts, part_stride, int(rows_fast));
      return hipGetLastError();
    }
    const int R = dft_rows_per_block(k, nrows);
    hipLaunchKernelGGL(idft_rows_kernel, dim3((unsigned)cdiv(nrows, R)), dim3(256), dft_tile_lds_bytes(k, R), s, in, out,
                       map, nrows, in_fstride, k, R, scale, bias, bias_div, relu, nparts, part_stride, int(rows_fast));
    return hipGetLastError();
  }
#define CALL(KK) launch_irfft_k<KK>(rows_fast, in, out, map, nrows, in_fstride, scale, bias, bias_div, relu, nparts, part_stride, s)
  CIRC_DISPATCH_K(k, CALL)
#undef CALL
}

// Number of k slices for a GEMM with few output tiles and a long reduction (backward-weights):
// enough slices to put about four workgroups of 64x64 tiles on every CU, each at least 64 deep.
inline int cgemm_ksplit(int k, int M, int N, int Kd) {
  const int NF = k / 2 + 1;
  const long long tiles = (long long)NF * cdiv(M, 64) * cdiv(N, 64);
  int ks = 1;
  while (ks < 16 && tiles * ks < 1024 && Kd / (ks * 2) >= 64) ks *= 2;
  return ks;
}

// Workgroups of the persistent tiled GEMM: two per CU.
constexpr int kGemmWorkgroups = 512;
template <int FM, int WM, int WN>
hipError_t launch_cgemm_tiled(const float2* A, const float2* B, float2* C, int NF, int M, int N, int Kd, long long sA,
                              long long sB, long long sC, bool conj_b, bool a_t, hipStream_t s, int ksplit, int kchunk,
                              long long part_stride) {
  using Sh = GemmShape<FM, WM, WN>;
  const int ntm = (int)cdiv(M, Sh::TM), ntn = (int)cdiv(N, Sh::TN);
  const long long ntiles = (long long)(NF - 1) * ksplit * ntm * ntn;   // bins 0 and NF-1 share a tile
  if (ntiles > (1ll << 31) - 8) return hipErrorInvalidValue;
  const long long chunk = cdiv(ntiles, kGemmWorkgroups);
  dim3 grid((unsigned)(cdiv(cdiv(ntiles, chunk), 8) * 8));
#define CIRC_TILED(CJ, AT)                                                                                              \
  hipLaunchKernelGGL((cgemm_tiled_kernel<FM, WM, WN, CJ, AT>), grid, dim3(256), 0, s, A, B, C, M, N, Kd, NF, sA, sB, sC, ntm, \
                     ntn, ksplit, kchunk, part_stride, (unsigned)ntiles, (unsigned)chunk)
  if (conj_b && a_t) CIRC_TILED(true, true);
  else if (conj_b) CIRC_TILED(true, false);
  else if (a_t) CIRC_TILED(false, true);
  else CIRC_TILED(false, false);
#undef CIRC_TILED
  return hipGetLastError();
}

// C[f][m][n] = sum_kd A[f][kd][m] * (conj?)B[f][kd][n] for f in [0, NF); with ksplit > 1 slice s
// writes its partial sums to C + s*part_stride.  sA, sB, sC: elements between consecutive
// frequencies of A, B, C.
// Problems with a narrow output and a long reduction (backward-weights: N = q <= 64, reduction
// over the batch) run on LDS-staged 64x64 workgroup tiles (measured at the 16384x16384, k=256,
// batch 1024 layer: 58 us against 64 us); all others run one wave per 32x32 or 16x16 tile
// straight from global memory, which was measured faster there (56 us against 62 us for
// 64x128 tiles): its many independent waves drift apart, whereas the workgroups of the tiled
// kernel stay in step and load, multiply and store at the same moments.
constexpr long long kGemmTiledMinTiles = 256;
inline bool cgemm_takes_tiled(int k, int M, int N, int Kd, int ksplit) {
  if (k & 1) return false;   // the tiled kernel pairs bin 0 with a real Nyquist bin, which odd sizes lack
  const int NF = k / 2 + 1;
  const long long tiles_s = (long long)(NF - 1) * ksplit * cdiv(M, 64) * cdiv(N, 64);
  // the tiled kernel keeps offsets inside one frequency of an operand in 32 bits
  const long long lim = (1ll << 31) - 1;
  const bool fits32 = (long long)Kd * M <= lim && (long long)Kd * N <= lim && (long long)M * N <= lim;
  return fits32 && M > 32 && N <= 64 && tiles_s >= kGemmTiledMinTiles;
}
// Wide outputs without split-K (forward and backward-data of large layers) run on the bfloat16
// matrix instruction with every fp32 operand split into three bfloat16 terms (circ_gemm_split.h):
// the fp32 matrix instruction bounds the one-wave kernel there (16384x16384, k=256, batch 1024:
// 35 us against 47 us; the error against a float64 sum is no larger, 3.8e-7 against 5.3e-7 of
// the largest output).  Workgroups: two per CU, each with its share of consecutive tiles.
constexpr long long kGemmSplitMinTiles = 256;
constexpr int kGemmSplitWorkgroups = 512;
inline bool cgemm_takes_split(int k, int M, int N, int Kd, int ksplit) {
  const int NF = k / 2 + 1;
  const long long tiles = (long long)NF * cdiv(M, SplitGemmShape::TM) * cdiv(N, SplitGemmShape::TN);
  const long long lim = (1ll << 31) - 1;       // offsets inside one frequency of an operand are kept in 32 bits
  const bool fits32 = (long long)Kd * M <= lim && (long long)Kd * N <= lim && (long long)M * N <= lim;
  return ksplit == 1 && fits32 && M > 32 && Kd >= 16 && tiles >= kGemmSplitMinTiles && tiles <= lim;
}
hipError_t launch_cgemm_split(const float2* A, const float2* B, float2* C, int NF, int M, int N, int Kd, long long sA,
                              long long sB, long long sC, bool conj_b, hipStream_t s) {
  const int ntm = (int)cdiv(M, SplitGemmShape::TM), ntn = (int)cdiv(N, SplitGemmShape::TN);
  const long long ntiles = (long long)NF * ntm * ntn;
  const long long nwg = ntiles < kGemmSplitWorkgroups ? ntiles : kGemmSplitWorkgroups;
  dim3 grid((unsigned)(cdiv(nwg, 8) * 8));
  const unsigned base = (unsigned)(ntiles / nwg), rem = (unsigned)(ntiles % nwg);
  if (conj_b)
    hipLaunchKernelGGL((cgemm_split_kernel<true>), grid, dim3(SplitGemmShape::NT), 0, s, A, B, C, M, N, Kd, sA, sB, sC, ntm, ntn,
                       (unsigned)ntiles, base, rem);
  else
    hipLaunchKernelGGL((cgemm_split_kernel<false>), grid, dim3(SplitGemmShape::NT), 0, s, A, B, C, M, N, Kd, sA, sB, sC, ntm, ntn,
                       (unsigned)ntiles, base, rem);
  return hipGetLastError();
}
hipError_t launch_cgemm_split_dw(const float2* A, const float2* B, float2* C, int NF, int M, int N, int Kd, long long sA,
                                 long long sB, long long sC, hipStream_t s, int ksplit, int kchunk, long long part_stride) {
  const int ntm = (int)cdiv(M, 64), ntn = (int)cdiv(N, 64);
  const long long ntiles = (long long)NF * ntm * ntn * ksplit;
  if (ntiles > (1ll << 31) - 8) return hipErrorInvalidValue;
  const long long nwg = ntiles < kGemmSplitWorkgroups ? ntiles : kGemmSplitWorkgroups;
  dim3 grid((unsigned)(cdiv(nwg, 8) * 8));
  hipLaunchKernelGGL(cgemm_split_dw_kernel, grid, dim3(SplitGemmShape::NT), 0, s, A, B, C, M, N, Kd, sA, sB, sC, ntm, ntn, ksplit,
                     kchunk, part_stride, (unsigned)ntiles, (unsigned)(ntiles / nwg), (unsigned)(ntiles % nwg));
  return hipGetLastError();
}
// a_t: A is stored [f][m][kd] instead of [f][kd][m]; only the tiled kernels read that layout, so
// callers pass it only when cgemm_takes_tiled() holds.
hipError_t launch_cgemm(const float2* A, const float2* B, float2* C, int k, int M, int N, int Kd, long long sA,
                        long long sB, long long sC, bool conj_b, hipStream_t s, int ksplit = 1,
                        long long part_stride = 0, bool a_t = false) {
  const int NF = k / 2 + 1;                                    // one complex product per bin 0..k/2
  const int kchunk = (int)(cdiv(cdiv(Kd, ksplit), 32) * 32);   // whole operand groups per slice
  if (cgemm_takes_tiled(k, M, N, Kd, ksplit)) {
    // backward-weights of large layers: the split arithmetic (whole quads and slabs of the reduction only)
    const long long tiles = (long long)NF * cdiv(M, 64) * cdiv(N, 64) * ksplit;
    if (conj_b && a_t && Kd % 4 == 0 && kchunk % SplitGemmShape::KA == 0 && (sA & 1) == 0 && tiles >= kGemmSplitMinTiles)
      return launch_cgemm_split_dw(A, B, C, NF, M, N, Kd, sA, sB, sC, s, ksplit, kchunk, part_stride);
    return launch_cgemm_tiled<1, 2, 2>(A, B, C, NF, M, N, Kd, sA, sB, sC, conj_b, a_t, s, ksplit, kchunk, part_stride);
  }
  if (a_t) return hipErrorInvalidValue;
  if (cgemm_takes_split(k, M, N, Kd, ksplit)) return launch_cgemm_split(A, B, C, NF, M, N, Kd, sA, sB, sC, conj_b, s);
  bool big = (long long)NF * cdiv(M, 32) * cdiv(N, 32) * ksplit >= 1024;
  int tile = big ? 32 : 16;
  const int ntn = (int)cdiv(N, tile);
  dim3 grid((unsigned)(ntn * ksplit), (unsigned)cdiv(M, tile), (unsigned)NF);
  if (big) {
    if (conj_b) hipLaunchKernelGGL((cgemm_kernel<32, true>), grid, dim3(64), 0, s, A, B, C, M, N, Kd, sA, sB, sC, ntn, kchunk, part_stride);
    else hipLaunchKernelGGL((cgemm_kernel<32, false>), grid, dim3(64), 0, s, A, B, C, M, N, Kd, sA, sB, sC, ntn, kchunk, part_stride);
  } else {
    if (conj_b) hipLaunchKernelGGL((cgemm_kernel<16, true>), grid, dim3(64), 0, s, A, B, C, M, N, Kd, sA, sB, sC, ntn, kchunk, part_stride);
    else hipLaunchKernelGGL((cgemm_kernel<16, false>), grid, dim3(64), 0, s, A, B, C, M, N, Kd, sA, sB, sC, ntn, kchunk, part_stride);
  }
  return hipGetLastError();
}

// Kernels whose LDS tile exceeds the 64 KB default opt in (gfx950: 160 KB per workgroup).  The
// attribute belongs to the kernel on one device, so what has been granted is remembered per kernel
// instantiation and device: an atomic read on the fast path, a lock around the runtime call, so
// that first calls from several host threads, or on several devices, neither race nor miss it.
constexpr int kMaxDevices = 64;
struct LdsOptIn {
  std::atomic<size_t> granted[kMaxDevices];   // static storage: starts at zero
};
inline std::mutex& lds_opt_in_mutex() {
  static std::mutex m;
  return m;
}
template <class Kern>
hipError_t ensure_lds(Kern kern, size_t bytes, LdsOptIn& st) {
  if (bytes <= 64 * 1024) return hipSuccess;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return hipErrorInvalidDevice;
  const bool tracked = dev >= 0 && dev < kMaxDevices;
  if (tracked && st.granted[dev].load(std::memory_order_acquire) >= bytes) return hipSuccess;
  std::lock_guard<std::mutex> lock(lds_opt_in_mutex());
  if (tracked && st.granted[dev].load(std::memory_order_relaxed) >= bytes) return hipSuccess;
  const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e != hipSuccess) return e;
  if (tracked) st.granted[dev].store(bytes, std::memory_order_release);
  return hipSuccess;
}

// ONE: all q input blocks fit one chunk of the kernel (no double buffering of the operands).
// HM: 0 fp32, 1 fp16, 2 bfloat16 storage (wf, x, y then point to the 16-bit data).
template <int K, int IT, int NP, int NT, bool ONE, int HM>
hipError_t launch_fused_v(const float4* wf, const float* x, const float* bias, float* y, int p, int q, int batch,
                          int relu, hipStream_t s) {
  using Sh = FusedShape<K, IT, NP, NT>;
  static_assert((4096 / K) % Sh::JC == 0, "packed weights are padded to chunks of 4096/K input blocks");
  static LdsOptIn opted_in;
  if (ensure_lds(&fc_fused_kernel<K, IT, NP, NT, ONE, HM>, Sh::lds_bytes(ONE), opted_in) != hipSuccess) return hipErrorInvalidValue;
  const FusedTileMap tm = make_fused_tile_map(p, q, K, IT, NP, batch);
  hipLaunchKernelGGL((fc_fused_kernel<K, IT, NP, NT, ONE, HM>), dim3(tm.grid), dim3(NT), Sh::lds_bytes(ONE), s, wf, x, bias,
                     y, p, q, batch, tm, fused_q2p(q, K), relu);
  return hipGetLastError();
}

template <int K, int IT, int NP, int NT, int HM>
hipError_t launch_fused_t(const float4* wf, const float* x, const float* bias, float* y, int p, int q, int batch,
                          int relu, hipStream_t s) {
  if (q <= FusedShape<K, IT, NP, NT>::JC) return launch_fused_v<K, IT, NP, NT, true, HM>(wf, x, bias, y, p, q, batch, relu, s);
  return launch_fused_v<K, IT, NP, NT, false, HM>(wf, x, bias, y, p, q, batch, relu, s);
}

// Packed batch pairs per workgroup: two when that still leaves at least 256 tiles (one per
// CU); the weight tile is then streamed half as often.
inline int fused_np(int p, int k, int batch) {
  const long long tiles2 = cdiv(p, fused_it(k)) * cdiv(batch, 4);
  return (k >= 64 && tiles2 >= 256) ? 2 : 1;
}

template <int HM>
hipError_t launch_fused_h(int k, const float4* wf, const float* x, const float* bias, float* y, int p, int q, int batch,
                          int relu, hipStream_t s) {
  const int np = fused_np(p, k, batch);
  switch (k) {
    case 32: return launch_fused_t<32, 16, 1, 256, HM>(wf, x, bias, y, p, q, batch, relu, s);
    case 64: return np == 2 ? launch_fused_t<64, 8, 2, 512, HM>(wf, x, bias, y, p, q, batch, relu, s)
                            : launch_fused_t<64, 8, 1, 512, HM>(wf, x, bias, y, p, q, batch, relu, s);
    case 128: return np == 2 ? launch_fused_t<128, 8, 2, 512, HM>(wf, x, bias, y, p, q, batch, relu, s)
                             : launch_fused_t<128, 8, 1, 512, HM>(wf, x, bias, y, p, q, batch, relu, s);
    case 256: return np == 2 ? launch_fused_t<256, 8, 2, 256, HM>(wf, x, bias, y, p, q, batch, relu, s)
                             : launch_fused_t<256, 8, 1, 256, HM>(wf, x, bias, y, p, q, batch, relu, s);
    default: return hipErrorInvalidValue;
  }
}
hipError_t launch_fused(int k, const float4* wf, const float* x, const float* bias, float* y, int p, int q, int batch,
                        int relu, hipStream_t s) {
  return launch_fused_h<0>(k, wf, x, bias, y, p, q, batch, relu, s);
}
// 16-bit storage: wf = operands packed by pack_fused_half_kernel, x and y 16-bit values
hipError_t launch_fused_half(bool bf, int k, const void* wf, const void* x, const float* bias, void* y, int p, int q,
                             int batch, int relu, hipStream_t s) {
  const float4* w4 = static_cast<const float4*>(wf);
  const float* xf = static_cast<const float*>(x);
  float* yf = static_cast<float*>(y);
  return bf ? launch_fused_h<2>(k, w4, xf, bias, yf, p, q, batch, relu, s) : launch_fused_h<1>(k, w4, xf, bias, yf, p, q, batch, relu, s);
}

// Upper bound, in MiB, of the operand bytes all workgroups of the fused kernel pull through
// L2 (see use_fused_forward).
constexpr double kFusedMaxL2MiB = 256.0;

// Fused or unfused forward?  The fused kernel re-reads the weight tile once per tile of batch
// rows and the x tile once per tile of output block rows, all through L2 (about 45 GB/s per
// CU for data first touched in a launch), and recomputes the FFT of x once per tile of output
// block rows.  That wins while the problem is small (one launch, no spectra round trip through
// HBM); for large batches the unfused route, whose GEMM reuses operands from registers over
// 32x32 tiles, is faster.
inline bool use_fused_forward(int p, int q, int k, int batch) {
  const int it = fused_it(k);
  if (it == 0) return false;
  const double n_it = double(cdiv(p, it)), n_bt = double(cdiv(batch, 2 * fused_np(p, k, batch)));
  const double w_bytes = double(p) * q * k * 4.0, x_bytes = double(batch) * q * k * 4.0;
  const double l2_bytes = n_bt * w_bytes + n_it * x_bytes;
  return n_it <= 8 && l2_bytes <= kFusedMaxL2MiB * 1048576.0;
}

// Batch <= 2 on few block rows with long rows: split the input blocks over several workgroups per
// block row (two launches, partial spectra through the workspace).  Returns the number of splits
// (1 = single launch).  Each split keeps at least 8 input blocks; the split pays for its second
// launch only when a workgroup would otherwise transform >= 8192 input values.
inline int gemv_splits(int p, int q, int k) {
  constexpr int kMaxWg = 256;              // workgroups of the split launch: one per CU
  constexpr long long kSplitMin = 8192;    // input values per workgroup from which the split pays
  if ((long long)q * k < kSplitMin || p * 2 > kMaxWg) return 1;
  int ns = 1;
  while (ns < 16 && p * ns * 2 <= kMaxWg && q / (ns * 2) >= 8) ns *= 2;
  return ns;
}
inline size_t gemv_partial_bytes(int p, int q, int k) {
  const int ns = gemv_splits(p, q, k);
  return ns > 1 ? size_t(ns) * p * k * sizeof(float2) : 0;
}

// HM: 0 fp32, 1 fp16, 2 bfloat16 storage (wg, x, y then point to the 16-bit data)
template <int K, int HM>
hipError_t launch_gemv_k(const float2* wg, const float* x, const float* bias, float* y, int p, int q, int batch, int relu,
                         void* workspace, hipStream_t s) {
  using Sh = GemvShape<K>;
  static LdsOptIn opted_in;
  const int ns = gemv_splits(p, q, K);
  if (ns > 1) {
    static LdsOptIn opted1, opted2;
    if (ensure_lds(&fc_gemv_kernel<K, 1, HM>, Sh::LDS_BYTES, opted1) != hipSuccess) return hipErrorInvalidValue;
    if (ensure_lds(&fc_gemv_kernel<K, 2, HM>, Sh::LDS_BYTES, opted2) != hipSuccess) return hipErrorInvalidValue;
    float2* part = static_cast<float2*>(workspace);
    const int jper = (int)cdiv(q, ns);
    hipLaunchKernelGGL((fc_gemv_kernel<K, 1, HM>), dim3((unsigned)p, (unsigned)ns), dim3(Sh::NT), Sh::LDS_BYTES, s, wg, x,
                       (const float*)nullptr, (float*)nullptr, p, q, batch, 0, part, ns, jper);
    if (hipGetLastError() != hipSuccess) return hipErrorInvalidValue;
    hipLaunchKernelGGL((fc_gemv_kernel<K, 2, HM>), dim3((unsigned)p), dim3(Sh::NT), Sh::LDS_BYTES, s, wg, x, bias, y, p, q, batch,
                       relu, part, ns, jper);
    return hipGetLastError();
  }
  if (ensure_lds(&fc_gemv_kernel<K, 0, HM>, Sh::LDS_BYTES, opted_in) != hipSuccess) return hipErrorInvalidValue;
  hipLaunchKernelGGL((fc_gemv_kernel<K, 0, HM>), dim3((unsigned)p), dim3(Sh::NT), Sh::LDS_BYTES, s, wg, x, bias, y, p, q, batch,
                     relu, (float2*)nullptr, 1, q);
  return hipGetLastError();
}

template <int HM>
hipError_t launch_gemv_h(int k, const float2* wg, const float* x, const float* bias, float* y, int p, int q, int batch,
                         int relu, void* workspace, hipStream_t s) {
  switch (k) {
    case 4: return launch_gemv_k<4, HM>(wg, x, bias, y, p, q, batch, relu, workspace, s);
    case 8: return launch_gemv_k<8, HM>(wg, x, bias, y, p, q, batch, relu, workspace, s);
    case 16: return launch_gemv_k<16, HM>(wg, x, bias, y, p, q, batch, relu, workspace, s);
    case 32: return launch_gemv_k<32, HM>(wg, x, bias, y, p, q, batch, relu, workspace, s);
    case 64: return launch_gemv_k<64, HM>(wg, x, bias, y, p, q, batch, relu, workspace, s);
    case 128: return launch_gemv_k<128, HM>(wg, x, bias, y, p, q, batch, relu, workspace, s);
    case 256: return launch_gemv_k<256, HM>(wg, x, bias, y, p, q, batch, relu, workspace, s);
    case 512: return launch_gemv_k<512, HM>(wg, x, bias, y, p, q, batch, relu, workspace, s);
    default: return hipErrorInvalidValue;
  }
}
hipError_t launch_gemv(int k, const float2* wg, const float* x, const float* bias, float* y, int p, int q, int batch,
                       int relu, void* workspace, hipStream_t s) {
  return launch_gemv_h<0>(k, wg, x, bias, y, p, q, batch, relu, workspace, s);
}
hipError_t launch_gemv_half(bool bf, int k, const void* wg, const void* x, const float* bias, void* y, int p, int q,
                            int batch, int relu, void* workspace, hipStream_t s) {
  const float2* w2 = static_cast<const float2*>(wg);
  const float* xf = static_cast<const float*>(x);
  float* yf = static_cast<float*>(y);
  return bf ? launch_gemv_h<2>(k, w2, xf, bias, yf, p, q, batch, relu, workspace, s)
            : launch_gemv_h<1>(k, w2, xf, bias, yf, p, q, batch, relu, workspace, s);
}

inline bool overlaps(const void* a, size_t na, const void* b, size_t nb) {
  uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
  return x < y + nb && y < x + na;
}

// dims whose products must stay inside what the kernels index with 32-bit grid sizes
inline bool fc_dims_ok(int p, int q, int k, int batch) {
  if (p <= 0 || q <= 0 || batch <= 0 || !valid_k(k)) return false;
  if ((long long)p * k > (1ll << 30) || (long long)q * k > (1ll << 30)) return false;
  if ((long long)p * batch > (1ll << 31) - 1 || (long long)q * batch > (1ll << 31) - 1) return false;
  if ((long long)p * q > (1ll << 31) - 1) return false;
  if (batch > 65535 * 16 || p > 65535 * 16 || q > 65535 * 16) return false;   // gridDim.x/y limits of the GEMM
  return true;
}

// Sections 2.. of the blob (the operand orders of the fused, streaming and CONV kernels) are
// rearrangements of the two spectrum sections; this rewrites all of them from those two.
circ_status pack_derived_sections(void* w_hat, int n_grids, int p, int q, int k, hipStream_t s) {
  const BlobLayout bl = blob_layout(n_grids, p, q, k);
  const float2* fwd = blob_at<float2>(w_hat, bl.fwd);
  const float2* bwd = blob_at<float2>(w_hat, bl.bwd);
  // The backward section [f][i][j] (conjugated) is exactly the "[f][j'][i']" forward section of the
  // transposed grid (p' = q output block rows, q' = p input blocks), so the same packing
  // produces the operands that make backward-data a forward pass.  For CONV, backward-data is
  // the forward kernel on the transposed grids with the conjugated spectra and the reflected filter.
  PackPlan pl;
  pl.n = 0;
  unsigned blocks = 0;
  auto add = [&](int kind, const float2* spec, size_t off, int pp, int qq, int a, int b, size_t elems) {
    if (!elems) return;
    const int i = pl.n++;
    pl.first[i] = blocks;
    pl.kind[i] = kind; pl.spec[i] = spec; pl.dst[i] = blob_at<char>(w_hat, off);
    pl.p[i] = pp; pl.q[i] = qq; pl.a[i] = a; pl.b[i] = b;
    blocks += (unsigned)cdiv((long long)elems, 256);
  };
  const bool fused = fused_section_elems(n_grids, p, q, k) != 0;   // block size served by the fused FC kernel
  add(0, fwd, bl.fused_fwd, p, q, fused ? fused_igp(p, k) : 0, fused ? fused_q2p(q, k) : 0, fused_section_elems(n_grids, p, q, k));
  add(1, fwd, bl.gemv_fwd, p, q, 0, 0, gemv_section_elems(n_grids, p, q, k));
  add(0, bwd, bl.fused_bwd, q, p, fused ? fused_igp(q, k) : 0, fused ? fused_q2p(p, k) : 0, fused_section_elems(n_grids, q, p, k));
  add(1, bwd, bl.gemv_bwd, q, p, 0, 0, gemv_section_elems(n_grids, q, p, k));
  const size_t nconv = conv_section_elems(n_grids, p, q, k), nconvb = conv_section_elems(n_grids, q, p, k);
  add(2, fwd, bl.conv, p, q, nconv ? int(nconv / (size_t(n_grids) * q * 64)) : 0, 0, nconv);
  add(2, bwd, bl.conv_bwd, q, p, nconvb ? int(nconvb / (size_t(n_grids) * p * 64)) : 0, 1, nconvb);
  if (pl.n == 0) return CIRC_OK;
  pl.first[pl.n] = blocks;
  hipLaunchKernelGGL(pack_sections_kernel, dim3(blocks), dim3(256), 0, s, pl, n_grids, k);
  if (hipGetLastError() != hipSuccess) return CIRC_EHIP;
  return CIRC_OK;
}

}  // namespace

extern "C" {

const char* circ_status_string(circ_status s) {
  switch (s) {
    case CIRC_OK: return "CIRC_OK";
    case CIRC_EINVAL: return "CIRC_EINVAL: invalid argument";
    case CIRC_ENOTSUP: return "CIRC_ENOTSUP: not supported";
    case CIRC_EWORKSPACE: return "CIRC_EWORKSPACE: workspace missing or too small";
    case CIRC_EHIP: return "CIRC_EHIP: HIP launch failed";
  }
  return "unknown circ_status";
}

size_t circ_spectra_bytes(int n_grids, int p, int q, int k) {
  if (n_grids <= 0 || p <= 0 || q <= 0 || !valid_k(k)) return 0;
  if ((long long)p * q > (1ll << 31) - 1) return 0;
  return blob_layout(n_grids, p, q, k).total;
}

circ_status circ_precompute_spectra(const float* w, int n_grids, int p, int q, int k, void* w_hat, void* stream) {
  if (!w || !w_hat || n_grids <= 0 || n_grids > 65535 || p <= 0 || q <= 0 || !valid_k(k)) return CIRC_EINVAL;
  if ((long long)p * q > (1ll << 31) - 1) return CIRC_EINVAL;
  if (!aligned16(w) || !aligned16(w_hat)) return CIRC_EINVAL;
  size_t wbytes = size_t(n_grids) * p * q * k * sizeof(float);
  if (overlaps(w, wbytes, w_hat, circ_spectra_bytes(n_grids, p, q, k))) return CIRC_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const BlobLayout bl = blob_layout(n_grids, p, q, k);
  float2* fwd = blob_at<float2>(w_hat, bl.fwd);
  float2* bwd = blob_at<float2>(w_hat, bl.bwd);
  const long long rows = (long long)p * q;
  const long long in_g = rows * k, out_g = (long long)spectrum_elems(k, rows);
  const float inv_k = 1.0f / float(k);
  // forward operand: row id = j*p + i  ->  w[i][j][:]
  RowMap mf{p, q, (long long)q * k, (long long)k, 0, 1};
  if (launch_rfft(k, false, w, fwd, mf, rows, rows, n_grids, in_g, out_g, inv_k, 0, s) != hipSuccess) return CIRC_EHIP;
  // backward operand: row id = i*q + j, conjugated
  RowMap mb{q, p, (long long)k, (long long)q * k, 0, 1};
  if (launch_rfft(k, false, w, bwd, mb, rows, rows, n_grids, in_g, out_g, inv_k, 1, s) != hipSuccess) return CIRC_EHIP;
  return pack_derived_sections(w_hat, n_grids, p, q, k, s);
}

size_t circ_fc_workspace_bytes(int p, int q, int k, int batch, int backward) {
  if (!fc_dims_ok(p, q, k, batch)) return 0;
  size_t xa = align_up(ws_spectrum_elems(k, (long long)q * batch) * sizeof(float2), 256);
  size_t ya = align_up(ws_spectrum_elems(k, (long long)p * batch) * sizeof(float2), 256);
  // batch <= 2: partial spectra of the split streaming kernel (forward grid, or the transposed
  // grid for backward-data); they live at the start of the workspace, which nothing else uses
  // at that time
  size_t gp = 0;
  if (batch <= 2 && gemv_k(k)) gp = align_up(backward ? gemv_partial_bytes(q, p, k) : gemv_partial_bytes(p, q, k), 256);
  if (!backward) return xa + ya > gp ? xa + ya : gp;
  size_t wa = align_up(spectrum_elems(k, (long long)p * q) * sizeof(float2), 256);
  const size_t tot = xa + ya + wa * cgemm_ksplit(k, p, q, batch);   // one dW^ buffer per k slice
  return tot > gp ? tot : gp;
}

circ_status circ_fc_forward(const void* w_hat, const float* x, const float* bias, float* y, int p, int q, int k,
                            int batch, int epilogue, void* workspace, size_t workspace_bytes, void* stream) {
  if (!fc_dims_ok(p, q, k, batch)) return CIRC_EINVAL;
  if (!w_hat || !x || !y) return CIRC_EINVAL;
  if (epilogue & ~(CIRC_EPI_BIAS | CIRC_EPI_RELU)) return CIRC_EINVAL;
  const bool use_bias = epilogue & CIRC_EPI_BIAS;
  if (use_bias && !bias) return CIRC_EINVAL;
  if (!aligned16(w_hat) || !aligned16(x) || !aligned16(y) || (use_bias && !aligned16(bias))) return CIRC_EINVAL;
  const size_t xbytes = size_t(batch) * q * k * sizeof(float), ybytes = size_t(batch) * p * k * sizeof(float);
  if (overlaps(x, xbytes, y, ybytes)) return CIRC_EINVAL;
  const size_t need = circ_fc_workspace_bytes(p, q, k, batch, 0);
  if (!workspace || workspace_bytes < need) return CIRC_EWORKSPACE;
  if (!aligned16(workspace)) return CIRC_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);

  const BlobLayout bl = blob_layout(1, p, q, k);
  if (batch <= 2 && gemv_k(k)) {   // one or two vectors: streaming matrix-vector kernel
    const float2* wg = blob_at<float2>(w_hat, bl.gemv_fwd);
    if (launch_gemv(k, wg, x, use_bias ? bias : nullptr, y, p, q, batch, (epilogue & CIRC_EPI_RELU) ? 1 : 0, workspace, s) != hipSuccess)
      return CIRC_EHIP;
    return CIRC_OK;
  }
  if (use_fused_forward(p, q, k, batch)) {
    const float4* wfu = blob_at<float4>(w_hat, bl.fused_fwd);
    if (launch_fused(k, wfu, x, use_bias ? bias : nullptr, y, p, q, batch, (epilogue & CIRC_EPI_RELU) ? 1 : 0, s) !=
        hipSuccess)
      return CIRC_EHIP;
    return CIRC_OK;
  }

  const int NF = k / 2 + 1;
  float2* xh = static_cast<float2*>(workspace);
  float2* yh = reinterpret_cast<float2*>(static_cast<char*>(workspace) +
                                         align_up(ws_spectrum_elems(k, (long long)q * batch) * sizeof(float2), 256));
  const float2* wf = static_cast<const float2*>(w_hat);
  const long long xrows = (long long)q * batch, yrows = (long long)p * batch;
  // X^[f][j][b]: row id = j*batch + b -> x[b][j*k : (j+1)*k]
  RowMap mx{batch, q, (long long)q * k, (long long)k, 0, 1};
  const long long xfs = ws_fstride(xrows), yfs = ws_fstride(yrows);
  if (launch_rfft(k, false, x, xh, mx, xrows, xfs, 1, 0, 0, 1.0f, 0, s) != hipSuccess) return CIRC_EHIP;
  // Y^[f][i][b] = sum_j W^[f][j][i] X^[f][j][b]
  if (launch_cgemm(wf, xh, yh, k, p, batch, q, (long long)p * q, xfs, yfs, false, s) != hipSuccess) return CIRC_EHIP;
  RowMap my{batch, p, (long long)p * k, (long long)k, 0, 1};
  if (launch_irfft(k, false, yh, y, my, yrows, yfs, 1.0f, use_bias ? bias : nullptr, batch,
                   (epilogue & CIRC_EPI_RELU) ? 1 : 0, s) != hipSuccess)
    return CIRC_EHIP;
  return CIRC_OK;
}

}  // extern "C"

// ---- FC forward for callers that cannot allocate ------------------------------------------------
// The workspace of circ_fc_forward (activation spectra of the three-kernel route, partial
// spectra of the split batch <= 2 kernel) lives in this array instead of a caller's buffer.  In
// host code the name `scratch` is only a handle for the symbol, not a device address: the
// address of the current device's copy is looked up once per device and that pointer is what
// the kernels receive.
static __device__ __align__(256) unsigned char scratch[CIRC_STATIC_SCRATCH_BYTES];

namespace {

struct StaticScratch {
  std::atomic<void*> ptr[kMaxDevices];   // static storage: starts at null
};
StaticScratch g_static_scratch;

// Device address of `scratch` on the current device (each device holds its own copy).
hipError_t static_scratch_ptr(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return hipErrorInvalidDevice;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  void* p = g_static_scratch.ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    std::lock_guard<std::mutex> lock(lds_opt_in_mutex());
    p = g_static_scratch.ptr[dev].load(std::memory_order_relaxed);
    if (!p) {
      const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess) return e;
      if (!p) return hipErrorInvalidSymbol;
      g_static_scratch.ptr[dev].store(p, std::memory_order_release);
    }
  }
  *out = p;
  return hipSuccess;
}

}  // namespace

extern "C" {

circ_status circ_fc_forward_static(const void* w_hat, const float* x, const float* bias, float* y, int p, int q, int k,
                                   int batch, int epilogue, void* stream) {
  if (!fc_dims_ok(p, q, k, batch)) return CIRC_EINVAL;
  if (circ_fc_workspace_bytes(p, q, k, batch, 0) > size_t(CIRC_STATIC_SCRATCH_BYTES)) return CIRC_EWORKSPACE;
  void* ws = nullptr;
  if (static_scratch_ptr(&ws) != hipSuccess) return CIRC_EHIP;
  // every kernel of the forward pass writes the part of the workspace it later reads, so nothing
  // has to be cleared between calls
  return circ_fc_forward(w_hat, x, bias, y, p, q, k, batch, epilogue, ws, size_t(CIRC_STATIC_SCRATCH_BYTES), stream);
}

}  // extern "C"

namespace {

// Launch one step (kernel above) on the spectrum sections of `w_hat`, then rebuild the operand
// sections that are rearrangements of them.  `src` holds nparts partial spectra
// [f][g][i][j] (strides given), not normalised: a = lr / k.
circ_status apply_spectra_step(void* w_hat, const float2* src, int nparts, long long part_stride, long long src_fstride,
                               long long src_gstride, int n_grids, int p, int q, int k, float lr, hipStream_t s) {
  const BlobLayout bl = blob_layout(n_grids, p, q, k);
  const int NF = k / 2 + 1;
  dim3 grid((unsigned)(cdiv(p, 32) * cdiv(q, 32)), (unsigned)NF, (unsigned)n_grids);
  hipLaunchKernelGGL(spectra_step_kernel, grid, dim3(256), 0, s, src, nparts, part_stride, src_fstride, src_gstride,
                     blob_at<float2>(w_hat, bl.fwd), blob_at<float2>(w_hat, bl.bwd), p, q, NF, k, lr / float(k));
  if (hipGetLastError() != hipSuccess) return CIRC_EHIP;
  return pack_derived_sections(w_hat, n_grids, p, q, k, s);
}

// FC backward.  `dw` receives the gradient of the block vectors; `w_upd` (the same blob as
// w_hat, writable) takes the step -lr * gradient in the frequency domain instead.  Either, both
// or neither may be given; backward-data always reads the spectra as they are on entry.
circ_status fc_backward_impl(const void* w_hat, const float* x, const float* dy, float* dx, float* dw, void* w_upd,
                             float lr, int p, int q, int k, int batch, void* workspace, size_t workspace_bytes,
                             void* stream) {
  if (!fc_dims_ok(p, q, k, batch)) return CIRC_EINVAL;
  if (!w_hat || !dy) return CIRC_EINVAL;
  if (!dx && !dw && !w_upd) return CIRC_EINVAL;
  if ((dw || w_upd) && !x) return CIRC_EINVAL;
  if (!aligned16(w_hat) || !aligned16(dy) || !aligned16(x) || !aligned16(dx) || !aligned16(dw)) return CIRC_EINVAL;
  const size_t xbytes = size_t(batch) * q * k * sizeof(float), ybytes = size_t(batch) * p * k * sizeof(float);
  const size_t wbytes = size_t(p) * q * k * sizeof(float);
  if (dx && (overlaps(dx, xbytes, dy, ybytes) || (x && overlaps(dx, xbytes, x, xbytes)))) return CIRC_EINVAL;
  if (dw && (overlaps(dw, wbytes, dy, ybytes) || overlaps(dw, wbytes, x, xbytes))) return CIRC_EINVAL;
  if (dx && dw && overlaps(dx, xbytes, dw, wbytes)) return CIRC_EINVAL;
  if (w_upd) {   // the blob is rewritten: none of the operands may lie inside it
    const size_t bbytes = circ_spectra_bytes(1, p, q, k);
    if (overlaps(w_upd, bbytes, x, xbytes) || overlaps(w_upd, bbytes, dy, ybytes) || (dx && overlaps(w_upd, bbytes, dx, xbytes)) ||
        (dw && overlaps(w_upd, bbytes, dw, wbytes)))
      return CIRC_EINVAL;
  }
  const size_t need = circ_fc_workspace_bytes(p, q, k, batch, 1);
  if (!workspace || workspace_bytes < need) return CIRC_EWORKSPACE;
  if (!aligned16(workspace)) return CIRC_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);

  const int NF = k / 2 + 1;
  const size_t xa = align_up(ws_spectrum_elems(k, (long long)q * batch) * sizeof(float2), 256);
  const size_t ya = align_up(ws_spectrum_elems(k, (long long)p * batch) * sizeof(float2), 256);
  float2* bufx = static_cast<float2*>(workspace);
  float2* bufy = reinterpret_cast<float2*>(static_cast<char*>(workspace) + xa);
  float2* bufw = reinterpret_cast<float2*>(static_cast<char*>(workspace) + xa + ya);
  const BlobLayout bl = blob_layout(1, p, q, k);
  const float2* wb = blob_at<float2>(w_hat, bl.bwd);
  const long long xrows = (long long)q * batch, yrows = (long long)p * batch;
  const long long xfs = ws_fstride(xrows), yfs = ws_fstride(yrows), wfs = (long long)p * q;

  // Backward-data is a forward pass on the transposed, conjugated grid (q output block rows,
  // p input blocks, no epilogue): the small-problem kernels serve it from their own sections.
  const int ksplit = cgemm_ksplit(k, p, q, batch);
  // The tiled GEMM reads dY^ in the [f][i][b] order of backward-data, so dy is transformed once
  // for both results; the one-wave-per-tile GEMM needs the batch-major order [f][b][i].
  const bool want_dw = dw || w_upd;
  const bool dw_shares_dy = want_dw && cgemm_takes_tiled(k, p, q, batch, ksplit);
  bool have_dyh = false;   // bufy holds dY^[f][i][b]
  if (dx && batch <= 2 && gemv_k(k)) {
    if (launch_gemv(k, blob_at<float2>(w_hat, bl.gemv_bwd), dy, nullptr, dx, q, p, batch, 0, workspace, s) != hipSuccess) return CIRC_EHIP;
  } else if (dx && use_fused_forward(q, p, k, batch)) {
    if (launch_fused(k, blob_at<float4>(w_hat, bl.fused_bwd), dy, nullptr, dx, q, p, batch, 0, s) != hipSuccess)
      return CIRC_EHIP;
  } else if (dx) {
    // dY^[f][i][b];  dX^[f][j][b] = sum_i conj(W^)[f][i][j] dY^[f][i][b]
    RowMap mdy{batch, p, (long long)p * k, (long long)k, 0, 1};
    if (launch_rfft(k, false, dy, bufy, mdy, yrows, yfs, 1, 0, 0, 1.0f, 0, s) != hipSuccess) return CIRC_EHIP;
    have_dyh = true;
    if (launch_cgemm(wb, bufy, bufx, k, q, batch, p, wfs, yfs, xfs, false, s) != hipSuccess) return CIRC_EHIP;
    RowMap mdx{batch, q, (long long)q * k, (long long)k, 0, 1};
    if (launch_irfft(k, false, bufx, dx, mdx, xrows, xfs, 1.0f, nullptr, 1, 0, s) != hipSuccess) return CIRC_EHIP;
  }
  if (want_dw) {
    // dW^[f][i][j] = sum_b dY^[f][i][b] conj(X^[f][b][j]); X^ is batch-major, dY^ is [f][i][b] for
    // the tiled GEMM (shared with backward-data above) and batch-major [f][b][i] otherwise
    if (dw_shares_dy) {
      if (!have_dyh) {
        RowMap mdy{batch, p, (long long)p * k, (long long)k, 0, 1};
        if (launch_rfft(k, false, dy, bufy, mdy, yrows, yfs, 1, 0, 0, 1.0f, 0, s) != hipSuccess) return CIRC_EHIP;
      }
    } else {
      RowMap mdy{p, batch, (long long)k, (long long)p * k, 0, 1};
      if (launch_rfft(k, false, dy, bufy, mdy, yrows, yfs, 1, 0, 0, 1.0f, 0, s) != hipSuccess) return CIRC_EHIP;
    }
    RowMap mx{q, batch, (long long)k, (long long)q * k, 0, 1};
    if (launch_rfft(k, false, x, bufx, mx, xrows, xfs, 1, 0, 0, 1.0f, 0, s) != hipSuccess) return CIRC_EHIP;
    // the reduction over the batch is cut into slices; the IFFT adds the partial spectra in order
    const long long wpart = (long long)(align_up(spectrum_elems(k, (long long)p * q) * sizeof(float2), 256) / sizeof(float2));
    if (launch_cgemm(bufy, bufx, bufw, k, p, q, batch, yfs, xfs, wfs, true, s, ksplit, wpart, dw_shares_dy) != hipSuccess)
      return CIRC_EHIP;
    const long long wrows = (long long)p * q;
    RowMap mw{q, p, (long long)k, (long long)q * k, 0, 1};
    if (dw && launch_irfft(k, false, bufw, dw, mw, wrows, wrows, 1.0f / float(k), nullptr, 1, 0, s, ksplit, wpart) != hipSuccess)
      return CIRC_EHIP;
    if (w_upd) return apply_spectra_step(w_upd, bufw, ksplit, wpart, wrows, 0, 1, p, q, k, lr, s);
  }
  return CIRC_OK;
}

}  // namespace

extern "C" {

circ_status circ_fc_backward(const void* w_hat, const float* x, const float* dy, float* dx, float* dw, int p, int q,
                             int k, int batch, void* workspace, size_t workspace_bytes, void* stream) {
  if (!dx && !dw) return CIRC_EINVAL;
  return fc_backward_impl(w_hat, x, dy, dx, dw, nullptr, 0.f, p, q, k, batch, workspace, workspace_bytes, stream);
}

circ_status circ_fc_sgd_step(void* w_hat, const float* x, const float* dy, float* dx, float lr, int p, int q, int k,
                             int batch, void* workspace, size_t workspace_bytes, void* stream) {
  if (!w_hat || !(lr == lr)) return CIRC_EINVAL;   // NaN step
  return fc_backward_impl(w_hat, x, dy, dx, nullptr, w_hat, lr, p, q, k, batch, workspace, workspace_bytes, stream);
}

circ_status circ_export_weights(const void* w_hat, int n_grids, int p, int q, int k, float* w, void* stream) {
  if (!w || !w_hat || n_grids <= 0 || n_grids > 65535 || p <= 0 || q <= 0 || !valid_k(k)) return CIRC_EINVAL;
  if ((long long)p * q > (1ll << 31) - 1) return CIRC_EINVAL;
  if (!aligned16(w) || !aligned16(w_hat)) return CIRC_EINVAL;
  if (overlaps(w, size_t(n_grids) * p * q * k * sizeof(float), w_hat, circ_spectra_bytes(n_grids, p, q, k)))
    return CIRC_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const BlobLayout bl = blob_layout(n_grids, p, q, k);
  const float2* fwd = blob_at<float2>(w_hat, bl.fwd);
  const long long rows = (long long)p * q;
  // forward section of grid g: [f][j*p + i] = FFT(w[g][i][j])/k, so the plain inverse sum returns w
  RowMap mf{p, q, (long long)q * k, (long long)k, 0, 1};
  for (int g = 0; g < n_grids; ++g)
    if (launch_irfft(k, false, fwd + (long long)g * spectrum_elems(k, rows), w + (long long)g * rows * k, mf, rows, rows,
                     1.0f, nullptr, 1, 0, s) != hipSuccess)
      return CIRC_EHIP;
  return CIRC_OK;
}

}  // extern "C"

namespace {

struct ConvTilePlan { int TH, TW, tiles_h, tiles_w; size_t lds; };

// Output tile of the fused CONV kernel: the one with the fewest transformed input positions
// in total (tile + halo, summed over the tiles) that fits LDS and the per-wave task limit.
template <int K, int NT>
bool plan_conv_tile(int p, int qh, int r, int Ho, int Wo, int ncombo, ConvTilePlan& best) {
  using Sh = ConvFusedShape<K, NT>;
  const int max_pos = Sh::MAXT * (Sh::NW / ncombo);
  long long best_cost = -1;
  for (int th = 1; th <= Ho && th + r - 1 <= 16; ++th)
    for (int tw = 2; tw <= Wo + (Wo & 1) && tw + r - 1 <= 16; tw += 2) {   // row pitch of 16 input positions; outputs stored in pairs
      if (th * tw > max_pos) continue;
      const int ipos = (th + r - 1) * 16;
      const size_t lds = conv_fused_lds_bytes<K, NT>(qh * ipos, p * th * tw);
      if (lds > 160 * 1024) continue;
      const long long nt = cdiv(Ho, th) * cdiv(Wo, tw);
      // FFT chunks (PT columns each, per channel block) over all tiles, then fewer tiles, then wider tiles
      const long long cost = nt * cdiv(ipos, Sh::PT) * 1024 + nt * 8 - tw;
      if (best_cost < 0 || cost < best_cost) {
        best_cost = cost;
        best = ConvTilePlan{th, tw, (int)cdiv(Ho, th), (int)cdiv(Wo, tw), lds};
      }
    }
  return best_cost >= 0;
}

// NT threads per workgroup, QH input channel blocks whose spectra are held in LDS at a time.
// RAGGED: rows that are not 4n input pixels and 2n output pixels long (element-wise loads and
// stores instead of aligned 16-byte loads and paired stores).
template <int Q, int NT, int QH, int HM, bool RAGGED>
hipError_t launch_conv_fused_r(const float2* wc, const float* x, const float* bias, float* y, int N, int C_out, int H,
                               int W, int Ho, int Wo, int pad, int ncombo, int relu, hipStream_t s) {
  constexpr int K = 64, R = 3;
  ConvTilePlan pl;
  if (!plan_conv_tile<K, NT>(C_out / K, QH, R, Ho, Wo, ncombo, pl)) return hipErrorInvalidValue;
  static LdsOptIn opted;   // the tile, and with it the LDS size, depends on the image: granted sizes only grow
  if (ensure_lds(&conv_fused_kernel<K, NT, R, Q, QH, HM, RAGGED>, pl.lds, opted) != hipSuccess) return hipErrorInvalidValue;
  const long long grid = (long long)cdiv(N, 2) * pl.tiles_h * pl.tiles_w;
  hipLaunchKernelGGL((conv_fused_kernel<K, NT, R, Q, QH, HM, RAGGED>), dim3((unsigned)grid), dim3(NT), pl.lds, s, wc, x, bias, y,
                     N, C_out, H, W, Ho, Wo, pad, pl.TH, pl.TW, pl.tiles_h, pl.tiles_w, ncombo, relu);
  return hipGetLastError();
}
template <int Q, int NT, int QH, int HM>
hipError_t launch_conv_fused_t(const float2* wc, const float* x, const float* bias, float* y, int N, int C_out, int H,
                               int W, int Ho, int Wo, int pad, int ncombo, int relu, hipStream_t s) {
  if (W % 4 != 0 || Wo % 2 != 0)
    return launch_conv_fused_r<Q, NT, QH, HM, true>(wc, x, bias, y, N, C_out, H, W, Ho, Wo, pad, ncombo, relu, s);
  return launch_conv_fused_r<Q, NT, QH, HM, false>(wc, x, bias, y, N, C_out, H, W, Ho, Wo, pad, ncombo, relu, s);
}

// Up to 4 (slot group, row group) combinations (p <= 8) run as workgroups of 256 threads with one
// channel block of spectra in LDS at a time: two such workgroups share a CU, so the loads and
// stores of one overlap the transforms and the contraction of the other.  More combinations need
// the 8 waves of a 512-thread workgroup.
template <int Q, int HM>
hipError_t launch_conv_fused_q(const float2* wc, const float* x, const float* bias, float* y, int N, int C_out, int H,
                               int W, int Ho, int Wo, int pad, int ncombo, int relu, hipStream_t s) {
  // ... provided there are enough of them for two per CU; a grid that leaves most CUs with one
  // workgroup is served faster by the larger workgroups (twice the waves on every serial phase)
  ConvTilePlan pl;
  const bool small_wg = ncombo <= 4 && plan_conv_tile<64, 256>(C_out / 64, 1, 3, Ho, Wo, ncombo, pl) &&
                        (long long)cdiv(N, 2) * pl.tiles_h * pl.tiles_w >= 384;
  if (small_wg)
    return launch_conv_fused_t<Q, 256, 1, HM>(wc, x, bias, y, N, C_out, H, W, Ho, Wo, pad, ncombo, relu, s);
  return launch_conv_fused_t<Q, 512, (Q % 2 == 0 ? 2 : 1), HM>(wc, x, bias, y, N, C_out, H, W, Ho, Wo, pad, ncombo, relu, s);
}

}  // namespace

namespace {

// The fused CONV kernel serves k = 64, 3x3 filters, 1, 2, 3, 4, 6 or 8 input channel blocks and up
// to 16 output channel blocks; it keeps offsets inside an image pair in 32 bits.  p, q: output / input channel blocks; H x W the
// input image, Ho x Wo the output image.
inline bool conv_fused_applicable(int p, int q, int k, int r, int N, int H, int W, int Ho, int Wo) {
  const long long HW = (long long)H * W, HWo = (long long)Ho * Wo;
  return conv_fused_ncombo(p, q, k, r) > 0 && Wo >= 2 && 2 * (long long)q * k * HW < (1ll << 31) &&
         2 * (long long)p * k * HWo < (1ll << 31) && (long long)cdiv(N, 2) * HWo < (1ll << 31);
}

// HM: 0 fp32, 1 fp16, 2 bfloat16 activations (x, y then point to the 16-bit data)
template <int HM>
hipError_t launch_conv_fused_h(const float2* wc, const float* x, const float* bias, float* y, int N, int p, int q, int k,
                               int r, int H, int W, int Ho, int Wo, int pad, int relu, hipStream_t s) {
  const int ncombo = conv_fused_ncombo(p, q, k, r), C_out = p * k;
  switch (q) {
    case 1: return launch_conv_fused_q<1, HM>(wc, x, bias, y, N, C_out, H, W, Ho, Wo, pad, ncombo, relu, s);
    case 2: return launch_conv_fused_q<2, HM>(wc, x, bias, y, N, C_out, H, W, Ho, Wo, pad, ncombo, relu, s);
    case 3: return launch_conv_fused_q<3, HM>(wc, x, bias, y, N, C_out, H, W, Ho, Wo, pad, ncombo, relu, s);
    case 4: return launch_conv_fused_q<4, HM>(wc, x, bias, y, N, C_out, H, W, Ho, Wo, pad, ncombo, relu, s);
    case 6: return launch_conv_fused_q<6, HM>(wc, x, bias, y, N, C_out, H, W, Ho, Wo, pad, ncombo, relu, s);
    case 8: return launch_conv_fused_q<8, HM>(wc, x, bias, y, N, C_out, H, W, Ho, Wo, pad, ncombo, relu, s);
    default: return hipErrorInvalidValue;
  }
}
hipError_t launch_conv_fused(const float2* wc, const float* x, const float* bias, float* y, int N, int p, int q, int k,
                             int r, int H, int W, int Ho, int Wo, int pad, int relu, hipStream_t s) {
  return launch_conv_fused_h<0>(wc, x, bias, y, N, p, q, k, r, H, W, Ho, Wo, pad, relu, s);
}

}  // namespace

namespace {

// Unfused CONV contraction.  pout output and qin input channel blocks; a thread keeps 4 output
// blocks of its pixel, or 8 when there are more than 4: each spectrum value it loads and each
// tap's index arithmetic then serve twice the products, and 5..7 output blocks no longer cost a
// second, mostly empty pass over the input (6 x 6 blocks of 64, 26 x 26 stride 2, batch 32:
// 66 -> 37 us).
hipError_t launch_conv_contract(const float2* what, const float2* xh, float2* yh, int pout, int qin, int NF, int N, int H,
                                int W, int Ho, int Wo, int r, int pad, int flip, int stride, int dil, hipStream_t s) {
  const long long npix = (long long)N * Ho * Wo;
  if (pout > 4) {
    dim3 grid((unsigned)cdiv(npix, 256), (unsigned)NF, (unsigned)cdiv(pout, 8));
    hipLaunchKernelGGL((conv_contract_kernel<8>), grid, dim3(256), 0, s, what, xh, yh, pout, qin, NF, N, H, W, Ho, Wo, r, pad,
                       flip, stride, dil);
  } else {
    dim3 grid((unsigned)cdiv(npix, 256), (unsigned)NF, 1);
    hipLaunchKernelGGL((conv_contract_kernel<4>), grid, dim3(256), 0, s, what, xh, yh, pout, qin, NF, N, H, W, Ho, Wo, r, pad,
                       flip, stride, dil);
  }
  return hipGetLastError();
}

}  // namespace

extern "C" {

// Output positions along one axis (the filter is placed every `stride` pixels while it fits the
// zero-padded input).
static int conv_out(int n, int r, int pad, int stride) { return (n + 2 * pad - r) / stride + 1; }

static bool conv_dims_ok(int N, int C_in, int C_out, int H, int W, int r, int pad, int k) {
  if (N <= 0 || C_in <= 0 || C_out <= 0 || H <= 0 || W <= 0 || r <= 0 || !valid_k(k)) return false;
  if (C_in % k || C_out % k) return false;
  if (pad < 0 || pad >= r) return false;
  if (H + 2 * pad < r || W + 2 * pad < r) return false;
  long long pix = (long long)N * H * W;
  if (pix * (C_in / k) > (1ll << 31) - 1 || pix * (C_out / k) > (1ll << 31) - 1) return false;
  if (r * r > 65535 || (C_out / k) > 65535 * 4 || k / 2 + 1 > 65535) return false;
  return true;
}

size_t circ_conv_workspace_bytes(int N, int C_in, int C_out, int H, int W, int r, int stride, int pad, int k) {
  if (!conv_dims_ok(N, C_in, C_out, H, W, r, pad, k) || stride < 1) return 0;
  const int Ho = conv_out(H, r, pad, stride), Wo = conv_out(W, r, pad, stride);
  size_t xa = align_up(spectrum_elems(k, (long long)(C_in / k) * N * H * W) * sizeof(float2), 256);
  size_t ya = align_up(spectrum_elems(k, (long long)(C_out / k) * N * Ho * Wo) * sizeof(float2), 256);
  return xa + ya;
}

circ_status circ_conv_forward(const void* w_hat, const float* x, const float* bias, float* y, int N, int C_in,
                              int C_out, int H, int W, int r, int stride, int pad, int k, int epilogue,
                              void* workspace, size_t workspace_bytes, void* stream) {
  if (!conv_dims_ok(N, C_in, C_out, H, W, r, pad, k)) return CIRC_EINVAL;
  if (stride <= 0) return CIRC_EINVAL;
  if (!w_hat || !x || !y) return CIRC_EINVAL;
  if (epilogue & ~(CIRC_EPI_BIAS | CIRC_EPI_RELU)) return CIRC_EINVAL;
  const bool use_bias = epilogue & CIRC_EPI_BIAS;
  if (use_bias && !bias) return CIRC_EINVAL;
  if (!aligned16(w_hat) || !aligned16(x) || !aligned16(y) || (use_bias && !aligned16(bias))) return CIRC_EINVAL;
  const int Ho = conv_out(H, r, pad, stride), Wo = conv_out(W, r, pad, stride);
  const size_t xbytes = size_t(N) * C_in * H * W * sizeof(float), ybytes = size_t(N) * C_out * Ho * Wo * sizeof(float);
  if (overlaps(x, xbytes, y, ybytes)) return CIRC_EINVAL;
  const size_t need = circ_conv_workspace_bytes(N, C_in, C_out, H, W, r, stride, pad, k);
  if (!workspace || workspace_bytes < need) return CIRC_EWORKSPACE;
  if (!aligned16(workspace)) return CIRC_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);

  const int p = C_out / k, q = C_in / k, NF = k / 2 + 1;
  const long long HW = (long long)H * W, HWo = (long long)Ho * Wo;
  if (stride == 1 && conv_fused_applicable(p, q, k, r, N, H, W, Ho, Wo)) {
    const float2* wc = blob_at<float2>(w_hat, blob_layout(r * r, p, q, k).conv);
    return launch_conv_fused(wc, x, use_bias ? bias : nullptr, y, N, p, q, k, r, H, W, Ho, Wo, pad,
                             (epilogue & CIRC_EPI_RELU) ? 1 : 0, s) == hipSuccess ? CIRC_OK : CIRC_EHIP;
  }
  const long long xrows = (long long)q * N * HW, yrows = (long long)p * N * HWo;
  float2* xh = static_cast<float2*>(workspace);
  float2* yh = reinterpret_cast<float2*>(static_cast<char*>(workspace) +
                                         align_up(spectrum_elems(k, xrows) * sizeof(float2), 256));
  // X^[f][j][n][pixel]: the FFT runs down the channel axis (element stride H*W)
  RowMap mx{(int)HW, N, 1, (long long)C_in * HW, (long long)k * HW, HW, HW % 4 == 0};
  if (launch_rfft(k, true, x, xh, mx, xrows, xrows, 1, 0, 0, 1.0f, 0, s) != hipSuccess) return CIRC_EHIP;
  if (launch_conv_contract(static_cast<const float2*>(w_hat), xh, yh, p, q, NF, N, H, W, Ho, Wo, r, pad, 0, stride, 1, s) !=
      hipSuccess)
    return CIRC_EHIP;
  RowMap my{(int)HWo, N, 1, (long long)C_out * HWo, (long long)k * HWo, HWo, HWo % 4 == 0};
  if (launch_irfft(k, true, yh, y, my, yrows, yrows, 1.0f, use_bias ? bias : nullptr, (long long)N * HWo,
                   (epilogue & CIRC_EPI_RELU) ? 1 : 0, s) != hipSuccess)
    return CIRC_EHIP;
  return CIRC_OK;
}


// Output pixels per block of conv_dw_mfma_kernel: at least 2048 (so that the block-wide sum at the
// end stays small beside the pixel loop) and at most 16 chunks (their partial spectra are added
// one after the other by the inverse FFT).
static long long conv_dw_pix_per_block(long long npix) {
  long long ppb = 2048;
  while (cdiv(npix, ppb) > 16) ppb *= 2;
  return ppb;
}

// Weight-gradient reduction of a CONV layer: the kernel with the input spectra staged in LDS when
// a band of rows of 4 input blocks fits 48 KB, else the one that reads every tap from global memory.
struct ConvDwPlan {
  bool lds;
  int ng, BR, nbands, cpb, nparts;
  size_t lds_bytes;
  long long ppb;
};
static ConvDwPlan plan_conv_dw(int N, int H, int W, int Ho, int Wo, int r, int pad, int stride) {
  ConvDwPlan pl{};
  const long long npix = (long long)N * Ho * Wo;
  pl.ppb = conv_dw_pix_per_block(npix);
  pl.nparts = (int)cdiv(npix, pl.ppb);
  pl.ng = 16;                                                      // offsets per block of the LDS kernel
  // a band of BR output rows needs (BR-1)*stride + r padded input rows of 4 input blocks and
  // BR rows of 4 output blocks
  const long long Wp = W + 2 * pad, el = 4 * (long long)sizeof(float2), budget = 40 * 1024;
  const long long first = el * (r * Wp + Wo), more = el * (stride * Wp + Wo);   // bytes of one row, of every further row
  // (W or Wo of 1: ceil(2^32 / 1) does not fit the 32-bit multipliers of the kernel)
  if (first > budget || (long long)N * Ho > (1ll << 30) || W < 2 || Wo < 2) return pl;
  const long long fit = 1 + (budget - first) / more;
  const int BR = (int)(fit < Ho ? fit : Ho);
  pl.nbands = (int)cdiv(Ho, BR);
  pl.BR = (int)cdiv(Ho, pl.nbands);                                // bands of equal height
  pl.nbands = (int)cdiv(Ho, pl.BR);
  const long long total = (long long)N * pl.nbands;
  pl.cpb = (int)cdiv(total, 32);                                   // at most 32 partial spectra
  pl.nparts = (int)cdiv(total, pl.cpb);
  pl.lds_bytes = size_t(4) * (dw_plane_stride(int(((pl.BR - 1) * stride + r) * Wp)) + dw_plane_stride(pl.BR * Wo)) * sizeof(float2);
  if (pl.lds_bytes < 8192) pl.lds_bytes = 8192;                    // room for the sums over the four waves
  pl.lds = true;
  return pl;
}

size_t circ_conv_backward_workspace_bytes(int N, int C_in, int C_out, int H, int W, int r, int stride, int pad, int k) {
  if (!conv_dims_ok(N, C_in, C_out, H, W, r, pad, k) || stride < 1) return 0;
  const int Ho = conv_out(H, r, pad, stride), Wo = conv_out(W, r, pad, stride);
  const int p = C_out / k, q = C_in / k;
  const size_t xa = align_up(spectrum_elems(k, (long long)q * N * H * W) * sizeof(float2), 256);
  const size_t ya = align_up(spectrum_elems(k, (long long)p * N * Ho * Wo) * sizeof(float2), 256);
  const long long npix = (long long)N * Ho * Wo;
  const size_t wa = align_up(spectrum_elems(k, (long long)r * r * p * q) * sizeof(float2), 256);
  (void)npix;
  return xa + ya + wa * size_t(plan_conv_dw(N, H, W, Ho, Wo, r, pad, stride).nparts);
}

}  // extern "C"

namespace {

// CONV backward; dw / w_upd as in fc_backward_impl.
// the channel-axis transforms with 16-bit rows (defined with the other 16-bit code below)
hipError_t launch_rfft_chan16(int k, bool bf, const void* in, float2* out, const RowMap& map, long long nrows,
                              long long out_fstride, hipStream_t s);
hipError_t launch_irfft_chan16(int k, bool bf, const float2* in, void* out, const RowMap& map, long long nrows,
                               long long in_fstride, const float* bias, long long bias_div, int relu, hipStream_t s);
inline bool half_k(int k);

// hm: 0 = fp32 activations; 1 (fp16) / 2 (bfloat16): x, dy and dx point to 16-bit values (all
// spectra, the weight gradient and the blob stay fp32)
circ_status conv_backward_impl(const void* w_hat, const float* x, const float* dy, float* dx, float* dw, void* w_upd,
                               float lr, int N, int C_in, int C_out, int H, int W, int r, int stride, int pad, int k,
                               void* workspace, size_t workspace_bytes, void* stream, int hm = 0) {
  if (!conv_dims_ok(N, C_in, C_out, H, W, r, pad, k)) return CIRC_EINVAL;
  if (hm != 0 && !half_k(k)) return CIRC_EINVAL;
  const bool bf = hm == 2;
  const size_t esz = hm ? sizeof(__half) : sizeof(float);
  if (stride <= 0) return CIRC_EINVAL;
  const bool want_dw = dw || w_upd;
  if (!w_hat || !dy || (!dx && !want_dw) || (want_dw && !x)) return CIRC_EINVAL;
  if (!aligned16(w_hat) || !aligned16(dy) || !aligned16(x) || !aligned16(dx) || !aligned16(dw)) return CIRC_EINVAL;
  const int Ho = conv_out(H, r, pad, stride), Wo = conv_out(W, r, pad, stride);
  const int p = C_out / k, q = C_in / k, NF = k / 2 + 1;
  // offsets inside one frequency of a spectrum are kept in 32 bits; grid.z holds tiles x offsets
  if ((long long)p * N * Ho * Wo > (1ll << 31) - 1 || (long long)r * r * cdiv(p, 4) * cdiv(q, 4) > 65535) return CIRC_EINVAL;
  const size_t xbytes = size_t(N) * C_in * H * W * esz, ybytes = size_t(N) * C_out * Ho * Wo * esz;
  const size_t wbytes = size_t(r) * r * p * q * k * sizeof(float);
  if (dx && (overlaps(dx, xbytes, dy, ybytes) || (x && overlaps(dx, xbytes, x, xbytes)))) return CIRC_EINVAL;
  if (dw && (overlaps(dw, wbytes, dy, ybytes) || overlaps(dw, wbytes, x, xbytes))) return CIRC_EINVAL;
  if (dx && dw && overlaps(dx, xbytes, dw, wbytes)) return CIRC_EINVAL;
  if (w_upd) {   // the blob is rewritten: none of the operands may lie inside it
    const size_t bbytes = circ_spectra_bytes(r * r, p, q, k);
    if (overlaps(w_upd, bbytes, x, xbytes) || overlaps(w_upd, bbytes, dy, ybytes) || (dx && overlaps(w_upd, bbytes, dx, xbytes)) ||
        (dw && overlaps(w_upd, bbytes, dw, wbytes)))
      return CIRC_EINVAL;
  }
  const size_t need = circ_conv_backward_workspace_bytes(N, C_in, C_out, H, W, r, stride, pad, k);
  if (!workspace || workspace_bytes < need) return CIRC_EWORKSPACE;
  if (!aligned16(workspace)) return CIRC_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);

  const long long HW = (long long)H * W, HWo = (long long)Ho * Wo;
  const long long xrows = (long long)q * N * HW, yrows = (long long)p * N * HWo;
  const size_t xa = align_up(spectrum_elems(k, xrows) * sizeof(float2), 256);
  const size_t ya = align_up(spectrum_elems(k, yrows) * sizeof(float2), 256);
  float2* xh = static_cast<float2*>(workspace);
  float2* yh = reinterpret_cast<float2*>(static_cast<char*>(workspace) + xa);
  float2* wpart = reinterpret_cast<float2*>(static_cast<char*>(workspace) + xa + ya);
  const BlobLayout bl = blob_layout(r * r, p, q, k);

  // backward-data: the fused forward kernel on the transposed grids when the shape allows it
  // (q output blocks, p input blocks, input image Ho x Wo, output image H x W, padding r-1-pad)
  const bool dx_fused = dx && stride == 1 && conv_fused_applicable(q, p, k, r, N, Ho, Wo, H, W);
  if (dx_fused) {
    const float2* wcb = blob_at<float2>(w_hat, bl.conv_bwd);
    const hipError_t e = hm == 0 ? launch_conv_fused_h<0>(wcb, dy, nullptr, dx, N, q, p, k, r, Ho, Wo, H, W, r - 1 - pad, 0, s)
                       : hm == 1 ? launch_conv_fused_h<1>(wcb, dy, nullptr, dx, N, q, p, k, r, Ho, Wo, H, W, r - 1 - pad, 0, s)
                                 : launch_conv_fused_h<2>(wcb, dy, nullptr, dx, N, q, p, k, r, Ho, Wo, H, W, r - 1 - pad, 0, s);
    if (e != hipSuccess) return CIRC_EHIP;
  }
  // dY^[f][i][n][pixel]: the FFT runs down the channel axis of dy
  RowMap my{(int)HWo, N, 1, (long long)C_out * HWo, (long long)k * HWo, HWo, HWo % 4 == 0};
  if (want_dw || (dx && !dx_fused)) {
    if ((hm ? launch_rfft_chan16(k, bf, dy, yh, my, yrows, yrows, s) : launch_rfft(k, true, dy, yh, my, yrows, yrows, 1, 0, 0, 1.0f, 0, s)) !=
        hipSuccess)
      return CIRC_EHIP;
  }
  RowMap mx{(int)HW, N, 1, (long long)C_in * HW, (long long)k * HW, HW, HW % 4 == 0};
  if (dx && !dx_fused) {
    // forward contraction on the transposed, conjugated section with reflected offsets:
    // q output blocks, p input blocks, input image Ho x Wo, output image H x W, padding r-1-pad
    if (launch_conv_contract(blob_at<float2>(w_hat, bl.bwd), yh, xh, q, p, NF, N, Ho, Wo, H, W, r, r - 1 - pad, 1, 1, stride,
                             s) != hipSuccess)
      return CIRC_EHIP;
    if ((hm ? launch_irfft_chan16(k, bf, xh, dx, mx, xrows, xrows, nullptr, 1, 0, s)
            : launch_irfft(k, true, xh, dx, mx, xrows, xrows, 1.0f, nullptr, 1, 0, s)) != hipSuccess)
      return CIRC_EHIP;
  }
  if (want_dw) {
    if ((hm ? launch_rfft_chan16(k, bf, x, xh, mx, xrows, xrows, s) : launch_rfft(k, true, x, xh, mx, xrows, xrows, 1, 0, 0, 1.0f, 0, s)) !=
        hipSuccess)
      return CIRC_EHIP;
    const ConvDwPlan dpl = plan_conv_dw(N, H, W, Ho, Wo, r, pad, stride);
    const long long npix = (long long)N * HWo, ppb = dpl.ppb;
    const int nchunks = dpl.nparts;
    const long long wrows = (long long)r * r * p * q;
    const long long wstride = (long long)(align_up(spectrum_elems(k, wrows) * sizeof(float2), 256) / sizeof(float2));
    constexpr int kDwOffsets = 3;   // consecutive filter offsets per block of conv_dw_mfma_kernel
    // exact division of the pixel index by a multiply-high: q = (pix * ceil(2^32/d)) >> 32 equals
    // pix / d whenever pix * d < 2^32 (the rounding excess of the multiplier, below d, times pix
    // stays below 2^32)
    auto fast_mul = [](long long limit, long long d) -> unsigned {
      if (d <= 1 || limit * d >= (1ll << 32)) return 0u;
      return (unsigned)(((1ll << 32) + d - 1) / d);
    };
    const unsigned mul_hwo = fast_mul(npix, HWo), mul_wo = fast_mul(HWo, Wo);
    // staged element index / W: indices stay below 48 KB / 32 B, so the multiply-high is exact
    const unsigned mul_w = (unsigned)(((1ll << 32) + W - 1) / W);
    if (dpl.lds) {
      const unsigned mul_wo_b = (unsigned)(((1ll << 32) + Wo - 1) / Wo);   // pixel index inside a band / Wo
      // tiles of 2 x 2 channel blocks (one matrix instruction per pixel) or of 4 x 4 (four per
      // pixel): a 2 x 2 tile measures about 0.65 of the time of a 4 x 4 tile (staging and LDS
      // reads, not the matrix instructions, set the pace), so the small tiles win only where they
      // are fewer than 1.5 times as many: layers with at most 2 blocks on either side
      const long long t2 = cdiv(p, 2) * cdiv(q, 2), t4 = cdiv(p, 4) * cdiv(q, 4);
      if (2 * t2 < 3 * t4 && cdiv(r * r, 16) * t2 <= 65535) {
        dim3 grid((unsigned)dpl.nparts, (unsigned)NF, (unsigned)(cdiv(r * r, 16) * t2));
        hipLaunchKernelGGL((conv_dw_lds_kernel<true>), grid, dim3(256), dpl.lds_bytes, s, yh, xh, wpart, p, q, NF, N, H, W, Ho,
                           Wo, r, pad, dpl.BR, dpl.nbands, dpl.cpb, wstride, mul_wo_b, mul_w, stride);
      } else {
        dim3 grid((unsigned)dpl.nparts, (unsigned)NF, (unsigned)(cdiv(r * r, 16) * t4));
        hipLaunchKernelGGL((conv_dw_lds_kernel<false>), grid, dim3(256), dpl.lds_bytes, s, yh, xh, wpart, p, q, NF, N, H, W, Ho,
                           Wo, r, pad, dpl.BR, dpl.nbands, dpl.cpb, wstride, mul_wo_b, mul_w, stride);
      }
    } else if (r % kDwOffsets == 0) {   // kDwOffsets consecutive offsets per block (for r = 3: one filter row)
      dim3 grid((unsigned)nchunks, (unsigned)NF, (unsigned)(r * r / kDwOffsets * cdiv(p, 4) * cdiv(q, 4)));
      hipLaunchKernelGGL((conv_dw_mfma_kernel<kDwOffsets>), grid, dim3(256), 0, s, yh, xh, wpart, p, q, NF, N, H, W, Ho, Wo,
                         r, pad, ppb, wstride, mul_hwo, mul_wo, stride);
    } else {            // one offset per block
      dim3 grid((unsigned)nchunks, (unsigned)NF, (unsigned)(r * r * cdiv(p, 4) * cdiv(q, 4)));
      hipLaunchKernelGGL((conv_dw_mfma_kernel<1>), grid, dim3(256), 0, s, yh, xh, wpart, p, q, NF, N, H, W, Ho, Wo, r, pad,
                         ppb, wstride, mul_hwo, mul_wo, stride);
    }
    if (hipGetLastError() != hipSuccess) return CIRC_EHIP;
    // many partial spectra are folded into the first one by a launch of their own (one thread per
    // value, fixed order); a few are added by the consumer while it loads them
    int nsum = nchunks;
    if (nchunks > 8) {
      const long long nval = 2 * (long long)spectrum_elems(k, wrows);
      hipLaunchKernelGGL(sum_parts_kernel, dim3((unsigned)cdiv(nval, 256)), dim3(256), 0, s, reinterpret_cast<float*>(wpart),
                         nchunks, 2 * wstride, nval);
      if (hipGetLastError() != hipSuccess) return CIRC_EHIP;
      nsum = 1;
    }
    // dw[g][i][j][:] = IFFT over f of the summed partial spectra, scale 1/k
    RowMap mw{(int)wrows, 1, (long long)k, 0, 0, 1};
    if (dw && launch_irfft(k, false, wpart, dw, mw, wrows, wrows, 1.0f / float(k), nullptr, 1, 0, s, nsum, wstride) != hipSuccess)
      return CIRC_EHIP;
    if (w_upd) return apply_spectra_step(w_upd, wpart, nsum, wstride, wrows, (long long)p * q, r * r, p, q, k, lr, s);
  }
  return CIRC_OK;
}

}  // namespace

extern "C" {

circ_status circ_conv_backward(const void* w_hat, const float* x, const float* dy, float* dx, float* dw, int N, int C_in,
                               int C_out, int H, int W, int r, int stride, int pad, int k, void* workspace,
                               size_t workspace_bytes, void* stream) {
  if (!dx && !dw) return CIRC_EINVAL;
  return conv_backward_impl(w_hat, x, dy, dx, dw, nullptr, 0.f, N, C_in, C_out, H, W, r, stride, pad, k, workspace,
                            workspace_bytes, stream);
}

circ_status circ_conv_sgd_step(void* w_hat, const float* x, const float* dy, float* dx, float lr, int N, int C_in,
                               int C_out, int H, int W, int r, int stride, int pad, int k, void* workspace,
                               size_t workspace_bytes, void* stream) {
  if (!w_hat || !(lr == lr)) return CIRC_EINVAL;   // NaN step
  return conv_backward_impl(w_hat, x, dy, dx, nullptr, w_hat, lr, N, C_in, C_out, H, W, r, stride, pad, k, workspace,
                            workspace_bytes, stream);
}

circ_status circ_bias_grad(const float* dy, float* db, long long outer, int channels, long long inner, void* stream) {
  if (!dy || !db || outer <= 0 || channels <= 0 || inner <= 0) return CIRC_EINVAL;
  if (!aligned16(dy) || !aligned16(db)) return CIRC_EINVAL;
  if (outer > (1ll << 40) / channels / inner) return CIRC_EINVAL;
  const size_t ybytes = size_t(outer) * channels * inner * sizeof(float);
  if (overlaps(db, size_t(channels) * sizeof(float), dy, ybytes)) return CIRC_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (inner == 1)
    hipLaunchKernelGGL(bias_grad_column_kernel, dim3((unsigned)cdiv(channels, 64)), dim3(1024), 0, s, dy, db, outer, channels);
  else
    hipLaunchKernelGGL(bias_grad_channel_kernel, dim3((unsigned)channels), dim3(1024), 0, s, dy, db, outer, channels, inner,
                       int(inner % 4 == 0 && outer * inner < (1ll << 32)));
  return hipGetLastError() == hipSuccess ? CIRC_OK : CIRC_EHIP;
}

}  // extern "C"

// ---- half-width storage (16-bit values in memory, fp32 arithmetic): FC forward and backward ----
namespace {

inline bool half_k(int k) { return is_pow2(k) && k >= 8 && k <= kMaxK; }

// hmode: kHalfSpectra (fp32 rows in) or kHalfSpectra | kHalfRows; bf: bfloat16 instead of fp16
template <int K>
hipError_t launch_rfft_half_k(int hmode, bool bf, const void* in, void* out, const RowMap& map, long long nrows,
                              long long out_fstride, float scale, int conj, hipStream_t s) {
  FftPlan pl = plan_fft(K, nrows);
  dim3 grid((unsigned)cdiv(nrows, 2 * pl.P), 1);
  const float* fin = static_cast<const float*>(in);
  float2* fout = static_cast<float2*>(out);
#define CIRC_RFFT_H(MODE)                                                                                              \
  if (!launch_rfft_stream<K, MODE>(fin, fout, map, nrows, out_fstride, scale, conj, s))                                \
  hipLaunchKernelGGL((rfft_kernel<K, false, MODE>), grid, dim3(pl.NT), pl.lds, s, fin, fout, map, nrows, out_fstride, 0ll, \
                     0ll, pl.P, scale, conj)
  if (hmode == kHalfSpectra) {
    if (bf) { CIRC_RFFT_H(kHalfSpectra | kHalfBf16); }
    else { CIRC_RFFT_H(kHalfSpectra); }
  } else {
    if (bf) { CIRC_RFFT_H(kHalfSpectra | kHalfRows | kHalfBf16); }
    else { CIRC_RFFT_H(kHalfSpectra | kHalfRows); }
  }
#undef CIRC_RFFT_H
  return hipGetLastError();
}

template <int K>
hipError_t launch_irfft_half_k(bool bf, const void* in, void* out, const RowMap& map, long long nrows, long long in_fstride,
                               float scale, const float* bias, long long bias_div, int relu, hipStream_t s) {
  const float2* fin = static_cast<const float2*>(in);
  float* fout = static_cast<float*>(out);
  if constexpr (stream_k<K>()) {
    // long runs of contiguous rows: the streaming form
    constexpr int P = 4096 / K;
    const long long ntiles = cdiv(nrows, 2 * P);
    if (ntiles >= kStreamMinTiles && ntiles <= (1ll << 31) - 1 && (nrows & 1) == 0 && (in_fstride & 1) == 0 && aligned16(in)) {
      const unsigned sgrid = unsigned(ntiles < kStreamMaxWorkgroups ? ntiles : kStreamMaxWorkgroups);
      if (bf)
        hipLaunchKernelGGL((irfft_stream_kernel<K, kHalfSpectra | kHalfRows | kHalfBf16>), dim3(sgrid), dim3(256), fft_tile_lds_bytes(K, P),
                           s, fin, fout, map, nrows, in_fstride, int(ntiles), scale, bias, bias_div, relu);
      else
        hipLaunchKernelGGL((irfft_stream_kernel<K, kHalfSpectra | kHalfRows>), dim3(sgrid), dim3(256), fft_tile_lds_bytes(K, P), s, fin,
                           fout, map, nrows, in_fstride, int(ntiles), scale, bias, bias_div, relu);
      return hipGetLastError();
    }
  }
  FftPlan pl = plan_fft(K, nrows);
  dim3 grid((unsigned)cdiv(nrows, 2 * pl.P));
  if (bf)
    hipLaunchKernelGGL((irfft_kernel<K, false, kHalfSpectra | kHalfRows | kHalfBf16>), grid, dim3(pl.NT), pl.lds, s, fin, fout,
                       map, nrows, in_fstride, pl.P, scale, bias, bias_div, relu, 1, 0ll);
  else
    hipLaunchKernelGGL((irfft_kernel<K, false, kHalfSpectra | kHalfRows>), grid, dim3(pl.NT), pl.lds, s, fin, fout, map, nrows,
                       in_fstride, pl.P, scale, bias, bias_div, relu, 1, 0ll);
  return hipGetLastError();
}

#define CIRC_DISPATCH_HALF_K(k, CALL) \
  switch (k) {                        \
    case 8: return CALL(8);           \
    case 16: return CALL(16);         \
    case 32: return CALL(32);         \
    case 64: return CALL(64);         \
    case 128: return CALL(128);       \
    case 256: return CALL(256);       \
    case 512: return CALL(512);       \
    default: return hipErrorInvalidValue; \
  }

hipError_t launch_rfft_half(int k, int hmode, bool bf, const void* in, void* out, const RowMap& map, long long nrows,
                            long long out_fstride, float scale, hipStream_t s, int conj = 0) {
#define CALL(KK) launch_rfft_half_k<KK>(hmode, bf, in, out, map, nrows, out_fstride, scale, conj, s)
  CIRC_DISPATCH_HALF_K(k, CALL)
#undef CALL
}

hipError_t launch_irfft_half(int k, bool bf, const void* in, void* out, const RowMap& map, long long nrows,
                             long long in_fstride, float scale, const float* bias, long long bias_div, int relu,
                             hipStream_t s) {
#define CALL(KK) launch_irfft_half_k<KK>(bf, in, out, map, nrows, in_fstride, scale, bias, bias_div, relu, s)
  CIRC_DISPATCH_HALF_K(k, CALL)
#undef CALL
}

// C[f][m][n] = scale * sum_k A[f][m][k] B[f][n][k] on 16-bit operands; TB: B is stored [f][k][n]
template <bool TB>
hipError_t launch_cgemm_h(bool bf, hipStream_t s, int NF, const __half2* A, const __half2* B, __half2* C, int M, int N, int Kd,
                          long long sA, long long sB, long long sC, float scale) {
  dim3 grid((unsigned)cdiv(N, 128), (unsigned)cdiv(M, 64), (unsigned)NF);
  const bool vec = Kd % 4 == 0 && (!TB || N % 4 == 0);
  if (vec) {
    if (bf) hipLaunchKernelGGL((cgemm_h_kernel<true, true, TB>), grid, dim3(256), 0, s, A, B, C, M, N, Kd, sA, sB, sC, scale);
    else hipLaunchKernelGGL((cgemm_h_kernel<true, false, TB>), grid, dim3(256), 0, s, A, B, C, M, N, Kd, sA, sB, sC, scale);
  } else {
    if (bf) hipLaunchKernelGGL((cgemm_h_kernel<false, true, TB>), grid, dim3(256), 0, s, A, B, C, M, N, Kd, sA, sB, sC, scale);
    else hipLaunchKernelGGL((cgemm_h_kernel<false, false, TB>), grid, dim3(256), 0, s, A, B, C, M, N, Kd, sA, sB, sC, scale);
  }
  return hipGetLastError();
}

inline size_t half_spectrum_bytes(int k, long long rows) { return align_up(size_t(k / 2 + 1) * size_t(rows) * sizeof(__half2), 256); }

// bytes of the fused kernel's 16-bit operand section for a p x q grid (0 where that kernel does not apply)
inline size_t half_fused_bytes(int p, int q, int k) {
  if (fused_it(k) == 0) return 0;
  return align_up(size_t(fused_igp(p, k)) * fused_q2p(q, k) * (k / 32) * 64 * sizeof(uint2), 256);
}
// 16-bit blob: W^[f][i][j], conj(W^)[f][j][i], then the fused kernel's operand order of either,
// then the batch <= 2 kernel's
struct HalfBlob { size_t fwd, bwd, fused_fwd, fused_bwd, gemv_fwd, gemv_bwd, total; };
inline HalfBlob half_blob(int p, int q, int k) {
  HalfBlob b;
  const size_t sec = half_spectrum_bytes(k, (long long)p * q);
  b.fwd = 0;
  b.bwd = sec;
  b.fused_fwd = 2 * sec;
  b.fused_bwd = b.fused_fwd + half_fused_bytes(p, q, k);
  // one word per value in the order of the batch <= 2 kernel, either orientation
  const size_t gsec = align_up(size_t(p) * q * (k / 2) * sizeof(unsigned), 256);
  b.gemv_fwd = b.fused_bwd + half_fused_bytes(q, p, k);
  b.gemv_bwd = b.gemv_fwd + gsec;
  b.total = b.gemv_bwd + gsec;
  return b;
}

size_t spectra_bytes_half(int p, int q, int k) {
  if (p <= 0 || q <= 0 || !half_k(k) || (long long)p * q > (1ll << 31) - 1) return 0;
  return half_blob(p, q, k).total;
}

circ_status precompute_spectra_half(bool bf, const float* w, int p, int q, int k, void* w_hat, void* stream) {
  if (!w || !w_hat || p <= 0 || q <= 0 || !half_k(k)) return CIRC_EINVAL;
  if ((long long)p * q > (1ll << 31) - 1) return CIRC_EINVAL;
  if (!aligned16(w) || !aligned16(w_hat)) return CIRC_EINVAL;
  if (overlaps(w, size_t(p) * q * k * sizeof(float), w_hat, spectra_bytes_half(p, q, k))) return CIRC_EINVAL;
  const long long rows = (long long)p * q;
  // W^[f][i][j] = FFT(w_ij)[f], not normalised (the 1/k is applied after the contraction, in fp32):
  // row id = i*q + j -> w[i][j][:]
  RowMap mw{q, p, (long long)k, (long long)q * k, 0, 1};
  if (launch_rfft_half(k, kHalfSpectra, bf, w, w_hat, mw, rows, rows, 1.0f, static_cast<hipStream_t>(stream)) != hipSuccess)
    return CIRC_EHIP;
  // conj(W^)[f][j][i] for backward-data (the transposed grid): row id = j*p + i -> w[i][j][:]
  RowMap mt{p, q, (long long)q * k, (long long)k, 0, 1};
  void* sec2 = static_cast<char*>(w_hat) + half_spectrum_bytes(k, rows);
  if (launch_rfft_half(k, kHalfSpectra, bf, w, sec2, mt, rows, rows, 1.0f, static_cast<hipStream_t>(stream), 1) != hipSuccess)
    return CIRC_EHIP;
  const HalfBlob hb = half_blob(p, q, k);
  char* base = static_cast<char*>(w_hat);
  for (int dir = 0; dir < 2; ++dir) {   // operand order of the batch <= 2 kernel
    const int pp = dir ? q : p, qq = dir ? p : q;
    const long long total = (long long)pp * qq * (k / 2);
    hipLaunchKernelGGL(pack_gemv_half_kernel, dim3((unsigned)cdiv(total, 256)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       reinterpret_cast<const unsigned*>(base + (dir ? hb.bwd : hb.fwd)),
                       reinterpret_cast<unsigned*>(base + (dir ? hb.gemv_bwd : hb.gemv_fwd)), pp, qq, k);
    if (hipGetLastError() != hipSuccess) return CIRC_EHIP;
  }
  if (fused_it(k) != 0) {
    // rearrangements of the two sections for the fused kernel (forward and backward-data)
    const int FG = k / 32;
    for (int dir = 0; dir < 2; ++dir) {
      const int pp = dir ? q : p, qq = dir ? p : q;
      const int igp = fused_igp(pp, k), q2p = fused_q2p(qq, k);
      const long long total = (long long)igp * q2p * FG * 64;
      hipLaunchKernelGGL(pack_fused_half_kernel, dim3((unsigned)cdiv(total, 256)), dim3(256), 0, static_cast<hipStream_t>(stream),
                         reinterpret_cast<const unsigned*>(base + (dir ? hb.bwd : hb.fwd)),
                         reinterpret_cast<uint2*>(base + (dir ? hb.fused_bwd : hb.fused_fwd)), pp, qq, k, igp, q2p);
      if (hipGetLastError() != hipSuccess) return CIRC_EHIP;
    }
  }
  return CIRC_OK;
}

size_t fc_workspace_bytes_half(int p, int q, int k, int batch) {
  if (!fc_dims_ok(p, q, k, batch) || !half_k(k)) return 0;
  const size_t sp = half_spectrum_bytes(k, (long long)q * batch) + half_spectrum_bytes(k, (long long)p * batch);
  const size_t gp = batch <= 2 ? align_up(gemv_partial_bytes(p, q, k), 256) : 0;   // partial spectra of the split batch <= 2 kernel
  return sp > gp ? sp : gp;
}

circ_status fc_forward_half(bool bf, const void* w_hat, const void* x, const float* bias, void* y, int p, int q, int k,
                            int batch, int epilogue, void* workspace, size_t workspace_bytes, void* stream) {
  if (!fc_dims_ok(p, q, k, batch) || !half_k(k)) return CIRC_EINVAL;
  if (!w_hat || !x || !y) return CIRC_EINVAL;
  if (epilogue & ~(CIRC_EPI_BIAS | CIRC_EPI_RELU)) return CIRC_EINVAL;
  const bool use_bias = epilogue & CIRC_EPI_BIAS;
  if (use_bias && !bias) return CIRC_EINVAL;
  if (!aligned16(w_hat) || !aligned16(x) || !aligned16(y) || (use_bias && !aligned16(bias))) return CIRC_EINVAL;
  const size_t xbytes = size_t(batch) * q * k * sizeof(__half), ybytes = size_t(batch) * p * k * sizeof(__half);
  if (overlaps(x, xbytes, y, ybytes)) return CIRC_EINVAL;
  if (!workspace || workspace_bytes < fc_workspace_bytes_half(p, q, k, batch)) return CIRC_EWORKSPACE;
  if (!aligned16(workspace)) return CIRC_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (batch <= 2) {   // one or two vectors: the streaming matrix-vector kernel on 16-bit operands
    const void* wg = static_cast<const char*>(w_hat) + half_blob(p, q, k).gemv_fwd;
    return launch_gemv_half(bf, k, wg, x, use_bias ? bias : nullptr, y, p, q, batch, (epilogue & CIRC_EPI_RELU) ? 1 : 0, workspace, s) == hipSuccess
               ? CIRC_OK
               : CIRC_EHIP;
  }
  if (use_fused_forward(p, q, k, batch)) {
    // one launch: 16-bit loads of x and of the packed operands, fp32 inside, 16-bit store of y
    const void* wfu = static_cast<const char*>(w_hat) + half_blob(p, q, k).fused_fwd;
    return launch_fused_half(bf, k, wfu, x, use_bias ? bias : nullptr, y, p, q, batch, (epilogue & CIRC_EPI_RELU) ? 1 : 0, s) == hipSuccess
               ? CIRC_OK
               : CIRC_EHIP;
  }
  const int NF = k / 2 + 1;
  const long long xrows = (long long)q * batch, yrows = (long long)p * batch;
  __half2* xh = static_cast<__half2*>(workspace);
  __half2* yh = reinterpret_cast<__half2*>(static_cast<char*>(workspace) + half_spectrum_bytes(k, xrows));
  // X^[f][b][j]: row id = b*q + j -> x[b][j*k : (j+1)*k]  (j fastest: the reduction index of the contraction)
  RowMap mx{q, batch, (long long)k, (long long)q * k, 0, 1};
  if (launch_rfft_half(k, kHalfSpectra | kHalfRows, bf, x, xh, mx, xrows, xrows, 1.0f, s) != hipSuccess) return CIRC_EHIP;
  // Y^[f][i][b] = (1/k) sum_j W^[f][i][j] X^[f][b][j]
  const __half2* wh = static_cast<const __half2*>(w_hat);
  if (launch_cgemm_h<false>(bf, s, NF, wh, xh, yh, p, batch, q, (long long)p * q, xrows, yrows, 1.0f / float(k)) != hipSuccess)
    return CIRC_EHIP;
  RowMap my{batch, p, (long long)p * k, (long long)k, 0, 1};
  if (launch_irfft_half(k, bf, yh, y, my, yrows, yrows, 1.0f, use_bias ? bias : nullptr, batch,
                        (epilogue & CIRC_EPI_RELU) ? 1 : 0, s) != hipSuccess)
    return CIRC_EHIP;
  return CIRC_OK;
}


// Slices of the batch for the weight-gradient contraction: enough workgroups to cover the chip,
// each slice a multiple of 64 and at least 128 long, at most 16 slices.
inline int half_dw_slices(int p, int q, int k, int batch) {
  const long long tiles = (long long)(k / 2 + 1) * cdiv(p, 64) * cdiv(q, 64);
  int ks = 1;
  while (ks < 16 && tiles * ks < 512 && cdiv(batch, ks * 2) >= 128) ks *= 2;
  return ks;
}
inline int half_dw_slice_len(int batch, int ks) { return int(align_up(size_t(cdiv(batch, ks)), 64)); }
inline size_t half_dw_part_elems(int p, int q, int k) {
  return align_up(size_t(k / 2 + 1) * size_t(p) * q * sizeof(float2), 256) / sizeof(float2);
}

// workspace: dY^[f][b][i] and dX^[f][j][b] (backward-data), X^[f][j][b] and dY^[f][i][b] (batch
// fastest, for the weight gradient), the fp32 partial spectra of the weight gradient
size_t fc_backward_workspace_bytes_half(int p, int q, int k, int batch) {
  if (!fc_dims_ok(p, q, k, batch) || !half_k(k)) return 0;
  const size_t sp = 2 * half_spectrum_bytes(k, (long long)q * batch) + 2 * half_spectrum_bytes(k, (long long)p * batch) +
                    size_t(half_dw_slices(p, q, k, batch)) * half_dw_part_elems(p, q, k) * sizeof(float2);
  // batch <= 2: partial spectra of the split streaming kernel on the transposed grid (they sit at
  // the start of the workspace, which the weight gradient only uses afterwards)
  const size_t gp = batch <= 2 ? align_up(gemv_partial_bytes(q, p, k), 256) : 0;
  return sp > gp ? sp : gp;
}

circ_status fc_backward_half(bool bf, const void* w_hat, const void* x, const void* dy, void* dx, float* dw, int p, int q,
                             int k, int batch, void* workspace, size_t workspace_bytes, void* stream) {
  if (!fc_dims_ok(p, q, k, batch) || !half_k(k)) return CIRC_EINVAL;
  if (!w_hat || !dy || (!dx && !dw) || (dw && !x)) return CIRC_EINVAL;
  if (!aligned16(w_hat) || !aligned16(dy) || !aligned16(x) || !aligned16(dx) || !aligned16(dw)) return CIRC_EINVAL;
  const size_t xbytes = size_t(batch) * q * k * sizeof(__half), ybytes = size_t(batch) * p * k * sizeof(__half);
  const size_t wbytes = size_t(p) * q * k * sizeof(float);
  if (dx && (overlaps(dx, xbytes, dy, ybytes) || (x && overlaps(dx, xbytes, x, xbytes)))) return CIRC_EINVAL;
  if (dw && (overlaps(dw, wbytes, dy, ybytes) || overlaps(dw, wbytes, x, xbytes) || (dx && overlaps(dw, wbytes, dx, xbytes))))
    return CIRC_EINVAL;
  if (!workspace || workspace_bytes < fc_backward_workspace_bytes_half(p, q, k, batch)) return CIRC_EWORKSPACE;
  if (!aligned16(workspace)) return CIRC_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int NF = k / 2 + 1;
  const long long xrows = (long long)q * batch, yrows = (long long)p * batch, wrows = (long long)p * q;
  const size_t xs = half_spectrum_bytes(k, xrows), ys = half_spectrum_bytes(k, yrows);
  char* ws = static_cast<char*>(workspace);
  __half2* dyh = reinterpret_cast<__half2*>(ws);                  // dY^[f][b][i]
  __half2* dxh = reinterpret_cast<__half2*>(ws + ys);             // dX^[f][j][b]
  __half2* xt = reinterpret_cast<__half2*>(ws + ys + xs);         // X^[f][j][b]
  __half2* dyt = reinterpret_cast<__half2*>(ws + ys + 2 * xs);    // dY^[f][i][b]
  float2* wpart = reinterpret_cast<float2*>(ws + 2 * ys + 2 * xs);
  const int hm = kHalfSpectra | kHalfRows;
  // dY^[f][i][b] (batch fastest) serves the weight gradient directly and, transposed on its way
  // into the contraction, backward-data as well: dy is transformed once when both are wanted.
  // Backward-data alone takes dY^[f][b][i], which its contraction reads without the transposition.
  // (The one-launch kernels of small problems read dy itself; the batch <= 2 one may use the start
  // of the workspace for its partial spectra, so the transform for the weight gradient follows it.)
  const bool dx_one_launch = batch <= 2 || use_fused_forward(q, p, k, batch);
  RowMap myt{batch, p, (long long)p * k, (long long)k, 0, 1};
  if (dw && dx && !dx_one_launch) {
    if (launch_rfft_half(k, hm, bf, dy, dyt, myt, yrows, yrows, 1.0f, s) != hipSuccess) return CIRC_EHIP;
  }
  if (dx) {
    // backward-data = the forward route on the transposed, conjugated grid (Algorithm 2):
    // dX^[f][j][b] = (1/k) sum_i conj(W^)[f][j][i] dY^[f][.][.]
    const HalfBlob hb = half_blob(p, q, k);
    const __half2* wt = reinterpret_cast<const __half2*>(static_cast<const char*>(w_hat) + hb.bwd);
    if (batch <= 2) {
      if (launch_gemv_half(bf, k, static_cast<const char*>(w_hat) + hb.gemv_bwd, dy, nullptr, dx, q, p, batch, 0, workspace, s) != hipSuccess)
        return CIRC_EHIP;
    } else if (use_fused_forward(q, p, k, batch)) {
      // small problems: the fused kernel on the transposed grid's operands, one launch
      if (launch_fused_half(bf, k, static_cast<const char*>(w_hat) + hb.fused_bwd, dy, nullptr, dx, q, p, batch, 0, s) != hipSuccess)
        return CIRC_EHIP;
    } else {
      if (dw) {
        if (launch_cgemm_h<true>(bf, s, NF, wt, dyt, dxh, q, batch, p, wrows, yrows, xrows, 1.0f / float(k)) != hipSuccess)
          return CIRC_EHIP;
      } else {
        RowMap mdy{p, batch, (long long)k, (long long)p * k, 0, 1};
        if (launch_rfft_half(k, hm, bf, dy, dyh, mdy, yrows, yrows, 1.0f, s) != hipSuccess) return CIRC_EHIP;
        if (launch_cgemm_h<false>(bf, s, NF, wt, dyh, dxh, q, batch, p, wrows, yrows, xrows, 1.0f / float(k)) != hipSuccess)
          return CIRC_EHIP;
      }
      RowMap mdx{batch, q, (long long)q * k, (long long)k, 0, 1};
      if (launch_irfft_half(k, bf, dxh, dx, mdx, xrows, xrows, 1.0f, nullptr, 1, 0, s) != hipSuccess) return CIRC_EHIP;
    }
  }
  if (dw) {
    // dW^[f][i][j] = sum_b dY^[f][i][b] conj(X^[f][j][b]): both operands with the batch fastest
    if (!dx || dx_one_launch) {
      if (launch_rfft_half(k, hm, bf, dy, dyt, myt, yrows, yrows, 1.0f, s) != hipSuccess) return CIRC_EHIP;
    }
    RowMap mxt{batch, q, (long long)q * k, (long long)k, 0, 1};
    if (launch_rfft_half(k, hm, bf, x, xt, mxt, xrows, xrows, 1.0f, s) != hipSuccess) return CIRC_EHIP;
    const int ks = half_dw_slices(p, q, k, batch), klen = half_dw_slice_len(batch, ks);
    const long long ps = (long long)half_dw_part_elems(p, q, k);
    dim3 grid((unsigned)(cdiv(q, 64) * ks), (unsigned)cdiv(p, 64), (unsigned)NF);
    if (batch % 4 == 0) {
      if (bf) hipLaunchKernelGGL((cgemm_h_dw_kernel<true, true>), grid, dim3(256), 0, s, dyt, xt, wpart, p, q, batch, yrows, xrows, wrows, 1.0f, klen, ps);
      else hipLaunchKernelGGL((cgemm_h_dw_kernel<true, false>), grid, dim3(256), 0, s, dyt, xt, wpart, p, q, batch, yrows, xrows, wrows, 1.0f, klen, ps);
    } else {
      if (bf) hipLaunchKernelGGL((cgemm_h_dw_kernel<false, true>), grid, dim3(256), 0, s, dyt, xt, wpart, p, q, batch, yrows, xrows, wrows, 1.0f, klen, ps);
      else hipLaunchKernelGGL((cgemm_h_dw_kernel<false, false>), grid, dim3(256), 0, s, dyt, xt, wpart, p, q, batch, yrows, xrows, wrows, 1.0f, klen, ps);
    }
    if (hipGetLastError() != hipSuccess) return CIRC_EHIP;
    RowMap mw{q, p, (long long)k, (long long)q * k, 0, 1};
    if (launch_irfft(k, false, wpart, dw, mw, wrows, wrows, 1.0f / float(k), nullptr, 1, 0, s, ks, ps) != hipSuccess)
      return CIRC_EHIP;
  }
  return CIRC_OK;
}


// ---- CONV forward with 16-bit activations (the cached weight spectra stay fp32) ----------------
template <int K>
hipError_t launch_rfft_chan16_k(bool bf, const void* in, float2* out, const RowMap& map, long long nrows, long long out_fstride,
                                hipStream_t s) {
  FftPlan pl = plan_fft(K, nrows);
  dim3 grid((unsigned)cdiv(nrows, 2 * pl.P), 1);
  const float* fin = static_cast<const float*>(in);
  if (bf)
    hipLaunchKernelGGL((rfft_kernel<K, true, kHalfRows | kHalfBf16>), grid, dim3(pl.NT), pl.lds, s, fin, out, map, nrows,
                       out_fstride, 0ll, 0ll, pl.P, 1.0f, 0);
  else
    hipLaunchKernelGGL((rfft_kernel<K, true, kHalfRows>), grid, dim3(pl.NT), pl.lds, s, fin, out, map, nrows, out_fstride, 0ll,
                       0ll, pl.P, 1.0f, 0);
  return hipGetLastError();
}
template <int K>
hipError_t launch_irfft_chan16_k(bool bf, const float2* in, void* out, const RowMap& map, long long nrows, long long in_fstride,
                                 const float* bias, long long bias_div, int relu, hipStream_t s) {
  FftPlan pl = plan_fft(K, nrows);
  dim3 grid((unsigned)cdiv(nrows, 2 * pl.P));
  float* fout = static_cast<float*>(out);
  if (bf)
    hipLaunchKernelGGL((irfft_kernel<K, true, kHalfRows | kHalfBf16>), grid, dim3(pl.NT), pl.lds, s, in, fout, map, nrows,
                       in_fstride, pl.P, 1.0f, bias, bias_div, relu, 1, 0ll);
  else
    hipLaunchKernelGGL((irfft_kernel<K, true, kHalfRows>), grid, dim3(pl.NT), pl.lds, s, in, fout, map, nrows, in_fstride, pl.P,
                       1.0f, bias, bias_div, relu, 1, 0ll);
  return hipGetLastError();
}
hipError_t launch_rfft_chan16(int k, bool bf, const void* in, float2* out, const RowMap& map, long long nrows,
                              long long out_fstride, hipStream_t s) {
#define CALL(KK) launch_rfft_chan16_k<KK>(bf, in, out, map, nrows, out_fstride, s)
  CIRC_DISPATCH_HALF_K(k, CALL)
#undef CALL
}
hipError_t launch_irfft_chan16(int k, bool bf, const float2* in, void* out, const RowMap& map, long long nrows,
                               long long in_fstride, const float* bias, long long bias_div, int relu, hipStream_t s) {
#define CALL(KK) launch_irfft_chan16_k<KK>(bf, in, out, map, nrows, in_fstride, bias, bias_div, relu, s)
  CIRC_DISPATCH_HALF_K(k, CALL)
#undef CALL
}

circ_status conv_forward_half(bool bf, const void* w_hat, const void* x, const float* bias, void* y, int N, int C_in, int C_out,
                              int H, int W, int r, int stride, int pad, int k, int epilogue, void* workspace,
                              size_t workspace_bytes, void* stream) {
  if (!conv_dims_ok(N, C_in, C_out, H, W, r, pad, k) || !half_k(k)) return CIRC_EINVAL;
  if (stride <= 0) return CIRC_EINVAL;
  if (!w_hat || !x || !y) return CIRC_EINVAL;
  if (epilogue & ~(CIRC_EPI_BIAS | CIRC_EPI_RELU)) return CIRC_EINVAL;
  const bool use_bias = epilogue & CIRC_EPI_BIAS;
  if (use_bias && !bias) return CIRC_EINVAL;
  if (!aligned16(w_hat) || !aligned16(x) || !aligned16(y) || (use_bias && !aligned16(bias))) return CIRC_EINVAL;
  const int Ho = conv_out(H, r, pad, stride), Wo = conv_out(W, r, pad, stride);
  const size_t xbytes = size_t(N) * C_in * H * W * sizeof(__half), ybytes = size_t(N) * C_out * Ho * Wo * sizeof(__half);
  if (overlaps(x, xbytes, y, ybytes)) return CIRC_EINVAL;
  const size_t need = circ_conv_workspace_bytes(N, C_in, C_out, H, W, r, stride, pad, k);
  if (!workspace || workspace_bytes < need) return CIRC_EWORKSPACE;
  if (!aligned16(workspace)) return CIRC_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int p = C_out / k, q = C_in / k, NF = k / 2 + 1;
  const long long HW = (long long)H * W, HWo = (long long)Ho * Wo;
  const int relu = (epilogue & CIRC_EPI_RELU) ? 1 : 0;
  if (stride == 1 && conv_fused_applicable(p, q, k, r, N, H, W, Ho, Wo)) {
    const float2* wc = blob_at<float2>(w_hat, blob_layout(r * r, p, q, k).conv);
    const float* xf = static_cast<const float*>(x);
    float* yf = static_cast<float*>(y);
    const hipError_t e = bf ? launch_conv_fused_h<2>(wc, xf, use_bias ? bias : nullptr, yf, N, p, q, k, r, H, W, Ho, Wo, pad, relu, s)
                            : launch_conv_fused_h<1>(wc, xf, use_bias ? bias : nullptr, yf, N, p, q, k, r, H, W, Ho, Wo, pad, relu, s);
    return e == hipSuccess ? CIRC_OK : CIRC_EHIP;
  }
  const long long xrows = (long long)q * N * HW, yrows = (long long)p * N * HWo;
  float2* xh = static_cast<float2*>(workspace);
  float2* yh = reinterpret_cast<float2*>(static_cast<char*>(workspace) + align_up(spectrum_elems(k, xrows) * sizeof(float2), 256));
  // the three kernels of the unfused route; only the loads of x and the stores of y are 16-bit
  RowMap mx{(int)HW, N, 1, (long long)C_in * HW, (long long)k * HW, HW, HW % 4 == 0};
  if (launch_rfft_chan16(k, bf, x, xh, mx, xrows, xrows, s) != hipSuccess) return CIRC_EHIP;
  if (launch_conv_contract(static_cast<const float2*>(w_hat), xh, yh, p, q, NF, N, H, W, Ho, Wo, r, pad, 0, stride, 1, s) !=
      hipSuccess)
    return CIRC_EHIP;
  RowMap my{(int)HWo, N, 1, (long long)C_out * HWo, (long long)k * HWo, HWo, HWo % 4 == 0};
  if (launch_irfft_chan16(k, bf, yh, y, my, yrows, yrows, use_bias ? bias : nullptr, (long long)N * HWo, relu, s) != hipSuccess)
    return CIRC_EHIP;
  return CIRC_OK;
}

}  // namespace

extern "C" {

size_t circ_spectra_bytes_f16(int p, int q, int k) { return spectra_bytes_half(p, q, k); }
size_t circ_spectra_bytes_bf16(int p, int q, int k) { return spectra_bytes_half(p, q, k); }
circ_status circ_precompute_spectra_f16(const float* w, int p, int q, int k, void* w_hat, void* stream) {
  return precompute_spectra_half(false, w, p, q, k, w_hat, stream);
}
circ_status circ_precompute_spectra_bf16(const float* w, int p, int q, int k, void* w_hat, void* stream) {
  return precompute_spectra_half(true, w, p, q, k, w_hat, stream);
}
size_t circ_fc_workspace_bytes_f16(int p, int q, int k, int batch) { return fc_workspace_bytes_half(p, q, k, batch); }
size_t circ_fc_workspace_bytes_bf16(int p, int q, int k, int batch) { return fc_workspace_bytes_half(p, q, k, batch); }
circ_status circ_fc_forward_f16(const void* w_hat, const void* x, const float* bias, void* y, int p, int q, int k,
                                int batch, int epilogue, void* workspace, size_t workspace_bytes, void* stream) {
  return fc_forward_half(false, w_hat, x, bias, y, p, q, k, batch, epilogue, workspace, workspace_bytes, stream);
}
circ_status circ_fc_forward_bf16(const void* w_hat, const void* x, const float* bias, void* y, int p, int q, int k,
                                 int batch, int epilogue, void* workspace, size_t workspace_bytes, void* stream) {
  return fc_forward_half(true, w_hat, x, bias, y, p, q, k, batch, epilogue, workspace, workspace_bytes, stream);
}
circ_status circ_conv_forward_f16(const void* w_hat, const void* x, const float* bias, void* y, int N, int C_in, int C_out, int H,
                                  int W, int r, int stride, int pad, int k, int epilogue, void* workspace,
                                  size_t workspace_bytes, void* stream) {
  return conv_forward_half(false, w_hat, x, bias, y, N, C_in, C_out, H, W, r, stride, pad, k, epilogue, workspace, workspace_bytes,
                           stream);
}
circ_status circ_conv_forward_bf16(const void* w_hat, const void* x, const float* bias, void* y, int N, int C_in, int C_out, int H,
                                   int W, int r, int stride, int pad, int k, int epilogue, void* workspace,
                                   size_t workspace_bytes, void* stream) {
  return conv_forward_half(true, w_hat, x, bias, y, N, C_in, C_out, H, W, r, stride, pad, k, epilogue, workspace, workspace_bytes,
                           stream);
}
circ_status circ_conv_backward_f16(const void* w_hat, const void* x, const void* dy, void* dx, float* dw, int N, int C_in,
                                   int C_out, int H, int W, int r, int stride, int pad, int k, void* workspace,
                                   size_t workspace_bytes, void* stream) {
  if (!dx && !dw) return CIRC_EINVAL;
  return conv_backward_impl(w_hat, static_cast<const float*>(x), static_cast<const float*>(dy), static_cast<float*>(dx), dw,
                            nullptr, 0.f, N, C_in, C_out, H, W, r, stride, pad, k, workspace, workspace_bytes, stream, 1);
}
circ_status circ_conv_backward_bf16(const void* w_hat, const void* x, const void* dy, void* dx, float* dw, int N, int C_in,
                                    int C_out, int H, int W, int r, int stride, int pad, int k, void* workspace,
                                    size_t workspace_bytes, void* stream) {
  if (!dx && !dw) return CIRC_EINVAL;
  return conv_backward_impl(w_hat, static_cast<const float*>(x), static_cast<const float*>(dy), static_cast<float*>(dx), dw,
                            nullptr, 0.f, N, C_in, C_out, H, W, r, stride, pad, k, workspace, workspace_bytes, stream, 2);
}
size_t circ_fc_backward_workspace_bytes_f16(int p, int q, int k, int batch) { return fc_backward_workspace_bytes_half(p, q, k, batch); }
size_t circ_fc_backward_workspace_bytes_bf16(int p, int q, int k, int batch) { return fc_backward_workspace_bytes_half(p, q, k, batch); }
circ_status circ_fc_backward_f16(const void* w_hat, const void* x, const void* dy, void* dx, float* dw, int p, int q, int k,
                                 int batch, void* workspace, size_t workspace_bytes, void* stream) {
  return fc_backward_half(false, w_hat, x, dy, dx, dw, p, q, k, batch, workspace, workspace_bytes, stream);
}
circ_status circ_fc_backward_bf16(const void* w_hat, const void* x, const void* dy, void* dx, float* dw, int p, int q, int k,
                                  int batch, void* workspace, size_t workspace_bytes, void* stream) {
  return fc_backward_half(true, w_hat, x, dy, dx, dw, p, q, k, batch, workspace, workspace_bytes, stream);
}

}  // extern "C"

// ---- max-pooling and chains of layers (the single-image regime of Sec. 5.3) ----------------------
namespace {

inline int pool_out(int n, int window, int stride) { return (n - window) / stride + 1; }

inline bool pool_dims_ok(int N, int C, int H, int W, int window, int stride) {
  if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || window <= 0 || stride <= 0 || window > H || window > W) return false;
  const long long Ho = pool_out(H, window, stride), Wo = pool_out(W, window, stride);
  // image planes fit the grid, the in-plane index its 32-bit reciprocal division
  return (long long)N * C <= 65535ll * 65535ll && (long long)N * C * H * W <= (1ll << 40) && Ho * Wo * Wo < (1ll << 32);
}

// elements per batch item that a layer consumes / produces (0: invalid descriptor)
long long layer_in_elems(const circ_layer& l) {
  switch (l.kind) {
    case CIRC_LAYER_FC: return (long long)l.q * l.k;
    case CIRC_LAYER_CONV:
    case CIRC_LAYER_MAXPOOL: return (long long)l.C_in * l.H * l.W;
  }
  return 0;
}
long long layer_out_elems(const circ_layer& l) {
  switch (l.kind) {
    case CIRC_LAYER_FC: return (long long)l.p * l.k;
    case CIRC_LAYER_CONV: return (long long)l.C_out * conv_out(l.H, l.r, l.pad, l.stride) * conv_out(l.W, l.r, l.pad, l.stride);
    case CIRC_LAYER_MAXPOOL: return (long long)l.C_in * pool_out(l.H, l.r, l.stride) * pool_out(l.W, l.r, l.stride);
  }
  return 0;
}
bool layer_ok(const circ_layer& l, int batch) {
  switch (l.kind) {
    case CIRC_LAYER_FC: return fc_dims_ok(l.p, l.q, l.k, batch);
    case CIRC_LAYER_CONV: return conv_dims_ok(batch, l.C_in, l.C_out, l.H, l.W, l.r, l.pad, l.k) && l.stride >= 1;
    case CIRC_LAYER_MAXPOOL: return pool_dims_ok(batch, l.C_in, l.H, l.W, l.r, l.stride);
  }
  return false;
}
size_t layer_workspace(const circ_layer& l, int batch) {
  switch (l.kind) {
    case CIRC_LAYER_FC: return circ_fc_workspace_bytes(l.p, l.q, l.k, batch, 0);
    case CIRC_LAYER_CONV: return circ_conv_workspace_bytes(batch, l.C_in, l.C_out, l.H, l.W, l.r, l.stride, l.pad, l.k);
    default: return 0;
  }
}
// Layers that fit together: every layer valid, each output as long as the next input.
// Returns the largest intermediate activation (elements per batch item) through *mid.
bool chain_ok(const circ_layer* layers, int n_layers, int batch, long long* mid) {
  if (!layers || n_layers <= 0 || n_layers > 4096 || batch <= 0) return false;
  long long m = 0;
  for (int i = 0; i < n_layers; ++i) {
    if (!layer_ok(layers[i], batch)) return false;
    if (i + 1 < n_layers) {
      const long long o = layer_out_elems(layers[i]);
      if (o != layer_in_elems(layers[i + 1])) return false;
      if (o > m) m = o;
    }
  }
  *mid = m;
  return true;
}

}  // namespace

extern "C" {

circ_status circ_maxpool_forward(const float* x, float* y, int N, int C, int H, int W, int window, int stride, void* stream) {
  if (!x || !y || !pool_dims_ok(N, C, H, W, window, stride)) return CIRC_EINVAL;
  if (!aligned16(x) || !aligned16(y)) return CIRC_EINVAL;
  const int Ho = pool_out(H, window, stride), Wo = pool_out(W, window, stride);
  const long long planes = (long long)N * C, total = planes * Ho * Wo;
  if (overlaps(x, size_t(planes) * H * W * sizeof(float), y, size_t(total) * sizeof(float))) return CIRC_EINVAL;
  const unsigned mul_wo = Wo > 1 ? unsigned(((1ull << 32) + unsigned(Wo) - 1) / unsigned(Wo)) : 0u;
  const dim3 grid((unsigned)cdiv((long long)Ho * Wo, 256), (unsigned)(planes < 65535 ? planes : 65535), (unsigned)cdiv(planes, 65535));
  hipLaunchKernelGGL(maxpool_kernel, grid, dim3(256), 0, static_cast<hipStream_t>(stream), x, y, (unsigned)planes, H, W, Ho, Wo,
                     window, stride, mul_wo);
  return hipGetLastError() == hipSuccess ? CIRC_OK : CIRC_EHIP;
}

size_t circ_chain_workspace_bytes(const circ_layer* layers, int n_layers, int batch) {
  long long mid = 0;
  if (!chain_ok(layers, n_layers, batch, &mid)) return 0;
  size_t ws = 0;
  for (int i = 0; i < n_layers; ++i) {
    const size_t w = layer_workspace(layers[i], batch);
    if (w > ws) ws = w;
  }
  // two buffers for the activations between the layers, then the largest layer workspace
  const size_t act = align_up(size_t(mid) * batch * sizeof(float), 256);
  return 2 * act + align_up(ws, 256) + 256;
}

circ_status circ_chain_forward(const circ_layer* layers, int n_layers, const float* x, float* y, int batch, void* workspace,
                               size_t workspace_bytes, void* stream) {
  long long mid = 0;
  if (!chain_ok(layers, n_layers, batch, &mid)) return CIRC_EINVAL;
  if (!x || !y || !aligned16(x) || !aligned16(y)) return CIRC_EINVAL;
  for (int i = 0; i < n_layers; ++i) {
    const circ_layer& l = layers[i];
    if (l.kind == CIRC_LAYER_MAXPOOL) continue;
    if (!l.w_hat || !aligned16(l.w_hat)) return CIRC_EINVAL;
    if (l.epilogue & ~(CIRC_EPI_BIAS | CIRC_EPI_RELU)) return CIRC_EINVAL;
    if ((l.epilogue & CIRC_EPI_BIAS) && (!l.bias || !aligned16(l.bias))) return CIRC_EINVAL;
  }
  const size_t xin = size_t(layer_in_elems(layers[0])) * batch * sizeof(float);
  const size_t yout = size_t(layer_out_elems(layers[n_layers - 1])) * batch * sizeof(float);
  if (overlaps(x, xin, y, yout)) return CIRC_EINVAL;
  const size_t need = circ_chain_workspace_bytes(layers, n_layers, batch);
  if (!workspace || workspace_bytes < need) return CIRC_EWORKSPACE;
  if (!aligned16(workspace)) return CIRC_EINVAL;
  if (overlaps(workspace, need, x, xin) || overlaps(workspace, need, y, yout)) return CIRC_EINVAL;
  const size_t act = align_up(size_t(mid) * batch * sizeof(float), 256);
  float* buf[2] = {static_cast<float*>(workspace), reinterpret_cast<float*>(static_cast<char*>(workspace) + act)};
  void* lws = static_cast<char*>(workspace) + 2 * act;
  const size_t lws_bytes = workspace_bytes - 2 * act;
  const float* src = x;
  for (int i = 0; i < n_layers; ++i) {
    const circ_layer& l = layers[i];
    float* dst = i + 1 == n_layers ? y : buf[i & 1];
    circ_status st = CIRC_EINVAL;
    switch (l.kind) {
      case CIRC_LAYER_FC:
        st = circ_fc_forward(l.w_hat, src, l.bias, dst, l.p, l.q, l.k, batch, l.epilogue, lws, lws_bytes, stream);
        break;
      case CIRC_LAYER_CONV:
        st = circ_conv_forward(l.w_hat, src, l.bias, dst, batch, l.C_in, l.C_out, l.H, l.W, l.r, l.stride, l.pad, l.k, l.epilogue,
                               lws, lws_bytes, stream);
        break;
      case CIRC_LAYER_MAXPOOL:
        st = circ_maxpool_forward(src, dst, batch, l.C_in, l.H, l.W, l.r, l.stride, stream);
        break;
    }
    if (st != CIRC_OK) return st;
    src = dst;
  }
  return CIRC_OK;
}

}  // extern "C"
