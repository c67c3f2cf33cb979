// Measurement helpers for bench.py (not part of the layer library): kernels that do no
// arithmetic and only show how long the machine takes to launch a grid of the fused FC kernel's
// shape, and to move that kernel's bytes.  They give the time below which no kernel with the
// same launch shape / memory footprint can finish on this machine.
//
//   circ_floor_empty      grid x block launch of a kernel that returns at once
//   circ_floor_stream     every workgroup reads piece ia of region A (`rd_a` bytes each) and piece
//                         ib of region B (`rd_b` bytes each), then writes `wr` bytes at
//                         blockIdx * wr.  xa = 0: ia = ib = blockIdx (a plain copy that touches
//                         every byte once).  xa > 0: the tile map of the fused FC kernel, so that
//                         pieces are shared between workgroups and XCDs exactly as its weight
//                         tiles (A) and x rows (B) are: xcd = blockIdx % 8, local = blockIdx / 8,
//                         ia = (xcd % xa) * ni + local % ni, ib = (xcd / xa) * nb + local / ni
// All pointers are device pointers, 16-byte aligned; sizes are multiples of 16 bytes; the sizes
// of the three regions are passed and every piece index is checked against them on the host
// (-1 = invalid argument, nothing launched).  Nothing is allocated; launches go to `stream`.
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

namespace {

__global__ void empty_kernel(int* sink) {
  if (sink != nullptr && threadIdx.x == 4096) *sink = 0;   // never true: keeps the argument alive
}

__global__ void stream_kernel(const float4* __restrict__ a, const float4* __restrict__ b, float4* __restrict__ out,
                              unsigned rd_a16, unsigned rd_b16, unsigned wr16, unsigned xa, unsigned ni, unsigned nb) {
  const unsigned tid = threadIdx.x, nt = blockDim.x;
  unsigned ia = blockIdx.x, ib = blockIdx.x;
  if (xa > 0) {
    const unsigned xcd = blockIdx.x & 7u, local = blockIdx.x >> 3;
    ia = (xcd % xa) * ni + local % ni;
    ib = (xcd / xa) * nb + local / ni;
  }
  const float4* pa = a + size_t(ia) * rd_a16;
  const float4* pb = b + size_t(ib) * rd_b16;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  // The loads of a thread are independent; they are issued in batches of 16 before any value is
  // used (the fused kernel has 20 in flight per thread).  B first: the fused kernel needs x first.
  constexpr int BATCH = 16;
  auto sweep = [&](const float4* src, unsigned n16) {
    for (unsigned base = 0; base < n16; base += BATCH * nt) {
      float4 v[BATCH];
#pragma unroll
      for (int u = 0; u < BATCH; ++u) {
        const unsigned i = base + u * nt + tid;
        v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (i < n16) v[u] = src[i];
      }
#pragma unroll
      for (int u = 0; u < BATCH; ++u) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
    }
  };
  sweep(pb, rd_b16);
  sweep(pa, rd_a16);
  float4* po = out + size_t(blockIdx.x) * wr16;
  for (unsigned i = tid; i < wr16; i += nt) po[i] = acc;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" {

int circ_floor_empty(int grid, int block, void* stream) {
  if (grid <= 0 || block <= 0 || block > 1024) return -1;
  hipLaunchKernelGGL(empty_kernel, dim3((unsigned)grid), dim3((unsigned)block), 0, static_cast<hipStream_t>(stream),
                     static_cast<int*>(nullptr));
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

int circ_floor_stream(const void* a, size_t a_bytes, const void* b, size_t b_bytes, void* out, size_t out_bytes, int grid,
                      int block, size_t rd_a, size_t rd_b, size_t wr, int xa, int ni, int nb, void* stream) {
  if (grid <= 0 || block <= 0 || block > 1024 || xa < 0 || xa > 8 || (xa > 0 && (ni <= 0 || nb <= 0))) return -1;
  if (rd_a + rd_b == 0) return -1;
  // every piece a workgroup can address must lie inside its region
  size_t max_ia = size_t(grid) - 1, max_ib = size_t(grid) - 1;
  if (xa > 0) {
    max_ia = size_t(xa - 1) * ni + (ni - 1);
    max_ib = size_t(7 / xa) * nb + size_t(grid - 1) / 8 / ni;
  }
  if ((max_ia + 1) * rd_a > a_bytes || (max_ib + 1) * rd_b > b_bytes || size_t(grid) * wr > out_bytes) return -1;
  if (!a || !b || !out || !aligned16(a) || !aligned16(b) || !aligned16(out)) return -1;
  if ((rd_a | rd_b | wr) & 15u) return -1;
  if (rd_a > (size_t(1) << 31) || rd_b > (size_t(1) << 31) || wr > (size_t(1) << 31)) return -1;
  hipLaunchKernelGGL(stream_kernel, dim3((unsigned)grid), dim3((unsigned)block), 0, static_cast<hipStream_t>(stream),
                     static_cast<const float4*>(a), static_cast<const float4*>(b), static_cast<float4*>(out),
                     (unsigned)(rd_a / 16), (unsigned)(rd_b / 16), (unsigned)(wr / 16), (unsigned)xa, (unsigned)ni,
                     (unsigned)nb);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

}  // extern "C"
