// Test-only header, force-included when tests/test_host_dry_run.py compiles the library for a
// CPU dry run: a kernel launch only checks its geometry against the limits of the device (grid
// dimensions, threads per workgroup, LDS per workgroup; a violation traps) and reports success,
// so that the host code of every entry point (argument checks, workspace carving, launch
// planning) runs to its end on a machine without a GPU, under the compiler's
// undefined-behaviour checks.
#include <hip/hip_runtime.h>
static inline void circ_dry_check(dim3 g, dim3 b, size_t lds) {
  const unsigned long long threads = (unsigned long long)b.x * b.y * b.z;
  if (g.x == 0 || g.y == 0 || g.z == 0 || g.x > 2147483647u || g.y > 65535u || g.z > 65535u || threads == 0 ||
      threads > 1024 || lds > 160u * 1024u)
    __builtin_trap();
}
#undef hipLaunchKernelGGL
#define hipLaunchKernelGGL(kern, grid, block, lds, stream, ...) circ_dry_check(dim3(grid), dim3(block), size_t(lds))
#define hipGetLastError() hipSuccess
#define hipFuncSetAttribute(...) hipSuccess
#define hipGetDevice(p) ((*(p) = 0), hipSuccess)
#define hipGetSymbolAddress(pp, sym) ((*(pp) = reinterpret_cast<void*>(0x7000000000ull)), hipSuccess)
