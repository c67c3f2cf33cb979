// Phase-timing hook of the fused kernels (fc_fused_kernel, fc_gemv_kernel, conv_fused_kernel).
//
// In the library CIRC_PROBE(id) expands to nothing.  A profiling build is a separate
// translation unit, outside the product, that defines CIRC_PROBE(id) before it includes the
// library source, e.g. as "thread 0 of the workgroup stores the clock (s_memtime) into slot
// (workgroup, id) of a device array", and reads that array back after one launch.  The ids mark
// phase boundaries: 0 kernel start; for chunk c: 2 + 4c first transform pass done, 3 + 4c
// second pass written, 1 + 4c barrier passed (operands ready), 4 + 4c contraction issued; 60 .. 62
// output spectra assembled, inverse transform done, outputs stored.  This is the only profiling switch in the sources.
#pragma once

#ifndef CIRC_PROBE
#define CIRC_PROBE(id)
#endif
