// Diagnostic, not part of the path: what the int8 matrix cores of this device sustain when
// nothing else limits them.  Four wavefronts per workgroup run the forward kernel's register
// pattern (4 x 4 MFMA 32x32x32 tiles per wavefront, 256 accumulators per lane) on operand
// fragments that stay in registers: no LDS, no memory traffic in the timed loop.  The rate
// depends on the CONTENT of the operands (switching activity moves the clock the device can hold
// under its power limit), which is why the caller supplies them.
#include "qlinear_common.h"

namespace cwac {
namespace {

__global__ __launch_bounds__(256) void mfma_probe_kernel(const v4i *__restrict__ operands, int iters,
                                                         int32_t *sink) {
  v4i a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = operands[(threadIdx.x + 64 * i) & 511];
    b[i] = operands[512 + ((threadIdx.x + 64 * i) & 511)];
  }
  v16i acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
  }
  int s = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) s += acc[i][j][e];
  if (s == 0x12345678) sink[0] = s;  // keeps the loop alive; practically never taken
}

}  // namespace
}  // namespace cwac

using namespace cwac;

extern "C" cwac_status cwac_mfma_probe(const int32_t *operands, int32_t iters, int32_t workgroups,
                                       int32_t *sink, void *stream) {
  if (!operands || !sink) return CWAC_E_NULL;
  if (iters < 1 || iters > (1 << 24) || workgroups < 1 || workgroups > (1 << 20)) return CWAC_E_SHAPE;
  if (!aligned(operands, 16)) return CWAC_E_ALIGN;
  mfma_probe_kernel<<<(unsigned)workgroups, 256, 0, as_stream(stream)>>>(
      reinterpret_cast<const v4i *>(operands), iters, sink);
  return launch_status();
}
