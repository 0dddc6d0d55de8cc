// Internal helpers shared by the HIP translation units of libcwac_hip.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "cwac.h"

namespace cwac {

constexpr int kWave = 64;  // CDNA wavefront width

inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

inline cwac_status launch_status() {
  return hipGetLastError() == hipSuccess ? CWAC_OK : CWAC_E_LAUNCH;
}

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Butterfly reductions over the 64 lanes of a wavefront (cross-lane permutes, no memory).
template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}
__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o, kWave));
  return v;
}

// The requantizing tail of the engine epilogue (Eq. 10 with the clip of Eq. 1):
// round half to even, clamp in fp32 to [qmin - Z_r, qmax - Z_r], then add Z_r.
__device__ __forceinline__ int requant_code(float u, float lo, float hi, int zr) {
  float r = rintf(u);
  r = fmaxf(r, lo);
  r = fminf(r, hi);
  return static_cast<int>(r) + zr;
}

}  // namespace cwac
