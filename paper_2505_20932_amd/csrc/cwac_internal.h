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

// ---- calibration state (layout documented in cwac.h): 64-byte header (int64 row count at
// byte 0, merge ticket at byte 16), pivot_q[C], pivot_f[C] (fp32), sum[kStats][C] (fp64).
constexpr int kStats = 5;  // sum dq, sum df, sum dq*dq, sum dq*df, sum df*df
constexpr int kStatsHeaderBytes = 64;

struct StatsView {
  int64_t *n;
  float *pivot_q;
  float *pivot_f;
  double *sum;  // [kStats][c]
};

__host__ __device__ inline StatsView stats_view(void *stats, int c) {
  char *b = static_cast<char *>(stats);
  StatsView v;
  v.n = reinterpret_cast<int64_t *>(b);
  v.pivot_q = reinterpret_cast<float *>(b + kStatsHeaderBytes);
  v.pivot_f = v.pivot_q + c;
  v.sum = reinterpret_cast<double *>(b + kStatsHeaderBytes + (size_t)8 * c);
  return v;
}

// Second stage of a statistics pass (calib_stats.hip): adds partial[row_group][kStats][c_out] into
// the state in a fixed order and bumps its row count by n_rows.  A first batch also records the
// pivots: pivot_q = pivot_q_src[0..c_out), pivot_f = pivot_f_src[0..c_out).  fresh: the state is
// taken as empty whatever it holds (sums overwritten, header written, row count = n_rows).
cwac_status launch_stats_merge(const double *partial, int row_groups, int c_out,
                               const float *pivot_f_src, const float *pivot_q_src, void *stats,
                               int64_t n_rows, bool fresh, hipStream_t st);

}  // namespace cwac
