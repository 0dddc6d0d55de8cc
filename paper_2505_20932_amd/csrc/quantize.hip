// Quantizers of Sec. 3.2 (Eq. 1-2) and the weight column sums used by the
// zero-point term of Eq. 7.  All arithmetic is single fp32 operations with
// IEEE division and round-half-to-even, so codes are reproducible bit for bit.
#include <float.h>
#include <math.h>

#include "cwac_internal.h"

namespace cwac {
namespace {

constexpr int kRangeBlocks = 1024;
constexpr int kThreads = 256;

// ---- min / max (inputs of Eq. 2): two deterministic stages ------------------
__global__ __launch_bounds__(kThreads) void range_partial_kernel(const float *__restrict__ x,
                                                                 int64_t count, int vec_ok,
                                                                 float *__restrict__ partial) {
  float lo = FLT_MAX, hi = -FLT_MAX;
  const int64_t tid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  const int64_t nthreads = (int64_t)gridDim.x * kThreads;
  if (vec_ok) {
    const int64_t nvec = count >> 2;
    const float4 *xv = reinterpret_cast<const float4 *>(x);
    for (int64_t i = tid; i < nvec; i += nthreads) {
      const float4 v = xv[i];
      lo = fminf(fminf(lo, v.x), fminf(v.y, fminf(v.z, v.w)));
      hi = fmaxf(fmaxf(hi, v.x), fmaxf(v.y, fmaxf(v.z, v.w)));
    }
    for (int64_t i = (nvec << 2) + tid; i < count; i += nthreads) {
      lo = fminf(lo, x[i]);
      hi = fmaxf(hi, x[i]);
    }
  } else {
    for (int64_t i = tid; i < count; i += nthreads) {
      lo = fminf(lo, x[i]);
      hi = fmaxf(hi, x[i]);
    }
  }
  lo = wave_min(lo);
  hi = wave_max(hi);
  __shared__ float s_lo[kThreads / kWave], s_hi[kThreads / kWave];
  const int w = threadIdx.x / kWave;
  if ((threadIdx.x & (kWave - 1)) == 0) {
    s_lo[w] = lo;
    s_hi[w] = hi;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int i = 1; i < kThreads / kWave; ++i) {
      lo = fminf(lo, s_lo[i]);
      hi = fmaxf(hi, s_hi[i]);
    }
    partial[2 * blockIdx.x] = lo;
    partial[2 * blockIdx.x + 1] = hi;
  }
}

__global__ __launch_bounds__(kThreads) void range_final_kernel(const float *__restrict__ partial,
                                                               int nblocks,
                                                               float *__restrict__ minmax) {
  float lo = FLT_MAX, hi = -FLT_MAX;
  for (int i = threadIdx.x; i < nblocks; i += kThreads) {
    lo = fminf(lo, partial[2 * i]);
    hi = fmaxf(hi, partial[2 * i + 1]);
  }
  lo = wave_min(lo);
  hi = wave_max(hi);
  __shared__ float s_lo[kThreads / kWave], s_hi[kThreads / kWave];
  const int w = threadIdx.x / kWave;
  if ((threadIdx.x & (kWave - 1)) == 0) {
    s_lo[w] = lo;
    s_hi[w] = hi;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int i = 1; i < kThreads / kWave; ++i) {
      lo = fminf(lo, s_lo[i]);
      hi = fmaxf(hi, s_hi[i]);
    }
    minmax[0] = lo;
    minmax[1] = hi;
  }
}

// ---- Eq. 1, per-tensor parameters, b-bit codes in signed 8-bit storage ------
// zu = unsigned zero-point, levels = 2^b - 1, half = 2^(b-1)
struct ActQ {
  float s, zu, levels;
  int half;
};
__device__ __forceinline__ int act_code(float x, const ActQ &a) {
  float v = rintf(__fdiv_rn(x, a.s)) + a.zu;
  v = fmaxf(v, 0.0f);
  v = fminf(v, a.levels);
  return static_cast<int>(v) - a.half;
}

__global__ __launch_bounds__(kThreads) void quantize_act_vec_kernel(const float *__restrict__ x,
                                                                    int64_t ldx, int64_t rows,
                                                                    int kv, ActQ a,
                                                                    int8_t *__restrict__ q,
                                                                    int64_t ldq) {
  const int64_t total = rows * kv;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * kThreads) {
    const int64_t r = i / kv;
    const int c = static_cast<int>(i - r * kv) * 4;
    const float4 v = *reinterpret_cast<const float4 *>(x + r * ldx + c);
    const uint32_t b0 = act_code(v.x, a) & 0xff, b1 = act_code(v.y, a) & 0xff,
                   b2 = act_code(v.z, a) & 0xff, b3 = act_code(v.w, a) & 0xff;
    *reinterpret_cast<uint32_t *>(q + r * ldq + c) = b0 | (b1 << 8) | (b2 << 16) | (b3 << 24);
  }
}

__global__ __launch_bounds__(kThreads) void quantize_act_kernel(const float *__restrict__ x,
                                                                int64_t ldx, int64_t rows, int k,
                                                                ActQ a, int8_t *__restrict__ q,
                                                                int64_t ldq) {
  const int64_t total = rows * k;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * kThreads) {
    const int64_t r = i / k;
    const int64_t c = i - r * k;
    q[r * ldq + c] = static_cast<int8_t>(act_code(x[r * ldx + c], a));
  }
}

// ---- symmetric per-row quantizer: one workgroup per row ---------------------
__device__ __forceinline__ int sym_code(float x, float s, float qmax) {
  float v = rintf(__fdiv_rn(x, s));
  v = fmaxf(v, -qmax);
  v = fminf(v, qmax);
  return static_cast<int>(v);
}

__global__ __launch_bounds__(kThreads) void quantize_rows_sym_kernel(
    const float *__restrict__ x, int64_t ldx, int k, int vec_ok, float qmax,
    float *__restrict__ scale, int8_t *__restrict__ q, int64_t ldq) {
  const int64_t row = blockIdx.x;
  const float *xr = x + row * ldx;
  int8_t *qr = q + row * ldq;
  float amax = 0.0f;
  if (vec_ok) {
    for (int c = threadIdx.x * 4; c < k; c += kThreads * 4) {
      const float4 v = *reinterpret_cast<const float4 *>(xr + c);
      amax = fmaxf(fmaxf(amax, fabsf(v.x)), fmaxf(fabsf(v.y), fmaxf(fabsf(v.z), fabsf(v.w))));
    }
  } else {
    for (int c = threadIdx.x; c < k; c += kThreads) amax = fmaxf(amax, fabsf(xr[c]));
  }
  amax = wave_max(amax);
  __shared__ float s_max[kThreads / kWave];
  if ((threadIdx.x & (kWave - 1)) == 0) s_max[threadIdx.x / kWave] = amax;
  __syncthreads();
  amax = s_max[0];
  for (int i = 1; i < kThreads / kWave; ++i) amax = fmaxf(amax, s_max[i]);
  float s = __fdiv_rn(amax, qmax);
  const float floor_s = FLT_MIN * 256.0f;
  if (!(s >= floor_s)) s = floor_s;
  if (threadIdx.x == 0) scale[row] = s;
  if (vec_ok) {
    for (int c = threadIdx.x * 4; c < k; c += kThreads * 4) {
      const float4 v = *reinterpret_cast<const float4 *>(xr + c);
      const uint32_t b0 = sym_code(v.x, s, qmax) & 0xff, b1 = sym_code(v.y, s, qmax) & 0xff,
                     b2 = sym_code(v.z, s, qmax) & 0xff, b3 = sym_code(v.w, s, qmax) & 0xff;
      *reinterpret_cast<uint32_t *>(qr + c) = b0 | (b1 << 8) | (b2 << 16) | (b3 << 24);
    }
  } else {
    for (int c = threadIdx.x; c < k; c += kThreads)
      qr[c] = static_cast<int8_t>(sym_code(xr[c], s, qmax));
  }
}

// ---- colsum[n] = sum_k w_q[n,k]: one wavefront per row ----------------------
__global__ __launch_bounds__(kThreads) void colsum_kernel(const int8_t *__restrict__ w,
                                                          int64_t ldw, int n, int k, int vec_ok,
                                                          int32_t *__restrict__ colsum) {
  const int row = blockIdx.x * (kThreads / kWave) + threadIdx.x / kWave;
  if (row >= n) return;
  const int lane = threadIdx.x & (kWave - 1);
  const int8_t *wr = w + (int64_t)row * ldw;
  int s = 0;
  if (vec_ok) {
    for (int c = lane * 16; c < k; c += kWave * 16) {
      const int4 v = *reinterpret_cast<const int4 *>(wr + c);
      const int words[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int j = 0; j < 4; ++j)
        s += (words[j] << 24 >> 24) + (words[j] << 16 >> 24) + (words[j] << 8 >> 24) +
             (words[j] >> 24);
    }
  } else {
    for (int c = lane; c < k; c += kWave) s += wr[c];
  }
  s = wave_sum(s);
  if (lane == 0) colsum[row] = s;
}

}  // namespace
}  // namespace cwac

using namespace cwac;

extern "C" size_t cwac_range_workspace(int64_t count) {
  (void)count;
  return (size_t)kRangeBlocks * 2 * sizeof(float);
}

extern "C" cwac_status cwac_range_f32(const float *x, int64_t count, float *minmax,
                                      void *workspace, size_t workspace_bytes, void *stream) {
  if (!x || !minmax) return CWAC_E_NULL;
  if (count < 1) return CWAC_E_SHAPE;
  if (!workspace || workspace_bytes < cwac_range_workspace(count)) return CWAC_E_WORKSPACE;
  if (!aligned(x, 4) || !aligned(minmax, 4) || !aligned(workspace, 8)) return CWAC_E_ALIGN;
  const int vec_ok = aligned(x, 16);
  int blocks = (int)(ceil_div(count, (int64_t)kThreads * 16) < kRangeBlocks
                         ? ceil_div(count, (int64_t)kThreads * 16)
                         : kRangeBlocks);
  float *partial = static_cast<float *>(workspace);
  range_partial_kernel<<<blocks, kThreads, 0, as_stream(stream)>>>(x, count, vec_ok, partial);
  range_final_kernel<<<1, kThreads, 0, as_stream(stream)>>>(partial, blocks, minmax);
  return launch_status();
}

extern "C" cwac_status cwac_qparams_from_range(float mn, float mx, int32_t bits, float *s,
                                               int32_t *z) {
  if (!s || !z) return CWAC_E_NULL;
  if (bits < 2 || bits > 8) return CWAC_E_SHAPE;
  // Eq. 2 in fp32; volatile keeps each operation a separately rounded fp32 op.
  const float levels = (float)((1 << bits) - 1);
  volatile float diff = mx - mn;
  volatile float scale = diff / levels;
  const float floor_s = FLT_MIN * (float)(1 << bits);
  if (!(scale >= floor_s)) scale = floor_s;
  volatile float ratio = -mn / scale;
  float zf = rintf(ratio);
  if (zf < 0.0f) zf = 0.0f;
  if (zf > levels) zf = levels;
  *s = scale;
  *z = (int32_t)zf;
  return CWAC_OK;
}

extern "C" cwac_status cwac_quantize_act_bits(const float *x, int64_t ldx, int64_t rows, int32_t k,
                                              float s, int32_t z, int32_t bits, int8_t *q,
                                              int64_t ldq, void *stream) {
  if (!x || !q) return CWAC_E_NULL;
  if (bits < 2 || bits > 8) return CWAC_E_SHAPE;
  const int half = 1 << (bits - 1);
  if (rows < 0 || k < 1 || ldx < k || ldq < k || !(s > 0.0f) || z < -half || z > half - 1)
    return CWAC_E_SHAPE;
  if (!aligned(x, 4)) return CWAC_E_ALIGN;
  if (rows == 0) return CWAC_OK;
  ActQ a;
  a.s = s;
  a.zu = (float)(z + half);
  a.levels = (float)((1 << bits) - 1);
  a.half = half;
  const bool vec = (k % 4 == 0) && (ldx % 4 == 0) && (ldq % 4 == 0) && aligned(x, 16) &&
                   aligned(q, 4);
  const int64_t work = vec ? rows * (k / 4) : rows * (int64_t)k;
  const int64_t want = ceil_div(work, kThreads);
  const int blocks = (int)(want < 65536 ? want : 65536);
  if (vec)
    quantize_act_vec_kernel<<<blocks, kThreads, 0, as_stream(stream)>>>(x, ldx, rows, k / 4, a, q,
                                                                         ldq);
  else
    quantize_act_kernel<<<blocks, kThreads, 0, as_stream(stream)>>>(x, ldx, rows, k, a, q, ldq);
  return launch_status();
}

extern "C" cwac_status cwac_quantize_act(const float *x, int64_t ldx, int64_t rows, int32_t k,
                                         float s, int32_t z, int8_t *q, int64_t ldq,
                                         void *stream) {
  return cwac_quantize_act_bits(x, ldx, rows, k, s, z, 8, q, ldq, stream);
}

extern "C" cwac_status cwac_quantize_rows_sym_bits(const float *x, int64_t ldx, int64_t rows,
                                                   int32_t k, int32_t bits, float *scale,
                                                   int8_t *q, int64_t ldq, void *stream) {
  if (!x || !q || !scale) return CWAC_E_NULL;
  if (bits < 2 || bits > 8) return CWAC_E_SHAPE;
  if (rows < 0 || rows > 0x7fffffff || k < 1 || ldx < k || ldq < k) return CWAC_E_SHAPE;
  if (!aligned(x, 4) || !aligned(scale, 4)) return CWAC_E_ALIGN;
  if (rows == 0) return CWAC_OK;
  const int vec = (k % 4 == 0) && (ldx % 4 == 0) && (ldq % 4 == 0) && aligned(x, 16) &&
                  aligned(q, 4);
  const float qmax = (float)((1 << (bits - 1)) - 1);
  quantize_rows_sym_kernel<<<(unsigned)rows, kThreads, 0, as_stream(stream)>>>(x, ldx, k, vec, qmax,
                                                                                scale, q, ldq);
  return launch_status();
}

extern "C" cwac_status cwac_quantize_rows_sym(const float *x, int64_t ldx, int64_t rows,
                                              int32_t k, float *scale, int8_t *q, int64_t ldq,
                                              void *stream) {
  return cwac_quantize_rows_sym_bits(x, ldx, rows, k, 8, scale, q, ldq, stream);
}

extern "C" cwac_status cwac_colsum(const int8_t *w_q, int64_t ldw, int32_t n, int32_t k,
                                   int32_t *colsum, void *stream) {
  if (!w_q || !colsum) return CWAC_E_NULL;
  if (n < 1 || k < 1 || ldw < k) return CWAC_E_SHAPE;
  if (!aligned(colsum, 4)) return CWAC_E_ALIGN;
  const int vec = (k % 16 == 0) && (ldw % 16 == 0) && aligned(w_q, 16);
  const int rows_per_block = kThreads / kWave;
  colsum_kernel<<<(unsigned)ceil_div(n, rows_per_block), kThreads, 0, as_stream(stream)>>>(
      w_q, ldw, n, k, vec, colsum);
  return launch_status();
}
