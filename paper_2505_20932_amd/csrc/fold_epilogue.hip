// Folding of the compensation into the engine parameters (Sec. 3.4, Eq. 7-8 and
// Eq. 10-11), and the two un-fused comparators: the epilogue as a separate pass
// over stored accumulators, and the compensation as a separate affine module.
#include "cwac_internal.h"

namespace cwac {
namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ double sat_round(double v, double lim, int &nsat) {
  double r = rint(v);
  if (!(r <= lim)) {
    r = (r != r) ? 0.0 : lim;
    ++nsat;
  } else if (r < -lim) {
    r = -lim;
    ++nsat;
  }
  return r;
}

__global__ void zero_count_kernel(int32_t *p) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *p = 0;
}

// Grid-stride over channels, O(channels) work.  With several workgroups the saturation count is
// added atomically (integer, order-independent) to a counter the host zeroed beforehand.
__global__ __launch_bounds__(256) void fold_kernel(
    const float *__restrict__ alpha, const float *__restrict__ beta,
    const float *__restrict__ sw, const float *__restrict__ bias,
    const int32_t *__restrict__ colsum, int n_out, int mode, int per_token, float sx, int zx,
    float sr, float *__restrict__ mult, int32_t *__restrict__ offset, float *__restrict__ fbias,
    int32_t *__restrict__ n_saturated) {
  int nsat = 0;
  const double lim = 1073741824.0;  // 2^30
  for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < n_out; c += gridDim.x * blockDim.x) {
    const double a = alpha ? (double)alpha[c] : 1.0;
    const double b = beta ? (double)beta[c] : 0.0;
    const double w = (double)sw[c];
    if (mode == CWAC_EPI_INT_OFFSET) {
      const double asx = a * (double)sx;
      const double den = asx * w;
      mult[c] = (float)(den / (double)sr);
      const double unit = (double)sx * w;
      double bq = 0.0;
      if (b != 0.0) bq = rint(b / den);
      double biasq = 0.0;
      if (bias) biasq = rint((double)bias[c] / unit);
      const double sum = sat_round(bq + biasq, lim, nsat);
      offset[c] = (int32_t)sum - zx * colsum[c];
    } else {
      double num;
      if (per_token) num = a * w;
      else num = (a * (double)sx) * w;
      mult[c] = (float)(num / (double)sr);
      const double bb = bias ? (double)bias[c] : 0.0;
      const double ab = a * bb;
      fbias[c] = (float)((ab + b) / (double)sr);
      offset[c] = -zx * colsum[c];
    }
  }
  if (n_saturated) {
    __shared__ int s_cnt[256 / kWave];
    nsat = wave_sum(nsat);
    if ((threadIdx.x & (kWave - 1)) == 0) s_cnt[threadIdx.x / kWave] = nsat;
    __syncthreads();
    if (threadIdx.x == 0) {
      int t = 0;
      for (int i = 0; i < (int)(blockDim.x / kWave); ++i) t += s_cnt[i];
      if (gridDim.x == 1) *n_saturated = t;
      else if (t) atomicAdd(n_saturated, t);
    }
  }
}

// Fixed-point form of a real multiplier: M0 * 2^-shift with 2^30 <= |M0| < 2^31 (31 significant
// bits), 1 <= shift <= 62; larger multipliers are clamped (counted), smaller ones become 0.
__device__ inline void fixed_point_of(double mreal, int32_t &m0, int32_t &shift, int &nsat) {
  m0 = 0;
  shift = 1;
  if (!(mreal == mreal) || mreal == 0.0) return;
  int e = 0;
  const double mant = frexp(fabs(mreal), &e);
  long long q = llrint(mant * 2147483648.0);
  if (q == 2147483648LL) {
    q = 1073741824LL;
    e += 1;
  }
  int sh = 31 - e;
  if (sh > 62) return;
  if (sh < 1) {
    q = 2147483647LL;
    sh = 1;
    ++nsat;
  }
  m0 = (int32_t)(mreal < 0.0 ? -q : q);
  shift = sh;
}

// Eq. 10-11 with the multiplier in fixed point (integer-only engine form); the offset is the
// integer-offset fold's.
__global__ __launch_bounds__(256) void fold_fixed_kernel(
    const float *__restrict__ alpha, const float *__restrict__ beta,
    const float *__restrict__ sw, const float *__restrict__ bias,
    const int32_t *__restrict__ colsum, int n_out, float sx, int zx, float sr,
    int32_t *__restrict__ m0, int32_t *__restrict__ shift, int32_t *__restrict__ offset,
    int32_t *__restrict__ n_saturated) {
  int nsat = 0;
  const double lim = 1073741824.0;  // 2^30
  for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < n_out; c += gridDim.x * blockDim.x) {
    const double a = alpha ? (double)alpha[c] : 1.0;
    const double b = beta ? (double)beta[c] : 0.0;
    const double w = (double)sw[c];
    const double asx = a * (double)sx;
    const double den = asx * w;
    int32_t q, sh;
    fixed_point_of(den / (double)sr, q, sh, nsat);
    m0[c] = q;
    shift[c] = sh;
    const double unit = (double)sx * w;
    double bq = 0.0;
    if (b != 0.0) bq = rint(b / den);
    double biasq = 0.0;
    if (bias) biasq = rint((double)bias[c] / unit);
    const double sum = sat_round(bq + biasq, lim, nsat);
    offset[c] = (int32_t)sum - zx * colsum[c];
  }
  if (n_saturated) {
    __shared__ int s_cnt[256 / kWave];
    nsat = wave_sum(nsat);
    if ((threadIdx.x & (kWave - 1)) == 0) s_cnt[threadIdx.x / kWave] = nsat;
    __syncthreads();
    if (threadIdx.x == 0) {
      int t = 0;
      for (int i = 0; i < (int)(blockDim.x / kWave); ++i) t += s_cnt[i];
      if (gridDim.x == 1) *n_saturated = t;
      else if (t) atomicAdd(n_saturated, t);
    }
  }
}

// Epilogue of Eq. 10 as its own pass: int32 accumulators in, codes (or fp32) out.
template <int OUT_KIND>
__global__ __launch_bounds__(kThreads) void epilogue_pass_kernel(
    const int32_t *__restrict__ acc, int64_t ldacc, int64_t m, int n, int nv,
    const float *__restrict__ mult, const int32_t *__restrict__ offset,
    const float *__restrict__ fbias, const float *__restrict__ sx_row, float lo, float hi, int zr,
    void *__restrict__ out, int64_t ldo) {
  // each lane: 4 adjacent channels of one row (16-byte accumulator load)
  const int64_t total = m * nv;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * kThreads) {
    const int64_t r = i / nv;
    const int c = (int)(i - r * nv) * 4;
    const int4 a = *reinterpret_cast<const int4 *>(acc + r * ldacc + c);
    const int t[4] = {a.x, a.y, a.z, a.w};
    float u[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float f = (float)(t[j] + (offset ? offset[c + j] : 0));
      if (sx_row) f = f * sx_row[r];
      float v = f * mult[c + j];
      if (fbias) v = v + fbias[c + j];
      u[j] = v;
    }
    if (OUT_KIND == CWAC_OUT_INT8) {
      uint32_t pk = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) pk |= (uint32_t)(requant_code(u[j], lo, hi, zr) & 0xff) << (8 * j);
      *reinterpret_cast<uint32_t *>(static_cast<int8_t *>(out) + r * ldo + c) = pk;
    } else {
      *reinterpret_cast<float4 *>(static_cast<float *>(out) + r * ldo + c) =
          make_float4(u[0], u[1], u[2], u[3]);
    }
  }
}

// Generic layout fallback: one element per lane.
template <int OUT_KIND>
__global__ __launch_bounds__(kThreads) void epilogue_pass_scalar_kernel(
    const int32_t *__restrict__ acc, int64_t ldacc, int64_t m, int n,
    const float *__restrict__ mult, const int32_t *__restrict__ offset,
    const float *__restrict__ fbias, const float *__restrict__ sx_row, float lo, float hi, int zr,
    void *__restrict__ out, int64_t ldo) {
  const int64_t total = m * n;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * kThreads) {
    const int64_t r = i / n;
    const int c = (int)(i - r * n);
    float f = (float)(acc[r * ldacc + c] + (offset ? offset[c] : 0));
    if (sx_row) f = f * sx_row[r];
    float v = f * mult[c];
    if (fbias) v = v + fbias[c];
    if (OUT_KIND == CWAC_OUT_INT8)
      static_cast<int8_t *>(out)[r * ldo + c] = (int8_t)requant_code(v, lo, hi, zr);
    else
      static_cast<float *>(out)[r * ldo + c] = v;
  }
}

// out = alpha .* y + beta, two fp32 roundings (Sec. 3.3).
__global__ __launch_bounds__(kThreads) void apply_unfolded_kernel(
    const float *y, int64_t ldy, int64_t rows, int c, int vec, const float *__restrict__ alpha,
    const float *__restrict__ beta, float *out, int64_t ldo) {
  if (vec) {
    const int cv = c / 4;
    const int64_t total = rows * cv;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * kThreads) {
      const int64_t r = i / cv;
      const int ch = (int)(i - r * cv) * 4;
      const float4 v = *reinterpret_cast<const float4 *>(y + r * ldy + ch);
      const float4 a = *reinterpret_cast<const float4 *>(alpha + ch);
      const float4 b = *reinterpret_cast<const float4 *>(beta + ch);
      float4 o;
      o.x = a.x * v.x; o.x = o.x + b.x;
      o.y = a.y * v.y; o.y = o.y + b.y;
      o.z = a.z * v.z; o.z = o.z + b.z;
      o.w = a.w * v.w; o.w = o.w + b.w;
      *reinterpret_cast<float4 *>(out + r * ldo + ch) = o;
    }
  } else {
    const int64_t total = rows * c;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * kThreads) {
      const int64_t r = i / c;
      const int ch = (int)(i - r * c);
      float v = alpha[ch] * y[r * ldy + ch];
      out[r * ldo + ch] = v + beta[ch];
    }
  }
}

inline unsigned grid_for(int64_t work) {
  const int64_t want = ceil_div(work, kThreads);
  const int64_t cap = 256 * 32;  // 32 workgroups per compute unit, grid-stride beyond
  return (unsigned)(want < cap ? want : cap);
}

}  // namespace
}  // namespace cwac

using namespace cwac;

static cwac_status check_qparams(const cwac_qparams *qp) {
  if (!qp) return CWAC_E_NULL;
  if (qp->mode != CWAC_EPI_INT_OFFSET && qp->mode != CWAC_EPI_FP_BIAS) return CWAC_E_MODE;
  if (qp->act_per_token && qp->mode != CWAC_EPI_FP_BIAS) return CWAC_E_MODE;
  if (qp->act_per_token && qp->z_x != 0) return CWAC_E_MODE;
  if (!(qp->s_r > 0.0f)) return CWAC_E_SHAPE;
  if (!qp->act_per_token && !(qp->s_x > 0.0f)) return CWAC_E_SHAPE;
  if (qp->z_x < -128 || qp->z_x > 127) return CWAC_E_SHAPE;
  return CWAC_OK;
}

extern "C" cwac_status cwac_fold(const float *alpha, const float *beta, const float *s_w,
                                 const float *bias, const int32_t *colsum, int32_t n_out,
                                 const cwac_qparams *qp, float *mult, int32_t *offset,
                                 float *fbias, int32_t *n_saturated, void *stream) {
  if (!s_w || !colsum || !mult || !offset) return CWAC_E_NULL;
  cwac_status st = check_qparams(qp);
  if (st != CWAC_OK) return st;
  if ((alpha == nullptr) != (beta == nullptr)) return CWAC_E_MODE;
  if (qp->mode == CWAC_EPI_FP_BIAS && !fbias) return CWAC_E_NULL;
  if (n_out < 1 || n_out > 65536) return CWAC_E_SHAPE;
  const unsigned blocks = (unsigned)ceil_div(n_out, 256);
  if (n_saturated && blocks > 1) zero_count_kernel<<<1, 64, 0, as_stream(stream)>>>(n_saturated);
  fold_kernel<<<blocks, 256, 0, as_stream(stream)>>>(alpha, beta, s_w, bias, colsum, n_out, qp->mode,
                                                 qp->act_per_token, qp->s_x, qp->z_x, qp->s_r,
                                                 mult, offset, fbias, n_saturated);
  return launch_status();
}

extern "C" cwac_status cwac_fold_fixed_point(const float *alpha, const float *beta, const float *s_w,
                                             const float *bias, const int32_t *colsum,
                                             int32_t n_out, const cwac_qparams *qp, int32_t *m0,
                                             int32_t *shift, int32_t *offset,
                                             int32_t *n_saturated, void *stream) {
  if (!s_w || !colsum || !m0 || !shift || !offset) return CWAC_E_NULL;
  cwac_status st = check_qparams(qp);
  if (st != CWAC_OK) return st;
  if ((alpha == nullptr) != (beta == nullptr)) return CWAC_E_MODE;
  if (qp->mode != CWAC_EPI_INT_OFFSET || qp->act_per_token) return CWAC_E_MODE;
  if (n_out < 1 || n_out > 65536) return CWAC_E_SHAPE;
  const unsigned blocks = (unsigned)ceil_div(n_out, 256);
  if (n_saturated && blocks > 1) zero_count_kernel<<<1, 64, 0, as_stream(stream)>>>(n_saturated);
  fold_fixed_kernel<<<blocks, 256, 0, as_stream(stream)>>>(alpha, beta, s_w, bias, colsum, n_out,
                                                           qp->s_x, qp->z_x, qp->s_r, m0, shift,
                                                           offset, n_saturated);
  return launch_status();
}

extern "C" cwac_status cwac_epilogue_int32(const int32_t *acc, int64_t ldacc, int64_t m, int32_t n,
                                           const cwac_qparams *qp, const float *mult,
                                           const int32_t *offset, const float *fbias,
                                           const float *s_x_row, int32_t out_kind, void *out,
                                           int64_t ldo, void *stream) {
  if (!acc || !mult || !out) return CWAC_E_NULL;
  if (out_kind != CWAC_OUT_INT8 && out_kind != CWAC_OUT_FP32) return CWAC_E_MODE;
  if (m < 0 || n < 1 || ldacc < n || ldo < n) return CWAC_E_SHAPE;
  float lo = 0.0f, hi = 0.0f;
  int zr = 0;
  if (out_kind == CWAC_OUT_INT8) {
    if (!qp) return CWAC_E_NULL;
    if (qp->qmin < -128 || qp->qmax > 127 || qp->qmin > qp->qmax) return CWAC_E_SHAPE;
    zr = qp->z_r;
    lo = (float)(qp->qmin - zr);
    hi = (float)(qp->qmax - zr);
  }
  if (m == 0) return CWAC_OK;
  const size_t esz = out_kind == CWAC_OUT_INT8 ? 1 : 4;
  const bool vec = (n % 4 == 0) && (ldacc % 4 == 0) && aligned(acc, 16) &&
                   ((ldo * esz) % (4 * esz) == 0) && aligned(out, 4 * esz);
  hipStream_t st = as_stream(stream);
  if (vec) {
    const unsigned g = grid_for(m * (n / 4));
    if (out_kind == CWAC_OUT_INT8)
      epilogue_pass_kernel<CWAC_OUT_INT8><<<g, kThreads, 0, st>>>(
          acc, ldacc, m, n, n / 4, mult, offset, fbias, s_x_row, lo, hi, zr, out, ldo);
    else
      epilogue_pass_kernel<CWAC_OUT_FP32><<<g, kThreads, 0, st>>>(
          acc, ldacc, m, n, n / 4, mult, offset, fbias, s_x_row, lo, hi, zr, out, ldo);
  } else {
    const unsigned g = grid_for(m * (int64_t)n);
    if (out_kind == CWAC_OUT_INT8)
      epilogue_pass_scalar_kernel<CWAC_OUT_INT8><<<g, kThreads, 0, st>>>(
          acc, ldacc, m, n, mult, offset, fbias, s_x_row, lo, hi, zr, out, ldo);
    else
      epilogue_pass_scalar_kernel<CWAC_OUT_FP32><<<g, kThreads, 0, st>>>(
          acc, ldacc, m, n, mult, offset, fbias, s_x_row, lo, hi, zr, out, ldo);
  }
  return launch_status();
}

extern "C" cwac_status cwac_apply_unfolded(const float *y, int64_t ldy, int64_t rows, int32_t c,
                                           const float *alpha, const float *beta, float *out,
                                           int64_t ldo, void *stream) {
  if (!y || !alpha || !beta || !out) return CWAC_E_NULL;
  if (rows < 0 || c < 1 || ldy < c || ldo < c) return CWAC_E_SHAPE;
  if (rows == 0) return CWAC_OK;
  const int vec = (c % 4 == 0) && (ldy % 4 == 0) && (ldo % 4 == 0) && aligned(y, 16) &&
                  aligned(out, 16) && aligned(alpha, 16) && aligned(beta, 16);
  const int64_t work = vec ? rows * (c / 4) : rows * (int64_t)c;
  apply_unfolded_kernel<<<grid_for(work), kThreads, 0, as_stream(stream)>>>(y, ldy, rows, c, vec,
                                                                             alpha, beta, out, ldo);
  return launch_status();
}
