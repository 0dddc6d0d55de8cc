/*
 * CPU oracle for the QwT-v2 quantized-linear + CWAC hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow definition that the
 * GPU library is checked against.  Nothing in the product path may include,
 * link or call it; only tests, the smoke check and the benchmark's CPU-baseline
 * leg do.  It shares no code, header, table or helper with the HIP sources.
 *
 * Style: scalar loops, one output at a time, in the order and notation of the
 * paper.  Floating point follows the precision the method fixes: the engine
 * epilogue (Sec. 3.4, Eq. 7-11) is a chain of single fp32 operations with no
 * fused multiply-add; statistics, the closed-form fit (Sec. 3.3, Eq. 3-5) and
 * the fold (Eq. 10-11) are evaluated in fp64 and rounded once to the stored
 * type.  Build with -O2 -ffp-contract=off and no fast-math.  The optional
 * OpenMP pragmas only distribute independent outputs (rows / channel blocks)
 * over threads; every output is still produced by one thread in a fixed order,
 * so results do not depend on the thread count.
 *
 * Parity status: every function below is pinned by tests that do not call it
 * to produce their own expectation (hand-derived fixtures, exact rational
 * arithmetic, numpy library routines, algebraic identities, brute force).
 * The accuracy tables of the paper need datasets and weights and are
 * "parity unpinned" (not attempted).
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ */
/* thread control (timing only)                                        */
/* ------------------------------------------------------------------ */
void orc_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

int orc_get_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* Quantizers (Sec. 3.2, Eq. 1-2)                                      */
/* ------------------------------------------------------------------ */

/* min and max of a tensor (inputs of Eq. 2). */
void orc_range_f32(const float *x, int64_t count, float *mn, float *mx) {
  float lo = x[0], hi = x[0];
  for (int64_t i = 1; i < count; ++i) {
    if (x[i] < lo) lo = x[i];
    if (x[i] > hi) hi = x[i];
  }
  *mn = lo;
  *mx = hi;
}

/* Eq. 2: s = (max - min) / (2^b - 1), z = clip(round(-min / s), 0, 2^b - 1).
 * fp32 arithmetic, round-half-to-even.  A constant tensor would give s = 0;
 * the scale is floored at FLT_MIN * 2^b so that Eq. 1 stays defined. */
void orc_qparams_asym(float mn, float mx, int32_t bits, float *s, int32_t *z) {
  const float levels = (float)((1 << bits) - 1);
  float scale = (mx - mn) / levels;
  const float floor_s = FLT_MIN * (float)(1 << bits);
  if (!(scale >= floor_s)) scale = floor_s;
  float zf = rintf(-mn / scale);
  if (zf < 0.0f) zf = 0.0f;
  if (zf > levels) zf = levels;
  *s = scale;
  *z = (int32_t)zf;
}

/* Eq. 1: x_q = clip(round(x / s) + z, 0, 2^b - 1), unsigned codes. */
void orc_quantize_asym(const float *x, int64_t count, float s, int32_t z,
                       int32_t bits, int32_t *codes) {
  const float levels = (float)((1 << bits) - 1);
  for (int64_t i = 0; i < count; ++i) {
    float v = rintf(x[i] / s) + (float)z;
    if (v < 0.0f) v = 0.0f;
    if (v > levels) v = levels;
    codes[i] = (int32_t)v;
  }
}

/* 8-bit activations in signed storage: stored value = Eq. 1 code - 128 and the
 * zero-point is shifted by the same 128, so s * (q - z) is unchanged. */
void orc_quantize_act_i8(const float *x, int64_t count, float s, int32_t z_signed,
                         int8_t *q) {
  const int32_t z_u = z_signed + 128;
  for (int64_t i = 0; i < count; ++i) {
    float v = rintf(x[i] / s) + (float)z_u;
    if (v < 0.0f) v = 0.0f;
    if (v > 255.0f) v = 255.0f;
    q[i] = (int8_t)((int32_t)v - 128);
  }
}

/* Symmetric per-row quantizer (weights per output channel; activations per
 * token): scale[r] = max_k |x[r,k]| / 127, q = clip(round(x / scale), -127, 127),
 * zero-point 0.  An all-zero row gets the floored scale and all-zero codes. */
void orc_quantize_rows_sym(const float *x, int64_t rows, int64_t k, int64_t ld,
                           float *scale, int8_t *q, int64_t ldq) {
  for (int64_t r = 0; r < rows; ++r) {
    const float *xr = x + r * ld;
    float amax = 0.0f;
    for (int64_t j = 0; j < k; ++j) {
      float a = fabsf(xr[j]);
      if (a > amax) amax = a;
    }
    float s = amax / 127.0f;
    const float floor_s = FLT_MIN * 256.0f;
    if (!(s >= floor_s)) s = floor_s;
    scale[r] = s;
    for (int64_t j = 0; j < k; ++j) {
      float v = rintf(xr[j] / s);
      if (v < -127.0f) v = -127.0f;
      if (v > 127.0f) v = 127.0f;
      q[r * ldq + j] = (int8_t)(int32_t)v;
    }
  }
}

/* The same two quantizers at b bits (2 <= b <= 8) with the codes kept in int8
 * containers - the low-bit settings of the paper's tables (W4A4, W6A6):
 * activations: stored value = Eq. 1 code - 2^(b-1), zero-point shifted alike;
 * weights / per-token activations: symmetric, scale = max|x| / (2^(b-1) - 1),
 * codes in [-(2^(b-1) - 1), 2^(b-1) - 1]. */
void orc_quantize_act_bits(const float *x, int64_t count, float s, int32_t z_signed,
                           int32_t bits, int8_t *q) {
  const int32_t half = 1 << (bits - 1);
  const float levels = (float)((1 << bits) - 1);
  const int32_t z_u = z_signed + half;
  for (int64_t i = 0; i < count; ++i) {
    float v = rintf(x[i] / s) + (float)z_u;
    if (v < 0.0f) v = 0.0f;
    if (v > levels) v = levels;
    q[i] = (int8_t)((int32_t)v - half);
  }
}

void orc_quantize_rows_sym_bits(const float *x, int64_t rows, int64_t k, int64_t ld,
                                int32_t bits, float *scale, int8_t *q, int64_t ldq) {
  const float qmax = (float)((1 << (bits - 1)) - 1);
  for (int64_t r = 0; r < rows; ++r) {
    const float *xr = x + r * ld;
    float amax = 0.0f;
    for (int64_t j = 0; j < k; ++j) {
      float a = fabsf(xr[j]);
      if (a > amax) amax = a;
    }
    float s = amax / qmax;
    const float floor_s = FLT_MIN * 256.0f;
    if (!(s >= floor_s)) s = floor_s;
    scale[r] = s;
    for (int64_t j = 0; j < k; ++j) {
      float v = rintf(xr[j] / s);
      if (v < -qmax) v = -qmax;
      if (v > qmax) v = qmax;
      q[r * ldq + j] = (int8_t)(int32_t)v;
    }
  }
}

/* ------------------------------------------------------------------ */
/* Integer product (the W_q x_q term of Eq. 7 / Eq. 10)                */
/* ------------------------------------------------------------------ */

/* acc[i, n] = sum_k x_q[row(i), k] * w_q[n, k].  rows == NULL means all m rows
 * in order; otherwise rows[0..n_rows) selects input rows and acc has n_rows
 * rows.  x_q is [m, k], w_q is [n, k], both with contiguous k. */
void orc_gemm_i8(const int8_t *xq, const int8_t *wq, int64_t m, int64_t n,
                 int64_t k, const int64_t *rows, int64_t n_rows, int32_t *acc) {
  const int64_t cnt = rows ? n_rows : m;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < cnt; ++i) {
    const int8_t *xr = xq + (rows ? rows[i] : i) * k;
    for (int64_t c = 0; c < n; ++c) {
      const int8_t *wr = wq + c * k;
      int32_t s = 0;
      for (int64_t j = 0; j < k; ++j) s += (int32_t)xr[j] * (int32_t)wr[j];
      acc[i * n + c] = s;
    }
  }
}

/* colsum[n] = sum_k w_q[n, k]: the Z_x W_q term of Eq. 7 is Z_x * colsum[n]. */
void orc_colsum_i8(const int8_t *wq, int64_t n, int64_t k, int32_t *colsum) {
  for (int64_t c = 0; c < n; ++c) {
    int32_t s = 0;
    for (int64_t j = 0; j < k; ++j) s += (int32_t)wq[c * k + j];
    colsum[c] = s;
  }
}

/* Quantized convolution (Sec. 3.3: a CWAC module follows every quantized
 * convolutional layer of a CNN; Sec. 3.4: the fold extends to it): the integer
 * product of Eq. 7 with the sum running over the receptive field,
 *   acc[b, oh, ow, n] = sum_{kh, kw, c} x_q[b, oh*stride + kh - pad, ow*stride + kw - pad, c]
 *                                      * w_q[n, kh, kw, c],
 * where a position outside the image holds the code of the real value zero,
 * i.e. the zero-point Z_x (so that (x_q - Z_x) vanishes there and the zero-point
 * term of Eq. 7 stays Z_x * sum_{kh,kw,c} w_q[n, kh, kw, c]).
 *   x_q  [batch, h, w, c_in]      channels last
 *   w_q  [c_out, kh, kw, c_in]
 *   acc  [batch * oh * ow, c_out] with oh = (h + 2 pad - kh) / stride + 1, likewise ow */
void orc_conv2d_i8(const int8_t *xq, const int8_t *wq, int64_t batch, int64_t h, int64_t w,
                   int64_t c_in, int64_t c_out, int64_t kh, int64_t kw, int64_t stride,
                   int64_t pad, int32_t zx, int32_t *acc) {
  const int64_t oh = (h + 2 * pad - kh) / stride + 1, ow = (w + 2 * pad - kw) / stride + 1;
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < batch * oh * ow; ++m) {
    const int64_t b = m / (oh * ow), y = (m / ow) % oh, x = m % ow;
    for (int64_t n = 0; n < c_out; ++n) {
      int32_t s = 0;
      for (int64_t i = 0; i < kh; ++i)
        for (int64_t j = 0; j < kw; ++j) {
          const int64_t iy = y * stride + i - pad, ix = x * stride + j - pad;
          const int inside = iy >= 0 && iy < h && ix >= 0 && ix < w;
          for (int64_t c = 0; c < c_in; ++c) {
            const int32_t xv = inside ? (int32_t)xq[((b * h + iy) * w + ix) * c_in + c] : zx;
            s += xv * (int32_t)wq[((n * kh + i) * kw + j) * c_in + c];
          }
        }
      acc[m * c_out + n] = s;
    }
  }
}

/* Right-hand side of Eq. 6 without the scales, written directly:
 * sum_k (w_q[n,k] - Z_W[n]) * (x_q[m,k] - Z_x), in 64-bit integers. */
void orc_product_zp_direct(const int8_t *xq, const int8_t *wq, int64_t m,
                           int64_t n, int64_t k, int32_t zx, const int32_t *zw,
                           int64_t *out) {
  for (int64_t i = 0; i < m; ++i)
    for (int64_t c = 0; c < n; ++c) {
      int64_t s = 0;
      for (int64_t j = 0; j < k; ++j)
        s += ((int64_t)wq[c * k + j] - zw[c]) * ((int64_t)xq[i * k + j] - zx);
      out[i * n + c] = s;
    }
}

/* The bracket of Eq. 7, term by term:
 * W_q x_q - Z_W (sum_k x_q) - Z_x (sum_k W_q) + K Z_x Z_W. */
void orc_product_zp_expanded(const int8_t *xq, const int8_t *wq, int64_t m,
                             int64_t n, int64_t k, int32_t zx, const int32_t *zw,
                             int64_t *out) {
  for (int64_t i = 0; i < m; ++i) {
    int64_t rowsum = 0;
    for (int64_t j = 0; j < k; ++j) rowsum += xq[i * k + j];
    for (int64_t c = 0; c < n; ++c) {
      int64_t dot = 0, colsum = 0;
      for (int64_t j = 0; j < k; ++j) {
        dot += (int64_t)wq[c * k + j] * (int64_t)xq[i * k + j];
        colsum += wq[c * k + j];
      }
      out[i * n + c] = dot - (int64_t)zw[c] * rowsum - (int64_t)zx * colsum +
                       k * (int64_t)zx * (int64_t)zw[c];
    }
  }
}

/* ------------------------------------------------------------------ */
/* Unfolded layer: quantized linear, then CWAC as a separate affine,   */
/* then output quantization (Sec. 3.3 last sentence; Eq. 9; Eq. 1).    */
/* ------------------------------------------------------------------ */

/* Dequantized output of the quantized module, Y_quant (Sec. 3.3):
 *   t0 = acc - Z_x * colsum[n]
 *   y  = fl(fl(fl((float)t0 * sx_row[m]) * deq[n]) + bias[n])    per-token
 *   y  = fl(fl((float)t0 * deq[n]) + bias[n])                    per-tensor
 * with deq[n] = fl(S_x * S_W[n]) (per-tensor) or S_W[n] (per-token).
 * sx_row == NULL selects per-tensor; bias == NULL means no bias term at all.
 * acc is [rows, n]; sx_row is indexed by the same local row index. */
void orc_dequant_output(const int32_t *acc, int64_t rows, int64_t n,
                        const int32_t *colsum, int32_t zx, const float *sx_row,
                        const float *deq, const float *bias, float *y) {
  for (int64_t i = 0; i < rows; ++i)
    for (int64_t c = 0; c < n; ++c) {
      const int32_t t0 = acc[i * n + c] - zx * colsum[c];
      float f = (float)t0;
      if (sx_row) f = f * sx_row[i];
      float v = f * deq[c];
      if (bias) v = v + bias[c];
      y[i * n + c] = v;
    }
}

/* deq[n] = fl(S_x * S_W[n]) */
void orc_deq_scale(const float *sw, int64_t n, float sx, float *deq) {
  for (int64_t c = 0; c < n; ++c) deq[c] = sx * sw[c];
}

/* Compensated output alpha .* Y_quant + beta (Sec. 3.3), fp32, two roundings. */
void orc_cwac_apply(const float *yq, int64_t rows, int64_t n, const float *alpha,
                    const float *beta, float *yc) {
  for (int64_t i = 0; i < rows; ++i)
    for (int64_t c = 0; c < n; ++c) {
      float v = alpha[c] * yq[i * n + c];
      yc[i * n + c] = v + beta[c];
    }
}

/* Eq. 1 on the compensated output with the output parameters (S_r, Z_r),
 * signed 8-bit storage: r = clip(round(y / S_r) + Z_r, qmin, qmax). */
void orc_requant_output(const float *y, int64_t count, float sr, int32_t zr,
                        int32_t qmin, int32_t qmax, int8_t *r) {
  for (int64_t i = 0; i < count; ++i) {
    float v = rintf(y[i] / sr) + (float)zr;
    if (v < (float)qmin) v = (float)qmin;
    if (v > (float)qmax) v = (float)qmax;
    r[i] = (int8_t)(int32_t)v;
  }
}

/* Same unfolded chain in fp64 from the integer accumulator, returning the
 * real-valued pre-rounding code u = (alpha * y_quant + beta) / S_r, used by
 * tests to bound the effect of the fold's roundings. */
void orc_unfolded_real(const int32_t *acc, int64_t rows, int64_t n,
                       const int32_t *colsum, int32_t zx, const float *sx_row,
                       const float *sw, float sx, const float *bias,
                       const float *alpha, const float *beta, float sr,
                       double *u) {
  for (int64_t i = 0; i < rows; ++i)
    for (int64_t c = 0; c < n; ++c) {
      const double t0 = (double)acc[i * n + c] - (double)zx * (double)colsum[c];
      const double sxv = sx_row ? (double)sx_row[i] : (double)sx;
      double y = t0 * sxv * (double)sw[c];
      if (bias) y += (double)bias[c];
      u[i * n + c] = ((double)alpha[c] * y + (double)beta[c]) / (double)sr;
    }
}

/* ------------------------------------------------------------------ */
/* CWAC fit (Sec. 3.3, Eq. 3-5)                                        */
/* ------------------------------------------------------------------ */

/* Per-channel empirical moments, two passes in fp64 over all rows:
 * moments[0][c] = E[Y_full], [1] = E[Y_quant], [2] = Var(Y_quant),
 * [3] = Cov(Y_quant, Y_full), [4] = Var(Y_full), all with 1/N. */
void orc_channel_moments(const float *yf, const float *yq, int64_t rows,
                         int64_t c_out, int64_t ldf, int64_t ldq,
                         double *moments) {
  double *mf = moments, *mq = moments + c_out, *vq = moments + 2 * c_out,
         *cqf = moments + 3 * c_out, *vf = moments + 4 * c_out;
  const int64_t blk = 64;
#pragma omp parallel for schedule(static)
  for (int64_t c0 = 0; c0 < c_out; c0 += blk) {
    const int64_t c1 = c0 + blk < c_out ? c0 + blk : c_out;
    for (int64_t c = c0; c < c1; ++c) mf[c] = mq[c] = vq[c] = cqf[c] = vf[c] = 0.0;
    for (int64_t i = 0; i < rows; ++i)
      for (int64_t c = c0; c < c1; ++c) {
        mf[c] += (double)yf[i * ldf + c];
        mq[c] += (double)yq[i * ldq + c];
      }
    for (int64_t c = c0; c < c1; ++c) {
      mf[c] /= (double)rows;
      mq[c] /= (double)rows;
    }
    for (int64_t i = 0; i < rows; ++i)
      for (int64_t c = c0; c < c1; ++c) {
        const double dq = (double)yq[i * ldq + c] - mq[c];
        const double df = (double)yf[i * ldf + c] - mf[c];
        vq[c] += dq * dq;
        cqf[c] += dq * df;
        vf[c] += df * df;
      }
    for (int64_t c = c0; c < c1; ++c) {
      vq[c] /= (double)rows;
      cqf[c] /= (double)rows;
      vf[c] /= (double)rows;
    }
  }
}

/* Eq. 4-5: alpha = Cov / Var, beta = E[Y_full] - alpha E[Y_quant], per channel,
 * fp64, rounded to fp32 at the end.  Where the regression is undetermined
 * (Var(Y_quant) not above var_eps * max(E[Y_quant]^2, 1e-300)) or its slope is
 * exactly zero (which Eq. 10 cannot fold), the channel falls back to the pure
 * shift alpha = 1, beta = E[Y_full] - E[Y_quant]; such channels are counted. */
void orc_solve(const double *moments, int64_t c_out, double var_eps,
               float *alpha, float *beta, int32_t *n_degenerate) {
  const double *mf = moments, *mq = moments + c_out, *vq = moments + 2 * c_out,
               *cqf = moments + 3 * c_out;
  int32_t deg = 0;
  for (int64_t c = 0; c < c_out; ++c) {
    double m2 = mq[c] * mq[c];
    if (m2 < 1e-300) m2 = 1e-300;
    double a, b;
    if (!(vq[c] > var_eps * m2) || cqf[c] == 0.0) {
      a = 1.0;
      b = mf[c] - mq[c];
      ++deg;
    } else {
      a = cqf[c] / vq[c];
      b = mf[c] - a * mq[c];
    }
    alpha[c] = (float)a;
    beta[c] = (float)b;
  }
  if (n_degenerate) *n_degenerate = deg;
}

/* ------------------------------------------------------------------ */
/* Fold into the engine parameters (Sec. 3.4, Eq. 10-11)               */
/* ------------------------------------------------------------------ */

static double sat_round(double v, double lim, int32_t *n_sat) {
  double r = rint(v);
  if (!(r <= lim)) { /* also catches NaN */
    if (r != r) r = 0.0; else r = lim;
    if (n_sat) ++*n_sat;
  } else if (r < -lim) {
    r = -lim;
    if (n_sat) ++*n_sat;
  }
  return r;
}

/* Integer-offset form (Eq. 10-11), per output channel n, in fp64:
 *   mult[n]   = (float)(((alpha * S_x) * S_W[n]) / S_r)            = M'
 *   beta_q    = round(beta / ((alpha * S_x) * S_W[n]))             Eq. 10 offset
 *   bias_q    = round(bias / (S_x * S_W[n]))                       engine's int bias
 *   offset[n] = sat(bias_q + beta_q) - Z_x * colsum[n]
 * sat clamps the sum to +-2^30 so that acc + offset cannot wrap in int32;
 * clamped channels are counted.  alpha/beta NULL mean alpha = 1, beta = 0
 * (Eq. 7-8, plain PTQ).  bias NULL means no bias. */
void orc_fold_int_offset(const float *alpha, const float *beta, const float *sw,
                         const float *bias, const int32_t *colsum, int64_t n,
                         float sx, int32_t zx, float sr, float *mult,
                         int32_t *offset, int32_t *n_saturated) {
  int32_t nsat = 0;
  const double lim = 1073741824.0;
  for (int64_t c = 0; c < n; ++c) {
    const double a = alpha ? (double)alpha[c] : 1.0;
    const double b = beta ? (double)beta[c] : 0.0;
    const double asx = a * (double)sx;
    const double den = asx * (double)sw[c];
    mult[c] = (float)(den / (double)sr);
    const double unit = (double)sx * (double)sw[c];
    double bq = 0.0;
    if (b != 0.0) bq = rint(b / den);
    double biasq = 0.0;
    if (bias) biasq = rint((double)bias[c] / unit);
    const double sum = sat_round(bq + biasq, lim, &nsat);
    offset[c] = (int32_t)sum - zx * colsum[c];
  }
  if (n_saturated) *n_saturated = nsat;
}

/* Floating-bias form (beta kept un-rounded; also the only form possible when
 * the activation scale varies per token), in fp64:
 *   mult[n]   = (float)(((alpha * S_x) * S_W[n]) / S_r)   per-tensor S_x
 *   mult[n]   = (float)((alpha * S_W[n]) / S_r)           per-token (S_x applied per row)
 *   fbias[n]  = (float)((alpha * bias[n] + beta[n]) / S_r)
 *   offset[n] = -Z_x * colsum[n]
 */
void orc_fold_fp_bias(const float *alpha, const float *beta, const float *sw,
                      const float *bias, const int32_t *colsum, int64_t n,
                      int32_t per_token, float sx, int32_t zx, float sr,
                      float *mult, float *fbias, int32_t *offset) {
  for (int64_t c = 0; c < n; ++c) {
    const double a = alpha ? (double)alpha[c] : 1.0;
    const double b = beta ? (double)beta[c] : 0.0;
    double num;
    if (per_token) num = a * (double)sw[c];
    else num = (a * (double)sx) * (double)sw[c];
    mult[c] = (float)(num / (double)sr);
    const double bb = bias ? (double)bias[c] : 0.0;
    fbias[c] = (float)((a * bb + b) / (double)sr);
    offset[c] = -zx * colsum[c];
  }
}

/* ------------------------------------------------------------------ */
/* Folded engine forward (Eq. 10): integer accumulator -> int8 code    */
/* ------------------------------------------------------------------ */

/* Per output element, single fp32 operations in this order, no fused
 * multiply-add:
 *   t = acc + offset[n]                     int32
 *   f = (float)t                            round-to-nearest-even
 *   f = f * sx_row[m]                       only if sx_row != NULL
 *   u = f * mult[n]
 *   u = u + fbias[n]                        only if fbias != NULL
 *   r = clamp(rint(u), qmin - Z_r, qmax - Z_r)   in float
 *   out = (int8)((int32)r + Z_r)
 * out_f32 != NULL additionally receives u (the un-rounded value). */
void orc_folded_forward(const int32_t *acc, int64_t rows, int64_t n,
                        const int32_t *offset, const float *sx_row,
                        const float *mult, const float *fbias, int32_t zr,
                        int32_t qmin, int32_t qmax, int8_t *out, float *out_f32) {
  const float lo = (float)(qmin - zr), hi = (float)(qmax - zr);
  for (int64_t i = 0; i < rows; ++i)
    for (int64_t c = 0; c < n; ++c) {
      const int32_t t = acc[i * n + c] + (offset ? offset[c] : 0);
      float f = (float)t;
      if (sx_row) f = f * sx_row[i];
      float u = f * mult[c];
      if (fbias) u = u + fbias[c];
      if (out_f32) out_f32[i * n + c] = u;
      if (out) {
        float r = rintf(u);
        r = fmaxf(r, lo);
        r = fminf(r, hi);
        out[i * n + c] = (int8_t)((int32_t)r + zr);
      }
    }
}

/* ------------------------------------------------------------------ */
/* Integer-only form of the engine multiplier (Sec. 3.4: after the     */
/* fold the layer needs "no floating-point computation"; the paper      */
/* gives no scheme, this is the usual fixed-point one)                  */
/* ------------------------------------------------------------------ */

/* The real multiplier M' of Eq. 11 (fp64) is replaced by M0 * 2^-shift with
 * M0 a signed 32-bit integer, 2^30 <= |M0| < 2^31, i.e. M' to 31 significant
 * bits:  |M'| = mant * 2^e with mant in [0.5, 1);  M0 = sign * rne(mant * 2^31)
 * (a mantissa that rounds up to 2^31 becomes 2^30 with e + 1);  shift = 31 - e.
 * Representable range 1 <= shift <= 62: a larger multiplier (|M'| >= 2^30)
 * is clamped to +-(2^31 - 1) * 2^-1 and counted, a smaller one (and M' = 0)
 * becomes M0 = 0, shift = 1. */
static void fixed_point_of(double mreal, int32_t *m0, int32_t *shift, int32_t *n_sat) {
  *m0 = 0;
  *shift = 1;
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
    if (n_sat) ++*n_sat;
  }
  *m0 = (int32_t)(mreal < 0.0 ? -q : q);
  *shift = sh;
}

/* Eq. 10-11 with the multiplier in fixed point; offset exactly as in
 * orc_fold_int_offset.  n_saturated counts clamped offsets and clamped
 * multipliers. */
void orc_fold_fixed_point(const float *alpha, const float *beta, const float *sw,
                          const float *bias, const int32_t *colsum, int64_t n,
                          float sx, int32_t zx, float sr, int32_t *m0,
                          int32_t *shift, int32_t *offset, int32_t *n_saturated) {
  int32_t nsat = 0;
  const double lim = 1073741824.0;
  for (int64_t c = 0; c < n; ++c) {
    const double a = alpha ? (double)alpha[c] : 1.0;
    const double b = beta ? (double)beta[c] : 0.0;
    const double asx = a * (double)sx;
    const double den = asx * (double)sw[c];
    fixed_point_of(den / (double)sr, &m0[c], &shift[c], &nsat);
    const double unit = (double)sx * (double)sw[c];
    double bq = 0.0;
    if (b != 0.0) bq = rint(b / den);
    double biasq = 0.0;
    if (bias) biasq = rint((double)bias[c] / unit);
    const double sum = sat_round(bq + biasq, lim, &nsat);
    offset[c] = (int32_t)sum - zx * colsum[c];
  }
  if (n_saturated) *n_saturated = nsat;
}

/* Integer-only epilogue of Eq. 10:
 *   t = acc + offset[n]                               int32
 *   v = floor((t * M0[n] + 2^(shift[n]-1)) / 2^shift[n])   exact in 64 bits:
 *       the nearest integer to t * M0 * 2^-shift, ties towards +infinity
 *   out = clamp(v + Z_r, qmin, qmax) */
void orc_fixed_point_forward(const int32_t *acc, int64_t rows, int64_t n,
                             const int32_t *offset, const int32_t *m0,
                             const int32_t *shift, int32_t zr, int32_t qmin,
                             int32_t qmax, int8_t *out) {
  for (int64_t i = 0; i < rows; ++i)
    for (int64_t c = 0; c < n; ++c) {
      const int64_t t = (int64_t)acc[i * n + c] + (offset ? offset[c] : 0);
      const int sh = shift[c];
      const int64_t prod = t * (int64_t)m0[c] + ((int64_t)1 << (sh - 1));
      /* floor division by 2^sh without relying on the shift of a negative value */
      int64_t v = prod / ((int64_t)1 << sh);
      if (prod % ((int64_t)1 << sh) != 0 && prod < 0) v -= 1;
      v += zr;
      if (v < qmin) v = qmin;
      if (v > qmax) v = qmax;
      out[i * n + c] = (int8_t)v;
    }
}
