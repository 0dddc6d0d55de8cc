/*
 * CPU oracle for the weight-only INT4 linear layer with the CWAC epilogue (the
 * LLM setting of Sec. 4.4: group-wise asymmetric 4-bit weights, group size
 * 128, 16-bit floating-point activations; CWAC of Sec. 3.3 after the layer).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain definition that the GPU library is checked
 * against; nothing in the product path may include, link or call it.  It
 * shares no code, header, table or helper with the HIP sources.
 *
 * What is fixed here (the paper names the setting, not the arithmetic):
 *   - quantizer: Eq. 1-2 with b = 4 on each group of `group` consecutive input
 *     channels of one output channel; the scale is STORED in IEEE binary16 and
 *     the codes are taken against that stored scale;
 *   - dequantized weight: Wd = RN16(s * (c - z)), one binary16 rounding;
 *   - layer output: sum over k of x[m,k] * Wd[n,k], x binary16, exact here
 *     (fp64 accumulation of products that are exact in fp64);
 *   - compensation (Sec. 3.3): alpha * (y + b) + beta, folded (Sec. 3.4) into
 *     a per-channel multiplier alpha and a constant alpha*b + beta.
 *
 * binary16 values travel as their bit patterns (uint16_t); conversions are
 * written out below and pinned against an independent implementation.
 *
 * Parity status: every function is pinned by tests that do not call it to
 * produce their own expectation (numpy's float16, exact rational arithmetic,
 * hand-derived fixtures, numpy matmul).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ */
/* IEEE binary16 <-> binary32                                          */
/* ------------------------------------------------------------------ */

/* binary16 bit pattern -> float (exact). */
float w4o_f16_to_f32(uint16_t h) {
  const uint32_t sign = (uint32_t)(h >> 15) & 1u;
  const int32_t e = (h >> 10) & 0x1f;
  const uint32_t f = h & 0x3ffu;
  float v;
  if (e == 0) {
    v = ldexpf((float)f, -24);               /* zero and subnormals: f * 2^-24 */
  } else if (e == 31) {
    v = f ? NAN : INFINITY;
  } else {
    v = ldexpf((float)(f | 0x400u), e - 25); /* (1.f) * 2^(e-15) */
  }
  return sign ? -v : v;
}

/* float -> nearest binary16, ties to even; overflow to infinity; subnormals kept. */
uint16_t w4o_f32_to_f16(float x) {
  uint32_t u;
  memcpy(&u, &x, 4);
  const uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
  const float a = fabsf(x);
  if (isnan(x)) return (uint16_t)(sign | 0x7e00u);
  if (a >= 65520.0f) return (uint16_t)(sign | 0x7c00u);  /* 65520 = midpoint above the largest finite value, ties to even -> inf */
  if (a < 6.103515625e-05f) {
    /* below 2^-14: multiples of 2^-24; a * 2^24 is exact, rintf rounds half to even */
    const float q = rintf(ldexpf(a, 24));
    return (uint16_t)(sign | (uint16_t)q);   /* q = 1024 is the smallest normal number: same pattern */
  }
  int ex;
  const float m = frexpf(a, &ex);            /* a = m * 2^ex, m in [0.5, 1) */
  /* 11 significant bits: m * 2^11 in [1024, 2048) */
  float q = rintf(ldexpf(m, 11));
  if (q == 2048.0f) {
    q = 1024.0f;
    ex += 1;
  }
  const int32_t e = ex - 1 + 15;             /* value = (q / 1024) * 2^(ex-1) */
  return (uint16_t)(sign | (uint16_t)(e << 10) | ((uint16_t)q & 0x3ffu));
}

/* ------------------------------------------------------------------ */
/* Group-wise asymmetric 4-bit weight quantizer (Sec. 4.4; Eq. 1-2)    */
/* ------------------------------------------------------------------ */

/* For every output channel n and every group g of `group` consecutive input
 * channels: Eq. 2 with b = 4 gives s = (max - min) / 15 in fp32; the stored
 * scale is RN16(s), floored at the smallest normal binary16 number (2^-14) so
 * that Eq. 1 stays defined for a constant group; z = clip(round(-min / s), 0,
 * 15) and c = clip(round(w / s) + z, 0, 15) with the STORED scale, fp32
 * division, round-half-to-even.
 *   w      [n, k]          fp32, row pitch ld
 *   codes  [n, k]          one code per byte, 0..15
 *   scales [n, k / group]  binary16 bit patterns
 *   zeros  [n, k / group]  0..15 */
void w4o_quantize_groupwise(const float *w, int64_t n, int64_t k, int64_t ld, int64_t group,
                            uint8_t *codes, uint16_t *scales, uint8_t *zeros) {
  const int64_t groups = k / group;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < n; ++r) {
    for (int64_t g = 0; g < groups; ++g) {
      const float *wg = w + r * ld + g * group;
      float mn = wg[0], mx = wg[0];
      for (int64_t i = 1; i < group; ++i) {
        if (wg[i] < mn) mn = wg[i];
        if (wg[i] > mx) mx = wg[i];
      }
      uint16_t sb = w4o_f32_to_f16((mx - mn) / 15.0f);
      if (sb < 0x0400u) sb = 0x0400u;        /* zero or subnormal -> 2^-14 */
      if (sb >= 0x7c00u) sb = 0x7bffu;       /* never infinite */
      const float s = w4o_f16_to_f32(sb);
      float zf = rintf(-mn / s);
      if (zf < 0.0f) zf = 0.0f;
      if (zf > 15.0f) zf = 15.0f;
      scales[r * groups + g] = sb;
      zeros[r * groups + g] = (uint8_t)zf;
      for (int64_t i = 0; i < group; ++i) {
        float c = rintf(wg[i] / s) + zf;
        if (c < 0.0f) c = 0.0f;
        if (c > 15.0f) c = 15.0f;
        codes[r * k + g * group + i] = (uint8_t)c;
      }
    }
  }
}

/* Dequantized weights Wd[n, k] = RN16(s[n, g] * (c[n, k] - z[n, g])), returned
 * as floats holding exact binary16 values.  s * (c - z) is an 11-bit by 5-bit
 * product, exact in fp32; the conversion is the single rounding. */
void w4o_dequant(const uint8_t *codes, const uint16_t *scales, const uint8_t *zeros, int64_t n,
                 int64_t k, int64_t group, float *wd) {
  const int64_t groups = k / group;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < n; ++r)
    for (int64_t i = 0; i < k; ++i) {
      const int64_t g = i / group;
      const float s = w4o_f16_to_f32(scales[r * groups + g]);
      const float d = (float)((int32_t)codes[r * k + i] - (int32_t)zeros[r * groups + g]);
      wd[r * k + i] = w4o_f16_to_f32(w4o_f32_to_f16(s * d));
    }
}

/* ------------------------------------------------------------------ */
/* Layer product                                                       */
/* ------------------------------------------------------------------ */

/* acc[i, n] = sum_k x[rows[i], k] * wd[n, k] in fp64 (every product of two
 * binary16 values is exact in fp64; the sum is rounded in fp64 only), and
 * mag[i, n] = sum_k |x * wd| (the scale of the rounding error of any
 * lower-precision summation).  rows == NULL: all m rows in order.
 *   x   [m, k] binary16 bit patterns, row pitch k
 *   wd  [n, k] floats */
void w4o_product(const uint16_t *x, const float *wd, int64_t m, int64_t n, int64_t k,
                 const int64_t *rows, int64_t n_rows, double *acc, double *mag) {
  const int64_t cnt = rows ? n_rows : m;
#pragma omp parallel
  {
    double *xr = (double *)malloc((size_t)k * sizeof(double)); /* one activation row, converted once */
#pragma omp for schedule(static)
    for (int64_t i = 0; i < cnt; ++i) {
      const int64_t r = rows ? rows[i] : i;
      for (int64_t j = 0; j < k; ++j) xr[j] = (double)w4o_f16_to_f32(x[r * k + j]);
      for (int64_t c = 0; c < n; ++c) {
        double s = 0.0, a = 0.0;
        for (int64_t j = 0; j < k; ++j) {
          const double p = xr[j] * (double)wd[c * k + j];
          s += p;
          a += fabs(p);
        }
        acc[i * n + c] = s;
        if (mag) mag[i * n + c] = a;
      }
    }
    free(xr);
  }
}

/* ------------------------------------------------------------------ */
/* Compensation (Sec. 3.3) and its folded form (Sec. 3.4)              */
/* ------------------------------------------------------------------ */

/* Unfolded: the quantized layer's output y = acc + b[n], then alpha[n] * y + beta[n], fp64. */
void w4o_unfolded(const double *acc, int64_t rows, int64_t n, const float *bias,
                  const float *alpha, const float *beta, double *out) {
  for (int64_t i = 0; i < rows; ++i)
    for (int64_t c = 0; c < n; ++c) {
      const double y = acc[i * n + c] + (bias ? (double)bias[c] : 0.0);
      out[i * n + c] = (double)alpha[c] * y + (double)beta[c];
    }
}

/* Fold: the epilogue keeps one multiplier and one constant per output channel,
 * mult[n] = alpha[n] (unchanged) and fbias[n] = RN32(alpha[n] * b[n] + beta[n])
 * evaluated in fp64.  alpha == NULL: no compensation (mult = 1, fbias = b). */
void w4o_fold(const float *alpha, const float *beta, const float *bias, int64_t n, float *mult,
              float *fbias) {
  for (int64_t c = 0; c < n; ++c) {
    const double a = alpha ? (double)alpha[c] : 1.0;
    const double be = beta ? (double)beta[c] : 0.0;
    const double b = bias ? (double)bias[c] : 0.0;
    mult[c] = (float)a;
    fbias[c] = (float)(a * b + be);
  }
}

/* Folded epilogue on the exact product: r = acc * mult[n] + fbias[n] in fp64 -
 * the real number that the engine's fp32 epilogue fl(fl(acc * mult) + fbias)
 * approximates. */
void w4o_folded_real(const double *acc, int64_t rows, int64_t n, const float *mult,
                     const float *fbias, double *out) {
  for (int64_t i = 0; i < rows; ++i)
    for (int64_t c = 0; c < n; ++c)
      out[i * n + c] = acc[i * n + c] * (double)mult[c] + (fbias ? (double)fbias[c] : 0.0);
}

/* The engine's epilogue applied to an fp32 accumulator value, as defined:
 * u = fl32(fl32(acc * mult[n]) + fbias[n]); out32 = u, out16 = RN16(u); a
 * missing multiplier is 1 and a missing constant is +0 (both operations are
 * always carried out, so a result of -0 becomes +0).
 * Used where the accumulator itself is exact in fp32 (integer-valued cases),
 * which makes the whole layer output reproducible bit for bit. */
void w4o_epilogue_f32(const float *acc, int64_t rows, int64_t n, const float *mult,
                      const float *fbias, float *out32, uint16_t *out16) {
  for (int64_t i = 0; i < rows; ++i)
    for (int64_t c = 0; c < n; ++c) {
      volatile float t = acc[i * n + c] * (mult ? mult[c] : 1.0f);
      volatile float u = t + (fbias ? fbias[c] : 0.0f);
      if (out32) out32[i * n + c] = u;
      if (out16) out16[i * n + c] = w4o_f32_to_f16(u);
    }
}
