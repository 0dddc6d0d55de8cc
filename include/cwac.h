/*
 * cwac.h - C ABI of the MI355X (gfx950) library for the QwT-v2 hot path:
 * a W8A8 quantized linear layer whose GEMM epilogue carries the folded
 * channel-wise affine compensation (CWAC), and the calibration pass that fits it.
 *
 * Conventions (all entry points)
 *   - Pointers marked "device" are device addresses owned by the caller and must
 *     stay valid until the work enqueued on `stream` has finished.  Pointers
 *     marked "host" are ordinary host pointers read or written during the call.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 *     device work is enqueued asynchronously on it; no call synchronizes.
 *   - The library allocates no device memory and keeps no state between calls;
 *     scratch space is passed in as an explicit workspace (one entry point,
 *     cwac_calibrate_stats_static, uses a fixed buffer of the library's own instead and says so).
 *     It reads no environment
 *     variable: where several kernels compute the same result, the choice is the
 *     library's unless the caller passes a cwac_tuning to an _ex entry point.
 *   - Errors are reported through the return value; when a call returns an error
 *     nothing has been launched.  No call aborts or throws.
 *   - Matrices are row-major with an explicit leading dimension in ELEMENTS.
 *   - Rounding is round-half-to-even everywhere ("the rounding function" of
 *     Sec. 3.2).  The fp32 epilogue is a fixed sequence of single fp32
 *     operations without fused multiply-add, so integer codes are reproducible
 *     bit for bit.
 */
#ifndef CWAC_H_
#define CWAC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t cwac_status;
enum {
  CWAC_OK = 0,
  CWAC_E_NULL = -1,      /* a required pointer is NULL */
  CWAC_E_SHAPE = -2,     /* a size is out of the supported range */
  CWAC_E_ALIGN = -3,     /* a pointer or leading dimension violates the stated alignment */
  CWAC_E_MODE = -4,      /* inconsistent mode / optional-argument combination */
  CWAC_E_WORKSPACE = -5, /* workspace missing or too small */
  CWAC_E_LAUNCH = -6     /* the HIP runtime refused a launch */
};

/* Static description of an error code (host). */
const char *cwac_status_string(cwac_status s);

/* ------------------------------------------------------------------------- */
/* Quantizers - Sec. 3.2, Eq. 1-2                                             */
/* ------------------------------------------------------------------------- */

/* Workspace bytes needed by cwac_range_f32 for `count` elements. */
size_t cwac_range_workspace(int64_t count);

/* min and max of a contiguous fp32 tensor, the inputs of Eq. 2.
 *   x        device, [count], count >= 1
 *   minmax   device, float[2]: {min, max}
 *   workspace device, at least cwac_range_workspace(count) bytes, 8-byte aligned */
cwac_status cwac_range_f32(const float *x, int64_t count, float *minmax, void *workspace,
                           size_t workspace_bytes, void *stream);

/* Eq. 2 (host arithmetic, fp32): s = (max - min) / (2^bits - 1),
 * z = clip(round(-min / s), 0, 2^bits - 1); s is floored at FLT_MIN * 2^bits so
 * that a constant tensor stays quantizable.  bits in [2, 8].
 *   s, z     host outputs; z is the zero-point of the UNSIGNED code of Eq. 1.
 * For signed 8-bit storage use z - 128 as zero-point (see cwac_quantize_act). */
cwac_status cwac_qparams_from_range(float mn, float mx, int32_t bits, float *s, int32_t *z);

/* Eq. 1 with per-tensor parameters, 8 bit, signed storage:
 * q = clip(round(x / s) + (z + 128), 0, 255) - 128, i.e. the Eq. 1 code shifted
 * by 128 together with its zero-point (s * (q - z) is unchanged).
 *   x   device fp32 [rows, k], leading dimension ldx
 *   q   device int8 [rows, k], leading dimension ldq
 *   s   scale (> 0), z signed zero-point in [-128, 127] */
cwac_status cwac_quantize_act(const float *x, int64_t ldx, int64_t rows, int32_t k, float s,
                              int32_t z, int8_t *q, int64_t ldq, void *stream);

/* Symmetric per-row quantizer (per output channel for weights [N, K]; per token
 * for activations [M, K]): scale[r] = max_k |x[r,k]| / 127 (floored at
 * FLT_MIN * 256), q = clip(round(x / scale[r]), -127, 127), zero-point 0.
 *   x device fp32 [rows, k]; scale device fp32 [rows]; q device int8 [rows, k] */
cwac_status cwac_quantize_rows_sym(const float *x, int64_t ldx, int64_t rows, int32_t k,
                                   float *scale, int8_t *q, int64_t ldq, void *stream);

/* The two quantizers at `bits` bits (2..8) with the codes kept in int8 containers,
 * for the low-bit settings (W4A4, W6A6): the forward kernels are the same, and
 * the output range is set by qmin / qmax of cwac_qparams.
 *   cwac_quantize_act_bits: q = clip(round(x / s) + (z + 2^(bits-1)), 0, 2^bits - 1) - 2^(bits-1),
 *       z the signed zero-point in [-2^(bits-1), 2^(bits-1) - 1] (Eq. 2's z - 2^(bits-1))
 *   cwac_quantize_rows_sym_bits: scale[r] = max_k |x[r,k]| / (2^(bits-1) - 1),
 *       q = clip(round(x / scale[r]), -(2^(bits-1) - 1), 2^(bits-1) - 1)
 * bits = 8 gives exactly the two functions above; other arguments as there. */
cwac_status cwac_quantize_act_bits(const float *x, int64_t ldx, int64_t rows, int32_t k, float s,
                                   int32_t z, int32_t bits, int8_t *q, int64_t ldq, void *stream);
cwac_status cwac_quantize_rows_sym_bits(const float *x, int64_t ldx, int64_t rows, int32_t k,
                                        int32_t bits, float *scale, int8_t *q, int64_t ldq,
                                        void *stream);

/* colsum[n] = sum_k w_q[n, k]: the Z_x W_q term of Eq. 7 is Z_x * colsum[n].
 *   w_q device int8 [n, k]; colsum device int32 [n] */
cwac_status cwac_colsum(const int8_t *w_q, int64_t ldw, int32_t n, int32_t k, int32_t *colsum,
                        void *stream);

/* ------------------------------------------------------------------------- */
/* Calibration statistics and closed-form fit - Sec. 3.3, Eq. 3-5             */
/* ------------------------------------------------------------------------- */

/* The calibration state is a caller-owned DEVICE buffer of cwac_stats_bytes(c_out)
 * bytes, 16-byte aligned.  Layout (stable, so that a caller may copy it out and
 * resume later):
 *   bytes  0..7    int64  n            rows accumulated so far
 *   bytes  8..11   int32  c_out
 *   bytes 12..15   reserved (zero)
 *   bytes 16..19   uint32 internal launch ticket (zero between calls)
 *   bytes 20..63   reserved (zero)
 *   float  pivot_q[c_out], float pivot_f[c_out]   per-channel shift, fixed by the
 *                                                  first row ever accumulated
 *   double sum[5][c_out]   over all rows so far, with dq = y_quant - pivot_q and
 *                          df = y_full - pivot_f:
 *                          sum dq, sum df, sum dq*dq, sum dq*df, sum df*df        */
size_t cwac_stats_bytes(int32_t c_out);

/* Sets the state to "no rows seen".  stats: device. */
cwac_status cwac_stats_reset(void *stats, int32_t c_out, void *stream);

/* Workspace bytes needed by cwac_calibrate_stats for one call with these sizes. */
size_t cwac_calibrate_stats_workspace(int64_t n_rows, int32_t c_out);

/* Accumulates one batch of calibration outputs into the state: for every output
 * channel the sums listed above over the batch's rows (Y_full and Y_quant of
 * Sec. 3.3; rows = calibration samples x tokens).  May be called any number of
 * times; the result does not depend on how the rows are split into batches
 * beyond fp64 summation order, and is bit-reproducible for a given split.
 *   y_full, y_quant  device fp32 [n_rows, c_out], leading dimensions ld_full, ld_quant
 *   n_rows >= 0 (0 is a no-op), 1 <= c_out <= 65536
 *   stats      device, in/out
 *   workspace  device, >= cwac_calibrate_stats_workspace(n_rows, c_out) bytes, 16-byte aligned
 * Fast path when c_out, ld_full, ld_quant are multiples of 4 and both matrices
 * are 16-byte aligned; any other layout takes a slower generic kernel. */
cwac_status cwac_calibrate_stats(const float *y_full, int64_t ld_full, const float *y_quant,
                                 int64_t ld_quant, int64_t n_rows, int32_t c_out, void *stats,
                                 void *workspace, size_t workspace_bytes, void *stream);

/* cwac_calibrate_stats for the FIRST batch of a calibration run: the state is taken
 * as "no rows seen" whatever it holds (it need not have been reset or even
 * initialised), so a run is reset-free: _first for batch 0, cwac_calibrate_stats for
 * the others.  Afterwards the state is exactly what cwac_stats_reset followed by
 * cwac_calibrate_stats leaves.  n_rows >= 1; other arguments and errors as there. */
cwac_status cwac_calibrate_stats_first(const float *y_full, int64_t ld_full, const float *y_quant,
                                       int64_t ld_quant, int64_t n_rows, int32_t c_out, void *stats,
                                       void *workspace, size_t workspace_bytes, void *stream);

/* cwac_calibrate_stats for callers that cannot allocate device memory or carry a workspace -
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc: the partial
 * sums go to a fixed buffer of cwac_static_scratch_bytes() = 8 MiB that is part of the library's
 * device image (every GPU the library runs on holds its own copy until the process ends).  The
 * call allocates nothing, frees nothing and computes exactly what cwac_calibrate_stats computes
 * (same kernels, same split: the state is bit-identical).
 *   - Sizes whose partial sums would not fit return CWAC_E_WORKSPACE (nothing launched); with the
 *     present row split every n_rows and c_out <= 65536 needs at most 7.5 MiB.
 *   - All calls on one GPU share that GPU's buffer: calls that overlap in time on one GPU (two
 *     streams, two threads) race on it.  Serialize them, or use cwac_calibrate_stats with
 *     workspaces of your own.  Nothing needs clearing between calls: a call writes every partial
 *     sum it later reads.
 *   - The first call on a device looks the buffer's address up (hipGetSymbolAddress, not an
 *     allocation); make that first call outside a stream capture.
 * Arguments and the other errors as cwac_calibrate_stats. */
size_t cwac_static_scratch_bytes(void);
cwac_status cwac_calibrate_stats_static(const float *y_full, int64_t ld_full, const float *y_quant,
                                        int64_t ld_quant, int64_t n_rows, int32_t c_out, void *stats,
                                        void *stream);

/* Eq. 4-5 per channel from the state, evaluated in fp64 and rounded to fp32:
 *   alpha = Cov(Y_full, Y_quant) / Var(Y_quant),  beta = E[Y_full] - alpha E[Y_quant].
 * Channels where the regression is undetermined (no rows; Var(Y_quant) not above
 * var_eps * max(E[Y_quant]^2, 1e-300)) or whose slope is exactly 0 (which Eq. 10
 * cannot fold) get alpha = 1, beta = E[Y_full] - E[Y_quant] and are counted.
 *   alpha, beta    device fp32 [c_out]
 *   moments        device fp64 [5][c_out] or NULL: E[Y_full], E[Y_quant],
 *                  Var(Y_quant), Cov(Y_quant, Y_full), Var(Y_full), all with 1/n
 *   n_degenerate   device int32[1] or NULL: number of fallback channels */
cwac_status cwac_solve(const void *stats, int32_t c_out, double var_eps, float *alpha,
                       float *beta, double *moments, int32_t *n_degenerate, void *stream);

/* ------------------------------------------------------------------------- */
/* Fold into the engine parameters - Sec. 3.4, Eq. 7-8 and Eq. 10-11          */
/* ------------------------------------------------------------------------- */

enum { CWAC_EPI_INT_OFFSET = 0, CWAC_EPI_FP_BIAS = 1 };

/* Quantization parameters of one layer in the notation of Sec. 3.4 (host struct).
 * Weights are symmetric per output channel (Z_W = 0), so of the four terms of
 * Eq. 7 only W_q x_q and Z_x W_q remain. */
typedef struct cwac_qparams {
  int32_t mode;          /* CWAC_EPI_INT_OFFSET: beta rounded into the integer offset (Eq. 10);
                            CWAC_EPI_FP_BIAS: beta kept as an fp32 bias added after the multiplier */
  int32_t act_per_token; /* 0: per-tensor (S_x, Z_x) below; 1: per-row scales s_x_row[m], Z_x = 0
                            (requires CWAC_EPI_FP_BIAS) */
  float s_x;             /* S_x (ignored when act_per_token) */
  int32_t z_x;           /* Z_x, signed-storage zero-point */
  float s_r;             /* S_r */
  int32_t z_r;           /* Z_r, signed-storage zero-point */
  int32_t qmin, qmax;    /* output code range, e.g. -128, 127; -128 <= qmin <= qmax <= 127 */
} cwac_qparams;

/* Per-output-channel engine parameters, evaluated in fp64 and rounded once.
 * alpha == NULL and beta == NULL mean alpha = 1, beta = 0: the plain PTQ layer of
 * Eq. 7-8.  With a = alpha[n], unit = S_x * S_W[n]:
 *   INT_OFFSET:  mult[n]   = (float)(((a * S_x) * S_W[n]) / S_r)                       (Eq. 11)
 *                offset[n] = sat(round(beta[n] / ((a * S_x) * S_W[n])) + round(bias[n] / unit))
 *                            - Z_x * colsum[n]                                          (Eq. 10)
 *                sat clamps to +-2^30 so that accumulator + offset cannot wrap.
 *   FP_BIAS:     mult[n]   = as above (per-tensor) or (float)((a * S_W[n]) / S_r) (per-token)
 *                fbias[n]  = (float)((a * bias[n] + beta[n]) / S_r)
 *                offset[n] = -Z_x * colsum[n]
 *   alpha, beta, s_w, bias (nullable = no bias), colsum: device [n_out]
 *   qp           host
 *   mult, offset device [n_out]; fbias device [n_out], required in FP_BIAS mode
 *   n_saturated  device int32[1] or NULL: channels whose offset was clamped
 * With s_r = 1, alpha = beta = NULL and FP_BIAS mode, (mult, fbias, offset) are the
 * dequantization parameters that make the forward return Y_quant of Sec. 3.3. */
cwac_status cwac_fold(const float *alpha, const float *beta, const float *s_w, const float *bias,
                      const int32_t *colsum, int32_t n_out, const cwac_qparams *qp, float *mult,
                      int32_t *offset, float *fbias, int32_t *n_saturated, void *stream);

/* ------------------------------------------------------------------------- */
/* Quantized linear layer with the compensation in its epilogue - Eq. 10      */
/* ------------------------------------------------------------------------- */

enum { CWAC_OUT_INT8 = 0, CWAC_OUT_FP32 = 1, CWAC_OUT_INT32 = 2 };

/* out = epilogue(x_q * w_q^T), int8 x int8 -> int32 on the matrix cores, the
 * accumulators never leaving registers.  Per output element (m, n):
 *   t = acc[m,n] + offset[n]                    int32        (offset NULL: 0)
 *   f = (float)t                                round to nearest even
 *   f = f * s_x_row[m]                          only if s_x_row != NULL
 *   u = f * mult[n]
 *   u = u + fbias[n]                            only if fbias != NULL
 *   CWAC_OUT_INT8:  r = clamp(rint(u), qmin - Z_r, qmax - Z_r) in fp32;
 *                   out = (int8)((int32)r + Z_r)               (Eq. 10, clip of Eq. 1)
 *   CWAC_OUT_FP32:  out = u       (calibration forward: Y_quant, Sec. 3.3)
 *   CWAC_OUT_INT32: out = t       (raw accumulator + offset; mult, fbias, s_x_row unused)
 *
 *   x_q   device int8 [m, k], ldx;  w_q device int8 [n, k], ldw (nn.Linear layout)
 *   m >= 1, n >= 1, 16 <= k <= 32768, k % 16 == 0; x_q, w_q 16-byte aligned,
 *   ldx % 16 == 0, ldw % 16 == 0
 *   qp    host; supplies z_r, qmin, qmax for CWAC_OUT_INT8 (may be NULL otherwise).  When given,
 *         it is checked against the vectors that define the epilogue (CWAC_E_MODE, nothing
 *         launched): act_per_token must equal (s_x_row != NULL), and for CWAC_OUT_INT8 mode
 *         CWAC_EPI_FP_BIAS requires fbias (a fold in that mode always produces one)
 *   mult  device fp32 [n] (required unless CWAC_OUT_INT32)
 *   offset device int32 [n] or NULL; fbias device fp32 [n] or NULL;
 *   s_x_row device fp32 [m] or NULL
 *   out   device, element type per out_kind, [m, n] with leading dimension ldo >= n;
 *         vectorized stores need out aligned to 16 bytes and ldo * sizeof(element)
 *         a multiple of 16, other layouts take an element-wise store path
 *   Any ldx, ldw >= k is legal; the direct-to-LDS kernel keeps per-lane byte offsets in 32 bits
 *   and is only chosen while ldx, ldw <= 2^24 (larger pitches take the generic kernel). */
cwac_status qlinear_cwac_forward(const int8_t *x_q, int64_t ldx, const int8_t *w_q, int64_t ldw,
                                 int64_t m, int32_t n, int32_t k, const cwac_qparams *qp,
                                 const float *mult, const int32_t *offset, const float *fbias,
                                 const float *s_x_row, int32_t out_kind, void *out, int64_t ldo,
                                 void *stream);

/* qlinear_cwac_forward (CWAC_OUT_INT8, integer-offset epilogue of Eq. 10: no fbias, no per-row scales)
 * followed by a 256-entry code table: out = table[r_q + 128].  An activation function between two
 * int8 layers acts on one code at a time (vit_gelu_table builds the GELU's table), so it costs a
 * byte read from LDS in the epilogue of large layers and no pass over the tensor; small layers run
 * the forward and then a lookup pass in place.  Arguments as qlinear_cwac_forward, plus
 *   table  device int8 [256], 4-byte aligned
 *   n % 16 == 0; out 16-byte aligned, ldo % 16 == 0 */
cwac_status qlinear_cwac_forward_table(const int8_t *x_q, int64_t ldx, const int8_t *w_q, int64_t ldw,
                                       int64_t m, int32_t n, int32_t k, const cwac_qparams *qp,
                                       const float *mult, const int32_t *offset, const int8_t *table,
                                       int8_t *out, int64_t ldo, void *stream);

/* Quantized convolutional layer with the compensation in its epilogue: the CWAC
 * module that follows every quantized convolutional layer of a CNN (Sec. 3.3)
 * folds into it as into a linear layer (Sec. 3.4).  Implicit GEMM: row m = (b, oh,
 * ow), column n = output channel, the sum of Eq. 7 runs over the receptive field
 *   acc[m, n] = sum_{i, j, c} x_q[b, oh*stride + i - pad, ow*stride + j - pad, c] * w_q[n, i, j, c]
 * and a position outside the image holds the zero-point Z_x = qp->z_x (the code of
 * the real value 0), so the zero-point term stays Z_x * sum_{i,j,c} w_q[n, i, j, c]:
 * cwac_colsum and cwac_fold apply unchanged to w_q seen as [c_out, kh*kw*c_in].
 * Epilogue and out_kind exactly as in qlinear_cwac_forward (no per-row scales).
 *   x_q   device int8 [batch, h, w, c_in], channels last, contiguous, 16-byte aligned
 *   w_q   device int8 [c_out, kh, kw, c_in], contiguous, 16-byte aligned
 *   c_in % 16 == 0, kh * kw * c_in <= 32768, 1 <= kh, kw, stride <= 16, 0 <= pad < min(kh, kw)
 *   qp    host, required (z_x; z_r, qmin, qmax for CWAC_OUT_INT8); act_per_token must be 0
 *   out   device [batch * oh * ow, c_out] (= channels-last [batch, oh, ow, c_out]), ldo >= c_out,
 *         oh = (h + 2 pad - kh) / stride + 1, ow likewise */
cwac_status qconv2d_cwac_forward(const int8_t *x_q, const int8_t *w_q, int32_t batch, int32_t h,
                                 int32_t w, int32_t c_in, int32_t c_out, int32_t kh, int32_t kw,
                                 int32_t stride, int32_t pad, const cwac_qparams *qp,
                                 const float *mult, const int32_t *offset, const float *fbias,
                                 int32_t out_kind, void *out, int64_t ldo, void *stream);

/* Calibration forward with the statistics taken in its epilogue (Sec. 3.3: the
 * sums of Eq. 4-5 over Y_quant = the CWAC_OUT_FP32 output above and the matching
 * rows of Y_full).  Equivalent to qlinear_cwac_forward(..., CWAC_OUT_FP32, y_quant)
 * followed by cwac_calibrate_stats(y_full, y_quant, ...), except that Y_quant is
 * never written to memory (Y_full is read once: 4 bytes per element instead of
 * 4 written + 8 read); the state differs from the two-call result only by the
 * order of its fp64 additions.
 *   x_q, w_q, mult, offset, fbias, s_x_row   as in qlinear_cwac_forward
 *   y_full     device fp32 [m, n], ld_full; 16-byte aligned, ld_full % 4 == 0
 *   stats      device, in/out (cwac_stats_bytes(n) bytes)
 *   workspace  device, >= cwac_calibrate_fused_workspace(m, n) bytes, 16-byte aligned
 * Shapes: m >= 256, n >= 256, n % 4 == 0, k % 128 == 0; anything else returns
 * CWAC_E_SHAPE and launches nothing (use the two separate calls). */
size_t cwac_calibrate_fused_workspace(int64_t m, int32_t n);
cwac_status qlinear_cwac_calibrate_fused(const int8_t *x_q, int64_t ldx, const int8_t *w_q,
                                         int64_t ldw, int64_t m, int32_t n, int32_t k,
                                         const float *mult, const int32_t *offset,
                                         const float *fbias, const float *s_x_row,
                                         const float *y_full, int64_t ld_full, void *stats,
                                         void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------- */
/* Integer-only engine form (Sec. 3.4: after the fold the layer runs with "no  */
/* floating-point computation"; the paper names no scheme - this is the usual  */
/* fixed-point one)                                                            */
/* ------------------------------------------------------------------------- */

/* cwac_fold in CWAC_EPI_INT_OFFSET form with the multiplier M' of Eq. 11 as
 * m0[n] * 2^-shift[n]: m0 a signed 32-bit integer with 2^30 <= |m0| < 2^31
 * (M' rounded to 31 significant bits; the sign is alpha's), 1 <= shift <= 62.
 * |M'| >= 2^30 is clamped to (2^31 - 1) * 2^-1 and counted in n_saturated with
 * the clamped offsets; |M'| < 2^-32 gives m0 = 0, shift = 1.  offset[n] is
 * cwac_fold's.  qp: host, mode CWAC_EPI_INT_OFFSET, act_per_token 0.
 *   m0, shift, offset   device int32 [n_out];  other arguments as in cwac_fold */
cwac_status cwac_fold_fixed_point(const float *alpha, const float *beta, const float *s_w,
                                  const float *bias, const int32_t *colsum, int32_t n_out,
                                  const cwac_qparams *qp, int32_t *m0, int32_t *shift,
                                  int32_t *offset, int32_t *n_saturated, void *stream);

/* qlinear_cwac_forward with an epilogue that uses no floating point.  Per element:
 *   t = acc[m,n] + offset[n]                                    int32
 *   v = floor((t * m0[n] + 2^(shift[n]-1)) / 2^shift[n])        exact, 64-bit: the nearest
 *                                       integer to t * m0 * 2^-shift, ties towards +infinity
 *   out = (int8)(clamp(v, qmin - Z_r, qmax - Z_r) + Z_r)
 * It differs from the fp32 epilogue by at most one code, and only where the real
 * value lies within that epilogue's own rounding error of a tie.
 *   m0, shift  device int32 [n] as produced by cwac_fold_fixed_point.  Precondition: 1 <= shift[n] <= 62.
 *              They are device data and are not checked: a shift outside that range gives
 *              unspecified codes for its channel (no fault, no error status)
 *   qp         host, required; act_per_token must be 0 and mode CWAC_EPI_INT_OFFSET (CWAC_E_MODE)
 *   out        device int8 [m, n], ldo;  other arguments and limits as in qlinear_cwac_forward */
cwac_status qlinear_cwac_forward_fixed_point(const int8_t *x_q, int64_t ldx, const int8_t *w_q,
                                             int64_t ldw, int64_t m, int32_t n, int32_t k,
                                             const cwac_qparams *qp, const int32_t *m0,
                                             const int32_t *shift, const int32_t *offset,
                                             int8_t *out, int64_t ldo, void *stream);

/* ------------------------------------------------------------------------- */
/* Un-fused comparators (what the fold removes; Sec. 3.3 last sentence,       */
/* Sec. 3.4 first paragraph)                                                  */
/* ------------------------------------------------------------------------- */

/* The same epilogue as a separate pass over int32 accumulators in memory
 * (4 bytes read + 1 written per element instead of none).
 *   acc device int32 [m, n], ldacc; other arguments as in qlinear_cwac_forward;
 *   out_kind CWAC_OUT_INT8 or CWAC_OUT_FP32 */
cwac_status cwac_epilogue_int32(const int32_t *acc, int64_t ldacc, int64_t m, int32_t n,
                                const cwac_qparams *qp, const float *mult, const int32_t *offset,
                                const float *fbias, const float *s_x_row, int32_t out_kind,
                                void *out, int64_t ldo, void *stream);

/* The compensation as a separate module: out = alpha .* y + beta (two fp32
 * roundings), y and out device fp32 [rows, c], may alias. */
cwac_status cwac_apply_unfolded(const float *y, int64_t ldy, int64_t rows, int32_t c,
                                const float *alpha, const float *beta, float *out, int64_t ldo,
                                void *stream);

/* ------------------------------------------------------------------------- */
/* Weight-only INT4 linear layer with the compensation in its epilogue -       */
/* the LLM setting of Sec. 4.4 (group-wise asymmetric 4-bit weights, group     */
/* size 128, 16-bit floating-point activations) with the CWAC of Sec. 3.3      */
/* folded as in Sec. 3.4                                                       */
/* ------------------------------------------------------------------------- */

/* binary16 values cross this interface as their bit patterns (uint16_t). */
enum { CWAC_W4_GROUP = 128 };
enum { CWAC_OUT_FP16 = 3 };

/* Eq. 1-2 with b = 4 on every group of 128 consecutive input channels of one
 * output channel.  s = (max - min) / 15 in fp32, STORED as binary16 (nearest
 * even; floored at 2^-14, capped at 65504); z = clip(round(-min / s), 0, 15) and
 * c = clip(round(w / s) + z, 0, 15) against the stored scale (fp32 division).
 *   w       device fp32 [n, k], ldw;  n >= 1, k % 128 == 0, ldw % 2 == 0, w 8-byte aligned
 *   codes   device uint8 [n, k] (one code per byte, pitch k)
 *   scales  device uint16 [n, k / 128] binary16 bit patterns
 *   zeros   device uint8 [n, k / 128] */
cwac_status cwac_w4_quantize_groupwise(const float *w, int64_t ldw, int32_t n, int32_t k,
                                       uint8_t *codes, uint16_t *scales, uint8_t *zeros,
                                       void *stream);

/* Re-orders the quantized weights into the layout the forward kernel streams
 * (done once per layer, offline in an engine).  An activation re-ordering
 * ("act-order") is a fixed permutation of the k axis applied to the weight
 * columns and activation channels beforehand; here groups are contiguous in k.
 *   packed_w   device, cwac_w4_packed_w_bytes(n, k) = n * k / 2 bytes, 16-byte aligned:
 *              1 KiB blocks indexed [n / 32][k / 64]; in a block, 16 bytes per lane
 *              (lane = 32 * h + n % 32, h = 0, 1); dword j of a lane holds the 8 codes of
 *              input channels 64 * block + 16 * j + 8 * h + e, e = 0..7, code e in bits
 *              4 * p(e) .. 4 * p(e) + 3 with p = (0, 4, 1, 5, 2, 6, 3, 7)
 *   packed_sz  device uint32 [k / 128][n]: scale bits | zero << 16
 *   n % 32 == 0, k % 128 == 0 */
size_t cwac_w4_packed_w_bytes(int32_t n, int32_t k);
cwac_status cwac_w4_pack(const uint8_t *codes, const uint16_t *scales, const uint8_t *zeros,
                         int32_t n, int32_t k, void *packed_w, uint32_t *packed_sz, void *stream);

/* Fold of the compensation into the weight-only layer's epilogue (the analogue of
 * Eq. 10-11 where nothing is requantized): the multiplier is alpha itself and the
 * constant is alpha * bias + beta, evaluated in fp64 and rounded once to fp32.
 * alpha == NULL and beta == NULL: mult = 1, fbias = bias (0 without bias).
 *   alpha, beta, bias (nullable)  device fp32 [n_out];  mult, fbias  device fp32 [n_out] */
cwac_status cwac_fold_weight_only(const float *alpha, const float *beta, const float *bias,
                                  int32_t n_out, float *mult, float *fbias, void *stream);

/* out = epilogue(x * Wd^T) with Wd[n, k] = RN16(s[n, g] * (c[n, k] - z[n, g])), g = k / 128,
 * dequantized in registers (one binary16 rounding), binary16 x binary16 -> fp32 on
 * the matrix cores.  Per output element:
 *   acc = sum_k x[m, k] * Wd[n, k]      fp32 accumulation (order unspecified)
 *   u   = acc * mult[n]                 mult == NULL: multiplier 1
 *   u   = u + fbias[n]                  fbias == NULL: constant +0  (single fp32 operations)
 *   CWAC_OUT_FP16: out = RN16(u);   CWAC_OUT_FP32: out = u  (calibration forward: Y_quant)
 *   x          device binary16 [m, k], ldx; 16-byte aligned, ldx % 8 == 0
 *   packed_w, packed_sz   as produced by cwac_w4_pack
 *   m >= 1, n >= 256, n % 32 == 0, 128 <= k <= 32768, k % 128 == 0
 *   mult, fbias  device fp32 [n] or NULL
 *   out        device [m, n], ldo; 16-byte aligned, ldo * sizeof(element) % 16 == 0
 * Batches of at most 32 rows (decoding steps) take a kernel that streams the packed
 * weights once, 32 output channels per workgroup; batches of up to 256 rows take one such
 * pass per 32 rows while that is estimated to beat a tile's K loop (it does up to 96-256
 * rows, the more the smaller n and the longer k); larger batches tiles of 256 channels x 128
 * tokens while those fit the chip in one round, else x 256 tokens.
 * All compute the sum above; they differ in the order of the fp32 accumulation only. */
cwac_status qlinear_w4a16_cwac_forward(const uint16_t *x, int64_t ldx, const void *packed_w,
                                       const uint32_t *packed_sz, int64_t m, int32_t n, int32_t k,
                                       const float *mult, const float *fbias, int32_t out_kind,
                                       void *out, int64_t ldo, void *stream);

/* ------------------------------------------------------------------------- */
/* Glue of a Transformer block between its W8A8 linear layers                  */
/* ------------------------------------------------------------------------- */
/* Per-layer compensation exists because the rest of the block is non-linear (Sec. 3.2); the
 * paper does not define that rest.  These entry points are the standard pre-norm Vision
 * Transformer block around the linear layers of Sec. 3.4 (int8 codes in, int8 codes out, Eq. 10):
 *   x1 = Q(LN1(h))  r1 = qkv(x1)  a = Q(MHSA(deq(r1)))  r2 = proj(a)  h1 = RN16(h + deq(r2))
 *   x2 = Q(LN2(h1)) r3 = fc1(x2)  g = Q(GELU(deq(r3)))  r4 = fc2(g)   h2 = RN16(h1 + deq(r4))
 * Q(y) = clip(rne(y / s + z), -128, 127) (Eq. 1; evaluated in fp32 as one fused multiply-add with the
 * rounded reciprocal of s), deq(c) = s * (c - z); the residual stream h is IEEE binary16.  All pointers are device pointers owned by the caller; work is enqueued on
 * `stream`; argument errors are returned before anything is launched. */

/* Residual add, layer normalization and quantizer of one row-major [m, c] tensor, any subset
 * that makes sense:
 *   r != NULL:    t = h + s_r * (r - z_r) in fp32; h_out (nullable) receives RN16(t), and the
 *                 layer norm reads that rounded value
 *   x_q != NULL:  x_q = Q(LN(t; gamma, beta, eps); s_x, z_x); LN over the c channels of a row,
 *                 biased variance, fp32, two passes over the register-resident row
 *   h, h_out   binary16 [m, c], pitches ldh, ldho (elements); 16-byte aligned, pitch % 8 == 0
 *   r, x_q     int8 [m, c], pitches ldr, ldxq; 8-byte aligned, pitch % 8 == 0
 *   gamma, beta  fp32 [c], 16-byte aligned (required with x_q)
 *   8 <= c <= 2048, c % 8 == 0, m >= 1; s_x > 0
 * Errors: CWAC_E_NULL (h missing, or neither r nor x_q), CWAC_E_MODE (h_out without r, s_x <= 0),
 * CWAC_E_SHAPE, CWAC_E_ALIGN. */
cwac_status vit_residual_ln_quant(const uint16_t *h, int64_t ldh, const int8_t *r, int64_t ldr,
                                  float s_r, int32_t z_r, uint16_t *h_out, int64_t ldho,
                                  const float *gamma, const float *beta, float eps, float s_x,
                                  int32_t z_x, int8_t *x_q, int64_t ldxq, int64_t m, int32_t c,
                                  void *stream);

/* The GELU between fc1 and fc2 acts on one int8 code at a time, so it is a table:
 * table[code + 128] = Q(GELU(s_in * (code - z_in)); s_out, z_out), GELU(x) = x * Phi(x) with the
 * exact normal distribution function, evaluated in fp64.  table: device int8 [256]. */
cwac_status vit_gelu_table(float s_in, int32_t z_in, float s_out, int32_t z_out, int8_t *table,
                           void *stream);

/* out[i, j] = table[in[i, j] + 128] for an int8 [m, n] tensor (n % 16 == 0; both pitches % 16 == 0,
 * both base pointers 16-byte aligned; in and out may be the same buffer). */
cwac_status vit_table_lookup(const int8_t *in, int64_t ld_in, const int8_t *table, int8_t *out,
                             int64_t ld_out, int64_t m, int32_t n, void *stream);

/* Multi-head self-attention on the requantized output of the qkv layer, head width d = head_dim (64 or 32):
 *   r_qkv  int8 [batch * tokens, 3 * c], c = d * heads, row = (q | k | v), head h in columns
 *          [d h, d h + d) of each third; pitch ld (ld % 8 == 0, base 8-byte aligned);
 *          quantization parameters (s, z) of the whole tensor
 *   a_q    int8 [batch * tokens, c] = Q(softmax(q k^T / sqrt(d)) v; s_a, z_a) per image and head;
 *          pitch lda (lda % 16 == 0, base 16-byte aligned)
 *   1 <= tokens <= 4096 (up to 224 tokens one workgroup holds a head's keys and values; beyond, the keys
 *   pass through it in chunks of 224 with a running softmax), heads <= 64
 *   bias   NULL, or device binary16 [heads, tokens, ldb] added to the logits q k^T / sqrt(d) before the
 *          softmax (the relative position bias - or a mask of large negative values - of a windowed
 *          model; shared by all images); ldb % 4 == 0 and ldb >= tokens rounded up to a multiple of 32
 *          (the padding is read, not used); 8-byte aligned.  Every entry must be FINITE: mask with a
 *          large negative value such as -100, not with -inf (a query whose leading keys are all
 *          -inf would get NaN weights)
 * "image" is whatever attends within itself: an image of a ViT, a window of a windowed model.
 * Scores are exact (integers in fp32 accumulators), the softmax is fp32, the weights meet the
 * values as binary16 (relative error 2^-11 per term), accumulation in fp32. */
cwac_status vit_attention_int8(const int8_t *r_qkv, int64_t ld, float s, int32_t z, int32_t batch,
                               int32_t tokens, int32_t heads, int32_t head_dim, const uint16_t *bias,
                               int64_t ldb, float s_a, int32_t z_a, int8_t *a_q, int64_t lda, void *stream);

/* One whole block: the chain above in eight launches (the GELU table rides in fc1's epilogue where
 * qlinear_cwac_forward_table fuses it) on `stream`, from the residual stream h
 * [batch * tokens, c] (c = head_dim * heads, pitch c) to h_out (same shape; may be h itself).  Linear
 * layer i (0 qkv [3c, c], 1 proj [c, c], 2 fc1 [hidden, c], 3 fc2 [c, hidden]; weights int8
 * row-major [n, k], pitch k) runs qlinear_cwac_forward in CWAC_EPI_INT_OFFSET form with per-tensor
 * activations: mult / offset are cwac_fold's, (s_x, z_x) its input quantizer - which is the
 * quantizer of the glue step that produces its input - and (s_r, z_r) its requantization.
 * gelu_table is vit_gelu_table(layer[2].s_r, layer[2].z_r, layer[3].s_x, layer[3].z_x).
 * workspace: device, vit_block_workspace(...) bytes, 16-byte aligned; after the call it holds, in
 * this order: x2 = Q(LN2(h1)) [m, c], r1 (qkv output) [m, 3c], r4 (fc2 output) [m, c],
 * g (GELU codes) [m, hidden] - exposed so that a caller can check every stage.
 * Errors: those of the single calls; CWAC_E_WORKSPACE if workspace_bytes is too small. */
typedef struct vit_block_layer {
  const int8_t *w_q;
  const float *mult;
  const int32_t *offset;
  float s_x;
  int32_t z_x;
  float s_r;
  int32_t z_r;
} vit_block_layer;

typedef struct vit_block_params {
  int32_t batch, tokens, heads, hidden;
  float eps;
  const float *ln1_gamma, *ln1_beta, *ln2_gamma, *ln2_beta;
  vit_block_layer layer[4];
  const int8_t *gelu_table;
  int32_t head_dim; /* 64 or 32; 0 means 64 */
  const uint16_t *attn_bias; /* vit_attention_int8's bias, or NULL */
  int64_t attn_bias_ld;
} vit_block_params;

/* Bytes of workspace of a block; sized for head width 64 (a block of 32-wide heads needs less). */
size_t vit_block_workspace(int32_t batch, int32_t tokens, int32_t heads, int32_t hidden);
/* A stack of n_blocks blocks of one shape (blocks[b].batch / tokens / heads / hidden all equal;
 * CWAC_E_SHAPE otherwise), block b + 1 reading what block b wrote.  Between two blocks the last residual
 * add of one and the LN1 + quantizer of the next are one pass over the stream.  The same workspace
 * (vit_block_workspace bytes) serves every block; h_out may be h. */
cwac_status vit_encoder_w8a8_forward(const vit_block_params *blocks /* host, [n_blocks] */, int32_t n_blocks,
                                     const uint16_t *h, uint16_t *h_out, void *workspace,
                                     size_t workspace_bytes, void *stream);
cwac_status vit_block_w8a8_forward(const vit_block_params *params /* host */, const uint16_t *h,
                                   uint16_t *h_out, void *workspace, size_t workspace_bytes,
                                   void *stream);

/* ------------------------------------------------------------------------- */
/* Kernel choice override (_ex entry points)                                  */
/* ------------------------------------------------------------------------- */
/* Several kernels and tile shapes stand behind each forward entry point; all compute the values
 * the entry point documents (the int8 layer: bit for bit; the weight-only layer: up to the order
 * of its fp32 sums) and the library picks by problem size.  An _ex entry point is the plain one
 * with a trailing `tuning` (host struct, read during the call; NULL = the plain call) that
 * overrides the pick - for tests that must reach every kernel and for tuning sweeps.  A field
 * left 0 keeps the library's choice for that aspect; a value outside the lists below returns
 * CWAC_E_MODE; a forced shape whose constraints the problem does not meet falls back as stated. */
enum {
  CWAC_KERNEL_AUTO = 0,
  CWAC_KERNEL_DIRECT_LDS = 1,    /* the direct-to-LDS kernel wherever its constraints hold (m >= 256,
                                    n >= 64, k % 64 == 0, ldx and ldw <= 2^24; convolution: c_in % 64
                                    == 0, image below 2 GiB); otherwise the automatic choice */
  CWAC_KERNEL_GENERIC_64 = 64,   /* the register-staged kernel with 64 x 64, 128 x 128 or 256 x 256 */
  CWAC_KERNEL_GENERIC_128 = 128, /* output tiles (any shape)                                       */
  CWAC_KERNEL_GENERIC_256 = 256
};
enum {
  CWAC_SHAPE_AUTO = 0,
  CWAC_SHAPE_256_8W = 1,      /* 256 tokens x 256 channels, eight wavefronts, K steps of 128 (k % 128 == 0) */
  CWAC_SHAPE_256_4W_K128 = 2, /* the same tile, four wavefronts, K steps of 128, two stages */
  CWAC_SHAPE_256_4W_K64 = 3,  /* four wavefronts, K steps of 64, four stages */
  CWAC_SHAPE_128_PAIR = 4,    /* 128 tokens x 256 channels, two workgroups per compute unit */
  CWAC_SHAPE_128_128 = 5,     /* 128 x 128, four wavefronts of 64 x 64 */
  CWAC_SHAPE_256_PERSIST = 6  /* CWAC_SHAPE_256_8W's tile on persistent workgroups, one per compute unit, the
                                 next tile's first loads in flight under a tile's epilogue (linear layers, every
                                 epilogue but the fused statistics; convolutions take CWAC_SHAPE_256_8W) */
};
typedef struct cwac_tuning {
  int32_t kernel;         /* CWAC_KERNEL_*: int8 linear / convolution / table / fixed-point forwards */
  int32_t shape;          /* CWAC_SHAPE_*: tile shape of the direct-to-LDS kernel for n >= 256 (used when that
                             kernel runs; k % 128 != 0 always takes CWAC_SHAPE_128_PAIR or _128_128) */
  int32_t stats_waves;    /* qlinear_cwac_calibrate_fused_ex: 0 (= 8) | 8 | 4 wavefronts per tile */
  int32_t w4_tile;        /* qlinear_w4a16_cwac_forward_ex: 0 | 256 | 128: the tiled kernel with that many
                             tokens per tile (256 channels wide) at every batch size; 512: its tile of 512
                             channels x 128 tokens (needs n >= 512, else CWAC_E_MODE) */
  int32_t w4_small_waves; /* ... its weight-streaming kernel (small batches): 0 | 4 | 8 wavefronts per workgroup */
  int32_t persist_workgroups; /* CWAC_SHAPE_256_PERSIST: 0 = one workgroup per compute unit; n > 0 = at most n
                                 (each then walks more tiles; leaves compute units to concurrent work) */
  int32_t w4_small_depth; /* ... and its ring depth: 0 | 2 | 3 | 4 groups of 128 input channels in flight per
                             wavefront (a depth whose rings do not fit the LDS is lowered to one that does) */
  int32_t persist_loaders; /* CWAC_SHAPE_256_PERSIST: how many of the eight wavefronts issue the panel loads:
                              0 (= 4 from k = 4096, else 8) | 4 | 8 */
} cwac_tuning;

/* Which kernel qlinear_cwac_forward(_ex) would run for these sizes and this tuning (host
 * arithmetic only; nothing is launched, no pointer is involved): CWAC_KERNEL_DIRECT_LDS or
 * CWAC_KERNEL_GENERIC_64 / _128 / _256; a negative cwac_status for sizes the forward rejects. */
int32_t cwac_forward_kernel_for(int64_t m, int32_t n, int32_t k, int64_t ldx, int64_t ldw,
                                int32_t out_kind, const cwac_tuning *tuning);

cwac_status qlinear_cwac_forward_ex(const int8_t *x_q, int64_t ldx, const int8_t *w_q, int64_t ldw,
                                    int64_t m, int32_t n, int32_t k, const cwac_qparams *qp,
                                    const float *mult, const int32_t *offset, const float *fbias,
                                    const float *s_x_row, int32_t out_kind, void *out, int64_t ldo,
                                    const cwac_tuning *tuning, void *stream);
cwac_status qlinear_cwac_forward_table_ex(const int8_t *x_q, int64_t ldx, const int8_t *w_q, int64_t ldw,
                                          int64_t m, int32_t n, int32_t k, const cwac_qparams *qp,
                                          const float *mult, const int32_t *offset, const int8_t *table,
                                          int8_t *out, int64_t ldo, const cwac_tuning *tuning, void *stream);
cwac_status qconv2d_cwac_forward_ex(const int8_t *x_q, const int8_t *w_q, int32_t batch, int32_t h,
                                    int32_t w, int32_t c_in, int32_t c_out, int32_t kh, int32_t kw,
                                    int32_t stride, int32_t pad, const cwac_qparams *qp,
                                    const float *mult, const int32_t *offset, const float *fbias,
                                    int32_t out_kind, void *out, int64_t ldo, const cwac_tuning *tuning,
                                    void *stream);
cwac_status qlinear_cwac_calibrate_fused_ex(const int8_t *x_q, int64_t ldx, const int8_t *w_q,
                                            int64_t ldw, int64_t m, int32_t n, int32_t k,
                                            const float *mult, const int32_t *offset,
                                            const float *fbias, const float *s_x_row,
                                            const float *y_full, int64_t ld_full, void *stats,
                                            void *workspace, size_t workspace_bytes,
                                            const cwac_tuning *tuning, void *stream);
cwac_status qlinear_cwac_forward_fixed_point_ex(const int8_t *x_q, int64_t ldx, const int8_t *w_q,
                                                int64_t ldw, int64_t m, int32_t n, int32_t k,
                                                const cwac_qparams *qp, const int32_t *m0,
                                                const int32_t *shift, const int32_t *offset,
                                                int8_t *out, int64_t ldo, const cwac_tuning *tuning,
                                                void *stream);
cwac_status qlinear_w4a16_cwac_forward_ex(const uint16_t *x, int64_t ldx, const void *packed_w,
                                          const uint32_t *packed_sz, int64_t m, int32_t n, int32_t k,
                                          const float *mult, const float *fbias, int32_t out_kind,
                                          void *out, int64_t ldo, const cwac_tuning *tuning, void *stream);

/* ------------------------------------------------------------------------- */
/* Diagnostic (measurement aid, not a step of the method)                     */
/* ------------------------------------------------------------------------- */

/* Runs the forward kernel's matrix-core pattern (per wavefront 4 x 4 int8 MFMA
 * 32x32x32 tiles, 256 accumulators per lane) with register-resident operands
 * and no memory traffic, `iters` times: 2 * 32768 * 16 * iters * 4 * workgroups
 * int8 operations.  Timed by the caller, it gives the rate the matrix cores
 * sustain on this device for operands of the given CONTENT (the clock a device
 * holds under its power limit depends on the operands' switching activity).
 *   operands  device, 16 KiB (1024 x 16 bytes): the first 8 KiB feed the weight
 *             fragments, the second 8 KiB the activation fragments
 *   1 <= iters <= 2^24, 1 <= workgroups <= 2^20 (256 threads each)
 *   sink      device int32[1]; written only if a checksum takes one particular value */
cwac_status cwac_mfma_probe(const int32_t *operands, int32_t iters, int32_t workgroups,
                            int32_t *sink, void *stream);

/* Diagnostic: a read-only stream over `bytes` of device memory (16-byte non-temporal loads at a
 * grid stride, 8 in flight per lane, `workgroups` x 256 threads), timed by the caller: the rate
 * at which this device delivers a plain stream, beside which the statistics pass (8 bytes read
 * per row and channel) is reported.
 *   src    device, 16-byte aligned, bytes >= 16 (a multiple of 16 is read)
 *   sink   device int32[1]; written only if a checksum takes one particular value */
cwac_status cwac_hbm_read_probe(const void *src, size_t bytes, int32_t workgroups, int32_t *sink,
                                void *stream);

/* The same for the binary16 matrix cores, the weight-only layer's (per wavefront 4 x 4 MFMA
 * 32x32x16 tiles, fp32 accumulators): 2 * 16384 * 16 * iters * 4 * workgroups floating-point
 * operations.
 *   operands  device, 16 KiB of binary16 values (1024 x 16 bytes), 16-byte aligned: first half the
 *             weight fragments, second half the activation fragments
 *   iters, workgroups, sink: as above */
cwac_status cwac_mfma_probe_f16(const uint16_t *operands, int32_t iters, int32_t workgroups,
                                int32_t *sink, void *stream);

/* Diagnostic as well: the K loop of the forward's 256 x 256 tile (512 threads, 128 KiB of
 * LDS, one workgroup per compute unit; per stage 256 MFMAs of 32x32x32 per workgroup =
 * 2 * 32768 * 256 int8 operations) with its ingredients added one at a time -
 *   mode 0  the MFMAs alone, fragments in registers
 *   mode 1  + the six 16-byte LDS fragment reads per wavefront and k-step
 *   mode 2  + the wait and barrier that end a stage
 *   mode 3  + the panel stream: eight direct-to-LDS loads of 1 KiB per wavefront and stage
 *   mode 4  the same stream issued by wavefronts 0-3 only (sixteen loads each, one loading wavefront per SIMD)
 * - timed by the caller: what each ingredient costs of the matrix cores' rate.
 *   operands  device, 16 KiB as for cwac_mfma_probe (they also fill the LDS panels)
 *   panels    device, 64 KiB, 16-byte aligned: the source of mode 3's loads (read by every workgroup)
 *   1 <= stages <= 2^24, 1 <= workgroups <= 2^20; mode outside 0..4: CWAC_E_MODE */
cwac_status cwac_kloop_probe(const int32_t *operands, const int8_t *panels, int32_t mode, int32_t stages,
                             int32_t workgroups, int32_t *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CWAC_H_ */
