// Quantized linear layer with the CWAC epilogue (Sec. 3.4, Eq. 10) for gfx950.
//
// acc = x_q * w_q^T on the int8 matrix cores (v_mfma_i32_32x32x32_i8), A/B
// panels staged through LDS, the int32 accumulators kept in registers, and the
// whole epilogue (offset add, int->fp32, multiplier, optional fp32 bias, round,
// clamp, pack) applied to them in registers, so that compensation costs no
// extra pass over memory.
//
// Operand orientation.  The MFMA computes D[i][j] = sum_k A[i][k] B[j][k] with a
// lane owning one column j and, per 32x32 tile, 4 groups of 4 consecutive rows i.
// Feeding the WEIGHT tile as A (i <-> output channel n) and the ACTIVATION tile
// as B (j <-> token row m) makes every lane hold 4 consecutive output channels
// of one token, which is exactly a packed 4 x int8 (or one float4) store into
// the row-major [M, N] output.
#include "qlinear_common.h"

namespace cwac {
namespace {

// LDS tile: ROWS x BK bytes, 16-byte chunks XOR-swizzled inside each row so that
// the 16 lanes that read the same chunk index of 16 consecutive rows (one MFMA
// operand fetch) and the 8 lanes that write one row hit distinct banks.
template <int BK>
__device__ __forceinline__ int lds_off(int row, int chunk) {
  constexpr int CPR = BK / 16;  // chunks per row
  return row * BK + (((chunk ^ (row >> 1)) & (CPR - 1)) << 4);
}

template <int BM, int BN, int BK, int WGM, int WGN>
struct Tile {
  static constexpr int NT = 64 * WGM * WGN;
  static constexpr int WM = BM / WGM, WN = BN / WGN;
  static constexpr int TM = WM / 32, TN = WN / 32;
  static constexpr int CPR = BK / 16;
  static constexpr int XCH = BM * CPR / NT;  // 16-byte chunks per thread, activation tile
  static constexpr int WCH = BN * CPR / NT;  // 16-byte chunks per thread, weight tile
  static_assert(BM % (32 * WGM) == 0 && BN % (32 * WGN) == 0, "wave tile must be whole MFMA tiles");
  static_assert((BM * CPR) % NT == 0 && (BN * CPR) % NT == 0, "tile must split evenly over threads");
  static_assert(BK % 32 == 0 && CPR >= 2 && (CPR & (CPR - 1)) == 0, "BK must be a power of two >= 32");
};

// CONV: the activation operand is gathered from an image tensor (implicit GEMM): the CWAC module
// that follows a quantized convolutional layer (Sec. 3.3) folds into it exactly as into a linear
// layer (Sec. 3.4), the sum of Eq. 7 running over the receptive field.
template <int BM, int BN, int BK, int WGM, int WGN, int OUT_KIND, bool INT_ONLY, bool CONV>
__global__ __launch_bounds__(64 * WGM * WGN) void qlinear_kernel(const FwdParams p) {
  using T = Tile<BM, BN, BK, WGM, WGN>;
  constexpr int NT = T::NT, TM = T::TM, TN = T::TN, CPR = T::CPR;

  __shared__ __attribute__((aligned(16))) int8_t lds_x[BM * BK];
  __shared__ __attribute__((aligned(16))) int8_t lds_w[BN * BK];

  int tile_m, tile_n;
  tile_of_block(blockIdx.x, p.tiles_m, p.tiles_n, tile_m, tile_n);
  const int64_t bm0 = (int64_t)tile_m * BM;
  const int bn0 = tile_n * BN;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave % WGM, wave_n = wave / WGM;
  const int l32 = lane & 31, half = lane >> 5;

  // ---- global -> register staging: thread owns chunk (row, c) = (q / CPR, q % CPR), q = tid + i*NT
  const int ld_c = tid % CPR;
  const int ld_r = tid / CPR;
  constexpr int RSTEP = NT / CPR;  // rows between a thread's successive chunks
  const int8_t *xg[T::XCH];
  const int8_t *wg[T::WCH];
  int ih0[T::XCH], iw0[T::XCH];  // CONV: top-left input position of the row's receptive field
#pragma unroll
  for (int i = 0; i < T::XCH; ++i) {
    int64_t r = bm0 + ld_r + i * RSTEP;
    if (r > p.m - 1) r = p.m - 1;  // rows past the edge re-read the last row; never stored
    if (CONV) {
      const int per = p.cv_oh * p.cv_ow;
      const int64_t b = r / per;
      const int rem = (int)(r - b * per);
      const int y = rem / p.cv_ow, x = rem - y * p.cv_ow;
      ih0[i] = y * p.cv_stride - p.cv_pad;
      iw0[i] = x * p.cv_stride - p.cv_pad;
      xg[i] = p.x + b * ((int64_t)p.cv_h * p.cv_w * p.cv_cin);
    } else {
      xg[i] = p.x + r * p.ldx + ld_c * 16;
    }
  }
#pragma unroll
  for (int i = 0; i < T::WCH; ++i) {
    int r = bn0 + ld_r + i * RSTEP;
    if (r > p.n - 1) r = p.n - 1;
    wg[i] = p.w + (int64_t)r * p.ldw + ld_c * 16;
  }
  v4i xr[T::XCH], wr[T::WCH];

  auto load_stage = [&](int k0) {
    const bool in_k = (k0 + ld_c * 16) < p.k;  // k % 16 == 0: a chunk is all in or all out
    if (CONV) {
      // c_in % 16 == 0: the 16 channels of a chunk belong to one filter tap
      const int kc = k0 + ld_c * 16;
      const int tap = kc / p.cv_cin, c = kc - tap * p.cv_cin;
      const int kh = tap / p.cv_kw, kw = tap - kh * p.cv_kw;
      const v4i pad = {p.cv_pad4, p.cv_pad4, p.cv_pad4, p.cv_pad4};
#pragma unroll
      for (int i = 0; i < T::XCH; ++i) {
        const int ih = ih0[i] + kh, iw = iw0[i] + kw;
        const bool inside = in_k && (unsigned)ih < (unsigned)p.cv_h && (unsigned)iw < (unsigned)p.cv_w;
        const int64_t pos = ((int64_t)ih * p.cv_w + iw) * p.cv_cin + c;
        xr[i] = inside ? *reinterpret_cast<const v4i *>(xg[i] + pos) : pad;  // beyond k: weights are 0
      }
    } else {
#pragma unroll
      for (int i = 0; i < T::XCH; ++i)
        xr[i] = in_k ? *reinterpret_cast<const v4i *>(xg[i] + k0) : v4i{0, 0, 0, 0};
    }
#pragma unroll
    for (int i = 0; i < T::WCH; ++i)
      wr[i] = in_k ? *reinterpret_cast<const v4i *>(wg[i] + k0) : v4i{0, 0, 0, 0};
  };
  auto store_stage = [&]() {
#pragma unroll
    for (int i = 0; i < T::XCH; ++i)
      *reinterpret_cast<v4i *>(lds_x + lds_off<BK>(ld_r + i * RSTEP, ld_c)) = xr[i];
#pragma unroll
    for (int i = 0; i < T::WCH; ++i)
      *reinterpret_cast<v4i *>(lds_w + lds_off<BK>(ld_r + i * RSTEP, ld_c)) = wr[i];
  };

  v16i acc[TN][TM];
#pragma unroll
  for (int a = 0; a < TN; ++a)
#pragma unroll
    for (int b = 0; b < TM; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][b][e] = 0;

  const int xrow0 = wave_m * T::WM + l32;
  const int wrow0 = wave_n * T::WN + l32;

  const int kt_count = (p.k + BK - 1) / BK;
  load_stage(0);
  for (int kt = 0; kt < kt_count; ++kt) {
    store_stage();
    __syncthreads();
    if (kt + 1 < kt_count) load_stage((kt + 1) * BK);  // in flight while this stage is multiplied
#pragma unroll
    for (int kk = 0; kk < BK / 32; ++kk) {
      const int chunk = 2 * kk + half;
      v4i fw[TN], fx[TM];
#pragma unroll
      for (int a = 0; a < TN; ++a)
        fw[a] = *reinterpret_cast<const v4i *>(lds_w + lds_off<BK>(wrow0 + a * 32, chunk));
#pragma unroll
      for (int b = 0; b < TM; ++b)
        fx[b] = *reinterpret_cast<const v4i *>(lds_x + lds_off<BK>(xrow0 + b * 32, chunk));
#pragma unroll
      for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[a], fx[b], acc[a][b], 0, 0, 0);
    }
    __syncthreads();
  }

  epilogue_tiles<TM, TN, OUT_KIND, INT_ONLY>(p, acc, bm0 + wave_m * T::WM, bn0 + wave_n * T::WN, l32, half,
                                             p.vec_store);
}

template <int BM, int BN, int BK, int WGM, int WGN, bool CONV = false>
cwac_status launch_tile(FwdParams p, int out_kind, bool int_only, hipStream_t st) {
  p.tiles_m = (int)ceil_div(p.m, BM);
  p.tiles_n = (int)ceil_div(p.n, BN);
  const int64_t blocks = (int64_t)p.tiles_m * p.tiles_n;
  if (blocks > 0x7fffffff) return CWAC_E_SHAPE;
  const dim3 grid((unsigned)blocks), block(64 * WGM * WGN);
  if (out_kind == kOutFixed) {
    if (CONV) return CWAC_E_MODE;
    qlinear_kernel<BM, BN, BK, WGM, WGN, kOutFixed, true, false><<<grid, block, 0, st>>>(p);
  } else if (out_kind == CWAC_OUT_INT8) {
    if (int_only)
      qlinear_kernel<BM, BN, BK, WGM, WGN, CWAC_OUT_INT8, true, CONV><<<grid, block, 0, st>>>(p);
    else
      qlinear_kernel<BM, BN, BK, WGM, WGN, CWAC_OUT_INT8, false, CONV><<<grid, block, 0, st>>>(p);
  } else if (out_kind == CWAC_OUT_FP32) {
    qlinear_kernel<BM, BN, BK, WGM, WGN, CWAC_OUT_FP32, false, CONV><<<grid, block, 0, st>>>(p);
  } else {
    qlinear_kernel<BM, BN, BK, WGM, WGN, CWAC_OUT_INT32, false, CONV><<<grid, block, 0, st>>>(p);
  }
  return launch_status();
}

// Y_quant of token row 0 for every channel (the fp32 output mode's arithmetic on one row): the
// pivot of a calibration state's first batch.  One wavefront per channel at a time, 16 bytes of
// K per lane and step; does nothing when the state already holds rows.
__global__ __launch_bounds__(256) void row0_kernel(const FwdParams p, float *__restrict__ yq_row0) {
  const StatsView sv = stats_view(const_cast<void *>(p.stats), p.n);
  if (*sv.n != 0) return;
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
  const int waves = gridDim.x * (blockDim.x / kWave);
  for (int ch = wave; ch < p.n; ch += waves) {
    const int8_t *w = p.w + (int64_t)ch * p.ldw;
    int acc = 0;
    for (int k0 = lane * 16; k0 < p.k; k0 += kWave * 16) {
      const v4i xv = *reinterpret_cast<const v4i *>(p.x + k0);
      const v4i wv = *reinterpret_cast<const v4i *>(w + k0);
#pragma unroll
      for (int i = 0; i < 4; ++i) acc = __builtin_amdgcn_sdot4(xv[i], wv[i], acc, false);
    }
    acc = wave_sum(acc);
    if (lane == 0) {
      float f = (float)(acc + (p.offset ? p.offset[ch] : 0));
      if (p.sx_row) f = f * p.sx_row[0];
      float v = f * p.mult[ch];
      if (p.fbias) v = v + p.fbias[ch];
      yq_row0[ch] = v;
    }
  }
}

}  // namespace
}  // namespace cwac

using namespace cwac;

// Kernel and tile choice shared by the forward entry points: CWAC_KERNEL_DIRECT_LDS or the generic
// kernel's tile (CWAC_KERNEL_GENERIC_*).  Host arithmetic on sizes only.
static int choose_forward(int64_t m, int n, int k, int64_t ldx, int64_t ldw, int out_kind, const Tune &tune) {
  // Tile choice: the largest tile that still gives the 256 compute units at least
  // two workgroups each; small problems fall back to small tiles.
  const int64_t t256 = ceil_div(m, 256) * ceil_div(n, 256);
  const int64_t t128 = ceil_div(m, 128) * ceil_div(n, 128);
  int tile = t256 >= 512 ? 256 : (t128 >= 512 ? 128 : 64);
  // narrow layers: a tile much wider than the layer would multiply mostly padding
  if (n <= 160 && tile > 128) tile = 128;
  if (n <= 80 && tile > 64) tile = 64;
  // the large-problem kernel: K a multiple of 128, or of 64 (then only its 128-token tile, which
  // steps K by 64); 64 <= N < 256: its 256 x 128 or 256 x 64 tile; pitches its 32-bit lane offsets hold
  const bool fast_ok = m >= kFastTile && n >= 64 && (k % 64) == 0 && fast_pitch_ok(ldx, ldw);
  // it wants most compute units busy: 160 full tiles, or 256 half tiles
  const int out_bytes = (out_kind == CWAC_OUT_INT8 || out_kind == kOutFixed) ? 1 : 4;
  bool fast = fast_ok && n >= kFastTile && (k % kFastKStep) == 0 &&
              (t256 >= 160 || fast_prefers_half_tile(m, n, k, out_bytes));
  if (fast_ok && n >= kFastTile && (k % kFastKStep) != 0) fast = ceil_div(m, 128) * ceil_div(n, 256) >= 160;
  if (fast_ok && n < kFastTile) fast = ceil_div(m, 256) * ceil_div(n, n < 128 ? 64 : 128) >= 160;
  if (fast_ok && n >= kFastTile && fast_prefers_quarter_tile(m, n)) fast = true;
  // the caller's override (results are identical)
  if (tune.kernel == CWAC_KERNEL_DIRECT_LDS) {
    fast = fast_ok;
  } else if (tune.kernel != CWAC_KERNEL_AUTO) {
    tile = tune.kernel;
    fast = false;
  }
  return fast ? CWAC_KERNEL_DIRECT_LDS : tile;
}

static cwac_status dispatch_forward(const FwdParams &p, int out_kind, bool int_only, const Tune &tune,
                                    hipStream_t st) {
  const int choice = choose_forward(p.m, p.n, p.k, p.ldx, p.ldw, out_kind, tune);
  if (choice == CWAC_KERNEL_DIRECT_LDS) return launch_fast(p, out_kind, int_only, tune, st);
  if (choice == 256) return launch_tile<256, 256, 128, 2, 2>(p, out_kind, int_only, st);
  if (choice == 128) return launch_tile<128, 128, 128, 2, 2>(p, out_kind, int_only, st);
  return launch_tile<64, 64, 128, 2, 2>(p, out_kind, int_only, st);
}

extern "C" int32_t cwac_forward_kernel_for(int64_t m, int32_t n, int32_t k, int64_t ldx, int64_t ldw,
                                           int32_t out_kind, const cwac_tuning *tuning) {
  Tune tune;
  if (!tune_from(tuning, tune)) return CWAC_E_MODE;
  if (out_kind != CWAC_OUT_INT8 && out_kind != CWAC_OUT_FP32 && out_kind != CWAC_OUT_INT32) return CWAC_E_MODE;
  if (m < 1 || n < 1 || k < 16 || k > 32768 || (k % 16) != 0 || ldx < k || ldw < k) return CWAC_E_SHAPE;
  return choose_forward(m, n, k, ldx, ldw, out_kind, tune);
}

extern "C" cwac_status qlinear_cwac_forward_ex(const int8_t *x_q, int64_t ldx, const int8_t *w_q,
                                               int64_t ldw, int64_t m, int32_t n, int32_t k,
                                               const cwac_qparams *qp, const float *mult,
                                               const int32_t *offset, const float *fbias,
                                               const float *s_x_row, int32_t out_kind, void *out,
                                               int64_t ldo, const cwac_tuning *tuning, void *stream) {
  if (!x_q || !w_q || !out) return CWAC_E_NULL;
  if (out_kind != CWAC_OUT_INT8 && out_kind != CWAC_OUT_FP32 && out_kind != CWAC_OUT_INT32)
    return CWAC_E_MODE;
  Tune tune;
  if (!tune_from(tuning, tune)) return CWAC_E_MODE;
  if (out_kind != CWAC_OUT_INT32 && !mult) return CWAC_E_NULL;
  if (m < 1 || m > ((int64_t)1 << 40) || n < 1 || k < 16 || k > 32768 || (k % 16) != 0)
    return CWAC_E_SHAPE;
  if (ldx < k || ldw < k || ldo < n) return CWAC_E_SHAPE;
  if (!aligned(x_q, 16) || !aligned(w_q, 16) || (ldx % 16) != 0 || (ldw % 16) != 0)
    return CWAC_E_ALIGN;
  if (qp && out_kind != CWAC_OUT_INT32) {
    // the vectors define the epilogue; a qp that says otherwise was folded for another one
    if ((qp->act_per_token != 0) != (s_x_row != nullptr)) return CWAC_E_MODE;
    if (out_kind == CWAC_OUT_INT8 && qp->mode == CWAC_EPI_FP_BIAS && !fbias) return CWAC_E_MODE;
  }
  FwdParams p = {};
  p.x = x_q; p.w = w_q; p.ldx = ldx; p.ldw = ldw; p.ldo = ldo;
  p.m = m; p.n = n; p.k = k;
  p.mult = mult; p.offset = offset; p.fbias = fbias; p.sx_row = s_x_row; p.out = out;
  p.lo = p.hi = 0.0f; p.zr = 0;
  if (out_kind == CWAC_OUT_INT8) {
    if (!qp) return CWAC_E_NULL;
    if (qp->qmin < -128 || qp->qmax > 127 || qp->qmin > qp->qmax) return CWAC_E_SHAPE;
    if (qp->z_r < -(1 << 20) || qp->z_r > (1 << 20)) return CWAC_E_SHAPE;
    p.zr = qp->z_r;
    p.lo = (float)(qp->qmin - qp->z_r);
    p.hi = (float)(qp->qmax - qp->z_r);
  }
  const size_t esz = out_kind == CWAC_OUT_INT8 ? 1 : 4;
  if (!aligned(out, esz)) return CWAC_E_ALIGN;
  p.vec_store = ((ldo * esz) % (4 * esz) == 0) && aligned(out, 4 * esz);
  const bool int_only = (out_kind == CWAC_OUT_INT8) && !fbias && !s_x_row;
  return dispatch_forward(p, out_kind, int_only, tune, as_stream(stream));
}

extern "C" cwac_status qlinear_cwac_forward(const int8_t *x_q, int64_t ldx, const int8_t *w_q,
                                            int64_t ldw, int64_t m, int32_t n, int32_t k,
                                            const cwac_qparams *qp, const float *mult,
                                            const int32_t *offset, const float *fbias,
                                            const float *s_x_row, int32_t out_kind, void *out,
                                            int64_t ldo, void *stream) {
  return qlinear_cwac_forward_ex(x_q, ldx, w_q, ldw, m, n, k, qp, mult, offset, fbias, s_x_row, out_kind, out,
                                 ldo, nullptr, stream);
}

extern "C" cwac_status qlinear_cwac_forward_table_ex(const int8_t *x_q, int64_t ldx, const int8_t *w_q,
                                                     int64_t ldw, int64_t m, int32_t n, int32_t k,
                                                     const cwac_qparams *qp, const float *mult,
                                                     const int32_t *offset, const int8_t *table, int8_t *out,
                                                     int64_t ldo, const cwac_tuning *tuning, void *stream) {
  if (!x_q || !w_q || !out || !qp || !mult || !table) return CWAC_E_NULL;
  Tune tune;
  if (!tune_from(tuning, tune)) return CWAC_E_MODE;
  if (qp->act_per_token) return CWAC_E_MODE;  // the integer-offset epilogue has no per-row scales
  if (m < 1 || m > ((int64_t)1 << 40) || n < 16 || (n % 16) != 0 || k < 16 || k > 32768 || (k % 16) != 0)
    return CWAC_E_SHAPE;
  if (ldx < k || ldw < k || ldo < n) return CWAC_E_SHAPE;
  if (qp->qmin < -128 || qp->qmax > 127 || qp->qmin > qp->qmax) return CWAC_E_SHAPE;
  if (qp->z_r < -(1 << 20) || qp->z_r > (1 << 20)) return CWAC_E_SHAPE;
  if (!aligned(x_q, 16) || !aligned(w_q, 16) || (ldx % 16) != 0 || (ldw % 16) != 0 || !aligned(out, 16) ||
      (ldo % 16) != 0 || !aligned(table, 4))
    return CWAC_E_ALIGN;
  // Where the plain forward would take the direct-to-LDS kernel in one of its two large tiles, the table
  // is applied in that kernel's epilogue; elsewhere the forward is followed by a lookup pass in place.
  const int64_t t256 = ceil_div(m, 256) * ceil_div(n, 256), t_half = ceil_div(m, 128) * ceil_div(n, 256);
  const bool fused_ok = m >= kFastTile && n >= kFastTile && (k % 64) == 0 && fast_pitch_ok(ldx, ldw);
  bool fused = fused_ok && !fast_prefers_quarter_tile(m, n);
  if (fused) fused = (k % kFastKStep) == 0 ? (t256 >= 160 || fast_prefers_half_tile(m, n, k, 1)) : t_half >= 160;
  // the caller's override: the direct-to-LDS kernel means the fused form where its shape constraints
  // hold, a generic tile means two passes
  if (tune.kernel != CWAC_KERNEL_AUTO) fused = fused_ok && tune.kernel == CWAC_KERNEL_DIRECT_LDS;
  if (!fused) {
    const cwac_status st = qlinear_cwac_forward_ex(x_q, ldx, w_q, ldw, m, n, k, qp, mult, offset, nullptr, nullptr,
                                                   CWAC_OUT_INT8, out, ldo, tuning, stream);
    if (st != CWAC_OK) return st;
    return vit_table_lookup(out, ldo, table, out, ldo, m, n, stream);
  }
  FwdParams p = {};
  p.x = x_q; p.w = w_q; p.ldx = ldx; p.ldw = ldw; p.ldo = ldo;
  p.m = m; p.n = n; p.k = k;
  p.mult = mult; p.offset = offset; p.out = out;
  p.zr = qp->z_r;
  p.lo = (float)(qp->qmin - qp->z_r);
  p.hi = (float)(qp->qmax - qp->z_r);
  p.code_table = table;
  return launch_fast_table(p, tune.shape, tune.persist_workgroups, tune.persist_loaders, as_stream(stream));
}

extern "C" cwac_status qlinear_cwac_forward_table(const int8_t *x_q, int64_t ldx, const int8_t *w_q, int64_t ldw,
                                                  int64_t m, int32_t n, int32_t k, const cwac_qparams *qp,
                                                  const float *mult, const int32_t *offset, const int8_t *table,
                                                  int8_t *out, int64_t ldo, void *stream) {
  return qlinear_cwac_forward_table_ex(x_q, ldx, w_q, ldw, m, n, k, qp, mult, offset, table, out, ldo, nullptr,
                                       stream);
}

extern "C" cwac_status qconv2d_cwac_forward_ex(const int8_t *x_q, const int8_t *w_q, int32_t batch,
                                               int32_t h, int32_t w, int32_t c_in, int32_t c_out,
                                               int32_t kh, int32_t kw, int32_t stride, int32_t pad,
                                               const cwac_qparams *qp, const float *mult,
                                               const int32_t *offset, const float *fbias,
                                               int32_t out_kind, void *out, int64_t ldo,
                                               const cwac_tuning *tuning, void *stream) {
  if (!x_q || !w_q || !out || !qp) return CWAC_E_NULL;
  Tune tune;
  if (!tune_from(tuning, tune)) return CWAC_E_MODE;
  if (out_kind != CWAC_OUT_INT8 && out_kind != CWAC_OUT_FP32 && out_kind != CWAC_OUT_INT32)
    return CWAC_E_MODE;
  if (out_kind != CWAC_OUT_INT32 && !mult) return CWAC_E_NULL;
  if (qp->act_per_token) return CWAC_E_MODE;  // a convolution's rows share activations: per-tensor only
  if (batch < 1 || h < 1 || w < 1 || c_in < 16 || (c_in % 16) != 0 || c_out < 1 || kh < 1 || kw < 1 ||
      kh > 16 || kw > 16 || stride < 1 || stride > 16 || pad < 0 || pad >= kh || pad >= kw ||
      h > 32768 || w > 32768)
    return CWAC_E_SHAPE;
  if (h + 2 * pad < kh || w + 2 * pad < kw) return CWAC_E_SHAPE;
  const int64_t k = (int64_t)kh * kw * c_in;
  if (k > 32768) return CWAC_E_SHAPE;
  if (qp->z_x < -128 || qp->z_x > 127) return CWAC_E_SHAPE;
  const int oh = (h + 2 * pad - kh) / stride + 1, ow = (w + 2 * pad - kw) / stride + 1;
  const int64_t m = (int64_t)batch * oh * ow;
  if (m > ((int64_t)1 << 40) || (int64_t)oh * ow > 0x7fffffff || ldo < c_out) return CWAC_E_SHAPE;
  if (!aligned(x_q, 16) || !aligned(w_q, 16)) return CWAC_E_ALIGN;
  FwdParams p = {};
  p.x = x_q; p.w = w_q; p.ldx = 0; p.ldw = k; p.ldo = ldo;
  p.m = m; p.n = c_out; p.k = (int)k;
  p.mult = mult; p.offset = offset; p.fbias = fbias; p.sx_row = nullptr; p.out = out;
  p.cv_h = h; p.cv_w = w; p.cv_cin = c_in; p.cv_kw = kw; p.cv_stride = stride; p.cv_pad = pad;
  p.cv_oh = oh; p.cv_ow = ow;
  p.cv_pad4 = (int)(0x01010101u * (uint32_t)(uint8_t)(int8_t)qp->z_x);
  if (out_kind == CWAC_OUT_INT8) {
    if (qp->qmin < -128 || qp->qmax > 127 || qp->qmin > qp->qmax) return CWAC_E_SHAPE;
    if (qp->z_r < -(1 << 20) || qp->z_r > (1 << 20)) return CWAC_E_SHAPE;
    p.zr = qp->z_r;
    p.lo = (float)(qp->qmin - qp->z_r);
    p.hi = (float)(qp->qmax - qp->z_r);
  }
  const size_t esz = out_kind == CWAC_OUT_INT8 ? 1 : 4;
  if (!aligned(out, esz)) return CWAC_E_ALIGN;
  p.vec_store = ((ldo * esz) % (4 * esz) == 0) && aligned(out, 4 * esz);
  const bool int_only = (out_kind == CWAC_OUT_INT8) && !fbias;
  hipStream_t st = as_stream(stream);
  if (kh == 1 && kw == 1 && stride == 1 && pad == 0) {
    // a pointwise convolution is the linear layer on the [batch * h * w, c_in] matrix
    p.ldx = c_in;
    return dispatch_forward(p, out_kind, int_only, tune, st);
  }
  const int64_t t256 = ceil_div(m, 256) * ceil_div(c_out, 256);
  const int64_t t128 = ceil_div(m, 128) * ceil_div(c_out, 128);
  int tile = t256 >= 512 ? 256 : (t128 >= 512 ? 128 : 64);
  // narrow layers: a tile much wider than the layer would multiply mostly padding
  if (c_out <= 160 && tile > 128) tile = 128;
  if (c_out <= 80 && tile > 64) tile = 64;
  // the direct-to-LDS kernel where its shape constraints hold and its 128 x 256 tiles occupy at
  // least a quarter of the compute units (measured on ResNet-50 layer shapes: ahead of the generic
  // kernel's small tiles from there on)
  const int64_t image_bytes = (int64_t)batch * h * w * c_in;
  const bool fast_ok = fast_conv_ok(p, image_bytes);
  bool fast = fast_ok && (c_out >= 256 ? ceil_div(m, 128) * ceil_div(c_out, 256)
                                      : ceil_div(m, 256) * ceil_div(c_out, c_out < 128 ? 64 : 128)) >= 64;
  if (fast_ok && c_out >= 256 && fast_prefers_quarter_tile(m, c_out)) fast = true;
  if (tune.kernel == CWAC_KERNEL_DIRECT_LDS) {  // the caller's override, as for the linear layer
    fast = fast_ok;
  } else if (tune.kernel != CWAC_KERNEL_AUTO) {
    tile = tune.kernel;
    fast = false;
  }
  if (fast) return launch_fast_conv(p, out_kind, int_only, tune.shape, st);
  if (tile == 256) return launch_tile<256, 256, 128, 2, 2, true>(p, out_kind, int_only, st);
  if (tile == 128) return launch_tile<128, 128, 128, 2, 2, true>(p, out_kind, int_only, st);
  return launch_tile<64, 64, 128, 2, 2, true>(p, out_kind, int_only, st);
}

extern "C" cwac_status qconv2d_cwac_forward(const int8_t *x_q, const int8_t *w_q, int32_t batch,
                                            int32_t h, int32_t w, int32_t c_in, int32_t c_out,
                                            int32_t kh, int32_t kw, int32_t stride, int32_t pad,
                                            const cwac_qparams *qp, const float *mult,
                                            const int32_t *offset, const float *fbias,
                                            int32_t out_kind, void *out, int64_t ldo, void *stream) {
  return qconv2d_cwac_forward_ex(x_q, w_q, batch, h, w, c_in, c_out, kh, kw, stride, pad, qp, mult, offset, fbias,
                                 out_kind, out, ldo, nullptr, stream);
}

extern "C" size_t cwac_calibrate_fused_workspace(int64_t m, int32_t n) {
  if (m < 1 || n < 1) return 16;
  // partial sums [row tiles][kStats][n] fp64, then Y_quant of row 0 [n] fp32
  return (size_t)ceil_div(m, kFastTile) * kStats * (size_t)n * sizeof(double) + (size_t)n * sizeof(float);
}

extern "C" cwac_status qlinear_cwac_calibrate_fused_ex(const int8_t *x_q, int64_t ldx,
                                                       const int8_t *w_q, int64_t ldw, int64_t m,
                                                       int32_t n, int32_t k, const float *mult,
                                                       const int32_t *offset, const float *fbias,
                                                       const float *s_x_row, const float *y_full,
                                                       int64_t ld_full, void *stats, void *workspace,
                                                       size_t workspace_bytes,
                                                       const cwac_tuning *tuning, void *stream) {
  if (!x_q || !w_q || !mult || !y_full || !stats) return CWAC_E_NULL;
  Tune tune;
  if (!tune_from(tuning, tune)) return CWAC_E_MODE;
  if (m < kFastTile || m > ((int64_t)1 << 40) || n < kFastTile || n > 65536 || (n % 4) != 0 ||
      k < kFastKStep || k > 32768 || (k % kFastKStep) != 0)
    return CWAC_E_SHAPE;
  if (ldx < k || ldw < k || ld_full < n) return CWAC_E_SHAPE;
  if (!aligned(x_q, 16) || !aligned(w_q, 16) || (ldx % 16) != 0 || (ldw % 16) != 0 ||
      !aligned(y_full, 16) || (ld_full % 4) != 0 || !aligned(stats, 16))
    return CWAC_E_ALIGN;
  // per-lane byte offsets into a tile of Y_full and into the panels are kept in 32 bits
  if (ld_full > ((int64_t)1 << 26) || !fast_pitch_ok(ldx, ldw)) return CWAC_E_SHAPE;
  if (!workspace || workspace_bytes < cwac_calibrate_fused_workspace(m, n)) return CWAC_E_WORKSPACE;
  if (!aligned(workspace, 16)) return CWAC_E_ALIGN;
  FwdParams p = {};
  p.x = x_q; p.w = w_q; p.ldx = ldx; p.ldw = ldw;
  p.m = m; p.n = n; p.k = k;
  p.mult = mult; p.offset = offset; p.fbias = fbias; p.sx_row = s_x_row;
  p.y_full = y_full; p.ld_full = ld_full; p.stats = stats;
  p.partial = static_cast<double *>(workspace);
  const int row_tiles = (int)ceil_div(m, kFastTile);
  float *yq_row0 = reinterpret_cast<float *>(p.partial + (size_t)row_tiles * kStats * n);
  p.yq_row0 = yq_row0;
  hipStream_t st = as_stream(stream);
  row0_kernel<<<(unsigned)ceil_div(n, 4), 256, 0, st>>>(p, yq_row0);  // one channel per wavefront
  cwac_status rc = launch_status();
  if (rc != CWAC_OK) return rc;
  rc = launch_fast_stats(p, tune.stats_waves, st);
  if (rc != CWAC_OK) return rc;
  return launch_stats_merge(p.partial, row_tiles, n, y_full, yq_row0, stats, m, false, st);
}

extern "C" cwac_status qlinear_cwac_calibrate_fused(const int8_t *x_q, int64_t ldx,
                                                    const int8_t *w_q, int64_t ldw, int64_t m,
                                                    int32_t n, int32_t k, const float *mult,
                                                    const int32_t *offset, const float *fbias,
                                                    const float *s_x_row, const float *y_full,
                                                    int64_t ld_full, void *stats, void *workspace,
                                                    size_t workspace_bytes, void *stream) {
  return qlinear_cwac_calibrate_fused_ex(x_q, ldx, w_q, ldw, m, n, k, mult, offset, fbias, s_x_row, y_full,
                                         ld_full, stats, workspace, workspace_bytes, nullptr, stream);
}

extern "C" cwac_status qlinear_cwac_forward_fixed_point_ex(const int8_t *x_q, int64_t ldx,
                                                           const int8_t *w_q, int64_t ldw, int64_t m,
                                                           int32_t n, int32_t k, const cwac_qparams *qp,
                                                           const int32_t *m0, const int32_t *shift,
                                                           const int32_t *offset, int8_t *out,
                                                           int64_t ldo, const cwac_tuning *tuning,
                                                           void *stream) {
  if (!x_q || !w_q || !out || !qp || !m0 || !shift) return CWAC_E_NULL;
  Tune tune;
  if (!tune_from(tuning, tune)) return CWAC_E_MODE;
  // per-row scales and an fp32 bias have no fixed-point form
  if (qp->act_per_token || qp->mode != CWAC_EPI_INT_OFFSET) return CWAC_E_MODE;
  if (m < 1 || m > ((int64_t)1 << 40) || n < 1 || k < 16 || k > 32768 || (k % 16) != 0)
    return CWAC_E_SHAPE;
  if (ldx < k || ldw < k || ldo < n) return CWAC_E_SHAPE;
  if (!aligned(x_q, 16) || !aligned(w_q, 16) || (ldx % 16) != 0 || (ldw % 16) != 0)
    return CWAC_E_ALIGN;
  if (qp->qmin < -128 || qp->qmax > 127 || qp->qmin > qp->qmax) return CWAC_E_SHAPE;
  if (qp->z_r < -(1 << 20) || qp->z_r > (1 << 20)) return CWAC_E_SHAPE;
  FwdParams p = {};
  p.x = x_q; p.w = w_q; p.ldx = ldx; p.ldw = ldw; p.ldo = ldo;
  p.m = m; p.n = n; p.k = k;
  p.offset = offset; p.out = out;
  p.m0 = m0; p.shift = shift;
  p.zr = qp->z_r;
  p.qlo = qp->qmin - qp->z_r;
  p.qhi = qp->qmax - qp->z_r;
  p.vec_store = (ldo % 4 == 0) && aligned(out, 4);
  return dispatch_forward(p, kOutFixed, true, tune, as_stream(stream));
}

extern "C" cwac_status qlinear_cwac_forward_fixed_point(const int8_t *x_q, int64_t ldx,
                                                        const int8_t *w_q, int64_t ldw, int64_t m,
                                                        int32_t n, int32_t k, const cwac_qparams *qp,
                                                        const int32_t *m0, const int32_t *shift,
                                                        const int32_t *offset, int8_t *out,
                                                        int64_t ldo, void *stream) {
  return qlinear_cwac_forward_fixed_point_ex(x_q, ldx, w_q, ldw, m, n, k, qp, m0, shift, offset, out, ldo, nullptr,
                                             stream);
}
