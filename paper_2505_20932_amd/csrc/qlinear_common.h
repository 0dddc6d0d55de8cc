// Pieces shared by the quantized-linear forward kernels: parameter block, workgroup -> tile
// mapping, and the reference form of the Eq. 10 epilogue on register-resident accumulators.
#pragma once

#include "cwac_internal.h"

namespace cwac {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

struct FwdParams {
  const int8_t *x;
  const int8_t *w;
  int64_t ldx, ldw, ldo;
  int64_t m;
  int n, k;
  const float *mult;
  const int32_t *offset;
  const float *fbias;
  const float *sx_row;
  void *out;
  float lo, hi;
  int zr;
  int vec_store;  // output layout allows 4-element vector stores
  int tiles_m, tiles_n;
  // fused calibration statistics (kOutStats): Y_full of the same rows and channels, the
  // calibration state (read: row count, pivots) and partial[tiles_m][kStats][n] (written)
  const float *y_full;
  int64_t ld_full;
  const void *stats;
  double *partial;
  const float *yq_row0;  // Y_quant of row 0 [n]: the pivot of a state's first batch
  // integer-only epilogue (kOutFixed): multiplier m0[n] * 2^-shift[n], clamp [qlo, qhi] then + zr
  const int32_t *m0;
  const int32_t *shift;
  int qlo, qhi;
  // convolution as an implicit GEMM (generic kernel, CONV instantiation): x is the image tensor
  // [batch, cv_h, cv_w, cv_cin] (channels last), row m = (b, oh, ow), k = (kh * cv_kw + kw) * cv_cin + c;
  // positions outside the image read cv_pad4 (the zero-point code in all four bytes)
  int cv_h, cv_w, cv_cin, cv_kw, cv_stride, cv_pad, cv_oh, cv_ow;
  int cv_pad4;
  const int8_t *code_table;  // kOutTable: table[code + 128]
};

// Internal output kind of the large-problem kernel: nothing is stored but the per-channel sums
// of the tile's rows of (Y_full, Y_quant).
constexpr int kOutStats = 3;
// Internal output kind: int8 codes through the integer-only epilogue (no floating point).
constexpr int kOutFixed = 4;
// Internal output kind: the int8 codes of the integer-offset epilogue mapped through a 256-entry code
// table (an activation function between two int8 layers) before they are stored.
constexpr int kOutTable = 5;

// Integer-only requantization (fixed-point form of Eq. 10): the nearest integer to
// t * m0 * 2^-shift, ties towards +infinity, exact in 64 bits (|t|, |m0| < 2^31, 1 <= shift <= 62),
// saturated to int32, clamped to [qlo, qhi] = [qmin - Z_r, qmax - Z_r], plus Z_r.
__device__ __forceinline__ int fixed_point_code(int t, int m0, int shift, int qlo, int qhi, int zr) {
  const int64_t prod = (int64_t)t * (int64_t)m0 + ((int64_t)1 << (shift - 1));
  const int64_t v = prod >> shift;  // arithmetic shift: floor
  const int lo32 = (int)v, hi32 = (int)(v >> 32);
  int r = (hi32 == (lo32 >> 31)) ? lo32 : (hi32 < 0 ? (int)0x80000000 : 0x7fffffff);
  r = r < qlo ? qlo : r;
  r = r > qhi ? qhi : r;
  return r + zr;
}

// Workgroup id -> output tile.  Consecutive workgroup ids are dealt round-robin
// to the 8 XCDs (each with its own L2), so ids are first regrouped so that every
// XCD works on a contiguous range of tiles, and tiles are then walked in bands of
// GROUP_M tile-rows so that the tiles in flight on one XCD share weight and
// activation panels in its L2.
__device__ __forceinline__ void tile_of_block(int pid, int tiles_m, int tiles_n, int &tm, int &tn) {
  const int total = tiles_m * tiles_n;
  constexpr int XCDS = 8;
  const int per = total / XCDS, rem = total - per * XCDS;
  const int xcd = pid % XCDS, local = pid / XCDS;
  // ids dealt to xcd: `per` of them, plus one more for the first `rem` xcds
  const int start = xcd * per + (xcd < rem ? xcd : rem);
  const int id = start + local;
  constexpr int GROUP_M = 8;
  const int band = GROUP_M * tiles_n;
  const int g = id / band;
  const int first_m = g * GROUP_M;
  const int rows = (tiles_m - first_m) < GROUP_M ? (tiles_m - first_m) : GROUP_M;
  const int in = id - g * band;
  tm = first_m + in % rows;
  tn = in / rows;
}

template <int OUT_KIND, bool INT_ONLY>
struct Epilogue {
  // Applies Eq. 10 to 4 consecutive channels nn..nn+3 of row mm and stores them.
  __device__ static __forceinline__ void run(const FwdParams &p, int64_t mm, int nn,
                                             const int (&acc)[4], const float (&mu)[4],
                                             const int (&off)[4], const float (&fb)[4],
                                             float rs) {
    if (OUT_KIND == CWAC_OUT_INT32) {
      int t[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) t[r] = acc[r] + off[r];
      int32_t *o = static_cast<int32_t *>(p.out) + mm * p.ldo + nn;
      if (p.vec_store && nn + 3 < p.n) {
        *reinterpret_cast<int4 *>(o) = make_int4(t[0], t[1], t[2], t[3]);
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (nn + r < p.n) o[r] = t[r];
      }
      return;
    }
    if (OUT_KIND == kOutFixed) {
      int c[4];
#pragma unroll
      for (int r = 0; r < 4; ++r)
        c[r] = fixed_point_code(acc[r] + off[r], __float_as_int(mu[r]), __float_as_int(fb[r]), p.qlo,
                                p.qhi, p.zr);
      int8_t *o = static_cast<int8_t *>(p.out) + mm * p.ldo + nn;
      if (p.vec_store && nn + 3 < p.n) {
        *reinterpret_cast<uint32_t *>(o) = (uint32_t)(c[0] & 0xff) | ((uint32_t)(c[1] & 0xff) << 8) |
                                           ((uint32_t)(c[2] & 0xff) << 16) | ((uint32_t)c[3] << 24);
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (nn + r < p.n) o[r] = (int8_t)c[r];
      }
      return;
    }
    float u[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float f = (float)(acc[r] + off[r]);
      if (!INT_ONLY) {
        if (p.sx_row) f = f * rs;
      }
      float v = f * mu[r];
      if (!INT_ONLY) {
        if (p.fbias) v = v + fb[r];
      }
      u[r] = v;
    }
    if (OUT_KIND == CWAC_OUT_FP32) {
      float *o = static_cast<float *>(p.out) + mm * p.ldo + nn;
      if (p.vec_store && nn + 3 < p.n) {
        *reinterpret_cast<float4 *>(o) = make_float4(u[0], u[1], u[2], u[3]);
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (nn + r < p.n) o[r] = u[r];
      }
    } else {
      int c[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) c[r] = requant_code(u[r], p.lo, p.hi, p.zr);
      int8_t *o = static_cast<int8_t *>(p.out) + mm * p.ldo + nn;
      if (p.vec_store && nn + 3 < p.n) {
        *reinterpret_cast<uint32_t *>(o) = (uint32_t)(c[0] & 0xff) | ((uint32_t)(c[1] & 0xff) << 8) |
                                           ((uint32_t)(c[2] & 0xff) << 16) | ((uint32_t)c[3] << 24);
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (nn + r < p.n) o[r] = (int8_t)c[r];
      }
    }
  }
};

// Epilogue over a wave's TN x TM accumulator tiles.  Accumulator element 4*g + r of
// tile (a, b) belongs to channel n = n0 + a*32 + 8*g + 4*half + r and token
// m = m0 + b*32 + l32 (n0, m0: first channel / token of the wave tile).
template <int TM, int TN, int OUT_KIND, bool INT_ONLY>
__device__ __forceinline__ void epilogue_tiles(const FwdParams &p, v16i (&acc)[TN][TM], int64_t m0,
                                               int n0, int l32, int half, int vec_store) {
  FwdParams q = p;
  q.vec_store = vec_store;
#pragma unroll
  for (int a = 0; a < TN; ++a) {
    const int nb = n0 + a * 32 + 4 * half;
    float mu[4][4], fb[4][4];
    int off[4][4];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        int idx = nb + 8 * g + r;
        if (idx > p.n - 1) idx = p.n - 1;  // clamped read; such channels are never stored
        off[g][r] = p.offset ? p.offset[idx] : 0;
        if (OUT_KIND == kOutFixed) {  // the two float slots carry the integer multiplier and shift
          mu[g][r] = __int_as_float(p.m0[idx]);
          fb[g][r] = __int_as_float(p.shift[idx]);
        } else {
          mu[g][r] = (OUT_KIND != CWAC_OUT_INT32) ? p.mult[idx] : 0.0f;
          fb[g][r] = (!INT_ONLY && OUT_KIND != CWAC_OUT_INT32 && p.fbias) ? p.fbias[idx] : 0.0f;
        }
      }
#pragma unroll
    for (int b = 0; b < TM; ++b) {
      const int64_t mm = m0 + b * 32 + l32;
      if (mm < p.m) {
        const float rs =
            (!INT_ONLY && OUT_KIND != CWAC_OUT_INT32 && OUT_KIND != kOutFixed && p.sx_row) ? p.sx_row[mm] : 1.0f;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int nn = nb + 8 * g;
          if (nn < p.n) {
            const int av[4] = {acc[a][b][4 * g], acc[a][b][4 * g + 1], acc[a][b][4 * g + 2],
                               acc[a][b][4 * g + 3]};
            Epilogue<OUT_KIND, INT_ONLY>::run(q, mm, nn, av, mu[g], off[g], fb[g], rs);
          }
        }
      }
    }
  }
}


// Kernel choice override of the _ex entry points (cwac.h: cwac_tuning), validated.
struct Tune {
  int kernel = CWAC_KERNEL_AUTO, shape = CWAC_SHAPE_AUTO, stats_waves = 0, persist_workgroups = 0, persist_loaders = 0;
};
// False where a field holds a value outside its list (the entry point returns CWAC_E_MODE).
inline bool tune_from(const cwac_tuning *t, Tune &o) {
  o = Tune{};
  if (!t) return true;
  if (t->kernel != CWAC_KERNEL_AUTO && t->kernel != CWAC_KERNEL_DIRECT_LDS && t->kernel != CWAC_KERNEL_GENERIC_64 &&
      t->kernel != CWAC_KERNEL_GENERIC_128 && t->kernel != CWAC_KERNEL_GENERIC_256)
    return false;
  if (t->shape < CWAC_SHAPE_AUTO || t->shape > CWAC_SHAPE_256_PERSIST) return false;
  if (t->stats_waves != 0 && t->stats_waves != 4 && t->stats_waves != 8) return false;
  o.kernel = t->kernel;
  o.shape = t->shape;
  o.stats_waves = t->stats_waves;
  if (t->persist_workgroups < 0) return false;
  o.persist_workgroups = t->persist_workgroups;
  if (t->persist_loaders != 0 && t->persist_loaders != 4 && t->persist_loaders != 8) return false;
  o.persist_loaders = t->persist_loaders;
  return true;
}

// The direct-to-LDS kernel keeps a lane's byte offset inside a tile's panel (row * pitch + chunk,
// rows < 256) in 32 bits: pitches up to 2^24 bytes cannot wrap it (255 * 2^24 + 128 < 2^32).
constexpr int64_t kFastMaxPitch = (int64_t)1 << 24;
inline bool fast_pitch_ok(int64_t ldx, int64_t ldw) { return ldx <= kFastMaxPitch && ldw <= kFastMaxPitch; }

// Large-problem kernel (qlinear_fast.hip).  Requires m >= 256, n >= 64, k % 64 == 0 (its 256 x 256
// tile: n >= 256 and k % 128 == 0) and fast_pitch_ok(ldx, ldw).  tune.shape: CWAC_SHAPE_* (0 = by cost model).
cwac_status launch_fast(FwdParams p, int out_kind, bool int_only, const Tune &tune, hipStream_t st);
// The integer-offset int8 forward with p.code_table applied to every output code (kOutTable); shapes as
// launch_fast with n >= 256.
cwac_status launch_fast_table(FwdParams p, int shape, int max_workgroups, int loaders, hipStream_t st);
// True where that kernel would take its 128-token tile shape (two workgroups per compute unit).
bool fast_prefers_half_tile(int64_t m, int n, int k, int out_bytes);
// True where it would take 128 x 128 tiles (layers with few tiles and a long K loop).
bool fast_prefers_quarter_tile(int64_t m, int n);
// The tile shape (CWAC_SHAPE_*) launch_fast picks by itself for a linear layer with n >= 256.
int fast_linear_shape(int64_t m, int n, int k, int out_bytes);
// The same kernel as an implicit-GEMM convolution (p.cv_* set, p.ldx unused).  fast_conv_ok: its shape
// constraints (m >= 256, n >= 64, c_in % 64 == 0, image below 2 GiB).
bool fast_conv_ok(const FwdParams &p, int64_t image_bytes);
cwac_status launch_fast_conv(FwdParams p, int out_kind, bool int_only, int shape, hipStream_t st);
// Same kernel with the statistics epilogue; additionally requires n % 4 == 0, ld_full % 4 == 0
// and a 16-byte aligned y_full.  p.partial receives ceil(m / 256) row groups.  waves: 8 (0) or 4.
cwac_status launch_fast_stats(FwdParams p, int waves, hipStream_t st);
constexpr int kFastTile = 256;
constexpr int kFastKStep = 128;

}  // namespace cwac
