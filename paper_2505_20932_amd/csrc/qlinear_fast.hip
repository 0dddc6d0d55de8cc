// Large-problem kernel of the quantized linear layer with the CWAC epilogue (Sec. 3.4,
// Eq. 10): 256 x 256 output tile, one workgroup per compute unit, of eight wavefronts (4 x 2,
// each 64 x 128 = 2 x 4 MFMA tiles, 128 int32 accumulators per lane, two wavefronts per SIMD so
// that one's load issue and LDS reads run under the other's MFMAs) or of four wavefronts (2 x 2,
// each 128 x 128, 256 accumulators per lane; the shape the statistics epilogue uses).
//
//   * Panels go global -> LDS directly (global_load_lds_dwordx4, no register staging).  One
//     wavefront load lands as 1 KiB of contiguous LDS, so the bank swizzle is applied on the
//     GLOBAL side: lane (row r, slot p) fetches chunk p ^ swz(r) of its row.
//   * A ring of NSTAGE LDS stages of BK bytes of K; the loads of stage s + NSTAGE are issued as
//     soon as every wavefront has fetched its last fragments of stage s; one barrier per stage,
//     NSTAGE - 1 stages of loads in flight behind the MFMAs.
//   * MFMA operand fragments are double-buffered in registers; the LDS reads of step kk + 1 are
//     interleaved with the MFMAs of step kk.
//   * The epilogue parameters of the tile's 256 channels (and the 256 row scales) are staged in
//     LDS while the first panels are in flight; accumulators START at offset[n], so the integer
//     offset add of Eq. 10 costs nothing, and rounding uses one fp32 add of 1.5 * 2^23, which
//     rounds half to even exactly like rint for the clamped (|x| < 2^22) values it sees.
//
//   * A second shape of the same kernel for layers with a short K loop (ViT / Swin linears): a
//     128-token x 256-channel tile (wave tile 64 x 128), 64-byte K steps, three stages, at most 256
//     registers per lane, so that TWO workgroups share a compute unit and one's prologue and
//     epilogue run under the other's main loop.
//
// Requires m >= 256, n >= 256, k % 128 == 0 (the 128-token shape: k % 64 == 0).  Edge tiles are shifted inwards to overlap their
// neighbours (identical values are written twice) instead of being predicated.
#include <type_traits>

#include "qlinear_common.h"

namespace cwac {
namespace {

#define CWAC_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#define CWAC_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void *)(p))

// Convolution: the 16 bytes a load fetches for a filter tap outside the image.  Row c holds the
// code c sixteen times; a direct-to-LDS load cannot substitute a value, so it is pointed here.
struct PadCodes {
  uint8_t v[256 * 16];
  constexpr PadCodes() : v() {
    for (int i = 0; i < 256 * 16; ++i) v[i] = (uint8_t)(i >> 4);
  }
};
__device__ __attribute__((aligned(16))) const PadCodes kPadCodes{};

#ifdef CWAC_V_STAMP
// timing probe (development builds only): 100 MHz time stamps of every wavefront at five points
__device__ unsigned long long g_stamps[4096 * 8 * 5];
#define CWAC_STAMP(i)                                                                                  \
  if (blockIdx.x < 4096 && (threadIdx.x & 63) == 0)                                                    \
  g_stamps[(blockIdx.x * 8 + (threadIdx.x >> 6)) * 5 + (i)] = __builtin_amdgcn_s_memrealtime()
#define CWAC_STAMPT(id, i)                                                                             \
  if ((id) < 4096 && (threadIdx.x & 63) == 0)                                                          \
  g_stamps[((id) * 8 + (threadIdx.x >> 6)) * 5 + (i)] = __builtin_amdgcn_s_memrealtime()
#else
#define CWAC_STAMP(i)
#define CWAC_STAMPT(id, i)
#endif

constexpr int s_waitcnt_imm(int vmcnt, int lgkmcnt) {
  // gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] << 14 ; expcnt = 7 (no wait)
  return (vmcnt & 15) | (7 << 4) | ((lgkmcnt & 15) << 8) | (((vmcnt >> 4) & 3) << 14);
}

template <int BM_, int WM_, int BK, int NSTAGE, int NCHUNK, int BN_ = 256, int TA_ = 0>
struct FastCfg {
  static constexpr int BM = BM_, BN = BN_;
  static constexpr int TA = TA_ ? TA_ : (BN >= 128 ? 4 : BN / 32);  // 32-channel MFMA tiles per wavefront
  static constexpr int WM = WM_, WN = BN / (32 * TA);  // wavefronts along m and n
  static constexpr int NWAVES = WN * WM, NT = 64 * NWAVES;
  static constexpr int TB = BM / (32 * WM);      // 32-token MFMA tiles per wavefront
  static constexpr int KK = BK / 32;  // MFMA k-steps per stage
  static constexpr int X_BYTES = BM * BK, W_BYTES = BN * BK, STAGE = X_BYTES + W_BYTES;
  static constexpr int RING = NSTAGE * STAGE;
  static constexpr int PARAM_BYTES = 4 * 256 * 4;  // offset, mult, fbias [256 channels], row scale [256 rows]
  static constexpr int LDS_BYTES = RING + PARAM_BYTES;
  // statistics epilogue: + the two pivots of the 256 channels
  static constexpr int STATS_LDS_BYTES = RING + PARAM_BYTES + 2 * 256 * 4;
  static constexpr int CPR = BK / 16;        // 16-byte chunks per row
  static constexpr int RPL = 64 / CPR;       // rows covered by one wavefront load
  static constexpr int XROWS = BM / NWAVES;   // activation rows each wavefront loads per stage
  static constexpr int WLROWS = BN / NWAVES;  // weight rows each wavefront loads per stage
  static constexpr int LOADS_X = XROWS / RPL;  // loads per wavefront and stage, activation panel
  static constexpr int LOADS_W = WLROWS / RPL;  // ... weight panel
  static constexpr int LPS = LOADS_X + LOADS_W;  // loads per wavefront and stage
  static constexpr int CHUNK = (LPS + NCHUNK - 1) / NCHUNK;  // most loads issued in one k-step
  // chunk c of a stage's loads = loads [chunk_begin(c), chunk_begin(c + 1))
  __host__ __device__ static constexpr int chunk_begin(int c) { return c * LPS / NCHUNK; }
  static_assert((BM == 256 || BM == 128) && (BN == 256 || BN == 128 || BN == 64) && (WM == 2 || WM == 4) &&
                    (TB == 4 || TB == 2),
                "tile and wave grid");
  static_assert(XROWS % RPL == 0 && WLROWS % RPL == 0, "whole loads per wavefront");
  static_assert(BK == 64 || BK == 128, "K step");
  static_assert(NCHUNK >= 1 && NCHUNK <= KK && NCHUNK <= LPS, "load chunks per stage");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS budget of one compute unit");
  static_assert((NSTAGE - 1) * LPS < 64, "vmcnt is a 6-bit counter");
  // swizzle of the 16-byte chunk position inside a row, a function of the row's low 4 bits
  __host__ __device__ static constexpr int swz(int r) {
    return BK == 128 ? ((r >> 1) & 7) : (((r >> 2) & 1) | ((((r >> 1) ^ (r >> 3)) & 1) << 1));
  }
};

__device__ __forceinline__ uint32_t pack4(int b0, int b1, int b2, int b3) {
  const uint32_t t01 = __builtin_amdgcn_perm((uint32_t)b1, (uint32_t)b0, 0x0c0c0400u);
  const uint32_t t23 = __builtin_amdgcn_perm((uint32_t)b3, (uint32_t)b2, 0x0c0c0400u);
  return __builtin_amdgcn_perm(t23, t01, 0x05040100u);
}

// Epilogue (Eq. 10) on the register-resident accumulators, which already hold acc + offset.
// Element 4*g + r of tile (a, b): channel n = bn0 + wave_n*128 + a*32 + 8*g + 4*half + r,
// token m = bm0 + wave_m*128 + b*32 + l32.
//
// VEC path: a lane's results are 4-channel groups scattered over 32 token rows, which would
// make every store instruction touch 32 cache lines with a few bytes each.  Instead each
// wavefront transposes a slab of 128 rows x 128 bytes through its private LDS region (row
// stride 144 bytes: conflict-free 16-byte accesses) and writes it out as whole 128-byte lines,
// 8 rows per store instruction.  int8: one slab holds all 128 channels of the wave tile (the
// two half-waves first swap packed words so that a lane owns 16 consecutive channels);
// fp32 / int32: one slab per 32-channel MFMA column.
// Non-VEC path (unaligned output): element-wise stores.
constexpr int kSlabStride = 144;

template <int OUT_KIND, int ROWS, int ROW_BYTES = 128>
__device__ __forceinline__ void store_slab(const int8_t *slab, char *gbase, int64_t row_bytes, int lane) {
  constexpr int CPR = ROW_BYTES / 16, RPP = 64 / CPR;  // 16-byte chunks per row, rows per store instruction
  const int rd_row = lane / CPR, rd_chunk = lane % CPR;
#pragma unroll
  for (int i = 0; i < ROWS / RPP; ++i) {
    const int row = i * RPP + rd_row;
    const v4i v = *reinterpret_cast<const v4i *>(slab + row * kSlabStride + rd_chunk * 16);
    v4i *dst = reinterpret_cast<v4i *>(gbase + row * row_bytes + rd_chunk * 16);
    // 4-byte outputs (the calibration forward's Y_quant) are far larger than the caches and are
    // streamed out: written normally they linger as dirty lines whose write-back then competes
    // with the reads of the statistics pass that follows
    // (int8 results stay cacheable for the layer that consumes them)
    if (OUT_KIND != CWAC_OUT_INT8 && OUT_KIND != kOutFixed && OUT_KIND != kOutTable)
      __builtin_nontemporal_store(v, dst);
    else
      *dst = v;
  }
}

//
// ZFOLD (int8 codes through the floating-point multiplier): how Z_r reaches the code.
//   0: added to the integer read off the rounding sum (one more instruction per result).
//   1: Z_r even - it rides in the rounding constant: u + (1.5 * 2^23 + Z_r) rounds u to the nearest integer
//      with ties to the even SUM, which is the even round(u) exactly when the constant is even.
//   2: Z_r odd - the chain runs on -u (the converted accumulator enters the first multiply negated and the
//      bias is subtracted: sign modifiers, and round-to-nearest is symmetric, so every intermediate is the
//      exact negative), the constant carries the even -Z_r - 1, and the packed word is complemented:
//      ~(c - n) = n - c - 1 = n + Z_r in every byte.
template <int OUT_KIND, bool INT_ONLY, bool VEC, int TB, int WM, int TA, int ZFOLD = 0>
__device__ __forceinline__ void fast_epilogue(const FwdParams &p, v16i (&acc)[TA][TB], int8_t *smem,
                                              const float *s_mult, const float *s_fb,
                                              const float *s_rs, int64_t bm0, int bn0, int wave_m,
                                              int wave_n, int lane) {
  constexpr bool I8 = OUT_KIND == CWAC_OUT_INT8 || OUT_KIND == kOutFixed || OUT_KIND == kOutTable;  // packed int8 codes
  // kOutTable: the code table sits in the (otherwise unused) fp-bias slot of the parameter block
  const uint8_t *s_tab = reinterpret_cast<const uint8_t *>(s_fb);
  constexpr int ESZ = I8 ? 1 : 4;
  const int l32 = lane & 31, half = lane >> 5;
  const int wave = wave_m + WM * wave_n;
  constexpr int WROWS = 32 * TB;  // token rows of the wave tile = rows of a slab
  int8_t *slab = smem + wave * (WROWS * kSlabStride);
  const int64_t row_bytes = p.ldo * ESZ;
  // first element of the wave tile in the output
  char *wbase = static_cast<char *>(p.out) + ((bm0 + wave_m * WROWS) * p.ldo + bn0 + wave_n * (32 * TA)) * ESZ;
  float rs[TB];
#pragma unroll
  for (int b = 0; b < TB; ++b) rs[b] = s_rs[wave_m * WROWS + b * 32 + l32];
  const bool use_rs = !INT_ONLY && p.sx_row != nullptr;
  const bool use_fb = !INT_ONLY && p.fbias != nullptr;
  // 1.5 * 2^23: adding it rounds to nearest even at unit steps; with ZFOLD the zero point rides along (the
  // code table is indexed by code + 128, which is even and rides along as well)
  const int zfold = (ZFOLD == 2 ? -p.zr - 1 : ZFOLD == 1 ? p.zr : 0) +
                    (ZFOLD && OUT_KIND == kOutTable ? (ZFOLD == 2 ? -128 : 128) : 0);
  const float magic = 12582912.0f + (float)zfold;
#pragma unroll
  for (int a = 0; a < TA; ++a) {
    float mu[4][4], fb[4][4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int cl = wave_n * (32 * TA) + a * 32 + 8 * g + 4 * half;  // channel inside the tile
      if (OUT_KIND != CWAC_OUT_INT32) {
        const float4 m4 = *reinterpret_cast<const float4 *>(s_mult + cl);
        mu[g][0] = m4.x; mu[g][1] = m4.y; mu[g][2] = m4.z; mu[g][3] = m4.w;
        if (!INT_ONLY || OUT_KIND == kOutFixed) {  // fixed point: the shift travels in this slot
          const float4 f4 = *reinterpret_cast<const float4 *>(s_fb + cl);
          fb[g][0] = f4.x; fb[g][1] = f4.y; fb[g][2] = f4.z; fb[g][3] = f4.w;
        }
      }
    }
#pragma unroll
    for (int b = 0; b < TB; ++b) {
      const int row = b * 32 + l32;  // row inside the wave tile
      uint32_t packed[4];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = a * 32 + 8 * g + 4 * half;  // channel inside the wave tile
        if (OUT_KIND == CWAC_OUT_INT32) {
          const v4i t = {acc[a][b][4 * g], acc[a][b][4 * g + 1], acc[a][b][4 * g + 2],
                         acc[a][b][4 * g + 3]};
          if (VEC) {
            *reinterpret_cast<v4i *>(slab + row * kSlabStride + (8 * g + 4 * half) * 4) = t;
          } else {
            int32_t *o = reinterpret_cast<int32_t *>(wbase + row * row_bytes) + col;
#pragma unroll
            for (int r = 0; r < 4; ++r) o[r] = t[r];
          }
          continue;
        }
        if (OUT_KIND == kOutFixed) {
          int c[4];
#pragma unroll
          for (int r = 0; r < 4; ++r)
            c[r] = fixed_point_code(acc[a][b][4 * g + r], __float_as_int(mu[g][r]),
                                    __float_as_int(fb[g][r]), p.qlo, p.qhi, p.zr);
          if (VEC) {
            packed[g] = pack4(c[0], c[1], c[2], c[3]);
          } else {
            int8_t *o = reinterpret_cast<int8_t *>(wbase + row * row_bytes) + col;
#pragma unroll
            for (int r = 0; r < 4; ++r) o[r] = (int8_t)c[r];
          }
          continue;
        }
        float u[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          float f = (float)acc[a][b][4 * g + r];
          if (ZFOLD == 2) f = -f;
          if (use_rs) f = f * rs[b];
          float v = f * mu[g][r];
          if (use_fb) v = ZFOLD == 2 ? v - fb[g][r] : v + fb[g][r];
          u[r] = v;
        }
        if (OUT_KIND == CWAC_OUT_FP32) {
          if (VEC) {
            *reinterpret_cast<float4 *>(slab + row * kSlabStride + (8 * g + 4 * half) * 4) =
                make_float4(u[0], u[1], u[2], u[3]);
          } else {
            float *o = reinterpret_cast<float *>(wbase + row * row_bytes) + col;
#pragma unroll
            for (int r = 0; r < 4; ++r) o[r] = u[r];
          }
        } else {
          int c[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            // clamp(rint(u), lo, hi) == rint(clamp(u, lo, hi)) for integer bounds; the low bits
            // of (clamped + 1.5 * 2^23) are its rounded value in two's complement
            const float cl_u = ZFOLD == 2 ? __builtin_amdgcn_fmed3f(u[r], -p.lo, -p.hi)
                                          : __builtin_amdgcn_fmed3f(u[r], p.lo, p.hi);
            c[r] = __float_as_int(cl_u + magic);
            if (ZFOLD == 0) c[r] += p.zr;
            if (OUT_KIND == kOutTable) {  // low byte of the sum: the code (ZFOLD: already code + 128)
              if (ZFOLD == 2) c[r] = ~c[r];
              c[r] = s_tab[(ZFOLD ? c[r] : c[r] + 128) & 255];
            }
          }
          if (VEC) {
            packed[g] = pack4(c[0], c[1], c[2], c[3]);
            if (ZFOLD == 2 && OUT_KIND != kOutTable) packed[g] = ~packed[g];
          } else {
            int8_t *o = reinterpret_cast<int8_t *>(wbase + row * row_bytes) + col;
#pragma unroll
            for (int r = 0; r < 4; ++r) o[r] = (int8_t)c[r];
          }
        }
      }
      if (I8 && VEC) {
        // lower half-wave holds channels 8g..8g+3, upper 8g+4..8g+7: after swapping
        // (upper's g0, lower's g2) and (upper's g1, lower's g3) the lower lane owns
        // channels 0..15 of this MFMA column and the upper lane 16..31
        const auto s02 = __builtin_amdgcn_permlane32_swap(packed[0], packed[2], false, false);
        const auto s13 = __builtin_amdgcn_permlane32_swap(packed[1], packed[3], false, false);
        const v4i q = {(int)s02[0], (int)s02[1], (int)s13[0], (int)s13[1]};
        *reinterpret_cast<v4i *>(slab + row * kSlabStride + a * 32 + half * 16) = q;
      }
    }
    if (VEC && !I8) store_slab<OUT_KIND, WROWS>(slab, wbase + a * 32 * ESZ, row_bytes, lane);
  }
  if (VEC && I8) store_slab<OUT_KIND, WROWS, 32 * TA>(slab, wbase, row_bytes, lane);
}

// Statistics epilogue (Sec. 3.3, Eq. 4-5 fused into the calibration forward): instead of storing
// Y_quant, the tile adds up, per channel, the five pivot-shifted sums of (Y_quant, Y_full) over
// its rows and writes them to partial[tile_m][stat][channel]; Y_quant never reaches memory and
// Y_full is read once.
//
// The accumulators hold a channel's rows spread over 32 lanes, the sums need them in one lane.
// So each wavefront works in 8 phases of (32 channels) x (PR = 16 * TB rows, half its wave tile):
// it writes the phase's Y_quant values to a private LDS slab, Y_full of the same rows and
// channels arrives in a second slab straight from global memory (global_load_lds, issued two
// phases ahead), and then lane (c, h) walks rows h, h + 2, ... of channel c in both slabs with
// fp64 sums.  Slab layout: row-major, 128 bytes per row, the 16-byte chunk position XORed with
// (row & 7): conflict-free for the 16-byte row writes and for the 4-byte column reads (the two
// half-waves read rows of different parity).  A wavefront owns four slabs (Y_quant, three of
// Y_full) of PR * 128 bytes in the ring, which the main loop has left.  Rows below `skip` (an edge
// tile shifted inwards: rows its upper neighbour already counts) contribute zeros.
template <bool MASKED, int PR>
__device__ __forceinline__ void stats_column_pass(const int8_t *yq_slab, const int8_t *yf_slab,
                                                  const int (&o4)[4], int h, float pq, float pf,
                                                  int row0, int skip, double (&sum)[kStats]) {
#pragma unroll 8
  for (int j = 0; j < PR / 2; ++j) {
    const int off = o4[j & 3] + (j >> 2) * 1024;
    float q = *reinterpret_cast<const float *>(yq_slab + off) - pq;
    float f = *reinterpret_cast<const float *>(yf_slab + off) - pf;
    if (MASKED) {
      const bool ok = row0 + 2 * j + h >= skip;
      q = ok ? q : 0.0f;
      f = ok ? f : 0.0f;
    }
    const double dq = (double)q, df = (double)f;
    sum[0] += dq;
    sum[1] += df;
    sum[2] = fma(dq, dq, sum[2]);
    sum[3] = fma(dq, df, sum[3]);
    sum[4] = fma(df, df, sum[4]);
  }
}

template <int TB, int WM>
__device__ __forceinline__ void stats_epilogue(const FwdParams &p, v16i (&acc)[4][TB], int8_t *smem,
                                               const float *s_mult, const float *s_fb,
                                               const float *s_rs, const float *s_pq,
                                               const float *s_pf, int64_t bm0, int bn0, int tile_m,
                                               int wave_m, int wave_n, int wave_s, int lane) {
  constexpr int WROWS = 32 * TB;    // token rows of the wave tile
  constexpr int PR = WROWS / 2;     // rows per phase
  constexpr int SLAB = PR * 128;    // bytes per slab
  constexpr int YL = PR / 8;        // Y_full loads per phase (8 rows x 128 bytes each)
  static_assert(2 * WM * 4 * SLAB <= 131072, "the slabs of all wavefronts fit the ring");
  const int l32 = lane & 31, half = lane >> 5;
  int8_t *wl = smem + wave_s * (4 * SLAB);  // this wavefront's slabs: Y_quant, three of Y_full
  int8_t *yq_slab = wl;
  const bool use_rs = p.sx_row != nullptr, use_fb = p.fbias != nullptr;
  // rows of this wave tile that the tile above already counts
  int64_t skip64 = (int64_t)tile_m * 256 - (bm0 + wave_m * WROWS);
  const int skip = skip64 < 0 ? 0 : (skip64 > WROWS ? WROWS : (int)skip64);

  // Y_full loads: one instruction = 8 rows x 128 bytes; lane (row lr, slot) fetches chunk slot ^ lr
  const int lr = lane >> 3, slot = lane & 7;
  const uint32_t yvo = (uint32_t)lr * (uint32_t)(p.ld_full * 4) + (uint32_t)((slot ^ lr) << 4);
  const char *yf_wave = reinterpret_cast<const char *>(p.y_full + (bm0 + wave_m * WROWS) * p.ld_full + bn0 +
                                                       wave_n * 128);
  auto issue_yf = [&](int phase) {
    const int a = phase >> 1, hb = phase & 1;
    const char *g = yf_wave + ((int64_t)hb * PR * p.ld_full + a * 32) * 4;
    int8_t *dst = wl + SLAB * (1 + phase % 3);
#pragma unroll
    for (int i = 0; i < YL; ++i)
      __builtin_amdgcn_global_load_lds(CWAC_GLOBAL_PTR(g + (int64_t)i * 8 * p.ld_full * 4 + yvo),
                                       CWAC_LDS_PTR(dst + i * 1024), 16, 0, 0);
  };
  float rs[TB];
#pragma unroll
  for (int b = 0; b < TB; ++b) rs[b] = s_rs[wave_m * WROWS + b * 32 + l32];
  // column pass: lane (channel c, row parity h); offsets of rows h, 2 + h, 4 + h, 6 + h
  const int c = l32, h = half;
  int o4[4];
#pragma unroll
  for (int jj = 0; jj < 4; ++jj) {
    const int r = 2 * jj + h;
    o4[jj] = r * 128 + (((c >> 2) ^ r) << 4) + (c & 3) * 4;
  }
  double tot[4][kStats];

  __builtin_amdgcn_s_waitcnt(s_waitcnt_imm(0, 0));  // only Y_full loads are counted from here on
  __builtin_amdgcn_sched_barrier(0);
  issue_yf(0);
  issue_yf(1);
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    float mu[4][4], fb[4][4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int cl = wave_n * 128 + a * 32 + 8 * g + 4 * half;  // channel inside the tile
      const float4 m4 = *reinterpret_cast<const float4 *>(s_mult + cl);
      mu[g][0] = m4.x; mu[g][1] = m4.y; mu[g][2] = m4.z; mu[g][3] = m4.w;
      const float4 f4 = *reinterpret_cast<const float4 *>(s_fb + cl);
      fb[g][0] = f4.x; fb[g][1] = f4.y; fb[g][2] = f4.z; fb[g][3] = f4.w;
    }
    const float pq = s_pq[wave_n * 128 + a * 32 + c], pf = s_pf[wave_n * 128 + a * 32 + c];
    double sum[kStats];
#pragma unroll
    for (int s = 0; s < kStats; ++s) sum[s] = 0.0;
#pragma unroll
    for (int hb = 0; hb < 2; ++hb) {
      const int phase = 2 * a + hb;
      // Y_quant of rows hb*PR .. +PR-1, channels a*32 .. +31 (the arithmetic of the fp32 output mode)
#pragma unroll
      for (int bb = 0; bb < TB / 2; ++bb) {
        const int b = (TB / 2) * hb + bb;
        const int row = bb * 32 + l32;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float u[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            float f = (float)acc[a][b][4 * g + r];
            if (use_rs) f = f * rs[b];
            float v = f * mu[g][r];
            if (use_fb) v = v + fb[g][r];
            u[r] = v;
          }
          *reinterpret_cast<float4 *>(yq_slab + row * 128 + (((2 * g + half) ^ (l32 & 7)) << 4)) =
              make_float4(u[0], u[1], u[2], u[3]);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      if (phase + 2 < 8) {
        issue_yf(phase + 2);
        __builtin_amdgcn_s_waitcnt(s_waitcnt_imm(2 * YL, 0));
      } else if (phase + 1 < 8) {
        __builtin_amdgcn_s_waitcnt(s_waitcnt_imm(YL, 0));
      } else {
        __builtin_amdgcn_s_waitcnt(s_waitcnt_imm(0, 0));
      }
      asm volatile("" ::: "memory");  // the slab reads below stay below the wait
      __builtin_amdgcn_sched_barrier(0);
      const int8_t *yf_slab = wl + SLAB * (1 + phase % 3);
      if (skip == 0)
        stats_column_pass<false, PR>(yq_slab, yf_slab, o4, h, pq, pf, hb * PR, skip, sum);
      else
        stats_column_pass<true, PR>(yq_slab, yf_slab, o4, h, pq, pf, hb * PR, skip, sum);
      __builtin_amdgcn_sched_barrier(0);  // the slabs are rewritten next: keep the reads above
    }
    // rows of both parities
#pragma unroll
    for (int s = 0; s < kStats; ++s) tot[a][s] = sum[s] + __shfl_xor(sum[s], 32, 64);
  }
  // The lower wave rows hand their sums to the top one through LDS (over the slabs, once every
  // wavefront has left them): exch[wave row - 1][wave column][a][stat][channel], fp64.
  double *exch = reinterpret_cast<double *>(smem);
  __syncthreads();
  if (wave_m > 0 && lane < 32) {
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int s = 0; s < kStats; ++s)
        exch[((((wave_m - 1) * 2 + wave_n) * 4 + a) * kStats + s) * 32 + c] = tot[a][s];
  }
  __syncthreads();
  if (wave_m == 0 && lane < 32) {
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int s = 0; s < kStats; ++s) {
        double t = tot[a][s];
#pragma unroll
        for (int r = 1; r < WM; ++r) t += exch[((((r - 1) * 2 + wave_n) * 4 + a) * kStats + s) * 32 + c];
        p.partial[((int64_t)tile_m * kStats + s) * p.n + bn0 + wave_n * 128 + a * 32 + c] = t;
      }
  }
}

template <int BM, int WM, int BK, int NSTAGE, int NCHUNK, int OUT_KIND, bool INT_ONLY, bool CONV = false,
          int BN = 256, int TA_ = 0>
__global__ __launch_bounds__((FastCfg<BM, WM, BK, NSTAGE, NCHUNK, BN, TA_>::NT), (BM / (32 * WM)) == 2 ? 2 : 1) void qlinear_fast_kernel(
    const FwdParams p) {
  using C = FastCfg<BM, WM, BK, NSTAGE, NCHUNK, BN, TA_>;
  constexpr int TB = C::TB, TA = C::TA;
  static_assert(OUT_KIND != kOutStats ||
                    (BM == 256 && BN == 256 && C::RING >= 131072 && C::STATS_LDS_BYTES <= 160 * 1024),
                "statistics epilogue: full-height tile, 128 KiB of ring for the slabs");
  extern __shared__ __attribute__((aligned(16))) int8_t smem[];
  int32_t *s_off = reinterpret_cast<int32_t *>(smem + C::RING);
  float *s_mult = reinterpret_cast<float *>(smem + C::RING + 1024);
  float *s_fb = reinterpret_cast<float *>(smem + C::RING + 2048);
  float *s_rs = reinterpret_cast<float *>(smem + C::RING + 3072);
  float *s_pq = reinterpret_cast<float *>(smem + C::RING + 4096);  // statistics epilogue only
  float *s_pf = reinterpret_cast<float *>(smem + C::RING + 5120);

  int tile_m, tile_n;
  tile_of_block(blockIdx.x, p.tiles_m, p.tiles_n, tile_m, tile_n);
  int64_t bm0 = (int64_t)tile_m * C::BM;
  if (bm0 > p.m - C::BM) bm0 = p.m - C::BM;
  int bn0 = tile_n * C::BN;
  if (bn0 > p.n - C::BN) bn0 = p.n - C::BN;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave % WM, wave_n = wave / WM;
  const int l32 = lane & 31, half = lane >> 5;
  CWAC_STAMP(0);

  // ---- epilogue parameters of this tile: issue their loads first (oldest in the load queue);
  // thread t < BN stages channel t (and thread t < BM row t)
  const int ptid = tid < BN ? tid : BN - 1;
  const int p_off = p.offset ? p.offset[bn0 + ptid] : 0;
  float p_mult = 0.0f, p_fb = 0.0f, p_rs = 1.0f;
  if (OUT_KIND == kOutFixed) {  // integer multiplier and shift travel in the two float slots
    p_mult = __int_as_float(p.m0[bn0 + ptid]);
    p_fb = __int_as_float(p.shift[bn0 + ptid]);
  } else if (OUT_KIND != CWAC_OUT_INT32) {
    p_mult = p.mult[bn0 + ptid];
  }
  if (OUT_KIND == kOutTable)  // 64 words of code table ride in the fp-bias slot (INT_ONLY: unused)
    p_fb = __int_as_float(reinterpret_cast<const int32_t *>(p.code_table)[tid & 63]);
  if (!INT_ONLY && OUT_KIND != CWAC_OUT_INT32 && OUT_KIND != kOutFixed) {
    if (p.fbias) p_fb = p.fbias[bn0 + ptid];
    if (p.sx_row && tid < BM) p_rs = p.sx_row[bm0 + tid];
  }
  // pivots of the shifted sums: the state's, or for the first batch of a state its row 0
  float p_pq = 0.0f, p_pf = 0.0f;
  if (OUT_KIND == kOutStats) {
    const StatsView sv = stats_view(const_cast<void *>(p.stats), p.n);
    if (*sv.n == 0) {
      p_pq = p.yq_row0[bn0 + ptid];
      p_pf = p.y_full[bn0 + ptid];
    } else {
      p_pq = sv.pivot_q[bn0 + ptid];
      p_pf = sv.pivot_f[bn0 + ptid];
    }
  }

  // ---- global -> LDS: wavefront `wave` owns a quarter of the rows of both panels (XROWS
  // activation rows, 64 weight rows), loads of RPL rows each; lane = (row lr, slot pc) inside a load.  Addresses are a
  // wave-uniform 64-bit base (tile origin + k) plus a per-lane 32-bit offset that never changes,
  // so the loop body issues the loads without any vector address arithmetic.
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  const int lr = lane / C::CPR, pc = lane % C::CPR;
  uint32_t xvo[C::LOADS_X], wvo[C::LOADS_W];
  // Convolution (implicit GEMM; c_in % BK == 0, so a stage lies inside ONE filter tap and the tap
  // is wave-uniform): row m = (b, oy, ox) reads the image at (oy * stride - pad + kh, ox * stride -
  // pad + kw).  Per load: xvo = byte offset of tap (0, 0), channel chunk included (it may lie
  // before the image: only taps inside it are dereferenced); xin = bit kh set where row kh of the
  // filter falls inside the image, bit 16 + kw likewise for its columns.
  uint32_t xin[C::LOADS_X];
#pragma unroll
  for (int i = 0; i < C::LOADS_X; ++i) {
    const int row = wave * C::XROWS + i * C::RPL + lr;
    if (CONV) {
      const int r = (int)bm0 + row, plane = p.cv_oh * p.cv_ow;
      const int b = r / plane, rem = r - b * plane;
      const int oy = rem / p.cv_ow, ox = rem - oy * p.cv_ow;
      const int iy0 = oy * p.cv_stride - p.cv_pad, ix0 = ox * p.cv_stride - p.cv_pad;
      // (mod 2^32: the sum with the tap offset is the true offset, below 2^31, for every tap inside)
      xvo[i] = ((uint32_t)(b * p.cv_h + iy0) * (uint32_t)p.cv_w + (uint32_t)ix0) * (uint32_t)p.cv_cin +
               (uint32_t)((pc ^ C::swz(row)) * 16);
      // taps kh with 0 <= iy0 + kh < h: kh in [max(0, -iy0), min(15, h - 1 - iy0)] (never empty)
      auto span = [](int lo, int hi) {
        lo = lo < 0 ? 0 : lo;
        hi = hi > 15 ? 15 : hi;
        return ((2u << hi) - 1u) & ~((1u << lo) - 1u);
      };
      xin[i] = span(-iy0, p.cv_h - 1 - iy0) | (span(-ix0, p.cv_w - 1 - ix0) << 16);
    } else {
      xvo[i] = (uint32_t)row * (uint32_t)p.ldx + (pc ^ C::swz(row)) * 16;
    }
  }
#pragma unroll
  for (int i = 0; i < C::LOADS_W; ++i) {
    const int row = wave * C::WLROWS + i * C::RPL + lr;
    wvo[i] = (uint32_t)row * (uint32_t)p.ldw + (pc ^ C::swz(row)) * 16;
  }
  const int8_t *xtile = CONV ? p.x : p.x + bm0 * p.ldx;
  const int8_t *wtile = p.w + (int64_t)bn0 * p.ldw;
  // convolution: the tap of the stage whose loads are being issued (wave-uniform; stages are
  // loaded in order, so it steps forward at the first chunk of every stage after stage 0)
  int tap_c = 0, tap_kw = 0, tap_kh = 0;
  uint32_t tap_off = 0;      // byte offset of the tap and channel block from tap (0, 0), channel 0 (mod 2^32)
  uint32_t tap_sel = 0x10001u;  // bit kh | bit 16 + kw
  const int8_t *pad = reinterpret_cast<const int8_t *>(kPadCodes.v) + (p.cv_pad4 & 255) * 16;

  // chunk c of a stage's 2*LOADS loads (activation loads first, then weight loads)
  auto issue_chunk = [&](int buf, int k0, int c) {
    int8_t *sx = smem + buf * C::STAGE + wave_s * C::XROWS * BK;
    int8_t *sw = smem + buf * C::STAGE + C::X_BYTES + wave_s * C::WLROWS * BK;
    const int8_t *xk = xtile + k0, *wk = wtile + k0;
    if (CONV && c == 0 && k0 != 0) {
      tap_c += BK;
      if (tap_c >= p.cv_cin) {
        tap_c = 0;
        if (++tap_kw == p.cv_kw) {
          tap_kw = 0;
          ++tap_kh;
        }
      }
      tap_off = ((uint32_t)tap_kh * (uint32_t)p.cv_w + (uint32_t)tap_kw) * (uint32_t)p.cv_cin + (uint32_t)tap_c;
      tap_sel = (1u << tap_kh) | (0x10000u << tap_kw);
    }
#pragma unroll
    for (int j = 0; j < C::CHUNK; ++j) {
      const int i = C::chunk_begin(c) + j;
      if (i >= C::chunk_begin(c + 1)) break;
      if (i < C::LOADS_X && CONV) {
        const bool inside = (xin[i] & tap_sel) == tap_sel;
        const int8_t *src = inside ? xtile + (uint32_t)(xvo[i] + tap_off) : pad;
        __builtin_amdgcn_global_load_lds(CWAC_GLOBAL_PTR(src), CWAC_LDS_PTR(sx + i * C::RPL * BK), 16, 0, 0);
      }
      else if (i < C::LOADS_X)
        __builtin_amdgcn_global_load_lds(CWAC_GLOBAL_PTR(xk + xvo[i]), CWAC_LDS_PTR(sx + i * C::RPL * BK), 16, 0, 0);
      else
        __builtin_amdgcn_global_load_lds(CWAC_GLOBAL_PTR(wk + wvo[i - C::LOADS_X]),
                                         CWAC_LDS_PTR(sw + (i - C::LOADS_X) * C::RPL * BK), 16, 0, 0);
    }
  };
  auto issue_stage = [&](int buf, int k0) {
#pragma unroll
    for (int c = 0; c < NCHUNK; ++c) issue_chunk(buf, k0, c);
  };

  // ---- LDS -> MFMA operand fragments (rows of a 32-row MFMA tile start at multiples of 16)
  const int swz_l = C::swz(l32);
  const int x_off = (wave_m * 32 * TB + l32) * BK;
  const int w_off = C::X_BYTES + (wave_n * (32 * TA) + l32) * BK;
  auto read_frags = [&](int buf, int kk, v4i(&fw)[TA], v4i(&fx)[TB]) {
    const int8_t *base = smem + buf * C::STAGE + (((2 * kk + half) ^ swz_l) << 4);
#pragma unroll
    for (int a = 0; a < TA; ++a) fw[a] = *reinterpret_cast<const v4i *>(base + w_off + a * 32 * BK);
#pragma unroll
    for (int b = 0; b < TB; ++b) fx[b] = *reinterpret_cast<const v4i *>(base + x_off + b * 32 * BK);
  };

  v16i acc[TA][TB];
  auto mma = [&](const v4i(&fw)[TA], const v4i(&fx)[TB]) {
#pragma unroll
    for (int a = 0; a < TA; ++a)
#pragma unroll
      for (int b = 0; b < TB; ++b)
        acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[a], fx[b], acc[a][b], 0, 0, 0);
  };
  // Scheduler hint for one k-step (TA * TB MFMAs, TA + TB LDS reads of the next step's fragments and,
  // when `loads`, one chunk of panel loads): the LDS reads go behind the first MFMAs one by one,
  // so that they land well before they are needed; the panel loads are spread over the remaining
  // MFMAs, so that their issue never holds up the matrix pipe.  (The 64 x 64 wave tile has as many
  // reads as MFMAs: there the loads follow the reads, one group behind every MFMA.)
  auto interleave = [&](bool loads) {
    constexpr int READS = TA + TB, REST = TA * TB - READS;
    if constexpr (REST <= 0) {
      constexpr int GRP = (C::CHUNK + TA * TB - 1) / (TA * TB);
#pragma unroll
      for (int i = 0; i < TA * TB; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, (READS + TA * TB - 1) / (TA * TB), 0);
        if (loads) __builtin_amdgcn_sched_group_barrier(0x020, GRP, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    } else {
#pragma unroll
      for (int i = 0; i < READS; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      if (loads) {
        constexpr int GRP = (C::CHUNK + REST - 1) / REST;  // loads behind each remaining MFMA
#pragma unroll
        for (int i = 0; i < REST; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x020, GRP, 0);
        }
      } else {
        __builtin_amdgcn_sched_group_barrier(0x008, REST, 0);
      }
      __builtin_amdgcn_sched_barrier(0);  // one k-step per scheduling region
    }
  };

  // ---- prologue: fill the ring, stage the parameters, start the accumulators at offset[n]
  const int stages = p.k / BK;
#pragma unroll
  for (int s = 0; s < NSTAGE; ++s)
    if (s < stages) issue_stage(s, s * BK);
  if (tid < BN) {
    s_off[tid] = p_off;
    s_mult[tid] = p_mult;
    s_fb[tid] = p_fb;
  }
  if (tid < BM) s_rs[tid] = p_rs;
  if (OUT_KIND == kOutStats && tid < BN) {
    s_pq[tid] = p_pq;
    s_pf[tid] = p_pf;
  }
  if (stages >= NSTAGE)
    __builtin_amdgcn_s_waitcnt(s_waitcnt_imm((NSTAGE - 1) * C::LPS, 0));  // stage 0 has landed
  else
    __builtin_amdgcn_s_waitcnt(s_waitcnt_imm(0, 0));
  __builtin_amdgcn_s_barrier();
#pragma unroll
  for (int a = 0; a < TA; ++a)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const v4i o = *reinterpret_cast<const v4i *>(s_off + wave_n * (32 * TA) + a * 32 + 8 * g + 4 * half);
#pragma unroll
      for (int b = 0; b < TB; ++b)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[a][b][4 * g + r] = o[r];
    }

  v4i fwA[TA], fxA[TB], fwB[TA], fxB[TB];
  read_frags(0, 0, fwA, fxA);

  // One stage: KK k-steps.  Before the MFMAs of the last one, everybody has fetched its last
  // fragments of this stage (its buffer is free) and the next stage has landed.  The loads of
  // stage s + NSTAGE go into the freed buffer in NCHUNK chunks, one per k-step: chunk 0 in this
  // stage's last k-step, chunk c in k-step c - 1 of the next stage.
  // STEADY: 1 <= s and s + NSTAGE < stages, so every chunk exists and the wait count is constant.
  auto stage_body = [&](int s, int buf, auto steady_tag) {
    constexpr bool STEADY = decltype(steady_tag)::value;
    const bool late_ok = STEADY || (s >= 1 && s - 1 + NSTAGE < stages);  // chunks >= 1 of stage s-1+NSTAGE
    const bool first_ok = STEADY || (s + NSTAGE < stages);               // chunk 0 of stage s+NSTAGE
#pragma unroll
    for (int kk = 0; kk + 1 < C::KK; ++kk) {
      const bool ld = (kk + 1 < NCHUNK) && late_ok;
      if (ld) issue_chunk((buf + NSTAGE - 1) % NSTAGE, (s - 1 + NSTAGE) * BK, kk + 1);
      if (kk & 1) {
        read_frags(buf, kk + 1, fwA, fxA);
        mma(fwB, fxB);
      } else {
        read_frags(buf, kk + 1, fwB, fxB);
        mma(fwA, fxA);
      }
      interleave(ld);
    }
    __builtin_amdgcn_sched_barrier(0);  // keep the MFMAs above on this side of the wait
    // loads issued so far reach stage min(stages, s + NSTAGE) - 1; stage s + 1 must have landed
    if (STEADY || s == 0) {
      if (STEADY || stages >= NSTAGE)
        __builtin_amdgcn_s_waitcnt(s_waitcnt_imm((NSTAGE - 2) * C::LPS, 0));
      else
        __builtin_amdgcn_s_waitcnt(s_waitcnt_imm(0, 0));
    } else {
      const int beyond = (s - 1 + NSTAGE < stages ? s - 1 + NSTAGE : stages - 1) - (s + 1);
      if (NSTAGE >= 3 && beyond >= NSTAGE - 2)
        __builtin_amdgcn_s_waitcnt(s_waitcnt_imm((NSTAGE - 2) * C::LPS, 0));
      else if (NSTAGE >= 4 && beyond == NSTAGE - 3)
        __builtin_amdgcn_s_waitcnt(s_waitcnt_imm((NSTAGE - 3) * C::LPS, 0));
      else
        __builtin_amdgcn_s_waitcnt(s_waitcnt_imm(0, 0));
    }
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    if (first_ok) issue_chunk(buf, (s + NSTAGE) * BK, 0);
    // KK is even: the last step's fragments are in B, the next stage's first go to A
    if (STEADY || s + 1 < stages) read_frags((buf + 1) % NSTAGE, 0, fwA, fxA);
    mma(fwB, fxB);
    interleave(first_ok);
  };

  int s = 0;
  CWAC_STAMP(1);
  if (stages > 0) stage_body(0, 0, std::false_type{});
  s = 1;
  // steady state, unrolled over the ring so that LDS offsets are compile-time constants
  for (; s % NSTAGE != 0 && s + NSTAGE < stages; ++s) stage_body(s, s % NSTAGE, std::true_type{});
  for (; s + 2 * NSTAGE <= stages; s += NSTAGE) {
#pragma unroll
    for (int j = 0; j < NSTAGE; ++j) stage_body(s + j, j, std::true_type{});
  }
  for (; s + NSTAGE < stages; ++s) stage_body(s, s % NSTAGE, std::true_type{});
  for (; s < stages; ++s) stage_body(s, s % NSTAGE, std::false_type{});

  CWAC_STAMP(2);
  if constexpr (OUT_KIND == kOutStats) {
    __builtin_amdgcn_s_barrier();  // every wavefront is done with the ring, which the slabs overlay
    stats_epilogue<TB, WM>(p, acc, smem, s_mult, s_fb, s_rs, s_pq, s_pf, bm0, bn0, tile_m, wave_m, wave_n,
                           wave_s, lane);
  } else {
    // whole-line stores need 16-byte aligned rows and tile origin (p.vec_store: base and row pitch)
    constexpr int ESZ = (OUT_KIND == CWAC_OUT_INT8 || OUT_KIND == kOutFixed || OUT_KIND == kOutTable) ? 1 : 4;
    const int vs = p.vec_store && (((bn0 * ESZ) & 15) == 0);
    if (vs) {
      if constexpr (OUT_KIND == CWAC_OUT_INT8 || OUT_KIND == kOutTable) {
        if (p.zr & 1)
          fast_epilogue<OUT_KIND, INT_ONLY, true, TB, WM, TA, 2>(p, acc, smem, s_mult, s_fb, s_rs, bm0, bn0, wave_m, wave_n, lane);
        else
          fast_epilogue<OUT_KIND, INT_ONLY, true, TB, WM, TA, 1>(p, acc, smem, s_mult, s_fb, s_rs, bm0, bn0, wave_m, wave_n, lane);
      } else {
        fast_epilogue<OUT_KIND, INT_ONLY, true, TB, WM, TA>(p, acc, smem, s_mult, s_fb, s_rs, bm0, bn0, wave_m, wave_n, lane);
      }
    } else
      fast_epilogue<OUT_KIND, INT_ONLY, false, TB, WM, TA>(p, acc, smem, s_mult, s_fb, s_rs, bm0, bn0, wave_m, wave_n, lane);
  }
  CWAC_STAMP(3);
#ifdef CWAC_V_STAMP
  __builtin_amdgcn_s_waitcnt(s_waitcnt_imm(0, 0));  // stores acknowledged
  CWAC_STAMP(4);
#endif
}

// Persistent form of the 256 x 256 tile of eight wavefronts (linear layers; int8 / fp32 / int32 output, the
// integer-only epilogue and the code-table epilogue):
// one workgroup per compute unit walks work items id = blockIdx.x + j * gridDim.x (the same XCD-aware
// tile order: ids congruent mod 8 stay on one XCD).  What a fresh workgroup pays per tile - kernel
// arguments, tile arithmetic, the round trip of the epilogue parameters and of the first panels,
// the gap between two workgroups on a compute unit: 2.5-3 us, a quarter of a K = 512 tile - is
// taken off the critical path:
//   * once the last fragments of item i have been fetched (the ring is free), the parameter loads of
//     item i + 1 (global -> LDS, into the other of two parameter blocks) and the panel loads of its
//     stage 0 (into ring stage 0) are issued, and travel while the epilogue of item i runs;
//   * the epilogue's transposition slabs therefore live behind stage 0 (they overlap stage 1 and
//     part of what the ring leaves free); after a barrier that ends the epilogue, stage 1 of item
//     i + 1 is issued.
// Panel loads are buffer loads (descriptor of the item's panel in scalar registers, extent = the
// item's own rows, scalar row / K offset): a wavefront's load i covers rows 8 i + lr of its share,
// and the swizzle of row r depends on bits 1-3 of r only, so two per-lane offsets (i even, i odd)
// serve all loads of a panel and stay live across the epilogue instead of eight.
// The last round.  With T tiles on G workgroups the last R = T mod G tiles would keep that many compute
// units busy for a whole tile while the others idle.  When R <= G / 2, each of them is split into two
// work items of 128 tokens x 256 channels (the same eight wavefronts, each 32 tokens x 128 channels: one
// activation fragment per k-step instead of two), so the last round takes about half a tile; when
// R <= G / 4, into four items of 64 tokens x 256 channels (the eight wavefronts as 2 x 4, each 32 tokens x
// 64 channels).  Items [0, F) are the full tiles, [F, F + pieces * R) the pieces (F = T - R).
template <int OUT_KIND, bool INT_ONLY, int LOADERS>
__global__ __launch_bounds__(512, 1) void qlinear_persist_kernel(const FwdParams p) {
  static_assert(LOADERS == 8 || LOADERS == 4, "wavefronts that issue the panel loads");
  constexpr int SHARES = 8 / LOADERS;  // 32-row shares of a panel per loading wavefront
  using C = FastCfg<256, 4, 128, 2, 2, 256>;
  constexpr int BK = 128, NSTAGE = 2;
  constexpr int kSlabBase = C::STAGE;                         // slabs: behind stage 0
  constexpr int kParamBase = 160 * 1024 - 2 * C::PARAM_BYTES;  // two parameter blocks: the top 8 KiB
  static_assert(C::LOADS_X == 4 && C::LOADS_W == 4 && C::RPL == 8 && C::KK == 4, "load schedule below");
  static_assert(kSlabBase + C::NWAVES * 64 * kSlabStride <= kParamBase, "slabs clear of the parameters");
  extern __shared__ __attribute__((aligned(16))) int8_t smem[];
  // parameter block b (items alternate between the two): offset, mult, fbias [256 channels], row scale [256 rows]
  auto param_block = [&](int b) { return smem + kParamBase + b * C::PARAM_BYTES; };

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  const int lr = lane >> 3, pc = lane & 7;
  // per-lane byte offset inside a load: row lr of the load's 8 rows, chunk pc ^ swz(row); loads with
  // odd i sit 8 rows further, which flips bit 2 of the swizzle (a wavefront's share starts at a
  // multiple of 16 rows, which does not touch bits 1-3)
  const int sw0 = (lr >> 1) & 7;
  const uint32_t xv0 = (uint32_t)lr * (uint32_t)p.ldx + (uint32_t)((pc ^ sw0) << 4);
  const uint32_t xv1 = (uint32_t)lr * (uint32_t)p.ldx + (uint32_t)((pc ^ sw0 ^ 4) << 4);
  const uint32_t wv0 = (uint32_t)lr * (uint32_t)p.ldw + (uint32_t)((pc ^ sw0) << 4);
  const uint32_t wv1 = (uint32_t)lr * (uint32_t)p.ldw + (uint32_t)((pc ^ sw0 ^ 4) << 4);
  const uint32_t xstep = 8u * (uint32_t)p.ldx, wstep = 8u * (uint32_t)p.ldw;

  const int total = p.tiles_m * p.tiles_n;
  const int stages = p.k / BK;
  // work items: full tiles, then the halves of the last round's tiles
  const int G = (int)gridDim.x;
  const int rest = total % G;
  // quarters only in the form for short K loops (LOADERS = 8): the long-K form runs at the register limit without them
  constexpr bool kQuarters = LOADERS == 8;
  const int pieces = rest == 0 ? 1 : (kQuarters && 4 * rest <= G ? 4 : (2 * rest <= G ? 2 : 1));  // of a last-round tile
  const int n_split = pieces > 1 ? rest : 0;
  const int n_full = total - n_split;
  const int n_items = n_full + pieces * n_split;

  // state of the item whose panels are being loaded / multiplied
  int64_t bm0 = 0;
  int bn0 = 0;
  int kind = 0;  // 0: whole tile (256 tokens), 1: half (128), 2: quarter (64)
  __amdgpu_buffer_rsrc_t xdesc, wdesc;
  // The parameters go global -> LDS directly as well (4 bytes per lane, 256 bytes per wavefront load):
  // wavefronts 2a and 2a + 1 fetch the four quarters of array a (0 offset, 1 mult, 2 fbias, 3 row scale).
  // An absent offset vector reads as zeros (both blocks cleared once); absent fbias / row scales are
  // never read by the epilogue.
  const int p_arr = wave_s >> 1, p_elem = (wave_s & 1) * 128 + lane;
  if (!p.offset && tid < 512) {
    reinterpret_cast<int32_t *>(param_block(tid >> 8))[tid & 255] = 0;
  }
  // the code table (64 words) rides in the fp-bias slot of both blocks, which that epilogue leaves unused
  if (OUT_KIND == kOutTable && tid < 128)
    reinterpret_cast<int32_t *>(param_block(tid >> 6) + 2048)[tid & 63] =
        reinterpret_cast<const int32_t *>(p.code_table)[tid & 63];

  // item origin and kind, panel descriptors, parameter loads into block pb, panel loads of stage 0
  auto open_item = [&](int id, int pb) {
    const int sub = id - n_full;  // index among the pieces
    const int tile = id < n_full ? id : n_full + sub / pieces;
    kind = id < n_full ? 0 : (pieces == 4 ? 2 : 1);
    int tile_m, tile_n;
    tile_of_block(tile, p.tiles_m, p.tiles_n, tile_m, tile_n);
    bm0 = (int64_t)tile_m * 256;
    if (bm0 > p.m - 256) bm0 = p.m - 256;
    const int rows = 256 >> kind;
    if (kind) bm0 += (sub % pieces) * rows;
    bn0 = tile_n * 256;
    if (bn0 > p.n - 256) bn0 = p.n - 256;
    const uint32_t x_extent = (uint32_t)((uint64_t)(rows - 1) * (uint64_t)p.ldx + (uint64_t)p.k);
    const uint32_t w_extent = (uint32_t)((uint64_t)255 * (uint64_t)p.ldw + (uint64_t)p.k);
    xdesc = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(p.x + bm0 * p.ldx), 0, (int)x_extent, 0x00020000);
    wdesc = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(p.w + (int64_t)bn0 * p.ldw), 0, (int)w_extent,
                                              0x00020000);
    const void *src = nullptr;
    if (p_arr == 0) src = p.offset ? p.offset + bn0 : nullptr;
    if (p_arr == 1 && OUT_KIND != CWAC_OUT_INT32) src = p.mult + bn0;
    if (OUT_KIND == kOutFixed) {  // integer multiplier and shift travel in the two float slots
      if (p_arr == 1) src = p.m0 + bn0;
      if (p_arr == 2) src = p.shift + bn0;
    }
    if (!INT_ONLY && OUT_KIND != CWAC_OUT_INT32) {
      if (p_arr == 2) src = p.fbias ? p.fbias + bn0 : nullptr;
      // a half item has 128 rows, a quarter 64: only the first of the two wavefronts of this array loads,
      // for a quarter only its first 64 lanes' worth (nothing beyond the item's rows is read)
      if (p_arr == 3 && !(kind && (wave_s & 1))) src = p.sx_row ? p.sx_row + bm0 : nullptr;
    }
    if (src) {  // wave-uniform
      int8_t *dst = param_block(pb) + p_arr * 1024 + (wave_s & 1) * 512;
      const int n_loads = (p_arr == 3 && kind == 2) ? 1 : 2;
#pragma unroll
      for (int j = 0; j < 2; ++j)
        if (j < n_loads)
          __builtin_amdgcn_global_load_lds(CWAC_GLOBAL_PTR(static_cast<const int32_t *>(src) + p_elem + j * 64),
                                           CWAC_LDS_PTR(dst + j * 256), 4, 0, 0);
    }
  };
  // Panel loads of one stage.  A share is 32 rows (four loads) of a 256-row panel, 16 rows (two loads) of a
  // half item's 128 activation rows, 8 rows (one load) of a quarter's 64.  LOADERS = 8: every wavefront loads its own share.  LOADERS = 4: only
  // wavefronts 0-3 - one per SIMD - issue loads, each for shares w and w + 4: a direct-to-LDS load holds up
  // the issuing wavefront's MFMAs for some tens of cycles, and with one loading wavefront per SIMD the other
  // one keeps the matrix pipe fed meanwhile (with all eight loading, both wavefronts of a SIMD stall at about
  // the same time).  That pays in long K loops (measured, the two forms alternated
  // on workload 5's layers: -1 to -3.5 % time at K = 4096 .. 11008); in short ones the loading wavefronts'
  // doubled share at the start of every tile takes the gain back (within +-1 % at K = 512 .. 3072), so the
  // launcher picks by K; cwac_tuning.persist_loaders forces either form.
  const bool loader = wave_s < LOADERS;
  // Ring geometry by item kind.  A whole tile: two stages of 64 KiB (activation panel, weight panel).  A piece has
  // so little MFMA work per stage that with two stages the loads' round trip would set its pace (a stage's loads
  // can only go out once the stage two back has been read), so pieces run three compact stages of (rows + 256)
  // x 128 bytes: 48 KiB (half), 40 KiB (quarter).  Stage 0 starts at the same place for every kind.
  auto x_bytes = [](int kd) { return (256 >> kd) * BK; };
  auto stage_bytes = [](int kd) { return ((256 >> kd) + 256) * BK; };
  auto issue_x = [&](int buf, int k0, int kd) {
    if (!loader) return;
#pragma unroll
    for (int h = 0; h < SHARES; ++h) {
      const int share = wave_s + LOADERS * h;
      if (kQuarters && kd == 2) {
        // rows 8 share .. 8 share + 7: bit 3 of the row, which the swizzle reads, is the share's parity
        int8_t *dst = smem + buf * stage_bytes(2) + share * (8 * BK);
        const uint32_t row0 = (uint32_t)(share * 8) * (uint32_t)p.ldx + (uint32_t)k0;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(xdesc, CWAC_LDS_PTR(dst), 16, (int)((share & 1) ? xv1 : xv0),
                                                 (int)row0, 0, 0);
      } else if (kd == 0) {
        int8_t *dst = smem + buf * C::STAGE + share * (32 * BK);
        const uint32_t row0 = (uint32_t)(share * 32) * (uint32_t)p.ldx + (uint32_t)k0;
#pragma unroll
        for (int i = 0; i < 4; ++i)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(xdesc, CWAC_LDS_PTR(dst + i * 8 * BK), 16,
                                                   (int)((i & 1) ? xv1 : xv0), (int)(row0 + (uint32_t)i * xstep), 0, 0);
      } else {
        int8_t *dst = smem + buf * stage_bytes(1) + share * (16 * BK);
        const uint32_t row0 = (uint32_t)(share * 16) * (uint32_t)p.ldx + (uint32_t)k0;
#pragma unroll
        for (int i = 0; i < 2; ++i)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(xdesc, CWAC_LDS_PTR(dst + i * 8 * BK), 16,
                                                   (int)((i & 1) ? xv1 : xv0), (int)(row0 + (uint32_t)i * xstep), 0, 0);
      }
    }
  };
  auto issue_w = [&](int buf, int k0, int kd) {
    if (!loader) return;
#pragma unroll
    for (int h = 0; h < SHARES; ++h) {
      const int share = wave_s + LOADERS * h;
      int8_t *dst = smem + buf * stage_bytes(kd) + x_bytes(kd) + share * (32 * BK);
      const uint32_t row0 = (uint32_t)(share * 32) * (uint32_t)p.ldw + (uint32_t)k0;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(wdesc, CWAC_LDS_PTR(dst + i * 8 * BK), 16, (int)((i & 1) ? wv1 : wv0),
                                                 (int)(row0 + (uint32_t)i * wstep), 0, 0);
    }
  };
  const int swz_l = C::swz(l32);

  int id = blockIdx.x;
  if (id >= n_items) return;
  int pb = 0;  // parameter block of the item being multiplied
  bool more = true;

  // One work item from the barrier that ended the previous one to the barrier that ends this one;
  // TB = 32-token MFMA tiles per wavefront: 2 (full tile) or 1 (half).
  auto run_item = [&](auto tb_tag, auto ta_tag) {
    constexpr int TB = decltype(tb_tag)::value;
    constexpr int TA = decltype(ta_tag)::value;       // 32-channel MFMA tiles per wavefront: 4, or 2 in a quarter
    constexpr int KIND = TA == 2 ? 2 : (TB == 1 ? 1 : 0);
    constexpr bool HF = KIND != 0;
    constexpr int WM = TA == 2 ? 2 : 4;               // wavefronts along the tokens
    constexpr int LPS = KIND == 2 ? 5 : (KIND == 1 ? 6 : 8);  // panel loads per wavefront and stage
    constexpr int XB = (256 >> KIND) * BK, STG = XB + 256 * BK;  // bytes of a stage's activation panel, of a stage
    const int wave_m = wave % WM, wave_n = wave / WM;
    const int x_off = (wave_m * 32 * TB + l32) * BK;
    const int w_off = XB + (wave_n * (32 * TA) + l32) * BK;
    auto read_frags = [&](int buf, int kk, v4i(&fw)[TA], v4i(&fx)[TB]) {
      const int8_t *base = smem + buf * STG + (((2 * kk + half) ^ swz_l) << 4);
      fw[0] = *reinterpret_cast<const v4i *>(base + w_off);
#pragma unroll
      for (int b = 0; b < TB; ++b) fx[b] = *reinterpret_cast<const v4i *>(base + x_off + b * 32 * BK);
#pragma unroll
      for (int a = 1; a < TA; ++a) fw[a] = *reinterpret_cast<const v4i *>(base + w_off + a * 32 * BK);
    };
    v16i acc[TA][TB];
    auto mma = [&](const v4i(&fw)[TA], const v4i(&fx)[TB]) {
#pragma unroll
      for (int a = 0; a < TA; ++a)
#pragma unroll
        for (int b = 0; b < TB; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[a], fx[b], acc[a][b], 0, 0, 0);
    };
    // one k-step for the scheduler: TA * TB MFMAs, the TA + TB LDS reads of the next step's fragments
    // spread behind the first of them, and (loads: how many) panel loads behind the last two
    auto interleave = [&](int loads) {
      if constexpr (!HF) {
#pragma unroll
        for (int i = 0; i < TA + TB; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        if (loads) {
#pragma unroll
          for (int i = 0; i < 2; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);
          }
        } else {
          __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        }
      } else if constexpr (KIND == 2) {  // two MFMAs, three reads: left to the scheduler
      } else {  // four MFMAs, five reads
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        if (loads == 4) __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);
        if (loads == 2) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (loads == 4) __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);
        if (loads == 2) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    };
    v4i fwA[TA], fxA[TB], fwB[TA], fxB[TB];
    // Stage s of this item (buffer s % 2), as in the one-tile kernel: the weight loads of stage
    // s + 1 go out in the first k-step, the activation loads of stage s + 2 in the last one, behind the
    // barrier that frees this stage's buffer.
    auto stage_body = [&](int s, int buf, auto steady_tag) {
      constexpr bool STEADY = decltype(steady_tag)::value;
      const bool late_ok = STEADY || (s >= 1 && s + 1 < stages);
      const bool first_ok = STEADY || (s + NSTAGE < stages);
#pragma unroll
      for (int kk = 0; kk + 1 < C::KK; ++kk) {
        const bool ld = kk == 0 && late_ok;
        if (ld) issue_w(buf ^ 1, (s + 1) * BK, KIND);
        if (kk & 1) {
          read_frags(buf, kk + 1, fwA, fxA);
          mma(fwB, fxB);
        } else {
          read_frags(buf, kk + 1, fwB, fxB);
          mma(fwA, fxA);
        }
        interleave(ld ? 4 : 0);
      }
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_waitcnt(s_waitcnt_imm(0, 0));  // stage s + 1 has landed (nothing else is in flight)
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
      if (first_ok) issue_x(buf, (s + NSTAGE) * BK, KIND);
      if (STEADY || s + 1 < stages) read_frags(buf ^ 1, 0, fwA, fxA);
      mma(fwB, fxB);
      interleave(first_ok ? (HF ? 2 : 4) : 0);
    };

    CWAC_STAMPT(id, 0);
    const int32_t *s_off = reinterpret_cast<const int32_t *>(param_block(pb));
    // First k-step of an item.  The accumulators START at offset[n] (the integer offset add of Eq. 10 costs
    // nothing): the first MFMA of every accumulator takes the offsets of its 32 channels - four 16-byte LDS
    // reads that land in 16 consecutive registers - as its C operand, so no register is initialised by hand.
    auto first_kstep = [&]() {
      read_frags(0, 1, fwB, fxB);
#pragma unroll
      for (int a = 0; a < TA; ++a) {
        v16i pat;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const v4i o = *reinterpret_cast<const v4i *>(s_off + wave_n * (32 * TA) + a * 32 + 8 * g + 4 * half);
#pragma unroll
          for (int r = 0; r < 4; ++r) pat[4 * g + r] = o[r];
        }
#pragma unroll
        for (int b = 0; b < TB; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fwA[a], fxA[b], pat, 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    };
    auto kstep = [&](int buf, int kk) {  // MFMAs of k-step kk, fragments of k-step kk + 1
      if (kk & 1) {
        read_frags(buf, kk + 1, fwA, fxA);
        mma(fwB, fxB);
      } else {
        read_frags(buf, kk + 1, fwB, fxB);
        mma(fwA, fxA);
      }
      interleave(0);
    };
    if constexpr (KIND == 0) {
    // stage 0 of this item is in flight (or has landed), as are its parameters; ring stage 1, the slabs
    // and the other parameter block are free (barrier at the end of the previous epilogue)
    if (stages > 1) {
      issue_x(1, BK, KIND);
      issue_w(1, BK, KIND);
      // all but stage 1: stage 0 and the parameters have landed (a loading wavefront has its shares of
      // stage 1 in flight, the others nothing)
      if (loader)
        __builtin_amdgcn_s_waitcnt(s_waitcnt_imm(SHARES * LPS, 0));
      else
        __builtin_amdgcn_s_waitcnt(s_waitcnt_imm(0, 0));
    } else {
      __builtin_amdgcn_s_waitcnt(s_waitcnt_imm(0, 0));
    }
    __builtin_amdgcn_s_barrier();
    read_frags(0, 0, fwA, fxA);
    CWAC_STAMPT(id, 1);
    // stage 0: the loads of stage 1 are out already (above), so only its last k-step issues loads.
    {
      first_kstep();
#pragma unroll
      for (int kk = 1; kk + 1 < C::KK; ++kk) kstep(0, kk);
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_waitcnt(s_waitcnt_imm(0, 0));
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
      const bool first_ok = NSTAGE < stages;
      if (first_ok) issue_x(0, NSTAGE * BK, KIND);
      if (stages > 1) read_frags(1, 0, fwA, fxA);
      mma(fwB, fxB);
      interleave(first_ok ? 4 : 0);
    }
    int s = 1;
    for (; s + 2 * NSTAGE <= stages; s += NSTAGE) {  // steady state, unrolled over the ring
      stage_body(s, 1, std::true_type{});
      stage_body(s + 1, 0, std::true_type{});
    }
    for (; s + NSTAGE < stages; ++s) stage_body(s, s & 1, std::true_type{});
    for (; s < stages; ++s) stage_body(s, s & 1, std::false_type{});
    } else {
      // ---- a piece: three stages.  Stage 0 is in flight (or has landed), as are the parameters; stages 1 and 2
      // go out now (the rest of the ring, the slabs and the other parameter block are free: barrier at the end
      // of the previous epilogue).  Memory operations return in order, so "at most N outstanding" means that
      // everything older than the newest N has arrived.
      if (stages > 1) {
        issue_x(1, BK, KIND);
        issue_w(1, BK, KIND);
      }
      if (stages > 2) {
        issue_x(2, 2 * BK, KIND);
        issue_w(2, 2 * BK, KIND);
      }
      if (loader && stages > 2)
        __builtin_amdgcn_s_waitcnt(s_waitcnt_imm(2 * SHARES * LPS, 0));
      else if (loader && stages > 1)
        __builtin_amdgcn_s_waitcnt(s_waitcnt_imm(SHARES * LPS, 0));
      else
        __builtin_amdgcn_s_waitcnt(s_waitcnt_imm(0, 0));
      __builtin_amdgcn_s_barrier();
      read_frags(0, 0, fwA, fxA);
      CWAC_STAMPT(id, 1);
      // stage s in ring buffer s % 3: three k-steps, then - every wavefront has fetched the stage's last
      // fragments, and stage s + 1 has landed once at most the loads of stage s + 2 are outstanding - the
      // barrier that frees the buffer for stage s + 3, whose loads go out under the last k-step.
      auto piece_stage = [&](int s, int buf, auto first_tag) {
        const int nbuf = buf == 2 ? 0 : buf + 1;
        if constexpr (decltype(first_tag)::value)
          first_kstep();
        else
          kstep(buf, 0);
        kstep(buf, 1);
        kstep(buf, 2);
        __builtin_amdgcn_sched_barrier(0);
        if (loader && s + 2 < stages)
          __builtin_amdgcn_s_waitcnt(s_waitcnt_imm(SHARES * LPS, 0));
        else
          __builtin_amdgcn_s_waitcnt(s_waitcnt_imm(0, 0));
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        if (s + 3 < stages) {
          issue_x(buf, (s + 3) * BK, KIND);
          issue_w(buf, (s + 3) * BK, KIND);
        }
        if (s + 1 < stages) read_frags(nbuf, 0, fwA, fxA);
        mma(fwB, fxB);
        interleave(0);
      };
      piece_stage(0, 0, std::true_type{});
      int buf = 1;
#pragma unroll 1
      for (int s = 1; s < stages; ++s) {
        piece_stage(s, buf, std::false_type{});
        buf = buf == 2 ? 0 : buf + 1;
      }
    }

    // ---- the ring is free (every wavefront fetched its last fragments before the last barrier):
    // open the next item - its parameter loads and the panel loads of its stage 0 travel under this
    // item's epilogue.  The epilogue reads this item's origin, so that is kept aside first.
    CWAC_STAMPT(id, 2);
    const int64_t e_bm0 = bm0;
    const int e_bn0 = bn0;
    const int next = id + G;
    more = next < n_items;
    if (more) {
      open_item(next, pb ^ 1);
      issue_x(0, 0, kind);
      issue_w(0, 0, kind);
    }
    __builtin_amdgcn_sched_barrier(0);
    {
      const float *s_mult = reinterpret_cast<const float *>(param_block(pb) + 1024);
      const float *s_fb = reinterpret_cast<const float *>(param_block(pb) + 2048);
      const float *s_rs = reinterpret_cast<const float *>(param_block(pb) + 3072);
      // the lane index the epilogue derives its addresses from is made opaque per item: otherwise all of
      // that lane arithmetic is hoisted out of the item loop and lives (spilled) across the main loop
      int lane_e = lane;
      asm volatile("" : "+v"(lane_e));
      constexpr int ESZ = (OUT_KIND == CWAC_OUT_INT8 || OUT_KIND == kOutFixed || OUT_KIND == kOutTable) ? 1 : 4;
      const int vs = p.vec_store && (((e_bn0 * ESZ) & 15) == 0);
      if (vs) {
        if constexpr (OUT_KIND == CWAC_OUT_INT8 || OUT_KIND == kOutTable) {
          if (p.zr & 1)
            fast_epilogue<OUT_KIND, INT_ONLY, true, TB, WM, TA, 2>(p, acc, smem + kSlabBase, s_mult, s_fb, s_rs, e_bm0,
                                                                   e_bn0, wave_m, wave_n, lane_e);
          else
            fast_epilogue<OUT_KIND, INT_ONLY, true, TB, WM, TA, 1>(p, acc, smem + kSlabBase, s_mult, s_fb, s_rs, e_bm0,
                                                                   e_bn0, wave_m, wave_n, lane_e);
        } else {
          fast_epilogue<OUT_KIND, INT_ONLY, true, TB, WM, TA>(p, acc, smem + kSlabBase, s_mult, s_fb, s_rs, e_bm0, e_bn0,
                                                              wave_m, wave_n, lane_e);
        }
      } else
        fast_epilogue<OUT_KIND, INT_ONLY, false, TB, WM, TA>(p, acc, smem + kSlabBase, s_mult, s_fb, s_rs, e_bm0, e_bn0,
                                                             wave_m, wave_n, lane_e);
    }
    CWAC_STAMPT(id, 3);
    CWAC_STAMPT(id, 4);
    id = next;
  };

  // ---- first item: nothing was prefetched
  open_item(id, 0);
  issue_x(0, 0, kind);
  issue_w(0, 0, kind);
  while (true) {
    const int kd = kind;  // of the item about to run (open_item inside run_item overwrites it)
    if (kQuarters && kd == 2) {
      if constexpr (kQuarters) run_item(std::integral_constant<int, 1>{}, std::integral_constant<int, 2>{});
    } else if (kd == 1)
      run_item(std::integral_constant<int, 1>{}, std::integral_constant<int, 4>{});
    else
      run_item(std::integral_constant<int, 2>{}, std::integral_constant<int, 4>{});
    if (!more) break;
    pb ^= 1;
    __builtin_amdgcn_s_barrier();  // every wavefront is done with the slabs and that item's parameter block
  }
}

template <int OUT_KIND, bool INT_ONLY, int LOADERS>
cwac_status launch_persist_loaders(const FwdParams &p, int workgroups, hipStream_t st) {
  constexpr int LDS = 160 * 1024;
  static const hipError_t attr =
      hipFuncSetAttribute(reinterpret_cast<const void *>(&qlinear_persist_kernel<OUT_KIND, INT_ONLY, LOADERS>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
  if (attr != hipSuccess) return CWAC_E_LAUNCH;
  qlinear_persist_kernel<OUT_KIND, INT_ONLY, LOADERS><<<dim3((unsigned)workgroups), 512, LDS, st>>>(p);
  return launch_status();
}

constexpr int kLoaderWavesFromK = 4096;  // K from which four wavefronts issue all panel loads (see the kernel)

template <int OUT_KIND, bool INT_ONLY>
cwac_status launch_persist_one(const FwdParams &p, int workgroups, int loaders, hipStream_t st) {
  if (loaders == 0) loaders = p.k >= kLoaderWavesFromK ? 4 : 8;  // else: the caller's override (cwac_tuning)
  return loaders == 4 ? launch_persist_loaders<OUT_KIND, INT_ONLY, 4>(p, workgroups, st)
                      : launch_persist_loaders<OUT_KIND, INT_ONLY, 8>(p, workgroups, st);
}

// The persistent kernel on a 256 x 256 tiling of the layer: one workgroup per compute unit (fewer
// when there are fewer tiles).  out_kind: CWAC_OUT_INT8 | CWAC_OUT_FP32 | CWAC_OUT_INT32 | kOutFixed | kOutTable.
cwac_status launch_persist(FwdParams p, int out_kind, bool int_only, int max_workgroups, int loaders, hipStream_t st) {
  const size_t esz = (out_kind == CWAC_OUT_INT8 || out_kind == kOutFixed || out_kind == kOutTable) ? 1 : 4;
  p.vec_store = aligned(p.out, 16) && ((p.ldo * esz) % 16) == 0;
  p.tiles_m = (int)ceil_div(p.m, 256);
  p.tiles_n = (int)ceil_div(p.n, 256);
  const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
  if (tiles > 0x7fffffff) return CWAC_E_LAUNCH;
  int device = 0, cus = 0;
  if (hipGetDevice(&device) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || cus < 1)
    return CWAC_E_LAUNCH;
  int wgs = (int)(tiles < cus ? tiles : cus);
  if (max_workgroups > 0 && max_workgroups < wgs) wgs = max_workgroups;  // cwac_tuning.persist_workgroups
  if (out_kind == CWAC_OUT_INT8)
    return int_only ? launch_persist_one<CWAC_OUT_INT8, true>(p, wgs, loaders, st)
                    : launch_persist_one<CWAC_OUT_INT8, false>(p, wgs, loaders, st);
  if (out_kind == CWAC_OUT_FP32) return launch_persist_one<CWAC_OUT_FP32, false>(p, wgs, loaders, st);
  if (out_kind == kOutFixed) return launch_persist_one<kOutFixed, true>(p, wgs, loaders, st);
  if (out_kind == kOutTable) return launch_persist_one<kOutTable, true>(p, wgs, loaders, st);
  return launch_persist_one<CWAC_OUT_INT32, false>(p, wgs, loaders, st);
}

template <int BM, int WM, int BK, int NSTAGE, int NCHUNK, int OUT_KIND, bool INT_ONLY, bool CONV = false,
          int BN = 256, int TA = 0>
cwac_status launch_one(const FwdParams &p, dim3 grid, hipStream_t st) {
  using C = FastCfg<BM, WM, BK, NSTAGE, NCHUNK, BN, TA>;
  constexpr int LDS = OUT_KIND == kOutStats ? C::STATS_LDS_BYTES : C::LDS_BYTES;
  static const hipError_t attr = hipFuncSetAttribute(
      reinterpret_cast<const void *>(&qlinear_fast_kernel<BM, WM, BK, NSTAGE, NCHUNK, OUT_KIND, INT_ONLY, CONV, BN, TA>),
      hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
  if (attr != hipSuccess) return CWAC_E_LAUNCH;
  qlinear_fast_kernel<BM, WM, BK, NSTAGE, NCHUNK, OUT_KIND, INT_ONLY, CONV, BN, TA><<<grid, C::NT, LDS, st>>>(p);
  return launch_status();
}

template <int BM, int WM, int BK, int NSTAGE, int NCHUNK, bool CONV = false, int BN = 256, int TA = 0>
cwac_status launch_cfg(FwdParams p, int out_kind, bool int_only, hipStream_t st) {
  p.tiles_m = (int)ceil_div(p.m, BM);
  p.tiles_n = (int)ceil_div(p.n, BN);
  const int64_t blocks = (int64_t)p.tiles_m * p.tiles_n;
  if (blocks > 0x7fffffff) return CWAC_E_LAUNCH;
  const dim3 grid((unsigned)blocks);
  if constexpr (!CONV) {
    if (out_kind == kOutFixed)
      return launch_one<BM, WM, BK, NSTAGE, NCHUNK, kOutFixed, true, false, BN, TA>(p, grid, st);
  }
  if (out_kind == CWAC_OUT_INT8)
    return int_only ? launch_one<BM, WM, BK, NSTAGE, NCHUNK, CWAC_OUT_INT8, true, CONV, BN, TA>(p, grid, st)
                    : launch_one<BM, WM, BK, NSTAGE, NCHUNK, CWAC_OUT_INT8, false, CONV, BN, TA>(p, grid, st);
  if (out_kind == CWAC_OUT_FP32)
    return launch_one<BM, WM, BK, NSTAGE, NCHUNK, CWAC_OUT_FP32, false, CONV, BN, TA>(p, grid, st);
  return launch_one<BM, WM, BK, NSTAGE, NCHUNK, CWAC_OUT_INT32, false, CONV, BN, TA>(p, grid, st);
}

template <int BM, int WM, int BK, int NSTAGE>
cwac_status launch_table_cfg(FwdParams p, hipStream_t st) {
  p.tiles_m = (int)ceil_div(p.m, BM);
  p.tiles_n = (int)ceil_div(p.n, 256);
  const int64_t blocks = (int64_t)p.tiles_m * p.tiles_n;
  if (blocks > 0x7fffffff) return CWAC_E_LAUNCH;
  return launch_one<BM, WM, BK, NSTAGE, 2, kOutTable, true>(p, dim3((unsigned)blocks), st);
}

}  // namespace

cwac_status launch_fast_table(FwdParams p, int shape, int max_workgroups, int loaders, hipStream_t st) {
  p.vec_store = aligned(p.out, 16) && (p.ldo % 16) == 0;
  // the tiles of the plain int8 forward of a layer with n >= 256, by the same rule: the persistent
  // 256 x 256 tile, the same tile with one workgroup per tile, or the 128-token pair
  if (shape == CWAC_SHAPE_AUTO) shape = fast_linear_shape(p.m, p.n, p.k, 1);
  if ((p.k % 128) != 0 || shape == CWAC_SHAPE_128_128) shape = CWAC_SHAPE_128_PAIR;
  if (shape == CWAC_SHAPE_128_PAIR) return launch_table_cfg<128, 2, 64, 3>(p, st);
  if (shape == CWAC_SHAPE_256_PERSIST) return launch_persist(p, kOutTable, true, max_workgroups, loaders, st);
  return launch_table_cfg<256, 4, 128, 2>(p, st);
}

bool fast_prefers_half_tile(int64_t m, int n, int k, int out_bytes) {
  // Cost model fitted to a sweep of 140 layer shapes per output width (microseconds per compute
  // unit).  A 256-token tile (eight wavefronts) costs a + b k.  Two 128-token workgroups sharing a
  // compute unit overlap each other's prologue and epilogue but move 1.5x the panel bytes per MAC:
  // the pair costs c + d k, a lone one e + f k.  Tiles run in rounds of 256 (512) at a time.
  // The constants grow with the width of the output element (more bytes for the epilogue to store).
  const bool wide = out_bytes > 1;
  const double a = wide ? 10.7 : 6.05, b = wide ? 0.01112 : 0.01136;
  const double c = wide ? 7.56 : 4.18, d = 0.01559;
  const double e = wide ? 9.71 : 5.64, f = wide ? 0.00411 : 0.00524;
  const int64_t t_full = ceil_div(m, 256) * ceil_div(n, 256), t_half = ceil_div(m, 128) * ceil_div(n, 256);
  if (t_half < 160) return false;
  const double cost_full = (double)ceil_div(t_full, 256) * (a + b * k);
  const int64_t rest = t_half % 512;
  const double cost_half =
      (double)(t_half / 512) * (c + d * k) + (rest == 0 ? 0.0 : rest <= 256 ? e + f * k : c + d * k);
  // int8 output: on 24 shapes within 6 % of a tie, launched back to back until the clock had settled, the
  // full tile was the faster one on 20, by 5 % on average - the half tile has to win by that much
  return cost_half < (wide ? 1.0 : 0.95) * cost_full;
}

bool fast_prefers_quarter_tile(int64_t m, int n) {
  // Layers with too few 128 x 256 tiles to occupy the chip: a tile's duration is the K loop of one
  // wavefront, so 128 x 128 tiles of four 64 x 64 wavefronts (half the MFMAs per wavefront and K step,
  // twice the tiles) finish sooner.  Thresholds from measurements on LLM layer shapes at 256-2048
  // tokens and ResNet-50 stage 5: ahead from 96 such tiles on, until 160 half tiles exist.
  const int64_t t_half = ceil_div(m, 128) * ceil_div(n, 256), t_q = ceil_div(m, 128) * ceil_div(n, 128);
  return n >= 128 && t_half < 160 && t_q >= 96;
}

cwac_status launch_fast(FwdParams p, int out_kind, bool int_only, const Tune &tune, hipStream_t st) {
  int shape = tune.shape;
  const size_t esz = (out_kind == CWAC_OUT_INT8 || out_kind == kOutFixed) ? 1 : 4;
  p.vec_store = aligned(p.out, 16) && ((p.ldo * esz) % 16) == 0;
  // layers narrower than 256 channels: 256 tokens x 128 (64) channels, four wavefronts (4 x 1) of
  // 64 x 128 (64 x 64), 64-byte K steps, two workgroups per compute unit
  if (p.n < 128) return launch_cfg<256, 4, 64, 3, 2, false, 64>(p, out_kind, int_only, st);
  if (p.n < 256) return launch_cfg<256, 4, 64, 3, 2, false, 128>(p, out_kind, int_only, st);
  // `shape` (cwac_tuning, same results): CWAC_SHAPE_256_PERSIST is the 256 x 256 tile of eight wavefronts
  // on persistent workgroups (the choice for large layers), _256_8W the same tile with one workgroup per
  // tile, _256_4W_K128 / _K64 that tile with four wavefronts and that K step and ring depth, _128_PAIR
  // the 128-token tile, two workgroups of four wavefronts per compute unit, _128_128 the quarter tile.
  const int out_bytes = (out_kind == CWAC_OUT_INT8 || out_kind == kOutFixed) ? 1 : 4;
  if (shape == CWAC_SHAPE_AUTO) shape = fast_linear_shape(p.m, p.n, p.k, out_bytes);
  if (shape == CWAC_SHAPE_128_128) return launch_cfg<128, 2, 64, 3, 2, false, 128, 2>(p, out_kind, int_only, st);
  if ((p.k % 128) != 0) shape = CWAC_SHAPE_128_PAIR;  // K a multiple of 64 only: the tile that steps K by 64
  if (shape == CWAC_SHAPE_128_PAIR) return launch_cfg<128, 2, 64, 3, 2>(p, out_kind, int_only, st);
  if (shape == CWAC_SHAPE_256_4W_K64) return launch_cfg<256, 2, 64, 4, 2>(p, out_kind, int_only, st);
  if (shape == CWAC_SHAPE_256_8W) return launch_cfg<256, 4, 128, 2, 2>(p, out_kind, int_only, st);
  if (shape == CWAC_SHAPE_256_4W_K128) return launch_cfg<256, 2, 128, 2, 2>(p, out_kind, int_only, st);
  // CWAC_SHAPE_256_PERSIST: the eight-wavefront 256 x 256 tile on persistent workgroups
  return launch_persist(p, out_kind, int_only, tune.persist_workgroups, tune.persist_loaders, st);
}

int fast_linear_shape(int64_t m, int n, int k, int out_bytes) {
  // The automatic tile shape of a linear layer with n >= 256, from measurements on the ViT / Swin / LLM
  // layer shapes (K 512 .. 11008, 196 .. 3072 tiles of 256 x 256).
  //  * Few tiles and a long K loop: 128 x 128 tiles (fast_prefers_quarter_tile).
  //  * Less than a round of 256 x 256 tiles: the 128-token tile where the one-tile cost model prefers it.
  //  * Otherwise the persistent 256 x 256 tile (which splits the tiles of a thin last round in two).
  //    With 4-byte outputs and a short K loop the tile's store burst weighs as much as its K loop:
  //    when, on top, the last round leaves a good part of the chip idle, the 128 x 128 tile (three
  //    workgroups per compute unit, four times as many tiles, stores spread out) finishes sooner.
  if (fast_prefers_quarter_tile(m, n)) return CWAC_SHAPE_128_128;
  if ((k % 128) != 0) return CWAC_SHAPE_128_PAIR;
  const int64_t t256 = ceil_div(m, 256) * ceil_div(n, 256);
  if (t256 < 160) return fast_prefers_half_tile(m, n, k, out_bytes) ? CWAC_SHAPE_128_PAIR : CWAC_SHAPE_256_PERSIST;
  const double fill = (double)t256 / (double)(256 * ceil_div(t256, 256));  // busy share of the rounds
  if (out_bytes > 1 && k <= 1024 && fill < 0.85) return CWAC_SHAPE_128_128;
  return CWAC_SHAPE_256_PERSIST;
}

bool fast_conv_ok(const FwdParams &p, int64_t image_bytes) {
  return p.m >= kFastTile && p.m < ((int64_t)1 << 31) && p.n >= 64 && (p.k % 64) == 0 &&
         (p.cv_cin % 64) == 0 && image_bytes < ((int64_t)1 << 31);
}

cwac_status launch_fast_conv(FwdParams p, int out_kind, bool int_only, int shape, hipStream_t st) {
  const size_t esz = out_kind == CWAC_OUT_INT8 ? 1 : 4;
  p.vec_store = aligned(p.out, 16) && ((p.ldo * esz) % 16) == 0;
  if (p.n < 128) return launch_cfg<256, 4, 64, 3, 2, true, 64>(p, out_kind, int_only, st);
  if (p.n < 256) return launch_cfg<256, 4, 64, 3, 2, true, 128>(p, out_kind, int_only, st);
  // a stage must lie inside one filter tap: the 256-token tile steps K by 128, the 128-token tile by 64
  const bool full_ok = (p.cv_cin % 128) == 0;
  // `shape` (cwac_tuning, same results): _256_8W | _128_PAIR | _128_128; the four-wavefront forms of
  // the 256-token tile are not instantiated for the convolution and leave the choice automatic
  if (shape == CWAC_SHAPE_128_128 || (shape == CWAC_SHAPE_AUTO && fast_prefers_quarter_tile(p.m, p.n)))
    return launch_cfg<128, 2, 64, 3, 2, true, 128, 2>(p, out_kind, int_only, st);
  bool half = !full_ok || fast_prefers_half_tile(p.m, p.n, p.k, (int)esz) ||
              ceil_div(p.m, 256) * ceil_div(p.n, 256) < 160;
  if (shape == CWAC_SHAPE_128_PAIR) half = true;
  if (shape == CWAC_SHAPE_256_8W && full_ok) half = false;
  if (half) return launch_cfg<128, 2, 64, 3, 2, true>(p, out_kind, int_only, st);
  return launch_cfg<256, 4, 128, 2, 2, true>(p, out_kind, int_only, st);
}

cwac_status launch_fast_stats(FwdParams p, int waves, hipStream_t st) {
  p.tiles_m = (int)ceil_div(p.m, 256);
  p.tiles_n = (int)ceil_div(p.n, 256);
  p.vec_store = 0;
  const int64_t blocks = (int64_t)p.tiles_m * p.tiles_n;
  if (blocks > 0x7fffffff) return CWAC_E_LAUNCH;
  // four wavefronts per tile add the fp64 sums up in another order than eight (cwac_tuning.stats_waves)
  if (waves == 4) return launch_one<256, 2, 128, 2, 2, kOutStats, false>(p, dim3((unsigned)blocks), st);
  return launch_one<256, 4, 128, 2, 2, kOutStats, false>(p, dim3((unsigned)blocks), st);
}

}  // namespace cwac

#ifdef CWAC_V_STAMP
extern "C" int cwac_debug_stamps(void *dst_device, size_t bytes, void *stream) {
  return (int)hipMemcpyFromSymbolAsync(dst_device, HIP_SYMBOL(cwac::g_stamps), bytes, 0, hipMemcpyDeviceToDevice,
                                       (hipStream_t)stream);
}
#endif
