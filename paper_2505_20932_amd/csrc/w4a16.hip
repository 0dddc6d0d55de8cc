// Weight-only INT4 linear layer with the CWAC epilogue (LLM setting of Sec. 4.4: group-wise
// asymmetric 4-bit weights, group size 128, binary16 activations; compensation of Sec. 3.3
// folded into the epilogue as in Sec. 3.4), plus its quantizer, weight re-ordering and fold.
//
// Forward kernel: 256 x 256 output tile, eight wavefronts (2 x 4, each 128 tokens x 64 channels =
// 4 x 2 tiles of v_mfma_f32_32x32x16_f16, 128 fp32 accumulators per lane), one workgroup per
// compute unit, two wavefronts per SIMD.  Measured on this device with register-resident operands:
// beside one such MFMA (32 cycles of the matrix pipe) a SIMD issues about five vector ALU
// instructions per wavefront for free when two wavefronts share it, but only about three when one
// wavefront has it alone - and the weight expansion needs five per MFMA.
//   * Activation panels go global -> LDS directly (global_load_lds_dwordx4); one K stage is one
//     quantization group (128 channels = 256 bytes per row, 64 KiB per stage, two stages).  The
//     bank swizzle (16-byte chunk position XOR row & 15) is applied on the global-address side.
//   * Weights never touch LDS: they were re-ordered once into the order in which a wavefront's
//     lanes consume them, so each wavefront streams its own 4-bit codes with contiguous 1 KiB
//     loads straight into registers, one stage ahead, together with the group's scale and
//     zero-point, and expands them to binary16 MFMA operands right before use:
//     (code | 0x6400) is the binary16 number 1024 + code, so (1024 + c) - (1024 + z) and
//     fma(1024 + 16 c, 1/16, -(64 + z)) give c - z exactly with one packed instruction each,
//     and one packed multiply by the scale is the single rounding of RN16(s * (c - z)).
//   * Epilogue in registers: acc * mult[n] + fbias[n] (two fp32 operations), conversion to
//     binary16, transposition through a wave-private LDS slab, whole 128-byte line stores.
// The same kernel with 128-token tiles (two token blocks per wavefront) serves batches whose
// 128-token tiles fit the chip in one round; small batches (a decoding step, and up to 256
// tokens while passes of 32 rows are estimated to be cheaper) take the weight-streaming kernel
// further down.
#include <hip/hip_runtime.h>


#include "qlinear_common.h"

namespace cwac {
namespace {

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) u4 GU4;        // in global memory (not a generic address)
typedef __attribute__((address_space(1))) uint32_t GU32;

#define CWAC_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#define CWAC_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void *)(p))

constexpr int wait_imm(int vmcnt, int lgkmcnt) {
  // gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] << 14 ; expcnt = 7 (no wait)
  return (vmcnt & 15) | (7 << 4) | ((lgkmcnt & 15) << 8) | (((vmcnt >> 4) & 3) << 14);
}

constexpr int kGroup = CWAC_W4_GROUP;  // input channels per scale / zero-point = per K stage
constexpr int kThreads = 256;

// ------------------------------------------------------------------------------------------
// Quantizer (Eq. 1-2, b = 4, per group): one wavefront per (output channel, group), two
// weights per lane.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void w4_quantize_kernel(const float *__restrict__ w, int64_t ldw,
                                                               int n, int groups,
                                                               uint8_t *__restrict__ codes,
                                                               uint16_t *__restrict__ scales,
                                                               uint8_t *__restrict__ zeros) {
  const int lane = threadIdx.x & 63;
  const int64_t task = (int64_t)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  if (task >= (int64_t)n * groups) return;
  const int r = (int)(task / groups), g = (int)(task - (int64_t)r * groups);
  const float2 v = *reinterpret_cast<const float2 *>(w + (int64_t)r * ldw + g * kGroup + 2 * lane);
  const float mn = wave_min(fminf(v.x, v.y)), mx = wave_max(fmaxf(v.x, v.y));
  const _Float16 sh = (_Float16)__fdiv_rn(mx - mn, 15.0f);  // round to nearest even
  uint16_t sb = __builtin_bit_cast(uint16_t, sh);
  if (sb < 0x0400u) sb = 0x0400u;   // zero or subnormal: 2^-14
  if (sb >= 0x7c00u) sb = 0x7bffu;  // never infinite
  const float s = (float)__builtin_bit_cast(_Float16, sb);
  float zf = rintf(__fdiv_rn(-mn, s));
  zf = fminf(fmaxf(zf, 0.0f), 15.0f);
  float c0 = rintf(__fdiv_rn(v.x, s)) + zf, c1 = rintf(__fdiv_rn(v.y, s)) + zf;
  c0 = fminf(fmaxf(c0, 0.0f), 15.0f);
  c1 = fminf(fmaxf(c1, 0.0f), 15.0f);
  const int64_t kk = (int64_t)groups * kGroup;
  *reinterpret_cast<uint16_t *>(codes + (int64_t)r * kk + g * kGroup + 2 * lane) =
      (uint16_t)((uint32_t)c0 | ((uint32_t)c1 << 8));
  if (lane == 0) {
    scales[(int64_t)r * groups + g] = sb;
    zeros[(int64_t)r * groups + g] = (uint8_t)zf;
  }
}

// ------------------------------------------------------------------------------------------
// Re-ordering into the forward kernel's streaming layout: one thread per output dword.
// dword index = (((n / 32) * (k / 64) + kb) * 64 + lane) * 4 + j, lane = 32 * h + n % 32; it
// holds the codes of input channels 64 * kb + 16 * j + 8 * h + e (e = 0..7) at nibble p(e).
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void w4_pack_kernel(const uint8_t *__restrict__ codes, int n, int k,
                                                           uint32_t *__restrict__ packed) {
  const int64_t total = (int64_t)n * (k / 8);
  for (int64_t d = (int64_t)blockIdx.x * kThreads + threadIdx.x; d < total;
       d += (int64_t)gridDim.x * kThreads) {
    const int j = (int)(d & 3), lane = (int)((d >> 2) & 63);
    const int64_t blk = d >> 8;
    const int kb64 = k / 64;
    const int nb = (int)(blk / kb64), kb = (int)(blk - (int64_t)nb * kb64);
    const int row = nb * 32 + (lane & 31), h = lane >> 5;
    const uint8_t *src = codes + (int64_t)row * k + kb * 64 + j * 16 + h * 8;
    const uint2 raw = *reinterpret_cast<const uint2 *>(src);  // 8 codes, 8-byte aligned
    uint32_t word = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t c = ((e < 4 ? raw.x : raw.y) >> (8 * (e & 3))) & 15u;
      const int p = (e >> 1) + 4 * (e & 1);  // (0, 4, 1, 5, 2, 6, 3, 7)
      word |= c << (4 * p);
    }
    packed[d] = word;
  }
}

__global__ __launch_bounds__(kThreads) void w4_pack_sz_kernel(const uint16_t *__restrict__ scales,
                                                              const uint8_t *__restrict__ zeros, int n,
                                                              int groups, uint32_t *__restrict__ sz) {
  const int64_t total = (int64_t)n * groups;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * kThreads) {
    const int g = (int)(i / n), r = (int)(i - (int64_t)g * n);
    sz[i] = (uint32_t)scales[(int64_t)r * groups + g] | ((uint32_t)zeros[(int64_t)r * groups + g] << 16);
  }
}

// Fold (Sec. 3.4 for a layer without requantization): mult = alpha, fbias = alpha * b + beta.
__global__ __launch_bounds__(kThreads) void fold_weight_only_kernel(const float *__restrict__ alpha,
                                                                    const float *__restrict__ beta,
                                                                    const float *__restrict__ bias, int n,
                                                                    float *__restrict__ mult,
                                                                    float *__restrict__ fbias) {
  const int c = blockIdx.x * kThreads + threadIdx.x;
  if (c >= n) return;
  const double a = alpha ? (double)alpha[c] : 1.0;
  const double be = beta ? (double)beta[c] : 0.0;
  const double b = bias ? (double)bias[c] : 0.0;
  mult[c] = (float)a;
  fbias[c] = (float)(__dadd_rn(__dmul_rn(a, b), be));
}

// ------------------------------------------------------------------------------------------
// Forward
// ------------------------------------------------------------------------------------------
struct W4Params {
  const char *x;  // binary16 [m, k]
  int64_t ldx_bytes;
  const u4 *wp;
  const uint32_t *sz;
  int64_t m;
  int n, k;
  const float *mult;
  const float *fbias;
  char *out;
  int64_t ldo;
  int tiles_m, tiles_n;
};

constexpr int kFwdThreads = 512;  // 8 wavefronts: 2 per SIMD
constexpr int kTA = 2;            // MFMA row blocks per wavefront: 64 channels
constexpr int kSlabStride = 144;
// Tile of WM x (8 / WM) wavefronts, each TB token blocks x kTA channel blocks of 32: (32 * TB * WM) tokens x
// (512 / WM) channels.  WM = 2: 256 channels x 256 tokens (TB = 4), or 128 tokens (TB = 2) for batches of a few
// hundred tokens, where one row of 256-token tiles would leave most compute units idle.  WM = 1 (TB = 4): 512
// channels x 128 tokens - every wavefront expands weights that no other wavefront of the tile needs (with WM = 2
// the two wavefronts of a channel block expand the same codes), so the tile spends half the vector work per MFMA.
template <int TB, int WM = 2>
struct W4Cfg {
  static_assert(WM == 1 || WM == 2, "wavefronts along the tokens");
  static constexpr int BM = 32 * TB * WM;
  static constexpr int BN = 64 * (8 / WM);
  static constexpr int STAGE_BYTES = BM * 256;  // BM rows x 128 binary16
  static constexpr int RING = 2 * STAGE_BYTES;
  static constexpr int XROWS = BM / 8;          // activation rows one wavefront fetches per stage
  static constexpr int XLOADS = XROWS / 4;      // global_load_lds per wavefront and stage (4 rows x 256 bytes each)
  static constexpr int SLAB_ROWS = 32 * TB;
  static constexpr int SLAB_BYTES = SLAB_ROWS * kSlabStride;
  // epilogue parameters sit behind the ring and the slabs
  static constexpr int PARAMS = 8 * SLAB_BYTES > RING ? 8 * SLAB_BYTES : RING;
  static constexpr int LDS = PARAMS + 2 * BN * 4;
  static_assert(LDS <= 160 * 1024, "LDS budget of one compute unit");
};

__device__ __forceinline__ h2 as_h2(uint32_t u) { return __builtin_bit_cast(h2, u); }

// Scale and zero-point of one weight row in the three forms the expansion needs.
struct GroupConst {
  h2 s, zlo, zhi;  // (s, s), (1024 + z) twice, (64 + z) twice
};
__device__ __forceinline__ GroupConst group_const(uint32_t sz) {
  GroupConst g;
  const uint32_t z = sz >> 16;
  g.s = as_h2((sz & 0xffffu) * 0x00010001u);
  g.zlo = as_h2(0x64006400u + z * 0x00010001u);  // 1024 + z: one unit per mantissa step
  g.zhi = as_h2(0x54005400u + z * 0x00100010u);  // 64 + z: sixteen mantissa steps per unit
  return g;
}

// Eight codes (one dword in the packed order) -> the MFMA operand of 8 consecutive input channels.
__device__ __forceinline__ h8 expand8(uint32_t w, const GroupConst &g) {
  const uint32_t w8 = w >> 8;
  const h2 t0 = as_h2((w & 0x000f000fu) | 0x64006400u);   // 1024 + c      channels 0, 1
  const h2 t1 = as_h2((w & 0x00f000f0u) | 0x64006400u);   // 1024 + 16 c   channels 2, 3
  const h2 t2 = as_h2((w8 & 0x000f000fu) | 0x64006400u);  //               channels 4, 5
  const h2 t3 = as_h2((w8 & 0x00f000f0u) | 0x64006400u);  //               channels 6, 7
  const h2 sixteenth = {(_Float16)0.0625f, (_Float16)0.0625f};
  const h2 d0 = t0 - g.zlo;                                        // c - z, exact
  const h2 d1 = __builtin_elementwise_fma(t1, sixteenth, -g.zhi);  // c - z, exact
  const h2 d2 = t2 - g.zlo;
  const h2 d3 = __builtin_elementwise_fma(t3, sixteenth, -g.zhi);
  const h2 r0 = d0 * g.s, r1 = d1 * g.s, r2 = d2 * g.s, r3 = d3 * g.s;  // the one rounding
  return h8{r0.x, r0.y, r1.x, r1.y, r2.x, r2.y, r3.x, r3.y};
}

// The same with the two masks in scalar registers and the exponent pattern in a vector register,
// which lets the compiler fuse every mask-and-set into one v_and_or_b32 (13 instead of 17
// instructions); pays where the expansion is what bounds the kernel.
struct ExpandConst {
  uint32_t mask_lo, mask_hi;  // wave-uniform
  uint32_t magic;             // per lane (the same value in all)
};
__device__ __forceinline__ ExpandConst expand_const() {
  ExpandConst c;
  c.mask_lo = 0x000f000fu;
  c.mask_hi = 0x00f000f0u;
  c.magic = 0x64006400u;
  asm volatile("" : "+s"(c.mask_lo), "+s"(c.mask_hi));  // opaque: not folded back into literals
  asm volatile("" : "+v"(c.magic));
  return c;
}
__device__ __forceinline__ h8 expand8(uint32_t w, const GroupConst &g, const ExpandConst &c) {
  const uint32_t w8 = w >> 8;
  const h2 t0 = as_h2((w & c.mask_lo) | c.magic);
  const h2 t1 = as_h2((w & c.mask_hi) | c.magic);
  const h2 t2 = as_h2((w8 & c.mask_lo) | c.magic);
  const h2 t3 = as_h2((w8 & c.mask_hi) | c.magic);
  const h2 sixteenth = {(_Float16)0.0625f, (_Float16)0.0625f};
  const h2 d0 = t0 - g.zlo;
  const h2 d1 = __builtin_elementwise_fma(t1, sixteenth, -g.zhi);
  const h2 d2 = t2 - g.zlo;
  const h2 d3 = __builtin_elementwise_fma(t3, sixteenth, -g.zhi);
  const h2 r0 = d0 * g.s, r1 = d1 * g.s, r2 = d2 * g.s, r3 = d3 * g.s;
  return h8{r0.x, r0.y, r1.x, r1.y, r2.x, r2.y, r3.x, r3.y};
}

template <int OUT_KIND, int ROWS>
__device__ __forceinline__ void store_slab(const int8_t *slab, char *gbase, int64_t row_bytes,
                                           int64_t rows_left, int lane) {
  const int rd_row = lane >> 3, rd_chunk = lane & 7;
#pragma unroll
  for (int i = 0; i < ROWS / 8; ++i) {
    const int row = i * 8 + rd_row;
    const u4 v = *reinterpret_cast<const u4 *>(slab + row * kSlabStride + rd_chunk * 16);
    u4 *dst = reinterpret_cast<u4 *>(gbase + row * row_bytes + rd_chunk * 16);
    if (row < rows_left) {
      // fp32 results (the calibration forward's Y_quant) are far larger than the caches and are
      // streamed out; binary16 results stay cacheable for the layer that consumes them
      if (OUT_KIND == CWAC_OUT_FP32)
        __builtin_nontemporal_store(v, dst);
      else
        *dst = v;
    }
  }
}

// Accumulator element 4*g + r of tile (a, b): channel n = bn0 + wave_n*64 + a*32 + 8*g + 4*half + r,
// token m = bm0 + wave_m*32*TB + b*32 + l32.  Each wavefront transposes its 32*TB rows x 128 bytes
// through a private LDS slab (row stride 144 bytes) and writes whole 128-byte lines: binary16
// output = all 64 channels of the wave tile in one slab, fp32 output = one slab per MFMA column.
template <int OUT_KIND, int TB, int WM>
__device__ __forceinline__ void w4_epilogue(const W4Params &p, v16f (&acc)[kTA][TB], int8_t *smem,
                                            const float *s_mult, const float *s_fb, int64_t bm0, int bn0,
                                            int wave_m, int wave_n, int lane) {
  constexpr int ESZ = OUT_KIND == CWAC_OUT_FP16 ? 2 : 4;
  constexpr int APS = OUT_KIND == CWAC_OUT_FP16 ? 2 : 1;  // MFMA columns per 128-byte slab row
  const int l32 = lane & 31, half = lane >> 5;
  const int wave = wave_m + WM * wave_n;
  int8_t *slab = smem + wave * W4Cfg<TB, WM>::SLAB_BYTES;
  const int64_t row_bytes = p.ldo * ESZ;
  const int64_t wrow0 = bm0 + wave_m * 32 * TB;
  char *wbase = p.out + (wrow0 * p.ldo + bn0 + wave_n * 64) * ESZ;
  const int64_t rows_left = p.m - wrow0;
#pragma unroll
  for (int a = 0; a < kTA; ++a) {
    float mu[4][4], fb[4][4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int cl = wave_n * 64 + a * 32 + 8 * g + 4 * half;  // channel inside the tile
      const float4 m4 = *reinterpret_cast<const float4 *>(s_mult + cl);
      mu[g][0] = m4.x; mu[g][1] = m4.y; mu[g][2] = m4.z; mu[g][3] = m4.w;
      const float4 f4 = *reinterpret_cast<const float4 *>(s_fb + cl);
      fb[g][0] = f4.x; fb[g][1] = f4.y; fb[g][2] = f4.z; fb[g][3] = f4.w;
    }
#pragma unroll
    for (int b = 0; b < TB; ++b) {
      const int row = b * 32 + l32;  // row inside the wave tile
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float u[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float v = acc[a][b][4 * g + r] * mu[g][r];  // mult == NULL: 1
          u[r] = v + fb[g][r];                              // fbias == NULL: +0
        }
        const int col = (a % APS) * 32 + 8 * g + 4 * half;  // channel inside the slab row
        if (OUT_KIND == CWAC_OUT_FP16) {
          const h2 lo = {(_Float16)u[0], (_Float16)u[1]}, hi = {(_Float16)u[2], (_Float16)u[3]};
          *reinterpret_cast<uint2 *>(slab + row * kSlabStride + col * 2) =
              make_uint2(__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi));
        } else {
          *reinterpret_cast<float4 *>(slab + row * kSlabStride + col * 4) = make_float4(u[0], u[1], u[2], u[3]);
        }
      }
    }
    if (a % APS == APS - 1)
      store_slab<OUT_KIND, 32 * TB>(slab, wbase + (a / APS) * 128, row_bytes, rows_left, lane);
  }
}

template <int OUT_KIND, int TB, int WM>
__global__ __launch_bounds__(kFwdThreads) void w4a16_kernel(const W4Params p) {
  using Cfg = W4Cfg<TB, WM>;
  constexpr int BN = Cfg::BN;
  constexpr int kXLoads = Cfg::XLOADS, kStageBytes = Cfg::STAGE_BYTES, kParams = Cfg::PARAMS;
  extern __shared__ __attribute__((aligned(16))) int8_t smem[];
  float *s_mult = reinterpret_cast<float *>(smem + kParams);
  float *s_fb = reinterpret_cast<float *>(smem + kParams + BN * 4);

  int tile_m, tile_n;
  tile_of_block(blockIdx.x, p.tiles_m, p.tiles_n, tile_m, tile_n);
  const int64_t bm0 = (int64_t)tile_m * Cfg::BM;  // row edges: clamped loads, predicated stores
  int bn0 = tile_n * BN;
  if (bn0 > p.n - BN) bn0 = p.n - BN;  // channel edge: tile shifted inwards (n % 32 == 0)

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave % WM, wave_n = wave / WM;  // WM x (8 / WM) wavefronts of 32*TB tokens x 64 channels
  const int l32 = lane & 31, half = lane >> 5;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);

  float p_mult = 1.0f, p_fb = 0.0f;
  if (tid < BN) {
    if (p.mult) p_mult = p.mult[bn0 + tid];
    if (p.fbias) p_fb = p.fbias[bn0 + tid];
  }

  // ---- activations, global -> LDS: wavefront `wave` owns XROWS consecutive rows, fetched 4
  // rows per load; lane = (row lr, slot pc) fetches 16-byte chunk pc ^ (row & 15) of its row
  const int lr = lane >> 4, pc = lane & 15;
  uint32_t xvo[kXLoads];
#pragma unroll
  for (int i = 0; i < kXLoads; ++i) {
    const int row = wave * Cfg::XROWS + i * 4 + lr;
    int64_t grow = bm0 + row;
    if (grow > p.m - 1) grow = p.m - 1;
    xvo[i] = (uint32_t)((grow - bm0) * p.ldx_bytes) + (uint32_t)((pc ^ (row & 15)) << 4);
  }
  const char *xtile = p.x + bm0 * p.ldx_bytes;
  // a wave-uniform 64-bit address that the compiler must keep in scalar registers, so that loads
  // take the (scalar base + 32-bit lane offset) form and need no vector address arithmetic
  auto uniform = [](const char *q) {
    const uint64_t v = reinterpret_cast<uint64_t>(q);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const char *>(((uint64_t)hi << 32) | lo);
  };
  auto issue_x = [&](int buf, int stage) {
    int8_t *sx = smem + buf * kStageBytes + wave_s * Cfg::XROWS * 256;
    const char *xk = uniform(xtile + (int64_t)stage * 256);
#pragma unroll
    for (int i = 0; i < kXLoads; ++i)
      __builtin_amdgcn_global_load_lds(CWAC_GLOBAL_PTR(xk + xvo[i]), CWAC_LDS_PTR(sx + i * 1024), 16, 0, 0);
  };

  // ---- weights, global -> registers: per MFMA row block a, 2 x 16 bytes per lane and stage
  const int kb64 = p.k / 64;
  const int n0w = bn0 + wave_s / WM * 64;  // first channel of this wavefront
  const uint32_t w_lane = (uint32_t)lane * 16u, sz_lane = (uint32_t)l32 * 4u;
  struct RawW {
    u4 c[kTA][2];
    uint32_t sz[kTA];
  };
  auto issue_w = [&](RawW &r, int stage) {
#pragma unroll
    for (int a = 0; a < kTA; ++a) {
      const int nb = (n0w + a * 32) >> 5;
      const char *wb = uniform(reinterpret_cast<const char *>(p.wp) +
                               ((int64_t)nb * kb64 + 2 * stage) * 1024);
      r.c[a][0] = *reinterpret_cast<const GU4 *>(CWAC_GLOBAL_PTR(wb + w_lane));
      r.c[a][1] = *reinterpret_cast<const GU4 *>(CWAC_GLOBAL_PTR(wb + 1024 + w_lane));
      const char *sb = uniform(reinterpret_cast<const char *>(p.sz) +
                               ((int64_t)stage * p.n + n0w + a * 32) * 4);
      r.sz[a] = *reinterpret_cast<const GU32 *>(CWAC_GLOBAL_PTR(sb + sz_lane));
    }
  };
  constexpr int kWLoads = 3 * kTA;

  // ---- LDS -> activation operand fragments
  const int x_off = (wave_m * 32 * TB + l32) * 256;
  const int swz_l = l32 & 15;
  auto read_x = [&](int buf, int kk, h8(&fx)[TB]) {
    const int8_t *base = smem + buf * kStageBytes + x_off + (((2 * kk + half) ^ swz_l) << 4);
#pragma unroll
    for (int b = 0; b < TB; ++b) fx[b] = *reinterpret_cast<const h8 *>(base + b * 32 * 256);
  };
  auto expand_w = [&](const RawW &r, const GroupConst (&gc)[kTA], int kk, h8(&fw)[kTA]) {
#pragma unroll
    for (int a = 0; a < kTA; ++a) fw[a] = expand8(r.c[a][kk >> 2][kk & 3], gc[a]);
  };

  v16f acc[kTA][TB];
#pragma unroll
  for (int a = 0; a < kTA; ++a)
#pragma unroll
    for (int b = 0; b < TB; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.0f;
  auto mma = [&](const h8(&fw)[kTA], const h8(&fx)[TB]) {
#pragma unroll
    for (int a = 0; a < kTA; ++a)
#pragma unroll
      for (int b = 0; b < TB; ++b)
        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fw[a], fx[b], acc[a][b], 0, 0, 0);
  };
  // Scheduler hint for one k-step: first the LDS reads of the next step's activation fragments,
  // then kTA * TB MFMAs; the expansion of the next step's weight fragments (about
  // 35 vector ALU operations) spread evenly behind all of them; `vmem` loads spread likewise.
  auto interleave = [&](int vmem) {
    __builtin_amdgcn_sched_group_barrier(0x100, TB, 0);  // the next step's LDS reads go first
#pragma unroll
    for (int i = 0; i < kTA * TB; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      if (i < vmem) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, 40 / (kTA * TB), 0);
    }
    __builtin_amdgcn_sched_barrier(0);  // one k-step per scheduling region
  };

  // ---- prologue.  Load order: X(0), W(0), X(1); waiting for all but the last kXLoads leaves X(1) in flight.
  const int stages = p.k / kGroup;
  RawW rawA, rawB;
  GroupConst gc[kTA];
  h8 fxA[TB], fxB[TB], fwA[kTA], fwB[kTA];
  issue_x(0, 0);
  issue_w(rawA, 0);
  if (stages > 1) issue_x(1, 1);
  if (tid < BN) {
    s_mult[tid] = p_mult;
    s_fb[tid] = p_fb;
  }
  if (stages > 1)
    __builtin_amdgcn_s_waitcnt(wait_imm(kXLoads, 0));
  else
    __builtin_amdgcn_s_waitcnt(wait_imm(0, 0));
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int a = 0; a < kTA; ++a) gc[a] = group_const(rawA.sz[a]);
  read_x(0, 0, fxA);
  expand_w(rawA, gc, 0, fwA);

  // One stage = one group.  `cur` holds this stage's codes (landed), `nxt` receives the next
  // stage's during k-step 0.  Every k-step fetches and expands the fragments of the following
  // one while its own MFMAs run.  Before the MFMAs of the last k-step every wavefront has fetched
  // its last fragments of this stage (its buffer is free for stage s + 2) and stage s + 1 has
  // landed; that k-step prepares the first fragments of the next stage.
  auto stage_body = [&](int s, int buf, RawW &cur, RawW &nxt) {
    const bool more = s + 1 < stages;
#pragma unroll
    for (int kk = 0; kk < 7; ++kk) {
      if (kk == 0 && more) issue_w(nxt, s + 1);
      if (kk & 1) {
        read_x(buf, kk + 1, fxA);
        expand_w(cur, gc, kk + 1, fwA);
        mma(fwB, fxB);
      } else {
        read_x(buf, kk + 1, fxB);
        expand_w(cur, gc, kk + 1, fwB);
        mma(fwA, fxA);
      }
      interleave(kk == 0 ? kWLoads : 0);
    }
    __builtin_amdgcn_s_waitcnt(wait_imm(0, 0));  // X(s + 1) and W(s + 1) have landed; fragments read
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    if (s + 2 < stages) issue_x(buf, s + 2);
    if (more) {
#pragma unroll
      for (int a = 0; a < kTA; ++a) gc[a] = group_const(nxt.sz[a]);  // this stage's are dead by now
      read_x(buf ^ 1, 0, fxA);
      expand_w(nxt, gc, 0, fwA);
    }
    mma(fwB, fxB);  // k-step 7
    interleave(kXLoads);
  };

  int s = 0;
  for (; s + 2 <= stages; s += 2) {
    stage_body(s, 0, rawA, rawB);
    stage_body(s + 1, 1, rawB, rawA);
  }
  if (s < stages) stage_body(s, 0, rawA, rawB);

  // every wavefront is past its last LDS read of the ring (the barrier of the last stage)
  w4_epilogue<OUT_KIND, TB, WM>(p, acc, smem, s_mult, s_fb, bm0, bn0, wave_m, wave_n, lane);
}

template <int OUT_KIND, int TB, int WM = 2>
cwac_status launch_w4(const W4Params &p, hipStream_t st) {
  static const hipError_t attr =
      hipFuncSetAttribute(reinterpret_cast<const void *>(&w4a16_kernel<OUT_KIND, TB, WM>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, W4Cfg<TB, WM>::LDS);
  if (attr != hipSuccess) return CWAC_E_LAUNCH;
  const int64_t blocks = (int64_t)p.tiles_m * p.tiles_n;
  if (blocks > 0x7fffffff) return CWAC_E_LAUNCH;
  w4a16_kernel<OUT_KIND, TB, WM><<<dim3((unsigned)blocks), kFwdThreads, W4Cfg<TB, WM>::LDS, st>>>(p);
  return launch_status();
}

// ------------------------------------------------------------------------------------------
// Small batches (32 tokens per launch: the decode step of an LLM).  The layer is then bound by the
// stream of 4-bit weights, not by the matrix cores: one workgroup of NW (4 or 8) wavefronts owns 32
// output channels (one row of 1 KiB blocks of the packed layout) over the whole of K, each wavefront
// a contiguous share of the groups.  Neither operand passes through registers on its way in: every
// wavefront owns a ring of D slots in LDS - per group 2 KiB of codes, the 32 scale / zero-point
// words and the group's block of activations (MP rows x 256 bytes, MP = m rounded up to 8, 16 or
// 32) - that global_load_lds fills D groups ahead of the arithmetic.  The activations are fetched
// four rows per instruction (whole 256-byte row pieces: a lane-per-row register load would touch 32
// cache lines per instruction, which bounded the kernel by the L1's tag rate), with the chunk
// position XOR (row & 15) applied on the global-address side so that the MFMA operand reads
// (lane = token row) are free of bank conflicts.  Rows beyond m repeat row m - 1 (their results are
// not stored).  Codes are expanded in registers and meet the activations in one 32 x 32 MFMA tile
// per 16 input channels.  The wavefronts' partial tiles are added in wavefront order through LDS
// (deterministic), then the epilogue of the tiled kernel.  No workspace, no atomics.
// ------------------------------------------------------------------------------------------
constexpr int kSmallM = 32;
constexpr int kHalfTileUpTo = 256;  // 128-token tiles in a launch up to which they are taken (one per compute unit)
constexpr int kSmallPasses = 8;  // at most this many launches of 32 rows each
// Whether ceil(m / 32) passes of the weight-streaming kernel beat one launch of the tiled kernel with
// 128-token tiles.  Fitted to measurements on 4096 .. 12288 channels x 4096 .. 11008 input channels
// (microseconds): a pass costs 5.5 + packed bytes / 2.6 MB, a single round of 128-token tiles 3 + 0.0127 k.
inline bool small_passes_pay(int64_t m, int n, int k) {
  if (m > kSmallPasses * kSmallM) return false;
  const double passes = (double)((m + kSmallM - 1) / kSmallM);
  const double pass_us = 5.5 + (double)n * (double)k * 0.5 / 2.6e6;
  return m <= kSmallM || passes * pass_us < 3.0 + 0.0127 * (double)k;
}

template <int NW, int MP, int D_>
struct StreamCfg {
  static constexpr int D = D_;                     // ring slots per wavefront
  static constexpr int X_OFF = 2048 + 256;         // codes, then 64 lanes x 4 bytes of scale words, then activations
  static constexpr int SLOT = X_OFF + MP * 256;
  static constexpr int RING = D * SLOT;
  static constexpr int LX = MP / 4, LW = 3, L = LX + LW;  // load instructions per group
  static constexpr int PART = (NW - 1) * 16 * 64 * 4;  // partial tiles of wavefronts 1 .. NW - 1 (over the rings)
  static constexpr int LDS = NW * RING > PART ? NW * RING : PART;
  static_assert(LDS <= 160 * 1024, "LDS budget of one compute unit");
  static_assert(D >= 2 && D <= 4 && (D - 1) * L < 64, "waits below are written for up to three groups in flight");
};

template <int OUT_KIND, int NW, int MP, int D_>
__global__ __launch_bounds__(64 * NW) void w4a16_small_m_kernel(const W4Params p) {
  using S = StreamCfg<NW, MP, D_>;
  constexpr int D = S::D, L = S::L;
  extern __shared__ __attribute__((aligned(16))) int8_t smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  const int nb = blockIdx.x, n0 = nb * 32;
  const int groups = p.k / kGroup, kb64 = p.k / 64;
  const int g_begin = wave * groups / NW, g_end = (wave + 1) * groups / NW;
  const bool row_ok = l32 < p.m;
  int8_t *ring = smem + wave * S::RING;

  const char *wrow = reinterpret_cast<const char *>(p.wp) + (int64_t)nb * kb64 * 1024 + lane * 16;
  const uint32_t *szp = p.sz + n0 + l32;
  // activation loads: instruction t covers rows 4 t .. 4 t + 3 of the block, lane i = (row i / 16,
  // chunk position i % 16), which receives the row's chunk (i % 16) ^ (row & 15)
  uint32_t xoff[S::LX];
#pragma unroll
  for (int t = 0; t < S::LX; ++t) {
    const int row = 4 * t + (lane >> 4);
    const int src_row = row < (int)p.m ? row : (int)p.m - 1;
    xoff[t] = (uint32_t)src_row * (uint32_t)p.ldx_bytes + (uint32_t)(((lane & 15) ^ (row & 15)) << 4);
  }
  // group g -> slot: two 1 KiB blocks of codes, one scale word per lane (the upper half-wave repeats
  // the lower one's 32 words), MP / 4 blocks of four activation rows
  auto issue = [&](int g, int slot_i) {
    int8_t *slot = ring + slot_i * S::SLOT;
    __builtin_amdgcn_global_load_lds(CWAC_GLOBAL_PTR(wrow + (int64_t)(2 * g) * 1024), CWAC_LDS_PTR(slot), 16, 0, 0);
    __builtin_amdgcn_global_load_lds(CWAC_GLOBAL_PTR(wrow + (int64_t)(2 * g + 1) * 1024), CWAC_LDS_PTR(slot + 1024),
                                     16, 0, 0);
    __builtin_amdgcn_global_load_lds(CWAC_GLOBAL_PTR(szp + (int64_t)g * p.n), CWAC_LDS_PTR(slot + 2048), 4, 0, 0);
    const char *xg = p.x + (int64_t)g * 256;
#pragma unroll
    for (int t = 0; t < S::LX; ++t)
      __builtin_amdgcn_global_load_lds(CWAC_GLOBAL_PTR(xg + xoff[t]), CWAC_LDS_PTR(slot + S::X_OFF + t * 1024), 16, 0,
                                       0);
  };
  // MFMA operand of k-step kk: row l32 (clamped into the block), chunk 2 kk + half
  const int xrow = l32 < MP ? l32 : MP - 1;
  const int xrd = S::X_OFF + xrow * 256, xsw = xrow & 15;
  // two accumulators (even / odd k-steps): consecutive MFMAs do not wait for each other
  v16f acc, acc1;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = acc1[i] = 0.0f;
  const ExpandConst ec = expand_const();

  // Memory operations return in order, so "at most N outstanding" means everything older than the
  // newest N has arrived: with r groups issued behind group g, group g is complete at r * L.
  int slot_i = 0;
#pragma unroll 1
  for (int i = 0; i < D; ++i)
    if (g_begin + i < g_end) issue(g_begin + i, i);
#pragma unroll 1
  for (int g = g_begin; g < g_end; ++g) {
    const int behind = g_end - 1 - g < D - 1 ? g_end - 1 - g : D - 1;
    if (behind >= 3)
      __builtin_amdgcn_s_waitcnt(wait_imm(3 * L, 15));
    else if (behind == 2)
      __builtin_amdgcn_s_waitcnt(wait_imm(2 * L, 15));
    else if (behind == 1)
      __builtin_amdgcn_s_waitcnt(wait_imm(L, 15));
    else
      __builtin_amdgcn_s_waitcnt(wait_imm(0, 15));
    asm volatile("" ::: "memory");  // the slot reads stay below the wait
    __builtin_amdgcn_sched_barrier(0);
    const int8_t *slot = ring + slot_i * S::SLOT;
    const u4 c0 = *reinterpret_cast<const u4 *>(slot + lane * 16);
    const u4 c1 = *reinterpret_cast<const u4 *>(slot + 1024 + lane * 16);
    const uint32_t sz = *reinterpret_cast<const uint32_t *>(slot + 2048 + l32 * 4);
    h8 x[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
      x[kk] = *reinterpret_cast<const h8 *>(slot + xrd + (((2 * kk + half) ^ xsw) << 4));
    if (g + D < g_end) {
      // the slot's contents are in registers before the next group may land in it
      __builtin_amdgcn_s_waitcnt(wait_imm(63, 0));
      asm volatile("" ::: "memory");
      __builtin_amdgcn_sched_barrier(0);
      issue(g + D, slot_i);
    }
    slot_i = slot_i + 1 == D ? 0 : slot_i + 1;
    const GroupConst gc = group_const(sz);
#pragma unroll
    for (int kk = 0; kk < 8; kk += 2) {
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(expand8(kk < 4 ? c0[kk & 3] : c1[kk & 3], gc, ec), x[kk], acc, 0, 0,
                                                   0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(expand8(kk + 1 < 4 ? c0[(kk + 1) & 3] : c1[(kk + 1) & 3], gc, ec),
                                                    x[kk + 1], acc1, 0, 0, 0);
    }
  }
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] += acc1[i];

  // partial tiles over the rings, once every wavefront has left its ring
  float *s_part = reinterpret_cast<float *>(smem);
  __syncthreads();
  if (wave > 0) {
#pragma unroll
    for (int i = 0; i < 16; ++i) s_part[((wave - 1) * 16 + i) * 64 + lane] = acc[i];
  }
  __syncthreads();
  if (wave != 0) return;
#pragma unroll 1
  for (int w = 0; w < NW - 1; ++w)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] += s_part[(w * 16 + i) * 64 + lane];
  if (!row_ok) return;
  constexpr int ESZ = OUT_KIND == CWAC_OUT_FP16 ? 2 : 4;
  char *orow = p.out + ((int64_t)l32 * p.ldo + n0) * ESZ;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int ch = 8 * q + 4 * half;  // channel inside the block: accumulator elements 4q .. 4q + 3
    float u[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float v = acc[4 * q + r] * (p.mult ? p.mult[n0 + ch + r] : 1.0f);
      u[r] = v + (p.fbias ? p.fbias[n0 + ch + r] : 0.0f);
    }
    if (OUT_KIND == CWAC_OUT_FP16) {
      const h2 lo = {(_Float16)u[0], (_Float16)u[1]}, hi = {(_Float16)u[2], (_Float16)u[3]};
      *reinterpret_cast<uint2 *>(orow + ch * 2) =
          make_uint2(__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi));
    } else {
      *reinterpret_cast<float4 *>(orow + ch * 4) = make_float4(u[0], u[1], u[2], u[3]);
    }
  }
}

template <int OUT_KIND, int NW, int MP, int D>
cwac_status launch_w4_small_cfg(const W4Params &p, hipStream_t st) {
  static const hipError_t attr =
      hipFuncSetAttribute(reinterpret_cast<const void *>(&w4a16_small_m_kernel<OUT_KIND, NW, MP, D>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, StreamCfg<NW, MP, D>::LDS);
  if (attr != hipSuccess) return CWAC_E_LAUNCH;
  w4a16_small_m_kernel<OUT_KIND, NW, MP, D><<<dim3((unsigned)(p.n / 32)), 64 * NW, StreamCfg<NW, MP, D>::LDS, st>>>(p);
  return launch_status();
}

template <int OUT_KIND>
cwac_status launch_w4_small(const W4Params &p, int waves, int depth, hipStream_t st) {
  // Four wavefronts per workgroup where the layer has at least as many channel blocks as the chip
  // has compute units, eight with fewer blocks (waves, depth: the caller's overrides,
  // cwac_tuning.w4_small_waves / w4_small_depth).  The ring depth trades bytes in flight per
  // wavefront against resident wavefronts per compute unit (the rings are what fills its LDS):
  // two slots - four workgroups of four wavefronts per compute unit at up to 8 rows - measured
  // best on every layer shape, since what a wavefront waits for most is its first group.  A
  // combination whose rings do not fit the LDS takes the nearest one that does.
  int nw = waves ? waves : (p.n / 32 >= 256 ? 4 : 8);
  const int mp = p.m <= 8 ? 8 : (p.m <= 16 ? 16 : 32);
  if (mp == 32) nw = 4;  // 32-row activation blocks leave room for the rings of four wavefronts only
  int d = depth ? depth : 2;
  if (mp == 32 && d > 3) d = 3;
  if (mp == 16 && nw == 8 && d > 3) d = 3;
#define CWAC_W4_SMALL(NW, MP, D) \
  if (nw == NW && mp == MP && d == D) return launch_w4_small_cfg<OUT_KIND, NW, MP, D>(p, st)
  CWAC_W4_SMALL(4, 8, 2);
  CWAC_W4_SMALL(4, 8, 3);
  CWAC_W4_SMALL(4, 8, 4);
  CWAC_W4_SMALL(8, 8, 2);
  CWAC_W4_SMALL(8, 8, 3);
  CWAC_W4_SMALL(8, 8, 4);
  CWAC_W4_SMALL(4, 16, 2);
  CWAC_W4_SMALL(4, 16, 3);
  CWAC_W4_SMALL(4, 16, 4);
  CWAC_W4_SMALL(8, 16, 2);
  CWAC_W4_SMALL(8, 16, 3);
  CWAC_W4_SMALL(4, 32, 2);
  CWAC_W4_SMALL(4, 32, 3);
#undef CWAC_W4_SMALL
  return CWAC_E_MODE;
}


int grid_for(int64_t items) {
  const int64_t b = ceil_div(items, kThreads);
  return (int)(b < 1 ? 1 : (b > 65536 ? 65536 : b));
}

}  // namespace
}  // namespace cwac

using namespace cwac;

extern "C" {

cwac_status cwac_w4_quantize_groupwise(const float *w, int64_t ldw, int32_t n, int32_t k, uint8_t *codes,
                                       uint16_t *scales, uint8_t *zeros, void *stream) {
  if (!w || !codes || !scales || !zeros) return CWAC_E_NULL;
  if (n < 1 || k < kGroup || k % kGroup != 0 || ldw < k) return CWAC_E_SHAPE;
  if (!aligned(w, 8) || ldw % 2 != 0 || !aligned(codes, 2)) return CWAC_E_ALIGN;
  const int groups = k / kGroup;
  const int64_t tasks = (int64_t)n * groups;
  const int64_t blocks = ceil_div(tasks, kThreads / 64);
  if (blocks > 0x7fffffff) return CWAC_E_SHAPE;
  w4_quantize_kernel<<<dim3((unsigned)blocks), kThreads, 0, as_stream(stream)>>>(w, ldw, n, groups, codes,
                                                                                 scales, zeros);
  return launch_status();
}

size_t cwac_w4_packed_w_bytes(int32_t n, int32_t k) {
  if (n < 1 || k < 1) return 0;
  return (size_t)n * (size_t)k / 2;
}

cwac_status cwac_w4_pack(const uint8_t *codes, const uint16_t *scales, const uint8_t *zeros, int32_t n,
                         int32_t k, void *packed_w, uint32_t *packed_sz, void *stream) {
  if (!codes || !scales || !zeros || !packed_w || !packed_sz) return CWAC_E_NULL;
  if (n < 32 || n % 32 != 0 || k < kGroup || k % kGroup != 0) return CWAC_E_SHAPE;
  if (!aligned(codes, 8) || !aligned(packed_w, 16) || !aligned(packed_sz, 4)) return CWAC_E_ALIGN;
  hipStream_t st = as_stream(stream);
  w4_pack_kernel<<<grid_for((int64_t)n * (k / 8)), kThreads, 0, st>>>(codes, n, k,
                                                                      static_cast<uint32_t *>(packed_w));
  if (launch_status() != CWAC_OK) return CWAC_E_LAUNCH;
  w4_pack_sz_kernel<<<grid_for((int64_t)n * (k / kGroup)), kThreads, 0, st>>>(scales, zeros, n, k / kGroup,
                                                                              packed_sz);
  return launch_status();
}

cwac_status cwac_fold_weight_only(const float *alpha, const float *beta, const float *bias, int32_t n_out,
                                  float *mult, float *fbias, void *stream) {
  if (!mult || !fbias) return CWAC_E_NULL;
  if ((alpha == nullptr) != (beta == nullptr)) return CWAC_E_MODE;
  if (n_out < 1) return CWAC_E_SHAPE;
  fold_weight_only_kernel<<<grid_for(n_out), kThreads, 0, as_stream(stream)>>>(alpha, beta, bias, n_out, mult,
                                                                                fbias);
  return launch_status();
}

cwac_status qlinear_w4a16_cwac_forward_ex(const uint16_t *x, int64_t ldx, const void *packed_w,
                                          const uint32_t *packed_sz, int64_t m, int32_t n, int32_t k,
                                          const float *mult, const float *fbias, int32_t out_kind, void *out,
                                          int64_t ldo, const cwac_tuning *tuning, void *stream) {
  if (!x || !packed_w || !packed_sz || !out) return CWAC_E_NULL;
  if (out_kind != CWAC_OUT_FP16 && out_kind != CWAC_OUT_FP32) return CWAC_E_MODE;
  const int w4_tile = tuning ? tuning->w4_tile : 0, small_waves = tuning ? tuning->w4_small_waves : 0;
  const int small_depth = tuning ? tuning->w4_small_depth : 0;
  if ((w4_tile != 0 && w4_tile != 256 && w4_tile != 128 && w4_tile != 512) || (w4_tile == 512 && n < 512) ||
      (small_waves != 0 && small_waves != 4 && small_waves != 8) || (small_depth != 0 && (small_depth < 2 || small_depth > 4)))
    return CWAC_E_MODE;
  if (m < 1 || n < 256 || n % 32 != 0 || k < kGroup || k > 32768 || k % kGroup != 0 || ldx < k || ldo < n)
    return CWAC_E_SHAPE;
  const int64_t esz = out_kind == CWAC_OUT_FP16 ? 2 : 4;
  if (!aligned(x, 16) || ldx % 8 != 0 || !aligned(packed_w, 16) || !aligned(packed_sz, 4) ||
      !aligned(out, 16) || (ldo * esz) % 16 != 0)
    return CWAC_E_ALIGN;
  if (ceil_div(m, 256) > 0x7fffff) return CWAC_E_SHAPE;
  // per-lane activation offsets inside a tile are 32-bit
  if (255 * ldx * 2 + 32768 * 2 > 0xffffffffLL) return CWAC_E_SHAPE;
  W4Params p;
  p.x = reinterpret_cast<const char *>(x);
  p.ldx_bytes = ldx * 2;
  p.wp = static_cast<const u4 *>(packed_w);
  p.sz = packed_sz;
  p.m = m;
  p.n = n;
  p.k = k;
  p.mult = mult;
  p.fbias = fbias;
  p.out = static_cast<char *>(out);
  p.ldo = ldo;
  p.tiles_n = (int)ceil_div(n, 256);
  // The caller's override (results agree to the rounding of the fp32 sums): w4_tile = 256 keeps the
  // 256-token tiles at every batch size, 128 the 128-token tiles.
  if (w4_tile == 0 && small_passes_pay(m, n, k)) {
    // passes of the weight-streaming kernel over blocks of 32 rows: the packed weights of a layer
    // stay in the last-level cache between passes, and a row of 128- or 256-token tiles would leave
    // most of the chip idle at these sizes (each tile as long as its K loop)
    for (int64_t r0 = 0; r0 < m; r0 += kSmallM) {
      W4Params q = p;
      q.x = p.x + r0 * p.ldx_bytes;
      q.out = p.out + r0 * ldo * esz;
      q.m = m - r0 < kSmallM ? m - r0 : kSmallM;
      const cwac_status s = out_kind == CWAC_OUT_FP16
                                ? launch_w4_small<CWAC_OUT_FP16>(q, small_waves, small_depth, as_stream(stream))
                                : launch_w4_small<CWAC_OUT_FP32>(q, small_waves, small_depth, as_stream(stream));
      if (s != CWAC_OK) return s;
    }
    return CWAC_OK;
  }
  // 128-token tiles while they fit the chip in one round (one tile per compute unit): a half tile
  // takes about two thirds of a full tile's time (the weight expansion is per channel block, not
  // per token, so it spends more vector work per MFMA), which pays exactly while the full tiles
  // would leave compute units idle
  const bool half = w4_tile == 128 || (w4_tile == 0 && ceil_div(m, 128) * p.tiles_n <= kHalfTileUpTo);
  if (half) {
    p.tiles_m = (int)ceil_div(m, 128);
    return out_kind == CWAC_OUT_FP16 ? launch_w4<CWAC_OUT_FP16, 2>(p, as_stream(stream))
                                     : launch_w4<CWAC_OUT_FP32, 2>(p, as_stream(stream));
  }
  // large batches: the tile of 512 channels x 128 tokens (no wavefront expands another one's weights)
  if (w4_tile == 512 || (w4_tile == 0 && n >= 512)) {
    p.tiles_m = (int)ceil_div(m, 128);
    p.tiles_n = (int)ceil_div(n, 512);
    return out_kind == CWAC_OUT_FP16 ? launch_w4<CWAC_OUT_FP16, 4, 1>(p, as_stream(stream))
                                     : launch_w4<CWAC_OUT_FP32, 4, 1>(p, as_stream(stream));
  }
  p.tiles_m = (int)ceil_div(m, 256);
  return out_kind == CWAC_OUT_FP16 ? launch_w4<CWAC_OUT_FP16, 4>(p, as_stream(stream))
                                   : launch_w4<CWAC_OUT_FP32, 4>(p, as_stream(stream));
}

cwac_status qlinear_w4a16_cwac_forward(const uint16_t *x, int64_t ldx, const void *packed_w,
                                       const uint32_t *packed_sz, int64_t m, int32_t n, int32_t k,
                                       const float *mult, const float *fbias, int32_t out_kind, void *out,
                                       int64_t ldo, void *stream) {
  return qlinear_w4a16_cwac_forward_ex(x, ldx, packed_w, packed_sz, m, n, k, mult, fbias, out_kind, out, ldo,
                                       nullptr, stream);
}

}  // extern "C"
