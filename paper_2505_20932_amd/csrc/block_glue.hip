// The non-linear glue between the W8A8 linear layers of a pre-norm Transformer block (the part
// of the block that per-layer compensation steps around, Sec. 3.2): residual add + layer
// normalization + quantizer, the GELU of the MLP as a 256-entry code table, and multi-head
// self-attention on the requantized output of the qkv layer.  Every linear layer consumes int8
// codes and requantizes to int8 codes (Eq. 10); the residual stream is binary16.
//
// Arithmetic, in fp32 unless stated (no contraction: each line is one rounding):
//   residual   t = h + s_r * (float)(c - z_r);  h1 = RN16(t);  the layer norm reads h1
//   layer norm mean = sum(x) * (1 / C);  var = sum((x - mean)^2) * (1 / C);  y = fma((x - mean) * rsq(var + eps), gamma, beta)
//   quantizer  code = clip(rne(fma(y, 1 / s, z)), -128, 127)                            (Eq. 1)
//   attention  S = (K - z)(Q - z)^T exactly (integers below 2^24 in the fp32 MFMA accumulators);
//              P = 1024 p = exp2(fma(S, s^2 / sqrt(d) * log2 e, 10 - that * max S));  O = (sum_j RN16(P_j) (V_j - z)) * s / sum_j P_j,
//              keys taken in groups of 96 with the running maximum (earlier partial sums rescaled)
//   GELU table entry(c) = clip(rne(GELU(s_in (c - z_in)) / s_out + z_out)) evaluated in fp64 (erf form)
#include <hip/hip_runtime.h>

#include <math.h>

#include "cwac_internal.h"

namespace cwac {
namespace {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef int v4i __attribute__((ext_vector_type(4)));

// sum over aligned groups of LPR lanes (the same value in every lane of a group)
template <int LPR>
__device__ __forceinline__ float group_sum(float v) {
#pragma unroll
  for (int off = LPR / 2; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// Four int8 codes (one word) -> (code - z) as four binary16 values, exactly: a byte u = code + 128 under
// the high byte 0x64 is the binary16 number 1024 + u, and (1024 + u) - (1152 + z) is an integer below
// 2048 in magnitude.  `bias` = 1152 + z in both halves.
__device__ __forceinline__ void codes_to_h4(uint32_t w, h2 bias, h2 &lo, h2 &hi) {
  const uint32_t u = w ^ 0x80808080u;
  lo = __builtin_bit_cast(h2, __builtin_amdgcn_perm(0x64646464u, u, 0x04010400u)) - bias;
  hi = __builtin_bit_cast(h2, __builtin_amdgcn_perm(0x64646464u, u, 0x04030402u)) - bias;
}

__device__ __forceinline__ h8 codes_to_h8(uint2 c, h2 bias) {
  h2 a, b, d, e;
  codes_to_h4(c.x, bias, a, b);
  codes_to_h4(c.y, bias, d, e);
  return h8{a[0], a[1], b[0], b[1], d[0], d[1], e[0], e[1]};
}

// Eq. 1 with the division by the scale as a fused multiply-add with its fp32 reciprocal (the
// reciprocal's rounding instead of the division's: far inside what decides a code only at a tie).
__device__ __forceinline__ int quant_code(float y, float inv_s, float zf) {
  const float v = __builtin_fmaf(y, inv_s, zf);
  return (int)__builtin_amdgcn_fmed3f(rintf(v), -128.0f, 127.0f);
}

// ------------------------------------------------------------------------------------------
// Residual add + layer norm + quantizer: LPR (16, 32 or 64) lanes per token row, the row in
// registers (NV vectors of 8 channels per lane: C <= 8 * LPR * NV; the host picks the pair that
// leaves the fewest idle lanes, e.g. 32 x 3 for C = 768), two-pass mean / variance; LDS holds gamma and beta only.
// HBM bytes per element: 2 (h) [+ 1 (codes) + 2 (h1)] + 1 (x_q).
// ------------------------------------------------------------------------------------------
struct LnParams {
  const _Float16 *h;
  int64_t ldh;
  const int8_t *r;
  int64_t ldr;
  float s_r;
  int z_r;
  _Float16 *h_out;
  int64_t ldho;
  const float *gamma, *beta;
  float eps, inv_s_x, inv_c;  // 1 / s_x and 1 / c, rounded once on the host
  int z_x;
  int8_t *x_q;
  int64_t ldxq;
  int64_t m;
  int c;
};

// FULL: every lane's every vector is inside the row (C = 8 * LPR * NV): no masks.
template <int LPR, int NV, bool FULL>
__global__ __launch_bounds__(256) void residual_ln_quant_kernel(const LnParams p) {
  const int lane = threadIdx.x & (LPR - 1);  // position inside the row's group of LPR lanes
  const int nvec = p.c >> 3;
  // A lane group walks rows first, first + stride, ...; the loads of its next row are in flight while it
  // reduces and quantizes the current one.  Groups past the end read the last row and store nothing: the
  // shuffles then always run with every lane active, and the trip count is uniform over the workgroup
  // (h_out may be h itself, so such a group must not store).
  const int64_t stride = (int64_t)gridDim.x * (256 / LPR);
  int64_t row = ((int64_t)blockIdx.x * 256 + threadIdx.x) / LPR;
  const int64_t block_row0 = (int64_t)blockIdx.x * (256 / LPR);
  struct Raw {
    h8 hv[NV];
    uint2 cw[NV];
  };
  auto load = [&](Raw &r, int64_t at) {
    if (at > p.m - 1) at = p.m - 1;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int v = (FULL || lane + LPR * j < nvec) ? lane + LPR * j : 0;
      r.hv[j] = *reinterpret_cast<const h8 *>(p.h + at * p.ldh + 8 * v);
      if (p.r) r.cw[j] = *reinterpret_cast<const uint2 *>(p.r + at * p.ldr + 8 * v);
    }
  };
  // gamma and beta are the same for every row: staged once per workgroup in LDS (c <= 2048)
  __shared__ __attribute__((aligned(16))) float s_gamma[2048], s_beta[2048];
  if (p.x_q) {
    for (int i = threadIdx.x; i < p.c; i += 256) {
      s_gamma[i] = p.gamma[i];
      s_beta[i] = p.beta[i];
    }
  }
  __syncthreads();
  const float zf = (float)p.z_x, inv_s = p.inv_s_x;
  Raw cur, nxt;
  load(cur, row);
  for (int64_t base = block_row0; base < p.m; base += stride, row += stride) {
    const bool more = base + stride < p.m;  // uniform over the workgroup
    if (more) load(nxt, row + stride);
    const bool live = row < p.m;
    const int64_t at = live ? row : p.m - 1;
    float x[NV][8];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int v = lane + LPR * j;
      const bool ok = FULL || v < nvec;
#pragma unroll
      for (int e = 0; e < 8; ++e) x[j][e] = ok ? (float)cur.hv[j][e] : 0.0f;
      if (p.r) {
        h8 ho;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const uint32_t w = e < 4 ? cur.cw[j].x : cur.cw[j].y;
          const int code = (int)(int8_t)(w >> (8 * (e & 3)));
          const float t = x[j][e] + p.s_r * (float)(code - p.z_r);
          ho[e] = (_Float16)t;
          x[j][e] = ok ? (float)ho[e] : 0.0f;
        }
        if (p.h_out && live && ok) *reinterpret_cast<h8 *>(p.h_out + at * p.ldho + 8 * v) = ho;
      }
    }
    if (p.x_q) {
      float s = 0.0f;
#pragma unroll
      for (int j = 0; j < NV; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) s += x[j][e];
      const float mean = group_sum<LPR>(s) * p.inv_c;
      float ss = 0.0f;
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        const bool ok = FULL || lane + LPR * j < nvec;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float d = ok ? x[j][e] - mean : 0.0f;
          x[j][e] = d;
          ss += d * d;
        }
      }
      const float var = group_sum<LPR>(ss) * p.inv_c;
      const float rstd = __builtin_amdgcn_rsqf(var + p.eps);  // 1 ulp
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        const int v = lane + LPR * j;
        const int vs = (FULL || v < nvec) ? v : 0;
        const float4 g0 = *reinterpret_cast<const float4 *>(s_gamma + 8 * vs),
                     g1 = *reinterpret_cast<const float4 *>(s_gamma + 8 * vs + 4),
                     b0 = *reinterpret_cast<const float4 *>(s_beta + 8 * vs),
                     b1 = *reinterpret_cast<const float4 *>(s_beta + 8 * vs + 4);
        const float g[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
        const float b[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
        uint32_t w[2] = {0u, 0u};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float y = __builtin_fmaf(x[j][e] * rstd, g[e], b[e]);
          const int code = quant_code(y, inv_s, zf);
          w[e >> 2] |= (uint32_t)(code & 0xff) << (8 * (e & 3));
        }
        if (live && (FULL || v < nvec)) *reinterpret_cast<uint2 *>(p.x_q + at * p.ldxq + 8 * v) = make_uint2(w[0], w[1]);
      }
    }
    if (more) cur = nxt;
  }
}

// ------------------------------------------------------------------------------------------
// GELU between fc1 and fc2 on int8 codes: a function of one code, so a 256-entry table.
// ------------------------------------------------------------------------------------------
__global__ void gelu_table_kernel(float s_in, int z_in, float s_out, int z_out, int8_t *table) {
  const int code = (int)threadIdx.x - 128;
  const double x = (double)s_in * (double)(code - z_in);
  const double g = 0.5 * x * (1.0 + erf(x * 0.70710678118654752440));
  double v = rint(g / (double)s_out + (double)z_out);
  v = fmin(fmax(v, -128.0), 127.0);
  table[threadIdx.x] = (int8_t)(int)v;
}

// out[i] = table[in[i] + 128]; 16 codes per lane and pass, the table in LDS (64 words: the lanes
// of a read hit distinct banks or the same word).  HBM bytes per element: 1 + 1.
__global__ __launch_bounds__(256) void table_lookup_kernel(const int8_t *in, int64_t ld_in, const int8_t *table,
                                                           int8_t *out, int64_t ld_out, int64_t m, int n) {
  __shared__ uint8_t s_tab[256];
  s_tab[threadIdx.x] = (uint8_t)table[threadIdx.x];
  __syncthreads();
  const int vec_per_row = n >> 4;
  const int64_t total = m * vec_per_row;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t row = i / vec_per_row;
    const int v = (int)(i - row * vec_per_row);
    const v4i cw = __builtin_nontemporal_load(reinterpret_cast<const v4i *>(in + row * ld_in + 16 * v));
    v4i ow;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const uint32_t w = (uint32_t)cw[q];
      uint32_t o = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) o |= (uint32_t)s_tab[((w >> (8 * e)) & 0xff) ^ 0x80] << (8 * e);
      ow[q] = (int)o;
    }
    *reinterpret_cast<v4i *>(out + row * ld_out + 16 * v) = ow;
  }
}

// ------------------------------------------------------------------------------------------
// Multi-head self-attention, head width D = 64 or 32, up to 224 tokens: one workgroup per (image, head),
// one wavefront per 32 queries.  K (as (code - z) in binary16, row-major, rows of 2 D + 16 bytes) and V
// (transposed, rows of 64 NT + 8 bytes) of the head sit in LDS; both row strides make the operand reads
// conflict-free.  S^T = K Q^T: 32 x 32 x 16 MFMA tiles with keys along M, so a lane owns one
// query (its N index) and, with its partner lane ^ 32, all of that query's scores - the softmax
// is a reduction over the lane's own registers plus one exchange.  Registers 8u .. 8u + 7 of score
// tile t are, in order, the B operand of k-step (t, u) of O^T = V^T P^T; the A operand gathers
// the same keys, 32 t + 16 u + 8 (e >> 2) + 4 half + (e & 3), from the transposed V with two
// 8-byte reads.  Scores are exact integers; p is scaled by 1024 before its conversion to binary16
// so that no term that matters falls into the subnormal range.
// ------------------------------------------------------------------------------------------
constexpr int kHeadDim = 64;     // widest head; 32 is the other width
constexpr int kMaxTokens = 4096; // longest sequence
// bytes per K row in LDS: the head's binary16 values + 16 (conflict-free 16-byte operand reads for both widths)
constexpr int k_stride(int d) { return 2 * d + 16; }
// bytes per V^T row in LDS: 2 * 32 * NT of keys + 8; in words twice an odd number, so the 8-byte operand
// reads of 32 consecutive rows cover all 64 banks once
constexpr int v_stride(int nt) { return 64 * nt + 8; }

struct AttnParams {
  const int8_t *r;
  int64_t ld;
  float s;
  int z;
  int tokens, heads;
  int64_t pairs;  // batch * heads
  const uint16_t *bias;  // binary16 [heads][tokens][ldb] added to the logits, or NULL
  int64_t ldb;
  float s_a;
  int z_a;
  int8_t *a;
  int64_t lda;
};

// Scores, softmax weights and the second product for CNT key tiles starting at tile t0, with the
// running maximum `mx`, the running (lane-local) sum of weights and the output accumulators
// rescaled when a later group raises the maximum (the usual streaming form of the softmax: the
// result is the same up to fp32 rounding, and only CNT score tiles are live at a time).
// With LONG the tiles in LDS are one chunk of a longer sequence: tile t0 + t holds keys from
// key0 + 32 (t0 + t) on, and a tile may lie wholly beyond the last token (its scores are masked and its
// bias is not read).
template <int CNT, int D, int VS, bool BIAS, bool LONG = false>
__device__ __forceinline__ void attention_key_group(int t0, bool first, const int8_t *s_k, const int8_t *s_v,
                                                    const h8 (&fq)[D / 16], const uint16_t *bias_row, int tokens,
                                                    float lscale, int l32, int half,
                                                    float &mx, float &sum, v16f (&oc)[D / 32], int key0 = 0) {
  v16f sc[CNT];
#pragma unroll
  for (int t = 0; t < CNT; ++t) {
#pragma unroll
    for (int i = 0; i < 16; ++i) sc[t][i] = 0.0f;
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
      const h8 fk = *reinterpret_cast<const h8 *>(s_k + (32 * (t0 + t) + l32) * k_stride(D) + (2 * s + half) * 16);
      sc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fk, fq[s], sc[t], 0, 0, 0);
    }
  }
  // register 4 g + r of tile t is key 32 t + 8 g + 4 half + r of this lane's query
  if (BIAS) {
    // with a bias the scores become logits in the log2 domain first: x = S * lscale + bias * log2(e)
    // (the bias rows are padded to whole key tiles, so the loads of padded keys stay inside them)
#pragma unroll
    for (int t = 0; t < CNT; ++t)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        if (LONG && key0 + 32 * (t0 + t) >= tokens) continue;  // uniform: the tile is masked below
        const uint2 bw = *reinterpret_cast<const uint2 *>(bias_row + key0 + 32 * (t0 + t) + 8 * g + 4 * half);
        const h2 b01 = __builtin_bit_cast(h2, bw.x), b23 = __builtin_bit_cast(h2, bw.y);
        const float bf[4] = {(float)b01[0], (float)b01[1], (float)b23[0], (float)b23[1]};
#pragma unroll
        for (int r = 0; r < 4; ++r)
          sc[t][4 * g + r] = __builtin_fmaf(sc[t][4 * g + r], lscale, bf[r] * 1.44269504088896340736f);
      }
  }
  const float dscale = BIAS ? 1.0f : lscale;  // what turns a score difference into a log2 difference
  float gmx = -INFINITY;
#pragma unroll
  for (int t = 0; t < CNT; ++t) {
    if (key0 + 32 * (t0 + t) + 32 > tokens) {  // only the last tiles can hold padded keys (uniform branch)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = key0 + 32 * (t0 + t) + 8 * (i >> 2) + 4 * half + (i & 3);
        if (key >= tokens) sc[t][i] = -INFINITY;
      }
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) gmx = fmaxf(gmx, sc[t][i]);
  }
  gmx = fmaxf(gmx, __shfl_xor(gmx, 32, 64));  // a group's first tile holds at least one real key: finite
  if (first) {
    mx = gmx;
  } else if (gmx > mx) {  // the same decision in both lanes of a query
    const float corr = __builtin_amdgcn_exp2f((mx - gmx) * dscale);
    sum *= corr;
#pragma unroll
    for (int a = 0; a < D / 32; ++a)
#pragma unroll
      for (int i = 0; i < 16; ++i) oc[a][i] *= corr;
    mx = gmx;
  }
  // 1024 p = exp2(S * lscale + (10 - mx * lscale)), one fused multiply-add per exponent;
  // exp2(-inf) = 0 for masked keys
  const float eoff = 10.0f - mx * dscale;
#pragma unroll
  for (int t = 0; t < CNT; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      sc[t][i] = __builtin_amdgcn_exp2f(BIAS ? sc[t][i] + eoff : __builtin_fmaf(sc[t][i], lscale, eoff));
      sum += sc[t][i];
    }
#pragma unroll
  for (int t = 0; t < CNT; ++t)
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      h8 fp;
#pragma unroll
      for (int e = 0; e < 8; ++e) fp[e] = (_Float16)sc[t][8 * u + e];
#pragma unroll
      for (int a = 0; a < D / 32; ++a) {
        const int8_t *vb = s_v + (32 * a + l32) * VS + (32 * (t0 + t) + 16 * u + 4 * half) * 2;
        const h4 lo = *reinterpret_cast<const h4 *>(vb), hi = *reinterpret_cast<const h4 *>(vb + 16);
        const h8 fv = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        oc[a] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fv, fp, oc[a], 0, 0, 0);
      }
    }
}

// Normalizes, quantizes and stores one query's output row.  O^T: register 4 g + r of tile a is channel
// 32 a + 8 g + 4 half + r of this lane's query; `sum` is the lane-local sum of weights.
template <int D>
__device__ __forceinline__ void attention_store_row(const AttnParams &p, float sum, const v16f (&oc)[D / 32], int8_t *orow,
                                                    int half, bool store) {
  sum += __shfl_xor(sum, 32, 64);
  const float onorm = p.s * (1.0f / sum);  // sum and the accumulators both carry the factor 1024
  const float zf = (float)p.z_a, inv_sa = 1.0f / p.s_a;
#pragma unroll
  for (int a = 0; a < D / 32; ++a) {
    uint32_t packed[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      uint32_t w = 0;
#pragma unroll
      for (int r = 0; r < 4; ++r) w |= (uint32_t)(quant_code(oc[a][4 * g + r] * onorm, inv_sa, zf) & 0xff) << (8 * r);
      packed[g] = w;
    }
    // lower half-wave holds channels 8g .. 8g+3, upper 8g+4 .. 8g+7: after the two swaps the lower
    // lane owns channels 0 .. 15 of this 32-channel tile and the upper lane 16 .. 31
    const auto s02 = __builtin_amdgcn_permlane32_swap(packed[0], packed[2], false, false);
    const auto s13 = __builtin_amdgcn_permlane32_swap(packed[1], packed[3], false, false);
    const v4i o = {(int)s02[0], (int)s02[1], (int)s13[0], (int)s13[1]};
    if (store) *reinterpret_cast<v4i *>(orow + 32 * a + 16 * half) = o;
  }
}

constexpr int kKeyGroup = 3;  // key tiles per group: 48 score registers live, two workgroups per compute unit

// G heads per workgroup (short sequences: a head of two wavefronts alone would leave the compute unit to
// workgroup turnover); the wavefronts of a head work only on that head's slice of LDS.
template <int NT, int D, int G, bool BIAS>
__global__ __launch_bounds__(64 * NT * G) void attention_int8_kernel(const AttnParams p) {
  constexpr int TP = 32 * NT;
  __shared__ __attribute__((aligned(16))) int8_t s_k_all[G * TP * k_stride(D)];
  __shared__ __attribute__((aligned(16))) int8_t s_v_all[G * D * v_stride(NT)];
  const int slot = threadIdx.x / (64 * NT);  // which of the workgroup's heads
  int8_t *s_k = s_k_all + slot * (TP * k_stride(D));
  int8_t *s_v = s_v_all + slot * (D * v_stride(NT));
  const int tid = threadIdx.x % (64 * NT), lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  // (image, head) pairs beyond the last repeat it and store nothing (every wavefront reaches the barrier)
  int64_t pair = (int64_t)blockIdx.x * G + slot;
  const bool live = pair < p.pairs;
  if (!live) pair = p.pairs - 1;
  const int head = (int)(pair % p.heads);
  const int64_t row0 = (pair / p.heads) * p.tokens;
  const int c = p.heads * D;
  const int8_t *qbase = p.r + row0 * p.ld + head * D;

  const _Float16 zb = (_Float16)(float)(1152 + p.z);
  const h2 zbias = {zb, zb};
  // K and V of the head -> LDS as (code - z) in binary16; rows beyond the last token are zero
  constexpr int CH = D / 8;  // 8-channel chunks per row
  constexpr int IT = CH / 2;  // chunks per thread: TP * CH / (64 * NT)
  // all of the thread's loads go out before the first conversion (one round trip to memory, not IT + 1);
  // a key beyond the last token reads as the zero point, i.e. as (code - z) = 0
  const uint32_t zword = 0x01010101u * (uint32_t)(p.z & 0xff);
  uint2 kraw[IT], vraw[IT];
#pragma unroll
  for (int j = 0; j < IT; ++j) {
    const int i = tid + j * (64 * NT);
    const int key = i / CH, ch = i % CH;
    kraw[j] = vraw[j] = make_uint2(zword, zword);
    if (key < p.tokens) {
      kraw[j] = *reinterpret_cast<const uint2 *>(qbase + key * p.ld + c + 8 * ch);
      vraw[j] = *reinterpret_cast<const uint2 *>(qbase + key * p.ld + 2 * c + 8 * ch);
    }
  }
  // this lane's query row as B operands (rows beyond the last token repeat it; never stored)
  const int q = wave * 32 + l32;
  const int qrow = q < p.tokens ? q : p.tokens - 1;
  uint2 qraw[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; ++s)
    qraw[s] = *reinterpret_cast<const uint2 *>(qbase + qrow * p.ld + 16 * s + 8 * half);
#pragma unroll
  for (int j = 0; j < IT; ++j) {
    const int i = tid + j * (64 * NT);
    const int key = i / CH, ch = i % CH;
    const h8 kv = codes_to_h8(kraw[j], zbias), vv = codes_to_h8(vraw[j], zbias);
    *reinterpret_cast<h8 *>(s_k + key * k_stride(D) + ch * 16) = kv;
#pragma unroll
    for (int e = 0; e < 8; ++e) *reinterpret_cast<_Float16 *>(s_v + (8 * ch + e) * v_stride(NT) + key * 2) = vv[e];
  }
  h8 fq[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; ++s) fq[s] = codes_to_h8(qraw[s], zbias);
  __syncthreads();

  // s^2 / sqrt(D) * log2(e)
  const float lscale = p.s * p.s * (D == 64 ? 0.125f : 0.17677669529663687f) * 1.44269504088896340736f;
  // this lane's row of the bias: [head][query][key], rows padded to whole key tiles
  const uint16_t *bias_row = BIAS ? p.bias + ((int64_t)head * p.tokens + qrow) * p.ldb : nullptr;
  float mx = 0.0f, sum = 0.0f;
  v16f oc[D / 32];
#pragma unroll
  for (int a = 0; a < D / 32; ++a)
#pragma unroll
    for (int i = 0; i < 16; ++i) oc[a][i] = 0.0f;
#pragma unroll
  for (int g = 0; g < NT / kKeyGroup; ++g) {
    attention_key_group<kKeyGroup, D, v_stride(NT), BIAS>(g * kKeyGroup, g == 0, s_k, s_v, fq, bias_row, p.tokens, lscale, l32, half, mx, sum, oc);
    __builtin_amdgcn_sched_barrier(0);  // one group's score tiles live at a time
  }
  if constexpr (NT % kKeyGroup != 0)
    attention_key_group<NT % kKeyGroup, D, v_stride(NT), BIAS>(NT / kKeyGroup * kKeyGroup, NT < kKeyGroup, s_k, s_v, fq,
                                                               bias_row, p.tokens, lscale, l32,
                                        half, mx, sum, oc);

  attention_store_row<D>(p, sum, oc, p.a + (row0 + qrow) * p.lda + head * D, half, q < p.tokens && live);
}

template <int NT, int D>
cwac_status launch_attention(const AttnParams &p, int batch, hipStream_t st) {
  constexpr int G = NT == 1 ? 4 : (NT == 2 ? 2 : 1);  // 256 threads per workgroup for short sequences
  const int64_t blocks = ceil_div((int64_t)batch * p.heads, G);
  if (p.bias)
    attention_int8_kernel<NT, D, G, true><<<dim3((unsigned)blocks), 64 * NT * G, 0, st>>>(p);
  else
    attention_int8_kernel<NT, D, G, false><<<dim3((unsigned)blocks), 64 * NT * G, 0, st>>>(p);
  return launch_status();
}

// Sequences of more than 224 tokens: one workgroup per (image, head, block of 224 queries); the keys and
// values pass through LDS in chunks of 224, the running maximum, sum and accumulators carried from chunk
// to chunk exactly as from key group to key group.
constexpr int kChunkTiles = 7, kChunk = 32 * kChunkTiles;
template <int D, bool BIAS>
__global__ __launch_bounds__(64 * kChunkTiles) void attention_long_kernel(const AttnParams p) {
  constexpr int NT = kChunkTiles;
  __shared__ __attribute__((aligned(16))) int8_t s_k[kChunk * k_stride(D)];
  __shared__ __attribute__((aligned(16))) int8_t s_v[D * v_stride(NT)];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int64_t pair = blockIdx.x;
  const int head = (int)(pair % p.heads);
  const int64_t row0 = (pair / p.heads) * p.tokens;
  const int c = p.heads * D;
  const int8_t *qbase = p.r + row0 * p.ld + head * D;
  const _Float16 zb = (_Float16)(float)(1152 + p.z);
  const h2 zbias = {zb, zb};

  const int q0 = blockIdx.y * kChunk + wave * 32;  // this wavefront's first query
  const bool wave_live = q0 < p.tokens;            // otherwise it only helps to fill LDS
  const int q = q0 + l32;
  const int qrow = q < p.tokens ? q : p.tokens - 1;
  h8 fq[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; ++s) {
    fq[s] = codes_to_h8(*reinterpret_cast<const uint2 *>(qbase + (int64_t)qrow * p.ld + 16 * s + 8 * half), zbias);
  }
  const float lscale = p.s * p.s * (D == 64 ? 0.125f : 0.17677669529663687f) * 1.44269504088896340736f;
  const uint16_t *bias_row = BIAS ? p.bias + ((int64_t)head * p.tokens + qrow) * p.ldb : nullptr;
  float mx = 0.0f, sum = 0.0f;
  v16f oc[D / 32];
#pragma unroll
  for (int a = 0; a < D / 32; ++a)
#pragma unroll
    for (int i = 0; i < 16; ++i) oc[a][i] = 0.0f;

  constexpr int CH = D / 8;
  for (int key0 = 0; key0 < p.tokens; key0 += kChunk) {
    // the chunk's loads first (one round trip), then the conversions; keys beyond the last token read as the
    // zero point, i.e. as (code - z) = 0
    static_assert(kChunk * CH % (64 * NT) == 0, "whole chunks per thread");
    constexpr int IT = kChunk * CH / (64 * NT);
    const uint32_t zword = 0x01010101u * (uint32_t)(p.z & 0xff);
    uint2 kraw[IT], vraw[IT];
#pragma unroll
    for (int j = 0; j < IT; ++j) {
      const int i = tid + j * (64 * NT);
      const int kl = i / CH, ch = i % CH, key = key0 + kl;
      kraw[j] = vraw[j] = make_uint2(zword, zword);
      if (key < p.tokens) {
        kraw[j] = *reinterpret_cast<const uint2 *>(qbase + (int64_t)key * p.ld + c + 8 * ch);
        vraw[j] = *reinterpret_cast<const uint2 *>(qbase + (int64_t)key * p.ld + 2 * c + 8 * ch);
      }
    }
    if (key0 > 0) __syncthreads();  // every wavefront is done with the previous chunk
#pragma unroll
    for (int j = 0; j < IT; ++j) {
      const int i = tid + j * (64 * NT);
      const int kl = i / CH, ch = i % CH;
      const h8 kv = codes_to_h8(kraw[j], zbias), vv = codes_to_h8(vraw[j], zbias);
      *reinterpret_cast<h8 *>(s_k + kl * k_stride(D) + ch * 16) = kv;
#pragma unroll
      for (int e = 0; e < 8; ++e) *reinterpret_cast<_Float16 *>(s_v + (8 * ch + e) * v_stride(NT) + kl * 2) = vv[e];
    }
    __syncthreads();
    if (wave_live) {
#pragma unroll
      for (int t0 = 0; t0 + kKeyGroup <= NT; t0 += kKeyGroup) {
        if (key0 + 32 * t0 < p.tokens)
          attention_key_group<kKeyGroup, D, v_stride(NT), BIAS, true>(t0, key0 + t0 == 0, s_k, s_v, fq, bias_row, p.tokens,
                                                                     lscale, l32, half, mx, sum, oc, key0);
      }
      constexpr int TAIL = NT / kKeyGroup * kKeyGroup;
      if (NT % kKeyGroup != 0 && key0 + 32 * TAIL < p.tokens)
        attention_key_group<(NT % kKeyGroup ? NT % kKeyGroup : 1), D, v_stride(NT), BIAS, true>(
            TAIL, false, s_k, s_v, fq, bias_row, p.tokens, lscale, l32, half, mx, sum, oc, key0);
    }
  }
  if (wave_live)
    attention_store_row<D>(p, sum, oc, p.a + (row0 + qrow) * p.lda + head * D, half, q < p.tokens);
}

template <int D>
cwac_status launch_attention_long(const AttnParams &p, int batch, hipStream_t st) {
  const dim3 grid((unsigned)((int64_t)batch * p.heads), (unsigned)ceil_div(p.tokens, kChunk));
  if (p.bias)
    attention_long_kernel<D, true><<<grid, 64 * kChunkTiles, 0, st>>>(p);
  else
    attention_long_kernel<D, false><<<grid, 64 * kChunkTiles, 0, st>>>(p);
  return launch_status();
}

template <int D>
cwac_status launch_attention_d(const AttnParams &p, int batch, hipStream_t st) {
  if (p.tokens > kChunk) return launch_attention_long<D>(p, batch, st);
  switch ((p.tokens + 31) / 32) {
    case 1: return launch_attention<1, D>(p, batch, st);
    case 2: return launch_attention<2, D>(p, batch, st);
    case 3: return launch_attention<3, D>(p, batch, st);
    case 4: return launch_attention<4, D>(p, batch, st);
    case 5: return launch_attention<5, D>(p, batch, st);
    case 6: return launch_attention<6, D>(p, batch, st);
    default: return launch_attention<7, D>(p, batch, st);
  }
}

}  // namespace
}  // namespace cwac

using namespace cwac;

extern "C" {

cwac_status vit_residual_ln_quant(const uint16_t *h, int64_t ldh, const int8_t *r, int64_t ldr, float s_r,
                                  int32_t z_r, uint16_t *h_out, int64_t ldho, const float *gamma,
                                  const float *beta, float eps, float s_x, int32_t z_x, int8_t *x_q,
                                  int64_t ldxq, int64_t m, int32_t c, void *stream) {
  if (!h || (!r && !x_q)) return CWAC_E_NULL;
  if (x_q && (!gamma || !beta)) return CWAC_E_NULL;
  if (h_out && !r) return CWAC_E_MODE;
  if (m < 1 || c < 8 || c % 8 != 0 || c > 2048 || ldh < c || (r && ldr < c) || (h_out && ldho < c) ||
      (x_q && ldxq < c) || m > 0x7fffffff)
    return CWAC_E_SHAPE;
  if (!(s_x > 0.0f) && x_q) return CWAC_E_MODE;
  if (!aligned(h, 16) || ldh % 8 != 0 || (r && (!aligned(r, 8) || ldr % 8 != 0)) ||
      (h_out && (!aligned(h_out, 16) || ldho % 8 != 0)) || (x_q && (!aligned(x_q, 8) || ldxq % 8 != 0)) ||
      (x_q && (!aligned(gamma, 16) || !aligned(beta, 16))))
    return CWAC_E_ALIGN;
  LnParams p;
  p.h = reinterpret_cast<const _Float16 *>(h);
  p.ldh = ldh;
  p.r = r;
  p.ldr = ldr;
  p.s_r = s_r;
  p.z_r = z_r;
  p.h_out = reinterpret_cast<_Float16 *>(h_out);
  p.ldho = ldho;
  p.gamma = gamma;
  p.beta = beta;
  p.eps = eps;
  p.inv_s_x = x_q ? 1.0f / s_x : 1.0f;
  p.inv_c = 1.0f / (float)c;
  p.z_x = z_x;
  p.x_q = x_q;
  p.ldxq = ldxq;
  p.m = m;
  p.c = c;
  // lanes per row and vectors per lane: the pair with the fewest idle vector slots, ties to the wider group
  const int nvec = c / 8;
  int lpr = 64, nv = (nvec + 63) / 64;
  for (int cand = 32; cand >= 16; cand /= 2) {
    const int cnv = (nvec + cand - 1) / cand;
    if (cnv <= 4 && cnv * cand < nv * lpr) lpr = cand, nv = cnv;
  }
  // at most 8 workgroups per compute unit: beyond that a lane group walks several rows
  int64_t blocks = ceil_div(m, 256 / lpr);
  if (blocks > 2048) blocks = 2048;
  const dim3 grid((unsigned)blocks);
  hipStream_t st = as_stream(stream);
#define CWAC_LN_CASE(L, N)                                                                     \
  if (lpr == L && nv == N) {                                                                   \
    if (nvec == L * N)                                                                         \
      residual_ln_quant_kernel<L, N, true><<<grid, 256, 0, st>>>(p);                           \
    else                                                                                       \
      residual_ln_quant_kernel<L, N, false><<<grid, 256, 0, st>>>(p);                          \
  }
  // clang-format off
  CWAC_LN_CASE(64, 1) else CWAC_LN_CASE(64, 2) else CWAC_LN_CASE(64, 3) else CWAC_LN_CASE(64, 4)
  else CWAC_LN_CASE(32, 1) else CWAC_LN_CASE(32, 2) else CWAC_LN_CASE(32, 3) else CWAC_LN_CASE(32, 4)
  else CWAC_LN_CASE(16, 1) else CWAC_LN_CASE(16, 2) else CWAC_LN_CASE(16, 3) else CWAC_LN_CASE(16, 4)
  else return CWAC_E_SHAPE;
  // clang-format on
#undef CWAC_LN_CASE
  return launch_status();
}

cwac_status vit_gelu_table(float s_in, int32_t z_in, float s_out, int32_t z_out, int8_t *table, void *stream) {
  if (!table) return CWAC_E_NULL;
  if (!(s_in > 0.0f) || !(s_out > 0.0f)) return CWAC_E_MODE;
  gelu_table_kernel<<<1, 256, 0, as_stream(stream)>>>(s_in, z_in, s_out, z_out, table);
  return launch_status();
}

cwac_status vit_table_lookup(const int8_t *in, int64_t ld_in, const int8_t *table, int8_t *out, int64_t ld_out,
                             int64_t m, int32_t n, void *stream) {
  if (!in || !table || !out) return CWAC_E_NULL;
  if (m < 1 || n < 16 || n % 16 != 0 || ld_in < n || ld_out < n) return CWAC_E_SHAPE;
  if (!aligned(in, 16) || !aligned(out, 16) || ld_in % 16 != 0 || ld_out % 16 != 0) return CWAC_E_ALIGN;
  const int64_t vecs = m * (n / 16);
  int64_t blocks = ceil_div(vecs, 256);
  if (blocks > 256 * 16) blocks = 256 * 16;  // grid-stride beyond 16 workgroups per compute unit
  table_lookup_kernel<<<dim3((unsigned)blocks), 256, 0, as_stream(stream)>>>(in, ld_in, table, out, ld_out, m, n);
  return launch_status();
}

cwac_status vit_attention_int8(const int8_t *r_qkv, int64_t ld, float s, int32_t z, int32_t batch, int32_t tokens,
                               int32_t heads, int32_t head_dim, const uint16_t *bias, int64_t ldb, float s_a,
                               int32_t z_a, int8_t *a_q, int64_t lda, void *stream) {
  if (!r_qkv || !a_q) return CWAC_E_NULL;
  if (bias && (ldb < 32 * ((tokens + 31) / 32) || ldb % 4 != 0)) return CWAC_E_SHAPE;
  if (bias && !aligned(bias, 8)) return CWAC_E_ALIGN;
  if (head_dim != 64 && head_dim != 32) return CWAC_E_SHAPE;
  if (batch < 1 || tokens < 1 || tokens > kMaxTokens || heads < 1 || heads > 64) return CWAC_E_SHAPE;
  const int64_t c = (int64_t)heads * head_dim;
  if (ld < 3 * c || lda < c || (int64_t)batch * heads > 0x7fffffff) return CWAC_E_SHAPE;
  if (!(s > 0.0f) || !(s_a > 0.0f) || z < -128 || z > 127) return CWAC_E_MODE;
  if (!aligned(r_qkv, 8) || ld % 8 != 0 || !aligned(a_q, 16) || lda % 16 != 0) return CWAC_E_ALIGN;
  if (tokens * ld > 0x7fffffff) return CWAC_E_SHAPE;  // 32-bit row offsets inside one image
  AttnParams p;
  p.r = r_qkv;
  p.ld = ld;
  p.s = s;
  p.z = z;
  p.tokens = tokens;
  p.heads = heads;
  p.pairs = (int64_t)batch * heads;
  p.bias = bias;
  p.ldb = ldb;
  p.s_a = s_a;
  p.z_a = z_a;
  p.a = a_q;
  p.lda = lda;
  hipStream_t st = as_stream(stream);
  return head_dim == 64 ? launch_attention_d<64>(p, batch, st) : launch_attention_d<32>(p, batch, st);
}

size_t vit_block_workspace(int32_t batch, int32_t tokens, int32_t heads, int32_t hidden) {
  if (batch < 1 || tokens < 1 || heads < 1 || hidden < 1) return 0;
  const size_t m = (size_t)batch * (size_t)tokens, c = (size_t)heads * kHeadDim;
  return m * (5 * c + (size_t)hidden);
}

}  // extern "C"

namespace {

cwac_status check_block(const vit_block_params *bp) {
  if (!bp->gelu_table || !bp->ln1_gamma || !bp->ln1_beta || !bp->ln2_gamma || !bp->ln2_beta) return CWAC_E_NULL;
  if (bp->batch < 1 || bp->tokens < 1 || bp->heads < 1 || bp->heads > 64 || bp->hidden < 16 || bp->hidden % 16 != 0)
    return CWAC_E_SHAPE;
  if (bp->head_dim != 0 && bp->head_dim != 64 && bp->head_dim != 32) return CWAC_E_SHAPE;
  for (int i = 0; i < 4; ++i)
    if (!bp->layer[i].w_q || !bp->layer[i].mult || !bp->layer[i].offset) return CWAC_E_NULL;
  return CWAC_OK;
}

// One block.  x1_ready: the workspace already holds x1 = Q(LN1(h)) (the block before produced it with its
// last residual); next: the block that follows, whose LN1 and input quantizer then ride on this block's
// last residual pass.  h_out may be h: every kernel that writes the stream reads, in the same lanes, only
// the elements it writes, and the stream is otherwise read by earlier launches only.
cwac_status run_block(const vit_block_params *bp, bool x1_ready, const vit_block_params *next, const uint16_t *h,
                      uint16_t *h_out, void *workspace, void *stream) {
  const int64_t m = (int64_t)bp->batch * bp->tokens;
  const int32_t hd = bp->head_dim ? bp->head_dim : kHeadDim;
  const int32_t c = bp->heads * hd, hid = bp->hidden;
  int8_t *xq = static_cast<int8_t *>(workspace);  // x1, then the attention output, then x2 (then the next x1)
  int8_t *r_qkv = xq + m * c;
  int8_t *r_c = r_qkv + m * 3 * c;  // proj output, then fc2 output
  int8_t *r_h = r_c + m * c;        // GELU codes (fc1's output through the table)
  const vit_block_layer *L = bp->layer;
  auto params = [&](int i) {
    cwac_qparams qp;
    qp.mode = CWAC_EPI_INT_OFFSET;
    qp.act_per_token = 0;
    qp.s_x = L[i].s_x;
    qp.z_x = L[i].z_x;
    qp.s_r = L[i].s_r;
    qp.z_r = L[i].z_r;
    qp.qmin = -128;
    qp.qmax = 127;
    return qp;
  };
  auto linear = [&](int i, const int8_t *x, int32_t n, int32_t k, int8_t *out) {
    const cwac_qparams qp = params(i);
    return qlinear_cwac_forward(x, k, L[i].w_q, k, m, n, k, &qp, L[i].mult, L[i].offset, nullptr, nullptr, CWAC_OUT_INT8,
                                out, n, stream);
  };
  cwac_status st;
  if (!x1_ready) {
    st = vit_residual_ln_quant(h, c, nullptr, 0, 0.0f, 0, nullptr, 0, bp->ln1_gamma, bp->ln1_beta, bp->eps, L[0].s_x,
                               L[0].z_x, xq, c, m, c, stream);
    if (st != CWAC_OK) return st;
  }
  if ((st = linear(0, xq, 3 * c, c, r_qkv)) != CWAC_OK) return st;
  st = vit_attention_int8(r_qkv, 3 * c, L[0].s_r, L[0].z_r, bp->batch, bp->tokens, bp->heads, hd, bp->attn_bias, bp->attn_bias_ld,
                          L[1].s_x, L[1].z_x, xq, c, stream);
  if (st != CWAC_OK) return st;
  if ((st = linear(1, xq, c, c, r_c)) != CWAC_OK) return st;
  st = vit_residual_ln_quant(h, c, r_c, c, L[1].s_r, L[1].z_r, h_out, c, bp->ln2_gamma, bp->ln2_beta, bp->eps, L[2].s_x,
                             L[2].z_x, xq, c, m, c, stream);
  if (st != CWAC_OK) return st;
  {  // fc1 with the GELU table in its epilogue (large layers) or as a pass in place behind it
    const cwac_qparams qp = params(2);
    st = qlinear_cwac_forward_table(xq, c, L[2].w_q, c, m, hid, c, &qp, L[2].mult, L[2].offset, bp->gelu_table, r_h,
                                    hid, stream);
    if (st != CWAC_OK) return st;
  }
  if ((st = linear(3, r_h, c, hid, r_c)) != CWAC_OK) return st;
  // h2 = RN16(h1 + deq(r4)) in place over h1, with the next block's x1 = Q(LN1(h2)) in the same pass
  if (next)
    return vit_residual_ln_quant(h_out, c, r_c, c, L[3].s_r, L[3].z_r, h_out, c, next->ln1_gamma, next->ln1_beta,
                                 next->eps, next->layer[0].s_x, next->layer[0].z_x, xq, c, m, c, stream);
  return vit_residual_ln_quant(h_out, c, r_c, c, L[3].s_r, L[3].z_r, h_out, c, nullptr, nullptr, 0.0f, 1.0f, 0, nullptr,
                               0, m, c, stream);
}

}  // namespace

extern "C" {

cwac_status vit_block_w8a8_forward(const vit_block_params *bp, const uint16_t *h, uint16_t *h_out, void *workspace,
                                   size_t workspace_bytes, void *stream) {
  return vit_encoder_w8a8_forward(bp, 1, h, h_out, workspace, workspace_bytes, stream);
}

cwac_status vit_encoder_w8a8_forward(const vit_block_params *blocks, int32_t n_blocks, const uint16_t *h,
                                     uint16_t *h_out, void *workspace, size_t workspace_bytes, void *stream) {
  if (!blocks || !h || !h_out || !workspace) return CWAC_E_NULL;
  if (n_blocks < 1) return CWAC_E_SHAPE;
  for (int b = 0; b < n_blocks; ++b) {
    const cwac_status st = check_block(blocks + b);
    if (st != CWAC_OK) return st;
    if (blocks[b].batch != blocks[0].batch || blocks[b].tokens != blocks[0].tokens ||
        blocks[b].heads != blocks[0].heads || blocks[b].hidden != blocks[0].hidden ||
        blocks[b].head_dim != blocks[0].head_dim)  // (each block may bring its own attention bias)
      return CWAC_E_SHAPE;
  }
  if (workspace_bytes < vit_block_workspace(blocks[0].batch, blocks[0].tokens, blocks[0].heads, blocks[0].hidden))
    return CWAC_E_WORKSPACE;
  if (!aligned(workspace, 16)) return CWAC_E_ALIGN;
  for (int b = 0; b < n_blocks; ++b) {
    const cwac_status st = run_block(blocks + b, b > 0, b + 1 < n_blocks ? blocks + b + 1 : nullptr, b == 0 ? h : h_out,
                                     h_out, workspace, stream);
    if (st != CWAC_OK) return st;
  }
  return CWAC_OK;
}

}  // extern "C"
