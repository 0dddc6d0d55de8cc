// Diagnostic, not part of the path: what the int8 matrix cores of this device sustain when
// nothing else limits them.  Four wavefronts per workgroup run the forward kernel's register
// pattern (4 x 4 MFMA 32x32x32 tiles per wavefront, 256 accumulators per lane) on operand
// fragments that stay in registers: no LDS, no memory traffic in the timed loop.  The rate
// depends on the CONTENT of the operands (switching activity moves the clock the device can hold
// under its power limit), which is why the caller supplies them.
#include "qlinear_common.h"

namespace cwac {
namespace {

__global__ __launch_bounds__(256) void mfma_probe_kernel(const v4i *__restrict__ operands, int iters,
                                                         int32_t *sink) {
  v4i a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = operands[(threadIdx.x + 64 * i) & 511];
    b[i] = operands[512 + ((threadIdx.x + 64 * i) & 511)];
  }
  v16i acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
  }
  int s = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) s += acc[i][j][e];
  if (s == 0x12345678) sink[0] = s;  // keeps the loop alive; practically never taken
}

// Read-only stream: every lane sums 16-byte non-temporal loads at a grid stride (8 loads in flight per lane).
// What the statistics pass - two such streams and a little arithmetic - can be compared with.
typedef unsigned int probe_u4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void hbm_read_probe_kernel(const probe_u4 *__restrict__ src, size_t n16,
                                                             int32_t *sink) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  probe_u4 s = {0u, 0u, 0u, 0u};
  for (; i + 7 * stride < n16; i += 8 * stride) {
    probe_u4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = __builtin_nontemporal_load(src + i + j * stride);
#pragma unroll
    for (int j = 0; j < 8; ++j) s ^= v[j];
  }
  for (; i < n16; i += stride) s ^= __builtin_nontemporal_load(src + i);
  if ((s.x ^ s.y ^ s.z ^ s.w) == 0x12345678u) sink[0] = 1;  // keeps the loads alive; practically never taken
}

// The same for the binary16 matrix cores (the weight-only layer's MFMA, 32 x 32 x 16, fp32 accumulators).
typedef _Float16 probe_h8 __attribute__((ext_vector_type(8)));
typedef float probe_v16f __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(256) void mfma_probe_f16_kernel(const probe_h8 *__restrict__ operands, int iters,
                                                             int32_t *sink) {
  probe_h8 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = operands[(threadIdx.x + 64 * i) & 511];
    b[i] = operands[512 + ((threadIdx.x + 64 * i) & 511)];
  }
  probe_v16f acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
  }
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) s += acc[i][j][e];
  if (__float_as_int(s) == 0x12345678) sink[0] = 1;  // keeps the loop alive; practically never taken
}

// Second diagnostic: the K loop of the 256 x 256 forward tile (eight wavefronts, two stages of 64 KiB, per
// wavefront and k-step eight MFMAs on 64 tokens x 128 channels) built up one ingredient at a time, so that
// the cost of each shows as a rate: MODE 0 the MFMAs alone on register-resident fragments; 1 + the six
// 16-byte LDS fragment reads per k-step (swizzled panel layout, fragments double-buffered in registers,
// reads interleaved behind the MFMAs); 2 + the wait and workgroup barrier that end a stage; 3 + the panel
// stream (per wavefront and stage eight direct-to-LDS loads of 1 KiB, from a 64 KiB buffer that stays in
// the caches); 4 the same stream issued by wavefronts 0-3 only, sixteen loads each (one loading wavefront per
// SIMD).  No epilogue, no tile start: what is left of the matrix cores' rate inside the loop.
#define CWAC_PROBE_LDS(p) ((__attribute__((address_space(3))) void *)(p))
#define CWAC_PROBE_GLOBAL(p) ((const __attribute__((address_space(1))) void *)(p))

constexpr int probe_wait_all() { return (0 & 15) | (7 << 4) | (0 << 8) | (0 << 14); }  // vmcnt 0, lgkmcnt 0

template <int MODE>
__global__ __launch_bounds__(512, 1) void kloop_probe_kernel(const v4i *__restrict__ operands,
                                                             const int8_t *__restrict__ panels, int stages,
                                                             int32_t *sink) {
  constexpr int BK = 128, STAGE = 65536, X_BYTES = 32768;
  extern __shared__ __attribute__((aligned(16))) int8_t smem[];  // two stages: activation panel, weight panel
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave_m = wave & 3, wave_n = wave >> 2, l32 = lane & 31, half = lane >> 5;
  for (int i = tid; i < 2 * STAGE / 16; i += 512) reinterpret_cast<v4i *>(smem)[i] = operands[i & 1023];
  __syncthreads();
  v4i fwA[4], fxA[2], fwB[4], fxB[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    fwA[i] = operands[(tid + 64 * i) & 511];
    fwB[i] = operands[(tid + 64 * i + 32) & 511];
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    fxA[i] = operands[512 + ((tid + 64 * i) & 511)];
    fxB[i] = operands[512 + ((tid + 64 * i + 32) & 511)];
  }
  v16i acc[4][2];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][b][e] = 0;
  const int swz = (l32 >> 1) & 7;
  const int x_off = (wave_m * 64 + l32) * BK, w_off = X_BYTES + (wave_n * 128 + l32) * BK;
  const int lr = lane >> 3, pc = lane & 7;
  const int8_t *src_x = panels + (wave * 32 + lr) * BK + (pc << 4);  // this wavefront's 32 rows of either panel
  auto read_frags = [&](int buf, int kk, v4i(&fw)[4], v4i(&fx)[2]) {
    const int8_t *base = smem + buf * STAGE + (((2 * kk + half) ^ swz) << 4);
#pragma unroll
    for (int a = 0; a < 4; ++a) fw[a] = *reinterpret_cast<const v4i *>(base + w_off + a * 32 * BK);
#pragma unroll
    for (int b = 0; b < 2; ++b) fx[b] = *reinterpret_cast<const v4i *>(base + x_off + b * 32 * BK);
  };
  auto mma = [&](const v4i(&fw)[4], const v4i(&fx)[2]) {
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b) acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[a], fx[b], acc[a][b], 0, 0, 0);
  };
  auto issue_share = [&](int buf, int region, int share) {  // four loads: 32 rows x 128 bytes of one panel
    int8_t *dst = smem + buf * STAGE + region + share * (32 * BK);
    const int8_t *src = src_x + region + (share - wave) * (32 * BK);
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_global_load_lds(CWAC_PROBE_GLOBAL(src + i * 8 * BK), CWAC_PROBE_LDS(dst + i * 8 * BK), 16, 0, 0);
  };
  auto issue_panel = [&](int buf, int region) {
    if (MODE == 3) {
      issue_share(buf, region, wave);
    } else if (wave < 4) {
      issue_share(buf, region, wave);
      issue_share(buf, region, wave + 4);
    }
  };
  for (int s = 0; s < stages; ++s) {
    const int buf = s & 1;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      if (MODE >= 3 && kk == 0) issue_panel(buf ^ 1, X_BYTES);
      if (MODE >= 3 && kk == 3) issue_panel(buf ^ 1, 0);
      if (kk & 1) {
        if (MODE >= 1) read_frags(buf, (kk + 1) & 3, fwA, fxA);
        mma(fwB, fxB);
      } else {
        if (MODE >= 1) read_frags(buf, (kk + 1) & 3, fwB, fxB);
        mma(fwA, fxA);
      }
      if (MODE >= 1) {
#pragma unroll
        for (int i = 0; i < 6; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        if (MODE == 3 && (kk == 0 || kk == 3)) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);
        } else {
          __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (MODE >= 2) {
      __builtin_amdgcn_s_waitcnt(probe_wait_all());
      __builtin_amdgcn_s_barrier();
    }
  }
  int sum = 0;
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) sum += acc[a][b][e];
  if (sum == 0x12345678) sink[0] = sum;  // keeps the loop alive; practically never taken
}

template <int MODE>
cwac_status launch_kloop_probe(const int32_t *operands, const int8_t *panels, int stages, int workgroups,
                               int32_t *sink, hipStream_t st) {
  constexpr int LDS = 131072;
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(&kloop_probe_kernel<MODE>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
  if (attr != hipSuccess) return CWAC_E_LAUNCH;
  kloop_probe_kernel<MODE><<<(unsigned)workgroups, 512, LDS, st>>>(reinterpret_cast<const v4i *>(operands), panels,
                                                                    stages, sink);
  return launch_status();
}

}  // namespace
}  // namespace cwac

using namespace cwac;

extern "C" cwac_status cwac_kloop_probe(const int32_t *operands, const int8_t *panels, int32_t mode, int32_t stages,
                                        int32_t workgroups, int32_t *sink, void *stream) {
  if (!operands || !panels || !sink) return CWAC_E_NULL;
  if (mode < 0 || mode > 4) return CWAC_E_MODE;
  if (stages < 1 || stages > (1 << 24) || workgroups < 1 || workgroups > (1 << 20)) return CWAC_E_SHAPE;
  if (!aligned(operands, 16) || !aligned(panels, 16)) return CWAC_E_ALIGN;
  hipStream_t st = as_stream(stream);
  switch (mode) {
    case 0: return launch_kloop_probe<0>(operands, panels, stages, workgroups, sink, st);
    case 1: return launch_kloop_probe<1>(operands, panels, stages, workgroups, sink, st);
    case 2: return launch_kloop_probe<2>(operands, panels, stages, workgroups, sink, st);
    case 3: return launch_kloop_probe<3>(operands, panels, stages, workgroups, sink, st);
    default: return launch_kloop_probe<4>(operands, panels, stages, workgroups, sink, st);
  }
}

extern "C" cwac_status cwac_hbm_read_probe(const void *src, size_t bytes, int32_t workgroups, int32_t *sink,
                                           void *stream) {
  if (!src || !sink) return CWAC_E_NULL;
  if (bytes < 16 || workgroups < 1 || workgroups > (1 << 20)) return CWAC_E_SHAPE;
  if (!aligned(src, 16)) return CWAC_E_ALIGN;
  hbm_read_probe_kernel<<<(unsigned)workgroups, 256, 0, as_stream(stream)>>>(
      static_cast<const probe_u4 *>(src), bytes / 16, sink);
  return launch_status();
}

extern "C" cwac_status cwac_mfma_probe_f16(const uint16_t *operands, int32_t iters, int32_t workgroups,
                                           int32_t *sink, void *stream) {
  if (!operands || !sink) return CWAC_E_NULL;
  if (iters < 1 || iters > (1 << 24) || workgroups < 1 || workgroups > (1 << 20)) return CWAC_E_SHAPE;
  if (!aligned(operands, 16)) return CWAC_E_ALIGN;
  mfma_probe_f16_kernel<<<(unsigned)workgroups, 256, 0, as_stream(stream)>>>(
      reinterpret_cast<const probe_h8 *>(operands), iters, sink);
  return launch_status();
}

extern "C" cwac_status cwac_mfma_probe(const int32_t *operands, int32_t iters, int32_t workgroups,
                                       int32_t *sink, void *stream) {
  if (!operands || !sink) return CWAC_E_NULL;
  if (iters < 1 || iters > (1 << 24) || workgroups < 1 || workgroups > (1 << 20)) return CWAC_E_SHAPE;
  if (!aligned(operands, 16)) return CWAC_E_ALIGN;
  mfma_probe_kernel<<<(unsigned)workgroups, 256, 0, as_stream(stream)>>>(
      reinterpret_cast<const v4i *>(operands), iters, sink);
  return launch_status();
}
