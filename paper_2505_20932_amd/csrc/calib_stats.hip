// Per-output-channel calibration statistics for the CWAC fit (Sec. 3.3, Eq. 3-5).
//
// The pass is a pure streaming read of Y_full and Y_quant (8 bytes per row and
// channel), so the kernel is shaped for HBM bandwidth: every lane owns 4
// adjacent channels (one 16-byte load per matrix and row), a wavefront covers
// 1 KiB of contiguous row, 16 loads are in flight per lane, the streaming loop
// touches no LDS and no barrier, and nothing is written but O(channels) partial
// sums (the four wavefronts of a workgroup add theirs up through LDS first).  Sums are taken of pivot-shifted values
// in fp64, so channels whose mean dwarfs their spread lose no precision, and in a
// fixed order (no floating-point atomics), so results are bit-reproducible.
#include <mutex>

#include "cwac_internal.h"

namespace cwac {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
// Row split of one call: the same function sizes the workspace and the launch.
// The unit of work is a WAVE TASK: one wavefront owns 64*VEC adjacent channels over a block of
// rows.  The four wavefronts of a workgroup take four consecutive row blocks of the SAME channel
// group and add their sums up before writing, so there is one partial sum per channel and
// workgroup (row group); consecutive workgroups take adjacent channel groups.
struct Split {
  int col_groups;       // wave tasks along channels
  int row_blocks;       // wave tasks along rows
  int row_groups;       // workgroups along rows = number of partial sums per channel
  int64_t rows_per_block;
};

inline Split make_split(int64_t n_rows, int c_out, int vec) {
  Split s;
  s.col_groups = (int)ceil_div(c_out, kWave * vec);
  // As many tasks as the chip holds at once: 256 compute units x 4 SIMDs x 3 resident wavefronts
  // (the kernel's register budget).  All tasks then start together, do equal work and finish
  // together; a few more than that would leave a second, nearly empty round.
  const int64_t resident_tasks = 256 * 4 * 3;
  int64_t rb = resident_tasks / s.col_groups / kWaves * kWaves;
  const int64_t max_rb = ceil_div(n_rows, 64);  // at least 64 rows per task
  if (rb > max_rb) rb = max_rb;
  if (rb < 1) rb = 1;
  s.rows_per_block = ceil_div(n_rows, rb);
  s.row_blocks = (int)ceil_div(n_rows, s.rows_per_block);
  s.row_groups = (int)ceil_div(s.row_blocks, kWaves);
  return s;
}

template <int VEC>
struct Ld;
typedef float vf4 __attribute__((ext_vector_type(4)));
template <>
struct Ld<4> {
  using T = vf4;
  __device__ static void unpack(const vf4 &v, float (&o)[4]) {
    o[0] = v[0]; o[1] = v[1]; o[2] = v[2]; o[3] = v[3];
  }
};
template <>
struct Ld<1> {
  using T = float;
  __device__ static void unpack(const float &v, float (&o)[1]) { o[0] = v; }
};

// Stage 1.  One wave task per wavefront: lane l owns channels c0 + VEC*l .. +VEC-1 and walks
// its row block with 2*U to 4*U 16-byte loads in flight.  Workgroup (cg, rg) = channel group cg,
// row blocks 4*rg .. 4*rg+3; partial[rg][stat][channel] receives the sum of its four tasks,
// added in wavefront order.
template <int VEC>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(3, 8))) void stats_partial_kernel(
    const float *__restrict__ yf, int64_t ldf, const float *__restrict__ yq, int64_t ldq,
    int64_t n_rows, int c_out, int col_groups, int row_blocks, int64_t rows_per_block,
    const void *stats, int fresh, double *__restrict__ partial) {
  using V = typename Ld<VEC>::T;
  __shared__ double red[kWaves - 1][kStats * VEC][kWave];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int cg = (int)(blockIdx.x % (unsigned)col_groups);
  const int rg = (int)(blockIdx.x / (unsigned)col_groups);
  const int rb = rg * kWaves + wave;
  const int c = (cg * kWave + lane) * VEC;
  // VEC == 4 requires c_out % 4 == 0, so a lane is all in or all out
  const bool lane_in = c < c_out;
  const bool active = lane_in && rb < row_blocks;

  const StatsView sv = stats_view(const_cast<void *>(stats), c_out);
  // fresh: the caller declares the state empty (its contents are not even read)
  const bool first = fresh ? true : (*sv.n == 0);
  float pq[VEC], pf[VEC];
#pragma unroll
  for (int j = 0; j < VEC; ++j) pq[j] = pf[j] = 0.0f;
  if (active) {
    V vq = first ? *reinterpret_cast<const V *>(yq + c) : *reinterpret_cast<const V *>(sv.pivot_q + c);
    V vf = first ? *reinterpret_cast<const V *>(yf + c) : *reinterpret_cast<const V *>(sv.pivot_f + c);
    Ld<VEC>::unpack(vq, pq);
    Ld<VEC>::unpack(vf, pf);
  }

  double acc[VEC][kStats];
#pragma unroll
  for (int j = 0; j < VEC; ++j)
#pragma unroll
    for (int s = 0; s < kStats; ++s) acc[j][s] = 0.0;

  const int64_t r_begin = active ? rb * rows_per_block : 0;
  int64_t r_end = active ? r_begin + rows_per_block : 0;  // inactive tasks walk no rows
  if (r_end > n_rows) r_end = n_rows;

  auto consume = [&](const V &vq, const V &vf) {
    float q[VEC], f[VEC];
    Ld<VEC>::unpack(vq, q);
    Ld<VEC>::unpack(vf, f);
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
      const double dq = (double)(q[j] - pq[j]);
      const double df = (double)(f[j] - pf[j]);
      acc[j][0] += dq;
      acc[j][1] += df;
      acc[j][2] = fma(dq, dq, acc[j][2]);  // explicit fused ops: sums carry no bit-exactness contract
      acc[j][3] = fma(dq, df, acc[j][3]);
      acc[j][4] = fma(df, df, acc[j][4]);
    }
  };

  // Software pipeline over batches of U rows: the 2*U loads of the next batch are issued
  // before the current batch is consumed, so every wavefront always has loads in flight.
  constexpr int U = 4;
  const float *pq_row = yq + r_begin * ldq + c;
  const float *pf_row = yf + r_begin * ldf + c;
  auto load_batch = [&](V(&vq)[U], V(&vf)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      vq[u] = __builtin_nontemporal_load(reinterpret_cast<const V *>(pq_row + u * ldq));
      vf[u] = __builtin_nontemporal_load(reinterpret_cast<const V *>(pf_row + u * ldf));
    }
    pq_row += U * ldq;
    pf_row += U * ldf;
  };
  auto consume_batch = [&](const V(&vq)[U], const V(&vf)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) consume(vq[u], vf[u]);
  };
  const int64_t n_batches = (r_end - r_begin) / U;
  V aq[U], af[U], bq[U], bf[U];
  if (n_batches > 0) load_batch(aq, af);
  int64_t b = 0;
  for (; b + 2 < n_batches; b += 2) {
    load_batch(bq, bf);
    __builtin_amdgcn_sched_barrier(0);
    consume_batch(aq, af);
    __builtin_amdgcn_sched_barrier(0);
    load_batch(aq, af);
    __builtin_amdgcn_sched_barrier(0);
    consume_batch(bq, bf);
    __builtin_amdgcn_sched_barrier(0);
  }
  if (b < n_batches) {  // one or two batches left; the first is already in flight
    if (b + 1 < n_batches) load_batch(bq, bf);
    consume_batch(aq, af);
    if (b + 1 < n_batches) consume_batch(bq, bf);
  }
  for (int64_t r = r_begin + n_batches * U; r < r_end; ++r) {
    const V vq = *reinterpret_cast<const V *>(pq_row);
    const V vf = *reinterpret_cast<const V *>(pf_row);
    pq_row += ldq;
    pf_row += ldf;
    consume(vq, vf);
  }

  // wavefronts 1..3 hand their sums to wavefront 0, which adds them in order and writes
  if (wave > 0) {
#pragma unroll
    for (int s = 0; s < kStats; ++s)
#pragma unroll
      for (int j = 0; j < VEC; ++j) red[wave - 1][s * VEC + j][lane] = acc[j][s];
  }
  __syncthreads();
  if (wave == 0 && lane_in) {
#pragma unroll
    for (int s = 0; s < kStats; ++s)
#pragma unroll
      for (int j = 0; j < VEC; ++j) {
        double t = acc[j][s];
#pragma unroll
        for (int w = 0; w < kWaves - 1; ++w) t += red[w][s * VEC + j][lane];
        partial[((int64_t)rg * kStats + s) * c_out + c + j] = t;
      }
  }
}

// Stage 2: fixed-order sum over row groups, added into the state; the first batch also
// records the pivots (row 0 of that batch).  A task = (statistic, 64 channels); a workgroup holds G
// tasks of W wavefronts each: wavefront w of a task sums row groups w, w + W, ... (eight loads in
// flight per lane) and the W wave sums are combined in order.  W follows the number of row groups;
// G keeps the workgroups few, because each ends with one ticket on a single counter and those
// serialize (960 tickets cost as much as the rest of the kernel).
// The last workgroup to finish bumps the row count: every workgroup reads the count before
// it takes its ticket, so none can see the new value.  fresh (a run's first batch, state taken as
// empty): nobody reads the count, so workgroup 0 simply writes the whole 64-byte header.
template <int W, int G>
__global__ __launch_bounds__(W *G *kWave) void stats_merge_kernel(
    const double *__restrict__ partial, int row_blocks, int c_out, const float *__restrict__ yf,
    const float *__restrict__ yq, void *stats, int64_t n_rows, int fresh) {
  const int groups = (c_out + kWave - 1) / kWave;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int g = wave / W, w = wave % W;
  const int task = blockIdx.x * G + g;
  const bool has_task = task < kStats * groups;
  const int s = has_task ? task / groups : 0, cg = has_task ? task - s * groups : 0;
  const int ch = cg * kWave + lane;
  const bool active = has_task && ch < c_out;
  const StatsView sv = stats_view(stats, c_out);
  const bool first = fresh ? true : (*sv.n == 0);
  double t = 0.0;
  if (active) {
    const double *src = partial + (int64_t)s * c_out + ch;
    const int64_t step = (int64_t)kStats * c_out;
    int rb = w;
    for (; rb + 7 * W < row_blocks; rb += 8 * W) {
      double a[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) a[j] = src[(int64_t)(rb + j * W) * step];
#pragma unroll
      for (int j = 0; j < 8; ++j) t += a[j];
    }
    for (; rb < row_blocks; rb += W) t += src[(int64_t)rb * step];
  }
  double total = t;
  if (W > 1) {
    __shared__ double red[G][W][kWave];
    red[g][w][lane] = t;
    __syncthreads();
    if (w == 0) {
      total = red[g][0][lane];
#pragma unroll
      for (int i = 1; i < W; ++i) total += red[g][i][lane];
    }
  }
  if (w == 0 && active) {
    const int i = s * c_out + ch;
    sv.sum[i] = first ? total : sv.sum[i] + total;
    if (first && s == 0) {
      sv.pivot_q[ch] = yq[ch];
      sv.pivot_f[ch] = yf[ch];
    }
  }
  if (fresh) {
    if (blockIdx.x == 0 && threadIdx.x < kStatsHeaderBytes / 4) {
      uint32_t v = 0;  // header: int64 row count, int32 channel count, zeros (ticket included)
      if (threadIdx.x == 0) v = (uint32_t)((uint64_t)n_rows & 0xffffffffu);
      if (threadIdx.x == 1) v = (uint32_t)((uint64_t)n_rows >> 32);
      if (threadIdx.x == 2) v = (uint32_t)c_out;
      static_cast<uint32_t *>(stats)[threadIdx.x] = v;
    }
    return;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    // no fence needed: this workgroup's read of the count has already returned its value, and
    // its sums only have to be visible at the end of the kernel
    unsigned *ticket = reinterpret_cast<unsigned *>(static_cast<char *>(stats) + 16);
    if (atomicAdd(ticket, 1u) == gridDim.x - 1) {
      *ticket = 0;
      *sv.n += n_rows;
    }
  }
}

__global__ __launch_bounds__(kThreads) void stats_reset_kernel(void *stats, int c_out,
                                                               size_t words) {
  const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (i < words) {
    uint32_t v = 0;
    if (i == 2) v = (uint32_t)c_out;  // bytes 8..11
    static_cast<uint32_t *>(stats)[i] = v;
  }
}

__global__ void zero_i32_kernel(int32_t *p) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *p = 0;
}

// Eq. 4-5 from the shifted sums, fp64.
// Eq. 4-5 per channel; grid-stride over channels.  With several workgroups the fallback count is
// added atomically (integer, order-independent) to a counter the host zeroed beforehand.
__global__ __launch_bounds__(256) void solve_kernel(const void *stats, int c_out, double var_eps,
                                                     float *__restrict__ alpha,
                                                     float *__restrict__ beta,
                                                     double *__restrict__ moments,
                                                     int32_t *__restrict__ n_degenerate) {
  const StatsView sv = stats_view(const_cast<void *>(stats), c_out);
  const int64_t n = *sv.n;
  int deg = 0;
  for (int ch = blockIdx.x * blockDim.x + threadIdx.x; ch < c_out; ch += gridDim.x * blockDim.x) {
    double mf = 0.0, mq = 0.0, vq = 0.0, cqf = 0.0, vf = 0.0;
    if (n > 0) {
      const double dn = (double)n;
      const double sq = sv.sum[ch], sf = sv.sum[c_out + ch];
      const double eq = sq / dn, ef = sf / dn;  // means of the shifted values
      mq = (double)sv.pivot_q[ch] + eq;
      mf = (double)sv.pivot_f[ch] + ef;
      vq = sv.sum[2 * c_out + ch] / dn - eq * eq;
      cqf = sv.sum[3 * c_out + ch] / dn - eq * ef;
      vf = sv.sum[4 * c_out + ch] / dn - ef * ef;
      if (vq < 0.0) vq = 0.0;
      if (vf < 0.0) vf = 0.0;
    }
    double m2 = mq * mq;
    if (m2 < 1e-300) m2 = 1e-300;
    double a, b;
    if (n <= 0 || !(vq > var_eps * m2) || cqf == 0.0) {
      a = 1.0;
      b = mf - mq;
      ++deg;
    } else {
      a = cqf / vq;
      b = mf - a * mq;
    }
    alpha[ch] = (float)a;
    beta[ch] = (float)b;
    if (moments) {
      moments[ch] = mf;
      moments[c_out + ch] = mq;
      moments[2 * c_out + ch] = vq;
      moments[3 * c_out + ch] = cqf;
      moments[4 * c_out + ch] = vf;
    }
  }
  if (n_degenerate) {
    __shared__ int s_deg[256 / kWave];
    deg = wave_sum(deg);
    if ((threadIdx.x & (kWave - 1)) == 0) s_deg[threadIdx.x / kWave] = deg;
    __syncthreads();
    if (threadIdx.x == 0) {
      int t = 0;
      for (int i = 0; i < (int)(blockDim.x / kWave); ++i) t += s_deg[i];
      if (gridDim.x == 1) *n_degenerate = t;
      else if (t) atomicAdd(n_degenerate, t);
    }
  }
}

}  // namespace

cwac_status launch_stats_merge(const double *partial, int row_groups, int c_out,
                               const float *pivot_f_src, const float *pivot_q_src, void *stats,
                               int64_t n_rows, bool fresh, hipStream_t st) {
  const int tasks = (int)(kStats * ceil_div(c_out, kWave));
  const int fr = fresh ? 1 : 0;
  if (row_groups <= 32)
    stats_merge_kernel<1, 8><<<(unsigned)ceil_div(tasks, 8), 8 * kWave, 0, st>>>(partial, row_groups, c_out, pivot_f_src,
                                                                             pivot_q_src, stats, n_rows, fr);
  else if (row_groups <= 128)
    stats_merge_kernel<4, 4><<<(unsigned)ceil_div(tasks, 4), 16 * kWave, 0, st>>>(partial, row_groups, c_out,
                                                                              pivot_f_src, pivot_q_src, stats, n_rows, fr);
  else
    stats_merge_kernel<16, 1><<<(unsigned)tasks, 16 * kWave, 0, st>>>(partial, row_groups, c_out, pivot_f_src,
                                                                      pivot_q_src, stats, n_rows, fr);
  return launch_status();
}

// Argument checks and the two launches shared by the statistics entry points.  `partial` is the
// caller's workspace (or the library's static scratch), already known to be large enough.
static cwac_status calibrate_stats_impl(const float *y_full, int64_t ld_full, const float *y_quant,
                                        int64_t ld_quant, int64_t n_rows, int32_t c_out, void *stats,
                                        double *partial, bool fresh, hipStream_t st) {
  const bool vec = (c_out % 4 == 0) && (ld_full % 4 == 0) && (ld_quant % 4 == 0) &&
                   aligned(y_full, 16) && aligned(y_quant, 16);
  const Split sp = make_split(n_rows, c_out, vec ? 4 : 1);
  const int64_t blocks = (int64_t)sp.col_groups * sp.row_groups;
  if (blocks > 0x7fffffff) return CWAC_E_SHAPE;
  const unsigned grid = (unsigned)blocks;
  const int fr = fresh ? 1 : 0;
  if (vec)
    stats_partial_kernel<4><<<grid, kThreads, 0, st>>>(y_full, ld_full, y_quant, ld_quant, n_rows,
                                                       c_out, sp.col_groups, sp.row_blocks,
                                                       sp.rows_per_block, stats, fr, partial);
  else
    stats_partial_kernel<1><<<grid, kThreads, 0, st>>>(y_full, ld_full, y_quant, ld_quant, n_rows,
                                                       c_out, sp.col_groups, sp.row_blocks,
                                                       sp.rows_per_block, stats, fr, partial);
  const cwac_status rc = launch_status();
  if (rc != CWAC_OK) return rc;
  return launch_stats_merge(partial, sp.row_groups, c_out, y_full, y_quant, stats, n_rows, fresh, st);
}

static cwac_status calibrate_stats_check(const float *y_full, int64_t ld_full, const float *y_quant,
                                         int64_t ld_quant, int64_t n_rows, int32_t c_out, const void *stats) {
  if (!stats) return CWAC_E_NULL;
  if (c_out < 1 || c_out > 65536 || n_rows < 0) return CWAC_E_SHAPE;
  if (n_rows == 0) return CWAC_OK;
  if (!y_full || !y_quant) return CWAC_E_NULL;
  if (ld_full < c_out || ld_quant < c_out) return CWAC_E_SHAPE;
  if (!aligned(stats, 16) || !aligned(y_full, 4) || !aligned(y_quant, 4)) return CWAC_E_ALIGN;
  return CWAC_OK;
}

}  // namespace cwac

using namespace cwac;

extern "C" size_t cwac_stats_bytes(int32_t c_out) {
  if (c_out < 1) return 0;
  return (size_t)kStatsHeaderBytes + (size_t)8 * c_out + (size_t)kStats * 8 * c_out;
}

extern "C" cwac_status cwac_stats_reset(void *stats, int32_t c_out, void *stream) {
  if (!stats) return CWAC_E_NULL;
  if (c_out < 1 || c_out > 65536) return CWAC_E_SHAPE;
  if (!aligned(stats, 16)) return CWAC_E_ALIGN;
  const size_t words = cwac_stats_bytes(c_out) / 4;
  stats_reset_kernel<<<(unsigned)ceil_div((int64_t)words, kThreads), kThreads, 0,
                       as_stream(stream)>>>(stats, c_out, words);
  return launch_status();
}

extern "C" size_t cwac_calibrate_stats_workspace(int64_t n_rows, int32_t c_out) {
  if (n_rows < 1 || c_out < 1) return 16;
  // sized for the generic (one channel per lane) split, which never needs less
  const Split a = make_split(n_rows, c_out, 1), b = make_split(n_rows, c_out, 4);
  const int rg = a.row_groups > b.row_groups ? a.row_groups : b.row_groups;
  return (size_t)rg * kStats * c_out * sizeof(double);
}

extern "C" cwac_status cwac_calibrate_stats(const float *y_full, int64_t ld_full,
                                            const float *y_quant, int64_t ld_quant,
                                            int64_t n_rows, int32_t c_out, void *stats,
                                            void *workspace, size_t workspace_bytes,
                                            void *stream) {
  const cwac_status rc = calibrate_stats_check(y_full, ld_full, y_quant, ld_quant, n_rows, c_out, stats);
  if (rc != CWAC_OK || n_rows == 0) return rc;
  if (!workspace || workspace_bytes < cwac_calibrate_stats_workspace(n_rows, c_out))
    return CWAC_E_WORKSPACE;
  if (!aligned(workspace, 16)) return CWAC_E_ALIGN;
  return calibrate_stats_impl(y_full, ld_full, y_quant, ld_quant, n_rows, c_out, stats,
                              static_cast<double *>(workspace), false, as_stream(stream));
}

extern "C" cwac_status cwac_calibrate_stats_first(const float *y_full, int64_t ld_full,
                                                  const float *y_quant, int64_t ld_quant,
                                                  int64_t n_rows, int32_t c_out, void *stats,
                                                  void *workspace, size_t workspace_bytes,
                                                  void *stream) {
  const cwac_status rc = calibrate_stats_check(y_full, ld_full, y_quant, ld_quant, n_rows, c_out, stats);
  if (rc != CWAC_OK) return rc;
  if (n_rows < 1) return CWAC_E_SHAPE;  // a first batch has a first row: it fixes the pivots
  if (!workspace || workspace_bytes < cwac_calibrate_stats_workspace(n_rows, c_out))
    return CWAC_E_WORKSPACE;
  if (!aligned(workspace, 16)) return CWAC_E_ALIGN;
  return calibrate_stats_impl(y_full, ld_full, y_quant, ld_quant, n_rows, c_out, stats,
                              static_cast<double *>(workspace), true, as_stream(stream));
}

// ---- statistics for callers that cannot allocate: the partial sums go to a buffer that is part of
// the library's device image.  Each GPU holds its own copy of the array at its own address; host
// code never uses the array's name as an address, only the per-device pointer looked up below.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on device i, once looked up

static cwac_status static_scratch(double **out) {
  int device = -1;
  if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return CWAC_E_LAUNCH;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return CWAC_E_LAUNCH;
    }
    g_scratch_ptr[device] = ptr;
  }
  *out = static_cast<double *>(g_scratch_ptr[device]);
  return CWAC_OK;
}

extern "C" size_t cwac_static_scratch_bytes(void) { return kStaticScratchBytes; }

extern "C" cwac_status cwac_calibrate_stats_static(const float *y_full, int64_t ld_full,
                                                   const float *y_quant, int64_t ld_quant,
                                                   int64_t n_rows, int32_t c_out, void *stats,
                                                   void *stream) {
  const cwac_status rc = calibrate_stats_check(y_full, ld_full, y_quant, ld_quant, n_rows, c_out, stats);
  if (rc != CWAC_OK || n_rows == 0) return rc;
  if (cwac_calibrate_stats_workspace(n_rows, c_out) > kStaticScratchBytes) return CWAC_E_WORKSPACE;
  double *partial = nullptr;
  const cwac_status rs = static_scratch(&partial);
  if (rs != CWAC_OK) return rs;
  // every partial sum the merge reads is written by this call's first kernel: nothing to clear
  return calibrate_stats_impl(y_full, ld_full, y_quant, ld_quant, n_rows, c_out, stats, partial, false,
                              as_stream(stream));
}

extern "C" cwac_status cwac_solve(const void *stats, int32_t c_out, double var_eps, float *alpha,
                                  float *beta, double *moments, int32_t *n_degenerate,
                                  void *stream) {
  if (!stats || !alpha || !beta) return CWAC_E_NULL;
  if (c_out < 1 || c_out > 65536 || !(var_eps >= 0.0)) return CWAC_E_SHAPE;
  if (!aligned(stats, 16) || !aligned(alpha, 4) || !aligned(beta, 4) ||
      (moments && !aligned(moments, 8)))
    return CWAC_E_ALIGN;
  const unsigned blocks = (unsigned)ceil_div(c_out, 256);
  if (n_degenerate && blocks > 1) zero_i32_kernel<<<1, 64, 0, as_stream(stream)>>>(n_degenerate);
  solve_kernel<<<blocks, 256, 0, as_stream(stream)>>>(stats, c_out, var_eps, alpha, beta, moments,
                                                     n_degenerate);
  return launch_status();
}
