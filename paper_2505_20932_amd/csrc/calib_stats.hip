// Per-output-channel calibration statistics for the CWAC fit (Sec. 3.3, Eq. 3-5).
//
// The pass is a pure streaming read of Y_full and Y_quant (8 bytes per row and
// channel), so the kernel is shaped for HBM bandwidth: every lane owns 4
// adjacent channels (one 16-byte load per matrix and row), a wavefront covers
// 1 KiB of contiguous row, several rows are in flight per lane, and nothing is
// written but O(channels) partial sums.  Sums are taken of pivot-shifted values
// in fp64, so channels whose mean dwarfs their spread lose no precision, and in a
// fixed order (no floating-point atomics), so results are bit-reproducible.
#include "cwac_internal.h"

namespace cwac {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kStats = 5;  // sum dq, sum df, sum dq*dq, sum dq*df, sum df*df
constexpr int kHeaderBytes = 64;

struct StatsView {
  int64_t *n;
  float *pivot_q;
  float *pivot_f;
  double *sum;  // [kStats][c]
};

__host__ __device__ inline StatsView view(void *stats, int c) {
  char *b = static_cast<char *>(stats);
  StatsView v;
  v.n = reinterpret_cast<int64_t *>(b);
  v.pivot_q = reinterpret_cast<float *>(b + kHeaderBytes);
  v.pivot_f = v.pivot_q + c;
  v.sum = reinterpret_cast<double *>(b + kHeaderBytes + (size_t)8 * c);
  return v;
}

// Row split of one call: the same function sizes the workspace and the launch.
struct Split {
  int col_blocks;      // workgroups along channels
  int row_blocks;      // workgroups along rows = number of partial sums per channel
  int64_t rows_per_block;
};

inline Split make_split(int64_t n_rows, int c_out, int vec) {
  Split s;
  s.col_blocks = (int)ceil_div(c_out, kWave * vec);
  const int64_t target_blocks = 2048;  // ~8 workgroups per compute unit
  int64_t rb = ceil_div(target_blocks, s.col_blocks);
  const int64_t max_rb = ceil_div(n_rows, 32);  // at least 32 rows per workgroup
  if (rb > max_rb) rb = max_rb;
  if (rb < 1) rb = 1;
  if (rb > 65535) rb = 65535;
  s.rows_per_block = ceil_div(ceil_div(n_rows, rb), kWaves) * kWaves;
  s.row_blocks = (int)ceil_div(n_rows, s.rows_per_block);
  return s;
}

template <int VEC>
struct Ld;
template <>
struct Ld<4> {
  using T = float4;
  __device__ static void unpack(const float4 &v, float (&o)[4]) {
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
  }
};
template <>
struct Ld<1> {
  using T = float;
  __device__ static void unpack(const float &v, float (&o)[1]) { o[0] = v; }
};

// Stage 1.  grid = (col_blocks, row_blocks).  Lane l of every wavefront owns
// channels c0 + VEC*l .. +VEC-1; wavefront w takes rows r0 + w, r0 + w + 4, ...
// partial[row_block][stat][channel] receives the workgroup's sums.
template <int VEC>
__global__ __launch_bounds__(kThreads) void stats_partial_kernel(
    const float *__restrict__ yf, int64_t ldf, const float *__restrict__ yq, int64_t ldq,
    int64_t n_rows, int c_out, int64_t rows_per_block, const void *stats,
    double *__restrict__ partial) {
  using V = typename Ld<VEC>::T;
  const int lane = threadIdx.x & (kWave - 1);
  const int w = threadIdx.x / kWave;
  const int c = (blockIdx.x * kWave + lane) * VEC;
  const bool active = c < c_out;  // VEC == 4 requires c_out % 4 == 0, so all-or-nothing
  const int cc = active ? c : 0;

  const StatsView sv = view(const_cast<void *>(stats), c_out);
  const bool first = (*sv.n == 0);
  float pq[VEC], pf[VEC];
  {
    V vq = first ? *reinterpret_cast<const V *>(yq + cc) : *reinterpret_cast<const V *>(sv.pivot_q + cc);
    V vf = first ? *reinterpret_cast<const V *>(yf + cc) : *reinterpret_cast<const V *>(sv.pivot_f + cc);
    Ld<VEC>::unpack(vq, pq);
    Ld<VEC>::unpack(vf, pf);
  }

  double acc[VEC][kStats];
#pragma unroll
  for (int j = 0; j < VEC; ++j)
#pragma unroll
    for (int s = 0; s < kStats; ++s) acc[j][s] = 0.0;

  const int64_t r_begin = (int64_t)blockIdx.y * rows_per_block;
  int64_t r_end = r_begin + rows_per_block;
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
      acc[j][2] += dq * dq;
      acc[j][3] += dq * df;
      acc[j][4] += df * df;
    }
  };

  if (active) {
    constexpr int U = 4;  // rows in flight per lane: 2*U 16-byte loads outstanding
    int64_t r = r_begin + w;
    for (; r + (U - 1) * kWaves < r_end; r += U * kWaves) {
      V vq[U], vf[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        vq[u] = *reinterpret_cast<const V *>(yq + (r + u * kWaves) * ldq + c);
        vf[u] = *reinterpret_cast<const V *>(yf + (r + u * kWaves) * ldf + c);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) consume(vq[u], vf[u]);
    }
    for (; r < r_end; r += kWaves) {
      const V vq = *reinterpret_cast<const V *>(yq + r * ldq + c);
      const V vf = *reinterpret_cast<const V *>(yf + r * ldf + c);
      consume(vq, vf);
    }
  }

  // Fixed-order merge of the four wavefronts through LDS.
  __shared__ double red[kWaves][kStats][kWave * VEC];
#pragma unroll
  for (int j = 0; j < VEC; ++j)
#pragma unroll
    for (int s = 0; s < kStats; ++s) red[w][s][lane * VEC + j] = acc[j][s];
  __syncthreads();
  const int chans = kWave * VEC;
  for (int i = threadIdx.x; i < kStats * chans; i += kThreads) {
    const int s = i / chans, j = i - s * chans;
    const int ch = blockIdx.x * chans + j;
    if (ch < c_out) {
      double t = red[0][s][j];
#pragma unroll
      for (int ww = 1; ww < kWaves; ++ww) t += red[ww][s][j];
      partial[((int64_t)blockIdx.y * kStats + s) * c_out + ch] = t;
    }
  }
}

// Stage 2: fixed-order sum over row blocks, added into the state; the first
// batch also records the pivots (row 0 of that batch).
__global__ __launch_bounds__(kThreads) void stats_merge_kernel(
    const double *__restrict__ partial, int row_blocks, int c_out, const float *__restrict__ yf,
    const float *__restrict__ yq, void *stats) {
  const int i = blockIdx.x * kThreads + threadIdx.x;
  if (i >= kStats * c_out) return;
  const int s = i / c_out, ch = i - s * c_out;
  const StatsView sv = view(stats, c_out);
  const bool first = (*sv.n == 0);
  double t = 0.0;
  for (int rb = 0; rb < row_blocks; ++rb) t += partial[((int64_t)rb * kStats + s) * c_out + ch];
  sv.sum[i] = first ? t : sv.sum[i] + t;
  if (first && s == 0) {
    sv.pivot_q[ch] = yq[ch];
    sv.pivot_f[ch] = yf[ch];
  }
}

// Stage 3: bump the row count (its own launch: every workgroup of stage 2 reads it).
__global__ void stats_commit_kernel(void *stats, int64_t n_rows) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *static_cast<int64_t *>(stats) += n_rows;
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

// Eq. 4-5 from the shifted sums, fp64.
__global__ __launch_bounds__(1024) void solve_kernel(const void *stats, int c_out, double var_eps,
                                                     float *__restrict__ alpha,
                                                     float *__restrict__ beta,
                                                     double *__restrict__ moments,
                                                     int32_t *__restrict__ n_degenerate) {
  const StatsView sv = view(const_cast<void *>(stats), c_out);
  const int64_t n = *sv.n;
  int deg = 0;
  for (int ch = threadIdx.x; ch < c_out; ch += blockDim.x) {
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
    __shared__ int s_deg[1024 / kWave];
    deg = wave_sum(deg);
    if ((threadIdx.x & (kWave - 1)) == 0) s_deg[threadIdx.x / kWave] = deg;
    __syncthreads();
    if (threadIdx.x == 0) {
      int t = 0;
      for (int i = 0; i < (int)(blockDim.x / kWave); ++i) t += s_deg[i];
      *n_degenerate = t;
    }
  }
}

}  // namespace
}  // namespace cwac

using namespace cwac;

extern "C" size_t cwac_stats_bytes(int32_t c_out) {
  if (c_out < 1) return 0;
  return (size_t)kHeaderBytes + (size_t)8 * c_out + (size_t)kStats * 8 * c_out;
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
  const int rb = a.row_blocks > b.row_blocks ? a.row_blocks : b.row_blocks;
  return (size_t)rb * kStats * c_out * sizeof(double);
}

extern "C" cwac_status cwac_calibrate_stats(const float *y_full, int64_t ld_full,
                                            const float *y_quant, int64_t ld_quant,
                                            int64_t n_rows, int32_t c_out, void *stats,
                                            void *workspace, size_t workspace_bytes,
                                            void *stream) {
  if (!stats) return CWAC_E_NULL;
  if (c_out < 1 || c_out > 65536 || n_rows < 0) return CWAC_E_SHAPE;
  if (n_rows == 0) return CWAC_OK;
  if (!y_full || !y_quant) return CWAC_E_NULL;
  if (ld_full < c_out || ld_quant < c_out) return CWAC_E_SHAPE;
  if (!aligned(stats, 16) || !aligned(y_full, 4) || !aligned(y_quant, 4)) return CWAC_E_ALIGN;
  if (!workspace || workspace_bytes < cwac_calibrate_stats_workspace(n_rows, c_out))
    return CWAC_E_WORKSPACE;
  if (!aligned(workspace, 16)) return CWAC_E_ALIGN;
  const bool vec = (c_out % 4 == 0) && (ld_full % 4 == 0) && (ld_quant % 4 == 0) &&
                   aligned(y_full, 16) && aligned(y_quant, 16);
  const Split sp = make_split(n_rows, c_out, vec ? 4 : 1);
  double *partial = static_cast<double *>(workspace);
  const dim3 grid(sp.col_blocks, sp.row_blocks);
  hipStream_t st = as_stream(stream);
  if (vec)
    stats_partial_kernel<4><<<grid, kThreads, 0, st>>>(y_full, ld_full, y_quant, ld_quant, n_rows,
                                                       c_out, sp.rows_per_block, stats, partial);
  else
    stats_partial_kernel<1><<<grid, kThreads, 0, st>>>(y_full, ld_full, y_quant, ld_quant, n_rows,
                                                       c_out, sp.rows_per_block, stats, partial);
  stats_merge_kernel<<<(unsigned)ceil_div((int64_t)kStats * c_out, kThreads), kThreads, 0, st>>>(
      partial, sp.row_blocks, c_out, y_full, y_quant, stats);
  stats_commit_kernel<<<1, 64, 0, st>>>(stats, n_rows);
  return launch_status();
}

extern "C" cwac_status cwac_solve(const void *stats, int32_t c_out, double var_eps, float *alpha,
                                  float *beta, double *moments, int32_t *n_degenerate,
                                  void *stream) {
  if (!stats || !alpha || !beta) return CWAC_E_NULL;
  if (c_out < 1 || c_out > 65536 || !(var_eps >= 0.0)) return CWAC_E_SHAPE;
  if (!aligned(stats, 16) || !aligned(alpha, 4) || !aligned(beta, 4) ||
      (moments && !aligned(moments, 8)))
    return CWAC_E_ALIGN;
  solve_kernel<<<1, 1024, 0, as_stream(stream)>>>(stats, c_out, var_eps, alpha, beta, moments,
                                                  n_degenerate);
  return launch_status();
}
