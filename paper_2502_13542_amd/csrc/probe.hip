// Activation Bias and probe-Query (Sec. 4.1, Eq. (7)-(9)).
//
// Each phase needs a result over the whole window from the phase before, so the
// call is a chain of four short kernels over the window's queries Q^t [m][d]
// (a kernel boundary is the cheapest grid-wide dependency on this chip: device-scope
// fences inside a kernel write back and invalidate the whole L2):
//   stats     per-channel sums of the window, merged into the running (n, mean, M2) of Eq. (8);
//   bias      a_j = sum_c (q_jc - mean_c)^2 / var_c = |phi_j|_1 of Eq. (7), one row per token;
//   reduce    partial sums of a_j q_j over row slices, column slabs in parallel;
//   finish    probe = sum_j (a_j / sum a) q_j of Eq. (9), its norm and its per-KV-head sum.
// All sums are fp32 and are taken in a fixed order, so results are reproducible.
#include "common.h"
#include "launch.h"

namespace actqkv {

constexpr int kStatsBatch = 8;   // 16-byte loads a thread keeps in flight
constexpr int kStatsColLanes = 8, kStatsRowLanes = 32;

// Running statistics of Eq. (8).  grid (column slabs of 8*V channels, batch); 256 threads
// = 8 column lanes x 32 row lanes.  A workgroup owns its channels for ALL rows of the
// window, so it can merge them into the running (mean, M2) itself (pairwise update) and no
// second pass over partial sums is needed.  Sums are taken of (q - shift), shift = the old
// mean (or the window's first query when there is no history), which keeps the squares
// free of cancellation.  The count n is published by the next kernel of the chain (every
// workgroup here reads the old one).
template <typename T>
__global__ __launch_bounds__(256) void probe_stats_kernel(const T* __restrict__ q_win,
                                                          float* __restrict__ stats,
                                                          float* __restrict__ scratch, int m, int d,
                                                          float eps, size_t stats_stride,
                                                          size_t scratch_stride) {
  constexpr int V = Vec<T>::N;
  constexpr int SLAB = kStatsColLanes * V;
  __shared__ float red[2][kStatsRowLanes][SLAB];
  const int s = blockIdx.y;
  const T* q = q_win + size_t(s) * m * d;
  float* st = stats + size_t(s) * stats_stride;
  float* sc = scratch + size_t(s) * scratch_stride;
  const int cl = threadIdx.x % kStatsColLanes, rl = threadIdx.x / kStatsColLanes;
  const int ch0 = blockIdx.x * SLAB + cl * V;
  const float n_old = st[0];

  float c[V], s1[V], s2[V];
#pragma unroll
  for (int v = 0; v < V; ++v) c[v] = s1[v] = s2[v] = 0.f;
  if (ch0 < d) {
    if (n_old > 0.f) {
#pragma unroll
      for (int v = 0; v < V; ++v) c[v] = st[4 + ch0 + v];
    } else {
      Vec<T>::load(q + ch0, c);
    }
    for (int r0 = rl; r0 < m; r0 += kStatsRowLanes * kStatsBatch) {
      float x[kStatsBatch][V];
#pragma unroll
      for (int i = 0; i < kStatsBatch; ++i) {   // all loads first: they overlap
        const int r = r0 + kStatsRowLanes * i;
        Vec<T>::load(q + size_t(r < m ? r : 0) * d + ch0, x[i]);
      }
#pragma unroll
      for (int i = 0; i < kStatsBatch; ++i) {
        if (r0 + kStatsRowLanes * i < m) {
#pragma unroll
          for (int v = 0; v < V; ++v) {
            float t = x[i][v] - c[v];
            s1[v] += t;
            s2[v] += t * t;
          }
        }
      }
    }
  }
#pragma unroll
  for (int v = 0; v < V; ++v) {
    red[0][rl][cl * V + v] = s1[v];
    red[1][rl][cl * V + v] = s2[v];
  }
  __syncthreads();
  const int col = threadIdx.x, ch = blockIdx.x * SLAB + col;
  if (col < SLAB && ch < d) {
    float t1 = 0.f, t2 = 0.f;
#pragma unroll
    for (int k = 0; k < kStatsRowLanes; ++k) {
      t1 += red[0][k][col];
      t2 += red[1][k][col];
    }
    const float nb = float(m), n_new = n_old + nb;
    const float mean_a = st[4 + ch];
    const float shift = n_old > 0.f ? mean_a : to_f32(q[ch]);
    const float mean_b = shift + t1 / nb;
    const float m2_b = fmaxf(t2 - t1 * t1 / nb, 0.f);
    const float delta = mean_b - mean_a;
    const float mean = n_old > 0.f ? mean_a + delta * (nb / n_new) : mean_b;
    const float m2 = n_old > 0.f ? st[4 + d + ch] + m2_b + delta * delta * (n_old * nb / n_new) : m2_b;
    st[4 + ch] = mean;
    st[4 + d + ch] = m2;
    const float var = n_new > 1.f ? m2 / (n_new - 1.f) : 0.f;
    sc[ch] = mean;
    sc[d + ch] = 1.f / fmaxf(var, eps);
  }
}

// Statistics used as they are: only mean and 1/var are put where the next phase reads them.
__global__ void probe_prepare_kernel(const float* __restrict__ stats, float* __restrict__ scratch,
                                     int d, float eps, size_t stats_stride, size_t scratch_stride) {
  const int s = blockIdx.y;
  const float* st = stats + size_t(s) * stats_stride;
  float* sc = scratch + size_t(s) * scratch_stride;
  const float n = st[0];
  int ch = blockIdx.x * blockDim.x + threadIdx.x;
  if (ch < d) {
    float var = n > 1.f ? st[4 + d + ch] / (n - 1.f) : 0.f;
    sc[ch] = st[4 + ch];
    sc[d + ch] = 1.f / fmaxf(var, eps);
  }
}

constexpr int kBiasRows = 4;

template <typename T>
__global__ __launch_bounds__(256) void probe_bias_kernel(const T* __restrict__ q_win,
                                                         float* __restrict__ scratch,
                                                         float* __restrict__ stats, int add_count, int m,
                                                         int d, size_t scratch_stride,
                                                         size_t stats_stride) {
  constexpr int V = Vec<T>::N;
  __shared__ float red[4][kBiasRows];
  const int s = blockIdx.y;
  const T* q = q_win + size_t(s) * m * d;
  float* sc = scratch + size_t(s) * scratch_stride;
  const float* mean = sc;
  const float* inv = sc + d;
  float* a = sc + 2 * size_t(d);
  const int r0 = blockIdx.x * kBiasRows;
  if (add_count && blockIdx.x == 0 && threadIdx.x == 0) stats[size_t(s) * stats_stride] += float(m);
  float acc[kBiasRows];
#pragma unroll
  for (int i = 0; i < kBiasRows; ++i) acc[i] = 0.f;
  for (int ch = threadIdx.x * V; ch < d; ch += 256 * V) {
    float mu[V], iv[V];
#pragma unroll
    for (int v = 0; v < V; v += 4) {
      f32x4 a4 = *reinterpret_cast<const f32x4*>(mean + ch + v);
      f32x4 b4 = *reinterpret_cast<const f32x4*>(inv + ch + v);
      mu[v] = a4.x; mu[v + 1] = a4.y; mu[v + 2] = a4.z; mu[v + 3] = a4.w;
      iv[v] = b4.x; iv[v + 1] = b4.y; iv[v + 2] = b4.z; iv[v + 3] = b4.w;
    }
    float x[kBiasRows][V];
#pragma unroll
    for (int i = 0; i < kBiasRows; ++i)          // all loads first: they overlap
      Vec<T>::load(q + size_t(r0 + i < m ? r0 + i : r0) * d + ch, x[i]);
#pragma unroll
    for (int i = 0; i < kBiasRows; ++i) {
      if (r0 + i < m) {
#pragma unroll
        for (int v = 0; v < V; ++v) {
          float t = x[i][v] - mu[v];
          acc[i] += t * t * iv[v];
        }
      }
    }
  }
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < kBiasRows; ++i) {
    float t = wave_sum(acc[i]);
    if (lane == 0) red[w][i] = t;
  }
  __syncthreads();
  if (threadIdx.x < kBiasRows && r0 + threadIdx.x < m)
    a[r0 + threadIdx.x] = red[0][threadIdx.x] + red[1][threadIdx.x] + red[2][threadIdx.x] +
                          red[3][threadIdx.x];
}

// probe_kv and the norm of the probe; run by one workgroup that sees the whole probe.
__device__ __forceinline__ void probe_finish(const float* probe, float* probe_kv, float* probe_norm,
                                             int n_q_heads, int n_kv_heads, int head_dim,
                                             float* red) {
  const int g = n_q_heads / n_kv_heads, d = n_q_heads * head_dim;
  float ss = 0.f;
  for (int ch = threadIdx.x; ch < d; ch += blockDim.x) ss += probe[ch] * probe[ch];
  ss = block_sum(ss, red);
  if (threadIdx.x == 0) *probe_norm = sqrtf(ss);
  for (int e = threadIdx.x; e < n_kv_heads * head_dim; e += blockDim.x) {
    int hk = e / head_dim, dd = e - hk * head_dim;
    float t = 0.f;
    for (int i = 0; i < g; ++i) t += probe[(hk * g + i) * head_dim + dd];
    probe_kv[e] = t;
  }
}

constexpr int kReduceRowSplits = 4;

// grid (column slabs of 16*V channels, kReduceRowSplits, batch); 256 threads = 16 column
// lanes x 16 row lanes.  Partial weighted sums sum_j w_j q_j over a slice of the rows.
template <typename T>
__global__ __launch_bounds__(256) void probe_reduce_kernel(const T* __restrict__ q_win,
                                                           float* __restrict__ scratch,
                                                           float* __restrict__ weights_out, int m,
                                                           int d, size_t scratch_stride) {
  constexpr int V = Vec<T>::N;
  __shared__ float red[32];
  __shared__ float buf[16][16 * V];
  const int s = blockIdx.z;
  const T* q = q_win + size_t(s) * m * d;
  float* sc = scratch + size_t(s) * scratch_stride;
  const float* a = sc + 2 * size_t(d);
  float* part = sc + 2 * size_t(d) + probe_a_floats(m);   // [kReduceRowSplits][d]

  float tsum = 0.f;
  for (int j = threadIdx.x; j < m; j += 256) tsum += a[j];
  const float total = block_sum(tsum, red);          // |Phi|_1
  const float inv_total = total > 0.f ? 1.f / total : 0.f;
  const float uniform = 1.f / float(m);

  const int cl = threadIdx.x & 15, rl = threadIdx.x >> 4;
  const int ch0 = (blockIdx.x * 16 + cl) * V;
  const int rows_per = (m + kReduceRowSplits - 1) / kReduceRowSplits;
  const int r_begin = blockIdx.y * rows_per, r_end = min(m, r_begin + rows_per);
  float acc[V];
#pragma unroll
  for (int v = 0; v < V; ++v) acc[v] = 0.f;
  if (ch0 < d) {
    for (int j0 = r_begin + rl; j0 < r_end; j0 += 16 * 8) {
      float x[8][V], w[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {                    // 8 independent loads in flight
        const int j = j0 + 16 * i;
        const int jj = j < r_end ? j : r_begin;
        Vec<T>::load(q + size_t(jj) * d + ch0, x[i]);
        w[i] = j < r_end ? (total > 0.f ? a[jj] * inv_total : uniform) : 0.f;
      }
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < V; ++v) acc[v] += w[i] * x[i][v];
    }
  }
#pragma unroll
  for (int v = 0; v < V; ++v) buf[rl][cl * V + v] = acc[v];
  __syncthreads();
  if (threadIdx.x < 16 * V) {
    int ch = blockIdx.x * 16 * V + threadIdx.x;
    if (ch < d) {
      float t = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) t += buf[i][threadIdx.x];
      part[size_t(blockIdx.y) * d + ch] = t;
    }
  }
  if (blockIdx.x == 0 && blockIdx.y == 0 && weights_out != nullptr) {
    for (int j = threadIdx.x; j < m; j += 256)
      weights_out[size_t(s) * m + j] = total > 0.f ? a[j] * inv_total : uniform;
  }
}

// One workgroup per sequence: adds the row slices up in a fixed order and finishes the probe.
__global__ __launch_bounds__(1024) void probe_finish_kernel(const float* __restrict__ scratch,
                                                            float* __restrict__ probe_out,
                                                            float* __restrict__ probe_kv_out,
                                                            float* __restrict__ probe_norm_out, int m,
                                                            int n_q_heads, int n_kv_heads, int head_dim,
                                                            size_t scratch_stride) {
  __shared__ float red[32];
  const int d = n_q_heads * head_dim;
  const int s = blockIdx.x;
  const float* part = scratch + size_t(s) * scratch_stride + 2 * size_t(d) + probe_a_floats(m);
  float* probe = probe_out + size_t(s) * d;
  for (int ch = threadIdx.x * 4; ch < d; ch += 1024 * 4) {
    f32x4 t = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < kReduceRowSplits; ++i) t += *reinterpret_cast<const f32x4*>(part + size_t(i) * d + ch);
    *reinterpret_cast<f32x4*>(probe + ch) = t;
  }
  __syncthreads();
  probe_finish(probe, probe_kv_out + size_t(s) * n_kv_heads * head_dim, probe_norm_out + s,
               n_q_heads, n_kv_heads, head_dim, red);
}

// A window of one token (decode): Eq. (9) has a single weight, 1, so the probe is the query.
// One workgroup of 1024 threads per sequence; a thread owns up to 4 groups of 4 channels.
template <typename T>
__global__ __launch_bounds__(1024) void probe_identity_kernel(
    const T* __restrict__ q_win, float* __restrict__ stats, int add_count, size_t stats_stride,
    float* __restrict__ probe_out, float* __restrict__ probe_kv_out, float* __restrict__ probe_norm_out,
    float* __restrict__ weights_out, int n_q_heads, int n_kv_heads, int head_dim) {
  __shared__ float red[32];
  extern __shared__ __attribute__((aligned(16))) float probe_lds[];   // [d]
  const int d = n_q_heads * head_dim, g = n_q_heads / n_kv_heads;
  const int s = blockIdx.x;
  const T* q = q_win + size_t(s) * d;
  float* probe = probe_out + size_t(s) * d;
  if (add_count && threadIdx.x == 0) stats[size_t(s) * stats_stride] += 1.f;
  float x[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {                  // all loads first: they overlap
    const int ch = (threadIdx.x + 1024 * i) * 4;
#pragma unroll
    for (int v = 0; v < 4; ++v) x[i][v] = ch < d ? to_f32(q[ch + v]) : 0.f;
  }
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int ch = (threadIdx.x + 1024 * i) * 4;
    if (ch < d) {
      f32x4 v = {x[i][0], x[i][1], x[i][2], x[i][3]};
      *reinterpret_cast<f32x4*>(probe + ch) = v;
      *reinterpret_cast<f32x4*>(probe_lds + ch) = v;
      ss += x[i][0] * x[i][0] + x[i][1] * x[i][1] + x[i][2] * x[i][2] + x[i][3] * x[i][3];
    }
  }
  ss = block_sum(ss, red);                       // also orders the LDS writes before the reads below
  if (threadIdx.x == 0) {
    probe_norm_out[s] = sqrtf(ss);
    if (weights_out != nullptr) weights_out[s] = 1.f;
  }
  float* probe_kv = probe_kv_out + size_t(s) * n_kv_heads * head_dim;
  for (int e = threadIdx.x; e < n_kv_heads * head_dim; e += 1024) {
    const int hk = e / head_dim, dd = e - hk * head_dim;
    float t = 0.f;
    for (int i = 0; i < g; ++i) t += probe_lds[(hk * g + i) * head_dim + dd];
    probe_kv[e] = t;
  }
}

template <typename T>
static int launch_probe_t(const actqkv_shape& sh, int batch, int m, const T* q_win, float* stats,
                          int update_stats, float* probe, float* probe_kv, float* probe_norm,
                          float* weights, const Workspace& ws, hipStream_t stream) {
  constexpr int V = Vec<T>::N;
  const int d = sh.n_q_heads * sh.head_dim;
  const float eps = sh.var_eps > 0.f ? sh.var_eps : 1e-12f;
  const size_t stats_stride = stats_floats(sh);
  const size_t scratch_stride = probe_scratch_floats(sh, m);
  float* scratch = ws.scratch_f32();
  if (update_stats) {
    dim3 grid((d + kStatsColLanes * V - 1) / (kStatsColLanes * V), batch);
    hipLaunchKernelGGL(probe_stats_kernel<T>, grid, dim3(256), 0, stream, q_win, stats, scratch, m, d,
                       eps, stats_stride, scratch_stride);
  } else if (m > 1) {
    dim3 grid((d + 255) / 256, batch);
    hipLaunchKernelGGL(probe_prepare_kernel, grid, dim3(256), 0, stream, stats, scratch, d, eps,
                       stats_stride, scratch_stride);
  }
  if (m == 1) {
    hipLaunchKernelGGL(probe_identity_kernel<T>, dim3(batch), dim3(1024), size_t(d) * sizeof(float),
                       stream, q_win, stats,
                       update_stats, stats_stride, probe, probe_kv, probe_norm, weights, sh.n_q_heads,
                       sh.n_kv_heads, sh.head_dim);
    return hip_status("probe");
  }
  {
    dim3 grid((m + kBiasRows - 1) / kBiasRows, batch);
    hipLaunchKernelGGL(probe_bias_kernel<T>, grid, dim3(256), 0, stream, q_win, scratch, stats,
                       update_stats, m, d, scratch_stride, stats_stride);
  }
  {
    dim3 grid((d + 16 * V - 1) / (16 * V), kReduceRowSplits, batch);
    hipLaunchKernelGGL(probe_reduce_kernel<T>, grid, dim3(256), 0, stream, q_win, scratch, weights, m,
                       d, scratch_stride);
    hipLaunchKernelGGL(probe_finish_kernel, dim3(batch), dim3(1024), 0, stream, scratch, probe,
                       probe_kv, probe_norm, m, sh.n_q_heads, sh.n_kv_heads, sh.head_dim,
                       scratch_stride);
  }
  return hip_status("probe");
}

int launch_probe(const actqkv_shape& sh, int batch, int m, const void* q_win, float* stats,
                 int update_stats, float* probe, float* probe_kv, float* probe_norm, float* weights,
                 const Workspace& ws, hipStream_t stream) {
  if (sh.dtype == ACTQKV_F32)
    return launch_probe_t<float>(sh, batch, m, static_cast<const float*>(q_win), stats, update_stats,
                                 probe, probe_kv, probe_norm, weights, ws, stream);
  return launch_probe_t<uint16_t>(sh, batch, m, static_cast<const uint16_t*>(q_win), stats,
                                  update_stats, probe, probe_kv, probe_norm, weights, ws, stream);
}

}  // namespace actqkv
