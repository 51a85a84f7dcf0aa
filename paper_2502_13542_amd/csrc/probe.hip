// Activation Bias and probe-Query (Sec. 4.1, Eq. (7)-(9)).
//
// Three phases, each bounded by one pass over the window's queries Q^t [m][d]:
//   stats   per-channel sums of the window, merged into the running
//           (n, mean, M2) of Eq. (8) by the last workgroup to finish;
//   bias    a_j = sum_c (q_jc - mean_c)^2 / var_c = |phi_j|_1 of Eq. (7), one row per token;
//   reduce  probe = sum_j (a_j / sum a) q_j of Eq. (9), column slabs in parallel, then
//           the last workgroup adds the norm and the per-KV-head sum of the probe.
// All sums are fp32 and are taken in a fixed order, so results are reproducible.
#include "common.h"
#include "launch.h"

namespace actqkv {

constexpr int kStatsThreads = 1024;  // 64 column lanes x 16 row lanes
constexpr int kStatsRowLanes = 16;

template <typename T>
__global__ __launch_bounds__(kStatsThreads) void probe_stats_kernel(
    const T* __restrict__ q_win, float* __restrict__ stats, float* __restrict__ scratch,
    unsigned int* __restrict__ counters, int m, int d, float eps, size_t stats_stride,
    size_t scratch_stride) {
  constexpr int V = Vec<T>::N;
  __shared__ float red[kStatsRowLanes][64 * V];
  __shared__ int flag;
  const int s = blockIdx.z;
  const T* q = q_win + size_t(s) * m * d;
  float* st = stats + size_t(s) * stats_stride;
  float* sc = scratch + size_t(s) * scratch_stride;
  float* sc_mean = sc;
  float* sc_inv = sc + d;
  float* part = sc + 2 * size_t(d) + probe_a_floats(m);  // [splits][2][d]
  const int splits = gridDim.y;
  const int cl = threadIdx.x & 63, rl = threadIdx.x >> 6;
  const int ch0 = (blockIdx.x * 64 + cl) * V;
  const float n_old = st[0];
  const float* mean_old = st + 4;

  // shift: the old mean, or the window's first query when there is no history
  float c[V], s1[V], s2[V];
  const bool active = ch0 < d;
  if (active) {
    if (n_old > 0.f) {
#pragma unroll
      for (int v = 0; v < V; ++v) c[v] = mean_old[ch0 + v];
    } else {
      Vec<T>::load(q + ch0, c);
    }
  }
#pragma unroll
  for (int v = 0; v < V; ++v) s1[v] = s2[v] = 0.f;
  const int rows_per = (m + splits - 1) / splits;
  const int r0 = blockIdx.y * rows_per, r1 = min(m, r0 + rows_per);
  if (active) {
    for (int r = r0 + rl; r < r1; r += kStatsRowLanes) {
      float x[V];
      Vec<T>::load(q + size_t(r) * d + ch0, x);
#pragma unroll
      for (int v = 0; v < V; ++v) {
        float t = x[v] - c[v];
        s1[v] += t;
        s2[v] += t * t;
      }
    }
  }
  // reduce over the 16 row lanes, first the sums, then the sums of squares
  for (int pass = 0; pass < 2; ++pass) {
    __syncthreads();
#pragma unroll
    for (int v = 0; v < V; ++v) red[rl][cl * V + v] = pass == 0 ? s1[v] : s2[v];
    __syncthreads();
    for (int col = threadIdx.x; col < 64 * V; col += kStatsThreads) {
      int ch = blockIdx.x * 64 * V + col;
      if (ch < d) {
        float t = 0.f;
#pragma unroll
        for (int i = 0; i < kStatsRowLanes; ++i) t += red[i][col];
        part[(size_t(blockIdx.y) * 2 + pass) * d + ch] = t;
      }
    }
  }

  if (!last_block_done(counters + s, gridDim.x * gridDim.y, &flag)) return;

  // merge the window into the running statistics (pairwise update of Eq. (8))
  const float nb = float(m), n_new = n_old + nb;
  for (int ch = threadIdx.x; ch < d; ch += kStatsThreads) {
    float t1 = 0.f, t2 = 0.f;
    for (int i = 0; i < splits; ++i) {
      t1 += part[(size_t(i) * 2 + 0) * d + ch];
      t2 += part[(size_t(i) * 2 + 1) * d + ch];
    }
    float mean_a = mean_old[ch];
    float shift = n_old > 0.f ? mean_a : to_f32(q[ch]);
    float mean_b = shift + t1 / nb;
    float m2_b = fmaxf(t2 - t1 * t1 / nb, 0.f);
    float delta = mean_b - mean_a;
    float mean = n_old > 0.f ? mean_a + delta * (nb / n_new) : mean_b;
    float m2 = n_old > 0.f ? st[4 + d + ch] + m2_b + delta * delta * (n_old * nb / n_new) : m2_b;
    st[4 + ch] = mean;
    st[4 + d + ch] = m2;
    float var = n_new > 1.f ? m2 / (n_new - 1.f) : 0.f;
    sc_mean[ch] = mean;
    sc_inv[ch] = 1.f / fmaxf(var, eps);
  }
  __syncthreads();
  if (threadIdx.x == 0) st[0] = n_new;
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
                                                         float* __restrict__ scratch, int m, int d,
                                                         size_t scratch_stride) {
  constexpr int V = Vec<T>::N;
  __shared__ float red[4][kBiasRows];
  const int s = blockIdx.y;
  const T* q = q_win + size_t(s) * m * d;
  float* sc = scratch + size_t(s) * scratch_stride;
  const float* mean = sc;
  const float* inv = sc + d;
  float* a = sc + 2 * size_t(d);
  const int r0 = blockIdx.x * kBiasRows;
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
#pragma unroll
    for (int i = 0; i < kBiasRows; ++i) {
      if (r0 + i < m) {
        float x[V];
        Vec<T>::load(q + size_t(r0 + i) * d + ch, x);
#pragma unroll
        for (int v = 0; v < V; ++v) {
          float t = x[v] - mu[v];
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

template <typename T>
__global__ __launch_bounds__(256) void probe_reduce_kernel(
    const T* __restrict__ q_win, const float* __restrict__ scratch, unsigned int* __restrict__ counters,
    float* __restrict__ probe_out, float* __restrict__ probe_kv_out, float* __restrict__ probe_norm_out,
    float* __restrict__ weights_out, int m, int n_q_heads, int n_kv_heads, int head_dim,
    size_t scratch_stride) {
  constexpr int V = Vec<T>::N;
  __shared__ float red[32];
  __shared__ float buf[16][16 * V];
  __shared__ int flag;
  const int d = n_q_heads * head_dim;
  const int s = blockIdx.y;
  const T* q = q_win + size_t(s) * m * d;
  const float* a = scratch + size_t(s) * scratch_stride + 2 * size_t(d);
  float* probe = probe_out + size_t(s) * d;

  float part = 0.f;
  for (int j = threadIdx.x; j < m; j += 256) part += a[j];
  const float total = block_sum(part, red);          // |Phi|_1
  const float inv_total = total > 0.f ? 1.f / total : 0.f;
  const float uniform = 1.f / float(m);

  const int cl = threadIdx.x & 15, rl = threadIdx.x >> 4;
  const int ch0 = (blockIdx.x * 16 + cl) * V;
  float acc[V];
#pragma unroll
  for (int v = 0; v < V; ++v) acc[v] = 0.f;
  if (ch0 < d) {
    for (int j = rl; j < m; j += 16) {
      float w = total > 0.f ? a[j] * inv_total : uniform;
      float x[V];
      Vec<T>::load(q + size_t(j) * d + ch0, x);
#pragma unroll
      for (int v = 0; v < V; ++v) acc[v] += w * x[v];
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
      probe[ch] = t;
    }
  }
  if (blockIdx.x == 0 && weights_out != nullptr) {
    for (int j = threadIdx.x; j < m; j += 256)
      weights_out[size_t(s) * m + j] = total > 0.f ? a[j] * inv_total : uniform;
  }
  if (!last_block_done(counters + s, gridDim.x, &flag)) return;
  probe_finish(probe, probe_kv_out + size_t(s) * n_kv_heads * head_dim, probe_norm_out + s,
               n_q_heads, n_kv_heads, head_dim, red);
}

// A window of one token (decode): Eq. (9) has a single weight, 1, so the probe is the query.
template <typename T>
__global__ __launch_bounds__(256) void probe_identity_kernel(
    const T* __restrict__ q_win, float* __restrict__ probe_out, float* __restrict__ probe_kv_out,
    float* __restrict__ probe_norm_out, float* __restrict__ weights_out, int n_q_heads,
    int n_kv_heads, int head_dim) {
  __shared__ float red[32];
  const int d = n_q_heads * head_dim;
  const int s = blockIdx.x;
  float* probe = probe_out + size_t(s) * d;
  for (int ch = threadIdx.x; ch < d; ch += 256) probe[ch] = to_f32(q_win[size_t(s) * d + ch]);
  __syncthreads();
  probe_finish(probe, probe_kv_out + size_t(s) * n_kv_heads * head_dim, probe_norm_out + s,
               n_q_heads, n_kv_heads, head_dim, red);
  if (threadIdx.x == 0 && weights_out != nullptr) weights_out[s] = 1.f;
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
  const int splits = probe_stat_splits(m);
  if (update_stats) {
    dim3 grid((d + 64 * V - 1) / (64 * V), splits, batch);
    hipLaunchKernelGGL(probe_stats_kernel<T>, grid, dim3(kStatsThreads), 0, stream, q_win, stats,
                       scratch, ws.counters(), m, d, eps, stats_stride, scratch_stride);
  } else if (m > 1) {
    dim3 grid((d + 255) / 256, batch);
    hipLaunchKernelGGL(probe_prepare_kernel, grid, dim3(256), 0, stream, stats, scratch, d, eps,
                       stats_stride, scratch_stride);
  }
  if (m == 1) {
    hipLaunchKernelGGL(probe_identity_kernel<T>, dim3(batch), dim3(256), 0, stream, q_win, probe,
                       probe_kv, probe_norm, weights, sh.n_q_heads, sh.n_kv_heads, sh.head_dim);
    return hip_status("probe");
  }
  {
    dim3 grid((m + kBiasRows - 1) / kBiasRows, batch);
    hipLaunchKernelGGL(probe_bias_kernel<T>, grid, dim3(256), 0, stream, q_win, scratch, m, d,
                       scratch_stride);
  }
  {
    dim3 grid((d + 16 * V - 1) / (16 * V), batch);
    hipLaunchKernelGGL(probe_reduce_kernel<T>, grid, dim3(256), 0, stream, q_win, scratch,
                       ws.counters(), probe, probe_kv, probe_norm, weights, m, sh.n_q_heads,
                       sh.n_kv_heads, sh.head_dim, scratch_stride);
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
