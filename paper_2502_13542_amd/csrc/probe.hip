// Activation Bias and probe-Query (Sec. 4.1, Eq. (7)-(9)).
//
// The statistics of Eq. (8) reduce over the rows of the window and the weights of Eq. (9)
// over the channels, so the call is a chain of three short kernels over the window's
// queries Q^t [m][d] (a kernel boundary is the cheapest grid-wide dependency on this chip:
// device-scope fences inside a kernel write back and invalidate the whole L2):
//   stats_bias  a workgroup owns a slab of channels for ALL rows: merges the window into the
//               running (n, mean, M2) of Eq. (8), then sums phi of Eq. (7) over its channels,
//               one partial |phi_j|_1 per row and slab;
//   weigh       adds the slabs' partials to a_j = |phi_j|_1, w_j = a_j / sum a, and forms its
//               slab of probe = sum_j w_j q_j of Eq. (9);
//   finish      norm of the probe and its per-KV-head sum.
// All sums are fp32 and are taken in a fixed order, so results are reproducible.
//
// Consecutive windows of one sequence can be taken in one call: Eq. (8) merges the windows
// into the running statistics one after the other, but the merge is a function of each
// window's own (mean, M2) only.  So window_moments computes those for all windows at once,
// chain_bias (one workgroup per window and slab) replays the merges up to its window -
// a few operations per channel - and takes the bias partials of its window, and weigh and
// finish run once for all windows.  Four launches for n windows instead of 3 n.
#include "common.h"
#include "launch.h"
#include "probe_identity.h"

namespace actqkv {

constexpr int kColLanes = 8;      // 16-byte column lanes of a slab
constexpr int kRowsPerThread = 16;   // 16-byte loads a thread keeps in flight
constexpr int kStatsRowLanes = 32;
constexpr int kStatsRowsPerPass = kStatsRowLanes * kRowsPerThread;

// apart[j] = sum over the slab's channels of (q_jc - mean_c)^2 / var_c for the rows of the
// window (Eq. (7) summed over a slab); x holds pass 0 of the rows when there is one pass only.
template <typename T, typename LoadPass>
__device__ __forceinline__ void bias_partials(typename Vec<T>::raw (&x)[kRowsPerThread], LoadPass&& load_pass,
                                              const float* mu_lds, const float* iv_lds,
                                              float* __restrict__ apart, int m, int m_pad, int n_pass,
                                              int cl, int rl) {
  constexpr int V = Vec<T>::N;
  float mu[V], iv[V];
#pragma unroll
  for (int v = 0; v < V; ++v) {
    mu[v] = mu_lds[cl * V + v];
    iv[v] = iv_lds[cl * V + v];
  }
  for (int pass = 0; pass < n_pass; ++pass) {
    if (n_pass > 1) load_pass(pass);
    const int r0 = pass * kStatsRowsPerPass + rl * kRowsPerThread;
    float a[kRowsPerThread];
#pragma unroll
    for (int i = 0; i < kRowsPerThread; ++i) {
      float f[V];
      Vec<T>::widen(x[i], f);
      float t = 0.f;
#pragma unroll
      for (int v = 0; v < V; ++v) {
        float e = f[v] - mu[v];
        t += e * e * iv[v];
      }
      // the 8 column lanes of a row are neighbouring lanes of one wave
      t += __shfl_xor(t, 1, 64);
      t += __shfl_xor(t, 2, 64);
      t += __shfl_xor(t, 4, 64);
      a[i] = r0 + i < m ? t : 0.f;
    }
    if (cl == 0 && r0 < m_pad) {
#pragma unroll
      for (int i = 0; i < kRowsPerThread; i += 4) {
        f32x4 o = {a[i], a[i + 1], a[i + 2], a[i + 3]};
        *reinterpret_cast<f32x4*>(apart + r0 + i) = o;
      }
    }
  }
}

// grid (column slabs of 8*V channels, batch); 256 threads = 8 column lanes x 32 row lanes;
// row lane rl takes rows rl*16 .. rl*16+15 of every pass of 512 rows.
// Pass 1 (update != 0): sums of (q - shift), shift = the old mean (or the window's first
// query when there is no history), which keeps the squares free of cancellation; pairwise
// merge into the running mean and M2.  The count n is published by the next kernel of the
// chain (every workgroup here reads the old one).
// Pass 2 (m > 1): apart[slab][j] = sum over the slab's channels of (q_jc - mean_c)^2 / var_c.
// A window of at most 512 rows stays in registers between the passes.
template <typename T>
__global__ __launch_bounds__(256) void probe_stats_bias_kernel(const T* __restrict__ q_win,
                                                               float* __restrict__ stats,
                                                               float* __restrict__ scratch, int update,
                                                               int m, int m_pad, int d, float eps,
                                                               size_t stats_stride,
                                                               size_t scratch_stride) {
  constexpr int V = Vec<T>::N;
  constexpr int SLAB = kColLanes * V;
  typedef typename Vec<T>::raw raw_t;
  __shared__ float red[2][kStatsRowLanes][SLAB];
  __shared__ float mu_lds[SLAB], iv_lds[SLAB];
  const int s = blockIdx.y;
  const T* q = q_win + size_t(s) * m * d;
  float* st = stats + size_t(s) * stats_stride;
  float* apart = scratch + size_t(s) * scratch_stride + size_t(blockIdx.x) * m_pad;
  const int cl = threadIdx.x % kColLanes, rl = threadIdx.x / kColLanes;
  const int ch0 = blockIdx.x * SLAB + cl * V;
  const bool col_ok = ch0 < d;
  const float n_old = st[0];
  const int n_pass = (m + kStatsRowsPerPass - 1) / kStatsRowsPerPass;

  raw_t x[kRowsPerThread];
  auto load_pass = [&](int pass) {
#pragma unroll
    for (int i = 0; i < kRowsPerThread; ++i) {   // all loads first: they overlap
      const int r = pass * kStatsRowsPerPass + rl * kRowsPerThread + i;
      x[i] = Vec<T>::load_raw(q + size_t(r < m ? r : 0) * d + (col_ok ? ch0 : 0));
    }
  };
  load_pass(0);

  if (update) {
    float c[V], s1[V], s2[V];
#pragma unroll
    for (int v = 0; v < V; ++v) c[v] = s1[v] = s2[v] = 0.f;
    if (col_ok) {
      if (n_old > 0.f) {
#pragma unroll
        for (int v = 0; v < V; ++v) c[v] = st[4 + ch0 + v];
      } else {
        Vec<T>::load(q + ch0, c);
      }
    }
    for (int pass = 0; pass < n_pass; ++pass) {
      if (pass > 0) load_pass(pass);
#pragma unroll
      for (int i = 0; i < kRowsPerThread; ++i) {
        if (pass * kStatsRowsPerPass + rl * kRowsPerThread + i < m) {
          float f[V];
          Vec<T>::widen(x[i], f);
#pragma unroll
          for (int v = 0; v < V; ++v) {
            float t = f[v] - c[v];
            s1[v] += t;
            s2[v] += t * t;
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
  }
  {
    const int col = threadIdx.x, ch = blockIdx.x * SLAB + col;
    if (col < SLAB && ch >= d) mu_lds[col] = iv_lds[col] = 0.f;
    if (col < SLAB && ch < d) {
      float mean, m2, n_new;
      if (update) {
        float t1 = 0.f, t2 = 0.f;
#pragma unroll
        for (int k = 0; k < kStatsRowLanes; ++k) {
          t1 += red[0][k][col];
          t2 += red[1][k][col];
        }
        const float nb = float(m);
        n_new = n_old + nb;
        const float mean_a = st[4 + ch];
        const float shift = n_old > 0.f ? mean_a : to_f32(q[ch]);
        const float mean_b = shift + t1 / nb;
        const float m2_b = fmaxf(t2 - t1 * t1 / nb, 0.f);
        const float delta = mean_b - mean_a;
        mean = n_old > 0.f ? mean_a + delta * (nb / n_new) : mean_b;
        m2 = n_old > 0.f ? st[4 + d + ch] + m2_b + delta * delta * (n_old * nb / n_new) : m2_b;
        st[4 + ch] = mean;
        st[4 + d + ch] = m2;
      } else {
        n_new = n_old;
        mean = st[4 + ch];
        m2 = st[4 + d + ch];
      }
      const float var = n_new > 1.f ? m2 / (n_new - 1.f) : 0.f;
      mu_lds[col] = mean;
      iv_lds[col] = 1.f / fmaxf(var, eps);
    }
  }
  if (m == 1) return;   // a single token is its own probe: no weights needed
  __syncthreads();

  bias_partials<T>(x, load_pass, mu_lds, iv_lds, apart, m, m_pad, n_pass, cl, rl);
}

// ---- consecutive windows of one sequence in one call
// Scratch behind the bias partials: mom[n][2][d] = (mean, M2) of every window on its own,
// then base[4 + 2 d] = the running statistics as they were before the call.
//
// grid (column slabs, n windows); threads as in probe_stats_bias_kernel.  The sums are taken
// about the window's first query (no cancellation in the squares).  The workgroups of window
// 0 also copy their slab of the old statistics to `base`, which chain_bias reads: it
// overwrites the statistics themselves while other workgroups still need the old ones.
template <typename T>
__global__ __launch_bounds__(256) void probe_window_moments_kernel(const T* __restrict__ q_win,
                                                                   const float* __restrict__ stats,
                                                                   float* __restrict__ mom,
                                                                   float* __restrict__ base, int m, int d) {
  constexpr int V = Vec<T>::N;
  constexpr int SLAB = kColLanes * V;
  typedef typename Vec<T>::raw raw_t;
  __shared__ float red[2][kStatsRowLanes][SLAB];
  const int w = blockIdx.y;
  const T* q = q_win + size_t(w) * m * d;
  const int cl = threadIdx.x % kColLanes, rl = threadIdx.x / kColLanes;
  const int ch0 = blockIdx.x * SLAB + cl * V;
  const bool col_ok = ch0 < d;
  const int n_pass = (m + kStatsRowsPerPass - 1) / kStatsRowsPerPass;
  float c[V], s1[V], s2[V];
#pragma unroll
  for (int v = 0; v < V; ++v) c[v] = s1[v] = s2[v] = 0.f;
  if (col_ok) Vec<T>::load(q + ch0, c);
  for (int pass = 0; pass < n_pass; ++pass) {
    raw_t x[kRowsPerThread];
#pragma unroll
    for (int i = 0; i < kRowsPerThread; ++i) {   // all loads first: they overlap
      const int r = pass * kStatsRowsPerPass + rl * kRowsPerThread + i;
      x[i] = Vec<T>::load_raw(q + size_t(r < m ? r : 0) * d + (col_ok ? ch0 : 0));
    }
#pragma unroll
    for (int i = 0; i < kRowsPerThread; ++i) {
      if (pass * kStatsRowsPerPass + rl * kRowsPerThread + i < m) {
        float f[V];
        Vec<T>::widen(x[i], f);
#pragma unroll
        for (int v = 0; v < V; ++v) {
          float t = f[v] - c[v];
          s1[v] += t;
          s2[v] += t * t;
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
    const float nb = float(m);
    mom[(size_t(w) * 2 + 0) * d + ch] = to_f32(q[ch]) + t1 / nb;
    mom[(size_t(w) * 2 + 1) * d + ch] = fmaxf(t2 - t1 * t1 / nb, 0.f);
    if (w == 0) {
      base[4 + ch] = stats[4 + ch];
      base[4 + d + ch] = stats[4 + d + ch];
      if (ch == 0) base[0] = stats[0];
    }
  }
}

constexpr int kChainBatch = 16;   // window moments a thread requests together

// grid (column slabs, n windows), 256 threads.  Merges the windows 0 .. w into the old
// statistics in window order (the merge of Eq. (8), as in probe_stats_bias_kernel), which
// gives the statistics window w sees; the workgroups of the last window store them.  Then
// the bias partials of window w, whose rows were requested first and arrive meanwhile.
template <typename T>
__global__ __launch_bounds__(256) void probe_chain_bias_kernel(const T* __restrict__ q_win,
                                                               float* __restrict__ stats,
                                                               const float* __restrict__ mom,
                                                               const float* __restrict__ base,
                                                               float* __restrict__ scratch, int m,
                                                               int m_pad, int d, float eps,
                                                               size_t scratch_stride) {
  constexpr int V = Vec<T>::N;
  constexpr int SLAB = kColLanes * V;
  typedef typename Vec<T>::raw raw_t;
  __shared__ float mu_lds[SLAB], iv_lds[SLAB];
  const int w = blockIdx.y, n_win = gridDim.y;
  const T* q = q_win + size_t(w) * m * d;
  float* apart = scratch + size_t(w) * scratch_stride + size_t(blockIdx.x) * m_pad;
  const int cl = threadIdx.x % kColLanes, rl = threadIdx.x / kColLanes;
  const int ch0 = blockIdx.x * SLAB + cl * V;
  const bool col_ok = ch0 < d;
  const int n_pass = (m + kStatsRowsPerPass - 1) / kStatsRowsPerPass;
  raw_t x[kRowsPerThread];
  auto load_pass = [&](int pass) {
#pragma unroll
    for (int i = 0; i < kRowsPerThread; ++i) {
      const int r = pass * kStatsRowsPerPass + rl * kRowsPerThread + i;
      x[i] = Vec<T>::load_raw(q + size_t(r < m ? r : 0) * d + (col_ok ? ch0 : 0));
    }
  };
  load_pass(0);
  {
    const int col = threadIdx.x, ch = blockIdx.x * SLAB + col;
    if (col < SLAB && ch >= d) mu_lds[col] = iv_lds[col] = 0.f;
    if (col < SLAB && ch < d) {
      float n_run = base[0], mean = base[4 + ch], m2 = base[4 + d + ch];
      const float nb = float(m);
      for (int u0 = 0; u0 <= w; u0 += kChainBatch) {
        float mean_b[kChainBatch], m2_b[kChainBatch];
#pragma unroll
        for (int i = 0; i < kChainBatch; ++i) {   // all loads first: they overlap
          const int u = min(u0 + i, w);
          mean_b[i] = mom[(size_t(u) * 2 + 0) * d + ch];
          m2_b[i] = mom[(size_t(u) * 2 + 1) * d + ch];
        }
#pragma unroll
        for (int i = 0; i < kChainBatch; ++i) {
          if (u0 + i <= w) {
            const float n_new = n_run + nb;
            if (n_run > 0.f) {
              const float delta = mean_b[i] - mean;
              mean += delta * (nb / n_new);
              m2 += m2_b[i] + delta * delta * (n_run * nb / n_new);
            } else {
              mean = mean_b[i];
              m2 = m2_b[i];
            }
            n_run = n_new;
          }
        }
      }
      if (w == n_win - 1) {
        stats[4 + ch] = mean;
        stats[4 + d + ch] = m2;
        if (ch == 0) stats[0] = n_run;
      }
      const float var = n_run > 1.f ? m2 / (n_run - 1.f) : 0.f;
      mu_lds[col] = mean;
      iv_lds[col] = 1.f / fmaxf(var, eps);
    }
  }
  __syncthreads();
  bias_partials<T>(x, load_pass, mu_lds, iv_lds, apart, m, m_pad, n_pass, cl, rl);
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

constexpr int kWeighRowLanes = 64;
constexpr int kWeighRows = 8;    // rows a thread takes per pass
constexpr int kWeighRowsPerPass = kWeighRowLanes * kWeighRows;
constexpr int kWeighSlabBatch = 16;

// grid (column slabs of 8*V channels, batch); 512 threads = 8 column lanes x 64 row lanes.
// Every workgroup adds the slabs' partials up to a_j (slab order), turns them into the
// weights of Eq. (9) and sums w_j q_j over all rows for its channels.  The queries of the
// first pass are requested before the partials, so both are in flight together.
template <typename T>
__global__ __launch_bounds__(512) void probe_weigh_kernel(const T* __restrict__ q_win,
                                                          const float* __restrict__ scratch,
                                                          float* __restrict__ stats, int add_count,
                                                          int mean_pooling,
                                                          float* __restrict__ probe_out,
                                                          float* __restrict__ weights_out, int m,
                                                          int m_pad, int n_slabs, int d,
                                                          size_t scratch_stride, size_t stats_stride) {
  constexpr int V = Vec<T>::N;
  constexpr int SLAB = kColLanes * V;
  typedef typename Vec<T>::raw raw_t;
  __shared__ float red[32];
  __shared__ float w_lds[kMaxWindow];
  __shared__ float buf[8][SLAB];
  const int s = blockIdx.y;
  const T* q = q_win + size_t(s) * m * d;
  const float* apart = scratch + size_t(s) * scratch_stride;
  const int cl = threadIdx.x % kColLanes, rl = threadIdx.x / kColLanes;
  const int ch0 = blockIdx.x * SLAB + cl * V;
  const bool col_ok = ch0 < d;
  if (add_count && blockIdx.x == 0 && threadIdx.x == 0) stats[size_t(s) * stats_stride] += float(m);

  raw_t x[kWeighRows];
  auto load_pass = [&](int pass) {
#pragma unroll
    for (int i = 0; i < kWeighRows; ++i) {
      const int r = pass * kWeighRowsPerPass + rl * kWeighRows + i;
      x[i] = Vec<T>::load_raw(q + size_t(r < m ? r : 0) * d + (col_ok ? ch0 : 0));
    }
  };
  load_pass(0);

  float tsum = 0.f;
  for (int j = threadIdx.x; j < m && !mean_pooling; j += 512) {
    float t = 0.f;
    for (int s0 = 0; s0 < n_slabs; s0 += kWeighSlabBatch) {
      float p[kWeighSlabBatch];
#pragma unroll
      for (int i = 0; i < kWeighSlabBatch; ++i)   // all loads first: they overlap
        p[i] = apart[size_t(s0 + i < n_slabs ? s0 + i : s0) * m_pad + j];
#pragma unroll
      for (int i = 0; i < kWeighSlabBatch; ++i) t += s0 + i < n_slabs ? p[i] : 0.f;
    }
    w_lds[j] = t;
    tsum += t;
  }
  const float total = block_sum(tsum, red);          // |Phi|_1; orders the LDS writes as well
  const float inv_total = total > 0.f ? 1.f / total : 0.f;
  const float uniform = 1.f / float(m);

  float acc[V];
#pragma unroll
  for (int v = 0; v < V; ++v) acc[v] = 0.f;
  const int n_pass = (m + kWeighRowsPerPass - 1) / kWeighRowsPerPass;
  for (int pass = 0; pass < n_pass; ++pass) {
    if (pass > 0) load_pass(pass);
#pragma unroll
    for (int i = 0; i < kWeighRows; ++i) {
      const int r = pass * kWeighRowsPerPass + rl * kWeighRows + i;
      const float w = r < m ? (total > 0.f ? w_lds[r] * inv_total : uniform) : 0.f;
      float f[V];
      Vec<T>::widen(x[i], f);
#pragma unroll
      for (int v = 0; v < V; ++v) acc[v] += w * f[v];
    }
  }
  // the 8 row lanes of a wave first, then the 8 waves through LDS
#pragma unroll
  for (int v = 0; v < V; ++v) {
    acc[v] += __shfl_xor(acc[v], 8, 64);
    acc[v] += __shfl_xor(acc[v], 16, 64);
    acc[v] += __shfl_xor(acc[v], 32, 64);
  }
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  if (lane < kColLanes) {
#pragma unroll
    for (int v = 0; v < V; ++v) buf[wv][cl * V + v] = acc[v];
  }
  __syncthreads();
  if (threadIdx.x < SLAB) {
    const int ch = blockIdx.x * SLAB + threadIdx.x;
    if (ch < d) {
      float t = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) t += buf[i][threadIdx.x];
      probe_out[size_t(s) * d + ch] = t;
    }
  }
  if (blockIdx.x == 0 && weights_out != nullptr) {
    for (int j = threadIdx.x; j < m; j += 512)
      weights_out[size_t(s) * m + j] = total > 0.f ? w_lds[j] * inv_total : uniform;
  }
}

// One workgroup per sequence that sees the whole probe.
__global__ __launch_bounds__(1024) void probe_finish_kernel(const float* __restrict__ probe,
                                                            float* __restrict__ probe_kv_out,
                                                            float* __restrict__ probe_norm_out,
                                                            int n_q_heads, int n_kv_heads,
                                                            int head_dim) {
  __shared__ float red[32];
  const int s = blockIdx.x;
  probe_finish(probe + size_t(s) * n_q_heads * head_dim,
               probe_kv_out + size_t(s) * n_kv_heads * head_dim, probe_norm_out + s, n_q_heads,
               n_kv_heads, head_dim, red);
}

// A window of one token (decode): the probe is the query (probe_identity.h).
template <typename T>
__global__ __launch_bounds__(1024) void probe_identity_kernel(
    const T* __restrict__ q_win, float* __restrict__ stats, int add_count, size_t stats_stride,
    float* __restrict__ probe_out, float* __restrict__ probe_kv_out, float* __restrict__ probe_norm_out,
    float* __restrict__ weights_out, int n_q_heads, int n_kv_heads, int head_dim) {
  __shared__ float red[32];
  extern __shared__ __attribute__((aligned(16))) float probe_lds[];   // [d]
  const int d = n_q_heads * head_dim;
  const int s = blockIdx.x;
  if (add_count && threadIdx.x == 0) stats[size_t(s) * stats_stride] += 1.f;
  probe_identity_body<T>(q_win + size_t(s) * d, probe_out + size_t(s) * d,
                         probe_kv_out + size_t(s) * n_kv_heads * head_dim, probe_norm_out + s,
                         weights_out != nullptr ? weights_out + s : nullptr, n_q_heads, n_kv_heads, head_dim,
                         probe_lds, red);
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
  const int m_pad = int(probe_a_floats(m));
  const int n_slabs = probe_slabs(sh);
  static_assert(kColLanes * 8 == kProbeSlabBytes / 2 && kColLanes * 4 == kProbeSlabBytes / 4, "slab width");
  float* scratch = ws.scratch_f32();
  const int mean_pooling = (update_stats & ACTQKV_PROBE_MEAN_POOLING) != 0;
  if (update_stats & ACTQKV_PROBE_WINDOW_CHAIN) {
    // the batch entries are consecutive windows of one sequence with one set of statistics
    float* mom = scratch + size_t(batch) * scratch_stride;
    float* base = mom + size_t(batch) * 2 * d;
    hipLaunchKernelGGL(probe_window_moments_kernel<T>, dim3(n_slabs, batch), dim3(256), 0, stream, q_win,
                       stats, mom, base, m, d);
    hipLaunchKernelGGL(probe_chain_bias_kernel<T>, dim3(n_slabs, batch), dim3(256), 0, stream, q_win, stats,
                       mom, base, scratch, m, m_pad, d, eps, scratch_stride);
    hipLaunchKernelGGL(probe_weigh_kernel<T>, dim3(n_slabs, batch), dim3(512), 0, stream, q_win, scratch,
                       stats, 0, mean_pooling, probe, weights, m, m_pad, n_slabs, d, scratch_stride,
                       size_t(0));
    hipLaunchKernelGGL(probe_finish_kernel, dim3(batch), dim3(1024), 0, stream, probe, probe_kv,
                       probe_norm, sh.n_q_heads, sh.n_kv_heads, sh.head_dim);
    return hip_status("probe");
  }
  update_stats &= ACTQKV_STATS_UPDATE;
  if (update_stats || (m > 1 && !mean_pooling)) {
    hipLaunchKernelGGL(probe_stats_bias_kernel<T>, dim3(n_slabs, batch), dim3(256), 0, stream, q_win,
                       stats, scratch, update_stats, m, m_pad, d, eps, stats_stride, scratch_stride);
  }
  if (m == 1) {
    hipLaunchKernelGGL(probe_identity_kernel<T>, dim3(batch), dim3(1024), size_t(d) * sizeof(float),
                       stream, q_win, stats,
                       update_stats, stats_stride, probe, probe_kv, probe_norm, weights, sh.n_q_heads,
                       sh.n_kv_heads, sh.head_dim);
    return hip_status("probe");
  }
  hipLaunchKernelGGL(probe_weigh_kernel<T>, dim3(n_slabs, batch), dim3(512), 0, stream, q_win, scratch,
                     stats, update_stats, mean_pooling, probe, weights, m, m_pad, n_slabs, d, scratch_stride,
                     stats_stride);
  hipLaunchKernelGGL(probe_finish_kernel, dim3(batch), dim3(1024), 0, stream, probe, probe_kv,
                     probe_norm, sh.n_q_heads, sh.n_kv_heads, sh.head_dim);
  (void)V;
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
