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
// into the running statistics one after the other, but a merge is a function of each window's
// own (mean, M2) only, so everything else is done for all windows at once (kernels further
// down).  Four launches for n windows instead of 3 n.
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

// ---- consecutive windows of one sequence in one call
// With many windows in a call there is enough work to read the queries the way they lie in
// memory: a workgroup takes 64 whole rows (rows x all channels, 16-byte loads of consecutive
// lanes are consecutive in memory), where the one-window kernels above take 128-byte column
// slabs of all rows.  Reductions over rows leave one partial per 64-row chunk, summed in chunk
// order by the next kernel; reductions over channels are whole-row sums inside a wavefront, so
// the bias weight a_j of a row is complete while the row is still in registers and Eq. (9)'s
// weighted sum is taken in the same pass: the queries are read twice, not three times.
//   rows_moments     (chunks x windows): sums of (q - c) and (q - c)^2 per channel over the
//                    chunk's rows, c = the window's first query;
//   chain_stats      per channel: every window's own (mean, M2) from its chunks, then the merges
//                    of Eq. (8) window after window, which give the (mean, 1/var) each window
//                    sees; stores the final statistics;
//   rows_bias_weigh  (chunks x windows): a_j = |phi_j|_1 per row, sum of a_j q_j over the chunk's
//                    rows per channel, sum of a_j;
//   chain_finish     per window: probe = sum over chunks / sum of a_j, norm, per-KV-head sum,
//                    weights.
// Scratch per call, in floats: part [n][chunks][2][d], stat [n][3][d] (mean, 1/var, the window's
// own mean), pprobe [n][chunks][d], asum [n][chunks rounded up to 16], a [n][m rounded up to 16].
constexpr int kRmThreads = 256;

template <typename T>
__global__ __launch_bounds__(kRmThreads) void probe_rows_moments_kernel(const T* __restrict__ q_win,
                                                                        float* __restrict__ part, int m, int d,
                                                                        int n_chunks) {
  constexpr int V = Vec<T>::N;
  constexpr int G = 2;                               // 16-byte channel groups per thread
  constexpr int R = 8;                               // rows requested together
  typedef typename Vec<T>::raw raw_t;
  const int rc = blockIdx.x, w = blockIdx.y;
  const T* q = q_win + size_t(w) * m * d;
  int ch[G];
  bool ok[G];
  float c[G][V], s1[G][V], s2[G][V];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    ch[g] = ((blockIdx.z * G + g) * kRmThreads + threadIdx.x) * V;
    ok[g] = ch[g] < d;
    Vec<T>::load(q + (ok[g] ? ch[g] : 0), c[g]);
#pragma unroll
    for (int v = 0; v < V; ++v) s1[g][v] = s2[g][v] = 0.f;
  }
  const int r0 = rc * kRowChunk, r1 = min(r0 + kRowChunk, m);
  for (int r = r0; r < r1; r += R) {
    raw_t x[R][G];
#pragma unroll
    for (int i = 0; i < R; ++i)
#pragma unroll
      for (int g = 0; g < G; ++g)
        x[i][g] = Vec<T>::load_raw(q + size_t(min(r + i, r1 - 1)) * d + (ok[g] ? ch[g] : 0));
#pragma unroll
    for (int i = 0; i < R; ++i) {
      if (r + i < r1) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
          float f[V];
          Vec<T>::widen(x[i][g], f);
#pragma unroll
          for (int v = 0; v < V; ++v) {
            const float t = f[v] - c[g][v];
            s1[g][v] += t;
            s2[g][v] += t * t;
          }
        }
      }
    }
  }
  float* p1 = part + (size_t(w) * n_chunks + rc) * 2 * d;
#pragma unroll
  for (int g = 0; g < G; ++g) {
    if (ok[g]) {
#pragma unroll
      for (int v = 0; v < V; v += 4) {
        *reinterpret_cast<f32x4*>(p1 + ch[g] + v) = f32x4{s1[g][v], s1[g][v + 1], s1[g][v + 2], s1[g][v + 3]};
        *reinterpret_cast<f32x4*>(p1 + d + ch[g] + v) = f32x4{s2[g][v], s2[g][v + 1], s2[g][v + 2], s2[g][v + 3]};
      }
    }
  }
}

// grid (d / 32), 1024 threads = 32 channels x 32 window lanes.  Window lane wl first turns the
// chunk sums of windows wl, wl + 32, ... into the window's own (mean, M2) in LDS; then window
// lane 0 merges them into the running statistics in window order (the merge of Eq. (8), as in
// probe_stats_bias_kernel).  The count is published by the next kernel (every thread here
// reads the old one).
template <typename T>
__global__ __launch_bounds__(1024) void probe_chain_stats_kernel(const T* __restrict__ q_win,
                                                                 const float* __restrict__ part,
                                                                 float* __restrict__ stats,
                                                                 float* __restrict__ stat_out, int n, int m,
                                                                 int d, int n_chunks, float eps) {
  extern __shared__ float wm[];                      // [n][2][32]: the windows' own mean and M2
  const int cl = threadIdx.x & 31, wl = threadIdx.x >> 5;
  const int ch = blockIdx.x * 32 + cl;
  const float nb = float(m);
  if (ch < d) {
    for (int w = wl; w < n; w += 32) {
      const float* p1 = part + size_t(w) * n_chunks * 2 * d + ch;
      float t1 = 0.f, t2 = 0.f;
      for (int rc = 0; rc < n_chunks; ++rc) {
        t1 += p1[size_t(rc) * 2 * d];
        t2 += p1[size_t(rc) * 2 * d + d];
      }
      wm[(w * 2 + 0) * 32 + cl] = to_f32(q_win[size_t(w) * m * d + ch]) + t1 / nb;
      wm[(w * 2 + 1) * 32 + cl] = fmaxf(t2 - t1 * t1 / nb, 0.f);
    }
  }
  __syncthreads();
  if (wl != 0 || ch >= d) return;
  float n_run = stats[0], mean = stats[4 + ch], m2 = stats[4 + d + ch];
  for (int w = 0; w < n; ++w) {
    const float mean_b = wm[(w * 2 + 0) * 32 + cl], m2_b = wm[(w * 2 + 1) * 32 + cl];
    const float n_new = n_run + nb;
    if (n_run > 0.f) {
      const float delta = mean_b - mean;
      mean += delta * (nb / n_new);
      m2 += m2_b + delta * delta * (n_run * nb / n_new);
    } else {
      mean = mean_b;
      m2 = m2_b;
    }
    n_run = n_new;
    const float var = n_run > 1.f ? m2 / (n_run - 1.f) : 0.f;
    float* o = stat_out + size_t(w) * 3 * d + ch;
    o[0] = mean;
    o[d] = 1.f / fmaxf(var, eps);
    o[2 * d] = mean_b;
  }
  stats[4 + ch] = mean;
  stats[4 + d + ch] = m2;
}

// grid (chunks, windows), 4 wavefronts; wavefront v takes rows v, v + 4, ... of the chunk, a lane
// the 16-byte groups lane, lane + 64, ... of a row (NI of them: d <= 64 * NI * V channels).
// LDS: mean and 1/var of the window (2 d floats), reused for the sum over the 4 wavefronts.
template <typename T>
__global__ __launch_bounds__(kRmThreads) void probe_rows_bias_weigh_kernel(
    const T* __restrict__ q_win, const float* __restrict__ stat_in, float* __restrict__ stats, float add_count,
    int mean_pooling, float* __restrict__ pprobe, float* __restrict__ asum, float* __restrict__ a_rows, int m,
    int m_pad, int d, int n_chunks, int asum_stride) {
  constexpr int V = Vec<T>::N;
  constexpr int NI = 64 / V;
  typedef typename Vec<T>::raw raw_t;
  constexpr int kRowLen = 64 * NI * V;                             // channels a wavefront covers
  extern __shared__ __attribute__((aligned(16))) float rw_lds[];   // [2][kRowLen]
  __shared__ float red[4];
  const int rc = blockIdx.x, w = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const T* q = q_win + size_t(w) * m * d;
  float* mu = rw_lds;
  float* iv = rw_lds + kRowLen;
  // channels past d (rows shorter than a wavefront's 64 * NI * V) get mean 0 and weight 0
  for (int i = threadIdx.x * 4; i < kRowLen; i += kRmThreads * 4) {
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    *reinterpret_cast<f32x4*>(mu + i) = i < d ? *reinterpret_cast<const f32x4*>(stat_in + size_t(w) * 3 * d + i) : zero;
    *reinterpret_cast<f32x4*>(iv + i) = i < d ? *reinterpret_cast<const f32x4*>(stat_in + size_t(w) * 3 * d + d + i) : zero;
  }
  if (add_count != 0.f && rc == 0 && w == 0 && threadIdx.x == 0) stats[0] += add_count;
  __syncthreads();
  float acc[NI][V];
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int v = 0; v < V; ++v) acc[i][v] = 0.f;
  float a_sum = 0.f;
  const int r0 = rc * kRowChunk, r1 = min(r0 + kRowChunk, m);
  auto load_row = [&](int r, raw_t (&x)[NI]) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int c = (lane + 64 * i) * V;
      x[i] = Vec<T>::load_raw(q + size_t(r) * d + (c < d ? c : 0));
    }
  };
  raw_t x[NI];
  if (r0 + wave < r1) load_row(r0 + wave, x);
  for (int r = r0 + wave; r < r1; r += 4) {
    // the wavefront's next row is requested before this one is used: a row's worth of loads is in
    // flight the whole time (the last row asks for itself once more, which costs nothing that matters)
    raw_t xn[NI];
    load_row(r + 4 < r1 ? r + 4 : r, xn);
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int c = (lane + 64 * i) * V;
      float f[V];
      Vec<T>::widen(x[i], f);
      f32x4 mu4[V / 4], iv4[V / 4];
#pragma unroll
      for (int u = 0; u < V / 4; ++u) {
        mu4[u] = *reinterpret_cast<const f32x4*>(mu + c + 4 * u);
        iv4[u] = *reinterpret_cast<const f32x4*>(iv + c + 4 * u);
      }
#pragma unroll
      for (int v = 0; v < V; ++v) {
        const float e = f[v] - mu4[v >> 2][v & 3];
        t += e * e * iv4[v >> 2][v & 3];
      }
    }
    float a = wave_sum(t);                           // |phi_j|_1 of Eq. (7), the row's weight before normalisation
    if (mean_pooling) a = 1.f;
    if (lane == 0) a_rows[size_t(w) * m_pad + r] = a;
    a_sum += a;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      float f[V];
      Vec<T>::widen(x[i], f);
#pragma unroll
      for (int v = 0; v < V; ++v) acc[i][v] += a * f[v];
    }
#pragma unroll
    for (int i = 0; i < NI; ++i) x[i] = xn[i];
  }
  // sum over the 4 wavefronts, in a fixed order: (0 + 2) + (1 + 3)
  __syncthreads();                                   // mean and 1/var are no longer needed
  if (lane == 0) red[wave] = a_sum;
  auto put = [&](float* dst) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int c = (lane + 64 * i) * V;
      if (c < d) {
#pragma unroll
        for (int v = 0; v < V; v += 4)
          *reinterpret_cast<f32x4*>(dst + c + v) = f32x4{acc[i][v], acc[i][v + 1], acc[i][v + 2], acc[i][v + 3]};
      }
    }
  };
  auto add = [&](const float* src) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int c = (lane + 64 * i) * V;
      if (c < d) {
#pragma unroll
        for (int v = 0; v < V; ++v) acc[i][v] += src[c + v];
      }
    }
  };
  if (wave >= 2) put(rw_lds + (wave - 2) * d);
  __syncthreads();
  if (wave < 2) add(rw_lds + wave * d);
  __syncthreads();
  if (wave == 1) put(rw_lds);
  __syncthreads();
  if (wave == 0) {
    add(rw_lds);
    put(pprobe + (size_t(w) * n_chunks + rc) * d);
    if (lane == 0) asum[size_t(w) * asum_stride + rc] = (red[0] + red[2]) + (red[1] + red[3]);
  }
}

// One workgroup per window: the chunk sums in chunk order, Eq. (9)'s normalisation (uniform
// weights, i.e. the window's mean, if every bias is zero), the weights, and what probe_finish
// computes.
__global__ __launch_bounds__(1024) void probe_chain_finish_kernel(
    const float* __restrict__ pprobe, const float* __restrict__ asum, const float* __restrict__ a_rows,
    const float* __restrict__ stat_in, float* __restrict__ probe_out, float* __restrict__ probe_kv_out,
    float* __restrict__ probe_norm_out, float* __restrict__ weights_out, int m, int m_pad, int d, int n_chunks,
    int asum_stride, int n_q_heads, int n_kv_heads, int head_dim) {
  __shared__ float red[32];
  extern __shared__ __attribute__((aligned(16))) float probe_lds[];   // [d]
  const int w = blockIdx.x;
  float total = 0.f;
  for (int rc = 0; rc < n_chunks; ++rc) total += asum[size_t(w) * asum_stride + rc];
  const bool uniform = !(total > 0.f);
  const float inv = uniform ? 0.f : 1.f / total;
  float* probe = probe_out + size_t(w) * d;
  float ss = 0.f;
  for (int ch = threadIdx.x; ch < d; ch += 1024) {
    float t = 0.f;
    for (int rc = 0; rc < n_chunks; ++rc) t += pprobe[(size_t(w) * n_chunks + rc) * d + ch];
    t = uniform ? stat_in[size_t(w) * 3 * d + 2 * d + ch] : t * inv;
    probe[ch] = t;
    probe_lds[ch] = t;
    ss += t * t;
  }
  if (weights_out != nullptr) {
    for (int j = threadIdx.x; j < m; j += 1024)
      weights_out[size_t(w) * m + j] = uniform ? 1.f / float(m) : a_rows[size_t(w) * m_pad + j] * inv;
  }
  ss = block_sum(ss, red);                           // also orders the LDS writes before the reads below
  if (threadIdx.x == 0) probe_norm_out[w] = sqrtf(ss);
  const int g = n_q_heads / n_kv_heads;
  float* probe_kv = probe_kv_out + size_t(w) * n_kv_heads * head_dim;
  for (int e = threadIdx.x; e < n_kv_heads * head_dim; e += 1024) {
    const int hk = e / head_dim, dd = e - hk * head_dim;
    float t = 0.f;
    for (int i = 0; i < g; ++i) t += probe_lds[(hk * g + i) * head_dim + dd];
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
    if (d > 64 * 64) {
      // rows wider than a wavefront of the row-major kernels holds: window after window
      const int dk = sh.n_kv_heads * sh.head_dim;
      for (int w = 0; w < batch; ++w) {
        const int rc = launch_probe_t<T>(sh, 1, m, q_win + size_t(w) * m * d, stats,
                                         update_stats & ~ACTQKV_PROBE_WINDOW_CHAIN, probe + size_t(w) * d,
                                         probe_kv + size_t(w) * dk, probe_norm + w,
                                         weights != nullptr ? weights + size_t(w) * m : nullptr, ws, stream);
        if (rc != ACTQKV_OK) return rc;
      }
      return ACTQKV_OK;
    }
    const ChainScratch cl = chain_scratch(sh, batch, m);
    float* part = scratch;
    float* stat = part + cl.part;
    float* pprobe = stat + cl.stat;
    float* asum = pprobe + cl.pprobe;
    float* a_rows = asum + cl.asum;
    const int n_chunks = cl.n_chunks;
    hipLaunchKernelGGL(probe_rows_moments_kernel<T>, dim3(n_chunks, batch, (d + 2 * kRmThreads * V - 1) / (2 * kRmThreads * V)),
                       dim3(kRmThreads), 0, stream, q_win, part, m, d, n_chunks);
    hipLaunchKernelGGL(probe_chain_stats_kernel<T>, dim3((d + 31) / 32), dim3(1024), size_t(batch) * 64 * sizeof(float),
                       stream, q_win, part, stats, stat, batch, m, d, n_chunks, eps);
    hipLaunchKernelGGL(probe_rows_bias_weigh_kernel<T>, dim3(n_chunks, batch), dim3(kRmThreads),
                       size_t(2) * 4096 * sizeof(float), stream, q_win, stat, stats, float(batch) * float(m), mean_pooling,
                       pprobe, asum, a_rows, m, m_pad, d, n_chunks, cl.asum_stride);
    hipLaunchKernelGGL(probe_chain_finish_kernel, dim3(batch), dim3(1024), size_t(d) * sizeof(float), stream, pprobe,
                       asum, a_rows, stat,
                       probe, probe_kv, probe_norm, weights, m, m_pad, d, n_chunks, cl.asum_stride, sh.n_q_heads,
                       sh.n_kv_heads, sh.head_dim);
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
