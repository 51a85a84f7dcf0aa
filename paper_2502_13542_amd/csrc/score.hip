// Block scores (Sec. 4.2, Eq. (10), applied to the r representative keys of a block;
// the objective of Sec. 3.2, Eq. (5) ranks blocks by the sum of these cosines).
//
// HBM-bound streaming kernel: every representative key is read exactly once with
// 16-byte loads.  One wavefront scores one block; each group of 16 lanes walks one
// representative key (consecutive lanes read consecutive 16-byte chunks), so a
// wavefront keeps four keys in flight.  The group-summed probe sits in LDS.
#include "common.h"
#include "launch.h"
#include "score_body.h"

namespace actqkv {

template <typename T>
__global__ __launch_bounds__(1024) void score_blocks_kernel(
    const float* __restrict__ probe_kv, const float* __restrict__ probe_norm,
    const T* __restrict__ rep_keys, int64_t seq_stride, int nb_capacity, int nb_begin,
    const int32_t* __restrict__ nb_end, float* __restrict__ scores, int64_t score_stride, int n_rep,
    int key_len, float inv_sqrt_g) {
  extern __shared__ __attribute__((aligned(16))) float probe_lds[];  // [key_len]
  const int s = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int end = min(nb_end[s], nb_capacity);
  const int b = nb_begin + blockIdx.x * int(blockDim.x >> 6) + wave;
  const bool live = b < end;
  // the first batch of key loads is in flight while the probe goes to LDS
  BlockScorer<T> scorer;
  scorer.start(rep_keys + size_t(s) * seq_stride + size_t(live ? b : nb_begin) * n_rep * key_len, n_rep,
               key_len, lane);
  {
    const float* src = probe_kv + size_t(s) * key_len;
    for (int i = threadIdx.x * 4; i < key_len; i += int(blockDim.x) * 4)
      *reinterpret_cast<f32x4*>(probe_lds + i) = *reinterpret_cast<const f32x4*>(src + i);
  }
  __syncthreads();
  if (!live) return;
  const float total = scorer.finish(probe_lds, probe_norm[s], inv_sqrt_g);
  if (lane == 0) scores[size_t(s) * score_stride + b] = total;
}

// The same score for every KV head on its own (the alternative to the head-merged reading):
// scores[s][hk][b] = mean over the r keys of cos(probe of the G query heads of group hk, key of
// head hk repeated to those heads) = mean_j <probe_kv[hk], k_j[hk]> / (|probe_hk| sqrt(G) |k_j[hk]|).
// grid (blocks / (16 wavefronts x 4), Hk, batch); a wavefront scores 4 blocks of one KV head, a
// 16-lane group walking one key's D elements of that head, the loads of all 4 blocks requested
// before the first is used.  The workgroup first forms the group's summed probe and the norm
// of the group's share of the probe in LDS (amortised over its 64 blocks).
constexpr int kPhBlocksPerWave = 4;

template <typename T>
__global__ __launch_bounds__(1024) void score_blocks_per_head_kernel(
    const float* __restrict__ probe, const T* __restrict__ rep_keys, int64_t seq_stride, int nb_capacity,
    int nb_begin, const int32_t* __restrict__ nb_end, float* __restrict__ scores, int64_t score_stride,
    int n_rep, int n_kv_heads, int group, int head_dim, float inv_sqrt_g) {
  constexpr int V = Vec<T>::N;
  extern __shared__ __attribute__((aligned(16))) float probe_lds[];  // [head_dim]
  __shared__ float red[32];
  const int hk = blockIdx.y, s = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
  const int gq = lane >> 4, l16 = lane & 15;
  const int chunks = head_dim / V;
  const float* pr = probe + (size_t(s) * n_kv_heads + hk) * group * head_dim;
  float ss = 0.f;
  for (int i = threadIdx.x; i < group * head_dim; i += blockDim.x) ss += pr[i] * pr[i];
  ss = block_sum(ss, red);
  for (int dd = threadIdx.x; dd < head_dim; dd += blockDim.x) {
    float t = 0.f;
    for (int g = 0; g < group; ++g) t += pr[g * head_dim + dd];
    probe_lds[dd] = t;
  }
  __syncthreads();
  const float pn = sqrtf(ss);
  const int end = min(nb_end[size_t(s) * n_kv_heads + hk], nb_capacity);
  const int b0 = nb_begin + (blockIdx.x * n_waves + wave) * kPhBlocksPerWave;
  if (b0 >= end) return;
  const int key_len = n_kv_heads * head_dim;
  const T* head_keys = rep_keys + size_t(s) * seq_stride + size_t(hk) * head_dim;
  float total[kPhBlocksPerWave];
#pragma unroll
  for (int u = 0; u < kPhBlocksPerWave; ++u) total[u] = 0.f;
  for (int j0 = 0; j0 < n_rep; j0 += 4) {
    const int j = j0 + gq;
    float dot[kPhBlocksPerWave], nrm[kPhBlocksPerWave];
#pragma unroll
    for (int u = 0; u < kPhBlocksPerWave; ++u) dot[u] = nrm[u] = 0.f;
    for (int c = l16; c < chunks; c += 16) {
      float k[kPhBlocksPerWave][V];
#pragma unroll
      for (int u = 0; u < kPhBlocksPerWave; ++u) {                   // all loads first: they overlap
        const int b = min(b0 + u, end - 1);
        Vec<T>::load(head_keys + (size_t(b) * n_rep + (j < n_rep ? j : 0)) * key_len + c * V, k[u]);
      }
#pragma unroll
      for (int u = 0; u < kPhBlocksPerWave; ++u)
#pragma unroll
        for (int v = 0; v < V; ++v) {
          dot[u] += probe_lds[c * V + v] * k[u][v];
          nrm[u] += k[u][v] * k[u][v];
        }
    }
#pragma unroll
    for (int u = 0; u < kPhBlocksPerWave; ++u) {
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) {
        dot[u] += __shfl_xor(dot[u], o, 64);
        nrm[u] += __shfl_xor(nrm[u], o, 64);
      }
      float c = (j < n_rep && nrm[u] > 0.f && pn > 0.f) ? dot[u] * inv_sqrt_g / (pn * sqrtf(nrm[u])) : 0.f;
      c += __shfl_xor(c, 16, 64);
      c += __shfl_xor(c, 32, 64);
      total[u] += c;
    }
  }
  if (lane < kPhBlocksPerWave && b0 + lane < end) {
    float t = total[0];
#pragma unroll
    for (int u = 1; u < kPhBlocksPerWave; ++u) t = lane == u ? total[u] : t;
    scores[(size_t(s) * n_kv_heads + hk) * score_stride + b0 + lane] = t / float(n_rep);
  }
}

int launch_score_per_head(const actqkv_shape& sh, int batch, const float* probe, const void* rep_keys,
                          int64_t seq_stride, int nb_capacity, int nb_begin, const int32_t* nb_end,
                          float* scores, int64_t score_stride, hipStream_t stream) {
  const int n = nb_capacity - nb_begin;
  if (n <= 0) return ACTQKV_OK;
  const int group = sh.n_q_heads / sh.n_kv_heads;
  const float inv_sqrt_g = 1.f / sqrtf(float(group));
  const int waves = 16, per_wg = waves * kPhBlocksPerWave;
  dim3 grid((n + per_wg - 1) / per_wg, sh.n_kv_heads, batch), block(64 * waves);
  const size_t lds = size_t(sh.head_dim) * sizeof(float);
  if (sh.dtype == ACTQKV_F32)
    hipLaunchKernelGGL(score_blocks_per_head_kernel<float>, grid, block, lds, stream, probe,
                       static_cast<const float*>(rep_keys), seq_stride, nb_capacity, nb_begin, nb_end, scores,
                       score_stride, sh.n_rep, sh.n_kv_heads, group, sh.head_dim, inv_sqrt_g);
  else
    hipLaunchKernelGGL(score_blocks_per_head_kernel<uint16_t>, grid, block, lds, stream, probe,
                       static_cast<const uint16_t*>(rep_keys), seq_stride, nb_capacity, nb_begin, nb_end,
                       scores, score_stride, sh.n_rep, sh.n_kv_heads, group, sh.head_dim, inv_sqrt_g);
  return hip_status("score_blocks_per_head");
}

int launch_score(const actqkv_shape& sh, int batch, const float* probe_kv, const float* probe_norm,
                 const void* rep_keys, int64_t seq_stride, int nb_capacity, int nb_begin,
                 const int32_t* nb_end, float* scores, int64_t score_stride, hipStream_t stream) {
  const int n = nb_capacity - nb_begin;
  if (n <= 0) return ACTQKV_OK;
  const int key_len = sh.n_kv_heads * sh.head_dim;
  const float inv_sqrt_g = 1.f / sqrtf(float(sh.n_q_heads / sh.n_kv_heads));
  // One wavefront per block.  A single long sequence (prefill) gets at most 64 workgroups,
  // so that the kernel fits beside a prefill attention that leaves 64 compute units free.
  int waves = 4;
  if (batch == 1) {
    while (waves < 16 && (n + waves - 1) / waves > 64) waves *= 2;
  }
  dim3 grid((n + waves - 1) / waves, batch), block(64 * waves);
  const size_t lds = size_t(key_len) * sizeof(float);
  if (sh.dtype == ACTQKV_F32)
    hipLaunchKernelGGL(score_blocks_kernel<float>, grid, block, lds, stream, probe_kv, probe_norm,
                       static_cast<const float*>(rep_keys), seq_stride, nb_capacity, nb_begin, nb_end,
                       scores, score_stride, sh.n_rep, key_len, inv_sqrt_g);
  else
    hipLaunchKernelGGL(score_blocks_kernel<uint16_t>, grid, block, lds, stream, probe_kv,
                       probe_norm, static_cast<const uint16_t*>(rep_keys), seq_stride, nb_capacity,
                       nb_begin, nb_end, scores, score_stride, sh.n_rep, key_len, inv_sqrt_g);
  return hip_status("score_blocks");
}

}  // namespace actqkv
