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

#include <algorithm>
#include <mutex>

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

// ---- many windows of ONE sequence against the same representative keys ----------------------
// The prefill pass scores 32 consecutive windows in one call (seq_stride 0: they share the keys).
// Then the dot products of Eq. (10) are a [windows x key_len] x [key_len x keys] contraction, and
// a kernel that walks the keys once per window reads every key 32 times from the caches.  Here a
// wavefront loads a tile of 32 keys ONCE, straight from memory in the matrix-core operand
// layout (lane l: key l % 32, channels 8 (l / 32) .. + 8 of each step of 16 channels), and
// multiplies it with the probes of 32 windows, which the workgroup keeps in LDS split into two
// bf16 halves (p = hi + lo, |p - hi - lo| <= 2^-17 |p|: the products with bf16 keys are exact in
// fp32, so the result is that of fp32 arithmetic up to the order of the additions).
// D[window][key]: a lane ends with one key (column l % 32) and 16 windows (rows 4 (l / 32) +
// 8 (i / 4) + i % 4), so the key's norm is the lane's own and the r keys of a block sit in
// adjacent lanes.  grid (workgroups that take tiles round-robin, groups of 32 windows).
constexpr int kSsWaves = 4;
constexpr int kSsLoads = 16;    // 16-byte key loads a lane keeps in flight

__device__ __forceinline__ void ss_split(float p, uint32_t& hi, uint32_t& lo) {
  hi = f32_to_bf16_bits(p);
  lo = f32_to_bf16_bits(p - __uint_as_float(hi << 16));
}

__global__ __launch_bounds__(64 * kSsWaves) void score_shared_mfma_kernel(
    const float* __restrict__ probe_kv, const float* __restrict__ probe_norm,
    const uint16_t* __restrict__ rep_keys, int nb_capacity, int nb_begin, const int32_t* __restrict__ nb_end,
    float* __restrict__ scores, int64_t score_stride, int batch, int n_rep, int key_len, float inv_sqrt_g) {
  extern __shared__ __attribute__((aligned(16))) u32x4 ss_lds[];   // [hi, lo][key_len / 8][32 windows] x 8 bf16
  const int chunks = key_len / 8;
  const int w0 = blockIdx.y * 32;
  u32x4* lds_hi = ss_lds;
  u32x4* lds_lo = ss_lds + chunks * 32;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int h = lane >> 5, col = lane & 31;
  const int n_keys = (nb_capacity - nb_begin) * n_rep;
  const int n_tiles = (n_keys + 31) / 32;
  const int steps = key_len / 16;                      // a multiple of kSsLoads (the launcher checks)
  const uint16_t* keys0 = rep_keys + size_t(nb_begin) * n_rep * key_len + h * 8;
  auto tile_keys = [&](int tile) {                     // the lane's key of a tile (a valid one for any tile)
    return keys0 + size_t(min(min(tile, n_tiles - 1) * 32 + col, n_keys - 1)) * key_len;
  };
  // a ring of kSsLoads key loads per lane, refilled as it is used; its first round is in flight
  // while the probes go to LDS
  int tile = blockIdx.x * kSsWaves + wave;
  const uint16_t* kp = tile_keys(tile);
  u32x4 kb[kSsLoads];
#pragma unroll
  for (int i = 0; i < kSsLoads; ++i) kb[i] = *reinterpret_cast<const u32x4*>(kp + i * 16);

  for (int e0 = threadIdx.x; e0 < chunks * 32; e0 += 4 * int(blockDim.x)) {
    f32x4 a[4], b[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {                      // four chunks' loads before the first conversion
      const int e = e0 + u * int(blockDim.x);
      const int wl = e & 31, ch = e >> 5;
      a[u] = f32x4{0.f, 0.f, 0.f, 0.f};
      b[u] = a[u];
      if (e < chunks * 32 && w0 + wl < batch) {
        const float* src = probe_kv + size_t(w0 + wl) * key_len + ch * 8;
        a[u] = *reinterpret_cast<const f32x4*>(src);
        b[u] = *reinterpret_cast<const f32x4*>(src + 4);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int e = e0 + u * int(blockDim.x);
      if (e >= chunks * 32) break;
      const float p[8] = {a[u].x, a[u].y, a[u].z, a[u].w, b[u].x, b[u].y, b[u].z, b[u].w};
      uint32_t hi[8], lo[8];
#pragma unroll
      for (int v = 0; v < 8; ++v) ss_split(p[v], hi[v], lo[v]);
      lds_hi[e] = u32x4{hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16), hi[4] | (hi[5] << 16), hi[6] | (hi[7] << 16)};
      lds_lo[e] = u32x4{lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16), lo[4] | (lo[5] << 16), lo[6] | (lo[7] << 16)};
    }
  }
  // the lane's 16 windows: the probe's norm and the end of the eligible blocks
  float pn_w[16];
  int end_w[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int w = w0 + 4 * h + 8 * (i >> 2) + (i & 3);
    const bool ok = w < batch;
    pn_w[i] = ok ? probe_norm[w] : 0.f;
    end_w[i] = ok ? min(nb_end[w], nb_capacity) : 0;
  }
  __syncthreads();
  const int stride = gridDim.x * kSsWaves;
  while (tile < n_tiles) {
    const uint16_t* kp_next = tile_keys(tile + stride);
    f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    float nrm = 0.f;
    for (int s0 = 0; s0 < steps; s0 += kSsLoads) {
      const uint16_t* refill = s0 + kSsLoads < steps ? kp + size_t(s0 + kSsLoads) * 16 : kp_next;
#pragma unroll
      for (int i = 0; i < kSsLoads; ++i) {
        const int at = ((s0 + i) * 2 + h) * 32 + col;
        const bf16x8 k8 = __builtin_bit_cast(bf16x8, kb[i]);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, lds_hi[at]), k8, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, lds_lo[at]), k8, acc, 0, 0, 0);
        dot2_bf16(nrm, kb[i].x, kb[i].x);
        dot2_bf16(nrm, kb[i].y, kb[i].y);
        dot2_bf16(nrm, kb[i].z, kb[i].z);
        dot2_bf16(nrm, kb[i].w, kb[i].w);
        kb[i] = *reinterpret_cast<const u32x4*>(refill + i * 16);
      }
    }
    nrm += lane_xor_f32<32>(nrm);                      // the other half of the key's channels
    const float kn = sqrtf(nrm);
    const int kk = tile * 32 + col;
    const bool live = kk < n_keys && nrm > 0.f;
    const int b = nb_begin + kk / n_rep;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      float c = (live && pn_w[i] > 0.f) ? acc[i] * inv_sqrt_g / (pn_w[i] * kn) : 0.f;
      if (n_rep >= 2) c += lane_xor_f32<1>(c);
      if (n_rep >= 4) c += lane_xor_f32<2>(c);
      if (kk % n_rep == 0 && b < end_w[i])
        scores[size_t(w0 + 4 * h + 8 * (i >> 2) + (i & 3)) * score_stride + b] = c / float(n_rep);
    }
    tile += stride;
    kp = kp_next;
  }
}

static int score_shared_lds_attribute(size_t bytes) {
  static std::mutex mu;
  static size_t set_for = 0;
  std::lock_guard<std::mutex> lock(mu);
  if (bytes <= set_for) return ACTQKV_OK;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(score_shared_mfma_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, int(bytes));
  if (e != hipSuccess) return set_error(ACTQKV_EHIP, "hipFuncSetAttribute: %s", hipGetErrorString(e));
  set_for = bytes;
  return ACTQKV_OK;
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
  // Several windows of one sequence (they share the keys): the matrix-core kernel, which reads the keys once.
  if (sh.dtype == ACTQKV_BF16 && batch >= 4 && seq_stride == 0 && key_len % (16 * kSsLoads) == 0 && key_len <= 1024 &&
      (sh.n_rep == 1 || sh.n_rep == 2 || sh.n_rep == 4)) {
    const size_t lds = size_t(key_len) * 128;          // 32 windows x key_len x (hi, lo) bf16
    if (int rc = score_shared_lds_attribute(lds)) return rc;
    const int n_tiles = (n * sh.n_rep + 31) / 32;
    dim3 grid(std::min((n_tiles + kSsWaves - 1) / kSsWaves, 64), (batch + 31) / 32), block(64 * kSsWaves);
    hipLaunchKernelGGL(score_shared_mfma_kernel, grid, block, lds, stream, probe_kv, probe_norm,
                       static_cast<const uint16_t*>(rep_keys), nb_capacity, nb_begin, nb_end, scores, score_stride,
                       batch, sh.n_rep, key_len, inv_sqrt_g);
    return hip_status("score_blocks");
  }
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
