// Everything of a decode step that comes before the attention, in two launches instead of
// four: the cache update (Sec. 3.1, Eq. (4)), the probe of the step's one-token window (the
// query itself, Sec. 4.2) and the block scores (Eq. (10)) in the first, the selection with the
// cut-off (Eq. (11), Eq. (12), Alg. 1) in the second.  The update and the probe are a few
// microseconds of work each; as launches of their own they cost more in launch and drain time.
//
// First launch: grid (scoring workgroups + 2, batch), 256 threads.  A scoring workgroup forms
// the group-summed probe and the probe's norm for itself (8 KB of query, from L2, while its
// first key loads are in flight) and scores 4 blocks, one per wavefront.  The two other
// workgroups of a sequence write the new token into the cache and, if the token completes a
// block, pick the block's representatives; they share nothing with the scoring: the block that
// receives the token lies in the local span and is never eligible.
//
// Selecting in the same launch (the workgroup of a sequence that finishes last, found by a
// ticket, goes on to select) was measured and is slower: the write-through of the scores, the
// ticket and the read-back cost as much as the launch they replace.
#include <algorithm>

#include "append_body.h"
#include "common.h"
#include "launch.h"
#include "score_body.h"

namespace actqkv {

constexpr int kDrThreads = 256;
constexpr int kDrWaves = kDrThreads / 64;   // blocks per scoring workgroup

template <typename T>
struct DrParams {
  const T* q_tok;
  const T* k_new;           // NULL: no cache update
  const T* v_new;
  const int32_t* pos0;
  T* k_cache;
  T* v_cache;
  int64_t cache_stride;
  T* rep_keys;
  int64_t rep_stride;
  int nb_capacity, nb_begin;
  const int32_t* nb_end;
  float* probe;             // optional outputs of the probe step
  float* probe_kv;
  float* probe_norm;
  float* scores;
  int64_t score_stride;
  int n_score_wg;
  int n_q_heads, n_kv_heads, head_dim, n_rep;
  float inv_sqrt_g;
};

template <typename T>
__global__ __launch_bounds__(kDrThreads) void decode_score_kernel(DrParams<T> p) {
  constexpr int V = Vec<T>::N;
  extern __shared__ __attribute__((aligned(16))) unsigned char dr_lds[];
  __shared__ float red[32];
  const int s = blockIdx.y;
  const int key_len = p.n_kv_heads * p.head_dim;
  const int role = int(blockIdx.x) - p.n_score_wg;
  if (role == 0) {
    // ---- the new token's keys and values into the cache: K rows as they are, V transposed
    const int pos = max(p.pos0[s], 0), block = pos / kBlock, j0 = pos - block * kBlock;
    if (block >= p.nb_capacity) return;
    const T* kn = p.k_new + size_t(s) * key_len;
    const T* vn = p.v_new + size_t(s) * key_len;
    for (int e = threadIdx.x; e < key_len; e += kDrThreads) {
      const int hk = e / p.head_dim, dd = e - hk * p.head_dim;
      const size_t tile = size_t(s) * p.cache_stride + (size_t(block) * p.n_kv_heads + hk) * kBlock * p.head_dim;
      p.k_cache[tile + size_t(j0) * p.head_dim + dd] = kn[e];
      p.v_cache[tile + size_t(dd) * kBlock + j0] = vn[e];
    }
    return;
  }
  if (role == 1) {
    // ---- the representatives of the block, if the token completes it
    append_body<T, kDrThreads>(p.n_kv_heads, 0, s, p.k_new, p.v_new, p.pos0[s], p.k_cache, p.v_cache,
                               p.cache_stride, p.rep_keys, p.rep_stride, p.nb_capacity, 1, p.n_kv_heads,
                               p.head_dim, p.n_rep, dr_lds);
    return;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float* pkv_lds = reinterpret_cast<float*>(dr_lds);     // [key_len]
  const int end = min(p.nb_end[s], p.nb_capacity);
  const int b0 = p.nb_begin + int(blockIdx.x) * kDrWaves, b = b0 + wave;
  const bool first = blockIdx.x == 0, live = b < end;
  // a workgroup whose blocks all lie behind the sequence's last eligible one (the grid is sized by
  // the capacity) has nothing to do; the first one still writes the probe
  if (!first && b0 >= end) return;
  // The probe is the query: summed over the G query heads of a KV head, and its norm.  A thread's
  // first query loads go out BEFORE its key loads: outstanding loads are counted in order, so
  // waiting for a load issued behind the keys would wait for the keys too.
  const int group = p.n_q_heads / p.n_kv_heads, n_chunks = key_len / V;
  const T* __restrict__ q = p.q_tok + size_t(s) * p.n_q_heads * p.head_dim;
  auto load_q = [&](int c, int g0, float (&x)[4][V]) {    // chunk c of heads g0 .. g0 + 3 of its KV head
    const int hk = (c * V) / p.head_dim, dd = c * V - hk * p.head_dim;
#pragma unroll
    for (int i = 0; i < 4; ++i)                            // all loads first: they overlap
      Vec<T>::load(q + (hk * group + min(g0 + i, group - 1)) * p.head_dim + dd, x[i]);
  };
  float ss = 0.f;
  auto add_q = [&](int g0, const float (&x)[4][V], float (&acc)[V]) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (g0 + i < group) {
#pragma unroll
        for (int v = 0; v < V; ++v) {
          acc[v] += x[i][v];
          ss += x[i][v] * x[i][v];
        }
      }
  };
  // heads g_from .. of chunk c, then the chunk's sum to LDS
  auto finish_chunk = [&](int c, int g_from, float (&acc)[V]) {
    for (int g0 = g_from; g0 < group; g0 += 4) {
      float x[4][V];
      load_q(c, g0, x);
      add_q(g0, x, acc);
    }
#pragma unroll
    for (int v = 0; v < V; ++v) pkv_lds[c * V + v] = acc[v];
  };
  float x0[4][V];
  load_q(min(int(threadIdx.x), n_chunks - 1), 0, x0);
  __builtin_amdgcn_sched_barrier(0);
  // the first batch of key loads is in flight while the probe is formed
  BlockScorer<T> scorer;
  scorer.start(p.rep_keys + size_t(s) * p.rep_stride +
                   size_t(live ? b : min(p.nb_begin, p.nb_capacity - 1)) * p.n_rep * key_len,
               p.n_rep, key_len, lane);
  __builtin_amdgcn_sched_barrier(0);
  if (int(threadIdx.x) < n_chunks) {
    float acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = 0.f;
    add_q(0, x0, acc);
    finish_chunk(threadIdx.x, 4, acc);
  }
  for (int c = threadIdx.x + kDrThreads; c < n_chunks; c += kDrThreads) {
    float acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = 0.f;
    finish_chunk(c, 0, acc);
  }
  const float pn = sqrtf(block_sum(ss, red));            // its barriers also publish pkv_lds
  if (first) {
    if (p.probe != nullptr)
      for (int e = threadIdx.x; e < p.n_q_heads * p.head_dim; e += kDrThreads)
        p.probe[size_t(s) * p.n_q_heads * p.head_dim + e] = to_f32(q[e]);
    if (p.probe_kv != nullptr)
      for (int e = threadIdx.x; e < key_len; e += kDrThreads) p.probe_kv[size_t(s) * key_len + e] = pkv_lds[e];
    if (p.probe_norm != nullptr && threadIdx.x == 0) p.probe_norm[s] = pn;
  }
  if (!live) return;
  const float total = scorer.finish(pkv_lds, pn, p.inv_sqrt_g);
  if (lane == 0) p.scores[size_t(s) * p.score_stride + b] = total;
}

template <typename T>
static int launch_decode_score_t(const actqkv_shape& sh, int batch, DrParams<T> p, hipStream_t stream) {
  const int n = std::max(p.nb_capacity - p.nb_begin, 0);
  p.n_score_wg = std::max((n + kDrWaves - 1) / kDrWaves, 1);   // at least one: it writes the probe
  p.n_q_heads = sh.n_q_heads;
  p.n_kv_heads = sh.n_kv_heads;
  p.head_dim = sh.head_dim;
  p.n_rep = sh.n_rep;
  p.inv_sqrt_g = 1.f / sqrtf(float(sh.n_q_heads / sh.n_kv_heads));
  const int roles = p.k_new != nullptr ? 2 : 0;
  const size_t lds = std::max(size_t(sh.n_kv_heads) * sh.head_dim * sizeof(float), size_t(2 * kBlock) * 4);
  hipLaunchKernelGGL(decode_score_kernel<T>, dim3(p.n_score_wg + roles, batch), dim3(kDrThreads), lds, stream,
                     p);
  return hip_status("decode_retrieve (scores)");
}

int launch_decode_retrieve(const actqkv_shape& sh, int batch, const void* q_tok, const void* k_new,
                           const void* v_new, const int32_t* pos0, void* k_cache, void* v_cache,
                           int64_t cache_stride, void* rep_keys, int64_t rep_stride, int nb_capacity,
                           int nb_begin, const int32_t* nb_end, float* probe, float* probe_kv,
                           float* probe_norm, float* scores, int64_t score_stride, int k_cap, int flags,
                           float* budget_remaining, const float* theta_rest_sum, int32_t* idx,
                           int32_t* n_sel, float* theta, float* budget, hipStream_t stream) {
  auto fill = [&](auto& p) {
    p.pos0 = pos0;
    p.cache_stride = cache_stride;
    p.rep_stride = rep_stride;
    p.nb_capacity = nb_capacity;
    p.nb_begin = nb_begin;
    p.nb_end = nb_end;
    p.probe = probe;
    p.probe_kv = probe_kv;
    p.probe_norm = probe_norm;
    p.scores = scores;
    p.score_stride = score_stride;
  };
  int rc;
  if (sh.dtype == ACTQKV_F32) {
    DrParams<float> p;
    p.q_tok = static_cast<const float*>(q_tok);
    p.k_new = static_cast<const float*>(k_new);
    p.v_new = static_cast<const float*>(v_new);
    p.k_cache = static_cast<float*>(k_cache);
    p.v_cache = static_cast<float*>(v_cache);
    p.rep_keys = static_cast<float*>(rep_keys);
    fill(p);
    rc = launch_decode_score_t(sh, batch, p, stream);
  } else {
    DrParams<uint16_t> p;
    p.q_tok = static_cast<const uint16_t*>(q_tok);
    p.k_new = static_cast<const uint16_t*>(k_new);
    p.v_new = static_cast<const uint16_t*>(v_new);
    p.k_cache = static_cast<uint16_t*>(k_cache);
    p.v_cache = static_cast<uint16_t*>(v_cache);
    p.rep_keys = static_cast<uint16_t*>(rep_keys);
    fill(p);
    rc = launch_decode_score_t(sh, batch, p, stream);
  }
  if (rc != ACTQKV_OK || (flags & ACTQKV_DECODE_SCORES_ONLY)) return rc;
  return launch_select(batch, scores, score_stride, nb_capacity, nb_begin, nb_end, k_cap, flags,
                       budget_remaining, theta_rest_sum, idx, n_sel, theta, budget, stream);
}

}  // namespace actqkv
