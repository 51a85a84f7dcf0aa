// The cache update of one (role, block segment, sequence) as a device function (Sec. 3.1,
// Eq. (4)); shared by the append kernel and by the first launch of a decode step's retrieval.
#pragma once

#include "common.h"

namespace actqkv {

constexpr int kApThreads = 1024;

// Called by all kThreads (a multiple of 128) threads of a workgroup.  Roles 0 .. Hk-1 copy the new tokens of one KV
// head that fall into cache block pos0/128 + seg: K rows as they are, V through an LDS tile so
// that it lands transposed ([D][128]).  Role Hk picks the representatives (the r tokens whose
// key, taken over all KV heads together, has the largest L2 norm; ties: lower position; kept
// in position order) if the block is full after this call and was not before; it reads tokens
// older than pos0 from the cache and the others from the new keys, so it does not depend on
// the copies of the same launch.  ap_lds: max(head_dim * 130 elements, 256 floats) of LDS.
template <typename T, int kThreads = kApThreads>
__device__ __forceinline__ void append_body(int role, int seg, int s, const T* __restrict__ k_new,
                                            const T* __restrict__ v_new,
                                            int pos0_of_s, T* __restrict__ k_cache,
                                            T* __restrict__ v_cache, int64_t cache_stride,
                                            T* __restrict__ rep_keys, int64_t rep_stride, int nb_capacity,
                                            int m, int n_kv_heads, int head_dim, int n_rep,
                                            unsigned char* ap_lds) {
  constexpr int V = Vec<T>::N;
  const int pos0 = max(pos0_of_s, 0);            // tokens already in sequence s's cache
  const int block = pos0 / kBlock + seg;
  if (block >= nb_capacity) return;
  const int lo = max(pos0, block * kBlock), hi = min(pos0 + m, block * kBlock + kBlock);
  if (hi <= lo) return;
  const int row_len = n_kv_heads * head_dim;                       // elements of one token's keys
  const T* kn = k_new + size_t(s) * m * row_len;
  const T* vn = v_new + size_t(s) * m * row_len;

  if (role < n_kv_heads) {
    // ---- copy the tokens [lo, hi) of KV head `role` into block `block`
    const int hk = role, n_tok = hi - lo, j0 = lo - block * kBlock;
    const size_t tile = (size_t(block) * n_kv_heads + hk) * kBlock * head_dim;
    T* kd = k_cache + size_t(s) * cache_stride + tile + size_t(j0) * head_dim;
    T* vd = v_cache + size_t(s) * cache_stride + tile;
    T* vt = reinterpret_cast<T*>(ap_lds);                           // [head_dim][kBlock + 2]
    constexpr int kPad = kBlock + 2;
    const int chunks = head_dim / V;
    for (int i = threadIdx.x; i < n_tok * chunks; i += kThreads) {
      const int tk = i / chunks, c = i - tk * chunks;
      const size_t src = size_t(lo - pos0 + tk) * row_len + size_t(hk) * head_dim + c * V;
      const typename Vec<T>::raw kraw = Vec<T>::load_raw(kn + src);
      const typename Vec<T>::raw vraw = Vec<T>::load_raw(vn + src);
      *reinterpret_cast<typename Vec<T>::raw*>(kd + size_t(tk) * head_dim + c * V) = kraw;
      alignas(16) T ve[V];
      *reinterpret_cast<typename Vec<T>::raw*>(ve) = vraw;
#pragma unroll
      for (int e = 0; e < V; ++e) vt[(c * V + e) * kPad + tk] = ve[e];
    }
    __syncthreads();
    for (int i = threadIdx.x; i < head_dim * n_tok; i += kThreads) {
      const int d = i / n_tok, tk = i - d * n_tok;
      vd[size_t(d) * kBlock + j0 + tk] = vt[d * kPad + tk];
    }
    return;
  }

  // ---- representatives of the block, if these tokens complete it
  if (hi != block * kBlock + kBlock || rep_keys == nullptr) return;
  float* norm = reinterpret_cast<float*>(ap_lds);                  // [kBlock]
  int* chosen = reinterpret_cast<int*>(ap_lds) + kBlock;           // [kBlock]: output slot or -1
  const T* kb = k_cache + size_t(s) * cache_stride + size_t(block) * n_kv_heads * kBlock * head_dim;
  auto token_chunk = [&](int tk, int c) -> const T* {   // chunk c (V elements) of the token's [Hk][D] keys
    const int pos = block * kBlock + tk;
    if (pos >= pos0) return kn + size_t(pos - pos0) * row_len + size_t(c) * V;
    const int hk = (c * V) / head_dim, d = c * V - hk * head_dim;
    return kb + (size_t(hk) * kBlock + tk) * head_dim + d;
  };
  const int chunks = row_len / V;
  {
    // 8 neighbouring lanes share a token; lane part p takes chunks p, p + 8, ...
    const int part = threadIdx.x & 7;
    for (int tk = threadIdx.x >> 3; tk < kBlock; tk += kThreads >> 3) {
      float acc = 0.f;
      for (int c0 = part; c0 < chunks; c0 += 8 * 8) {
        float x[8][V];
#pragma unroll
        for (int i = 0; i < 8; ++i) {                                // all loads first: they overlap
          const int c = c0 + 8 * i;
          Vec<T>::load(token_chunk(tk, c < chunks ? c : part), x[i]);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
          if (c0 + 8 * i < chunks) {
#pragma unroll
            for (int e = 0; e < V; ++e) acc += x[i][e] * x[i][e];
          }
      }
      acc += __shfl_xor(acc, 1, 64);
      acc += __shfl_xor(acc, 2, 64);
      acc += __shfl_xor(acc, 4, 64);
      if (part == 0) norm[tk] = acc;
    }
  }
  __syncthreads();
  if (threadIdx.x < kBlock) {
    const int i = threadIdx.x;
    const float mine = norm[i];
    int rank = 0;
    for (int j = 0; j < kBlock; ++j) {
      const float o = norm[j];
      rank += (o > mine) || (o == mine && j < i);
    }
    chosen[i] = rank < n_rep ? 1 : 0;
  }
  __syncthreads();
  int slot_of_mine = -1;
  if (threadIdx.x < kBlock) {
    const int i = threadIdx.x;
    int before = 0;
    for (int j = 0; j < i; ++j) before += chosen[j];
    slot_of_mine = chosen[i] ? before : -1;
  }
  __syncthreads();
  if (threadIdx.x < kBlock) chosen[threadIdx.x] = slot_of_mine;
  __syncthreads();
  T* rd = rep_keys + size_t(s) * rep_stride + size_t(block) * n_rep * row_len;
  for (int i = threadIdx.x; i < kBlock * chunks; i += kThreads) {
    const int tk = i / chunks, c = i - tk * chunks;
    const int slot = chosen[tk];
    if (slot >= 0)
      *reinterpret_cast<typename Vec<T>::raw*>(rd + size_t(slot) * row_len + size_t(c) * V) =
          Vec<T>::load_raw(token_chunk(tk, c));
  }
}

}  // namespace actqkv
