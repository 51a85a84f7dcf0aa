// The score of one block by one wavefront (Sec. 4.2, Eq. (10), applied to the r representative
// keys of a block): shared by the scoring kernel and by the first launch of a decode step's retrieval.
#pragma once

#include "common.h"

namespace actqkv {

constexpr int kScoreBatch = 8;  // 16-byte loads a lane keeps in flight

// Each group of 16 lanes walks one representative key (consecutive lanes read consecutive
// 16-byte chunks), so a wavefront keeps four keys in flight.  start() requests the first batch
// of loads (nothing else is needed for it, so the caller can form the probe meanwhile);
// finish() wants the group-summed probe [key_len] in LDS and its norm.
template <typename T>
struct BlockScorer {
  static constexpr int V = Vec<T>::N;
  const T* block_keys;
  int n_rep, key_len, chunks, gq, l16;
  typedef typename Vec<T>::raw raw_t;
  raw_t k0[kScoreBatch];          // as loaded (16 bytes each): widened only where they are used

  // kScoreBatch chunks of key j, starting at chunk c0: all loads are issued before any is used
  __device__ __forceinline__ void load_batch(int j, int c0, raw_t (&k)[kScoreBatch]) const {
    const T* key = block_keys + size_t(j < n_rep ? j : 0) * key_len;
#pragma unroll
    for (int i = 0; i < kScoreBatch; ++i) {
      const int c = c0 + 16 * i;
      k[i] = Vec<T>::load_raw(key + (c < chunks ? c : l16) * V);
    }
  }
  __device__ __forceinline__ void accumulate(const float* probe_lds, int j, int c0,
                                             const raw_t (&k)[kScoreBatch], float& dot, float& nrm) const {
#pragma unroll
    for (int i = 0; i < kScoreBatch; ++i) {
      const int c = c0 + 16 * i;
      if (c < chunks && j < n_rep) {
        float f[V];
        Vec<T>::widen(k[i], f);
#pragma unroll
        for (int v = 0; v < V; ++v) {
          dot += probe_lds[c * V + v] * f[v];
          nrm += f[v] * f[v];
        }
      }
    }
  }
  // cosine of the probe with key j repeated to the G query heads, summed over the 4 lane groups
  __device__ __forceinline__ float finish_keys(int j, float dot, float nrm, float pn, float inv_sqrt_g) const {
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) {
      dot += __shfl_xor(dot, o, 64);
      nrm += __shfl_xor(nrm, o, 64);
    }
    float c = (j < n_rep && nrm > 0.f && pn > 0.f) ? dot * inv_sqrt_g / (pn * sqrtf(nrm)) : 0.f;
    c += __shfl_xor(c, 16, 64);
    c += __shfl_xor(c, 32, 64);
    return c;
  }

  // block_keys: the block's [n_rep][key_len] representative keys (any valid block for an idle wavefront)
  __device__ __forceinline__ void start(const T* keys, int n_rep_, int key_len_, int lane) {
    block_keys = keys;
    n_rep = n_rep_;
    key_len = key_len_;
    chunks = key_len_ / V;
    gq = lane >> 4;
    l16 = lane & 15;
    load_batch(gq, l16, k0);
  }
  // the block's score, in every lane
  __device__ __forceinline__ float finish(const float* probe_lds, float pn, float inv_sqrt_g) {
    float total = 0.f;
    {
      float dot = 0.f, nrm = 0.f;
      accumulate(probe_lds, gq, l16, k0, dot, nrm);
      for (int c0 = l16 + 16 * kScoreBatch; c0 < chunks; c0 += 16 * kScoreBatch) {
        raw_t kk[kScoreBatch];
        load_batch(gq, c0, kk);
        accumulate(probe_lds, gq, c0, kk, dot, nrm);
      }
      total += finish_keys(gq, dot, nrm, pn, inv_sqrt_g);
    }
    for (int j0 = 4; j0 < n_rep; j0 += 4) {
      const int j = j0 + gq;
      float dot = 0.f, nrm = 0.f;
      for (int c0 = l16; c0 < chunks; c0 += 16 * kScoreBatch) {
        raw_t kk[kScoreBatch];
        load_batch(j, c0, kk);
        accumulate(probe_lds, j, c0, kk, dot, nrm);
      }
      total += finish_keys(j, dot, nrm, pn, inv_sqrt_g);
    }
    return total / float(n_rep);
  }
};

}  // namespace actqkv
