// The probe of a window of one token (decode): Eq. (9) has a single weight, 1, so the probe is
// the query (Sec. 4.2).  Shared by the probe kernel for m == 1 and by the fused first launch of
// a decode step (cache update + probe).
#pragma once

#include "common.h"

namespace actqkv {

// One workgroup of 1024 threads per sequence; a thread owns up to 4 groups of 4 channels.
// probe_lds: [d] floats of LDS, red: [32] floats of LDS.
template <typename T>
__device__ __forceinline__ void probe_identity_body(const T* __restrict__ q, float* __restrict__ probe,
                                                    float* __restrict__ probe_kv,
                                                    float* __restrict__ probe_norm_out,
                                                    float* __restrict__ weight_out, int n_q_heads,
                                                    int n_kv_heads, int head_dim, float* probe_lds,
                                                    float* red) {
  const int d = n_q_heads * head_dim, g = n_q_heads / n_kv_heads;
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
    *probe_norm_out = sqrtf(ss);
    if (weight_out != nullptr) *weight_out = 1.f;
  }
  for (int e = threadIdx.x; e < n_kv_heads * head_dim; e += 1024) {
    const int hk = e / head_dim, dd = e - hk * head_dim;
    float t = 0.f;
    for (int i = 0; i < g; ++i) t += probe_lds[(hk * g + i) * head_dim + dd];
    probe_kv[e] = t;
  }
}

}  // namespace actqkv
