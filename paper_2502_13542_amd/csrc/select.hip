// Information density, per-layer budget and block selection
// (Sec. 4.2, Eq. (11), Eq. (12); Alg. 1, second and third loop).
//
// One workgroup of 16 wavefronts per sequence.  The density is a two-pass softmax
// entropy over the eligible scores (or, as a variant, over the scores of the k_cap best
// blocks once the tournament has found them).  The E best blocks come from a tournament:
// every wavefront bitonic-sorts 64 (score, index) keys at a time across its lanes
// with shuffles and keeps a running sorted top-64; the 16 lists are then merged
// pairwise through LDS, each merge keeping the better 64.  Keys are 64-bit:
// order-preserving score bits above the inverted block index, so equal scores
// rank by ascending index and the result does not depend on timing.
#include "common.h"
#include "launch.h"

namespace actqkv {

constexpr int kSelectThreads = 1024;
constexpr int kSelectWaves = kSelectThreads / 64;

__device__ __forceinline__ unsigned long long select_key(float s, int block) {
  s += 0.f;  // -0 -> +0, so the two zeros tie
  uint32_t u = __float_as_uint(s);
  u ^= (u >> 31) ? 0xffffffffu : 0x80000000u;
  return (static_cast<unsigned long long>(u) << 32) | (0xffffffffu - uint32_t(block));
}
__device__ __forceinline__ unsigned long long shfl64(unsigned long long v, int src) {
  uint32_t lo = __shfl(uint32_t(v), src, 64), hi = __shfl(uint32_t(v >> 32), src, 64);
  return (static_cast<unsigned long long>(hi) << 32) | lo;
}
__device__ __forceinline__ unsigned long long umax64(unsigned long long a, unsigned long long b) {
  return a > b ? a : b;
}
__device__ __forceinline__ unsigned long long umin64(unsigned long long a, unsigned long long b) {
  return a < b ? a : b;
}
// A bitonic sequence across the 64 lanes -> sorted, lane 0 largest.
__device__ __forceinline__ unsigned long long bitonic_merge_desc(unsigned long long v, int lane) {
#pragma unroll
  for (int j = 32; j > 0; j >>= 1) {
    unsigned long long o = shfl64(v, lane ^ j);
    v = (lane & j) == 0 ? umax64(v, o) : umin64(v, o);
  }
  return v;
}
// Any 64 keys across the lanes -> sorted, lane 0 largest.
__device__ __forceinline__ unsigned long long bitonic_sort_desc(unsigned long long v, int lane) {
#pragma unroll
  for (int k = 2; k <= 64; k <<= 1) {
#pragma unroll
    for (int j = k >> 1; j > 0; j >>= 1) {
      unsigned long long o = shfl64(v, lane ^ j);
      bool keep_max = ((lane & k) == 0) == ((lane & j) == 0);
      v = keep_max ? umax64(v, o) : umin64(v, o);
    }
  }
  return v;
}

// Eq. (12), the budget update that follows it, and E^l (Alg. 1); called by one thread.
__device__ __forceinline__ int cutoff_count(float theta, int s, int n, int k_cap,
                                            float* __restrict__ budget_remaining,
                                            const float* __restrict__ theta_rest_sum,
                                            int32_t* __restrict__ n_sel, float* __restrict__ theta_out,
                                            float* __restrict__ budget_out) {
  float b_l;
  int e;
  if (budget_remaining != nullptr) {
    float b_kv = budget_remaining[s], rest = theta_rest_sum[s];
    float den = theta + rest;
    b_l = den > 0.f ? theta / den * b_kv : b_kv;
    float r = fminf(fmaxf(floorf(b_l + 0.5f), 1.f), float(k_cap));
    e = min(int(r), n);
    budget_remaining[s] = b_kv - b_l;
  } else {
    e = min(k_cap, n);
    b_l = float(e);
  }
  n_sel[s] = e;
  if (theta_out) theta_out[s] = theta;
  if (budget_out) budget_out[s] = b_l;
  return e;
}

// the score a tournament key was made from
__device__ __forceinline__ float key_score(unsigned long long key) {
  uint32_t u = uint32_t(key >> 32);
  u ^= (u >> 31) ? 0x80000000u : 0xffffffffu;
  return __uint_as_float(u);
}

__global__ __launch_bounds__(kSelectThreads) void select_kernel(
    const float* __restrict__ scores, int64_t score_stride, int nb_capacity, int nb_begin,
    const int32_t* __restrict__ nb_end, int k_cap, int entropy_topk, float* __restrict__ budget_remaining,
    const float* __restrict__ theta_rest_sum, int32_t* __restrict__ idx, int32_t* __restrict__ n_sel, float* __restrict__ theta_out,
    float* __restrict__ budget_out) {
  __shared__ float red[32];
  __shared__ unsigned long long lists[kSelectWaves][64];
  __shared__ int e_shared;
  const int s = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* sc_mem = scores + size_t(s) * score_stride + nb_begin;
  // The scores of the first 1024 blocks stay in registers for all three passes; their load does
  // not wait for nb_end (the row has nb_capacity entries whatever nb_end says).
  const float sc_first = tid < nb_capacity - nb_begin ? sc_mem[tid] : 0.f;
  int end = min(nb_end[s], nb_capacity);
  const int n = max(end - nb_begin, 0);
  struct {
    const float* mem;
    float first;
    __device__ __forceinline__ float operator[](int i) const { return i < kSelectThreads ? first : mem[i]; }
  } sc{sc_mem, sc_first};                        // indexed with i = tid + c * 1024 only
  int32_t* my_idx = idx + size_t(s) * k_cap;
  if (n == 0) {
    if (tid < k_cap) my_idx[tid] = -1;
    if (tid == 0) {
      n_sel[s] = 0;
      if (theta_out) theta_out[s] = 0.f;
      if (budget_out) budget_out[s] = 0.f;
    }
    return;
  }
  if (!entropy_topk) {
    // Eq. (11): theta = -sum P ln P with P = softmax(s) = ln Z + max - sum P s
    float mx = -INFINITY;
    for (int i = tid; i < n; i += kSelectThreads) mx = fmaxf(mx, sc[i]);
    mx = block_max(mx, red);
    float z = 0.f, t = 0.f;
    for (int i = tid; i < n; i += kSelectThreads) {
      float v = sc[i], e = __expf(v - mx);
      z += e;
      t += e * v;
    }
    z = block_sum(z, red);
    t = block_sum(t, red);
    if (tid == 0)
      e_shared = cutoff_count(fmaxf(logf(z) + mx - t / z, 0.f), s, n, k_cap, budget_remaining, theta_rest_sum,
                              n_sel, theta_out, budget_out);
  }
  // Alg. 1, third loop: the best blocks, best first
  unsigned long long run = 0ull;
  for (int c = 0; c * kSelectThreads < n; ++c) {
    int i = c * kSelectThreads + wave * 64 + lane;
    unsigned long long key = i < n ? select_key(sc[i], nb_begin + i) : 0ull;
    key = bitonic_sort_desc(key, lane);
    if (c == 0) {
      run = key;
    } else {
      run = umax64(run, shfl64(key, 63 - lane));
      run = bitonic_merge_desc(run, lane);
    }
  }
  lists[wave][lane] = run;
  for (int stride = kSelectWaves / 2; stride > 0; stride >>= 1) {
    __syncthreads();
    if (wave < stride) {
      run = umax64(run, lists[wave + stride][63 - lane]);
      run = bitonic_merge_desc(run, lane);
      lists[wave][lane] = run;
    }
  }
  if (entropy_topk && wave == 0) {
    // the same entropy over the scores of the min(k_cap, n) best blocks, which sit in lanes
    // 0 .. of wavefront 0, best first (lane 0 holds the maximum)
    const bool in = lane < min(k_cap, n);
    const float v = in ? key_score(run) : 0.f;
    const float mx = __shfl(v, 0, 64);
    const float e = in ? __expf(v - mx) : 0.f;
    float z = e, t = e * v;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      z += __shfl_xor(z, o, 64);
      t += __shfl_xor(t, o, 64);
    }
    if (lane == 0)
      e_shared = cutoff_count(fmaxf(logf(z) + mx - t / z, 0.f), s, n, k_cap, budget_remaining, theta_rest_sum,
                              n_sel, theta_out, budget_out);
  }
  __syncthreads();
  if (wave == 0 && lane < k_cap) {
    int e = e_shared;
    my_idx[lane] = lane < e ? int(0xffffffffu - uint32_t(run)) : -1;
  }
}

int launch_select(int batch, const float* scores, int64_t score_stride, int nb_capacity, int nb_begin,
                  const int32_t* nb_end, int k_cap, int flags, float* budget_remaining,
                  const float* theta_rest_sum, int32_t* idx, int32_t* n_sel, float* theta,
                  float* budget, hipStream_t stream) {
  hipLaunchKernelGGL(select_kernel, dim3(batch), dim3(kSelectThreads), 0, stream, scores,
                     score_stride, nb_capacity, nb_begin, nb_end, k_cap,
                     (flags & ACTQKV_SELECT_ENTROPY_TOPK) != 0, budget_remaining, theta_rest_sum, idx,
                     n_sel, theta, budget);
  return hip_status("select");
}

}  // namespace actqkv
