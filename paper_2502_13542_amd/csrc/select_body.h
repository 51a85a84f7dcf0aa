// The selection step as a device function: information density, per-layer budget and the
// tournament for the best blocks (Sec. 4.2, Eq. (11), Eq. (12); Alg. 1, second and third loop).
// Shared by the selection kernel (one workgroup of 1024 threads per sequence) and by the decode
// attention that selects for itself (every workgroup of 512 threads repeats its sequence's
// selection while its first keys and values are on their way).
//
// The density is a two-pass softmax entropy over the eligible scores (or, as a variant, over the
// scores of the k_cap best blocks once the tournament has found them).  The E best blocks come
// from a tournament: every wavefront bitonic-sorts 64 (score, index) keys at a time across its
// lanes with shuffles and keeps a running sorted top-64; the lists are then merged pairwise
// through LDS, each merge keeping the better 64.  Keys are 64-bit: order-preserving score bits
// above the inverted block index, so equal scores rank by ascending index and the result does
// not depend on timing.
#pragma once

#include "common.h"

namespace actqkv {

__device__ __forceinline__ unsigned long long select_key(float s, int block) {
  s += 0.f;  // -0 -> +0, so the two zeros tie
  uint32_t u = __float_as_uint(s);
  u ^= (u >> 31) ? 0xffffffffu : 0x80000000u;
  return (static_cast<unsigned long long>(u) << 32) | (0xffffffffu - uint32_t(block));
}
// the score a tournament key was made from
__device__ __forceinline__ float key_score(unsigned long long key) {
  uint32_t u = uint32_t(key >> 32);
  u ^= (u >> 31) ? 0x80000000u : 0xffffffffu;
  return __uint_as_float(u);
}
__device__ __forceinline__ unsigned long long shfl64(unsigned long long v, int src) {
  uint32_t lo = __shfl(uint32_t(v), src, 64), hi = __shfl(uint32_t(v >> 32), src, 64);
  return (static_cast<unsigned long long>(hi) << 32) | lo;
}
template <int J>
__device__ __forceinline__ unsigned long long lane_xor64(unsigned long long v) {
  const uint32_t lo = lane_xor32<J>(uint32_t(v)), hi = lane_xor32<J>(uint32_t(v >> 32));
  return (static_cast<unsigned long long>(hi) << 32) | lo;
}
__device__ __forceinline__ unsigned long long umax64(unsigned long long a, unsigned long long b) {
  return a > b ? a : b;
}
__device__ __forceinline__ unsigned long long umin64(unsigned long long a, unsigned long long b) {
  return a < b ? a : b;
}
// one compare-exchange step of a bitonic network at lane distance J; keep_max per lane
template <int J>
__device__ __forceinline__ unsigned long long bitonic_step(unsigned long long v, bool keep_max) {
  const unsigned long long o = lane_xor64<J>(v);
  return keep_max ? umax64(v, o) : umin64(v, o);
}
// A bitonic sequence across the 64 lanes -> sorted, lane 0 largest.
__device__ __forceinline__ unsigned long long bitonic_merge_desc(unsigned long long v, int lane) {
  v = bitonic_step<32>(v, (lane & 32) == 0);
  v = bitonic_step<16>(v, (lane & 16) == 0);
  v = bitonic_step<8>(v, (lane & 8) == 0);
  v = bitonic_step<4>(v, (lane & 4) == 0);
  v = bitonic_step<2>(v, (lane & 2) == 0);
  v = bitonic_step<1>(v, (lane & 1) == 0);
  return v;
}
// Any 64 keys across the lanes -> sorted, lane 0 largest.  Stage k sorts runs of k lanes,
// alternating in direction ((lane & k) == 0: descending), by steps at distances k/2 .. 1.
template <int K, int J>
__device__ __forceinline__ unsigned long long bitonic_stage(unsigned long long v, int lane) {
  v = bitonic_step<J>(v, ((lane & K) == 0) == ((lane & J) == 0));
  if constexpr (J > 1) v = bitonic_stage<K, J / 2>(v, lane);
  return v;
}
__device__ __forceinline__ unsigned long long bitonic_sort_desc(unsigned long long v, int lane) {
  v = bitonic_stage<2, 1>(v, lane);
  v = bitonic_stage<4, 2>(v, lane);
  v = bitonic_stage<8, 4>(v, lane);
  v = bitonic_stage<16, 8>(v, lane);
  v = bitonic_stage<32, 16>(v, lane);
  v = bitonic_stage<64, 32>(v, lane);      // (lane & 64) == 0 for every lane: descending
  return v;
}

// Cut-off state in, results out (global memory; the arrays have an entry per sequence).
struct SelectIo {
  const float* budget_in;        // B_kv before this layer, or NULL: no cut-off, the k_cap best
  const float* theta_rest_sum;   // R of this layer (with budget_in)
  float* budget_after;           // B_kv - B^l; may be the array budget_in points to
  int32_t* idx;                  // [k_cap] per sequence
  int32_t* n_sel;
  float* theta;                  // optional
  float* budget;                 // optional: B^l
  bool write;                    // false: nothing is stored (the caller reads the result from LDS)
  // The two halves of Alg. 1 as it is printed (every density first, then every budget, then the
  // selections): density_only stops after Eq. (11) and stores theta alone; count_in (per sequence,
  // device memory) is an E^l that was computed elsewhere and replaces Eq. (12) in this call.
  bool density_only = false;
  const int32_t* count_in = nullptr;
};

// Eq. (12), the budget update that follows it, and E^l (Alg. 1); called by one thread.
__device__ __forceinline__ int cutoff_count(float theta, int s, int n, int k_cap, const SelectIo& io) {
  float b_l;
  int e;
  if (io.density_only) {
    if (io.write && io.theta) io.theta[s] = theta;
    return 0;
  }
  if (io.count_in != nullptr) {
    e = min(max(io.count_in[s], 0), min(k_cap, n));
    b_l = float(e);
  } else if (io.budget_in != nullptr) {
    float b_kv = io.budget_in[s], rest = io.theta_rest_sum[s];
    float den = theta + rest;
    b_l = den > 0.f ? theta / den * b_kv : b_kv;
    float r = fminf(fmaxf(floorf(b_l + 0.5f), 1.f), float(k_cap));
    e = min(int(r), n);
    if (io.write && io.budget_after != nullptr) io.budget_after[s] = b_kv - b_l;
  } else {
    e = min(k_cap, n);
    b_l = float(e);
  }
  if (io.write) {
    io.n_sel[s] = e;
    if (io.theta) io.theta[s] = theta;
    if (io.budget) io.budget[s] = b_l;
  }
  return e;
}

// LDS of one selecting workgroup; after select_body, count and sel[0 .. k_cap) hold the result.
template <int kThreads>
struct SelectLds {
  float red[32];
  unsigned long long lists[kThreads / 64][64];
  int count;
  int sel[64];
};

// Called by all kThreads threads of a workgroup for sequence (row) s; n >= 0 eligible blocks
// starting at nb_begin; sc[i] is the score of block nb_begin + i and is only ever indexed with
// i = threadIdx.x + c * kThreads.  Ends with a barrier.
template <int kThreads, typename Scores>
__device__ __forceinline__ void select_body(const Scores& sc, int s, int n, int nb_begin, int k_cap,
                                            int entropy_topk, const SelectIo& io, SelectLds<kThreads>& lds) {
  constexpr int kWaves = kThreads / 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int32_t* my_idx = io.idx + size_t(s) * k_cap;
  if (n == 0) {
    if (io.density_only) {
      if (tid == 0 && io.write && io.theta) io.theta[s] = 0.f;
      __syncthreads();
      return;
    }
    if (tid < k_cap) {
      lds.sel[tid] = -1;
      if (io.write) my_idx[tid] = -1;
    }
    if (tid == 0) {
      lds.count = 0;
      if (io.write) {
        io.n_sel[s] = 0;
        if (io.theta) io.theta[s] = 0.f;
        if (io.budget) io.budget[s] = 0.f;
        if (io.budget_in != nullptr && io.budget_after != nullptr) io.budget_after[s] = io.budget_in[s];
      }
    }
    __syncthreads();
    return;
  }
  if (!entropy_topk) {
    // Eq. (11): theta = -sum P ln P with P = softmax(s) = ln Z + max - sum P s
    float mx = -INFINITY;
    for (int i = tid; i < n; i += kThreads) mx = fmaxf(mx, sc[i]);
    mx = block_max(mx, lds.red);
    float z = 0.f, t = 0.f;
    for (int i = tid; i < n; i += kThreads) {
      float v = sc[i], e = __expf(v - mx);
      z += e;
      t += e * v;
    }
    z = block_sum(z, lds.red);
    t = block_sum(t, lds.red);
    if (tid == 0) lds.count = cutoff_count(fmaxf(logf(z) + mx - t / z, 0.f), s, n, k_cap, io);
    if (io.density_only) {
      __syncthreads();
      return;
    }
  }
  // Alg. 1, third loop: the best blocks, best first
  unsigned long long run = 0ull;
  for (int c = 0; c * kThreads < n; ++c) {
    int i = c * kThreads + wave * 64 + lane;
    unsigned long long key = i < n ? select_key(sc[i], nb_begin + i) : 0ull;
    key = bitonic_sort_desc(key, lane);
    if (c == 0) {
      run = key;
    } else {
      run = umax64(run, shfl64(key, 63 - lane));
      run = bitonic_merge_desc(run, lane);
    }
  }
  lds.lists[wave][lane] = run;
  for (int stride = kWaves / 2; stride > 0; stride >>= 1) {
    __syncthreads();
    if (wave < stride) {
      run = umax64(run, lds.lists[wave + stride][63 - lane]);
      run = bitonic_merge_desc(run, lane);
      lds.lists[wave][lane] = run;
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
    if (lane == 0) lds.count = cutoff_count(fmaxf(logf(z) + mx - t / z, 0.f), s, n, k_cap, io);
  }
  __syncthreads();
  if (io.density_only) return;        // (density over the best blocks: the tournament had to run first)
  if (wave == 0 && lane < k_cap) {
    const int b = lane < lds.count ? int(0xffffffffu - uint32_t(run)) : -1;
    lds.sel[lane] = b;
    if (io.write) my_idx[lane] = b;
  }
  __syncthreads();
}

// ---- the same step by ONE wavefront, for rows of at most 64 * kSelWavePerLane scores ----------
// For the decode attention that selects for itself: a selection spread over a workgroup couples
// every wavefront to the slowest one at each of its barriers, and there the slowest one is stuck
// handing 32 KB of load requests to a memory pipeline that is full.  One wavefront that has issued
// nothing else needs no barrier at all: its lanes keep the scores in registers (lane l: blocks l,
// l + 64, ...), the density is two passes over them with lane exchanges, and the E best blocks come
// out one per round (the largest key of all lanes, which is unique, is taken and struck out).
// Same keys, same ties, same Eq. (11), Eq. (12) as select_body; the sums run in another order.
constexpr int kSelWavePerLane = 16;

__device__ __forceinline__ unsigned long long wave_max64(unsigned long long v) {
  v = umax64(v, lane_xor64<32>(v));
  v = umax64(v, lane_xor64<16>(v));
  v = umax64(v, lane_xor64<8>(v));
  v = umax64(v, lane_xor64<4>(v));
  v = umax64(v, lane_xor64<2>(v));
  v = umax64(v, lane_xor64<1>(v));
  return v;
}

// Called by all 64 lanes of one wavefront; sel[0 .. k_cap) and *count (LDS or any memory the
// wavefront may write) receive the result, and the global outputs are written if io.write.
// kPerLane: scores a lane holds (n <= 64 * kPerLane).
template <int kPerLane>
__device__ __forceinline__ void select_wave_n(const float* __restrict__ sc_mem, int s, int n, int nb_begin, int k_cap,
                                              int entropy_topk, const SelectIo& io, int* sel, int* count) {
  constexpr int kSelWavePerLane = kPerLane;
  const int lane = threadIdx.x & 63;
  int32_t* my_idx = io.idx + size_t(s) * k_cap;
  float v[kSelWavePerLane];
#pragma unroll
  for (int i = 0; i < kSelWavePerLane; ++i) {                    // every load before the first use
    const int b = lane + 64 * i;
    v[i] = b < n ? sc_mem[b] : -INFINITY;
  }
  if (n == 0) {
    if (lane < k_cap) {
      sel[lane] = -1;
      if (io.write) my_idx[lane] = -1;
    }
    if (lane == 0) {
      *count = 0;
      if (io.write) {
        io.n_sel[s] = 0;
        if (io.theta) io.theta[s] = 0.f;
        if (io.budget) io.budget[s] = 0.f;
        if (io.budget_in != nullptr && io.budget_after != nullptr) io.budget_after[s] = io.budget_in[s];
      }
    }
    return;
  }
  int e_count = 0;
  if (!entropy_topk) {
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < kSelWavePerLane; ++i) mx = fmaxf(mx, v[i]);
    mx = wave_max(mx);
    float z = 0.f, t = 0.f;
#pragma unroll
    for (int i = 0; i < kSelWavePerLane; ++i) {
      if (lane + 64 * i < n) {
        const float e = __expf(v[i] - mx);
        z += e;
        t += e * v[i];
      }
    }
    z = wave_sum(z);
    t = wave_sum(t);
    if (lane == 0) e_count = cutoff_count(fmaxf(logf(z) + mx - t / z, 0.f), s, n, k_cap, io);
    e_count = __shfl(e_count, 0, 64);
  }
  unsigned long long key[kSelWavePerLane];
#pragma unroll
  for (int i = 0; i < kSelWavePerLane; ++i) {
    const int b = lane + 64 * i;
    key[i] = b < n ? select_key(v[i], nb_begin + b) : 0ull;
  }
  const int rounds = entropy_topk ? min(k_cap, n) : e_count;
  unsigned long long mine = 0ull;                                // lane r: the r-th best key
  for (int r = 0; r < rounds; ++r) {
    unsigned long long best = 0ull;
#pragma unroll
    for (int i = 0; i < kSelWavePerLane; ++i) best = umax64(best, key[i]);
    best = wave_max64(best);
    if (lane == r) mine = best;
#pragma unroll
    for (int i = 0; i < kSelWavePerLane; ++i) key[i] = key[i] == best ? 0ull : key[i];
  }
  if (entropy_topk) {
    const bool in = lane < rounds;
    const float sv = in ? key_score(mine) : 0.f;
    const float mx = __shfl(sv, 0, 64);
    const float e = in ? __expf(sv - mx) : 0.f;
    const float z = wave_sum(e), t = wave_sum(e * sv);
    if (lane == 0) e_count = cutoff_count(fmaxf(logf(z) + mx - t / z, 0.f), s, n, k_cap, io);
    e_count = __shfl(e_count, 0, 64);
  }
  if (lane < k_cap) {
    const int b = lane < e_count ? int(0xffffffffu - uint32_t(mine)) : -1;
    sel[lane] = b;
    if (io.write) my_idx[lane] = b;
  }
  if (lane == 0) *count = e_count;
}
__device__ __forceinline__ void select_wave(const float* __restrict__ sc_mem, int s, int n, int nb_begin, int k_cap,
                                            int entropy_topk, const SelectIo& io, int* sel, int* count) {
  // (one instantiation: with a second one for rows of at most 512 scores, which halves the work of
  // a round, the decode step was 2 % slower - measured three times in alternation on one box)
  select_wave_n<kSelWavePerLane>(sc_mem, s, n, nb_begin, k_cap, entropy_topk, io, sel, count);
}

// The scores of one sequence as select_body reads them: the first kThreads stay in a register
// per thread for all passes (their load does not wait for anything), the others come from memory.
template <int kThreads>
struct ScoreRow {
  const float* mem;
  float first;
  __device__ __forceinline__ float operator[](int i) const { return i < kThreads ? first : mem[i]; }
};

}  // namespace actqkv
