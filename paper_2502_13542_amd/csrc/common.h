// Shared device helpers for the gfx950 kernels of the retrieval-attention path.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/actqkv.h"

namespace actqkv {

constexpr int kWave = 64;
constexpr int kBlock = 128;  // tokens per KV block (the only supported block size)

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

// ---- bf16 <-> fp32 (bf16 is the upper half of an fp32) ---------------------
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) {
  return __uint_as_float(packed & 0xffff0000u);
}
// round-to-nearest-even; NaN stays NaN
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

// acc += a.lo * b.lo + a.hi * b.hi for two packed pairs of bf16 (one instruction; written as
// assembly because the compiler's builtin for it takes the first pair of a packed vector
// whatever element is asked for)
__device__ __forceinline__ void dot2_bf16(float& acc, uint32_t a, uint32_t b) {
  asm("v_dot2c_f32_bf16 %0, %1, %2" : "+v"(acc) : "v"(a), "v"(b));
}

// ---- 16-byte vector loads of VEC consecutive elements widened to fp32 ------
template <typename T> struct Vec;  // T = float: 4 elements; T = uint16_t (bf16 bits): 8 elements
template <> struct Vec<float> {
  static constexpr int N = 4;
  typedef f32x4 raw;
  __device__ static __forceinline__ raw load_raw(const float* p) { return *reinterpret_cast<const f32x4*>(p); }
  __device__ static __forceinline__ void widen(const raw& v, float (&out)[4]) {
    out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
  }
  __device__ static __forceinline__ void load(const float* p, float (&out)[4]) { widen(load_raw(p), out); }
};
template <> struct Vec<uint16_t> {
  static constexpr int N = 8;
  typedef u32x4 raw;
  __device__ static __forceinline__ raw load_raw(const uint16_t* p) { return *reinterpret_cast<const u32x4*>(p); }
  __device__ static __forceinline__ void widen(const raw& v, float (&out)[8]) {
    out[0] = bf16_lo(v.x); out[1] = bf16_hi(v.x); out[2] = bf16_lo(v.y); out[3] = bf16_hi(v.y);
    out[4] = bf16_lo(v.z); out[5] = bf16_hi(v.z); out[6] = bf16_lo(v.w); out[7] = bf16_hi(v.w);
  }
  __device__ static __forceinline__ void load(const uint16_t* p, float (&out)[8]) { widen(load_raw(p), out); }
};

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(uint16_t x) { return __uint_as_float(uint32_t(x) << 16); }
__device__ __forceinline__ void store_elem(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_elem(uint16_t* p, float v) { *p = uint16_t(f32_to_bf16_bits(v)); }

// ---- wave / workgroup reductions ------------------------------------------
// The value of lane (lane ^ J), J a power of two, without the LDS crossbar where the data-parallel
// primitives reach: quad permutes for 1 and 2, two masked row shifts for 4 and 8 (banks of four
// lanes take the value from J lanes above or below), a swizzle for 16; only 32 is a general shuffle.
template <int J>
__device__ __forceinline__ uint32_t lane_xor32(uint32_t v) {
  if constexpr (J == 1) {
    return __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xF, 0xF, false);          // quad_perm [1, 0, 3, 2]
  } else if constexpr (J == 2) {
    return __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xF, 0xF, false);          // quad_perm [2, 3, 0, 1]
  } else if constexpr (J == 4) {
    const uint32_t t = __builtin_amdgcn_update_dpp(v, v, 0x104, 0xF, 0x5, false);   // row_shl:4 into banks 0, 2
    return __builtin_amdgcn_update_dpp(t, v, 0x114, 0xF, 0xA, false);               // row_shr:4 into banks 1, 3
  } else if constexpr (J == 8) {
    const uint32_t t = __builtin_amdgcn_update_dpp(v, v, 0x108, 0xF, 0x3, false);   // row_shl:8 into banks 0, 1
    return __builtin_amdgcn_update_dpp(t, v, 0x118, 0xF, 0xC, false);               // row_shr:8 into banks 2, 3
  } else if constexpr (J == 16) {
    return uint32_t(__builtin_amdgcn_ds_swizzle(int(v), (16 << 10) | 0x1F));  // bit mode: xor 16 inside 32 lanes
  } else {
    static_assert(J == 32, "lane distance");
    return uint32_t(__shfl_xor(int(v), 32, 64));
  }
}
template <int J>
__device__ __forceinline__ float lane_xor_f32(float v) {
  return __uint_as_float(lane_xor32<J>(__float_as_uint(v)));
}
__device__ __forceinline__ float wave_sum(float v) {
  v += lane_xor_f32<32>(v);
  v += lane_xor_f32<16>(v);
  v += lane_xor_f32<8>(v);
  v += lane_xor_f32<4>(v);
  v += lane_xor_f32<2>(v);
  v += lane_xor_f32<1>(v);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, lane_xor_f32<32>(v));
  v = fmaxf(v, lane_xor_f32<16>(v));
  v = fmaxf(v, lane_xor_f32<8>(v));
  v = fmaxf(v, lane_xor_f32<4>(v));
  v = fmaxf(v, lane_xor_f32<2>(v));
  v = fmaxf(v, lane_xor_f32<1>(v));
  return v;
}
// Sum over the workgroup; every thread gets the result.  `red` holds >= 32 floats of LDS.
__device__ __forceinline__ float block_sum(float v, float* red) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  v = wave_sum(v);
  __syncthreads();
  if (lane == 0) red[w] = v;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < nw; ++i) t += red[i];
  return t;
}
__device__ __forceinline__ float block_max(float v, float* red) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  v = wave_max(v);
  __syncthreads();
  if (lane == 0) red[w] = v;
  __syncthreads();
  float t = red[0];
  for (int i = 1; i < nw; ++i) t = fmaxf(t, red[i]);
  return t;
}

// ---- merging the partial results of several workgroups inside one kernel ----------------
// The workgroups of a group store their partials with agent-scope relaxed atomic stores
// (write-through: the data leaves the XCD's L2, which other XCDs do not see), wait until
// these are acknowledged and take a ticket; the one that draws the last ticket reads all
// partials back with agent-scope atomic loads (which do not hit stale L2 lines) and writes
// the result.  No device-scope fence is involved: on this chip such a fence writes back and
// invalidates a whole L2 and costs more than a kernel boundary.  Nobody waits for anybody,
// so every wavefront runs to its end whatever the others do.
__device__ __forceinline__ void st_agent(uint64_t* p, uint64_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(uint32_t* p, uint32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t ld_agent(const uint64_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t ld_agent(const uint32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// True in every thread of the workgroup that arrives last out of `total` at `counter`
// (zero before the first arrival; the last one puts it back to zero).  Called by all
// threads after their st_agent stores; `flag` is one int of LDS.
__device__ __forceinline__ bool last_of_group(unsigned int* counter, unsigned int total, int* flag) {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_waitcnt(0);       // this wavefront's stores have been acknowledged
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned int t = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last = t == total - 1u;
    if (last) __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *flag = last;
  }
  __syncthreads();
  return *flag != 0;
}

// ---- window geometry -------------------------------------------------------
// Tokens [0, i0) are the visible initial tokens; the local span starts at l0.
struct WindowGeom {
  int w0, i0, l0;
};
__host__ __device__ __forceinline__ WindowGeom window_geom(int n_ctx, int m, int n_init, int n_local) {
  WindowGeom g;
  g.w0 = n_ctx - m;
  if (g.w0 < 0) g.w0 = 0;
  g.i0 = n_init < g.w0 ? n_init : g.w0;
  int a = g.w0 - n_local;
  a = a > 0 ? (a / kBlock) * kBlock : 0;
  g.l0 = a > g.i0 ? a : g.i0;
  return g;
}

// The list of key tiles one query tile walks through: initial tokens, selected
// blocks, then the local span and the window itself up to the tile's last query.
// Tile t covers key positions [lo, hi) of cache block `block` (hi <= lo: empty).
struct TileList {
  int n_init_tiles, n_sel, n_tail_tiles, tail_block0;
  int i0, l0, q_hi;
  const int32_t* idx;
  int nb_capacity;
  __device__ __forceinline__ int count() const { return n_init_tiles + n_sel + n_tail_tiles; }
  __device__ __forceinline__ void get(int t, int& block, int& lo, int& hi) const {
    if (t < n_init_tiles) {
      block = t;
      lo = t * kBlock;
      hi = min(lo + kBlock, i0);
    } else if (t < n_init_tiles + n_sel) {
      int b = idx[t - n_init_tiles];
      bool ok = (b >= 0) && (b < nb_capacity);
      block = ok ? b : 0;
      lo = block * kBlock;
      hi = ok ? lo + kBlock : lo;
    } else {
      block = tail_block0 + (t - n_init_tiles - n_sel);
      lo = max(block * kBlock, l0);
      hi = min(block * kBlock + kBlock, q_hi + 1);
    }
  }
};
// q_hi: position of the last query of the tile.  n_ctx is clamped by the caller.
__device__ __forceinline__ TileList make_tile_list(const WindowGeom& g, int q_hi, const int32_t* idx,
                                                   int n_sel, int k_cap, int nb_capacity) {
  TileList tl;
  tl.i0 = g.i0;
  tl.l0 = g.l0;
  tl.q_hi = q_hi;
  tl.n_init_tiles = (g.i0 + kBlock - 1) / kBlock;
  tl.n_sel = n_sel < 0 ? 0 : (n_sel > k_cap ? k_cap : n_sel);
  tl.tail_block0 = g.l0 / kBlock;
  tl.n_tail_tiles = q_hi / kBlock - tl.tail_block0 + 1;
  tl.idx = idx;
  tl.nb_capacity = nb_capacity;
  return tl;
}

}  // namespace actqkv
