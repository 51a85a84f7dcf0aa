// Cache update (Sec. 3.1, Eq. (4): the cache of step t is the cache of step t-1 with the
// step's keys and values appended) in the blocked layouts the attention kernels read, and
// the representative keys of every block the new tokens complete.
//
// The paper takes the choice of a block's representatives over from earlier block-retrieval
// work without stating it; the rule here: the r tokens of the block whose key, taken over all
// KV heads together, has the largest L2 norm (ties: lower position), kept in position order.
//
// One launch, grid (Hk + 1, segments, batch), 1024 threads.  Segment g of a sequence is cache
// block pos0/128 + g.  Roles 0 .. Hk-1 copy the new tokens of one KV head that fall into the
// block: K rows as they are, V through an LDS tile so that it lands transposed ([D][128]).
// Role Hk picks the representatives if the block is full after this call and was not before;
// it reads tokens older than pos0 from the cache and the others from the new keys, so it
// does not depend on the copies of the same launch.
//
// A decode step starts with this update and with the probe of its one-token window, which is
// the query itself (Sec. 4.2); the two have nothing to do with each other, and each is a few
// microseconds of work behind a launch.  With a query given, one more role (Hk + 1, first
// segment) forms that probe in the same launch.
#include <algorithm>

#include "common.h"
#include "launch.h"
#include "probe_identity.h"

namespace actqkv {

constexpr int kApThreads = 1024;

template <typename T>
__global__ __launch_bounds__(kApThreads) void append_kv_kernel(
    const T* __restrict__ k_new, const T* __restrict__ v_new, const int32_t* __restrict__ pos0_all,
    T* __restrict__ k_cache, T* __restrict__ v_cache, int64_t cache_stride, T* __restrict__ rep_keys,
    int64_t rep_stride, int nb_capacity, int m, int n_kv_heads, int head_dim, int n_rep,
    const T* __restrict__ q_tok, float* __restrict__ probe, float* __restrict__ probe_kv,
    float* __restrict__ probe_norm, int n_q_heads) {
  constexpr int V = Vec<T>::N;
  extern __shared__ __attribute__((aligned(16))) unsigned char ap_lds[];
  const int role = blockIdx.x, s = blockIdx.z;
  if (role == n_kv_heads + 1) {
    // ---- the probe of the step's one-token window
    if (blockIdx.y != 0) return;
    __shared__ float red[32];
    const int d = n_q_heads * head_dim;
    probe_identity_body<T>(q_tok + size_t(s) * d, probe + size_t(s) * d,
                           probe_kv + size_t(s) * n_kv_heads * head_dim, probe_norm + s, nullptr, n_q_heads,
                           n_kv_heads, head_dim, reinterpret_cast<float*>(ap_lds), red);
    return;
  }
  const int pos0 = max(pos0_all[s], 0);
  const int block = pos0 / kBlock + blockIdx.y;
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
    for (int i = threadIdx.x; i < n_tok * chunks; i += kApThreads) {
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
    for (int i = threadIdx.x; i < head_dim * n_tok; i += kApThreads) {
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
    const int tk = threadIdx.x >> 3, part = threadIdx.x & 7;
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
  for (int i = threadIdx.x; i < kBlock * chunks; i += kApThreads) {
    const int tk = i / chunks, c = i - tk * chunks;
    const int slot = chosen[tk];
    if (slot >= 0)
      *reinterpret_cast<typename Vec<T>::raw*>(rd + size_t(slot) * row_len + size_t(c) * V) =
          Vec<T>::load_raw(token_chunk(tk, c));
  }
}

int launch_append(const actqkv_shape& sh, int batch, int m, const void* k_new, const void* v_new,
                  const int32_t* pos0, void* k_cache, void* v_cache, int64_t cache_stride,
                  void* rep_keys, int64_t rep_stride, int nb_capacity, const void* q_tok, float* probe,
                  float* probe_kv, float* probe_norm, hipStream_t stream) {
  const int segments = (m + kBlock - 1) / kBlock + 1;              // a window may straddle one more block
  dim3 grid(sh.n_kv_heads + 1 + (q_tok != nullptr ? 1 : 0), segments, batch);
  const size_t elem = sh.dtype == ACTQKV_F32 ? 4 : 2;
  size_t lds = std::max(size_t(sh.head_dim) * (kBlock + 2) * elem, size_t(2 * kBlock) * 4);
  if (q_tok != nullptr) lds = std::max(lds, size_t(sh.n_q_heads) * sh.head_dim * sizeof(float));
  if (sh.dtype == ACTQKV_F32) {
    static bool attr_set = false;
    if (!attr_set) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(append_kv_kernel<float>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 128 * (kBlock + 2) * 4);
      if (e != hipSuccess) return set_error(ACTQKV_EHIP, "hipFuncSetAttribute: %s", hipGetErrorString(e));
      attr_set = true;
    }
    hipLaunchKernelGGL(append_kv_kernel<float>, grid, dim3(kApThreads), lds, stream,
                       static_cast<const float*>(k_new), static_cast<const float*>(v_new), pos0,
                       static_cast<float*>(k_cache), static_cast<float*>(v_cache), cache_stride,
                       static_cast<float*>(rep_keys), rep_stride, nb_capacity, m, sh.n_kv_heads,
                       sh.head_dim, sh.n_rep, static_cast<const float*>(q_tok), probe, probe_kv, probe_norm,
                       sh.n_q_heads);
  } else {
    hipLaunchKernelGGL(append_kv_kernel<uint16_t>, grid, dim3(kApThreads), lds, stream,
                       static_cast<const uint16_t*>(k_new), static_cast<const uint16_t*>(v_new), pos0,
                       static_cast<uint16_t*>(k_cache), static_cast<uint16_t*>(v_cache), cache_stride,
                       static_cast<uint16_t*>(rep_keys), rep_stride, nb_capacity, m, sh.n_kv_heads,
                       sh.head_dim, sh.n_rep, static_cast<const uint16_t*>(q_tok), probe, probe_kv,
                       probe_norm, sh.n_q_heads);
  }
  return hip_status("append_kv");
}

}  // namespace actqkv
