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
#include <mutex>

#include "common.h"
#include "append_body.h"
#include "launch.h"
#include "probe_identity.h"

namespace actqkv {

template <typename T>
__global__ __launch_bounds__(kApThreads) void append_kv_kernel(
    const T* __restrict__ k_new, const T* __restrict__ v_new, const int32_t* __restrict__ pos0_all,
    T* __restrict__ k_cache, T* __restrict__ v_cache, int64_t cache_stride, T* __restrict__ rep_keys,
    int64_t rep_stride, int nb_capacity, int m, int n_kv_heads, int head_dim, int n_rep,
    const T* __restrict__ q_tok, float* __restrict__ probe, float* __restrict__ probe_kv,
    float* __restrict__ probe_norm, int n_q_heads) {
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
  append_body<T>(role, int(blockIdx.y), s, k_new, v_new, pos0_all[s], k_cache, v_cache, cache_stride, rep_keys,
                 rep_stride, nb_capacity, m, n_kv_heads, head_dim, n_rep, ap_lds);
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
    static std::mutex mu;       // once per process, from whichever thread comes first
    static bool attr_set = false;
    std::lock_guard<std::mutex> lock(mu);
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
