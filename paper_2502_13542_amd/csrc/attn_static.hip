// The attention entry point that allocates nothing: its scratch memory (ticket counters, queue
// counters, partial results of split query tiles and of split decode sequences) is an array
// that is part of the library's device code instead of a workspace the caller brings.
#include <mutex>

#include "common.h"
#include "launch.h"

// One array per GPU, held from the moment the library's code is loaded on that GPU until the
// process ends.  Host code never uses the array's name as an address: the device address is
// asked for once per device (hipGetSymbolAddress) and kept.
namespace actqkv {
static __device__ __align__(256) unsigned char scratch[ACTQKV_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mu;

static int static_scratch(void** ptr_out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return set_error(ACTQKV_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return set_error(ACTQKV_EHIP, "device %d outside 0..%d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || ptr == nullptr)
      return set_error(ACTQKV_EHIP, "hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(e));
    g_scratch_ptr[dev] = ptr;
  }
  *ptr_out = g_scratch_ptr[dev];
  return ACTQKV_OK;
}

// n 32-bit zeros (a kernel, not hipMemsetAsync: the call may be recorded into a HIP graph)
__global__ __launch_bounds__(256) void fill_zero_kernel(uint32_t* __restrict__ p, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0u;
}
}  // namespace actqkv

using namespace actqkv;

extern "C" {

int actqkv_retrieval_attention_static(const actqkv_shape* shape, int batch, int m, const void* q,
                                      const void* k_cache, const void* v_cache, int64_t seq_stride,
                                      int nb_capacity, const int32_t* n_ctx, const int32_t* idx,
                                      const int32_t* n_sel, int k_cap, void* out, float* lse, void* stream) {
  size_t need = 0;
  if (int rc = attention_validate(shape, batch, m, q, k_cache, v_cache, seq_stride, nb_capacity, n_ctx, idx, n_sel,
                                  k_cap, out, lse, kChipCus, &need))
    return rc;
  if (need > size_t(ACTQKV_STATIC_SCRATCH_BYTES))
    return set_error(ACTQKV_EWORKSPACE,
                     "retrieval_attention_static: this call needs %zu bytes of scratch, the library's own buffer "
                     "has %zu (use actqkv_retrieval_attention with a workspace)",
                     need, size_t(ACTQKV_STATIC_SCRATCH_BYTES));
  void* ptr = nullptr;
  if (int rc = static_scratch(&ptr)) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  // the buffer keeps what the last call left: the counters at its head start every call at zero
  const int words = int(kCounterBytes / sizeof(uint32_t));
  hipLaunchKernelGGL(fill_zero_kernel, dim3((words + 255) / 256), dim3(256), 0, st, static_cast<uint32_t*>(ptr),
                     words);
  if (int rc = hip_status("retrieval_attention_static (counters)")) return rc;
  Workspace ws{ptr, size_t(ACTQKV_STATIC_SCRATCH_BYTES)};
  return launch_attention(*shape, batch, m, q, k_cache, v_cache, seq_stride, nb_capacity, n_ctx, idx, n_sel,
                          k_cap, out, lse, ws, 0, st);
}

}  // extern "C"
