// Selected blocks from a block store into the working cache (Sec. 3.1: the key-value cache
// may be kept in CPU memory and only what a step retrieves is brought to the GPU).
//
// The store holds the whole context in the blocked layouts of the cache; it is usually pinned
// host memory, which the kernel reads in place over the host link (no staging copy, no host
// synchronisation: the block indices come from actqkv_select on the device).  Block idx[s][j],
// j < n_sel[s], goes to block slot0 + j of the working cache, whose other blocks hold what is
// always resident: the initial tokens before the slots, the local span and the window behind
// them.  Attention then runs on the working cache with the slot numbers as its selection.
//
// grid (kGatherWgs, batch), 256 threads.  A few persistent workgroups walk over the (block, KV
// head) tiles of a sequence; a thread keeps 2 x kGatherBatch 16-byte loads in flight.  The host
// link needs about 100 KB of requests in flight to stay busy (60 GB/s times 2 us); a workgroup
// per tile had fifty times that outstanding, which fills the memory system's queues with slow
// host reads and slows every other kernel on the chip (a 9 us probe kernel beside such a
// gather took 200 us).
#include "common.h"
#include "launch.h"

namespace actqkv {

constexpr int kGatherThreads = 256;
constexpr int kGatherBatch = 4;   // 16-byte loads per tile kind a thread keeps in flight
constexpr int kGatherWgs = 8;

__global__ __launch_bounds__(kGatherThreads) void gather_blocks_kernel(
    const u32x4* __restrict__ k_store, const u32x4* __restrict__ v_store, int64_t store_stride16,
    int nb_store, const int32_t* __restrict__ idx, const int32_t* __restrict__ n_sel, int k_cap,
    u32x4* __restrict__ k_cache, u32x4* __restrict__ v_cache, int64_t cache_stride16, int slot0,
    int32_t* __restrict__ idx_slots, int n_kv_heads, int tile16) {
  const int s = blockIdx.y;
  const int e = min(max(n_sel[s], 0), k_cap);
  if (blockIdx.x == 0 && idx_slots != nullptr) {
    for (int j = threadIdx.x; j < k_cap; j += kGatherThreads) {
      const int b = idx[size_t(s) * k_cap + j];
      idx_slots[size_t(s) * k_cap + j] = (j < e && b >= 0 && b < nb_store) ? slot0 + j : -1;
    }
  }
  for (int tile = blockIdx.x; tile < e * n_kv_heads; tile += gridDim.x) {
    const int j = tile / n_kv_heads, hk = tile - j * n_kv_heads;
    const int b = idx[size_t(s) * k_cap + j];
    if (b < 0 || b >= nb_store) continue;
    const size_t src = size_t(s) * store_stride16 + (size_t(b) * n_kv_heads + hk) * tile16;
    const size_t dst = size_t(s) * cache_stride16 + (size_t(slot0 + j) * n_kv_heads + hk) * tile16;
    for (int c0 = threadIdx.x; c0 < tile16; c0 += kGatherThreads * kGatherBatch) {
      u32x4 kk[kGatherBatch], vv[kGatherBatch];
#pragma unroll
      for (int i = 0; i < kGatherBatch; ++i) {
        const int c = c0 + i * kGatherThreads;
        kk[i] = k_store[src + (c < tile16 ? c : c0)];
        vv[i] = v_store[src + (c < tile16 ? c : c0)];
      }
#pragma unroll
      for (int i = 0; i < kGatherBatch; ++i) {
        const int c = c0 + i * kGatherThreads;
        if (c < tile16) {
          k_cache[dst + c] = kk[i];
          v_cache[dst + c] = vv[i];
        }
      }
    }
  }
}

int launch_gather(const actqkv_shape& sh, int batch, const void* k_store, const void* v_store,
                  int64_t store_stride, int nb_store, const int32_t* idx, const int32_t* n_sel, int k_cap,
                  void* k_cache, void* v_cache, int64_t cache_stride, int slot0, int32_t* idx_slots,
                  hipStream_t stream) {
  const int elem = sh.dtype == ACTQKV_F32 ? 4 : 2;
  const int per16 = 16 / elem;                                   // elements per 16 bytes
  const int tile16 = sh.block_size * sh.head_dim / per16;
  hipLaunchKernelGGL(gather_blocks_kernel, dim3(kGatherWgs, batch), dim3(kGatherThreads), 0, stream,
                     static_cast<const u32x4*>(k_store), static_cast<const u32x4*>(v_store),
                     store_stride / per16, nb_store, idx, n_sel, k_cap, static_cast<u32x4*>(k_cache),
                     static_cast<u32x4*>(v_cache), cache_stride / per16, slot0, idx_slots, sh.n_kv_heads,
                     tile16);
  return hip_status("gather_blocks");
}

}  // namespace actqkv
