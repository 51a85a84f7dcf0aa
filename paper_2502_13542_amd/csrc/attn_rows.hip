// Retrieval attention, plain-ALU form (Sec. 3.1, Eq. (2)): one thread owns one
// query row of one head and walks the key tiles (initial tokens, selected
// blocks, local span, causal part of the window) with an online softmax in
// fp32.  This is the fp32-mode kernel (no bf16 rounding anywhere), and the
// fallback for shapes the matrix-core kernel does not take.
#include "common.h"
#include "launch.h"

namespace actqkv {

constexpr int kRowsPerWG = 128;
constexpr int kSub = 64;  // keys staged in LDS at a time

template <typename T, int D>
__global__ __launch_bounds__(kRowsPerWG) void attn_rows_kernel(
    const T* __restrict__ q, const T* __restrict__ k_cache, const T* __restrict__ v_cache,
    int64_t seq_stride, int nb_capacity, const int32_t* __restrict__ n_ctx_arr,
    const int32_t* __restrict__ idx, const int32_t* __restrict__ n_sel, int k_cap,
    T* __restrict__ out, float* __restrict__ lse, int m, int n_q_heads, int n_kv_heads, int n_init,
    int n_local, float scale, int sel_per_head) {
  __shared__ float ks[kSub][D];
  __shared__ float vs[D][kSub];
  const int s = blockIdx.z, h = blockIdx.y, hk = h / (n_q_heads / n_kv_heads);
  const int row = blockIdx.x * kRowsPerWG + threadIdx.x;
  const bool active = row < m;
  int n_ctx = min(max(n_ctx_arr[s], m), nb_capacity * kBlock);
  const WindowGeom g = window_geom(n_ctx, m, n_init, n_local);
  const int p = g.w0 + row;  // this thread's query position
  const int q_hi = g.w0 + min(m, (int(blockIdx.x) + 1) * kRowsPerWG) - 1;
  const size_t sel_row = sel_per_head ? size_t(s) * n_kv_heads + hk : size_t(s);
  const TileList tl = make_tile_list(g, q_hi, idx + sel_row * k_cap, n_sel[sel_row], k_cap, nb_capacity);
  const T* kc = k_cache + size_t(s) * seq_stride;
  const T* vc = v_cache + size_t(s) * seq_stride;

  float qr[D], acc[D];
  if (active) {
    const T* qp = q + ((size_t(s) * m + row) * n_q_heads + h) * D;
#pragma unroll
    for (int d = 0; d < D; ++d) qr[d] = to_f32(qp[d]) * scale;
  }
#pragma unroll
  for (int d = 0; d < D; ++d) acc[d] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  const int n_tiles = tl.count();
  for (int t = 0; t < n_tiles; ++t) {
    int block, lo, hi;
    tl.get(t, block, lo, hi);
    if (hi <= lo) continue;
    for (int sub = 0; sub < kBlock / kSub; ++sub) {
      const int kp0 = block * kBlock + sub * kSub;
      if (kp0 >= hi || kp0 + kSub <= lo) continue;
      __syncthreads();
      const T* kt = kc + ((size_t(block) * n_kv_heads + hk) * kBlock + sub * kSub) * D;
      for (int i = threadIdx.x; i < kSub * D; i += kRowsPerWG) ks[i / D][i % D] = to_f32(kt[i]);
      const T* vt = vc + (size_t(block) * n_kv_heads + hk) * D * kBlock + sub * kSub;
      for (int i = threadIdx.x; i < kSub * D; i += kRowsPerWG) {
        int d = i / kSub, j = i % kSub;
        vs[d][j] = to_f32(vt[size_t(d) * kBlock + j]);
      }
      __syncthreads();
      if (!active) continue;
      for (int c0 = 0; c0 < kSub; c0 += 16) {
        float sc[16];
        float cmax = -INFINITY;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const int kp = kp0 + c0 + j;
          float dot = 0.f;
#pragma unroll
          for (int d = 0; d < D; ++d) dot += qr[d] * ks[c0 + j][d];
          const bool ok = kp >= lo && kp < hi && kp <= p;
          sc[j] = ok ? dot : -INFINITY;
          cmax = fmaxf(cmax, sc[j]);
        }
        if (cmax == -INFINITY) continue;
        if (cmax > m_run) {
          const float alpha = __expf(m_run - cmax);  // 0 when m_run is -inf
          l_run *= alpha;
#pragma unroll
          for (int d = 0; d < D; ++d) acc[d] *= alpha;
          m_run = cmax;
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const float pj = __expf(sc[j] - m_run);  // exp(-inf) = 0 for masked keys
          l_run += pj;
#pragma unroll
          for (int d = 0; d < D; ++d) acc[d] += pj * vs[d][c0 + j];
        }
      }
    }
  }
  if (!active) return;
  const float inv = l_run > 0.f ? 1.f / l_run : 0.f;
  T* op = out + ((size_t(s) * m + row) * n_q_heads + h) * D;
#pragma unroll
  for (int d = 0; d < D; ++d) store_elem(op + d, acc[d] * inv);
  if (lse != nullptr) lse[(size_t(s) * n_q_heads + h) * m + row] = m_run + logf(l_run);
}

template <typename T, int D>
static void launch_rows_t(const actqkv_shape& sh, int batch, int m, const void* q, const void* k_cache,
                          const void* v_cache, int64_t seq_stride, int nb_capacity,
                          const int32_t* n_ctx, const int32_t* idx, const int32_t* n_sel, int k_cap,
                          void* out, float* lse, float scale, int sel_per_head, hipStream_t stream) {
  dim3 grid((m + kRowsPerWG - 1) / kRowsPerWG, sh.n_q_heads, batch);
  hipLaunchKernelGGL((attn_rows_kernel<T, D>), grid, dim3(kRowsPerWG), 0, stream,
                     static_cast<const T*>(q), static_cast<const T*>(k_cache),
                     static_cast<const T*>(v_cache), seq_stride, nb_capacity, n_ctx, idx, n_sel, k_cap,
                     static_cast<T*>(out), lse, m, sh.n_q_heads, sh.n_kv_heads, sh.n_init, sh.n_local,
                     scale, sel_per_head);
}

int launch_attention_rows(const actqkv_shape& sh, int batch, int m, const void* q, const void* k_cache,
                          const void* v_cache, int64_t seq_stride, int nb_capacity,
                          const int32_t* n_ctx, const int32_t* idx, const int32_t* n_sel, int k_cap,
                          void* out, float* lse, float scale, int sel_per_head, hipStream_t stream) {
#define ACTQKV_ROWS(T, D)                                                                         \
  launch_rows_t<T, D>(sh, batch, m, q, k_cache, v_cache, seq_stride, nb_capacity, n_ctx, idx, n_sel, \
                      k_cap, out, lse, scale, sel_per_head, stream)
  if (sh.dtype == ACTQKV_F32) {
    if (sh.head_dim == 64) ACTQKV_ROWS(float, 64); else ACTQKV_ROWS(float, 128);
  } else {
    if (sh.head_dim == 64) ACTQKV_ROWS(uint16_t, 64); else ACTQKV_ROWS(uint16_t, 128);
  }
#undef ACTQKV_ROWS
  return hip_status("attention (rows)");
}

}  // namespace actqkv
