// Retrieval attention of a decode step (Sec. 3.1, Eq. (3): one query token per sequence
// over [k^t, K*]; bf16 storage, fp32 accumulation).  HBM-bound: every selected key and
// value byte is read exactly once, by exactly one wavefront.
//
// A wavefront owns whole 128-key tiles of one (sequence, KV head): initial tokens, the
// blocks chosen by actqkv_select (read from device memory) or the local span up to the new
// token.  The G query heads of the KV head ride along as columns of a 16-wide matrix-core
// tile, so a key or value byte is loaded once for all of them, straight from global memory
// into MFMA operands (no LDS staging: nothing is shared between wavefronts):
//   S^T[key][head] = K[key][:] Q^T        v_mfma_f32_16x16x32_bf16, A = 16 keys x 32 channels
//   O^T[d][head]  += V^T[d][keys] P^T     A = 16 channels x 32 keys of the transposed V block
// A lane of an A operand reads 16 contiguous bytes and four lanes cover 64 contiguous
// bytes of a row.  Keys enter S^T in a permuted row order such that each lane's accumulator
// registers hold 8 consecutive keys of every 32-key step, which is exactly the B-operand
// layout of the second product; no cross-lane traffic is needed apart from two shuffles
// for the row maximum.  The 8 wavefronts of a workgroup merge their (max, sum, O) through
// LDS.  If one workgroup covers a whole (sequence, KV head) it writes the output itself;
// otherwise the workgroups store partials and the one that finishes last merges them.
#include "common.h"
#include "launch.h"

namespace actqkv {

constexpr int kDcD = 128;
constexpr int kDcMaxWaves = 8;   // 512 threads: the register budget stays at 256 per lane
#ifndef ACTQKV_DC_ITEM_KEYS
#define ACTQKV_DC_ITEM_KEYS 64
#endif
constexpr int kDcItemKeys = ACTQKV_DC_ITEM_KEYS;   // keys per work item: 64 or 128

struct DcParams {
  const uint16_t* q;
  const uint16_t* k_cache;
  const uint16_t* v_cache;
  int64_t seq_stride;
  int nb_capacity;
  const int32_t* n_ctx;
  const int32_t* idx;
  const int32_t* n_sel;
  int k_cap;
  uint16_t* out;
  float* lse;
  uint32_t* part;           // [batch][Hk][n_wg][G][D + 2] fp32 bits
  unsigned int* counters;   // one ticket counter per (sequence, KV head), zero between launches
  int n_q_heads, n_kv_heads, n_init, n_local;
  int n_wg;     // workgroups per (sequence, KV head); 1: the workgroup writes the output itself
  int sel_per_head;   // 1: idx and n_sel have a row per (sequence, KV head), 0: per sequence
  float scale_log2e;
};

__device__ __forceinline__ bf16x8 dc_as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// grid (n_wg, Hk, batch); blockDim = 64 * (wavefronts per workgroup).  Wavefront w of
// workgroup g walks tiles g*W + w, g*W + w + n_wg*W, ...
__global__ __launch_bounds__(kDcMaxWaves * 64) void attn_decode_kernel(DcParams p) {
  extern __shared__ __attribute__((aligned(16))) float dc_lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
  const int n = lane & 15, kq = lane >> 4;       // MFMA column (query head) and lane quarter
  const int wg = blockIdx.x, hk = blockIdx.y, s = blockIdx.z;
  const int group = p.n_q_heads / p.n_kv_heads;
  float* red_ml = dc_lds;                        // [n_waves][group][2]
  float* red_o = dc_lds + n_waves * group * 2;   // [n_waves][group][D]

  const int n_ctx = min(max(p.n_ctx[s], 1), p.nb_capacity * kBlock);
  const WindowGeom g = window_geom(n_ctx, 1, p.n_init, p.n_local);
  const size_t sel_row = p.sel_per_head ? size_t(s) * p.n_kv_heads + hk : size_t(s);
  const TileList tl = make_tile_list(g, n_ctx - 1, p.idx + sel_row * p.k_cap, p.n_sel[sel_row], p.k_cap,
                                     p.nb_capacity);
  const int n_tiles = tl.count();

  // Q^T as B operand: lane (n, kq) holds channels ks*32 + 8*kq .. +7 of head n (zero for n >= G)
  bf16x8 qb[4];
  {
    const uint16_t* qp = p.q + (size_t(s) * p.n_q_heads + hk * group + min(n, group - 1)) * kDcD + 8 * kq;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      u32x4 v = *reinterpret_cast<const u32x4*>(qp + ks * 32);
      if (n >= group) v = u32x4{0u, 0u, 0u, 0u};
      qb[ks] = dc_as_bf16x8(v);
    }
  }
  float m_run = -INFINITY, l_run = 0.f;
  f32x4 acc_o[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc_o[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  const size_t tile_elems = size_t(kBlock) * kDcD;
  const uint16_t* kc = p.k_cache + size_t(s) * p.seq_stride;
  const uint16_t* vc = p.v_cache + size_t(s) * p.seq_stride;

  // Work items are spans of kDcItemKeys keys of a tile; item i of the list goes to wavefront i mod (all
  // wavefronts of the pair).  Keys AND values of an item are requested before anything is computed.
  constexpr int kSteps = kDcItemKeys / 32, kPerTile = kBlock / kDcItemKeys;
  const int n_items = n_tiles * kPerTile;
  for (int it = wg * n_waves + wave; it < n_items; it += p.n_wg * n_waves) {
    int block, lo, hi;
    tl.get(it / kPerTile, block, lo, hi);
    const int part = it % kPerTile;
    const int kpos0 = block * kBlock + part * kDcItemKeys;
    lo = max(lo, kpos0);
    hi = min(hi, kpos0 + kDcItemKeys);
    if (hi <= lo) continue;                      // wave-uniform
    const uint16_t* kt = kc + (size_t(block) * p.n_kv_heads + hk) * tile_elems + size_t(part) * kDcItemKeys * kDcD;
    const uint16_t* vt = vc + (size_t(block) * p.n_kv_heads + hk) * tile_elems + part * kDcItemKeys;

    // A operands of S^T: MFMA row r of sub-tile h of 32-key step st is key 32*st + 8*(r/4) + 4*h + r%4,
    // so that lane quarter kq ends up with keys 32*st + 8*kq + 4*h + i in register i.
    u32x4 ka[8 * kSteps];
    {
      const uint16_t* base = kt + size_t(8 * (n >> 2) + (n & 3)) * kDcD + 8 * kq;
#pragma unroll
      for (int st = 0; st < kSteps; ++st)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int ks = 0; ks < 4; ++ks)
            ka[(st * 2 + h) * 4 + ks] =
                *reinterpret_cast<const u32x4*>(base + size_t(32 * st + 4 * h) * kDcD + ks * 32);
    }
    // V^T A operands: lane (row = channel within a group of 16, kq) reads keys 32*st + 8*kq .. +7
    u32x4 va[8 * kSteps];
    {
      const uint16_t* base = vt + size_t(n) * kBlock + 8 * kq;
#pragma unroll
      for (int dg = 0; dg < 8; ++dg)
#pragma unroll
        for (int st = 0; st < kSteps; ++st)
          va[dg * kSteps + st] = *reinterpret_cast<const u32x4*>(base + size_t(16 * dg) * kBlock + 32 * st);
    }
    __builtin_amdgcn_sched_barrier(0);   // all key and value loads are in flight before the first MFMA
    f32x4 sc[2 * kSteps];
#pragma unroll
    for (int j = 0; j < 2 * kSteps; ++j) sc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)       // the sub-tiles take turns: no MFMA waits for the one before it
#pragma unroll
      for (int j = 0; j < 2 * kSteps; ++j)
        sc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(dc_as_bf16x8(ka[j * 4 + ks]), qb[ks], sc[j], 0, 0, 0);
    // mask and online softmax: sc[2*st + h][i] is key kpos0 + 32*st + 8*kq + 4*h + i
    float mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < 2 * kSteps; ++j)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int kp = kpos0 + 32 * (j >> 1) + 8 * kq + 4 * (j & 1) + i;
        const float v = (kp >= lo && kp < hi) ? sc[j][i] : -INFINITY;
        sc[j][i] = v;
        mx = fmaxf(mx, v);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx * p.scale_log2e);   // finite: the item has a visible key
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    float psum = 0.f;
#pragma unroll
    for (int j = 0; j < 2 * kSteps; ++j)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float pv = __builtin_amdgcn_exp2f(sc[j][i] * p.scale_log2e - m_new);
        sc[j][i] = pv;
        psum += pv;
      }
    psum += __shfl_xor(psum, 16, 64);
    psum += __shfl_xor(psum, 32, 64);
    l_run = l_run * alpha + psum;
#pragma unroll
    for (int dg = 0; dg < 8; ++dg) acc_o[dg] *= alpha;
    // O^T += V^T P^T
    typedef __attribute__((ext_vector_type(8))) float f32x8;
#pragma unroll
    for (int st = 0; st < kSteps; ++st) {
      f32x8 pf = {sc[2 * st][0], sc[2 * st][1], sc[2 * st][2], sc[2 * st][3],
                  sc[2 * st + 1][0], sc[2 * st + 1][1], sc[2 * st + 1][2], sc[2 * st + 1][3]};
      const bf16x8 pb = __builtin_convertvector(pf, bf16x8);
#pragma unroll
      for (int dg = 0; dg < 8; ++dg)
        acc_o[dg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(dc_as_bf16x8(va[dg * kSteps + st]), pb, acc_o[dg], 0, 0, 0);
    }
  }

  // merge the wavefronts: lane (n < G, kq) holds channels 16*dg + 4*kq + i of head n
  if (n < group) {
    if (kq == 0) {
      red_ml[(wave * group + n) * 2 + 0] = m_run;
      red_ml[(wave * group + n) * 2 + 1] = l_run;
    }
#pragma unroll
    for (int dg = 0; dg < 8; ++dg)
      *reinterpret_cast<f32x4*>(&red_o[(wave * group + n) * kDcD + 16 * dg + 4 * kq]) = acc_o[dg];
  }
  __syncthreads();
  uint32_t* pair_part = p.part + (size_t(s) * p.n_kv_heads + hk) * p.n_wg * group * (kDcD + 2);
  uint32_t* part = pair_part + size_t(wg) * group * (kDcD + 2);
  for (int e = threadIdx.x; e < group * kDcD; e += blockDim.x) {
    const int h = e / kDcD, d = e - h * kDcD;
    float mm = -INFINITY;
    for (int w = 0; w < n_waves; ++w) mm = fmaxf(mm, red_ml[(w * group + h) * 2]);
    const float m_safe = mm == -INFINITY ? 0.f : mm;
    float l = 0.f, o = 0.f;
    for (int w = 0; w < n_waves; ++w) {
      const float sc_w = __builtin_amdgcn_exp2f(red_ml[(w * group + h) * 2] - m_safe);
      l += sc_w * red_ml[(w * group + h) * 2 + 1];
      o += sc_w * red_o[(w * group + h) * kDcD + d];
    }
    if (p.n_wg == 1) {
      const int head = hk * group + h;
      p.out[(size_t(s) * p.n_q_heads + head) * kDcD + d] = uint16_t(f32_to_bf16_bits(l > 0.f ? o / l : 0.f));
      if (p.lse != nullptr && d == 0)
        p.lse[size_t(s) * p.n_q_heads + head] = (mm + log2f(l)) * 0.6931471805599453f;
    } else {
      st_agent(part + size_t(h) * (kDcD + 2) + d, __float_as_uint(o));
      if (d == 0) {
        st_agent(part + size_t(h) * (kDcD + 2) + kDcD, __float_as_uint(mm));
        st_agent(part + size_t(h) * (kDcD + 2) + kDcD + 1, __float_as_uint(l));
      }
    }
  }
  if (p.n_wg == 1) return;
  __shared__ int last_flag;
  if (!last_of_group(p.counters + size_t(s) * p.n_kv_heads + hk, unsigned(p.n_wg), &last_flag)) return;

  // ---- the workgroup that finished last merges the partials, in workgroup order:
  //   out[head][:] = sum_w 2^(m_w - M) O_w / sum_w 2^(m_w - M) l_w
  const size_t stride = size_t(group) * (kDcD + 2);
  constexpr int kB = 8;
  for (int e = threadIdx.x; e < group * kDcD; e += blockDim.x) {
    const int h = e / kDcD, d = e - h * kDcD;
    const uint32_t* src = pair_part + size_t(h) * (kDcD + 2);
    float mm = -INFINITY, l = 0.f, o = 0.f;
    for (int w0 = 0; w0 < p.n_wg; w0 += kB) {
      uint32_t pm[kB], pl[kB], po[kB];
#pragma unroll
      for (int i = 0; i < kB; ++i) {               // all loads first: they overlap
        const int w = w0 + i < p.n_wg ? w0 + i : w0;
        pm[i] = ld_agent(src + w * stride + kDcD);
        pl[i] = ld_agent(src + w * stride + kDcD + 1);
        po[i] = ld_agent(src + w * stride + d);
      }
#pragma unroll
      for (int i = 0; i < kB; ++i) {
        if (w0 + i < p.n_wg) {
          const float pmf = __uint_as_float(pm[i]);
          const float m_new = fmaxf(mm, pmf);
          const float m_safe = m_new == -INFINITY ? 0.f : m_new;
          const float wa = __builtin_amdgcn_exp2f(mm - m_safe), wb = __builtin_amdgcn_exp2f(pmf - m_safe);
          l = l * wa + __uint_as_float(pl[i]) * wb;
          o = o * wa + __uint_as_float(po[i]) * wb;
          mm = m_new;
        }
      }
    }
    const float inv = l > 0.f ? 1.f / l : 0.f;
    const int head = hk * group + h;
    p.out[(size_t(s) * p.n_q_heads + head) * kDcD + d] = uint16_t(f32_to_bf16_bits(o * inv));
    if (p.lse != nullptr && d == 0)
      p.lse[size_t(s) * p.n_q_heads + head] = (mm + log2f(l)) * 0.6931471805599453f;
  }
}

bool decode_mfma_supported(const actqkv_shape& sh, int m) {
  const int g = sh.n_q_heads / sh.n_kv_heads;
  return sh.dtype == ACTQKV_BF16 && sh.head_dim == kDcD && m == 1 && g <= 8;
}

// Launch shape: workgroups of 8 wavefronts; about 2048 wavefronts in total (two per SIMD,
// each with a whole tile's loads in flight) unless the tile list is shorter than that.
// One workgroup per (sequence, KV head) writes the output itself; with more, the one that
// finishes last merges the partials.
static int decode_tiles_max(const actqkv_shape& sh, int k_cap) {
  return (sh.n_init + kBlock - 1) / kBlock + k_cap + sh.n_local / kBlock + 2;
}
int decode_mfma_workgroups(const actqkv_shape& sh, int batch, int k_cap) {
  const int pairs = batch * sh.n_kv_heads;
  const int want = (2048 + pairs * kDcMaxWaves - 1) / (pairs * kDcMaxWaves);
  const int most = (decode_tiles_max(sh, k_cap) + kDcMaxWaves - 1) / kDcMaxWaves;
  return want < 1 ? 1 : (want > most ? most : want);
}

size_t decode_mfma_scratch_floats(const actqkv_shape& sh, int batch, int k_cap) {
  return size_t(batch) * sh.n_q_heads * decode_mfma_workgroups(sh, batch, k_cap) * (kDcD + 2);
}

int launch_attention_decode_mfma(const actqkv_shape& sh, int batch, const void* q, const void* k_cache,
                                 const void* v_cache, int64_t seq_stride, int nb_capacity,
                                 const int32_t* n_ctx, const int32_t* idx, const int32_t* n_sel,
                                 int k_cap, void* out, float* lse, float* scratch,
                                 unsigned int* counters, float scale, int sel_per_head, hipStream_t stream) {
  DcParams p;
  p.q = static_cast<const uint16_t*>(q);
  p.k_cache = static_cast<const uint16_t*>(k_cache);
  p.v_cache = static_cast<const uint16_t*>(v_cache);
  p.seq_stride = seq_stride;
  p.nb_capacity = nb_capacity;
  p.n_ctx = n_ctx;
  p.idx = idx;
  p.n_sel = n_sel;
  p.sel_per_head = sel_per_head;
  p.k_cap = k_cap;
  p.out = static_cast<uint16_t*>(out);
  p.lse = lse;
  p.part = reinterpret_cast<uint32_t*>(scratch);
  p.counters = counters;
  p.n_q_heads = sh.n_q_heads;
  p.n_kv_heads = sh.n_kv_heads;
  p.n_init = sh.n_init;
  p.n_local = sh.n_local;
  p.n_wg = decode_mfma_workgroups(sh, batch, k_cap);
  p.scale_log2e = scale * 1.4426950408889634f;
  const int group = sh.n_q_heads / sh.n_kv_heads;
  const int n_waves = kDcMaxWaves;
  const size_t lds = size_t(n_waves) * group * (kDcD + 2) * sizeof(float);
  if (p.n_wg > 1 && size_t(batch) * sh.n_kv_heads > kTicketCounters)
    return set_error(ACTQKV_EINVAL, "decode attention: more split (sequence, KV head) pairs than ticket counters");
  hipLaunchKernelGGL(attn_decode_kernel, dim3(p.n_wg, sh.n_kv_heads, batch), dim3(n_waves * 64), lds,
                     stream, p);
  return hip_status("attention (decode)");
}

}  // namespace actqkv
