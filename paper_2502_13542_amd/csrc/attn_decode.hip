// Retrieval attention of a decode step (Sec. 3.1, Eq. (3): one query token per sequence
// over [k^t, K*]; bf16 storage, fp32 accumulation).  HBM-bound: every selected key and
// value byte is read exactly once, by exactly one wavefront.
//
// A wavefront owns work items of 64 keys (half a block) of one (sequence, KV head): initial
// tokens, the blocks chosen by the selection step or the local span up to the new token; the
// keys and the values of an item are requested together, before anything is computed.  The G query heads of the KV head ride along as columns of a 16-wide matrix-core
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
#include <algorithm>
#include <mutex>

#include "append_body.h"
#include "common.h"
#include "launch.h"
#include "score_body.h"
#include "select_body.h"

namespace actqkv {

constexpr int kDcD = 128;
constexpr int kDcMaxWaves = 8;   // 512 threads: the register budget stays at 256 per lane
constexpr int kDcThreads = kDcMaxWaves * 64;
constexpr int kDcItemKeys = 64;  // keys per work item (half a block)
constexpr int kDcSteps = kDcItemKeys / 32, kDcPerTile = kBlock / kDcItemKeys;

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

// What the kernel that selects for itself needs on top (the arguments of the selection step).
struct DcSelectParams {
  const float* scores;
  int64_t score_stride;
  int nb_begin;
  const int32_t* nb_end;
  int entropy_topk;
  SelectIo io;              // io.write is set per workgroup by the kernel
};

__device__ __forceinline__ bf16x8 dc_as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// Keys and values of one work item (kDcItemKeys keys of a tile of one KV head) on their way into
// MFMA operands, and the key positions [lo, hi) of the item that the query may see.
struct DcItem {
  u32x4 ka[8 * kDcSteps];
  u32x4 va[8 * kDcSteps];
  int kpos0, lo, hi;
};
// Running softmax state of a wavefront: lane (n, kq) holds channels 16*dg + 4*kq + i of head n.
struct DcAcc {
  float m_run, l_run;
  f32x4 acc_o[8];
};

// Item `it` of a tile list -> its block and visible span; false if the query sees none of it.
__device__ __forceinline__ bool dc_item_span(const TileList& tl, int it, int& block, int& part, DcItem& r) {
  int lo, hi;
  tl.get(it / kDcPerTile, block, lo, hi);
  part = it % kDcPerTile;
  r.kpos0 = block * kBlock + part * kDcItemKeys;
  r.lo = max(lo, r.kpos0);
  r.hi = min(hi, r.kpos0 + kDcItemKeys);
  return r.hi > r.lo;
}

// Requests the item's keys AND values (nothing is computed before both are on their way).
// A operands of S^T: MFMA row r of sub-tile h of 32-key step st is key 32*st + 8*(r/4) + 4*h + r%4,
// so that lane quarter kq ends up with keys 32*st + 8*kq + 4*h + i in register i.
// V^T A operands: lane (row = channel within a group of 16, kq) reads keys 32*st + 8*kq .. +7.
__device__ __forceinline__ void dc_issue(DcItem& r, const uint16_t* kc, const uint16_t* vc, int block, int part,
                                         int hk, int n_kv_heads, int n, int kq) {
  const size_t tile = (size_t(block) * n_kv_heads + hk) * size_t(kBlock) * kDcD;
  const uint16_t* kbase = kc + tile + size_t(part) * kDcItemKeys * kDcD + size_t(8 * (n >> 2) + (n & 3)) * kDcD + 8 * kq;
  const uint16_t* vbase = vc + tile + part * kDcItemKeys + size_t(n) * kBlock + 8 * kq;
#pragma unroll
  for (int st = 0; st < kDcSteps; ++st)
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
        r.ka[(st * 2 + h) * 4 + ks] =
            *reinterpret_cast<const u32x4*>(kbase + size_t(32 * st + 4 * h) * kDcD + ks * 32);
#pragma unroll
  for (int dg = 0; dg < 8; ++dg)
#pragma unroll
    for (int st = 0; st < kDcSteps; ++st)
      r.va[dg * kDcSteps + st] = *reinterpret_cast<const u32x4*>(vbase + size_t(16 * dg) * kBlock + 32 * st);
}

// Scores, mask, online softmax and O^T += V^T P^T for one item.
__device__ __forceinline__ void dc_consume(const DcItem& r, const bf16x8 (&qb)[4], DcAcc& a, float scale_log2e,
                                           int kq) {
  f32x4 sc[2 * kDcSteps];
#pragma unroll
  for (int j = 0; j < 2 * kDcSteps; ++j) sc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)       // the sub-tiles take turns: no MFMA waits for the one before it
#pragma unroll
    for (int j = 0; j < 2 * kDcSteps; ++j)
      sc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(dc_as_bf16x8(r.ka[j * 4 + ks]), qb[ks], sc[j], 0, 0, 0);
  // mask and online softmax: sc[2*st + h][i] is key kpos0 + 32*st + 8*kq + 4*h + i
  float mx = -INFINITY;
#pragma unroll
  for (int j = 0; j < 2 * kDcSteps; ++j)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int kp = r.kpos0 + 32 * (j >> 1) + 8 * kq + 4 * (j & 1) + i;
      const float v = (kp >= r.lo && kp < r.hi) ? sc[j][i] : -INFINITY;
      sc[j][i] = v;
      mx = fmaxf(mx, v);
    }
  mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
  mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
  const float m_new = fmaxf(a.m_run, mx * scale_log2e);   // finite: the item has a visible key
  const float alpha = __builtin_amdgcn_exp2f(a.m_run - m_new);
  a.m_run = m_new;
  float psum = 0.f;
#pragma unroll
  for (int j = 0; j < 2 * kDcSteps; ++j)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float pv = __builtin_amdgcn_exp2f(sc[j][i] * scale_log2e - m_new);
      sc[j][i] = pv;
      psum += pv;
    }
  psum += __shfl_xor(psum, 16, 64);
  psum += __shfl_xor(psum, 32, 64);
  a.l_run = a.l_run * alpha + psum;
#pragma unroll
  for (int dg = 0; dg < 8; ++dg) a.acc_o[dg] *= alpha;
  typedef __attribute__((ext_vector_type(8))) float f32x8;
#pragma unroll
  for (int st = 0; st < kDcSteps; ++st) {
    f32x8 pf = {sc[2 * st][0], sc[2 * st][1], sc[2 * st][2], sc[2 * st][3],
                sc[2 * st + 1][0], sc[2 * st + 1][1], sc[2 * st + 1][2], sc[2 * st + 1][3]};
    const bf16x8 pb = __builtin_convertvector(pf, bf16x8);
#pragma unroll
    for (int dg = 0; dg < 8; ++dg)
      a.acc_o[dg] =
          __builtin_amdgcn_mfma_f32_16x16x32_bf16(dc_as_bf16x8(r.va[dg * kDcSteps + st]), pb, a.acc_o[dg], 0, 0, 0);
  }
}

// Q^T as B operand: lane (n, kq) holds channels ks*32 + 8*kq .. +7 of head n (zero for n >= G)
__device__ __forceinline__ void dc_load_q(const DcParams& p, int s, int hk, int group, int n, int kq,
                                          bf16x8 (&qb)[4]) {
  const uint16_t* qp = p.q + (size_t(s) * p.n_q_heads + hk * group + min(n, group - 1)) * kDcD + 8 * kq;
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    u32x4 v = *reinterpret_cast<const u32x4*>(qp + ks * 32);
    if (n >= group) v = u32x4{0u, 0u, 0u, 0u};
    qb[ks] = dc_as_bf16x8(v);
  }
}

// The wavefronts of a workgroup merge their (max, sum, O) through LDS.  If one workgroup covers
// the whole (sequence, KV head) it writes the output itself; otherwise the workgroups store
// partials and the one that finishes last merges them.  dc_lds: n_waves * G * (D + 2) floats.
__device__ __forceinline__ void dc_finish(const DcParams& p, const DcAcc& a, float* dc_lds, int s, int hk, int wg,
                                          int group, int n, int kq, int wave, int n_waves) {
  float* red_ml = dc_lds;                        // [n_waves][group][2]
  float* red_o = dc_lds + n_waves * group * 2;   // [n_waves][group][D]
  if (n < group) {
    if (kq == 0) {
      red_ml[(wave * group + n) * 2 + 0] = a.m_run;
      red_ml[(wave * group + n) * 2 + 1] = a.l_run;
    }
#pragma unroll
    for (int dg = 0; dg < 8; ++dg)
      *reinterpret_cast<f32x4*>(&red_o[(wave * group + n) * kDcD + 16 * dg + 4 * kq]) = a.acc_o[dg];
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

// grid (n_wg, Hk, batch); blockDim = 64 * (wavefronts per workgroup).  Item i of the tile list
// of a (sequence, KV head) goes to wavefront i mod (all wavefronts of the pair).
__global__ __launch_bounds__(kDcThreads) void attn_decode_kernel(DcParams p) {
  extern __shared__ __attribute__((aligned(16))) float dc_lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
  const int n = lane & 15, kq = lane >> 4;       // MFMA column (query head) and lane quarter
  const int wg = blockIdx.x, hk = blockIdx.y, s = blockIdx.z;
  const int group = p.n_q_heads / p.n_kv_heads;

  const int n_ctx = min(max(p.n_ctx[s], 1), p.nb_capacity * kBlock);
  const WindowGeom g = window_geom(n_ctx, 1, p.n_init, p.n_local);
  const size_t sel_row = p.sel_per_head ? size_t(s) * p.n_kv_heads + hk : size_t(s);
  const TileList tl = make_tile_list(g, n_ctx - 1, p.idx + sel_row * p.k_cap, p.n_sel[sel_row], p.k_cap,
                                     p.nb_capacity);
  const int n_items = tl.count() * kDcPerTile;
  bf16x8 qb[4];
  dc_load_q(p, s, hk, group, n, kq, qb);
  DcAcc a;
  a.m_run = -INFINITY;
  a.l_run = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) a.acc_o[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  const uint16_t* kc = p.k_cache + size_t(s) * p.seq_stride;
  const uint16_t* vc = p.v_cache + size_t(s) * p.seq_stride;

  for (int it = wg * n_waves + wave; it < n_items; it += p.n_wg * n_waves) {
    DcItem r;
    int block, part;
    if (!dc_item_span(tl, it, block, part, r)) continue;   // wave-uniform
    dc_issue(r, kc, vc, block, part, hk, p.n_kv_heads, n, kq);
    __builtin_amdgcn_sched_barrier(0);   // all key and value loads are in flight before the first MFMA
    dc_consume(r, qb, a, p.scale_log2e, kq);
  }
  dc_finish(p, a, dc_lds, s, hk, wg, group, n, kq, wave, n_waves);
}

// The same attention with the selection step (Sec. 4.2, Eq. (11), Eq. (12); Alg. 1) inside it:
// the step needs a launch of its own only because of its latency (two memory round trips and a
// dozen barriers for 2 KB of scores), and an attention workgroup has exactly that much time to
// spare while its first keys and values are on their way.  Every workgroup of a sequence repeats
// the sequence's selection (same code, same inputs: the same result in all of them) and keeps it
// in LDS; the first workgroup of the sequence also writes it out.  Items that do not depend on
// the selection (initial tokens, local span) come first in the list, so a wavefront's first
// loads go out before the selection starts.
// blockDim = kDcThreads (the selection is written for that many threads).
__global__ __launch_bounds__(kDcThreads) void attn_decode_select_kernel(DcParams p, DcSelectParams sp) {
  extern __shared__ __attribute__((aligned(16))) float dc_lds[];
  __shared__ SelectLds<kDcThreads> sel_lds;
  __shared__ int sel_ready;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  constexpr int n_waves = kDcMaxWaves;
  const int n = lane & 15, kq = lane >> 4;
  const int wg = blockIdx.x, hk = blockIdx.y, s = blockIdx.z;
  const int group = p.n_q_heads / p.n_kv_heads;

  const float* sc_mem = sp.scores + size_t(s) * sp.score_stride + sp.nb_begin;
  const int end = min(max(sp.nb_end[s], sp.nb_begin), p.nb_capacity);   // (no wrap-around in the subtraction)
  const int n_elig = max(end - sp.nb_begin, 0);
  // Rows that fit a wavefront's registers are selected by ONE wavefront, the last of the workgroup,
  // which does that before anything else; the others never meet a barrier on their way to their
  // first item and pick the result up from LDS when they need it.  Longer rows take the selection
  // that is spread over the workgroup.
  const bool by_wave = n_elig <= 64 * kSelWavePerLane;
  const bool selector = by_wave && wave == n_waves - 1;
  if (by_wave) {
    if (threadIdx.x == 0) sel_ready = 0;
    __syncthreads();                     // (nobody has asked the memory for anything yet: all arrive at once)
  }
  SelectIo io = sp.io;
  io.write = wg == 0 && hk == 0;
  if (selector) {
    select_wave(sc_mem, s, n_elig, sp.nb_begin, p.k_cap, sp.entropy_topk, io, sel_lds.sel, &sel_lds.count);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    if (lane == 0) __hip_atomic_store(&sel_ready, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  }
  // the scores of the sequence for the workgroup-wide selection: the load of the first 512 does not wait for anything
  const ScoreRow<kDcThreads> sc{sc_mem, (!by_wave && int(threadIdx.x) < p.nb_capacity - sp.nb_begin) ? sc_mem[threadIdx.x] : 0.f};
  const int n_ctx = min(max(p.n_ctx[s], 1), p.nb_capacity * kBlock);
  const WindowGeom g = window_geom(n_ctx, 1, p.n_init, p.n_local);
  // the list without the selection: initial tokens, then the local span
  const TileList fixed = make_tile_list(g, n_ctx - 1, nullptr, 0, p.k_cap, p.nb_capacity);
  const int n_fixed = fixed.count() * kDcPerTile;
  bf16x8 qb[4];
  dc_load_q(p, s, hk, group, n, kq, qb);
  DcAcc a;
  a.m_run = -INFINITY;
  a.l_run = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) a.acc_o[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  const uint16_t* kc = p.k_cache + size_t(s) * p.seq_stride;
  const uint16_t* vc = p.v_cache + size_t(s) * p.seq_stride;

  // this wavefront's first item, if it is one that does not depend on the selection
  const int it0 = wg * n_waves + wave, stride = p.n_wg * n_waves;
  DcItem r0;
  int block0, part0;
  const bool have0 = it0 < n_fixed && dc_item_span(fixed, it0, block0, part0, r0);
  if (have0) dc_issue(r0, kc, vc, block0, part0, hk, p.n_kv_heads, n, kq);
  __builtin_amdgcn_sched_barrier(0);

  if (!by_wave) select_body<kDcThreads>(sc, s, n_elig, sp.nb_begin, p.k_cap, sp.entropy_topk, io, sel_lds);
  __builtin_amdgcn_sched_barrier(0);
  if (have0) dc_consume(r0, qb, a, p.scale_log2e, kq);
  if (by_wave) {
    // the selector has long finished as a rule; it always does, whatever the others do
    while (__hip_atomic_load(&sel_ready, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) == 0) __builtin_amdgcn_s_sleep(1);
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  }

  // the rest of the list: what is left of the fixed items, then the selected blocks
  TileList chosen = fixed;
  chosen.n_init_tiles = 0;
  chosen.n_tail_tiles = 0;
  chosen.n_sel = min(max(sel_lds.count, 0), p.k_cap);
  chosen.idx = sel_lds.sel;
  const int n_items = n_fixed + chosen.n_sel * kDcPerTile;
  for (int it = it0 < n_fixed ? it0 + stride : it0; it < n_items; it += stride) {
    DcItem r;
    int block, part;
    const bool ok = it < n_fixed ? dc_item_span(fixed, it, block, part, r)
                                 : dc_item_span(chosen, it - n_fixed, block, part, r);
    if (!ok) continue;                   // wave-uniform
    dc_issue(r, kc, vc, block, part, hk, p.n_kv_heads, n, kq);
    __builtin_amdgcn_sched_barrier(0);
    dc_consume(r, qb, a, p.scale_log2e, kq);
  }
  dc_finish(p, a, dc_lds, s, hk, wg, group, n, kq, wave, n_waves);
}

// ---- a whole decode layer in ONE launch ---------------------------------------------------
// Cache update (Sec. 3.1, Eq. (4)), the probe of the one-token window (the query itself,
// Sec. 4.2), block scores (Eq. (10)), density, budget and selection (Eq. (11), Eq. (12),
// Alg. 1) and the attention (Eq. (3)).  The selection of a sequence needs the scores of ALL
// its blocks, which is what a launch boundary used to provide; here the workgroups of a
// sequence share the scoring (block i of the sequence goes to wavefront i mod all its
// wavefronts), publish their scores with write-through stores and a ticket, then stream the
// items of the attention that do not depend on the selection (initial tokens, local span)
// and only afterwards look for the others' scores.  By then these are there as a rule;
// otherwise one thread polls the ticket counter for a bounded time, and a workgroup whose time
// runs out scores the whole sequence for itself (same code, same bits), so every wavefront
// reaches its end whatever the other workgroups do.  Each workgroup then repeats the
// sequence's selection, as attn_decode_select_kernel does, and attends over the chosen blocks.
struct DlParams {
  const uint16_t* k_new;       // [batch][Hk][D], NULL: the cache already holds the step's token
  const uint16_t* v_new;
  uint16_t* k_cache;           // the same caches as DcParams', writable
  uint16_t* v_cache;
  uint16_t* rep_keys;          // [nb_capacity][r][Hk][D] per sequence
  int64_t rep_stride;
  int n_rep;
  float* scores;               // [batch][score_stride], written for the eligible blocks
  unsigned int* seq_counters;  // [batch][2]: workgroups that have published their scores / that have left
  int wait_us;                 // bound of the wait for the other workgroups' scores; 0: do not wait at all
  float inv_sqrt_g;
};

struct LdsScores {
  const float* v;
  __device__ __forceinline__ float operator[](int i) const { return v[i]; }
};

__global__ __launch_bounds__(kDcThreads) void decode_layer_kernel(DcParams p, DcSelectParams sp, DlParams lp) {
  extern __shared__ __attribute__((aligned(16))) float dc_lds[];   // merge area | probe_kv | representatives step | scores
  __shared__ SelectLds<kDcThreads> sel_lds;
  __shared__ float red[32];
  __shared__ int have_all;
  constexpr int V = 8;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int n_waves = kDcMaxWaves;
  const int n = lane & 15, kq = lane >> 4;
  const int wg = blockIdx.x, hk = blockIdx.y, s = blockIdx.z;
  const int group = p.n_q_heads / p.n_kv_heads, key_len = p.n_kv_heads * kDcD;
  const int wgs_per_seq = p.n_wg * p.n_kv_heads, wg_in_seq = hk * p.n_wg + wg;
  const int waves_per_seq = wgs_per_seq * n_waves, wave_in_seq = wg_in_seq * n_waves + wave;
  float* pkv_lds = dc_lds + n_waves * group * (kDcD + 2);
  // (an area of its own for the representatives step, whose last loop has no barrier behind it)
  float* ap_lds = pkv_lds + key_len;
  float* sc_lds = ap_lds + 2 * kBlock;

  const int end = min(max(sp.nb_end[s], sp.nb_begin), p.nb_capacity);
  const int n_elig = max(end - sp.nb_begin, 0);
  const int n_ctx = min(max(p.n_ctx[s], 1), p.nb_capacity * kBlock);
  const WindowGeom g = window_geom(n_ctx, 1, p.n_init, p.n_local);
  const TileList fixed = make_tile_list(g, n_ctx - 1, nullptr, 0, p.k_cap, p.nb_capacity);
  const int n_fixed = fixed.count() * kDcPerTile;

  // ---- the probe: the query summed over the G heads of every KV head, and its norm.  The
  // query loads go out before the key loads (outstanding loads are counted in order).
  const uint16_t* __restrict__ qrow = p.q + size_t(s) * p.n_q_heads * kDcD;
  const int n_chunks = key_len / V;
  auto load_q = [&](int c, int g0, float (&x)[4][V]) {
    const int h = (c * V) / kDcD, dd = c * V - h * kDcD;
#pragma unroll
    for (int i = 0; i < 4; ++i) Vec<uint16_t>::load(qrow + (h * group + min(g0 + i, group - 1)) * kDcD + dd, x[i]);
  };
  float ss = 0.f;
  auto add_q = [&](int g0, const float (&x)[4][V], float (&acc)[V]) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (g0 + i < group) {
#pragma unroll
        for (int v = 0; v < V; ++v) {
          acc[v] += x[i][v];
          ss += x[i][v] * x[i][v];
        }
      }
  };
  float x0[4][V];
  load_q(min(tid, n_chunks - 1), 0, x0);
  bf16x8 qb[4];
  dc_load_q(p, s, hk, group, n, kq, qb);              // Q^T operand of the attention, from the same 8 KB
  __builtin_amdgcn_sched_barrier(0);
  if (tid < n_chunks) {
    float acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = 0.f;
    add_q(0, x0, acc);
    for (int g0 = 4; g0 < group; g0 += 4) {
      float x[4][V];
      load_q(tid, g0, x);
      add_q(g0, x, acc);
    }
#pragma unroll
    for (int v = 0; v < V; ++v) pkv_lds[tid * V + v] = acc[v];
  }
  for (int c = tid + kDcThreads; c < n_chunks; c += kDcThreads) {
    float acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = 0.f;
    for (int g0 = 0; g0 < group; g0 += 4) {
      float x[4][V];
      load_q(c, g0, x);
      add_q(g0, x, acc);
    }
#pragma unroll
    for (int v = 0; v < V; ++v) pkv_lds[c * V + v] = acc[v];
  }
  const float pn = sqrtf(block_sum(ss, red));            // its barriers also publish pkv_lds
  // ---- this wavefront's first four blocks of the sequence, all requested before any is used.  (They
  // go out behind the probe: a wavefront stalls while it issues this many loads, and the barriers
  // of the probe would wait for the slowest one.)
  const uint16_t* rep = lp.rep_keys + size_t(s) * lp.rep_stride;
  const size_t block_elems = size_t(lp.n_rep) * key_len;
  auto block_keys = [&](int i) { return rep + size_t(sp.nb_begin + i) * block_elems; };   // i < n_elig
  BlockScorer<uint16_t> sc0, sc1, sc2, sc3;
  const int i0 = wave_in_seq, i1 = i0 + waves_per_seq, i2 = i1 + waves_per_seq, i3 = i2 + waves_per_seq;
  if (i0 < n_elig) sc0.start(block_keys(i0), lp.n_rep, key_len, lane);   // (wave-uniform conditions)
  if (i1 < n_elig) sc1.start(block_keys(i1), lp.n_rep, key_len, lane);
  if (i2 < n_elig) sc2.start(block_keys(i2), lp.n_rep, key_len, lane);
  if (i3 < n_elig) sc3.start(block_keys(i3), lp.n_rep, key_len, lane);
  __builtin_amdgcn_sched_barrier(0);
  uint32_t* sc_out = reinterpret_cast<uint32_t*>(lp.scores + size_t(s) * sp.score_stride + sp.nb_begin);
  auto finish_block = [&](BlockScorer<uint16_t>& sc, int i) {
    if (i < n_elig) {
      const float v = sc.finish(pkv_lds, pn, lp.inv_sqrt_g);
      if (lane == 0) st_agent(sc_out + i, __float_as_uint(v));
    }
  };
  finish_block(sc0, i0);
  finish_block(sc1, i1);
  finish_block(sc2, i2);
  finish_block(sc3, i3);
  for (int i = i3 + waves_per_seq; i < n_elig; i += 2 * waves_per_seq) {   // longer sequences: two at a time
    sc0.start(block_keys(i), lp.n_rep, key_len, lane);
    if (i + waves_per_seq < n_elig) sc1.start(block_keys(i + waves_per_seq), lp.n_rep, key_len, lane);
    __builtin_amdgcn_sched_barrier(0);
    finish_block(sc0, i);
    finish_block(sc1, i + waves_per_seq);
  }
  // ---- publish: the stores above have been acknowledged, then one ticket per workgroup
  unsigned int* arrived = lp.seq_counters + 2 * s;
  unsigned int* left = arrived + 1;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  if (tid == 0) __hip_atomic_fetch_add(arrived, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

  // ---- the representatives of the block the step's token completes (one workgroup per sequence;
  // reads the older tokens from the cache and the new one from k_new, so it depends on no copy)
  const int pos_new = n_ctx - 1;
  if (lp.k_new != nullptr && wg_in_seq == 0)
    append_body<uint16_t, kDcThreads>(p.n_kv_heads, 0, s, lp.k_new, lp.v_new, pos_new, lp.k_cache, lp.v_cache,
                                      p.seq_stride, lp.rep_keys, lp.rep_stride, p.nb_capacity, 1, p.n_kv_heads,
                                      kDcD, lp.n_rep, reinterpret_cast<unsigned char*>(ap_lds));

  // ---- The wavefront that owns the item holding the step's own token writes that token into the
  // cache (its KV head's key row and value column) and waits for the stores, so that its loads
  // of the item see it; nobody else reads those cache lines in this launch.
  DcAcc a;
  a.m_run = -INFINITY;
  a.l_run = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) a.acc_o[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  const uint16_t* kc = p.k_cache + size_t(s) * p.seq_stride;
  const uint16_t* vc = p.v_cache + size_t(s) * p.seq_stride;
  // item i of the list goes to wavefront i mod (all wavefronts of the pair), wavefront-major across
  // the pair's workgroups, so that every workgroup gets its share of short lists
  const int it0 = wave * p.n_wg + wg, stride = p.n_wg * n_waves;
  // item of the fixed list that holds position pos_new: the last tile of the list, by construction
  const int it_new = (fixed.count() - 1) * kDcPerTile + (pos_new % kBlock) / kDcItemKeys;
  if (lp.k_new != nullptr && it0 == it_new % stride) {
    const int block = pos_new / kBlock, j0 = pos_new - block * kBlock;
    const size_t tile = size_t(s) * p.seq_stride + (size_t(block) * p.n_kv_heads + hk) * size_t(kBlock) * kDcD;
    const uint16_t* kn = lp.k_new + (size_t(s) * p.n_kv_heads + hk) * kDcD;
    const uint16_t* vn = lp.v_new + (size_t(s) * p.n_kv_heads + hk) * kDcD;
    if (lane < kDcD / 8)
      *reinterpret_cast<u32x4*>(lp.k_cache + tile + size_t(j0) * kDcD + 8 * lane) =
          *reinterpret_cast<const u32x4*>(kn + 8 * lane);
#pragma unroll
    for (int r = 0; r < kDcD / 64; ++r) lp.v_cache[tile + size_t(lane + 64 * r) * kBlock + j0] = vn[lane + 64 * r];
    __builtin_amdgcn_s_waitcnt(0);
  }
  __builtin_amdgcn_sched_barrier(0);

  // ---- attention over the items that do not depend on the selection (initial tokens, local span):
  // they stream while the other workgroups' scores and tickets become visible.  (Measured
  // alternatives: requesting these items first and selecting while they are on their way makes
  // the reads of the scores wait behind the items' 32 KB - loads return in order - and a
  // wavefront set aside for those reads still shares the compute unit's load queue with the
  // other seven: both orders were slower than this one.)
  for (int it = it0; it < n_fixed; it += stride) {
    DcItem r;
    int block, part;
    if (!dc_item_span(fixed, it, block, part, r)) continue;   // wave-uniform
    dc_issue(r, kc, vc, block, part, hk, p.n_kv_heads, n, kq);
    __builtin_amdgcn_sched_barrier(0);
    dc_consume(r, qb, a, p.scale_log2e, kq);
  }

  // ---- the sequence's scores: wait (bounded) until every workgroup has published its share
  if (tid == 0) {
    int ok = 0;
    if (lp.wait_us > 0) {
      const uint64_t t_end = wall_clock64() + uint64_t(lp.wait_us) * 100u;   // the counter runs at 100 MHz
      for (;;) {
        ok = __hip_atomic_load(arrived, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= unsigned(wgs_per_seq);
        if (ok || wall_clock64() >= t_end) break;
        __builtin_amdgcn_s_sleep(2);
      }
    }
    have_all = ok;
  }
  __syncthreads();
  if (have_all) {
    for (int i = tid; i < n_elig; i += kDcThreads) sc_lds[i] = __uint_as_float(ld_agent(sc_out + i));
  } else {
    for (int i = wave; i < n_elig; i += n_waves) {        // the whole sequence, by this workgroup alone
      sc0.start(block_keys(i), lp.n_rep, key_len, lane);
      const float v0 = sc0.finish(pkv_lds, pn, lp.inv_sqrt_g);
      if (lane == 0) sc_lds[i] = v0;
    }
  }
  __syncthreads();

  SelectIo io = sp.io;
  io.write = wg_in_seq == 0;
  select_body<kDcThreads>(LdsScores{sc_lds}, s, n_elig, sp.nb_begin, p.k_cap, sp.entropy_topk, io, sel_lds);
  __builtin_amdgcn_sched_barrier(0);

  // ---- the selected blocks
  TileList chosen = fixed;
  chosen.n_init_tiles = 0;
  chosen.n_tail_tiles = 0;
  chosen.n_sel = min(max(sel_lds.count, 0), p.k_cap);
  chosen.idx = sel_lds.sel;
  const int n_items = n_fixed + chosen.n_sel * kDcPerTile;
  int it = it0;
  while (it < n_fixed) it += stride;
  for (; it < n_items; it += stride) {
    DcItem r;
    int block, part;
    if (!dc_item_span(chosen, it - n_fixed, block, part, r)) continue;   // wave-uniform
    dc_issue(r, kc, vc, block, part, hk, p.n_kv_heads, n, kq);
    __builtin_amdgcn_sched_barrier(0);
    dc_consume(r, qb, a, p.scale_log2e, kq);
  }
  dc_finish(p, a, dc_lds, s, hk, wg, group, n, kq, wave, n_waves);

  // ---- the last workgroup of the sequence to get here (nobody polls any more) resets the counters
  if (tid == 0) {
    const unsigned int t = __hip_atomic_fetch_add(left, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (t == unsigned(wgs_per_seq) - 1u) {
      __hip_atomic_store(arrived, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(left, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
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
  const int most = (decode_tiles_max(sh, k_cap) * kDcPerTile + kDcMaxWaves - 1) / kDcMaxWaves;
  return want < 1 ? 1 : (want > most ? most : want);
}

size_t decode_mfma_scratch_floats(const actqkv_shape& sh, int batch, int k_cap) {
  return size_t(batch) * sh.n_q_heads * decode_mfma_workgroups(sh, batch, k_cap) * (kDcD + 2);
}

static DcParams decode_params(const actqkv_shape& sh, int batch, const void* q, const void* k_cache,
                              const void* v_cache, int64_t seq_stride, int nb_capacity, const int32_t* n_ctx,
                              const int32_t* idx, const int32_t* n_sel, int k_cap, void* out, float* lse,
                              float* scratch, unsigned int* counters, float scale, int sel_per_head) {
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
  return p;
}

int launch_attention_decode_mfma(const actqkv_shape& sh, int batch, const void* q, const void* k_cache,
                                 const void* v_cache, int64_t seq_stride, int nb_capacity,
                                 const int32_t* n_ctx, const int32_t* idx, const int32_t* n_sel,
                                 int k_cap, void* out, float* lse, float* scratch,
                                 unsigned int* counters, float scale, int sel_per_head, hipStream_t stream) {
  const DcParams p = decode_params(sh, batch, q, k_cache, v_cache, seq_stride, nb_capacity, n_ctx, idx, n_sel,
                                   k_cap, out, lse, scratch, counters, scale, sel_per_head);
  const int group = sh.n_q_heads / sh.n_kv_heads;
  const size_t lds = size_t(kDcMaxWaves) * group * (kDcD + 2) * sizeof(float);
  if (p.n_wg > 1 && size_t(batch) * sh.n_kv_heads > kTicketCounters)
    return set_error(ACTQKV_EINVAL, "decode attention: more split (sequence, KV head) pairs than ticket counters");
  hipLaunchKernelGGL(attn_decode_kernel, dim3(p.n_wg, sh.n_kv_heads, batch), dim3(kDcThreads), lds, stream, p);
  return hip_status("attention (decode)");
}

int launch_attention_decode_select(const actqkv_shape& sh, int batch, const void* q, const void* k_cache,
                                   const void* v_cache, int64_t seq_stride, int nb_capacity,
                                   const int32_t* n_ctx, const float* scores, int64_t score_stride, int nb_begin,
                                   const int32_t* nb_end, int k_cap, int flags, const float* budget_in,
                                   const float* theta_rest_sum, float* budget_after, int32_t* idx,
                                   int32_t* n_sel, float* theta, float* budget, void* out, float* lse,
                                   float* scratch, unsigned int* counters, float scale, hipStream_t stream) {
  const DcParams p = decode_params(sh, batch, q, k_cache, v_cache, seq_stride, nb_capacity, n_ctx, nullptr,
                                   nullptr, k_cap, out, lse, scratch, counters, scale, 0);
  DcSelectParams sp;
  sp.scores = scores;
  sp.score_stride = score_stride;
  sp.nb_begin = nb_begin;
  sp.nb_end = nb_end;
  sp.entropy_topk = (flags & ACTQKV_SELECT_ENTROPY_TOPK) != 0;
  sp.io = SelectIo{budget_in, theta_rest_sum, budget_after, idx, n_sel, theta, budget, false};
  const int group = sh.n_q_heads / sh.n_kv_heads;
  const size_t lds = size_t(kDcMaxWaves) * group * (kDcD + 2) * sizeof(float);
  if (p.n_wg > 1 && size_t(batch) * sh.n_kv_heads > kTicketCounters)
    return set_error(ACTQKV_EINVAL, "decode attention: more split (sequence, KV head) pairs than ticket counters");
  hipLaunchKernelGGL(attn_decode_select_kernel, dim3(p.n_wg, sh.n_kv_heads, batch), dim3(kDcThreads), lds,
                     stream, p, sp);
  return hip_status("attention with selection (decode)");
}

int launch_decode_layer(const actqkv_shape& sh, int batch, const void* q, const void* k_new, const void* v_new,
                        void* k_cache, void* v_cache, int64_t seq_stride, void* rep_keys, int64_t rep_stride,
                        int nb_capacity, const int32_t* n_ctx, int nb_begin, const int32_t* nb_end, float* scores,
                        int64_t score_stride, int k_cap, int flags, const float* budget_in,
                        const float* theta_rest_sum, float* budget_after, int32_t* idx, int32_t* n_sel,
                        float* theta, float* budget, void* out, float* lse, float* scratch,
                        unsigned int* counters, float scale, int wait_us, hipStream_t stream) {
  const DcParams p = decode_params(sh, batch, q, k_cache, v_cache, seq_stride, nb_capacity, n_ctx, nullptr,
                                   nullptr, k_cap, out, lse, scratch, counters, scale, 0);
  DcSelectParams sp;
  sp.scores = scores;
  sp.score_stride = score_stride;
  sp.nb_begin = nb_begin;
  sp.nb_end = nb_end;
  sp.entropy_topk = (flags & ACTQKV_SELECT_ENTROPY_TOPK) != 0;
  sp.io = SelectIo{budget_in, theta_rest_sum, budget_after, idx, n_sel, theta, budget, false};
  DlParams lp;
  lp.k_new = static_cast<const uint16_t*>(k_new);
  lp.v_new = static_cast<const uint16_t*>(v_new);
  lp.k_cache = static_cast<uint16_t*>(k_cache);
  lp.v_cache = static_cast<uint16_t*>(v_cache);
  lp.rep_keys = static_cast<uint16_t*>(rep_keys);
  lp.rep_stride = rep_stride;
  lp.n_rep = sh.n_rep;
  lp.scores = scores;
  lp.seq_counters = counters + kSeqCounterOffset;
  lp.wait_us = wait_us;
  const int group = sh.n_q_heads / sh.n_kv_heads;
  lp.inv_sqrt_g = 1.f / sqrtf(float(group));
  if (p.n_wg > 1 && size_t(batch) * sh.n_kv_heads > kTicketCounters)
    return set_error(ACTQKV_EINVAL, "decode layer: more split (sequence, KV head) pairs than ticket counters");
  if (2 * size_t(batch) > kSeqCounters)
    return set_error(ACTQKV_ESHAPE, "decode layer: batch %d > %d", batch, int(kSeqCounters / 2));
  // merge area of the wavefronts | group-summed probe | the representatives step | the sequence's scores
  const size_t lds = (size_t(kDcMaxWaves) * group * (kDcD + 2) + size_t(sh.n_kv_heads) * kDcD + 2 * kBlock +
                      size_t(std::max(nb_capacity - nb_begin, 1))) * sizeof(float);
  if (lds > 150 * 1024) return set_error(ACTQKV_ESHAPE, "decode layer: %zu bytes of LDS", lds);
  static std::mutex mu;
  static size_t lds_set = 48 * 1024;
  {
    std::lock_guard<std::mutex> lock(mu);
    if (lds > lds_set) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(decode_layer_kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
      if (e != hipSuccess) return set_error(ACTQKV_EHIP, "hipFuncSetAttribute: %s", hipGetErrorString(e));
      lds_set = 150 * 1024;
    }
  }
  hipLaunchKernelGGL(decode_layer_kernel, dim3(p.n_wg, sh.n_kv_heads, batch), dim3(kDcThreads), lds, stream, p,
                     sp, lp);
  return hip_status("decode layer");
}

}  // namespace actqkv
