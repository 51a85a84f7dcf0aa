// Retrieval attention of a prefill window on the matrix cores
// (Sec. 3.1, Eq. (2): O^t = Attention(Q^t, [K^t, K*], [V^t, V*]); bf16 storage, fp32 accumulation).
//
// Work split.  A workgroup of 8 wavefronts owns 256 query rows that share one KV
// head: all G query heads of the group times 256/G consecutive window positions;
// each wavefront owns 32 rows (one head, 32 positions).  The key tiles of the
// window - initial tokens, the blocks chosen by actqkv_select (read from device
// memory), the local span and the causal part of the window - form one list of
// 128-key blocks; it is cut into `splits` contiguous pieces, one workgroup each,
// so that a 512-token window still fills all 256 compute units; the workgroup that
// finishes last among the pieces of a query tile merges them.  Workgroups of one
// KV head sit on one XCD (blockIdx % Hk picks the head), so that head's gathered
// tiles stay in that XCD's L2.
//
// Data flow per tile.  K [128 keys][D] and V^T [D][128 keys] go from HBM straight into
// LDS (global_load_lds_dwordx4, double buffered, 16-byte chunks XOR-swizzled with the row
// index so that operand reads of 16 consecutive rows hit all 64 banks).  A 16x16x32 tiling
// with one wavefront per SIMD and no key splits was measured and rejected: one wavefront
// can only issue a 1 KB LDS operand read every ~35 cycles, which caps a 16-cycle MFMA per
// read at ~40 % and left that variant at 0.4 PFLOP/s.  Each wavefront computes S^T = K Q^T with
// v_mfma_f32_32x32x16_bf16 (A = K rows from LDS, B = Q^T kept in registers), so a
// lane ends up holding scores of ONE query: the softmax needs no cross-lane work
// except one exchange between the two half-waves, and the probabilities are
// already in the register layout the next product wants as its B operand:
// O^T += V^T P^T (A = V^T rows from LDS).  To make that work the K rows are fed in
// a permuted order (bits 2 and 3 of the row index swapped); the permutation is
// undone for free because a lane's 8 consecutive accumulator registers then hold
// 8 consecutive keys.
#include <algorithm>
#include <mutex>

#include "common.h"
#include "launch.h"

namespace actqkv {

constexpr int kPfThreads = 512;
constexpr int kPfWaves = 8;
constexpr int kPfD = 128;
constexpr int kRowPad = 128;                         // bf16 elements per LDS row (16 chunks of 16 bytes)
constexpr int kTileElems = kBlock * kRowPad;         // one K or V^T tile in LDS
constexpr int kPfMaxTiles = 96;                      // initial + selected (<= 64) + local + window
constexpr int kPfLdsBytes = 2 * 2 * kTileElems * 2 + kPfMaxTiles * 12;  // 2 stages x (K, V^T) + tile table
constexpr int kPfPartWords = 17;                     // 64-bit words per lane: 16 x 4 bf16 + (max, sum)
constexpr int kMaxPfSplits = 8;
constexpr float kLazyMaxLog2 = 8.f;                  // how far a tile's maximum may exceed the reference one
constexpr int kPfOrderMax = 64;                      // batch entries the queue hands out longest first
constexpr int kPfQueueDone = 128;                    // index of the "left" counter behind the per-head queue counters

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// sum += the eight bf16 values of a packed operand (as fp32): four dot products of a pair with
// (1, 1).  (Written as assembly: the compiler's builtin for this instruction takes the first
// pair of a packed vector whatever element is asked for.)
__device__ __forceinline__ void add_bf16x8(float& sum, bf16x8 v, uint32_t ones) {
  const u32x4 w = __builtin_bit_cast(u32x4, v);
  asm("v_dot2c_f32_bf16 %0, %1, %2" : "+v"(sum) : "v"(w.x), "v"(ones));
  asm("v_dot2c_f32_bf16 %0, %1, %2" : "+v"(sum) : "v"(w.y), "v"(ones));
  asm("v_dot2c_f32_bf16 %0, %1, %2" : "+v"(sum) : "v"(w.z), "v"(ones));
  asm("v_dot2c_f32_bf16 %0, %1, %2" : "+v"(sum) : "v"(w.w), "v"(ones));
}

// 8 fp32 -> 8 bf16 (round to nearest even), packed as an MFMA operand
__device__ __forceinline__ bf16x8 pack8(float a0, float a1, float a2, float a3, float a4, float a5,
                                        float a6, float a7) {
  typedef __attribute__((ext_vector_type(8))) float f32x8;
  f32x8 v = {a0, a1, a2, a3, a4, a5, a6, a7};
  return __builtin_convertvector(v, bf16x8);
}

// A pointer that is the same in all lanes, pinned to scalar registers (so that adding a
// 32-bit lane offset to it becomes the scalar-base addressing mode of the load).
__device__ __forceinline__ const char* uniform_ptr(const char* ptr) {
  const uint64_t v = reinterpret_cast<uint64_t>(ptr);
  const uint32_t lo = __builtin_amdgcn_readfirstlane(uint32_t(v));
  const uint32_t hi = __builtin_amdgcn_readfirstlane(uint32_t(v >> 32));
  return reinterpret_cast<const char*>((uint64_t(hi) << 32) | lo);
}

__host__ __device__ __forceinline__ int padded_group(int g) { return g <= 1 ? 1 : (g <= 2 ? 2 : (g <= 4 ? 4 : 8)); }

// MFMA row -> key row inside a 32-key group: swap bits 2 and 3.
__device__ __forceinline__ int perm_row(int i) {
  return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1);
}

struct PfParams {
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
  uint64_t* part;          // [workgroup][split][wave][16 x 4 bf16 + (max, sum)][64 lanes]
  unsigned int* counters;  // one ticket counter per (sequence, query tile, KV head), zero between launches
  int m, n_q_heads, n_kv_heads, n_init, n_local;
  int s_lo, rem, slots, n_qtiles;   // pieces per query tile (PfSplits)
  int items_per_head, wgs_per_head; // work items and (first-team) workgroups of one KV head
  int team_total;                   // workgroups of both teams together (the last one to leave resets the queue)
  int late;                         // 1: this launch is the second team, which only draws from the queue
  int sel_per_head;                 // 1: idx and n_sel have a row per (sequence, KV head), 0: per sequence
  unsigned int* queue;              // per KV head: items handed out beyond the first round; [kPfQueueDone]: workgroups that left
  float scale_log2e;
};

// Final normalisation and store of one lane's share of a query row:
// acc_o[db][4j + r] is channel d = db*32 + 8j + 4*half + r.
__device__ __forceinline__ void store_rows(const PfParams& p, const f32x16 (&acc_o)[4], float m_run,
                                           float l_tot, int s, int my_row, int head, int half) {
  const size_t grow = (size_t(s) * p.m + my_row) * p.n_q_heads + head;
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  uint16_t* op = p.out + grow * kPfD;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      u32x2 v;
      v.x = pack_bf16x2(acc_o[db][4 * j + 0] * inv, acc_o[db][4 * j + 1] * inv);
      v.y = pack_bf16x2(acc_o[db][4 * j + 2] * inv, acc_o[db][4 * j + 3] * inv);
      *reinterpret_cast<u32x2*>(op + db * 32 + 8 * j + 4 * half) = v;
    }
  if (p.lse != nullptr && half == 0)
    p.lse[(size_t(s) * p.n_q_heads + head) * p.m + my_row] = (m_run + log2f(l_tot)) * 0.6931471805599453f;
}

// One work item: piece `slot` of the query tiles of (sequence s, KV head hk).
template <bool kInLoop>
__device__ __forceinline__ void attn_prefill_item(const PfParams& p, uint16_t* lds, int hk, int slot, int s) {
  // (inside an item loop the thread index is made opaque, so that nothing derived from it is
  // hoisted out of the loop and kept in registers across the whole item)
  int tid = threadIdx.x;
  if (kInLoop) asm volatile("" : "+v"(tid));
  const int lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, half = lane >> 5;
  const int group = p.n_q_heads / p.n_kv_heads;
  // a group size that does not divide 8 (7 heads per KV head, say) is rounded up to the next
  // power of two: the surplus wavefronts help to fetch tiles and otherwise idle
  const int waves_per_head = kPfWaves / padded_group(group);
  const int pos_per_wg = 32 * waves_per_head;

  // The slots of a (sequence, KV head) are the pieces of its query tiles, in order.
  const int n_lo = p.n_qtiles - p.rem;
  int qtile, split, splits;
  if (slot < n_lo * p.s_lo) {
    qtile = slot / p.s_lo;
    split = slot - qtile * p.s_lo;
    splits = p.s_lo;
  } else {
    const int r = slot - n_lo * p.s_lo;
    splits = p.s_lo + 1;
    qtile = n_lo + r / splits;
    split = r - (qtile - n_lo) * splits;
  }

  // the selected block indices are requested together with the two scalars they are used
  // with, not after them (one memory round trip less before the first tile can be fetched)
  __shared__ int32_t idx_lds[64];
  const size_t sel_row = p.sel_per_head ? size_t(s) * p.n_kv_heads + hk : size_t(s);
  const int32_t my_idx = tid < p.k_cap ? p.idx[sel_row * p.k_cap + tid] : -1;
  const int n_ctx_raw = p.n_ctx[s], n_sel_raw = p.n_sel[sel_row];
  if (tid < 64) idx_lds[tid] = my_idx;
  __syncthreads();
  const int n_ctx = min(max(n_ctx_raw, p.m), p.nb_capacity * kBlock);
  const WindowGeom g = window_geom(n_ctx, p.m, p.n_init, p.n_local);
  const int row0 = qtile * pos_per_wg;                       // first window row of the workgroup
  const int row_hi = min(row0 + pos_per_wg, p.m) - 1;
  const TileList tl = make_tile_list(g, g.w0 + row_hi, idx_lds, n_sel_raw, p.k_cap, p.nb_capacity);
  const int n_tiles = tl.count();
  const int per = (n_tiles + splits - 1) / splits;
  const int t_begin = split * per, t_end = min(n_tiles, t_begin + per);

  const int head_in_group = wave / waves_per_head;
  const bool head_ok = head_in_group < group;
  const int head = hk * group + min(head_in_group, group - 1);
  const int wrow0 = row0 + (wave % waves_per_head) * 32;     // first window row of this wavefront
  const int my_row = wrow0 + n;
  const bool row_ok = my_row < p.m && head_ok;
  const int my_pos = g.w0 + my_row;                          // this lane's query position

  // Q^T as B operand: lane (n, half) holds d = ks*16 + 8*half .. +7 of query row n.  (Folding
  // scale * log2(e) into these operands, rounded to bf16 again, and starting the score
  // accumulators at minus the reference maximum would spare the multiply-add per score, but the
  // second rounding of the queries moves large logits by 2^-9 of their size: 2 % output error on
  // heavy-tailed inputs.)
  bf16x8 qreg[kPfD / 16];
  {
    const int r = min(my_row, p.m - 1);
    const uint16_t* qp = p.q + ((size_t(s) * p.m + r) * p.n_q_heads + head) * kPfD + 8 * half;
#pragma unroll
    for (int ks = 0; ks < kPfD / 16; ++ks)
      qreg[ks] = as_bf16x8(*reinterpret_cast<const u32x4*>(qp + ks * 16));
  }

  f32x16 acc_o[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc_o[i][j] = 0.f;
  float m_run = -INFINITY;                // running max (log2 units)
  const uint32_t bf16_ones = 0x3f803f80u;

  const char* kc = reinterpret_cast<const char*>(p.k_cache + size_t(s) * p.seq_stride);
  const char* vc = reinterpret_cast<const char*>(p.v_cache + size_t(s) * p.seq_stride);
  constexpr uint32_t kTileBytes = kBlock * kPfD * 2;     // one (block, KV head) tile in HBM
  constexpr uint32_t kSlotBytes = kTileElems * 2;        // one tile in LDS
  char* lds_b = reinterpret_cast<char*>(lds);
  // LDS: stage s holds K at (2s) * kSlotBytes and V^T at (2s + 1) * kSlotBytes; behind the
  // stages sits the table {block, lo, hi} of this workgroup's tiles (the selected indices
  // are read from global memory once, not once per use).
  int* tile_tab = reinterpret_cast<int*>(lds_b + 4 * kSlotBytes);
  for (int i = tid; i < t_end - t_begin; i += kPfThreads) {
    int block, lo, hi;
    tl.get(t_begin + i, block, lo, hi);
    tile_tab[3 * i + 0] = block;
    tile_tab[3 * i + 1] = lo;
    tile_tab[3 * i + 2] = hi;
  }
  __syncthreads();

  // Tiles go from HBM straight into LDS (global_load_lds_dwordx4: lane i of a wavefront
  // fills the i-th 16-byte chunk of a contiguous 1 KB piece of LDS, i.e. 4 rows; no staging
  // registers, no ds_write).  Wavefront w fills rows 16*w .. 16*w + 15 of a K and of a V^T
  // tile with 4 such loads each.  The 16 chunks of an LDS row are XOR-swizzled with
  // (row % 16), so that the 16 rows an MFMA operand load touches hit all 64 banks; the
  // swizzle is applied on the global side: the lane that fills chunk c' of row r fetches
  // chunk c' ^ (r % 16) of that row.
  const int lq = lane >> 4, c16 = lane & 15;
  const uint32_t g_row = uint32_t(16 * wave + lq) * (kPfD * 2);          // + 4*i rows per load
  const uint32_t g_chunk = uint32_t(c16 ^ lq) << 4;                      // ^ (i << 6)
  // per-lane byte offsets inside a tile, one per load; the tile's base and the LDS
  // destination are the same for all lanes and stay in scalar registers
  uint32_t go[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) go[i] = g_row + i * 4 * (kPfD * 2) + (g_chunk ^ (uint32_t(i) << 6));
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  auto fetch_tile = [&](int u, int stage) {
    const int block = __builtin_amdgcn_readfirstlane(tile_tab[3 * u]);
    const size_t off = (size_t(block) * p.n_kv_heads + hk) * kTileBytes;
    const char* kt = uniform_ptr(kc + off);
    const char* vt = uniform_ptr(vc + off);
    char* dst = lds_b + stage * 2 * kSlotBytes + wave_s * (16 * kRowPad * 2);
    const __amdgpu_buffer_rsrc_t kr = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(kt), 0, kTileBytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t vr = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(vt), 0, kTileBytes, 0x00020000);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      __builtin_amdgcn_raw_ptr_buffer_load_lds(kr, (__attribute__((address_space(3))) void*)(dst + i * 4 * (kRowPad * 2)), 16, go[i], 0, 0, 0);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(vr, (__attribute__((address_space(3))) void*)(dst + kSlotBytes + i * 4 * (kRowPad * 2)), 16, go[i], 0, 0, 0);
    }
  };

  if (t_begin < t_end) fetch_tile(0, 0);
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();

  const int a_row = perm_row(n);
  // Byte offsets of this lane's MFMA A operands inside a K / V^T slot.  K: row perm(n), chunk
  // 2*ks + half, swizzle key perm(n) % 16; V^T: row n, chunk c = 4*kb + 2*s2 + half, swizzle
  // key n % 16.  A row is 256 bytes, so the offset of chunk pair c is that of pair 0 with
  // c << 5 XOR-ed in: one register per operand kind and one XOR per read, instead of eight
  // registers each.  The 32-row blocks (kb, db) add a compile-time constant.
  uint32_t a_off0 = uint32_t(a_row) * (kRowPad * 2) + (uint32_t(half ^ (a_row & 15)) << 4);
  uint32_t v_off0 = uint32_t(n) * (kRowPad * 2) + (uint32_t(half ^ (n & 15)) << 4);
  float l_run = 0.f;                           // this lane's share of the running sum of its query row
  for (int t = t_begin; t < t_end; ++t) {
    const int u = t - t_begin, stage = u & 1;
    // (opaque per iteration: the XOR-ed offsets are recomputed, not kept across the loop)
    asm volatile("" : "+v"(a_off0), "+v"(v_off0));

    const int block = __builtin_amdgcn_readfirstlane(tile_tab[3 * u]);
    const int lo = __builtin_amdgcn_readfirstlane(tile_tab[3 * u + 1]);
    const int hi = __builtin_amdgcn_readfirstlane(tile_tab[3 * u + 2]);
    const int kpos0 = block * kBlock;
    // the wavefront skips tiles none of its rows can see; it masks tiles that are
    // clipped or that reach past its first row's position
    const bool visible = head_ok && hi > lo && lo <= g.w0 + min(wrow0 + 31, p.m - 1);
    const bool masked = lo > kpos0 || hi < kpos0 + kBlock || hi - 1 > g.w0 + wrow0;
    const char* ks_ = lds_b + stage * 2 * kSlotBytes;
    const char* vs_ = ks_ + kSlotBytes;
    f32x16 acc_s[4];
    if (visible) {
      // ---- S^T = K Q^T : 4 groups of 32 keys
      const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      // the four key groups take turns, so that an MFMA never waits for the one just before it
      // (a dependent 32x32x16 MFMA issues only about 90 cycles after its producer, an
      // independent one after 32)
      // (written in the order it should issue: a ring of 8 operands, each read 8 MFMAs ahead)
      auto k_read = [&](int i) {
        return *reinterpret_cast<const u32x4*>(ks_ + (a_off0 ^ (uint32_t(i >> 2) << 5)) + (i & 3) * 32 * (kRowPad * 2));
      };
      u32x4 ring[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) ring[i] = k_read(i);
#pragma unroll
      for (int i = 0; i < 32; ++i) {
        const int ks = i >> 2, kb = i & 3;
        acc_s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(ring[i & 7]), qreg[ks], ks == 0 ? zero16 : acc_s[kb], 0, 0, 0);
        if (i + 8 < 32) ring[i & 7] = k_read(i + 8);
      }
      // issue order: 8 operand reads ahead of the first MFMA, then one read per MFMA, so that an
      // operand is requested about 8 MFMAs before it is needed (0x100 = LDS read, 0x008 = MFMA)
      __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
      for (int i = 0; i < 24; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    // The next tile is requested here, after the score MFMAs and not at the top of the
    // iteration: while an LDS-direct load (a FLAT-encoded instruction) is in flight the
    // compiler must treat LDS operations as completing out of order and waits for ALL
    // outstanding operand reads before each use, which stalled the score phase every 8 MFMAs.
    // It still has the softmax and the value phase of this tile to land.
    if (t + 1 < t_end) fetch_tile(u + 1, stage ^ 1);
    if (visible) {
      // register i of group kb holds key kpos0 + kb*32 + 16*(i/8) + 8*half + (i%8)
      if (masked) {
#pragma unroll
        for (int kb = 0; kb < 4; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int kp = kpos0 + kb * 32 + 16 * (i >> 3) + 8 * half + (i & 7);
            const bool ok = kp >= lo && kp < hi && kp <= my_pos;
            acc_s[kb][i] = ok ? acc_s[kb][i] : -INFINITY;
          }
      }
      // ---- online softmax, one query per lane (two lanes share a query: n and n+32)
      // the first V^T operands are requested now and land during the max reduction;
      // operand j = 4 * (2*kb + s2) + db belongs to keys kb*32 + s2*16 .. +15, rows db*32 .. +31
      auto v_read = [&](int j) {
        return *reinterpret_cast<const u32x4*>(vs_ + (v_off0 ^ (uint32_t(j >> 2) << 5)) + (j & 3) * 32 * (kRowPad * 2));
      };
      u32x4 vring[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) vring[i] = v_read(i);
      float mx = acc_s[0][0];
#pragma unroll
      for (int kb = 0; kb < 4; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) mx = fmaxf(mx, acc_s[kb][i]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      // the reference maximum follows the true one lazily: it moves only when a tile exceeds
      // it by more than 2^8, so the rescaling of the accumulators below is rare after the first
      // tiles; probabilities up to 2^8 are as exact in bf16 and fp32 as those up to 1
      const float m_tile = mx * p.scale_log2e;
      const float m_new = m_tile - m_run > kLazyMaxLog2 ? m_tile : m_run;
      const float m_safe = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
      m_run = m_new;
      if (!__all(alpha == 1.f)) {
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
          for (int i = 0; i < 16; ++i) acc_o[db][i] *= alpha;
        l_run *= alpha;
      }
#pragma unroll
      for (int i = 0; i < 16; ++i) acc_s[0][i] = __builtin_amdgcn_exp2f(acc_s[0][i] * p.scale_log2e - m_safe);
      __builtin_amdgcn_sched_barrier(0);
      // ---- O^T += V^T P^T.  Written in issue order: the exponentials of the next 32 keys sit
      // between the MFMAs of these 32 (the vector ALU works while the matrix pipe does), and every
      // V^T operand is read 8 MFMAs ahead.  The row sums add the bf16 probabilities the product
      // itself uses, a pair per instruction, each lane summing its own 64 keys of the tile.
#pragma unroll
      for (int g8 = 0; g8 < 8; ++g8) {
        const int kb = g8 >> 1, s2 = g8 & 1;
        const bf16x8 pb = pack8(acc_s[kb][8 * s2 + 0], acc_s[kb][8 * s2 + 1], acc_s[kb][8 * s2 + 2],
                                acc_s[kb][8 * s2 + 3], acc_s[kb][8 * s2 + 4], acc_s[kb][8 * s2 + 5],
                                acc_s[kb][8 * s2 + 6], acc_s[kb][8 * s2 + 7]);
        add_bf16x8(l_run, pb, bf16_ones);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          if (kb < 3) {
#pragma unroll
            for (int i = 8 * s2 + 2 * db; i < 8 * s2 + 2 * db + 2; ++i)
              acc_s[kb + 1][i] = __builtin_amdgcn_exp2f(acc_s[kb + 1][i] * p.scale_log2e - m_safe);
          }
          __builtin_amdgcn_sched_barrier(0);
          const int j = 4 * g8 + db;
          acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(vring[j & 7]), pb, acc_o[db], 0, 0, 0);
          if (j + 8 < 32) vring[j & 7] = v_read(j + 8);
        }
      }
    }
    __builtin_amdgcn_s_waitcnt(0);   // this wavefront's pieces of the next tile have landed in LDS
    __syncthreads();
  }

  // ---- epilogue
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (splits == 1) {
    if (row_ok) store_rows(p, acc_o, m_run, l_tot, s, my_row, head, half);
    return;
  }
  // The split stores its normalised output as bf16 in the order the registers hold it
  // (register-major, lane-minor: every store instruction writes one contiguous 512-byte
  // row), plus its running max and sum.
  __shared__ int last_flag;
  const size_t group_id = (size_t(s) * p.n_qtiles + qtile) * p.n_kv_heads + hk;
  uint64_t* group_part = p.part + ((size_t(s) * p.n_kv_heads + hk) * p.slots + (slot - split)) *
                                      (kPfWaves * (kPfPartWords * 64));
  {
    uint64_t* mine = group_part + (size_t(split) * kPfWaves + wave) * (kPfPartWords * 64);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t lo = pack_bf16x2(acc_o[db][4 * i] * inv, acc_o[db][4 * i + 1] * inv);
        const uint32_t hi = pack_bf16x2(acc_o[db][4 * i + 2] * inv, acc_o[db][4 * i + 3] * inv);
        st_agent(mine + (db * 4 + i) * 64 + lane, uint64_t(lo) | (uint64_t(hi) << 32));
      }
    st_agent(mine + 16 * 64 + lane, uint64_t(__float_as_uint(m_run)) | (uint64_t(__float_as_uint(l_tot)) << 32));
  }
  if (!last_of_group(p.counters + group_id, unsigned(splits), &last_flag)) return;

  // ---- the last split of the query tile merges all of them, in split order:
  //   out = sum_s w_s o_s / sum_s w_s with w_s = l_s 2^(m_s - M), M = max_s m_s
  // (its own piece is read back like the others, so the result does not depend on who is last)
  const uint64_t* piece0 = group_part + size_t(wave) * (kPfPartWords * 64) + lane;
  const size_t piece_stride = size_t(kPfWaves) * (kPfPartWords * 64);
  // the loads of the first pieces go out together with the (max, sum) words of all pieces
  constexpr int kMergeBatch = 3;
  uint64_t ml[kMaxPfSplits], raw[kMergeBatch][16];
#pragma unroll
  for (int s2 = 0; s2 < kMaxPfSplits; ++s2)
    ml[s2] = s2 < splits ? ld_agent(piece0 + s2 * piece_stride + 16 * 64) : 0;
#pragma unroll
  for (int j = 0; j < kMergeBatch; ++j)
#pragma unroll
    for (int k = 0; k < 16; ++k) raw[j][k] = j < splits ? ld_agent(piece0 + j * piece_stride + k * 64) : 0;
  __builtin_amdgcn_sched_barrier(0);
  float w_s[kMaxPfSplits + kMergeBatch];
  float m_all = -INFINITY;
#pragma unroll
  for (int s2 = 0; s2 < kMaxPfSplits; ++s2)
    if (s2 < splits) m_all = fmaxf(m_all, __uint_as_float(uint32_t(ml[s2])));
  const float m_safe = m_all == -INFINITY ? 0.f : m_all;
#pragma unroll
  for (int s2 = 0; s2 < kMaxPfSplits + kMergeBatch; ++s2)
    w_s[s2] = s2 < splits ? __uint_as_float(uint32_t(ml[s2 < kMaxPfSplits ? s2 : 0] >> 32)) *
                                  __builtin_amdgcn_exp2f(__uint_as_float(uint32_t(ml[s2 < kMaxPfSplits ? s2 : 0])) - m_safe)
                            : 0.f;
  float l_all = 0.f;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc_o[db][i] = 0.f;
#pragma unroll
  for (int b0 = 0; b0 < kMaxPfSplits; b0 += kMergeBatch) {
    if (b0 < splits) {
      if (b0 > 0) {
#pragma unroll
        for (int j = 0; j < kMergeBatch; ++j)
#pragma unroll
          for (int k = 0; k < 16; ++k)
            raw[j][k] = b0 + j < splits ? ld_agent(piece0 + (b0 + j) * piece_stride + k * 64) : 0;
      }
#pragma unroll
      for (int j = 0; j < kMergeBatch; ++j) {
        const float w = w_s[b0 + j];
        l_all += w;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const uint32_t lo = uint32_t(raw[j][db * 4 + i]), hi = uint32_t(raw[j][db * 4 + i] >> 32);
            acc_o[db][4 * i + 0] += w * bf16_lo(lo);
            acc_o[db][4 * i + 1] += w * bf16_hi(lo);
            acc_o[db][4 * i + 2] += w * bf16_lo(hi);
            acc_o[db][4 * i + 3] += w * bf16_hi(hi);
          }
      }
    }
  }
  if (row_ok) store_rows(p, acc_o, m_all, l_all, s, my_row, head, half);
}

// blockIdx.x = w * Hk + hk: consecutive ids differ in hk, and ids are dealt round-robin to the
// XCDs, so each XCD serves few KV heads and that head's tiles stay in its L2.  The items of a
// KV head are its (sequence, slot) pairs.  If there are no more of them than workgroups, each
// workgroup takes one.  Otherwise (several windows in one call, fewer compute units than
// items) the workgroups of a head draw the remaining items from a counter: windows differ in
// how many blocks they retrieve, and a fixed assignment would wait for the unluckiest
// workgroup.  Nobody waits for anybody: a workgroup leaves when the counter runs out, and the
// last one to leave puts the counters back to zero for the next launch.
__global__ __launch_bounds__(kPfThreads) void attn_prefill_mfma_kernel(PfParams p) {
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  const int item = blockIdx.x / p.n_kv_heads, s = item / p.slots;
  attn_prefill_item<false>(p, lds, blockIdx.x % p.n_kv_heads, item - s * p.slots, s);
}

__global__ __launch_bounds__(kPfThreads) void attn_prefill_mfma_queued_kernel(PfParams p) {
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  __shared__ int next_item;
  const int hk = blockIdx.x % p.n_kv_heads;
  auto draw = [&]() {
    if (threadIdx.x == 0)
      next_item = p.wgs_per_head + int(__hip_atomic_fetch_add(p.queue + hk, 1u, __ATOMIC_RELAXED,
                                                              __HIP_MEMORY_SCOPE_AGENT));
    __syncthreads();
    return next_item;
  };
  // Longest items first, so that the launch does not end with a few workgroups on long items
  // while the others have left: the batch entries in descending order of the number of blocks
  // they retrieve (ties: ascending index), and within an entry the later query tiles, which see
  // more of the window, before the earlier ones.
  __shared__ int order[kPfOrderMax];
  const int batch = p.items_per_head / p.slots;
  const bool sorted = batch <= kPfOrderMax;
  if (sorted) {
    const int t = threadIdx.x;
    if (t < batch) {
      const size_t stride = p.sel_per_head ? p.n_kv_heads : 1, off = p.sel_per_head ? hk : 0;
      const int mine = p.n_sel[size_t(t) * stride + off];
      int rank = 0;
      for (int j = 0; j < batch; ++j) {
        const int other = p.n_sel[size_t(j) * stride + off];
        rank += (other > mine) || (other == mine && j < t);
      }
      order[rank] = t;
    }
    __syncthreads();
  }
  // A second team of workgroups (a launch of its own, on compute units that were busy with
  // something else when the first team started) has no first-round items: it only draws.
  int item = p.late ? draw() : int(blockIdx.x) / p.n_kv_heads;
  while (item < p.items_per_head) {
    int s = item / p.slots, slot = item - s * p.slots;
    if (sorted) {
      s = order[s];
      slot = p.slots - 1 - slot;
    }
    attn_prefill_item<true>(p, lds, hk, slot, s);
    __syncthreads();                         // everybody is done with the LDS tiles of this item
    item = draw();
  }
  if (threadIdx.x == 0) {
    unsigned int* done = p.queue + kPfQueueDone;
    const unsigned int t = __hip_atomic_fetch_add(done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (t == unsigned(p.team_total) - 1u) {
      for (int h = 0; h < p.n_kv_heads; ++h)
        __hip_atomic_store(p.queue + h, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(done, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

bool prefill_mfma_supported(const actqkv_shape& sh, int m) {
  const int g = sh.n_q_heads / sh.n_kv_heads;
  // longest possible tile list: initial + selected + local + window (+ 2 partial blocks)
  const int tiles = sh.n_init / kBlock + 64 + sh.n_local / kBlock + (m + kBlock - 1) / kBlock + 2;
  return sh.dtype == ACTQKV_BF16 && sh.head_dim == kPfD && m > 1 && g <= 8 && tiles <= kPfMaxTiles;
}

int prefill_mfma_qtiles(const actqkv_shape& sh, int m) {
  const int g = sh.n_q_heads / sh.n_kv_heads;
  const int pos_per_wg = 32 * (kPfWaves / padded_group(g));
  return (m + pos_per_wg - 1) / pos_per_wg;
}

// workgroups per (sequence, split): query tiles x KV heads
int prefill_mfma_workgroups(const actqkv_shape& sh, int m) {
  return prefill_mfma_qtiles(sh, m) * sh.n_kv_heads;
}

// hipFuncSetAttribute once per process, from whichever thread comes first
static int prefill_lds_attribute() {
  static std::mutex mu;
  static bool attr_set = false;
  std::lock_guard<std::mutex> lock(mu);
  if (attr_set) return ACTQKV_OK;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_prefill_mfma_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, kPfLdsBytes);
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_prefill_mfma_queued_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kPfLdsBytes);
  if (e != hipSuccess) return set_error(ACTQKV_EHIP, "hipFuncSetAttribute: %s", hipGetErrorString(e));
  attr_set = true;
  return ACTQKV_OK;
}

// first_cus: compute units the first team may fill (the pieces in `splits` were chosen for it);
// late_cus > 0: a second team of that many workgroups is launched on stream_late by the same
// call, so that the two launches can never disagree about the queue they share.
int launch_attention_prefill_mfma(const actqkv_shape& sh, int batch, int m, const void* q,
                                  const void* k_cache, const void* v_cache, int64_t seq_stride,
                                  int nb_capacity, const int32_t* n_ctx, const int32_t* idx,
                                  const int32_t* n_sel, int k_cap, void* out, float* lse,
                                  const PfSplits& splits, float* scratch, unsigned int* counters,
                                  float scale, int sel_per_head, int first_cus, int late_cus,
                                  hipStream_t stream, hipStream_t stream_late) {
  if (int rc = prefill_lds_attribute()) return rc;
  PfParams p;
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
  p.part = reinterpret_cast<uint64_t*>(scratch);
  p.counters = counters;
  p.m = m;
  p.n_q_heads = sh.n_q_heads;
  p.n_kv_heads = sh.n_kv_heads;
  p.n_init = sh.n_init;
  p.n_local = sh.n_local;
  p.s_lo = splits.s_lo;
  p.rem = splits.rem;
  p.slots = splits.slots;
  p.n_qtiles = prefill_mfma_qtiles(sh, m);
  p.scale_log2e = scale * 1.4426950408889634f;
  if (splits.slots < p.n_qtiles || splits.slots != splits.s_lo * p.n_qtiles + splits.rem)
    return set_error(ACTQKV_EINVAL, "prefill attention: inconsistent split of the key tiles");
  if (splits.slots > p.n_qtiles && size_t(batch) * p.n_qtiles * sh.n_kv_heads > kTicketCounters)
    return set_error(ACTQKV_EINVAL, "prefill attention: more split query tiles than ticket counters");
  if (sh.n_kv_heads > kPfQueueDone)
    return set_error(ACTQKV_ESHAPE, "prefill attention: more than %d KV heads", kPfQueueDone);
  p.items_per_head = splits.slots * batch;
  p.wgs_per_head = std::min(p.items_per_head, std::max(1, first_cus / sh.n_kv_heads));
  p.queue = counters + kTicketCounters;
  int late_per_head = late_cus / sh.n_kv_heads;
  if (p.items_per_head <= p.wgs_per_head) late_per_head = 0;   // a workgroup per item: no queue, no second team
  p.team_total = (p.wgs_per_head + late_per_head) * sh.n_kv_heads;
  p.late = 0;
  dim3 grid(p.wgs_per_head * sh.n_kv_heads);
  if (p.items_per_head > p.wgs_per_head)
    hipLaunchKernelGGL(attn_prefill_mfma_queued_kernel, grid, dim3(kPfThreads), kPfLdsBytes, stream, p);
  else
    hipLaunchKernelGGL(attn_prefill_mfma_kernel, grid, dim3(kPfThreads), kPfLdsBytes, stream, p);
  if (int rc = hip_status("attention (prefill, matrix cores)")) return rc;
  if (late_per_head > 0) {
    p.late = 1;
    hipLaunchKernelGGL(attn_prefill_mfma_queued_kernel, dim3(late_per_head * sh.n_kv_heads), dim3(kPfThreads),
                       kPfLdsBytes, stream_late, p);
    // (if this launch fails after the first one went out, the first team still does all the work, but
    // the queue is not put back to zero: the workspace must be zero-filled again before its next use)
    if (int rc = hip_status("attention (prefill, matrix cores, second team)")) return rc;
  }
  return ACTQKV_OK;
}

}  // namespace actqkv
