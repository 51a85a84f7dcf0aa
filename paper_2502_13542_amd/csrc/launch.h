// Host-side plumbing shared by the C ABI and the kernel launchers: workspace
// layout, launch declarations, error reporting.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/actqkv.h"

namespace actqkv {

// ---- error reporting -------------------------------------------------------
int set_error(int code, const char* fmt, ...);
// Turns the last HIP launch error, if any, into ACTQKV_EHIP.
int hip_status(const char* what);

// ---- sizes -----------------------------------------------------------------
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline size_t stats_floats(const actqkv_shape& sh) {
  return 4 + 2 * size_t(sh.n_q_heads) * sh.head_dim;
}
// The probe kernels cut the d channels into slabs of 128 bytes of a query row.
constexpr int kProbeSlabBytes = 128;
inline int probe_slabs(const actqkv_shape& sh) {
  int per = kProbeSlabBytes / (sh.dtype == ACTQKV_F32 ? 4 : 2);
  return (sh.n_q_heads * sh.head_dim + per - 1) / per;
}
inline size_t probe_a_floats(int m) { return (size_t(m) + 15) / 16 * 16; }
// per sequence: partial |phi_j|_1 [slabs][m rounded up to 16]
inline size_t probe_scratch_floats(const actqkv_shape& sh, int m) {
  return size_t(probe_slabs(sh)) * probe_a_floats(m);
}
// A call over consecutive windows of one sequence reads whole rows, kRowChunk of them per
// workgroup, and keeps, in floats: part [n][chunks][2][d] (sums and sums of squares per chunk),
// stat [n][3][d] (mean, 1/var, the window's own mean), pprobe [n][chunks][d] (weighted sums per
// chunk), asum [n][chunks rounded up to 16], a [n][m rounded up to 16].
constexpr int kRowChunk = 64;
struct ChainScratch {
  int n_chunks, asum_stride;
  size_t part, stat, pprobe, asum, a;
  size_t total() const { return part + stat + pprobe + asum + a; }
};
inline ChainScratch chain_scratch(const actqkv_shape& sh, int batch, int m) {
  ChainScratch c;
  const size_t d = size_t(sh.n_q_heads) * sh.head_dim;
  c.n_chunks = (m + kRowChunk - 1) / kRowChunk;
  c.asum_stride = (c.n_chunks + 15) / 16 * 16;
  c.part = size_t(batch) * c.n_chunks * 2 * d;
  c.stat = size_t(batch) * 3 * d;
  c.pprobe = size_t(batch) * c.n_chunks * d;
  c.asum = size_t(batch) * c.asum_stride;
  c.a = size_t(batch) * probe_a_floats(m);
  return c;
}
// the whole call: the slab partials of every entry, or what the row-major kernels keep
inline size_t probe_call_floats(const actqkv_shape& sh, int batch, int m) {
  const size_t slabs = size_t(batch) * probe_scratch_floats(sh, m);
  const size_t rows = chain_scratch(sh, batch, m).total();
  return (slabs > rows ? slabs : rows) + 4;
}

// Key-tile splits of the prefill attention.
// The first n_qtiles - rem query tiles of a sequence are cut into s_lo pieces, the last rem
// (which see more of the causal window) into s_lo + 1; slots = pieces per (sequence, KV head).
struct PfSplits {
  int s_lo, rem, slots;
};
PfSplits prefill_splits(const actqkv_shape& sh, int batch, int m, int k_cap, int cus);   // cus: compute units to fill
// prefill on the matrix cores: per workgroup and piece, 8 wavefronts x (16 eight-byte words of
// four bf16 of normalised output + one word (max, sum)) x 64 lanes, counted in floats
constexpr size_t kPfPartialFloats = 8 * (32 + 2) * 64;
constexpr int kMaxWindow = 8192;

// head of the workspace: 1024 uint32 tickets, then the work queue counters of the prefill attention
constexpr size_t kTicketCounters = 1024;
constexpr size_t kCounterBytes = 8192;
// behind the queue counters: two counters per sequence for the decode layer in one launch
constexpr size_t kSeqCounterOffset = kTicketCounters + 256, kSeqCounters = 768;
constexpr int kChipCus = 256;   // compute units of the chip
constexpr int kMaxBatch = 1024;

// what exactly this call needs when the prefill attention may fill `cus` compute units (never more
// than with all of them)
size_t workspace_bytes(const actqkv_shape& sh, int batch, int m, int nb_capacity, int k_cap, int cus = kChipCus);

size_t attention_scratch_bytes(const actqkv_shape& sh, int batch, int m, int k_cap, int cus);   // the attention alone
// Host-side checks of an attention call (ACTQKV_OK or the error); *need = the scratch bytes it uses.
int attention_validate(const actqkv_shape* shape, int batch, int m, const void* q, const void* k_cache,
                       const void* v_cache, int64_t seq_stride, int nb_capacity, const int32_t* n_ctx,
                       const int32_t* idx, const int32_t* n_sel, int k_cap, void* out, float* lse, int first_cus,
                       size_t* need);

struct Workspace {
  void* base;
  size_t bytes;
  unsigned int* counters() const { return static_cast<unsigned int*>(base); }
  float* scratch_f32() const {
    return reinterpret_cast<float*>(static_cast<char*>(base) + kCounterBytes);
  }
};

// ---- launchers (one per entry point; arguments already validated) ----------
int launch_probe(const actqkv_shape& sh, int batch, int m, const void* q_win, float* stats,
                 int update_stats, float* probe, float* probe_kv, float* probe_norm, float* weights,
                 const Workspace& ws, hipStream_t stream);
int launch_score(const actqkv_shape& sh, int batch, const float* probe_kv, const float* probe_norm,
                 const void* rep_keys, int64_t seq_stride, int nb_capacity, int nb_begin,
                 const int32_t* nb_end, float* scores, int64_t score_stride, hipStream_t stream);
int launch_select(int batch, const float* scores, int64_t score_stride, int nb_capacity, int nb_begin,
                  const int32_t* nb_end, int k_cap, int flags, float* budget_remaining,
                  const float* theta_rest_sum, int32_t* idx, int32_t* n_sel, float* theta,
                  float* budget, hipStream_t stream);
int launch_attention(const actqkv_shape& sh, int batch, int m, const void* q, const void* k_cache,
                     const void* v_cache, int64_t seq_stride, int nb_capacity, const int32_t* n_ctx,
                     const int32_t* idx, const int32_t* n_sel, int k_cap, void* out, float* lse,
                     const Workspace& ws, int sel_per_head, hipStream_t stream, int first_cus = kChipCus,
                     int late_cus = 0, hipStream_t stream_late = nullptr);   // late_cus > 0: a second team of
                                                       // workgroups for the queue, on stream_late
int launch_score_per_head(const actqkv_shape& sh, int batch, const float* probe, const void* rep_keys,
                          int64_t seq_stride, int nb_capacity, int nb_begin, const int32_t* nb_end,
                          float* scores, int64_t score_stride, hipStream_t stream);

int launch_append(const actqkv_shape& sh, int batch, int m, const void* k_new, const void* v_new,
                  const int32_t* pos0, void* k_cache, void* v_cache, int64_t cache_stride,
                  void* rep_keys, int64_t rep_stride, int nb_capacity, const void* q_tok, float* probe,
                  float* probe_kv, float* probe_norm, hipStream_t stream);   // q_tok: fused one-token probe, or NULL

int launch_decode_retrieve(const actqkv_shape& sh, int batch, const void* q_tok, const void* k_new,
                           const void* v_new, const int32_t* pos0, void* k_cache, void* v_cache,
                           int64_t cache_stride, void* rep_keys, int64_t rep_stride, int nb_capacity,
                           int nb_begin, const int32_t* nb_end, float* probe, float* probe_kv,
                           float* probe_norm, float* scores, int64_t score_stride, int k_cap, int flags,
                           float* budget_remaining, const float* theta_rest_sum, int32_t* idx,
                           int32_t* n_sel, float* theta, float* budget,
                           hipStream_t stream);   // k_new NULL: no cache update

// a whole decode layer in one launch (bf16, head_dim 128); k_new NULL: no cache update
int launch_decode_layer(const actqkv_shape& sh, int batch, const void* q, const void* k_new, const void* v_new,
                        void* k_cache, void* v_cache, int64_t seq_stride, void* rep_keys, int64_t rep_stride,
                        int nb_capacity, const int32_t* n_ctx, int nb_begin, const int32_t* nb_end, float* scores,
                        int64_t score_stride, int k_cap, int flags, const float* budget_in,
                        const float* theta_rest_sum, float* budget_after, int32_t* idx, int32_t* n_sel,
                        float* theta, float* budget, void* out, float* lse, float* scratch,
                        unsigned int* counters, float scale, int wait_us, hipStream_t stream);

int launch_gather(const actqkv_shape& sh, int batch, const void* k_store, const void* v_store,
                  int64_t store_stride, int nb_store, const int32_t* idx, const int32_t* n_sel, int k_cap,
                  void* k_cache, void* v_cache, int64_t cache_stride, int slot0, int32_t* idx_slots,
                  hipStream_t stream);

int launch_cutoff_budgets(int batch, int n_layers, float k_mean, int k_cap, const float* theta, float* budget,
                          int32_t* count, float* budget_left, hipStream_t stream);
int launch_cutoff_next_step(int batch, int n_layers, float k_mean, float theta_prior,
                            const float* theta_prev, float* theta_sum, float* n_steps,
                            float* budget_remaining, float* theta_rest_sum, hipStream_t stream);

}  // namespace actqkv
