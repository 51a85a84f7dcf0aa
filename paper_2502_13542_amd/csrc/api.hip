// C ABI of the library: host-side argument checks, then one launcher per entry point.
// The checks need no GPU, so every error path can be exercised on a CPU-only machine.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "common.h"
#include "launch.h"

namespace actqkv {

static thread_local char g_error[512] = "";

int set_error(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
  return code;
}

int hip_status(const char* what) {
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) return ACTQKV_OK;
  return set_error(ACTQKV_EHIP, "%s: %s", what, hipGetErrorString(e));
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static int check_shape(const actqkv_shape* sh) {
  if (sh == nullptr) return set_error(ACTQKV_EINVAL, "shape is NULL");
  if (sh->n_q_heads < 1 || sh->n_kv_heads < 1 || sh->head_dim < 1 || sh->n_rep < 1 ||
      sh->n_init < 0 || sh->n_local < 0)
    return set_error(ACTQKV_EINVAL, "shape has a non-positive field");
  if (sh->dtype != ACTQKV_F32 && sh->dtype != ACTQKV_BF16)
    return set_error(ACTQKV_EINVAL, "dtype %d is neither ACTQKV_F32 nor ACTQKV_BF16", sh->dtype);
  if (!(sh->softmax_scale >= 0.f) || !(sh->var_eps >= 0.f))
    return set_error(ACTQKV_EINVAL, "softmax_scale and var_eps must be >= 0");
  if (sh->head_dim != 64 && sh->head_dim != 128)
    return set_error(ACTQKV_ESHAPE, "head_dim %d not supported (64 or 128)", sh->head_dim);
  if (sh->n_q_heads % sh->n_kv_heads != 0)
    return set_error(ACTQKV_ESHAPE, "n_q_heads %d is not a multiple of n_kv_heads %d", sh->n_q_heads,
                     sh->n_kv_heads);
  const int g = sh->n_q_heads / sh->n_kv_heads;
  if (g < 1 || g > 8) return set_error(ACTQKV_ESHAPE, "group size %d not supported (1..8)", g);
  if (sh->block_size != 128)
    return set_error(ACTQKV_ESHAPE, "block_size %d not supported (128)", sh->block_size);
  if (sh->n_rep > 16) return set_error(ACTQKV_ESHAPE, "n_rep %d not supported (1..16)", sh->n_rep);
  if (sh->n_init % sh->block_size != 0 || sh->n_local % sh->block_size != 0)
    return set_error(ACTQKV_ESHAPE, "n_init and n_local must be multiples of block_size");
  if (sh->n_q_heads * sh->head_dim > 16384)
    return set_error(ACTQKV_ESHAPE, "H*D = %d not supported (at most 16384)",
                     sh->n_q_heads * sh->head_dim);
  return ACTQKV_OK;
}

static int check_batch(int batch) {
  if (batch < 1) return set_error(ACTQKV_EINVAL, "batch %d < 1", batch);
  if (batch > kMaxBatch) return set_error(ACTQKV_ESHAPE, "batch %d > %d", batch, kMaxBatch);
  return ACTQKV_OK;
}

static int check_blocks(int nb_capacity, int nb_begin, int k_cap, bool use_k) {
  if (nb_capacity < 0 || nb_begin < 0)
    return set_error(ACTQKV_EINVAL, "nb_capacity %d or nb_begin %d negative", nb_capacity, nb_begin);
  if (use_k && (k_cap < 1 || k_cap > 64))
    return set_error(ACTQKV_ESHAPE, "k_cap %d not supported (1..64)", k_cap);
  if (nb_capacity - nb_begin > 8192)
    return set_error(ACTQKV_ESHAPE, "%d blocks in one selection (at most 8192)",
                     nb_capacity - nb_begin);
  return ACTQKV_OK;
}

#define ACTQKV_REQUIRE_PTR(p)                                                       \
  do {                                                                              \
    if ((p) == nullptr) return set_error(ACTQKV_EINVAL, #p " is NULL");             \
    if (!aligned16(p)) return set_error(ACTQKV_EALIGN, #p " is not 16-byte aligned"); \
  } while (0)
#define ACTQKV_REQUIRE_SMALL(p, a)                                                          \
  do {                                                                                      \
    if ((p) == nullptr) return set_error(ACTQKV_EINVAL, #p " is NULL");                     \
    if ((reinterpret_cast<uintptr_t>(p) & ((a)-1)) != 0)                                    \
      return set_error(ACTQKV_EALIGN, #p " is not %d-byte aligned", int(a));                \
  } while (0)
#define ACTQKV_OPTIONAL_SMALL(p, a)                                                         \
  do {                                                                                      \
    if ((p) != nullptr && (reinterpret_cast<uintptr_t>(p) & ((a)-1)) != 0)                  \
      return set_error(ACTQKV_EALIGN, #p " is not %d-byte aligned", int(a));                \
  } while (0)
#define ACTQKV_OPTIONAL_PTR(p)                                                                   \
  do {                                                                                           \
    if ((p) != nullptr && !aligned16(p)) return set_error(ACTQKV_EALIGN, #p " is not 16-byte aligned"); \
  } while (0)
#define ACTQKV_TRY(expr)      \
  do {                        \
    int rc_ = (expr);         \
    if (rc_ != ACTQKV_OK) return rc_; \
  } while (0)

bool prefill_mfma_supported(const actqkv_shape& sh, int m);
int prefill_mfma_workgroups(const actqkv_shape& sh, int m);
int prefill_mfma_qtiles(const actqkv_shape& sh, int m);
int launch_attention_prefill_mfma(const actqkv_shape& sh, int batch, int m, const void* q,
                                  const void* k_cache, const void* v_cache, int64_t seq_stride,
                                  int nb_capacity, const int32_t* n_ctx, const int32_t* idx,
                                  const int32_t* n_sel, int k_cap, void* out, float* lse,
                                  const PfSplits& splits, float* scratch, unsigned int* counters,
                                  float scale, int sel_per_head, int first_cus, int late_cus,
                                  hipStream_t stream, hipStream_t stream_late);

// Enough key splits to give every compute unit it may fill a workgroup, never more than 8
// per query tile; what does not divide evenly goes to the last query tiles of the window.
PfSplits prefill_splits(const actqkv_shape& sh, int batch, int m, int k_cap, int cus) {
  (void)k_cap;
  PfSplits r{1, 0, 1};
  if (!prefill_mfma_supported(sh, m)) return r;
  const int n_qtiles = prefill_mfma_qtiles(sh, m);
  const int pairs = batch * sh.n_kv_heads;                   // each has n_qtiles query tiles
  int per_pair = cus / (pairs > 0 ? pairs : 1);              // workgroups one pair may have
  if (per_pair < n_qtiles) per_pair = n_qtiles;
  r.s_lo = per_pair / n_qtiles;
  if (r.s_lo >= 8) {
    r.s_lo = 8;
    r.rem = 0;
  } else {
    r.rem = per_pair - r.s_lo * n_qtiles;
  }
  r.slots = r.s_lo * n_qtiles + r.rem;
  return r;
}
bool decode_mfma_supported(const actqkv_shape& sh, int m);
size_t decode_mfma_scratch_floats(const actqkv_shape& sh, int batch, int k_cap);
int launch_attention_decode_mfma(const actqkv_shape& sh, int batch, const void* q, const void* k_cache,
                                 const void* v_cache, int64_t seq_stride, int nb_capacity,
                                 const int32_t* n_ctx, const int32_t* idx, const int32_t* n_sel,
                                 int k_cap, void* out, float* lse, float* scratch,
                                 unsigned int* counters, float scale, int sel_per_head, hipStream_t stream);

int launch_attention_decode_select(const actqkv_shape& sh, int batch, const void* q, const void* k_cache,
                                   const void* v_cache, int64_t seq_stride, int nb_capacity,
                                   const int32_t* n_ctx, const float* scores, int64_t score_stride, int nb_begin,
                                   const int32_t* nb_end, int k_cap, int flags, const float* budget_in,
                                   const float* theta_rest_sum, float* budget_after, int32_t* idx,
                                   int32_t* n_sel, float* theta, float* budget, void* out, float* lse,
                                   float* scratch, unsigned int* counters, float scale, hipStream_t stream);

// scratch of the attention alone: the ticket and queue counters, then the partial results
size_t attention_scratch_bytes(const actqkv_shape& sh, int batch, int m, int k_cap, int cus) {
  size_t attn = 0;
  if (decode_mfma_supported(sh, m)) attn = decode_mfma_scratch_floats(sh, batch, k_cap) * sizeof(float);
  if (prefill_mfma_supported(sh, m)) {
    // partial results exist only where a query tile's key tiles are cut into pieces
    const PfSplits splits = prefill_splits(sh, batch, m, k_cap, cus);
    if (splits.slots > prefill_mfma_qtiles(sh, m))
      attn = size_t(batch) * sh.n_kv_heads * splits.slots * kPfPartialFloats * sizeof(float);
  }
  return kCounterBytes + align_up(attn, 256);
}

// what exactly this (batch, m) needs; the pieces a query tile is cut into, and with them the
// partial results, only grow with the compute units the attention may fill
size_t workspace_bytes(const actqkv_shape& sh, int batch, int m, int nb_capacity, int k_cap, int cus) {
  (void)nb_capacity;
  const size_t probe = kCounterBytes + align_up(probe_call_floats(sh, batch, m) * sizeof(float), 256);
  return std::max(probe, attention_scratch_bytes(sh, batch, m, k_cap, cus));
}

// What a caller should allocate: enough for every call with 1 .. batch entries and windows of
// 1 .. m tokens.  The need is not monotone: few short windows are cut into many pieces with
// partial results, many long ones into none, and a window too long for the matrix-core kernel
// needs no scratch at all; so a workspace sized for a layer's nominal window must also serve
// its ragged last window and a decode step.
static size_t workspace_bytes_upto(const actqkv_shape& sh, int batch, int m, int nb_capacity, int k_cap) {
  size_t need = 0;
  for (int b = 1; b <= batch; ++b) {
    need = std::max(need, workspace_bytes(sh, b, 1, nb_capacity, k_cap));
    for (int mm = 32; mm < m + 32; mm += 32)       // query tiles are multiples of 32 positions
      need = std::max(need, workspace_bytes(sh, b, std::min(mm, m), nb_capacity, k_cap));
  }
  return need;
}

int launch_attention_rows(const actqkv_shape& sh, int batch, int m, const void* q, const void* k_cache,
                          const void* v_cache, int64_t seq_stride, int nb_capacity,
                          const int32_t* n_ctx, const int32_t* idx, const int32_t* n_sel, int k_cap,
                          void* out, float* lse, float scale, int sel_per_head, hipStream_t stream);

int launch_attention(const actqkv_shape& sh, int batch, int m, const void* q, const void* k_cache,
                     const void* v_cache, int64_t seq_stride, int nb_capacity, const int32_t* n_ctx,
                     const int32_t* idx, const int32_t* n_sel, int k_cap, void* out, float* lse,
                     const Workspace& ws, int sel_per_head, hipStream_t stream, int first_cus, int late_cus,
                     hipStream_t stream_late) {
  const float scale = sh.softmax_scale > 0.f ? sh.softmax_scale : 1.f / std::sqrt(float(sh.head_dim));
  if (decode_mfma_supported(sh, m))   // (no queue: one launch does all the work)
    return launch_attention_decode_mfma(sh, batch, q, k_cache, v_cache, seq_stride, nb_capacity, n_ctx,
                                        idx, n_sel, k_cap, out, lse, ws.scratch_f32(), ws.counters(), scale,
                                        sel_per_head, stream);
  if (prefill_mfma_supported(sh, m))
    return launch_attention_prefill_mfma(sh, batch, m, q, k_cache, v_cache, seq_stride, nb_capacity,
                                         n_ctx, idx, n_sel, k_cap, out, lse,
                                         prefill_splits(sh, batch, m, k_cap, first_cus), ws.scratch_f32(),
                                         ws.counters(), scale, sel_per_head, first_cus, late_cus, stream,
                                         stream_late);
  return launch_attention_rows(sh, batch, m, q, k_cache, v_cache, seq_stride, nb_capacity, n_ctx, idx,
                               n_sel, k_cap, out, lse, scale, sel_per_head, stream);
}

// Host-side checks of an attention call; `need` receives the scratch bytes the call uses.
int attention_validate(const actqkv_shape* shape, int batch, int m, const void* q, const void* k_cache,
                              const void* v_cache, int64_t seq_stride, int nb_capacity, const int32_t* n_ctx,
                              const int32_t* idx, const int32_t* n_sel, int k_cap, void* out, float* lse,
                              int first_cus, size_t* need) {
  ACTQKV_TRY(check_shape(shape));
  ACTQKV_TRY(check_batch(batch));
  if (m < 1) return set_error(ACTQKV_EINVAL, "m %d < 1", m);
  if (m > kMaxWindow) return set_error(ACTQKV_ESHAPE, "m %d > %d", m, kMaxWindow);
  // (the attention selects nothing: the 8192-block limit of a selection does not apply to its cache)
  if (k_cap < 1 || k_cap > 64) return set_error(ACTQKV_ESHAPE, "k_cap %d not supported (1..64)", k_cap);
  if (nb_capacity < 1) return set_error(ACTQKV_EINVAL, "nb_capacity %d < 1", nb_capacity);
  if (int64_t(nb_capacity) * shape->block_size < m)
    return set_error(ACTQKV_EINVAL, "cache of %d blocks cannot hold a window of %d tokens", nb_capacity, m);
  if (int64_t(nb_capacity) * shape->block_size > (int64_t(1) << 30))
    return set_error(ACTQKV_ESHAPE, "cache of %d blocks exceeds 2^30 tokens", nb_capacity);
  ACTQKV_REQUIRE_PTR(q);
  ACTQKV_REQUIRE_PTR(k_cache);
  ACTQKV_REQUIRE_PTR(v_cache);
  ACTQKV_REQUIRE_SMALL(n_ctx, 4);
  ACTQKV_REQUIRE_SMALL(idx, 4);
  ACTQKV_REQUIRE_SMALL(n_sel, 4);
  ACTQKV_REQUIRE_PTR(out);
  ACTQKV_OPTIONAL_SMALL(lse, 4);
  const int64_t per_seq = int64_t(nb_capacity) * shape->n_kv_heads * shape->block_size * shape->head_dim;
  // seq_stride 0: all batch entries read one cache (several windows of one sequence)
  if (batch > 1 && seq_stride != 0 && seq_stride < per_seq)
    return set_error(ACTQKV_EINVAL, "seq_stride %lld < one sequence's cache %lld", (long long)seq_stride,
                     (long long)per_seq);
  if (seq_stride % 8 != 0) return set_error(ACTQKV_EALIGN, "seq_stride must be a multiple of 8 elements");
  *need = attention_scratch_bytes(*shape, batch, m, k_cap, first_cus);
  return ACTQKV_OK;
}

}  // namespace actqkv

using namespace actqkv;

namespace actqkv {
// Grid-stride copy of n 16-byte words (traffic-counter calibration).
__global__ __launch_bounds__(256) void copy_bytes_kernel(u32x4* __restrict__ dst,
                                                         const u32x4* __restrict__ src, size_t n) {
  for (size_t i = size_t(blockIdx.x) * 256 + threadIdx.x; i < n; i += size_t(gridDim.x) * 256)
    dst[i] = src[i];
}
}  // namespace actqkv

extern "C" {

size_t actqkv_stats_floats(const actqkv_shape* shape) {
  if (check_shape(shape) != ACTQKV_OK) return 0;
  return stats_floats(*shape);
}

size_t actqkv_workspace_bytes(const actqkv_shape* shape, int batch, int m, int nb_capacity, int k_cap) {
  if (check_shape(shape) != ACTQKV_OK) return 0;
  if (batch < 1 || batch > kMaxBatch || m < 1 || nb_capacity < 0 || k_cap < 1 || k_cap > 64) {
    set_error(ACTQKV_EINVAL, "workspace_bytes: bad batch/m/nb_capacity/k_cap");
    return 0;
  }
  return workspace_bytes_upto(*shape, batch, m, nb_capacity, k_cap);
}

int actqkv_build_probe(const actqkv_shape* shape, int batch, int m, const void* q_win, float* stats,
                       int update_stats, float* probe, float* probe_kv, float* probe_norm,
                       float* weights, void* workspace, size_t ws_bytes, void* stream) {
  ACTQKV_TRY(check_shape(shape));
  ACTQKV_TRY(check_batch(batch));
  if (m < 1) return set_error(ACTQKV_EINVAL, "m %d < 1", m);
  if (m > kMaxWindow) return set_error(ACTQKV_ESHAPE, "m %d > %d", m, kMaxWindow);
  ACTQKV_REQUIRE_PTR(q_win);
  ACTQKV_REQUIRE_PTR(probe);
  ACTQKV_REQUIRE_PTR(probe_kv);
  ACTQKV_REQUIRE_SMALL(probe_norm, 4);
  ACTQKV_OPTIONAL_SMALL(weights, 4);
  if (m > 1 || update_stats) ACTQKV_REQUIRE_PTR(stats);
  if (update_stats & ~(ACTQKV_STATS_UPDATE | ACTQKV_PROBE_MEAN_POOLING | ACTQKV_PROBE_WINDOW_CHAIN))
    return set_error(ACTQKV_EINVAL, "update_stats has unknown bits: %d", update_stats);
  if ((update_stats & ACTQKV_PROBE_WINDOW_CHAIN) && (!(update_stats & ACTQKV_STATS_UPDATE) || m < 2))
    return set_error(ACTQKV_EINVAL, "consecutive windows need ACTQKV_STATS_UPDATE and m >= 2");
  if (workspace == nullptr || !aligned16(workspace))
    return set_error(ACTQKV_EWORKSPACE, "workspace is NULL or not 16-byte aligned");
  size_t need = kCounterBytes + probe_call_floats(*shape, batch, m) * sizeof(float);
  if (ws_bytes < need)
    return set_error(ACTQKV_EWORKSPACE, "workspace has %zu bytes, build_probe needs %zu", ws_bytes, need);
  Workspace ws{workspace, ws_bytes};
  return launch_probe(*shape, batch, m, q_win, stats, update_stats, probe, probe_kv, probe_norm,
                      weights, ws, static_cast<hipStream_t>(stream));
}

int actqkv_score_blocks(const actqkv_shape* shape, int batch, const float* probe_kv,
                        const float* probe_norm, const void* rep_keys, int64_t seq_stride,
                        int nb_capacity, int nb_begin, const int32_t* nb_end, float* scores,
                        int64_t score_stride, void* stream) {
  ACTQKV_TRY(check_shape(shape));
  ACTQKV_TRY(check_batch(batch));
  ACTQKV_TRY(check_blocks(nb_capacity, nb_begin, 1, false));
  ACTQKV_REQUIRE_PTR(probe_kv);
  ACTQKV_REQUIRE_SMALL(probe_norm, 4);
  ACTQKV_REQUIRE_PTR(rep_keys);
  ACTQKV_REQUIRE_SMALL(nb_end, 4);
  ACTQKV_REQUIRE_SMALL(scores, 4);
  if (score_stride < nb_capacity)
    return set_error(ACTQKV_EINVAL, "score_stride %lld < nb_capacity %d", (long long)score_stride,
                     nb_capacity);
  const int64_t per_seq = int64_t(nb_capacity) * shape->n_rep * shape->n_kv_heads * shape->head_dim;
  if (batch > 1 && seq_stride != 0 && seq_stride < per_seq)
    return set_error(ACTQKV_EINVAL, "seq_stride %lld < one sequence's representative keys %lld",
                     (long long)seq_stride, (long long)per_seq);
  if (seq_stride % 8 != 0) return set_error(ACTQKV_EALIGN, "seq_stride must be a multiple of 8 elements");
  return launch_score(*shape, batch, probe_kv, probe_norm, rep_keys, seq_stride, nb_capacity, nb_begin,
                      nb_end, scores, score_stride, static_cast<hipStream_t>(stream));
}

int actqkv_select(int batch, const float* scores, int64_t score_stride, int nb_capacity, int nb_begin,
                  const int32_t* nb_end, int k_cap, int flags, float* budget_remaining,
                  const float* theta_rest_sum, int32_t* idx, int32_t* n_sel, float* theta,
                  float* budget, void* stream) {
  if (flags & ~(ACTQKV_SELECT_ENTROPY_TOPK | ACTQKV_SELECT_DENSITY_ONLY | ACTQKV_SELECT_GIVEN_COUNT))
    return set_error(ACTQKV_EINVAL, "select: unknown flag bits: %d", flags);
  if ((flags & ACTQKV_SELECT_DENSITY_ONLY) && (flags & ACTQKV_SELECT_GIVEN_COUNT))
    return set_error(ACTQKV_EINVAL, "select: density only and a given count exclude each other");
  if ((flags & ACTQKV_SELECT_DENSITY_ONLY) && theta == nullptr)
    return set_error(ACTQKV_EINVAL, "select: density only needs theta");
  if ((flags & (ACTQKV_SELECT_DENSITY_ONLY | ACTQKV_SELECT_GIVEN_COUNT)) && budget_remaining != nullptr)
    return set_error(ACTQKV_EINVAL, "select: the cut-off state is not used with density only or a given count");
  ACTQKV_TRY(check_batch(batch));
  ACTQKV_TRY(check_blocks(nb_capacity, nb_begin, k_cap, true));
  ACTQKV_REQUIRE_SMALL(scores, 4);
  ACTQKV_REQUIRE_SMALL(nb_end, 4);
  ACTQKV_REQUIRE_SMALL(idx, 4);
  ACTQKV_REQUIRE_SMALL(n_sel, 4);
  if ((budget_remaining == nullptr) != (theta_rest_sum == nullptr))
    return set_error(ACTQKV_EINVAL, "budget_remaining and theta_rest_sum must be given together");
  ACTQKV_OPTIONAL_SMALL(budget_remaining, 4);
  ACTQKV_OPTIONAL_SMALL(theta_rest_sum, 4);
  ACTQKV_OPTIONAL_SMALL(theta, 4);
  ACTQKV_OPTIONAL_SMALL(budget, 4);
  if (score_stride < nb_capacity)
    return set_error(ACTQKV_EINVAL, "score_stride %lld < nb_capacity %d", (long long)score_stride,
                     nb_capacity);
  return launch_select(batch, scores, score_stride, nb_capacity, nb_begin, nb_end, k_cap, flags,
                       budget_remaining, theta_rest_sum, idx, n_sel, theta, budget,
                       static_cast<hipStream_t>(stream));
}

static int attention_checked(const actqkv_shape* shape, int batch, int m, const void* q, const void* k_cache,
                             const void* v_cache, int64_t seq_stride, int nb_capacity, const int32_t* n_ctx,
                             const int32_t* idx, const int32_t* n_sel, int k_cap, void* out, float* lse,
                             void* workspace, size_t ws_bytes, int sel_per_head, void* stream,
                             int first_cus = kChipCus, int late_cus = 0, void* stream_late = nullptr) {
  size_t need = 0;
  ACTQKV_TRY(attention_validate(shape, batch, m, q, k_cache, v_cache, seq_stride, nb_capacity, n_ctx, idx, n_sel,
                                k_cap, out, lse, first_cus, &need));
  if (workspace == nullptr || !aligned16(workspace))
    return set_error(ACTQKV_EWORKSPACE, "workspace is NULL or not 16-byte aligned");
  if (ws_bytes < need)
    return set_error(ACTQKV_EWORKSPACE, "workspace has %zu bytes, retrieval_attention needs %zu", ws_bytes,
                     need);
  Workspace ws{workspace, ws_bytes};
  return launch_attention(*shape, batch, m, q, k_cache, v_cache, seq_stride, nb_capacity, n_ctx, idx,
                          n_sel, k_cap, out, lse, ws, sel_per_head, static_cast<hipStream_t>(stream), first_cus,
                          late_cus, static_cast<hipStream_t>(stream_late));
}

int actqkv_retrieval_attention(const actqkv_shape* shape, int batch, int m, const void* q,
                               const void* k_cache, const void* v_cache, int64_t seq_stride,
                               int nb_capacity, const int32_t* n_ctx, const int32_t* idx,
                               const int32_t* n_sel, int k_cap, void* out, float* lse, void* workspace,
                               size_t ws_bytes, void* stream) {
  return attention_checked(shape, batch, m, q, k_cache, v_cache, seq_stride, nb_capacity, n_ctx, idx, n_sel,
                           k_cap, out, lse, workspace, ws_bytes, 0, stream);
}

int actqkv_retrieval_attention_teams(const actqkv_shape* shape, int batch, int m, const void* q,
                                     const void* k_cache, const void* v_cache, int64_t seq_stride,
                                     int nb_capacity, const int32_t* n_ctx, const int32_t* idx,
                                     const int32_t* n_sel, int k_cap, void* out, float* lse,
                                     void* workspace, size_t ws_bytes, int first_cus, int late_cus,
                                     void* stream, void* stream_late) {
  if (first_cus < 1 || first_cus > kChipCus)
    return set_error(ACTQKV_EINVAL, "first_cus %d outside 1..%d", first_cus, kChipCus);
  if (late_cus != 0 && shape != nullptr && (late_cus < shape->n_kv_heads || late_cus > kChipCus))
    return set_error(ACTQKV_EINVAL, "late_cus %d neither 0 nor in n_kv_heads..%d", late_cus, kChipCus);
  return attention_checked(shape, batch, m, q, k_cache, v_cache, seq_stride, nb_capacity, n_ctx, idx, n_sel,
                           k_cap, out, lse, workspace, ws_bytes, 0, stream, first_cus, late_cus, stream_late);
}

int actqkv_retrieval_attention_per_head(const actqkv_shape* shape, int batch, int m, const void* q,
                                        const void* k_cache, const void* v_cache, int64_t seq_stride,
                                        int nb_capacity, const int32_t* n_ctx, const int32_t* idx,
                                        const int32_t* n_sel, int k_cap, void* out, float* lse,
                                        void* workspace, size_t ws_bytes, void* stream) {
  return attention_checked(shape, batch, m, q, k_cache, v_cache, seq_stride, nb_capacity, n_ctx, idx, n_sel,
                           k_cap, out, lse, workspace, ws_bytes, 1, stream);
}

int actqkv_decode_select_attention(const actqkv_shape* shape, int batch, const void* q,
                                   const void* k_cache, const void* v_cache, int64_t seq_stride,
                                   int nb_capacity, const int32_t* n_ctx, const float* scores,
                                   int64_t score_stride, int nb_begin, const int32_t* nb_end,
                                   int k_cap, int flags, const float* budget_in,
                                   const float* theta_rest_sum, float* budget_after, int32_t* idx,
                                   int32_t* n_sel, float* theta, float* budget, void* out,
                                   float* lse, void* workspace, size_t ws_bytes, void* stream) {
  ACTQKV_TRY(check_shape(shape));
  ACTQKV_TRY(check_batch(batch));
  if (!decode_mfma_supported(*shape, 1))
    return set_error(ACTQKV_ESHAPE, "decode_select_attention: bf16, head_dim 128 and at most 8 query heads per KV head");
  if (flags & ~ACTQKV_SELECT_ENTROPY_TOPK)
    return set_error(ACTQKV_EINVAL, "decode_select_attention: unknown flag bits: %d", flags);
  if (nb_capacity < 1) return set_error(ACTQKV_EINVAL, "nb_capacity %d < 1", nb_capacity);
  if (int64_t(nb_capacity) * shape->block_size > (int64_t(1) << 30))
    return set_error(ACTQKV_ESHAPE, "cache of %d blocks exceeds 2^30 tokens", nb_capacity);
  ACTQKV_TRY(check_blocks(nb_capacity, nb_begin, k_cap, true));
  ACTQKV_REQUIRE_PTR(q);
  ACTQKV_REQUIRE_PTR(k_cache);
  ACTQKV_REQUIRE_PTR(v_cache);
  ACTQKV_REQUIRE_SMALL(n_ctx, 4);
  ACTQKV_REQUIRE_SMALL(scores, 4);
  ACTQKV_REQUIRE_SMALL(nb_end, 4);
  ACTQKV_REQUIRE_SMALL(idx, 4);
  ACTQKV_REQUIRE_SMALL(n_sel, 4);
  ACTQKV_REQUIRE_PTR(out);
  ACTQKV_OPTIONAL_SMALL(lse, 4);
  if ((budget_in == nullptr) != (theta_rest_sum == nullptr))
    return set_error(ACTQKV_EINVAL, "budget_in and theta_rest_sum must be given together");
  ACTQKV_OPTIONAL_SMALL(budget_in, 4);
  ACTQKV_OPTIONAL_SMALL(theta_rest_sum, 4);
  ACTQKV_OPTIONAL_SMALL(budget_after, 4);
  ACTQKV_OPTIONAL_SMALL(theta, 4);
  ACTQKV_OPTIONAL_SMALL(budget, 4);
  if (budget_after != nullptr && budget_after == budget_in)
    return set_error(ACTQKV_EINVAL, "budget_after must not be the array budget_in points to");
  if (score_stride < nb_capacity)
    return set_error(ACTQKV_EINVAL, "score_stride %lld < nb_capacity %d", (long long)score_stride,
                     nb_capacity);
  const int64_t per_seq = int64_t(nb_capacity) * shape->n_kv_heads * shape->block_size * shape->head_dim;
  if (batch > 1 && seq_stride != 0 && seq_stride < per_seq)
    return set_error(ACTQKV_EINVAL, "seq_stride %lld < one sequence's cache %lld", (long long)seq_stride,
                     (long long)per_seq);
  if (seq_stride % 8 != 0) return set_error(ACTQKV_EALIGN, "seq_stride must be a multiple of 8 elements");
  if (workspace == nullptr || !aligned16(workspace))
    return set_error(ACTQKV_EWORKSPACE, "workspace is NULL or not 16-byte aligned");
  const size_t need = workspace_bytes(*shape, batch, 1, nb_capacity, k_cap);
  if (ws_bytes < need)
    return set_error(ACTQKV_EWORKSPACE, "workspace has %zu bytes, decode_select_attention needs %zu", ws_bytes,
                     need);
  Workspace ws{workspace, ws_bytes};
  const float scale = shape->softmax_scale > 0.f ? shape->softmax_scale : 1.f / std::sqrt(float(shape->head_dim));
  return launch_attention_decode_select(*shape, batch, q, k_cache, v_cache, seq_stride, nb_capacity, n_ctx,
                                        scores, score_stride, nb_begin, nb_end, k_cap, flags, budget_in,
                                        theta_rest_sum, budget_after, idx, n_sel, theta, budget, out, lse,
                                        ws.scratch_f32(), ws.counters(), scale,
                                        static_cast<hipStream_t>(stream));
}

int actqkv_decode_layer(const actqkv_shape* shape, int batch, const void* q, const void* k_new,
                        const void* v_new, void* k_cache, void* v_cache, int64_t cache_seq_stride,
                        void* rep_keys, int64_t rep_seq_stride, int nb_capacity, const int32_t* n_ctx,
                        int nb_begin, const int32_t* nb_end, float* scores, int64_t score_stride, int k_cap,
                        int flags, const float* budget_in, const float* theta_rest_sum, float* budget_after,
                        int32_t* idx, int32_t* n_sel, float* theta, float* budget, void* out, float* lse,
                        void* workspace, size_t ws_bytes, void* stream) {
  ACTQKV_TRY(check_shape(shape));
  ACTQKV_TRY(check_batch(batch));
  if (!decode_mfma_supported(*shape, 1))
    return set_error(ACTQKV_ESHAPE, "decode_layer: bf16, head_dim 128 and at most 8 query heads per KV head");
  if (flags & ~(ACTQKV_SELECT_ENTROPY_TOPK | ACTQKV_DECODE_NO_WAIT))
    return set_error(ACTQKV_EINVAL, "decode_layer: unknown flag bits: %d", flags);
  if (nb_capacity < 1) return set_error(ACTQKV_EINVAL, "nb_capacity %d < 1", nb_capacity);
  if (int64_t(nb_capacity) * shape->block_size > (int64_t(1) << 30))
    return set_error(ACTQKV_ESHAPE, "cache of %d blocks exceeds 2^30 tokens", nb_capacity);
  ACTQKV_TRY(check_blocks(nb_capacity, nb_begin, k_cap, true));
  if (batch > int(kSeqCounters / 2))
    return set_error(ACTQKV_ESHAPE, "decode_layer: batch %d > %d", batch, int(kSeqCounters / 2));
  ACTQKV_REQUIRE_PTR(q);
  if ((k_new == nullptr) != (v_new == nullptr))
    return set_error(ACTQKV_EINVAL, "k_new and v_new must be given together");
  ACTQKV_OPTIONAL_PTR(k_new);
  ACTQKV_OPTIONAL_PTR(v_new);
  ACTQKV_REQUIRE_PTR(k_cache);
  ACTQKV_REQUIRE_PTR(v_cache);
  ACTQKV_REQUIRE_PTR(rep_keys);
  ACTQKV_REQUIRE_SMALL(n_ctx, 4);
  ACTQKV_REQUIRE_SMALL(nb_end, 4);
  ACTQKV_REQUIRE_SMALL(scores, 4);
  ACTQKV_REQUIRE_SMALL(idx, 4);
  ACTQKV_REQUIRE_SMALL(n_sel, 4);
  ACTQKV_REQUIRE_PTR(out);
  ACTQKV_OPTIONAL_SMALL(lse, 4);
  if ((budget_in == nullptr) != (theta_rest_sum == nullptr))
    return set_error(ACTQKV_EINVAL, "budget_in and theta_rest_sum must be given together");
  ACTQKV_OPTIONAL_SMALL(budget_in, 4);
  ACTQKV_OPTIONAL_SMALL(theta_rest_sum, 4);
  ACTQKV_OPTIONAL_SMALL(budget_after, 4);
  ACTQKV_OPTIONAL_SMALL(theta, 4);
  ACTQKV_OPTIONAL_SMALL(budget, 4);
  if (budget_after != nullptr && budget_after == budget_in)
    return set_error(ACTQKV_EINVAL, "budget_after must not be the array budget_in points to");
  if (score_stride < nb_capacity)
    return set_error(ACTQKV_EINVAL, "score_stride %lld < nb_capacity %d", (long long)score_stride,
                     nb_capacity);
  const int64_t per_seq = int64_t(nb_capacity) * shape->n_kv_heads * shape->block_size * shape->head_dim;
  const int64_t rep_per_seq = int64_t(nb_capacity) * shape->n_rep * shape->n_kv_heads * shape->head_dim;
  if (batch > 1 && cache_seq_stride < per_seq)
    return set_error(ACTQKV_EINVAL, "cache_seq_stride %lld < one sequence's cache %lld",
                     (long long)cache_seq_stride, (long long)per_seq);
  if (batch > 1 && rep_seq_stride < rep_per_seq)
    return set_error(ACTQKV_EINVAL, "rep_seq_stride %lld < one sequence's representative keys %lld",
                     (long long)rep_seq_stride, (long long)rep_per_seq);
  if (cache_seq_stride % 8 != 0 || rep_seq_stride % 8 != 0)
    return set_error(ACTQKV_EALIGN, "sequence strides must be multiples of 8 elements");
  if (workspace == nullptr || !aligned16(workspace))
    return set_error(ACTQKV_EWORKSPACE, "workspace is NULL or not 16-byte aligned");
  const size_t need = workspace_bytes(*shape, batch, 1, nb_capacity, k_cap);
  if (ws_bytes < need)
    return set_error(ACTQKV_EWORKSPACE, "workspace has %zu bytes, decode_layer needs %zu", ws_bytes, need);
  Workspace ws{workspace, ws_bytes};
  const float scale = shape->softmax_scale > 0.f ? shape->softmax_scale : 1.f / std::sqrt(float(shape->head_dim));
  // the wait for the other workgroups' scores is bounded: 2 ms is a hundred times a whole launch
  const int wait_us = (flags & ACTQKV_DECODE_NO_WAIT) ? 0 : 2000;
  return launch_decode_layer(*shape, batch, q, k_new, v_new, k_cache, v_cache, cache_seq_stride, rep_keys,
                             rep_seq_stride, nb_capacity, n_ctx, nb_begin, nb_end, scores, score_stride, k_cap,
                             flags & ACTQKV_SELECT_ENTROPY_TOPK, budget_in, theta_rest_sum, budget_after, idx,
                             n_sel, theta, budget, out, lse, ws.scratch_f32(), ws.counters(), scale, wait_us,
                             static_cast<hipStream_t>(stream));
}

int actqkv_score_blocks_per_head(const actqkv_shape* shape, int batch, const float* probe, const void* rep_keys,
                                 int64_t seq_stride, int nb_capacity, int nb_begin, const int32_t* nb_end,
                                 float* scores, int64_t score_stride, void* stream) {
  ACTQKV_TRY(check_shape(shape));
  ACTQKV_TRY(check_batch(batch));
  ACTQKV_TRY(check_blocks(nb_capacity, nb_begin, 1, false));
  ACTQKV_REQUIRE_PTR(probe);
  ACTQKV_REQUIRE_PTR(rep_keys);
  ACTQKV_REQUIRE_SMALL(nb_end, 4);
  ACTQKV_REQUIRE_SMALL(scores, 4);
  if (score_stride < nb_capacity)
    return set_error(ACTQKV_EINVAL, "score_stride %lld < nb_capacity %d", (long long)score_stride,
                     nb_capacity);
  const int64_t per_seq = int64_t(nb_capacity) * shape->n_rep * shape->n_kv_heads * shape->head_dim;
  if (batch > 1 && seq_stride != 0 && seq_stride < per_seq)
    return set_error(ACTQKV_EINVAL, "seq_stride %lld < one sequence's representative keys %lld",
                     (long long)seq_stride, (long long)per_seq);
  if (seq_stride % 8 != 0) return set_error(ACTQKV_EALIGN, "seq_stride must be a multiple of 8 elements");
  return launch_score_per_head(*shape, batch, probe, rep_keys, seq_stride, nb_capacity, nb_begin, nb_end,
                               scores, score_stride, static_cast<hipStream_t>(stream));
}

int actqkv_copy_bytes(void* dst, const void* src, size_t bytes, void* stream) {
  if (dst == nullptr || src == nullptr) return set_error(ACTQKV_EINVAL, "copy_bytes: null pointer");
  if (bytes % 16 != 0) return set_error(ACTQKV_EINVAL, "copy_bytes: %zu bytes is not a multiple of 16", bytes);
  if (reinterpret_cast<uintptr_t>(dst) % 16 != 0 || reinterpret_cast<uintptr_t>(src) % 16 != 0)
    return set_error(ACTQKV_EALIGN, "copy_bytes: pointers must be 16-byte aligned");
  if (bytes == 0) return ACTQKV_OK;
  const size_t n = bytes / 16;
  const unsigned blocks = unsigned(std::min<size_t>((n + 255) / 256, 256 * 16));
  hipLaunchKernelGGL(copy_bytes_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<u32x4*>(dst), static_cast<const u32x4*>(src), n);
  return hip_status("copy_bytes");
}

int actqkv_gather_blocks(const actqkv_shape* shape, int batch, const void* k_store, const void* v_store,
                         int64_t store_seq_stride, int nb_store, const int32_t* idx, const int32_t* n_sel,
                         int k_cap, void* k_cache, void* v_cache, int64_t cache_seq_stride,
                         int nb_capacity, int slot0, int32_t* idx_slots, void* stream) {
  ACTQKV_TRY(check_shape(shape));
  ACTQKV_TRY(check_batch(batch));
  if (k_cap < 1 || k_cap > 64) return set_error(ACTQKV_ESHAPE, "k_cap %d outside 1..64", k_cap);
  if (nb_store < 1 || nb_capacity < 1) return set_error(ACTQKV_EINVAL, "gather_blocks: empty store or cache");
  if (slot0 < 0 || int64_t(slot0) + k_cap > nb_capacity)
    return set_error(ACTQKV_EINVAL, "gather_blocks: slots %d .. %d outside the cache of %d blocks", slot0,
                     slot0 + k_cap - 1, nb_capacity);
  ACTQKV_REQUIRE_PTR(k_store);
  ACTQKV_REQUIRE_PTR(v_store);
  ACTQKV_REQUIRE_PTR(k_cache);
  ACTQKV_REQUIRE_PTR(v_cache);
  ACTQKV_REQUIRE_SMALL(idx, 4);
  ACTQKV_REQUIRE_SMALL(n_sel, 4);
  ACTQKV_OPTIONAL_SMALL(idx_slots, 4);
  const int64_t block_elems = int64_t(shape->n_kv_heads) * shape->block_size * shape->head_dim;
  if (batch > 1 && (store_seq_stride < nb_store * block_elems || cache_seq_stride < nb_capacity * block_elems))
    return set_error(ACTQKV_EINVAL, "gather_blocks: a sequence stride is smaller than one sequence");
  if (store_seq_stride % 8 != 0 || cache_seq_stride % 8 != 0)
    return set_error(ACTQKV_EALIGN, "sequence strides must be multiples of 8 elements");
  return launch_gather(*shape, batch, k_store, v_store, store_seq_stride, nb_store, idx, n_sel, k_cap, k_cache,
                       v_cache, cache_seq_stride, slot0, idx_slots, static_cast<hipStream_t>(stream));
}

static int append_checked(const actqkv_shape* shape, int batch, int m, const void* k_new, const void* v_new,
                          const int32_t* pos0, void* k_cache, void* v_cache, int64_t cache_seq_stride,
                          void* rep_keys, int64_t rep_seq_stride, int nb_capacity, const void* q_tok,
                          float* probe, float* probe_kv, float* probe_norm, void* stream) {
  ACTQKV_TRY(check_shape(shape));
  ACTQKV_TRY(check_batch(batch));
  if (m < 1) return set_error(ACTQKV_EINVAL, "m %d < 1", m);
  if (m > kMaxWindow) return set_error(ACTQKV_ESHAPE, "m %d > %d", m, kMaxWindow);
  if (nb_capacity < 1) return set_error(ACTQKV_EINVAL, "nb_capacity %d < 1", nb_capacity);
  if (int64_t(nb_capacity) * shape->block_size > (int64_t(1) << 30))
    return set_error(ACTQKV_ESHAPE, "cache of %d blocks exceeds 2^30 tokens", nb_capacity);
  ACTQKV_REQUIRE_PTR(k_new);
  ACTQKV_REQUIRE_PTR(v_new);
  ACTQKV_REQUIRE_SMALL(pos0, 4);
  ACTQKV_REQUIRE_PTR(k_cache);
  ACTQKV_REQUIRE_PTR(v_cache);
  ACTQKV_OPTIONAL_PTR(rep_keys);
  const int64_t per_seq = int64_t(nb_capacity) * shape->n_kv_heads * shape->block_size * shape->head_dim;
  const int64_t rep_per_seq = int64_t(nb_capacity) * shape->n_rep * shape->n_kv_heads * shape->head_dim;
  if (batch > 1 && cache_seq_stride < per_seq)
    return set_error(ACTQKV_EINVAL, "cache_seq_stride %lld < one sequence's cache %lld",
                     (long long)cache_seq_stride, (long long)per_seq);
  if (batch > 1 && rep_keys != nullptr && rep_seq_stride < rep_per_seq)
    return set_error(ACTQKV_EINVAL, "rep_seq_stride %lld < one sequence's representative keys %lld",
                     (long long)rep_seq_stride, (long long)rep_per_seq);
  if (cache_seq_stride % 8 != 0 || rep_seq_stride % 8 != 0)
    return set_error(ACTQKV_EALIGN, "sequence strides must be multiples of 8 elements");
  return launch_append(*shape, batch, m, k_new, v_new, pos0, k_cache, v_cache, cache_seq_stride, rep_keys,
                       rep_seq_stride, nb_capacity, q_tok, probe, probe_kv, probe_norm,
                       static_cast<hipStream_t>(stream));
}

int actqkv_append_kv(const actqkv_shape* shape, int batch, int m, const void* k_new, const void* v_new,
                     const int32_t* pos0, void* k_cache, void* v_cache, int64_t cache_seq_stride,
                     void* rep_keys, int64_t rep_seq_stride, int nb_capacity, void* stream) {
  return append_checked(shape, batch, m, k_new, v_new, pos0, k_cache, v_cache, cache_seq_stride, rep_keys,
                        rep_seq_stride, nb_capacity, nullptr, nullptr, nullptr, nullptr, stream);
}

int actqkv_append_kv_probe(const actqkv_shape* shape, int batch, const void* q_tok, const void* k_new,
                           const void* v_new, const int32_t* pos0, void* k_cache, void* v_cache,
                           int64_t cache_seq_stride, void* rep_keys, int64_t rep_seq_stride,
                           int nb_capacity, float* probe, float* probe_kv, float* probe_norm,
                           void* stream) {
  ACTQKV_REQUIRE_PTR(q_tok);
  ACTQKV_REQUIRE_PTR(probe);
  ACTQKV_REQUIRE_PTR(probe_kv);
  ACTQKV_REQUIRE_SMALL(probe_norm, 4);
  return append_checked(shape, batch, 1, k_new, v_new, pos0, k_cache, v_cache, cache_seq_stride, rep_keys,
                        rep_seq_stride, nb_capacity, q_tok, probe, probe_kv, probe_norm, stream);
}

int actqkv_decode_retrieve(const actqkv_shape* shape, int batch, const void* q_tok, const void* k_new,
                           const void* v_new, const int32_t* pos0, void* k_cache, void* v_cache,
                           int64_t cache_seq_stride, void* rep_keys, int64_t rep_seq_stride,
                           int nb_capacity, int nb_begin, const int32_t* nb_end, float* probe,
                           float* probe_kv, float* probe_norm, float* scores, int64_t score_stride,
                           int k_cap, int flags, float* budget_remaining,
                           const float* theta_rest_sum, int32_t* idx, int32_t* n_sel, float* theta,
                           float* budget, void* stream) {
  ACTQKV_TRY(check_shape(shape));
  ACTQKV_TRY(check_batch(batch));
  if (flags & ~(ACTQKV_SELECT_ENTROPY_TOPK | ACTQKV_DECODE_SCORES_ONLY))
    return set_error(ACTQKV_EINVAL, "decode_retrieve: unknown flag bits: %d", flags);
  const bool select_too = !(flags & ACTQKV_DECODE_SCORES_ONLY);
  if (nb_capacity < 1) return set_error(ACTQKV_EINVAL, "nb_capacity %d < 1", nb_capacity);
  if (int64_t(nb_capacity) * shape->block_size > (int64_t(1) << 30))
    return set_error(ACTQKV_ESHAPE, "cache of %d blocks exceeds 2^30 tokens", nb_capacity);
  ACTQKV_TRY(check_blocks(nb_capacity, nb_begin, k_cap, true));
  ACTQKV_REQUIRE_PTR(q_tok);
  const bool update = k_new != nullptr || v_new != nullptr || pos0 != nullptr;
  if (update) {
    ACTQKV_REQUIRE_PTR(k_new);
    ACTQKV_REQUIRE_PTR(v_new);
    ACTQKV_REQUIRE_SMALL(pos0, 4);
    ACTQKV_REQUIRE_PTR(k_cache);
    ACTQKV_REQUIRE_PTR(v_cache);
  }
  ACTQKV_REQUIRE_PTR(rep_keys);
  ACTQKV_REQUIRE_SMALL(nb_end, 4);
  ACTQKV_OPTIONAL_PTR(probe);
  ACTQKV_OPTIONAL_PTR(probe_kv);
  ACTQKV_OPTIONAL_SMALL(probe_norm, 4);
  ACTQKV_REQUIRE_SMALL(scores, 4);
  if (select_too) {
    ACTQKV_REQUIRE_SMALL(idx, 4);
    ACTQKV_REQUIRE_SMALL(n_sel, 4);
  }
  if ((budget_remaining == nullptr) != (theta_rest_sum == nullptr))
    return set_error(ACTQKV_EINVAL, "budget_remaining and theta_rest_sum must be given together");
  ACTQKV_OPTIONAL_SMALL(budget_remaining, 4);
  ACTQKV_OPTIONAL_SMALL(theta_rest_sum, 4);
  ACTQKV_OPTIONAL_SMALL(theta, 4);
  ACTQKV_OPTIONAL_SMALL(budget, 4);
  if (score_stride < nb_capacity)
    return set_error(ACTQKV_EINVAL, "score_stride %lld < nb_capacity %d", (long long)score_stride,
                     nb_capacity);
  const int64_t per_seq = int64_t(nb_capacity) * shape->n_kv_heads * shape->block_size * shape->head_dim;
  const int64_t rep_per_seq = int64_t(nb_capacity) * shape->n_rep * shape->n_kv_heads * shape->head_dim;
  if (batch > 1 && update && cache_seq_stride < per_seq)
    return set_error(ACTQKV_EINVAL, "cache_seq_stride %lld < one sequence's cache %lld",
                     (long long)cache_seq_stride, (long long)per_seq);
  if (batch > 1 && rep_seq_stride < rep_per_seq)
    return set_error(ACTQKV_EINVAL, "rep_seq_stride %lld < one sequence's representative keys %lld",
                     (long long)rep_seq_stride, (long long)rep_per_seq);
  if (cache_seq_stride % 8 != 0 || rep_seq_stride % 8 != 0)
    return set_error(ACTQKV_EALIGN, "sequence strides must be multiples of 8 elements");
  return launch_decode_retrieve(*shape, batch, q_tok, k_new, v_new, pos0, k_cache, v_cache, cache_seq_stride,
                                rep_keys, rep_seq_stride, nb_capacity, nb_begin, nb_end, probe, probe_kv,
                                probe_norm, scores, score_stride, k_cap, flags, budget_remaining,
                                theta_rest_sum, idx, n_sel, theta, budget, static_cast<hipStream_t>(stream));
}

int actqkv_cutoff_budgets(int batch, int n_layers, float k_mean, int k_cap, const float* theta, float* budget,
                          int32_t* count, float* budget_left, void* stream) {
  ACTQKV_TRY(check_batch(batch));
  if (n_layers < 1 || n_layers > 1024)
    return set_error(ACTQKV_ESHAPE, "n_layers %d not supported (1..1024)", n_layers);
  if (!(k_mean > 0.f)) return set_error(ACTQKV_EINVAL, "k_mean must be positive");
  if (k_cap < 1 || k_cap > 64) return set_error(ACTQKV_ESHAPE, "k_cap %d not supported (1..64)", k_cap);
  ACTQKV_REQUIRE_SMALL(theta, 4);
  ACTQKV_REQUIRE_SMALL(budget, 4);
  ACTQKV_REQUIRE_SMALL(count, 4);
  ACTQKV_OPTIONAL_SMALL(budget_left, 4);
  return launch_cutoff_budgets(batch, n_layers, k_mean, k_cap, theta, budget, count, budget_left,
                               static_cast<hipStream_t>(stream));
}

int actqkv_cutoff_next_step(int batch, int n_layers, float k_mean, float theta_prior,
                            const float* theta_prev, float* theta_sum, float* n_steps,
                            float* budget_remaining, float* theta_rest_sum, void* stream) {
  ACTQKV_TRY(check_batch(batch));
  if (n_layers < 1 || n_layers > 1024)
    return set_error(ACTQKV_ESHAPE, "n_layers %d not supported (1..1024)", n_layers);
  if (!(k_mean > 0.f)) return set_error(ACTQKV_EINVAL, "k_mean must be positive");
  if (!(theta_prior >= 0.f)) return set_error(ACTQKV_EINVAL, "theta_prior must not be negative");
  ACTQKV_OPTIONAL_SMALL(theta_prev, 4);
  ACTQKV_REQUIRE_SMALL(theta_sum, 4);
  ACTQKV_REQUIRE_SMALL(n_steps, 4);
  ACTQKV_REQUIRE_SMALL(budget_remaining, 4);
  ACTQKV_REQUIRE_SMALL(theta_rest_sum, 4);
  return launch_cutoff_next_step(batch, n_layers, k_mean, theta_prior, theta_prev, theta_sum, n_steps,
                                 budget_remaining, theta_rest_sum, static_cast<hipStream_t>(stream));
}

const char* actqkv_last_error(void) { return g_error; }

int actqkv_version(void) { return ACTQKV_VERSION; }

}  // extern "C"
