/*
 * actqkv.h - C ABI of the ActQKV per-layer retrieval-attention path for MI355X (gfx950).
 *
 * One layer, one context window (prefill) or one new token (decode) per call chain:
 *
 *   actqkv_build_probe   Activation Bias and probe-Query      (Sec. 4.1, Eq. (7)-(9))
 *   actqkv_score_blocks  cosine scores of the KV blocks       (Sec. 3.2 Eq. (5), Sec. 4.2 Eq. (10))
 *   actqkv_select        information density, budget, top-E   (Sec. 4.2 Eq. (11)-(12), Alg. 1)
 *   actqkv_retrieval_attention  attention over initial tokens, retrieved blocks,
 *                        local span and the window itself     (Sec. 3.1 Eq. (2)-(3))
 *
 * Conventions shared by every call
 *   - Every tensor pointer is a DEVICE pointer owned by the caller.  The library
 *     never allocates, frees or keeps a pointer beyond the call; scratch memory
 *     comes from the caller's workspace (actqkv_workspace_bytes sizes it).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  A
 *     call only enqueues kernels: no device synchronisation, no read-back.  The
 *     number of selected blocks, their indices and the cut-off budget stay on
 *     the device between the calls.
 *   - Pointers to q, the caches, rep_keys, stats, probe, probe_kv, out and the
 *     workspace must be 16-byte aligned (they are read with 16-byte loads);
 *     per-sequence arrays (n_ctx, nb_end, n_sel, idx, scores, theta, budget,
 *     probe_norm, weights, lse, budget_remaining, theta_rest_sum) need 4-byte alignment.
 *   - Return value: ACTQKV_OK, or a negative error code.  Arguments are checked
 *     on the host before anything is launched; on error nothing has been
 *     enqueued.  actqkv_last_error() gives a thread-local message.  Nothing
 *     throws or aborts across this boundary.
 *   - Values that live on the device (n_ctx, nb_end, idx, n_sel) cannot be
 *     checked by the host; kernels clamp them to the stated capacities, so a
 *     wrong value gives a wrong result but no out-of-bounds access.
 *   - Layouts are row-major with the last index fastest.  "storage dtype" is
 *     shape->dtype: fp32, or bf16 with fp32 accumulation.
 *
 * Blocked KV cache (per sequence; block b holds tokens [b*Bs, (b+1)*Bs)):
 *     k_cache  [nb_capacity][Hk][Bs][D]     keys, token-major inside a block
 *     v_cache  [nb_capacity][Hk][D][Bs]     values, TRANSPOSED inside a block
 *     rep_keys [nb_capacity][r][Hk][D]      r representative keys per block
 *   Values are stored channel-major so that a block's tile is a ready matrix-core
 *   operand for P*V without any transposition on the hot path.  Cache memory
 *   past the last valid token of a partial block must hold finite numbers
 *   (zero-fill the cache once); it is masked, never trusted.
 */
#ifndef ACTQKV_H
#define ACTQKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ACTQKV_VERSION 107

enum {
  ACTQKV_OK = 0,
  ACTQKV_EINVAL = -1,     /* null pointer, negative or inconsistent argument */
  ACTQKV_ESHAPE = -2,     /* H/Hk/D/Bs/r/m/k_cap combination not supported   */
  ACTQKV_EALIGN = -3,     /* a tensor pointer is not 16-byte aligned          */
  ACTQKV_EWORKSPACE = -4, /* workspace missing or too small                   */
  ACTQKV_EHIP = -5        /* a HIP call or kernel launch failed               */
};

enum { ACTQKV_F32 = 0, ACTQKV_BF16 = 1 };

/* Bits of the update_stats argument of actqkv_build_probe. */
enum {
  ACTQKV_STATS_UPDATE = 1,        /* merge the window into the running statistics first */
  ACTQKV_PROBE_MEAN_POOLING = 2,  /* ablation baseline (Sec. 5.3): every token weighs 1/m */
  ACTQKV_PROBE_WINDOW_CHAIN = 4   /* the batch entries are consecutive windows of ONE sequence */
};

/* Bits of the flags argument of actqkv_select and of the decode-step calls. */
enum {
  ACTQKV_SELECT_ENTROPY_TOPK = 1, /* density over the k_cap best blocks only (see actqkv_select) */
  ACTQKV_DECODE_SCORES_ONLY = 2,  /* actqkv_decode_retrieve stops after the scores (the caller selects,
                                     for instance inside actqkv_decode_select_attention) */
  ACTQKV_DECODE_NO_WAIT = 4,      /* actqkv_decode_layer: no workgroup waits for the scores of the others;
                                     each scores its whole sequence itself (same results, slower) */
  ACTQKV_SELECT_DENSITY_ONLY = 8, /* actqkv_select: Eq. (11) only; theta is the one output */
  ACTQKV_SELECT_GIVEN_COUNT = 16  /* actqkv_select: E is read from n_sel instead of following from Eq. (12) */
};

/* Limits checked by every call (ACTQKV_ESHAPE otherwise):
 *   head_dim in {64, 128}; n_q_heads a multiple of n_kv_heads, group size
 *   n_q_heads/n_kv_heads in 1..8; block_size == 128; 1 <= n_rep <= 16;
 *   n_init and n_local multiples of block_size (0 allowed);
 *   1 <= k_cap <= 64; at most 8192 blocks take part in one selection. */
typedef struct actqkv_shape {
  int32_t n_q_heads;     /* H                                              */
  int32_t n_kv_heads;    /* Hk                                             */
  int32_t head_dim;      /* D                                              */
  int32_t block_size;    /* Bs, tokens per KV block                        */
  int32_t n_rep;         /* r, representative keys per block               */
  int32_t n_init;        /* initial tokens that are always attended        */
  int32_t n_local;       /* tokens before the window that are always attended */
  int32_t dtype;         /* ACTQKV_F32 or ACTQKV_BF16 (storage of q, k, v, rep_keys, out) */
  float softmax_scale;   /* 0 means 1/sqrt(D)                              */
  float var_eps;         /* floor of the variance in Eq. (7); 0 means 1e-12 */
} actqkv_shape;

/* Number of floats of running statistics per sequence: {n, pad[3], mean[d], m2[d]},
 * d = H*D.  n is the number of queries seen, mean their per-channel mean, m2 the
 * per-channel sum of squared deviations from it (Eq. (8) is mean and m2/(n-1)).
 * Zero-fill it before the first window. */
size_t actqkv_stats_floats(const actqkv_shape* shape);

/* Bytes of workspace that any of the calls below may need for these sizes or smaller
 * ones: every call with 1 .. batch entries and windows of 1 .. m tokens (a layer's ragged
 * last window, a decode step), whatever launch shape it asks for, is served by a workspace of
 * this size.  The
 * workspace must be zero-filled once after allocation (the kernels leave the
 * counters it holds at zero); calls sharing one workspace must be ordered on
 * one stream. */
size_t actqkv_workspace_bytes(const actqkv_shape* shape, int batch, int m, int nb_capacity,
                              int k_cap);

/* Activation Bias and probe-Query of one window per sequence (Sec. 4.1).
 *   q_win   [batch][m][H][D], storage dtype: the window's queries.
 *   stats   [batch][actqkv_stats_floats] fp32.  update_stats & ACTQKV_STATS_UPDATE: the
 *           window is merged into it first, so mean and variance cover every query up to
 *           and including this window (Eq. (8)); otherwise it is used as it is.
 *           update_stats & ACTQKV_PROBE_MEAN_POOLING: the weights of Eq. (9) are replaced by
 *           1/m (the probe is the mean of the window's queries; the statistics are still
 *           maintained if asked for).
 *           update_stats & ACTQKV_PROBE_WINDOW_CHAIN (needs ACTQKV_STATS_UPDATE and m >= 2):
 *           the batch entries are `batch` consecutive windows of one sequence and stats is
 *           that sequence's single record.  Entry b gets the probe that batch calls of one
 *           window each, in order, would give it (statistics over every query up to and
 *           including window b, Eq. (8)); stats ends as after the last window.
 *   For each token j: phi_j = (q_j - mean)^2 / max(var, eps) per channel (Eq. (7));
 *   weight_j = |phi_j|_1 / sum_j |phi_j|_1 (uniform if the sum is 0);
 *   probe = sum_j weight_j q_j (Eq. (9)).  m == 1 gives probe = q (Sec. 4.2, decode).
 * Outputs (fp32):
 *   probe      [batch][H*D]
 *   probe_kv   [batch][Hk*D]  probe summed over the G query heads of each KV head
 *   probe_norm [batch]        L2 norm of probe
 *   weights    [batch][m]     may be NULL
 * Errors: EINVAL (null, batch < 1, m < 1), ESHAPE, EALIGN, EWORKSPACE. */
int actqkv_build_probe(const actqkv_shape* shape, int batch, int m, const void* q_win,
                       float* stats, int update_stats, float* probe, float* probe_kv,
                       float* probe_norm, float* weights, void* workspace, size_t ws_bytes,
                       void* stream);

/* Block scores (Eq. (10), applied to a block's representative keys; Eq. (5)).
 *   rep_keys  [batch][nb_capacity][r][Hk][D], storage dtype; seq_stride = elements
 *             between two sequences; 0 = all entries score the same keys (the entries
 *             are then windows of one sequence, each with its own probe and nb_end).
 *   nb_end    device int32 [batch]: blocks nb_begin <= b < nb_end[s] are scored
 *             (clamped to nb_capacity); other entries of `scores` are left alone.
 *   scores    [batch][score_stride] fp32, score_stride >= nb_capacity:
 *             scores[s][b] = mean over the r keys of cos(probe, key repeated to the
 *             H query heads) = mean_j  <probe_kv, k_j> / (probe_norm * sqrt(G) * |k_j|),
 *             0 where a norm is 0. */
int actqkv_score_blocks(const actqkv_shape* shape, int batch, const float* probe_kv,
                        const float* probe_norm, const void* rep_keys, int64_t seq_stride,
                        int nb_capacity, int nb_begin, const int32_t* nb_end, float* scores,
                        int64_t score_stride, void* stream);

/* Information density, budget and selection (Eq. (11), (12), Alg. 1) over the
 * eligible blocks nb_begin <= b < nb_end[s] of each sequence.
 *   theta = entropy (natural log) of softmax(scores over the eligible blocks).
 *           flags & ACTQKV_SELECT_ENTROPY_TOPK: of softmax(scores over the min(k_cap,
 *           n_eligible) best blocks) instead - the other way to read Eq. (11), whose
 *           Fig. 3 values (a perplexity near the number of retrieved chunks) fit a
 *           distribution over the candidates rather than over the whole cache.
 *   Dynamic cut-off state (device memory, Sec. 4.2), both pointers or neither:
 *     budget_remaining [batch] fp32  B_kv, in blocks; B^l is subtracted from it, so the same
 *                                    array is handed from layer to layer within a step
 *     theta_rest_sum   [batch] fp32  R = sum over the layers still to come of their mean density
 *   Without it: E = min(k_cap, n_eligible); budget is reported as E.
 *   With it:    B = theta / (theta + R) * B_kv   (B = B_kv if the denominator is 0);
 *               E = min(k_cap, n_eligible, max(1, floor(B + 0.5)));  B_kv -= B.
 *   idx     [batch][k_cap] int32: the E best blocks, best first, equal scores by
 *           ascending block index; unused entries are -1.
 *   n_sel   [batch] int32 = E (0 when nothing is eligible; theta and budget are 0 then
 *           and budget_remaining is left alone).
 *   theta, budget  [batch] fp32, may be NULL.
 *   Alg. 1 as it is printed runs in three loops over the layers - every density, then every
 *   budget, then the selections - which two flags make callable (neither takes the cut-off state):
 *     flags & ACTQKV_SELECT_DENSITY_ONLY: only theta[s] is computed and written (required);
 *       idx, n_sel, budget are left alone.
 *     flags & ACTQKV_SELECT_GIVEN_COUNT: n_sel[s] holds E on entry (for instance a row of the
 *       counts actqkv_cutoff_budgets wrote); the min(E, k_cap, n_eligible) best blocks are
 *       selected, that number is written back to n_sel[s], and budget reports it.
 * Errors: EINVAL (null, one cut-off pointer without the other, unknown or contradictory flag
 * bits), ESHAPE (k_cap, more than 8192 blocks), EALIGN. */
int actqkv_select(int batch, const float* scores, int64_t score_stride, int nb_capacity,
                  int nb_begin, const int32_t* nb_end, int k_cap, int flags, float* budget_remaining,
                  const float* theta_rest_sum, int32_t* idx, int32_t* n_sel, float* theta,
                  float* budget, void* stream);

/* Attention of a window over [current window, selected cache] (Eq. (2); Eq. (3) for m == 1).
 *   q        [batch][m][H][D], storage dtype.
 *   k_cache, v_cache  blocked caches (layouts above), seq_stride = elements between
 *            two sequences; they already hold the window's own keys and values.
 *            seq_stride = 0 makes all batch entries read the same cache: the entries are then
 *            several windows of one sequence (each with its own n_ctx, idx, n_sel, q and out),
 *            whose attentions do not depend on each other.
 *   n_ctx    device int32 [batch]: valid tokens in the cache, the m current ones
 *            included; the window is [w0, w0+m) with w0 = n_ctx - m.
 *   idx, n_sel  from actqkv_select ([batch][k_cap], [batch]); entries outside
 *            [0, nb_capacity) are ignored.  The caller keeps selected blocks disjoint
 *            from the initial tokens and the local span (actqkv_select on the
 *            eligible range guarantees it).
 *   The query at position p sees: tokens [0, min(n_init, w0)); the selected blocks;
 *   [l0, p] with l0 = max(min(n_init, w0), (w0 - n_local) rounded down to a block
 *   boundary).  Query head h reads KV head h / G.  out = softmax(q K^T scale) V.
 *   out      [batch][m][H][D], storage dtype.
 *   lse      [batch][H][m] fp32, natural-log sum of exp of the scaled logits; may be NULL. */
int actqkv_retrieval_attention(const actqkv_shape* shape, int batch, int m, const void* q,
                               const void* k_cache, const void* v_cache, int64_t seq_stride,
                               int nb_capacity, const int32_t* n_ctx, const int32_t* idx,
                               const int32_t* n_sel, int k_cap, void* out, float* lse,
                               void* workspace, size_t ws_bytes, void* stream);

/* actqkv_retrieval_attention for callers that cannot allocate or bring a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The scratch memory
 * the attention kernels use (ticket and queue counters, partial results of query tiles whose key
 * tiles are cut into pieces, partial results of decode sequences split over several workgroups)
 * is an array of ACTQKV_STATIC_SCRATCH_BYTES that is part of the library's device code; every
 * GPU the library runs on holds its own copy from the first call on it until the process ends.
 * The call allocates and frees nothing.  The first call on a device looks the array's address up
 * (it may load the library's code onto the device): make that one call outside graph capture.
 *   Arguments, results and errors as in actqkv_retrieval_attention, without the workspace.
 *   A call that would need more scratch than the array holds is refused with ACTQKV_EWORKSPACE
 *   and a message that states both sizes (one window of up to 8192 tokens and decode batches of
 *   up to 1024 sequences at the 32-head shape fit).
 *   All calls on one GPU share the array: two calls that overlap in time on one GPU (two streams,
 *   two threads) race and give wrong results; order them on one stream.  Every call first puts the
 *   counters at the head of the array back to zero with a small kernel on `stream`. */
#define ACTQKV_STATIC_SCRATCH_BYTES (32u << 20)
int actqkv_retrieval_attention_static(const actqkv_shape* shape, int batch, int m, const void* q,
                                      const void* k_cache, const void* v_cache, int64_t seq_stride,
                                      int nb_capacity, const int32_t* n_ctx, const int32_t* idx,
                                      const int32_t* n_sel, int k_cap, void* out, float* lse,
                                      void* stream);

/* Cache update (Sec. 3.1, Eq. (4): the cache after a step is the cache before it with the
 * step's keys and values appended), written in the blocked layouts above, and the
 * representative keys of every block the new tokens complete.
 *   k_new, v_new  [batch][m][Hk][D], storage dtype: keys and values of the m new tokens.
 *   pos0     device int32 [batch]: tokens already in the sequence's cache; the new tokens take
 *            positions pos0 .. pos0 + m - 1.  Tokens that would fall behind block
 *            nb_capacity - 1 are dropped.
 *   k_cache, v_cache  as in actqkv_retrieval_attention; only the new positions are written.
 *   rep_keys [nb_capacity][r][Hk][D] per sequence, or NULL.  For every block that is complete
 *            after the call and was not before, its r entries are written: the keys of the r
 *            tokens of the block whose key over all KV heads together has the largest L2
 *            norm (squares summed in fp32; equal norms: the lower position), in position
 *            order.  The paper leaves this choice to the block-retrieval work it builds on.
 *   cache_seq_stride, rep_seq_stride  elements between two sequences (multiples of 8).
 * The call reads tokens older than pos0 of a completed block from k_cache, so earlier appends
 * to the same cache must be ordered before it on the stream. */
int actqkv_append_kv(const actqkv_shape* shape, int batch, int m, const void* k_new, const void* v_new,
                     const int32_t* pos0, void* k_cache, void* v_cache, int64_t cache_seq_stride,
                     void* rep_keys, int64_t rep_seq_stride, int nb_capacity, void* stream);

/* The second loop of Alg. 1 with every density of the step known (Sec. 4.2, Eq. (12) with the
 * mean density of a layer still to come taken to be that layer's own density of this step):
 *   B_kv = n_layers * k_mean;  for l = 0 .. n_layers - 1:
 *     B^l = theta^l / (theta^l + sum_{j > l} theta^j) * B_kv  (B_kv if the denominator is 0);
 *     B_kv -= B^l;  E^l = min(k_cap, max(1, floor(B^l + 0.5))).
 *   theta   device [n_layers][batch] fp32: the densities actqkv_select wrote with
 *           ACTQKV_SELECT_DENSITY_ONLY, one row per layer.
 *   budget  device [n_layers][batch] fp32: B^l.   count  device [n_layers][batch] int32: E^l; pass
 *           row l as n_sel to actqkv_select with ACTQKV_SELECT_GIVEN_COUNT in layer l.
 *   budget_left  device [batch] fp32, may be NULL: what is left of B_kv (0 up to rounding: the
 *           budgets add up to n_layers * k_mean).
 * Errors: EINVAL (null, k_mean <= 0), ESHAPE (n_layers outside 1..1024, k_cap outside 1..64). */
int actqkv_cutoff_budgets(int batch, int n_layers, float k_mean, int k_cap, const float* theta, float* budget,
                          int32_t* count, float* budget_left, void* stream);

/* Start of a step of the dynamic cut-off (Sec. 4.2, Eq. (12); Alg. 1): keeps the history of
 * the layers' information densities on the device and prepares the two cut-off inputs of
 * actqkv_select for all layers of the step that begins.
 *   theta_prev  device [n_layers][batch] fp32: the densities actqkv_select reported for the
 *               layers of the step before (its `theta` output, one row per layer), or NULL
 *               for the first step; they are added to the history.
 *   theta_sum   device [batch][n_layers], n_steps device [batch], fp32: the history (sum of the
 *               densities per layer, number of steps), zero before the first step; updated.
 *   budget_remaining  device [batch]: set to n_layers * k_mean, the step's budget B_kv.
 *   theta_rest_sum    device [n_layers][batch]: row l = sum over the layers j > l of the mean
 *               density of layer j so far (theta_prior for every layer while there is no
 *               history); pass row l to actqkv_select in layer l.
 * One short kernel; nothing is read back. */
int actqkv_cutoff_next_step(int batch, int n_layers, float k_mean, float theta_prior,
                            const float* theta_prev, float* theta_sum, float* n_steps,
                            float* budget_remaining, float* theta_rest_sum, void* stream);

/* Retrieval per KV head - the alternative to the head-merged reading of the method, in which
 * every KV head, with the G query heads it serves, scores, cuts off and selects for itself.
 *
 * actqkv_score_blocks_per_head: scores [batch][Hk][score_stride]; row hk is the score of
 *   actqkv_score_blocks for the model cut down to KV head hk: mean_j <probe_kv[hk], k_j[hk]> /
 *   (|probe of group hk| * sqrt(G) * |k_j[hk]|).  probe [batch][H*D] as written by
 *   actqkv_build_probe; nb_end device int32 [batch][Hk] (one entry per row); the other
 *   arguments as in actqkv_score_blocks.
 * actqkv_select then runs on batch * Hk rows (cut-off state, idx, n_sel, theta, budget all
 *   [batch][Hk]...).
 * actqkv_retrieval_attention_per_head: as actqkv_retrieval_attention with idx [batch][Hk][k_cap]
 *   and n_sel [batch][Hk]: the query heads of group hk attend over the blocks of row hk. */
int actqkv_score_blocks_per_head(const actqkv_shape* shape, int batch, const float* probe,
                                 const void* rep_keys, int64_t seq_stride, int nb_capacity,
                                 int nb_begin, const int32_t* nb_end, float* scores,
                                 int64_t score_stride, void* stream);
int actqkv_retrieval_attention_per_head(const actqkv_shape* shape, int batch, int m, const void* q,
                                        const void* k_cache, const void* v_cache,
                                        int64_t seq_stride, int nb_capacity, const int32_t* n_ctx,
                                        const int32_t* idx, const int32_t* n_sel, int k_cap,
                                        void* out, float* lse, void* workspace, size_t ws_bytes,
                                        void* stream);

/* actqkv_retrieval_attention for a caller that runs other kernels beside the prefill attention
 * (for instance the probes, scores and selections of the next windows on a second stream, which
 * depend on earlier selections but on no attention): the launch shape is an argument of the call.
 *   first_cus  1..256: the attention fills only that many of the chip's 256 compute units and
 *            leaves the rest to the concurrent work (a single window is cut into fewer pieces;
 *            a batch of windows (m > 1, bf16, head_dim 128), whose (query tile, KV head) items go
 *            through a queue, gets that many persistent workgroups).
 *   late_cus   0, or n_kv_heads..256: a second team of that many workgroups for the same queue,
 *            launched by this call on `stream_late`, typically the stream that carries the other
 *            work, so that the team starts once that work has drained and takes its share of
 *            whatever is left in the queue.  Nobody waits: if nothing is left, or the call has no
 *            queue (m = 1, fp32, a workgroup per item already), the second team leaves at once or
 *            is not launched at all.  The output does not depend on who runs which item.
 *   stream, stream_late  both must be ordered behind the selection that wrote idx and n_sel.  The
 *            two launches share the workspace (the one case where work on two streams does); the
 *            next call on the same workspace must be ordered behind both streams.
 *   A workspace of actqkv_workspace_bytes serves every first_cus.  The other arguments, the
 *   results and the errors as in actqkv_retrieval_attention; first_cus or late_cus out of range:
 *   ACTQKV_EINVAL. */
int actqkv_retrieval_attention_teams(const actqkv_shape* shape, int batch, int m, const void* q,
                                     const void* k_cache, const void* v_cache, int64_t seq_stride,
                                     int nb_capacity, const int32_t* n_ctx, const int32_t* idx,
                                     const int32_t* n_sel, int k_cap, void* out, float* lse,
                                     void* workspace, size_t ws_bytes, int first_cus, int late_cus,
                                     void* stream, void* stream_late);

/* The first launch of a decode step: actqkv_append_kv with m = 1 and the probe of the step's
 * one-token window (actqkv_build_probe with m = 1 and no statistics: probe = the query,
 * Sec. 4.2) in ONE launch; the two are independent, and each is a few microseconds of work
 * behind a launch of its own.
 *   q_tok  [batch][H][D], storage dtype; probe, probe_kv, probe_norm as in actqkv_build_probe.
 *   The other arguments, and the errors, as in actqkv_append_kv. */
int actqkv_append_kv_probe(const actqkv_shape* shape, int batch, const void* q_tok, const void* k_new,
                           const void* v_new, const int32_t* pos0, void* k_cache, void* v_cache,
                           int64_t cache_seq_stride, void* rep_keys, int64_t rep_seq_stride,
                           int nb_capacity, float* probe, float* probe_kv, float* probe_norm,
                           void* stream);

/* Everything of a decode step that comes before the attention, in ONE call of two launches
 * instead of four: the cache update (Sec. 3.1, Eq. (4); actqkv_append_kv with m = 1), the probe
 * of the one-token window (the query itself, Sec. 4.2; actqkv_build_probe with m = 1 and no
 * statistics) and the block scores (Eq. (10); actqkv_score_blocks) in the first, the selection
 * with the cut-off (Eq. (11), Eq. (12), Alg. 1; actqkv_select) in the second.  Same results as
 * the four calls (the probe's norm, and with it the scores, up to the order of an fp32 sum);
 * what is saved is launch and drain time, which exceeds the work of the update and the probe.
 *   q_tok  [batch][H][D], storage dtype.
 *   k_new, v_new, pos0  as in actqkv_append_kv with m = 1; k_new = v_new = pos0 = NULL: no cache
 *            update (k_cache, v_cache may then be NULL too).  nb_end[s] must not reach block
 *            pos0[s] / Bs: the block that receives the token lies in the local span, and a block
 *            has representatives only once it is full.
 *   k_cache, v_cache, cache_seq_stride, rep_keys, rep_seq_stride, nb_capacity (>= 1)
 *            as in actqkv_append_kv; rep_keys is required (it is what gets scored).
 *   nb_begin, nb_end, scores, score_stride  as in actqkv_score_blocks.
 *   probe, probe_kv, probe_norm  optional outputs (NULL: not written) as in actqkv_build_probe.
 *   k_cap, flags, budget_remaining, theta_rest_sum, idx, n_sel, theta, budget
 *            as in actqkv_select; with flags & ACTQKV_DECODE_SCORES_ONLY the call ends after its
 *            first launch and none of these but k_cap is used (idx, n_sel may be NULL).
 * Errors: as in the four calls. */
int actqkv_decode_retrieve(const actqkv_shape* shape, int batch, const void* q_tok, const void* k_new,
                           const void* v_new, const int32_t* pos0, void* k_cache, void* v_cache,
                           int64_t cache_seq_stride, void* rep_keys, int64_t rep_seq_stride,
                           int nb_capacity, int nb_begin, const int32_t* nb_end, float* probe,
                           float* probe_kv, float* probe_norm, float* scores, int64_t score_stride,
                           int k_cap, int flags, float* budget_remaining,
                           const float* theta_rest_sum, int32_t* idx, int32_t* n_sel, float* theta,
                           float* budget, void* stream);

/* The selection and the attention of a decode step in ONE launch (actqkv_select followed by
 * actqkv_retrieval_attention with m = 1; Sec. 4.2, Eq. (11), Eq. (12), Alg. 1; Sec. 3.1, Eq. (3)).
 * The selection step is all latency, and an attention workgroup has that much time to spare
 * while its first keys and values are on their way: every workgroup repeats its sequence's
 * selection (identical in all of them) and then attends over what it selected.
 * Supported for bf16 storage, head_dim 128 and at most 8 query heads per KV head
 * (ACTQKV_ESHAPE otherwise: make the two calls).
 *   q [batch][1][H][D]; k_cache, v_cache, seq_stride, nb_capacity, n_ctx, out, lse, workspace
 *            as in actqkv_retrieval_attention with m = 1.
 *   scores, score_stride, nb_begin, nb_end, k_cap, flags  as in actqkv_select; the scores of
 *            blocks nb_begin .. min(nb_end[s], nb_capacity) - 1 are read.
 *   budget_in, theta_rest_sum  the cut-off state as actqkv_select reads it (both NULL: the k_cap
 *            best blocks); budget_after receives B_kv - B^l and must NOT be the array
 *            budget_in points to: all workgroups of a sequence read budget_in while one of
 *            them writes budget_after (NULL: not written).
 *   idx, n_sel (required), theta, budget (optional)  outputs as of actqkv_select.
 * Results: the selection is that of actqkv_select (the density up to the order of an fp32
 * sum, since 512 instead of 1024 threads add it up); the output is that of
 * actqkv_retrieval_attention up to fp32 summation order (the key spans are merged in another
 * order). */
int actqkv_decode_select_attention(const actqkv_shape* shape, int batch, const void* q,
                                   const void* k_cache, const void* v_cache, int64_t seq_stride,
                                   int nb_capacity, const int32_t* n_ctx, const float* scores,
                                   int64_t score_stride, int nb_begin, const int32_t* nb_end,
                                   int k_cap, int flags, const float* budget_in,
                                   const float* theta_rest_sum, float* budget_after, int32_t* idx,
                                   int32_t* n_sel, float* theta, float* budget, void* out,
                                   float* lse, void* workspace, size_t ws_bytes, void* stream);

/* A whole layer of a decode step in ONE launch: the cache update (Sec. 3.1, Eq. (4)), the probe of
 * the one-token window (the query itself, Sec. 4.2), the block scores (Eq. (10)), density, budget
 * and selection (Eq. (11), Eq. (12), Alg. 1) and the attention (Sec. 3.1, Eq. (3)) - what
 * actqkv_decode_retrieve followed by actqkv_decode_select_attention do in two.  The workgroups of
 * a sequence share its scoring, publish their scores and attend over the initial tokens and the
 * local span; then each repeats the sequence's selection and attends over the chosen blocks.  A
 * workgroup waits for the others' scores for a bounded time only (2 ms) and otherwise scores the
 * whole sequence itself, so the launch ends whatever else occupies the chip.
 * Supported for bf16 storage, head_dim 128, at most 8 query heads per KV head, batch <= 384
 * (ACTQKV_ESHAPE otherwise).
 *   q        [batch][1][H][D]: the step's queries.
 *   k_new, v_new  [batch][Hk][D]: key and value of the step's token, written to position
 *            n_ctx[s] - 1 of the caches (both NULL: the caches already hold it).
 *   k_cache, v_cache, cache_seq_stride, rep_keys, rep_seq_stride, nb_capacity
 *            as in actqkv_append_kv; rep_keys is required (it is what gets scored); the entries of
 *            a block that the token completes are written.
 *   n_ctx    device int32 [batch]: tokens in the cache including the step's token.
 *   nb_begin, nb_end, scores, score_stride  as in actqkv_score_blocks; scores of the eligible
 *            blocks are written.  nb_end[s] must not reach the block of position n_ctx[s] - 1.
 *   k_cap, flags (ACTQKV_SELECT_ENTROPY_TOPK, ACTQKV_DECODE_NO_WAIT), budget_in, theta_rest_sum,
 *   budget_after, idx, n_sel, theta, budget  as in actqkv_decode_select_attention.
 *   out, lse, workspace  as in actqkv_retrieval_attention with m = 1.
 * Results: scores and selection as the two calls give them; the output up to the order of fp32
 * sums. */
int actqkv_decode_layer(const actqkv_shape* shape, int batch, const void* q, const void* k_new,
                        const void* v_new, void* k_cache, void* v_cache, int64_t cache_seq_stride,
                        void* rep_keys, int64_t rep_seq_stride, int nb_capacity, const int32_t* n_ctx,
                        int nb_begin, const int32_t* nb_end, float* scores, int64_t score_stride, int k_cap,
                        int flags, const float* budget_in, const float* theta_rest_sum, float* budget_after,
                        int32_t* idx, int32_t* n_sel, float* theta, float* budget, void* out, float* lse,
                        void* workspace, size_t ws_bytes, void* stream);

/* Selected blocks from a block store into a working cache (Sec. 3.1: the cache may be kept
 * in CPU memory).
 *   k_store, v_store  the whole context in the blocked cache layouts,
 *            [batch][nb_store][Hk][Bs][D] and [batch][nb_store][Hk][D][Bs]; any memory the
 *            device can read in place: pinned host memory (hipHostMalloc) or device memory.
 *            store_seq_stride = elements between two sequences.
 *   idx, n_sel, k_cap  as written by actqkv_select (device memory).
 *   k_cache, v_cache   device working cache of nb_capacity blocks; block idx[s][j], j < n_sel[s],
 *            is copied to block slot0 + j (slot0 + k_cap <= nb_capacity).  The caller keeps the
 *            initial tokens in the blocks before slot0 and the local span and the window in the
 *            blocks from slot0 + k_cap on, i.e. at positions shifted by a multiple of Bs, and
 *            passes n_ctx in those shifted positions to actqkv_retrieval_attention.
 *   idx_slots [batch][k_cap] int32, device, may be NULL: slot0 + j for j < n_sel[s], else -1 -
 *            the selection actqkv_retrieval_attention takes on the working cache.
 * Entries of idx outside [0, nb_store) are skipped (their idx_slots entry is -1).
 * Errors: EINVAL (null, slots outside the cache), ESHAPE, EALIGN. */
int actqkv_gather_blocks(const actqkv_shape* shape, int batch, const void* k_store,
                         const void* v_store, int64_t store_seq_stride, int nb_store,
                         const int32_t* idx, const int32_t* n_sel, int k_cap, void* k_cache,
                         void* v_cache, int64_t cache_seq_stride, int nb_capacity, int slot0,
                         int32_t* idx_slots, void* stream);

/* A plain copy of `bytes` bytes (a multiple of 16; both pointers memory the device can access -
 * device memory or pinned host memory -, 16-byte aligned, not overlapping) done by one kernel
 * with 16-byte loads and stores.  Not a step of the method: between device buffers it reads and
 * writes exactly `bytes` bytes of HBM, which calibrates the hardware traffic counters against a
 * known size; with the cache kept in host memory (see actqkv_gather_blocks) it carries the local
 * span from one working cache to the next and new blocks back to the host store. */
int actqkv_copy_bytes(void* dst, const void* src, size_t bytes, void* stream);

/* Message of the last error on this thread ("" if none). */
const char* actqkv_last_error(void);

/* ACTQKV_VERSION of the built library. */
int actqkv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ACTQKV_H */
