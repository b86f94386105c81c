/*
 * d2o.h - C ABI of the MI355X (gfx950) implementation of the D2O KV-cache compression
 * hot path (Dynamic Discriminative Operations, arxiv 2406.13035).
 *
 * The library never allocates device memory: the caller supplies two device workspaces
 * whose sizes d2o_workspace_bytes() reports.  All device work is enqueued on the stream
 * the caller passes (a hipStream_t, typed void* here so the header needs no HIP include;
 * NULL = the default stream).  Unless stated otherwise a call returns without
 * synchronising: d2o_create, d2o_reset, d2o_prefill_attend, d2o_compress_layer,
 * d2o_prefill_compress and d2o_decode_step only enqueue kernels and read no host memory after
 * they return; the calls that move data to or from host buffers (density, scores, cache,
 * events, timing) and d2o_layer_reserve wait for the stream and say so below.  Every
 * function returns 0 on success or a negative d2o_status; d2o_last_error() gives the
 * message of the last failure on a context.
 *
 * Pointer kinds: "device" = device memory, "host" = ordinary host memory.
 * Token identity across the ABI is the ORIGINAL TOKEN POSITION (prompt tokens 0..n-1,
 * generated tokens n, n+1, ...), never a physical cache slot.
 *
 * Notation (paper, Sec. 3-4): B batch, L layers, Hq query heads, Hkv KV heads, G = Hq/Hkv,
 * d head dimension, N prompt length, S_l cache budget of layer l (slots per KV head),
 * T attention-sink tokens, M recent window, beta EMA constant, tau EMA threshold.
 */
#ifndef D2O_H
#define D2O_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct d2o_ctx d2o_ctx;

typedef enum { D2O_F32 = 0, D2O_BF16 = 1 } d2o_dtype;

typedef enum {
  D2O_OK = 0,
  D2O_ERR_INVALID_ARG = -1, /* null pointer, index out of range, inconsistent sizes        */
  D2O_ERR_UNSUPPORTED = -2, /* head_dim / dtype combination without a kernel               */
  D2O_ERR_CAPACITY = -3,    /* cache slots or a workspace too small                        */
  D2O_ERR_STATE = -4,       /* call order violated (compress before attend, ...)           */
  D2O_ERR_HIP = -5          /* a HIP runtime call failed                                   */
} d2o_status;

/* Immutable after d2o_create. */
typedef struct {
  int32_t batch;          /* B                                                             */
  int32_t n_layers;       /* L                                                             */
  int32_t n_q_heads;      /* Hq, a multiple of n_kv_heads with G = Hq / Hkv in {1, 2, 4, 8}  */
  int32_t n_kv_heads;     /* Hkv                                                           */
  int32_t head_dim;       /* d: 64 or 128 for D2O_F32, 128 for D2O_BF16                    */
  int32_t max_prompt_len; /* largest n any prefill call will pass                          */
  int64_t slots_per_seq;  /* cache capacity per (sequence, KV head) over all layers:       */
                          /* must hold sum_l (S_l + 1)                                     */
  int32_t dtype;          /* d2o_dtype of Q, K, V, O and of the cache                      */
  int32_t n_sink;         /* T of Eq. 7: the first T prompt tokens are always kept         */
  double beta;            /* Eq. 10 smoothing constant, 0 <= beta < 1                      */
  double tau_force;       /* NaN: threshold of Eq. 10.  +inf: never merge (pure eviction). */
                          /* -inf: merge every evicted token.                              */
  int32_t out_f32;        /* 0: attention outputs (O, out) in `dtype`; 1: in fp32, which    */
                          /* keeps the fp32 accumulator's precision (bf16 storage alone     */
                          /* costs up to 2^-8 relative)                                     */
  int32_t merge_average;  /* 0: similarity-weighted merge, Eq. 11-12.  1: average merging,  */
                          /* the alternative of the merge-policy ablation (Sec. 5): the     */
                          /* plain mean of the retained row and the tokens merged into it   */
  int32_t max_append;     /* largest block of tokens d2o_append_chunk will be given (0 or 1: */
                          /* single-token generation steps only).  A layer's cache region    */
                          /* holds S_l + max(1, max_append) rows, so slots_per_seq must hold */
                          /* sum_l (S_l + max(1, max_append)), and S_l + max_append must not */
                          /* exceed max_prompt_len (the block's token-level stages reuse the */
                          /* prompt-phase scratch)                                           */
  int32_t split_rows;     /* generation steps: a head whose cache holds more entries than    */
                          /* this has its closing work (normaliser, score update, eviction   */
                          /* choice) split over several workgroups in two extra launches     */
                          /* instead of done by one.  0: chosen per launch (half a percent   */
                          /* of the rows the launch streams, within [6144, 16384]).          */
                          /* Otherwise at least 256.  A tuning knob: events and scores do    */
                          /* not depend on it, outputs only in fp32 summation order.         */
  int32_t cache_fp8;      /* 1: the cache stores a K or V row as d codes of the 8-bit float   */
                          /* format E4M3 and one power of two per row (the smallest that      */
                          /* brings the row's largest magnitude to 448 or below; round to     */
                          /* nearest even).  Rows are encoded when they enter the cache (after */
                          /* prompt compression, new tokens before they are attended to,      */
                          /* merged rows); every read sees the decoded values.  The paper      */
                          /* names KV-cache quantisation as future work and fixes no format.   */
                          /* Needs dtype D2O_BF16.  0: cache in `dtype`.                       */
} d2o_config;

/* A strided tensor whose last dimension (d) is contiguous.  Strides are in elements.
 * Prefill tensors are [b][head][token][d]; decode tensors are [layer][b][head][d] and use
 * stride_n as the stride between consecutive layers. */
typedef struct {
  void* ptr;        /* device */
  int64_t stride_b;
  int64_t stride_h;
  int64_t stride_n;
} d2o_view;

/* Sizes in bytes of the two device workspaces a context needs: `persistent` holds the
 * compressed cache, per-key scores and statistics for the context's life; `scratch` holds
 * per-call temporaries (contents are undefined between calls, except that the prefill
 * events of the most recent d2o_compress_layer call stay readable until the next prefill
 * call).  Errors: INVALID_ARG, UNSUPPORTED. */
int d2o_workspace_bytes(const d2o_config* cfg, size_t* persistent, size_t* scratch);

/* Creates a context over caller-owned device workspaces (256-byte aligned, at least the
 * sizes reported above; the caller keeps them alive and untouched until d2o_destroy).
 * The persistent workspace is cleared on `stream`.  Errors: INVALID_ARG, UNSUPPORTED,
 * CAPACITY (workspace too small), HIP. */
int d2o_create(const d2o_config* cfg, void* persistent_dev, size_t persistent_bytes,
               void* scratch_dev, size_t scratch_bytes, void* stream, d2o_ctx** out);

/* Frees the host-side context only. */
void d2o_destroy(d2o_ctx* ctx);

/* Message of the last error on this context ("" if none); valid until the next call. */
const char* d2o_last_error(const d2o_ctx* ctx);

/* Forgets all layers' caches, scores and thresholds (the workspaces are reused). */
int d2o_reset(d2o_ctx* ctx, void* stream);

/* Upstream step (Sec. 3 Eq. 1): Q = X W_Q, K = X W_K, V = X W_V of one layer as one matrix
 * product, with the rotary position embedding of the evaluated models applied to queries and
 * keys (feature i < d/2 pairs with i + d/2; angle = position * rope_base^(-2i/d); positions pos0,
 * pos0 + 1, ... along the tokens of every sequence), results rounded once to `dtype` and written
 * in the layout the attention calls read.  No context is needed.
 * X: device [batch * n][hidden]; W: device [(Hq + 2 Hkv) * d][hidden] (a row = one output
 * feature; queries first, then keys, then values), both contiguous and 16-byte aligned;
 * Q: [B][Hq][n][d], K, V: [B][Hkv][n][d] views.  Built for D2O_BF16, d = 128, hidden a multiple
 * of 32 (fp32 accumulation on the matrix cores).  Enqueues only.
 * Errors: INVALID_ARG, UNSUPPORTED (other dtype / head_dim / hidden), HIP. */
int d2o_qkv_project(int32_t batch, int32_t n, int32_t hidden, int32_t n_q_heads, int32_t n_kv_heads,
                    int32_t head_dim, int32_t dtype, const void* X, const void* W, d2o_view Q,
                    d2o_view K, d2o_view V, int32_t pos0, double rope_base, void* stream);

/* Prompt encoding, attention part (Sec. 4.1 Eq. 4; Sec. 4.2.1 Eq. 6, prompt case).
 * For one layer computes, per query head, O = softmax(Q K^T / sqrt(d)) V with a causal
 * mask; per KV head the cumulative attention score of every key (column sums of the
 * attention matrix, added over the G query heads of the group) and, per query head, the
 * population variance of its column sums, whose mean over heads is the layer's density
 * statistic F.  Scores and statistics are kept in the context.
 * Q, O: [B][Hq][n][d]; K, V: [B][Hkv][n][d]; n <= max_prompt_len.  O.ptr may be NULL to skip
 * the output write; O holds fp32 when out_f32 is set (strides in its own elements).  Errors: INVALID_ARG, STATE (layer already compressed), HIP. */
int d2o_prefill_attend(d2o_ctx* ctx, int32_t layer, d2o_view Q, d2o_view K, d2o_view V,
                       int32_t n, d2o_view O, void* stream);

/* Copies the density statistics to the host and waits for them (synchronises `stream`).
 * F_layers: host [B][L] (layers not yet attended read as NaN); F_heads: host
 * [B][L][Hq] per-query-head variances, may be NULL.  Errors: INVALID_ARG, HIP. */
int d2o_get_density(d2o_ctx* ctx, double* F_layers, double* F_heads, void* stream);

/* Dynamic layer budgets (Sec. 4.1 Eq. 5, App. A.2): S_l proportional to exp(-F_l) with
 * sum_l S_l = total_budget, every S_l clipped to [min_budget, seq_len] (the unique clipped
 * proportional split), shares floored and the leftover units given to the largest
 * fractional parts (ties: lower layer).  Pure host function on host arrays, fp64.
 * Errors: INVALID_ARG (also when n_layers*min_budget <= total_budget <= n_layers*seq_len
 * fails or an F is not finite). */
int d2o_allocate_budgets(const double* F, int32_t n_layers, int32_t seq_len,
                         int64_t total_budget, int32_t min_budget, int32_t* S_out);

/* The designs of the layer allocation factor alpha_l that the allocation-policy analysis of
 * Sec. 5 compares.  SOFTMAX is Eq. 5 (weight exp(-F_l)), RECIPROCAL weighs a layer by 1/F_l
 * (every F_l must be positive), UNIFORM by 1 (alpha_l = rho): these three split total_budget
 * exactly as d2o_allocate_budgets does (same clipping and integer rule) and differ only in
 * the weight.  EXP_DECAY takes alpha_l = exp(-F_l) as the layer's own ratio: S_l =
 * floor(exp(-F_l) * seq_len) clipped to [min_budget, seq_len]; it has no sum constraint and
 * ignores total_budget. */
typedef enum {
  D2O_ALLOC_SOFTMAX = 0,
  D2O_ALLOC_RECIPROCAL = 1,
  D2O_ALLOC_EXP_DECAY = 2,
  D2O_ALLOC_UNIFORM = 3
} d2o_alloc_policy;

/* d2o_allocate_budgets with the design of alpha_l chosen by `policy` (SOFTMAX gives the same
 * result as d2o_allocate_budgets).  Pure host function on host arrays, fp64.
 * Errors: INVALID_ARG (unknown policy, infeasible bounds or total, an F that is not finite,
 * or not positive under RECIPROCAL). */
int d2o_allocate_budgets_policy(int32_t policy, const double* F, int32_t n_layers, int32_t seq_len,
                                int64_t total_budget, int32_t min_budget, int32_t* S_out);

/* Replaces a layer's per-key scores by host values ([B][Hkv][n] floats) as if
 * d2o_prefill_attend had produced them (used to drive the token-level stages from given
 * scores).  Synchronises `stream`.  Errors: INVALID_ARG, STATE, HIP. */
int d2o_scores_import(d2o_ctx* ctx, int32_t layer, const float* scores, int32_t n, void* stream);

/* Copies a layer's per-key scores to the host ([B][Hkv][n] floats); synchronises. */
int d2o_scores_export(d2o_ctx* ctx, int32_t layer, float* scores, int32_t n, void* stream);

/* Prompt encoding, token-level operation for one layer (Sec. 4.2): eviction by cumulative
 * score (Eq. 7-8: keep T sinks, the top S-T-M scores of the middle, the last M tokens; equal
 * scores: the lower position is kept), nearest-neighbour matching of evicted keys to
 * retained keys by cosine similarity (Eq. 9, first maximum in ascending position), the
 * initial threshold tau_0 = mean of the best similarities (Eq. 10) and the similarity-
 * weighted merge of passing tokens into their matches (Eq. 11-12, weights
 * e/Z and exp(u)/Z with Z = e + sum exp(u)).  Requires the layer's scores
 * (d2o_prefill_attend or d2o_scores_import) and the same K, V.
 * budget, recent: host [B], the layer's S_l and M per sequence (read before the call returns);
 * budget >= n keeps everything.  Enqueues only.  Errors: INVALID_ARG (budget < T + M, ...),
 * STATE, CAPACITY, HIP. */
int d2o_compress_layer(d2o_ctx* ctx, int32_t layer, d2o_view K, d2o_view V, int32_t n,
                       const int32_t* budget, const int32_t* recent, void* stream);

/* d2o_compress_layer with a budget and a recent window of its own for every KV head: budget,
 * recent are host [B][Hkv] (per-head allocation, App. A.8).  Everything else as above. */
int d2o_compress_layer_heads(d2o_ctx* ctx, int32_t layer, d2o_view K, d2o_view V, int32_t n,
                             const int32_t* budget, const int32_t* recent, void* stream);

/* Per-head dynamic allocation (App. A.8): alpha_l^h proportional to exp(-F^{l,h}) over ALL
 * (layer, head) pairs, S_l^h = alpha_l^h * total_budget, the layer's share being the sum over
 * its heads.  F_heads: host [L][Hq] per-query-head variances (one sequence's slice of what
 * d2o_get_density returns); a KV head's statistic is the mean over the G query heads it serves;
 * total_budget counts cache rows per sequence over all layers and KV heads (rho * N * L * Hkv).
 * Bounds and integer rule as in d2o_allocate_budgets.  S_out: host [L][Hkv].  Pure host
 * function, fp64.  Errors: INVALID_ARG. */
int d2o_allocate_budgets_heads(const double* F_heads, int32_t n_layers, int32_t n_q_heads,
                               int32_t n_kv_heads, int32_t seq_len, int64_t total_budget,
                               int32_t min_budget, int32_t* S_out);

/* d2o_prefill_attend followed by d2o_compress_layer with caller-chosen budgets. */
int d2o_prefill_compress(d2o_ctx* ctx, int32_t layer, d2o_view Q, d2o_view K, d2o_view V,
                         int32_t n, d2o_view O, const int32_t* budget, const int32_t* recent,
                         void* stream);

/* One generation step on layers [layer, layer + n_layers_in_call) (Sec. 3 Eq. 2-3; Sec. 4.2
 * Eq. 6-12): append (k_new, v_new), attend over the cache, add the softmax rows of the G
 * query heads to the scores, and, when a cache exceeds its budget, evict one token by
 * Eq. 7-8 (equal scores: the later position is evicted), match it (Eq. 9), update the EMA
 * threshold (Eq. 10, update first, then test) and merge or discard it (Eq. 11-12).
 * q, out: [layers][B][Hq][d]; k_new, v_new: [layers][B][Hkv][d].
 * Errors: INVALID_ARG, STATE (a layer not compressed), CAPACITY, HIP. */
int d2o_decode_step(d2o_ctx* ctx, int32_t layer, int32_t n_layers_in_call, d2o_view q,
                    d2o_view k_new, d2o_view v_new, d2o_view out, void* stream);

/* A block of m new tokens on one layer (the chunked / multi-turn form of a generation step:
 * Sec. 3 Eq. 2-3 and Sec. 4.2 Eq. 6-12 applied to m tokens at once).  Token i of the block is
 * appended, attends to the cache and to the block's tokens up to itself, and adds its softmax
 * rows to the cumulative scores (Eq. 6, no eviction inside the block); then every cache that
 * exceeds its budget evicts count - S_l tokens together by Eq. 7-8, matches them on the keys as
 * they are (Eq. 9), updates the threshold with the step's mean best similarity, tau <- beta *
 * mean + (1 - beta) * tau (tau <- mean while unset; Eq. 10 with several evicted tokens in one
 * step), and merges the passing ones (Eq. 11-12).  m = 1 gives the results of d2o_decode_step.
 * Q, O: [B][Hq][m][d]; K, V: [B][Hkv][m][d] (views as for d2o_prefill_attend); 1 <= m <=
 * max_append.  Enqueues only.  Errors: INVALID_ARG, STATE (layer not compressed), CAPACITY, HIP. */
int d2o_append_chunk(d2o_ctx* ctx, int32_t layer, d2o_view Q, d2o_view K, d2o_view V, int32_t m,
                     d2o_view O, void* stream);

/* What the most recent d2o_append_chunk call did on one (sequence, KV head): evicted positions
 * [n_evi] ascending and per evicted token its match (position), best similarity and whether it
 * passed the threshold.  Host buffers of max_append + budget entries each; any may be NULL.
 * Synchronises `stream`. */
int d2o_append_events(d2o_ctx* ctx, int32_t layer, int32_t b, int32_t kv_head, int32_t* evicted_pos,
                      int32_t* n_evi, int32_t* target_pos, double* u_star, uint8_t* passed,
                      void* stream);

/* d2o_decode_step for callers that cannot allocate or hand over scratch memory at the time of
 * the call: code under HIP graph capture, tight serving loops, harnesses that forbid
 * allocation.  Same arguments, same results (bit for bit) and same errors as d2o_decode_step,
 * but the step's temporaries (per-slot softmax terms, per-chunk partial outputs and records,
 * the fp64 operand vectors) live in a static device array inside the library instead of the
 * context's scratch workspace, and the call makes no allocation of any kind (no device or
 * host memory, no events: kernel timing is off for these calls).  The array holds 64 MiB
 * (67108864 bytes) per GPU from the moment the library's code is loaded there until the
 * process ends; a context whose decode step needs more (about 10 G + 3 bytes per cache slot
 * of slots_per_seq, sequence and KV head, plus G + 3 KiB per layer, sequence and KV head at
 * d = 128) gets D2O_ERR_CAPACITY and nothing is launched.  All contexts on a GPU share the array, which keeps the last call's
 * contents: calls that overlap in time on one GPU (different streams or threads) race; calls
 * ordered on one stream do not.  Nothing is carried in it from one step to the next, so a
 * context may mix the two entry points freely. */
int d2o_decode_step_static(d2o_ctx* ctx, int32_t layer, int32_t n_layers_in_call, d2o_view q,
                           d2o_view k_new, d2o_view v_new, d2o_view out, void* stream);

/* Reserves a layer's cache region for the given budgets without running the prefill
 * stages (so that d2o_cache_import can fill it).  n is the prompt length the positions
 * refer to.  Writes the layer's geometry on the default stream and waits for it.
 * Errors: INVALID_ARG, STATE (already reserved), CAPACITY, HIP. */
int d2o_layer_reserve(d2o_ctx* ctx, int32_t layer, int32_t n, const int32_t* budget,
                      const int32_t* recent);

/* Cache of one (layer, sequence, KV head) to host buffers, rows in ascending token position:
 * K, V [count][d] in the cache dtype, score [count], pos [count]; buffers must hold
 * budget+1 rows.  Any pointer may be NULL.  Synchronises `stream`. */
int d2o_cache_export(d2o_ctx* ctx, int32_t layer, int32_t b, int32_t kv_head, void* K, void* V,
                     double* score, int32_t* pos, int32_t* count, double* tau, void* stream);

/* Host buffers into the cache of one (layer, sequence, KV head) of a reserved layer;
 * count <= budget, `next_pos` = position the next generated token will get (same for every
 * head of the layer).  The generation steps protect the recent window by position (the
 * last M positions before the new token), which equals the last M cache entries of Eq. 7
 * only while those positions are all present: an imported cache must hold every position
 * of [next_pos - M, next_pos), as every cache this library produces does.
 * Synchronises `stream`. */
int d2o_cache_import(d2o_ctx* ctx, int32_t layer, int32_t b, int32_t kv_head, const void* K,
                     const void* V, const double* score, const int32_t* pos, int32_t count,
                     double tau, int32_t next_pos, void* stream);

/* What the last decode step did on one layer, host arrays [B][Hkv]: position of the evicted
 * token (-1 none), position it was merged into (-1 discarded / none), its best similarity
 * (NaN none).  Synchronises `stream`. */
int d2o_last_events(d2o_ctx* ctx, int32_t layer, int32_t* evicted_pos, int32_t* target_pos,
                    double* u_star, void* stream);

/* Diagnostic: how many evictions of generation steps, over all layers and heads since d2o_create
 * or d2o_reset, took a token that was not among the candidates predicted one step ahead (each
 * costs the head's closing workgroup a second pass over the head's keys; the first step after
 * d2o_cache_import always does).  Results never depend on the prediction.  Synchronises `stream`. */
int d2o_candidate_misses(d2o_ctx* ctx, int64_t* misses, void* stream);

/* What the most recent d2o_compress_layer call did on one (sequence, KV head): retained
 * positions [n_ret] and evicted positions [n_evi] ascending, and per evicted token its
 * match (position), best similarity and whether it passed the threshold.  Host buffers of n
 * entries each; any may be NULL.  Synchronises `stream`. */
int d2o_prefill_events(d2o_ctx* ctx, int32_t layer, int32_t b, int32_t kv_head,
                       int32_t* retained_pos, int32_t* n_ret, int32_t* evicted_pos,
                       int32_t* n_evi, int32_t* target_pos, double* u_star, uint8_t* passed,
                       void* stream);

/* Kernel timing aid for benchmarks (not part of the method).  While enabled (on >= 1), launches
 * of the kernels below are bracketed by two HIP events recorded on the launch stream: every
 * launch of the prompt-phase kernels, and every on-th launch of the two decode kernels (the
 * on-th, 2 on-th, ... after enabling; the events of a decode step cost it about 3 % at the
 * largest configuration; on = 1 times every step).  d2o_timing_read synchronises `stream`, returns the summed duration in milliseconds and
 * the number of timed launches of one kernel since the last read of that kernel, and forgets
 * them. */
typedef enum {
  D2O_K_ATTN_FWD = 0,      /* prefill attention, pass 1 (O and row log-sum-exp)            */
  D2O_K_COLSUM = 1,        /* prefill attention, pass 2 (per-key column sums)              */
  D2O_K_SELECT = 2,
  D2O_K_MATCH_FILTER = 3,  /* matrix-core cosine candidate filter                          */
  D2O_K_MATCH_REFINE = 4,  /* exact fp64 cosine / arg-max                                  */
  D2O_K_MERGE = 5,
  D2O_K_DECODE_ATTEND = 6,  /* attention over the cache + score update + evict/merge         */
  D2O_K_DECODE_PREPARE = 7, /* append of the new token, operand set-up                      */
  D2O_K_DECODE_CLOSE = 8,   /* closing work of very large heads, split over workgroups        */
  D2O_K_COUNT = 9
} d2o_kernel_id;
int d2o_timing_enable(d2o_ctx* ctx, int32_t on);
int d2o_timing_read(d2o_ctx* ctx, int32_t kernel_id, double* total_ms, int64_t* launches,
                    void* stream);

#ifdef __cplusplus
}
#endif
#endif /* D2O_H */
