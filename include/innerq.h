/*
 * innerq.h -- C ABI of libinnerq: decode attention over a KV cache quantised
 * group-wise along the inner dimension (InnerQ, arXiv 2602.23200), for AMD
 * MI355X (gfx950).
 *
 * Conventions that hold for every entry point
 *   - Plain C: no C++ types, no exceptions.  Every call returns an
 *     innerq_status_t (0 = OK, negative = error).  On error nothing has been
 *     launched and no buffer has been touched.
 *   - Every data pointer is DEVICE memory owned by the caller unless the
 *     comment says "host".  The library never allocates, frees or keeps device
 *     memory, never synchronises, and enqueues all its work on the HIP stream
 *     the caller passes (a hipStream_t cast to void*; NULL = the null stream).
 *   - Device pointers must be 16-byte aligned (the kernels use 128-bit loads).
 *   - The library keeps no state of a cache between calls: the token counter lives in the
 *     caller's innerq_cache_t (host memory) and is the same for the whole batch.  What it does
 *     keep, process-wide and host-side only: the kernel choice set by
 *     innerq_select_inner_kernel, the one-shot per-thread request of
 *     innerq_profile_next_attention, remembered answers of occupancy / device-attribute
 *     queries (atomics; set once), and the device address of the static workspace of
 *     innerq_decode_attention_static.
 *   - The exception to "on error nothing has been launched": innerq_decode_step makes two
 *     launches, and INNERQ_E_HIP from the second one arrives after the first was enqueued
 *     (every argument check is done before the first).
 *   - Inputs are assumed finite; NaN/Inf in K, V or q give unspecified output.
 *
 * Notation (paper, Sections "KV Caching", "Quantization Scheme"):
 *   B batch, Hq query heads, Hk kv heads (query head hq reads kv head
 *   hq / (Hq/Hk)), d = head_dim, G = group size, b = bits, N = cached tokens.
 *
 * Partition of the N cached tokens of one tensor (Eq.
 * kv_cache_init_quantized_window; Section "High-precision Window"):
 *   sink      tokens [0, n_s)               fp16, n_s = min(N, w_sink)
 *   quantised tokens [w_sink, w_sink + n_q) packed codes
 *   recent    tokens [w_sink + n_q, N)      fp16 ring, slot = token index mod slots
 *   with n_q = max(0, N - w_sink - w_recent), rounded DOWN to a multiple of G
 *   for a tensor whose groups run along tokens (such a tensor can only quantise
 *   G tokens at a time: Section "Latency", eviction pattern).
 *
 * Storage layout (this library's own; the paper does not define one)
 *   "per-token" form (groups of G consecutive channels inside one token;
 *   keys under inner grouping, values under outer grouping):
 *     codes  u8   [B][Hk][capacity][d*b/8]   channel c at bit b*c of the row (little-endian)
 *     scales fp16 [B][Hk][capacity][d/G]
 *     zeros  fp16 [B][Hk][capacity][d/G]
 *   "per-channel" form (groups of G consecutive tokens inside one channel;
 *   values under inner grouping, keys under outer grouping):
 *     codes  u8   [B][Hk][capacity/G][d][G*b/8]   token j of the group at bit b*j
 *     scales fp16 [B][Hk][capacity/G][d]
 *     zeros  fp16 [B][Hk][capacity/G][d]
 *   b = 3 (the width of the paper's presets, Section "Experimental Setup"): each packed run
 *   (the d*3/8 bytes of a token row; the G*3/8 bytes of one channel of one token-group) is two
 *   planes one after the other: the low two bits of every field as 2-bit fields (field i at
 *   bit 2*i), then the high bits as 1-bit fields (field i at bit i).
 *   fp16 form (kind INNERQ_KIND_FP16): codes fp16 [B][Hk][capacity][d], no scales/zeros.
 *   Store row r holds token w_sink + r.
 *   Stored b-bit field: the unsigned code of an asymmetric group (Eq. asym_quant),
 *   code + 2^(b-1) for a symmetric group (signed code, Section "Asymmetric and
 *   Symmetric Quantization").  The sign BIT of the stored scale is the mask M of
 *   Section "Hybrid Quantization" (set = asymmetric); zeros holds Z for an
 *   asymmetric group and +0 otherwise.  Decoding is Eq. hybrid_dequant:
 *   x^ = |scale| * code + M * zero.
 *   Windows: k_sink, v_sink fp16 [B][Hk][w_sink][d];
 *   k_recent, v_recent fp16 [B][Hk][slots][d], slots = w_recent + 1 for a per-token
 *   or fp16 tensor and w_recent + G for a per-channel tensor (the window itself holds
 *   w_recent, resp. up to w_recent + G - 1, tokens; the spare slot lets a decode step
 *   write the new token without waiting for the evicted one to be read).
 */
#ifndef INNERQ_H
#define INNERQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  INNERQ_OK = 0,
  INNERQ_E_NULL = -1,        /* a required pointer is NULL */
  INNERQ_E_ARG = -2,         /* inconsistent or out-of-range argument */
  INNERQ_E_UNSUPPORTED = -3, /* valid in the paper, not built here (e.g. group = 128) */
  INNERQ_E_CAPACITY = -4,    /* the cache cannot hold that many tokens */
  INNERQ_E_ALIGN = -5,       /* a device pointer is not 16-byte aligned */
  INNERQ_E_WORKSPACE = -6,   /* workspace smaller than innerq_workspace_bytes() */
  INNERQ_E_HIP = -7          /* a kernel launch failed */
} innerq_status_t;

/* Quantisation mode of a tensor (Sections "Asymmetric and Symmetric
 * Quantization", "Hybrid Quantization"). */
typedef enum { INNERQ_SYM = 0, INNERQ_ASYM = 1, INNERQ_HYBRID = 2 } innerq_mode_t;

/* Grouping of the cache.  INNER is the method (Section "InnerQ": keys per-token
 * group-wise, values per-channel group-wise).  OUTER (keys per-channel, values
 * per-token: the layout the paper compares against) and FP16 (no quantisation)
 * exist so that the same calls drive the comparison kernels. */
typedef enum { INNERQ_KIND_INNER = 0, INNERQ_KIND_OUTER = 1, INNERQ_KIND_FP16 = 2 } innerq_kind_t;

typedef struct {
  int32_t batch, n_q_heads, n_kv_heads, head_dim; /* head_dim = 128; n_q_heads % n_kv_heads == 0 */
  int32_t bits;            /* width of the key codes (and of the value codes unless v_bits is set): 2, 3 or 4 */
  int32_t group;           /* 32 or 64; head_dim % group == 0 */
  int32_t w_sink;          /* >= 0 */
  int32_t w_recent;        /* >= 1 */
  int32_t k_mode, v_mode;  /* innerq_mode_t */
  int32_t sym_denominator; /* symmetric scale = max|g| / den: 0 -> den = 2^(b-1)-1 (nothing
                              saturates), 1 -> den = 2^b-1 (the formula as printed; codes saturate
                              at -2^(b-1) and 2^(b-1)-1) */
  int32_t kind;            /* innerq_kind_t */
  int64_t capacity_tokens; /* most tokens the cache may ever hold; a multiple of group */
  int32_t v_bits;          /* width of the value codes: 2, 3 or 4; 0 = same as bits, which is then the
                              width of both (the paper's Hybrid and Small presets pair 3-bit keys
                              with 2-bit values: Section "Experimental Setup") */
  int32_t sparse_zeros;    /* 0 or 1; a hint for innerq_decode_attention on inner-grouped caches whose value
                              mode is INNERQ_HYBRID, results identical either way.  0: zero-points are streamed
                              with the codes (right when many groups are asymmetric).  1: a zero-point is read
                              only where its group's flag is set, so 128-byte lines of zero-points that hold no
                              asymmetric group are never fetched (Section "Sparsity of M": the paper measures
                              about 1 % asymmetric groups and leaves exploiting that to future work). */
  int64_t page_pool_pages; /* 0: the quantised store is contiguous per sequence (the layout above).
                              > 0: a paged store (this library's own; Section "Limitations and Future Work"
                              leaves integration with serving systems open).  The six store buffers
                              (codes, scales, zeros of K and V) are then pools of this many pages.  A page holds
                              64 consecutive store rows of one sequence for all kv heads, in the layout above
                              read with B = page_pool_pages and capacity = 64; cache->page_table names the page
                              of every 64-row block of every sequence.  capacity_tokens must be a multiple of
                              64 and is then only the most tokens ONE sequence may hold (the length of a
                              page-table row); the windows (sink, recent) stay per sequence. */
} innerq_config_t;

typedef struct {
  void *k_codes, *k_scales, *k_zeros; /* device; zeros may be NULL when the mode is INNERQ_SYM; */
  void *v_codes, *v_scales, *v_zeros; /* scales and zeros are NULL for INNERQ_KIND_FP16 */
  void *k_sink, *v_sink;              /* device, may be NULL when w_sink == 0 */
  void *k_recent, *v_recent;          /* device */
  int64_t n_tokens;                   /* host: tokens cached so far; updated by innerq_quantize_append */
  int64_t store_ahead_tokens;         /* host, maintained by the library: the quantised store holds every row
                                         that a cache of this many tokens needs.  n_tokens after an ordinary
                                         append; n_tokens + 1 once the store has been run one step ahead
                                         (innerq_quantize_ahead, innerq_append_deferred, innerq_decode_step),
                                         which innerq_decode_attention_next and innerq_decode_step require.
                                         Zero-initialise it with the struct; to reuse the buffers for a new
                                         sequence set it and n_tokens back to 0. */
  const int32_t *page_table;          /* device, int32 [B][capacity_tokens / 64], 4-byte aligned; read only when
                                         cfg->page_pool_pages > 0 (else may be NULL).  Entry [b][j] is the pool page
                                         that holds store rows 64 j .. 64 j + 63 of sequence b.  Owned and filled by
                                         the caller (the allocator is the serving system's): before a call, every
                                         block the store reaches after that call (rows below the quantised count of
                                         innerq_partition, for the token count the call leaves, plus one token for the
                                         calls that run the store a step ahead) must name a page no other live block
                                         uses.  Entries beyond that are not read for data; an entry outside
                                         [0, page_pool_pages) is clamped into the pool, never followed out of it. */
} innerq_cache_t;

typedef enum {
  INNERQ_BUF_K_CODES = 0, INNERQ_BUF_K_SCALES, INNERQ_BUF_K_ZEROS,
  INNERQ_BUF_V_CODES, INNERQ_BUF_V_SCALES, INNERQ_BUF_V_ZEROS,
  INNERQ_BUF_K_SINK, INNERQ_BUF_V_SINK, INNERQ_BUF_K_RECENT, INNERQ_BUF_V_RECENT,
  INNERQ_BUF_COUNT
} innerq_buffer_t;

/* Host-only helpers.  innerq_validate_config returns INNERQ_OK or the reason
 * the configuration is rejected.  innerq_buffer_bytes gives the exact size of
 * one cache buffer (0 for a buffer the configuration does not use, and for an
 * invalid configuration).  innerq_workspace_bytes gives the size of the
 * split-K scratch innerq_decode_attention needs (partial max, sum and output
 * per query head and token split). */
int innerq_validate_config(const innerq_config_t *cfg);
size_t innerq_buffer_bytes(const innerq_config_t *cfg, int which /* innerq_buffer_t */);
size_t innerq_workspace_bytes(const innerq_config_t *cfg);
const char *innerq_status_string(int status);

/* Counts of the partition above for tensor which = 0 (K) or 1 (V) when n_tokens
 * are cached.  Host-only; out pointers are host memory and may be NULL. */
int innerq_partition(const innerq_config_t *cfg, int which, int64_t n_tokens,
                     int64_t *n_sink, int64_t *n_quantised, int64_t *n_recent);

/* Per-channel key normalisation factors (Section "Per-channel Normalization of
 * K"): norm_c = sqrt(max |K[.,.,.,c]|), computed once at the end of prefill.
 *   k_fp16        device, fp16 [B][Hk][n_tokens][d], contiguous, read only
 *   per_head      0: the maximum runs over batch, heads and tokens (the paper's
 *                 definition; every row of the outputs is the same vector);
 *                 1: over batch and tokens only, one vector per kv head
 *   norm_out      device, fp32 [Hk][d]: what the caller multiplies into W_Q
 *   inv_norm_out  device, fp32 [Hk][d]: 1/norm, what the caller multiplies into W_K
 * A channel that is identically zero gets norm = 1.  n_tokens >= 1. */
int innerq_calibrate_key_norm(const innerq_config_t *cfg, const void *k_fp16, int64_t n_tokens,
                              int per_head, float *norm_out, float *inv_norm_out, void *hip_stream);

/* Append t_new tokens to the cache (Eq. kv_cached; Section "High-precision
 * Window"): the new k, v join the fp16 windows (first the sink window until it
 * holds w_sink tokens, then the recent ring); recent tokens beyond the window
 * are quantised (Eq. asym_quant / symmetric / hybrid rule of Figure "hybrid"),
 * packed and moved to the quantised store -- one token per step for a
 * per-token tensor, G tokens every G steps for a per-channel tensor.  The
 * result does not depend on how the tokens were split over calls: appending
 * the whole prefill at once equals Eq. kv_cache_init_quantized_window.
 *   k_new, v_new  device, fp16 [B][Hk][t_new][d], contiguous, read only
 *   k_inv_norm    device, fp32 [Hk][d] or NULL.  When given, every new key is
 *                 replaced by fp16(float(k) * k_inv_norm[hk][c]) on its way in
 *                 (for keys produced before the factors were folded into W_K):
 *                 the fp32 product is rounded to fp32, then to fp16, as a plain
 *                 fp32 multiply followed by a conversion does.
 * Quantiser arithmetic is IEEE fp32 on the fp16 inputs, scale rounded to fp16
 * before the codes are formed, round-half-to-even.  On success
 * cache->n_tokens += t_new.  INNERQ_E_CAPACITY if the result would exceed
 * capacity_tokens. */
int innerq_quantize_append(const innerq_config_t *cfg, innerq_cache_t *cache, const void *k_new,
                           const void *v_new, int64_t t_new, const float *k_inv_norm,
                           void *hip_stream);

/* The end of prefill in one call: innerq_calibrate_key_norm over the keys of a prompt followed by
 * innerq_quantize_append of that prompt with the keys divided by the factors on their way in
 * (Section "Per-channel Normalization of K": the factors are computed once at the end of prefill;
 * Eq. kv_cache_init_quantized_window).  Same arguments as those two calls; the cache must be empty
 * (n_tokens == 0, else INNERQ_E_ARG); norm_out / inv_norm_out are written as by
 * innerq_calibrate_key_norm and the cache contents are bit-identical to the two separate calls.
 * What it saves: the maximum over the keys runs in the same launch as everything that does not
 * depend on it (quantising the values, filling the value windows), so the prompt's keys are read
 * twice and its values once in three launches instead of four, and the memory-bound maximum hides
 * behind the arithmetic-bound value quantisation. */
int innerq_prefill(const innerq_config_t *cfg, innerq_cache_t *cache, const void *k_fp16,
                   const void *v_fp16, int64_t n_tokens, int per_head, float *norm_out,
                   float *inv_norm_out, void *hip_stream);

/* One decode step of attention for one new query per sequence (Eq. att:1-3
 * with Eq. kv_cached_quantized): out = softmax(q K^T / sqrt(d)) V over all
 * cache->n_tokens cached tokens, where K and V are the fp16 windows and the
 * dequantised store (Eq. hybrid_dequant) -- dequantisation is fused into the
 * two vector-matrix products, the quantised and window parts are merged before
 * the softmax is normalised (Figure "quantization_overall").
 *   q_fp16     device, fp16 [B][Hq][d], read only
 *   q_scale    device, fp32 [Hk][d] or NULL.  When given, the query of head hq
 *              is first replaced by fp16(float(q) * q_scale[hq/(Hq/Hk)][c]), rounded
 *              in the same two steps as the keys,
 *              (for callers that have not folded the key norm into W_Q).
 *   out        device, [B][Hq][d], fp32 if out_is_fp32 else fp16
 *   workspace  device scratch of at least innerq_workspace_bytes(cfg) bytes;
 *              contents need not be initialised and are undefined afterwards
 * Accumulation is fp32.  n_tokens must be >= 1.
 * Input range: inputs are assumed finite (NaN / Inf behaviour is unspecified).  On the fused
 * kernels the query (after q_scale) enters the matrix cores as fp16 times a power of two.  The
 * inner-grouped kernel chooses that power per head from the head's largest |q|, so every finite
 * fp16 query is accepted and the accuracy does not depend on its magnitude.  The outer-grouped
 * comparison kernel folds the groups' scales into the query (keys) and into the softmax weights
 * (values) as fp16 tables; it normalises the query per head and the scales and zero-points per
 * 64-token tile by powers of two, so the magnitudes of query and cache do not matter either, as
 * long as the scales and zero-points of one tile lie within 2^14 of each other (smaller ones
 * lose precision against the tile's largest, not against themselves). */
int innerq_decode_attention(const innerq_config_t *cfg, const innerq_cache_t *cache,
                            const void *q_fp16, const float *q_scale, void *out, int out_is_fp32,
                            void *workspace, size_t workspace_bytes, void *hip_stream);

/* innerq_decode_attention for callers that cannot allocate device memory or pass a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, kernels, launch plan and results as innerq_decode_attention, except that the
 * split-K partials live in an array that is part of the library's code object
 * (INNERQ_STATIC_WORKSPACE_BYTES bytes of device memory per GPU, held from the first use of the
 * library on that GPU until the process ends).  The call allocates and frees nothing; on its
 * first use on a device it looks the array's device address up (a symbol query, no allocation:
 * make that first call outside a graph capture).
 *   - INNERQ_E_WORKSPACE if innerq_workspace_bytes(cfg) exceeds INNERQ_STATIC_WORKSPACE_BYTES
 *     (nothing is launched); INNERQ_E_HIP if the address lookup fails.
 *   - The partials need no clearing: every slot a call reads was written by that call.
 *   - All calls on one GPU share the one array: two calls that overlap in time on the same GPU
 *     (different streams or host threads) race on it and give undefined outputs.  Calls on one
 *     stream are ordered and safe. */
#define INNERQ_STATIC_WORKSPACE_BYTES (32u << 20)
int innerq_decode_attention_static(const innerq_config_t *cfg, const innerq_cache_t *cache,
                                   const void *q_fp16, const float *q_scale, void *out,
                                   int out_is_fp32, void *hip_stream);

/* Quantisation off the critical path of a decode step (the paper names this as future work at
 * the end of its Section "Latency": the quantisation of evicted tokens can be overlapped with
 * attention).  What leaves the recent windows at step t + 1 is already known at step t, and
 * the packed form of a token (or of a group of G tokens) depends on its own values only, so
 * it can be written to the store one step early, into rows that no attention call reads before
 * they become valid.  Three calls; the results (outputs and cache contents) are those of
 * innerq_quantize_append followed by innerq_decode_attention, bit for bit in the cache.
 *
 * innerq_quantize_ahead: writes to the store what a single-token append to the current
 *   cache would evict (one key token; one group of values if that append completes a group).
 *   n_tokens does not change.  Call once after the prompt has been appended, before the first
 *   innerq_decode_attention_next.  Idempotent.
 * innerq_decode_attention_next: attention for the query of the NEXT token over the
 *   n_tokens + 1 tokens formed by the cache and that token, whose key and value rows are read
 *   from k_new / v_new (device, fp16 [B][Hk][1][d], keys already normalised if a key norm is
 *   in use) instead of the ring.  Requires that the store already holds what the append of
 *   that token evicts (innerq_quantize_ahead, or the previous innerq_append_deferred).
 *   Does not modify the cache.  Other arguments as innerq_decode_attention.  INNERQ_E_ARG if
 *   cache->store_ahead_tokens != n_tokens + 1 (the store was not run ahead: the kernels would
 *   read rows that were never written).
 * innerq_append_deferred: copies the new token into its window, n_tokens += 1, and does
 *   the innerq_quantize_ahead work for the step after.  It reads the rings and writes one
 *   ring slot and store rows that innerq_decode_attention_next of the same step does not
 *   touch, so the two may run concurrently on different streams: with the attention call on
 *   the main stream and this call on a side stream, a step's critical path is the attention
 *   alone.  Ordering the caller must provide (events): this call after k_new / v_new are
 *   ready and after the previous innerq_append_deferred; the NEXT step's attention after this
 *   call.
 * (w_recent >= 1, which every configuration satisfies, is what makes this possible: the newest
 * token is never quantised in the step that appends it.)  innerq_decode_attention_next and
 * innerq_append_deferred return INNERQ_E_CAPACITY when the cache is full. */
int innerq_quantize_ahead(const innerq_config_t *cfg, innerq_cache_t *cache, void *hip_stream);
int innerq_decode_attention_next(const innerq_config_t *cfg, const innerq_cache_t *cache,
                                 const void *k_new, const void *v_new, const void *q_fp16,
                                 const float *q_scale, void *out, int out_is_fp32, void *workspace,
                                 size_t workspace_bytes, void *hip_stream);
int innerq_append_deferred(const innerq_config_t *cfg, innerq_cache_t *cache, const void *k_new,
                           const void *v_new, void *hip_stream);

/* One decode step in two launches instead of three: innerq_decode_attention_next followed by
 * innerq_append_deferred on the same stream, with the log-sum-exp merge of the attention call
 * and the append sharing one launch (they touch disjoint memory).  Same preconditions, results
 * and errors as those two calls (INNERQ_E_ARG unless store_ahead_tokens == n_tokens + 1); on
 * success n_tokens += 1 and the store already holds what the next step evicts.  Every argument is
 * checked before the first launch; only INNERQ_E_HIP of the second launch can follow an enqueued
 * first one. */
int innerq_decode_step(const innerq_config_t *cfg, innerq_cache_t *cache, const void *k_new,
                       const void *v_new, const void *q_fp16, const float *q_scale, void *out,
                       int out_is_fp32, void *workspace, size_t workspace_bytes, void *hip_stream);

/* innerq_decode_step for a batch whose sequences are not equally long, with the token counts in
 * DEVICE memory (the paper's Section "Latency" leaves sequences of different lengths and the
 * scheduling around them to future work; a step whose lengths never pass through the host can
 * also be recorded once in a HIP graph and replayed: the library records no memset and makes no
 * host-side decision that depends on a length).
 *   n_tokens_dev  device, int32 [B]: tokens cached per sequence before the step.  Read by the
 *                 kernels; the second launch adds one to every entry.  cache->n_tokens and
 *                 cache->store_ahead_tokens (host) are neither read nor written.
 *   max_tokens    host: a bound, n_tokens_dev[b] + 1 <= max_tokens <= capacity_tokens for every b.
 *                 It only sizes the launch (one wavefront per split of the longest sequence
 *                 allowed; a shorter sequence leaves some of its wavefronts without work), so a
 *                 loose bound costs idle wavefronts, never correctness.  A count outside the bound
 *                 is clamped on the device (that sequence's result is then unspecified; no buffer
 *                 is overrun).
 * Per sequence b the result equals innerq_decode_step on a cache of n_tokens_dev[b] tokens, bit for
 * bit in the cache; every sequence's store must have been run one step ahead (innerq_quantize_ahead
 * when it was filled, then this call keeps it so).  Inner-grouped caches on the fused kernel only
 * (INNERQ_E_UNSUPPORTED otherwise: outer-grouped and fp16 caches, more than 8 query heads per kv
 * head).  Other arguments and errors as innerq_decode_step. */
int innerq_decode_step_ragged(const innerq_config_t *cfg, const innerq_cache_t *cache,
                              int32_t *n_tokens_dev, int64_t max_tokens, const void *k_new,
                              const void *v_new, const void *q_fp16, const float *q_scale,
                              void *out, int out_is_fp32, void *workspace, size_t workspace_bytes,
                              void *hip_stream);

/* Measurement hook (no counterpart in the paper; its Section "Latency" times the fused
 * dequantise-and-multiply kernels on their own, and this lets a benchmark do the same).
 * The next attention call made by the calling host thread (innerq_decode_attention,
 * innerq_decode_attention_static, innerq_decode_attention_next or innerq_decode_step) attaches
 * ev_start and ev_stop to the dispatch of its dominant kernel (the fused dequantise +
 * score + value pass over the quantised range) on that call's stream: they take the
 * begin and end timestamps of that dispatch, so their difference is the kernel's own
 * duration as a profiler reports it.  Both are hipEvent_t created by the caller with
 * timing enabled; the request is consumed by that one call.  Passing NULL for either
 * cancels a pending request. */
int innerq_profile_next_attention(void *ev_start, void *ev_stop);

/* Measurement switch (no counterpart in the paper).  2-bit inner-grouped caches have a second
 * fused kernel that computes the same partial results: it forms the inner sums over the stored
 * fields with the block-scaled fp8 x fp4 matrix instruction (2-bit keys and values, at most 4
 * query heads per kv head) instead of 4x4x4 fp16 matrix instructions.  It is slower on the
 * measured configurations and off by default.  which = 0: every configuration on the 4x4x4 form
 * (default); which = 1: the fp8 x fp4 form where it applies, for side-by-side timing and parity
 * runs.  Process-wide, host-side only; returns INNERQ_E_ARG for any other value. */
int innerq_select_inner_kernel(int which);

/* Measurement yardstick (no counterpart in the paper): a plain read-only streaming kernel
 * over `bytes` bytes of device memory at `data` (16-byte aligned, bytes a multiple of 16),
 * launched on hip_stream.  It gives the rate a pure HBM read of that size reaches on this
 * device, launch and ramp included, to set beside the fused kernel's rate over the same
 * number of bytes.  `sink` is 4 bytes of writable device memory (written practically never;
 * it keeps the loads alive).  ev_start / ev_stop (hipEvent_t, may be NULL) take the begin and
 * end timestamps of the dispatch.  Returns INNERQ_E_NULL / _ALIGN / _ARG before any launch. */
int innerq_stream_read_probe(const void *data, size_t bytes, void *sink, void *hip_stream,
                             void *ev_start, void *ev_stop);

#ifdef __cplusplus
}
#endif
#endif /* INNERQ_H */
