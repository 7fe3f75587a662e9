// C ABI of libinnerq (see include/innerq.h): argument checks, the window /
// eviction arithmetic on the host, and kernel dispatch.  No device memory is
// allocated here and nothing synchronises.
#include <mutex>

#include "innerq_dev.h"

using namespace innerq;

namespace {

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

inline long long ceil_div(long long a, long long b) { return (a + b - 1) / b; }

// Most window chunks a launch may use (chunks of kWindowChunkMin tokens); bounds the workspace.
inline int window_chunk_cap(const innerq_config_t& c) {
  return (int)ceil_div((long long)c.w_sink + c.w_recent + 2LL * c.group, kWindowChunkMin) + 1;
}
// Most token splits a launch may use for the quantised range; bounds the workspace.  Never below
// the window chunk count plus one: the fused inner kernel needs one wavefront beyond those that
// carry a window chunk.
inline int split_cap(const innerq_config_t& c) {
  long long s = ceil_div(4096, (long long)c.batch * c.n_kv_heads);
  if (s < 4) s = 4;
  if (s > 512) s = 512;
  if (s < window_chunk_cap(c) + 1) s = window_chunk_cap(c) + 1;
  return (int)s;
}

// Bytes at the start of the workspace for one int per sequence: the fused kernel of a ragged step leaves
// the sequences' token counts there for the append that follows it.
inline size_t seq_bytes(const innerq_config_t& c) { return (((size_t)c.batch * sizeof(int) + 255) / 256) * 256; }

int check_config(const innerq_config_t* c) {
  if (!c) return INNERQ_E_NULL;
  if (c->batch < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->head_dim < 1) return INNERQ_E_ARG;
  if (c->n_q_heads % c->n_kv_heads != 0) return INNERQ_E_ARG;
  if ((long long)c->batch * c->n_kv_heads > 65535) return INNERQ_E_ARG;
  if (c->kind < INNERQ_KIND_INNER || c->kind > INNERQ_KIND_FP16) return INNERQ_E_ARG;
  if (c->k_mode < INNERQ_SYM || c->k_mode > INNERQ_HYBRID) return INNERQ_E_ARG;
  if (c->v_mode < INNERQ_SYM || c->v_mode > INNERQ_HYBRID) return INNERQ_E_ARG;
  if (c->sym_denominator != 0 && c->sym_denominator != 1) return INNERQ_E_ARG;
  if (c->w_sink < 0 || c->w_recent < 1) return INNERQ_E_ARG;
  if (c->bits < 1 || c->bits > 8 || c->group < 1) return INNERQ_E_ARG;
  if (c->head_dim % c->group != 0) return INNERQ_E_ARG;          // groups must tile the head dimension
  if (c->capacity_tokens < 1 || c->capacity_tokens % c->group != 0) return INNERQ_E_ARG;
  if (c->head_dim != kHeadDim) return INNERQ_E_UNSUPPORTED;
  if (c->bits != 2 && c->bits != 3 && c->bits != 4) return INNERQ_E_UNSUPPORTED;
  if (c->v_bits < 0 || c->v_bits > 8) return INNERQ_E_ARG;
  if (c->v_bits != 0 && c->v_bits != 2 && c->v_bits != 3 && c->v_bits != 4) return INNERQ_E_UNSUPPORTED;
  if (c->group != 32 && c->group != 64) return INNERQ_E_UNSUPPORTED;
  if (c->sparse_zeros != 0 && c->sparse_zeros != 1) return INNERQ_E_ARG;
  if (c->page_pool_pages < 0 || c->page_pool_pages > 0x7fffffffLL) return INNERQ_E_ARG;
  if (c->page_pool_pages > 0 && c->capacity_tokens % kPageTokens != 0) return INNERQ_E_ARG;
  return INNERQ_OK;
}

bool uses_zeros(const innerq_config_t& c, int which) {
  if (c.kind == INNERQ_KIND_FP16) return false;
  return (which == 0 ? c.k_mode : c.v_mode) != INNERQ_SYM;
}

int check_cache(const innerq_config_t& c, const innerq_cache_t* k) {
  if (!k) return INNERQ_E_NULL;
  if (!k->k_codes || !k->v_codes || !k->k_recent || !k->v_recent) return INNERQ_E_NULL;
  if (c.w_sink > 0 && (!k->k_sink || !k->v_sink)) return INNERQ_E_NULL;
  if (c.kind != INNERQ_KIND_FP16) {
    if (!k->k_scales || !k->v_scales) return INNERQ_E_NULL;
    if (uses_zeros(c, 0) && !k->k_zeros) return INNERQ_E_NULL;
    if (uses_zeros(c, 1) && !k->v_zeros) return INNERQ_E_NULL;
  }
  const void* ptrs[] = {k->k_codes, k->k_scales, k->k_zeros, k->v_codes, k->v_scales,
                        k->v_zeros, k->k_sink,   k->v_sink,  k->k_recent, k->v_recent};
  for (const void* p : ptrs)
    if (p && misaligned(p)) return INNERQ_E_ALIGN;
  if (k->n_tokens < 0 || k->n_tokens > c.capacity_tokens) return INNERQ_E_ARG;
  if (c.page_pool_pages > 0) {
    if (!k->page_table) return INNERQ_E_NULL;
    if (reinterpret_cast<uintptr_t>(k->page_table) & 3u) return INNERQ_E_ALIGN;
  }
  return INNERQ_OK;
}

TensorView view_of(const innerq_config_t& c, const innerq_cache_t& k, int which, long long n) {
  const Partition p = partition_of(c, which, n);
  TensorView v;
  v.codes = static_cast<const uint8_t*>(which == 0 ? k.k_codes : k.v_codes);
  v.scales = static_cast<const __half*>(which == 0 ? k.k_scales : k.v_scales);
  v.zeros = uses_zeros(c, which) ? static_cast<const __half*>(which == 0 ? k.k_zeros : k.v_zeros) : nullptr;
  v.sink = static_cast<const __half*>(which == 0 ? k.k_sink : k.v_sink);
  v.ring = static_cast<const __half*>(which == 0 ? k.k_recent : k.v_recent);
  v.newest = nullptr;
  v.form = form_of(c.kind, which);
  v.slots = ring_slots(c, which);
  v.n_sink = (int)p.n_sink;
  v.bits = bits_of(c, which);
  v.n_quant = p.n_quant;
  return v;
}

PageMap pages_of(const innerq_config_t& c, const innerq_cache_t& k) {
  PageMap pm;
  pm.table = c.page_pool_pages > 0 ? static_cast<const int*>(k.page_table) : nullptr;
  pm.tiles_per_seq = (int)(c.capacity_tokens / kPageTokens);
  pm.pool_pages = (int)c.page_pool_pages;
  return pm;
}

// Compute units of the current device (queried once per device; a host-side attribute read).
int compute_units() {
  static CachedInt cached[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  return cached[dev].get([&] {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    return n;
  });
}

thread_local hipEvent_t g_prof_start = nullptr, g_prof_stop = nullptr;

}  // namespace

extern "C" {

int innerq_profile_next_attention(void* ev_start, void* ev_stop) {
  const bool on = ev_start && ev_stop;
  g_prof_start = on ? static_cast<hipEvent_t>(ev_start) : nullptr;
  g_prof_stop = on ? static_cast<hipEvent_t>(ev_stop) : nullptr;
  return INNERQ_OK;
}

int innerq_select_inner_kernel(int which) {
  if (which != 0 && which != 1) return INNERQ_E_ARG;
  g_inner_variant.store(which, std::memory_order_relaxed);
  return INNERQ_OK;
}

int innerq_validate_config(const innerq_config_t* cfg) { return check_config(cfg); }

const char* innerq_status_string(int status) {
  switch (status) {
    case INNERQ_OK: return "ok";
    case INNERQ_E_NULL: return "a required pointer is NULL";
    case INNERQ_E_ARG: return "inconsistent or out-of-range argument";
    case INNERQ_E_UNSUPPORTED: return "configuration not supported by this build";
    case INNERQ_E_CAPACITY: return "cache capacity exceeded";
    case INNERQ_E_ALIGN: return "device pointer not 16-byte aligned";
    case INNERQ_E_WORKSPACE: return "workspace too small";
    case INNERQ_E_HIP: return "HIP kernel launch failed";
    default: return "unknown status";
  }
}

size_t innerq_buffer_bytes(const innerq_config_t* cfg, int which) {
  if (check_config(cfg) != INNERQ_OK || which < 0 || which >= INNERQ_BUF_COUNT) return 0;
  const innerq_config_t& c = *cfg;
  const size_t BH = (size_t)c.batch * c.n_kv_heads, d = (size_t)c.head_dim;
  // rows of the quantised store, over all sequences and kv heads (paged: over all pages of the pool)
  const size_t rows = c.page_pool_pages > 0 ? (size_t)c.page_pool_pages * c.n_kv_heads * kPageTokens
                                            : BH * (size_t)c.capacity_tokens;
  const int t = (which == INNERQ_BUF_K_CODES || which == INNERQ_BUF_K_SCALES || which == INNERQ_BUF_K_ZEROS ||
                 which == INNERQ_BUF_K_SINK || which == INNERQ_BUF_K_RECENT) ? 0 : 1;
  const int form = form_of(c.kind, t);
  switch (which) {
    case INNERQ_BUF_K_CODES: case INNERQ_BUF_V_CODES:
      return form == kFp16 ? rows * d * 2 : rows * d * (size_t)bits_of(c, t) / 8;
    case INNERQ_BUF_K_SCALES: case INNERQ_BUF_V_SCALES:
      return form == kFp16 ? 0 : rows * d / (size_t)c.group * 2;
    case INNERQ_BUF_K_ZEROS: case INNERQ_BUF_V_ZEROS:
      return uses_zeros(c, t) ? rows * d / (size_t)c.group * 2 : 0;
    case INNERQ_BUF_K_SINK: case INNERQ_BUF_V_SINK:
      return BH * (size_t)c.w_sink * d * 2;
    default:
      return BH * (size_t)ring_slots(c, t) * d * 2;
  }
}

size_t innerq_workspace_bytes(const innerq_config_t* cfg) {
  if (check_config(cfg) != INNERQ_OK) return 0;
  const size_t heads = (size_t)cfg->batch * cfg->n_q_heads;
  const size_t partials = (size_t)split_cap(*cfg) + window_chunk_cap(*cfg);
  return seq_bytes(*cfg) + heads * partials * (kHeadDim + 2) * sizeof(float) + 64;
}

int innerq_partition(const innerq_config_t* cfg, int which, int64_t n_tokens, int64_t* n_sink,
                     int64_t* n_quantised, int64_t* n_recent) {
  const int st = check_config(cfg);
  if (st != INNERQ_OK) return st;
  if ((which != 0 && which != 1) || n_tokens < 0) return INNERQ_E_ARG;
  const Partition p = partition_of(*cfg, which, n_tokens);
  if (n_sink) *n_sink = p.n_sink;
  if (n_quantised) *n_quantised = p.n_quant;
  if (n_recent) *n_recent = p.n_recent;
  return INNERQ_OK;
}

int innerq_calibrate_key_norm(const innerq_config_t* cfg, const void* k_fp16, int64_t n_tokens, int per_head,
                              float* norm_out, float* inv_norm_out, void* hip_stream) {
  int st = check_config(cfg);
  if (st != INNERQ_OK) return st;
  if (!k_fp16 || !norm_out || !inv_norm_out) return INNERQ_E_NULL;
  if (n_tokens < 1 || (per_head != 0 && per_head != 1)) return INNERQ_E_ARG;
  if (misaligned(k_fp16) || misaligned(norm_out) || misaligned(inv_norm_out)) return INNERQ_E_ALIGN;
  const hipError_t e = launch_calibrate(static_cast<const __half*>(k_fp16), cfg->batch, cfg->n_kv_heads, n_tokens,
                                        per_head, norm_out, inv_norm_out, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? INNERQ_OK : INNERQ_E_HIP;
}

}  // extern "C"

// Appends t_new tokens (their window copies) and quantises the store rows between two states of the
// cache: from the rows state `from` needs to the rows state `to` needs (a state = a token count).
// The ordinary append has from = n_tokens, to = n_tokens + t_new; the deferred forms run one
// token ahead.

// Kernel arguments of an append of t_new tokens that quantises the store rows between the states
// `from` and `to` (token counts).
static QuantArgs quant_args(const innerq_config_t* cfg, const innerq_cache_t* cache, const void* k_new,
                            const void* v_new, int64_t t_new, const float* k_inv_norm, long long from, long long to) {
  const long long n0 = cache->n_tokens, n1 = n0 + t_new;
  QuantArgs a;
  a.inv_norm = k_inv_norm;
  a.batch = cfg->batch; a.n_kv_heads = cfg->n_kv_heads; a.group = cfg->group;
  a.w_sink = cfg->w_sink; a.sym_den_literal = cfg->sym_denominator;
  a.capacity = cfg->capacity_tokens; a.n_old = n0; a.t_new = t_new;
  a.w_recent = cfg->w_recent; a.n_dev = nullptr; a.n_dev_out = nullptr;
  a.pages = pages_of(*cfg, *cache);
  for (int w = 0; w < 2; ++w) {
    QuantTensorJob& j = a.job[w];
    j.is_keys = w == 0;
    j.codes = static_cast<uint8_t*>(w == 0 ? cache->k_codes : cache->v_codes);
    j.scales = static_cast<__half*>(w == 0 ? cache->k_scales : cache->v_scales);
    j.zeros = uses_zeros(*cfg, w) ? static_cast<__half*>(w == 0 ? cache->k_zeros : cache->v_zeros) : nullptr;
    j.sink = static_cast<__half*>(w == 0 ? cache->k_sink : cache->v_sink);
    j.ring = static_cast<__half*>(w == 0 ? cache->k_recent : cache->v_recent);
    j.x_new = static_cast<const __half*>(w == 0 ? k_new : v_new);
    j.form = form_of(cfg->kind, w);
    j.bits = bits_of(*cfg, w);
    j.mode = w == 0 ? cfg->k_mode : cfg->v_mode;
    j.slots = ring_slots(*cfg, w);
    // rows that leave the recent window during this call (oldest first)
    j.row_begin = partition_of(*cfg, w, from).n_quant;
    j.row_end = partition_of(*cfg, w, to).n_quant;
    // new tokens from this index on stay in the recent ring at the end of this call
    j.ring_from = cfg->w_sink + partition_of(*cfg, w, n1).n_quant;
    // per-token form: eight lanes share a group when the call is short (a decode step: the
    // dependent chain is what costs), one lane takes a whole group when there is bulk to fill the chip
    const long long groups = (long long)cfg->batch * cfg->n_kv_heads * (j.row_end - j.row_begin) * (kHeadDim / cfg->group);
    j.lanes = groups >= 4096 ? 1 : 8;
    j.normalise = (w == 0 && k_inv_norm) ? 1 : 0;
  }
  return a;
}

static int quantize_impl(const innerq_config_t* cfg, innerq_cache_t* cache, const void* k_new, const void* v_new,
                         int64_t t_new, const float* k_inv_norm, long long from, long long to, void* hip_stream,
                         const AttnArgs* merge = nullptr) {
  if (t_new > 0 && (!k_new || !v_new)) return INNERQ_E_NULL;
  if ((k_new && misaligned(k_new)) || (v_new && misaligned(v_new)) || (k_inv_norm && misaligned(k_inv_norm)))
    return INNERQ_E_ALIGN;
  const long long n1 = cache->n_tokens + t_new;
  if (n1 > cfg->capacity_tokens) return INNERQ_E_CAPACITY;
  if (to > cfg->capacity_tokens) to = cfg->capacity_tokens;
  if (from > to) from = to;
  const QuantArgs a = quant_args(cfg, cache, k_new, v_new, t_new, k_inv_norm, from, to);
  const hipError_t e = launch_quantize(a, static_cast<hipStream_t>(hip_stream), merge);
  if (e != hipSuccess) return INNERQ_E_HIP;
  cache->n_tokens = n1;
  cache->store_ahead_tokens = to;
  return INNERQ_OK;
}

extern "C" {

int innerq_quantize_append(const innerq_config_t* cfg, innerq_cache_t* cache, const void* k_new,
                           const void* v_new, int64_t t_new, const float* k_inv_norm, void* hip_stream) {
  int st = check_config(cfg);
  if (st != INNERQ_OK) return st;
  st = check_cache(*cfg, cache);
  if (st != INNERQ_OK) return st;
  if (t_new < 0) return INNERQ_E_ARG;
  if (t_new == 0) return INNERQ_OK;
  if (!k_new || !v_new) return INNERQ_E_NULL;
  return quantize_impl(cfg, cache, k_new, v_new, t_new, k_inv_norm, cache->n_tokens, cache->n_tokens + t_new,
                       hip_stream);
}

int innerq_prefill(const innerq_config_t* cfg, innerq_cache_t* cache, const void* k_fp16, const void* v_fp16,
                   int64_t n_tokens, int per_head, float* norm_out, float* inv_norm_out, void* hip_stream) {
  int st = check_config(cfg);
  if (st != INNERQ_OK) return st;
  st = check_cache(*cfg, cache);
  if (st != INNERQ_OK) return st;
  if (!k_fp16 || !v_fp16 || !norm_out || !inv_norm_out) return INNERQ_E_NULL;
  if (misaligned(k_fp16) || misaligned(v_fp16) || misaligned(norm_out) || misaligned(inv_norm_out)) return INNERQ_E_ALIGN;
  if (n_tokens < 1 || (per_head != 0 && per_head != 1) || cache->n_tokens != 0) return INNERQ_E_ARG;
  if (n_tokens > cfg->capacity_tokens) return INNERQ_E_CAPACITY;
  const QuantArgs a = quant_args(cfg, cache, k_fp16, v_fp16, n_tokens, inv_norm_out, 0, n_tokens);
  const hipError_t e = launch_prefill(a, static_cast<const __half*>(k_fp16), n_tokens, per_head, norm_out, inv_norm_out,
                                      static_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return INNERQ_E_HIP;
  cache->n_tokens = n_tokens;
  cache->store_ahead_tokens = n_tokens;
  return INNERQ_OK;
}

int innerq_quantize_ahead(const innerq_config_t* cfg, innerq_cache_t* cache, void* hip_stream) {
  int st = check_config(cfg);
  if (st != INNERQ_OK) return st;
  st = check_cache(*cfg, cache);
  if (st != INNERQ_OK) return st;
  return quantize_impl(cfg, cache, nullptr, nullptr, 0, nullptr, cache->n_tokens, cache->n_tokens + 1, hip_stream);
}

int innerq_append_deferred(const innerq_config_t* cfg, innerq_cache_t* cache, const void* k_new, const void* v_new,
                           void* hip_stream) {
  int st = check_config(cfg);
  if (st != INNERQ_OK) return st;
  st = check_cache(*cfg, cache);
  if (st != INNERQ_OK) return st;
  if (!k_new || !v_new) return INNERQ_E_NULL;
  return quantize_impl(cfg, cache, k_new, v_new, 1, nullptr, cache->n_tokens + 1, cache->n_tokens + 2, hip_stream);
}

}  // extern "C"

// Attention over the first N tokens of the cache.  k_newest / v_newest (both or neither): fp16 rows
// [B][Hk][d] of token N - 1 when that token has not been copied into its window yet.
// defer_merge (may be null): the final merge is not launched; its arguments are returned instead.
// n_dev (may be null): per-sequence token counts on the device (the count before this step); N is then
// only the bound the launch is planned for.
static int attention_impl(const innerq_config_t* cfg, const innerq_cache_t* cache, long long N,
                          const void* k_newest, const void* v_newest, const void* q_fp16, const float* q_scale,
                          void* out, int out_is_fp32, void* workspace, size_t workspace_bytes, void* hip_stream,
                          AttnArgs* defer_merge = nullptr, const int* n_dev = nullptr) {
  if (!q_fp16 || !out || !workspace) return INNERQ_E_NULL;
  if (misaligned(q_fp16) || misaligned(out) || misaligned(workspace) || (q_scale && misaligned(q_scale)))
    return INNERQ_E_ALIGN;
  if (N < 1) return INNERQ_E_ARG;
  if (workspace_bytes < innerq_workspace_bytes(cfg)) return INNERQ_E_WORKSPACE;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const innerq_config_t& c = *cfg;

  AttnArgs a;
  a.k = view_of(c, *cache, 0, N);
  a.v = view_of(c, *cache, 1, N);
  a.k.newest = static_cast<const __half*>(k_newest);
  a.v.newest = static_cast<const __half*>(v_newest);
  a.q = static_cast<const __half*>(q_fp16);
  a.q_scale = q_scale;
  a.out = out; a.out_is_fp32 = out_is_fp32;
  a.batch = c.batch; a.n_q_heads = c.n_q_heads; a.n_kv_heads = c.n_kv_heads;
  a.bits = bits_of(c, 0); a.v_bits = bits_of(c, 1); a.group = c.group; a.w_sink = c.w_sink;
  a.capacity = c.capacity_tokens; a.n_tokens = N;
  a.sparse_zeros = c.sparse_zeros;
  a.n_dev = n_dev;
  a.n_copy = n_dev ? static_cast<int*>(workspace) : nullptr;
  a.pages = pages_of(c, *cache);

  // Tokens [w_sink, w_sink + n_both) are in the quantised store for both K and V: the split-K
  // range.  Everything else (sink window, recent windows, and the < G tokens quantised in only
  // one of the two tensors) goes through the generic window pass.
  long long n_both = a.k.n_quant < a.v.n_quant ? a.k.n_quant : a.v.n_quant;
  const long long n_sink = a.k.n_sink;
  const long long win_b0 = c.w_sink + n_both, win_b1 = N > win_b0 ? N : win_b0;
  long long win_tokens = n_sink + (win_b1 - win_b0);
  if (n_dev) {
    // planned for any length up to N: at least one tile's worth of wavefronts, and window chunks for the
    // largest window set a sequence can have (sink + recent + a value group in waiting)
    if (!attention_inner_supported(a)) return INNERQ_E_UNSUPPORTED;
    if (n_both < 64) n_both = 64;
    const long long most = (long long)c.w_sink + c.w_recent + c.group;
    win_tokens = N < most ? N : most;
  }
  const int r = c.n_q_heads / c.n_kv_heads;
  int n_splits = 0, win_chunk_len = kWindowChunk;
  // which fused kernel serves this cache (0 = none: element-by-element fallback)
  const int fused_kind =
      attention_inner_supported(a) ? 1 : attention_fp16_supported(a) ? 2 : attention_outer_supported(a) ? 3 : 0;
  const bool fused = fused_kind != 0;
  if (n_both > 0 && fused) {
    // one wavefront per split; every wavefront of the launch resident at once, no tail round
    // (the window wavefronts of the same launch take their share of the slots)
    const long long slots = (long long)compute_units() *
                            (fused_kind == 1   ? attention_inner_waves_per_cu(a)
                             : fused_kind == 2 ? attention_fp16_waves_per_cu(a)
                                               : attention_outer_waves_per_cu(a));
    const long long n_tiles = ceil_div(n_both, 64);
    long long per_head = slots / ((long long)c.batch * c.n_kv_heads);
    // Short contexts: with fewer than about four tiles per wavefront, a launch of half as many
    // wavefronts (one per SIMD instead of two) is the faster one -- every wavefront pays its query
    // set-up once, and the launch itself costs time per wavefront (measured on the 32-head 4k-token
    // configuration: 17.8 -> 14.3 us per step; the two meet at four tiles per wavefront).
    if (fused_kind == 1 && n_tiles < 4 * per_head && per_head >= 8) per_head /= 2;
    // Window chunk length and the number of plain wavefronts.
    long long best_len = kWindowChunk, best_cost = -1, best_plain = 1;
    auto plain_for = [&](long long len) {
      const long long nw = ceil_div(win_tokens, len);
      long long plain = per_head - nw;
      if (plain > n_tiles) plain = n_tiles;
      // the workspace holds split_cap + window_chunk_cap partials; the inner kernel's wavefronts
      // that carry a window chunk count as splits too
      const long long most = fused_kind == 1 ? split_cap(c) - nw : split_cap(c);
      if (plain > most) plain = most;
      return plain < 1 ? 1 : plain;
    };
    if (fused_kind == 1) {
      // Inner kernel, as measured (a window chunk costs its wavefront about as much whatever its
      // length, so short chunks pay only where wavefront slots go begging): 16 tokens while the
      // whole launch fills at most a quarter of the SIMDs (4-head 512-token configuration: 10.4 us
      // per step against 10.8 at 64); 32 tokens for short contexts on a busy chip (8 x 8 heads at 2k
      // tokens: 12.5 us against 13.0 at 64 and 14.1 at 16); 64 tokens from about 3k tokens on
      // (32 heads at 4k tokens: 13.4 us against 14.1 at 32 and 15.0 at 16) and wherever the slots
      // are all needed for tiles.
      const long long simds = (long long)compute_units() * 4;
      const long long waves16 = (long long)c.batch * c.n_kv_heads * (plain_for(kWindowChunkMin) + ceil_div(win_tokens, kWindowChunkMin));
      best_len = waves16 * 4 <= simds ? kWindowChunkMin : (n_tiles < 48 ? 32 : kWindowChunk);
      best_plain = plain_for(best_len);
    } else {
      // Comparison kernels: 64 tokens when the wavefront slots are all needed for tiles (long
      // contexts: a chunk then hides behind the tile work), shorter when slots are to spare and the
      // window chunk would be the longest wavefront of the launch.  Costs in units of one tile of
      // one wavefront: a chunk of L tokens about 4 + 14 L / 64.
      for (long long len = kWindowChunk; len >= kWindowChunkMin; len /= 2) {
        const long long nw = ceil_div(win_tokens, len);
        const long long plain = plain_for(len);
        const long long tile_cost = ceil_div(n_tiles, plain) * 8, win_cost = nw ? 32 + 14 * len / 8 : 0;   // x 8
        const long long cost = tile_cost > win_cost ? tile_cost : win_cost;
        if (best_cost < 0 || cost < best_cost) { best_cost = cost; best_len = len; best_plain = plain; }
      }
    }
    win_chunk_len = (int)best_len;
    const long long n_win_chunks = ceil_div(win_tokens, best_len);
    // the inner kernel's first wavefronts each carry a window chunk besides their tiles; the
    // comparison kernels run the window chunks as extra wavefronts of the same launch
    n_splits = (int)(fused_kind == 1 ? best_plain + n_win_chunks : best_plain);
  } else if (n_both > 0) {
    const long long blocks_per_split = (long long)c.batch * c.n_kv_heads * ceil_div(r, kHeadTile);
    long long s = ceil_div(2048, blocks_per_split);
    const long long by_len = ceil_div(n_both, 128);
    if (s > by_len) s = by_len;
    if (s > split_cap(c)) s = split_cap(c);
    if (s < 1) s = 1;
    n_splits = (int)s;
  }
  const int n_win = (int)ceil_div(win_tokens, win_chunk_len);
  if (n_win > window_chunk_cap(c)) return INNERQ_E_ARG;
  a.n_partials = n_splits + n_win;
  const size_t heads = (size_t)c.batch * c.n_q_heads;
  if (seq_bytes(c) + heads * (size_t)a.n_partials * (kHeadDim + 2) * sizeof(float) + 64 > workspace_bytes)
    return INNERQ_E_WORKSPACE;
  a.ws_ml = reinterpret_cast<float*>(static_cast<char*>(workspace) + seq_bytes(c));
  a.ws_o = a.ws_ml + ((heads * a.n_partials * 2 + 3) / 4) * 4;

  hipError_t e = hipSuccess;
  hipEvent_t prof_start = g_prof_start, prof_stop = g_prof_stop;
  g_prof_start = g_prof_stop = nullptr;
  if (n_splits > 0) {
    if (fused) {
      // the events take the timestamps of the dispatch itself
      const WindowSet win = {n_sink, win_b0, win_b1 - win_b0, n_win};
      e = fused_kind == 1   ? launch_attention_inner(a, n_both, n_splits, win, stream, prof_start, prof_stop)
          : fused_kind == 2 ? launch_attention_fp16(a, n_both, n_splits, win, stream, prof_start, prof_stop)
                            : launch_attention_outer(a, n_both, n_splits, win, stream, prof_start, prof_stop);
    } else {
      if (prof_start) (void)hipEventRecord(prof_start, stream);
      e = launch_attention_generic(a, c.w_sink, c.w_sink + n_both, 0, 0, n_splits, 0, stream);
      if (prof_stop) (void)hipEventRecord(prof_stop, stream);
    }
    if (e != hipSuccess) return INNERQ_E_HIP;
  }
  if (n_win > 0 && !(fused && n_splits > 0)) {
    e = launch_attention_generic(a, 0, n_sink, win_b0, win_b1, n_win, n_splits, stream);
    if (e != hipSuccess) return INNERQ_E_HIP;
  }
  if (defer_merge) {
    *defer_merge = a;
    return INNERQ_OK;
  }
  e = launch_attention_merge(a, stream);
  return e == hipSuccess ? INNERQ_OK : INNERQ_E_HIP;
}

extern "C" {

int innerq_decode_attention(const innerq_config_t* cfg, const innerq_cache_t* cache, const void* q_fp16,
                            const float* q_scale, void* out, int out_is_fp32, void* workspace,
                            size_t workspace_bytes, void* hip_stream) {
  int st = check_config(cfg);
  if (st != INNERQ_OK) return st;
  st = check_cache(*cfg, cache);
  if (st != INNERQ_OK) return st;
  return attention_impl(cfg, cache, cache->n_tokens, nullptr, nullptr, q_fp16, q_scale, out, out_is_fp32, workspace,
                        workspace_bytes, hip_stream);
}

}  // extern "C"

// Split-K partials for innerq_decode_attention_static: one array per GPU, part of the loaded code
// object, so no allocation call is ever made for it.  Host code never uses the array's name as an
// address; it asks the runtime for the device address once per device and passes that.
static __device__ __align__(256) unsigned char scratch[INNERQ_STATIC_WORKSPACE_BYTES];

namespace {
std::mutex g_scratch_mutex;
void* g_scratch_ptr[64] = {nullptr};        // per device, filled on the first call with that device current

// Device address of `scratch` on the current device (null on failure).
void* static_workspace() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}
}  // namespace

extern "C" {

int innerq_decode_attention_static(const innerq_config_t* cfg, const innerq_cache_t* cache, const void* q_fp16,
                                   const float* q_scale, void* out, int out_is_fp32, void* hip_stream) {
  int st = check_config(cfg);
  if (st != INNERQ_OK) return st;
  st = check_cache(*cfg, cache);
  if (st != INNERQ_OK) return st;
  if (innerq_workspace_bytes(cfg) > (size_t)INNERQ_STATIC_WORKSPACE_BYTES) return INNERQ_E_WORKSPACE;
  void* ws = static_workspace();
  if (!ws) return INNERQ_E_HIP;
  return attention_impl(cfg, cache, cache->n_tokens, nullptr, nullptr, q_fp16, q_scale, out, out_is_fp32, ws,
                        (size_t)INNERQ_STATIC_WORKSPACE_BYTES, hip_stream);
}

int innerq_decode_attention_next(const innerq_config_t* cfg, const innerq_cache_t* cache, const void* k_new,
                                 const void* v_new, const void* q_fp16, const float* q_scale, void* out,
                                 int out_is_fp32, void* workspace, size_t workspace_bytes, void* hip_stream) {
  int st = check_config(cfg);
  if (st != INNERQ_OK) return st;
  st = check_cache(*cfg, cache);
  if (st != INNERQ_OK) return st;
  if (!k_new || !v_new) return INNERQ_E_NULL;
  if (misaligned(k_new) || misaligned(v_new)) return INNERQ_E_ALIGN;
  if (cache->n_tokens + 1 > cfg->capacity_tokens) return INNERQ_E_CAPACITY;
  if (cache->store_ahead_tokens != cache->n_tokens + 1) return INNERQ_E_ARG;   // the store was not run one step ahead
  return attention_impl(cfg, cache, cache->n_tokens + 1, k_new, v_new, q_fp16, q_scale, out, out_is_fp32, workspace,
                        workspace_bytes, hip_stream);
}

int innerq_decode_step_ragged(const innerq_config_t* cfg, const innerq_cache_t* cache, int32_t* n_tokens_dev,
                              int64_t max_tokens, const void* k_new, const void* v_new, const void* q_fp16,
                              const float* q_scale, void* out, int out_is_fp32, void* workspace,
                              size_t workspace_bytes, void* hip_stream) {
  int st = check_config(cfg);
  if (st != INNERQ_OK) return st;
  innerq_cache_t view = cache ? *cache : innerq_cache_t{};
  view.n_tokens = 0;                                    // (the host counter is not used on this path)
  st = check_cache(*cfg, cache ? &view : nullptr);
  if (st != INNERQ_OK) return st;
  if (!k_new || !v_new || !n_tokens_dev) return INNERQ_E_NULL;
  if (misaligned(k_new) || misaligned(v_new) || (reinterpret_cast<uintptr_t>(n_tokens_dev) & 3u)) return INNERQ_E_ALIGN;
  if (cfg->kind != INNERQ_KIND_INNER) return INNERQ_E_UNSUPPORTED;
  if (max_tokens < 1) return INNERQ_E_ARG;
  if (max_tokens > cfg->capacity_tokens) return INNERQ_E_CAPACITY;
  AttnArgs merge;
  st = attention_impl(cfg, &view, max_tokens, k_new, v_new, q_fp16, q_scale, out, out_is_fp32, workspace,
                      workspace_bytes, hip_stream, &merge, n_tokens_dev);
  if (st != INNERQ_OK) return st;
  // second launch: merge + the deferred single-token append of every sequence, each from its own count
  // (read from the copy the fused kernel left in the workspace; the caller's counters are advanced here).
  // The plan is the most any sequence needs: one key row, one value group, one window copy.
  QuantArgs a = quant_args(cfg, &view, k_new, v_new, 1, nullptr, 0, 0);
  a.n_old = 0;
  a.n_dev = merge.n_copy;
  a.n_dev_out = n_tokens_dev;
  for (int w = 0; w < 2; ++w) {
    QuantTensorJob& j = a.job[w];
    j.row_begin = 0;
    j.row_end = j.form == kPerChannel ? cfg->group : 1;
    j.ring_from = 0;
    j.lanes = 8;
  }
  return launch_quantize(a, static_cast<hipStream_t>(hip_stream), &merge) == hipSuccess ? INNERQ_OK : INNERQ_E_HIP;
}

int innerq_decode_step(const innerq_config_t* cfg, innerq_cache_t* cache, const void* k_new, const void* v_new,
                       const void* q_fp16, const float* q_scale, void* out, int out_is_fp32, void* workspace,
                       size_t workspace_bytes, void* hip_stream) {
  int st = check_config(cfg);
  if (st != INNERQ_OK) return st;
  st = check_cache(*cfg, cache);
  if (st != INNERQ_OK) return st;
  if (!k_new || !v_new) return INNERQ_E_NULL;
  if (misaligned(k_new) || misaligned(v_new)) return INNERQ_E_ALIGN;
  if (cache->n_tokens + 1 > cfg->capacity_tokens) return INNERQ_E_CAPACITY;
  if (cache->store_ahead_tokens != cache->n_tokens + 1) return INNERQ_E_ARG;   // the store was not run one step ahead
  AttnArgs merge;
  st = attention_impl(cfg, cache, cache->n_tokens + 1, k_new, v_new, q_fp16, q_scale, out, out_is_fp32, workspace,
                      workspace_bytes, hip_stream, &merge);
  if (st != INNERQ_OK) return st;
  // second launch: the merge of this step together with the append of its token and the
  // quantisation the next step needs
  return quantize_impl(cfg, cache, k_new, v_new, 1, nullptr, cache->n_tokens + 1, cache->n_tokens + 2, hip_stream,
                       &merge);
}

}  // extern "C"

extern "C" {

int innerq_stream_read_probe(const void* data, size_t bytes, void* sink, void* hip_stream, void* ev_start,
                             void* ev_stop) {
  if (!data || !sink) return INNERQ_E_NULL;
  if (misaligned(data) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return INNERQ_E_ALIGN;
  if (bytes == 0 || bytes % 16 != 0) return INNERQ_E_ARG;
  // as many resident work-groups as the device holds (8 of 256 lanes per compute unit), fewer for small sizes
  long long blocks = (long long)compute_units() * 8;
  const long long needed = (long long)((bytes / 16 + 1023) / 1024);
  if (blocks > needed) blocks = needed;
  const hipError_t e = launch_stream_read(data, bytes, static_cast<uint32_t*>(sink), (int)blocks,
                                          static_cast<hipStream_t>(hip_stream), static_cast<hipEvent_t>(ev_start),
                                          static_cast<hipEvent_t>(ev_stop));
  return e == hipSuccess ? INNERQ_OK : INNERQ_E_HIP;
}

}  // extern "C"
