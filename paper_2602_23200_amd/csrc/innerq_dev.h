// Internal declarations shared by the HIP translation units of libinnerq.
// Nothing here is part of the C ABI (see include/innerq.h for that).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include <atomic>

#include "../../include/innerq.h"

namespace innerq {

constexpr int kHeadDim = 128;          // the only head_dim built
constexpr int kWindowChunk = 64;       // most window tokens per wavefront / work-group chunk
constexpr int kWindowChunkMin = 16;    // fewest (short contexts, slots to spare)
constexpr int kHeadTile = 4;           // query heads served by one work-group pass
constexpr int kPageTokens = 64;        // tokens per page of a paged store (= one tile of the fused kernels)

// A paged store (no counterpart in the paper, which leaves memory management to future work): the six
// store buffers are pools of pages of 64 token rows, laid out like the contiguous store of a cache with
// batch = pool pages and capacity = 64, and table[b][r / 64] names the page that holds store row r of
// sequence b.  table == null: the contiguous store.
struct PageMap {
  const int* table;        // device, [B][tiles_per_seq]
  int tiles_per_seq;       // capacity_tokens / 64
  int pool_pages;          // page ids are clamped to [0, pool_pages): a bad entry cannot leave the buffers
};
// Linear row index, in the store buffers, of store row `row` of sequence-head bh (a row of the per-token
// form; row / G is the linear group index of the per-channel form when row is a multiple of G).
__device__ __forceinline__ long long store_row(const PageMap& pm, int n_kv_heads, long long capacity, long long bh,
                                               long long row) {
  if (!pm.table) return bh * capacity + row;
  const uint32_t b = (uint32_t)bh / (uint32_t)n_kv_heads, hk = (uint32_t)bh % (uint32_t)n_kv_heads;
  int page = pm.table[(long long)b * pm.tiles_per_seq + (row >> 6)];
  page = page < 0 ? 0 : (page >= pm.pool_pages ? pm.pool_pages - 1 : page);
  return ((long long)page * n_kv_heads + hk) * kPageTokens + (row & 63);
}


enum Form : int { kPerToken = 0, kPerChannel = 1, kFp16 = 2 };

inline __host__ __device__ int form_of(int kind, int which) {
  if (kind == INNERQ_KIND_FP16) return kFp16;
  const int inner = which == 0 ? kPerToken : kPerChannel;
  const int outer = which == 0 ? kPerChannel : kPerToken;
  return kind == INNERQ_KIND_INNER ? inner : outer;
}

// One tensor (K or V) of the cache as the kernels see it.
struct TensorView {
  const uint8_t* codes;
  const __half* scales;
  const __half* zeros;
  const __half* sink;
  const __half* ring;
  const __half* newest;   // [B][Hk][d] rows of token n_tokens - 1 when it is not in the ring yet, else null
  int form;            // Form
  int bits;            // code width of this tensor
  int slots;           // ring slots
  int n_sink;          // tokens currently in the sink window
  long long n_quant;   // tokens currently in the quantised store
};

// fp16_rn(fp32_rn(x * s)): a key (or query) times its normalisation factor, rounded the way a plain fp32
// multiply followed by a conversion rounds it.  Left alone, the compiler merges the two into one
// mixed-precision instruction that rounds the exact product once, and about one element in 2^13
// (an fp32 product that lands on an fp16 midpoint) then differs by one fp16 step.
__device__ inline __half scaled_half(float x, float s) {
  float p = x * s;
  asm("" : "+v"(p));
  return __float2half_rn(p);
}

struct Partition { long long n_sink, n_quant, n_recent; };

inline int bits_of(const innerq_config_t& c, int which) { return (which == 1 && c.v_bits) ? c.v_bits : c.bits; }

// Rows of a tensor's quantised store when n tokens are cached (the arithmetic of partition_of, for device code too).
__host__ __device__ inline long long quantised_rows(int w_sink, int w_recent, int group, int form, long long n) {
  long long mid = n - w_sink - w_recent;
  if (mid < 0) mid = 0;
  if (form == kPerChannel) mid -= mid % group;
  return mid;
}

inline Partition partition_of(const innerq_config_t& c, int which, long long n) {
  Partition p;
  p.n_sink = n < c.w_sink ? n : c.w_sink;
  long long mid = n - c.w_sink - c.w_recent;
  if (mid < 0) mid = 0;
  if (form_of(c.kind, which) == kPerChannel) mid -= mid % c.group;
  p.n_quant = mid;
  p.n_recent = n - p.n_sink - mid;
  return p;
}

inline int ring_slots(const innerq_config_t& c, int which) {
  // one spare slot (or G of them) beyond the window: the newest token never has to land in the
  // slot of a token that is evicted in the same step
  return c.w_recent + (form_of(c.kind, which) == kPerChannel ? c.group : 1);
}

// ---- launchers implemented in the kernel translation units --------------------------------

struct QuantTensorJob {
  // destination store
  uint8_t* codes; __half* scales; __half* zeros; __half* sink; __half* ring;
  const __half* x_new;       // [B][Hk][t_new][d]
  int form, mode, slots, bits;
  int lanes;                      // per-token form: lanes that share one group (8: short calls, 1: bulk)
  long long row_begin, row_end;   // store rows to quantise in this call (token = w_sink + row)
  long long ring_from;            // new tokens with index >= ring_from go to the ring
  int normalise;                  // apply k_inv_norm to tokens taken from x_new
  int is_keys;                    // tensor 0 of the cache
};

struct QuantArgs {
  QuantTensorJob job[2];          // K, V
  const float* inv_norm;          // [Hk][d] or null
  int batch, n_kv_heads, group, w_sink, sym_den_literal;
  long long capacity, n_old, t_new;
  // per-sequence token counts (device, [B], the count before the step), or null: a.n_old holds for all;
  // n_dev_out: the caller's counters, advanced by one per sequence by the append
  int w_recent;
  const int* n_dev;
  int* n_dev_out;
  PageMap pages;
};

struct AttnArgs;
// merge (may be null): the log-sum-exp merge of an attention call whose partials are complete on
// this stream rides in the same launch (or, for the rare two-launch appends, goes first).
hipError_t launch_quantize(const QuantArgs& a, hipStream_t stream, const AttnArgs* merge = nullptr);
// Calibration and bulk append of one prompt into an empty cache in three launches (zero, maxima + values, keys).
hipError_t launch_prefill(const QuantArgs& a, const __half* k, long long n_tokens, int per_head, float* norm_out,
                          float* inv_out, hipStream_t stream);
hipError_t launch_calibrate(const __half* k, int batch, int n_kv_heads, long long n_tokens, int per_head,
                            float* norm_out, float* inv_out, hipStream_t stream);

struct AttnArgs {
  TensorView k, v;
  const __half* q;          // [B][Hq][d]
  const float* q_scale;     // [Hk][d] or null
  void* out; int out_is_fp32;
  float* ws_ml;             // [B*Hq][n_partials][2]
  float* ws_o;              // [B*Hq][n_partials][d]
  int n_partials;           // partial slots per head in this launch
  int batch, n_q_heads, n_kv_heads, bits, v_bits, group, w_sink;   // bits: key codes, v_bits: value codes
  long long capacity, n_tokens;
  int sparse_zeros;         // value zero-points of the fused inner kernel: read only where a group is flagged asymmetric
  // per-sequence token counts (device, [B], the count before this step) or null; n_copy: where the fused
  // kernel leaves a copy of them for the append that follows in the same step (workspace, [B])
  const int* n_dev;
  int* n_copy;
  PageMap pages;
};

// Generic (any form, element-by-element) partial attention over the token set
// [a0,a1) U [b0,b1), cut into n_chunks equal chunks, written to partial slots
// first_slot .. first_slot+n_chunks.
hipError_t launch_attention_generic(const AttnArgs& a, long long a0, long long a1, long long b0, long long b1,
                                    int n_chunks, int first_slot, hipStream_t stream);
hipError_t launch_attention_merge(const AttnArgs& a, hipStream_t stream);

// Fused MFMA kernel for the inner-grouped layout: tokens [w_sink, w_sink + n_both) cut into
// n_splits contiguous ranges of 64-token tiles, one wavefront each, partial slots 0 .. n_splits.
// The window token set [0, na) U [b0, b0 + nb) is cut into win.n_chunks chunks (partial slots
// n_splits .. n_splits + n_chunks).  The inner kernel gives one chunk each to its first
// win.n_chunks wavefronts, which take fewer tiles in exchange (n_splits > win.n_chunks); the
// comparison kernels run the chunks as win.n_chunks extra wavefronts per (batch, kv-head).
struct WindowSet { long long na, b0, nb; int n_chunks; };
bool attention_inner_supported(const AttnArgs& a);
int attention_inner_waves_per_cu(const AttnArgs& a);   // resident wavefronts per compute unit
// ev_start / ev_stop (may be null) take the begin and end timestamps of the kernel dispatch itself.
struct Launch { hipStream_t stream; hipEvent_t ev_start, ev_stop; };
hipError_t launch_attention_inner(const AttnArgs& a, long long n_both, int n_splits, const WindowSet& win,
                                  hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop);

// The same kernels compiled for a paged store (a.pages.table set); launch_attention_inner and
// attention_inner_waves_per_cu route there.
int attention_inner_paged_waves_per_cu(const AttnArgs& a);
hipError_t launch_attention_inner_paged(const AttnArgs& a, long long n_both, int n_splits, const WindowSet& win,
                                        hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop);

// The same partial results for 2-bit codes from the block-scaled fp8 x fp4 matrix instruction
// (128-token tiles).  Parity-green but slower than the 4x4x4 form (see the file header), so it runs
// only on request: launch_attention_inner and attention_inner_waves_per_cu route to it when
// g_inner_variant == 1 and it applies.
bool attention_inner_f4_supported(const AttnArgs& a);
int attention_inner_f4_waves_per_cu(const AttnArgs& a);
hipError_t launch_attention_inner_f4(const AttnArgs& a, long long n_both, int n_splits, const WindowSet& win,
                                     hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop);
extern std::atomic<int> g_inner_variant;   // 0: 4x4x4 fp16 form everywhere (default); 1: fp8 x fp4 form where it applies

// A host-side answer that depends on the kernel instance only (an occupancy query, a device attribute),
// looked up once and kept: relaxed atomics, so that concurrent first callers race benignly (both store
// the same value).  0 = not asked yet.
struct CachedInt {
  std::atomic<int> v{0};
  template <typename F>
  int get(F ask) {
    int x = v.load(std::memory_order_relaxed);
    if (x == 0) { x = ask(); v.store(x, std::memory_order_relaxed); }
    return x;
  }
};

// Comparison kernel over an unquantised fp16 store, same launch shape.
bool attention_fp16_supported(const AttnArgs& a);
int attention_fp16_waves_per_cu(const AttnArgs& a);
hipError_t launch_attention_fp16(const AttnArgs& a, long long n_rows, int n_splits, const WindowSet& win,
                                 hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop);

// Comparison kernel over an outer-grouped cache, same launch shape.
bool attention_outer_supported(const AttnArgs& a);
int attention_outer_waves_per_cu(const AttnArgs& a);
hipError_t launch_attention_outer(const AttnArgs& a, long long n_both, int n_splits, const WindowSet& win,
                                  hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop);

// Plain streaming read of `bytes` bytes (a multiple of 16) by n_blocks work-groups of 256 lanes;
// `sink` is 4 writable bytes.
hipError_t launch_stream_read(const void* data, size_t bytes, uint32_t* sink, int n_blocks, hipStream_t stream,
                              hipEvent_t ev_start, hipEvent_t ev_stop);

}  // namespace innerq
