// Quantise / pack kernels, window copies and key-norm calibration.
//
// This translation unit is compiled with -ffp-contract=off: the integer codes
// and the symmetric/asymmetric flag depend on every fp32 rounding, so each
// multiply, add, subtract and divide below is a separate IEEE operation
// (Section "Quantization Scheme", Eq. asym_quant; Figure "hybrid").
#include "innerq_dev.h"
#include "merge.h"

namespace innerq {
namespace {

__device__ inline float h2f(__half h) { return __half2float(h); }

// One quantisation group of G values.
//   asymmetric (Eq. asym_quant):  Z = min, S = (max - Z) / (2^b - 1), code = clip(rint((x - Z) / S), 0, 2^b-1)
//   symmetric:                    S = max|x| / den, code = clip(rint(x / S), -2^(b-1), 2^(b-1)-1)
//   hybrid (Figure "hybrid"):     both; L1 reconstruction errors summed in index order; asymmetric
//                                 only if its error is strictly smaller
// The scale is rounded to fp16 (its stored precision) before the codes are formed.
// Stored field: code (asymmetric) or code + 2^(b-1) (symmetric); scale sign bit = asymmetric.
// The correctly rounded fp32 quotient num / S, given r = fl(1 / S) correctly rounded (one IEEE
// division per group instead of one per element): q0 = fl(num * r) is within one ulp, the
// remainder num - S * q0 is exact in the fused multiply-add, and q0 + rem * r then rounds to
// the nearest fp32 to num / S (Markstein's division step; no underflow at these magnitudes:
// num is a multiple of 2^-24 below 2^17, S an fp16 value).  Callers pass r = 0 for S == 0.
__device__ inline float code_quotient(float num, float S, float r) {
  const float q0 = num * r;
  const float rem = __builtin_fmaf(-S, q0, num);
  return __builtin_fmaf(rem, r, q0);
}

// 1 / S for code_quotient, 0 for S == 0: every quotient of such a group is then exactly 0, which
// is the code the formula assigns when the scale is 0.
__device__ inline float group_reciprocal(float S) { return S == 0.f ? 0.f : 1.0f / S; }

// One pass over a group held in registers: packed fields and L1 error of the asymmetric and of
// the symmetric variant (each only if the mode can choose it).
template <int G, int BITS, typename X>
__device__ inline void group_codes(X x, int mode, float mn, float Saf, float Ssf,
                                   uint32_t (&wa)[G * BITS / 32], uint32_t (&ws)[G * BITS / 32], float& ea,
                                   float& es) {
  constexpr int W = G * BITS / 32;
  constexpr int QMAX = (1 << BITS) - 1;
  constexpr int HALF = 1 << (BITS - 1);
#pragma unroll
  for (int i = 0; i < W; ++i) { wa[i] = 0u; ws[i] = 0u; }
  ea = 0.f; es = 0.f;
  if (mode != INNERQ_SYM) {
    const float rS = group_reciprocal(Saf);
#pragma unroll
    for (int i = 0; i < G; ++i) {
      const float ca = __builtin_amdgcn_fmed3f(rintf(code_quotient(x(i) - mn, Saf, rS)), 0.f, (float)QMAX);
      const float ra = Saf * ca + mn;
      ea = ea + fabsf(x(i) - ra);
      const uint32_t ua = (uint32_t)(int)ca;
      if constexpr (BITS == 3) {
        // a plane of 2-bit low parts (G/16 words), then a plane of high bits
        wa[(i * 2) / 32] |= (ua & 3u) << ((i * 2) % 32);
        wa[G / 16 + i / 32] |= (ua >> 2) << (i % 32);
      } else {
        wa[(i * BITS) / 32] |= ua << ((i * BITS) % 32);
      }
    }
  }
  if (mode != INNERQ_ASYM) {
    const float rS = group_reciprocal(Ssf);
#pragma unroll
    for (int i = 0; i < G; ++i) {
      const float cs = __builtin_amdgcn_fmed3f(rintf(code_quotient(x(i), Ssf, rS)), (float)(-HALF), (float)(HALF - 1));
      const float rs = Ssf * cs;
      es = es + fabsf(x(i) - rs);
      const uint32_t us = (uint32_t)((int)cs + HALF);
      if constexpr (BITS == 3) {
        ws[(i * 2) / 32] |= (us & 3u) << ((i * 2) % 32);
        ws[G / 16 + i / 32] |= (us >> 2) << (i % 32);
      } else {
        ws[(i * BITS) / 32] |= us << ((i * BITS) % 32);
      }
    }
  }
}

// x(i), i = 0 .. G-1 with i a compile-time constant after unrolling, returns element i of the group
// (a register array of floats, or packed fp16 pairs for groups too large to hold as floats).
template <int G, int BITS, typename X>
__device__ inline void quantize_group(X x, int mode, int sym_den_literal,
                                      uint32_t (&words)[G * BITS / 32], __half& scale, __half& zero) {
  constexpr int W = G * BITS / 32;
  constexpr int QMAX = (1 << BITS) - 1;
  constexpr int HALF = 1 << (BITS - 1);
  float mn = x(0), mx = mn, am = fabsf(mn);
#pragma unroll
  for (int i = 1; i < G; ++i) {
    const float v = x(i);
    mn = fminf(mn, v);
    mx = fmaxf(mx, v);
    am = fmaxf(am, fabsf(v));
  }
  const float den = sym_den_literal ? (float)QMAX : (float)(HALF - 1);
  const __half Sa = __float2half_rn((mx - mn) / (float)QMAX);
  const __half Ss = __float2half_rn(am / den);
  const float Saf = h2f(Sa), Ssf = h2f(Ss);
  uint32_t wa[W], ws[W];
  float ea, es;
  group_codes<G, BITS>(x, mode, mn, Saf, Ssf, wa, ws, ea, es);
  const bool asym = (mode == INNERQ_ASYM) || (mode == INNERQ_HYBRID && ea < es);
#pragma unroll
  for (int i = 0; i < W; ++i) words[i] = asym ? wa[i] : ws[i];
  scale = asym ? __hneg(Sa) : Ss;
  zero = asym ? __float2half_rn(mn) : __float2half_rn(0.f);
}

// Element i of a group kept as packed fp16 pairs.
template <int N>
__device__ inline float packed_half(const uint32_t (&xp)[N], int i) {
  const uint32_t w = xp[i / 2];
  return h2f(__ushort_as_half((unsigned short)((i & 1) ? (w >> 16) : (w & 0xffffu))));
}

// The same group quantiser spread over 8 neighbouring lanes (lane `sub` of the group holds the
// G/8 consecutive values x): the per-element divisions run in parallel, minimum / maximum are
// exact in any order, and the two error sums are still taken one element after the other in
// index order (every lane adds the whole chain from shuffled copies), so codes and flag are
// bit-identical to quantize_group.  Returns this lane's share of the packed fields, shifted to
// its place inside its 32-bit word and OR-ed over the lanes that share that word.
template <int CTRL>
__device__ inline float lane_swap(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
template <int CTRL>
__device__ inline uint32_t lane_swap_u(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}
// (3-bit fields: the return value is the word of the plane of 2-bit low parts, word_hi that of
// the plane of high bits, OR-ed over the lanes that share it.)
template <int G, int BITS>
__device__ inline uint32_t quantize_group_lanes(const float (&x)[G / 8], int sub, int mode, int sym_den_literal,
                                                __half& scale, __half& zero, uint32_t& word_hi) {
  constexpr int E = G / 8;
  constexpr int QMAX = (1 << BITS) - 1;
  constexpr int HALF = 1 << (BITS - 1);
  float mn = x[0], mx = x[0], am = fabsf(x[0]);
#pragma unroll
  for (int i = 1; i < E; ++i) {
    mn = fminf(mn, x[i]);
    mx = fmaxf(mx, x[i]);
    am = fmaxf(am, fabsf(x[i]));
  }
  // butterflies over the 8 lanes of the group: pairs, quads, the two quads
  mn = fminf(mn, lane_swap<0xB1>(mn)); mx = fmaxf(mx, lane_swap<0xB1>(mx)); am = fmaxf(am, lane_swap<0xB1>(am));
  mn = fminf(mn, lane_swap<0x4E>(mn)); mx = fmaxf(mx, lane_swap<0x4E>(mx)); am = fmaxf(am, lane_swap<0x4E>(am));
  mn = fminf(mn, lane_swap<0x141>(mn)); mx = fmaxf(mx, lane_swap<0x141>(mx)); am = fmaxf(am, lane_swap<0x141>(am));
  const float den = sym_den_literal ? (float)QMAX : (float)(HALF - 1);
  const __half Sa = __float2half_rn((mx - mn) / (float)QMAX);
  const __half Ss = __float2half_rn(am / den);
  const float Saf = h2f(Sa), Ssf = h2f(Ss);
  const float rSa = group_reciprocal(Saf), rSs = group_reciprocal(Ssf);
  uint32_t fa = 0u, fs = 0u, ha = 0u, hs = 0u;
  float da[E], ds[E];
#pragma unroll
  for (int i = 0; i < E; ++i) {
    const float ca = __builtin_amdgcn_fmed3f(rintf(code_quotient(x[i] - mn, Saf, rSa)), 0.f, (float)QMAX);
    const float cs = __builtin_amdgcn_fmed3f(rintf(code_quotient(x[i], Ssf, rSs)), (float)(-HALF), (float)(HALF - 1));
    const float ra = Saf * ca + mn;
    const float rs = Ssf * cs;
    da[i] = fabsf(x[i] - ra);
    ds[i] = fabsf(x[i] - rs);
    const uint32_t ua = (uint32_t)(int)ca, us = (uint32_t)((int)cs + HALF);
    if constexpr (BITS == 3) {
      fa |= (ua & 3u) << (i * 2);
      fs |= (us & 3u) << (i * 2);
      ha |= (ua >> 2) << i;
      hs |= (us >> 2) << i;
    } else {
      fa |= ua << (i * BITS);
      fs |= us << (i * BITS);
    }
  }
  // The two error sums in index order, as a relay over the 8 lanes: at stage s lane s of the group
  // holds the sum of all elements before its own, adds its E elements one after the other and
  // hands the result to lane s + 1 (one DPP shift).  Every lane runs every stage; only the stage
  // that matches its position produces a value that is used.  Same additions in the same order as
  // one lane summing all G values, 8 (E + 1) dependent steps instead of G cross-lane reads.
  float ra_run = 0.f, rs_run = 0.f, ea = 0.f, es = 0.f;
#pragma unroll
  for (int st = 0; st < 8; ++st) {
    ea = ra_run;
    es = rs_run;
#pragma unroll
    for (int i = 0; i < E; ++i) {
      ea = ea + da[i];
      es = es + ds[i];
    }
    if (st < 7) {
      ra_run = lane_swap<0x111>(ea);                     // row_shr:1: lane j takes lane j - 1's value
      rs_run = lane_swap<0x111>(es);
    }
  }
  // lane 7 of the group now holds both totals: to all 8 lanes
  const int last = ((int)(threadIdx.x & 63u) & ~7) + 7;
  ea = __shfl(ea, last);
  es = __shfl(es, last);
  const bool asym = (mode == INNERQ_ASYM) || (mode == INNERQ_HYBRID && ea < es);
  scale = asym ? __hneg(Sa) : Ss;
  zero = asym ? __float2half_rn(mn) : __float2half_rn(0.f);
  constexpr int LB = BITS == 3 ? 2 : BITS;             // bits per field of the (low) plane
  constexpr int LPW = 32 / (E * LB);                   // lanes that share one 32-bit word of it
  uint32_t w = (asym ? fa : fs) << ((sub % LPW) * E * LB);
  if constexpr (LPW >= 2) w |= lane_swap_u<0xB1>(w);
  if constexpr (LPW >= 4) w |= lane_swap_u<0x4E>(w);
  word_hi = 0u;
  if constexpr (BITS == 3) {
    constexpr int LPH = 32 / E;                        // lanes per word of the high-bit plane: 8 or 4
    uint32_t h = (asym ? ha : hs) << ((sub % LPH) * E);
    h |= lane_swap_u<0xB1>(h);
    h |= lane_swap_u<0x4E>(h);
    if constexpr (LPH == 8) h |= lane_swap_u<0x141>(h);
    word_hi = h;
  }
  return w;
}

// Index arithmetic of one launch is 32-bit: the host refuses launches of 2^32 or more threads, token
// indices stay below 2^24 (capacity * head_dim <= 2^31), and a 64-bit division by a run-time value
// is an inlined routine of well over a hundred instructions where the 32-bit one takes about twenty.
__device__ __forceinline__ uint32_t div32(long long n, long long d) { return (uint32_t)n / (uint32_t)d; }
__device__ __forceinline__ uint32_t mod32(long long n, long long d) { return (uint32_t)n % (uint32_t)d; }

// Where the fp16 row of token t (absolute index) of sequence-head bh lives when the quantiser
// wants it: still in the recent ring if it was appended by an earlier call, else in x_new.
// (n_old: tokens cached before this call: a.n_old, or the sequence's own count.)
__device__ __forceinline__ const __half* token_row(const QuantTensorJob& j, const QuantArgs& a, long long n_old,
                                          long long bh, long long t, bool& from_new) {
  from_new = t >= n_old;
  if (from_new) return j.x_new + ((bh * a.t_new) + (t - n_old)) * kHeadDim;
  return j.ring + (bh * j.slots + mod32(t, j.slots)) * kHeadDim;
}

// Per-sequence token counts (a.n_dev: device memory, the count of every sequence before the step; Section
// "Latency", closing remark: sequences of a batch need not be equally long).  The launch is planned for
// the most any sequence can need (one key row, one value group, one window copy per sequence and head);
// each thread then takes its own sequence's state: the deferred single-token append of a cache of n0
// tokens copies token n0 into its window and quantises the rows between the states n0 + 1 and n0 + 2.
// Returns false when this sequence has nothing to quantise in this step (or is full).
__device__ __forceinline__ bool sequence_rows(const QuantArgs& a, const QuantTensorJob& j, long long bh,
                                              long long& n_old, long long& row_begin) {
  const long long n0 = a.n_dev[div32(bh, a.n_kv_heads)];
  if (n0 < 0 || n0 + 1 > a.capacity) return false;
  const long long to = n0 + 2 > a.capacity ? a.capacity : n0 + 2;
  const long long rb = quantised_rows(a.w_sink, a.w_recent, a.group, j.form, n0 + 1);
  const long long re = quantised_rows(a.w_sink, a.w_recent, a.group, j.form, to);
  n_old = n0;
  row_begin = rb;
  return re > rb;
}

// Which of the t_new new tokens (index i, absolute token n_old + i) go to a window: i < n_a to
// the sink, i >= i_b to the recent ring; the ones between were quantised by this same call.
struct CopySpan { long long n_a, i_b; };
__host__ __device__ inline CopySpan copy_span(const QuantArgs& a, long long n_old, long long ring_from) {
  long long n_a = a.w_sink - n_old;
  n_a = n_a < 0 ? 0 : (n_a > a.t_new ? a.t_new : n_a);
  long long i_b = ring_from - n_old;
  i_b = i_b < n_a ? n_a : (i_b > a.t_new ? a.t_new : i_b);
  return {n_a, i_b};
}
__host__ __device__ inline CopySpan copy_span(const QuantArgs& a, const QuantTensorJob& j) {
  return copy_span(a, a.n_old, j.ring_from);
}

// New tokens join the fp16 windows: the sink window while it has room, otherwise the recent
// ring -- unless this same call already moved them on to the quantised store.
__device__ __forceinline__ void window_copy(const QuantArgs& a, const QuantTensorJob& j, long long idx) {
  constexpr int CPR = kHeadDim / 8;
  const long long BH = (long long)a.batch * a.n_kv_heads;
  // only the new tokens that stay in a window are visited: the first n_a (sink) and those from i_b on (ring)
  CopySpan sp = copy_span(a, j);
  const long long n_cp = sp.n_a + (a.t_new - sp.i_b);
  if (idx >= BH * n_cp * CPR) return;
  const int ch = (int)(idx % CPR);
  const long long bh = div32(idx / CPR, n_cp);
  const long long k = idx / CPR - bh * n_cp;
  long long n_old = a.n_old;
  if (a.n_dev) {
    // per-sequence count: the one new token of this sequence (the plan has n_cp = 1 for every sequence)
    const uint32_t b = div32(bh, a.n_kv_heads);
    n_old = a.n_dev[b];
    if (n_old < 0 || n_old + 1 > a.capacity) return;
    sp = copy_span(a, n_old, a.w_sink + quantised_rows(a.w_sink, a.w_recent, a.group, j.form, n_old + 1));
    // the caller's counter of this sequence moves on: one thread per sequence (a.n_dev is a copy of it)
    if (a.n_dev_out && j.is_keys && ch == 0 && mod32(bh, a.n_kv_heads) == 0) a.n_dev_out[b] = (int)(n_old + 1);
  }
  const long long i = k < sp.n_a ? k : sp.i_b + (k - sp.n_a);
  const long long t = n_old + i;
  __half* dst;
  if (t < a.w_sink) dst = j.sink + (bh * a.w_sink + t) * kHeadDim;
  else dst = j.ring + (bh * j.slots + mod32(t, j.slots)) * kHeadDim;
  uint4 raw = *reinterpret_cast<const uint4*>(j.x_new + (bh * a.t_new + i) * kHeadDim + ch * 8);
  if (j.normalise) {
    __half* h = reinterpret_cast<__half*>(&raw);
    const float* inv = a.inv_norm + mod32(bh, a.n_kv_heads) * kHeadDim + ch * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) h[e] = scaled_half(h2f(h[e]), inv[e]);
  }
  *reinterpret_cast<uint4*>(dst + ch * 8) = raw;
}

// Job y (0: keys, 1: values) of a launch, field by field: indexing the by-value kernel argument
// with blockIdx.y makes the compiler copy the whole argument block to scratch first (so does any
// function that takes the block by reference and is not inlined: hence the forced inlining of
// quantize_rows, window_copy and token_row).
__device__ __forceinline__ QuantTensorJob pick_job(const QuantArgs& a, int y) {
  const QuantTensorJob& k = a.job[0];
  const QuantTensorJob& v = a.job[1];
  QuantTensorJob j;
  j.codes = y ? v.codes : k.codes;
  j.scales = y ? v.scales : k.scales;
  j.zeros = y ? v.zeros : k.zeros;
  j.sink = y ? v.sink : k.sink;
  j.ring = y ? v.ring : k.ring;
  j.x_new = y ? v.x_new : k.x_new;
  j.form = y ? v.form : k.form;
  j.mode = y ? v.mode : k.mode;
  j.slots = y ? v.slots : k.slots;
  j.bits = y ? v.bits : k.bits;
  j.lanes = y ? v.lanes : k.lanes;
  j.row_begin = y ? v.row_begin : k.row_begin;
  j.row_end = y ? v.row_end : k.row_end;
  j.ring_from = y ? v.ring_from : k.ring_from;
  j.normalise = y ? v.normalise : k.normalise;
  j.is_keys = y ? 0 : 1;
  return j;
}

__global__ void __launch_bounds__(256) window_copy_kernel(QuantArgs a) {
  const QuantTensorJob j = pick_job(a, (int)blockIdx.y);
  window_copy(a, j, (long long)blockIdx.x * blockDim.x + threadIdx.x);
}

// The quantise work of thread idx of tensor job j (keys and values may have different widths).
template <int G, int BITS>
__device__ __forceinline__ void quantize_rows(const QuantArgs& a, const QuantTensorJob& j, long long idx) {
  const long long n_rows = j.row_end - j.row_begin;
  if (n_rows <= 0) return;
  const long long BH = (long long)a.batch * a.n_kv_heads;
  constexpr int W = G * BITS / 32;

  if (j.form == kPerToken && j.lanes == 1) {
    // bulk calls: one lane per group (its G channels are 2 G contiguous bytes).  No cross-lane
    // traffic, and a wavefront has 64 groups' worth of loads in flight.
    constexpr int GPR = kHeadDim / G;                    // groups per row
    if (idx >= BH * n_rows * GPR) return;
    const int g = (int)(idx % GPR);
    const long long bh = div32(idx / GPR, n_rows);
    long long n_old = a.n_old, row_begin = j.row_begin;
    if (a.n_dev && !sequence_rows(a, j, bh, n_old, row_begin)) return;
    const long long row = row_begin + (idx / GPR - bh * n_rows);
    bool from_new;
    const __half* src = token_row(j, a, n_old, bh, a.w_sink + row, from_new) + g * G;
    const bool norm = from_new && j.normalise;
    const float* inv = a.inv_norm + mod32(bh, a.n_kv_heads) * kHeadDim + g * G;
    uint32_t words[W];
    __half s, z;
    if constexpr (G <= 32) {
      float x[G];
#pragma unroll
      for (int p = 0; p < G / 8; ++p) {
        const uint4 raw = reinterpret_cast<const uint4*>(src)[p];
        const __half* h = reinterpret_cast<const __half*>(&raw);
#pragma unroll
        for (int e = 0; e < 8; ++e) x[8 * p + e] = h2f(h[e]);
      }
      if (norm) {
#pragma unroll
        for (int i = 0; i < G; ++i) x[i] = h2f(scaled_half(x[i], inv[i]));
      }
      quantize_group<G, BITS>([&](int i) { return x[i]; }, j.mode, a.sym_den_literal, words, s, z);
    } else {
      // 64 floats do not fit the register file next to the rest: the group stays packed as fp16 pairs
      uint32_t xp[G / 2];
#pragma unroll
      for (int p = 0; p < G / 8; ++p) {
        const uint4 raw = reinterpret_cast<const uint4*>(src)[p];
        xp[4 * p] = raw.x; xp[4 * p + 1] = raw.y; xp[4 * p + 2] = raw.z; xp[4 * p + 3] = raw.w;
      }
      if (norm) {
#pragma unroll
        for (int p = 0; p < G / 2; ++p) {
          const uint32_t lo = __half_as_ushort(scaled_half(packed_half(xp, 2 * p), inv[2 * p]));
          const uint32_t hi = __half_as_ushort(scaled_half(packed_half(xp, 2 * p + 1), inv[2 * p + 1]));
          xp[p] = lo | (hi << 16);
        }
      }
      quantize_group<G, BITS>([&](int i) { return packed_half(xp, i); }, j.mode, a.sym_den_literal, words, s, z);
    }
    // a row is one plane of LB-bit fields over all channels (3-bit: followed by the plane of high bits)
    constexpr int LB = BITS == 3 ? 2 : BITS;
    constexpr int WL = G * LB / 32;                      // words of the (low) plane of one group
    const long long lin = store_row(a.pages, a.n_kv_heads, a.capacity, bh, row);
    uint32_t* rowp = reinterpret_cast<uint32_t*>(j.codes + (lin * kHeadDim * BITS) / 8);
#pragma unroll
    for (int i = 0; i < WL; ++i) rowp[g * WL + i] = words[i];
    if constexpr (BITS == 3) {
#pragma unroll
      for (int i = 0; i < G / 32; ++i) rowp[kHeadDim * 2 / 32 + g * (G / 32) + i] = words[WL + i];
    }
    const long long so = lin * GPR + g;
    j.scales[so] = s;
    if (j.zeros) j.zeros[so] = z;
  } else if (j.form == kPerToken) {
    // 8 lanes per group, G/8 consecutive channels each
    constexpr int GPR = kHeadDim / G;                    // groups per row
    constexpr int E = G / 8;
    constexpr int LB = BITS == 3 ? 2 : BITS;             // bits per field of the (low) plane
    constexpr int LPW = 32 / (E * LB);
    if (idx >= BH * n_rows * GPR * 8) return;
    const int sub = (int)(idx % 8);
    const long long gi = idx / 8;
    const int g = (int)(gi % GPR);
    const long long bh = div32(gi / GPR, n_rows);
    long long n_old = a.n_old, row_begin = j.row_begin;
    if (a.n_dev && !sequence_rows(a, j, bh, n_old, row_begin)) return;
    const long long row = row_begin + (gi / GPR - bh * n_rows);
    bool from_new;
    const __half* src = token_row(j, a, n_old, bh, a.w_sink + row, from_new) + g * G + sub * E;
    float x[E];
    if constexpr (E == 4) {
      const uint2 raw = *reinterpret_cast<const uint2*>(src);
      const __half* h = reinterpret_cast<const __half*>(&raw);
#pragma unroll
      for (int e = 0; e < 4; ++e) x[e] = h2f(h[e]);
    } else {
      const uint4 raw = *reinterpret_cast<const uint4*>(src);
      const __half* h = reinterpret_cast<const __half*>(&raw);
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = h2f(h[e]);
    }
    if (from_new && j.normalise) {
      const float* inv = a.inv_norm + mod32(bh, a.n_kv_heads) * kHeadDim + g * G + sub * E;
#pragma unroll
      for (int i = 0; i < E; ++i) x[i] = h2f(scaled_half(x[i], inv[i]));
    }
    __half s, z;
    uint32_t word_hi;
    const uint32_t word = quantize_group_lanes<G, BITS>(x, sub, j.mode, a.sym_den_literal, s, z, word_hi);
    // a row is one plane of LB-bit fields over all channels (3-bit: followed by the plane of high bits)
    const long long lin = store_row(a.pages, a.n_kv_heads, a.capacity, bh, row);
    uint32_t* rowp = reinterpret_cast<uint32_t*>(j.codes + (lin * kHeadDim * BITS) / 8);
    if (sub % LPW == 0) rowp[g * (G * LB / 32) + sub / LPW] = word;
    if constexpr (BITS == 3) {
      constexpr int LPH = 32 / E;
      if (sub % LPH == 0) rowp[kHeadDim * 2 / 32 + g * (G / 32) + sub / LPH] = word_hi;
    }
    if (sub == 0) {
      const long long so = lin * GPR + g;
      j.scales[so] = s;
      if (j.zeros) j.zeros[so] = z;
    }
  } else if (j.form == kPerChannel) {
    const long long n_groups = n_rows / G;
    if (idx >= BH * n_groups * kHeadDim) return;
    const int c = (int)(idx % kHeadDim);
    const long long bh = div32(idx / kHeadDim, n_groups);
    long long n_old = a.n_old, row_begin = j.row_begin;
    if (a.n_dev && !sequence_rows(a, j, bh, n_old, row_begin)) return;
    const long long tg = row_begin / G + (idx / kHeadDim - bh * n_groups);   // token-group index in the store
    const float inv = j.normalise ? a.inv_norm[mod32(bh, a.n_kv_heads) * kHeadDim + c] : 1.f;
    uint32_t words[W];
    __half s, z;
    auto run = [&](auto fetch) {
      if constexpr (G <= 32) {
        float x[G];
#pragma unroll
        for (int i = 0; i < G; ++i) x[i] = h2f(fetch(i));
        quantize_group<G, BITS>([&](int i) { return x[i]; }, j.mode, a.sym_den_literal, words, s, z);
      } else {
        // 64 floats do not fit the register file next to the rest: the group stays packed as fp16 pairs
        uint32_t xp[G / 2];
#pragma unroll
        for (int p = 0; p < G / 2; ++p) {
          const uint32_t lo = __half_as_ushort(fetch(2 * p)), hi = __half_as_ushort(fetch(2 * p + 1));
          xp[p] = lo | (hi << 16);
        }
        quantize_group<G, BITS>([&](int i) { return packed_half(xp, i); }, j.mode, a.sym_den_literal, words, s, z);
      }
    };
    const long long t0 = a.w_sink + tg * G;              // first token of the group
    if (t0 >= n_old) {
      // the whole group comes from x_new (bulk calls): one base address, a fixed stride
      const __half* src0 = j.x_new + ((bh * a.t_new) + (t0 - n_old)) * kHeadDim + c;
      run([&](int i) -> __half {
        __half v = src0[i * kHeadDim];
        if (j.normalise) v = scaled_half(h2f(v), inv);
        return v;
      });
    } else {
      run([&](int i) -> __half {
        bool from_new;
        const __half* src = token_row(j, a, n_old, bh, t0 + i, from_new);
        __half v = src[c];
        if (from_new && j.normalise) v = scaled_half(h2f(v), inv);
        return v;
      });
    }
    const long long go = (store_row(a.pages, a.n_kv_heads, a.capacity, bh, tg * G) / G) * kHeadDim + c;
    uint32_t* dst = reinterpret_cast<uint32_t*>(j.codes) + go * W;
#pragma unroll
    for (int i = 0; i < W; ++i) dst[i] = words[i];
    j.scales[go] = s;
    if (j.zeros) j.zeros[go] = z;
  } else {
    // fp16 "store": copy the rows, 8 halfs per thread
    constexpr int CPR = kHeadDim / 8;
    if (idx >= BH * n_rows * CPR) return;
    const int ch = (int)(idx % CPR);
    const long long bh = div32(idx / CPR, n_rows);
    long long n_old = a.n_old, row_begin = j.row_begin;
    if (a.n_dev && !sequence_rows(a, j, bh, n_old, row_begin)) return;
    const long long row = row_begin + (idx / CPR - bh * n_rows);
    bool from_new;
    const __half* src = token_row(j, a, n_old, bh, a.w_sink + row, from_new) + ch * 8;
    uint4 raw = *reinterpret_cast<const uint4*>(src);
    if (from_new && j.normalise) {
      __half* h = reinterpret_cast<__half*>(&raw);
      const float* inv = a.inv_norm + mod32(bh, a.n_kv_heads) * kHeadDim + ch * 8;
#pragma unroll
      for (int e = 0; e < 8; ++e) h[e] = scaled_half(h2f(h[e]), inv[e]);
    }
    __half* dst = reinterpret_cast<__half*>(j.codes) + store_row(a.pages, a.n_kv_heads, a.capacity, bh, row) * kHeadDim + ch * 8;
    *reinterpret_cast<uint4*>(dst) = raw;
  }
}

template <int G>
__global__ void __launch_bounds__(256) quantize_kernel(QuantArgs a, long long copy_from) {
  // Thread indices below copy_from quantise evicted tokens, those from copy_from on write the
  // new tokens into the windows (one launch; only used when no new token lands in a ring slot
  // that this call still has to read).  copy_from < 0: no copy work in this launch.
  const QuantTensorJob j = pick_job(a, (int)blockIdx.y);
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (copy_from >= 0 && idx >= copy_from) {
    window_copy(a, j, idx - copy_from);
    return;
  }
  if (j.bits == 2) quantize_rows<G, 2>(a, j, idx);
  else if (j.bits == 3) quantize_rows<G, 3>(a, j, idx);
  else quantize_rows<G, 4>(a, j, idx);
}

// The same launch with the log-sum-exp merge of an attention call riding along: the last
// merge_blocks work-groups (of job 0) merge four query heads each, the ones before them are
// quantize_kernel (the longer dependent chain, so it is dispatched first).  The two jobs touch
// disjoint memory (partials and output against store rows and window slots).
template <int G>
__global__ void __launch_bounds__(256) quantize_merge_kernel(QuantArgs a, long long copy_from, AttnArgs m,
                                                             int quant_blocks) {
  if ((int)blockIdx.x >= quant_blocks) {
    const long long bhq = (long long)(blockIdx.x - quant_blocks) * 4 + (threadIdx.x >> 6);
    if (blockIdx.y == 0 && bhq < (long long)m.batch * m.n_q_heads) merge_head(m, bhq, threadIdx.x & 63);
    return;
  }
  const QuantTensorJob j = pick_job(a, (int)blockIdx.y);
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (copy_from >= 0 && idx >= copy_from) {
    window_copy(a, j, idx - copy_from);
    return;
  }
  if (j.bits == 2) quantize_rows<G, 2>(a, j, idx);
  else if (j.bits == 3) quantize_rows<G, 3>(a, j, idx);
  else quantize_rows<G, 4>(a, j, idx);
}

// Threads the quantise work / the window copies of one tensor job need.
template <int G>
long long quantize_threads(const QuantArgs& a, const QuantTensorJob& j) {
  const long long BH = (long long)a.batch * a.n_kv_heads;
  const long long rows = j.row_end - j.row_begin;
  if (rows <= 0) return 0;
  if (j.form == kPerToken) return BH * rows * (kHeadDim / G) * j.lanes;
  if (j.form == kPerChannel) return BH * (rows / G) * kHeadDim;
  return BH * rows * (kHeadDim / 8);
}
inline long long copy_threads(const QuantArgs& a, const QuantTensorJob& j) {
  const CopySpan sp = copy_span(a, j);
  return (long long)a.batch * a.n_kv_heads * (sp.n_a + (a.t_new - sp.i_b)) * (kHeadDim / 8);
}

template <int G>
hipError_t launch_quantize_t(const QuantArgs& a, hipStream_t stream, const AttnArgs* merge) {
  long long threads = 0, cthreads = 0;
  for (int w = 0; w < 2; ++w) {
    const long long n = quantize_threads<G>(a, a.job[w]), c = copy_threads(a, a.job[w]);
    threads = n > threads ? n : threads;
    cthreads = c > cthreads ? c : cthreads;
  }
  if (threads >= (1LL << 32)) return hipErrorInvalidValue;   // (device index arithmetic is 32-bit)
  // A new token may overwrite a ring slot only after the old token in it has been read.  If
  // every token from the oldest one evicted in this call to the newest one appended fits the
  // ring at once, no slot is shared and one launch does both jobs.
  bool disjoint = true;
  for (int w = 0; w < 2; ++w) {
    const QuantTensorJob& j = a.job[w];
    if (j.row_end > j.row_begin && a.w_sink + j.row_begin < a.n_old &&
        a.n_old + a.t_new - (a.w_sink + j.row_begin) > j.slots)
      disjoint = false;
  }
  if (merge && disjoint) {
    // one launch: the quantise threads, the window-copy threads, then the merge blocks
    const long long qthreads = ((threads + 255) / 256) * 256;
    const int merge_blocks = (int)(((long long)merge->batch * merge->n_q_heads + 3) / 4);
    const int quant_blocks = (int)((qthreads + cthreads + 255) / 256);
    dim3 grid((unsigned)(quant_blocks + merge_blocks), 2);
    quantize_merge_kernel<G><<<grid, 256, 0, stream>>>(a, qthreads, *merge, quant_blocks);
    return hipGetLastError();
  }
  if (merge) {
    const hipError_t e = launch_attention_merge(*merge, stream);
    if (e != hipSuccess) return e;
  }
  if (threads > 0 && disjoint) {
    const long long qthreads = ((threads + 255) / 256) * 256;
    dim3 grid((unsigned)((qthreads + cthreads + 255) / 256), 2);
    quantize_kernel<G><<<grid, 256, 0, stream>>>(a, qthreads);
    return hipGetLastError();
  }
  if (threads > 0) {
    dim3 grid((unsigned)((threads + 255) / 256), 2);
    quantize_kernel<G><<<grid, 256, 0, stream>>>(a, -1);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (cthreads == 0) return hipSuccess;
  dim3 grid((unsigned)((cthreads + 255) / 256), 2);
  window_copy_kernel<<<grid, 256, 0, stream>>>(a);
  return hipGetLastError();
}

// ---- key-norm calibration (Section "Per-channel Normalization of K") ----------------------

__global__ void fill_u32_kernel(uint32_t* p, int n, uint32_t v) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// max |K| per (kv head, channel): each work-group scans a slice of tokens of one (b, hk) and
// folds its 128 channel maxima into the table with an unsigned atomic max on the float bits
// (monotone for non-negative floats).
constexpr int kCalibRows = 16;     // token rows read per pass by a 256-thread group
__global__ void __launch_bounds__(256) absmax_kernel(const __half* __restrict__ k, int n_kv_heads,
                                                     long long n_tokens, long long tokens_per_block,
                                                     uint32_t* table) {
  const long long bh = blockIdx.y;
  const int hk = (int)(bh % n_kv_heads);
  const int ch = threadIdx.x % 16, r = threadIdx.x / 16;
  const long long t0 = (long long)blockIdx.x * tokens_per_block;
  long long t1 = t0 + tokens_per_block;
  if (t1 > n_tokens) t1 = n_tokens;
  float m[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) m[e] = 0.f;
  for (long long t = t0 + r; t < t1; t += kCalibRows) {
    const uint4 raw = *reinterpret_cast<const uint4*>(k + (bh * n_tokens + t) * kHeadDim + ch * 8);
    const __half* h = reinterpret_cast<const __half*>(&raw);
#pragma unroll
    for (int e = 0; e < 8; ++e) m[e] = fmaxf(m[e], fabsf(__half2float(h[e])));
  }
  __shared__ float red[kCalibRows][kHeadDim];
#pragma unroll
  for (int e = 0; e < 8; ++e) red[r][ch * 8 + e] = m[e];
  __syncthreads();
  if (threadIdx.x < kHeadDim) {
    float v = 0.f;
    for (int i = 0; i < kCalibRows; ++i) v = fmaxf(v, red[i][threadIdx.x]);
    atomicMax(table + hk * kHeadDim + threadIdx.x, __float_as_uint(v));
  }
}

// One thread per channel: read every head's maximum first, then write norm and 1/norm
// (the maxima table aliases inv_out).
__global__ void norm_finalize_kernel(uint32_t* table, int n_kv_heads, int per_head, float* norm_out,
                                     float* inv_out) {
  const int c = threadIdx.x;
  float all = 0.f;
  for (int h = 0; h < n_kv_heads; ++h) all = fmaxf(all, __uint_as_float(table[h * kHeadDim + c]));
  for (int h = 0; h < n_kv_heads; ++h) {
    const float v = per_head ? __uint_as_float(table[h * kHeadDim + c]) : all;
    const float n = v == 0.f ? 1.f : sqrtf(v);
    norm_out[h * kHeadDim + c] = n;
    inv_out[h * kHeadDim + c] = 1.0f / n;
  }
}

// ---- prefill in one go (Section "Per-channel Normalization of K" with Eq. kv_cache_init_quantized_window):
// the key factors come from the prompt that is being appended, so the keys are read twice (maximum,
// then quantisation with the factors) and the values once.  First launch: the maximum over the keys
// next to everything that does not depend on the factors (value quantisation, value window copies);
// the work-group that finishes the maximum last turns the table into norm and 1 / norm.  Second
// launch: the keys.
struct AbsmaxPlan {
  const __half* k;
  long long n_tokens, tokens_per_block;
  int blocks_per_bh, n_blocks;        // n_blocks = blocks_per_bh * batch * n_kv_heads
  int every;                          // work-group x of the launch takes maxima if x % every == 0 and x / every < n_blocks
  int n_kv_heads, per_head;
  uint32_t* table;                    // [Hk][d] maxima as float bits (aliases inv_out), zeroed beforehand
  uint32_t* done;                     // work-groups finished so far (aliases norm_out[0]), zeroed beforehand
  float* norm_out;
  float* inv_out;
};

__global__ void prefill_zero_kernel(uint32_t* table, int n, uint32_t* done) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) table[i] = 0u;
  if (i == 0) *done = 0u;
}

template <int G>
__global__ void __launch_bounds__(256) prefill_values_and_absmax_kernel(QuantArgs a, long long copy_from, AbsmaxPlan m) {
  // The two kinds of work-group are interleaved over the launch (one maxima group every m.every
  // groups), so that the memory-bound maxima run next to the arithmetic-bound quantisation on every
  // compute unit instead of in front of it.
  const int x = (int)blockIdx.x;
  const bool takes_maxima = x % m.every == 0 && x / m.every < m.n_blocks;
  if (takes_maxima) {
    // ---- maximum of |K| per (kv head, channel) over this work-group's slice of tokens
    const int ab = x / m.every;
    const long long bh = ab / m.blocks_per_bh;
    const int hk = (int)(bh % m.n_kv_heads);
    const int ch = threadIdx.x % 16, r = threadIdx.x / 16;
    const long long t0 = (long long)(ab % m.blocks_per_bh) * m.tokens_per_block;
    long long t1 = t0 + m.tokens_per_block;
    if (t1 > m.n_tokens) t1 = m.n_tokens;
    float mx[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) mx[e] = 0.f;
    for (long long t = t0 + r; t < t1; t += kCalibRows) {
      const uint4 raw = *reinterpret_cast<const uint4*>(m.k + (bh * m.n_tokens + t) * kHeadDim + ch * 8);
      const __half* h = reinterpret_cast<const __half*>(&raw);
#pragma unroll
      for (int e = 0; e < 8; ++e) mx[e] = fmaxf(mx[e], fabsf(__half2float(h[e])));
    }
    __shared__ float red[kCalibRows][kHeadDim];
    __shared__ uint32_t ticket;
#pragma unroll
    for (int e = 0; e < 8; ++e) red[r][ch * 8 + e] = mx[e];
    __syncthreads();
    // The table is only ever touched by device-scope atomics (performed at the memory side, past the
    // caches), so no cache has to be written back or invalidated: a work-group counts itself done once
    // its own atomic maxima have RETURNED (their old values are consumed before the barrier), and the
    // group that counts last reads the table with the same atomic.  (A device-scope fence here would
    // write back and invalidate the whole L2 of the XCD 2 x n_blocks times, under the feet of the
    // value quantisation that shares the launch: measured 0.66 ms against 0.2 ms.)
    uint32_t seen = 0u;
    if (threadIdx.x < kHeadDim) {
      float v = 0.f;
      for (int i = 0; i < kCalibRows; ++i) v = fmaxf(v, red[i][threadIdx.x]);
      seen = atomicMax(m.table + hk * kHeadDim + threadIdx.x, __float_as_uint(v));
    }
    if (__syncthreads_or(seen == 0xffffffffu)) return;   // (never true: a maximum of |fp16| is finite)
    if (threadIdx.x == 0) ticket = atomicAdd(m.done, 1u);
    __syncthreads();
    if (ticket != (uint32_t)(m.n_blocks - 1)) return;
    if (threadIdx.x < kHeadDim) {
      // one thread per channel: it alone reads and then overwrites the table entries of its channel
      // (the table aliases inv_out).  The maxima are read with the same atomic that wrote them.
      const int c = threadIdx.x;
      float all = 0.f;
      for (int h = 0; h < m.n_kv_heads; ++h) all = fmaxf(all, __uint_as_float(atomicMax(m.table + h * kHeadDim + c, 0u)));
      for (int h = 0; h < m.n_kv_heads; ++h) {
        const float x = m.per_head ? __uint_as_float(atomicMax(m.table + h * kHeadDim + c, 0u)) : all;
        const float n = x == 0.f ? 1.f : sqrtf(x);
        m.norm_out[h * kHeadDim + c] = n;
        m.inv_out[h * kHeadDim + c] = 1.0f / n;
      }
    }
    return;
  }
  // ---- the value tensor: quantise what leaves the windows, copy what stays
  const QuantTensorJob j = pick_job(a, 1);
  int before = (x - 1) / m.every + 1;                    // maxima groups in front of this one (x >= 1 here)
  before = before > m.n_blocks ? m.n_blocks : before;
  const long long idx = (long long)(x - before) * blockDim.x + threadIdx.x;
  if (copy_from >= 0 && idx >= copy_from) {
    window_copy(a, j, idx - copy_from);
    return;
  }
  if (j.bits == 2) quantize_rows<G, 2>(a, j, idx);
  else if (j.bits == 3) quantize_rows<G, 3>(a, j, idx);
  else quantize_rows<G, 4>(a, j, idx);
}

template <int G>
hipError_t launch_prefill_t(const QuantArgs& a, AbsmaxPlan m, hipStream_t stream) {
  // the table and the counter start at zero (a fill kernel: safe inside a captured graph)
  const int n = m.n_kv_heads * kHeadDim;
  prefill_zero_kernel<<<(n + 255) / 256, 256, 0, stream>>>(m.table, n, m.done);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  // first launch: maxima + values
  const long long vthreads = ((quantize_threads<G>(a, a.job[1]) + 255) / 256) * 256;
  const long long vcopy = copy_threads(a, a.job[1]);
  if (vthreads + vcopy >= (1LL << 32)) return hipErrorInvalidValue;
  const long long vblocks = (vthreads + vcopy + 255) / 256;
  const long long every = (m.n_blocks + vblocks) / m.n_blocks;      // >= 1; (n_blocks - 1) * every < total
  m.every = (int)(every > (1 << 20) ? (1 << 20) : every);
  prefill_values_and_absmax_kernel<G><<<(unsigned)(m.n_blocks + vblocks), 256, 0, stream>>>(a, vthreads, m);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  // second launch: the keys (quantisation and window copies of tensor 0 only: a grid one job high)
  const long long kthreads = ((quantize_threads<G>(a, a.job[0]) + 255) / 256) * 256;
  const long long kcopy = copy_threads(a, a.job[0]);
  if (kthreads + kcopy >= (1LL << 32)) return hipErrorInvalidValue;
  if (kthreads + kcopy == 0) return hipSuccess;
  dim3 grid((unsigned)((kthreads + kcopy + 255) / 256), 1);
  quantize_kernel<G><<<grid, 256, 0, stream>>>(a, kthreads);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_prefill(const QuantArgs& a, const __half* k, long long n_tokens, int per_head, float* norm_out,
                          float* inv_out, hipStream_t stream) {
  for (int w = 0; w < 2; ++w)
    if (a.job[w].form != kFp16 && (a.job[w].bits < 2 || a.job[w].bits > 4)) return hipErrorInvalidValue;
  AbsmaxPlan m;
  m.k = k; m.n_tokens = n_tokens; m.tokens_per_block = 1024;
  m.blocks_per_bh = (int)((n_tokens + m.tokens_per_block - 1) / m.tokens_per_block);
  m.n_blocks = m.blocks_per_bh * a.batch * a.n_kv_heads;
  m.n_kv_heads = a.n_kv_heads; m.per_head = per_head;
  m.table = reinterpret_cast<uint32_t*>(inv_out);
  m.done = reinterpret_cast<uint32_t*>(norm_out);
  m.norm_out = norm_out; m.inv_out = inv_out;
  if (a.group == 32) return launch_prefill_t<32>(a, m, stream);
  if (a.group == 64) return launch_prefill_t<64>(a, m, stream);
  return hipErrorInvalidValue;
}

hipError_t launch_quantize(const QuantArgs& a, hipStream_t stream, const AttnArgs* merge) {
  for (int w = 0; w < 2; ++w)
    if (a.job[w].form != kFp16 && (a.job[w].bits < 2 || a.job[w].bits > 4)) return hipErrorInvalidValue;
  if (a.group == 32) return launch_quantize_t<32>(a, stream, merge);
  if (a.group == 64) return launch_quantize_t<64>(a, stream, merge);
  return hipErrorInvalidValue;
}

hipError_t launch_calibrate(const __half* k, int batch, int n_kv_heads, long long n_tokens, int per_head,
                            float* norm_out, float* inv_out, hipStream_t stream) {
  uint32_t* table = reinterpret_cast<uint32_t*>(inv_out);
  const int n = n_kv_heads * kHeadDim;
  fill_u32_kernel<<<(n + 255) / 256, 256, 0, stream>>>(table, n, 0u);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const long long tokens_per_block = 1024;
  dim3 grid((unsigned)((n_tokens + tokens_per_block - 1) / tokens_per_block), (unsigned)(batch * n_kv_heads));
  absmax_kernel<<<grid, 256, 0, stream>>>(k, n_kv_heads, n_tokens, tokens_per_block, table);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  norm_finalize_kernel<<<1, kHeadDim, 0, stream>>>(table, n_kv_heads, per_head, norm_out, inv_out);
  return hipGetLastError();
}

}  // namespace innerq
