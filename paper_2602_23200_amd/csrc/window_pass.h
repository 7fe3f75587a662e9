// Attention over the high-precision windows (Section "High-precision Window"):
// the sink tokens, the recent ring, and the few tokens that are quantised in
// only one of K / V.  One wavefront handles one chunk of window tokens of one
// (batch, kv-head) for up to 4*NH4 query heads and writes one split-K partial.
// Included by every fused kernel so that the window work rides in the same
// launch as the quantised range.
#pragma once

#include "innerq_dev.h"

namespace innerq {

typedef _Float16 w_half2_t __attribute__((ext_vector_type(2)));
typedef uint32_t w_u32x4 __attribute__((ext_vector_type(4)));
typedef float w_float4_t __attribute__((ext_vector_type(4)));
typedef _Float16 w_half4_t __attribute__((ext_vector_type(4)));
typedef uint32_t w_u32x2 __attribute__((ext_vector_type(2)));

// Element (token t, channel c) of one tensor of sequence-head bh, decoded per Eq. hybrid_dequant.
__device__ inline float fetch_element(const TensorView& tv, const AttnArgs& a, long long bh, long long t, int c) {
  constexpr int D = kHeadDim;
  if (tv.newest && t == a.n_tokens - 1) return __half2float(tv.newest[bh * D + c]);
  if (t < tv.n_sink) return __half2float(tv.sink[(bh * a.w_sink + t) * D + c]);
  const long long row = t - a.w_sink;
  if (row >= tv.n_quant) return __half2float(tv.ring[(bh * tv.slots + (t % tv.slots)) * D + c]);
  const long long lin = store_row(a.pages, a.n_kv_heads, a.capacity, bh, row);     // (contiguous: bh * capacity + row)
  if (tv.form == kFp16) return __half2float(reinterpret_cast<const __half*>(tv.codes)[lin * D + c]);
  const int bits = tv.bits, G = a.group;
  long long si;
  unsigned field;
  // field i of a packed run of n fields that starts at byte address p (3-bit: a plane of 2-bit
  // low parts, n/4 bytes, then a plane of high bits)
  auto field_of = [&](const uint8_t* p, int i, int n) -> unsigned {
    if (bits == 3) return ((p[i / 4] >> (2 * (i % 4))) & 3u) | (((p[n / 4 + i / 8] >> (i % 8)) & 1u) << 2);
    return (p[(i * bits) / 8] >> ((i * bits) % 8)) & ((1u << bits) - 1u);
  };
  if (tv.form == kPerToken) {
    field = field_of(tv.codes + (lin * D * bits) / 8, c, D);
    si = lin * (D / G) + c / G;
  } else {
    si = (store_row(a.pages, a.n_kv_heads, a.capacity, bh, row - row % G) / G) * D + c;
    field = field_of(tv.codes + si * ((G * bits) / 8), (int)(row % G), G);
  }
  const float s = __half2float(tv.scales[si]);
  const bool asym = __float_as_uint(s) >> 31;
  const float S = fabsf(s);
  return asym ? S * (float)field + __half2float(tv.zeros[si]) : S * (float)((int)field - (1 << (bits - 1)));
}

// fp16 row of token t if that tensor keeps it in fp16 (sink window, recent ring, fp16 store, or the
// not yet appended newest token), else null.  For the contiguous store only (the fused kernels whose store is
// fp16 do not take paged caches).  Written for a caller that asks for many rows per
// lane: everything that depends on bh alone is wave-uniform (scalar registers), the per-lane part
// is 32-bit (token indices stay below 2^24: capacity * head_dim <= 2^31), and the ring slot
// t mod slots comes from a float reciprocal with a one-step correction instead of an integer
// division (a 64-bit modulo per row used to cost more instructions than the row's arithmetic).
__device__ __forceinline__ const __half* fp16_row(const TensorView& tv, const AttnArgs& a, long long bh, long long t) {
  constexpr int D = kHeadDim;
  const uint32_t tt = (uint32_t)t, ws = (uint32_t)a.w_sink, slots = (uint32_t)tv.slots;
  const uint32_t row = tt - ws;                               // meaningful when tt >= n_sink
  // tt mod slots
  uint32_t q = (uint32_t)((float)tt * (1.0f / (float)slots));
  uint32_t slot = tt - q * slots;                             // off by at most one multiple of slots
  slot = (int32_t)slot < 0 ? slot + slots : slot;
  slot = slot >= slots ? slot - slots : slot;
  const bool is_new = tv.newest != nullptr && tt == (uint32_t)(a.n_tokens - 1);
  const bool is_sink = tt < (uint32_t)tv.n_sink;
  const bool is_ring = !is_sink && row >= (uint32_t)tv.n_quant;
  const bool is_store = tv.form == kFp16;
  const __half* base_new = tv.newest + bh * D;
  const __half* base_sink = tv.sink + bh * a.w_sink * D;
  const __half* base_ring = tv.ring + bh * tv.slots * D;
  const __half* base_store = reinterpret_cast<const __half*>(tv.codes) + bh * a.capacity * D;
  const __half* base = is_new ? base_new : is_sink ? base_sink : is_ring ? base_ring : base_store;
  const uint32_t off = is_new ? 0u : is_sink ? tt * D : is_ring ? slot * D : row * D;
  return (is_new || is_sink || is_ring || is_store) ? base + off : nullptr;
}

// Wave-wide reductions: butterflies inside a row of 16 lanes via DPP, then the four rows through
// scalar registers.
__device__ inline float window_wave_max(float x) {
  x = fmaxf(x, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true)));
  x = fmaxf(x, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, true)));
  x = fmaxf(x, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xF, 0xF, true)));
  x = fmaxf(x, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xF, 0xF, true)));
  const float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 0));
  const float b = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 16));
  const float c = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 32));
  const float d = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 48));
  return fmaxf(fmaxf(a, b), fmaxf(c, d));
}
__device__ inline float window_wave_sum(float x) {
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true));
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, true));
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xF, 0xF, true));
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xF, 0xF, true));
  const float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 0));
  const float b = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 16));
  const float c = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 32));
  const float d = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 48));
  return (a + b) + (c + d);
}

__device__ inline float window_half_lo(uint32_t w) { return __half2float(__ushort_as_half((unsigned short)(w & 0xffffu))); }
__device__ inline float window_half_hi(uint32_t w) { return __half2float(__ushort_as_half((unsigned short)(w >> 16))); }

// Window token set: virtual index v in [0, na + nb) -> token v (v < na) or b0 + v - na.
// Chunk `chunk` of `n_chunks` equal chunks of that set; partial written to `slot`.
//
// A window token is kept in fp16 by both tensors, except the fewer than G tokens that the
// per-token-grouped tensor has already quantised while the per-channel-grouped one still waits
// for a full group: KQ says the key may be such a packed row (inner grouping), VQ the value
// (outer grouping).  BITS and G describe those packed rows.
//
// Every global load of a 64-token step (the lane's key row, its pieces of the value rows) is issued
// before any of them is used, so a step pays one memory round trip; the query set-up runs under
// that round trip too.
//
// Keys: lane = token.  Values without packed rows (!VQ): lane = a pair of channels, every token's row
// read as one coalesced 256-byte load whose base address is wave-uniform -- each lane works out the
// row address of its own token once and the loads fetch it from that lane -- and the weighted sums
// come out of the matrix instructions already complete per lane (no reduction across lanes).  With
// packed value rows (VQ): 16 lanes share a row, four rows per load, summed across the lane groups at
// the end.
// PAGED: the packed rows are looked up through the page table (else the table is never consulted).
template <int NH4, int BITS, int G, bool KQ, bool VQ, bool PAGED = false>
__device__ __forceinline__ void window_pass(const AttnArgs& a, long long bh, long long na, long long b0,
                                            long long nb, int chunk, int n_chunks, int slot) {
  constexpr int D = kHeadDim;
  constexpr int NH = NH4 * 4;
  constexpr int NG = D / G;
  constexpr int FPW = 32 / BITS;             // fields per 32-bit word
  constexpr int KVEC = D * BITS / 128;       // 16-byte pieces of a packed row
  constexpr uint32_t FMASK = (1u << BITS) - 1u;
  constexpr float HALFCODE = (float)(1 << (BITS - 1));
  const int lane = threadIdx.x & 63;
  // (32-bit: bh is a grid index)
  const int b = (int)((uint32_t)bh / (uint32_t)a.n_kv_heads), hk = (int)((uint32_t)bh % (uint32_t)a.n_kv_heads);
  const int r = a.n_q_heads / a.n_kv_heads;
  const long long total = na + nb;
  const long long chunk_len = (long long)((uint32_t)(total + n_chunks - 1) / (uint32_t)n_chunks);
  const long long v0 = chunk * chunk_len;
  const long long v1 = v0 + chunk_len < total ? v0 + chunk_len : total;

  __shared__ __attribute__((aligned(16))) _Float16 wq[NH][D];       // query, fp16 (exact)
  __shared__ __attribute__((aligned(16))) float wqs[NG][NH];        // their sums over each key group
  __shared__ __attribute__((aligned(16))) float wp[VQ ? 64 : 1][NH];   // probabilities of the current 64 tokens
  // the same, rounded to fp16, as matrix operands: [head][token]
  __shared__ __attribute__((aligned(16))) _Float16 wp16[VQ ? 4 : NH * 64];

  const int cg = lane & 15, tg = lane >> 4;
  // (every index here is below 2^24: 32-bit arithmetic per lane)
  const uint32_t na32 = (uint32_t)na, b032 = (uint32_t)b0;
  auto token_of = [&](long long v) -> long long {
    const uint32_t vv = (uint32_t)v;
    return (long long)(vv < na32 ? vv : b032 + (vv - na32));
  };

  const float c_log2 = 0.08838834764831845f * 1.4426950408889634f;    // log2(e) / sqrt(d)
  // o[h][e]: head h, channel 8 cg + e, the tokens 4 k + tg of every step.  Without packed value
  // rows the same sums are held as matrix-instruction results oq[e][n] (heads 4 n .. 4 n + 3).
  float m_run[NH], l_run[NH], o[VQ ? NH : 1][8];
  w_float4_t oq[2][NH4];                   // (!VQ) [channel of the lane's pair][heads 4 n .. 4 n + 3]
#pragma unroll
  for (int h = 0; h < NH; ++h) {
    m_run[h] = -INFINITY;
    l_run[h] = 0.f;
    if constexpr (VQ) {
#pragma unroll
      for (int e = 0; e < 8; ++e) o[h][e] = 0.f;
    }
  }
#pragma unroll
  for (int e = 0; e < 2; ++e)
#pragma unroll
    for (int n = 0; n < NH4; ++n) oq[e][n] = w_float4_t{0.f, 0.f, 0.f, 0.f};

  // the query (and its per-channel factors, if any) first: what the step below waits for first
  w_u32x4 q_raw[NH4];
  w_float4_t q_fac[NH4][2];
#pragma unroll
  for (int rnd = 0; rnd < NH4; ++rnd) {
    const int idx = rnd * 64 + lane;
    const int h = idx / (D / 8), c0 = 8 * (idx % (D / 8));
    q_raw[rnd] = w_u32x4{0u, 0u, 0u, 0u};
    if (h < r) q_raw[rnd] = *reinterpret_cast<const w_u32x4*>(a.q + ((long long)b * a.n_q_heads + hk * r + h) * D + c0);
    if (a.q_scale) {
      q_fac[rnd][0] = *reinterpret_cast<const w_float4_t*>(a.q_scale + hk * D + c0);
      q_fac[rnd][1] = *reinterpret_cast<const w_float4_t*>(a.q_scale + hk * D + c0 + 4);
    }
  }

  for (long long base = v0; base < v1; base += 64) {
    // ---- all loads of this step
    w_u32x4 kreg[16], vreg[VQ ? 16 : 1];
    uint32_t vw[VQ ? 1 : 64];                      // (!VQ) this lane's channel pair of every token of the step
    uint32_t ks[2] = {0u, 0u}, kz[2] = {0u, 0u};   // packed key row: scales and zero-points, fp16 pairs
    bool k_packed = false;
    uint32_t v_packed = 0u;                        // bit k: value row k of this lane is a packed row
    const long long v = base + lane;
    const bool valid = v < v1;
    const int n_here = (int)(v1 - base < 64 ? v1 - base : 64);
    {
      const long long t = token_of(valid ? v : v1 - 1);        // idle lanes re-read the last row
      const __half* krow = fp16_row(a.k, a, bh, t);
      if (KQ && !krow) {
        k_packed = true;
        const long long row = PAGED ? store_row(a.pages, a.n_kv_heads, a.capacity, bh, t - a.w_sink)
                                    : bh * a.capacity + (t - a.w_sink);
        const w_u32x4* rowp = reinterpret_cast<const w_u32x4*>(a.k.codes + row * (D * BITS / 8));
#pragma unroll
        for (int i = 0; i < KVEC; ++i) kreg[i] = rowp[i];
        const uint32_t* sp = reinterpret_cast<const uint32_t*>(a.k.scales + row * NG);
#pragma unroll
        for (int i = 0; i < NG / 2; ++i) ks[i] = sp[i];
        if (a.k.zeros) {
          const uint32_t* zp = reinterpret_cast<const uint32_t*>(a.k.zeros + row * NG);
#pragma unroll
          for (int i = 0; i < NG / 2; ++i) kz[i] = zp[i];
        }
      } else {                                              // an fp16 row (always, unless KQ)
#pragma unroll
        for (int i = 0; i < 16; ++i) kreg[i] = *reinterpret_cast<const w_u32x4*>(krow + i * 8);
      }
    }
    if constexpr (VQ) {
#pragma unroll
      for (int k = 0; k < 16; ++k) {
        if (4 * k >= n_here) {                             // (uniform) no row left in this step
          vreg[k] = w_u32x4{0u, 0u, 0u, 0u};               // meets weight 0 below: must be finite
          continue;
        }
        const int j = 4 * k + tg;
        const long long tj = token_of(base + (j < n_here ? j : n_here - 1));
        const __half* vrow = fp16_row(a.v, a, bh, tj);
        if (VQ && !vrow) {
          v_packed |= 1u << k;
          const long long row = PAGED ? store_row(a.pages, a.n_kv_heads, a.capacity, bh, tj - a.w_sink)
                                      : bh * a.capacity + (tj - a.w_sink);
          const int c0 = 8 * cg;
          const uint8_t* cp = a.v.codes + row * (D * BITS / 8) + (c0 * BITS) / 8;
          const long long si = row * NG + c0 / G;
          w_u32x4 m = w_u32x4{0u, 0u, 0u, 0u};
          if constexpr (BITS == 2) m.x = (uint32_t)*reinterpret_cast<const unsigned short*>(cp);
          else m.x = *reinterpret_cast<const uint32_t*>(cp);
          m.y = (uint32_t)__half_as_ushort(a.v.scales[si]);
          if (a.v.zeros) m.z = (uint32_t)__half_as_ushort(a.v.zeros[si]);
          vreg[k] = m;
        } else {                                              // an fp16 row (always, unless VQ)
          vreg[k] = *reinterpret_cast<const w_u32x4*>(vrow + 8 * cg);
        }
      }
    } else {
      // the value row of this lane's token, as two 32-bit halves that the loads below read lane by lane
      const uintptr_t vrow_own = reinterpret_cast<uintptr_t>(fp16_row(a.v, a, bh, token_of(valid ? v : v1 - 1)));
      const int own_lo = (int)(uint32_t)vrow_own, own_hi = (int)(uint32_t)(vrow_own >> 32);
#pragma unroll
      for (int kq = 0; kq < 16; ++kq) {
        if (4 * kq >= n_here) {                          // (uniform) no row left in this step
#pragma unroll
          for (int i = 0; i < 4; ++i) vw[4 * kq + i] = 0u;   // meets weight 0 below: must be finite
          continue;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int j = 4 * kq + i < n_here ? 4 * kq + i : n_here - 1;     // rows past the end re-read the last one
          const uintptr_t row = ((uintptr_t)(uint32_t)__builtin_amdgcn_readlane(own_hi, j) << 32) |
                                (uintptr_t)(uint32_t)__builtin_amdgcn_readlane(own_lo, j);
          vw[4 * kq + i] = reinterpret_cast<const uint32_t*>(row)[lane];
        }
      }
    }

    if (base == v0) {
      // ---- query: a lane takes 8 consecutive channels of one head (one 16-byte load)
#pragma unroll
      for (int rnd = 0; rnd < NH4; ++rnd) {
        const int idx = rnd * 64 + lane;
        const int h = idx / (D / 8), c0 = 8 * (idx % (D / 8));
        const w_u32x4 raw = q_raw[rnd];
        const uint32_t rw[4] = {raw.x, raw.y, raw.z, raw.w};
        float part = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          float qv = (e & 1) ? window_half_hi(rw[e / 2]) : window_half_lo(rw[e / 2]);
          if (a.q_scale) qv = __half2float(scaled_half(qv, q_fac[rnd][e / 4][e % 4]));
          wq[h][c0 + e] = (_Float16)qv;
          part += qv;
        }
        if constexpr (KQ) {
          // sum over the G/8 lanes that hold one key group (4 lanes: one quad; 8 lanes: two quads)
          part += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, part), 0xB1, 0xF, 0xF, true));
          part += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, part), 0x4E, 0xF, 0xF, true));
          if constexpr (G == 64)
            part += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, part), 0x141, 0xF, 0xF, true));
          if ((idx % (G / 8)) == 0) wqs[c0 / G][h] = part;
        }
      }
    }
    __syncthreads();

    // ---- packed key rows (KQ): the stored fields take the place of the fp16 row, as the fp16
    // integers they are (0x6400 | u is 1024 + u; minus 1024, exact), so that one pass through the
    // matrix cores serves both kinds of row; the scale and zero-point of each group go on afterwards
    // (Eq. hybrid_dequant: |S| * sum(q * field) + Zeff * sum(q), the fields taken as they are stored).
    if (KQ && k_packed) {
      uint32_t pk[KVEC * 4];
#pragma unroll
      for (int i = 0; i < KVEC; ++i) { pk[4 * i] = kreg[i].x; pk[4 * i + 1] = kreg[i].y; pk[4 * i + 2] = kreg[i].z; pk[4 * i + 3] = kreg[i].w; }
      auto field = [&](int c) -> uint32_t {
        if constexpr (BITS == 3)      // a plane of 2-bit low parts (D/16 words), then a plane of high bits (D/32 words)
          return ((pk[c / 16] >> (2 * (c % 16))) & 3u) | (((pk[D / 16 + c / 32] >> (c % 32)) & 1u) << 2);
        else
          return (pk[c / FPW] >> ((c % FPW) * BITS)) & FMASK;
      };
      typedef _Float16 w_half2_t __attribute__((ext_vector_type(2)));
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        uint32_t wd[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int c = 8 * i + 2 * k;
          const uint32_t both = field(c) | (field(c + 1) << 16) | 0x64006400u;
          const w_half2_t u = __builtin_bit_cast(w_half2_t, both) - w_half2_t{(_Float16)1024.0f, (_Float16)1024.0f};
          wd[k] = __builtin_bit_cast(uint32_t, u);
        }
        kreg[i] = w_u32x4{wd[0], wd[1], wd[2], wd[3]};
      }
    }

    // ---- scores: lane = token, through the matrix cores: 4x4x4 blocks, B = four consecutive
    // channels of the lane's row, A = the same channels of the four heads (from wq), the four
    // results land in the lane that holds the token.  One accumulator per key group: independent
    // chains, and what a packed row needs.
    float s[NH];
    {
      w_float4_t sacc[NH4][NG];
#pragma unroll
      for (int n = 0; n < NH4; ++n)
#pragma unroll
        for (int g = 0; g < NG; ++g) sacc[n][g] = w_float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < 16; ++i) {
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
          w_u32x2 bw;
          bw.x = hf ? kreg[i].z : kreg[i].x;
          bw.y = hf ? kreg[i].w : kreg[i].y;
          const w_half4_t bop = __builtin_bit_cast(w_half4_t, bw);
#pragma unroll
          for (int n = 0; n < NH4; ++n) {
            const w_half4_t aop = *reinterpret_cast<const w_half4_t*>(&wq[4 * n + (lane & 3)][8 * i + 4 * hf]);
            sacc[n][(8 * i) / G] = __builtin_amdgcn_mfma_f32_4x4x4f16(aop, bop, sacc[n][(8 * i) / G], 0, 0, 0);
          }
        }
      }
#pragma unroll
      for (int h = 0; h < NH; ++h) {
        s[h] = 0.f;
#pragma unroll
        for (int g = 0; g < NG; ++g) s[h] += sacc[h / 4][g][h % 4];
      }
      if (KQ && k_packed) {
#pragma unroll
        for (int h = 0; h < NH; ++h) s[h] = 0.f;
#pragma unroll
        for (int g = 0; g < NG; ++g) {
          const float sc = (g & 1) ? window_half_hi(ks[g / 2]) : window_half_lo(ks[g / 2]);
          const float zp = (g & 1) ? window_half_hi(kz[g / 2]) : window_half_lo(kz[g / 2]);
          const float S = fabsf(sc);
          const float zeff = (__float_as_uint(sc) >> 31) ? zp : -S * HALFCODE;
#pragma unroll
          for (int h = 0; h < NH; ++h) s[h] += S * sacc[h / 4][g][h % 4] + zeff * wqs[g][h];
        }
      }
    }
    __syncthreads();
    // ---- running softmax
#pragma unroll
    for (int h = 0; h < NH; ++h) {
      const float sv = valid ? s[h] * c_log2 : -INFINITY;
      const float m_new = fmaxf(m_run[h], window_wave_max(sv));
      const float alpha = __builtin_amdgcn_exp2f(m_run[h] - m_new);
      float p = __builtin_amdgcn_exp2f(sv - m_new);      // 0 for the idle lanes
      if constexpr (!VQ) {
        // the weight the matrix cores will use, so that the normaliser stays consistent
        const _Float16 p16 = (_Float16)p;
        p = (float)p16;
        wp16[h * 64 + lane] = p16;
      } else {
        wp[lane][h] = p;
      }
      l_run[h] = l_run[h] * alpha + window_wave_sum(p);
      m_run[h] = m_new;
      if constexpr (VQ) {
#pragma unroll
        for (int e = 0; e < 8; ++e) o[h][e] *= alpha;
      } else {
#pragma unroll
        for (int e = 0; e < 2; ++e) oq[e][h / 4][h % 4] *= alpha;
      }
    }
    __syncthreads();
    // ---- values: 16 lanes share one token row (8 channels = 16 bytes each), 4 rows per load
    // instruction; a lane keeps o[head][8 channels] of the tokens (4k + lane/16) and the four
    // lane groups are summed at the end.  Rows past the end carry probability 0.
    if constexpr (!VQ) {
      // matrix cores: contraction over four tokens (4 kq .. 4 kq + 3), B = one channel of this lane
      // for those tokens (halves gathered from the four row words), A = the fp16 weights of the four
      // heads for the same tokens; the four results are the lane's own channel for the four heads
#pragma unroll
      for (int kq = 0; kq < 16; ++kq) {
        if (4 * kq >= n_here) break;                     // (uniform) no row left in this step
        const uint32_t w0 = vw[4 * kq], w1 = vw[4 * kq + 1], w2 = vw[4 * kq + 2], w3 = vw[4 * kq + 3];
        w_u32x2 lo, hi;
        lo.x = __builtin_amdgcn_perm(w1, w0, 0x05040100u);   // low halves: channel 2 lane of tokens 0, 1
        lo.y = __builtin_amdgcn_perm(w3, w2, 0x05040100u);
        hi.x = __builtin_amdgcn_perm(w1, w0, 0x07060302u);   // high halves: channel 2 lane + 1
        hi.y = __builtin_amdgcn_perm(w3, w2, 0x07060302u);
        const w_half4_t blo = __builtin_bit_cast(w_half4_t, lo), bhi = __builtin_bit_cast(w_half4_t, hi);
#pragma unroll
        for (int n = 0; n < NH4; ++n) {
          const w_half4_t aop = *reinterpret_cast<const w_half4_t*>(&wp16[(4 * n + (lane & 3)) * 64 + 4 * kq]);
          oq[0][n] = __builtin_amdgcn_mfma_f32_4x4x4f16(aop, blo, oq[0][n], 0, 0, 0);
          oq[1][n] = __builtin_amdgcn_mfma_f32_4x4x4f16(aop, bhi, oq[1][n], 0, 0, 0);
        }
      }
    } else {
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      if (4 * k >= n_here) break;                        // (uniform) no row left in this step
      const int j = 4 * k + tg;
      float x[8];
      if (VQ && ((v_packed >> k) & 1u)) {
        const uint32_t wbits = vreg[k].x;
        const float sc = window_half_lo(vreg[k].y);
        const float S = fabsf(sc);
        const float zeff = (__float_as_uint(sc) >> 31) ? window_half_lo(vreg[k].z) : -S * HALFCODE;
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = S * (float)((wbits >> (e * BITS)) & FMASK) + zeff;
      } else {
        const uint32_t pw[4] = {vreg[k].x, vreg[k].y, vreg[k].z, vreg[k].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          x[2 * e] = window_half_lo(pw[e]);
          x[2 * e + 1] = window_half_hi(pw[e]);
        }
      }
#pragma unroll
      for (int n = 0; n < NH4; ++n) {
        const w_float4_t pj = *reinterpret_cast<const w_float4_t*>(&wp[j][n * 4]);
        const float pv[4] = {pj.x, pj.y, pj.z, pj.w};
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int e = 0; e < 8; ++e) o[n * 4 + i][e] += pv[i] * x[e];
      }
    }
    }
    __syncthreads();
  }

  if constexpr (!VQ) {
    // ---- every lane holds its two channels, complete
#pragma unroll
    for (int h = 0; h < NH; ++h) {
      if (h < r) {
        const long long bhq = (long long)b * a.n_q_heads + hk * r + h;
        float2 ov;
        ov.x = oq[0][h / 4][h % 4];
        ov.y = oq[1][h / 4][h % 4];
        *reinterpret_cast<float2*>(&a.ws_o[(bhq * a.n_partials + slot) * D + 2 * lane]) = ov;
        if (lane == 0) {
          a.ws_ml[(bhq * a.n_partials + slot) * 2 + 0] = m_run[h] * 0.6931471805599453f;
          a.ws_ml[(bhq * a.n_partials + slot) * 2 + 1] = l_run[h];
        }
      }
    }
  } else {
  // ---- sum the four lane groups; lanes 0..15 then hold channels 8*lane .. 8*lane+7
#pragma unroll
  for (int h = 0; h < NH; ++h)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      o[h][e] += __shfl_xor(o[h][e], 16);
      o[h][e] += __shfl_xor(o[h][e], 32);
    }
#pragma unroll
  for (int h = 0; h < NH; ++h) {
    if (h < r) {
      const long long bhq = (long long)b * a.n_q_heads + hk * r + h;
      if (lane < 16) {
        float* dst = &a.ws_o[(bhq * a.n_partials + slot) * D + 8 * lane];
        *reinterpret_cast<w_float4_t*>(dst) = w_float4_t{o[h][0], o[h][1], o[h][2], o[h][3]};
        *reinterpret_cast<w_float4_t*>(dst + 4) = w_float4_t{o[h][4], o[h][5], o[h][6], o[h][7]};
      }
      if (lane == 0) {
        a.ws_ml[(bhq * a.n_partials + slot) * 2 + 0] = m_run[h] * 0.6931471805599453f;
        a.ws_ml[(bhq * a.n_partials + slot) * 2 + 1] = l_run[h];
      }
    }
  }
  }
}

}  // namespace innerq
