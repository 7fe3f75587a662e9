// Fused dequantise + score + softmax + value kernel for 2-bit inner-grouped caches on the
// block-scaled matrix instruction of CDNA4 (v_mfma_scale_f32_16x16x128_f8f6f4).
//
// Same decomposition as attention_inner.hip (Section "InnerQ": with groups along the inner
// dimension a group's scale and zero-point factor out of the inner sums, Eq. hybrid_dequant), same
// launch shape, same partial results.  What differs is how the raw inner sums over the stored
// fields are formed:
//   * a 2-bit field u, zero-extended to a nibble, IS the E2M1 number u/2 (0, 0.5, 1, 1.5).  A
//     packed word therefore becomes two fp4 operand registers with one shift and two ANDs (16
//     fields), against eight ANDs for the fp16-denormal form of the 4x4x4 kernel.
//   * the other operand (query; softmax weights) must then be fp8.  An fp16 query value, scaled
//     per head by a power of two into [128, 256), is exactly a1 + a2/16 + a3/256 with three E4M3
//     numbers (4 significant bits each; the factors 1/16 and 1/256 are the instruction's block
//     scales), so three instructions reproduce the exact fp16 product sums.  A softmax weight
//     x = 32 p <= 256 is split the same way: relative error <= 2^-12, absolute floor 2^-23 in p.
//   * one instruction contracts K = 128 in four blocks of 32 (one block per 16-lane row of the B
//     operand).  The A operand is block diagonal: row (g, h) holds head h's values in the k-blocks
//     of inner group g and zeros elsewhere, so the 16 x 16 result holds, for 16 tokens (keys) or
//     16 channels (values), the sums of every group separately: C[(g, h), n].  Three quarters of
//     the multiplies hit zeros; the instruction is still 4x cheaper per useful product than the
//     4x4x4 form, and the A operands are shared by every token (keys) or channel (values) of a tile.
//   * k-index layout, measured: an fp8 operand register block of lane (m, kb) holds
//     k = 16 kb + 0..15 (registers 0-3, byte order) and k = 64 + 16 kb + 0..15 (registers 4-7);
//     an fp4 operand of lane (n, kb) holds k = 32 kb + 0..31 (registers 0-3, nibble order).
//     C[row 4 mb + i, n] sits in register i of lane (n, mb).
//   * keys: B lane (n, kb) holds bytes 8 kb .. 8 kb + 7 of the row of token 16 i + n (four
//     instructions i per 64 tokens); the results (lane row = group) are transposed across the
//     four lane rows with v_permlane32_swap / v_permlane16_swap so that lane = token owns all
//     groups and all heads, next to that token's scales (one 8-byte load, as before).
//   * values: a tile is 128 tokens = 4 (G = 32) or 2 (G = 64) token groups; B lane (n, kb) holds the
//     32 tokens of block kb for channels 2 (16 r' + n) and + 1 (one 16-byte load per r').  The
//     result for token group T lands in lane row T, which loaded that group's scales; each lane
//     row accumulates its own token groups and the rows are added once, at the end.
//
// Status: parity-green (same tolerance as the 4x4x4 kernel) and NOT the default.  On the 32k-token
// Llama-3-8B-shaped configuration it takes 61 us against 40 us for the 4x4x4 kernel, with or
// without its loads.  Counters: 25 % fewer vector instructions per token than the 4x4x4 kernel,
// but an fp8 x fp4 instruction occupies the matrix pipe for 32 cycles (the fp8 rate: 8 passes, not
// the 4 of an all-fp4 product), so the matrix-pipe time per token is 27 % higher, and with two
// wavefronts per SIMD the longer dependent chains (three chained instructions per sum, the row
// transposes, the three-way split of the weights) leave the SIMD idle 40 % of the time.
#include "innerq_dev.h"
#include "window_pass.h"

namespace innerq {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float f4_float4 __attribute__((ext_vector_type(4)));
typedef float f4_float2 __attribute__((ext_vector_type(2)));
typedef _Float16 f4_half2 __attribute__((ext_vector_type(2)));
typedef uint32_t f4_u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t f4_u32x4 __attribute__((ext_vector_type(4)));

constexpr int D = kHeadDim;
constexpr int ST = 128;                        // tokens per wave iteration
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kSmScale = 0.08838834764831845f;   // 1/sqrt(128)
constexpr uint32_t kNib = 0x33333333u;         // the low two bits of every nibble
constexpr int kScale0 = 127, kScale1 = 123, kScale2 = 119;   // E8M0 block scales 1, 1/16, 1/256
constexpr float kXShift = 5.0f;                // softmax weights are stored as x = 32 p
constexpr float kSlack = 3.0f;                 // p <= 2^3 before the reference level is raised

__device__ inline _Float16 f4_half_of(uint32_t w, int hi) {
  return __builtin_bit_cast(_Float16, (unsigned short)(hi ? (w >> 16) : (w & 0xffffu)));
}

template <typename T>
__device__ inline T f4_stream_load(const T* p) { return __builtin_nontemporal_load(p); }

// maximum over the 16 lanes of a row (DPP butterflies)
__device__ inline float f4_row_max(float x) {
  x = fmaxf(x, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true)));
  x = fmaxf(x, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, true)));
  x = fmaxf(x, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xF, 0xF, true)));
  x = fmaxf(x, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xF, 0xF, true)));
  return x;
}

__device__ inline float f4_wave_max(float x) {
  x = f4_row_max(x);
  const float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 0));
  const float b = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 16));
  const float c = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 32));
  const float d = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 48));
  return fmaxf(fmaxf(a, b), fmaxf(c, d));
}

// Four values (|x| <= 256) as three E4M3 numbers each, x = a1 + a2/16 + a3/256 (+ at most 2^-12 |x|
// or 2^-18): the bytes of d1, d2, d3 in argument order.
__device__ inline void split3(float x0, float x1, float x2, float x3, uint32_t& d1, uint32_t& d2, uint32_t& d3) {
  int p = __builtin_amdgcn_cvt_pk_fp8_f32(x0, x1, 0, false);
  p = __builtin_amdgcn_cvt_pk_fp8_f32(x2, x3, p, true);
  d1 = (uint32_t)p;
  f4_float2 lo = __builtin_amdgcn_cvt_pk_f32_fp8(p, false), hi = __builtin_amdgcn_cvt_pk_f32_fp8(p, true);
  const float y0 = (x0 - lo.x) * 16.f, y1 = (x1 - lo.y) * 16.f, y2 = (x2 - hi.x) * 16.f, y3 = (x3 - hi.y) * 16.f;
  p = __builtin_amdgcn_cvt_pk_fp8_f32(y0, y1, 0, false);
  p = __builtin_amdgcn_cvt_pk_fp8_f32(y2, y3, p, true);
  d2 = (uint32_t)p;
  lo = __builtin_amdgcn_cvt_pk_f32_fp8(p, false);
  hi = __builtin_amdgcn_cvt_pk_f32_fp8(p, true);
  const float z0 = (y0 - lo.x) * 16.f, z1 = (y1 - lo.y) * 16.f, z2 = (y2 - hi.x) * 16.f, z3 = (y3 - hi.y) * 16.f;
  p = __builtin_amdgcn_cvt_pk_fp8_f32(z0, z1, 0, false);
  p = __builtin_amdgcn_cvt_pk_fp8_f32(z2, z3, p, true);
  d3 = (uint32_t)p;
}

// Two packed words (32 two-bit fields) as an fp4 operand: registers lo(w0), hi(w0), lo(w1), hi(w1).
// k = 8 v + j of the block holds field 16 (v / 2) + 2 j + (v % 2).
__device__ inline v8i expand(uint32_t w0, uint32_t w1) {
  v8i b = {0, 0, 0, 0, 0, 0, 0, 0};
  b[0] = (int)(w0 & kNib);
  b[1] = (int)((w0 >> 2) & kNib);
  b[2] = (int)(w1 & kNib);
  b[3] = (int)((w1 >> 2) & kNib);
  return b;
}

// c + A (fp8, block scale 2^(sa - 127)) x B (fp4)
__device__ inline f4_float4 mma(const v8i& a, const v8i& b, f4_float4 c, int sa) {
  return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 0, 4, 0, sa, 0, kScale0);
}

// v_permlane32_swap: a' = [a rows 0-1, b rows 0-1], b' = [a rows 2-3, b rows 2-3] (rows of 16 lanes);
// v_permlane16_swap: a' = [a row 0, b row 0, a row 2, b row 2], b' = [a row 1, b row 1, a row 3, b row 3].
__device__ inline void swap32(float& a, float& b) {
  auto r = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(unsigned, a), __builtin_bit_cast(unsigned, b), false, false);
  const unsigned r0 = r[0], r1 = r[1];                 // (a subscript inside the bit cast reads element 0 twice)
  a = __builtin_bit_cast(float, r0);
  b = __builtin_bit_cast(float, r1);
}
__device__ inline void swap16(float& a, float& b) {
  auto r = __builtin_amdgcn_permlane16_swap(__builtin_bit_cast(unsigned, a), __builtin_bit_cast(unsigned, b), false, false);
  const unsigned r0 = r[0], r1 = r[1];                 // (a subscript inside the bit cast reads element 0 twice)
  a = __builtin_bit_cast(float, r0);
  b = __builtin_bit_cast(float, r1);
}

// What one wave iteration (128 tokens) reads from the quantised store: the key part (two copies in
// ping-pong) and the value part (one copy, re-loaded piece by piece as soon as a piece is used).
template <int G>
struct KeyRegsF4 {
  static constexpr int NG = D / G;
  f4_u32x2 kk[2][4];                 // [64-token half][token set i]: this lane's 8 bytes of the row of token 16 i + n
  uint32_t ks[2][NG / 2], kz[2][NG / 2];   // fp16 pairs: scales / zero-points of token `lane` of each half
};
struct ValueRegsF4 {
  f4_u32x4 vv[4];                    // [r']: 32 tokens of channels 2 (16 r' + n) and + 1
  uint32_t vs[4], vz[4];             // fp16 pairs for those two channels
};

template <int G, bool ZK, bool ZV>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2, 2)))
attention_inner_f4_kernel(AttnArgs a, int n_both, int n_splits, WindowSet win, int win_tiles) {
  using KRegs = KeyRegsF4<G>;
  using VRegs = ValueRegsF4;
  constexpr int NG = D / G;                            // key groups per token (4 or 2)
  constexpr int NH = 4;

  const int lane = threadIdx.x;
  const int n = lane & 15, kb = lane >> 4;
  const long long bh = blockIdx.y;
  const int b = (int)(bh / a.n_kv_heads), hk = (int)(bh % a.n_kv_heads);
  const int r = a.n_q_heads / a.n_kv_heads;

  // ---- range of 128-token tiles of this wavefront.  The first win.n_chunks wavefronts of a
  // (batch, kv-head) also serve one chunk of the fp16 windows each (after their tiles) and get
  // win_tiles tiles; the others share the remaining tiles evenly.
  const int n_tiles = (n_both + ST - 1) / ST;
  const int s_idx = (int)blockIdx.x;
  int t0, t1;
  if (s_idx < win.n_chunks) {
    t0 = s_idx * win_tiles;
    t1 = t0 + win_tiles;
  } else {
    const int rest = n_tiles - win.n_chunks * win_tiles, others = n_splits - win.n_chunks, j = s_idx - win.n_chunks;
    const int base_t = rest / others, rem_t = rest % others;
    t0 = win.n_chunks * win_tiles + j * base_t + (j < rem_t ? j : rem_t);
    t1 = t0 + base_t + (j < rem_t ? 1 : 0);
  }

  __shared__ __attribute__((aligned(16))) float qtab[NH][D];            // query times 2^eh (set-up only)
  __shared__ __attribute__((aligned(16))) float qsum[NG][NH];           // log2e/sqrt(d) * sum of q over each key group
  __shared__ __attribute__((aligned(16))) float hsc[NH];                // log2e/sqrt(d) * 2^(1 - eh)
  __shared__ __attribute__((aligned(16))) uint8_t xtab[3 * NH * ST + 16];   // weights [piece][head][k], then 16 zero bytes

  const uint8_t* kcodes = a.k.codes + bh * a.capacity * (D / 4);
  const __half* kscales = a.k.scales + bh * a.capacity * NG;
  const __half* kzeros = ZK ? a.k.zeros + bh * a.capacity * NG : nullptr;
  const long long vgroups = a.capacity / G;
  const uint8_t* vcodes = a.v.codes + bh * vgroups * D * (G / 4);
  const __half* vscales = a.v.scales + bh * vgroups * D;
  const __half* vzeros = ZV ? a.v.zeros + bh * vgroups * D : nullptr;
  const int last_row = n_both - 1, last_group = n_both / G - 1;

  // All offsets inside one (b, hk) slab fit 32 bits; bases are wave-uniform.
  auto load_keys = [&](int tile, KRegs& t) {
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        int row = tile * ST + sub * 64 + i * 16 + n;
        row = row > last_row ? last_row : row;
        t.kk[sub][i] = f4_stream_load(reinterpret_cast<const f4_u32x2*>(kcodes + (uint32_t)row * (D / 4) + 8 * kb));
      }
      int row = tile * ST + sub * 64 + lane;
      row = row > last_row ? last_row : row;
      if constexpr (NG == 4) {
        const f4_u32x2 s = f4_stream_load(reinterpret_cast<const f4_u32x2*>(kscales + (uint32_t)row * NG));
        t.ks[sub][0] = s.x; t.ks[sub][1] = s.y;
        if constexpr (ZK) {
          const f4_u32x2 z = f4_stream_load(reinterpret_cast<const f4_u32x2*>(kzeros + (uint32_t)row * NG));
          t.kz[sub][0] = z.x; t.kz[sub][1] = z.y;
        }
      } else {
        t.ks[sub][0] = f4_stream_load(reinterpret_cast<const uint32_t*>(kscales + (uint32_t)row * NG));
        if constexpr (ZK) t.kz[sub][0] = f4_stream_load(reinterpret_cast<const uint32_t*>(kzeros + (uint32_t)row * NG));
      }
    }
  };
  // values, piece rp of a tile: the codes of k-block kb; the scales of the token group whose
  // results land in lane row kb
  auto load_values = [&](int tile, int rp, VRegs& t) {
    int cgrp, sgrp;
    if constexpr (G == 32) {
      cgrp = tile * 4 + kb;
      sgrp = cgrp;
    } else {
      cgrp = tile * 2 + (kb >> 1);
      sgrp = tile * 2 + (kb & 1);
    }
    cgrp = cgrp > last_group ? last_group : cgrp;
    sgrp = sgrp > last_group ? last_group : sgrp;
    const uint32_t ch = 2 * (16 * rp + n);
    if constexpr (G == 32) {
      t.vv[rp] = f4_stream_load(reinterpret_cast<const f4_u32x4*>(vcodes + ((uint32_t)cgrp * D + ch) * 8));
    } else {
      const uint8_t* p = vcodes + ((uint32_t)cgrp * D + ch) * 16 + 8 * (kb & 1);
      const f4_u32x2 c0 = f4_stream_load(reinterpret_cast<const f4_u32x2*>(p));
      const f4_u32x2 c1 = f4_stream_load(reinterpret_cast<const f4_u32x2*>(p + 16));
      t.vv[rp] = f4_u32x4{c0.x, c0.y, c1.x, c1.y};
    }
    t.vs[rp] = f4_stream_load(reinterpret_cast<const uint32_t*>(vscales + (uint32_t)sgrp * D + ch));
    if constexpr (ZV) t.vz[rp] = f4_stream_load(reinterpret_cast<const uint32_t*>(vzeros + (uint32_t)sgrp * D + ch));
  };

  // ---- the query loads go out first, the first tile's loads right behind them
  const int h_ld = lane >> 4, c0 = 8 * (lane & 15);          // set-up: a lane takes 8 channels of one head
  f4_u32x4 q_raw = {0u, 0u, 0u, 0u};
  if (h_ld < r) q_raw = *reinterpret_cast<const f4_u32x4*>(a.q + ((long long)b * a.n_q_heads + hk * r + h_ld) * D + c0);
  KRegs keyA, keyB;
  VRegs val;
  if (t1 > t0) {
    load_keys(t0, keyA);
#pragma unroll
    for (int rp = 0; rp < 4; ++rp) load_values(t0, rp, val);
  }

  // ---- query: fp16 (optionally rescaled), scaled per head by 2^eh into [128, 256)
  {
    const uint32_t rw[4] = {q_raw.x, q_raw.y, q_raw.z, q_raw.w};
    float qv[8], part = 0.f, amax = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t hb = (e & 1) ? (rw[e / 2] >> 16) : (rw[e / 2] & 0xffffu);
      qv[e] = __half2float(__ushort_as_half((unsigned short)hb));
      if (a.q_scale) qv[e] = __half2float(scaled_half(qv[e], a.q_scale[hk * D + c0 + e]));
      part += qv[e];
      amax = fmaxf(amax, __builtin_fabsf(qv[e]));
    }
    // sum over the G/8 lanes of the group (4 lanes: one quad; 8 lanes: two quads)
    part += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, part), 0xB1, 0xF, 0xF, true));
    part += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, part), 0x4E, 0xF, 0xF, true));
    if constexpr (G == 64)
      part += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, part), 0x141, 0xF, 0xF, true));
    if ((lane % (G / 8)) == 0) qsum[c0 / G][h_ld] = part * (kSmScale * kLog2e);
    amax = f4_row_max(amax);                                  // the 16 lanes of a row hold one head
    const int eh = amax > 0.f ? 8 - __builtin_amdgcn_frexp_expf(amax) : 0;   // amax * 2^eh in [128, 256)
#pragma unroll
    for (int e = 0; e < 8; ++e) qtab[h_ld][c0 + e] = __builtin_ldexpf(qv[e], eh);
    if ((lane & 15) == 0) hsc[h_ld] = __builtin_ldexpf(kSmScale * kLog2e, 1 - eh);   // fp4 fields are u/2
    if (lane < 4) reinterpret_cast<uint32_t*>(xtab + 3 * NH * ST)[lane] = 0u;
  }
  __syncthreads();

  // ---- A operands of the score pass: row m = (group, head); registers 0-3 hold k = 16 kb + i,
  // registers 4-7 k = 64 + 16 kb + i; k stands for channel 16 (k / 16) + 2 (i % 8) + i / 8.
  v8i AK[3];
  {
    const int hA = n & 3, gA = n >> 2;
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
      const int k0 = 64 * hf + 16 * kb;
      const bool active = (k0 / G) == gA;
      float v[16];
#pragma unroll
      for (int j4 = 0; j4 < 4; ++j4) {
        const f4_float4 t = *reinterpret_cast<const f4_float4*>(&qtab[hA][k0 + 4 * j4]);
        v[4 * j4] = t.x; v[4 * j4 + 1] = t.y; v[4 * j4 + 2] = t.z; v[4 * j4 + 3] = t.w;
      }
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        uint32_t d1, d2, d3;
        // bytes i = 4 d .. 4 d + 3 hold channels 2 (i % 8) + i / 8 of the 16
        const int i0 = 4 * d;
        split3(v[2 * (i0 % 8) + i0 / 8], v[2 * ((i0 + 1) % 8) + (i0 + 1) / 8], v[2 * ((i0 + 2) % 8) + (i0 + 2) / 8],
               v[2 * ((i0 + 3) % 8) + (i0 + 3) / 8], d1, d2, d3);
        AK[0][4 * hf + d] = active ? (int)d1 : 0;
        AK[1][4 * hf + d] = active ? (int)d2 : 0;
        AK[2][4 * hf + d] = active ? (int)d3 : 0;
      }
    }
  }
  float hs[NH];
  {
    const f4_float4 t = *reinterpret_cast<const f4_float4*>(&hsc[0]);
    hs[0] = t.x; hs[1] = t.y; hs[2] = t.z; hs[3] = t.w;
  }

  // ---- where the softmax weights go (lane = token of a 64-token half) and come from (A operand)
  // token tau of the tile sits at k = 16 (tau / 16) + 8 (tau % 2) + (tau % 16) / 2
  int x_write[2];
#pragma unroll
  for (int sub = 0; sub < 2; ++sub) {
    const int tau = 64 * sub + lane;
    x_write[sub] = 16 * (tau / 16) + 8 * (tau % 2) + (tau % 16) / 2;
  }
  int x_read[2];                                             // byte offsets inside one piece's table
#pragma unroll
  for (int hf = 0; hf < 2; ++hf) {
    const int k0 = 64 * hf + 16 * kb;
    const bool active = (k0 / G) == (n >> 2);
    x_read[hf] = active ? (n & 3) * ST + k0 : -1;
  }

  // ---- running softmax state (log2 domain) and output accumulators.  m_run is a reference
  // level, not the exact running maximum: it is raised (and l, o rescaled) only when some score
  // exceeds it by more than kSlack.  o[2 r' + c][h]: channel 2 (16 r' + n) + c, this lane row's
  // token groups only; l_run likewise.  Both are kept times 16.
  float m_run[NH], l_run[NH], o[8][NH];
#pragma unroll
  for (int h = 0; h < NH; ++h) {
    m_run[h] = 0.f; l_run[h] = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i][h] = 0.f;
  }
  v8i ones = {0x11111111, 0x11111111, 0x11111111, 0x11111111, 0, 0, 0, 0};   // every field 0.5

  auto process = [&](const KRegs& cur, int tile, bool first, bool more) {
    // ================= scores (Eq. att:1 with Eq. hybrid_dequant fused) =================
    float e[2][NH];
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      f4_float4 acc[4];
      v8i bop[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        bop[i] = expand(cur.kk[sub][i].x, cur.kk[sub][i].y);
        acc[i] = mma(AK[0], bop[i], f4_float4{0.f, 0.f, 0.f, 0.f}, kScale0);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = mma(AK[1], bop[i], acc[i], kScale1);
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = mma(AK[2], bop[i], acc[i], kScale2);
      // acc[i][h] in lane (n, g): token 16 i + n, group g.  Transpose the 4 x 4 (i, lane row)
      // blocks: afterwards lane (n, row) = token 16 row + n holds group g in grp[g][h].
      float grp[NG][NH];
#pragma unroll
      for (int h = 0; h < NH; ++h) {
        float a0 = acc[0][h], a1 = acc[1][h], a2 = acc[2][h], a3 = acc[3][h];
        swap32(a0, a2);
        swap32(a1, a3);
        swap16(a0, a1);
        grp[0][h] = a0; grp[1][h] = a1;
        if constexpr (NG == 4) {
          swap16(a2, a3);
          grp[2][h] = a2; grp[3][h] = a3;
        }
      }
      // per group: |S| * (raw inner sum) + Zeff * (sum of q); Zeff = Z - 2 max(s, 0) (the scale's
      // sign bit marks an asymmetric group, whose fields start at Z; a symmetric one stores +0)
      float t[NH];
#pragma unroll
      for (int h = 0; h < NH; ++h) { e[sub][h] = kXShift - m_run[h]; t[h] = 0.f; }
#pragma unroll
      for (int g = 0; g < NG; ++g) {
        const uint32_t spair = cur.ks[sub][g / 2];
        const _Float16 s16 = f4_half_of(spair, g & 1);
        float zeff;
        if constexpr (ZK) {
          const uint32_t mpair = __builtin_bit_cast(
              uint32_t, __builtin_elementwise_max(__builtin_bit_cast(f4_half2, spair), f4_half2{(_Float16)0, (_Float16)0}));
          zeff = __builtin_fmaf((float)f4_half_of(mpair, g & 1), -2.0f, (float)f4_half_of(cur.kz[sub][g / 2], g & 1));
        } else {
          zeff = (float)s16 * -2.0f;
        }
        const float S = __builtin_fabsf((float)s16);
        const f4_float4 qs = *reinterpret_cast<const f4_float4*>(&qsum[g][0]);
#pragma unroll
        for (int h = 0; h < NH; ++h) {
          t[h] = __builtin_fmaf(S, grp[g][h], t[h]);
          e[sub][h] = __builtin_fmaf(zeff, qs[h], e[sub][h]);
        }
      }
#pragma unroll
      for (int h = 0; h < NH; ++h) e[sub][h] = __builtin_fmaf(hs[h], t[h], e[sub][h]);
      if (tile * ST + sub * 64 + 63 > last_row) {          // ragged end: lanes past it weigh nothing
        const bool valid = tile * ST + sub * 64 + lane <= last_row;
#pragma unroll
        for (int h = 0; h < NH; ++h) e[sub][h] = valid ? e[sub][h] : -INFINITY;
      }
    }

    // ================= running softmax (Eq. att:2) =================
    bool raise = false;
#pragma unroll
    for (int h = 0; h < NH; ++h) raise |= fmaxf(e[0][h], e[1][h]) > kSlack + kXShift;
    if (first || __builtin_amdgcn_ballot_w64(raise) != 0) {   // rare after the first tiles
#pragma unroll
      for (int h = 0; h < NH; ++h) {
        const float mx = f4_wave_max(fmaxf(e[0][h], e[1][h]) - kXShift);   // largest score relative to the level
        const float d = first ? mx : fmaxf(mx, 0.f);
        const float alpha = first ? 1.f : __builtin_amdgcn_exp2f(-d);
        m_run[h] += d;
        e[0][h] -= d;
        e[1][h] -= d;
        l_run[h] *= alpha;
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i][h] *= alpha;
      }
    }
    __syncthreads();                                   // the previous tile's A operands are read
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      uint32_t d[3];
      split3(__builtin_amdgcn_exp2f(e[sub][0]), __builtin_amdgcn_exp2f(e[sub][1]), __builtin_amdgcn_exp2f(e[sub][2]),
             __builtin_amdgcn_exp2f(e[sub][3]), d[0], d[1], d[2]);
#pragma unroll
      for (int pc = 0; pc < 3; ++pc)
#pragma unroll
        for (int h = 0; h < NH; ++h) xtab[(pc * NH + h) * ST + x_write[sub]] = (uint8_t)(d[pc] >> (8 * h));
    }
    __syncthreads();

    // ================= values (Eq. att:3 with Eq. hybrid_dequant fused) =================
    v8i AV[3];
#pragma unroll
    for (int pc = 0; pc < 3; ++pc) {
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        const int off = x_read[hf] >= 0 ? pc * NH * ST + x_read[hf] : 3 * NH * ST;
        const f4_u32x4 w = *reinterpret_cast<const f4_u32x4*>(xtab + off);
        AV[pc][4 * hf] = (int)w.x; AV[pc][4 * hf + 1] = (int)w.y; AV[pc][4 * hf + 2] = (int)w.z; AV[pc][4 * hf + 3] = (int)w.w;
      }
    }
    // P[h] = 16 * (sum of the weights of this lane row's token group)
    f4_float4 P = mma(AV[0], ones, f4_float4{0.f, 0.f, 0.f, 0.f}, kScale0);
    P = mma(AV[1], ones, P, kScale1);
    P = mma(AV[2], ones, P, kScale2);
#pragma unroll
    for (int rp = 0; rp < 4; ++rp) {
      const v8i b0 = expand(val.vv[rp].x, val.vv[rp].y), b1 = expand(val.vv[rp].z, val.vv[rp].w);
      f4_float4 acc0 = mma(AV[0], b0, f4_float4{0.f, 0.f, 0.f, 0.f}, kScale0);
      f4_float4 acc1 = mma(AV[0], b1, f4_float4{0.f, 0.f, 0.f, 0.f}, kScale0);
      acc0 = mma(AV[1], b0, acc0, kScale1);
      acc1 = mma(AV[1], b1, acc1, kScale1);
      acc0 = mma(AV[2], b0, acc0, kScale2);
      acc1 = mma(AV[2], b1, acc1, kScale2);
      const uint32_t spair = val.vs[rp];
      const float S0 = __builtin_fabsf((float)f4_half_of(spair, 0)), S1 = __builtin_fabsf((float)f4_half_of(spair, 1));
      float z0, z1;
      if constexpr (ZV) {
        const uint32_t mpair = __builtin_bit_cast(
            uint32_t, __builtin_elementwise_max(__builtin_bit_cast(f4_half2, spair), f4_half2{(_Float16)0, (_Float16)0}));
        z0 = __builtin_fmaf((float)f4_half_of(mpair, 0), -2.0f, (float)f4_half_of(val.vz[rp], 0));
        z1 = __builtin_fmaf((float)f4_half_of(mpair, 1), -2.0f, (float)f4_half_of(val.vz[rp], 1));
      } else {
        z0 = S0 * -2.0f;
        z1 = S1 * -2.0f;
      }
      if (more) load_values(tile + 1, rp, val);          // this piece's registers are free again
#pragma unroll
      for (int h = 0; h < NH; ++h) {
        o[2 * rp][h] = __builtin_fmaf(S0, acc0[h], __builtin_fmaf(z0, P[h], o[2 * rp][h]));
        o[2 * rp + 1][h] = __builtin_fmaf(S1, acc1[h], __builtin_fmaf(z1, P[h], o[2 * rp + 1][h]));
      }
    }
#pragma unroll
    for (int h = 0; h < NH; ++h) l_run[h] += P[h];
  };

  // ---- keys: two register buffers in ping-pong (the next tile's keys are in flight while this
  // tile is computed); values: one buffer, each piece re-loaded for the next tile once it is used
  {
    const int nt = t1 - t0;
    int i = 0;
    while (i + 2 < nt) {
      // the wavefront that is behind gets the SIMD first, so the two of a SIMD finish together
      if (4 * i < nt) __builtin_amdgcn_s_setprio(3);
      else if (2 * i < nt) __builtin_amdgcn_s_setprio(2);
      else if (4 * i < 3 * nt) __builtin_amdgcn_s_setprio(1);
      else __builtin_amdgcn_s_setprio(0);
      load_keys(t0 + i + 1, keyB);
      process(keyA, t0 + i, i == 0, true);
      load_keys(t0 + i + 2, keyA);
      process(keyB, t0 + i + 1, false, true);
      i += 2;
    }
    if (nt - i == 2) {
      load_keys(t0 + i + 1, keyB);
      process(keyA, t0 + i, i == 0, true);
      process(keyB, t0 + i + 1, false, false);
    } else if (nt - i == 1) {
      process(keyA, t0 + i, i == 0, false);
    }
    if (nt <= 0) {                                      // no tile for this wavefront: an empty partial
#pragma unroll
      for (int h = 0; h < NH; ++h) m_run[h] = -INFINITY;
    }
  }

  // ---- add the four lane rows (each holds its own token groups): afterwards lane (n, row) owns
  // channels 2 (16 row + n) and + 1 = 2 lane, 2 lane + 1
  float oc[2][NH], l_tot[NH];
#pragma unroll
  for (int h = 0; h < NH; ++h) {
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      float a0 = o[0 + c][h], a1 = o[2 + c][h], a2 = o[4 + c][h], a3 = o[6 + c][h];   // r' = 0..3
      swap32(a0, a2);
      const float s02 = a0 + a2;                        // lower rows: r' = 0, upper rows: r' = 2
      swap32(a1, a3);
      float s13 = a1 + a3;
      float s = s02;
      swap16(s, s13);
      oc[c][h] = s + s13;
    }
    const float la = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, l_run[h]), 0));
    const float lb = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, l_run[h]), 16));
    const float lc = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, l_run[h]), 32));
    const float ld = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, l_run[h]), 48));
    l_tot[h] = (la + lb) + (lc + ld);
  }

  // ---- partial (m, l, o) of every real head
  const int slot = s_idx;
#pragma unroll
  for (int h = 0; h < NH; ++h) {
    if (h < r) {
      const long long bhq = (long long)b * a.n_q_heads + hk * r + h;
      float2 ov;
      ov.x = oc[0][h] * 0.0625f;                        // weights were stored as 32 p, fields as u/2
      ov.y = oc[1][h] * 0.0625f;
      *reinterpret_cast<float2*>(&a.ws_o[(bhq * a.n_partials + slot) * D + 2 * lane]) = ov;
      if (lane == 0) {
        a.ws_ml[(bhq * a.n_partials + slot) * 2 + 0] = m_run[h] * kLn2;
        a.ws_ml[(bhq * a.n_partials + slot) * 2 + 1] = l_tot[h] * 0.0625f;
      }
    }
  }

  // ---- the window chunk of this wavefront, with a partial slot of its own
  if (s_idx < win.n_chunks) {
    __syncthreads();
    window_pass<1, 2, G, true, false>(a, bh, win.na, win.b0, win.nb, s_idx, win.n_chunks, n_splits + s_idx);
  }
}

// 128-token tiles' worth of time a window chunk of `len` tokens costs the wavefront that carries it.
inline int window_cost_f4(long long len) { return (int)(1 + 6 * len / 64); }

template <int G, bool ZK, bool ZV>
hipError_t launch_z(const AttnArgs& a, int n_both, int n_splits, const WindowSet& win, const Launch& L) {
  const int n_tiles = (n_both + ST - 1) / ST;
  const int cost = win.n_chunks > 0 ? window_cost_f4((win.na + win.nb + win.n_chunks - 1) / win.n_chunks) : 0;
  const int quota = (n_tiles + win.n_chunks * cost + n_splits - 1) / n_splits;
  int win_tiles = quota > cost ? quota - cost : 0;
  if (win.n_chunks > 0 && win_tiles > n_tiles / win.n_chunks) win_tiles = n_tiles / win.n_chunks;
  if (n_splits <= win.n_chunks) return hipErrorInvalidValue;
  dim3 grid((unsigned)n_splits, (unsigned)(a.batch * a.n_kv_heads));
  hipExtLaunchKernelGGL((attention_inner_f4_kernel<G, ZK, ZV>), grid, dim3(64), 0, L.stream, L.ev_start, L.ev_stop, 0,
                        a, n_both, n_splits, win, win_tiles);
  return hipGetLastError();
}

template <int G, bool ZK, bool ZV>
int resident_z(const AttnArgs&) {
  int n = 0;
  const hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, attention_inner_f4_kernel<G, ZK, ZV>, 64, 0);
  return (e == hipSuccess && n > 0) ? n : 8;
}

template <int G>
hipError_t launch_g(const AttnArgs& a, int n_both, int n_splits, const WindowSet& win, const Launch& L) {
  const bool zk = a.k.zeros != nullptr, zv = a.v.zeros != nullptr;
  if (zk && zv) return launch_z<G, true, true>(a, n_both, n_splits, win, L);
  if (zk) return launch_z<G, true, false>(a, n_both, n_splits, win, L);
  if (zv) return launch_z<G, false, true>(a, n_both, n_splits, win, L);
  return launch_z<G, false, false>(a, n_both, n_splits, win, L);
}

template <int G>
int resident_g(const AttnArgs& a) {
  const bool zk = a.k.zeros != nullptr, zv = a.v.zeros != nullptr;
  if (zk && zv) return resident_z<G, true, true>(a);
  if (zk) return resident_z<G, true, false>(a);
  if (zv) return resident_z<G, false, true>(a);
  return resident_z<G, false, false>(a);
}

}  // namespace

bool attention_inner_f4_supported(const AttnArgs& a) {
  const int r = a.n_q_heads / a.n_kv_heads;
  // offsets inside one (batch, kv-head) slab are 32-bit in the kernel
  return a.k.form == kPerToken && a.v.form == kPerChannel && a.bits == 2 && a.v_bits == 2 && r <= 4 &&
         (a.group == 32 || a.group == 64) && a.capacity * D <= (1LL << 31) && !a.pages.table && !a.n_dev;
}

int attention_inner_f4_waves_per_cu(const AttnArgs& a) {
  static CachedInt cache[2][2][2];
  return cache[a.group == 64][a.k.zeros != nullptr][a.v.zeros != nullptr].get(
      [&] { return a.group == 32 ? resident_g<32>(a) : resident_g<64>(a); });
}

hipError_t launch_attention_inner_f4(const AttnArgs& a, long long n_both_ll, int n_splits, const WindowSet& win,
                                     hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop) {
  if (!attention_inner_f4_supported(a)) return hipErrorInvalidValue;
  const Launch L = {stream, ev_start, ev_stop};
  return a.group == 32 ? launch_g<32>(a, (int)n_both_ll, n_splits, win, L) : launch_g<64>(a, (int)n_both_ll, n_splits, win, L);
}

}  // namespace innerq
