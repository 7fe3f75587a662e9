// Comparison kernel: fused split-K decode attention over an OUTER-dimension-grouped cache
// (kind = INNERQ_KIND_OUTER: keys grouped along tokens per channel, values along channels per
// token -- the layout the paper compares against, Figure "inner_outer" (a)).
//
// Same skeleton as the inner-grouped and fp16 kernels (one wavefront per token range, 64-token
// tiles, register prefetch of the next tile, window wavefronts in the same launch, same merge), and
// built the same way as the inner-grouped kernel: the stored fields go to the 4x4x4 fp16 matrix
// instructions as they are, masked in place (a field inside bits 0..10 of a 16-bit half reads as
// field * 2^position * 2^-24), and scales and zero-points stay out of the element loop.  With outer
// grouping a group's scale depends on the index that is summed over, so it cannot be applied to the
// finished inner sum; it is folded into the OTHER operand instead, once per group:
//     q . K^[j]        = sum_c (q_c S_{c,T}) u[j][c]  +  sum_c q_c Zeff_{c,T}      (T: token group of j)
//     sum_j p_j V^[j][c] = sum_j (p_j S_{j,g}) u[j][c]  +  sum_j p_j Zeff_{j,g}    (g: channel group of c)
// i.e. a query table per token group and a weight table per channel group, rebuilt for every tile, and the
// zero-point terms as constants per group, summed on the matrix cores too.  (u = stored field, Zeff = Z for
// an asymmetric group and -2^(b-1) |S| for a symmetric one: Eq. hybrid_dequant.)
// What the grouping still forces, and the inner-grouped kernel does not pay:
//   * the tables themselves: products rounded to fp16 (the query table in two pieces, or the rounding of a
//     large channel's entry shows at 1e-3 on heavy-tailed keys), per-tile normalising shifts so that they
//     stay in fp16's normal range, their way through LDS, and twice the matrix instructions on the keys;
//   * the packing runs ACROSS the inner dimension (a key word holds 16 tokens of ONE channel, a value word
//     16 channels of ONE token) while every operand layout of the matrix instructions gives a lane
//     consecutive indices of the inner dimension: the key fields go through an LDS tile to reach the
//     one-token-per-lane score pass, and the value fields of two rows are put side by side in a register
//     so that one AND leaves one channel of two tokens.
#include "innerq_dev.h"
#include "window_pass.h"

namespace innerq {
namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int D = kHeadDim;
constexpr int TILE = 64;
constexpr int KROW = D + 8;                 // padded LDS row of the token-major key tile (halves)

// wave-wide maximum: the DPP form shared with the window pass
__device__ inline float wave_max_o(float x) { return window_wave_max(x); }
__device__ inline float half_lo(uint32_t p) { return __half2float(__ushort_as_half((unsigned short)(p & 0xffffu))); }
__device__ inline float half_hi(uint32_t p) { return __half2float(__ushort_as_half((unsigned short)(p >> 16))); }

template <int BITS, int G>
struct OuterRegs {
  static constexpr int GPT = TILE / G;                 // key token-groups per tile
  static constexpr int KC = 2 * G * BITS / 8 / 16;     // 16-byte pieces: two channels of one key group
  static constexpr int VC = D * BITS / 8 / 16;         // 16-byte pieces of one value row
  static constexpr int NG = D / G;                     // value groups per token
  u32x4 kc[GPT][KC];
  uint32_t ks[GPT], kz[GPT];                           // fp16 pairs (this lane's two channels)
  u32x4 vc[VC];
  uint32_t vs[NG / 2], vz[NG / 2];                     // fp16 pairs
};

typedef _Float16 half4_t __attribute__((ext_vector_type(4)));

typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));

// A b-bit field masked in place inside a 16-bit half reads, as fp16, as field * 2^(bit position) * 2^-24
// as long as it lies within bits 0..10 (the mantissa and the lowest exponent bit: the step from the
// denormals to the first binade keeps the spacing).  Fields above that are taken from a copy of the word
// shifted down by SH.  f = index of the field inside its half.
template <int BITS>
struct InPlace {
  static constexpr int HALF = 16 / BITS;
  static constexpr int SH = BITS == 2 ? 10 : 8;
  static constexpr int NDIRECT = BITS == 2 ? 5 : 2;
  static __host__ __device__ constexpr int pos(int f) { return f < NDIRECT ? f : f - NDIRECT; }
  static __host__ __device__ constexpr uint32_t mask(int f) {
    return (uint32_t)(((1u << BITS) - 1u) * 0x00010001u) << (BITS * pos(f));
  }
  // 2^24 / 2^(bit position): what brings the masked field back to its value
  static __host__ __device__ constexpr float undo(int f) { return (float)(1 << (24 - BITS * pos(f))); }
};

__device__ __forceinline__ half2_t as_half2(uint32_t w) { return __builtin_bit_cast(half2_t, w); }
__device__ __forceinline__ uint32_t as_u32(half2_t h) { return __builtin_bit_cast(uint32_t, h); }
__device__ __forceinline__ float pow2f(int e) { return __uint_as_float((uint32_t)(127 + e) << 23); }   // -126 <= e <= 127

// Power of two, as an fp16 pair, that brings the largest of the given fp16 magnitudes (bit patterns with
// the sign cleared, two per word; wave-wide) below 1, and its exponent: the scales of a tile are folded
// into the other operand of the products in that normalised form, so that the folded tables use the
// normal range of fp16 whatever the magnitude of the cache.
__device__ __forceinline__ int tile_shift(uint32_t magnitudes) {
  const uint32_t m = magnitudes & 0xffffu, n = magnitudes >> 16;
  const int top = (int)wave_max_o((float)(m > n ? m : n));       // (fp16 magnitudes order like integers)
  const int sh = 14 - (top >> 10);                                // value < 2^(biased exponent - 14)
  return sh < -14 ? -14 : sh;                                     // (at most 14: 2^sh is an fp16 number either way)
}
__device__ __forceinline__ half2_t pow2_half2(int e) {            // -14 <= e <= 15
  return as_half2((uint32_t)((15 + e) << 10) * 0x00010001u);
}

template <int BITS, int G, int NH4, bool ZK, bool ZV>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(NH4 == 1 ? 2 : 1, 2)))
attention_outer_kernel(AttnArgs a, int n_both, int n_splits, WindowSet win) {
  using Regs = OuterRegs<BITS, G>;
  using IP = InPlace<BITS>;
  constexpr int NH = NH4 * 4;
  constexpr int GPT = Regs::GPT, KC = Regs::KC, VC = Regs::VC, NG = Regs::NG;
  constexpr int FPW = 32 / BITS;
  constexpr int HALF = FPW / 2;                        // fields per 16-bit half of a word
  constexpr int WPG = G / FPW;                         // words per channel of one key group
  constexpr int ROWB = D * BITS / 8;
  constexpr int ROWW = ROWB / 4;                       // words of one packed value row
  constexpr int QROW = D + 8, AROW = 64 + 8;           // padded rows of the folded query tables (halves)
  constexpr float kLevel = (float)(1 << (BITS - 1));   // symmetric zero-point: -2^(b-1) |S|  (Eq. hybrid_dequant)
  // The fields enter the products as stored (0 .. 2^b - 1), so the rounding error of a folded table entry
  // would be multiplied by up to 2^b - 1.  Taking the middle of the field range out of the zero-point term
  // with the ROUNDED table entries,  S u + Zeff = S (u - kMid) + (Zeff + kMid S),  leaves each entry's
  // error multiplied by |u - kMid| <= kMid only, and the explicit constant small.
  constexpr float kMid = (float)((1 << BITS) - 1) * 0.5f;
  // LDS operands are asked for well ahead of their use where the registers allow it (four heads, 2-bit
  // codes: the measured configuration); the other instances read step by step
  constexpr bool kAhead = NH4 == 1 && BITS == 2;
  constexpr float kSlack = 6.0f;                       // scores may exceed the reference level by this (log2)

  const int lane = threadIdx.x;
  const long long bh = blockIdx.y;
  const int b = (int)(bh / a.n_kv_heads), hk = (int)(bh % a.n_kv_heads);
  const int r = a.n_q_heads / a.n_kv_heads;

  if ((int)blockIdx.x < win.n_chunks) {
    window_pass<NH4, BITS, G, false, true>(a, bh, win.na, win.b0, win.nb, (int)blockIdx.x, win.n_chunks, n_splits + (int)blockIdx.x);
    return;
  }
  const int n_tiles = (n_both + TILE - 1) / TILE;
  const int base_t = n_tiles / n_splits, rem_t = n_tiles % n_splits;
  const int s_idx = (int)blockIdx.x - win.n_chunks;
  const int t0 = s_idx * base_t + (s_idx < rem_t ? s_idx : rem_t);
  const int t1 = t0 + base_t + (s_idx < rem_t ? 1 : 0);

  // folded operand tables of the current tile (see the header): per key token-group the query times the
  // group's scales, and the lanes' pieces of the zero-point term; per value channel-group the softmax
  // weights times the tokens' scales ([NG]: the weights themselves), and the tokens' zero-points
  __shared__ __attribute__((aligned(16))) _Float16 qT[NH][QROW];        // q S of the current token group, rounded to fp16 ...
  __shared__ __attribute__((aligned(16))) _Float16 qL[NH][QROW];        // ... and what the rounding left (q S = qT + qL to 2^-22)
  __shared__ __attribute__((aligned(16))) _Float16 aT[NH][AROW];        // the lanes' pieces of the group's constant term
  // One region serves as the key tile of a 32-token sub-pass (fields masked in place, token-major) and,
  // once the score pass has read that, as the value pass's tables and packed rows (a workgroup is one
  // wavefront, whose LDS operations complete in order).  14 to 20 KB per workgroup with the window
  // pass's arrays: eight workgroups to a compute unit, two wavefronts to a SIMD.
  constexpr int SUB = 32;                              // tokens per key sub-pass
  // rows of 16 tokens in the weight tables, 20 halves apart: the 16 rows that one 64-bit read touches
  // (four token classes x four heads) then start in 16 different pairs of banks
  constexpr int PROW = 20;
  constexpr int kTablesHalves = (NG + 1) * 4 * NH * PROW + NG * 4 * PROW;
  constexpr int kKeyBytes = SUB * KROW * 2, kValueBytes = kTablesHalves * 2 + TILE * (ROWW + 1) * 4;
  __shared__ __attribute__((aligned(16))) unsigned char region[kKeyBytes > kValueBytes ? kKeyBytes : kValueBytes];
  _Float16 (*kt)[KROW] = reinterpret_cast<_Float16 (*)[KROW]>(region);
  _Float16 (*pT)[4 * NH * PROW] = reinterpret_cast<_Float16 (*)[4 * NH * PROW]>(region);       // [NG + 1][token % 4][head][token / 4]
  _Float16 (*zT)[4 * PROW] = reinterpret_cast<_Float16 (*)[4 * PROW]>(region + (NG + 1) * 4 * NH * PROW * 2);   // [NG][token % 4][token / 4]
  uint32_t (*vcode)[ROWW + 1] = reinterpret_cast<uint32_t (*)[ROWW + 1]>(region + kTablesHalves * 2);     // packed value rows (padded)

  // ---- query: this lane's two channels of every head, each head scaled by a power of two into [1/4, 1/2)
  half2_t qn[NH];
  int qe[NH];
#pragma unroll
  for (int h = 0; h < NH; ++h) {
    float q0 = 0.f, q1 = 0.f;
    if (h < r) {
      const uint32_t raw = *reinterpret_cast<const uint32_t*>(a.q + ((long long)b * a.n_q_heads + hk * r + h) * D + 2 * lane);
      q0 = half_lo(raw);
      q1 = half_hi(raw);
      if (a.q_scale) {
        q0 = __half2float(scaled_half(q0, a.q_scale[hk * D + 2 * lane]));
        q1 = __half2float(scaled_half(q1, a.q_scale[hk * D + 2 * lane + 1]));
      }
    }
    const float mx = wave_max_o(fmaxf(fabsf(q0), fabsf(q1)));
    const int e = mx > 0.f ? (int)((__float_as_uint(mx) >> 23) & 0xffu) - 127 + 2 : 0;
    qe[h] = e;
    const float f = pow2f(-e);
    qn[h] = half2_t{(_Float16)(q0 * f), (_Float16)(q1 * f)};
  }

  const long long kgroups = a.capacity / G;
  const uint8_t* kcodes = a.k.codes + bh * kgroups * D * (G * BITS / 8);
  const __half* kscales = a.k.scales + bh * kgroups * D;
  const __half* kzeros = ZK ? a.k.zeros + bh * kgroups * D : nullptr;
  const uint8_t* vcodes = a.v.codes + bh * a.capacity * ROWB;
  const __half* vscales = a.v.scales + bh * a.capacity * NG;
  const __half* vzeros = ZV ? a.v.zeros + bh * a.capacity * NG : nullptr;
  const int last_row = n_both - 1, last_group = n_both / G - 1;

  auto load_tile = [&](int tile, Regs& t) {
#pragma unroll
    for (int gi = 0; gi < GPT; ++gi) {
      int grp = tile * GPT + gi;
      grp = grp > last_group ? last_group : grp;
      const uint32_t ch = (uint32_t)grp * D + 2 * lane;
      const u32x4* kp = reinterpret_cast<const u32x4*>(kcodes + ch * (G * BITS / 8));
#pragma unroll
      for (int i = 0; i < KC; ++i) t.kc[gi][i] = __builtin_nontemporal_load(kp + i);
      t.ks[gi] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(kscales + ch));
      if constexpr (ZK) t.kz[gi] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(kzeros + ch));
    }
    int row = tile * TILE + lane;
    row = row > last_row ? last_row : row;
    const u32x4* vp = reinterpret_cast<const u32x4*>(vcodes + (uint32_t)row * ROWB);
#pragma unroll
    for (int i = 0; i < VC; ++i) t.vc[i] = __builtin_nontemporal_load(vp + i);
    if constexpr (NG == 4) {
      const u32x2 s = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(vscales + (uint32_t)row * NG));
      t.vs[0] = s.x; t.vs[1] = s.y;
      if constexpr (ZV) {
        const u32x2 z = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(vzeros + (uint32_t)row * NG));
        t.vz[0] = z.x; t.vz[1] = z.y;
      }
    } else {
      t.vs[0] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(vscales + (uint32_t)row * NG));
      if constexpr (ZV) t.vz[0] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(vzeros + (uint32_t)row * NG));
    }
  };

  const float c_log2 = 0.08838834764831845f * 1.4426950408889634f;
  // ---- running softmax state and accumulators.  m_run is a reference level that is raised (with a
  // wave-wide reduction and a rescale) only when a score exceeds it by more than kSlack.
  // oq[c][n]: channel c of this lane's eight, heads 4 n .. 4 n + 3, over the tokens 4 k + tg, in units of
  // the masked fields and of the running value shift; oz: the zero-point term of the lane's channel
  // group; ol: the sum of the weights.
  float m_run[NH];
  float4_t oq[8][NH4], oz[NH4], ol[NH4];
#pragma unroll
  for (int h = 0; h < NH; ++h) m_run[h] = -INFINITY;
#pragma unroll
  for (int n = 0; n < NH4; ++n) {
    oz[n] = float4_t{0.f, 0.f, 0.f, 0.f};
    ol[n] = oz[n];
#pragma unroll
    for (int c = 0; c < 8; ++c) oq[c][n] = oz[n];
  }
  int shv_run = 64;                                    // the values' scales enter as S * 2^shv_run (64: nothing yet)
  const int cg = lane & 15, tg = lane >> 4;
  const int gch = (8 * cg) / G;                        // value channel-group of this lane's channels (value pass)
  const int ptok = (lane % FPW) % HALF;                // where this lane's token sits in its half-word
  const float ftok = pow2f(24 - BITS * (ptok < IP::NDIRECT ? ptok : ptok - IP::NDIRECT));
  const uint32_t sel16 = (cg & 1) ? 0x07060302u : 0x05040100u;   // 2-bit: which half of a row word holds this lane's channels
  const u32x2 ones2 = {0x3C003C00u, 0x3C003C00u};
  const half4_t ones = __builtin_bit_cast(half4_t, ones2);
  const half4_t mids = {(_Float16)(-kMid), (_Float16)(-kMid), (_Float16)(-kMid), (_Float16)(-kMid)};

  auto process = [&](const Regs& cur, int tile) {
    __syncthreads();                                   // previous tile's readers of the LDS tiles are done

    // ---- keys.  K^[j][c] = S_{c,T} u[j][c] + Zeff_{c,T} (T = token group), so
    //   q . K^[j] = sum_c (q_c S_{c,T}) u[j][c]  +  sum_c q_c Zeff_{c,T}:
    // the scales go into a query table per token group (this lane owns channels 2 lane, 2 lane + 1),
    // the zero-point term is a constant per token group and head, summed over the lanes' pieces on the
    // matrix cores.  Everything is scaled by 2^shk so that the tables stay in fp16's normal range.
    // The 64 tokens of the tile go through in two sub-passes of 32 (half the LDS for the token-major
    // tile): in a sub-pass a lane takes one token and one half of the channels, and the two halves of a
    // token's sum meet across lanes 32 apart.
    uint32_t kmag = 0;
#pragma unroll
    for (int gi = 0; gi < GPT; ++gi) {
      kmag = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, kmag),
                                                                    __builtin_bit_cast(ushort2_t, cur.ks[gi] & 0x7fff7fffu)));
      if constexpr (ZK)
        kmag = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, kmag),
                                                                      __builtin_bit_cast(ushort2_t, cur.kz[gi] & 0x7fff7fffu)));
    }
    const int shk = tile_shift(kmag);
    const half2_t fk = pow2_half2(shk);
    // ---- values' scales: the shift that normalises this tile's, and the running one
    uint32_t vmag = 0;
#pragma unroll
    for (int gp = 0; gp < (NG + 1) / 2; ++gp) {
      vmag = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, vmag),
                                                                    __builtin_bit_cast(ushort2_t, cur.vs[gp] & 0x7fff7fffu)));
      if constexpr (ZV)
        vmag = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, vmag),
                                                                      __builtin_bit_cast(ushort2_t, cur.vz[gp] & 0x7fff7fffu)));
    }
    const int shv_tile = tile_shift(vmag);

    float s[NH];
    const int tl = lane & (SUB - 1), chh = lane / SUB;   // sub-pass: this lane's token and half of the channels
#pragma unroll
    for (int sp = 0; sp < TILE / SUB; ++sp) {
      const int gi = sp * SUB / G;                        // the sub-pass's token group (G = 64: one for both)
      if (sp > 0) __syncthreads();                        // the first sub-pass has read the tile and the tables
      if (G == SUB || sp == 0) {
        const half2_t sn = as_half2(cur.ks[gi] & 0x7fff7fffu) * fk;
        half2_t zn;
        if constexpr (ZK) {
          // the sign bit of a scale marks an asymmetric group, whose zero-point is stored; a symmetric
          // group stores +0 there and has Zeff = -2^(b-1) S
          const half2_t ssym = __builtin_elementwise_max(as_half2(cur.ks[gi]), half2_t{(_Float16)0, (_Float16)0}) * fk;
          zn = __builtin_elementwise_fma(as_half2(cur.kz[gi]), fk, ssym * half2_t{(_Float16)(-kLevel), (_Float16)(-kLevel)});
        } else {
          zn = sn * half2_t{(_Float16)(-kLevel), (_Float16)(-kLevel)};
        }
        const half2_t zc = __builtin_elementwise_fma(sn, half2_t{(_Float16)kMid, (_Float16)kMid}, zn);   // Zeff + kMid S
#pragma unroll
        for (int h = 0; h < NH; ++h) {
          // q S in two fp16 pieces: with one, the rounding of a large channel's entry (2^-12 of it, times
          // the field) shows in the output at 1e-3 on heavy-tailed keys
          const half2_t qs = qn[h] * sn;
          const float l0 = __builtin_fmaf((float)qn[h][0], (float)sn[0], -(float)qs[0]);
          const float l1 = __builtin_fmaf((float)qn[h][1], (float)sn[1], -(float)qs[1]);
          *reinterpret_cast<uint32_t*>(&qT[h][2 * lane]) = as_u32(qs);
          *reinterpret_cast<uint32_t*>(&qL[h][2 * lane]) = as_u32(half2_t{(_Float16)l0, (_Float16)l1});
          // this lane's piece of sum_c q_c (Zeff_c + kMid S_c)
          aT[h][lane] = (_Float16)__builtin_amdgcn_fdot2(qn[h], zc, 0.f, false);
        }
      }
      // the fields themselves, masked in place, into the token-major tile: a word holds 2 x HALF tokens of
      // one channel, so one AND handles tokens (p, HALF + p) of it
      constexpr int WPS = SUB / FPW;                      // words of one channel per sub-pass
#pragma unroll
      for (int ws = 0; ws < WPS; ++ws) {
        const int wd = (sp * SUB - gi * G) / FPW + ws;    // word inside the group's run
        const uint32_t w0 = cur.kc[gi][wd / 4][wd % 4], w1 = cur.kc[gi][(WPG + wd) / 4][(WPG + wd) % 4];
        const uint32_t w0s = w0 >> IP::SH, w1s = w1 >> IP::SH;
#pragma unroll
        for (int p = 0; p < HALF; ++p) {
          const uint32_t u0 = (p < IP::NDIRECT ? w0 : w0s) & IP::mask(p);   // channel 2 lane: tokens p, HALF + p
          const uint32_t u1 = (p < IP::NDIRECT ? w1 : w1s) & IP::mask(p);   // channel 2 lane + 1
          const int tok = ws * FPW + p;                   // token inside the sub-pass
          *reinterpret_cast<uint32_t*>(&kt[tok][2 * lane]) = __builtin_amdgcn_perm(u1, u0, 0x05040100u);          // low halves
          *reinterpret_cast<uint32_t*>(&kt[tok + HALF][2 * lane]) = __builtin_amdgcn_perm(u1, u0, 0x07060302u);   // high halves
        }
      }
      __syncthreads();

      // ---- scores of the sub-pass (Eq. att:1), 4x4x4 blocks: B = four consecutive channels of the lane's
      // row of fields, A = the same channels of four heads from the group's table.  Four independent
      // chains: fields times the table and times its remainder, and the same two tables times the constant
      // -kMid (the middle of the field range, taken with the rounded entries).
      float4_t su[NH4], sl[NH4], sm[NH4], sn2[NH4], sz[NH4];
#pragma unroll
      for (int n = 0; n < NH4; ++n) {
        su[n] = float4_t{0.f, 0.f, 0.f, 0.f};
        sl[n] = su[n]; sm[n] = su[n]; sn2[n] = su[n]; sz[n] = su[n];
      }
      // The operands come from LDS in stages of STG steps (8 channels each), a stage's reads issued before
      // the previous stage's matrix instructions: left to itself the compiler reads one or two steps ahead
      // and the wavefront waits out an LDS round trip every few instructions.
      constexpr int NSTEP = D / 2 / 8, NPIECE = 64 / 2 / 8;
      constexpr int STG = kAhead ? 2 : 1, NST = NSTEP / STG;
      u32x4 kvb[2][STG], qab[2][STG][NH4], qbb[2][STG][NH4], zab[NPIECE][NH4];
      auto read_stage = [&](int st, int buf) {
#pragma unroll
        for (int j = 0; j < STG; ++j) {
          const int c0 = (D / 2) * chh + 8 * (st * STG + j);
          kvb[buf][j] = *reinterpret_cast<const u32x4*>(&kt[tl][c0]);
#pragma unroll
          for (int n = 0; n < NH4; ++n) {
            qab[buf][j][n] = *reinterpret_cast<const u32x4*>(&qT[4 * n + (lane & 3)][c0]);
            qbb[buf][j][n] = *reinterpret_cast<const u32x4*>(&qL[4 * n + (lane & 3)][c0]);
          }
        }
      };
      read_stage(0, 0);
#pragma unroll
      for (int st = 0; st < NST; ++st) {
        if (st + 1 < NST) {
          read_stage(st + 1, (st + 1) & 1);
        } else {
#pragma unroll
          for (int i = 0; i < NPIECE; ++i)
#pragma unroll
            for (int n = 0; n < NH4; ++n) zab[i][n] = *reinterpret_cast<const u32x4*>(&aT[4 * n + (lane & 3)][32 * chh + 8 * i]);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < STG; ++j) {
          const u32x4 kv = kvb[st & 1][j];
          const half4_t k0 = __builtin_bit_cast(half4_t, u32x2{kv.x, kv.y}), k1 = __builtin_bit_cast(half4_t, u32x2{kv.z, kv.w});
#pragma unroll
          for (int n = 0; n < NH4; ++n) {
            const u32x4 qa = qab[st & 1][j][n], qb = qbb[st & 1][j][n];
            const half4_t a0 = __builtin_bit_cast(half4_t, u32x2{qa.x, qa.y}), a1 = __builtin_bit_cast(half4_t, u32x2{qa.z, qa.w});
            const half4_t b0 = __builtin_bit_cast(half4_t, u32x2{qb.x, qb.y}), b1 = __builtin_bit_cast(half4_t, u32x2{qb.z, qb.w});
            su[n] = __builtin_amdgcn_mfma_f32_4x4x4f16(a0, k0, su[n], 0, 0, 0);
            sl[n] = __builtin_amdgcn_mfma_f32_4x4x4f16(b0, k0, sl[n], 0, 0, 0);
            sm[n] = __builtin_amdgcn_mfma_f32_4x4x4f16(a0, mids, sm[n], 0, 0, 0);
            sn2[n] = __builtin_amdgcn_mfma_f32_4x4x4f16(b0, mids, sn2[n], 0, 0, 0);
            su[n] = __builtin_amdgcn_mfma_f32_4x4x4f16(a1, k1, su[n], 0, 0, 0);
            sl[n] = __builtin_amdgcn_mfma_f32_4x4x4f16(b1, k1, sl[n], 0, 0, 0);
            sm[n] = __builtin_amdgcn_mfma_f32_4x4x4f16(a1, mids, sm[n], 0, 0, 0);
            sn2[n] = __builtin_amdgcn_mfma_f32_4x4x4f16(b1, mids, sn2[n], 0, 0, 0);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int i = 0; i < NPIECE; ++i) {
#pragma unroll
        for (int n = 0; n < NH4; ++n) {
          const u32x4 za = zab[i][n];
          sz[n] = __builtin_amdgcn_mfma_f32_4x4x4f16(__builtin_bit_cast(half4_t, u32x2{za.x, za.y}), ones, sz[n], 0, 0, 0);
          sz[n] = __builtin_amdgcn_mfma_f32_4x4x4f16(__builtin_bit_cast(half4_t, u32x2{za.z, za.w}), ones, sz[n], 0, 0, 0);
        }
      }
#pragma unroll
      for (int h = 0; h < NH; ++h) {
        float part = __builtin_fmaf(su[h / 4][h % 4] + sl[h / 4][h % 4], ftok, (sm[h / 4][h % 4] + sn2[h / 4][h % 4]) + sz[h / 4][h % 4]);
        part += __shfl_xor(part, SUB);                    // the other half of the channels
        part *= c_log2 * pow2f(qe[h] - shk);
        s[h] = (sp == 0 || chh == sp) ? part : s[h];      // lane = token from here on: 32 sp + (lane % 32)
      }
    }
    __syncthreads();                                      // the score pass has left the tile

    // ---- stage this lane's packed value row (in the key tile's memory, which the score pass has left),
    // and ask for the rows the value pass will want: used after the softmax
#pragma unroll
    for (int i = 0; i < VC; ++i) {
      vcode[lane][4 * i + 0] = cur.vc[i].x;
      vcode[lane][4 * i + 1] = cur.vc[i].y;
      vcode[lane][4 * i + 2] = cur.vc[i].z;
      vcode[lane][4 * i + 3] = cur.vc[i].w;
    }
    __syncthreads();
    uint32_t vrow[4][4];
    if constexpr (kAhead) {
#pragma unroll
      for (int kq = 0; kq < 4; ++kq)
#pragma unroll
        for (int i = 0; i < 4; ++i) vrow[kq][i] = vcode[16 * kq + 4 * i + tg][BITS == 2 ? cg / 2 : cg];
    }
    // ---- running softmax (Eq. att:2); the weights are rounded to fp16 for the matrix cores and the
    // normaliser is the matrix cores' sum of the rounded weights
    const bool valid = tile * TILE + lane <= last_row;
    bool raise = false;
#pragma unroll
    for (int h = 0; h < NH; ++h) {
      s[h] = valid ? s[h] : -INFINITY;
      raise |= s[h] > m_run[h] + kSlack;
    }
    const int shv_new = shv_tile < shv_run ? shv_tile : shv_run;
    if (__builtin_amdgcn_ballot_w64(raise) != 0 || shv_new != shv_run) {
      const float fshift = shv_run == 64 ? 0.f : pow2f(shv_new - shv_run);   // (nothing accumulated yet: any factor)
#pragma unroll
      for (int h = 0; h < NH; ++h) {
        const float m_new = fmaxf(m_run[h], wave_max_o(s[h]));
        const float alpha = __builtin_amdgcn_exp2f(m_run[h] - m_new);        // 0 the first time
        m_run[h] = m_new;
        ol[h / 4][h % 4] *= alpha;
        oz[h / 4][h % 4] *= alpha * fshift;
#pragma unroll
        for (int c = 0; c < 8; ++c) oq[c][h / 4][h % 4] *= alpha * fshift;
      }
      shv_run = shv_new;
    }
    {
      // sum_j p_j V^[j][c] = sum_j (p_j S_{j,g}) u[j][c] + sum_j p_j Zeff_{j,g}  (g = channel group of c):
      // weight tables per channel group, and the tokens' zero-points as one more operand
      const half2_t fv = pow2_half2(shv_run);
      half2_t vsn[(NG + 1) / 2], vzn[(NG + 1) / 2];
#pragma unroll
      for (int gp = 0; gp < (NG + 1) / 2; ++gp) {
        vsn[gp] = as_half2(cur.vs[gp] & 0x7fff7fffu) * fv;
        if constexpr (ZV) {
          const half2_t ssym = __builtin_elementwise_max(as_half2(cur.vs[gp]), half2_t{(_Float16)0, (_Float16)0}) * fv;
          vzn[gp] = __builtin_elementwise_fma(as_half2(cur.vz[gp]), fv, ssym * half2_t{(_Float16)(-kLevel), (_Float16)(-kLevel)});
        } else {
          vzn[gp] = vsn[gp] * half2_t{(_Float16)(-kLevel), (_Float16)(-kLevel)};
        }
      }
      const int slot = (lane & 3) * PROW + (lane >> 2);
#pragma unroll
      for (int gp = 0; gp < (NG + 1) / 2; ++gp)        // Zeff + kMid S (see kMid)
        vzn[gp] = __builtin_elementwise_fma(vsn[gp], half2_t{(_Float16)kMid, (_Float16)kMid}, vzn[gp]);
#pragma unroll
      for (int g = 0; g < NG; ++g) zT[g][slot] = vzn[g / 2][g & 1];
#pragma unroll
      for (int h = 0; h < NH; ++h) {
        const _Float16 p16 = (_Float16)__builtin_amdgcn_exp2f(s[h] - m_run[h]);
        const int idx = ((lane & 3) * NH + h) * PROW + (lane >> 2);
        pT[NG][idx] = p16;
#pragma unroll
        for (int g = 0; g < NG; ++g) pT[g][idx] = p16 * vsn[g / 2][g & 1];
      }
    }
    __syncthreads();
    // ---- values (Eq. att:3): lane = 8 channels (8 cg ..) of the tokens 4 k + tg.  Two rows' chunks side
    // by side in the two halves of a register: one AND then leaves one channel of two tokens, half of a
    // B operand (one channel of four tokens)
    half4_t aops[4][NH4], aopls[4][NH4], zops[4];
    auto read_weights = [&](int kq) {
#pragma unroll
      for (int n = 0; n < NH4; ++n) {
        aops[kq][n] = *reinterpret_cast<const half4_t*>(&pT[gch][(tg * NH + 4 * n + (lane & 3)) * PROW + 4 * kq]);
        aopls[kq][n] = *reinterpret_cast<const half4_t*>(&pT[NG][(tg * NH + 4 * n + (lane & 3)) * PROW + 4 * kq]);
      }
      zops[kq] = *reinterpret_cast<const half4_t*>(&zT[gch][tg * PROW + 4 * kq]);
    };
    if constexpr (kAhead) {
#pragma unroll
      for (int kq = 0; kq < 4; ++kq) read_weights(kq);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int kq = 0; kq < 4; ++kq) {
      if constexpr (!kAhead) {
        read_weights(kq);
#pragma unroll
        for (int i = 0; i < 4; ++i) vrow[kq][i] = vcode[16 * kq + 4 * i + tg][BITS == 2 ? cg / 2 : cg];
      }
      const half4_t* aop = aops[kq];
      const half4_t* aopl = aopls[kq];
      const half4_t zop = zops[kq];
      uint32_t src[2][8 / IP::HALF][2];                  // [direct | shifted][16-bit chunk][rows 0,1 | rows 2,3]
      const uint32_t x0 = vrow[kq][0], x1 = vrow[kq][1], x2 = vrow[kq][2], x3 = vrow[kq][3];   // rows 16 kq + tg + 0, 4, 8, 12
      if constexpr (BITS == 2) {
        src[0][0][0] = __builtin_amdgcn_perm(x1, x0, sel16);
        src[0][0][1] = __builtin_amdgcn_perm(x3, x2, sel16);
      } else {
        src[0][0][0] = __builtin_amdgcn_perm(x1, x0, 0x05040100u);   // channels 0..3 of rows 0, 1
        src[0][0][1] = __builtin_amdgcn_perm(x3, x2, 0x05040100u);
        src[0][1][0] = __builtin_amdgcn_perm(x1, x0, 0x07060302u);   // channels 4..7
        src[0][1][1] = __builtin_amdgcn_perm(x3, x2, 0x07060302u);
      }
#pragma unroll
      for (int ck = 0; ck < 8 / IP::HALF; ++ck)
#pragma unroll
        for (int pr = 0; pr < 2; ++pr) src[1][ck][pr] = src[0][ck][pr] >> IP::SH;
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const int ck = c / IP::HALF, f = c % IP::HALF;
        const int sh = f < IP::NDIRECT ? 0 : 1;
        const u32x2 bw = {src[sh][ck][0] & IP::mask(f), src[sh][ck][1] & IP::mask(f)};
        const half4_t bop = __builtin_bit_cast(half4_t, bw);
#pragma unroll
        for (int n = 0; n < NH4; ++n) oq[c][n] = __builtin_amdgcn_mfma_f32_4x4x4f16(aop[n], bop, oq[c][n], 0, 0, 0);
      }
#pragma unroll
      for (int n = 0; n < NH4; ++n) {
        oz[n] = __builtin_amdgcn_mfma_f32_4x4x4f16(aopl[n], zop, oz[n], 0, 0, 0);
        oz[n] = __builtin_amdgcn_mfma_f32_4x4x4f16(aop[n], mids, oz[n], 0, 0, 0);       // - kMid * (weights times scales, as rounded)
        ol[n] = __builtin_amdgcn_mfma_f32_4x4x4f16(aopl[n], ones, ol[n], 0, 0, 0);
      }
    }
  };

  // two register buffers in turn: the next tile's loads are in flight while this one is computed
  {
    Regs bufA, bufB;
    if (t0 < t1) load_tile(t0, bufA);
    int tile = t0;
    while (tile + 1 < t1) {
      load_tile(tile + 1, bufB);
      process(bufA, tile);
      if (tile + 2 < t1) load_tile(tile + 2, bufA);
      process(bufB, tile + 1);
      tile += 2;
    }
    if (tile < t1) process(bufA, tile);
  }

  // ---- partial result: undo the field positions and the value shift, add the zero-point term, and sum
  // over the four token classes (lanes 16 apart)
  const float fv_undo = shv_run == 64 ? 0.f : pow2f(-shv_run);
  float o[NH][8], l_run[NH];
#pragma unroll
  for (int h = 0; h < NH; ++h) {
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      o[h][c] = __builtin_fmaf(oq[c][h / 4][h % 4], IP::undo(c % IP::HALF), oz[h / 4][h % 4]) * fv_undo;
      o[h][c] += __shfl_xor(o[h][c], 16);
      o[h][c] += __shfl_xor(o[h][c], 32);
    }
    l_run[h] = ol[h / 4][h % 4];
    l_run[h] += __shfl_xor(l_run[h], 16);
    l_run[h] += __shfl_xor(l_run[h], 32);
  }
  const int slot = s_idx;
#pragma unroll
  for (int h = 0; h < NH; ++h) {
    if (h < r) {
      const long long bhq = (long long)b * a.n_q_heads + hk * r + h;
      if (lane < 16) {
        float* dst = &a.ws_o[(bhq * a.n_partials + slot) * D + 8 * lane];
        *reinterpret_cast<float4_t*>(dst) = float4_t{o[h][0], o[h][1], o[h][2], o[h][3]};
        *reinterpret_cast<float4_t*>(dst + 4) = float4_t{o[h][4], o[h][5], o[h][6], o[h][7]};
      }
      if (lane == 0) {
        a.ws_ml[(bhq * a.n_partials + slot) * 2 + 0] = m_run[h] * 0.6931471805599453f;
        a.ws_ml[(bhq * a.n_partials + slot) * 2 + 1] = l_run[h];
      }
    }
  }
}

template <int BITS, int G, bool ZK, bool ZV>
hipError_t launch_z(const AttnArgs& a, int n_both, int n_splits, const WindowSet& win, const Launch& L) {
  const int r = a.n_q_heads / a.n_kv_heads;
  dim3 grid((unsigned)(n_splits + win.n_chunks), (unsigned)(a.batch * a.n_kv_heads));
  if (r <= 4)
    hipExtLaunchKernelGGL((attention_outer_kernel<BITS, G, 1, ZK, ZV>), grid, dim3(64), 0, L.stream, L.ev_start,
                          L.ev_stop, 0, a, n_both, n_splits, win);
  else
    hipExtLaunchKernelGGL((attention_outer_kernel<BITS, G, 2, ZK, ZV>), grid, dim3(64), 0, L.stream, L.ev_start,
                          L.ev_stop, 0, a, n_both, n_splits, win);
  return hipGetLastError();
}

template <int BITS, int G>
hipError_t launch_t(const AttnArgs& a, int n_both, int n_splits, const WindowSet& win, const Launch& L) {
  const bool zk = a.k.zeros != nullptr, zv = a.v.zeros != nullptr;
  if (zk && zv) return launch_z<BITS, G, true, true>(a, n_both, n_splits, win, L);
  if (zk) return launch_z<BITS, G, true, false>(a, n_both, n_splits, win, L);
  if (zv) return launch_z<BITS, G, false, true>(a, n_both, n_splits, win, L);
  return launch_z<BITS, G, false, false>(a, n_both, n_splits, win, L);
}

}  // namespace

bool attention_outer_supported(const AttnArgs& a) {
  const int r = a.n_q_heads / a.n_kv_heads;
  return a.k.form == kPerChannel && a.v.form == kPerToken && (a.bits == 2 || a.bits == 4) && a.v_bits == a.bits && r <= 8 &&
         a.capacity * D <= (1LL << 31) && !a.pages.table;
}

namespace {
// Resident workgroups per compute unit of one instance: the runtime's answer, bounded by the LDS the
// instance declares rounded up to the allocation granule (the runtime's answer was one too many for a
// workgroup of 27 264 bytes: six counted, five resident, and the launch ran in two rounds).
template <int BITS, int G, int NH4>
int resident_outer() {
  const auto kernel = attention_outer_kernel<BITS, G, NH4, true, true>;
  int n = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, 64, 0) != hipSuccess || n <= 0) return 4;
  hipFuncAttributes fa;
  if (hipFuncGetAttributes(&fa, reinterpret_cast<const void*>(kernel)) == hipSuccess && fa.sharedSizeBytes > 0) {
    const size_t granule = 1024, lds_per_cu = 160 * 1024;
    const int by_lds = (int)(lds_per_cu / (((fa.sharedSizeBytes + granule - 1) / granule) * granule));
    if (by_lds >= 1 && by_lds < n) n = by_lds;
  }
  return n;
}
}  // namespace

int attention_outer_waves_per_cu(const AttnArgs& a) {
  // 64-thread groups, 22 to 33 KB of LDS each: the LDS budget of a compute unit decides; the instances
  // for more than four heads per kv head also run one wavefront to a SIMD (registers)
  static CachedInt c[2][2][2];
  const int r = a.n_q_heads / a.n_kv_heads;
  const bool b4 = a.bits == 4, g64 = a.group == 64, wide = r > 4;
  return c[b4][g64][wide].get([&] {
    if (b4) {
      if (g64) return wide ? resident_outer<4, 64, 2>() : resident_outer<4, 64, 1>();
      return wide ? resident_outer<4, 32, 2>() : resident_outer<4, 32, 1>();
    }
    if (g64) return wide ? resident_outer<2, 64, 2>() : resident_outer<2, 64, 1>();
    return wide ? resident_outer<2, 32, 2>() : resident_outer<2, 32, 1>();
  });
}

hipError_t launch_attention_outer(const AttnArgs& a, long long n_both_ll, int n_splits, const WindowSet& win,
                                  hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop) {
  const int n_both = (int)n_both_ll;
  const Launch L = {stream, ev_start, ev_stop};
  if (a.bits == 2 && a.group == 32) return launch_t<2, 32>(a, n_both, n_splits, win, L);
  if (a.bits == 2 && a.group == 64) return launch_t<2, 64>(a, n_both, n_splits, win, L);
  if (a.bits == 4 && a.group == 32) return launch_t<4, 32>(a, n_both, n_splits, win, L);
  if (a.bits == 4 && a.group == 64) return launch_t<4, 64>(a, n_both, n_splits, win, L);
  return hipErrorInvalidValue;
}

}  // namespace innerq
