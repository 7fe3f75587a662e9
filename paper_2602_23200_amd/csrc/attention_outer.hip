// Comparison kernel: fused split-K decode attention over an OUTER-dimension-grouped cache
// (kind = INNERQ_KIND_OUTER: keys grouped along tokens per channel, values along channels per
// token -- the layout the paper compares against, Figure "inner_outer" (a)).
//
// Same skeleton as the inner-grouped and fp16 kernels (one wavefront per token range, 64-token
// tiles, register prefetch of the next tile, window wavefronts in the same launch, same merge), and
// the multiply-accumulates run on the same 4x4x4 fp16 matrix instructions.  What differs is forced
// by the grouping.  The packing runs across the inner dimension instead of along it (a key word
// holds 16 tokens of ONE channel, a value word 16 channels of ONE token), while every operand layout
// of the matrix instructions gives a lane consecutive indices of the inner dimension: the fields of
// one inner sum never sit in one lane, so every element has to be taken out of its word and moved --
// the keys through an LDS tile to reach the one-token-per-lane score pass, the value rows through an
// LDS staging area to reach the channel-per-lane value pass -- at one vector instruction or more per
// element.  The inner-grouped kernel masks two fields in place per instruction and moves nothing.
// The scales themselves could be kept out of the element loop here too (a group's scale depends on
// the summed index, so it can be folded into the OTHER operand once per group: a query table
// q_c * S_{c,T} per token group, weight tables p_j * S_{j,g} per channel group, the zero-points as one
// constant per group); that would replace the subtract and the multiply-add below (two of the four to
// five instructions per pair of elements) by table set-up per tile, and leave the extraction and the
// move.  Not built: the elements are dequantised (Eq. asym_dequant) to fp16 on their way.
// Dequantisation costs two vector instructions per element: a field moved to mantissa bits 8..9 (6..9
// for 4-bit codes) of an fp16 number with a fixed exponent reads as bias + u (bias 4, resp. 16), two
// fields per 32-bit instruction; a packed subtract takes the bias off (exactly) and one packed fp16
// fused multiply-add forms S * u + Zeff for both, rounded once: the correctly rounded fp16 value of
// the dequantised element.  (Folding the bias into the constant, S * (bias + u) + (Zeff - bias * S),
// saves the subtract but rounds a constant several times larger than the element: 1e-2 on the
// output with heavy-tailed keys, measured.)
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
constexpr int KROW = D + 8;                 // padded LDS row of the dequantised key tile (halves)

// wave-wide reductions: the DPP forms shared with the window pass
__device__ inline float wave_max_o(float x) { return window_wave_max(x); }
__device__ inline float wave_sum_o(float x) { return window_wave_sum(x); }
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

// Two b-bit fields (one in each 16-bit half of w, at bit `at` of its half) as the fp16 pair (u, u'):
// the field lands on the top mantissa bits under a fixed exponent, which reads as bias + u.
template <int BITS>
__device__ __forceinline__ half2_t fields_as_half2(uint32_t w, int at) {
  constexpr int TOP = 10 - BITS;                           // first mantissa bit the field occupies
  constexpr uint32_t MASK = (((1u << BITS) - 1u) << TOP) * 0x00010001u;
  constexpr uint32_t EXPO = (BITS == 2 ? 0x4400u : 0x4C00u) * 0x00010001u;    // 4.0 resp. 16.0
  constexpr _Float16 BIAS = BITS == 2 ? (_Float16)4.0f : (_Float16)16.0f;
  const uint32_t moved = at < TOP ? w << (TOP - at) : w >> (at - TOP);
  return __builtin_bit_cast(half2_t, (moved & MASK) | EXPO) - half2_t{BIAS, BIAS};
}

// (|S|, Zeff) of one group as an fp16 pair; Zeff = Z for an asymmetric group (scale sign bit set),
// -2^(b-1) |S| for a symmetric one (Eq. hybrid_dequant).
template <int BITS, bool HASZ>
__device__ __forceinline__ half2_t scale_and_offset(float sc, float zp) {
  const float S = fabsf(sc);
  float z = -S * (float)(1 << (BITS - 1));
  if constexpr (HASZ) z = (__float_as_uint(sc) >> 31) ? zp : z;
  half2_t r;
  r[0] = (_Float16)S;
  r[1] = (_Float16)z;
  return r;
}

template <int BITS, int G, int NH4, bool ZK, bool ZV>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2, 2)))
attention_outer_kernel(AttnArgs a, int n_both, int n_splits, WindowSet win) {
  using Regs = OuterRegs<BITS, G>;
  constexpr int NH = NH4 * 4;
  constexpr int GPT = Regs::GPT, KC = Regs::KC, VC = Regs::VC, NG = Regs::NG;
  constexpr int FPW = 32 / BITS;
  constexpr int HALF = FPW / 2;                        // fields per 16-bit half of a word
  constexpr int WPG = G / FPW;                         // words per channel of one key group
  constexpr int ROWB = D * BITS / 8;
  constexpr int ROWW = ROWB / 4;                       // words of one packed value row

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

  __shared__ __attribute__((aligned(16))) _Float16 qs[NH][D];           // query, fp16 (exact)
  __shared__ __attribute__((aligned(16))) _Float16 kt[TILE][KROW];      // dequantised keys, token-major
  // probabilities of the tile, rounded to fp16, as matrix operands: [token % 4][head][token / 4]
  __shared__ __attribute__((aligned(16))) _Float16 wp16[4 * NH * 16];
  __shared__ __attribute__((aligned(16))) uint32_t vcode[TILE][ROWW + 1];   // packed value rows (padded)
  __shared__ __attribute__((aligned(16))) half2_t vsz[TILE][NG];        // (|S|, Zeff) of each value group

  for (int i = lane; i < NH * D; i += 64) {
    const int h = i / D, c = i % D;
    float qv = 0.f;
    if (h < r) {
      const __half qh = a.q[((long long)b * a.n_q_heads + hk * r + h) * D + c];
      qv = a.q_scale ? __half2float(scaled_half(__half2float(qh), a.q_scale[hk * D + c])) : __half2float(qh);
    }
    qs[h][c] = (_Float16)qv;
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
  // oq[e][n]: channel 8 cg + e of this lane, heads 4 n .. 4 n + 3, the tokens 4 k + tg of every tile
  float m_run[NH], l_run[NH];
  float4_t oq[8][NH4];
#pragma unroll
  for (int h = 0; h < NH; ++h) {
    m_run[h] = -INFINITY;
    l_run[h] = 0.f;
  }
#pragma unroll
  for (int e = 0; e < 8; ++e)
#pragma unroll
    for (int n = 0; n < NH4; ++n) oq[e][n] = float4_t{0.f, 0.f, 0.f, 0.f};
  const int cg = lane & 15, tg = lane >> 4;

  Regs cur, nxt;
  if (t0 < t1) load_tile(t0, cur);
  for (int tile = t0; tile < t1; ++tile) {
    if (tile + 1 < t1) load_tile(tile + 1, nxt);       // in flight while this tile is computed
    __syncthreads();                                   // previous tile's readers of the LDS tiles are done

    // ---- dequantise this lane's two key channels of all 64 tokens into the token-major tile: a word
    // holds 2 x HALF tokens of one channel, so one instruction handles tokens (p, HALF + p) of it
#pragma unroll
    for (int gi = 0; gi < GPT; ++gi) {
      const uint32_t sp = cur.ks[gi], zp = ZK ? cur.kz[gi] : 0u;
      const half2_t sz0 = scale_and_offset<BITS, ZK>(half_lo(sp), half_lo(zp));
      const half2_t sz1 = scale_and_offset<BITS, ZK>(half_hi(sp), half_hi(zp));
      const half2_t S0 = {sz0[0], sz0[0]}, Z0 = {sz0[1], sz0[1]}, S1 = {sz1[0], sz1[0]}, Z1 = {sz1[1], sz1[1]};
#pragma unroll
      for (int wd = 0; wd < WPG; ++wd) {
        const uint32_t w0 = cur.kc[gi][wd / 4][wd % 4], w1 = cur.kc[gi][(WPG + wd) / 4][(WPG + wd) % 4];
#pragma unroll
        for (int p = 0; p < HALF; ++p) {
          const half2_t x0 = __builtin_elementwise_fma(fields_as_half2<BITS>(w0, p * BITS), S0, Z0);   // channel 2 lane: tokens p, HALF + p
          const half2_t x1 = __builtin_elementwise_fma(fields_as_half2<BITS>(w1, p * BITS), S1, Z1);   // channel 2 lane + 1
          const uint32_t u0 = __builtin_bit_cast(uint32_t, x0), u1 = __builtin_bit_cast(uint32_t, x1);
          const int tok = gi * G + wd * FPW + p;
          *reinterpret_cast<uint32_t*>(&kt[tok][2 * lane]) = __builtin_amdgcn_perm(u1, u0, 0x05040100u);          // low halves
          *reinterpret_cast<uint32_t*>(&kt[tok + HALF][2 * lane]) = __builtin_amdgcn_perm(u1, u0, 0x07060302u);   // high halves
        }
      }
    }
    // ---- stage this lane's packed value row and its group constants
#pragma unroll
    for (int i = 0; i < VC; ++i) {
      vcode[lane][4 * i + 0] = cur.vc[i].x;
      vcode[lane][4 * i + 1] = cur.vc[i].y;
      vcode[lane][4 * i + 2] = cur.vc[i].z;
      vcode[lane][4 * i + 3] = cur.vc[i].w;
    }
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const uint32_t sp = cur.vs[g / 2], zp = ZV ? cur.vz[g / 2] : 0u;
      vsz[lane][g] = scale_and_offset<BITS, ZV>((g & 1) ? half_hi(sp) : half_lo(sp), (g & 1) ? half_hi(zp) : half_lo(zp));
    }
    __syncthreads();

    // ---- scores: lane = token (Eq. att:1), 4x4x4 blocks: B = four consecutive channels of the lane's
    // dequantised row, A = the same channels of four heads
    float s[NH];
    {
      float4_t sacc[NH4];
#pragma unroll
      for (int n = 0; n < NH4; ++n) sacc[n] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < D / 8; ++i) {
        const u32x4 kv = *reinterpret_cast<const u32x4*>(&kt[lane][i * 8]);
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
          u32x2 bw;
          bw.x = hf ? kv.z : kv.x;
          bw.y = hf ? kv.w : kv.y;
          const half4_t bop = __builtin_bit_cast(half4_t, bw);
#pragma unroll
          for (int n = 0; n < NH4; ++n) {
            const half4_t aop = *reinterpret_cast<const half4_t*>(&qs[4 * n + (lane & 3)][8 * i + 4 * hf]);
            sacc[n] = __builtin_amdgcn_mfma_f32_4x4x4f16(aop, bop, sacc[n], 0, 0, 0);
          }
        }
      }
#pragma unroll
      for (int n = 0; n < NH4; ++n) {
        s[4 * n] = sacc[n].x; s[4 * n + 1] = sacc[n].y; s[4 * n + 2] = sacc[n].z; s[4 * n + 3] = sacc[n].w;
      }
    }
    // ---- running softmax (Eq. att:2); the weights are rounded to fp16 for the matrix cores and the
    // normaliser is formed from the rounded weights
    const bool valid = tile * TILE + lane <= last_row;
#pragma unroll
    for (int h = 0; h < NH; ++h) {
      const float sv = valid ? s[h] * c_log2 : -INFINITY;
      const float m_new = fmaxf(m_run[h], wave_max_o(sv));
      const float alpha = __builtin_amdgcn_exp2f(m_run[h] - m_new);
      const _Float16 p16 = (_Float16)__builtin_amdgcn_exp2f(sv - m_new);
      wp16[((lane & 3) * NH + h) * 16 + (lane >> 2)] = p16;
      l_run[h] = l_run[h] * alpha + wave_sum_o((float)p16);
      m_run[h] = m_new;
#pragma unroll
      for (int e = 0; e < 8; ++e) oq[e][h / 4][h % 4] *= alpha;
    }
    __syncthreads();
    // ---- values (Eq. att:3): lane = 8 channels (8 cg ..) of the tokens 4 k + tg; every row chunk is
    // dequantised to four fp16 pairs, then four rows give the B operands (one channel of four tokens)
#pragma unroll
    for (int kq = 0; kq < 4; ++kq) {
      half4_t aop[NH4];
#pragma unroll
      for (int n = 0; n < NH4; ++n)
        aop[n] = *reinterpret_cast<const half4_t*>(&wp16[(tg * NH + 4 * n + (lane & 3)) * 16 + 4 * kq]);
      uint32_t x[4][4];                                  // [row][pair]: dequantised fp16 pairs
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int j = 4 * (4 * kq + i) + tg;
        const half2_t sz = vsz[j][(8 * cg) / G];
        const half2_t S = {sz[0], sz[0]}, Z = {sz[1], sz[1]};
        if constexpr (BITS == 2) {
          // 8 fields in 16 bits: low half = the chunk, high half = the chunk >> 2, so that pair e holds
          // fields 2 e (low half) and 2 e + 1 (high half) at bit 4 e of their halves
          const uint32_t c16 = (vcode[j][cg / 2] >> ((cg & 1) * 16)) & 0xffffu;
          const uint32_t w = (c16 << 14) | c16;
#pragma unroll
          for (int e = 0; e < 4; ++e)
            x[i][e] = __builtin_bit_cast(uint32_t, __builtin_elementwise_fma(fields_as_half2<2>(w, 4 * e), S, Z));
        } else {
          // 8 fields in 32 bits: pair e holds fields e (low half) and e + 4 (high half) at bit 4 e
          const uint32_t w = vcode[j][cg];
#pragma unroll
          for (int e = 0; e < 4; ++e)
            x[i][e] = __builtin_bit_cast(uint32_t, __builtin_elementwise_fma(fields_as_half2<4>(w, 4 * e), S, Z));
        }
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        u32x2 lo, hi;
        lo.x = __builtin_amdgcn_perm(x[1][e], x[0][e], 0x05040100u);   // low halves of rows 0, 1
        lo.y = __builtin_amdgcn_perm(x[3][e], x[2][e], 0x05040100u);
        hi.x = __builtin_amdgcn_perm(x[1][e], x[0][e], 0x07060302u);   // high halves
        hi.y = __builtin_amdgcn_perm(x[3][e], x[2][e], 0x07060302u);
        const half4_t blo = __builtin_bit_cast(half4_t, lo), bhi = __builtin_bit_cast(half4_t, hi);
        // channel of the low / high half of pair e (see the two packings above)
        constexpr int STEP = BITS == 2 ? 1 : 4;
        const int c_lo = BITS == 2 ? 2 * e : e, c_hi = c_lo + STEP;
#pragma unroll
        for (int n = 0; n < NH4; ++n) {
          oq[c_lo][n] = __builtin_amdgcn_mfma_f32_4x4x4f16(aop[n], blo, oq[c_lo][n], 0, 0, 0);
          oq[c_hi][n] = __builtin_amdgcn_mfma_f32_4x4x4f16(aop[n], bhi, oq[c_hi][n], 0, 0, 0);
        }
      }
    }
    cur = nxt;
  }

  float o[NH][8];
#pragma unroll
  for (int h = 0; h < NH; ++h)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      o[h][e] = oq[e][h / 4][h % 4];
      o[h][e] += __shfl_xor(o[h][e], 16);
      o[h][e] += __shfl_xor(o[h][e], 32);
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

int attention_outer_waves_per_cu(const AttnArgs& a) {
  // 64-thread groups, about 26 KB of LDS each: the LDS budget of a compute unit decides
  (void)a;
  static CachedInt c;
  return c.get([] {
    int n = 0;
    const hipError_t e =
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, attention_outer_kernel<2, 32, 1, true, true>, 64, 0);
    return (e == hipSuccess && n > 0) ? n : 4;
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
