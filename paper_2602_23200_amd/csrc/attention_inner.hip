// Fused dequantise + score + softmax + value kernel for the inner-grouped cache
// (keys per-token group-wise, values per-channel group-wise; Section "InnerQ").
//
// One wavefront streams a contiguous range of quantised tokens once and serves
// every query head that shares the kv head from those bytes.
//
// Why the grouping matters here (Section "InnerQ", Figure "inner_outer"): with
// groups along the inner dimension of each product, a group's scale and
// zero-point factor out of the inner sum,
//     q . k_j      = sum_g |S_jg| * (sum_{c in g} q_c u_jc) + Zeff_jg * (sum_{c in g} q_c)
//     sum_j p_j v_jc = sum_T |S_Tc| * (sum_{j in T} p_j u_jc) + Zeff_Tc * (sum_{j in T} p_j)
// (u = stored field, Zeff = Z for an asymmetric group and -|S| 2^(b-1) for a
// symmetric one: Eq. hybrid_dequant), so the inner sums run on the raw integer
// fields and one multiply per group applies the scale.
//
// Mapping to CDNA4:
//   * inner sums run on the matrix cores with v_mfma_f32_4x4x4_16B_f16: 16
//     independent 4x4x4 blocks per instruction, A = 4 query heads x 4 inner
//     indices (shared by all blocks), B = 4 inner indices x 4 lanes.  In the score
//     pass a lane owns one token, in the value pass two channels, and the result
//     lands in the lane that holds that token's / channel's scale: no cross-lane
//     traffic.
//   * a b-bit field becomes an fp16 operand with ONE and per two fields: masked in
//     place inside a 16-bit half it is the fp16 denormal u * 2^(b*pos) * 2^-24
//     (the matrix cores keep fp16 denormals); the position factor is folded into
//     the A operand (query / probabilities), the constant into the group scale.
//   * 3-bit fields are stored as a plane of 2-bit low parts followed by a plane of
//     high bits; the high bits are 1-bit fields of the same kind (2^(pos - 24)) and
//     join the same MFMA chains through operand tables that carry their weight 4.
//     Keys and values may have different widths (template parameters KB, VB).
//   * softmax probabilities are rounded to fp16 for the value pass and the
//     normaliser is the MFMA sum of those same rounded values (an extra all-ones B
//     operand), so the weights stay consistent.
//   * schedule: n_splits + n_window_chunks wavefronts per (batch, kv-head), all
//     resident at once at two per SIMD; contiguous tile ranges; two register
//     buffers in ping-pong; the wavefront that is behind its SIMD partner gets the
//     higher issue priority, so both finish together.
//   * paged store: this file is compiled twice.  attention_inner_paged.hip includes it with
//     INNERQ_PAGED_STORE set and gets the kernels that look every tile up in the page table (a page is
//     one 64-token tile); the build for the contiguous store carries no trace of that.
#include "innerq_dev.h"
#include "window_pass.h"

#ifndef INNERQ_PAGED_STORE
#define INNERQ_PAGED_STORE 0
#endif

namespace innerq {
namespace {

constexpr bool kPagedStore = INNERQ_PAGED_STORE != 0;

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int D = kHeadDim;
constexpr int TILE = 64;                       // tokens per wave iteration (one per lane)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kSmScale = 0.08838834764831845f;   // 1/sqrt(128)

// Half `hi` (0 or 1) of a 32-bit word as fp16.
__device__ inline _Float16 half_of(uint32_t w, int hi) {
  return __builtin_bit_cast(_Float16, (unsigned short)(hi ? (w >> 16) : (w & 0xffffu)));
}

template <int BITS>
struct Fields {
  static constexpr int FPW = 32 / BITS;        // fields per 32-bit word
  static constexpr int HALF = FPW / 2;         // fields per 16-bit half
  static constexpr int MPW = HALF / 2;         // MFMAs per word (each eats two field positions x two halves)
  static constexpr int SH = BITS == 2 ? 10 : 8;        // one shift brings the upper fields of both halves down
  static constexpr int NDIRECT = BITS == 2 ? 5 : (BITS == 1 ? 8 : 2);   // field positions used unshifted
  static __host__ __device__ constexpr int pos(int f) { return f < NDIRECT ? f : f - NDIRECT; }
  static __host__ __device__ constexpr uint32_t mask(int f) {
    return (uint32_t)(((1u << BITS) - 1u) * 0x00010001u) << (BITS * pos(f));
  }
  static __host__ __device__ constexpr uint32_t ones(int f) { return 0x00010001u << (BITS * pos(f)); }
  // index of inner position e (0..FPW) inside its word's operand table: [mfma][slot]
  static __host__ __device__ constexpr int slot(int e) {
    const int hi = e / HALF, f = e % HALF;
    return (f / 2) * 4 + (f % 2) * 2 + hi;
  }
};

template <int BITS>
__device__ inline half4_t operand(uint32_t w, uint32_t w_shifted, int m) {
  using F = Fields<BITS>;
  const int f0 = 2 * m, f1 = 2 * m + 1;
  u32x2 r;
  r.x = (f0 < F::NDIRECT ? w : w_shifted) & F::mask(f0);
  r.y = (f1 < F::NDIRECT ? w : w_shifted) & F::mask(f1);
  return __builtin_bit_cast(half4_t, r);
}

template <int BITS>
__device__ inline half4_t ones_operand(int m) {
  using F = Fields<BITS>;
  u32x2 r;
  r.x = F::ones(2 * m);
  r.y = F::ones(2 * m + 1);
  return __builtin_bit_cast(half4_t, r);
}

__device__ inline float wave_max(float x) {
  // butterflies inside a row of 16 lanes via DPP, then the four rows through scalar registers
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

template <typename T>
__device__ inline T stream_load(const T* p) { return __builtin_nontemporal_load(p); }

// Everything one wave iteration reads from the quantised store.  3-bit codes are two planes per
// packed run (2-bit low parts, then 1-bit high parts): a key row is 32 + 16 bytes, one channel of
// one value group G/4 + G/8 bytes.
template <int KB, int VB, int G>
struct TileRegs {
  static constexpr int KC = D * KB / 8 / 16;           // 16-byte pieces of one key row
  static constexpr int NG = D / G;                     // key groups per token
  static constexpr int GPT = TILE / G;                 // value token-groups per tile
  static constexpr int CW = G * VB / 32;               // words of one channel of one value group
  static constexpr int VW = 2 * CW;                    // ... of this lane's two channels
  u32x4 kc[KC];
  uint32_t ks[NG / 2], kz[NG / 2];                     // fp16 pairs
  uint32_t vw[GPT][VW];
  uint32_t vs[GPT], vz[GPT];                           // fp16 pairs (this lane's two channels)
  long long gshift;                                    // paged store: where the tile's value groups sit (wave-uniform)
  __device__ uint32_t k_word(int w) const { return kc[w / 4][w % 4]; }                 // (low) plane of the row
  __device__ uint32_t k_high(int w) const { return kc[(D * 2 / 32 + w) / 4][(D * 2 / 32 + w) % 4]; }
  __device__ uint32_t v_word(int gi, int ch, int w) const { return vw[gi][ch * CW + w]; }
  __device__ uint32_t v_high(int gi, int ch, int w) const { return vw[gi][ch * CW + G * 2 / 32 + w]; }
};

// Tiles' worth of time a window chunk of `len` tokens costs the wavefront that carries it.  The
// chunk runs at the lowest issue priority next to a partner that is busy about three quarters of
// the time, so its wall time is several times its own instruction count; the slope is the one that
// balances the launch best when swept (3 to 11 per 64 tokens: flat between 5 and 11 on the 32k-token
// G = 32 configuration, best at 9; best at 5 on the 8k x 32 G = 64 one, 6 % better than at 11).
__host__ __device__ inline int window_cost(long long len, int group) { return (int)(2 + (group == 64 ? 5 : 9) * len / 64); }

// KB, VB: widths of the key and value codes.  ZK: the key zero-point array exists (the key mode is not
// symmetric-only).  ZV: 0 = no value zero-point array; 1 = zero-points read densely, one tile ahead with
// everything else; 2 = sparse (Section "Sparsity of M": the flag matrix is mostly zero): a lane reads the
// zero-points of its two channels only if one of the two groups is flagged asymmetric (the flag is the
// sign bit of the scale it already holds), at the start of the tile that needs them, so a 128-byte line
// of zero-points (64 channels of one token-group) that holds no asymmetric group is never fetched.
template <int KB, int VB, int G, int NH4, bool ZK, int ZV>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2, 2))) attention_inner_kernel(AttnArgs a_in, int n_both_in, int n_splits, WindowSet win_in, int win_tiles_in, int base_t_in,
                                                                                                 int rem_t_in, int r) {
  constexpr int LBK = KB == 3 ? 2 : KB, LBV = VB == 3 ? 2 : VB;   // field width of the (low) plane
  constexpr bool HIK = KB == 3, HIV = VB == 3;                     // a plane of high bits follows it
  using FK = Fields<LBK>;
  using FV = Fields<LBV>;
  using F1 = Fields<1>;
  using Regs = TileRegs<KB, VB, G>;
  constexpr int NG = Regs::NG, GPT = Regs::GPT, KC = Regs::KC, VW = Regs::VW;
  constexpr int HWG = G / 32;                          // words of the high-bit plane per group
  constexpr int NW = D / FK::FPW;                      // words per key row
  constexpr int WPGK = G / FK::FPW, WPGV = G / FV::FPW;   // words per group (key: channels; value: tokens)
  constexpr int MPWK = FK::MPW, MPWV = FV::MPW;
  constexpr int HALFK = 1 << (KB - 1), HALFV = 1 << (VB - 1);
  constexpr int NH = NH4 * 4;

  // No division on the way to the first load: the grid is (splits, kv heads, batch), and the
  // host passes the quotients (heads per kv head; tiles per plain wavefront and their remainder).
  const int lane = threadIdx.x;
  const int hk = (int)blockIdx.y, b = (int)blockIdx.z;
  // The host's plan holds for every sequence -- unless the token counts live on the device
  // (a.n_dev: one count per sequence, the tokens cached BEFORE this step; attention runs over them
  // plus the new token).  Then the launch shape (wavefronts, window chunks, partial slots) is the
  // host's, planned for the longest sequence allowed, and everything that depends on the length is
  // recomputed here for this wavefront's sequence: the partition of Eq. kv_cache_init_quantized_window,
  // the window set and the split of the tiles over the wavefronts.  Wavefronts left without a tile
  // write an empty partial.
  AttnArgs a = a_in;
  int n_both = n_both_in, win_tiles = win_tiles_in, base_t = base_t_in, rem_t = rem_t_in;
  WindowSet win = win_in;
  if (a_in.n_dev) {
    long long N = (long long)a_in.n_dev[b] + 1;
    N = N < 1 ? 1 : (N > a.capacity ? a.capacity : N);
    if (a.n_copy && blockIdx.x == 0 && hk == 0 && lane == 0) a.n_copy[b] = (int)(N - 1);   // for the append that follows
    const int w_recent = a.k.slots - 1;                  // (the per-token key ring has w_recent + 1 slots)
    const long long kq = quantised_rows(a.w_sink, w_recent, a.group, kPerToken, N);
    const long long vq = quantised_rows(a.w_sink, w_recent, a.group, kPerChannel, N);
    const int n_sink = (int)(N < a.w_sink ? N : a.w_sink);
    a.n_tokens = N;
    a.k.n_sink = n_sink; a.v.n_sink = n_sink;
    a.k.n_quant = kq; a.v.n_quant = vq;
    n_both = (int)vq;
    win.na = n_sink;
    win.b0 = a.w_sink + vq;
    win.nb = N > win.b0 ? N - win.b0 : 0;
    const int tiles = (n_both + TILE - 1) / TILE;
    const int cost = win.n_chunks > 0 ? window_cost((win.na + win.nb + win.n_chunks - 1) / win.n_chunks, G) : 0;
    const int quota = (tiles + win.n_chunks * cost + n_splits - 1) / n_splits;
    win_tiles = quota > cost ? quota - cost : 0;
    if (win.n_chunks > 0 && win_tiles > tiles / win.n_chunks) win_tiles = tiles / win.n_chunks;
    const int rest = tiles - win.n_chunks * win_tiles, others = n_splits - win.n_chunks;
    base_t = rest / others;
    rem_t = rest % others;
  }
  const long long bh = (long long)b * a.n_kv_heads + hk;
  constexpr bool has_kz = ZK, has_vz = ZV != 0;  // zero-point arrays exist unless the tensor is symmetric-only
  constexpr bool late_vz = ZV == 2;              // value zero-points: only where flagged, at the start of their tile

  // ---- tile range of this wavefront.  The first win.n_chunks wavefronts of a (batch, kv-head)
  // also serve one chunk of the fp16 windows each (after their tiles) and get win_tiles tiles;
  // the others share the remaining tiles evenly.
  const int n_tiles = (n_both + TILE - 1) / TILE;
  const int s_idx = (int)blockIdx.x;
  int t0, t1;
  if (s_idx < win.n_chunks) {
    t0 = s_idx * win_tiles;
    t1 = t0 + win_tiles;
  } else {
    const int j = s_idx - win.n_chunks;                  // base_t, rem_t: (n_tiles - n_chunks * win_tiles) divided by the plain wavefronts
    t0 = win.n_chunks * win_tiles + j * base_t + (j < rem_t ? j : rem_t);
    t1 = t0 + base_t + (j < rem_t ? 1 : 0);
  }

  __shared__ __attribute__((aligned(16))) _Float16 qA[NH * D];          // query operand table [head][word][mfma][slot]
  __shared__ __attribute__((aligned(16))) float qsum[NH4][NG][4];       // log2e/sqrt(d) * sum of q over each key group
  __shared__ __attribute__((aligned(16))) _Float16 pA[NH * TILE];       // probability operand table [head][word][mfma][slot]
  // the same two tables for the plane of high bits (1-bit fields, weight 4): [head][word][mfma][slot]
  __shared__ __attribute__((aligned(16))) _Float16 qA1[HIK ? NH * D : 8];
  __shared__ __attribute__((aligned(16))) _Float16 pA1[HIV ? NH * TILE : 8];

  // A wavefront without a tile (a launch with more wavefronts than tiles gives the window chunks
  // wavefronts of their own) skips all of the tile machinery, query tables included.
  float part_m[NH], part_l[NH];
  float2 part_o[NH];
#pragma unroll
  for (int h = 0; h < NH; ++h) { part_m[h] = -INFINITY; part_l[h] = 0.f; part_o[h] = float2{0.f, 0.f}; }   // (an empty partial)
  if (t1 > t0) {
  // ---- per-(b, hk) base pointers
  const long long slab = kPagedStore ? 0 : bh * a.capacity;             // first store row of (b, hk); paged: see below
  const uint8_t* kcodes_slab = a.k.codes + slab * (D * KB / 8);
  const __half* kscales_slab = a.k.scales + slab * NG;
  const __half* kzeros_slab = has_kz ? a.k.zeros + slab * NG : nullptr;
  const long long vgroups = slab / G;
  const uint8_t* vcodes_slab = a.v.codes + vgroups * D * (G * VB / 8);
  const __half* vscales_slab = a.v.scales + vgroups * D;
  const __half* vzeros_slab = has_vz ? a.v.zeros + vgroups * D : nullptr;
  const int last_row = n_both - 1, last_group = n_both / G - 1;
  constexpr int ROWB = D * KB / 8;                     // bytes of one key row
  constexpr int GB = G * VB / 8;                       // bytes of one channel of one value group

  // Paged store: a tile is one page (kPageTokens == TILE), so the tile's rows sit `shift` rows away
  // from where the contiguous layout of a pool-sized cache would put rows tile * 64 .. of (b = 0, hk = 0):
  // a wave-uniform 64-bit shift of the six bases, looked up once per tile.
  static_assert(kPageTokens == TILE, "a page of the store is one tile of this kernel");
  // The table entries of this wavefront's tiles come in one vector load, lane i holding the entry of
  // tile pages_from + i (a wavefront with more than 64 tiles reloads every 64), and a tile reads its
  // entry with a lane read.  (A scalar load per tile, even issued a tile ahead, costs more: scalar loads
  // return out of order, so the first wait for an LDS operation behind it waits for the load as well.)
  constexpr bool paged = kPagedStore;
  int pages_from = t0, pages_held = 0;
  auto fetch_pages = [&](int from) {
    const int tile = from + lane < t1 ? from + lane : t1 - 1;
    pages_from = from;
    pages_held = a.pages.table[(long long)b * a.pages.tiles_per_seq + tile];
  };
  if constexpr (paged) {
    if (t1 > t0) fetch_pages(t0);
  }

  // All offsets inside one (b, hk) slab fit 32 bits; bases are wave-uniform.
  auto load_tile = [&](int tile, Regs& t) {
    const uint8_t *kcodes = kcodes_slab, *vcodes = vcodes_slab;
    const __half *kscales = kscales_slab, *kzeros = kzeros_slab, *vscales = vscales_slab, *vzeros = vzeros_slab;
    if constexpr (paged) {
      if (tile - pages_from >= 64) fetch_pages(tile);
      int page = __builtin_amdgcn_readlane(pages_held, tile - pages_from);
      page = page < 0 ? 0 : (page >= a.pages.pool_pages ? a.pages.pool_pages - 1 : page);
      const long long shift = (((long long)page * a.n_kv_heads + hk) - tile) * TILE, gshift = shift / G * D;
      kcodes += shift * ROWB; kscales += shift * NG;
      if constexpr (has_kz) kzeros += shift * NG;
      vcodes += gshift * GB; vscales += gshift;
      if constexpr (has_vz) vzeros += gshift;
      t.gshift = gshift;
    }
    int row = tile * TILE + lane;
    row = row > last_row ? last_row : row;
    const u32x4* kp = reinterpret_cast<const u32x4*>(kcodes + (uint32_t)row * ROWB);
#pragma unroll
    for (int i = 0; i < KC; ++i) t.kc[i] = stream_load(kp + i);
    if constexpr (NG == 4) {
      const u32x2 s = stream_load(reinterpret_cast<const u32x2*>(kscales + (uint32_t)row * NG));
      t.ks[0] = s.x; t.ks[1] = s.y;
      if constexpr (has_kz) {
        const u32x2 z = stream_load(reinterpret_cast<const u32x2*>(kzeros + (uint32_t)row * NG));
        t.kz[0] = z.x; t.kz[1] = z.y;
      }
    } else {
      t.ks[0] = stream_load(reinterpret_cast<const uint32_t*>(kscales + (uint32_t)row * NG));
      if constexpr (has_kz) t.kz[0] = stream_load(reinterpret_cast<const uint32_t*>(kzeros + (uint32_t)row * NG));
    }
#pragma unroll
    for (int gi = 0; gi < GPT; ++gi) {
      int grp = tile * GPT + gi;
      grp = grp > last_group ? last_group : grp;
      const uint32_t ch = (uint32_t)grp * D + 2 * lane;
      if constexpr (VW % 4 == 0) {
        const u32x4* vp = reinterpret_cast<const u32x4*>(vcodes + ch * GB);
#pragma unroll
        for (int i = 0; i < VW / 4; ++i) {
          const u32x4 v = stream_load(vp + i);
          t.vw[gi][4 * i] = v.x; t.vw[gi][4 * i + 1] = v.y; t.vw[gi][4 * i + 2] = v.z; t.vw[gi][4 * i + 3] = v.w;
        }
      } else {                                          // 3-bit, G = 32: 24 bytes per lane
        const u32x2* vp = reinterpret_cast<const u32x2*>(vcodes + ch * GB);
#pragma unroll
        for (int i = 0; i < VW / 2; ++i) {
          const u32x2 v = stream_load(vp + i);
          t.vw[gi][2 * i] = v.x; t.vw[gi][2 * i + 1] = v.y;
        }
      }
      t.vs[gi] = stream_load(reinterpret_cast<const uint32_t*>(vscales + ch));
      if constexpr (has_vz && !late_vz) t.vz[gi] = stream_load(reinterpret_cast<const uint32_t*>(vzeros + ch));
    }
  };

  // ---- the query loads go out first (the set-up below waits for them), the first tile's loads
  // right behind them: those overlap the query set-up
  u32x4 q_raw[NH4];
  float4_t q_fac[NH4][2];                              // per-channel query factors, when given
#pragma unroll
  for (int rnd = 0; rnd < NH4; ++rnd) {
    const int h = (rnd * 64 + lane) / (D / 8), c0 = 8 * ((rnd * 64 + lane) % (D / 8));
    q_raw[rnd] = u32x4{0u, 0u, 0u, 0u};
    if (h < r) q_raw[rnd] = *reinterpret_cast<const u32x4*>(a.q + ((long long)b * a.n_q_heads + hk * r + h) * D + c0);
    if (a.q_scale) {
      q_fac[rnd][0] = *reinterpret_cast<const float4_t*>(a.q_scale + hk * D + c0);
      q_fac[rnd][1] = *reinterpret_cast<const float4_t*>(a.q_scale + hk * D + c0 + 4);
    }
  }
  Regs bufA, bufB;
  if (t1 > t0) load_tile(t0, bufA);

  float q_coef[NH];
  // ---- query: fp16 (optionally rescaled), position factors folded in.  A lane takes 8
  // consecutive channels of one head (one 16-byte load); the channels of one key group sit in
  // G/8 neighbouring lanes, so the group sums of q come from a few DPP adds.
#pragma unroll
  for (int rnd = 0; rnd < NH4; ++rnd) {
    const int idx = rnd * 64 + lane;
    const int h = idx / (D / 8), c0 = 8 * (idx % (D / 8));
    const uint32_t rw[4] = {q_raw[rnd].x, q_raw[rnd].y, q_raw[rnd].z, q_raw[rnd].w};
    float qv[8], part = 0.f, mx = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t hb = (e & 1) ? (rw[e / 2] >> 16) : (rw[e / 2] & 0xffffu);
      qv[e] = __half2float(__ushort_as_half((unsigned short)hb));
      if (a.q_scale) qv[e] = __half2float(scaled_half(qv[e], q_fac[rnd][e / 4][e % 4]));
      part += qv[e];
      mx = __builtin_fmaxf(mx, __builtin_fabsf(qv[e]));
    }
    // power of two that brings the head's largest |q| into [2^8, 2^9): the position factors span
    // up to 2^-10 .. 2^6, so the table entries stay normal fp16 numbers down to 2^-13 of the
    // head's maximum whatever the magnitude of the queries (a head is D/8 = 16 neighbouring lanes)
    static_assert(D / 8 == 16, "a head is one 16-lane row of the cross-lane operations below");
    mx = __builtin_fmaxf(mx, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, mx), 0xB1, 0xF, 0xF, true)));    // lane ^ 1
    mx = __builtin_fmaxf(mx, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, mx), 0x4E, 0xF, 0xF, true)));    // lane ^ 2
    mx = __builtin_fmaxf(mx, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, mx), 0x141, 0xF, 0xF, true)));   // mirror within 8
    mx = __builtin_fmaxf(mx, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, mx), 0x140, 0xF, 0xF, true)));   // mirror within 16
    const int q_exp = mx > 0.f ? (int)((__float_as_uint(mx) >> 23) & 0xffu) - 127 : 8;
    const float q_pow = __uint_as_float((uint32_t)(127 + 8 - q_exp) << 23);
    // per-head constant of the score, log2e/sqrt(d) * 2^20 / (the head's factor): wave-uniform, so it
    // goes to scalar registers straight from the first lane of each head's row
    const float coef = (kSmScale * kLog2e * 1048576.0f) * __uint_as_float((uint32_t)(127 - 8 + q_exp) << 23);
#pragma unroll
    for (int j = 0; j < 4; ++j)
      q_coef[rnd * 4 + j] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, coef), 16 * j));
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int c = c0 + e;
      const int word = c / FK::FPW, ep = c % FK::FPW;
      const int f = ep % FK::HALF;
      const float factor = (float)(1 << (4 + LBK * 4)) / (float)(1 << (LBK * FK::pos(f) + LBK * 4));   // 2^(4 - b*pos)
      qA[(h * NW + word) * (MPWK * 4) + FK::slot(ep)] = (_Float16)(qv[e] * q_pow * factor);
      if constexpr (HIK) {
        // 1-bit field at position pos of its half: 2^(pos - 24); weight 4 -> q * 2^(6 - pos)
        const int word1 = c / 32, ep1 = c % 32;
        const float factor1 = 64.0f / (float)(1 << F1::pos(ep1 % 16));
        qA1[(h * (D / 32) + word1) * (F1::MPW * 4) + F1::slot(ep1)] = (_Float16)(qv[e] * q_pow * factor1);
      }
    }
    // sum over the G/8 lanes of the group (4 lanes: one quad; 8 lanes: two quads)
    part += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, part), 0xB1, 0xF, 0xF, true));
    part += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, part), 0x4E, 0xF, 0xF, true));
    if constexpr (G == 64)
      part += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, part), 0x141, 0xF, 0xF, true));
    if ((idx % (G / 8)) == 0) qsum[h / 4][c0 / G][h % 4] = part * (kSmScale * kLog2e);
  }
  __syncthreads();

  // ---- A operands of the zero-point term: sum over groups of Zeff_g * (sum of q over group g) is a
  // 4 (heads) x 4 (groups) product per token, one more matrix instruction.  The group sums of q
  // enter as two fp16 pieces (hi + lo, 2^-22 relative) so that the term keeps fp32 accuracy; Zeff
  // is an exact fp16 number (Z for an asymmetric group, -2^(b-1) S for a symmetric one).  The
  // operands carry 2 * qsum and Zeff / 2: S is at most 65504 / (2^(b-1) - 1), so 2^(b-2) S is
  // finite in fp16 for every finite cache where 2^(b-1) S is not; Z / 2 is exact unless Z is an fp16
  // denormal with an odd last bit (2^-25 off).
  half4_t qs_hi[NH4], qs_lo[NH4];
#pragma unroll
  for (int n = 0; n < NH4; ++n) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float v = g < NG ? 2.f * qsum[n][g][lane & 3] : 0.f;
      const _Float16 hi = (_Float16)v;
      qs_hi[n][g] = hi;
      qs_lo[n][g] = (_Float16)(v - (float)hi);
    }
  }

  // ---- running softmax state (log2 domain) and output accumulators.
  // m_run is a reference level, not the exact running maximum: it is raised (and l, o rescaled)
  // only when some score exceeds it by more than kSlack, so the common tile pays no wave-wide
  // reduction and no rescale.  Probabilities are then at most 2^kSlack, times the position
  // factor 2^8: still inside fp16.  l_run and o are kept divided by 2^16 (the raw MFMA scale).
  // The first tile sets the level to its exact maximum.
  constexpr float kSlack = HIV ? 5.0f : 6.0f;           // (the high-bit plane's factors reach 2^10)
  float m_run[NH], l_run[NH], o[NH][2];
#pragma unroll
  for (int h = 0; h < NH; ++h) { m_run[h] = 0.f; l_run[h] = 0.f; o[h][0] = 0.f; o[h][1] = 0.f; }

  // where this lane's token sits in the probability operand table, and its position factor
  const int p_e = lane % FV::FPW;
  const int p_index = (lane / FV::FPW) * (MPWV * 4) + FV::slot(p_e);
  const float p_shift = (float)(8 - LBV * FV::pos(p_e % FV::HALF));        // p is stored as p * 2^(8 - b*pos)
  // the same token in the high-bit plane's table: p * 4 * 2^(8 - pos), as a factor on the stored p
  const int p1_e = lane % 32;
  const int p1_index = (lane / 32) * (F1::MPW * 4) + F1::slot(p1_e);
  const float p1_factor = __builtin_amdgcn_exp2f((float)(10 - F1::pos(p1_e % 16)) - p_shift);
  const int qa_lane = (lane & 3) * D;                                   // this lane supplies head (lane & 3) to A
  const int pa_lane = (lane & 3) * TILE;

  auto process = [&](const Regs& cur, int tile, bool first) {
    // sparse value zero-points: the lanes whose scale pair carries a flag fetch theirs now; they are
    // needed at the end of the tile
    uint32_t vz_late[GPT];
    if constexpr (late_vz) {
      const __half* vz_tile = vzeros_slab;
      if constexpr (paged) vz_tile += cur.gshift;
#pragma unroll
      for (int gi = 0; gi < GPT; ++gi) {
        int grp = tile * GPT + gi;
        grp = grp > last_group ? last_group : grp;
        vz_late[gi] = 0u;
        if (cur.vs[gi] & 0x80008000u)
          vz_late[gi] = stream_load(reinterpret_cast<const uint32_t*>(vz_tile + (uint32_t)grp * D + 2 * lane));
      }
    }
    // ================= scores: lane = token (Eq. att:1 with Eq. hybrid_dequant fused) =================
    // one MFMA chain per key group, the chains interleaved so that consecutive MFMAs are independent
    float4_t acc[NG][NH4];
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
      for (int n = 0; n < NH4; ++n) acc[g][n] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int wd = 0; wd < WPGK; ++wd) {
      uint32_t w[NG], wsft[NG];
#pragma unroll
      for (int g = 0; g < NG; ++g) {
        const int word = g * WPGK + wd;
        w[g] = cur.k_word(word);
        wsft[g] = w[g] >> FK::SH;
      }
#pragma unroll
      for (int m = 0; m < MPWK; ++m) {
#pragma unroll
        for (int g = 0; g < NG; ++g) {
          const int word = g * WPGK + wd;
          const half4_t bop = operand<LBK>(w[g], wsft[g], m);
#pragma unroll
          for (int n = 0; n < NH4; ++n) {
            const half4_t aop = *reinterpret_cast<const half4_t*>(&qA[n * 4 * D + qa_lane + (word * MPWK + m) * 4]);
            acc[g][n] = __builtin_amdgcn_mfma_f32_4x4x4f16(aop, bop, acc[g][n], 0, 0, 0);
          }
        }
      }
    }
    if constexpr (HIK) {
      // the plane of high bits joins the same chains: its query table carries the weight 4
#pragma unroll
      for (int j = 0; j < HWG; ++j) {
        uint32_t w[NG], wsft[NG];
#pragma unroll
        for (int g = 0; g < NG; ++g) {
          w[g] = cur.k_high(g * HWG + j);
          wsft[g] = w[g] >> F1::SH;
        }
#pragma unroll
        for (int m = 0; m < F1::MPW; ++m) {
#pragma unroll
          for (int g = 0; g < NG; ++g) {
            const int word = g * HWG + j;
            const half4_t bop = operand<1>(w[g], wsft[g], m);
#pragma unroll
            for (int n = 0; n < NH4; ++n) {
              const half4_t aop =
                  *reinterpret_cast<const half4_t*>(&qA1[n * 4 * D + qa_lane + (word * F1::MPW + m) * 4]);
              acc[g][n] = __builtin_amdgcn_mfma_f32_4x4x4f16(aop, bop, acc[g][n], 0, 0, 0);
            }
          }
        }
      }
    }
    // e[h] = score (log2 domain) + position shift - reference level: the exponent of the stored probability.
    // Per group: |S| * (raw inner sum) + Zeff * (sum of q).  The scale sign bit marks an asymmetric
    // group, so max(s, 0) is |S| for a symmetric group and 0 for an asymmetric one, and
    // Zeff = Z - 2^(b-1) * max(s, 0) needs no select (Z is stored as +0 for symmetric groups).
    // Scales and zero-points enter the FMAs as fp16 sources; the constant factor is applied once.
    float e[NH], t[NH];
    {
      // Zeff / 2 of this token's groups as fp16: Z / 2 - 2^(b-2) max(s, 0) (one of the two terms is 0)
      u32x2 zw = {0u, 0u};
#pragma unroll
      for (int gp = 0; gp < NG / 2; ++gp) {
        const half2_t sp = __builtin_bit_cast(half2_t, cur.ks[gp]);
        const half2_t mp = __builtin_elementwise_max(sp, half2_t{(_Float16)0, (_Float16)0});
        half2_t zp;
        constexpr _Float16 kNegQuarterK = (_Float16)(-HALFK / 2), kHalf = (_Float16)0.5f;
        if constexpr (has_kz)
          zp = mp * half2_t{kNegQuarterK, kNegQuarterK} + __builtin_bit_cast(half2_t, cur.kz[gp]) * half2_t{kHalf, kHalf};
        else zp = sp * half2_t{kNegQuarterK, kNegQuarterK};
        zw[gp] = __builtin_bit_cast(uint32_t, zp);
      }
      const half4_t zop = __builtin_bit_cast(half4_t, zw);
#pragma unroll
      for (int n = 0; n < NH4; ++n) {
        float4_t ez = float4_t{p_shift - m_run[4 * n], p_shift - m_run[4 * n + 1], p_shift - m_run[4 * n + 2],
                               p_shift - m_run[4 * n + 3]};
        ez = __builtin_amdgcn_mfma_f32_4x4x4f16(qs_hi[n], zop, ez, 0, 0, 0);
        ez = __builtin_amdgcn_mfma_f32_4x4x4f16(qs_lo[n], zop, ez, 0, 0, 0);
        e[4 * n] = ez.x; e[4 * n + 1] = ez.y; e[4 * n + 2] = ez.z; e[4 * n + 3] = ez.w;
      }
    }
#pragma unroll
    for (int h = 0; h < NH; ++h) t[h] = 0.f;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const float S = __builtin_fabsf((float)half_of(cur.ks[g / 2], g & 1));
#pragma unroll
      for (int h = 0; h < NH; ++h) t[h] = __builtin_fmaf(S, acc[g][h / 4][h % 4], t[h]);
    }
#pragma unroll
    for (int h = 0; h < NH; ++h)
      e[h] = __builtin_fmaf(q_coef[h], t[h], e[h]);   // undoes the operand factors (2^20) and the head's query factor

    // ================= running softmax (Eq. att:2), probabilities to the operand table =================
    if (tile * TILE + (TILE - 1) > last_row) {         // ragged last tile: lanes past the end weigh nothing
      const bool valid = tile * TILE + lane <= last_row;
#pragma unroll
      for (int h = 0; h < NH; ++h) e[h] = valid ? e[h] : -INFINITY;
    }
    bool raise = false;
#pragma unroll
    for (int h = 0; h < NH; ++h) raise |= e[h] > kSlack + p_shift;
    if (first || __builtin_amdgcn_ballot_w64(raise) != 0) {   // rare after the first tiles
#pragma unroll
      for (int h = 0; h < NH; ++h) {
        const float mx = wave_max(e[h] - p_shift);           // largest score relative to the current level
        const float d = first ? mx : fmaxf(mx, 0.f);         // the level only rises, except when it is first set
        const float alpha = first ? 1.f : __builtin_amdgcn_exp2f(-d);
        m_run[h] += d;
        e[h] -= d;
        l_run[h] *= alpha;
        o[h][0] *= alpha;
        o[h][1] *= alpha;
      }
    }
    __syncthreads();                                   // previous tile's readers of pA are done
#pragma unroll
    for (int h = 0; h < NH; ++h) {
      const float p = __builtin_amdgcn_exp2f(e[h]);
      pA[h * TILE + p_index] = (_Float16)p;
      if constexpr (HIV) pA1[h * TILE + p1_index] = (_Float16)(p * p1_factor);
    }
    __syncthreads();

    // ================= values: lane = two channels (Eq. att:3 with Eq. hybrid_dequant fused) =================
#pragma unroll
    for (int gi = 0; gi < GPT; ++gi) {
      float4_t acc0[NH4], acc1[NH4], accl[NH4];
#pragma unroll
      for (int n = 0; n < NH4; ++n) {
        acc0[n] = float4_t{0.f, 0.f, 0.f, 0.f};
        acc1[n] = acc0[n];
        accl[n] = acc0[n];
      }
#pragma unroll
      for (int wd = 0; wd < WPGV; ++wd) {
        const uint32_t wa = cur.v_word(gi, 0, wd), wb = cur.v_word(gi, 1, wd);
        const uint32_t was = wa >> FV::SH, wbs = wb >> FV::SH;
#pragma unroll
        for (int m = 0; m < MPWV; ++m) {
          const half4_t b0 = operand<LBV>(wa, was, m);
          const half4_t b1 = operand<LBV>(wb, wbs, m);
          const half4_t b1s = ones_operand<LBV>(m);
#pragma unroll
          for (int n = 0; n < NH4; ++n) {
            const half4_t aop =
                *reinterpret_cast<const half4_t*>(&pA[n * 4 * TILE + pa_lane + ((gi * WPGV + wd) * MPWV + m) * 4]);
            acc0[n] = __builtin_amdgcn_mfma_f32_4x4x4f16(aop, b0, acc0[n], 0, 0, 0);
            acc1[n] = __builtin_amdgcn_mfma_f32_4x4x4f16(aop, b1, acc1[n], 0, 0, 0);
            accl[n] = __builtin_amdgcn_mfma_f32_4x4x4f16(aop, b1s, accl[n], 0, 0, 0);
          }
        }
      }
      if constexpr (HIV) {
#pragma unroll
        for (int j = 0; j < HWG; ++j) {
          const uint32_t wa = cur.v_high(gi, 0, j), wb = cur.v_high(gi, 1, j);
          const uint32_t was = wa >> F1::SH, wbs = wb >> F1::SH;
#pragma unroll
          for (int m = 0; m < F1::MPW; ++m) {
            const half4_t b0 = operand<1>(wa, was, m);
            const half4_t b1 = operand<1>(wb, wbs, m);
#pragma unroll
            for (int n = 0; n < NH4; ++n) {
              const half4_t aop = *reinterpret_cast<const half4_t*>(
                  &pA1[n * 4 * TILE + pa_lane + ((gi * HWG + j) * F1::MPW + m) * 4]);
              acc0[n] = __builtin_amdgcn_mfma_f32_4x4x4f16(aop, b0, acc0[n], 0, 0, 0);
              acc1[n] = __builtin_amdgcn_mfma_f32_4x4x4f16(aop, b1, acc1[n], 0, 0, 0);
            }
          }
        }
      }
      const uint32_t spair = cur.vs[gi];
      const float S0 = __builtin_fabsf((float)half_of(spair, 0)), S1 = __builtin_fabsf((float)half_of(spair, 1));
      float z0, z1;
      if constexpr (has_vz) {
        const uint32_t mpair = __builtin_bit_cast(
            uint32_t, __builtin_elementwise_max(__builtin_bit_cast(half2_t, spair), half2_t{(_Float16)0, (_Float16)0}));
        const uint32_t zpair = late_vz ? vz_late[gi] : cur.vz[gi];
        z0 = __builtin_fmaf((float)half_of(mpair, 0), (float)(-HALFV), (float)half_of(zpair, 0));
        z1 = __builtin_fmaf((float)half_of(mpair, 1), (float)(-HALFV), (float)half_of(zpair, 1));
      } else {
        z0 = S0 * (float)(-HALFV);
        z1 = S1 * (float)(-HALFV);
      }
      // accl = 2^-16 * (sum of the fp16 probabilities of this group); l and o stay in that scale
#pragma unroll
      for (int n = 0; n < NH4; ++n) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          l_run[n * 4 + i] += accl[n][i];
          o[n * 4 + i][0] = __builtin_fmaf(S0, acc0[n][i], __builtin_fmaf(z0, accl[n][i], o[n * 4 + i][0]));
          o[n * 4 + i][1] = __builtin_fmaf(S1, acc1[n][i], __builtin_fmaf(z1, accl[n][i], o[n * 4 + i][1]));
        }
      }
    }
  };

  // ---- two register buffers, ping-pong: the next tile's loads are in flight while this one is computed
  {
    const int n = t1 - t0;
    int i = 0;
    // (one or two tiles only: ahead of the wavefronts that carry nothing but a window chunk)
    if (n <= 2) __builtin_amdgcn_s_setprio(2);
    while (i + 2 < n) {
      // the wavefront that is behind gets the SIMD first: the two wavefronts of a SIMD then
      // finish together instead of one running alone (and at a lower rate) at the end
      if (4 * i < n) __builtin_amdgcn_s_setprio(3);
      else if (2 * i < n) __builtin_amdgcn_s_setprio(2);
      else if (4 * i < 3 * n) __builtin_amdgcn_s_setprio(1);
      else __builtin_amdgcn_s_setprio(0);
      load_tile(t0 + i + 1, bufB);
      process(bufA, t0 + i, i == 0);
      load_tile(t0 + i + 2, bufA);
      process(bufB, t0 + i + 1, false);
      i += 2;
    }
    if (n - i == 2) {
      load_tile(t0 + i + 1, bufB);
      process(bufA, t0 + i, i == 0);
      process(bufB, t0 + i + 1, false);
    } else if (n - i == 1) {
      process(bufA, t0 + i, i == 0);
    }
  }

  // ---- partial (m, l, o) of every real head, kept in registers over the window pass
#pragma unroll
  for (int h = 0; h < NH; ++h) {
    part_o[h].x = o[h][0] * 65536.0f;                  // 2^16 undoes the operand factors of the value pass
    part_o[h].y = o[h][1] * 65536.0f;
    part_m[h] = m_run[h] * kLn2;
    part_l[h] = l_run[h] * 65536.0f;
  }
  }

  // ---- the window chunk of this wavefront, with a partial slot of its own
  if (s_idx < win.n_chunks) {
    __builtin_amdgcn_s_setprio(0);
    window_pass<NH4, KB, G, true, false, kPagedStore>(a, bh, win.na, win.b0, win.nb, s_idx, win.n_chunks, n_splits + s_idx);
  }

  // ---- the tile partial goes out last: nothing after these stores reuses their registers (which
  // would have to wait for the stores to complete)
#pragma unroll
  for (int h = 0; h < NH; ++h) {
    if (h < r) {
      const long long bhq = (long long)b * a.n_q_heads + hk * r + h;
      *reinterpret_cast<float2*>(&a.ws_o[(bhq * a.n_partials + s_idx) * D + 2 * lane]) = part_o[h];
      if (lane == 0) {
        a.ws_ml[(bhq * a.n_partials + s_idx) * 2 + 0] = part_m[h];
        a.ws_ml[(bhq * a.n_partials + s_idx) * 2 + 1] = part_l[h];
      }
    }
  }
}

template <int KB, int VB, int G, bool ZK, int ZV>
hipError_t launch_z(const AttnArgs& a, int n_both, int n_splits, const WindowSet& win, const Launch& L) {
  const int r = a.n_q_heads / a.n_kv_heads;
  // A window chunk costs its wavefront about as much time as window_cost() tiles: the wavefronts
  // that carry one get that many tiles fewer than the common quota.
  const int n_tiles = (n_both + TILE - 1) / TILE;
  const int cost = win.n_chunks > 0 ? window_cost((win.na + win.nb + win.n_chunks - 1) / win.n_chunks, G) : 0;
  const int quota = (n_tiles + win.n_chunks * cost + n_splits - 1) / n_splits;
  int win_tiles = quota > cost ? quota - cost : 0;
  if (win.n_chunks > 0 && win_tiles > n_tiles / win.n_chunks) win_tiles = n_tiles / win.n_chunks;
  if (n_splits <= win.n_chunks) return hipErrorInvalidValue;      // the host gives at least one plain wavefront
  if (a.batch > 65535 || a.n_kv_heads > 65535) return hipErrorInvalidValue;
  const int rest = n_tiles - win.n_chunks * win_tiles, others = n_splits - win.n_chunks;
  const int base_t = rest / others, rem_t = rest % others;
  dim3 grid((unsigned)n_splits, (unsigned)a.n_kv_heads, (unsigned)a.batch);
  // (the launch with dispatch events only when events were asked for: the plain launch is the one a
  // stream capture is sure to record)
  const bool timed = L.ev_start || L.ev_stop;
  if (r <= 4) {
    if (timed)
      hipExtLaunchKernelGGL((attention_inner_kernel<KB, VB, G, 1, ZK, ZV>), grid, dim3(64), 0, L.stream, L.ev_start,
                            L.ev_stop, 0, a, n_both, n_splits, win, win_tiles, base_t, rem_t, r);
    else
      hipLaunchKernelGGL((attention_inner_kernel<KB, VB, G, 1, ZK, ZV>), grid, dim3(64), 0, L.stream, a, n_both,
                         n_splits, win, win_tiles, base_t, rem_t, r);
  } else {
    if (timed)
      hipExtLaunchKernelGGL((attention_inner_kernel<KB, VB, G, 2, ZK, ZV>), grid, dim3(64), 0, L.stream, L.ev_start,
                            L.ev_stop, 0, a, n_both, n_splits, win, win_tiles, base_t, rem_t, r);
    else
      hipLaunchKernelGGL((attention_inner_kernel<KB, VB, G, 2, ZK, ZV>), grid, dim3(64), 0, L.stream, a, n_both,
                         n_splits, win, win_tiles, base_t, rem_t, r);
  }
  return hipGetLastError();
}

// Wavefronts of this kernel instance that one compute unit holds at once (a host-side query).
template <int KB, int VB, int G, bool ZK, int ZV>
int resident_z(const AttnArgs& a) {
  const int r = a.n_q_heads / a.n_kv_heads;
  int n = 0;
  hipError_t e = r <= 4
      ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, attention_inner_kernel<KB, VB, G, 1, ZK, ZV>, 64, 0)
      : hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, attention_inner_kernel<KB, VB, G, 2, ZK, ZV>, 64, 0);
  return (e == hipSuccess && n > 0) ? n : 8;
}

// 0: no value zero-point array; 1: read densely; 2: read only where a group is flagged
inline int value_zero_mode(const AttnArgs& a) { return a.v.zeros == nullptr ? 0 : (a.sparse_zeros ? 2 : 1); }

template <int KB, int VB, int G>
hipError_t launch_t(const AttnArgs& a, int n_both, int n_splits, const WindowSet& win, const Launch& L) {
  const bool zk = a.k.zeros != nullptr;
  const int zv = value_zero_mode(a);
  if (zk) {
    if (zv == 2) return launch_z<KB, VB, G, true, 2>(a, n_both, n_splits, win, L);
    if (zv == 1) return launch_z<KB, VB, G, true, 1>(a, n_both, n_splits, win, L);
    return launch_z<KB, VB, G, true, 0>(a, n_both, n_splits, win, L);
  }
  if (zv == 2) return launch_z<KB, VB, G, false, 2>(a, n_both, n_splits, win, L);
  if (zv == 1) return launch_z<KB, VB, G, false, 1>(a, n_both, n_splits, win, L);
  return launch_z<KB, VB, G, false, 0>(a, n_both, n_splits, win, L);
}

template <int KB, int VB, int G>
int resident_t(const AttnArgs& a) {
  const bool zk = a.k.zeros != nullptr;
  const int zv = value_zero_mode(a);
  if (zk) return zv == 2 ? resident_z<KB, VB, G, true, 2>(a) : zv == 1 ? resident_z<KB, VB, G, true, 1>(a) : resident_z<KB, VB, G, true, 0>(a);
  return zv == 2 ? resident_z<KB, VB, G, false, 2>(a) : zv == 1 ? resident_z<KB, VB, G, false, 1>(a) : resident_z<KB, VB, G, false, 0>(a);
}

// Width pairs (keys, values) the fused kernel is built for: equal widths, and the paper's
// Hybrid / Small presets (3-bit keys, 2-bit values).
inline int width_pair(const AttnArgs& a) {
  if (a.bits == a.v_bits && a.bits >= 2 && a.bits <= 4) return a.bits - 2;   // 0, 1, 2
  if (a.bits == 3 && a.v_bits == 2) return 3;
  return -1;
}

// Calls f.template operator()<KB, VB, G>() for the configuration's widths and group size.
template <typename Fn>
auto for_widths(const AttnArgs& a, Fn f) {
  const int wp = width_pair(a);
  if (a.group == 32) {
    if (wp == 0) return f.template operator()<2, 2, 32>();
    if (wp == 1) return f.template operator()<3, 3, 32>();
    if (wp == 2) return f.template operator()<4, 4, 32>();
    return f.template operator()<3, 2, 32>();
  }
  if (wp == 0) return f.template operator()<2, 2, 64>();
  if (wp == 1) return f.template operator()<3, 3, 64>();
  if (wp == 2) return f.template operator()<4, 4, 64>();
  return f.template operator()<3, 2, 64>();
}

struct ResidentFn {
  const AttnArgs& a;
  template <int KB, int VB, int G>
  int operator()() const { return resident_t<KB, VB, G>(a); }
};
struct LaunchFn {
  const AttnArgs& a; int n_both, n_splits; const WindowSet& win; const Launch& L;
  template <int KB, int VB, int G>
  hipError_t operator()() const { return launch_t<KB, VB, G>(a, n_both, n_splits, win, L); }
};

// cached per (widths, group, zero flags, head tile): the answer depends on the kernel instance only
int waves_per_cu_of_this_build(const AttnArgs& a) {
  static CachedInt cache[4][2][2][3][2];
  const int r = a.n_q_heads / a.n_kv_heads;
  const int wp = width_pair(a);
  if (wp < 0) return 8;
  return cache[wp][a.group == 64][a.k.zeros != nullptr][value_zero_mode(a)][r > 4].get(
      [&] { return for_widths(a, ResidentFn{a}); });
}

}  // namespace

#if INNERQ_PAGED_STORE

int attention_inner_paged_waves_per_cu(const AttnArgs& a) { return waves_per_cu_of_this_build(a); }

hipError_t launch_attention_inner_paged(const AttnArgs& a, long long n_both_ll, int n_splits, const WindowSet& win,
                                        hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop) {
  if (!a.pages.table || !attention_inner_supported(a)) return hipErrorInvalidValue;
  const Launch L = {stream, ev_start, ev_stop};
  return for_widths(a, LaunchFn{a, (int)n_both_ll, n_splits, win, L});
}

#else

bool attention_inner_supported(const AttnArgs& a) {
  const int r = a.n_q_heads / a.n_kv_heads;
  // offsets inside one (batch, kv-head) slab are 32-bit in the kernel
  return a.k.form == kPerToken && a.v.form == kPerChannel && width_pair(a) >= 0 && r <= 8 &&
         (a.group == 32 || a.group == 64) && a.capacity * D <= (1LL << 31);
}

std::atomic<int> g_inner_variant{0};

int attention_inner_waves_per_cu(const AttnArgs& a) {
  if (a.pages.table) return attention_inner_paged_waves_per_cu(a);
  if (g_inner_variant.load(std::memory_order_relaxed) == 1 && attention_inner_f4_supported(a))
    return attention_inner_f4_waves_per_cu(a);
  return waves_per_cu_of_this_build(a);
}

hipError_t launch_attention_inner(const AttnArgs& a, long long n_both_ll, int n_splits, const WindowSet& win,
                                  hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop) {
  if (!attention_inner_supported(a)) return hipErrorInvalidValue;
  if (a.pages.table) return launch_attention_inner_paged(a, n_both_ll, n_splits, win, stream, ev_start, ev_stop);
  if (g_inner_variant.load(std::memory_order_relaxed) == 1 && attention_inner_f4_supported(a))
    return launch_attention_inner_f4(a, n_both_ll, n_splits, win, stream, ev_start, ev_stop);
  const Launch L = {stream, ev_start, ev_stop};
  return for_widths(a, LaunchFn{a, (int)n_both_ll, n_splits, win, L});
}

#endif

}  // namespace innerq
