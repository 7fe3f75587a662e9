// Comparison kernel: fused split-K decode attention over an OUTER-dimension-grouped cache
// (kind = INNERQ_KIND_OUTER: keys grouped along tokens per channel, values along channels per
// token -- the layout the paper compares against, Figure "inner_outer" (a)).
//
// Same skeleton as the inner-grouped and fp16 kernels (one wavefront per token range, 64-token
// tiles, register prefetch of the next tile, window wavefronts in the same launch, same merge).
// What differs is forced by the grouping: along the inner dimension of q.K^T every channel of a
// key row has its own scale and zero-point, so nothing factors out of the inner sum and every
// element is dequantised (Eq. asym_dequant) before it is multiplied; the packed key codes are
// token-minor, so the dequantised tile goes through LDS to reach the one-token-per-lane score
// pass.  Values are dequantised element by element on their way into the value pass.
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

__device__ inline float wave_max_o(float x) {
  for (int off = 32; off; off >>= 1) x = fmaxf(x, __shfl_xor(x, off));
  return x;
}
__device__ inline float wave_sum_o(float x) {
  for (int off = 32; off; off >>= 1) x += __shfl_xor(x, off);
  return x;
}
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

template <int BITS, int G, int NH4, bool ZK, bool ZV>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2, 2)))
attention_outer_kernel(AttnArgs a, int n_both, int n_splits, WindowSet win) {
  using Regs = OuterRegs<BITS, G>;
  constexpr int NH = NH4 * 4;
  constexpr int GPT = Regs::GPT, KC = Regs::KC, VC = Regs::VC, NG = Regs::NG;
  constexpr int FPW = 32 / BITS;
  constexpr int WPG = G / FPW;                         // words per channel of one key group
  constexpr uint32_t FMASK = (1u << BITS) - 1u;
  constexpr float HALFCODE = (float)(1 << (BITS - 1));
  constexpr int ROWB = D * BITS / 8;

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

  __shared__ __attribute__((aligned(16))) _Float16 qs[NH][D];
  __shared__ __attribute__((aligned(16))) _Float16 kt[TILE][KROW];      // dequantised keys, token-major
  __shared__ __attribute__((aligned(16))) float wp[TILE][NH];
  __shared__ __attribute__((aligned(16))) uint32_t vcode[TILE][ROWB / 4 + 1];   // packed value rows (padded)
  __shared__ __attribute__((aligned(16))) float2_t vsz[TILE][NG];       // (|S|, Zeff) of each value group

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
  float m_run[NH], l_run[NH], o[NH][8];
#pragma unroll
  for (int h = 0; h < NH; ++h) {
    m_run[h] = -INFINITY;
    l_run[h] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[h][e] = 0.f;
  }
  const int cg = lane & 15, tg = lane >> 4;

  Regs cur, nxt;
  if (t0 < t1) load_tile(t0, cur);
  for (int tile = t0; tile < t1; ++tile) {
    if (tile + 1 < t1) load_tile(tile + 1, nxt);       // in flight while this tile is computed
    __syncthreads();                                   // previous tile's readers of the LDS tiles are done

    // ---- dequantise this lane's two key channels of all 64 tokens into the token-major tile
#pragma unroll
    for (int gi = 0; gi < GPT; ++gi) {
      const uint32_t sp = cur.ks[gi];
      const float S0 = fabsf(half_lo(sp)), S1 = fabsf(half_hi(sp));
      float z0 = -S0 * HALFCODE, z1 = -S1 * HALFCODE;
      if constexpr (ZK) {
        const uint32_t zp = cur.kz[gi];
        z0 = ((sp >> 15) & 1u) ? half_lo(zp) : z0;
        z1 = (sp >> 31) ? half_hi(zp) : z1;
      }
#pragma unroll
      for (int wd = 0; wd < WPG; ++wd) {
        const uint32_t w0 = cur.kc[gi][wd / 4][wd % 4], w1 = cur.kc[gi][(WPG + wd) / 4][(WPG + wd) % 4];
#pragma unroll
        for (int e = 0; e < FPW; ++e) {
          const float x0 = S0 * (float)((w0 >> (e * BITS)) & FMASK) + z0;
          const float x1 = S1 * (float)((w1 >> (e * BITS)) & FMASK) + z1;
          half2_t hx;
          hx[0] = (_Float16)x0;
          hx[1] = (_Float16)x1;
          *reinterpret_cast<half2_t*>(&kt[gi * G + wd * FPW + e][2 * lane]) = hx;
        }
      }
    }
    // ---- stage this lane's packed value row and its group scales
#pragma unroll
    for (int i = 0; i < VC; ++i) {
      vcode[lane][4 * i + 0] = cur.vc[i].x;
      vcode[lane][4 * i + 1] = cur.vc[i].y;
      vcode[lane][4 * i + 2] = cur.vc[i].z;
      vcode[lane][4 * i + 3] = cur.vc[i].w;
    }
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const uint32_t sp = cur.vs[g / 2];
      const float sc = (g & 1) ? half_hi(sp) : half_lo(sp);
      const float S = fabsf(sc);
      float z = -S * HALFCODE;
      if constexpr (ZV) {
        const uint32_t zp = cur.vz[g / 2];
        const bool asym = (g & 1) ? (sp >> 31) : ((sp >> 15) & 1u);
        z = asym ? ((g & 1) ? half_hi(zp) : half_lo(zp)) : z;
      }
      vsz[lane][g] = float2_t{S, z};
    }
    __syncthreads();

    // ---- scores: lane = token (Eq. att:1)
    float s[NH];
#pragma unroll
    for (int h = 0; h < NH; ++h) s[h] = 0.f;
#pragma unroll 4
    for (int i = 0; i < D / 8; ++i) {
      const u32x4 kv = *reinterpret_cast<const u32x4*>(&kt[lane][i * 8]);
      const uint32_t kw[4] = {kv.x, kv.y, kv.z, kv.w};
#pragma unroll
      for (int h = 0; h < NH; ++h) {
        const u32x4 qv = *reinterpret_cast<const u32x4*>(&qs[h][i * 8]);
        const uint32_t qw[4] = {qv.x, qv.y, qv.z, qv.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const half2_t kk = __builtin_bit_cast(half2_t, kw[e]), qq = __builtin_bit_cast(half2_t, qw[e]);
          s[h] += (float)kk[0] * (float)qq[0];
          s[h] += (float)kk[1] * (float)qq[1];
        }
      }
    }
    // ---- running softmax (Eq. att:2)
    const bool valid = tile * TILE + lane <= last_row;
#pragma unroll
    for (int h = 0; h < NH; ++h) {
      const float sv = valid ? s[h] * c_log2 : -INFINITY;
      const float m_new = fmaxf(m_run[h], wave_max_o(sv));
      const float alpha = __builtin_amdgcn_exp2f(m_run[h] - m_new);
      const float p = __builtin_amdgcn_exp2f(sv - m_new);
      l_run[h] = l_run[h] * alpha + wave_sum_o(p);
      m_run[h] = m_new;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[h][e] *= alpha;
      wp[lane][h] = p;
    }
    __syncthreads();
    // ---- values: lane = 8 channels of tokens 4i + tg, dequantised on the way (Eq. att:3)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int j = 4 * i + tg;
      // the 8 fields of channels 8cg .. 8cg+7: 8*BITS bits at bit offset 8*cg*BITS of the row
      uint32_t bitsw;
      if constexpr (BITS == 2) bitsw = (vcode[j][cg / 2] >> ((cg & 1) * 16)) & 0xffffu;
      else bitsw = vcode[j][cg];
      const float2_t sz = vsz[j][(8 * cg) / G];
      float x[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = sz[0] * (float)((bitsw >> (e * BITS)) & FMASK) + sz[1];
#pragma unroll
      for (int n = 0; n < NH4; ++n) {
        const float4_t pj = *reinterpret_cast<const float4_t*>(&wp[j][n * 4]);
#pragma unroll
        for (int hh = 0; hh < 4; ++hh)
#pragma unroll
          for (int e = 0; e < 8; ++e) o[n * 4 + hh][e] += pj[hh] * x[e];
      }
    }
    cur = nxt;
  }

#pragma unroll
  for (int h = 0; h < NH; ++h)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
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
         a.capacity * D <= (1LL << 31);
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
