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

// Element (token t, channel c) of one tensor of sequence-head bh, decoded per Eq. hybrid_dequant.
__device__ inline float fetch_element(const TensorView& tv, const AttnArgs& a, long long bh, long long t, int c) {
  constexpr int D = kHeadDim;
  if (t < tv.n_sink) return __half2float(tv.sink[(bh * a.w_sink + t) * D + c]);
  const long long row = t - a.w_sink;
  if (row >= tv.n_quant) return __half2float(tv.ring[(bh * tv.slots + (t % tv.slots)) * D + c]);
  if (tv.form == kFp16) return __half2float(reinterpret_cast<const __half*>(tv.codes)[(bh * a.capacity + row) * D + c]);
  const int bits = a.bits, G = a.group;
  const unsigned mask = (1u << bits) - 1u;
  long long si;
  unsigned field;
  if (tv.form == kPerToken) {
    const unsigned byte = tv.codes[((bh * a.capacity + row) * D * bits) / 8 + (c * bits) / 8];
    field = (byte >> ((c * bits) % 8)) & mask;
    si = (bh * a.capacity + row) * (D / G) + c / G;
  } else {
    const long long tg = row / G;
    const int j = (int)(row % G);
    si = (bh * (a.capacity / G) + tg) * D + c;
    const unsigned byte = tv.codes[si * ((G * bits) / 8) + (j * bits) / 8];
    field = (byte >> ((j * bits) % 8)) & mask;
  }
  const float s = __half2float(tv.scales[si]);
  const bool asym = __float_as_uint(s) >> 31;
  const float S = fabsf(s);
  return asym ? S * (float)field + __half2float(tv.zeros[si]) : S * (float)((int)field - (1 << (bits - 1)));
}

// fp16 row of token t if that tensor keeps it in fp16 (sink window, recent ring, fp16 store), else null.
__device__ inline const __half* fp16_row(const TensorView& tv, const AttnArgs& a, long long bh, long long t) {
  constexpr int D = kHeadDim;
  if (t < tv.n_sink) return tv.sink + (bh * a.w_sink + t) * D;
  const long long row = t - a.w_sink;
  if (row >= tv.n_quant) return tv.ring + (bh * tv.slots + (t % tv.slots)) * D;
  if (tv.form == kFp16) return reinterpret_cast<const __half*>(tv.codes) + (bh * a.capacity + row) * D;
  return nullptr;
}

__device__ inline float window_wave_max(float x) {
  for (int off = 32; off; off >>= 1) x = fmaxf(x, __shfl_xor(x, off));
  return x;
}
__device__ inline float window_wave_sum(float x) {
  for (int off = 32; off; off >>= 1) x += __shfl_xor(x, off);
  return x;
}

// Window token set: virtual index v in [0, na + nb) -> token v (v < na) or b0 + v - na.
// Chunk `chunk` of `n_chunks` equal chunks of that set; partial written to `slot`.
template <int NH4>
__device__ inline void window_pass(const AttnArgs& a, long long bh, long long na, long long b0, long long nb,
                                   int chunk, int n_chunks, int slot) {
  constexpr int D = kHeadDim;
  constexpr int NH = NH4 * 4;
  const int lane = threadIdx.x & 63;
  const int b = (int)(bh / a.n_kv_heads), hk = (int)(bh % a.n_kv_heads);
  const int r = a.n_q_heads / a.n_kv_heads;
  const long long total = na + nb;
  const long long chunk_len = (total + n_chunks - 1) / n_chunks;
  const long long v0 = chunk * chunk_len;
  const long long v1 = v0 + chunk_len < total ? v0 + chunk_len : total;

  __shared__ __attribute__((aligned(16))) _Float16 wq[NH][D];       // query, fp16 (exact)
  __shared__ __attribute__((aligned(16))) float wp[64][NH];         // probabilities of the current 64 tokens

  for (int i = lane; i < NH * D; i += 64) {
    const int h = i / D, c = i % D;
    float qv = 0.f;
    if (h < r) {
      const __half qh = a.q[((long long)b * a.n_q_heads + hk * r + h) * D + c];
      qv = a.q_scale ? __half2float(__float2half_rn(__half2float(qh) * a.q_scale[hk * D + c])) : __half2float(qh);
    }
    wq[h][c] = (_Float16)qv;
  }
  __syncthreads();

  const float c_log2 = 0.08838834764831845f * 1.4426950408889634f;    // log2(e) / sqrt(d)
  float m_run[NH], l_run[NH], o[NH][8];
#pragma unroll
  for (int h = 0; h < NH; ++h) {
    m_run[h] = -INFINITY;
    l_run[h] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[h][e] = 0.f;
  }

  const int bits = a.bits, G = a.group;
  const unsigned fmask = (1u << bits) - 1u;
  const float halfcode = (float)(1 << (bits - 1));

  for (long long base = v0; base < v1; base += 64) {
    // ---- scores: lane = token
    const long long v = base + lane;
    const bool valid = v < v1;
    const long long t = valid ? (v < na ? v : b0 + (v - na)) : 0;
    float s[NH];
#pragma unroll
    for (int h = 0; h < NH; ++h) s[h] = 0.f;
    if (valid) {
      const __half* krow = fp16_row(a.k, a, bh, t);
      if (krow) {
#pragma unroll 4
        for (int i = 0; i < D / 8; ++i) {
          const w_u32x4 kv = *reinterpret_cast<const w_u32x4*>(krow + i * 8);
          const uint32_t kw[4] = {kv.x, kv.y, kv.z, kv.w};
#pragma unroll
          for (int h = 0; h < NH; ++h) {
            const w_u32x4 qv = *reinterpret_cast<const w_u32x4*>(&wq[h][i * 8]);
            const uint32_t qw[4] = {qv.x, qv.y, qv.z, qv.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const w_half2_t kk = __builtin_bit_cast(w_half2_t, kw[e]), qq = __builtin_bit_cast(w_half2_t, qw[e]);
              s[h] += (float)kk[0] * (float)qq[0];
              s[h] += (float)kk[1] * (float)qq[1];
            }
          }
        }
      } else if (a.k.form == kPerToken) {
        // a key that is already quantised while its value still waits in the recent ring:
        // decode the packed row group by group (Eq. hybrid_dequant)
        const long long row = t - a.w_sink;
        const uint32_t* rowp =
            reinterpret_cast<const uint32_t*>(a.k.codes + ((bh * a.capacity + row) * D * bits) / 8);
        const int fpw = 32 / bits, wpg = G / fpw;
        for (int g = 0; g < D / G; ++g) {
          const long long si = (bh * a.capacity + row) * (D / G) + g;
          const float sc = __half2float(a.k.scales[si]);
          const float S = fabsf(sc);
          const float zeff = (__float_as_uint(sc) >> 31) ? __half2float(a.k.zeros[si]) : -S * halfcode;
          for (int wd = 0; wd < wpg; ++wd) {
            const uint32_t w = rowp[g * wpg + wd];
            for (int e = 0; e < fpw; ++e) {
              const float x = S * (float)((w >> (e * bits)) & fmask) + zeff;
              const int c = (g * wpg + wd) * fpw + e;
#pragma unroll
              for (int h = 0; h < NH; ++h) s[h] += (float)wq[h][c] * x;
            }
          }
        }
      } else {
        for (int c = 0; c < D; ++c) {
          const float kx = fetch_element(a.k, a, bh, t, c);
#pragma unroll
          for (int h = 0; h < NH; ++h) s[h] += (float)wq[h][c] * kx;
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
      const float p = __builtin_amdgcn_exp2f(sv - m_new);
      l_run[h] = l_run[h] * alpha + window_wave_sum(p);
      m_run[h] = m_new;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[h][e] *= alpha;
      wp[lane][h] = p;
    }
    __syncthreads();
    // ---- values: 16 lanes share one token row (8 channels = 16 bytes each), 4 rows per load
    // instruction, every load of the tile in flight at once; lane keeps o[head][8 channels] of
    // the tokens (4k + lane/16) and the four lane groups are summed at the end.
    const int n_here = (int)(v1 - base < 64 ? v1 - base : 64);
    const int cg = lane & 15, tg = lane >> 4;
    for (int k0 = 0; k0 < 16 && 4 * k0 < n_here; k0 += 8) {      // two batches of 8 rows per lane
    float x[8][8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int j = 4 * (k0 + k) + tg;
#pragma unroll
      for (int e = 0; e < 8; ++e) x[k][e] = 0.f;
      if (j < n_here) {
        const long long vj = base + j;
        const long long tj = vj < na ? vj : b0 + (vj - na);
        const __half* vrow = fp16_row(a.v, a, bh, tj);
        if (vrow) {
          const w_u32x4 pr = *reinterpret_cast<const w_u32x4*>(vrow + 8 * cg);
          const uint32_t pw[4] = {pr.x, pr.y, pr.z, pr.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const w_half2_t hh = __builtin_bit_cast(w_half2_t, pw[e]);
            x[k][2 * e] = (float)hh[0];
            x[k][2 * e + 1] = (float)hh[1];
          }
        } else if (a.v.form == kPerToken) {
          // a value quantised per token while its key still waits in the ring (outer grouping)
          const long long row = tj - a.w_sink;
          const int c0 = 8 * cg;
          const uint8_t* cp = a.v.codes + ((bh * a.capacity + row) * D * bits) / 8 + (c0 * bits) / 8;
          const unsigned wbits = bits == 2 ? (unsigned)cp[0] | ((unsigned)cp[1] << 8)
                                           : *reinterpret_cast<const uint32_t*>(cp);
          const long long si = (bh * a.capacity + row) * (D / G) + c0 / G;
          const float sc = __half2float(a.v.scales[si]);
          const float S = fabsf(sc);
          const float zeff = (__float_as_uint(sc) >> 31) ? __half2float(a.v.zeros[si]) : -S * halfcode;
#pragma unroll
          for (int e = 0; e < 8; ++e) x[k][e] = S * (float)((wbits >> (e * bits)) & fmask) + zeff;
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e) x[k][e] = fetch_element(a.v, a, bh, tj, 8 * cg + e);
        }
      }
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int j = 4 * (k0 + k) + tg;                    // rows past n_here carry x = 0
#pragma unroll
      for (int n = 0; n < NH4; ++n) {
        const w_float4_t pj = *reinterpret_cast<const w_float4_t*>(&wp[j][n * 4]);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int e = 0; e < 8; ++e) o[n * 4 + i][e] += pj[i] * x[k][e];
      }
    }
    }
  }

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

}  // namespace innerq
