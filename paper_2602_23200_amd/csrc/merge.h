// Log-sum-exp merge of the split-K partial results of one query head (Eq. att:2 over the
// concatenation of the quantised range and the windows, Figure "quantization_overall"), as a
// device function so that it can ride in more than one launch.
#pragma once

#include "innerq_dev.h"
#include "window_pass.h"

namespace innerq {

// One batch of NB partial outputs of a 64-partial chunk: every load is issued before the weights
// (which come from a separate, concurrent load) are needed.  Indices past the end re-read the last
// partial with weight zero.
template <int NB>
struct MergeBatch {
  static constexpr int D = kHeadDim;
  float2 ov[NB];
  __device__ __forceinline__ void load(const float* po, int first, int n) {
#pragma unroll
    for (int k = 0; k < NB; ++k) {
      const int pp = k < n ? k : n - 1;
      ov[k] = *reinterpret_cast<const float2*>(po + (long long)(first + pp) * D);
    }
  }
  __device__ __forceinline__ void add(float w_l, int n, float& n0, float& n1) const {
#pragma unroll
    for (int k = 0; k < NB; ++k) {
      float w = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, w_l), k));
      w = k < n ? w : 0.f;
      n0 = __builtin_fmaf(w, ov[k].x, n0);          // explicit: the same rounding whatever the contraction setting
      n1 = __builtin_fmaf(w, ov[k].y, n1);
    }
  }
};

// out[b][hq][:] = sum_p w_p o_p / sum_p w_p l_p,  w_p = exp(m_p - max_p m_p).
// One wavefront per query head, a lane per channel pair; the partial index is wave-uniform.
// The partial outputs do not depend on the weights, so the loads of up to 64 of them go out
// together with the loads of (m, l): one memory round trip for the usual 30 to 50 partials.
__device__ inline void merge_head(const AttnArgs& a, long long bhq, int lane) {
  constexpr int D = kHeadDim;
  const int P = a.n_partials;
  const float* ml = a.ws_ml + bhq * P * 2;
  const float* po = a.ws_o + bhq * P * D + 2 * lane;
  float n0 = 0.f, n1 = 0.f, den = 0.f;
  // (m, l) of partial 64 i + lane, for the first two chunks (the rest is re-read below)
  float2 mlv0 = {-INFINITY, 0.f}, mlv1 = {-INFINITY, 0.f};
  if (lane < P) mlv0 = *reinterpret_cast<const float2*>(ml + 2 * lane);
  if (64 + lane < P) mlv1 = *reinterpret_cast<const float2*>(ml + 2 * (64 + lane));
  MergeBatch<32> first;                                  // partials 0 .. 31 of the first chunk
  MergeBatch<16> second;                                 // partials 32 .. 47
  const int n_first = P < 32 ? P : 32, n_second = P <= 32 ? 0 : (P < 48 ? P - 32 : 16);
  first.load(po, 0, n_first);
  if (n_second > 0) second.load(po, 32, n_second);
  float mloc = fmaxf(mlv0.x, mlv1.x);
  for (int p = 128 + lane; p < P; p += 64) mloc = fmaxf(mloc, ml[2 * p]);
  const float M = window_wave_max(mloc);
  for (int base = 0; base < P; base += 64) {
    const int p_l = base + lane;
    float2 mlv = base == 0 ? mlv0 : mlv1;
    if (base >= 128 && p_l < P) mlv = *reinterpret_cast<const float2*>(ml + 2 * p_l);
    float w_l = 0.f, l_l = 0.f;
    if (p_l < P) {
      w_l = mlv.x == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((mlv.x - M) * 1.4426950408889634f);           // an empty partial has m = -inf
      l_l = mlv.y;
    }
    float wl = w_l * l_l;
    asm("" : "+v"(wl));                                 // keeps the product out of a fused add in the reduction
    den += window_wave_sum(wl);
    const int n = P - base < 64 ? P - base : 64;
    int p0 = 0;
    if (base == 0) {
      first.add(w_l, n_first, n0, n1);
      if (n_second > 0) {
        const float w_s = __shfl(w_l, (lane + 32) & 63);  // weight of partial 32 + k in lane k
        second.add(w_s, n_second, n0, n1);
      }
      p0 = 48;
    }
    for (; p0 < n; p0 += 16) {
      MergeBatch<16> more;
      more.load(po, base + p0, n - p0 < 16 ? n - p0 : 16);
      const float w_s = __shfl(w_l, (lane + p0) & 63);
      more.add(w_s, n - p0 < 16 ? n - p0 : 16, n0, n1);
    }
  }
  const float inv = 1.0f / den;
  if (a.out_is_fp32) {
    float2 r;
    r.x = n0 * inv;
    r.y = n1 * inv;
    *reinterpret_cast<float2*>(reinterpret_cast<float*>(a.out) + bhq * D + 2 * lane) = r;
  } else {
    __half2 r = __floats2half2_rn(n0 * inv, n1 * inv);
    *reinterpret_cast<__half2*>(reinterpret_cast<__half*>(a.out) + bhq * D + 2 * lane) = r;
  }
}


}  // namespace innerq
