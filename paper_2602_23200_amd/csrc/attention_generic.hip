// Generic partial attention and the split-K merge.
//
// attention_generic_kernel decodes the cache element by element (any grouping
// form, any window) and is used for the fp16 windows, for the few tokens whose
// key is quantised while their value still sits in the recent ring (or the
// reverse), and as the fallback for shapes the fused kernels do not cover.
// attention_merge_kernel joins all partial results by log-sum-exp: the
// quantised part and the window parts are concatenated before the softmax is
// normalised (Eq. att:1-3; Figure "quantization_overall").
#include "innerq_dev.h"
#include "window_pass.h"

namespace innerq {
namespace {

constexpr int D = kHeadDim;
constexpr int RT = kHeadTile;
constexpr int TILE = 64;          // tokens per inner tile

__device__ inline float h2f(__half h) { return __half2float(h); }

__device__ inline float fetch(const TensorView& tv, const AttnArgs& a, long long bh, long long t, int c) {
  return fetch_element(tv, a, bh, t, c);
}

__global__ void __launch_bounds__(256) attention_generic_kernel(AttnArgs a, long long a0, long long a1,
                                                                long long b0, long long b1, int n_chunks,
                                                                int first_slot) {
  const int tid = threadIdx.x;
  const long long bh = blockIdx.y;                      // b * Hk + hk
  const int r = a.n_q_heads / a.n_kv_heads;
  const int b = (int)(bh / a.n_kv_heads), hk = (int)(bh % a.n_kv_heads);
  const int h0 = blockIdx.z * RT;                       // first query head (within the kv head) of this pass
  const int nh = min(RT, r - h0);
  const long long na = a1 - a0, total = na + (b1 - b0);
  const long long chunk_len = (total + n_chunks - 1) / n_chunks;
  const long long v0 = (long long)blockIdx.x * chunk_len;
  const long long v1 = min(total, v0 + chunk_len);

  __shared__ float q_s[RT][D];
  __shared__ float s_s[RT][TILE];
  __shared__ float alpha_s[RT];
  __shared__ float o_s[RT][D];

  for (int i = tid; i < RT * D; i += 256) {
    const int h = i / D, c = i % D;
    float qv = 0.f;
    if (h < nh) {
      const __half qh = a.q[((long long)b * a.n_q_heads + hk * r + h0 + h) * D + c];
      qv = a.q_scale ? h2f(scaled_half(h2f(qh), a.q_scale[hk * D + c])) : h2f(qh);
    }
    q_s[h][c] = qv;
  }
  __syncthreads();

  const float sm_scale = 0.08838834764831845f;          // 1 / sqrt(128)
  const int tok = tid >> 2, part = tid & 3;             // score phase: 4 threads per token
  const int vc = tid & (D - 1), vhalf = tid >> 7;       // value phase: 2 threads per channel
  const int wave = tid >> 6, lane = tid & 63;
  float m_run = -INFINITY, l_run = 0.f;                 // running max / sum of head `wave`
  float o[RT];
#pragma unroll
  for (int h = 0; h < RT; ++h) o[h] = 0.f;

  for (long long base = v0; base < v1; base += TILE) {
    // ---- scores of up to TILE tokens (Eq. att:1, scaled by 1/sqrt(d))
    {
      const long long v = base + tok;
      const bool valid = v < v1;
      float acc[RT];
#pragma unroll
      for (int h = 0; h < RT; ++h) acc[h] = 0.f;
      if (valid) {
        const long long t = v < na ? a0 + v : b0 + (v - na);
        for (int c = part * 32; c < part * 32 + 32; ++c) {
          const float kx = fetch(a.k, a, bh, t, c);
#pragma unroll
          for (int h = 0; h < RT; ++h) acc[h] += q_s[h][c] * kx;
        }
      }
#pragma unroll
      for (int h = 0; h < RT; ++h) {
        acc[h] += __shfl_xor(acc[h], 1);
        acc[h] += __shfl_xor(acc[h], 2);
      }
      if (part == 0) {
#pragma unroll
        for (int h = 0; h < RT; ++h) s_s[h][tok] = valid ? acc[h] * sm_scale : -INFINITY;
      }
    }
    __syncthreads();
    // ---- running softmax of head `wave` (Eq. att:2), one token per lane
    {
      const float s = s_s[wave][lane];
      float mx = s;
      for (int off = 32; off; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
      const float m_new = fmaxf(m_run, mx);
      const float p = expf(s - m_new);
      float ps = p;
      for (int off = 32; off; off >>= 1) ps += __shfl_xor(ps, off);
      const float alpha = expf(m_run - m_new);           // 0 on the first tile (m_run = -inf)
      l_run = l_run * alpha + ps;
      m_run = m_new;
      s_s[wave][lane] = p;
      if (lane == 0) alpha_s[wave] = alpha;
    }
    __syncthreads();
    // ---- weighted sum of values (Eq. att:3): thread = (channel, half of the tile)
    {
#pragma unroll
      for (int h = 0; h < RT; ++h) o[h] *= alpha_s[h];
      for (int j = vhalf * (TILE / 2); j < (vhalf + 1) * (TILE / 2); ++j) {
        const long long v = base + j;
        if (v >= v1) break;
        const long long t = v < na ? a0 + v : b0 + (v - na);
        const float vx = fetch(a.v, a, bh, t, vc);
#pragma unroll
        for (int h = 0; h < RT; ++h) o[h] += s_s[h][j] * vx;
      }
    }
    __syncthreads();
  }

  // ---- combine the two token halves and write the partial (m, l, o) of each head
  if (vhalf == 1) {
#pragma unroll
    for (int h = 0; h < RT; ++h) o_s[h][vc] = o[h];
  }
  __syncthreads();
  const int slot = first_slot + blockIdx.x;
  if (vhalf == 0) {
#pragma unroll
    for (int h = 0; h < RT; ++h) {
      if (h < nh) {
        const long long bhq = (long long)b * a.n_q_heads + hk * r + h0 + h;
        a.ws_o[(bhq * a.n_partials + slot) * D + vc] = o[h] + o_s[h][vc];
      }
    }
  }
  if (lane == 0 && wave < nh) {
    const long long bhq = (long long)b * a.n_q_heads + hk * r + h0 + wave;
    a.ws_ml[(bhq * a.n_partials + slot) * 2 + 0] = m_run;
    a.ws_ml[(bhq * a.n_partials + slot) * 2 + 1] = l_run;
  }
}

// One batch of NB partial outputs of a 64-partial chunk: every load is issued before the weights
// (which come from a separate, concurrent load) are needed.  Indices past the end re-read the last
// partial with weight zero.
template <int NB>
struct MergeBatch {
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
      n0 += w * ov[k].x;
      n1 += w * ov[k].y;
    }
  }
};

// out[b][hq][:] = sum_p w_p o_p / sum_p w_p l_p,  w_p = exp(m_p - max_p m_p).
// One wavefront per query head, a lane per channel pair; the partial index is wave-uniform.
// The partial outputs do not depend on the weights, so the loads of up to 64 of them go out
// together with the loads of (m, l): one memory round trip for the usual 30 to 50 partials.
__global__ void __launch_bounds__(64) attention_merge_kernel(AttnArgs a) {
  const long long bhq = blockIdx.x;
  const int lane = threadIdx.x;
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
      w_l = mlv.x == -INFINITY ? 0.f : __expf(mlv.x - M);           // an empty partial has m = -inf
      l_l = mlv.y;
    }
    den += window_wave_sum(w_l * l_l);
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

}  // namespace

hipError_t launch_attention_generic(const AttnArgs& a, long long a0, long long a1, long long b0, long long b1,
                                    int n_chunks, int first_slot, hipStream_t stream) {
  const int r = a.n_q_heads / a.n_kv_heads;
  dim3 grid((unsigned)n_chunks, (unsigned)(a.batch * a.n_kv_heads), (unsigned)((r + RT - 1) / RT));
  attention_generic_kernel<<<grid, 256, 0, stream>>>(a, a0, a1, b0, b1, n_chunks, first_slot);
  return hipGetLastError();
}

hipError_t launch_attention_merge(const AttnArgs& a, hipStream_t stream) {
  attention_merge_kernel<<<(unsigned)(a.batch * a.n_q_heads), 64, 0, stream>>>(a);
  return hipGetLastError();
}

}  // namespace innerq
