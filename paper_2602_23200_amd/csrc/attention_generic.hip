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
#include "merge.h"

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

__global__ void __launch_bounds__(64) attention_merge_kernel(AttnArgs a) {
  merge_head(a, blockIdx.x, threadIdx.x);
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
