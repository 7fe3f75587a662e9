// Comparison kernel: the same fused split-K decode attention over an UNQUANTISED fp16 store
// (kind = INNERQ_KIND_FP16; the "Baseline (FP16)" rows of the paper's latency table).
// Same skeleton as the inner-grouped kernel: one wavefront streams a contiguous range of
// 64-token tiles of one (batch, kv-head) once and serves all query heads of that kv head,
// the window wavefronts ride in the same launch, partials go to the same merge kernel.
//
// Loads are 128-bit and fully coalesced (16 lanes cover one 256-byte row, four rows per
// instruction).  Keys pass through an LDS tile so that the score pass can run with one token
// per lane; values are consumed straight from registers (lane = 8 channels of every 4th token).
#include "innerq_dev.h"
#include "window_pass.h"

namespace innerq {
namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int D = kHeadDim;
constexpr int TILE = 64;
constexpr int KROW = D + 8;                 // padded LDS row (halves): 272 bytes

__device__ inline float wave_max_f(float x) {
  for (int off = 32; off; off >>= 1) x = fmaxf(x, __shfl_xor(x, off));
  return x;
}
__device__ inline float wave_sum_f(float x) {
  for (int off = 32; off; off >>= 1) x += __shfl_xor(x, off);
  return x;
}

template <int NH4>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2, 2))) attention_fp16_kernel(AttnArgs a, int n_rows, int n_splits, WindowSet win) {
  constexpr int NH = NH4 * 4;
  const int lane = threadIdx.x;
  const long long bh = blockIdx.y;
  const int b = (int)(bh / a.n_kv_heads), hk = (int)(bh % a.n_kv_heads);
  const int r = a.n_q_heads / a.n_kv_heads;

  if ((int)blockIdx.x < win.n_chunks) {
    window_pass<NH4, 4, 32, false, false>(a, bh, win.na, win.b0, win.nb, (int)blockIdx.x, win.n_chunks, n_splits + (int)blockIdx.x);
    return;
  }
  const int n_tiles = (n_rows + TILE - 1) / TILE;
  const int base_t = n_tiles / n_splits, rem_t = n_tiles % n_splits;
  const int s_idx = (int)blockIdx.x - win.n_chunks;
  const int t0 = s_idx * base_t + (s_idx < rem_t ? s_idx : rem_t);
  const int t1 = t0 + base_t + (s_idx < rem_t ? 1 : 0);

  __shared__ __attribute__((aligned(16))) _Float16 qs[NH][D];
  __shared__ __attribute__((aligned(16))) _Float16 kt[TILE][KROW];
  __shared__ __attribute__((aligned(16))) float wp[TILE][NH];

  for (int i = lane; i < NH * D; i += 64) {
    const int h = i / D, c = i % D;
    float qv = 0.f;
    if (h < r) {
      const __half qh = a.q[((long long)b * a.n_q_heads + hk * r + h) * D + c];
      qv = a.q_scale ? __half2float(scaled_half(__half2float(qh), a.q_scale[hk * D + c])) : __half2float(qh);
    }
    qs[h][c] = (_Float16)qv;
  }

  const __half* kbase = reinterpret_cast<const __half*>(a.k.codes) + bh * a.capacity * D;
  const __half* vbase = reinterpret_cast<const __half*>(a.v.codes) + bh * a.capacity * D;
  const int cg = lane & 15, tg = lane >> 4;            // load pattern: 16 lanes per row, 4 rows per instruction
  const int last_row = n_rows - 1;

  auto load_rows = [&](const __half* base, int tile, u32x4 (&buf)[16]) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      int row = tile * TILE + 4 * i + tg;
      row = row > last_row ? last_row : row;
      buf[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + (uint32_t)row * D + 8 * cg));
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

  u32x4 kbuf[16], vbuf[16];
  if (t0 < t1) load_rows(kbase, t0, kbuf);
  for (int tile = t0; tile < t1; ++tile) {
    __syncthreads();                                   // previous tile's readers of kt / wp are done
#pragma unroll
    for (int i = 0; i < 16; ++i) *reinterpret_cast<u32x4*>(&kt[4 * i + tg][8 * cg]) = kbuf[i];
    load_rows(vbase, tile, vbuf);                      // in flight during the score pass
    if (tile + 1 < t1) load_rows(kbase, tile + 1, kbuf);
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
      const float m_new = fmaxf(m_run[h], wave_max_f(sv));
      const float alpha = __builtin_amdgcn_exp2f(m_run[h] - m_new);
      const float p = __builtin_amdgcn_exp2f(sv - m_new);
      l_run[h] = l_run[h] * alpha + wave_sum_f(p);
      m_run[h] = m_new;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[h][e] *= alpha;
      wp[lane][h] = p;
    }
    __syncthreads();
    // ---- values: lane = 8 channels of tokens 4i + tg (Eq. att:3)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const uint32_t vw[4] = {vbuf[i].x, vbuf[i].y, vbuf[i].z, vbuf[i].w};
      float x[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const half2_t hh = __builtin_bit_cast(half2_t, vw[e]);
        x[2 * e] = (float)hh[0];
        x[2 * e + 1] = (float)hh[1];
      }
#pragma unroll
      for (int n = 0; n < NH4; ++n) {
        const float4_t pj = *reinterpret_cast<const float4_t*>(&wp[4 * i + tg][n * 4]);
#pragma unroll
        for (int hh = 0; hh < 4; ++hh)
#pragma unroll
          for (int e = 0; e < 8; ++e) o[n * 4 + hh][e] += pj[hh] * x[e];
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

}  // namespace

bool attention_fp16_supported(const AttnArgs& a) {
  const int r = a.n_q_heads / a.n_kv_heads;
  return a.k.form == kFp16 && a.v.form == kFp16 && r <= 8 && a.capacity * D <= (1LL << 31) && !a.pages.table;
}

int attention_fp16_waves_per_cu(const AttnArgs& a) {
  static CachedInt cache[2];
  const int r = a.n_q_heads / a.n_kv_heads;
  return cache[r > 4].get([&] {
    int n = 0;
    const hipError_t e = r <= 4 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, attention_fp16_kernel<1>, 64, 0)
                                : hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, attention_fp16_kernel<2>, 64, 0);
    return (e == hipSuccess && n > 0) ? n : 4;
  });
}

hipError_t launch_attention_fp16(const AttnArgs& a, long long n_rows, int n_splits, const WindowSet& win,
                                 hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop) {
  const int r = a.n_q_heads / a.n_kv_heads;
  dim3 grid((unsigned)(n_splits + win.n_chunks), (unsigned)(a.batch * a.n_kv_heads));
  if (r <= 4)
    hipExtLaunchKernelGGL(attention_fp16_kernel<1>, grid, dim3(64), 0, stream, ev_start, ev_stop, 0, a, (int)n_rows,
                          n_splits, win);
  else
    hipExtLaunchKernelGGL(attention_fp16_kernel<2>, grid, dim3(64), 0, stream, ev_start, ev_stop, 0, a, (int)n_rows,
                          n_splits, win);
  return hipGetLastError();
}

}  // namespace innerq
