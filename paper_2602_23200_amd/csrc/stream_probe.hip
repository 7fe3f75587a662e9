// A plain read-only streaming kernel: the practical ceiling of a pure HBM read of a given size
// on this device, measured next to the fused attention kernel (the paper's Section "Latency"
// compares kernels by latency only; a bandwidth target needs a yardstick that pays the same
// launch and ramp costs as the kernel it is compared with).
#include "innerq_dev.h"

namespace innerq {
namespace {

typedef uint32_t p_u32x4 __attribute__((ext_vector_type(4)));
constexpr int kUnroll = 4;

__global__ void __launch_bounds__(256) stream_read_kernel(const p_u32x4* __restrict__ p, size_t n, uint32_t* sink) {
  size_t i = (size_t)blockIdx.x * (256 * kUnroll) + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * (256 * kUnroll);
  uint32_t acc = 0;
  for (; i + (kUnroll - 1) * 256 < n; i += stride) {
    p_u32x4 v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) v[u] = __builtin_nontemporal_load(p + i + u * 256);
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < n; i += 256) {                              // ragged end of the last pass
    const p_u32x4 v = __builtin_nontemporal_load(p + i);
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  // the loads must not be optimised away; the store itself practically never happens
  if (acc == 0x9e3779b9u) sink[0] = acc;
}

}  // namespace

hipError_t launch_stream_read(const void* data, size_t bytes, uint32_t* sink, int n_blocks, hipStream_t stream,
                              hipEvent_t ev_start, hipEvent_t ev_stop) {
  const size_t n = bytes / 16;
  hipExtLaunchKernelGGL(stream_read_kernel, dim3((unsigned)n_blocks), dim3(256), 0, stream, ev_start, ev_stop, 0,
                        static_cast<const p_u32x4*>(data), n, sink);
  return hipGetLastError();
}

}  // namespace innerq
