// Plain streaming-read kernel: the practical HBM read ceiling the decode kernels are compared
// with in the bench (no gather, no arithmetic beyond an xor fold).
#include "seer_internal.h"

namespace seer {

__global__ __launch_bounds__(256) void seer_stream_read_kernel(const uint4* __restrict__ src, size_t n16,
                                                               uint4* sink) {
  const size_t stride = (size_t)gridDim.x * 256;
  size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  uint4 acc = make_uint4(0, 0, 0, 0);
  for (; idx + 7 * stride < n16; idx += 8 * stride) {
    uint4 r[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) r[u] = load_stream16(reinterpret_cast<const uint16_t*>(src + idx + u * stride));
#pragma unroll
    for (int u = 0; u < 8; ++u) { acc.x ^= r[u].x; acc.y ^= r[u].y; acc.z ^= r[u].z; acc.w ^= r[u].w; }
  }
  for (; idx < n16; idx += stride) {
    const uint4 r = load_stream16(reinterpret_cast<const uint16_t*>(src + idx));
    acc.x ^= r.x; acc.y ^= r.y; acc.z ^= r.z; acc.w ^= r.w;
  }
  // practically never true; keeps the loads alive
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u && acc.x == 0x7f4a7c15u) *sink = acc;
}

hipError_t launch_stream_read(const void* src, size_t bytes, void* sink, int wgs, hipStream_t s) {
  hipLaunchKernelGGL(seer_stream_read_kernel, dim3(wgs), dim3(256), 0, s, static_cast<const uint4*>(src),
                     bytes / 16, static_cast<uint4*>(sink));
  return hipGetLastError();
}

}  // namespace seer
