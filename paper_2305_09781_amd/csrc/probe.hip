// Measurement aid, not part of the method: a plain read stream over a device buffer. Its rate on a buffer
// far larger than the caches is the practical ceiling any HBM-bound kernel of this library can be held
// against (the published peak is not reachable by a kernel that only reads).
#include "spec_internal.h"

namespace spec {

__global__ void __launch_bounds__(256) read_stream_kernel(const uint4* __restrict__ p, size_t n, uint4* sink) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  uint4 acc = {0, 0, 0, 0};
  for (; i + 3 * stride < n; i += 4 * stride) {   // four independent 16-byte loads in flight per thread
    const uint4 a = p[i], b = p[i + stride], c = p[i + 2 * stride], d = p[i + 3 * stride];
    acc.x ^= a.x ^ b.x ^ c.x ^ d.x; acc.y ^= a.y ^ b.y ^ c.y ^ d.y;
    acc.z ^= a.z ^ b.z ^ c.z ^ d.z; acc.w ^= a.w ^ b.w ^ c.w ^ d.w;
  }
  for (; i < n; i += stride) { const uint4 a = p[i]; acc.x ^= a.x; acc.y ^= a.y; acc.z ^= a.z; acc.w ^= a.w; }
  // the loads must not be optimised away; the condition practically never holds
  if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u && acc.z == 0x0fedcba9u && acc.w == 0x87654321u) sink[0] = acc;
}

hipError_t launch_read_stream(const void* buf, size_t bytes, void* sink, int workgroups, hipStream_t s) {
  hipLaunchKernelGGL(read_stream_kernel, dim3(workgroups), dim3(256), 0, s, (const uint4*)buf, bytes / 16, (uint4*)sink);
  return hipGetLastError();
}

}  // namespace spec
