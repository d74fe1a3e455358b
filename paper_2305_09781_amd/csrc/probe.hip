// Measurement aid, not part of the method: a plain read stream over a device buffer. Its rate on a buffer
// far larger than the caches is the practical ceiling any HBM-bound kernel of this library can be held
// against (the published peak is not reachable by a kernel that only reads).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spec_probe.h"

namespace {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

// Every workgroup reads one contiguous piece, eight independent non-temporal 16-byte loads in flight per
// thread: the fastest read-only shape found on this machine (a grid-stride loop of plain loads is 15-25 % slower).
__global__ void __launch_bounds__(256) read_stream_kernel(const u32x4* __restrict__ p, size_t n, u32x4* sink) {
  constexpr int INF = 8;
  const size_t per = (n + gridDim.x - 1) / gridDim.x;
  const size_t lo = per * blockIdx.x, hi = lo + per < n ? lo + per : n;
  u32x4 acc = {0, 0, 0, 0};
  size_t i = lo + threadIdx.x;
  for (; i + (INF - 1) * 256 < hi; i += INF * 256) {
    u32x4 v[INF];
#pragma unroll
    for (int j = 0; j < INF; ++j) v[j] = __builtin_nontemporal_load(p + i + j * 256);
#pragma unroll
    for (int j = 0; j < INF; ++j) acc ^= v[j];
  }
  for (; i < hi; i += 256) acc ^= __builtin_nontemporal_load(p + i);
  // the loads must not be optimised away; the condition practically never holds
  if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u && acc.z == 0x0fedcba9u && acc.w == 0x87654321u) sink[0] = acc;
}

}  // namespace

extern "C" int spec_probe_read_stream(const void* buf, size_t bytes, void* sink, void* hip_stream) {
  if (!buf || !sink || bytes < 16 || (reinterpret_cast<uintptr_t>(buf) & 15u) || (reinterpret_cast<uintptr_t>(sink) & 15u))
    return -1;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
    cus = 256;
  // enough workgroups to fill every compute unit several times over
  hipLaunchKernelGGL(read_stream_kernel, dim3(cus * 8), dim3(256), 0, (hipStream_t)hip_stream, (const u32x4*)buf,
                     bytes / 16, (u32x4*)sink);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}
