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

// The memory requests of one fused append + attention launch on bf16 rows of 128 elements, and nothing else:
// one workgroup per (request, head) pair streams the pair's K and V rows [0, P + N) through a ring of four
// 32-key LDS stages with direct global->LDS loads (three stages ahead, two LDS barriers per stage, like the
// 32-query attention kernel), optionally reads the queries first, takes the last N rows from k_new / v_new,
// writes those rows to the cache from LDS, and writes N output rows at the end. No arithmetic: what it takes
// is what the traffic alone takes in that access pattern.
constexpr int TR_ROW = 256;                 // bytes per row (128 bf16)
constexpr int TR_SK = 32;                   // keys per stage
constexpr int TR_MAT = TR_SK * TR_ROW;      // K (or V) part of a stage
constexpr int TR_STAGE = 2 * TR_MAT;
constexpr int TR_NST = 4, TR_AHEAD = 3, TR_LPS = 4;

__device__ __forceinline__ void tr_load_to_lds(const unsigned char* src, unsigned lds_dst) {
  // 16 bytes per lane to LDS address lds_dst + 16 * lane (lds_dst wave-uniform), non-temporal
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt" ::"v"(src), "s"(lds_dst) : "memory");
}
template <int N>
__device__ __forceinline__ void tr_wait_but() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
__device__ __forceinline__ void tr_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

__global__ void __launch_bounds__(256, 2) attention_traffic_kernel(unsigned char* kc, unsigned char* vc, const unsigned char* q,
                                                                   const unsigned char* kn, const unsigned char* vn,
                                                                   unsigned char* out, int H, int N, int P, int S_cap,
                                                                   int flags) {
  __shared__ __attribute__((aligned(1024))) unsigned char ring[TR_NST * TR_STAGE];
  const int t = threadIdx.x, lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const unsigned ring_lds = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)ring;
  const unsigned wave_lds = ring_lds + wave * 1024;
  const long pair = blockIdx.x;                    // b * H + h
  const long b = pair / H, h = pair % H;
  const int len = P + N, last = len - 1;
  const int n_st = (len + TR_SK - 1) / TR_SK;
  const unsigned char* kb = kc + pair * S_cap * TR_ROW;
  const unsigned char* vb = vc + pair * S_cap * TR_ROW;
  const long new_row = (long)H * TR_ROW;           // [B, N, H, 128]: rows of one (request, head) are H rows apart
  const long new_base = (b * N * H + h) * TR_ROW;
  const int ld_row = t >> 4, ld_col = (t & 15) * 16;
  const bool want_q = flags & SPEC_PROBE_TRAFFIC_QUERIES, want_new = flags & SPEC_PROBE_TRAFFIC_NEW_ROWS,
             want_append = flags & SPEC_PROBE_TRAFFIC_APPEND, want_out = flags & SPEC_PROBE_TRAFFIC_OUTPUTS;
  auto request = [&](int slot, int st) {
    const unsigned dst = wave_lds + slot * TR_STAGE;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int row = min(st * TR_SK + ld_row + 16 * j, last);   // rows past the end repeat the last row
      const bool from_new = want_new && row >= P;
      const long in_cache = (long)row * TR_ROW, in_new = new_base + (long)(row - P) * new_row;
      tr_load_to_lds((from_new ? kn + in_new : kb + in_cache) + ld_col, dst + j * 4096);
      tr_load_to_lds((from_new ? vn + in_new : vb + in_cache) + ld_col, dst + TR_MAT + j * 4096);
    }
  };
#pragma unroll
  for (int s = 0; s < TR_AHEAD; ++s)
    if (s < n_st) request(s, s);
  if (want_q) {
    const int node = min(32 * wave + (lane & 31), N - 1), hh = lane >> 5;
    u32x4 qr[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      qr[ks] = *(const u32x4*)(q + new_base + (long)node * new_row + ks * 32 + hh * 16);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) asm volatile("" ::"v"(qr[ks]));
  }
  int slot = 0;
#pragma nounroll
  for (int i = 0; i < n_st; ++i) {
    tr_barrier();   // everybody is done with stage i - 1: its slot is free
    int ns = slot + TR_AHEAD;
    if (ns >= TR_NST) ns -= TR_NST;
    if (i + TR_AHEAD < n_st) request(ns, i + TR_AHEAD);
    const int younger = min(TR_AHEAD, n_st - 1 - i);   // stages requested after stage i
    if (younger >= 3) tr_wait_but<3 * TR_LPS>();
    else if (younger == 2) tr_wait_but<2 * TR_LPS>();
    else if (younger == 1) tr_wait_but<TR_LPS>();
    else tr_wait_but<0>();
    tr_barrier();   // stage i has landed for every lane
    if (want_append && (i + 1) * TR_SK > P) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int row = i * TR_SK + ld_row + 16 * j;
        if (row >= P && row < len) {
          const unsigned char* src = ring + slot * TR_STAGE + (ld_row + 16 * j) * TR_ROW + ld_col;
          __builtin_nontemporal_store(*(const u32x4*)src, (u32x4*)(kc + pair * S_cap * TR_ROW + (long)row * TR_ROW + ld_col));
          __builtin_nontemporal_store(*(const u32x4*)(src + TR_MAT),
                                      (u32x4*)(vc + pair * S_cap * TR_ROW + (long)row * TR_ROW + ld_col));
        }
      }
    }
    slot = slot + 1 == TR_NST ? 0 : slot + 1;
  }
  tr_wait_but<0>();   // no direct load may land after the workgroup has ended
  if (want_out) {
    tr_barrier();
    const unsigned char* stg = ring + wave * (32 * TR_ROW);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int r = 4 * j + (lane >> 4), piece = lane & 15;
      const int node = 32 * wave + r;
      if (node < N)
        __builtin_nontemporal_store(*(const u32x4*)(stg + r * TR_ROW + piece * 16),
                                    (u32x4*)(out + new_base + (long)node * new_row + piece * 16));
    }
  }
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

extern "C" int spec_probe_attention_traffic(int B, int H, int N, int P, int S_cap, void* k_cache, void* v_cache, const void* q,
                                            const void* k_new, const void* v_new, void* out, int flags, void* hip_stream) {
  const void* ptrs[6] = {k_cache, v_cache, q, k_new, v_new, out};
  for (const void* p : ptrs)
    if (p == nullptr || (reinterpret_cast<uintptr_t>(p) & 15u)) return -1;
  if (B < 1 || H < 1 || N < 1 || N > 128 || P < 0 || S_cap < 1 || (long)P + N > S_cap) return -1;
  if ((long)B * H > 65535L * 32 || (flags & ~15) != 0) return -1;
  hipLaunchKernelGGL(attention_traffic_kernel, dim3(B * H), dim3(256), 0, (hipStream_t)hip_stream, (unsigned char*)k_cache,
                     (unsigned char*)v_cache, (const unsigned char*)q, (const unsigned char*)k_new,
                     (const unsigned char*)v_new, (unsigned char*)out, H, N, P, S_cap, flags);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}
