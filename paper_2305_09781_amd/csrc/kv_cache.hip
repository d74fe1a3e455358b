// KV-cache update kernels: append of the tree tokens' K/V in node order (Section 4.2, one shared
// cache region for the whole tree) and commit of the accepted path (Algorithm 2 main loop: the
// verified tokens join the sequence, so their rows become the contiguous continuation of the prefix).
// Both are pure 16-byte-vector copies; they are bound by HBM traffic that is tiny next to attention.
#include <hip/hip_bf16.h>

#include "spec_internal.h"

namespace spec {

// One thread moves 16 bytes of K and 16 bytes of V of one (request, node, head) row.
__global__ void __launch_bounds__(256) kv_append_kernel(const uint4* __restrict__ k_new, const uint4* __restrict__ v_new,
                                                        uint4* __restrict__ k_cache, uint4* __restrict__ v_cache,
                                                        const int32_t* __restrict__ prefix_len, int32_t* status,
                                                        int B, int N, int H, int S_cap, int vec_per_row,
                                                        long q_sb, long q_sn, long q_sh,     // in uint4 units
                                                        long kv_sb, long kv_sh, long kv_ss, Pages pg) {
  const long total = (long)B * N * H * vec_per_row;
  long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int c = (int)(idx % vec_per_row);
  idx /= vec_per_row;
  const int h = (int)(idx % H);
  idx /= H;
  const int i = (int)(idx % N);
  const int b = (int)(idx / N);
  const int p = prefix_len[b];
  if (p < 0 || p > S_cap - N) {
    if (i == 0 && h == 0 && c == 0) set_status(status, b, SPEC_ST_CAPACITY);
    return;
  }
  const long src = b * q_sb + i * q_sn + h * q_sh + c;
  bool blk_ok;
  const long dst = cache_row_offset(pg, b, p + i, kv_sb, kv_ss, &blk_ok) + h * kv_sh + c;
  if (!blk_ok) {   // a row of a block outside the pool is not written
    if (h == 0 && c == 0) set_status(status, b, SPEC_ST_BAD_BLOCK);
    return;
  }
  k_cache[dst] = k_new[src];
  v_cache[dst] = v_new[src];
}

// KV append with the rotary position embedding applied to K on the way in (half-split pairing:
// dimension i < D/2 rotates with i + D/2), and optionally to the queries in place. Token i of request b sits at
// position prefix_len[b] + tree_depth[b,i]; cos / sin come from the caller's tables [rope_len, D/2]. grid =
// (chunks, B); a block first checks that the request fits the cache and that all its positions lie inside
// the tables (else it is left untouched and flagged), then every thread moves the two 16-byte pieces of one K
// row that rotate with each other and the same two pieces of V unchanged, or (threads past the K/V work,
// q != nullptr) rotates the two pieces of one query row in place.
template <bool BF16>
__global__ void __launch_bounds__(256) kv_append_rope_kernel(const uint4* __restrict__ k_new, const uint4* __restrict__ v_new,
                                                             uint4* __restrict__ k_cache, uint4* __restrict__ v_cache,
                                                             const int32_t* __restrict__ tree_depth,
                                                             const int32_t* __restrict__ prefix_len,
                                                             const float* __restrict__ rope_cos,
                                                             const float* __restrict__ rope_sin, int rope_len,
                                                             int32_t* status, int N, int H, int D, int S_cap,
                                                             int vec_per_row, long q_sb, long q_sn, long q_sh,
                                                             long kv_sb, long kv_sh, long kv_ss, Pages pg, uint4* q,
                                                             int Hq, long qq_sb, long qq_sn, long qq_sh) {
  constexpr int EPV = BF16 ? 8 : 4;   // elements per 16-byte piece
  __shared__ int s_bad;
  const int b = blockIdx.y, t = threadIdx.x;
  const int p = prefix_len[b];
  if (t == 0) s_bad = (p < 0 || p > S_cap - N) ? 1 : 0;
  __syncthreads();
  for (int i = t; i < N; i += 256) {
    const long pos = (long)p + tree_depth[(long)b * N + i];
    if (pos < 0 || pos >= rope_len) atomicOr(&s_bad, 1);
  }
  __syncthreads();
  if (s_bad != 0) {
    if (blockIdx.x == 0 && t == 0) set_status(status, b, SPEC_ST_CAPACITY);
    return;
  }
  const int half = vec_per_row / 2;
  const long kv_items = (long)N * H * half;
  long idx = (long)blockIdx.x * 256 + t;
  if (idx >= kv_items) {   // query rows (when asked for)
    idx -= kv_items;
    if (q == nullptr || idx >= (long)N * Hq * half) return;
    const int c = (int)(idx % half);
    idx /= half;
    const int h = (int)(idx % Hq);
    const int i = (int)(idx / Hq);
    const int pos = p + tree_depth[(long)b * N + i];
    uint4* row = q + b * qq_sb + i * qq_sn + h * qq_sh + c;
    uint4 olo, ohi;
    rope_pair<BF16>(row[0], row[half], rope_cos + (long)pos * (D / 2) + c * EPV, rope_sin + (long)pos * (D / 2) + c * EPV,
                    &olo, &ohi);
    row[0] = olo;
    row[half] = ohi;
    return;
  }
  const int c = (int)(idx % half);
  idx /= half;
  const int h = (int)(idx % H);
  const int i = (int)(idx / H);
  const int pos = p + tree_depth[(long)b * N + i];
  const long src = b * q_sb + i * q_sn + h * q_sh + c;
  bool blk_ok;
  const long dst = cache_row_offset(pg, b, p + i, kv_sb, kv_ss, &blk_ok) + h * kv_sh + c;
  if (!blk_ok) {   // a row of a block outside the pool is not written
    if (h == 0 && c == 0) set_status(status, b, SPEC_ST_BAD_BLOCK);
    return;
  }
  uint4 olo, ohi;
  rope_pair<BF16>(k_new[src], k_new[src + half], rope_cos + (long)pos * (D / 2) + c * EPV,
                  rope_sin + (long)pos * (D / 2) + c * EPV, &olo, &ohi);
  k_cache[dst] = olo;
  k_cache[dst + half] = ohi;
  v_cache[dst] = v_new[src];
  v_cache[dst + half] = v_new[src + half];
}

struct LayerPtrs {
  uint4* k[SPEC_MAX_COMMIT_LAYERS];
  uint4* v[SPEC_MAX_COMMIT_LAYERS];
};

// grid = (ceil(H * vec_per_row / 256), n_layers, B). A thread owns one 16-byte column of one head and
// walks the path in order. Row prefix+k is written only after rows prefix+path[j], j <= k, were read
// by the same thread (batches of 8: all loads, then all stores), and path[j] > k for j > k, so no
// source is overwritten before it is read.
__global__ void __launch_bounds__(256) kv_commit_kernel(LayerPtrs ptrs, const int32_t* __restrict__ path,
                                                        const int32_t* __restrict__ len,
                                                        const int32_t* __restrict__ prefix_len,
                                                        int32_t* __restrict__ prefix_len_out, int32_t* status, int N,
                                                        int H, int S_cap, int Lmax, int vec_per_row, long kv_sb,
                                                        long kv_sh, long kv_ss, Pages pg) {
  __shared__ int s_path[SPEC_MAX_TREE_NODES];
  __shared__ int s_bad;
  const int b = blockIdx.z;
  const int layer = blockIdx.y;
  const int t = threadIdx.x;
  const int n = len[b];
  const int p = prefix_len[b];
  if (t == 0) s_bad = 0;
  __syncthreads();
  const bool cap_ok = (p >= 0) && (p <= S_cap - N);
  const bool head_ok = cap_ok && (n >= 1) && (n <= Lmax) && (n <= N);
  if (head_ok) {
    for (int k = t; k < n; k += blockDim.x) {
      const int v = path[(long)b * Lmax + k];
      s_path[k] = v;
      bool ok = (k == 0) ? (v == 0) : (v > path[(long)b * Lmax + k - 1] && v < N);
      if (!ok) atomicOr(&s_bad, 1);
    }
  }
  __syncthreads();
  const bool ok = head_ok && s_bad == 0;
  __syncthreads();   // every thread has read the result of the path check before the flag is used again below
  // paged cache: every block that holds a row of the tree must lie inside the pool, else nothing moves
  if (ok && pg.table != nullptr) {
    for (int j = (p >> pg.log2_tokens) + t; j <= ((p + N - 1) >> pg.log2_tokens); j += blockDim.x) {
      const int e = pg.table[(long)b * pg.max_blocks + j];
      if (e < 0 || e >= pg.n_blocks) atomicOr(&s_bad, 2);
    }
  }
  __syncthreads();   // reached by every thread: `ok` is uniform, and the barrier is outside the condition
  const bool blocks_ok = !ok || s_bad == 0;
  if (blockIdx.x == 0 && layer == 0 && t == 0) {
    prefix_len_out[b] = (ok && blocks_ok) ? p + n : p;
    if (!ok) set_status(status, b, cap_ok ? SPEC_ST_BAD_PATH : SPEC_ST_CAPACITY);
    else if (!blocks_ok) set_status(status, b, SPEC_ST_BAD_BLOCK);
  }
  if (!ok || !blocks_ok) return;
  const int col = blockIdx.x * blockDim.x + t;
  if (col >= H * vec_per_row) return;
  const int h = col / vec_per_row, c = col % vec_per_row;
  uint4* kc = ptrs.k[layer] + h * kv_sh + c;
  uint4* vc = ptrs.v[layer] + h * kv_sh + c;
  bool in_pool;   // checked for all of the tree's blocks above
  for (int k0 = 0; k0 < n; k0 += 8) {
    uint4 kr[8], vr[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int k = k0 + j;
      if (k < n && s_path[k] != k) {
        const long src = cache_row_offset(pg, b, p + s_path[k], kv_sb, kv_ss, &in_pool);
        kr[j] = kc[src];
        vr[j] = vc[src];
      }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int k = k0 + j;
      if (k < n && s_path[k] != k) {
        const long dst = cache_row_offset(pg, b, p + k, kv_sb, kv_ss, &in_pool);
        kc[dst] = kr[j];
        vc[dst] = vr[j];
      }
    }
  }
}

static inline int elem_bytes(int dtype) { return dtype == SPEC_F32 ? 4 : 2; }

hipError_t launch_kv_append(const spec_attn_desc_t& d, const Pages& pg, const void* k_new, const void* v_new,
                            void* k_cache, void* v_cache, const int32_t* prefix_len, int32_t* status, hipStream_t s) {
  const int e = elem_bytes(d.dtype);
  const int per16 = 16 / e;
  const int vec_per_row = d.D / per16;
  const long total = (long)d.B * d.N * d.H_kv * vec_per_row;
  const int grid = (int)((total + 255) / 256);
  const NewStrides ns = attn_new_strides(d);
  hipLaunchKernelGGL(kv_append_kernel, dim3(grid), dim3(256), 0, s, (const uint4*)k_new, (const uint4*)v_new,
                     (uint4*)k_cache, (uint4*)v_cache, prefix_len, status, d.B, d.N, d.H_kv, d.S_cap, vec_per_row,
                     ns.b / per16, ns.n / per16, ns.h / per16, d.kv_stride_b / per16, d.kv_stride_h / per16,
                     d.kv_stride_s / per16, pg);
  return hipGetLastError();
}

hipError_t launch_kv_append_rope(const spec_attn_desc_t& d, const Pages& pg, const void* k_new, const void* v_new,
                                 void* k_cache, void* v_cache, const int32_t* tree_depth, const int32_t* prefix_len,
                                 const float* rope_cos, const float* rope_sin, int rope_len, int32_t* status,
                                 hipStream_t s, void* q) {
  const int e = elem_bytes(d.dtype);
  const int per16 = 16 / e;
  const int vec_per_row = d.D / per16;
  const long per_request = (long)d.N * (d.H_kv + (q != nullptr ? d.H : 0)) * (vec_per_row / 2);
  const dim3 grid((unsigned)((per_request + 255) / 256), d.B);
  const NewStrides ns = attn_new_strides(d);
#define SPEC_ROPE(BF)                                                                                                 \
  hipLaunchKernelGGL(kv_append_rope_kernel<BF>, grid, dim3(256), 0, s, (const uint4*)k_new, (const uint4*)v_new,      \
                     (uint4*)k_cache, (uint4*)v_cache, tree_depth, prefix_len, rope_cos, rope_sin, rope_len, status,  \
                     d.N, d.H_kv, d.D, d.S_cap, vec_per_row, ns.b / per16, ns.n / per16, ns.h / per16,                \
                     d.kv_stride_b / per16, d.kv_stride_h / per16, d.kv_stride_s / per16, pg, (uint4*)q, d.H,          \
                     d.q_stride_b / per16, d.q_stride_n / per16, d.q_stride_h / per16)
  if (d.dtype == SPEC_BF16) SPEC_ROPE(true);
  else SPEC_ROPE(false);
#undef SPEC_ROPE
  return hipGetLastError();
}

hipError_t launch_kv_commit(const spec_attn_desc_t& d, const Pages& pg, int n_layers, void* const* k_caches,
                            void* const* v_caches,
                            const int32_t* path, int Lmax, const int32_t* len, const int32_t* prefix_len,
                            int32_t* prefix_len_out, int32_t* status, hipStream_t s) {
  const int e = elem_bytes(d.dtype);
  const int per16 = 16 / e;
  const int vec_per_row = d.D / per16;
  LayerPtrs ptrs;
  for (int l = 0; l < SPEC_MAX_COMMIT_LAYERS; ++l) {
    ptrs.k[l] = (uint4*)(l < n_layers ? k_caches[l] : nullptr);
    ptrs.v[l] = (uint4*)(l < n_layers ? v_caches[l] : nullptr);
  }
  const int cols = d.H_kv * vec_per_row;
  dim3 grid((cols + 255) / 256, n_layers, d.B);
  hipLaunchKernelGGL(kv_commit_kernel, grid, dim3(256), 0, s, ptrs, path, len, prefix_len, prefix_len_out, status, d.N,
                     d.H_kv, d.S_cap, Lmax, vec_per_row, d.kv_stride_b / per16, d.kv_stride_h / per16,
                     d.kv_stride_s / per16, pg);
  return hipGetLastError();
}

}  // namespace spec
