// Internal declarations shared by the translation units of libspectree (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#ifdef __HIPCC__
#include <hip/hip_bf16.h>
#endif
#include <stdint.h>

#include "spec_tree.h"

namespace spec {

// ---------------------------------------------------------------------------------------------
// Launch plan of one tree-attention call: how the key range [0, prefix_len + N) of every
// (request, head) is cut into chunks (one workgroup each) and where the partial results live.
// ---------------------------------------------------------------------------------------------
struct AttnPlan {
  int chunk_keys;   // keys per workgroup (multiple of 32)
  int n_splits;     // chunks covering max_prefix_len + N; balanced plan: partial slots per (request, head)
  int balanced_wgs; // > 0: balanced plan with this many workgroups (see balanced_share), chunk_keys unused
  int balanced_tile;// keys per tile of the balanced deal (the tile of the kernel that runs the plan)
  bool wide;        // bf16: the wide kernel runs the plan (several query tiles per K/V head, or k_new not laid out like q)
  int heads_per_wg; // wide kernel, whole key ranges: consecutive K/V heads of a request served by one workgroup
  bool m32;         // 5..8 query tiles, D = 128: the kernel of tree_attention_bf16_wide32.hip (four wavefronts of 32
                    // queries, two workgroups per compute unit) instead of the wide kernel's eight wavefronts of 16
  size_t ws_o_off;  // float [B][H][n_splits][N][D]   un-normalised partial outputs
  size_t ws_ml_off; // float [B][H][n_splits][N][2]   running max (log2 domain) and partial sum
  size_t ws_bytes;
};

// Block table of a paged cache as the kernels take it (by value). table == nullptr: the cache is contiguous,
// [B, H_kv, S_cap, D]. Otherwise the cache is [n_blocks, H_kv, 2^log2_tokens, D] and the descriptor's
// kv_stride_b is the stride between blocks.
struct Pages {
  const int32_t* table;   // [B, max_blocks]
  int max_blocks;
  int log2_tokens;
  int n_blocks;
};
inline Pages no_pages() { return Pages{nullptr, 0, 0, 0}; }

// Rotary position embedding applied inside the fused append + attention call (cos == nullptr: none): the caller's
// float32 device tables [len, D/2]. Token i of request b sits at position prefix_len[b] + tree_depth[b, i].
struct Rope {
  const float* cos;
  const float* sin;
  int len;
};
inline Rope no_rope() { return Rope{nullptr, nullptr, 0}; }

AttnPlan make_attn_plan(const spec_attn_desc_t& d, bool paged = false);

// Tree queries handled by one workgroup of the attention kernel chosen for this shape
// (bf16: 16 / 32 in the few-query kernel, 64 / 128 in the wide-tree kernel; float32: all of them).
#define SPEC_SMALL_TILE_KEYS 32   // keys per wavefront tile of the few-query bf16 kernel (N <= 16)
#define SPEC_WIDE_TILE_KEYS 64    // keys per workgroup tile of the wide bf16 kernel (N > 16)

inline int attn_queries_per_workgroup(const spec_attn_desc_t& d) {
  if (d.dtype != SPEC_BF16) return SPEC_MAX_TREE_NODES;
  return d.N <= 16 ? 16 : d.N <= 32 ? 32 : d.N <= 64 ? 64 : 128;
}

// Query heads per key/value head, and how the bf16 kernels split them. Every query head of a group brings
// ceil(N / 16) 16-query MFMA tiles; a workgroup holds at most 8 tiles, i.e. `heads_per_wg` whole heads, so a
// (request, K/V head) pair is served by `n_qgroups` workgroups ("virtual heads" hv = h_kv * n_qgroups + qg),
// each streaming the pair's K/V for its own heads (the repeats are served by the caches).
struct QueryGroups {
  int group;          // query heads per K/V head
  int tiles_per_head; // ceil(N / 16)
  int heads_per_wg;   // query heads one workgroup serves
  int n_qgroups;      // workgroups per (request, K/V head) pair
  int tiles_per_wg;   // heads_per_wg * tiles_per_head, 1..8
};
inline QueryGroups attn_query_groups(const spec_attn_desc_t& d) {
  QueryGroups g;
  g.group = d.H / d.H_kv;
  g.tiles_per_head = (d.N + 15) / 16;
  const int fit = 8 / g.tiles_per_head > 0 ? 8 / g.tiles_per_head : 1;
  g.heads_per_wg = g.group < fit ? g.group : fit;
  g.n_qgroups = (g.group + g.heads_per_wg - 1) / g.heads_per_wg;
  g.tiles_per_wg = g.heads_per_wg * g.tiles_per_head;
  return g;
}

// Strides of k_new / v_new (all zero in the descriptor: laid out like q).
struct NewStrides { long b, n, h; };
inline NewStrides attn_new_strides(const spec_attn_desc_t& d) {
  if (d.new_stride_b == 0 && d.new_stride_n == 0 && d.new_stride_h == 0)
    return {(long)d.q_stride_b, (long)d.q_stride_n, (long)d.q_stride_h};
  return {(long)d.new_stride_b, (long)d.new_stride_n, (long)d.new_stride_h};
}

// Kernel launchers (defined in the .hip files). All return hipError_t of the launch.
hipError_t launch_kv_append(const spec_attn_desc_t& d, const Pages& pg, const void* k_new, const void* v_new,
                            void* k_cache, void* v_cache, const int32_t* prefix_len, int32_t* status, hipStream_t s);
hipError_t launch_kv_append_rope(const spec_attn_desc_t& d, const Pages& pg, const void* k_new, const void* v_new,
                                 void* k_cache, void* v_cache, const int32_t* tree_depth, const int32_t* prefix_len,
                                 const float* rope_cos, const float* rope_sin, int rope_len, int32_t* status,
                                 hipStream_t s, void* q = nullptr);
hipError_t launch_kv_commit(const spec_attn_desc_t& d, const Pages& pg, int n_layers, void* const* k_caches,
                            void* const* v_caches,
                            const int32_t* path, int Lmax, const int32_t* len, const int32_t* prefix_len,
                            int32_t* prefix_len_out, int32_t* status, hipStream_t s);
hipError_t launch_tree_attention_f32(const spec_attn_desc_t& d, const AttnPlan& plan, const Pages& pg, const float* q,
                                     const float* k_cache, const float* v_cache, const int32_t* parent,
                                     const int32_t* depth, const int32_t* prefix_len, float* out, void* ws,
                                     int32_t* status, hipStream_t s);
// k_new / v_new non-null: the kernel also appends the tree rows to the cache (fused KV append).
// rope.cos non-null (with k_new / v_new): the queries (in registers) and the new K rows (before they are used and
// stored) are rotated by their positions' angles.
hipError_t launch_tree_attention_bf16(const spec_attn_desc_t& d, const AttnPlan& plan, const Pages& pg, const void* q, void* k_cache,
                                      void* v_cache, const void* k_new, const void* v_new, const int32_t* parent,
                                      const int32_t* depth, const int32_t* prefix_len, void* out, void* ws,
                                      int32_t* status, hipStream_t s, const Rope& rope = no_rope());
// Wide trees (N > 32): the workgroup's wavefronts split the queries and share the K/V stream through LDS.
hipError_t launch_tree_attention_bf16_wide(const spec_attn_desc_t& d, const AttnPlan& plan, const Pages& pg, const void* q, void* k_cache,
                                           void* v_cache, const void* k_new, const void* v_new, const int32_t* parent,
                                           const int32_t* depth, const int32_t* prefix_len, void* out, void* ws,
                                           int32_t* status, hipStream_t s, const Rope& rope = no_rope());
// Five to eight query tiles per K/V head, D = 128: 32-query MFMA tiles, K/V loaded straight into an LDS ring.
hipError_t launch_tree_attention_bf16_wide32(const spec_attn_desc_t& d, const AttnPlan& plan, const Pages& pg, const void* q,
                                             void* k_cache, void* v_cache, const void* k_new, const void* v_new,
                                             const int32_t* parent, const int32_t* depth, const int32_t* prefix_len,
                                             void* out, void* ws, int32_t* status, hipStream_t s,
                                             const Rope& rope = no_rope());
hipError_t launch_attn_combine(const spec_attn_desc_t& d, const AttnPlan& plan, const int32_t* parent,
                               const int32_t* depth, const int32_t* prefix_len, const void* ws, void* out,
                               int32_t* status, hipStream_t s);
hipError_t launch_expand_topk(int B, int F, int V, int logits_dtype, const void* logits, int k, const int32_t* child_slot,
                              int N, int32_t* tree_token, int32_t* status, hipStream_t s);
hipError_t launch_tree_merge(int B, int M, int Nin, const int32_t* in_parent, const int32_t* in_token,
                             const int32_t* in_size, int Nout, int32_t* out_parent, int32_t* out_depth,
                             int32_t* out_token, int32_t* out_ssm, int32_t* out_size, int32_t* node_map, int32_t* status,
                             hipStream_t s);
// LM head + arg-max (lm_head.hip). Workspace: per row one (max, arg-max) pair per vocabulary tile.
#define SPEC_LM_HEAD_VOCAB_TILE 64   // the smaller of the two workgroup shapes: sizes the partials
inline int lm_head_waves(int M) {
  return M <= 32 ? 4 : 8;   // few rows: the stream is everything, and two workgroups per CU overlap their starts and ends
}
inline size_t lm_head_partials_bytes(int M, int V) {
  const size_t n_vtiles = ((size_t)V + SPEC_LM_HEAD_VOCAB_TILE - 1) / SPEC_LM_HEAD_VOCAB_TILE;
  return 2 * (((size_t)M * n_vtiles * 4 + 255) / 256 * 256);
}
hipError_t launch_lm_head_argmax(int M, int K, int V, const void* hidden, const void* weight, int32_t* node_argmax,
                                 float* node_max, void* ws, hipStream_t s);
// The same pass over the weights that also writes bf16 logits and their softmax statistics; the workspace holds
// three partial arrays (lm_head_partials_bytes(M, V) / 2 each).
hipError_t launch_lm_head(int M, int K, int V, const void* hidden, const void* weight, void* logits_out, float inv_temp,
                          int32_t* node_argmax, float* node_max, float* node_sumexp, void* ws, hipStream_t s);
hipError_t launch_node_stats(int B, int N, int V, int logits_dtype, const void* logits, float inv_temp,
                             int32_t* node_argmax, float* node_max, float* node_sumexp, hipStream_t s);
hipError_t launch_node_sample(int B, int N, int V, int logits_dtype, const void* logits, float inv_temp,
                              const float* node_max, const float* u_sample, int32_t* node_sample, hipStream_t s);
hipError_t launch_greedy_walk(int B, int N, const int32_t* node_argmax, const int32_t* token, const int32_t* parent,
                              int Lmax, int32_t* path, int32_t* len, int32_t* out_tokens, int32_t* status,
                              hipStream_t s);
hipError_t launch_stochastic_walk(int B, int N, int V, int logits_dtype, const void* logits, const float* probs_ssm,
                                  int R, const int32_t* ssm_row, const int32_t* token, const int32_t* parent,
                                  const float* u_accept, const float* u_order, const float* u_final, float inv_temp,
                                  const float* node_max, const float* node_sumexp, float* resid, int Lmax,
                                  int32_t* path, int32_t* len, int32_t* out_tokens, int32_t* status, hipStream_t s);

// ---------------------------------------------------------------------------------------------
// Device helpers
// ---------------------------------------------------------------------------------------------
#ifdef __HIPCC__

// Validates one request's tree with the threads of a workgroup (blockDim.x >= N).
// Returns true for every thread iff parent[0] == -1, 0 <= parent[i] < i and depth[i] == depth[parent[i]] + 1.
// `flag` is one int of LDS. Contains two __syncthreads().
__device__ inline bool tree_is_valid(const int32_t* __restrict__ parent, const int32_t* __restrict__ depth, int N,
                                     int* flag) {
  const int t = threadIdx.x;
  if (t == 0) *flag = 0;
  __syncthreads();
  if (t < N) {
    const int p = parent[t];
    bool ok;
    if (t == 0) {
      ok = (p == -1) && (depth == nullptr || depth[0] == 0);
    } else {
      ok = (p >= 0) && (p < t);
      if (ok && depth != nullptr) ok = depth[t] == depth[p] + 1;
    }
    if (!ok) atomicOr(flag, 1);
  }
  __syncthreads();
  return *flag == 0;
}

// Balanced plan: the key tiles (`tile` keys each) of all (request, head) pairs, ordered by (request,
// head, key), are dealt to `n_wg` workgroups in equal contiguous shares of `share` tiles (the last may
// be shorter). A request that does not fit the cache capacity contributes no tiles.
struct BalancedShare {
  long total;   // tiles over all requests and heads
  long share;   // tiles per workgroup (>= 1)
};
__device__ inline int request_tiles(int P, int N, int S_cap, int tile) {
  return (P >= 0 && P <= S_cap - N) ? (P + N + tile - 1) / tile : 0;
}
__device__ inline BalancedShare balanced_share(const int32_t* __restrict__ prefix_len, int B, int N, int H, int S_cap,
                                               int tile, int n_wg) {
  long tiles = 0;
  for (int b = 0; b < B; ++b) tiles += request_tiles(prefix_len[b], N, S_cap, tile);
  BalancedShare r;
  r.total = tiles * H;
  r.share = (r.total + n_wg - 1) / n_wg;
  if (r.share < 1) r.share = 1;
  return r;
}

// Rotation of the two 16-byte pieces of a row that pair up under the half-split rotary embedding (piece `lo`
// holds dimensions c .. c + EPV, `hi` the same dimensions + D/2), by the angles whose cosines / sines are cs / sn.
// float32 arithmetic in one fixed order (product, then fused multiply-add: the product is kept out of the
// compiler's contraction so that every kernel that rotates a row produces the same bits), rounded to the storage
// type.
template <bool BF16>
__device__ __forceinline__ void rope_pair(const uint4 lo, const uint4 hi, const float* __restrict__ cs,
                                          const float* __restrict__ sn, uint4* olo, uint4* ohi) {
  constexpr int EPV = BF16 ? 8 : 4;   // elements per 16-byte piece
  float x1[EPV], x2[EPV];
  if (BF16) {
    const unsigned a[4] = {lo.x, lo.y, lo.z, lo.w}, bb[4] = {hi.x, hi.y, hi.z, hi.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      x1[2 * j] = __uint_as_float(a[j] << 16);
      x1[2 * j + 1] = __uint_as_float(a[j] & 0xffff0000u);
      x2[2 * j] = __uint_as_float(bb[j] << 16);
      x2[2 * j + 1] = __uint_as_float(bb[j] & 0xffff0000u);
    }
  } else {
    x1[0] = __uint_as_float(lo.x); x1[1] = __uint_as_float(lo.y); x1[2] = __uint_as_float(lo.z); x1[3] = __uint_as_float(lo.w);
    x2[0] = __uint_as_float(hi.x); x2[1] = __uint_as_float(hi.y); x2[2] = __uint_as_float(hi.z); x2[3] = __uint_as_float(hi.w);
  }
  float y1[EPV], y2[EPV];
#pragma unroll
  for (int j = 0; j < EPV; ++j) {
    const float co = cs[j], si = sn[j];
    float p1 = x2[j] * si, p2 = x1[j] * si;
    asm("" : "+v"(p1), "+v"(p2));
    y1[j] = fmaf(x1[j], co, -p1);
    y2[j] = fmaf(x2[j], co, p2);
  }
  if (BF16) {
    unsigned o1[4], o2[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      union { __hip_bfloat16 h; unsigned short u; } a0, a1, b0, b1;
      a0.h = __float2bfloat16(y1[2 * j]); a1.h = __float2bfloat16(y1[2 * j + 1]);
      b0.h = __float2bfloat16(y2[2 * j]); b1.h = __float2bfloat16(y2[2 * j + 1]);
      o1[j] = (unsigned)a0.u | ((unsigned)a1.u << 16);
      o2[j] = (unsigned)b0.u | ((unsigned)b1.u << 16);
    }
    *olo = make_uint4(o1[0], o1[1], o1[2], o1[3]);
    *ohi = make_uint4(o2[0], o2[1], o2[2], o2[3]);
  } else {
    *olo = make_uint4(__float_as_uint(y1[0]), __float_as_uint(y1[1]), __float_as_uint(y1[2]), __float_as_uint(y1[3]));
    *ohi = make_uint4(__float_as_uint(y2[0]), __float_as_uint(y2[1]), __float_as_uint(y2[2]), __float_as_uint(y2[3]));
  }
}

__device__ inline void set_status(int32_t* status, int b, int bit) {
  if (status != nullptr) atomicOr(&status[b], bit);
}

// Offset, in the units of the two strides, of logical cache row `row` of request b before the head and
// column terms. Paged: `ok` tells whether the table entry lies inside the pool; an entry outside is
// replaced by one inside (block 0 or the last), so the offset always stays within the cache.
__device__ inline long cache_row_offset(const Pages& pg, int b, int row, long kv_sb, long kv_ss, bool* ok) {
  *ok = true;
  if (pg.table == nullptr) return b * kv_sb + (long)row * kv_ss;
  const int e = pg.table[(long)b * pg.max_blocks + (row >> pg.log2_tokens)];
  *ok = e >= 0 && e < pg.n_blocks;
  const int blk = min(max(e, 0), pg.n_blocks - 1);
  return blk * kv_sb + (long)(row & ((1 << pg.log2_tokens) - 1)) * kv_ss;
}

#endif  // __HIPCC__

}  // namespace spec
