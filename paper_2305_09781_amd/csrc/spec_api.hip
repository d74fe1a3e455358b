// C ABI of libspectree: host-side argument checks and kernel launches. Every entry point validates
// what the host can see, enqueues its kernels on the caller's stream and returns; nothing here
// allocates or synchronises.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>

#include "spec_internal.h"

// Scratch of spec_tree_attention_append_static: the split plans' float32 partial results, for callers that can
// neither allocate nor bring a workspace. Part of the code object, so every GPU that loads the library holds
// its own copy at its own address. In host code this name is only a handle for hipGetSymbolAddress; the
// device address it returns is what kernels and copies take.
static __device__ __align__(256) unsigned char scratch[SPEC_STATIC_SCRATCH_BYTES];

namespace spec {

// Device address of `scratch` on the current device, looked up once per device.
static int static_scratch(void** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptr[kMaxDevices] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SPEC_ERR_HIP;
  std::lock_guard<std::mutex> lock(mu);
  if (ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return SPEC_ERR_HIP;
    ptr[dev] = p;
  }
  *out = ptr[dev];
  return SPEC_OK;
}

static inline int elem_bytes(int dtype) { return dtype == SPEC_F32 ? 4 : 2; }
static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Host-checkable part of the attention descriptor. Returns SPEC_OK or an error code.
static int check_desc(const spec_attn_desc_t* d) {
  if (d == nullptr) return SPEC_ERR_INVALID_ARG;
  if (d->B <= 0 || d->H <= 0 || d->H_kv <= 0 || d->N <= 0 || d->S_cap <= 0 || d->D <= 0) return SPEC_ERR_INVALID_ARG;
  if (d->plan_chunk_keys < 0 || d->plan_balanced_wgs < -1 || d->plan_heads_per_wg < 0) return SPEC_ERR_INVALID_ARG;
  if (d->dtype != SPEC_F32 && d->dtype != SPEC_BF16) return SPEC_ERR_UNSUPPORTED;
  if (d->D != 64 && d->D != 128) return SPEC_ERR_UNSUPPORTED;
  if (d->N > SPEC_MAX_TREE_NODES) return SPEC_ERR_UNSUPPORTED;
  if (d->H % d->H_kv != 0) return SPEC_ERR_UNSUPPORTED;
  {
    const bool none = d->new_stride_b == 0 && d->new_stride_n == 0 && d->new_stride_h == 0;
    if (!none && (d->new_stride_b <= 0 || d->new_stride_n <= 0 || d->new_stride_h < d->D)) return SPEC_ERR_INVALID_ARG;
  }
  if (d->N > d->S_cap) return SPEC_ERR_CAPACITY;
  if (d->max_prefix_len < 0 || (long)d->max_prefix_len + d->N > d->S_cap) return SPEC_ERR_CAPACITY;
  if (!(d->softmax_scale >= 0.f) || std::isinf(d->softmax_scale)) return SPEC_ERR_INVALID_ARG;
  const int per16 = 16 / elem_bytes(d->dtype);
  const int64_t strides[6] = {d->q_stride_b, d->q_stride_n, d->q_stride_h, d->kv_stride_b, d->kv_stride_h, d->kv_stride_s};
  for (int64_t s : strides)
    if (s <= 0 || s % per16 != 0) return SPEC_ERR_INVALID_ARG;
  const int64_t new_strides[3] = {d->new_stride_b, d->new_stride_n, d->new_stride_h};
  for (int64_t s : new_strides)
    if (s % per16 != 0) return SPEC_ERR_INVALID_ARG;
  if (d->q_stride_h < d->D || d->kv_stride_s < d->D) return SPEC_ERR_INVALID_ARG;
  // the kernels compute row offsets inside one (request, head) span (paged: one block) in 32 bits
  if ((double)d->S_cap * (double)d->kv_stride_s * elem_bytes(d->dtype) >= 4294967296.0) return SPEC_ERR_UNSUPPORTED;
  return SPEC_OK;
}

// k_new / v_new cannot share q's layout when there are fewer K/V heads than query heads.
static bool new_strides_missing(const spec_attn_desc_t* d) {
  return d->H_kv != d->H && d->new_stride_b == 0 && d->new_stride_n == 0 && d->new_stride_h == 0;
}

// Host-checkable part of a paged-cache description; fills the form the kernels take.
static int check_pages(const spec_attn_desc_t* d, const spec_kv_pages_t* p, Pages* out) {
  if (p == nullptr || p->block_table == nullptr || p->max_blocks <= 0 || p->n_blocks <= 0) return SPEC_ERR_INVALID_ARG;
  const int bt = p->block_tokens;
  if (bt < 64 || bt > 65536 || (bt & (bt - 1)) != 0) return SPEC_ERR_UNSUPPORTED;
  if ((long)d->S_cap > (long)p->max_blocks * bt) return SPEC_ERR_CAPACITY;
  int lg = 0;
  while ((1 << lg) < bt) ++lg;
  *out = Pages{p->block_table, p->max_blocks, lg, p->n_blocks};
  return SPEC_OK;
}

// Compute units of the current device (256 when no device can be queried, e.g. sizing a workspace on a
// machine without a GPU). Asked on every call: the answer belongs to the device that is current now.
static int compute_units() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) == hipSuccess &&
      hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
    return n;
  return 256;
}

AttnPlan make_attn_plan(const spec_attn_desc_t& d, bool paged) {
  AttnPlan p;
  p.balanced_wgs = 0;
  p.balanced_tile = 0;
  p.heads_per_wg = 1;
  p.m32 = false;
  const int max_prefix = d.max_prefix_len > 0 ? d.max_prefix_len : d.S_cap - d.N;
  const int max_len = max_prefix + d.N;
  // bf16: one workgroup serves all query heads of a K/V head; float32: one per query head
  const QueryGroups qg = attn_query_groups(d);
  const int virtual_heads = d.H_kv * qg.n_qgroups;
  const long groups = (long)d.B * (d.dtype == SPEC_BF16 ? virtual_heads : d.H);
  const int tiles = qg.tiles_per_wg;   // 16-query tiles per workgroup
  // The few-query kernel serves one query tile per K/V head with k_new / v_new laid out like q; everything
  // else in bf16 runs on the wide kernel.
  const NewStrides ns = attn_new_strides(d);
  p.wide = d.dtype == SPEC_BF16 &&
           (tiles > 1 || ns.b != d.q_stride_b || ns.n != d.q_stride_n || ns.h != d.q_stride_h);
  int chunk = d.plan_chunk_keys;   // caller's hint; 0 = chosen below
  // Five to eight query tiles: four wavefronts of 32 queries unless the caller asks for several heads per
  // workgroup, which only the eight-wavefront shape serves.
  p.m32 = p.wide && tiles > 4 && d.D == 128 && d.plan_heads_per_wg == 0;
  // workgroups the device holds at once: four-wavefront shapes of the wide kernel run two per compute unit
  const long resident = (long)compute_units() * ((p.wide && (tiles <= 4 || p.m32)) ? 2 : 1);
  if (chunk <= 0 && d.dtype == SPEC_BF16) {
    // Several requests with few (request, head) pairs and long key ranges (long-context serving, ragged
    // lengths): the bf16 kernels deal the key tiles of all pairs to as many workgroups as the device holds at
    // once, in equal shares, so the stream is balanced whatever the individual lengths are. A share that
    // crosses a pair boundary is two segments in a row, each with its own first-load latency and epilogue
    // (about 6 us, measured against fixed chunks on equal lengths from 1024 to 16384 keys), so the deal is
    // used only when a share is long enough for that to be small next to what unequal lengths would cost
    // fixed chunks (a quarter of the stream for lengths uniform in [max/2, max]): at least 2048 keys per
    // share at the stated maximum length. One request has no lengths to balance: fixed chunks.
    const int tile = p.wide ? SPEC_WIDE_TILE_KEYS : SPEC_SMALL_TILE_KEYS;
    int wgs = d.plan_balanced_wgs;   // caller's hint: > 0 that many workgroups, -1 never, 0 = chosen here
    if (wgs < 0) {
      wgs = 0;
    } else if (wgs == 0) {
      const long max_tiles = groups * ((max_len + tile - 1) / tile);
      long cand = (max_tiles * tile / resident >= 2048) ? resident : 0;
      // every workgroup writes (and the combine step reads back) float32 partials for all queries of its
      // pair: keep that traffic under a quarter of the K/V stream (it matters with grouped-query heads,
      // where a pair has many queries and the batch few pairs)
      const double stream_bytes = (double)d.B * d.H_kv * max_len * d.D * 2.0 * 2.0;
      const double partial_bytes_per_wg = 2.0 * (double)qg.heads_per_wg * d.N * (d.D + 2) * 4.0;
      cand = std::min<long>(cand, (long)(0.25 * stream_bytes / partial_bytes_per_wg));
      // every workgroup walks prefix_len[0..B) with scalar loads to find its share: only for small batches
      wgs = (cand > groups && d.B > 1 && d.B <= 64) ? (int)cand : 0;
    }
    if (wgs > 0) {
      p.balanced_wgs = wgs;
      p.balanced_tile = tile;
      p.chunk_keys = 0;
      p.n_splits = (wgs + virtual_heads - 1) / virtual_heads + 1;   // a pair is overlapped by at most this many shares
    }
  }
  if (p.balanced_wgs == 0) {
    if (chunk <= 0) {
      // One workgroup per (request, head, query group) streams its whole key range when that already
      // gives every compute unit a workgroup: a workgroup's fixed cost (first loads, tree set-up, final
      // merge, and the extra combine launch) outweighs any gain from more parallel slack. With fewer pairs
      // the key range is cut into as many equal chunks as fill the device once, of at least 256 keys
      // (measured on one to four requests of 32 heads, 1024 to 16384 keys: 13 us instead of 22 for one
      // request of 1024 keys, 50 instead of 57 for 16384).
      long splits = std::max<long>(1, resident / std::max<long>(1, groups));
      const long max_splits = std::max<long>(1, max_len / 256);
      if (splits > max_splits) splits = max_splits;
      chunk = (int)((max_len + splits - 1) / splits);
      if (chunk < 128) chunk = 128;
    }
    // chunks start at tile boundaries (with paged caches a tile must not straddle two blocks)
    chunk = (int)round_up((size_t)chunk, (paged && p.wide) ? SPEC_WIDE_TILE_KEYS : 32);
    p.chunk_keys = chunk;
    p.n_splits = (max_len + chunk - 1) / chunk;
  }
  if (p.wide && p.n_splits <= 1 && p.balanced_wgs == 0 && qg.n_qgroups == 1 && tiles > 4 && !p.m32) {
    // Eight-wavefront workgroups (one per compute unit) and more (request, head) pairs than compute units: a
    // workgroup then serves several heads of a request in a row, which costs one prologue and one tree set-up
    // instead of one per head (measured: 3 % on 512 pairs of 640 keys; no gain for the four-wavefront shape,
    // where two workgroups per compute unit already overlap each other's prologues). Chosen to minimise
    // (rounds of workgroups) x (heads in a row + the fixed cost of a workgroup, about a third of a head).
    int best = 1;
    double best_cost = 1e30;
    for (int nh = 1; nh <= 8 && nh <= d.H_kv; ++nh) {
      const long wgs = (long)d.B * ((d.H_kv + nh - 1) / nh);
      const double cost = (double)((wgs + resident - 1) / resident) * (nh + 0.35);
      if (cost < best_cost - 1e-9) { best_cost = cost; best = nh; }
    }
    p.heads_per_wg = d.plan_heads_per_wg > 0 ? d.plan_heads_per_wg : best;
    if (p.heads_per_wg < 1) p.heads_per_wg = 1;
    if (p.heads_per_wg > d.H_kv) p.heads_per_wg = d.H_kv;
  }
  if (p.n_splits <= 1 && p.balanced_wgs == 0) {
    p.n_splits = 1;
    p.ws_o_off = p.ws_ml_off = 0;
    p.ws_bytes = 0;
  } else {
    const size_t rows = (size_t)d.B * d.H * p.n_splits * d.N;
    p.ws_o_off = 0;
    p.ws_ml_off = round_up(rows * d.D * sizeof(float), 256);
    p.ws_bytes = p.ws_ml_off + round_up(rows * 2 * sizeof(float), 256);
  }
  return p;
}

}  // namespace spec

using namespace spec;

extern "C" {

int spec_version(void) { return 100; }

const char* spec_strerror(int code) {
  switch (code) {
    case SPEC_OK: return "ok";
    case SPEC_ERR_INVALID_ARG: return "invalid argument (null pointer, non-positive size, bad stride or alignment)";
    case SPEC_ERR_UNSUPPORTED: return "unsupported shape or dtype";
    case SPEC_ERR_CAPACITY: return "tree does not fit the cache capacity";
    case SPEC_ERR_HIP: return "HIP runtime error";
    case SPEC_ERR_WORKSPACE: return "workspace missing or too small";
    default: return "unknown error code";
  }
}

// Every cache-touching entry point exists in a contiguous and a paged form; `pages` is NULL in the first.
static int kv_append_impl(const spec_attn_desc_t* desc, const spec_kv_pages_t* pages, bool paged, const void* k_new,
                          const void* v_new, void* k_cache, void* v_cache, const int32_t* prefix_len, int32_t* status,
                          void* hip_stream) {
  int rc = check_desc(desc);
  if (rc != SPEC_OK) return rc;
  Pages pg = no_pages();
  if (paged && (rc = check_pages(desc, pages, &pg)) != SPEC_OK) return rc;
  if (!k_new || !v_new || !k_cache || !v_cache || !prefix_len) return SPEC_ERR_INVALID_ARG;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_cache) || !aligned16(v_cache)) return SPEC_ERR_INVALID_ARG;
  if (new_strides_missing(desc)) return SPEC_ERR_INVALID_ARG;
  return launch_kv_append(*desc, pg, k_new, v_new, k_cache, v_cache, prefix_len, status, (hipStream_t)hip_stream) ==
                 hipSuccess
             ? SPEC_OK
             : SPEC_ERR_HIP;
}

int spec_kv_append(const spec_attn_desc_t* desc, const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                   const int32_t* prefix_len, int32_t* status, void* hip_stream) {
  return kv_append_impl(desc, nullptr, false, k_new, v_new, k_cache, v_cache, prefix_len, status, hip_stream);
}

int spec_kv_append_paged(const spec_attn_desc_t* desc, const spec_kv_pages_t* pages, const void* k_new, const void* v_new,
                         void* k_cache, void* v_cache, const int32_t* prefix_len, int32_t* status, void* hip_stream) {
  return kv_append_impl(desc, pages, true, k_new, v_new, k_cache, v_cache, prefix_len, status, hip_stream);
}

static int kv_append_rope_impl(const spec_attn_desc_t* desc, const spec_kv_pages_t* pages, bool paged, const void* k_new,
                               const void* v_new, void* k_cache, void* v_cache, const int32_t* tree_depth,
                               const int32_t* prefix_len, const float* rope_cos, const float* rope_sin, int32_t rope_len,
                               int32_t* status, void* hip_stream, void* q = nullptr, bool with_q = false) {
  if (with_q && (q == nullptr || !aligned16(q))) return check_desc(desc) != SPEC_OK ? check_desc(desc) : SPEC_ERR_INVALID_ARG;
  int rc = check_desc(desc);
  if (rc != SPEC_OK) return rc;
  Pages pg = no_pages();
  if (paged && (rc = check_pages(desc, pages, &pg)) != SPEC_OK) return rc;
  if (!k_new || !v_new || !k_cache || !v_cache || !prefix_len || !tree_depth || !rope_cos || !rope_sin) return SPEC_ERR_INVALID_ARG;
  if (rope_len <= 0 || new_strides_missing(desc)) return SPEC_ERR_INVALID_ARG;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_cache) || !aligned16(v_cache)) return SPEC_ERR_INVALID_ARG;
  return launch_kv_append_rope(*desc, pg, k_new, v_new, k_cache, v_cache, tree_depth, prefix_len, rope_cos, rope_sin,
                               rope_len, status, (hipStream_t)hip_stream, q) == hipSuccess
             ? SPEC_OK
             : SPEC_ERR_HIP;
}

int spec_qk_rope_append(const spec_attn_desc_t* desc, void* q, const void* k_new, const void* v_new, void* k_cache,
                        void* v_cache, const int32_t* tree_depth, const int32_t* prefix_len, const float* rope_cos,
                        const float* rope_sin, int32_t rope_len, int32_t* status, void* hip_stream) {
  return kv_append_rope_impl(desc, nullptr, false, k_new, v_new, k_cache, v_cache, tree_depth, prefix_len, rope_cos,
                             rope_sin, rope_len, status, hip_stream, q, true);
}

int spec_qk_rope_append_paged(const spec_attn_desc_t* desc, const spec_kv_pages_t* pages, void* q, const void* k_new,
                              const void* v_new, void* k_cache, void* v_cache, const int32_t* tree_depth,
                              const int32_t* prefix_len, const float* rope_cos, const float* rope_sin, int32_t rope_len,
                              int32_t* status, void* hip_stream) {
  return kv_append_rope_impl(desc, pages, true, k_new, v_new, k_cache, v_cache, tree_depth, prefix_len, rope_cos, rope_sin,
                             rope_len, status, hip_stream, q, true);
}

int spec_kv_append_rope(const spec_attn_desc_t* desc, const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                        const int32_t* tree_depth, const int32_t* prefix_len, const float* rope_cos, const float* rope_sin,
                        int32_t rope_len, int32_t* status, void* hip_stream) {
  return kv_append_rope_impl(desc, nullptr, false, k_new, v_new, k_cache, v_cache, tree_depth, prefix_len, rope_cos,
                             rope_sin, rope_len, status, hip_stream);
}

int spec_kv_append_rope_paged(const spec_attn_desc_t* desc, const spec_kv_pages_t* pages, const void* k_new,
                              const void* v_new, void* k_cache, void* v_cache, const int32_t* tree_depth,
                              const int32_t* prefix_len, const float* rope_cos, const float* rope_sin, int32_t rope_len,
                              int32_t* status, void* hip_stream) {
  return kv_append_rope_impl(desc, pages, true, k_new, v_new, k_cache, v_cache, tree_depth, prefix_len, rope_cos, rope_sin,
                             rope_len, status, hip_stream);
}

size_t spec_tree_attention_workspace_bytes(const spec_attn_desc_t* desc) {
  if (check_desc(desc) != SPEC_OK) return 0;
  return make_attn_plan(*desc).ws_bytes;
}

size_t spec_tree_attention_paged_workspace_bytes(const spec_attn_desc_t* desc, const spec_kv_pages_t* pages) {
  Pages pg;
  if (check_desc(desc) != SPEC_OK || check_pages(desc, pages, &pg) != SPEC_OK) return 0;
  return make_attn_plan(*desc, true).ws_bytes;
}

// Shared body of spec_tree_attention (k_new == NULL) and spec_tree_attention_append.
static int tree_attention_impl(const spec_attn_desc_t* desc, const spec_kv_pages_t* pages, bool paged, const void* q,
                               const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                               const int32_t* tree_parent, const int32_t* tree_depth, const int32_t* prefix_len, void* out,
                               void* workspace, size_t workspace_bytes, int32_t* status, void* hip_stream,
                               const Rope& rope = no_rope()) {
  int rc = check_desc(desc);
  if (rc != SPEC_OK) return rc;
  Pages pg = no_pages();
  if (paged && (rc = check_pages(desc, pages, &pg)) != SPEC_OK) return rc;
  if (!q || !k_cache || !v_cache || !tree_parent || !tree_depth || !prefix_len || !out) return SPEC_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out)) return SPEC_ERR_INVALID_ARG;
  const bool append = k_new != nullptr || v_new != nullptr;
  if (append && (!k_new || !v_new || !aligned16(k_new) || !aligned16(v_new) || new_strides_missing(desc)))
    return SPEC_ERR_INVALID_ARG;
  const AttnPlan plan = make_attn_plan(*desc, paged);
  if (plan.ws_bytes > 0) {
    if (workspace == nullptr || workspace_bytes < plan.ws_bytes) return SPEC_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return SPEC_ERR_INVALID_ARG;
  }
  // The launch plan covers keys up to max_prefix_len + N. A request whose prefix_len exceeds the stated
  // maximum must not be attended over a truncated key range: the kernels treat the stated maximum as the
  // capacity, so such a request is flagged SPEC_ST_CAPACITY like one that does not fit the cache.
  spec_attn_desc_t d = *desc;
  if (d.max_prefix_len > 0) d.S_cap = d.max_prefix_len + d.N;   // <= S_cap (checked above); strides are unchanged
  // Rotary tables: they must cover every position of a tree of N nodes, so their length bounds the capacity too.
  if (rope.cos != nullptr && rope.len < d.S_cap) d.S_cap = rope.len;
  hipStream_t s = (hipStream_t)hip_stream;
  hipError_t e;
  if (d.dtype == SPEC_BF16) {
    e = launch_tree_attention_bf16(d, plan, pg, q, k_cache, v_cache, k_new, v_new, tree_parent, tree_depth, prefix_len, out,
                                   workspace, status, s, rope);
  } else {
    if (append) {
      e = launch_kv_append(d, pg, k_new, v_new, k_cache, v_cache, prefix_len, status, s);
      if (e != hipSuccess) return SPEC_ERR_HIP;
    }
    e = launch_tree_attention_f32(d, plan, pg, (const float*)q, (const float*)k_cache, (const float*)v_cache, tree_parent,
                                  tree_depth, prefix_len, (float*)out, workspace, status, s);
  }
  if (e != hipSuccess) return SPEC_ERR_HIP;
  if (plan.n_splits > 1 || plan.balanced_wgs > 0) {
    e = launch_attn_combine(d, plan, tree_parent, tree_depth, prefix_len, workspace, out, status, s);
    if (e != hipSuccess) return SPEC_ERR_HIP;
  }
  return SPEC_OK;
}

int spec_tree_attention(const spec_attn_desc_t* desc, const void* q, const void* k_cache, const void* v_cache,
                        const int32_t* tree_parent, const int32_t* tree_depth, const int32_t* prefix_len, void* out,
                        void* workspace, size_t workspace_bytes, int32_t* status, void* hip_stream) {
  return tree_attention_impl(desc, nullptr, false, q, nullptr, nullptr, const_cast<void*>(k_cache),
                             const_cast<void*>(v_cache), tree_parent, tree_depth, prefix_len, out, workspace,
                             workspace_bytes, status, hip_stream);
}

int spec_tree_attention_paged(const spec_attn_desc_t* desc, const spec_kv_pages_t* pages, const void* q,
                              const void* k_cache, const void* v_cache, const int32_t* tree_parent,
                              const int32_t* tree_depth, const int32_t* prefix_len, void* out, void* workspace,
                              size_t workspace_bytes, int32_t* status, void* hip_stream) {
  return tree_attention_impl(desc, pages, true, q, nullptr, nullptr, const_cast<void*>(k_cache),
                             const_cast<void*>(v_cache), tree_parent, tree_depth, prefix_len, out, workspace,
                             workspace_bytes, status, hip_stream);
}

int spec_tree_attention_append(const spec_attn_desc_t* desc, const void* q, const void* k_new, const void* v_new,
                               void* k_cache, void* v_cache, const int32_t* tree_parent, const int32_t* tree_depth,
                               const int32_t* prefix_len, void* out, void* workspace, size_t workspace_bytes,
                               int32_t* status, void* hip_stream) {
  if (!k_new || !v_new) return check_desc(desc) != SPEC_OK ? check_desc(desc) : SPEC_ERR_INVALID_ARG;
  return tree_attention_impl(desc, nullptr, false, q, k_new, v_new, k_cache, v_cache, tree_parent, tree_depth,
                             prefix_len, out, workspace, workspace_bytes, status, hip_stream);
}

static int rope_args(const spec_attn_desc_t* desc, const void* k_new, const void* v_new, const float* rope_cos,
                     const float* rope_sin, int32_t rope_len) {
  const int rc = check_desc(desc);
  if (rc != SPEC_OK) return rc;
  if (!k_new || !v_new || !rope_cos || !rope_sin || rope_len <= 0) return SPEC_ERR_INVALID_ARG;
  if (desc->dtype != SPEC_BF16) return SPEC_ERR_UNSUPPORTED;
  return SPEC_OK;
}

int spec_tree_attention_append_rope(const spec_attn_desc_t* desc, const void* q, const void* k_new, const void* v_new,
                                    void* k_cache, void* v_cache, const int32_t* tree_parent, const int32_t* tree_depth,
                                    const int32_t* prefix_len, const float* rope_cos, const float* rope_sin,
                                    int32_t rope_len, void* out, void* workspace, size_t workspace_bytes,
                                    int32_t* status, void* hip_stream) {
  const int rc = rope_args(desc, k_new, v_new, rope_cos, rope_sin, rope_len);
  if (rc != SPEC_OK) return rc;
  return tree_attention_impl(desc, nullptr, false, q, k_new, v_new, k_cache, v_cache, tree_parent, tree_depth,
                             prefix_len, out, workspace, workspace_bytes, status, hip_stream,
                             Rope{rope_cos, rope_sin, rope_len});
}

int spec_tree_attention_append_rope_paged(const spec_attn_desc_t* desc, const spec_kv_pages_t* pages, const void* q,
                                          const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                                          const int32_t* tree_parent, const int32_t* tree_depth,
                                          const int32_t* prefix_len, const float* rope_cos, const float* rope_sin,
                                          int32_t rope_len, void* out, void* workspace, size_t workspace_bytes,
                                          int32_t* status, void* hip_stream) {
  const int rc = rope_args(desc, k_new, v_new, rope_cos, rope_sin, rope_len);
  if (rc != SPEC_OK) return rc;
  return tree_attention_impl(desc, pages, true, q, k_new, v_new, k_cache, v_cache, tree_parent, tree_depth, prefix_len,
                             out, workspace, workspace_bytes, status, hip_stream, Rope{rope_cos, rope_sin, rope_len});
}

int spec_tree_attention_append_static(const spec_attn_desc_t* desc, const void* q, const void* k_new, const void* v_new,
                                      void* k_cache, void* v_cache, const int32_t* tree_parent,
                                      const int32_t* tree_depth, const int32_t* prefix_len, void* out, int32_t* status,
                                      void* hip_stream) {
  const int rc = check_desc(desc);
  if (rc != SPEC_OK) return rc;
  if (!k_new || !v_new) return SPEC_ERR_INVALID_ARG;
  // the plan of the contiguous call decides how much scratch the launch needs
  const size_t need = make_attn_plan(*desc).ws_bytes;
  if (need > (size_t)SPEC_STATIC_SCRATCH_BYTES) return SPEC_ERR_WORKSPACE;
  void* ws = nullptr;
  if (need > 0) {
    const int src = static_scratch(&ws);
    if (src != SPEC_OK) return src;
  }
  return tree_attention_impl(desc, nullptr, false, q, k_new, v_new, k_cache, v_cache, tree_parent, tree_depth,
                             prefix_len, out, ws, need, status, hip_stream);
}

int spec_tree_attention_append_paged(const spec_attn_desc_t* desc, const spec_kv_pages_t* pages, const void* q,
                                     const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                                     const int32_t* tree_parent, const int32_t* tree_depth, const int32_t* prefix_len,
                                     void* out, void* workspace, size_t workspace_bytes, int32_t* status,
                                     void* hip_stream) {
  if (!k_new || !v_new) return check_desc(desc) != SPEC_OK ? check_desc(desc) : SPEC_ERR_INVALID_ARG;
  return tree_attention_impl(desc, pages, true, q, k_new, v_new, k_cache, v_cache, tree_parent, tree_depth, prefix_len,
                             out, workspace, workspace_bytes, status, hip_stream);
}

static int check_verify_common(int32_t B, int32_t N, int32_t V, int32_t logits_dtype, const void* logits,
                               const int32_t* tree_token, const int32_t* tree_parent, int32_t Lmax,
                               const int32_t* accepted_path, const int32_t* accepted_len, const int32_t* out_tokens) {
  if (B <= 0 || N <= 0 || V <= 0 || Lmax <= 0) return SPEC_ERR_INVALID_ARG;
  if (N > SPEC_MAX_TREE_NODES) return SPEC_ERR_UNSUPPORTED;
  if (logits_dtype != SPEC_F32 && logits_dtype != SPEC_BF16) return SPEC_ERR_UNSUPPORTED;
  if (!logits || !tree_token || !tree_parent || !accepted_path || !accepted_len || !out_tokens) return SPEC_ERR_INVALID_ARG;
  if (!aligned16(logits)) return SPEC_ERR_INVALID_ARG;
  return SPEC_OK;
}

int spec_tree_expand_topk(int32_t B, int32_t F, int32_t V, int32_t logits_dtype, const void* ssm_logits, int32_t k,
                          const int32_t* child_slot, int32_t N, int32_t* tree_token, int32_t* status, void* hip_stream) {
  if (B <= 0 || F <= 0 || V <= 0 || N <= 0 || k <= 0) return SPEC_ERR_INVALID_ARG;
  if (k > V || k > SPEC_MAX_TOPK || N > SPEC_MAX_TREE_NODES) return SPEC_ERR_UNSUPPORTED;
  if (logits_dtype != SPEC_F32 && logits_dtype != SPEC_BF16) return SPEC_ERR_UNSUPPORTED;
  if (!ssm_logits || !child_slot || !tree_token) return SPEC_ERR_INVALID_ARG;
  return launch_expand_topk(B, F, V, logits_dtype, ssm_logits, k, child_slot, N, tree_token, status,
                            (hipStream_t)hip_stream) == hipSuccess
             ? SPEC_OK
             : SPEC_ERR_HIP;
}

int spec_tree_merge(int32_t B, int32_t M, int32_t Nin, const int32_t* in_parent, const int32_t* in_token,
                    const int32_t* in_size, int32_t Nout, int32_t* out_parent, int32_t* out_depth, int32_t* out_token,
                    int32_t* out_ssm, int32_t* out_size, int32_t* node_map, int32_t* status, void* hip_stream) {
  if (B <= 0 || M <= 0 || Nin <= 0 || Nout <= 0) return SPEC_ERR_INVALID_ARG;
  if ((long)M * Nin > SPEC_MAX_MERGE_INPUT_NODES || Nout > SPEC_MAX_TREE_NODES) return SPEC_ERR_UNSUPPORTED;
  if (!in_parent || !in_token || !in_size || !out_parent || !out_depth || !out_token || !out_ssm || !out_size)
    return SPEC_ERR_INVALID_ARG;
  return launch_tree_merge(B, M, Nin, in_parent, in_token, in_size, Nout, out_parent, out_depth, out_token, out_ssm,
                           out_size, node_map, status, (hipStream_t)hip_stream) == hipSuccess
             ? SPEC_OK
             : SPEC_ERR_HIP;
}

int spec_verify_greedy(int32_t B, int32_t N, int32_t V, int32_t logits_dtype, const void* logits_llm,
                       const int32_t* tree_token, const int32_t* tree_parent, int32_t Lmax, int32_t* accepted_path,
                       int32_t* accepted_len, int32_t* out_tokens, int32_t* node_argmax, void* workspace,
                       size_t workspace_bytes, int32_t* status, void* hip_stream) {
  const int rc = check_verify_common(B, N, V, logits_dtype, logits_llm, tree_token, tree_parent, Lmax, accepted_path,
                                     accepted_len, out_tokens);
  if (rc != SPEC_OK) return rc;
  if (node_argmax == nullptr) {
    if (workspace == nullptr || workspace_bytes < (size_t)B * N * sizeof(int32_t)) return SPEC_ERR_WORKSPACE;
    node_argmax = (int32_t*)workspace;
  }
  hipStream_t s = (hipStream_t)hip_stream;
  if (launch_node_stats(B, N, V, logits_dtype, logits_llm, 1.0f, node_argmax, nullptr, nullptr, s) != hipSuccess)
    return SPEC_ERR_HIP;
  if (launch_greedy_walk(B, N, node_argmax, tree_token, tree_parent, Lmax, accepted_path, accepted_len, out_tokens,
                         status, s) != hipSuccess)
    return SPEC_ERR_HIP;
  return SPEC_OK;
}

size_t spec_lm_head_argmax_workspace_bytes(int32_t M, int32_t V) {
  if (M <= 0 || V <= 0) return 0;
  // the partials, then room for node_argmax when the caller of spec_verify_greedy_lm_head does not want it
  return lm_head_partials_bytes(M, V) + round_up((size_t)M * sizeof(int32_t), 256);
}

static int check_lm_head(int32_t M, int32_t K, int32_t V, const void* hidden, const void* weight, const void* workspace,
                         size_t workspace_bytes) {
  if (M <= 0 || K <= 0 || V <= 0) return SPEC_ERR_INVALID_ARG;
  if (K % 256 != 0) return SPEC_ERR_UNSUPPORTED;
  if (!hidden || !weight || !aligned16(hidden) || !aligned16(weight)) return SPEC_ERR_INVALID_ARG;
  if (workspace == nullptr || workspace_bytes < spec_lm_head_argmax_workspace_bytes(M, V)) return SPEC_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return SPEC_ERR_INVALID_ARG;
  return SPEC_OK;
}

int spec_lm_head_argmax(int32_t M, int32_t K, int32_t V, const void* hidden, const void* weight, int32_t* node_argmax,
                        float* node_max, void* workspace, size_t workspace_bytes, void* hip_stream) {
  const int rc = check_lm_head(M, K, V, hidden, weight, workspace, workspace_bytes);
  if (rc != SPEC_OK) return rc;
  if (!node_argmax) return SPEC_ERR_INVALID_ARG;
  return launch_lm_head_argmax(M, K, V, hidden, weight, node_argmax, node_max, workspace, (hipStream_t)hip_stream) ==
                 hipSuccess
             ? SPEC_OK
             : SPEC_ERR_HIP;
}

int spec_verify_greedy_lm_head(int32_t B, int32_t N, int32_t K, int32_t V, const void* hidden, const void* weight,
                               const int32_t* tree_token, const int32_t* tree_parent, int32_t Lmax,
                               int32_t* accepted_path, int32_t* accepted_len, int32_t* out_tokens, int32_t* node_argmax,
                               void* workspace, size_t workspace_bytes, int32_t* status, void* hip_stream) {
  if (B <= 0 || N <= 0 || Lmax <= 0) return SPEC_ERR_INVALID_ARG;
  if (N > SPEC_MAX_TREE_NODES) return SPEC_ERR_UNSUPPORTED;
  if ((long)B * N > 0x7fffffffL) return SPEC_ERR_UNSUPPORTED;
  const int M = B * N;
  const int rc = check_lm_head(M, K, V, hidden, weight, workspace, workspace_bytes);
  if (rc != SPEC_OK) return rc;
  if (!tree_token || !tree_parent || !accepted_path || !accepted_len || !out_tokens) return SPEC_ERR_INVALID_ARG;
  if (node_argmax == nullptr) node_argmax = (int32_t*)((char*)workspace + lm_head_partials_bytes(M, V));
  hipStream_t s = (hipStream_t)hip_stream;
  if (launch_lm_head_argmax(M, K, V, hidden, weight, node_argmax, nullptr, workspace, s) != hipSuccess) return SPEC_ERR_HIP;
  if (launch_greedy_walk(B, N, node_argmax, tree_token, tree_parent, Lmax, accepted_path, accepted_len, out_tokens,
                         status, s) != hipSuccess)
    return SPEC_ERR_HIP;
  return SPEC_OK;
}

size_t spec_verify_naive_workspace_bytes(int32_t B, int32_t N, int32_t V) {
  if (B <= 0 || N <= 0 || V <= 0) return 0;
  // node max, then the sampled tokens when the caller does not want them
  return round_up((size_t)B * N * sizeof(float), 256) + round_up((size_t)B * N * sizeof(int32_t), 256);
}

int spec_verify_naive(int32_t B, int32_t N, int32_t V, int32_t logits_dtype, const void* logits_llm,
                      const int32_t* tree_token, const int32_t* tree_parent, const float* u_sample, float temperature,
                      int32_t Lmax, int32_t* accepted_path, int32_t* accepted_len, int32_t* out_tokens,
                      int32_t* node_sample, void* workspace, size_t workspace_bytes, int32_t* status,
                      void* hip_stream) {
  const int rc = check_verify_common(B, N, V, logits_dtype, logits_llm, tree_token, tree_parent, Lmax, accepted_path,
                                     accepted_len, out_tokens);
  if (rc != SPEC_OK) return rc;
  if (!u_sample) return SPEC_ERR_INVALID_ARG;
  if (!(temperature > 0.f) || std::isinf(temperature)) return SPEC_ERR_INVALID_ARG;
  if (workspace == nullptr || workspace_bytes < spec_verify_naive_workspace_bytes(B, N, V)) return SPEC_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return SPEC_ERR_INVALID_ARG;
  float* node_max = (float*)workspace;
  if (node_sample == nullptr) node_sample = (int32_t*)((char*)workspace + round_up((size_t)B * N * sizeof(float), 256));
  hipStream_t s = (hipStream_t)hip_stream;
  const float inv_temp = 1.0f / temperature;
  if (launch_node_stats(B, N, V, logits_dtype, logits_llm, inv_temp, nullptr, node_max, nullptr, s) != hipSuccess)
    return SPEC_ERR_HIP;
  if (launch_node_sample(B, N, V, logits_dtype, logits_llm, inv_temp, node_max, u_sample, node_sample, s) != hipSuccess)
    return SPEC_ERR_HIP;
  if (launch_greedy_walk(B, N, node_sample, tree_token, tree_parent, Lmax, accepted_path, accepted_len, out_tokens,
                         status, s) != hipSuccess)
    return SPEC_ERR_HIP;
  return SPEC_OK;
}

size_t spec_verify_stochastic_workspace_bytes(int32_t B, int32_t N, int32_t V) {
  if (B <= 0 || N <= 0 || V <= 0) return 0;
  // node max + node sum-exp, then two residual buffers of V floats per request
  return round_up((size_t)B * N * 2 * sizeof(float), 256) + round_up((size_t)2 * B * V * sizeof(float), 256);
}

int spec_verify_stochastic(int32_t B, int32_t N, int32_t V, int32_t logits_dtype, const void* logits_llm,
                           const float* probs_ssm, int32_t R, const int32_t* ssm_row, const int32_t* tree_token,
                           const int32_t* tree_parent, const float* u_accept, const float* u_order,
                           const float* u_final, float temperature, int32_t Lmax, int32_t* accepted_path,
                           int32_t* accepted_len, int32_t* out_tokens, void* workspace, size_t workspace_bytes,
                           int32_t* status, void* hip_stream) {
  const int rc = check_verify_common(B, N, V, logits_dtype, logits_llm, tree_token, tree_parent, Lmax, accepted_path,
                                     accepted_len, out_tokens);
  if (rc != SPEC_OK) return rc;
  if (!ssm_row || !u_accept || !u_order || !u_final) return SPEC_ERR_INVALID_ARG;
  if (R < 0 || (R > 0 && probs_ssm == nullptr)) return SPEC_ERR_INVALID_ARG;
  if (!(temperature > 0.f) || std::isinf(temperature)) return SPEC_ERR_INVALID_ARG;
  const size_t need = spec_verify_stochastic_workspace_bytes(B, N, V);
  if (workspace == nullptr || workspace_bytes < need) return SPEC_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return SPEC_ERR_INVALID_ARG;
  float* node_max = (float*)workspace;
  float* node_sumexp = node_max + (size_t)B * N;
  float* resid = (float*)((char*)workspace + round_up((size_t)B * N * 2 * sizeof(float), 256));
  const float inv_temp = 1.0f / temperature;
  hipStream_t s = (hipStream_t)hip_stream;
  if (launch_node_stats(B, N, V, logits_dtype, logits_llm, inv_temp, nullptr, node_max, node_sumexp, s) != hipSuccess)
    return SPEC_ERR_HIP;
  if (launch_stochastic_walk(B, N, V, logits_dtype, logits_llm, probs_ssm, R, ssm_row, tree_token, tree_parent, u_accept,
                             u_order, u_final, inv_temp, node_max, node_sumexp, resid, Lmax, accepted_path, accepted_len,
                             out_tokens, status, s) != hipSuccess)
    return SPEC_ERR_HIP;
  return SPEC_OK;
}

size_t spec_lm_head_logits_stats_workspace_bytes(int32_t M, int32_t V) {
  if (M <= 0 || V <= 0) return 0;
  return 3 * (lm_head_partials_bytes(M, V) / 2);   // (max, arg-max, sum) per row and vocabulary tile
}

int spec_lm_head_logits_stats(int32_t M, int32_t K, int32_t V, const void* hidden, const void* weight, float temperature,
                              void* logits, int32_t* node_argmax, float* node_max, float* node_sumexp, void* workspace,
                              size_t workspace_bytes, void* hip_stream) {
  if (M <= 0 || K <= 0 || V <= 0) return SPEC_ERR_INVALID_ARG;
  if (K % 256 != 0) return SPEC_ERR_UNSUPPORTED;
  if (!hidden || !weight || !aligned16(hidden) || !aligned16(weight)) return SPEC_ERR_INVALID_ARG;
  if (!logits || !node_max || !node_sumexp || (reinterpret_cast<uintptr_t>(logits) & 7u)) return SPEC_ERR_INVALID_ARG;
  if (!(temperature > 0.f) || std::isinf(temperature)) return SPEC_ERR_INVALID_ARG;
  if (workspace == nullptr || workspace_bytes < spec_lm_head_logits_stats_workspace_bytes(M, V)) return SPEC_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return SPEC_ERR_INVALID_ARG;
  return launch_lm_head(M, K, V, hidden, weight, logits, 1.0f / temperature, node_argmax, node_max, node_sumexp, workspace,
                        (hipStream_t)hip_stream) == hipSuccess
             ? SPEC_OK
             : SPEC_ERR_HIP;
}

size_t spec_verify_stochastic_stats_workspace_bytes(int32_t B, int32_t V) {
  if (B <= 0 || V <= 0) return 0;
  return round_up((size_t)2 * B * V * sizeof(float), 256);   // two residual buffers of V floats per request
}

int spec_verify_stochastic_stats(int32_t B, int32_t N, int32_t V, int32_t logits_dtype, const void* logits_llm,
                                 const float* node_max, const float* node_sumexp, const float* probs_ssm, int32_t R,
                                 const int32_t* ssm_row, const int32_t* tree_token, const int32_t* tree_parent,
                                 const float* u_accept, const float* u_order, const float* u_final, float temperature,
                                 int32_t Lmax, int32_t* accepted_path, int32_t* accepted_len, int32_t* out_tokens,
                                 void* workspace, size_t workspace_bytes, int32_t* status, void* hip_stream) {
  const int rc = check_verify_common(B, N, V, logits_dtype, logits_llm, tree_token, tree_parent, Lmax, accepted_path,
                                     accepted_len, out_tokens);
  if (rc != SPEC_OK) return rc;
  if (!ssm_row || !u_accept || !u_order || !u_final || !node_max || !node_sumexp) return SPEC_ERR_INVALID_ARG;
  if (R < 0 || (R > 0 && probs_ssm == nullptr)) return SPEC_ERR_INVALID_ARG;
  if (!(temperature > 0.f) || std::isinf(temperature)) return SPEC_ERR_INVALID_ARG;
  if (workspace == nullptr || workspace_bytes < spec_verify_stochastic_stats_workspace_bytes(B, V)) return SPEC_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return SPEC_ERR_INVALID_ARG;
  return launch_stochastic_walk(B, N, V, logits_dtype, logits_llm, probs_ssm, R, ssm_row, tree_token, tree_parent, u_accept,
                                u_order, u_final, 1.0f / temperature, node_max, node_sumexp, (float*)workspace, Lmax,
                                accepted_path, accepted_len, out_tokens, status, (hipStream_t)hip_stream) == hipSuccess
             ? SPEC_OK
             : SPEC_ERR_HIP;
}

static int kv_commit_impl(const spec_attn_desc_t* desc, const spec_kv_pages_t* pages, bool paged, int32_t n_layers,
                          void* const* k_caches, void* const* v_caches, const int32_t* accepted_path, int32_t Lmax,
                          const int32_t* accepted_len, const int32_t* prefix_len, int32_t* prefix_len_out, int32_t* status,
                          void* hip_stream) {
  int rc = check_desc(desc);
  if (rc != SPEC_OK) return rc;
  Pages pg = no_pages();
  if (paged && (rc = check_pages(desc, pages, &pg)) != SPEC_OK) return rc;
  if (n_layers <= 0 || Lmax <= 0) return SPEC_ERR_INVALID_ARG;
  if (n_layers > SPEC_MAX_COMMIT_LAYERS) return SPEC_ERR_UNSUPPORTED;
  if (!k_caches || !v_caches || !accepted_path || !accepted_len || !prefix_len || !prefix_len_out) return SPEC_ERR_INVALID_ARG;
  if (prefix_len_out == prefix_len) return SPEC_ERR_INVALID_ARG;
  for (int l = 0; l < n_layers; ++l)
    if (!k_caches[l] || !v_caches[l] || !aligned16(k_caches[l]) || !aligned16(v_caches[l])) return SPEC_ERR_INVALID_ARG;
  return launch_kv_commit(*desc, pg, n_layers, k_caches, v_caches, accepted_path, Lmax, accepted_len, prefix_len,
                          prefix_len_out, status, (hipStream_t)hip_stream) == hipSuccess
             ? SPEC_OK
             : SPEC_ERR_HIP;
}

int spec_kv_commit(const spec_attn_desc_t* desc, int32_t n_layers, void* const* k_caches, void* const* v_caches,
                   const int32_t* accepted_path, int32_t Lmax, const int32_t* accepted_len, const int32_t* prefix_len,
                   int32_t* prefix_len_out, int32_t* status, void* hip_stream) {
  return kv_commit_impl(desc, nullptr, false, n_layers, k_caches, v_caches, accepted_path, Lmax, accepted_len, prefix_len,
                        prefix_len_out, status, hip_stream);
}

int spec_kv_commit_paged(const spec_attn_desc_t* desc, const spec_kv_pages_t* pages, int32_t n_layers,
                         void* const* k_caches, void* const* v_caches, const int32_t* accepted_path, int32_t Lmax,
                         const int32_t* accepted_len, const int32_t* prefix_len, int32_t* prefix_len_out, int32_t* status,
                         void* hip_stream) {
  return kv_commit_impl(desc, pages, true, n_layers, k_caches, v_caches, accepted_path, Lmax, accepted_len, prefix_len,
                        prefix_len_out, status, hip_stream);
}

}  // extern "C"
