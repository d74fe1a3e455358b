/*
 * spec_tree.h - C ABI of the tree-based parallel decoding library for AMD MI355X (gfx950).
 *
 * One decoding iteration of a speculative-inference server verifies, for every request, a whole
 * speculated token tree in a single pass of the LLM (SpecInfer, arxiv 2305.09781, Section 4 and
 * Algorithm 2). The calls below are the per-layer and per-pass steps of that iteration:
 *
 *   before the pass: spec_tree_expand_topk (per speculation step) | spec_tree_merge   (build the token tree)
 *   for each layer:  spec_kv_append  ->  spec_tree_attention      (or the fused spec_tree_attention_append)
 *   once per pass:   spec_verify_greedy | spec_verify_stochastic | spec_verify_naive  ->  spec_kv_commit (all layers)
 *   every cache-touching call also exists as *_paged, for caches kept as pools of blocks behind a block table
 *
 * Conventions common to every call
 *   - Every data pointer is a DEVICE pointer unless its comment says "host". The caller owns all
 *     buffers; the library allocates nothing and keeps no state between calls. Scratch memory comes
 *     from a caller-supplied workspace whose size is returned by the matching *_workspace_bytes call
 *     (one call, spec_tree_attention_append_static, uses a scratch array of the library instead).
 *   - Every call only enqueues work on `hip_stream` (a hipStream_t passed as void*, NULL = the null
 *     stream) and returns without synchronising. Outputs are valid once the stream reaches that point.
 *   - Return value: SPEC_OK (0) or a negative SPEC_ERR_* code for anything the host can check
 *     (null pointers, unsupported shapes, misaligned pointers or strides, workspace too small). When an
 *     error is returned nothing has been enqueued.
 *   - Data-dependent faults (a malformed tree, a request that does not fit its cache, a malformed
 *     accepted path) are detected on the device: the request's outputs become a defined no-op and the
 *     SPEC_ST_* bit is OR-ed into status[b]. `status` ([B] int32, device) may be NULL; the caller
 *     clears it. No such input can cause an out-of-bounds access.
 *   - Token tree (Definition 3.1): N nodes per request in a topological order, node 0 is the root (the
 *     last verified token, whose K/V is not cached yet), tree_parent[b][0] = -1 and
 *     0 <= tree_parent[b][i] < i. Depth-first order (Section 4.2) is one such order.
 *     tree_depth[b][i] = tree_depth[b][parent] + 1, tree_depth[b][0] = 0. N <= SPEC_MAX_TREE_NODES.
 *   - Layouts. q / out / k_new / v_new: [B, N, H, D] addressed with (q_stride_b, q_stride_n,
 *     q_stride_h), D contiguous. KV cache of one layer: [B, H_kv, S_cap, D] addressed with
 *     (kv_stride_b, kv_stride_h, kv_stride_s), D contiguous; row s of request b holds token s of the
 *     request's sequence, rows [0, prefix_len[b]) are the verified prefix and rows
 *     [prefix_len[b], prefix_len[b] + N) hold the tree in node order after spec_kv_append.
 *     All strides are in ELEMENTS and must be multiples of 16 bytes; base pointers 16-byte aligned.
 *     The rows of one (request, head) must span less than 4 GiB (S_cap * kv_stride_s * element size
 *     < 2^32, with S_cap the logical capacity of a request for paged caches; SPEC_ERR_UNSUPPORTED
 *     otherwise): row offsets inside that span are computed in 32 bits.
 */
#ifndef SPEC_TREE_H
#define SPEC_TREE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPEC_MAX_TREE_NODES 128
#define SPEC_MAX_MERGE_INPUT_NODES 1024 /* spec_tree_merge: trees per request x node slots per tree */
#define SPEC_MAX_TOPK 16                /* spec_tree_expand_topk: children per frontier node        */
#define SPEC_MAX_COMMIT_LAYERS 128

/* return codes */
#define SPEC_OK 0
#define SPEC_ERR_INVALID_ARG (-1) /* null pointer, non-positive size, bad stride or alignment        */
#define SPEC_ERR_UNSUPPORTED (-2) /* D not in {64,128}, N > SPEC_MAX_TREE_NODES, dtype, H_kv not a   */
                                  /* divisor of H, a (request, head) span of 4 GiB or more           */
#define SPEC_ERR_CAPACITY (-3)    /* N > S_cap, max_prefix_len + N > S_cap                           */
#define SPEC_ERR_HIP (-4)         /* a HIP runtime call failed (launch error)                        */
#define SPEC_ERR_WORKSPACE (-5)   /* workspace NULL or smaller than *_workspace_bytes reports        */

/* per-request status bits (device side) */
#define SPEC_ST_BAD_TREE 1      /* tree_parent / tree_depth violate the token-tree contract          */
#define SPEC_ST_CAPACITY 2      /* prefix_len[b] < 0 or prefix_len[b] + N > S_cap                    */
#define SPEC_ST_BAD_PATH 4      /* accepted path: len out of range, path[0] != 0, not increasing     */
#define SPEC_ST_ZERO_RESIDUAL 8 /* stochastic verify: residual distribution had no mass left         */
#define SPEC_ST_BAD_BLOCK 16    /* paged cache: a block-table entry the request uses is not in       */
                                /* [0, n_blocks)                                                     */

typedef enum { SPEC_F32 = 0, SPEC_BF16 = 1 } spec_dtype_t;

/* Shape of one attention layer call; passed by pointer (host memory), read during the call only. */
typedef struct spec_attn_desc {
  int32_t B;              /* requests in the batch                                                   */
  int32_t H;              /* query heads                                                             */
  int32_t H_kv;           /* key/value heads, a divisor of H. H_kv = H: multi-head (the paper's      */
                          /* models); H_kv < H: grouped-query heads, query head h reads K/V head      */
                          /* h / (H / H_kv)                                                           */
  int32_t D;              /* head dimension: 64 or 128                                               */
  int32_t N;              /* tree nodes per request, 1..SPEC_MAX_TREE_NODES                          */
  int32_t S_cap;          /* rows per (request, head) in the cache                                   */
  int32_t dtype;          /* spec_dtype_t of q, out, k_new, v_new and the caches                     */
  int32_t max_prefix_len; /* upper bound of prefix_len[b], sizes grid and workspace; 0 = S_cap - N.  */
                          /* The attention calls treat a request above it like one that does not fit */
                          /* (SPEC_ST_CAPACITY, out = 0, not appended)                               */
  int64_t q_stride_b, q_stride_n, q_stride_h;       /* q, out: [B,N,H,D], in elements                */
  int64_t kv_stride_b, kv_stride_h, kv_stride_s;    /* caches: [B,H_kv,S_cap,D]                      */
  int64_t new_stride_b, new_stride_n, new_stride_h; /* k_new, v_new: [B,N,H_kv,D]; all 0 = the q     */
                                                    /* strides (only meaningful when H_kv = H)       */
  float softmax_scale;    /* 0 = 1/sqrt(D)                                                           */
  /* Launch-plan hints of the attention calls, all 0 = the library chooses (by shape and device). They   */
  /* change how the key range is dealt to workgroups, never what is computed (results agree up to        */
  /* float32 rounding order); the workspace size follows them. For callers that tune a shape, and for    */
  /* tests that drive small inputs through every plan.                                                    */
  int32_t plan_chunk_keys;   /* > 0: fixed chunks of this many keys (rounded up to the kernel's tile), one */
                             /* workgroup per (request, head, chunk), partials merged by a second launch  */
  int32_t plan_balanced_wgs; /* > 0: bf16 only, the key tiles of all (request, head) pairs dealt in equal  */
                             /* shares to this many workgroups; -1: never use that plan                    */
  int32_t plan_heads_per_wg; /* > 0: trees of 65..128 nodes streamed whole: consecutive K/V heads of a     */
                             /* request served by one workgroup                                            */
} spec_attn_desc_t;

/*
 * KV append (Section 4.2, "depth-first search to update key-value cache"): one cache region is shared
 * by every sequence of the tree; tree token i of request b goes to cache row prefix_len[b] + i:
 *     cache[b, h, prefix_len[b] + i, :] = new[b, i, h, :]      (K and V, bit copy)
 * A request with prefix_len[b] < 0 or prefix_len[b] + N > S_cap is skipped (SPEC_ST_CAPACITY).
 */
int spec_kv_append(const spec_attn_desc_t* desc, const void* k_new, const void* v_new, void* k_cache,
                   void* v_cache, const int32_t* prefix_len /*[B]*/, int32_t* status /*[B] or NULL*/,
                   void* hip_stream);

/*
 * KV append with the rotary position embedding applied to the keys on the way in (the paper's LLaMA
 * models rotate q and k by position; the paper itself is silent on where). Tree token i of request b
 * sits at sequence position prefix_len[b] + tree_depth[b,i] - its depth below the last verified
 * token, not its row in the cache. Half-split pairing: dimension j < D/2 rotates with j + D/2,
 *     k'[j] = k[j] cos - k[j+D/2] sin,   k'[j+D/2] = k[j+D/2] cos + k[j] sin,
 * cos / sin = rope_cos / rope_sin[position, j] (float32 DEVICE tables [rope_len, D/2] supplied by the
 * caller), computed in float32 and rounded to the cache's element type; V is copied unchanged.
 * A request that does not fit the cache or has a position outside [0, rope_len) is left untouched and
 * flagged SPEC_ST_CAPACITY. Queries are expected to arrive already rotated.
 */
int spec_kv_append_rope(const spec_attn_desc_t* desc, const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                        const int32_t* tree_depth /*[B,N]*/, const int32_t* prefix_len /*[B]*/,
                        const float* rope_cos /*[rope_len, D/2]*/, const float* rope_sin /*[rope_len, D/2]*/,
                        int32_t rope_len, int32_t* status /*[B] or NULL*/, void* hip_stream);

/*
 * The same append with the queries rotated too, in one launch: q [B,N,H,D] (the descriptor's q strides) is
 * rotated IN PLACE, row (b, i) of every head by position prefix_len[b] + tree_depth[b,i], same tables, same
 * pairing, float32 arithmetic rounded to the element type. After this call spec_tree_attention on (q, caches)
 * is the attention of a model with rotary embeddings. A request that is skipped (see above) keeps its q; in
 * the paged form a request with SPEC_ST_BAD_BLOCK has its q rotated and the rows of the bad block unwritten.
 * q == NULL is SPEC_ERR_INVALID_ARG.
 */
int spec_qk_rope_append(const spec_attn_desc_t* desc, void* q, const void* k_new, const void* v_new, void* k_cache,
                        void* v_cache, const int32_t* tree_depth /*[B,N]*/, const int32_t* prefix_len /*[B]*/,
                        const float* rope_cos, const float* rope_sin, int32_t rope_len, int32_t* status,
                        void* hip_stream);

/*
 * Tree attention (Definition 4.1; attention equations of Section 4.1; topology-aware causal mask of
 * Section 4.2). For every request b, head h and tree node i:
 *     out[b,i,h,:] = softmax_j( q[b,i,h,:] . k[b,h,j,:] * scale ) . v[b,h,j,:]
 * over j in [0, prefix_len[b])  union  { prefix_len[b] + a : a is node i or an ancestor of i },
 * i.e. exactly the sequence attention of the node's root-to-node token sequence behind the prefix.
 * The caches must already hold the tree rows (spec_kv_append). Scores, softmax and accumulation are
 * float32; `out` has the input dtype. A request with a malformed tree (SPEC_ST_BAD_TREE) or that
 * does not fit (SPEC_ST_CAPACITY) gets out = 0. tree_depth is only validated here.
 * workspace: spec_tree_attention_workspace_bytes(desc) bytes, 256-byte aligned; contents are scratch.
 */
int spec_tree_attention(const spec_attn_desc_t* desc, const void* q, const void* k_cache,
                        const void* v_cache, const int32_t* tree_parent /*[B,N]*/,
                        const int32_t* tree_depth /*[B,N]*/, const int32_t* prefix_len /*[B]*/,
                        void* out, void* workspace, size_t workspace_bytes,
                        int32_t* status /*[B] or NULL*/, void* hip_stream);
size_t spec_tree_attention_workspace_bytes(const spec_attn_desc_t* desc);

/*
 * Fused form of spec_kv_append followed by spec_tree_attention (same sections of the paper): the tree
 * rows are read from k_new / v_new, used by the attention and written to the caches in the same
 * pass, which saves one launch and re-reading the 2N new rows per (request, head). Results, status
 * bits and workspace are those of the two calls made one after the other, except that for a request
 * flagged SPEC_ST_BAD_TREE (out = 0) it is unspecified whether its tree rows were written to the cache.
 * A request flagged SPEC_ST_CAPACITY is neither appended nor attended.
 */
int spec_tree_attention_append(const spec_attn_desc_t* desc, const void* q, const void* k_new, const void* v_new,
                               void* k_cache, void* v_cache, const int32_t* tree_parent /*[B,N]*/,
                               const int32_t* tree_depth /*[B,N]*/, const int32_t* prefix_len /*[B]*/, void* out,
                               void* workspace, size_t workspace_bytes, int32_t* status /*[B] or NULL*/,
                               void* hip_stream);

/*
 * The fused call for a model with rotary embeddings (the paper's LLaMA models; Sections 4.1-4.2 for the
 * attention and the cache, the rotation as in spec_kv_append_rope): spec_qk_rope_append followed by
 * spec_tree_attention in ONE launch. The queries are rotated in registers (q itself is NOT modified), the new K
 * rows are rotated before they are used by the attention and written to the cache, V is copied; positions,
 * pairing, tables and arithmetic are those of spec_kv_append_rope, and the cache rows and `out` come out
 * bit-identical to the two calls made one after the other. bf16 only (other dtypes: SPEC_ERR_UNSUPPORTED).
 * Capacity rule: the tables must cover every position a tree of N nodes can take, so a request with
 * prefix_len[b] + N > min(S_cap, rope_len) is neither appended nor attended and is flagged SPEC_ST_CAPACITY
 * (the two-launch form checks each node's own position instead). Workspace: spec_tree_attention_workspace_bytes
 * (paged form: spec_tree_attention_paged_workspace_bytes). NULL tables or rope_len <= 0: SPEC_ERR_INVALID_ARG.
 */
int spec_tree_attention_append_rope(const spec_attn_desc_t* desc, const void* q, const void* k_new, const void* v_new,
                                    void* k_cache, void* v_cache, const int32_t* tree_parent /*[B,N]*/,
                                    const int32_t* tree_depth /*[B,N]*/, const int32_t* prefix_len /*[B]*/,
                                    const float* rope_cos /*[rope_len, D/2]*/, const float* rope_sin /*[rope_len, D/2]*/,
                                    int32_t rope_len, void* out, void* workspace, size_t workspace_bytes,
                                    int32_t* status /*[B] or NULL*/, void* hip_stream);

/*
 * spec_tree_attention_append for callers that cannot allocate or bring a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc. Same arguments, results and status bits as
 * spec_tree_attention_append, without the workspace: the float32 partial results of a split key range live
 * in a device array of SPEC_STATIC_SCRATCH_BYTES that is part of the library's code object (every GPU the
 * library runs on holds its own copy until the process ends). The call allocates nothing and calls no
 * allocating routine; a shape whose launch plan needs more scratch than that is refused with
 * SPEC_ERR_WORKSPACE (nothing enqueued). The array's device address is looked up once per device, on the
 * first call made with that device current (do that first call outside graph capture, like any kernel's).
 * Every call on a GPU shares that GPU's array, which keeps the previous call's contents: nothing in it has
 * to start at zero (each launch writes every slot it later reads), but two calls whose work overlaps in
 * time on one GPU (different streams, or threads on different streams) race on it. Calls on one stream are
 * safe back to back.
 */
#define SPEC_STATIC_SCRATCH_BYTES (64u << 20)
int spec_tree_attention_append_static(const spec_attn_desc_t* desc, const void* q, const void* k_new,
                                      const void* v_new, void* k_cache, void* v_cache,
                                      const int32_t* tree_parent /*[B,N]*/, const int32_t* tree_depth /*[B,N]*/,
                                      const int32_t* prefix_len /*[B]*/, void* out,
                                      int32_t* status /*[B] or NULL*/, void* hip_stream);

/*
 * Expansion-based token tree construction, one step (Section 3): for every frontier node f of every
 * request, the k tokens with the largest ssm_logits[b,f,:] (largest first; ties: lowest token id) become
 * the tokens of its children: tree_token[b, child_slot[f*k + j]] = j-th pick. The tree's shape is fixed
 * by the static expansion configuration <k_1,...,k_m>, so parent / depth arrays and child_slot are
 * the caller's constants; only tokens are data. child_slot: DEVICE array [F,k] of node indices in
 * [0, N); an index outside sets SPEC_ST_BAD_TREE for the request and writes nothing. 1 <= k <=
 * min(V, SPEC_MAX_TOPK). ssm_logits: SPEC_F32 or SPEC_BF16, [B,F,V] contiguous.
 */
int spec_tree_expand_topk(int32_t B, int32_t F, int32_t V, int32_t logits_dtype, const void* ssm_logits, int32_t k,
                          const int32_t* child_slot /*[F,k]*/, int32_t N, int32_t* tree_token /*[B,N]*/,
                          int32_t* status /*[B] or NULL*/, void* hip_stream);

/*
 * Token tree merge (Definition 3.2): the M token trees of a request (one per SSM) become one tree that
 * holds exactly their token sequences S_u, each once. Input tree i of request b uses the first
 * in_size[b,i] of its Nin slots (root first, in_parent < own index, tokens >= 0); all roots carry the
 * same token (the last verified token). M * Nin <= SPEC_MAX_MERGE_INPUT_NODES, Nout <= SPEC_MAX_TREE_NODES.
 * Output, per request, Nout slots: merged nodes numbered depth-first (pre-order), the children of a node
 * ordered by first appearance when the trees are scanned i = 0..M-1, nodes in index order;
 * out_ssm[b,n] = lowest tree index whose tree holds node n's sequence (the draft distribution
 * spec_verify_stochastic should test it against); out_size[b] = number of merged nodes; slots at and
 * beyond it are padding nodes (parent 0, depth 1, token -1, ssm -1) that no verifier accepts, so the
 * arrays can go straight to the attention and verification calls with N = Nout.
 * node_map[b,i,u] (may be NULL) = merged index of input node u of tree i, -1 for unused slots.
 * Status: SPEC_ST_BAD_TREE (malformed input tree, differing roots) or SPEC_ST_CAPACITY (more than Nout
 * sequences): out_size = 0, a root slot plus padding, node_map = -1.
 */
int spec_tree_merge(int32_t B, int32_t M, int32_t Nin, const int32_t* in_parent /*[B,M,Nin]*/,
                    const int32_t* in_token /*[B,M,Nin]*/, const int32_t* in_size /*[B,M]*/, int32_t Nout,
                    int32_t* out_parent /*[B,Nout]*/, int32_t* out_depth /*[B,Nout]*/, int32_t* out_token /*[B,Nout]*/,
                    int32_t* out_ssm /*[B,Nout]*/, int32_t* out_size /*[B]*/, int32_t* node_map /*[B,M,Nin] or NULL*/,
                    int32_t* status /*[B] or NULL*/, void* hip_stream);

/*
 * Greedy verification (Algorithm 2, VerifyGreedy). O(u) = argmax_x logits_llm[b,u,x] (lowest token id
 * on ties). Starting at the root, while some child v of u has tree_token[b,v] == O(u) (lowest node
 * index if several) accept v and continue from it; finally emit the bonus token O(u).
 * Outputs: accepted_path[b, 0..len) node indices, root first; out_tokens[b, 0..len) = tokens of the
 * accepted children followed by the bonus token (same count as path nodes); both padded with -1 up to
 * Lmax; accepted_len[b] = len >= 1; node_argmax[b,u] = O(u) (may be NULL, then `workspace` must hold
 * B*N*4 bytes). Lmax >= max depth + 1 (N always suffices). A malformed tree gives accepted_len = 0.
 * logits_dtype: SPEC_F32 or SPEC_BF16, [B,N,V] contiguous.
 */
int spec_verify_greedy(int32_t B, int32_t N, int32_t V, int32_t logits_dtype, const void* logits_llm,
                       const int32_t* tree_token /*[B,N]*/, const int32_t* tree_parent /*[B,N]*/,
                       int32_t Lmax, int32_t* accepted_path /*[B,Lmax]*/, int32_t* accepted_len /*[B]*/,
                       int32_t* out_tokens /*[B,Lmax]*/, int32_t* node_argmax /*[B,N] or NULL*/,
                       void* workspace, size_t workspace_bytes, int32_t* status, void* hip_stream);

/*
 * Naive-sampling verification (Section 4.3: the straightforward alternative that multi-step
 * speculative sampling is compared with in Theorem 4.3 and Table 3). For every node u one token
 * x_u ~ softmax(logits_llm[b,u,:] / temperature) is drawn by inverse CDF over ascending token id: the
 * first k with cumsum(P)[k] > u_sample[b,u] * sum(P) (uniforms supplied by the caller, float32 in
 * [0,1)). Starting at the root, while some child v of u has tree_token[b,v] == x_u (lowest node index
 * if several) the token is emitted and the walk continues from v; otherwise x_u is emitted and the walk
 * stops. Outputs as for spec_verify_greedy; node_sample[b,u] = x_u (may be NULL).
 * workspace: spec_verify_naive_workspace_bytes(B, N, V) bytes, 256-byte aligned.
 */
size_t spec_verify_naive_workspace_bytes(int32_t B, int32_t N, int32_t V);
int spec_verify_naive(int32_t B, int32_t N, int32_t V, int32_t logits_dtype, const void* logits_llm,
                      const int32_t* tree_token /*[B,N]*/, const int32_t* tree_parent /*[B,N]*/,
                      const float* u_sample /*[B,N]*/, float temperature, int32_t Lmax,
                      int32_t* accepted_path /*[B,Lmax]*/, int32_t* accepted_len /*[B]*/,
                      int32_t* out_tokens /*[B,Lmax]*/, int32_t* node_sample /*[B,N] or NULL*/, void* workspace,
                      size_t workspace_bytes, int32_t* status, void* hip_stream);

/*
 * Stochastic verification (Algorithm 2, VerifyStochastic: multi-step speculative sampling, Section
 * 4.3). At node u: P = softmax(logits_llm[b,u,:] / temperature). The children of u are tried in
 * ascending order of (u_order[b,v], v). Child s with token x = tree_token[b,s] and draft distribution
 * Q = probs_ssm[ssm_row[b,s], :] passes iff u_accept[b,s] * Q[x] <= P[x] (float32); then x is emitted
 * and the walk continues from s. Otherwise P := normalise(max(0, P - Q)) for the remaining siblings.
 * When no child is left (or u is a leaf) the last token is drawn from the current P by inverse CDF
 * over ascending token id: the first k with cumsum(P)[k] > u_final[b] * sum(P).
 * The uniforms are supplied by the caller (float32 in [0,1)); the library draws no random numbers.
 * A node with a negative tree_token is a padding node (spec_tree_merge produces them): no verifier
 * ever accepts it.
 * Outputs as for spec_verify_greedy. SPEC_ST_ZERO_RESIDUAL: a residual had no mass; the previous P
 * was kept. workspace: spec_verify_stochastic_workspace_bytes(B, N, V) bytes.
 */
int spec_verify_stochastic(int32_t B, int32_t N, int32_t V, int32_t logits_dtype, const void* logits_llm,
                           const float* probs_ssm /*[R,V]*/, int32_t R, const int32_t* ssm_row /*[B,N]*/,
                           const int32_t* tree_token, const int32_t* tree_parent,
                           const float* u_accept /*[B,N]*/, const float* u_order /*[B,N]*/,
                           const float* u_final /*[B]*/, float temperature, int32_t Lmax,
                           int32_t* accepted_path, int32_t* accepted_len, int32_t* out_tokens,
                           void* workspace, size_t workspace_bytes, int32_t* status, void* hip_stream);
size_t spec_verify_stochastic_workspace_bytes(int32_t B, int32_t N, int32_t V);

/*
 * Stochastic verification from statistics the caller already has (Algorithm 2, VerifyStochastic: before any
 * rejection at a node the walk needs P(x | u) for single tokens only, i.e. the row's maximum and its sum of
 * exponentials). Exactly spec_verify_stochastic without its first pass over the logits: node_max[b,u] = max_x
 * logits_llm[b,u,x] and node_sumexp[b,u] = sum_x exp((logits_llm[b,u,x] - node_max[b,u]) / temperature), float32
 * [B,N], computed from the logits AS STORED (spec_lm_head_logits_stats produces all three in one pass over the
 * LLM's output projection). The logits themselves are still read for the tokens tested, after a rejection and
 * for the final draw. workspace: spec_verify_stochastic_stats_workspace_bytes(B, V) bytes, 256-byte aligned.
 */
size_t spec_verify_stochastic_stats_workspace_bytes(int32_t B, int32_t V);
int spec_verify_stochastic_stats(int32_t B, int32_t N, int32_t V, int32_t logits_dtype, const void* logits_llm,
                                 const float* node_max /*[B,N]*/, const float* node_sumexp /*[B,N]*/,
                                 const float* probs_ssm /*[R,V]*/, int32_t R, const int32_t* ssm_row /*[B,N]*/,
                                 const int32_t* tree_token, const int32_t* tree_parent, const float* u_accept,
                                 const float* u_order, const float* u_final, float temperature, int32_t Lmax,
                                 int32_t* accepted_path, int32_t* accepted_len, int32_t* out_tokens, void* workspace,
                                 size_t workspace_bytes, int32_t* status, void* hip_stream);

/*
 * KV commit (Algorithm 2 main loop: every verified token is appended to the sequence, so the accepted
 * path's K/V must become the contiguous continuation of the prefix). For every layer l, request b,
 * head h and k in [0, accepted_len[b]):
 *     cache_l[b, h, prefix_len[b] + k, :] = cache_l[b, h, prefix_len[b] + accepted_path[b,k], :]
 * (K and V, bit copy), and prefix_len_out[b] = prefix_len[b] + accepted_len[b]. Source rows are read
 * before any destination row that could alias them is written. Rows at and beyond the new prefix
 * length are unspecified afterwards. A malformed path (SPEC_ST_BAD_PATH) leaves the request's caches
 * untouched and prefix_len_out[b] = prefix_len[b].
 * k_caches / v_caches: HOST arrays of n_layers device pointers (n_layers <= SPEC_MAX_COMMIT_LAYERS),
 * read during the call. prefix_len_out must not alias prefix_len.
 */
int spec_kv_commit(const spec_attn_desc_t* desc, int32_t n_layers, void* const* k_caches /*host*/,
                   void* const* v_caches /*host*/, const int32_t* accepted_path /*[B,Lmax]*/,
                   int32_t Lmax, const int32_t* accepted_len /*[B]*/, const int32_t* prefix_len /*[B]*/,
                   int32_t* prefix_len_out /*[B]*/, int32_t* status, void* hip_stream);

/*
 * LM head in front of the greedy verifier (Algorithm 2, VerifyGreedy: O(u) is the arg-max of the LLM's
 * distribution at node u, so greedy verification needs no logits in memory). For every row m of `hidden`:
 *     node_argmax[m] = argmax_v  sum_k hidden[m,k] * weight[v,k]    (lowest v among equal maxima),
 *     node_max[m]    = that maximum (float32; may be NULL),
 * hidden [M,K] and weight [V,K] bf16, K contiguous (the layout of a linear layer's weight), K a multiple of
 * 256, both 16-byte aligned; products accumulate in float32 on the matrix cores, so two logits closer than
 * float32 rounding of the sum may compare either way. Built for the few hundred rows of a verification
 * pass (M = B*N), where the product is bound by one pass over `weight`; larger M is served in slices of
 * 128 rows, each streaming `weight` again.
 * spec_verify_greedy_lm_head = this (M = B*N, row b*N + u is node u of request b) followed by the walk of
 * spec_verify_greedy; node_argmax [B,N] may be NULL (then it lives in the workspace).
 * workspace: spec_lm_head_argmax_workspace_bytes(M, V) bytes, 256-byte aligned; contents are scratch.
 */
size_t spec_lm_head_argmax_workspace_bytes(int32_t M, int32_t V);
int spec_lm_head_argmax(int32_t M, int32_t K, int32_t V, const void* hidden, const void* weight,
                        int32_t* node_argmax /*[M]*/, float* node_max /*[M] or NULL*/, void* workspace,
                        size_t workspace_bytes, void* hip_stream);
int spec_verify_greedy_lm_head(int32_t B, int32_t N, int32_t K, int32_t V, const void* hidden /*[B*N,K]*/,
                               const void* weight /*[V,K]*/, const int32_t* tree_token, const int32_t* tree_parent,
                               int32_t Lmax, int32_t* accepted_path, int32_t* accepted_len, int32_t* out_tokens,
                               int32_t* node_argmax /*[B,N] or NULL*/, void* workspace, size_t workspace_bytes,
                               int32_t* status, void* hip_stream);

/*
 * LM head in front of the stochastic verifiers (Algorithm 2, VerifyStochastic: P(x | u, LLM) = softmax of the
 * LLM's logits at node u). One pass over `weight` that writes the logits, rounded to bf16, and the per-row
 * statistics of the ROUNDED values that spec_verify_stochastic_stats starts from:
 *     logits[m,v]    = bf16( sum_k hidden[m,k] * weight[v,k] )            [M,V] contiguous
 *     node_max[m]    = max_v logits[m,v],  node_argmax[m] = its lowest v (may be NULL)
 *     node_sumexp[m] = sum_v exp((logits[m,v] - node_max[m]) / temperature)          (float32)
 * Shapes, alignment and accumulation as for spec_lm_head_argmax. temperature > 0.
 * workspace: spec_lm_head_logits_stats_workspace_bytes(M, V) bytes, 256-byte aligned; contents are scratch.
 */
size_t spec_lm_head_logits_stats_workspace_bytes(int32_t M, int32_t V);
int spec_lm_head_logits_stats(int32_t M, int32_t K, int32_t V, const void* hidden, const void* weight,
                              float temperature, void* logits /*[M,V] bf16*/, int32_t* node_argmax /*[M] or NULL*/,
                              float* node_max /*[M]*/, float* node_sumexp /*[M]*/, void* workspace,
                              size_t workspace_bytes, void* hip_stream);

/*
 * Paged KV caches (beyond the paper, whose cache is one contiguous region per request; the steps are
 * those of Section 4.2 and Algorithm 2 unchanged, only the place of a cache row differs). Each cache is
 * a pool of n_blocks blocks of block_tokens rows, [n_blocks, H_kv, block_tokens, D]: in the descriptor
 * kv_stride_b is the stride between BLOCKS, kv_stride_h / kv_stride_s those inside a block, and S_cap the
 * logical capacity of a request in rows (S_cap <= max_blocks * block_tokens). Logical row s of request b
 * is row s % block_tokens of block block_table[b, s / block_tokens]; every call below is its contiguous
 * namesake with that one substitution. Requests may share blocks they only read (a common prefix);
 * rows a call writes (appended rows, committed rows) must lie in blocks no other request of the call
 * uses. A table entry outside [0, n_blocks) among the blocks a request uses sets SPEC_ST_BAD_BLOCK:
 * rows of such a block are never written, reads are redirected to a block inside the pool, and the
 * request's outputs are unspecified; no memory outside the caches is touched. Entries of blocks a
 * request does not reach (beyond prefix_len[b] + N rows) may hold any value. bf16 attention reads one
 * table entry per key tile; next to the contiguous calls this costs about 5 % on short prefixes and
 * nothing measurable on long ones.
 */
typedef struct spec_kv_pages {
  const int32_t* block_table; /* DEVICE, [B, max_blocks]: physical block of each logical block        */
  int32_t max_blocks;         /* row length of block_table                                            */
  int32_t block_tokens;       /* rows per block: a power of two, 64 .. 65536                          */
  int32_t n_blocks;           /* blocks in each cache                                                 */
} spec_kv_pages_t;

int spec_kv_append_paged(const spec_attn_desc_t* desc, const spec_kv_pages_t* pages, const void* k_new,
                         const void* v_new, void* k_cache, void* v_cache, const int32_t* prefix_len,
                         int32_t* status, void* hip_stream);
int spec_kv_append_rope_paged(const spec_attn_desc_t* desc, const spec_kv_pages_t* pages, const void* k_new,
                              const void* v_new, void* k_cache, void* v_cache, const int32_t* tree_depth,
                              const int32_t* prefix_len, const float* rope_cos, const float* rope_sin,
                              int32_t rope_len, int32_t* status, void* hip_stream);
int spec_qk_rope_append_paged(const spec_attn_desc_t* desc, const spec_kv_pages_t* pages, void* q, const void* k_new,
                              const void* v_new, void* k_cache, void* v_cache, const int32_t* tree_depth,
                              const int32_t* prefix_len, const float* rope_cos, const float* rope_sin,
                              int32_t rope_len, int32_t* status, void* hip_stream);
int spec_tree_attention_paged(const spec_attn_desc_t* desc, const spec_kv_pages_t* pages, const void* q,
                              const void* k_cache, const void* v_cache, const int32_t* tree_parent,
                              const int32_t* tree_depth, const int32_t* prefix_len, void* out, void* workspace,
                              size_t workspace_bytes, int32_t* status, void* hip_stream);
int spec_tree_attention_append_paged(const spec_attn_desc_t* desc, const spec_kv_pages_t* pages, const void* q,
                                     const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                                     const int32_t* tree_parent, const int32_t* tree_depth,
                                     const int32_t* prefix_len, void* out, void* workspace, size_t workspace_bytes,
                                     int32_t* status, void* hip_stream);
int spec_tree_attention_append_rope_paged(const spec_attn_desc_t* desc, const spec_kv_pages_t* pages, const void* q,
                                          const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                                          const int32_t* tree_parent, const int32_t* tree_depth,
                                          const int32_t* prefix_len, const float* rope_cos, const float* rope_sin,
                                          int32_t rope_len, void* out, void* workspace, size_t workspace_bytes,
                                          int32_t* status, void* hip_stream);
/* workspace of the paged attention calls (the launch plan of a paged call may differ) */
size_t spec_tree_attention_paged_workspace_bytes(const spec_attn_desc_t* desc, const spec_kv_pages_t* pages);
int spec_kv_commit_paged(const spec_attn_desc_t* desc, const spec_kv_pages_t* pages, int32_t n_layers,
                         void* const* k_caches /*host*/, void* const* v_caches /*host*/,
                         const int32_t* accepted_path, int32_t Lmax, const int32_t* accepted_len,
                         const int32_t* prefix_len, int32_t* prefix_len_out, int32_t* status, void* hip_stream);

/* Text for a SPEC_ERR_* code (static storage). Library version as major*10000 + minor*100 + patch. */

const char* spec_strerror(int code);
int spec_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPEC_TREE_H */
