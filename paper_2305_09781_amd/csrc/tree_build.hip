// Token-tree construction on the GPU (Section 3), the step right before verification, so that the
// speculated tree never visits the host:
//   expand_topk_kernel   one step of expansion-based construction: the k most likely next tokens of every
//                        frontier node (most likely first, ties to the lowest token id), written to the
//                        tree's token array at the slots the static expansion configuration assigns.
//   tree_merge_kernel    token tree merge (Definition 3.2): the M trees of a request become one tree that
//                        holds exactly their token sequences, numbered depth-first.
// Both are small integer / comparison kernels: one workgroup per row or per request.
#include <hip/hip_bf16.h>

#include "spec_internal.h"

namespace spec {

constexpr int TOPK_THREADS = 1024;
constexpr int MERGE_THREADS = SPEC_MAX_MERGE_INPUT_NODES;

// ---------------------------------------------------------------------------------------------
// top-k of one row of V logits by k rounds of a block-wide arg-max. Round j only considers elements that
// come after the previous pick in the order (value descending, token id ascending), so the picks are
// that order's first k elements and no set of picked ids has to be kept.
// ---------------------------------------------------------------------------------------------
template <bool BF16>
__global__ void __launch_bounds__(TOPK_THREADS) expand_topk_kernel(const void* __restrict__ logits, int F, int V, int k,
                                                                   const int32_t* __restrict__ child_slot, int N,
                                                                   int32_t* __restrict__ tree_token, int32_t* status) {
  __shared__ float s_val[TOPK_THREADS / 64];
  __shared__ int s_idx[TOPK_THREADS / 64];
  const int row = blockIdx.x, b = row / F, f = row % F, t = threadIdx.x;
  const long base = (long)row * V;
  float prev_v = INFINITY;
  int prev_i = -1;
  for (int j = 0; j < k; ++j) {
    float best = -INFINITY;
    int best_i = 0x7fffffff;
    for (int i = t; i < V; i += TOPK_THREADS) {
      const float x = BF16 ? __bfloat162float(((const __hip_bfloat16*)logits)[base + i]) : ((const float*)logits)[base + i];
      const bool eligible = (x < prev_v) || (x == prev_v && i > prev_i);
      if (eligible && (x > best || (x == best && i < best_i))) { best = x; best_i = i; }
    }
    for (int o = 32; o > 0; o >>= 1) {
      const float ov = __shfl_xor(best, o);
      const int oi = __shfl_xor(best_i, o);
      if (oi != 0x7fffffff && (best_i == 0x7fffffff || ov > best || (ov == best && oi < best_i))) { best = ov; best_i = oi; }
    }
    __syncthreads();
    if ((t & 63) == 0) { s_val[t >> 6] = best; s_idx[t >> 6] = best_i; }
    __syncthreads();
    best = s_val[0];
    best_i = s_idx[0];
    for (int w = 1; w < TOPK_THREADS / 64; ++w) {
      const float ov = s_val[w];
      const int oi = s_idx[w];
      if (oi != 0x7fffffff && (best_i == 0x7fffffff || ov > best || (ov == best && oi < best_i))) { best = ov; best_i = oi; }
    }
    if (t == 0) {
      const int slot = child_slot[f * k + j];
      if (slot >= 0 && slot < N) tree_token[(long)b * N + slot] = best_i == 0x7fffffff ? -1 : best_i;   // fewer than k finite logits: padding
      else set_status(status, b, SPEC_ST_BAD_TREE);
    }
    prev_v = best;
    prev_i = best_i;
  }
}

// ---------------------------------------------------------------------------------------------
// token tree merge: one workgroup per request, thread g = i * Nin + u stands for node u of input tree i.
// Two input nodes are the same merged node iff they carry the same token and their parents are the same
// merged node; the representative of a merged node is its input node with the smallest g (first
// appearance), which also orders siblings. Levels are resolved top-down (a node's identity needs its
// parent's), sub-tree sizes bottom-up, depth-first positions top-down.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(MERGE_THREADS) tree_merge_kernel(
    int M, int Nin, const int32_t* __restrict__ in_parent, const int32_t* __restrict__ in_token,
    const int32_t* __restrict__ in_size, int Nout, int32_t* __restrict__ out_parent, int32_t* __restrict__ out_depth,
    int32_t* __restrict__ out_token, int32_t* __restrict__ out_ssm, int32_t* __restrict__ out_size,
    int32_t* __restrict__ node_map, int32_t* status) {
  __shared__ int s_par[MERGE_THREADS];     // parent as a thread index g (-1 for roots)
  __shared__ int s_tok[MERGE_THREADS];
  __shared__ int s_dep[MERGE_THREADS];     // depth, -1 for unused slots
  __shared__ int s_rep[MERGE_THREADS];     // representative (smallest g of the same merged node)
  __shared__ int s_rank[MERGE_THREADS];    // rank among the nodes of the same depth, by g
  __shared__ int s_lvl[MERGE_THREADS];     // nodes sorted by (depth, g)
  __shared__ int s_sub[MERGE_THREADS];     // sub-tree size of a representative
  __shared__ int s_pos[MERGE_THREADS];     // depth-first index of a representative
  __shared__ int s_lvl_count[SPEC_MAX_MERGE_INPUT_NODES + 1];
  __shared__ int s_lvl_start[SPEC_MAX_MERGE_INPUT_NODES + 2];
  __shared__ int s_bad, s_max_depth, s_size;

  const int b = blockIdx.x, g = threadIdx.x;
  const int n_total = M * Nin;
  const int i = g / Nin, u = g % Nin;
  const int32_t* par_b = in_parent + (long)b * n_total;
  const int32_t* tok_b = in_token + (long)b * n_total;
  if (g == 0) { s_bad = 0; s_max_depth = 0; s_size = 0; }
  for (int d = g; d <= SPEC_MAX_MERGE_INPUT_NODES; d += MERGE_THREADS) s_lvl_count[d] = 0;
  __syncthreads();

  // ---- load and validate
  bool active = false;
  int my_tok = -1, my_par = -1;
  if (g < n_total) {
    const int sz = in_size[(long)b * M + i];
    if (u == 0 && (sz < 1 || sz > Nin)) atomicOr(&s_bad, 1);
    active = u < sz && sz <= Nin;
    if (active) {
      const int p = par_b[g];
      my_tok = tok_b[g];
      if (u == 0) {
        if (p != -1 || my_tok != tok_b[0]) atomicOr(&s_bad, 1);
      } else {
        if (p < 0 || p >= u || my_tok < 0) atomicOr(&s_bad, 1);
        my_par = i * Nin + p;
      }
    }
  }
  s_par[g] = my_par;
  s_tok[g] = my_tok;
  s_dep[g] = -1;
  __syncthreads();
  const bool bad = s_bad != 0;

  // ---- depth (walk up; parents have smaller indices, so the walk ends), level lists
  int my_dep = -1;
  if (active && !bad) {
    my_dep = 0;
    for (int v = my_par; v >= 0; v = s_par[v]) ++my_dep;
    s_dep[g] = my_dep;
    atomicAdd(&s_lvl_count[my_dep], 1);
    atomicMax(&s_max_depth, my_dep);
  }
  __syncthreads();
  const int max_depth = s_max_depth;
  if (g == 0) {
    int acc = 0;
    for (int d = 0; d <= max_depth; ++d) { s_lvl_start[d] = acc; acc += s_lvl_count[d]; }
    s_lvl_start[max_depth + 1] = acc;
  }
  int my_rank = 0;
  if (my_dep >= 0)
    for (int o = 0; o < g; ++o) my_rank += s_dep[o] == my_dep;
  s_rank[g] = my_rank;
  __syncthreads();
  if (my_dep >= 0) s_lvl[s_lvl_start[my_dep] + my_rank] = g;
  s_rep[g] = (my_dep == 0) ? 0 : g;   // every root is the merged root, first seen as thread 0
  s_sub[g] = 1;
  __syncthreads();

  // ---- identity, level by level
  for (int d = 1; d <= max_depth; ++d) {
    if (my_dep == d) {
      const int pr = s_rep[my_par];
      const int start = s_lvl_start[d];
      for (int j = 0; j < my_rank; ++j) {
        const int o = s_lvl[start + j];
        if (s_tok[o] == my_tok && s_rep[s_par[o]] == pr) { s_rep[g] = o; break; }   // the first match has the smallest index
      }
    }
    __syncthreads();
  }
  const bool is_rep = my_dep >= 0 && s_rep[g] == g && (my_dep > 0 || g == 0);
  if (is_rep) atomicAdd(&s_size, 1);
  __syncthreads();
  const int size = s_size;
  const bool overflow = size > Nout;

  if (bad || overflow) {   // defined result: an empty tree (root slot and padding), size 0, everything unmapped
    for (int n = g; n < Nout; n += MERGE_THREADS) {
      out_parent[(long)b * Nout + n] = n == 0 ? -1 : 0;
      out_depth[(long)b * Nout + n] = n == 0 ? 0 : 1;
      out_token[(long)b * Nout + n] = -1;
      out_ssm[(long)b * Nout + n] = -1;
    }
    if (node_map != nullptr && g < n_total) node_map[(long)b * n_total + g] = -1;
    if (g == 0) {
      out_size[b] = 0;
      set_status(status, b, bad ? SPEC_ST_BAD_TREE : SPEC_ST_CAPACITY);
    }
    return;
  }

  // ---- sub-tree sizes, bottom-up
  for (int d = max_depth; d >= 1; --d) {
    if (is_rep && my_dep == d) atomicAdd(&s_sub[s_rep[my_par]], s_sub[g]);
    __syncthreads();
  }
  // ---- depth-first positions, top-down: after the parent, behind the sub-trees of the earlier siblings
  if (g == 0) s_pos[0] = 0;
  __syncthreads();
  for (int d = 1; d <= max_depth; ++d) {
    if (is_rep && my_dep == d) {
      const int pr = s_rep[my_par];
      int pos = s_pos[pr] + 1;
      const int start = s_lvl_start[d];
      for (int j = 0; j < my_rank; ++j) {
        const int o = s_lvl[start + j];
        if (s_rep[o] == o && s_rep[s_par[o]] == pr) pos += s_sub[o];
      }
      s_pos[g] = pos;
    }
    __syncthreads();
  }

  // ---- outputs
  if (is_rep) {
    const long n = (long)b * Nout + s_pos[g];
    out_parent[n] = my_dep == 0 ? -1 : s_pos[s_rep[my_par]];
    out_depth[n] = my_dep;
    out_token[n] = my_tok;
    out_ssm[n] = i;
  }
  for (int n = size + g; n < Nout; n += MERGE_THREADS) {   // padding nodes: children of the root without a token
    out_parent[(long)b * Nout + n] = 0;
    out_depth[(long)b * Nout + n] = 1;
    out_token[(long)b * Nout + n] = -1;
    out_ssm[(long)b * Nout + n] = -1;
  }
  if (node_map != nullptr && g < n_total) node_map[(long)b * n_total + g] = my_dep >= 0 ? s_pos[s_rep[g]] : -1;
  if (g == 0) out_size[b] = size;
}

hipError_t launch_expand_topk(int B, int F, int V, int logits_dtype, const void* logits, int k, const int32_t* child_slot,
                              int N, int32_t* tree_token, int32_t* status, hipStream_t s) {
  if (logits_dtype == SPEC_BF16)
    hipLaunchKernelGGL(expand_topk_kernel<true>, dim3(B * F), dim3(TOPK_THREADS), 0, s, logits, F, V, k, child_slot, N,
                       tree_token, status);
  else
    hipLaunchKernelGGL(expand_topk_kernel<false>, dim3(B * F), dim3(TOPK_THREADS), 0, s, logits, F, V, k, child_slot, N,
                       tree_token, status);
  return hipGetLastError();
}

hipError_t launch_tree_merge(int B, int M, int Nin, const int32_t* in_parent, const int32_t* in_token,
                             const int32_t* in_size, int Nout, int32_t* out_parent, int32_t* out_depth,
                             int32_t* out_token, int32_t* out_ssm, int32_t* out_size, int32_t* node_map, int32_t* status,
                             hipStream_t s) {
  hipLaunchKernelGGL(tree_merge_kernel, dim3(B), dim3(MERGE_THREADS), 0, s, M, Nin, in_parent, in_token, in_size, Nout,
                     out_parent, out_depth, out_token, out_ssm, out_size, node_map, status);
  return hipGetLastError();
}

}  // namespace spec
