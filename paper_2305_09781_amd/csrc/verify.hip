// Token-tree verification on the GPU (Algorithm 2: VerifyGreedy and VerifyStochastic, Section 4.3).
//
// The paper runs verification on the host after copying the LLM's per-node outputs back; here it
// stays on the device so an iteration needs no host round trip. Three kernels:
//   node_stats_kernel      one workgroup per (request, node) row of logits: argmax (lowest token id on
//                          ties), max, and sum of exp((x - max)/T). All nodes in parallel, so the
//                          sequential tree walk that follows needs P(x) at a node in O(1).
//   greedy_walk_kernel     one workgroup per request: follow children whose token equals the node's
//                          argmax; emit the bonus token.
//   stochastic_walk_kernel one workgroup per request: multi-step speculative sampling. The first ratio
//                          test at a node uses the precomputed softmax statistics; only a rejection
//                          materialises the residual distribution norm(max(0, P - Q)) (one pass over
//                          the vocabulary per rejection, kept un-normalised with its mass Z). The last
//                          token is drawn by inverse CDF with a float64 block scan in token-id order.
//   node_sample_kernel     naive sampling (the alternative of Section 4.3): one inverse-CDF draw per
//                          (request, node) row; the greedy walk then runs on the sampled tokens.
#include <hip/hip_bf16.h>

#include "spec_internal.h"

namespace spec {

template <bool BF16>
__device__ inline float load_logit(const void* base, long idx) {
  if (BF16) return __bfloat162float(((const __hip_bfloat16*)base)[idx]);
  return ((const float*)base)[idx];
}

// ---------------------------------------------------------------------------------------------
// Vocabulary sweeps. A row of V values is visited in groups of VEC consecutive elements (VEC = 4 when
// V is a multiple of 4, so that every group is one aligned 16-byte (float) or 8-byte (bf16) access;
// else 1). A block of NT threads takes U groups per thread at a time, all loads issued before any is
// used: with V = 32000, NT = 1024, U = 8 a whole row is one round trip to memory.
// ---------------------------------------------------------------------------------------------
constexpr int SWEEP_U = 8;

template <int VEC, bool BF16>
__device__ __forceinline__ void load_logit_group(const void* base, long elem, float (&v)[VEC]) {
  if (VEC == 4) {
    if (BF16) {
      const uint2 raw = *(const uint2*)((const __hip_bfloat16*)base + elem);
      v[0] = __uint_as_float(raw.x << 16);
      v[1] = __uint_as_float(raw.x & 0xffff0000u);
      v[2] = __uint_as_float(raw.y << 16);
      v[3] = __uint_as_float(raw.y & 0xffff0000u);
    } else {
      const float4 raw = *(const float4*)((const float*)base + elem);
      v[0] = raw.x; v[1] = raw.y; v[2] = raw.z; v[3] = raw.w;
    }
  } else {
    v[0] = load_logit<BF16>(base, elem);
  }
}
template <int VEC>
__device__ __forceinline__ void load_f32_group(const float* p, float (&v)[VEC]) {
  if (VEC == 4) {
    const float4 raw = *(const float4*)p;
    v[0] = raw.x; v[1] = raw.y; v[2] = raw.z; v[3] = raw.w;
  } else {
    v[0] = *p;
  }
}
template <int VEC>
__device__ __forceinline__ void store_f32_group(float* p, const float (&v)[VEC]) {
  if (VEC == 4) *(float4*)p = make_float4(v[0], v[1], v[2], v[3]);
  else *p = v[0];
}

// ---------------------------------------------------------------------------------------------
// block-wide reductions (blockDim.x multiple of 64, <= 1024); `scratch` holds >= 16 entries
// ---------------------------------------------------------------------------------------------
template <typename T>
__device__ inline T block_sum(T v, T* scratch) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) scratch[w] = v;
  __syncthreads();
  T tot = 0;
  for (int i = 0; i < nw; ++i) tot += scratch[i];
  return tot;
}

// ---------------------------------------------------------------------------------------------
// per-node statistics: one block of 1024 threads per (request, node) row, one pass over the row.
// Each thread keeps (max, lowest index of the max, sum of exp((x - max) / T)) of its elements; the
// block combines the triples.
// ---------------------------------------------------------------------------------------------
// Workgroup size: 1024 threads when there are few rows (a row is then one round trip to memory), 256 when there
// are thousands: eight small workgroups per compute unit overlap one another's loads and arithmetic, where two
// large ones alternate between a load phase and a compute phase (2048 rows of 32000 floats: 61 us before).

// exp(x) for x <= 0 as one v_exp_f32 (1 ulp; results below 2^-126 become 0). The sum over a vocabulary row is
// bound by this instruction count: the library expf costs about ten instructions per element, and the
// statistics kernel ran at half the speed of its max-only form with it.
__device__ __forceinline__ float fast_exp(float x) { return __builtin_amdgcn_exp2f(x * 1.4426950408889634f); }

template <bool BF16, int VEC, int NS_THREADS>
__global__ void __launch_bounds__(NS_THREADS) node_stats_kernel(const void* __restrict__ logits, int V, float inv_temp,
                                                                int32_t* __restrict__ node_argmax,
                                                                float* __restrict__ node_max,
                                                                float* __restrict__ node_sumexp) {
  __shared__ float s_val[NS_THREADS / 64];
  __shared__ int s_idx[NS_THREADS / 64];
  __shared__ float s_sum[NS_THREADS / 64];
  const long row = blockIdx.x;
  const int t = threadIdx.x;
  const long base = row * V;
  const int n_groups = V / VEC;
  const bool want_sum = node_sumexp != nullptr;
  float best = -INFINITY, sum = 0.f;
  int best_i = 0x7fffffff;
  for (int g0 = 0; g0 < n_groups; g0 += NS_THREADS * SWEEP_U) {
    float x[SWEEP_U][VEC];
#pragma unroll
    for (int j = 0; j < SWEEP_U; ++j) {
      const int gi = g0 + j * NS_THREADS + t;
      if (gi < n_groups) {
        load_logit_group<VEC, BF16>(logits, base + (long)gi * VEC, x[j]);
      } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) x[j][e] = -INFINITY;
      }
    }
    float m = best;
#pragma unroll
    for (int j = 0; j < SWEEP_U; ++j)
#pragma unroll
      for (int e = 0; e < VEC; ++e)
        if (x[j][e] > m) { m = x[j][e]; best_i = (g0 + j * NS_THREADS + t) * VEC + e; }   // ascending index: lowest wins ties
    if (want_sum && m > -INFINITY) {
      sum *= fast_exp((best - m) * inv_temp);     // best = -inf gives 0
#pragma unroll
      for (int j = 0; j < SWEEP_U; ++j)
#pragma unroll
        for (int e = 0; e < VEC; ++e) sum += fast_exp((x[j][e] - m) * inv_temp);   // padding: exp(-inf) = 0
    }
    best = m;
  }
  // combine (value desc, index asc); sums are rescaled to the common maximum
  const float my_best = best;
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(best, o);
    const int oi = __shfl_xor(best_i, o);
    if (ov > best || (ov == best && oi < best_i)) { best = ov; best_i = oi; }
  }
  if ((t & 63) == 0) { s_val[t >> 6] = best; s_idx[t >> 6] = best_i; }
  __syncthreads();
  best = s_val[0]; best_i = s_idx[0];
  for (int w = 1; w < NS_THREADS / 64; ++w)
    if (s_val[w] > best || (s_val[w] == best && s_idx[w] < best_i)) { best = s_val[w]; best_i = s_idx[w]; }
  if (best_i == 0x7fffffff) best_i = 0;   // all -inf / NaN row
  if (want_sum) {
    if (my_best > -INFINITY) sum *= fast_exp((my_best - best) * inv_temp); else sum = 0.f;
    sum = block_sum(sum, s_sum);
  }
  if (t == 0) {
    if (node_argmax != nullptr) node_argmax[row] = best_i;
    if (node_max != nullptr) node_max[row] = best;
    if (want_sum) node_sumexp[row] = sum;
  }
}

// ---------------------------------------------------------------------------------------------
// Inverse-CDF draw by a block of SW_THREADS threads over V weights in ascending token id:
// w_i = exp((logits[lrow + i] - mx) * inv_temp) (implicit) or resid[i]. Every thread owns a contiguous
// range and sums its weights in float64; a block scan finds the thread whose range holds the target
// r * total, which then walks its range in order. Returns, to every thread, the first index whose
// inclusive sum exceeds the target (V - 1 if rounding leaves none).
// ---------------------------------------------------------------------------------------------
constexpr int SW_THREADS = 1024;

template <bool BF16, int VEC>
__device__ inline int inverse_cdf_draw(const void* __restrict__ logits, long lrow, const float* resid, bool implicit,
                                       float mx, float inv_temp, int V, float r, double* s_scan, int* s_pick, int* s_ans) {
  const int t = threadIdx.x;
  const int n_groups = V / VEC;
  const int per_thread = ((V + SW_THREADS - 1) / SW_THREADS + VEC - 1) / VEC;    // groups per thread
  const int g_lo = min(t * per_thread, n_groups), g_hi = min(g_lo + per_thread, n_groups);
  double mine = 0.0;
  for (int g0 = g_lo; g0 < g_hi; g0 += SWEEP_U) {
    float w[SWEEP_U][VEC];
#pragma unroll
    for (int jj = 0; jj < SWEEP_U; ++jj)
      if (g0 + jj < g_hi) {
        if (implicit) load_logit_group<VEC, BF16>(logits, lrow + (long)(g0 + jj) * VEC, w[jj]);
        else load_f32_group<VEC>(resid + (long)(g0 + jj) * VEC, w[jj]);
      }
#pragma unroll
    for (int jj = 0; jj < SWEEP_U; ++jj)
      if (g0 + jj < g_hi) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) mine += (double)(implicit ? expf((w[jj][e] - mx) * inv_temp) : w[jj][e]);
      }
  }
  // inclusive scan over threads: wave-level shuffles, then wave totals
  double incl = mine;
  const int lane = t & 63, wv = t >> 6;
  for (int o = 1; o < 64; o <<= 1) {
    const double up = __shfl_up(incl, o);
    if (lane >= o) incl += up;
  }
  __syncthreads();   // earlier readers of the shared slots are done
  if (lane == 63) s_scan[wv] = incl;
  if (t == 0) { *s_pick = 0x7fffffff; *s_ans = V - 1; }
  __syncthreads();
  double before = 0.0, total = 0.0;
  for (int w = 0; w < SW_THREADS / 64; ++w) {
    if (w < wv) before += s_scan[w];
    total += s_scan[w];
  }
  incl += before;
  const double excl = incl - mine;
  const double target = (double)r * total;
  // the first thread whose inclusive sum exceeds the target holds the answer
  if (incl > target && excl <= target && g_hi > g_lo) atomicMin(s_pick, t);
  __syncthreads();
  if (t == *s_pick) {
    double run = excl;
    int ans = g_hi * VEC - 1;
    for (int i = g_lo * VEC; i < g_hi * VEC; ++i) {
      const float w = implicit ? expf((load_logit<BF16>(logits, lrow + i) - mx) * inv_temp) : resid[i];
      run += (double)w;
      if (run > target) { ans = i; break; }
    }
    *s_ans = ans;
  }
  __syncthreads();
  return *s_ans;
}

// ---------------------------------------------------------------------------------------------
// greedy walk: blockDim = 128, thread v <-> node v
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(128) greedy_walk_kernel(int N, const int32_t* __restrict__ node_argmax,
                                                          const int32_t* __restrict__ token,
                                                          const int32_t* __restrict__ parent, int Lmax,
                                                          int32_t* __restrict__ path, int32_t* __restrict__ len,
                                                          int32_t* __restrict__ out_tokens, int32_t* status) {
  __shared__ int s_next;
  __shared__ int s_flag;
  const int b = blockIdx.x, v = threadIdx.x;
  const bool valid = tree_is_valid(parent + (long)b * N, nullptr, N, &s_flag);
  for (int k = v; k < Lmax; k += 128) {
    path[(long)b * Lmax + k] = -1;
    out_tokens[(long)b * Lmax + k] = -1;
  }
  if (!valid) {
    if (v == 0) { len[b] = 0; set_status(status, b, SPEC_ST_BAD_TREE); }
    return;
  }
  const int my_parent = v < N ? parent[(long)b * N + v] : -2;
  const int my_token = v < N ? token[(long)b * N + v] : -1;
  __syncthreads();   // padding writes above are ordered before the walk's writes (same block)
  int u = 0, k = 0;
  if (v == 0) path[(long)b * Lmax] = 0;
  while (k + 1 < Lmax) {
    if (v == 0) s_next = 0x7fffffff;
    __syncthreads();
    const int want = node_argmax[(long)b * N + u];
    if (my_parent == u && my_token == want) atomicMin(&s_next, v);
    __syncthreads();
    const int nxt = s_next;
    __syncthreads();
    if (nxt == 0x7fffffff) break;
    if (v == 0) {
      out_tokens[(long)b * Lmax + k] = token[(long)b * N + nxt];
      path[(long)b * Lmax + k + 1] = nxt;
    }
    ++k;
    u = nxt;
  }
  if (v == 0) {
    out_tokens[(long)b * Lmax + k] = node_argmax[(long)b * N + u];
    len[b] = k + 1;
  }
}

// ---------------------------------------------------------------------------------------------
// stochastic walk: blockDim = 1024
// ---------------------------------------------------------------------------------------------

template <bool BF16, int VEC>
__global__ void __launch_bounds__(SW_THREADS) stochastic_walk_kernel(
    int N, int V, const void* __restrict__ logits, const float* __restrict__ probs_ssm, int R,
    const int32_t* __restrict__ ssm_row, const int32_t* __restrict__ token, const int32_t* __restrict__ parent,
    const float* __restrict__ u_accept, const float* __restrict__ u_order, const float* __restrict__ u_final,
    float inv_temp, const float* __restrict__ node_max, const float* __restrict__ node_sumexp, float* resid_all, int Lmax,
    int32_t* __restrict__ path, int32_t* __restrict__ len, int32_t* __restrict__ out_tokens, int32_t* status) {
  __shared__ int s_flag;
  __shared__ int s_child[SPEC_MAX_TREE_NODES];
  __shared__ int s_sorted[SPEC_MAX_TREE_NODES];
  __shared__ int s_cx[SPEC_MAX_TREE_NODES];       // per child in test order: its token,
  __shared__ float s_cq[SPEC_MAX_TREE_NODES];     // the draft's probability of that token,
  __shared__ float s_cl[SPEC_MAX_TREE_NODES];     // the LLM's logit of that token at u,
  __shared__ float s_cr[SPEC_MAX_TREE_NODES];     // and the child's uniform
  __shared__ int s_nchild;
  __shared__ float s_fsum[SW_THREADS / 64];
  __shared__ double s_scan[SW_THREADS / 64];
  __shared__ int s_pick, s_ans;

  const int b = blockIdx.x, t = threadIdx.x;
  float* resid0 = resid_all + (long)b * V;
  float* resid1 = resid_all + ((long)gridDim.x + b) * V;
  float* resid = resid0;
  int cur = 0;   // resid == (cur ? resid1 : resid0)
  const int32_t* par = parent + (long)b * N;
  const int32_t* tok = token + (long)b * N;
  const int n_groups = V / VEC;

  bool valid = tree_is_valid(par, nullptr, N, &s_flag);
  __syncthreads();
  if (t == 0) s_flag = 0;
  __syncthreads();
  if (valid && t >= 1 && t < N) {   // a negative token marks a padding node: never a candidate, nothing to check
    const int x = tok[t], r = ssm_row[(long)b * N + t];
    if (x >= 0 && (x >= V || r < 0 || r >= R)) atomicOr(&s_flag, 1);
  }
  __syncthreads();
  valid = valid && (s_flag == 0);
  for (int k = t; k < Lmax; k += SW_THREADS) {
    path[(long)b * Lmax + k] = -1;
    out_tokens[(long)b * Lmax + k] = -1;
  }
  if (!valid) {
    if (t == 0) { len[b] = 0; set_status(status, b, SPEC_ST_BAD_TREE); }
    return;
  }
  __syncthreads();
  if (t == 0) path[(long)b * Lmax] = 0;

  int u = 0, k = 0;
  bool implicit = true;   // current P is softmax(logits[u]) given by (node_max, node_sumexp); else resid / Z
  float Z = 1.f;
  float mx = node_max[(long)b * N], se = node_sumexp[(long)b * N];
  while (true) {
    // children of u in ascending (u_order, index)
    if (t == 0) s_nchild = 0;
    __syncthreads();
    if (t < N && par[t] == u && tok[t] >= 0) s_child[atomicAdd(&s_nchild, 1)] = t;
    __syncthreads();
    const int nchild = (k + 1 < Lmax) ? s_nchild : 0;
    if (nchild == 0) break;
    if (t < nchild) {
      const int me = s_child[t];
      const float mk = u_order[(long)b * N + me];
      int rank = 0;
      for (int j = 0; j < nchild; ++j) {
        const int o = s_child[j];
        const float ok = u_order[(long)b * N + o];
        rank += (ok < mk) || (ok == mk && o < me);
      }
      s_sorted[rank] = me;
    }
    __syncthreads();
    bool accepted = false;
    int next_u = -1;
    const long lrow = ((long)b * N + u) * V;
    // everything a ratio test needs from memory, for all children at once (one round trip instead of one
    // chain of dependent loads per test)
    if (t < nchild) {
      const int s = s_sorted[t];
      const int x = tok[s];
      s_cx[t] = x;
      s_cq[t] = probs_ssm[(long)ssm_row[(long)b * N + s] * V + x];
      s_cl[t] = load_logit<BF16>(logits, lrow + x);
      s_cr[t] = u_accept[(long)b * N + s];
    }
    __syncthreads();
    for (int j = 0; j < nchild; ++j) {
      const int s = s_sorted[j];
      const int x = s_cx[j];
      const float* Q = probs_ssm + (long)ssm_row[(long)b * N + s] * V;
      const float r = s_cr[j];
      float px;
      if (implicit) px = expf((s_cl[j] - mx) * inv_temp) / se;
      else px = resid[x] / Z;
      if (r * s_cq[j] <= px) {
        accepted = true;
        next_u = s;
        if (t == 0) {
          out_tokens[(long)b * Lmax + k] = x;
          path[(long)b * Lmax + k + 1] = s;
        }
        break;
      }
      // rejected: P := norm(max(0, P - Q)), kept as un-normalised values plus their sum Z. The new
      // residual goes to the other buffer, so an empty residual simply keeps the previous P.
      float* dst = cur ? resid0 : resid1;
      float part = 0.f;
      const float invZ = 1.f / Z, inv_se = 1.f / se;
      for (int g0 = 0; g0 < n_groups; g0 += SW_THREADS * SWEEP_U) {
        float pv[SWEEP_U][VEC], qv[SWEEP_U][VEC];
#pragma unroll
        for (int jj = 0; jj < SWEEP_U; ++jj) {
          const int gi = g0 + jj * SW_THREADS + t;
          if (gi < n_groups) {
            if (implicit) load_logit_group<VEC, BF16>(logits, lrow + (long)gi * VEC, pv[jj]);
            else load_f32_group<VEC>(resid + (long)gi * VEC, pv[jj]);
            load_f32_group<VEC>(Q + (long)gi * VEC, qv[jj]);
          }
        }
#pragma unroll
        for (int jj = 0; jj < SWEEP_U; ++jj) {
          const int gi = g0 + jj * SW_THREADS + t;
          if (gi < n_groups) {
            float d[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
              const float p = implicit ? expf((pv[jj][e] - mx) * inv_temp) * inv_se : pv[jj][e] * invZ;
              d[e] = fmaxf(0.f, p - qv[jj][e]);
              part += d[e];
            }
            store_f32_group<VEC>(dst + (long)gi * VEC, d);
          }
        }
      }
      const float Znew = block_sum(part, s_fsum);
      if (Znew > 0.f) {
        Z = Znew;
        implicit = false;
        resid = dst;
        cur ^= 1;
      } else if (t == 0) {
        set_status(status, b, SPEC_ST_ZERO_RESIDUAL);
      }
      __syncthreads();   // the new residual is visible to every thread before the next test reads it
    }
    if (!accepted) break;
    u = next_u;
    ++k;
    implicit = true;
    resid = resid0;
    cur = 0;
    mx = node_max[(long)b * N + u];
    se = node_sumexp[(long)b * N + u];
    __syncthreads();
  }

  // final token: inverse CDF in ascending token id over the current P
  const int ans = inverse_cdf_draw<BF16, VEC>(logits, ((long)b * N + u) * V, resid, implicit, mx, inv_temp, V, u_final[b],
                                              s_scan, &s_pick, &s_ans);
  if (t == 0) {
    out_tokens[(long)b * Lmax + k] = ans;
    len[b] = k + 1;
  }
}

// ---------------------------------------------------------------------------------------------
// naive sampling (Section 4.3): x_u ~ softmax(logits[u] / T) for every node at once, one block per
// (request, node) row, by inverse CDF with the caller's uniform. The walk that follows is the greedy
// walk on these tokens: move to the child whose token equals x_u, else emit x_u and stop.
// ---------------------------------------------------------------------------------------------
template <bool BF16, int VEC>
__global__ void __launch_bounds__(SW_THREADS) node_sample_kernel(const void* __restrict__ logits, int V, float inv_temp,
                                                                 const float* __restrict__ node_max,
                                                                 const float* __restrict__ u_sample,
                                                                 int32_t* __restrict__ node_sample) {
  __shared__ double s_scan[SW_THREADS / 64];
  __shared__ int s_pick, s_ans;
  const long row = blockIdx.x;
  const int ans = inverse_cdf_draw<BF16, VEC>(logits, row * V, nullptr, true, node_max[row], inv_temp, V, u_sample[row],
                                              s_scan, &s_pick, &s_ans);
  if (threadIdx.x == 0) node_sample[row] = ans;
}

// ---------------------------------------------------------------------------------------------
hipError_t launch_node_stats(int B, int N, int V, int logits_dtype, const void* logits, float inv_temp,
                             int32_t* node_argmax, float* node_max, float* node_sumexp, hipStream_t s) {
  const bool bf16 = logits_dtype == SPEC_BF16, vec = (V % 4 == 0);
  const bool many = (long)B * N >= 1024;
#define SPEC_NS(BF, VE)                                                                                                  \
  if (many)                                                                                                              \
    hipLaunchKernelGGL((node_stats_kernel<BF, VE, 256>), dim3(B * N), dim3(256), 0, s, logits, V, inv_temp, node_argmax,  \
                       node_max, node_sumexp);                                                                           \
  else                                                                                                                   \
    hipLaunchKernelGGL((node_stats_kernel<BF, VE, 1024>), dim3(B * N), dim3(1024), 0, s, logits, V, inv_temp, node_argmax, \
                       node_max, node_sumexp)
  if (bf16 && vec) { SPEC_NS(true, 4); }
  else if (bf16) { SPEC_NS(true, 1); }
  else if (vec) { SPEC_NS(false, 4); }
  else { SPEC_NS(false, 1); }
#undef SPEC_NS
  return hipGetLastError();
}

hipError_t launch_node_sample(int B, int N, int V, int logits_dtype, const void* logits, float inv_temp,
                              const float* node_max, const float* u_sample, int32_t* node_sample, hipStream_t s) {
  const bool bf16 = logits_dtype == SPEC_BF16, vec = (V % 4 == 0);
#define SPEC_NSM(BF, VE)                                                                                          \
  hipLaunchKernelGGL((node_sample_kernel<BF, VE>), dim3(B * N), dim3(SW_THREADS), 0, s, logits, V, inv_temp, node_max, \
                     u_sample, node_sample)
  if (bf16 && vec) SPEC_NSM(true, 4);
  else if (bf16) SPEC_NSM(true, 1);
  else if (vec) SPEC_NSM(false, 4);
  else SPEC_NSM(false, 1);
#undef SPEC_NSM
  return hipGetLastError();
}

hipError_t launch_greedy_walk(int B, int N, const int32_t* node_argmax, const int32_t* token, const int32_t* parent,
                              int Lmax, int32_t* path, int32_t* len, int32_t* out_tokens, int32_t* status,
                              hipStream_t s) {
  hipLaunchKernelGGL(greedy_walk_kernel, dim3(B), dim3(128), 0, s, N, node_argmax, token, parent, Lmax, path, len,
                     out_tokens, status);
  return hipGetLastError();
}

hipError_t launch_stochastic_walk(int B, int N, int V, int logits_dtype, const void* logits, const float* probs_ssm,
                                  int R, const int32_t* ssm_row, const int32_t* token, const int32_t* parent,
                                  const float* u_accept, const float* u_order, const float* u_final, float inv_temp,
                                  const float* node_max, const float* node_sumexp, float* resid, int Lmax,
                                  int32_t* path, int32_t* len, int32_t* out_tokens, int32_t* status, hipStream_t s) {
  const bool bf16 = logits_dtype == SPEC_BF16, vec = (V % 4 == 0);
#define SPEC_SW(BF, VE)                                                                                              \
  hipLaunchKernelGGL((stochastic_walk_kernel<BF, VE>), dim3(B), dim3(SW_THREADS), 0, s, N, V, logits, probs_ssm, R,    \
                     ssm_row, token, parent, u_accept, u_order, u_final, inv_temp, node_max, node_sumexp, resid, Lmax, \
                     path, len, out_tokens, status)
  if (bf16 && vec) SPEC_SW(true, 4);
  else if (bf16) SPEC_SW(true, 1);
  else if (vec) SPEC_SW(false, 4);
  else SPEC_SW(false, 1);
#undef SPEC_SW
  return hipGetLastError();
}

}  // namespace spec
