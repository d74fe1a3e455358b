// Tree attention for float32 inputs (Definition 4.1 with the topology-aware causal mask of Section
// 4.2), plus the split-combine step shared with the bf16 kernel.
//
// float32 K/V cannot use the bf16 matrix cores without losing the 1e-5 accuracy this dtype is held
// to, so scores and P.V are plain float32 FMAs. This path serves small, accuracy-checking shapes; the
// bandwidth-critical path is the bf16 kernel.
//
// Work split: grid = (n_splits, H, B); a workgroup owns one chunk of the key range of one
// (request, head) and all N tree queries, keeps an online softmax (running max m, sum l, un-normalised
// output O) and either writes the final output (one split) or a partial (m, l, O) that
// attn_combine_kernel merges.
#include <hip/hip_bf16.h>

#include "spec_internal.h"

namespace spec {

constexpr int F32_TK = 32;       // keys per inner tile
constexpr float kLog2e = 1.4426950408889634f;

template <int D>
__global__ void __launch_bounds__(256) tree_attention_f32_kernel(
    const float* __restrict__ q, const float* __restrict__ k_cache, const float* __restrict__ v_cache,
    const int32_t* __restrict__ parent, const int32_t* __restrict__ depth, const int32_t* __restrict__ prefix_len,
    float* __restrict__ out, float* __restrict__ ws_o, float* __restrict__ ws_ml, int32_t* status, int N, int H,
    int S_cap, int group, int chunk_keys, int n_splits, long q_sb, long q_sn, long q_sh, long kv_sb, long kv_sh,
    long kv_ss, float scale_log2, Pages pg) {
  extern __shared__ float smem[];
  __shared__ unsigned long long s_anc[SPEC_MAX_TREE_NODES][2];
  __shared__ int s_flag;
  float* q_s = smem;                          // [N][D]
  float* s_s = q_s + N * D;                   // [N][F32_TK + 1]
  float* m_s = s_s + N * (F32_TK + 1);        // [N] running max
  float* l_s = m_s + N;                       // [N] running sum
  float* a_s = l_s + N;                       // [N] rescale factor of this tile

  const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z, t = threadIdx.x;
  const int P = prefix_len[b];
  const bool cap_ok = (P >= 0) && (P <= S_cap - N);
  const bool valid = tree_is_valid(parent + (long)b * N, depth + (long)b * N, N, &s_flag) && cap_ok;
  if (!valid) {
    if (n_splits == 1) {   // this workgroup owns the final output: defined result = 0
      for (int i = t; i < N * D; i += 256) out[b * q_sb + (i / D) * q_sn + h * q_sh + (i % D)] = 0.f;
      if (h == 0 && t == 0) set_status(status, b, cap_ok ? SPEC_ST_BAD_TREE : SPEC_ST_CAPACITY);
    }
    return;
  }
  const int len = P + N;
  const int c0 = split * chunk_keys;
  const int c1 = min(c0 + chunk_keys, len);
  if (c0 >= len) return;   // the combine step never reads this split

  // ancestor-or-self bitmask of every node: walk up the parent chain (bounded by N steps)
  if (t < N) {
    unsigned long long lo = 0, hi = 0;
    int u = t;
    for (int step = 0; step < N && u >= 0; ++step) {
      if (u < 64) lo |= 1ull << u; else hi |= 1ull << (u - 64);
      u = parent[(long)b * N + u];
    }
    s_anc[t][0] = lo;
    s_anc[t][1] = hi;
    m_s[t] = -INFINITY;
    l_s[t] = 0.f;
  }
  for (int i = t; i < N * D; i += 256) q_s[i] = q[b * q_sb + (i / D) * q_sn + h * q_sh + (i % D)];
  __syncthreads();

  constexpr int CG = D / 4;          // float4 column groups
  constexpr int RG = 256 / CG;       // row groups
  constexpr int RMAX = (SPEC_MAX_TREE_NODES + RG - 1) / RG;
  const int cg = t % CG, rg = t / CG;
  float4 acc[RMAX];
#pragma unroll
  for (int r = 0; r < RMAX; ++r) acc[r] = make_float4(0.f, 0.f, 0.f, 0.f);

  const long head_off = (h / group) * kv_sh;   // grouped-query heads: `group` query heads per K/V head

  for (int k0 = c0; k0 < c1; k0 += F32_TK) {
    const int tk = min(F32_TK, c1 - k0);
    // a tile starts at a multiple of 32 rows, so it lies inside one block of a paged cache
    bool blk_ok;
    const long tile_off = head_off + cache_row_offset(pg, b, k0, kv_sb, kv_ss, &blk_ok);
    if (!blk_ok && t == 0) set_status(status, b, SPEC_ST_BAD_BLOCK);
    const float* kb = k_cache + tile_off;
    const float* vb = v_cache + tile_off;
    // scores of (query n, key k0+kk)
    for (int idx = t; idx < N * F32_TK; idx += 256) {
      const int n = idx / F32_TK, kk = idx % F32_TK;
      float s = -INFINITY;
      if (kk < tk) {
        const int key = k0 + kk;
        const int rel = key - P;
        bool vis = rel < 0;
        if (!vis) vis = (s_anc[n][rel >> 6] >> (rel & 63)) & 1ull;
        if (vis) {
          const float4* kr = (const float4*)(kb + (long)kk * kv_ss);
          const float4* qr = (const float4*)(q_s + n * D);
          float d0 = 0.f, d1 = 0.f, d2 = 0.f, d3 = 0.f;
#pragma unroll 8
          for (int j = 0; j < D / 4; ++j) {
            const float4 kv = kr[j], qv = qr[j];
            d0 = fmaf(qv.x, kv.x, d0);
            d1 = fmaf(qv.y, kv.y, d1);
            d2 = fmaf(qv.z, kv.z, d2);
            d3 = fmaf(qv.w, kv.w, d3);
          }
          s = ((d0 + d1) + (d2 + d3)) * scale_log2;
        }
      }
      s_s[n * (F32_TK + 1) + kk] = s;
    }
    __syncthreads();
    if (t < N) {
      float mx = m_s[t];
      for (int kk = 0; kk < tk; ++kk) mx = fmaxf(mx, s_s[t * (F32_TK + 1) + kk]);
      const float m_use = (mx == -INFINITY) ? 0.f : mx;
      const float alpha = exp2f(m_s[t] - m_use);     // m_s = -inf -> 0
      float sum = 0.f;
      for (int kk = 0; kk < tk; ++kk) {
        const float p = exp2f(s_s[t * (F32_TK + 1) + kk] - m_use);
        s_s[t * (F32_TK + 1) + kk] = p;
        sum += p;
      }
      l_s[t] = l_s[t] * alpha + sum;
      m_s[t] = mx;
      a_s[t] = alpha;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < RMAX; ++r) {
      const int n = rg + r * RG;
      if (n < N) {
        const float alpha = a_s[n];
        float4 a = acc[r];
        a.x *= alpha; a.y *= alpha; a.z *= alpha; a.w *= alpha;
        for (int kk = 0; kk < tk; ++kk) {
          const float p = s_s[n * (F32_TK + 1) + kk];
          const float4 vv = *(const float4*)(vb + (long)kk * kv_ss + cg * 4);
          a.x = fmaf(p, vv.x, a.x); a.y = fmaf(p, vv.y, a.y); a.z = fmaf(p, vv.z, a.z); a.w = fmaf(p, vv.w, a.w);
        }
        acc[r] = a;
      }
    }
    __syncthreads();
  }

  if (n_splits == 1) {
#pragma unroll
    for (int r = 0; r < RMAX; ++r) {
      const int n = rg + r * RG;
      if (n < N) {
        const float inv = 1.f / l_s[n];
        float4 a = acc[r];
        a.x *= inv; a.y *= inv; a.z *= inv; a.w *= inv;
        *(float4*)(out + b * q_sb + n * q_sn + h * q_sh + cg * 4) = a;
      }
    }
  } else {
    const long base = (((long)b * H + h) * n_splits + split) * N;
#pragma unroll
    for (int r = 0; r < RMAX; ++r) {
      const int n = rg + r * RG;
      if (n < N) *(float4*)(ws_o + (base + n) * D + cg * 4) = acc[r];
    }
    if (t < N) {
      ws_ml[(base + t) * 2 + 0] = m_s[t];
      ws_ml[(base + t) * 2 + 1] = l_s[t];
    }
  }
}

// Merge of the partials of one (request, head): out = sum_s O_s 2^(m_s - M) / sum_s l_s 2^(m_s - M),
// M = max_s m_s. grid = (H, B, ceil(N * D/4 / 256)), 256 threads; a thread owns 4 consecutive d of one
// query. The partials of a pair are `slots` consecutive blocks of N rows; how many are filled follows
// from the plan: fixed chunks (chunk_keys > 0) or the balanced deal (bal_wgs > 0). Also the place where
// a malformed request gets its defined result (zeros) and its status bit.
template <bool BF16>
__global__ void __launch_bounds__(256) attn_combine_kernel(const float* __restrict__ ws_o, const float* __restrict__ ws_ml,
                                                           const int32_t* __restrict__ parent,
                                                           const int32_t* __restrict__ depth,
                                                           const int32_t* __restrict__ prefix_len, void* __restrict__ out,
                                                           int32_t* status, int B, int N, int H, int H_kv, int n_qg,
                                                           int hpw, int D, int S_cap, int chunk_keys, int slots,
                                                           int bal_wgs, int bal_tile, long q_sb, long q_sn, long q_sh) {
  constexpr int CH = 4;   // partial slots fetched together
  __shared__ int s_flag;
  const int h = blockIdx.x, b = blockIdx.y, t = threadIdx.x;
  const int CG = D / 4;
  const int idx = blockIdx.z * 256 + t;
  const bool active = idx < N * CG;
  const int n = active ? idx / CG : 0, cg = active ? idx % CG : 0;
  const long base = (((long)b * H + h) * slots) * N + n;
  // The first slots are fetched before anything is known about the request (every slot exists in the
  // workspace, whatever it holds), so that the reads overlap the tree check and the slot count below.
  float m_s[CH], l_s[CH];
  float4 o_s[CH];
  auto fetch = [&](int s0) {
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      const long row = base + (long)min(s0 + j, slots - 1) * N;
      m_s[j] = ws_ml[row * 2];
      l_s[j] = ws_ml[row * 2 + 1];
      o_s[j] = *(const float4*)(ws_o + row * D + cg * 4);
    }
  };
  fetch(0);
  const int P = prefix_len[b];
  const bool cap_ok = (P >= 0) && (P <= S_cap - N);
  const bool valid = tree_is_valid(parent + (long)b * N, depth + (long)b * N, N, &s_flag) && cap_ok;
  if (!valid && h == 0 && blockIdx.z == 0 && t == 0) set_status(status, b, cap_ok ? SPEC_ST_BAD_TREE : SPEC_ST_CAPACITY);
  int ns = 0;
  if (valid) {
    if (bal_wgs > 0) {
      // the deal is over (request, virtual head) pairs: virtual head = K/V head and query group (hpw query
      // heads); the query heads of one virtual head have the same partial slots
      const int H_v = H_kv * n_qg, group = H / H_kv;
      const int hv = (h / group) * n_qg + (h % group) / hpw;
      const BalancedShare bs = balanced_share(prefix_len, B, N, H_v, S_cap, bal_tile, bal_wgs);
      long req_start = 0;
      for (int bb = 0; bb < b; ++bb) req_start += (long)H_v * request_tiles(prefix_len[bb], N, S_cap, bal_tile);
      const int tb = request_tiles(P, N, S_cap, bal_tile);
      const long pair_start = req_start + (long)hv * tb;
      ns = (int)((pair_start + tb - 1) / bs.share - pair_start / bs.share) + 1;
    } else {
      ns = min(slots, (P + N + chunk_keys - 1) / chunk_keys);
    }
  }
  if (!active) return;
  // online merge over chunks of CH slots (slots at and beyond ns hold nothing meaningful: skipped)
  float M = -INFINITY, l = 0.f;
  float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int s0 = 0; s0 < ns || s0 == 0; s0 += CH) {
    if (s0 > 0) fetch(s0);
    float Mc = M;
#pragma unroll
    for (int j = 0; j < CH; ++j)
      if (s0 + j < ns) Mc = fmaxf(Mc, m_s[j]);
    const float keep = (M == -INFINITY) ? 0.f : exp2f(M - Mc);   // Mc = -inf only while nothing carried mass
    l *= keep;
    o.x *= keep; o.y *= keep; o.z *= keep; o.w *= keep;
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      if (s0 + j < ns && m_s[j] != -INFINITY) {   // an all-masked partial carries nothing
        const float w = exp2f(m_s[j] - Mc);
        l = fmaf(l_s[j], w, l);
        o.x = fmaf(o_s[j].x, w, o.x); o.y = fmaf(o_s[j].y, w, o.y); o.z = fmaf(o_s[j].z, w, o.z); o.w = fmaf(o_s[j].w, w, o.w);
      }
    }
    M = Mc;
  }
  const float inv = (l > 0.f) ? 1.f / l : 0.f;
  o.x *= inv; o.y *= inv; o.z *= inv; o.w *= inv;
  const long off = b * q_sb + n * q_sn + h * q_sh + cg * 4;
  if (BF16) {
    __hip_bfloat16* ob = (__hip_bfloat16*)out + off;
    union { uint2 u; __hip_bfloat16 h4[4]; } pk;
    pk.h4[0] = __float2bfloat16(o.x); pk.h4[1] = __float2bfloat16(o.y);
    pk.h4[2] = __float2bfloat16(o.z); pk.h4[3] = __float2bfloat16(o.w);
    *(uint2*)ob = pk.u;
  } else {
    *(float4*)((float*)out + off) = o;
  }
}

hipError_t launch_tree_attention_f32(const spec_attn_desc_t& d, const AttnPlan& plan, const Pages& pg, const float* q,
                                     const float* k_cache, const float* v_cache, const int32_t* parent,
                                     const int32_t* depth, const int32_t* prefix_len, float* out, void* ws,
                                     int32_t* status, hipStream_t s) {
  const float scale = (d.softmax_scale != 0.f ? d.softmax_scale : 1.0f / sqrtf((float)d.D)) * kLog2e;
  float* ws_o = ws ? (float*)((char*)ws + plan.ws_o_off) : nullptr;
  float* ws_ml = ws ? (float*)((char*)ws + plan.ws_ml_off) : nullptr;
  const size_t smem = sizeof(float) * ((size_t)d.N * d.D + (size_t)d.N * (F32_TK + 1) + 3 * (size_t)d.N);
  dim3 grid(plan.n_splits, d.H, d.B);
  auto kern = d.D == 64 ? tree_attention_f32_kernel<64> : tree_attention_f32_kernel<128>;
  hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, grid, dim3(256), smem, s, q, k_cache, v_cache, parent, depth, prefix_len, out, ws_o, ws_ml,
                     status, d.N, d.H, d.S_cap, d.H / d.H_kv, plan.chunk_keys, plan.n_splits, (long)d.q_stride_b, (long)d.q_stride_n,
                     (long)d.q_stride_h, (long)d.kv_stride_b, (long)d.kv_stride_h, (long)d.kv_stride_s, scale, pg);
  return hipGetLastError();
}

hipError_t launch_attn_combine(const spec_attn_desc_t& d, const AttnPlan& plan, const int32_t* parent,
                               const int32_t* depth, const int32_t* prefix_len, const void* ws, void* out,
                               int32_t* status, hipStream_t s) {
  const float* ws_o = (const float*)((const char*)ws + plan.ws_o_off);
  const float* ws_ml = (const float*)((const char*)ws + plan.ws_ml_off);
  const int items = d.N * (d.D / 4);
  const QueryGroups qg = attn_query_groups(d);
  const int n_qg = d.dtype == SPEC_BF16 ? qg.n_qgroups : 1, hpw = d.dtype == SPEC_BF16 ? qg.heads_per_wg : 1;
  dim3 grid(d.H, d.B, (items + 255) / 256);
  if (d.dtype == SPEC_BF16) {
    hipLaunchKernelGGL(attn_combine_kernel<true>, grid, dim3(256), 0, s, ws_o, ws_ml, parent, depth, prefix_len, out,
                       status, d.B, d.N, d.H, d.H_kv, n_qg, hpw, d.D, d.S_cap, plan.chunk_keys, plan.n_splits, plan.balanced_wgs, plan.balanced_tile,
                       (long)d.q_stride_b, (long)d.q_stride_n, (long)d.q_stride_h);
  } else {
    hipLaunchKernelGGL(attn_combine_kernel<false>, grid, dim3(256), 0, s, ws_o, ws_ml, parent, depth, prefix_len, out,
                       status, d.B, d.N, d.H, d.H_kv, n_qg, hpw, d.D, d.S_cap, plan.chunk_keys, plan.n_splits, plan.balanced_wgs, plan.balanced_tile,
                       (long)d.q_stride_b, (long)d.q_stride_n, (long)d.q_stride_h);
  }
  return hipGetLastError();
}

}  // namespace spec
