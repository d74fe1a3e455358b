// Tree attention for bf16 K/V on the gfx950 matrix cores (Definition 4.1; topology-aware causal mask
// of Section 4.2), written for the decode-shaped case: few tree queries (N <= 128) against a long
// cached prefix, so the kernel is bound by streaming K and V from HBM exactly once.
//
// Decomposition
//   grid = (n_splits, H * n_qgroups, B). A workgroup (4 wavefronts) owns one chunk of the key range
//   of one (request, head) and a group of NT*16 tree queries. The four wavefronts take the chunk's
//   32-key tiles round-robin and are completely independent inside the main loop (no barrier): each
//   keeps its own online-softmax state and merges with the others once, through LDS, at the end.
//
// Per 32-key tile and wavefront
//   S^T = K Q^T   v_mfma_f32_16x16x32_bf16, A = K rows read straight from global memory into the
//                 MFMA operand layout (lane r of a 16-lane group holds 8 consecutive d of key r),
//                 B = Q^T resident in registers. The transposed product leaves lane l with scores of
//                 query l%16 for keys 4*(l/16)+v of each 16-key half: exactly the B-operand layout
//                 P^T needs for the second product, so probabilities never leave registers.
//   mask          only for tiles that reach past the prefix: bit (key - prefix_len) of the query's
//                 128-bit ancestor-or-self mask (built once per workgroup from the parent array).
//   softmax       online, in the exp2 domain; row max over the tile = 8 in-lane values + 2 cross-lane
//                 exchanges; the rescale factor of a query is lane-local for its O^T fragment.
//   O^T += V^T P^T  A = V^T needs 8 keys x 1 d per lane, the transpose of how V lies in memory: V is
//                 loaded fully coalesced (four 256-byte rows per instruction), staged in a
//                 wavefront-private LDS tile and read back with ds_read_b64_tr_b16.
//
// Results are written as the final bf16 output when one chunk covers the whole key range, else as
// float32 partials (m, l, O) merged by attn_combine_kernel.
#include <hip/hip_bf16.h>

#include "spec_internal.h"

namespace spec {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;

constexpr float kLog2eB = 1.4426950408889634f;
constexpr int TILE = 32;          // keys per wavefront tile
constexpr int WAVES = 4;

template <int D>
struct VTile {
  static constexpr int ROW_BYTES = D * 2 + 16;        // +16 B pad: 4 consecutive rows fall in distinct banks
  static constexpr int BYTES = TILE * ROW_BYTES;
};

__device__ inline float wave_max_over_lane_groups(float v) {
  // lanes l, l^16, l^32, l^48 hold the same query: reduce over the four 16-lane groups
  v = fmaxf(v, __shfl_xor(v, 16));
  v = fmaxf(v, __shfl_xor(v, 32));
  return v;
}
__device__ inline float wave_sum_over_lane_groups(float v) {
  v += __shfl_xor(v, 16);
  v += __shfl_xor(v, 32);
  return v;
}

template <int D, int NT>
__global__ void __launch_bounds__(256, 2) tree_attention_bf16_kernel(
    const __hip_bfloat16* __restrict__ q, const __hip_bfloat16* __restrict__ k_cache,
    const __hip_bfloat16* __restrict__ v_cache, const int32_t* __restrict__ parent, const int32_t* __restrict__ depth,
    const int32_t* __restrict__ prefix_len, __hip_bfloat16* __restrict__ out, float* __restrict__ ws_o,
    float* __restrict__ ws_ml, int32_t* status, int N, int H, int S_cap, int n_qgroups, int chunk_keys, int n_splits,
    long q_sb, long q_sn, long q_sh, long kv_sb, long kv_sh, long kv_ss, float scale_log2) {
  constexpr int KS = D / 32;            // k-steps of the QK^T product
  constexpr int DB = D / 16;            // 16-wide d blocks of the output
  constexpr int LPR = D * 2 / 16;       // lanes (16-byte pieces) per K/V row
  constexpr int RPI = 64 / LPR;         // rows covered by one wave-wide 16-byte load
  constexpr int NVL = TILE / RPI;       // V loads per lane per tile
  constexpr int VROW = VTile<D>::ROW_BYTES;
  constexpr int NQ = NT * 16;           // queries per workgroup
  constexpr int MROW = D + 4;           // floats per merge row: O[D], m, l, 2 pad (keeps rows 16-byte aligned)
  constexpr int MERGE_BYTES = WAVES * NQ * MROW * 4;
  constexpr int STAGE_BYTES = WAVES * VTile<D>::BYTES;
  constexpr int LDS_BYTES = MERGE_BYTES > STAGE_BYTES ? MERGE_BYTES : STAGE_BYTES;

  __shared__ __attribute__((aligned(16))) unsigned char lds[LDS_BYTES];
  __shared__ unsigned long long s_anc[SPEC_MAX_TREE_NODES][2];
  __shared__ int s_parent[SPEC_MAX_TREE_NODES];
  __shared__ int s_depth[SPEC_MAX_TREE_NODES];
  __shared__ int s_flag;

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int r16 = lane & 15, g = lane >> 4;
  const int split = blockIdx.x;
  const int h = blockIdx.y / n_qgroups, qg = blockIdx.y % n_qgroups;
  const int b = blockIdx.z;
  const int q0 = qg * NQ;

  const int P = prefix_len[b];
  const bool cap_ok = (P >= 0) && (P <= S_cap - N);
  const int len = P + N;
  const int c0 = split * chunk_keys;
  if (!cap_ok) {
    if (n_splits == 1) {
      for (int i = t; i < NQ * D; i += 256) {
        const int n = q0 + i / D;
        if (n < N) out[b * q_sb + n * q_sn + h * q_sh + (i % D)] = __float2bfloat16(0.f);
      }
      if (h == 0 && qg == 0 && t == 0) set_status(status, b, SPEC_ST_CAPACITY);
    }
    return;
  }
  if (c0 >= len) return;
  const int c1 = min(c0 + chunk_keys, len);
  const bool touches_tree = c1 > P;

  unsigned long long anc_lo[NT], anc_hi[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) anc_lo[nt] = anc_hi[nt] = 0ull;

  if (touches_tree) {
    // stage the tree, validate it, build ancestor-or-self masks by walking up the parent chain
    if (t == 0) s_flag = 0;
    if (t < N) {
      s_parent[t] = parent[(long)b * N + t];
      s_depth[t] = depth[(long)b * N + t];
    }
    __syncthreads();
    if (t < N) {
      const int p = s_parent[t];
      bool ok = (t == 0) ? (p == -1 && s_depth[0] == 0) : (p >= 0 && p < t);
      if (ok && t > 0) ok = s_depth[t] == s_depth[p] + 1;
      if (!ok) atomicOr(&s_flag, 1);
    }
    __syncthreads();
    if (s_flag != 0) {
      if (n_splits == 1) {
        for (int i = t; i < NQ * D; i += 256) {
          const int n = q0 + i / D;
          if (n < N) out[b * q_sb + n * q_sn + h * q_sh + (i % D)] = __float2bfloat16(0.f);
        }
        if (h == 0 && qg == 0 && t == 0) set_status(status, b, SPEC_ST_BAD_TREE);
      }
      return;
    }
    if (t < N) {
      unsigned long long lo = 0, hi = 0;
      int u = t;
      for (int step = 0; step < N && u >= 0; ++step) {
        if (u < 64) lo |= 1ull << u; else hi |= 1ull << (u - 64);
        u = s_parent[u];
      }
      s_anc[t][0] = lo;
      s_anc[t][1] = hi;
    }
    __syncthreads();
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int n = q0 + nt * 16 + r16;
      if (n < N) { anc_lo[nt] = s_anc[n][0]; anc_hi[nt] = s_anc[n][1]; }
    }
  }

  // ---- Q^T as the B operand: lane (r16, g) holds Q[n = r16][d = ks*32 + g*8 .. +8]
  bf16x8 qB[NT][KS];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int n = q0 + nt * 16 + r16;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint4 raw = make_uint4(0, 0, 0, 0);
      if (n < N) raw = *(const uint4*)(q + b * q_sb + n * q_sn + h * q_sh + ks * 32 + g * 8);
      qB[nt][ks] = __builtin_bit_cast(bf16x8, raw);
    }
  }

  f32x4 O[NT][DB];
  float m_run[NT], l_run[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    m_run[nt] = -INFINITY;
    l_run[nt] = 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db) O[nt][db] = (f32x4){0.f, 0.f, 0.f, 0.f};
  }

  const __hip_bfloat16* kb = k_cache + b * kv_sb + h * kv_sh;
  const __hip_bfloat16* vb = v_cache + b * kv_sb + h * kv_sh;
  unsigned char* vst = lds + wave * VTile<D>::BYTES;
  const int n_tiles = (c1 - c0 + TILE - 1) / TILE;
  const int last_row = len - 1;

  uint4 Kn[2][KS], Vn[NVL];
  auto issue_loads = [&](int ti) {
    const int k0 = c0 + ti * TILE;
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
      const int row = min(k0 + hf * 16 + r16, last_row);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) Kn[hf][ks] = *(const uint4*)(kb + (long)row * kv_ss + ks * 32 + g * 8);
    }
#pragma unroll
    for (int j = 0; j < NVL; ++j) {
      const int row = min(k0 + j * RPI + lane / LPR, last_row);
      Vn[j] = *(const uint4*)(vb + (long)row * kv_ss + (lane % LPR) * 8);
    }
  };

  int ti = wave;
  if (ti < n_tiles) issue_loads(ti);
  for (; ti < n_tiles; ti += WAVES) {
    const int k0 = c0 + ti * TILE;
    // current tile: K operands to their own registers, V to the wavefront's LDS tile
    bf16x8 Kc[2][KS];
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) Kc[hf][ks] = __builtin_bit_cast(bf16x8, Kn[hf][ks]);
#pragma unroll
    for (int j = 0; j < NVL; ++j)
      *(uint4*)(vst + (j * RPI + lane / LPR) * VROW + (lane % LPR) * 16) = Vn[j];
    if (ti + WAVES < n_tiles) issue_loads(ti + WAVES);

    // ---- S^T = K Q^T : sc[nt][hf][v] = score of query nt*16+r16 and key k0 + hf*16 + 4g + v
    f32x4 sc[NT][2];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Kc[hf][ks], qB[nt][ks], acc, 0, 0, 0);
        sc[nt][hf] = acc;
      }

    const bool need_mask = (k0 + TILE > P) || (k0 + TILE > c1);
    bf16x8 pB[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      float s[8];
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int v = 0; v < 4; ++v) s[hf * 4 + v] = sc[nt][hf][v] * scale_log2;
      if (need_mask) {
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int key = k0 + hf * 16 + 4 * g + v;
            const int rel = key - P;
            bool vis = key < c1;
            if (vis && rel >= 0) {
              const unsigned long long w = rel < 64 ? anc_lo[nt] : anc_hi[nt];
              vis = (w >> (rel & 63)) & 1ull;
            }
            if (!vis) s[hf * 4 + v] = -INFINITY;
          }
      }
      float mx = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
      mx = wave_max_over_lane_groups(mx);
      const float m_new = fmaxf(m_run[nt], mx);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m_run[nt] - m_use);
      m_run[nt] = m_new;
      float psum = 0.f;
      bf16x8 pb;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float p = __builtin_amdgcn_exp2f(s[i] - m_use);
        psum += p;
        pb[i] = (__bf16)p;
      }
      pB[nt] = pb;
      l_run[nt] = l_run[nt] * alpha + psum;
#pragma unroll
      for (int db = 0; db < DB; ++db) O[nt][db] *= alpha;
    }

    // ---- O^T += V^T P^T : A operand = V^T through the transposing LDS read
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      const unsigned char* base = vst + (4 * g + (r16 >> 2)) * VROW + db * 32 + (r16 & 3) * 8;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(base));
      const s16x4 hi =
          __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(base + 16 * VROW));
      union { struct { s16x4 a, b; } p; bf16x8 v; } vt;
      vt.p.a = lo;
      vt.p.b = hi;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        O[nt][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt.v, pB[nt], O[nt][db], 0, 0, 0);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }

  // ---- merge the four wavefronts through LDS: layout [wave][n][MROW] floats (O row, m, l)
  __syncthreads();
  float* mg = (float*)lds;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const float l_tot = wave_sum_over_lane_groups(l_run[nt]);
    float* row = mg + ((wave * NQ) + nt * 16 + r16) * MROW;
#pragma unroll
    for (int db = 0; db < DB; ++db) *(f32x4*)(row + db * 16 + 4 * g) = O[nt][db];
    if (g == 0) {
      row[D] = m_run[nt];
      row[D + 1] = l_tot;
    }
  }
  __syncthreads();
  constexpr int CG = D / 4;
  for (int idx = t; idx < NQ * CG; idx += 256) {
    const int nl = idx / CG, cg = idx % CG;
    const int n = q0 + nl;
    if (n >= N) continue;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) M = fmaxf(M, mg[(w * NQ + nl) * MROW + D]);
    const float M_use = (M == -INFINITY) ? 0.f : M;
    f32x4 o = {0.f, 0.f, 0.f, 0.f};
    float l = 0.f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
      const float* row = mg + (w * NQ + nl) * MROW;
      const float wgt = __builtin_amdgcn_exp2f(row[D] - M_use);
      l += row[D + 1] * wgt;
      o += *(const f32x4*)(row + cg * 4) * wgt;
    }
    if (n_splits == 1) {
      const float inv = 1.f / l;
      union { uint2 u; __hip_bfloat16 h4[4]; } pk;
#pragma unroll
      for (int i = 0; i < 4; ++i) pk.h4[i] = __float2bfloat16(o[i] * inv);
      *(uint2*)(out + b * q_sb + n * q_sn + h * q_sh + cg * 4) = pk.u;
    } else {
      const long base = (((long)b * H + h) * n_splits + split) * N + n;
      *(f32x4*)(ws_o + base * D + cg * 4) = o;
      if (cg == 0) {
        ws_ml[base * 2 + 0] = M;
        ws_ml[base * 2 + 1] = l;
      }
    }
  }
}

hipError_t launch_tree_attention_bf16(const spec_attn_desc_t& d, const AttnPlan& plan, const void* q,
                                      const void* k_cache, const void* v_cache, const int32_t* parent,
                                      const int32_t* depth, const int32_t* prefix_len, void* out, void* ws,
                                      int32_t* status, hipStream_t s) {
  const float scale = (d.softmax_scale != 0.f ? d.softmax_scale : 1.0f / sqrtf((float)d.D)) * kLog2eB;
  float* ws_o = ws ? (float*)((char*)ws + plan.ws_o_off) : nullptr;
  float* ws_ml = ws ? (float*)((char*)ws + plan.ws_ml_off) : nullptr;
  const int nt = d.N <= 16 ? 1 : 2;
  const int nq = nt * 16;
  const int n_qgroups = (d.N + nq - 1) / nq;
  dim3 grid(plan.n_splits, d.H * n_qgroups, d.B);
#define SPEC_LAUNCH(DD, NTT)                                                                                          \
  hipLaunchKernelGGL((tree_attention_bf16_kernel<DD, NTT>), grid, dim3(256), 0, s, (const __hip_bfloat16*)q,          \
                     (const __hip_bfloat16*)k_cache, (const __hip_bfloat16*)v_cache, parent, depth, prefix_len,       \
                     (__hip_bfloat16*)out, ws_o, ws_ml, status, d.N, d.H, d.S_cap, n_qgroups, plan.chunk_keys,        \
                     plan.n_splits, (long)d.q_stride_b, (long)d.q_stride_n, (long)d.q_stride_h, (long)d.kv_stride_b,  \
                     (long)d.kv_stride_h, (long)d.kv_stride_s, scale)
  if (d.D == 128 && nt == 1) SPEC_LAUNCH(128, 1);
  else if (d.D == 128) SPEC_LAUNCH(128, 2);
  else if (nt == 1) SPEC_LAUNCH(64, 1);
  else SPEC_LAUNCH(64, 2);
#undef SPEC_LAUNCH
  return hipGetLastError();
}

}  // namespace spec
