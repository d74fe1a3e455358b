// LM head in front of the greedy verifier (Algorithm 2, VerifyGreedy: O(u) is the arg-max of the LLM's
// distribution at node u, so for greedy decoding the logits [B*N, V] never have to exist in memory):
//     node_argmax[m] = argmax_v  sum_k hidden[m, k] * weight[v, k]        (lowest v on ties)
// bf16 inputs, float32 accumulation on the matrix cores. With the few hundred rows a verification pass has
// (M = B*N), the product is bound by streaming the weight matrix once from HBM (V x K x 2 bytes, 262 MB for
// a 32000 x 4096 head), not by arithmetic.
//
// lm_head_argmax_kernel: a workgroup of eight (four when M <= 32) wavefronts owns 16 vocabulary rows per
// wavefront and up to 128 rows of `hidden` (NMT tiles of 16). Every wavefront streams ITS 16 rows of W straight from global
// memory into the MFMA A-operand layout (lane (r, g) holds W[v0 + r][k0 + 8g .. 8g + 8)), PF chunks of 64 k
// in flight, independent of the other wavefronts; `hidden` (L2-resident, shared by all wavefronts) is staged
// through LDS in slices of 256 k, double-buffered, one barrier per slice. The product is taken transposed,
// C[v, m], so a lane ends up with four vocabulary entries of ONE row m and the arg-max over v is four
// compares, two cross-lane steps and one pass through LDS over the eight wavefronts. Each workgroup writes its
// (max, arg-max) per row; lm_head_reduce_kernel merges a row's partials (one per workgroup).
#include <hip/hip_bf16.h>

#include <type_traits>

#include "spec_internal.h"

namespace spec {
namespace lmh {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

constexpr int KC = 64;                        // k per chunk of W (two MFMA k-steps)
constexpr int HC = 256;                       // k per LDS slice of hidden (four chunks)
constexpr int CPS = HC / KC;                  // chunks per slice
constexpr int PF = 8;                         // chunks of W in flight per wavefront
constexpr int HROW = HC * 2 + 16;             // LDS bytes per hidden row (+16: 16 rows fall into 16 distinct bank groups)

// f(integral_constant<int, I>) for I = 0 .. N - 1, unrolled at compile time.
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// (value desc, index asc): does (v2, i2) beat (v1, i1)?
__device__ __forceinline__ bool beats(float v2, int i2, float v1, int i1) { return v2 > v1 || (v2 == v1 && i2 < i1); }

// WAVES wavefronts of 16 vocabulary rows each: eight (128 rows, one workgroup per CU) or four (64 rows, two
// workgroups per CU, so that one's start and end overlap the other's stream).
// STATS: the logits are also written out, rounded to bf16, and every partial carries the sum of
// exp((x - max) / T) over the workgroup's vocabulary rows - of the ROUNDED values, which are what a verifier
// reading those logits will see (maximum and arg-max are then those of the rounded values too).
template <int NMT, int WAVES, bool STATS>
__global__ void __launch_bounds__(WAVES * 64) lm_head_argmax_kernel(const __hip_bfloat16* __restrict__ hidden,
                                                                  const __hip_bfloat16* __restrict__ weight,
                                                                  float* __restrict__ part_val, int32_t* __restrict__ part_idx,
                                                                  float* __restrict__ part_sum,
                                                                  __hip_bfloat16* __restrict__ logits_out, float inv_temp_log2,
                                                                  int M, int K, int V, int n_vtiles) {
  constexpr int NTHREADS = WAVES * 64, VT = WAVES * 16;
  constexpr int MROWS = NMT * 16;
  constexpr int STAGE = MROWS * HROW;
  constexpr int PIECES = MROWS * (HC * 2 / 16);                       // 16-byte pieces of one slice
  constexpr int NPT = (PIECES + NTHREADS - 1) / NTHREADS;             // per thread
  __shared__ __attribute__((aligned(16))) unsigned char lds[2 * STAGE];
  __shared__ float s_val[WAVES][MROWS];
  __shared__ int s_idx[WAVES][MROWS];
  __shared__ float s_sum[STATS ? WAVES : 1][MROWS];

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int r16 = lane & 15, g = lane >> 4;
  const int v0 = blockIdx.x * VT + wave * 16, m0 = blockIdx.y * MROWS;
  const int NC = K / KC, NS = K / HC;

  // this lane's row of W, in the MFMA A-operand layout (rows past V repeat the last one; their results are
  // masked at the end). Requesting whole 128-byte lines per row instead (eight lanes per row) and transposing
  // through LDS was measured: the loads alone are 5 % faster, the transposition costs as much.
  // The loads stay plain: a load covers 64 bytes of each of 16 rows, the other half of every 128-byte line comes
  // with the next load, and with the non-temporal hint the line is not kept for it (measured: 59 us against 52).
  const unsigned char* wrow = (const unsigned char*)(weight + (long)min(v0 + r16, V - 1) * K) + g * 16;
  u32x4 Wr[PF][2];
  auto issue_w = [&](u32x4 (&dst)[2], int c) {
    dst[0] = *(const u32x4*)(wrow + (long)c * (KC * 2));
    dst[1] = *(const u32x4*)(wrow + (long)c * (KC * 2) + 64);
  };
#pragma unroll
  for (int c = 0; c < PF; ++c)
    if (c < NC) issue_w(Wr[c], c);

  // hidden slice s: rows m0 .. m0 + MROWS (rows past M repeat the last one), k in [s * HC, s * HC + HC)
  // A slice is requested one slice (four chunks) before it is staged. Loads return in order, so waiting for a
  // slice also waits for every older load of W; at a distance of four chunks those are loads that had to be
  // back by then anyway, and the chunks of W requested since stay in flight (with slices of two chunks the
  // compiler's wait counts showed the stream being cut to 2-3 chunks per wavefront at every slice boundary).
  u32x4 Hreg[NPT];
  auto issue_h = [&](u32x4 (&Hr)[NPT], int s) {
#pragma unroll
    for (int j = 0; j < NPT; ++j) {
      const int p = t + j * NTHREADS;
      if (NPT * NTHREADS == PIECES || p < PIECES) {
        const int row = p / (HC * 2 / 16), col = p % (HC * 2 / 16);
        Hr[j] = *(const u32x4*)((const unsigned char*)(hidden + (long)min(m0 + row, M - 1) * K + s * HC) + col * 16);
      }
    }
  };
  auto stage_h = [&](u32x4 (&Hr)[NPT], unsigned char* stage) {
#pragma unroll
    for (int j = 0; j < NPT; ++j) {
      const int p = t + j * NTHREADS;
      if (NPT * NTHREADS == PIECES || p < PIECES) {
        const int row = p / (HC * 2 / 16), col = p % (HC * 2 / 16);
        *(u32x4*)(stage + row * HROW + col * 16) = Hr[j];
      }
    }
  };
  issue_h(Hreg, 0);
  stage_h(Hreg, lds);
  if (NS > 1) issue_h(Hreg, 1);
  __syncthreads();

  f32x4 acc[NMT];
#pragma unroll
  for (int mt = 0; mt < NMT; ++mt) acc[mt] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // chunk c of W (register set c % PF) against quarter (c % 4) of hidden slice c / 4
  auto chunk = [&](u32x4 (&w)[2], int c) {
    const unsigned char* hs = lds + ((c / CPS) & 1) * STAGE + r16 * HROW + (c % CPS) * (KC * 2) + g * 16;
    // The B operands are requested from LDS ahead of the products that use them (each product then waits for its
    // own operand only; left to itself the compiler pairs every product with its read): all of the chunk's, or,
    // with eight tiles of hidden, one k-step's at a time (the register file does not hold both).
    constexpr int KSB = NMT == 8 ? 1 : 2;   // k-steps per batch of reads
#pragma unroll
    for (int k0 = 0; k0 < 2; k0 += KSB) {
      bf16x8 b[KSB][NMT];
#pragma unroll
      for (int ks = 0; ks < KSB; ++ks)
#pragma unroll
        for (int mt = 0; mt < NMT; ++mt) b[ks][mt] = *(const bf16x8*)(hs + mt * 16 * HROW + (k0 + ks) * 64);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int ks = 0; ks < KSB; ++ks) {
        const bf16x8 a = __builtin_bit_cast(bf16x8, w[k0 + ks]);
#pragma unroll
        for (int mt = 0; mt < NMT; ++mt) acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b[ks][mt], acc[mt], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // End of slice s: the slice after it goes from registers to the other LDS stage (last read during slice
  // s - 1, before the previous barrier), and the slice two ahead is requested into the registers this frees.
  // FULL: both exist (no branch). `odd`: parity of s + 1 (a compile-time constant at every call: blocks
  // start at multiples of PF chunks, i.e. at even slices).
  auto next_slice = [&](int s, auto odd_tag, auto full_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
    constexpr int ODD = decltype(odd_tag)::value;
    if (FULL || s + 1 < NS) stage_h(Hreg, lds + ODD * STAGE);
    if (FULL || s + 2 < NS) issue_h(Hreg, s + 2);
    __syncthreads();
  };
  // PF chunks starting at c0. FULL: PF more chunks follow, so every register set is refilled and the block is
  // straight-line code (the waits for the loads in flight are then exact counts, not worst cases).
  auto block = [&](int c0, auto full_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
    static_for<0, PF>([&](auto d_tag) {
      constexpr int d = decltype(d_tag)::value;
      const int c = c0 + d;
      if (FULL || c < NC) {
        chunk(Wr[d], c);
        if (FULL || c + PF < NC) issue_w(Wr[d], c + PF);
        if constexpr (d % CPS == CPS - 1) next_slice(c / CPS, std::integral_constant<int, ((d / CPS) + 1) & 1>{}, full_tag);
      }
    });
  };
  int c0 = 0;
  for (; c0 + 2 * PF <= NC; c0 += PF) block(c0, std::true_type{});   // FULL: slices up to c0 / 4 + 3 exist
  for (; c0 < NC; c0 += PF) block(c0, std::false_type{});

  // ---- arg-max over this wavefront's 16 vocabulary rows, per row m: in the lane, then across the four lane groups
#pragma unroll
  for (int mt = 0; mt < NMT; ++mt) {
    float x[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) x[i] = acc[mt][i];
    if (STATS) {   // round to the stored type first: statistics and arg-max are those of the stored logits
      union { uint2 u; __hip_bfloat16 h4[4]; } pk;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        pk.h4[i] = __float2bfloat16(x[i]);
        x[i] = __bfloat162float(pk.h4[i]);
      }
      const int m = m0 + mt * 16 + r16, v = v0 + 4 * g;
      if (m < M) {
        __hip_bfloat16* dst = logits_out + (long)m * V + v;
        if (v + 3 < V && (((long)m * V + v) & 3) == 0) {
          *(uint2*)dst = pk.u;
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (v + i < V) dst[i] = pk.h4[i];
        }
      }
    }
    float best = -INFINITY;
    int best_i = 0x7fffffff;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int v = v0 + 4 * g + i;
      if (v < V && x[i] > best) { best = x[i]; best_i = v; }   // ascending v: the lowest wins ties
    }
    const float lane_best = best;
#pragma unroll
    for (int o = 16; o <= 32; o <<= 1) {
      const float ov = __shfl_xor(best, o);
      const int oi = __shfl_xor(best_i, o);
      if (beats(ov, oi, best, best_i)) { best = ov; best_i = oi; }
    }
    float sum = 0.f;
    if (STATS) {   // sum of exp((x - best) / T) over the wavefront's 16 vocabulary rows (best: the wavefront's maximum)
      if (best > -INFINITY) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (v0 + 4 * g + i < V) sum += __builtin_amdgcn_exp2f((x[i] - best) * inv_temp_log2);
      }
      sum += __shfl_xor(sum, 16);
      sum += __shfl_xor(sum, 32);
      (void)lane_best;
    }
    if (g == 0) {
      s_val[wave][mt * 16 + r16] = best;
      s_idx[wave][mt * 16 + r16] = best_i;
      if (STATS) s_sum[wave][mt * 16 + r16] = sum;
    }
  }
  __syncthreads();
  if (t < MROWS && m0 + t < M) {
    float best = s_val[0][t];
    int best_i = s_idx[0][t];
#pragma unroll
    for (int w = 1; w < WAVES; ++w)
      if (beats(s_val[w][t], s_idx[w][t], best, best_i)) { best = s_val[w][t]; best_i = s_idx[w][t]; }
    part_val[(long)(m0 + t) * n_vtiles + blockIdx.x] = best;
    part_idx[(long)(m0 + t) * n_vtiles + blockIdx.x] = best_i;
    if (STATS) {
      float sum = 0.f;
#pragma unroll
      for (int w = 0; w < WAVES; ++w)
        if (s_val[w][t] > -INFINITY) sum += s_sum[w][t] * __builtin_amdgcn_exp2f((s_val[w][t] - best) * inv_temp_log2);
      part_sum[(long)(m0 + t) * n_vtiles + blockIdx.x] = sum;
    }
  }
}

// One workgroup per row: merges the row's n_vtiles partials (part_sum != nullptr: also the sums, rescaled to
// the row's maximum).
__global__ void __launch_bounds__(256) lm_head_reduce_kernel(const float* __restrict__ part_val,
                                                             const int32_t* __restrict__ part_idx,
                                                             const float* __restrict__ part_sum, float inv_temp_log2,
                                                             int n_vtiles, int32_t* __restrict__ node_argmax,
                                                             float* __restrict__ node_max, float* __restrict__ node_sumexp) {
  __shared__ float s_val[4];
  __shared__ int s_idx[4];
  __shared__ float s_sum[4];
  const int m = blockIdx.x, t = threadIdx.x;
  float best = -INFINITY;
  int best_i = 0x7fffffff;
  for (int j = t; j < n_vtiles; j += 256) {
    const float v = part_val[(long)m * n_vtiles + j];
    const int i = part_idx[(long)m * n_vtiles + j];
    if (beats(v, i, best, best_i)) { best = v; best_i = i; }
  }
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(best, o);
    const int oi = __shfl_xor(best_i, o);
    if (beats(ov, oi, best, best_i)) { best = ov; best_i = oi; }
  }
  if ((t & 63) == 0) { s_val[t >> 6] = best; s_idx[t >> 6] = best_i; }
  __syncthreads();
  best = s_val[0]; best_i = s_idx[0];
  for (int w = 1; w < 4; ++w)
    if (beats(s_val[w], s_idx[w], best, best_i)) { best = s_val[w]; best_i = s_idx[w]; }
  if (part_sum != nullptr) {
    float sum = 0.f;
    for (int j = t; j < n_vtiles; j += 256) {
      const float v = part_val[(long)m * n_vtiles + j];
      if (v > -INFINITY) sum += part_sum[(long)m * n_vtiles + j] * __builtin_amdgcn_exp2f((v - best) * inv_temp_log2);
    }
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
    if ((t & 63) == 0) s_sum[t >> 6] = sum;
    __syncthreads();
    if (t == 0 && node_sumexp != nullptr) node_sumexp[m] = (s_sum[0] + s_sum[1]) + (s_sum[2] + s_sum[3]);
  }
  if (t == 0) {
    if (node_argmax != nullptr) node_argmax[m] = best_i == 0x7fffffff ? 0 : best_i;   // a row of NaN / -inf logits
    if (node_max != nullptr) node_max[m] = best;
  }
}

}  // namespace lmh

// logits_out != nullptr: the kernel also writes the bf16 logits [M, V] and the softmax statistics of the rounded
// values (node_sumexp; inv_temp = 1 / temperature); the workspace then holds a third partial array.
hipError_t launch_lm_head(int M, int K, int V, const void* hidden, const void* weight, void* logits_out, float inv_temp,
                          int32_t* node_argmax, float* node_max, float* node_sumexp, void* ws, hipStream_t s) {
  const bool stats = logits_out != nullptr;
  const size_t arr = lm_head_partials_bytes(M, V) / 2;
  float* part_val = (float*)ws;
  int32_t* part_idx = (int32_t*)((char*)ws + arr);
  float* part_sum = stats ? (float*)((char*)ws + 2 * arr) : nullptr;
  const float itl2 = inv_temp * 1.4426950408889634f;
  const int nmt = M <= 16 ? 1 : M <= 32 ? 2 : M <= 64 ? 4 : 8;
  const int waves = lm_head_waves(M);
  const int n_vtiles = (V + waves * 16 - 1) / (waves * 16);
  const dim3 grid(n_vtiles, (M + nmt * 16 - 1) / (nmt * 16));
#define SPEC_LMH(NMT, WV, ST)                                                                                              \
  hipLaunchKernelGGL((lmh::lm_head_argmax_kernel<NMT, WV, ST>), grid, dim3(WV * 64), 0, s, (const __hip_bfloat16*)hidden, \
                     (const __hip_bfloat16*)weight, part_val, part_idx, part_sum, (__hip_bfloat16*)logits_out, itl2, M, K, \
                     V, n_vtiles)
#define SPEC_LMH_T(WV, ST)                  \
  if (nmt == 1) SPEC_LMH(1, WV, ST);        \
  else if (nmt == 2) SPEC_LMH(2, WV, ST);   \
  else if (nmt == 4) SPEC_LMH(4, WV, ST);   \
  else SPEC_LMH(8, WV, ST)
  if (waves == 4) {
    if (stats) { SPEC_LMH_T(4, true); } else { SPEC_LMH_T(4, false); }
  } else {
    if (stats) { SPEC_LMH_T(8, true); } else { SPEC_LMH_T(8, false); }
  }
#undef SPEC_LMH_T
#undef SPEC_LMH
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(lmh::lm_head_reduce_kernel, dim3(M), dim3(256), 0, s, part_val, part_idx, part_sum, itl2, n_vtiles,
                     node_argmax, node_max, node_sumexp);
  return hipGetLastError();
}

hipError_t launch_lm_head_argmax(int M, int K, int V, const void* hidden, const void* weight, int32_t* node_argmax,
                                 float* node_max, void* ws, hipStream_t s) {
  return launch_lm_head(M, K, V, hidden, weight, nullptr, 1.f, node_argmax, node_max, nullptr, ws, s);
}

}  // namespace spec
