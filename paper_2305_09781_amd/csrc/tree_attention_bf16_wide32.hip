// Tree attention for bf16 K/V, head dimension 128, five to eight 16-query tiles per K/V head (trees of 65..128
// nodes, or grouped-query heads that bring as many): Definition 4.1 with the topology-aware causal mask of
// Section 4.2, same mathematics as tree_attention_bf16_wide.hip, on a workgroup shape built for many queries
// per key.
//
//   * Four wavefronts, each owning 32 queries on v_mfma_f32_32x32x16_bf16: S^T = K Q^T leaves lane (n, h) with
//     the scores of query n for 16 of a block's 32 keys, which is the B-operand layout P^T needs for
//     O^T += V^T P^T. Every K and V^T operand read from LDS feeds 32 queries.
//   * K and V go from global memory straight into LDS (global_load_lds_dwordx4), into a ring of four stages of
//     32 keys. Data in flight occupies no registers, so a lane needs well under 256 of them and two workgroups
//     share a compute unit: three stages (48 KB) are in flight per workgroup while a fourth is consumed, and one
//     workgroup's stream overlaps the other's arithmetic.
//   * LDS rows are unpadded (a wave-wide direct load writes 1 KB contiguously: four 256-byte rows). Bank
//     conflicts are avoided by a swizzle applied on the global side: slot s of row r holds the 16-byte piece
//     s ^ f(r), f(r) = ((r & 7) << 1) | ((r >> 3) & 1), which keeps both operand reads conflict-free (sixteen
//     consecutive rows of one piece, and four consecutive rows of two adjacent pieces, land in distinct slots).
//   * The direct loads are issued from inline assembly and waited for with explicit s_waitcnt vmcnt(n): the
//     compiler would otherwise drain every outstanding load before each LDS read. Counting is safe against any
//     other vector memory operation in flight (queries, appended-row stores): loads return in order, so extra
//     operations can only make a wait longer, never too short. Every exit path drains the loads first: a
//     workgroup's LDS must not be written after it has ended.
//
//   iteration t:  barrier (everybody finished stage t-1); request stage t+3 into the slot stage t-1 used, so that
//                 up to four stages are in flight while stage t is awaited; wait for this lane's loads of stage t;
//                 barrier (everybody's loads landed); appended rows of a tree stage go from LDS to the cache; S^T,
//                 mask, online softmax (lazy running maximum), O^T for stage t.
//
// Stages that reach past prefix_len take their rows at and beyond it from k_new / v_new when the append is
// fused; rows at and beyond the end of the segment are replaced by the segment's last row (finite data whose
// scores are masked, so their weight is exactly zero). Work split (PLAN) and partial results as in the wide
// kernel: fixed chunks, or the balanced deal of 64-key tiles.
#include <hip/hip_bf16.h>

#include <type_traits>

#include "spec_internal.h"

namespace spec {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

namespace wide32 {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int D = 128;
constexpr int SK = 32;               // keys per ring stage
constexpr int NST = 4;               // ring stages
constexpr int AHEAD = NST - 1;       // stages requested ahead of the one being consumed
constexpr int ROWB = D * 2;          // bytes per row, unpadded
constexpr int MAT = SK * ROWB;       // K (or V) part of a stage
constexpr int STAGE = 2 * MAT;
constexpr int NTHREADS = 256;
constexpr int LPS = 4;               // direct loads per lane and stage: two rows of K, two of V
constexpr int KSQ = D / 16;          // k-steps of the score product
constexpr int DB32 = D / 32;         // 32-wide d blocks of the output
constexpr int PLAN_GRID = 0, PLAN_TILES = 1;
static_assert(SPEC_WIDE_TILE_KEYS % SK == 0, "segments are made of whole stages");

__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
template <int N>
__device__ __forceinline__ void wait_loads_but() {   // at most N vector memory operations of this lane still in flight
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// 16 bytes per lane from global memory to LDS address lds_dst + 16 * lane (lds_dst wave-uniform), non-temporal:
// the K/V stream is read once per launch.
__device__ __forceinline__ void load_to_lds(const unsigned char* src, unsigned lds_dst) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt" ::"v"(src), "s"(lds_dst) : "memory");
}
// The same with the address given as a wave-uniform base and a 32-bit byte offset per lane.
__device__ __forceinline__ void load_to_lds(const unsigned char* base, unsigned off, unsigned lds_dst) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt" ::"v"(off), "s"(base), "s"(lds_dst) : "memory");
}
// A pointer that is the same in every lane, made visibly so (the base of the form above must be in scalar registers).
__device__ __forceinline__ const unsigned char* uniform_ptr(const unsigned char* p) {
  const unsigned long long v = (unsigned long long)p;
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v), hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return (const unsigned char*)(((unsigned long long)hi << 32) | lo);
}
__device__ __forceinline__ void store_nt(void* p, u32x4 v) {
  // (the builtin, not inline assembly: the compiler then keeps the store's data registers untouched for the wait
  // states a 16-byte store needs after issue)
  __builtin_nontemporal_store(v, (u32x4*)p);
}
__device__ __forceinline__ int swizzle(int row) { return ((row & 7) << 1) | ((row >> 3) & 1); }
// The value, hidden from loop-invariant code motion. The paths taken for a few stages per segment (requests that
// reach the tree, appended rows, masks) recompute their lane constants from the thread index behind this instead
// of keeping them in registers across the hot loop, where they would be spilled: a scratch reload is a vector
// memory operation and returns in order behind every direct load in flight.
__device__ __forceinline__ int opaque(int v) {
  asm volatile("" : "+v"(v));
  return v;
}

template <bool APPEND, int PLAN, bool PAGED, bool ROPE>
__global__ void __launch_bounds__(NTHREADS, 2) tree_attention_bf16_wide32_kernel(
    const __hip_bfloat16* __restrict__ q, __hip_bfloat16* k_cache, __hip_bfloat16* v_cache,
    const __hip_bfloat16* __restrict__ k_new, const __hip_bfloat16* __restrict__ v_new,
    const int32_t* __restrict__ parent, const int32_t* __restrict__ depth, const int32_t* __restrict__ prefix_len,
    __hip_bfloat16* __restrict__ out, float* __restrict__ ws_o, float* __restrict__ ws_ml, int32_t* status, int B, int N,
    int H, int H_v, int n_qg, int hpw, int S_cap, int chunk_keys, int n_splits, long q_sb, long q_sn, long q_sh,
    long n_sb, long n_sn, long n_sh, long kv_sb, long kv_sh, long kv_ss, float scale_log2, Pages pg, Rope rope) {
  __shared__ __attribute__((aligned(1024))) unsigned char ring[NST * STAGE];
  __shared__ unsigned long long s_anc[SPEC_MAX_TREE_NODES][2];
  __shared__ int s_parent[SPEC_MAX_TREE_NODES];
  __shared__ int s_depth[SPEC_MAX_TREE_NODES];
  __shared__ int s_flag;

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int r16 = lane & 15, g = lane >> 4;
  const int n32 = lane & 31, hh = lane >> 5;   // query of this lane within the wavefront's 32, half of the k range
  // loader role: in each of a stage's two rounds the 256 lanes cover 16 rows x 16 slots of K and of V; this lane
  // fills slot ld_slot of row ld_row (+16 in the second round) with the piece the swizzle assigns to it
  const int ld_col = ((t & 15) ^ swizzle(t >> 4)) * 16;
  const unsigned ring_lds = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)ring;
  const unsigned wave_lds = ring_lds + wave * 1024;
  // operand-read role: K row n32, piece 2 ks + hh; V^T rows 4 hh + (r16 >> 2) (+8), pieces 4 db + 2 (g & 1) + ...
  const int k_read = n32 * ROWB, k_xor = (hh ^ swizzle(n32 & 15)) << 4;
  const int v_row = 4 * hh + (r16 >> 2);
  const int v_read = v_row * ROWB;
  const int v_xor = (((2 * (g & 1) + ((r16 & 3) >> 1)) ^ (v_row << 1)) << 4) | ((r16 & 1) << 3);

  const unsigned cache_row_bytes = (unsigned)kv_ss * 2u, new_row_bytes = (unsigned)n_sn * 2u;
  auto page_shift = [&](int b, int k0, bool* ok) -> long {
    const int j = __builtin_amdgcn_readfirstlane(min(k0, S_cap - 1) >> pg.log2_tokens);
    const int e = pg.table[(long)b * pg.max_blocks + j];
    *ok = e >= 0 && e < pg.n_blocks;
    const int blk = min(max(e, 0), pg.n_blocks - 1);
    return (long)blk * kv_sb * 2 - (long)((unsigned)(j << pg.log2_tokens) * cache_row_bytes);
  };

  // One segment: keys [c0, min(c1_cap, prefix_len + N)) of request b, virtual head hv = K/V head h and query group
  // qg. The result is the final output (slot < 0) or float32 partials in slot `slot` of every query head served.
  auto segment = [&](const int b, const int hv, const int c0, const int c1_cap, const int slot) {
    const bool final_out = slot < 0;
    const int h = hv / n_qg, qg = hv % n_qg;
    const int P = prefix_len[b];
    const unsigned char* kc = (const unsigned char*)(k_cache + (PAGED ? 0 : b * kv_sb) + h * kv_sh);
    const unsigned char* vc = (const unsigned char*)(v_cache + (PAGED ? 0 : b * kv_sb) + h * kv_sh);
    const unsigned char* kn = APPEND ? (const unsigned char*)(k_new + b * n_sb + h * n_sh) : nullptr;
    const unsigned char* vn = APPEND ? (const unsigned char*)(v_new + b * n_sb + h * n_sh) : nullptr;

    // Requests of one stage (the 32 keys from k0) into ring slot rs. MODE 0: speculative (cache rows clamped to
    // the capacity: prefix_len is not needed), 1: clean (inside the prefix: uniform base + 32-bit lane offset),
    // 2: tail (rows clamped to the segment's last row; rows at and beyond Pk from the new K/V when the append is
    // fused).
    const unsigned lane_off = (unsigned)(t >> 4) * cache_row_bytes + (unsigned)ld_col;
    auto request = [&](int rs, int k0, auto mode_tag, int Pk, int last) {
      constexpr int MODE = decltype(mode_tag)::value;
      bool in_pool;
      const long shift = PAGED ? page_shift(b, k0, &in_pool) : 0;
      const unsigned dst = wave_lds + rs * STAGE;
      if (MODE == 1) {
        const unsigned off = lane_off + (unsigned)k0 * cache_row_bytes;
        const unsigned char* kb = uniform_ptr(kc + shift);
        const unsigned char* vb = uniform_ptr(vc + shift);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          load_to_lds(kb, off + j * 16 * cache_row_bytes, dst + j * 4096);
          load_to_lds(vb, off + j * 16 * cache_row_bytes, dst + MAT + j * 4096);
        }
      } else {
        const int tt = opaque(t);
        const int ld_row = tt >> 4, ld_col = ((tt & 15) ^ swizzle(tt >> 4)) * 16;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int row = min(k0 + ld_row + 16 * j, MODE == 0 ? S_cap - 1 : last);
          const bool from_new = (MODE == 2) && APPEND && row >= Pk;
          const long in_cache = (long)((unsigned)row * cache_row_bytes) + shift;
          const long in_new = (long)((unsigned)(row - Pk) * new_row_bytes);
          load_to_lds((from_new ? kn + in_new : kc + in_cache) + ld_col, dst + j * 4096);
          load_to_lds((from_new ? vn + in_new : vc + in_cache) + ld_col, dst + MAT + j * 4096);
        }
      }
    };
#pragma unroll
    for (int s = 0; s < AHEAD; ++s) request(s, c0 + s * SK, std::integral_constant<int, 0>{}, 0, 0);

    // The query of this lane: 16-query tile tl of the workgroup (head qg * hpw + tl / tiles_per_head of the group,
    // nodes (tl % tiles_per_head) * 16 ..), node r16 of it. Tiles past the workgroup's heads idle.
    const int group = H / (H_v / n_qg), tiles_per_head = (N + 15) / 16;
    const int tl = 2 * wave + (g & 1);
    // the last node among this wavefront's queries: a tree stage whose keys all come after it is skipped (a node
    // sees no later node; the skipped arithmetic would have added exact zeros)
    const int wave_last_node = max((2 * wave) % tiles_per_head, (2 * wave + 1) % tiles_per_head) * 16 + 15;
    const int hg = qg * hpw + tl / tiles_per_head;
    const bool live = tl / tiles_per_head < hpw && hg < group;
    const int q_head = h * group + min(hg, group - 1);
    const int node = (tl % tiles_per_head) * 16 + r16;
    bf16x8 qB[KSQ];   // Q^T as the B operand: lane (n32, hh) holds d = 16 ks + 8 hh .. + 8 of its query
#pragma unroll
    for (int ks = 0; ks < KSQ; ++ks) {
      const u32x4 raw = *(const u32x4*)(q + b * q_sb + min(node, N - 1) * q_sn + q_head * q_sh + ks * 16 + hh * 8);
      qB[ks] = __builtin_bit_cast(bf16x8, raw);
    }
    const int my_parent = parent[(long)b * N + min(t, N - 1)];
    const int my_depth = depth[(long)b * N + min(t, N - 1)];
    if (t == 0) s_flag = 0;
    if (t < N) {
      s_parent[t] = my_parent;
      s_depth[t] = my_depth;
    }
    lds_barrier();
    if (APPEND && ROPE) {
      // Rotary embedding of the queries, in registers: k-step ks of a lane holds dimensions 16 ks + 8 hh .., its
      // partner ks + KSQ/2 the same dimensions + D/2. The position is clamped into the tables (a malformed tree is
      // found only later, and its outputs are zeros).
      const int pos = min(max(P + s_depth[min(node, N - 1)], 0), rope.len - 1);
#pragma unroll
      for (int ks = 0; ks < KSQ / 2; ++ks) {
        const long at = (long)pos * (D / 2) + ks * 16 + hh * 8;
        uint4 olo, ohi;
        rope_pair<true>(__builtin_bit_cast(uint4, qB[ks]), __builtin_bit_cast(uint4, qB[ks + KSQ / 2]), rope.cos + at,
                        rope.sin + at, &olo, &ohi);
        qB[ks] = __builtin_bit_cast(bf16x8, olo);
        qB[ks + KSQ / 2] = __builtin_bit_cast(bf16x8, ohi);
      }
    }

    const bool cap_ok = (P >= 0) && (P <= S_cap - N);
    const int len = P + N;
    auto zero_outputs = [&](int bit) {
      if (final_out) {
        for (int i = t; i < hpw * N * D; i += NTHREADS) {   // every query head served here, every node
          const int hz = qg * hpw + i / (N * D), n = (i / D) % N;
          if (hz < group) out[b * q_sb + n * q_sn + (h * group + hz) * q_sh + (i % D)] = __float2bfloat16(0.f);
        }
        if (hv == 0 && t == 0) set_status(status, b, bit);
      }
    };
    if (!cap_ok) {
      zero_outputs(SPEC_ST_CAPACITY);
      wait_loads_but<0>();
      return;
    }
    if (c0 >= len) {
      wait_loads_but<0>();
      return;
    }
    const int c1 = min(c1_cap, len);
    const bool touches_tree = c1 > P;
    const int n_st = (c1 - c0 + SK - 1) / SK;
    const int n_clean = max(0, min(P, c1) - c0) / SK;
    if (PAGED) {   // every block this segment reads must lie inside the pool
      for (int j = (c0 >> pg.log2_tokens) + t; j <= ((c1 - 1) >> pg.log2_tokens); j += NTHREADS) {
        const int e = pg.table[(long)b * pg.max_blocks + j];
        if (e < 0 || e >= pg.n_blocks) set_status(status, b, SPEC_ST_BAD_BLOCK);
      }
    }
    // speculative stages that reach the tree or the end of the segment are requested again from the right
    // sources (same slot: loads land in order); one drain then makes the schedule below regular from the start
    {
      bool again = false;
#pragma unroll
      for (int s = 0; s < AHEAD; ++s)
        if (s < n_st && s >= n_clean) {
          request(s, c0 + s * SK, std::integral_constant<int, 2>{}, P, c1 - 1);
          again = true;
        }
      if (again) wait_loads_but<0>();
    }

    // ---- tree: validate, build ancestor-or-self masks
    if (touches_tree) {
      if (t < N) {
        bool ok = (t == 0) ? (my_parent == -1 && my_depth == 0) : (my_parent >= 0 && my_parent < t);
        if (ok && t > 0) ok = my_depth == s_depth[my_parent] + 1;
        if (!ok) atomicOr(&s_flag, 1);
      }
      lds_barrier();
      if (s_flag != 0) {
        zero_outputs(SPEC_ST_BAD_TREE);
        wait_loads_but<0>();
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
      lds_barrier();
    }

    f32x16 O[DB32];   // O^T: lane (n32, hh) holds d = 32 db + 8 (i / 4) + 4 hh + i % 4 of its query
    float m_run = -INFINITY, l_run = 0.f;
#pragma unroll
    for (int db = 0; db < DB32; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) O[db][i] = 0.f;

    // One stage of 32 keys from ring slot rs. S^T = K Q^T on eight 32x32x16 products: register i of lane (n32, hh)
    // is key 8 (i / 4) + 4 hh + i % 4 of the stage for query n32: the B-operand layout of P^T for two k = 16
    // products per d block (registers 0..7 and 8..15), with V^T read transposed from LDS in the same key order.
    auto compute = [&](const int st, auto rs_tag, const bool masked) {
      constexpr int rs = decltype(rs_tag)::value;   // compile-time slot: stage offsets fold into the LDS instructions
      const unsigned char* Ks = ring + rs * STAGE;
      const unsigned char* Vs = Ks + MAT;
      f32x16 sc;
#pragma unroll
      for (int i = 0; i < 16; ++i) sc[i] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KSQ; ++ks) {
        const bf16x8 a = *(const bf16x8*)(Ks + k_read + (k_xor ^ (ks << 5)));
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qB[ks], sc, 0, 0, 0);
      }
      // Schedule: all eight K operand reads of the stage, then the eight products (one exposed LDS latency
      // instead of eight); the three phases of a stage (scores, softmax, output) are kept apart: moving operand
      // reads of one phase across another buys little with two wavefronts per SIMD and costs registers.
      __builtin_amdgcn_sched_group_barrier(0x100, KSQ, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, KSQ, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (masked) {   // (a branch inside one body: two bodies per slot made the compiler copy O between them)
        const int nd = opaque(node);   // the ancestor mask is read back from LDS rather than held across clean stages
        const unsigned long long anc_lo = nd < N ? s_anc[nd][0] : 0ull, anc_hi = nd < N ? s_anc[nd][1] : 0ull;
        // visibility of the stage's 32 keys for this lane's query as one word: bit j = key kb + j is inside the
        // prefix, or tree node (kb + j - P) is the query or one of its ancestors; keys at and beyond c1 are not
        // visible. rel0 = kb - P is negative while the stage starts inside the prefix.
        const int kb = c0 + st * SK;
        const int rel0 = kb - P;
        unsigned vis32;
        if (rel0 >= 0) {
          const unsigned long long w =
              rel0 >= 64 ? (anc_hi >> (rel0 - 64)) : ((anc_lo >> rel0) | (rel0 ? anc_hi << (64 - rel0) : 0ull));
          vis32 = (unsigned)w;
        } else {
          vis32 = rel0 <= -32 ? 0xffffffffu : (((unsigned)anc_lo << (-rel0)) | ((1u << (-rel0)) - 1u));
        }
        const int left = c1 - kb;   // keys of the stage before the end of the segment
        if (left < 32) vis32 &= left <= 0 ? 0u : ((1u << left) - 1u);
        const unsigned mine = vis32 >> (4 * hh);
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (!((mine >> (8 * (i >> 2) + (i & 3))) & 1u)) sc[i] = -INFINITY;
      }
      // Lazy running maximum. m_run (exp2 domain, identical in the two lanes of a query) only has to be close to
      // the true maximum: probabilities are exp2(score - m_run) and everything is normalised by the same sum at
      // the end. It is refreshed, with the exact maximum and the usual rescaling of l and O, only when some score
      // of the wavefront exceeds it by more than 2^16 (or it is still -inf).
      float mx = fmaxf(sc[0], sc[1]);
#pragma unroll
      for (int i = 2; i < 16; ++i) mx = fmaxf(mx, sc[i]);
      mx *= scale_log2;
      if (__any(mx > m_run + 16.f)) {
        const float m_new = fmaxf(m_run, fmaxf(mx, __shfl_xor(mx, 32)));
        const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_ref);
        m_run = m_new;
        l_run *= alpha;
        // O *= alpha written as O += O * (alpha - 1): the multiply-accumulate has its destination tied to the
        // addend, which keeps the 64 accumulator registers in place on both sides of this branch (after a plain
        // multiply the compiler carried a second copy of O through the loop and moved one into the other on every
        // stage). alpha - 1 is exact for alpha in [1/2, 1]; below that the error is 2^-24 of the old O, which the
        // new reference has just made negligible.
        const float am1 = alpha - 1.f;
#pragma unroll
        for (int db = 0; db < DB32; ++db)
#pragma unroll
          for (int i = 0; i < 16; ++i) O[db][i] = __builtin_fmaf(O[db][i], am1, O[db][i]);
      }
      const float neg_m = (m_run == -INFINITY) ? 0.f : -m_run;
      float psum = 0.f;
      bf16x8 pb[2];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float p = __builtin_amdgcn_exp2f(fmaf(sc[i], scale_log2, neg_m));
        psum += p;
        pb[i >> 3][i & 7] = (__bf16)p;
      }
      l_run += psum;
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int db = 0; db < DB32; ++db) {
          const unsigned char* base = Vs + c * (16 * ROWB) + v_read + (v_xor ^ (db << 6));
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(base));
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (__attribute__((address_space(3))) s16x4*)(Vs + c * (16 * ROWB) + v_read + 8 * ROWB + ((v_xor ^ 16) ^ (db << 6))));
          union { struct { s16x4 a, b; } p; bf16x8 v; } vt;
          vt.p.a = lo;
          vt.p.b = hi;
          O[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt.v, pb[c], O[db], 0, 0, 0);
        }
      // Schedule: the V^T reads of the first four products, then each product followed by the reads of the one
      // four further on, then the last four products.
      __builtin_amdgcn_sched_group_barrier(0x100, 2 * DB32, 0);
#pragma unroll
      for (int i = 0; i < DB32; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, DB32, 0);
    };

    // Every compiler-visible load (the queries) is waited for here, before the ring starts: a wait the compiler
    // places inside the loop would count the direct loads too and drain the ring on every stage.
#pragma unroll
    for (int ks = 0; ks < KSQ; ++ks) asm volatile("" ::"v"(qB[ks]));

    // ---- ring pipeline, unrolled over the ring so that a stage's slot is a compile-time constant
    auto iteration = [&](const int st, auto rs_tag) {
      constexpr int rs = decltype(rs_tag)::value;
      lds_barrier();   // every wavefront is done with stage st - 1: its slot is free
      const int nx = st + AHEAD;
      if (nx < n_st) {
        if (nx < n_clean) request((rs + AHEAD) & (NST - 1), c0 + nx * SK, std::integral_constant<int, 1>{}, P, c1 - 1);
        else request((rs + AHEAD) & (NST - 1), c0 + nx * SK, std::integral_constant<int, 2>{}, P, c1 - 1);
      }
      // this lane's loads of stage st: every stage requested after it (up to AHEAD of them) may stay in flight
      const int younger = min(AHEAD, n_st - 1 - st);
      if (younger >= 3) wait_loads_but<3 * LPS>();
      else if (younger == 2) wait_loads_but<2 * LPS>();
      else if (younger == 1) wait_loads_but<LPS>();
      else wait_loads_but<0>();
      lds_barrier();   // stage st has landed for every lane
      const bool masked = st >= n_clean;
      if (APPEND && ROPE && masked) {
        // New K rows are rotated where they landed, before they are stored and used: a thread takes the two
        // pieces of one row that rotate with each other (piece c and c + 8 of row t / 8, at their swizzled slots).
        const int tt = opaque(t);
        const int rr = tt >> 3, c = tt & 7;
        const int row = c0 + st * SK + rr;
        if (row >= P && row < c1) {
          unsigned char* at_row = ring + rs * STAGE + rr * ROWB;
          u32x4* lo = (u32x4*)(at_row + ((c ^ swizzle(rr & 15)) << 4));
          u32x4* hi = (u32x4*)(at_row + (((c + 8) ^ swizzle(rr & 15)) << 4));
          const int pos = min(max(P + s_depth[row - P], 0), rope.len - 1);
          const long at = (long)pos * (D / 2) + c * 8;
          uint4 olo, ohi;
          rope_pair<true>(__builtin_bit_cast(uint4, *lo), __builtin_bit_cast(uint4, *hi), rope.cos + at, rope.sin + at, &olo,
                          &ohi);
          *lo = __builtin_bit_cast(u32x4, olo);
          *hi = __builtin_bit_cast(u32x4, ohi);
        }
        lds_barrier();
      }
      if (APPEND && masked && qg == 0) {   // the pair's first query group writes the appended rows to the cache
        const int k0 = c0 + st * SK;
        bool in_pool = true;               // paged cache: rows of a block outside the pool are not written
        const long shift = PAGED ? page_shift(b, k0, &in_pool) : 0;
        const int tt = opaque(t);
        const int ld_row = tt >> 4, ld_slot = tt & 15, ld_col = (ld_slot ^ swizzle(ld_row)) * 16;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int row = k0 + ld_row + 16 * j;
          if (row >= P && row < c1 && in_pool) {
            const unsigned char* src = ring + rs * STAGE + (ld_row + 16 * j) * ROWB + ld_slot * 16;
            const long off = (long)((unsigned)row * cache_row_bytes) + shift + ld_col;
            store_nt((unsigned char*)kc + off, *(const u32x4*)src);
            store_nt((unsigned char*)vc + off, *(const u32x4*)(src + MAT));
          }
        }
      }
      if (!masked || c0 + st * SK - P <= wave_last_node) compute(st, rs_tag, masked);   // else: every key is a later node
    };
#pragma nounroll
    for (int st0 = 0; st0 < n_st; st0 += NST) {
      iteration(st0, std::integral_constant<int, 0>{});
      if (st0 + 1 < n_st) iteration(st0 + 1, std::integral_constant<int, 1>{});
      if (st0 + 2 < n_st) iteration(st0 + 2, std::integral_constant<int, 2>{});
      if (st0 + 3 < n_st) iteration(st0 + 3, std::integral_constant<int, 3>{});
    }

    // ---- normalise and write, or emit the partial
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (final_out) {
      // A lane holds 8-byte pieces of its query's output row, 16 of them spread over the row: written as they are,
      // a store touches 64 rows for 8 bytes each. The wavefront's 32 rows go through its quarter of the first ring
      // slots instead (16-byte piece p of row r at slot p ^ (r & 15): the 16 lanes of a row meet no bank twice) and
      // leave as whole 256-byte rows, four rows per store.
      lds_barrier();   // every wavefront is done with the ring
      unsigned char* stg = ring + wave * (32 * ROWB);
      const float inv = 1.f / l_tot;
#pragma unroll
      for (int db = 0; db < DB32; ++db)
#pragma unroll
        for (int c4 = 0; c4 < 4; ++c4) {
          union { uint2 u; __hip_bfloat16 h4[4]; } pk;
#pragma unroll
          for (int i = 0; i < 4; ++i) pk.h4[i] = __float2bfloat16(O[db][c4 * 4 + i] * inv);
          *(uint2*)(stg + n32 * ROWB + (((db * 4 + c4) ^ (n32 & 15)) << 4) + hh * 8) = pk.u;
        }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the wavefront's own writes have landed
      const int tt = opaque(lane);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int r = 4 * j + (tt >> 4), piece = tt & 15;
        const int tl_r = 2 * wave + (r >> 4);
        const int hg_r = qg * hpw + tl_r / tiles_per_head, node_r = (tl_r % tiles_per_head) * 16 + (r & 15);
        if (tl_r / tiles_per_head < hpw && hg_r < group && node_r < N)
          store_nt((unsigned char*)(out + b * q_sb + node_r * q_sn + (h * group + hg_r) * q_sh) + piece * 16,
                   *(const u32x4*)(stg + r * ROWB + ((piece ^ (r & 15)) << 4)));
      }
    } else if (live && node < N) {
      {
        const long base = (((long)b * H + q_head) * n_splits + slot) * N + node;
#pragma unroll
        for (int db = 0; db < DB32; ++db)
#pragma unroll
          for (int c4 = 0; c4 < 4; ++c4)
            *(f32x4*)(ws_o + base * D + db * 32 + c4 * 8 + 4 * hh) =
                (f32x4){O[db][c4 * 4], O[db][c4 * 4 + 1], O[db][c4 * 4 + 2], O[db][c4 * 4 + 3]};
        if (hh == 0) {
          ws_ml[base * 2 + 0] = m_run;
          ws_ml[base * 2 + 1] = l_tot;
        }
      }
    }
  };   // segment

  if constexpr (PLAN == PLAN_GRID) {
    const int split = blockIdx.x, b = blockIdx.z;
    int hv = blockIdx.y;
    // the query groups of one (request, K/V head) pair read the same K/V: numbered 8 apart they land on one XCD
    // (workgroups go to the eight XCDs round-robin in launch order), close in time, so repeats can hit its L2
    if (n_qg > 1 && (H_v / n_qg) % 8 == 0 && gridDim.x == 1) {
      const int r = hv % (8 * n_qg), blk = hv / (8 * n_qg);
      hv = (blk * 8 + r % 8) * n_qg + r / 8;
    }
    segment(b, hv, split * chunk_keys, split * chunk_keys + chunk_keys, n_splits == 1 ? -1 : split);
  } else {
    // Tiles [pos, end) of the flattened (request, head, key tile) order belong to this workgroup; n_splits is the
    // number of partial slots per pair, filled in order by the workgroups that overlap the pair.
    constexpr int KT = SPEC_WIDE_TILE_KEYS;
    const BalancedShare bs = balanced_share(prefix_len, B, N, H_v, S_cap, KT, (int)gridDim.x);
    long pos = (long)blockIdx.x * bs.share;
    const long end = min(bs.total, pos + bs.share);
    int b = 0;
    long req_start = 0;
    int tb = request_tiles(prefix_len[0], N, S_cap, KT);
    while (pos < end) {
      while (pos >= req_start + (long)H_v * tb) {   // pos < total: a request with tiles left lies ahead
        req_start += (long)H_v * tb;
        ++b;
        tb = request_tiles(prefix_len[b], N, S_cap, KT);
      }
      const long in_req = pos - req_start;
      const int hv = (int)(in_req / tb), tile0 = (int)(in_req % tb);
      const int n_take = (int)min((long)(tb - tile0), end - pos);
      const int slot = (int)blockIdx.x - (int)((req_start + (long)hv * tb) / bs.share);
      segment(b, hv, tile0 * KT, (tile0 + n_take) * KT, slot);
      pos += n_take;
      lds_barrier();   // the ring and the tree arrays are reused by the next segment
    }
  }
}

}  // namespace wide32

hipError_t launch_tree_attention_bf16_wide32(const spec_attn_desc_t& d, const AttnPlan& plan, const Pages& pg, const void* q,
                                             void* k_cache, void* v_cache, const void* k_new, const void* v_new,
                                             const int32_t* parent, const int32_t* depth, const int32_t* prefix_len,
                                             void* out, void* ws, int32_t* status, hipStream_t s, const Rope& rope) {
  const float scale = (d.softmax_scale != 0.f ? d.softmax_scale : 1.0f / sqrtf((float)d.D)) * wide32::kLog2e;
  float* ws_o = ws ? (float*)((char*)ws + plan.ws_o_off) : nullptr;
  float* ws_ml = ws ? (float*)((char*)ws + plan.ws_ml_off) : nullptr;
  const QueryGroups qgr = attn_query_groups(d);
  const int virtual_heads = d.H_kv * qgr.n_qgroups;
  const NewStrides ns = attn_new_strides(d);
  const bool append = k_new != nullptr;
  const bool tiles_plan = plan.balanced_wgs > 0;
  const dim3 grid = tiles_plan ? dim3(plan.balanced_wgs, 1, 1) : dim3(plan.n_splits, virtual_heads, d.B);
#define SPEC_LAUNCH(APP, PLAN, PGD, RP)                                                                                  \
  hipLaunchKernelGGL((wide32::tree_attention_bf16_wide32_kernel<APP, PLAN, PGD, RP>), grid, dim3(wide32::NTHREADS), 0, s, \
                     (const __hip_bfloat16*)q, (__hip_bfloat16*)k_cache, (__hip_bfloat16*)v_cache,                   \
                     (const __hip_bfloat16*)k_new, (const __hip_bfloat16*)v_new, parent, depth, prefix_len,          \
                     (__hip_bfloat16*)out, ws_o, ws_ml, status, d.B, d.N, d.H, virtual_heads, qgr.n_qgroups,          \
                     qgr.heads_per_wg, d.S_cap, plan.chunk_keys, plan.n_splits, (long)d.q_stride_b,                  \
                     (long)d.q_stride_n, (long)d.q_stride_h, ns.b, ns.n, ns.h, (long)d.kv_stride_b,                  \
                     (long)d.kv_stride_h, (long)d.kv_stride_s, scale, pg, rope)
#define SPEC_PLANS(APP, PGD, RP)                                          \
  if (tiles_plan) SPEC_LAUNCH(APP, wide32::PLAN_TILES, PGD, RP);          \
  else SPEC_LAUNCH(APP, wide32::PLAN_GRID, PGD, RP)
#define SPEC_DISPATCH(APP, RP)                              \
  if (pg.table != nullptr) { SPEC_PLANS(APP, true, RP); }   \
  else { SPEC_PLANS(APP, false, RP); }
  // (the rotary embedding is a template parameter here, not a run-time branch as in the other kernels: this kernel
  // uses every register it may, and the extra live values of a branch that is never taken cost it 7 % of its speed)
  if (append && rope.cos != nullptr) { SPEC_DISPATCH(true, true); }
  else if (append) { SPEC_DISPATCH(true, false); }
  else { SPEC_DISPATCH(false, false); }
#undef SPEC_DISPATCH
#undef SPEC_PLANS
#undef SPEC_LAUNCH
  return hipGetLastError();
}

}  // namespace spec
