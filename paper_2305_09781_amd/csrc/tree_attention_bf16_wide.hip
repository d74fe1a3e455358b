// Tree attention for bf16 K/V, trees of 17..128 nodes per request: Definition 4.1 with the
// topology-aware causal mask of Section 4.2, same mathematics as tree_attention_bf16.hip.
//
// With many queries per K/V head (a tree of more than 16 nodes, or grouped-query heads: the query heads
// that share a K/V head bring ceil(N/16) tiles each) the wavefronts of a workgroup split the QUERIES
// (one 16-query tile each) and
// share one stream of K and V: every 64-key tile is loaded from HBM once, fully coalesced, staged in
// LDS (double-buffered, rows padded by 32 bytes), and read from there by every wavefront - K as the
// MFMA A operand (ds_read_b128), V^T through ds_read_b64_tr_b16. Shapes:
//     N <= 32 : 2 query tiles x 2 key halves (each wavefront takes one 32-key half of every tile;
//               the two halves of a query tile are merged once, through LDS, at the end)
//     N <= 64 : 4 query tiles, N <= 128 : 8 query tiles (a wavefront owns its queries over the whole
//               key range: nothing to merge).
//
//   prologue:      tiles 0 and 1 are requested together (before prefix_len is known) and staged
//   iteration ti:  S^T, online softmax, O^T for tile ti from LDS stage ti&1
//                  LDS-only barrier (it does not wait for the global loads in flight)
//                  registers holding tile ti+2 -> stage ti&1; request tile ti+2+DEPTH into them
//   so DEPTH = 2 tiles are always in flight from HBM per workgroup and one more is ready in LDS (four
//   in flight measured slower on the eight-wavefront shape, whose loop is bound inside the CU).
//
// Masked tiles (those reaching past prefix_len or the end of the segment) take the MASKED variant of
// the compute step; the loader threads zero rows past the end, and with APPEND fetch rows >= prefix_len
// from k_new / v_new and write them to the cache.
//
// Work split (PLAN): fixed chunks, grid = (n_splits, H, B); or the balanced deal of 64-key tiles over
// gridDim.x workgroups described at balanced_share(), a share that crosses a (request, head) boundary
// being processed as several segments.
#include <hip/hip_bf16.h>

#include <algorithm>
#include <type_traits>

#include "spec_internal.h"

namespace spec {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

namespace wide {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int KT = SPEC_WIDE_TILE_KEYS;   // keys per workgroup tile
constexpr int PLAN_GRID = 0, PLAN_TILES = 1;   // how work reaches the workgroups (see the end of the kernel)

__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
// 16-byte load of a K/V row piece. Marked non-temporal: the K/V stream is read once per launch, and a plain
// read of the same bytes is measurably faster with the hint.
__device__ __forceinline__ u32x4 load_kv(const unsigned char* p) {
  return __builtin_nontemporal_load((const u32x4*)p);
}
__device__ __forceinline__ void store_nt(void* p, u32x4 v) {
  // (the builtin, not inline assembly: the compiler then keeps the store's data registers untouched for the wait
  // states a 16-byte store needs after issue)
  __builtin_nontemporal_store(v, (u32x4*)p);
}
__device__ inline float max_over_lane_groups(float v) {
  v = fmaxf(v, __shfl_xor(v, 16));
  v = fmaxf(v, __shfl_xor(v, 32));
  return v;
}
__device__ inline float sum_over_lane_groups(float v) {
  v += __shfl_xor(v, 16);
  v += __shfl_xor(v, 32);
  return v;
}

// QW query wavefronts (NTW 16-query tiles each) x KW key parts: wavefront w serves query tiles
// (w % QW) * NTW .. + NTW and (KW == 2) the 32-key half w / QW of every 64-key tile.
// PAGED: the caches are pools of blocks addressed through pg.table (see cache_row_offset). Key tiles start
// at multiples of 64 rows and a block holds a multiple of 64 rows, so a tile lies inside one block: its
// rows are addressed as in a contiguous cache plus one per-tile offset (page_shift below).
template <int D, int QW, int NTW, int KW, int DEPTH, bool APPEND, int PLAN, bool PAGED>
__global__ void __launch_bounds__(QW * KW * 64, 2) tree_attention_bf16_wide_kernel(
    const __hip_bfloat16* __restrict__ q, __hip_bfloat16* k_cache, __hip_bfloat16* v_cache,
    const __hip_bfloat16* __restrict__ k_new, const __hip_bfloat16* __restrict__ v_new,
    const int32_t* __restrict__ parent, const int32_t* __restrict__ depth, const int32_t* __restrict__ prefix_len,
    __hip_bfloat16* __restrict__ out, float* __restrict__ ws_o, float* __restrict__ ws_ml, int32_t* status, int B, int N,
    int H, int H_v, int n_qg, int hpw, int heads_per_wg, int S_cap, int chunk_keys, int n_splits, long q_sb, long q_sn, long q_sh, long n_sb, long n_sn,
    long n_sh, long kv_sb, long kv_sh, long kv_ss, float scale_log2, Pages pg, Rope rope) {
  static_assert(KW == 1 || KW == 2, "a 64-key tile is consumed as two 32-key halves");
  static_assert(DEPTH == 2 || DEPTH == 4, "register sets of tiles in flight");
  constexpr int WAVES = QW * KW;
  constexpr int NTHREADS = WAVES * 64;
  constexpr int KS = D / 32, DB = D / 16;
  constexpr int LPR = D * 2 / 16;            // 16-byte pieces per row
  constexpr int NPT = KT * LPR / NTHREADS;   // pieces of K (and of V) per thread and tile
  constexpr int ROWB = D * 2 + 32;           // LDS bytes per staged row (+32: consecutive rows shift by 8 banks)
  constexpr int MAT_BYTES = KT * ROWB;       // one staged matrix (K or V)
  constexpr int STAGE_BYTES = 2 * MAT_BYTES;
  constexpr int ROW_STEP = NTHREADS / LPR;
  static_assert(NPT >= 1 && KT % ROW_STEP == 0, "loader layout");
  static_assert(KW == 1 || QW * NTW * 64 * (DB * 4 + 2) * 4 <= 2 * STAGE_BYTES, "merge area fits the staging area");

  __shared__ __attribute__((aligned(16))) unsigned char lds[2 * STAGE_BYTES];
  __shared__ unsigned long long s_anc[SPEC_MAX_TREE_NODES][2];
  __shared__ int s_parent[SPEC_MAX_TREE_NODES];
  __shared__ int s_depth[SPEC_MAX_TREE_NODES];
  __shared__ int s_flag;

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int r16 = lane & 15, g = lane >> 4;
  const int qt = wave % QW, kpart = wave / QW;
  // loader role of this thread: piece j of a tile is row (t + NTHREADS j) / LPR, 16-byte column (t % LPR)
  const int ld_row0 = t / LPR, ld_col = (t % LPR) * 16;

  // DEPTH register sets: the tiles in flight from global memory (tiles ti+2 .. ti+1+DEPTH while tile ti
  // is consumed from LDS and tile ti+1 waits there)
  u32x4 Kr[DEPTH][NPT], Vr[DEPTH][NPT];
  const unsigned cache_row_bytes = (unsigned)kv_ss * 2u, new_row_bytes = (unsigned)n_sn * 2u;
  // Speculative request of one tile: cache rows only, clamped to the capacity, no prefix_len needed.
  // Paged cache: byte offset that, added to `row * cache_row_bytes`, gives the place of logical row `row` of
  // request b for every row of the 64-row tile at k0 (rows clamped to the capacity or to the request's last
  // row stay inside the tile, hence inside its block). `ok`: the table entry lies inside the pool; one that
  // does not is replaced by a block of the pool.
  auto page_shift = [&](int b, int k0, bool* ok) -> long {
    const int j = __builtin_amdgcn_readfirstlane(min(k0, S_cap - 1) >> pg.log2_tokens);
    const int e = pg.table[(long)b * pg.max_blocks + j];
    *ok = e >= 0 && e < pg.n_blocks;
    const int blk = min(max(e, 0), pg.n_blocks - 1);
    return (long)blk * kv_sb * 2 - (long)((unsigned)(j << pg.log2_tokens) * cache_row_bytes);
  };
  auto issue_speculative = [&](u32x4 (&Kd)[NPT], u32x4 (&Vd)[NPT], const unsigned char* kbase, const unsigned char* vbase,
                               int k0, long shift) {
#pragma unroll
    for (int j = 0; j < NPT; ++j) {
      const int row = min(k0 + ld_row0 + j * ROW_STEP, S_cap - 1);
      const long off = (long)((unsigned)row * cache_row_bytes) + shift;
      Vd[j] = load_kv(vbase + off + ld_col);
      Kd[j] = load_kv(kbase + off + ld_col);
    }
  };

  // One segment: keys [c0, min(c1_cap, prefix_len + N)) of request b, virtual head hv = K/V head h and query
  // group qg (hpw of the H / H_kv query heads that share h). The result is the final output (slot < 0) or
  // float32 partials in slot `slot` of every query head served here.
  // nh > 1 (only with one query group per K/V head, one key part per wavefront and final outputs): the
  // workgroup serves the nh consecutive K/V heads h .. h + nh - 1 of the request as ONE stream of nh * n_tiles
  // tiles. The tree work is done once, the next head's first tiles are requested while the current head's
  // last ones are computed, and its queries wait in registers (qB_next): a head boundary costs a normalise and
  // store, not a prologue.
  auto segment = [&](const int b, const int hv, const int c0, const int c1_cap, const int slot, const int nh) {
    const bool final_out = slot < 0;
    const int h = hv / n_qg, qg = hv % n_qg;

    // ---- straight-line prologue: first two tiles (they do not depend on prefix_len), Q, one tree node per thread
    const int P = prefix_len[b];
    const unsigned char* kc = (const unsigned char*)(k_cache + (PAGED ? 0 : b * kv_sb) + h * kv_sh);
    const unsigned char* vc = (const unsigned char*)(v_cache + (PAGED ? 0 : b * kv_sb) + h * kv_sh);
    const unsigned char* kn = APPEND ? (const unsigned char*)(k_new + b * n_sb + h * n_sh) : nullptr;
    const unsigned char* vn = APPEND ? (const unsigned char*)(v_new + b * n_sb + h * n_sh) : nullptr;
    const long new_minus_cache_k = APPEND ? (long)(kn - kc) : 0, new_minus_cache_v = APPEND ? (long)(vn - vc) : 0;

    // MODE: 1 = clean (no clamp), 2 = tail (clamp, new rows)
    auto issue = [&](u32x4 (&Kd)[NPT], u32x4 (&Vd)[NPT], int k0, auto mode_tag, int Pk, int last_row, int hi) {
      constexpr int MODE = decltype(mode_tag)::value;
      bool in_pool;
      // head hi of the stream: its cache rows lie hi * kv_sh further, its new rows hi * n_sh
      const long shift = (PAGED ? page_shift(b, k0, &in_pool) : 0) + (long)hi * kv_sh * 2;
      const long new_shift = (long)hi * n_sh * 2;
#pragma unroll
      for (int j = 0; j < NPT; ++j) {
        int row = k0 + ld_row0 + j * ROW_STEP;
        long off_k, off_v;   // byte offsets from the cache bases (new rows: through the distance between the buffers)
        if (MODE == 1) {
          off_k = off_v = (long)((unsigned)row * cache_row_bytes) + shift;
        } else {
          row = min(row, last_row);
          const bool from_new = (MODE == 2) && APPEND && row >= Pk;
          const long in_cache = (long)((unsigned)row * cache_row_bytes) + shift;
          const long in_new = (long)((unsigned)(row - Pk) * new_row_bytes);
          off_k = from_new ? new_minus_cache_k + new_shift + in_new : in_cache;
          off_v = from_new ? new_minus_cache_v + new_shift + in_new : in_cache;
        }
        Vd[j] = load_kv(vc + off_v + ld_col);
        Kd[j] = load_kv(kc + off_k + ld_col);
      }
    };
    // The first two tiles are requested before prefix_len is known. Where they stand relative to the queries and
    // the tree words decides what the first wait leaves in flight (loads return in order): tiles first on the shapes
    // with one key part per wavefront; on the 2 x 2 shape the tree words and queries first, so that the wait for the
    // tree words does not wait for the tiles too (alternating builds on the same buffers: 145.8 -> 144.5 us on a
    // ragged batch of 8192-16384 keys, while the other shapes lose half a percent with that order).
    auto first_tiles = [&]() {
      bool in_pool;   // entries past the request's end may hold anything: not judged here
      issue_speculative(Kr[0], Vr[0], kc, vc, c0, PAGED ? page_shift(b, c0, &in_pool) : 0);
      issue_speculative(Kr[1], Vr[1], kc, vc, c0 + KT, PAGED ? page_shift(b, c0 + KT, &in_pool) : 0);
    };
    if (KW == 1) first_tiles();

    // Query tiles of this workgroup: hpw of the `group` query heads that share the K/V head (heads
    // qg * hpw .. of the group), ceil(N/16) tiles each (multi-head attention: group = hpw = 1). Tile tl of
    // a wavefront serves head h * group + qg * hpw + tl / tiles_per_head, nodes (tl % tiles_per_head) * 16 ..
    // + 16; tiles past the workgroup's heads idle.
    const int group = H / (H_v / n_qg), tiles_per_head = (N + 15) / 16;
    int tile_head[NTW], tile_node[NTW];   // head within the group (clamped), node of this lane (may be >= N)
    bool tile_live[NTW];
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt) {
      const int tl = (qt * NTW + nt);
      const int hg = qg * hpw + tl / tiles_per_head;
      tile_live[nt] = tl / tiles_per_head < hpw && hg < group;
      tile_head[nt] = min(hg, group - 1);
      tile_node[nt] = (tl % tiles_per_head) * 16 + r16;
    }
    bf16x8 qB[NTW][KS], qB_next[NTW][KS];
    auto load_q = [&](bf16x8 (&dst)[NTW][KS], int hi) {
#pragma unroll
      for (int nt = 0; nt < NTW; ++nt) {
        const int n = tile_node[nt], head = (h + hi) * group + tile_head[nt];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const u32x4 raw = *(const u32x4*)(q + b * q_sb + min(n, N - 1) * q_sn + head * q_sh + ks * 32 + g * 8);
          dst[nt][ks] = __builtin_bit_cast(bf16x8, raw);
        }
      }
    };
    const int my_parent = parent[(long)b * N + min(t, N - 1)];
    const int my_depth = depth[(long)b * N + min(t, N - 1)];
    load_q(qB, 0);
    if (nh > 1) load_q(qB_next, 1);
    if (KW == 2) {
      __builtin_amdgcn_sched_barrier(0);   // (keeps the compiler from moving the tile requests ahead again)
      first_tiles();
      __builtin_amdgcn_sched_barrier(0);
    }
    if (t == 0) s_flag = 0;
    if (t < N) {
      s_parent[t] = my_parent;
      s_depth[t] = my_depth;
    }
    lds_barrier();
    // Rotary embedding of the queries, in registers: k-step ks of a lane holds dimensions 32 ks + 8 g .., its
    // partner ks + KS/2 the same dimensions + D/2. A position is clamped into the tables (a malformed tree is
    // found only later, and its outputs are zeros).
    auto rotate_q = [&](bf16x8 (&dst)[NTW][KS]) {
#pragma unroll
      for (int nt = 0; nt < NTW; ++nt) {
        const int pos = min(max(P + s_depth[min(tile_node[nt], N - 1)], 0), rope.len - 1);
#pragma unroll
        for (int ks = 0; ks < KS / 2; ++ks) {
          const long at = (long)pos * (D / 2) + ks * 32 + g * 8;
          uint4 olo, ohi;
          rope_pair<true>(__builtin_bit_cast(uint4, dst[nt][ks]), __builtin_bit_cast(uint4, dst[nt][ks + KS / 2]),
                          rope.cos + at, rope.sin + at, &olo, &ohi);
          dst[nt][ks] = __builtin_bit_cast(bf16x8, olo);
          dst[nt][ks + KS / 2] = __builtin_bit_cast(bf16x8, ohi);
        }
      }
    };
    if (APPEND && rope.cos != nullptr) rotate_q(qB);

    const bool cap_ok = (P >= 0) && (P <= S_cap - N);
    const int len = P + N;
    auto zero_outputs = [&](int bit) {
      if (final_out) {
        for (int hi = 0; hi < nh; ++hi)
          for (int i = t; i < hpw * N * D; i += NTHREADS) {   // every query head served here, every node
            const int hg = qg * hpw + i / (N * D), n = (i / D) % N;
            if (hg < group) out[b * q_sb + n * q_sn + ((h + hi) * group + hg) * q_sh + (i % D)] = __float2bfloat16(0.f);
          }
        if (hv == 0 && t == 0) set_status(status, b, bit);
      }
    };
    if (!cap_ok) {
      zero_outputs(SPEC_ST_CAPACITY);
      return;
    }
    if (c0 >= len) return;
    const int c1 = min(c1_cap, len);
    const bool touches_tree = c1 > P;
    const int n_tiles = (c1 - c0 + KT - 1) / KT;
    const int n_clean = max(0, min(P, c1) - c0) / KT;
    const int last_row = len - 1;
    if (PAGED) {   // every block this segment reads must lie inside the pool
      for (int j = (c0 >> pg.log2_tokens) + t; j <= ((c1 - 1) >> pg.log2_tokens); j += NTHREADS) {
        const int e = pg.table[(long)b * pg.max_blocks + j];
        if (e < 0 || e >= pg.n_blocks) set_status(status, b, SPEC_ST_BAD_BLOCK);
      }
    }

    // speculative tiles that reach the tree are fetched again from the right sources
    if (APPEND && n_clean == 0) issue(Kr[0], Vr[0], c0, std::integral_constant<int, 2>{}, P, last_row, 0);
    if (n_tiles > 1) {
      if (APPEND && n_clean <= 1) issue(Kr[1], Vr[1], c0 + KT, std::integral_constant<int, 2>{}, P, last_row, 0);
    } else if (nh > 1) {   // the second tile of the stream is the next head's first
      if (KT <= P) issue(Kr[1], Vr[1], c0, std::integral_constant<int, 1>{}, P, last_row, 1);
      else issue(Kr[1], Vr[1], c0, std::integral_constant<int, 2>{}, P, last_row, 1);
    }
    const int total_tiles = nh * n_tiles;   // tile gt of the stream: head gt / n_tiles, tile gt % n_tiles of that head

    // ---- tree: validate, build ancestor-or-self masks (LDS-only barriers: the tile loads stay in flight)
    unsigned long long anc_lo[NTW], anc_hi[NTW];
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt) anc_lo[nt] = anc_hi[nt] = 0ull;
    if (touches_tree) {
      if (t < N) {
        bool ok = (t == 0) ? (my_parent == -1 && my_depth == 0) : (my_parent >= 0 && my_parent < t);
        if (ok && t > 0) ok = my_depth == s_depth[my_parent] + 1;
        if (!ok) atomicOr(&s_flag, 1);
      }
      lds_barrier();
      if (s_flag != 0) {
        zero_outputs(SPEC_ST_BAD_TREE);
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
#pragma unroll
      for (int nt = 0; nt < NTW; ++nt) {
        const int n = tile_node[nt];
        if (n < N) { anc_lo[nt] = s_anc[n][0]; anc_hi[nt] = s_anc[n][1]; }
      }
    }

    // registers -> LDS stage; masked tiles: rows past the segment end become zeros, appended rows go to the cache
    auto stage_tile = [&](u32x4 (&Ks_)[NPT], u32x4 (&Vs_)[NPT], int gt, unsigned char* stage) {
      int hi = 0, ti = gt;
      while (ti >= n_tiles) { ti -= n_tiles; ++hi; }
      const int k0 = c0 + ti * KT;
      const bool masked = ti >= n_clean;
      bool in_pool = true;   // paged cache: rows of a block outside the pool are not written
      const long shift = ((PAGED && APPEND && masked) ? page_shift(b, k0, &in_pool) : 0) + (long)hi * kv_sh * 2;
      if (APPEND && masked && rope.cos != nullptr) {
        // New K rows are rotated before they are stored and used. A thread holds one 16-byte piece of a row; the
        // piece it rotates with (the same dimensions -+ D/2) is held LPR/2 lanes away in the same wavefront.
#pragma unroll
        for (int j = 0; j < NPT; ++j) {
          u32x4 other;
#pragma unroll
          for (int e = 0; e < 4; ++e) other[e] = __shfl_xor(Ks_[j][e], LPR / 2);
          const int row = k0 + ld_row0 + j * ROW_STEP;
          if (row >= P && row < c1) {
            const int piece = t % LPR;
            const bool low = piece < LPR / 2;
            const int pos = min(max(P + s_depth[row - P], 0), rope.len - 1);
            const long at = (long)pos * (D / 2) + (piece % (LPR / 2)) * 8;
            uint4 olo, ohi;
            rope_pair<true>(__builtin_bit_cast(uint4, low ? Ks_[j] : other), __builtin_bit_cast(uint4, low ? other : Ks_[j]),
                            rope.cos + at, rope.sin + at, &olo, &ohi);
            Ks_[j] = __builtin_bit_cast(u32x4, low ? olo : ohi);
          }
        }
      }
#pragma unroll
      for (int j = 0; j < NPT; ++j) {
        const int rit = ld_row0 + j * ROW_STEP;
        if (masked) {
          const int row = k0 + rit;
          if (row >= c1) {
            Ks_[j] = (u32x4){0u, 0u, 0u, 0u};
            Vs_[j] = (u32x4){0u, 0u, 0u, 0u};
          } else if (APPEND && qg == 0 && row >= P && in_pool) {   // the pair's first query group writes the new rows
            store_nt((unsigned char*)kc + (unsigned)row * cache_row_bytes + shift + ld_col, Ks_[j]);
            store_nt((unsigned char*)vc + (unsigned)row * cache_row_bytes + shift + ld_col, Vs_[j]);
          }
        }
        *(u32x4*)(stage + rit * ROWB + ld_col) = Ks_[j];
        *(u32x4*)(stage + MAT_BYTES + rit * ROWB + ld_col) = Vs_[j];
      }
    };
    auto issue_tile = [&](u32x4 (&Kd)[NPT], u32x4 (&Vd)[NPT], int gt) {
      int hi = 0, ti = gt;
      while (ti >= n_tiles) { ti -= n_tiles; ++hi; }
      const int k0 = c0 + ti * KT;
      if (k0 + KT <= P) issue(Kd, Vd, k0, std::integral_constant<int, 1>{}, P, last_row, hi);
      else issue(Kd, Vd, k0, std::integral_constant<int, 2>{}, P, last_row, hi);
    };

    f32x4 O[NTW][DB];
    float m_run[NTW], l_run[NTW];
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt) {
      m_run[nt] = -INFINITY;
      l_run[nt] = 0.f;
#pragma unroll
      for (int db = 0; db < DB; ++db) O[nt][db] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }

    auto compute = [&](const int ti, const unsigned char* stage, auto masked_tag) {
      constexpr bool MASKED = decltype(masked_tag)::value;
      const int k0 = c0 + ti * KT;
      const unsigned char* Ks = stage;
      const unsigned char* Vs = stage + MAT_BYTES;
      // The 64-key stage is consumed as 32-key halves: both by this wavefront, or (KW == 2) one each.
#pragma unroll
      for (int part = 0; part < 2 / KW; ++part) {
        const int grp = KW == 2 ? kpart : part;
        // ---- S^T = K Q^T for two 16-key quarters; a K operand is read once and used by all query tiles
        f32x4 sc[NTW][2];
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
          for (int hf = 0; hf < 2; ++hf) sc[nt][hf] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 a = *(const bf16x8*)(Ks + (grp * 32 + hf * 16 + r16) * ROWB + ks * 64 + g * 16);
#pragma unroll
            for (int nt = 0; nt < NTW; ++nt)
              sc[nt][hf] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qB[nt][ks], sc[nt][hf], 0, 0, 0);
          }

        bf16x8 pB[NTW];
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) {
          float s[8];   // raw scores (before the softmax scale)
#pragma unroll
          for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int v = 0; v < 4; ++v) s[hf * 4 + v] = sc[nt][hf][v];
          if (MASKED) {
#pragma unroll
            for (int hf = 0; hf < 2; ++hf)
#pragma unroll
              for (int v = 0; v < 4; ++v) {
                const int key = k0 + grp * 32 + hf * 16 + 4 * g + v;
                const int rel = key - P;
                bool vis = key < c1;
                if (vis && rel >= 0) {
                  const unsigned long long w = rel < 64 ? anc_lo[nt] : anc_hi[nt];
                  vis = (w >> (rel & 63)) & 1ull;
                }
                if (!vis) s[hf * 4 + v] = -INFINITY;
              }
          }
          // Lazy running maximum. m_run (exp2 domain, identical in the four lanes of a query) only has to
          // be close to the true maximum: probabilities are exp2(score - m_run) and everything is
          // normalised by the same sum at the end. It is refreshed, with the exact cross-lane maximum and
          // the usual rescaling of l and O, only when some score of the wavefront exceeds it by more than
          // 2^16 (or it is still -inf); otherwise the tile costs one fma and one exp2 per score.
          const float mx =
              fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7]))) * scale_log2;
          if (__any(mx > m_run[nt] + 16.f)) {
            const float m_new = fmaxf(m_run[nt], max_over_lane_groups(mx));
            const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = __builtin_amdgcn_exp2f(m_run[nt] - m_ref);
            m_run[nt] = m_new;
            l_run[nt] *= alpha;
#pragma unroll
            for (int db = 0; db < DB; ++db) O[nt][db] *= alpha;
          }
          const float neg_m = (m_run[nt] == -INFINITY) ? 0.f : -m_run[nt];
          float psum = 0.f;
          bf16x8 pb;
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const float p = __builtin_amdgcn_exp2f(fmaf(s[i], scale_log2, neg_m));   // i<4: first quarter, i>=4: second
            psum += p;
            pb[i] = (__bf16)p;
          }
          pB[nt] = pb;
          l_run[nt] += psum;
        }

        // ---- O^T += V^T P^T; a V^T operand is read once and used by all query tiles
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const unsigned char* base = Vs + (grp * 32 + 4 * g + (r16 >> 2)) * ROWB + db * 32 + (r16 & 3) * 8;
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(base));
          const s16x4 hi =
              __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(base + 16 * ROWB));
          union { struct { s16x4 a, b; } p; bf16x8 v; } vt;
          vt.p.a = lo;
          vt.p.b = hi;
#pragma unroll
          for (int nt = 0; nt < NTW; ++nt)
            O[nt][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt.v, pB[nt], O[nt][db], 0, 0, 0);
        }
      }
    };

    // ---- pipeline. Tile ti is consumed from LDS stage ti&1 while tile ti+1 sits in the other stage and
    // tiles ti+2 .. ti+1+DEPTH are in flight, tile k in register set k % DEPTH. Tiles 0 and 1 were
    // requested at the start; the others of the first DEPTH are requested now. After the barrier that
    // ends tile ti, tile ti+2 is written over it from its register set and tile ti+2+DEPTH is requested
    // into that set.
#pragma unroll
    for (int d = 2; d < DEPTH; ++d)
      if (d < total_tiles) issue_tile(Kr[d], Vr[d], d);
    stage_tile(Kr[0], Vr[0], 0, lds);
    if (DEPTH < total_tiles) issue_tile(Kr[0], Vr[0], DEPTH);
    if (total_tiles > 1) stage_tile(Kr[1], Vr[1], 1, lds + STAGE_BYTES);
    if (DEPTH + 1 < total_tiles) issue_tile(Kr[1], Vr[1], DEPTH + 1);
    lds_barrier();
    // Normalised output of the query tiles of stream head hi (final outputs only).
    auto write_out = [&](const float (&l_tot)[NTW], int hi) {
#pragma unroll
      for (int nt = 0; nt < NTW; ++nt) {
        const int n = tile_node[nt], head = (h + hi) * group + tile_head[nt];
        if (kpart == 0 && tile_live[nt] && n < N) {
          const float inv = 1.f / l_tot[nt];
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            union { uint2 u; __hip_bfloat16 h4[4]; } pk;
#pragma unroll
            for (int i = 0; i < 4; ++i) pk.h4[i] = __float2bfloat16(O[nt][db][i] * inv);
            *(uint2*)(out + b * q_sb + n * q_sn + head * q_sh + db * 16 + 4 * g) = pk.u;
          }
        }
      }
    };
    int cur_head = 0, cur_ti = 0;   // head and in-head tile of the stream tile being computed
    auto step = [&](int gt, u32x4 (&Kd)[NPT], u32x4 (&Vd)[NPT]) {   // Kd, Vd: the register set of tile gt+2
      unsigned char* cur = lds + (gt & 1) * STAGE_BYTES;
      if (cur_ti >= n_clean) compute(cur_ti, cur, std::true_type{});
      else compute(cur_ti, cur, std::false_type{});
      if (++cur_ti == n_tiles && cur_head + 1 < nh) {
        // Head boundary (KW == 1: a wavefront owns its query tiles' whole state): write this head's outputs,
        // take the next head's queries from qB_next, request the queries of the head after it.
        float l_tot[NTW];
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) l_tot[nt] = sum_over_lane_groups(l_run[nt]);
        write_out(l_tot, cur_head);
        ++cur_head;
        cur_ti = 0;
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) {
          m_run[nt] = -INFINITY;
          l_run[nt] = 0.f;
#pragma unroll
          for (int db = 0; db < DB; ++db) O[nt][db] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) qB[nt][ks] = qB_next[nt][ks];
        }
        if (APPEND && rope.cos != nullptr) rotate_q(qB);
        if (cur_head + 1 < nh) load_q(qB_next, cur_head + 1);
      }
      lds_barrier();
      if (gt + 2 < total_tiles) {
        stage_tile(Kd, Vd, gt + 2, cur);
        if (gt + 2 + DEPTH < total_tiles) issue_tile(Kd, Vd, gt + 2 + DEPTH);
      }
    };
    for (int gt = 0; gt < total_tiles; gt += DEPTH) {
#pragma unroll
      for (int d = 0; d < DEPTH; ++d)
        if (gt + d < total_tiles) step(gt + d, Kr[(d + 2) % DEPTH], Vr[(d + 2) % DEPTH]);
    }
    lds_barrier();

    // ---- two key halves per query tile: the wavefront of the second half hands its state over through
    // LDS (layout [query wavefront][tile][register][lane], then m and l), the first merges.
    float l_tot[NTW];
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt) l_tot[nt] = sum_over_lane_groups(l_run[nt]);
    if (KW == 2) {
      constexpr int MG_TILE = 64 * (DB * 4 + 2);
      float* mg = (float*)lds + qt * NTW * MG_TILE;
      if (kpart == 1) {
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) {
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 4; ++i) mg[nt * MG_TILE + (db * 4 + i) * 64 + lane] = O[nt][db][i];
          mg[nt * MG_TILE + (DB * 4) * 64 + lane] = m_run[nt];
          mg[nt * MG_TILE + (DB * 4 + 1) * 64 + lane] = l_tot[nt];
        }
      }
      lds_barrier();
      if (kpart == 0) {
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) {
          const float m_other = mg[nt * MG_TILE + (DB * 4) * 64 + lane], l_other = mg[nt * MG_TILE + (DB * 4 + 1) * 64 + lane];
          const float m_new = fmaxf(m_run[nt], m_other);
          const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;
          const float a_self = __builtin_amdgcn_exp2f(m_run[nt] - m_ref), a_other = __builtin_amdgcn_exp2f(m_other - m_ref);
          m_run[nt] = m_new;
          l_tot[nt] = l_tot[nt] * a_self + l_other * a_other;
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 4; ++i)
              O[nt][db][i] = O[nt][db][i] * a_self + mg[nt * MG_TILE + (db * 4 + i) * 64 + lane] * a_other;
        }
      }
    }

    // ---- normalise and write the (last) head, or emit the partial
    if (final_out) write_out(l_tot, nh - 1);
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt) {
      const int n = tile_node[nt], head = h * group + tile_head[nt];
      if (kpart == 0 && tile_live[nt] && n < N) {
        if (!final_out) {
          const long base = (((long)b * H + head) * n_splits + slot) * N + n;
#pragma unroll
          for (int db = 0; db < DB; ++db) *(f32x4*)(ws_o + base * D + db * 16 + 4 * g) = O[nt][db];
          if (g == 0) {
            ws_ml[base * 2 + 0] = m_run[nt];
            ws_ml[base * 2 + 1] = l_tot[nt];
          }
        }
      }
    }
  };   // segment

  if constexpr (PLAN == PLAN_GRID) {
    const int split = blockIdx.x, b = blockIdx.z;
    int hv = blockIdx.y;
    // Workgroups are handed to the eight XCDs round-robin in launch order and every XCD has its own L2. The
    // query groups of one (request, K/V head) pair read the same K/V: numbering them 8 apart puts them on
    // one XCD, close in time, so that the repeats can be L2 hits.
    if (n_qg > 1 && (H_v / n_qg) % 8 == 0 && gridDim.x == 1) {
      const int r = hv % (8 * n_qg), blk = hv / (8 * n_qg);
      hv = (blk * 8 + r % 8) * n_qg + r / 8;
    }
    if (heads_per_wg > 1) {   // several K/V heads per workgroup (host: one query group per head, no key split)
      hv *= heads_per_wg;
      segment(b, hv, 0, chunk_keys, -1, min(heads_per_wg, H_v - hv));
    } else {
      segment(b, hv, split * chunk_keys, split * chunk_keys + chunk_keys, n_splits == 1 ? -1 : split, 1);
    }
  } else {
    // Tiles [pos, end) of the flattened (request, head, key tile) order belong to this workgroup.
    // n_splits is the number of partial slots per pair; the workgroups overlapping a pair fill slots
    // 0, 1, ... in order.
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
      segment(b, hv, tile0 * KT, (tile0 + n_take) * KT, slot, 1);
      pos += n_take;
      lds_barrier();   // LDS (staging tiles, merge area, tree arrays) is reused by the next segment
    }
  }
}

}  // namespace wide

hipError_t launch_tree_attention_bf16_wide(const spec_attn_desc_t& d, const AttnPlan& plan, const Pages& pg, const void* q, void* k_cache,
                                           void* v_cache, const void* k_new, const void* v_new, const int32_t* parent,
                                           const int32_t* depth, const int32_t* prefix_len, void* out, void* ws,
                                           int32_t* status, hipStream_t s, const Rope& rope) {
  const float scale = (d.softmax_scale != 0.f ? d.softmax_scale : 1.0f / sqrtf((float)d.D)) * wide::kLog2e;
  float* ws_o = ws ? (float*)((char*)ws + plan.ws_o_off) : nullptr;
  float* ws_ml = ws ? (float*)((char*)ws + plan.ws_ml_off) : nullptr;
  // one 16-query tile per wavefront: 2 x 2 key halves up to 32 nodes, four up to 64, eight up to 128
  const QueryGroups qgr = attn_query_groups(d);
  const int tiles = qgr.tiles_per_wg;   // (query heads per workgroup) x ceil(N / 16)
  const int virtual_heads = d.H_kv * qgr.n_qgroups;
  const int qw = tiles <= 2 ? 2 : tiles <= 4 ? 4 : 8;
  if (plan.m32)   // five to eight query tiles, head dimension 128: four wavefronts of 32 queries, K/V straight to LDS
    return launch_tree_attention_bf16_wide32(d, plan, pg, q, k_cache, v_cache, k_new, v_new, parent, depth, prefix_len, out,
                                             ws, status, s, rope);
  const NewStrides ns = attn_new_strides(d);
  const bool append = k_new != nullptr;
  const int mode = plan.balanced_wgs == 0 ? wide::PLAN_GRID : wide::PLAN_TILES;
  // Whole key ranges, one query group per K/V head, a wavefront per query tile: a workgroup may serve several
  // consecutive K/V heads of a request as one stream (the plan decides how many).
  const int heads_per_wg = (mode == wide::PLAN_GRID && plan.n_splits == 1 && qgr.n_qgroups == 1 && qw == 8)
                               ? std::max(1, plan.heads_per_wg) : 1;
  const dim3 grid = mode != wide::PLAN_GRID
                        ? dim3(plan.balanced_wgs, 1, 1)
                        : dim3(plan.n_splits, (virtual_heads + heads_per_wg - 1) / heads_per_wg, d.B);
#define SPEC_LAUNCH(DD, QQ, NTT, KK, DP, APP, PLAN, PGD)                                                              \
  hipLaunchKernelGGL((wide::tree_attention_bf16_wide_kernel<DD, QQ, NTT, KK, DP, APP, PLAN, PGD>), grid, dim3(QQ * KK * 64), 0, s, \
                     (const __hip_bfloat16*)q, (__hip_bfloat16*)k_cache, (__hip_bfloat16*)v_cache,                    \
                     (const __hip_bfloat16*)k_new, (const __hip_bfloat16*)v_new, parent, depth, prefix_len,           \
                     (__hip_bfloat16*)out, ws_o, ws_ml, status, d.B, d.N, d.H, virtual_heads, qgr.n_qgroups,           \
                     qgr.heads_per_wg, heads_per_wg, d.S_cap, plan.chunk_keys,                                        \
                     plan.n_splits, (long)d.q_stride_b, (long)d.q_stride_n, (long)d.q_stride_h, ns.b, ns.n, ns.h,     \
                     (long)d.kv_stride_b, (long)d.kv_stride_h, (long)d.kv_stride_s, scale, pg, rope)
#define SPEC_SHAPES(DD, APP, PLAN, PGD)                          \
  if (qw == 2) SPEC_LAUNCH(DD, 2, 1, 2, 2, APP, PLAN, PGD);      \
  else if (qw == 4) SPEC_LAUNCH(DD, 4, 1, 1, 2, APP, PLAN, PGD); \
  else SPEC_LAUNCH(DD, 8, 1, 1, 2, APP, PLAN, PGD)
#define SPEC_DIMS(APP, PLAN, PGD)                            \
  if (d.D == 128) { SPEC_SHAPES(128, APP, PLAN, PGD); }      \
  else { SPEC_SHAPES(64, APP, PLAN, PGD); }
#define SPEC_PLANS(APP, PGD)                                                 \
  if (mode == wide::PLAN_GRID) { SPEC_DIMS(APP, wide::PLAN_GRID, PGD); }     \
  else { SPEC_DIMS(APP, wide::PLAN_TILES, PGD); }
#define SPEC_DISPATCH(APP)                               \
  if (pg.table != nullptr) { SPEC_PLANS(APP, true); }    \
  else { SPEC_PLANS(APP, false); }
  if (append) { SPEC_DISPATCH(true); } else { SPEC_DISPATCH(false); }
#undef SPEC_DISPATCH
#undef SPEC_PLANS
#undef SPEC_DIMS
#undef SPEC_SHAPES
#undef SPEC_LAUNCH
  return hipGetLastError();
}

}  // namespace spec
