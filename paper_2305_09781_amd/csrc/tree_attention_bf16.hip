// Tree attention for bf16 K/V on the gfx950 matrix cores (Definition 4.1; topology-aware causal mask
// of Section 4.2), written for the decode-shaped case: few tree queries (N <= 16, one MFMA query
// tile; larger trees go to the kernel in tree_attention_bf16_wide.hip) against a long cached prefix,
// so the kernel is bound by streaming K and V from HBM exactly once.
//
// Decomposition
//   grid = (n_splits, H, B), or (BAL) gridDim.x workgroups that share the 32-key tiles of all
//   (request, head) pairs equally (see balanced_share()). A workgroup owns one segment of the key
//   range of one (request, head) at a time and all its tree queries. It has five wavefronts:
//     - four streaming wavefronts take the chunk's mask-free 32-key tiles (entirely inside the cached
//       prefix) round-robin; they never need the tree, a mask, or a barrier inside their loop;
//     - one tail wavefront owns the ragged end: the tiles that reach past prefix_len (the tree rows,
//       the end of the sequence). It alone validates the tree, builds the ancestor masks, applies
//       them, and (fused append) writes the new rows to the cache. Its few tiles run concurrently
//       with the stream instead of forming a serial tail, and the stream stays evenly divided.
//   Each wavefront keeps its own online-softmax state; the five are merged once, through LDS.
//
// Per 32-key tile and wavefront
//   S^T = K Q^T   v_mfma_f32_16x16x32_bf16, A = K rows read straight from global memory into the
//                 MFMA operand layout (lane r of a 16-lane group holds 8 consecutive d of key r),
//                 B = Q^T resident in registers. The transposed product leaves lane l with scores of
//                 query l%16 for keys 4*(l/16)+v of each 16-key half: exactly the B-operand layout
//                 P^T needs for the second product, so probabilities never leave registers.
//   mask          tail wavefront only: bit (key - prefix_len) of the query's 128-bit ancestor-or-self
//                 mask (built from the parent array by walking up the parent chain in LDS).
//   softmax       online, in the exp2 domain, with a lazy running maximum (refreshed, with two cross-lane
//                 exchanges and a rescale of the lane-local O^T fragment, only when a score outgrows it).
//   O^T += V^T P^T  A = V^T needs 8 keys x 1 d per lane, the transpose of how V lies in memory: V is
//                 loaded fully coalesced (four 256-byte rows per instruction), staged in a
//                 wavefront-private LDS tile and read back with ds_read_b64_tr_b16.
//
// Latency structure. A workgroup's fixed costs are what separate this kernel from a pure stream: the
// first tile's loads are issued before prefix_len is known (rows clamped to the cache capacity), in
// straight-line code so that all kernel arguments arrive in one batch; every tile's loads are issued
// one tile ahead; nothing in the loop waits on more than its own tile.
//
// With APPEND the kernel also performs the KV append of the tree tokens (Section 4.2): rows at and
// beyond prefix_len are taken from k_new / v_new and written to the cache by query group 0.
//
// Results are written as the final bf16 output when one workgroup covers the whole key range of a
// pair, else as float32 partials (m, l, O) merged by attn_combine_kernel.
#include <hip/hip_bf16.h>

#include <cstdlib>
#include <type_traits>

#include "spec_internal.h"

namespace spec {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;   // 16-byte load/store unit (plain vector: stays in registers)


constexpr float kLog2eB = 1.4426950408889634f;
constexpr int TILE = SPEC_SMALL_TILE_KEYS;          // keys per wavefront tile
constexpr int SWAVES = 4;         // streaming wavefronts
constexpr int WAVES = SWAVES + 1; // plus the tail wavefront
constexpr int TAIL = SWAVES;      // its index

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
// 16-byte load of a K/V row piece. Marked non-temporal: the K/V stream is read once per launch, and a plain
// read of the same bytes is measurably faster with the hint (the lines do not displace one another in the L2).
__device__ __forceinline__ u32x4 load_kv(const unsigned char* p) {
  return __builtin_nontemporal_load((const u32x4*)p);
}
// 16-byte store of an appended cache row. Marked non-temporal: the rows are not read again by this
// kernel, and dirty lines left in the L2 lengthen the write-back at the end of the kernel.
__device__ __forceinline__ void store_cache_row(void* p, u32x4 v) {
  // (the builtin, not inline assembly: the compiler then keeps the store's data registers untouched for the wait
  // states a 16-byte store needs after issue)
  __builtin_nontemporal_store(v, (u32x4*)p);
}

// Orders LDS accesses of the lanes of one wavefront (they execute in lockstep; this stops the
// compiler from moving LDS operations across the point).
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int D, int NT>
struct AttnTraits {
  static constexpr int KS = D / 32;            // k-steps of the QK^T product
  static constexpr int DB = D / 16;            // 16-wide d blocks of the output
  static constexpr int LPR = D * 2 / 16;       // lanes (16-byte pieces) per K/V row
  static constexpr int RPI = 64 / LPR;         // rows covered by one wave-wide 16-byte load
  static constexpr int NVL = TILE / RPI;       // V loads per lane per tile
  static constexpr int VROW = D * 2 + 16;      // LDS bytes per staged V row (+16 B pad)
  static constexpr int VTILE_BYTES = TILE * VROW;
  static constexpr int NQ = NT * 16;           // queries per workgroup
  static constexpr int MROW = D + 4;           // floats per merge row: O[D], m, l, 2 pad (16-byte aligned rows)
  static constexpr int MERGE_BYTES = WAVES * NQ * MROW * 4;
  static constexpr int STAGE_BYTES = WAVES * VTILE_BYTES;
  // One query tile: the merge area lies behind the staging tiles, so a wavefront can publish its
  // partial result as soon as it is done. Two query tiles: the merge area reuses the staging tiles.
  static constexpr bool MERGE_SEPARATE = (NT == 1);
  static constexpr int MERGE_OFF = MERGE_SEPARATE ? STAGE_BYTES : 0;
  static constexpr int LDS_BYTES = MERGE_SEPARATE ? STAGE_BYTES + MERGE_BYTES
                                                  : (MERGE_BYTES > STAGE_BYTES ? MERGE_BYTES : STAGE_BYTES);
};

// Pointers and strides one lane needs to fetch its pieces of a tile.
struct TileSrc {
  const unsigned char* kc;   // cache K of this (request, head), byte pointer at the lane's column
  const unsigned char* vc;
  const unsigned char* kn;   // new K of this (request, head) at node 0, lane's column (APPEND only)
  const unsigned char* vn;
  unsigned cache_row_bytes;
  unsigned new_row_bytes;
};

// Loads of one tile, V rows and K rows separately (V is consumed first). CLEAN: every row lies inside
// the cached prefix (no clamp, no source select). Otherwise rows are clamped to `last_row`; with
// APPEND rows >= P come from the new K/V.
template <int D, int NT, bool APPEND, bool CLEAN>
__device__ __forceinline__ void issue_v_loads(const TileSrc& s, int k0, int P, int last_row, int lane,
                                              u32x4 (&Vn)[AttnTraits<D, NT>::NVL], long shift = 0) {
  using T = AttnTraits<D, NT>;
#pragma unroll
  for (int j = 0; j < T::NVL; ++j) {
    int row = k0 + j * T::RPI + lane / T::LPR;
    const unsigned char* p;
    if (CLEAN) {
      p = s.vc + (unsigned)row * s.cache_row_bytes + shift;
    } else {
      row = min(row, last_row);
      p = (APPEND && row >= P) ? s.vn + (unsigned)(row - P) * s.new_row_bytes
                               : s.vc + (unsigned)row * s.cache_row_bytes + shift;
    }
    Vn[j] = load_kv(p);
  }
}
template <int D, int NT, bool APPEND, bool CLEAN>
__device__ __forceinline__ void issue_k_loads(const TileSrc& s, int k0, int P, int last_row, int r16,
                                              u32x4 (&Kn)[2][AttnTraits<D, NT>::KS], long shift = 0) {
  using T = AttnTraits<D, NT>;
#pragma unroll
  for (int hf = 0; hf < 2; ++hf) {
    int row = k0 + hf * 16 + r16;
    const unsigned char* p;
    if (CLEAN) {
      p = s.kc + (unsigned)row * s.cache_row_bytes + shift;
    } else {
      row = min(row, last_row);
      p = (APPEND && row >= P) ? s.kn + (unsigned)(row - P) * s.new_row_bytes
                               : s.kc + (unsigned)row * s.cache_row_bytes + shift;
    }
#pragma unroll
    for (int ks = 0; ks < T::KS; ++ks) Kn[hf][ks] = load_kv(p + ks * 64);
  }
}
template <int D, int NT, bool APPEND, bool CLEAN>
__device__ __forceinline__ void issue_tile_loads(const TileSrc& s, int k0, int P, int last_row, int r16, int lane,
                                                 u32x4 (&Kn)[2][AttnTraits<D, NT>::KS],
                                                 u32x4 (&Vn)[AttnTraits<D, NT>::NVL], long shift = 0) {
  issue_v_loads<D, NT, APPEND, CLEAN>(s, k0, P, last_row, lane, Vn, shift);
  issue_k_loads<D, NT, APPEND, CLEAN>(s, k0, P, last_row, r16, Kn, shift);
}

// PAGED: the caches are pools of blocks addressed through pg.table (see cache_row_offset). A wavefront's
// 32-key tile starts at a multiple of 32 rows and a block holds a multiple of 64, so a tile lies inside one
// block: its rows are addressed as in a contiguous cache plus one per-tile offset (page_shift below).
template <int D, int NT, bool APPEND, bool BAL, bool PAGED>
__global__ void __launch_bounds__(WAVES * 64, 2) tree_attention_bf16_kernel(
    const __hip_bfloat16* __restrict__ q, __hip_bfloat16* k_cache, __hip_bfloat16* v_cache,
    const __hip_bfloat16* __restrict__ k_new, const __hip_bfloat16* __restrict__ v_new,
    const int32_t* __restrict__ parent, const int32_t* __restrict__ depth, const int32_t* __restrict__ prefix_len,
    __hip_bfloat16* __restrict__ out, float* __restrict__ ws_o, float* __restrict__ ws_ml, int32_t* status, int B, int N,
    int H, int S_cap, int n_qgroups, int chunk_keys, int n_splits, long q_sb, long q_sn, long q_sh, long kv_sb,
    long kv_sh, long kv_ss, float scale_log2, Pages pg, Rope rope) {
  using T = AttnTraits<D, NT>;
  constexpr int KS = T::KS, DB = T::DB, LPR = T::LPR, RPI = T::RPI, NVL = T::NVL, VROW = T::VROW, NQ = T::NQ,
                MROW = T::MROW;
  constexpr int NTHREADS = WAVES * 64;

  __shared__ __attribute__((aligned(16))) unsigned char lds[T::LDS_BYTES];
  __shared__ unsigned long long s_anc[SPEC_MAX_TREE_NODES][2];
  __shared__ int s_parent[SPEC_MAX_TREE_NODES];
  __shared__ int s_depth[SPEC_MAX_TREE_NODES];
  __shared__ int s_bad_tree;

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int r16 = lane & 15, g = lane >> 4;

  // Paged cache: byte offset that, added to `row * row_bytes`, gives the place of logical row `row` of request
  // b for every row of the 32-row tile at k0 (clamped rows stay inside the tile, hence inside its block).
  // `ok`: the table entry lies inside the pool; one that does not is replaced by a block of the pool.
  auto page_shift = [&](int b, int k0, bool* ok) -> long {
    const int j = __builtin_amdgcn_readfirstlane(min(k0, S_cap - 1) >> pg.log2_tokens);
    const int e = pg.table[(long)b * pg.max_blocks + j];
    *ok = e >= 0 && e < pg.n_blocks;
    const int blk = min(max(e, 0), pg.n_blocks - 1);
    return (long)blk * kv_sb * 2 - (long)((unsigned)(j << pg.log2_tokens) * ((unsigned)kv_ss * 2u));
  };

  // One segment: keys [c0, min(c1_cap, prefix_len + N)) of request b, head h, query group qg. The result is
  // the final output (part_row < 0) or the float32 partial whose first row in the workspace is part_row.
  auto segment = [&](const int b, const int h, const int qg, const int c0, const int c1_cap, const long part_row) {
  const bool final_out = part_row < 0;
  const int q0 = qg * NQ;

  // ---- straight-line prologue (no branch before the first loads, so every kernel argument is
  // fetched in one batch): the streaming wavefronts' first tile does not depend on prefix_len (rows
  // clamped to the cache capacity keep the addresses valid; the tail wavefront's copy is discarded),
  // Q, and two tree nodes per lane for the tail wavefront.
  const int P = prefix_len[b];
  TileSrc src;
  src.cache_row_bytes = (unsigned)kv_ss * 2u;
  src.new_row_bytes = (unsigned)q_sn * 2u;
  src.kc = (const unsigned char*)(k_cache + (PAGED ? 0 : b * kv_sb) + h * kv_sh) + g * 16;
  src.vc = (const unsigned char*)(v_cache + (PAGED ? 0 : b * kv_sb) + h * kv_sh) + (lane % LPR) * 16;
  src.kn = APPEND ? (const unsigned char*)(k_new + b * q_sb + h * q_sh) + g * 16 : nullptr;
  src.vn = APPEND ? (const unsigned char*)(v_new + b * q_sb + h * q_sh) + (lane % LPR) * 16 : nullptr;

  u32x4 KA[2][KS], VA[NVL];   // tile buffer: loads land here one step ahead of use
  bool in_pool;   // entries past the request's end may hold anything: the speculative tile does not judge them
  issue_tile_loads<D, NT, false, false>(src, c0 + min(wave, SWAVES - 1) * TILE, 0, S_cap - 1, r16, lane, KA, VA,
                                        PAGED ? page_shift(b, c0 + min(wave, SWAVES - 1) * TILE, &in_pool) : 0);

  bf16x8 qB[NT][KS];   // Q^T as the B operand: lane (r16, g) holds Q[n = r16][d = ks*32 + g*8 .. +8]
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int n = q0 + nt * 16 + r16;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      // rows past N repeat the last query (their results are never written): the load is unconditional
      const u32x4 raw = *(const u32x4*)(q + b * q_sb + min(n, N - 1) * q_sn + h * q_sh + ks * 32 + g * 8);
      qB[nt][ks] = __builtin_bit_cast(bf16x8, raw);
    }
  }
  const int node0 = min(lane, N - 1), node1 = min(lane + 64, N - 1);
  const int par0 = parent[(long)b * N + node0], par1 = parent[(long)b * N + node1];
  const int dep0 = depth[(long)b * N + node0], dep1 = depth[(long)b * N + node1];

  const bool cap_ok = (P >= 0) && (P <= S_cap - N);
  const int len = P + N;
  if (!cap_ok) {
    if (final_out) {
      for (int i = t; i < NQ * D; i += NTHREADS) {
        const int n = q0 + i / D;
        if (n < N) out[b * q_sb + n * q_sn + h * q_sh + (i % D)] = __float2bfloat16(0.f);
      }
      if (h == 0 && qg == 0 && t == 0) set_status(status, b, SPEC_ST_CAPACITY);
    }
    return;
  }
  if (c0 >= len) return;
  const int c1 = min(c1_cap, len);
  const bool touches_tree = c1 > P;
  const int n_tiles = (c1 - c0 + TILE - 1) / TILE;
  const int n_clean = max(0, min(P, c1) - c0) / TILE;     // tiles entirely inside the prefix and the chunk
  const int last_row = len - 1;
  const bool is_tail = wave == TAIL;

  // Rotary embedding: a lane's pieces of a query or key row pair up within the lane (k-step ks holds dimensions
  // 32 ks + 8 g .., its partner ks + KS/2 the same dimensions + D/2), so a row is rotated in registers.
  auto rotate_row = [&](auto& lo, auto& hi, int pos, int ks) {
    const long at = (long)min(max(pos, 0), rope.len - 1) * (D / 2) + ks * 32 + g * 8;
    uint4 olo, ohi;
    rope_pair<true>(__builtin_bit_cast(uint4, lo), __builtin_bit_cast(uint4, hi), rope.cos + at, rope.sin + at, &olo, &ohi);
    lo = __builtin_bit_cast(std::remove_reference_t<decltype(lo)>, olo);
    hi = __builtin_bit_cast(std::remove_reference_t<decltype(hi)>, ohi);
  };
  if (APPEND && rope.cos != nullptr) {   // the queries, at their nodes' positions
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int pos = P + depth[(long)b * N + min(q0 + nt * 16 + r16, N - 1)];
#pragma unroll
      for (int ks = 0; ks < KS / 2; ++ks) rotate_row(qB[nt][ks], qB[nt][ks + KS / 2], pos, ks);
    }
  }

  // tiles of this wavefront: first, stride, count
  const int ti_first = is_tail ? n_clean : wave;
  const int ti_stride = is_tail ? 1 : SWAVES;
  const int ti_end = is_tail ? n_tiles : n_clean;
  if (is_tail && ti_first < ti_end)   // the tail wavefront's first tile (needs prefix_len: rows >= P have other sources)
    issue_tile_loads<D, NT, APPEND, false>(src, c0 + ti_first * TILE, P, last_row, r16, lane, KA, VA,
                                           PAGED ? page_shift(b, c0 + ti_first * TILE, &in_pool) : 0);
  if (PAGED && is_tail) {   // every block this segment reads must lie inside the pool
    for (int j = (c0 >> pg.log2_tokens) + lane; j <= ((c1 - 1) >> pg.log2_tokens); j += 64) {
      const int e = pg.table[(long)b * pg.max_blocks + j];
      if (e < 0 || e >= pg.n_blocks) set_status(status, b, SPEC_ST_BAD_BLOCK);
    }
  }

  f32x4 O[NT][DB];
  float m_run[NT], l_run[NT];
  unsigned long long anc_lo[NT], anc_hi[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    m_run[nt] = -INFINITY;
    l_run[nt] = 0.f;
    anc_lo[nt] = anc_hi[nt] = 0ull;
#pragma unroll
    for (int db = 0; db < DB; ++db) O[nt][db] = (f32x4){0.f, 0.f, 0.f, 0.f};
  }

  // ---- tail wavefront: validate the tree and build the ancestor-or-self masks (LDS, this wavefront only)
  bool bad_tree = false;
  if (is_tail) {
    if (lane == 0) s_bad_tree = 0;
    if (touches_tree) {
      if (lane < N) { s_parent[lane] = par0; s_depth[lane] = dep0; }
      if (lane + 64 < N) { s_parent[lane + 64] = par1; s_depth[lane + 64] = dep1; }
      wave_lds_sync();
      bool ok = true;
      if (lane < N) {
        ok = (lane == 0) ? (par0 == -1 && dep0 == 0) : (par0 >= 0 && par0 < lane);
        if (ok && lane > 0) ok = dep0 == s_depth[par0] + 1;
      }
      if (lane + 64 < N) {
        bool ok1 = par1 >= 0 && par1 < lane + 64;
        if (ok1) ok1 = dep1 == s_depth[par1] + 1;
        ok = ok && ok1;
      }
      bad_tree = __any(!ok);
      if (!bad_tree) {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const int node = lane + 64 * half;
          if (node < N) {
            unsigned long long lo = 0, hi = 0;
            int u = node;
            for (int step = 0; step < N && u >= 0; ++step) {
              if (u < 64) lo |= 1ull << u; else hi |= 1ull << (u - 64);
              u = s_parent[u];
            }
            s_anc[node][0] = lo;
            s_anc[node][1] = hi;
          }
        }
        wave_lds_sync();
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          const int n = q0 + nt * 16 + r16;
          if (n < N) { anc_lo[nt] = s_anc[n][0]; anc_hi[nt] = s_anc[n][1]; }
        }
      } else if (lane == 0) {
        s_bad_tree = 1;
      }
    }
  }
  unsigned char* vst = lds + wave * T::VTILE_BYTES;

  // One tile: consume the buffer filled by earlier loads, refill it for the next step, S^T, softmax, O^T.
  auto tile_step = [&](const int ti, const int ti_refill, auto masked_tag) {
    constexpr bool MASKED = decltype(masked_tag)::value;
    const int k0 = c0 + ti * TILE;
    if (MASKED) {
      // rows at and beyond the end of the chunk hold stale data: their V must not reach the product
#pragma unroll
      for (int j = 0; j < NVL; ++j)
        if (k0 + j * RPI + lane / LPR >= c1) VA[j] = (u32x4){0u, 0u, 0u, 0u};
      if (APPEND && rope.cos != nullptr) {   // new K rows are rotated before they are used and stored
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
          const int row = k0 + hf * 16 + r16;
          if (row >= P && row < c1) {
            const int pos = P + s_depth[row - P];
#pragma unroll
            for (int ks = 0; ks < KS / 2; ++ks) rotate_row(KA[hf][ks], KA[hf][ks + KS / 2], pos, ks);
          }
        }
      }
      if (APPEND && qg == 0) {   // this tile carries tree rows taken from k_new / v_new: put them in the cache
        bool dst_ok = true;      // paged cache: rows of a block outside the pool are not written
        const long dst_shift = PAGED ? page_shift(b, k0, &dst_ok) : 0;
#pragma unroll
        for (int j = 0; j < NVL; ++j) {
          const int row = k0 + j * RPI + lane / LPR;
          if (row >= P && row < c1 && dst_ok)
            store_cache_row((unsigned char*)src.vc + (unsigned)row * src.cache_row_bytes + dst_shift, VA[j]);
        }
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
          const int row = k0 + hf * 16 + r16;
          if (row >= P && row < c1 && dst_ok) {
            unsigned char* dst = (unsigned char*)src.kc + (unsigned)row * src.cache_row_bytes + dst_shift;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) store_cache_row(dst + ks * 64, KA[hf][ks]);
          }
        }
      }
    }
#pragma unroll
    for (int j = 0; j < NVL; ++j) *(u32x4*)(vst + (j * RPI + lane / LPR) * VROW + (lane % LPR) * 16) = VA[j];
    // Refill in place: V's registers are free once staged, K's once the S^T products have read them. The
    // scheduling fences keep the compiler from moving the requests above those uses: it would then need a second
    // set of registers for the rows in flight and copy it into the first on every tile, after the rows have arrived
    // and before the next request, which is time with nothing in flight.
    const int kn0 = c0 + ti_refill * TILE;
    bool refill_ok;
    const long refill_shift = (PAGED && ti_refill >= 0) ? page_shift(b, kn0, &refill_ok) : 0;
    __builtin_amdgcn_sched_barrier(0);
    if (ti_refill >= 0) issue_v_loads<D, NT, APPEND, !MASKED>(src, kn0, P, last_row, lane, VA, refill_shift);
    __builtin_amdgcn_sched_barrier(0);

    // ---- S^T = K Q^T : sc[nt][hf][v] = score of query nt*16+r16 and key k0 + hf*16 + 4g + v
    f32x4 sc[NT][2];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, KA[hf][ks]), qB[nt][ks], acc, 0, 0, 0);
        sc[nt][hf] = acc;
      }
    __builtin_amdgcn_sched_barrier(0);
    if (ti_refill >= 0) issue_k_loads<D, NT, APPEND, !MASKED>(src, kn0, P, last_row, r16, KA, refill_shift);
    __builtin_amdgcn_sched_barrier(0);

    bf16x8 pB[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      float s[8];
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int v = 0; v < 4; ++v) s[hf * 4 + v] = sc[nt][hf][v] * scale_log2;
      if (MASKED) {
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
      // Lazy running maximum. m_run (exp2 domain, identical in the four lanes of a query) only has to be close to
      // the true maximum: probabilities are exp2(score - m_run) and everything is normalised by the same sum at the
      // end. It is refreshed, with the exact cross-lane maximum and the usual rescaling of l and O, only when some
      // score of the wavefront exceeds it by more than 2^16 (or it is still -inf); otherwise a tile costs no
      // cross-lane exchange and no pass over the accumulators, which a lone wavefront on its SIMD cannot hide.
      const float mx = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
      if (__any(mx > m_run[nt] + 16.f)) {
        const float m_new = fmaxf(m_run[nt], wave_max_over_lane_groups(mx));
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
        const float p = __builtin_amdgcn_exp2f(s[i] + neg_m);
        psum += p;
        pb[i] = (__bf16)p;
      }
      pB[nt] = pb;
      l_run[nt] += psum;
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
  };

  if (is_tail) {
    if (!bad_tree)
      for (int ti = ti_first; ti < ti_end; ++ti) tile_step(ti, ti + 1 < ti_end ? ti + 1 : -1, std::true_type{});
  } else {
    for (int ti = ti_first; ti < ti_end; ti += SWAVES)
      tile_step(ti, ti + SWAVES < ti_end ? ti + SWAVES : -1, std::false_type{});
  }

  // ---- merge the five wavefronts through LDS: layout [wave][n][MROW] floats (O row, m, l)
  if (!T::MERGE_SEPARATE) __syncthreads();   // the merge area overlays the staging tiles still being read
  float* mg = (float*)(lds + T::MERGE_OFF);
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
  if (s_bad_tree != 0) {   // malformed tree: defined result = zeros (written here when this workgroup owns the output)
    if (final_out) {
      for (int i = t; i < NQ * D; i += NTHREADS) {
        const int n = q0 + i / D;
        if (n < N) out[b * q_sb + n * q_sn + h * q_sh + (i % D)] = __float2bfloat16(0.f);
      }
      if (h == 0 && qg == 0 && t == 0) set_status(status, b, SPEC_ST_BAD_TREE);
    }
    return;
  }
  constexpr int CG = D / 4;
  for (int idx = t; idx < NQ * CG; idx += NTHREADS) {
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
    if (final_out) {
      const float inv = 1.f / l;
      union { uint2 u; __hip_bfloat16 h4[4]; } pk;
#pragma unroll
      for (int i = 0; i < 4; ++i) pk.h4[i] = __float2bfloat16(o[i] * inv);
      *(uint2*)(out + b * q_sb + n * q_sn + h * q_sh + cg * 4) = pk.u;
    } else {
      const long base = part_row + n;
      *(f32x4*)(ws_o + base * D + cg * 4) = o;
      if (cg == 0) {
        ws_ml[base * 2 + 0] = M;
        ws_ml[base * 2 + 1] = l;
      }
    }
  }
  };   // segment

  if constexpr (!BAL) {
    // grid = (n_splits, H * n_qgroups, B): one fixed-size chunk of one (request, head, query group)
    const int split = blockIdx.x;
    const int h = blockIdx.y / n_qgroups, qg = blockIdx.y % n_qgroups;
    const int b = blockIdx.z;
    segment(b, h, qg, split * chunk_keys, split * chunk_keys + chunk_keys,
            n_splits == 1 ? -1l : (((long)b * H + h) * n_splits + split) * N);
  } else {
    // Balanced stream: the 32-key tiles of all (request, head) pairs, in (request, head, key) order,
    // are dealt to the gridDim.x workgroups in equal contiguous shares, whatever the requests'
    // lengths; a share that crosses a pair boundary becomes several segments. n_splits is the number
    // of partial slots per pair: the workgroups overlapping a pair fill slots 0, 1, ... in order.
    const BalancedShare bs = balanced_share(prefix_len, B, N, H, S_cap, TILE, (int)gridDim.x);
    long pos = (long)blockIdx.x * bs.share;
    const long end = min(bs.total, pos + bs.share);
    int b = 0;
    long req_start = 0;
    int tb = request_tiles(prefix_len[0], N, S_cap, TILE);
    while (pos < end) {
      while (pos >= req_start + (long)H * tb) {   // pos < total: a request with tiles left lies ahead
        req_start += (long)H * tb;
        ++b;
        tb = request_tiles(prefix_len[b], N, S_cap, TILE);
      }
      const long in_req = pos - req_start;
      const int h = (int)(in_req / tb), tile0 = (int)(in_req % tb);
      const int n_take = (int)min((long)(tb - tile0), end - pos);
      const int slot = (int)blockIdx.x - (int)((req_start + (long)h * tb) / bs.share);
      segment(b, h, 0, tile0 * TILE, (tile0 + n_take) * TILE, (((long)b * H + h) * n_splits + slot) * N);
      pos += n_take;
      __syncthreads();   // LDS (staging tiles, merge area, flags) is reused by the next segment
    }
  }
}

hipError_t launch_tree_attention_bf16(const spec_attn_desc_t& d, const AttnPlan& plan, const Pages& pg, const void* q, void* k_cache,
                                      void* v_cache, const void* k_new, const void* v_new, const int32_t* parent,
                                      const int32_t* depth, const int32_t* prefix_len, void* out, void* ws,
                                      int32_t* status, hipStream_t s, const Rope& rope) {
  // This kernel: one 16-query tile per K/V head, k_new / v_new laid out like q. Larger trees, grouped-query
  // heads and separately laid out k_new go to the wide kernel (the plan decides).
  if (plan.wide)
    return launch_tree_attention_bf16_wide(d, plan, pg, q, k_cache, v_cache, k_new, v_new, parent, depth, prefix_len, out, ws,
                                           status, s, rope);
  const float scale = (d.softmax_scale != 0.f ? d.softmax_scale : 1.0f / sqrtf((float)d.D)) * kLog2eB;
  float* ws_o = ws ? (float*)((char*)ws + plan.ws_o_off) : nullptr;
  float* ws_ml = ws ? (float*)((char*)ws + plan.ws_ml_off) : nullptr;
  const int n_qgroups = 1;   // one 16-query tile covers the trees this kernel serves
  const bool append = k_new != nullptr;
  const bool bal = plan.balanced_wgs > 0;
  const dim3 grid = bal ? dim3(plan.balanced_wgs, 1, 1) : dim3(plan.n_splits, d.H * n_qgroups, d.B);
#define SPEC_LAUNCH(DD, NTT, APP, BAL, PGD)                                                                      \
  hipLaunchKernelGGL((tree_attention_bf16_kernel<DD, NTT, APP, BAL, PGD>), grid, dim3(WAVES * 64), 0, s,         \
                     (const __hip_bfloat16*)q, (__hip_bfloat16*)k_cache, (__hip_bfloat16*)v_cache,               \
                     (const __hip_bfloat16*)k_new, (const __hip_bfloat16*)v_new, parent, depth, prefix_len,      \
                     (__hip_bfloat16*)out, ws_o, ws_ml, status, d.B, d.N, d.H, d.S_cap, n_qgroups,               \
                     plan.chunk_keys, plan.n_splits, (long)d.q_stride_b, (long)d.q_stride_n, (long)d.q_stride_h, \
                     (long)d.kv_stride_b, (long)d.kv_stride_h, (long)d.kv_stride_s, scale, pg, rope)
#define SPEC_DIMS(APP, BAL, PGD)                      \
  if (d.D == 128) SPEC_LAUNCH(128, 1, APP, BAL, PGD); \
  else SPEC_LAUNCH(64, 1, APP, BAL, PGD)
#define SPEC_DISPATCH(APP, BAL)                             \
  if (pg.table != nullptr) { SPEC_DIMS(APP, BAL, true); }   \
  else { SPEC_DIMS(APP, BAL, false); }
  if (append && bal) { SPEC_DISPATCH(true, true); }
  else if (append) { SPEC_DISPATCH(true, false); }
  else if (bal) { SPEC_DISPATCH(false, true); }
  else { SPEC_DISPATCH(false, false); }
#undef SPEC_DISPATCH
#undef SPEC_DIMS
#undef SPEC_LAUNCH
  return hipGetLastError();
}

}  // namespace spec
