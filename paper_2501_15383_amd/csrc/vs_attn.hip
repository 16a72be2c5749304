// Block-sparse / dense causal online-softmax attention for gfx950 (CDNA4), bf16 MFMA with
// fp32 accumulation.  One kernel serves both the vertical-slash sparse path and the dense
// fallback: it walks a per-head bitmap of block diagonals (dense = all ones) and then the
// gathered vertical columns.
//
// What is computed (section 5.2, MInference paragraph: attention only on the selected
// critical tokens; softmax_lse as in the "Sparsity refinement" paragraph): row i at position
// p attends key j <= p iff j is a selected column or floor(p/64) - floor(j/64) is a computed
// block diagonal.
//
// Layout of the work
//  * workgroup = NQB query blocks of 64 rows (2 waves each, a wave owns 32 rows) of one head.
//    Key block n = m0 - c is staged once in LDS and used by query block t iff diagonal
//    c + t is computed, so adjacent diagonals share their K/V fetch.
//  * S^T = K Q^T with v_mfma_f32_32x32x16_bf16: the accumulator then holds, per lane, one
//    query and 16 keys, so the row maximum / sum need one cross-lane step, and P^T is already
//    the B operand of the second MFMA (O^T = V^T P^T) -- P never goes through LDS.
//  * V stays row-major in LDS and is read with the transposing LDS load (ds_read_b64_tr_b16)
//    as the A operand of the PV contraction, which runs over keys.
//  * K/V tiles go from global memory straight into LDS (global_load_lds_dwordx4, no staging
//    registers), double-buffered: the copy of tile t+1 runs under the MFMA work of tile t,
//    one barrier per tile.  Rows are unpadded; 16-byte chunks are XOR-swizzled instead.
//  * the exponentials use one fixed reference per row (the maximum of the row's first tile;
//    an exact path with the true maximum is kept for masked tiles, first tiles and an
//    overflow guard), so the steady state has no running-maximum update.  The V^T P^T product
//    of a tile runs one step behind its K Q^T product, in one hand-interleaved instruction
//    stream with the exponentials, operands three LDS reads ahead.
//  * the tile walk reads a per-head list of (key block, query-block mask) entries through
//    a 64-entry lane cache and lives entirely in scalar registers.
//  * persistent launch: two workgroups per compute unit in eight groups (one per XCD); a group
//    works on consecutive query tiles of one head per round and keeps its members within a
//    few sync segments of keys, so that K/V blocks are shared through the L2.  Which group
//    takes which round is decided on the device from the lengths of the block lists.
//  * template parameters: DCA (three rotations of the queries, chosen per (query, key)
//    pattern; section 5.1) and SPLIT (short chunks: the key walk cut into ranges, partial
//    results folded by k_attn_combine).  The plain kernel is its own instantiation.
#include <atomic>
#include <mutex>

#include "vs_common.h"

namespace vs {

// a 64-bit value that is the same in every lane, moved into scalar registers
template <typename T>
__device__ __forceinline__ T uniform64(T x) {
  static_assert(sizeof(T) == 8, "uniform64 takes pointers and 64-bit integers");
  const uint64_t b = (uint64_t)x;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b), hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
  return (T)(((uint64_t)hi << 32) | lo);
}

struct AttnArgs {
  const __bf16* q;
  // Dual Chunk Attention (template parameter DCA): the chunk's queries rotated for the
  // successive-chunk and the inter-chunk pattern (q is the intra-chunk one; same strides),
  // chunk length and local window in 64-key blocks
  const __bf16* q_succ;
  const __bf16* q_inter;
  int32_t dca_cblk, dca_wblk;
  // Key split (template parameter SPLIT) for chunks with few query tiles: the walk of a (tile,
  // head) is cut into n_split ranges of key-block distances, one workgroup each; every
  // workgroup writes its unnormalised result (relative to its own reference) and k_attn_combine
  // folds them.  part_o [n_split][Hq][q_len][D], part_ml [n_split][Hq][q_len][2] (reference, sum)
  int32_t n_split;
  float* part_o;
  float* part_ml;
  const __bf16* k;
  const __bf16* v;
  __bf16* out;
  float* lse;
  int64_t q_stride_tok, q_stride_head, k_stride_tok, k_stride_head;
  int64_t v_stride_tok, v_stride_head, o_stride_tok, o_stride_head;
  const uint32_t* bm_a;  // block-diagonal bitmap per head
  const uint32_t* ent;   // key-block entry list per head (see BlockList)
  int64_t bm_stride;     // words per head, 0 = one bitmap shared by all heads (dense)
  int32_t bm_words;      // words of one bitmap row; its last word holds the head's segment shift
  int64_t ent_stride;    // entries per head, 0 = one list shared by all heads (dense)
  int64_t ent_len;       // entries of one list (sentinel padding included)
  const int32_t* v_idx;  // null: no vertical phase
  const int32_t* v_cnt;
  int32_t v_budget;
  int32_t n_q_heads, n_kv_heads, group;
  int32_t n_qtiles;
  // q_start is rounded down to a multiple of 64 and q_len grown by the same row_pad rows, so that
  // query blocks stay aligned to absolute positions; the first row_pad rows of the launch are
  // padding (nothing is loaded or stored for them).  q_rows is the caller's q_len.
  int64_t q_len, q_start;
  int32_t row_pad;
  int64_t q_rows;
  int64_t n_k;  // keys visible to the chunk
  // Single-token dense decode with grouped queries: the G query heads of a KV group are the
  // rows of one tile (so K and V are read once per group, not once per head); all rows then
  // stand at the same position, pos_in_block keys into the diagonal block.
  int32_t same_pos, pos_in_block;
  float scale_log2;  // softmax_scale * log2(e)
  // persistent launch: n_wg workgroups, workgroup b is member b / 8 of group b % 8 (the groups
  // follow the round-robin of workgroups over the 8 XCDs); in round r group g works on
  // group-round k = 8 r + g, one query tile per member.  The top n_full * members tiles of
  // every head go first, as (chunk of `members` consecutive tiles, head) rounds, latest chunks
  // first; the n_rem tiles per head that are left are packed, head after head, into the rounds
  // that follow, so that only the very last round can have idle members.
  int32_t n_wg, members, n_full, n_rem;
  // pace keeping: arrive[g][s] counts the members of group g that are done with key blocks
  // [s * sync_blocks, (s + 1) * sync_blocks) over all rounds so far; sync_blocks = 1 << sync_shift
  int32_t sync_blocks, sync_shift, n_sync;
  uint32_t* arrive;
  // sched[g][r]: the group-round that group g works on in its r-th round, -1 = none left
  // (written by k_attn_schedule from the lengths of the heads' block lists; n_gr entries per group)
  const int32_t* sched;
  int32_t n_gr;
  // Several requests in one launch (template parameter BATCH, always with SPLIT): a unit is
  // (request, head, query tile, key range); the request's pointers, position and length come
  // from req[r] and replace the fields above (batch_view).  n_qtiles is then the tile count of
  // the longest request, bm_a / ent hold one list per (request, head), part_o / part_ml one
  // region of n_split x Hq x rows_cap rows per request.  Requests beyond max_q_len / max_n_k
  // (the bounds the workspace was sized for) are skipped.
  const vs_request* req;
  int32_t n_req, rows_cap, head_dim;
  int64_t max_q_len, max_n_k;
  // Sparse attention of ONE token with grouped queries (BATCH only; set per request by batch_view):
  // the G <= 16 heads of a KV group are the rows of one tile, as in the dense case, so K and V are
  // read once per group.  The tile walks the UNION of the heads' block lists (ent_u, one list per
  // (request, KV head), entries ((diagonal + 1) << 4) | 1); ent_hm holds, per entry, the heads
  // whose own list has that diagonal (bit j = head j of the group): a row takes part in a tile
  // iff its bit is set.  The gathered columns then follow head by head (every head has its own
  // column set; only that head's row is live in its tiles).
  const uint32_t* ent_u;
  const uint32_t* ent_hm;
  uint32_t* bm_u;          // union bitmaps [n_req][Hkv][words] (scratch of the list builder)
  const uint32_t* hm;      // this request's masks (set by batch_view)
  int32_t packed_sparse, group_rows;
};
constexpr int kPackedSparseMaxGroup = 16;

// The arguments as request r of a batch sees them.  False: the request is outside the stated
// bounds or has a null pointer, and is skipped (nothing of it is read or written).
__device__ __forceinline__ bool batch_view(const AttnArgs& a0, int r, AttnArgs& a) {
  vs_request rq = a0.req[r];   // the same address in every lane: the fields are uniform
  rq.q = uniform64(rq.q); rq.k = uniform64(rq.k); rq.v = uniform64(rq.v); rq.out = uniform64(rq.out);
  rq.lse = uniform64(rq.lse); rq.v_idx = uniform64(rq.v_idx); rq.v_cnt = uniform64(rq.v_cnt);
  rq.s_idx = uniform64(rq.s_idx); rq.s_cnt = uniform64(rq.s_cnt);
  rq.q_start = uniform64(rq.q_start); rq.q_len = uniform64(rq.q_len);
  if (!rq.q || !rq.k || !rq.v || !rq.out) return false;
  if (rq.q_len < 1 || rq.q_len > a0.max_q_len || rq.q_start < 0 || rq.q_start + rq.q_len > a0.max_n_k) return false;
  const bool dense = rq.s_idx == nullptr;
  if (!dense && (!rq.v_idx || !rq.v_cnt || !rq.s_cnt)) return false;
  a.q = (const __bf16*)rq.q; a.k = (const __bf16*)rq.k; a.v = (const __bf16*)rq.v;
  a.out = (__bf16*)rq.out; a.lse = rq.lse;
  a.v_idx = dense ? nullptr : rq.v_idx;
  a.v_cnt = dense ? nullptr : rq.v_cnt;
  a.row_pad = (int32_t)(rq.q_start % kBlock);
  a.q_start = rq.q_start - a.row_pad;
  a.q_len = rq.q_len + a.row_pad;
  a.q_rows = rq.q_len;
  a.n_k = rq.q_start + rq.q_len;
  a.bm_a = a0.bm_a + (int64_t)r * a0.n_q_heads * a0.bm_stride;
  a.ent = a0.ent + (int64_t)r * a0.n_q_heads * a0.ent_stride;
  const int64_t slot = (int64_t)r * a0.n_split * a0.n_q_heads * a0.rows_cap;
  a.part_o = a0.part_o + slot * a0.head_dim;
  a.part_ml = a0.part_ml + slot * 2;
  a.packed_sparse = 0;
  a.group_rows = a0.group;
  const bool pack_sparse = !dense && a0.ent_u && a0.group <= kPackedSparseMaxGroup;
  if (rq.q_len == 1 && a0.group > 1 && (dense || pack_sparse)) {
    // attention of one token: the G heads of a KV group are the rows of one tile
    if (!dense) {
      a.packed_sparse = 1;
      a.v_idx = rq.v_idx; a.v_cnt = rq.v_cnt;   // indexed by the heads of the unit's group
      a.ent = a0.ent_u + (int64_t)r * a0.n_kv_heads * a0.ent_stride;
      a.hm = a0.ent_hm + (int64_t)r * a0.n_kv_heads * a0.ent_stride;
    }
    a.q_stride_tok = a0.q_stride_head; a.q_stride_head = (int64_t)a0.group * a0.q_stride_head;
    a.o_stride_tok = a0.o_stride_head; a.o_stride_head = (int64_t)a0.group * a0.o_stride_head;
    a.n_q_heads = a0.n_kv_heads; a.group = 1;
    a.same_pos = 1; a.pos_in_block = a.row_pad;
    a.row_pad = 0; a.q_len = a0.group; a.q_rows = a0.group;
    a.n_split = a0.n_split * a0.group;   // see the unit decode of k_attention
  }
  a.n_qtiles = (int32_t)((a.q_len + 64 * kAttnQBlocks - 1) / (64 * kAttnQBlocks));
  return true;
}

__device__ __forceinline__ bool bm_test(const uint32_t* bm, int i) {
  return (bm[i >> 5] >> (i & 31)) & 1u;
}

// LDS bytes of one workgroup: K and V tiles (unpadded, chunk-swizzled), double-buffered, the
// gathered column indices of a vertical tile, and per-wave mask thresholds.
template <int D>
constexpr int attn_lds_bytes() { return 4 * 64 * D * 2 + 2 * 64 * 4 + 4 * kAttnQBlocks * 64; }

// Direct global -> LDS copy, 16 bytes per lane: lane L's bytes land at lds_addr + 16 L
// (lds_addr is wave-uniform and goes through M0).  Completion is tracked by vmcnt.
// N such copies from one scalar base with per-copy lane offsets; the LDS destinations are
// lds_addr, lds_addr + step, ...  (M0 is read when a copy issues, so it can move on at once;
// a write to M0 needs one wait state before the copy that uses it.)
// (lds_addr, sbase and step are the same in every lane; where the compiler cannot see that, the
// values are moved into scalar registers here: the instructions take them from there)
__device__ __forceinline__ void dma16x4(uint32_t lds_addr, const void* sbase, uint32_t o0, uint32_t o1,
                                        uint32_t o2, uint32_t o3, uint32_t step) {
  lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);
  step = __builtin_amdgcn_readfirstlane(step);
  sbase = uniform64(sbase);
  asm volatile(
      "s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %5\n\t"
      "s_add_u32 m0, m0, %6\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %5\n\t"
      "s_add_u32 m0, m0, %6\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %3, %5\n\t"
      "s_add_u32 m0, m0, %6\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %4, %5"
      :: "s"(lds_addr), "v"(o0), "v"(o1), "v"(o2), "v"(o3), "s"(sbase), "s"(step) : "memory", "scc");
}
__device__ __forceinline__ void dma16x2(uint32_t lds_addr, const void* sbase, uint32_t o0, uint32_t o1,
                                        uint32_t step) {
  lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);
  step = __builtin_amdgcn_readfirstlane(step);
  sbase = uniform64(sbase);
  asm volatile(
      "s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %3\n\t"
      "s_add_u32 m0, m0, %4\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3"
      :: "s"(lds_addr), "v"(o0), "v"(o1), "s"(sbase), "s"(step) : "memory", "scc");
}
__device__ __forceinline__ void dma16_lane_ptr(uint32_t lds_addr, const void* ptr) {
  lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
               :: "s"(lds_addr), "v"(ptr) : "memory");
}
__device__ __forceinline__ uint32_t lds_address(const void* p) {
  return (uint32_t)(size_t)(const __attribute__((address_space(3))) char*)p;
}

// Timing diagnostics (never defined in the library that ships; results are WRONG with any of them,
// all accesses stay in bounds and every barrier that remains is reached by all waves):
//   VS_X_NOVLDS     the V^T fragments of the fused step come from a register instead of LDS
//                   (half of the LDS operand reads gone, same MFMA count)
//   VS_X_NOCOPY     the global -> LDS copies of whole key blocks are skipped after the first two
//   VS_X_SAMEBLK    every whole-block copy reads key block 0 or 1 of the head (always in the L2)
//   VS_X_NOBARRIER  no workgroup barrier at the end of a step
//   VS_X_TIGHT      dense list only: the steady-state steps run in a loop with no list reads, no
//                   tile classification and no bookkeeping beyond the pace keeping (right results)
// They split the time of a step into what the arithmetic stream, the operand reads, the copies
// and the barrier cost.
template <int D, int NQB, bool DCA, bool SPLIT, bool BATCH = false>
__global__ __launch_bounds__(128 * NQB, 2) void k_attention(const AttnArgs a0) {
  static_assert(!BATCH || (SPLIT && !DCA), "several requests per launch ride on the key-split kernel");
  constexpr int DCH = D / 8;           // 16-byte chunks per row
  constexpr int DSTEPS = D / 16;       // MFMA k-steps of QK^T
  constexpr int DB = D / 32;           // 32-row blocks of O^T
  constexpr int TILE = 64 * D;         // elements of one K or V tile in LDS (rows unpadded)
  constexpr int RPG = 512 / D;         // rows in one 1 KiB group (= one wave-wide copy)
  constexpr int NG = 64 / RPG;         // groups per tile
  constexpr int GPW = NG / (2 * NQB);  // groups per wave
  constexpr int R = 128 / D;           // rows per 256 bytes of LDS
  static_assert(NG % (2 * NQB) == 0, "tile must divide over the waves");
  // LDS layout.  Row r of a tile starts at r * D elements; its 16-byte chunk c is stored in
  // slot c ^ f(r) for K and c ^ g(r) for V, which spreads the MFMA operand reads over all
  // banks without padding (the copy engine writes 1 KiB contiguously per instruction):
  //   f(r) = (r / R) % DCH                      16 consecutive keys of one d-chunk (K reads)
  //   g(r) = (((r / R) & 3) << 2) & (DCH - 1)   4 keys x 4 d-chunks (transposing V reads)

  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  __bf16* const Ks = (__bf16*)smem_raw;               // [2][TILE]
  __bf16* const Vs = Ks + 2 * TILE;                   // [2][TILE]
  int32_t* const vidx_s = (int32_t*)(Vs + 2 * TILE);  // [2][64]
  uint8_t* const need_s = (uint8_t*)(vidx_s + 2 * 64);  // [waves][64], private to each wave
  static_assert(2 * (2 * NQB) * 64 <= 4 * kAttnQBlocks * 64, "need_s and dcak_s share the bytes after vidx_s");
  uint8_t* const dcak_s = need_s + 2 * NQB * 64;        // [waves][64], DCA pattern code of a tile's keys
  const uint32_t ks_addr = lds_address(Ks), vs_addr = lds_address(Vs);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave index, known uniform
  const int t = wv >> 1;                          // query block of this wave inside the tile
  const int il = ((wv & 1) << 5) + (lane & 31);   // row inside the query block
  const int hh = lane >> 5;

  // ---- persistent workgroup: one (query tile, head) per round ------------------------------
  // The `members` workgroups of a group take consecutive query tiles of ONE head, so they walk
  // the same entry list, shifted by two key blocks per tile, at the same pace; the arrive
  // counters below keep the group inside a window of a few sync segments, small enough for
  // the XCD's L2, so that a K/V block is fetched from memory once per group and round.
  // Waiting is bounded and only shapes the timing: results never depend on it.
  const int grp = blockIdx.x & 7, member = blockIdx.x >> 3;
  const int n_full_gr = a0.n_full * a0.n_q_heads;   // full rounds: latest chunks first, heads inside
  const int n_gr = SPLIT ? (a0.n_qtiles * a0.n_split * a0.n_q_heads * (BATCH ? a0.n_req : 1) + a0.members - 1) / a0.members
                         : n_full_gr + (a0.n_rem * a0.n_q_heads + a0.members - 1) / a0.members;
  uint32_t* const arr = a0.arrive + (int64_t)grp * a0.n_sync;
  const int s_glob_top = (int)((a0.n_k - 1) / 64) >> a0.sync_shift;  // highest sync segment of the chunk
  for (int rnd = 0; SPLIT ? rnd * 8 + grp < n_gr : rnd < n_gr; ++rnd) {
  int gr = rnd * 8 + grp;
  if constexpr (!SPLIT) {
    gr = __builtin_amdgcn_readfirstlane(a0.sched[grp * n_gr + rnd]);
    if (gr < 0) break;
  }
  // this round's view of the arguments: the kernel's own, or (BATCH) those of the unit's request
  AttnArgs a_req;
  if constexpr (BATCH) a_req = a0;
  const AttnArgs& a = BATCH ? a_req : a0;
  int h, qt, sp = 0;
  if constexpr (BATCH) {
    const int per_head = a0.n_qtiles * a0.n_split, per_req = per_head * a0.n_q_heads;
    const int u = gr * a0.members + member;
    const int r = u / per_req;
    if (r >= a0.n_req) continue;
    int v = u - r * per_req;
    h = v / per_head;
    v -= h * per_head;
    qt = v / a0.n_split;
    sp = v - qt * a0.n_split;
    if (!batch_view(a0, r, a_req)) continue;
    if (a.same_pos) {
      // heads packed into rows: the unit slots of the G heads of a group become G times as many key
      // ranges of the group's one tile
      sp += (h % a0.group) * a0.n_split;
      h /= a0.group;
    }
    if (h >= a.n_q_heads) continue;
  } else
  if constexpr (SPLIT) {
    // unit u = ((head, tile), split), no pace keeping (the members walk different key ranges)
    const int per_head = a.n_qtiles * a.n_split;
    const int u = gr * a.members + member;
    h = u / per_head;
    const int v = u - h * per_head;
    qt = h < a.n_q_heads ? v / a.n_split : a.n_qtiles;
    sp = v % a.n_split;
    if (h >= a.n_q_heads) h = 0;
  } else if (gr < n_full_gr) {
    h = gr % a.n_q_heads;
    qt = a.n_rem + (a.n_full - 1 - gr / a.n_q_heads) * a.members + (a.members - 1 - member);
  } else {  // packed rounds: unit u = (head, tile below n_rem), tiles descending inside a head
    const int u = (gr - n_full_gr) * a.members + member;
    h = u / a.n_rem;
    qt = h < a.n_q_heads ? a.n_rem - 1 - u % a.n_rem : a.n_qtiles;
    if (h >= a.n_q_heads) h = 0;
  }
  const int64_t n_k = a.n_k;
  const int g = h / a.group;
  const uint32_t expected = (uint32_t)(rnd + 1) * (uint32_t)a.members;
  // marks key segments seg_done - 1, ..., s_new done for this member, then holds the workgroup
  // back (wave 0 polls, the others meet it at the step barrier) until the whole group is done
  // with segment s_new + 2
  int seg_done = s_glob_top + 1;
  bool patient = true;  // a wait that ran out (group not co-resident?) ends the waiting for this tile
  auto enter_segment = [&](int s_new, bool wait) {
    if constexpr (SPLIT) return;
    if (s_new >= seg_done - 1) return;  // still in the segment entered last
    if (wv == 0) {
      for (int sg = seg_done - 1 - lane; sg > s_new; sg -= 64) atomicAdd(&arr[sg], 1u);
      if (wait && patient && s_new + 2 <= s_glob_top) {
        int spins = 0;
        while (__hip_atomic_load(&arr[s_new + 2], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < expected &&
               spins < 2048) {
          __builtin_amdgcn_s_sleep(16);
          ++spins;
        }
        patient = spins < 2048;
      }
    }
    seg_done = s_new + 1;
  };
  if (qt >= a.n_qtiles) {  // no tile for this member in this round
    enter_segment(-1, false);
    continue;
  }
  const int64_t row0 = (int64_t)qt * (64 * NQB);
  const int64_t row = row0 + 64 * t + il;
  const int m0 = (int)(a.q_start / 64) + qt * NQB;  // absolute index of query block t = 0
  const bool wave_valid = row0 + 64 * t + ((wv & 1) << 5) < a.q_len;
  const int64_t rows_in_tile = (a.q_len - row0) < 64 * NQB ? (a.q_len - row0) : 64 * NQB;
  const int64_t last_pos = a.same_pos ? n_k - 1 : a.q_start + row0 + rows_in_tile - 1;

  // heads packed into the rows of a sparse single-token tile: the unit's "head" is the KV head, the
  // block bitmaps and column sets are those of head ps_h0 + j of the group (j = row of the tile)
  const bool ps = BATCH && a.packed_sparse;
  const int ps_h0 = h * a.group_rows;
  const int ps_vt = (a.v_budget + 63) >> 6;   // vertical tiles per head at most; tile index = j * ps_vt + vt
  const uint32_t* bmA = a.bm_a + (int64_t)(ps ? ps_h0 : h) * a.bm_stride;
  const int seg_shift = __builtin_amdgcn_readfirstlane((int)bmA[a.bm_words - 1]);  // sparser list, longer sync segments
  const uint32_t* ent_h = a.ent + (int64_t)h * a.ent_stride;
  const uint32_t* hm_h = ps ? a.hm + (int64_t)h * a.ent_stride : nullptr;
  const int32_t* vidx_h = a.v_idx ? a.v_idx + (int64_t)(ps ? ps_h0 : h) * a.v_budget : nullptr;
  const int vcnt = a.v_idx ? __builtin_amdgcn_readfirstlane(a.v_cnt[ps ? ps_h0 : h]) : 0;
  const int n_vt = (vcnt + 63) >> 6;
  bool row_live = true;   // packed sparse: this lane's row (head) takes part in the current tile
  const int cc_last = m0 + NQB - 1;  // entry cc stands for key block m0 + (NQB - 1) - cc >= 0

  const __bf16* kbase = a.k + (int64_t)g * a.k_stride_head;
  const __bf16* vbase = a.v + (int64_t)g * a.v_stride_head;

  // ---- Q^T operand: lane (i = lane%32, hh) holds Q[i][16 st + 8 hh .. +7] ----------------
  // With DCA the operand is one of three rotations of the same rows; q_var says which one the
  // registers hold (the walk goes from the query block's own keys backwards, so it changes
  // at most a few times per tile).
  bf16x8 qreg[DSTEPS];
  int q_var = 0;
  auto load_q = [&](int var) {
    const __bf16* qb = a.q;
    if constexpr (DCA) {
      if (var == 1) qb = a.q_succ;
      if (var == 2) qb = a.q_inter;
    }
    int64_t rc = row - a.row_pad;  // the caller's row (clamped: padding and tail rows load a valid one)
    rc = rc < 0 ? 0 : (rc < a.q_rows ? rc : a.q_rows - 1);
    const __bf16* qp = qb + rc * a.q_stride_tok + (int64_t)h * a.q_stride_head + 8 * hh;
#pragma unroll
    for (int st = 0; st < DSTEPS; ++st) qreg[st] = *(const bf16x8*)(qp + 16 * st);
    q_var = var;
  };
  load_q(0);

  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int x = 0; x < 16; ++x) oacc[db][x] = 0.f;
  // ---- softmax state of this wave's rows, and the tile whose PV contraction is still owed ----
  // The V^T P^T product of a tile runs one step after its K Q^T product (see the main loop), so
  // between two steps a wave carries the tile's probabilities as four bf16 MFMA operands and
  // their row sum.
  // Probabilities are 2^(score - m_o) with ONE reference m_o per row for accumulators, row sum
  // and pending tile alike.  Any reference gives the same softmax; it only has to keep the
  // numbers in range.  m_o is the true maximum of the row's first tile and is raised (with a
  // rescale, on the exact path only) when a score outruns it by more than 2^64, so the
  // steady-state path never touches the accumulators except through the MFMAs.
  float l_run = 0.f;
  float m_o = -INFINITY;  // scaled reference (log2 domain)
  bool have_max = false;  // every row of this wave has a finite m_o (uniform)
  bool pend = false;      // uniform
  bf16x8 pp[4];           // P^T operands of the pending tile: keys 16 u .. 16 u + 15 (in MFMA k order)
  float pend_ps = 0.f;
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int x = 0; x < 8; ++x) pp[u][x] = (__bf16)0.f;

  // ---- tile iterator (uniform over the workgroup, kept in scalar registers) -----------------
  // kind 0: slash tile, idx = cc, mask = query blocks that use it; kind 1: vertical tile,
  // idx = vt; kind 2: end.  Entries are fetched 64 at a time (one per lane), one batch ahead.
  // With a key split this workgroup walks the entries with cc in [cc_lo, cc_end] and every
  // n_split-th vertical tile; the first entry is found by bisection (the list ascends in cc and
  // ends in sentinels).
  int cc_end = cc_last, ei0 = 0;
  const int vstep = SPLIT ? a.n_split : 1;
  if constexpr (SPLIT) {
    const int per = (cc_last + a.n_split) / a.n_split;  // ceil((cc_last + 1) / n_split)
    const int cc_lo = sp * per;
    cc_end = cc_lo + per - 1 < cc_last ? cc_lo + per - 1 : cc_last;
    int lo = 0, hi = (int)a.ent_len - 1;  // the last entry is a sentinel: an answer always exists
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      const int cm = (int)(__builtin_amdgcn_readfirstlane(ent_h[mid]) >> 4);
      if (cm >= cc_lo) hi = mid; else lo = mid + 1;
    }
    ei0 = lo;
  }
  uint32_t ecache = ent_h[(ei0 & ~63) + lane], ecache_nx = ent_h[(ei0 & ~63) + 64 + lane];
  uint32_t hcache = 0, hcache_nx = 0;   // packed sparse: the head masks of the same entries
  if constexpr (BATCH) {
    if (ps) { hcache = hm_h[(ei0 & ~63) + lane]; hcache_nx = hm_h[(ei0 & ~63) + 64 + lane]; }
  }
  int ei = ei0 - 1;
  // (packed sparse) column set, count and block bitmap of head j of the group
  auto ps_head = [&](int j, const int32_t*& vi, int& vc, const uint32_t*& bm) {
    vi = a.v_idx + (int64_t)(ps_h0 + j) * a.v_budget;
    vc = __builtin_amdgcn_readfirstlane(a.v_cnt[ps_h0 + j]);
    bm = a.bm_a + (int64_t)(ps_h0 + j) * a.bm_stride;
  };
  auto advance = [&](int& kind, int& idx, int& mask) {
    int k2 = kind, i2 = idx, m2 = 0;
    if (k2 == 0) {
      ++ei;
      if (__builtin_expect((ei & 63) == 0 && ei > ei0, 0)) {
        ecache = ecache_nx;
        ecache_nx = ent_h[(ei & ~63) + 64 + lane];
        if constexpr (BATCH) {
          if (ps) { hcache = hcache_nx; hcache_nx = hm_h[(ei & ~63) + 64 + lane]; }
        }
      }
      const uint32_t e = __builtin_amdgcn_readlane(ecache, ei & 63);
      const int cc = (int)(e >> 4);
      if (cc <= cc_end) {
        i2 = cc; m2 = (int)(e & 15u);
        if constexpr (BATCH) {
          if (ps) m2 |= (int)((__builtin_amdgcn_readlane(hcache, ei & 63) & 0xFFFFu) << 4);
        }
        enter_segment((cc_last - cc) >> (a.sync_shift + seg_shift), true);
      } else {
        k2 = 1; i2 = sp - vstep;
        enter_segment(-1, false);  // the slash walk is over
      }
    }
    if (k2 == 1) {
      if (BATCH && ps) {
        // tiles of head 0, then of head 1, ...: the next one (in steps of vstep) that exists and has a
        // column the token can see
        int tl = i2 + vstep;
        bool more = false;
        while (tl < a.group_rows * ps_vt) {
          const int j = tl / ps_vt, vt = tl - j * ps_vt;
          const int32_t* vi; int vc; const uint32_t* bm;
          ps_head(j, vi, vc, bm);
          if (64 * vt < vc && (int64_t)__builtin_amdgcn_readfirstlane(vi[64 * vt]) <= last_pos) { more = true; break; }
          tl += vstep;
        }
        if (more) i2 = tl; else { k2 = 2; i2 = 0; }
      } else {
      const int vt = i2 + vstep;
      bool more = vt < n_vt;
      if (more) more = (int64_t)__builtin_amdgcn_readfirstlane(vidx_h[64 * vt]) <= last_pos;
      if (more) i2 = vt; else { k2 = 2; i2 = 0; }
      }
    }
    // the descriptor is uniform by construction; say so, so that it lives in scalar registers
    kind = __builtin_amdgcn_readfirstlane(k2);
    idx = __builtin_amdgcn_readfirstlane(i2);
    mask = __builtin_amdgcn_readfirstlane(m2);
  };
  // key index that tile row r comes from (general path)
  auto src_row = [&](int kind, int idx, int r) -> int64_t {
    if (kind == 0) {
      int64_t j = (int64_t)(m0 - (idx - (NQB - 1))) * 64 + r;
      return j < n_k ? j : n_k - 1;
    }
    if (BATCH && ps) {
      const int j = idx / ps_vt;
      const int32_t* vi; int vc; const uint32_t* bm;
      ps_head(j, vi, vc, bm);
      const int pos = 64 * (idx - j * ps_vt) + r;
      return pos < vc ? (int64_t)vi[pos] : 0;
    }
    int pos = 64 * idx + r;
    return pos < vcnt ? (int64_t)vidx_h[pos] : 0;
  };

  // ---- staging: global -> LDS copies, GPW groups of RPG rows per wave for K and for V --------
  // wave wv copies groups q = e * (2 NQB) + wv, e = 0..GPW-1; with this interleaving the
  // swizzle of a lane's row does not depend on e, so one 32-bit offset per lane serves all
  // its copies and the e-dependent part stays in scalar registers.
  constexpr int WAVES = 2 * NQB;
  const int lr = lane / DCH, lc = lane % DCH;  // this lane's row inside a group, and its LDS slot
  const int r0 = wv * RPG + lr;                // its row in the group e = 0
  const int kch = lc ^ ((r0 / R) % DCH);       // d-chunk it fetches for K (after the swizzle)
  const int vch = lc ^ ((((r0 / R) & 3) << 2) & (DCH - 1));  // ... and for V
  static_assert((WAVES * RPG / R) % DCH == 0 && (WAVES * RPG / R) % 4 == 0, "swizzle must not depend on e");
  static_assert(GPW == 1 || GPW == 2 || GPW == 4, "copies of a tile per wave");
  uint32_t koff[GPW], voff[GPW];  // byte offset of this lane's 16 bytes in copy e of a tile
#pragma unroll
  for (int e = 0; e < GPW; ++e) {
    koff[e] = (uint32_t)((e * WAVES * RPG + r0) * a.k_stride_tok * 2 + kch * 16);
    voff[e] = (uint32_t)((e * WAVES * RPG + r0) * a.v_stride_tok * 2 + vch * 16);
  }
  auto issue_k = [&](int kind, int idx, int buf) {
    const uint32_t kdst = ks_addr + (uint32_t)(buf * TILE * 2 + wv * 1024);
    bool fast = false;
    if (kind == 0) {
      const int64_t j0 = (int64_t)(m0 - (idx - (NQB - 1))) * 64;
      if (__builtin_expect(j0 + 64 <= n_k, 1)) {  // whole block in range: uniform bases + one per-lane 32-bit offset
        fast = true;
#ifdef VS_X_NOCOPY
        if (ei > ei0 + 1) return;
#endif
#ifdef VS_X_SAMEBLK
        const char* kt = (const char*)kbase + (j0 & 64) * a.k_stride_tok * 2;
#else
        const char* kt = (const char*)kbase + j0 * a.k_stride_tok * 2;
#endif
        if constexpr (GPW == 4) dma16x4(kdst, kt, koff[0], koff[1], koff[2], koff[3], WAVES * 1024);
        else if constexpr (GPW == 2) dma16x2(kdst, kt, koff[0], koff[1], WAVES * 1024);
        else dma16_lane_ptr(kdst, kt + koff[0]);
      }
    }
    if (__builtin_expect(!fast, 0)) {
#pragma unroll
      for (int e = 0; e < GPW; ++e) {
        const int64_t j = src_row(kind, idx, e * WAVES * RPG + r0);
        dma16_lane_ptr(kdst + e * WAVES * 1024, kbase + j * a.k_stride_tok + kch * 8);
      }
      if (kind == 1 && tid < 64) vidx_s[buf * 64 + tid] = (int32_t)src_row(kind, idx, tid);
    }
  };
  auto issue_v = [&](int kind, int idx, int buf) {
    const uint32_t vdst = vs_addr + (uint32_t)(buf * TILE * 2 + wv * 1024);
    bool fast = false;
    if (kind == 0) {
      const int64_t j0 = (int64_t)(m0 - (idx - (NQB - 1))) * 64;
      if (__builtin_expect(j0 + 64 <= n_k, 1)) {
        fast = true;
#ifdef VS_X_NOCOPY
        if (ei > ei0 + 1) return;
#endif
#ifdef VS_X_SAMEBLK
        const char* vt = (const char*)vbase + (j0 & 64) * a.v_stride_tok * 2;
#else
        const char* vt = (const char*)vbase + j0 * a.v_stride_tok * 2;
#endif
        if constexpr (GPW == 4) dma16x4(vdst, vt, voff[0], voff[1], voff[2], voff[3], WAVES * 1024);
        else if constexpr (GPW == 2) dma16x2(vdst, vt, voff[0], voff[1], WAVES * 1024);
        else dma16_lane_ptr(vdst, vt + voff[0]);
      }
    }
    if (__builtin_expect(!fast, 0)) {
#pragma unroll
      for (int e = 0; e < GPW; ++e) {
        const int64_t j = src_row(kind, idx, e * WAVES * RPG + r0);
        dma16_lane_ptr(vdst + e * WAVES * 1024, vbase + j * a.v_stride_tok + vch * 8);
      }
    }
  };
  auto wait_copies = [&]() { __builtin_amdgcn_s_waitcnt(0x0F70); };  // vmcnt(0)

  // ---- per-lane LDS element offsets of the MFMA operands -------------------------------------
  // K rows as A operand of S^T = K Q^T: lane (j = lane%32, hh) reads d-chunk 2 st + hh of row j
  int k_ofs[DSTEPS];
  {
    const int y = hh ^ (((lane & 31) / R) % DCH);
#pragma unroll
    for (int st = 0; st < DSTEPS; ++st) k_ofs[st] = (lane & 31) * D + ((2 * st) ^ y) * 8;
  }
  // V^T operand through the transposing LDS read: inside each 16-lane group, lane L supplies
  // the address of V[J0 + L/4][D0 + 4 (L%4) .. +3] and receives V[J0 .. J0+3][D0 + L];
  // D0 = 32 db + 16 * (group & 1), J0 = (multiple of 8) + 4 hh.
  int v_ofs[DB];
  {
    const int rl = ((lane & 15) >> 2) + 4 * hh;
    const int gl = (((rl / R) & 3) << 2) & (DCH - 1);
    const int ul = 2 * ((lane >> 4) & 1) + ((lane >> 1) & 1);
#pragma unroll
    for (int db = 0; db < DB; ++db) v_ofs[db] = rl * D + (((4 * db + ul) ^ gl) * 8) + 4 * (lane & 1);
  }

  auto k_load = [&](const __bf16* kb, int jb, int st) -> bf16x8 {
    return *(const bf16x8*)&kb[k_ofs[st] + 32 * jb * D];
  };
  auto v_load = [&](const __bf16* vb, int jb, int tt, int db) -> bf16x8 {
    typedef bf16x4 __attribute__((address_space(3))) * lds_b4;
    const __bf16* p0 = &vb[v_ofs[db] + (32 * jb + 16 * tt) * D];
    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_b4)(p0));
    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_b4)(p0 + 8 * D));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  };
  auto qk_step = [&](f32x16& acc, const __bf16* kb, int jb, int st) {
    const bf16x8 ka = *(const bf16x8*)&kb[k_ofs[st] + 32 * jb * D];
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[st], acc, 0, 0, 0);
  };
  auto to_bf16 = [&](const f32x16& sv, int tt) -> bf16x8 {
    f32x8 pf;
#pragma unroll
    for (int x = 0; x < 8; ++x) pf[x] = sv[8 * tt + x];
    return __builtin_convertvector(pf, bf16x8);
  };
  auto block_max = [&](const f32x16& sv) -> float {
    float mx = sv[0];
#pragma unroll
    for (int x = 1; x < 16; ++x) mx = fmaxf(mx, sv[x]);
    return mx;
  };
  // sv <- exp2(sv * scale_log2 - m_ref); returns this lane's sum of the 16 probabilities
  auto exp_block = [&](f32x16& sv, float m_ref) -> float {
    float ps = 0.f;
#pragma unroll
    for (int x = 0; x < 16; ++x) {
      const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[x], a.scale_log2, -m_ref));
      sv[x] = p;
      ps += p;
    }
    return ps;
  };

  // ---- per-step building blocks ----------------------------------------------------------------
  const float c = a.scale_log2;
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  typedef __attribute__((ext_vector_type(2))) float f32x2;
  constexpr float kTooLarge = 1.8446744e19f;  // 2^64: a probability above it means the reference is stale
  // probabilities of score pair (x, x + 1) of sv relative to ref, rounded to bf16 into operand
  // P0 (x < 8) or P1; the row sum takes the unrounded values (it also feeds the lse output)
  auto exp_pair = [&](const f32x16& sv, int x, float ref, bf16x8& P0, bf16x8& P1, float& ps) {
    f32x2 pf;
    pf[0] = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[x], c, -ref));
    pf[1] = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[x + 1], c, -ref));
    const bf16x2 pk = __builtin_convertvector(pf, bf16x2);
    ps += pf[0] + pf[1];
    bf16x8& P = x < 8 ? P0 : P1;
    P[x & 7] = pk[0];
    P[(x & 7) + 1] = pk[1];
  };
  constexpr int NM = DSTEPS;  // MFMAs of one 32-key half of K Q^T, and of one half of V^T P^T
  static_assert(2 * DB == DSTEPS, "both contractions of a half take the same number of MFMAs");
  // V fragment u (0 .. 2 NM - 1) of the pending tile: half u / NM, k-step tt, output block db
  auto v_frag = [&](const __bf16* vbp, int u) -> bf16x8 { return v_load(vbp, u / NM, (u % NM) / DB, u % DB); };

  // V^T P^T of the pending tile alone (this wave has no K Q^T to pair it with in this step)
  auto drain = [&](const __bf16* vbp) {
    constexpr int VPF = 3, VNB = VPF + 1;
    bf16x8 vf[VNB];
#pragma unroll
    for (int j = 0; j < VPF; ++j) vf[j] = v_frag(vbp, j);
#pragma unroll
    for (int u = 0; u < 2 * NM; ++u) {
      if (u + VPF < 2 * NM) vf[(u + VPF) % VNB] = v_frag(vbp, u + VPF);
      oacc[u % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[u % VNB], pp[u / DB], oacc[u % DB], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    l_run += pend_ps;
    pend = false;
  };

  // K Q^T of a masked tile, of the first tile of a row block, or of a tile whose scores
  // outran the reference: true maximum first, then the exponentials.  Nothing may be pending
  // (the accumulators must be up to date when the reference moves).  Leaves the tile pending.
  // offset of this row's position inside its 64-key block (the last key of the diagonal block it
  // may use); packed decode: all rows stand at the same position
  const int il_diag = a.same_pos ? a.pos_in_block : il;
  // DCA: first key block of the chunk that holds this wave's query block
  const int dca_cs = DCA ? ((m0 + t) / a.dca_cblk) * a.dca_cblk : 0;
  int need_var = 0;       // DCA: rotation this wave's tile needs; 3 = it differs inside the tile (codes in dcak_s)
  uint32_t dca_need = 0;  //      need_var == 3: bit v set iff some usable element needs rotation v
  bool qsw = false;       //      the registers hold another rotation than the tile needs
  auto qk_exact = [&](const __bf16* kb, bool diag, bool vert, auto&& apply_mask) {
    f32x16 s0, s1;
#pragma unroll
    for (int x = 0; x < 16; ++x) { s0[x] = 0.f; s1[x] = 0.f; }
    if (DCA && need_var == 3) {
      // one product per rotation that occurs in the tile; an element takes the product of its
      // own pattern.  Code of key r: 100 = intra-chunk; otherwise a threshold thr: rows
      // il < thr are inside the local window (successive-chunk), the others inter-chunk.
#pragma unroll
      for (int var = 0; var < 3; ++var) {
        if (!((dca_need >> var) & 1u)) continue;
        if (q_var != var) load_q(var);
#pragma unroll
        for (int jb = 0; jb < 2; ++jb) {
          f32x16 tt;
#pragma unroll
          for (int x = 0; x < 16; ++x) tt[x] = 0.f;
#pragma unroll
          for (int st = 0; st < DSTEPS; ++st) qk_step(tt, kb, jb, st);
#pragma unroll
          for (int xq = 0; xq < 4; ++xq) {
            const uint32_t cd = *(const uint32_t*)&dcak_s[wv * 64 + 32 * jb + 8 * xq + 4 * hh];
#pragma unroll
            for (int x = 0; x < 4; ++x) {
              const int code = (int)((cd >> (8 * x)) & 255u);
              const int ev = code == 100 ? 0 : (il_diag < code ? 1 : 2);
              if (ev == var) {
                if (jb == 0) s0[4 * xq + x] = tt[4 * xq + x];
                else s1[4 * xq + x] = tt[4 * xq + x];
              }
            }
          }
        }
      }
    } else {
#pragma unroll
      for (int st = 0; st < DSTEPS; ++st) qk_step(s0, kb, 0, st);
#pragma unroll
      for (int st = 0; st < DSTEPS; ++st) qk_step(s1, kb, 1, st);
    }
    if (diag || vert) {
      apply_mask(s0, 0);
      apply_mask(s1, 1);
    }
    if constexpr (BATCH) {
      if (ps && !row_live) {
#pragma unroll
        for (int x = 0; x < 16; ++x) { s0[x] = -INFINITY; s1[x] = -INFINITY; }
      }
    }
    float mx = fmaxf(block_max(s0), block_max(s1));
    mx = fmaxf(mx, __shfl_xor(mx, 32)) * c;
    if (!have_max || __any(mx > m_o + 64.f)) {
      const float m_new = fmaxf(m_o, mx);
      const float alpha = m_new == m_o ? 1.f : __builtin_amdgcn_exp2f(m_o - m_new);
      m_o = m_new;
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int x = 0; x < 16; ++x) oacc[db][x] *= alpha;
      have_max = !__any(m_o == -INFINITY);
    }
    const float m_use = (m_o == -INFINITY) ? 0.f : m_o;
    float ps = 0.f;
#pragma unroll
    for (int x = 0; x < 16; x += 2) exp_pair(s0, x, m_use, pp[0], pp[1], ps);
#pragma unroll
    for (int x = 0; x < 16; x += 2) exp_pair(s1, x, m_use, pp[2], pp[3], ps);
    pend_ps = ps;
    pend = true;
  };

  // K Q^T of an unmasked tile with nothing pending: S(keys 0..31), then S(keys 32..63) with the
  // exponentials of the first half between its MFMAs.  Returns false if a score outran the
  // reference (the caller then redoes the tile on the exact path).
  auto qk_fast = [&](const __bf16* kb) -> bool {
    constexpr int PF = 3, NB = PF + 1;
    bf16x8 kf[NB];
    f32x16 sa, sn;
#pragma unroll
    for (int x = 0; x < 16; ++x) { sa[x] = 0.f; sn[x] = 0.f; }
#pragma unroll
    for (int j = 0; j < PF; ++j) kf[j] = k_load(kb, j / NM, j % NM);
#pragma unroll
    for (int st = 0; st < NM; ++st) {
      const int j = st + PF;
      kf[j % NB] = k_load(kb, j / NM, j % NM);
      sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[st % NB], qreg[st], sa, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    float ps = 0.f;
#pragma unroll
    for (int st = 0; st < NM; ++st) {
      const int j = NM + st + PF;
      if (j < 2 * NM) kf[j % NB] = k_load(kb, 1, j - NM);
      sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[(NM + st) % NB], qreg[st], sn, 0, 0, 0);
#pragma unroll
      for (int x = (16 / NM) * st; x < (16 / NM) * (st + 1); x += 2) exp_pair(sa, x, m_o, pp[0], pp[1], ps);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int x = 0; x < 16; x += 2) exp_pair(sn, x, m_o, pp[2], pp[3], ps);
    if (__builtin_expect(__any(!(ps < kTooLarge)), 0)) return false;
    pend_ps = ps;
    pend = true;
    return true;
  };

  // The steady state: K Q^T of this tile and V^T P^T of the previous one in one instruction
  // stream, so that most MFMAs have a share of the softmax arithmetic next to them:
  //   A  NM MFMAs      QK(keys 0..31)
  //   B  3 NM / 2      QK(keys 32..63) with a quarter of PV(prev) mixed in | exp of keys 0..31
  //   C  3 NM / 2      the rest of PV(prev)                               | exp of keys 32..63
  // LDS operands are fetched PF MFMAs ahead; the scheduling fences pin the interleaving.
  // Returns false if a score outran the reference; the previous tile is folded in either way.
  auto fused = [&](const __bf16* kb, const __bf16* vbp, auto&& launch) -> bool {
    constexpr int PF = 3, NB = PF + 1;
    constexpr int NBQ = NM / 2;  // PV MFMAs mixed into phase B
    // MFMA n of the step: which operand it takes from LDS
    auto is_k = [&](int n) -> bool { return n < NM || (n < NM + 3 * NBQ && (n - NM) % 3 != 2); };
    auto k_index = [&](int n) -> int { return n < NM ? n : NM + 2 * ((n - NM) / 3) + (n - NM) % 3; };  // jb * NM + st
    auto v_index = [&](int n) -> int { return n < NM + 3 * NBQ ? (n - NM) / 3 : n - NM - 2 * NBQ; };
    auto frag = [&](int n) -> bf16x8 {
      if (is_k(n)) return k_load(kb, k_index(n) / NM, k_index(n) % NM);
#ifdef VS_X_NOVLDS
      return qreg[v_index(n) % DSTEPS];
#else
      return v_frag(vbp, v_index(n));
#endif
    };
    bf16x8 fq[NB];
    f32x16 sa, sn;
#pragma unroll
    for (int x = 0; x < 16; ++x) { sa[x] = 0.f; sn[x] = 0.f; }
#pragma unroll
    for (int j = 0; j < PF; ++j) fq[j] = frag(j);
    // the first operands are on their way from LDS while the copies are launched
    __builtin_amdgcn_sched_barrier(0);
    launch();
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(2);  // this wave's MFMA stream goes before the other workgroup's bookkeeping
    bf16x8 q0, q1;  // the second half's operands replace pp[0], pp[1], which are spent by then
    float ps = 0.f;
    int xa = 0, xb = 0;  // next score pair of each half (compile-time after unrolling)
#pragma unroll
    for (int n = 0; n < 4 * NM; ++n) {
      if (n + PF < 4 * NM) fq[(n + PF) % NB] = frag(n + PF);
      if (is_k(n)) {
        const int ki = k_index(n);
        if (ki < NM) sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq[n % NB], qreg[ki], sa, 0, 0, 0);
        else sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq[n % NB], qreg[ki - NM], sn, 0, 0, 0);
      } else {
        const int u = v_index(n);
        oacc[u % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq[n % NB], pp[u / DB], oacc[u % DB], 0, 0, 0);
      }
      if (n >= NM && n < NM + 3 * NBQ) {
        const int hi = 16 * (n - NM + 1) / (3 * NBQ);
        for (; xa + 2 <= hi; xa += 2) exp_pair(sa, xa, m_o, q0, q1, ps);
      } else if (n >= NM + 3 * NBQ) {
        const int hi = 16 * (n - NM - 3 * NBQ + 1) / (3 * NBQ);
        for (; xb + 2 <= hi; xb += 2) exp_pair(sn, xb, m_o, pp[0], pp[1], ps);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    __builtin_amdgcn_s_setprio(0);
    l_run += pend_ps;
    pend = false;
    if (__builtin_expect(__any(!(ps < kTooLarge)), 0)) return false;
    pp[2] = pp[0]; pp[3] = pp[1]; pp[0] = q0; pp[1] = q1;
    pend_ps = ps;
    pend = true;
    return true;
  };

  // ---- prologue: K of tile 0 -> LDS buffer 0 ----------------------------------------------------
  int cur_kind = 0, cur_idx = -1, cur_mask = 0;
  advance(cur_kind, cur_idx, cur_mask);
  int nxt_kind = cur_kind, nxt_idx = cur_idx, nxt_mask = cur_mask;
  if (cur_kind != 2) {
    issue_k(cur_kind, cur_idx, 0);
    advance(nxt_kind, nxt_idx, nxt_mask);
  }
  wait_copies();
  __syncthreads();
  int buf = 0;

  // Step i multiplies K of tile i (LDS buffer i % 2) with Q and V of tile i - 1 (buffer
  // (i - 1) % 2) with its probabilities.  The copies of K(i + 1) and V(i) into the two free
  // buffers run under this arithmetic; one barrier per step.  One extra step after the last
  // tile drains the pipeline.
  bool last = false, part = false, diag = false, vert = false;
  const __bf16* kb = Ks;
  const __bf16* vbp = Vs;
  // element x of block jb is key r = 32 jb + 8 (x/4) + 4 hh + (x%4) of the tile
  auto apply_mask = [&](f32x16& sv, int jb) {
    if (diag) {
#pragma unroll
      for (int x = 0; x < 16; ++x) {
        const int r = 32 * jb + 8 * (x >> 2) + 4 * hh + (x & 3);
        if (r > il_diag) sv[x] = -INFINITY;
      }
    } else {
#pragma unroll
      for (int xq = 0; xq < 4; ++xq) {
        const uint32_t nd = *(const uint32_t*)&need_s[wv * 64 + 32 * jb + 8 * xq + 4 * hh];
#pragma unroll
        for (int x = 0; x < 4; ++x)
          if (il < (int)((nd >> (8 * x)) & 255u)) sv[4 * xq + x] = -INFINITY;
      }
    }
  };
  // start of a step: find out whether this wave takes part in tile i and with which element
  // mask.  A masked tile gives every key r of the tile a threshold need[r]:
  // row il of the query block may use it iff il >= need[r] (64 = never).  Slash tile on the
  // block's own diagonal: need[r] = r.  Vertical tile: 0 for a column of an earlier, uncovered
  // key block; the column's offset inside the block when it lies in the query block's own key
  // block; 64 when it is out of range, in a later block, or already covered by a computed
  // diagonal.
  auto classify = [&]() {
    last = cur_kind == 2;
    kb = Ks + buf * TILE;
    vbp = Vs + (buf ^ 1) * TILE;
    part = wave_valid && !last;
    diag = false;
    bool usable = false;  // vertical tile: this lane's key can be used by some row of the block
    if (BATCH && ps && !last) {
      // heads packed into rows, every head with its own lists: every tile takes the masked path
      if (cur_kind == 0) {
        part = part && (cur_mask & 1);
        diag = cur_idx - (NQB - 1) + t == 0;
        row_live = il < kPackedSparseMaxGroup && (((cur_mask >> 4) >> il) & 1);
        need_s[wv * 64 + lane] = 0;           // no key of a slash tile is masked (the diagonal tile masks by position)
      } else {
        const int jh = cur_idx / ps_vt;       // the head whose columns this tile gathers
        const int32_t* vi; int vc; const uint32_t* bm;
        ps_head(jh, vi, vc, bm);
        const int pos = 64 * (cur_idx - jh * ps_vt) + lane;
        const int j = vidx_s[buf * 64 + lane];
        const int ad = (m0 + t) - (j >> 6);
        int need = 64;   // all rows stand at the token's position: a column is usable or not
        if (pos < vc && ad >= 0 && !bm_test(bm, ad) && !(ad == 0 && (j & 63) > a.pos_in_block)) need = 0;
        need_s[wv * 64 + lane] = (uint8_t)need;
        usable = need < 64;
        part = part && __ballot(usable) != 0;
        row_live = il == jh;
      }
      part = part && __ballot(row_live) != 0;
      vert = true;
    } else {
    if (__builtin_expect(cur_kind == 0, 1)) {
      part = part && ((cur_mask >> t) & 1);
      diag = cur_idx - (NQB - 1) + t == 0;  // block diagonal 0 of (query block t, this key block)
    } else if (!last) {
      const int pos = 64 * cur_idx + lane;
      const int j = vidx_s[buf * 64 + lane];
      const int ad = (m0 + t) - (j >> 6);
      int need = 64;
      if (pos < vcnt && ad >= 0 && !bm_test(bmA, ad)) need = ad == 0 ? (j & 63) : 0;
      need_s[wv * 64 + lane] = (uint8_t)need;
      usable = need < 64;
      part = part && __ballot(usable) != 0;
    }
    vert = cur_kind == 1;
    }
    if constexpr (DCA) {
      // which rotation of Q meets this tile's keys (section 5.1, DCA paragraph): keys of the
      // query block's own chunk the intra-chunk one; keys of the chunk before it, closer than
      // the local window, the successive-chunk one; all others the inter-chunk one
      qsw = false;
      if (part) {
        if (cur_kind == 0) {
          const int dblk = cur_idx - (NQB - 1) + t;  // block distance, >= 0 for a tile this wave takes
          const int cb = m0 + t - dblk;               // the key block
          if (cb >= dca_cs) need_var = 0;
          else if (cb >= dca_cs - a.dca_cblk && dblk < a.dca_wblk) need_var = 1;
          else if (cb >= dca_cs - a.dca_cblk && dblk == a.dca_wblk) {
            // the window ends inside this block: distance 64 dblk + il - r < window iff il < r
            need_var = 3;
            dca_need = 6u;
            dcak_s[wv * 64 + lane] = (uint8_t)lane;
          } else need_var = 2;
        } else {
          const int j = vidx_s[buf * 64 + lane];
          const int cb = j >> 6;
          int code = 0;
          if (cb >= dca_cs) code = 100;
          else if (cb >= dca_cs - a.dca_cblk) {
            const int thr = 64 * a.dca_wblk - (64 * (m0 + t) - j);  // il < thr: inside the window
            code = thr < 0 ? 0 : (thr > 64 ? 64 : thr);
          }
          dcak_s[wv * 64 + lane] = (uint8_t)code;
          dca_need = (__ballot(usable && code == 100) != 0 ? 1u : 0u) |
                     (__ballot(usable && code != 100 && code > 0) != 0 ? 2u : 0u) |
                     (__ballot(usable && code < 64) != 0 ? 4u : 0u);
          need_var = 3;
        }
        qsw = need_var != q_var;
        if (qsw && cur_kind == 0) {
          // a slash tile that needs another rotation takes the path of the masked tiles, with
          // a mask that lets every row use every key
          vert = true;
          need_s[wv * 64 + lane] = 0;
        }
      }
    }
  };
  // copies of K(i + 1) and V(i) into the buffers that step i - 1 used last
  auto launch_copies = [&]() {
    if (!last) {
      if (nxt_kind != 2) issue_k(nxt_kind, nxt_idx, buf ^ 1);
      issue_v(cur_kind, cur_idx, buf);
    }
  };
  auto end_step = [&]() {
    int nn_kind = nxt_kind, nn_idx = nxt_idx, nn_mask = nxt_mask;
    if (nxt_kind != 2) advance(nn_kind, nn_idx, nn_mask);
    wait_copies();
#ifndef VS_X_NOBARRIER
    __syncthreads();
#endif
    cur_kind = nxt_kind; cur_idx = nxt_idx; cur_mask = nxt_mask;
    nxt_kind = nn_kind; nxt_idx = nn_idx; nxt_mask = nn_mask;
    buf ^= 1;
  };

  for (;;) {
    classify();
    // steady state: runs of steps in which this wave multiplies tile i and folds in tile i - 1
    while (__builtin_expect(pend && part && !(diag || vert || !have_max), 1)) {
#ifdef VS_X_TIGHT
      // timing diagnostic (dense list only: entry index = cc, every mask full): the steps of the walk with
      // nothing but the fused arithmetic, the copies, the pace keeping and the barrier
      if (!DCA && !SPLIT && a.bm_stride == 0 && cur_kind == 0 && nxt_kind == 0 && cur_idx >= NQB) {
        while (cur_idx + 2 <= cc_end) {
          const int ci = cur_idx;
          auto launch = [&]() { issue_k(0, ci + 1, buf ^ 1); issue_v(0, ci, buf); };
          fused(Ks + buf * TILE, Vs + (buf ^ 1) * TILE, launch);
          enter_segment((cc_last - (ci + 2)) >> (a.sync_shift + seg_shift), true);
          wait_copies();
          __syncthreads();
          ++cur_idx;
          buf ^= 1;
        }
        nxt_idx = cur_idx + 1; nxt_mask = 3; cur_mask = 3;
        ei = nxt_idx;
        ecache = ent_h[(ei & ~63) + lane]; ecache_nx = ent_h[(ei & ~63) + 64 + lane];
        classify();
      }
#endif
      if (__builtin_expect(!fused(kb, vbp, launch_copies), 0)) qk_exact(kb, diag, vert, apply_mask);
      end_step();
      classify();
    }
    launch_copies();
    if (pend) drain(vbp);
    bool exact = diag || vert || !have_max;
    if constexpr (DCA) {
      if (part && qsw && need_var < 3) load_q(need_var);
    }
    if (part && !exact) exact = !qk_fast(kb);
    if (__builtin_expect(part && exact, 0)) qk_exact(kb, diag, vert, apply_mask);
    if (last) break;
    end_step();
  }

  // ---- normalise and store ------------------------------------------------------------------
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
  if constexpr (SPLIT) {
    // this split's share of the row: accumulators and row sum relative to the reference m_o
    const int64_t ro = row - a.row_pad;
    if (ro >= 0 && ro < a.q_rows) {
      const int64_t pr = ((int64_t)sp * a.n_q_heads + h) * a.q_rows + ro;
      float* op = a.part_o + pr * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          f32x4 o4;
#pragma unroll
          for (int x = 0; x < 4; ++x) o4[x] = oacc[db][4 * vq + x];
          *(f32x4*)(op + 32 * db + 8 * vq + 4 * hh) = o4;
        }
      if (hh == 0) {
        a.part_ml[2 * pr] = m_o;
        a.part_ml[2 * pr + 1] = l_tot;
      }
    }
  } else
  if (row >= a.row_pad && row < a.q_len) {
    const int64_t ro = row - a.row_pad;
    __bf16* op = a.out + ro * a.o_stride_tok + (int64_t)h * a.o_stride_head;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        f32x4 o4;
#pragma unroll
        for (int x = 0; x < 4; ++x) o4[x] = oacc[db][4 * vq + x] * inv;
        *(bf16x4*)(op + 32 * db + 8 * vq + 4 * hh) = __builtin_convertvector(o4, bf16x4);
      }
    if (a.lse && hh == 0)
      a.lse[(int64_t)h * a.q_rows + ro] =
          l_tot > 0.f ? (m_o + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
  }
  enter_segment(-1, false);  // (a tile whose walk ended early has marked nothing yet)
  __syncthreads();           // the LDS tiles are reused by the next round
  }  // rounds
}

// ---------------------------------------------------------------------------------------------
// Block list of one head from its selected slash offsets (one workgroup per head).
// Offset o crosses, inside a 64-aligned query block, the key blocks of diagonals floor(o/64)
// and, when o is not a multiple of 64, floor(o/64) + 1: these set the bitmap A.  The entry
// list then holds every cc for which A has a bit in [cc - (NQB-1), cc], with the per-query-
// block mask, in ascending order, followed by sentinels up to the end of the row.
// ---------------------------------------------------------------------------------------------
// With req != null the launch builds one list per (request, head), blockIdx.x = r * n_heads + h:
// offsets, their count, the number of key blocks and "dense" (no offsets given) come from the
// request; a request outside the bounds the workspace was sized for gets no list (the attention
// kernel skips it).
template <int NQB>
__global__ __launch_bounds__(256) void k_build_blocklist(const int32_t* s_idx, const int32_t* s_cnt,
                                                         int32_t s_budget, int dense, int n_blk,
                                                         int n_words, int ent_stride, uint32_t* bm_a,
                                                         uint32_t* ent, const vs_request* req, int n_heads,
                                                         int64_t max_q_len, int64_t max_n_k) {
  int h = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  uint32_t* A = bm_a + (int64_t)blockIdx.x * n_words;
  uint32_t* E = ent + (int64_t)blockIdx.x * ent_stride;
  if (req) {
    const vs_request rq = req[blockIdx.x / n_heads];
    h = blockIdx.x % n_heads;
    if (rq.q_len < 1 || rq.q_len > max_q_len || rq.q_start < 0 || rq.q_start + rq.q_len > max_n_k) return;
    dense = rq.s_idx == nullptr;
    if (!dense && !rq.s_cnt) return;
    s_idx = rq.s_idx; s_cnt = rq.s_cnt;
    n_blk = (int)((rq.q_start + rq.q_len + kBlock - 1) / kBlock);
  }
  __shared__ uint32_t wsum[4];
  __shared__ uint32_t running;
  for (int w = tid; w < n_words; w += 256) {
    uint32_t x = 0;
    if (dense) {
      const int lo = w * 32;
      if (lo + 32 <= n_blk) x = ~0u;
      else if (lo < n_blk) x = (1u << (n_blk - lo)) - 1u;
    }
    A[w] = x;
  }
  if (tid == 0) running = 0;
  __syncthreads();
  if (!dense) {
    const int cnt = s_cnt[h];
    const int32_t* so = s_idx + (int64_t)h * s_budget;
    for (int i = tid; i < cnt; i += 256) {
      const int o = so[i], ad = o >> 6;
      if (ad < n_blk) atomicOr(&A[ad >> 5], 1u << (ad & 31));
      if ((o & 63) && ad + 1 < n_blk) atomicOr(&A[(ad + 1) >> 5], 1u << ((ad + 1) & 31));
    }
    __syncthreads();
  }
  // ordered compaction of the U bits, 256 words per round
  for (int w0 = 0; w0 < n_words; w0 += 256) {
    const int w = w0 + tid;
    uint32_t cur = 0, prev = 0;
    if (w < n_words) { cur = A[w]; prev = w ? A[w - 1] : 0u; }
    uint32_t u = cur;
#pragma unroll
    for (int sft = 1; sft < NQB; ++sft) u |= (cur << sft) | (prev >> (32 - sft));
    const uint32_t c = __popc(u);
    // exclusive scan of c over the workgroup
    uint32_t inc = c;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const uint32_t y = __shfl_up(inc, d);
      if (lane >= d) inc += y;
    }
    if (lane == 63) wsum[wv] = inc;
    __syncthreads();
    uint32_t pos = running + inc - c;
    for (int x = 0; x < wv; ++x) pos += wsum[x];
    const uint64_t a64 = ((uint64_t)cur << 32) | prev;  // bit (32 + b) = A bit 32 w + b
    while (u) {
      const int b = __builtin_ctz(u);
      u &= u - 1;
      // mask bit t = A bit (32 w + b - (NQB-1) + t)
      const uint32_t mask = (uint32_t)(a64 >> (32 + b - (NQB - 1))) & ((1u << NQB) - 1u);
      E[pos++] = ((uint32_t)(32 * w + b) << 4) | mask;
    }
    __syncthreads();
    if (tid == 255) running = pos;
    __syncthreads();
  }
  for (int i = running + tid; i < ent_stride; i += 256) E[i] = kEntSentinel;
  // The last words of the bitmap row (beyond every diagonal): the last one tells the attention kernel how
  // sparse the list is: sync segments of this head are 2^shift times the base size, so that a
  // segment holds about as many listed key blocks as it would in a dense list.
  if (tid == 0) {
    const uint32_t n_ent = running > 0 ? running : 1u;
    int shift = 0;
    while (shift < 4 && ((uint32_t)n_blk >> (shift + 1)) >= n_ent) ++shift;
    A[n_words - 1] = (uint32_t)shift;
    A[n_words - 2] = running;  // length of the list: the head's share of the work (k_attn_schedule)
  }
}

// Union list of a sparse single-token request whose heads are packed into rows (one workgroup per
// (request, KV head), after k_build_blocklist has made the bitmaps of the request's heads): the
// bitmap words of the G heads are OR-ed; every set bit b becomes the entry ((b + 1) << 4) | 1 (key
// block m0 - b for the one query block of the tile) with, in ent_hm, the heads whose own bitmap has
// the bit.  Ascending, sentinels to the end of the row.  Requests of any other kind are left alone.
__global__ __launch_bounds__(256) void k_build_union(const vs_request* req, int n_q_heads, int n_kv_heads,
                                                     int64_t max_q_len, int64_t max_n_k, int n_words, int ent_stride,
                                                     const uint32_t* bm_a, uint32_t* bm_u, uint32_t* ent_u,
                                                     uint32_t* ent_hm) {
  const int r = blockIdx.x / n_kv_heads, g = blockIdx.x % n_kv_heads;
  const int G = n_q_heads / n_kv_heads;
  const vs_request rq = req[r];
  if (rq.q_len != 1 || rq.q_len > max_q_len || rq.q_start < 0 || rq.q_start + rq.q_len > max_n_k) return;
  if (!rq.s_idx || !rq.s_cnt || G < 2 || G > kPackedSparseMaxGroup) return;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const uint32_t* A0 = bm_a + ((int64_t)r * n_q_heads + (int64_t)g * G) * n_words;   // bitmaps of the group's heads
  uint32_t* U = bm_u + (int64_t)blockIdx.x * n_words;
  uint32_t* E = ent_u + (int64_t)blockIdx.x * ent_stride;
  uint32_t* M = ent_hm + (int64_t)blockIdx.x * ent_stride;
  const int n_bits = 32 * (n_words - 2);   // the last two words of a head's bitmap row hold other things
  __shared__ uint32_t wsum[4];
  __shared__ uint32_t running;
  if (tid == 0) running = 0;
  __syncthreads();
  for (int w0 = 0; w0 < n_words - 2; w0 += 256) {
    const int w = w0 + tid;
    uint32_t u = 0;
    if (w < n_words - 2)
      for (int j = 0; j < G; ++j) u |= A0[(int64_t)j * n_words + w];
    if (w < n_words - 2) U[w] = u;
    const uint32_t c = __popc(u);
    uint32_t inc = c;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const uint32_t y = __shfl_up(inc, d);
      if (lane >= d) inc += y;
    }
    if (lane == 63) wsum[wv] = inc;
    __syncthreads();
    uint32_t pos = running + inc - c;
    for (int x = 0; x < wv; ++x) pos += wsum[x];
    while (u) {
      const int b = __builtin_ctz(u);
      u &= u - 1;
      uint32_t hm = 0;
      for (int j = 0; j < G; ++j) hm |= ((A0[(int64_t)j * n_words + w] >> b) & 1u) << j;
      E[pos] = ((uint32_t)(32 * w + b + 1) << 4) | 1u;
      M[pos] = hm;
      ++pos;
    }
    __syncthreads();
    if (tid == 255) running = pos;
    __syncthreads();
  }
  (void)n_bits;
  for (int i = running + tid; i < ent_stride; i += 256) { E[i] = kEntSentinel; M[i] = 0; }
}

// Issued-tile accounting, one workgroup per head: for every query block of the chunk, the
// number of slash tiles (computed diagonals a <= m) and of vertical tiles (groups of 64
// gathered columns with at least one usable column).  Mirrors what k_attention executes.
__global__ __launch_bounds__(256) void k_count_tiles(const int32_t* v_idx, const int32_t* v_cnt,
                                                    int32_t v_budget, const uint32_t* bm_a,
                                                    int n_words, int64_t q_start, int64_t q_len,
                                                    int64_t* tiles) {
  const int h = blockIdx.x;
  const uint32_t* A = bm_a + (int64_t)h * n_words;
  const int32_t* vi = v_idx + (int64_t)h * v_budget;
  const int vcnt = v_cnt[h];
  const int n_vt = (vcnt + 63) >> 6;
  const int mb0 = (int)(q_start / 64), n_qb = (int)((q_len + 63) / 64);
  __shared__ unsigned long long acc[2];
  if (threadIdx.x < 2) acc[threadIdx.x] = 0;
  __syncthreads();
  unsigned long long ns = 0, nv = 0;
  for (int qb = threadIdx.x; qb < n_qb; qb += blockDim.x) {
    const int m = mb0 + qb;
    for (int w = 0; w <= (m >> 5); ++w) {
      uint32_t x = A[w];
      if (w == (m >> 5) && (m & 31) != 31) x &= (2u << (m & 31)) - 1u;
      ns += __popc(x);
    }
    const int64_t rows = (q_len - 64ll * qb) < 64 ? (q_len - 64ll * qb) : 64;
    const int64_t lastp = q_start + 64ll * qb + rows - 1;
    for (int vt = 0; vt < n_vt; ++vt) {
      bool any = false;
      for (int r = 0; r < 64 && 64 * vt + r < vcnt; ++r) {
        const int j = vi[64 * vt + r];
        const int ad = m - (j >> 6);
        if (j <= lastp && ad >= 0 && !((A[ad >> 5] >> (ad & 31)) & 1u)) { any = true; break; }
      }
      nv += any;
    }
  }
  atomicAdd(&acc[0], ns);
  atomicAdd(&acc[1], nv);
  __syncthreads();
  if (threadIdx.x < 2) tiles[2 * h + threadIdx.x] = (int64_t)acc[threadIdx.x];
}

// ---------------------------------------------------------------------------------------------
hipError_t launch_build_blocklist(const vs_params& p, const int32_t* s_idx, const int32_t* s_cnt,
                                  bool dense, const BlockList& bl, hipStream_t st) {
  const int64_t n_k = p.q_start + p.q_len;
  const int n_blk = (int)ceil_div(n_k, kBlock);
  hipLaunchKernelGGL((k_build_blocklist<kAttnQBlocks>), dim3(bl.heads), dim3(256), 0, st, s_idx, s_cnt,
                     p.slash_budget, dense ? 1 : 0, n_blk, (int)bl.words, (int)bl.ent_stride, bl.bm_a, bl.ent,
                     (const vs_request*)nullptr, 1, (int64_t)0, (int64_t)0);
  return hipGetLastError();
}

// Pace keeping of the persistent launch: key blocks per sync segment.  The members of a group
// (one XCD) may be at most two segments apart, so about three segments of K and V (64 KiB per
// block at D = 128) are live in the caches at a time.  0 = automatic: 64 blocks at D = 128
// (measured best for full lists; sparse lists scale it up per head, see k_build_blocklist).
// (The tuning switches are process-wide atomics: a size query and the call it is for must see the
// same values; a call under a setting that needs more workspace than it was given is refused by
// the size check of the entry point.)
static std::atomic<int> g_sync_blocks{0};
void set_attn_segment_blocks(int blocks) { g_sync_blocks.store(blocks < 0 ? 0 : blocks, std::memory_order_relaxed); }
static int attn_sync_blocks(const vs_params& p) {
  const int forced = g_sync_blocks.load(std::memory_order_relaxed);
  if (forced > 0) {   // a power of two (rounded down): the kernel finds a block's segment with a shift
    int sb = 1;
    while (sb * 2 <= forced) sb *= 2;
    return sb;
  }
  const int per_block = kBlock * p.head_dim * 2 * 2;  // K and V of one KV head
  int sb = 1;
  while (sb * 2 * 3 * per_block <= (6 << 20)) sb *= 2;
  return sb;
}
static size_t attn_counter_bytes(const vs_params& p) {
  const int64_t n_blk = ceil_div(p.q_start + p.q_len, kBlock);
  return align_up((size_t)8 * (size_t)ceil_div(n_blk, attn_sync_blocks(p)) * sizeof(uint32_t), 256);
}
size_t attn_sync_bytes(const vs_params& p) {
  // counters, then the schedule: 8 rows of at most Hq x (query tiles) group-rounds
  const size_t rounds = (size_t)p.n_q_heads * (size_t)ceil_div(p.q_len + p.q_start % kBlock, (int64_t)64 * kAttnQBlocks);
  return attn_counter_bytes(p) + align_up(8 * rounds * sizeof(int32_t), 256);
}

// Key split of short chunks.  With few (query tile, head) units the persistent launch would
// leave most of the chip idle, each unit walking the whole context alone; the walk is then cut
// into n_split ranges.  The policy is fixed (512 workgroup slots: 256 compute units x 2), so
// that workspace sizes do not depend on the device.
static std::atomic<int> g_key_split{0};  // 0: automatic, 1: never, n: n ranges (still at least 16 key blocks each)
void set_attn_key_split(int n) { g_key_split.store(n < 0 ? 0 : (n > 16 ? 16 : n), std::memory_order_relaxed); }
// dense attention of one token with grouped queries: the heads of a KV group share a tile
bool attn_packed_decode(const vs_params& p, bool dense) {
  return dense && p.q_len == 1 && p.n_q_heads > p.n_kv_heads && p.n_q_heads / p.n_kv_heads <= 64 * kAttnQBlocks;
}
int attn_split(const vs_params& p, bool dense) {
  const int forced = g_key_split.load(std::memory_order_relaxed);
  if (forced == 1) return 1;
  const bool packed = attn_packed_decode(p, dense);
  const int64_t units = packed ? p.n_kv_heads
                               : ceil_div(p.q_len + p.q_start % kBlock, (int64_t)64 * kAttnQBlocks) * p.n_q_heads;
  const int64_t n_blk = ceil_div(p.q_start + p.q_len, kBlock);
  int64_t s = forced > 1 ? forced : 512 / units;
  const int64_t cap = packed && forced == 0 ? 128 : 16;  // few units when the heads are packed: more ranges
  if (s > cap) s = cap;
  if (s > n_blk / 16) s = n_blk / 16;  // at least 16 key blocks per range
  return s < 2 ? 1 : (int)s;
}
size_t attn_split_bytes(const vs_params& p, bool dense) {
  const int s = attn_split(p, dense);
  if (s == 1) return 0;
  const size_t rows = (size_t)s * p.n_q_heads * (size_t)p.q_len;
  return align_up(rows * p.head_dim * sizeof(float), 256) + align_up(rows * 2 * sizeof(float), 256);
}

// out = sum_s O_s 2^(m_s - M) / sum_s l_s 2^(m_s - M), M = max_s m_s; one wave per (row, head),
// splits folded in ascending order (fixed, so the result is run-to-run identical).
template <int D, bool BATCH = false>
__global__ __launch_bounds__(256) void k_attn_combine(const AttnArgs a0) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int h = blockIdx.y;
  AttnArgs a = a0;
  if constexpr (BATCH) {
    if (!batch_view(a0, blockIdx.z, a)) return;
    if (h >= a.n_q_heads) return;
  }
  if (row >= a.q_rows) return;
  float M = -INFINITY;
  for (int sp = 0; sp < a.n_split; ++sp)
    M = fmaxf(M, a.part_ml[2 * (((int64_t)sp * a.n_q_heads + h) * a.q_rows + row)]);
  float L = 0.f, acc[D / 64];
#pragma unroll
  for (int e = 0; e < D / 64; ++e) acc[e] = 0.f;
  if (M != -INFINITY) {
    for (int sp = 0; sp < a.n_split; ++sp) {
      const int64_t pr = ((int64_t)sp * a.n_q_heads + h) * a.q_rows + row;
      const float m = a.part_ml[2 * pr];
      if (m == -INFINITY) continue;
      const float w = __builtin_amdgcn_exp2f(m - M);
      L += a.part_ml[2 * pr + 1] * w;
#pragma unroll
      for (int e = 0; e < D / 64; ++e) acc[e] += a.part_o[pr * D + 64 * e + lane] * w;
    }
  }
  const float inv = L > 0.f ? 1.0f / L : 0.f;
  __bf16* op = a.out + row * a.o_stride_tok + (int64_t)h * a.o_stride_head;
#pragma unroll
  for (int e = 0; e < D / 64; ++e) op[64 * e + lane] = (__bf16)(acc[e] * inv);
  if (a.lse && lane == 0)
    a.lse[(int64_t)h * a.q_rows + row] = L > 0.f ? (M + __builtin_amdgcn_logf(L)) * kLn2 : -INFINITY;
}

// Which group takes which group-round.  Heads differ in the length of their block lists (by a
// factor of almost two in the 1M workloads), so dealing the rounds out in turn leaves some
// groups idle at the end.  The rounds are weighed (list length x number of key blocks the
// tiles can reach), sorted, and given one by one to the group with the least work so far; a
// group works through its rounds in that (descending) order.  One workgroup; only the timing
// of the attention launch depends on the result.
constexpr int kSchedMax = 8192;  // rounds the sort is done for (beyond it: dealt out in turn)
static std::atomic<int> g_sched_in_turn{0};
void set_attn_schedule_in_turn(int on) { g_sched_in_turn.store(on ? 1 : 0, std::memory_order_relaxed); }
__global__ __launch_bounds__(1024) void k_attn_schedule(const AttnArgs a, int32_t* sched, int in_turn) {
  __shared__ float w[kSchedMax];
  __shared__ uint16_t order[kSchedMax];
  __shared__ float avg_ent;
  const int tid = threadIdx.x, n_gr = a.n_gr;
  if (n_gr > kSchedMax || in_turn) {
    for (int x = tid; x < 8 * n_gr; x += 1024) {
      const int g = x / n_gr, r = x - g * n_gr;
      sched[x] = r * 8 + g < n_gr ? r * 8 + g : -1;
    }
    return;
  }
  if (tid == 0) {
    double sum = 0;
    for (int h = 0; h < a.n_q_heads; ++h) sum += (double)a.bm_a[(int64_t)h * a.bm_stride + a.bm_words - 2];
    avg_ent = (float)(sum / a.n_q_heads);
  }
  __syncthreads();
  const int n_full_gr = a.n_full * a.n_q_heads;
  const int mb = (int)(a.q_start / 64);
  for (int gr = tid; gr < n_gr; gr += 1024) {
    float ent, reach;
    if (gr < n_full_gr) {
      const int h = gr % a.n_q_heads, c = a.n_full - 1 - gr / a.n_q_heads;
      ent = (float)a.bm_a[(int64_t)h * a.bm_stride + a.bm_words - 2];
      reach = (float)(mb + 2 * (a.n_rem + c * a.members + a.members / 2) + 2);  // key blocks before the chunk's middle tile
    } else {
      ent = avg_ent;  // leftover tiles of several heads
      reach = (float)(mb + a.n_rem + 2);
    }
    w[gr] = ent * reach;
  }
  __syncthreads();
  for (int gr = tid; gr < n_gr; gr += 1024) {
    const float mine = w[gr];
    int rank = 0;
    for (int j = 0; j < n_gr; ++j) rank += (w[j] > mine || (w[j] == mine && j < gr)) ? 1 : 0;
    order[rank] = (uint16_t)gr;
  }
  __syncthreads();
  if (tid == 0) {
    float load[8];
    int cnt[8];
    for (int g = 0; g < 8; ++g) { load[g] = 0.f; cnt[g] = 0; }
    for (int i = 0; i < n_gr; ++i) {
      int g = 0;
      for (int x = 1; x < 8; ++x)
        if (load[x] < load[g]) g = x;
      const int gr = order[i];
      sched[g * n_gr + cnt[g]++] = gr;
      load[g] += w[gr];
    }
    for (int g = 0; g < 8; ++g)
      for (int r = cnt[g]; r < n_gr; ++r) sched[g * n_gr + r] = -1;
  }
}

__global__ __launch_bounds__(256) void k_fill_zero_u32(uint32_t* p, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) p[i] = 0u;
}

// Per-device set-up, done once for each device a launch is made on (with that device current):
// its number of compute units, and the opt-in of every attention instantiation to more than
// 64 KiB of LDS per workgroup (a function attribute, held per device by the runtime).
constexpr int kMaxDevices = 64;
static hipError_t attn_device_setup(int* n_cu_out) {
  static std::mutex mu;
  static int cu_of[kMaxDevices] = {0};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (cu_of[dev] == 0) {
    constexpr int NQB = kAttnQBlocks;
    int cu = 0;
    e = hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    if (cu < 1) return hipErrorInvalidDevice;
    const void* fns[10] = {reinterpret_cast<const void*>(&k_attention<128, NQB, false, false>),
                          reinterpret_cast<const void*>(&k_attention<64, NQB, false, false>),
                          reinterpret_cast<const void*>(&k_attention<128, NQB, true, false>),
                          reinterpret_cast<const void*>(&k_attention<64, NQB, true, false>),
                          reinterpret_cast<const void*>(&k_attention<128, NQB, false, true>),
                          reinterpret_cast<const void*>(&k_attention<64, NQB, false, true>),
                          reinterpret_cast<const void*>(&k_attention<128, NQB, true, true>),
                          reinterpret_cast<const void*>(&k_attention<64, NQB, true, true>),
                          reinterpret_cast<const void*>(&k_attention<128, NQB, false, true, true>),
                          reinterpret_cast<const void*>(&k_attention<64, NQB, false, true, true>)};
    for (int i = 0; i < 10; ++i) {
      e = hipFuncSetAttribute(fns[i], hipFuncAttributeMaxDynamicSharedMemorySize,
                              i % 2 == 0 ? attn_lds_bytes<128>() : attn_lds_bytes<64>());
      if (e != hipSuccess) return e;
    }
    cu_of[dev] = cu;
  }
  *n_cu_out = cu_of[dev];
  return hipSuccess;
}

hipError_t launch_attention(const vs_params& p, const void* q, const DcaArgs* dca, const void* k, const void* v,
                            const int32_t* v_idx, const int32_t* v_cnt, bool dense,
                            const BlockList& bl, void* out, float* lse, void* sync_ws, void* split_ws,
                            hipStream_t st) {
  constexpr int NQB = kAttnQBlocks;
  if (!sync_ws) return hipErrorInvalidValue;
  AttnArgs a;
  a.q = (const __bf16*)q; a.k = (const __bf16*)k; a.v = (const __bf16*)v;
  a.q_succ = dca ? (const __bf16*)dca->q_succ : nullptr;
  a.q_inter = dca ? (const __bf16*)dca->q_inter : nullptr;
  a.dca_cblk = dca ? (int32_t)(dca->chunk / kBlock) : 0;
  a.dca_wblk = dca ? (int32_t)(dca->window / kBlock) : 0;
  a.out = (__bf16*)out; a.lse = lse;
  a.q_stride_tok = p.q_stride_tok; a.q_stride_head = p.q_stride_head;
  a.k_stride_tok = p.k_stride_tok; a.k_stride_head = p.k_stride_head;
  a.v_stride_tok = p.v_stride_tok; a.v_stride_head = p.v_stride_head;
  a.o_stride_tok = p.o_stride_tok; a.o_stride_head = p.o_stride_head;
  a.bm_a = bl.bm_a; a.ent = bl.ent;
  a.bm_stride = dense ? 0 : bl.words;
  a.bm_words = (int32_t)bl.words;
  a.ent_stride = dense ? 0 : bl.ent_stride;
  a.ent_len = bl.ent_stride;
  a.v_idx = dense ? nullptr : v_idx; a.v_cnt = dense ? nullptr : v_cnt;
  a.v_budget = p.vertical_budget;
  a.n_q_heads = p.n_q_heads; a.n_kv_heads = p.n_kv_heads; a.group = p.n_q_heads / p.n_kv_heads;
  a.row_pad = (int32_t)(p.q_start % kBlock);
  a.q_start = p.q_start - a.row_pad;
  a.q_len = p.q_len + a.row_pad;
  a.q_rows = p.q_len;
  a.n_k = p.q_start + p.q_len;
  a.same_pos = 0; a.pos_in_block = 0;
  if (attn_packed_decode(p, dense)) {
    // rows = the G heads of a KV group, "heads" = the KV heads: the strides say so
    const int G = p.n_q_heads / p.n_kv_heads;
    a.q_stride_tok = p.q_stride_head; a.q_stride_head = (int64_t)G * p.q_stride_head;
    a.o_stride_tok = p.o_stride_head; a.o_stride_head = (int64_t)G * p.o_stride_head;
    a.n_q_heads = p.n_kv_heads; a.group = 1;
    a.same_pos = 1; a.pos_in_block = a.row_pad;
    a.row_pad = 0; a.q_len = G; a.q_rows = G;   // lse [Hkv][G] is the caller's [Hq][1]
  }
  a.n_qtiles = (int)ceil_div(a.q_len, 64 * NQB);
  a.scale_log2 = p.softmax_scale * kLog2e;
  // two workgroups fit a compute unit; one persistent workgroup per slot, in 8 groups
  int n_cu = 0;
  {
    const hipError_t e = attn_device_setup(&n_cu);
    if (e != hipSuccess) return e;
  }
  int members = ((4 / kAttnQBlocks) * n_cu) / 8;   // resident workgroups per XCD
  if (members < 1) members = 1;
  a.n_split = attn_split(p, dense);
  a.part_o = a.part_ml = nullptr;
  if (a.n_split > 1) {
    if (!split_ws) return hipErrorInvalidValue;
    const size_t rows = (size_t)a.n_split * p.n_q_heads * (size_t)p.q_len;  // (packed decode: Hkv x G rows, the same)
    a.part_o = (float*)split_ws;
    a.part_ml = (float*)((char*)split_ws + align_up(rows * p.head_dim * sizeof(float), 256));
  }
  const int64_t units = (int64_t)a.n_qtiles * a.n_q_heads * a.n_split;
  if (units < 8 * (int64_t)members) members = (int)ceil_div(units, 8);  // small launches: no idle workgroups
  a.members = members;
  a.n_wg = 8 * members;
  a.n_full = a.n_qtiles / members;
  a.n_rem = a.n_qtiles - a.n_full * members;
  a.sync_blocks = attn_sync_blocks(p);
  a.sync_shift = 0;
  while ((1 << (a.sync_shift + 1)) <= a.sync_blocks) ++a.sync_shift;
  a.n_sync = (int)ceil_div(ceil_div(p.q_start + p.q_len, kBlock), a.sync_blocks);
  a.arrive = (uint32_t*)sync_ws;
  a.n_gr = a.n_full * a.n_q_heads + (int)ceil_div((int64_t)a.n_rem * a.n_q_heads, a.members);
  int32_t* const sched = (int32_t*)((char*)sync_ws + attn_counter_bytes(p));
  a.sched = sched;
  if (a.n_split == 1) hipLaunchKernelGGL(k_attn_schedule, dim3(1), dim3(1024), 0, st, a, sched,
                                        g_sched_in_turn.load(std::memory_order_relaxed));
  hipLaunchKernelGGL(k_fill_zero_u32, dim3((unsigned)ceil_div(8 * (int64_t)a.n_sync, 256)), dim3(256), 0, st,
                     a.arrive, 8 * (int64_t)a.n_sync);
  const dim3 grid((unsigned)a.n_wg), block(128 * NQB);
  const bool split = a.n_split > 1;
#define VS_ATTN_LAUNCH(DD, DCA_, SPLIT_) \
  hipLaunchKernelGGL((k_attention<DD, NQB, DCA_, SPLIT_>), grid, block, attn_lds_bytes<DD>(), st, a)
  if (p.head_dim == 128) {
    if (dca && split) VS_ATTN_LAUNCH(128, true, true);
    else if (dca) VS_ATTN_LAUNCH(128, true, false);
    else if (split) VS_ATTN_LAUNCH(128, false, true);
    else VS_ATTN_LAUNCH(128, false, false);
  } else {
    if (dca && split) VS_ATTN_LAUNCH(64, true, true);
    else if (dca) VS_ATTN_LAUNCH(64, true, false);
    else if (split) VS_ATTN_LAUNCH(64, false, true);
    else VS_ATTN_LAUNCH(64, false, false);
  }
#undef VS_ATTN_LAUNCH
  if (split) {
    const dim3 cgrid((unsigned)ceil_div(a.q_rows, 4), (unsigned)a.n_q_heads);
    if (p.head_dim == 128) hipLaunchKernelGGL(k_attn_combine<128>, cgrid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL(k_attn_combine<64>, cgrid, dim3(256), 0, st, a);
  }
  return hipGetLastError();
}

// ---- several requests per launch ----------------------------------------------------------------
// p.q_len is the longest request, p.q_start + p.q_len the most keys any request sees.  The number
// of key ranges is one for the whole batch, chosen so that about 512 workgroups have a unit.
static int batch_rows_cap(const vs_params& p) {
  const int G = p.n_q_heads / p.n_kv_heads;
  return (int)(p.q_len > G ? p.q_len : G);   // a packed single-token request has G rows per KV head
}
static int batch_tiles(const vs_params& p) { return (int)ceil_div(p.q_len + kBlock - 1, (int64_t)64 * kAttnQBlocks); }
int attn_batch_split(const vs_params& p, int n_req) {
  // (a single-token request whose heads are packed into rows turns its G head slots into G times as
  // many key ranges, so the count of unit slots is the same for every kind of request)
  const int64_t units = (int64_t)n_req * p.n_q_heads * batch_tiles(p);
  const int64_t n_blk = ceil_div(p.q_start + p.q_len, kBlock);
  int64_t s = 512 / units;
  const int64_t cap = 16;
  if (s > cap) s = cap;
  if (s > n_blk / 16) s = n_blk / 16;
  return s < 1 ? 1 : (int)s;
}
size_t attn_batch_bytes(const vs_params& p, int n_req) {
  const int64_t n_k = p.q_start + p.q_len;
  const size_t lists = (size_t)n_req * p.n_q_heads;
  const size_t rows = (size_t)n_req * attn_batch_split(p, n_req) * p.n_q_heads * (size_t)batch_rows_cap(p);
  const size_t ulists = (size_t)n_req * p.n_kv_heads;   // union lists of packed sparse single-token requests
  return align_up(lists * (size_t)bitmap_words(n_k) * 4, 256) + align_up(lists * (size_t)entry_stride(n_k) * 4, 256) +
         align_up(rows * p.head_dim * sizeof(float), 256) + align_up(rows * 2 * sizeof(float), 256) + 256 +
         align_up(ulists * (size_t)bitmap_words(n_k) * 4, 256) + 2 * align_up(ulists * (size_t)entry_stride(n_k) * 4, 256);
}

hipError_t launch_attention_batch(const vs_params& p, const vs_request* req, int n_req, void* ws, hipStream_t st) {
  constexpr int NQB = kAttnQBlocks;
  const int64_t n_k = p.q_start + p.q_len;
  const size_t lists = (size_t)n_req * p.n_q_heads;
  const int64_t words = bitmap_words(n_k), ent_stride = entry_stride(n_k);
  char* w = (char*)ws;
  uint32_t* bm_a = (uint32_t*)w;
  w += align_up(lists * (size_t)words * 4, 256);
  uint32_t* ent = (uint32_t*)w;
  w += align_up(lists * (size_t)ent_stride * 4, 256);
  AttnArgs a = {};
  a.n_split = attn_batch_split(p, n_req);
  a.rows_cap = batch_rows_cap(p);
  const size_t rows = (size_t)n_req * a.n_split * p.n_q_heads * (size_t)a.rows_cap;
  a.part_o = (float*)w;
  w += align_up(rows * p.head_dim * sizeof(float), 256);
  a.part_ml = (float*)w;
  w += align_up(rows * 2 * sizeof(float), 256);
  a.arrive = (uint32_t*)w;   // unused by the key-split kernel; one valid word
  w += 256;
  const size_t ulists = (size_t)n_req * p.n_kv_heads;
  a.bm_u = (uint32_t*)w;
  w += align_up(ulists * (size_t)words * 4, 256);
  uint32_t* ent_u = (uint32_t*)w;
  w += align_up(ulists * (size_t)ent_stride * 4, 256);
  uint32_t* ent_hm = (uint32_t*)w;
  a.ent_u = ent_u; a.ent_hm = ent_hm;
  a.n_sync = 1; a.sync_blocks = 1 << 30; a.sync_shift = 30; a.sched = nullptr; a.n_gr = 0;
  a.q_stride_tok = p.q_stride_tok; a.q_stride_head = p.q_stride_head;
  a.k_stride_tok = p.k_stride_tok; a.k_stride_head = p.k_stride_head;
  a.v_stride_tok = p.v_stride_tok; a.v_stride_head = p.v_stride_head;
  a.o_stride_tok = p.o_stride_tok; a.o_stride_head = p.o_stride_head;
  a.bm_a = bm_a; a.ent = ent;
  a.bm_stride = words; a.bm_words = (int32_t)words;
  a.ent_stride = ent_stride; a.ent_len = ent_stride;
  a.v_budget = p.vertical_budget;
  a.n_q_heads = p.n_q_heads; a.n_kv_heads = p.n_kv_heads; a.group = p.n_q_heads / p.n_kv_heads;
  a.n_qtiles = batch_tiles(p);
  a.n_k = n_k;
  a.scale_log2 = p.softmax_scale * kLog2e;
  a.req = req; a.n_req = n_req; a.head_dim = p.head_dim;
  a.max_q_len = p.q_len; a.max_n_k = n_k;
  int n_cu = 0;
  hipError_t e = attn_device_setup(&n_cu);
  if (e != hipSuccess) return e;
  const int64_t units = (int64_t)n_req * a.n_q_heads * a.n_qtiles * a.n_split;
  int members = ((4 / kAttnQBlocks) * n_cu) / 8;   // resident workgroups per XCD
  if (members < 1) members = 1;
  if (units < 8 * (int64_t)members) members = (int)ceil_div(units, 8);
  a.members = members; a.n_wg = 8 * members; a.n_full = 0; a.n_rem = 0;
  hipLaunchKernelGGL((k_build_blocklist<NQB>), dim3((unsigned)lists), dim3(256), 0, st, (const int32_t*)nullptr,
                     (const int32_t*)nullptr, p.slash_budget, 0, 0, (int)words, (int)ent_stride, bm_a, ent, req,
                     (int)p.n_q_heads, (int64_t)p.q_len, n_k);
  if (a.group > 1 && a.group <= kPackedSparseMaxGroup)
    hipLaunchKernelGGL(k_build_union, dim3((unsigned)ulists), dim3(256), 0, st, req, (int)p.n_q_heads,
                       (int)p.n_kv_heads, (int64_t)p.q_len, n_k, (int)words, (int)ent_stride, bm_a, a.bm_u, ent_u, ent_hm);
  else
    a.ent_u = nullptr;   // no grouped queries (or too many heads per group for the row masks): nothing to pack
  const dim3 grid((unsigned)a.n_wg), block(128 * NQB);
  const dim3 cgrid((unsigned)ceil_div(a.rows_cap, 4), (unsigned)a.n_q_heads, (unsigned)n_req);
  if (p.head_dim == 128) {
    hipLaunchKernelGGL((k_attention<128, NQB, false, true, true>), grid, block, attn_lds_bytes<128>(), st, a);
    hipLaunchKernelGGL((k_attn_combine<128, true>), cgrid, dim3(256), 0, st, a);
  } else {
    hipLaunchKernelGGL((k_attention<64, NQB, false, true, true>), grid, block, attn_lds_bytes<64>(), st, a);
    hipLaunchKernelGGL((k_attn_combine<64, true>), cgrid, dim3(256), 0, st, a);
  }
  return hipGetLastError();
}

// Sparse attention of one token with grouped queries through the batch machinery (one request):
// the heads of a KV group share a tile and the walk of the union of their lists, so K and V are
// read once per group.  The request's descriptor is written into the workspace by a kernel.
bool attn_single_token_packs(const vs_params& p) {
  const int G = p.n_q_heads / p.n_kv_heads;
  return p.q_len == 1 && G > 1 && G <= kPackedSparseMaxGroup;
}
size_t attn_single_token_bytes(const vs_params& p) { return 256 + attn_batch_bytes(p, 1); }
__global__ void k_write_request(vs_request* dst, const vs_request rq) { *dst = rq; }
hipError_t launch_attention_single_token(const vs_params& p, const void* q, const void* k, const void* v,
                                         const int32_t* v_idx, const int32_t* v_cnt, const int32_t* s_idx,
                                         const int32_t* s_cnt, void* out, float* lse, void* ws, hipStream_t st) {
  vs_request rq;
  rq.q = q; rq.k = k; rq.v = v; rq.out = out; rq.lse = lse;
  rq.v_idx = v_idx; rq.v_cnt = v_cnt; rq.s_idx = s_idx; rq.s_cnt = s_cnt;
  rq.q_start = p.q_start; rq.q_len = p.q_len;
  hipLaunchKernelGGL(k_write_request, dim3(1), dim3(1), 0, st, (vs_request*)ws, rq);
  return launch_attention_batch(p, (const vs_request*)ws, 1, (char*)ws + 256, st);
}

hipError_t launch_count_tiles(const vs_params& p, const int32_t* v_idx, const int32_t* v_cnt,
                              const BlockList& bl, int64_t* tiles, hipStream_t st) {
  hipLaunchKernelGGL(k_count_tiles, dim3(p.n_q_heads), dim3(256), 0, st, v_idx, v_cnt,
                     p.vertical_budget, bl.bm_a, (int)bl.words, p.q_start - p.q_start % kBlock,
                     p.q_len + p.q_start % kBlock, tiles);
  return hipGetLastError();
}

}  // namespace vs
