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
//  * V is transposed while it is written to LDS (4x8 register tiles, v_perm) because the PV
//    contraction runs over keys; key slots are permuted so that a lane's 8 keys are one
//    16-byte LDS read.
//  * global -> register prefetch of tile t+1 overlaps the MFMA work of tile t.
//  * blockIdx -> (tile, head): the G heads that share a KV head and the same query tile run
//    on one XCD back to back (shared L2), heaviest (latest) query tiles first.
#include "vs_common.h"

namespace vs {

struct AttnArgs {
  const __bf16* q;
  const __bf16* k;
  const __bf16* v;
  __bf16* out;
  float* lse;
  int64_t q_stride_tok, q_stride_head, k_stride_tok, k_stride_head;
  int64_t v_stride_tok, v_stride_head, o_stride_tok, o_stride_head;
  const uint32_t* bm_a;
  const uint32_t* bm_u;
  int64_t bm_stride;  // words per head, 0 = one bitmap shared by all heads (dense)
  const int32_t* v_idx;  // null: no vertical phase
  const int32_t* v_cnt;
  int32_t v_budget;
  int32_t n_q_heads, n_kv_heads, group;
  int32_t n_qtiles;
  int64_t q_len, q_start;
  float scale_log2;  // softmax_scale * log2(e)
};

__device__ __forceinline__ bool bm_test(const uint32_t* bm, int i) {
  return (bm[i >> 5] >> (i & 31)) & 1u;
}

// smallest set bit index >= from and < limit, else limit
__device__ __forceinline__ int bm_next(const uint32_t* bm, int from, int limit) {
  if (from >= limit) return limit;
  int w = from >> 5;
  uint32_t x = bm[w] & (~0u << (from & 31));
  while (true) {
    if (x) {
      int r = (w << 5) + __builtin_ctz(x);
      return r < limit ? r : limit;
    }
    ++w;
    if ((w << 5) >= limit) return limit;
    x = bm[w];
  }
}

// LDS bytes of one workgroup: K and V tiles double-buffered + the gathered column indices.
template <int D>
constexpr int attn_lds_bytes() { return 2 * 64 * (D + 8) * 2 + 2 * 64 * (D + 32) * 2 + 2 * 64 * 4; }

template <int D, int NQB>
__global__ __launch_bounds__(128 * NQB, 2) void k_attention(const AttnArgs a) {
  constexpr int NT = 128 * NQB;        // threads
  constexpr int KS = D + 8;            // LDS row stride of the K tile [64 keys][D], elements
  constexpr int VR = D + 32;           // LDS row stride of the V tile [64 keys][D], elements
  constexpr int DCH = D / 8;           // 16-byte chunks per row
  constexpr int DSTEPS = D / 16;       // MFMA k-steps of QK^T
  constexpr int DB = D / 32;           // 32-row blocks of O^T
  constexpr int CPT = 64 * DCH / NT;   // chunks per thread per tile, for K and for V
  constexpr int KBUF = 64 * KS, VBUF = 64 * VR;
  static_assert(64 * DCH % NT == 0, "tile must divide over the threads");

  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  __bf16* const Ks = (__bf16*)smem_raw;                 // [2][KBUF]
  __bf16* const Vs = Ks + 2 * KBUF;                     // [2][VBUF]
  int32_t* const vidx_s = (int32_t*)(Vs + 2 * VBUF);    // [2][64]

  // ---- which (query tile, head) -------------------------------------------------------
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int gi = (slot / a.group) * 8 + xcd, hin = slot % a.group;
  if (gi >= a.n_qtiles * a.n_kv_heads) return;
  const int qt = a.n_qtiles - 1 - gi / a.n_kv_heads;
  const int g = gi % a.n_kv_heads, h = g * a.group + hin;

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int t = wv >> 1;                          // query block of this wave inside the tile
  const int il = ((wv & 1) << 5) + (lane & 31);   // row inside the query block
  const int hh = lane >> 5;
  const int64_t row0 = (int64_t)qt * (64 * NQB);
  const int64_t row = row0 + 64 * t + il;
  const int m0 = (int)(a.q_start / 64) + qt * NQB;  // absolute index of query block t = 0
  const bool wave_valid = row0 + 64 * t + ((wv & 1) << 5) < a.q_len;
  const int64_t n_k = a.q_start + a.q_len;
  const int64_t rows_in_tile = (a.q_len - row0) < 64 * NQB ? (a.q_len - row0) : 64 * NQB;
  const int64_t last_pos = a.q_start + row0 + rows_in_tile - 1;

  const uint32_t* bmA = a.bm_a + (int64_t)h * a.bm_stride;
  const uint32_t* bmU = a.bm_u + (int64_t)h * a.bm_stride;
  const int32_t* vidx_h = a.v_idx ? a.v_idx + (int64_t)h * a.v_budget : nullptr;
  const int vcnt = a.v_idx ? a.v_cnt[h] : 0;
  const int n_vt = (vcnt + 63) >> 6;
  const int cc_limit = m0 + NQB;  // cc = c + NQB - 1, c <= m0

  const __bf16* kbase = a.k + (int64_t)g * a.k_stride_head;
  const __bf16* vbase = a.v + (int64_t)g * a.v_stride_head;

  // ---- Q^T operand: lane (i = lane%32, hh) holds Q[i][16 st + 8 hh .. +7] ----------------
  bf16x8 qreg[DSTEPS];
  {
    const int64_t rc = row < a.q_len ? row : a.q_len - 1;
    const __bf16* qp = a.q + rc * a.q_stride_tok + (int64_t)h * a.q_stride_head + 8 * hh;
#pragma unroll
    for (int st = 0; st < DSTEPS; ++st) qreg[st] = *(const bf16x8*)(qp + 16 * st);
  }

  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int x = 0; x < 16; ++x) oacc[db][x] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  // ---- tile iterator (uniform over the workgroup) -----------------------------------------
  // kind 0: slash tile, idx = cc; kind 1: vertical tile, idx = vt; kind 2: end
  auto advance = [&](int& kind, int& idx) {
    if (kind == 0) {
      int cc = bm_next(bmU, idx + 1, cc_limit);
      if (cc < cc_limit) { idx = cc; return; }
      kind = 1; idx = -1;
    }
    if (kind == 1) {
      int vt = idx + 1;
      if (vt < n_vt && (int64_t)vidx_h[64 * vt] <= last_pos) { idx = vt; return; }
    }
    kind = 2; idx = 0;
  };
  // key index that tile row r comes from (general path)
  auto src_row = [&](int kind, int idx, int r) -> int64_t {
    if (kind == 0) {
      int64_t j = (int64_t)(m0 - (idx - (NQB - 1))) * 64 + r;
      return j < n_k ? j : n_k - 1;
    }
    int pos = 64 * idx + r;
    return pos < vcnt ? (int64_t)vidx_h[pos] : 0;
  };

  // ---- staging: global -> registers -> LDS ------------------------------------------------
  // chunk x = tid + e NT of a tile: row x / DCH, 16-byte chunk x % DCH
  uint32_t koff[CPT], voff[CPT];  // byte offsets inside a contiguous 64-key block
#pragma unroll
  for (int e = 0; e < CPT; ++e) {
    const int x = tid + e * NT, r = x / DCH, ch = x % DCH;
    koff[e] = (uint32_t)(r * a.k_stride_tok * 2 + ch * 16);
    voff[e] = (uint32_t)(r * a.v_stride_tok * 2 + ch * 16);
  }
  u32x4 kst[CPT], vst[CPT];
  int32_t my_vidx = 0;
  auto load_tile = [&](int kind, int idx) {
    if (kind == 0) {
      const int64_t j0 = (int64_t)(m0 - (idx - (NQB - 1))) * 64;
      if (j0 + 64 <= n_k) {  // whole block in range: one uniform base + per-thread 32-bit offsets
        const char* kt = (const char*)kbase + j0 * a.k_stride_tok * 2;
        const char* vt = (const char*)vbase + j0 * a.v_stride_tok * 2;
#pragma unroll
        for (int e = 0; e < CPT; ++e) kst[e] = *(const u32x4*)(kt + koff[e]);
#pragma unroll
        for (int e = 0; e < CPT; ++e) vst[e] = *(const u32x4*)(vt + voff[e]);
        return;
      }
    }
#pragma unroll
    for (int e = 0; e < CPT; ++e) {
      const int x = tid + e * NT, r = x / DCH, ch = x % DCH;
      const int64_t j = src_row(kind, idx, r);
      kst[e] = *(const u32x4*)(kbase + j * a.k_stride_tok + ch * 8);
      vst[e] = *(const u32x4*)(vbase + j * a.v_stride_tok + ch * 8);
    }
    if (kind == 1 && tid < 64) my_vidx = (int32_t)src_row(kind, idx, tid);
  };
  auto store_tile = [&](int buf, int kind) {
#pragma unroll
    for (int e = 0; e < CPT; ++e) {
      const int x = tid + e * NT, r = x / DCH, ch = x % DCH;
      *(u32x4*)&Ks[buf * KBUF + r * KS + ch * 8] = kst[e];
      *(u32x4*)&Vs[buf * VBUF + r * VR + ch * 8] = vst[e];
    }
    if (kind == 1 && tid < 64) vidx_s[buf * 64 + tid] = my_vidx;
  };

  // per-lane LDS element offsets of the MFMA operands
  const int k_lane = (lane & 31) * KS + 8 * hh;  // K rows as A operand of S^T = K Q^T
  // V^T operand through the transposing LDS read: inside each 16-lane group, lane L supplies
  // the address of V[J0 + L/4][D0 + 4 (L%4) .. +3] and receives V[J0 .. J0+3][D0 + L]
  const int v_lane = (((lane & 15) >> 2) + 4 * hh) * VR + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);

  auto qk_step = [&](f32x16& acc, const __bf16* kb, int jb, int st) {
    const bf16x8 ka = *(const bf16x8*)&kb[k_lane + 32 * jb * KS + 16 * st];
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[st], acc, 0, 0, 0);
  };
  // keys of MFMA k-slots 8 hh + 0..7 in step tt of key block jb: 32 jb + 16 tt + 8 (e/4) + 4 hh + e%4
  auto pv_step = [&](const __bf16* vb, const bf16x8 pb, int jb, int tt, int db) {
    typedef bf16x4 __attribute__((address_space(3))) * lds_b4;
    const __bf16* p0 = &vb[v_lane + (32 * jb + 16 * tt) * VR + 32 * db];
    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_b4)(p0));
    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_b4)(p0 + 8 * VR));
    const bf16x8 va = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb, oacc[db], 0, 0, 0);
  };
  auto to_bf16 = [&](const f32x16& sv, int tt) -> bf16x8 {
    f32x8 pf;
#pragma unroll
    for (int x = 0; x < 8; ++x) pf[x] = sv[8 * tt + x];
    return __builtin_convertvector(pf, bf16x8);
  };
  // running-max update with the maximum of a block of scores (base-2 domain).  When some row's
  // maximum grows, everything already expressed relative to the old maximum is rescaled: the
  // row sum, O, and `pend` (probabilities computed but not yet multiplied into O) if has_pend.
  auto update_max_impl = [&](float mx, f32x16& pend, const bool has_pend) -> float {
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx * a.scale_log2);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
    m_run = m_new;
    if (__any(alpha != 1.0f)) {
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int x = 0; x < 16; ++x) oacc[db][x] *= alpha;
      if (has_pend) {
#pragma unroll
        for (int x = 0; x < 16; ++x) pend[x] *= alpha;
      }
    }
    return m_use;
  };
  auto block_max = [&](const f32x16& sv) -> float {
    float mx = sv[0];
#pragma unroll
    for (int x = 1; x < 16; ++x) mx = fmaxf(mx, sv[x]);
    return mx;
  };
  auto exp_block = [&](f32x16& sv, float m_use) {
    float ps = 0.f;
#pragma unroll
    for (int x = 0; x < 16; ++x) {
      const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[x], a.scale_log2, -m_use));
      sv[x] = p;
      ps += p;
    }
    l_run += ps;
  };

  // ---- prologue: tile 0 -> LDS buffer 0, tile 1 -> registers ---------------------------------
  int cur_kind = 0, cur_idx = -1;
  advance(cur_kind, cur_idx);
  if (cur_kind != 2) {
    load_tile(cur_kind, cur_idx);
    store_tile(0, cur_kind);
  }
  int nxt_kind = cur_kind, nxt_idx = cur_idx;
  if (cur_kind != 2) {
    advance(nxt_kind, nxt_idx);
    if (nxt_kind != 2) load_tile(nxt_kind, nxt_idx);
  }
  __syncthreads();
  int buf = 0;

  while (cur_kind != 2) {
    const __bf16* kb = Ks + buf * KBUF;
    const __bf16* vb = Vs + buf * VBUF;
    // ---- does this wave take part, and with which element mask? ----------------------
    bool part = wave_valid;
    bool diag = false;            // slash tile on the query block's own diagonal
    uint64_t vmask = ~0ull;       // vertical tile: keys this query block may use
    uint64_t dmask = 0;           // vertical tile: keys inside the query block's own key block
    if (cur_kind == 0) {
      const int ad = cur_idx - (NQB - 1) + t;  // block diagonal of (query block t, this key block)
      part = part && ad >= 0 && bm_test(bmA, ad);
      diag = ad == 0;
    } else {
      const int pos = 64 * cur_idx + lane;
      const int j = vidx_s[buf * 64 + lane];
      const int ad = (m0 + t) - (j >> 6);
      const bool ok = pos < vcnt && ad >= 0 && !bm_test(bmA, ad);
      vmask = __ballot(ok);
      dmask = __ballot(ok && ad == 0);
      part = part && vmask != 0;
    }
    const bool masked = diag || cur_kind == 1;

    f32x16 s[2];
    if (part) {
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int x = 0; x < 16; ++x) s[jb][x] = 0.f;
      if (!masked) {
        // -------- fast path: the two 32-key halves are software-pipelined --------------
        // S0; first half of S1 ahead of the max of S0; exp(S0) under the rest of S1;
        // PV(0) under exp(S1); PV(1) after the staging below.
#pragma unroll
        for (int st = 0; st < DSTEPS; ++st) qk_step(s[0], kb, 0, st);
#pragma unroll
        for (int st = 0; st < DSTEPS / 2; ++st) qk_step(s[1], kb, 1, st);
        const float mu0 = update_max_impl(block_max(s[0]), s[0], false);
#pragma unroll
        for (int st = DSTEPS / 2; st < DSTEPS; ++st) qk_step(s[1], kb, 1, st);
        exp_block(s[0], mu0);
        // P0 is relative to the old maximum: if S1 raises it, P0 is rescaled with O before PV(0)
        const float mu1 = update_max_impl(block_max(s[1]), s[0], true);
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
          const bf16x8 pb = to_bf16(s[0], tt);
#pragma unroll
          for (int db = 0; db < DB; ++db) pv_step(vb, pb, 0, tt, db);
        }
        exp_block(s[1], mu1);
      } else {
        // -------- masked tile (own diagonal block, or gathered columns): plain order ------
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
          for (int st = 0; st < DSTEPS; ++st) qk_step(s[jb], kb, jb, st);
        // element x of block jb is key r = 32 jb + 8 (x/4) + 4 hh + (x%4) of the tile
        if (diag) {
#pragma unroll
          for (int jb = 0; jb < 2; ++jb)
#pragma unroll
            for (int x = 0; x < 16; ++x) {
              const int r = 32 * jb + 8 * (x >> 2) + 4 * hh + (x & 3);
              if (r > il) s[jb][x] = -INFINITY;
            }
        } else {
#pragma unroll
          for (int jb = 0; jb < 2; ++jb) {
            const uint32_t vb_ = (uint32_t)(vmask >> (32 * jb + 4 * hh));
            const uint32_t db_ = (uint32_t)(dmask >> (32 * jb + 4 * hh));
#pragma unroll
            for (int x = 0; x < 16; ++x) {
              const int bit = 8 * (x >> 2) + (x & 3);
              bool ok = (vb_ >> bit) & 1u;
              if (dmask != 0 && ((db_ >> bit) & 1u)) {
                const int r = 32 * jb + 8 * (x >> 2) + 4 * hh + (x & 3);
                ok = ok && (vidx_s[buf * 64 + r] & 63) <= il;
              }
              if (!ok) s[jb][x] = -INFINITY;
            }
          }
        }
        const float mu = update_max_impl(fmaxf(block_max(s[0]), block_max(s[1])), s[0], false);
        exp_block(s[0], mu);
        exp_block(s[1], mu);
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
          const bf16x8 pb = to_bf16(s[0], tt);
#pragma unroll
          for (int db = 0; db < DB; ++db) pv_step(vb, pb, 0, tt, db);
        }
      }
    }

    // ---- staging: next tile registers -> other LDS buffer; tile after next -> registers ----
    int nn_kind = nxt_kind, nn_idx = nxt_idx;
    if (nxt_kind != 2) {
      store_tile(buf ^ 1, nxt_kind);
      advance(nn_kind, nn_idx);
      if (nn_kind != 2) load_tile(nn_kind, nn_idx);
    }

    if (part) {
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        const bf16x8 pb = to_bf16(s[1], tt);
#pragma unroll
        for (int db = 0; db < DB; ++db) pv_step(vb, pb, 1, tt, db);
      }
    }
    __syncthreads();
    cur_kind = nxt_kind; cur_idx = nxt_idx;
    nxt_kind = nn_kind; nxt_idx = nn_idx;
    buf ^= 1;
  }

  // ---- normalise and store ------------------------------------------------------------------
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
  if (row < a.q_len) {
    __bf16* op = a.out + row * a.o_stride_tok + (int64_t)h * a.o_stride_head;
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
      a.lse[(int64_t)h * a.q_len + row] =
          l_tot > 0.f ? (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
  }
}

// ---------------------------------------------------------------------------------------------
// Bitmaps of block diagonals from the selected slash offsets (one workgroup per head).
// Offset o crosses, inside a 64-aligned query block, the key blocks of diagonals floor(o/64)
// and, when o is not a multiple of 64, floor(o/64) + 1.
// ---------------------------------------------------------------------------------------------
template <int NQB>
__global__ __launch_bounds__(256) void k_build_bitmaps(const int32_t* s_idx, const int32_t* s_cnt,
                                                       int32_t s_budget, int dense, int n_blk,
                                                       int n_words, uint32_t* bm_a, uint32_t* bm_u) {
  const int h = blockIdx.x;
  uint32_t* A = bm_a + (int64_t)h * n_words;
  uint32_t* U = bm_u + (int64_t)h * n_words;
  for (int w = threadIdx.x; w < n_words; w += blockDim.x) {
    uint32_t x = 0;
    if (dense) {
      const int lo = w * 32;
      if (lo + 32 <= n_blk) x = ~0u;
      else if (lo < n_blk) x = (1u << (n_blk - lo)) - 1u;
    }
    A[w] = x;
  }
  __syncthreads();
  if (!dense) {
    const int cnt = s_cnt[h];
    const int32_t* so = s_idx + (int64_t)h * s_budget;
    for (int i = threadIdx.x; i < cnt; i += blockDim.x) {
      const int o = so[i], ad = o >> 6;
      if (ad < n_blk) atomicOr(&A[ad >> 5], 1u << (ad & 31));
      if ((o & 63) && ad + 1 < n_blk) atomicOr(&A[(ad + 1) >> 5], 1u << ((ad + 1) & 31));
    }
    __syncthreads();
  }
  // U bit cc = OR of A bits cc-(NQB-1) .. cc
  for (int w = threadIdx.x; w < n_words; w += blockDim.x) {
    const uint32_t cur = A[w], prev = w ? A[w - 1] : 0u;
    uint32_t u = cur;
#pragma unroll
    for (int sft = 1; sft < NQB; ++sft) u |= (cur << sft) | (prev >> (32 - sft));
    U[w] = u;
  }
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
hipError_t launch_build_bitmaps(const vs_params& p, const int32_t* s_idx, const int32_t* s_cnt,
                                bool dense, uint32_t* bm_a, uint32_t* bm_u, hipStream_t st) {
  const int64_t n_k = p.q_start + p.q_len;
  const int n_blk = (int)ceil_div(n_k, kBlock), n_words = (int)bitmap_words(n_k);
  const int heads = dense ? 1 : p.n_q_heads;
  hipLaunchKernelGGL((k_build_bitmaps<kAttnQBlocks>), dim3(heads), dim3(256), 0, st, s_idx, s_cnt,
                     p.slash_budget, dense ? 1 : 0, n_blk, n_words, bm_a, bm_u);
  return hipGetLastError();
}

hipError_t launch_attention(const vs_params& p, const void* q, const void* k, const void* v,
                            const int32_t* v_idx, const int32_t* v_cnt, bool dense,
                            const uint32_t* bm_a, const uint32_t* bm_u, void* out, float* lse,
                            hipStream_t st) {
  constexpr int NQB = kAttnQBlocks;
  AttnArgs a;
  a.q = (const __bf16*)q; a.k = (const __bf16*)k; a.v = (const __bf16*)v;
  a.out = (__bf16*)out; a.lse = lse;
  a.q_stride_tok = p.q_stride_tok; a.q_stride_head = p.q_stride_head;
  a.k_stride_tok = p.k_stride_tok; a.k_stride_head = p.k_stride_head;
  a.v_stride_tok = p.v_stride_tok; a.v_stride_head = p.v_stride_head;
  a.o_stride_tok = p.o_stride_tok; a.o_stride_head = p.o_stride_head;
  a.bm_a = bm_a; a.bm_u = bm_u;
  a.bm_stride = dense ? 0 : bitmap_words(p.q_start + p.q_len);
  a.v_idx = dense ? nullptr : v_idx; a.v_cnt = dense ? nullptr : v_cnt;
  a.v_budget = p.vertical_budget;
  a.n_q_heads = p.n_q_heads; a.n_kv_heads = p.n_kv_heads; a.group = p.n_q_heads / p.n_kv_heads;
  a.n_qtiles = (int)ceil_div(p.q_len, 64 * NQB);
  a.q_len = p.q_len; a.q_start = p.q_start;
  a.scale_log2 = p.softmax_scale * kLog2e;
  const int64_t groups = (int64_t)a.n_qtiles * p.n_kv_heads;
  const int64_t blocks = ceil_div(groups, 8) * 8 * a.group;
  // more than 64 KiB of LDS per workgroup needs an explicit opt-in, once per kernel
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attention<128, NQB>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, attn_lds_bytes<128>());
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attention<64, NQB>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, attn_lds_bytes<64>());
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  if (p.head_dim == 128)
    hipLaunchKernelGGL((k_attention<128, NQB>), dim3((unsigned)blocks), dim3(128 * NQB),
                       attn_lds_bytes<128>(), st, a);
  else
    hipLaunchKernelGGL((k_attention<64, NQB>), dim3((unsigned)blocks), dim3(128 * NQB),
                       attn_lds_bytes<64>(), st, a);
  return hipGetLastError();
}

hipError_t launch_count_tiles(const vs_params& p, const int32_t* v_idx, const int32_t* v_cnt,
                              const uint32_t* bm_a, int64_t* tiles, hipStream_t st) {
  hipLaunchKernelGGL(k_count_tiles, dim3(p.n_q_heads), dim3(256), 0, st, v_idx, v_cnt,
                     p.vertical_budget, bm_a, (int)bitmap_words(p.q_start + p.q_len), p.q_start,
                     p.q_len, tiles);
  return hipGetLastError();
}

}  // namespace vs
