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

template <int D, int NQB>
__global__ __launch_bounds__(128 * NQB, 2) void k_attention(const AttnArgs a) {
  constexpr int NT = 128 * NQB;        // threads
  constexpr int KS = D + 8;            // LDS row stride of K tile [64][D], elements
  constexpr int VS = 64 + 8;           // LDS row stride of V^T tile [D][64], elements
  constexpr int DCH = D / 8;           // 16-byte chunks per row
  constexpr int DSTEPS = D / 16;       // MFMA k-steps of QK^T
  constexpr int DB = D / 32;           // 32-row blocks of O^T
  constexpr int KPT = 64 * DCH / NT;   // K chunks per thread
  constexpr int VUNITS = 16 * DCH;     // (4 keys x 8 dims) register tiles of V
  constexpr int VPT = (VUNITS + NT - 1) / NT;
  static_assert(64 * DCH % NT == 0, "K tile must divide over the threads");

  __shared__ __attribute__((aligned(16))) __bf16 Ks[64 * KS];
  __shared__ __attribute__((aligned(16))) __bf16 Vt[D * VS];
  __shared__ int32_t vidx_s[64];

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
  int cur_kind = 0, cur_idx = -1;
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

  // key index that tile row r comes from
  auto src_row = [&](int kind, int idx, int r) -> int64_t {
    if (kind == 0) {
      int64_t j = (int64_t)(m0 - (idx - (NQB - 1))) * 64 + r;
      return j < n_k ? j : n_k - 1;
    }
    int pos = 64 * idx + r;
    return pos < vcnt ? (int64_t)vidx_h[pos] : 0;
  };

  u32x4 kst[KPT];
  u32x4 vst[VPT][4];
  int32_t my_vidx = 0;
  auto load_tile = [&](int kind, int idx) {
#pragma unroll
    for (int e = 0; e < KPT; ++e) {
      const int x = tid + e * NT, r = x / DCH, ch = x % DCH;
      kst[e] = *(const u32x4*)(kbase + src_row(kind, idx, r) * a.k_stride_tok + ch * 8);
    }
#pragma unroll
    for (int e = 0; e < VPT; ++e) {
      const int x = tid + e * NT;
      if (x < VUNITS) {
        const int jq = x & 15, ch = x >> 4;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr)
          vst[e][rr] = *(const u32x4*)(vbase + src_row(kind, idx, 4 * jq + rr) * a.v_stride_tok + ch * 8);
      }
    }
    if (kind == 1 && tid < 64) my_vidx = (int32_t)src_row(kind, idx, tid);
  };
  auto store_tile = [&](int kind) {
#pragma unroll
    for (int e = 0; e < KPT; ++e) {
      const int x = tid + e * NT, r = x / DCH, ch = x % DCH;
      *(u32x4*)&Ks[r * KS + ch * 8] = kst[e];
    }
#pragma unroll
    for (int e = 0; e < VPT; ++e) {
      const int x = tid + e * NT;
      if (x < VUNITS) {
        const int jq = x & 15, ch = x >> 4;
        // key quad jq = [jb t u h] is stored at slot quad [jb t h u]: a lane's 8 PV keys are contiguous
        const int sq = (jq & 12) | ((jq & 1) << 1) | ((jq >> 1) & 1);
#pragma unroll
        for (int e2 = 0; e2 < 8; ++e2) {
          const int w = e2 >> 1;
          const uint32_t sel = (e2 & 1) ? 0x07060302u : 0x05040100u;
          u32x2 pk;
          pk[0] = __builtin_amdgcn_perm(vst[e][1][w], vst[e][0][w], sel);
          pk[1] = __builtin_amdgcn_perm(vst[e][3][w], vst[e][2][w], sel);
          *(u32x2*)&Vt[(ch * 8 + e2) * VS + 4 * sq] = pk;
        }
      }
    }
    if (kind == 1 && tid < 64) vidx_s[tid] = my_vidx;
  };

  advance(cur_kind, cur_idx);
  if (cur_kind != 2) load_tile(cur_kind, cur_idx);

  while (cur_kind != 2) {
    store_tile(cur_kind);
    __syncthreads();
    int nxt_kind = cur_kind, nxt_idx = cur_idx;
    advance(nxt_kind, nxt_idx);
    if (nxt_kind != 2) load_tile(nxt_kind, nxt_idx);

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
      const int j = vidx_s[lane];
      const int ad = (m0 + t) - (j >> 6);
      const bool ok = pos < vcnt && ad >= 0 && !bm_test(bmA, ad);
      vmask = __ballot(ok);
      dmask = __ballot(ok && ad == 0);
      part = part && vmask != 0;
    }

    if (part) {
      // ---- S^T = K Q^T : two 32-key blocks --------------------------------------------
      f32x16 s[2];
#pragma unroll
      for (int jb = 0; jb < 2; ++jb) {
#pragma unroll
        for (int x = 0; x < 16; ++x) s[jb][x] = 0.f;
#pragma unroll
        for (int st = 0; st < DSTEPS; ++st) {
          const bf16x8 ka = *(const bf16x8*)&Ks[(32 * jb + (lane & 31)) * KS + 16 * st + 8 * hh];
          s[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[st], s[jb], 0, 0, 0);
        }
      }
      // element x of block jb is key r = 32 jb + 8 (x/4) + 4 hh + (x%4) of the tile
      if (diag) {
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
          for (int x = 0; x < 16; ++x) {
            const int r = 32 * jb + 8 * (x >> 2) + 4 * hh + (x & 3);
            if (r > il) s[jb][x] = -INFINITY;
          }
      } else if (cur_kind == 1) {
#pragma unroll
        for (int jb = 0; jb < 2; ++jb) {
          const uint32_t vb = (uint32_t)(vmask >> (32 * jb + 4 * hh));
          const uint32_t db_ = (uint32_t)(dmask >> (32 * jb + 4 * hh));
#pragma unroll
          for (int x = 0; x < 16; ++x) {
            const int bit = 8 * (x >> 2) + (x & 3);
            bool ok = (vb >> bit) & 1u;
            if (dmask != 0 && ((db_ >> bit) & 1u)) {
              const int r = 32 * jb + 8 * (x >> 2) + 4 * hh + (x & 3);
              ok = ok && (vidx_s[r] & 63) <= il;
            }
            if (!ok) s[jb][x] = -INFINITY;
          }
        }
      }
      // ---- online softmax (base 2) ----------------------------------------------------
      float mx = s[0][0];
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int x = 0; x < 16; ++x) mx = fmaxf(mx, s[jb][x]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run, mx * a.scale_log2);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
      m_run = m_new;
      l_run *= alpha;
      if (__any(alpha != 1.0f)) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int x = 0; x < 16; ++x) oacc[db][x] *= alpha;
      }
      float psum = 0.f;
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int x = 0; x < 16; ++x) {
          const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[jb][x], a.scale_log2, -m_use));
          s[jb][x] = p;
          psum += p;
        }
      l_run += psum;
      // ---- O^T += V^T P^T ----------------------------------------------------------------
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
          f32x8 pf;
#pragma unroll
          for (int x = 0; x < 8; ++x) pf[x] = s[jb][8 * tt + x];
          const bf16x8 pb = __builtin_convertvector(pf, bf16x8);
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            const bf16x8 va = *(const bf16x8*)&Vt[(32 * db + (lane & 31)) * VS + 32 * jb + 16 * tt + 8 * hh];
            oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb, oacc[db], 0, 0, 0);
          }
        }
    }
    __syncthreads();
    cur_kind = nxt_kind;
    cur_idx = nxt_idx;
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
  if (p.head_dim == 128)
    hipLaunchKernelGGL((k_attention<128, NQB>), dim3((unsigned)blocks), dim3(128 * NQB), 0, st, a);
  else
    hipLaunchKernelGGL((k_attention<64, NQB>), dim3((unsigned)blocks), dim3(128 * NQB), 0, st, a);
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
