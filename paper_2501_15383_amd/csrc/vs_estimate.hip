// Estimation for the vertical-slash pattern (section 5.2, MInference paragraph: attention
// between the last query tokens and all key tokens; chunked-prefill paragraph: the last 64
// tokens of each chunk).  For the W' <= 64 window rows of every head: causal softmax rows
// over all n_k keys, summed along columns (vscore) and along diagonals pos - j (sscore).
//
// Two sweeps over the K cache, both tiled the same way: a workgroup owns one KV head and a
// contiguous range of keys; a wave is (query head of that KV group, half of the window rows),
// so every K tile is fetched from HBM once per sweep for all heads of the group and staged
// in LDS (two buffers, one barrier per tile).
//   sweep A  per-row running (max, sum) over the range -> partials -> k_estimate_combine -> lse
//   sweep B  P = exp2(S * scale*log2e - lse2).  Column sums: the wave of the upper half hands
//            its sums to the wave of the lower half through LDS, which stores them (a column
//            belongs to exactly one workgroup).  Diagonal sums of every 32 x 32 block come
//            from lane rotations and are collected in an LDS strip private to the wave; the
//            two strips of a head are added to the zero-filled global array at the end (at
//            most two workgroups touch one offset, and x + y is commutative), so scores are
//            run-to-run identical.
// bf16 MFMA (32x32x16) with fp32 accumulation; sweep A uses the K Q^T orientation (a lane
// owns one query), sweep B the Q K^T orientation (a lane owns one key).  Both sweeps are
// bound by the exponential (one per score, quarter rate), not by memory.
#include <type_traits>

#include "vs_common.h"

namespace vs {

constexpr int kEstRange = 1024;  // keys per workgroup

struct EstArgs {
  const __bf16* q;
  // Dual Chunk Attention (template parameter DCA; section 5.1 and "Integrating with DCA" in
  // section 5.2): the window rows rotated for the successive-chunk and the inter-chunk pattern
  // (q is the intra-chunk one; same strides), chunk length and local window in tokens
  const __bf16* q_succ;
  const __bf16* q_inter;
  int64_t dca_chunk, dca_window;
  const __bf16* k;
  int64_t q_stride_tok, q_stride_head, k_stride_tok, k_stride_head;
  float* vscore;
  float* sscore;
  float* lse_lastq;  // optional, natural log
  float* part;       // [Hq][n_ranges][64][2]  (max, sum) in the base-2 scaled domain
  float* lse2;       // [Hq][64] base-2 scaled lse (+inf for rows >= W')
  int32_t n_q_heads, n_kv_heads, group;
  int32_t wp;        // W'
  int32_t n_ranges;
  int32_t n_hb;      // workgroups per (key range, KV head): the heads of a group may be split
  int64_t q_len, n_k, p0;  // p0: position of window row 0
  float scale_log2;
};

template <int D, int NH, int PASS, bool DCA>
__global__ __launch_bounds__(128 * NH, DCA ? 1 : 4) void k_estimate(const EstArgs a) {
  constexpr int NW = 2 * NH, NT = 64 * NW, KS = D + 8, DCH = D / 8, DSTEPS = D / 16;
  constexpr int KPT = (64 * DCH + NT - 1) / NT;
  constexpr int STRIP = kEstRange + 64;
  __shared__ __attribute__((aligned(16))) __bf16 Ks[2][64 * KS];
  __shared__ float strip[PASS == 1 ? NW * STRIP : 1];
  __shared__ float colbuf[PASS == 1 ? 2 * NH * 64 : 1];
  __shared__ __attribute__((aligned(16))) float lse_s[PASS == 1 ? NH * 64 : 4];

  // Workgroups b and b + 8 land on the same XCD (they are dealt to the 8 XCDs in turn) at about
  // the same time.  The n_hb workgroups that share a (key range, KV head) unit are placed that
  // way, so that the second one finds the unit's K rows in the L2 of that XCD:
  //   b = 8 n_hb (unit / 8) + 8 hb + unit % 8
  const int b_lin = blockIdx.x;
  const int unit = (b_lin / (8 * a.n_hb)) * 8 + (b_lin & 7);
  const int hb = (b_lin >> 3) % a.n_hb;
  if (unit >= a.n_ranges * a.n_kv_heads) return;
  const int rng = unit % a.n_ranges, g = unit / a.n_ranges;
  const int tid = threadIdx.x, lane = tid & 63, hh = lane >> 5;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hw = wv >> 1, ib = wv & 1;  // head inside the workgroup, half of the window rows
  const int hin = hb * NH + hw;
  const bool head_ok = hin < a.group;
  const int h = g * a.group + (head_ok ? hin : 0);
  const int64_t ja = (int64_t)rng * kEstRange;
  const int64_t jb_ = ja + kEstRange < a.n_k ? ja + kEstRange : a.n_k;
  const int n_tiles = (int)((jb_ - ja + 63) >> 6);
  const __bf16* kbase = a.k + (int64_t)g * a.k_stride_head;

  // window rows of this wave, as MFMA operand: lane (r = 32 ib + lane%32, hh).  With DCA the
  // operand is one of three rotations of the same rows; q_var says which one is loaded.
  bf16x8 qreg[DSTEPS];
  int q_var = 0;
  auto load_q = [&](int var) {
    const __bf16* qb = a.q;
    if constexpr (DCA) {
      if (var == 1) qb = a.q_succ;
      if (var == 2) qb = a.q_inter;
    }
    int r = 32 * ib + (lane & 31);
    if (r > a.wp - 1) r = a.wp - 1;
    const __bf16* qp = qb + (a.q_len - a.wp + r) * a.q_stride_tok + (int64_t)h * a.q_stride_head + 8 * hh;
#pragma unroll
    for (int st = 0; st < DSTEPS; ++st) qreg[st] = *(const bf16x8*)(qp + 16 * st);
    q_var = var;
  };
  load_q(0);
  // DCA: chunk of the wave's first row, and the position at which its rows enter the next chunk
  const int64_t dca_c = DCA ? a.dca_chunk : 1;
  const int64_t pos_lo = a.p0 + 32 * ib, pos_hi = pos_lo + 31;
  const int64_t cq_lo = DCA ? pos_lo / dca_c : 0, cq_hi = DCA ? pos_hi / dca_c : 0;
  const int64_t dca_bound = (cq_lo + 1) * dca_c;
  // rows of this half at or past row_bound lie in the next chunk (32: none of them)
  const int row_bound = DCA && dca_bound - pos_lo < 32 ? (int)(dca_bound - pos_lo) : 32;
  const int win32 = DCA ? (int)(a.dca_window < (1 << 30) ? a.dca_window : (1 << 30)) : 0;
  // pattern of (row r of this wave's half, key j0 + jrel) for a tile whose keys lie ck_rel chunks
  // after the chunk of the half's first row, and whose first key is dist0 tokens before that row
  auto var_of = [&](int ck_rel, int dist0, int r_in_half, int jrel) -> int {
    const int cq = r_in_half >= row_bound ? 1 : 0;
    if (ck_rel == cq) return 0;
    if (ck_rel == cq - 1 && dist0 + r_in_half - jrel < win32) return 1;
    return 2;
  };

  float* const my_strip = &strip[PASS == 1 ? wv * STRIP : 0];
  if (PASS == 1) {
    for (int x = tid; x < NW * STRIP; x += NT) strip[x] = 0.f;
  }

  // sweep A state: this lane's (max, sum) for query 32 ib + lane%32 over its half of the keys
  float mrun = -INFINITY, lrun = 0.f;
  // sweep B: lse2 of the head's window rows; a lane meets queries 32 ib + 8 (x/4) + 4 hh + (x%4)
  if (PASS == 1) {
    if (ib == 0) lse_s[hw * 64 + lane] = a.lse2[(int64_t)h * 64 + lane];
  }
  const f32x4* const lse_q = (const f32x4*)&lse_s[PASS == 1 ? hw * 64 + 32 * ib + 4 * hh : 0];
  float col_prev = 0.f;  // sweep B, lower half: own column sum of the previous tile, column `lane`

  u32x4 kst[KPT];
  auto load_tile = [&](int tile) {
#pragma unroll
    for (int e = 0; e < KPT; ++e) {
      const int x = tid + e * NT;
      if (KPT * NT == 64 * DCH || x < 64 * DCH) {
        const int r = x / DCH, ch = x % DCH;
        int64_t j = ja + 64 * tile + r;
        if (j > a.n_k - 1) j = a.n_k - 1;
        kst[e] = *(const u32x4*)(kbase + j * a.k_stride_tok + ch * 8);
      }
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int e = 0; e < KPT; ++e) {
      const int x = tid + e * NT;
      if (KPT * NT == 64 * DCH || x < 64 * DCH) {
        const int r = x / DCH, ch = x % DCH;
        *(u32x4*)&Ks[buf][r * KS + ch * 8] = kst[e];
      }
    }
  };
  // column sums of tile `tile` of this head: own half in col_prev, the other half in colbuf
  auto flush_columns = [&](int tile) {
    const int64_t j = ja + 64 * tile + lane;
    const float other = colbuf[((tile & 1) * NH + hw) * 64 + lane];
    if (j < a.n_k) a.vscore[(int64_t)h * a.n_k + j] = col_prev + other;
  };

  int64_t ck = DCA ? ja / dca_c : 0, ck_next = (ck + 1) * dca_c;
  load_tile(0);
  store_tile(0);
  __syncthreads();
  for (int tile = 0; tile < n_tiles; ++tile) {
    const int buf = tile & 1;
    if (tile + 1 < n_tiles) load_tile(tile + 1);
    const int64_t j0 = ja + 64 * tile;
    const bool need_mask = j0 + 63 > a.p0;  // some (row, key) of this tile is acausal

    // DCA: which rotation(s) this wave's rows need against the keys of this tile (all in chunk ck)
    uint32_t need = 1u;
    int ck_rel = 0, dist0 = 0;
    if constexpr (DCA) {
      if (j0 >= ck_next) { ++ck; ck_next += dca_c; }  // chunk of the tile's keys, without a division per tile
      const int64_t rel = ck - cq_lo;  // <= 1 for causal keys; far chunks all count as "earlier than the one before"
      ck_rel = rel < -2 ? -2 : (int)rel;
      const int64_t d0 = pos_lo - j0;  // < 2^31 by the limit on the number of keys
      dist0 = d0 < -(1 << 30) ? -(1 << 30) : (int)d0;
      if (cq_lo == cq_hi) {
        if (ck == cq_lo) need = 1u;
        else if (ck == cq_lo - 1) {
          if (pos_hi - j0 < a.dca_window) need = 2u;              // the largest distance is inside the window
          else if (pos_lo - (j0 + 63) >= a.dca_window) need = 4u;  // the smallest one is outside
          else need = 6u;
        } else need = 4u;
      } else {
        need = ck < cq_lo - 1 ? 4u : 7u;  // rows on both sides of a chunk boundary
      }
      if (head_ok && (need & (need - 1)) == 0) {  // one rotation for the whole tile
        const int var = need == 1u ? 0 : (need == 2u ? 1 : 2);
        if (q_var != var) load_q(var);
      }
    }
    const bool multi = DCA && (need & (need - 1)) != 0;

    if (head_ok) {
      if (PASS == 1 && ib == 0 && tile > 0) flush_columns(tile - 1);
      float col[2] = {0.f, 0.f};
      // a tile whose pairs are of several patterns is taken once per rotation, each pass keeping
      // the pairs of its own pattern (every sum below is additive over the passes)
      // (the body exists twice, so that the common one-rotation tiles carry none of the pattern tests)
      // (... and once more with and without the causal mask, which only the last tiles of the keys need)
      auto blocks = [&](auto masked, auto causal, const int rot) {
      constexpr bool MASKED = decltype(masked)::value;
      constexpr bool CAUSAL = decltype(causal)::value;
#pragma unroll
      for (int jb = 0; jb < 2; ++jb) {
        const __bf16* const kfp = &Ks[buf][(32 * jb + (lane & 31)) * KS + 8 * hh];
        f32x16 s;
#pragma unroll
        for (int x = 0; x < 16; ++x) s[x] = 0.f;
        if (PASS == 0) {
          // D[j][i]: lane = query i, element x = key 32 jb + 8 (x/4) + 4 hh + (x%4)
#pragma unroll
          for (int st = 0; st < DSTEPS; ++st)
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8*)(kfp + 16 * st), qreg[st], s, 0, 0, 0);
          if (MASKED) {
            // this pass holds rotation `rot`: pairs of another pattern are left to their own pass
#pragma unroll
            for (int x = 0; x < 16; ++x)
              if (var_of(ck_rel, dist0, lane & 31, 32 * jb + 8 * (x >> 2) + 4 * hh + (x & 3)) != rot) s[x] = -INFINITY;
          }
          if (CAUSAL) {
            // key j is masked for query r iff j - p0 > r; dr = r - (j0 - p0) - 32 jb - 4 hh
            const int dr = 32 * ib + (lane & 31) - (int)(j0 - a.p0) - 32 * jb - 4 * hh;
#pragma unroll
            for (int x = 0; x < 16; ++x)
              if (8 * (x >> 2) + (x & 3) > dr) s[x] = -INFINITY;
          }
          float mx = s[0];
#pragma unroll
          for (int x = 1; x < 16; ++x) mx = fmaxf(mx, s[x]);
          const float m_new = fmaxf(mrun, mx * a.scale_log2);
          const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
          float acc = lrun * __builtin_amdgcn_exp2f(mrun - m_use);
#pragma unroll
          for (int x = 0; x < 16; ++x)
            acc += __builtin_amdgcn_exp2f(__builtin_fmaf(s[x], a.scale_log2, -m_use));
          lrun = acc;
          mrun = m_new;
        } else {
          // D[i][j]: lane = key j = 32 jb + lane%32, element x = query 32 ib + 8 (x/4) + 4 hh + (x%4)
#pragma unroll
          for (int half = 0; half < 2; ++half) {
            // K operands in two batches, so that only half of them are live at a time
            bf16x8 kf[DSTEPS / 2];
#pragma unroll
            for (int st = 0; st < DSTEPS / 2; ++st) kf[st] = *(const bf16x8*)(kfp + 16 * (st + half * (DSTEPS / 2)));
#pragma unroll
            for (int st = 0; st < DSTEPS / 2; ++st)
              s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qreg[st + half * (DSTEPS / 2)], kf[st], s, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
          }
          // causal mask in 32 bits: key j is masked for query i iff j - p0 > i; dj = j - p0 - 4 hh
          // is compared with the uniform 32 ib + q0 (only tiles at the end of the keys need it)
          const int dj = CAUSAL ? (int)(j0 - a.p0) + 32 * jb + (lane & 31) - 4 * hh : 0;
          // Diagonal sums of this 32 x 32 block without atomics.  Element x of a lane is
          // query q = 8 (x/4) + 4 hh + (x%4) of the block against key t = lane % 32, on block
          // diagonal e = q - t.  Rotating the 32-lane vector of element x by q lanes (inside
          // each half-wave) puts e = -t (no wrap) or e = 32 - t (wrapped) into lane t for
          // every x, so two accumulators per lane collect all 63 diagonals of the block.
          // (all of a lane's elements go into `dall`, the wrapped ones into `dpos` as well: the
          // unwrapped sum is the difference, exact in the lanes that never or always wrap)
          float colsum = 0.f, dall = 0.f, dpos = 0.f;
          const int t4 = (lane & 31) + 4 * hh;
#pragma unroll
          for (int x = 0; x < 16; ++x) {
            const int q0 = 8 * (x >> 2) + (x & 3);
            const f32x4 lse4 = lse_q[2 * (x >> 2)];
            float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[x], a.scale_log2, -lse4[x & 3]));
            if (CAUSAL && dj > 32 * ib + q0) p = 0.f;
            if (MASKED && var_of(ck_rel, dist0, q0 + 4 * hh, 32 * jb + (lane & 31)) != rot) p = 0.f;  // another pass's pair
            colsum += p;
            const int src = ((t4 + q0) & 31) | (lane & 32);
#ifdef VS_X_EST_NODIAG   // timing diagnostic, never defined in the library that ships (results are wrong): no lane rotation
            const float r = p; (void)src;
#else
            const float r = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(src << 2, __builtin_bit_cast(int, p)));
#endif
            const bool wrapped = t4 + q0 >= 32;
            dall += r;
            dpos += wrapped ? r : 0.f;
          }
          float dneg = dall - dpos;
          dneg += __shfl_xor(dneg, 32);
          dpos += __shfl_xor(dpos, 32);
          // strip index of (query i, key jl) is i - jl + (kEstRange - 1); the strip is private
          // to the wave and the 32 addresses of one update are distinct
          if (hh == 0) {
            float* sp = &my_strip[32 * (ib - jb) - 64 * tile + (kEstRange - 1) - (lane & 31)];
            sp[0] += dneg;
            if ((lane & 31) != 0) sp[32] += dpos;
          }
          col[jb] += colsum + __shfl_xor(colsum, 32);
        }
      }
      };
      if (!multi) {
        if (need_mask) blocks(std::false_type{}, std::true_type{}, 0);
        else blocks(std::false_type{}, std::false_type{}, 0);
      } else {
        for (int rot = 0; rot < 3; ++rot) {
          if (!((need >> rot) & 1u)) continue;
          if (q_var != rot) load_q(rot);
          blocks(std::true_type{}, std::true_type{}, rot);
        }
      }
      if (PASS == 1) {
        // every lane now has the sums of columns lane%32 (jb = 0) and 32 + lane%32 (jb = 1)
        const float mine = hh ? col[1] : col[0];  // column `lane` of the tile
        if (ib == 1) colbuf[(buf * NH + hw) * 64 + lane] = mine;
        else col_prev = mine;
      }
    }
    if (tile + 1 < n_tiles) store_tile(buf ^ 1);
    __syncthreads();
  }

  if (!head_ok) return;
  if (PASS == 0) {
    // merge the two key halves of each query, then one partial per (head, range, row)
    const float m2 = __shfl_xor(mrun, 32), l2 = __shfl_xor(lrun, 32);
    const float M = fmaxf(mrun, m2);
    const float Mu = (M == -INFINITY) ? 0.f : M;
    const float L = lrun * __builtin_amdgcn_exp2f(mrun - Mu) + l2 * __builtin_amdgcn_exp2f(m2 - Mu);
    if (hh == 0) {
      float* pp = a.part + (((int64_t)h * a.n_ranges + rng) * 64 + 32 * ib + (lane & 31)) * 2;
      pp[0] = M;
      pp[1] = L;
    }
  } else {
    if (ib == 0) flush_columns(n_tiles - 1);
    // the two strips of the head, added; strip index x <-> offset o = p0 - ja - (kEstRange - 1) + x
    const float* s0 = &strip[(2 * hw) * STRIP];
    const float* s1 = s0 + STRIP;
    const int64_t o0 = a.p0 - ja - (kEstRange - 1);
    for (int x = lane + 64 * ib; x < STRIP; x += 128) {
      const int64_t o = o0 + x;
      const float val = s0[x] + s1[x];
      if (o >= 0 && o < a.n_k && val != 0.f) atomicAdd(&a.sscore[(int64_t)h * a.n_k + o], val);
    }
  }
}

// lse2[h][r] = M + log2(L) over all range partials; rows >= W' get +inf (their P is 0).
// 16 groups of 64 threads each fold every 16th range, then group 0 folds the 16 results: a
// fixed order, so the result is run-to-run identical.
__global__ __launch_bounds__(1024) void k_estimate_combine(const EstArgs a) {
  const int h = blockIdx.x, r = threadIdx.x & 63, grp = threadIdx.x >> 6;
  auto fold = [](float& M, float& L, float m, float l) {
    const float Mn = fmaxf(M, m);
    const float Mu = (Mn == -INFINITY) ? 0.f : Mn;
    L = L * __builtin_amdgcn_exp2f(M - Mu) + l * __builtin_amdgcn_exp2f(m - Mu);
    M = Mn;
  };
  float M = -INFINITY, L = 0.f;
  for (int rg = grp; rg < a.n_ranges; rg += 16) {
    const float* pp = a.part + (((int64_t)h * a.n_ranges + rg) * 64 + r) * 2;
    fold(M, L, pp[0], pp[1]);
  }
  __shared__ float sm[16][64], sl[16][64];
  sm[grp][r] = M;
  sl[grp][r] = L;
  __syncthreads();
  if (grp != 0) return;
  for (int g2 = 1; g2 < 16; ++g2) fold(M, L, sm[g2][r], sl[g2][r]);
  const float l2 = M + __builtin_amdgcn_logf(L);
  a.lse2[(int64_t)h * 64 + r] = r < a.wp ? l2 : INFINITY;
  if (a.lse_lastq && r < a.wp) a.lse_lastq[(int64_t)h * a.wp + r] = l2 * kLn2;
}

__global__ __launch_bounds__(256) void k_fill_zero(float* p, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) p[i] = 0.f;
}

// heads per workgroup (two waves each)
static int pick_waves(int group) {
  const int cand[] = {1, 2, 4, 5, 7, 8};
  for (int c : cand)
    if (c >= group) return c;
  return 8;
}

size_t estimate_ws_bytes(const vs_params& p) {
  const int64_t n_k = p.q_start + p.q_len;
  const int64_t n_ranges = ceil_div(n_k, kEstRange);
  return align_up((size_t)p.n_q_heads * n_ranges * 64 * 2 * sizeof(float), 256) +
         align_up((size_t)p.n_q_heads * 64 * sizeof(float), 256);
}

template <int D, int NH>
static hipError_t launch_est(EstArgs a, int hb, hipStream_t st) {
  a.n_hb = hb;
  const dim3 grid((unsigned)(ceil_div((int64_t)a.n_ranges * a.n_kv_heads, 8) * 8 * hb));
  if (a.dca_chunk > 0) {
    hipLaunchKernelGGL((k_estimate<D, NH, 0, true>), grid, dim3(128 * NH), 0, st, a);
    hipLaunchKernelGGL(k_estimate_combine, dim3(a.n_q_heads), dim3(1024), 0, st, a);
    hipLaunchKernelGGL((k_estimate<D, NH, 1, true>), grid, dim3(128 * NH), 0, st, a);
    return hipGetLastError();
  }
  hipLaunchKernelGGL((k_estimate<D, NH, 0, false>), grid, dim3(128 * NH), 0, st, a);
  hipLaunchKernelGGL(k_estimate_combine, dim3(a.n_q_heads), dim3(1024), 0, st, a);
  hipLaunchKernelGGL((k_estimate<D, NH, 1, false>), grid, dim3(128 * NH), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_estimate(const vs_params& p, const void* q, const DcaArgs* dca, const void* k, float* vscore,
                           float* sscore, float* lse_lastq, void* ws, hipStream_t st) {
  EstArgs a;
  a.q = (const __bf16*)q; a.k = (const __bf16*)k;
  a.q_succ = dca ? (const __bf16*)dca->q_succ : nullptr;
  a.q_inter = dca ? (const __bf16*)dca->q_inter : nullptr;
  a.dca_chunk = dca ? dca->chunk : 0;
  a.dca_window = dca ? dca->window : 0;
  a.q_stride_tok = p.q_stride_tok; a.q_stride_head = p.q_stride_head;
  a.k_stride_tok = p.k_stride_tok; a.k_stride_head = p.k_stride_head;
  a.vscore = vscore; a.sscore = sscore; a.lse_lastq = lse_lastq;
  a.n_q_heads = p.n_q_heads; a.n_kv_heads = p.n_kv_heads; a.group = p.n_q_heads / p.n_kv_heads;
  a.wp = (int32_t)(p.last_q < p.q_len ? p.last_q : p.q_len);
  a.q_len = p.q_len; a.n_k = p.q_start + p.q_len; a.p0 = a.n_k - a.wp;
  a.n_ranges = (int32_t)ceil_div(a.n_k, kEstRange);
  a.scale_log2 = p.softmax_scale * kLog2e;
  a.part = (float*)ws;
  a.lse2 = (float*)((char*)ws + align_up((size_t)p.n_q_heads * a.n_ranges * 64 * 2 * sizeof(float), 256));
  const int64_t n_sc = (int64_t)p.n_q_heads * a.n_k;
  hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)(n_sc / 1024 < 1 ? 1 : (n_sc / 1024 > 8192 ? 8192 : n_sc / 1024))),
                     dim3(256), 0, st, sscore, n_sc);
  // large groups are split over two workgroups: two of them fit a compute unit, and the DCA
  // instantiation needs the registers (the two are placed on one XCD, see the kernel)
  const int nw = pick_waves(a.group > 4 ? (a.group + 1) / 2 : a.group);
  const int hb = (int)ceil_div(a.group, nw);
#define VS_EST_CASE(DD, WW) \
  if (p.head_dim == DD && nw == WW) return launch_est<DD, WW>(a, hb, st);
  VS_EST_CASE(128, 1) VS_EST_CASE(128, 2) VS_EST_CASE(128, 4) VS_EST_CASE(128, 5)
  VS_EST_CASE(128, 7) VS_EST_CASE(128, 8)
  VS_EST_CASE(64, 1) VS_EST_CASE(64, 2) VS_EST_CASE(64, 4) VS_EST_CASE(64, 5)
  VS_EST_CASE(64, 7) VS_EST_CASE(64, 8)
#undef VS_EST_CASE
  return hipErrorInvalidValue;
}

}  // namespace vs
