// Selection of the vertical and slash lines (section 5.2, MInference paragraph: critical
// tokens are chosen by the vertical-slash pattern with a per-head count of vertical and
// diagonal lines).  One workgroup per (head, kind) problem: exact top-k of up to 2^31 fp32
// scores without sorting.
//   1. forced entries (the lowest `keep` indices) are taken first;
//   2. a most-significant-digit radix select (4 x 8 bits on an order-preserving integer image
//      of the float) finds the threshold key T and how many entries equal to T are needed;
//   3. one ordered compaction pass emits indices in ascending order: every key > T, and the
//      lowest-index keys == T (ties go to the lower index).  Ranks come from wave ballots and
//      a 16-entry cross-wave scan, all integer, so the result is exact and deterministic.
#include "vs_common.h"

namespace vs {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelItems = 8;  // elements per lane per compaction step

__device__ __forceinline__ uint32_t order_key(float x) {
  const uint32_t b = __float_as_uint(x);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

struct SelArgs {
  const float* vscore;
  const float* sscore;
  int64_t n;  // n_k
  int32_t v_budget, s_budget, keep_v, keep_s;  // budgets: row lengths of the outputs (maxima)
  const int32_t* v_budget_h;  // optional per-head budgets (clamped to 1 .. maximum), else null
  const int32_t* s_budget_h;
  int32_t* v_idx;
  int32_t* v_cnt;
  int32_t* s_idx;
  int32_t* s_cnt;
};

__global__ __launch_bounds__(kSelThreads) void k_select(const SelArgs a) {
  const int h = blockIdx.x, kind = blockIdx.y;
  const int64_t n = a.n;
  const float* sc = (kind ? a.sscore : a.vscore) + (int64_t)h * n;
  const int row_len = kind ? a.s_budget : a.v_budget;
  const int32_t* per_head = kind ? a.s_budget_h : a.v_budget_h;
  int budget = row_len;
  if (per_head) {
    budget = per_head[h];
    budget = budget < 1 ? 1 : (budget > row_len ? row_len : budget);
  }
  const int keep = kind ? a.keep_s : a.keep_v;
  int32_t* out = (kind ? a.s_idx : a.v_idx) + (int64_t)h * row_len;
  const int k = budget < n ? budget : (int)n;
  const int f = keep < k ? keep : k;  // forced entries 0..f-1
  const int kp = k - f;               // still to choose among indices f..n-1

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  // 16 copies of the 256-bin histogram, copy = lane % 16 in consecutive banks: the top digits of
  // real scores crowd into a few bins, and 64 lanes adding to one address would serialise
  __shared__ uint32_t hist16[256 * 16];
  __shared__ uint32_t hist[256];
  __shared__ uint32_t sh_prefix, sh_krem;
  __shared__ uint32_t wtot[2][kSelWaves][2];

  for (int t = tid; t < row_len; t += kSelThreads) {
    if (t < f) out[t] = t;
    else if (t >= k) out[t] = -1;
  }
  if (tid == 0) (kind ? a.s_cnt : a.v_cnt)[h] = k;
  if (kp == 0) return;

  // ---- radix select: threshold key T = kp-th largest key among candidates ------------------
  uint32_t prefix = 0, krem = (uint32_t)kp;
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    const uint32_t himask = pass == 0 ? 0u : (0xFFFFFFFFu << (shift + 8));
    for (int x = tid; x < 256 * 16; x += kSelThreads) hist16[x] = 0;
    __syncthreads();
    // kSelItems independent loads per thread in flight (the pass is latency-bound otherwise)
    for (int64_t base = f; base < n; base += (int64_t)kSelThreads * kSelItems) {
      uint32_t key[kSelItems];
      bool ok[kSelItems];
#pragma unroll
      for (int e = 0; e < kSelItems; ++e) {
        const int64_t i = base + (int64_t)e * kSelThreads + tid;
        ok[e] = i < n;
        key[e] = ok[e] ? order_key(sc[i]) : 0u;
      }
#pragma unroll
      for (int e = 0; e < kSelItems; ++e)
        if (ok[e] && (key[e] & himask) == prefix)
          atomicAdd(&hist16[(((key[e] >> shift) & 255u) << 4) | (lane & 15)], 1u);
    }
    __syncthreads();
    if (tid < 256) {
      uint32_t c = 0;
#pragma unroll
      for (int x = 0; x < 16; ++x) c += hist16[(tid << 4) | x];
      hist[tid] = c;
    }
    __syncthreads();
    if (tid == 0) {
      uint32_t cum = 0;
      int b = 255;
      for (; b > 0; --b) {
        const uint32_t c = hist[b];
        if (cum + c >= krem) break;
        cum += c;
      }
      sh_prefix = prefix | ((uint32_t)b << shift);
      sh_krem = krem - cum;
    }
    __syncthreads();
    prefix = sh_prefix;
    krem = sh_krem;
  }
  const uint32_t T = prefix;
  const uint32_t need_eq = krem;  // >= 1

  // ---- ordered compaction -------------------------------------------------------------------
  uint32_t run_gt = 0, run_eq = 0;  // totals over the chunks already done
  const uint64_t lt_mask = lane == 0 ? 0ull : (~0ull >> (64 - lane));
  int par = 0;
  for (int64_t base = f; base < n; base += (int64_t)kSelThreads * kSelItems, par ^= 1) {
    uint64_t bg[kSelItems], be[kSelItems];
    uint32_t tg = 0, te = 0;
#pragma unroll
    for (int e = 0; e < kSelItems; ++e) {
      const int64_t i = base + (int64_t)wv * (64 * kSelItems) + e * 64 + lane;
      uint32_t key = 0;
      if (i < n) key = order_key(sc[i]);
      bg[e] = __ballot(i < n && key > T);
      be[e] = __ballot(i < n && key == T);
      tg += __popcll(bg[e]);
      te += __popcll(be[e]);
    }
    if (lane == 0) { wtot[par][wv][0] = tg; wtot[par][wv][1] = te; }
    __syncthreads();
    uint32_t gt_before = run_gt, eq_before = run_eq, cg = 0, ce = 0;
    for (int w = 0; w < kSelWaves; ++w) {
      const uint32_t g_ = wtot[par][w][0], e_ = wtot[par][w][1];
      if (w < wv) { gt_before += g_; eq_before += e_; }
      cg += g_; ce += e_;
    }
#pragma unroll
    for (int e = 0; e < kSelItems; ++e) {
      const int64_t i = base + (int64_t)wv * (64 * kSelItems) + e * 64 + lane;
      const uint32_t gr = gt_before + __popcll(bg[e] & lt_mask);
      const uint32_t er = eq_before + __popcll(be[e] & lt_mask);
      const bool is_g = (bg[e] >> lane) & 1ull, is_e = (be[e] >> lane) & 1ull;
      if (is_g) out[f + gr + (er < need_eq ? er : need_eq)] = (int32_t)i;
      else if (is_e && er < need_eq) out[f + gr + er] = (int32_t)i;
      gt_before += __popcll(bg[e]);
      eq_before += __popcll(be[e]);
    }
    run_gt += cg;
    run_eq += ce;
    if (run_gt + (run_eq < need_eq ? run_eq : need_eq) >= (uint32_t)kp) break;
  }
}

size_t select_ws_bytes(const vs_params&) { return 0; }

hipError_t launch_select(const vs_params& p, const float* vscore, const float* sscore,
                         const int32_t* v_budget_h, const int32_t* s_budget_h,
                         int32_t* v_idx, int32_t* v_cnt, int32_t* s_idx, int32_t* s_cnt, void*,
                         hipStream_t st) {
  SelArgs a;
  a.vscore = vscore; a.sscore = sscore; a.n = p.q_start + p.q_len;
  a.v_budget = p.vertical_budget; a.s_budget = p.slash_budget;
  a.keep_v = p.keep_first_cols; a.keep_s = p.keep_local_band;
  a.v_budget_h = v_budget_h; a.s_budget_h = s_budget_h;
  a.v_idx = v_idx; a.v_cnt = v_cnt; a.s_idx = s_idx; a.s_cnt = s_cnt;
  hipLaunchKernelGGL(k_select, dim3(p.n_q_heads, 2), dim3(kSelThreads), 0, st, a);
  return hipGetLastError();
}

// ---- sparsity refinement ("Sparsity refinement" paragraph and Algorithm 1) --------------------
// recall[h] = mean over the chunk's rows of exp(lse_sparse - lse_full); a row without any
// selected key counts 0.  One workgroup per head, fixed reduction tree.
__global__ __launch_bounds__(256) void k_recall(const float* lse_sparse, const float* lse_full, int64_t rows,
                                                float* recall) {
  const int h = blockIdx.x, tid = threadIdx.x;
  const float* ls = lse_sparse + (int64_t)h * rows;
  const float* lf = lse_full + (int64_t)h * rows;
  float acc = 0.f;
  for (int64_t i = tid; i < rows; i += 256) {
    const float r = __expf(ls[i] - lf[i]);
    acc += (r == r && r <= 3.0e38f) ? r : 0.f;
  }
  __shared__ float part[256];
  part[tid] = acc;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (tid < w) part[tid] += part[tid + w];
    __syncthreads();
  }
  if (tid == 0) recall[h] = rows > 0 ? part[0] / (float)rows : 0.f;
}

// One pass of Algorithm 1 over the heads: a head below the threshold gets dv / ds more lines.
__global__ __launch_bounds__(256) void k_refine(const float* recall, float threshold, int32_t dv, int32_t ds,
                                                int32_t v_max, int32_t s_max, int n_heads,
                                                int32_t* v_budget, int32_t* s_budget, int32_t* changed) {
  __shared__ int cnt;
  if (threadIdx.x == 0) cnt = 0;
  __syncthreads();
  for (int h = threadIdx.x; h < n_heads; h += 256) {
    if (recall[h] < threshold) {
      int nv = v_budget[h] + dv, ns = s_budget[h] + ds;
      nv = nv > v_max ? v_max : nv;
      ns = ns > s_max ? s_max : ns;
      if (nv != v_budget[h] || ns != s_budget[h]) atomicAdd(&cnt, 1);
      v_budget[h] = nv;
      s_budget[h] = ns;
    }
  }
  __syncthreads();
  if (threadIdx.x == 0 && changed) *changed = cnt;
}

hipError_t launch_recall(const vs_params& p, const float* lse_sparse, const float* lse_full, float* recall,
                         hipStream_t st) {
  hipLaunchKernelGGL(k_recall, dim3(p.n_q_heads), dim3(256), 0, st, lse_sparse, lse_full, (int64_t)p.q_len, recall);
  return hipGetLastError();
}

hipError_t launch_refine(const vs_params& p, const float* recall, float threshold, int32_t dv, int32_t ds,
                         int32_t* v_budget, int32_t* s_budget, int32_t* changed, hipStream_t st) {
  hipLaunchKernelGGL(k_refine, dim3(1), dim3(256), 0, st, recall, threshold, dv, ds, p.vertical_budget,
                     p.slash_budget, p.n_q_heads, v_budget, s_budget, changed);
  return hipGetLastError();
}

}  // namespace vs
