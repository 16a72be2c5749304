// Selection of the vertical and slash lines (section 5.2, MInference paragraph: critical
// tokens are chosen by the vertical-slash pattern with a per-head count of vertical and
// diagonal lines).  Exact top-k of up to 2^31 fp32 scores per (head, kind) row without sorting:
//   1. forced entries (the lowest `keep` indices) are taken first (k_sel_init);
//   2. a most-significant-digit radix select (4 x 8 bits on an order-preserving integer image
//      of the float) finds the threshold key T and how many entries equal to T are needed.
//      A row is cut into slices, one workgroup each; every workgroup adds its 256-bin
//      histogram to the row's, and the workgroup that finishes last picks the digit
//      (k_sel_hist, once per digit);
//   3. the keys > T and == T of every slice are counted (k_sel_count), and one ordered
//      compaction pass emits indices in ascending order: every key > T, and the lowest-index
//      keys == T (ties go to the lower index).  Ranks come from the slice counts, wave
//      ballots and a 16-entry cross-wave scan (k_sel_write).
// All of it is integer work, so the result is exact and run-to-run identical.
#include <mutex>

#include "vs_common.h"

namespace vs {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelItems = 8;  // elements per lane per step
constexpr int kSelStep = kSelThreads * kSelItems;
constexpr int kSelMaxSlices = 64;
// control block of a row in the workspace, in 32-bit words
constexpr int kWHist = 0;      // [4][256] histogram of every digit
constexpr int kWDone = 1024;   // [4] workgroups done with the digit
constexpr int kWState = 1028;  // [5][2] (prefix, entries still to find) before digit 0..3 and after
constexpr int kWForced = 1038, kWChoose = 1039;
constexpr int kWCount = 1056;  // [slices][2] keys > T, keys == T
constexpr int kSelRowWords = kWCount + 2 * kSelMaxSlices;

__device__ __forceinline__ uint32_t order_key(float x) {
  const uint32_t b = __float_as_uint(x);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

struct SelArgs {
  const float* vscore;
  const float* sscore;
  int64_t n;  // n_k
  int64_t slice_len;
  int32_t n_q_heads;
  int32_t v_budget, s_budget, keep_v, keep_s;  // budgets: row lengths of the outputs (maxima)
  const int32_t* v_budget_h;  // optional per-head budgets (clamped to 1 .. maximum), else null
  const int32_t* s_budget_h;
  int32_t* v_idx;
  int32_t* v_cnt;
  int32_t* s_idx;
  int32_t* s_cnt;
  uint32_t* ws;  // [2 Hq][kSelRowWords]
};

// row = kind * Hq + h
struct SelRow {
  const float* sc;
  int32_t* out;
  uint32_t* w;
  int row_len;
};
__device__ __forceinline__ SelRow sel_row(const SelArgs& a, int row) {
  const int kind = row >= a.n_q_heads, h = row - kind * a.n_q_heads;
  SelRow r;
  r.sc = (kind ? a.sscore : a.vscore) + (int64_t)h * a.n;
  r.row_len = kind ? a.s_budget : a.v_budget;
  r.out = (kind ? a.s_idx : a.v_idx) + (int64_t)h * r.row_len;
  r.w = a.ws + (int64_t)row * kSelRowWords;
  return r;
}

// Forced entries, padding, the count, and a cleared control block.
__global__ __launch_bounds__(256) void k_sel_init(const SelArgs a) {
  const int row = blockIdx.x, kind = row >= a.n_q_heads, h = row - kind * a.n_q_heads;
  const SelRow r = sel_row(a, row);
  const int32_t* per_head = kind ? a.s_budget_h : a.v_budget_h;
  int budget = r.row_len;
  if (per_head) {
    budget = per_head[h];
    budget = budget < 1 ? 1 : (budget > r.row_len ? r.row_len : budget);
  }
  const int keep = kind ? a.keep_s : a.keep_v;
  const int k = budget < a.n ? budget : (int)a.n;
  const int f = keep < k ? keep : k;  // forced entries 0..f-1
  const int kp = k - f;               // still to choose among indices f..n-1
  const int tid = threadIdx.x;
  for (int x = tid; x < kSelRowWords; x += 256) {
    uint32_t v = 0;
    if (x == kWState + 1 || x == kWChoose) v = (uint32_t)kp;
    if (x == kWForced) v = (uint32_t)f;
    r.w[x] = v;
  }
  for (int t = tid; t < r.row_len; t += 256) {
    if (t < f) r.out[t] = t;
    else if (t >= k) r.out[t] = -1;
  }
  if (tid == 0) (kind ? a.s_cnt : a.v_cnt)[h] = k;
}

// One digit of the radix select: threshold key T = kp-th largest key among the candidates.
__global__ __launch_bounds__(kSelThreads) void k_sel_hist(const SelArgs a, const int pass) {
  const SelRow r = sel_row(a, blockIdx.y);
  const uint32_t kp = r.w[kWChoose];
  if (kp == 0) return;
  const int64_t lo = (int64_t)r.w[kWForced] + (int64_t)blockIdx.x * a.slice_len;
  const int64_t hi = lo + a.slice_len < a.n ? lo + a.slice_len : a.n;
  const uint32_t prefix = r.w[kWState + 2 * pass], krem = r.w[kWState + 2 * pass + 1];
  const int tid = threadIdx.x, lane = tid & 63;
  // 16 copies of the 256-bin histogram, copy = lane % 16 in consecutive banks: the top digits of
  // real scores crowd into a few bins, and 64 lanes adding to one address would serialise
  __shared__ uint32_t hist16[256 * 16];
  __shared__ uint32_t hist[256];
  __shared__ bool last;
  const int shift = 24 - 8 * pass;
  const uint32_t himask = pass == 0 ? 0u : (0xFFFFFFFFu << (shift + 8));
  for (int x = tid; x < 256 * 16; x += kSelThreads) hist16[x] = 0;
  __syncthreads();
  // kSelItems independent loads per thread in flight (the pass is latency-bound otherwise)
  for (int64_t base = lo; base < hi; base += kSelStep) {
    uint32_t key[kSelItems];
    bool ok[kSelItems];
#pragma unroll
    for (int e = 0; e < kSelItems; ++e) {
      const int64_t i = base + (int64_t)e * kSelThreads + tid;
      ok[e] = i < hi;
      key[e] = order_key(r.sc[ok[e] ? i : hi - 1]);  // unconditional, so that the loads overlap
    }
#pragma unroll
    for (int e = 0; e < kSelItems; ++e)
      if (ok[e] && (key[e] & himask) == prefix)
        atomicAdd(&hist16[(((key[e] >> shift) & 255u) << 4) | (lane & 15)], 1u);
  }
  __syncthreads();
  uint32_t* const gh = r.w + kWHist + 256 * pass;
  // The additions and the ticket are device-wide atomics, performed where all workgroups see
  // them.  The additions return a value, and the wait for it is the wait for their completion;
  // only then does the workgroup draw its ticket, so the one that draws the last ticket finds
  // every addition done.  (No cache is involved: a fence would write back the whole L2.)
  if (tid < 256) {
    uint32_t c = 0;
#pragma unroll
    for (int x = 0; x < 16; ++x) c += hist16[(tid << 4) | x];
    uint32_t old = 0;
    if (c) old = __hip_atomic_fetch_add(&gh[tid], c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(old) : : "memory");
  }
  __syncthreads();
  if (tid == 0)
    last = __hip_atomic_fetch_add(&r.w[kWDone + pass], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == gridDim.x - 1;
  __syncthreads();
  if (!last) return;
  if (tid < 256) hist[tid] = __hip_atomic_load(&gh[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  if (tid == 0) {
    uint32_t cum = 0;
    int b = 255;
    for (; b > 0; --b) {
      const uint32_t c = hist[b];
      if (cum + c >= krem) break;
      cum += c;
    }
    r.w[kWState + 2 * (pass + 1)] = prefix | ((uint32_t)b << shift);
    r.w[kWState + 2 * (pass + 1) + 1] = krem - cum;
  }
}

// Keys above and equal to the threshold in every slice.
__global__ __launch_bounds__(kSelThreads) void k_sel_count(const SelArgs a) {
  const SelRow r = sel_row(a, blockIdx.y);
  if (r.w[kWChoose] == 0) return;
  const int64_t lo = (int64_t)r.w[kWForced] + (int64_t)blockIdx.x * a.slice_len;
  const int64_t hi = lo + a.slice_len < a.n ? lo + a.slice_len : a.n;
  const uint32_t T = r.w[kWState + 8];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  __shared__ uint32_t wtot[kSelWaves][2];
  uint32_t tg = 0, te = 0;
  for (int64_t base = lo; base < hi; base += kSelStep) {
    uint32_t key[kSelItems];
#pragma unroll
    for (int e = 0; e < kSelItems; ++e) {
      const int64_t i = base + (int64_t)e * kSelThreads + tid;
      key[e] = order_key(r.sc[i < hi ? i : hi - 1]);
    }
#pragma unroll
    for (int e = 0; e < kSelItems; ++e) {
      const bool in = base + (int64_t)e * kSelThreads + tid < hi;
      tg += __popcll(__ballot(in && key[e] > T));
      te += __popcll(__ballot(in && key[e] == T));
    }
  }
  if (lane == 0) { wtot[wv][0] = tg; wtot[wv][1] = te; }
  __syncthreads();
  if (tid == 0) {
    uint32_t g = 0, e = 0;
    for (int w = 0; w < kSelWaves; ++w) { g += wtot[w][0]; e += wtot[w][1]; }
    r.w[kWCount + 2 * blockIdx.x] = g;
    r.w[kWCount + 2 * blockIdx.x + 1] = e;
  }
}

// Ordered compaction of one slice.
__global__ __launch_bounds__(kSelThreads) void k_sel_write(const SelArgs a) {
  const SelRow r = sel_row(a, blockIdx.y);
  const uint32_t kp = r.w[kWChoose];
  if (kp == 0) return;
  const int f = (int)r.w[kWForced];
  const int64_t lo = (int64_t)f + (int64_t)blockIdx.x * a.slice_len;
  const int64_t hi = lo + a.slice_len < a.n ? lo + a.slice_len : a.n;
  const uint32_t T = r.w[kWState + 8];
  const uint32_t need_eq = r.w[kWState + 9];  // >= 1
  int32_t* const out = r.out;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  __shared__ uint32_t wtot[2][kSelWaves][2];
  uint32_t run_gt = 0, run_eq = 0;  // totals over everything before this slice, then before the step
  for (int sl = 0; sl < (int)blockIdx.x; ++sl) {
    run_gt += r.w[kWCount + 2 * sl];
    run_eq += r.w[kWCount + 2 * sl + 1];
  }
  if (run_gt + (run_eq < need_eq ? run_eq : need_eq) >= kp) return;  // the row is complete already
  const uint64_t lt_mask = lane == 0 ? 0ull : (~0ull >> (64 - lane));
  int par = 0;
  for (int64_t base = lo; base < hi; base += kSelStep, par ^= 1) {
    uint64_t bg[kSelItems], be[kSelItems];
    uint32_t tg = 0, te = 0, keys[kSelItems];
#pragma unroll
    for (int e = 0; e < kSelItems; ++e) {
      const int64_t i = base + (int64_t)wv * (64 * kSelItems) + e * 64 + lane;
      keys[e] = order_key(r.sc[i < hi ? i : hi - 1]);
    }
#pragma unroll
    for (int e = 0; e < kSelItems; ++e) {
      const int64_t i = base + (int64_t)wv * (64 * kSelItems) + e * 64 + lane;
      const uint32_t key = keys[e];
      bg[e] = __ballot(i < hi && key > T);
      be[e] = __ballot(i < hi && key == T);
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
    if (run_gt + (run_eq < need_eq ? run_eq : need_eq) >= kp) break;
  }
}

size_t select_ws_bytes(const vs_params& p) {
  return align_up((size_t)2 * p.n_q_heads * kSelRowWords * sizeof(uint32_t), 256);
}

hipError_t launch_select(const vs_params& p, const float* vscore, const float* sscore,
                         const int32_t* v_budget_h, const int32_t* s_budget_h,
                         int32_t* v_idx, int32_t* v_cnt, int32_t* s_idx, int32_t* s_cnt, void* ws,
                         hipStream_t st) {
  SelArgs a;
  a.vscore = vscore; a.sscore = sscore; a.n = p.q_start + p.q_len;
  a.n_q_heads = p.n_q_heads;
  a.v_budget = p.vertical_budget; a.s_budget = p.slash_budget;
  a.keep_v = p.keep_first_cols; a.keep_s = p.keep_local_band;
  a.v_budget_h = v_budget_h; a.s_budget_h = s_budget_h;
  a.v_idx = v_idx; a.v_cnt = v_cnt; a.s_idx = s_idx; a.s_cnt = s_cnt;
  a.ws = (uint32_t*)ws;
  // slices: whole steps of the workgroup, enough of them for about 2048 workgroups in all
  const int rows = 2 * p.n_q_heads;
  int64_t want = 2048 / rows;
  want = want < 1 ? 1 : (want > kSelMaxSlices ? kSelMaxSlices : want);
  const int64_t steps = ceil_div(a.n, kSelStep);
  a.slice_len = ceil_div(steps, want) * kSelStep;
  const int n_slices = (int)ceil_div(a.n, a.slice_len);
  const dim3 grid(n_slices, rows);
  hipLaunchKernelGGL(k_sel_init, dim3(rows), dim3(256), 0, st, a);
  for (int pass = 0; pass < 4; ++pass) hipLaunchKernelGGL(k_sel_hist, grid, dim3(kSelThreads), 0, st, a, pass);
  hipLaunchKernelGGL(k_sel_count, grid, dim3(kSelThreads), 0, st, a);
  hipLaunchKernelGGL(k_sel_write, grid, dim3(kSelThreads), 0, st, a);
  return hipGetLastError();
}

// ---- the selection for callers that cannot allocate ------------------------------------------
// vs_select_static: the control blocks of the rows (histograms, tickets, slice counts) live in
// a file-scope device array instead of a caller workspace.  Every device the library runs on
// holds its own copy of the array (2 x 128 rows x 4,736 bytes = 1.2 MB) at its own address
// until the process ends; in host code the array's name is only a handle, the address comes
// from hipGetSymbolAddress, once per device, with that device current.  k_sel_init clears the
// rows a call uses, so a call never sees the contents the call before it left behind; calls
// that overlap in time on one device share the array and race.
constexpr int kSelStaticMaxHeads = 128;
static __device__ __align__(256) uint32_t scratch[2 * kSelStaticMaxHeads * kSelRowWords];

int select_static_max_heads() { return kSelStaticMaxHeads; }

hipError_t select_static_scratch(void** ptr_out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptr_of[kMaxDevices] = {nullptr};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr_of[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    ptr_of[dev] = ptr;
  }
  *ptr_out = ptr_of[dev];
  return hipSuccess;
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
