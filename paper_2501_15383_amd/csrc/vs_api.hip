// Host side of libvs: the extern "C" entry points declared in include/vs.h.  Every argument
// is checked here, before the first HIP call, so a bad call returns a status without touching
// a device; the kernels may then assume consistent shapes.
#include <math.h>

#include "vs_common.h"

namespace vs {
namespace {

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// the kernels keep a lane's byte offset inside a 64-token tile in 32 bits
bool stride_ok(int64_t tok, int64_t head, int d) {
  return tok >= d && head >= d && tok % 8 == 0 && head % 8 == 0 && tok < (int64_t(1) << 23);
}

// shape / stride checks common to every entry point
int check_params(const vs_params* p, bool need_budgets) {
  if (!p) return VS_ERR_INVALID_ARG;
  if (p->n_q_heads < 1 || p->n_kv_heads < 1 || p->n_q_heads % p->n_kv_heads != 0) return VS_ERR_INVALID_ARG;
  if (p->head_dim < 1 || p->q_len < 1 || p->q_start < 0) return VS_ERR_INVALID_ARG;
  if (p->block < 1 || p->last_q < 1) return VS_ERR_INVALID_ARG;
  if (!(p->softmax_scale > 0.f) || !isfinite(p->softmax_scale)) return VS_ERR_INVALID_ARG;
  if (p->q_start > (int64_t)INT32_MAX || p->q_len > (int64_t)INT32_MAX ||
      p->q_start + p->q_len > (int64_t)INT32_MAX - 4096)
    return VS_ERR_INVALID_ARG;
  if (p->keep_first_cols < 0 || p->keep_local_band < 0) return VS_ERR_INVALID_ARG;
  if (need_budgets && (p->vertical_budget < 1 || p->slash_budget < 1)) return VS_ERR_INVALID_ARG;
  if (p->head_dim != 64 && p->head_dim != 128) return VS_ERR_UNSUPPORTED;
  if (p->block != kBlock) return VS_ERR_UNSUPPORTED;
  if (p->last_q > 64) return VS_ERR_UNSUPPORTED;
  const int d = p->head_dim;
  if (!stride_ok(p->q_stride_tok, p->q_stride_head, d) || !stride_ok(p->k_stride_tok, p->k_stride_head, d) ||
      !stride_ok(p->v_stride_tok, p->v_stride_head, d) || !stride_ok(p->o_stride_tok, p->o_stride_head, d))
    return VS_ERR_INVALID_ARG;
  return VS_OK;
}

int check_ws(const void* ws, size_t have, size_t need) {
  if (need == 0) return VS_OK;
  if (!ws || !aligned(ws, 256) || have < need) return VS_ERR_WORKSPACE;
  return VS_OK;
}

size_t sparse_ws_bytes(const vs_params& p, bool dense) {
  const size_t own = blocklist_bytes(p, dense) + attn_sync_bytes(p) + attn_split_bytes(p, dense);
  // (a sparse single-token call without DCA takes the packed path, a DCA one the plain path: room for either)
  if (!dense && attn_single_token_packs(p)) return own > attn_single_token_bytes(p) ? own : attn_single_token_bytes(p);
  return own;
}

// layout of the VS_WS_CHUNK workspace
struct ChunkWs {
  size_t vscore, sscore, v_idx, s_idx, v_cnt, s_cnt, sub, total;
};
ChunkWs chunk_layout(const vs_params& p) {
  const size_t n_k = (size_t)(p.q_start + p.q_len), hq = (size_t)p.n_q_heads;
  ChunkWs w;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
  w.vscore = take(hq * n_k * sizeof(float));
  w.sscore = take(hq * n_k * sizeof(float));
  w.v_idx = take(hq * (size_t)p.vertical_budget * sizeof(int32_t));
  w.s_idx = take(hq * (size_t)p.slash_budget * sizeof(int32_t));
  w.v_cnt = take(hq * sizeof(int32_t));
  w.s_cnt = take(hq * sizeof(int32_t));
  w.sub = off;
  const size_t a = estimate_ws_bytes(p), b = select_ws_bytes(p), c = sparse_ws_bytes(p, false);
  off += a > b ? (a > c ? a : c) : (b > c ? b : c);
  w.total = off;
  return w;
}

int hip_status(hipError_t e) { return e == hipSuccess ? VS_OK : VS_ERR_HIP; }

}  // namespace
}  // namespace vs

using namespace vs;

extern "C" {

size_t vs_workspace_bytes(const vs_params* p, int which) {
  if (check_params(p, which == VS_WS_SELECT || which == VS_WS_SPARSE || which == VS_WS_CHUNK || which == VS_WS_COUNT_TILES) != VS_OK) return 0;
  switch (which) {
    case VS_WS_ESTIMATE: return estimate_ws_bytes(*p);
    case VS_WS_SELECT: return select_ws_bytes(*p);
    case VS_WS_SPARSE: return sparse_ws_bytes(*p, false);
    case VS_WS_DENSE: return sparse_ws_bytes(*p, true);
    case VS_WS_CHUNK: return chunk_layout(*p).total;
    case VS_WS_COUNT_TILES: return blocklist_bytes(*p, false);
    default: return 0;
  }
}

const char* vs_status_string(int status) {
  switch (status) {
    case VS_OK: return "ok";
    case VS_ERR_INVALID_ARG: return "invalid argument (null pointer, shape, stride or alignment)";
    case VS_ERR_UNSUPPORTED: return "unsupported configuration (head_dim must be 64 or 128, block 64, last_q <= 64; DCA chunk and window multiples of 64)";
    case VS_ERR_WORKSPACE: return "workspace missing, not 256-byte aligned, or too small";
    case VS_ERR_HIP: return "HIP runtime error at launch";
    case VS_ERR_TOO_LARGE: return "request beyond the fixed capacity of this entry point (vs_select_static: at most 128 query heads)";
    default: return "unknown status";
  }
}

double vs_chunk_cost(int64_t q_start, int64_t q_len, int32_t model, int32_t vertical_budget,
                     int32_t slash_budget) {
  if (q_start < 0 || q_len < 1 || q_start % kBlock != 0) return -1.0;
  if (model != VS_COST_DENSE && model != VS_COST_SPARSE) return -1.0;
  if (model == VS_COST_SPARSE && (vertical_budget < 1 || slash_budget < 1)) return -1.0;
  const int64_t m0 = q_start / kBlock, nqb = ceil_div(q_len, kBlock);
  // sum over m = m0 .. m0 + nqb - 1 of (m + 1)
  const double causal = (double)nqb * (double)m0 + 0.5 * (double)nqb * (double)(nqb + 1);
  if (model == VS_COST_DENSE) return causal;
  const int64_t n_k = q_start + q_len, nb = ceil_div(n_k, kBlock);
  const double bs = (double)(slash_budget < n_k ? slash_budget : n_k);
  const double density = nb <= 2 ? 1.0 : 1.0 - pow(1.0 - 2.0 / (double)nb, bs);
  const double bv = (double)(vertical_budget < n_k ? vertical_budget : n_k);
  return causal * density + (double)nqb * ceil(bv / kBlock);
}

int vs_plan_chunks(int64_t n_ctx, int32_t n_chunks, int32_t model, int32_t vertical_budget,
                   int32_t slash_budget, int64_t* bounds) {
  if (!bounds || n_chunks < 1 || n_ctx < (int64_t)kBlock * n_chunks) return VS_ERR_INVALID_ARG;
  if (vs_chunk_cost(0, kBlock, model, vertical_budget, slash_budget) < 0) return VS_ERR_INVALID_ARG;
  const int64_t nb = ceil_div(n_ctx, kBlock);  // boundaries move in whole blocks
  auto cost = [&](int64_t b0, int64_t b1) {     // blocks [b0, b1)
    const int64_t t0 = b0 * kBlock, t1 = b1 * kBlock < n_ctx ? b1 * kBlock : n_ctx;
    return vs_chunk_cost(t0, t1 - t0, model, vertical_budget, slash_budget);
  };
  // start from equal sizes, then a few rounds of: target = mean cost; boundary c goes where the
  // cost of chunks 0 .. c-1 together is closest to c targets (so rounding does not pile up in
  // the last chunk).  Rounds are needed because the sparse cost of a chunk depends on its end.
  for (int c = 0; c <= n_chunks; ++c) bounds[c] = nb * c / n_chunks;
  for (int round = 0; round < 8; ++round) {
    double total = 0;
    for (int c = 0; c < n_chunks; ++c) total += cost(bounds[c], bounds[c + 1]);
    const double target = total / n_chunks;
    int64_t b = 0;
    double before = 0;  // cost of the chunks already cut
    for (int c = 1; c < n_chunks; ++c) {
      const double want = target * c - before;
      // smallest end e in (b, nb - (n_chunks - c)] whose cost reaches `want` (cost grows with e)
      int64_t lo = b + 1, hi = nb - (n_chunks - c);
      while (lo < hi) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (cost(b, mid) >= want) hi = mid; else lo = mid + 1;
      }
      // the end just below may be closer
      if (lo > b + 1 && fabs(cost(b, lo - 1) - want) <= fabs(cost(b, lo) - want)) --lo;
      bounds[c] = lo;
      before += cost(b, lo);
      b = lo;
    }
  }
  for (int c = 0; c < n_chunks; ++c) bounds[c] *= kBlock;
  bounds[n_chunks] = n_ctx;
  return VS_OK;
}

int vs_set_option(int which, int64_t value) {
  switch (which) {
    case VS_OPT_ATTN_SEGMENT_BLOCKS:
      if (value < 0 || value > (int64_t)INT32_MAX) return VS_ERR_INVALID_ARG;
      set_attn_segment_blocks((int)value);
      return VS_OK;
    case VS_OPT_ATTN_ROUNDS_IN_TURN:
      if (value != 0 && value != 1) return VS_ERR_INVALID_ARG;
      set_attn_schedule_in_turn((int)value);
      return VS_OK;
    case VS_OPT_ATTN_KEY_SPLIT:
      if (value < 0 || value > 16) return VS_ERR_INVALID_ARG;
      set_attn_key_split((int)value);
      return VS_OK;
    default: return VS_ERR_INVALID_ARG;
  }
}

float vs_yarn_softmax_scale(float s, int32_t head_dim) {
  if (!(s >= 1.f) || head_dim < 1) return 0.f;
  const float r = 0.1f * logf(s) + 1.0f;  // sqrt(1/t)
  return r * r / sqrtf((float)head_dim);
}

namespace {
int check_dca(const vs_dca* dca, DcaArgs* out);

int estimate_any(const vs_params* p, const void* q, const vs_dca* dca, const void* k, float* vscore,
                 float* sscore, float* lse_lastq, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_params(p, false);
  if (rc != VS_OK) return rc;
  DcaArgs da;
  if (dca && (rc = check_dca(dca, &da)) != VS_OK) return rc;
  if (!q || !k || !vscore || !sscore) return VS_ERR_INVALID_ARG;
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(vscore, 4) || !aligned(sscore, 4)) return VS_ERR_INVALID_ARG;
  rc = check_ws(ws, ws_bytes, estimate_ws_bytes(*p));
  if (rc != VS_OK) return rc;
  return hip_status(launch_estimate(*p, q, dca ? &da : nullptr, k, vscore, sscore, lse_lastq, ws,
                                    (hipStream_t)stream));
}
}  // namespace

int vs_estimate(const vs_params* p, const void* q, const void* k, float* vscore, float* sscore,
                float* lse_lastq, void* ws, size_t ws_bytes, void* stream) {
  return estimate_any(p, q, nullptr, k, vscore, sscore, lse_lastq, ws, ws_bytes, stream);
}

int vs_estimate_dca(const vs_params* p, const void* q_intra, const vs_dca* dca, const void* k,
                    float* vscore, float* sscore, float* lse_lastq, void* ws, size_t ws_bytes,
                    void* stream) {
  if (!dca) return VS_ERR_INVALID_ARG;
  return estimate_any(p, q_intra, dca, k, vscore, sscore, lse_lastq, ws, ws_bytes, stream);
}

int vs_select(const vs_params* p, const float* vscore, const float* sscore, int32_t* v_idx,
              int32_t* v_cnt, int32_t* s_idx, int32_t* s_cnt, void* ws, size_t ws_bytes,
              void* stream) {
  int rc = check_params(p, true);
  if (rc != VS_OK) return rc;
  if (!vscore || !sscore || !v_idx || !v_cnt || !s_idx || !s_cnt) return VS_ERR_INVALID_ARG;
  rc = check_ws(ws, ws_bytes, select_ws_bytes(*p));
  if (rc != VS_OK) return rc;
  return hip_status(launch_select(*p, vscore, sscore, nullptr, nullptr, v_idx, v_cnt, s_idx, s_cnt, ws,
                                  (hipStream_t)stream));
}

int vs_select_static(const vs_params* p, const float* vscore, const float* sscore, int32_t* v_idx,
                     int32_t* v_cnt, int32_t* s_idx, int32_t* s_cnt, void* stream) {
  int rc = check_params(p, true);
  if (rc != VS_OK) return rc;
  if (!vscore || !sscore || !v_idx || !v_cnt || !s_idx || !s_cnt) return VS_ERR_INVALID_ARG;
  if (p->n_q_heads > select_static_max_heads()) return VS_ERR_TOO_LARGE;
  void* scratch_ptr = nullptr;
  if (select_static_scratch(&scratch_ptr) != hipSuccess) return VS_ERR_HIP;
  return hip_status(launch_select(*p, vscore, sscore, nullptr, nullptr, v_idx, v_cnt, s_idx, s_cnt, scratch_ptr,
                                  (hipStream_t)stream));
}

int vs_select_heads(const vs_params* p, const float* vscore, const float* sscore,
                    const int32_t* v_budget_h, const int32_t* s_budget_h, int32_t* v_idx,
                    int32_t* v_cnt, int32_t* s_idx, int32_t* s_cnt, void* ws, size_t ws_bytes,
                    void* stream) {
  int rc = check_params(p, true);
  if (rc != VS_OK) return rc;
  if (!vscore || !sscore || !v_budget_h || !s_budget_h || !v_idx || !v_cnt || !s_idx || !s_cnt)
    return VS_ERR_INVALID_ARG;
  rc = check_ws(ws, ws_bytes, select_ws_bytes(*p));
  if (rc != VS_OK) return rc;
  return hip_status(launch_select(*p, vscore, sscore, v_budget_h, s_budget_h, v_idx, v_cnt, s_idx, s_cnt, ws,
                                  (hipStream_t)stream));
}

int vs_attention_recall(const vs_params* p, const float* lse_sparse, const float* lse_full,
                        float* recall, void* stream) {
  int rc = check_params(p, false);
  if (rc != VS_OK) return rc;
  if (!lse_sparse || !lse_full || !recall) return VS_ERR_INVALID_ARG;
  return hip_status(launch_recall(*p, lse_sparse, lse_full, recall, (hipStream_t)stream));
}

int vs_refine_step(const vs_params* p, const float* recall, float threshold, int32_t add_vertical,
                   int32_t add_slash, int32_t* v_budget_h, int32_t* s_budget_h, int32_t* changed,
                   void* stream) {
  int rc = check_params(p, true);
  if (rc != VS_OK) return rc;
  if (!recall || !v_budget_h || !s_budget_h) return VS_ERR_INVALID_ARG;
  if (!(threshold >= 0.f) || add_vertical < 0 || add_slash < 0) return VS_ERR_INVALID_ARG;
  return hip_status(launch_refine(*p, recall, threshold, add_vertical, add_slash, v_budget_h, s_budget_h, changed,
                                  (hipStream_t)stream));
}

namespace {
// dca == null: plain attention.  Otherwise the descriptor is checked and turned into DcaArgs.
int check_dca(const vs_dca* dca, DcaArgs* out) {
  if (!dca->q_succ || !dca->q_inter || !aligned(dca->q_succ, 16) || !aligned(dca->q_inter, 16))
    return VS_ERR_INVALID_ARG;
  if (dca->chunk < 1 || dca->window < 0) return VS_ERR_INVALID_ARG;
  if (dca->chunk % kBlock != 0 || dca->window % kBlock != 0) return VS_ERR_UNSUPPORTED;
  if (dca->chunk / kBlock > INT32_MAX || dca->window / kBlock > INT32_MAX) return VS_ERR_INVALID_ARG;
  out->q_succ = dca->q_succ; out->q_inter = dca->q_inter;
  out->chunk = dca->chunk; out->window = dca->window;
  return VS_OK;
}

int sparse_attn(const vs_params* p, const void* q, const vs_dca* dca, const void* k, const void* v,
                const int32_t* v_idx, const int32_t* v_cnt, const int32_t* s_idx,
                const int32_t* s_cnt, void* out, float* lse, void* ws, size_t ws_bytes,
                void* stream) {
  int rc = check_params(p, true);
  if (rc != VS_OK) return rc;
  DcaArgs da;
  if (dca && (rc = check_dca(dca, &da)) != VS_OK) return rc;
  if (!q || !k || !v || !out || !v_idx || !v_cnt || !s_idx || !s_cnt) return VS_ERR_INVALID_ARG;
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(out, 16)) return VS_ERR_INVALID_ARG;
  rc = check_ws(ws, ws_bytes, sparse_ws_bytes(*p, false));
  if (rc != VS_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  if (!dca && attn_single_token_packs(*p))
    return hip_status(launch_attention_single_token(*p, q, k, v, v_idx, v_cnt, s_idx, s_cnt, out, lse, ws, st));
  const BlockList bl = blocklist_layout(*p, false, ws);
  hipError_t e = launch_build_blocklist(*p, s_idx, s_cnt, false, bl, st);
  if (e != hipSuccess) return VS_ERR_HIP;
  char* sync = (char*)ws + blocklist_bytes(*p, false);
  return hip_status(launch_attention(*p, q, dca ? &da : nullptr, k, v, v_idx, v_cnt, false, bl, out, lse, sync,
                                     sync + attn_sync_bytes(*p), st));
}

int dense_attn(const vs_params* p, const void* q, const vs_dca* dca, const void* k, const void* v,
               void* out, float* lse, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_params(p, false);
  if (rc != VS_OK) return rc;
  DcaArgs da;
  if (dca && (rc = check_dca(dca, &da)) != VS_OK) return rc;
  if (!q || !k || !v || !out) return VS_ERR_INVALID_ARG;
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(out, 16)) return VS_ERR_INVALID_ARG;
  rc = check_ws(ws, ws_bytes, sparse_ws_bytes(*p, true));
  if (rc != VS_OK) return rc;
  const BlockList bl = blocklist_layout(*p, true, ws);
  hipStream_t st = (hipStream_t)stream;
  hipError_t e = launch_build_blocklist(*p, nullptr, nullptr, true, bl, st);
  if (e != hipSuccess) return VS_ERR_HIP;
  char* sync = (char*)ws + blocklist_bytes(*p, true);
  return hip_status(launch_attention(*p, q, dca ? &da : nullptr, k, v, nullptr, nullptr, true, bl, out, lse, sync,
                                     sync + attn_sync_bytes(*p), st));
}
}  // namespace

int vs_sparse_attn_prefill(const vs_params* p, const void* q, const void* k, const void* v,
                           const int32_t* v_idx, const int32_t* v_cnt, const int32_t* s_idx,
                           const int32_t* s_cnt, void* out, float* lse, void* ws, size_t ws_bytes,
                           void* stream) {
  return sparse_attn(p, q, nullptr, k, v, v_idx, v_cnt, s_idx, s_cnt, out, lse, ws, ws_bytes, stream);
}

int vs_dense_causal_prefill(const vs_params* p, const void* q, const void* k, const void* v,
                            void* out, float* lse, void* ws, size_t ws_bytes, void* stream) {
  return dense_attn(p, q, nullptr, k, v, out, lse, ws, ws_bytes, stream);
}

int vs_sparse_attn_prefill_dca(const vs_params* p, const void* q_intra, const vs_dca* dca, const void* k,
                               const void* v, const int32_t* v_idx, const int32_t* v_cnt,
                               const int32_t* s_idx, const int32_t* s_cnt, void* out, float* lse,
                               void* ws, size_t ws_bytes, void* stream) {
  if (!dca) return VS_ERR_INVALID_ARG;
  return sparse_attn(p, q_intra, dca, k, v, v_idx, v_cnt, s_idx, s_cnt, out, lse, ws, ws_bytes, stream);
}

int vs_dense_causal_prefill_dca(const vs_params* p, const void* q_intra, const vs_dca* dca, const void* k,
                                const void* v, void* out, float* lse, void* ws, size_t ws_bytes,
                                void* stream) {
  if (!dca) return VS_ERR_INVALID_ARG;
  return dense_attn(p, q_intra, dca, k, v, out, lse, ws, ws_bytes, stream);
}

namespace {
// dca == null: plain.  sel: the rotations the estimate uses (null: those of dca).
int prefill_chunk_any(const vs_params* p, const void* q, const vs_dca* dca, const vs_dca* sel, const void* k,
                      const void* v, void* out, float* lse, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_params(p, true);
  if (rc != VS_OK) return rc;
  if (!q || !k || !v || !out) return VS_ERR_INVALID_ARG;
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(out, 16)) return VS_ERR_INVALID_ARG;
  // both descriptors are checked before the first launch: a bad one must leave the stream untouched
  DcaArgs scratch_da;
  if (dca && (rc = check_dca(dca, &scratch_da)) != VS_OK) return rc;
  if (sel && (rc = check_dca(sel, &scratch_da)) != VS_OK) return rc;
  const ChunkWs w = chunk_layout(*p);
  rc = check_ws(ws, ws_bytes, w.total);
  if (rc != VS_OK) return rc;
  char* b = (char*)ws;
  float* vscore = (float*)(b + w.vscore);
  float* sscore = (float*)(b + w.sscore);
  int32_t* v_idx = (int32_t*)(b + w.v_idx);
  int32_t* s_idx = (int32_t*)(b + w.s_idx);
  int32_t* v_cnt = (int32_t*)(b + w.v_cnt);
  int32_t* s_cnt = (int32_t*)(b + w.s_cnt);
  void* sub = b + w.sub;
  const size_t sub_bytes = w.total - w.sub;
  rc = estimate_any(p, q, dca ? (sel ? sel : dca) : nullptr, k, vscore, sscore, nullptr, sub, sub_bytes, stream);
  if (rc != VS_OK) return rc;
  rc = vs_select(p, vscore, sscore, v_idx, v_cnt, s_idx, s_cnt, sub, sub_bytes, stream);
  if (rc != VS_OK) return rc;
  return sparse_attn(p, q, dca, k, v, v_idx, v_cnt, s_idx, s_cnt, out, lse, sub, sub_bytes, stream);
}
}  // namespace

int vs_prefill_chunk(const vs_params* p, const void* q, const void* k, const void* v, void* out,
                     float* lse, void* ws, size_t ws_bytes, void* stream) {
  return prefill_chunk_any(p, q, nullptr, nullptr, k, v, out, lse, ws, ws_bytes, stream);
}

int vs_prefill_chunk_dca(const vs_params* p, const void* q_intra, const vs_dca* dca, const vs_dca* dca_select,
                         const void* k, const void* v, void* out, float* lse, void* ws, size_t ws_bytes,
                         void* stream) {
  if (!dca) return VS_ERR_INVALID_ARG;
  return prefill_chunk_any(p, q_intra, dca, dca_select, k, v, out, lse, ws, ws_bytes, stream);
}

namespace {
int check_batch(const vs_params* p, int32_t n_requests) {
  int rc = check_params(p, true);
  if (rc != VS_OK) return rc;
  if (n_requests < 1) return VS_ERR_INVALID_ARG;
  if (p->q_len > 4096 || n_requests > 4096) return VS_ERR_UNSUPPORTED;
  return VS_OK;
}
}  // namespace

size_t vs_batch_workspace_bytes(const vs_params* p, int32_t n_requests) {
  if (check_batch(p, n_requests) != VS_OK) return 0;
  return attn_batch_bytes(*p, n_requests);
}

int vs_attn_batch(const vs_params* p, const vs_request* requests, int32_t n_requests, void* ws,
                  size_t ws_bytes, void* stream) {
  int rc = check_batch(p, n_requests);
  if (rc != VS_OK) return rc;
  if (!requests || !aligned(requests, 8)) return VS_ERR_INVALID_ARG;
  rc = check_ws(ws, ws_bytes, attn_batch_bytes(*p, n_requests));
  if (rc != VS_OK) return rc;
  return hip_status(launch_attention_batch(*p, requests, n_requests, ws, (hipStream_t)stream));
}

int vs_count_tiles(const vs_params* p, const int32_t* v_idx, const int32_t* v_cnt,
                   const int32_t* s_idx, const int32_t* s_cnt, int64_t* tiles, void* ws,
                   size_t ws_bytes, void* stream) {
  int rc = check_params(p, true);
  if (rc != VS_OK) return rc;
  if (!v_idx || !v_cnt || !s_idx || !s_cnt || !tiles) return VS_ERR_INVALID_ARG;
  rc = check_ws(ws, ws_bytes, blocklist_bytes(*p, false));
  if (rc != VS_OK) return rc;
  const BlockList bl = blocklist_layout(*p, false, ws);
  hipStream_t st = (hipStream_t)stream;
  hipError_t e = launch_build_blocklist(*p, s_idx, s_cnt, false, bl, st);
  if (e != hipSuccess) return VS_ERR_HIP;
  return hip_status(launch_count_tiles(*p, v_idx, v_cnt, bl, tiles, st));
}

}  // extern "C"
