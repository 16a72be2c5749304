/*
 * vs.h -- C ABI of the vertical-slash sparse prefill library for MI355X (gfx950).
 *
 * The method (Qwen2.5-1M technical report, section 5.2, "MInference" and
 * "Integrating with Chunked prefill" paragraphs): for every query chunk of a
 * long prompt and every attention head,
 *   1. estimate  -- attention of the chunk's last 64 queries against all keys
 *                   seen so far, summed along columns ("vertical lines") and
 *                   along diagonals pos - j = const ("slash lines");
 *   2. select    -- keep a per-head number of the best vertical and slash lines;
 *   3. attend    -- softmax attention over the selected keys only.
 * A dense causal kernel is the fallback / comparison (the paper's "full
 * attention").  softmax_lse is an optional output of both attention calls (the
 * quantity the paper's Attention_Recall is built from).
 *
 * Conventions
 *  - Every pointer is a DEVICE pointer unless the comment says host.  The
 *    library never allocates, frees or synchronises: work is enqueued on
 *    `stream` (a hipStream_t passed as void*, NULL = the null stream) and
 *    VS_OK means "enqueued".  The caller owns every buffer, including the
 *    workspace, and keeps them alive until the stream reaches the work.
 *  - Q / K / V / out hold bf16; element strides are given in vs_params, the
 *    innermost (head_dim) stride is 1.  Base pointers must be 16-byte aligned
 *    and strides multiples of 8 elements.
 *  - Keys and values of the current chunk must already be in the cache:
 *    positions 0 .. q_start + q_len - 1 are read ("all key tokens").
 *  - Query head h uses key/value head h / (n_q_heads / n_kv_heads).
 *  - Arguments are validated on the host before any HIP call; a negative
 *    status is returned and nothing is enqueued.  No exception or abort crosses
 *    this boundary.  Inputs must be finite.
 *  - Calls that share a workspace must be ordered on one stream.
 */
#ifndef VS_H_
#define VS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  VS_OK = 0,
  VS_ERR_INVALID_ARG = -1, /* null pointer, bad shape, bad stride, misalignment      */
  VS_ERR_UNSUPPORTED = -2, /* a valid request this build has no kernel for           */
  VS_ERR_WORKSPACE = -3,   /* workspace missing, misaligned or too small             */
  VS_ERR_HIP = -4,         /* the HIP runtime refused a launch                       */
  VS_ERR_TOO_LARGE = -5    /* beyond the fixed capacity of an entry point that has one */
};

/* which workspace size vs_workspace_bytes() reports */
enum { VS_WS_ESTIMATE = 0, VS_WS_SELECT = 1, VS_WS_SPARSE = 2, VS_WS_DENSE = 3, VS_WS_CHUNK = 4, VS_WS_COUNT_TILES = 5 };

typedef struct vs_params {
  int32_t n_q_heads;       /* Hq                                                      */
  int32_t n_kv_heads;      /* Hkv, divides Hq                                         */
  int32_t head_dim;        /* D: 64 or 128                                            */
  int32_t last_q;          /* W: estimation window, 1..64 (the paper uses the last 64
                              tokens of each chunk); effective W' = min(W, q_len)     */
  int64_t q_len;           /* C: rows of this chunk, >= 1                             */
  int64_t q_start;         /* s: absolute position of row 0, >= 0 (any value: the 64-key
                              blocks of the mask are aligned to absolute positions;
                              vs_chunk_cost alone wants a multiple of 64);
                              keys visible n_k = s + C (< 2^31)                       */
  int64_t q_stride_tok, q_stride_head;   /* Q  [C][Hq][D]     => (Hq*D, D)            */
  int64_t k_stride_tok, k_stride_head;   /* K  [>=n_k][Hkv][D] => (Hkv*D, D)          */
  int64_t v_stride_tok, v_stride_head;   /* V  like K                                 */
  int64_t o_stride_tok, o_stride_head;   /* out like Q                                */
  float softmax_scale;     /* 1/sqrt(D), or 1/(t sqrt(D)) with YaRN's temperature     */
  int32_t block;           /* B: edge of the computed slash blocks, must be 64        */
  int32_t vertical_budget; /* Bv >= 1: vertical lines kept per head, forced included  */
  int32_t slash_budget;    /* Bs >= 1: slash lines kept per head, forced included     */
  int32_t keep_first_cols; /* columns 0..keep_first_cols-1 are always kept (>= 0)     */
  int32_t keep_local_band; /* offsets 0..keep_local_band-1 are always kept (>= 0)     */
} vs_params;

/* Bytes of workspace the call named by `which` needs for these parameters
 * (0 on invalid parameters).  Host function; touches no device.  The workspace
 * must be 256-byte aligned.  VS_WS_CHUNK covers vs_prefill_chunk. */
size_t vs_workspace_bytes(const vs_params *p, int which);

/* Host: static, NUL-terminated description of a status code. */
const char *vs_status_string(int status);

/* Host: softmax scale with the attention temperature of the YaRN equation
 * (section 5.1): 1/(t sqrt(D)) with sqrt(1/t) = 0.1 ln(s) + 1, where s is the
 * ratio of inference length to training length (s >= 1; s = 1 gives 1/sqrt(D)). */
float vs_yarn_softmax_scale(float s, int32_t head_dim);

/* Step 1 (section 5.2, MInference paragraph: attention between the last query
 * tokens and all key tokens; chunked-prefill paragraph: the last 64 tokens of
 * each chunk).  With P the causal softmax rows of the W' window queries
 * (chunk rows C-W'..C-1) over keys 0..n_k-1:
 *   vscore[h][j] = sum_r P[r][j]              column (vertical) score of key j
 *   sscore[h][o] = sum_r P[r][pos(r) - o]     diagonal (slash) score of offset o
 *   lse_lastq[h][r] = log sum_j exp(scale q_r.k_j)        (optional, may be NULL)
 * vscore, sscore: fp32 [Hq][n_k], fully overwritten.  lse_lastq: fp32 [Hq][W'].
 * Only the window rows of q are read.  Results are run-to-run identical. */
int vs_estimate(const vs_params *p, const void *q, const void *k, float *vscore,
                float *sscore, float *lse_lastq, void *ws, size_t ws_bytes,
                void *stream);

/* Step 2 (section 5.2: critical tokens chosen by the vertical-slash pattern with
 * a per-head count of vertical and slash lines).  Per head, keeps the
 * kv = min(Bv, n_k) best columns and ks = min(Bs, n_k) best offsets, where
 * "best" is the order (score descending, index ascending) with the forced
 * entries (keep_first_cols, keep_local_band) counted as +infinity.  Scores must
 * be >= 0 and finite.
 *   v_idx: int32 [Hq][Bv], s_idx: int32 [Hq][Bs], ascending, tail filled with -1
 *   v_cnt, s_cnt: int32 [Hq] = kv, ks */
int vs_select(const vs_params *p, const float *vscore, const float *sscore,
              int32_t *v_idx, int32_t *v_cnt, int32_t *s_idx, int32_t *s_cnt,
              void *ws, size_t ws_bytes, void *stream);

/* vs_select for callers that cannot allocate device memory and have no workspace to
 * hand over: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, outputs and results as vs_select, minus the workspace:
 * the per-row control blocks (histograms, tickets, slice counts) live in a device
 * array inside the library, 1.2 MB on every GPU the library runs on, for the life
 * of the process.  The call allocates and frees nothing and clears what it uses
 * with its own kernel.  Limits: n_q_heads <= 128 (VS_ERR_TOO_LARGE beyond, checked
 * on the host before any device work).  All calls on one GPU share the array:
 * calls that may overlap in time on one GPU (two streams, two threads) race --
 * order them on one stream.  The first call on a device looks the array up
 * (hipGetSymbolAddress); make that call outside graph capture. */
int vs_select_static(const vs_params *p, const float *vscore, const float *sscore,
                     int32_t *v_idx, int32_t *v_cnt, int32_t *s_idx, int32_t *s_cnt,
                     void *stream);

/* Step 3 (section 5.2: attention only on the selected critical tokens; section
 * 5.3.1: sparse K/V loading is what the kernel is tuned for).  The computed mask
 * widens each slash line to the 64x64 blocks it crosses: with block-diagonal set
 * A = { floor(o/64) } U { floor(o/64)+1 : o mod 64 != 0 } over the selected
 * offsets o, row i (position p = s+i) attends key j <= p iff
 *     j is a selected column   or   floor(p/64) - floor(j/64) is in A.
 *   out[i][h][:] = sum_j softmax(scale q_i.k_j) V_j over those keys (bf16, fp32
 *   accumulation), lse[h][i] = log of the softmax denominator (optional fp32
 *   [Hq][C]; softmax_lse_sparse of the paper).  A row with no key gets 0 / -inf.
 * v_idx/s_idx/v_cnt/s_cnt as produced by vs_select (ascending, in range). */
int vs_sparse_attn_prefill(const vs_params *p, const void *q, const void *k,
                           const void *v, const int32_t *v_idx,
                           const int32_t *v_cnt, const int32_t *s_idx,
                           const int32_t *s_cnt, void *out, float *lse, void *ws,
                           size_t ws_bytes, void *stream);

/* Dense causal attention of the chunk: every key j <= p (section 5.2, "Sparsity
 * refinement": the full attention whose softmax_lse_full the recall is measured
 * against, `full_attention` in Algorithm 1; section 5.2 opening: the quadratic
 * cost the sparse path avoids).  Same outputs as above; lse is softmax_lse_full.
 * Budget fields of p are ignored. */
int vs_dense_causal_prefill(const vs_params *p, const void *q, const void *k,
                            const void *v, void *out, float *lse, void *ws,
                            size_t ws_bytes, void *stream);

/* One chunk of the whole path on one stream, no host synchronisation (section
 * 5.2, "Integrating with Chunked prefill": every chunk selects its own critical
 * tokens from its last 64 queries and then attends):
 * vs_estimate -> vs_select -> vs_sparse_attn_prefill.  Scores and index sets
 * live in the workspace (VS_WS_CHUNK). */
int vs_prefill_chunk(const vs_params *p, const void *q, const void *k,
                     const void *v, void *out, float *lse, void *ws,
                     size_t ws_bytes, void *stream);

/* Work accounting for a set of index sets: per head, the number of 64x64
 * (query block, key block) tiles the sparse kernel issues for this chunk
 * (slash tiles, then vertical tiles of up to 64 gathered columns).  This is the
 * unit in which the FLOPs "on computed blocks" are counted (section 5.3.1 quotes
 * the kernel's FLOPs utilisation) and the cost that section 5.3.2 sizes chunks by.
 *   tiles: int64 [Hq][2] = {slash tiles, vertical tiles}. */
int vs_count_tiles(const vs_params *p, const int32_t *v_idx, const int32_t *v_cnt,
                   const int32_t *s_idx, const int32_t *s_cnt, int64_t *tiles,
                   void *ws, size_t ws_bytes, void *stream);

/* Step a2 with one budget pair per head (sec. 5.2: the configuration, i.e. the
 * number of vertical and slash lines, is searched per attention head).
 *   v_budget_h, s_budget_h: device int32 [Hq], clamped to 1 .. p->vertical_budget
 *   / p->slash_budget, which stay the row lengths of v_idx / s_idx (rows padded
 *   with -1).  Everything else as vs_select. */
int vs_select_heads(const vs_params *p, const float *vscore, const float *sscore,
                    const int32_t *v_budget_h, const int32_t *s_budget_h,
                    int32_t *v_idx, int32_t *v_cnt, int32_t *s_idx, int32_t *s_cnt,
                    void *ws, size_t ws_bytes, void *stream);

/* Attention recall of every head over the chunk (sec. 5.2 "Sparsity refinement":
 * Attention_Recall = exp(softmax_lse_sparse - softmax_lse_full) per query; here
 * its mean over the chunk's rows, a row without selected keys counting 0).
 *   lse_sparse, lse_full: device fp32 [Hq][C] as written by the attention calls
 *   recall: device fp32 [Hq].  Deterministic (fixed reduction order). */
int vs_attention_recall(const vs_params *p, const float *lse_sparse,
                        const float *lse_full, float *recall, void *stream);

/* One pass of the sparsity refinement over the heads (sec. 5.2, Algorithm 1):
 * a head whose recall is below `threshold` gets add_vertical / add_slash more
 * lines, up to p->vertical_budget / p->slash_budget.
 *   recall: device fp32 [Hq]; v_budget_h, s_budget_h: device int32 [Hq], updated
 *   in place; changed: optional device int32, number of heads whose budgets grew.
 * The calibration data, the threshold and the step sizes are the caller's: the
 * paper does not print them. */
int vs_refine_step(const vs_params *p, const float *recall, float threshold,
                   int32_t add_vertical, int32_t add_slash, int32_t *v_budget_h,
                   int32_t *s_budget_h, int32_t *changed, void *stream);

/* Dual Chunk Attention (sec. 5.1, "Dual Chunk Attention" paragraph; sec. 5.2,
 * "Integrating with DCA").  The sequence is cut into chunks of `chunk` tokens and a
 * (query, key) pair falls into one of three patterns, each with its own remapped
 * relative positions, i.e. its own rotation of the query against the keys as stored:
 *   intra-chunk       query and key in the same chunk                       -> q_intra
 *   successive-chunk  key in the chunk before the query's and
 *                     pos_q - pos_k < window                                -> q_succ
 *   inter-chunk       every other pair                                      -> q_inter
 * The rotations themselves (RoPE at the remapped positions) are the caller's; the
 * calls below choose, per pair, which of the three tensors meets the key, under one
 * softmax.  q_succ and q_inter have the shape, strides and alignment of the q
 * argument (device bf16 [C][Hq][D], strides of vs_params).  chunk > 0 and
 * window >= 0 must be multiples of 64 (VS_ERR_UNSUPPORTED otherwise).  The paper
 * selects the critical tokens with other ("continuous") relative positions than it
 * attends with: pass the rotations made for the selection to vs_estimate_dca and
 * those of DCA proper to the attention calls.  Everything else (masks, outputs,
 * workspaces, errors) is as in the calls without _dca. */
typedef struct vs_dca {
  const void *q_succ;
  const void *q_inter;
  int64_t chunk;
  int64_t window;
} vs_dca;
int vs_sparse_attn_prefill_dca(const vs_params *p, const void *q_intra, const vs_dca *dca,
                               const void *k, const void *v, const int32_t *v_idx,
                               const int32_t *v_cnt, const int32_t *s_idx, const int32_t *s_cnt,
                               void *out, float *lse, void *ws, size_t ws_bytes, void *stream);
int vs_dense_causal_prefill_dca(const vs_params *p, const void *q_intra, const vs_dca *dca,
                                const void *k, const void *v, void *out, float *lse, void *ws,
                                size_t ws_bytes, void *stream);
int vs_estimate_dca(const vs_params *p, const void *q_intra, const vs_dca *dca, const void *k,
                    float *vscore, float *sscore, float *lse_lastq, void *ws, size_t ws_bytes,
                    void *stream);
/* vs_prefill_chunk with DCA: the estimate takes the rotations of dca_select (null: those of
 * dca), the attention those of dca; both share q_intra. */
int vs_prefill_chunk_dca(const vs_params *p, const void *q_intra, const vs_dca *dca,
                         const vs_dca *dca_select, const void *k, const void *v, void *out,
                         float *lse, void *ws, size_t ws_bytes, void *stream);

/* Several requests in one launch (section 5.2, "Integrating with Chunked prefill": with
 * chunked prefill, decoding of other requests is not held up behind a long prefill -- so
 * an engine has, at any step, many short pieces of attention to run: single-token decode
 * steps and short chunks of different requests against caches of different lengths).
 * One call per request leaves most of the chip idle; this call packs the (request, head,
 * query tile, key range) units of all requests into one persistent launch.
 *
 *   requests    DEVICE array [n_requests] of vs_request.  Every request has its own
 *               q / out (bf16 [q_len][Hq][D]), cache k / v (bf16 [>= q_start + q_len][Hkv][D]),
 *               optional lse (fp32 [Hq][q_len]), position and length; all share the head
 *               counts, head_dim, strides, softmax scale and index-row lengths of p.
 *               Index sets as for vs_sparse_attn_prefill (rows of p->vertical_budget /
 *               p->slash_budget entries); all four index pointers null = dense causal
 *               attention for that request.  Dense and sparse requests may be mixed.
 *   p->q_len    the longest request of the batch (1 .. 4096)
 *   p->q_start  such that p->q_start + p->q_len >= q_start + q_len of every request
 *               (the most keys any request sees); the workspace is sized from these
 *               two bounds, which is why they are host values while the requests
 *               themselves stay on the device (no copy, no synchronisation).
 * A request outside these bounds, or with a null q / k / v / out, is skipped on the
 * device: its outputs are left untouched.  Results per request are those of
 * vs_dense_causal_prefill / vs_sparse_attn_prefill up to the rounding of the fp32
 * partial sums (the key walk of every unit may be cut into ranges, folded in a fixed
 * order: run-to-run identical).  Workspace: vs_batch_workspace_bytes(p, n_requests).
 * Returns VS_ERR_UNSUPPORTED for p->q_len > 4096 or n_requests > 4096. */
typedef struct vs_request {
  const void *q, *k, *v;
  void *out;
  float *lse;                                   /* may be null */
  const int32_t *v_idx, *v_cnt, *s_idx, *s_cnt; /* all null: dense causal */
  int64_t q_start, q_len;
} vs_request;
size_t vs_batch_workspace_bytes(const vs_params *p, int32_t n_requests);
int vs_attn_batch(const vs_params *p, const vs_request *requests, int32_t n_requests,
                  void *ws, size_t ws_bytes, void *stream);

/* Cost model and chunk planner (host functions; sec. 5.3.2 "Dynamic Chunked Pipeline
 * Parallelism": chunk sizes are adjusted to the complexity of the attention
 * kernel so that every chunk takes about the same time).  The unit is one 64x64
 * tile of one head.
 *   VS_COST_DENSE    query block m (absolute index) costs m + 1 tiles
 *   VS_COST_SPARSE   expected tiles when the slash_budget offsets scatter
 *                    uniformly over the n_k = q_start + q_len keys of the chunk:
 *                    (m + 1) (1 - (1 - 2/nb)^Bs) with nb = ceil(n_k / 64), plus
 *                    ceil(min(Bv, n_k) / 64) tiles of gathered columns
 * vs_chunk_cost returns the sum over the query blocks of the chunk (< 0 on bad
 * arguments).  vs_plan_chunks writes n_chunks + 1 ascending token boundaries,
 * bounds[0] = 0, bounds[n_chunks] = n_ctx, the inner ones multiples of 64 chosen
 * so that the chunk costs are as equal as 64-token steps allow; returns VS_OK or
 * VS_ERR_INVALID_ARG (n_chunks < 1, n_ctx < 64 n_chunks, null pointer). */
enum { VS_COST_DENSE = 0, VS_COST_SPARSE = 1 };
double vs_chunk_cost(int64_t q_start, int64_t q_len, int32_t model,
                     int32_t vertical_budget, int32_t slash_budget);
int vs_plan_chunks(int64_t n_ctx, int32_t n_chunks, int32_t model,
                   int32_t vertical_budget, int32_t slash_budget, int64_t *bounds);

/* Host: process-wide tuning switches (no device call).  Each switch is one atomic
 * value, read by every later size query and launch of the process on any device;
 * a size query and the call it is made for must see the same values, so do not
 * change a switch between the two or while another thread is launching.  A call
 * made under a setting that needs more workspace than it is given returns
 * VS_ERR_WORKSPACE.  Returns VS_OK or VS_ERR_INVALID_ARG.
 *   VS_OPT_ATTN_SEGMENT_BLOCKS  value = number of 64-key blocks per sync segment of the
 *     attention launches (rounded down to a power of two), 0 = automatic.  The attention kernels are persistent;
 *     workgroups that walk the same head keep within two sync segments of each
 *     other (bounded waits on counters in the workspace) so that their K/V
 *     blocks are shared through the L2.  Only the timing depends on it.  The
 *     choice changes VS_WS_SPARSE / VS_WS_DENSE / VS_WS_CHUNK sizes, so set it
 *     before asking for them.
 *   VS_OPT_ATTN_KEY_SPLIT  chunks with few (query tile, head) units (a decode step, a short
 *     last chunk) have their key walk cut into ranges, one workgroup each, and a second
 *     kernel folds the partial results: 0 = automatic (up to 16 ranges, so that about 512
 *     workgroups run), 1 = never, 2..16 = that many ranges (at least 16 key blocks each).
 *     Results agree within the rounding of the fp32 partial sums.  Changes the workspace
 *     sizes like the option above.
 *   VS_OPT_ATTN_ROUNDS_IN_TURN  0 (default): the rounds of the persistent attention launch are
 *     dealt to its eight workgroup groups by weight (length of each head's block list), the
 *     heaviest first to the least loaded group; 1: in turn.  Only the timing depends on it. */
enum { VS_OPT_ATTN_SEGMENT_BLOCKS = 0, VS_OPT_ATTN_KEY_SPLIT = 1, VS_OPT_ATTN_ROUNDS_IN_TURN = 2 };
int vs_set_option(int which, int64_t value);

#ifdef __cplusplus
}
#endif
#endif /* VS_H_ */
