/*
 * vs_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * Plain, slow, fp64 CPU statement of what chunked-prefill vertical-slash sparse
 * attention computes (Qwen2.5-1M technical report, section 5.2 "Efficient
 * Inference with Sparse Attention": the MInference paragraph and the
 * "Integrating with Chunked prefill" paragraph; softmax_lse and
 * Attention_Recall from the "Sparsity refinement" paragraph; attention
 * temperature from the YaRN equation and the three attention patterns of Dual
 * Chunk Attention from section 5.1).
 *
 * It exists so that the GPU library can be checked against something that a
 * reader can compare with the paper by eye.  Only tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  It shares no code, header, table or
 * helper with the HIP library and neither includes the other.
 *
 * Every function works on HOST pointers.  Q/K/V are bf16 bit patterns
 * (uint16_t); each value is widened exactly to fp64 and all arithmetic is fp64.
 * There is no blocking, no fusion and no reordering: every softmax is the
 * two-sweep textbook form (maximum, then sum of exponentials).  OpenMP is used
 * only across independent rows / heads.
 *
 * Notation (as in the paper where it has one):
 *   Hq, Hkv  query / key-value heads, G = Hq/Hkv, kv head of query head h is h/G
 *   D        head dimension
 *   C        q_len, rows of the chunk; s = q_start, absolute position of row 0
 *   n_k      s + C, the keys visible to the chunk ("all key tokens")
 *   W        last_q window (the last 64 tokens within each chunk), W' = min(W, C)
 *   B        block edge of the computed mask (64 in the contract, 1 = token exact)
 *
 * Pins (tests/test_oracle_*.py): dense attention against an independent
 * brute-force softmax, closed forms at Q = 0, rows of P summing to one,
 * score conservation, hand-written tiny masks, everything-selected == dense,
 * recall in (0,1], selection against a stable sort; the Dual Chunk Attention
 * variants against a hand-written pattern matrix, a brute force that reads its
 * patterns from that matrix, and the cases in which they must reduce to the
 * plain functions; the pattern rule also reproduces, with the positions of the
 * input recipe, the two diagonal lists that the caption of the figure of
 * "Integrating with DCA" prints (tests/golden/dca_diagonal_lists.txt; chunk
 * length 5, largest position 7, distance 7).  Accuracy of the sparse
 * result against dense attention on real text is parity unpinned (it needs
 * trained weights and the paper's evaluation suites).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct vso_params {
  int32_t n_q_heads, n_kv_heads, head_dim;
  int64_t q_len;   /* C */
  int64_t q_start; /* s */
  int64_t q_stride_tok, q_stride_head; /* element strides, innermost stride 1 */
  int64_t k_stride_tok, k_stride_head;
  int64_t v_stride_tok, v_stride_head;
  double softmax_scale;
  int32_t last_q;          /* W */
  int32_t block;           /* B */
  int32_t vertical_budget; /* Bv, forced column(s) included */
  int32_t slash_budget;    /* Bs, forced band included */
  int32_t keep_first_cols; /* columns 0..keep_first_cols-1 always kept */
  int32_t keep_local_band; /* offsets 0..keep_local_band-1 always kept */
} vso_params;

static double bf16_to_f64(uint16_t b) {
  uint32_t u = ((uint32_t)b) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

/* ---------------------------------------------------------------------------
 * Dual Chunk Attention (section 5.1, DCA paragraph): the sequence is cut into
 * chunks of `chunk` tokens and the (query, key) pairs fall into three patterns
 *   0 intra-chunk       query and key in the same chunk
 *   1 successive-chunk  key in the chunk before the query's AND the distance
 *                       pos_q - pos_k inside the local window (< window)
 *   2 inter-chunk       every other pair
 * Each pattern has its own rotation of the query (the remapped relative
 * positions); the keys are stored once.  The caller supplies the three rotated
 * query tensors; what is computed here is which of them meets which key.
 * ------------------------------------------------------------------------- */
typedef struct vso_dca {
  int64_t chunk;  /* 0 = no DCA: every pair uses the first query tensor */
  int64_t window;
  const uint16_t *q_succ, *q_inter;
} vso_dca;

int vso_dca_region(int64_t pos_q, int64_t pos_k, int64_t chunk, int64_t window) {
  const int64_t cq = pos_q / chunk, ck = pos_k / chunk;
  if (cq == ck) return 0;
  if (cq == ck + 1 && pos_q - pos_k < window) return 1;
  return 2;
}

/* scale * <q_i, k_j> for query head h (kv head g); i is the row of the chunk,
 * pos its absolute position. */
static double logit(const vso_params *p, const vso_dca *dca, const uint16_t *q,
                    const uint16_t *k, int64_t i, int h, int g, int64_t j) {
  if (dca && dca->chunk > 0) {
    const int r = vso_dca_region(p->q_start + i, j, dca->chunk, dca->window);
    if (r == 1) q = dca->q_succ;
    if (r == 2) q = dca->q_inter;
  }
  const uint16_t *qr = q + i * p->q_stride_tok + (int64_t)h * p->q_stride_head;
  const uint16_t *kr = k + j * p->k_stride_tok + (int64_t)g * p->k_stride_head;
  double acc = 0.0;
  for (int d = 0; d < p->head_dim; ++d) acc += bf16_to_f64(qr[d]) * bf16_to_f64(kr[d]);
  return p->softmax_scale * acc;
}

/* ---------------------------------------------------------------------------
 * Attention temperature (YaRN equation, section 5.1):
 *   weights = softmax(q.k / (t sqrt(D))),  sqrt(1/t) = 0.1 ln(s) + 1,
 * s = inference length / training length.  Returns 1/(t sqrt(D)).
 * ------------------------------------------------------------------------- */
double vso_yarn_softmax_scale(double s, int head_dim) {
  double r = 0.1 * log(s) + 1.0; /* sqrt(1/t) */
  return r * r / sqrt((double)head_dim);
}

/* ---------------------------------------------------------------------------
 * Step 1, estimation (section 5.2: attention between the last query tokens and
 * all key tokens; with chunked prefill the last 64 tokens of each chunk).
 * For each listed head: causal softmax rows of the W' window queries over keys
 * 0..n_k-1, then
 *   vscore[j] = sum_r P[r][j]                      (a vertical line = a column)
 *   sscore[o] = sum_r P[r][pos(r) - o]             (a slash = constant pos - j)
 *   lse_lastq[r] = log sum_j exp(logit)
 * Outputs are [n_heads][n_k] (scores) and [n_heads][W'] (lse), fp64.
 * ------------------------------------------------------------------------- */
static int estimate_impl(const vso_params *p, const vso_dca *dca, const uint16_t *q,
                         const uint16_t *k, int n_heads, const int32_t *heads,
                         double *vscore, double *sscore, double *lse_lastq) {
  const int64_t C = p->q_len, s = p->q_start, n_k = s + C;
  const int64_t Wp = p->last_q < C ? p->last_q : C;
  const int G = p->n_q_heads / p->n_kv_heads;
  double *P = (double *)malloc(sizeof(double) * (size_t)Wp * (size_t)n_k);
  if (!P) return -1;
  for (int hs = 0; hs < n_heads; ++hs) {
    const int h = heads[hs], g = h / G;
    double *vs = vscore + (int64_t)hs * n_k, *ss = sscore + (int64_t)hs * n_k;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < Wp; ++r) {
      const int64_t i = C - Wp + r, pos = s + i;
      double *Pr = P + r * n_k;
      double m = -INFINITY;
      for (int64_t j = 0; j <= pos; ++j) {
        Pr[j] = logit(p, dca, q, k, i, h, g, j);
        if (Pr[j] > m) m = Pr[j];
      }
      double L = 0.0;
      for (int64_t j = 0; j <= pos; ++j) L += exp(Pr[j] - m);
      for (int64_t j = 0; j <= pos; ++j) Pr[j] = exp(Pr[j] - m) / L;
      for (int64_t j = pos + 1; j < n_k; ++j) Pr[j] = 0.0;
      if (lse_lastq) lse_lastq[(int64_t)hs * Wp + r] = m + log(L);
    }
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < n_k; ++j) {
      double a = 0.0;
      for (int64_t r = 0; r < Wp; ++r) a += P[r * n_k + j];
      vs[j] = a;
    }
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < n_k; ++o) {
      double a = 0.0;
      for (int64_t r = 0; r < Wp; ++r) {
        const int64_t pos = s + (C - Wp + r);
        if (pos - o >= 0) a += P[r * n_k + (pos - o)];
      }
      ss[o] = a;
    }
  }
  free(P);
  return 0;
}

int vso_estimate(const vso_params *p, const uint16_t *q, const uint16_t *k,
                 int n_heads, const int32_t *heads, double *vscore,
                 double *sscore, double *lse_lastq) {
  return estimate_impl(p, NULL, q, k, n_heads, heads, vscore, sscore, lse_lastq);
}

/* The same with DCA: window row i meets key j through the query tensor of their
 * pattern ("Integrating with DCA", section 5.2: the selection may be given other
 * rotations than the attention itself; that choice is the caller's). */
int vso_estimate_dca(const vso_params *p, const uint16_t *q_intra, const uint16_t *q_succ,
                     const uint16_t *q_inter, int64_t chunk, int64_t window,
                     const uint16_t *k, int n_heads, const int32_t *heads,
                     double *vscore, double *sscore, double *lse_lastq) {
  const vso_dca dca = {chunk, window, q_succ, q_inter};
  return estimate_impl(p, &dca, q_intra, k, n_heads, heads, vscore, sscore, lse_lastq);
}

/* ---------------------------------------------------------------------------
 * Step 2, selection (section 5.2: critical tokens chosen by the vertical-slash
 * pattern with a per-head number of vertical and diagonal lines).
 * One problem: n scores, keep k = min(budget, n) of them.  Indices
 * 0..n_forced-1 are always kept (their score counts as +infinity).  The kept set
 * is the first k entries of the order (score descending, index ascending);
 * it is returned in ascending index order.
 * ------------------------------------------------------------------------- */
typedef struct { double sc; int32_t idx; } vso_pair;

static int cmp_score_desc_idx_asc(const void *a, const void *b) {
  const vso_pair *x = (const vso_pair *)a, *y = (const vso_pair *)b;
  if (x->sc > y->sc) return -1;
  if (x->sc < y->sc) return 1;
  return (x->idx > y->idx) - (x->idx < y->idx);
}
static int cmp_i32(const void *a, const void *b) {
  int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
  return (x > y) - (x < y);
}

int vso_select_one(int64_t n, const double *score, int64_t budget,
                   int64_t n_forced, int32_t *idx_out, int32_t *cnt_out) {
  const int64_t k = budget < n ? budget : n;
  vso_pair *pr = (vso_pair *)malloc(sizeof(vso_pair) * (size_t)(n > 0 ? n : 1));
  if (!pr) return -1;
  for (int64_t i = 0; i < n; ++i) {
    pr[i].sc = (i < n_forced) ? INFINITY : score[i];
    pr[i].idx = (int32_t)i;
  }
  qsort(pr, (size_t)n, sizeof(vso_pair), cmp_score_desc_idx_asc);
  for (int64_t i = 0; i < k; ++i) idx_out[i] = pr[i].idx;
  qsort(idx_out, (size_t)k, sizeof(int32_t), cmp_i32);
  *cnt_out = (int32_t)k;
  free(pr);
  return 0;
}

/* All heads, both kinds.  vscore/sscore are [n_heads][n_k]; v_idx is
 * [n_heads][Bv], s_idx is [n_heads][Bs]; unused tail entries are set to -1. */
int vso_select(const vso_params *p, int n_heads, const double *vscore,
               const double *sscore, int32_t *v_idx, int32_t *v_cnt,
               int32_t *s_idx, int32_t *s_cnt) {
  const int64_t n_k = p->q_start + p->q_len;
  int rc = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int t = 0; t < 2 * n_heads; ++t) {
    const int h = t / 2;
    if (t % 2 == 0) {
      int32_t *o = v_idx + (int64_t)h * p->vertical_budget;
      for (int i = 0; i < p->vertical_budget; ++i) o[i] = -1;
      int64_t f = p->keep_first_cols < n_k ? p->keep_first_cols : n_k;
      if (vso_select_one(n_k, vscore + (int64_t)h * n_k, p->vertical_budget, f, o, v_cnt + h)) rc = -1;
    } else {
      int32_t *o = s_idx + (int64_t)h * p->slash_budget;
      for (int i = 0; i < p->slash_budget; ++i) o[i] = -1;
      int64_t f = p->keep_local_band < n_k ? p->keep_local_band : n_k;
      if (vso_select_one(n_k, sscore + (int64_t)h * n_k, p->slash_budget, f, o, s_cnt + h)) rc = -1;
    }
  }
  return rc;
}

/* ---------------------------------------------------------------------------
 * Step 3, the computed mask.  "Attention only on the selected critical tokens"
 * with the slash lines widened to the B x B blocks they cross:
 *   A = union over selected offsets o of { floor(o/B) } and, when o mod B != 0,
 *       { floor(o/B) + 1 }
 *   M[i][j] = (j <= pos(i)) and ( j in vertical set  or  (floor(pos(i)/B) - floor(j/B)) in A )
 * With B = 1 this is the token-exact rule  j in V or pos(i)-j in S.
 * is_v: n_k bytes, in_a: (n_blocks + 1) bytes, both zero-initialised by caller.
 * ------------------------------------------------------------------------- */
static void build_sets(const vso_params *p, const int32_t *v_idx, int32_t v_cnt,
                       const int32_t *s_idx, int32_t s_cnt, uint8_t *is_v,
                       uint8_t *in_a, int64_t n_a) {
  const int64_t B = p->block;
  for (int32_t t = 0; t < v_cnt; ++t) is_v[v_idx[t]] = 1;
  for (int32_t t = 0; t < s_cnt; ++t) {
    const int64_t o = s_idx[t];
    if (o / B < n_a) in_a[o / B] = 1;
    if (o % B != 0 && o / B + 1 < n_a) in_a[o / B + 1] = 1;
  }
}

static int in_mask(const vso_params *p, const uint8_t *is_v, const uint8_t *in_a,
                   int64_t pos, int64_t j) {
  if (j > pos) return 0;
  if (!is_v) return 1; /* dense causal */
  const int64_t B = p->block;
  return is_v[j] || in_a[pos / B - j / B];
}

/* mask_out: [n_rows][n_k] bytes for one head's index sets (for the hand-mask pins). */
int vso_mask(const vso_params *p, const int32_t *v_idx, int32_t v_cnt,
             const int32_t *s_idx, int32_t s_cnt, int64_t n_rows,
             const int64_t *rows, uint8_t *mask_out) {
  const int64_t n_k = p->q_start + p->q_len, n_a = n_k / p->block + 2;
  uint8_t *is_v = (uint8_t *)calloc((size_t)n_k, 1), *in_a = (uint8_t *)calloc((size_t)n_a, 1);
  if (!is_v || !in_a) return -1;
  build_sets(p, v_idx, v_cnt, s_idx, s_cnt, is_v, in_a, n_a);
  for (int64_t t = 0; t < n_rows; ++t)
    for (int64_t j = 0; j < n_k; ++j)
      mask_out[t * n_k + j] = (uint8_t)in_mask(p, is_v, in_a, p->q_start + rows[t], j);
  free(is_v);
  free(in_a);
  return 0;
}

/* ---------------------------------------------------------------------------
 * Steps 3 and 4, attention over the mask (sparse) or over all causal keys
 * (dense: pass v_idx == NULL).  For each listed head and each listed chunk row:
 *   out = sum_{j in M} softmax_M(logit_j) V_j      lse = log sum_{j in M} exp(logit_j)
 * (softmax_lse of the "Sparsity refinement" paragraph: full when dense, sparse
 * otherwise).  A row whose mask is empty gives out = 0, lse = -inf.
 * v_idx / s_idx are [Hq][Bv] / [Hq][Bs] indexed by the head number itself.
 * out: [n_heads][n_rows][D] fp64, lse: [n_heads][n_rows] fp64.
 * ------------------------------------------------------------------------- */
static int attention_impl(const vso_params *p, const vso_dca *dca, const uint16_t *q,
                          const uint16_t *k, const uint16_t *v, const int32_t *v_idx,
                          const int32_t *v_cnt, const int32_t *s_idx, const int32_t *s_cnt,
                          int n_heads, const int32_t *heads, int64_t n_rows,
                          const int64_t *rows, double *out, double *lse) {
  const int64_t n_k = p->q_start + p->q_len, n_a = n_k / p->block + 2;
  const int G = p->n_q_heads / p->n_kv_heads, D = p->head_dim;
  uint8_t *is_v = NULL, *in_a = NULL;
  if (v_idx) {
    is_v = (uint8_t *)malloc((size_t)n_k);
    in_a = (uint8_t *)malloc((size_t)n_a);
    if (!is_v || !in_a) return -1;
  }
  for (int hs = 0; hs < n_heads; ++hs) {
    const int h = heads[hs], g = h / G;
    if (v_idx) {
      memset(is_v, 0, (size_t)n_k);
      memset(in_a, 0, (size_t)n_a);
      build_sets(p, v_idx + (int64_t)h * p->vertical_budget, v_cnt[h],
                 s_idx + (int64_t)h * p->slash_budget, s_cnt[h], is_v, in_a, n_a);
    }
#pragma omp parallel
    {
      /* x[j]: this row's logits, kept so that each is computed once */
      double *x = (double *)malloc(sizeof(double) * (size_t)n_k);
#pragma omp for schedule(dynamic, 1)
      for (int64_t t = 0; t < n_rows; ++t) {
        const int64_t i = rows[t], pos = p->q_start + i;
        double *o = out + ((int64_t)hs * n_rows + t) * D;
        double m = -INFINITY;
        for (int64_t j = 0; j <= pos; ++j)
          if (in_mask(p, is_v, in_a, pos, j)) {
            x[j] = logit(p, dca, q, k, i, h, g, j);
            if (x[j] > m) m = x[j];
          }
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        if (m == -INFINITY) {
          if (lse) lse[(int64_t)hs * n_rows + t] = -INFINITY;
          continue;
        }
        double L = 0.0;
        for (int64_t j = 0; j <= pos; ++j)
          if (in_mask(p, is_v, in_a, pos, j)) L += exp(x[j] - m);
        for (int64_t j = 0; j <= pos; ++j)
          if (in_mask(p, is_v, in_a, pos, j)) {
            const double w = exp(x[j] - m) / L;
            const uint16_t *vr = v + j * p->v_stride_tok + (int64_t)g * p->v_stride_head;
            for (int d = 0; d < D; ++d) o[d] += w * bf16_to_f64(vr[d]);
          }
        if (lse) lse[(int64_t)hs * n_rows + t] = m + log(L);
      }
      free(x);
    }
  }
  free(is_v);
  free(in_a);
  return 0;
}

int vso_attention(const vso_params *p, const uint16_t *q, const uint16_t *k,
                  const uint16_t *v, const int32_t *v_idx, const int32_t *v_cnt,
                  const int32_t *s_idx, const int32_t *s_cnt, int n_heads,
                  const int32_t *heads, int64_t n_rows, const int64_t *rows,
                  double *out, double *lse) {
  return attention_impl(p, NULL, q, k, v, v_idx, v_cnt, s_idx, s_cnt, n_heads, heads,
                        n_rows, rows, out, lse);
}

/* The same with DCA: the mask is unchanged, every logit uses the query tensor of
 * its (query, key) pattern, one softmax over all of them. */
int vso_attention_dca(const vso_params *p, const uint16_t *q_intra, const uint16_t *q_succ,
                      const uint16_t *q_inter, int64_t chunk, int64_t window,
                      const uint16_t *k, const uint16_t *v, const int32_t *v_idx,
                      const int32_t *v_cnt, const int32_t *s_idx, const int32_t *s_cnt,
                      int n_heads, const int32_t *heads, int64_t n_rows,
                      const int64_t *rows, double *out, double *lse) {
  const vso_dca dca = {chunk, window, q_succ, q_inter};
  return attention_impl(p, &dca, q_intra, k, v, v_idx, v_cnt, s_idx, s_cnt, n_heads, heads,
                        n_rows, rows, out, lse);
}

/* Attention recall of one head over a chunk: the mean over the chunk's rows of
 * exp(lse_sparse - lse_full) ("Sparsity refinement" paragraph; the paper gives the
 * per-query quantity and compares it with a threshold per head -- the mean over the rows
 * is this build's reading of "the recall of a head").  A row with no selected key
 * (lse_sparse = -inf) counts 0.  lse arrays are [rows]. */
double vso_recall_mean(const double *lse_sparse, const double *lse_full, int64_t rows) {
  double acc = 0.0;
  for (int64_t i = 0; i < rows; ++i) {
    const double r = exp(lse_sparse[i] - lse_full[i]);
    acc += isfinite(r) ? r : 0.0;
  }
  return rows > 0 ? acc / (double)rows : 0.0;
}

/* One pass of the sparsity refinement (Algorithm 1) over the heads of a layer: a head whose
 * recall is below the threshold gets dv more vertical and ds more slash lines, up to the
 * given maxima.  Returns the number of heads whose configuration changed. */
int vso_refine_step(int n_heads, const double *recall, double threshold, int32_t dv, int32_t ds,
                    int32_t v_max, int32_t s_max, int32_t *v_budget, int32_t *s_budget) {
  int changed = 0;
  for (int h = 0; h < n_heads; ++h) {
    if (!(recall[h] < threshold)) continue;
    int32_t nv = v_budget[h] + dv, ns = s_budget[h] + ds;
    if (nv > v_max) nv = v_max;
    if (ns > s_max) ns = s_max;
    if (nv != v_budget[h] || ns != s_budget[h]) ++changed;
    v_budget[h] = nv;
    s_budget[h] = ns;
  }
  return changed;
}

/* Number of OpenMP threads the calls above will use (reported beside timings). */
#ifdef _OPENMP
#include <omp.h>
int vso_num_threads(void) { return omp_get_max_threads(); }
#else
int vso_num_threads(void) { return 1; }
#endif
