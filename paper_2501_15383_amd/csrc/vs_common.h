// Internal declarations shared by the HIP sources of libvs (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/vs.h"

namespace vs {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) float f32x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kBlock = 64;            // B: edge of the computed slash blocks
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t a, size_t b) { return (a + b - 1) / b * b; }

// ---- block list (built per head from the selected slash offsets) -----------------------
// A: bitmap, bit a set <=> block diagonal a is computed.
// ent: ascending list of key-block entries for a query tile of kAttnQBlocks query blocks:
//   entry = (cc << 4) | mask, cc = c + (kAttnQBlocks - 1); the tile whose first query block is
//   m0 uses key block m0 - c, and query block t of the tile takes part iff mask bit t is set
//   (diagonal c + t is in A).  The list is padded with sentinels (cc = 0x7FFFFFF) so that a
//   reader may fetch whole batches of 64 entries without bounds checks.
#ifdef VS_X_QBLOCKS
constexpr int kAttnQBlocks = VS_X_QBLOCKS;   // timing experiment (4 = one workgroup of eight waves per compute unit):
                                             // the prefill paths stay correct, the packed single-token path does not
#else
constexpr int kAttnQBlocks = 2;       // query blocks (of 64 rows) per attention workgroup
#endif
constexpr uint32_t kEntSentinel = 0x7FFFFFF0u;

struct BlockList {
  uint32_t* bm_a;     // [heads][words]
  uint32_t* ent;      // [heads][ent_stride]
  int64_t words, ent_stride;
  int heads;          // n_q_heads, or 1 for the dense list shared by all heads
};
static inline int64_t bitmap_words(int64_t n_k) { return ceil_div(ceil_div(n_k, kBlock) + 8, 32) + 2; }
static inline int64_t entry_stride(int64_t n_k) {
  return ceil_div(ceil_div(n_k, kBlock) + kAttnQBlocks, 64) * 64 + 128;
}
static inline size_t blocklist_bytes(const vs_params& p, bool dense) {
  const size_t heads = dense ? 1 : (size_t)p.n_q_heads;
  const int64_t n_k = p.q_start + p.q_len;
  return align_up(heads * (size_t)bitmap_words(n_k) * 4, 256) + align_up(heads * (size_t)entry_stride(n_k) * 4, 256);
}
static inline BlockList blocklist_layout(const vs_params& p, bool dense, void* ws) {
  BlockList b;
  const int64_t n_k = p.q_start + p.q_len;
  b.heads = dense ? 1 : p.n_q_heads;
  b.words = bitmap_words(n_k);
  b.ent_stride = entry_stride(n_k);
  b.bm_a = (uint32_t*)ws;
  b.ent = (uint32_t*)((char*)ws + align_up((size_t)b.heads * (size_t)b.words * 4, 256));
  return b;
}

// ---- launchers (defined in the .hip files; all enqueue on `st`, return hipError_t) ------
hipError_t launch_build_blocklist(const vs_params& p, const int32_t* s_idx, const int32_t* s_cnt,
                                  bool dense, const BlockList& bl, hipStream_t st);
// Dual Chunk Attention: the two other rotations of the chunk's queries (same strides as q),
// chunk length and local window in tokens (multiples of 64)
struct DcaArgs {
  const void* q_succ;
  const void* q_inter;
  int64_t chunk, window;
};
// sync_ws: attn_sync_bytes(p) bytes of counters (zero-filled by the launch itself); split_ws:
// attn_split_bytes(p) bytes (may be null when that is 0); dca may be null
hipError_t launch_attention(const vs_params& p, const void* q, const DcaArgs* dca, const void* k, const void* v,
                            const int32_t* v_idx, const int32_t* v_cnt, bool dense,
                            const BlockList& bl, void* out, float* lse, void* sync_ws, void* split_ws,
                            hipStream_t st);
// several requests in one launch (short chunks, decode steps): p.q_len = the longest request,
// p.q_start + p.q_len = the most keys any request sees; req is a device array
size_t attn_batch_bytes(const vs_params& p, int n_req);
hipError_t launch_attention_batch(const vs_params& p, const vs_request* req, int n_req, void* ws, hipStream_t st);
// sparse attention of a single token with 2..16 query heads per KV head runs as a batch of one
bool attn_single_token_packs(const vs_params& p);
size_t attn_single_token_bytes(const vs_params& p);
hipError_t launch_attention_single_token(const vs_params& p, const void* q, const void* k, const void* v,
                                         const int32_t* v_idx, const int32_t* v_cnt, const int32_t* s_idx,
                                         const int32_t* s_cnt, void* out, float* lse, void* ws, hipStream_t st);
size_t attn_sync_bytes(const vs_params& p);
// key split of short chunks: number of ranges (1 = none) and bytes of partial results
int attn_split(const vs_params& p, bool dense);
void set_attn_key_split(int n);
void set_attn_schedule_in_turn(int on);
size_t attn_split_bytes(const vs_params& p, bool dense);
void set_attn_segment_blocks(int blocks);
hipError_t launch_count_tiles(const vs_params& p, const int32_t* v_idx, const int32_t* v_cnt,
                              const BlockList& bl, int64_t* tiles, hipStream_t st);

size_t estimate_ws_bytes(const vs_params& p);
hipError_t launch_estimate(const vs_params& p, const void* q, const DcaArgs* dca, const void* k, float* vscore,
                           float* sscore, float* lse_lastq, void* ws, hipStream_t st);

size_t select_ws_bytes(const vs_params& p);
hipError_t launch_select(const vs_params& p, const float* vscore, const float* sscore,
                         const int32_t* v_budget_h, const int32_t* s_budget_h,
                         int32_t* v_idx, int32_t* v_cnt, int32_t* s_idx, int32_t* s_cnt,
                         void* ws, hipStream_t st);
// the selection's control blocks in a file-scope device array (callers that cannot allocate):
// the most query heads it holds, and its address on the current device
int select_static_max_heads();
hipError_t select_static_scratch(void** ptr_out);
hipError_t launch_recall(const vs_params& p, const float* lse_sparse, const float* lse_full, float* recall,
                         hipStream_t st);
hipError_t launch_refine(const vs_params& p, const float* recall, float threshold, int32_t dv, int32_t ds,
                         int32_t* v_budget, int32_t* s_budget, int32_t* changed, hipStream_t st);

}  // namespace vs
