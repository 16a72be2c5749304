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

// ---- block-diagonal bitmaps (built per head from the selected slash offsets) ----------
// A: bit a set <=> block diagonal a is computed.  U: bit cc set <=> some query block t of a
// tile of NQB query blocks uses key block (m0 - (cc - (NQB-1))), i.e. A has a bit in
// [cc-NQB+1, cc].  Both are padded so that every word a kernel may touch exists.
static inline int64_t bitmap_words(int64_t n_k) { return ceil_div(ceil_div(n_k, kBlock) + 8, 32) + 1; }

constexpr int kAttnQBlocks = 2;       // query blocks (of 64 rows) per attention workgroup

// ---- launchers (defined in the .hip files; all enqueue on `st`, return hipError_t) ------
hipError_t launch_build_bitmaps(const vs_params& p, const int32_t* s_idx, const int32_t* s_cnt,
                                bool dense, uint32_t* bm_a, uint32_t* bm_u, hipStream_t st);
hipError_t launch_attention(const vs_params& p, const void* q, const void* k, const void* v,
                            const int32_t* v_idx, const int32_t* v_cnt, bool dense,
                            const uint32_t* bm_a, const uint32_t* bm_u, void* out, float* lse,
                            hipStream_t st);
hipError_t launch_count_tiles(const vs_params& p, const int32_t* v_idx, const int32_t* v_cnt,
                              const uint32_t* bm_a, int64_t* tiles, hipStream_t st);

size_t estimate_ws_bytes(const vs_params& p);
hipError_t launch_estimate(const vs_params& p, const void* q, const void* k, float* vscore,
                           float* sscore, float* lse_lastq, void* ws, hipStream_t st);

size_t select_ws_bytes(const vs_params& p);
hipError_t launch_select(const vs_params& p, const float* vscore, const float* sscore,
                         int32_t* v_idx, int32_t* v_cnt, int32_t* s_idx, int32_t* s_cnt,
                         void* ws, hipStream_t st);

}  // namespace vs
