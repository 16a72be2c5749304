"""Vertical-slash sparse prefill attention for MI355X (gfx950): HIP kernels behind a C ABI
(include/vs.h, libvs.so) and this thin ctypes binding."""
from .binding import (  # noqa: F401
    Chunk, VsError, VsParams, VsDca, alloc_index_sets, count_tiles, dense_causal_prefill, estimate, lib, prefill_chunk, select,
    sparse_attn_prefill, chunk_cost, plan_chunks, VS_COST_DENSE, VS_COST_SPARSE, select_heads, attention_recall, refine_step, set_option, status_string, workspace_bytes, yarn_softmax_scale,
    VS_OK, VS_ERR_INVALID_ARG, VS_ERR_UNSUPPORTED, VS_ERR_WORKSPACE, VS_ERR_HIP, VS_ERR_TOO_LARGE, select_static, VsRequest, request_table, attn_batch,
    VS_WS_ESTIMATE, VS_WS_SELECT, VS_WS_SPARSE, VS_WS_DENSE, VS_WS_CHUNK, VS_WS_COUNT_TILES,
    VS_OPT_ATTN_SEGMENT_BLOCKS, VS_OPT_ATTN_KEY_SPLIT, VS_OPT_ATTN_ROUNDS_IN_TURN, EXPORTS, LIB_PATH,
)
