"""Thin ctypes binding of libvs (include/vs.h): argument marshalling only.

Every step of the path runs in the HIP kernels of the library; torch is used here only to
hold device memory and to name the current stream.  There is no fallback of any kind: if
the library has not been built, importing the entry points raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# VS_LIB_PATH names another build of the library (paper_2501_15383_amd.build --variant); there is still no fallback
LIB_PATH = os.environ.get("VS_LIB_PATH") or os.path.join(_HERE, "libvs.so")

VS_OK = 0
VS_ERR_INVALID_ARG, VS_ERR_UNSUPPORTED, VS_ERR_WORKSPACE, VS_ERR_HIP, VS_ERR_TOO_LARGE = -1, -2, -3, -4, -5
VS_WS_ESTIMATE, VS_WS_SELECT, VS_WS_SPARSE, VS_WS_DENSE, VS_WS_CHUNK, VS_WS_COUNT_TILES = range(6)
VS_OPT_ATTN_SEGMENT_BLOCKS = 0
VS_OPT_ATTN_KEY_SPLIT = 1
VS_OPT_ATTN_ROUNDS_IN_TURN = 2


class VsParams(C.Structure):
    """Mirror of `vs_params` in include/vs.h."""
    _fields_ = [
        ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("last_q", C.c_int32),
        ("q_len", C.c_int64), ("q_start", C.c_int64),
        ("q_stride_tok", C.c_int64), ("q_stride_head", C.c_int64),
        ("k_stride_tok", C.c_int64), ("k_stride_head", C.c_int64),
        ("v_stride_tok", C.c_int64), ("v_stride_head", C.c_int64),
        ("o_stride_tok", C.c_int64), ("o_stride_head", C.c_int64),
        ("softmax_scale", C.c_float), ("block", C.c_int32),
        ("vertical_budget", C.c_int32), ("slash_budget", C.c_int32),
        ("keep_first_cols", C.c_int32), ("keep_local_band", C.c_int32),
    ]


class VsDca(C.Structure):
    """Mirror of `vs_dca` in include/vs.h."""
    _fields_ = [("q_succ", C.c_void_p), ("q_inter", C.c_void_p), ("chunk", C.c_int64), ("window", C.c_int64)]


class VsRequest(C.Structure):
    """Mirror of `vs_request` in include/vs.h (11 eight-byte fields)."""
    _fields_ = [("q", C.c_void_p), ("k", C.c_void_p), ("v", C.c_void_p), ("out", C.c_void_p), ("lse", C.c_void_p),
                ("v_idx", C.c_void_p), ("v_cnt", C.c_void_p), ("s_idx", C.c_void_p), ("s_cnt", C.c_void_p),
                ("q_start", C.c_int64), ("q_len", C.c_int64)]


class VsError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def lib() -> C.CDLL:
    """Load libvs.so (built by paper_2501_15383_amd.build); raises if it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2501_15383_amd.build` "
                "(there is no CPU or PyTorch fallback for this library)")
        L = C.CDLL(LIB_PATH)
        P, vp, sz = C.POINTER(VsParams), C.c_void_p, C.c_size_t
        L.vs_workspace_bytes.restype = sz
        L.vs_workspace_bytes.argtypes = [P, C.c_int]
        L.vs_status_string.restype = C.c_char_p
        L.vs_status_string.argtypes = [C.c_int]
        L.vs_yarn_softmax_scale.restype = C.c_float
        L.vs_yarn_softmax_scale.argtypes = [C.c_float, C.c_int32]
        L.vs_estimate.restype = C.c_int
        L.vs_estimate.argtypes = [P, vp, vp, vp, vp, vp, vp, sz, vp]
        L.vs_select.restype = C.c_int
        L.vs_select.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.vs_select_static.restype = C.c_int
        L.vs_select_static.argtypes = [P, vp, vp, vp, vp, vp, vp, vp]
        L.vs_sparse_attn_prefill.restype = C.c_int
        L.vs_sparse_attn_prefill.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.vs_dense_causal_prefill.restype = C.c_int
        L.vs_dense_causal_prefill.argtypes = [P, vp, vp, vp, vp, vp, vp, sz, vp]
        L.vs_prefill_chunk.restype = C.c_int
        L.vs_prefill_chunk.argtypes = [P, vp, vp, vp, vp, vp, vp, sz, vp]
        L.vs_select_heads.restype = C.c_int
        L.vs_select_heads.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.vs_attention_recall.restype = C.c_int
        L.vs_attention_recall.argtypes = [P, vp, vp, vp, vp]
        L.vs_refine_step.restype = C.c_int
        L.vs_refine_step.argtypes = [P, vp, C.c_float, C.c_int32, C.c_int32, vp, vp, vp, vp]
        L.vs_chunk_cost.restype = C.c_double
        L.vs_chunk_cost.argtypes = [C.c_int64, C.c_int64, C.c_int32, C.c_int32, C.c_int32]
        L.vs_plan_chunks.restype = C.c_int
        L.vs_plan_chunks.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_int32, vp]
        L.vs_set_option.restype = C.c_int
        L.vs_set_option.argtypes = [C.c_int, C.c_int64]
        L.vs_count_tiles.restype = C.c_int
        L.vs_count_tiles.argtypes = [P, vp, vp, vp, vp, vp, vp, sz, vp]
        L.vs_batch_workspace_bytes.restype = sz
        L.vs_batch_workspace_bytes.argtypes = [P, C.c_int32]
        L.vs_attn_batch.restype = C.c_int
        L.vs_attn_batch.argtypes = [P, vp, C.c_int32, vp, sz, vp]
        DP = C.POINTER(VsDca)
        L.vs_estimate_dca.restype = C.c_int
        L.vs_estimate_dca.argtypes = [P, vp, DP, vp, vp, vp, vp, vp, sz, vp]
        L.vs_sparse_attn_prefill_dca.restype = C.c_int
        L.vs_sparse_attn_prefill_dca.argtypes = [P, vp, DP, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.vs_dense_causal_prefill_dca.restype = C.c_int
        L.vs_dense_causal_prefill_dca.argtypes = [P, vp, DP, vp, vp, vp, vp, vp, sz, vp]
        L.vs_prefill_chunk_dca.restype = C.c_int
        L.vs_prefill_chunk_dca.argtypes = [P, vp, DP, DP, vp, vp, vp, vp, vp, sz, vp]
        _lib = L
    return _lib


EXPORTS = ["vs_workspace_bytes", "vs_status_string", "vs_yarn_softmax_scale", "vs_estimate", "vs_select", "vs_select_static",
           "vs_sparse_attn_prefill", "vs_dense_causal_prefill", "vs_prefill_chunk", "vs_count_tiles",
           "vs_set_option", "vs_chunk_cost", "vs_plan_chunks", "vs_select_heads", "vs_attention_recall", "vs_refine_step",
           "vs_sparse_attn_prefill_dca", "vs_dense_causal_prefill_dca", "vs_estimate_dca", "vs_prefill_chunk_dca",
           "vs_batch_workspace_bytes", "vs_attn_batch"]


def status_string(status: int) -> str:
    return lib().vs_status_string(int(status)).decode()


def yarn_softmax_scale(s: float, head_dim: int) -> float:
    return float(lib().vs_yarn_softmax_scale(float(s), int(head_dim)))


@dataclass
class Chunk:
    """Parameters of one chunk call; strides are taken from the tensors at call time."""
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    q_len: int
    q_start: int
    softmax_scale: float
    last_q: int = 64
    block: int = 64
    vertical_budget: int = 1
    slash_budget: int = 1
    keep_first_cols: int = 1
    keep_local_band: int = 64

    @property
    def n_k(self) -> int:
        return self.q_start + self.q_len

    def params(self, q=None, k=None, v=None, out=None) -> VsParams:
        hq, hkv, d = self.n_q_heads, self.n_kv_heads, self.head_dim

        def st(t, heads):
            return (t.stride(0), t.stride(1)) if t is not None else (heads * d, d)

        qs, ks, vs_, os_ = st(q, hq), st(k, hkv), st(v, hkv), st(out, hq)
        return VsParams(hq, hkv, d, self.last_q, self.q_len, self.q_start, qs[0], qs[1], ks[0], ks[1],
                        vs_[0], vs_[1], os_[0], os_[1], float(self.softmax_scale), self.block,
                        self.vertical_budget, self.slash_budget, self.keep_first_cols, self.keep_local_band)


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc, where):
    if rc != VS_OK:
        raise VsError(rc, where)


VS_COST_DENSE, VS_COST_SPARSE = 0, 1


def chunk_cost(q_start: int, q_len: int, model: int, vertical_budget: int = 1, slash_budget: int = 1) -> float:
    """vs_chunk_cost (host): modelled 64x64 tiles per head of one chunk."""
    return float(lib().vs_chunk_cost(int(q_start), int(q_len), int(model), int(vertical_budget), int(slash_budget)))


def plan_chunks(n_ctx: int, n_chunks: int, model: int, vertical_budget: int = 1, slash_budget: int = 1):
    """vs_plan_chunks (host): n_chunks + 1 token boundaries of chunks of about equal modelled cost."""
    bounds = (C.c_int64 * (n_chunks + 1))()
    _check(lib().vs_plan_chunks(int(n_ctx), int(n_chunks), int(model), int(vertical_budget), int(slash_budget), bounds),
           "vs_plan_chunks")
    return list(bounds)


def set_option(which: int, value: int) -> None:
    """vs_set_option (process-wide tuning switch, e.g. VS_OPT_ATTN_SEGMENT_BLOCKS)."""
    _check(lib().vs_set_option(int(which), C.c_int64(int(value))), "vs_set_option")


def workspace_bytes(ck: Chunk, which: int) -> int:
    p = ck.params()
    return int(lib().vs_workspace_bytes(C.byref(p), which))


def _ws(ck: Chunk, which: int, device):
    n = workspace_bytes(ck, which)
    return torch.empty(max(n, 256), dtype=torch.uint8, device=device), n


def _chk_inner(t, name, d):
    assert t.dtype == torch.bfloat16 and t.dim() == 3 and t.stride(2) == 1 and t.shape[2] == d, name


def estimate(ck: Chunk, q, k, want_lse=False, vscore=None, sscore=None, ws=None, dca=None):
    """vs_estimate, or vs_estimate_dca when dca = (q_succ, q_inter, chunk, window) is given.
    q: bf16 [C][Hq][D] (the chunk), k: bf16 [>=n_k][Hkv][D].
    Returns vscore, sscore (fp32 [Hq][n_k]) and lse_lastq (fp32 [Hq][W'] or None).
    vscore / sscore / ws may be passed in to avoid allocating."""
    _chk_inner(q, "q", ck.head_dim); _chk_inner(k, "k", ck.head_dim)
    assert q.shape[0] == ck.q_len and k.shape[0] >= ck.n_k
    dev = q.device
    if vscore is None:
        vscore = torch.empty((ck.n_q_heads, ck.n_k), dtype=torch.float32, device=dev)
    if sscore is None:
        sscore = torch.empty((ck.n_q_heads, ck.n_k), dtype=torch.float32, device=dev)
    for t in (vscore, sscore):
        assert t.dtype == torch.float32 and t.is_contiguous() and t.shape == (ck.n_q_heads, ck.n_k)
    lse = torch.empty((ck.n_q_heads, min(ck.last_q, ck.q_len)), dtype=torch.float32, device=dev) if want_lse else None
    if ws is None:
        ws = torch.empty(max(workspace_bytes(ck, VS_WS_ESTIMATE), 256), dtype=torch.uint8, device=dev)
    p = ck.params(q=q, k=k)
    if dca is not None:
        d = _dca_struct(ck, q, dca)
        _check(lib().vs_estimate_dca(C.byref(p), _ptr(q), C.byref(d), _ptr(k), _ptr(vscore), _ptr(sscore), _ptr(lse),
                                     _ptr(ws), ws.numel(), _stream()), "vs_estimate_dca")
        return vscore, sscore, lse
    _check(lib().vs_estimate(C.byref(p), _ptr(q), _ptr(k), _ptr(vscore), _ptr(sscore), _ptr(lse),
                             _ptr(ws), ws.numel(), _stream()), "vs_estimate")
    return vscore, sscore, lse


def alloc_index_sets(ck: Chunk, device):
    """Uninitialised v_idx [Hq][Bv], v_cnt [Hq], s_idx [Hq][Bs], s_cnt [Hq] (int32)."""
    return (torch.empty((ck.n_q_heads, ck.vertical_budget), dtype=torch.int32, device=device),
            torch.empty(ck.n_q_heads, dtype=torch.int32, device=device),
            torch.empty((ck.n_q_heads, ck.slash_budget), dtype=torch.int32, device=device),
            torch.empty(ck.n_q_heads, dtype=torch.int32, device=device))


def select(ck: Chunk, vscore, sscore, sets=None):
    """vs_select.  Returns v_idx [Hq][Bv], v_cnt [Hq], s_idx [Hq][Bs], s_cnt [Hq] (int32);
    `sets` (from alloc_index_sets) may be passed in to avoid allocating."""
    assert vscore.dtype == torch.float32 and vscore.is_contiguous() and vscore.shape == (ck.n_q_heads, ck.n_k)
    assert sscore.dtype == torch.float32 and sscore.is_contiguous() and sscore.shape == (ck.n_q_heads, ck.n_k)
    dev = vscore.device
    v_idx, v_cnt, s_idx, s_cnt = alloc_index_sets(ck, dev) if sets is None else sets
    _sets_ok(ck, v_idx, v_cnt, s_idx, s_cnt)
    ws, n = _ws(ck, VS_WS_SELECT, dev)
    p = ck.params()
    _check(lib().vs_select(C.byref(p), _ptr(vscore), _ptr(sscore), _ptr(v_idx), _ptr(v_cnt), _ptr(s_idx),
                           _ptr(s_cnt), _ptr(ws) if n else C.c_void_p(0), n, _stream()), "vs_select")
    return v_idx, v_cnt, s_idx, s_cnt


def select_static(ck: Chunk, vscore, sscore, sets):
    """vs_select_static: vs_select with the library's own scratch array; `sets` (from alloc_index_sets) must be
    passed in, nothing is allocated on the way."""
    assert vscore.dtype == torch.float32 and vscore.is_contiguous() and vscore.shape == (ck.n_q_heads, ck.n_k)
    assert sscore.dtype == torch.float32 and sscore.is_contiguous() and sscore.shape == (ck.n_q_heads, ck.n_k)
    v_idx, v_cnt, s_idx, s_cnt = sets
    _sets_ok(ck, v_idx, v_cnt, s_idx, s_cnt)
    p = ck.params()
    _check(lib().vs_select_static(C.byref(p), _ptr(vscore), _ptr(sscore), _ptr(v_idx), _ptr(v_cnt), _ptr(s_idx),
                                  _ptr(s_cnt), _stream()), "vs_select_static")
    return v_idx, v_cnt, s_idx, s_cnt


def select_heads(ck: Chunk, vscore, sscore, v_budget_h, s_budget_h, sets=None):
    """vs_select_heads: vs_select with one (vertical, slash) budget pair per head (device int32 [Hq])."""
    assert vscore.dtype == torch.float32 and vscore.is_contiguous() and vscore.shape == (ck.n_q_heads, ck.n_k)
    assert sscore.dtype == torch.float32 and sscore.is_contiguous() and sscore.shape == (ck.n_q_heads, ck.n_k)
    for t in (v_budget_h, s_budget_h):
        assert t.dtype == torch.int32 and t.is_contiguous() and t.shape == (ck.n_q_heads,)
    dev = vscore.device
    v_idx, v_cnt, s_idx, s_cnt = alloc_index_sets(ck, dev) if sets is None else sets
    _sets_ok(ck, v_idx, v_cnt, s_idx, s_cnt)
    ws, n = _ws(ck, VS_WS_SELECT, dev)
    p = ck.params()
    _check(lib().vs_select_heads(C.byref(p), _ptr(vscore), _ptr(sscore), _ptr(v_budget_h), _ptr(s_budget_h),
                                 _ptr(v_idx), _ptr(v_cnt), _ptr(s_idx), _ptr(s_cnt),
                                 _ptr(ws) if n else C.c_void_p(0), n, _stream()), "vs_select_heads")
    return v_idx, v_cnt, s_idx, s_cnt


def attention_recall(ck: Chunk, lse_sparse, lse_full):
    """vs_attention_recall.  lse tensors fp32 [Hq][C] -> recall fp32 [Hq]."""
    for t in (lse_sparse, lse_full):
        assert t.dtype == torch.float32 and t.is_contiguous() and t.shape == (ck.n_q_heads, ck.q_len)
    recall = torch.empty((ck.n_q_heads,), dtype=torch.float32, device=lse_sparse.device)
    p = ck.params()
    _check(lib().vs_attention_recall(C.byref(p), _ptr(lse_sparse), _ptr(lse_full), _ptr(recall), _stream()),
           "vs_attention_recall")
    return recall


def refine_step(ck: Chunk, recall, threshold, add_vertical, add_slash, v_budget_h, s_budget_h):
    """vs_refine_step: budgets (device int32 [Hq]) grow in place; returns a device int32[1] with
    the number of heads that changed."""
    assert recall.dtype == torch.float32 and recall.shape == (ck.n_q_heads,)
    changed = torch.zeros((1,), dtype=torch.int32, device=recall.device)
    p = ck.params()
    _check(lib().vs_refine_step(C.byref(p), _ptr(recall), C.c_float(threshold), C.c_int32(add_vertical),
                                C.c_int32(add_slash), _ptr(v_budget_h), _ptr(s_budget_h), _ptr(changed), _stream()),
           "vs_refine_step")
    return changed


def _sets_ok(ck, v_idx, v_cnt, s_idx, s_cnt):
    for t in (v_idx, v_cnt, s_idx, s_cnt):
        assert t.dtype == torch.int32 and t.is_contiguous()
    assert v_idx.shape == (ck.n_q_heads, ck.vertical_budget) and s_idx.shape == (ck.n_q_heads, ck.slash_budget)


def _dca_struct(ck: Chunk, q, dca):
    """dca = (q_succ, q_inter, chunk, window); the two tensors must look like q."""
    q_succ, q_inter, chunk, window = dca
    for t, nm in ((q_succ, "q_succ"), (q_inter, "q_inter")):
        _chk_inner(t, nm, ck.head_dim)
        assert t.shape == q.shape and t.stride() == q.stride() and t.device == q.device, nm
    return VsDca(q_succ.data_ptr(), q_inter.data_ptr(), int(chunk), int(window))


def sparse_attn_prefill(ck: Chunk, q, k, v, v_idx, v_cnt, s_idx, s_cnt, want_lse=False, out=None, ws=None, dca=None):
    """vs_sparse_attn_prefill, or vs_sparse_attn_prefill_dca when dca = (q_succ, q_inter, chunk, window)
    is given (q is then the intra-chunk rotation).  Returns out bf16 [C][Hq][D] and lse fp32 [Hq][C] (or None)."""
    for t, nm in ((q, "q"), (k, "k"), (v, "v")):
        _chk_inner(t, nm, ck.head_dim)
    assert q.shape[0] == ck.q_len and k.shape[0] >= ck.n_k and v.shape[0] >= ck.n_k
    _sets_ok(ck, v_idx, v_cnt, s_idx, s_cnt)
    dev = q.device
    if out is None:
        out = torch.empty((ck.q_len, ck.n_q_heads, ck.head_dim), dtype=torch.bfloat16, device=dev)
    lse = torch.empty((ck.n_q_heads, ck.q_len), dtype=torch.float32, device=dev) if want_lse else None
    n = workspace_bytes(ck, VS_WS_SPARSE)
    if ws is None:
        ws = torch.empty(max(n, 256), dtype=torch.uint8, device=dev)
    p = ck.params(q=q, k=k, v=v, out=out)
    if dca is not None:
        d = _dca_struct(ck, q, dca)
        _check(lib().vs_sparse_attn_prefill_dca(C.byref(p), _ptr(q), C.byref(d), _ptr(k), _ptr(v), _ptr(v_idx),
                                                _ptr(v_cnt), _ptr(s_idx), _ptr(s_cnt), _ptr(out), _ptr(lse),
                                                _ptr(ws), ws.numel(), _stream()), "vs_sparse_attn_prefill_dca")
        return out, lse
    _check(lib().vs_sparse_attn_prefill(C.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(v_idx), _ptr(v_cnt),
                                        _ptr(s_idx), _ptr(s_cnt), _ptr(out), _ptr(lse), _ptr(ws), ws.numel(),
                                        _stream()), "vs_sparse_attn_prefill")
    return out, lse


def dense_causal_prefill(ck: Chunk, q, k, v, want_lse=False, out=None, ws=None, dca=None):
    """vs_dense_causal_prefill, or vs_dense_causal_prefill_dca when dca = (q_succ, q_inter, chunk, window)
    is given.  Returns out bf16 [C][Hq][D] and lse fp32 [Hq][C] (or None)."""
    for t, nm in ((q, "q"), (k, "k"), (v, "v")):
        _chk_inner(t, nm, ck.head_dim)
    assert q.shape[0] == ck.q_len and k.shape[0] >= ck.n_k and v.shape[0] >= ck.n_k
    dev = q.device
    if out is None:
        out = torch.empty((ck.q_len, ck.n_q_heads, ck.head_dim), dtype=torch.bfloat16, device=dev)
    lse = torch.empty((ck.n_q_heads, ck.q_len), dtype=torch.float32, device=dev) if want_lse else None
    n = workspace_bytes(ck, VS_WS_DENSE)
    if ws is None:
        ws = torch.empty(max(n, 256), dtype=torch.uint8, device=dev)
    p = ck.params(q=q, k=k, v=v, out=out)
    if dca is not None:
        d = _dca_struct(ck, q, dca)
        _check(lib().vs_dense_causal_prefill_dca(C.byref(p), _ptr(q), C.byref(d), _ptr(k), _ptr(v), _ptr(out),
                                                 _ptr(lse), _ptr(ws), ws.numel(), _stream()),
               "vs_dense_causal_prefill_dca")
        return out, lse
    _check(lib().vs_dense_causal_prefill(C.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), _ptr(ws),
                                         ws.numel(), _stream()), "vs_dense_causal_prefill")
    return out, lse


def prefill_chunk(ck: Chunk, q, k, v, want_lse=False, out=None, ws=None, dca=None, dca_select=None):
    """vs_prefill_chunk: estimate -> select -> sparse attention on the current stream; with
    dca = (q_succ, q_inter, chunk, window) vs_prefill_chunk_dca (dca_select: the rotations the
    estimate uses, default those of dca)."""
    for t, nm in ((q, "q"), (k, "k"), (v, "v")):
        _chk_inner(t, nm, ck.head_dim)
    assert q.shape[0] == ck.q_len and k.shape[0] >= ck.n_k and v.shape[0] >= ck.n_k
    dev = q.device
    if out is None:
        out = torch.empty((ck.q_len, ck.n_q_heads, ck.head_dim), dtype=torch.bfloat16, device=dev)
    lse = torch.empty((ck.n_q_heads, ck.q_len), dtype=torch.float32, device=dev) if want_lse else None
    n = workspace_bytes(ck, VS_WS_CHUNK)
    if ws is None:
        ws = torch.empty(max(n, 256), dtype=torch.uint8, device=dev)
    p = ck.params(q=q, k=k, v=v, out=out)
    if dca is not None:
        d = _dca_struct(ck, q, dca)
        ds = _dca_struct(ck, q, dca_select) if dca_select is not None else None
        _check(lib().vs_prefill_chunk_dca(C.byref(p), _ptr(q), C.byref(d), C.byref(ds) if ds is not None else None,
                                          _ptr(k), _ptr(v), _ptr(out), _ptr(lse), _ptr(ws), ws.numel(), _stream()),
               "vs_prefill_chunk_dca")
        return out, lse
    _check(lib().vs_prefill_chunk(C.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), _ptr(ws),
                                  ws.numel(), _stream()), "vs_prefill_chunk")
    return out, lse


def count_tiles(ck: Chunk, v_idx, v_cnt, s_idx, s_cnt):
    """vs_count_tiles.  Returns int64 [Hq][2] = (slash tiles, vertical tiles) issued for the chunk."""
    _sets_ok(ck, v_idx, v_cnt, s_idx, s_cnt)
    dev = v_idx.device
    tiles = torch.empty((ck.n_q_heads, 2), dtype=torch.int64, device=dev)
    ws, n = _ws(ck, VS_WS_COUNT_TILES, dev)
    p = ck.params()
    _check(lib().vs_count_tiles(C.byref(p), _ptr(v_idx), _ptr(v_cnt), _ptr(s_idx), _ptr(s_cnt), _ptr(tiles),
                                _ptr(ws), n, _stream()), "vs_count_tiles")
    return tiles


def request_table(requests, device):
    """The device array of vs_request for vs_attn_batch.  requests: dicts with q, k, v, out (bf16 tensors),
    q_start, and optionally lse (fp32 [Hq][q_len]) and sets = (v_idx, v_cnt, s_idx, s_cnt) (absent: dense).
    Returns an int64 tensor [n][11] (every field of vs_request is eight bytes); the tensors it points
    to must stay alive until the call has run."""
    rows = []
    for r in requests:
        sets = r.get("sets")
        lse = r.get("lse")
        rows.append([r["q"].data_ptr(), r["k"].data_ptr(), r["v"].data_ptr(), r["out"].data_ptr(),
                     lse.data_ptr() if lse is not None else 0] +
                    ([t.data_ptr() for t in sets] if sets is not None else [0, 0, 0, 0]) +
                    [int(r["q_start"]), int(r["q"].shape[0])])
    assert C.sizeof(VsRequest) == 88
    return torch.tensor(rows, dtype=torch.int64).to(device)


def attn_batch(ck: Chunk, table, n_requests, q, k, v, out, ws=None):
    """vs_attn_batch.  ck: the shared shape with q_len = the longest request and q_start + q_len = the most
    keys any request sees; table: from request_table; q / k / v / out: one request's tensors, for the strides."""
    p = ck.params(q=q, k=k, v=v, out=out)
    n = int(lib().vs_batch_workspace_bytes(C.byref(p), int(n_requests)))
    if ws is None:
        ws = torch.empty(max(n, 256), dtype=torch.uint8, device=table.device)
    _check(lib().vs_attn_batch(C.byref(p), _ptr(table), int(n_requests), _ptr(ws), ws.numel(), _stream()), "vs_attn_batch")
    return ws
