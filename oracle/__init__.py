"""ctypes front end of the fp64 CPU oracle (oracle/vs_oracle.c).

TEST INFRASTRUCTURE, NOT THE PRODUCT: only tests, the smoke check and the
benchmark's cpu_baseline leg may import this package.  It imports nothing from
the HIP package and the HIP package imports nothing from here.

All tensors are numpy arrays on the host.  Q/K/V are bf16 bit patterns held as
``uint16`` arrays of shape ``[tokens][heads][D]`` (C-contiguous).  Everything
the oracle returns is fp64 (scores, outputs, lse) or int32 (index sets).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "vs_oracle.c")
_LIB = os.path.join(_HERE, "libvs_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (fp64, OpenMP across independent rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Params(C.Structure):
    _fields_ = [
        ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("q_len", C.c_int64), ("q_start", C.c_int64),
        ("q_stride_tok", C.c_int64), ("q_stride_head", C.c_int64),
        ("k_stride_tok", C.c_int64), ("k_stride_head", C.c_int64),
        ("v_stride_tok", C.c_int64), ("v_stride_head", C.c_int64),
        ("softmax_scale", C.c_double),
        ("last_q", C.c_int32), ("block", C.c_int32),
        ("vertical_budget", C.c_int32), ("slash_budget", C.c_int32),
        ("keep_first_cols", C.c_int32), ("keep_local_band", C.c_int32),
    ]


@dataclass
class Problem:
    """One chunk of one attention layer, in the paper's terms (section 5.2)."""
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    q_len: int            # C, rows of the chunk
    q_start: int          # s, absolute position of the chunk's first row
    softmax_scale: float
    last_q: int = 64      # W: the last 64 tokens of each chunk
    block: int = 64       # B
    vertical_budget: int = 0
    slash_budget: int = 0
    keep_first_cols: int = 1
    keep_local_band: int = 64

    @property
    def n_k(self) -> int:
        return self.q_start + self.q_len

    def _c(self) -> _Params:
        hq, hkv, d = self.n_q_heads, self.n_kv_heads, self.head_dim
        return _Params(hq, hkv, d, self.q_len, self.q_start, hq * d, d, hkv * d, d,
                       hkv * d, d, float(self.softmax_scale), self.last_q, self.block,
                       self.vertical_budget, self.slash_budget,
                       self.keep_first_cols, self.keep_local_band)


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.vso_yarn_softmax_scale.restype = C.c_double
        _lib.vso_yarn_softmax_scale.argtypes = [C.c_double, C.c_int]
    return _lib


def _p(a, ty):
    return a.ctypes.data_as(C.POINTER(ty)) if a is not None else None


def _u16(a, shape_tail):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16 and a.shape[1:] == tuple(shape_tail), (a.dtype, a.shape, shape_tail)
    return a


def num_threads() -> int:
    return int(lib().vso_num_threads())


def yarn_softmax_scale(s: float, head_dim: int) -> float:
    return float(lib().vso_yarn_softmax_scale(float(s), int(head_dim)))


def attention_recall(lse_sparse, lse_full):
    """Attention_Recall of every query: exp(softmax_lse_sparse - softmax_lse_full)
    ("Sparsity refinement" paragraph), the definition written out."""
    return np.exp(np.asarray(lse_sparse, np.float64) - np.asarray(lse_full, np.float64))


def recall_mean(lse_sparse, lse_full):
    """Per-head attention recall of a chunk: mean over rows of exp(lse_sparse - lse_full).
    lse arrays [nh][rows] -> [nh]."""
    a = np.ascontiguousarray(lse_sparse, np.float64); b = np.ascontiguousarray(lse_full, np.float64)
    assert a.shape == b.shape and a.ndim == 2
    L = lib()
    L.vso_recall_mean.restype = C.c_double
    return np.array([L.vso_recall_mean(_p(a[h], C.c_double), _p(b[h], C.c_double), C.c_int64(a.shape[1]))
                     for h in range(a.shape[0])])


def refine_step(recall, threshold, dv, ds, v_max, s_max, v_budget, s_budget):
    """One pass of the sparsity refinement over the heads.  Returns (v_budget, s_budget, changed)."""
    recall = np.ascontiguousarray(recall, np.float64)
    vb = np.array(v_budget, np.int32); sb = np.array(s_budget, np.int32)
    L = lib()
    L.vso_refine_step.restype = C.c_int
    ch = L.vso_refine_step(C.c_int(len(recall)), _p(recall, C.c_double), C.c_double(threshold), C.c_int32(dv),
                           C.c_int32(ds), C.c_int32(v_max), C.c_int32(s_max), _p(vb, C.c_int32), _p(sb, C.c_int32))
    return vb, sb, int(ch)


def select_heads(pb: Problem, vscore, sscore, v_budget, s_budget):
    """Step 2 with one (vertical, slash) budget pair per head; rows padded with -1 to the
    budgets of `pb` (the maxima)."""
    nh = len(v_budget)
    v_idx = np.full((nh, pb.vertical_budget), -1, np.int32); v_cnt = np.zeros(nh, np.int32)
    s_idx = np.full((nh, pb.slash_budget), -1, np.int32); s_cnt = np.zeros(nh, np.int32)
    for h in range(nh):
        assert 1 <= v_budget[h] <= pb.vertical_budget and 1 <= s_budget[h] <= pb.slash_budget
        v = select_one(vscore[h], int(v_budget[h]), pb.keep_first_cols)
        s = select_one(sscore[h], int(s_budget[h]), pb.keep_local_band)
        v_idx[h, :len(v)] = v; v_cnt[h] = len(v); s_idx[h, :len(s)] = s; s_cnt[h] = len(s)
    return v_idx, v_cnt, s_idx, s_cnt


@dataclass
class Dca:
    """Dual Chunk Attention (section 5.1): chunk length, local window and the two other
    rotations of the chunk's queries (u16 [C][Hq][D] each); q itself is the intra-chunk one."""
    chunk: int
    window: int
    q_succ: np.ndarray
    q_inter: np.ndarray


def dca_region(pos_q: int, pos_k: int, chunk: int, window: int) -> int:
    """0 intra-chunk, 1 successive-chunk (inside the local window), 2 inter-chunk."""
    return int(lib().vso_dca_region(C.c_int64(pos_q), C.c_int64(pos_k), C.c_int64(chunk), C.c_int64(window)))


def estimate(pb: Problem, q, k, heads=None, dca: Dca | None = None):
    """Step 1.  q: [C][Hq][D] u16 (the chunk), k: [>=n_k][Hkv][D] u16.
    Returns vscore [nh][n_k], sscore [nh][n_k], lse_lastq [nh][W'] (fp64)."""
    q = _u16(q, (pb.n_q_heads, pb.head_dim)); k = _u16(k, (pb.n_kv_heads, pb.head_dim))
    assert q.shape[0] == pb.q_len and k.shape[0] >= pb.n_k
    if dca is not None:
        qs = _u16(dca.q_succ, (pb.n_q_heads, pb.head_dim)); qi = _u16(dca.q_inter, (pb.n_q_heads, pb.head_dim))
        assert qs.shape == q.shape and qi.shape == q.shape and dca.chunk > 0 and dca.window >= 0
        heads = np.arange(pb.n_q_heads, dtype=np.int32) if heads is None else np.asarray(heads, np.int32)
        wp = min(pb.last_q, pb.q_len)
        vs = np.zeros((len(heads), pb.n_k)); ss = np.zeros((len(heads), pb.n_k)); lse = np.zeros((len(heads), wp))
        prm = pb._c()
        rc = lib().vso_estimate_dca(C.byref(prm), _p(q, C.c_uint16), _p(qs, C.c_uint16), _p(qi, C.c_uint16),
                                    C.c_int64(dca.chunk), C.c_int64(dca.window), _p(k, C.c_uint16), len(heads),
                                    _p(heads, C.c_int32), _p(vs, C.c_double), _p(ss, C.c_double), _p(lse, C.c_double))
        assert rc == 0
        return vs, ss, lse
    heads = np.arange(pb.n_q_heads, dtype=np.int32) if heads is None else np.asarray(heads, np.int32)
    wp = min(pb.last_q, pb.q_len)
    vs = np.zeros((len(heads), pb.n_k)); ss = np.zeros((len(heads), pb.n_k))
    lse = np.zeros((len(heads), wp))
    prm = pb._c()
    rc = lib().vso_estimate(C.byref(prm), _p(q, C.c_uint16), _p(k, C.c_uint16), len(heads),
                            _p(heads, C.c_int32), _p(vs, C.c_double), _p(ss, C.c_double),
                            _p(lse, C.c_double))
    assert rc == 0
    return vs, ss, lse


def select_one(score, budget: int, n_forced: int):
    """Step 2 for one score vector: ascending indices of the kept set."""
    score = np.ascontiguousarray(score, np.float64)
    n = score.shape[0]
    out = np.full(max(min(budget, n), 1), -1, np.int32)
    cnt = C.c_int32(0)
    rc = lib().vso_select_one(C.c_int64(n), _p(score, C.c_double), C.c_int64(budget),
                              C.c_int64(min(n_forced, n)), _p(out, C.c_int32), C.byref(cnt))
    assert rc == 0
    return out[:cnt.value].copy()


def select(pb: Problem, vscore, sscore):
    """Step 2 for every head.  Returns v_idx [nh][Bv], v_cnt [nh], s_idx [nh][Bs], s_cnt [nh]."""
    vscore = np.ascontiguousarray(vscore, np.float64); sscore = np.ascontiguousarray(sscore, np.float64)
    nh = vscore.shape[0]
    assert vscore.shape == (nh, pb.n_k) and sscore.shape == (nh, pb.n_k)
    v_idx = np.full((nh, pb.vertical_budget), -1, np.int32); v_cnt = np.zeros(nh, np.int32)
    s_idx = np.full((nh, pb.slash_budget), -1, np.int32); s_cnt = np.zeros(nh, np.int32)
    prm = pb._c()
    rc = lib().vso_select(C.byref(prm), nh, _p(vscore, C.c_double), _p(sscore, C.c_double),
                          _p(v_idx, C.c_int32), _p(v_cnt, C.c_int32),
                          _p(s_idx, C.c_int32), _p(s_cnt, C.c_int32))
    assert rc == 0
    return v_idx, v_cnt, s_idx, s_cnt


def mask(pb: Problem, v_idx, s_idx, rows=None):
    """The computed 0/1 mask [n_rows][n_k] of one head's index sets (step 3)."""
    v_idx = np.ascontiguousarray(v_idx, np.int32); s_idx = np.ascontiguousarray(s_idx, np.int32)
    rows = np.arange(pb.q_len, dtype=np.int64) if rows is None else np.asarray(rows, np.int64)
    m = np.zeros((len(rows), pb.n_k), np.uint8)
    prm = pb._c()
    rc = lib().vso_mask(C.byref(prm), _p(v_idx, C.c_int32), C.c_int32(len(v_idx)),
                        _p(s_idx, C.c_int32), C.c_int32(len(s_idx)), C.c_int64(len(rows)),
                        _p(rows, C.c_int64), _p(m, C.c_uint8))
    assert rc == 0
    return m


def _attention(pb, q, k, v, sets, heads, rows, dca=None):
    q = _u16(q, (pb.n_q_heads, pb.head_dim)); k = _u16(k, (pb.n_kv_heads, pb.head_dim))
    v = _u16(v, (pb.n_kv_heads, pb.head_dim))
    assert q.shape[0] == pb.q_len and k.shape[0] >= pb.n_k and v.shape[0] >= pb.n_k
    heads = np.arange(pb.n_q_heads, dtype=np.int32) if heads is None else np.asarray(heads, np.int32)
    rows = np.arange(pb.q_len, dtype=np.int64) if rows is None else np.asarray(rows, np.int64)
    assert rows.size == 0 or (rows.min() >= 0 and rows.max() < pb.q_len)
    out = np.zeros((len(heads), len(rows), pb.head_dim)); lse = np.zeros((len(heads), len(rows)))
    prm = pb._c()
    if sets is None:
        a = (None, None, None, None)
    else:
        v_idx, v_cnt, s_idx, s_cnt = [np.ascontiguousarray(x, np.int32) for x in sets]
        assert v_idx.shape == (pb.n_q_heads, pb.vertical_budget)
        assert s_idx.shape == (pb.n_q_heads, pb.slash_budget)
        a = (v_idx, v_cnt, s_idx, s_cnt)
    tail = (_p(a[0], C.c_int32), _p(a[1], C.c_int32), _p(a[2], C.c_int32),
            _p(a[3], C.c_int32), len(heads), _p(heads, C.c_int32),
            C.c_int64(len(rows)), _p(rows, C.c_int64), _p(out, C.c_double), _p(lse, C.c_double))
    if dca is None:
        rc = lib().vso_attention(C.byref(prm), _p(q, C.c_uint16), _p(k, C.c_uint16), _p(v, C.c_uint16), *tail)
    else:
        qs = _u16(dca.q_succ, (pb.n_q_heads, pb.head_dim)); qi = _u16(dca.q_inter, (pb.n_q_heads, pb.head_dim))
        assert qs.shape == q.shape and qi.shape == q.shape and dca.chunk > 0 and dca.window >= 0
        rc = lib().vso_attention_dca(C.byref(prm), _p(q, C.c_uint16), _p(qs, C.c_uint16), _p(qi, C.c_uint16),
                                     C.c_int64(dca.chunk), C.c_int64(dca.window), _p(k, C.c_uint16),
                                     _p(v, C.c_uint16), *tail)
    assert rc == 0
    return out, lse


def sparse_attention(pb: Problem, q, k, v, v_idx, v_cnt, s_idx, s_cnt, heads=None, rows=None, dca: Dca | None = None):
    """Step 3.  Index sets are [Hq][Bv] / [Hq][Bs] for ALL heads; ``heads``/``rows``
    pick which outputs are computed.  Returns out [nh][nr][D], lse [nh][nr] (fp64)."""
    return _attention(pb, q, k, v, (v_idx, v_cnt, s_idx, s_cnt), heads, rows, dca)


def dense_attention(pb: Problem, q, k, v, heads=None, rows=None, dca: Dca | None = None):
    """Step 4: causal softmax attention over every key j <= pos(i)."""
    return _attention(pb, q, k, v, None, heads, rows, dca)
