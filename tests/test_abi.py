"""The C-ABI library: it loads without a GPU, exports every symbol include/vs.h declares,
and rejects bad arguments on the host before any HIP call."""
import ctypes as C
import os
import re

import pytest

import paper_2501_15383_amd as vs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    txt = open(os.path.join(ROOT, "include", "vs.h")).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    return sorted(set(re.findall(r"\b(vs_[a-z_]+)\s*\(", txt)))


def test_every_declared_symbol_is_exported():
    L = vs.lib()
    names = _declared()
    assert set(names) == set(vs.EXPORTS), names
    for n in names:
        assert hasattr(L, n), n


def test_params_struct_matches_header_field_order():
    txt = open(os.path.join(ROOT, "include", "vs.h")).read()
    body = re.search(r"typedef struct vs_params \{(.*?)\} vs_params;", txt, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = []
    for decl in body.split(";"):
        decl = decl.strip()
        if decl:
            fields += [x.strip() for x in decl.split(None, 1)[1].split(",")]
    assert fields == [f[0] for f in vs.VsParams._fields_]


def _good():
    return vs.Chunk(4, 1, 64, 128, 256, 0.125, vertical_budget=8, slash_budget=70)


def test_status_strings_and_workspace_sizes():
    for st in (0, -1, -2, -3, -4, -99):
        assert isinstance(vs.status_string(st), str) and vs.status_string(st)
    ck = _good()
    assert vs.workspace_bytes(ck, vs.VS_WS_ESTIMATE) > 0
    assert vs.workspace_bytes(ck, vs.VS_WS_SPARSE) >= vs.workspace_bytes(ck, vs.VS_WS_DENSE) > 0
    assert vs.workspace_bytes(ck, vs.VS_WS_CHUNK) > vs.workspace_bytes(ck, vs.VS_WS_ESTIMATE)
    assert vs.workspace_bytes(ck, 17) == 0
    bad = _good(); bad.head_dim = 80
    assert vs.workspace_bytes(bad, vs.VS_WS_ESTIMATE) == 0


def test_yarn_scale_helper():
    assert abs(vs.yarn_softmax_scale(4.0, 64) * 8 - 1.2964770) < 1e-5
    assert vs.yarn_softmax_scale(1.0, 64) == 0.125
    assert vs.yarn_softmax_scale(0.5, 64) == 0.0


@pytest.mark.parametrize("mut,status", [
    (dict(head_dim=96), vs.VS_ERR_UNSUPPORTED),
    (dict(block=32), vs.VS_ERR_UNSUPPORTED),
    (dict(last_q=65), vs.VS_ERR_UNSUPPORTED),
    (dict(q_start=100), vs.VS_ERR_UNSUPPORTED),
    (dict(n_kv_heads=3), vs.VS_ERR_INVALID_ARG),
    (dict(q_len=0), vs.VS_ERR_INVALID_ARG),
    (dict(softmax_scale=0.0), vs.VS_ERR_INVALID_ARG),
    (dict(softmax_scale=float("nan")), vs.VS_ERR_INVALID_ARG),
    (dict(vertical_budget=0), vs.VS_ERR_INVALID_ARG),
    (dict(keep_local_band=-1), vs.VS_ERR_INVALID_ARG),
    (dict(q_start=2**31), vs.VS_ERR_INVALID_ARG),
])
def test_bad_parameters_are_rejected_before_any_device_work(mut, status):
    ck = _good()
    for k, v in mut.items():
        setattr(ck, k, v)
    p = ck.params()
    L = vs.lib()
    fake = C.c_void_p(4096)   # never dereferenced: validation fails first
    rc = L.vs_sparse_attn_prefill(C.byref(p), fake, fake, fake, fake, fake, fake, fake, fake, None, fake, 1 << 30, None)
    assert rc == status
    rc = L.vs_prefill_chunk(C.byref(p), fake, fake, fake, fake, None, fake, 1 << 30, None)
    assert rc == status


def test_null_misaligned_and_workspace_errors():
    L = vs.lib()
    p = _good().params()
    ok, odd = C.c_void_p(4096), C.c_void_p(4100)
    assert L.vs_estimate(None, ok, ok, ok, ok, None, ok, 1 << 30, None) == vs.VS_ERR_INVALID_ARG
    assert L.vs_estimate(C.byref(p), None, ok, ok, ok, None, ok, 1 << 30, None) == vs.VS_ERR_INVALID_ARG
    assert L.vs_estimate(C.byref(p), odd, ok, ok, ok, None, ok, 1 << 30, None) == vs.VS_ERR_INVALID_ARG
    assert L.vs_estimate(C.byref(p), ok, ok, ok, ok, None, None, 0, None) == vs.VS_ERR_WORKSPACE
    assert L.vs_estimate(C.byref(p), ok, ok, ok, ok, None, ok, 16, None) == vs.VS_ERR_WORKSPACE
    assert L.vs_estimate(C.byref(p), ok, ok, ok, ok, None, C.c_void_p(4096 + 64), 1 << 30, None) == vs.VS_ERR_WORKSPACE
    assert L.vs_dense_causal_prefill(C.byref(p), ok, ok, ok, None, None, ok, 1 << 30, None) == vs.VS_ERR_INVALID_ARG
    assert L.vs_select(C.byref(p), ok, ok, ok, ok, ok, None, None, 0, None) == vs.VS_ERR_INVALID_ARG
    assert L.vs_count_tiles(C.byref(p), ok, ok, ok, ok, None, ok, 1 << 30, None) == vs.VS_ERR_INVALID_ARG
    bad = _good().params(); bad.k_stride_tok = 60
    assert L.vs_dense_causal_prefill(C.byref(bad), ok, ok, ok, ok, None, ok, 1 << 30, None) == vs.VS_ERR_INVALID_ARG
