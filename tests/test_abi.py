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
    for st in (0, -1, -2, -3, -4, -5, -99):
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


def test_dca_descriptor_is_checked_on_the_host():
    L = vs.lib()
    p = _good().params()
    ok, odd = C.c_void_p(4096), C.c_void_p(4100)

    def dca(q_succ=4096, q_inter=4096, chunk=128, window=64):
        return vs.VsDca(q_succ, q_inter, chunk, window)

    def dense(d):
        return L.vs_dense_causal_prefill_dca(C.byref(p), ok, C.byref(d) if d is not None else None, ok, ok, ok, None,
                                             None, 0, None)

    assert dense(None) == vs.VS_ERR_INVALID_ARG
    assert dense(dca(q_succ=None)) == vs.VS_ERR_INVALID_ARG
    assert dense(dca(q_inter=4100)) == vs.VS_ERR_INVALID_ARG
    assert dense(dca(chunk=0)) == vs.VS_ERR_INVALID_ARG
    assert dense(dca(window=-64)) == vs.VS_ERR_INVALID_ARG
    assert dense(dca(chunk=100)) == vs.VS_ERR_UNSUPPORTED
    assert dense(dca(window=65)) == vs.VS_ERR_UNSUPPORTED
    assert dense(dca()) == vs.VS_ERR_WORKSPACE          # the descriptor is fine: the next check is the workspace
    d = dca(chunk=100)
    assert L.vs_estimate_dca(C.byref(p), ok, C.byref(d), ok, ok, ok, None, ok, 1 << 30, None) == vs.VS_ERR_UNSUPPORTED
    assert L.vs_sparse_attn_prefill_dca(C.byref(p), ok, C.byref(d), ok, ok, ok, ok, ok, ok, ok, None, ok, 1 << 30,
                                        None) == vs.VS_ERR_UNSUPPORTED
    assert L.vs_prefill_chunk_dca(C.byref(p), ok, C.byref(d), None, ok, ok, ok, None, ok, 1 << 30, None) == vs.VS_ERR_UNSUPPORTED
    good, bad_sel = dca(), dca(window=65)
    assert L.vs_prefill_chunk_dca(C.byref(p), ok, C.byref(good), C.byref(bad_sel), ok, ok, ok, None, ok, 1 << 30,
                                  None) == vs.VS_ERR_UNSUPPORTED
    assert L.vs_estimate_dca(C.byref(p), odd, C.byref(good), ok, ok, ok, None, ok, 1 << 30, None) == vs.VS_ERR_INVALID_ARG
    # a bad attention descriptor is found before the estimate and the selection are enqueued, although
    # the selection's own descriptor is fine (nothing may reach the stream when a status is negative)
    bad_att = dca(chunk=100)
    assert L.vs_prefill_chunk_dca(C.byref(p), ok, C.byref(bad_att), C.byref(good), ok, ok, ok, None, ok, 1 << 30,
                                  None) == vs.VS_ERR_UNSUPPORTED
    bad_att = dca(q_succ=None)
    assert L.vs_prefill_chunk_dca(C.byref(p), ok, C.byref(bad_att), C.byref(good), ok, ok, ok, None, ok, 1 << 30,
                                  None) == vs.VS_ERR_INVALID_ARG


def test_dca_entry_points_have_prototypes():
    """Every pointer and the size_t workspace size of the _dca calls go through declared argument types
    (a workspace of 2 GiB or more would not survive ctypes' default int conversion)."""
    L = vs.lib()
    for name, n_args in (("vs_estimate_dca", 10), ("vs_sparse_attn_prefill_dca", 14),
                         ("vs_dense_causal_prefill_dca", 10), ("vs_prefill_chunk_dca", 11)):
        fn = getattr(L, name)
        assert fn.argtypes is not None and len(fn.argtypes) == n_args, name
        assert fn.argtypes[-2] is C.c_size_t and fn.restype is C.c_int, name
        assert fn.argtypes[2] == C.POINTER(vs.VsDca), name
    p = _good().params()
    ok = C.c_void_p(4096)
    d = vs.VsDca(4096, 4096, 128, 64)
    # 3 GiB stated, but the pointer is null: the size must arrive whole for the check to say "workspace"
    assert L.vs_dense_causal_prefill_dca(C.byref(p), ok, C.byref(d), ok, ok, ok, None, None, 3 << 30, None) == vs.VS_ERR_WORKSPACE


def test_options_and_the_workspaces_they_change():
    ck = vs.Chunk(4, 1, 128, 64, 64 * 1024, 0.1, vertical_budget=8, slash_budget=70)   # one short chunk, long cache
    try:
        vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, 1)
        unsplit = vs.workspace_bytes(ck, vs.VS_WS_DENSE)
        vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, 0)
        auto = vs.workspace_bytes(ck, vs.VS_WS_DENSE)
        vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, 2)
        two = vs.workspace_bytes(ck, vs.VS_WS_DENSE)
        # partial results: (D + 2) floats per row, head and range, each array rounded up to 256 bytes
        assert two - unsplit == 2 * 4 * 64 * 128 * 4 + 2 * 4 * 64 * 2 * 4
        assert auto - unsplit == 8 * (two - unsplit)          # 16 ranges chosen for 4 units
        for bad in (-1, 17):
            with pytest.raises(vs.VsError):
                vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, bad)
        with pytest.raises(vs.VsError):
            vs.set_option(99, 0)
        with pytest.raises(vs.VsError):
            vs.set_option(vs.VS_OPT_ATTN_ROUNDS_IN_TURN, 2)
        vs.set_option(vs.VS_OPT_ATTN_ROUNDS_IN_TURN, 1)
        vs.set_option(vs.VS_OPT_ATTN_ROUNDS_IN_TURN, 0)
    finally:
        vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, 0)
    # the size query and the call must see the same options: a workspace sized under one setting is
    # refused, on the host, by a call made under a setting that needs more
    L = vs.lib()
    ok = C.c_void_p(4096)
    p = ck.params()
    vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, 1)
    small = vs.workspace_bytes(ck, vs.VS_WS_DENSE)
    vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, 0)
    assert L.vs_dense_causal_prefill(C.byref(p), ok, ok, ok, ok, None, ok, small, None) == vs.VS_ERR_WORKSPACE
    # a long chunk is never split
    long_ck = vs.Chunk(28, 4, 128, 32768, 32768, 0.1, vertical_budget=8, slash_budget=70)
    vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, 1)
    a = vs.workspace_bytes(long_ck, vs.VS_WS_DENSE)
    vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, 0)
    assert vs.workspace_bytes(long_ck, vs.VS_WS_DENSE) == a
    assert vs.workspace_bytes(long_ck, vs.VS_WS_SELECT) > 0
    L = vs.lib()
    ok = C.c_void_p(4096)
    p = long_ck.params()
    assert L.vs_select(C.byref(p), ok, ok, ok, ok, ok, ok, None, 0, None) == vs.VS_ERR_WORKSPACE


def test_static_select_checks_its_capacity_on_the_host():
    """vs_select_static holds 128 query heads; more is refused before any device work."""
    L = vs.lib()
    ok = C.c_void_p(4096)
    big = vs.Chunk(160, 160, 64, 64, 0, 0.1, vertical_budget=4, slash_budget=70).params()
    assert L.vs_select_static(C.byref(big), ok, ok, ok, ok, ok, ok, None) == vs.VS_ERR_TOO_LARGE
    assert "128" in vs.status_string(vs.VS_ERR_TOO_LARGE)
    p = _good().params()
    assert L.vs_select_static(C.byref(p), None, ok, ok, ok, ok, ok, None) == vs.VS_ERR_INVALID_ARG
    bad = _good(); bad.slash_budget = 0
    assert L.vs_select_static(C.byref(bad.params()), ok, ok, ok, ok, ok, ok, None) == vs.VS_ERR_INVALID_ARG


def test_batch_argument_checks():
    """vs_attn_batch: request table, counts, bounds and workspace are checked on the host."""
    ck = vs.Chunk(4, 1, 64, 16, 0, 0.125, vertical_budget=8, slash_budget=70)
    p = ck.params()
    L = vs.lib()
    ok = C.c_void_p(4096)
    assert L.vs_attn_batch(C.byref(p), None, 2, ok, 1 << 30, None) == vs.VS_ERR_INVALID_ARG
    assert L.vs_attn_batch(C.byref(p), ok, 0, ok, 1 << 30, None) == vs.VS_ERR_INVALID_ARG
    assert L.vs_attn_batch(C.byref(p), ok, 5000, ok, 1 << 30, None) == vs.VS_ERR_UNSUPPORTED
    assert L.vs_attn_batch(C.byref(p), ok, 2, ok, 16, None) == vs.VS_ERR_WORKSPACE
    long = vs.Chunk(4, 1, 64, 5000, 0, 0.125, vertical_budget=8, slash_budget=70).params()
    assert L.vs_attn_batch(C.byref(long), ok, 2, ok, 1 << 30, None) == vs.VS_ERR_UNSUPPORTED
    assert L.vs_batch_workspace_bytes(C.byref(long), 2) == 0
