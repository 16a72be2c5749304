"""vs_select_static, the entry point for callers that cannot allocate: its scratch is a device
array inside the library.  Checked through the C ABI against vs_select (same kernels, caller
workspace) bit for bit, on two calls in a row, the second with a smaller input -- the array
keeps the first call's contents, and the second call must not see them."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2501_15383_amd as vs

pytestmark = pytest.mark.gpu


def _call_static(ck, vsc, ssc):
    sets = vs.alloc_index_sets(ck, vsc.device)
    for t in sets:
        t.fill_(-7)          # stale output buffers: every element must be written
    p = ck.params()
    vp = lambda t: C.c_void_p(t.data_ptr())
    rc = vs.lib().vs_select_static(C.byref(p), vp(vsc), vp(ssc), vp(sets[0]), vp(sets[1]), vp(sets[2]), vp(sets[3]),
                                   C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == vs.VS_OK, vs.status_string(rc)
    return sets


def _scores(g, hq, n_k, ties):
    dev = torch.device("cuda:0")
    if ties:   # a few distinct values: thousands of ties at every threshold
        mk = lambda: (torch.randint(0, 23, (hq, n_k), generator=g, device=dev).float() / 32.0).contiguous()
    else:
        mk = lambda: torch.rand((hq, n_k), generator=g, device=dev).contiguous()
    return mk(), mk()


def test_static_select_equals_select_on_two_calls_in_a_row():
    g = torch.Generator(device="cuda:0").manual_seed(5)
    # first call: 28 heads x 300,000 scores (many slices per row); second call: fewer heads, a short
    # ragged row, smaller budgets -- rows and slice counters of the first call stay behind in the array
    cases = [(28, 300_000, 1000, 6096, True), (5, 20_011, 40, 300, False), (28, 300_000, 1000, 6096, False)]
    for hq, n_k, bv, bs, ties in cases:
        ck = vs.Chunk(hq, 1, 128, 64, n_k - 64, 0.1, vertical_budget=bv, slash_budget=bs)
        vsc, ssc = _scores(g, hq, n_k, ties)
        want = vs.select(ck, vsc, ssc)
        got = _call_static(ck, vsc, ssc)
        torch.cuda.synchronize()
        for a, b, nm in zip(got, want, ("v_idx", "v_cnt", "s_idx", "s_cnt")):
            assert torch.equal(a, b), f"{nm} differs (Hq {hq}, n_k {n_k})"


def test_static_select_rejects_more_heads_than_it_holds():
    ck = vs.Chunk(129, 129, 64, 64, 0, 0.1, vertical_budget=4, slash_budget=70)
    vsc = torch.zeros((129, 64), device="cuda"); ssc = torch.zeros_like(vsc)
    with pytest.raises(vs.VsError) as e:
        vs.select_static(ck, vsc, ssc, vs.alloc_index_sets(ck, vsc.device))
    assert e.value.status == vs.VS_ERR_TOO_LARGE
