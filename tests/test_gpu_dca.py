"""GPU parity of the Dual Chunk Attention variants (section 5.1; "Integrating with DCA",
section 5.2) against the fp64 oracle, element by element, through the C ABI.  The three
rotations of the queries are independent random tensors here, which makes every wrong choice
of pattern visible."""
import numpy as np
import pytest
import torch

import oracle
import paper_2501_15383_amd as vs
from gpu_util import assert_attn_close, chunk_of, dev
from helpers import rand_bf16
from test_gpu_attention import _rand_sets, _t

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, params=[0, 1], ids=["key_split_auto", "key_split_off"])
def _key_split(request):
    """Every case runs with the key split of short chunks chosen automatically (most of these
    small shapes then take it) and switched off (the kernel the full-size launches use)."""
    vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, request.param)
    yield
    vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, 0)


def _inputs(rng, hq, hkv, d, c, s):
    qs = [rand_bf16(rng, (c, hq, d)) for _ in range(3)]
    k = rand_bf16(rng, (s + c, hkv, d)); v = rand_bf16(rng, (s + c, hkv, d))
    return qs, k, v


@pytest.mark.parametrize("hq,hkv,d,c,s,chunk,window", [
    (4, 1, 64, 256, 512, 256, 128),     # chunk boundary at the start of the query chunk
    (4, 2, 128, 320, 448, 192, 64),     # boundaries inside the query chunk and inside query tiles
    (2, 1, 128, 200, 1280, 512, 256),   # ragged chunk, two chunks back = inter
    (7, 1, 128, 130, 640, 64, 64),      # smallest chunk: every block its own chunk
    (2, 2, 64, 256, 256, 128, 0),       # no local window
    (2, 1, 128, 192, 320, 128, 384),    # window longer than the chunk
    (3, 1, 64, 128, 384, 4096, 64),     # one chunk holds everything: intra only
])
def test_dense_dca_matches_oracle(hq, hkv, d, c, s, chunk, window):
    rng = np.random.default_rng(700 + c + chunk)
    qs, k, v = _inputs(rng, hq, hkv, d, c, s)
    pb = oracle.Problem(hq, hkv, d, c, s, 1.0 / np.sqrt(d))
    ref_out, ref_lse = oracle.dense_attention(pb, qs[0], k, v, dca=oracle.Dca(chunk, window, qs[1], qs[2]))
    out, lse = vs.dense_causal_prefill(chunk_of(pb), dev(qs[0]), dev(k), dev(v), want_lse=True,
                                       dca=(dev(qs[1]), dev(qs[2]), chunk, window))
    torch.cuda.synchronize()
    assert_attn_close(out, lse, ref_out, ref_lse, f"dense dca C={c} s={s} chunk={chunk} window={window}")


@pytest.mark.parametrize("hq,hkv,d,c,s,nv,ns,band,chunk,window", [
    (4, 1, 64, 512, 1024, 60, 12, 64, 512, 128),
    (4, 2, 128, 320, 960, 150, 20, 64, 256, 64),    # vertical columns of all three patterns in one tile
    (2, 1, 128, 256, 512, 70, 6, 0, 128, 128),
    (7, 1, 128, 200, 1280, 130, 30, 64, 640, 192),
])
def test_sparse_dca_matches_oracle_on_given_sets(hq, hkv, d, c, s, nv, ns, band, chunk, window):
    rng = np.random.default_rng(800 + c)
    qs, k, v = _inputs(rng, hq, hkv, d, c, s)
    pb = oracle.Problem(hq, hkv, d, c, s, 1.0 / np.sqrt(d), vertical_budget=nv + 8, slash_budget=ns + band + 8,
                        keep_first_cols=1 if band else 0, keep_local_band=band)
    sets = _rand_sets(rng, pb, nv, ns, force_cols=[0] if band else [], force_offs=range(band))
    ref_out, ref_lse = oracle.sparse_attention(pb, qs[0], k, v, *sets, dca=oracle.Dca(chunk, window, qs[1], qs[2]))
    out, lse = vs.sparse_attn_prefill(chunk_of(pb), dev(qs[0]), dev(k), dev(v), *[_t(x) for x in sets],
                                      want_lse=True, dca=(dev(qs[1]), dev(qs[2]), chunk, window))
    torch.cuda.synchronize()
    assert_attn_close(out, lse, ref_out, ref_lse, f"sparse dca C={c} s={s} chunk={chunk} window={window}")


def test_dca_with_equal_rotations_is_the_plain_kernel():
    rng = np.random.default_rng(900)
    hq, hkv, d, c, s = 4, 1, 128, 256, 768
    qs, k, v = _inputs(rng, hq, hkv, d, c, s)
    ck = chunk_of(oracle.Problem(hq, hkv, d, c, s, 1.0 / np.sqrt(d)))
    q = dev(qs[0])
    plain, lse_p = vs.dense_causal_prefill(ck, q, dev(k), dev(v), want_lse=True)
    same, lse_s = vs.dense_causal_prefill(ck, q, dev(k), dev(v), want_lse=True, dca=(q.clone(), q.clone(), 256, 128))
    torch.cuda.synchronize()
    assert (plain.float() - same.float()).abs().max().item() <= 2e-2
    assert (lse_p - lse_s).abs().max().item() < 1e-3


def test_dca_argument_checks():
    ck = vs.Chunk(2, 1, 64, 64, 0, 0.125)
    q = torch.zeros((64, 2, 64), dtype=torch.bfloat16, device="cuda"); kv = torch.zeros((64, 1, 64), dtype=torch.bfloat16, device="cuda")
    for chunk, window, status in ((100, 64, vs.VS_ERR_UNSUPPORTED), (128, 10, vs.VS_ERR_UNSUPPORTED),
                                  (0, 64, vs.VS_ERR_INVALID_ARG), (128, -64, vs.VS_ERR_INVALID_ARG)):
        with pytest.raises(vs.VsError) as e:
            vs.dense_causal_prefill(ck, q, kv, kv, dca=(q, q, chunk, window))
        assert e.value.status == status


@pytest.mark.parametrize("hq,hkv,d,c,s,w,chunk,window", [
    (4, 1, 64, 1024, 3072, 64, 1024, 256),    # window rows at the end of a chunk; window boundary inside a key tile row
    (7, 1, 128, 300, 2048, 64, 512, 128),     # ragged n_k: the window rows straddle 64-blocks
    (4, 2, 128, 96, 1984, 64, 2048, 64),      # ... and a chunk boundary (rows 2048.. enter the next chunk)
    (5, 1, 128, 40, 0, 64, 64, 64),           # chunk shorter than the window, first chunk
    (8, 2, 128, 128, 1152, 16, 128, 0),       # short window of rows, no local window
    (2, 1, 64, 256, 1792, 64, 64, 192),       # smallest chunk
    (3, 3, 64, 128, 384, 64, 4096, 64),       # intra only
])
def test_estimate_dca_matches_oracle(hq, hkv, d, c, s, w, chunk, window):
    from gpu_util import f64
    rng = np.random.default_rng(1000 + c + chunk)
    n_k = s + c
    qs = [rand_bf16(rng, (c, hq, d)) for _ in range(3)]
    k = rand_bf16(rng, (n_k, hkv, d))
    pb = oracle.Problem(hq, hkv, d, c, s, 1.0 / np.sqrt(d), last_q=w)
    rvs, rss, rlse = oracle.estimate(pb, qs[0], k, dca=oracle.Dca(chunk, window, qs[1], qs[2]))
    vsc, ssc, lse = vs.estimate(chunk_of(pb), dev(qs[0]), dev(k), want_lse=True,
                                dca=(dev(qs[1]), dev(qs[2]), chunk, window))
    torch.cuda.synchronize()
    np.testing.assert_allclose(f64(lse), rlse, atol=2e-4, rtol=0)
    np.testing.assert_allclose(f64(vsc), rvs, rtol=2e-4, atol=1e-7)
    np.testing.assert_allclose(f64(ssc), rss, rtol=2e-4, atol=1e-7)


@pytest.mark.parametrize("hq,hkv,d,c,s,chunk,window,sel_chunk,sel_window", [
    (4, 1, 64, 512, 1536, 512, 128, 512, 1024),    # the selection covers the whole chunk before the query's
    (4, 2, 128, 384, 1408, 256, 64, 128, 0),       # different chunk lengths for the selection and the attention
    (7, 1, 128, 200, 1848, 640, 192, 640, 1280),   # ragged chunk, GQA 7
])
def test_prefill_chunk_dca_selects_with_its_own_rotations(hq, hkv, d, c, s, chunk, window, sel_chunk, sel_window):
    """Section 5.2, "Integrating with DCA": critical tokens are selected with other relative
    positions than the attention uses.  The selection's rotations and the attention's are four
    independent random tensors here (plus the shared intra-chunk one), so a call that estimated
    with the attention's rotations, or attended with the selection's, cannot pass."""
    from gpu_util import check_index_sets, f64
    rng = np.random.default_rng(1100 + c)
    n_k = s + c
    q = rand_bf16(rng, (c, hq, d))
    att = [rand_bf16(rng, (c, hq, d)) for _ in range(2)]
    sel = [rand_bf16(rng, (c, hq, d)) for _ in range(2)]
    k = rand_bf16(rng, (n_k, hkv, d)); v = rand_bf16(rng, (n_k, hkv, d))
    bv, bs = 96, 200
    pb = oracle.Problem(hq, hkv, d, c, s, 1.0 / np.sqrt(d), vertical_budget=bv, slash_budget=bs)
    ck = chunk_of(pb)
    qd, kd, vd = dev(q), dev(k), dev(v)
    g_att = (dev(att[0]), dev(att[1]), chunk, window)
    g_sel = (dev(sel[0]), dev(sel[1]), sel_chunk, sel_window)
    out, lse = vs.prefill_chunk(ck, qd, kd, vd, want_lse=True, dca=g_att, dca_select=g_sel)
    # the same three stages one by one: estimate with the selection's rotations, attend with DCA's
    vsc, ssc, _ = vs.estimate(ck, qd, kd, dca=g_sel)
    sets = vs.select(ck, vsc, ssc)
    out2, lse2 = vs.sparse_attn_prefill(ck, qd, kd, vd, *sets, want_lse=True, dca=g_att)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16)) and torch.equal(lse, lse2)
    # oracle: estimate with the selection's rotations ...
    o_sel = oracle.Dca(sel_chunk, sel_window, sel[0], sel[1])
    o_att = oracle.Dca(chunk, window, att[0], att[1])
    rvs, rss, _ = oracle.estimate(pb, q, k, dca=o_sel)
    np.testing.assert_allclose(f64(vsc), rvs, rtol=2e-4, atol=1e-7)
    np.testing.assert_allclose(f64(ssc), rss, rtol=2e-4, atol=1e-7)
    # ... which is not what the attention's rotations would have scored
    wvs, _, _ = oracle.estimate(pb, q, k, dca=o_att)
    assert np.abs(wvs - rvs).max() > 1e-3
    sets_h = [x.cpu().numpy() for x in sets]
    for h in range(hq):
        check_index_sets(rvs[h], sets_h[0][h], sets_h[1][h], bv, 1, f"head {h} vertical")
        check_index_sets(rss[h], sets_h[2][h], sets_h[3][h], bs, 64, f"head {h} slash")
    # ... select, then attention with DCA's own rotations on the GPU's index sets
    ref_out, ref_lse = oracle.sparse_attention(pb, q, k, v, *sets_h, dca=o_att)
    assert_attn_close(out, lse, ref_out, ref_lse, f"chunk call with selection rotations C={c} s={s}")
    # end to end from the oracle's own selection, wherever the two selections agree exactly
    o_sets = oracle.select(pb, rvs, rss)
    if all(np.array_equal(a, b) for a, b in zip(o_sets, sets_h)):
        e2e_out, e2e_lse = oracle.sparse_attention(pb, q, k, v, *o_sets, dca=o_att)
        assert_attn_close(out, lse, e2e_out, e2e_lse, "end to end")
