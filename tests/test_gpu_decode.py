"""Short chunks against a long cache (a decode step, a short last chunk; the paper's chunked
prefill is meant to interleave with decoding): the key walk of the few (query tile, head)
units is cut into ranges and a second kernel folds the partial results.  Parity against the
fp64 oracle through the C ABI, dense, sparse and with Dual Chunk Attention."""
import numpy as np
import pytest
import torch

import oracle
import paper_2501_15383_amd as vs
from gpu_util import assert_attn_close, chunk_of, dev
from helpers import rand_bf16
from test_gpu_attention import _rand_sets, _t

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("split", [0, 2, 5, 16])
@pytest.mark.parametrize("hq,hkv,d,c,s", [
    (4, 1, 128, 1, 20480),      # one query
    (7, 1, 128, 17, 12288),     # a few queries, GQA 7
    (2, 2, 64, 64, 8192),       # one query block
    (4, 2, 128, 128, 16384),    # one query tile
    (2, 1, 128, 200, 6400),     # two tiles, ragged
])
def test_dense_short_chunk_matches_oracle(split, hq, hkv, d, c, s):
    rng = np.random.default_rng(1100 + c)
    q = rand_bf16(rng, (c, hq, d)); k = rand_bf16(rng, (s + c, hkv, d)); v = rand_bf16(rng, (s + c, hkv, d))
    pb = oracle.Problem(hq, hkv, d, c, s, 1.0 / np.sqrt(d))
    ref_out, ref_lse = oracle.dense_attention(pb, q, k, v)
    vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, split)
    try:
        out, lse = vs.dense_causal_prefill(chunk_of(pb), dev(q), dev(k), dev(v), want_lse=True)
        torch.cuda.synchronize()
    finally:
        vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, 0)
    assert_attn_close(out, lse, ref_out, ref_lse, f"dense short chunk C={c} s={s} split={split}")


@pytest.mark.parametrize("split", [0, 3, 16])
@pytest.mark.parametrize("hq,hkv,d,c,s,nv,ns,band,dca", [
    (4, 1, 128, 1, 20480, 200, 40, 64, None),
    (7, 1, 128, 64, 12288, 300, 60, 64, None),
    (2, 1, 64, 128, 8192, 100, 4, 0, None),            # few diagonals: ranges without work, empty rows
    (4, 2, 128, 48, 16384, 150, 30, 64, (4096, 1024)), # Dual Chunk Attention
    (2, 1, 128, 130, 9600, 600, 50, 64, (3200, 640)),  # ... the chunk boundary inside the walk of a range
])
def test_sparse_short_chunk_matches_oracle(split, hq, hkv, d, c, s, nv, ns, band, dca):
    rng = np.random.default_rng(1200 + c)
    n_k = s + c
    qs = [rand_bf16(rng, (c, hq, d)) for _ in range(3)]
    k = rand_bf16(rng, (n_k, hkv, d)); v = rand_bf16(rng, (n_k, hkv, d))
    pb = oracle.Problem(hq, hkv, d, c, s, 1.0 / np.sqrt(d), vertical_budget=nv + 8, slash_budget=ns + band + 8,
                        keep_first_cols=1 if band else 0, keep_local_band=band)
    sets = _rand_sets(rng, pb, nv, ns, force_cols=[0] if band else [], force_offs=range(band))
    od = None if dca is None else oracle.Dca(dca[0], dca[1], qs[1], qs[2])
    gd = None if dca is None else (dev(qs[1]), dev(qs[2]), dca[0], dca[1])
    ref_out, ref_lse = oracle.sparse_attention(pb, qs[0], k, v, *sets, dca=od)
    vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, split)
    try:
        out, lse = vs.sparse_attn_prefill(chunk_of(pb), dev(qs[0]), dev(k), dev(v), *[_t(x) for x in sets],
                                          want_lse=True, dca=gd)
        torch.cuda.synchronize()
    finally:
        vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, 0)
    assert_attn_close(out, lse, ref_out, ref_lse, f"sparse short chunk C={c} s={s} split={split}")


def test_key_split_is_run_to_run_identical_and_close_to_the_unsplit_kernel():
    rng = np.random.default_rng(1300)
    hq, hkv, d, c, s = 4, 1, 128, 64, 32768
    q = dev(rand_bf16(rng, (c, hq, d))); k = dev(rand_bf16(rng, (s + c, hkv, d))); v = dev(rand_bf16(rng, (s + c, hkv, d)))
    ck = vs.Chunk(hq, hkv, d, c, s, 1.0 / np.sqrt(d))
    a, la = vs.dense_causal_prefill(ck, q, k, v, want_lse=True)
    b, lb = vs.dense_causal_prefill(ck, q, k, v, want_lse=True)
    vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, 1)
    try:
        p, lp = vs.dense_causal_prefill(ck, q, k, v, want_lse=True)
        torch.cuda.synchronize()
    finally:
        vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, 0)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16)) and torch.equal(la, lb)
    assert (a.float() - p.float()).abs().max().item() <= 2e-2 and (la - lp).abs().max().item() < 1e-3


@pytest.mark.parametrize("hq,hkv,d,c,s,dca", [
    (4, 1, 128, 1, 20000, None),        # a decode step at an arbitrary position
    (4, 2, 64, 5, 777, None),
    (2, 1, 128, 100, 1000, None),       # a chunk that starts and ends inside 64-key blocks
    (7, 1, 128, 300, 8191, None),       # ... over several query tiles
    (3, 1, 128, 64, 63, None),
    (4, 2, 128, 130, 5000, (1024, 256)),  # with Dual Chunk Attention
])
def test_chunks_that_start_anywhere_match_the_oracle(hq, hkv, d, c, s, dca):
    """q_start need not be a multiple of 64: the launch is padded back to the block boundary."""
    rng = np.random.default_rng(1400 + c + s)
    n_k = s + c
    qs = [rand_bf16(rng, (c, hq, d)) for _ in range(3)]
    k = rand_bf16(rng, (n_k, hkv, d)); v = rand_bf16(rng, (n_k, hkv, d))
    pb = oracle.Problem(hq, hkv, d, c, s, 1.0 / np.sqrt(d), vertical_budget=60, slash_budget=100)
    od = None if dca is None else oracle.Dca(dca[0], dca[1], qs[1], qs[2])
    gd = None if dca is None else (dev(qs[1]), dev(qs[2]), dca[0], dca[1])
    ck = chunk_of(pb)
    # dense
    ref_out, ref_lse = oracle.dense_attention(pb, qs[0], k, v, dca=od)
    out, lse = vs.dense_causal_prefill(ck, dev(qs[0]), dev(k), dev(v), want_lse=True, dca=gd)
    torch.cuda.synchronize()
    assert_attn_close(out, lse, ref_out, ref_lse, f"dense C={c} s={s}")
    # sparse on given sets
    sets = _rand_sets(rng, pb, 50, 30, force_cols=[0], force_offs=range(64))
    ref_out, ref_lse = oracle.sparse_attention(pb, qs[0], k, v, *sets, dca=od)
    out, lse = vs.sparse_attn_prefill(ck, dev(qs[0]), dev(k), dev(v), *[_t(x) for x in sets], want_lse=True, dca=gd)
    torch.cuda.synchronize()
    assert_attn_close(out, lse, ref_out, ref_lse, f"sparse C={c} s={s}")
    # estimate, and the whole chunk against its own stages
    from gpu_util import f64
    rvs, rss, _ = oracle.estimate(pb, qs[0], k, dca=od)
    vsc, ssc, _ = vs.estimate(ck, dev(qs[0]), dev(k), dca=gd)
    np.testing.assert_allclose(f64(vsc), rvs, rtol=2e-4, atol=1e-7)
    np.testing.assert_allclose(f64(ssc), rss, rtol=2e-4, atol=1e-7)
    sel = vs.select(ck, vsc, ssc)
    a, _ = vs.sparse_attn_prefill(ck, dev(qs[0]), dev(k), dev(v), *sel, dca=gd)
    b, _ = vs.prefill_chunk(ck, dev(qs[0]), dev(k), dev(v), dca=gd)
    tiles = vs.count_tiles(ck, *sel)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    assert (tiles[:, 0] > 0).all()


@pytest.mark.parametrize("split", [0, 1, 7])
@pytest.mark.parametrize("hq,hkv,d,s,dca", [
    (28, 4, 128, 20000, None),       # the 7B shape: 7 query heads per KV head share a tile
    (40, 8, 128, 4095, None),        # the 14B shape, last key of a block
    (8, 2, 64, 4096, None),          # first key of a block
    (6, 1, 128, 130, None),
    (28, 4, 128, 9000, (2048, 512)), # with Dual Chunk Attention
    (4, 4, 128, 5000, None),         # no grouping: the ordinary path
])
def test_single_token_dense_decode_matches_oracle(split, hq, hkv, d, s, dca):
    """Dense attention of one token: the query heads of a KV group are packed into one tile."""
    rng = np.random.default_rng(1500 + s)
    qs = [rand_bf16(rng, (1, hq, d)) for _ in range(3)]
    k = rand_bf16(rng, (s + 1, hkv, d)); v = rand_bf16(rng, (s + 1, hkv, d))
    pb = oracle.Problem(hq, hkv, d, 1, s, 1.0 / np.sqrt(d))
    od = None if dca is None else oracle.Dca(dca[0], dca[1], qs[1], qs[2])
    gd = None if dca is None else (dev(qs[1]), dev(qs[2]), dca[0], dca[1])
    ref_out, ref_lse = oracle.dense_attention(pb, qs[0], k, v, dca=od)
    vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, split)
    try:
        out, lse = vs.dense_causal_prefill(chunk_of(pb), dev(qs[0]), dev(k), dev(v), want_lse=True, dca=gd)
        torch.cuda.synchronize()
    finally:
        vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, 0)
    assert_attn_close(out, lse, ref_out, ref_lse, f"decode {hq}/{hkv} s={s} split={split}")
