"""GPU parity of the attention kernels (dense fallback and block-sparse) against the fp64
oracle, element by element, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2501_15383_amd as vs
from gpu_util import assert_attn_close, chunk_of, dev
from helpers import rand_bf16

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, params=[0, 1], ids=["key_split_auto", "key_split_off"])
def _key_split(request):
    """Every case runs with the key split of short chunks chosen automatically (most of these
    small shapes then take it) and switched off (the kernel the full-size launches use)."""
    vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, request.param)
    yield
    vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, 0)


def _rand_sets(rng, pb, nv, ns, force_cols=(), force_offs=()):
    """Random ascending index sets in the layout vs_select produces."""
    hq, n_k = pb.n_q_heads, pb.n_k
    v_idx = np.full((hq, pb.vertical_budget), -1, np.int32); s_idx = np.full((hq, pb.slash_budget), -1, np.int32)
    v_cnt = np.zeros(hq, np.int32); s_cnt = np.zeros(hq, np.int32)
    for h in range(hq):
        v = sorted(set(rng.choice(n_k, min(nv, n_k), replace=False).tolist()) | set(force_cols))[: pb.vertical_budget]
        s = sorted(set(rng.choice(n_k, min(ns, n_k), replace=False).tolist()) | set(force_offs))[: pb.slash_budget]
        v_idx[h, :len(v)] = v; v_cnt[h] = len(v); s_idx[h, :len(s)] = s; s_cnt[h] = len(s)
    return v_idx, v_cnt, s_idx, s_cnt


def _t(x):
    return torch.from_numpy(x).cuda()


@pytest.mark.parametrize("hq,hkv,d,c,s", [
    (4, 1, 64, 64, 0),          # one tile
    (4, 1, 64, 1024, 3072),     # last chunk of the small configuration
    (4, 2, 128, 200, 128),      # ragged chunk, D = 128
    (7, 1, 128, 384, 640),      # GQA 7 as in the 7B shape
    (2, 2, 128, 1, 0),          # a single query
    (5, 1, 128, 130, 64),       # GQA 5 (14B shape), two rows past a tile edge
])
def test_dense_matches_oracle(hq, hkv, d, c, s):
    rng = np.random.default_rng(100 + c)
    n_k = s + c
    q = rand_bf16(rng, (c, hq, d)); k = rand_bf16(rng, (n_k, hkv, d)); v = rand_bf16(rng, (n_k, hkv, d))
    pb = oracle.Problem(hq, hkv, d, c, s, 1.0 / np.sqrt(d))
    ref_out, ref_lse = oracle.dense_attention(pb, q, k, v)
    out, lse = vs.dense_causal_prefill(chunk_of(pb), dev(q), dev(k), dev(v), want_lse=True)
    torch.cuda.synchronize()
    assert_attn_close(out, lse, ref_out, ref_lse, f"dense {hq}/{hkv}/{d} C={c} s={s}")


@pytest.mark.parametrize("hq,hkv,d,c,s,nv,ns,band", [
    (4, 1, 64, 512, 1024, 40, 12, 64),     # sparse diagonals + verticals, local band kept
    (4, 2, 128, 320, 960, 100, 20, 64),
    (2, 1, 128, 256, 512, 70, 6, 0),       # no forced band: verticals inside the diagonal block, empty rows
    (7, 1, 128, 200, 1280, 130, 30, 64),   # ragged chunk
    (4, 1, 64, 128, 0, 10, 3, 0),          # first chunk
])
def test_sparse_matches_oracle_on_given_sets(hq, hkv, d, c, s, nv, ns, band):
    rng = np.random.default_rng(200 + c)
    n_k = s + c
    q = rand_bf16(rng, (c, hq, d)); k = rand_bf16(rng, (n_k, hkv, d)); v = rand_bf16(rng, (n_k, hkv, d))
    pb = oracle.Problem(hq, hkv, d, c, s, 1.0 / np.sqrt(d), vertical_budget=nv + 8, slash_budget=ns + band + 8,
                        keep_first_cols=1 if band else 0, keep_local_band=band)
    sets = _rand_sets(rng, pb, nv, ns, force_cols=[0] if band else [], force_offs=range(band))
    ref_out, ref_lse = oracle.sparse_attention(pb, q, k, v, *sets)
    out, lse = vs.sparse_attn_prefill(chunk_of(pb), dev(q), dev(k), dev(v), *[_t(x) for x in sets], want_lse=True)
    torch.cuda.synchronize()
    assert_attn_close(out, lse, ref_out, ref_lse, f"sparse {hq}/{hkv}/{d} C={c} s={s}")


def test_sparse_with_everything_selected_equals_dense_kernel():
    rng = np.random.default_rng(300)
    hq, hkv, d, c, s = 4, 2, 128, 256, 256
    n_k = s + c
    q = rand_bf16(rng, (c, hq, d)); k = rand_bf16(rng, (n_k, hkv, d)); v = rand_bf16(rng, (n_k, hkv, d))
    pb = oracle.Problem(hq, hkv, d, c, s, 1.0 / np.sqrt(d), vertical_budget=n_k, slash_budget=n_k)
    allv = np.tile(np.arange(n_k, dtype=np.int32), (hq, 1)); cnt = np.full(hq, n_k, np.int32)
    ck = chunk_of(pb)
    o_s, l_s = vs.sparse_attn_prefill(ck, dev(q), dev(k), dev(v), _t(allv), _t(cnt), _t(allv), _t(cnt), want_lse=True)
    o_d, l_d = vs.dense_causal_prefill(ck, dev(q), dev(k), dev(v), want_lse=True)
    torch.cuda.synchronize()
    # same tiles in the same order: bit-identical
    assert torch.equal(o_s.view(torch.int16), o_d.view(torch.int16)) and torch.equal(l_s, l_d)


def test_strided_inputs_and_yarn_scale():
    # K and V interleaved in one cache tensor, Q a slice of a fused QKV buffer, softmax scale with YaRN temperature
    rng = np.random.default_rng(301)
    hq, hkv, d, c, s = 4, 2, 128, 192, 128
    n_k = s + c
    q = rand_bf16(rng, (c, hq, d)); k = rand_bf16(rng, (n_k, hkv, d)); v = rand_bf16(rng, (n_k, hkv, d))
    scale = vs.yarn_softmax_scale(4.0, d)
    assert abs(scale - oracle.yarn_softmax_scale(4.0, d)) < 1e-7
    pb = oracle.Problem(hq, hkv, d, c, s, scale)
    ref_out, ref_lse = oracle.dense_attention(pb, q, k, v)
    kv = torch.empty((n_k, 2, hkv, d), dtype=torch.bfloat16, device="cuda")
    kv[:, 0] = dev(k); kv[:, 1] = dev(v)
    qkv = torch.zeros((c, hq + 3, d), dtype=torch.bfloat16, device="cuda"); qkv[:, 1:hq + 1] = dev(q)
    out, lse = vs.dense_causal_prefill(chunk_of(pb), qkv[:, 1:hq + 1], kv[:, 0], kv[:, 1], want_lse=True)
    torch.cuda.synchronize()
    assert_attn_close(out, lse, ref_out, ref_lse, "strided")


def test_count_tiles_matches_mask_blocks():
    rng = np.random.default_rng(302)
    hq, d, c, s = 2, 64, 256, 512
    pb = oracle.Problem(hq, 1, d, c, s, 0.125, vertical_budget=48, slash_budget=80)
    sets = _rand_sets(rng, pb, 40, 10, force_cols=[0], force_offs=range(64))
    tiles = vs.count_tiles(chunk_of(pb), *[_t(x) for x in sets]).cpu().numpy()
    for h in range(hq):
        sl = sets[2][h, :sets[3][h]]
        A = set((sl // 64).tolist()) | set((sl[sl % 64 != 0] // 64 + 1).tolist())
        expect = sum(1 for qb in range(c // 64) for a in A if a <= s // 64 + qb)
        assert tiles[h, 0] == expect
        assert 0 <= tiles[h, 1] <= (c // 64) * ((sets[1][h] + 63) // 64)


@pytest.mark.parametrize("seg_blocks", [1, 3, 8])
@pytest.mark.parametrize("hq,hkv,d,c,s,nv,ns,band", [
    (4, 1, 64, 512, 1024, 40, 12, 64),
    (7, 1, 128, 200, 1280, 130, 30, 64),   # ragged chunk
    (2, 1, 128, 256, 512, 70, 6, 0),       # no forced band: segments with no work, empty rows
])
def test_sparse_with_other_sync_segments_matches_oracle(seg_blocks, hq, hkv, d, c, s, nv, ns, band):
    """Pace keeping of the persistent launch with sync segments of seg_blocks key blocks: the
    waiting only shapes the timing, the contract is the same."""
    rng = np.random.default_rng(200 + c)
    n_k = s + c
    q = rand_bf16(rng, (c, hq, d)); k = rand_bf16(rng, (n_k, hkv, d)); v = rand_bf16(rng, (n_k, hkv, d))
    pb = oracle.Problem(hq, hkv, d, c, s, 1.0 / np.sqrt(d), vertical_budget=nv + 8, slash_budget=ns + band + 8,
                        keep_first_cols=1 if band else 0, keep_local_band=band)
    sets = _rand_sets(rng, pb, nv, ns, force_cols=[0] if band else [], force_offs=range(band))
    ref_out, ref_lse = oracle.sparse_attention(pb, q, k, v, *sets)
    ck = chunk_of(pb)
    vs.set_option(vs.VS_OPT_ATTN_SEGMENT_BLOCKS, seg_blocks)
    try:
        out, lse = vs.sparse_attn_prefill(ck, dev(q), dev(k), dev(v), *[_t(x) for x in sets], want_lse=True)
        torch.cuda.synchronize()
    finally:
        vs.set_option(vs.VS_OPT_ATTN_SEGMENT_BLOCKS, 0)
    assert_attn_close(out, lse, ref_out, ref_lse, f"sync {seg_blocks}: sparse {hq}/{hkv}/{d} C={c} s={s}")


def test_sparse_cost_model_follows_counted_tiles():
    """vs_chunk_cost(VS_COST_SPARSE) against the tiles the block list really holds when the slash offsets
    scatter uniformly (the model's premise).  One head's count scatters by about 2 % around the expectation,
    so the mean over 16 heads is compared (within 2 %); gathered columns never exceed the model's."""
    rng = np.random.default_rng(303)
    hq, d, c, s, nv, ns = 16, 128, 2048, 63488, 500, 300
    pb = oracle.Problem(hq, 1, d, c, s, 0.1, vertical_budget=nv, slash_budget=ns, keep_first_cols=0, keep_local_band=0)
    sets = _rand_sets(rng, pb, nv, ns)
    tiles = vs.count_tiles(chunk_of(pb), *[_t(x) for x in sets]).cpu().numpy()
    slash_model = vs.chunk_cost(s, c, vs.VS_COST_SPARSE, 1, ns) - (c // 64)   # one tile of columns per query block
    column_model = vs.chunk_cost(s, c, vs.VS_COST_SPARSE, nv, ns) - slash_model
    assert abs(tiles[:, 0].mean() - slash_model) <= 0.02 * slash_model, (tiles[:, 0].mean(), slash_model)
    assert (tiles[:, 1] <= column_model).all()


@pytest.mark.parametrize("in_turn", [0, 1])
def test_rounds_dealt_by_weight_or_in_turn_give_the_same_result(in_turn):
    """Several rounds per group, heads with block lists of very different lengths: the order in which
    the groups take the rounds only shapes the timing."""
    rng = np.random.default_rng(310)
    hq, hkv, d, c, s = 6, 1, 64, 2048, 4096      # 16 query tiles x 6 heads over 8 groups
    n_k = s + c
    q = rand_bf16(rng, (c, hq, d)); k = rand_bf16(rng, (n_k, hkv, d)); v = rand_bf16(rng, (n_k, hkv, d))
    pb = oracle.Problem(hq, hkv, d, c, s, 1.0 / np.sqrt(d), vertical_budget=40, slash_budget=100)
    sets = list(_rand_sets(rng, pb, 30, 30, force_cols=[0], force_offs=range(64)))
    sets[3][1] = 70; sets[3][4] = 65                      # two heads with short lists
    rows = np.sort(rng.choice(c, 48, replace=False))
    ref_out, ref_lse = oracle.sparse_attention(pb, q, k, v, *sets, rows=rows)
    vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, 1)
    vs.set_option(vs.VS_OPT_ATTN_ROUNDS_IN_TURN, in_turn)
    try:
        out, lse = vs.sparse_attn_prefill(chunk_of(pb), dev(q), dev(k), dev(v), *[_t(x) for x in sets], want_lse=True)
        torch.cuda.synchronize()
    finally:
        vs.set_option(vs.VS_OPT_ATTN_ROUNDS_IN_TURN, 0)
    rt = torch.from_numpy(rows).cuda()
    assert_attn_close(out[rt], lse[:, rt], ref_out, ref_lse, f"rounds in turn = {in_turn}")


@pytest.mark.parametrize("d", [64, 128])
def test_scores_that_outrun_the_first_tiles_by_far(d):
    """The walk starts at a row's own keys and goes backwards; its softmax reference is fixed by the
    first tile.  Here earlier keys score 60 to 180 nats above everything seen before them, in three
    steps, so the reference has to be raised (and the accumulators rescaled) several times per row;
    a fourth group scores far below and must vanish."""
    rng = np.random.default_rng(320 + d)
    hq, hkv, c, s = 2, 1, 192, 2048
    n_k = s + c
    scale = 1.0 / np.sqrt(d)
    qf = np.full((c, hq, d), 0.5, np.float32) + 0.01 * rng.standard_normal((c, hq, d)).astype(np.float32)
    kf = 0.05 * rng.standard_normal((n_k, hkv, d)).astype(np.float32)
    step = 60.0 / (scale * d * 0.5)                 # key value that adds 60 nats to the logit
    kf[1280:1344] += step; kf[640:700] += 2 * step; kf[3:40] += 3 * step; kf[1500:1530] -= 3 * step
    vf = rng.standard_normal((n_k, hkv, d)).astype(np.float32)
    to_u16 = lambda x: (torch.from_numpy(x).bfloat16().view(torch.int16).numpy().view(np.uint16))
    q, k, v = to_u16(qf), to_u16(kf), to_u16(vf)
    pb = oracle.Problem(hq, hkv, d, c, s, scale, vertical_budget=48, slash_budget=n_k)
    ref_out, ref_lse = oracle.dense_attention(pb, q, k, v)
    assert ref_lse.min() > 150                     # the big keys dominate every row
    out, lse = vs.dense_causal_prefill(chunk_of(pb), dev(q), dev(k), dev(v), want_lse=True)
    torch.cuda.synchronize()
    assert_attn_close(out, lse, ref_out, ref_lse, f"outrunning scores, dense, D={d}")
    # sparse: every diagonal computed except those of the second group, which comes in as vertical columns
    offs = np.array(sorted(set(range(n_k)) - set(range(s - 700, s + c - 640))), np.int32)
    s_idx = np.full((hq, n_k), -1, np.int32); s_idx[:, :len(offs)] = offs
    cols = np.array([0] + list(range(640, 680)), np.int32)
    v_idx = np.full((hq, 48), -1, np.int32); v_idx[:, :len(cols)] = cols
    sets = (v_idx, np.full(hq, len(cols), np.int32), s_idx, np.full(hq, len(offs), np.int32))
    ref_out, ref_lse = oracle.sparse_attention(pb, q, k, v, *sets)
    out, lse = vs.sparse_attn_prefill(chunk_of(pb), dev(q), dev(k), dev(v), *[_t(x) for x in sets], want_lse=True)
    torch.cuda.synchronize()
    assert_attn_close(out, lse, ref_out, ref_lse, f"outrunning scores, sparse, D={d}")
