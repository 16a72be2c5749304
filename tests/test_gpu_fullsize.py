"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times, on sampled outputs the oracle can compute one by one, plus properties that
hold at any size.  Inputs come from the seeded generator (synthetic stand-ins for the
post-RoPE Q/K/V of the paper's models)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2501_15383_amd as vs
import vsgen
from gpu_util import block_class_values, check_class_mass, check_index_sets, check_lse, check_rows, chunk_of, f64

pytestmark = pytest.mark.gpu


def _sample_rows(rng, c, n):
    """first / last rows, rows around 64-row block edges and tile (128-row) edges, random rows"""
    fixed = [0, 1, 63, 64, 127, 128, c // 2 - 1, c // 2, c - 129, c - 65, c - 64, c - 1]
    rows = sorted(set([r for r in fixed if 0 <= r < c] + rng.choice(c, n, replace=False).tolist()))
    return np.array(rows, np.int64)


def _check_rows(out, lse, ref_out, ref_lse, heads, rows, what):
    """Sampled rows: the element rule, the row-normalised rules and the tight lse rule."""
    check_rows(np.transpose(f64(out[rows][:, heads]), (1, 0, 2)), ref_out, what)
    check_lse(f64(lse[heads][:, rows]), ref_lse, what)


def _check_block_classes(run, oracle_rows, n_k, w, heads, rows, what):
    """Values that are 1 in dimension floor(j / 64) mod D: every output is the probability mass of
    one class of key blocks, a sum of non-negative terms of the size of the output itself, so a
    single dropped, doubled or misplaced 64-key tile shows (one tile is 1 / (tiles per class) of its
    element: 1.7 % at 7,600 tiles per row, against a bound of 0.6 %)."""
    Vc = block_class_values(n_k, w.n_kv_heads, w.head_dim)
    oc = run(Vc)
    torch.cuda.synchronize()
    ref_c, _ = oracle_rows(vsgen.as_u16(Vc))
    got = np.transpose(f64(oc[rows][:, heads]), (1, 0, 2))
    np.testing.assert_allclose(ref_c.sum(-1), 1.0, rtol=1e-9)
    check_class_mass(got, ref_c, what + ", block-class values")


def _run_sparse_chunk(name, chunk_index, heads, n_rows, seed):
    w = vsgen.WORKLOADS[name]
    ci = chunk_index % w.n_chunks
    s = ci * w.chunk
    C, n_k = w.chunk, s + w.chunk
    dev = torch.device("cuda:0")
    K, V = vsgen.make_kv(w, n_k, device=dev)
    dca = odca = sel = osel = None
    if w.dca_chunk > 0:
        # Dual Chunk Attention positions: three rotations of the queries for the attention, and the
        # selection's own (continuous relative positions, "Integrating with DCA")
        Q, q_succ, q_inter = vsgen.make_q_dca(w, s, s + C, device=dev)
        dca = (q_succ, q_inter, w.dca_chunk, w.dca_window)
        odca = oracle.Dca(w.dca_chunk, w.dca_window, vsgen.as_u16(q_succ), vsgen.as_u16(q_inter))
        sel = vsgen.make_q_dca_select(w, s, s + C, device=dev)
        osel = oracle.Dca(sel[2], sel[3], vsgen.as_u16(sel[0]), vsgen.as_u16(sel[1]))
    else:
        Q = vsgen.make_q(w, s, s + C, device=dev)
    pb = oracle.Problem(w.n_q_heads, w.n_kv_heads, w.head_dim, C, s, w.softmax_scale, last_q=w.last_q,
                        vertical_budget=w.vertical_budget, slash_budget=w.slash_budget,
                        keep_first_cols=w.keep_first_cols, keep_local_band=w.keep_local_band)
    ck = chunk_of(pb)
    vsc, ssc, lse_w = vs.estimate(ck, Q, K, want_lse=True, dca=sel)
    sets = vs.select(ck, vsc, ssc)
    out, lse = vs.sparse_attn_prefill(ck, Q, K, V, *sets, want_lse=True, dca=dca)
    out2, _ = vs.prefill_chunk(ck, Q, K, V, dca=dca, dca_select=sel)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16)), "vs_prefill_chunk differs from its stages"

    qh, kh, vh = vsgen.as_u16(Q), vsgen.as_u16(K), vsgen.as_u16(V)
    # ---- estimation and selection of the sampled heads against the oracle
    rvs, rss, rlse = oracle.estimate(pb, qh, kh, heads=heads, dca=osel)
    gv, gs = f64(vsc[heads]), f64(ssc[heads])
    np.testing.assert_allclose(f64(lse_w[heads]), rlse, atol=5e-4, rtol=0)
    np.testing.assert_allclose(gv.sum(1), min(w.last_q, C), rtol=2e-4)
    np.testing.assert_allclose(gs.sum(1), min(w.last_q, C), rtol=2e-4)
    np.testing.assert_allclose(gv, rvs, rtol=1e-3, atol=1e-8)
    np.testing.assert_allclose(gs, rss, rtol=1e-3, atol=1e-8)
    sets_h = [x.cpu().numpy() for x in sets]
    for i, h in enumerate(heads):
        check_index_sets(rvs[i], sets_h[0][h], sets_h[1][h], w.vertical_budget, w.keep_first_cols, f"{name} head {h} vertical")
        check_index_sets(rss[i], sets_h[2][h], sets_h[3][h], w.slash_budget, w.keep_local_band, f"{name} head {h} slash")
    # ---- attention of sampled rows: the oracle is fed the GPU's own index sets
    rows = _sample_rows(np.random.default_rng(seed), C, n_rows)
    ref_out, ref_lse = oracle.sparse_attention(pb, qh, kh, vh, *sets_h, heads=heads, rows=rows, dca=odca)
    _check_rows(out, lse, ref_out, ref_lse, heads, rows, f"{name} chunk {ci}")
    # ---- at any size: weights of every row sum to one (V == 1 gives out == 1)
    ones = torch.ones_like(V)
    o1, _ = vs.sparse_attn_prefill(ck, Q, K, ones, *sets, dca=dca)
    torch.cuda.synchronize()
    dev1 = (o1.float() - 1.0).abs().max().item()
    assert dev1 < 1e-2, f"{name}: rows of P do not sum to one ({dev1})"
    del ones, o1
    # ---- values that make every output a block-class mass
    _check_block_classes(lambda Vc: vs.sparse_attn_prefill(ck, Q, K, Vc, *sets, dca=dca)[0],
                         lambda vc: oracle.sparse_attention(pb, qh, kh, vc, *sets_h, heads=heads, rows=rows, dca=odca),
                         n_k, w, heads, rows, f"{name} chunk {ci}")
    # ---- recall against the dense kernel on a slice of rows lies in (0, 1]
    tiles = vs.count_tiles(ck, *sets).cpu().numpy()
    assert (tiles[:, 0] > 0).all()
    return dict(out=out, lse=lse, Q=Q, K=K, V=V, ck=ck, pb=pb)


def test_dense_7b_64k_sampled_rows():
    # configuration 1: 32768 queries at q_start 32768, every key attended
    w = vsgen.WORKLOADS["dense_7b_64k"]
    s, C = w.chunk, w.chunk
    dev = torch.device("cuda:0")
    K, V = vsgen.make_kv(w, s + C, device=dev)
    Q = vsgen.make_q(w, s, s + C, device=dev)
    pb = oracle.Problem(w.n_q_heads, w.n_kv_heads, w.head_dim, C, s, w.softmax_scale)
    ck = chunk_of(pb)
    out, lse = vs.dense_causal_prefill(ck, Q, K, V, want_lse=True)
    torch.cuda.synchronize()
    heads = [0, 13, 27]
    rows = _sample_rows(np.random.default_rng(1), C, 20)
    ref_out, ref_lse = oracle.dense_attention(pb, vsgen.as_u16(Q), vsgen.as_u16(K), vsgen.as_u16(V), heads=heads, rows=rows)
    _check_rows(out, lse, ref_out, ref_lse, heads, rows, "dense_7b_64k")
    _check_block_classes(lambda Vc: vs.dense_causal_prefill(ck, Q, K, Vc)[0],
                         lambda vc: oracle.dense_attention(pb, vsgen.as_u16(Q), vsgen.as_u16(K), vc, heads=heads, rows=rows),
                         s + C, w, heads, rows, "dense_7b_64k")
    # the sparse entry point with every diagonal selected runs the same tiles: identical bits
    n_k = s + C
    ck2 = vs.Chunk(w.n_q_heads, w.n_kv_heads, w.head_dim, C, s, w.softmax_scale, vertical_budget=1, slash_budget=n_k)
    all_s = torch.arange(n_k, dtype=torch.int32, device=dev).repeat(w.n_q_heads, 1).contiguous()
    cnt_s = torch.full((w.n_q_heads,), n_k, dtype=torch.int32, device=dev)
    v_idx = torch.zeros((w.n_q_heads, 1), dtype=torch.int32, device=dev)
    v_cnt = torch.ones(w.n_q_heads, dtype=torch.int32, device=dev)
    out2, lse2 = vs.sparse_attn_prefill(ck2, Q, K, V, v_idx, v_cnt, all_s, cnt_s, want_lse=True)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16)) and torch.equal(lse, lse2)


def test_sparse_7b_128k_last_chunk():
    _run_sparse_chunk("7b_128k", -1, heads=[0, 9, 27], n_rows=12, seed=2)      # configuration 2


def test_sparse_7b_1m_last_chunk():
    r = _run_sparse_chunk("7b_1m", -1, heads=[3, 20], n_rows=10, seed=3)       # configuration 3
    # recall of the sparse result against the dense kernel (softmax_lse of both, "Sparsity
    # refinement" paragraph) on the first 128 rows of the chunk
    ck, Q, K, V = r["ck"], r["Q"], r["K"], r["V"]
    ck_d = vs.Chunk(ck.n_q_heads, ck.n_kv_heads, ck.head_dim, 128, ck.q_start, ck.softmax_scale)
    _, lse_d = vs.dense_causal_prefill(ck_d, Q[:128], K, V, want_lse=True)
    torch.cuda.synchronize()
    rec = torch.exp(r["lse"][:, :128] - lse_d)
    assert (rec > 0).all() and (rec <= 1 + 1e-3).all()


def test_sparse_7b_1m_middle_chunk():
    _run_sparse_chunk("7b_1m", 15, heads=[11], n_rows=8, seed=4)


def test_sparse_7b_1m_first_chunks():
    # the first chunks of the whole-layer run: no keys before the chunk; budgets that cover nearly every diagonal
    _run_sparse_chunk("7b_1m", 0, heads=[2, 25], n_rows=8, seed=8)
    _run_sparse_chunk("7b_1m", 1, heads=[14], n_rows=8, seed=9)


def test_sparse_7b_1m_local_last_chunk():
    # the clustered regime (slashes close to the diagonal, as real attention maps have them): 11 % of the blocks,
    # long sync segments, short lists
    _run_sparse_chunk("7b_1m_local", -1, heads=[1, 19], n_rows=8, seed=10)


def test_sparse_14b_1m_last_chunk():
    _run_sparse_chunk("14b_1m", -1, heads=[7, 38], n_rows=8, seed=5)            # configuration 4


def test_sparse_7b_1m_dca_chunks():
    # Dual Chunk Attention positions (chunks of 256K): the last prefill chunk meets keys of all three
    # patterns; prefill chunk 8 starts a DCA chunk, so its rows cross the end of the local window
    _run_sparse_chunk("7b_1m_dca", -1, heads=[5, 22], n_rows=8, seed=6)
    _run_sparse_chunk("7b_1m_dca", 8, heads=[16], n_rows=8, seed=7)


def test_determinism_at_headline_size():
    """Run-to-run identical bytes at the sizes of configuration 3: the selection on 56 rows (28 heads x
    {vertical, slash}) of 1,048,576 scores with heavy ties, and the whole chunk call on the last chunk
    (every workgroup slot of the persistent attention launch busy, pace keeping active)."""
    w = vsgen.WORKLOADS["7b_1m"]
    dev = torch.device("cuda:0")
    n_k, C = w.n_ctx, w.chunk
    s = n_k - C
    ck = vs.Chunk(w.n_q_heads, w.n_kv_heads, w.head_dim, C, s, w.softmax_scale, last_q=w.last_q,
                  vertical_budget=w.vertical_budget, slash_budget=w.slash_budget,
                  keep_first_cols=w.keep_first_cols, keep_local_band=w.keep_local_band)
    g = torch.Generator(device=dev).manual_seed(91)
    # 37 distinct score values: thousands of ties at the threshold of every row
    vsc = (torch.randint(0, 37, (w.n_q_heads, n_k), generator=g, device=dev).float() / 64.0).contiguous()
    ssc = (torch.randint(0, 37, (w.n_q_heads, n_k), generator=g, device=dev).float() / 64.0).contiguous()
    a = [x.clone() for x in vs.select(ck, vsc, ssc)]
    b = vs.select(ck, vsc, ssc)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x, y), "vs_select differs between two runs"
    # ties go to the lower index: two heads against the oracle's full sort
    for h in (0, 27):
        ref_v = oracle.select_one(f64(vsc[h]), w.vertical_budget, w.keep_first_cols)
        ref_s = oracle.select_one(f64(ssc[h]), w.slash_budget, w.keep_local_band)
        assert np.array_equal(a[0][h].cpu().numpy()[:len(ref_v)], ref_v) and int(a[1][h]) == len(ref_v)
        assert np.array_equal(a[2][h].cpu().numpy()[:len(ref_s)], ref_s) and int(a[3][h]) == len(ref_s)
    del vsc, ssc
    K, V = vsgen.make_kv(w, n_k, device=dev)
    Q = vsgen.make_q(w, s, n_k, device=dev)
    o1, l1 = vs.prefill_chunk(ck, Q, K, V, want_lse=True)
    o2, l2 = vs.prefill_chunk(ck, Q, K, V, want_lse=True)
    torch.cuda.synchronize()
    assert torch.equal(o1.view(torch.int16), o2.view(torch.int16)), "vs_prefill_chunk: out differs between two runs"
    assert torch.equal(l1, l2), "vs_prefill_chunk: lse differs between two runs"


def test_batched_requests_at_bench_size():
    """The `batched_requests` rows of bench.py (vs_attn_batch, 7B shape, eight requests against caches of
    262,144 keys: single-token steps and chunks of 17 to 64 rows, dense and sparse mixed), in the launch
    bench.py times, on sampled heads and rows; the sparse requests use the index sets the GPU selected."""
    n_keys = 262144
    w = vsgen.scaled(vsgen.WORKLOADS["7b_1m"], n_ctx=n_keys)
    dev = torch.device("cuda:0")
    K, V = vsgen.make_kv(w, n_keys, device=dev)
    kh, vh = vsgen.as_u16(K), vsgen.as_u16(V)
    hq, hkv, d = w.n_q_heads, w.n_kv_heads, w.head_dim
    bv, bs = w.vertical_budget, w.slash_budget
    heads = np.array([0, 6, 7, 27])
    rng = np.random.default_rng(2300)
    for lens, flags in (([1] * 8, [False] * 8), ([1] * 8, [True] * 8),
                        ([1, 17, 64, 1, 17, 64, 33, 64], [False, True, False, True, False, True, False, True])):
        reqs = []
        for i, (c, sp) in enumerate(zip(lens, flags)):
            s = n_keys - c - 64 * i            # every request at its own position
            Q = vsgen.make_q(w, s, s + c, device=dev)
            pb = oracle.Problem(hq, hkv, d, c, s, w.softmax_scale, last_q=w.last_q, vertical_budget=bv, slash_budget=bs,
                                keep_first_cols=w.keep_first_cols, keep_local_band=w.keep_local_band)
            sets = None
            if sp:
                vsc, ssc, _ = vs.estimate(chunk_of(pb), Q, K)
                sets = vs.select(chunk_of(pb), vsc, ssc)
            reqs.append(dict(q=Q, k=K, v=V, q_start=s, sets=sets, pb=pb,
                             out=torch.full((c, hq, d), -3.0, dtype=torch.bfloat16, device=dev),
                             lse=torch.full((hq, c), 7.0, dtype=torch.float32, device=dev)))
        mx = max(lens)
        ckb = vs.Chunk(hq, hkv, d, mx, n_keys - mx, w.softmax_scale, vertical_budget=bv, slash_budget=bs)
        table = vs.request_table(reqs, dev)
        vs.attn_batch(ckb, table, len(reqs), reqs[0]["q"], K, V, reqs[0]["out"])
        torch.cuda.synchronize()
        for i, r in enumerate(reqs):
            pb = r["pb"]
            rows = np.array(sorted(set([0, pb.q_len - 1] + rng.choice(pb.q_len, min(3, pb.q_len), replace=False).tolist())))
            qh = vsgen.as_u16(r["q"])
            if r["sets"] is None:
                ref_out, ref_lse = oracle.dense_attention(pb, qh, kh[:pb.n_k], vh[:pb.n_k], heads=heads, rows=rows)
            else:
                sh = [x.cpu().numpy() for x in r["sets"]]
                ref_out, ref_lse = oracle.sparse_attention(pb, qh, kh[:pb.n_k], vh[:pb.n_k], *sh, heads=heads, rows=rows)
            _check_rows(r["out"], r["lse"], ref_out, ref_lse, heads, rows,
                        f"request {i} ({'sparse' if r['sets'] is not None else 'dense'}, {pb.q_len} rows at {pb.q_start})")


@pytest.mark.parametrize("rows_in_chunk", [1, 64, 1024])
def test_short_chunks_at_1m_keys(rows_in_chunk):
    """The last `rows_in_chunk` tokens of the 1M context (a decode step; the `--chunk-rows` figures of the
    profiles): the key walk of every (tile, head) is cut into ranges and folded, a single token packs the
    heads of a KV group into one tile.  Dense and sparse, sampled heads and rows."""
    w = vsgen.scaled(vsgen.WORKLOADS["7b_1m"], chunk=rows_in_chunk)
    dev = torch.device("cuda:0")
    C = rows_in_chunk
    s, n_k = w.n_ctx - C, w.n_ctx
    K, V = vsgen.make_kv(w, n_k, device=dev)
    Q = vsgen.make_q(w, s, n_k, device=dev)
    pb = oracle.Problem(w.n_q_heads, w.n_kv_heads, w.head_dim, C, s, w.softmax_scale, last_q=w.last_q,
                        vertical_budget=w.vertical_budget, slash_budget=w.slash_budget,
                        keep_first_cols=w.keep_first_cols, keep_local_band=w.keep_local_band)
    ck = chunk_of(pb)
    vsc, ssc, _ = vs.estimate(ck, Q, K)
    sets = vs.select(ck, vsc, ssc)
    out_s, lse_s = vs.sparse_attn_prefill(ck, Q, K, V, *sets, want_lse=True)
    out_d, lse_d = vs.dense_causal_prefill(ck, Q, K, V, want_lse=True)
    torch.cuda.synchronize()
    rng = np.random.default_rng(2400 + C)
    heads = np.array([0, 5, 13, 27])
    rows = np.array(sorted(set([0, C - 1] + rng.choice(C, min(4, C), replace=False).tolist())))
    qh, kh, vh = vsgen.as_u16(Q), vsgen.as_u16(K), vsgen.as_u16(V)
    ref_out, ref_lse = oracle.dense_attention(pb, qh, kh, vh, heads=heads, rows=rows)
    _check_rows(out_d, lse_d, ref_out, ref_lse, heads, rows, f"dense, {C} rows at 1M keys")
    sh = [x.cpu().numpy() for x in sets]
    ref_out, ref_lse = oracle.sparse_attention(pb, qh, kh, vh, *sh, heads=heads, rows=rows)
    _check_rows(out_s, lse_s, ref_out, ref_lse, heads, rows, f"sparse, {C} rows at 1M keys")
