"""Pins for the oracle's attention (dense and masked) -- CPU only.

Each test checks the oracle against something fixed by the paper or by the
mathematics, not against itself: an independent numpy brute force, closed forms,
hand-written masks (tests/golden), invariants of softmax."""
import os

import numpy as np
import pytest

import oracle
from helpers import bf16_to_f64, brute_attention, rand_bf16

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _load_mask(name):
    rows = [l.strip() for l in open(os.path.join(GOLD, name)) if l.strip() and not l.startswith("#")]
    return np.array([[int(c) for c in r] for r in rows], np.uint8)


def _sets(hq, v_list, s_list, bv, bs):
    v_idx = np.full((hq, bv), -1, np.int32); s_idx = np.full((hq, bs), -1, np.int32)
    v_cnt = np.zeros(hq, np.int32); s_cnt = np.zeros(hq, np.int32)
    for h in range(hq):
        v_idx[h, :len(v_list[h])] = v_list[h]; v_cnt[h] = len(v_list[h])
        s_idx[h, :len(s_list[h])] = s_list[h]; s_cnt[h] = len(s_list[h])
    return v_idx, v_cnt, s_idx, s_cnt


@pytest.mark.parametrize("hq,hkv,d,c,s", [(2, 1, 16, 24, 0), (4, 2, 8, 16, 32), (3, 3, 32, 7, 9)])
def test_dense_equals_brute_force(hq, hkv, d, c, s):
    rng = np.random.default_rng(1)
    q = rand_bf16(rng, (c, hq, d)); k = rand_bf16(rng, (s + c, hkv, d)); v = rand_bf16(rng, (s + c, hkv, d))
    pb = oracle.Problem(hq, hkv, d, c, s, 0.37)
    out, lse = oracle.dense_attention(pb, q, k, v)
    ref, ref_lse = brute_attention(bf16_to_f64(q), bf16_to_f64(k), bf16_to_f64(v), s, 0.37, group=hq // hkv)
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, ref_lse, rtol=1e-12, atol=1e-13)


def test_dense_closed_forms_at_zero_queries():
    # Q = 0: uniform weights, so out[i] = mean(V[0..pos]) and lse = log(pos + 1).
    rng = np.random.default_rng(2)
    c, s, d = 20, 12, 8
    q = np.zeros((c, 2, d), np.uint16); k = rand_bf16(rng, (s + c, 1, d)); v = rand_bf16(rng, (s + c, 1, d))
    out, lse = oracle.dense_attention(oracle.Problem(2, 1, d, c, s, 1.0), q, k, v)
    vf = bf16_to_f64(v)[:, 0, :]
    for i in range(c):
        np.testing.assert_allclose(out[0, i], vf[: s + i + 1].mean(0), rtol=1e-13, atol=1e-14)
        np.testing.assert_allclose(lse[1, i], np.log(s + i + 1), rtol=1e-14)


def test_rows_of_weights_sum_to_one_dense_and_sparse():
    # V == 1 -> out == 1 for any mask with at least one key (a key in both a vertical
    # line and a slash block must be counted once).
    rng = np.random.default_rng(3)
    c, s, d, hq = 48, 16, 16, 2
    q = rand_bf16(rng, (c, hq, d)); k = rand_bf16(rng, (s + c, 1, d))
    v = np.full((s + c, 1, d), 0x3F80, np.uint16)  # bf16 1.0
    pb = oracle.Problem(hq, 1, d, c, s, 0.5, block=4, vertical_budget=6, slash_budget=5)
    sets = _sets(hq, [[0, 3, 17, 18, 40, 63]] * hq, [[0, 1, 2, 9, 30]] * hq, 6, 5)
    o_s, _ = oracle.sparse_attention(pb, q, k, v, *sets)
    o_d, _ = oracle.dense_attention(pb, q, k, v)
    np.testing.assert_allclose(o_s, 1.0, rtol=1e-13)
    np.testing.assert_allclose(o_d, 1.0, rtol=1e-13)


def test_hand_mask_block_mode():
    gold = _load_mask("hand_mask_n24_b4.txt")
    assert gold.shape == (24, 24)
    pb = oracle.Problem(1, 1, 8, 24, 0, 1.0, block=4, vertical_budget=2, slash_budget=3)
    m = oracle.mask(pb, [0, 5], [0, 1, 6])
    np.testing.assert_array_equal(m, gold)


def test_hand_mask_token_mode_and_literal_rule():
    gold = _load_mask("hand_mask_n12_b1.txt")
    pb = oracle.Problem(1, 1, 8, 12, 0, 1.0, block=1, vertical_budget=2, slash_budget=3)
    m = oracle.mask(pb, [0, 5], [0, 1, 6])
    np.testing.assert_array_equal(m, gold)
    # B = 1 is the literal rule "j in V or pos - j in S" for any sets / any chunk offset
    rng = np.random.default_rng(4)
    s, c = 40, 23
    V = sorted(rng.choice(s + c, 7, replace=False).tolist()); S = sorted(rng.choice(s + c, 9, replace=False).tolist())
    pb = oracle.Problem(1, 1, 8, c, s, 1.0, block=1, vertical_budget=7, slash_budget=9)
    m = oracle.mask(pb, V, S)
    for i in range(c):
        for j in range(s + c):
            assert m[i, j] == int(j <= s + i and (j in V or (s + i - j) in S))


def test_block_mask_contains_token_mask_and_block_rule():
    rng = np.random.default_rng(5)
    s, c, B = 32, 40, 8
    V = sorted(rng.choice(s + c, 5, replace=False).tolist()); S = sorted(rng.choice(s + c, 6, replace=False).tolist())
    mb = oracle.mask(oracle.Problem(1, 1, 8, c, s, 1.0, block=B, vertical_budget=5, slash_budget=6), V, S)
    mt = oracle.mask(oracle.Problem(1, 1, 8, c, s, 1.0, block=1, vertical_budget=5, slash_budget=6), V, S)
    assert np.all(mb >= mt)
    # a (query block, key block) tile is attended iff some selected diagonal crosses it
    for i in range(c):
        for j in range(s + c):
            if j > s + i or j in V:
                continue
            mq, nk = (s + i) // B, j // B
            crosses = any(0 <= (mq * B + a) - o - nk * B < B for o in S for a in range(B))
            assert mb[i, j] == int(crosses), (i, j)


def test_sparse_attention_equals_brute_force_on_oracle_mask_gold():
    # attention over the hand-written mask, computed by an independent brute force
    gold = _load_mask("hand_mask_n24_b4.txt")
    rng = np.random.default_rng(6)
    d = 16
    q = rand_bf16(rng, (24, 1, d)); k = rand_bf16(rng, (24, 1, d)); v = rand_bf16(rng, (24, 1, d))
    pb = oracle.Problem(1, 1, d, 24, 0, 0.25, block=4, vertical_budget=2, slash_budget=3)
    out, lse = oracle.sparse_attention(pb, q, k, v, *_sets(1, [[0, 5]], [[0, 1, 6]], 2, 3))
    ref, ref_lse = brute_attention(bf16_to_f64(q), bf16_to_f64(k), bf16_to_f64(v), 0, 0.25, mask=gold[None])
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, ref_lse, rtol=1e-12, atol=1e-13)


def test_everything_selected_is_dense_bit_for_bit():
    rng = np.random.default_rng(7)
    hq, hkv, d, c, s = 4, 2, 16, 40, 24
    n_k = s + c
    q = rand_bf16(rng, (c, hq, d)); k = rand_bf16(rng, (n_k, hkv, d)); v = rand_bf16(rng, (n_k, hkv, d))
    pb = oracle.Problem(hq, hkv, d, c, s, 0.25, block=8, vertical_budget=n_k, slash_budget=n_k)
    allv = [list(range(n_k))] * hq
    o_d, l_d = oracle.dense_attention(pb, q, k, v)
    o_s, l_s = oracle.sparse_attention(pb, q, k, v, *_sets(hq, allv, allv, n_k, n_k))
    assert np.array_equal(o_d, o_s) and np.array_equal(l_d, l_s)
    # all diagonals alone already give dense
    o_s2, _ = oracle.sparse_attention(pb, q, k, v, *_sets(hq, [[0]] * hq, allv, n_k, n_k))
    assert np.array_equal(o_d, o_s2)


def test_recall_in_unit_interval_and_monotone_in_budget():
    # Attention_Recall = exp(lse_sparse - lse_full) lies in (0, 1] and cannot fall when
    # lines are added ("Sparsity refinement" paragraph).
    rng = np.random.default_rng(8)
    hq, d, c, s = 2, 16, 32, 32
    n_k = s + c
    q = rand_bf16(rng, (c, hq, d)); k = rand_bf16(rng, (n_k, 1, d)); v = rand_bf16(rng, (n_k, 1, d))
    base = oracle.Problem(hq, 1, d, c, s, 0.25, block=8, vertical_budget=n_k, slash_budget=n_k)
    _, l_full = oracle.dense_attention(base, q, k, v)
    order_v = rng.permutation(n_k).tolist(); order_s = rng.permutation(n_k).tolist()
    prev = None
    for nv, ns in [(1, 8), (4, 8), (4, 12), (16, 20), (n_k, n_k)]:
        vl = sorted(set([0] + order_v[:nv])); sl = sorted(set(list(range(8)) + order_s[:ns]))
        _, l_sp = oracle.sparse_attention(base, q, k, v, *_sets(hq, [vl] * hq, [sl] * hq, n_k, n_k))
        rec = oracle.attention_recall(l_sp, l_full)
        assert np.all(rec > 0) and np.all(rec <= 1 + 1e-12)
        if prev is not None:
            assert np.all(rec >= prev - 1e-12)
        prev = rec
    np.testing.assert_allclose(prev, 1.0, rtol=1e-12)


def test_gqa_equals_expanded_mha():
    rng = np.random.default_rng(9)
    hq, hkv, d, c, s = 6, 2, 8, 16, 8
    n_k = s + c
    q = rand_bf16(rng, (c, hq, d)); k = rand_bf16(rng, (n_k, hkv, d)); v = rand_bf16(rng, (n_k, hkv, d))
    sets = _sets(hq, [[0, 3, 9]] * hq, [[0, 1, 2, 3, 13]] * hq, 3, 5)
    pg = oracle.Problem(hq, hkv, d, c, s, 0.3, block=4, vertical_budget=3, slash_budget=5)
    pm = oracle.Problem(hq, hq, d, c, s, 0.3, block=4, vertical_budget=3, slash_budget=5)
    ke = np.repeat(k, hq // hkv, axis=1); ve = np.repeat(v, hq // hkv, axis=1)
    a = oracle.sparse_attention(pg, q, k, v, *sets); b = oracle.sparse_attention(pm, q, ke, ve, *sets)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_dense_chunked_equals_one_shot():
    rng = np.random.default_rng(10)
    hq, d, n = 2, 8, 48
    q = rand_bf16(rng, (n, hq, d)); k = rand_bf16(rng, (n, 1, d)); v = rand_bf16(rng, (n, 1, d))
    full, _ = oracle.dense_attention(oracle.Problem(hq, 1, d, n, 0, 0.4), q, k, v)
    for s in range(0, n, 16):
        part, _ = oracle.dense_attention(oracle.Problem(hq, 1, d, 16, s, 0.4), q[s:s + 16], k, v)
        assert np.array_equal(part, full[:, s:s + 16])


def test_row_and_head_subsets_match_full_run():
    rng = np.random.default_rng(11)
    hq, d, c, s = 4, 8, 24, 8
    q = rand_bf16(rng, (c, hq, d)); k = rand_bf16(rng, (s + c, 2, d)); v = rand_bf16(rng, (s + c, 2, d))
    pb = oracle.Problem(hq, 2, d, c, s, 0.4, block=4, vertical_budget=2, slash_budget=4)
    sets = _sets(hq, [[0, 7]] * hq, [[0, 1, 2, 3]] * hq, 2, 4)
    full, lf = oracle.sparse_attention(pb, q, k, v, *sets)
    sub, ls = oracle.sparse_attention(pb, q, k, v, *sets, heads=[3, 1], rows=[23, 0, 5])
    assert np.array_equal(sub, full[[3, 1]][:, [23, 0, 5]]) and np.array_equal(ls, lf[[3, 1]][:, [23, 0, 5]])


def test_empty_mask_row_gives_zero_and_minus_inf():
    rng = np.random.default_rng(12)
    d, c = 8, 12
    q = rand_bf16(rng, (c, 1, d)); k = rand_bf16(rng, (c, 1, d)); v = rand_bf16(rng, (c, 1, d))
    pb = oracle.Problem(1, 1, d, c, 0, 1.0, block=1, vertical_budget=1, slash_budget=1,
                        keep_first_cols=0, keep_local_band=0)
    out, lse = oracle.sparse_attention(pb, q, k, v, *_sets(1, [[3]], [[2]], 1, 1))
    # rows 0, 1 see neither column 3 nor offset 2
    assert np.all(out[0, :2] == 0) and np.all(np.isneginf(lse[0, :2])) and np.isfinite(lse[0, 2:]).all()


def test_yarn_temperature_closed_form():
    # sqrt(1/t) = 0.1 ln s + 1 (YaRN equation); s = 4 -> 1/t = 1.2964...
    assert abs(oracle.yarn_softmax_scale(4.0, 128) * np.sqrt(128) - (0.1 * np.log(4.0) + 1) ** 2) < 1e-15
    assert abs(oracle.yarn_softmax_scale(4.0, 64) * 8 - 1.2964769) < 1e-6
    assert oracle.yarn_softmax_scale(1.0, 64) == 1 / 8
