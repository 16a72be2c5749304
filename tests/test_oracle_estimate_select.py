"""Pins for the oracle's estimation (last-q scoring) and selection -- CPU only."""
import numpy as np
import pytest

import oracle
from helpers import bf16_round, bf16_to_f64, rand_bf16


def _brute_estimate(q, k, s, W, scale, group):
    """Independent numpy statement: causal softmax of the last W rows, then column sums
    and sums along diagonals pos - j = o."""
    C, Hq, D = q.shape
    n_k = s + C
    Wp = min(W, C)
    vs = np.zeros((Hq, n_k)); ss = np.zeros((Hq, n_k)); lse = np.zeros((Hq, Wp))
    for h in range(Hq):
        for r in range(Wp):
            i = C - Wp + r; pos = s + i
            x = scale * (k[: pos + 1, h // group, :] @ q[i, h, :])
            p = np.exp(x - x.max()); L = p.sum(); p /= L
            lse[h, r] = x.max() + np.log(L)
            vs[h, : pos + 1] += p
            ss[h, pos - np.arange(pos + 1)] += p
    return vs, ss, lse


@pytest.mark.parametrize("hq,hkv,d,c,s,w", [(2, 1, 16, 40, 24, 8), (4, 2, 8, 5, 0, 8), (3, 1, 32, 64, 192, 64)])
def test_estimate_equals_brute_force(hq, hkv, d, c, s, w):
    rng = np.random.default_rng(20)
    q = rand_bf16(rng, (c, hq, d)); k = rand_bf16(rng, (s + c, hkv, d))
    pb = oracle.Problem(hq, hkv, d, c, s, 0.3, last_q=w)
    vs, ss, lse = oracle.estimate(pb, q, k)
    bvs, bss, blse = _brute_estimate(bf16_to_f64(q), bf16_to_f64(k), s, w, 0.3, hq // hkv)
    np.testing.assert_allclose(vs, bvs, rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(ss, bss, rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(lse, blse, rtol=1e-12)


def test_score_conservation():
    # every window row is a probability vector, so both score vectors total W'
    rng = np.random.default_rng(21)
    for c, w in [(100, 64), (10, 64), (64, 16)]:
        q = rand_bf16(rng, (c, 2, 16), 2.0); k = rand_bf16(rng, (32 + c, 1, 16), 2.0)
        vs, ss, _ = oracle.estimate(oracle.Problem(2, 1, 16, c, 32, 0.25, last_q=w), q, k)
        np.testing.assert_allclose(vs.sum(1), min(w, c), rtol=1e-12)
        np.testing.assert_allclose(ss.sum(1), min(w, c), rtol=1e-12)
        assert (vs >= 0).all() and (ss >= 0).all()


def test_closed_form_at_zero_queries():
    # Q = 0: P[r][j] = 1/(pos_r + 1), hence vscore[j] = sum_{r: pos_r >= j} 1/(pos_r+1) and
    # sscore[o] has the same closed form in o.
    c, s, w = 24, 40, 8
    rng = np.random.default_rng(22)
    q = np.zeros((c, 1, 8), np.uint16); k = rand_bf16(rng, (s + c, 1, 8))
    vs, ss, lse = oracle.estimate(oracle.Problem(1, 1, 8, c, s, 1.0, last_q=w), q, k)
    pos = s + c - w + np.arange(w)
    for x in range(s + c):
        expect = sum(1.0 / (p + 1) for p in pos if p >= x)
        assert abs(vs[0, x] - expect) < 1e-14 and abs(ss[0, x] - expect) < 1e-14
    np.testing.assert_allclose(lse[0], np.log(pos + 1.0), rtol=1e-14)


def test_dominant_key_makes_a_vertical_line_and_its_diagonals():
    # one key aligned with every query and much larger than the rest: its column collects
    # every window row that can see it, and each row puts its mass on offset pos_r - j*.
    c, s, w, d = 32, 32, 8, 8
    q = np.zeros((c, 1, d)); q[:, 0, 0] = 8.0
    k = np.zeros((s + c, 1, d)); jstar = 37; k[jstar, 0, 0] = 8.0
    vs, ss, _ = oracle.estimate(oracle.Problem(1, 1, d, c, s, 1.0, last_q=w), bf16_round(q), bf16_round(k))
    assert abs(vs[0, jstar] - w) < 1e-9
    pos = s + c - w + np.arange(w)
    for p in pos:
        assert abs(ss[0, p - jstar] - 1.0) < 1e-9
    assert abs(ss[0].sum() - w) < 1e-9 and np.delete(vs[0], jstar).max() < 1e-9


def test_lse_of_window_rows_equals_dense_lse():
    rng = np.random.default_rng(23)
    c, s, w = 20, 12, 8
    q = rand_bf16(rng, (c, 2, 16)); k = rand_bf16(rng, (s + c, 1, 16)); v = rand_bf16(rng, (s + c, 1, 16))
    pb = oracle.Problem(2, 1, 16, c, s, 0.25, last_q=w)
    _, _, lse_w = oracle.estimate(pb, q, k)
    _, lse_d = oracle.dense_attention(pb, q, k, v, rows=list(range(c - w, c)))
    np.testing.assert_allclose(lse_w, lse_d, rtol=1e-13)


def test_selection_depends_only_on_window_queries():
    # the chunk's own last W tokens decide its lines ("Integrating with Chunked prefill")
    rng = np.random.default_rng(24)
    c, s, w = 40, 24, 8
    q = rand_bf16(rng, (c, 2, 16)); k = rand_bf16(rng, (s + c, 1, 16))
    pb = oracle.Problem(2, 1, 16, c, s, 0.25, last_q=w, vertical_budget=6, slash_budget=10, keep_local_band=4)
    a = oracle.estimate(pb, q, k)
    q2 = q.copy(); q2[: c - w] = rand_bf16(rng, (c - w, 2, 16))
    b = oracle.estimate(pb, q2, k)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    q3 = q.copy(); q3[c - 1] = rand_bf16(rng, (2, 16))
    assert not np.array_equal(oracle.estimate(pb, q3, k)[0], a[0])


# ----------------------------------------------------------------------------- selection
def _brute_select(score, budget, n_forced):
    sc = np.array(score, np.float64); sc[:n_forced] = np.inf
    order = np.argsort(-sc, kind="stable")          # score descending, index ascending on ties
    return np.sort(order[: min(budget, len(sc))]).astype(np.int32)


def test_select_equals_stable_argsort():
    rng = np.random.default_rng(30)
    for n, k, f in [(100, 10, 1), (100, 100, 4), (50, 80, 0), (257, 64, 64), (1000, 37, 3), (8, 3, 5)]:
        sc = rng.random(n)
        np.testing.assert_array_equal(oracle.select_one(sc, k, f), _brute_select(sc, k, f))


def test_select_ties_go_to_the_lowest_index_and_forced_are_kept():
    np.testing.assert_array_equal(oracle.select_one(np.ones(20), 5, 0), np.arange(5))
    sc = np.zeros(30); sc[[7, 9, 11]] = 1.0
    np.testing.assert_array_equal(oracle.select_one(sc, 6, 2), [0, 1, 2, 7, 9, 11])
    # forced entries survive even with the lowest scores
    sc = np.linspace(0, 1, 40)
    got = oracle.select_one(sc, 5, 3)
    np.testing.assert_array_equal(got, [0, 1, 2, 38, 39])


def test_select_nested_in_budget_and_permutation_equivariant():
    rng = np.random.default_rng(31)
    sc = rng.random(200)
    prev = set()
    for k in range(1, 60, 7):
        cur = set(oracle.select_one(sc, k, 1).tolist())
        assert prev <= cur and len(cur) == k
        prev = cur
    perm = rng.permutation(200)
    a = oracle.select_one(sc, 25, 0); b = oracle.select_one(sc[perm], 25, 0)
    assert set(perm[b].tolist()) == set(a.tolist())


def test_select_all_heads_wrapper_counts_and_padding():
    rng = np.random.default_rng(32)
    pb = oracle.Problem(3, 1, 8, 16, 16, 1.0, vertical_budget=40, slash_budget=6, keep_first_cols=1, keep_local_band=4)
    vs = rng.random((3, 32)); ss = rng.random((3, 32))
    v_idx, v_cnt, s_idx, s_cnt = oracle.select(pb, vs, ss)
    assert list(v_cnt) == [32] * 3 and list(s_cnt) == [6] * 3          # budget clamped to n_k
    assert (v_idx[:, 32:] == -1).all()
    for h in range(3):
        np.testing.assert_array_equal(v_idx[h, :32], np.arange(32))
        np.testing.assert_array_equal(s_idx[h], _brute_select(ss[h], 6, 4))
