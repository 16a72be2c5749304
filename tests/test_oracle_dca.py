"""Pins for the oracle's Dual Chunk Attention variants (section 5.1) -- CPU only.

The pattern of every (query, key) pair is checked against a matrix written out by hand; the
attention and the estimate are checked against numpy brute force that takes its patterns
from that hand-written matrix, and against the plain functions in the cases where DCA must
reduce to them."""
import os

import numpy as np
import pytest

import oracle
from helpers import bf16_to_f64, rand_bf16

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _regions():
    rows = [l.strip() for l in open(os.path.join(GOLD, "dca_regions_c4_w3.txt")) if l.strip() and not l.startswith("#")]
    return [[-1 if c == "." else int(c) for c in r] for r in rows]


def test_patterns_match_the_hand_written_matrix():
    reg = _regions()
    for i in range(10):
        for j in range(i + 1):
            assert oracle.dca_region(i, j, 4, 3) == reg[i][j], (i, j)


def _brute(qv, k, v, q_start, scale, reg, group):
    """Softmax attention where logit (i, j) takes the query tensor qv[reg[pos_i][j]]."""
    C, Hq, D = qv[0].shape
    out = np.zeros((Hq, C, D)); lse = np.zeros((Hq, C)); P = np.zeros((Hq, C, q_start + C))
    for h in range(Hq):
        g = h // group
        for i in range(C):
            pos = q_start + i
            x = np.array([scale * (qv[reg[pos][j]][i, h] @ k[j, g]) for j in range(pos + 1)])
            e = np.exp(x - x.max())
            P[h, i, :pos + 1] = e / e.sum()
            out[h, i] = P[h, i, :pos + 1] @ v[:pos + 1, g]
            lse[h, i] = x.max() + np.log(e.sum())
    return out, lse, P


@pytest.mark.parametrize("c,s", [(10, 0), (6, 4), (3, 7)])
def test_dense_attention_with_dca_equals_brute_force(c, s):
    rng = np.random.default_rng(40 + c)
    hq, hkv, d = 4, 2, 16
    qs = [rand_bf16(rng, (c, hq, d)) for _ in range(3)]
    k = rand_bf16(rng, (s + c, hkv, d)); v = rand_bf16(rng, (s + c, hkv, d))
    pb = oracle.Problem(hq, hkv, d, c, s, 0.3)
    out, lse = oracle.dense_attention(pb, qs[0], k, v, dca=oracle.Dca(4, 3, qs[1], qs[2]))
    ref, ref_lse, _ = _brute([bf16_to_f64(x) for x in qs], bf16_to_f64(k), bf16_to_f64(v), s, 0.3, _regions(), 2)
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, ref_lse, rtol=1e-12, atol=1e-13)


def test_estimate_with_dca_equals_brute_force():
    rng = np.random.default_rng(44)
    hq, hkv, d, c, s, w = 2, 1, 8, 6, 4, 3
    qs = [rand_bf16(rng, (c, hq, d)) for _ in range(3)]
    k = rand_bf16(rng, (s + c, hkv, d))
    pb = oracle.Problem(hq, hkv, d, c, s, 0.5, last_q=w)
    vs, ss, lse = oracle.estimate(pb, qs[0], k, dca=oracle.Dca(4, 3, qs[1], qs[2]))
    _, ref_lse, P = _brute([bf16_to_f64(x) for x in qs], bf16_to_f64(k), np.zeros((s + c, hkv, 1)), s, 0.5, _regions(), 2)
    for h in range(hq):
        Pw = P[h, c - w:]                                   # the window rows
        np.testing.assert_allclose(vs[h], Pw.sum(0), rtol=1e-12, atol=1e-14)
        for o in range(s + c):
            want = sum(Pw[r, s + c - w + r - o] for r in range(w) if s + c - w + r - o >= 0)
            np.testing.assert_allclose(ss[h, o], want, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(lse[h], ref_lse[h, c - w:], rtol=1e-12)


def test_dca_reduces_to_the_plain_functions():
    rng = np.random.default_rng(45)
    hq, hkv, d, c, s = 3, 1, 16, 40, 24
    q = rand_bf16(rng, (c, hq, d)); junk1 = rand_bf16(rng, (c, hq, d)); junk2 = rand_bf16(rng, (c, hq, d))
    k = rand_bf16(rng, (s + c, hkv, d)); v = rand_bf16(rng, (s + c, hkv, d))
    pb = oracle.Problem(hq, hkv, d, c, s, 0.25, block=8, vertical_budget=4, slash_budget=6)
    sets = (np.array([[0, 5, 17, 40]] * hq, np.int32), np.full(hq, 4, np.int32),
            np.array([[0, 1, 2, 9, 30, -1]] * hq, np.int32), np.full(hq, 5, np.int32))
    plain = oracle.sparse_attention(pb, q, k, v, *sets)
    # the three rotations equal: DCA changes nothing
    same = oracle.sparse_attention(pb, q, k, v, *sets, dca=oracle.Dca(16, 8, q, q))
    np.testing.assert_array_equal(same[0], plain[0]); np.testing.assert_array_equal(same[1], plain[1])
    # one chunk holds the whole sequence: only the intra-chunk rotation is ever used
    one = oracle.sparse_attention(pb, q, k, v, *sets, dca=oracle.Dca(64, 8, junk1, junk2))
    np.testing.assert_array_equal(one[0], plain[0])
    e_plain = oracle.estimate(pb, q, k); e_one = oracle.estimate(pb, q, k, dca=oracle.Dca(64, 8, junk1, junk2))
    for a, b in zip(e_plain, e_one):
        np.testing.assert_array_equal(a, b)
    # no local window: the successive-chunk rotation is never used
    a = oracle.dense_attention(pb, q, k, v, dca=oracle.Dca(16, 0, junk1, junk2))
    b = oracle.dense_attention(pb, q, k, v, dca=oracle.Dca(16, 0, junk2, junk2))
    np.testing.assert_array_equal(a[0], b[0])
    # ... and with a window it is: changing it changes rows past the first chunk boundary only
    a = oracle.dense_attention(pb, q, k, v, dca=oracle.Dca(16, 8, junk1, q))
    b = oracle.dense_attention(pb, q, k, v, dca=oracle.Dca(16, 8, junk2, q))
    assert not np.array_equal(a[0], b[0])
