"""Pins of the oracle's sparsity-refinement pieces (section 5.2, "Sparsity refinement" and
Algorithm 1): recall of a head, one refinement pass, per-head selection."""
import numpy as np

import oracle
from helpers import rand_bf16


def _problem(rng, hq=3, hkv=1, d=64, c=128, s=128, bv=24, bs=40):
    n_k = s + c
    q = rand_bf16(rng, (c, hq, d)); k = rand_bf16(rng, (n_k, hkv, d)); v = rand_bf16(rng, (n_k, hkv, d))
    pb = oracle.Problem(hq, hkv, d, c, s, 1.0 / np.sqrt(d), vertical_budget=bv, slash_budget=bs,
                        keep_first_cols=1, keep_local_band=8)
    return pb, q, k, v


def test_recall_mean_closed_form():
    # lse_sparse = lse_full + log r  =>  recall = mean r; a row with no selected key counts 0
    r = np.array([[1.0, 0.5, 0.25, 0.125], [0.1, 0.2, 0.3, 0.0]])
    lf = np.array([[3.0, -2.0, 7.5, 0.0], [1.0, 2.0, 3.0, 4.0]])
    with np.errstate(divide="ignore"):
        ls = lf + np.log(r)
    got = oracle.recall_mean(ls, lf)
    assert np.allclose(got, [0.46875, 0.15], rtol=0, atol=1e-15)


def test_recall_is_one_when_everything_is_selected_and_grows_with_budgets():
    rng = np.random.default_rng(5)
    pb, q, k, v = _problem(rng)
    vs_, ss_, _ = oracle.estimate(pb, q, k)
    _, lse_full = oracle.dense_attention(pb, q, k, v)
    prev = None
    for bv, bs in [(2, 9), (8, 16), (24, 40), (pb.n_k, pb.n_k)]:
        pbb = oracle.Problem(pb.n_q_heads, pb.n_kv_heads, pb.head_dim, pb.q_len, pb.q_start, pb.softmax_scale,
                             vertical_budget=bv, slash_budget=bs, keep_first_cols=1, keep_local_band=8)
        sets = oracle.select(pbb, vs_, ss_)
        _, lse_s = oracle.sparse_attention(pbb, q, k, v, *sets)
        rec = oracle.recall_mean(lse_s, lse_full)
        assert np.all(rec > 0) and np.all(rec <= 1 + 1e-12)
        if prev is not None:
            assert np.all(rec >= prev - 1e-12)      # nested sets => nested masks => recall cannot drop
        prev = rec
    assert np.allclose(prev, 1.0, rtol=0, atol=1e-12)   # every column and diagonal selected


def test_refine_step_hand_example():
    # head 0 below the threshold: grows; head 1 at the threshold: unchanged (strictly below only);
    # head 2 below: clamped at the maxima; head 3 below but already at the maxima: not counted
    vb, sb, ch = oracle.refine_step([0.5, 0.9, 0.2, 0.1], 0.9, 10, 100, 25, 1000, [20, 20, 20, 25], [100, 100, 950, 1000])
    assert vb.tolist() == [25, 20, 25, 25] and sb.tolist() == [200, 100, 1000, 1000] and ch == 2
    vb2, sb2, ch2 = oracle.refine_step([0.95, 0.9, 0.99, 1.0], 0.9, 10, 100, 25, 1000, vb, sb)
    assert vb2.tolist() == vb.tolist() and sb2.tolist() == sb.tolist() and ch2 == 0


def test_select_heads_equals_select_one_per_head():
    rng = np.random.default_rng(6)
    pb, q, k, v = _problem(rng)
    vs_, ss_, _ = oracle.estimate(pb, q, k)
    vbud, sbud = [1, 7, 24], [8, 40, 13]
    v_idx, v_cnt, s_idx, s_cnt = oracle.select_heads(pb, vs_, ss_, vbud, sbud)
    for h in range(3):
        # independent statement of the rule: stable order by (score desc, index asc) with forced entries first
        for score, bud, keep, idx, cnt in ((vs_[h], vbud[h], 1, v_idx[h], v_cnt[h]), (ss_[h], sbud[h], 8, s_idx[h], s_cnt[h])):
            sc = score.copy(); sc[:keep] = np.inf
            want = np.sort(np.argsort(-sc, kind="stable")[:bud])
            assert cnt == bud and idx[:cnt].tolist() == want.tolist() and np.all(idx[cnt:] == -1)


def test_refinement_loop_terminates_and_only_grows():
    rng = np.random.default_rng(7)
    pb, q, k, v = _problem(rng, bv=64, bs=128)
    vs_, ss_, _ = oracle.estimate(pb, q, k)
    _, lse_full = oracle.dense_attention(pb, q, k, v)
    vb = np.array([2, 2, 2], np.int32); sb = np.array([9, 9, 9], np.int32)
    history = []
    for _ in range(40):
        sets = oracle.select_heads(pb, vs_, ss_, vb, sb)
        _, lse_s = oracle.sparse_attention(pb, q, k, v, *sets)
        rec = oracle.recall_mean(lse_s, lse_full)
        history.append(rec)
        nvb, nsb, ch = oracle.refine_step(rec, 0.95, 4, 8, pb.vertical_budget, pb.slash_budget, vb, sb)
        assert np.all(nvb >= vb) and np.all(nsb >= sb)
        vb, sb = nvb, nsb
        if ch == 0:
            break
    assert ch == 0
    done = (history[-1] >= 0.95) | ((vb == pb.vertical_budget) & (sb == pb.slash_budget))
    assert np.all(done)
    assert all(np.all(b >= a - 1e-12) for a, b in zip(history, history[1:]))
