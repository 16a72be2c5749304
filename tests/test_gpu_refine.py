"""GPU parity of the sparsity-refinement pieces (per-head selection, attention recall, one
refinement pass) against the fp64 oracle, through the C ABI, and the loop built from them."""
import numpy as np
import pytest
import torch

import oracle
import paper_2501_15383_amd as vs
from gpu_util import chunk_of, dev, f64
from helpers import rand_bf16

pytestmark = pytest.mark.gpu


def _i32(x):
    return torch.tensor(np.asarray(x, np.int32), dtype=torch.int32, device="cuda")


@pytest.mark.parametrize("n,bv,bs,kf,kb", [(4096, 128, 256, 1, 64), (1000, 37, 90, 0, 0), (70000, 1000, 6096, 1, 64)])
def test_select_heads_is_exact_on_given_scores(n, bv, bs, kf, kb):
    hq = 4
    rng = np.random.default_rng(900 + n)
    vsc = rng.random((hq, n)).astype(np.float32) ** 4
    ssc = rng.random((hq, n)).astype(np.float32) ** 4
    vsc[:, ::7] = vsc[:, 3:4]
    q_start = (n - 1) // 64 * 64
    pb = oracle.Problem(hq, 1, 64, n - q_start, q_start, 1.0, vertical_budget=bv, slash_budget=bs,
                        keep_first_cols=kf, keep_local_band=kb)
    vbud = [1, bv // 3 + 1, bv, bv + 50]          # the last one is clamped to the row length
    sbud = [bs, 1, bs // 2 + 1, 0]                # the last one is clamped to 1
    ref = oracle.select_heads(pb, vsc.astype(np.float64), ssc.astype(np.float64),
                              np.clip(vbud, 1, bv), np.clip(sbud, 1, bs))
    got = vs.select_heads(chunk_of(pb), torch.from_numpy(vsc).cuda(), torch.from_numpy(ssc).cuda(), _i32(vbud), _i32(sbud))
    torch.cuda.synchronize()
    for r, g, nm in zip(ref, got, ["v_idx", "v_cnt", "s_idx", "s_cnt"]):
        np.testing.assert_array_equal(g.cpu().numpy(), r, err_msg=nm)


def test_recall_matches_oracle():
    rng = np.random.default_rng(901)
    hq, c = 5, 3000
    lf = rng.normal(5.0, 2.0, (hq, c))
    ls = lf + np.log(rng.random((hq, c)))
    ls[1, ::9] = -np.inf                               # rows without a selected key
    ls[2] = lf[2]                                      # everything selected
    pb = oracle.Problem(hq, 1, 64, c, 0, 1.0)
    ref = oracle.recall_mean(ls.astype(np.float32).astype(np.float64), lf.astype(np.float32).astype(np.float64))
    got = vs.attention_recall(chunk_of(pb), torch.from_numpy(ls.astype(np.float32)).cuda(),
                              torch.from_numpy(lf.astype(np.float32)).cuda())
    torch.cuda.synchronize()
    np.testing.assert_allclose(f64(got), ref, rtol=2e-6, atol=0)
    assert f64(got)[2] == pytest.approx(1.0, abs=1e-6)


def test_refine_step_matches_oracle():
    hq = 6
    pb = oracle.Problem(hq, 1, 64, 64, 0, 1.0, vertical_budget=25, slash_budget=1000)
    rec = np.array([0.5, 0.9, 0.2, 0.1, 0.95, 0.0], np.float32)
    vb0, sb0 = [20, 20, 20, 25, 3, 1], [100, 100, 950, 1000, 7, 1]
    rvb, rsb, rch = oracle.refine_step(rec.astype(np.float64), float(np.float32(0.9)), 10, 100, 25, 1000, vb0, sb0)
    vb, sb = _i32(vb0), _i32(sb0)
    ch = vs.refine_step(chunk_of(pb), torch.from_numpy(rec).cuda(), 0.9, 10, 100, vb, sb)
    torch.cuda.synchronize()
    assert vb.cpu().tolist() == rvb.tolist() and sb.cpu().tolist() == rsb.tolist() and int(ch.item()) == rch


def test_refinement_loop_on_the_gpu_follows_the_oracle():
    """Algorithm 1 as a loop: dense lse once, then select -> sparse attention -> recall -> refine
    until no head changes.  Budgets and recalls must follow the oracle's loop on the same data."""
    rng = np.random.default_rng(902)
    hq, hkv, d, c, s = 4, 1, 64, 256, 768
    n_k = s + c
    q = rand_bf16(rng, (c, hq, d)); k = rand_bf16(rng, (n_k, hkv, d)); v = rand_bf16(rng, (n_k, hkv, d))
    pb = oracle.Problem(hq, hkv, d, c, s, 1.0 / np.sqrt(d), vertical_budget=96, slash_budget=256,
                        keep_first_cols=1, keep_local_band=64)
    ck = chunk_of(pb)
    Q, K, V = dev(q), dev(k), dev(v)
    thr, dv, ds = 0.9, 16, 32
    # oracle loop
    ovs, oss, _ = oracle.estimate(pb, q, k)
    _, olf = oracle.dense_attention(pb, q, k, v)
    ovb = np.full(hq, 4, np.int32); osb = np.full(hq, 64, np.int32)
    otrace = []
    for _ in range(20):
        sets = oracle.select_heads(pb, ovs, oss, ovb, osb)
        _, ols = oracle.sparse_attention(pb, q, k, v, *sets)
        rec = oracle.recall_mean(ols, olf)
        otrace.append((ovb.copy(), osb.copy(), rec))
        ovb, osb, ch = oracle.refine_step(rec, thr, dv, ds, pb.vertical_budget, pb.slash_budget, ovb, osb)
        if ch == 0:
            break
    # GPU loop
    vsc, ssc, _ = vs.estimate(ck, Q, K)
    _, lf = vs.dense_causal_prefill(ck, Q, K, V, want_lse=True)
    vb = _i32(np.full(hq, 4)); sb = _i32(np.full(hq, 64))
    gtrace = []
    for _ in range(20):
        sets = vs.select_heads(ck, vsc, ssc, vb, sb)
        _, ls = vs.sparse_attn_prefill(ck, Q, K, V, *sets, want_lse=True)
        rec = vs.attention_recall(ck, ls, lf)
        gtrace.append((vb.cpu().numpy().copy(), sb.cpu().numpy().copy(), f64(rec)))
        ch = vs.refine_step(ck, rec, thr, dv, ds, vb, sb)
        if int(ch.item()) == 0:
            break
    # recalls agree to the accuracy of the fp32 lse (scores near the selection threshold may tie
    # differently, which moves a recall by far less than the margin asked for here)
    margin = 5e-3
    clear = all(np.all(np.abs(r - thr) > margin) for _, _, r in otrace)
    assert len(gtrace) == len(otrace) or not clear
    for (gv, gs, gr), (ov, os_, orr) in zip(gtrace, otrace):
        np.testing.assert_allclose(gr, orr, atol=margin, rtol=0)
        if clear:
            assert gv.tolist() == ov.tolist() and gs.tolist() == os_.tolist()
    assert np.all(gtrace[-1][2] >= thr - margin) or np.all(gtrace[-1][0] == pb.vertical_budget)
