"""End-to-end GPU parity of one chunk of the whole path (estimate -> select -> sparse
attention) on the small configuration, plus the chunk entry point against its stages."""
import numpy as np
import pytest
import torch

import oracle
import paper_2501_15383_amd as vs
import vsgen
from gpu_util import assert_attn_close, chunk_of

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("bv,bs", [(128, 256), (64, 80)])
def test_small_configuration_all_chunks(bv, bs):
    # Bs = 256 of <= 4096 offsets covers every block diagonal (sparse == dense there); Bs = 80
    # leaves 16 free diagonals so the mask is really sparse.
    w = vsgen.scaled(vsgen.WORKLOADS["tiny_4k"], vertical_budget=bv, slash_budget=bs)
    K, V = vsgen.make_kv(w); Q = vsgen.make_q(w, 0, w.n_ctx)
    Kd, Vd = K.cuda(), V.cuda()
    ku, vu = vsgen.as_u16(K), vsgen.as_u16(V)
    for ci in range(w.n_chunks):
        s = ci * w.chunk
        pb = oracle.Problem(w.n_q_heads, w.n_kv_heads, w.head_dim, w.chunk, s, w.softmax_scale,
                            vertical_budget=bv, slash_budget=bs)
        ck = chunk_of(pb)
        qd = Q[s:s + w.chunk].cuda()
        vsc, ssc, _ = vs.estimate(ck, qd, Kd)
        sets = vs.select(ck, vsc, ssc)
        out, lse = vs.sparse_attn_prefill(ck, qd, Kd, Vd, *sets, want_lse=True)
        out2, lse2 = vs.prefill_chunk(ck, qd, Kd, Vd, want_lse=True)
        torch.cuda.synchronize()
        # the one-call entry point is the same three stages
        assert torch.equal(out.view(torch.int16), out2.view(torch.int16)) and torch.equal(lse, lse2)
        # oracle attention fed the GPU's index sets isolates the attention stage
        ref_out, ref_lse = oracle.sparse_attention(pb, vsgen.as_u16(Q[s:s + w.chunk]), ku, vu,
                                                   *[x.cpu().numpy() for x in sets])
        assert_attn_close(out, lse, ref_out, ref_lse, f"chunk {ci} Bv={bv} Bs={bs}")
        # recall against the dense kernel lies in (0, 1]
        _, lse_d = vs.dense_causal_prefill(ck, qd, Kd, Vd, want_lse=True)
        rec = torch.exp(lse - lse_d)
        assert (rec > 0).all() and (rec <= 1 + 1e-4).all()


def test_clustered_slash_workload_last_chunks():
    """The extra workload with planted, clustered slash lines (scaled down): whole path against the
    oracle, index sets by the band rule, attention on the GPU's own sets."""
    from gpu_util import check_index_sets, f64
    w = vsgen.scaled(vsgen.WORKLOADS["7b_1m_local"], n_ctx=12288, chunk=1024, n_q_heads=4, n_kv_heads=2,
                     vertical_budget=96, slash_budget=320, n_sink=24)
    K, V = vsgen.make_kv(w)
    Kd, Vd = K.cuda(), V.cuda()
    ku, vu = vsgen.as_u16(K), vsgen.as_u16(V)
    for ci in (w.n_chunks - 2, w.n_chunks - 1):
        s = ci * w.chunk
        Q = vsgen.make_q(w, s, s + w.chunk)
        pb = oracle.Problem(w.n_q_heads, w.n_kv_heads, w.head_dim, w.chunk, s, w.softmax_scale,
                            vertical_budget=w.vertical_budget, slash_budget=w.slash_budget)
        ck = chunk_of(pb)
        qd = Q.cuda()
        vsc, ssc, _ = vs.estimate(ck, qd, Kd)
        sets = vs.select(ck, vsc, ssc)
        out, lse = vs.sparse_attn_prefill(ck, qd, Kd, Vd, *sets, want_lse=True)
        torch.cuda.synchronize()
        rvs, rss, _ = oracle.estimate(pb, vsgen.as_u16(Q), ku)
        np.testing.assert_allclose(f64(vsc), rvs, rtol=2e-4, atol=1e-7)
        np.testing.assert_allclose(f64(ssc), rss, rtol=2e-4, atol=1e-7)
        v_idx, v_cnt, s_idx, s_cnt = [x.cpu().numpy() for x in sets]
        for h in range(w.n_q_heads):
            check_index_sets(rvs[h], v_idx[h], v_cnt[h], w.vertical_budget, 1, f"chunk {ci} head {h} vertical")
            check_index_sets(rss[h], s_idx[h], s_cnt[h], w.slash_budget, 64, f"chunk {ci} head {h} slash")
        # the planted structure shows: most selected offsets are small
        assert np.median(s_idx[0][: s_cnt[0]]) < pb.n_k / 8
        ref_out, ref_lse = oracle.sparse_attention(pb, vsgen.as_u16(Q), ku, vu, v_idx, v_cnt, s_idx, s_cnt)
        assert_attn_close(out, lse, ref_out, ref_lse, f"clustered chunk {ci}")
