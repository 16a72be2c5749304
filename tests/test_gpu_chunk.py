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
