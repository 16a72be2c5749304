"""The whole chunk path under HIP graph capture: the library allocates nothing, synchronises
nothing and clears its workspaces with fill kernels, so a captured chunk can be replayed.
Every replay is compared with the eager result, with eager work between the replays."""
import numpy as np
import pytest
import torch

import paper_2501_15383_amd as vs
import vsgen

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("rows", [512, 64])     # several query tiles; a short chunk (key split and combine kernel)
def test_prefill_chunk_replays_from_a_graph(rows):
    w = vsgen.scaled(vsgen.WORKLOADS["tiny_4k"], n_ctx=8192, chunk=rows)
    dev = torch.device("cuda:0")
    K, V = vsgen.make_kv(w, device=dev)
    s = w.n_ctx - rows
    Q = vsgen.make_q(w, s, w.n_ctx, device=dev)
    ck = vs.Chunk(w.n_q_heads, w.n_kv_heads, w.head_dim, rows, s, w.softmax_scale,
                  vertical_budget=w.vertical_budget, slash_budget=w.slash_budget)
    ws = torch.empty(vs.workspace_bytes(ck, vs.VS_WS_CHUNK), dtype=torch.uint8, device=dev)
    out = torch.empty((rows, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device=dev)
    eager, lse_e = vs.prefill_chunk(ck, Q, K, V, want_lse=True)      # also the first call: one-time set-up happens here
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        lse = torch.empty_like(lse_e)
        with torch.cuda.graph(graph, stream=side):
            p = ck.params(q=Q, k=K, v=V, out=out)
            import ctypes as C
            rc = vs.lib().vs_prefill_chunk(C.byref(p), C.c_void_p(Q.data_ptr()), C.c_void_p(K.data_ptr()),
                                           C.c_void_p(V.data_ptr()), C.c_void_p(out.data_ptr()),
                                           C.c_void_p(lse.data_ptr()), C.c_void_p(ws.data_ptr()), ws.numel(),
                                           C.c_void_p(torch.cuda.current_stream().cuda_stream))
            assert rc == vs.VS_OK
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        out.zero_(); lse.zero_(); ws.random_(0, 255)            # eager work between the replays; stale workspace contents
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), eager.view(torch.int16)), f"replay {rep}"
        assert torch.equal(lse, lse_e), f"replay {rep}"
        again, _ = vs.prefill_chunk(ck, Q, K, V)                 # and an eager call in between
        torch.cuda.synchronize()
        assert torch.equal(again.view(torch.int16), eager.view(torch.int16))


def test_attn_batch_replays_from_a_graph_with_an_updated_request_table():
    """A decode loop as a graph user would run it: the launch is captured once; the request table lives in
    device memory, so each replay serves whatever the table holds by then (here: every request one token on)."""
    import oracle
    from gpu_util import assert_attn_close, dev
    from helpers import rand_bf16
    from test_gpu_attention import _rand_sets, _t
    hq, hkv, d, bv, bs, n_max = 8, 2, 128, 96, 100, 6000
    rng = np.random.default_rng(1900)
    starts = [int(x) for x in rng.integers(100, n_max - 8, 6)]
    host, reqs = [], []
    for i, s in enumerate(starts):
        q_all = rand_bf16(rng, (4, hq, d)); k = rand_bf16(rng, (n_max, hkv, d)); v = rand_bf16(rng, (n_max, hkv, d))
        host.append((q_all, k, v))
        reqs.append(dict(q=dev(q_all[:1]), k=dev(k), v=dev(v), q_start=s,
                         out=torch.zeros((1, hq, d), dtype=torch.bfloat16, device="cuda"),
                         lse=torch.zeros((hq, 1), dtype=torch.float32, device="cuda"), sets=None))
    sets_host = {}
    ck = vs.Chunk(hq, hkv, d, 1, n_max - 1, 1.0 / np.sqrt(d), vertical_budget=bv, slash_budget=bs)

    def fill(step):
        """requests of decode step `step`: token s + step of every cache; odd requests sparse"""
        for i, (r, s) in enumerate(zip(reqs, starts)):
            r["q"].copy_(dev(host[i][0][step:step + 1]))
            r["q_start"] = s + step
            if i % 2:
                pb = oracle.Problem(hq, hkv, d, 1, s + step, 1.0 / np.sqrt(d), vertical_budget=bv, slash_budget=bs)
                sh = _rand_sets(rng, pb, min(bv - 1, 40), 30, force_cols=[0], force_offs=range(64))
                sets_host[i] = (pb, sh)
                if r["sets"] is None:
                    r["sets"] = tuple(_t(x) for x in sh)
                else:
                    for dst, src in zip(r["sets"], sh):
                        dst.copy_(_t(src))
        return vs.request_table(reqs, "cuda")

    table = fill(0)
    ws = vs.attn_batch(ck, table, len(reqs), reqs[0]["q"], reqs[0]["k"], reqs[0]["v"], reqs[0]["out"])   # eager first call
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            vs.attn_batch(ck, table, len(reqs), reqs[0]["q"], reqs[0]["k"], reqs[0]["v"], reqs[0]["out"], ws=ws)
    torch.cuda.current_stream().wait_stream(side)
    for step in range(3):
        table.copy_(fill(step))                                  # eager work between the replays
        for r in reqs:
            r["out"].fill_(-3.0); r["lse"].fill_(7.0)
        ws.random_(0, 255)                                       # stale workspace contents
        graph.replay()
        torch.cuda.synchronize()
        for i, r in enumerate(reqs):
            q = host[i][0][step:step + 1]
            if i % 2:
                pb, sh = sets_host[i]
                ref_out, ref_lse = oracle.sparse_attention(pb, q, host[i][1][:pb.n_k], host[i][2][:pb.n_k], *sh)
            else:
                pb = oracle.Problem(hq, hkv, d, 1, starts[i] + step, 1.0 / np.sqrt(d))
                ref_out, ref_lse = oracle.dense_attention(pb, q, host[i][1][:pb.n_k], host[i][2][:pb.n_k])
            assert_attn_close(r["out"], r["lse"], ref_out, ref_lse, f"replay {step}, request {i}")
