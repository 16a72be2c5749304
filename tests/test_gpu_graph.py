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
