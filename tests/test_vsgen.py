"""The seeded input generator: determinism, slice-ability, stated distribution."""
import math

import torch

import vsgen


def test_slices_reproduce_the_whole():
    w = vsgen.scaled(vsgen.WORKLOADS["tiny_4k"], n_ctx=1024, chunk=256)
    K, V = vsgen.make_kv(w)
    K2, V2 = vsgen.make_kv(w, 700, slab=333)
    assert torch.equal(K2, K[:700]) and torch.equal(V2, V[:700])
    Q = vsgen.make_q(w, 0, 1024)
    assert torch.equal(vsgen.make_q(w, 256, 512), Q[256:512])
    assert torch.equal(vsgen.make_q(w, 0, 1024), Q)            # same seed, same bytes


def test_streams_differ_between_configs_and_tensors():
    a = vsgen.scaled(vsgen.WORKLOADS["tiny_4k"], n_ctx=256, n_sink=0)
    b = vsgen.scaled(a, config_id=7)
    Ka, Va = vsgen.make_kv(a); Kb, _ = vsgen.make_kv(b)
    assert not torch.equal(Ka, Kb) and not torch.equal(Ka, Va)


def test_moments_and_sinks():
    w = vsgen.scaled(vsgen.WORKLOADS["7b_128k"], n_ctx=8192, chunk=2048, n_sink=32)
    K, V = vsgen.make_kv(w)
    v = V.float()
    assert abs(v.mean().item()) < 0.01 and abs(v.std().item() - 1.0) < 0.01
    sinks, mags, u = vsgen.sink_positions(w), vsgen.sink_magnitudes(w), vsgen.unit_vectors(w)
    assert mags == [3.0, 6.0, 12.0, 24.0]
    for g in range(w.n_kv_heads):
        assert len(set(sinks[g].tolist())) == 32 and sinks[g].max() < w.n_ctx
        proj = (K[:, g, :].float() @ u[g])
        assert abs(proj[sinks[g]].mean().item() - mags[g]) < 1.0     # planted component
        assert abs(torch.linalg.norm(u[g]).item() - 1.0) < 1e-5
    # queries carry + u: mean projection on u is 1
    Q = vsgen.make_q(w, 0, 2048)
    G = w.n_q_heads // w.n_kv_heads
    assert abs((Q[:, 0, :].float() @ u[0]).mean().item() - 1.0) < 0.1
    assert abs((Q[:, G, :].float() @ u[1]).mean().item() - 1.0) < 0.1


def test_rope_keeps_norms_and_relative_phase():
    # RoPE is a rotation of (d, d + D/2) pairs: norms are unchanged by it
    w = vsgen.scaled(vsgen.WORKLOADS["dense_7b_64k"], n_ctx=512)
    idx = vsgen._counters(100, 110, 1, 128, "cpu")
    x = vsgen._normal(idx, 1234)
    y = vsgen._rope(x, 100, w.rope_theta)
    assert torch.allclose(x.norm(dim=-1), y.norm(dim=-1), rtol=1e-5)
    # position 0 is the identity
    assert torch.allclose(vsgen._rope(x[:1], 0, 1e7), x[:1])
    # first pair rotates by exactly `pos` radians (frequency theta^0 = 1)
    e = torch.zeros(1, 1, 128); e[0, 0, 0] = 1.0
    r = vsgen._rope(e, 3, 1e7)
    assert abs(r[0, 0, 0].item() - math.cos(3.0)) < 1e-6 and abs(r[0, 0, 64].item() - math.sin(3.0)) < 1e-6


def test_heavy_tail_and_ranged_sink_counts():
    w = vsgen.scaled(vsgen.WORKLOADS["14b_1m"], n_ctx=4096, chunk=1024)
    cnt = vsgen.sink_counts(w)
    assert len(cnt) == 8 and all(32 <= c <= 512 for c in cnt) and len(set(cnt)) > 1
    K, _ = vsgen.make_kv(w)
    norms = K.float().norm(dim=-1) / math.sqrt(128)
    frac_big = (norms > 1.6).float().mean().item()      # exp(z) > 1.6 for ~32% of the 5% picked
    assert 0.005 < frac_big < 0.05


def test_dca_positions_reproduce_the_diagonal_lists_the_paper_prints():
    """Section 5.2, "Integrating with DCA": the caption of its figure prints the relative positions along one
    diagonal in DCA and in the selection of critical tokens.  The pattern of a pair comes from the oracle's
    rule (vso_dca_region), the positions from the input recipe; together they must give the printed lists."""
    import os
    import oracle
    path = os.path.join(os.path.dirname(__file__), "golden", "dca_diagonal_lists.txt")
    rows = [[int(x) for x in l.split()] for l in open(path) if l.strip() and not l.startswith("#")]
    in_dca, in_selection = rows
    c, w, dist = 5, 3, 7
    i = torch.arange(0, 20, dtype=torch.int64)
    key, *q_att = vsgen.dca_positions(i, c, w)
    key_s, *q_sel, w_sel = vsgen.dca_select_positions(i, c, w)
    assert torch.equal(key, key_s) and torch.equal(q_att[0], q_sel[0])     # keys and the intra-chunk rotation are shared
    got_dca, got_sel = [], []
    for qi in range(14, 6, -1):
        kj = qi - dist
        got_dca.append(int(q_att[oracle.dca_region(qi, kj, c, w)][qi] - key[kj]))
        got_sel.append(int(q_sel[oracle.dca_region(qi, kj, c, w_sel)][qi] - key[kj]))
    assert got_dca == in_dca
    assert got_sel == in_selection
    # and the properties the paragraph states: inside a chunk and inside the local window the true distance, in both
    for qi in range(20):
        for kj in range(qi + 1):
            r = oracle.dca_region(qi, kj, c, w)
            rel = int(q_att[r][qi] - key[kj])
            if r < 2:
                assert rel == qi - kj
            assert 0 <= rel <= c + w - 1                                   # never beyond the largest position
            rs = oracle.dca_region(qi, kj, c, w_sel)
            if rs < 2:
                assert int(q_sel[rs][qi] - key[kj]) == qi - kj             # adjacent chunks: continuous
