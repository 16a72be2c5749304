"""Seeded random sweep over shapes, positions, index sets and launch options: every stage of the
path against the fp64 oracle through the C ABI (dense and sparse attention, with and without
Dual Chunk Attention, estimate, selection).  The point is the combinations the hand-picked cases
of the other files do not list."""
import numpy as np
import pytest
import torch

import oracle
import paper_2501_15383_amd as vs
from gpu_util import assert_attn_close, chunk_of, dev, f64
from helpers import rand_bf16
from test_gpu_attention import _rand_sets, _t

pytestmark = pytest.mark.gpu


def _case(rng, max_start, long_chunks):
    d = int(rng.choice([64, 128])); hkv = int(rng.choice([1, 2, 3])); g = int(rng.choice([1, 2, 4, 5, 7])); hq = hkv * g
    c = int(rng.choice([1, 3, 31, 64, 65, 100, 128, 200, 256, 384, 513] + ([1024, 2500] if long_chunks else [])))
    s = int(rng.integers(0, max_start))
    if rng.random() < 0.5:
        s = s // 64 * 64
    n_k = s + c
    dca = (int(rng.choice([64, 128, 256, 512, 1024])), int(rng.choice([0, 64, 128, 320]))) if rng.random() < 0.4 else None
    opts = (int(rng.choice([0, 1, 2, 3, 16])), int(rng.choice([0, 1, 2, 7])), int(rng.integers(0, 2)))
    nv = int(rng.integers(1, min(n_k, 200) + 1)); ns = int(rng.integers(1, min(n_k, 60) + 1)); band = int(rng.choice([0, 64]))
    pb = oracle.Problem(hq, hkv, d, c, s, 1.0 / np.sqrt(d), last_q=int(rng.choice([64, 16, 1])),
                        vertical_budget=nv + 8, slash_budget=ns + band + 8,
                        keep_first_cols=1 if band else 0, keep_local_band=band)
    return pb, dca, opts, nv, ns, band


@pytest.mark.parametrize("seed,n_cases,max_start,long_chunks", [(11, 60, 3000, False), (12, 20, 30000, True)])
def test_random_cases_match_the_oracle(seed, n_cases, max_start, long_chunks):
    rng = np.random.default_rng(seed)
    try:
        for it in range(n_cases):
            pb, dca, (split, seg, turn), nv, ns, band = _case(rng, max_start, long_chunks)
            what = (f"seed {seed} case {it}: Hq {pb.n_q_heads} Hkv {pb.n_kv_heads} D {pb.head_dim} C {pb.q_len} s {pb.q_start} "
                    f"W {pb.last_q} dca {dca} split {split} segment {seg} in_turn {turn} nv {nv} ns {ns} band {band}")
            print(what, flush=True)   # names the case if the run dies inside it
            c, hq, hkv, d, n_k = pb.q_len, pb.n_q_heads, pb.n_kv_heads, pb.head_dim, pb.n_k
            qs = [rand_bf16(rng, (c, hq, d)) for _ in range(3)]
            k = rand_bf16(rng, (n_k, hkv, d)); v = rand_bf16(rng, (n_k, hkv, d))
            sets = _rand_sets(rng, pb, nv, ns, force_cols=[0] if band else [], force_offs=range(min(band, n_k)))
            od = oracle.Dca(dca[0], dca[1], qs[1], qs[2]) if dca else None
            gd = (dev(qs[1]), dev(qs[2]), dca[0], dca[1]) if dca else None
            vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, split)
            vs.set_option(vs.VS_OPT_ATTN_SEGMENT_BLOCKS, seg)
            vs.set_option(vs.VS_OPT_ATTN_ROUNDS_IN_TURN, turn)
            ck = chunk_of(pb)
            ref_out, ref_lse = oracle.dense_attention(pb, qs[0], k, v, dca=od)
            out, lse = vs.dense_causal_prefill(ck, dev(qs[0]), dev(k), dev(v), want_lse=True, dca=gd)
            torch.cuda.synchronize()
            assert_attn_close(out, lse, ref_out, ref_lse, "dense, " + what)
            ref_out, ref_lse = oracle.sparse_attention(pb, qs[0], k, v, *sets, dca=od)
            out, lse = vs.sparse_attn_prefill(ck, dev(qs[0]), dev(k), dev(v), *[_t(x) for x in sets], want_lse=True, dca=gd)
            torch.cuda.synchronize()
            assert_attn_close(out, lse, ref_out, ref_lse, "sparse, " + what)
            rvs, rss, rlse = oracle.estimate(pb, qs[0], k, dca=od)
            vsc, ssc, lw = vs.estimate(ck, dev(qs[0]), dev(k), want_lse=True, dca=gd)
            torch.cuda.synchronize()
            np.testing.assert_allclose(f64(vsc), rvs, rtol=3e-4, atol=1e-7, err_msg=what)
            np.testing.assert_allclose(f64(ssc), rss, rtol=3e-4, atol=1e-7, err_msg=what)
            np.testing.assert_allclose(f64(lw), rlse, atol=3e-4, rtol=0, err_msg=what)
            # selection on the GPU's own fp32 scores: identical sets, ties included
            ref_sets = oracle.select(pb, f64(vsc), f64(ssc))
            got_sets = vs.select(ck, vsc, ssc)
            torch.cuda.synchronize()
            for r, gset in zip(ref_sets, got_sets):
                np.testing.assert_array_equal(gset.cpu().numpy(), r, err_msg=what)
    finally:
        vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, 0)
        vs.set_option(vs.VS_OPT_ATTN_SEGMENT_BLOCKS, 0)
        vs.set_option(vs.VS_OPT_ATTN_ROUNDS_IN_TURN, 0)
