"""GPU parity of vs_attn_batch (several requests per launch: decode steps and short chunks of
different requests against caches of different lengths, dense and sparse mixed; section 5.2,
"Integrating with Chunked prefill") against the fp64 oracle.  The oracle side is a plain loop
over the requests."""
import numpy as np
import pytest
import torch

import oracle
import paper_2501_15383_amd as vs
from gpu_util import assert_attn_close, chunk_of, dev
from helpers import rand_bf16
from test_gpu_attention import _rand_sets, _t

pytestmark = pytest.mark.gpu


def _make_requests(rng, hq, hkv, d, specs, bv, bs):
    """specs: (q_len, q_start, sparse).  Every request gets its own Q and its own K/V cache."""
    reqs = []
    for c, s, sparse in specs:
        n_k = s + c
        q = rand_bf16(rng, (c, hq, d)); k = rand_bf16(rng, (n_k, hkv, d)); v = rand_bf16(rng, (n_k, hkv, d))
        pb = oracle.Problem(hq, hkv, d, c, s, 1.0 / np.sqrt(d), vertical_budget=bv, slash_budget=bs)
        sets = None
        if sparse:
            sets = _rand_sets(rng, pb, min(bv - 1, max(n_k // 6, 1)), min(bs - 64, max(n_k // 200, 1)),
                              force_cols=[0], force_offs=range(min(64, n_k)))
        reqs.append(dict(pb=pb, q=q, k=k, v=v, sets=sets))
    return reqs


def _run_batch(reqs, hq, hkv, d, bv, bs, poison=None):
    gpu = []
    for r in reqs:
        pb = r["pb"]
        out = torch.full((pb.q_len, hq, d), -3.0, dtype=torch.bfloat16, device="cuda")
        lse = torch.full((hq, pb.q_len), 7.0, dtype=torch.float32, device="cuda")
        gpu.append(dict(q=dev(r["q"]), k=dev(r["k"]), v=dev(r["v"]), out=out, lse=lse, q_start=pb.q_start,
                        sets=None if r["sets"] is None else tuple(_t(x) for x in r["sets"])))
    max_len = max(r["pb"].q_len for r in reqs)
    max_nk = max(r["pb"].n_k for r in reqs)
    ck = vs.Chunk(hq, hkv, d, max_len, max_nk - max_len, 1.0 / np.sqrt(d), vertical_budget=bv, slash_budget=bs)
    table = vs.request_table(gpu, "cuda")
    if poison is not None:
        poison(table)
    vs.attn_batch(ck, table, len(gpu), gpu[0]["q"], gpu[0]["k"], gpu[0]["v"], gpu[0]["out"])
    torch.cuda.synchronize()
    return gpu


def _check(reqs, gpu, skip=()):
    for i, (r, g) in enumerate(zip(reqs, gpu)):
        if i in skip:
            continue
        pb = r["pb"]
        if r["sets"] is None:
            ref_out, ref_lse = oracle.dense_attention(pb, r["q"], r["k"], r["v"])
        else:
            ref_out, ref_lse = oracle.sparse_attention(pb, r["q"], r["k"], r["v"], *r["sets"])
        assert_attn_close(g["out"], g["lse"], ref_out, ref_lse,
                          f"request {i}: {'sparse' if r['sets'] is not None else 'dense'} C={pb.q_len} s={pb.q_start}")


@pytest.mark.parametrize("hq,hkv,d", [(7, 1, 128), (4, 2, 64)])
def test_mixed_requests_match_the_oracle_loop(hq, hkv, d):
    rng = np.random.default_rng(1500 + d)
    bv, bs = 160, 112
    specs = [(1, 2999, False), (1, 1777, True), (17, 2048, False), (17, 3055, True), (64, 4032, False),
             (64, 1984, True), (1, 0, False), (130, 1211, True), (33, 95, False), (1, 4160, True), (3, 640, True)]
    reqs = _make_requests(rng, hq, hkv, d, specs, bv, bs)
    gpu = _run_batch(reqs, hq, hkv, d, bv, bs)
    _check(reqs, gpu)


def test_batch_of_decode_steps_only():
    # every request one token (dense requests pack the heads of a KV group into one tile, sparse ones cannot)
    hq, hkv, d, bv, bs = 8, 2, 128, 96, 100
    rng = np.random.default_rng(1600)
    specs = [(1, int(s), bool(i % 2)) for i, s in enumerate(rng.integers(0, 9000, 12))]
    reqs = _make_requests(rng, hq, hkv, d, specs, bv, bs)
    gpu = _run_batch(reqs, hq, hkv, d, bv, bs)
    _check(reqs, gpu)


def test_batch_equals_one_call_per_request_and_repeats_exactly():
    hq, hkv, d, bv, bs = 4, 1, 128, 64, 90
    rng = np.random.default_rng(1700)
    specs = [(64, 8128, True), (64, 8128, False), (20, 5000, True), (1, 9000, False)]
    reqs = _make_requests(rng, hq, hkv, d, specs, bv, bs)
    a = _run_batch(reqs, hq, hkv, d, bv, bs)
    b = _run_batch(reqs, hq, hkv, d, bv, bs)
    for x, y in zip(a, b):
        assert torch.equal(x["out"].view(torch.int16), y["out"].view(torch.int16)) and torch.equal(x["lse"], y["lse"])
    for r, g in zip(reqs, a):
        ck = chunk_of(r["pb"])
        if r["sets"] is None:
            o, l = vs.dense_causal_prefill(ck, g["q"], g["k"], g["v"], want_lse=True)
        else:
            o, l = vs.sparse_attn_prefill(ck, g["q"], g["k"], g["v"], *g["sets"], want_lse=True)
        torch.cuda.synchronize()
        # the two calls may cut the key walk differently: equal up to the rounding of the fp32 partial sums
        assert (o.float() - g["out"].float()).abs().max().item() <= 2e-2
        assert (l - g["lse"]).abs().max().item() < 1e-4


def test_requests_outside_the_stated_bounds_are_skipped():
    hq, hkv, d, bv, bs = 4, 1, 64, 64, 90
    rng = np.random.default_rng(1800)
    specs = [(16, 512, False), (16, 300, True), (16, 100, False)]
    reqs = _make_requests(rng, hq, hkv, d, specs, bv, bs)

    def poison(table):
        table[1, 10] = 17          # q_len beyond the stated maximum of 16
        table[2, 0] = 0            # null q
    gpu = _run_batch(reqs, hq, hkv, d, bv, bs, poison=poison)
    _check(reqs, gpu, skip=(1, 2))
    for i in (1, 2):
        assert (gpu[i]["out"].float() == -3.0).all() and (gpu[i]["lse"] == 7.0).all(), "a skipped request was written"
