#!/usr/bin/env python3
"""Benchmark of the vertical-slash sparse prefill path on one MI355X.

A step = one 32,768-token query chunk through the whole hot path
(vs_estimate -> vs_select -> vs_sparse_attn_prefill) with the K/V cache already resident in
HBM; the default workload is the LAST chunk of a 1,048,576-token context at the Qwen2.5-7B
attention shape (28 query / 4 KV heads, head_dim 128), i.e. n_k = 1M keys visible.  The
dense-causal kernel is timed on the same chunk for the speedup, and the fp64 CPU oracle is
timed on a bounded sample of the same chunk.  One JSON line is printed.  Next to the timed
steps the default run also measures, once each (none of it inside the timed region): the
vertical (gathered-column) phase on its own, every chunk of the whole-layer prefill, the last
chunk at the Qwen2.5-14B shape, and several short requests in one launch against one call per
request; --no-extras leaves these out.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 7b_1m] [--chunk-index -1]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0


def _events(n):
    import torch
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


def cpu_baseline(w, pb_kwargs, Q, K, V, sets_host, target_s, dca=None):
    """Time the fp64 oracle on a bounded sample of this chunk and extrapolate to the chunk."""
    import numpy as np

    import oracle
    import vsgen
    pb = oracle.Problem(**pb_kwargs)
    qh, kh, vh = vsgen.as_u16(Q), vsgen.as_u16(K), vsgen.as_u16(V)
    cores = oracle.num_threads()
    od = None if dca is None else oracle.Dca(dca[2], dca[3], vsgen.as_u16(dca[0]), vsgen.as_u16(dca[1]))
    t0 = time.time()
    vs_, ss_, _ = oracle.estimate(pb, qh, kh, heads=[0], dca=od)
    t_est = time.time() - t0
    t0 = time.time()
    oracle.select_one(vs_[0], pb.vertical_budget, pb.keep_first_cols)
    oracle.select_one(ss_[0], pb.slash_budget, pb.keep_local_band)
    t_sel = time.time() - t0
    # attention rows: spread over the chunk, sized from a 2-row probe to fill the time budget
    rng = np.random.default_rng(7)
    t0 = time.time()
    oracle.sparse_attention(pb, qh, kh, vh, *sets_host, heads=[0], rows=[0, pb.q_len - 1], dca=od)
    t_probe = max(time.time() - t0, 1e-3)
    budget = max(target_s - t_est - t_sel - t_probe, 1.0)
    # two rows ran side by side, so one row costs about t_probe on one core
    n_rows = int(min(pb.q_len, cores * max(1, int(budget / t_probe))))
    rows = np.sort(rng.choice(pb.q_len, n_rows, replace=False))
    t0 = time.time()
    oracle.sparse_attention(pb, qh, kh, vh, *sets_host, heads=[0], rows=rows, dca=od)
    t_att = time.time() - t0
    hq = pb.n_q_heads
    chunk_s = hq * (t_est + t_sel) + t_att * (hq * pb.q_len) / n_rows
    return {
        "value": chunk_s * 1e3, "unit": "ms per 32K chunk (extrapolated from the sample)",
        "cores": cores, "kind": "oracle",
        "sample": (f"head 0 of {hq}: estimate ({t_est:.2f}s) + select ({t_sel:.2f}s) for the whole head, "
                   f"masked attention for {n_rows} of {pb.q_len} rows ({t_att:.2f}s); "
                   f"scaled by heads and rows to one chunk"),
        "sample_seconds": t_est + t_sel + t_probe + t_att,
    }


def kernel_source_hash():
    """sha256 of the attention kernel's sources: a counter figure stored under profiles/ is quoted
    only while it was measured on these very sources."""
    import hashlib
    h = hashlib.sha256()
    for f in ("paper_2501_15383_amd/csrc/vs_attn.hip", "paper_2501_15383_amd/csrc/vs_common.h"):
        h.update(open(os.path.join(ROOT, f), "rb").read())
    return h.hexdigest()[:16]


def gather_probe(vs, torch, ck, w, Q, K, V, sets, out, ws_a, dca, reps=3):
    """The vertical phase on its own: a sparse launch whose slash set is only the forced local band
    (offsets 0..63: two block diagonals per query block) with the chunk's real vertical set, so
    that nearly all of its time is spent gathering the selected key/value rows 64 at a time into
    LDS tiles.  Bytes = rows gathered (K and V) x 2 D bytes; a 128-row query tile gathers
    ceil(visible columns / 64) tiles of 64 rows."""
    v_idx, v_cnt, _, _ = sets
    dev = v_idx.device
    s_band = torch.full_like(sets[2], -1)
    nb = min(64, ck.slash_budget, ck.n_k)
    s_band[:, :nb] = torch.arange(nb, dtype=torch.int32, device=dev)
    s_cnt = torch.full_like(sets[3], nb)
    args = (v_idx, v_cnt, s_band, s_cnt)
    vs.sparse_attn_prefill(ck, Q, K, V, *args, out=out, ws=ws_a, dca=dca)
    e = _events(2)
    e[0].record()
    for _ in range(reps):
        vs.sparse_attn_prefill(ck, Q, K, V, *args, out=out, ws=ws_a, dca=dca)
    e[1].record()
    torch.cuda.synchronize()
    ms = e[0].elapsed_time(e[1]) / reps
    pad = ck.q_start % 64
    n_t = (ck.q_len + pad + 127) // 128
    last_pos = torch.clamp((torch.arange(n_t, device=dev) + 1) * 128 - pad - 1, max=ck.q_len - 1) + ck.q_start
    vi = torch.where(v_idx >= 0, v_idx, torch.full_like(v_idx, 2 ** 31 - 1)).long()
    vis = torch.searchsorted(vi, last_pos.expand(vi.shape[0], -1).contiguous(), right=True)   # [Hq][tiles]
    tiles = int(((vis + 63) // 64).sum())
    nbytes = tiles * 64 * w.head_dim * 2 * 2
    t = vs.count_tiles(ck, *args).cpu()
    return {"ms": ms, "gathered_tiles_of_64_rows": tiles, "gathered_bytes": nbytes, "gbs": nbytes / (ms * 1e-3) / 1e9,
            "issued_tiles": {"slash": int(t[:, 0].sum()), "vertical": int(t[:, 1].sum())},
            "what": "sparse launch with only the forced band (offsets 0..63) as slash set and the chunk's own vertical "
                    "set; bytes = K and V rows gathered into LDS (64 per vertical tile of a 128-row query tile); the "
                    "gathered rows come out of the L2 / HBM at this rate; HBM-side bytes of this launch by counters: "
                    "profiles/"}


def side_chunk(vs, torch, vsgen, dev, name, steps=3):
    """estimate -> select -> sparse attention and the dense kernel on the last chunk of another workload."""
    w = vsgen.WORKLOADS[name]
    s = (w.n_chunks - 1) * w.chunk
    C, n_k = w.chunk, w.n_ctx
    K, V = vsgen.make_kv(w, n_k, device=dev)
    Q = vsgen.make_q(w, s, n_k, device=dev)
    ck = vs.Chunk(w.n_q_heads, w.n_kv_heads, w.head_dim, C, s, w.softmax_scale, last_q=w.last_q,
                  vertical_budget=w.vertical_budget, slash_budget=w.slash_budget,
                  keep_first_cols=w.keep_first_cols, keep_local_band=w.keep_local_band)
    out = torch.empty((C, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device=dev)
    vscore = torch.empty((w.n_q_heads, n_k), dtype=torch.float32, device=dev)
    sscore = torch.empty_like(vscore)
    sets = vs.alloc_index_sets(ck, dev)
    ws_e = torch.empty(max(vs.workspace_bytes(ck, vs.VS_WS_ESTIMATE), 256), dtype=torch.uint8, device=dev)
    ws_a = torch.empty(max(vs.workspace_bytes(ck, vs.VS_WS_SPARSE), vs.workspace_bytes(ck, vs.VS_WS_DENSE), 256),
                       dtype=torch.uint8, device=dev)

    def step(ev=None):
        if ev: ev[0].record()
        vs.estimate(ck, Q, K, vscore=vscore, sscore=sscore, ws=ws_e)
        if ev: ev[1].record()
        vs.select(ck, vscore, sscore, sets=sets)
        if ev: ev[2].record()
        vs.sparse_attn_prefill(ck, Q, K, V, *sets, out=out, ws=ws_a)
        if ev: ev[3].record()
    step()
    torch.cuda.synchronize()
    evs = [_events(4) for _ in range(steps)]
    for e in evs:
        step(e)
    torch.cuda.synchronize()
    ph = [sum(e[i].elapsed_time(e[i + 1]) for e in evs) / steps for i in range(3)]
    tiles = vs.count_tiles(ck, *sets).cpu()
    issued = int(tiles.sum())
    dense_tiles = w.n_q_heads * sum(s // 64 + qb + 1 for qb in range((C + 63) // 64))
    tile_flops = 4.0 * w.head_dim * 64 * 64
    vs.dense_causal_prefill(ck, Q, K, V, out=out, ws=ws_a)
    e = _events(2)
    e[0].record()
    vs.dense_causal_prefill(ck, Q, K, V, out=out, ws=ws_a)
    e[1].record()
    torch.cuda.synchronize()
    dense_ms = e[0].elapsed_time(e[1])
    return {"workload": f"{w.name}: last chunk (q_start {s}, {C} rows, n_k {n_k}), Hq {w.n_q_heads} / Hkv {w.n_kv_heads} / "
                        f"D {w.head_dim}, Bv {w.vertical_budget}, Bs {w.slash_budget}",
            "ms": sum(ph), "phases_ms": {"estimate": ph[0], "select": ph[1], "sparse_attention": ph[2]},
            "computed_fraction": issued / dense_tiles, "effective_tflops": issued * tile_flops / (ph[2] * 1e-3) / 1e12,
            "dense_ms": dense_ms, "dense_tflops": dense_tiles * tile_flops / (dense_ms * 1e-3) / 1e12,
            "speedup_vs_dense": dense_ms / sum(ph)}


def batch_rows(vs, torch, vsgen, dev, n_keys=262144, n_req=8):
    """Several short requests in one launch (vs_attn_batch) against one call per request, 7B shape,
    every request with its own K/V cache of n_keys keys.  Rows: single-token dense decode steps;
    single-token sparse steps; a mix of 1-, 17- and 64-row chunks, dense and sparse."""
    w = vsgen.scaled(vsgen.WORKLOADS["7b_1m"], n_ctx=n_keys)
    K0, V0 = vsgen.make_kv(w, n_keys, device=dev)
    caches = [(K0, V0)] + [(K0.clone(), V0.clone()) for _ in range(n_req - 1)]
    hq, hkv, d = w.n_q_heads, w.n_kv_heads, w.head_dim
    bv, bs = w.vertical_budget, w.slash_budget

    def make(lens, sparse_flags):
        reqs = []
        for i, (c, sp) in enumerate(zip(lens, sparse_flags)):
            s = n_keys - c
            K, V = caches[i]
            Q = vsgen.make_q(w, s, n_keys, device=dev)
            ck = vs.Chunk(hq, hkv, d, c, s, w.softmax_scale, last_q=w.last_q, vertical_budget=bv, slash_budget=bs)
            sets = None
            if sp:
                vsc, ssc, _ = vs.estimate(ck, Q, K)
                sets = vs.select(ck, vsc, ssc)
            reqs.append(dict(q=Q, k=K, v=V, out=torch.empty_like(Q), q_start=s, sets=sets, ck=ck))
        return reqs

    def timed(fn, reps=5):
        fn()
        e = _events(2)
        e[0].record()
        for _ in range(reps):
            fn()
        e[1].record()
        torch.cuda.synchronize()
        return e[0].elapsed_time(e[1]) / reps

    rows = []
    for name, lens, flags in (("decode_dense", [1] * n_req, [False] * n_req),
                              ("decode_sparse", [1] * n_req, [True] * n_req),
                              ("mixed_short_chunks", [1, 17, 64, 1, 17, 64, 33, 64][:n_req],
                               [False, True, False, True, False, True, False, True][:n_req])):
        reqs = make(lens, flags)
        mx = max(lens)
        ckb = vs.Chunk(hq, hkv, d, mx, n_keys - mx, w.softmax_scale, vertical_budget=bv, slash_budget=bs)
        table = vs.request_table(reqs, dev)
        ws = vs.attn_batch(ckb, table, len(reqs), reqs[0]["q"], reqs[0]["k"], reqs[0]["v"], reqs[0]["out"])
        t_batch = timed(lambda: vs.attn_batch(ckb, table, len(reqs), reqs[0]["q"], reqs[0]["k"], reqs[0]["v"],
                                              reqs[0]["out"], ws=ws))
        wss = [torch.empty(max(vs.workspace_bytes(r["ck"], vs.VS_WS_SPARSE), vs.workspace_bytes(r["ck"], vs.VS_WS_DENSE), 256),
                           dtype=torch.uint8, device=dev) for r in reqs]

        def one_by_one():
            for r, wsr in zip(reqs, wss):
                if r["sets"] is None:
                    vs.dense_causal_prefill(r["ck"], r["q"], r["k"], r["v"], out=r["out"], ws=wsr)
                else:
                    vs.sparse_attn_prefill(r["ck"], r["q"], r["k"], r["v"], *r["sets"], out=r["out"], ws=wsr)
        t_loop = timed(one_by_one)
        kv_bytes = sum(2 * n_keys * hkv * d * 2 for r in reqs if r["sets"] is None)
        rows.append({"case": name, "requests": len(reqs), "rows_per_request": lens[:len(reqs)], "keys_per_request": n_keys,
                     "batch_ms": t_batch, "one_call_per_request_ms": t_loop, "per_request_ms_batched": t_batch / len(reqs),
                     "per_request_ms_single_calls": t_loop / len(reqs), "speedup": t_loop / t_batch,
                     "dense_kv_gbs_batched": (kv_bytes / (t_batch * 1e-3) / 1e9) if name == "decode_dense" else None})
        del reqs, table, ws, wss
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="7b_1m")
    ap.add_argument("--chunk-index", type=int, default=-1, help="which chunk of the context (-1 = last)")
    ap.add_argument("--n-ctx", type=int, default=0, help="override the context length (tokens)")
    ap.add_argument("--segment-blocks", type=int, default=0,
                    help="64-key blocks per key segment of the sparse launch (0 = the library's choice)")
    ap.add_argument("--local-mag", type=float, default=-1.0,
                    help="override the strength of the planted slash structure of the workload (vsgen local_mag)")
    ap.add_argument("--chunk-rows", type=int, default=0,
                    help="rows of the chunk (a multiple of 64) instead of the workload's 32768: short chunks at the end "
                         "of a long context, the decode-side use of the kernels")
    ap.add_argument("--rounds-in-turn", type=int, default=0, help="VS_OPT_ATTN_ROUNDS_IN_TURN (1: no load balancing)")
    ap.add_argument("--key-split", type=int, default=0, help="VS_OPT_ATTN_KEY_SPLIT: 0 automatic, 1 never, n ranges")
    ap.add_argument("--layer-plan", choices=["equal", "dense", "sparse"], default="equal",
                    help="chunk boundaries of --layer: equal lengths, or vs_plan_chunks with that cost model")
    ap.add_argument("--layer", action="store_true",
                    help="also time every chunk of the context once (whole-layer prefill); needs the last chunk")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the timed chunk: no gather probe, no whole-layer prefill, no 14B chunk, no batched requests")
    ap.add_argument("--gather-probe", action="store_true", help="run the gather probe even with --no-extras")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--kv-head-major", action="store_true",
                    help="allocate the K and V caches as [Hkv][n_k][D] (each KV head contiguous) instead of [n_k][Hkv][D]")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=20.0)
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one 1 GiB device copy (the reference kernel that scales rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path shards by KV head with no exchange inside "
              "attention; multi-GPU figures are not produced). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2501_15383_amd as vs
    vs.set_option(vs.VS_OPT_ATTN_SEGMENT_BLOCKS, args.segment_blocks)
    import vsgen
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    vs.lib()   # fail loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    w = vsgen.WORKLOADS[args.workload]
    if args.n_ctx:
        w = vsgen.scaled(w, n_ctx=args.n_ctx)
    if args.local_mag >= 0:
        w = vsgen.scaled(w, local_mag=args.local_mag)
    if args.chunk_rows:
        w = vsgen.scaled(w, chunk=args.chunk_rows)
    vs.set_option(vs.VS_OPT_ATTN_KEY_SPLIT, args.key_split)
    vs.set_option(vs.VS_OPT_ATTN_ROUNDS_IN_TURN, args.rounds_in_turn)
    ci = args.chunk_index % w.n_chunks
    s = ci * w.chunk
    C = min(w.chunk, w.n_ctx - s)
    n_k = s + C

    t0 = time.time()
    K, V = vsgen.make_kv(w, n_k, device=dev)
    if args.kv_head_major:   # same values, another placement: the calls take the strides from the tensors
        K, V = (t.permute(1, 0, 2).contiguous().permute(1, 0, 2) for t in (K, V))
    dca = sel = None   # Dual Chunk Attention workloads: (q_succ, q_inter, chunk, window) next to the intra-chunk Q,
    if w.dca_chunk > 0:  # for the attention and (continuous relative positions) for the selection
        Q, q_succ, q_inter = vsgen.make_q_dca(w, s, s + C, device=dev)
        dca = (q_succ, q_inter, w.dca_chunk, w.dca_window)
        sel = vsgen.make_q_dca_select(w, s, s + C, device=dev)
    else:
        Q = vsgen.make_q(w, s, s + C, device=dev)
    torch.cuda.synchronize()
    t_gen = time.time() - t0

    bv = w.vertical_budget if not w.dense else 1
    bs = w.slash_budget if not w.dense else 1
    ck = vs.Chunk(w.n_q_heads, w.n_kv_heads, w.head_dim, C, s, w.softmax_scale, last_q=w.last_q,
                  vertical_budget=bv, slash_budget=bs, keep_first_cols=w.keep_first_cols,
                  keep_local_band=w.keep_local_band)
    out = torch.empty((C, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device=dev)
    vscore = torch.empty((w.n_q_heads, n_k), dtype=torch.float32, device=dev)
    sscore = torch.empty_like(vscore)
    sets = vs.alloc_index_sets(ck, dev)
    ws_e = torch.empty(max(vs.workspace_bytes(ck, vs.VS_WS_ESTIMATE), 256), dtype=torch.uint8, device=dev)
    ws_a = torch.empty(max(vs.workspace_bytes(ck, vs.VS_WS_SPARSE), 256), dtype=torch.uint8, device=dev)

    def step(ev=None):
        # the three stages of vs_prefill_chunk, called one by one on the same stream so that
        # HIP events between them give the per-kernel times
        if ev: ev[0].record()
        if w.dense:
            vs.dense_causal_prefill(ck, Q, K, V, out=out, ws=ws_a, dca=dca)
            if ev: ev[1].record(); ev[2].record(); ev[3].record()
            return
        vs.estimate(ck, Q, K, vscore=vscore, sscore=sscore, ws=ws_e, dca=sel)
        if ev: ev[1].record()
        vs.select(ck, vscore, sscore, sets=sets)
        if ev: ev[2].record()
        vs.sparse_attn_prefill(ck, Q, K, V, *sets, out=out, ws=ws_a, dca=dca)
        if ev: ev[3].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [_events(4) for _ in range(args.steps)]
    t0 = time.time()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    wall_ms = (time.time() - t0) * 1e3 / args.steps
    est_ms = sum(e[0].elapsed_time(e[1]) for e in evs) / args.steps
    sel_ms = sum(e[1].elapsed_time(e[2]) for e in evs) / args.steps
    att_ms = sum(e[2].elapsed_time(e[3]) for e in evs) / args.steps
    if w.dense:
        att_ms, est_ms, sel_ms = est_ms, 0.0, 0.0
    gpu_ms = est_ms + sel_ms + att_ms

    # ---- work accounting: issued 64x64 tiles -> FLOPs ---------------------------------------
    tile_flops = 4.0 * w.head_dim * 64 * 64
    n_qb = (C + 63) // 64
    mb0 = s // 64
    dense_tiles = w.n_q_heads * sum(mb0 + qb + 1 for qb in range(n_qb))
    if w.dense:
        issued = dense_tiles
        slash_tiles = vert_tiles = 0
    else:
        tiles = vs.count_tiles(ck, *sets).cpu()
        slash_tiles, vert_tiles = int(tiles[:, 0].sum()), int(tiles[:, 1].sum())
        issued = slash_tiles + vert_tiles
    att_tflops = issued * tile_flops / (att_ms * 1e-3) / 1e12

    # ---- dense-causal kernel on the same chunk ----------------------------------------------
    dense_ms = None
    if not args.no_dense and not w.dense:
        ws_d = torch.empty(max(vs.workspace_bytes(ck, vs.VS_WS_DENSE), 256), dtype=torch.uint8, device=dev)
        out_d = torch.empty_like(out)
        vs.dense_causal_prefill(ck, Q, K, V, out=out_d, ws=ws_d, dca=dca)
        torch.cuda.synchronize()
        e = _events(2)
        e[0].record()
        for _ in range(2):
            vs.dense_causal_prefill(ck, Q, K, V, out=out_d, ws=ws_d, dca=dca)
        e[1].record()
        torch.cuda.synchronize()
        dense_ms = e[0].elapsed_time(e[1]) / 2
        del out_d

    if args.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- optional: every chunk of the context once (whole-layer prefill of one attention layer) --
    layer = None
    extras = not args.no_extras and not w.dense and not args.chunk_rows and not args.n_ctx and ci == w.n_chunks - 1
    if (args.layer or extras) and not w.dense and ci == w.n_chunks - 1:
        per_chunk = []
        if args.layer_plan == "equal":
            bounds = [min(i * w.chunk, w.n_ctx) for i in range(w.n_chunks + 1)]
        else:
            bounds = vs.plan_chunks(w.n_ctx, w.n_chunks, vs.VS_COST_DENSE if args.layer_plan == "dense" else vs.VS_COST_SPARSE,
                                    bv, bs)
        out_l = torch.empty((max(b - a for a, b in zip(bounds, bounds[1:])), w.n_q_heads, w.head_dim),
                            dtype=torch.bfloat16, device=dev) if args.layer_plan != "equal" else out
        ws_e_l, ws_a_l = ws_e, ws_a
        if args.layer_plan != "equal":   # chunks longer than the equal ones need larger workspaces
            cks = [vs.Chunk(w.n_q_heads, w.n_kv_heads, w.head_dim, b - a, a, w.softmax_scale, last_q=w.last_q,
                            vertical_budget=bv, slash_budget=bs) for a, b in zip(bounds, bounds[1:])]
            ws_e_l = torch.empty(max(vs.workspace_bytes(c, vs.VS_WS_ESTIMATE) for c in cks), dtype=torch.uint8, device=dev)
            ws_a_l = torch.empty(max(vs.workspace_bytes(c, vs.VS_WS_SPARSE) for c in cks), dtype=torch.uint8, device=dev)
        for i in range(w.n_chunks):
            si, Ci = bounds[i], bounds[i + 1] - bounds[i]
            cki = vs.Chunk(w.n_q_heads, w.n_kv_heads, w.head_dim, Ci, si, w.softmax_scale, last_q=w.last_q,
                           vertical_budget=bv, slash_budget=bs, keep_first_cols=w.keep_first_cols,
                           keep_local_band=w.keep_local_band)
            dca_i = sel_i = None
            if w.dca_chunk > 0:
                Qi, qs_i, qi_i = vsgen.make_q_dca(w, si, si + Ci, device=dev)
                dca_i = (qs_i, qi_i, w.dca_chunk, w.dca_window)
                sel_i = vsgen.make_q_dca_select(w, si, si + Ci, device=dev)
            else:
                Qi = vsgen.make_q(w, si, si + Ci, device=dev)
            nki = si + Ci
            vsc_i, ssc_i = vscore[:, :nki].contiguous(), sscore[:, :nki].contiguous()
            oi = out_l[:Ci]
            e = _events(4)
            torch.cuda.synchronize()
            e[0].record()
            vs.estimate(cki, Qi, K, vscore=vsc_i, sscore=ssc_i, ws=ws_e_l, dca=sel_i)
            vs.select(cki, vsc_i, ssc_i, sets=sets)
            e[1].record()
            vs.sparse_attn_prefill(cki, Qi, K, V, *sets, out=oi, ws=ws_a_l, dca=dca_i)
            e[2].record()
            if not args.no_dense:
                vs.dense_causal_prefill(cki, Qi, K, V, out=oi, ws=ws_a_l, dca=dca_i)
            e[3].record()
            torch.cuda.synchronize()
            tl = vs.count_tiles(cki, *sets).sum().item()
            dt = w.n_q_heads * sum(si // 64 + qb + 1 for qb in range((Ci + 63) // 64))
            per_chunk.append({"chunk": i, "q_start": si, "q_len": Ci, "sparse_ms": e[0].elapsed_time(e[2]), "estimate_select_ms": e[0].elapsed_time(e[1]),
                              "dense_ms": None if args.no_dense else e[2].elapsed_time(e[3]),
                              "computed_fraction": tl / dt})
            del Qi, vsc_i, ssc_i
        tot_s = sum(c["sparse_ms"] for c in per_chunk)
        tot_d = None if args.no_dense else sum(c["dense_ms"] for c in per_chunk)
        layer = {"chunks": w.n_chunks, "plan": args.layer_plan, "sparse_ms_total": tot_s, "dense_ms_total": tot_d,
                 "speedup": (tot_d / tot_s) if tot_d else None, "per_chunk": per_chunk}

    # counter figures measured earlier on these very kernel sources (bench_counters.py writes the file)
    traffic = gather_hbm = None
    tpath = os.path.join(ROOT, "profiles", f"traffic_k_attention_{w.name}.json")
    if os.path.exists(tpath):
        tj = json.load(open(tpath))
        if tj.get("kernel_source_sha") == kernel_source_hash():
            traffic = tj.get("hbm_bytes_per_launch")
            gather_hbm = tj.get("gather_probe")

    gather = None
    if (extras or args.gather_probe) and not w.dense:
        gather = gather_probe(vs, torch, ck, w, Q, K, V, sets, out, ws_a, dca)
        if gather_hbm:
            gather["hbm_bytes_by_counters"] = gather_hbm.get("hbm_bytes")
            gather["hbm_gbs_by_counters"] = gather_hbm.get("hbm_bytes") / (gather["ms"] * 1e-3) / 1e9

    est = None
    if not w.dense:
        k_bytes = n_k * w.n_kv_heads * w.head_dim * 2
        sc_bytes = w.n_q_heads * n_k * 4
        algorithmic = k_bytes + 2 * sc_bytes + min(w.last_q, C) * w.n_q_heads * w.head_dim * 2
        moved = 2 * k_bytes + 2 * sc_bytes + 2 * sc_bytes   # two sweeps over K; vscore written; sscore zero-filled, then written
        est = {"ms": est_ms, "algorithmic_bytes": algorithmic, "moved_bytes": moved,
               "gbs_on_algorithmic_bytes": algorithmic / (est_ms * 1e-3) / 1e9,
               "gbs_on_moved_bytes": moved / (est_ms * 1e-3) / 1e9, "moved_over_one_pass_minimum": moved / algorithmic,
               "frac_of_hbm_peak_on_algorithmic_bytes": algorithmic / (est_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
               "what": "moved = K twice (two sweeps) + vscore written + sscore zero-filled and written; the counter "
                       "figures of the two sweeps are in profiles/"}

    second = None
    if extras and args.workload == "7b_1m":
        # the second shape (configuration 4): last chunk at the Qwen2.5-14B shape, measured once
        second = side_chunk(vs, torch, vsgen, dev, "14b_1m")

    batch = None
    if extras:
        batch = batch_rows(vs, torch, vsgen, dev)

    cpu = None
    if not args.no_cpu:
        pbk = dict(n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, q_len=C, q_start=s,
                   softmax_scale=w.softmax_scale, last_q=w.last_q, vertical_budget=bv, slash_budget=bs,
                   keep_first_cols=w.keep_first_cols, keep_local_band=w.keep_local_band)
        if w.dense:
            import numpy as np
            allv = np.zeros((w.n_q_heads, 1), np.int32)
            sets_h = (allv, np.ones(w.n_q_heads, np.int32), allv.copy(), np.ones(w.n_q_heads, np.int32))
        else:
            sets_h = tuple(x.cpu().numpy() for x in sets)
        cpu = cpu_baseline(w, pbk, Q, K, V, sets_h, args.cpu_seconds, dca=dca)

    res = {
        "metric": ("ms per 32K prefill chunk at 1M ctx (estimate + select + block-sparse attention)" if not args.chunk_rows
                   and not args.n_ctx else f"ms per {C}-row chunk at {n_k} keys (estimate + select + block-sparse attention)"),
        "value": gpu_ms, "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": gpu_ms, "wall_ms_per_step": wall_ms, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: chunk {ci} of {w.n_chunks} (q_start {s}, {C} rows, n_k {n_k}), "
                               f"Hq {w.n_q_heads} / Hkv {w.n_kv_heads} / D {w.head_dim}, W {w.last_q}, "
                               f"Bv {bv}, Bs {bs}", "input_gen_s": round(t_gen, 2)},
        "phases_ms": {"estimate": est_ms, "select": sel_ms, "sparse_attention": att_ms},
        "tiles": {"slash": slash_tiles, "vertical": vert_tiles, "dense_equivalent": dense_tiles,
                  "computed_fraction": issued / dense_tiles},
        "effective_tflops": att_tflops, "pct_bf16_mfma_peak": 100.0 * att_tflops / PEAK_BF16_TFLOPS,
        "dense_ms": dense_ms,
        "dense_tflops": (dense_tiles * tile_flops / (dense_ms * 1e-3) / 1e12) if dense_ms else None,
        "speedup_vs_dense": (dense_ms / gpu_ms) if dense_ms else None,
        "roofline": {"kernel": "k_attention", "bound": "mfma", "achieved": att_tflops, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": att_tflops / PEAK_BF16_TFLOPS, "traffic": traffic,
                     "flops_per_launch": issued * tile_flops, "avg_launch_ms": att_ms},
        "estimate_hbm": est,
        "gather_phase": gather,
        "cpu_baseline": cpu,
    }
    if layer:
        res["layer_prefill"] = layer
    if second:
        res["second_shape"] = second
    if batch:
        res["batched_requests"] = batch
    print(json.dumps(res))


if __name__ == "__main__":
    main()
