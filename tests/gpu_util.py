"""Helpers of the GPU parity tests: host<->device conversion and the tolerance rules."""
import numpy as np
import torch

import oracle
import paper_2501_15383_amd as vs
from tolerances import ATOL, RTOL, check_class_mass, check_lse, check_rows, v_block_classes  # noqa: F401

# index sets must agree wherever the oracle's score differs from the k-th score by more than this (relative)
SCORE_BAND = 1e-4


def dev(u16):
    """numpy uint16 bf16 bit patterns -> bf16 tensor on the GPU."""
    return torch.from_numpy(np.ascontiguousarray(u16).view(np.int16)).view(torch.bfloat16).cuda()


def host_u16(t):
    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


def f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def chunk_of(pb: oracle.Problem) -> vs.Chunk:
    return vs.Chunk(pb.n_q_heads, pb.n_kv_heads, pb.head_dim, pb.q_len, pb.q_start, pb.softmax_scale,
                    last_q=pb.last_q, block=pb.block, vertical_budget=max(pb.vertical_budget, 1),
                    slash_budget=max(pb.slash_budget, 1), keep_first_cols=pb.keep_first_cols,
                    keep_local_band=pb.keep_local_band)


def assert_attn_close(out_gpu, lse_gpu, ref_out, ref_lse, what=""):
    """out_gpu: bf16 [C][Hq][D] tensor (rows/heads already subset to match), ref_out: [nh][nr][D] fp64.
    The element rule of the contract plus the row rules and the tight lse rule of tolerances.py."""
    check_rows(np.transpose(f64(out_gpu), (1, 0, 2)), ref_out, what)
    if lse_gpu is not None:
        check_lse(f64(lse_gpu), ref_lse, what)


def block_class_values(n_tokens, n_kv_heads, d):
    """V with out[i][d] = probability mass of the key blocks of class d (see tolerances.py), on the GPU."""
    return dev(v_block_classes(n_tokens, n_kv_heads, d))


def check_index_sets(score64, got_idx, got_cnt, budget, n_forced, what=""):
    """The rule for GPU index sets: exactly k members, ascending, forced present, everything
    clearly above the oracle's k-th score in, everything clearly below out."""
    n = score64.shape[0]
    k = min(budget, n)
    assert int(got_cnt) == k, f"{what}: count {int(got_cnt)} != {k}"
    idx = np.asarray(got_idx[:k], np.int64)
    assert np.all(np.diff(idx) > 0) and idx.min() >= 0 and idx.max() < n, f"{what}: not ascending / out of range"
    assert np.all(np.asarray(got_idx[k:]) == -1), f"{what}: tail not -1"
    f = min(n_forced, n, k)
    sel = np.zeros(n, bool); sel[idx] = True
    assert sel[:f].all(), f"{what}: forced entries missing"
    if k - f == 0 or k == n:
        return
    cand = score64[f:]
    tau = np.sort(cand)[::-1][k - f - 1]
    must_in = np.nonzero(cand > tau * (1 + SCORE_BAND))[0] + f
    must_out = np.nonzero(cand < tau * (1 - SCORE_BAND))[0] + f
    assert sel[must_in].all(), f"{what}: {np.count_nonzero(~sel[must_in])} clear winners missing"
    assert not sel[must_out].any(), f"{what}: {np.count_nonzero(sel[must_out])} clear losers selected"
