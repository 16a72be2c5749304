"""Host logic of the chunk planner (section 5.3.2: chunk sizes follow the complexity of the attention
kernel so that every chunk takes about the same time) and its cost model."""
import math

import pytest

import paper_2501_15383_amd as vs


def _dense_brute(q_start, q_len):
    return sum(q_start // 64 + qb + 1 for qb in range((q_len + 63) // 64))


@pytest.mark.parametrize("s,c", [(0, 64), (0, 100), (1024, 1024), (65536, 32768), (64, 1)])
def test_dense_cost_is_the_causal_tile_count(s, c):
    assert vs.chunk_cost(s, c, vs.VS_COST_DENSE) == _dense_brute(s, c)


def test_sparse_cost_written_out():
    s, c, bv, bs = 4096, 2048, 100, 50
    nb = (s + c) // 64
    density = 1 - (1 - 2 / nb) ** bs
    want = _dense_brute(s, c) * density + (c // 64) * math.ceil(bv / 64)
    assert vs.chunk_cost(s, c, vs.VS_COST_SPARSE, bv, bs) == pytest.approx(want, rel=1e-12)
    # budgets beyond the context: every diagonal expected, every key a column
    assert vs.chunk_cost(0, 128, vs.VS_COST_SPARSE, 10**6, 10**6) == pytest.approx(3 + 2 * 2, rel=1e-12)


def test_cost_model_rejects_bad_arguments():
    assert vs.chunk_cost(10, 64, vs.VS_COST_DENSE) < 0          # q_start not on a block edge
    assert vs.chunk_cost(0, 0, vs.VS_COST_DENSE) < 0
    assert vs.chunk_cost(0, 64, 7) < 0
    assert vs.chunk_cost(0, 64, vs.VS_COST_SPARSE, 0, 5) < 0
    with pytest.raises(vs.VsError):
        vs.plan_chunks(1000, 0, vs.VS_COST_DENSE)
    with pytest.raises(vs.VsError):
        vs.plan_chunks(64 * 3, 4, vs.VS_COST_DENSE)


@pytest.mark.parametrize("n_ctx,k", [(1048576, 32), (131072, 4), (100000, 7)])
def test_dense_plan_follows_the_square_root_law(n_ctx, k):
    b = vs.plan_chunks(n_ctx, k, vs.VS_COST_DENSE)
    assert b[0] == 0 and b[-1] == n_ctx and all(y > x for x, y in zip(b, b[1:]))
    assert all(x % 64 == 0 for x in b[:-1])
    # the cost of the first t tokens grows like t^2, so equal-cost cuts sit at n sqrt(c / k)
    for c in range(1, k):
        assert abs(b[c] - n_ctx * math.sqrt(c / k)) <= 128


def test_plan_with_one_block_per_chunk_has_no_choice():
    assert vs.plan_chunks(64 * 9, 9, vs.VS_COST_DENSE) == [64 * i for i in range(10)]
    assert vs.plan_chunks(64 * 9, 9, vs.VS_COST_SPARSE, 3, 3) == [64 * i for i in range(10)]


@pytest.mark.parametrize("model,bv,bs", [(vs.VS_COST_DENSE, 1, 1), (vs.VS_COST_SPARSE, 1000, 6096), (vs.VS_COST_SPARSE, 64, 200)])
def test_planned_chunks_cost_about_the_same(model, bv, bs):
    n_ctx, k = 1048576, 32
    b = vs.plan_chunks(n_ctx, k, model, bv, bs)
    cost = [vs.chunk_cost(b[i], b[i + 1] - b[i], model, bv, bs) for i in range(k)]
    equal = [vs.chunk_cost(i * n_ctx // k, n_ctx // k, model, bv, bs) for i in range(k)]
    # one 64-token step at the end of the context changes a chunk by about this much
    step = vs.chunk_cost(n_ctx - 64, 64, model, bv, bs)
    assert max(cost) - min(cost) <= 4 * step
    assert max(cost) - min(cost) < 0.05 * (max(equal) - min(equal))
