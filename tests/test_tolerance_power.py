"""What the comparison rules of the GPU parity tests reject (tests/tolerances.py).

Mistakes are planted in oracle results on the CPU -- a zeroed output, a half-scaled one, a
dropped 64-key tile, a swapped pair of value tiles -- at a context long enough (131,072 keys,
diffuse softmax) that the element rule of the contract, 2e-2 + 1e-2 |ref|, accepts them all;
the row rules, the lse rule and the block-class values must not."""
import numpy as np
import pytest

import oracle
from helpers import rand_bf16
from tolerances import ATOL, RTOL, check_class_mass, check_lse, check_rows, v_block_classes

N_K, D = 131072, 128
ROWS = [N_K - 1 - 64 * 5, N_K - 1]


@pytest.fixture(scope="module")
def case():
    rng = np.random.default_rng(77)
    q = rand_bf16(rng, (N_K, 1, D)); k = rand_bf16(rng, (N_K, 1, D)); v = rand_bf16(rng, (N_K, 1, D))
    pb = oracle.Problem(1, 1, D, N_K, 0, 1.0 / np.sqrt(D))
    out, lse = oracle.dense_attention(pb, q, k, v, rows=ROWS)
    return pb, q, k, v, out, lse


def _all_but_one_diagonal(pb, skip):
    """Index sets that select every block diagonal except `skip` (and no extra column)."""
    offs = np.array([o for o in range(pb.n_k) if o // 64 != skip and not (o % 64 and o // 64 + 1 == skip)], np.int32)
    pbs = oracle.Problem(pb.n_q_heads, pb.n_kv_heads, pb.head_dim, pb.q_len, pb.q_start, pb.softmax_scale,
                         vertical_budget=1, slash_budget=pb.n_k, keep_first_cols=0, keep_local_band=0)
    s_idx = np.full((1, pb.n_k), -1, np.int32); s_idx[0, :len(offs)] = offs
    # the one column is key 0, which lies on a selected diagonal of both sampled rows (counted once)
    return pbs, (np.zeros((1, 1), np.int32), np.ones(1, np.int32), s_idx, np.array([len(offs)], np.int32))


def test_element_rule_alone_accepts_wrong_outputs_at_long_context(case):
    _, _, _, _, out, _ = case
    for wrong in (np.zeros_like(out), 0.5 * out):
        assert (np.abs(wrong - out) <= ATOL + RTOL * np.abs(out)).all()


def test_row_rules_reject_zero_and_half_scaled_outputs(case):
    _, _, _, _, out, _ = case
    check_rows(out, out)
    check_rows(out * (1 + 2e-3), out)            # what bf16 rounding does
    for wrong in (np.zeros_like(out), 0.5 * out, 0.9 * out):
        with pytest.raises(AssertionError):
            check_rows(wrong, out)


def test_row_rules_reject_swapped_value_rows(case):
    pb, q, k, v, out, _ = case
    v2 = v.copy()
    v2[[0, 1]] = v[[4096, 4097]]; v2[[4096, 4097]] = v[[0, 1]]
    wrong, _ = oracle.dense_attention(pb, q, k, v2, rows=ROWS)
    # two of 131,072 value rows out of place: too small for any output rule (that is what the small shapes
    # with element-by-element comparison are for) -- but a whole tile of them is not
    v3 = v.copy(); v3[0:64] = v[4096:4160]; v3[4096:4160] = v[0:64]
    wrong3, _ = oracle.dense_attention(pb, q, k, v3, rows=ROWS)
    with pytest.raises(AssertionError):
        check_rows(wrong3, out)
    assert np.abs(wrong - out).max() < np.abs(wrong3 - out).max()


def test_lse_rule_rejects_a_dropped_tile(case):
    pb, q, k, v, _, lse = case
    check_lse(lse + 1e-5, lse)
    pbs, sets = _all_but_one_diagonal(pb, skip=100)
    _, lse_drop = oracle.sparse_attention(pbs, q, k, v, *sets, rows=ROWS)
    assert (lse_drop < lse).all() and np.abs(lse_drop - lse).max() < 2e-3   # the old bound saw nothing
    with pytest.raises(AssertionError):
        check_lse(lse_drop, lse)


def test_block_class_values_reject_a_dropped_and_a_doubled_tile(case):
    pb, q, k, _, _, _ = case
    vc = v_block_classes(N_K, 1, D)
    ref, _ = oracle.dense_attention(pb, q, k, vc, rows=ROWS)
    np.testing.assert_allclose(ref.sum(-1), 1.0, rtol=1e-12)
    check_class_mass(ref * (1 + 1.5e-3), ref)    # bf16 rounding of the output
    # dropped from numerator and denominator alike (a tile the walk skipped)
    pbs, sets = _all_but_one_diagonal(pb, skip=100)
    drop, _ = oracle.sparse_attention(pbs, q, k, vc, *sets, rows=ROWS)
    with pytest.raises(AssertionError):
        check_class_mass(drop, ref)
    # dropped from the PV product only (a stale value tile): the values of one tile are zero
    vz = vc.copy(); vz[64 * 37: 64 * 38] = 0
    stale, _ = oracle.dense_attention(pb, q, k, vz, rows=ROWS)
    with pytest.raises(AssertionError):
        check_class_mass(stale, ref)
    # doubled: the values of one tile count twice
    v2 = vc.copy(); v2[64 * 37: 64 * 38][v2[64 * 37: 64 * 38] != 0] = 0x4000  # bf16 2.0
    twice, _ = oracle.dense_attention(pb, q, k, v2, rows=ROWS)
    with pytest.raises(AssertionError):
        check_class_mass(twice, ref)
    # and with random values the element rule of the contract sees none of the three
    for wrong in (drop, stale, twice):
        assert (np.abs(wrong - ref) <= ATOL + RTOL * np.abs(ref)).all()
