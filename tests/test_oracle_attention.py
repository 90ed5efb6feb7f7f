"""Pins for the oracle's dense attention (O1) and top-M selection (O3).

Each check compares the oracle with something that is not the oracle: a library softmax / SDPA, a closed
form, an invariance, or a brute-force count on tiny inputs.
"""
import numpy as np
import pytest
import scipy.special
import torch

import oracle


def _rand(n, d, seed):
    r = np.random.default_rng(seed)
    return (r.standard_normal(d).astype(np.float32), r.standard_normal((n, d)).astype(np.float32),
            r.standard_normal((n, d)).astype(np.float32))


@pytest.mark.parametrize("n,d", [(1, 4), (7, 8), (65, 64), (640, 128)])
def test_dense_matches_library_softmax(n, d):
    q, K, V = _rand(n, d, 10 + n)
    scale = 1.0 / np.sqrt(d)
    o, p32, p64 = oracle.dense_attend(q, K, V, n, scale)
    z = (K.astype(np.float64) @ q.astype(np.float64)) * scale
    p_ref = scipy.special.softmax(z)
    np.testing.assert_allclose(p64, p_ref, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(o, p_ref @ V.astype(np.float64), rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(p32, p_ref.astype(np.float32), rtol=1e-6, atol=1e-12)
    # torch's fused attention in double, one query
    tq = torch.from_numpy(q).double().view(1, 1, 1, d)
    tk = torch.from_numpy(K).double().view(1, 1, n, d)
    tv = torch.from_numpy(V).double().view(1, 1, n, d)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=scale).view(d).numpy()
    np.testing.assert_allclose(o, ref, rtol=1e-6, atol=1e-7)


def test_probabilities_sum_to_one():
    for seed in range(5):
        q, K, V = _rand(200, 32, seed)
        _, p32, p64 = oracle.dense_attend(q * 3, K, V, 200, 0.3)
        assert abs(p64.sum() - 1.0) < 1e-12
        assert abs(p32.astype(np.float64).sum() - 1.0) < 1e-6
        assert (p64 >= 0).all()


def test_equal_keys_give_mean_of_values():
    q, K, V = _rand(33, 16, 3)
    K[:] = K[0]
    o, _, p = oracle.dense_attend(q, K, V, 33, 0.25)
    np.testing.assert_allclose(p, np.full(33, 1 / 33), rtol=1e-12)
    np.testing.assert_allclose(o, V.astype(np.float64).mean(0), rtol=1e-6, atol=1e-7)


def test_dominant_key_returns_its_value_row():
    d = 8
    q = np.zeros(d, np.float32); q[0] = 1
    K = np.zeros((10, d), np.float32); K[6, 0] = 40.0
    V = np.random.default_rng(0).standard_normal((10, d)).astype(np.float32)
    o, _, p = oracle.dense_attend(q, K, V, 10, 1.0)
    assert p[6] > 1 - 1e-15
    np.testing.assert_allclose(o, V[6], rtol=1e-6, atol=1e-7)


def test_logit_shift_invariance_and_scale_zero():
    q, K, V = _rand(50, 16, 7)
    o1, _, p1 = oracle.dense_attend(q, K, V, 50, 0.25)
    # adding t*q/|q|^2 to every key adds the same constant to every logit
    K2 = (K.astype(np.float64) + 5.0 * q / (q.astype(np.float64) @ q)).astype(np.float32)
    o2, _, p2 = oracle.dense_attend(q, K2, V, 50, 0.25)
    np.testing.assert_allclose(p1, p2, rtol=1e-4)
    np.testing.assert_allclose(o1, o2, rtol=1e-4, atol=1e-5)
    _, _, p0 = oracle.dense_attend(q, K, V, 50, 0.0)
    np.testing.assert_allclose(p0, np.full(50, 0.02), rtol=1e-12)


def test_row_list_is_a_gather_and_order_free():
    q, K, V = _rand(40, 8, 11)
    rows = np.array([3, 5, 6, 20, 39], np.int32)
    o, p32, p64 = oracle.attend(q, K, V, rows, 0.35)
    o_g, _, p_g = oracle.dense_attend(q, K[rows], V[rows], len(rows), 0.35)
    np.testing.assert_array_equal(o, o_g)
    np.testing.assert_array_equal(p64, p_g)
    perm = np.array([4, 0, 3, 1, 2])
    o_p, _, p_p = oracle.attend(q, K, V, rows[perm], 0.35)
    np.testing.assert_allclose(o_p, o, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(p_p, p64[perm], rtol=1e-12)
    # q and K are not interchangeable with V: swapping V for K changes the answer
    o_swapped, _, _ = oracle.attend(q, V, K, rows, 0.35)
    assert np.abs(o_swapped - o).max() > 1e-3


def test_empty_row_list_gives_zero_output():
    q, K, V = _rand(4, 8, 1)
    o, p32, _ = oracle.attend(q, K, V, np.zeros(0, np.int32), 1.0)
    assert (o == 0).all() and len(p32) == 0


# ---------------------------------------------------------------- O3 ----

def test_top_m_ties_go_to_lower_position():
    keep, gap = oracle.top_m([1, 2, 2, 1, 2], [0, 1, 2, 3, 4], 2)
    assert keep.tolist() == [1, 2]
    assert gap == 0.0
    keep, _ = oracle.top_m([5, 5, 5], [9, 4, 7], 1)
    assert keep.tolist() == [1]            # position 4 is the lowest


def test_top_m_keeps_all_when_few_candidates():
    keep, gap = oracle.top_m([0.5, 0.1, 0.9], [10, 20, 30], 3)
    assert keep.tolist() == [0, 1, 2] and gap == -1.0
    keep, gap = oracle.top_m([0.5, 0.1, 0.9], [10, 20, 30], 8)
    assert keep.tolist() == [0, 1, 2] and gap == -1.0
    keep, _ = oracle.top_m(np.zeros(0), np.zeros(0), 4)
    assert len(keep) == 0


def test_top_m_reports_by_position_and_gap():
    keep, gap = oracle.top_m([0.1, 0.9, 0.5, 0.7], [30, 20, 10, 0], 2)
    # kept are scores 0.9 (pos 20) and 0.7 (pos 0) -> by position: index 3 then index 1
    assert keep.tolist() == [3, 1]
    assert abs(gap - (0.7 - 0.5) / 0.7) < 1e-6


@pytest.mark.parametrize("seed", range(6))
def test_top_m_matches_lexsort_and_brute_force(seed):
    r = np.random.default_rng(seed)
    n = int(r.integers(1, 90))
    M = int(r.integers(1, 40))
    score = r.integers(0, 6, n).astype(np.float32) / 4      # many exact ties
    pos = r.permutation(1000)[:n].astype(np.int32)
    keep, _ = oracle.top_m(score, pos, M)
    order = np.lexsort((pos, -score))                       # library sort: score desc, then pos asc
    want = set(pos[order[:M]].tolist())
    assert set(pos[keep].tolist()) == want
    assert list(pos[keep]) == sorted(pos[keep])
    # definition by counting: kept iff fewer than M candidates come strictly before it
    for i in range(n):
        before = sum(1 for j in range(n) if (score[j] > score[i]) or (score[j] == score[i] and pos[j] < pos[i]))
        assert (before < M) == (pos[i] in want)
