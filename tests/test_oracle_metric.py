"""Pins for the oracle's sparsity metric and head typing (O2): closed forms, a library mean, the strict
threshold, and recovery of the planted head types."""
import os

import numpy as np
import pytest

import oracle
import workload

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "metric_closed_forms.txt")


def _closed_forms():
    rows = []
    for line in open(GOLDEN):
        line = line.strip()
        if line and not line.startswith("#"):
            name, T, w, s = line.split()
            rows.append((name, int(T), int(w), float(s)))
    return rows


def _pattern(name, n0, T, d=2):
    n = n0 + T
    q = np.zeros((n, d), np.float32); q[:, 0] = 1.0
    K = np.zeros((n, d), np.float32)
    V = np.zeros((n, d), np.float32)
    if name == "uniform":
        pass                                   # all keys equal
    elif name == "recent_only":
        K[:, 0] = np.arange(n) * 60.0          # the newest key dominates every step
    elif name == "first_visual_only":
        K[n0, 0] = 80.0
    return q, K, V


@pytest.mark.parametrize("name,T,w,expected", _closed_forms())
@pytest.mark.parametrize("n0", [0, 5])
def test_metric_closed_forms(name, T, w, expected, n0):
    q, K, V = _pattern(name, n0, T)
    far, tot = oracle.profile_unit(q, K, V, n0, T, w, 1.0)
    s, ty = oracle.classify(far.reshape(1, 1, 1, T), tot.reshape(1, 1, 1, T), 0.5)
    assert abs(s[0, 0] - expected) < 2e-6
    assert ty[0, 0] == (1 if expected > 0.5 else 0)


def test_far_tot_index_ranges():
    p = np.arange(1, 11, dtype=np.float64)          # n0 = 3 prompt rows, t = 7 visual rows
    far, tot = oracle.far_tot(p, 3, 7, 2)
    assert tot == sum(range(4, 11))                  # visual rows only
    assert far == sum(range(4, 9))                   # visual rows 0..t-1-w = 0..4
    assert oracle.far_tot(p, 3, 7, 7)[0] == 0.0      # t <= w: empty numerator
    assert oracle.far_tot(p, 3, 7, 6)[0] == 4.0      # exactly one far row
    assert oracle.far_tot(p, 0, 10, 0) == (55.0, 55.0)


def test_classify_is_a_mean_of_ratios_with_strict_threshold():
    r = np.random.default_rng(0)
    L, P, H, T = 3, 4, 5, 17
    tot = r.uniform(0.2, 1.0, (L, P, H, T)).astype(np.float32)
    far = (tot * r.uniform(0, 1, (L, P, H, T))).astype(np.float32)
    s, ty = oracle.classify(far, tot, 0.5)
    ref = (far.astype(np.float64) / tot.astype(np.float64)).mean(axis=(1, 3))
    np.testing.assert_allclose(s, ref, rtol=1e-12)
    np.testing.assert_array_equal(ty, (ref > 0.5).astype(np.uint8))
    # s == tau is Spatial (strict inequality of Eq. 3)
    far1 = np.ones((1, 2, 1, 4), np.float32); tot1 = 2 * far1
    assert oracle.classify(far1, tot1, 0.5)[1][0, 0] == 0
    assert oracle.classify(far1, tot1, 0.49999)[1][0, 0] == 1
    # a zero denominator contributes ratio 0
    tot1[0, 0, 0, 0] = 0
    assert abs(oracle.classify(far1, tot1, 0.5)[0][0, 0] - 0.5 * 7 / 8) < 1e-12


def test_planted_head_types_are_recovered():
    wl = workload.config(1)
    data = workload.generate(wl)
    ht = workload.head_map(wl)
    w = 16                                            # an 8x8 grid is shorter than the paper's w = 32 window
    far = np.zeros((wl.L, wl.B, wl.H, wl.N), np.float32)
    tot = np.zeros_like(far)
    for b in range(wl.B):
        for h in range(wl.H):
            q, K, V = workload.unit_arrays(data, 0, b, h)
            far[0, b, h], tot[0, b, h] = oracle.profile_unit(q, K, V, wl.n0, wl.N, w, wl.scale)
    s, ty = oracle.classify(far, tot, 0.3)
    np.testing.assert_array_equal(ty, ht)
    assert s[ht == workload.SPATIAL].max() < 0.2
    assert s[ht == workload.SEMANTIC].min() > 0.4


# ------------------------------------------------------------------ prefill scores ----

def test_prefill_scores_closed_forms_and_library_softmax():
    import scipy.special
    r = np.random.default_rng(3)
    n, d = 37, 16
    q = r.standard_normal((n, d)).astype(np.float32)
    K = r.standard_normal((n, d)).astype(np.float32)
    s = oracle.prefill_scores(q, K, 0.25)
    # every query row distributes exactly one unit of mass
    assert abs(float(s.astype(np.float64).sum()) - n) < 1e-4
    # library softmax with a causal mask, column sums
    z = (q.astype(np.float64) @ K.astype(np.float64).T) * 0.25
    z[np.triu_indices(n, 1)] = -np.inf
    ref = scipy.special.softmax(z, axis=1).sum(axis=0)
    np.testing.assert_allclose(s, ref, rtol=1e-6, atol=1e-7)
    # uniform attention (all keys equal): score[j] = sum_{i>=j} 1/(i+1) = H_n - H_j
    Ku = np.zeros_like(K)
    su = oracle.prefill_scores(q, Ku, 1.0)
    H = np.concatenate([[0.0], np.cumsum(1.0 / np.arange(1, n + 1))])
    np.testing.assert_allclose(su, H[n] - H[:n], rtol=1e-6)
    # the last token is only ever seen by itself; the first by everyone
    assert abs(su[-1] - 1.0 / n) < 1e-7 and su[0] == su.max()
    # one dominant key at position 5: it collects one unit from every later query
    Kd = np.zeros((n, d), np.float32); Kd[5, 0] = 60.0
    qd = np.zeros((n, d), np.float32); qd[:, 0] = 1.0
    sd = oracle.prefill_scores(qd, Kd, 1.0)
    assert abs(sd[5] - (n - 5)) < 1e-5


def test_prefill_scores_equal_what_decode_steps_accumulate():
    # the same prompt fed token by token through the cache policy without any compression
    r = np.random.default_rng(4)
    n, d = 20, 8
    q, K, V = (r.standard_normal((n, d)).astype(np.float32) for _ in range(3))
    u = oracle.Unit(True, W=0, S=0, M=n, R=1, C_=n + 1)
    u.run(q, K, V, 0.3, np.zeros(n, np.uint8))
    _, _, sp, ss = u.state()
    assert sp.tolist() == list(range(n))
    np.testing.assert_allclose(ss, oracle.prefill_scores(q, K, 0.3), rtol=2e-6, atol=1e-6)


# ---- O6: classifier-free guidance, Eq. (1) -------------------------------------------------------------

def test_cfg_mix_pinned_values_and_special_cases():
    # hand-computed: c + gamma (c - u)
    p = np.array([[0.5, 0.25, 0.25],        # prompt 0, conditional
                  [0.25, 0.5, 0.25],        # prompt 0, unconditional
                  [1.0, 0.0, -2.0],         # prompt 1, conditional
                  [0.0, 0.0, 2.0]], np.float32)
    got = oracle.cfg_mix(p, 2.0)
    assert got.tolist() == [[1.0, -0.25, 0.25], [3.0, 0.0, -10.0]]
    # gamma = 0 returns the conditional rows; equal rows are a fixed point for every gamma
    assert np.array_equal(oracle.cfg_mix(p, 0.0), p[0::2])
    same = np.repeat(p[0::2], 2, axis=0)
    assert np.array_equal(oracle.cfg_mix(same, 7.5), p[0::2])
    # gamma = -1 returns the unconditional rows (the formula is affine in gamma)
    assert np.array_equal(oracle.cfg_mix(p, -1.0), p[1::2])


def test_cfg_mix_matches_numpy_and_keeps_the_total_mass():
    r = np.random.default_rng(3)
    p = r.random((6, 37)).astype(np.float32)
    p /= p.sum(axis=1, keepdims=True)
    for gamma in (1.0, 5.0):
        got = oracle.cfg_mix(p, gamma)
        ref = p[0::2].astype(np.float64) * (1 + gamma) - gamma * p[1::2].astype(np.float64)
        np.testing.assert_allclose(got, ref, rtol=1e-6, atol=1e-7)
        # both inputs sum to one, so the guided row does too (it need not stay non-negative)
        np.testing.assert_allclose(got.sum(axis=1), 1.0, atol=1e-5)
    # the pair order matters: swapping conditional and unconditional changes the result
    sw = p.reshape(3, 2, 37)[:, ::-1].reshape(6, 37)
    assert not np.allclose(oracle.cfg_mix(sw, 5.0), oracle.cfg_mix(p, 5.0))


# ---- O7: rotary position embedding (not from the paper; Su et al., "RoFormer") ----------------------

def _perm_half_to_interleaved(d):
    """index map: position in the interleaved layout of each element of the half layout"""
    return np.array([2 * i for i in range(d // 2)] + [2 * i + 1 for i in range(d // 2)])


def test_rope_special_cases_and_invariants():
    r = np.random.default_rng(0)
    for d in (2, 8, 64, 128):
        x = r.standard_normal((5, d)).astype(np.float32)
        cos_t, sin_t = workload.rope_tables(40, d)
        for layout in (oracle.ROPE_HALF, oracle.ROPE_INTERLEAVED):
            # position 0 turns nothing; any position keeps every pair's (hence the row's) length
            np.testing.assert_array_equal(oracle.rope(x, cos_t[0], sin_t[0], layout), x)
            y = oracle.rope(x, cos_t[17], sin_t[17], layout)
            np.testing.assert_allclose((y.astype(np.float64) ** 2).sum(-1), (x.astype(np.float64) ** 2).sum(-1), rtol=1e-6)
            # rotating to position p and then by the angles of position s lands at position p + s
            z = oracle.rope(oracle.rope(x, cos_t[5], sin_t[5], layout), cos_t[12], sin_t[12], layout)
            np.testing.assert_allclose(z, y, atol=2e-6)
    # a quarter turn of one pair: (a, b) -> (-b, a); which elements form the pair is what the layouts differ in
    x = np.array([1.0, 2.0, 3.0, 4.0], np.float32)
    c, s = np.zeros(2, np.float32), np.ones(2, np.float32)
    np.testing.assert_array_equal(oracle.rope(x, c, s, oracle.ROPE_HALF), [-3.0, -4.0, 1.0, 2.0])
    np.testing.assert_array_equal(oracle.rope(x, c, s, oracle.ROPE_INTERLEAVED), [-2.0, 1.0, -4.0, 3.0])
    # only the second pair turned
    c, s = np.array([1.0, 0.0], np.float32), np.array([0.0, 1.0], np.float32)
    np.testing.assert_array_equal(oracle.rope(x, c, s, oracle.ROPE_HALF), [1.0, -4.0, 3.0, 2.0])
    np.testing.assert_array_equal(oracle.rope(x, c, s, oracle.ROPE_INTERLEAVED), [1.0, 2.0, -4.0, 3.0])


def test_rope_is_complex_multiplication_and_depends_on_relative_position_only():
    r = np.random.default_rng(1)
    d, n = 64, 50
    cos_t, sin_t = workload.rope_tables(n, d)
    q = r.standard_normal(d).astype(np.float32)
    k = r.standard_normal(d).astype(np.float32)
    # the textbook statement: pair i as a complex number times e^{i * angle_i}
    ang = np.arctan2(sin_t[23].astype(np.float64), cos_t[23].astype(np.float64))
    zi = (q[0::2].astype(np.float64) + 1j * q[1::2]) * np.exp(1j * ang)
    want_i = np.empty(d)
    want_i[0::2], want_i[1::2] = zi.real, zi.imag
    np.testing.assert_allclose(oracle.rope(q, cos_t[23], sin_t[23], oracle.ROPE_INTERLEAVED), want_i, atol=1e-6)
    zh = (q[: d // 2].astype(np.float64) + 1j * q[d // 2:]) * np.exp(1j * ang)
    np.testing.assert_allclose(oracle.rope(q, cos_t[23], sin_t[23], oracle.ROPE_HALF), np.concatenate([zh.real, zh.imag]), atol=1e-6)
    # the two layouts are one rotation seen through a permutation of the elements
    perm = _perm_half_to_interleaved(d)
    xi = np.empty(d, np.float32)
    xi[perm] = q
    np.testing.assert_array_equal(oracle.rope(xi, cos_t[23], sin_t[23], oracle.ROPE_INTERLEAVED)[perm],
                                  oracle.rope(q, cos_t[23], sin_t[23], oracle.ROPE_HALF))
    # the property the embedding exists for: <R_p q, R_s k> depends on p - s only
    for layout in (oracle.ROPE_HALF, oracle.ROPE_INTERLEAVED):
        ref = float(np.dot(oracle.rope(q, cos_t[9], sin_t[9], layout).astype(np.float64), k))
        for p, s_ in ((9, 0), (20, 11), (49, 40)):
            got = float(np.dot(oracle.rope(q, cos_t[p], sin_t[p], layout).astype(np.float64),
                               oracle.rope(k, cos_t[s_], sin_t[s_], layout).astype(np.float64)))
            assert abs(got - ref) < 2e-4 * (1 + abs(ref))
        other = float(np.dot(oracle.rope(q, cos_t[10], sin_t[10], layout).astype(np.float64), k))
        assert abs(other - ref) > 1e-3      # and it does depend on it


def test_rope_tables_are_the_standard_angles():
    cos_t, sin_t = workload.rope_tables(9, 8, base=10000.0)
    assert cos_t.shape == sin_t.shape == (9, 4)
    np.testing.assert_array_equal(cos_t[0], 1.0)
    np.testing.assert_array_equal(sin_t[0], 0.0)
    np.testing.assert_allclose(cos_t ** 2 + sin_t ** 2, 1.0, atol=1e-6)
    # pair i turns by position * base^(-2i/d): pair 0 by one radian per position, the last pair slowest
    np.testing.assert_allclose(np.arctan2(sin_t[1], cos_t[1]), [1.0, 0.1, 0.01, 0.001], rtol=1e-5)
    np.testing.assert_allclose(np.arctan2(sin_t[3, 1:], cos_t[3, 1:]), [0.3, 0.03, 0.003], rtol=1e-5)
