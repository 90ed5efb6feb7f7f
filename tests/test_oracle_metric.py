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
