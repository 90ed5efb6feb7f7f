"""Pins for the oracle's cache policy (O4): the hand-worked case, an exact-rational brute force,
closed-form window sets, the unbounded limit, structural invariants and the planted sinks."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workload

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "handcase_semantic.txt")


def _load_handcase():
    cases = {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tok = line.split()
        name, step, out = tok[0], int(tok[1]), Fraction(tok[2])
        scores = {int(t.split(":")[0]): Fraction(t.split(":")[1]) for t in tok[3:-1]}
        heavy = [] if tok[-1] == "-" else [int(x) for x in tok[-1].split(",")]
        cases.setdefault(name, []).append((step, out, scores, heavy))
    return cases


HAND_K = np.array([[0.0], [math.log(3.0)], [0.0], [0.0], [0.0]], np.float32)
HAND_V = np.array([[1.0], [2.0], [3.0], [4.0], [5.0]], np.float32)
HAND_Q = np.ones((5, 1), np.float32)


@pytest.mark.parametrize("name,M", [("m2", 2), ("m1", 1)])
def test_hand_worked_case(name, M):
    steps = _load_handcase()[name]
    u = oracle.Unit(True, W=0, S=0, M=M, R=1, C_=2)
    for step, out, scores, heavy in steps:
        assert u.append() == 0
        o, p = u.attend(HAND_Q[step], HAND_K, HAND_V, 1.0, accumulate=True)
        assert abs(float(o[0]) - float(out)) < 2e-6
        hp, hs, sp, ss = u.state()
        got = dict(zip(hp.tolist() + sp.tolist(), hs.tolist() + ss.tolist()))
        assert sorted(got) == sorted(scores)
        for pos, val in scores.items():
            assert abs(got[pos] - float(val)) < 2e-6, (step, pos)
        u.compress()
        hp, _, sp, _ = u.state()
        assert hp.tolist() == heavy
        assert sp.tolist() == [step]           # the newest token is always kept


def _rational_sim(weights, values, M, R, C, compress_after):
    """Exact simulation with integer attention weights: dict-based, Fractions only (no exp, no floats)."""
    heavy, staged, score = [], [], {}
    outs, heavies = [], []
    for p in range(len(weights)):
        assert len(staged) < C
        staged.append(p); score[p] = Fraction(0)
        ret = heavy + staged
        tot = sum(Fraction(weights[j]) for j in ret)
        outs.append(sum(Fraction(weights[j]) * Fraction(values[j]) for j in ret) / tot)
        for j in ret:
            score[j] += Fraction(weights[j]) / tot
        if compress_after[p]:
            keep_new = staged[-R:] if R > 0 else []
            cand = heavy + [j for j in staged if j not in keep_new]
            cand.sort(key=lambda j: (-score[j], j))
            for j in cand[M:]:
                del score[j]
            heavy = sorted(cand[:M]); staged = keep_new
        heavies.append(list(heavy))
    return outs, heavies, score


@pytest.mark.parametrize("seed", range(8))
def test_against_exact_rational_brute_force(seed):
    r = np.random.default_rng(100 + seed)
    n = 24
    M, R = int(r.integers(1, 6)), int(r.integers(1, 4))
    cadence = int(r.integers(1, 5))
    C = R + cadence
    weights = [int(x) for x in r.integers(1, 9, n)]
    values = [int(x) for x in r.integers(-5, 6, n)]
    ca = [(p + 1) % cadence == 0 for p in range(n)]
    outs, heavies, score = _rational_sim(weights, values, M, R, C, ca)
    K = np.log(np.array(weights, np.float64)).astype(np.float32).reshape(n, 1)
    # float32 keys carry ~1e-7 relative error in the weights; compare with a matching tolerance
    V = np.array(values, np.float32).reshape(n, 1)
    u = oracle.Unit(True, W=0, S=0, M=M, R=R, C_=C)
    o, hl, gl = u.run(np.ones((n, 1), np.float32), K, V, 1.0, np.array(ca, np.uint8), log=True)
    for p in range(n):
        assert abs(float(o[p, 0]) - float(outs[p])) < 1e-5
        # sets must agree whenever the exact cut is not a near-tie
        if gl[p] < 0 or gl[p] > 1e-5:
            assert [x for x in hl[p].tolist() if x >= 0] == heavies[p], p
    hp, hs, sp, ss = u.state()
    for pos, val in zip(hp.tolist() + sp.tolist(), hs.tolist() + ss.tolist()):
        assert abs(val - float(score[pos])) < 1e-5


@pytest.mark.parametrize("S,W", [(0, 4), (1, 4), (1, 1), (2, 16), (3, 2), (0, 1)])
def test_spatial_retained_set_closed_form(S, W):
    u = oracle.Unit(False, W=W, S=S, M=0, R=0, C_=0)
    for p in range(40):
        assert u.append() == 0
        n = p + 1
        want = sorted(set(range(min(S, n))) | set(range(max(S, n - W), n)))
        assert u.retained().tolist() == want
        assert len(want) <= S + W
        assert u.compress() == (0, -1.0)
        assert u.retained().tolist() == want


def test_unbounded_window_and_budget_reproduce_dense_attention_exactly():
    r = np.random.default_rng(5)
    n, d = 48, 16
    q, K, V = (r.standard_normal((n, d)).astype(np.float32) for _ in range(3))
    ca = np.ones(n, np.uint8)
    sp = oracle.Unit(False, W=n, S=0, M=0, R=0, C_=0)
    se = oracle.Unit(True, W=0, S=0, M=n, R=1, C_=2)
    se_lazy = oracle.Unit(True, W=0, S=0, M=n, R=3, C_=n + 1)
    o_sp, _, _ = sp.run(q, K, V, 0.25, ca)
    o_se, _, _ = se.run(q, K, V, 0.25, ca)
    o_lz, _, _ = se_lazy.run(q, K, V, 0.25, np.zeros(n, np.uint8))
    for p in range(n):
        o_ref, _, _ = oracle.dense_attend(q[p], K, V, p + 1, 0.25)
        np.testing.assert_array_equal(o_sp[p], o_ref)
        np.testing.assert_array_equal(o_se[p], o_ref)
        np.testing.assert_array_equal(o_lz[p], o_ref)


def test_row_buffer_overflow_is_an_error_and_changes_nothing():
    u = oracle.Unit(True, W=0, S=0, M=4, R=1, C_=3)
    assert [u.append() for _ in range(3)] == [0, 0, 0]
    before = u.retained().tolist()
    assert u.append() == -1
    assert u.n == 3 and u.retained().tolist() == before
    u.compress()
    assert u.append() == 0 and u.n == 4
    with pytest.raises(OverflowError):
        v = oracle.Unit(True, W=0, S=0, M=4, R=1, C_=2)
        z = np.zeros((8, 2), np.float32)
        v.run(z, z, z, 1.0, np.zeros(8, np.uint8))


@pytest.mark.parametrize("M,R,cadence", [(4, 1, 1), (6, 2, 3), (3, 3, 5), (8, 1, 8)])
def test_semantic_invariants(M, R, cadence):
    r = np.random.default_rng(M * 100 + R * 10 + cadence)
    n, d = 60, 8
    q, K, V = (r.standard_normal((n, d)).astype(np.float32) for _ in range(3))
    C = R + cadence
    u = oracle.Unit(True, W=0, S=0, M=M, R=R, C_=C)
    for p in range(n):
        assert u.append() == 0
        hp0, hs0, sp0, ss0 = u.state()
        mass0 = float(hs0.astype(np.float64).sum() + ss0.astype(np.float64).sum())
        _, prob = u.attend(q[p], K, V, 0.35, accumulate=True)
        hp1, hs1, sp1, ss1 = u.state()
        mass1 = float(hs1.astype(np.float64).sum() + ss1.astype(np.float64).sum())
        assert abs(prob.astype(np.float64).sum() - 1) < 1e-6
        assert abs((mass1 - mass0) - 1.0) < 1e-5      # every step adds exactly one unit of mass
        assert (hs1 >= 0).all() and (ss1 >= 0).all()
        assert len(hp1) <= M and len(sp1) <= C
        if (p + 1) % cadence == 0:
            u.compress()
            hp2, hs2, sp2, ss2 = u.state()
            assert set(hp2.tolist()) <= set(hp1.tolist()) | set(sp1.tolist())
            assert sp2.tolist() == list(range(max(0, p + 1 - R), p + 1))     # the R newest stay
            assert len(hp2) == min(M, len(hp1) + len(sp1) - len(sp2))
            assert max(hp2.tolist() + [-1]) < min(sp2.tolist())
            kept = dict(zip(hp1.tolist() + sp1.tolist(), hs1.tolist() + ss1.tolist()))
            for pos, sc in zip(hp2.tolist(), hs2.tolist()):
                assert sc == kept[pos]                                        # scores travel with tokens
            dropped = [kept[x] for x in set(kept) - set(hp2.tolist()) - set(sp2.tolist())]
            if dropped:
                assert max(dropped) <= min(hs2.tolist())


def test_evicted_token_never_returns():
    r = np.random.default_rng(9)
    n, d = 80, 4
    q, K, V = (r.standard_normal((n, d)).astype(np.float32) for _ in range(3))
    u = oracle.Unit(True, W=0, S=0, M=5, R=1, C_=2)
    _, hl, _ = u.run(q, K, V, 0.5, np.ones(n, np.uint8), log=True)
    gone = set()
    prev = set()
    for p in range(n):
        cur = set(x for x in hl[p].tolist() if x >= 0)
        assert not (cur & gone)
        gone |= (prev | ({p - 1} if p >= 1 else set())) - cur - {p}
        prev = cur


def test_load_dense_selects_by_given_scores():
    r = np.random.default_rng(2)
    n_src, M, R = 50, 7, 3
    score = (r.integers(0, 5, n_src) / 4).astype(np.float32)
    u = oracle.Unit(True, W=0, S=0, M=M, R=R, C_=R + 4)
    u.load_dense(n_src, score)
    hp, hs, sp, ss = u.state()
    order = np.lexsort((np.arange(n_src - R), -score[: n_src - R]))
    assert hp.tolist() == sorted(order[:M].tolist())
    np.testing.assert_array_equal(hs, score[hp])
    assert sp.tolist() == [47, 48, 49]
    np.testing.assert_array_equal(ss, score[47:])
    assert u.n == n_src and u.append() == 0
    # without scores every candidate ties at 0: the lowest positions win
    z = oracle.Unit(True, W=0, S=0, M=M, R=R, C_=R + 4)
    z.load_dense(n_src, None)
    assert z.state()[0].tolist() == list(range(M))
    s = oracle.Unit(False, W=8, S=1, M=0, R=0, C_=0)
    s.load_dense(n_src, None)
    assert s.retained().tolist() == [0] + list(range(42, 50))


def test_planted_sinks_are_kept_on_the_tiny_config():
    wl = workload.config(1)
    data = workload.generate(wl)
    ht = workload.head_map(wl)
    sinks = workload.sink_positions(wl)
    ca = workload.compress_schedule(wl)
    checked = 0
    for b in range(wl.B):
        for h in range(wl.H):
            if ht[0, h] != workload.SEMANTIC:
                continue
            q, K, V = workload.unit_arrays(data, 0, b, h)
            u = oracle.Unit(True, wl.W, wl.S, wl.M, wl.R, wl.C)
            u.run(q, K, V, wl.scale, ca)
            hp, _, sp, _ = u.state()
            assert set(sinks) <= set(hp.tolist()) | set(sp.tolist())
            assert len(hp) == wl.M
            checked += 1
    assert checked == wl.B * wl.H // 2


# ------------------------------------------------ Algorithm 2: spatial heads read the row buffer too ----

def _alg2_spatial_lists(n_tokens, S, W, R, C, compress_after):
    """Algorithm 2 as written, with explicit lists: `cached` (sink + recent as of the last compression) and
    `buf` (row buffer); the head attends to their concatenation; a compression rebuilds cached from all
    tokens seen so far and resets the buffer (keeping the R newest buffered, as semantic heads do)."""
    cached, buf, out = [], [], []
    for p in range(n_tokens):
        assert len(buf) < C
        buf.append(p)
        out.append(sorted(set(cached) | set(buf)))
        if compress_after[p]:
            seen = list(range(p + 1))
            cached = sorted(set(seen[:S]) | set(seen[S:][-W:] if W > 0 else []))
            buf = buf[len(buf) - min(R, len(buf)):]
    return out


@pytest.mark.parametrize("S,W,R,C,cadence", [(1, 4, 0, 3, 3), (1, 8, 0, 24, 24), (0, 5, 2, 6, 4), (2, 3, 1, 2, 1), (1, 6, 0, 1, 1)])
def test_algorithm2_spatial_row_buffer(S, W, R, C, cadence):
    n = 70
    ca = [(p + 1) % cadence == 0 for p in range(n)]
    want = _alg2_spatial_lists(n, S, W, R, C, ca)
    u = oracle.Unit(False, W=W, S=S, M=0, R=R, C_=C, buffered_spatial=True)
    sizes = set()
    for p in range(n):
        assert u.append() == 0
        assert u.retained().tolist() == want[p], p
        sizes.add(len(want[p]))
        if ca[p]:
            u.compress()
    if cadence > 1:
        assert max(sizes) == S + W + cadence          # the window breathes between W+1 and W+cadence
    if cadence == 1 and R == 0:
        # compressing after every token makes Algorithm 2 keep W older tokens plus the new one
        plain = oracle.Unit(False, W=W + 1, S=S, M=0, R=0, C_=0)
        for p in range(n):
            plain.append()
        assert want[n - 1] == plain.retained().tolist()


def test_algorithm2_spatial_overflow_and_dense_source():
    u = oracle.Unit(False, W=4, S=1, M=0, R=0, C_=3, buffered_spatial=True)
    assert [u.append() for _ in range(4)] == [0, 0, 0, -1]
    u.compress()
    assert u.append() == 0
    assert u.retained().tolist() == [0, 1, 2, 3]
    v = oracle.Unit(False, W=4, S=1, M=0, R=0, C_=3, buffered_spatial=True)
    v.load_dense(20)
    assert v.retained().tolist() == [0, 16, 17, 18, 19]
    v.append(); v.append()
    assert v.retained().tolist() == [0, 16, 17, 18, 19, 20, 21]
