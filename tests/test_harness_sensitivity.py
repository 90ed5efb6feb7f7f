"""The parity comparators must notice plausible mistakes.  Each case plants one mistake on the CPU -- in a
second run of the oracle with a wrong parameter or a perturbed input -- and checks that the comparison the
GPU tests rely on (output tolerance, exact index sets) rejects it.  No GPU is involved."""
import numpy as np
import pytest

import oracle
import workload
from harness import TOL, check_outputs, spatial_positions


def _unit(wl, ht, data, l, b, h, **over):
    q, K, V = workload.unit_arrays(data, l, b, h)
    p = dict(W=wl.W, S=wl.S, M=wl.M, R=wl.R, C=wl.C)
    p.update({k: v for k, v in over.items() if k in p})
    u = oracle.Unit(ht[l, h] == workload.SEMANTIC, p["W"], p["S"], p["M"], p["R"], p["C"], buffered_spatial=wl.alg2)
    scale = over.get("scale", wl.scale)
    if "q_row_shift" in over:
        q = np.roll(q, over["q_row_shift"], axis=0)
    o, hl, gl = u.run(q, K, V, scale, workload.compress_schedule(wl), accumulate=over.get("accumulate", True), log=True)
    return o, hl


@pytest.fixture(scope="module")
def case():
    wl = workload.Workload("sens", L=1, prompts=1, H=4, d=128, dtype="bf16", n0=8, grid_h=8, grid_w=10, W=12, M=9,
                           S=1, R=2, C=6, cadence=4, seed=21, plain=True)
    ht = workload.head_map(wl)
    return wl, ht, workload.generate(wl, head_type=ht)


def _rejected(wl, ref, bad):
    try:
        check_outputs(bad, ref, wl.dtype, "planted")
    except AssertionError:
        return True
    return False


@pytest.mark.parametrize("h,over", [(0, dict(W=11)), (0, dict(W=13)), (0, dict(S=0)), (0, dict(S=2)),
                                    (0, dict(scale=0.0884 * 1.05)), (0, dict(q_row_shift=1)),
                                    (3, dict(M=8)), (3, dict(M=10)), (3, dict(R=1)), (3, dict(accumulate=False)),
                                    (3, dict(scale=0.0884 * 0.95))])
def test_planted_mistake_is_detected(case, h, over):
    wl, ht, data = case
    o_ref, hl_ref = _unit(wl, ht, data, 0, 0, h)
    o_bad, hl_bad = _unit(wl, ht, data, 0, 0, h, **over)
    sets_differ = ht[0, h] == workload.SEMANTIC and not np.array_equal(hl_ref, hl_bad)
    assert _rejected(wl, o_ref, o_bad) or sets_differ, over


def test_identical_runs_pass_and_bf16_rounding_is_inside_the_tolerance(case):
    wl, ht, data = case
    o_ref, _ = _unit(wl, ht, data, 0, 1, 2)
    check_outputs(o_ref.copy(), o_ref, wl.dtype, "same")
    import torch
    rounded = torch.from_numpy(o_ref).to(torch.bfloat16).float().numpy()
    check_outputs(rounded, o_ref, wl.dtype, "bf16 rounding of the reference")
    atol, rtol = TOL["bf16"]
    assert _rejected(wl, o_ref, o_ref + (atol + rtol * np.abs(o_ref)) * 1.01)


def test_closed_form_window_sets_used_by_the_harness():
    wl = workload.Workload("w", L=1, prompts=1, H=2, d=64, dtype="f32", n0=2, grid_h=2, grid_w=2, W=3, M=2, S=1)
    assert spatial_positions(wl, 1) == [0]
    assert spatial_positions(wl, 6) == [0, 3, 4, 5]
    assert spatial_positions(wl.replace(alg2=True), 6, 4) == [0, 1, 2, 3, 4, 5]
    assert spatial_positions(wl.replace(alg2=True), 6, 6) == [0, 3, 4, 5]


def _rope_unit(wl, ht, data, h, layout_q, layout_k, shift_k=0, flip_k=False, rotate_q=True):
    q, K, V = workload.unit_arrays(data, 0, 0, h)
    cos_t, sin_t = workload.rope_tables(wl.n_total + 1, wl.d)
    import torch
    rnd = lambda x: torch.from_numpy(x).to(torch.bfloat16).float().numpy()
    qr = np.stack([oracle.rope(q[p], cos_t[p], sin_t[p], layout_q) for p in range(wl.n_total)]) if rotate_q else q
    kr = np.stack([oracle.rope(K[p], cos_t[p + shift_k], (-sin_t if flip_k else sin_t)[p + shift_k], layout_k)
                   for p in range(wl.n_total)])
    u = oracle.Unit(ht[0, h] == workload.SEMANTIC, wl.W, wl.S, wl.M, wl.R, wl.C)
    o, hl, _ = u.run(rnd(qr), rnd(kr), V, wl.scale, workload.compress_schedule(wl), log=True)
    return o, hl


@pytest.mark.parametrize("h", [0, 3])
@pytest.mark.parametrize("bad", [dict(layout_q=2, layout_k=2), dict(layout_q=1, layout_k=2), dict(shift_k=1), dict(flip_k=True),
                                 dict(rotate_q=False)])
def test_planted_rotary_mistake_is_detected(case, h, bad):
    # wrong pairing, k one position off, k turned the other way, q left unrotated
    wl, ht, data = case
    o_ref, hl_ref = _rope_unit(wl, ht, data, h, 1, 1)
    o_bad, hl_bad = _rope_unit(wl, ht, data, h, **dict(dict(layout_q=1, layout_k=1), **bad))
    sets_differ = ht[0, h] == workload.SEMANTIC and not np.array_equal(hl_ref, hl_bad)
    assert _rejected(wl, o_ref, o_bad) or sets_differ, bad
