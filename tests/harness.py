"""Shared driver for the GPU parity tests: runs a workload through the C-ABI library step by step and
compares sampled (layer, sequence, head) units with the CPU oracle.

Index sets are compared exactly.  Because GPU and CPU exponentials differ in the last bits, a top-M cut
whose oracle margin is below GAP_MARGIN (relative) may legitimately fall the other way.  That is the only
excuse for a differing heavy set, and it is granted for the cut of the near-tie itself only: the first
difference must appear between the last exported step at which the sets agreed and the step at which they
differ, at a compression whose oracle margin is within GAP_MARGIN; the caller then has to show that the GPU's
selection at that very step is the oracle's selection routine applied to the GPU's own scores (`verify_near_tie`).
Such a unit is counted and not compared further (its later state legitimately differs).

The own-score check (selection routine of the oracle on the scores the GPU held just before the cut) is also run
unconditionally at every exported compression step, on both paths:
  three calls : the tables are exported between ssd_decode_attn and ssd_compress_kv;
  fused step  : the attention, the score update and the selection are one launch, so nothing can be exported in
                between.  A second cache is kept in step with the first on the host only (launches switched off);
                at an exported compression step it receives a copy of the first cache's memory and takes the
                same fused step with compress = 0 -- the same kernel up to and including the score update -- which
                leaves exactly the scores the first cache's selection worked on."""
from __future__ import annotations

import sys
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

import oracle
import paper_2510_18716_amd as ssd
import workload
from paper_2510_18716_amd.binding import make_config

GAP_MARGIN = 1e-4

# The rotary step in bf16.  The kernel rotates k in fp32 (one product, one fused multiply-add) and rounds to bf16; the oracle
# rotates in double and rounds to bf16.  Where the exact value lies within 2^-24 (relative) of a bf16 rounding boundary --
# about 3 elements in 10^5 -- the two stored keys differ by one bf16 ulp, 2^-8 of the element.  The logit of that row then
# differs by scale * |q_i| * |k_i| * 2^-8, at most 0.125 * 3 * 3 * 2^-8 = 4.4e-3 for entries within three standard deviations
# (d = 64; 3.1e-3 at d = 128), and so does the row's probability, relatively, at every step it is attended, hence its
# accumulated score.  Scores and near-tie margins of such runs are therefore compared at 5e-3; outputs keep the bf16
# tolerance, index sets stay exact outside the margin, and the own-score check applies unchanged.
ROPE_BF16_MARGIN = 5e-3

# |gpu - ref| <= atol + rtol |ref|.
#   bf16: the target stated for the bf16 path (the output is rounded to bf16: half an ulp at |o| < 8 is 1.6e-2).
#   f32 : the error model of the kernel's arithmetic.  Logits: d <= 128 products accumulated in fp32,
#         |z| <~ 30, error <~ 64 * 2^-24 * |z| ~ 1e-4 absolute in the exponent's argument -- a relative error of
#         that size in one probability only when that row dominates, and common factors cancel in p = e / sum.
#         Hardware exp2: 1 ulp = 6e-8 relative.  Sum over <= a few hundred rows of p * v in fp32: <~ sqrt(rows) *
#         6e-8 * |v|max.  Together a few 1e-6 at |o| ~ 1; observed <= 1.5e-6.  The bound leaves a factor of ~6.
TOL = {"bf16": (2e-2, 1e-2),
       "f32": (1e-5, 1e-5)}


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def make_cache(wl: workload.Workload, ht: np.ndarray, device="cuda") -> ssd.Cache:
    cfg = make_config(wl.L, wl.B, wl.H, wl.d, wl.dtype, wl.W, wl.S, wl.M, wl.R, wl.C,
                      0.0 if wl.softmax_scale is None else wl.softmax_scale, int(wl.alg2))
    if wl.head_budget is not None:
        return ssd.Cache(cfg, ht, device=device, head_budget=np.asarray(wl.head_budget, np.int32))
    return ssd.Cache(cfg, ht, device=device, window=wl.W_layers, budget=wl.M_layers)


def heavy_cap(wl: workload.Workload, ht: np.ndarray, layer: int) -> int:
    """Slots of the heavy region of a layer's semantic units (where their row buffer starts): the layer's M,
    or the largest M_h of its semantic heads when budgets are per head."""
    if wl.head_budget is None:
        return wl.M_of(layer)
    sem = [int(wl.head_budget[layer][h]) for h in range(wl.H) if ht[layer, h] == workload.SEMANTIC]
    return max(sem) if sem else wl.M


def flat_index(wl: workload.Workload, units: Sequence[Tuple[int, int, int]]) -> torch.Tensor:
    return torch.tensor([(l * wl.B + b) * wl.H + h for (l, b, h) in units], dtype=torch.long)


def sample_units(wl: workload.Workload, ht: np.ndarray, k: int, seed: int = 0) -> List[Tuple[int, int, int]]:
    """k units, half spatial and half semantic where both exist, always including the corners."""
    r = np.random.default_rng(seed)
    total = wl.L * wl.B * wl.H
    if k >= total:
        return [(l, b, h) for l in range(wl.L) for b in range(wl.B) for h in range(wl.H)]
    picks = {(0, 0, 0), (wl.L - 1, wl.B - 1, wl.H - 1)}
    want = {0: k // 2, 1: k - k // 2}
    for t in (0, 1):
        cand = np.argwhere(ht == t)
        if len(cand) == 0:
            continue
        for _ in range(want[t]):
            l, h = cand[r.integers(len(cand))]
            picks.add((int(l), int(r.integers(wl.B)), int(h)))
    return sorted(picks)


def gpu_decode(wl: workload.Workload, data: Dict[str, torch.Tensor], ht: np.ndarray, schedule: np.ndarray,
               units: Sequence[Tuple[int, int, int]], layers_per_call: Optional[int] = None,
               export_steps: Optional[Sequence[int]] = None, p_end: Optional[int] = None,
               cache: Optional[ssd.Cache] = None, p_begin: int = 0, accumulate: bool = True, fused: bool = False,
               rope: int = 0, shape: Optional[Tuple[int, int, int]] = None, split: int = 0, shadow: bool = True):
    """Decode positions [p_begin, p_end) on the GPU.  Returns
         outs   float32 numpy [steps, len(units), d]  outputs of the sampled units
         exports {step: {"pre": (pos, score) or None, "post": (pos, score)}} numpy [len(layers), B, H, slots]
         cache
    `export_steps`: steps at which the index tables of the sampled units' layers are exported, both
    before the compression of that step (if one is due) and after it (module docstring: how "before" is
    obtained on the fused path; `shadow=False` skips that).
    `rope`: 0, or the element pairing with which the fused step rotates q and k on the way in (fused only).
    `shape`: launch-shape override (ch, wpb, new_rows) of the cache.
    `split`: > 0: the fused step through ssd_decode_step_split on that many streams, forked at the first call
    of a token and joined at its last."""
    dev = data["q"].device
    p_end = wl.n_total if p_end is None else p_end
    cache = make_cache(wl, ht, dev) if cache is None else cache
    if shape is not None:
        cache.set_launch_shape(*shape)
    lpc = wl.L if layers_per_call is None else layers_per_call
    out = torch.empty((wl.L, wl.B, wl.H, wl.d), dtype=wl.torch_dtype, device=dev)
    idx = flat_index(wl, units).to(dev)
    steps = p_end - p_begin
    outs = torch.empty((steps, len(units), wl.d), dtype=torch.float32, device=dev)
    export_steps = set(export_steps or [])
    layers = sorted(set(l for (l, _, _) in units))
    exports = {}
    if rope:
        assert fused
        cos_t, sin_t = (torch.from_numpy(t).to(dev) for t in workload.rope_tables(wl.n_total, wl.d))
    streams = None
    if split:
        assert fused
        main = torch.cuda.current_stream()
        streams = ssd.stream_array([main] + [torch.cuda.Stream() for _ in range(split - 1)])      # default priority
    calls = [(lb, min(wl.L, lb + lpc)) for lb in range(0, wl.L, lpc)]

    # the second cache of the fused path's own-score check: same calls, host side only
    twin = None
    if fused and shadow and any(schedule[p] for p in export_steps if p_begin <= p < p_end):
        twin = make_cache(wl, ht, dev)
        if shape is not None:
            twin.set_launch_shape(*shape)
        if p_begin > 0:
            raise AssertionError("the fused path's own-score check needs a decode that starts at position 0")
        assert ssd.lib.ssd_cache_set_launch(twin.handle, 0) == 0

    def export_layers(c):
        pos, sc = [], []
        for l in layers:
            p_, _, s_ = c.export(l)
            pos.append(p_.cpu().numpy()); sc.append(s_.cpu().numpy())
        return np.stack(pos), np.stack(sc)

    def fused_step(c, p, q, k, v, o, compress):
        for ci, (lb, le) in enumerate(calls):
            sync = (ssd.SSD_SPLIT_FORK if ci == 0 else 0) | (ssd.SSD_SPLIT_JOIN if ci == len(calls) - 1 else 0)
            if rope and split:
                ssd.ssd_decode_step_split_rope(c, lb, le, q[lb:le], k[lb:le], v[lb:le], o[lb:le], cos_t[p], sin_t[p], rope,
                                               streams, sync, accumulate, compress)
            elif rope:
                ssd.ssd_decode_step_rope(c, lb, le, q[lb:le], k[lb:le], v[lb:le], o[lb:le], cos_t[p], sin_t[p], rope,
                                         accumulate, compress)
            elif split:
                ssd.ssd_decode_step_split(c, lb, le, q[lb:le], k[lb:le], v[lb:le], o[lb:le], streams, sync, accumulate, compress)
            else:
                ssd.ssd_decode_step(c, lb, le, q[lb:le], k[lb:le], v[lb:le], o[lb:le], accumulate, compress)

    for p in range(p_begin, p_end):
        q, k, v = data["q"][p], data["k"][p], data["v"][p]
        rec = {"pre": None, "post": None}
        comp = bool(schedule[p])
        if fused:
            if twin is not None:
                if p in export_steps and comp:
                    # same memory, same counters, same kernel up to and including the score update, no selection
                    assert twin.mem.data_ptr() % 256 == 0 and cache.mem.data_ptr() % 256 == 0 and twin.mem.numel() == cache.mem.numel()
                    twin.mem.copy_(cache.mem)
                    assert ssd.lib.ssd_cache_set_launch(twin.handle, 1) == 0
                    fused_step(twin, p, q, k, v, torch.empty_like(out), False)
                    rec["pre"] = export_layers(twin)
                    assert ssd.lib.ssd_cache_set_launch(twin.handle, 0) == 0
                    for (lb, le) in calls:
                        ssd.ssd_compress_kv(twin, lb, le)       # counters only
                else:
                    fused_step(twin, p, q, k, v, out, comp)     # counters only
            fused_step(cache, p, q, k, v, out, comp)
        else:
            for (lb, le) in calls:
                ssd.ssd_append_token(cache, lb, le, k[lb:le], v[lb:le])
                ssd.ssd_decode_attn(cache, lb, le, q[lb:le], out[lb:le], accumulate)
        outs[p - p_begin] = out.view(-1, wl.d)[idx].float()
        if not fused:
            if p in export_steps and comp:
                rec["pre"] = export_layers(cache)
            if comp:
                for (lb, le) in calls:
                    ssd.ssd_compress_kv(cache, lb, le)
        if p in export_steps:
            rec["post"] = export_layers(cache)
            exports[p] = rec
    torch.cuda.synchronize()
    if twin is not None:
        for l in range(wl.L):
            assert twin.layer_state(l) == cache.layer_state(l), "the second cache fell out of step"
    return outs.cpu().numpy(), exports, cache


def rotate_rows(wl: workload.Workload, x: torch.Tensor, rope: int) -> torch.Tensor:
    """Oracle-side rotary embedding of x [n_total, ..., d] (row p at position p): the oracle's definition in
    double, rounded to the workload dtype the way the cache holds it."""
    cos_t, sin_t = workload.rope_tables(wl.n_total, wl.d)
    xf = x.to(torch.float32).cpu().numpy()
    out = np.stack([oracle.rope(xf[p], cos_t[p], sin_t[p], rope) for p in range(xf.shape[0])])
    return torch.from_numpy(out).to(wl.torch_dtype)


def oracle_unit(wl: workload.Workload, data: Dict[str, torch.Tensor], ht: np.ndarray, schedule: np.ndarray,
                unit: Tuple[int, int, int], p_end: Optional[int] = None, layer: Optional[int] = None,
                head: Optional[int] = None, accumulate: bool = True):
    """Oracle decode of one unit: (o [steps,d], heavy_log, gap_log, Unit).  `unit` indexes `data` and `ht`;
    `layer` and `head` are the unit's layer and head in the workload where those are slices (they select the
    W and M that apply to it)."""
    l, b, h = unit
    lw = l if layer is None else layer
    hw = h if head is None else head
    q, K, V = workload.unit_arrays(data, l, b, h)
    u = oracle.Unit(ht[l, h] == workload.SEMANTIC, wl.W_of(lw, hw), wl.S, wl.M_of(lw, hw), wl.R, wl.C, buffered_spatial=wl.alg2)
    o, hl, gl = u.run(q, K, V, wl.scale, schedule, p_end=p_end, accumulate=accumulate, log=True)
    return o, hl, gl, u


def check_outputs(gpu: np.ndarray, ref: np.ndarray, dtype: str, what: str):
    atol, rtol = TOL[dtype]
    err = np.abs(gpu - ref)
    bound = atol + rtol * np.abs(ref)
    bad = err > bound
    assert not bad.any(), "%s: %d of %d outputs outside %g + %g|ref| (max abs err %.3e at %s)" % (
        what, int(bad.sum()), bad.size, atol, rtol, float(err.max()), np.unravel_index(err.argmax(), err.shape))
    return float(err.max())


def spatial_positions(wl: workload.Workload, n: int, n_c: Optional[int] = None, layer: int = 0, head: Optional[int] = None) -> List[int]:
    """Closed form of a spatial head's retained set after n tokens; under Algorithm 2 the window is cut at
    n_c, the token count at the last compression."""
    ref = n if not wl.alg2 else n_c
    return sorted(set(range(min(wl.S, n))) | set(range(max(wl.S, ref - wl.W_of(layer, head)), n)))


def compare_unit_sets(wl, ht, unit, layer_index, exports, heavy_log, gap_log, schedule, p_begin: int = 0, margin: float = GAP_MARGIN):
    """Exact comparison of the exported index tables of one unit with the oracle's log (row p - p_begin = step
    p) at every exported step.  Returns None, or -- for a heavy set that differs because of a permitted near-tie
    -- the pair (s, p): s the compression step whose oracle margin excuses it, p the exported step at which the
    difference was seen.  A difference with no near-tie between the last agreeing export and p fails."""
    l, b, h = unit
    sem = ht[l, h] == workload.SEMANTIC
    M = heavy_cap(wl, ht, l)
    agreed = p_begin - 1                  # last exported step at which the heavy sets agreed
    for p in sorted(exports):
        pos, score = exports[p]["post"]
        row = pos[layer_index, b, h]
        got = sorted(int(x) for x in row if x >= 0)
        n = p + 1
        if not sem:
            n_c = max([s + 1 for s in range(p + 1) if schedule[s]], default=0)
            assert got == spatial_positions(wl, n, n_c, l, h), ("spatial set", unit, p)
            continue
        heavy_gpu = sorted(int(x) for x in row[:M] if x >= 0)
        staged_gpu = sorted(int(x) for x in row[M:] if x >= 0)
        heavy_ref = [int(x) for x in heavy_log[p - p_begin] if x >= 0]
        if heavy_gpu != heavy_ref:
            # allowed only if a cut since the last agreeing export was a near-tie in the oracle
            near = [s for s in range(agreed + 1, p + 1) if schedule[s] and 0 <= gap_log[s - p_begin] <= margin]
            assert near, ("heavy set differs above the tie margin", unit, p, heavy_gpu, heavy_ref)
            return near[0], p
        agreed = p
        # staged = the tokens appended since the last compression plus the R protected ones
        last = max([s for s in range(p + 1) if schedule[s]], default=-1)
        if last >= 0:
            want = list(range(max(0, last + 1 - wl.R), last + 1)) + list(range(last + 1, n))
            # tokens that a compression before any token became a candidate left in place
            want = sorted(set(want) - set(heavy_ref))
        else:
            want = list(range(n))
        assert staged_gpu == want, ("row buffer", unit, p, staged_gpu, want)
    return None


def check_selection_on_own_scores(wl, ht, unit, layer_index, exports):
    """At every exported step with a compression, selecting on the GPU's own pre-compression scores with the
    oracle's selection routine must give the GPU's post-compression heavy set.  Returns the steps checked."""
    l, b, h = unit
    if ht[l, h] != workload.SEMANTIC:
        return []
    checked = []
    for p in sorted(exports):
        if exports[p]["pre"] is None:
            continue
        pos0, sc0 = exports[p]["pre"]
        pos1, sc1 = exports[p]["post"]
        row_p, row_s = pos0[layer_index, b, h], sc0[layer_index, b, h]
        valid = row_p >= 0
        cand_pos = row_p[valid]
        cand_sc = row_s[valid]
        newest = np.sort(cand_pos)[len(cand_pos) - min(wl.R, len(cand_pos)):] if wl.R > 0 else np.zeros(0, np.int32)
        is_cand = ~np.isin(cand_pos, newest)
        keep, _ = oracle.top_m(cand_sc[is_cand], cand_pos[is_cand], wl.M_of(l, h))
        want = sorted(int(x) for x in cand_pos[is_cand][keep])
        got = sorted(int(x) for x in pos1[layer_index, b, h][: heavy_cap(wl, ht, l)] if x >= 0)
        assert got == want, ("selection on the GPU's own scores", unit, p)
        # scores travel with their tokens, bit for bit
        after = {int(pp): float(ss) for pp, ss in zip(pos1[layer_index, b, h], sc1[layer_index, b, h]) if pp >= 0}
        before = {int(pp): float(ss) for pp, ss in zip(row_p, row_s) if pp >= 0}
        for pp, ss in after.items():
            assert before[pp] == ss, ("score moved with token", unit, p, pp)
        checked.append(p)
    return checked


def verify_near_tie(wl, data, ht, schedule, unit, s, fused, lpc=None, rope=0, shape=None, accumulate=True):
    """The duty that comes with a near-tie excuse: decode again up to and including compression step s, on the
    same path, exporting the sampled unit's layer before and after that cut, and require that the GPU's selection
    there is the oracle's selection routine applied to the GPU's own scores."""
    l, b, h = unit
    _, ex, _ = gpu_decode(wl, data, ht, schedule, [unit], layers_per_call=lpc, export_steps=[s], p_end=s + 1,
                          accumulate=accumulate, fused=fused, rope=rope, shape=shape)
    assert ex[s]["pre"] is not None, ("no tables before the cut", unit, s)
    assert check_selection_on_own_scores(wl, ht, unit, 0, ex) == [s], ("own-score check at the near-tie", unit, s)


def near_tie_cap(n_units: int) -> int:
    """Units that may be excused as near-ties in one comparison (none has been seen so far)."""
    return max(1, n_units // 10)


def settle_near_tie(wl, data, ht, schedule, unit, layer_index, exports, s, fused, **kw):
    """Own-score check at near-tie step s: from this run's tables if step s was exported with its "before"
    tables, else by decoding again up to s."""
    if s in exports and exports[s]["pre"] is not None:
        assert check_selection_on_own_scores(wl, ht, unit, layer_index, {s: exports[s]}) == [s], ("own-score check at the near-tie", unit, s)
    else:
        verify_near_tie(wl, data, ht, schedule, unit, s, fused, **kw)
