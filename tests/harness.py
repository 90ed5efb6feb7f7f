"""Shared driver for the GPU parity tests: runs a workload through the C-ABI library step by step and
compares sampled (layer, sequence, head) units with the CPU oracle.

Index sets are compared exactly.  Because GPU and CPU exponentials differ in the last bits, a top-M cut
whose oracle margin is below GAP_MARGIN (relative) may legitimately fall the other way; such a unit is
counted as a near-tie, must then agree with a selection done on the GPU's own exported scores, and is not
compared further (its later state legitimately differs)."""
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

TOL = {"bf16": (2e-2, 1e-2),     # |gpu - ref| <= 2e-2 + 1e-2 |ref|   (target stated for the bf16 path)
       "f32": (2e-4, 2e-4)}      # fp32 path: fp32 accumulation over <= a few hundred rows plus the hardware exp2


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def make_cache(wl: workload.Workload, ht: np.ndarray, device="cuda") -> ssd.Cache:
    cfg = make_config(wl.L, wl.B, wl.H, wl.d, wl.dtype, wl.W, wl.S, wl.M, wl.R, wl.C, 0.0, int(wl.alg2))
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
               rope: int = 0):
    """Decode positions [p_begin, p_end) on the GPU.  Returns
         outs   float32 numpy [steps, len(units), d]  outputs of the sampled units
         exports {step: {"pre": (pos, score) or None, "post": (pos, score)}} numpy [len(layers), B, H, slots]
         cache
    `export_steps`: steps at which the index tables of the sampled units' layers are exported, both
    before the compression of that step (if one is due) and after it.
    `rope`: 0, or the element pairing with which the fused step rotates q and k on the way in (fused only)."""
    dev = data["q"].device
    p_end = wl.n_total if p_end is None else p_end
    cache = make_cache(wl, ht, dev) if cache is None else cache
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

    def export_layers():
        pos, sc = [], []
        for l in layers:
            p_, _, s_ = cache.export(l)
            pos.append(p_.cpu().numpy()); sc.append(s_.cpu().numpy())
        return np.stack(pos), np.stack(sc)

    for p in range(p_begin, p_end):
        q, k, v = data["q"][p], data["k"][p], data["v"][p]
        # the fused entry point does append + attend + compress in one launch (no look at the tables between
        # attention and compression is possible then: "pre" exports exist only on the three-call path)
        fuse_now = fused
        for lb in range(0, wl.L, lpc):
            le = min(wl.L, lb + lpc)
            if fuse_now and rope:
                ssd.ssd_decode_step_rope(cache, lb, le, q[lb:le], k[lb:le], v[lb:le], out[lb:le], cos_t[p], sin_t[p], rope,
                                         accumulate, bool(schedule[p]))
            elif fuse_now:
                ssd.ssd_decode_step(cache, lb, le, q[lb:le], k[lb:le], v[lb:le], out[lb:le], accumulate, bool(schedule[p]))
            else:
                ssd.ssd_append_token(cache, lb, le, k[lb:le], v[lb:le])
                ssd.ssd_decode_attn(cache, lb, le, q[lb:le], out[lb:le], accumulate)
        outs[p - p_begin] = out.view(-1, wl.d)[idx].float()
        rec = {"pre": None, "post": None}
        if p in export_steps and schedule[p] and not fuse_now:
            rec["pre"] = export_layers()
        if schedule[p] and not fuse_now:
            for lb in range(0, wl.L, lpc):
                le = min(wl.L, lb + lpc)
                ssd.ssd_compress_kv(cache, lb, le)
        if p in export_steps:
            rec["post"] = export_layers()
            exports[p] = rec
    torch.cuda.synchronize()
    return outs.cpu().numpy(), exports, cache


def rotate_rows(wl: workload.Workload, x: torch.Tensor, rope: int) -> torch.Tensor:
    """Oracle-side rotary embedding of x [n_total, ..., d] (row p at position p), rounded to the workload dtype
    the way the cache holds it.  bf16: the float form of the oracle's routine (the rounding that follows is a
    quantisation both sides must take from the same float); f32: the definition in double."""
    cos_t, sin_t = workload.rope_tables(wl.n_total, wl.d)
    xf = x.to(torch.float32).cpu().numpy()
    out = np.stack([oracle.rope(xf[p], cos_t[p], sin_t[p], rope, single=(wl.dtype == "bf16")) for p in range(xf.shape[0])])
    return torch.from_numpy(out).to(wl.torch_dtype)


def oracle_unit(wl: workload.Workload, data: Dict[str, torch.Tensor], ht: np.ndarray, schedule: np.ndarray,
                unit: Tuple[int, int, int], p_end: Optional[int] = None, layer: Optional[int] = None,
                head: Optional[int] = None):
    """Oracle decode of one unit: (o [steps,d], heavy_log, gap_log, Unit).  `unit` indexes `data` and `ht`;
    `layer` and `head` are the unit's layer and head in the workload where those are slices (they select the
    W and M that apply to it)."""
    l, b, h = unit
    lw = l if layer is None else layer
    hw = h if head is None else head
    q, K, V = workload.unit_arrays(data, l, b, h)
    u = oracle.Unit(ht[l, h] == workload.SEMANTIC, wl.W_of(lw, hw), wl.S, wl.M_of(lw, hw), wl.R, wl.C, buffered_spatial=wl.alg2)
    o, hl, gl = u.run(q, K, V, wl.scale, schedule, p_end=p_end, log=True)
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


def compare_unit_sets(wl, ht, unit, layer_index, exports, heavy_log, gap_log, schedule):
    """Exact comparison of the exported index tables of one unit with the oracle's log at every exported
    step.  Returns the first step at which a permitted near-tie divergence was seen, or None."""
    l, b, h = unit
    sem = ht[l, h] == workload.SEMANTIC
    M = heavy_cap(wl, ht, l)
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
        heavy_ref = [int(x) for x in heavy_log[p] if x >= 0]
        if heavy_gpu != heavy_ref:
            # allowed only if some cut so far was a near-tie in the oracle
            near = [s for s in range(p + 1) if 0 <= gap_log[s] <= GAP_MARGIN]
            assert near, ("heavy set differs above the tie margin", unit, p, heavy_gpu, heavy_ref)
            return near[0]
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
    """T3: at every exported step with a compression, selecting on the GPU's own pre-compression scores
    with the oracle's selection routine must give the GPU's post-compression heavy set."""
    l, b, h = unit
    if ht[l, h] != workload.SEMANTIC:
        return 0
    n_checked = 0
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
        n_checked += 1
    return n_checked
