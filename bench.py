#!/usr/bin/env python3
"""Benchmark of the SSD compressed decode-attention path on one MI355X.

A "step" is one generated visual token for the whole batch: for every layer, append the token's K/V,
attend over the compressed cache (with score accumulation) and compress -- one library call per layer, as a
model whose layers depend on each other has to issue it -- on synthetic Janus-Pro-shaped inputs that are
already resident in HBM.  The cache is first filled by decoding the prompt and the earlier part of the image
(untimed), so the timed steps run at the end of the raster decode with every window and budget full.

Schedule of the headline (--streams N, default 2): ssd_decode_step_split -- the batch dealt to N streams,
forked at a token's first layer and joined at its last, every part's layers in order on that part's stream
(sequences are independent), so that one part's launch ramps up and drains while another's is streaming.
--streams 1 is ssd_decode_step on one stream; that figure is always reported beside the headline (`one_stream`).

Prints ONE JSON line:
  value            visual tokens/s = prompts x steps / wall time of the timed steps
  roofline         the dominant kernel (step_kernel): algorithmic bytes of a token's launches / the time from the
                   first launch's start to the last one's end (HIP events on the stream that forks and joins),
                   against the 8 TB/s HBM peak.  With one stream that is bytes per launch / launch duration.
  one_stream       the same steps through ssd_decode_step on one stream, with its own roofline
  all_layers_one_launch   the same steps with all layers handed to the library in one call (possible only
                   because the synthetic queries of all layers exist up front: an upper bound)
  stream_ceiling   a plain read of as many units of as many bytes per launch, no arithmetic, without and with the
                   least a step must store: what the memory system allows a launch of this shape, on one stream
                   and (headline on several streams) dealt to the streams as the headline's launches are
  paper_head_mix   the same shape with the head mix of the paper's own settings (few long semantic heads beside many
                   short spatial ones), on the headline's schedule and on one stream
  dense_baseline   the same steps through the full-cache decode kernel
  cpu_baseline     the CPU oracle timed on a sample of (layer, sequence, head) units
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

PROFILES = os.path.join(ROOT, "profiles")


def library_source_digest():
    """sha256 over the library's sources (include/*.h, csrc/*.h, csrc/*.hip, in sorted order): names the build a
    counter measurement was taken on."""
    import glob
    import hashlib
    h = hashlib.sha256()
    files = sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))) + \
        sorted(glob.glob(os.path.join(ROOT, "paper_2510_18716_amd", "csrc", "*.h"))) + \
        sorted(glob.glob(os.path.join(ROOT, "paper_2510_18716_amd", "csrc", "*.hip")))
    for f in files:
        h.update(os.path.basename(f).encode() + b"\0" + open(f, "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(workload_name, entry_point, streams, layers_per_call):
    """HBM bytes of one step_kernel launch as counted by rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), from the
    `traffic-record:` lines of the summaries under profiles/.  A record counts only if it was taken on this very
    build of the library (source digest) and on this workload and schedule; otherwise None."""
    import glob
    digest = library_source_digest()
    for f in sorted(glob.glob(os.path.join(PROFILES, "*.md"))):
        for line in open(f):
            if not line.startswith("traffic-record:"):
                continue
            try:
                r = json.loads(line[len("traffic-record:"):])
            except ValueError:
                continue
            if (r.get("workload"), r.get("entry_point"), r.get("streams"), r.get("layers_per_call"), r.get("library_source_digest")) == \
                    (workload_name, entry_point, streams, layers_per_call, digest):
                return {"bytes_per_launch": r["fetch_bytes_per_launch"] + r["write_bytes_per_launch"],
                        "fetch_bytes_per_launch": r["fetch_bytes_per_launch"], "write_bytes_per_launch": r["write_bytes_per_launch"],
                        "source": os.path.relpath(f, ROOT)}
    return None


def row_bytes(wl):
    return wl.d * (2 if wl.dtype == "bf16" else 4)


def algorithmic_bytes_attend(wl, ht, layers, state):
    """Bytes one attention launch over `layers` must move: K and V rows of every retained token, q in,
    output out, and the score read-modify-write of semantic heads."""
    n, m, c = state
    row = row_bytes(wl)
    # Algorithm 2: a spatial head also reads the tokens appended since the last compression (c - R of them)
    total = 0
    for l in layers:
        for h in range(wl.H) if wl.head_budget is not None else (None,):     # budgets per head: head by head
            heads = 1 if h is not None else None
            if h is None or ht[l, h] == 0:
                rows_sp = min(n, wl.S + wl.W_of(l, h) + (max(c - wl.R, 0) if wl.alg2 else 0))
                hs = int((ht[l] == 0).sum()) if heads is None else 1
                total += wl.B * hs * (rows_sp * 2 * row + 2 * row)
            if h is None or ht[l, h] == 1:
                rows_se = min(m, wl.M_of(l, h)) + c
                hm = int((ht[l] == 1).sum()) if heads is None else 1
                total += wl.B * hm * (rows_se * 2 * row + rows_se * 8 + 2 * row)
    return total


def algorithmic_bytes_append(wl, ht, layers):
    """Bytes the append moves: the new K and V rows read and written, plus position and score of a semantic head."""
    row = row_bytes(wl)
    total = 0
    for l in layers:
        hm = int((ht[l] == 1).sum())
        total += wl.B * wl.H * 4 * row + wl.B * hm * 8
    return total


def sweep5(args, dev):
    """Configuration 5: B = 512 sequences, 32 heads, d = 128; spatial fraction in {25, 50, 75} %, W and M in
    {32, 64, 128}.  Steady-state fused per-layer launches on `--layers` layers (default 4; a per-layer launch has
    the full configuration's shape whatever the layer count), inputs plain Gaussians (timing does not depend on
    the values).  Each point on one stream (ssd_decode_step) and, unless --streams 1, in the headline's schedule
    (ssd_decode_step_split on --streams streams, default 2, every part running free)."""
    import numpy as np
    import torch

    import paper_2510_18716_amd as ssd
    import workload
    from paper_2510_18716_amd.binding import make_config
    L = args.layers or 4
    rows = []
    base = workload.config(5).replace(L=L, plain=True, grid_h=8)          # 64 + 192 tokens: every window fills
    data = workload.generate(base, device=dev)
    K_steps = 40
    n_split = 2 if args.streams == 0 else max(1, min(args.streams, ssd.SSD_MAX_SPLIT))
    side = [torch.cuda.Stream() for _ in range(n_split - 1)]                     # default priority
    stream_arr = ssd.stream_array([torch.cuda.current_stream()] + side)
    for frac in (0.25, 0.5, 0.75):
        for W in (32, 64, 128):
            for M in (32, 64, 128):
                wl = base.replace(spatial_frac=frac, W=W, M=M)
                ht = workload.head_map(wl)
                cache = ssd.Cache(make_config(wl.L, wl.B, wl.H, wl.d, wl.dtype, W, wl.S, M, wl.R, wl.C), ht, device=dev)
                out = torch.empty((wl.L, wl.B, wl.H, wl.d), dtype=wl.torch_dtype, device=dev)
                stride_l = wl.B * wl.H * wl.d * 2
                qb, kb, vb, ob = data["q"].data_ptr(), data["k"].data_ptr(), data["v"].data_ptr(), out.data_ptr()
                stream = torch.cuda.current_stream().cuda_stream

                def timed(ns):
                    def step(p):
                        for l in range(wl.L):
                            o = (p * wl.L + l) * stride_l
                            if ns > 1:
                                rc = ssd.lib.ssd_decode_step_split(cache.handle, l, l + 1, qb + o, kb + o, vb + o, ob + l * stride_l, 1, 1,
                                                                   stream_arr, ns, 0)
                            else:
                                rc = ssd.lib.ssd_decode_step(cache.handle, l, l + 1, qb + o, kb + o, vb + o, ob + l * stride_l, 1, 1, stream)
                            assert rc == 0, ssd.ssd_last_error()
                    cache.reset()
                    p_timed = wl.n_total - K_steps
                    for p in range(p_timed):
                        step(p)
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    for p in range(p_timed, wl.n_total):
                        step(p)
                    torch.cuda.synchronize()
                    return (time.perf_counter() - t0) / K_steps
                dt = timed(1)
                n_, m_, c_, _ = cache.layer_state(0)
                gb = (algorithmic_bytes_attend(wl, ht, range(wl.L), (n_, m_, c_ + 1)) + algorithmic_bytes_append(wl, ht, range(wl.L))) / 1e9
                row = {"spatial_frac": frac, "W": W, "M": M, "ms_per_layer": dt / wl.L * 1e3, "GB_per_layer": gb / wl.L,
                       "GBps": gb / dt, "frac_of_hbm_peak": gb / dt / HBM_PEAK_GBS,
                       "tokens_per_s_at_30_layers": wl.prompts / (dt / wl.L * 30)}
                if n_split > 1:
                    dt2 = timed(n_split)
                    row["split"] = {"streams": n_split, "ms_per_layer": dt2 / wl.L * 1e3, "GBps": gb / dt2, "frac_of_hbm_peak": gb / dt2 / HBM_PEAK_GBS,
                                    "tokens_per_s_at_30_layers": wl.prompts / (dt2 / wl.L * 30)}
                rows.append(row)
                del cache
    print(json.dumps({"metric": "visual tokens/sec per GPU (compressed decode attn, all layers)", "unit": "tokens/s",
                      "config": {"workload": "cfg5-large sweep", "sequences": base.B, "heads": base.H, "head_dim": base.d,
                                 "layers_timed": L, "launches": "ssd_decode_step, one per layer; 'split': ssd_decode_step_split, one call per layer"},
                      "sweep": rows}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=3, help="workload: index into the benchmark configurations (1-based)")
    ap.add_argument("--layers-per-call", type=int, default=1,
                    help="layers handed to each library call for the headline figure (1 = as a real model would)")
    ap.add_argument("--prompts", type=int, default=0, help="override the number of prompts (0 = the configuration's)")
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers (0 = the configuration's)")
    ap.add_argument("--window", type=int, default=0, help="override W of the configuration (0 = the configuration's)")
    ap.add_argument("--budget", type=int, default=0, help="override M of the configuration (0 = the configuration's)")
    ap.add_argument("--spatial-heads", type=int, default=-1,
                    help="override the number of spatial heads per layer (-1 = the configuration's half); the paper's tau = 0.8 leaves "
                         "about 2 of 32 heads semantic on the 7B model (Table 6)")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-prefill", action="store_true")
    ap.add_argument("--no-ceiling", action="store_true")
    ap.add_argument("--no-roofline", action="store_true")
    ap.add_argument("--no-all-layers", action="store_true")
    ap.add_argument("--streams", type=int, default=0,
                    help="streams the batch is dealt to for the headline (ssd_decode_step_split); 1 = ssd_decode_step on one stream; "
                         "0 = 2 if a layer has at least 2048 (sequence, head) units, else 1 (smaller launches are bound by their fixed "
                         "cost, and splitting them only adds launches)")
    ap.add_argument("--sync", choices=["run", "step"], default="run",
                    help="split schedule: 'step' forks at every token's first layer and joins at its last (a caller with one stream "
                         "of its own); 'run' lets the parts run free on their streams between host synchronisations (a caller "
                         "that runs its model on the parts of the batch in turn, each on its stream)")
    ap.add_argument("--input-layers", type=int, default=0,
                    help="generate the per-token inputs (q, k_new, v_new) for this many layers only and let layer l read those of layer "
                         "l mod this (0 = every layer its own).  For configurations whose inputs for all layers and all tokens would not fit "
                         "beside the cache (the large batch: 240 GB); the cache itself stays that of all layers")
    ap.add_argument("--no-head-mix", action="store_true",
                    help="skip the 'paper_head_mix' leg: the same shape with the head mix of the paper's own settings (W = 32, M = 128, 2 "
                         "semantic heads of 32; Sec. 4.1, Table 6), timed on the headline's schedule and on one stream")
    ap.add_argument("--no-one-stream", action="store_true", help="skip the one-stream figure reported beside a split headline")
    ap.add_argument("--only", choices=["dense", "prefill", "ceiling"], default="",
                    help="run one of the side legs alone, without the decode measurement (for a profiler run of its own)")
    ap.add_argument("--counter-reference", action="store_true",
                    help="start with two launches of a plain copy kernel of exactly 1 GiB (ssd_bench_copy): the known traffic against "
                         "which the profiler's FETCH_SIZE / WRITE_SIZE readings of the same run are scaled")
    ap.add_argument("--tune", type=str, default="", help="ch,wpb[,new_rows] launch-shape override of the attention kernel (test hook)")
    ap.add_argument("--separate", action="store_true",
                    help="three launches per layer (append, attend, compress) instead of the fused ssd_decode_step")
    ap.add_argument("--cpu-units", type=int, default=4096)
    ap.add_argument("--grid-rows", type=int, default=0, help="profiling aid: shorten the image to this many grid rows (0 = full image)")
    ap.add_argument("--no-accumulate", action="store_true", help="experiment: attention without the running-score update")
    ap.add_argument("--sweep5", action="store_true",
                    help="large-batch sweep (configuration 5): spatial fraction x W x M at B = 512, one JSON line with a list")
    ap.add_argument("--head-budgets", type=str, default="",
                    help="LO,HI: head-wise allocation -- every head its own W_h / M_h, seeded uniform in [LO, HI]")
    ap.add_argument("--replicas", type=int, default=1,
                    help="decode this many copies of the cache side by side (every step runs on each in turn), so that a small "
                         "configuration's working set exceeds the 256 MB memory-side cache and its figure is an HBM figure")
    ap.add_argument("--rope", type=int, default=0,
                    help="1 / 2: time ssd_decode_step_rope (q and k rotated inside the step; pairs (i, i + d/2) / (2i, 2i+1))")
    ap.add_argument("--alg2", action="store_true",
                    help="row-buffer variant (Algorithm 2): both head types read a 24-token row buffer, compression every 24 tokens")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every (layer, sequence, head) unit is independent, so it "
              "shards over GPUs without communication, but nothing here drives a second GPU); --gpus %d is not supported" % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2510_18716_amd as ssd
    import workload
    from paper_2510_18716_amd.binding import make_config

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    if args.sweep5:
        return sweep5(args, dev)
    wl = workload.config(args.config)
    if args.prompts:
        wl = wl.replace(prompts=args.prompts)
    if args.layers:
        wl = wl.replace(L=args.layers, name=wl.name + "-L%d" % args.layers)
    if args.window or args.budget or args.spatial_heads >= 0:
        wl = wl.replace(W=args.window or wl.W, M=args.budget or wl.M,
                        spatial_frac=wl.spatial_frac if args.spatial_heads < 0 else args.spatial_heads / wl.H,
                        name=wl.name + "-W%d-M%d-sp%d" % (args.window or wl.W, args.budget or wl.M,
                                                        round(wl.spatial_frac * wl.H) if args.spatial_heads < 0 else args.spatial_heads))
    if args.alg2:
        wl = wl.replace(alg2=True, R=0, C=wl.grid_w, cadence=wl.grid_w, name=wl.name + "-alg2")
    if args.grid_rows:
        wl = wl.replace(grid_h=args.grid_rows, name=wl.name + "-rows%d" % args.grid_rows)
    accumulate = not args.no_accumulate
    ht = workload.head_map(wl)
    if args.head_budgets:
        lo, hi = (int(x) for x in args.head_budgets.split(","))
        rng = np.random.default_rng(wl.seed)
        hb = rng.integers(lo, hi + 1, (wl.L, wl.H))
        # W and M of the description become the largest budgets (what sizes the units and bounds the fill time)
        wl = wl.replace(head_budget=tuple(tuple(int(x) for x in r) for r in hb), W=int(hb.max()), M=int(hb.max()),
                        name=wl.name + "-heads%d-%d" % (lo, hi))
    K_steps, W_steps = args.steps, args.warmup
    assert K_steps >= 1 and W_steps >= 0
    # Timed steps are the last ones of a raster decode, when every window and budget is full.  One decode has
    # room for max_k of them after the fill and the warm-up; more are taken from further decodes of the same image.
    # (every decode starts with hundreds of untimed steps that fill the cache; the W warm-up steps are the last
    # of them, so a W larger than the image leaves room for is as good as the largest that fits)
    W_steps = min(W_steps, wl.n_total - wl.S - wl.W - 4)
    max_k = wl.n_total - wl.S - wl.W - 3 - W_steps
    assert max_k >= 1, "the workload is too short to time a step in steady state"
    passes = [max_k] * (K_steps // max_k) + ([K_steps % max_k] if K_steps % max_k else [])
    fused = not args.separate
    want_streams = args.streams if args.streams > 0 else (2 if wl.B * wl.H >= 2048 else 1)
    n_streams = max(1, min(want_streams, ssd.SSD_MAX_SPLIT)) if fused else 1

    t0 = time.time()
    Ld = wl.L if not args.input_layers else min(wl.L, args.input_layers)       # layers that have inputs of their own
    assert Ld == wl.L or Ld % 2 == 0, "--input-layers: an even number (the head map alternates)"
    data = workload.generate(wl, device=dev, head_type=ht, layers=range(Ld))
    torch.cuda.synchronize()
    t_gen = time.time() - t0
    sched = workload.compress_schedule(wl)
    cfg = make_config(wl.L, wl.B, wl.H, wl.d, wl.dtype, wl.W, wl.S, wl.M, wl.R, wl.C, 0.0, int(wl.alg2))
    caches = [ssd.Cache(cfg, ht, device=dev, head_budget=None if wl.head_budget is None else np.asarray(wl.head_budget, np.int32))
              for _ in range(max(1, args.replicas))]
    cache = caches[0]
    R_rep = len(caches)
    if args.tune:
        t = [int(x) for x in args.tune.split(",")] + [0]
        for c_i in caches:
            c_i.set_launch_shape(t[0], t[1], t[2])
    side_streams = [torch.cuda.Stream() for _ in range(ssd.SSD_MAX_SPLIT - 1)]      # default priority
    out = torch.empty((wl.L, wl.B, wl.H, wl.d), dtype=wl.torch_dtype, device=dev)
    if args.rope:
        assert fused, "--rope times the fused step"
        rope_tabs = [torch.from_numpy(t).to(dev) for t in workload.rope_tables(wl.n_total, wl.d)]
        wl = wl.replace(name=wl.name + "-rope%d" % args.rope)
    p_timed = wl.n_total - passes[0]          # first timed position of the first (usually the only) decode

    def measure(lpc, with_events, ns):
        """Decode the whole sequence from an empty cache with `lpc` layers per call, the batch dealt to `ns`
        streams; time the last K_steps.  Returns wall seconds of the timed steps and, if asked, the mean
        HIP-event time per call."""
        calls = [(lb, min(wl.L, lb + lpc)) for lb in range(0, wl.L, lpc)]
        stream_arr = ssd.stream_array([torch.cuda.current_stream()] + side_streams[: ns - 1])
        FORK, JOIN = ssd.SSD_SPLIT_FORK, ssd.SSD_SPLIT_JOIN
        sync_step = args.sync == "step"          # else: the parts meet only at the host's device-wide synchronisations
        n_parts = cache.split_plan(lpc, ns)[1]                                  # launches per call: the library's cut of the batch

        # raw device addresses: a launch should cost the host a ctypes call, not four tensor slices
        stride_l = wl.B * wl.H * wl.d * (2 if wl.dtype == "bf16" else 4)
        stride_p = Ld * stride_l
        qb, kb, vb, ob = data["q"].data_ptr(), data["k"].data_ptr(), data["v"].data_ptr(), out.data_ptr()
        stream = torch.cuda.current_stream().cuda_stream
        L_ = ssd.lib
        acc_i = int(accumulate)
        if args.rope:
            cos_p, sin_p = rope_tabs[0].data_ptr(), rope_tabs[1].data_ptr()

        def step(p, ev=None, acct=None):
            comp = int(bool(sched[p]))
            if ev is not None and fused:
                ev[0].record()
            for c_i in caches:                      # every replica takes the step (one replica unless --replicas)
                step_one(c_i.handle, p, comp, ev, acct if c_i is cache else None)
            if ev is not None and fused:
                ev[1].record()

        def step_one(h, p, comp, ev, acct):
            for ci, (lb, le) in enumerate(calls):
                o = p * stride_p + (lb % Ld) * stride_l
                if fused:
                    if acct is not None:            # what this launch has to move, from the live counters
                        n_, m_, c_, _ = cache.layer_state(lb)
                        acct.append(algorithmic_bytes_attend(wl, ht, range(lb, le), (n_ + 1, m_, c_ + 1)) +
                                    algorithmic_bytes_append(wl, ht, range(lb, le)))
                    if args.rope and ns > 1:
                        rc = L_.ssd_decode_step_split_rope(h, lb, le, qb + o, kb + o, vb + o, ob + lb * stride_l, acc_i, comp,
                                                           cos_p + p * wl.d * 2, sin_p + p * wl.d * 2, args.rope, stream_arr, ns,
                                                           ((FORK if ci == 0 else 0) | (JOIN if ci == len(calls) - 1 else 0)) if sync_step else 0)
                    elif args.rope:
                        rc = L_.ssd_decode_step_rope(h, lb, le, qb + o, kb + o, vb + o, ob + lb * stride_l, acc_i, comp,
                                                     cos_p + p * wl.d * 2, sin_p + p * wl.d * 2, args.rope, stream)
                    elif ns > 1:
                        rc = L_.ssd_decode_step_split(h, lb, le, qb + o, kb + o, vb + o, ob + lb * stride_l, acc_i, comp, stream_arr, ns,
                                                      ((FORK if ci == 0 else 0) | (JOIN if ci == len(calls) - 1 else 0)) if sync_step else 0)
                    else:
                        rc = L_.ssd_decode_step(h, lb, le, qb + o, kb + o, vb + o, ob + lb * stride_l, acc_i, comp, stream)
                    assert rc == 0, ssd.ssd_last_error()
                    continue
                rc = L_.ssd_append_token(h, lb, le, kb + o, vb + o, stream)
                assert rc == 0, ssd.ssd_last_error()
                if acct is not None:
                    acct.append(algorithmic_bytes_attend(wl, ht, range(lb, le), cache.layer_state(lb)[:3]))
                if ev is not None:
                    ev[2 * ci].record()
                rc = L_.ssd_decode_attn(h, lb, le, qb + o, ob + lb * stride_l, acc_i, stream)
                assert rc == 0, ssd.ssd_last_error()
                if ev is not None:
                    ev[2 * ci + 1].record()
                if comp:
                    rc = L_.ssd_compress_kv(h, lb, le, None, None, None, 0, stream)
                    assert rc == 0, ssd.ssd_last_error()

        dt, whole = 0.0, None
        for k_i in passes:
            p_t = wl.n_total - k_i
            p_w = p_t - W_steps
            for c_i in caches:
                c_i.reset()
            for p in range(0, wl.n0):               # the prompt, through ordinary decode steps
                step(p)
            torch.cuda.synchronize()
            t_vis = time.perf_counter()
            for p in range(wl.n0, p_w):             # the earlier part of the image (fills every window and budget)
                step(p)
            torch.cuda.synchronize()
            for p in range(p_w, p_t):
                step(p)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for p in range(p_t, wl.n_total):
                step(p)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            dt += t1 - t0
            if whole is None:
                whole = t1 - t_vis                  # all N visual tokens, two intermediate synchronisations included

        # algorithmic bytes of the timed launches, from the counters each launch ran with (host-only replay)
        acct = []
        for c_i in caches:
            ssd.lib.ssd_cache_set_launch(c_i.handle, 0)
        for k_i in passes:
            for c_i in caches:
                c_i.reset()
            for p in range(0, wl.n_total):
                step(p, acct=acct if p >= wl.n_total - k_i else None)
        for c_i in caches:
            ssd.lib.ssd_cache_set_launch(c_i.handle, 1)
        bytes_launch = float(np.mean(acct))
        res = {"seconds": dt, "ms_per_step": dt / (K_steps * R_rep) * 1e3, "value": wl.prompts * K_steps * R_rep / dt,
               "whole_decode": {"visual_tokens": wl.N, "seconds": whole, "value": wl.prompts * wl.N * R_rep / whole, "unit": "tokens/s",
                                "note": "all %d visual tokens of the raster decode from the end of the prompt, cache filling up "
                                        "on the way" % wl.N},
               "launches_per_step": len(calls) * (n_parts if fused else 3), "bytes_per_call": bytes_launch,
               "algorithmic_GB_per_step": bytes_launch * len(calls) / 1e9}
        if not with_events:
            return res
        # second pass, same decode from an empty cache, with HIP events on the launch stream.  Fused: one
        # event pair around the back-to-back launches of a step (they are all the dominant kernel), so the
        # events themselves do not sit between launches.  Separate: a pair around each attention launch.
        n_ev = 2 if fused else 2 * len(calls)
        evs = []
        if fused and ns > 1 and not sync_step:
            # free-running parts: one start event (every stream is idle after the synchronisation), one end event per
            # stream behind its last launch; the span of a pass is the latest end
            span_ms = 0.0
            for k_i in passes:
                for c_i in caches:
                    c_i.reset()
                for p in range(0, wl.n_total - k_i):
                    step(p)
                torch.cuda.synchronize()
                e0 = torch.cuda.Event(enable_timing=True)
                ends = [torch.cuda.Event(enable_timing=True) for _ in range(ns)]
                e0.record()
                for p in range(wl.n_total - k_i, wl.n_total):
                    step(p)
                ends[0].record()
                for e_i, st_i in zip(ends[1:], side_streams):
                    e_i.record(st_i)
                torch.cuda.synchronize()
                span_ms += max(e0.elapsed_time(e_i) for e_i in ends)
            durs = [span_ms / (K_steps * len(calls) * R_rep)]
            passes_ev = []
        else:
            passes_ev = passes
        for k_i in passes_ev:
            for c_i in caches:
                c_i.reset()
            for p in range(0, wl.n_total - k_i):
                step(p)
            evs_i = [[torch.cuda.Event(enable_timing=True) for _ in range(n_ev)] for _ in range(k_i)]
            torch.cuda.synchronize()
            for i, p in enumerate(range(wl.n_total - k_i, wl.n_total)):
                step(p, ev=evs_i[i])
            torch.cuda.synchronize()
            evs += evs_i
        if fused and evs:
            durs = [e[0].elapsed_time(e[1]) / (len(calls) * R_rep) for e in evs]
        elif not fused:
            durs = [e[2 * ci].elapsed_time(e[2 * ci + 1]) for e in evs for ci in range(len(calls))]
        avg_ms = float(np.mean(durs))
        achieved = bytes_launch / 1e9 / (avg_ms / 1e3)
        entry = (("ssd_decode_step_split_rope" if ns > 1 else "ssd_decode_step_rope") if args.rope else
                 "ssd_decode_step_split" if ns > 1 else "ssd_decode_step") if fused else "ssd_decode_attn"
        traffic = measured_traffic(wl.name, entry, ns, lpc)
        res["roofline"] = {
            "bound": "hbm",
            "kernel": "step_kernel via %s%s" % (entry, " (append + attention + score update + top-M selection)" if fused else ""),
            "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": None if traffic is None else traffic["bytes_per_launch"], "traffic_record": traffic,
            "streams": ns, "launches_per_call": n_parts if fused else 1,
            "algorithmic_bytes_per_launch": bytes_launch / (n_parts if fused else 1),
            "algorithmic_bytes_per_call": bytes_launch, "avg_call_ms": avg_ms,
            "median_call_ms": float(np.median(durs)), "layers_per_call": lpc,
            "timer": ("HIP events: one before the first timed launch (all streams idle), one on every stream behind its last launch; the "
                      "latest end minus the start, divided by the %d steps x %d calls; launches of different parts overlap, so this "
                      "is the bytes of a call over its share of the span, not one kernel's duration" % (K_steps, len(calls)))
                     if (fused and ns > 1 and not sync_step)
                     else ("HIP events on the stream that forks and joins, around the %d calls (%d launches) of each step: first launch's start "
                      "to last launch's end, divided by %d; launches of different parts overlap, so this is bytes of a call over "
                      "its share of the span, not one kernel's duration" % (len(calls), len(calls) * n_parts, len(calls))) if (fused and ns > 1)
                     else ("HIP events on the launch stream around the %d back-to-back launches of each step, divided by %d"
                           % (len(calls), len(calls))) if fused else "HIP events on the launch stream around each launch"}
        return res

    lpc = max(1, min(wl.L, args.layers_per_call))
    if args.counter_reference:
        src = torch.ones(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(2):
            assert ssd.lib.ssd_bench_copy(dst.data_ptr(), src.data_ptr(), 1 << 30, torch.cuda.current_stream().cuda_stream) == 0
        torch.cuda.synchronize()
        assert torch.equal(dst[:4096], src[:4096]) and bool((dst[-4096:] == 1).all())
        del src, dst
    if args.only:
        head = None
        result = {"metric": "side leg '%s' alone" % args.only, "config": {"workload": wl.name, "layers": wl.L}}
        args.no_all_layers = args.no_one_stream = args.no_cpu = args.no_head_mix = True
        args.no_dense, args.no_prefill, args.no_ceiling = args.only != "dense", args.only != "prefill", args.only != "ceiling"
    else:
        head = measure(lpc, with_events=not args.no_roofline, ns=n_streams)
    if head is not None:
        entry = (("ssd_decode_step_split_rope" if n_streams > 1 else "ssd_decode_step_rope") if args.rope else
                 "ssd_decode_step_split" if n_streams > 1 else "ssd_decode_step") if fused \
            else "ssd_append_token, ssd_decode_attn, ssd_compress_kv"
        result = {
            "metric": "visual tokens/sec per GPU (compressed decode attn, all layers)",
            "value": head["value"], "unit": "tokens/s", "n_gpus": 1, "steps": K_steps, "warmup": args.warmup,
            "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": wl.dtype, "data": "synthetic",
            "config": {"workload": wl.name, "layers": wl.L, "prompts": wl.prompts, "sequences": wl.B, "heads": wl.H,
                       "head_dim": wl.d, "prompt_tokens": wl.n0, "visual_tokens": wl.N, "window": wl.W, "budget": wl.M,
                       "init_sink": wl.S, "recent": wl.R, "stage_cap": wl.C, "cadence": wl.cadence,
                       "spatial_fraction": wl.spatial_frac, "layers_per_call": lpc, "replicas": R_rep, "layers_with_own_inputs": Ld,
                       "step": "append + attend(+score accumulate) + compress, every layer",
                       "streams": n_streams,
                       "schedule": ("the batch dealt to %d streams (ssd_decode_step_split), every part's layers in order on its stream"
                                    % n_streams) if n_streams > 1
                                   else "one stream, one launch per call",
                       "sync": ("none between host synchronisations: every part runs free on its stream" if args.sync == "run" else
                                "fork at every token's first layer, join at its last") if n_streams > 1 else None,
                       "launches_per_step": head["launches_per_step"],
                       "entry_points": entry,
                       "timed_at": "last %d tokens of the raster decode (n -> %d)" % (passes[0], wl.n_total) +
                                   ("" if len(passes) == 1 else ", over %d decodes of the image" % len(passes))},
            "algorithmic_GB_per_step": head["algorithmic_GB_per_step"],
            "whole_step_GBps": head["algorithmic_GB_per_step"] / (head["ms_per_step"] / 1e3),
            "library_source_digest": library_source_digest(),
            "setup_s": {"generate_inputs": round(t_gen, 2)},
        }
        dense_bytes_total = 2 * wl.L * wl.B * wl.H * wl.n_total * row_bytes(wl)
        result["memory"] = {"compressed_cache_GB": cache.nbytes / 1e9, "full_cache_GB_at_end_of_image": dense_bytes_total / 1e9,
                            "ratio": dense_bytes_total / cache.nbytes,
                            "note": "K and V of all layers: the compressed cache block (ssd_cache_bytes: rows, scores, positions) "
                                    "against n = %d rows for every head" % wl.n_total}
        if "roofline" in head:
            result["roofline"] = head["roofline"]
        result["whole_decode"] = head["whole_decode"]

    # ---- the same steps on one stream, one launch per layer (what a caller without a second stream gets) ----
    if head is not None and n_streams > 1 and not args.no_one_stream:
        one = measure(lpc, with_events=not args.no_roofline, ns=1)
        result["one_stream"] = {"value": one["value"], "unit": "tokens/s", "ms_per_step": one["ms_per_step"],
                                "launches_per_step": one["launches_per_step"],
                                "entry_points": "ssd_decode_step_rope" if args.rope else "ssd_decode_step",
                                "whole_step_GBps": one["algorithmic_GB_per_step"] / (one["ms_per_step"] / 1e3)}
        if "roofline" in one:
            result["one_stream"]["roofline"] = one["roofline"]

    if head is not None and not args.no_all_layers and lpc != wl.L and Ld == wl.L:
        alt = measure(wl.L, with_events=not args.no_roofline, ns=1)
        result["all_layers_one_launch"] = {
            "value": alt["value"], "unit": "tokens/s", "ms_per_step": alt["ms_per_step"],
            "launches_per_step": alt["launches_per_step"],
            "note": "all %d layers in one library call: possible only because the synthetic queries of every layer exist "
                    "up front; in a model each layer's query depends on the layer before, so this is an upper bound" % wl.L}
        if "roofline" in alt:
            result["all_layers_one_launch"]["roofline"] = alt["roofline"]

    # ---- what the memory system allows a launch of this shape: a plain read of as many units of as many bytes,
    #      one launch per layer, without and with the least a decode step must store (two 256-byte rows per unit)
    if not args.no_ceiling:
        n_units = wl.B * wl.H
        n_, m_, c_, _ = cache.layer_state(0)
        if head is None:                                 # no decode has run: the counters a finished decode leaves behind
            n_, m_, c_ = wl.n_total, min(wl.M, wl.n_total), wl.R
        rows_u = max(2, int(round((algorithmic_bytes_attend(wl, ht, range(1), (n_, m_, c_)) / n_units) / (2 * row_bytes(wl)))))
        unit_b = rows_u * 2 * row_bytes(wl)
        unit_b = (unit_b + 511) // 512 * 512
        per_launch = n_units * unit_b
        # distinct memory per launch: as many regions as layers, more if that is needed to exceed the memory-side
        # cache several times over (1.5 GB), at most 6 GiB in all
        layers_c = max(1, min(max(wl.L, -(-1500000000 // per_launch)), (6 << 30) // per_launch))
        buf = torch.zeros(layers_c * n_units * unit_b, dtype=torch.uint8, device=dev)
        sink = torch.zeros(64, dtype=torch.uint8, device=dev)
        stream = torch.cuda.current_stream().cuda_stream
        ceil = {}
        for key, rows_w in (("read_only", 0), ("read_and_two_row_writes", 2)):
            def one_pass():
                for l in range(layers_c):
                    rc = ssd.lib.ssd_bench_stream(buf.data_ptr() + l * n_units * unit_b, unit_b, n_units, rows_w, sink.data_ptr(), stream)
                    assert rc == 0, ssd.ssd_last_error()
            one_pass()
            torch.cuda.synchronize()
            reps = 10
            t0 = time.perf_counter()
            for _ in range(reps):
                one_pass()
            torch.cuda.synchronize()
            us = (time.perf_counter() - t0) / (reps * layers_c) * 1e6
            moved = n_units * (unit_b + 256 * rows_w)
            ceil[key] = {"us_per_launch": us, "GBps": moved / 1e3 / us, "frac_of_hbm_peak": moved / 1e3 / us / HBM_PEAK_GBS}
            if head is not None and n_streams > 1:
                # the same bytes in the headline's schedule: every layer's units dealt to the streams, each stream running free
                st = [stream] + [x.cuda_stream for x in side_streams[: n_streams - 1]]
                cut = [n_units * i // n_streams for i in range(n_streams + 1)]

                def split_pass():
                    for l in range(layers_c):
                        for i in range(n_streams):
                            rc = ssd.lib.ssd_bench_stream(buf.data_ptr() + (l * n_units + cut[i]) * unit_b, unit_b, cut[i + 1] - cut[i],
                                                          rows_w, sink.data_ptr(), st[i])
                            assert rc == 0, ssd.ssd_last_error()
                split_pass()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(reps):
                    split_pass()
                torch.cuda.synchronize()
                us2 = (time.perf_counter() - t0) / (reps * layers_c) * 1e6
                ceil[key + "_on_%d_streams" % n_streams] = {"us_per_layer": us2, "GBps": moved / 1e3 / us2,
                                                            "frac_of_hbm_peak": moved / 1e3 / us2 / HBM_PEAK_GBS}
        result["stream_ceiling"] = dict(ceil, units_per_launch=n_units, bytes_per_unit=unit_b, launches_timed=layers_c,
                                        kind="ssd_bench_stream: every unit read once by one wavefront, no arithmetic; the second line "
                                             "also stores one 256-byte row into each plane of every unit (a new token's K and V)")
        del buf

    # ---- prompt scoring (accumulated causal scores of the n0 prompt tokens), one launch per layer ------------
    if not args.no_prefill:
        n0 = wl.n0
        Qp = [workload.dense_layout(data["q"][:n0, l:l + 1])[0].contiguous() for l in range(Ld)]
        Kp = [workload.dense_layout(data["k"][:n0, l:l + 1])[0].contiguous() for l in range(Ld)]
        sc = torch.empty((wl.B, wl.H, n0), device=dev)
        units = wl.B * wl.H

        def prefill_pass():
            for l in range(wl.L):
                ssd.ssd_prefill_scores(Qp[l % Ld], Kp[l % Ld], units, n0, wl.d, wl.dtype, sc)
        prefill_pass()
        torch.cuda.synchronize()
        reps = 5
        t0 = time.perf_counter()
        for _ in range(reps):
            prefill_pass()
        torch.cuda.synchronize()
        tp = (time.perf_counter() - t0) / reps
        pf_bytes = wl.L * units * (2 * n0 * row_bytes(wl) + 4 * n0)
        nb = (n0 + 31) // 32
        sweeps = 1 if nb <= 4 else 2                                                # short prompts keep their logits in registers
        pf_flops = wl.L * units * sweeps * (nb * (nb + 1) // 2) * 2 * 32 * 32 * wl.d   # tiles on or below the diagonal
        result["prefill_scores"] = {"ms_all_layers": tp * 1e3, "us_per_layer_launch": tp * 1e6 / wl.L, "prompt_tokens": n0,
                                    "algorithmic_GB": pf_bytes / 1e9, "GBps": pf_bytes / 1e9 / tp,
                                    "frac_of_hbm_peak": pf_bytes / 1e9 / tp / HBM_PEAK_GBS, "mfma_TFLOPs": pf_flops / 1e12 / tp,
                                    "kind": "ssd_prefill_scores, Q and K of the prompt read once, fp32 column sums written"}
        if n_streams > 1:
            # the same launches with the units of a layer dealt to the streams (units are independent: the caller offsets the
            # pointers), every stream running free, as the decode headline's parts do
            sts = [torch.cuda.current_stream()] + side_streams[: n_streams - 1]
            cut = [units * i // n_streams for i in range(n_streams + 1)]
            Qv = [x.view(units, n0, wl.d) for x in Qp]
            Kv = [x.view(units, n0, wl.d) for x in Kp]
            scv = sc.view(units, n0)

            def prefill_split_pass():
                for l in range(wl.L):
                    for i in range(n_streams):
                        ssd.ssd_prefill_scores(Qv[l % Ld][cut[i]:cut[i + 1]], Kv[l % Ld][cut[i]:cut[i + 1]], cut[i + 1] - cut[i], n0, wl.d,
                                               wl.dtype, scv[cut[i]:cut[i + 1]], stream=sts[i])
            prefill_split_pass()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                prefill_split_pass()
            torch.cuda.synchronize()
            tp2 = (time.perf_counter() - t0) / reps
            result["prefill_scores"]["on_%d_streams" % n_streams] = {"ms_all_layers": tp2 * 1e3, "us_per_layer": tp2 * 1e6 / wl.L,
                                                                      "GBps": pf_bytes / 1e9 / tp2,
                                                                      "frac_of_hbm_peak": pf_bytes / 1e9 / tp2 / HBM_PEAK_GBS}
        del Qp, Kp

    # ---- the same steps through the dense full-cache kernel -----------------------------------------------
    if not args.no_dense:
        t0 = time.time()
        n = wl.n_total
        Kd = [workload.dense_layout(data["k"][:, l:l + 1])[0] for l in range(Ld)]     # layer l reads the rows of layer l mod Ld
        Vd = [workload.dense_layout(data["v"][:, l:l + 1])[0] for l in range(Ld)]
        ws = torch.empty(ssd.ssd_dense_workspace_bytes(wl.B, wl.H, wl.d, n), dtype=torch.uint8, device=dev)
        outd = torch.empty((wl.B, wl.H, wl.d), dtype=wl.torch_dtype, device=dev)
        torch.cuda.synchronize()
        t_dense_setup = time.time() - t0
        reps = max(3, min(K_steps, 20))

        def dense_step(p):
            for l in range(wl.L):
                ssd.ssd_dense_decode_attn(data["q"][p, l % Ld], Kd[l % Ld], Vd[l % Ld], outd, wl.B, wl.H, wl.d, wl.dtype, n, p + 1, 0.0,
                                          None, None, 1, 0, 32, ws)
        for p in range(n - reps - 2, n - reps):
            dense_step(p)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for p in range(n - reps, n):
            dense_step(p)
        torch.cuda.synchronize()
        dtd = (time.perf_counter() - t0) / reps
        row = row_bytes(wl)
        dense_bytes = wl.L * wl.B * wl.H * ((n - (reps - 1) / 2) * 2 * row + 2 * row)
        # whole raster decode through the dense kernel (its cost grows with n)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for p in range(n - reps if (args.only == "dense") else wl.n0, n):        # a counter run of the dense kernel alone stays short
            dense_step(p)
        torch.cuda.synchronize()
        dense_whole = time.perf_counter() - t0
        result["dense_baseline"] = {"value": wl.prompts / dtd, "unit": "tokens/s", "ms_per_step": dtd * 1e3,
                                    "algorithmic_GB_per_step": dense_bytes / 1e9, "GBps": dense_bytes / 1e9 / dtd,
                                    "frac_of_hbm_peak": dense_bytes / 1e9 / dtd / HBM_PEAK_GBS, "steps": reps,
                                    "kind": "hand-written HIP split-K decode attention over all n rows, one launch per layer, "
                                            "appending the new token not included",
                                    "speedup_of_compressed": None if head is None else dtd / (head["ms_per_step"] / 1e3),
                                    "whole_decode": {"visual_tokens": wl.N, "seconds": dense_whole,
                                                     "value": wl.prompts * wl.N / dense_whole, "unit": "tokens/s",
                                                     "speedup_of_compressed": None if head is None else dense_whole / head["whole_decode"]["seconds"]}}
        result.setdefault("setup_s", {})["dense_layout"] = round(t_dense_setup, 2)
        del Kd, Vd

    # ---- the head mix of the paper's own settings: few long semantic heads beside many short spatial ones --------------
    if not args.no_head_mix and head is not None and fused and wl.H >= 16 and not args.rope and wl.head_budget is None and Ld == wl.L \
            and R_rep == 1:
        wl_m = wl.replace(W=32, M=128, spatial_frac=(wl.H - max(1, wl.H // 16)) / wl.H, alg2=False, R=1, C=2, cadence=1, name=wl.name + "-paper-mix")
        ht_m = workload.head_map(wl_m)
        cfg_m = make_config(wl_m.L, wl_m.B, wl_m.H, wl_m.d, wl_m.dtype, wl_m.W, wl_m.S, wl_m.M, wl_m.R, wl_m.C, 0.0, 0)
        cache_m = ssd.Cache(cfg_m, ht_m, device=dev)
        stride_l = wl.B * wl.H * wl.d * (2 if wl.dtype == "bf16" else 4)
        qb, kb, vb, ob = data["q"].data_ptr(), data["k"].data_ptr(), data["v"].data_ptr(), out.data_ptr()
        stream = torch.cuda.current_stream().cuda_stream
        arr = ssd.stream_array([torch.cuda.current_stream()] + side_streams[: n_streams - 1])

        def mix_timed(ns):
            def step(p):                                  # the inputs are the headline's (their values do not matter for the time)
                for l in range(wl_m.L):
                    o = (p * wl_m.L + l) * stride_l
                    if ns > 1:
                        rc = ssd.lib.ssd_decode_step_split(cache_m.handle, l, l + 1, qb + o, kb + o, vb + o, ob + l * stride_l, 1, 1, arr, ns, 0)
                    else:
                        rc = ssd.lib.ssd_decode_step(cache_m.handle, l, l + 1, qb + o, kb + o, vb + o, ob + l * stride_l, 1, 1, stream)
                    assert rc == 0, ssd.ssd_last_error()
            cache_m.reset()
            for p in range(wl_m.n_total - K_steps):
                step(p)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for p in range(wl_m.n_total - K_steps, wl_m.n_total):
                step(p)
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / K_steps
        n_, m_, c_, _ = (wl_m.n_total, wl_m.M, 1, 0)
        gb = (algorithmic_bytes_attend(wl_m, ht_m, range(wl_m.L), (n_, m_, c_ + 1)) + algorithmic_bytes_append(wl_m, ht_m, range(wl_m.L))) / 1e9
        leg = {"window": wl_m.W, "budget": wl_m.M, "spatial_heads": int((ht_m[0] == 0).sum()), "semantic_heads": int((ht_m[0] == 1).sum()),
               "algorithmic_GB_per_step": gb}
        for key, ns in (("headline_schedule", n_streams), ("one_stream", 1)):
            dt_m = mix_timed(ns)
            leg[key] = {"streams": ns, "ms_per_step": dt_m * 1e3, "value": wl_m.prompts / dt_m, "unit": "tokens/s",
                        "frac_of_hbm_peak": gb / dt_m / HBM_PEAK_GBS}
            if ns == 1:
                break
        result["paper_head_mix"] = leg
        del cache_m

    # ---- CPU oracle on a sample of units ------------------------------------------------------------------
    if not args.no_cpu:
        import oracle
        cores = min(16, os.cpu_count() or 1)
        # whole (layer, sequence) slices: all heads of a pair are one contiguous read per position
        rng = np.random.default_rng(1)
        n_pairs = max(1, min(wl.L * wl.B, args.cpu_units // wl.H))
        pairs = sorted(set((int(rng.integers(wl.L)), int(rng.integers(wl.B))) for _ in range(n_pairs)))
        host = {}
        for (l, b) in pairs:
            host[(l, b)] = tuple(np.ascontiguousarray(data[x][:, l % Ld, b].float().cpu().numpy().transpose(1, 0, 2)) for x in "qkv")
        units = [(l, b, h) for (l, b) in pairs for h in range(wl.H)]

        def run_unit(i):
            l, b, h = units[i]
            u = oracle.Unit(ht[l, h] == workload.SEMANTIC, wl.W, wl.S, wl.M, wl.R, wl.C, buffered_spatial=wl.alg2)
            q_, k_, v_ = (a[h] for a in host[(l, b)])
            u.run(q_, k_, v_, wl.scale, sched)
            return 0

        t0 = time.perf_counter()
        with ThreadPoolExecutor(cores) as ex:
            list(ex.map(run_unit, range(len(units))))
        t_cpu = time.perf_counter() - t0
        unit_steps_per_s = len(units) * wl.n_total / t_cpu
        units_per_step = wl.L * wl.B * wl.H
        result["cpu_baseline"] = {"value": wl.prompts * unit_steps_per_s / units_per_step, "unit": "tokens/s", "cores": cores,
                                  "kind": "oracle",
                                  "sample": "%d of %d (layer, sequence, head) units decoded over all %d tokens in %.1f s on %d "
                                            "threads, extrapolated to all units (units are independent)" % (
                                                len(units), units_per_step, wl.n_total, t_cpu, cores)}

    print(json.dumps(result))


if __name__ == "__main__":
    main()
