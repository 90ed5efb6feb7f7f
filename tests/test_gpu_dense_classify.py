"""GPU parity of the full-cache baseline kernel, the (far, tot) masses it emits, head classification, and
the dense-source mode of ssd_compress_kv (selection fed identical scores, exact ties included)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_18716_amd as ssd
import workload
from harness import TOL, check_outputs, gpu_decode, heavy_cap, make_cache, oracle_unit, sample_units, say

pytestmark = pytest.mark.gpu


def _dense_case(B, H, d, dtype, n_cap, n, splits, seed, vis_start=0, w=32):
    say("dense case", B, H, d, dtype, n_cap, n, "splits", splits)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    g = torch.Generator().manual_seed(seed)
    q = torch.randn((B, H, d), generator=g).to(tdt)
    K = torch.randn((B, H, n_cap, d), generator=g).to(tdt)
    V = torch.randn((B, H, n_cap, d), generator=g).to(tdt)
    out = torch.empty((B, H, d), dtype=tdt, device="cuda")
    far = torch.full((B, H, 3), -7.0, device="cuda")
    tot = torch.full((B, H, 3), -7.0, device="cuda")
    ws = torch.empty(ssd.ssd_dense_workspace_bytes(B, H, d, n), dtype=torch.uint8, device="cuda")
    # splits = 0: the entry point itself (the library's choice); otherwise the hook that fixes the split count
    ssd.ssd_dense_decode_attn(q.cuda(), K.cuda(), V.cuda(), out, B, H, d, dtype, n_cap, n, 0.0,
                              far[:, :, 1:].data_ptr(), tot[:, :, 1:].data_ptr(), 3, vis_start, w, ws,
                              splits=splits if splits else None)
    torch.cuda.synchronize()
    o = out.float().cpu().numpy()
    farh, toth = far.cpu().numpy(), tot.cpu().numpy()
    scale = 1.0 / np.sqrt(d)
    for b in range(B):
        for h in range(H):
            ref, _, p64 = oracle.dense_attend(q[b, h].float().numpy(), K[b, h].float().numpy(), V[b, h].float().numpy(), n, scale)
            check_outputs(o[b, h], ref, dtype, "dense unit (%d,%d)" % (b, h))
            t = n - vis_start
            if t >= 1:
                f_ref, t_ref = oracle.far_tot(p64, vis_start, t, w)
                assert abs(farh[b, h, 1] - f_ref) < 2e-5 + 1e-4 * f_ref
                assert abs(toth[b, h, 1] - t_ref) < 2e-5 + 1e-4 * t_ref
            # the strided mass outputs touched nothing else
            assert farh[b, h, 0] == -7.0 and farh[b, h, 2] == -7.0 and toth[b, h, 0] == -7.0


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 64), ("bf16", 64), ("f32", 128)])
def test_dense_kernel_matches_oracle(dtype, d):
    _dense_case(2, 3, d, dtype, 70, 1, 1, 1)
    _dense_case(2, 3, d, dtype, 70, 67, 1, 2, vis_start=9, w=32)
    _dense_case(2, 3, d, dtype, 300, 257, 3, 3, vis_start=64, w=32)
    _dense_case(1, 2, d, dtype, 700, 640, 0, 4, vis_start=64, w=32)


def test_dense_kernel_long_rows_and_many_splits():
    _dense_case(1, 2, 128, "bf16", 2368, 2368, 0, 5, vis_start=64, w=32)
    _dense_case(1, 2, 128, "bf16", 2368, 2001, 16, 6, vis_start=64, w=32)


def test_classification_recovers_planted_head_types():
    # a profiling run of the dense kernel over every visual step feeds the reduction (Sec. 3.3)
    wl = workload.config(1).replace(name="cfg1-classify", L=2, prompts=2)
    ht = workload.head_map(wl)
    data = workload.generate(wl, head_type=ht)
    dev = {k: v.cuda() for k, v in data.items()}
    w = 16
    L, P, H, T = wl.L, wl.B, wl.H, wl.N
    far = torch.zeros((L, P, H, T), device="cuda")
    tot = torch.zeros((L, P, H, T), device="cuda")
    K = workload.dense_layout(dev["k"])
    V = workload.dense_layout(dev["v"])
    out = torch.empty((P, H, wl.d), dtype=wl.torch_dtype, device="cuda")
    ws = torch.empty(ssd.ssd_dense_workspace_bytes(P, H, wl.d, wl.n_total), dtype=torch.uint8, device="cuda")
    for t in range(1, T + 1):
        n = wl.n0 + t
        for l in range(L):
            ssd.ssd_dense_decode_attn(dev["q"][n - 1, l], K[l], V[l], out, P, H, wl.d, wl.dtype, wl.n_total, n, 0.0,
                                      far[l, :, :, t - 1:].data_ptr(), tot[l, :, :, t - 1:].data_ptr(), T, wl.n0, w, ws)
    s_gpu = torch.zeros((L, H), device="cuda")
    ty_gpu = torch.zeros((L, H), dtype=torch.uint8, device="cuda")
    tau = 0.3
    ssd.ssd_classify_heads(far, tot, L, P, H, T, tau, s_gpu, ty_gpu)
    torch.cuda.synchronize()
    # oracle: its own far/tot from the same inputs, its own reduction
    far_o = np.zeros((L, P, H, T), np.float32); tot_o = np.zeros_like(far_o)
    for l in range(L):
        for b in range(P):
            for h in range(H):
                q_, K_, V_ = workload.unit_arrays(data, l, b, h)
                far_o[l, b, h], tot_o[l, b, h] = oracle.profile_unit(q_, K_, V_, wl.n0, T, w, wl.scale)
    s_ref, ty_ref = oracle.classify(far_o, tot_o, tau)
    np.testing.assert_allclose(far.cpu().numpy(), far_o, atol=2e-5, rtol=1e-4)
    np.testing.assert_allclose(tot.cpu().numpy(), tot_o, atol=2e-5, rtol=1e-4)
    np.testing.assert_allclose(s_gpu.cpu().numpy(), s_ref, atol=1e-5, rtol=1e-4)
    assert (np.abs(s_ref - tau) > 1e-3).all()          # no head sits on the threshold
    np.testing.assert_array_equal(ty_gpu.cpu().numpy(), ty_ref)
    np.testing.assert_array_equal(ty_ref, ht)
    # the reduction alone, fed the oracle's masses: the threshold decision must agree exactly
    ssd.ssd_classify_heads(torch.from_numpy(far_o).cuda(), torch.from_numpy(tot_o).cuda(), L, P, H, T, tau, s_gpu, ty_gpu)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(ty_gpu.cpu().numpy(), ty_ref)


def test_classification_strict_threshold_and_zero_denominator():
    far = torch.ones((1, 2, 2, 8), device="cuda")
    tot = 2 * torch.ones((1, 2, 2, 8), device="cuda")
    tot[0, 0, 1, 0] = 0.0                               # one term of head 1 contributes ratio 0
    s = torch.zeros((1, 2), device="cuda"); ty = torch.zeros((1, 2), dtype=torch.uint8, device="cuda")
    ssd.ssd_classify_heads(far, tot, 1, 2, 2, 8, 0.5, s, ty)
    torch.cuda.synchronize()
    assert s.cpu().tolist() == [[0.5, 0.5 * 15 / 16]]
    assert ty.cpu().tolist() == [[0, 0]]                # s == tau is Spatial (strict inequality of Eq. 3)
    ssd.ssd_classify_heads(far, tot, 1, 2, 2, 8, 0.46875 - 1e-6, s, ty)
    torch.cuda.synchronize()
    assert ty.cpu().tolist() == [[1, 1]]


def _dense_source_case(wl, ht, n_src, fused=False):
    """Dense-source compression of the first n_src tokens with scores full of exact ties, then ordinary decode of
    the rest, against an oracle unit that took the same route (load_dense, then run)."""
    say("dense-source case", wl.name, wl.dtype, wl.d, "n_src", n_src, "M", wl.M, "R", wl.R, "W", wl.W, "S", wl.S, "alg2", wl.alg2,
        "per-head", wl.head_budget is not None, "fused", fused)
    data = workload.generate(wl, head_type=ht)
    dev = {k: v.cuda() for k, v in data.items()}
    r = np.random.default_rng(n_src)
    # few distinct values: many exact ties, decided by position
    score = (r.integers(0, 7, (wl.L, wl.B, wl.H, n_src)) / 8).astype(np.float32)
    K = workload.dense_layout(dev["k"][:n_src])
    V = workload.dense_layout(dev["v"][:n_src])
    cache = make_cache(wl, ht)
    ssd.ssd_compress_kv(cache, 0, wl.L, K, V, torch.from_numpy(score).cuda(), n_src)
    first = [x.cpu().numpy() for x in cache.export(0)]          # state right after the dense-source call, layer 0
    # then decode the remaining tokens normally on both sides
    units = sample_units(wl, ht, 10 ** 9)
    sched = workload.compress_schedule(wl)
    steps = list(range(n_src, wl.n_total))
    outs, exports, _ = gpu_decode(wl, dev, ht, sched, units, export_steps=steps, cache=cache, p_begin=n_src, fused=fused,
                                  shadow=False)
    for ui, (l, b, h) in enumerate(units):
        q_, K_, V_ = workload.unit_arrays(data, l, b, h)
        sem = ht[l, h] == workload.SEMANTIC
        W_h, M_h = wl.W_of(l, h), wl.M_of(l, h)
        u = oracle.Unit(sem, W_h, wl.S, M_h, wl.R, wl.C, buffered_spatial=wl.alg2)
        u.load_dense(n_src, score[l, b, h])
        if l == 0:      # the call's own result, before any further token
            got = sorted(int(x) for x in first[0][b, h] if x >= 0)
            assert got == sorted(int(x) for x in u.retained()), ("retained set after the dense-source call", (l, b, h))
            if sem:
                hp, hs, sp, ss = u.state()
                ref = dict(zip(hp.tolist() + sp.tolist(), hs.tolist() + ss.tolist()))
                assert {int(p): float(x) for p, x in zip(first[0][b, h], first[2][b, h]) if p >= 0} == ref
        o_ref, hl, gl = u.run(q_, K_, V_, wl.scale, sched, log=True)
        check_outputs(outs[:, ui], o_ref, wl.dtype, "unit %s after dense-source compression" % ((l, b, h),))
        Mcap = heavy_cap(wl, ht, l)
        for p in steps:
            row = exports[p]["post"][0][l, b, h]
            if sem:
                assert sorted(int(x) for x in row[:Mcap] if x >= 0) == [int(x) for x in hl[p - n_src] if x >= 0], ((l, b, h), p)
            else:
                n = p + 1
                n_c = max([s + 1 for s in range(n_src, p + 1) if sched[s]], default=n_src)
                ref_n = n_c if wl.alg2 else n
                assert sorted(int(x) for x in row if x >= 0) == sorted(set(range(min(wl.S, n))) | set(range(max(wl.S, ref_n - W_h), n))), ((l, b, h), p)


@pytest.mark.parametrize("dtype,d,n_src,M,R,W,S", [("bf16", 128, 200, 16, 3, 24, 2), ("f32", 64, 37, 40, 1, 50, 1),
                                                    ("bf16", 128, 2368, 128, 1, 128, 1), ("bf16", 64, 5, 4, 8, 3, 1)])
def test_dense_source_compression_with_tied_scores(dtype, d, n_src, M, R, W, S):
    wl = workload.Workload("dsrc", L=2, prompts=1, H=4, d=d, dtype=dtype, n0=n_src, grid_h=2, grid_w=3, W=W, M=M,
                           S=S, R=R, C=R + 3, cadence=2, seed=31 + n_src, plain=True)
    _dense_source_case(wl, workload.head_map(wl), n_src)


@pytest.mark.parametrize("fused", [False, True], ids=["three-calls", "fused-step"])
@pytest.mark.parametrize("dtype,d,n_src,M,R,W,S,C,cadence", [("bf16", 128, 200, 16, 0, 24, 2, 6, 6), ("f32", 64, 37, 40, 2, 50, 1, 7, 4),
                                                             ("bf16", 64, 5, 4, 3, 3, 1, 5, 2), ("bf16", 128, 90, 12, 1, 100, 0, 4, 3)])
def test_dense_source_compression_under_algorithm2(dtype, d, n_src, M, R, W, S, C, cadence, fused):
    # the prefill branch of Algorithm 2 with the row buffer read by both head types: the spatial heads' window is
    # cut at n_src ("Compress spatial cache (sink + recent)"), their ring has W + C slots, and the tokens decoded
    # afterwards pile up in the row buffer until the next compression
    wl = workload.Workload("dsrc-alg2", L=2, prompts=1, H=4, d=d, dtype=dtype, n0=n_src, grid_h=3, grid_w=5, W=W, M=M,
                           S=S, R=R, C=C, cadence=cadence, seed=131 + n_src, plain=True, alg2=True)
    assert R + cadence <= C          # room in the row buffer until the first compression after the prompt
    _dense_source_case(wl, workload.head_map(wl), n_src, fused=fused)


@pytest.mark.parametrize("fused", [False, True], ids=["three-calls", "fused-step"])
@pytest.mark.parametrize("alg2", [False, True], ids=["alg1", "alg2"])
def test_dense_source_compression_with_budgets_per_head(alg2, fused):
    # head-wise allocation: every head keeps its own W_h newest / top-M_h tokens of the dense segment, inside units
    # sized for the layer's largest head; includes W_h = 1, M_h = 1 and budgets beyond the segment
    hb = ((24, 5, 1, 7, 200, 3), (9, 9, 30, 2, 1, 17))
    n_src = 60
    wl = workload.Workload("dsrc-per-head", L=2, prompts=1, H=6, d=128, dtype="bf16", n0=n_src, grid_h=3, grid_w=5, W=99, M=99,
                           S=1, R=(0 if alg2 else 2), C=5, cadence=(5 if alg2 else 3), seed=137, plain=True, head_budget=hb, alg2=alg2)
    _dense_source_case(wl, workload.head_map(wl), n_src, fused=fused)
    wl = wl.replace(name="dsrc-per-head-f32", dtype="f32", d=64, seed=139)
    _dense_source_case(wl, workload.head_map(wl), n_src, fused=fused)


def test_dense_source_without_scores_keeps_lowest_positions():
    wl = workload.Workload("dsrc-noscore", L=1, prompts=1, H=2, d=64, dtype="f32", n0=30, grid_h=1, grid_w=1, W=4, M=6,
                           S=1, R=2, C=4, cadence=1, seed=8, plain=True)
    ht = np.array([[0, 1]], np.uint8)
    dev = {k: v.cuda() for k, v in workload.generate(wl, head_type=ht).items()}
    cache = make_cache(wl, ht)
    ssd.ssd_compress_kv(cache, 0, 1, workload.dense_layout(dev["k"][:30]), workload.dense_layout(dev["v"][:30]), None, 30)
    pos, cnt, sc = [x.cpu().numpy() for x in cache.export(0)]
    assert sorted(int(x) for x in pos[0, 1] if x >= 0) == [0, 1, 2, 3, 4, 5, 28, 29]
    assert sorted(int(x) for x in pos[0, 0] if x >= 0) == [0, 26, 27, 28, 29]
    assert cnt[0].tolist() == [5, 8] and (sc == 0).all()
    assert cache.layer_state(0) == (30, 6, 2, 0)


def test_stream_benchmark_reads_everything_and_writes_only_its_two_rows():
    # the measurement aid behind bench.py's "stream_ceiling": it must touch what it says and nothing else
    n_units, rows = 37, 5                                   # a ragged last workgroup
    unit_b = rows * 2 * 256
    buf = torch.randint(0, 255, (n_units + 1, unit_b), dtype=torch.uint8, device="cuda")     # one guard unit behind
    before = buf.clone()
    sink = torch.zeros(64, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    assert ssd.lib.ssd_bench_stream(buf.data_ptr(), unit_b, n_units, 0, sink.data_ptr(), stream) == 0
    torch.cuda.synchronize()
    assert torch.equal(buf, before) and int(sink.sum()) == 0
    assert ssd.lib.ssd_bench_stream(buf.data_ptr(), unit_b, n_units, 2, sink.data_ptr(), stream) == 0
    torch.cuda.synchronize()
    changed = (buf != before).view(n_units + 1, 2, rows, 256).any(dim=3)      # [unit, plane, row]
    assert not changed[n_units].any()                       # nothing behind the last unit
    assert not changed[:, :, 1:].any()                      # only row 0 of each plane
    assert changed[:n_units, :, 0].float().mean() > 0.9     # and that one is written (a random row rarely stays equal)


def test_copy_benchmark_copies_exactly_what_it_says():
    # the kernel whose known traffic scales the profiler's byte counters: dst = src over `bytes`, nothing beyond
    n = (1 << 20) + 16 * 37                                  # not a multiple of the workgroup's stride
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda")
    dst = torch.full((n + 256,), 7, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    assert ssd.lib.ssd_bench_copy(dst.data_ptr(), src.data_ptr(), n, stream) == 0
    torch.cuda.synchronize()
    assert torch.equal(dst[:n], src) and bool((dst[n:] == 7).all())
