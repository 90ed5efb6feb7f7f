"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares, and its
host-side logic (validation, counters, ordering and overflow errors) behaves as the header says.
No kernel is launched here: caches are created over a fake address with launches switched off."""
import os
import re

import numpy as np
import pytest

import oracle
import paper_2510_18716_amd as ssd
from paper_2510_18716_amd.binding import make_config

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 1 << 24          # a 16-byte aligned non-null "device pointer" that is never dereferenced


def test_library_exports_every_declared_symbol():
    import glob
    headers = sorted(glob.glob(os.path.join(ROOT, "include", "*.h")))
    assert [os.path.basename(h) for h in headers] == ["ssd.h", "ssd_hooks.h"]
    text = "".join(open(h).read() for h in headers)
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(ssd_[a-z_0-9]+)\s*\(", text)))
    assert {"ssd_classify_heads", "ssd_compress_kv", "ssd_decode_attn", "ssd_append_token", "ssd_decode_step_split"} <= set(names)
    # the method's header holds no launch-shape or benchmark hook
    api = re.sub(r"/\*.*?\*/", "", open(headers[0]).read(), flags=re.S)
    assert "ssd_bench_stream" not in api and "launch_shape" not in api and "ssd_cache_set_launch" not in api
    for n in names:
        assert hasattr(ssd.lib, n), n
    assert ssd.ssd_version() >= 100
    assert ssd.ssd_last_error() == "" or isinstance(ssd.ssd_last_error(), str)


def _ht(L, H, frac=0.5):
    m = np.ones((L, H), np.uint8)
    m[:, : int(H * frac)] = 0
    return m


def test_cache_bytes_matches_layout_formula():
    L, B, H, d, W, S, M, R, C_ = 3, 4, 8, 128, 64, 1, 64, 1, 2
    cfg = make_config(L, B, H, d, "bf16", W, S, M, R, C_)
    ht = _ht(L, H)
    row = d * 2
    per_layer = B * 4 * 2 * (S + W) * row + B * 4 * 2 * (M + C_) * row + 2 * B * 4 * (M + C_) * 4
    got = ssd.ssd_cache_bytes(cfg, ht)
    assert per_layer * L <= got <= per_layer * L + 4096 + 4 * 256 * L
    # fp32 rows are twice as long
    cfg32 = make_config(L, B, H, d, "f32", W, S, M, R, C_)
    assert ssd.ssd_cache_bytes(cfg32, ht) > 1.9 * per_layer * L


@pytest.mark.parametrize("field,value", [
    ("n_layers", 0), ("n_seqs", 0), ("n_heads", 0), ("head_dim", 96), ("dtype", 7), ("window", 0),
    ("n_init_sink", -1), ("budget", 0), ("recent", -1), ("stage_cap", 1), ("softmax_scale", -1.0),
    ("softmax_scale", float("nan")), ("budget", 4096),
])
def test_bad_config_is_refused(field, value):
    cfg = make_config(2, 2, 4, 64, "f32", 8, 1, 8, 1, 2)
    setattr(cfg, field, value)
    assert ssd.ssd_cache_bytes(cfg, _ht(2, 4)) == 0
    assert ssd.ssd_last_error() != ""
    with pytest.raises(ssd.SsdError):
        ssd.Cache(cfg, _ht(max(cfg.n_layers, 1), max(cfg.n_heads, 1)), device=None)


def test_bad_head_type_and_reserved_fields():
    cfg = make_config(1, 2, 4, 64, "f32", 8, 1, 8, 1, 2)
    bad = np.array([[0, 1, 2, 0]], np.uint8)
    assert ssd.ssd_cache_bytes(cfg, bad) == 0
    cfg.reserved[2] = 5
    assert ssd.ssd_cache_bytes(cfg, _ht(1, 4)) == 0


def test_init_checks_pointer_and_size():
    import ctypes as C
    cfg = make_config(1, 2, 4, 64, "f32", 8, 1, 8, 1, 2)
    ht = _ht(1, 4)
    need = ssd.ssd_cache_bytes(cfg, ht)
    h = C.c_void_p()
    assert ssd.lib.ssd_cache_init(C.byref(cfg), ht.ctypes.data, None, need, C.byref(h)) == ssd.SSD_ERR_INVALID_ARG
    assert ssd.lib.ssd_cache_init(C.byref(cfg), ht.ctypes.data, FAKE + 16, need, C.byref(h)) == ssd.SSD_ERR_INVALID_ARG
    assert "256" in ssd.ssd_last_error()
    assert ssd.lib.ssd_cache_init(C.byref(cfg), ht.ctypes.data, FAKE, need - 1, C.byref(h)) == ssd.SSD_ERR_INVALID_ARG
    assert ssd.lib.ssd_cache_init(C.byref(cfg), ht.ctypes.data, FAKE, need, C.byref(h)) == ssd.SSD_OK
    ssd.lib.ssd_cache_free(h)
    ssd.lib.ssd_cache_free(None)


def test_layer_range_order_and_pointer_errors():
    cfg = make_config(3, 2, 4, 64, "f32", 8, 1, 8, 1, 3)
    c = ssd.Cache(cfg, _ht(3, 4), device=None)
    for lb, le in [(-1, 1), (0, 4), (2, 2), (2, 1)]:
        with pytest.raises(ssd.SsdError) as e:
            ssd.ssd_append_token(c, lb, le, FAKE, FAKE)
        assert e.value.code == ssd.SSD_ERR_LAYER_RANGE
    with pytest.raises(ssd.SsdError) as e:
        ssd.ssd_decode_attn(c, 0, 3, FAKE, FAKE)
    assert e.value.code == ssd.SSD_ERR_ORDER                      # nothing appended yet
    ssd.ssd_append_token(c, 0, 2, FAKE, FAKE)
    ssd.ssd_decode_attn(c, 0, 2, FAKE, FAKE)
    with pytest.raises(ssd.SsdError) as e:
        ssd.ssd_decode_attn(c, 0, 3, FAKE, FAKE)                  # layer 2 is still empty
    assert e.value.code == ssd.SSD_ERR_ORDER
    for args in [(None, FAKE), (FAKE, None), (FAKE + 4, FAKE)]:
        with pytest.raises(ssd.SsdError) as e:
            ssd.ssd_append_token(c, 0, 1, *args)
        assert e.value.code == ssd.SSD_ERR_INVALID_ARG
    assert c.layer_state(0)[0] == 1                               # failed calls changed nothing
    with pytest.raises(ssd.SsdError) as e:
        ssd.ssd_compress_kv(c, 0, 1, FAKE, None, None, 4)
    assert e.value.code == ssd.SSD_ERR_INVALID_ARG
    with pytest.raises(ssd.SsdError):
        ssd.ssd_compress_kv(c, 0, 1, FAKE, FAKE, None, 0)
    with pytest.raises(ssd.SsdError):
        ssd.ssd_compress_kv(c, 0, 1, FAKE, FAKE, None, 4097)


def test_row_buffer_overflow_refuses_the_whole_call():
    cfg = make_config(2, 2, 4, 64, "f32", 8, 1, 8, 1, 3)
    c = ssd.Cache(cfg, _ht(2, 4), device=None)
    ssd.ssd_append_token(c, 0, 1, FAKE, FAKE)                     # layer 0 one token ahead
    for _ in range(2):
        ssd.ssd_append_token(c, 0, 2, FAKE, FAKE)
    assert c.layer_state(0)[:3] == (3, 0, 3) and c.layer_state(1)[:3] == (2, 0, 2)
    with pytest.raises(ssd.SsdError) as e:
        ssd.ssd_append_token(c, 0, 2, FAKE, FAKE)
    assert e.value.code == ssd.SSD_ERR_STAGE_OVERFLOW and "overflow" in ssd.ssd_last_error()
    assert c.layer_state(1)[:3] == (2, 0, 2)                      # layer 1 was not touched either
    ssd.ssd_compress_kv(c, 0, 2)
    assert c.layer_state(0) == (3, 2, 1, 2) and c.layer_state(1) == (2, 1, 1, 1)
    ssd.ssd_append_token(c, 0, 2, FAKE, FAKE)
    c.reset()
    assert c.layer_state(0) == (0, 0, 0, 0)


def test_all_spatial_layer_has_no_row_buffer():
    cfg = make_config(1, 2, 4, 64, "f32", 8, 1, 8, 1, 2)
    c = ssd.Cache(cfg, np.zeros((1, 4), np.uint8), device=None)
    for _ in range(50):
        ssd.ssd_append_token(c, 0, 1, FAKE, FAKE)
    assert c.layer_state(0) == (50, 0, 0, 0)
    ssd.ssd_compress_kv(c, 0, 1)
    assert c.layer_state(0) == (50, 0, 0, 0)


@pytest.mark.parametrize("seed", range(6))
def test_host_counters_follow_the_oracle_policy(seed):
    r = np.random.default_rng(seed)
    M, R = int(r.integers(1, 9)), int(r.integers(0, 4))
    C_ = R + int(r.integers(1, 7))
    cfg = make_config(1, 2, 2, 64, "f32", 4, 1, M, R, C_)
    c = ssd.Cache(cfg, np.array([[0, 1]], np.uint8), device=None)
    u = oracle.Unit(True, 4, 1, M, R, C_)
    for step in range(60):
        rc = u.append()
        if rc != 0:
            with pytest.raises(ssd.SsdError) as e:
                ssd.ssd_append_token(c, 0, 1, FAKE, FAKE)
            assert e.value.code == ssd.SSD_ERR_STAGE_OVERFLOW
            u.compress(); ssd.ssd_compress_kv(c, 0, 1)
            assert u.append() == 0
        ssd.ssd_append_token(c, 0, 1, FAKE, FAKE)
        if r.random() < 0.4:
            u.compress(); ssd.ssd_compress_kv(c, 0, 1)
        hp, _, sp, _ = u.state()
        n, m, cc, base = c.layer_state(0)
        assert (n, m, cc) == (u.n, len(hp), len(sp))
        assert 0 <= base < C_
    # dense-source mode sets the counters as one compression of n_src tokens would
    for n_src in (1, R, R + 1, M + R, M + R + 5):
        if n_src < 1:
            continue
        ssd.ssd_compress_kv(c, 0, 1, FAKE, FAKE, None, n_src)
        v = oracle.Unit(True, 4, 1, M, R, C_)
        v.load_dense(n_src)
        hp, _, sp, _ = v.state()
        assert c.layer_state(0) == (n_src, len(hp), len(sp), 0)


def test_dense_and_classify_argument_checks():
    lib = ssd.lib
    ok = dict(B=2, H=2, d=64, dtype=0, n_cap=8, n=8)
    def dense(**kw):
        a = dict(ok); a.update(kw)
        return lib.ssd_dense_decode_attn(kw.get("q", FAKE), FAKE, FAKE, FAKE, a["B"], a["H"], a["d"], a["dtype"], a["n_cap"],
                                         a["n"], 0.0, kw.get("far"), kw.get("tot"), 1, 0, 32, None, 0, None)
    assert dense(q=None) == ssd.SSD_ERR_INVALID_ARG
    assert dense(d=80) == ssd.SSD_ERR_INVALID_ARG
    assert dense(n=9) == ssd.SSD_ERR_INVALID_ARG
    assert dense(n=0) == ssd.SSD_ERR_INVALID_ARG
    assert dense(dtype=3) == ssd.SSD_ERR_INVALID_ARG
    assert dense(far=FAKE) == ssd.SSD_ERR_INVALID_ARG              # far without tot
    assert ssd.ssd_dense_workspace_bytes(2, 2, 64, 100) >= 2 * 2 * 68 * 4
    assert lib.ssd_classify_heads(None, FAKE, 1, 1, 1, 1, 0.5, FAKE, FAKE, None) == ssd.SSD_ERR_INVALID_ARG
    assert lib.ssd_classify_heads(FAKE, FAKE, 1, 0, 1, 1, 0.5, FAKE, FAKE, None) == ssd.SSD_ERR_INVALID_ARG
    assert lib.ssd_classify_heads(FAKE, FAKE, 1, 1, 1, 1, 0.5, None, None, None) == ssd.SSD_ERR_INVALID_ARG


@pytest.mark.parametrize("seed", range(4))
def test_fused_step_counters_equal_the_three_calls(seed):
    r = np.random.default_rng(50 + seed)
    M, R = int(r.integers(1, 9)), int(r.integers(0, 4))
    C_ = R + int(r.integers(1, 7))
    cfg = make_config(3, 2, 4, 64, "f32", 5, 1, M, R, C_)
    ht = np.array([[0, 0, 1, 1], [0, 0, 0, 0], [1, 1, 1, 1]], np.uint8)     # one layer has no row buffer
    a = ssd.Cache(cfg, ht, device=None)
    b = ssd.Cache(cfg, ht, device=None)
    for step in range(50):
        full = a.layer_state(0)[2] >= C_
        comp = bool(r.random() < 0.5) or a.layer_state(0)[2] + 1 >= C_
        if full:
            with pytest.raises(ssd.SsdError) as e:
                ssd.ssd_decode_step(a, 0, 3, FAKE, FAKE, FAKE, FAKE, True, comp)
            assert e.value.code == ssd.SSD_ERR_STAGE_OVERFLOW
            ssd.ssd_compress_kv(a, 0, 3); ssd.ssd_compress_kv(b, 0, 3)
        ssd.ssd_decode_step(a, 0, 3, FAKE, FAKE, FAKE, FAKE, True, comp)
        ssd.ssd_append_token(b, 0, 3, FAKE, FAKE)
        ssd.ssd_decode_attn(b, 0, 3, FAKE, FAKE, True)
        if comp:
            ssd.ssd_compress_kv(b, 0, 3)
        for l in range(3):
            assert a.layer_state(l) == b.layer_state(l), (step, l)
    assert a.layer_state(1)[1:] == (0, 0, 0)
    for args in [(None, FAKE, FAKE, FAKE), (FAKE, None, FAKE, FAKE), (FAKE, FAKE, FAKE, None), (FAKE, FAKE + 8, FAKE, FAKE)]:
        with pytest.raises(ssd.SsdError) as e:
            ssd.ssd_decode_step(a, 0, 3, *args)
        assert e.value.code == ssd.SSD_ERR_INVALID_ARG
    with pytest.raises(ssd.SsdError) as e:
        ssd.ssd_decode_step(a, 1, 4, FAKE, FAKE, FAKE, FAKE)
    assert e.value.code == ssd.SSD_ERR_LAYER_RANGE


def test_algorithm2_mode_counters_and_limits():
    cfg = make_config(2, 2, 4, 64, "f32", 6, 1, 4, 0, 3, 0.0, 1)
    ht = np.array([[0, 0, 0, 0], [0, 0, 1, 1]], np.uint8)
    c = ssd.Cache(cfg, ht, device=None)
    u = oracle.Unit(False, 6, 1, 4, 0, 3, buffered_spatial=True)
    assert c.export_slots == 1 + 6 + 3
    for step in range(20):
        if u.append() != 0:
            with pytest.raises(ssd.SsdError) as e:
                ssd.ssd_append_token(c, 0, 2, FAKE, FAKE)          # the all-spatial layer has a row buffer too
            assert e.value.code == ssd.SSD_ERR_STAGE_OVERFLOW
            u.compress(); ssd.ssd_compress_kv(c, 0, 2)
            assert c.layer_window(0) == c.layer_state(0)[0] == u.n
            assert u.append() == 0
        ssd.ssd_append_token(c, 0, 2, FAKE, FAKE)
        assert c.layer_state(0)[0] == u.n and c.layer_state(0)[2] == c.layer_state(1)[2]
    cfg.spatial_row_buffer = 2
    assert ssd.ssd_cache_bytes(cfg, ht) == 0


def test_prefill_scores_rejects_bad_arguments_before_any_launch():
    ok = dict(Q=FAKE, K=FAKE, n_units=4, n_src=64, d=128, dtype=ssd.SSD_BF16, scale=0.0, out=FAKE)

    def call(**kw):
        a = dict(ok, **kw)
        return ssd.lib.ssd_prefill_scores(a["Q"], a["K"], a["n_units"], a["n_src"], a["d"], a["dtype"], a["scale"], a["out"], None)

    for bad in (dict(Q=None), dict(K=None), dict(out=None), dict(Q=FAKE + 8), dict(n_units=0), dict(n_src=0), dict(n_src=4097),
                dict(d=96), dict(dtype=7), dict(scale=-1.0), dict(scale=float("nan"))):
        assert call(**bad) == ssd.SSD_ERR_INVALID_ARG, bad
        assert ssd.ssd_last_error() != ""


def test_per_layer_window_and_budget_layout_counters_and_limits():
    L, B, H, d, S, R, C_ = 3, 2, 4, 64, 1, 1, 3
    Wl, Ml = [8, 3, 16], [5, 12, 2]
    cfg = make_config(L, B, H, d, "f32", 99, S, 99, R, C_)
    ht = _ht(L, H)                                   # two spatial, two semantic heads per layer
    row = d * 4
    want = sum(B * 2 * 2 * (S + w) * row + B * 2 * 2 * (m + C_) * row + 2 * B * 2 * (m + C_) * 4 for w, m in zip(Wl, Ml))
    got = ssd.ssd_cache_bytes(cfg, ht, Wl, Ml)
    assert want <= got <= want + 4 * 256 * L
    assert got < ssd.ssd_cache_bytes(cfg, ht)        # the per-layer values replace the config's (99, 99)
    # either array alone; the config value fills in for the other
    assert ssd.ssd_cache_bytes(cfg, ht, Wl, None) > ssd.ssd_cache_bytes(cfg, ht, Wl, Ml)
    c = ssd.Cache(cfg, ht, device=None, window=Wl, budget=Ml)
    assert [c.layer_budget(l) for l in range(L)] == list(zip(Wl, Ml))
    assert c.export_slots == max(max(S + w for w in Wl), max(m + C_ for m in Ml))
    # counters: each layer's heavy count saturates at its own budget
    units = [oracle.Unit(True, Wl[l], S, Ml[l], R, C_) for l in range(L)]
    for step in range(30):
        ssd.ssd_decode_step(c, 0, L, FAKE, FAKE, FAKE, FAKE, True, step % 2 == 1)
        for u in units:
            assert u.append() == 0
            if step % 2 == 1:
                u.compress()
        for l, u in enumerate(units):
            hp, _, sp, _ = u.state()
            assert c.layer_state(l)[:3] == (u.n, len(hp), len(sp))
    assert [c.layer_state(l)[1] for l in range(L)] == Ml
    # dense-source mode: the same per layer
    ssd.ssd_compress_kv(c, 0, L, FAKE, FAKE, None, 10)
    assert [c.layer_state(l)[1] for l in range(L)] == [min(m, 10 - R) for m in Ml]
    # limits hold per entry
    for bad_w, bad_m in (([8, 0, 16], Ml), (Wl, [5, 0, 2]), (Wl, [5, 4094, 2]), ([8, 70000, 16], Ml)):
        assert ssd.ssd_cache_bytes(cfg, ht, bad_w, bad_m) == 0
        with pytest.raises(ssd.SsdError):
            ssd.Cache(cfg, ht, device=None, window=bad_w, budget=bad_m)
    with pytest.raises(ValueError):
        ssd.Cache(cfg, ht, device=None, window=[1, 2])


def test_per_head_budgets_layout_counters_and_limits():
    L, B, H, d, S, R, C_ = 2, 2, 4, 64, 1, 1, 3
    ht = _ht(L, H)                                   # two spatial, two semantic heads per layer
    hb = np.array([[8, 3, 5, 12], [16, 2, 7, 1]], np.int32)
    # (entry = W_h for the spatial heads 0 and 1, M_h for the semantic heads 2 and 3)
    cfg = make_config(L, B, H, d, "f32", 99, S, 99, R, C_)
    # units are sized for the largest head of their type in the layer: the layout equals the per-layer one with the maxima
    Wl = [int(hb[l][ht[l] == 0].max()) for l in range(L)]
    Ml = [int(hb[l][ht[l] == 1].max()) for l in range(L)]
    assert ssd.ssd_cache_bytes(cfg, ht, head_budget=hb) == ssd.ssd_cache_bytes(cfg, ht, Wl, Ml)
    c = ssd.Cache(cfg, ht, device=None, head_budget=hb)
    assert [c.layer_budget(l) for l in range(L)] == list(zip(Wl, Ml))
    assert [[c.head_budget(l, h) for h in range(H)] for l in range(L)] == hb.tolist()
    assert c.export_slots == max(max(S + w for w in Wl), max(m + C_ for m in Ml))
    # a cache with uniform budgets answers the same query from its layer values
    cu = ssd.Cache(cfg, ht, device=None)
    assert [cu.head_budget(0, h) for h in range(H)] == [99] * H
    # counters: the layer's heavy count is that of its largest semantic head
    units = [oracle.Unit(True, 1, S, Ml[l], R, C_) for l in range(L)]
    for step in range(40):
        ssd.ssd_decode_step(c, 0, L, FAKE, FAKE, FAKE, FAKE, True, step % 2 == 1)
        for u in units:
            assert u.append() == 0
            if step % 2 == 1:
                u.compress()
        for l, u in enumerate(units):
            hp, _, sp, _ = u.state()
            assert c.layer_state(l)[:3] == (u.n, len(hp), len(sp))
    assert [c.layer_state(l)[1] for l in range(L)] == Ml
    # limits hold per entry, by head type; the arrays are not mixed with per-layer ones
    for l, h, v in ((0, 0, 0), (0, 0, 70000), (1, 3, 0), (1, 3, 4094)):
        bad = hb.copy()
        bad[l, h] = v
        assert ssd.ssd_cache_bytes(cfg, ht, head_budget=bad) == 0
        with pytest.raises(ssd.SsdError):
            ssd.Cache(cfg, ht, device=None, head_budget=bad)
    with pytest.raises(ValueError):
        ssd.Cache(cfg, ht, device=None, head_budget=hb[:1])
    with pytest.raises(ValueError):
        ssd.Cache(cfg, ht, device=None, window=Wl, head_budget=hb)
    with pytest.raises(ssd.SsdError):
        c.head_budget(0, H)


def test_cfg_mix_rejects_bad_arguments_before_any_launch():
    ok = dict(p=FAKE, n_seqs=4, V=64, dtype=ssd.SSD_BF16, gamma=5.0, out=FAKE)

    def call(**kw):
        a = dict(ok, **kw)
        return ssd.lib.ssd_cfg_mix(a["p"], a["n_seqs"], a["V"], a["dtype"], a["gamma"], a["out"], None)

    for bad in (dict(p=None), dict(out=None), dict(p=FAKE + 4), dict(out=FAKE + 8), dict(n_seqs=0), dict(n_seqs=3), dict(V=0),
                dict(dtype=2), dict(gamma=float("inf")), dict(gamma=float("nan"))):
        assert call(**bad) == ssd.SSD_ERR_INVALID_ARG, bad
        assert ssd.ssd_last_error() != ""


@pytest.mark.parametrize("seed", range(24))
def test_slot_arithmetic_holds_the_oracles_retained_sets(seed):
    """The valid-slot runs and ring slots the kernels compute (the same host/device functions) against the oracle's
    position sets, step by step, without a GPU: every retained position of a spatial head has its own slot inside
    the runs and nothing else is in them; a semantic head's runs have as many slots as it retains tokens."""
    r = np.random.default_rng(300 + seed)
    L, B, H, d = 2, 2, int(r.integers(2, 7)), 64
    S, R = int(r.integers(0, 4)), int(r.integers(0, 3))
    cadence = int(r.integers(1, 7))
    C_ = R + cadence + int(r.integers(0, 2))
    alg2 = bool(r.integers(0, 2))
    ht = (r.random((L, H)) < 0.5).astype(np.uint8)
    per_head = bool(r.integers(0, 2))
    hb = r.integers(1, 12, (L, H)).astype(np.int32)
    W, M = int(r.integers(1, 12)), int(r.integers(1, 12))
    cfg = make_config(L, B, H, d, "bf16", W, S, M, R, C_, 0.0, int(alg2))
    c = ssd.Cache(cfg, ht, device=None, head_budget=hb if per_head else None)
    units = [[oracle.Unit(bool(ht[l, h]), int(hb[l, h]) if per_head else W, S, int(hb[l, h]) if per_head else M, R, C_,
                          buffered_spatial=alg2) for h in range(H)] for l in range(L)]
    for step in range(45):
        comp = (step + 1) % cadence == 0
        ssd.ssd_append_token(c, 0, L, FAKE, FAKE)
        for l in range(L):
            for h in range(H):
                u = units[l][h]
                assert u.append() == 0
                runs = c.head_runs(l, h)
                slots = [s for (a, n) in runs for s in range(a, a + n)]
                assert len(slots) == len(set(slots))
                kept = u.retained()
                if ht[l, h] == 0:
                    assert sorted(c.spatial_slot(l, h, int(p)) for p in kept) == sorted(slots), (l, h, step)
                    if alg2:    # the runs of Algorithm 2's ring follow the positions, oldest first
                        by_slot = {c.spatial_slot(l, h, int(p)): int(p) for p in kept}
                        ring = [by_slot[s] for s in slots if s >= S]
                        assert ring == sorted(ring)
                else:
                    assert len(slots) == len(kept), (l, h, step)
        if comp:
            ssd.ssd_compress_kv(c, 0, L)
            for row in units:
                for u in row:
                    u.compress()
    with pytest.raises(ssd.SsdError):
        c.head_runs(0, H)
    sem = [(l, h) for l in range(L) for h in range(H) if ht[l, h] == 1]
    if sem:
        with pytest.raises(ssd.SsdError):
            c.spatial_slot(sem[0][0], sem[0][1], 0)


def test_rotary_step_rejects_bad_arguments_and_keeps_the_counters():
    L, B, H, d = 2, 2, 4, 64
    c = ssd.Cache(make_config(L, B, H, d, "bf16", 8, 1, 4, 1, 3), _ht(L, H), device=None)
    ok = dict(q=FAKE, k=FAKE, v=FAKE, out=FAKE, cos=FAKE, sin=FAKE, layout=ssd.SSD_ROPE_HALF)

    def call(**kw):
        a = dict(ok, **kw)
        return ssd.lib.ssd_decode_step_rope(c.handle, 0, L, a["q"], a["k"], a["v"], a["out"], 1, 1, a["cos"], a["sin"], a["layout"], None)

    for bad in (dict(cos=None), dict(sin=None), dict(cos=FAKE + 4), dict(sin=FAKE + 8), dict(layout=0), dict(layout=3), dict(q=None),
                dict(k=FAKE + 2)):
        assert call(**bad) == ssd.SSD_ERR_INVALID_ARG, bad
        assert ssd.ssd_last_error() != ""
        assert c.layer_state(0)[0] == 0                  # a refused call appends nothing
    assert ssd.lib.ssd_decode_step_rope(c.handle, 0, L + 1, FAKE, FAKE, FAKE, FAKE, 1, 1, FAKE, FAKE, 1, None) == ssd.SSD_ERR_LAYER_RANGE
    # accepted calls move the counters exactly like the plain fused step
    c2 = ssd.Cache(make_config(L, B, H, d, "bf16", 8, 1, 4, 1, 3), _ht(L, H), device=None)
    for step in range(12):
        assert call(layout=1 + step % 2) == ssd.SSD_OK
        ssd.ssd_decode_step(c2, 0, L, FAKE, FAKE, FAKE, FAKE, True, True)
        assert [c.layer_state(l) for l in range(L)] == [c2.layer_state(l) for l in range(L)]


def test_stream_benchmark_rejects_bad_arguments_before_any_launch():
    ok = dict(buf=FAKE, unit_bytes=66 * 512, n_units=4096, rows=2, sink=FAKE)

    def call(**kw):
        a = dict(ok, **kw)
        return ssd.lib.ssd_bench_stream(a["buf"], a["unit_bytes"], a["n_units"], a["rows"], a["sink"], None)

    for bad in (dict(buf=None), dict(sink=None), dict(buf=FAKE + 8), dict(unit_bytes=0), dict(unit_bytes=512), dict(unit_bytes=1000),
                dict(n_units=0), dict(rows=1), dict(rows=3)):
        assert call(**bad) == ssd.SSD_ERR_INVALID_ARG, bad
        assert ssd.ssd_last_error() != ""


def test_copy_benchmark_rejects_bad_arguments_before_any_launch():
    lib = ssd.lib
    for dst, src, nbytes in [(None, FAKE, 1024), (FAKE, None, 1024), (FAKE + 8, FAKE, 1024), (FAKE, FAKE + 4, 1024), (FAKE, FAKE, 0),
                             (FAKE, FAKE, 1000)]:
        assert lib.ssd_bench_copy(dst, src, nbytes, None) == ssd.SSD_ERR_INVALID_ARG, (dst, src, nbytes)
        assert ssd.ssd_last_error() != ""


def test_package_without_its_library_fails_loudly(tmp_path):
    """No CPU or PyTorch fallback: a copy of the package without the built library, on a machine where it
    cannot be built either, must refuse to import."""
    import shutil
    import subprocess
    import sys
    src = os.path.join(ROOT, "paper_2510_18716_amd")
    dst = tmp_path / "paper_2510_18716_amd"
    shutil.copytree(src, dst, ignore=shutil.ignore_patterns("*.so", "*.so.tmp*", "__pycache__"))
    shutil.copytree(os.path.join(ROOT, "include"), tmp_path / "include")
    env = dict(os.environ, HIPCC="/nonexistent/hipcc", PYTHONPATH=str(tmp_path))
    r = subprocess.run([sys.executable, "-c", "import paper_2510_18716_amd"], cwd=str(tmp_path), env=env,
                       stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
    assert r.returncode != 0
    assert "hipcc" in r.stderr or "No such file" in r.stderr
    assert not (dst / "libssd_hip.so").exists()


def test_product_and_oracle_do_not_import_each_other():
    """The oracle is test infrastructure: nothing under the package may name it, and it may not name the package
    (the two share only the input generator)."""
    def sources(top, exts):
        for dirpath, _, files in os.walk(top):
            for f in files:
                if f.endswith(exts):
                    yield os.path.join(dirpath, f)
    for path in sources(os.path.join(ROOT, "paper_2510_18716_amd"), (".py", ".hip", ".h")):
        text = open(path).read()
        assert not re.search(r"^\s*(import|from)\s+oracle\b", text, flags=re.M), path
        assert "ssd_oracle" not in text, path
    for path in sources(os.path.join(ROOT, "oracle"), (".py", ".c", ".h")):
        text = open(path).read()
        assert "paper_2510_18716_amd" not in text and "ssd.h" not in text and "csrc" not in text, path
    wl = open(os.path.join(ROOT, "workload", "__init__.py")).read()
    assert not re.search(r"^\s*(import|from)\s+(oracle|paper_2510_18716_amd)\b", wl, flags=re.M)


def test_split_step_checks_its_stream_list_and_moves_the_counters_once():
    """ssd_decode_step_split on the host: the counters advance once per call whatever the number of streams (the
    parts of the batch move together), and a bad stream list or sync value is refused before anything else."""
    import ctypes as C
    cfg = make_config(3, 10, 4, 64, "f32", 5, 1, 4, 1, 3)
    ht = np.array([[0, 0, 1, 1], [0, 0, 0, 0], [1, 1, 1, 1]], np.uint8)
    a = ssd.Cache(cfg, ht, device=None)
    b = ssd.Cache(cfg, ht, device=None)
    fake_streams = [FAKE + 64 * i for i in range(1, 5)]           # never dereferenced: launches are off
    for step in range(12):
        comp = step % 2 == 1
        n = 1 + step % ssd.SSD_MAX_SPLIT
        ssd.ssd_decode_step_split(a, 0, 3, FAKE, FAKE, FAKE, FAKE, fake_streams[:n], ssd.SSD_SPLIT_FORK | ssd.SSD_SPLIT_JOIN, True, comp)
        ssd.ssd_decode_step(b, 0, 3, FAKE, FAKE, FAKE, FAKE, True, comp)
        for l in range(3):
            assert a.layer_state(l) == b.layer_state(l), (step, l)
    lib = ssd.lib
    arr = ssd.stream_array(fake_streams)
    ok = (a.handle, 0, 3, FAKE, FAKE, FAKE, FAKE, 1, 1)
    before = [a.layer_state(l) for l in range(3)]
    assert lib.ssd_decode_step_split(*ok, None, 2, 0) == ssd.SSD_ERR_INVALID_ARG
    assert lib.ssd_decode_step_split(*ok, arr, 0, 0) == ssd.SSD_ERR_INVALID_ARG
    assert lib.ssd_decode_step_split(*ok, arr, ssd.SSD_MAX_SPLIT + 1, 0) == ssd.SSD_ERR_INVALID_ARG
    assert lib.ssd_decode_step_split(*ok, arr, 2, 4) == ssd.SSD_ERR_INVALID_ARG                   # unknown sync bit
    assert "sync" in ssd.ssd_last_error()
    dup = (C.c_void_p * 2)(fake_streams[0], fake_streams[0])
    assert lib.ssd_decode_step_split(*ok, dup, 2, 0) == ssd.SSD_ERR_INVALID_ARG                   # the same stream twice
    assert lib.ssd_decode_step_split(a.handle, 0, 3, None, FAKE, FAKE, FAKE, 1, 1, arr, 2, 0) == ssd.SSD_ERR_INVALID_ARG
    assert lib.ssd_decode_step_split(a.handle, 2, 4, FAKE, FAKE, FAKE, FAKE, 1, 1, arr, 2, 0) == ssd.SSD_ERR_LAYER_RANGE
    assert [a.layer_state(l) for l in range(3)] == before          # a refused call changes nothing
    # a full row buffer refuses the whole call, as in ssd_decode_step
    for _ in range(2):
        ssd.ssd_decode_step_split(a, 0, 3, FAKE, FAKE, FAKE, FAKE, fake_streams[:2], 0, True, False)
    with pytest.raises(ssd.SsdError) as e:
        ssd.ssd_decode_step_split(a, 0, 3, FAKE, FAKE, FAKE, FAKE, fake_streams[:2], 0, True, False)
    assert e.value.code == ssd.SSD_ERR_STAGE_OVERFLOW


def test_split_plan_keeps_prompt_pairs_together_and_launches_near_one_resident_round():
    def plan(B, H, L, layers, n):
        c = ssd.Cache(make_config(L, B, H, 128, "bf16", 8, 1, 8, 1, 2), _ht(L, H), device=None)
        return c.split_plan(layers, n)
    assert plan(128, 32, 30, 1, 1) == (128, 1)                # one stream: one part
    assert plan(128, 32, 30, 1, 2) == (64, 2)                 # 7B shape: 2048 units per launch, one part per stream
    assert plan(128, 32, 30, 1, 4) == (32, 4)
    assert plan(512, 32, 30, 1, 2) == (128, 4)                # large batch: 4096 units per launch, two parts per stream
    assert plan(512, 32, 30, 1, 1) == (512, 1)
    assert plan(512, 32, 30, 30, 2) == (64, 8)                # many layers per call: never more than four parts per stream
    assert plan(32, 16, 24, 1, 2) == (16, 2)
    assert plan(10, 4, 2, 1, 3) == (4, 3)                     # 4 + 4 + 2
    assert plan(10, 4, 2, 1, 4) == (4, 3)                     # fewer parts than streams when pairs run out
    assert plan(3, 4, 2, 1, 2) == (2, 2)
    for B, H, L, layers, n in [(2, 1, 1, 1, 4), (65534, 2, 1, 1, 3), (100, 128, 3, 3, 2), (6, 128, 40, 32, 4)]:
        P, parts = plan(B, H, L, layers, n)
        assert P % 2 == 0 and P >= 2 and (parts - 1) * P < B <= parts * P and parts <= 4 * n
    c = ssd.Cache(make_config(2, 4, 4, 64, "f32", 5, 1, 4, 1, 3), _ht(2, 4), device=None)
    import ctypes as C
    for layers, n in [(0, 1), (3, 1), (1, 0), (1, ssd.SSD_MAX_SPLIT + 1)]:
        assert ssd.lib.ssd_decode_step_split_plan(c.handle, layers, n, None, None) == ssd.SSD_ERR_INVALID_ARG
    assert ssd.lib.ssd_decode_step_split_plan(None, 1, 1, None, None) == ssd.SSD_ERR_INVALID_ARG
    assert ssd.lib.ssd_decode_step_split_plan(c.handle, 1, 2, None, None) == ssd.SSD_OK


def test_launch_shape_hook_accepts_only_shapes_the_library_has():
    cfg = make_config(1, 2, 4, 64, "f32", 5, 1, 4, 1, 3)
    a = ssd.Cache(cfg, _ht(1, 4), device=None)
    for ch, wpb, rows in [(0, 0, 0), (1, 1, 1), (2, 2, 2), (4, 4, 0), (2, 12, 1), (4, 14, 2)]:
        a.set_launch_shape(ch, wpb, rows)
    for ch, wpb, rows in [(3, 1, 0), (8, 1, 0), (1, 3, 0), (1, 8, 0), (1, 13, 0), (1, 1, 3), (1, 1, -1), (-1, 0, 0)]:
        with pytest.raises(ssd.SsdError) as e:
            a.set_launch_shape(ch, wpb, rows)
        assert e.value.code == ssd.SSD_ERR_INVALID_ARG
    assert ssd.lib.ssd_cache_set_launch_shape(None, 0, 0, 0) == ssd.SSD_ERR_INVALID_ARG
    # results of host-side calls are unaffected
    ssd.ssd_decode_step(a, 0, 1, FAKE, FAKE, FAKE, FAKE, True, True)
    assert a.layer_state(0)[0] == 1
    # no launch has happened (launches are off): nothing to report yet
    assert a.last_launch_shape() == (0, 0, 0)
    assert ssd.lib.ssd_cache_last_launch_shape(None, None) == ssd.SSD_ERR_INVALID_ARG
    assert ssd.lib.ssd_cache_last_launch_shape(a.handle, None) == ssd.SSD_ERR_INVALID_ARG


def test_dense_split_hook_rejects_bad_split_counts_before_any_launch():
    lib = ssd.lib
    ok = (FAKE, FAKE, FAKE, FAKE, 1, 1, 64, ssd.SSD_F32, 8, 4, 0.0, None, None, 1, 0, 32)
    assert lib.ssd_dense_decode_attn_splits(*ok, -1, FAKE, 1 << 20, None) == ssd.SSD_ERR_INVALID_ARG
    assert lib.ssd_dense_decode_attn_splits(*ok, 65, FAKE, 1 << 20, None) == ssd.SSD_ERR_INVALID_ARG
    assert "splits" in ssd.ssd_last_error()
    assert lib.ssd_dense_decode_attn_splits(*ok, 4, None, 0, None) == ssd.SSD_ERR_INVALID_ARG      # splits need a workspace
    assert lib.ssd_dense_decode_attn_splits(*ok, 4, FAKE, 16, None) == ssd.SSD_ERR_INVALID_ARG     # ... that is large enough


def test_rotary_split_step_checks_rotary_and_stream_arguments():
    cfg = make_config(2, 4, 4, 64, "f32", 5, 1, 4, 1, 3)
    a = ssd.Cache(cfg, _ht(2, 4), device=None)
    b = ssd.Cache(cfg, _ht(2, 4), device=None)
    lib = ssd.lib
    arr = ssd.stream_array([FAKE + 64, FAKE + 128])
    ok = (a.handle, 0, 2, FAKE, FAKE, FAKE, FAKE, 1, 1)
    assert lib.ssd_decode_step_split_rope(*ok, None, FAKE, ssd.SSD_ROPE_HALF, arr, 2, 0) == ssd.SSD_ERR_INVALID_ARG
    assert lib.ssd_decode_step_split_rope(*ok, FAKE, FAKE + 4, ssd.SSD_ROPE_HALF, arr, 2, 0) == ssd.SSD_ERR_INVALID_ARG
    assert lib.ssd_decode_step_split_rope(*ok, FAKE, FAKE, 3, arr, 2, 0) == ssd.SSD_ERR_INVALID_ARG
    assert lib.ssd_decode_step_split_rope(*ok, FAKE, FAKE, ssd.SSD_ROPE_HALF, None, 2, 0) == ssd.SSD_ERR_INVALID_ARG
    assert lib.ssd_decode_step_split_rope(*ok, FAKE, FAKE, ssd.SSD_ROPE_HALF, arr, 2, 8) == ssd.SSD_ERR_INVALID_ARG
    assert a.layer_state(0)[0] == 0                                 # nothing moved
    ssd.ssd_decode_step_split_rope(a, 0, 2, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, ssd.SSD_ROPE_INTERLEAVED, [FAKE + 64, FAKE + 128],
                                   ssd.SSD_SPLIT_FORK | ssd.SSD_SPLIT_JOIN)
    ssd.ssd_decode_step_rope(b, 0, 2, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, ssd.SSD_ROPE_INTERLEAVED)
    assert [a.layer_state(l) for l in range(2)] == [b.layer_state(l) for l in range(2)]
