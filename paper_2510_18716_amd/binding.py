"""ctypes binding of include/ssd.h and include/ssd_hooks.h.  Same names, same argument order; tensors are passed as
`data_ptr()` and the stream as the raw hipStream_t of torch's current stream."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np
import torch

SSD_F32, SSD_BF16 = 0, 1
SSD_SPATIAL, SSD_SEMANTIC = 0, 1
SSD_OK = 0
SSD_ERR_INVALID_ARG, SSD_ERR_LAYER_RANGE, SSD_ERR_STAGE_OVERFLOW, SSD_ERR_ORDER, SSD_ERR_HIP = -1, -2, -3, -4, -5

_HERE = os.path.dirname(os.path.abspath(__file__))
lib_path = os.path.join(_HERE, "libssd_hip.so")


def _load():
    if not os.path.exists(lib_path):
        # build only if nothing is built; never fall back to another implementation
        from . import build as _b
        _b.build(force=True, verbose=False)
    return C.CDLL(lib_path)


lib = _load()


class SsdConfig(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("n_seqs", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32),
        ("dtype", C.c_int32), ("window", C.c_int32), ("n_init_sink", C.c_int32), ("budget", C.c_int32),
        ("recent", C.c_int32), ("stage_cap", C.c_int32), ("softmax_scale", C.c_float), ("spatial_row_buffer", C.c_int32),
        ("reserved", C.c_int32 * 4),
    ]


_vp = C.c_void_p
lib.ssd_cache_bytes.argtypes = [C.POINTER(SsdConfig), _vp]
lib.ssd_cache_bytes.restype = C.c_size_t
lib.ssd_cache_init.argtypes = [C.POINTER(SsdConfig), _vp, _vp, C.c_size_t, C.POINTER(_vp)]
lib.ssd_cache_init.restype = C.c_int
lib.ssd_cache_bytes_layered.argtypes = [C.POINTER(SsdConfig), _vp, _vp, _vp]
lib.ssd_cache_bytes_layered.restype = C.c_size_t
lib.ssd_cache_init_layered.argtypes = [C.POINTER(SsdConfig), _vp, _vp, _vp, _vp, C.c_size_t, C.POINTER(_vp)]
lib.ssd_cache_init_layered.restype = C.c_int
lib.ssd_cache_layer_budget.argtypes = [_vp, C.c_int, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
lib.ssd_cache_layer_budget.restype = C.c_int
lib.ssd_cache_bytes_heads.argtypes = [C.POINTER(SsdConfig), _vp, _vp]
lib.ssd_cache_bytes_heads.restype = C.c_size_t
lib.ssd_cache_init_heads.argtypes = [C.POINTER(SsdConfig), _vp, _vp, _vp, C.c_size_t, C.POINTER(_vp)]
lib.ssd_cache_init_heads.restype = C.c_int
lib.ssd_cache_head_budget.argtypes = [_vp, C.c_int, C.c_int, C.POINTER(C.c_int32)]
lib.ssd_cache_head_budget.restype = C.c_int
lib.ssd_cache_head_runs.argtypes = [_vp, C.c_int, C.c_int, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
lib.ssd_cache_head_runs.restype = C.c_int
lib.ssd_cache_spatial_slot.argtypes = [_vp, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int32)]
lib.ssd_cache_spatial_slot.restype = C.c_int
lib.ssd_cache_free.argtypes = [_vp]
lib.ssd_cache_free.restype = None
lib.ssd_cache_reset.argtypes = [_vp]
lib.ssd_cache_reset.restype = C.c_int
lib.ssd_cache_layer_state.argtypes = [_vp, C.c_int, C.POINTER(C.c_int32 * 4)]
lib.ssd_cache_layer_state.restype = C.c_int
lib.ssd_cache_layer_window.argtypes = [_vp, C.c_int, C.POINTER(C.c_int32)]
lib.ssd_cache_layer_window.restype = C.c_int
lib.ssd_cache_set_launch.argtypes = [_vp, C.c_int]
lib.ssd_cache_set_launch.restype = C.c_int
lib.ssd_classify_heads.argtypes = [_vp, _vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_float, _vp, _vp, _vp]
lib.ssd_classify_heads.restype = C.c_int
lib.ssd_append_token.argtypes = [_vp, C.c_int, C.c_int, _vp, _vp, _vp]
lib.ssd_append_token.restype = C.c_int
lib.ssd_decode_attn.argtypes = [_vp, C.c_int, C.c_int, _vp, _vp, C.c_int, _vp]
lib.ssd_decode_attn.restype = C.c_int
lib.ssd_decode_step.argtypes = [_vp, C.c_int, C.c_int, _vp, _vp, _vp, _vp, C.c_int, C.c_int, _vp]
lib.ssd_decode_step.restype = C.c_int
lib.ssd_decode_step_rope.argtypes = [_vp, C.c_int, C.c_int, _vp, _vp, _vp, _vp, C.c_int, C.c_int, _vp, _vp, C.c_int, _vp]
lib.ssd_decode_step_rope.restype = C.c_int
lib.ssd_bench_stream.argtypes = [_vp, C.c_size_t, C.c_longlong, C.c_int, _vp, _vp]
lib.ssd_bench_stream.restype = C.c_int
lib.ssd_bench_copy.argtypes = [_vp, _vp, C.c_size_t, _vp]
lib.ssd_bench_copy.restype = C.c_int
lib.ssd_compress_kv.argtypes = [_vp, C.c_int, C.c_int, _vp, _vp, _vp, C.c_int, _vp]
lib.ssd_compress_kv.restype = C.c_int
lib.ssd_prefill_scores.argtypes = [_vp, _vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_float, _vp, _vp]
lib.ssd_prefill_scores.restype = C.c_int
lib.ssd_cfg_mix.argtypes = [_vp, C.c_int, C.c_int, C.c_int, C.c_float, _vp, _vp]
lib.ssd_cfg_mix.restype = C.c_int
lib.ssd_cache_export_slots.argtypes = [_vp]
lib.ssd_cache_export_slots.restype = C.c_int
lib.ssd_cache_export.argtypes = [_vp, C.c_int, _vp, _vp, _vp, _vp]
lib.ssd_cache_export.restype = C.c_int
lib.ssd_dense_workspace_bytes.argtypes = [C.c_int] * 4
lib.ssd_dense_workspace_bytes.restype = C.c_size_t
lib.ssd_dense_decode_attn.argtypes = [_vp, _vp, _vp, _vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                      C.c_float, _vp, _vp, C.c_int, C.c_int, C.c_int, _vp, C.c_size_t, _vp]
lib.ssd_dense_decode_attn.restype = C.c_int
lib.ssd_dense_decode_attn_static.argtypes = [_vp, _vp, _vp, _vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                             C.c_float, _vp, _vp, C.c_int, C.c_int, C.c_int, _vp]
lib.ssd_dense_decode_attn_static.restype = C.c_int
lib.ssd_last_error.argtypes = []
lib.ssd_last_error.restype = C.c_char_p
lib.ssd_version.argtypes = []
lib.ssd_version.restype = C.c_int
lib.ssd_cache_set_launch_shape.argtypes = [_vp, C.c_int, C.c_int, C.c_int]
lib.ssd_cache_set_launch_shape.restype = C.c_int
lib.ssd_cache_last_launch_shape.argtypes = [_vp, C.POINTER(C.c_int32)]
lib.ssd_cache_last_launch_shape.restype = C.c_int
lib.ssd_dense_decode_attn_splits.argtypes = [_vp, _vp, _vp, _vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                             C.c_float, _vp, _vp, C.c_int, C.c_int, C.c_int, C.c_int, _vp, C.c_size_t, _vp]
lib.ssd_dense_decode_attn_splits.restype = C.c_int
lib.ssd_decode_step_split.argtypes = [_vp, C.c_int, C.c_int, _vp, _vp, _vp, _vp, C.c_int, C.c_int, C.POINTER(_vp), C.c_int, C.c_int]
lib.ssd_decode_step_split.restype = C.c_int
lib.ssd_decode_step_split_rope.argtypes = [_vp, C.c_int, C.c_int, _vp, _vp, _vp, _vp, C.c_int, C.c_int, _vp, _vp, C.c_int,
                                           C.POINTER(_vp), C.c_int, C.c_int]
lib.ssd_decode_step_split_rope.restype = C.c_int
lib.ssd_decode_step_split_plan.argtypes = [_vp, C.c_int, C.c_int, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
lib.ssd_decode_step_split_plan.restype = C.c_int


class SsdError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s failed with %d: %s" % (where, code, ssd_last_error()))


def ssd_last_error() -> str:
    return lib.ssd_last_error().decode()


def ssd_version() -> int:
    return lib.ssd_version()


def _check(rc: int, where: str) -> None:
    if rc != SSD_OK:
        raise SsdError(rc, where)


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_contiguous(), "tensors handed to the library must be contiguous"
    return t.data_ptr()


def _stream(stream=None) -> Optional[int]:
    if stream is not None:
        return stream if isinstance(stream, int) else stream.cuda_stream
    if torch.cuda.is_available():
        return torch.cuda.current_stream().cuda_stream
    return None


def _dtype_code(dt) -> int:
    if isinstance(dt, int):
        return dt                      # passed through; the library validates it
    if dt in (torch.bfloat16, "bf16"):
        return SSD_BF16
    if dt in (torch.float32, "f32"):
        return SSD_F32
    raise ValueError("unsupported dtype %r" % (dt,))


def make_config(L, B, H, d, dtype, W, S, M, R, C_, softmax_scale=0.0, spatial_row_buffer=0) -> SsdConfig:
    cfg = SsdConfig()
    cfg.n_layers, cfg.n_seqs, cfg.n_heads, cfg.head_dim = L, B, H, d
    cfg.dtype = _dtype_code(dtype)
    cfg.window, cfg.n_init_sink, cfg.budget, cfg.recent, cfg.stage_cap = W, S, M, R, C_
    cfg.softmax_scale = softmax_scale
    cfg.spatial_row_buffer = int(spatial_row_buffer)
    return cfg


def _per_layer(x, L):
    """Host int32 [L] array for a per-layer window / budget list, or None."""
    if x is None:
        return None
    a = np.ascontiguousarray(x, dtype=np.int32)
    if a.shape != (L,):
        raise ValueError("per-layer array must have one entry per layer")
    return a


def _per_head(x, L, H):
    """Host int32 [L*H] array of per-head budgets, or None."""
    if x is None:
        return None
    a = np.ascontiguousarray(x, dtype=np.int32)
    if a.size != L * H:
        raise ValueError("per-head array must have one entry per (layer, head)")
    return a.reshape(-1)


def ssd_cache_bytes(cfg: SsdConfig, head_type: np.ndarray, window=None, budget=None, head_budget=None) -> int:
    ht = np.ascontiguousarray(head_type, dtype=np.uint8)
    hb = _per_head(head_budget, cfg.n_layers, cfg.n_heads)
    if hb is not None:
        return lib.ssd_cache_bytes_heads(C.byref(cfg), ht.ctypes.data, hb.ctypes.data)
    w, m = _per_layer(window, cfg.n_layers), _per_layer(budget, cfg.n_layers)
    return lib.ssd_cache_bytes_layered(C.byref(cfg), ht.ctypes.data, None if w is None else w.ctypes.data,
                                       None if m is None else m.ctypes.data)


class Cache:
    """Owner of one ssd_cache descriptor and of the torch tensor that backs it in HBM.

    `device=None` creates a descriptor over a fake, never dereferenced address with launches
    switched off: the host-side logic (validation, counters, error codes) can then be exercised
    on a machine without a GPU.
    """

    def __init__(self, cfg: SsdConfig, head_type: np.ndarray, device="cuda", window=None, budget=None, head_budget=None):
        """window, budget: optional per-layer lists [L] (ssd_cache_init_layered);
        head_budget: optional [L, H] array, W_h of a spatial head / M_h of a semantic head (ssd_cache_init_heads)."""
        self.cfg = cfg
        self.head_type = np.ascontiguousarray(head_type, dtype=np.uint8)
        w, m = _per_layer(window, cfg.n_layers), _per_layer(budget, cfg.n_layers)
        hb = _per_head(head_budget, cfg.n_layers, cfg.n_heads)
        if hb is not None and (w is not None or m is not None):
            raise ValueError("budgets are given per layer or per head, not both")
        wp, mp = (None if w is None else w.ctypes.data), (None if m is None else m.ctypes.data)
        if hb is not None:
            nbytes = lib.ssd_cache_bytes_heads(C.byref(cfg), self.head_type.ctypes.data, hb.ctypes.data)
        else:
            nbytes = lib.ssd_cache_bytes_layered(C.byref(cfg), self.head_type.ctypes.data, wp, mp)
        if nbytes == 0:
            raise SsdError(SSD_ERR_INVALID_ARG, "ssd_cache_bytes")
        self.head_type = self.head_type.reshape(cfg.n_layers, cfg.n_heads)
        self.nbytes = nbytes
        self._h = _vp()
        if device is None:
            self.mem = None
            base = 1 << 20
        else:
            self.mem = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
            base = (self.mem.data_ptr() + 255) // 256 * 256
        if hb is not None:
            _check(lib.ssd_cache_init_heads(C.byref(cfg), self.head_type.ctypes.data, hb.ctypes.data, base, nbytes, C.byref(self._h)),
                   "ssd_cache_init_heads")
        else:
            _check(lib.ssd_cache_init_layered(C.byref(cfg), self.head_type.ctypes.data, wp, mp, base, nbytes, C.byref(self._h)),
                   "ssd_cache_init")
        if device is None:
            _check(lib.ssd_cache_set_launch(self._h, 0), "ssd_cache_set_launch")
        self.torch_dtype = torch.bfloat16 if cfg.dtype == SSD_BF16 else torch.float32

    def __del__(self):
        h = getattr(self, "_h", None)
        if h is not None and h.value:
            lib.ssd_cache_free(h)
            self._h = None

    @property
    def handle(self):
        return self._h

    def reset(self):
        _check(lib.ssd_cache_reset(self._h), "ssd_cache_reset")

    def set_launch_shape(self, ch: int = 0, wpb: int = 0, new_rows: int = 0):
        """Test / sweep hook: override the attention launch shape of this cache ((0, 0, 0) = the library's choice)."""
        _check(lib.ssd_cache_set_launch_shape(self._h, ch, wpb, new_rows), "ssd_cache_set_launch_shape")

    def last_launch_shape(self):
        """Test hook: (ch, wpb, new_rows) of the newest attention / step launch, in set_launch_shape's codes."""
        out = (C.c_int32 * 3)()
        _check(lib.ssd_cache_last_launch_shape(self._h, out), "ssd_cache_last_launch_shape")
        return tuple(out)

    def split_plan(self, layers_per_call: int, n_streams: int):
        """(sequences per part, number of parts) of ssd_decode_step_split for a call over that many layers."""
        p, n = C.c_int32(0), C.c_int32(0)
        _check(lib.ssd_decode_step_split_plan(self._h, layers_per_call, n_streams, C.byref(p), C.byref(n)), "ssd_decode_step_split_plan")
        return p.value, n.value

    def layer_state(self, layer: int):
        out = (C.c_int32 * 4)()
        _check(lib.ssd_cache_layer_state(self._h, layer, C.byref(out)), "ssd_cache_layer_state")
        return tuple(out)

    def layer_budget(self, layer: int):
        """(W, M) of one layer."""
        w, m = C.c_int32(0), C.c_int32(0)
        _check(lib.ssd_cache_layer_budget(self._h, layer, C.byref(w), C.byref(m)), "ssd_cache_layer_budget")
        return w.value, m.value

    def head_budget(self, layer: int, head: int) -> int:
        """W_h of a spatial head, M_h of a semantic head."""
        v = C.c_int32(0)
        _check(lib.ssd_cache_head_budget(self._h, layer, head, C.byref(v)), "ssd_cache_head_budget")
        return v.value

    def head_runs(self, layer: int, head: int):
        """[(start, len), ...] of the valid-slot runs of one head's unit (host arithmetic only)."""
        st, ln = (C.c_int32 * 3)(), (C.c_int32 * 3)()
        _check(lib.ssd_cache_head_runs(self._h, layer, head, st, ln), "ssd_cache_head_runs")
        return [(st[k], ln[k]) for k in range(3) if ln[k] > 0]

    def spatial_slot(self, layer: int, head: int, position: int) -> int:
        v = C.c_int32(0)
        _check(lib.ssd_cache_spatial_slot(self._h, layer, head, position, C.byref(v)), "ssd_cache_spatial_slot")
        return v.value

    def layer_window(self, layer: int) -> int:
        out = C.c_int32(0)
        _check(lib.ssd_cache_layer_window(self._h, layer, C.byref(out)), "ssd_cache_layer_window")
        return out.value

    @property
    def export_slots(self) -> int:
        return lib.ssd_cache_export_slots(self._h)

    def export(self, layer: int, stream=None):
        """(pos int32 [B,H,slots], count int32 [B,H], score float32 [B,H,slots]) on the cache's device."""
        B, H, slots = self.cfg.n_seqs, self.cfg.n_heads, self.export_slots
        dev = self.mem.device
        pos = torch.empty((B, H, slots), dtype=torch.int32, device=dev)
        cnt = torch.empty((B, H), dtype=torch.int32, device=dev)
        sc = torch.empty((B, H, slots), dtype=torch.float32, device=dev)
        _check(lib.ssd_cache_export(self._h, layer, _ptr(pos), _ptr(cnt), _ptr(sc), _stream(stream)), "ssd_cache_export")
        return pos, cnt, sc


def ssd_append_token(cache: Cache, layer_begin: int, layer_end: int, k_new, v_new, stream=None) -> None:
    _check(lib.ssd_append_token(cache.handle, layer_begin, layer_end, _ptr(k_new), _ptr(v_new), _stream(stream)),
           "ssd_append_token")


def ssd_decode_attn(cache: Cache, layer_begin: int, layer_end: int, q, out, accumulate_scores: bool = True,
                    stream=None) -> None:
    _check(lib.ssd_decode_attn(cache.handle, layer_begin, layer_end, _ptr(q), _ptr(out), int(bool(accumulate_scores)),
                               _stream(stream)), "ssd_decode_attn")


def ssd_decode_step(cache: Cache, layer_begin: int, layer_end: int, q, k_new, v_new, out, accumulate_scores: bool = True,
                    compress: bool = True, stream=None) -> None:
    _check(lib.ssd_decode_step(cache.handle, layer_begin, layer_end, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out),
                               int(bool(accumulate_scores)), int(bool(compress)), _stream(stream)), "ssd_decode_step")


SSD_MAX_SPLIT = 4
SSD_SPLIT_FORK, SSD_SPLIT_JOIN = 1, 2


def stream_array(streams):
    """ctypes array of raw hipStream_t for ssd_decode_step_split (torch streams or raw handles)."""
    raw = [(s if isinstance(s, int) else s.cuda_stream) for s in streams]
    return (_vp * len(raw))(*raw)


def ssd_decode_step_split(cache: Cache, layer_begin: int, layer_end: int, q, k_new, v_new, out, streams, sync: int = 0,
                          accumulate_scores: bool = True, compress: bool = True) -> None:
    arr = streams if isinstance(streams, C.Array) else stream_array(streams)
    _check(lib.ssd_decode_step_split(cache.handle, layer_begin, layer_end, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out),
                                     int(bool(accumulate_scores)), int(bool(compress)), arr, len(arr), int(sync)),
           "ssd_decode_step_split")


SSD_ROPE_HALF, SSD_ROPE_INTERLEAVED = 1, 2


def ssd_decode_step_split_rope(cache: Cache, layer_begin: int, layer_end: int, q, k_new, v_new, out, cos, sin, rope_layout: int,
                               streams, sync: int = 0, accumulate_scores: bool = True, compress: bool = True) -> None:
    arr = streams if isinstance(streams, C.Array) else stream_array(streams)
    _check(lib.ssd_decode_step_split_rope(cache.handle, layer_begin, layer_end, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out),
                                          int(bool(accumulate_scores)), int(bool(compress)), _ptr(cos), _ptr(sin), int(rope_layout),
                                          arr, len(arr), int(sync)), "ssd_decode_step_split_rope")


def ssd_decode_step_rope(cache: Cache, layer_begin: int, layer_end: int, q, k_new, v_new, out, cos, sin, rope_layout: int,
                         accumulate_scores: bool = True, compress: bool = True, stream=None) -> None:
    _check(lib.ssd_decode_step_rope(cache.handle, layer_begin, layer_end, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out),
                                    int(bool(accumulate_scores)), int(bool(compress)), _ptr(cos), _ptr(sin), int(rope_layout),
                                    _stream(stream)), "ssd_decode_step_rope")


def ssd_compress_kv(cache: Cache, layer_begin: int, layer_end: int, K_src=None, V_src=None, score_src=None,
                    n_src: int = 0, stream=None) -> None:
    _check(lib.ssd_compress_kv(cache.handle, layer_begin, layer_end, _ptr(K_src), _ptr(V_src), _ptr(score_src), int(n_src),
                               _stream(stream)), "ssd_compress_kv")


def ssd_prefill_scores(Q, K, n_units: int, n_src: int, d: int, dtype, score_out, softmax_scale: float = 0.0, stream=None) -> None:
    _check(lib.ssd_prefill_scores(_ptr(Q), _ptr(K), int(n_units), int(n_src), int(d), _dtype_code(dtype), float(softmax_scale),
                                  _ptr(score_out), _stream(stream)), "ssd_prefill_scores")


def ssd_cfg_mix(p, n_seqs: int, V: int, dtype, gamma: float, out, stream=None) -> None:
    _check(lib.ssd_cfg_mix(_ptr(p), int(n_seqs), int(V), _dtype_code(dtype), float(gamma), _ptr(out), _stream(stream)), "ssd_cfg_mix")


def ssd_classify_heads(far, tot, L: int, P: int, H: int, T: int, tau: float, s_out, type_out, stream=None) -> None:
    _check(lib.ssd_classify_heads(_ptr(far), _ptr(tot), L, P, H, T, float(tau), _ptr(s_out), _ptr(type_out),
                                  _stream(stream)), "ssd_classify_heads")


def ssd_dense_workspace_bytes(B: int, H: int, d: int, n: int) -> int:
    return lib.ssd_dense_workspace_bytes(B, H, d, n)


def ssd_dense_decode_attn(q, K, V, out, B: int, H: int, d: int, dtype, n_cap: int, n: int, softmax_scale: float = 0.0,
                          far=None, tot=None, mass_stride: int = 1, vis_start: int = 0, w: int = 32, workspace=None,
                          stream=None, splits: Optional[int] = None) -> None:
    """splits=None: ssd_dense_decode_attn; an integer: the test hook ssd_dense_decode_attn_splits with that many row splits."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    if splits is None:
        _check(lib.ssd_dense_decode_attn(_ptr(q), _ptr(K), _ptr(V), _ptr(out), B, H, d, _dtype_code(dtype), n_cap, n,
                                         float(softmax_scale), _ptr(far), _ptr(tot), mass_stride, vis_start, w,
                                         _ptr(workspace), ws_bytes, _stream(stream)), "ssd_dense_decode_attn")
    else:
        _check(lib.ssd_dense_decode_attn_splits(_ptr(q), _ptr(K), _ptr(V), _ptr(out), B, H, d, _dtype_code(dtype), n_cap, n,
                                                float(softmax_scale), _ptr(far), _ptr(tot), mass_stride, vis_start, w,
                                                int(splits), _ptr(workspace), ws_bytes, _stream(stream)),
               "ssd_dense_decode_attn_splits")


SSD_DENSE_STATIC_SCRATCH_BYTES = 8 << 20


def ssd_dense_decode_attn_static(q, K, V, out, B: int, H: int, d: int, dtype, n_cap: int, n: int, softmax_scale: float = 0.0,
                                 far=None, tot=None, mass_stride: int = 1, vis_start: int = 0, w: int = 32, stream=None) -> None:
    _check(lib.ssd_dense_decode_attn_static(_ptr(q), _ptr(K), _ptr(V), _ptr(out), B, H, d, _dtype_code(dtype), n_cap, n,
                                            float(softmax_scale), _ptr(far), _ptr(tot), mass_stride, vis_start, w,
                                            _stream(stream)), "ssd_dense_decode_attn_static")
