"""ctypes face of the CPU oracle (oracle/ssd_oracle.c).

TEST INFRASTRUCTURE: only tests/, __graft_entry__.smoke() and bench.py's
cpu_baseline leg may import this package.  Nothing here touches the GPU
library, and the GPU library never touches this.

All arrays are numpy, C-contiguous; float inputs are float32 (a bf16 workload
is widened first, which is exact), accumulation inside the C code is double.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ssd_oracle.c")
_LIB = os.path.join(_HERE, "libssd_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no threading, no fast-math)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-Wall", "-Wextra", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


_lib = C.CDLL(build())

_f32p = np.ctypeslib.ndpointer(dtype=np.float32, flags="C_CONTIGUOUS")
_f64p = np.ctypeslib.ndpointer(dtype=np.float64, flags="C_CONTIGUOUS")
_i32p = np.ctypeslib.ndpointer(dtype=np.int32, flags="C_CONTIGUOUS")
_u8p = np.ctypeslib.ndpointer(dtype=np.uint8, flags="C_CONTIGUOUS")
_vp = C.c_void_p


def _opt(a):
    return None if a is None else a.ctypes.data_as(_vp)


_lib.ssd_oracle_attend.argtypes = [_f32p, _f32p, _f32p, C.c_int, _i32p, C.c_int, C.c_double, _f32p, _vp, _vp]
_lib.ssd_oracle_attend.restype = C.c_int
_lib.ssd_oracle_dense_attend.argtypes = [_f32p, _f32p, _f32p, C.c_int, C.c_int, C.c_double, _f32p, _vp, _vp]
_lib.ssd_oracle_dense_attend.restype = C.c_int
_lib.ssd_oracle_far_tot.argtypes = [_f64p, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double)]
_lib.ssd_oracle_far_tot.restype = None
_lib.ssd_oracle_profile_unit.argtypes = [_f32p, _f32p, _f32p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_double, _f32p, _f32p]
_lib.ssd_oracle_profile_unit.restype = None
_lib.ssd_oracle_classify.argtypes = [_f32p, _f32p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_double, _f64p, _u8p]
_lib.ssd_oracle_classify.restype = None
_lib.ssd_oracle_prefill_scores.argtypes = [_f32p, _f32p, C.c_int, C.c_int, C.c_double, _f32p]
_lib.ssd_oracle_prefill_scores.restype = None
_lib.ssd_oracle_cfg_mix.argtypes = [_f32p, C.c_int, C.c_int, C.c_double, _f32p]
_lib.ssd_oracle_cfg_mix.restype = None
_lib.ssd_oracle_rope.argtypes = [_f32p, C.c_int, _f32p, _f32p, C.c_int, _f32p]
_lib.ssd_oracle_rope.restype = None
_lib.ssd_oracle_top_m.argtypes = [_f32p, _i32p, C.c_int, C.c_int, _i32p, C.POINTER(C.c_double)]
_lib.ssd_oracle_top_m.restype = C.c_int
_lib.ssd_oracle_unit_new.argtypes = [C.c_int] * 6
_lib.ssd_oracle_unit_new.restype = _vp
_lib.ssd_oracle_unit_free.argtypes = [_vp]
_lib.ssd_oracle_unit_free.restype = None
_lib.ssd_oracle_unit_set_buffered.argtypes = [_vp, C.c_int]
_lib.ssd_oracle_unit_set_buffered.restype = None
_lib.ssd_oracle_unit_append.argtypes = [_vp]
_lib.ssd_oracle_unit_append.restype = C.c_int
_lib.ssd_oracle_unit_n.argtypes = [_vp]
_lib.ssd_oracle_unit_n.restype = C.c_int
_lib.ssd_oracle_unit_retained.argtypes = [_vp, _i32p]
_lib.ssd_oracle_unit_retained.restype = C.c_int
_lib.ssd_oracle_unit_max_retained.argtypes = [_vp]
_lib.ssd_oracle_unit_max_retained.restype = C.c_int
_lib.ssd_oracle_unit_attend.argtypes = [_vp, _f32p, _f32p, _f32p, C.c_int, C.c_double, C.c_int, _f32p, _vp]
_lib.ssd_oracle_unit_attend.restype = C.c_int
_lib.ssd_oracle_unit_compress.argtypes = [_vp, C.POINTER(C.c_double)]
_lib.ssd_oracle_unit_compress.restype = C.c_int
_lib.ssd_oracle_unit_load_dense.argtypes = [_vp, C.c_int, _vp, C.POINTER(C.c_double)]
_lib.ssd_oracle_unit_load_dense.restype = C.c_int
_lib.ssd_oracle_unit_state.argtypes = [_vp, _i32p, _f32p, C.POINTER(C.c_int32), _i32p, _f32p, C.POINTER(C.c_int32)]
_lib.ssd_oracle_unit_state.restype = None
_lib.ssd_oracle_unit_run.argtypes = [_vp, C.c_int, C.c_int, C.c_int, _f32p, _f32p, _f32p, C.c_double, _u8p,
                                     C.c_int, _f32p, _vp, _vp]
_lib.ssd_oracle_unit_run.restype = C.c_int


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def attend(q, K, V, rows, scale):
    """O1 over the listed rows.  Returns (o float32[d], p float32[n_rows], p float64[n_rows])."""
    q, K, V = _f32(q), _f32(K), _f32(V)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    d = q.shape[-1]
    o = np.zeros(d, np.float32)
    p32 = np.zeros(max(len(rows), 1), np.float32)
    p64 = np.zeros(max(len(rows), 1), np.float64)
    _lib.ssd_oracle_attend(q, K, V, d, rows, len(rows), float(scale), o, _opt(p32), _opt(p64))
    return o, p32[: len(rows)], p64[: len(rows)]


def dense_attend(q, K, V, n, scale):
    """O1 over rows 0..n-1.  Returns (o, p32, p64)."""
    q, K, V = _f32(q), _f32(K), _f32(V)
    d = q.shape[-1]
    o = np.zeros(d, np.float32)
    p32 = np.zeros(max(n, 1), np.float32)
    p64 = np.zeros(max(n, 1), np.float64)
    _lib.ssd_oracle_dense_attend(q, K, V, d, int(n), float(scale), o, _opt(p32), _opt(p64))
    return o, p32[:n], p64[:n]


def far_tot(p64, n0, t, w):
    """One (far, tot) term of the sparsity metric from a distribution over n0+t rows."""
    p64 = np.ascontiguousarray(p64, dtype=np.float64)
    far, tot = C.c_double(), C.c_double()
    _lib.ssd_oracle_far_tot(p64, int(n0), int(t), int(w), C.byref(far), C.byref(tot))
    return far.value, tot.value


def profile_unit(q, K, V, n0, T, w, scale):
    """far[T], tot[T] (float32) of one (sequence, head) whose q, K, V are [n0+T, d]."""
    q, K, V = _f32(q), _f32(K), _f32(V)
    far = np.zeros(T, np.float32)
    tot = np.zeros(T, np.float32)
    _lib.ssd_oracle_profile_unit(q, K, V, q.shape[-1], int(n0), int(T), int(w), float(scale), far, tot)
    return far, tot


def classify(far, tot, tau):
    """far, tot [L,P,H,T] -> (s float64 [L,H], head_type uint8 [L,H]; 1 = semantic)."""
    far, tot = _f32(far), _f32(tot)
    L, P, H, T = far.shape
    s = np.zeros((L, H), np.float64)
    ty = np.zeros((L, H), np.uint8)
    _lib.ssd_oracle_classify(far, tot, L, P, H, T, float(tau), s, ty)
    return s, ty


def prefill_scores(q, K, scale):
    """Accumulated causal attention scores of a prompt: q, K [n, d] -> float32 [n]."""
    q, K = _f32(q), _f32(K)
    n, d = q.shape
    out = np.zeros(max(n, 1), np.float32)
    _lib.ssd_oracle_prefill_scores(q, K, d, n, float(scale), out)
    return out[:n]


def cfg_mix(p, gamma):
    """O6.  p [2 * prompts, V] (rows 2i conditional, 2i+1 unconditional) -> float32 [prompts, V], Eq. (1)."""
    p = _f32(p)
    B, V = p.shape
    assert B % 2 == 0
    out = np.zeros((max(B // 2, 1), max(V, 1)), np.float32)
    _lib.ssd_oracle_cfg_mix(p, B // 2, V, float(gamma), out)
    return out[: B // 2, :V]


ROPE_HALF, ROPE_INTERLEAVED = 1, 2


def rope(x, cos, sin, layout):
    """O7.  Rotary position embedding of rows x [..., d] at one position (cos, sin: [d/2]) -> float32 [..., d].
    layout ROPE_HALF pairs element i with i + d/2, ROPE_INTERLEAVED pairs 2i with 2i+1.  The definition, in double."""
    x = _f32(x)
    d = x.shape[-1]
    cos, sin = _f32(cos), _f32(sin)
    assert d % 2 == 0 and cos.shape == (d // 2,) and sin.shape == (d // 2,) and layout in (ROPE_HALF, ROPE_INTERLEAVED)
    rows = np.ascontiguousarray(x.reshape(-1, d))
    out = np.zeros_like(rows)
    for i in range(rows.shape[0]):
        _lib.ssd_oracle_rope(rows[i], d, cos, sin, int(layout), out[i])
    return out.reshape(x.shape)


def top_m(score, pos, M):
    """O3.  Returns (kept candidate indices ordered by position, relative gap at the cut or -1)."""
    score = _f32(score)
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    keep = np.zeros(max(len(score), 1), np.int32)
    gap = C.c_double()
    k = _lib.ssd_oracle_top_m(score, pos, len(score), int(M), keep, C.byref(gap))
    return keep[:k].copy(), gap.value


class Unit:
    """O4: the cache policy of one (layer, sequence, head) over dense K, V held by the caller."""

    def __init__(self, is_semantic, W, S, M, R, C_, buffered_spatial=False):
        """buffered_spatial: a spatial head follows Algorithm 2 (window frozen at the last compression plus
        the row buffer) instead of Algorithm 1 (exact sliding window)."""
        self.is_semantic = bool(is_semantic)
        self.W, self.S, self.M, self.R, self.C = int(W), int(S), int(M), int(R), int(C_)
        self._h = _lib.ssd_oracle_unit_new(int(self.is_semantic), self.W, self.S, self.M, self.R, self.C)
        if buffered_spatial:
            _lib.ssd_oracle_unit_set_buffered(self._h, 1)

    def __del__(self):
        if getattr(self, "_h", None):
            _lib.ssd_oracle_unit_free(self._h)
            self._h = None

    @property
    def n(self):
        return _lib.ssd_oracle_unit_n(self._h)

    def append(self):
        """Returns 0, or -1 on row-buffer overflow."""
        return _lib.ssd_oracle_unit_append(self._h)

    def retained(self):
        buf = np.zeros(_lib.ssd_oracle_unit_max_retained(self._h) + 1, np.int32)
        k = _lib.ssd_oracle_unit_retained(self._h, buf)
        return buf[:k].copy()

    def attend(self, q, K, V, scale, accumulate=True):
        q, K, V = _f32(q), _f32(K), _f32(V)
        d = q.shape[-1]
        o = np.zeros(d, np.float32)
        p = np.zeros(_lib.ssd_oracle_unit_max_retained(self._h) + 1, np.float32)
        k = _lib.ssd_oracle_unit_attend(self._h, q, K, V, d, float(scale), int(bool(accumulate)), o, _opt(p))
        return o, p[:k].copy()

    def compress(self):
        """Returns (new heavy count, relative gap at the cut or -1)."""
        gap = C.c_double()
        k = _lib.ssd_oracle_unit_compress(self._h, C.byref(gap))
        return k, gap.value

    def load_dense(self, n_src, score_src=None):
        gap = C.c_double()
        s = None if score_src is None else _f32(score_src)
        k = _lib.ssd_oracle_unit_load_dense(self._h, int(n_src), _opt(s), C.byref(gap))
        return k, gap.value

    def state(self):
        """(heavy_pos, heavy_score, staged_pos, staged_score); empty arrays for a spatial head."""
        cap = _lib.ssd_oracle_unit_max_retained(self._h) + 1
        hp, hs = np.zeros(cap, np.int32), np.zeros(cap, np.float32)
        sp, ss = np.zeros(cap, np.int32), np.zeros(cap, np.float32)
        nh, ns = C.c_int32(0), C.c_int32(0)
        if self.is_semantic:
            _lib.ssd_oracle_unit_state(self._h, hp, hs, C.byref(nh), sp, ss, C.byref(ns))
        return hp[: nh.value].copy(), hs[: nh.value].copy(), sp[: ns.value].copy(), ss[: ns.value].copy()

    def run(self, q, K, V, scale, compress_after, p_begin=None, p_end=None, accumulate=True, log=False):
        """Decode positions [p_begin, p_end).  Returns (o [steps,d], heavy_log or None, gap_log or None)."""
        q, K, V = _f32(q), _f32(K), _f32(V)
        d = q.shape[-1]
        p_begin = self.n if p_begin is None else int(p_begin)
        p_end = q.shape[0] if p_end is None else int(p_end)
        ca = np.ascontiguousarray(compress_after, dtype=np.uint8)
        assert len(ca) >= p_end
        steps = p_end - p_begin
        o = np.zeros((max(steps, 1), d), np.float32)
        hl = np.full((max(steps, 1), max(self.M, 1)), -1, np.int32) if log else None
        gl = np.full(max(steps, 1), -1.0, np.float64) if log else None
        rc = _lib.ssd_oracle_unit_run(self._h, d, p_begin, p_end, q, K, V, float(scale), ca,
                                      int(bool(accumulate)), o, _opt(hl), _opt(gl))
        if rc != 0:
            raise OverflowError("row buffer overflow at position %d" % (-rc - 1))
        return o[:steps], (hl[:steps] if log else None), (gl[:steps] if log else None)
