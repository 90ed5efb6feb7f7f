"""Seeded synthetic Janus-Pro-shaped decode workloads.

This module only makes inputs: shapes, head maps, sink positions, q/k/v
tensors and the compression schedule.  It holds none of the method's
arithmetic (no attention, no selection, no cache logic) and is the one thing
the CPU oracle's tests and the GPU path's tests both import, so that both
sides see the same bits: inputs are generated once, on one device, rounded to
the workload dtype there, and handed to the other side by copy.

Shapes follow the paper's Table 5 (Janus-Pro-1B: 24 layers x 16 heads,
Janus-Pro-7B: 30 layers x 32 heads, head_dim 128, 576 image tokens = 24x24
grid), the CFG pairing of Sec. 3.1 (two sequences per prompt) and the two
attention patterns of Sec. 3.3: spatial-locality heads whose queries look at
their raster predecessors, and semantic-sink heads whose queries look at a few
margin-column tokens (Sec. 3.2) and the first prompt token.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

SPATIAL = 0
SEMANTIC = 1


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    L: int                    # layers
    prompts: int              # B = 2 * prompts (cond/uncond adjacent)
    H: int                    # heads
    d: int                    # head_dim
    dtype: str                # "f32" | "bf16"
    n0: int                   # prompt tokens
    grid_h: int
    grid_w: int
    W: int                    # spatial window (counts the current token)
    M: int                    # semantic heavy-hitter budget
    S: int = 1                # initial sink rows of a spatial head
    R: int = 1                # protected recent tokens of a semantic head
    C: int = 2                # row-buffer (staging) capacity, C > R
    cadence: int = 1          # compress after every `cadence` tokens
    alg2: bool = False        # spatial heads follow Algorithm 2 (window as of the last compression + row buffer)
    spatial_frac: float = 0.5
    sink_rows: Optional[Sequence[int]] = None   # grid rows whose column-0 token is a sink (None = all)
    beta: float = 2.5         # query gain of spatial heads
    sink_gain: float = 4.0    # weight of the shared direction e in a semantic head's queries
    plain: bool = False       # True: no planted structure, q = k = v = N(0,1) in every head
    seed: int = 20251018
    w_metric: int = 32        # recency window of the sparsity metric
    W_layers: Optional[Sequence[int]] = None    # window per layer (None = W everywhere)
    M_layers: Optional[Sequence[int]] = None    # budget per layer (None = M everywhere)
    head_budget: Optional[Sequence[Sequence[int]]] = None   # [L][H]: W_h of a spatial head, M_h of a semantic head
    softmax_scale: Optional[float] = None       # None = 1/sqrt(d)

    @property
    def B(self) -> int:
        return 2 * self.prompts

    @property
    def N(self) -> int:
        return self.grid_h * self.grid_w

    @property
    def n_total(self) -> int:
        return self.n0 + self.N

    @property
    def torch_dtype(self):
        return {"f32": torch.float32, "bf16": torch.bfloat16}[self.dtype]

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.d) if self.softmax_scale is None else float(self.softmax_scale)

    def W_of(self, layer: int, head: Optional[int] = None) -> int:
        if self.head_budget is not None and head is not None:
            return int(self.head_budget[layer][head])
        return self.W if self.W_layers is None else int(self.W_layers[layer])

    def M_of(self, layer: int, head: Optional[int] = None) -> int:
        if self.head_budget is not None and head is not None:
            return int(self.head_budget[layer][head])
        return self.M if self.M_layers is None else int(self.M_layers[layer])

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


def config(k: int) -> Workload:
    """The k-th (1-based) benchmark configuration."""
    if k == 1:   # tiny, every unit checkable on the CPU
        return Workload("cfg1-tiny", L=1, prompts=1, H=8, d=64, dtype="f32", n0=32, grid_h=8, grid_w=8,
                        W=16, M=8, S=1, R=1, C=2, cadence=1, sink_rows=(0, 2, 4), seed=20251018 + 1)
    if k == 2:   # Janus-Pro-1B-shaped
        return Workload("cfg2-1b", L=24, prompts=16, H=16, d=128, dtype="bf16", n0=64, grid_h=24, grid_w=24,
                        W=64, M=64, seed=20251018 + 2)
    if k == 3:   # Janus-Pro-7B-shaped (headline)
        return Workload("cfg3-7b", L=30, prompts=64, H=32, d=128, dtype="bf16", n0=64, grid_h=24, grid_w=24,
                        W=64, M=64, seed=20251018 + 3)
    if k == 4:   # high resolution, one 7B-shaped layer, compress every 256 tokens
        return Workload("cfg4-hires", L=1, prompts=32, H=32, d=128, dtype="bf16", n0=64, grid_h=48, grid_w=48,
                        W=128, M=128, C=257, cadence=256, seed=20251018 + 4)
    if k == 5:   # large batch, 7B-shaped (one point of the sweep; use .replace for the others)
        return Workload("cfg5-large", L=30, prompts=256, H=32, d=128, dtype="bf16", n0=64, grid_h=24, grid_w=24,
                        W=64, M=64, seed=20251018 + 5)
    raise ValueError("config index must be 1..5")


def head_map(wl: Workload) -> np.ndarray:
    """uint8 [L, H], 0 = spatial, 1 = semantic.  Exactly round(frac*H) spatial heads per layer:
    the lowest head indices in even layers, the highest in odd layers."""
    n_sp = int(round(wl.spatial_frac * wl.H))
    m = np.full((wl.L, wl.H), SEMANTIC, np.uint8)
    for l in range(wl.L):
        if l % 2 == 0:
            m[l, :n_sp] = SPATIAL
        else:
            m[l, wl.H - n_sp:] = SPATIAL
    return m


def sink_positions(wl: Workload) -> List[int]:
    """Absolute positions of the planted sinks: the first prompt token and column 0 of the chosen grid rows."""
    rows = range(wl.grid_h) if wl.sink_rows is None else wl.sink_rows
    return [0] + [wl.n0 + r * wl.grid_w for r in rows]


def compress_schedule(wl: Workload, cadence: Optional[int] = None) -> np.ndarray:
    """uint8 [n_total]: 1 where a compression follows the attention of that position."""
    c = wl.cadence if cadence is None else cadence
    p = np.arange(wl.n_total)
    return ((p + 1) % c == 0).astype(np.uint8)


def generate(wl: Workload, device="cpu", head_type: Optional[np.ndarray] = None,
             layers: Optional[Sequence[int]] = None) -> Dict[str, torch.Tensor]:
    """q, k, v as [n_total, L', B, H, d] tensors of the workload dtype on `device`
    (L' = len(layers), default all), token-major so that x[p] is one decode step's input.

    Every entry starts as N(0,1).  Spatial heads: q_p = beta*(0.8*u_p + 0.6*eps_p) with u_p the sum of
    the (up to) four predecessor keys divided by sqrt(their number).  Semantic heads: one unit direction e per
    (layer, head); sink positions carry k = 4*sqrt(d)*e; every query is eps + sink_gain*e.  One torch generator per
    layer, seeded from (seed, layer), so a layer can be regenerated alone on the same device type.
    """
    ht = head_map(wl) if head_type is None else np.asarray(head_type, np.uint8)
    layers = list(range(wl.L)) if layers is None else list(layers)
    n, B, H, d = wl.n_total, wl.B, wl.H, wl.d
    dev = torch.device(device)
    out = {x: torch.empty((n, len(layers), B, H, d), dtype=wl.torch_dtype, device=dev) for x in "qkv"}
    sinks = torch.tensor(sink_positions(wl), device=dev, dtype=torch.long)
    cnt = torch.clamp(torch.arange(n, device=dev), max=4).clamp(min=1).to(torch.float32).sqrt().view(n, 1, 1, 1)
    for li, l in enumerate(layers):
        g = torch.Generator(device=dev)
        g.manual_seed(wl.seed * 4096 + l)
        k = torch.randn((n, B, H, d), generator=g, device=dev)
        eps = torch.randn((n, B, H, d), generator=g, device=dev)
        v = torch.randn((n, B, H, d), generator=g, device=dev)
        e = torch.randn((H, d), generator=g, device=dev)
        e = e / e.norm(dim=-1, keepdim=True)
        sem = torch.from_numpy(ht[l].astype(np.bool_)).to(dev).view(1, 1, H, 1)
        # spatial queries: weight 0.8 on the common direction of the raster predecessors
        u = torch.zeros_like(k)
        for i in range(1, 5):
            u[i:] += k[:-i]
        u /= cnt
        q_sp = wl.beta * (0.8 * u + 0.6 * eps)
        del u
        # semantic keys: planted sinks; semantic queries lean on e
        k_se = k.clone()
        k_se[sinks] = (4.0 * math.sqrt(d)) * e.view(1, 1, H, d)
        q_se = eps + wl.sink_gain * e.view(1, 1, H, d)
        if wl.plain:
            q_se, q_sp, k_se = eps, eps, k
        out["q"][:, li] = torch.where(sem, q_se, q_sp).to(wl.torch_dtype)
        out["k"][:, li] = torch.where(sem, k_se, k).to(wl.torch_dtype)
        out["v"][:, li] = v.to(wl.torch_dtype)
        del k, eps, v, q_sp, q_se, k_se
    return out


def rope_tables(n: int, d: int, base: float = 10000.0):
    """cos, sin float32 [n, d/2] of the angles position * base^(-2i/d): the tables a caller of the rotary variant
    of the fused step holds (an input to both sides; computed in float64, stored as float32)."""
    inv = base ** (-np.arange(0, d, 2, dtype=np.float64) / d)
    ang = np.arange(n, dtype=np.float64)[:, None] * inv[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def unit_arrays(data: Dict[str, torch.Tensor], li: int, b: int, h: int):
    """(q, K, V) of one (layer index within data, sequence, head) as float32 numpy [n_total, d]."""
    return tuple(
        np.ascontiguousarray(data[x][:, li, b, h, :].to(torch.float32).cpu().numpy()) for x in "qkv"
    )


def dense_layout(x: torch.Tensor, n_cap: Optional[int] = None) -> torch.Tensor:
    """[n, L', B, H, d] -> [L', B, H, n_cap, d] (zero padded), the layout of a full cache."""
    n = x.shape[0]
    n_cap = n if n_cap is None else n_cap
    out = torch.zeros((x.shape[1], x.shape[2], x.shape[3], n_cap, x.shape[4]), dtype=x.dtype, device=x.device)
    out[:, :, :, :n] = x.permute(1, 2, 3, 0, 4)
    return out
