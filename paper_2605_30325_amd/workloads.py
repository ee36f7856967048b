"""Seeded synthetic workloads for the tile-sparse attention path.

This module only *draws inputs*: problem shapes, per-head tile shapes, Q/K/V
values, estimator weights and the per-head keep budget.  It holds none of the
method's arithmetic (no tiling, pooling, scoring, selection or attention) so
that the CPU oracle and the HIP library can both be fed from it without sharing
any computation.

The value recipe stands in for real video-DiT activations, which are smooth in
(t, h, w) plus token noise: each channel is a sum of four low-frequency
sinusoids over the latent grid (unit variance over the grid) plus N(0,1).
Every (tensor, head) pair has its own seed stream, so any subset of heads can
be regenerated bit-identically on the same device type.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

TILE_TOKENS = 64
# (p_t, p_h, p_w): extents of one tile along time, height and width.
TILE_SHAPES = ((4, 4, 4), (1, 8, 8), (16, 2, 2))

_TENSOR_ID = {"q": 0, "k": 1, "v": 2}


@dataclass(frozen=True)
class Workload:
    name: str
    index: int                      # position in the configuration list; also the seed
    heads: int
    head_dim: int
    dtype: str                      # "f32" or "bf16"
    grid: Tuple[int, int, int]      # latent (T, H, W)
    head_aware: bool                # True: per-head shape drawn from TILE_SHAPES
    keep: Tuple[int, int]           # kept fraction of key tiles (num, den)
    recipe: str                     # "tiny" | "unit" | "amp"
    fixed_k: Optional[int] = None   # explicit budget (overrides keep)
    batch: int = 1
    latent_dim: int = 64            # estimator latent size d'
    keep_sweep: Tuple[Tuple[int, int], ...] = ()

    @property
    def seed(self) -> int:
        return self.index

    @property
    def tokens(self) -> int:
        t, h, w = self.grid
        return t * h * w

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


WORKLOADS: Dict[str, Workload] = {
    w.name: w
    for w in (
        Workload("tiny", 0, 2, 64, "f32", (4, 8, 8), False, (1, 2), "tiny",
                 fixed_k=2, latent_dim=32),
        Workload("wan1p3b_480p", 1, 12, 128, "bf16", (21, 30, 52), False, (10, 100), "unit"),
        Workload("wan14b_480p", 2, 40, 128, "bf16", (21, 30, 52), True, (5, 100), "unit"),
        Workload("wan14b_720p", 3, 40, 128, "bf16", (21, 45, 80), True, (5, 100), "amp",
                 keep_sweep=((20, 100), (10, 100), (5, 100))),
        Workload("waver12b_720p_241f", 4, 24, 128, "bf16", (61, 45, 80), True, (5, 100), "unit"),
    )
}
WORKLOAD_ORDER: List[str] = [
    "tiny", "wan1p3b_480p", "wan14b_480p", "wan14b_720p", "waver12b_720p_241f"]


def custom_workload(name: str, heads: int, head_dim: int, dtype: str,
                    grid: Sequence[int], head_aware: bool, keep: Tuple[int, int],
                    seed: int, recipe: str = "unit", latent_dim: int = 64,
                    fixed_k: Optional[int] = None, batch: int = 1) -> Workload:
    """A test-sized workload drawn with the same recipe as the named ones."""
    return Workload(name, seed, heads, head_dim, dtype, tuple(grid), head_aware, keep,
                    recipe, fixed_k=fixed_k, latent_dim=latent_dim, batch=batch)


def tile_shapes(wl: Workload) -> np.ndarray:
    """int32 [heads, 3] of (p_t, p_h, p_w).  Head-aware workloads draw a shape id
    per head as the first draw of the workload's generator."""
    if not wl.head_aware:
        return np.tile(np.asarray(TILE_SHAPES[0], np.int32), (wl.heads, 1))
    rng = np.random.default_rng(wl.seed)
    ids = rng.integers(0, len(TILE_SHAPES), size=wl.heads)
    return np.asarray([TILE_SHAPES[i] for i in ids], np.int32)


def tiles_per_head(wl: Workload, shapes: Optional[np.ndarray] = None) -> np.ndarray:
    """Tile count of each head's ceil-padded tile grid (a size, used to draw k)."""
    shapes = tile_shapes(wl) if shapes is None else shapes
    t, h, w = wl.grid
    return np.asarray([(-(-t // s[0])) * (-(-h // s[1])) * (-(-w // s[2])) for s in shapes],
                      np.int64)


def keep_budget(wl: Workload, keep: Optional[Tuple[int, int]] = None,
                shapes: Optional[np.ndarray] = None) -> np.ndarray:
    """int32 [heads]: kept key tiles per query tile, max(1, ceil(num*N_T/den))."""
    nt = tiles_per_head(wl, shapes)
    if keep is None and wl.fixed_k is not None:
        return np.minimum(nt, wl.fixed_k).astype(np.int32)
    num, den = wl.keep if keep is None else keep
    return np.maximum(1, -(-(num * nt) // den)).astype(np.int32)


def _field_params(seed: int, tensor: str, head: int, channels: int):
    rng = np.random.default_rng([seed, _TENSOR_ID[tensor], head])
    freq = rng.integers(0, 3, size=(channels, 4, 3))
    zero = freq.sum(axis=2) == 0
    # a component with all-zero frequency would be a constant: move it to f_w = 1
    freq[..., 2] = np.where(zero, 1, freq[..., 2])
    phase = rng.uniform(0.0, 2.0 * math.pi, size=(channels, 4))
    amp = rng.uniform(0.5, 1.0, size=(channels, 4))
    return freq, phase, amp


def smooth_field(wl: Workload, tensor: str, head: int, device="cpu",
                 batch: int = 0) -> torch.Tensor:
    """fp32 [N, d]: four low-frequency sinusoids per channel, unit variance over the grid."""
    T, H, W = wl.grid
    d = wl.head_dim
    freq, phase, amp = _field_params(wl.seed + 7919 * batch, tensor, head, d)
    dev = torch.device(device)
    two_pi = 2.0 * math.pi
    f = torch.as_tensor(freq, dtype=torch.float32, device=dev)      # [d,4,3]
    ph = torch.as_tensor(phase, dtype=torch.float32, device=dev)    # [d,4]
    am = torch.as_tensor(amp, dtype=torch.float32, device=dev)
    at = torch.arange(T, device=dev, dtype=torch.float32) / T
    ah = torch.arange(H, device=dev, dtype=torch.float32) / H
    aw = torch.arange(W, device=dev, dtype=torch.float32) / W
    out = torch.zeros((T, H, W, d), dtype=torch.float32, device=dev)
    for m in range(4):
        ang = (two_pi * (at[:, None, None, None] * f[None, None, None, :, m, 0]
                         + ah[None, :, None, None] * f[None, None, None, :, m, 1]
                         + aw[None, None, :, None] * f[None, None, None, :, m, 2])
               + ph[None, None, None, :, m])
        out += am[None, None, None, :, m] * torch.sin(ang)
    out = out.reshape(T * H * W, d)
    # Sinusoids that do not vary over this grid (e.g. frequencies along t only and T = 1) are a
    # constant offset, not a field: the offset is removed (full periods sum to zero, so on
    # ordinary grids there is none and nothing changes), and a channel left with no variation at
    # all is set to zero instead of being blown up by a near-zero deviation.  A large offset
    # would also push bf16 outputs past the magnitude at which the tests' absolute error bars
    # make sense.
    mean = out.mean(dim=0, keepdim=True)
    out = out - torch.where(mean.abs() > 1e-3, mean, torch.zeros_like(mean))
    std = out.std(dim=0, keepdim=True, unbiased=False)
    flat = std < 1e-6
    out = torch.where(flat, torch.zeros_like(out), out / torch.where(flat, torch.ones_like(std), std))
    return out


def head_amplitudes(wl: Workload) -> np.ndarray:
    """Per-head smooth-field amplitude of the "amp" recipe, U[0.2, 1.0]."""
    rng = np.random.default_rng([wl.seed, 99])
    return rng.uniform(0.2, 1.0, size=wl.heads)


def make_head(wl: Workload, tensor: str, head: int, device="cpu", batch: int = 0) -> torch.Tensor:
    """[N, d] in the workload's dtype for one (tensor, head)."""
    dev = torch.device(device)
    fld = smooth_field(wl, tensor, head, dev, batch)
    gen = torch.Generator(device=dev)
    gen.manual_seed(((wl.seed + 7919 * batch) * 3 + _TENSOR_ID[tensor]) * 100003 + head)
    noise = torch.randn(fld.shape, generator=gen, device=dev, dtype=torch.float32)
    if wl.recipe == "tiny":
        x = 0.5 * fld + noise
    elif wl.recipe == "amp" and tensor in ("q", "k"):
        x = float(head_amplitudes(wl)[head]) * fld + noise
    else:
        x = (fld + noise) * (1.0 / math.sqrt(2.0))
    return x.to(wl.torch_dtype)


def make_qkv(wl: Workload, device="cpu", heads: Optional[Sequence[int]] = None):
    """(q, k, v), each [batch, len(heads), N, d] contiguous in the workload's dtype."""
    hs = list(range(wl.heads)) if heads is None else list(heads)
    out = []
    for name in ("q", "k", "v"):
        x = torch.empty((wl.batch, len(hs), wl.tokens, wl.head_dim),
                        dtype=wl.torch_dtype, device=device)
        for b in range(wl.batch):
            for j, h in enumerate(hs):
                x[b, j] = make_head(wl, name, h, device, b)
        out.append(x)
    return tuple(out)


@dataclass
class EstimatorWeights:
    """Per-head two-layer perceptron 3d -> hidden -> d' (fp32, row-major [in][out])."""
    in_dim: int
    hidden: int
    out_dim: int
    w1: np.ndarray   # [heads, in_dim, hidden]
    b1: np.ndarray   # [heads, hidden]
    w2: np.ndarray   # [heads, hidden, out_dim]
    b2: np.ndarray   # [heads, out_dim]
    relu: bool = True


def make_estimator(wl: Workload, which: str) -> EstimatorWeights:
    """Xavier-uniform weights and U(-0.05, 0.05) biases for phi_q ("q") or phi_k ("k")."""
    rng = np.random.default_rng([wl.seed + 1000, 0 if which == "q" else 1])
    d, dp = wl.head_dim, wl.latent_dim
    i, hdim = 3 * d, d

    def xavier(fan_in, fan_out):
        a = math.sqrt(6.0 / (fan_in + fan_out))
        return rng.uniform(-a, a, size=(wl.heads, fan_in, fan_out)).astype(np.float32)

    w1 = xavier(i, hdim)
    b1 = rng.uniform(-0.05, 0.05, size=(wl.heads, hdim)).astype(np.float32)
    w2 = xavier(hdim, dp)
    b2 = rng.uniform(-0.05, 0.05, size=(wl.heads, dp)).astype(np.float32)
    return EstimatorWeights(i, hdim, dp, w1, b1, w2, b2, True)
