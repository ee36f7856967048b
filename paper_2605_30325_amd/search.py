"""Head-aware tiling search (Sec. 4.2, Eq. 8; Alg. 1) as a sequence of library calls.

For every candidate tile shape pi the calibration tensors are tiled, the reference top-k mask is
taken from the full-attention target scores (veda_tile_heatmap + veda_tile_select), the tile-sparse
attention is run under that mask, and the squared distance to the full-attention output is added to
the candidate's error; each head gets the shape with the smallest error.  Everything numeric runs
in the library's kernels; this module only sequences the calls and takes the final argmin of a
[heads, candidates] table on the host.  The calibration set is the batch axis of q, k, v.
"""
import math
from typing import Optional, Sequence, Tuple

import numpy as np
import torch

from . import veda


def keep_budget(n_tiles: Sequence[int], keep: Tuple[int, int]) -> np.ndarray:
    """k = max(1, ceil(keep[0] * N_T / keep[1])) per head (the top-k budget of the search)."""
    return np.asarray([max(1, -(-keep[0] * int(n) // keep[1])) for n in n_tiles], np.int32)


def _dense_output(plan: veda.Plan, qt, kt, vt, vm, softmax_scale: float) -> torch.Tensor:
    """Full attention through the sparse kernel with every key tile kept."""
    dev = qt.device
    rows = []
    for n in plan.tiles:
        rows.append(torch.arange(n, dtype=torch.int32, device=dev).repeat(n))
    cols = torch.cat(rows).repeat(plan.batch)
    counts = torch.tensor([n for _ in range(plan.batch) for n in plan.tiles for _ in range(n)], dtype=torch.int64)
    row_ptr = torch.zeros(plan.batch * plan.total_tiles + 1, dtype=torch.int64)
    row_ptr[1:] = torch.cumsum(counts, 0)
    out, _ = veda.veda_sparse_attn_fwd(plan, qt, kt, vt, vm, row_ptr.to(torch.int32).to(dev), cols, softmax_scale)
    return out


def tiling_search(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, grid: Sequence[int],
                  candidates: Sequence[Sequence[int]], keep: Tuple[int, int],
                  softmax_scale: Optional[float] = None, tile_tokens: int = 64):
    """q, k, v: [samples, heads, N, d] device tensors (bf16 or fp32), N = T*H*W of `grid`;
    candidates: tile shapes whose product is tile_tokens (64, or 128 for bf16).
    Returns (best [heads, 3] int32 tile shapes, errors float64 [heads, len(candidates)])."""
    samples, heads, n_tok, d = q.shape
    scale = 1.0 / math.sqrt(d) if softmax_scale is None else float(softmax_scale)
    errors = torch.zeros((heads, len(candidates)), dtype=torch.float64, device=q.device)
    o_full = None
    for c, shape in enumerate(candidates):
        shapes = np.tile(np.asarray(shape, np.int32), (heads, 1))
        plan = veda.Plan(samples, heads, d, grid, shapes, q.dtype, tile_tokens=tile_tokens)
        qt, vm, _ = veda.veda_tile_layout(plan, q, veda.VEDA_TOKEN_MAJOR)
        kt, _, _ = veda.veda_tile_layout(plan, k, veda.VEDA_TOKEN_MAJOR, want_mask=False)
        vt, _, _ = veda.veda_tile_layout(plan, v, veda.VEDA_CHANNEL_MAJOR, want_mask=False)
        if o_full is None:   # the full-attention output does not depend on the tiling
            o_full = _dense_output(plan, qt, kt, vt, vm, scale)
        heat = veda.veda_tile_heatmap(plan, qt, kt, vm, scale)
        kph = keep_budget(plan.tiles, keep)
        row_ptr, col_idx = veda.veda_tile_select(plan, heat, kph)
        o_sp, _ = veda.veda_sparse_attn_fwd(plan, qt, kt, vt, vm, row_ptr, col_idx, scale)
        err = veda.veda_output_sqerr(plan, o_full, o_sp)          # [samples, heads]
        errors[:, c] = err.sum(dim=0)
        plan.close()
    table = errors.cpu().numpy()
    best = np.asarray([candidates[int(j)] for j in table.argmin(axis=1)], np.int32)
    return best, table
