"""Independent float64 / pure-Python statements of each stage, for tiny inputs only.

These are the pins of the C oracle: written from the paper's definitions with token-level
loops and NumPy library routines, sharing nothing with oracle/ or with the GPU package.
"""
import itertools

import numpy as np


def tile_grid(grid, shape):
    return tuple(-(-g // p) for g, p in zip(grid, shape))


def slots(grid, shape):
    """dict (tile index, slot) -> token index, by explicit enumeration of tiles then slots."""
    T, H, W = grid
    pt, ph, pw = shape
    nt, nh, nw = tile_grid(grid, shape)
    table = {}
    for i, (a, b, c) in enumerate(itertools.product(range(nt), range(nh), range(nw))):
        for l, (x, y, z) in enumerate(itertools.product(range(pt), range(ph), range(pw))):
            t, h, w = a * pt + x, b * ph + y, c * pw + z
            if t < T and h < H and w < W:
                table[(i, l)] = (t * H + h) * W + w
    return table


def tile_members(grid, shape):
    """list over tiles of the token indices in slot order (real tokens only)."""
    nt = int(np.prod(tile_grid(grid, shape)))
    B = int(np.prod(shape))
    tab = slots(grid, shape)
    return [[tab[(i, l)] for l in range(B) if (i, l) in tab] for i in range(nt)]


def trippool64(x, grid, shape):
    x = np.asarray(x, np.float64)
    out = []
    for mem in tile_members(grid, shape):
        blk = x[mem]
        out.append(np.concatenate([blk.mean(0), blk.max(0), blk.min(0)]))
    return np.asarray(out)


def mlp64(z, w1, b1, w2=None, b2=None, relu=True):
    z = np.asarray(z, np.float64)
    h = z @ np.asarray(w1, np.float64) + np.asarray(b1, np.float64)
    if w2 is None:
        return h
    if relu:
        h = np.maximum(h, 0.0)
    return h @ np.asarray(w2, np.float64) + np.asarray(b2, np.float64)


def topk_rows(s, k):
    """Per row: indices of the k largest, ties to the lower index, ascending."""
    s = np.asarray(s)
    out = []
    for row in s:
        row = np.where(np.isnan(row), -np.inf, row) + 0.0
        order = np.lexsort((np.arange(len(row)), -row))   # primary: -score, secondary: index
        out.append(np.sort(order[:k]))
    return np.asarray(out, np.int32)


def concat_tile_attention(q, k, v, grid, shape, sel, scale):
    """Eq. 2 form: per query tile, softmax over the concatenated kept key tiles. float64.
    Returns O in token order."""
    q, k, v = (np.asarray(a, np.float64) for a in (q, k, v))
    mem = tile_members(grid, shape)
    out = np.zeros_like(q)
    for i, qm in enumerate(mem):
        keys = [n for j in sel[i] for n in mem[j]]
        logits = q[qm] @ k[keys].T * scale
        logits -= logits.max(axis=1, keepdims=True)
        w = np.exp(logits)
        w /= w.sum(axis=1, keepdims=True)
        out[qm] = w @ v[keys]
    return out


def dense_attention64(q, k, v, scale):
    q, k, v = (np.asarray(a, np.float64) for a in (q, k, v))
    logits = q @ k.T * scale
    logits -= logits.max(axis=1, keepdims=True)
    w = np.exp(logits)
    w /= w.sum(axis=1, keepdims=True)
    return w @ v, w


def tile_heatmap64(q, k, grid, shape, scale):
    """Sec. 4.1 target: full softmax in float64, then the maximum over every (query tile, key tile)
    block of token pairs, by explicit enumeration of the tiles' members."""
    q = np.asarray(q, np.float64)
    k = np.asarray(k, np.float64)
    logits = (q @ k.T) * scale
    a = np.exp(logits - logits.max(axis=1, keepdims=True))
    a /= a.sum(axis=1, keepdims=True)
    mem = tile_members(grid, shape)
    heat = np.zeros((len(mem), len(mem)))
    for i, rows in enumerate(mem):
        for j, cols in enumerate(mem):
            heat[i, j] = a[np.ix_(rows, cols)].max()
    return heat


def recall64(sel_sp, sel_fu):
    """Sec. 3.2 tile recall with Python sets."""
    k = len(sel_sp[0])
    return float(np.mean([len(set(map(int, a)) & set(map(int, b))) / k for a, b in zip(sel_sp, sel_fu)]))
