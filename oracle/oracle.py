"""ctypes front end of the CPU oracle (oracle/veda_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
benchmark's CPU-baseline leg.  It never imports the GPU package and the GPU
package never imports it.  All arrays are NumPy; one head per call.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from pathlib import Path
from typing import Optional, Sequence

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "veda_oracle.c"
_LIB = _HERE / "libveda_oracle.so"
_lib = None


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (contraction off, OpenMP on)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".tmp{os.getpid()}.so")
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-Wall", "-shared",
                               "-fPIC", "-o", str(tmp), str(_SRC), "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(str(_LIB))
        i32, i64, f32, f64, vp = C.c_int, C.c_int64, C.c_float, C.c_double, C.c_void_p
        L.vo_num_tiles.restype = i64
        L.vo_num_tiles.argtypes = [i32] * 6
        L.vo_token_tile_map.argtypes = [i32] * 6 + [vp]
        L.vo_tile_layout.argtypes = [vp, i64, i32, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp]
        L.vo_untile.argtypes = [vp, i64, i32, i32, i32, i32, i32, i32, i32, vp]
        L.vo_trippool.argtypes = [vp, i32, i32, i32, i32, i32, i32, i32, vp]
        L.vo_mlp.argtypes = [vp, i64, i32, i32, i32, i32, vp, vp, vp, vp, vp]
        L.vo_score.argtypes = [vp, vp, i64, i64, i32, f32, vp]
        L.vo_select.argtypes = [vp, i64, i64, i32, vp, vp]
        L.vo_masked_attention.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, i32,
                                          f64, vp, i64, vp, vp, vp]
        L.vo_dense_attention.argtypes = [vp, vp, vp, i32, i64, f64, vp, i64, vp]
        L.vo_tile_heatmap.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, i32, f64, vp, i64, vp]
        L.vo_recall.argtypes = [vp, vp, i64, i32, vp]
        L.vo_closed_form_latent.argtypes = [vp, i64, i32, f32, vp]
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _ok(rc: int, what: str):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def num_tiles(grid: Sequence[int], shape: Sequence[int]) -> int:
    return int(lib().vo_num_tiles(*map(int, grid), *map(int, shape)))


def token_tile_map(grid, shape) -> np.ndarray:
    n = int(np.prod(grid))
    out = np.empty(n, np.int32)
    _ok(lib().vo_token_tile_map(*map(int, grid), *map(int, shape), _p(out)), "token_tile_map")
    return out


def tile_layout(x: np.ndarray, grid, shape, channel_major: bool = False):
    """x [N, d] of any fixed-size dtype -> (x_tiled, valid_mask u64 [N_T] (tiles of up to 64 tokens)
    or [N_T, 2] (up to 128), valid_cnt i32 [N_T])."""
    x = np.ascontiguousarray(x)
    n, d = x.shape
    assert n == int(np.prod(grid))
    nt = num_tiles(grid, shape)
    b = int(np.prod(shape))
    out = np.empty((nt, d, b) if channel_major else (nt, b, d), x.dtype)
    mask = np.empty(nt if b <= 64 else (nt, 2), np.uint64)
    cnt = np.empty(nt, np.int32)
    _ok(lib().vo_tile_layout(_p(x), x.dtype.itemsize, d, *map(int, grid), *map(int, shape),
                             int(channel_major), _p(out), _p(mask), _p(cnt)), "tile_layout")
    return out, mask, cnt


def untile(y_tiled: np.ndarray, grid, shape) -> np.ndarray:
    y_tiled = np.ascontiguousarray(y_tiled)
    nt, b, d = y_tiled.shape
    out = np.empty((int(np.prod(grid)), d), y_tiled.dtype)
    _ok(lib().vo_untile(_p(y_tiled), y_tiled.dtype.itemsize, d, *map(int, grid), *map(int, shape),
                        _p(out)), "untile")
    return out


def trippool(x: np.ndarray, grid, shape) -> np.ndarray:
    """x [N, d] -> z [N_T, 3d] = [avg | max | min] in fp32."""
    x = _f32(x)
    n, d = x.shape
    z = np.empty((num_tiles(grid, shape), 3 * d), np.float32)
    _ok(lib().vo_trippool(_p(x), d, *map(int, grid), *map(int, shape), _p(z)), "trippool")
    return z


def mlp(z: np.ndarray, w1, b1, w2=None, b2=None, relu: bool = True) -> np.ndarray:
    """Two-layer (or, with w2 None, single-layer) projection of descriptors z [n, in]."""
    z = _f32(z)
    n, in_dim = z.shape
    w1, b1 = _f32(w1), _f32(b1)
    if w2 is None:
        hidden, out_dim = 0, w1.shape[1]
        w2a = b2a = None
    else:
        w2a, b2a = _f32(w2), _f32(b2)
        hidden, out_dim = w1.shape[1], w2a.shape[1]
        assert w2a.shape[0] == hidden
    assert w1.shape[0] == in_dim
    y = np.empty((n, out_dim), np.float32)
    _ok(lib().vo_mlp(_p(z), n, in_dim, hidden, out_dim, int(relu), _p(w1), _p(b1), _p(w2a), _p(b2a),
                     _p(y)), "mlp")
    return y


def score(qh: np.ndarray, kh: np.ndarray, scale: float) -> np.ndarray:
    qh, kh = _f32(qh), _f32(kh)
    s = np.empty((qh.shape[0], kh.shape[0]), np.float32)
    _ok(lib().vo_score(_p(qh), _p(kh), qh.shape[0], kh.shape[0], qh.shape[1],
                       C.c_float(np.float32(scale)), _p(s)), "score")
    return s


def select(s: np.ndarray, k: int, want_mask: bool = False):
    s = _f32(s)
    rows, cols = s.shape
    idx = np.empty((rows, k), np.int32)
    mask = np.empty((rows, cols), np.uint8) if want_mask else None
    _ok(lib().vo_select(_p(s), rows, cols, int(k), _p(idx), _p(mask)), "select")
    return (idx, mask) if want_mask else idx


def masked_attention(q, k, v, grid, shape, sel: np.ndarray, scale: float, queries,
                     want_stats: bool = False):
    """Attention of the listed query tokens under the token mask induced by sel [N_T, ksel]."""
    q, k, v = _f32(q), _f32(k), _f32(v)
    d = q.shape[1]
    sel = np.ascontiguousarray(sel, np.int32)
    queries = np.ascontiguousarray(queries, np.int64)
    out = np.empty((len(queries), d), np.float64)
    lse = np.empty(len(queries), np.float64) if want_stats else None
    ws = np.empty(len(queries), np.float64) if want_stats else None
    _ok(lib().vo_masked_attention(_p(q), _p(k), _p(v), d, *map(int, grid), *map(int, shape), _p(sel),
                                  sel.shape[1], float(scale), _p(queries), len(queries), _p(out),
                                  _p(lse), _p(ws)), "masked_attention")
    return (out, lse, ws) if want_stats else out


def dense_attention(q, k, v, scale: float, queries) -> np.ndarray:
    q, k, v = _f32(q), _f32(k), _f32(v)
    queries = np.ascontiguousarray(queries, np.int64)
    out = np.empty((len(queries), q.shape[1]), np.float64)
    _ok(lib().vo_dense_attention(_p(q), _p(k), _p(v), q.shape[1], q.shape[0], float(scale),
                                 _p(queries), len(queries), _p(out)), "dense_attention")
    return out


def tile_heatmap(q, k, grid, shape, scale: float, query_tiles=None) -> np.ndarray:
    """Max-pooled full-attention probabilities per (query tile, key tile): [N_T, N_T] float64.
    With query_tiles given, only those rows are computed; the others are NaN."""
    q, k = _f32(q), _f32(k)
    nt = num_tiles(grid, shape)
    heat = np.full((nt, nt), np.nan, np.float64)
    if query_tiles is None:
        qt, n_qt = None, -1
    else:
        qt = np.ascontiguousarray(query_tiles, np.int32)
        n_qt = len(qt)
    _ok(lib().vo_tile_heatmap(_p(q), _p(k), q.shape[1], *map(int, grid), *map(int, shape), float(scale),
                              _p(qt), n_qt, _p(heat)), "tile_heatmap")
    return heat


def recall(sel_sp: np.ndarray, sel_fu: np.ndarray) -> float:
    """Tile recall of selection sel_sp against sel_fu, both [rows, k] lists of key tiles."""
    a = np.ascontiguousarray(sel_sp, np.int32)
    b = np.ascontiguousarray(sel_fu, np.int32)
    assert a.shape == b.shape and a.ndim == 2
    out = C.c_double(0.0)
    _ok(lib().vo_recall(_p(a), _p(b), a.shape[0], a.shape[1], C.byref(out)), "recall")
    return float(out.value)


def closed_form_latent(z: np.ndarray, lam: float) -> np.ndarray:
    """TripPool descriptors z [n, 3d] -> y [n, 2d] = [avg | sqrt(lambda) * sqrt((max-avg)(avg-min))]."""
    z = _f32(z)
    n, d3 = z.shape
    d = d3 // 3
    y = np.empty((n, 2 * d), np.float32)
    _ok(lib().vo_closed_form_latent(_p(z), n, d, C.c_float(np.sqrt(np.float32(lam))), _p(y)), "closed_form_latent")
    return y


def closed_form_scores(q, k, grid, shape, lam: float) -> np.ndarray:
    """Weight-free tile scores: mean product plus lambda times the dispersion product, per channel."""
    yq = closed_form_latent(trippool(q, grid, shape), lam)
    yk = closed_form_latent(trippool(k, grid, shape), lam)
    return score(yq, yk, np.float32(1.0))


def tiling_search_errors(q, k, v, grid, candidates, keep, scale: float) -> np.ndarray:
    """Alg. 1 (head-aware tiling search) for one head and one calibration sample: for every
    candidate tile shape, the squared Frobenius distance between the full-attention output and
    the tile-sparse output under the reference top-k mask of that tiling (Eq. 8's summand).
    The reference mask is the per-row top-k (k = ceil(keep[0] * N_T / keep[1]), at least 1) of the
    max-pooled full-attention map, rounded to fp32 before the selection (the precision the GPU
    path selects in).  Returns float64 [len(candidates)]; argmin is the head's tiling."""
    n = q.shape[0]
    queries = np.arange(n)
    o_full = dense_attention(q, k, v, scale, queries)
    errs = np.empty(len(candidates), np.float64)
    for c, shape in enumerate(candidates):
        nt = num_tiles(grid, shape)
        ksel = max(1, -(-keep[0] * nt // keep[1]))
        heat = tile_heatmap(q, k, grid, shape, scale)
        sel = select(heat.astype(np.float32), ksel)
        o_sp = masked_attention(q, k, v, grid, shape, sel, scale, queries)
        errs[c] = float(((o_full - o_sp) ** 2).sum())
    return errs


def estimate_and_select(q, k, grid, shape, phi_q, phi_k, head: int, ksel: int, scale=None):
    """Stages 2-3 for one head in the paper's order: TripPool -> phi -> score -> top-k.
    phi_* carry per-head arrays w1,b1,w2,b2 and out_dim.  Returns (z_q, z_k, qh, kh, s, idx)."""
    zq, zk = trippool(q, grid, shape), trippool(k, grid, shape)
    qh = mlp(zq, phi_q.w1[head], phi_q.b1[head], phi_q.w2[head], phi_q.b2[head], phi_q.relu)
    kh = mlp(zk, phi_k.w1[head], phi_k.b1[head], phi_k.w2[head], phi_k.b2[head], phi_k.relu)
    if scale is None:
        scale = np.float32(1.0) / np.sqrt(np.float32(phi_q.out_dim))
    s = score(qh, kh, scale)
    return zq, zk, qh, kh, s, select(s, ksel)
