"""Pins of the CPU oracle against things other than itself: brute force on tiny inputs,
closed forms, invariants, special cases that reduce to library routines, and the one
figure the paper prints (padded slot count).  CPU only."""
from pathlib import Path

import numpy as np
import pytest
import torch

from oracle import oracle as vo
from paper_2605_30325_amd import workloads as wlm
from tests import brute_force as bf

GRIDS = [((4, 8, 8), (4, 4, 4)), ((5, 6, 7), (4, 4, 4)), ((3, 9, 10), (1, 8, 8)),
         ((21, 5, 3), (16, 2, 2)), ((2, 3, 130), (1, 1, 64))]


def _rand(n, d, seed, dtype=np.float32):
    return np.random.default_rng(seed).standard_normal((n, d)).astype(dtype)


# ---------------------------------------------------------------- stage 1: layout
def test_padded_slot_count_matches_paper_figure():
    rows = [l.split() for l in Path(__file__).with_name("golden").joinpath("padded_slots.txt")
            .read_text().splitlines() if l.strip() and not l.startswith("#")]
    for T, H, W, pt, ph, pw, real, padded in (map(int, r) for r in rows):
        assert T * H * W == real
        assert vo.num_tiles((T, H, W), (pt, ph, pw)) * pt * ph * pw == padded


@pytest.mark.parametrize("grid,shape", GRIDS)
def test_layout_brute_force_bijection_roundtrip(grid, shape):
    n, d = int(np.prod(grid)), 5
    x = _rand(n, d, 1)
    xt, mask, cnt = vo.tile_layout(x, grid, shape)
    tab = bf.slots(grid, shape)
    B = int(np.prod(shape))
    ref = np.zeros_like(xt)
    for (i, l), tok in tab.items():
        ref[i, l] = x[tok]
    assert np.array_equal(xt, ref)
    # bijection: every token exactly once; padded slots are zero; mask/cnt agree
    assert sorted(tab.values()) == list(range(n))
    bits = np.array([[(int(m) >> l) & 1 for l in range(B)] for m in mask])
    assert bits.sum() == n and np.array_equal(bits.sum(1), cnt) and cnt.min() >= 1
    for i in range(xt.shape[0]):
        for l in range(B):
            assert bits[i, l] == ((i, l) in tab)
    assert np.array_equal(vo.untile(xt, grid, shape), x)
    # channel-major form is the per-tile transpose
    xc, mask2, _ = vo.tile_layout(x, grid, shape, channel_major=True)
    assert np.array_equal(xc, xt.transpose(0, 2, 1)) and np.array_equal(mask, mask2)
    # byte moves work for any element size
    x16 = x.view(np.uint16).reshape(n, 2 * d)
    assert np.array_equal(vo.tile_layout(x16, grid, shape)[0].view(np.float32), xt)


@pytest.mark.parametrize("grid,shape", [((8, 4, 8), (8, 4, 4)), ((5, 9, 10), (2, 8, 8)), ((33, 3, 5), (32, 2, 2)),
                                        ((3, 5, 130), (1, 1, 128))])
def test_128_token_tiles_layout_trippool_attention(grid, shape):
    # the paper's tile size (Sec. 4.2, B = 128): two mask words per tile, same definitions otherwise
    n, d = int(np.prod(grid)), 6
    x = _rand(n, d, 80)
    xt, mask, cnt = vo.tile_layout(x, grid, shape)
    tab = bf.slots(grid, shape)
    ref = np.zeros_like(xt)
    for (i, l), tok in tab.items():
        ref[i, l] = x[tok]
    assert xt.shape[1] == 128 and np.array_equal(xt, ref) and mask.shape == (xt.shape[0], 2)
    for i in range(xt.shape[0]):
        for l in range(128):
            assert ((int(mask[i, l // 64]) >> (l % 64)) & 1) == ((i, l) in tab)
    assert cnt.sum() == n and np.array_equal(vo.untile(xt, grid, shape), x)
    xc, _, _ = vo.tile_layout(x, grid, shape, channel_major=True)
    assert np.array_equal(xc, xt.transpose(0, 2, 1))
    z = vo.trippool(x, grid, shape)
    zr = bf.trippool64(x, grid, shape)
    assert np.array_equal(z[:, d:], zr[:, d:].astype(np.float32))
    assert np.allclose(z[:, :d], zr[:, :d], rtol=0, atol=128 * 2**-24 * 4)
    nt = vo.num_tiles(grid, shape)
    rng = np.random.default_rng(81)
    ksel = max(1, nt // 2)
    sel = np.stack([np.sort(rng.choice(nt, ksel, replace=False)) for _ in range(nt)]).astype(np.int32)
    q, k, v = _rand(n, d, 82), _rand(n, d, 83), _rand(n, d, 84)
    out = vo.masked_attention(q, k, v, grid, shape, sel, 0.4, np.arange(n))
    assert np.allclose(out, bf.concat_tile_attention(q, k, v, grid, shape, sel, 0.4), rtol=1e-12, atol=1e-12)


def test_layout_row_tiles_are_identity():
    # a 1x1xB tile on a grid whose width is a multiple of B keeps raster order
    grid, shape = (2, 3, 128), (1, 1, 64)
    x = _rand(int(np.prod(grid)), 4, 2)
    xt, mask, _ = vo.tile_layout(x, grid, shape)
    assert np.array_equal(xt.reshape(-1, 4), x) and np.all(mask == np.uint64(2**64 - 1))


@pytest.mark.parametrize("grid,shape", GRIDS[:4])
def test_layout_temporal_neighbours_distance(grid, shape):
    # App. A.5: tokens (t,h,w) and (t+1,h,w) of one tile sit exactly p_h*p_w slots apart
    T, H, W = grid
    pt, ph, pw = shape
    ids = np.arange(T * H * W, dtype=np.int64).reshape(-1, 1)
    xt, _, _ = vo.tile_layout(ids, grid, shape)
    pos = {int(tok): (i, l) for i in range(xt.shape[0]) for l, tok in enumerate(xt[i, :, 0])
           if not (tok == 0 and (i, l) != (0, 0))}
    tile_of = vo.token_tile_map(grid, shape)
    checked = 0
    for t in range(T - 1):
        for h in range(H):
            for w in range(W):
                a, b = (t * H + h) * W + w, ((t + 1) * H + h) * W + w
                assert tile_of[a] == pos[a][0]
                if pos[a][0] == pos[b][0]:
                    assert pos[b][1] - pos[a][1] == ph * pw
                    checked += 1
    assert checked > 0 or pt == 1


# ---------------------------------------------------------------- stage 2: statistics + score
@pytest.mark.parametrize("grid,shape", GRIDS[:4])
def test_trippool_brute_force_and_invariants(grid, shape):
    n, d = int(np.prod(grid)), 6
    x = _rand(n, d, 3)
    z = vo.trippool(x, grid, shape)
    ref = bf.trippool64(x, grid, shape)
    assert np.array_equal(z[:, d:], ref[:, d:].astype(np.float32))          # max, min exact
    assert np.allclose(z[:, :d], ref[:, :d], rtol=0, atol=64 * 2**-24 * 4)  # fp32 chain of <=64 adds
    avg, mx, mn = z[:, :d].astype(np.float64), z[:, d:2 * d], z[:, 2 * d:]
    assert np.all(mn <= avg + 1e-6) and np.all(avg <= mx + 1e-6)
    # Bhatia-Davis (App. A.3): variance <= (max - mean)(mean - min)
    for i, mem in enumerate(bf.tile_members(grid, shape)):
        var = x[mem].astype(np.float64).var(0)
        assert np.all(var <= (mx[i] - avg[i]) * (avg[i] - mn[i]) + 1e-5)


def test_trippool_constant_tile_and_order():
    grid, shape = (4, 4, 8), (4, 4, 4)
    x = np.full((128, 3), 1.25, np.float32)
    z = vo.trippool(x, grid, shape)
    assert np.all(z == np.float32(1.25))
    # the fp32 sum is a chain over ascending slot order: check one tile against an explicit chain
    x = _rand(128, 1, 4) * np.float32(1000.0)
    z = vo.trippool(x, grid, shape)
    for i, mem in enumerate(bf.tile_members(grid, shape)):
        acc = np.float32(0.0)
        for tok in mem:
            acc = np.float32(acc + x[tok, 0])
        assert z[i, 0] == np.float32(acc * (np.float32(1.0) / np.float32(len(mem))))


def test_mlp_matches_float64_and_special_cases():
    rng = np.random.default_rng(5)
    n, d, dp = 7, 8, 4
    z = rng.standard_normal((n, 3 * d)).astype(np.float32)
    w1 = rng.uniform(-0.3, 0.3, (3 * d, d)).astype(np.float32)
    b1 = rng.uniform(-0.1, 0.1, d).astype(np.float32)
    w2 = rng.uniform(-0.3, 0.3, (d, dp)).astype(np.float32)
    b2 = rng.uniform(-0.1, 0.1, dp).astype(np.float32)
    for relu in (True, False):
        y = vo.mlp(z, w1, b1, w2, b2, relu)
        assert np.allclose(y, bf.mlp64(z, w1, b1, w2, b2, relu), rtol=1e-5, atol=1e-5)
    assert not np.allclose(vo.mlp(z, w1, b1, w2, b2, True), vo.mlp(z, w1, b1, w2, b2, False))
    y1 = vo.mlp(z, w1, b1)
    assert np.allclose(y1, bf.mlp64(z, w1, b1), rtol=1e-5, atol=1e-5)
    # identity projection returns the descriptor bit for bit (fma(z,1,0) chains with zeros)
    eye = np.eye(3 * d, dtype=np.float32)
    assert np.array_equal(vo.mlp(z, eye, np.zeros(3 * d, np.float32)), z)


def test_score_special_cases():
    grid, shape, d = (4, 8, 8), (4, 4, 4), 16
    n = int(np.prod(grid))
    q, k = _rand(n, d, 6), _rand(n, d, 7)
    zq, zk = vo.trippool(q, grid, shape), vo.trippool(k, grid, shape)
    zeros = np.zeros(d, np.float32)
    # "AvgId": a single linear layer that keeps only the Avg block gives the mean-pooling score
    w_avg = np.zeros((3 * d, d), np.float32)
    w_avg[:d] = np.eye(d, dtype=np.float32)
    scale = np.float32(1.0 / np.sqrt(d))
    s = vo.score(vo.mlp(zq, w_avg, zeros), vo.mlp(zk, w_avg, zeros), scale)
    mem = bf.tile_members(grid, shape)
    mq = np.stack([q[m].astype(np.float64).mean(0) for m in mem])
    mk = np.stack([k[m].astype(np.float64).mean(0) for m in mem])
    assert np.allclose(s, mq @ mk.T / np.sqrt(d), rtol=1e-5, atol=1e-6)
    # identity on all 3d statistics: avg.avg + max.max + min.min over sqrt(3d)
    eye = np.eye(3 * d, dtype=np.float32)
    z3 = np.zeros(3 * d, np.float32)
    s3 = vo.score(vo.mlp(zq, eye, z3), vo.mlp(zk, eye, z3), np.float32(1.0 / np.sqrt(3 * d)))
    ref = sum(bf.trippool64(q, grid, shape)[:, a * d:(a + 1) * d]
              @ bf.trippool64(k, grid, shape)[:, a * d:(a + 1) * d].T for a in range(3)) / np.sqrt(3 * d)
    assert np.allclose(s3, ref, rtol=1e-5, atol=1e-5)
    # Q == K with shared weights gives a bitwise symmetric score matrix
    ss = vo.score(vo.mlp(zq, eye, z3), vo.mlp(zq, eye, z3), np.float32(0.125))
    assert np.array_equal(ss, ss.T)
    # transposed operands: score(q,k) == score(k,q)^T bitwise (fma chain is commutative per term)
    assert np.array_equal(vo.score(zq, zk, np.float32(0.5)), vo.score(zk, zq, np.float32(0.5)).T)


def test_fp32_chains_run_in_ascending_index_order():
    """The fp32 chains decide the top-k set, so their order is part of the definition: ascending index,
    the projections starting from the bias, the score from +0.  Inputs whose partial sums absorb a small
    term make the order visible: (1, 2^30, -2^30) summed left to right gives 0, right to left 1."""
    big = np.float32(2.0 ** 30)
    row = np.array([[1.0, big, -big]], np.float32)
    ones = np.ones((1, 3), np.float32)
    # score: fma chain from +0 over the latent index, then one multiply by the scale
    assert vo.score(row, ones, np.float32(0.5))[0, 0] == 0.0
    assert vo.score(row[:, ::-1].copy(), ones, np.float32(0.5))[0, 0] == 0.5
    # single layer: chain from the bias; the bias (0.25) is absorbed first, the trailing 1 survives
    w = np.ones((3, 1), np.float32)
    quarter = np.array([0.25], np.float32)
    assert vo.mlp(row, w, quarter)[0, 0] == 0.0                 # ((0.25 + 1) + 2^30) - 2^30
    assert vo.mlp(row[:, ::-1].copy(), w, quarter)[0, 0] == 1.0   # ((0.25 - 2^30) + 2^30) + 1
    # two layers, identity first layer (no activation): the second chain sees the same three terms
    eye, z3 = np.eye(3, dtype=np.float32), np.zeros(3, np.float32)
    assert vo.mlp(row, eye, z3, w, quarter, relu=False)[0, 0] == 0.0
    assert vo.mlp(row[:, ::-1].copy(), eye, z3, w, quarter, relu=False)[0, 0] == 1.0
    # first layer of two: hidden unit j sums the inputs in ascending order from its bias
    w1 = np.ones((3, 2), np.float32)
    b1 = np.array([0.25, 0.25], np.float32)
    w2 = np.array([[1.0], [0.0]], np.float32)
    assert vo.mlp(row, w1, b1, w2, np.zeros(1, np.float32), relu=False)[0, 0] == 0.0
    assert vo.mlp(row[:, ::-1].copy(), w1, b1, w2, np.zeros(1, np.float32), relu=False)[0, 0] == 1.0


# ---------------------------------------------------------------- stage 3: top-k
@pytest.mark.parametrize("cols,k", [(4, 2), (37, 1), (37, 5), (64, 64), (130, 17)])
def test_select_brute_force_and_invariants(cols, k):
    rng = np.random.default_rng(cols * 100 + k)
    s = rng.standard_normal((9, cols)).astype(np.float32)
    idx, mask = vo.select(s, k, want_mask=True)
    assert np.array_equal(idx, bf.topk_rows(s, k))
    assert np.all(mask.sum(1) == k)                                    # exactly k per row
    assert np.all(np.diff(idx, axis=1) > 0) if k > 1 else True          # strictly ascending
    for r in range(s.shape[0]):
        kept, dropped = s[r, mask[r] == 1], s[r, mask[r] == 0]
        if dropped.size:
            assert kept.min() >= dropped.max()
    if k == cols:
        assert np.array_equal(idx, np.tile(np.arange(cols, dtype=np.int32), (9, 1)))
    if k == 1:
        assert np.array_equal(idx[:, 0], np.argmax(s, axis=1))


def test_select_ties_nan_and_signed_zero():
    rng = np.random.default_rng(11)
    s = rng.integers(0, 4, size=(20, 50)).astype(np.float32)            # many equal scores
    for k in (1, 7, 25, 50):
        idx = vo.select(s, k)
        assert np.array_equal(idx, bf.topk_rows(s, k))
        for r in range(20):                                              # boundary ties -> lower index
            thr = np.sort(s[r])[::-1][k - 1]
            tied = np.flatnonzero(s[r] == thr)
            n_tied_kept = k - int((s[r] > thr).sum())
            assert set(tied[:n_tied_kept]) <= set(idx[r]) and not (set(tied[n_tied_kept:]) & set(idx[r]))
    s = np.array([[0.0, -0.0, np.nan, -1.0, 0.0]], np.float32)
    assert vo.select(s, 2).tolist() == [[0, 1]]                          # -0 == +0, lower index first
    assert vo.select(s, 4).tolist() == [[0, 1, 3, 4]]                    # NaN ranks last (as -inf)
    s = np.array([[np.nan, -np.inf, np.nan]], np.float32)
    assert vo.select(s, 2).tolist() == [[0, 1]]


# ---------------------------------------------------------------- stage 4: masked attention
def _tiny_problem(seed=0, grid=(4, 8, 8), shape=(4, 4, 4), d=8):
    n = int(np.prod(grid))
    q, k, v = _rand(n, d, seed), _rand(n, d, seed + 1), _rand(n, d, seed + 2)
    return grid, shape, n, d, q, k, v


@pytest.mark.parametrize("grid,shape", [((4, 8, 8), (4, 4, 4)), ((5, 6, 7), (4, 4, 4)),
                                        ((3, 9, 10), (1, 8, 8)), ((18, 3, 3), (16, 2, 2))])
def test_attention_matches_concat_form_brute_force(grid, shape):
    _, _, n, d, q, k, v = _tiny_problem(20, grid, shape)
    nt = vo.num_tiles(grid, shape)
    rng = np.random.default_rng(21)
    ksel = max(1, nt // 2)
    sel = np.stack([np.sort(rng.choice(nt, ksel, replace=False)) for _ in range(nt)]).astype(np.int32)
    scale = 1.0 / np.sqrt(d)
    out, lse, ws = vo.masked_attention(q, k, v, grid, shape, sel, scale, np.arange(n), want_stats=True)
    ref = bf.concat_tile_attention(q, k, v, grid, shape, sel, scale)    # Eq. 2 written independently
    assert np.allclose(out, ref, rtol=1e-12, atol=1e-12)
    assert np.allclose(ws, 1.0, atol=1e-12)                             # rows of A sum to one
    ones = vo.masked_attention(q, k, np.ones_like(v), grid, shape, sel, scale, np.arange(n))
    assert np.allclose(ones, 1.0, atol=1e-12)
    # order of the kept list does not matter
    out2 = vo.masked_attention(q, k, v, grid, shape, sel[:, ::-1].copy(), scale, np.arange(n))
    assert np.allclose(out, out2, rtol=0, atol=1e-13)


@pytest.mark.parametrize("shape", [(4, 4, 4), (1, 8, 8), (16, 2, 2)])
def test_zero_sparsity_equals_dense_attention(shape):
    grid = (5, 6, 9)
    _, _, n, d, q, k, v = _tiny_problem(30, grid, shape)
    nt = vo.num_tiles(grid, shape)
    sel = np.tile(np.arange(nt, dtype=np.int32), (nt, 1))
    scale = 1.0 / np.sqrt(d)
    out = vo.masked_attention(q, k, v, grid, shape, sel, scale, np.arange(n))
    ref, _ = bf.dense_attention64(q, k, v, scale)                       # Eq. 1 with library matmuls
    assert np.allclose(out, ref, rtol=1e-12, atol=1e-12)
    assert np.allclose(vo.dense_attention(q, k, v, scale, np.arange(n)), ref, rtol=1e-12, atol=1e-12)


def test_renormalisation_under_mask_and_equal_keys():
    grid, shape, n, d, q, k, v = _tiny_problem(40)
    nt = vo.num_tiles(grid, shape)
    sel = np.array([[0, 2], [1, 3], [0, 1], [2, 3]], np.int32)
    scale = 1.0 / np.sqrt(d)
    out, lse, _ = vo.masked_attention(q, k, v, grid, shape, sel, scale, np.arange(n), want_stats=True)
    _, P = bf.dense_attention64(q, k, v, scale)                          # full-attention weights
    tile_of = vo.token_tile_map(grid, shape)
    for u in range(n):
        kept = np.isin(tile_of, sel[tile_of[u]])
        # Prop. A.1: sparse weights are the dense ones restricted to the kept set, times Z/Z_hat
        ref = (P[u, kept, None] * v[kept]).sum(0) / P[u, kept].sum()
        assert np.allclose(out[u], ref, rtol=1e-10, atol=1e-12)
        logits = (q[u].astype(np.float64) @ k[kept].astype(np.float64).T) * scale
        assert np.isclose(lse[u], np.log(np.exp(logits).sum()), rtol=1e-12)
    # all keys equal: uniform weights, output is the mean of the kept value rows
    kk = np.tile(k[:1], (n, 1))
    out = vo.masked_attention(q, kk, v, grid, shape, sel, scale, np.arange(n))
    mem = bf.tile_members(grid, shape)
    for u in range(0, n, 17):
        keys = [t for j in sel[tile_of[u]] for t in mem[j]]
        assert np.allclose(out[u], v[keys].astype(np.float64).mean(0), atol=1e-12)


def test_planted_mistakes_are_caught_by_the_pins():
    """A transposed tile shape, an off-by-one budget or a wrong scale must change results."""
    grid, n, d = (4, 8, 8), 256, 8
    x = _rand(n, d, 50)
    assert not np.array_equal(vo.tile_layout(x, grid, (1, 8, 8))[0], vo.tile_layout(x, grid, (8, 8, 1))[0])
    s = _rand(6, 12, 51)
    assert not np.array_equal(vo.select(s, 3), vo.select(s, 4)[:, :3])
    q, k, v = _rand(n, d, 52), _rand(n, d, 53), _rand(n, d, 54)
    sel = np.array([[0, 1]] * 4, np.int32)
    a = vo.masked_attention(q, k, v, grid, (4, 4, 4), sel, 1.0 / np.sqrt(d), np.arange(8))
    b = vo.masked_attention(q, k, v, grid, (4, 4, 4), sel, 1.0 / d, np.arange(8))
    assert not np.allclose(a, b)


# ---------------------------------------------------------------- target heat map and recall
@pytest.mark.parametrize("grid,shape", [((4, 8, 8), (4, 4, 4)), ((3, 9, 10), (1, 8, 8)), ((17, 3, 5), (16, 2, 2))])
def test_tile_heatmap_against_brute_force(grid, shape):
    n, d = int(np.prod(grid)), 8
    q, k = 2.0 * _rand(n, d, 60), 2.0 * _rand(n, d, 61)
    scale = 1.0 / np.sqrt(d)
    heat = vo.tile_heatmap(q, k, grid, shape, scale)
    ref = bf.tile_heatmap64(q, k, grid, shape, scale)
    assert heat.shape == ref.shape and np.allclose(heat, ref, rtol=1e-10, atol=1e-15)
    # a subset of query tiles gives the same rows and leaves the others alone
    some = [0, heat.shape[0] - 1]
    part = vo.tile_heatmap(q, k, grid, shape, scale, query_tiles=some)
    assert np.array_equal(part[some], heat[some])
    rest = np.setdiff1d(np.arange(heat.shape[0]), some)
    assert np.isnan(part[rest]).all()


def test_tile_heatmap_closed_forms():
    grid, shape = (4, 8, 12), (4, 4, 4)        # 384 tokens, 6 full tiles
    n, d = 384, 8
    k = _rand(n, d, 62)
    # zero queries: uniform attention, every block maximum is 1/N
    heat = vo.tile_heatmap(np.zeros((n, d), np.float32), k, grid, shape, 0.3)
    assert np.allclose(heat, 1.0 / n, rtol=1e-12)
    # one key that every query prefers by a wide margin: its tile's column is ~1, the rest ~0
    q = np.abs(_rand(n, d, 63)) + 0.5
    kk = 0.01 * _rand(n, d, 64)
    v_star = 200
    kk[v_star] = 50.0
    heat = vo.tile_heatmap(q, kk, grid, shape, 1.0)
    j_star = vo.token_tile_map(grid, shape)[v_star]
    assert np.all(heat[:, j_star] > 1.0 - 1e-9)
    assert np.all(np.delete(heat, j_star, axis=1) < 1e-9)
    # a block maximum is a probability; the maxima of a row of blocks cover the row's largest weight
    q2, k2 = _rand(n, d, 65), _rand(n, d, 66)
    heat = vo.tile_heatmap(q2, k2, grid, shape, 0.5)
    assert np.all(heat > 0.0) and np.all(heat <= 1.0)
    assert np.all(heat.sum(axis=1) >= 1.0 / 64)   # some query of the tile puts >= 1/N_T of its mass in one tile
    # a ragged grid: padded slots take no part (same result as brute force above), and the
    # scale matters
    assert not np.allclose(heat, vo.tile_heatmap(q2, k2, grid, shape, 1.0))


def test_recall_against_sets_and_hand_values():
    rng = np.random.default_rng(67)
    a = np.stack([rng.choice(40, 8, replace=False) for _ in range(25)]).astype(np.int32)
    b = np.stack([rng.choice(40, 8, replace=False) for _ in range(25)]).astype(np.int32)
    assert np.isclose(vo.recall(a, b), bf.recall64(a, b), rtol=0, atol=1e-15)
    assert vo.recall(a, a[:, ::-1]) == 1.0
    assert vo.recall(a, a + 40) == 0.0
    assert vo.recall(np.array([[0, 1, 2, 3]], np.int32), np.array([[3, 9, 8, 0]], np.int32)) == 0.5
    # top-k of the heat map against itself shifted by one tile: every row shares k-1 tiles
    top = np.tile(np.arange(5, dtype=np.int32), (6, 1))
    assert np.isclose(vo.recall(top, top + 1), 0.8)


def test_tiling_search_errors_against_brute_force_and_limits():
    grid, n, d = (4, 8, 8), 256, 8
    cands = [(4, 4, 4), (1, 8, 8), (2, 4, 8)]
    q, k, v = 1.5 * _rand(n, d, 70), 1.5 * _rand(n, d, 71), _rand(n, d, 72)
    scale = 1.0 / np.sqrt(d)
    errs = vo.tiling_search_errors(q, k, v, grid, cands, (2, 4), scale)
    o_full, _ = bf.dense_attention64(q, k, v, scale)
    for c, shape in enumerate(cands):
        heat = bf.tile_heatmap64(q, k, grid, shape, scale).astype(np.float32)
        sel = bf.topk_rows(heat, 2)          # 4 tiles per tiling, keep 2/4
        o_sp = bf.concat_tile_attention(q, k, v, grid, shape, sel, scale)
        assert np.isclose(errs[c], ((o_full - o_sp) ** 2).sum(), rtol=1e-9)
    assert np.all(errs > 0)
    # keeping every tile reproduces full attention: the error vanishes for every tiling
    full = vo.tiling_search_errors(q, k, v, grid, cands, (1, 1), scale)
    assert np.all(full < 1e-20)
    # a head whose attention is local in time only: tiles that are thin in time must lose
    t_of = np.arange(n) // 64
    qq = np.zeros((n, d), np.float32)
    qq[np.arange(n), t_of] = 6.0
    local = vo.tiling_search_errors(qq, qq.copy(), v, grid, [(1, 8, 8), (4, 4, 4)], (1, 4), 1.0)
    assert local[0] < 1e-6 and local[1] > 1e-3 and int(np.argmin(local)) == 0


def test_closed_form_scorer_terms():
    grid, shape, d = (4, 8, 12), (4, 4, 4), 6
    n = int(np.prod(grid))
    q, k = _rand(n, d, 90), _rand(n, d, 91)
    mem = bf.tile_members(grid, shape)
    # lambda = 0: the score is the dot product of the tile means = the mean of q_u.k_v over the block
    s0 = vo.closed_form_scores(q, k, grid, shape, 0.0)
    q64, k64 = q.astype(np.float64), k.astype(np.float64)
    for i in (0, 3, 5):
        for j in (1, 4):
            block = q64[mem[i]] @ k64[mem[j]].T
            assert np.isclose(s0[i, j], block.mean(), rtol=1e-5, atol=1e-6)
    # the lambda term is lambda * sum_c Delta_q Delta_k with Delta^2 = (max - mean)(mean - min) >= variance
    lam = 0.7
    s1 = vo.closed_form_scores(q, k, grid, shape, lam)
    def delta(x, rows):
        x = x[rows]
        return np.sqrt((x.max(0) - x.mean(0)) * (x.mean(0) - x.min(0)))
    for i in (0, 5):
        for j in (2, 3):
            want = s0[i, j] + lam * float(delta(q64, mem[i]) @ delta(k64, mem[j]))
            assert np.isclose(s1[i, j], want, rtol=1e-5, atol=1e-6)
            assert np.all(delta(q64, mem[i]) ** 2 >= q64[mem[i]].var(0) - 1e-12)     # Bhatia-Davis
    # constant tiles have no dispersion: lambda does not matter
    qc = _rand(6, d, 92)[vo.token_tile_map(grid, shape)]
    assert np.array_equal(vo.closed_form_scores(qc, k, grid, shape, 0.0), vo.closed_form_scores(qc, k, grid, shape, 5.0))


# ---------------------------------------------------------------- workloads feed
def test_workload_sizes_match_the_size_table():
    w = wlm.WORKLOADS
    assert w["tiny"].tokens == 256 and wlm.keep_budget(w["tiny"]).tolist() == [2, 2]
    assert w["wan1p3b_480p"].tokens == 32760
    assert set(wlm.tiles_per_head(w["wan1p3b_480p"])) == {624}
    assert set(wlm.keep_budget(w["wan1p3b_480p"])) == {63}
    big = w["waver12b_720p_241f"]
    assert big.tokens == 219600
    nt = {tuple(s): n for s, n in zip(map(tuple, wlm.tile_shapes(big)), wlm.tiles_per_head(big))}
    for shape, n in nt.items():
        assert n == {(4, 4, 4): 3840, (1, 8, 8): 3660, (16, 2, 2): 3680}[shape]
        assert vo.num_tiles(big.grid, shape) == n
    q = wlm.make_head(w["tiny"], "q", 0)
    assert q.shape == (256, 64) and q.dtype.is_floating_point
    assert np.array_equal(q.numpy(), wlm.make_head(w["tiny"], "q", 0).numpy())


def test_generated_values_stay_bounded_on_degenerate_grids():
    # With T = 1 a channel whose sinusoids only vary along t is constant over the grid; the
    # unit-variance normalisation must drop it instead of dividing by ~0.
    wl = wlm.custom_workload("flat", 4, 128, "bf16", (1, 15, 17), True, (58, 100), 357998, batch=2)
    for b in range(2):
        for h in range(4):
            for t in ("q", "k", "v"):
                x = wlm.make_head(wl, t, h, batch=b).float()
                assert torch.isfinite(x).all() and float(x.abs().max()) < 8.0
