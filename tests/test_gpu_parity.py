"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Tile lists, masks, statistics and scores must match bit for bit; attention
outputs within the stated tolerances."""
import math
import sys

import numpy as np
import pytest
import torch

from oracle import oracle as vo
from paper_2605_30325_amd import veda
from paper_2605_30325_amd import workloads as wlm
from tests import harness as hz

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _full_check(wl, **kw):
    _say(f"[parity] {wl.name}: grid {wl.grid} heads {wl.heads} d {wl.head_dim} {wl.dtype}")
    run = hz.run_gpu_path(wl, **kw)
    assert torch.isfinite(run.out.float()).all(), "a real token was left unwritten or is not finite"
    for b in range(wl.batch):
        for h in range(wl.heads):
            st = hz.check_head(run, h, batch=b)
            _say(f"[parity] {wl.name} b{b} h{h} {tuple(run.shapes[h])}: {st}")
    return run


def test_tiny_config_everything():
    _full_check(wlm.WORKLOADS["tiny"])


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("f32", 64), ("f32", 128)])
def test_small_ragged_grids_all_shapes(dtype, d):
    # 6 heads cover the three tile shapes; every axis has a ragged tail for some shape
    wl = wlm.custom_workload(f"ragged_{dtype}_{d}", 6, d, dtype, (9, 10, 14), True, (25, 100), seed=11,
                             latent_dim=64 if d == 128 else 32)
    run = _full_check(wl)
    assert len({tuple(s) for s in run.shapes}) == 3


def test_batch_two_and_strided_input():
    wl = wlm.custom_workload("batch2", 3, 128, "bf16", (5, 8, 12), True, (30, 100), seed=12, batch=2)
    _full_check(wl)
    # [batch, N, heads, d] storage viewed as [batch, heads, N, d]: strides handed to the library
    dev = torch.device("cuda:0")
    shapes = wlm.tile_shapes(wl)
    q, _, _ = wlm.make_qkv(wl, dev)
    q_bnhd = q.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    assert not q_bnhd.is_contiguous()
    plan = veda.Plan(wl.batch, wl.heads, wl.head_dim, wl.grid, shapes, wl.torch_dtype)
    a, _, _ = veda.veda_tile_layout(plan, q)
    b, _, _ = veda.veda_tile_layout(plan, q_bnhd)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


@pytest.mark.parametrize("hidden,dp,relu,unit", [(0, 12, True, 0), (20, 12, True, 0), (131, 8, False, 0),
                                                  (260, 200, True, 0), (0, 12, True, 2), (131, 8, False, 2),
                                                  (260, 200, True, 2)])
def test_estimator_shapes_bit_exact(hidden, dp, relu, unit):
    # widths that are not multiples of the kernel's blocking, a single affine layer, no ReLU;
    # 135..180 tiles per head: several 64-row blocks and 128x128 score blocks, all with ragged tails.
    # unit = 2: the chains as scalar fmaf on the vector units (VEDA_OPT_FP32_CHAIN_UNIT), the form that
    # defines them; unit = 0: where the library's probe of this device put them (the matrix cores on gfx950)
    wl = wlm.custom_workload(f"mlp_{hidden}_{dp}", 2, 64, "f32", (10, 20, 36), True, (50, 100), seed=21,
                             latent_dim=dp)
    _say(f"[parity] {wl.name}: estimator 192 -> {hidden} -> {dp} relu={relu}")
    dev = torch.device("cuda:0")
    shapes = wlm.tile_shapes(wl)
    rng = np.random.default_rng(77 + hidden)
    first = hidden if hidden else dp

    def weights():
        w1 = rng.uniform(-0.1, 0.1, (wl.heads, 3 * wl.head_dim, first)).astype(np.float32)
        b1 = rng.uniform(-0.05, 0.05, (wl.heads, first)).astype(np.float32)
        if not hidden:
            return w1, b1, None, None
        return (w1, b1, rng.uniform(-0.2, 0.2, (wl.heads, hidden, dp)).astype(np.float32),
                rng.uniform(-0.05, 0.05, (wl.heads, dp)).astype(np.float32))

    wq, wk = weights(), weights()
    q, k, _ = wlm.make_qkv(wl, dev)
    plan = veda.Plan(wl.batch, wl.heads, wl.head_dim, wl.grid, shapes, wl.torch_dtype)
    if unit:
        plan.set_option(veda.VEDA_OPT_FP32_CHAIN_UNIT, unit)
        assert plan.chain_unit() == unit
    qt, vm, _ = veda.veda_tile_layout(plan, q, veda.VEDA_TOKEN_MAJOR)
    kt, _, _ = veda.veda_tile_layout(plan, k, veda.VEDA_TOKEN_MAJOR, want_mask=False)
    scale = hz.score_scale_of(wl)
    s, _ = veda.veda_tile_score(plan, qt, kt, vm, veda.Mlp(*wq, relu, dev), veda.Mlp(*wk, relu, dev), scale)
    torch.cuda.synchronize()
    for h in range(wl.heads):
        shape = tuple(int(x) for x in shapes[h])
        lat = []
        for x, w in ((q, wq), (k, wk)):
            z = vo.trippool(hz.to_f32_numpy(x[0, h]), wl.grid, shape)
            lat.append(vo.mlp(z, w[0][h], w[1][h], None if w[2] is None else w[2][h],
                              None if w[3] is None else w[3][h], relu))
        ref = vo.score(lat[0], lat[1], np.float32(scale))
        nt, soff = plan.tiles[h], plan.score_offset[h]
        got = s[0, soff:soff + nt * nt].view(nt, nt).cpu().numpy()
        assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), f"{wl.name} head {h}: scores not bit-exact"


def test_this_device_runs_the_fp32_chains_on_the_matrix_cores():
    """veda_plan_create probes the device: chains of v_mfma_f32_32x32x2_f32 against the fmaf chains they stand
    for (rounding, signed zeros, denormal sums and products).  On gfx950 every bit agrees, so plans use the
    matrix cores; were this to fail on another device or driver, the library would already have switched to
    the vector units by itself and every bit-exactness test would still hold."""
    wl = wlm.custom_workload("probe", 1, 64, "f32", (4, 8, 8), False, (1, 2), seed=5, latent_dim=4)
    plan = veda.Plan(wl.batch, wl.heads, wl.head_dim, wl.grid, wlm.tile_shapes(wl), wl.torch_dtype)
    assert plan.chain_unit() == veda.VEDA_CHAINS_MATRIX
    plan.set_option(veda.VEDA_OPT_FP32_CHAIN_UNIT, veda.VEDA_CHAINS_VECTOR)
    assert plan.chain_unit() == veda.VEDA_CHAINS_VECTOR
    plan.set_option(veda.VEDA_OPT_FP32_CHAIN_UNIT, 0)
    assert plan.chain_unit() == veda.VEDA_CHAINS_MATRIX
    with pytest.raises(RuntimeError):
        plan.set_option(veda.VEDA_OPT_FP32_CHAIN_UNIT, 3)


def test_projection_chains_of_odd_length_keep_signed_zeros():
    """Hidden width 5: the second layer's chains have an odd number of terms, so the last matrix-core
    instruction of each chain carries a padding term, which must leave a -0 accumulator as -0
    (bias -0, every product 1 * -0): the latents are -0 in the oracle and on the GPU."""
    wl = wlm.custom_workload("negzero", 1, 64, "f32", (4, 8, 8), False, (1, 2), seed=5, latent_dim=4)
    dev = torch.device("cuda:0")
    shapes = wlm.tile_shapes(wl)
    q, k, _ = wlm.make_qkv(wl, dev)
    plan = veda.Plan(wl.batch, wl.heads, wl.head_dim, wl.grid, shapes, wl.torch_dtype)
    qt, vm, _ = veda.veda_tile_layout(plan, q, veda.VEDA_TOKEN_MAJOR)
    kt, _, _ = veda.veda_tile_layout(plan, k, veda.VEDA_TOKEN_MAJOR, want_mask=False)
    w1 = np.zeros((1, 192, 5), np.float32)
    b1 = np.ones((1, 5), np.float32)
    w2 = np.full((1, 5, 4), -0.0, np.float32)
    b2 = np.full((1, 4), -0.0, np.float32)
    z = vo.trippool(hz.to_f32_numpy(q[0, 0]), wl.grid, (4, 4, 4))
    want = vo.mlp(z, w1[0], b1[0], w2[0], b2[0], True)
    assert np.all(want.view(np.uint32) == 0x80000000)
    phi = veda.Mlp(w1, b1, w2, b2, True, dev)
    _, ws = veda.veda_tile_score(plan, qt, kt, vm, phi, phi, 0.5)
    torch.cuda.synchronize()
    _, _, yq, yk = hz.score_intermediates(plan, phi, phi, ws)
    assert np.all(yq.cpu().numpy().view(np.uint32) == 0x80000000)
    assert np.all(yk.cpu().numpy().view(np.uint32) == 0x80000000)


def test_projection_and_score_chains_in_the_denormal_range():
    """Weights of magnitude 2^-136 (denormal themselves): every product and partial sum of the projection
    chains is a denormal number, and so are the latents; the scores underflow.  Nothing may be flushed to
    zero on the way: latents and scores have the oracle's bits (two layers and a single one)."""
    wl = wlm.custom_workload("denormal", 1, 64, "f32", (4, 8, 8), False, (1, 2), seed=6, latent_dim=8)
    dev = torch.device("cuda:0")
    shapes = wlm.tile_shapes(wl)
    q, k, _ = wlm.make_qkv(wl, dev)
    plan = veda.Plan(wl.batch, wl.heads, wl.head_dim, wl.grid, shapes, wl.torch_dtype)
    qt, vm, _ = veda.veda_tile_layout(plan, q, veda.VEDA_TOKEN_MAJOR)
    kt, _, _ = veda.veda_tile_layout(plan, k, veda.VEDA_TOKEN_MAJOR, want_mask=False)
    rng = np.random.default_rng(8)
    tiny = np.float32(2.0 ** -136)
    rows, d, dp = plan.total_tiles, 64, 8
    zq = vo.trippool(hz.to_f32_numpy(q[0, 0]), wl.grid, (4, 4, 4))
    zk = vo.trippool(hz.to_f32_numpy(k[0, 0]), wl.grid, (4, 4, 4))
    for hidden in (0, 12):
        first = hidden if hidden else dp
        w1 = (rng.uniform(-1, 1, (1, 3 * d, first)).astype(np.float32) * (tiny if not hidden else np.float32(1.0)))
        b1 = np.zeros((1, first), np.float32)
        w2 = rng.uniform(-1, 1, (1, hidden, dp)).astype(np.float32) * tiny if hidden else None
        b2 = rng.uniform(-1, 1, (1, dp)).astype(np.float32) * tiny if hidden else None
        args = (w1[0], b1[0], None if w2 is None else w2[0], None if b2 is None else b2[0], False)
        want_q, want_k = vo.mlp(zq, *args), vo.mlp(zk, *args)
        assert np.all(np.abs(want_q[want_q != 0]) < 1.1754944e-38) and np.count_nonzero(want_q) > want_q.size // 2
        phi = veda.Mlp(w1, b1, w2, b2, False, dev)
        s, ws = veda.veda_tile_score(plan, qt, kt, vm, phi, phi, 1.0)
        torch.cuda.synchronize()
        _, _, yq_g, yk_g = hz.score_intermediates(plan, phi, phi, ws)
        assert np.array_equal(yq_g.cpu().numpy().view(np.uint32), want_q.view(np.uint32)), hidden
        assert np.array_equal(yk_g.cpu().numpy().view(np.uint32), want_k.view(np.uint32)), hidden
        ref = vo.score(want_q, want_k, np.float32(1.0))
        assert np.array_equal(s[0].view(rows, rows).cpu().numpy().view(np.uint32), ref.view(np.uint32)), hidden
    # scores in the denormal range too: latents of magnitude 2^-68 give products near 2^-136
    w1 = rng.uniform(-1, 1, (1, 3 * d, dp)).astype(np.float32) * np.float32(2.0 ** -72)
    b1 = np.zeros((1, dp), np.float32)
    yq, yk = vo.mlp(zq, w1[0], b1[0], None, None, False), vo.mlp(zk, w1[0], b1[0], None, None, False)
    ref = vo.score(yq, yk, np.float32(1.0))
    assert np.count_nonzero(ref) > ref.size // 2 and np.all(np.abs(ref) < 1.1754944e-38)
    phi = veda.Mlp(w1, b1, None, None, False, dev)
    s, _ = veda.veda_tile_score(plan, qt, kt, vm, phi, phi, 1.0)
    torch.cuda.synchronize()
    assert np.array_equal(s[0].view(rows, rows).cpu().numpy().view(np.uint32), ref.view(np.uint32))


def test_zero_sparsity_equals_dense_attention_on_gpu():
    wl = wlm.custom_workload("dense_identity", 3, 128, "bf16", (6, 9, 11), True, (1, 1), seed=13)
    run = hz.run_gpu_path(wl)
    assert list(run.k_per_head) == run.plan.tiles
    for h in range(wl.heads):
        qf, kf, vf = (hz.to_f32_numpy(t[0, h]) for t in (run.q, run.k, run.v))
        ref = vo.dense_attention(qf, kf, vf, run.softmax_scale, np.arange(wl.tokens))
        err = np.abs(hz.to_f32_numpy(run.out[0, h]).astype(np.float64) - ref)
        _say(f"[dense-identity] head {h} {tuple(run.shapes[h])}: max {err.max():.3e} mean {err.mean():.3e}")
        assert err.max() <= hz.BF16_MAX_ABS and err.mean() <= hz.BF16_MEAN_ABS


def test_row_stochastic_weights_on_gpu():
    # V == 1 everywhere: any convex combination of value rows is exactly 1 (bf16 can hold it)
    wl = wlm.custom_workload("ones", 3, 128, "bf16", (6, 9, 11), True, (40, 100), seed=14)
    run = hz.run_gpu_path(wl)
    vt, _, _ = veda.veda_tile_layout(run.plan, torch.ones_like(run.v), veda.VEDA_CHANNEL_MAJOR, want_mask=False)
    out, _ = veda.veda_sparse_attn_fwd(run.plan, run.bufs["qt"], run.bufs["kt"], vt, run.bufs["vm"],
                                       run.bufs["rp"], run.bufs["ci"], run.softmax_scale)
    torch.cuda.synchronize()
    assert (out.float() - 1.0).abs().max().item() <= 2 ** -7


@pytest.mark.parametrize("dtype,d,walk", [("bf16", 128, False), ("bf16", 64, False), ("f32", 64, False),
                                          ("bf16", 128, True), ("bf16", 64, True), ("f32", 64, True)])
def test_attention_on_hand_made_lists(dtype, d, walk):
    # Stage 4 alone on kept lists that stage 3 would never write: unsorted, neighbours with
    # identical / disjoint / partly shared lists.  The grid gives every head an odd tile count
    # (the last query tile has no neighbour) and ragged tiles on every axis.  walk: the kernel
    # merging the lists inside its loop (VEDA_OPT_ATTN_LIST_WALK) instead of from its step table.
    _hand_made_lists(dtype, d, 1.0, 1.0, walk=walk)


def test_attention_with_large_logits_fp32():
    # Queries six times larger: logits spread over +-40 in log2 units, so the running softmax
    # reference moves on many steps and a stale one would overflow or flush rows to zero.
    _hand_made_lists("f32", 64, 6.0, 4.0)


def test_bf16_attention_error_against_logit_size():
    """Sweep of the query gain on the hand-made lists (logits q.k/sqrt(d) of standard deviation = gain).
    Default kernel: the pre-scaled queries are rounded to bf16 once, an error of 2^-9 of every logit, so the
    output error grows with the gain: the target's bars (max-abs 2e-2, mean-abs 2e-3) hold up to gain 2 and the
    measured growth stays inside the envelope the header documents.  With VEDA_OPT_EXACT_LOGIT_SCALE the
    bars hold at every gain, 6 (the large-logit case) and 16 included."""
    envelope = {1.0: (1e-2, 1e-3, 1e-2), 2.0: (2e-2, 2e-3, 2e-2), 4.0: (4e-2, 3e-3, 5e-2), 6.0: (8e-2, 4e-3, 1e-1),
                8.0: (1e-1, 4e-3, 1e-1)}
    for gain, (mx, mean, lse) in envelope.items():
        st = _hand_made_lists("bf16", 128, gain, 1.0, check=False)
        got = (max(s[0] for s in st), max(s[1] for s in st), max(s[2] for s in st))
        _say(f"[parity] default scale, gain {gain}: max_abs {got[0]:.2e} mean_abs {got[1]:.2e} lse {got[2]:.2e}")
        assert got[0] <= mx and got[1] <= mean and got[2] <= lse, (gain, got)
    for gain in (1.0, 2.0, 4.0, 6.0, 8.0, 16.0):
        st = _hand_made_lists("bf16", 128, gain, 1.0, check=True, exact_scale=True)
        got = (max(s[0] for s in st), max(s[1] for s in st), max(s[2] for s in st))
        _say(f"[parity] exact logit scale, gain {gain}: max_abs {got[0]:.2e} mean_abs {got[1]:.2e} lse {got[2]:.2e}")
    st = _hand_made_lists("bf16", 64, 6.0, 1.0, check=True, exact_scale=True)   # d = 64: residual factor 1.44


def _hand_made_lists(dtype, d, q_gain, tol_gain, check=True, exact_scale=False, walk=False):
    wl = wlm.custom_workload(f"lists_{dtype}_{d}", 3, d, dtype, (9, 18, 18), True, (25, 100), seed=31)
    dev = torch.device("cuda:0")
    shapes = wlm.tile_shapes(wl)
    q, k, v = wlm.make_qkv(wl, dev)
    q = (q.float() * q_gain).to(q.dtype)
    plan = veda.Plan(wl.batch, wl.heads, wl.head_dim, wl.grid, shapes, wl.torch_dtype)
    if exact_scale:
        plan.set_option(veda.VEDA_OPT_EXACT_LOGIT_SCALE, 1)
    if walk:
        plan.set_option(veda.VEDA_OPT_ATTN_LIST_WALK, 1)
    assert all(n % 2 for n in plan.tiles)
    qt, vm, _ = veda.veda_tile_layout(plan, q, veda.VEDA_TOKEN_MAJOR)
    kt, _, _ = veda.veda_tile_layout(plan, k, veda.VEDA_TOKEN_MAJOR, want_mask=False)
    vt, _, _ = veda.veda_tile_layout(plan, v, veda.VEDA_CHANNEL_MAJOR, want_mask=False)
    rng = np.random.default_rng(31)
    ksel = 7
    sels, cols = [], []
    for h in range(wl.heads):
        n = plan.tiles[h]
        sel = np.stack([rng.choice(n, ksel, replace=False) for _ in range(n)]).astype(np.int32)   # unsorted
        for i in range(0, n - 1, 2):
            kind = (i // 2) % 4
            if kind == 0:
                sel[i + 1] = sel[i][::-1]                                   # same tiles, other order
            elif kind == 1:
                rest = np.setdiff1d(np.arange(n), sel[i])
                sel[i + 1] = rng.choice(rest, ksel, replace=False)          # nothing shared
            elif kind == 2:
                sel[i], sel[i + 1] = np.sort(sel[i]), np.sort(sel[i + 1])   # ascending, as stage 3 writes
        sels.append(sel)
        cols.append(sel.reshape(-1))
    col_idx = torch.as_tensor(np.concatenate(cols)).to(dev)
    row_ptr = torch.arange(plan.total_tiles + 1, dtype=torch.int32, device=dev) * ksel
    scale = 1.0 / math.sqrt(d)
    out = torch.full((1, wl.heads, wl.tokens, d), float("nan"), dtype=wl.torch_dtype, device=dev)
    out, lse = veda.veda_sparse_attn_fwd(plan, qt, kt, vt, vm, row_ptr, col_idx, scale, out=out, want_lse=True)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    queries = np.arange(wl.tokens)
    stats = []
    for h in range(wl.heads):
        shape = tuple(int(x) for x in shapes[h])
        ref, lse_ref, _ = vo.masked_attention(hz.to_f32_numpy(q[0, h]), hz.to_f32_numpy(k[0, h]),
                                              hz.to_f32_numpy(v[0, h]), wl.grid, shape, sels[h], scale, queries,
                                              want_stats=True)
        err = np.abs(hz.to_f32_numpy(out[0, h]).astype(np.float64) - ref)
        lerr = np.abs(lse[0, h].cpu().numpy().astype(np.float64) - lse_ref)
        _say(f"[parity] {wl.name} gain {q_gain} head {h} {shape}: max_abs {err.max():.2e} mean_abs {err.mean():.2e} "
             f"lse {lerr.max():.2e} (lse spread {lse_ref.max() - lse_ref.min():.1f})")
        stats.append((float(err.max()), float(err.mean()), float(lerr.max())))
        if not check:
            continue
        if dtype == "bf16":
            assert err.max() <= tol_gain * hz.BF16_MAX_ABS and err.mean() <= tol_gain * hz.BF16_MEAN_ABS
            assert lerr.max() <= tol_gain * 2e-2
        else:
            assert err.max() <= tol_gain * hz.F32_MAX_ABS and lerr.max() <= tol_gain * 1e-4
    return stats


def test_a_head_too_long_for_the_step_table():
    """1,049,600 tokens in one head = 17,600 tiles of 4x4x4, more than the 16,384 the bf16 attention kernel's
    step table covers: the kernel then merges the kept lists inside its loop.  Hand-made ascending lists (the
    tile itself, its successor, four drawn ones); sampled query tiles (first, last, ragged ones) against the
    oracle."""
    wl = wlm.custom_workload("long_head", 1, 64, "bf16", (41, 160, 160), False, (1, 100), seed=44)
    dev = torch.device("cuda:0")
    shapes = wlm.tile_shapes(wl)
    shape = tuple(int(x) for x in shapes[0])
    q, k, v = wlm.make_qkv(wl, dev)
    plan = veda.Plan(wl.batch, wl.heads, wl.head_dim, wl.grid, shapes, wl.torch_dtype)
    n = plan.tiles[0]
    assert n == 17600
    rng = np.random.default_rng(44)
    ksel = 6
    sel = np.empty((n, ksel), np.int32)
    sel[:, 0] = np.arange(n)
    sel[:, 1] = (np.arange(n) + 1) % n
    sel[:, 2:] = rng.integers(0, n, (n, ksel - 2))
    for i in range(n):   # no tile twice in a row: redraw the few duplicates
        while len(set(sel[i])) < ksel:
            sel[i, 2:] = rng.integers(0, n, ksel - 2)
    sel.sort(axis=1)
    col_idx = torch.as_tensor(sel.reshape(-1)).to(dev)
    row_ptr = torch.arange(n + 1, dtype=torch.int32, device=dev) * ksel
    _, vm, _, _ = veda.veda_tile_layout_stats(plan, q, want_tiles=False)
    vt, _, _ = veda.veda_tile_layout(plan, v, veda.VEDA_CHANNEL_MAJOR, want_mask=False)
    scale = 1.0 / math.sqrt(wl.head_dim)
    out = torch.full((1, 1, wl.tokens, wl.head_dim), float("nan"), dtype=wl.torch_dtype, device=dev)
    out, lse = veda.veda_sparse_attn_fwd(plan, None, None, vt, vm, row_ptr, col_idx, scale, out=out, want_lse=True,
                                         q_tokens=q, k_tokens=k)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    T, H, W = wl.grid
    tiles = [0, 1, n // 2, n - 2, n - 1] + [int(x) for x in rng.integers(0, n, 3)]
    nh, nw = -(-H // shape[1]), -(-W // shape[2])
    queries = []
    for i in tiles:
        tt, th, tw = i // (nh * nw), (i // nw) % nh, i % nw
        for lt in range(shape[0]):
            for lh in range(shape[1]):
                for lw in range(shape[2]):
                    t, h, w = tt * shape[0] + lt, th * shape[1] + lh, tw * shape[2] + lw
                    if t < T and h < H and w < W:
                        queries.append((t * H + h) * W + w)
    queries = np.asarray(sorted(queries))
    ref, lse_ref, _ = vo.masked_attention(hz.to_f32_numpy(q[0, 0]), hz.to_f32_numpy(k[0, 0]), hz.to_f32_numpy(v[0, 0]),
                                          wl.grid, shape, sel, scale, queries, want_stats=True)
    got = hz.to_f32_numpy(out[0, 0][torch.as_tensor(queries, device=dev)]).astype(np.float64)
    err = np.abs(got - ref)
    lerr = np.abs(lse[0, 0][torch.as_tensor(queries, device=dev)].cpu().numpy().astype(np.float64) - lse_ref)
    _say(f"[parity] {wl.name}: {len(queries)} sampled queries of {n} tiles: max_abs {err.max():.2e} mean_abs {err.mean():.2e} "
         f"lse {lerr.max():.2e}")
    assert err.max() <= hz.BF16_MAX_ABS and err.mean() <= hz.BF16_MEAN_ABS and lerr.max() <= 2e-2


def test_maximum_head_count():
    # 128 heads (the library's limit) on a small ragged grid: per-head tables, the die-aware work
    # split and the 64-tile projection blocks all see many short heads
    wl = wlm.custom_workload("heads128", 128, 64, "bf16", (5, 6, 10), True, (50, 100), seed=41, latent_dim=16)
    run = hz.run_gpu_path(wl)
    assert torch.isfinite(run.out.float()).all()
    for h in (0, 1, 63, 126, 127):
        st = hz.check_head(run, h)
        _say(f"[parity] {wl.name} h{h} {tuple(run.shapes[h])}: {st}")
    with pytest.raises(veda.VedaError):
        veda.Plan(1, 129, 64, wl.grid, np.tile(np.asarray([[4, 4, 4]], np.int32), (129, 1)), torch.bfloat16)


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("f32", 64), ("f32", 128)])
def test_descriptors_during_gather_are_bit_identical(dtype, d):
    # veda_tile_layout_stats + veda_tile_score_stats against veda_tile_layout + veda_tile_score:
    # same tiled bytes, masks, descriptors (also checked against the oracle) and scores
    wl = wlm.custom_workload(f"fused_{dtype}_{d}", 5, d, dtype, (9, 10, 14), True, (25, 100), seed=51, batch=2,
                             latent_dim=32)
    dev = torch.device("cuda:0")
    shapes = wlm.tile_shapes(wl)
    q, k, _ = wlm.make_qkv(wl, dev)
    plan = veda.Plan(wl.batch, wl.heads, wl.head_dim, wl.grid, shapes, wl.torch_dtype)
    eq, ek = wlm.make_estimator(wl, "q"), wlm.make_estimator(wl, "k")
    pq = veda.Mlp(eq.w1, eq.b1, eq.w2, eq.b2, eq.relu, dev)
    pk = veda.Mlp(ek.w1, ek.b1, ek.w2, ek.b2, ek.relu, dev)
    scale = hz.score_scale_of(wl)
    qt, vm, vc = veda.veda_tile_layout(plan, q, veda.VEDA_TOKEN_MAJOR)
    kt, _, _ = veda.veda_tile_layout(plan, k, veda.VEDA_TOKEN_MAJOR, want_mask=False)
    s_ref, _ = veda.veda_tile_score(plan, qt, kt, vm, pq, pk, scale)
    qt2, vm2, vc2, zq = veda.veda_tile_layout_stats(plan, q)
    kt2, _, _, zk = veda.veda_tile_layout_stats(plan, k, want_mask=False)
    s2, _ = veda.veda_tile_score_stats(plan, zq, zk, pq, pk, scale)
    torch.cuda.synchronize()
    view = torch.int16 if dtype == "bf16" else torch.int32
    assert torch.equal(qt.view(view), qt2.view(view)) and torch.equal(kt.view(view), kt2.view(view))
    assert torch.equal(vm, vm2) and torch.equal(vc, vc2)
    assert torch.equal(s_ref.view(torch.int32), s2.view(torch.int32))
    for b in range(wl.batch):
        for h in range(wl.heads):
            shape = tuple(int(x) for x in shapes[h])
            nt, toff = plan.tiles[h], plan.tile_offset[h]
            for x, z in ((q, zq), (k, zk)):
                ref = vo.trippool(hz.to_f32_numpy(x[b, h]), wl.grid, shape)
                got = z[b, toff:toff + nt].cpu().numpy()
                assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), (b, h)


def test_select_on_constructed_ties_and_special_values():
    wl = wlm.custom_workload("ties", 2, 64, "f32", (4, 8, 40), False, (1, 4), seed=15, latent_dim=32)
    shapes = wlm.tile_shapes(wl)
    plan = veda.Plan(1, wl.heads, wl.head_dim, wl.grid, shapes, wl.torch_dtype)
    nt = plan.tiles[0]
    rng = np.random.default_rng(15)
    s = rng.integers(-2, 3, size=(wl.heads, nt, nt)).astype(np.float32)     # five levels: many ties
    s[0, 0, :5] = [np.nan, -0.0, 0.0, np.inf, -np.inf]
    s[1, 1, :] = 1.0                                                          # a fully tied row
    for k in (1, 3, nt // 2, nt):
        rp, ci = veda.veda_tile_select(plan, torch.as_tensor(s).reshape(1, -1).cuda(), [k] * wl.heads)
        torch.cuda.synchronize()
        got = ci.cpu().numpy().reshape(wl.heads, nt, k)
        for h in range(wl.heads):
            assert np.array_equal(got[h], vo.select(s[h], k)), (h, k)
        assert np.array_equal(rp.cpu().numpy(), np.arange(wl.heads * nt + 1) * k)


def test_select_long_rows_use_every_instantiation():
    # row lengths that land in the 4-, 16-, 32-, 64-item and the memory-resident kernels
    for grid in [(1, 8, 64), (32, 32, 64), (64, 32, 64), (128, 32, 64), (136, 32, 64)]:
        shapes = np.asarray([[1, 8, 8]], np.int32)
        plan = veda.Plan(1, 1, 64, grid, shapes, torch.float32)
        nt = plan.tiles[0]
        rows = min(nt, 48)
        s = np.random.default_rng(nt).standard_normal((nt, nt)).astype(np.float32)
        s[rows:] = 0.0
        # 5 % kept: rows of 1024 tiles and more take the sampled-pivot kernel; 50 % kept: the
        # register-resident (or memory-resident) full search
        for k in (max(1, nt // 20), nt // 2):
            _say(f"[parity] select grid {grid}: {nt} tiles, k {k}")
            rp, ci = veda.veda_tile_select(plan, torch.as_tensor(s).reshape(1, -1).cuda(), [k])
            torch.cuda.synchronize()
            got = ci.cpu().numpy().reshape(nt, k)
            assert np.array_equal(got[:rows], vo.select(s[:rows], k)), (grid, k)
            assert np.array_equal(got[rows:], np.tile(np.arange(k), (nt - rows, 1))), (grid, k)


def test_select_sampled_pivot_paths():
    # 2048-tile rows at 5 % kept go through the sampled-pivot kernel.  Rows are built so that the
    # candidate list comes out well sized, too short (large values only where the sample looks),
    # too long (mass ties at the threshold), and with NaN / infinities / signed zeros in it.
    shapes = np.asarray([[1, 8, 8]], np.int32)
    plan = veda.Plan(1, 1, 64, (64, 32, 64), shapes, torch.float32)
    nt = plan.tiles[0]
    assert nt == 2048
    rng = np.random.default_rng(5)
    s = np.zeros((nt, nt), np.float32)
    rows = 40
    s[:8] = rng.standard_normal((8, nt))
    s[8:12] = rng.integers(-3, 4, size=(4, nt))                       # 7 levels: long tie runs
    s[12:16] = rng.standard_normal((4, nt))
    s[12:16, ::8] += 10.0                                             # the 256 sampled columns are the large ones
    s[16:20] = rng.standard_normal((4, nt))
    s[16:20, rng.integers(0, nt, 300)] = np.inf
    s[20:24] = rng.standard_normal((4, nt))
    s[20:24, rng.integers(0, nt, 1900)] = np.nan
    s[24:28] = np.where(rng.random((4, nt)) < 0.5, -0.0, 0.0)
    s[28:32] = -np.inf
    s[28:32, rng.integers(0, nt, 50)] = 1.0
    s[32:36] = rng.standard_normal((4, nt)).astype(np.float32) * 1e-30   # tiny values near the zero keys
    s[36:40] = -np.abs(rng.standard_normal((4, nt)))                  # all negative
    for k in (1, 64, 102, 180):
        _say(f"[parity] sampled select: k {k}")
        rp, ci = veda.veda_tile_select(plan, torch.as_tensor(s).reshape(1, -1).cuda(), [k])
        torch.cuda.synchronize()
        got = ci.cpu().numpy().reshape(nt, k)
        ref = vo.select(s[:rows], k)
        for r in range(rows):
            assert np.array_equal(got[r], ref[r]), (k, r)


def _lists_of(plan, stats_q, stats_k, pq, pk, sscale, kph):
    """(row_ptr, col_idx) by the two-stage route and by the one-call route, from descriptors."""
    s, _ = veda.veda_tile_score_stats(plan, stats_q, stats_k, pq, pk, sscale)
    rp, ci = veda.veda_tile_select(plan, s, kph)
    rp2, ci2, _ = veda.veda_tile_score_select(plan, pq, pk, sscale, kph, stats_q=stats_q, stats_k=stats_k)
    torch.cuda.synchronize()
    return (rp, ci), (rp2, ci2)


def test_score_select_in_one_call_long_rows():
    # rows of 1260 - 1840 tiles at a 5 % budget: every score is compared with its row's pivot as it
    # is formed and never written.  Lists must equal the two-stage route's (which the other tests
    # hold against the oracle), from tiles and from descriptors; one head is checked against the
    # oracle directly as well.
    wl = wlm.custom_workload("one_call", 3, 128, "bf16", (21, 45, 80), True, (5, 100), seed=3)
    run = hz.run_gpu_path(wl)
    dev = torch.device("cuda:0")
    plan, kph = run.plan, run.k_per_head
    assert min(plan.tiles) >= 1024
    pq = veda.Mlp(run.phi_q.w1, run.phi_q.b1, run.phi_q.w2, run.phi_q.b2, run.phi_q.relu, dev)
    pk = veda.Mlp(run.phi_k.w1, run.phi_k.b1, run.phi_k.w2, run.phi_k.b2, run.phi_k.relu, dev)
    rp, ci, _ = veda.veda_tile_score_select(plan, pq, pk, run.score_scale, kph, q_tiled=run.bufs["qt"],
                                            k_tiled=run.bufs["kt"], valid_mask=run.bufs["vm"])
    torch.cuda.synchronize()
    assert torch.equal(rp, run.bufs["rp"]) and torch.equal(ci, run.bufs["ci"])
    _, _, _, zq = veda.veda_tile_layout_stats(plan, run.q)
    _, _, _, zk = veda.veda_tile_layout_stats(plan, run.k, want_mask=False)
    two, one = _lists_of(plan, zq, zk, pq, pk, run.score_scale, kph)
    assert torch.equal(two[0], run.bufs["rp"]) and torch.equal(two[1], run.bufs["ci"])
    assert torch.equal(one[0], run.bufs["rp"]) and torch.equal(one[1], run.bufs["ci"])
    st = hz.check_head(run, 0, attn_tiles=4)
    _say(f"[parity] {wl.name} head 0: lists equal on both routes and to the oracle; attention {st}")


@pytest.mark.parametrize("unit", [0, 2])
def test_score_select_in_one_call_ties_nan_and_redone_rows(unit):
    # Descriptors doctored against the candidate lists.  Head 0: every key tile is a copy of tile B
    # except 30 of the sampled columns, which are copies of tile A.  For a row that scores A above B
    # the pivot is A's score and only 30 < k candidates exist; for the other rows the pivot is B's
    # score and all 1152 > 1024 tiles pass: every row of the head is redone on its full score row,
    # all of it ties.  Head 1: key tiles are copies of six prototypes (whole runs of equal scores
    # around the k-th place, inside the candidate lists) and 40 of them hold NaN (rank as -inf).
    # Lists must equal the two-stage route's.
    wl = wlm.custom_workload("one_call_ties", 2, 64, "bf16", (16, 64, 72), False, (5, 100), seed=4, latent_dim=32)
    dev = torch.device("cuda:0")
    shapes = wlm.tile_shapes(wl)
    q, k, _ = wlm.make_qkv(wl, dev)
    plan = veda.Plan(wl.batch, wl.heads, wl.head_dim, wl.grid, shapes, wl.torch_dtype)
    if unit:   # projections and the redone score rows as scalar fmaf chains on the vector units
        plan.set_option(veda.VEDA_OPT_FP32_CHAIN_UNIT, unit)
    n = plan.tiles[0]
    assert n == 1152 and plan.tiles[1] == n
    kph = wlm.keep_budget(wl, None, shapes)
    assert int(kph[0]) == 58
    eq, ek = wlm.make_estimator(wl, "q"), wlm.make_estimator(wl, "k")
    pq = veda.Mlp(eq.w1, eq.b1, eq.w2, eq.b2, eq.relu, dev)
    pk = veda.Mlp(ek.w1, ek.b1, ek.w2, ek.b2, ek.relu, dev)
    _, _, _, zq = veda.veda_tile_layout_stats(plan, q)
    _, _, _, zk = veda.veda_tile_layout_stats(plan, k, want_mask=False)
    tile_a, tile_b = zk[0, 7].clone(), zk[0, 500].clone()
    zk[0, :n] = tile_b
    sampled = torch.as_tensor([(s * n) // 256 for s in range(30)], device=dev)
    zk[0, sampled] = tile_a
    g = torch.Generator(device="cpu").manual_seed(5)
    proto = torch.randint(0, 6, (n,), generator=g).to(dev)
    zk[0, n:2 * n] = zk[0, n:n + 6][proto]
    nan_at = torch.randperm(n, generator=g)[:40].to(dev) + n
    zk[0, nan_at, 0] = float("nan")
    sscale = hz.score_scale_of(wl)
    two, one = _lists_of(plan, zq, zk, pq, pk, sscale, kph)
    assert torch.equal(one[0], two[0]) and torch.equal(one[1], two[1])
    # the two-stage lists themselves against the oracle's selection on the same scores
    s, _ = veda.veda_tile_score_stats(plan, zq, zk, pq, pk, sscale)
    ksel = int(kph[0])
    for h in (0, 1):
        rows = s[0, h * n * n:(h + 1) * n * n].view(n, n)[[0, 1, n // 2, n - 1]].cpu().numpy()
        want = vo.select(rows, ksel)
        got = two[1][h * n * ksel:(h + 1) * n * ksel].view(n, ksel)[[0, 1, n // 2, n - 1]].cpu().numpy()
        assert np.array_equal(got, want), h
    a_first = (s[0, :n * n].view(n, n)[:, sampled[0]] > s[0, :n * n].view(n, n)[:, 1]).sum().item()
    _say(f"[parity] {wl.name}: head 0 redone in full ({a_first} rows short of candidates, {n - a_first} with too many)")


def test_score_select_in_one_call_other_shapes():
    # short rows, a large budget, 128-token tiles and a long latent: the call takes the two-stage
    # route inside and must give the same lists
    for tile_tokens, dp, keep in ((64, 64, (25, 100)), (128, 32, (25, 100)), (64, 128, (50, 100))):
        if tile_tokens == 64:
            wl = wlm.custom_workload("one_call_small", 3, 64, "bf16", (9, 18, 18), True, keep, seed=6, latent_dim=dp)
            shapes = wlm.tile_shapes(wl)
        else:
            shapes = np.asarray([(8, 4, 4), (2, 8, 8), (1, 8, 16)], np.int32)
            wl = wlm.custom_workload("one_call_128", 3, 64, "bf16", (9, 18, 18), True, keep, seed=6, latent_dim=dp)
        dev = torch.device("cuda:0")
        q, k, _ = wlm.make_qkv(wl, dev)
        plan = veda.Plan(wl.batch, wl.heads, wl.head_dim, wl.grid, shapes, wl.torch_dtype, tile_tokens=tile_tokens)
        kph = np.asarray([max(1, -(-n * keep[0] // keep[1])) for n in plan.tiles], np.int32)
        eq, ek = wlm.make_estimator(wl, "q"), wlm.make_estimator(wl, "k")
        pq = veda.Mlp(eq.w1, eq.b1, eq.w2, eq.b2, eq.relu, dev)
        pk = veda.Mlp(ek.w1, ek.b1, ek.w2, ek.b2, ek.relu, dev)
        qt, vm, _ = veda.veda_tile_layout(plan, q, veda.VEDA_TOKEN_MAJOR)
        kt, _, _ = veda.veda_tile_layout(plan, k, veda.VEDA_TOKEN_MAJOR, want_mask=False)
        sscale = hz.score_scale_of(wl)
        s, _ = veda.veda_tile_score(plan, qt, kt, vm, pq, pk, sscale)
        rp, ci = veda.veda_tile_select(plan, s, kph)
        rp2, ci2, ws = veda.veda_tile_score_select(plan, pq, pk, sscale, kph, q_tiled=qt, k_tiled=kt, valid_mask=vm)
        torch.cuda.synchronize()
        assert torch.equal(rp, rp2) and torch.equal(ci, ci2), (tile_tokens, dp)
        with pytest.raises(veda.VedaError) as e:
            veda.veda_tile_score_select(plan, pq, pk, sscale, kph, q_tiled=qt, k_tiled=kt, valid_mask=vm,
                                        workspace=ws[: ws.numel() // 2])
        assert e.value.status == veda.VEDA_ERR_WORKSPACE


@pytest.mark.parametrize("tile_tokens", [64, 128])
def test_whole_path_wrapper_routes_agree(tile_tokens):
    # veda_attention in its six routes (descriptors from the gather or not, stages 2+3 in one call
    # or two, Q and K tiled or read from token order): same lists, same output bits; buffers of a
    # first call are reused by a second.  With 128-token tiles the ragged grid leaves half tiles
    # without a single real token (8x4x4 on 9 frames, 1x8x16 on 18 columns).
    wl = wlm.custom_workload("routes", 3, 128, "bf16", (9, 18, 18), True, (25, 100), seed=12)
    dev = torch.device("cuda:0")
    shapes = wlm.tile_shapes(wl) if tile_tokens == 64 else np.asarray([(8, 4, 4), (2, 8, 8), (1, 8, 16)], np.int32)
    q, k, v = wlm.make_qkv(wl, dev)
    plan = veda.Plan(wl.batch, wl.heads, wl.head_dim, wl.grid, shapes, wl.torch_dtype, tile_tokens=tile_tokens)
    kph = wlm.keep_budget(wl, None, shapes)
    eq, ek = wlm.make_estimator(wl, "q"), wlm.make_estimator(wl, "k")
    pq = veda.Mlp(eq.w1, eq.b1, eq.w2, eq.b2, eq.relu, dev)
    pk = veda.Mlp(ek.w1, ek.b1, ek.w2, ek.b2, ek.relu, dev)
    outs = []
    for fused, one_call, from_tokens in ((False, False, False), (False, True, False), (True, False, False),
                                         (True, True, False), (True, False, True), (True, True, True)):
        out, bufs = veda.veda_attention(plan, q, k, v, pq, pk, kph, hz.score_scale_of(wl), 1.0 / math.sqrt(128),
                                        fused=fused, one_call=one_call, from_tokens=from_tokens)
        assert (bufs["qt"] is None and bufs["kt"] is None) == from_tokens
        first = out.clone()
        out2, _ = veda.veda_attention(plan, q, k, v, pq, pk, kph, hz.score_scale_of(wl), 1.0 / math.sqrt(128),
                                      buffers=bufs, fused=fused, one_call=one_call, from_tokens=from_tokens)
        torch.cuda.synchronize()
        assert out2.data_ptr() == out.data_ptr() and torch.equal(out2.view(torch.int16), first.view(torch.int16))
        outs.append((out2.view(torch.int16).clone(), bufs["ci"].clone(), bufs["vm"].clone(), bufs["vc"].clone(),
                     None if bufs.get("zq") is None or not fused else bufs["zq"].view(torch.int32).clone()))
    for o, ci, vm, vc, _ in outs[1:]:
        assert torch.equal(o, outs[0][0]) and torch.equal(ci, outs[0][1])
        assert torch.equal(vm, outs[0][2]) and torch.equal(vc, outs[0][3])     # masks and counts, from either gather
    # the descriptors of the gathers that write the tiles and of those that do not are the same bits
    assert torch.equal(outs[2][4], outs[4][4])
    # and they are the oracle's TripPool (Eq. 4) of every head
    zq = outs[2][4].view(torch.float32).cpu().numpy()
    for h in range(wl.heads):
        ref = vo.trippool(hz.to_f32_numpy(q[0, h]), wl.grid, tuple(int(x) for x in shapes[h]))
        got = zq[0, plan.tile_offset[h]:plan.tile_offset[h] + plan.tiles[h]]
        assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), (tile_tokens, h)


def test_whole_path_replayed_from_a_hip_graph():
    """The stage calls only enqueue kernels on the caller's stream, so one whole step can be captured into a
    HIP graph.  Replays with fresh inputs copied into the captured buffers, and unrelated eager work between
    them, must reproduce the eager results bit for bit every time."""
    wl = wlm.custom_workload("graph", 3, 128, "bf16", (9, 18, 18), True, (25, 100), seed=14)
    dev = torch.device("cuda:0")
    shapes = wlm.tile_shapes(wl)
    plan = veda.Plan(wl.batch, wl.heads, wl.head_dim, wl.grid, shapes, wl.torch_dtype)
    kph = wlm.keep_budget(wl, None, shapes)
    eq, ek = wlm.make_estimator(wl, "q"), wlm.make_estimator(wl, "k")
    pq = veda.Mlp(eq.w1, eq.b1, eq.w2, eq.b2, eq.relu, dev)
    pk = veda.Mlp(ek.w1, ek.b1, ek.w2, ek.b2, ek.relu, dev)
    args = (pq, pk, kph, hz.score_scale_of(wl), 1.0 / math.sqrt(128))
    kw = dict(fused=True, one_call=True, from_tokens=True)
    inputs = [wlm.make_qkv(wlm.custom_workload("graph", 3, 128, "bf16", (9, 18, 18), True, (25, 100), seed=14 + i), dev)
              for i in range(4)]
    q, k, v = (x.clone() for x in inputs[0])
    _, bufs = veda.veda_attention(plan, q, k, v, *args, **kw)        # allocates the step's buffers
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        veda.veda_attention(plan, q, k, v, *args, buffers=bufs, **kw)
    scratch = torch.zeros(1 << 20, device=dev)
    for rep, (qi, ki, vi) in enumerate(inputs[1:] + inputs[:1]):
        want, wb = veda.veda_attention(plan, qi, ki, vi, *args, **kw)   # eager, its own buffers
        want, want_ci = want.view(torch.int16).clone(), wb["ci"].clone()
        q.copy_(qi); k.copy_(ki); v.copy_(vi)
        scratch.add_(1.0).mul_(0.5)                                   # eager work between the replays
        bufs["out"].fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(bufs["ci"], want_ci), rep
        assert torch.equal(bufs["out"].view(torch.int16), want), rep


@pytest.mark.parametrize("d,tile_tokens", [(128, 64), (64, 64), (128, 128)])
def test_attention_with_q_in_token_order(d, tile_tokens):
    # the attention kernel gathering Q itself (no tiled copy of Q): same bits as with the tiled Q; and
    # the descriptors-only gather gives the same descriptors and masks as the full one
    if tile_tokens == 64:
        wl = wlm.custom_workload(f"qtok_{d}", 3, d, "bf16", (9, 18, 18), True, (25, 100), seed=14, batch=2)
        shapes = wlm.tile_shapes(wl)
    else:
        shapes = np.asarray([(8, 4, 4), (2, 8, 8), (1, 8, 16)], np.int32)
        wl = wlm.custom_workload(f"qtok128_{d}", 3, d, "bf16", (9, 18, 18), True, (25, 100), seed=14, batch=2)
    dev = torch.device("cuda:0")
    q, k, v = wlm.make_qkv(wl, dev)
    plan = veda.Plan(wl.batch, wl.heads, d, wl.grid, shapes, wl.torch_dtype, tile_tokens=tile_tokens)
    qt, vm, _ = veda.veda_tile_layout(plan, q, veda.VEDA_TOKEN_MAJOR)
    kt, _, _ = veda.veda_tile_layout(plan, k, veda.VEDA_TOKEN_MAJOR, want_mask=False)
    vt, _, _ = veda.veda_tile_layout(plan, v, veda.VEDA_CHANNEL_MAJOR, want_mask=False)
    rng = np.random.default_rng(14)
    kph = [max(1, n // 4) for n in plan.tiles]
    cols = [np.sort(rng.choice(n, kk, replace=False)) for _ in range(wl.batch) for n, kk in zip(plan.tiles, kph)
            for _ in range(n)]
    col_idx = torch.as_tensor(np.concatenate(cols).astype(np.int32)).to(dev)
    lens = np.concatenate([[kk] * n for _ in range(wl.batch) for n, kk in zip(plan.tiles, kph)])
    row_ptr = torch.as_tensor(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).to(dev)
    scale = 1.0 / math.sqrt(d)
    out1, lse1 = veda.veda_sparse_attn_fwd(plan, qt, kt, vt, vm, row_ptr, col_idx, scale, want_lse=True)
    # a strided view of Q: the gather must honour the strides
    qpad = torch.zeros((wl.batch, wl.heads, wl.tokens, d + 8), dtype=q.dtype, device=dev)
    qpad[..., :d] = q
    out2, lse2 = veda.veda_sparse_attn_fwd(plan, None, kt, vt, vm, row_ptr, col_idx, scale, want_lse=True,
                                           q_tokens=qpad[..., :d])
    # K from token order too, again through a strided view; the padded output starts as NaN so that a
    # real token left unwritten shows
    kpad = torch.zeros((wl.batch, wl.heads, wl.tokens, d + 8), dtype=k.dtype, device=dev)
    kpad[..., :d] = k
    out3 = torch.full_like(out1, float("nan"))
    out3, lse3 = veda.veda_sparse_attn_fwd(plan, None, None, vt, vm, row_ptr, col_idx, scale, out=out3, want_lse=True,
                                           q_tokens=qpad[..., :d], k_tokens=kpad[..., :d])
    torch.cuda.synchronize()
    assert torch.equal(out1.view(torch.int16), out2.view(torch.int16)) and torch.equal(lse1, lse2)
    assert torch.equal(out1.view(torch.int16), out3.view(torch.int16)) and torch.equal(lse1, lse3)
    # ascending rows: the lists merged inside the loop visit the key tiles in the step table's order
    plan.set_option(veda.VEDA_OPT_ATTN_LIST_WALK, 1)
    out4, lse4 = veda.veda_sparse_attn_fwd(plan, qt, kt, vt, vm, row_ptr, col_idx, scale, want_lse=True)
    out5 = torch.full_like(out1, float("nan"))
    out5, lse5 = veda.veda_sparse_attn_fwd(plan, None, None, vt, vm, row_ptr, col_idx, scale, out=out5, want_lse=True,
                                           q_tokens=qpad[..., :d], k_tokens=kpad[..., :d])
    plan.set_option(veda.VEDA_OPT_ATTN_LIST_WALK, 0)
    torch.cuda.synchronize()
    assert torch.equal(out1.view(torch.int16), out4.view(torch.int16)) and torch.equal(lse1, lse4)
    assert torch.equal(out1.view(torch.int16), out5.view(torch.int16)) and torch.equal(lse1, lse5)
    if tile_tokens == 64:
        _, vm_a, vc_a, z_a = veda.veda_tile_layout_stats(plan, q)
        none, vm_b, vc_b, z_b = veda.veda_tile_layout_stats(plan, q, want_tiles=False)
        torch.cuda.synchronize()
        assert none is None and torch.equal(vm_a, vm_b) and torch.equal(vc_a, vc_b)
        assert torch.equal(z_a.view(torch.int32), z_b.view(torch.int32)) and torch.equal(vm_a, vm)


def test_gpu_argument_errors_launch_nothing():
    wl = wlm.WORKLOADS["tiny"]
    run = hz.run_gpu_path(wl, want_lse=False)
    plan = run.plan
    with pytest.raises(veda.VedaError) as e:
        veda.veda_tile_select(plan, run.bufs["s"], [0, 2])
    assert e.value.status == veda.VEDA_ERR_INVALID_ARG
    with pytest.raises(veda.VedaError) as e:
        veda.veda_tile_select(plan, run.bufs["s"], [2, plan.tiles[1] + 1])
    assert e.value.status == veda.VEDA_ERR_INVALID_ARG
    pq = veda.Mlp(run.phi_q.w1, run.phi_q.b1, run.phi_q.w2, run.phi_q.b2)
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(veda.VedaError) as e:
        veda.veda_tile_score(plan, run.bufs["qt"], run.bufs["kt"], run.bufs["vm"], pq, pq, 0.125, workspace=small)
    assert e.value.status == veda.VEDA_ERR_WORKSPACE
    with pytest.raises(veda.VedaError) as e:
        veda.veda_sparse_attn_fwd(plan, run.bufs["qt"], run.bufs["kt"], run.bufs["vt"], run.bufs["vm"],
                                  run.bufs["rp"], run.bufs["ci"], float("nan"))
    assert e.value.status == veda.VEDA_ERR_INVALID_ARG


def test_outputs_are_deterministic():
    wl = wlm.custom_workload("determinism", 3, 128, "bf16", (6, 9, 11), True, (30, 100), seed=16)
    a, b = hz.run_gpu_path(wl), hz.run_gpu_path(wl)
    assert torch.equal(a.bufs["ci"], b.bufs["ci"]) and torch.equal(a.bufs["s"], b.bufs["s"])
    assert torch.equal(a.out.view(torch.int16), b.out.view(torch.int16))


def _default_route_matches(run):
    """The route bench.py times by default (descriptors from stats-only gathers of Q and K, stages 2+3 in
    one call, attention gathering Q and K rows from token order, only V tiled) against the stage-by-stage
    run that the oracle checks: same lists, same output bits."""
    wl, plan = run.wl, run.plan
    dev = run.q.device
    pq = veda.Mlp(run.phi_q.w1, run.phi_q.b1, run.phi_q.w2, run.phi_q.b2, run.phi_q.relu, dev)
    pk = veda.Mlp(run.phi_k.w1, run.phi_k.b1, run.phi_k.w2, run.phi_k.b2, run.phi_k.relu, dev)
    none_q, vm, _, zq = veda.veda_tile_layout_stats(plan, run.q, want_tiles=False)
    none_k, _, _, zk = veda.veda_tile_layout_stats(plan, run.k, want_mask=False, want_tiles=False)
    assert none_q is None and none_k is None and torch.equal(vm, run.bufs["vm"])
    rp, ci, _ = veda.veda_tile_score_select(plan, pq, pk, run.score_scale, run.k_per_head, stats_q=zq, stats_k=zk)
    out = torch.full_like(run.out, float("nan"))
    out, _ = veda.veda_sparse_attn_fwd(plan, None, None, run.bufs["vt"], vm, rp, ci, run.softmax_scale, out=out,
                                       q_tokens=run.q, k_tokens=run.k)
    torch.cuda.synchronize()
    assert torch.equal(rp, run.bufs["rp"]) and torch.equal(ci, run.bufs["ci"]), "kept lists differ"
    assert torch.equal(out.view(torch.int16), run.out.view(torch.int16)), "attention output differs"


def test_wan1p3b_480p_sampled():
    wl = wlm.WORKLOADS["wan1p3b_480p"]
    _say(f"[parity] {wl.name}")
    run = hz.run_gpu_path(wl)
    assert torch.isfinite(run.out.float()).all()
    for h in (0, 7):
        _say(f"[parity] {wl.name} head {h}: {hz.check_head(run, h, attn_tiles=12)}")
    _default_route_matches(run)


def _sampled_config(wl, keep=None, attn_tiles=6):
    """Full-size launch configuration; oracle on one head per tile shape and a seeded sample of
    query tiles (first and last tile always included)."""
    _say(f"[parity] {wl.name} keep {keep or wl.keep}: generating inputs")
    run = hz.run_gpu_path(wl, keep=keep, want_lse=False)
    for h in hz.heads_by_shape(run):
        _say(f"[parity] {wl.name} head {h} {tuple(run.shapes[h])} k {int(run.k_per_head[h])}: checking")
        _say(f"[parity] {wl.name} head {h}: {hz.check_head(run, h, attn_tiles=attn_tiles)}")
    # every real token of every head was written (the output buffer starts as NaN)
    for h in range(wl.heads):
        assert torch.isfinite(run.out[0, h].float()).all(), h
    _say(f"[parity] {wl.name}: the default route of bench.py against this run")
    _default_route_matches(run)


@pytest.mark.parametrize("name", ["wan14b_480p", "wan14b_720p", "waver12b_720p_241f"])
def test_large_configs_sampled(name):
    _sampled_config(wlm.WORKLOADS[name])


@pytest.mark.parametrize("keep", [(20, 100), (10, 100)])
def test_wan14b_720p_sparsity_sweep(keep):
    """The 80 % and 90 % points of the 75,600-token configuration's sparsity sweep (its 95 % point is the
    workload's default, above).  At these budgets stage 3 searches whole rows instead of sampling a pivot, and
    the one-call route of stages 2+3 goes through its two-stage path: both must still give the oracle's lists."""
    wl = wlm.WORKLOADS["wan14b_720p"]
    assert keep in wl.keep_sweep and wl.keep in wl.keep_sweep
    _sampled_config(wl, keep=keep, attn_tiles=4)


def test_waver12b_dense_heads_equal_full_attention():
    """0 % sparsity at 219,600 tokens: the full 24-head launch with k = N_T on the first head of every tile
    shape (the other heads keep their 5 %), against plain softmax attention over all tokens (Eq. 1) on sampled
    query tokens of the first and last tile and a seeded spread, and against the masked oracle on two tiles."""
    wl = wlm.WORKLOADS["waver12b_720p_241f"]
    shapes = wlm.tile_shapes(wl)
    kph = wlm.keep_budget(wl, None, shapes)
    nt = wlm.tiles_per_head(wl, shapes)
    dense_heads = []
    seen = set()
    for h, sh in enumerate(map(tuple, shapes)):
        if sh not in seen:
            seen.add(sh)
            dense_heads.append(h)
            kph[h] = nt[h]
    _say(f"[parity] {wl.name}: dense heads {dense_heads}, generating inputs")
    run = hz.run_gpu_path(wl, k_per_head=kph, want_lse=False)
    for h in range(wl.heads):
        assert torch.isfinite(run.out[0, h].float()).all(), h
    rng = np.random.default_rng(404)
    for h in dense_heads:
        shape = tuple(int(x) for x in shapes[h])
        tile_of = vo.token_tile_map(wl.grid, shape)
        first, last = np.flatnonzero(tile_of == 0), np.flatnonzero(tile_of == nt[h] - 1)
        queries = np.unique(np.concatenate([first[:24], last[-24:], rng.choice(wl.tokens, 80, replace=False)]))
        qf, kf, vf = (hz.to_f32_numpy(x[0, h]) for x in (run.q, run.k, run.v))
        ref = vo.dense_attention(qf, kf, vf, run.softmax_scale, queries)
        got = hz.to_f32_numpy(run.out[0, h])[queries].astype(np.float64)
        err = np.abs(got - ref)
        _say(f"[parity] {wl.name} dense head {h} {shape}: {len(queries)} tokens max_abs {err.max():.2e} "
             f"mean_abs {err.mean():.2e}")
        assert err.max() <= hz.BF16_MAX_ABS and err.mean() <= hz.BF16_MEAN_ABS
        # the kept lists are 0..N_T-1 on every row of a dense head
        r0 = run.plan.tile_offset[h]
        rp = run.bufs["rp"][r0:r0 + nt[h] + 1].cpu().numpy().astype(np.int64)
        assert np.all(np.diff(rp) == nt[h])
        for row in (0, int(nt[h]) // 2, int(nt[h]) - 1):
            lst = run.bufs["ci"][int(rp[row]):int(rp[row + 1])].cpu().numpy()
            assert np.array_equal(lst, np.arange(nt[h]))
    h = dense_heads[0]
    _say(f"[parity] {wl.name} dense head {h}: stages against the oracle, two tiles of masked attention")
    _say(f"[parity] {wl.name} dense head {h}: {hz.check_head(run, h, attn_tiles=2, check_layout=False)}")


@pytest.mark.parametrize("name", ["wan14b_720p", "waver12b_720p_241f"])
def test_128_token_tiles_at_full_size(name):
    """The paper's tile size at a named configuration's full launch size: every 64-token shape doubled along t
    (8x4x4, 2x8x8, 32x2x2), same kept fraction; one head per shape against the oracle on sampled tiles."""
    wl = wlm.WORKLOADS[name]
    shapes = wlm.tile_shapes(wl) * np.asarray([2, 1, 1], np.int32)
    kph = wlm.keep_budget(wl, None, shapes)
    _say(f"[parity] {wl.name} with 128-token tiles: generating inputs")
    run = hz.run_gpu_path(wl, k_per_head=kph, want_lse=False, shapes=shapes, tile_tokens=128)
    for h in hz.heads_by_shape(run):
        _say(f"[parity] {wl.name} head {h} {tuple(run.shapes[h])} k {int(kph[h])}: checking")
        _say(f"[parity] {wl.name} head {h}: {hz.check_head(run, h, attn_tiles=4)}")
    for h in range(wl.heads):
        assert torch.isfinite(run.out[0, h].float()).all(), h


@pytest.mark.parametrize("tile_tokens", [64, 128])
def test_list_walk_and_step_table_give_the_same_bits_at_full_size(tile_tokens):
    """wan14b_720p at its launch size: stage 3 writes ascending rows, so the attention kernel visits the key
    tiles in the same order whether it lays its steps out in LDS first or merges the lists inside its loop
    (VEDA_OPT_ATTN_LIST_WALK): every output bit agrees, from tiled K and Q and from token order."""
    wl = wlm.WORKLOADS["wan14b_720p"]
    shapes = wlm.tile_shapes(wl) * (np.asarray([2, 1, 1], np.int32) if tile_tokens == 128 else 1)
    run = hz.run_gpu_path(wl, k_per_head=wlm.keep_budget(wl, None, shapes), shapes=shapes, tile_tokens=tile_tokens)
    b, plan = run.bufs, run.plan
    args = (b["vt"], b["vm"], b["rp"], b["ci"], run.softmax_scale)
    outs = []
    for walk in (0, 1):
        plan.set_option(veda.VEDA_OPT_ATTN_LIST_WALK, walk)
        o1, l1 = veda.veda_sparse_attn_fwd(plan, b["qt"], b["kt"], *args, want_lse=True)
        o2, l2 = veda.veda_sparse_attn_fwd(plan, None, None, *args, want_lse=True, q_tokens=run.q, k_tokens=run.k)
        torch.cuda.synchronize()
        outs.append((o1, l1, o2, l2))
    plan.set_option(veda.VEDA_OPT_ATTN_LIST_WALK, 0)
    for x, y in zip(outs[0], outs[1]):
        assert torch.equal(x.view(torch.int16) if x.dtype == torch.bfloat16 else x, y.view(torch.int16) if y.dtype == torch.bfloat16 else y)
    assert torch.equal(outs[0][0].view(torch.int16), run.out.view(torch.int16))
    assert torch.equal(outs[0][0].view(torch.int16), outs[0][2].view(torch.int16))


def test_rows_three_times_longer_than_any_named_workload():
    """783,360 tokens in one head (12,240 tiles per score row): the whole path against the oracle at a 2 %
    budget (stages 2+3 in one call take the candidate route), then the lists at a 5 % budget (k = 612, where
    that call falls back to the two stages) against the oracle's selection on the same, already checked, scores."""
    wl = wlm.custom_workload("long_video", 1, 128, "bf16", (96, 68, 120), False, (2, 100), seed=31)
    _say(f"[parity] {wl.name}: generating inputs")
    run = hz.run_gpu_path(wl, want_lse=False)
    assert run.plan.tiles[0] == 12240 and int(run.k_per_head[0]) == 245
    _say(f"[parity] {wl.name}: checking against the oracle")
    _say(f"[parity] {wl.name}: {hz.check_head(run, 0, attn_tiles=4)}")
    assert torch.isfinite(run.out.float()).all()
    _default_route_matches(run)

    _say(f"[parity] {wl.name}: 5 % budget")
    k5 = wlm.keep_budget(wl, (5, 100), run.shapes)
    assert int(k5[0]) == 612
    rp2, ci2 = veda.veda_tile_select(run.plan, run.bufs["s"], k5)
    dev = run.q.device
    pq = veda.Mlp(run.phi_q.w1, run.phi_q.b1, run.phi_q.w2, run.phi_q.b2, run.phi_q.relu, dev)
    pk = veda.Mlp(run.phi_k.w1, run.phi_k.b1, run.phi_k.w2, run.phi_k.b2, run.phi_k.relu, dev)
    rp1, ci1, _ = veda.veda_tile_score_select(run.plan, pq, pk, run.score_scale, k5, q_tiled=run.bufs["qt"],
                                              k_tiled=run.bufs["kt"], valid_mask=run.bufs["vm"])
    torch.cuda.synchronize()
    assert torch.equal(rp1, rp2) and torch.equal(ci1, ci2)
    rows = hz.sample_tiles(12240, 64, 5)
    s = run.bufs["s"][0].view(12240, 12240)[torch.as_tensor(rows, device=dev)].cpu().numpy()
    want = vo.select(s, 612)
    got = ci2.view(12240, 612)[torch.as_tensor(rows, device=dev)].cpu().numpy()
    assert np.array_equal(got, want)


# ---------------------------------------------------------------- supervision side
@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("f32", 64), ("f32", 128)])
def test_target_heatmap_and_recall(dtype, d):
    # full-attention target tile scores (max-pooled softmax) and Recall@k against the oracle:
    # ragged grid, odd tile counts, all three tile shapes, batch 2, then a subset of query tiles
    wl = wlm.custom_workload(f"heat_{dtype}_{d}", 4, d, dtype, (9, 18, 18), True, (25, 100), seed=61, batch=2)
    dev = torch.device("cuda:0")
    shapes = wlm.tile_shapes(wl)
    q, k, _ = wlm.make_qkv(wl, dev)
    plan = veda.Plan(wl.batch, wl.heads, wl.head_dim, wl.grid, shapes, wl.torch_dtype)
    qt, vm, _ = veda.veda_tile_layout(plan, q, veda.VEDA_TOKEN_MAJOR)
    kt, _, _ = veda.veda_tile_layout(plan, k, veda.VEDA_TOKEN_MAJOR, want_mask=False)
    scale = 1.0 / math.sqrt(d)
    heat = veda.veda_tile_heatmap(plan, qt, kt, vm, scale)
    torch.cuda.synchronize()
    rtol = 2e-4 if dtype == "bf16" else 2e-5
    refs = {}
    for b in range(wl.batch):
        for h in range(wl.heads):
            shape = tuple(int(x) for x in shapes[h])
            nt, soff = plan.tiles[h], plan.score_offset[h]
            ref = vo.tile_heatmap(hz.to_f32_numpy(q[b, h]), hz.to_f32_numpy(k[b, h]), wl.grid, shape, scale)
            got = heat[b, soff:soff + nt * nt].view(nt, nt).cpu().numpy().astype(np.float64)
            rel = np.abs(got - ref) / ref
            _say(f"[parity] {wl.name} b{b} h{h} {shape}: heat max rel err {rel.max():.2e}")
            assert rel.max() <= rtol, (b, h, rel.max())
            refs[(b, h)] = ref
    # a subset of query tiles: listed rows equal the full run, the others are not touched
    total = plan.total_tiles
    some = np.asarray(sorted({0, 1, total // 2, total - 1, plan.tile_offset[1] + 3}), np.int32)
    part = torch.full_like(heat, -7.0)
    veda.veda_tile_heatmap(plan, qt, kt, vm, scale, torch.as_tensor(some).to(dev), part)
    torch.cuda.synchronize()
    for h in range(wl.heads):
        nt, soff, toff = plan.tiles[h], plan.score_offset[h], plan.tile_offset[h]
        a = part[:, soff:soff + nt * nt].view(wl.batch, nt, nt)
        f = heat[:, soff:soff + nt * nt].view(wl.batch, nt, nt)
        listed = np.asarray([g - toff for g in some if toff <= g < toff + nt], np.int64)
        others = np.setdiff1d(np.arange(nt), listed)
        assert torch.equal(a[:, listed], f[:, listed]) and bool((a[:, others] == -7.0).all())
    # Recall@k of the estimator's selection against the selection from the target scores
    kph = wlm.keep_budget(wl, None, shapes)
    eq, ek = wlm.make_estimator(wl, "q"), wlm.make_estimator(wl, "k")
    s_est, _ = veda.veda_tile_score(plan, qt, kt, vm, veda.Mlp(eq.w1, eq.b1, eq.w2, eq.b2, eq.relu, dev),
                                    veda.Mlp(ek.w1, ek.b1, ek.w2, ek.b2, ek.relu, dev), hz.score_scale_of(wl))
    _, ci_est = veda.veda_tile_select(plan, s_est, kph)
    _, ci_tgt = veda.veda_tile_select(plan, heat, kph)
    rec = veda.veda_tile_recall(plan, kph, ci_est, ci_tgt)
    torch.cuda.synchronize()
    a_np, b_np = ci_est.cpu().numpy(), ci_tgt.cpu().numpy()
    nnz = int(sum(int(n) * int(kk) for n, kk in zip(plan.tiles, kph)))
    off = 0
    for h in range(wl.heads):
        nt, kk = plan.tiles[h], int(kph[h])
        for b in range(wl.batch):
            lo = b * nnz + off
            ref = vo.recall(a_np[lo:lo + nt * kk].reshape(nt, kk), b_np[lo:lo + nt * kk].reshape(nt, kk))
            assert abs(float(rec[b, h]) - ref) <= 1e-6, (b, h, float(rec[b, h]), ref)
        off += nt * kk
    same = veda.veda_tile_recall(plan, kph, ci_tgt, ci_tgt)
    assert bool((same == 1.0).all())


@pytest.mark.parametrize("dtype,tile_tokens", [("f32", 64), ("bf16", 64), ("bf16", 128)])
def test_tiling_search_errors_and_choice(dtype, tile_tokens):
    # Alg. 1 on synthetic calibration tensors: error table against the oracle, same argmin where the
    # oracle's margin is clear.  Head 0 attends within its own frame only, so the frame-shaped
    # tiling must win it by a wide margin.
    from paper_2605_30325_amd import search
    grid, d, heads, samples = (8, 12, 16), 64, 3, 2
    n = int(np.prod(grid))
    cands = [(4, 4, 4), (1, 8, 8), (16, 2, 2)] if tile_tokens == 64 else [(8, 4, 4), (1, 8, 16), (32, 2, 2)]
    wl = wlm.custom_workload(f"search_{dtype}", heads, d, dtype, grid, False, (25, 100), seed=71, batch=samples)
    dev = torch.device("cuda:0")
    q, k, v = wlm.make_qkv(wl, dev)
    frame = torch.arange(n, device=dev) // (grid[1] * grid[2])
    onehot = torch.zeros((n, d), device=dev)
    onehot[torch.arange(n, device=dev), frame] = 8.0
    q[:, 0] = onehot.to(q.dtype)
    k[:, 0] = onehot.to(k.dtype)
    scale = 1.0 / math.sqrt(d)
    best, table = search.tiling_search(q, k, v, grid, cands, (25, 100), scale, tile_tokens=tile_tokens)
    torch.cuda.synchronize()
    ref = np.zeros_like(table)
    for h in range(heads):
        for b in range(samples):
            ref[h] += vo.tiling_search_errors(hz.to_f32_numpy(q[b, h]), hz.to_f32_numpy(k[b, h]),
                                              hz.to_f32_numpy(v[b, h]), grid, cands, (25, 100), scale)
    _say(f"[parity] tiling search {dtype}: gpu {table.tolist()} oracle {ref.tolist()} best {best.tolist()}")
    # bf16 outputs carry 2^-9 relative rounding on both tensors: an absolute floor per table entry
    floor = samples * n * d * (2.0 ** -8 * 0.5) ** 2 if dtype == "bf16" else 1e-6
    assert np.all(np.abs(table - ref) <= 0.03 * ref + floor), (table, ref)
    assert tuple(best[0]) == cands[1]          # the frame-shaped tiling
    for h in range(heads):
        order = np.sort(ref[h])
        if order[1] - order[0] > 0.1 * order[1] + 2 * floor:
            assert tuple(best[h]) == tuple(cands[int(np.argmin(ref[h]))]), (h, table[h], ref[h])


def test_target_heatmap_at_full_size_sampled_rows():
    # the 32,760-token workload in the configuration bench.py --heatmap times: whole launch on the
    # GPU, oracle on a seeded sample of query tiles (first and last included), all 624 columns
    wl = wlm.WORKLOADS["wan1p3b_480p"]
    dev = torch.device("cuda:0")
    shapes = wlm.tile_shapes(wl)
    q, k, _ = wlm.make_qkv(wl, dev)
    plan = veda.Plan(wl.batch, wl.heads, wl.head_dim, wl.grid, shapes, wl.torch_dtype)
    qt, vm, _ = veda.veda_tile_layout(plan, q, veda.VEDA_TOKEN_MAJOR)
    kt, _, _ = veda.veda_tile_layout(plan, k, veda.VEDA_TOKEN_MAJOR, want_mask=False)
    scale = 1.0 / math.sqrt(wl.head_dim)
    heat = veda.veda_tile_heatmap(plan, qt, kt, vm, scale)
    torch.cuda.synchronize()
    for h in (0, wl.heads - 1):
        shape = tuple(int(x) for x in shapes[h])
        nt, soff = plan.tiles[h], plan.score_offset[h]
        rows = hz.sample_tiles(nt, 6, 100 + h)
        ref = vo.tile_heatmap(hz.to_f32_numpy(q[0, h]), hz.to_f32_numpy(k[0, h]), wl.grid, shape, scale,
                              query_tiles=rows)[rows]
        got = heat[0, soff:soff + nt * nt].view(nt, nt)[torch.as_tensor(rows).to(dev)].cpu().numpy().astype(np.float64)
        rel = np.abs(got - ref) / ref
        _say(f"[parity] {wl.name} head {h}: target scores of {len(rows)} query tiles, max rel err {rel.max():.2e}")
        assert rel.max() <= 2e-4


# ---------------------------------------------------------------- 128-token tiles
@pytest.mark.parametrize("d", [128, 64])
def test_128_token_tiles_whole_path(d):
    # the paper's tile size: every stage against the oracle with 128-token tile shapes whose halves
    # are cut across t, h or w; ragged on every axis; batch 2
    shapes = np.asarray([(8, 4, 4), (2, 8, 8), (32, 2, 2), (1, 8, 16), (1, 1, 128)], np.int32)
    wl = wlm.custom_workload(f"b128_{d}", len(shapes), d, "bf16", (9, 18, 18), True, (25, 100), seed=81, batch=2,
                             latent_dim=32)
    _whole_path_128(wl, shapes)


def _whole_path_128(wl, shapes):
    d = wl.head_dim
    dev = torch.device("cuda:0")
    q, k, v = wlm.make_qkv(wl, dev)
    plan = veda.Plan(wl.batch, wl.heads, d, wl.grid, shapes, wl.torch_dtype, tile_tokens=128)
    eq, ek = wlm.make_estimator(wl, "q"), wlm.make_estimator(wl, "k")
    pq = veda.Mlp(eq.w1, eq.b1, eq.w2, eq.b2, eq.relu, dev)
    pk = veda.Mlp(ek.w1, ek.b1, ek.w2, ek.b2, ek.relu, dev)
    sscale = hz.score_scale_of(wl)
    scale = 1.0 / math.sqrt(d)
    qt, vm, vc = veda.veda_tile_layout(plan, q, veda.VEDA_TOKEN_MAJOR)
    kt, _, _ = veda.veda_tile_layout(plan, k, veda.VEDA_TOKEN_MAJOR, want_mask=False)
    vt, _, _ = veda.veda_tile_layout(plan, v, veda.VEDA_CHANNEL_MAJOR, want_mask=False)
    s, _ = veda.veda_tile_score(plan, qt, kt, vm, pq, pk, sscale)
    kph = np.asarray([max(1, -(-n // 4)) for n in plan.tiles], np.int32)
    rp, ci = veda.veda_tile_select(plan, s, kph)
    out = torch.full((wl.batch, wl.heads, wl.tokens, d), float("nan"), dtype=wl.torch_dtype, device=dev)
    out, lse = veda.veda_sparse_attn_fwd(plan, qt, kt, vt, vm, rp, ci, scale, out=out, want_lse=True)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    # target tile scores over whole 128-token tiles, all rows and then a subset
    heat = veda.veda_tile_heatmap(plan, qt, kt, vm, scale)
    some = np.asarray(sorted({0, plan.total_tiles - 1, plan.tile_offset[wl.heads // 2] + 1}), np.int32)
    part = torch.full_like(heat, -7.0)
    veda.veda_tile_heatmap(plan, qt, kt, vm, scale, torch.as_tensor(some).to(dev), part)
    torch.cuda.synchronize()
    rp_np, ci_np = rp.cpu().numpy(), ci.cpu().numpy()
    vm_np = vm.cpu().numpy().view(np.uint64).reshape(-1, 2)
    queries = np.arange(wl.tokens)
    for b in range(wl.batch):
        for h in range(wl.heads):
            shape = tuple(int(x) for x in shapes[h])
            nt, toff, soff, ksel = plan.tiles[h], plan.tile_offset[h], plan.score_offset[h], int(kph[h])
            assert nt == vo.num_tiles(wl.grid, shape)
            qh, kh, vh = q[b, h], k[b, h], v[b, h]
            ref_q, mask, cnt = vo.tile_layout(hz.raw_numpy(qh), wl.grid, shape)
            assert np.array_equal(hz.raw_numpy(qt[b, toff:toff + nt]).reshape(ref_q.shape), ref_q)
            assert np.array_equal(vm_np[toff:toff + nt], mask)
            assert np.array_equal(vc[toff:toff + nt].cpu().numpy(), cnt)
            ref_v, _, _ = vo.tile_layout(hz.raw_numpy(vh), wl.grid, shape, channel_major=True)   # [nt][d][128]
            got_v = hz.raw_numpy(vt[b, toff:toff + nt]).reshape(nt, 2, d, 64)                     # [nt][2][d][64]
            assert np.array_equal(got_v, ref_v.reshape(nt, d, 2, 64).transpose(0, 2, 1, 3))
            qf, kf, vf = hz.to_f32_numpy(qh), hz.to_f32_numpy(kh), hz.to_f32_numpy(vh)
            lat = []
            for x, e in ((qf, eq), (kf, ek)):
                lat.append(vo.mlp(vo.trippool(x, wl.grid, shape), e.w1[h], e.b1[h], e.w2[h], e.b2[h], e.relu))
            s_ref = vo.score(lat[0], lat[1], np.float32(sscale))
            g_s = s[b, soff:soff + nt * nt].view(nt, nt).cpu().numpy()
            assert np.array_equal(g_s.view(np.uint32), s_ref.view(np.uint32)), (b, h)
            sel = vo.select(s_ref, ksel)
            r0 = b * plan.total_tiles + toff
            lo = int(rp_np[r0])
            assert np.all(np.diff(rp_np[r0:r0 + nt + 1]) == ksel)
            assert np.array_equal(ci_np[lo:lo + nt * ksel].reshape(nt, ksel), sel), (b, h)
            ref, lse_ref, _ = vo.masked_attention(qf, kf, vf, wl.grid, shape, sel, scale, queries, want_stats=True)
            err = np.abs(hz.to_f32_numpy(out[b, h]).astype(np.float64) - ref)
            lerr = np.abs(lse[b, h].cpu().numpy().astype(np.float64) - lse_ref)
            h_ref = vo.tile_heatmap(qf, kf, wl.grid, shape, scale)
            h_got = heat[b, soff:soff + nt * nt].view(nt, nt).cpu().numpy().astype(np.float64)
            rel = (np.abs(h_got - h_ref) / h_ref).max()
            p_got = part[b, soff:soff + nt * nt].view(nt, nt).cpu().numpy()
            listed = np.asarray([g - toff for g in some if toff <= g < toff + nt], np.int64)
            assert np.array_equal(p_got[listed], heat[b, soff:soff + nt * nt].view(nt, nt).cpu().numpy()[listed])
            assert np.all(np.delete(p_got, listed, axis=0) == -7.0)
            _say(f"[parity] {wl.name} b{b} h{h} {shape}: max_abs {err.max():.2e} mean_abs {err.mean():.2e} "
                 f"lse {lerr.max():.2e} heat rel {rel:.2e}")
            assert err.max() <= hz.BF16_MAX_ABS and err.mean() <= hz.BF16_MEAN_ABS and lerr.max() <= 2e-2
            assert rel <= 2e-4


@pytest.mark.parametrize("dtype,d,tile_tokens", [("bf16", 128, 64), ("f32", 64, 64), ("bf16", 64, 128)])
def test_closed_form_scorer_bit_exact(dtype, d, tile_tokens):
    # weight-free scores against the oracle, bit for bit, then their recall against the target scores
    if tile_tokens == 64:
        wl = wlm.custom_workload(f"cf_{dtype}_{d}", 4, d, dtype, (9, 18, 18), True, (25, 100), seed=91)
        shapes = wlm.tile_shapes(wl)
    else:
        shapes = np.asarray([(8, 4, 4), (2, 8, 8), (1, 8, 16), (1, 1, 128)], np.int32)
        wl = wlm.custom_workload(f"cf128_{d}", 4, d, dtype, (9, 18, 18), True, (25, 100), seed=91)
    dev = torch.device("cuda:0")
    q, k, _ = wlm.make_qkv(wl, dev)
    plan = veda.Plan(wl.batch, wl.heads, d, wl.grid, shapes, wl.torch_dtype, tile_tokens=tile_tokens)
    qt, vm, _ = veda.veda_tile_layout(plan, q, veda.VEDA_TOKEN_MAJOR)
    kt, _, _ = veda.veda_tile_layout(plan, k, veda.VEDA_TOKEN_MAJOR, want_mask=False)
    for lam in (0.0, 0.37):
        s, _ = veda.veda_tile_score_closed_form(plan, qt, kt, vm, lam)
        torch.cuda.synchronize()
        for h in range(wl.heads):
            shape = tuple(int(x) for x in shapes[h])
            nt, soff = plan.tiles[h], plan.score_offset[h]
            ref = vo.closed_form_scores(hz.to_f32_numpy(q[0, h]), hz.to_f32_numpy(k[0, h]), wl.grid, shape, lam)
            got = s[0, soff:soff + nt * nt].view(nt, nt).cpu().numpy()
            assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), (lam, h)
    if tile_tokens == 64:
        kph = wlm.keep_budget(wl, None, shapes)
        heat = veda.veda_tile_heatmap(plan, qt, kt, vm, 1.0 / math.sqrt(d))
        _, ci_t = veda.veda_tile_select(plan, heat, kph)
        _, ci_c = veda.veda_tile_select(plan, s, kph)
        rec = veda.veda_tile_recall(plan, kph, ci_c, ci_t)
        torch.cuda.synchronize()
        _say(f"[parity] {wl.name}: recall of the closed-form scorer against the target scores {rec.cpu().numpy().round(3).tolist()}")
        assert bool((rec > 0.25).all())      # well above the 0.25 keep fraction a blind scorer would get
