"""Shared driver of the GPU-vs-oracle parity tests: runs the HIP path through the C ABI
binding on a workload and checks each stage against the CPU oracle, head by head."""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from oracle import oracle as vo
from paper_2605_30325_amd import veda
from paper_2605_30325_amd import workloads as wlm

# Tolerances of the attention output against the double-precision oracle (the target's
# acceptance bar): bf16 storage -> max-abs 2e-2 and mean-abs 2e-3; fp32 storage -> 1e-4.
BF16_MAX_ABS, BF16_MEAN_ABS, F32_MAX_ABS = 2e-2, 2e-3, 1e-4


def to_f32_numpy(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu", torch.float32).numpy()


def raw_numpy(t: torch.Tensor) -> np.ndarray:
    """Bytes of a tensor as a NumPy array of same-width unsigned integers."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.float32:
        return t.view(torch.int32).numpy().view(np.uint32)
    raise TypeError(t.dtype)


@dataclass
class GpuRun:
    wl: wlm.Workload
    plan: veda.Plan
    shapes: np.ndarray
    k_per_head: np.ndarray
    q: torch.Tensor
    k: torch.Tensor
    v: torch.Tensor
    phi_q: wlm.EstimatorWeights
    phi_k: wlm.EstimatorWeights
    score_scale: float
    softmax_scale: float
    bufs: Dict[str, torch.Tensor]
    out: torch.Tensor
    lse: Optional[torch.Tensor]
    mlp_q: Optional[veda.Mlp] = None      # the device-resident projections the run used
    mlp_k: Optional[veda.Mlp] = None


def score_scale_of(wl: wlm.Workload) -> float:
    return float(np.float32(1.0) / np.sqrt(np.float32(wl.latent_dim)))


def run_gpu_path(wl: wlm.Workload, keep=None, k_per_head=None, want_lse=True, shapes=None,
                 tile_tokens: int = 64) -> GpuRun:
    """Stage by stage through the C ABI.  shapes / tile_tokens: other tile shapes than the workload's own
    (128-token tiles: every stage works on whole tiles; the oracle takes the same shapes)."""
    dev = torch.device("cuda:0")
    shapes = wlm.tile_shapes(wl) if shapes is None else np.asarray(shapes, np.int32)
    q, k, v = wlm.make_qkv(wl, dev)
    plan = veda.Plan(wl.batch, wl.heads, wl.head_dim, wl.grid, shapes, wl.torch_dtype, tile_tokens=tile_tokens)
    kph = wlm.keep_budget(wl, keep, shapes) if k_per_head is None else np.asarray(k_per_head, np.int32)
    eq, ek = wlm.make_estimator(wl, "q"), wlm.make_estimator(wl, "k")
    pq = veda.Mlp(eq.w1, eq.b1, eq.w2, eq.b2, eq.relu, dev)
    pk = veda.Mlp(ek.w1, ek.b1, ek.w2, ek.b2, ek.relu, dev)
    sscale = score_scale_of(wl)
    softmax_scale = 1.0 / math.sqrt(wl.head_dim)
    qt, vm, vc = veda.veda_tile_layout(plan, q, veda.VEDA_TOKEN_MAJOR)
    kt, _, _ = veda.veda_tile_layout(plan, k, veda.VEDA_TOKEN_MAJOR, want_mask=False)
    vt, _, _ = veda.veda_tile_layout(plan, v, veda.VEDA_CHANNEL_MAJOR, want_mask=False)
    s, ws = veda.veda_tile_score(plan, qt, kt, vm, pq, pk, sscale)
    rp, ci = veda.veda_tile_select(plan, s, kph)
    out = torch.full((wl.batch, wl.heads, wl.tokens, wl.head_dim), float("nan"), dtype=wl.torch_dtype, device=dev)
    out, lse = veda.veda_sparse_attn_fwd(plan, qt, kt, vt, vm, rp, ci, softmax_scale, out=out, want_lse=want_lse)
    torch.cuda.synchronize()
    bufs = dict(qt=qt, kt=kt, vt=vt, vm=vm, vc=vc, s=s, ws=ws, rp=rp, ci=ci)
    return GpuRun(wl, plan, shapes, kph, q, k, v, eq, ek, sscale, softmax_scale, bufs, out, lse, pq, pk)


def score_intermediates(plan: veda.Plan, phi_q: "veda.Mlp", phi_k: "veda.Mlp", workspace: torch.Tensor):
    """(z_q, z_k, y_q, y_k) as veda_tile_score left them in its workspace, each [batch*total_tiles, width],
    found through the offsets the library documents (veda_plan_workspace_layout)."""
    lay = plan.workspace_layout(phi_q, phi_k)
    ws = workspace.view(torch.float32)
    rows, d, dp = plan.batch * plan.total_tiles, plan.head_dim, phi_q.out_dim
    cut = lambda off, width: ws[off: off + rows * width].view(rows, width)
    return cut(lay.stats_q, 3 * d), cut(lay.stats_k, 3 * d), cut(lay.latent_q, dp), cut(lay.latent_k, dp)


def sample_tiles(n_tiles: int, count: int, seed: int) -> np.ndarray:
    """Seeded sample of query tiles that always holds the first and last tile."""
    if count >= n_tiles:
        return np.arange(n_tiles)
    rng = np.random.default_rng(seed)
    pick = set(rng.choice(n_tiles, size=count, replace=False).tolist()) | {0, n_tiles - 1}
    return np.asarray(sorted(pick))


def check_head(run: GpuRun, head: int, batch: int = 0, attn_tiles: Optional[int] = None,
               check_layout: bool = True) -> Dict[str, float]:
    """Stage-by-stage comparison of one head against the oracle.  Raises AssertionError."""
    wl, plan = run.wl, run.plan
    grid, shape = wl.grid, tuple(int(x) for x in run.shapes[head])
    nt, toff, soff = plan.tiles[head], plan.tile_offset[head], plan.score_offset[head]
    d, ksel = wl.head_dim, int(run.k_per_head[head])
    assert nt == vo.num_tiles(grid, shape)
    qh, kh, vh = run.q[batch, head], run.k[batch, head], run.v[batch, head]
    tag = f"{wl.name} head {head} shape {shape}"

    # stage 1: bytes
    if check_layout:
        for name, x, order in (("q", qh, False), ("k", kh, False), ("v", vh, True)):
            ref, mask, cnt = vo.tile_layout(raw_numpy(x), grid, shape, channel_major=order)
            got = raw_numpy(run.bufs[name + "t"][batch, toff:toff + nt])
            if order and plan.tile_tokens == 128:   # the library keeps [tile][half][channel][64]
                ref = ref.reshape(nt, d, 2, 64).transpose(0, 2, 1, 3)
            assert np.array_equal(got.reshape(ref.shape), ref), f"{tag}: tiled {name} differs"
        words = plan.mask_words
        gm = run.bufs["vm"][words * toff:words * (toff + nt)].cpu().numpy().view(np.uint64).reshape(mask.shape)
        assert np.array_equal(gm, mask), f"{tag}: valid_mask differs"
        assert np.array_equal(run.bufs["vc"][toff:toff + nt].cpu().numpy(), cnt), f"{tag}: valid_cnt differs"

    # stages 2-3: bit-exact statistics, latents, scores, lists
    qf, kf, vf = to_f32_numpy(qh), to_f32_numpy(kh), to_f32_numpy(vh)
    zq, zk, yq, yk, s_ref, idx_ref = vo.estimate_and_select(qf, kf, grid, shape, run.phi_q, run.phi_k, head,
                                                            ksel, np.float32(run.score_scale))
    r0 = batch * plan.total_tiles + toff
    g_zq, g_zk, g_yq, g_yk = (t[r0:r0 + nt].cpu().numpy()
                              for t in score_intermediates(plan, run.mlp_q, run.mlp_k, run.bufs["ws"]))
    assert np.array_equal(g_zq.view(np.uint32), zq.view(np.uint32)), f"{tag}: TripPool(Q) not bit-exact"
    assert np.array_equal(g_zk.view(np.uint32), zk.view(np.uint32)), f"{tag}: TripPool(K) not bit-exact"
    assert np.array_equal(g_yq.view(np.uint32), yq.view(np.uint32)), f"{tag}: phi_q not bit-exact"
    assert np.array_equal(g_yk.view(np.uint32), yk.view(np.uint32)), f"{tag}: phi_k not bit-exact"
    g_s = run.bufs["s"][batch, soff:soff + nt * nt].view(nt, nt).cpu().numpy()
    assert np.array_equal(g_s.view(np.uint32), s_ref.view(np.uint32)), f"{tag}: scores not bit-exact"
    rp = run.bufs["rp"].cpu().numpy()
    lo, hi = int(rp[r0]), int(rp[r0 + nt])
    assert hi - lo == nt * ksel and np.all(np.diff(rp[r0:r0 + nt + 1]) == ksel), f"{tag}: row_ptr wrong"
    g_idx = run.bufs["ci"][lo:hi].view(nt, ksel).cpu().numpy()
    assert np.array_equal(g_idx, idx_ref), f"{tag}: kept tile lists differ"

    # stage 4: attention of every real token of the sampled query tiles
    tiles = sample_tiles(nt, nt if attn_tiles is None else attn_tiles, 1000 * wl.seed + head)
    tile_of = vo.token_tile_map(grid, shape)
    queries = np.flatnonzero(np.isin(tile_of, tiles))
    ref, lse_ref, _ = vo.masked_attention(qf, kf, vf, grid, shape, idx_ref, run.softmax_scale, queries,
                                          want_stats=True)
    got = to_f32_numpy(run.out[batch, head])[queries].astype(np.float64)
    assert np.all(np.isfinite(got)), f"{tag}: non-finite attention output"
    err = np.abs(got - ref)
    stats = dict(max_abs=float(err.max()), mean_abs=float(err.mean()), queries=int(len(queries)))
    if wl.dtype == "bf16":
        assert stats["max_abs"] <= BF16_MAX_ABS and stats["mean_abs"] <= BF16_MEAN_ABS, f"{tag}: {stats}"
    else:
        assert stats["max_abs"] <= F32_MAX_ABS, f"{tag}: {stats}"
    if run.lse is not None:
        lerr = np.abs(run.lse[batch, head].cpu().numpy()[queries].astype(np.float64) - lse_ref)
        stats["lse_max_abs"] = float(lerr.max())
        assert stats["lse_max_abs"] <= (2e-2 if wl.dtype == "bf16" else 1e-4), f"{tag}: lse {stats}"
    return stats


def heads_by_shape(run: GpuRun, per_shape: int = 1) -> List[int]:
    """First `per_shape` heads of every distinct tile shape."""
    seen: Dict[tuple, int] = {}
    out = []
    for h, s in enumerate(map(tuple, run.shapes)):
        if seen.get(s, 0) < per_shape:
            seen[s] = seen.get(s, 0) + 1
            out.append(h)
    return out
