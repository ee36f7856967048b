"""The entry point that allocates nothing (veda_tile_score_select_stats_noalloc) against the entry point it
is a variant of (veda_tile_score_select_stats, caller's workspace): same row_ptr and col_idx bit for bit, on
two calls in a row, the second with a smaller input that takes the other route inside the call; device memory
in use does not move across the calls; a plan beyond the fixed array's size is refused and launches nothing."""
import math

import numpy as np
import pytest
import torch

from paper_2605_30325_amd import veda
from paper_2605_30325_amd import workloads as wlm

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _case(wl, shapes, dev):
    q, k, _ = wlm.make_qkv(wl, dev)
    plan = veda.Plan(wl.batch, wl.heads, wl.head_dim, wl.grid, shapes, wl.torch_dtype)
    kph = wlm.keep_budget(wl, None, shapes)
    eq, ek = wlm.make_estimator(wl, "q"), wlm.make_estimator(wl, "k")
    pq = veda.Mlp(eq.w1, eq.b1, eq.w2, eq.b2, eq.relu, dev)
    pk = veda.Mlp(ek.w1, ek.b1, ek.w2, ek.b2, ek.relu, dev)
    _, _, _, zq = veda.veda_tile_layout_stats(plan, q, want_tiles=False)
    _, _, _, zk = veda.veda_tile_layout_stats(plan, k, want_mask=False, want_tiles=False)
    sscale = float(np.float32(1.0) / np.sqrt(np.float32(wl.latent_dim)))
    # the existing entry point, with a workspace of the caller's
    rp_ref, ci_ref, _ = veda.veda_tile_score_select(plan, pq, pk, sscale, kph, stats_q=zq, stats_k=zk)
    torch.cuda.synchronize()
    rp = torch.full_like(rp_ref, -1)
    ci = torch.full_like(ci_ref, -1)
    return dict(wl=wl, plan=plan, kph=kph, pq=pq, pk=pk, zq=zq, zk=zk, sscale=sscale, rp_ref=rp_ref, ci_ref=ci_ref,
                rp=rp, ci=ci)


def _call(c):
    veda.veda_tile_score_select_stats_noalloc(c["plan"], c["pq"], c["pk"], c["sscale"], c["kph"], c["zq"], c["zk"],
                                              c["rp"], c["ci"])


def test_no_alloc_entry_point_matches_and_allocates_nothing():
    dev = torch.device("cuda:0")
    # first: two heads of 1024 tiles at a 5 % budget -- long rows, candidates route (the score matrix is
    # never formed); second, smaller: three ragged heads of a few dozen tiles -- the two-stage route inside the call
    big = wlm.custom_workload("noalloc_big", 2, 128, "bf16", (16, 32, 128), False, (5, 100), seed=71)
    big_shapes = np.asarray([(4, 4, 4), (1, 8, 8)], np.int32)
    small = wlm.custom_workload("noalloc_small", 3, 128, "bf16", (9, 18, 18), True, (25, 100), seed=72)
    _say("[no-alloc] preparing inputs and the reference lists")
    cases = [_case(big, big_shapes, dev), _case(small, wlm.tile_shapes(small), dev)]
    assert cases[0]["plan"].tiles == [1024, 1024]
    _say("[no-alloc] warm-up call (loads the kernels), then the two calls in a row")
    _call(cases[0])
    torch.cuda.synchronize()
    for c in cases:
        c["rp"].fill_(-1)
        c["ci"].fill_(-1)
    torch.cuda.synchronize()
    free_before, _ = torch.cuda.mem_get_info()
    torch_before = torch.cuda.memory_allocated()
    _call(cases[0])
    _call(cases[1])
    torch.cuda.synchronize()
    free_after, _ = torch.cuda.mem_get_info()
    assert free_after == free_before and torch.cuda.memory_allocated() == torch_before
    for c in cases:
        assert torch.equal(c["rp"], c["rp_ref"]), c["wl"].name
        assert torch.equal(c["ci"], c["ci_ref"]), c["wl"].name
    # and once more the other way round: the array keeps the previous call's contents, which must not matter
    for c in cases:
        c["ci"].fill_(-1)
    _call(cases[1])
    _call(cases[0])
    torch.cuda.synchronize()
    for c in cases:
        assert torch.equal(c["ci"], c["ci_ref"]), c["wl"].name


def test_no_alloc_entry_point_refuses_plans_beyond_its_array():
    dev = torch.device("cuda:0")
    wl = wlm.WORKLOADS["wan14b_480p"]          # 40 heads: needs more than the fixed array holds
    shapes = wlm.tile_shapes(wl)
    plan = veda.Plan(wl.batch, wl.heads, wl.head_dim, wl.grid, shapes, wl.torch_dtype)
    eq, ek = wlm.make_estimator(wl, "q"), wlm.make_estimator(wl, "k")
    pq = veda.Mlp(eq.w1, eq.b1, eq.w2, eq.b2, eq.relu, dev)
    pk = veda.Mlp(ek.w1, ek.b1, ek.w2, ek.b2, ek.relu, dev)
    import ctypes as C
    need = int(veda.load().veda_plan_fused_workspace_bytes(plan.handle, C.byref(pq.struct()), C.byref(pk.struct())))
    assert need > veda.NOALLOC_SCRATCH_BYTES
    z = torch.zeros((1, plan.total_tiles, 3 * wl.head_dim), dtype=torch.float32, device=dev)
    rp = torch.full((plan.total_tiles + 1,), -1, dtype=torch.int32, device=dev)
    ci = torch.full((16,), -1, dtype=torch.int32, device=dev)
    with pytest.raises(veda.VedaError) as e:
        veda.veda_tile_score_select_stats_noalloc(plan, pq, pk, 0.125, wlm.keep_budget(wl, None, shapes), z, z, rp, ci)
    torch.cuda.synchronize()
    assert e.value.status == veda.VEDA_ERR_WORKSPACE and str(need) in str(e.value)
    assert bool((rp == -1).all()) and bool((ci == -1).all())     # nothing was launched
