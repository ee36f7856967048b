#!/usr/bin/env python3
"""Benchmark of the tile-sparse attention hot path on one MI355X.

One step = one pass of the whole path over one synthetic attention call:
    layout(Q), layout(K), layout(V) -> tile score -> top-k select -> sparse attention.
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--keep NUM/DEN]
                    [--dense] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import math
import os
import re
import sys
import threading
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_F32_VALU_TFLOPS = 157.3   # vector fp32 peak with packed instructions; the fp32 matrix peak is the same figure
PEAK_HBM_GBPS = 8000.0

# roofline.traffic comes from the tracked counter summaries under profiles/: a line
#   traffic_record kernel=<name> workload=<name> tile_tokens=<B> keep=<num>/<den> route=<q>,<k> source_sha=<12 hex>
#                  fetch_kib=<FETCH_SIZE> fetch_scale=<x> write_kib=<WRITE_SIZE> write_scale=<x>
# gives the rocprofv3 --pmc readings (KiB per dispatch) and the factors that calibrate them against a
# copy kernel of known size.  A record is used only if it names the workload, tile size, keep
# fraction and Q/K route of this run AND the hash of the attention kernel's sources as they are now;
# otherwise traffic is null and traffic_source says why.
KERNEL_SOURCES = ("attn_pair.hip", "attn_step.h", "attn_union.h", "attn_common.h", "attn.hip", "veda_internal.h", "geometry.h")


def kernel_source_sha() -> str:
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        h.update((ROOT / "paper_2605_30325_amd" / "csrc" / name).read_bytes())
    return h.hexdigest()[:12]


def measured_traffic(kernel: str, workload: str, tile_tokens: int, keep, route_qk: str):
    """(bytes per launch or None, where it came from / why there is none)."""
    sha = kernel_source_sha()
    want = {"kernel": kernel, "workload": workload, "tile_tokens": str(tile_tokens), "keep": f"{keep[0]}/{keep[1]}",
            "route": route_qk}
    stale = None
    for path in sorted((ROOT / "profiles").glob("*.txt")):
        for line in path.read_text().splitlines():
            if not line.startswith("traffic_record "):
                continue
            rec = dict(kv.split("=", 1) for kv in line.split()[1:])
            if any(rec.get(k) != v for k, v in want.items()):
                continue
            if rec.get("source_sha") != sha:
                stale = f"profiles/{path.name} has a record for this run, taken from other kernel sources ({rec.get('source_sha')}, now {sha})"
                continue
            nbytes = (float(rec["fetch_kib"]) * float(rec["fetch_scale"]) + float(rec["write_kib"]) * float(rec["write_scale"])) * 1024.0
            return nbytes, f"profiles/{path.name} (source_sha {sha})"
    return None, stale or f"no counter record under profiles/ for {want} at source_sha {sha}"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="waver12b_720p_241f")
    ap.add_argument("--keep", default=None, help="kept fraction NUM/DEN (default: the workload's)")
    ap.add_argument("--dense", action="store_true", help="also time one dense (k = N_T) attention call")
    ap.add_argument("--two-stage", action="store_true",
                    help="stages 2 and 3 as separate calls with the score matrix between them; default: one call "
                         "(veda_tile_score_select*, scores never written), whose time is reported under stage "
                         "'score' with stage 'select' 0")
    ap.add_argument("--tiled-q", action="store_true",
                    help="write the tiled copy of Q and let the attention kernel read it; default (bf16, 64-token "
                         "tiles, descriptors from the gather): Q's gather only takes descriptors and masks, the "
                         "attention kernel gathers Q rows from token order itself")
    ap.add_argument("--tiled-k", action="store_true",
                    help="write the tiled copy of K and let the attention kernel read key tiles from it; default "
                         "(with the default Q route): K's gather only takes descriptors and the attention kernel "
                         "gathers every kept key tile's rows from token order")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--attn-only", action="store_true", help="time only the sparse attention call per step")
    ap.add_argument("--tile-tokens", type=int, default=64, choices=(64, 128),
                    help="128: the paper's tile size; every head's 64-token shape doubled along t "
                         "(4x4x4 -> 8x4x4, 1x8x8 -> 2x8x8, 16x2x2 -> 32x2x2); same keep fraction")
    ap.add_argument("--heatmap", action="store_true",
                    help="also time the full-attention target tile scores (two dense Q K^T passes) and Recall@k")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph and time its replays (the per-stage times and the "
                         "roofline then come from eager steps run after the timed region)")
    ap.add_argument("--exact-logit-scale", action="store_true",
                    help="VEDA_OPT_EXACT_LOGIT_SCALE: Q scaled by a power of two only, the rest of softmax_scale*log2(e) "
                         "applied to the logits in fp32 (error independent of the logits' size, about 4 % more time)")
    ap.add_argument("--fp32-chains", default="probed", choices=("probed", "matrix", "vector"),
                    help="VEDA_OPT_FP32_CHAIN_UNIT: where the projections' (and a score matrix's) fp32 chains run; "
                         "probed = what the library's probe of this device allows (the matrix cores on gfx950)")
    ap.add_argument("--list-walk", action="store_true",
                    help="VEDA_OPT_ATTN_LIST_WALK: the bf16 attention kernel merges the kept lists inside its loop "
                         "instead of building its step table first")
    ap.add_argument("--lists", default="selected", choices=("selected", "partner", "head", "first"),
                    help="diagnostic for --attn-only (the outputs are no longer the method's): the kept lists the attention "
                         "call walks.  selected: as stages 2+3 chose them; partner: both query tiles of a workgroup get the "
                         "list of the first of them (every loaded key tile serves both: 0.5 loads per kept pair, own "
                         "neighbourhood); head: every row of a head gets the list of the head's middle row (the same, and "
                         "all workgroups walk the same ~k tiles: cache-hot); first: every row keeps tiles 0..k-1")
    ap.add_argument("--unfused", action="store_true",
                    help="stage 2 re-reads the tiled Q and K for its descriptors (veda_tile_layout + veda_tile_score) "
                         "instead of taking them during the gathers")
    return ap.parse_args()


def cpu_baseline(wl, shapes, kph, dense_flops, q, k, v, eq, ek, score_scale, softmax_scale):
    """Times the CPU oracle on a bounded sample and extrapolates to the whole call."""
    import numpy as np
    from oracle import oracle as vo
    head = 0
    shape = tuple(int(x) for x in shapes[head])
    qf, kf, vf = (t[0, head].to("cpu").float().numpy() for t in (q, k, v))
    t0 = time.perf_counter()
    for x, cm in ((qf, False), (kf, False), (vf, True)):
        vo.tile_layout(x, wl.grid, shape, channel_major=cm)
    *_, idx = vo.estimate_and_select(qf, kf, wl.grid, shape, eq, ek, head, int(kph[head]),
                                     np.float32(score_scale))
    t_prep = time.perf_counter() - t0
    # attention: sample query tokens for ~15 s of work
    rng = np.random.default_rng(0)
    n_probe = min(wl.tokens, 2048)
    queries = np.sort(rng.choice(wl.tokens, size=n_probe, replace=False))
    t0 = time.perf_counter()
    vo.masked_attention(qf, kf, vf, wl.grid, shape, idx, softmax_scale, queries)
    t_probe = time.perf_counter() - t0
    n_q = int(min(wl.tokens, max(n_probe, 15.0 / max(t_probe / n_probe, 1e-9))))
    queries = np.sort(rng.choice(wl.tokens, size=n_q, replace=False))
    t0 = time.perf_counter()
    vo.masked_attention(qf, kf, vf, wl.grid, shape, idx, softmax_scale, queries)
    t_attn = time.perf_counter() - t0
    total_s = wl.heads * (t_prep + t_attn / n_q * wl.tokens)
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {
        "value": dense_flops / total_s / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
        "sample": (f"head 0 of {wl.heads}: stages 1-3 in full ({t_prep:.2f} s) + masked attention on "
                   f"{n_q} of {wl.tokens} query tokens ({t_attn:.2f} s); extrapolated to all heads and tokens "
                   f"({total_s:.0f} s per call)"),
        "extrapolated_s_per_call": total_s,
    }


def altered_lists(kind, plan, shapes, kph, grid, row_ptr, col_idx):
    """The kept lists of --lists (see its help); partner lists follow the library's pairing rule
    (partners along the thinnest tile axis with an even tile count, ties to w, then h)."""
    import numpy as np
    import torch
    T, H, W = grid
    rp = row_ptr.cpu().numpy()
    out = col_idx.clone()
    for h in range(plan.heads):
        n, kk, lo = plan.tiles[h], int(kph[h]), int(rp[plan.tile_offset[h]])
        lists = col_idx[lo:lo + n * kk].view(n, kk)
        if kind == "first":
            new = torch.arange(kk, device=col_idx.device, dtype=col_idx.dtype).repeat(n)
        elif kind == "head":
            new = lists[n // 2].repeat(n)
        else:
            ext = [int(x) for x in shapes[h]]
            cnt = [-(-T // ext[0]), -(-H // ext[1]), -(-W // ext[2])]
            ax, best = -1, 0.0
            for a in (2, 1, 0):
                if cnt[a] < 2:
                    continue
                alone = 1.0 / cnt[a] if cnt[a] % 2 else 0.0
                cost = (1.0 - alone) * (0.60 if ext[a] == min(ext) else 0.68) + alone
                if ax < 0 or cost < best - 1e-12:
                    ax, best = a, cost
            idx = np.arange(n).reshape(cnt)
            lead = np.take(idx, np.arange(cnt[ax]) // 2 * 2, axis=ax).reshape(-1)
            new = lists[torch.as_tensor(lead, device=col_idx.device)].reshape(-1)
        out[lo:lo + n * kk] = new
    return out


class ShaderClockSampler(threading.Thread):
    """Reads the shader clock (sysfs pp_dpm_sclk, the starred entry) and the board power (hwmon
    power1_input, with its cap) the driver reports for device 0 every few milliseconds while the timed
    steps run: the attention kernel is power-limited, so the clock it is held at and the power drawn
    belong next to its rate.  Yields nothing for a file that is missing."""

    def __init__(self, period_s: float = 0.003):
        super().__init__(daemon=True)
        self.period, self.samples, self.stop_flag, self.path = period_s, [], threading.Event(), None
        self.power_path, self.power, self.power_cap = None, [], None
        try:
            import glob
            import torch
            props = torch.cuda.get_device_properties(0)
            want = "%04x:%02x:%02x." % (props.pci_domain_id, props.pci_bus_id, props.pci_device_id)
            for dev in glob.glob("/sys/class/drm/card*/device"):
                if os.path.realpath(dev).split("/")[-1].startswith(want) and os.path.exists(dev + "/pp_dpm_sclk"):
                    self.path = dev + "/pp_dpm_sclk"
                    for hw in glob.glob(dev + "/hwmon/hwmon*/power1_input"):
                        self.power_path = hw
                        cap = hw.replace("power1_input", "power1_cap")
                        if os.path.exists(cap):
                            self.power_cap = int(open(cap).read()) / 1e6
        except Exception:
            self.path = None

    def run(self):
        if self.path is None:
            return
        pat = re.compile(r"(\d+)\s*[Mm][Hh]z\s*\*")
        while not self.stop_flag.is_set():
            try:
                m = pat.search(open(self.path).read())
                if m:
                    self.samples.append(int(m.group(1)))
                if self.power_path:
                    self.power.append(int(open(self.power_path).read()) / 1e6)
            except (OSError, ValueError):
                return
            time.sleep(self.period)

    def summary(self):
        self.stop_flag.set()
        self.join(timeout=1.0)
        if not self.samples:
            return None
        a = self.samples
        out = {"mean": sum(a) / len(a), "min": float(min(a)), "max": float(max(a)), "samples": len(a)}
        if self.power:   # the driver's reading is a moving average: the later samples are the steady state
            tail = self.power[len(self.power) // 2:]
            out["board_power_w"] = {"mean_second_half": sum(tail) / len(tail), "max": max(self.power), "cap": self.power_cap}
        return out


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only; run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2605_30325_amd import veda, workloads as wlm

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    veda.load()
    dev = torch.device("cuda:0")
    wl = wlm.WORKLOADS[args.workload]
    keep = tuple(int(x) for x in args.keep.split("/")) if args.keep else None
    shapes = wlm.tile_shapes(wl)
    B = args.tile_tokens
    if B == 128:
        shapes = shapes * np.asarray([2, 1, 1], np.int32)
    q, k, v = wlm.make_qkv(wl, dev)
    plan = veda.Plan(wl.batch, wl.heads, wl.head_dim, wl.grid, shapes, wl.torch_dtype, tile_tokens=B)
    if args.exact_logit_scale:
        plan.set_option(veda.VEDA_OPT_EXACT_LOGIT_SCALE, 1)
    if args.list_walk:
        plan.set_option(veda.VEDA_OPT_ATTN_LIST_WALK, 1)
    if args.fp32_chains != "probed":
        plan.set_option(veda.VEDA_OPT_FP32_CHAIN_UNIT,
                        veda.VEDA_CHAINS_MATRIX if args.fp32_chains == "matrix" else veda.VEDA_CHAINS_VECTOR)
    kph = wlm.keep_budget(wl, keep, shapes)
    eq, ek = wlm.make_estimator(wl, "q"), wlm.make_estimator(wl, "k")
    pq = veda.Mlp(eq.w1, eq.b1, eq.w2, eq.b2, eq.relu, dev)
    pk = veda.Mlp(ek.w1, ek.b1, ek.w2, ek.b2, ek.relu, dev)
    score_scale = float(np.float32(1.0) / np.sqrt(np.float32(wl.latent_dim)))
    softmax_scale = 1.0 / math.sqrt(wl.head_dim)

    es = 2 if wl.dtype == "bf16" else 4
    d, N, heads = wl.head_dim, wl.tokens, wl.heads
    tiles = np.asarray(plan.tiles, np.int64)
    pairs = int((tiles * kph).sum()) * wl.batch
    kept_flops = pairs * 4 * B * B * d
    dense_flops = 4.0 * N * N * d * heads * wl.batch
    slots = int(tiles.sum()) * B * wl.batch
    bytes_layout = 3 * (N * heads * wl.batch * d * es + slots * d * es)
    stat_bytes = 2 * int(tiles.sum()) * wl.batch * 3 * d * 4     # descriptors of Q and K tiles
    if args.unfused:
        bytes_score = 2 * slots * d * es + int((tiles * tiles).sum()) * 4 * wl.batch
    else:   # the gathers also write the descriptors; the score stage reads them instead of the tiles
        bytes_layout += stat_bytes
        bytes_score = stat_bytes + int((tiles * tiles).sum()) * 4 * wl.batch
    bytes_select = int((tiles * tiles).sum()) * 4 * wl.batch + pairs * 4
    # one call: descriptors (or tiles) in, lists out; the score matrix makes no round trip
    bytes_score_select = bytes_score - int((tiles * tiles).sum()) * 4 * wl.batch + pairs * 4
    bytes_attn_kv = pairs * 2 * B * d * es

    # Q straight from token order: needs the descriptor-taking gather (64-token tiles) and the bf16 kernel
    q_from_tokens = not args.tiled_q and not args.unfused and wl.dtype == "bf16"
    k_from_tokens = q_from_tokens and not args.tiled_k
    if q_from_tokens:
        bytes_layout -= slots * d * es   # the tiled copy of Q is not written
    if k_from_tokens:
        bytes_layout -= slots * d * es   # nor that of K
    route = {"stage1": "gather + reread for descriptors" if args.unfused else "descriptors during the gather",
             "stages23": "two calls, score matrix in HBM" if args.two_stage else "one call, no score matrix",
             "q": "token order" if q_from_tokens else "tiled copy", "k": "token order" if k_from_tokens else "tiled copy",
             "logit_scale": "exact (power of two into Q)" if args.exact_logit_scale else "default (Q pre-scaled, rounded once)",
             "steps": "lists merged inside the loop" if args.list_walk else "step table in LDS",
             "fp32_chains": "matrix cores" if plan.chain_unit() == veda.VEDA_CHAINS_MATRIX else "vector units"}
    route_qk = ("tokens" if q_from_tokens else "tiled") + "," + ("tokens" if k_from_tokens else "tiled") + (
        ",exact" if args.exact_logit_scale else "") + (",walk" if args.list_walk else "")
    bufs = {}

    def step(events=None):
        ev = events
        if ev: ev[0].record()
        if args.unfused:
            qt, vm, vc = veda.veda_tile_layout(plan, q, veda.VEDA_TOKEN_MAJOR, bufs.get("qt"), bufs.get("vm"), bufs.get("vc"))
            kt, _, _ = veda.veda_tile_layout(plan, k, veda.VEDA_TOKEN_MAJOR, bufs.get("kt"), want_mask=False)
        else:   # TripPool descriptors taken during the Q and K gathers
            qt, vm, vc, zq = veda.veda_tile_layout_stats(plan, q, bufs.get("qt"), bufs.get("vm"), bufs.get("vc"),
                                                         bufs.get("zq"), want_tiles=not q_from_tokens)
            kt, _, _, zk = veda.veda_tile_layout_stats(plan, k, bufs.get("kt"), stats=bufs.get("zk"), want_mask=False,
                                                       want_tiles=not k_from_tokens)
            bufs.update(zq=zq, zk=zk)
        vt, _, _ = veda.veda_tile_layout(plan, v, veda.VEDA_CHANNEL_MAJOR, bufs.get("vt"), want_mask=False)
        if ev: ev[1].record()
        if not args.two_stage:
            s = None
            if args.unfused:
                rp, ci, ws = veda.veda_tile_score_select(plan, pq, pk, score_scale, kph, q_tiled=qt, k_tiled=kt,
                                                         valid_mask=vm, row_ptr=bufs.get("rp"),
                                                         col_idx=bufs.get("ci"), workspace=bufs.get("ws"))
            else:
                rp, ci, ws = veda.veda_tile_score_select(plan, pq, pk, score_scale, kph, stats_q=zq, stats_k=zk,
                                                         row_ptr=bufs.get("rp"), col_idx=bufs.get("ci"),
                                                         workspace=bufs.get("ws"))
            if ev: ev[2].record()
        else:
            if args.unfused:
                s, ws = veda.veda_tile_score(plan, qt, kt, vm, pq, pk, score_scale, bufs.get("s"), bufs.get("ws"))
            else:
                s, ws = veda.veda_tile_score_stats(plan, zq, zk, pq, pk, score_scale, bufs.get("s"), bufs.get("ws"))
            if ev: ev[2].record()
            rp, ci = veda.veda_tile_select(plan, s, kph, bufs.get("rp"), bufs.get("ci"))
        if ev: ev[3].record()
        out, _ = veda.veda_sparse_attn_fwd(plan, qt, kt, vt, vm, rp, ci, softmax_scale, bufs.get("out"),
                                           q_tokens=q if q_from_tokens else None,
                                           k_tokens=k if k_from_tokens else None)
        if ev: ev[4].record()
        bufs.update(qt=qt, kt=kt, vt=vt, vm=vm, vc=vc, s=s, ws=ws, rp=rp, ci=ci, out=out)

    def attn_only(events=None):
        if events: events[3].record()
        veda.veda_sparse_attn_fwd(plan, bufs["qt"], bufs["kt"], bufs["vt"], bufs["vm"], bufs["rp"], bufs["ci"],
                                  softmax_scale, bufs["out"], q_tokens=q if q_from_tokens else None,
                                  k_tokens=k if k_from_tokens else None)
        if events: events[4].record()

    step()
    torch.cuda.synchronize()
    if args.lists != "selected":
        if not args.attn_only or B != 64:
            print("bench.py: --lists is a diagnostic of the attention call alone: use it with --attn-only, 64-token tiles",
                  file=sys.stderr)
            sys.exit(2)
        bufs["ci"] = altered_lists(args.lists, plan, shapes, kph, wl.grid, bufs["rp"], bufs["ci"])
    run = attn_only if args.attn_only else step
    eager = run
    if args.graph:   # the stage calls only enqueue kernels: one step replayed as a single graph launch
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            eager()
        run = lambda events=None: graph.replay()
    for _ in range(args.warmup):
        run()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    clock = ShaderClockSampler()
    clock.start()
    t0 = time.perf_counter()
    for i in range(args.steps):
        run(evs[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    sclk = clock.summary()
    if args.graph:   # per-stage durations: the same kernels launched eagerly, outside the timed region
        for i in range(args.steps):
            eager(evs[i])
        torch.cuda.synchronize()
    ms_per_step = wall * 1e3 / args.steps
    # event index pairs of the stages; one call for stages 2+3 leaves no event between them
    spans = {"layout": (0, 1), "score": (1, 2), "select": (2, 3), "attn": (3, 4)}
    if not args.two_stage:
        spans = {"layout": (0, 1), "score_select": (1, 3), "attn": (3, 4)}
    if args.attn_only:
        spans = {"attn": (3, 4)}
    stage_ms = {n: sum(e[i].elapsed_time(e[j]) for e in evs) / args.steps for n, (i, j) in spans.items()}
    attn_ms = stage_ms["attn"]
    attn_each = sorted(e[3].elapsed_time(e[4]) for e in evs)
    attn_ms_median = attn_each[len(attn_each) // 2] if len(attn_each) % 2 else 0.5 * (
        attn_each[len(attn_each) // 2 - 1] + attn_each[len(attn_each) // 2])
    kept_tflops = kept_flops / (attn_ms * 1e-3) / 1e12

    kernel_name = "sparse_attn_bf16_pair_kernel" if wl.dtype == "bf16" else "sparse_attn_f32_kernel"
    traffic, traffic_source = measured_traffic(kernel_name, wl.name, B, keep or wl.keep, route_qk)
    result = {
        "metric": "dense_equiv_tflops_whole_path" if not args.attn_only else "dense_equiv_tflops_attn_only",
        "value": dense_flops / (ms_per_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic", "launch": "hip_graph" if args.graph else "eager",
        "config": {"workload": wl.name, "grid": list(wl.grid), "tokens": N, "heads": heads, "head_dim": d,
                   "tile_tokens": B, "keep": list(keep or wl.keep), "kept_tile_pairs": pairs,
                   "sparsity": 1.0 - pairs / float((tiles * tiles).sum() * wl.batch), "route": route,
                   "lists": args.lists},
        "attn_ms_per_call": attn_ms, "attn_ms_median": attn_ms_median,
        "attn_ms_min": attn_each[0], "attn_ms_max": attn_each[-1],
        "attn_dense_equiv_tflops": dense_flops / (attn_ms * 1e-3) / 1e12,
        "attn_kept_tflops": kept_tflops,
        "stage_ms": stage_ms,
        "roofline": {"kernel": kernel_name,
                     "bound": "mfma",   # bf16: bf16 matrix peak; fp32: the fp32 matrix peak (157.3 TFLOP/s)
                     "achieved": kept_tflops,
                     "peak": PEAK_BF16_TFLOPS if wl.dtype == "bf16" else PEAK_F32_VALU_TFLOPS,
                     "unit": "TFLOP/s",
                     "frac": kept_tflops / (PEAK_BF16_TFLOPS if wl.dtype == "bf16" else PEAK_F32_VALU_TFLOPS),
                     "traffic": traffic, "traffic_source": traffic_source,
                     "flops_per_launch": kept_flops, "kv_tile_bytes_per_launch": bytes_attn_kv},
        # Diagnostics only, never compared with the target (roofline.frac against the nominal peak
        # is): the clock the driver reported during the timed steps and the share of the matrix
        # pipes' cycles AT THAT CLOCK that the kept-tile FLOPs fill (256 CUs x 4096 FLOP per clock)
        "diagnostics": {"sclk_mhz": sclk,
                        "matrix_pipe_busy_at_observed_clock": (kept_tflops * 1e12 / (sclk["mean"] * 1e6 * 256 * 4096)
                                                               if sclk and wl.dtype == "bf16" else None)},
    }
    if not args.attn_only:
        stage_bytes = {"layout": bytes_layout, "score": bytes_score, "select": bytes_select,
                       "score_select": bytes_score_select}
        result["stage_hbm_gbps"] = {n: stage_bytes[n] / (ms * 1e-3) / 1e9 for n, ms in stage_ms.items() if n != "attn"}
        result["stage_hbm_frac"] = {n: g / PEAK_HBM_GBPS for n, g in result["stage_hbm_gbps"].items()}
        # stages 2+3 are bound by their fixed-order fp32 chains (plain fma, no packed fp32: half the
        # vector peak), not by memory: projections 2*(3d*d + d*d') flop per tile and estimator, scores
        # 2*d' flop per tile pair
        dp_, hid_ = int(eq.w2.shape[-1]), int(eq.w1.shape[-1])
        chain_flops = (2 * 2 * (3 * d * hid_ + hid_ * dp_) * int(tiles.sum()) + 2 * dp_ * int((tiles * tiles).sum())) * wl.batch
        t23 = stage_ms.get("score_select", stage_ms.get("score", 0.0) + stage_ms.get("select", 0.0))
        result["stage23_fp32"] = {"flop": chain_flops, "tflops": chain_flops / (t23 * 1e-3) / 1e12,
                                  "frac_of_unpacked_vector_peak": chain_flops / (t23 * 1e-3) / 1e12 / (PEAK_F32_VALU_TFLOPS / 2)}

    if (args.dense or args.heatmap) and bufs.get("qt") is None:   # these side runs read the tiled Q (and K)
        bufs["qt"] = veda.veda_tile_layout(plan, q, veda.VEDA_TOKEN_MAJOR, want_mask=False)[0]
    if (args.dense or args.heatmap) and bufs.get("kt") is None:
        bufs["kt"] = veda.veda_tile_layout(plan, k, veda.VEDA_TOKEN_MAJOR, want_mask=False)[0]

    if args.dense:
        kd = np.asarray(plan.tiles, np.int32)
        if bufs.get("s") is None:   # k = N_T keeps every tile whatever the scores are
            bufs["s"] = torch.zeros((plan.batch, plan.score_elems), dtype=torch.float32, device=dev)
        rp_d, ci_d = veda.veda_tile_select(plan, bufs["s"], kd)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        veda.veda_sparse_attn_fwd(plan, bufs["qt"], bufs["kt"], bufs["vt"], bufs["vm"], rp_d, ci_d, softmax_scale, bufs["out"])
        torch.cuda.synchronize()
        e0.record()
        veda.veda_sparse_attn_fwd(plan, bufs["qt"], bufs["kt"], bufs["vt"], bufs["vm"], rp_d, ci_d, softmax_scale, bufs["out"])
        e1.record()
        torch.cuda.synchronize()
        dense_ms = e0.elapsed_time(e1)
        padded_flops = float((tiles * tiles).sum()) * wl.batch * 4 * B * B * d
        result["dense_run"] = {"attn_ms": dense_ms, "tflops_on_padded_tiles": padded_flops / (dense_ms * 1e-3) / 1e12,
                               "speedup_sparse_vs_dense": dense_ms / attn_ms,
                               "paper_context": "paper reports 10.5x self-attention / 5.1x end-to-end on NVIDIA Hopper "
                                                "vs FlashAttention-3 with 128-token tiles (different hardware and baseline)"}
        del rp_d, ci_d

    if args.heatmap:
        # supervision side (not part of a step): two dense Q K^T passes over all tile pairs, then
        # the recall of the estimator's selection against the selection from the target scores
        heat = veda.veda_tile_heatmap(plan, bufs["qt"], bufs["kt"], bufs["vm"], softmax_scale)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        veda.veda_tile_heatmap(plan, bufs["qt"], bufs["kt"], bufs["vm"], softmax_scale, heat=heat)
        e1.record()
        torch.cuda.synchronize()
        heat_ms = e0.elapsed_time(e1)
        _, ci_t = veda.veda_tile_select(plan, heat, kph)
        rec = veda.veda_tile_recall(plan, kph, bufs["ci"], ci_t)
        torch.cuda.synchronize()
        qk_flops = 2.0 * float((tiles * tiles).sum()) * wl.batch * 2 * B * B * d
        result["heatmap_run"] = {"ms": heat_ms, "tflops_two_qk_passes_on_padded_tiles": qk_flops / (heat_ms * 1e-3) / 1e12,
                                 "recall_at_k_random_init_estimator_mean": float(rec.mean().item())}
        del heat, ci_t

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, shapes, kph, dense_flops, q, k, v, eq, ek, score_scale, softmax_scale)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
