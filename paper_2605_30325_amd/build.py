"""Builds libveda.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

Run as `python -m paper_2605_30325_amd.build`.  Each translation unit is compiled on its
own; score.hip and fused.hip additionally get -ffp-contract=off because their fp32 results decide
the top-k set and must follow a fixed operation order.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
ROOT = PKG.parent
CSRC = PKG / "csrc"
OBJ = PKG / "_build"
LIB = PKG / "libveda.so"

SOURCES = ["plan.hip", "layout.hip", "score.hip", "chains_vector.hip", "select.hip", "fused.hip", "attn.hip", "attn_pair.hip", "attn_f32.hip", "heatmap.hip"]
COMMON = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", f"-I{ROOT / 'include'}", f"-I{CSRC}",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-command-line-argument"]
PER_FILE = {"score.hip": ["-ffp-contract=off"], "fused.hip": ["-ffp-contract=off"], "chains_vector.hip": ["-ffp-contract=off"]}


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src: str, extra=()) -> Path:
    obj = OBJ / (src + ".o")
    cmd = [hipcc(), *COMMON, *PER_FILE.get(src, []), *extra, "-c", str(CSRC / src), "-o", str(obj)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    lines = [l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip()]
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, "\n".join(lines)))
    if lines and os.environ.get("VEDA_BUILD_VERBOSE"):
        print("\n".join(lines), file=sys.stderr)
    return obj


def build(verbose: bool = False, extra=()) -> Path:
    """Compile every translation unit and link libveda.so.  Always recompiles."""
    OBJ.mkdir(exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, extra), SOURCES))
    tmp = LIB.with_suffix(f".tmp{os.getpid()}.so")
    subprocess.check_call([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(tmp), *map(str, objs)])
    os.replace(tmp, LIB)
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build(verbose=True)
