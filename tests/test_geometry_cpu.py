"""Host geometry of the tilings, checked without a GPU: csrc/geometry.h is compiled with g++ into a
small program that prints, for ragged grids and both tile sizes, every tile's anchor token next to
the token of its slot 0; the oracle's own slot map says which tiles are real."""
import shutil
import subprocess
from pathlib import Path

import numpy as np
import pytest

from oracle import oracle as vo

ROOT = Path(__file__).resolve().parent.parent
CSRC = ROOT / "paper_2605_30325_amd" / "csrc"

PROGRAM = r"""
#include <cstdio>
#include <cstdlib>
#include "geometry.h"
int main(int argc, char** argv) {
    const int T = atoi(argv[1]), H = atoi(argv[2]), W = atoi(argv[3]), grp = atoi(argv[7]);
    const int32_t shape[3] = {atoi(argv[4]), atoi(argv[5]), atoi(argv[6])};
    veda::HeadGeom g;
    veda::head_extents(g, shape, grp, T, H, W);
    printf("%d\n", g.n_tiles);
    for (int i = 0; i < g.n_tiles; ++i) printf("%d\n", veda::tile_anchor_token(g, i, T, H, W));
    return 0;
}
"""

CASES = [
    # grid, whole-tile shape, 64-slot tiles per whole tile
    ((21, 5, 6), (16, 2, 4), 2),     # second halves along t wholly outside the grid
    ((9, 18, 18), (8, 4, 4), 2),
    ((9, 18, 18), (1, 8, 16), 2),    # cut along h: halves outside in h
    ((3, 5, 70), (1, 1, 128), 2),    # cut along w
    ((9, 18, 18), (2, 8, 8), 2),
    ((5, 9, 10), (4, 4, 4), 1),
    ((7, 9, 11), (16, 2, 2), 1),
    ((61, 45, 80), (1, 8, 8), 1),
]


@pytest.fixture(scope="module")
def geometry_tool(tmp_path_factory):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no C++ compiler")
    d = tmp_path_factory.mktemp("geom")
    (d / "geom.cc").write_text(PROGRAM)
    exe = d / "geom"
    subprocess.check_call([gxx, "-std=c++17", "-O1", "-Wall", "-Werror", f"-I{CSRC}", str(d / "geom.cc"), "-o", str(exe)])
    return exe


@pytest.mark.parametrize("grid,shape,grp", CASES)
def test_every_tile_anchor_is_a_real_token(geometry_tool, grid, shape, grp):
    out = subprocess.run([str(geometry_tool), *map(str, grid), *map(str, shape), str(grp)], capture_output=True,
                         text=True, check=True).stdout.split()
    n_tiles, anchors = int(out[0]), np.asarray(out[1:], np.int64)
    tokens = grid[0] * grid[1] * grid[2]
    whole = vo.num_tiles(grid, shape)
    assert n_tiles == grp * whole and len(anchors) == n_tiles
    assert anchors.min() >= 0 and anchors.max() < tokens, "an anchor outside the tensor"
    # the oracle's token -> (tile, slot) map of the whole tiles: slot 0 of 64-slot tile i is slot
    # 64*(i % grp) of whole tile i / grp
    tile_of = vo.token_tile_map(grid, shape)
    slot0 = {}
    B = shape[0] * shape[1] * shape[2]
    t, h, w = np.meshgrid(np.arange(grid[0]), np.arange(grid[1]), np.arange(grid[2]), indexing="ij")
    slot = ((t % shape[0]) * shape[1] + h % shape[1]) * shape[2] + w % shape[2]
    for n, (ti, sl) in enumerate(zip(tile_of.reshape(-1), slot.reshape(-1))):
        if sl % (B // grp) == 0:
            slot0[grp * int(ti) + int(sl) // (B // grp)] = n
    empty = 0
    for i in range(n_tiles):
        if i in slot0:
            assert anchors[i] == slot0[i], (i, anchors[i], slot0[i])
        else:      # a half with no real slot: anchored at its first half
            assert grp == 2 and i % 2 == 1 and anchors[i] == slot0[i - 1], i
            empty += 1
    if (grid, shape) in (((21, 5, 6), (16, 2, 4)), ((9, 18, 18), (1, 8, 16))):
        assert empty > 0
