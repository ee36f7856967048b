// Host-and-device geometry of the tilings (Sec. 3.1 tiles of size B; Sec. 4.2 per-head shapes,
// Eq. 7): the per-head table the kernels read and the pure host arithmetic that fills it.
// Plain C++ with no HIP types, so that host tools and CPU tests can include it on its own.
#pragma once

#include <stdint.h>

namespace veda {

// Per-head geometry, one entry per head, in device memory (plan->d_heads).
//
// 128-token tiles are handled as two 64-slot halves: a tile of extents (ot,oh,ow) is cut across
// its slowest axis of extent > 1, so that slots 0-63 are one half and slots 64-127 the other, and
// the two halves are tiles 2o and 2o+1 of an "inner" geometry (grp = 2).  There pt,ph,pw are
// the extents of a half, (ht,hh,hw) the token offset of the second half inside the whole tile,
// and nt,nh,nw still count whole tiles.  For 64-token tiles grp = 1, (ot,oh,ow) = (pt,ph,pw)
// and the offsets are zero.
struct HeadGeom {
    int32_t pt, ph, pw;      // extents of one 64-slot tile (or half tile)
    int32_t nt, nh, nw;      // grid of whole tiles (ceil)
    int32_t n_tiles;         // number of 64-slot tiles: grp*nt*nh*nw
    int32_t tile_off;        // first global tile index of this head
    int64_t score_off;       // first score element of this head (per batch)
    int32_t score_blk_off;   // first 128x128 score block of this head
    int32_t score_blk_dim;   // ceil(n_tiles / 128)
    int32_t ot, oh, ow;      // extents of a whole tile
    int32_t ht, hh, hw;      // token offset of the second half inside a whole tile
    int32_t grp;             // 64-slot tiles per whole tile: 1 or 2
    // Query tiles are processed two at a time by the bf16 attention and heat-map kernels.  Partners
    // are neighbours along pair_ax (0 = t, 1 = h, 2 = w: the axis along which a tile is thinnest, so
    // its neighbour is the closest one and keeps the most similar key tiles); a last layer without a
    // partner is processed alone.  pair_ax = 3: the two halves of a 128-token tile.
    int32_t pair_ax;
    int32_t n_pairs;         // work items (pairs and partnerless tiles) of this head
};

// Extents and tile grid of one head: shape = (p_t,p_h,p_w) of a whole tile, grp = 1 or 2.
// Offsets (tile_off, score_*), pair_ax and n_pairs are left to the caller.
inline void head_extents(HeadGeom& g, const int32_t* shape, int grp, int T, int H, int W) {
    g.ot = shape[0]; g.oh = shape[1]; g.ow = shape[2];
    g.pt = g.ot; g.ph = g.oh; g.pw = g.ow;
    g.ht = g.hh = g.hw = 0;
    g.grp = grp;
    if (grp == 2) {   // cut across the slowest axis of extent > 1 (a product of 128: it is even)
        if (g.ot > 1) { g.pt = g.ot / 2; g.ht = g.pt; }
        else if (g.oh > 1) { g.ph = g.oh / 2; g.hh = g.ph; }
        else { g.pw = g.ow / 2; g.hw = g.pw; }
    }
    g.nt = (T + g.ot - 1) / g.ot;
    g.nh = (H + g.oh - 1) / g.oh;
    g.nw = (W + g.ow - 1) / g.ow;
    g.n_tiles = (int32_t)((int64_t)grp * g.nt * g.nh * g.nw);
}

// Anchor token of 64-slot tile i: the token of its slot 0, from which a kernel finds the tile's
// rows in token order.  Every whole tile starts inside the grid, so its slot 0 is a real token;
// the second half of a 128-token tile may lie wholly outside a ragged grid (no real slot at
// all): such a half is anchored at the first half's token instead, so that the address formed
// from the anchor always stays inside the tensor (the rows fetched for it are masked anyway).
inline int32_t tile_anchor_token(const HeadGeom& g, int32_t i, int T, int H, int W) {
    const int o = g.grp == 2 ? i >> 1 : i, half = g.grp == 2 ? (i & 1) : 0;
    const int tw = o % g.nw, th = (o / g.nw) % g.nh, tt = o / (g.nw * g.nh);
    int64_t t = (int64_t)tt * g.ot + half * g.ht, h = (int64_t)th * g.oh + half * g.hh,
            w = (int64_t)tw * g.ow + half * g.hw;
    if (t >= T || h >= H || w >= W) { t -= half * g.ht; h -= half * g.hh; w -= half * g.hw; }
    return (int32_t)((t * H + h) * W + w);
}

}  // namespace veda
