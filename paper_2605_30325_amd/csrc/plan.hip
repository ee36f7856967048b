// Plan object: validates a problem, derives every head's ceil-padded tile grid (Sec. 3.1 tiles
// of size B; Sec. 4.2 per-head shapes from Omega, Eq. 7) and uploads the per-head table.
#include <algorithm>
#include <new>

#include "veda_internal.h"

namespace veda {

static thread_local std::string g_last_error;

void set_last_error(const std::string& s) { g_last_error = s; }

veda_status hip_fail(hipError_t e, const char* what) {
    g_last_error = std::string(what) + ": " + hipGetErrorString(e);
    return VEDA_ERR_HIP;
}

}  // namespace veda

using veda::HeadGeom;

extern "C" {

const char* veda_status_string(veda_status s) {
    switch (s) {
        case VEDA_OK: return "ok";
        case VEDA_ERR_INVALID_ARG: return "invalid argument";
        case VEDA_ERR_UNSUPPORTED: return "unsupported configuration";
        case VEDA_ERR_WORKSPACE: return "workspace too small";
        case VEDA_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

const char* veda_last_error(void) { return veda::g_last_error.c_str(); }

// Builds one plan object.  grp = 1: tiles of prob.tile_tokens tokens with the given extents.
// grp = 2: the 64-slot halves of 128-token tiles whose extents are `shapes` (halves 2o, 2o+1).
static veda_status build_plan(const veda_problem* p, const int32_t* shapes, int grp, veda_plan** out) {
    veda_plan* pl = new (std::nothrow) veda_plan();
    if (!pl) return VEDA_ERR_INVALID_ARG;
    pl->prob = *p;
    pl->shapes.assign(shapes, shapes + 3 * p->heads);
    pl->prob.tile_shape = pl->shapes.data();
    pl->heads.resize(p->heads);
    int64_t toff = 0, soff = 0, boff = 0;
    for (int h = 0; h < p->heads; ++h) {
        HeadGeom& g = pl->heads[h];
        veda::head_extents(g, &pl->shapes[3 * h], grp, p->T, p->H, p->W);
        const int64_t n = g.n_tiles;
        if (grp == 2) {
            g.pair_ax = 3;
            g.n_pairs = (int32_t)(n / 2);
        } else {
            // Expected K/V loads per kept tile pair if partners are taken along axis a: neighbours
            // along the thinnest extent share the most (about 0.60 of the loads of two separate
            // walks against 0.68 along a thicker one, measured on the synthetic workloads), and an
            // odd tile count leaves 1/cnt of the tiles without a partner (no sharing, half a
            // workgroup idle).  Smallest estimate wins; ties go to w, then h.
            const int ext[3] = {g.pt, g.ph, g.pw}, cnt[3] = {g.nt, g.nh, g.nw};
            const int thin = std::min(ext[0], std::min(ext[1], ext[2]));
            int ax = -1;
            double best = 0.0;
            for (int a = 2; a >= 0; --a) {
                if (cnt[a] < 2) continue;
                const double alone = cnt[a] % 2 ? 1.0 / cnt[a] : 0.0;
                const double cost = (1.0 - alone) * (ext[a] == thin ? 0.60 : 0.68) + alone;
                if (ax < 0 || cost < best - 1e-12) { ax = a; best = cost; }
            }
            g.pair_ax = ax < 0 ? 2 : ax;
            int64_t items = 1;
            for (int a = 0; a < 3; ++a) items *= a == g.pair_ax ? (cnt[a] + 1) / 2 : cnt[a];
            g.n_pairs = (int32_t)items;
        }
        g.tile_off = (int32_t)toff;
        g.score_off = soff;
        g.score_blk_dim = (int32_t)((n + 127) / 128);
        g.score_blk_off = (int32_t)boff;
        toff += n;
        soff += n * n;
        boff += (int64_t)g.score_blk_dim * g.score_blk_dim;
    }
    pl->total_tiles = toff;
    pl->score_elems = soff;
    pl->score_blocks = boff;
    if (toff * p->batch >= ((int64_t)1 << 31) - 1 || boff >= ((int64_t)1 << 31)) {
        delete pl;
        return VEDA_ERR_UNSUPPORTED;
    }

    std::vector<uint8_t> tile_head((size_t)toff);
    for (int h = 0; h < p->heads; ++h)
        for (int32_t i = 0; i < pl->heads[h].n_tiles; ++i) tile_head[(size_t)pl->heads[h].tile_off + i] = (uint8_t)h;

    // anchor token of every tile: what a kernel needs to find a tile's rows in token order
    std::vector<int32_t> tile_n0((size_t)toff);
    for (int h = 0; h < p->heads; ++h) {
        const HeadGeom& g = pl->heads[h];
        for (int32_t i = 0; i < g.n_tiles; ++i) {
            const int32_t n0 = veda::tile_anchor_token(g, i, p->T, p->H, p->W);
            if (n0 < 0 || n0 >= (int64_t)p->T * p->H * p->W) {   // would send a kernel outside the tensor
                delete pl;
                veda::set_last_error("veda_plan_create: tile anchor outside the grid");
                return VEDA_ERR_INVALID_ARG;
            }
            tile_n0[(size_t)g.tile_off + i] = n0;
        }
    }

    std::vector<int32_t> row_blk;
    for (int h = 0; h < p->heads; ++h)
        for (int32_t i = 0; i < (pl->heads[h].n_tiles + 63) / 64; ++i) row_blk.push_back((int32_t)((uint32_t)h << 24 | (uint32_t)i));
    pl->row_blocks = (int64_t)row_blk.size();

    // unit = 1: query tiles; unit = 2: pairs of adjacent query tiles
    auto die_split = [&](int unit, int32_t& max_total) {
        std::vector<int32_t> cum((size_t)veda::kXcd * (p->heads + 1), 0);
        for (int x = 0; x < veda::kXcd; ++x) {
            int32_t acc = 0;
            for (int h = 0; h < p->heads; ++h) {
                cum[(size_t)x * (p->heads + 1) + h] = acc;
                const int32_t n = unit == 2 ? pl->heads[h].n_pairs : pl->heads[h].n_tiles;
                acc += n / veda::kXcd + (x < n % veda::kXcd ? 1 : 0);
            }
            cum[(size_t)x * (p->heads + 1) + p->heads] = acc;
            max_total = acc > max_total ? acc : max_total;
        }
        return cum;
    };
    const std::vector<int32_t> xcd_cum = die_split(1, pl->xcd_max_tiles);
    const std::vector<int32_t> xcd_cum_pair = die_split(2, pl->xcd_max_pairs);

    hipError_t e = hipGetDevice(&pl->device);
    if (e == hipSuccess) {
        // set-up call of this device: the no-allocation entry point finds its scratch array resolved
        void* unused = nullptr;
        veda_status ns = veda::noalloc_scratch(pl->device, &unused);
        // ... and knows which unit reproduces the fp32 chains of stage 2
        if (ns == VEDA_OK) ns = veda::probe_chain_unit(pl->device, &pl->chain_probe);
        if (ns != VEDA_OK) {
            delete pl;
            return ns;
        }
    }
    if (e == hipSuccess) e = hipMalloc((void**)&pl->d_heads, sizeof(HeadGeom) * p->heads);
    if (e == hipSuccess) e = hipMalloc((void**)&pl->d_tile_head, tile_head.size());
    if (e == hipSuccess) e = hipMalloc((void**)&pl->d_tile_n0, tile_n0.size() * sizeof(int32_t));
    if (e == hipSuccess)
        e = hipMemcpy(pl->d_tile_n0, tile_n0.data(), tile_n0.size() * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMalloc((void**)&pl->d_xcd_cum, xcd_cum.size() * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc((void**)&pl->d_row_blk, row_blk.size() * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc((void**)&pl->d_xcd_cum_pair, xcd_cum_pair.size() * sizeof(int32_t));
    if (e == hipSuccess)
        e = hipMemcpy(pl->d_xcd_cum_pair, xcd_cum_pair.data(), xcd_cum_pair.size() * sizeof(int32_t),
                      hipMemcpyHostToDevice);
    if (e == hipSuccess)
        e = hipMemcpy(pl->d_row_blk, row_blk.data(), row_blk.size() * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e == hipSuccess)
        e = hipMemcpy(pl->d_xcd_cum, xcd_cum.data(), xcd_cum.size() * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e == hipSuccess)
        e = hipMemcpy(pl->d_heads, pl->heads.data(), sizeof(HeadGeom) * p->heads, hipMemcpyHostToDevice);
    if (e == hipSuccess)
        e = hipMemcpy(pl->d_tile_head, tile_head.data(), tile_head.size(), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        veda_status st = veda::hip_fail(e, "veda_plan_create");
        veda_plan_destroy(pl);
        return st;
    }
    *out = pl;
    return VEDA_OK;
}

veda_status veda_plan_create(const veda_problem* p, veda_plan** out) {
    if (!p || !out || !p->tile_shape) return VEDA_ERR_INVALID_ARG;
    if (p->batch < 1 || p->heads < 1 || p->T < 1 || p->H < 1 || p->W < 1) return VEDA_ERR_INVALID_ARG;
    if (p->dtype != VEDA_F32 && p->dtype != VEDA_BF16) return VEDA_ERR_INVALID_ARG;
    if (p->tile_tokens != veda::kTile && p->tile_tokens != 2 * veda::kTile) return VEDA_ERR_UNSUPPORTED;
    if (p->tile_tokens == 2 * veda::kTile && p->dtype != VEDA_BF16) return VEDA_ERR_UNSUPPORTED;
    if (p->head_dim != 64 && p->head_dim != 128) return VEDA_ERR_UNSUPPORTED;
    if (p->heads > veda::kMaxHeads) return VEDA_ERR_UNSUPPORTED;
    if ((int64_t)p->T * p->H * p->W > (int64_t)1 << 30) return VEDA_ERR_UNSUPPORTED;
    for (int h = 0; h < p->heads; ++h) {
        const int32_t* s = p->tile_shape + 3 * h;
        if (s[0] < 1 || s[1] < 1 || s[2] < 1) return VEDA_ERR_INVALID_ARG;
        if ((int64_t)s[0] * s[1] * s[2] != p->tile_tokens) return VEDA_ERR_INVALID_ARG;
    }
    veda_plan* pl = nullptr;
    veda_status st = build_plan(p, p->tile_shape, 1, &pl);
    if (st != VEDA_OK) return st;
    if (p->tile_tokens == 2 * veda::kTile) {
        st = build_plan(p, p->tile_shape, 2, &pl->inner);
        if (st != VEDA_OK) {
            veda_plan_destroy(pl);
            return st;
        }
    }
    *out = pl;
    return VEDA_OK;
}

void veda_plan_destroy(veda_plan* pl) {
    if (!pl) return;
    veda_plan_destroy(pl->inner);
    if (pl->d_heads) (void)hipFree(pl->d_heads);
    if (pl->d_tile_head) (void)hipFree(pl->d_tile_head);
    if (pl->d_tile_n0) (void)hipFree(pl->d_tile_n0);
    if (pl->d_xcd_cum) (void)hipFree(pl->d_xcd_cum);
    if (pl->d_row_blk) (void)hipFree(pl->d_row_blk);
    if (pl->d_xcd_cum_pair) (void)hipFree(pl->d_xcd_cum_pair);
    delete pl;
}

veda_status veda_plan_set_option(veda_plan* pl, veda_option option, int32_t value) {
    if (!pl) return VEDA_ERR_INVALID_ARG;
    switch (option) {
        case VEDA_OPT_EXACT_LOGIT_SCALE:
            if (value != 0 && value != 1) return VEDA_ERR_INVALID_ARG;
            pl->exact_logit_scale = value != 0;
            return VEDA_OK;
        case VEDA_OPT_ATTN_LIST_WALK:
            if (value != 0 && value != 1) return VEDA_ERR_INVALID_ARG;
            pl->attn_list_walk = value != 0;
            return VEDA_OK;
        case VEDA_OPT_FP32_CHAIN_UNIT:
            if (value != 0 && value != VEDA_CHAINS_MATRIX && value != VEDA_CHAINS_VECTOR) return VEDA_ERR_INVALID_ARG;
            pl->chain_option = value;
            if (pl->inner) pl->inner->chain_option = value;
            return VEDA_OK;
    }
    return VEDA_ERR_INVALID_ARG;
}

int32_t veda_plan_chain_unit(const veda_plan* pl) { return pl ? pl->chain_unit() : -1; }

int32_t veda_plan_tiles(const veda_plan* pl, int32_t head) {
    if (!pl || head < 0 || head >= pl->prob.heads) return -1;
    return pl->heads[head].n_tiles;
}

int64_t veda_plan_tile_offset(const veda_plan* pl, int32_t head) {
    if (!pl || head < 0 || head >= pl->prob.heads) return -1;
    return pl->heads[head].tile_off;
}

int64_t veda_plan_score_offset(const veda_plan* pl, int32_t head) {
    if (!pl || head < 0 || head >= pl->prob.heads) return -1;
    return pl->heads[head].score_off;
}

int64_t veda_plan_total_tiles(const veda_plan* pl) { return pl ? pl->total_tiles : -1; }

int64_t veda_plan_score_elems(const veda_plan* pl) { return pl ? pl->score_elems : -1; }

size_t veda_plan_workspace_bytes(const veda_plan* pl, const veda_mlp* phi_q, const veda_mlp* phi_k) {
    if (!pl || !phi_q || !phi_k) return 0;
    const size_t rows = (size_t)pl->prob.batch * (size_t)pl->total_tiles;
    // descriptors of Q and K, latents, and the hidden layers of the two projections
    const size_t per_row = (size_t)(2 * 3 * pl->prob.head_dim + phi_q->out_dim + phi_k->out_dim) +
                           (size_t)(phi_q->hidden > 0 ? phi_q->hidden : 0) + (size_t)(phi_k->hidden > 0 ? phi_k->hidden : 0);
    return ((rows * per_row * sizeof(float)) + 255) / 256 * 256;
}

}  // extern "C"
