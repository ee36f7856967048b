// Shared declarations of the library's translation units: the plan object, the per-head
// geometry table the kernels read, and small host helpers.  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "geometry.h"
#include "veda.h"

namespace veda {

constexpr int kTile = 64;        // B: tokens per tile
constexpr int kMaxHeads = 128;   // per-call tables passed by value are sized for this
constexpr int kXcd = 8;          // accelerator dies (each with its own L2); workgroup i runs on die i % 8

#if defined(__HIPCC__)
struct RecipTable { float v[2 * kTile + 1]; };  // v[c] = 1.0f / (float)c, computed on the host

template <typename E> struct Chunk;
template <> struct Chunk<uint16_t> {  // bf16: 8 channels per 16 bytes
    static constexpr int kN = 8;
    __device__ static void unpack(const uint4& u, float* f) {
        const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            f[2 * j] = __uint_as_float(w[j] << 16);
            f[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
        }
    }
};
template <> struct Chunk<uint32_t> {  // fp32: 4 channels per 16 bytes
    static constexpr int kN = 4;
    __device__ static void unpack(const uint4& u, float* f) {
        f[0] = __uint_as_float(u.x); f[1] = __uint_as_float(u.y);
        f[2] = __uint_as_float(u.z); f[3] = __uint_as_float(u.w);
    }
};

// Token index of slot l of tile i of a head, or -1 for a padded slot.  Tiles and slots are
// both raster order with time slowest (App. A.5: temporal neighbours p_h*p_w slots apart).
__device__ inline int slot_token(const HeadGeom& g, int i, int l, int T, int H, int W) {
    const int o = g.grp == 2 ? i >> 1 : i, half = g.grp == 2 ? (i & 1) : 0;
    const int tw = o % g.nw, th = (o / g.nw) % g.nh, tt = o / (g.nw * g.nh);
    const int lw = l % g.pw, lh = (l / g.pw) % g.ph, lt = l / (g.pw * g.ph);
    const int t = tt * g.ot + half * g.ht + lt, h = th * g.oh + half * g.hh + lh, w = tw * g.ow + half * g.hw + lw;
    return (t < T && h < H && w < W) ? (t * H + h) * W + w : -1;
}
#endif

}  // namespace veda

struct veda_plan {
    veda_problem prob;                  // tile_shape pointer is not kept valid; see shapes
    std::vector<int32_t> shapes;        // [heads][3]
    std::vector<veda::HeadGeom> heads;  // host copy
    int64_t total_tiles = 0;
    int64_t score_elems = 0;
    int64_t score_blocks = 0;
    int device = -1;
    bool exact_logit_scale = false;     // VEDA_OPT_EXACT_LOGIT_SCALE (bf16 attention kernel)
    bool attn_list_walk = false;        // VEDA_OPT_ATTN_LIST_WALK (attention kernels)
    // Where the fixed-order fp32 chains of stage 2 run: chain_probe is what probe_chain_unit found on
    // this plan's device, chain_option what VEDA_OPT_FP32_CHAIN_UNIT asks for (0 = as probed).
    int chain_probe = VEDA_CHAINS_MATRIX, chain_option = 0;
    int chain_unit() const { return chain_option ? chain_option : chain_probe; }
    // 128-token tiles: this plan describes the whole tiles (stages 2 and 3 work on them); `inner`
    // describes their 64-slot halves, in the order 2o, 2o+1 (stages 1 and 4 work on those).
    veda_plan* inner = nullptr;
    veda::HeadGeom* d_heads = nullptr;  // device [heads]
    uint8_t* d_tile_head = nullptr;     // device [total_tiles]: head of each global tile
    int32_t* d_tile_n0 = nullptr;       // device [total_tiles]: anchor token of each tile (tile_anchor_token: always a real token)
    // Blocks of 64 consecutive tiles that never straddle two heads (the projection kernel's work
    // items): d_row_blk[x] = head << 24 | block index inside the head.
    int32_t* d_row_blk = nullptr;       // device [row_blocks]
    int64_t row_blocks = 0;
    // Work split of the attention launch: die x takes the x-th eighth of every head's query
    // tiles, heads in order, so all dies work on the same head at the same time.
    // d_xcd_cum[x*(heads+1) + h] = number of query tiles die x owns in heads < h.
    int32_t* d_xcd_cum = nullptr;       // device [8][heads+1]
    int32_t xcd_max_tiles = 0;          // max over dies of the die's total
    // The same split over the pair work items of the heads (HeadGeom::n_pairs), for the pair kernels.
    int32_t* d_xcd_cum_pair = nullptr;  // device [8][heads+1]
    int32_t xcd_max_pairs = 0;
    int elem_size() const { return prob.dtype == VEDA_BF16 ? 2 : 4; }
    int64_t tokens() const { return (int64_t)prob.T * prob.H * prob.W; }
};

namespace veda {

void set_last_error(const std::string& s);
veda_status hip_fail(hipError_t e, const char* what);
// chains_vector.hip: VEDA_CHAINS_MATRIX or VEDA_CHAINS_VECTOR for the fp32 chains of stage 2 on GPU `device` (the current one).
veda_status probe_chain_unit(int device, int* unit);

#define VEDA_HIP_TRY(expr)                                              \
    do {                                                                \
        hipError_t e__ = (expr);                                        \
        if (e__ != hipSuccess) return ::veda::hip_fail(e__, #expr);     \
    } while (0)

// After a kernel launch: map a launch error to VEDA_ERR_HIP without synchronising.
inline veda_status launch_status(const char* what) {
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? VEDA_OK : hip_fail(e, what);
}

// Device address of the fixed scratch array of the no-allocation entry point (fused.hip) on GPU
// `device`, which must be current; resolved once per device.
veda_status noalloc_scratch(int device, void** out);

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace veda
