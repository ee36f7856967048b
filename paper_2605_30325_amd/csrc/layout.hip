// Stage 1 -- head-aware 3D tiling (Sec. 4.2: per-head pi = (p_t,p_h,p_w); Alg. 1 "Tiling";
// Alg. 2 "Tile"): gathers the tokens of every tile into one contiguous 64 x d block, zero
// fills padded slots and records which slots are real.  Pure byte movement, HBM bound:
// one workgroup per (tile, batch) moves 64 rows with 16-byte accesses.
#include "veda_internal.h"

namespace veda {

// out tile = [64][row_bytes]; each thread moves 16-byte chunks.
__global__ __launch_bounds__(256) void layout_token_major_kernel(
    const HeadGeom* __restrict__ heads, const uint8_t* __restrict__ tile_head,
    const char* __restrict__ x, int64_t sb, int64_t sh, int64_t sn, char* __restrict__ out,
    int64_t total_tiles, int row_bytes, int T, int H, int W,
    uint64_t* __restrict__ valid_mask, int32_t* __restrict__ valid_cnt) {
    __shared__ int tok[kTile];
    const int g = blockIdx.x, b = blockIdx.y;
    const int head = tile_head[g];
    const HeadGeom hg = heads[head];
    const int i = g - hg.tile_off;
    if (threadIdx.x < kTile) {
        const int n = slot_token(hg, i, threadIdx.x, T, H, W);
        tok[threadIdx.x] = n;
        const uint64_t m = __ballot(n >= 0);
        if (threadIdx.x == 0 && b == 0) {
            if (valid_mask) valid_mask[g] = m;
            if (valid_cnt) valid_cnt[g] = __popcll(m);
        }
    }
    __syncthreads();
    const int cpr = row_bytes >> 4;  // 16-byte chunks per row
    const char* xb = x + b * sb + head * sh;
    char* ob = out + ((int64_t)b * total_tiles + g) * (int64_t)kTile * row_bytes;
    for (int c = threadIdx.x; c < kTile * cpr; c += 256) {
        const int l = c / cpr, ch = c - l * cpr;
        const int n = tok[l];
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (n >= 0) v = *reinterpret_cast<const uint4*>(xb + (int64_t)n * sn + ch * 16);
        *reinterpret_cast<uint4*>(ob + (int64_t)c * 16) = v;
    }
}

// out tile = [d][64] elements.  The tile is staged in LDS as [64][d] with one pad dword per
// row so that the column gathers spread over the banks.
template <typename E, int D>
__global__ __launch_bounds__(256) void layout_channel_major_kernel(
    const HeadGeom* __restrict__ heads, const uint8_t* __restrict__ tile_head,
    const char* __restrict__ x, int64_t sb, int64_t sh, int64_t sn, char* __restrict__ out,
    int64_t total_tiles, int T, int H, int W,
    uint64_t* __restrict__ valid_mask, int32_t* __restrict__ valid_cnt) {
    constexpr int kRowBytes = D * (int)sizeof(E);
    constexpr int kRowWords = kRowBytes / 4;
    constexpr int kPitch = kRowWords + 1;   // dwords
    constexpr int kCpr = kRowBytes / 16;
    constexpr int kEpc = 16 / (int)sizeof(E);  // elements per 16-byte output chunk
    __shared__ int tok[kTile];
    __shared__ uint32_t stage[kTile * kPitch];
    const int g = blockIdx.x, b = blockIdx.y;
    const int head = tile_head[g];
    const HeadGeom hg = heads[head];
    const int i = g - hg.tile_off;
    if (threadIdx.x < kTile) {
        const int n = slot_token(hg, i, threadIdx.x, T, H, W);
        tok[threadIdx.x] = n;
        const uint64_t m = __ballot(n >= 0);
        if (threadIdx.x == 0 && b == 0) {
            if (valid_mask) valid_mask[g] = m;
            if (valid_cnt) valid_cnt[g] = __popcll(m);
        }
    }
    __syncthreads();
    const char* xb = x + b * sb + head * sh;
    for (int c = threadIdx.x; c < kTile * kCpr; c += 256) {
        const int l = c / kCpr, ch = c - l * kCpr;
        const int n = tok[l];
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (n >= 0) v = *reinterpret_cast<const uint4*>(xb + (int64_t)n * sn + ch * 16);
        uint32_t* s = stage + l * kPitch + ch * 4;
        s[0] = v.x; s[1] = v.y; s[2] = v.z; s[3] = v.w;
    }
    __syncthreads();
    const E* se = reinterpret_cast<const E*>(stage);
    constexpr int kPitchE = kPitch * 4 / (int)sizeof(E);
    constexpr int kChunksPerChannel = kTile / kEpc;
    char* ob = out + ((int64_t)b * total_tiles + g) * (int64_t)kTile * kRowBytes;
    for (int oc = threadIdx.x; oc < D * kChunksPerChannel; oc += 256) {
        const int ch = oc / kChunksPerChannel, l0 = (oc - ch * kChunksPerChannel) * kEpc;
        E tmp[kEpc];
#pragma unroll
        for (int j = 0; j < kEpc; ++j) tmp[j] = se[(l0 + j) * kPitchE + ch];
        *reinterpret_cast<uint4*>(ob + (int64_t)oc * 16) = *reinterpret_cast<const uint4*>(tmp);
    }
}

// 128-token tiles: number of real tokens of a whole tile from the masks of its two halves.
__global__ void valid_cnt_pairs_kernel(const uint64_t* __restrict__ mask, int32_t* __restrict__ cnt, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) cnt[i] = __popcll(mask[2 * i]) + __popcll(mask[2 * i + 1]);
}

// Token-major tiling with the TripPool descriptors (Eq. 4: Avg | Max | Min over the tile's real
// tokens, per channel) taken on the way, so the tiled tensor is not read back for them.
// One thread owns 16 bytes of the channel axis of one tile and walks its 64 slots in order:
// the sum is the same slot-ascending fp32 chain the scoring stage uses, so the descriptors are
// bit-identical to the ones it derives from the tiled tensor.  A workgroup holds 256 / (D / kN)
// consecutive global tiles (they may belong to different heads).
// kWrite = false: descriptors (and masks) only, the tiled tensor is not written.
// GRP = 2: 128-token tiles.  `heads`, `tile_head` and total_tiles are then those of the 64-slot
// halves (halves 2g, 2g+1 of whole tile g); a thread walks the 128 slots of a whole tile in order
// (first half, then second half: the oracle's raster slot order), the mask has two words per tile,
// and the tiled output [tile][128][channel] is the two halves back to back.
#pragma clang fp contract(off)
template <typename E, int D, bool kWrite, int GRP>
__global__ __launch_bounds__(256) void layout_stats_kernel(
    const HeadGeom* __restrict__ heads, const uint8_t* __restrict__ tile_head,
    const char* __restrict__ x, int64_t sb, int64_t sh, int64_t sn, char* __restrict__ out,
    float* __restrict__ stats, int64_t total_tiles, int T, int H, int W,
    uint64_t* __restrict__ valid_mask, int32_t* __restrict__ valid_cnt, RecipTable recip) {
    constexpr int kN = Chunk<E>::kN;
    constexpr int kTpt = D / kN;            // threads per tile
    constexpr int kTiles = 256 / kTpt;      // tiles per workgroup
    constexpr int kRowBytes = D * (int)sizeof(E);
    constexpr int kSlots = kTile * GRP;     // slots of a whole tile
    __shared__ int tok[kTiles][kSlots];
    const int64_t whole_tiles = total_tiles / GRP;
    const int64_t g0 = (int64_t)blockIdx.x * kTiles;
    const int b = blockIdx.y;
    for (int e = threadIdx.x; e < kTiles * kSlots; e += 256) {
        const int tl = e / kSlots, l = e % kSlots;
        const int64_t gi = (g0 + tl) * GRP + l / kTile;   // the 64-slot tile this slot belongs to
        int n = -1;
        if (g0 + tl < whole_tiles) {
            const HeadGeom hg = heads[tile_head[gi]];
            n = slot_token(hg, (int)(gi - hg.tile_off), l % kTile, T, H, W);
        }
        tok[tl][l] = n;
    }
    __syncthreads();
    const int tl = threadIdx.x / kTpt, chunk = threadIdx.x % kTpt;
    const int64_t g = g0 + tl;
    if (g >= whole_tiles) return;
    const int head = tile_head[g * GRP];
    const char* xb = x + b * sb + head * sh + chunk * 16;
    const int64_t row = (int64_t)b * whole_tiles + g;
    char* ob = out + row * (int64_t)kSlots * kRowBytes + chunk * 16;
    float sum[kN], mx[kN], mn[kN];
#pragma unroll
    for (int j = 0; j < kN; ++j) { sum[j] = 0.0f; mx[j] = -INFINITY; mn[j] = INFINITY; }
    uint64_t mask[GRP];
#pragma unroll
    for (int w = 0; w < GRP; ++w) {
        mask[w] = 0ull;
#pragma unroll 8
        for (int l = 0; l < kTile; ++l) {
            const int n = tok[tl][w * kTile + l];
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (n >= 0) {
                v = *reinterpret_cast<const uint4*>(xb + (int64_t)n * sn);
                mask[w] |= 1ull << l;
                float f[kN];
                Chunk<E>::unpack(v, f);
#pragma unroll
                for (int j = 0; j < kN; ++j) {
                    sum[j] = sum[j] + f[j];
                    mx[j] = f[j] > mx[j] ? f[j] : mx[j];
                    mn[j] = f[j] < mn[j] ? f[j] : mn[j];
                }
            }
            if (kWrite) *reinterpret_cast<uint4*>(ob + (w * kTile + l) * kRowBytes) = v;
        }
    }
    int cnt = 0;
#pragma unroll
    for (int w = 0; w < GRP; ++w) cnt += __popcll(mask[w]);
    const float inv = recip.v[cnt];
    float* z = stats + row * (3 * D) + chunk * kN;
#pragma unroll
    for (int j = 0; j < kN; ++j) {
        z[j] = sum[j] * inv;
        z[D + j] = mx[j];
        z[2 * D + j] = mn[j];
    }
    if (chunk == 0 && b == 0) {
        if (valid_mask) {
#pragma unroll
            for (int w = 0; w < GRP; ++w) valid_mask[g * GRP + w] = mask[w];
        }
        if (valid_cnt) valid_cnt[g] = cnt;
    }
}

}  // namespace veda

extern "C" veda_status veda_tile_layout(const veda_plan* pl, const void* x, veda_strides sx,
                                        veda_tile_order order, void* x_tiled, uint64_t* valid_mask,
                                        int32_t* valid_cnt, void* stream) {
    using namespace veda;
    if (!pl || !x || !x_tiled) return VEDA_ERR_INVALID_ARG;
    if (order != VEDA_TOKEN_MAJOR && order != VEDA_CHANNEL_MAJOR) return VEDA_ERR_INVALID_ARG;
    const int es = pl->elem_size();
    const int d = pl->prob.head_dim;
    if (sx.n < d || sx.b < 0 || sx.h < 0) return VEDA_ERR_INVALID_ARG;
    if (!aligned16(x) || !aligned16(x_tiled) || (sx.b * es) % 16 || (sx.h * es) % 16 || (sx.n * es) % 16)
        return VEDA_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    // 128-token tiles are laid out as their two 64-slot halves (tiles 2o, 2o+1 of the inner plan)
    const veda_plan* ip = pl->inner ? pl->inner : pl;
    if (pl->inner && valid_cnt && !valid_mask) return VEDA_ERR_INVALID_ARG;   // counts come from the masks
    int32_t* cnt_arg = pl->inner ? nullptr : valid_cnt;
    dim3 grid((unsigned)ip->total_tiles, (unsigned)pl->prob.batch);
    const int64_t sb = sx.b * es, sh = sx.h * es, sn = sx.n * es;
    const int T = pl->prob.T, H = pl->prob.H, W = pl->prob.W;
    if (order == VEDA_TOKEN_MAJOR) {
        hipLaunchKernelGGL(layout_token_major_kernel, grid, dim3(256), 0, st, ip->d_heads, ip->d_tile_head,
                           (const char*)x, sb, sh, sn, (char*)x_tiled, ip->total_tiles, d * es, T, H, W,
                           valid_mask, cnt_arg);
    } else {
#define VEDA_LAUNCH_CM(E, D)                                                                           \
    hipLaunchKernelGGL((layout_channel_major_kernel<E, D>), grid, dim3(256), 0, st, ip->d_heads,        \
                       ip->d_tile_head, (const char*)x, sb, sh, sn, (char*)x_tiled, ip->total_tiles, T, \
                       H, W, valid_mask, cnt_arg)
        if (es == 2 && d == 128) VEDA_LAUNCH_CM(uint16_t, 128);
        else if (es == 2 && d == 64) VEDA_LAUNCH_CM(uint16_t, 64);
        else if (es == 4 && d == 128) VEDA_LAUNCH_CM(uint32_t, 128);
        else VEDA_LAUNCH_CM(uint32_t, 64);
#undef VEDA_LAUNCH_CM
    }
    if (pl->inner && valid_cnt)
        hipLaunchKernelGGL(valid_cnt_pairs_kernel, dim3((unsigned)((pl->total_tiles + 255) / 256)), dim3(256), 0, st,
                           valid_mask, valid_cnt, pl->total_tiles);
    return launch_status("veda_tile_layout");
}

extern "C" veda_status veda_tile_layout_stats(const veda_plan* pl, const void* x, veda_strides sx, void* x_tiled,
                                              uint64_t* valid_mask, int32_t* valid_cnt, float* stats,
                                              void* stream) {
    using namespace veda;
    if (!pl || !x || !stats) return VEDA_ERR_INVALID_ARG;   // x_tiled may be null: descriptors only
    const int es = pl->elem_size();
    const int d = pl->prob.head_dim;
    if (sx.n < d || sx.b < 0 || sx.h < 0) return VEDA_ERR_INVALID_ARG;
    if (!aligned16(x) || (x_tiled && !aligned16(x_tiled)) || !aligned16(stats) || (sx.b * es) % 16 || (sx.h * es) % 16 ||
        (sx.n * es) % 16)
        return VEDA_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    const int64_t sb = sx.b * es, sh = sx.h * es, sn = sx.n * es;
    const int T = pl->prob.T, H = pl->prob.H, W = pl->prob.W;
    RecipTable recip;
    recip.v[0] = 0.0f;
    for (int c = 1; c <= 2 * kTile; ++c) recip.v[c] = 1.0f / (float)c;
    // 128-token tiles (bf16 plans only): the kernel walks the two 64-slot halves of every whole tile
    const veda_plan* ip = pl->inner ? pl->inner : pl;
#define VEDA_LAUNCH_LS2(E, D, WR, GRP)                                                                    \
    hipLaunchKernelGGL((layout_stats_kernel<E, D, WR, GRP>), grid, dim3(256), 0, st, ip->d_heads,         \
                       ip->d_tile_head, (const char*)x, sb, sh, sn, (char*)x_tiled, stats, ip->total_tiles, T, H, W, \
                       valid_mask, valid_cnt, recip)
#define VEDA_LAUNCH_LS(E, D)                                                                              \
    do {                                                                                                  \
        constexpr int tiles = 256 / (D / Chunk<E>::kN);                                                   \
        dim3 grid((unsigned)((pl->total_tiles + tiles - 1) / tiles), (unsigned)pl->prob.batch);           \
        if (pl->inner) {                                                                                  \
            if (x_tiled) VEDA_LAUNCH_LS2(E, D, true, 2);                                                  \
            else VEDA_LAUNCH_LS2(E, D, false, 2);                                                         \
        } else {                                                                                          \
            if (x_tiled) VEDA_LAUNCH_LS2(E, D, true, 1);                                                  \
            else VEDA_LAUNCH_LS2(E, D, false, 1);                                                         \
        }                                                                                                 \
    } while (0)
    if (es == 2 && d == 128) VEDA_LAUNCH_LS(uint16_t, 128);
    else if (es == 2 && d == 64) VEDA_LAUNCH_LS(uint16_t, 64);
    else if (es == 4 && d == 128) VEDA_LAUNCH_LS(uint32_t, 128);
    else VEDA_LAUNCH_LS(uint32_t, 64);
#undef VEDA_LAUNCH_LS
#undef VEDA_LAUNCH_LS2
    return launch_status("veda_tile_layout_stats");
}
