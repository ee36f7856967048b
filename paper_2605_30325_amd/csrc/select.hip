// Stage 3 -- per-query-tile top-k into CSR lists (Sec. 3.1: exactly k ones per mask row;
// Sec. 4.1 / Alg. 2: keep the k highest-scoring key tiles of each query tile).
//
// One 64-lane wavefront owns one score row.  Scores are mapped to order-preserving unsigned
// keys (NaN -> -inf, -0 -> +0).  The k-th largest key is found by a bitwise binary search:
// for each bit from the top, wave-wide ballots count the keys >= candidate.  Keys above the
// threshold are kept, and of the keys equal to it the lowest-indexed ones fill the remainder,
// which is exactly "ties go to the lower tile index".  Ballot prefix counts emit the kept
// columns in ascending order.  No atomics: the output is deterministic.
#include "veda_internal.h"

namespace veda {

struct SelectArgs {
    int32_t k[kMaxHeads];          // kept tiles per row, per head
    int64_t col_off[kMaxHeads];    // first col_idx element of each head (within one batch)
    int64_t nnz_per_batch;
};

__device__ inline uint32_t score_key(float s) {
    s = (s != s) ? -INFINITY : s + 0.0f;
    const uint32_t u = __float_as_uint(s);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// ITEMS > 0: the row (n <= 64*ITEMS columns) lives in registers.  ITEMS == 0: any length,
// re-read from memory (L2) on every pass.
template <int ITEMS>
__global__ __launch_bounds__(256) void select_kernel(const HeadGeom* __restrict__ heads,
                                                     const uint8_t* __restrict__ tile_head,
                                                     const float* __restrict__ scores, SelectArgs args,
                                                     int32_t* __restrict__ row_ptr, int32_t* __restrict__ col_idx,
                                                     int64_t total_tiles, int64_t score_elems, int64_t rows) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int64_t b = row / total_tiles;
    const int64_t g = row - b * total_tiles;
    const int head = tile_head[g];
    const HeadGeom hg = heads[head];
    const int n = hg.n_tiles;
    const int k = args.k[head];
    const int i = (int)(g - hg.tile_off);
    const int64_t out_off = b * args.nnz_per_batch + args.col_off[head] + (int64_t)i * k;
    if (lane == 0) {
        row_ptr[row] = (int32_t)out_off;
        if (row == rows - 1) row_ptr[rows] = (int32_t)(out_off + k);
    }
    const float* srow = scores + b * score_elems + hg.score_off + (int64_t)i * n;

    uint32_t key[ITEMS > 0 ? ITEMS : 1];
    if (ITEMS > 0) {
#pragma unroll
        for (int t = 0; t < ITEMS; ++t) {
            const int j = t * 64 + lane;
            key[t] = j < n ? score_key(srow[j]) : 0u;   // 0 is below every real key
        }
    }
    const int items = ITEMS > 0 ? ITEMS : (n + 63) / 64;
    auto get = [&](int t) -> uint32_t {
        if (ITEMS > 0) return key[t];
        const int j = t * 64 + lane;
        return j < n ? score_key(srow[j]) : 0u;
    };

    uint32_t thr = 0;
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t cand = thr | (1u << bit);
        int cnt = 0;
        if (ITEMS > 0) {
#pragma unroll
            for (int t = 0; t < ITEMS; ++t) cnt += __popcll(__ballot(key[t] >= cand));
        } else {
            for (int t = 0; t < items; ++t) cnt += __popcll(__ballot(get(t) >= cand));
        }
        if (cnt >= k) thr = cand;
    }
    // thr is now the k-th largest key of the row.
    int n_gt = 0;
    if (ITEMS > 0) {
#pragma unroll
        for (int t = 0; t < ITEMS; ++t) n_gt += __popcll(__ballot(key[t] > thr));
    } else {
        for (int t = 0; t < items; ++t) n_gt += __popcll(__ballot(get(t) > thr));
    }
    int ties_left = k - n_gt;   // >= 1
    int written = 0;
    const uint64_t below = (1ull << lane) - 1ull;
    int32_t* dst = col_idx + out_off;
    auto emit = [&](int t, uint32_t kv) {
        const int j = t * 64 + lane;
        const bool gt = kv > thr;
        const bool eq = (kv == thr) && j < n;
        const uint64_t eq_b = __ballot(eq);
        const bool take = gt || (eq && __popcll(eq_b & below) < ties_left);
        const uint64_t take_b = __ballot(take);
        if (take) dst[written + __popcll(take_b & below)] = j;
        written += __popcll(take_b);
        const int eq_n = __popcll(eq_b);
        ties_left = ties_left > eq_n ? ties_left - eq_n : 0;
    };
    if (ITEMS > 0) {
#pragma unroll
        for (int t = 0; t < ITEMS; ++t) emit(t, key[t]);
    } else {
        for (int t = 0; t < items; ++t) emit(t, get(t));
    }
}

}  // namespace veda

extern "C" veda_status veda_tile_select(const veda_plan* pl, const float* scores, const int32_t* k_per_head,
                                        int32_t* row_ptr, int32_t* col_idx, void* stream) {
    using namespace veda;
    if (!pl || !scores || !k_per_head || !row_ptr || !col_idx) return VEDA_ERR_INVALID_ARG;
    SelectArgs args;
    int64_t off = 0;
    int max_tiles = 0;
    for (int h = 0; h < pl->prob.heads; ++h) {
        const int n = pl->heads[h].n_tiles;
        if (k_per_head[h] < 1 || k_per_head[h] > n) return VEDA_ERR_INVALID_ARG;
        args.k[h] = k_per_head[h];
        args.col_off[h] = off;
        off += (int64_t)n * k_per_head[h];
        max_tiles = n > max_tiles ? n : max_tiles;
    }
    args.nnz_per_batch = off;
    if (off * pl->prob.batch >= ((int64_t)1 << 31)) return VEDA_ERR_UNSUPPORTED;  // row_ptr is int32
    const int64_t rows = pl->total_tiles * pl->prob.batch;
    dim3 grid((unsigned)((rows + 3) / 4)), block(256);
    hipStream_t s = (hipStream_t)stream;
    // The smallest register-resident instantiation that fits the longest row, else the
    // memory-resident one.
    int items = 0;
    for (int cand : {4, 16, 32, 64})
        if (max_tiles <= 64 * cand) { items = cand; break; }
#define VEDA_LAUNCH_SEL(I)                                                                                  \
    hipLaunchKernelGGL((select_kernel<I>), grid, block, 0, s, pl->d_heads, pl->d_tile_head, scores, args,   \
                       row_ptr, col_idx, pl->total_tiles, pl->score_elems, rows)
    switch (items) {
        case 4: VEDA_LAUNCH_SEL(4); break;
        case 16: VEDA_LAUNCH_SEL(16); break;
        case 32: VEDA_LAUNCH_SEL(32); break;
        case 64: VEDA_LAUNCH_SEL(64); break;
        default: VEDA_LAUNCH_SEL(0); break;
    }
#undef VEDA_LAUNCH_SEL
    return launch_status("select_kernel");
}
