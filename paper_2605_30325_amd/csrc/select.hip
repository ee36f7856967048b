// Stage 3 -- per-query-tile top-k into CSR lists (Sec. 3.1: exactly k ones per mask row;
// Sec. 4.1 / Alg. 2: keep the k highest-scoring key tiles of each query tile).
//
// One 64-lane wavefront owns one score row.  Scores are mapped to order-preserving unsigned
// keys (NaN -> -inf, -0 -> +0).  The k-th largest key is found by a bitwise binary search:
// for each bit from the top, wave-wide ballots count the keys >= candidate.  Keys above the
// threshold are kept, and of the keys equal to it the lowest-indexed ones fill the remainder,
// which is exactly "ties go to the lower tile index".  Ballot prefix counts emit the kept
// columns in ascending order.  No atomics: the output is deterministic.
#include "select_common.h"

namespace veda {

template <int ITEMS>
__global__ __launch_bounds__(256) void select_kernel(const HeadGeom* __restrict__ heads,
                                                     const uint8_t* __restrict__ tile_head,
                                                     const float* __restrict__ scores, SelectArgs args,
                                                     int32_t* __restrict__ row_ptr, int32_t* __restrict__ col_idx,
                                                     int64_t total_tiles, int64_t score_elems, int64_t rows) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const RowInfo ri = locate_row(heads, tile_head, scores, args, row_ptr, col_idx, total_tiles, score_elems, rows,
                                  row, lane);
    select_row<ITEMS>(ri.srow, ri.n, ri.k, ri.dst, lane);
}

__global__ __launch_bounds__(256) void select_sampled_kernel(const HeadGeom* __restrict__ heads,
                                                             const uint8_t* __restrict__ tile_head,
                                                             const float* __restrict__ scores, SelectArgs args,
                                                             SampleArgs sample, int32_t* __restrict__ row_ptr,
                                                             int32_t* __restrict__ col_idx, int64_t total_tiles,
                                                             int64_t score_elems, int64_t rows) {
    __shared__ uint32_t cand_key[4][kCandCap];
    __shared__ int32_t cand_col[4][kCandCap];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t row = (int64_t)blockIdx.x * 4 + w;
    if (row >= rows) return;
    const RowInfo ri = locate_row(heads, tile_head, scores, args, row_ptr, col_idx, total_tiles, score_elems, rows,
                                  row, lane);
    const int n = ri.n, k = ri.k, m = sample.m[ri.head];
    const float* __restrict__ srow = ri.srow;
    bool ok = m > 0 && n >= kSample;
    float pivot = 0.0f;
    if (ok) {
        uint32_t sk[kSample / 64];
#pragma unroll
        for (int e = 0; e < kSample / 64; ++e)
            sk[e] = score_key(srow[(int)(((int64_t)(e * 64 + lane) * n) / kSample)]);
        uint32_t pk = 0;
        for (int bit = 31; bit >= 0; --bit) {
            const uint32_t cand = pk | (1u << bit);
            int cnt = 0;
#pragma unroll
            for (int e = 0; e < kSample / 64; ++e) cnt += __popcll(__ballot(sk[e] >= cand));
            if (cnt >= m) pk = cand;
        }
        pivot = __uint_as_float((pk & 0x80000000u) ? (pk ^ 0x80000000u) : ~pk);   // inverse of score_key
        // A float comparison against -inf would miss NaN scores, which rank as -inf.
        ok = pivot > -INFINITY;
    }
    int m_cand = 0;
    if (ok) {
        const uint64_t below = (1ull << lane) - 1ull;
        const int items = (n + 63) / 64;
#pragma unroll 4
        for (int t = 0; t < items; ++t) {
            const int j = t * 64 + lane;
            const float sv = j < n ? srow[j] : -INFINITY;
            const bool c = sv >= pivot;
            const uint64_t cb = __ballot(c);
            const int pos = m_cand + __popcll(cb & below);
            if (c && pos < kCandCap) {
                cand_key[w][pos] = score_key(sv);
                cand_col[w][pos] = j;
            }
            m_cand += __popcll(cb);
        }
        ok = m_cand >= k && m_cand <= kCandCap;
    }
    if (!ok) {
        select_row<0>(srow, n, k, ri.dst, lane);
        return;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    if (m_cand <= 256) select_candidates<4>(cand_key[w], cand_col[w], m_cand, k, ri.dst, lane);
    else if (m_cand <= 512) select_candidates<8>(cand_key[w], cand_col[w], m_cand, k, ri.dst, lane);
    else select_candidates<16>(cand_key[w], cand_col[w], m_cand, k, ri.dst, lane);
}

// Per-head tables of a selection call.  Returns false on a bad budget or a list too long for
// the int32 row pointers.  sampled: every head has long rows and a keep budget small enough that
// the expected candidate count (n*m/256, m = pivot rank) stays well inside the candidate list.
bool select_setup(const veda_plan* pl, const int32_t* k_per_head, SelectArgs& args, SampleArgs& sample,
                  bool& sampled, int& max_tiles) {
    int64_t off = 0;
    max_tiles = 0;
    sampled = true;
    for (int h = 0; h < pl->prob.heads; ++h) {
        const int n = pl->heads[h].n_tiles;
        if (k_per_head[h] < 1 || k_per_head[h] > n) return false;
        args.k[h] = k_per_head[h];
        args.col_off[h] = off;
        off += (int64_t)n * k_per_head[h];
        max_tiles = n > max_tiles ? n : max_tiles;
        const double f = k_per_head[h] / (double)n;
        const int m = (int)std::ceil(kSample * f + 3.5 * std::sqrt(kSample * f * (1.0 - f)) + 1.0);
        sample.m[h] = m;
        if (n < 1024 || m > kSample || (double)n * m / kSample * 1.3 > kCandCap) sampled = false;
    }
    args.nnz_per_batch = off;
    return true;
}

veda_status launch_select(const veda_plan* pl, const float* scores, const int32_t* k_per_head, int32_t* row_ptr,
                          int32_t* col_idx, hipStream_t s) {
    SelectArgs args;
    SampleArgs sample;
    bool sampled;
    int max_tiles;
    if (!select_setup(pl, k_per_head, args, sample, sampled, max_tiles)) return VEDA_ERR_INVALID_ARG;
    if (args.nnz_per_batch * pl->prob.batch >= ((int64_t)1 << 31)) return VEDA_ERR_UNSUPPORTED;  // row_ptr is int32
    const int64_t rows = pl->total_tiles * pl->prob.batch;
    dim3 grid((unsigned)((rows + 3) / 4)), block(256);
    if (sampled) {
        hipLaunchKernelGGL(select_sampled_kernel, grid, block, 0, s, pl->d_heads, pl->d_tile_head, scores, args,
                           sample, row_ptr, col_idx, pl->total_tiles, pl->score_elems, rows);
        return launch_status("select_sampled_kernel");
    }
    // Otherwise the smallest register-resident instantiation that fits the longest row, else the
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

}  // namespace veda

extern "C" veda_status veda_tile_select(const veda_plan* pl, const float* scores, const int32_t* k_per_head,
                                        int32_t* row_ptr, int32_t* col_idx, void* stream) {
    if (!pl || !scores || !k_per_head || !row_ptr || !col_idx) return VEDA_ERR_INVALID_ARG;
    return veda::launch_select(pl, scores, k_per_head, row_ptr, col_idx, (hipStream_t)stream);
}
