// Stage 3 -- per-query-tile top-k into CSR lists (Sec. 3.1: exactly k ones per mask row;
// Sec. 4.1 / Alg. 2: keep the k highest-scoring key tiles of each query tile).
//
// One 64-lane wavefront owns one score row.  Scores are mapped to order-preserving unsigned
// keys (NaN -> -inf, -0 -> +0).  The k-th largest key is found by a bitwise binary search:
// for each bit from the top, wave-wide ballots count the keys >= candidate.  Keys above the
// threshold are kept, and of the keys equal to it the lowest-indexed ones fill the remainder,
// which is exactly "ties go to the lower tile index".  Ballot prefix counts emit the kept
// columns in ascending order.  No atomics: the output is deterministic.
#include <cmath>

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

// Exact selection on one row by one wavefront.  ITEMS > 0: the row (n <= 64*ITEMS columns)
// lives in registers.  ITEMS == 0: any length, re-read from memory (L2) on every pass.
template <int ITEMS>
__device__ __forceinline__ void select_row(const float* __restrict__ srow, int n, int k, int32_t* __restrict__ dst,
                                           int lane) {
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

// Everything a wavefront needs to know about its row.
struct RowInfo {
    const float* srow;
    int32_t* dst;
    int n, k, head;
};

__device__ __forceinline__ RowInfo locate_row(const HeadGeom* __restrict__ heads, const uint8_t* __restrict__ tile_head,
                                              const float* __restrict__ scores, const SelectArgs& args,
                                              int32_t* __restrict__ row_ptr, int32_t* __restrict__ col_idx,
                                              int64_t total_tiles, int64_t score_elems, int64_t rows, int64_t row,
                                              int lane) {
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
    return RowInfo{scores + b * score_elems + hg.score_off + (int64_t)i * n, col_idx + out_off, n, k, head};
}

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

// Long rows with a small keep budget: a pivot from a sample shrinks the row to a short
// candidate list before the exact search.
//   1. 256 columns spread evenly over the row are sampled; the pivot p is the sample's m-th
//      largest value (m per head from the host, a few standard deviations above 256*k/n, so
//      that the row almost surely has at least k values >= p, and not many more).
//   2. One pass over the row copies (key, column) of every value >= p to LDS, in column order.
//   3. If between k and 1024 candidates came out, the k-th largest row value is the k-th
//      largest candidate: the same bitwise search and tie rule run on the candidates only.
//      Otherwise the row is handled by the plain search over the whole row.
// The result is the exact top-k set whichever way is taken.
constexpr int kCandCap = 1024;
constexpr int kSample = 256;

template <int NI>
__device__ __forceinline__ void select_candidates(const uint32_t* ckey, const int32_t* ccol, int m_cand, int k,
                                                  int32_t* __restrict__ dst, int lane) {
    uint32_t key[NI];
#pragma unroll
    for (int t = 0; t < NI; ++t) {
        const int c = t * 64 + lane;
        key[t] = c < m_cand ? ckey[c] : 0u;
    }
    uint32_t thr = 0;
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t cand = thr | (1u << bit);
        int cnt = 0;
#pragma unroll
        for (int t = 0; t < NI; ++t) cnt += __popcll(__ballot(key[t] >= cand));
        if (cnt >= k) thr = cand;
    }
    int n_gt = 0;
#pragma unroll
    for (int t = 0; t < NI; ++t) n_gt += __popcll(__ballot(key[t] > thr));
    int ties_left = k - n_gt;
    int written = 0;
    const uint64_t below = (1ull << lane) - 1ull;
#pragma unroll
    for (int t = 0; t < NI; ++t) {
        const int c = t * 64 + lane;
        const bool gt = key[t] > thr;
        const bool eq = (key[t] == thr) && c < m_cand;
        const uint64_t eq_b = __ballot(eq);
        const bool take = gt || (eq && __popcll(eq_b & below) < ties_left);
        const uint64_t take_b = __ballot(take);
        if (take) dst[written + __popcll(take_b & below)] = ccol[c];
        written += __popcll(take_b);
        const int eq_n = __popcll(eq_b);
        ties_left = ties_left > eq_n ? ties_left - eq_n : 0;
    }
}

struct SampleArgs { int32_t m[kMaxHeads]; };   // pivot rank in the sample per head; 0 = no sampling

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
    // Sampled selection when every head has long rows and a keep budget small enough that the
    // expected candidate count (n*m/256, m = pivot rank) stays well inside the LDS list.
    SampleArgs sample;
    bool sampled = true;
    for (int h = 0; h < pl->prob.heads; ++h) {
        const double n = pl->heads[h].n_tiles, f = k_per_head[h] / n;
        const int m = (int)std::ceil(kSample * f + 3.5 * std::sqrt(kSample * f * (1.0 - f)) + 1.0);
        sample.m[h] = m;
        if (n < 1024 || m > kSample || n * m / kSample * 1.3 > kCandCap) sampled = false;
    }
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
