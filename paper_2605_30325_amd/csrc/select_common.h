// Pieces of the top-k selection shared by the stage-3 kernels (select.hip) and the fused
// score+select route (fused.hip): order-preserving keys, the exact one-wavefront searches and
// the row bookkeeping.  Not part of the public ABI.
#pragma once

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

// Candidate c (in column order) is stored at index at(c) of ckey / ccol; kRawScores: ckey holds
// the scores' bit patterns rather than their keys.
template <int NI, bool kRawScores, typename At>
__device__ __forceinline__ void select_candidates(const uint32_t* ckey, const int32_t* ccol, int m_cand, int k,
                                                  int32_t* __restrict__ dst, int lane, At at) {
    uint32_t key[NI];
#pragma unroll
    for (int t = 0; t < NI; ++t) {
        const int c = t * 64 + lane;
        const uint32_t raw = c < m_cand ? ckey[at(c)] : 0u;
        key[t] = c < m_cand ? (kRawScores ? score_key(__uint_as_float(raw)) : raw) : 0u;
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
        if (take) dst[written + __popcll(take_b & below)] = ccol[at(c)];
        written += __popcll(take_b);
        const int eq_n = __popcll(eq_b);
        ties_left = ties_left > eq_n ? ties_left - eq_n : 0;
    }
}

template <int NI>
__device__ __forceinline__ void select_candidates(const uint32_t* ckey, const int32_t* ccol, int m_cand, int k,
                                                  int32_t* __restrict__ dst, int lane) {
    select_candidates<NI, false>(ckey, ccol, m_cand, k, dst, lane, [](int c) { return c; });
}

struct SampleArgs { int32_t m[kMaxHeads]; };   // pivot rank in the sample per head; 0 = no sampling

// Host side of stage 3 (select.hip).  select_setup fills the per-head tables and decides whether
// every head qualifies for the sampled-pivot route; launch_select enqueues stage 3 on scores.
bool select_setup(const veda_plan* pl, const int32_t* k_per_head, SelectArgs& args, SampleArgs& sample,
                  bool& sampled, int& max_tiles);
veda_status launch_select(const veda_plan* pl, const float* scores, const int32_t* k_per_head, int32_t* row_ptr,
                          int32_t* col_idx, hipStream_t s);

}  // namespace veda
