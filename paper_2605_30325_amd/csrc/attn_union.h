// The union of the kept lists of a workgroup's query tiles as a step table in LDS (Sec. 4.3: a
// workgroup visits only kept key tiles; here several query tiles share one visit).
//
// A workgroup that owns N query tiles visits every key tile kept by at least one of them once.
// Walking the N lists with scalar loads inside the main loop costs a wave a scalar-memory
// round trip per step, and while one is in flight the compiler can only wait for LDS operand
// reads by waiting for everything.  So the walk is done up front, by all threads at once:
//   1. every list is turned into a bitmap over the head's key tiles (LDS atomics);
//   2. a block-wide prefix sum over the population counts of the OR of the bitmaps numbers the
//      kept key tiles in ascending order: these are the steps;
//   3. the table of steps is filled kUnionChunk entries at a time, one entry per thread: the
//      thread finds the bitmap word of its step by binary search in the prefix sums, the bit by
//      counting, and stores (key tile, who keeps it, the tile's anchor token, its validity mask).
// The main loop reads one 16-byte entry per step from LDS, steps ahead.  The table is a ring of
// two chunks; a chunk is refilled when the loop has left it.
// Lists may come in any order (the union is visited in ascending order regardless) and must not
// name a tile twice in a row of the CSR (the attention entry points' contract).
#pragma once

#include "attn_common.h"

namespace veda {

constexpr int kUnionMaxWords = 512;                 // bitmap words: list entries name at most 16384 different tiles
constexpr int kUnionMaxTiles = kUnionMaxWords * 32;

// x: key tile | keeper bits << 16 (0 = past the last step); y: anchor token; z, w: validity mask.
struct __align__(16) UnionEntry { int32_t x, y; uint32_t z, w; };

// kChunk: table entries filled at a time (a power of two); the ring holds two chunks.
template <int N, int kChunk> struct UnionLds {
    static constexpr int kRingEntries = 2 * kChunk;
    UnionEntry tab[kRingEntries];
    uint32_t bm[N][kUnionMaxWords];
    int32_t prefix[kUnionMaxWords];
    int32_t wave_sum[16];
    int32_t total;
};

// Steps 1 and 2.  cols[t], n[t]: list t (global memory).  All threads of the workgroup call it;
// it ends with a barrier.  Returns the number of steps.
// n_tiles: the range of the list entries.
template <int N, int kThreads, int kChunk>
__device__ inline int union_build(UnionLds<N, kChunk>& u, const int32_t* const (&cols)[N], const int (&n)[N], int n_tiles, int tid) {
    static_assert(kUnionMaxWords % kThreads == 0, "whole words per thread");
    constexpr int kPer = kUnionMaxWords / kThreads;
    const int words = (n_tiles + 31) >> 5;
    for (int i = tid; i < N * kUnionMaxWords; i += kThreads) (&u.bm[0][0])[i] = 0u;
    __syncthreads();
#pragma unroll
    for (int t = 0; t < N; ++t)
        for (int i = tid; i < n[t]; i += kThreads) {
            const int j = cols[t][i];
            if ((unsigned)j < (unsigned)n_tiles) atomicOr(&u.bm[t][j >> 5], 1u << (j & 31));
        }
    __syncthreads();
    // exclusive prefix sum of the words' population counts: kPer consecutive words per thread
    int cnt[kPer], mine = 0;
#pragma unroll
    for (int p = 0; p < kPer; ++p) {
        const int w = tid * kPer + p;
        uint32_t all = 0u;
        if (w < words) {
#pragma unroll
            for (int t = 0; t < N; ++t) all |= u.bm[t][w];
        }
        cnt[p] = __popc(all);
        mine += cnt[p];
    }
    int incl = mine;
    const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int up = __shfl_up(incl, d);
        if (lane >= d) incl += up;
    }
    if (lane == 63) u.wave_sum[wave] = incl;
    __syncthreads();
    int off = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) {
        const int s = u.wave_sum[w];
        off += w < wave ? s : 0;
        total += s;
    }
    int run = off + incl - mine;
#pragma unroll
    for (int p = 0; p < kPer; ++p) {
        u.prefix[tid * kPer + p] = run;
        run += cnt[p];
    }
    if (tid == 0) u.total = total;
    __syncthreads();
    return total;
}

// Step 3: entries [first, first + kChunk) of the step sequence into their places in the ring
// (entry s lives at s % (2 kChunk)).  No barrier inside: the caller separates it from the readers
// of these places.  total: number of steps.  kGrouped: the lists name whole 128-token tiles and
// every kept one makes two steps, its 64-slot halves 2o and 2o+1 (vmask, n0s are indexed by half),
// kept by all N query tiles alike.
template <int N, int kThreads, int kChunk, bool kGrouped>
__device__ inline void union_fill(UnionLds<N, kChunk>& u, int first, int total, int n_tiles, const uint64_t* __restrict__ vmask,
                                  const int32_t* __restrict__ n0s, int tid) {
    const int words = (n_tiles + 31) >> 5;
    for (int i = tid; i < kChunk; i += kThreads) {
        const int step = first + i;
        const int s = kGrouped ? step >> 1 : step;   // position in the ascending union
        UnionEntry e = {0, 0, 0u, 0u};
        if (step < total) {
            int lo = 0, hi = words - 1;   // the last word whose prefix is <= s holds step s
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (u.prefix[mid] <= s) lo = mid; else hi = mid - 1;
            }
            uint32_t b[N], all = 0u;
#pragma unroll
            for (int t = 0; t < N; ++t) {
                b[t] = u.bm[t][lo];
                all |= b[t];
            }
            for (int k = s - u.prefix[lo]; k > 0; --k) all &= all - 1u;
            if (all == 0u) all = 1u;   // cannot happen for s < total; keeps the index below in range regardless
            const int bit = __ffs((int)all) - 1;
            const int j = kGrouped ? 2 * (lo * 32 + bit) + (step & 1) : lo * 32 + bit;
            int fl = 0;
#pragma unroll
            for (int t = 0; t < N; ++t) fl |= (int)((b[t] >> bit) & 1u) << t;
            if (kGrouped) fl = (1 << N) - 1;
            const uint64_t vm = vmask[j];
            e.x = j | (fl << 16);
            e.y = n0s[j];
            e.z = (uint32_t)vm;
            e.w = (uint32_t)(vm >> 32);
        }
        u.tab[step & (2 * kChunk - 1)] = e;
    }
}

// One step as the main loop holds it (all fields wave-uniform, in scalar registers).
struct UnionStep {
    int j;         // key tile (head-local)
    int fl;        // bit t: query tile t of the workgroup keeps it; 0 = past the end
    uint64_t vm;   // validity mask of key tile j
    int n0;        // token index of its slot 0
};

typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef const __attribute__((address_space(3))) i32x4* lds_i32x4_ptr;

// The raw entry of step s (the same address in every lane), and its fields once it has arrived.
template <int kChunk> __device__ __forceinline__ i32x4 union_read(uint32_t tab_lds, int s) {
    return *(lds_i32x4_ptr)(uintptr_t)(tab_lds + (uint32_t)(s & (2 * kChunk - 1)) * 16u);
}
__device__ __forceinline__ UnionStep union_step(const i32x4& raw) {
    UnionStep e;
    const int x = __builtin_amdgcn_readfirstlane(raw[0]);
    e.j = x & 0xffff;
    e.fl = x >> 16;
    e.n0 = __builtin_amdgcn_readfirstlane(raw[1]);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane(raw[2]), hi = (uint32_t)__builtin_amdgcn_readfirstlane(raw[3]);
    e.vm = (uint64_t)hi << 32 | lo;
    return e;
}

}  // namespace veda
