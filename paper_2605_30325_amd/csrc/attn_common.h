// Declarations shared by the attention kernels: launch arguments, vector types, the direct
// global->LDS load and the die-aware work split.  Not part of the public ABI.
#pragma once

#include "veda_internal.h"

namespace veda {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct AttnArgs {
    const HeadGeom* heads;
    const uint8_t* tile_head;
    const int32_t* xcd_cum;
    const char* q;             // tiled Q, or null when q_tok is given
    const char* q_tok;         // Q in token order (bf16 kernel only): gathered by the kernel itself
    int64_t sq_b, sq_h, sq_n;  // its strides in bytes
    const char* k;             // tiled K, or null when k_tok is given
    const char* k_tok;         // K in token order (bf16 kernel only): key tiles gathered row by row
    int64_t sk_b, sk_h, sk_n;  // its strides in bytes
    const int32_t* tile_n0;    // token index of slot 0 of every tile (plan table)
    const char* v;
    const uint64_t* valid_mask;
    const int32_t* row_ptr;
    const int32_t* col_idx;
    char* out;
    float* lse;
    int64_t total_tiles, rows;
    int64_t so_b, so_h, so_n;  // output strides in bytes
    int64_t tokens;
    int n_heads, T, H, W;
    float scale_log2;          // softmax_scale * log2(e)
    // scale_log2 = scale_pow2 * scale_resid, scale_pow2 a power of two and 1 <= scale_resid < 2: with the
    // plan's exact-logit-scale option the bf16 kernel multiplies Q by scale_pow2 (exact in bf16) and the
    // logits by scale_resid on their way into the exponential, so no rounding of Q comes between the
    // inputs and the products; without it Q is multiplied by scale_log2 and rounded to bf16 once
    float scale_pow2, scale_resid;
};

// Workgroups are dealt round-robin to the 8 dies (XCDs), each with its own L2, all sharing
// the 256 MB memory-side cache.  Die x = blockIdx.x % 8 takes the x-th eighth of every head's
// query tiles and walks the heads in order: all dies then work on the same head at the same
// time (its K/V, ~120 MB at 220k tokens, stay in the memory-side cache), and the workgroups
// sharing an L2 hold neighbouring query tiles, whose kept key tiles overlap.
// The work item is a query tile (unit = 1) or a pair of adjacent query tiles (unit = 2);
// xcd_cum is the matching table of the plan.  Returns false for the padding workgroups of dies
// with fewer items.
__device__ inline bool xcd_work(const int32_t* __restrict__ xcd_cum, const HeadGeom* __restrict__ heads,
                                int n_heads, int unit, int& head, int& item) {
    const int x = blockIdx.x % kXcd, local = blockIdx.x / kXcd;
    const int32_t* cum = xcd_cum + x * (n_heads + 1);
    if (local >= cum[n_heads]) return false;
    int h = 0, hi = n_heads - 1;   // the last head whose first item is <= local: log2(heads) dependent loads
    while (h < hi) {
        const int mid = (h + hi + 1) >> 1;
        if (local >= cum[mid]) h = mid; else hi = mid - 1;
    }
    const int n = unit == 2 ? heads[h].n_pairs : heads[h].n_tiles;
    head = h;
    item = x * (n / kXcd) + (x < n % kXcd ? x : n % kXcd) + (local - cum[h]);
    return true;
}

// Work item p of a head -> its query tiles: A always, B = A's neighbour along g.pair_ax if it
// exists (the last layer of an odd-sized axis has none).
__device__ inline void pair_tiles(const HeadGeom& g, int p, int& qiA, int& qiB, bool& hasB) {
    if (g.pair_ax == 3) {            // halves of a 128-token tile
        qiA = 2 * p; qiB = qiA + 1; hasB = true;
    } else if (g.pair_ax == 2) {
        const int half = (g.nw + 1) / 2, tw2 = p % half, rest = p / half;
        qiA = rest * g.nw + 2 * tw2; qiB = qiA + 1; hasB = 2 * tw2 + 1 < g.nw;
    } else if (g.pair_ax == 1) {
        const int half = (g.nh + 1) / 2, tw = p % g.nw, th2 = (p / g.nw) % half, tt = p / (g.nw * half);
        qiA = (tt * g.nh + 2 * th2) * g.nw + tw; qiB = qiA + g.nw; hasB = 2 * th2 + 1 < g.nh;
    } else {
        const int plane = g.nh * g.nw, rest = p % plane, tt2 = p / plane;
        qiA = 2 * tt2 * plane + rest; qiB = qiA + plane; hasB = 2 * tt2 + 1 < g.nt;
    }
    if (!hasB) qiB = qiA;
}

__device__ inline int rho(int m) {  // swap bits 2 and 3
    return (m & ~12) | ((m & 4) << 1) | ((m & 8) >> 1);
}

// 16 bytes per lane straight from global memory into LDS: lane i of the wave lands at LDS byte
// lds_base + 16*i (lds_base wave-uniform), from global address base + voff (base uniform).
// Written as inline assembly so that the compiler does not serialise later LDS reads of OTHER
// buffers behind these loads; completion is awaited explicitly (vmcnt) before the barrier that
// publishes the buffer.  M0 carries the LDS base (declared clobbered).
__device__ __forceinline__ void dma16_to_lds(uint32_t lds_base, const void* base, uint32_t voff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_base), "v"(voff), "s"(base)
                 : "memory", "m0");
}

// N (1, 2 or 4) such loads with one M0 set-up: load j lands at lds_base + 1024*j + 16*lane and
// reads base + voff[j] + 1024*j -- the instruction's immediate offset moves the LDS address and
// the global address alike (measured on gfx950), so voff[j] is passed with 1024*j already taken off.
template <int N>
__device__ __forceinline__ void dma16_group_to_lds(uint32_t lds_base, const void* base, const uint32_t (&voff)[N]) {
    static_assert(N == 1 || N == 2 || N == 4, "1024*j must fit the 13-bit immediate offset");
    if constexpr (N == 4) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                     "global_load_lds_dwordx4 %1, %5\n\t"
                     "global_load_lds_dwordx4 %2, %5 offset:1024\n\t"
                     "global_load_lds_dwordx4 %3, %5 offset:2048\n\t"
                     "global_load_lds_dwordx4 %4, %5 offset:3072"
                     :
                     : "s"(lds_base), "v"(voff[0]), "v"(voff[1]), "v"(voff[2]), "v"(voff[3]), "s"(base)
                     : "memory", "m0");
    } else if constexpr (N == 2) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                     "global_load_lds_dwordx4 %1, %3\n\t"
                     "global_load_lds_dwordx4 %2, %3 offset:1024"
                     :
                     : "s"(lds_base), "v"(voff[0]), "v"(voff[1]), "s"(base)
                     : "memory", "m0");
    } else {
        dma16_to_lds(lds_base, base, voff[0]);
    }
}

// x of this lane and x of lane ^ 32, without a trip through LDS: the swap exchanges lanes 32-63
// of its first operand with lanes 0-31 of its second, leaving (low half, low half) in one
// register and (high half, high half) in the other.
__device__ __forceinline__ void both_halves(float x, float& lo, float& hi) {
    lo = x;
    hi = x;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(lo), "+v"(hi));
}
__device__ __forceinline__ float max_with_other_half(float x) {
    float lo, hi;
    both_halves(x, lo, hi);
    return fmaxf(lo, hi);
}
__device__ __forceinline__ float sum_with_other_half(float x) {
    float lo, hi;
    both_halves(x, lo, hi);
    return lo + hi;
}

// Launches the query-tile-pair bf16 kernel (attn_pair.hip) on plan pl's geometry; a.xcd_cum must be
// its pair table.  grouped: pl is the inner plan of 128-token tiles and the CSR counts whole tiles.
// exact: the power-of-two / residual split of the logit scale (AttnArgs::scale_pow2, scale_resid).
// walk: merge the kept lists inside the loop instead of building the step table first.
veda_status launch_sparse_attn_bf16_pair(const veda_plan* pl, const AttnArgs& a, bool grouped, bool exact, bool walk,
                                         hipStream_t s);

// The fp32 kernel (attn_f32.hip): same work items (a.xcd_cum must be the plan's pair table), tiled Q, K, V only.
veda_status launch_sparse_attn_f32(const veda_plan* pl, const AttnArgs& a, bool walk, hipStream_t s);

}  // namespace veda
