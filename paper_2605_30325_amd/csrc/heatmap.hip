// Target tile scores of full attention and tile recall -- the supervision side of the method
// (Sec. 4.1 "Target: Full-Attention Score Construction", Eq. 3: S_tgt[i][j] = max over the
// token pairs of (query tile i, key tile j) of Softmax(Q K^T / sqrt(d)); Sec. 4.3 "Efficient
// Ground-Truth Heatmap Generation": exact pooled scores in two passes without storing the
// attention map, optionally for a subset of query tiles; Sec. 3.2: Recall@k).
//
// The softmax couples all keys of a query row, so every query tile walks all key tiles of
// its head twice: pass 1 forms the row maximum m_u and the denominator l_u with an online
// softmax, pass 2 forms the logits again and reduces exp(s_uv - m_u) / l_u over each 64 x 64
// block.  exp is monotone, so the block maximum needs one exponential per query row and
// block: exp(max_v s_uv - m_u) / l_u, then the maximum over the rows u.  Both passes stay in
// one kernel: m_u and l_u never leave the registers and no workspace is needed.
//
// bf16 kernel: one workgroup owns two adjacent query tiles (waves 0,1: rows 0-31 / 32-63 of
// tile A, waves 2,3: of tile B) so that every K tile pulled into LDS feeds 128 query rows;
// S^T = K Q^T on bf16 MFMA with fp32 accumulation, lane = query, registers = keys (same
// operand layout and LDS swizzle as the sparse attention kernel).  Logits are scaled in fp32.
// fp32 kernel: plain VALU arithmetic, one workgroup per query tile.
#include "attn_common.h"

namespace veda {

typedef const __attribute__((address_space(3))) bf16x8* lds_bf16x8_ptr;
__device__ __forceinline__ bf16x8 hm_lds_read16(uint32_t addr) { return *(lds_bf16x8_ptr)(uintptr_t)addr; }

struct HeatArgs {
    const HeadGeom* heads;
    const uint8_t* tile_head;
    const int32_t* xcd_cum;       // pair table (bf16) or tile table (fp32); unused with a query list
    const int32_t* query_tiles;   // optional: global tile ids to process
    int64_t n_query_tiles;
    const char* q;
    const char* k;
    const uint64_t* valid_mask;
    float* heat;
    int64_t total_tiles, score_elems;
    int n_heads;
    float scale_log2;             // softmax_scale * log2(e)
};

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}

// S^T = K Q^T (64 keys x 32 queries, two 32x32 blocks) of one K tile in LDS: raw dot products,
// padded key slots of an edge tile set to -inf.  The MFMAs are issued at raised wave priority:
// the other wave of the SIMD, busy with vector work, otherwise delays them.
template <int D>
__device__ __forceinline__ void heat_logits(f32x16 (&s)[2], const bf16x8 (&qf)[D / 16], uint32_t ka, uint64_t vm,
                                            int hh) {
    constexpr int G = D / 16, kRowB = D * 2;
    const f32x16 zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int c = 0; c < 2; ++c) {
#pragma unroll
        for (int t = 0; t < G; ++t) {
            const bf16x8 kf = hm_lds_read16((ka ^ (uint32_t)(t << 5)) + (uint32_t)(c * 32 * kRowB));
            s[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[t], t == 0 ? zero : s[c], 0, 0, 0);
        }
    }
    __builtin_amdgcn_s_setprio(0);
    if (vm != ~0ull) {
        // register i of key block c is key slot 32c + 16*(i/8) + 8*hh + (i%8).  The empty asm
        // keeps this a real branch, taken for edge tiles only.
        asm volatile("" ::: "memory");
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const uint32_t half = (uint32_t)(vm >> (32 * c)) >> (8 * hh);
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (!((half >> (16 * (i >> 3) + (i & 7))) & 1u)) s[c][i] = -INFINITY;
        }
    }
}

// Largest raw dot product of the wave's query row over the 64 keys (both lane halves).
__device__ __forceinline__ float heat_row_max(const f32x16 (&s)[2]) {
    float mx = -INFINITY;
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[c][i]);
    return max_with_other_half(mx);
}

// kGrouped: 128-token tiles.  The geometry in `a` is that of the 64-slot halves; the workgroup's
// pair is one whole query tile, and the block maximum of a whole (query tile, key tile) pair is
// the maximum over its four half-tile blocks: both halves of the query tile, two consecutive steps.
template <int D, bool kGrouped>
__global__ __launch_bounds__(256) void tile_heatmap_bf16_kernel(HeatArgs a) {
    constexpr int kRowB = D * 2, kKBytes = kTile * kRowB, kKChunks = kRowB / 16;
    constexpr int kLoads = kKBytes / 1024 / 4;   // direct-load instructions per wave per K tile
    constexpr int G = D / 16;
    // dynamic LDS only, so the base is the workgroup's LDS origin (the XOR swizzle needs address
    // bits 4-9 of the base clear): two K slots, then the block maxima of the 4 waves by step parity
    extern __shared__ __align__(1024) char smem[];
    float (*part)[4] = reinterpret_cast<float (*)[4]>(smem + 2 * kKBytes);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int which = wave >> 1, r = wave & 1;
    const int lq = lane & 31, hh = lane >> 5;

    // work item: a pair of adjacent query tiles of one head
    int head, qiA, qiB;
    bool hasB;
    if (a.query_tiles) {
        // listed tiles are processed one per workgroup (tile B absent)
        if ((int64_t)blockIdx.x >= a.n_query_tiles) return;
        const int g = a.query_tiles[blockIdx.x];
        if (kGrouped) {   // g counts whole tiles
            head = a.tile_head[2 * g];
            qiA = 2 * g - a.heads[head].tile_off;
            qiB = qiA + 1;
            hasB = true;
        } else {
            head = a.tile_head[g];
            qiA = qiB = g - a.heads[head].tile_off;
            hasB = false;
        }
    } else {
        int pair;
        if (!xcd_work(a.xcd_cum, a.heads, a.n_heads, 2, head, pair)) return;
        pair_tiles(a.heads[head], pair, qiA, qiB, hasB);
    }
    const HeadGeom hg = a.heads[head];
    const int n = hg.n_tiles;
    const int64_t b = blockIdx.y;
    const bool active = which == 0 || hasB;
    const int qi = which ? qiB : qiA;
    const int64_t head_tile0 = b * a.total_tiles + hg.tile_off;
    const char* kt = a.k + head_tile0 * kKBytes;
    typedef const __attribute__((address_space(4))) uint64_t* const_u64_t;
    const const_u64_t vmask = (const_u64_t)(uintptr_t)(a.valid_mask + hg.tile_off);

    bf16x8 qf[G];
    {
        const char* qrow = a.q + (head_tile0 + qi) * kKBytes + (32 * r + lq) * kRowB + 16 * hh;
#pragma unroll
        for (int t = 0; t < G; ++t) qf[t] = *reinterpret_cast<const bf16x8*>(qrow + 32 * t);
    }
    const bool q_real = (vmask[qi] >> (32 * r + lq)) & 1ull;

    uint32_t k_src[kLoads];
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
        const int inst = wave * kLoads + j;
        const int krow = inst * (1024 / kRowB) + lane / kKChunks, kpos = lane % kKChunks;
        k_src[j] = krow * kRowB + ((kpos ^ (rho(krow & 31) & (kKChunks - 1))) << 4);
    }
    const uint32_t smem_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
    const uint32_t wave_lds = smem_base + (uint32_t)wave * (kLoads * 1024);
    const uint32_t k0 = smem_base + rho(lq) * kRowB + ((hh ^ (lq & (kKChunks - 1))) << 4);
#define VEDA_LOAD_K(j_tile, SLOT)                                                                \
    do {                                                                                         \
        const char* src_ = kt + (int64_t)(j_tile) * kKBytes;                                     \
        const uint32_t dst_ = wave_lds + (uint32_t)(SLOT) * kKBytes;                             \
        _Pragma("unroll") for (int u_ = 0; u_ < kLoads; ++u_)                                    \
            dma16_to_lds(dst_ + u_ * 1024, src_, k_src[u_]);                                     \
    } while (0)
#define VEDA_LOADS_DONE_BARRIER()               \
    do {                                        \
        __builtin_amdgcn_s_waitcnt(0x0F70);     \
        __syncthreads();                        \
    } while (0)

    // ---- pass 1: row maximum m (log2 units) and denominator l of the full softmax ----
    float m = -INFINITY, l = 0.0f;
    VEDA_LOAD_K(0, 0);
    VEDA_LOADS_DONE_BARRIER();
    for (int j = 0; j < n; ++j) {
        if (j + 1 < n) VEDA_LOAD_K(j + 1, (j + 1) & 1);
        const uint64_t vm = vmask[j];
        if (active) {
            f32x16 s[2];
            heat_logits<D>(s, qf, k0 + (uint32_t)((j & 1) * kKBytes), vm, hh);
            // softmax_scale > 0: the largest logit is the largest dot product, scaled
            // finite from j = 0 on: tile 0 starts at the grid origin (a later half tile of a ragged
            // grid may be all padding: its logits are -inf and add nothing)
            const float m_new = fmaxf(m, heat_row_max(s) * a.scale_log2);
            float psum = 0.0f;
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int i = 0; i < 16; ++i) psum += __builtin_amdgcn_exp2f(fmaf(s[c][i], a.scale_log2, -m_new));
            l = l * __builtin_amdgcn_exp2f(m - m_new) + psum;
            m = m_new;
        }
        VEDA_LOADS_DONE_BARRIER();
    }
    l = sum_with_other_half(l);                          // the two lane halves hold different keys
    const float inv_l = 1.0f / l;

    // ---- pass 2: block maxima of exp2(s - m) / l ----
    // whole-tile score blocks hold a quarter of the half-tile ones
    float* hrow = a.heat + b * a.score_elems + (kGrouped ? hg.score_off / 4 : hg.score_off);
    float even_step = 0.0f;   // grouped: maximum of the even step of the current whole key tile
    // publishes the block maxima of step jj (written before that step's barrier)
    auto publish = [&](int jj) {
        if (kGrouped) {
            if (tid == 0) {
                const float v = fmaxf(fmaxf(part[jj & 1][0], part[jj & 1][1]), fmaxf(part[jj & 1][2], part[jj & 1][3]));
                if (jj & 1) hrow[(int64_t)(qiA >> 1) * (n >> 1) + (jj >> 1)] = fmaxf(even_step, v);
                else even_step = v;
            }
        } else if (tid < 2 && (tid == 0 || hasB)) {
            hrow[(int64_t)(tid ? qiB : qiA) * n + jj] = fmaxf(part[jj & 1][2 * tid], part[jj & 1][2 * tid + 1]);
        }
    };
    VEDA_LOAD_K(0, 0);
    VEDA_LOADS_DONE_BARRIER();
    for (int j = 0; j < n; ++j) {
        if (j + 1 < n) VEDA_LOAD_K(j + 1, (j + 1) & 1);
        if (j > 0) publish(j - 1);
        const uint64_t vm = vmask[j];
        float blockmax = 0.0f;
        if (active) {
            f32x16 s[2];
            heat_logits<D>(s, qf, k0 + (uint32_t)((j & 1) * kKBytes), vm, hh);
            const float val = q_real ? __builtin_amdgcn_exp2f(fmaf(heat_row_max(s), a.scale_log2, -m)) * inv_l : 0.0f;
            blockmax = wave_max(val);
        }
        if (lane == 0) part[j & 1][wave] = blockmax;
        VEDA_LOADS_DONE_BARRIER();
    }
    publish(n - 1);
#undef VEDA_LOAD_K
#undef VEDA_LOADS_DONE_BARRIER
}

// fp32: thread (q = tid/4, part = tid%4) holds the logits of query row q against keys part+4e.
template <int D>
__global__ __launch_bounds__(256) void tile_heatmap_f32_kernel(HeatArgs a, float softmax_scale) {
    constexpr int kPitch = D + 1;
    __shared__ float ks[kTile * kPitch];
    __shared__ float wmax[4];
    const int tid = threadIdx.x, q = tid >> 2, part = tid & 3, wave = tid >> 6;
    int head, qi;
    if (a.query_tiles) {
        if ((int64_t)blockIdx.x >= a.n_query_tiles) return;
        const int g = a.query_tiles[blockIdx.x];
        head = a.tile_head[g];
        qi = g - a.heads[head].tile_off;
    } else if (!xcd_work(a.xcd_cum, a.heads, a.n_heads, 1, head, qi)) {
        return;
    }
    const HeadGeom hg = a.heads[head];
    const int n = hg.n_tiles;
    const int64_t b = blockIdx.y;
    const int64_t head_tile0 = b * a.total_tiles + hg.tile_off;
    const float* qrow = reinterpret_cast<const float*>(a.q) + ((head_tile0 + qi) * kTile + q) * D;
    const float* kt = reinterpret_cast<const float*>(a.k) + head_tile0 * kTile * D;
    const uint64_t* vmask = a.valid_mask + hg.tile_off;
    const bool q_real = (vmask[qi] >> q) & 1ull;
    float* hrow = a.heat + b * a.score_elems + hg.score_off + (int64_t)qi * n;

    float m = -INFINITY, l = 0.0f, inv_l = 0.0f;
    for (int pass = 0; pass < 2; ++pass) {
        for (int j = 0; j < n; ++j) {
            const uint64_t vm = vmask[j];
            const float* ksrc = kt + (int64_t)j * kTile * D;
            __syncthreads();
            for (int t = tid; t < kTile * D / 4; t += 256) {
                const float4 kv = *reinterpret_cast<const float4*>(ksrc + 4 * t);
                const int kr = (4 * t) / D, kc = (4 * t) % D;
                float* dst = ks + kr * kPitch + kc;
                dst[0] = kv.x; dst[1] = kv.y; dst[2] = kv.z; dst[3] = kv.w;
            }
            __syncthreads();
            float s[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) s[e] = 0.0f;
            for (int cc = 0; cc < D; cc += 4) {
                const float4 qv = *reinterpret_cast<const float4*>(qrow + cc);
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float* kr = ks + (part + 4 * e) * kPitch + cc;
                    s[e] = fmaf(qv.x, kr[0], s[e]);
                    s[e] = fmaf(qv.y, kr[1], s[e]);
                    s[e] = fmaf(qv.z, kr[2], s[e]);
                    s[e] = fmaf(qv.w, kr[3], s[e]);
                }
            }
            float mx = -INFINITY;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                s[e] = ((vm >> (part + 4 * e)) & 1ull) ? s[e] * softmax_scale : -INFINITY;
                mx = fmaxf(mx, s[e]);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 1));
            mx = fmaxf(mx, __shfl_xor(mx, 2));
            if (pass == 0) {
                const float m_new = fmaxf(m, mx);
                float psum = 0.0f;
#pragma unroll
                for (int e = 0; e < 16; ++e) psum += expf(s[e] - m_new);
                psum += __shfl_xor(psum, 1);
                psum += __shfl_xor(psum, 2);
                l = l * expf(m - m_new) + psum;
                m = m_new;
            } else {
                const float val = q_real ? expf(mx - m) * inv_l : 0.0f;
                const float wm = wave_max(val);
                if ((tid & 63) == 0) wmax[wave] = wm;
                __syncthreads();
                if (tid == 0) hrow[j] = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
            }
        }
        inv_l = 1.0f / l;
    }
}

// Recall@k: one wavefront per row counts the key tiles the two kept lists share (lists of
// distinct tiles in any order); integer atomics keep the per-head totals order-independent.
struct RecallArgs {
    int32_t k[kMaxHeads];
    int64_t col_off[kMaxHeads];
    int64_t nnz_per_batch;
};

__global__ __launch_bounds__(256) void recall_count_kernel(const HeadGeom* __restrict__ heads,
                                                           const uint8_t* __restrict__ tile_head, RecallArgs args,
                                                           const int32_t* __restrict__ col_a,
                                                           const int32_t* __restrict__ col_b,
                                                           unsigned long long* __restrict__ counts,
                                                           int64_t total_tiles, int64_t rows, int n_heads) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int64_t b = row / total_tiles, g = row - b * total_tiles;
    const int head = tile_head[g];
    const int k = args.k[head];
    const int64_t off = b * args.nnz_per_batch + args.col_off[head] + (g - heads[head].tile_off) * k;
    const int32_t* la = col_a + off;
    const int32_t* lb = col_b + off;
    int common = 0;
    for (int x = 0; x < k; ++x) {
        const int want = la[x];
        bool hit = false;
        for (int y = lane; y < k; y += 64) hit |= lb[y] == want;
        common += __any(hit) ? 1 : 0;
    }
    if (lane == 0) atomicAdd(&counts[b * n_heads + head], (unsigned long long)common);
}

__global__ void recall_clear_kernel(unsigned long long* counts, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) counts[i] = 0ull;
}

__global__ void recall_finish_kernel(const HeadGeom* __restrict__ heads, RecallArgs args,
                                     const unsigned long long* __restrict__ counts, float* __restrict__ recall,
                                     int n_heads, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int head = i % n_heads;
    recall[i] = (float)((double)counts[i] / ((double)heads[head].n_tiles * (double)args.k[head]));
}

}  // namespace veda

extern "C" veda_status veda_tile_heatmap(const veda_plan* pl, const void* q_tiled, const void* k_tiled,
                                         const uint64_t* valid_mask, float softmax_scale,
                                         const int32_t* query_tiles, int64_t n_query_tiles, float* heat,
                                         void* stream) {
    using namespace veda;
    if (!pl || !q_tiled || !k_tiled || !valid_mask || !heat) return VEDA_ERR_INVALID_ARG;
    if (!(softmax_scale > 0.0f) || !(softmax_scale < INFINITY)) return VEDA_ERR_INVALID_ARG;
    if (query_tiles ? (n_query_tiles < 1 || n_query_tiles > pl->total_tiles) : n_query_tiles != 0)
        return VEDA_ERR_INVALID_ARG;
    if (!aligned16(q_tiled) || !aligned16(k_tiled)) return VEDA_ERR_UNSUPPORTED;
    const int d = pl->prob.head_dim;
    const bool bf16 = pl->prob.dtype == VEDA_BF16;
    // 128-token tiles (bf16 only): the kernel walks their 64-slot halves, heat counts whole tiles
    const veda_plan* ip = pl->inner ? pl->inner : pl;
    HeatArgs a;
    a.heads = ip->d_heads;
    a.tile_head = ip->d_tile_head;
    a.xcd_cum = bf16 ? ip->d_xcd_cum_pair : ip->d_xcd_cum;
    a.query_tiles = query_tiles;
    a.n_query_tiles = query_tiles ? n_query_tiles : 0;
    a.q = (const char*)q_tiled; a.k = (const char*)k_tiled;
    a.valid_mask = valid_mask;
    a.heat = heat;
    a.total_tiles = ip->total_tiles;
    a.score_elems = pl->score_elems;
    a.n_heads = pl->prob.heads;
    a.scale_log2 = softmax_scale * kLog2e;
    hipStream_t s = (hipStream_t)stream;
    const int64_t items = query_tiles ? n_query_tiles : (int64_t)kXcd * (bf16 ? ip->xcd_max_pairs : ip->xcd_max_tiles);
    dim3 grid((unsigned)items, (unsigned)pl->prob.batch), block(256);
    if (bf16) {
        const size_t smem = (size_t)2 * kTile * d * 2 + 2 * 4 * sizeof(float);
        if (pl->inner) {
            if (d == 128) hipLaunchKernelGGL((tile_heatmap_bf16_kernel<128, true>), grid, block, smem, s, a);
            else hipLaunchKernelGGL((tile_heatmap_bf16_kernel<64, true>), grid, block, smem, s, a);
        } else {
            if (d == 128) hipLaunchKernelGGL((tile_heatmap_bf16_kernel<128, false>), grid, block, smem, s, a);
            else hipLaunchKernelGGL((tile_heatmap_bf16_kernel<64, false>), grid, block, smem, s, a);
        }
    } else {
        if (d == 128) hipLaunchKernelGGL(tile_heatmap_f32_kernel<128>, grid, block, 0, s, a, softmax_scale);
        else hipLaunchKernelGGL(tile_heatmap_f32_kernel<64>, grid, block, 0, s, a, softmax_scale);
    }
    return launch_status("veda_tile_heatmap");
}

extern "C" veda_status veda_tile_recall(const veda_plan* pl, const int32_t* k_per_head, const int32_t* col_idx_a,
                                        const int32_t* col_idx_b, float* recall, void* workspace,
                                        size_t workspace_bytes, void* stream) {
    using namespace veda;
    if (!pl || !k_per_head || !col_idx_a || !col_idx_b || !recall) return VEDA_ERR_INVALID_ARG;
    const int n = pl->prob.batch * pl->prob.heads;
    if (!workspace || workspace_bytes < sizeof(unsigned long long) * (size_t)n) return VEDA_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 7u) return VEDA_ERR_UNSUPPORTED;
    RecallArgs args;
    int64_t off = 0;
    for (int h = 0; h < pl->prob.heads; ++h) {
        const int nt = pl->heads[h].n_tiles;
        if (k_per_head[h] < 1 || k_per_head[h] > nt) return VEDA_ERR_INVALID_ARG;
        args.k[h] = k_per_head[h];
        args.col_off[h] = off;
        off += (int64_t)nt * k_per_head[h];
    }
    args.nnz_per_batch = off;
    hipStream_t s = (hipStream_t)stream;
    unsigned long long* counts = (unsigned long long*)workspace;
    const int64_t rows = pl->total_tiles * pl->prob.batch;
    hipLaunchKernelGGL(recall_clear_kernel, dim3((n + 255) / 256), dim3(256), 0, s, counts, n);
    hipLaunchKernelGGL(recall_count_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, pl->d_heads,
                       pl->d_tile_head, args, col_idx_a, col_idx_b, counts, pl->total_tiles, rows, pl->prob.heads);
    hipLaunchKernelGGL(recall_finish_kernel, dim3((n + 255) / 256), dim3(256), 0, s, pl->d_heads, args, counts,
                       recall, pl->prob.heads, n);
    return launch_status("veda_tile_recall");
}

// ---- squared Frobenius distance between two token-order tensors, per (batch, head) ----------
// (Eq. 8 / Alg. 1: the error a candidate tiling is scored by).  Two deterministic stages: 64
// workgroups per (batch, head) each reduce a contiguous share of the tokens in double precision
// (fixed tree inside the workgroup), then one thread adds the 64 partial sums in order.
namespace veda {

constexpr int kErrParts = 64;

template <typename E> __device__ __forceinline__ float err_elem(const char* p, int c);
template <> __device__ __forceinline__ float err_elem<uint16_t>(const char* p, int c) {
    return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(p)[c] << 16);
}
template <> __device__ __forceinline__ float err_elem<uint32_t>(const char* p, int c) {
    return reinterpret_cast<const float*>(p)[c];
}

template <typename E>
__global__ __launch_bounds__(256) void sqerr_partial_kernel(const char* __restrict__ a, int64_t ab, int64_t ah, int64_t an,
                                                            const char* __restrict__ b, int64_t bb, int64_t bh, int64_t bn,
                                                            double* __restrict__ partial, int64_t tokens, int d,
                                                            int n_heads) {
    __shared__ double red[256];
    const int part = blockIdx.x, head = blockIdx.y, bt = blockIdx.z;
    const int64_t per = (tokens + kErrParts - 1) / kErrParts;
    const int64_t lo = part * per, hi = lo + per < tokens ? lo + per : tokens;
    const char* pa = a + bt * ab + head * ah;
    const char* pb = b + bt * bb + head * bh;
    double acc = 0.0;
    for (int64_t e = lo * d + threadIdx.x; e < hi * d; e += 256) {
        const int64_t n = e / d;
        const int c = (int)(e - n * d);
        const float diff = err_elem<E>(pa + n * an, c) - err_elem<E>(pb + n * bn, c);
        acc += (double)diff * (double)diff;
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[((int64_t)bt * n_heads + head) * kErrParts + part] = red[0];
}

__global__ void sqerr_finish_kernel(const double* __restrict__ partial, double* __restrict__ err, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    double acc = 0.0;
    for (int p = 0; p < kErrParts; ++p) acc += partial[(int64_t)i * kErrParts + p];
    err[i] = acc;
}

}  // namespace veda

extern "C" veda_status veda_output_sqerr(const veda_plan* pl, const void* a, veda_strides sa, const void* b,
                                         veda_strides sb, double* err, void* workspace, size_t workspace_bytes,
                                         void* stream) {
    using namespace veda;
    if (!pl || !a || !b || !err) return VEDA_ERR_INVALID_ARG;
    const int d = pl->prob.head_dim, es = pl->elem_size();
    if (sa.n < d || sb.n < d || sa.b < 0 || sa.h < 0 || sb.b < 0 || sb.h < 0) return VEDA_ERR_INVALID_ARG;
    const int n = pl->prob.batch * pl->prob.heads;
    if (!workspace || workspace_bytes < sizeof(double) * (size_t)n * kErrParts) return VEDA_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(workspace) & 7u) || (reinterpret_cast<uintptr_t>(err) & 7u)) return VEDA_ERR_UNSUPPORTED;
    hipStream_t s = (hipStream_t)stream;
    double* partial = (double*)workspace;
    dim3 grid(kErrParts, (unsigned)pl->prob.heads, (unsigned)pl->prob.batch);
    if (es == 2)
        hipLaunchKernelGGL(sqerr_partial_kernel<uint16_t>, grid, dim3(256), 0, s, (const char*)a, sa.b * es, sa.h * es,
                           sa.n * es, (const char*)b, sb.b * es, sb.h * es, sb.n * es, partial, pl->tokens(), d,
                           pl->prob.heads);
    else
        hipLaunchKernelGGL(sqerr_partial_kernel<uint32_t>, grid, dim3(256), 0, s, (const char*)a, sa.b * es, sa.h * es,
                           sa.n * es, (const char*)b, sb.b * es, sb.h * es, sb.n * es, partial, pl->tokens(), d,
                           pl->prob.heads);
    hipLaunchKernelGGL(sqerr_finish_kernel, dim3((n + 255) / 256), dim3(256), 0, s, partial, err, n);
    return launch_status("veda_output_sqerr");
}
