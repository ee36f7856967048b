// Stage 2 -- statistics-aware tile scoring (Eq. 4 TripPool, Eq. 5 projections and score;
// Alg. 2 "Triplet Statistics Extraction" and "Projection & Score Estimation").
//
// The scores decide an integer (the top-k set), so every number here is produced by a fixed
// sequence of IEEE fp32 operations: this file is compiled with floating-point contraction
// off, every fused multiply-add is written as fmaf, and no chain is split or re-associated.
//   TripPool : sum over real slots in ascending slot order from +0; avg = sum * (1/count)
//              with 1/count rounded once on the host; max/min by plain comparisons.
//   phi      : per output, one fmaf chain over ascending input index started from the bias.
//   score    : per (i,j), one fmaf chain over ascending latent index from +0, then * scale.
#include "veda_internal.h"

#pragma clang fp contract(off)

namespace veda {

struct RecipTable { float v[kTile + 1]; };  // v[c] = 1.0f / (float)c, computed on the host

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

// One thread owns kN channels of one tile and walks its 64 slots in order.
// grid = (ceil(rows / tiles_per_block), 2 tensors); rows = batch * total_tiles.
template <typename E, int D>
__global__ __launch_bounds__(256) void trippool_kernel(const char* __restrict__ q_tiled,
                                                       const char* __restrict__ k_tiled,
                                                       const uint64_t* __restrict__ valid_mask,
                                                       float* __restrict__ zq, float* __restrict__ zk,
                                                       int64_t rows, int64_t total_tiles, RecipTable recip) {
    constexpr int kN = Chunk<E>::kN;
    constexpr int kTpt = D / kN;                 // threads per tile
    constexpr int kRowBytes = D * (int)sizeof(E);
    const int64_t row = (int64_t)blockIdx.x * (256 / kTpt) + threadIdx.x / kTpt;
    if (row >= rows) return;
    const int chunk = threadIdx.x % kTpt;
    const char* src = (blockIdx.y == 0 ? q_tiled : k_tiled) + row * (int64_t)kTile * kRowBytes + chunk * 16;
    float* z = (blockIdx.y == 0 ? zq : zk) + row * (3 * D) + chunk * kN;
    const uint64_t mask = valid_mask[row % total_tiles];
    float sum[kN], mx[kN], mn[kN];
#pragma unroll
    for (int j = 0; j < kN; ++j) { sum[j] = 0.0f; mx[j] = -INFINITY; mn[j] = INFINITY; }
    if (mask == ~0ull) {
#pragma unroll 8
        for (int l = 0; l < kTile; ++l) {
            float f[kN];
            Chunk<E>::unpack(*reinterpret_cast<const uint4*>(src + l * kRowBytes), f);
#pragma unroll
            for (int j = 0; j < kN; ++j) {
                sum[j] = sum[j] + f[j];
                mx[j] = f[j] > mx[j] ? f[j] : mx[j];
                mn[j] = f[j] < mn[j] ? f[j] : mn[j];
            }
        }
    } else {
        for (int l = 0; l < kTile; ++l) {
            if (!((mask >> l) & 1ull)) continue;
            float f[kN];
            Chunk<E>::unpack(*reinterpret_cast<const uint4*>(src + l * kRowBytes), f);
#pragma unroll
            for (int j = 0; j < kN; ++j) {
                sum[j] = sum[j] + f[j];
                mx[j] = f[j] > mx[j] ? f[j] : mx[j];
                mn[j] = f[j] < mn[j] ? f[j] : mn[j];
            }
        }
    }
    const float inv = recip.v[__popcll(mask)];
#pragma unroll
    for (int j = 0; j < kN; ++j) {
        z[j] = sum[j] * inv;
        z[D + j] = mx[j];
        z[2 * D + j] = mn[j];
    }
}

struct MlpDev {
    int in_dim, hidden, out_dim, relu;
    const float *w1, *b1, *w2, *b2;
};

constexpr int kMlpRows = 16;
constexpr int kMlpThreads = 128;

// One workgroup projects up to 16 consecutive tiles of one head.  Descriptors sit in LDS and
// are read as broadcasts; each thread owns output units and keeps 16 running chains.
// grid = (ceil(total_tiles/16) [blocks never mix heads' weights: see the while loop], 2, batch)
__global__ __launch_bounds__(kMlpThreads) void mlp_kernel(const HeadGeom* __restrict__ heads,
                                                         const uint8_t* __restrict__ tile_head,
                                                         const float* __restrict__ zq, const float* __restrict__ zk,
                                                         float* __restrict__ yq, float* __restrict__ yk,
                                                         MlpDev pq, MlpDev pk, int64_t total_tiles) {
    extern __shared__ float smem[];
    const MlpDev p = blockIdx.y == 0 ? pq : pk;
    const float* z = blockIdx.y == 0 ? zq : zk;
    float* y = blockIdx.y == 0 ? yq : yk;
    const int64_t b = blockIdx.z;
    float* zs = smem;                          // [16][in_dim]
    float* hs = smem + kMlpRows * p.in_dim;    // [16][hidden]
    const int64_t g_begin = (int64_t)blockIdx.x * kMlpRows;
    const int64_t g_end = g_begin + kMlpRows < total_tiles ? g_begin + kMlpRows : total_tiles;
    int64_t g = g_begin;
    while (g < g_end) {
        const int head = tile_head[g];
        const int64_t head_end = (int64_t)heads[head].tile_off + heads[head].n_tiles;
        const int64_t stop = head_end < g_end ? head_end : g_end;
        const int rows = (int)(stop - g);
        const float* zsrc = z + (b * total_tiles + g) * p.in_dim;
        __syncthreads();
        for (int t = threadIdx.x; t < kMlpRows * p.in_dim; t += kMlpThreads)
            zs[t] = t < rows * p.in_dim ? zsrc[t] : 0.0f;
        __syncthreads();
        const int first_out = p.hidden ? p.hidden : p.out_dim;
        const float* w1 = p.w1 + (int64_t)head * p.in_dim * first_out;
        const float* b1 = p.b1 + (int64_t)head * first_out;
        for (int j = threadIdx.x; j < first_out; j += kMlpThreads) {
            float acc[kMlpRows];
            const float bias = b1[j];
#pragma unroll
            for (int r = 0; r < kMlpRows; ++r) acc[r] = bias;
            for (int i = 0; i < p.in_dim; i += 4) {   // in_dim = 3*head_dim is a multiple of 4
                float w[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = w1[(int64_t)(i + e) * first_out + j];
#pragma unroll
                for (int r = 0; r < kMlpRows; ++r) {
                    const float4 zv = *reinterpret_cast<const float4*>(zs + r * p.in_dim + i);
                    acc[r] = __builtin_fmaf(zv.x, w[0], acc[r]);
                    acc[r] = __builtin_fmaf(zv.y, w[1], acc[r]);
                    acc[r] = __builtin_fmaf(zv.z, w[2], acc[r]);
                    acc[r] = __builtin_fmaf(zv.w, w[3], acc[r]);
                }
            }
            if (p.hidden) {
#pragma unroll
                for (int r = 0; r < kMlpRows; ++r)
                    hs[r * p.hidden + j] = (p.relu && !(acc[r] > 0.0f)) ? 0.0f : acc[r];
            } else {
#pragma unroll
                for (int r = 0; r < kMlpRows; ++r)
                    if (r < rows) y[(b * total_tiles + g + r) * p.out_dim + j] = acc[r];
            }
        }
        if (p.hidden) {
            __syncthreads();
            const float* w2 = p.w2 + (int64_t)head * p.hidden * p.out_dim;
            const float* b2 = p.b2 + (int64_t)head * p.out_dim;
            for (int o = threadIdx.x; o < p.out_dim; o += kMlpThreads) {
                float acc[kMlpRows];
                const float bias = b2[o];
#pragma unroll
                for (int r = 0; r < kMlpRows; ++r) acc[r] = bias;
                for (int j = 0; j < p.hidden; ++j) {
                    const float w = w2[(int64_t)j * p.out_dim + o];
#pragma unroll
                    for (int r = 0; r < kMlpRows; ++r) acc[r] = __builtin_fmaf(hs[r * p.hidden + j], w, acc[r]);
                }
#pragma unroll
                for (int r = 0; r < kMlpRows; ++r)
                    if (r < rows) y[(b * total_tiles + g + r) * p.out_dim + o] = acc[r];
            }
        }
        g = stop;
    }
}

constexpr int kSB = 64;       // score block edge
constexpr int kSPitch = 68;   // LDS pitch of one latent row (floats)

// One workgroup computes a 64x64 block of one head's score matrix; each thread a 4x4 patch
// (rows 4*ti..+3, columns tj+16*e).  Latent vectors are staged transposed in LDS, 64 latent
// coordinates at a time, and consumed in ascending order.
__global__ __launch_bounds__(256) void score_kernel(const HeadGeom* __restrict__ heads, int n_heads,
                                                    const float* __restrict__ yq, const float* __restrict__ yk,
                                                    float* __restrict__ scores, int dp, float scale,
                                                    int64_t total_tiles, int64_t score_elems) {
    __shared__ float qs[kSB * kSPitch];
    __shared__ float ks[kSB * kSPitch];
    int head = 0;
    while (head + 1 < n_heads && (int)blockIdx.x >= heads[head + 1].score_blk_off) ++head;
    const HeadGeom hg = heads[head];
    const int blk = blockIdx.x - hg.score_blk_off;
    const int bi = blk / hg.score_blk_dim, bj = blk - bi * hg.score_blk_dim;
    const int64_t b = blockIdx.y;
    const int nT = hg.n_tiles;
    const float* qbase = yq + (b * total_tiles + hg.tile_off) * dp;
    const float* kbase = yk + (b * total_tiles + hg.tile_off) * dp;
    const int ti = threadIdx.x / 16, tj = threadIdx.x % 16;
    float acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[a][e] = 0.0f;
    for (int c0 = 0; c0 < dp; c0 += kSB) {
        const int cn = dp - c0 < kSB ? dp - c0 : kSB;   // multiple of 4
        __syncthreads();
        for (int t = threadIdx.x; t < kSB * (kSB / 4); t += 256) {
            const int r = t / (kSB / 4), c4 = (t % (kSB / 4)) * 4;
            float4 qv = make_float4(0.f, 0.f, 0.f, 0.f), kv = qv;
            if (c4 < cn) {
                if (bi * kSB + r < nT) qv = *reinterpret_cast<const float4*>(qbase + (int64_t)(bi * kSB + r) * dp + c0 + c4);
                if (bj * kSB + r < nT) kv = *reinterpret_cast<const float4*>(kbase + (int64_t)(bj * kSB + r) * dp + c0 + c4);
            }
            qs[(c4 + 0) * kSPitch + r] = qv.x; qs[(c4 + 1) * kSPitch + r] = qv.y;
            qs[(c4 + 2) * kSPitch + r] = qv.z; qs[(c4 + 3) * kSPitch + r] = qv.w;
            ks[(c4 + 0) * kSPitch + r] = kv.x; ks[(c4 + 1) * kSPitch + r] = kv.y;
            ks[(c4 + 2) * kSPitch + r] = kv.z; ks[(c4 + 3) * kSPitch + r] = kv.w;
        }
        __syncthreads();
        for (int c = 0; c < cn; ++c) {
            const float4 qv = *reinterpret_cast<const float4*>(qs + c * kSPitch + 4 * ti);
            const float qa[4] = {qv.x, qv.y, qv.z, qv.w};
            float kb[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) kb[e] = ks[c * kSPitch + tj + 16 * e];
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[a][e] = __builtin_fmaf(qa[a], kb[e], acc[a][e]);
        }
    }
    float* sbase = scores + b * score_elems + hg.score_off;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const int i = bi * kSB + 4 * ti + a;
        if (i >= nT) continue;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int j = bj * kSB + tj + 16 * e;
            if (j < nT) sbase[(int64_t)i * nT + j] = acc[a][e] * scale;
        }
    }
}

static veda_status check_mlp(const veda_plan* pl, const veda_mlp* m) {
    if (!m || !m->w1 || !m->b1) return VEDA_ERR_INVALID_ARG;
    if (m->in_dim != 3 * pl->prob.head_dim) return VEDA_ERR_INVALID_ARG;
    if (m->hidden < 0 || m->out_dim < 1) return VEDA_ERR_INVALID_ARG;
    if (m->hidden > 0 && (!m->w2 || !m->b2)) return VEDA_ERR_INVALID_ARG;
    if (m->act != VEDA_ACT_IDENTITY && m->act != VEDA_ACT_RELU) return VEDA_ERR_INVALID_ARG;
    if (m->hidden > 512 || m->out_dim > 256 || (m->out_dim & 3)) return VEDA_ERR_UNSUPPORTED;
    return VEDA_OK;
}

}  // namespace veda

extern "C" veda_status veda_tile_score(const veda_plan* pl, const void* q_tiled, const void* k_tiled,
                                       const uint64_t* valid_mask, const veda_mlp* phi_q,
                                       const veda_mlp* phi_k, float scale, float* scores, void* workspace,
                                       size_t workspace_bytes, void* stream) {
    using namespace veda;
    if (!pl || !q_tiled || !k_tiled || !valid_mask || !scores) return VEDA_ERR_INVALID_ARG;
    veda_status st = check_mlp(pl, phi_q);
    if (st == VEDA_OK) st = check_mlp(pl, phi_k);
    if (st != VEDA_OK) return st;
    if (phi_q->out_dim != phi_k->out_dim) return VEDA_ERR_INVALID_ARG;
    if (!aligned16(q_tiled) || !aligned16(k_tiled) || !aligned16(workspace)) return VEDA_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < veda_plan_workspace_bytes(pl, phi_q, phi_k)) return VEDA_ERR_WORKSPACE;

    const int d = pl->prob.head_dim, dp = phi_q->out_dim;
    const int64_t total = pl->total_tiles, rows = total * pl->prob.batch;
    float* zq = (float*)workspace;
    float* zk = zq + rows * 3 * d;
    float* yq = zk + rows * 3 * d;
    float* yk = yq + rows * dp;
    hipStream_t s = (hipStream_t)stream;

    RecipTable recip;
    recip.v[0] = 0.0f;
    for (int c = 1; c <= kTile; ++c) recip.v[c] = 1.0f / (float)c;

    const bool bf16 = pl->prob.dtype == VEDA_BF16;
#define VEDA_LAUNCH_TP(E, D)                                                                               \
    do {                                                                                                   \
        constexpr int tpb = 256 / (D / Chunk<E>::kN);                                                      \
        dim3 grid((unsigned)((rows + tpb - 1) / tpb), 2);                                                  \
        hipLaunchKernelGGL((trippool_kernel<E, D>), grid, dim3(256), 0, s, (const char*)q_tiled,           \
                           (const char*)k_tiled, valid_mask, zq, zk, rows, total, recip);                  \
    } while (0)
    if (bf16 && d == 128) VEDA_LAUNCH_TP(uint16_t, 128);
    else if (bf16) VEDA_LAUNCH_TP(uint16_t, 64);
    else if (d == 128) VEDA_LAUNCH_TP(uint32_t, 128);
    else VEDA_LAUNCH_TP(uint32_t, 64);
#undef VEDA_LAUNCH_TP
    st = launch_status("trippool_kernel");
    if (st != VEDA_OK) return st;

    MlpDev pq{phi_q->in_dim, phi_q->hidden, phi_q->out_dim, phi_q->act == VEDA_ACT_RELU, phi_q->w1, phi_q->b1, phi_q->w2, phi_q->b2};
    MlpDev pk{phi_k->in_dim, phi_k->hidden, phi_k->out_dim, phi_k->act == VEDA_ACT_RELU, phi_k->w1, phi_k->b1, phi_k->w2, phi_k->b2};
    const int max_hidden = phi_q->hidden > phi_k->hidden ? phi_q->hidden : phi_k->hidden;
    const size_t smem = sizeof(float) * (size_t)kMlpRows * (size_t)(3 * d + max_hidden);
    dim3 mgrid((unsigned)((total + kMlpRows - 1) / kMlpRows), 2, (unsigned)pl->prob.batch);
    hipLaunchKernelGGL(mlp_kernel, mgrid, dim3(kMlpThreads), smem, s, pl->d_heads, pl->d_tile_head, zq, zk, yq,
                       yk, pq, pk, total);
    st = launch_status("mlp_kernel");
    if (st != VEDA_OK) return st;

    dim3 sgrid((unsigned)pl->score_blocks, (unsigned)pl->prob.batch);
    hipLaunchKernelGGL(score_kernel, sgrid, dim3(256), 0, s, pl->d_heads, pl->prob.heads, yq, yk, scores, dp,
                       scale, total, pl->score_elems);
    return launch_status("score_kernel");
}
