// Stage 2 -- statistics-aware tile scoring (Eq. 4 TripPool, Eq. 5 projections and score;
// Alg. 2 "Triplet Statistics Extraction" and "Projection & Score Estimation").
//
// The scores decide an integer (the top-k set), so every number here is produced by a fixed
// sequence of IEEE fp32 operations: this file is compiled with floating-point contraction
// off, every fused multiply-add is written as fmaf or issued as v_mfma_f32_32x32x2_f32 (which
// applies its two terms one after the other as fmas: see mlp_layer), and no chain is split or
// re-associated.
//   TripPool : sum over real slots in ascending slot order from +0; avg = sum * (1/count)
//              with 1/count rounded once on the host; max/min by plain comparisons.
//   phi      : per output, one fmaf chain over ascending input index started from the bias.
//   score    : per (i,j), one fmaf chain over ascending latent index from +0, then * scale.
#include "score_common.h"

#pragma clang fp contract(off)

namespace veda {

// One thread owns kN channels of one tile and walks its slots in order (kWords = 1: 64-token
// tiles; kWords = 2: 128-token tiles, stored as two consecutive 64-slot halves with one mask
// word each, so slot order is unchanged).
// grid = (ceil(rows / tiles_per_block), 2 tensors); rows = batch * total_tiles.
template <typename E, int D, int kWords>
__global__ __launch_bounds__(256) void trippool_kernel(const char* __restrict__ q_tiled,
                                                       const char* __restrict__ k_tiled,
                                                       const uint64_t* __restrict__ valid_mask,
                                                       float* __restrict__ zq, float* __restrict__ zk,
                                                       int64_t rows, int64_t total_tiles, RecipTable recip) {
    constexpr int kN = Chunk<E>::kN;
    constexpr int kTpt = D / kN;                 // threads per tile
    constexpr int kRowBytes = D * (int)sizeof(E);
    constexpr int kSlots = kWords * kTile;
    const int64_t row = (int64_t)blockIdx.x * (256 / kTpt) + threadIdx.x / kTpt;
    if (row >= rows) return;
    const int chunk = threadIdx.x % kTpt;
    const char* src = (blockIdx.y == 0 ? q_tiled : k_tiled) + row * (int64_t)kSlots * kRowBytes + chunk * 16;
    float* z = (blockIdx.y == 0 ? zq : zk) + row * (3 * D) + chunk * kN;
    uint64_t mask[kWords];
    bool full = true;
    int count = 0;
#pragma unroll
    for (int w = 0; w < kWords; ++w) {
        mask[w] = valid_mask[(row % total_tiles) * kWords + w];
        full = full && mask[w] == ~0ull;
        count += __popcll(mask[w]);
    }
    float sum[kN], mx[kN], mn[kN];
#pragma unroll
    for (int j = 0; j < kN; ++j) { sum[j] = 0.0f; mx[j] = -INFINITY; mn[j] = INFINITY; }
    if (full) {
#pragma unroll 8
        for (int l = 0; l < kSlots; ++l) {
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
#pragma unroll
        for (int w = 0; w < kWords; ++w) {
            for (int l = 0; l < kTile; ++l) {
                if (!((mask[w] >> l) & 1ull)) continue;
                float f[kN];
                Chunk<E>::unpack(*reinterpret_cast<const uint4*>(src + (w * kTile + l) * kRowBytes), f);
#pragma unroll
                for (int j = 0; j < kN; ++j) {
                    sum[j] = sum[j] + f[j];
                    mx[j] = f[j] > mx[j] ? f[j] : mx[j];
                    mn[j] = f[j] < mn[j] ? f[j] : mn[j];
                }
            }
        }
    }
    const float inv = recip.v[count];
#pragma unroll
    for (int j = 0; j < kN; ++j) {
        z[j] = sum[j] * inv;
        z[D + j] = mx[j];
        z[2 * D + j] = mn[j];
    }
}

constexpr int kMlpRows = 64;       // tiles per workgroup
constexpr int kMlpCols = 128;      // output units per pass
constexpr int kMlpK = 16;          // reduction indices staged per step
constexpr int kMlpThreads = 256;
constexpr int kMlpXPitch = kMlpK + 4;   // floats; keeps every staged row 16-byte aligned
constexpr int kMlpWsFloats = kMlpK * kMlpCols;        // one weight stage
constexpr int kMlpXsFloats = kMlpRows * kMlpXPitch;   // one input stage

// One affine layer for the 64 rows of a workgroup:
//   out[r][n] = act(bias[n] + sum_k x[r][k] * w[k][n]),  one fmaf chain per (r,n), k ascending.
// The chains run on the matrix cores: v_mfma_f32_32x32x2_f32 adds its two products to the
// accumulator one after the other, each with its own rounding, in ascending k -- measured on
// gfx950 to give the bits of fmaf(x[k+1], w[k+1], fmaf(x[k], w[k], acc)) on 245,760 random chains
// of 64 terms, denormal sums and products included -- so a chain of these instructions over
// k = 0, 2, 4, ... started from the bias IS the chain above, at twice the rate of scalar fp32
// fma.  Wave w of the four owns output columns c0+32w..+31 for both 32-row halves (two 32x32
// accumulators); lane (col = lane%32, kh = lane/32) feeds x[row = col (+32)][k+kh] and
// w[k+kh][column] and holds rows (r%4) + 8(r/4) + 4kh of its column in register r.
// The weights of 16 reduction indices x 128 outputs are staged in LDS per step (ws, two buffers);
// the inputs come either from global memory, staged alongside (xs, two buffers), or from a
// resident LDS array (x_lds).  The global loads of step s+1 are in flight while step s is
// computed; one barrier per step.  Results go to an LDS array (y_lds, pitch ldy) or to global
// rows (y_glb, pitch N).
typedef __attribute__((ext_vector_type(16))) float mlp_f32x16;

template <bool kXGlobal, bool kYLds>
__device__ __forceinline__ void mlp_layer(const float* __restrict__ x_glb, const float* x_lds, int ldx, int rows,
                                          int K, const float* __restrict__ w, const float* __restrict__ bias,
                                          int N, bool relu, float* y_lds, int ldy, float* __restrict__ y_glb,
                                          float* xs, float* ws) {
    constexpr int kWPer = kMlpWsFloats / kMlpThreads;   // staged weights per thread and step (8)
    static_assert(kMlpRows * (kMlpK / 4) == kMlpThreads, "one float4 of the inputs per thread and step");
    static_assert(kMlpRows == 64 && kMlpCols == 128 && kMlpThreads == 256, "four waves x (2 x 32 rows) x 32 columns");
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, col = lane & 31, kh = lane >> 5;
    const int xr = threadIdx.x / (kMlpK / 4), xi = (threadIdx.x % (kMlpK / 4)) * 4;   // staged input float4
    for (int c0 = 0; c0 < N; c0 += kMlpCols) {
        const int n = c0 + 32 * wave + col;
        const float bv = n < N ? bias[n] : 0.0f;
        mlp_f32x16 acc[2];
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[0][r] = acc[1][r] = bv;
        float wreg[kWPer];
        float4 xreg = make_float4(0.f, 0.f, 0.f, 0.f);
        auto fetch = [&](int k0) {
            const int kc = K - k0 < kMlpK ? K - k0 : kMlpK;
#pragma unroll
            for (int u = 0; u < kWPer; ++u) {
                const int t = threadIdx.x + u * kMlpThreads, i = t / kMlpCols, c = t % kMlpCols;
                wreg[u] = (i < kc && c0 + c < N) ? w[(int64_t)(k0 + i) * N + c0 + c] : 0.0f;
            }
            if (kXGlobal) {   // K is a multiple of 4 here
                xreg = (xr < rows && xi < kc) ? *reinterpret_cast<const float4*>(x_glb + (int64_t)xr * K + k0 + xi)
                                              : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        };
        auto stash = [&](int buf) {
#pragma unroll
            for (int u = 0; u < kWPer; ++u) ws[buf * kMlpWsFloats + threadIdx.x + u * kMlpThreads] = wreg[u];
            if (kXGlobal) *reinterpret_cast<float4*>(xs + buf * kMlpXsFloats + xr * kMlpXPitch + xi) = xreg;
        };
        __syncthreads();   // the previous pass (or layer) is done with both stages
        fetch(0);
        stash(0);
        __syncthreads();
        int buf = 0;
        for (int k0 = 0; k0 < K; k0 += kMlpK, buf ^= 1) {
            const int kc = K - k0 < kMlpK ? K - k0 : kMlpK;
            const bool more = k0 + kMlpK < K;
            if (more) fetch(k0 + kMlpK);
            const float* wb = ws + buf * kMlpWsFloats + 32 * wave + col + kh * kMlpCols;
            const int xp = kXGlobal ? kMlpXPitch : ldx;
            const float* xb = (kXGlobal ? xs + buf * kMlpXsFloats : x_lds + k0) + col * xp + kh;
            if (kc == kMlpK) {
#pragma unroll
                for (int kk = 0; kk < kMlpK; kk += 2) {
                    const float b = wb[kk * kMlpCols];
                    acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(xb[kk], b, acc[0], 0, 0, 0);
                    acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(xb[32 * xp + kk], b, acc[1], 0, 0, 0);
                }
            } else {
                int kk = 0;
                for (; kk + 2 <= kc; kk += 2) {
                    const float b = wb[kk * kMlpCols];
                    acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(xb[kk], b, acc[0], 0, 0, 0);
                    acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(xb[32 * xp + kk], b, acc[1], 0, 0, 0);
                }
                if (kk < kc) {
                    // odd reduction length: the instruction's second term is made -0 * +0 = -0, the one
                    // addend that leaves every accumulator value, signed zeros included, as it is
                    const float b = kh ? 0.0f : wb[kk * kMlpCols];
                    const float a0 = kh ? -0.0f : xb[kk], a1 = kh ? -0.0f : xb[32 * xp + kk];
                    acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b, acc[0], 0, 0, 0);
                    acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b, acc[1], 0, 0, 0);
                }
            }
            if (more) stash(buf ^ 1);
            __syncthreads();
        }
        if (n < N) {
            // one running pointer, advanced store by store: 32 precomputed 64-bit addresses would
            // not fit beside the accumulators
            float* yp = kYLds ? y_lds + (4 * kh) * ldy + n : y_glb + (int64_t)(4 * kh) * N + n;
            const int pitch = kYLds ? ldy : N;
            int row = 4 * kh;
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float v = (relu && !(acc[rb][r] > 0.0f)) ? 0.0f : acc[rb][r];
                    if (kYLds || row < rows) *yp = v;
                    // next row: +1 inside a group of four, +5 to the next group (rows 8g..8g+3 of this lane half)
                    const int step = (r & 3) == 3 ? 5 : 1;
                    yp += (int64_t)step * pitch;
                    row += step;
                    __builtin_amdgcn_sched_barrier(0);
                }
        }
    }
}

// One workgroup projects up to 64 consecutive tiles of one head (Eq. 5, phi_q or phi_k).
// row_blk[x] = head << 24 | index of the 64-tile block inside that head.
// grid = (row blocks of all heads, 2 estimators, batch); dynamic LDS = staging + hidden layer.
__global__ __launch_bounds__(kMlpThreads, 3) void mlp_kernel(const HeadGeom* __restrict__ heads,
                                                         const int32_t* __restrict__ row_blk,
                                                         const float* __restrict__ zq, const float* __restrict__ zk,
                                                         float* __restrict__ yq, float* __restrict__ yk,
                                                         MlpDev pq, MlpDev pk, int64_t total_tiles,
                                                         float* __restrict__ hq, float* __restrict__ hk) {
    extern __shared__ __align__(16) float smem[];
    const MlpDev p = blockIdx.y == 0 ? pq : pk;
    float* hglb = blockIdx.y == 0 ? hq : hk;   // hidden layer kept in global scratch instead of LDS, if given
    const float* z = blockIdx.y == 0 ? zq : zk;
    float* y = blockIdx.y == 0 ? yq : yk;
    float* ws = smem;                                   // 2 x [16][128]
    float* xs = ws + 2 * kMlpWsFloats;                  // 2 x [64][20]
    float* hs = xs + 2 * kMlpXsFloats;                  // [64][ldh]
    const int32_t code = row_blk[blockIdx.x];
    const int head = code >> 24, blk = code & 0xffffff;
    const HeadGeom hg = heads[head];
    const int rows = hg.n_tiles - blk * kMlpRows < kMlpRows ? hg.n_tiles - blk * kMlpRows : kMlpRows;
    const int64_t row0 = (int64_t)blockIdx.z * total_tiles + hg.tile_off + (int64_t)blk * kMlpRows;
    const float* x = z + row0 * p.in_dim;
    float* out = y + row0 * p.out_dim;
    if (p.hidden && hglb) {
        // The 64 x hidden intermediate goes through global memory (it stays in L2): without it in
        // LDS more workgroups fit on a compute unit (three instead of two).  The barrier that opens the second
        // layer also orders these stores before its loads (same workgroup).
        float* hrow = hglb + row0 * p.hidden;
        mlp_layer<true, false>(x, nullptr, 0, rows, p.in_dim, p.w1 + (int64_t)head * p.in_dim * p.hidden,
                  p.b1 + (int64_t)head * p.hidden, p.hidden, p.relu != 0, nullptr, 0, hrow, xs, ws);
        mlp_layer<true, false>(hrow, nullptr, 0, rows, p.hidden, p.w2 + (int64_t)head * p.hidden * p.out_dim,
                  p.b2 + (int64_t)head * p.out_dim, p.out_dim, false, nullptr, 0, out, xs, ws);
    } else if (p.hidden) {
        const int ldh = (p.hidden + 3) & ~3;
        mlp_layer<true, true>(x, nullptr, 0, rows, p.in_dim, p.w1 + (int64_t)head * p.in_dim * p.hidden,
                  p.b1 + (int64_t)head * p.hidden, p.hidden, p.relu != 0, hs, ldh, nullptr, xs, ws);
        mlp_layer<false, false>(nullptr, hs, ldh, rows, p.hidden, p.w2 + (int64_t)head * p.hidden * p.out_dim,
                  p.b2 + (int64_t)head * p.out_dim, p.out_dim, false, nullptr, 0, out, xs, ws);
    } else {
        mlp_layer<true, false>(x, nullptr, 0, rows, p.in_dim, p.w1 + (int64_t)head * p.in_dim * p.out_dim,
                  p.b1 + (int64_t)head * p.out_dim, p.out_dim, false, nullptr, 0, out, xs, ws);
    }
}

constexpr int kSB = 128;      // score block edge
constexpr int kSC = 32;       // latent coordinates staged per step
constexpr int kSPitch = 36;   // LDS pitch of one staged latent row (floats): rows stay 16-byte
                              // aligned and 8 consecutive rows start in 8 different bank groups

// A 128x128 block (bi, bj) of one head's score matrix (Eq. 5) by one workgroup.  Every score is
// one fma chain over ascending latent coordinate from +0, run on the matrix cores like the
// projections' (see mlp_layer: v_mfma_f32_32x32x2_f32 over the coordinate pairs gives the bits of
// the fmaf chain).  Wave w holds rows 32w..32w+31 x all 128 columns in four 32x32 accumulators:
// register r of lane (col = lane%32, kh = lane/32) is row (r%4) + 8(r/4) + 4kh, column 32cb + col.
// Latent rows are staged row-major in LDS, 32 coordinates at a time.
__device__ __forceinline__ void score_block_128(const HeadGeom& hg, int bi, int bj, int64_t b, float* qs, float* ks,
                                                const float* __restrict__ yq, const float* __restrict__ yk,
                                                float* __restrict__ scores, int dp, float scale,
                                                int64_t total_tiles, int64_t score_elems) {
    const int nT = hg.n_tiles;
    const float* qbase = yq + (b * total_tiles + hg.tile_off) * dp;
    const float* kbase = yk + (b * total_tiles + hg.tile_off) * dp;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, col = lane & 31, kh = lane >> 5;
    mlp_f32x16 acc[4];
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[cb][r] = 0.0f;
    for (int c0 = 0; c0 < dp; c0 += kSC) {
        const int cn = dp - c0 < kSC ? dp - c0 : kSC;   // multiple of 4
        __syncthreads();
        for (int t = threadIdx.x; t < kSB * (kSC / 4); t += 256) {
            const int r = t / (kSC / 4), c4 = (t % (kSC / 4)) * 4;
            float4 qv = make_float4(0.f, 0.f, 0.f, 0.f), kv = qv;
            if (c4 < cn) {
                if (bi * kSB + r < nT) qv = *reinterpret_cast<const float4*>(qbase + (int64_t)(bi * kSB + r) * dp + c0 + c4);
                if (bj * kSB + r < nT) kv = *reinterpret_cast<const float4*>(kbase + (int64_t)(bj * kSB + r) * dp + c0 + c4);
            }
            *reinterpret_cast<float4*>(qs + r * kSPitch + c4) = qv;
            *reinterpret_cast<float4*>(ks + r * kSPitch + c4) = kv;
        }
        __syncthreads();
        const float* qa = qs + (32 * wave + col) * kSPitch + kh;   // A: q[row = col][c + kh]
        const float* kb = ks + col * kSPitch + kh;                  // B: k[column = col][c + kh]
        if (cn == kSC) {
#pragma unroll
            for (int c = 0; c < kSC; c += 2) {
                const float a = qa[c];
#pragma unroll
                for (int cb = 0; cb < 4; ++cb)
                    acc[cb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, kb[32 * cb * kSPitch + c], acc[cb], 0, 0, 0);
            }
        } else {
            for (int c = 0; c < cn; c += 2) {
                const float a = qa[c];
#pragma unroll
                for (int cb = 0; cb < 4; ++cb)
                    acc[cb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, kb[32 * cb * kSPitch + c], acc[cb], 0, 0, 0);
            }
        }
    }
    float* sbase = scores + b * score_elems + hg.score_off;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int i = bi * kSB + 32 * wave + (r & 3) + 8 * (r >> 2) + 4 * kh;
        if (i >= nT) continue;
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) {
            const int j = bj * kSB + 32 * cb + col;
            if (j < nT) sbase[(int64_t)i * nT + j] = acc[cb][r] * scale;
        }
    }
}

// All score blocks, one workgroup each.
__global__ __launch_bounds__(256, 3) void score_kernel(const HeadGeom* __restrict__ heads, int n_heads,
                                                    const float* __restrict__ yq, const float* __restrict__ yk,
                                                    float* __restrict__ scores, int dp, float scale,
                                                    int64_t total_tiles, int64_t score_elems) {
    __shared__ __align__(16) float qs[kSB * kSPitch];
    __shared__ __align__(16) float ks[kSB * kSPitch];
    int lo = 0, hi = n_heads - 1;   // last head whose first block is <= blockIdx.x
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if ((int)blockIdx.x >= heads[mid].score_blk_off) lo = mid; else hi = mid - 1;
    }
    const HeadGeom hg = heads[lo];
    const int blk = blockIdx.x - hg.score_blk_off;
    const int bi = blk / hg.score_blk_dim, bj = blk - bi * hg.score_blk_dim;
    score_block_128(hg, bi, bj, blockIdx.y, qs, ks, yq, yk, scores, dp, scale, total_tiles, score_elems);
}

// Only the score rows somebody asked for: one workgroup per 128 rows of a head (the even
// entries of the 64-row table), which leaves at once unless one of the marks of its rows is set
// (marks: one per 128 consecutive rows of the latents, row >> 7) and otherwise forms all the
// blocks of its rows.
__global__ __launch_bounds__(256, 2) void score_marked_rows_kernel(const HeadGeom* __restrict__ heads,
                                                                const int32_t* __restrict__ row_blk,
                                                                const float* __restrict__ yq,
                                                                const float* __restrict__ yk,
                                                                float* __restrict__ scores, int dp, float scale,
                                                                int64_t total_tiles, int64_t score_elems,
                                                                const int32_t* __restrict__ marks) {
    __shared__ __align__(16) float qs[kSB * kSPitch];
    __shared__ __align__(16) float ks[kSB * kSPitch];
    const int32_t code = row_blk[blockIdx.x];
    if (code & 1) return;
    const HeadGeom hg = heads[code >> 24];
    const int bi = (code & 0xffffff) >> 1, nT = hg.n_tiles;
    const int64_t b = blockIdx.y;
    const int64_t g0 = b * total_tiles + hg.tile_off + (int64_t)bi * kSB;
    const int last = nT - 1 - bi * kSB < kSB - 1 ? nT - 1 - bi * kSB : kSB - 1;
    if (!(marks[g0 >> 7] | marks[(g0 + last) >> 7])) return;
    for (int bj = 0; bj < hg.score_blk_dim; ++bj)
        score_block_128(hg, bi, bj, b, qs, ks, yq, yk, scores, dp, scale, total_tiles, score_elems);
}

veda_status check_mlp(const veda_plan* pl, const veda_mlp* m) {
    if (!m || !m->w1 || !m->b1) return VEDA_ERR_INVALID_ARG;
    if (m->in_dim != 3 * pl->prob.head_dim) return VEDA_ERR_INVALID_ARG;
    if (m->hidden < 0 || m->out_dim < 1) return VEDA_ERR_INVALID_ARG;
    if (m->hidden > 0 && (!m->w2 || !m->b2)) return VEDA_ERR_INVALID_ARG;
    if (m->act != VEDA_ACT_IDENTITY && m->act != VEDA_ACT_RELU) return VEDA_ERR_INVALID_ARG;
    if (m->hidden > 512 || m->out_dim > 256 || (m->out_dim & 3)) return VEDA_ERR_UNSUPPORTED;
    return VEDA_OK;
}

static void fill_recip(RecipTable& recip) {
    recip.v[0] = 0.0f;
    for (int c = 1; c <= 2 * kTile; ++c) recip.v[c] = 1.0f / (float)c;
}

// TripPool (Eq. 4) of the tiled Q and K into zq, zk.
void launch_trippool(const veda_plan* pl, const void* q_tiled, const void* k_tiled, const uint64_t* valid_mask,
                            float* zq, float* zk, hipStream_t s) {
    const int d = pl->prob.head_dim;
    const int64_t total = pl->total_tiles, rows = total * pl->prob.batch;
    RecipTable recip;
    fill_recip(recip);

    const bool bf16 = pl->prob.dtype == VEDA_BF16;
#define VEDA_LAUNCH_TP(E, D)                                                                               \
    do {                                                                                                   \
        constexpr int tpb = 256 / (D / Chunk<E>::kN);                                                      \
        dim3 grid((unsigned)((rows + tpb - 1) / tpb), 2);                                                  \
        if (pl->inner)                                                                                     \
            hipLaunchKernelGGL((trippool_kernel<E, D, 2>), grid, dim3(256), 0, s, (const char*)q_tiled,    \
                               (const char*)k_tiled, valid_mask, zq, zk, rows, total, recip);              \
        else                                                                                               \
            hipLaunchKernelGGL((trippool_kernel<E, D, 1>), grid, dim3(256), 0, s, (const char*)q_tiled,    \
                               (const char*)k_tiled, valid_mask, zq, zk, rows, total, recip);              \
    } while (0)
    if (bf16 && d == 128) VEDA_LAUNCH_TP(uint16_t, 128);
    else if (bf16) VEDA_LAUNCH_TP(uint16_t, 64);
    else if (d == 128) VEDA_LAUNCH_TP(uint32_t, 128);
    else VEDA_LAUNCH_TP(uint32_t, 64);
#undef VEDA_LAUNCH_TP
}

// Weight-free scorer (App. A.3): latent y = [avg | root_lambda * sqrt(max(0, (max-avg)(avg-min)))] per tile,
// whose plain dot product is the mean product plus lambda times the dispersion product.
__global__ __launch_bounds__(256) void closed_form_latent_kernel(const float* __restrict__ zq, const float* __restrict__ zk,
                                                                 float* __restrict__ yq, float* __restrict__ yk,
                                                                 int64_t rows, int d, float root_lambda) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= rows * d) return;
    const int64_t i = e / d;
    const int c = (int)(e - i * d);
    const float* z = (blockIdx.y == 0 ? zq : zk) + i * 3 * d;
    float* y = (blockIdx.y == 0 ? yq : yk) + i * 2 * d;
    const float mu = z[c], mx = z[d + c], mn = z[2 * d + c];
    const float up = mx - mu, dn = mu - mn;
    float p = up * dn;
    p = p > 0.0f ? p : 0.0f;
    y[c] = mu;
    y[d + c] = root_lambda * sqrtf(p);
}

// Projections (Eq. 5 phi_q, phi_k) of the descriptors zq, zk into the latents yq, yk.
veda_status launch_projections(const veda_plan* pl, const veda_mlp* phi_q, const veda_mlp* phi_k, const float* zq,
                               const float* zk, float* yq, float* yk, float* hq, float* hk, hipStream_t s) {
    MlpDev pq{phi_q->in_dim, phi_q->hidden, phi_q->out_dim, phi_q->act == VEDA_ACT_RELU, phi_q->w1, phi_q->b1, phi_q->w2, phi_q->b2};
    MlpDev pk{phi_k->in_dim, phi_k->hidden, phi_k->out_dim, phi_k->act == VEDA_ACT_RELU, phi_k->w1, phi_k->b1, phi_k->w2, phi_k->b2};
    if (pl->chain_unit() == VEDA_CHAINS_VECTOR) return launch_projections_vector(pl, pq, pk, zq, zk, yq, yk, s);
    const int max_hidden = phi_q->hidden > phi_k->hidden ? phi_q->hidden : phi_k->hidden;
    // the global route reads the hidden layer back as float4 rows
    if (!hq || !hk || (phi_q->hidden & 3) || (phi_k->hidden & 3)) hq = hk = nullptr;
    const size_t smem = sizeof(float) * ((size_t)2 * kMlpWsFloats + (size_t)2 * kMlpXsFloats +
                                         (hq ? 0 : (size_t)kMlpRows * (size_t)((max_hidden + 3) & ~3)));
    if (smem > 64 * 1024)
        VEDA_HIP_TRY(hipFuncSetAttribute((const void*)mlp_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    dim3 mgrid((unsigned)pl->row_blocks, 2, (unsigned)pl->prob.batch);
    hipLaunchKernelGGL(mlp_kernel, mgrid, dim3(kMlpThreads), smem, s, pl->d_heads, pl->d_row_blk, zq, zk, yq,
                       yk, pq, pk, pl->total_tiles, hq, hk);
    return launch_status("mlp_kernel");
}

// The score blocks of all heads (Eq. 5) from latents of dp coordinates.  marks != nullptr: one
// mark per 128 consecutive rows of the latents (row >> 7); only the score rows of 128-row blocks
// that touch a marked group are formed.
veda_status launch_score_blocks(const veda_plan* pl, const float* yq, const float* yk, float* scores, int dp,
                                float scale, const int32_t* marks, hipStream_t s) {
    if (pl->chain_unit() == VEDA_CHAINS_VECTOR) return launch_score_blocks_vector(pl, yq, yk, scores, dp, scale, marks, s);
    if (marks) {
        dim3 rgrid((unsigned)pl->row_blocks, (unsigned)pl->prob.batch);
        hipLaunchKernelGGL(score_marked_rows_kernel, rgrid, dim3(256), 0, s, pl->d_heads, pl->d_row_blk, yq, yk, scores,
                           dp, scale, pl->total_tiles, pl->score_elems, marks);
        return launch_status("score_marked_rows_kernel");
    }
    dim3 sgrid((unsigned)pl->score_blocks, (unsigned)pl->prob.batch);
    hipLaunchKernelGGL(score_kernel, sgrid, dim3(256), 0, s, pl->d_heads, pl->prob.heads, yq, yk, scores, dp,
                       scale, pl->total_tiles, pl->score_elems);
    return launch_status("score_kernel");
}

// hq, hk: scratch for the hidden layers, or null.
static veda_status project_and_score(const veda_plan* pl, const veda_mlp* phi_q, const veda_mlp* phi_k, float scale,
                                     const float* zq, const float* zk, float* yq, float* yk, float* hq, float* hk,
                                     float* scores, hipStream_t s) {
    const veda_status st = launch_projections(pl, phi_q, phi_k, zq, zk, yq, yk, hq, hk, s);
    if (st != VEDA_OK) return st;
    return launch_score_blocks(pl, yq, yk, scores, phi_q->out_dim, scale, nullptr, s);
}

}  // namespace veda

extern "C" veda_status veda_plan_workspace_layout(const veda_plan* pl, const veda_mlp* phi_q, const veda_mlp* phi_k,
                                                  veda_workspace_layout* out) {
    if (!pl || !phi_q || !phi_k || !out || phi_q->out_dim != phi_k->out_dim) return VEDA_ERR_INVALID_ARG;
    const int64_t rows = pl->total_tiles * pl->prob.batch, d = pl->prob.head_dim, dp = phi_q->out_dim;
    out->stats_q = 0;                       // the order veda_tile_score carves its workspace in
    out->stats_k = rows * 3 * d;
    out->latent_q = 2 * rows * 3 * d;
    out->latent_k = 2 * rows * 3 * d + rows * dp;
    return VEDA_OK;
}

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

    const int dp = phi_q->out_dim;
    const int64_t total = pl->total_tiles, rows = total * pl->prob.batch;
    veda_workspace_layout lay;
    (void)veda_plan_workspace_layout(pl, phi_q, phi_k, &lay);
    float* zq = (float*)workspace + lay.stats_q;
    float* zk = (float*)workspace + lay.stats_k;
    float* yq = (float*)workspace + lay.latent_q;
    float* yk = (float*)workspace + lay.latent_k;
    float* hq = yk + rows * dp;               // the plan's workspace size has room for both hidden layers
    float* hk = hq + rows * (phi_q->hidden > 0 ? phi_q->hidden : 0);
    hipStream_t s = (hipStream_t)stream;

    launch_trippool(pl, q_tiled, k_tiled, valid_mask, zq, zk, s);
    st = launch_status("trippool_kernel");
    if (st != VEDA_OK) return st;

    return project_and_score(pl, phi_q, phi_k, scale, zq, zk, yq, yk, hq, hk, scores, s);
}

extern "C" veda_status veda_tile_score_stats(const veda_plan* pl, const float* stats_q, const float* stats_k,
                                             const veda_mlp* phi_q, const veda_mlp* phi_k, float scale,
                                             float* scores, void* workspace, size_t workspace_bytes,
                                             void* stream) {
    using namespace veda;
    if (!pl || !stats_q || !stats_k || !scores) return VEDA_ERR_INVALID_ARG;
    veda_status st = check_mlp(pl, phi_q);
    if (st == VEDA_OK) st = check_mlp(pl, phi_k);
    if (st != VEDA_OK) return st;
    if (phi_q->out_dim != phi_k->out_dim) return VEDA_ERR_INVALID_ARG;
    if (!aligned16(stats_q) || !aligned16(stats_k) || !aligned16(workspace)) return VEDA_ERR_UNSUPPORTED;
    const int64_t rows = pl->total_tiles * pl->prob.batch;
    const int dp = phi_q->out_dim;
    if (!workspace || workspace_bytes < sizeof(float) * (size_t)rows * 2 * (size_t)dp) return VEDA_ERR_WORKSPACE;
    float* yq = (float*)workspace;
    float* yk = yq + rows * dp;
    // with room for them the hidden layers go through the workspace too (twice the workgroups per
    // compute unit); the results are the same either way
    const size_t hid = (size_t)(phi_q->hidden > 0 ? phi_q->hidden : 0) + (size_t)(phi_k->hidden > 0 ? phi_k->hidden : 0);
    const bool roomy = workspace_bytes >= sizeof(float) * (size_t)rows * (2 * (size_t)dp + hid);
    float* hq = roomy ? yk + rows * dp : nullptr;
    float* hk = roomy ? hq + rows * (phi_q->hidden > 0 ? phi_q->hidden : 0) : nullptr;
    return project_and_score(pl, phi_q, phi_k, scale, stats_q, stats_k, yq, yk, hq, hk, scores, (hipStream_t)stream);
}

extern "C" veda_status veda_tile_score_closed_form(const veda_plan* pl, const void* q_tiled, const void* k_tiled,
                                                   const uint64_t* valid_mask, float lambda, float* scores,
                                                   void* workspace, size_t workspace_bytes, void* stream) {
    using namespace veda;
    if (!pl || !q_tiled || !k_tiled || !valid_mask || !scores) return VEDA_ERR_INVALID_ARG;
    if (!(lambda >= 0.0f) || !(lambda < INFINITY)) return VEDA_ERR_INVALID_ARG;
    if (!aligned16(q_tiled) || !aligned16(k_tiled) || !aligned16(workspace)) return VEDA_ERR_UNSUPPORTED;
    const int d = pl->prob.head_dim;
    const int64_t rows = pl->total_tiles * pl->prob.batch;
    if (!workspace || workspace_bytes < sizeof(float) * (size_t)rows * 10 * (size_t)d) return VEDA_ERR_WORKSPACE;
    float* zq = (float*)workspace;
    float* zk = zq + rows * 3 * d;
    float* yq = zk + rows * 3 * d;
    float* yk = yq + rows * 2 * d;
    hipStream_t s = (hipStream_t)stream;
    launch_trippool(pl, q_tiled, k_tiled, valid_mask, zq, zk, s);
    veda_status st = launch_status("trippool_kernel");
    if (st != VEDA_OK) return st;
    dim3 lgrid((unsigned)((rows * d + 255) / 256), 2);
    hipLaunchKernelGGL(closed_form_latent_kernel, lgrid, dim3(256), 0, s, zq, zk, yq, yk, rows, d, sqrtf(lambda));
    st = launch_status("closed_form_latent_kernel");
    if (st != VEDA_OK) return st;
    return launch_score_blocks(pl, yq, yk, scores, 2 * d, 1.0f, nullptr, s);
}
