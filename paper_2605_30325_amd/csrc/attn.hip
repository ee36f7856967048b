// Stage 4 -- block-sparse flash attention forward + un-tiling (Eq. 2: softmax over the
// concatenation of the kept key tiles; Sec. 3.1 masked form; Sec. 4.3 tile-skipping kernel;
// Alg. 1 "UnTile").
//
// bf16 kernel (CDNA4 MFMA, 64-wide wavefronts).  One workgroup of four wavefronts owns one
// query tile (64 rows).  Wave w = (r, c): r picks 32 query rows, c picks which 32 of each key
// tile's 64 slots the wave attends to.  Every wave runs its own online softmax over its key
// subset and the two key halves are merged once at the end, so each LDS byte of K/V is read
// by two waves only and each wave does 32x32 MFMAs.
//
// The products are formed transposed:  S^T = K Q^T  and  O^T = V^T P^T.  In the 32x32
// accumulator layout a lane then owns ONE query (column) and its registers run over keys,
// so the row max / row sum of the softmax are in-register reductions plus one exchange
// between lane l and l+32, and P^T in registers already has the B-operand layout of the
// second product: no LDS round trip for P.  The accumulator hands a lane keys in the
// interleaved order {8j + 4h + t}; loading K row rho(m) as MFMA row m (rho swaps bits 2,3)
// makes those eight keys per lane-half contiguous, so the V^T operand is one 16-byte LDS
// read from the channel-major V tile.
//
// K and V^T tiles are double buffered in LDS (2 x 32 KB for d = 128): the next tile is
// fetched from global memory into registers while the current one is multiplied, then
// stored to the other buffer.  16-byte chunks are XOR-swizzled inside each LDS row so the
// per-lane row-strided operand reads do not pile onto the same banks.
//
// fp32 kernel: plain fp32 VALU arithmetic, one workgroup per query tile (small problems and
// the 1e-4 accuracy bar; not a throughput path).
#include "veda_internal.h"

namespace veda {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct AttnArgs {
    const HeadGeom* heads;
    const uint8_t* tile_head;
    const char* q;
    const char* k;
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
};

// Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Give every XCD a
// contiguous run of (head, query tile) rows so that the workgroups sharing an L2 work on
// neighbouring query tiles of the same head, whose kept key tiles overlap.
__device__ inline int64_t xcd_row(int64_t pid, int64_t rows) {
    constexpr int kXcd = 8;
    const int64_t xcd = pid % kXcd, local = pid / kXcd;
    const int64_t base = rows / kXcd, rem = rows % kXcd;
    return xcd * base + (xcd < rem ? xcd : rem) + local;
}

__device__ inline int rho(int m) {  // swap bits 2 and 3
    return (m & ~12) | ((m & 4) << 1) | ((m & 8) >> 1);
}

template <int D>
__global__ __launch_bounds__(256, 2) void sparse_attn_bf16_kernel(AttnArgs a) {
    constexpr int kRowB = D * 2;              // bytes of one K row
    constexpr int kKBytes = kTile * kRowB;    // K tile
    constexpr int kVBytes = D * kTile * 2;    // V^T tile: D rows of 128 bytes
    constexpr int kStage = kKBytes + kVBytes;
    constexpr int kKChunks = kRowB / 16;      // 16-byte chunks per K row
    constexpr int kLoads = kKBytes / 16 / 256;  // 16-byte chunks per thread per tile (K; same for V)
    extern __shared__ __align__(16) char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = wave & 1, c = wave >> 1;
    const int lq = lane & 31, hh = lane >> 5;

    const int64_t row = xcd_row(blockIdx.x, a.rows);
    const int64_t b = row / a.total_tiles;
    const int64_t g = row - b * a.total_tiles;
    const int head = a.tile_head[g];
    const HeadGeom hg = a.heads[head];
    const int qi = (int)(g - hg.tile_off);
    const int beg = a.row_ptr[row];
    const int nsel = a.row_ptr[row + 1] - beg;
    const int32_t* cols = a.col_idx + beg;
    const int64_t head_tile0 = b * a.total_tiles + hg.tile_off;
    const char* kt = a.k + head_tile0 * kKBytes;
    const char* vt = a.v + head_tile0 * kVBytes;
    const uint64_t* vmask = a.valid_mask + hg.tile_off;

    // Q operand (B matrix of S^T = K Q^T): lane holds query row 32r+lq, channels 16t+8hh..+8.
    bf16x8 qf[D / 16];
    {
        const char* qrow = a.q + (head_tile0 + qi) * kKBytes + (32 * r + lq) * kRowB + 16 * hh;
#pragma unroll
        for (int t = 0; t < D / 16; ++t) qf[t] = *reinterpret_cast<const bf16x8*>(qrow + 32 * t);
    }

    // global -> LDS copy plan: chunk id = tid + 256*j, contiguous in global memory.
    int k_dst[kLoads], v_dst[kLoads];
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
        const int cid = tid + 256 * j;
        const int krow = cid / kKChunks, kch = cid % kKChunks;
        k_dst[j] = krow * kRowB + ((kch ^ (rho(krow & 31) & (kKChunks - 1))) << 4);
        const int vrow = cid >> 3, vch = cid & 7;
        v_dst[j] = kKBytes + vrow * 128 + ((vch ^ (((vrow >> 1) & 7) ^ ((vrow & 1) << 2))) << 4);
    }
    // Staging registers of the tile in flight (plain unrolled code: the arrays must stay in
    // VGPRs, so no lambdas or dynamic indexing touch them).
    u32x4 kreg[kLoads], vreg[kLoads];
#define VEDA_FETCH(j_tile)                                                            \
    do {                                                                              \
        const char* ks_ = kt + (int64_t)(j_tile) * kKBytes + tid * 16;                \
        const char* vs_ = vt + (int64_t)(j_tile) * kVBytes + tid * 16;                \
        _Pragma("unroll") for (int j = 0; j < kLoads; ++j) {                          \
            kreg[j] = *reinterpret_cast<const u32x4*>(ks_ + 4096 * j);                \
            vreg[j] = *reinterpret_cast<const u32x4*>(vs_ + 4096 * j);                \
        }                                                                             \
    } while (0)
#define VEDA_STASH(stage_)                                                            \
    do {                                                                              \
        char* base_ = smem + (stage_) * kStage;                                       \
        _Pragma("unroll") for (int j = 0; j < kLoads; ++j) {                          \
            *reinterpret_cast<u32x4*>(base_ + k_dst[j]) = kreg[j];                    \
            *reinterpret_cast<u32x4*>(base_ + v_dst[j]) = vreg[j];                    \
        }                                                                             \
    } while (0)

    // operand read offsets inside a stage
    const int k_row_off = (32 * c + rho(lq)) * kRowB;
    const int k_swz = lq & (kKChunks - 1);
    int v_row_off[D / 32], v_swz[D / 32];
#pragma unroll
    for (int nb = 0; nb < D / 32; ++nb) {
        const int vrow = 32 * nb + lq;
        v_row_off[nb] = kKBytes + vrow * 128;
        v_swz[nb] = ((vrow >> 1) & 7) ^ ((vrow & 1) << 2);
    }

    f32x16 o[D / 32];
#pragma unroll
    for (int nb = 0; nb < D / 32; ++nb)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[nb][i] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;

    int j_cur = nsel > 0 ? cols[0] : 0;
    uint64_t vm_cur = nsel > 0 ? vmask[j_cur] : 0ull;
    if (nsel > 0) {
        VEDA_FETCH(j_cur);
        VEDA_STASH(0);
    }
    __syncthreads();

    for (int it = 0; it < nsel; ++it) {
        const int stage = it & 1;
        const bool more = it + 1 < nsel;
        int j_next = 0;
        uint64_t vm_next = 0ull;
        if (more) {
            j_next = cols[it + 1];
            vm_next = vmask[j_next];
            VEDA_FETCH(j_next);
        }
        const char* sb = smem + stage * kStage;

        // S^T (32 keys x 32 queries) = K_half Q^T
        f32x16 s;
#pragma unroll
        for (int i = 0; i < 16; ++i) s[i] = 0.0f;
#pragma unroll
        for (int t = 0; t < D / 16; ++t) {
            const bf16x8 kf = *reinterpret_cast<const bf16x8*>(sb + k_row_off + (((2 * t + hh) ^ k_swz) << 4));
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[t], s, 0, 0, 0);
        }
        // register i of this lane is key slot 32c + 16*(i/8) + 8*hh + (i%8) of the tile
        if (vm_cur != ~0ull) {
            const uint32_t half = (uint32_t)(vm_cur >> (32 * c));
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (!((half >> (16 * (i >> 3) + 8 * hh + (i & 7))) & 1u)) s[i] = -INFINITY;
        }
        float mloc = s[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) mloc = fmaxf(mloc, s[i]);
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
        const float m_new = fmaxf(m_run, mloc);
        const float m_use = m_new == -INFINITY ? 0.0f : m_new;
        const float mc = m_use * a.scale_log2;
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_use) * a.scale_log2);
        float psum = 0.0f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            s[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], a.scale_log2, -mc));
            psum += s[i];
        }
        l_run = l_run * alpha + psum;
        m_run = m_new;
        if (__any(alpha != 1.0f)) {
#pragma unroll
            for (int nb = 0; nb < D / 32; ++nb)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[nb][i] *= alpha;
        }
        bf16x8 pf[2];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            pf[0][e] = (__bf16)s[e];
            pf[1][e] = (__bf16)s[8 + e];
        }
        // O^T (d x 32 queries) += V^T[:, keys of this half] P^T
#pragma unroll
        for (int nb = 0; nb < D / 32; ++nb) {
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                const int cv = 4 * c + 2 * s2 + hh;
                const bf16x8 vf = *reinterpret_cast<const bf16x8*>(sb + v_row_off[nb] + ((cv ^ v_swz[nb]) << 4));
                o[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[s2], o[nb], 0, 0, 0);
            }
        }
        if (more) VEDA_STASH(stage ^ 1);
        j_cur = j_next;
        vm_cur = vm_next;
        __syncthreads();
    }

#undef VEDA_FETCH
#undef VEDA_STASH
    // ---- merge the two key halves, normalise, transpose through LDS, scatter to tokens ----
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    float* xo = reinterpret_cast<float*>(smem) + r * (32 * D + 64);  // [D][32] + m[32] + l[32]
    char* obuf = smem + 2 * (32 * D + 64) * 4;                       // [64][D] bf16
    float* lse_s = reinterpret_cast<float*>(obuf + kTile * kRowB);   // [64]
    if (c == 1) {
#pragma unroll
        for (int nb = 0; nb < D / 32; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i)
                xo[(32 * nb + 8 * (i >> 2) + 4 * hh + (i & 3)) * 32 + lq] = o[nb][i];
        if (hh == 0) {
            xo[32 * D + lq] = m_run;
            xo[32 * D + 32 + lq] = l_tot;
        }
    }
    __syncthreads();
    if (c == 0) {
        const float m1 = xo[32 * D + lq], l1 = xo[32 * D + 32 + lq];
        const float m_all = fmaxf(m_run, m1);
        const float m_use = m_all == -INFINITY ? 0.0f : m_all;
        const float a0 = __builtin_amdgcn_exp2f((m_run - m_use) * a.scale_log2);
        const float a1 = __builtin_amdgcn_exp2f((m1 - m_use) * a.scale_log2);
        const float l_all = l_tot * a0 + l1 * a1;
        const float inv = l_all > 0.0f ? 1.0f / l_all : 0.0f;
        const float w0 = a0 * inv, w1 = a1 * inv;
#pragma unroll
        for (int nb = 0; nb < D / 32; ++nb)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int d0 = 32 * nb + 8 * j + 4 * hh;
                typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
                bf16x4 pk;
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    pk[t] = (__bf16)(o[nb][4 * j + t] * w0 + xo[(d0 + t) * 32 + lq] * w1);
                *reinterpret_cast<bf16x4*>(obuf + (32 * r + lq) * kRowB + d0 * 2) = pk;
            }
        if (hh == 0) lse_s[32 * r + lq] = (m_use * a.scale_log2 + __log2f(l_all)) * kLn2;
    }
    __syncthreads();
    char* ob = a.out + b * a.so_b + head * a.so_h;
    for (int cid = tid; cid < kTile * kKChunks; cid += 256) {
        const int l = cid / kKChunks, ch = cid % kKChunks;
        const int n = slot_token(hg, qi, l, a.T, a.H, a.W);
        if (n >= 0)
            *reinterpret_cast<uint4*>(ob + (int64_t)n * a.so_n + ch * 16) =
                *reinterpret_cast<const uint4*>(obuf + l * kRowB + ch * 16);
    }
    if (a.lse && tid < kTile) {
        const int n = slot_token(hg, qi, tid, a.T, a.H, a.W);
        if (n >= 0) a.lse[(b * a.n_heads + head) * a.tokens + n] = lse_s[tid];
    }
}

// fp32 path: thread (q = tid/4, part = tid%4).  Scores of row q are spread over the 4 threads
// of a quad (keys part+4e); outputs likewise (channels part+4e).
template <int D>
__global__ __launch_bounds__(256) void sparse_attn_f32_kernel(AttnArgs a, float softmax_scale) {
    constexpr int kPitch = D + 1;
    __shared__ float ks[kTile * kPitch];
    __shared__ float ps[kTile * (kTile + 1)];
    const int tid = threadIdx.x, q = tid >> 2, part = tid & 3;
    const int64_t row = xcd_row(blockIdx.x, a.rows);
    const int64_t b = row / a.total_tiles;
    const int64_t g = row - b * a.total_tiles;
    const int head = a.tile_head[g];
    const HeadGeom hg = a.heads[head];
    const int qi = (int)(g - hg.tile_off);
    const int beg = a.row_ptr[row];
    const int nsel = a.row_ptr[row + 1] - beg;
    const int32_t* cols = a.col_idx + beg;
    const int64_t head_tile0 = b * a.total_tiles + hg.tile_off;
    const float* qrow = reinterpret_cast<const float*>(a.q) + ((head_tile0 + qi) * kTile + q) * D;
    const float* kt = reinterpret_cast<const float*>(a.k) + head_tile0 * kTile * D;
    const float* vt = reinterpret_cast<const float*>(a.v) + head_tile0 * kTile * D;
    const uint64_t* vmask = a.valid_mask + hg.tile_off;

    float o[D / 4];
#pragma unroll
    for (int e = 0; e < D / 4; ++e) o[e] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;

    for (int it = 0; it < nsel; ++it) {
        const int j = cols[it];
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
        float mloc = -INFINITY;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            s[e] = ((vm >> (part + 4 * e)) & 1ull) ? s[e] * softmax_scale : -INFINITY;
            mloc = fmaxf(mloc, s[e]);
        }
        mloc = fmaxf(mloc, __shfl_xor(mloc, 1));
        mloc = fmaxf(mloc, __shfl_xor(mloc, 2));
        const float m_new = fmaxf(m_run, mloc);
        const float m_use = m_new == -INFINITY ? 0.0f : m_new;
        const float alpha = expf(m_run - m_use);
        float psum = 0.0f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const float p = expf(s[e] - m_use);
            psum += p;
            ps[q * (kTile + 1) + part + 4 * e] = p;
        }
        psum += __shfl_xor(psum, 1);
        psum += __shfl_xor(psum, 2);
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int e = 0; e < D / 4; ++e) o[e] *= alpha;
        __syncthreads();
        const float* vsrc = vt + (int64_t)j * kTile * D;   // channel-major [D][64]
        for (int key = 0; key < kTile; ++key) {
            const float p = ps[q * (kTile + 1) + key];
#pragma unroll
            for (int e = 0; e < D / 4; ++e) o[e] = fmaf(p, vsrc[(part + 4 * e) * kTile + key], o[e]);
        }
    }
    const int n = slot_token(hg, qi, q, a.T, a.H, a.W);
    if (n >= 0) {
        const float inv = l_run > 0.0f ? 1.0f / l_run : 0.0f;
        float* orow = reinterpret_cast<float*>(a.out + b * a.so_b + head * a.so_h + (int64_t)n * a.so_n);
#pragma unroll
        for (int e = 0; e < D / 4; ++e) orow[part + 4 * e] = o[e] * inv;
        if (a.lse && part == 0) a.lse[(b * a.n_heads + head) * a.tokens + n] = m_run + logf(l_run);
    }
}

}  // namespace veda

extern "C" veda_status veda_sparse_attn_fwd(const veda_plan* pl, const void* q_tiled, const void* k_tiled,
                                            const void* v_tiled, const uint64_t* valid_mask,
                                            const int32_t* row_ptr, const int32_t* col_idx,
                                            float softmax_scale, void* out, veda_strides so, float* lse,
                                            void* stream) {
    using namespace veda;
    if (!pl || !q_tiled || !k_tiled || !v_tiled || !valid_mask || !row_ptr || !col_idx || !out)
        return VEDA_ERR_INVALID_ARG;
    if (!(softmax_scale > 0.0f) || !(softmax_scale < INFINITY)) return VEDA_ERR_INVALID_ARG;
    const int es = pl->elem_size(), d = pl->prob.head_dim;
    if (so.n < d || so.b < 0 || so.h < 0) return VEDA_ERR_INVALID_ARG;
    if (!aligned16(q_tiled) || !aligned16(k_tiled) || !aligned16(v_tiled) || !aligned16(out) ||
        (so.b * es) % 16 || (so.h * es) % 16 || (so.n * es) % 16)
        return VEDA_ERR_UNSUPPORTED;
    AttnArgs a;
    a.heads = pl->d_heads;
    a.tile_head = pl->d_tile_head;
    a.q = (const char*)q_tiled; a.k = (const char*)k_tiled; a.v = (const char*)v_tiled;
    a.valid_mask = valid_mask; a.row_ptr = row_ptr; a.col_idx = col_idx;
    a.out = (char*)out; a.lse = lse;
    a.total_tiles = pl->total_tiles;
    a.rows = pl->total_tiles * pl->prob.batch;
    a.so_b = so.b * es; a.so_h = so.h * es; a.so_n = so.n * es;
    a.tokens = pl->tokens();
    a.n_heads = pl->prob.heads; a.T = pl->prob.T; a.H = pl->prob.H; a.W = pl->prob.W;
    a.scale_log2 = softmax_scale * kLog2e;
    hipStream_t s = (hipStream_t)stream;
    dim3 grid((unsigned)a.rows), block(256);
    if (pl->prob.dtype == VEDA_BF16) {
        if (d == 128) {
            constexpr size_t smem = 2 * (64 * 256 + 128 * 128);
            static_assert(smem >= 2 * (32 * 128 + 64) * 4 + 64 * 256 + 256, "epilogue fits in the stages");
            hipLaunchKernelGGL(sparse_attn_bf16_kernel<128>, grid, block, smem, s, a);
        } else {
            constexpr size_t smem = 2 * (64 * 128 + 64 * 128);
            static_assert(smem >= 2 * (32 * 64 + 64) * 4 + 64 * 128 + 256, "epilogue fits in the stages");
            hipLaunchKernelGGL(sparse_attn_bf16_kernel<64>, grid, block, smem, s, a);
        }
    } else {
        if (d == 128) hipLaunchKernelGGL(sparse_attn_f32_kernel<128>, grid, block, 0, s, a, softmax_scale);
        else hipLaunchKernelGGL(sparse_attn_f32_kernel<64>, grid, block, 0, s, a, softmax_scale);
    }
    return launch_status("veda_sparse_attn_fwd");
}
