// Stage 4 -- block-sparse flash attention forward + un-tiling (Eq. 2: softmax over the
// concatenation of the kept key tiles; Sec. 3.1 masked form; Sec. 4.3 tile-skipping kernel;
// Alg. 1 "UnTile"): the C entry point and the fp32 kernel.  bf16 inputs go to the MFMA kernel
// in attn_pair.hip.
//
// fp32 kernel: plain fp32 VALU arithmetic, one workgroup per query tile (small problems and
// the 1e-4 accuracy bar; not a throughput path).
#include "attn_common.h"

namespace veda {

// fp32 path: thread (q = tid/4, part = tid%4).  Scores of row q are spread over the 4 threads
// of a quad (keys part+4e); outputs likewise (channels part+4e).
template <int D>
__global__ __launch_bounds__(256) void sparse_attn_f32_kernel(AttnArgs a, float softmax_scale) {
    constexpr int kPitch = D + 1;
    __shared__ float ks[kTile * kPitch];
    __shared__ float ps[kTile * (kTile + 1)];
    const int tid = threadIdx.x, q = tid >> 2, part = tid & 3;
    int head, qi;
    if (!xcd_work(a.xcd_cum, a.heads, a.n_heads, 1, head, qi)) return;
    const HeadGeom hg = a.heads[head];
    const int64_t b = blockIdx.y;
    const int64_t row = b * a.total_tiles + hg.tile_off + qi;
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

namespace veda {

// Shared by the entry points: q_tiled or (q_tok, sq), k_tiled or (k_tok, sk).
static veda_status sparse_attn(const veda_plan* pl, const void* q_tiled, const void* q_tok, veda_strides sq,
                               const void* k_tiled, const void* k_tok, veda_strides sk, const void* v_tiled,
                               const uint64_t* valid_mask,
                               const int32_t* row_ptr, const int32_t* col_idx, float softmax_scale, void* out,
                               veda_strides so, float* lse, void* stream) {
    if (!pl || (!q_tiled && !q_tok) || (!k_tiled && !k_tok) || !v_tiled || !valid_mask || !row_ptr || !col_idx || !out)
        return VEDA_ERR_INVALID_ARG;
    if (!(softmax_scale > 0.0f) || !(softmax_scale < INFINITY)) return VEDA_ERR_INVALID_ARG;
    const int es = pl->elem_size(), d = pl->prob.head_dim;
    if (so.n < d || so.b < 0 || so.h < 0) return VEDA_ERR_INVALID_ARG;
    if (q_tok && (sq.n < d || sq.b < 0 || sq.h < 0)) return VEDA_ERR_INVALID_ARG;
    if (k_tok && (sk.n < d || sk.b < 0 || sk.h < 0)) return VEDA_ERR_INVALID_ARG;
    if ((q_tiled && !aligned16(q_tiled)) || (k_tiled && !aligned16(k_tiled)) || !aligned16(v_tiled) || !aligned16(out) ||
        (so.b * es) % 16 || (so.h * es) % 16 || (so.n * es) % 16)
        return VEDA_ERR_UNSUPPORTED;
    if (q_tok && (!aligned16(q_tok) || (sq.b * es) % 16 || (sq.h * es) % 16 || (sq.n * es) % 16 ||
                  pl->prob.dtype != VEDA_BF16))
        return VEDA_ERR_UNSUPPORTED;
    // a key row's byte offset from its tile's anchor token (plus a bias below 4 KiB) is kept in 32 bits
    if (k_tok && (!aligned16(k_tok) || (sk.b * es) % 16 || (sk.h * es) % 16 || (sk.n * es) % 16 ||
                  pl->prob.dtype != VEDA_BF16 || pl->tokens() * sk.n * es >= ((int64_t)1 << 32) - 4096))
        return VEDA_ERR_UNSUPPORTED;
    // 128-token tiles: the kernel works on the 64-slot halves (inner plan), the CSR on whole tiles
    const veda_plan* ip = pl->inner ? pl->inner : pl;
    AttnArgs a;
    a.heads = ip->d_heads;
    a.tile_head = ip->d_tile_head;
    a.q = (const char*)q_tiled; a.k = (const char*)k_tiled; a.v = (const char*)v_tiled;
    a.q_tok = (const char*)q_tok;
    a.sq_b = sq.b * es; a.sq_h = sq.h * es; a.sq_n = sq.n * es;
    a.k_tok = (const char*)k_tok;
    a.sk_b = sk.b * es; a.sk_h = sk.h * es; a.sk_n = sk.n * es;
    a.tile_n0 = ip->d_tile_n0;
    a.valid_mask = valid_mask; a.row_ptr = row_ptr; a.col_idx = col_idx;
    a.out = (char*)out; a.lse = lse;
    a.total_tiles = ip->total_tiles;
    a.rows = ip->total_tiles * pl->prob.batch;
    a.so_b = so.b * es; a.so_h = so.h * es; a.so_n = so.n * es;
    a.tokens = pl->tokens();
    a.n_heads = pl->prob.heads; a.T = pl->prob.T; a.H = pl->prob.H; a.W = pl->prob.W;
    a.scale_log2 = softmax_scale * kLog2e;
    {
        int ex = 0;
        const float mant = frexpf(a.scale_log2, &ex);   // scale_log2 = mant * 2^ex, 0.5 <= mant < 1
        a.scale_pow2 = ldexpf(1.0f, ex - 1);
        a.scale_resid = 2.0f * mant;
    }
    hipStream_t s = (hipStream_t)stream;
    if (pl->prob.dtype == VEDA_BF16) {
        a.xcd_cum = ip->d_xcd_cum_pair;
        return launch_sparse_attn_bf16_pair(ip, a, pl->inner != nullptr, pl->exact_logit_scale, s);
    }
    a.xcd_cum = pl->d_xcd_cum;
    dim3 grid((unsigned)(kXcd * pl->xcd_max_tiles), (unsigned)pl->prob.batch), block(256);
    if (d == 128) hipLaunchKernelGGL(sparse_attn_f32_kernel<128>, grid, block, 0, s, a, softmax_scale);
    else hipLaunchKernelGGL(sparse_attn_f32_kernel<64>, grid, block, 0, s, a, softmax_scale);
    return launch_status("veda_sparse_attn_fwd");
}

}  // namespace veda

extern "C" veda_status veda_sparse_attn_fwd(const veda_plan* pl, const void* q_tiled, const void* k_tiled,
                                            const void* v_tiled, const uint64_t* valid_mask,
                                            const int32_t* row_ptr, const int32_t* col_idx,
                                            float softmax_scale, void* out, veda_strides so, float* lse,
                                            void* stream) {
    if (!q_tiled) return VEDA_ERR_INVALID_ARG;
    if (!k_tiled) return VEDA_ERR_INVALID_ARG;
    return veda::sparse_attn(pl, q_tiled, nullptr, veda_strides{0, 0, 0}, k_tiled, nullptr, veda_strides{0, 0, 0},
                             v_tiled, valid_mask, row_ptr, col_idx, softmax_scale, out, so, lse, stream);
}

extern "C" veda_status veda_sparse_attn_fwd_q_tokens(const veda_plan* pl, const void* q, veda_strides sq,
                                                     const void* k_tiled, const void* v_tiled,
                                                     const uint64_t* valid_mask, const int32_t* row_ptr,
                                                     const int32_t* col_idx, float softmax_scale, void* out,
                                                     veda_strides so, float* lse, void* stream) {
    if (!q || !k_tiled) return VEDA_ERR_INVALID_ARG;
    return veda::sparse_attn(pl, nullptr, q, sq, k_tiled, nullptr, veda_strides{0, 0, 0}, v_tiled, valid_mask, row_ptr,
                             col_idx, softmax_scale, out, so, lse, stream);
}

extern "C" veda_status veda_sparse_attn_fwd_qk_tokens(const veda_plan* pl, const void* q, veda_strides sq,
                                                      const void* k, veda_strides sk, const void* v_tiled,
                                                      const uint64_t* valid_mask, const int32_t* row_ptr,
                                                      const int32_t* col_idx, float softmax_scale, void* out,
                                                      veda_strides so, float* lse, void* stream) {
    if (!q || !k) return VEDA_ERR_INVALID_ARG;
    return veda::sparse_attn(pl, nullptr, q, sq, nullptr, k, sk, v_tiled, valid_mask, row_ptr, col_idx, softmax_scale,
                             out, so, lse, stream);
}
