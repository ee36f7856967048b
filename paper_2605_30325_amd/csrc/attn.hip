// Stage 4 -- block-sparse flash attention forward + un-tiling (Eq. 2: softmax over the
// concatenation of the kept key tiles; Sec. 3.1 masked form; Sec. 4.3 tile-skipping kernel;
// Alg. 1 "UnTile"): the C entry points.  bf16 plans go to the kernel in attn_pair.hip, fp32
// plans to the one in attn_f32.hip; both run a workgroup per pair of partner query tiles.
#include "attn_common.h"

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
        return launch_sparse_attn_bf16_pair(ip, a, pl->inner != nullptr, pl->exact_logit_scale, pl->attn_list_walk, s);
    }
    a.xcd_cum = pl->d_xcd_cum_pair;
    return launch_sparse_attn_f32(pl, a, pl->attn_list_walk, s);
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
