/*
 * veda.h -- C ABI of the MI355X (gfx950) tile-sparse attention path for video DiTs:
 * head-aware 3D tiling -> statistics-aware tile scoring -> per-query-tile top-k ->
 * block-sparse flash attention with scatter back to token order.
 *
 * Conventions (all entry points):
 *  - "device" pointers are HIP device memory owned by the caller; "host" pointers are
 *    ordinary host memory read during the call.  The library allocates device memory only
 *    inside veda_plan_create (a few KB of per-head tables, freed by veda_plan_destroy).
 *  - Every stage call only enqueues kernels on `stream` (a hipStream_t passed as void*; NULL
 *    is the default stream) and returns without synchronising.
 *  - Arguments are checked on the host before anything is launched; a failed check returns
 *    an error code and launches nothing.  HIP launch failures map to VEDA_ERR_HIP.
 *  - No data-dependent scheduling of arithmetic and no floating-point atomics: equal inputs give
 *    equal bytes.  (The only atomics are integer ones whose result does not depend on their
 *    order: the adds of veda_tile_recall's hit counters, and the bit-sets in LDS with which the
 *    attention kernels turn a kept list into a bitmap.)
 *  - Tokens are the raster flattening n = (t*H + h)*W + w of a latent grid (T,H,W)
 *    (Sec. 3.1).  A head's tile shape pi = (p_t,p_h,p_w) with p_t*p_h*p_w = B (Eq. 7)
 *    partitions the grid, each axis padded up to a multiple of the tile extent.  Tile i and
 *    slot l of a token are
 *        i = ((t/p_t)*n_h + h/p_h)*n_w + w/p_w,   l = ((t%p_t)*p_h + h%p_h)*p_w + w%p_w
 *    so temporal neighbours inside a tile are p_h*p_w slots apart (App. A.5).  Heads may
 *    have different shapes, hence different tile counts N_T[h]; tiles of all heads are
 *    concatenated head by head ("global tile index" g = tile_off[h] + i).
 *  - Supported: B = 64 (f32 or bf16) and B = 128 (bf16 only; see veda_problem), head_dim in
 *    {64,128}, heads <= 128.
 */
#ifndef VEDA_H_
#define VEDA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    VEDA_OK = 0,
    VEDA_ERR_INVALID_ARG = 1,  /* null pointer, inconsistent sizes, k out of range, ...   */
    VEDA_ERR_UNSUPPORTED = 2,  /* a valid request outside what the kernels are built for   */
    VEDA_ERR_WORKSPACE = 3,    /* workspace_bytes smaller than veda_plan_workspace_bytes() */
    VEDA_ERR_HIP = 4           /* a HIP runtime call or kernel launch failed               */
} veda_status;

typedef enum { VEDA_F32 = 0, VEDA_BF16 = 1 } veda_dtype;
typedef enum { VEDA_ACT_IDENTITY = 0, VEDA_ACT_RELU = 1 } veda_act;

/* Order of the 64 x d elements inside one tile of a tiled tensor. */
typedef enum {
    VEDA_TOKEN_MAJOR = 0,   /* [slot][channel]  -- used for Q~ and K~                      */
    VEDA_CHANNEL_MAJOR = 1  /* [channel][slot]  -- used for V~ (K-major operand of P*V)     */
} veda_tile_order;

typedef struct veda_plan veda_plan; /* opaque; owned by the library */

/* One self-attention call of one layer (Sec. 3.1; Alg. 2 inputs). */
typedef struct {
    int32_t batch, heads, head_dim;
    int32_t T, H, W;            /* latent grid; N = T*H*W tokens                            */
    int32_t tile_tokens;        /* B: 64, or 128 (the size of Sec. 4.2; bf16 only) -- see below */
    const int32_t* tile_shape;  /* host, [heads][3] = (p_t,p_h,p_w), product == B (Eq. 7)   */
    veda_dtype dtype;           /* element type of Q,K,V,O and of the tiled tensors         */
} veda_problem;

/* 128-token tiles are kept as two 64-slot halves: a tile is cut across its slowest axis of extent
 * > 1, so slots 0-63 (raster order, time slowest) are one half and slots 64-127 the other.
 * Everything that counts tiles (plan sizes, scores, k, CSR rows and entries) counts whole tiles;
 *   a token-major tiled tensor is [tile][128][channel] as for any B;
 *   a channel-major tiled tensor is [tile][half][channel][64];
 *   valid_mask holds two u64 words per tile (word w covers slots 64w..64w+63);
 *   veda_tile_layout needs valid_mask whenever valid_cnt is asked for. */

/* Element strides of a token-order tensor x[b][h][n][c]; the channel stride is 1.
 * Each stride must be a multiple of 16 bytes and the base 16-byte aligned. */
typedef struct { int64_t b, h, n; } veda_strides;

/* Per-head projection phi of the score estimator (Eq. 5): y = W2^T act(W1^T z + b1) + b2,
 * or, with hidden == 0, the single affine layer y = W1^T z + b1 (w2,b2 ignored).
 * Device fp32 arrays, one block per head, row-major [in][out]:
 *   w1 [heads][in_dim][hidden ? hidden : out_dim], b1 [heads][hidden ? hidden : out_dim],
 *   w2 [heads][hidden][out_dim],                    b2 [heads][out_dim].                   */
typedef struct {
    int32_t in_dim;   /* must be 3*head_dim (Avg|Max|Min)          */
    int32_t hidden;   /* 0 or 1..512                                */
    int32_t out_dim;  /* latent size d', 1..256, multiple of 4      */
    veda_act act;
    const float *w1, *b1, *w2, *b2;
} veda_mlp;

/* ---- plan: host-side geometry of a problem --------------------------------------------- */

/* Validates the problem, derives each head's tile grid and offsets, uploads the per-head
 * table to the current device.  The first plan made on a device also resolves the address of
 * the no-allocation entry point's scratch array there and measures where stage 2's fp32 chains
 * may run (VEDA_OPT_FP32_CHAIN_UNIT): a few small kernel launches on the default stream and one
 * copy back, synchronous.  Not to be called under stream capture.  *out is written only on
 * VEDA_OK. */
veda_status veda_plan_create(const veda_problem* problem, veda_plan** out);
void veda_plan_destroy(veda_plan* plan); /* NULL is allowed */

/* Options of a plan; they take effect for the stage calls made after the setter returns.
 * VEDA_OPT_EXACT_LOGIT_SCALE (0 = off, the default; 1 = on), bf16 stage 4 (Eq. 2): see
 * veda_sparse_attn_fwd.
 * VEDA_OPT_ATTN_LIST_WALK (0 = off, the default; 1 = on), stage 4 (Sec. 4.3): the kernel
 * normally works out, before its main loop, the order in which a workgroup visits the key tiles
 * its query tiles keep (ascending, whatever the order inside the lists) into a table in LDS;
 * with this option it merges the lists as it goes instead, reading them entry by entry (then
 * ascending rows share the most loads).  The table covers heads of up to 16384 tiles; larger
 * heads take the walk on their own.  Both orders give the same O up to rounding, and the same
 * bits when the rows are ascending.
 * VEDA_OPT_FP32_CHAIN_UNIT (0 = as probed, the default; VEDA_CHAINS_MATRIX; VEDA_CHAINS_VECTOR),
 * stage 2 (Eq. 5): where the fixed-order fp32 chains of the projections and of the score matrix
 * run.  They are defined as scalar fmaf chains; on gfx950 chains of v_mfma_f32_32x32x2_f32 give
 * the same bits at twice the rate, which is a measured property of that instruction.
 * veda_plan_create measures it on the plan's device (both forms on chains with rounding,
 * signed zeros and denormal sums and products, once per device) and uses the matrix cores only
 * if every bit agrees; this option overrides the choice either way.
 * veda_plan_chain_unit tells which unit the plan's next call will use. */
typedef enum { VEDA_OPT_EXACT_LOGIT_SCALE = 0, VEDA_OPT_ATTN_LIST_WALK = 1, VEDA_OPT_FP32_CHAIN_UNIT = 2 } veda_option;
enum { VEDA_CHAINS_MATRIX = 1, VEDA_CHAINS_VECTOR = 2 };
veda_status veda_plan_set_option(veda_plan*, veda_option option, int32_t value);
int32_t veda_plan_chain_unit(const veda_plan*);          /* VEDA_CHAINS_*; -1 on bad args */

int32_t veda_plan_tiles(const veda_plan*, int32_t head);      /* N_T[h]; -1 on bad args        */
int64_t veda_plan_tile_offset(const veda_plan*, int32_t head);/* tile_off[h] = sum_{h'<h} N_T  */
int64_t veda_plan_score_offset(const veda_plan*, int32_t head);/* sum_{h'<h} N_T[h']^2          */
int64_t veda_plan_total_tiles(const veda_plan*);              /* sum_h N_T[h]                  */
int64_t veda_plan_score_elems(const veda_plan*);              /* sum_h N_T[h]^2 (per batch)    */
/* Bytes of scratch veda_tile_score needs for the given projections (descriptors, hidden layers
 * and latents). */
size_t veda_plan_workspace_bytes(const veda_plan*, const veda_mlp* phi_q, const veda_mlp* phi_k);
/* Where veda_tile_score leaves its intermediates in the workspace, as offsets in floats from its
 * start; each array is [batch*total_tiles] rows: TripPool descriptors z = [Avg|Max|Min] of Q and
 * K (3*head_dim floats per row, Eq. 4) and latents phi_q(z_q), phi_k(z_k) (out_dim floats per
 * row, Eq. 5).  veda_tile_score_stats leaves only the latents, at latent_q - 2*stats and
 * latent_k - 2*stats, i.e. at the start of its workspace (stats = batch*total_tiles*3*head_dim). */
typedef struct { int64_t stats_q, stats_k, latent_q, latent_k; } veda_workspace_layout;
veda_status veda_plan_workspace_layout(const veda_plan*, const veda_mlp* phi_q, const veda_mlp* phi_k,
                                       veda_workspace_layout* out);

/* ---- stage 1: head-aware 3D tiling (Sec. 4.2; Alg. 1 "Tiling"; Alg. 2 "Tile") ----------- */
/* x        device, token order, strides sx, plan dtype.
 * x_tiled  device, [batch][total_tiles][B*head_dim] in `order`; padded slots are zero.
 * valid_mask device u64 [total_tiles][B/64] (bit l set iff slot l holds a real token) and
 * valid_cnt  device i32 [total_tiles] (its popcount); either may be NULL.  Both depend
 * only on the geometry, not on x or the batch index. */
veda_status veda_tile_layout(const veda_plan*, const void* x, veda_strides sx, veda_tile_order order,
                             void* x_tiled, uint64_t* valid_mask, int32_t* valid_cnt, void* stream);

/* ---- stage 2: statistics-aware tile scoring (Eq. 4, Eq. 5; Alg. 2) ---------------------- */
/* q_tiled,k_tiled  device, VEDA_TOKEN_MAJOR tiled tensors from stage 1.
 * scores   device fp32 [batch][score_elems]; head h occupies a dense row-major
 *          N_T[h] x N_T[h] block at score_offset(h): S[i][j] = phi_q(z_q,i).phi_k(z_k,j)*scale,
 *          z = [Avg|Max|Min] over the tile's real tokens, per channel.
 * Arithmetic is fp32 with a fixed order (slot-ascending add chain for Avg; one fma chain per
 * output in ascending input index, started from the bias, for phi; one fma chain from +0 in
 * ascending latent index, then one multiply by `scale`, for the score), so any conforming fp32
 * implementation of that order gives the same bits.  On gfx950 the projection chains and the
 * chains of veda_tile_score's score matrix are issued as v_mfma_f32_32x32x2_f32 over ascending
 * index pairs: that this instruction applies its two terms one after the other, each rounded as
 * an fma, denormals kept, is a property measured on gfx950, not one its ISA manual states: the
 * library measures it again on every device it meets (veda_plan_create) and runs these chains as
 * scalar fmaf on the vector units wherever a bit differs (VEDA_OPT_FP32_CHAIN_UNIT forces either
 * form).  The fused route (veda_tile_score_select*) forms its scores with plain fmaf chains on
 * the vector units in any case; its projections follow the same choice.
 * workspace device scratch of at least veda_plan_workspace_bytes().  After the call it holds the
 * stage's intermediates at the float offsets veda_plan_workspace_layout() reports (descriptors
 * and latents, one row per (batch, global tile)); the rest is undefined. */
veda_status veda_tile_score(const veda_plan*, const void* q_tiled, const void* k_tiled,
                            const uint64_t* valid_mask, const veda_mlp* phi_q, const veda_mlp* phi_k,
                            float scale, float* scores, void* workspace, size_t workspace_bytes,
                            void* stream);

/* ---- stages 1 + 2 with the descriptors taken during the gather (Eq. 4; the Conclusion
 * names tighter fusion of mask preparation as the next step for the kernels) --------------- */
/* veda_tile_layout_stats = veda_tile_layout(VEDA_TOKEN_MAJOR) that also writes
 * stats   device fp32 [batch][total_tiles][3*head_dim] = [Avg|Max|Min] of every tile over its
 *         real tokens, per channel, bit-identical to the descriptors veda_tile_score derives.
 *         x_tiled may be NULL: descriptors (and masks) only.
 * veda_tile_score_stats = veda_tile_score starting from such descriptors (stats_q of Q, stats_k
 * of K); workspace needs batch*total_tiles*2*out_dim floats; given batch*total_tiles*(hidden_q +
 * hidden_k) floats more (veda_plan_workspace_bytes() is enough) the hidden layers pass through
 * it and the projections run faster.  scores are bit-identical to veda_tile_score on the same
 * inputs either way. */
veda_status veda_tile_layout_stats(const veda_plan*, const void* x, veda_strides sx, void* x_tiled,
                                   uint64_t* valid_mask, int32_t* valid_cnt, float* stats, void* stream);
veda_status veda_tile_score_stats(const veda_plan*, const float* stats_q, const float* stats_k,
                                  const veda_mlp* phi_q, const veda_mlp* phi_k, float scale, float* scores,
                                  void* workspace, size_t workspace_bytes, void* stream);

/* ---- stage 2 without trained weights (App. A.3 "Reconstructing Attention via Sufficient
 * Statistics": S ~ mean product + lambda * dispersion product, dispersion bounded from the
 * extrema).  The appendix states it for the elements of one vector; it is applied here per
 * channel to the TripPool descriptor [Avg|Max|Min] of a tile:
 *   S[i][j] = sum_c avg_q[i][c]*avg_k[j][c] + lambda * sum_c D_q[i][c]*D_k[j][c],
 *   D = sqrt(max(0, (Max - Avg)*(Avg - Min))),
 * computed in fp32 as the plain dot product (one fma chain from +0 over ascending index) of the
 * 2*head_dim-long latents [Avg | sqrtf(lambda)*D].  scores as in veda_tile_score; lambda >= 0;
 * workspace at least batch*total_tiles*10*head_dim floats. */
veda_status veda_tile_score_closed_form(const veda_plan*, const void* q_tiled, const void* k_tiled,
                                        const uint64_t* valid_mask, float lambda, float* scores,
                                        void* workspace, size_t workspace_bytes, void* stream);

/* ---- stage 3: per-query-tile top-k (Sec. 3.1 "exactly k per row"; Sec. 4.1; Alg. 2) ------ */
/* scores      device, as written by stage 2.
 * k_per_head  host i32 [heads], 1 <= k[h] <= N_T[h].
 * row_ptr     device i32 [batch*total_tiles + 1]; row r = b*total_tiles + g.
 * col_idx     device i32 [batch * sum_h N_T[h]*k[h]]; for each row the k[h] kept key tiles,
 *             head-local indices in ascending order.
 * A key tile is kept iff fewer than k[h] tiles of the row rank before it, where j ranks
 * before j' if s_j > s_j', or s_j == s_j' and j < j' (NaN counts as -inf, -0 as +0). */
veda_status veda_tile_select(const veda_plan*, const float* scores, const int32_t* k_per_head,
                             int32_t* row_ptr, int32_t* col_idx, void* stream);

/* ---- stages 2 + 3 in one call, the score matrix never written (Eq. 5; Sec. 3.1 "exactly k
 * per row"; Alg. 2; the Conclusion names tighter fusion of mask preparation as the next step
 * for the kernels) ---------------------------------------------------------------------------- */
/* veda_tile_score_select       = veda_tile_score followed by veda_tile_select,
 * veda_tile_score_select_stats = veda_tile_score_stats followed by veda_tile_select,
 * with identical row_ptr / col_idx (same arithmetic, same order, same tie rule), but for heads
 * with at least 1024 tiles, a small keep budget and out_dim <= 64 every score is compared with a
 * per-row pivot as soon as it is formed and only the candidates of the row's top-k reach memory;
 * a row whose candidates do not hold its top-k is redone on its full score row.  Other shapes
 * take the two-stage route inside the call.
 * workspace  device scratch of at least veda_plan_fused_workspace_bytes() (latents, candidate
 *            lists, and room for the score matrix, of which only redone rows are touched);
 *            contents undefined after. */
size_t veda_plan_fused_workspace_bytes(const veda_plan*, const veda_mlp* phi_q, const veda_mlp* phi_k);
veda_status veda_tile_score_select(const veda_plan*, const void* q_tiled, const void* k_tiled,
                                   const uint64_t* valid_mask, const veda_mlp* phi_q, const veda_mlp* phi_k,
                                   float scale, const int32_t* k_per_head, int32_t* row_ptr, int32_t* col_idx,
                                   void* workspace, size_t workspace_bytes, void* stream);
veda_status veda_tile_score_select_stats(const veda_plan*, const float* stats_q, const float* stats_k,
                                         const veda_mlp* phi_q, const veda_mlp* phi_k, float scale,
                                         const int32_t* k_per_head, int32_t* row_ptr, int32_t* col_idx,
                                         void* workspace, size_t workspace_bytes, void* stream);

/* ---- stages 2 + 3 for callers that cannot allocate device memory or bring a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc ---------------------- */
/* veda_tile_score_select_stats_noalloc = veda_tile_score_select_stats (same arguments, same row_ptr /
 * col_idx bit for bit) with the workspace taken from a fixed array of VEDA_NOALLOC_SCRATCH_BYTES that
 * the library holds in the memory of every GPU it is loaded on until the process ends.  The call
 * makes no hipMalloc / hipFree and calls no allocating routine; it only enqueues kernels on `stream`.
 * A plan with veda_plan_fused_workspace_bytes() above VEDA_NOALLOC_SCRATCH_BYTES is refused with
 * VEDA_ERR_WORKSPACE (veda_last_error() names both sizes) and nothing is launched; the plan's device
 * must be the current device.  Every call on a GPU uses that GPU's one array: calls that may overlap
 * on one GPU (different streams, different threads) race on it and must be serialised by the
 * caller.  The array keeps the last call's contents; nothing in it has to start at zero. */
#define VEDA_NOALLOC_SCRATCH_BYTES ((size_t)128 << 20)
veda_status veda_tile_score_select_stats_noalloc(const veda_plan*, const float* stats_q, const float* stats_k,
                                                 const veda_mlp* phi_q, const veda_mlp* phi_k, float scale,
                                                 const int32_t* k_per_head, int32_t* row_ptr, int32_t* col_idx,
                                                 void* stream);

/* ---- stage 4: block-sparse flash attention + un-tiling (Eq. 2; Sec. 4.3; Alg. 1 "UnTile") -- */
/* q_tiled,k_tiled  VEDA_TOKEN_MAJOR; v_tiled VEDA_CHANNEL_MAJOR; valid_mask from stage 1.
 * row_ptr/col_idx  CSR lists as written by stage 3 (any order within a row is accepted, no
 *                  index twice in a row; every row needs at least one entry, indices in
 *                  [0, N_T[h]); ascending rows let adjacent query tiles share loads).
 * out      device, token order, strides so, plan dtype: for every real query token u of
 *          query tile i, O[u] = softmax over the real tokens of the kept key tiles of
 *          (q_u.k_v * softmax_scale) applied to V.  Padded query slots write nothing.
 * lse      optional device fp32 [batch][heads][N]: natural-log sum of exp of the kept logits.
 * bf16: Q K^T and P V run on bf16 MFMA with fp32 accumulation, softmax in fp32, P is rounded to
 * bf16 before P V.  By default Q is multiplied by softmax_scale*log2(e) and rounded to bf16 once:
 * an error in every logit of about 2^-9 of its size, so the output error grows with the logits
 * (measured against the double-precision definition on N(0,1) keys and values: max-abs 5e-3 /
 * mean-abs 4e-4 with logits q.k*softmax_scale of standard deviation 1, 1.4e-2 / 7e-4 at 2,
 * 2.4e-2 / 1.6e-3 at 4, 5e-2 / 2e-3 at 6; lse 2e-3 ... 5e-2) and passes max-abs 2e-2 beyond a
 * standard deviation of about 3.  With VEDA_OPT_EXACT_LOGIT_SCALE Q is multiplied by the power
 * of two nearest below that factor (exact in bf16) and the logits by the remaining factor in fp32
 * on their way into the exponential: the error no longer depends on the logits' size (max-abs
 * <= 1.7e-2, mean-abs <= 1e-3, lse 1e-5 up to a standard deviation of 16) at about 4 % more time.
 * f32: fp32 arithmetic throughout. */
veda_status veda_sparse_attn_fwd(const veda_plan*, const void* q_tiled, const void* k_tiled,
                                 const void* v_tiled, const uint64_t* valid_mask,
                                 const int32_t* row_ptr, const int32_t* col_idx, float softmax_scale,
                                 void* out, veda_strides so, float* lse, void* stream);
/* The same with Q taken straight from token order (q, strides sq; bf16 plans only): the kernel
 * gathers each query tile's rows itself, so the tiled copy of Q need not be written at all
 * (veda_tile_layout_stats with x_tiled = NULL still gives its descriptors and the masks).
 * Results are bit-identical to veda_sparse_attn_fwd on the tiled Q. */
veda_status veda_sparse_attn_fwd_q_tokens(const veda_plan*, const void* q, veda_strides sq, const void* k_tiled,
                                          const void* v_tiled, const uint64_t* valid_mask,
                                          const int32_t* row_ptr, const int32_t* col_idx, float softmax_scale,
                                          void* out, veda_strides so, float* lse, void* stream);
/* And with K from token order as well (k, strides sk; bf16 plans; tokens * sk.n * 2 bytes must stay
 * below 4 GiB - 4 KiB): every kept key tile is gathered row by row on its way into the compute unit, so
 * only V needs a tiled copy.  Bit-identical results again.  Both token-order entry points take
 * either tile size (with B = 128 the kernel gathers the two 64-slot halves of a tile). */
veda_status veda_sparse_attn_fwd_qk_tokens(const veda_plan*, const void* q, veda_strides sq, const void* k,
                                           veda_strides sk, const void* v_tiled, const uint64_t* valid_mask,
                                           const int32_t* row_ptr, const int32_t* col_idx, float softmax_scale,
                                           void* out, veda_strides so, float* lse, void* stream);

/* ---- supervision side: target tile scores of full attention and tile recall ------------- */
/* veda_tile_heatmap (Sec. 4.1 Eq. 3; Sec. 4.3 "Efficient Ground-Truth Heatmap Generation"):
 * heat     device fp32 [batch][score_elems], same per-head block layout as the scores of
 *          stage 2: heat[i][j] = max over the real tokens u of query tile i and v of key tile j
 *          of Softmax_v(q_u.k_v * softmax_scale), the softmax running over ALL real tokens of
 *          the head (full attention).  Exact pooled values in two passes over the key tiles;
 *          the attention map is never stored.
 * query_tiles  optional device i32 [n_query_tiles] of global tile indices (tile_offset(h) + i,
 *          each in [0, total_tiles), no index twice): only those rows of heat are written, for
 *          every batch entry; NULL with n_query_tiles == 0 means all query tiles.
 * q_tiled,k_tiled VEDA_TOKEN_MAJOR.  bf16: Q K^T on bf16 MFMA, fp32 accumulation and softmax. */
veda_status veda_tile_heatmap(const veda_plan*, const void* q_tiled, const void* k_tiled,
                              const uint64_t* valid_mask, float softmax_scale, const int32_t* query_tiles,
                              int64_t n_query_tiles, float* heat, void* stream);
/* veda_tile_recall (Sec. 3.2, Recall@k): col_idx_a, col_idx_b device CSR column lists as stage 3
 * writes them for the same k_per_head (host i32 [heads]); each row a list of distinct tiles.
 * recall   device fp32 [batch][heads]: mean over the head's query tiles of |A_i & B_i| / k.
 * workspace device, 8-byte aligned, at least 8*batch*heads bytes. */
veda_status veda_tile_recall(const veda_plan*, const int32_t* k_per_head, const int32_t* col_idx_a,
                             const int32_t* col_idx_b, float* recall, void* workspace,
                             size_t workspace_bytes, void* stream);

/* veda_output_sqerr (Eq. 8; Alg. 1 "Compute Sparse Output and Error"): a, b device tensors in
 * token order with strides sa, sb (plan dtype); err device fp64 [batch][heads] =
 * sum over tokens and channels of (a - b)^2, accumulated in double in a fixed order.
 * workspace device, 8-byte aligned, at least 8*64*batch*heads bytes.  The tiling search of
 * Sec. 4.2 is this call around stages 1, heat map, 3 and 4 for every candidate tile shape. */
veda_status veda_output_sqerr(const veda_plan*, const void* a, veda_strides sa, const void* b, veda_strides sb,
                              double* err, void* workspace, size_t workspace_bytes, void* stream);

const char* veda_status_string(veda_status);
/* Text of the last HIP error seen by this thread inside the library ("" if none). */
const char* veda_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* VEDA_H_ */
