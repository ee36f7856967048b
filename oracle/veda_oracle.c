/*
 * CPU oracle for the tile-sparse attention path (Veda inference hot path).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * GPU library must compute.  It shares no code with the HIP kernels and must
 * never be reached from the product path; only tests, the smoke check and the
 * CPU-baseline leg of the benchmark call it.
 *
 * Every function works on ONE attention head, in the ORIGINAL token order
 * n = (t*H + h)*W + w (Sec. 3.1, "flattened into a token sequence of length
 * N = THW"), so that no function depends on another function's tiling code
 * except where stated.  A tile shape pi = (pt, ph, pw) with pt*ph*pw = B
 * (Eq. 7) partitions the ceil-padded grid; tile index and in-tile index are
 * both raster order with time slowest (App. A.5: temporal neighbours inside a
 * tile end up ph*pw apart).
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC.  Floating-point
 * contraction is off and the score path spells out fmaf(), because the
 * fp32 scores decide an integer (the top-k set) and the order of operations
 * is therefore part of the definition.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int T, H, W;     /* latent grid */
    int pt, ph, pw;  /* tile extents */
    int nt, nh, nw;  /* tile grid = ceil(grid / tile) */
} vo_geom;

static int vo_make_geom(vo_geom* g, int T, int H, int W, int pt, int ph, int pw) {
    if (T <= 0 || H <= 0 || W <= 0 || pt <= 0 || ph <= 0 || pw <= 0) return -1;
    g->T = T; g->H = H; g->W = W; g->pt = pt; g->ph = ph; g->pw = pw;
    g->nt = (T + pt - 1) / pt; g->nh = (H + ph - 1) / ph; g->nw = (W + pw - 1) / pw;
    return 0;
}

/* Number of tiles of the ceil-padded grid (Sec. 3.1: N tokens -> N_T tiles of size B;
 * grids that do not divide are padded up per axis). */
int64_t vo_num_tiles(int T, int H, int W, int pt, int ph, int pw) {
    vo_geom g;
    if (vo_make_geom(&g, T, H, W, pt, ph, pw)) return -1;
    return (int64_t)g.nt * g.nh * g.nw;
}

/* token (t,h,w) -> tile index i and slot l inside the tile */
static void vo_token_to_slot(const vo_geom* g, int t, int h, int w, int64_t* i, int* l) {
    *i = ((int64_t)(t / g->pt) * g->nh + (h / g->ph)) * g->nw + (w / g->pw);
    *l = ((t % g->pt) * g->ph + (h % g->ph)) * g->pw + (w % g->pw);
}

/* int32 [N]: tile index of every token. */
int vo_token_tile_map(int T, int H, int W, int pt, int ph, int pw, int32_t* tile_of) {
    vo_geom g;
    if (vo_make_geom(&g, T, H, W, pt, ph, pw)) return -1;
    for (int t = 0; t < T; ++t)
        for (int h = 0; h < H; ++h)
            for (int w = 0; w < W; ++w) {
                int64_t i; int l;
                vo_token_to_slot(&g, t, h, w, &i, &l);
                tile_of[((int64_t)t * H + h) * W + w] = (int32_t)i;
            }
    return 0;
}

/*
 * Stage 1 -- head-aware 3D tiling (Sec. 4.2 pi = (pt,ph,pw); Alg. 1 "Tiling"; Alg. 2 "Tile").
 * x        [N][d]   elements of elem_size bytes, token order
 * x_tiled  token-major  [N_T][B][d]  (channel_major == 0)
 *          channel-major [N_T][d][B] (channel_major != 0)
 * Padded slots are zero bytes.  valid_mask holds ceil(B/64) words per tile: bit l%64 of word
 * l/64 of tile i is set iff slot l holds a real token; valid_cnt[i] is the tile's population
 * count.  B <= 128 (the paper's tile size, Sec. 4.2).  Byte moves only.
 */
int vo_tile_layout(const void* x, int64_t elem_size, int d, int T, int H, int W,
                   int pt, int ph, int pw, int channel_major,
                   void* x_tiled, uint64_t* valid_mask, int32_t* valid_cnt) {
    vo_geom g;
    if (vo_make_geom(&g, T, H, W, pt, ph, pw)) return -1;
    const int B = pt * ph * pw;
    if (B > 128) return -2;
    const int words = (B + 63) / 64;
    const int64_t n_tiles = (int64_t)g.nt * g.nh * g.nw;
    memset(x_tiled, 0, (size_t)(n_tiles * B * d * elem_size));
    if (valid_mask) memset(valid_mask, 0, (size_t)n_tiles * words * sizeof(uint64_t));
    if (valid_cnt) memset(valid_cnt, 0, (size_t)n_tiles * sizeof(int32_t));
    const char* src = (const char*)x;
    char* dst = (char*)x_tiled;
    for (int t = 0; t < T; ++t)
        for (int h = 0; h < H; ++h)
            for (int w = 0; w < W; ++w) {
                const int64_t n = ((int64_t)t * H + h) * W + w;
                int64_t i; int l;
                vo_token_to_slot(&g, t, h, w, &i, &l);
                for (int c = 0; c < d; ++c) {
                    const int64_t o = channel_major ? ((i * d + c) * B + l) : ((i * B + l) * d + c);
                    memcpy(dst + o * elem_size, src + (n * d + c) * elem_size, (size_t)elem_size);
                }
                if (valid_mask) valid_mask[i * words + l / 64] |= (uint64_t)1 << (l % 64);
                if (valid_cnt) valid_cnt[i] += 1;
            }
    return 0;
}

/* Inverse of stage 1 for the token-major form (Alg. 1 "UnTile"): y[n] = y_tiled[slot(n)]. */
int vo_untile(const void* y_tiled, int64_t elem_size, int d, int T, int H, int W,
              int pt, int ph, int pw, void* y) {
    vo_geom g;
    if (vo_make_geom(&g, T, H, W, pt, ph, pw)) return -1;
    const int B = pt * ph * pw;
    for (int t = 0; t < T; ++t)
        for (int h = 0; h < H; ++h)
            for (int w = 0; w < W; ++w) {
                const int64_t n = ((int64_t)t * H + h) * W + w;
                int64_t i; int l;
                vo_token_to_slot(&g, t, h, w, &i, &l);
                memcpy((char*)y + n * d * elem_size,
                       (const char*)y_tiled + (i * B + l) * d * elem_size, (size_t)(d * elem_size));
            }
    return 0;
}

/*
 * Stage 2a -- TripPool (Eq. 4; Alg. 2 "Triplet Statistics Extraction"): for every tile and
 * channel, Avg, Max and Min over the tile's real tokens, concatenated as
 * z[i] = [avg(0..d-1) | max(0..d-1) | min(0..d-1)].
 * fp32 arithmetic with a fixed order: tokens are visited in ascending slot order
 * (lt, lh, lw raster), the sum starts at +0 and is a chain of fp32 additions, and
 * avg = sum * (1.0f / (float)count).
 * x [N][d] fp32 token order;  z [N_T][3d].
 */
int vo_trippool(const float* x, int d, int T, int H, int W, int pt, int ph, int pw, float* z) {
    vo_geom g;
    if (vo_make_geom(&g, T, H, W, pt, ph, pw)) return -1;
#pragma omp parallel for collapse(3) schedule(static)
    for (int tt = 0; tt < g.nt; ++tt)
        for (int th = 0; th < g.nh; ++th)
            for (int tw = 0; tw < g.nw; ++tw) {
                const int64_t i = ((int64_t)tt * g.nh + th) * g.nw + tw;
                float* zi = z + i * 3 * d;
                for (int c = 0; c < d; ++c) {
                    float sum = 0.0f, mx = -INFINITY, mn = INFINITY;
                    int cnt = 0;
                    for (int lt = 0; lt < pt; ++lt)
                        for (int lh = 0; lh < ph; ++lh)
                            for (int lw = 0; lw < pw; ++lw) {
                                const int t = tt * pt + lt, h = th * ph + lh, w = tw * pw + lw;
                                if (t >= T || h >= H || w >= W) continue;
                                const float v = x[(((int64_t)t * H + h) * W + w) * d + c];
                                sum = sum + v;
                                mx = v > mx ? v : mx;
                                mn = v < mn ? v : mn;
                                cnt += 1;
                            }
                    const float inv = 1.0f / (float)cnt;
                    zi[c] = sum * inv;
                    zi[d + c] = mx;
                    zi[2 * d + c] = mn;
                }
            }
    return 0;
}

/*
 * Stage 2b -- head-specific projection phi (Eq. 5; Alg. 2 "Projection"): a perceptron
 * in_dim -> hidden -> out_dim with bias on both layers and ReLU (relu != 0) or identity
 * between them; hidden == 0 means a single affine layer y = b1 + z*W1 with W1 [in][out].
 * Each output is one fmaf chain over ascending input index, started from the bias.
 * z [n][in_dim];  w1 [in_dim][hidden or out_dim];  w2 [hidden][out_dim];  y [n][out_dim].
 */
int vo_mlp(const float* z, int64_t n, int in_dim, int hidden, int out_dim, int relu,
           const float* w1, const float* b1, const float* w2, const float* b2, float* y) {
    if (hidden == 0) {
        for (int64_t r = 0; r < n; ++r)
            for (int o = 0; o < out_dim; ++o) {
                float acc = b1[o];
                for (int i = 0; i < in_dim; ++i) acc = fmaf(z[r * in_dim + i], w1[(int64_t)i * out_dim + o], acc);
                y[r * out_dim + o] = acc;
            }
        return 0;
    }
    int fail = 0;
#pragma omp parallel
    {
        float* hid = (float*)malloc(sizeof(float) * (size_t)hidden);
        if (!hid) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(static)
        for (int64_t r = 0; r < n; ++r) {
            if (!hid) continue;
            for (int j = 0; j < hidden; ++j) {
                float acc = b1[j];
                for (int i = 0; i < in_dim; ++i) acc = fmaf(z[r * in_dim + i], w1[(int64_t)i * hidden + j], acc);
                hid[j] = (relu && !(acc > 0.0f)) ? 0.0f : acc;
            }
            for (int o = 0; o < out_dim; ++o) {
                float acc = b2[o];
                for (int j = 0; j < hidden; ++j) acc = fmaf(hid[j], w2[(int64_t)j * out_dim + o], acc);
                y[r * out_dim + o] = acc;
            }
        }
        free(hid);
    }
    return fail ? -1 : 0;
}

/*
 * Stage 2c -- predicted tile score (Eq. 5): S[i][j] = (qh_i . kh_j) * scale with
 * scale = 1/sqrt(d').  One fmaf chain over ascending latent index from +0, then one
 * multiply.  qh [nq][dp], kh [nk][dp], s [nq][nk].
 */
int vo_score(const float* qh, const float* kh, int64_t nq, int64_t nk, int dp, float scale, float* s) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nq; ++i)
        for (int64_t j = 0; j < nk; ++j) {
            float acc = 0.0f;
            for (int c = 0; c < dp; ++c) acc = fmaf(qh[i * dp + c], kh[j * dp + c], acc);
            s[i * nk + j] = acc * scale;
        }
    return 0;
}

/*
 * Stage 3 -- per-query-tile top-k (Sec. 3.1: exactly k ones per mask row; Sec. 4.1: keep
 * the k highest-scoring key tiles).  Equal scores are ordered by lower tile index.  NaN
 * counts as -inf and -0 as +0.  idx [rows][k] lists the kept key tiles in ascending index;
 * mask [rows][cols] (optional) is the same set as 0/1 bytes.
 */
typedef struct { float s; int32_t j; } vo_pair;

static int vo_pair_cmp(const void* a, const void* b) {
    const vo_pair* x = (const vo_pair*)a;
    const vo_pair* y = (const vo_pair*)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->j > y->j) - (x->j < y->j);
}

static int vo_int_cmp(const void* a, const void* b) {
    const int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
    return (x > y) - (x < y);
}

int vo_select(const float* s, int64_t rows, int64_t cols, int k, int32_t* idx, uint8_t* mask) {
    if (k < 1 || k > cols) return -1;
    int fail = 0;
#pragma omp parallel
    {
        vo_pair* p = (vo_pair*)malloc(sizeof(vo_pair) * (size_t)cols);
        if (!p) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(static)
        for (int64_t r = 0; r < rows; ++r) {
            if (!p) continue;
            for (int64_t j = 0; j < cols; ++j) {
                float v = s[r * cols + j];
                v = (v != v) ? -INFINITY : v + 0.0f;
                p[j].s = v;
                p[j].j = (int32_t)j;
            }
            qsort(p, (size_t)cols, sizeof(vo_pair), vo_pair_cmp);
            for (int t = 0; t < k; ++t) idx[r * k + t] = p[t].j;
            qsort(idx + r * k, (size_t)k, sizeof(int32_t), vo_int_cmp);
            if (mask) {
                memset(mask + r * cols, 0, (size_t)cols);
                for (int t = 0; t < k; ++t) mask[r * cols + idx[r * k + t]] = 1;
            }
        }
        free(p);
    }
    return fail ? -2 : 0;
}

/*
 * Stage 4 -- attention under an explicit token mask (Sec. 3.1: A = Softmax(QK^T/sqrt(d) + M),
 * M in {0, -inf}; Eq. 2 is the same thing written with concatenated kept tiles).
 * For query token u in query tile i the additive mask is M[u][v] = 0 when tile(v) is in
 * sel[i][0..ksel), else -inf.  Only real tokens exist here, so padding never appears.
 * Everything is double precision.
 *   q,k,v   [N][d] fp32 token order (already rounded to the storage type under test)
 *   sel     [N_T][ksel] kept key tiles of each query tile
 *   queries [nq] token indices to evaluate
 *   out     [nq][d]   O[u] = sum_v A[u][v] V[v]
 *   lse     [nq]      log sum_v exp(logit)            (optional)
 *   wsum    [nq]      sum_v A[u][v] after normalising (optional; row-stochasticity)
 */
int vo_masked_attention(const float* q, const float* k, const float* v, int d,
                        int T, int H, int W, int pt, int ph, int pw,
                        const int32_t* sel, int ksel, double scale,
                        const int64_t* queries, int64_t nq,
                        double* out, double* lse, double* wsum) {
    vo_geom g;
    if (vo_make_geom(&g, T, H, W, pt, ph, pw)) return -1;
    const int64_t N = (int64_t)T * H * W;
    const int64_t n_tiles = (int64_t)g.nt * g.nh * g.nw;
    int32_t* tile_of = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
    if (!tile_of) return -2;
    vo_token_tile_map(T, H, W, pt, ph, pw, tile_of);
    int fail = 0;
#pragma omp parallel
    {
        double* M = (double*)malloc(sizeof(double) * (size_t)N);      /* additive mask row */
        double* a = (double*)malloc(sizeof(double) * (size_t)N);      /* logits, then weights */
        uint8_t* kept = (uint8_t*)malloc((size_t)n_tiles);
        if (!M || !a || !kept) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(dynamic, 8)
        for (int64_t r = 0; r < nq; ++r) {
            if (!M || !a || !kept) continue;
            const int64_t u = queries[r];
            const int32_t i = tile_of[u];
            memset(kept, 0, (size_t)n_tiles);
            for (int t = 0; t < ksel; ++t) kept[sel[(int64_t)i * ksel + t]] = 1;
            for (int64_t n = 0; n < N; ++n) M[n] = kept[tile_of[n]] ? 0.0 : -INFINITY;
            double mx = -INFINITY;
            for (int64_t n = 0; n < N; ++n) {
                if (M[n] != 0.0) { a[n] = -INFINITY; continue; }   /* finite + (-inf) = -inf */
                double dot = 0.0;
                for (int c = 0; c < d; ++c) dot += (double)q[u * d + c] * (double)k[n * d + c];
                a[n] = dot * scale + M[n];
                if (a[n] > mx) mx = a[n];
            }
            double denom = 0.0;
            for (int64_t n = 0; n < N; ++n) {
                a[n] = (a[n] == -INFINITY) ? 0.0 : exp(a[n] - mx);
                denom += a[n];
            }
            double* o = out + r * d;
            for (int c = 0; c < d; ++c) o[c] = 0.0;
            double ws = 0.0;
            for (int64_t n = 0; n < N; ++n) {
                if (a[n] == 0.0) continue;
                const double wgt = a[n] / denom;
                ws += wgt;
                for (int c = 0; c < d; ++c) o[c] += wgt * (double)v[n * d + c];
            }
            if (lse) lse[r] = mx + log(denom);
            if (wsum) wsum[r] = ws;
        }
        free(M); free(a); free(kept);
    }
    free(tile_of);
    return fail ? -3 : 0;
}

/* Dense attention, Eq. 1: A = Softmax(QK^T/sqrt(d)), O = AV, for the listed query tokens. */
int vo_dense_attention(const float* q, const float* k, const float* v, int d, int64_t N,
                       double scale, const int64_t* queries, int64_t nq, double* out) {
    int fail = 0;
#pragma omp parallel
    {
        double* a = (double*)malloc(sizeof(double) * (size_t)N);
        if (!a) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(dynamic, 8)
        for (int64_t r = 0; r < nq; ++r) {
            if (!a) continue;
            const int64_t u = queries[r];
            double mx = -INFINITY;
            for (int64_t n = 0; n < N; ++n) {
                double dot = 0.0;
                for (int c = 0; c < d; ++c) dot += (double)q[u * d + c] * (double)k[n * d + c];
                a[n] = dot * scale;
                if (a[n] > mx) mx = a[n];
            }
            double denom = 0.0;
            for (int64_t n = 0; n < N; ++n) { a[n] = exp(a[n] - mx); denom += a[n]; }
            double* o = out + r * d;
            for (int c = 0; c < d; ++c) o[c] = 0.0;
            for (int64_t n = 0; n < N; ++n) {
                const double wgt = a[n] / denom;
                for (int c = 0; c < d; ++c) o[c] += wgt * (double)v[n * d + c];
            }
        }
        free(a);
    }
    return fail ? -3 : 0;
}

/* Target tile scores of full attention (Sec. 4.1 "Target: Full-Attention Score Construction"):
 * A* = Softmax(Q K^T * scale) over all N tokens of the head, then max-pooling over each
 * (query tile, key tile) region:  S_tgt[i][j] = max over tokens u of tile i, v of tile j of
 * A*[u][v].  Padded slots hold no token and take no part.  The listed query tiles only
 * (Sec. 4.3 "partial query processing": rows of other tiles are left untouched); n_qt < 0
 * means all tiles.  heat is [N_T][N_T] row-major, double. */
int vo_tile_heatmap(const float* q, const float* k, int d, int T, int H, int W, int pt, int ph, int pw,
                    double scale, const int32_t* query_tiles, int64_t n_qt, double* heat) {
    vo_geom g;
    if (vo_make_geom(&g, T, H, W, pt, ph, pw)) return -1;
    const int64_t N = (int64_t)T * H * W;
    const int64_t NT = (int64_t)g.nt * g.nh * g.nw;
    int32_t* tile_of = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
    uint8_t* want = (uint8_t*)malloc((size_t)NT);
    if (!tile_of || !want) { free(tile_of); free(want); return -3; }
    vo_token_tile_map(T, H, W, pt, ph, pw, tile_of);
    memset(want, n_qt < 0 ? 1 : 0, (size_t)NT);
    for (int64_t r = 0; r < n_qt; ++r) {
        if (query_tiles[r] < 0 || query_tiles[r] >= NT) { free(tile_of); free(want); return -2; }
        want[query_tiles[r]] = 1;
    }
    for (int64_t i = 0; i < NT; ++i)
        if (want[i]) for (int64_t j = 0; j < NT; ++j) heat[i * NT + j] = 0.0;
    int fail = 0;
    /* one query tile per iteration: its rows of heat are written by one thread only */
#pragma omp parallel
    {
        double* a = (double*)malloc(sizeof(double) * (size_t)N);
        if (!a) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int64_t i = 0; i < NT; ++i) {
            if (!a || !want[i]) continue;
            for (int64_t u = 0; u < N; ++u) {
                if (tile_of[u] != i) continue;
                double mx = -INFINITY;
                for (int64_t n = 0; n < N; ++n) {
                    double dot = 0.0;
                    for (int c = 0; c < d; ++c) dot += (double)q[u * d + c] * (double)k[n * d + c];
                    a[n] = dot * scale;
                    if (a[n] > mx) mx = a[n];
                }
                double denom = 0.0;
                for (int64_t n = 0; n < N; ++n) { a[n] = exp(a[n] - mx); denom += a[n]; }
                for (int64_t n = 0; n < N; ++n) {
                    const double p = a[n] / denom;
                    double* cell = heat + i * NT + tile_of[n];
                    if (p > *cell) *cell = p;
                }
            }
        }
        free(a);
    }
    free(tile_of);
    free(want);
    return fail ? -3 : 0;
}

/* Tile recall (Sec. 3.2 "Metric: tile recall w.r.t. full attention"):
 * Recall@k = 1/rows * sum_i |S_sp_i  intersect  S_fu_i| / k, both selections given as
 * [rows][k] lists of distinct key tiles in any order. */
int vo_recall(const int32_t* sel_sp, const int32_t* sel_fu, int64_t rows, int k, double* recall) {
    if (rows <= 0 || k <= 0) return -1;
    double acc = 0.0;
    for (int64_t i = 0; i < rows; ++i) {
        int common = 0;
        for (int a = 0; a < k; ++a)
            for (int b = 0; b < k; ++b)
                if (sel_sp[i * k + a] == sel_fu[i * k + b]) { ++common; break; }
        acc += (double)common / (double)k;
    }
    *recall = acc / (double)rows;
    return 0;
}

/* Weight-free scorer from the sufficient-statistics argument (App. A.3, "Reconstructing
 * Attention via Sufficient Statistics": S ~ mean product + lambda * dispersion product, with
 * the dispersion bounded from the extrema, Delta = sqrt((M - mu)(mu - m))).  The appendix
 * states it for the elements of one vector; here it is read per channel over a tile's tokens,
 * on the TripPool descriptor z = [avg | max | min] of stage 2a:
 *     S[i][j] = sum_c mu_q[i][c] mu_k[j][c] + lambda * sum_c Delta_q[i][c] Delta_k[j][c].
 * This function forms the 2d-long latent  y = [ mu | sqrt(lambda) * Delta ]  whose plain dot
 * product (vo_score with scale 1) is that score.  fp32, fixed order:
 *     Delta = sqrtf(max(0, (M - mu) * (mu - m))),  y[d + c] = root_lambda * Delta,
 * root_lambda = sqrtf(lambda) rounded once by the caller.  z [n][3d], y [n][2d]. */
int vo_closed_form_latent(const float* z, int64_t n, int d, float root_lambda, float* y) {
    for (int64_t i = 0; i < n; ++i)
        for (int c = 0; c < d; ++c) {
            const float mu = z[i * 3 * d + c], mx = z[i * 3 * d + d + c], mn = z[i * 3 * d + 2 * d + c];
            const float up = mx - mu, dn = mu - mn;
            float p = up * dn;
            p = p > 0.0f ? p : 0.0f;
            y[i * 2 * d + c] = mu;
            y[i * 2 * d + d + c] = root_lambda * sqrtf(p);
        }
    return 0;
}
