// Stages 2 + 3 without the score matrix (Eq. 5 scores; Sec. 3.1 / Alg. 2 per-row top-k; the
// Conclusion names tighter fusion of mask preparation as the next step for the kernels).
//
// The N_T x N_T scores of a head are formed block by block exactly as score.hip forms them (one
// fmaf chain per score over ascending latent coordinate from +0, then one multiply by scale),
// but instead of being written out each score is compared with a pivot of its row, and only the
// few that pass leave the compute unit, as (score, column) candidates in column order.  The exact
// top-k of a row is then the exact top-k of its candidates:
//   1. fused_pivot_kernel: per row, the scores of 256 evenly spread columns; the pivot is their
//      m-th largest (m per head from the host, a few standard deviations above 256*k/n).
//   2. fused_candidates_kernel: a workgroup owns 64 rows and one of kFSeg column segments, which
//      it walks 128 columns at a time; the 16 lanes that share a row count their passing scores
//      with one ballot per column group, so the candidates of a row and segment land in ascending
//      column order without atomics.
//   3. fused_finish_kernel: one wavefront per row runs the bitwise search and the tie rule on the
//      candidates of its segments taken in order.  A row with fewer than k candidates, or more
//      than a segment's share of the 1024 slots in one segment, raises its flag.
//   4. Flagged rows only: their score rows are formed into a scratch matrix by the stage-2 kernel
//      and searched in full by the stage-3 search.  The result is the exact top-k either way.
// Heads with short rows or large keep budgets (where stage 3 would not sample either) and
// latents longer than 64 coordinates take the two-stage route through the scratch matrix.
#include <atomic>
#include <type_traits>

#include "score_common.h"
#include "select_common.h"

namespace veda {

constexpr int kFR = kLatentRows;      // rows of one entry of the plan's row-block table
constexpr int kFC = 128;              // columns per step
constexpr int kFMaxDp = 64;           // latent coordinates of the rows held in LDS
constexpr int kFQPitch = kFMaxDp + 4; // floats; 16-byte aligned rows, 4 consecutive rows in 4 bank groups
constexpr int kFStage = 32;           // column coordinates staged per step
constexpr int kFKPitch = kFStage + 4;
// Measured on 24 heads of ~3700 tiles: 64 rows x 2 segments 1.66 ms for the whole call, 64 x 1 1.76,
// 64 x 4 2.04 (segments overflow their share of the slots), 128 rows x 2 2.47 (too few workgroups).
constexpr int kFSeg = 2;                      // column segments, one workgroup each
constexpr int kFSegCap = kCandCap / kFSeg;    // candidate slots of a row in one segment
constexpr int kFRA = 4;                       // rows per thread of the candidates kernel: 16*kFRA rows per workgroup

// Latent rows r0 .. r0+16*RA-1 of one head into qs ([16*RA][kFQPitch]); rows past the head are zero.
template <int RA>
__device__ __forceinline__ void load_rows(float* qs, const float* __restrict__ qbase, int r0, int nT, int dp) {
    const int c4n = dp / 4;
    for (int t = threadIdx.x; t < 16 * RA * c4n; t += 256) {
        const int r = t / c4n, c4 = (t % c4n) * 4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (r0 + r < nT) v = *reinterpret_cast<const float4*>(qbase + (int64_t)(r0 + r) * dp + c4);
        *reinterpret_cast<float4*>(qs + r * kFQPitch + c4) = v;
    }
}

// acc[a][e] = q_row(ti + 16a) . k_col(col_of(tj + 16e)): a (16*RA) x 128 block of raw dot products,
// each one fmaf chain over ascending coordinate from +0 (the order score.hip and the oracle use).
// col_of(r) gives the key tile staged as column r of the block, or -1 for none (zeros).
template <int RA, typename ColOf>
__device__ __forceinline__ void score_block(float (&acc)[RA][8], const float* qs, float* ks,
                                            const float* __restrict__ kbase, int dp, ColOf col_of) {
    const int ti = threadIdx.x / 16, tj = threadIdx.x % 16;
#pragma unroll
    for (int a = 0; a < RA; ++a)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[a][e] = 0.0f;
    for (int c0 = 0; c0 < dp; c0 += kFStage) {
        const int cn = dp - c0 < kFStage ? dp - c0 : kFStage;   // multiple of 4
        __syncthreads();
        for (int t = threadIdx.x; t < kFC * (kFStage / 4); t += 256) {
            const int r = t / (kFStage / 4), c4 = (t % (kFStage / 4)) * 4;
            const int col = col_of(r);
            float4 kv = make_float4(0.f, 0.f, 0.f, 0.f);
            if (c4 < cn && col >= 0) kv = *reinterpret_cast<const float4*>(kbase + (int64_t)col * dp + c0 + c4);
            *reinterpret_cast<float4*>(ks + r * kFKPitch + c4) = kv;
        }
        __syncthreads();
        for (int c = 0; c < cn; c += 4) {
            float4 kb[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) kb[e] = *reinterpret_cast<const float4*>(ks + (tj + 16 * e) * kFKPitch + c);
#pragma unroll
            for (int a = 0; a < RA; ++a) {
                const float4 qa = *reinterpret_cast<const float4*>(qs + (ti + 16 * a) * kFQPitch + c0 + c);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    float v = acc[a][e];
                    v = __builtin_fmaf(qa.x, kb[e].x, v);
                    v = __builtin_fmaf(qa.y, kb[e].y, v);
                    v = __builtin_fmaf(qa.z, kb[e].z, v);
                    v = __builtin_fmaf(qa.w, kb[e].w, v);
                    acc[a][e] = v;
                }
            }
        }
    }
}

// Step 1: pivot[row] = the m-th largest of the row's scores at columns (s*n)/256, s = 0..255.
__global__ __launch_bounds__(256) void fused_pivot_kernel(const HeadGeom* __restrict__ heads,
                                                          const int32_t* __restrict__ row_blk,
                                                          const float* __restrict__ yq, const float* __restrict__ yk,
                                                          int dp, float scale, int64_t total_tiles, SampleArgs sample,
                                                          float* __restrict__ pivot, int32_t* __restrict__ group_flags,
                                                          float* __restrict__ samples) {
    // The 64 x 256 sample scores go through global scratch (they stay in L2) rather than LDS: with
    // only the operand stages in LDS four workgroups fit on a compute unit instead of two.
    __shared__ __align__(16) float qs[kFR * kFQPitch];
    __shared__ __align__(16) float ks[kFC * kFKPitch];
    const int32_t code = row_blk[blockIdx.x];
    const int head = code >> 24, r0 = (code & 0xffffff) * kFR;
    const HeadGeom hg = heads[head];
    const int nT = hg.n_tiles;
    const int64_t row_base = (int64_t)blockIdx.y * total_tiles + hg.tile_off;
    const float* qbase = yq + row_base * dp;
    const float* kbase = yk + row_base * dp;
    // this call's "some row of these 128 asked for its full score row" marks start cleared
    if (threadIdx.x < 2) group_flags[(row_base + r0 + 63 * threadIdx.x) >> 7] = 0;
    load_rows<4>(qs, qbase, r0, nT, dp);
    float acc[2][4][8];
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
        score_block<4>(acc[sb], qs, ks, kbase, dp,
                       [&](int r) { return (int)(((int64_t)(sb * kFC + r) * nT) / kSample); });
    const int ti = threadIdx.x / 16, tj = threadIdx.x % 16;
    float* smp = samples + (row_base + r0) * kSample;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        if (r0 + ti + 16 * a >= nT) continue;   // rows past the head belong to another workgroup
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
            for (int e = 0; e < 8; ++e) smp[(ti + 16 * a) * kSample + sb * kFC + tj + 16 * e] = acc[sb][a][e] * scale;
    }
    __syncthreads();   // orders the stores before the loads below (same workgroup)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = sample.m[head];
    for (int rr = 0; rr < kFR / 4; ++rr) {
        const int r = wave * (kFR / 4) + rr;
        if (r0 + r >= nT) break;
        uint32_t sk[kSample / 64];
#pragma unroll
        for (int e = 0; e < kSample / 64; ++e) sk[e] = score_key(smp[r * kSample + e * 64 + lane]);
        // Any pivot with at least k scores above it serves: the search stops after the top 20 key
        // bits, which leaves the pivot at or just below the sample's m-th largest value.
        uint32_t pk = 0;
        for (int bit = 31; bit >= 12; --bit) {
            const uint32_t cand = pk | (1u << bit);
            int cnt = 0;
#pragma unroll
            for (int e = 0; e < kSample / 64; ++e) cnt += __popcll(__ballot(sk[e] >= cand));
            if (cnt >= m) pk = cand;
        }
        if (lane == 0) pivot[row_base + r0 + r] = __uint_as_float((pk & 0x80000000u) ? (pk ^ 0x80000000u) : ~pk);
    }
}

// Step 2: (score, column) of every score >= its row's pivot.  Segment g of a row owns slots
// g*kFSegCap .. of the row's kCandCap, filled in ascending column order; cand_cnt[row*kFSeg + g]
// counts all passing scores of the segment, stored or not.
__global__ __launch_bounds__(256) void fused_candidates_kernel(const HeadGeom* __restrict__ heads,
                                                               const int32_t* __restrict__ row_blk,
                                                               const float* __restrict__ yq,
                                                               const float* __restrict__ yk, int dp, float scale,
                                                               int64_t total_tiles, const float* __restrict__ pivot,
                                                               uint2* __restrict__ cand,
                                                               int32_t* __restrict__ cand_cnt) {
    constexpr int RA = kFRA;
    __shared__ __align__(16) float qs[16 * RA * kFQPitch];
    __shared__ __align__(16) float ks[kFC * kFKPitch];
    const int32_t code = row_blk[blockIdx.x];
    static_assert(16 * RA == kFR, "one workgroup per entry of the row-block table");
    const int head = code >> 24, r0 = (code & 0xffffff) * kFR;
    const HeadGeom hg = heads[head];
    const int nT = hg.n_tiles;
    const int seg = blockIdx.y % kFSeg;
    const int64_t row_base = (int64_t)(blockIdx.y / kFSeg) * total_tiles + hg.tile_off;
    const int n_blk = (nT + kFC - 1) / kFC;
    const int c_begin = (seg * n_blk / kFSeg) * kFC, c_end = ((seg + 1) * n_blk / kFSeg) * kFC;
    const float* qbase = yq + row_base * dp;
    const float* kbase = yk + row_base * dp;
    load_rows<RA>(qs, qbase, r0, nT, dp);
    const int ti = threadIdx.x / 16, tj = threadIdx.x % 16;
    const int shift = 16 * ((threadIdx.x & 63) / 16);   // this lane's 16-lane group inside a ballot
    const uint32_t below = (1u << tj) - 1u;
    float pv[RA];
    int base[RA];
    bool real[RA];
#pragma unroll
    for (int a = 0; a < RA; ++a) {
        const int r = r0 + ti + 16 * a;
        real[a] = r < nT;
        // rows past the head: their latents are zero, so are their scores, and +inf passes none of
        // them; a NaN pivot passes nothing either
        pv[a] = real[a] ? pivot[row_base + r] : INFINITY;
        base[a] = 0;
    }
    // The workgroup's rows own one contiguous piece of the candidate array: a uniform base and a
    // 32-bit offset per store.
    char* wg_out = reinterpret_cast<char*>(cand + (row_base + r0) * kCandCap);
    uint32_t row_off[RA];
#pragma unroll
    for (int a = 0; a < RA; ++a) row_off[a] = (uint32_t)(((ti + 16 * a) * kCandCap + seg * kFSegCap) * sizeof(uint2));
    // pass: the score is a candidate; kept in ascending column order by one ballot per column group
    auto compact = [&](float (&acc)[RA][8], int c0, auto full) {
#pragma unroll
        for (int a = 0; a < RA; ++a) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float s = acc[a][e] * scale;
                const int col = c0 + tj + 16 * e;
                const bool pass = decltype(full)::value ? s >= pv[a] : (s >= pv[a]) & (col < nT);
                const uint32_t mine = (uint32_t)(__ballot(pass) >> shift) & 0xffffu;
                const int pos = base[a] + __popc(mine & below);
                if (pass && pos < kFSegCap)   // the score's bits; the search turns them into a key
                    *reinterpret_cast<uint2*>(wg_out + row_off[a] + (uint32_t)pos * sizeof(uint2)) =
                        make_uint2(__float_as_uint(s), (uint32_t)col);
                base[a] += __popc(mine);
            }
        }
    };
    for (int c0 = c_begin; c0 < c_end; c0 += kFC) {
        float acc[RA][8];
        score_block<RA>(acc, qs, ks, kbase, dp, [&](int r) { return c0 + r < nT ? c0 + r : -1; });
        if (c0 + kFC <= nT) compact(acc, c0, std::true_type{});
        else compact(acc, c0, std::false_type{});
    }
    if (tj == 0) {
#pragma unroll
        for (int a = 0; a < RA; ++a)
            if (real[a]) cand_cnt[(row_base + r0 + ti + 16 * a) * kFSeg + seg] = base[a];
    }
}

// Step 3: the exact top-k of a row from its candidates, or its flag if they do not hold it.
__global__ __launch_bounds__(256) void fused_finish_kernel(const HeadGeom* __restrict__ heads,
                                                           const uint8_t* __restrict__ tile_head,
                                                           const float* __restrict__ scratch, SelectArgs args,
                                                           const uint2* __restrict__ cand,
                                                           const int32_t* __restrict__ cand_cnt,
                                                           int32_t* __restrict__ row_ptr, int32_t* __restrict__ col_idx,
                                                           int32_t* __restrict__ flags,
                                                           int32_t* __restrict__ group_flags, int64_t total_tiles,
                                                           int64_t score_elems, int64_t rows) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const RowInfo ri = locate_row(heads, tile_head, scratch, args, row_ptr, col_idx, total_tiles, score_elems, rows,
                                  row, lane);
    int seg_end[kFSeg];   // candidates up to and including segment g
    int m_cand = 0;
    bool ok = true;
#pragma unroll
    for (int g = 0; g < kFSeg; ++g) {
        const int c = cand_cnt[row * kFSeg + g];
        ok = ok && c <= kFSegCap;
        m_cand += c;
        seg_end[g] = m_cand;
    }
    ok = ok && m_cand >= ri.k;
    if (lane == 0) {
        flags[row] = ok ? 0 : 1;
        if (!ok) group_flags[row >> 7] = 1;
    }
    if (!ok) return;
    // (score bits, column) pairs: scores at even words, columns at odd words of the row's slots
    const uint32_t* ckey = reinterpret_cast<const uint32_t*>(cand + row * kCandCap);
    const int32_t* ccol = reinterpret_cast<const int32_t*>(cand + row * kCandCap) + 1;
    auto at = [&](int c) {   // word offset of the c-th candidate of the row
        int slot = c;
#pragma unroll
        for (int g = 1; g < kFSeg; ++g)
            if (c >= seg_end[g - 1]) slot = g * kFSegCap + (c - seg_end[g - 1]);
        return 2 * slot;
    };
    if (m_cand <= 256) select_candidates<4, true>(ckey, ccol, m_cand, ri.k, ri.dst, lane, at);
    else if (m_cand <= 512) select_candidates<8, true>(ckey, ccol, m_cand, ri.k, ri.dst, lane, at);
    else select_candidates<16, true>(ckey, ccol, m_cand, ri.k, ri.dst, lane, at);
}

constexpr int kFallbackRows = 16;

// Step 4b: flagged rows, searched in full on the score rows step 4a wrote to the scratch matrix.
__global__ __launch_bounds__(256) void fused_fallback_kernel(const HeadGeom* __restrict__ heads,
                                                             const uint8_t* __restrict__ tile_head,
                                                             const float* __restrict__ scratch, SelectArgs args,
                                                             int32_t* __restrict__ row_ptr,
                                                             int32_t* __restrict__ col_idx,
                                                             const int32_t* __restrict__ flags, int64_t total_tiles,
                                                             int64_t score_elems, int64_t rows) {
    // one wavefront looks after kFallbackRows rows: a launch of a few workgroups that costs next to
    // nothing when no flag is up, which is the usual case
    const int lane = threadIdx.x & 63;
    const int64_t first = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * kFallbackRows;
    for (int64_t row = first; row < first + kFallbackRows && row < rows; ++row) {
        if (!flags[row]) continue;
        const RowInfo ri = locate_row(heads, tile_head, scratch, args, row_ptr, col_idx, total_tiles, score_elems,
                                      rows, row, lane);
        // keep the row in registers when it fits, instead of re-reading it on every pass
        if (ri.n <= 64 * 64) select_row<64>(ri.srow, ri.n, ri.k, ri.dst, lane);
        else select_row<0>(ri.srow, ri.n, ri.k, ri.dst, lane);
    }
}

struct FusedSpace {
    float *zq, *zk, *yq, *yk, *hq, *hk, *pivot, *samples, *scratch;
    int32_t *cnt, *flags, *group_flags;
    uint2* cand;
    size_t bytes;
};

// Carves the workspace; with_stats also reserves the two descriptor arrays.
static FusedSpace carve(const veda_plan* pl, int dp, int hidden_q, int hidden_k, bool with_stats, void* workspace) {
    const size_t rows = (size_t)pl->prob.batch * (size_t)pl->total_tiles;
    char* p = (char*)workspace;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char* q = p ? p + off : nullptr;
        off += (bytes + 255) / 256 * 256;
        return q;
    };
    FusedSpace f;
    const size_t zbytes = with_stats ? rows * 3 * (size_t)pl->prob.head_dim * sizeof(float) : 0;
    f.zq = (float*)take(zbytes);
    f.zk = (float*)take(zbytes);
    f.yq = (float*)take(rows * dp * sizeof(float));
    f.yk = (float*)take(rows * dp * sizeof(float));
    f.hq = (float*)take(rows * (size_t)hidden_q * sizeof(float));
    f.hk = (float*)take(rows * (size_t)hidden_k * sizeof(float));
    f.pivot = (float*)take(rows * sizeof(float));
    f.samples = (float*)take(rows * kSample * sizeof(float));
    f.cnt = (int32_t*)take(rows * kFSeg * sizeof(int32_t));
    f.flags = (int32_t*)take(rows * sizeof(int32_t));
    f.group_flags = (int32_t*)take((rows / 128 + 2) * sizeof(int32_t));
    f.cand = (uint2*)take(rows * kCandCap * sizeof(uint2));
    f.scratch = (float*)take((size_t)pl->score_elems * (size_t)pl->prob.batch * sizeof(float));
    f.bytes = off;
    return f;
}

// From descriptors zq, zk to the kept lists.
static veda_status score_select(const veda_plan* pl, const veda_mlp* phi_q, const veda_mlp* phi_k, float scale,
                                const float* zq, const float* zk, const int32_t* k_per_head, int32_t* row_ptr,
                                int32_t* col_idx, const FusedSpace& f, hipStream_t s) {
    const int dp = phi_q->out_dim;
    SelectArgs args;
    SampleArgs sample;
    bool sampled;
    int max_tiles;
    if (!select_setup(pl, k_per_head, args, sample, sampled, max_tiles)) return VEDA_ERR_INVALID_ARG;
    if (args.nnz_per_batch * pl->prob.batch >= ((int64_t)1 << 31)) return VEDA_ERR_UNSUPPORTED;  // row_ptr is int32
    veda_status st = launch_projections(pl, phi_q, phi_k, zq, zk, f.yq, f.yk, phi_q->hidden ? f.hq : nullptr,
                                        phi_k->hidden ? f.hk : nullptr, s);
    if (st != VEDA_OK) return st;
    if (!sampled || dp > kFMaxDp) {   // the two-stage route, through the scratch matrix
        st = launch_score_blocks(pl, f.yq, f.yk, f.scratch, dp, scale, nullptr, s);
        if (st != VEDA_OK) return st;
        return launch_select(pl, f.scratch, k_per_head, row_ptr, col_idx, s);
    }
    const int64_t rows = pl->total_tiles * pl->prob.batch;
    dim3 bgrid((unsigned)pl->row_blocks, (unsigned)pl->prob.batch), rgrid((unsigned)((rows + 3) / 4)), block(256);
    dim3 cgrid((unsigned)pl->row_blocks, (unsigned)(pl->prob.batch * kFSeg));
    hipLaunchKernelGGL(fused_pivot_kernel, bgrid, block, 0, s, pl->d_heads, pl->d_row_blk, f.yq, f.yk, dp, scale,
                       pl->total_tiles, sample, f.pivot, f.group_flags, f.samples);
    if ((st = launch_status("fused_pivot_kernel")) != VEDA_OK) return st;
    hipLaunchKernelGGL(fused_candidates_kernel, cgrid, block, 0, s, pl->d_heads, pl->d_row_blk, f.yq, f.yk, dp, scale,
                       pl->total_tiles, f.pivot, f.cand, f.cnt);
    if ((st = launch_status("fused_candidates_kernel")) != VEDA_OK) return st;
    hipLaunchKernelGGL(fused_finish_kernel, rgrid, block, 0, s, pl->d_heads, pl->d_tile_head, f.scratch, args, f.cand,
                       f.cnt, row_ptr, col_idx, f.flags, f.group_flags, pl->total_tiles, pl->score_elems, rows);
    if ((st = launch_status("fused_finish_kernel")) != VEDA_OK) return st;
    st = launch_score_blocks(pl, f.yq, f.yk, f.scratch, dp, scale, f.group_flags, s);
    if (st != VEDA_OK) return st;
    dim3 fgrid((unsigned)((rows + 4 * kFallbackRows - 1) / (4 * kFallbackRows)));
    hipLaunchKernelGGL(fused_fallback_kernel, fgrid, block, 0, s, pl->d_heads, pl->d_tile_head, f.scratch, args,
                       row_ptr, col_idx, f.flags, pl->total_tiles, pl->score_elems, rows);
    return launch_status("fused_fallback_kernel");
}

// Scratch of the entry point that allocates nothing: a fixed array in every GPU's memory, held
// from the moment the library is loaded on that GPU until the process ends.  In host code the
// array's name is only a handle; its address on the current device comes from
// hipGetSymbolAddress, once per device (noalloc_scratch below), and only that pointer is ever
// handed to a kernel.
constexpr size_t kNoAllocBytes = VEDA_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kNoAllocBytes];
constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on GPU `device`, which must be the current device.  Resolved on
// the first call per device (veda_plan_create makes that call), cached afterwards; two threads
// racing on the first call store the same value.
veda_status noalloc_scratch(int device, void** out) {
    if (device < 0 || device >= kMaxDevices) {
        set_last_error("no-allocation scratch: device index out of range");
        return VEDA_ERR_UNSUPPORTED;
    }
    void* p = g_scratch_ptr[device].load(std::memory_order_acquire);
    if (!p) {
        int cur = -1;
        VEDA_HIP_TRY(hipGetDevice(&cur));
        if (cur != device) {
            set_last_error("no-allocation scratch: the plan's device is not the current device");
            return VEDA_ERR_INVALID_ARG;
        }
        VEDA_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) {
            set_last_error("no-allocation scratch: hipGetSymbolAddress gave no address");
            return VEDA_ERR_HIP;
        }
        g_scratch_ptr[device].store(p, std::memory_order_release);
    }
    *out = p;
    return VEDA_OK;
}

static veda_status check_pair(const veda_plan* pl, const veda_mlp* phi_q, const veda_mlp* phi_k) {
    veda_status st = check_mlp(pl, phi_q);
    if (st == VEDA_OK) st = check_mlp(pl, phi_k);
    if (st != VEDA_OK) return st;
    return phi_q->out_dim == phi_k->out_dim ? VEDA_OK : VEDA_ERR_INVALID_ARG;
}

}  // namespace veda

extern "C" size_t veda_plan_fused_workspace_bytes(const veda_plan* pl, const veda_mlp* phi_q, const veda_mlp* phi_k) {
    if (!pl || !phi_q || !phi_k || phi_q->out_dim < 1) return 0;
    return veda::carve(pl, phi_q->out_dim, phi_q->hidden, phi_k->hidden, true, nullptr).bytes;
}

extern "C" veda_status veda_tile_score_select(const veda_plan* pl, const void* q_tiled, const void* k_tiled,
                                              const uint64_t* valid_mask, const veda_mlp* phi_q,
                                              const veda_mlp* phi_k, float scale, const int32_t* k_per_head,
                                              int32_t* row_ptr, int32_t* col_idx, void* workspace,
                                              size_t workspace_bytes, void* stream) {
    using namespace veda;
    if (!pl || !q_tiled || !k_tiled || !valid_mask || !k_per_head || !row_ptr || !col_idx) return VEDA_ERR_INVALID_ARG;
    const veda_status st = check_pair(pl, phi_q, phi_k);
    if (st != VEDA_OK) return st;
    if (!aligned16(q_tiled) || !aligned16(k_tiled) || !aligned16(workspace)) return VEDA_ERR_UNSUPPORTED;
    const FusedSpace f = carve(pl, phi_q->out_dim, phi_q->hidden, phi_k->hidden, true, workspace);
    if (!workspace || workspace_bytes < f.bytes) return VEDA_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    launch_trippool(pl, q_tiled, k_tiled, valid_mask, f.zq, f.zk, s);
    const veda_status tp = launch_status("trippool_kernel");
    if (tp != VEDA_OK) return tp;
    return score_select(pl, phi_q, phi_k, scale, f.zq, f.zk, k_per_head, row_ptr, col_idx, f, s);
}

extern "C" veda_status veda_tile_score_select_stats(const veda_plan* pl, const float* stats_q, const float* stats_k,
                                                    const veda_mlp* phi_q, const veda_mlp* phi_k, float scale,
                                                    const int32_t* k_per_head, int32_t* row_ptr, int32_t* col_idx,
                                                    void* workspace, size_t workspace_bytes, void* stream) {
    using namespace veda;
    if (!pl || !stats_q || !stats_k || !k_per_head || !row_ptr || !col_idx) return VEDA_ERR_INVALID_ARG;
    const veda_status st = check_pair(pl, phi_q, phi_k);
    if (st != VEDA_OK) return st;
    if (!aligned16(stats_q) || !aligned16(stats_k) || !aligned16(workspace)) return VEDA_ERR_UNSUPPORTED;
    const FusedSpace f = carve(pl, phi_q->out_dim, phi_q->hidden, phi_k->hidden, true, workspace);
    if (!workspace || workspace_bytes < f.bytes) return VEDA_ERR_WORKSPACE;
    return score_select(pl, phi_q, phi_k, scale, stats_q, stats_k, k_per_head, row_ptr, col_idx, f, (hipStream_t)stream);
}

extern "C" veda_status veda_tile_score_select_stats_noalloc(const veda_plan* pl, const float* stats_q,
                                                            const float* stats_k, const veda_mlp* phi_q,
                                                            const veda_mlp* phi_k, float scale,
                                                            const int32_t* k_per_head, int32_t* row_ptr,
                                                            int32_t* col_idx, void* stream) {
    using namespace veda;
    if (!pl || !stats_q || !stats_k || !k_per_head || !row_ptr || !col_idx) return VEDA_ERR_INVALID_ARG;
    const veda_status st = check_pair(pl, phi_q, phi_k);
    if (st != VEDA_OK) return st;
    if (!aligned16(stats_q) || !aligned16(stats_k)) return VEDA_ERR_UNSUPPORTED;
    const size_t need = carve(pl, phi_q->out_dim, phi_q->hidden, phi_k->hidden, true, nullptr).bytes;
    if (need > kNoAllocBytes) {
        set_last_error("veda_tile_score_select_stats_noalloc: this plan needs " + std::to_string(need) +
                       " bytes of scratch, the fixed array holds " + std::to_string(kNoAllocBytes) +
                       "; use veda_tile_score_select_stats with a workspace of the caller's");
        return VEDA_ERR_WORKSPACE;
    }
    int cur = -1;
    VEDA_HIP_TRY(hipGetDevice(&cur));
    if (cur != pl->device) {
        set_last_error("veda_tile_score_select_stats_noalloc: the plan's device is not the current device");
        return VEDA_ERR_INVALID_ARG;
    }
    void* ptr = nullptr;
    const veda_status ss = noalloc_scratch(pl->device, &ptr);
    if (ss != VEDA_OK) return ss;
    // Nothing in the scratch has to start at zero: the marks of redone row groups are cleared by the
    // first kernel of the call, every counter and flag of a real row is written before it is read.
    const FusedSpace f = carve(pl, phi_q->out_dim, phi_q->hidden, phi_k->hidden, true, ptr);
    return score_select(pl, phi_q, phi_k, scale, stats_q, stats_k, k_per_head, row_ptr, col_idx, f, (hipStream_t)stream);
}
