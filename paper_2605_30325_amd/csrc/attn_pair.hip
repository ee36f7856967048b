// Stage 4, bf16, query-tile-pair kernel (Eq. 2; Sec. 4.3 tile skipping; Alg. 1 "UnTile").
//
// A compute unit can pull K/V tiles from L2 into LDS at 64 bytes per clock at most, and a kept
// tile pair needs 32 KB of them for 512 matrix-pipe cycles of work: with one query tile per
// workgroup the loads, not the matrix cores, set the pace.  Neighbouring query tiles keep
// largely the same key tiles, so here one workgroup owns TWO neighbouring query tiles (partners
// along the axis in which the head's tile shape is thinnest: pair_tiles()) and walks the union
// of their two kept lists: a key tile kept by both is loaded once and used twice.
//
// Four wavefronts: waves 0,1 hold rows 0-31 / 32-63 of query tile A, waves 2,3 those of its
// partner B.  Every wave attends to all 64 slots of a key tile, so it needs no merge with
// another wave at the end.  A wave whose query tile does not keep the current key tile skips
// the step and only meets the others at the barrier; the matrix cores it leaves idle go to the
// second workgroup resident on the compute unit.
//
// The products are formed transposed (S^T = K Q^T, O^T = V^T P^T): a lane owns one query, its
// accumulator registers run over keys, P^T in registers already is the B operand of the second
// product.  K rows are loaded permuted by rho (bits 2,3 swapped) so that the eight keys a
// lane-half owns are contiguous in the channel-major V tile.  One step of one wave:
//     S^T block 0 (8 MFMA; in their shadow the wave's share of the NEXT tiles' global->LDS loads
//                  and the fetch of the step after next)
//     S^T block 1 (8 MFMA; in their shadow the row maximum of block 0 and, speculatively, the
//                  first 8 exponentials)
//     one comparison: need the reference move, has the tile padded slots?   (rarely: the slow path)
//     4 x [ 4 MFMA of O^T += V^T P^T ; the next 8 exponentials in their shadow ]   (at raised wave priority)
// K/V tiles are double buffered (2 x 32 KB at d = 128) and filled by direct global->LDS loads
// issued one step ahead.  Which key tile comes at which step is worked out before the loop, by all
// threads together, into a table in LDS (attn_union.h): a scalar-memory round trip inside the loop
// would make every wait for an LDS operand a wait for everything.
#include "attn_step.h"
#include "attn_union.h"

namespace veda {

// After the last step: normalise, transpose through LDS and scatter the real rows of the
// workgroup's two query tiles to token order.  obuf: [2 tiles][64 rows][D] bf16, then lse_s and tok_s.
template <int D>
__device__ __forceinline__ void finish_pair(const PairState<D>& st, const AttnArgs& a, const HeadGeom& hg, char* smem,
                                            int head, int qiA, int qiB, bool hasB, int64_t b, int tid, int which,
                                            int r, int lq, int hh) {
    constexpr int kRowB = D * 2, kKChunks = kRowB / 16;
    const float l_all = st.l_run + __shfl_xor(st.l_run, 32);
    const float inv = l_all > 0.0f ? 1.0f / l_all : 0.0f;
    char* obuf = smem;
    float* lse_s = reinterpret_cast<float*>(smem + 2 * kTile * kRowB);   // [2][64]
    int* tok_s = reinterpret_cast<int*>(lse_s + 2 * kTile);              // [2][64] token of each row, -1 = padding
    __syncthreads();
    // the slot -> token map costs a handful of integer divisions: once per row, not once per chunk
    if (tid < 2 * kTile) tok_s[tid] = slot_token(hg, tid / kTile ? qiB : qiA, tid % kTile, a.T, a.H, a.W);
    {
        char* orow = obuf + (which * kTile + 32 * r + lq) * kRowB;
#pragma unroll
        for (int nb = 0; nb < D / 32; ++nb)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int d0 = 32 * nb + 8 * j + 4 * hh;
                typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
                bf16x4 pk;
#pragma unroll
                for (int t = 0; t < 4; ++t) pk[t] = (__bf16)(st.o[nb][4 * j + t] * inv);
                *reinterpret_cast<bf16x4*>(orow + d0 * 2) = pk;
            }
        if (hh == 0) lse_s[which * kTile + 32 * r + lq] = (st.ref * st.resid + __log2f(l_all)) * kLn2;
    }
    __syncthreads();
    char* ob = a.out + b * a.so_b + head * a.so_h;
    const int n_tiles = hasB ? 2 : 1;
    for (int cid = tid; cid < n_tiles * kTile * kKChunks; cid += 256) {
        const int row = cid / kKChunks, ch = cid % kKChunks;
        const int n = tok_s[row];
        if (n >= 0)
            *reinterpret_cast<uint4*>(ob + (int64_t)n * a.so_n + ch * 16) =
                *reinterpret_cast<const uint4*>(obuf + row * kRowB + ch * 16);
    }
    if (a.lse && tid < n_tiles * kTile) {
        const int n = tok_s[tid];
        if (n >= 0) a.lse[(b * a.n_heads + head) * a.tokens + n] = lse_s[tid];
    }
}

// One step of the merged walk over the kept lists of the two query tiles of a workgroup.
struct MergedStep {
    int j;         // key tile (head-local)
    int fl;        // bit 0: tile A keeps it, bit 1: tile B keeps it; 0 = past the end
    uint64_t vm;   // validity mask of key tile j
    int n0;        // K from token order: token index of its slot 0
};

// kGrouped: 128-token tiles.  The geometry in `a` is that of the 64-slot halves (tiles 2o, 2o+1
// of whole tile o): the workgroup's pair IS one whole query tile, both halves keep the same list
// (the CSR rows and entries count whole tiles), and every entry expands to its two halves.
// kTokK: K is read from token order (a.k_tok) instead of the tiled tensor: a key tile's rows
// are found at first-token + (lt*H + lh)*W + lw; the rows of padded slots are fetched from slot 0
// instead (any finite or non-finite value will do: their logits are overwritten with -inf).
// kTable: the steps come from a table in LDS built before the main loop (attn_union.h; heads of up
// to 16384 whole tiles); otherwise the lists are walked with scalar loads as the loop goes.
constexpr int kPairChunk = 128;   // step-table entries filled at a time

template <int D, bool kGrouped, bool kTokK, bool kExact, bool kTable>
__global__ __launch_bounds__(256, 2) void sparse_attn_bf16_pair_kernel(AttnArgs a) {
    constexpr int kRowB = D * 2;                 // bytes of one K row
    constexpr int kKBytes = kTile * kRowB;       // K tile
    constexpr int kVBytes = D * kTile * 2;       // V^T tile: D rows of 128 bytes
    constexpr int kSlot = kKBytes + kVBytes;     // one LDS slot: K tile then V^T tile
    constexpr int kKChunks = kRowB / 16;         // 16-byte chunks per K row
    constexpr int kLoads = kKBytes / 1024 / 4;   // direct-load instructions per wave per tile (K; same for V)
    constexpr int G = D / 16, NB = D / 32;
    extern __shared__ __align__(1024) char smem[];   // base bits 4-9 clear: see PairAddr

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int which = wave >> 1, r = wave & 1;
    const int lq = lane & 31, hh = lane >> 5;

    int head, pair;
    if (!xcd_work(a.xcd_cum, a.heads, a.n_heads, 2, head, pair)) return;
    const HeadGeom hg = a.heads[head];
    const int64_t b = blockIdx.y;
    int qiA, qiB;
    bool hasB;
    pair_tiles(hg, pair, qiA, qiB, hasB);
    const int qi = which ? qiB : qiA;
    const int64_t row0 = kGrouped ? b * (a.total_tiles / 2) + hg.tile_off / 2 : b * a.total_tiles + hg.tile_off;
    const int64_t rowA = row0 + (kGrouped ? pair : qiA), rowB = row0 + (kGrouped ? pair : qiB);
    const int begA = a.row_ptr[rowA], nA = a.row_ptr[rowA + 1] - begA;
    const int begB = a.row_ptr[rowB], nB = hasB ? a.row_ptr[rowB + 1] - begB : 0;
    // The kept lists and the validity masks are read-only for the whole launch and indexed
    // uniformly: reading them through the constant address space makes them scalar loads, so
    // no vector-memory counter waits of the compiler's own end up inside the main loop.
    typedef const __attribute__((address_space(4))) int32_t* const_i32_t;
    typedef const __attribute__((address_space(4))) uint64_t* const_u64_t;
    const const_i32_t colsA = (const_i32_t)(uintptr_t)(a.col_idx + begA);
    const const_i32_t colsB = (const_i32_t)(uintptr_t)(a.col_idx + begB);
    const const_u64_t vmask = (const_u64_t)(uintptr_t)(a.valid_mask + hg.tile_off);
    const int64_t head_tile0 = b * a.total_tiles + hg.tile_off;
    const char* kt = kTokK ? a.k_tok + b * a.sk_b + head * a.sk_h : a.k + head_tile0 * kKBytes;
    const char* vt = a.v + head_tile0 * kVBytes;
    const const_i32_t n0s = (const_i32_t)(uintptr_t)(a.tile_n0 + hg.tile_off);

    // Q operand (B matrix of S^T = K Q^T): lane holds query row 32r+lq, channels 16t+8hh..+8.
    PairState<D> st;
    {
        // from the tiled tensor, or straight from token order (a padded slot reads as zeros, which is
        // what the tiled tensor holds there)
        const char* qrow;
        bool real = true;
        if (a.q_tok) {
            const int n = slot_token(hg, qi, 32 * r + lq, a.T, a.H, a.W);
            real = n >= 0;
            qrow = a.q_tok + b * a.sq_b + head * a.sq_h + (int64_t)(real ? n : 0) * a.sq_n + 16 * hh;
        } else {
            qrow = a.q + (head_tile0 + qi) * kKBytes + (32 * r + lq) * kRowB + 16 * hh;
        }
#pragma unroll
        for (int t = 0; t < G; ++t) {
            const bf16x8 raw = *reinterpret_cast<const bf16x8*>(qrow + 32 * t);
#pragma unroll
            for (int e = 0; e < 8; ++e) st.qf[t][e] = real ? (__bf16)((float)raw[e] * (kExact ? a.scale_pow2 : a.scale_log2)) : (__bf16)0.0f;
        }
    }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int i = 0; i < 16; ++i) st.o[nb][i] = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) st.start[i] = 0.0f;
    st.ref = st.l_run = 0.0f;
    st.resid = kExact ? a.scale_resid : 1.0f;
    st.started = false;

    // global -> LDS copy plan.  One wave instruction fills 1 KB of LDS, lane i at byte 16*i, so
    // the swizzle is applied on the global side: each lane fetches the chunk that belongs at
    // its fixed LDS position.  Wave w issues instructions w*kLoads .. w*kLoads+kLoads-1 of each
    // tile, all with one LDS base: instruction j carries the immediate offset 1024*j, which the
    // hardware adds to the LDS address AND to the global address, so every per-lane global offset
    // below is stored with 1024*j taken off again (plus kBias where it could go negative, the tile's
    // base address being lowered by the same amount).
    constexpr uint32_t kBias = kTokK ? 1024u * (kLoads - 1) : 0u;
    uint32_t k_src[kLoads], v_src[kLoads];
    uint32_t k_src0[kLoads];   // kTokK: the same chunk of the tile's anchor row
    int k_row[kLoads];
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
        const int inst = wave * kLoads + j;
        const int krow = inst * (1024 / kRowB) + lane / kKChunks, kpos = lane % kKChunks;
        const uint32_t chunk = (uint32_t)((kpos ^ (rho(krow & 31) & (kKChunks - 1))) << 4);
        k_row[j] = krow;
        k_src0[j] = chunk + kBias - 1024u * j;
        if (kTokK) {   // byte offset of the row's token from the tile's anchor token (host checked: fits 32 bits)
            const int lw = krow % hg.pw, lh = (krow / hg.pw) % hg.ph, lt = krow / (hg.pw * hg.ph);
            k_src[j] = (uint32_t)((((int64_t)lt * a.H + lh) * a.W + lw) * a.sk_n) + chunk + kBias - 1024u * j;
        } else {
            k_src[j] = krow * kRowB + chunk - 1024u * j;
        }
        const int vrow = inst * 8 + (lane >> 3), vpos = lane & 7;
        v_src[j] = vrow * 128 + ((vpos ^ (((vrow >> 1) & 7) ^ ((vrow & 1) << 2))) << 4) - 1024u * j;
    }
    const uint32_t smem_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
    const uint32_t wave_lds = smem_base + (uint32_t)wave * (kLoads * 1024);
    // The K tile (which = 0) or the V^T tile (which = 1) of step e into LDS slot `sl`.
    auto load_tile = [&](const MergedStep& e, int sl, int what) __attribute__((always_inline)) {
        if (what == 0) {
            const char* src = (kTokK ? kt + (int64_t)e.n0 * a.sk_n : kt + (int64_t)e.j * kKBytes) - kBias;
            const uint32_t dst = wave_lds + (uint32_t)sl * kSlot;
            if (kTokK && e.vm != ~0ull) {   // edge tile: padded rows have no token
                uint32_t off[kLoads];
#pragma unroll
                for (int j = 0; j < kLoads; ++j) off[j] = (e.vm >> k_row[j]) & 1ull ? k_src[j] : k_src0[j];
                dma16_group_to_lds<kLoads>(dst, src, off);
            } else {
                dma16_group_to_lds<kLoads>(dst, src, k_src);
            }
        } else {
            dma16_group_to_lds<kLoads>(wave_lds + (uint32_t)sl * kSlot + kKBytes, vt + (int64_t)e.j * kVBytes, v_src);
        }
    };
    // All of this wave's LDS-bound loads have landed (vmcnt 0), then meet the other waves.
#define VEDA_LOADS_DONE_BARRIER()   \
    do {                            \
        wait_vmcnt<0>();            \
        __syncthreads();            \
    } while (0)

    PairAddr fa;
    fa.hh = hh;
    fa.k0 = smem_base + rho(lq) * kRowB + ((hh ^ (lq & (kKChunks - 1))) << 4);
    fa.v0 = smem_base + kKBytes + lq * 128 + ((hh ^ (((lq >> 1) & 7) ^ ((lq & 1) << 2))) << 4);

    // The steps: every key tile kept by at least one of the two query tiles, once; a key tile kept by
    // both is loaded once and used by both halves of the workgroup.
    // Table mode: the sequence is laid out in LDS before the loop (attn_union.h: ascending union,
    // whatever the order inside the lists) and the loop reads one entry per step, ahead of its use.
    // Walk mode: at every step take the smaller of the two list heads (ascending lists, as stage 3
    // writes them, share the most; any order stays correct).  The list heads are kept as (raw loaded
    // value, in-range flag) and only combined when the next step is formed, one step later: the scalar
    // loads get a whole step to return.  A step is formed in two halves (next_head: which tile and who
    // keeps it; next_advance: move the list positions and fetch the new heads) so that each fits the
    // shadow of one MFMA.  Everything of the walk is kept in 32-bit integers (flags as 0/1, never as
    // booleans) and the step's flags pass through readfirstlane: the walk then stays on the scalar
    // unit and the branches on it are scalar branches.
    constexpr int kEnd = 0x7fffffff;
    int ia = 0, ib = 0;
    int rawA = 0, rawB = 0, okA = 0, okB = 0;
    int gh = 0;         // grouped walk: which half of the current entry comes next
    int ta = 0, tb = 0; // this step consumes the head of list A / B
    // table mode: the raw entry read one step ahead of its use, the next entry to read, steps done
    typedef UnionLds<2, kPairChunk> Table;
    Table& u = *reinterpret_cast<Table*>(smem + 2 * kSlot);
    const uint32_t tab_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)&u.tab[0];
    i32x4 raw_next = {0, 0, 0, 0};
    int s_read = 0, s_done = 0, total = 0;
    const int list_range = kGrouped ? hg.n_tiles / 2 : hg.n_tiles;
    const uint64_t* vmask_g = a.valid_mask + hg.tile_off;
    const int32_t* n0s_g = a.tile_n0 + hg.tile_off;
    if constexpr (kTable) {
        const int32_t* lists[2] = {a.col_idx + begA, a.col_idx + begB};
        const int counts[2] = {nA, kGrouped ? 0 : nB};
        total = union_build<2, 256, kPairChunk>(u, lists, counts, list_range, tid) * (kGrouped ? 2 : 1);
        union_fill<2, 256, kPairChunk, kGrouped>(u, 0, total, list_range, vmask_g, n0s_g, tid);
        union_fill<2, 256, kPairChunk, kGrouped>(u, kPairChunk, total, list_range, vmask_g, n0s_g, tid);
        __syncthreads();
    } else {
        rawA = colsA[0];
        rawB = colsB[0];
        okA = nA > 0 ? 1 : 0;
        okB = nB > 0 ? 1 : 0;
    }
    auto next_head = [&](MergedStep& e) __attribute__((always_inline)) {
        if constexpr (kTable) {
            const UnionStep t = union_step(raw_next);
            e.j = t.j; e.fl = t.fl; e.vm = t.vm; e.n0 = t.n0;
            return;
        }
        int j, fl;
        if (kGrouped) {
            j = okA ? 2 * rawA + gh : 0;
            fl = okA ? 3 : 0;
            ta = gh;
        } else {
            const int headA = okA ? rawA : kEnd, headB = okB ? rawB : kEnd;
            const int jm = headA < headB ? headA : headB;
            const int live = jm != kEnd ? 1 : 0;
            ta = headA == jm ? live : 0;
            tb = headB == jm ? live : 0;
            j = live ? jm : 0;
            fl = ta | (tb << 1);
        }
        e.j = __builtin_amdgcn_readfirstlane(j);
        e.fl = __builtin_amdgcn_readfirstlane(fl);
        e.vm = vmask[e.j];
        e.n0 = kTokK ? n0s[e.j] : 0;
    };
    auto next_advance = [&]() __attribute__((always_inline)) {
        if constexpr (kTable) {
            raw_next = union_read<kPairChunk>(tab_lds, s_read);
            ++s_read;
            return;
        }
        ia += ta;
        okA = ia < nA ? 1 : 0;
        rawA = colsA[okA ? ia : 0];
        if (kGrouped) {
            gh ^= 1;
        } else {
            ib += tb;
            okB = ib < nB ? 1 : 0;
            rawB = colsB[okB ? ib : 0];
        }
    };
    // After the barrier that ends a step (table mode): when the loop has left one half of the
    // table's ring, that half is refilled with the steps that follow the other half's.
    auto step_done = [&]() __attribute__((always_inline)) {
        if constexpr (kTable) {
            ++s_done;
            if ((s_done & (kPairChunk - 1)) == 0)
                union_fill<2, 256, kPairChunk, kGrouped>(u, s_done + kPairChunk, total, list_range, vmask_g, n0s_g, tid);
        }
    };
    if constexpr (kTable) next_advance();   // entry 0 on its way

    // Step s (P = s & 1) computes on slot P while the tiles of step s+1 land in slot P^1.
    const int my_bit = 1 << which;
    MergedStep e0, e1, e2;
    next_head(e0);
    next_advance();
    next_head(e1);
    next_advance();
    if (e0.fl) {
        load_tile(e0, 0, 0);
        load_tile(e0, 0, 1);
    }
    VEDA_LOADS_DONE_BARRIER();   // also the Q loads: nothing vector-memory is pending below

    // One step.  A wave whose query tile keeps the current key tile does its housekeeping (loads of
    // the next tiles, next step of the walk) between the pieces of its step; a wave that skips the
    // step does it on its own.  (Two separate conditionals with an opaque flag rather than
    // if/else: with an else branch the register allocator keeps a second copy of the accumulators.)
#define VEDA_STEP(P)                                                                                     \
    do {                                                                                                 \
        int todo = 1;                                                                                    \
        if (__builtin_expect((e0.fl & my_bit) != 0, 1)) {                                                \
            PairStep<D, kExact> w;                                                                       \
            w.begin(fa, (uint32_t)((P) * kSlot));                                                        \
            w.template block0<0>(st);                                                                    \
            if (e1.fl) load_tile(e1, (P) ^ 1, 0);                                                        \
            w.template block0<1>(st);                                                                    \
            if (e1.fl) load_tile(e1, (P) ^ 1, 1);                                                        \
            w.template block0<2>(st);                                                                    \
            next_head(e2);                                                                               \
            w.template block0<3>(st);                                                                    \
            next_advance();                                                                              \
            w.finish(st, fa, e0.vm);                                                                     \
            todo = 0;                                                                                    \
        }                                                                                                \
        asm volatile("" : "+s"(todo));                                                                   \
        if (todo) {                                                                                      \
            if (e1.fl) {                                                                                 \
                load_tile(e1, (P) ^ 1, 0);                                                               \
                load_tile(e1, (P) ^ 1, 1);                                                               \
            }                                                                                            \
            next_head(e2);                                                                               \
            next_advance();                                                                              \
        }                                                                                                \
        e0 = e1; e1 = e2;                                                                                \
        VEDA_LOADS_DONE_BARRIER();                                                                       \
        step_done();                                                                                     \
    } while (0)
    while (e0.fl) {
        VEDA_STEP(0);
        if (!e0.fl) break;
        VEDA_STEP(1);
    }
#undef VEDA_STEP
#undef VEDA_LOADS_DONE_BARRIER

    finish_pair<D>(st, a, hg, smem, head, qiA, qiB, hasB, b, tid, which, r, lq, hh);
}

veda_status launch_sparse_attn_bf16_pair(const veda_plan* pl, const AttnArgs& a, bool grouped, bool exact, bool walk,
                                         hipStream_t s) {
    const int d = pl->prob.head_dim;
    dim3 grid((unsigned)(kXcd * pl->xcd_max_pairs), (unsigned)pl->prob.batch), block(256);
    // the step table needs a bitmap over the tiles the lists may name
    bool table = !walk;
    for (const HeadGeom& g : pl->heads) table = table && (grouped ? g.n_tiles / 2 : g.n_tiles) <= kUnionMaxTiles;
    // two slots of (K tile + V^T tile), then the step table
    const size_t smem = (size_t)2 * 2 * kTile * d * 2 + (table ? sizeof(UnionLds<2, kPairChunk>) : 0);
#define VEDA_LAUNCH_PAIR_T(DD, GG, KK, EE, TT)                                                           \
    do {                                                                                                 \
        auto kern = sparse_attn_bf16_pair_kernel<DD, GG, KK, EE, TT>;                                    \
        if (smem > 64 * 1024)                                                                            \
            VEDA_HIP_TRY(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem)); \
        hipLaunchKernelGGL(kern, grid, block, smem, s, a);                                               \
    } while (0)
#define VEDA_LAUNCH_PAIR(DD, GG, KK)                                                                     \
    do {                                                                                                 \
        if (exact && table) VEDA_LAUNCH_PAIR_T(DD, GG, KK, true, true);                                  \
        else if (exact) VEDA_LAUNCH_PAIR_T(DD, GG, KK, true, false);                                     \
        else if (table) VEDA_LAUNCH_PAIR_T(DD, GG, KK, false, true);                                     \
        else VEDA_LAUNCH_PAIR_T(DD, GG, KK, false, false);                                               \
    } while (0)
    const int variant = (d == 128 ? 4 : 0) | (grouped ? 2 : 0) | (a.k_tok ? 1 : 0);
    switch (variant) {
        case 0: VEDA_LAUNCH_PAIR(64, false, false); break;
        case 1: VEDA_LAUNCH_PAIR(64, false, true); break;
        case 2: VEDA_LAUNCH_PAIR(64, true, false); break;
        case 3: VEDA_LAUNCH_PAIR(64, true, true); break;
        case 4: VEDA_LAUNCH_PAIR(128, false, false); break;
        case 5: VEDA_LAUNCH_PAIR(128, false, true); break;
        case 6: VEDA_LAUNCH_PAIR(128, true, false); break;
        default: VEDA_LAUNCH_PAIR(128, true, true); break;
    }
#undef VEDA_LAUNCH_PAIR
#undef VEDA_LAUNCH_PAIR_T
    return launch_status("sparse_attn_bf16_pair_kernel");
}

}  // namespace veda
