// Stage 4, fp32 (Eq. 2; Sec. 3.1 masked form; Sec. 4.3 tile skipping; Alg. 1 "UnTile"): the
// accuracy path (1e-4 against the double-precision definition), on the fp32 matrix cores.
//
// Same work split as the bf16 kernel: a workgroup of four wavefronts owns a pair of partner query
// tiles and walks the union of their two kept lists; waves 0,1 hold rows 0-31 / 32-63 of tile A,
// waves 2,3 those of tile B; K tiles ([64][d]) and V^T tiles ([d][64]) are double buffered in LDS
// (2 x 64 KB at d = 128) and filled by direct global->LDS loads issued one step ahead.
//
// Products are formed transposed with v_mfma_f32_32x32x2_f32 (S^T = K Q^T, O^T = V^T P^T): a lane
// owns one query (lane % 32) and one of the two terms of every instruction (h = lane / 32).  The
// pairing of the reduction index with h is free as long as both operands agree, and it is chosen so
// that one 16-byte LDS read feeds four instructions:
//   S^T, step (m, t):  h supplies channel 8m + 4h + t   (K row: float4 at channel 8m + 4h),
//   O^T, step (c, j, t): h supplies key 32c + 8j + 4h + t, which is exactly register 4j + t of the
//                        lane's S^T block c -- P^T needs no rearrangement at all.
// LDS rows are XOR-swizzled by 16-byte chunk (chunk ^ row) so that the 32 lanes reading the same
// chunk of 32 different rows spread over all banks; the swizzle is applied on the global side of
// the direct loads.  Plain online softmax (reference = running row maximum), exp2 with log2(e)
// folded into Q in fp32.
#include "attn_common.h"
#include "attn_union.h"

namespace veda {

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef const __attribute__((address_space(3))) f32x4* lds_f32x4_ptr;
__device__ __forceinline__ f32x4 lds_read_f32x4(uint32_t addr) { return *(lds_f32x4_ptr)(uintptr_t)addr; }

constexpr int kF32Chunk = 256;   // step-table entries filled at a time

// kTable: the steps come from the table in LDS (attn_union.h), as in the bf16 kernel; otherwise the two
// lists are merged inside the loop (heads above 16384 tiles, VEDA_OPT_ATTN_LIST_WALK).
template <int D, bool kTable>
__global__ __launch_bounds__(256, 1) void sparse_attn_f32_kernel(AttnArgs a) {
    constexpr int kKPitch = D * 4;               // bytes of one K row
    constexpr int kKBytes = kTile * kKPitch;     // K tile
    constexpr int kVPitch = kTile * 4;           // bytes of one V^T row (64 keys)
    constexpr int kVBytes = D * kVPitch;         // V^T tile (same size)
    constexpr int kSlot = kKBytes + kVBytes;
    constexpr int kKChunks = kKPitch / 16;       // 16-byte chunks per K row (32 or 16)
    constexpr int kLoads = kKBytes / 1024 / 4;   // direct loads per wave per tile: 8 (d = 128) or 4
    constexpr int kGroups = kLoads / 4;
    constexpr int NB = D / 32;                   // 32-channel blocks of O^T
    constexpr int kM = D / 8;                    // 16-byte K reads per key block and lane
    extern __shared__ __align__(1024) char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int which = wave >> 1, r = wave & 1;
    const int idx = lane & 31, h = lane >> 5;

    int head, pair;
    if (!xcd_work(a.xcd_cum, a.heads, a.n_heads, 2, head, pair)) return;
    const HeadGeom hg = a.heads[head];
    const int64_t b = blockIdx.y;
    int qiA, qiB;
    bool hasB;
    pair_tiles(hg, pair, qiA, qiB, hasB);
    const int qi = which ? qiB : qiA;
    const int64_t head_tile0 = b * a.total_tiles + hg.tile_off;
    const int64_t rowA = head_tile0 + qiA, rowB = head_tile0 + qiB;
    const int begA = a.row_ptr[rowA], nA = a.row_ptr[rowA + 1] - begA;
    const int begB = a.row_ptr[rowB], nB = hasB ? a.row_ptr[rowB + 1] - begB : 0;
    typedef const __attribute__((address_space(4))) int32_t* const_i32_t;
    typedef const __attribute__((address_space(4))) uint64_t* const_u64_t;
    const const_i32_t colsA = (const_i32_t)(uintptr_t)(a.col_idx + begA);
    const const_i32_t colsB = (const_i32_t)(uintptr_t)(a.col_idx + begB);
    const const_u64_t vmask = (const_u64_t)(uintptr_t)(a.valid_mask + hg.tile_off);
    const char* kt = a.k + head_tile0 * kKBytes;
    const char* vt = a.v + head_tile0 * kVBytes;

    // Q operand: lane (query 32r + idx, half h) holds channels 8m + 4h + t, scaled by softmax_scale*log2(e).
    float qreg[D / 2];
    {
        const float* qrow = reinterpret_cast<const float*>(a.q + (head_tile0 + qi) * kKBytes + (32 * r + idx) * kKPitch);
#pragma unroll
        for (int m = 0; m < kM; ++m) {
            const f32x4 v = *reinterpret_cast<const f32x4*>(qrow + 8 * m + 4 * h);
#pragma unroll
            for (int t = 0; t < 4; ++t) qreg[4 * m + t] = v[t] * a.scale_log2;
        }
    }
    f32x16 o[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[nb][i] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;

    // global -> LDS copy plan (see the bf16 kernel): wave w issues instructions w*kLoads .. of each
    // tile, four to an M0 set-up, instruction j of a group with immediate offset 1024*(j%4), which
    // moves the LDS and the global address alike.
    uint32_t k_src[kLoads], v_src[kLoads];
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
        const int inst = wave * kLoads + j;
        const int krow = inst * (1024 / kKPitch) + lane / kKChunks, kpos = lane % kKChunks;
        k_src[j] = krow * kKPitch + ((kpos ^ (krow & (kKChunks - 1))) << 4) - 1024u * (j % 4);
        const int vrow = inst * 4 + (lane >> 4), vpos = lane & 15;
        v_src[j] = vrow * kVPitch + ((vpos ^ (vrow & 15)) << 4) - 1024u * (j % 4);
    }
    const uint32_t smem_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
    const uint32_t wave_lds = smem_base + (uint32_t)wave * (kLoads * 1024);
    auto load_tile = [&](int j_tile, int sl) __attribute__((always_inline)) {
#pragma unroll
        for (int g = 0; g < kGroups; ++g) {
            uint32_t off[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) off[j] = k_src[4 * g + j];
            dma16_group_to_lds<4>(wave_lds + (uint32_t)sl * kSlot + g * 4096, kt + (int64_t)j_tile * kKBytes, off);
        }
#pragma unroll
        for (int g = 0; g < kGroups; ++g) {
            uint32_t off[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) off[j] = v_src[4 * g + j];
            dma16_group_to_lds<4>(wave_lds + (uint32_t)sl * kSlot + kKBytes + g * 4096, vt + (int64_t)j_tile * kVBytes, off);
        }
    };
    // LDS addresses of this lane's operand reads inside a slot, before the per-read XOR.
    const uint32_t k_row0 = smem_base + idx * kKPitch;               // key block 0: row idx (block 1: + 32 rows)
    const uint32_t v_row0 = smem_base + kKBytes + idx * kVPitch;     // channel block 0: row idx (block nb: + 32 nb rows)

    // The steps: the union of the two kept lists.  Table mode: laid out in LDS before the loop; walk mode:
    // merged with scalar loads as the loop goes (32-bit integers on the scalar unit; see the bf16 kernel).
    constexpr int kEnd = 0x7fffffff;
    int ia = 0, ib = 0;
    int rawA = 0, rawB = 0, okA = 0, okB = 0;
    struct Step { int j, fl; uint64_t vm; };
    typedef UnionLds<2, kF32Chunk> Table;
    Table& u = *reinterpret_cast<Table*>(smem + 2 * kSlot);
    const uint32_t tab_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)&u.tab[0];
    const uint64_t* vmask_g = a.valid_mask + hg.tile_off;
    const int32_t* n0s_g = a.tile_n0 + hg.tile_off;
    i32x4 raw_next = {0, 0, 0, 0};
    int s_read = 0, s_done = 0, total = 0;
    if constexpr (kTable) {
        const int32_t* lists[2] = {a.col_idx + begA, a.col_idx + begB};
        const int counts[2] = {nA, nB};
        total = union_build<2, 256, kF32Chunk>(u, lists, counts, hg.n_tiles, tid);
        union_fill<2, 256, kF32Chunk, false>(u, 0, total, hg.n_tiles, vmask_g, n0s_g, tid);
        union_fill<2, 256, kF32Chunk, false>(u, kF32Chunk, total, hg.n_tiles, vmask_g, n0s_g, tid);
        __syncthreads();
        raw_next = union_read<kF32Chunk>(tab_lds, 0);
        s_read = 1;
    } else {
        rawA = colsA[0];
        rawB = colsB[0];
        okA = nA > 0 ? 1 : 0;
        okB = nB > 0 ? 1 : 0;
    }
    auto next_step = [&](Step& e) __attribute__((always_inline)) {
        if constexpr (kTable) {
            const UnionStep t = union_step(raw_next);
            e.j = t.j; e.fl = t.fl; e.vm = t.vm;
            raw_next = union_read<kF32Chunk>(tab_lds, s_read);
            ++s_read;
            return;
        }
        const int headA = okA ? rawA : kEnd, headB = okB ? rawB : kEnd;
        const int jm = headA < headB ? headA : headB;
        const int live = jm != kEnd ? 1 : 0;
        const int ta = headA == jm ? live : 0, tb = headB == jm ? live : 0;
        e.j = __builtin_amdgcn_readfirstlane(live ? jm : 0);
        e.fl = __builtin_amdgcn_readfirstlane(ta | (tb << 1));
        e.vm = vmask[e.j];
        ia += ta;
        ib += tb;
        okA = ia < nA ? 1 : 0;
        okB = ib < nB ? 1 : 0;
        rawA = colsA[okA ? ia : 0];
        rawB = colsB[okB ? ib : 0];
    };

    const int my_bit = 1 << which;
    Step e0, e1, e2;
    next_step(e0);
    next_step(e1);
    if (e0.fl) load_tile(e0.j, 0);
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the Q loads and the first tile
    __syncthreads();

    for (int P = 0; e0.fl; P ^= 1) {
        if (e1.fl) load_tile(e1.j, P ^ 1);
        next_step(e2);
        if (e0.fl & my_bit) {
            const uint32_t slot = (uint32_t)P * kSlot;
            // S^T = K Q^T, two key blocks of 32
            f32x16 s[2];
#pragma unroll
            for (int c = 0; c < 2; ++c) {
#pragma unroll
                for (int i = 0; i < 16; ++i) s[c][i] = 0.0f;
                const int krow = 32 * c + idx;
                const uint32_t kaddr = k_row0 + slot + (uint32_t)(32 * c * kKPitch);
#pragma unroll
                for (int m = 0; m < kM; ++m) {
                    const f32x4 kf = lds_read_f32x4(kaddr + (uint32_t)((((2 * m + h) ^ krow) & (kKChunks - 1)) << 4));
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        s[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(kf[t], qreg[4 * m + t], s[c], 0, 0, 0);
                }
            }
            // padded key slots: register i of block c is key slot 32c + 8*(i/4) + 4h + i%4
            float mx = -INFINITY;
            const uint64_t vm = e0.vm;
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const uint32_t half = (uint32_t)(vm >> (32 * c)) >> (4 * h);
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    if (vm != ~0ull && !((half >> (8 * (i >> 2) + (i & 3))) & 1u)) s[c][i] = -INFINITY;
                    mx = fmaxf(mx, s[c][i]);
                }
            }
            mx = max_with_other_half(mx);
            const float m_new = fmaxf(m_run, mx);
            const float m_use = m_new == -INFINITY ? 0.0f : m_new;
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);   // 0 on the first step (m_run = -inf)
            float psum = 0.0f;
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    s[c][i] = __builtin_amdgcn_exp2f(s[c][i] - m_use);
                    psum += s[c][i];
                }
            l_run = l_run * alpha + psum;
            m_run = m_new;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[nb][i] *= alpha;
            // O^T += V^T P^T
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int vrow = 32 * nb + idx;
                const uint32_t vaddr = v_row0 + slot + (uint32_t)(32 * nb * kVPitch);
#pragma unroll
                for (int c = 0; c < 2; ++c)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const f32x4 vf = lds_read_f32x4(vaddr + (uint32_t)((((8 * c + 2 * j + h) ^ vrow) & 15) << 4));
#pragma unroll
                        for (int t = 0; t < 4; ++t)
                            o[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(vf[t], s[c][4 * j + t], o[nb], 0, 0, 0);
                    }
            }
        }
        e0 = e1;
        e1 = e2;
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's loads of the next tiles have landed
        __syncthreads();
        if constexpr (kTable) {   // the table's other half has been left behind: refill it
            ++s_done;
            if ((s_done & (kF32Chunk - 1)) == 0)
                union_fill<2, 256, kF32Chunk, false>(u, s_done + kF32Chunk, total, hg.n_tiles, vmask_g, n0s_g, tid);
        }
    }

    // Normalise, transpose through LDS ([2 tiles][64 rows][D] fp32) and scatter the real rows.
    const float l_all = l_run + __shfl_xor(l_run, 32);
    const float inv = l_all > 0.0f ? 1.0f / l_all : 0.0f;
    float* obuf = reinterpret_cast<float*>(smem);
    float* lse_s = obuf + 2 * kTile * D;
    int* tok_s = reinterpret_cast<int*>(lse_s + 2 * kTile);
    if (tid < 2 * kTile) tok_s[tid] = slot_token(hg, tid / kTile ? qiB : qiA, tid % kTile, a.T, a.H, a.W);
    {
        float* orow = obuf + (which * kTile + 32 * r + idx) * D;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                f32x4 v;
#pragma unroll
                for (int t = 0; t < 4; ++t) v[t] = o[nb][4 * j + t] * inv;
                *reinterpret_cast<f32x4*>(orow + 32 * nb + 8 * j + 4 * h) = v;
            }
        if (h == 0) lse_s[which * kTile + 32 * r + idx] = (m_run + __log2f(l_all)) * kLn2;
    }
    __syncthreads();
    char* ob = a.out + b * a.so_b + head * a.so_h;
    const int n_tiles = hasB ? 2 : 1;
    for (int cid = tid; cid < n_tiles * kTile * kKChunks; cid += 256) {
        const int row = cid / kKChunks, ch = cid % kKChunks;
        const int n = tok_s[row];
        if (n >= 0)
            *reinterpret_cast<uint4*>(ob + (int64_t)n * a.so_n + ch * 16) =
                *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(obuf) + row * kKPitch + ch * 16);
    }
    if (a.lse && tid < n_tiles * kTile) {
        const int n = tok_s[tid];
        if (n >= 0) a.lse[(b * a.n_heads + head) * a.tokens + n] = lse_s[tid];
    }
}

veda_status launch_sparse_attn_f32(const veda_plan* pl, const AttnArgs& a, bool walk, hipStream_t s) {
    const int d = pl->prob.head_dim;
    dim3 grid((unsigned)(kXcd * pl->xcd_max_pairs), (unsigned)pl->prob.batch), block(256);
    bool table = !walk;   // the step table's bitmaps cover 16384 tiles per head
    for (const HeadGeom& g : pl->heads) table = table && g.n_tiles <= kUnionMaxTiles;
    // two slots of (K tile + V^T tile), then the step table
    const size_t smem = (size_t)2 * 2 * kTile * d * 4 + (table ? sizeof(UnionLds<2, kF32Chunk>) : 0);
#define VEDA_LAUNCH_F32(DD, TT)                                                                          \
    do {                                                                                                 \
        auto kern = sparse_attn_f32_kernel<DD, TT>;                                                      \
        if (smem > 64 * 1024)                                                                            \
            VEDA_HIP_TRY(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem)); \
        hipLaunchKernelGGL(kern, grid, block, smem, s, a);                                               \
    } while (0)
    if (d == 128) {
        if (table) VEDA_LAUNCH_F32(128, true); else VEDA_LAUNCH_F32(128, false);
    } else {
        if (table) VEDA_LAUNCH_F32(64, true); else VEDA_LAUNCH_F32(64, false);
    }
#undef VEDA_LAUNCH_F32
    return launch_status("sparse_attn_f32_kernel");
}

}  // namespace veda
