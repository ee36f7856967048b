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
// K and V^T tiles are double buffered in LDS (2 x 32 KB for d = 128) and filled by direct
// global->LDS loads, K running one step ahead of V: while the vector ALUs do the softmax of
// step i the matrix cores already form S of step i+1.  16-byte chunks are XOR-swizzled inside
// each LDS row so the per-lane row-strided operand reads do not pile onto the same banks.
//
// fp32 kernel: plain fp32 VALU arithmetic, one workgroup per query tile (small problems and
// the 1e-4 accuracy bar; not a throughput path).
#include "veda_internal.h"

namespace veda {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct AttnArgs {
    const HeadGeom* heads;
    const uint8_t* tile_head;
    const int32_t* xcd_cum;
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

// Workgroups are dealt round-robin to the 8 dies (XCDs), each with its own L2, all sharing
// the 256 MB memory-side cache.  Die x = blockIdx.x % 8 takes the x-th eighth of every head's
// query tiles and walks the heads in order: all dies then work on the same head at the same
// time (its K/V, ~120 MB at 220k tokens, stay in the memory-side cache), and the workgroups
// sharing an L2 hold neighbouring query tiles, whose kept key tiles overlap.
// xcd_work() returns false for the padding workgroups of dies with fewer tiles.

__device__ inline int rho(int m) {  // swap bits 2 and 3
    return (m & ~12) | ((m & 4) << 1) | ((m & 8) >> 1);
}

// 16 bytes per lane straight from global memory into LDS: lane i of the wave lands at LDS byte
// lds_base + 16*i (lds_base wave-uniform), from global address base + voff (base uniform).
// Written as inline assembly so that the compiler does not serialise later LDS reads of OTHER
// buffers behind these loads; completion is awaited explicitly (vmcnt) before the barrier that
// publishes the buffer.  M0 carries the LDS base and is dead outside the statement.
__device__ __forceinline__ void dma16_to_lds(uint32_t lds_base, const void* base, uint32_t voff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_base), "v"(voff), "s"(base)
                 : "memory");
}

__device__ inline bool xcd_work(const int32_t* __restrict__ xcd_cum, const HeadGeom* __restrict__ heads,
                                int n_heads, int& head, int& qi) {
    const int x = blockIdx.x % kXcd, local = blockIdx.x / kXcd;
    const int32_t* cum = xcd_cum + x * (n_heads + 1);
    if (local >= cum[n_heads]) return false;
    int h = 0;
    while (local >= cum[h + 1]) ++h;
    const int n = heads[h].n_tiles;
    head = h;
    qi = x * (n / kXcd) + (x < n % kXcd ? x : n % kXcd) + (local - cum[h]);
    return true;
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

    int head, qi;
    if (!xcd_work(a.xcd_cum, a.heads, a.n_heads, head, qi)) return;
    const HeadGeom hg = a.heads[head];
    const int64_t b = blockIdx.y;
    const int64_t row = b * a.total_tiles + hg.tile_off + qi;
    const int beg = a.row_ptr[row];
    const int nsel = a.row_ptr[row + 1] - beg;
    // The kept list and the validity masks are read-only for the whole launch and indexed
    // uniformly: reading them through the constant address space makes them scalar loads, so
    // no vector-memory counter waits of the compiler's own end up inside the main loop.
    typedef const __attribute__((address_space(4))) int32_t* const_i32_t;
    typedef const __attribute__((address_space(4))) uint64_t* const_u64_t;
    const const_i32_t cols = (const_i32_t)(uintptr_t)(a.col_idx + beg);
    const int64_t head_tile0 = b * a.total_tiles + hg.tile_off;
    const char* kt = a.k + head_tile0 * kKBytes;
    const char* vt = a.v + head_tile0 * kVBytes;
    const const_u64_t vmask = (const_u64_t)(uintptr_t)(a.valid_mask + hg.tile_off);

    // Q operand (B matrix of S^T = K Q^T): lane holds query row 32r+lq, channels 16t+8hh..+8.
    bf16x8 qf[D / 16];
    {
        const char* qrow = a.q + (head_tile0 + qi) * kKBytes + (32 * r + lq) * kRowB + 16 * hh;
#pragma unroll
        for (int t = 0; t < D / 16; ++t) qf[t] = *reinterpret_cast<const bf16x8*>(qrow + 32 * t);
    }

    // global -> LDS copy plan.  Loads go straight from global memory into LDS (no staging
    // registers): one wave instruction fills 1 KB of LDS, lane i at byte 16*i, so the swizzle
    // is applied on the global side -- each lane fetches the chunk that belongs at its fixed
    // LDS position.  Wave w issues instructions w*kLoads .. w*kLoads+kLoads-1 of each tile.
    int k_src[kLoads], v_src[kLoads];
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
        const int inst = wave * kLoads + j;
        const int krow = inst * (1024 / kRowB) + lane / kKChunks, kpos = lane % kKChunks;
        k_src[j] = krow * kRowB + ((kpos ^ (rho(krow & 31) & (kKChunks - 1))) << 4);
        const int vrow = inst * 8 + (lane >> 3), vpos = lane & 7;
        v_src[j] = vrow * 128 + ((vpos ^ (((vrow >> 1) & 7) ^ ((vrow & 1) << 2))) << 4);
    }
    const uint32_t smem_base = (uint32_t)(uintptr_t)smem;
    const uint32_t wave_lds = smem_base + (uint32_t)__builtin_amdgcn_readfirstlane(wave) * (kLoads * 1024);
#define VEDA_LOAD_K(j_tile, SLOT)                                                                          \
    do {                                                                                                   \
        const char* src_ = kt + (int64_t)(j_tile) * kKBytes;                                               \
        _Pragma("unroll") for (int j = 0; j < kLoads; ++j)                                                 \
            dma16_to_lds(wave_lds + (SLOT) * kStage + j * 1024, src_, (uint32_t)k_src[j]);                 \
    } while (0)
#define VEDA_LOAD_V(j_tile, SLOT)                                                                          \
    do {                                                                                                   \
        const char* src_ = vt + (int64_t)(j_tile) * kVBytes;                                               \
        _Pragma("unroll") for (int j = 0; j < kLoads; ++j)                                                 \
            dma16_to_lds(wave_lds + (SLOT) * kStage + kKBytes + j * 1024, src_, (uint32_t)v_src[j]);       \
    } while (0)
    // All of this wave's LDS-bound loads have landed (vmcnt 0), then meet the other waves.
#define VEDA_LOADS_DONE_BARRIER()              \
    do {                                       \
        __builtin_amdgcn_s_waitcnt(0x0F70);    \
        __syncthreads();                       \
    } while (0)

    // per-lane operand read offsets inside a slot (swizzle folded in, one register each)
    const char* k_addr[D / 16];
    const char* v_addr[D / 32][2];
#pragma unroll
    for (int t = 0; t < D / 16; ++t)
        k_addr[t] = smem + (32 * c + rho(lq)) * kRowB + (((2 * t + hh) ^ (lq & (kKChunks - 1))) << 4);
#pragma unroll
    for (int nb = 0; nb < D / 32; ++nb) {
        const int vrow = 32 * nb + lq;
        const int swz = ((vrow >> 1) & 7) ^ ((vrow & 1) << 2);
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) v_addr[nb][s2] = smem + kKBytes + vrow * 128 + (((4 * c + 2 * s2 + hh) ^ swz) << 4);
    }

    f32x16 o[D / 32];
#pragma unroll
    for (int nb = 0; nb < D / 32; ++nb)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[nb][i] = 0.0f;
    // Online softmax state of this lane's query over this wave's key subset.  m_ref is the
    // reference point of the exponentials, not necessarily the running maximum: it is only
    // moved (and O, l rescaled) when some row's maximum outgrows it by more than 2^kSlack,
    // which keeps the 64-register rescale off the common path.  Any reference gives the
    // same O after the final division by l.
    constexpr float kSlack = 8.0f;
    float m_ref = -INFINITY, mc = 0.0f, l_run = 0.0f;

    // S^T (32 keys x 32 queries) = K_half Q^T from K slot SLOT into DST.
#define VEDA_QK(DST, SLOT)                                                                             \
    do {                                                                                               \
        _Pragma("unroll") for (int i = 0; i < 16; ++i) DST[i] = 0.0f;                                  \
        _Pragma("unroll") for (int t = 0; t < D / 16; ++t) {                                           \
            const bf16x8 kf = *reinterpret_cast<const bf16x8*>(k_addr[t] + (SLOT) * kStage);           \
            DST = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[t], DST, 0, 0, 0);                    \
        }                                                                                              \
    } while (0)

    // Value of the lane that holds the other 16 keys of the same query (lane ^ 32).
    const int swap_addr = (lane ^ 32) << 2;
#define VEDA_SWAP32(X) __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(swap_addr, __builtin_bit_cast(int, (X))))

    // Row maximum of a raw S^T accumulator: in-register over the lane's 16 keys, then one
    // exchange with the lane holding the other 16 keys of the same query.
#define VEDA_ROWMAX(S, M)                                                          \
    do {                                                                           \
        M = S[0];                                                                  \
        _Pragma("unroll") for (int i = 1; i < 16; ++i) M = fmaxf(M, S[i]);         \
        M = fmaxf(M, VEDA_SWAP32(M));                                              \
    } while (0)

    // Step `it` of the kept list, P = it & 1.  On entry LDS holds K(it+1) in K slot P^1 and
    // V(it) in V slot P; s_cur = S(it) (raw) and mloc = its row maximum.  The step starts the
    // loads of K(it+2) and V(it+1) into the slots step it-1 finished with.  Two rare branches
    // come first (edge tiles: mask padded keys; reference moved: rescale).  The rest is one
    // straight-line block cut into segments by scheduling barriers, one MFMA per segment: an
    // MFMA holds the matrix pipe for 32 cycles, a plain VALU op issues in 4 and exp2 in 8, so
    // each S(it+1) MFMA carries the scale-exponentiate-pack work of 2 (d=128) or 4 (d=64)
    // scores of S(it) in its shadow, and each P V(it) MFMA a share of the row-sum / next
    // row-maximum bookkeeping.  LDS operand reads are issued kAhead MFMAs early.
    // jA = tile of step it+1, jB = tile of step it+2 (clamped), vmA = mask of jA.
#define VEDA_STEP(P)                                                                                       \
    do {                                                                                                   \
        if (it + 2 < nsel) VEDA_LOAD_K(jB, (P));                                                           \
        if (it + 1 < nsel) VEDA_LOAD_V(jA, (P) ^ 1);                                                       \
        const int jC = cols[it + 3 < nsel ? it + 3 : nsel - 1];                                            \
        const uint64_t vmB = vmask[jB];                                                                    \
        /* register i of this lane is key slot 32c + 16*(i/8) + 8*hh + (i%8) of the tile */                \
        if (vm_cur != ~0ull) {                                                                             \
            const uint32_t half = (uint32_t)(vm_cur >> (32 * c));                                          \
            _Pragma("unroll") for (int i = 0; i < 16; ++i)                                                 \
                if (!((half >> (16 * (i >> 3) + 8 * hh + (i & 7))) & 1u)) s_cur[i] = -INFINITY;            \
            VEDA_ROWMAX(s_cur, mloc);                                                                      \
        }                                                                                                  \
        if (__any((mloc - m_ref) * a.scale_log2 > kSlack)) {                                               \
            const float m_new = fmaxf(m_ref, mloc);                                                        \
            const float m_use = m_new == -INFINITY ? 0.0f : m_new;                                         \
            const float alpha = __builtin_amdgcn_exp2f((m_ref - m_use) * a.scale_log2);                    \
            m_ref = m_new;                                                                                 \
            mc = m_use * a.scale_log2;                                                                     \
            l_run *= alpha;                                                                                \
            _Pragma("unroll") for (int nb = 0; nb < D / 32; ++nb)                                          \
                _Pragma("unroll") for (int i = 0; i < 16; ++i) o[nb][i] *= alpha;                          \
        }                                                                                                  \
        /* ---- straight-line block, issue order pinned segment by segment ---- */                          \
        /* S(it+1); on the last step this reads a stale slot and the result is dropped */                  \
        f32x16 s_next;                                                                                     \
        _Pragma("unroll") for (int i = 0; i < 16; ++i) s_next[i] = 0.0f;                                   \
        bf16x8 fr[2 * G];                                                                                  \
        bf16x8 pf[2];                                                                                      \
        float psum = 0.0f, mx0 = -INFINITY;                                                                \
        _Pragma("unroll") for (int f = 0; f < kAhead; ++f) fr[f] = VEDA_FRAG(f, P);                        \
        __builtin_amdgcn_sched_barrier(0);                                                                 \
        _Pragma("unroll") for (int g = 0; g < G; ++g) {                                                    \
            fr[g + kAhead] = VEDA_FRAG(g + kAhead, P);                                                     \
            s_next = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[g], qf[g], s_next, 0, 0, 0);               \
            _Pragma("unroll") for (int e = 0; e < 16 / G; ++e) {                                           \
                const int i = g * (16 / G) + e;                                                            \
                s_cur[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[i], a.scale_log2, -mc));            \
                pf[i >> 3][i & 7] = (__bf16)s_cur[i];                                                      \
            }                                                                                              \
            __builtin_amdgcn_sched_barrier(0);                                                             \
        }                                                                                                  \
        /* O^T (d x 32 queries) += V^T[:, keys of this half] P^T; bookkeeping rides along */               \
        _Pragma("unroll") for (int g = 0; g < G; ++g) {                                                    \
            if (g + kAhead < G) fr[G + g + kAhead] = VEDA_FRAG(G + g + kAhead, P);                         \
            const int nb = g % (D / 32), s2 = g / (D / 32);                                                \
            o[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[G + g], pf[s2], o[nb], 0, 0, 0);            \
            _Pragma("unroll") for (int e = 0; e < 16 / G; ++e) psum += s_cur[g * (16 / G) + e];            \
            if (g >= G / 2) {                                                                              \
                _Pragma("unroll") for (int e = 0; e < 16 / (G / 2); e += 2) {                              \
                    const int i = (g - G / 2) * (16 / (G / 2)) + e;                                        \
                    mx0 = fmaxf(fmaxf(mx0, s_next[i]), s_next[i + 1]);                                     \
                }                                                                                          \
            }                                                                                              \
            __builtin_amdgcn_sched_barrier(0);                                                             \
        }                                                                                                  \
        l_run += psum;                                                                                     \
        mloc = fmaxf(mx0, VEDA_SWAP32(mx0));                                                               \
        s_cur = s_next;                                                                                    \
        vm_cur = vmA;                                                                                      \
        vmA = vmB;                                                                                         \
        jA = jB;                                                                                           \
        jB = jC;                                                                                           \
        VEDA_LOADS_DONE_BARRIER();                                                                         \
    } while (0)

    // Operand fragment f of a step: f < G are the K fragments of S(it+1) (K slot P^1), the
    // rest the V^T fragments of P V(it) (V slot P) in issue order s2-major.
    constexpr int G = D / 16;
    constexpr int kAhead = 3;   // LDS reads run this many MFMAs ahead of their consumer
#define VEDA_FRAG(f, P)                                                                                  \
    (*reinterpret_cast<const bf16x8*>(                                                                   \
        (f) < G ? k_addr[(f) < G ? (f) : 0] + ((P) ^ 1) * kStage                                         \
                : v_addr[((f) < G ? 0 : (f) - G) % (D / 32)][((f) < G ? 0 : (f) - G) / (D / 32)] + (P) * kStage))

    f32x16 s_cur;
#pragma unroll
    for (int i = 0; i < 16; ++i) s_cur[i] = 0.0f;
    float mloc = -INFINITY;
    uint64_t vm_cur = 0ull, vmA = 0ull;
    int jA = 0, jB = 0;
    if (nsel > 0) {
        const int j0 = cols[0];
        jA = cols[nsel > 1 ? 1 : 0];
        jB = cols[nsel > 2 ? 2 : nsel - 1];
        vm_cur = vmask[j0];
        vmA = vmask[jA];
        VEDA_LOAD_K(j0, 0);
        VEDA_LOAD_V(j0, 0);
        if (nsel > 1) VEDA_LOAD_K(jA, 1);
        VEDA_LOADS_DONE_BARRIER();
        VEDA_QK(s_cur, 0);
        VEDA_ROWMAX(s_cur, mloc);
    }
    // K slot 0 has been read by every wave before step 0 refills it.  The vmcnt(0) here is on
    // every path into the loop, so the compiler knows the Q loads are complete and puts no
    // vector-memory waits of its own between the in-loop prefetches and their consumers.
    VEDA_LOADS_DONE_BARRIER();
    int it = 0;
    for (; it + 1 < nsel; it += 2) {
        VEDA_STEP(0);
        ++it;
        VEDA_STEP(1);
        --it;
    }
    if (it < nsel) VEDA_STEP(0);
    const float m_run = m_ref;

#undef VEDA_LOAD_K
#undef VEDA_LOAD_V
#undef VEDA_LOADS_DONE_BARRIER
#undef VEDA_QK
#undef VEDA_STEP
#undef VEDA_ROWMAX
#undef VEDA_FRAG
#undef VEDA_SWAP32
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
    int head, qi;
    if (!xcd_work(a.xcd_cum, a.heads, a.n_heads, head, qi)) return;
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
    a.xcd_cum = pl->d_xcd_cum;
    dim3 grid((unsigned)(kXcd * pl->xcd_max_tiles), (unsigned)pl->prob.batch), block(256);
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
