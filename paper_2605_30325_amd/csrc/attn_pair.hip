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
//                  and the next step of the list walk)
//     S^T block 1 (8 MFMA; in their shadow the row maximum of block 0 and, speculatively, the
//                  first 8 exponentials)
//     one comparison: need the reference move, has the tile padded slots?   (rarely: the slow path)
//     4 x [ 4 MFMA of O^T += V^T P^T ; the next 8 exponentials in their shadow ]   (at raised wave priority)
// K/V tiles are double buffered (2 x 32 KB at d = 128) and filled by direct global->LDS loads
// issued one step ahead.
#include "attn_common.h"

namespace veda {

typedef const __attribute__((address_space(3))) bf16x8* lds_bf16x8_ptr;
__device__ __forceinline__ bf16x8 lds_read16(uint32_t addr) { return *(lds_bf16x8_ptr)(uintptr_t)addr; }

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding).
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

constexpr float kPairSlack = 8.0f;   // log2 units a row maximum may outgrow the softmax reference

// Online-softmax state of one wave: 32 queries of one query tile (one per lane, duplicated in
// the two lane halves).  qf holds Q scaled by softmax_scale*log2(e) (rounded to bf16 once), so
// K Q^T is the logit in log2 units.  ref is the reference point of the exponentials in those
// units: every S^T accumulator STARTS at -ref, so the MFMA chain delivers logit - ref and P is
// a bare exp2 of it.  ref is moved (and S, O, l rescaled) on the first step and afterwards only
// when some row maximum outgrows it by more than kPairSlack; any reference gives the same O
// after the final division by l.
template <int D> struct PairState {
    f32x16 o[D / 32];
    f32x16 start;        // -ref in every register: the C operand of the first MFMA of an S^T block
    bf16x8 qf[D / 16];
    float ref, l_run;
    float resid;         // logits are held divided by this factor (see AttnArgs::scale_resid)
    bool started;
};

// LDS addresses of the wave's operand fragments inside a slot.  The XOR swizzle only touches
// address bits 4-7 (K) / 4-6 (V^T), which the row offsets leave clear, so one base per operand
// is enough: K fragment (key block c, channel step t) is at (k0 ^ (t << 5)) + c * 32 rows,
// V^T fragment (channel block nb, key step kk of 16 slots) at (v0 ^ (kk << 5)) + nb * 4096.
struct PairAddr {
    uint32_t k0, v0;
    int hh;
};

// One key tile for one wave; slot = LDS byte offset of the (K tile, V^T tile) pair.
// Issue order is pinned segment by segment (one MFMA each, scheduling barriers between): an
// MFMA holds the matrix pipe for 32 cycles, a plain VALU op issues in 4 and exp2 in 8, so the
// vector work placed in a segment runs in the MFMA's shadow.  LDS operand reads are issued
// kAhead MFMAs before their consumer.
//
// What a wave has to do besides its MFMAs is spread over their shadows, so that the stretches
// in which it offers the matrix pipe nothing are short (the SIMD's other wave, from the second
// resident workgroup, only fills them when it happens to be in a product of its own):
//   - the step comes in pieces (begin, block0<0..kSideCalls-1>, finish) between which the caller
//     places its per-step housekeeping (the next tiles' global->LDS loads, the next step of the
//     list walk): common code of all waves, not a second copy for the waves that skip the step,
//     which for the active ones runs in the shadow of block 0's MFMAs;
//   - the row maximum of block 0 and the exponentials of its first 8 registers ride on block 1's
//     MFMAs.  The exponentials are speculative: they assume that the reference need not move and
//     that the tile has no padded slot.  After block 1 one comparison per lane (no exchange
//     between the lane halves: the test is "any lane of the wave") decides; in the rare other
//     case the step falls back to masking, the exact row maximum, moving the reference and
//     forming those exponentials again.
constexpr int kSideCalls = 4;

template <int D, bool kExact> struct PairStep {
    static constexpr int G = D / 16, NB = D / 32, kAhead = 6;
    static constexpr int kRowB = D * 2;
    static constexpr int NF = 2 * G + 4 * NB;      // fragments per step: 2G of K, 4*NB of V^T
    static_assert(G % kSideCalls == 0, "block 0's MFMAs are dealt evenly to the side calls");
    static constexpr int kSeg = G / kSideCalls;    // MFMAs of block 0 before each side call
    bf16x8 fr[NF];
    bf16x8 pf[4];     // P^T operand of key step kk = 2c + s2: registers 8*s2..8*s2+7 of block c
    f32x16 s[2];
    uint32_t ka, va;
    // Fragment f in issue order.  f < 2G: K fragment (c = f/G, t = f%G); then V^T fragments
    // (kk = (f-2G)/NB, nb = (f-2G)%NB).
#define VEDA_KF(f) lds_read16((ka ^ (uint32_t)(((f) % G) << 5)) + (uint32_t)(((f) / G) * 32 * kRowB))
#define VEDA_VF(f) lds_read16((va ^ (uint32_t)(((f) / NB) << 5)) + (uint32_t)(((f) % NB) * 4096))
#define VEDA_FRAG(f) ((f) < 2 * G ? VEDA_KF((f) < 2 * G ? (f) : 0) : VEDA_VF((f) < 2 * G ? 0 : (f) - 2 * G))

    // The first operand reads of the step.
    __device__ __forceinline__ void begin(const PairAddr& fa, uint32_t slot) {
        ka = fa.k0 + slot;
        va = fa.v0 + slot;
#pragma unroll
        for (int f = 0; f < kAhead; ++f) fr[f] = VEDA_FRAG(f);
        __builtin_amdgcn_sched_barrier(0);
    }

    // MFMAs kSeg*H .. kSeg*H + kSeg - 1 of S^T block 0; side call H follows them in the caller.
    template <int H> __device__ __forceinline__ void block0(const PairState<D>& st) {
#pragma unroll
        for (int f = kSeg * H; f < kSeg * (H + 1); ++f) {
            fr[f + kAhead] = VEDA_FRAG(f + kAhead);
            s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[f], st.qf[f], f == 0 ? st.start : s[0], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // S^T block 1, the softmax and O^T += V^T P^T.
    __device__ __forceinline__ void finish(PairState<D>& st, const PairAddr& fa, uint64_t vm) {
        float psum = 0.0f;
        // P^T of key step kk: exponentials of registers 8*(kk%2)..+7 of block kk/2
        // two scores at a time, so that the pair is rounded to bf16 by one packed conversion
        typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
#define VEDA_EXP(kk, e)                                                                         \
    do {                                                                                        \
        const float x0_ = s[(kk) >> 1][8 * ((kk) & 1) + (e)], x1_ = s[(kk) >> 1][8 * ((kk) & 1) + (e) + 1]; \
        const float p0_ = __builtin_amdgcn_exp2f(kExact ? x0_ * st.resid : x0_);                \
        const float p1_ = __builtin_amdgcn_exp2f(kExact ? x1_ * st.resid : x1_);                \
        const bf16x2 pr_ = {(__bf16)p0_, (__bf16)p1_};                                          \
        psum += p0_;                                                                            \
        psum += p1_;                                                                            \
        pf[kk][e] = pr_[0];                                                                     \
        pf[kk][(e) + 1] = pr_[1];                                                               \
    } while (0)
        // S^T block 1.  Block 0's last MFMA needs two more to retire; then its row maximum (kMaxSeg
        // MFMAs) and the speculative exponentials of its first 8 registers (the rest) ride along.
        constexpr int kMaxSeg = G >= 8 ? 2 : 1, kExpSeg = G - 2 - kMaxSeg;
        static_assert(kExpSeg >= 1 && 8 % kExpSeg == 0 && (8 / kExpSeg) % 2 == 0, "exponentials come in pairs");
        float mx = -INFINITY;
#pragma unroll
        for (int f = G; f < 2 * G; ++f) {
            fr[f + kAhead] = VEDA_FRAG(f + kAhead);
            s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[f], st.qf[f - G], f == G ? st.start : s[1], 0, 0, 0);
            const int i = f - G - 2;
            if (i >= 0 && i < kMaxSeg) {
#pragma unroll
                for (int e = i * (16 / kMaxSeg); e < (i + 1) * (16 / kMaxSeg); ++e) mx = fmaxf(mx, s[0][e]);
            }
            if (i >= kMaxSeg) {
#pragma unroll
                for (int e = (i - kMaxSeg) * (8 / kExpSeg); e < (i - kMaxSeg + 1) * (8 / kExpSeg); e += 2) VEDA_EXP(0, e);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[1][i]);
        // this lane's half of the row maximum is enough to see whether ANY row of the wave outgrew its reference
        if (__builtin_expect(vm != ~0ull || !st.started || __any((kExact ? mx * st.resid : mx) > kPairSlack), 0)) {
            // The empty asm keeps this a real branch: if-converted into the main block its ~150 vector
            // ops would run on every step.
            asm volatile("" ::: "memory");
            if (vm != ~0ull) {
                // Edge tile: padded key slots get -inf.  Register i of key block c is key slot
                // 32c + 16*(i/8) + 8*hh + (i%8); the lane-dependent part is shifted out first so the
                // per-register tests use constant bit positions.
                mx = -INFINITY;
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const uint32_t half = (uint32_t)(vm >> (32 * c)) >> (8 * fa.hh);
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        if (!((half >> (16 * (i >> 3) + (i & 7))) & 1u)) s[c][i] = -INFINITY;
                        mx = fmaxf(mx, s[c][i]);
                    }
                }
            }
            mx = max_with_other_half(mx);   // row maximum relative to the reference
            if (!st.started || __any((kExact ? mx * st.resid : mx) > kPairSlack)) {
                // Move the reference of every row whose maximum is above it (first step: to the
                // maximum itself, up or down).
                float delta = st.started ? fmaxf(mx, 0.0f) : mx;
                delta = delta == -INFINITY ? 0.0f : delta;
                const float alpha = st.started ? __builtin_amdgcn_exp2f(kExact ? -delta * st.resid : -delta) : 1.0f;   // O = l = 0 before
                st.ref += delta;
                st.l_run *= alpha;
#pragma unroll
                for (int i = 0; i < 16; ++i) st.start[i] = -st.ref;
#pragma unroll
                for (int c = 0; c < 2; ++c)
#pragma unroll
                    for (int i = 0; i < 16; ++i) s[c][i] -= delta;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) st.o[nb][i] *= alpha;
                st.started = true;
            }
            psum = 0.0f;   // the speculative exponentials are void
#pragma unroll
            for (int e = 0; e < 8; e += 2) VEDA_EXP(0, e);
        }
        // The wave that has reached its O^T products goes first at the issue port: the other wave
        // of the SIMD (in its own softmax section, all vector ops) otherwise delays these MFMAs and
        // the matrix pipe idles.  Measured: 6 % fewer cycles for the whole kernel.
        __builtin_amdgcn_s_setprio(1);
        __builtin_amdgcn_sched_barrier(0);
        // O^T += V^T P^T; the 8 exponentials of the next key step are spread over this key step's
        // NB MFMAs
#pragma unroll
        for (int g = 0; g < 4 * NB; ++g) {
            const int f = 2 * G + g;
            if (f + kAhead < NF) fr[f + kAhead] = VEDA_FRAG(f + kAhead);
            const int kk = g / NB, nb = g % NB;
            st.o[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[f], pf[kk], st.o[nb], 0, 0, 0);
            if (kk < 3) {
#pragma unroll
                for (int e = nb * (8 / NB); e < (nb + 1) * (8 / NB); e += 2) VEDA_EXP(kk + 1, e);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_s_setprio(0);
        st.l_run += psum;
#undef VEDA_EXP
    }
#undef VEDA_FRAG
#undef VEDA_KF
#undef VEDA_VF
};

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
template <int D, bool kGrouped, bool kTokK, bool kExact>
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

    // Merged walk: at every step take the smaller of the two list heads; a key tile kept by
    // both query tiles is loaded once and used by both halves of the workgroup.  (Ascending
    // lists, as stage 3 writes them, share the most; any order stays correct.)
    // The list heads are kept as (raw loaded value, in-range flag) and only combined when the
    // next step is formed, one step later: the scalar loads get a whole step to return.
    // A step is formed in two halves (next_head: which tile and who keeps it; next_advance: move
    // the list positions and fetch the new heads) so that each fits the shadow of one MFMA.
    // Everything of the walk is kept in 32-bit integers (flags as 0/1, never as booleans) and the
    // step's flags pass through readfirstlane: the walk then stays on the scalar unit and the
    // branches on it are scalar branches.
    constexpr int kEnd = 0x7fffffff;
    int ia = 0, ib = 0;
    int rawA = colsA[0], rawB = colsB[0];
    int okA = nA > 0 ? 1 : 0, okB = nB > 0 ? 1 : 0;
    int gh = 0;         // grouped walk: which half of the current entry comes next
    int ta = 0, tb = 0; // this step consumes the head of list A / B
    auto next_head = [&](MergedStep& e) __attribute__((always_inline)) {
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
            PairStep<D, kExact> w;                                                                            \
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

veda_status launch_sparse_attn_bf16_pair(const veda_plan* pl, const AttnArgs& a, bool grouped, bool exact, hipStream_t s) {
    const int d = pl->prob.head_dim;
    dim3 grid((unsigned)(kXcd * pl->xcd_max_pairs), (unsigned)pl->prob.batch), block(256);
    const size_t smem = (size_t)2 * 2 * kTile * d * 2;   // two slots of (K tile + V^T tile)
#define VEDA_LAUNCH_PAIR(DD, GG, KK)                                                                     \
    do {                                                                                                 \
        if (exact) hipLaunchKernelGGL((sparse_attn_bf16_pair_kernel<DD, GG, KK, true>), grid, block, smem, s, a);   \
        else hipLaunchKernelGGL((sparse_attn_bf16_pair_kernel<DD, GG, KK, false>), grid, block, smem, s, a);        \
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
    return launch_status("sparse_attn_bf16_pair_kernel");
}

}  // namespace veda
