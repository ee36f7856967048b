// One key tile for one wave of the bf16 attention kernels: the online-softmax state, the LDS operand
// addresses and the step itself (S^T = K Q^T, softmax, O^T += V^T P^T), shared by the kernels that
// build on it (attn_pair.hip).  Not part of the public ABI.
#pragma once

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

}  // namespace veda
