// Host-side launchers of the stage-2 kernels (score.hip), shared with the fused score+select
// route (fused.hip).  Not part of the public ABI.
#pragma once

#include "veda_internal.h"

namespace veda {

constexpr int kLatentRows = 64;   // rows of one row block of the plan's d_row_blk table

// One estimator as the kernels take it (device pointers, per-head arrays back to back).
struct MlpDev {
    int in_dim, hidden, out_dim, relu;
    const float *w1, *b1, *w2, *b2;
};

// Argument check of one estimator (shapes against the plan, supported sizes).
veda_status check_mlp(const veda_plan* pl, const veda_mlp* m);

// TripPool (Eq. 4) of the tiled Q and K into the descriptors zq, zk ([rows][3d] fp32 each).
void launch_trippool(const veda_plan* pl, const void* q_tiled, const void* k_tiled, const uint64_t* valid_mask,
                     float* zq, float* zk, hipStream_t s);

// phi_q, phi_k (Eq. 5) of the descriptors into the latents yq, yk ([rows][out_dim] fp32 each).
// hq, hk: optional scratch of [rows][hidden] floats each for the hidden layers (else they stay
// in LDS, which leaves room for fewer workgroups per compute unit).
veda_status launch_projections(const veda_plan* pl, const veda_mlp* phi_q, const veda_mlp* phi_k, const float* zq,
                               const float* zk, float* yq, float* yk, float* hq, float* hk, hipStream_t s);

// The score blocks of all heads (Eq. 5) from latents of dp coordinates.  marks != nullptr: one
// mark per 128 consecutive rows of the latents (row >> 7); only the score rows of 128-row blocks
// that touch a marked group are formed.
veda_status launch_score_blocks(const veda_plan* pl, const float* yq, const float* yk, float* scores, int dp,
                                float scale, const int32_t* marks, hipStream_t s);

// The same two launches with every chain as scalar fmaf on the vector units (chains_vector.hip): the
// form the arithmetic is defined by, kept selectable (VEDA_OPT_FP32_CHAIN_UNIT) and taken on its own
// on a device where the matrix-core form does not reproduce it (probe_chain_unit).
veda_status launch_projections_vector(const veda_plan* pl, const MlpDev& pq, const MlpDev& pk, const float* zq,
                                      const float* zk, float* yq, float* yk, hipStream_t s);
veda_status launch_score_blocks_vector(const veda_plan* pl, const float* yq, const float* yk, float* scores, int dp,
                                       float scale, const int32_t* marks, hipStream_t s);

}  // namespace veda
