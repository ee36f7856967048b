// Host-side launchers of the stage-2 kernels (score.hip), shared with the fused score+select
// route (fused.hip).  Not part of the public ABI.
#pragma once

#include "veda_internal.h"

namespace veda {

constexpr int kLatentRows = 64;   // rows of one row block of the plan's d_row_blk table

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

}  // namespace veda
