// Stage 2's fixed-order fp32 chains in the form that defines them (Eq. 5): every projection output
// and every score is ONE chain of scalar fmaf over ascending index, on the vector units.
//
// The kernels in score.hip issue the same chains as v_mfma_f32_32x32x2_f32, which is twice as
// fast and gives the same bits on gfx950 -- a measured property of that instruction (its two
// products are added to the accumulator one after the other, each rounded like an fma, denormals
// kept), not one the instruction set promises.  So the measurement is part of the library:
// probe_chain_unit() runs both forms on chains that exercise rounding, signed zeros and the
// denormal range, once per device (veda_plan_create makes the call), and a plan uses the matrix
// cores only where every bit agreed.  The kernels here are what it uses otherwise, and what
// VEDA_OPT_FP32_CHAIN_UNIT = VEDA_CHAINS_VECTOR selects on any device.  They are written to be
// checked by eye, not to be fast.
#include <atomic>

#include "score_common.h"

namespace veda {

namespace {

constexpr int kVecRows = 8;   // tiles per workgroup of the projection kernel

// out[n] = act(bias[n] + sum_k x[k] * w[k][n]) for one row x: one fmaf chain, k ascending, from the bias.
__device__ inline float affine_chain(const float* x, const float* __restrict__ w, const float* __restrict__ bias,
                                     int K, int N, int n, bool relu) {
    float acc = bias[n];
    for (int k = 0; k < K; ++k) acc = __builtin_fmaf(x[k], w[(int64_t)k * N + n], acc);
    return (relu && !(acc > 0.0f)) ? 0.0f : acc;
}

// grid = (ceil(rows / 8), 2 estimators); one workgroup projects 8 consecutive rows (tiles) of the
// descriptors; tile_head gives each row's head.  Dynamic LDS: [8][in_dim] inputs, [8][hidden] hidden layer.
__global__ __launch_bounds__(256) void mlp_vector_kernel(const uint8_t* __restrict__ tile_head, const float* __restrict__ zq,
                                                         const float* __restrict__ zk, float* __restrict__ yq,
                                                         float* __restrict__ yk, MlpDev pq, MlpDev pk, int64_t total_tiles,
                                                         int64_t rows) {
    extern __shared__ float lds[];
    const MlpDev p = blockIdx.y == 0 ? pq : pk;
    const float* z = blockIdx.y == 0 ? zq : zk;
    float* y = blockIdx.y == 0 ? yq : yk;
    float* xs = lds;                          // [8][in_dim]
    float* hs = lds + kVecRows * p.in_dim;    // [8][hidden]
    const int64_t row0 = (int64_t)blockIdx.x * kVecRows;
    const int nrows = rows - row0 < kVecRows ? (int)(rows - row0) : kVecRows;
    for (int i = threadIdx.x; i < nrows * p.in_dim; i += 256) xs[i] = z[row0 * p.in_dim + i];
    __syncthreads();
    const int first = p.hidden ? p.hidden : p.out_dim;
    for (int i = threadIdx.x; i < nrows * first; i += 256) {
        const int r = i / first, n = i % first;
        const int head = tile_head[(row0 + r) % total_tiles];
        const float v = affine_chain(xs + r * p.in_dim, p.w1 + (int64_t)head * p.in_dim * first, p.b1 + (int64_t)head * first,
                                     p.in_dim, first, n, p.hidden ? p.relu != 0 : false);
        if (p.hidden) hs[r * p.hidden + n] = v;
        else y[(row0 + r) * p.out_dim + n] = v;
    }
    if (!p.hidden) return;
    __syncthreads();
    for (int i = threadIdx.x; i < nrows * p.out_dim; i += 256) {
        const int r = i / p.out_dim, n = i % p.out_dim;
        const int head = tile_head[(row0 + r) % total_tiles];
        y[(row0 + r) * p.out_dim + n] = affine_chain(hs + r * p.hidden, p.w2 + (int64_t)head * p.hidden * p.out_dim,
                                                     p.b2 + (int64_t)head * p.out_dim, p.hidden, p.out_dim, n, false);
    }
}

// Scores of rows [i0, i0 + 16) x all columns of one head: S[i][j] = scale * chain over the latent
// coordinates from +0.  grid = (16-row groups of all heads via row16 lookup, batch).
__global__ __launch_bounds__(256) void score_vector_kernel(const HeadGeom* __restrict__ heads, int n_heads,
                                                           const float* __restrict__ yq, const float* __restrict__ yk,
                                                           float* __restrict__ scores, int dp, float scale,
                                                           int64_t total_tiles, int64_t score_elems,
                                                           const int32_t* __restrict__ marks) {
    // which head: groups are numbered head after head, ceil(n_tiles / 16) each
    int head = 0, g = blockIdx.x;
    while (head < n_heads - 1 && g >= (heads[head].n_tiles + 15) / 16) {
        g -= (heads[head].n_tiles + 15) / 16;
        ++head;
    }
    const HeadGeom hg = heads[head];
    const int nT = hg.n_tiles, i0 = 16 * g;
    if (i0 >= nT) return;
    const int64_t b = blockIdx.y;
    const int64_t lat0 = b * total_tiles + hg.tile_off;
    if (marks) {
        // the matrix-core kernel forms the rows of a 128-row block when the 128-row latent group of its
        // first or of its last row is marked: the same rows here
        const int bi = i0 / 128;
        const int64_t g0 = lat0 + (int64_t)bi * 128;
        const int last = nT - 1 - bi * 128 < 127 ? nT - 1 - bi * 128 : 127;
        if (!(marks[g0 >> 7] | marks[(g0 + last) >> 7])) return;
    }
    float* sbase = scores + b * score_elems + hg.score_off;
    const int rows_here = nT - i0 < 16 ? nT - i0 : 16;
    for (int64_t e = threadIdx.x; e < (int64_t)rows_here * nT; e += 256) {
        const int i = i0 + (int)(e / nT), j = (int)(e % nT);
        const float4* q = reinterpret_cast<const float4*>(yq + (lat0 + i) * dp);   // dp is a multiple of 4
        const float4* k = reinterpret_cast<const float4*>(yk + (lat0 + j) * dp);
        float acc = 0.0f;
        for (int c = 0; c < dp / 4; ++c) {
            const float4 a = q[c], b4 = k[c];
            acc = __builtin_fmaf(a.x, b4.x, acc);
            acc = __builtin_fmaf(a.y, b4.y, acc);
            acc = __builtin_fmaf(a.z, b4.z, acc);
            acc = __builtin_fmaf(a.w, b4.w, acc);
        }
        sbase[(int64_t)i * nT + j] = acc * scale;
    }
}

// The probe: 128 threads x 16 chains of 64 terms, each computed as a chain of
// v_mfma_f32_32x32x2_f32 and as the fmaf chain it stands for; mismatch[thread] = chains whose
// bits differ.  Inputs come from a counter hash; `kinds` gives each of the two waves one of four
// recipes: ordinary magnitudes (products that round), sums in the denormal range, denormal
// products with signed zeros among the terms, large terms that cancel.
typedef __attribute__((ext_vector_type(16))) float probe_f32x16;

__device__ inline uint32_t probe_hash(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}
__device__ inline float probe_value(uint32_t i, int kind) {
    const uint32_t h = probe_hash(i);
    const float u = (float)(int32_t)(h & 0xffffffu) * (1.0f / 8388608.0f) - 1.0f;   // [-1, 1), 24 bits
    if (kind == 0) return u;
    if (kind == 1) return u * 1.0e-19f;                 // products near 1e-38: sums in the denormal range
    if (kind == 2) return (h >> 28) == 0 ? (h & 1 ? -0.0f : 0.0f) : u * 3.0e-22f;   // denormal products, signed zeros
    return (h >> 30) == 0 ? 0.0f : u * 1.0e18f;         // large terms that cancel
}

__global__ __launch_bounds__(128) void chain_probe_kernel(int32_t* __restrict__ mismatch, uint32_t seed, int kinds) {
    __shared__ float xa[2][32][64];   // per wave: A[row][k]
    __shared__ float wb[2][64][32];   // per wave: B[k][column]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, col = lane & 31, kh = lane >> 5;
    const int kind = (kinds + wave) & 3;
    for (int i = lane; i < 32 * 64; i += 64) {
        (&xa[wave][0][0])[i] = probe_value(seed + (uint32_t)(wave * 4096 + i), kind);
        (&wb[wave][0][0])[i] = probe_value(seed + 0x10000u + (uint32_t)(wave * 4096 + i), kind);
    }
    __syncthreads();
    probe_f32x16 acc;
    const float start = probe_value(seed + 0x20000u + wave, kind);
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = start;
    for (int k = 0; k < 64; k += 2)
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[wave][col][k + kh], wb[wave][k + kh][col], acc, 0, 0, 0);
    int bad = 0;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = (r & 3) + 8 * (r >> 2) + 4 * kh;   // the accumulator layout: register r of lane (col, kh)
        float ref = start;
        for (int k = 0; k < 64; ++k) ref = __builtin_fmaf(xa[wave][row][k], wb[wave][k][col], ref);
        bad += __float_as_uint(ref) != __float_as_uint(acc[r]) ? 1 : 0;
    }
    mismatch[threadIdx.x] = bad;
}

constexpr int kMaxDevices = 64;
std::atomic<int> g_chain_unit[kMaxDevices];   // 0 = not probed yet

}  // namespace

// Which unit reproduces the fmaf chains on GPU `device` (the current device): VEDA_CHAINS_MATRIX if
// the matrix-core chains of chain_probe_kernel agree with the fmaf chains in every bit for several
// seeds, else VEDA_CHAINS_VECTOR.  Probed on the first call per device (synchronous: one small
// allocation, a few launches, one copy back), cached afterwards.
veda_status probe_chain_unit(int device, int* unit) {
    if (device < 0 || device >= kMaxDevices) {
        *unit = VEDA_CHAINS_VECTOR;   // no cache slot: the defining form is always right
        return VEDA_OK;
    }
    int u = g_chain_unit[device].load(std::memory_order_acquire);
    if (!u) {
        int32_t* d_bad = nullptr;
        VEDA_HIP_TRY(hipMalloc((void**)&d_bad, 128 * sizeof(int32_t)));
        int total = 0;
        hipError_t e = hipSuccess;
        for (uint32_t pass = 0; pass < 8 && e == hipSuccess; ++pass) {
            int32_t bad[128];
            hipLaunchKernelGGL(chain_probe_kernel, dim3(1), dim3(128), 0, 0, d_bad, 0x9e3779b9u * (pass + 1), (int)(2 * pass));
            e = hipGetLastError();
            if (e == hipSuccess) e = hipMemcpy(bad, d_bad, sizeof(bad), hipMemcpyDeviceToHost);
            if (e == hipSuccess)
                for (int i = 0; i < 128; ++i) total += bad[i];
        }
        (void)hipFree(d_bad);
        if (e != hipSuccess) return hip_fail(e, "probe_chain_unit");
        u = total == 0 ? VEDA_CHAINS_MATRIX : VEDA_CHAINS_VECTOR;
        g_chain_unit[device].store(u, std::memory_order_release);
    }
    *unit = u;
    return VEDA_OK;
}

veda_status launch_projections_vector(const veda_plan* pl, const MlpDev& pq, const MlpDev& pk, const float* zq,
                                      const float* zk, float* yq, float* yk, hipStream_t s) {
    const int64_t rows = pl->total_tiles * pl->prob.batch;
    const int max_hidden = pq.hidden > pk.hidden ? pq.hidden : pk.hidden;
    const size_t smem = sizeof(float) * (size_t)kVecRows * (size_t)(pq.in_dim + max_hidden);
    dim3 grid((unsigned)((rows + kVecRows - 1) / kVecRows), 2);
    hipLaunchKernelGGL(mlp_vector_kernel, grid, dim3(256), smem, s, pl->d_tile_head, zq, zk, yq, yk, pq, pk,
                       pl->total_tiles, rows);
    return launch_status("mlp_vector_kernel");
}

veda_status launch_score_blocks_vector(const veda_plan* pl, const float* yq, const float* yk, float* scores, int dp,
                                       float scale, const int32_t* marks, hipStream_t s) {
    int64_t groups = 0;
    for (const HeadGeom& g : pl->heads) groups += (g.n_tiles + 15) / 16;
    dim3 grid((unsigned)groups, (unsigned)pl->prob.batch);
    hipLaunchKernelGGL(score_vector_kernel, grid, dim3(256), 0, s, pl->d_heads, pl->prob.heads, yq, yk, scores, dp,
                       scale, pl->total_tiles, pl->score_elems, marks);
    return launch_status("score_vector_kernel");
}

}  // namespace veda
