// Batch-norm statistics records and their merge, shared by the batch-norm kernels and by the
// convolution kernels that normalise their input while loading it.
//
// A record is (mean, sum of squared deviations from that mean) of one channel over a slab of
// rows; slabs have `rows_per_block` rows (the last one possibly fewer).  Records come either from
// bn_stats_partial_kernel (row slabs) or from the epilogue of a convolution kernel (one record per
// workgroup tile).  Every consumer merges them itself, with identical arithmetic, in its prologue.
#pragma once
#include "common.hpp"

namespace bnm {

constexpr int THREADS = 256;

struct BnLayout {
    int VC, RL;          // 16-byte columns per row, row lanes per workgroup
    long rows_per_block;
    int G;               // slabs = workgroups of the partial kernels
};

__host__ __device__ inline BnLayout bn_layout(long M, int C) {
    BnLayout L;
    L.VC = C / 4;
    L.RL = THREADS / L.VC;
    const long gmax = 32L * (THREADS / C);          // the merge takes at most 32 slab results per lane
    long rpb = (M + gmax - 1) / gmax;
    if (rpb < 64) rpb = 64;
    rpb = (rpb + L.RL - 1) / L.RL * L.RL;
    L.rows_per_block = rpb;
    L.G = (int)((M + rpb - 1) / rpb);
    return L;
}

// Sum `v` over the SUB lanes that share a channel (tree in LDS); result broadcast to all of them.
__device__ __forceinline__ float reduce_sub(float v, float* red, int c, int sub, int SUB, int C) {
    red[sub * C + c] = v;
    __syncthreads();
    for (int s = SUB >> 1; s >= 1; s >>= 1) {
        if (sub < s) red[sub * C + c] += red[(sub + s) * C + c];
        __syncthreads();
    }
    const float out = red[c];
    __syncthreads();
    return out;
}

// Merge of the slab results by the whole workgroup (THREADS / C lanes per channel):
// mean = sum n_g mean_g / M, M2 = sum (M2_g + n_g (mean_g - mean)^2).
// On return sh[c] = mean, sh[C + c] = 1 / sqrt(M2 / M + eps) for every channel.
__device__ __forceinline__ void bn_merge_stats(const float* __restrict__ partial, long M, int C, float eps, float* red, float* sh, const BnLayout& L) {
    const int SUB = THREADS / C;
    const int c = threadIdx.x % C, sub = threadIdx.x / C;
    // All slab results of this lane are fetched in one batch (G <= 32 * SUB: at most 32 per lane).
    // The loads are unconditional (index clamped) so that they are all in flight together; slabs past
    // the end get weight 0.
    float2 pv[32];
    float nn[32];
#pragma unroll
    for (int u = 0; u < 32; ++u) {
        const int g = sub + u * SUB;
        const int gc = min(g, L.G - 1);
        pv[u] = *reinterpret_cast<const float2*>(partial + ((long)gc * C + c) * 2);
        const long lo = (long)gc * L.rows_per_block;
        nn[u] = g < L.G ? (float)(min(M, lo + L.rows_per_block) - lo) : 0.f;
    }
    float s = 0.f;
#pragma unroll
    for (int u = 0; u < 32; ++u) s = fmaf(nn[u], pv[u].x, s);
    const float mean = reduce_sub(s, red, c, sub, SUB, C) / (float)M;
    float m2 = 0.f;
#pragma unroll
    for (int u = 0; u < 32; ++u) {
        const float d = pv[u].x - mean;
        m2 += nn[u] > 0.f ? pv[u].y + nn[u] * d * d : 0.f;
    }
    m2 = reduce_sub(m2, red, c, sub, SUB, C);
    if (sub == 0) {
        sh[c] = mean;
        sh[C + c] = 1.0f / sqrtf(m2 / (float)M + eps);
    }
    __syncthreads();
}

}  // namespace bnm
