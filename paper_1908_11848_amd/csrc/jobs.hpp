// Small per-layer jobs of the backward pass that have no kernel of their own: a larger kernel that
// is launched anyway, and does not depend on the job's result, carries them as extra workgroups
// after its own (blockIdx.x >= its own count).  What is saved is a dependent launch per job; the
// job's workgroups run beside the carrier's.  Both jobs are also available as plain kernels.
//
//   ReduceJob : second stage of a d-filter convolution, dw[e] = sum over chunks of partial[chunk][e]
//   TotalsJob : batch-norm backward sums, totals[c] = sum_g records[g][c].{0,1}
//               (= dbeta[c] = sum dz, dgamma[c] = sum dz * xhat), stored for the kernels that apply them
//
// Summation orders are fixed (a lane adds its items in ascending order, lanes are combined by a
// tree), so results do not depend on which kernel carried the job.
#pragma once
#include "common.hpp"

namespace jobs {

constexpr int THREADS = 256;
constexpr int LDS_FLOATS = 1024;        // LDS (16-byte aligned) either job needs

struct ReduceJob {
    const float* partial;   // [chunks][E]
    float* dw;              // [E]
    int E;                  // multiple of 4
    int chunks;
    int blocks;             // workgroups given to the job (0: none); each takes groups of elements round-robin
};

struct TotalsJob {
    const float* records;   // [G][C][2]
    int G;
    int C;                  // multiple of 4
    float* totals;          // [2C]: sum of component 0, then of component 1
    float* dgamma;          // [C] = component 1
    float* dbeta;           // [C] = component 0
    int blocks;             // workgroups given to the job (0: none); must be C / 4
};

// Two shapes, chosen by the number of chunks alone:
//   many chunks (> 64): a workgroup owns 32 consecutive elements (8 sixteen-byte columns) at a time and splits
//       the chunks over 32 row groups; every lane adds its chunks in ascending order and the row groups are
//       combined by a tree.  One "group" = 32 elements.
//   few chunks: a lane owns one sixteen-byte column and adds all chunks in ascending order, eight loads in
//       flight at a time.  One "group" = 1024 elements.
static inline bool reduce_by_rows(int chunks) { return chunks > 64; }
static inline int reduce_groups(int E, int chunks) { return reduce_by_rows(chunks) ? (E + 31) / 32 : (E + 1023) / 1024; }

__device__ __forceinline__ void wgrad_reduce(const ReduceJob& j, int block, float* lds) {
    if (j.chunks <= 64) {
        for (int e = (block * THREADS + (int)threadIdx.x) * 4; e < j.E; e += j.blocks * THREADS * 4) {
            float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int k0 = 0; k0 < j.chunks; k0 += 8) {
                float4 v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u)     // unconditional loads (index clamped), all in flight together
                    v[u] = *reinterpret_cast<const float4*>(j.partial + (long)min(k0 + u, j.chunks - 1) * j.E + e);
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (k0 + u < j.chunks) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
            }
            *reinterpret_cast<float4*>(j.dw + e) = s;
        }
        return;
    }
    float4(*part)[8] = reinterpret_cast<float4(*)[8]>(lds);
    const int cg = threadIdx.x & 7, rg = threadIdx.x >> 3;
    const int groups = (j.E + 31) / 32;
    for (int grp = block; grp < groups; grp += j.blocks) {
        const int e = (grp * 8 + cg) * 4;
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
        if (e < j.E)
            for (int k = rg; k < j.chunks; k += 128) {
                float4 v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    v[u] = (k + 32 * u < j.chunks) ? *reinterpret_cast<const float4*>(j.partial + (long)(k + 32 * u) * j.E + e)
                                                   : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                for (int u = 0; u < 4; ++u) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
            }
        part[rg][cg] = s;
        __syncthreads();
        for (int h = 16; h >= 1; h >>= 1) {
            if (rg < h) {
                float4 a = part[rg][cg];
                const float4 b = part[rg + h][cg];
                a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
                part[rg][cg] = a;
            }
            __syncthreads();
        }
        if (rg == 0 && e < j.E) *reinterpret_cast<float4*>(j.dw + e) = part[0][cg];
        __syncthreads();
    }
}

// One workgroup per 4 channels, 64 lanes per channel; a lane adds records g = lane, lane + 64, ...
__device__ __forceinline__ void bn_totals(const TotalsJob& j, int block, float* lds) {
    constexpr int CW = 4, SUB = THREADS / CW;
    const int cl = threadIdx.x % CW, sub = threadIdx.x / CW;
    const int c = block * CW + cl;
    float sb = 0.f, sg = 0.f;
    for (int g0 = sub; g0 < j.G; g0 += 8 * SUB) {
        float2 pv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)       // unconditional loads (index clamped): all eight in flight together
            pv[u] = *reinterpret_cast<const float2*>(j.records + ((long)min(g0 + u * SUB, j.G - 1) * j.C + c) * 2);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const bool in = g0 + u * SUB < j.G;
            sb += in ? pv[u].x : 0.f;
            sg += in ? pv[u].y : 0.f;
        }
    }
    float* red = lds;                   // [SUB][CW] and a second one behind it
    red[sub * CW + cl] = sb;
    red[THREADS + sub * CW + cl] = sg;
    __syncthreads();
    for (int s = SUB >> 1; s >= 1; s >>= 1) {
        if (sub < s) {
            red[sub * CW + cl] += red[(sub + s) * CW + cl];
            red[THREADS + sub * CW + cl] += red[THREADS + (sub + s) * CW + cl];
        }
        __syncthreads();
    }
    if (sub == 0) {
        const float tb = red[cl], tg = red[THREADS + cl];
        j.totals[c] = tb; j.totals[j.C + c] = tg;
        j.dbeta[c] = tb; j.dgamma[c] = tg;
    }
}

}  // namespace jobs
