// Server-side kernels: the weight update of a push (Alg. 1, server step 2) and the
// snapshot a worker pulls (Alg. 1, worker steps 2-3).  Both are pure streaming kernels:
// apply reads w and g and writes w (12 B / parameter), pull reads w and writes the
// snapshot (8 B / parameter); apply_pull does both for the pusher that may go on at once
// (16 instead of 20 B / parameter: the new weights go to w and to its snapshot in one pass).
// Each lane moves 16-byte vectors; consecutive lanes touch
// consecutive vectors, so every wavefront issues full 1 KiB coalesced requests.
#include "common.hpp"
#include "../../include/dssp_kernels.h"

namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;      // 16-byte vectors in flight per lane per operand

__global__ __launch_bounds__(kThreads) void apply_kernel(float* __restrict__ w, const float* __restrict__ g,
                                                          long n4, long n, float scale,
                                                          uint64_t* stamp, uint64_t version) {
    floatx4* __restrict__ w4 = reinterpret_cast<floatx4*>(w);
    const floatx4* __restrict__ g4 = reinterpret_cast<const floatx4*>(g);
    const long stride = (long)gridDim.x * kThreads * kUnroll;
    for (long base = (long)blockIdx.x * kThreads * kUnroll + threadIdx.x; base < n4; base += stride) {
        floatx4 wv[kUnroll], gv[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const long i = base + (long)u * kThreads;
            if (i < n4) { wv[u] = w4[i]; gv[u] = __builtin_nontemporal_load(&g4[i]); }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const long i = base + (long)u * kThreads;
            if (i < n4) {
#pragma unroll
                for (int e = 0; e < 4; ++e) wv[u][e] = fmaf(-scale, gv[u][e], wv[u][e]);
                w4[i] = wv[u];
            }
        }
    }
    if (blockIdx.x == 0) {
        const long t = n4 * 4 + threadIdx.x;            // scalar tail, fewer than 4 elements
        if (t < n) w[t] = fmaf(-scale, g[t], w[t]);
        if (threadIdx.x == 0) *stamp = version;
    }
}

__global__ __launch_bounds__(kThreads) void pull_kernel(float* __restrict__ dst, const float* __restrict__ w,
                                                         long n4, long n, uint64_t* dst_stamp, const uint64_t* stamp) {
    floatx4* __restrict__ d4 = reinterpret_cast<floatx4*>(dst);
    const floatx4* __restrict__ w4 = reinterpret_cast<const floatx4*>(w);
    const long stride = (long)gridDim.x * kThreads * kUnroll;
    for (long base = (long)blockIdx.x * kThreads * kUnroll + threadIdx.x; base < n4; base += stride) {
        floatx4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const long i = base + (long)u * kThreads;
            if (i < n4) v[u] = w4[i];
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const long i = base + (long)u * kThreads;
            if (i < n4) __builtin_nontemporal_store(v[u], &d4[i]);
        }
    }
    if (blockIdx.x == 0) {
        const long t = n4 * 4 + threadIdx.x;
        if (t < n) dst[t] = w[t];
        if (threadIdx.x == 0 && dst_stamp) *dst_stamp = *stamp;
    }
}

// apply, with the new weights also written to the pusher's snapshot and its stamp: the pull of a worker that is
// granted OK by its own push.  Same arithmetic as apply_kernel, so w and dst are what apply + pull would give.
__global__ __launch_bounds__(kThreads) void apply_pull_kernel(float* __restrict__ w, const float* __restrict__ g,
                                                               float* __restrict__ dst, long n4, long n, float scale,
                                                               uint64_t* stamp, uint64_t* dst_stamp, uint64_t version) {
    floatx4* __restrict__ w4 = reinterpret_cast<floatx4*>(w);
    floatx4* __restrict__ d4 = reinterpret_cast<floatx4*>(dst);
    const floatx4* __restrict__ g4 = reinterpret_cast<const floatx4*>(g);
    const long stride = (long)gridDim.x * kThreads * kUnroll;
    for (long base = (long)blockIdx.x * kThreads * kUnroll + threadIdx.x; base < n4; base += stride) {
        floatx4 wv[kUnroll], gv[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const long i = base + (long)u * kThreads;
            if (i < n4) { wv[u] = w4[i]; gv[u] = __builtin_nontemporal_load(&g4[i]); }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const long i = base + (long)u * kThreads;
            if (i < n4) {
#pragma unroll
                for (int e = 0; e < 4; ++e) wv[u][e] = fmaf(-scale, gv[u][e], wv[u][e]);
                w4[i] = wv[u];
                __builtin_nontemporal_store(wv[u], &d4[i]);
            }
        }
    }
    if (blockIdx.x == 0) {
        const long t = n4 * 4 + threadIdx.x;            // scalar tail, fewer than 4 elements
        if (t < n) { const float v = fmaf(-scale, g[t], w[t]); w[t] = v; dst[t] = v; }
        if (threadIdx.x == 0) { *stamp = version; if (dst_stamp) *dst_stamp = version; }
    }
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace

extern "C" int dsspk_apply(void* stream, float* w, const float* g, int64_t n, float scale,
                           uint64_t* stamp, uint64_t version) {
    if (!w || !g || !stamp || n < 0) return -1;
    const long n4 = (aligned16(w) && aligned16(g)) ? n / 4 : 0;
    if (n4 == 0 && n > 3) return -1;                  // buffers must be 16-byte aligned
    const int grid = stream_grid(ceil_div(n4, (long)kThreads * kUnroll));
    hipLaunchKernelGGL(apply_kernel, dim3(grid), dim3(kThreads), 0, (hipStream_t)stream,
                       w, g, n4, (long)n, scale, stamp, version);
    return DSSPK_LAUNCH_RC();
}

extern "C" int dsspk_pull(void* stream, float* dst, const float* w, int64_t n,
                          uint64_t* dst_stamp, const uint64_t* stamp) {
    if (!w || !dst || n < 0 || (dst_stamp && !stamp)) return -1;
    const long n4 = (aligned16(w) && aligned16(dst)) ? n / 4 : 0;
    if (n4 == 0 && n > 3) return -1;
    const int grid = stream_grid(ceil_div(n4, (long)kThreads * kUnroll));
    hipLaunchKernelGGL(pull_kernel, dim3(grid), dim3(kThreads), 0, (hipStream_t)stream,
                       dst, w, n4, (long)n, dst_stamp, stamp);
    return DSSPK_LAUNCH_RC();
}

extern "C" int dsspk_apply_pull(void* stream, float* w, const float* g, float* dst, int64_t n, float scale,
                                uint64_t* stamp, uint64_t* dst_stamp, uint64_t version) {
    if (!w || !g || !dst || !stamp || n < 0 || dst == w) return -1;
    const long n4 = (aligned16(w) && aligned16(g) && aligned16(dst)) ? n / 4 : 0;
    if (n4 == 0 && n > 3) return -1;
    const int grid = stream_grid(ceil_div(n4, (long)kThreads * kUnroll));
    hipLaunchKernelGGL(apply_pull_kernel, dim3(grid), dim3(kThreads), 0, (hipStream_t)stream,
                       w, g, dst, n4, (long)n, scale, stamp, dst_stamp, version);
    return DSSPK_LAUNCH_RC();
}
