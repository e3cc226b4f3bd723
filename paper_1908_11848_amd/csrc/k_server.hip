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

// Several pushes that reached the server at the same time, applied in ONE pass over the weights (Alg. 1, server step 2:
// gradients of simultaneous pushes are aggregated before the update).  The pushes keep their order: after gradient j
// the weights are exactly what j single applies would have left (the same fused multiply-add per gradient, in the same
// order), and whoever pulls between push j and push j + 1 - the pusher itself if it is granted OK at once, workers its
// push releases - gets that intermediate version written to its snapshot from registers.  w is read once and written
// once however many gradients there are: (4 m + 8 + 4 snapshots) bytes per parameter instead of 12 m + 8 snapshots.
struct ManyArgs {
    const float* g[DSSPK_APPLY_MANY_MAX];
    float* dst[DSSPK_APPLY_MANY_MAX_DST];
    uint64_t* dst_stamp[DSSPK_APPLY_MANY_MAX_DST];
    unsigned char dst_after[DSSPK_APPLY_MANY_MAX_DST];      // snapshot = weights after this many gradients; ascending
    int m, n_dst;
};

constexpr int kManyChunk = 4;       // gradients fetched together per vector

__global__ __launch_bounds__(kThreads) void apply_many_kernel(float* __restrict__ w, ManyArgs a, long n4, long n, float scale,
                                                               uint64_t* stamp, uint64_t version_first) {
    floatx4* __restrict__ w4 = reinterpret_cast<floatx4*>(w);
    const long stride = (long)gridDim.x * kThreads;
    for (long i = (long)blockIdx.x * kThreads + threadIdx.x; i < n4; i += stride) {
        floatx4 wv = w4[i];
        int d = 0;
        for (int j0 = 0; j0 < a.m; j0 += kManyChunk) {
            floatx4 gv[kManyChunk];
#pragma unroll
            for (int u = 0; u < kManyChunk; ++u)
                if (j0 + u < a.m) gv[u] = __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(a.g[j0 + u]) + i);
#pragma unroll
            for (int u = 0; u < kManyChunk; ++u)
                if (j0 + u < a.m) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) wv[e] = fmaf(-scale, gv[u][e], wv[e]);
                    for (; d < a.n_dst && a.dst_after[d] == j0 + u + 1; ++d)
                        __builtin_nontemporal_store(wv, reinterpret_cast<floatx4*>(a.dst[d]) + i);
                }
        }
        w4[i] = wv;
    }
    if (blockIdx.x == 0) {
        const long t = n4 * 4 + threadIdx.x;            // scalar tail, fewer than 4 elements
        if (t < n) {
            float v = w[t];
            int d = 0;
            for (int j = 0; j < a.m; ++j) {
                v = fmaf(-scale, a.g[j][t], v);
                for (; d < a.n_dst && a.dst_after[d] == j + 1; ++d) a.dst[d][t] = v;
            }
            w[t] = v;
        }
        if (threadIdx.x == 0) {
            *stamp = version_first + (uint64_t)a.m - 1;
            for (int d = 0; d < a.n_dst; ++d)
                if (a.dst_stamp[d]) *a.dst_stamp[d] = version_first + a.dst_after[d] - 1;
        }
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

extern "C" int dsspk_apply_many(void* stream, float* w, int m, const float* const* g, int64_t n, float scale, int n_dst,
                                float* const* dst, const int* dst_after, uint64_t* const* dst_stamp, uint64_t* stamp,
                                uint64_t version_first) {
    if (!w || !g || !stamp || n < 0 || m < 1 || m > DSSPK_APPLY_MANY_MAX || n_dst < 0 || n_dst > DSSPK_APPLY_MANY_MAX_DST) return -1;
    if (n_dst > 0 && (!dst || !dst_after)) return -1;
    ManyArgs a = {};
    a.m = m; a.n_dst = n_dst;
    bool al = aligned16(w);
    for (int j = 0; j < m; ++j) {
        if (!g[j]) return -1;
        a.g[j] = g[j];
        al = al && aligned16(g[j]);
    }
    for (int d = 0; d < n_dst; ++d) {
        if (!dst[d] || dst[d] == w || dst_after[d] < 1 || dst_after[d] > m || (d > 0 && dst_after[d] < dst_after[d - 1])) return -1;
        for (int e = 0; e < d; ++e)
            if (dst[e] == dst[d]) return -1;            // two versions into one snapshot: the caller's mistake
        a.dst[d] = dst[d];
        a.dst_after[d] = (unsigned char)dst_after[d];
        a.dst_stamp[d] = dst_stamp ? dst_stamp[d] : nullptr;
        al = al && aligned16(dst[d]);
    }
    const long n4 = al ? n / 4 : 0;
    if (n4 == 0 && n > 3) return -1;
    const int grid = stream_grid(ceil_div(n4, (long)kThreads * 2));
    hipLaunchKernelGGL(apply_many_kernel, dim3(grid), dim3(kThreads), 0, (hipStream_t)stream, w, a, n4, (long)n, scale, stamp,
                       version_first);
    return DSSPK_LAUNCH_RC();
}
