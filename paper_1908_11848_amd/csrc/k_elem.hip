// Bandwidth-bound pieces of the worker gradient (Alg. 1, worker step 4): batch normalisation,
// ReLU, residual shortcut, pooling, softmax cross-entropy.  Activations are [rows][C] with C
// contiguous; a workgroup is laid out as (row lanes) x (C/4 sixteen-byte columns), so every
// wavefront reads whole contiguous rows and per-channel sums are reduced across row lanes in a
// fixed tree order (results do not depend on timing).
#include "common.hpp"
#include "bn_merge.hpp"
#include "../../include/dssp_kernels.h"

namespace {

using bnm::BnLayout;
using bnm::bn_layout;
using bnm::reduce_sub;
using bnm::bn_merge_stats;
constexpr int THREADS = bnm::THREADS;

// ------------------------------------------------------------------ elementwise
__global__ __launch_bounds__(THREADS) void relu_bwd_kernel(float* __restrict__ dy, const float* __restrict__ a, long n4, long n) {
    float4* d4 = reinterpret_cast<float4*>(dy);
    const float4* a4 = reinterpret_cast<const float4*>(a);
    for (long i = (long)blockIdx.x * THREADS + threadIdx.x; i < n4; i += (long)gridDim.x * THREADS) {
        float4 d = d4[i];
        const float4 v = a4[i];
        d.x = v.x > 0.f ? d.x : 0.f; d.y = v.y > 0.f ? d.y : 0.f;
        d.z = v.z > 0.f ? d.z : 0.f; d.w = v.w > 0.f ? d.w : 0.f;
        d4[i] = d;
    }
    if (blockIdx.x == 0) {
        const long t = n4 * 4 + threadIdx.x;
        if (t < n) dy[t] = a[t] > 0.f ? dy[t] : 0.f;
    }
}

__global__ __launch_bounds__(THREADS) void add_kernel(float* __restrict__ out, const float* __restrict__ in, long n4, long n) {
    float4* o4 = reinterpret_cast<float4*>(out);
    const float4* i4 = reinterpret_cast<const float4*>(in);
    for (long i = (long)blockIdx.x * THREADS + threadIdx.x; i < n4; i += (long)gridDim.x * THREADS) {
        float4 o = o4[i];
        const float4 v = i4[i];
        o.x += v.x; o.y += v.y; o.z += v.z; o.w += v.w;
        o4[i] = o;
    }
    if (blockIdx.x == 0) {
        const long t = n4 * 4 + threadIdx.x;
        if (t < n) out[t] += in[t];
    }
}

// ------------------------------------------------------------------ max pooling 3x3 / 2
__global__ __launch_bounds__(THREADS) void maxpool_fwd_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                              uint8_t* __restrict__ arg, int N, int H, int W, int C, int Ho, int Wo) {
    const long total = (long)N * Ho * Wo * C;
    for (long i = (long)blockIdx.x * THREADS + threadIdx.x; i < total; i += (long)gridDim.x * THREADS) {
        const int c = (int)(i % C);
        long r = i / C;
        const int wo = (int)(r % Wo); r /= Wo;
        const int ho = (int)(r % Ho);
        const int n = (int)(r / Ho);
        const float* base = x + (((long)n * H + 2 * ho) * W + 2 * wo) * C + c;
        float best = base[0];
        int bi = 0;
#pragma unroll
        for (int k = 1; k < 9; ++k) {
            const float v = base[((long)(k / 3) * W + (k % 3)) * C];
            if (v > best) { best = v; bi = k; }
        }
        y[i] = best;
        arg[i] = (uint8_t)bi;
    }
}

// Gather form: each input element sums the windows that chose it (no atomics, fixed order).
__global__ __launch_bounds__(THREADS) void maxpool_bwd_kernel(const float* __restrict__ dy, const uint8_t* __restrict__ arg,
                                                              float* __restrict__ dx, int N, int H, int W, int C, int Ho, int Wo) {
    const long total = (long)N * H * W * C;
    for (long i = (long)blockIdx.x * THREADS + threadIdx.x; i < total; i += (long)gridDim.x * THREADS) {
        const int c = (int)(i % C);
        long r = i / C;
        const int wi = (int)(r % W); r /= W;
        const int hi = (int)(r % H);
        const int n = (int)(r / H);
        float s = 0.f;
        const int ho_lo = hi >= 2 ? (hi - 1) / 2 : 0, ho_hi = min(Ho - 1, hi / 2);
        const int wo_lo = wi >= 2 ? (wi - 1) / 2 : 0, wo_hi = min(Wo - 1, wi / 2);
        for (int ho = ho_lo; ho <= ho_hi; ++ho)
            for (int wo = wo_lo; wo <= wo_hi; ++wo) {
                const long o = (((long)n * Ho + ho) * Wo + wo) * C + c;
                if (arg[o] == (hi - 2 * ho) * 3 + (wi - 2 * wo)) s += dy[o];
            }
        dx[i] = s;
    }
}

// The same two kernels for channel counts that are multiples of 4 and tensors below 2^31 elements (every shape the
// networks here have): a lane owns 4 channels of one pixel (16-byte loads and stores, the four choices in one 4-byte
// word) and all index arithmetic is 32-bit (a 64-bit division per element costs more than the memory traffic).
// MASK: the backward kernel also applies the ReLU that precedes the pooling, dx = a > 0 ? gathered gradient : 0
// (a = the pooling's input, a post-ReLU activation), which saves a pass over dx.
__global__ __launch_bounds__(THREADS) void maxpool_fwd4_kernel(const float4* __restrict__ x, float4* __restrict__ y,
                                                               uchar4* __restrict__ arg, int H, int W, int C4, int Ho, int Wo, unsigned total) {
    for (unsigned i = blockIdx.x * THREADS + threadIdx.x; i < total; i += gridDim.x * THREADS) {
        const unsigned c = i % (unsigned)C4;
        unsigned r = i / (unsigned)C4;
        const unsigned wo = r % (unsigned)Wo; r /= (unsigned)Wo;
        const unsigned ho = r % (unsigned)Ho;
        const unsigned n = r / (unsigned)Ho;
        const float4* base = x + ((size_t)(n * H + 2 * ho) * W + 2 * wo) * C4 + c;
        float4 v[9];
#pragma unroll
        for (int k = 0; k < 9; ++k) v[k] = base[(size_t)((k / 3) * W + (k % 3)) * C4];
        float4 best = v[0];
        uchar4 bi = make_uchar4(0, 0, 0, 0);
#pragma unroll
        for (int k = 1; k < 9; ++k) {        // first maximum in scan order, per channel
            if (v[k].x > best.x) { best.x = v[k].x; bi.x = (unsigned char)k; }
            if (v[k].y > best.y) { best.y = v[k].y; bi.y = (unsigned char)k; }
            if (v[k].z > best.z) { best.z = v[k].z; bi.z = (unsigned char)k; }
            if (v[k].w > best.w) { best.w = v[k].w; bi.w = (unsigned char)k; }
        }
        y[i] = best;
        arg[i] = bi;
    }
}

template <bool MASK>
__global__ __launch_bounds__(THREADS) void maxpool_bwd4_kernel(const float4* __restrict__ dy, const uchar4* __restrict__ arg,
                                                               const float4* __restrict__ a, float4* __restrict__ dx, int H, int W,
                                                               int C4, int Ho, int Wo, unsigned total) {
    for (unsigned i = blockIdx.x * THREADS + threadIdx.x; i < total; i += gridDim.x * THREADS) {
        const unsigned c = i % (unsigned)C4;
        unsigned r = i / (unsigned)C4;
        const int wi = (int)(r % (unsigned)W); r /= (unsigned)W;
        const int hi = (int)(r % (unsigned)H);
        const unsigned n = r / (unsigned)H;
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
        const int ho_lo = hi >= 2 ? (hi - 1) / 2 : 0, ho_hi = min(Ho - 1, hi / 2);
        const int wo_lo = wi >= 2 ? (wi - 1) / 2 : 0, wo_hi = min(Wo - 1, wi / 2);
        // A pixel lies in at most 2 x 2 windows (3x3, stride 2).  All four candidates are fetched at once (index clamped,
        // contribution dropped where the window does not exist) and added in the scalar kernel's window order, so the sums
        // are identical; one window after the other, each fetch would wait for the one before.
        uchar4 ch[4];
        float4 g[4];
        bool use[4];
        unsigned char want[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int ho = ho_lo + (k >> 1), wo = wo_lo + (k & 1);
            use[k] = ho <= ho_hi && wo <= wo_hi;
            const int hc = min(ho, Ho - 1), wc = min(wo, Wo - 1);
            const size_t o = ((size_t)(n * Ho + hc) * Wo + wc) * C4 + c;
            want[k] = (unsigned char)((hi - 2 * ho) * 3 + (wi - 2 * wo));
            ch[k] = arg[o];
            g[k] = dy[o];
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (use[k] && ch[k].x == want[k]) s.x += g[k].x;
            if (use[k] && ch[k].y == want[k]) s.y += g[k].y;
            if (use[k] && ch[k].z == want[k]) s.z += g[k].z;
            if (use[k] && ch[k].w == want[k]) s.w += g[k].w;
        }
        if constexpr (MASK) {
            const float4 av = a[i];
            s.x = av.x > 0.f ? s.x : 0.f; s.y = av.y > 0.f ? s.y : 0.f;
            s.z = av.z > 0.f ? s.z : 0.f; s.w = av.w > 0.f ? s.w : 0.f;
        }
        dx[i] = s;
    }
}

// ------------------------------------------------------------------ batch normalisation
// Two kernels per direction, no cross-workgroup synchronisation:
//   forward : (1) per slab of rows, mean and sum of squared deviations per channel;
//             (2) every workgroup of the apply kernel merges the slab results (at most 32 per lane) in
//                 its prologue - identical arithmetic in every workgroup - then normalises.
//   backward: (1) per slab, sum dz and sum dz*xhat (ReLU mask applied, dz written back);
//             (2) every workgroup of the dx kernel sums the slab results in its prologue.
// Reduce one float4 per thread across the row lanes of the workgroup (tree, fixed order).
// Result valid in row lane 0.
__device__ __forceinline__ float4 reduce_rows(float4 v, float4* red, int rl, int vc, int RL, int VC) {
    red[rl * VC + vc] = v;
    __syncthreads();
    for (int s = RL >> 1; s >= 1; s >>= 1) {
        if (rl < s) {
            float4 a = red[rl * VC + vc];
            const float4 b = red[(rl + s) * VC + vc];
            a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
            red[rl * VC + vc] = a;
        }
        __syncthreads();
    }
    const float4 out = red[vc];
    __syncthreads();
    return out;
}

// Per slab of rows: mean and sum of squared deviations per channel.  Sums are taken about a
// pivot (the slab's first row) so that no large-minus-large cancellation occurs.
// partial[(g*C + c)*2 + {0,1}] = {mean_g, M2_g}
__global__ __launch_bounds__(THREADS) void bn_stats_partial_kernel(const float* __restrict__ x, float* __restrict__ partial, long M, int C, BnLayout L) {
    __shared__ float4 red[THREADS];
    const int rl = threadIdx.x / L.VC, vc = threadIdx.x % L.VC;
    const long r0 = (long)blockIdx.x * L.rows_per_block;
    const long r1 = min(M, r0 + L.rows_per_block);
    const float4 pivot = *reinterpret_cast<const float4*>(x + r0 * C + 4 * vc);
    float4 s1 = make_float4(0.f, 0.f, 0.f, 0.f), s2 = s1;
    for (long r = r0 + rl; r < r1; r += 4 * L.RL) {
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)            // four independent loads in flight; rows past the slab read as the pivot (adds 0)
            v[u] = (r + u * L.RL < r1) ? *reinterpret_cast<const float4*>(x + (r + u * L.RL) * C + 4 * vc) : pivot;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float dx_ = v[u].x - pivot.x, dy_ = v[u].y - pivot.y, dz_ = v[u].z - pivot.z, dw_ = v[u].w - pivot.w;
            s1.x += dx_; s1.y += dy_; s1.z += dz_; s1.w += dw_;
            s2.x = fmaf(dx_, dx_, s2.x); s2.y = fmaf(dy_, dy_, s2.y); s2.z = fmaf(dz_, dz_, s2.z); s2.w = fmaf(dw_, dw_, s2.w);
        }
    }
    s1 = reduce_rows(s1, red, rl, vc, L.RL, L.VC);
    s2 = reduce_rows(s2, red, rl, vc, L.RL, L.VC);
    if (rl == 0) {
        const float n = (float)(r1 - r0);
        float* out = partial + ((long)blockIdx.x * C + 4 * vc) * 2;
        out[0] = pivot.x + s1.x / n; out[1] = s2.x - s1.x * s1.x / n;
        out[2] = pivot.y + s1.y / n; out[3] = s2.y - s1.y * s1.y / n;
        out[4] = pivot.z + s1.z / n; out[5] = s2.z - s1.z * s1.z / n;
        out[6] = pivot.w + s1.w / n; out[7] = s2.w - s1.w * s1.w / n;
    }
}

// y = gamma * (x - mean) * invstd + beta (+ shortcut) (ReLU); workgroup 0 also stores mean / invstd
// to stats[] for the backward pass.
template <int SC_MODE>
__global__ __launch_bounds__(THREADS) void bn_apply_kernel(const float* __restrict__ x, const float* __restrict__ gamma,
                                                           const float* __restrict__ beta, const float* __restrict__ partial,
                                                           float* __restrict__ stats, float* __restrict__ y, long M, int C,
                                                           float eps, int relu, const float* __restrict__ sc, int sc_ho, int sc_wo,
                                                           BnLayout L) {
    __shared__ float red[THREADS];
    __shared__ __attribute__((aligned(16))) float sh[2 * THREADS];
    bn_merge_stats(partial, M, C, eps, red, sh, L);
    if (blockIdx.x == 0 && threadIdx.x < 2 * C) stats[threadIdx.x] = sh[threadIdx.x];
    const int VC = C / 4, vshift = __ffs(VC) - 1;
    const long total = M * VC;
    const long stride = (long)gridDim.x * THREADS;
    // four independent rows per lane and trip: all loads are issued before the first use
    for (long i0 = (long)blockIdx.x * THREADS + threadIdx.x; i0 < total; i0 += 4 * stride) {
        float4 v[4], s4[4];
        bool ok[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const long i = i0 + u * stride;
            ok[u] = i < total;
            const int vc = (int)(i & (VC - 1));     // VC is a power of two (C is 4 .. 64 and divides the workgroup size)
            const long row = i >> vshift;
            v[u] = ok[u] ? *reinterpret_cast<const float4*>(x + row * C + 4 * vc) : make_float4(0.f, 0.f, 0.f, 0.f);
            s4[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if constexpr (SC_MODE == 1) {
                if (ok[u]) s4[u] = *reinterpret_cast<const float4*>(sc + row * C + 4 * vc);
            } else if constexpr (SC_MODE == 2) {
                if (ok[u] && 4 * vc < C / 2) {   // first half of the channels: input pixel (2ho, 2wo), C/2 channels wide
                    const unsigned ru = (unsigned)row, rq = ru / (unsigned)sc_wo;       // M < 2^31: 32-bit divisions
                    const int wo = (int)(ru - rq * (unsigned)sc_wo);
                    const long n = rq / (unsigned)sc_ho;
                    const int ho = (int)(rq - (unsigned)n * (unsigned)sc_ho);
                    s4[u] = *reinterpret_cast<const float4*>(sc + ((n * (2 * sc_ho) + 2 * ho) * (2 * sc_wo) + 2 * wo) * (C / 2) + 4 * vc);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (!ok[u]) continue;
            const long i = i0 + u * stride;
            const int vc = (int)(i & (VC - 1));     // VC is a power of two (C is 4 .. 64 and divides the workgroup size)
            const long row = i >> vshift;
            const float4 mu = *reinterpret_cast<const float4*>(sh + 4 * vc);
            const float4 is = *reinterpret_cast<const float4*>(sh + C + 4 * vc);
            const float4 ga = *reinterpret_cast<const float4*>(gamma + 4 * vc);
            const float4 be = *reinterpret_cast<const float4*>(beta + 4 * vc);
            float4 o;
            o.x = fmaf((v[u].x - mu.x) * is.x, ga.x, be.x) + s4[u].x;
            o.y = fmaf((v[u].y - mu.y) * is.y, ga.y, be.y) + s4[u].y;
            o.z = fmaf((v[u].z - mu.z) * is.z, ga.z, be.z) + s4[u].z;
            o.w = fmaf((v[u].w - mu.w) * is.w, ga.w, be.w) + s4[u].w;
            if (relu) { o.x = fmaxf(o.x, 0.f); o.y = fmaxf(o.y, 0.f); o.z = fmaxf(o.z, 0.f); o.w = fmaxf(o.w, 0.f); }
            *reinterpret_cast<float4*>(y + row * C + 4 * vc) = o;
        }
    }
}

// Per slab: sum dz and sum dz * xhat per channel, dz = da * [out > 0] (written back in place).
// partial[(g*C + c)*2 + {0,1}]
__global__ __launch_bounds__(THREADS) void bn_bwd_partial_kernel(const float* __restrict__ x, const float* __restrict__ stats,
                                                                 float* __restrict__ da, const float* __restrict__ out,
                                                                 float* __restrict__ partial, long M, int C, BnLayout L) {
    __shared__ float4 red[THREADS];
    const int rl = threadIdx.x / L.VC, vc = threadIdx.x % L.VC;
    const long r0 = (long)blockIdx.x * L.rows_per_block;
    const long r1 = min(M, r0 + L.rows_per_block);
    const float4 mu = *reinterpret_cast<const float4*>(stats + 4 * vc);
    const float4 is = *reinterpret_cast<const float4*>(stats + C + 4 * vc);
    float4 sb = make_float4(0.f, 0.f, 0.f, 0.f), sg = sb;
    for (long r0u = r0 + rl; r0u < r1; r0u += 4 * L.RL) {
        float4 d[4], v[4], o[4];
        bool ok[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {           // four rows in flight per lane
            const long r = r0u + u * L.RL;
            ok[u] = r < r1;
            d[u] = ok[u] ? *reinterpret_cast<const float4*>(da + r * C + 4 * vc) : make_float4(0.f, 0.f, 0.f, 0.f);
            v[u] = ok[u] ? *reinterpret_cast<const float4*>(x + r * C + 4 * vc) : mu;
            o[u] = (ok[u] && out) ? *reinterpret_cast<const float4*>(out + r * C + 4 * vc) : make_float4(1.f, 1.f, 1.f, 1.f);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const long r = r0u + u * L.RL;
            if (out) {
                d[u].x = o[u].x > 0.f ? d[u].x : 0.f; d[u].y = o[u].y > 0.f ? d[u].y : 0.f;
                d[u].z = o[u].z > 0.f ? d[u].z : 0.f; d[u].w = o[u].w > 0.f ? d[u].w : 0.f;
                if (ok[u]) *reinterpret_cast<float4*>(da + r * C + 4 * vc) = d[u];
            }
            sb.x += d[u].x; sb.y += d[u].y; sb.z += d[u].z; sb.w += d[u].w;
            sg.x = fmaf(d[u].x, (v[u].x - mu.x) * is.x, sg.x);
            sg.y = fmaf(d[u].y, (v[u].y - mu.y) * is.y, sg.y);
            sg.z = fmaf(d[u].z, (v[u].z - mu.z) * is.z, sg.z);
            sg.w = fmaf(d[u].w, (v[u].w - mu.w) * is.w, sg.w);
        }
    }
    sb = reduce_rows(sb, red, rl, vc, L.RL, L.VC);
    sg = reduce_rows(sg, red, rl, vc, L.RL, L.VC);
    if (rl == 0) {
        float* o = partial + ((long)blockIdx.x * C + 4 * vc) * 2;
        o[0] = sb.x; o[1] = sg.x; o[2] = sb.y; o[3] = sg.y; o[4] = sb.z; o[5] = sg.z; o[6] = sb.w; o[7] = sg.w;
    }
}

// dx = gamma * invstd * (dz - dbeta / M - xhat * dgamma / M); dbeta = sum dz and dgamma = sum dz*xhat are
// summed from the slab results by every workgroup (same order everywhere); workgroup 0 stores them.
__global__ __launch_bounds__(THREADS) void bn_bwd_dx_kernel(const float* __restrict__ x, const float* __restrict__ gamma,
                                                            const float* __restrict__ stats, const float* __restrict__ dz,
                                                            const float* __restrict__ partial, float* __restrict__ dgamma,
                                                            float* __restrict__ dbeta, float* __restrict__ dx, long M, int C,
                                                            BnLayout L) {
    __shared__ float red[THREADS];
    __shared__ __attribute__((aligned(16))) float sh[2 * THREADS];      // [0,C): dbeta, [C,2C): dgamma
    {
        const int SUB = THREADS / C;
        const int c = threadIdx.x % C, sub = threadIdx.x / C;
        float2 pv[32];
#pragma unroll
        for (int u = 0; u < 32; ++u)            // one batch of unconditional loads (G <= 32 * SUB; index clamped)
            pv[u] = *reinterpret_cast<const float2*>(partial + ((long)min(sub + u * SUB, L.G - 1) * C + c) * 2);
        float sb = 0.f, sg = 0.f;
#pragma unroll
        for (int u = 0; u < 32; ++u) {
            const bool in = sub + u * SUB < L.G;
            sb += in ? pv[u].x : 0.f;
            sg += in ? pv[u].y : 0.f;
        }
        sb = reduce_sub(sb, red, c, sub, SUB, C);
        sg = reduce_sub(sg, red, c, sub, SUB, C);
        if (sub == 0) {
            sh[c] = sb; sh[C + c] = sg;
            if (blockIdx.x == 0) { dbeta[c] = sb; dgamma[c] = sg; }
        }
        __syncthreads();
    }
    const int VC = C / 4, vshift = __ffs(VC) - 1;
    const long total = M * VC;
    const float inv_m = 1.0f / (float)M;
    const long stride = (long)gridDim.x * THREADS;
    for (long i0 = (long)blockIdx.x * THREADS + threadIdx.x; i0 < total; i0 += 4 * stride) {
        float4 v[4], d[4];
        bool ok[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {            // all loads of the trip first
            const long i = i0 + u * stride;
            ok[u] = i < total;
            const int vc = (int)(i & (VC - 1));     // VC is a power of two (C is 4 .. 64 and divides the workgroup size)
            const long row = i >> vshift;
            v[u] = ok[u] ? *reinterpret_cast<const float4*>(x + row * C + 4 * vc) : make_float4(0.f, 0.f, 0.f, 0.f);
            d[u] = ok[u] ? *reinterpret_cast<const float4*>(dz + row * C + 4 * vc) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (!ok[u]) continue;
            const long i = i0 + u * stride;
            const int vc = (int)(i & (VC - 1));     // VC is a power of two (C is 4 .. 64 and divides the workgroup size)
            const long row = i >> vshift;
            const float4 mu = *reinterpret_cast<const float4*>(stats + 4 * vc);
            const float4 is = *reinterpret_cast<const float4*>(stats + C + 4 * vc);
            const float4 ga = *reinterpret_cast<const float4*>(gamma + 4 * vc);
            const float4 db = *reinterpret_cast<const float4*>(sh + 4 * vc);
            const float4 dg = *reinterpret_cast<const float4*>(sh + C + 4 * vc);
            float4 o;
            o.x = ga.x * is.x * (d[u].x - db.x * inv_m - (v[u].x - mu.x) * is.x * (dg.x * inv_m));
            o.y = ga.y * is.y * (d[u].y - db.y * inv_m - (v[u].y - mu.y) * is.y * (dg.y * inv_m));
            o.z = ga.z * is.z * (d[u].z - db.z * inv_m - (v[u].z - mu.z) * is.z * (dg.z * inv_m));
            o.w = ga.w * is.w * (d[u].w - db.w * inv_m - (v[u].w - mu.w) * is.w * (dg.w * inv_m));
            *reinterpret_cast<float4*>(dx + row * C + 4 * vc) = o;
        }
    }
}

// dx[n][2ho][2wo][c] += dy[n][ho][wo][c], c < C/2
__global__ __launch_bounds__(THREADS) void shortcut_bwd_acc_kernel(const float* __restrict__ dy, float* __restrict__ dx,
                                                                   int N, int Ho, int Wo, int C) {
    const int Ch = C / 2, VC = Ch / 4;
    const long total = (long)N * Ho * Wo * VC;
    for (long i = (long)blockIdx.x * THREADS + threadIdx.x; i < total; i += (long)gridDim.x * THREADS) {
        const int vc = (int)(i % VC);
        long r = i / VC;
        const int wo = (int)(r % Wo); r /= Wo;
        const int ho = (int)(r % Ho);
        const long n = r / Ho;
        const float4 d = *reinterpret_cast<const float4*>(dy + (((n * Ho + ho) * Wo + wo) * C) + 4 * vc);
        float4* p = reinterpret_cast<float4*>(dx + ((n * (2 * Ho) + 2 * ho) * (2 * Wo) + 2 * wo) * Ch + 4 * vc);
        float4 o = *p;
        o.x += d.x; o.y += d.y; o.z += d.z; o.w += d.w;
        *p = o;
    }
}

// ------------------------------------------------------------------ global average pooling
__global__ __launch_bounds__(THREADS) void gap_fwd_kernel(const float* __restrict__ x, float* __restrict__ y, int N, int HW, int C) {
    const int i = blockIdx.x * THREADS + threadIdx.x;
    if (i >= N * C) return;
    const int n = i / C, c = i % C;
    float s = 0.f;
    int k = 0;
    for (; k + 8 <= HW; k += 8) {            // eight loads in flight, added in pixel order
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = x[((long)n * HW + k + u) * C + c];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; k < HW; ++k) s += x[((long)n * HW + k) * C + c];
    y[i] = s / (float)HW;
}

__global__ __launch_bounds__(THREADS) void gap_bwd_kernel(const float* __restrict__ dy, float* __restrict__ dx, int N, int HW, int C) {
    const long total = (long)N * HW * C;
    const float inv = 1.0f / (float)HW;
    for (long i = (long)blockIdx.x * THREADS + threadIdx.x; i < total; i += (long)gridDim.x * THREADS) {
        const int c = (int)(i % C);
        const long n = i / ((long)HW * C);
        dx[i] = dy[n * C + c] * inv;
    }
}

// ------------------------------------------------------------------ softmax cross-entropy
// One wavefront per sample at a time (lanes stride over the classes, so rows are read coalesced); maxima and sums
// are combined across the lanes by a fixed butterfly; the batch mean of the loss is summed by thread 0 in index order.
__global__ void softmax_xent_kernel(const float* __restrict__ z, const int32_t* __restrict__ label,
                                    float* __restrict__ dz, float* __restrict__ loss, int m, int C) {
    extern __shared__ float row_loss[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const float invm = 1.0f / (float)m;
    for (int i = wave; i < m; i += nwaves) {
        const float* zi = z + (long)i * C;
        float mx = -INFINITY;
        for (int j = lane; j < C; j += 64) mx = fmaxf(mx, zi[j]);
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
        float se = 0.f;
        for (int j = lane; j < C; j += 64) se += expf(zi[j] - mx);
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) se += __shfl_xor(se, o);
        const int y = label[i];
        if (lane == 0) row_loss[i] = logf(se) + mx - zi[y];
        const float inv = 1.0f / se;
        for (int j = lane; j < C; j += 64) dz[(long)i * C + j] = (expf(zi[j] - mx) * inv - (j == y ? 1.f : 0.f)) * invm;
    }
    __syncthreads();
    if (threadIdx.x == 0 && loss) {
        float s = 0.f;
        for (int k = 0; k < m; ++k) s += row_loss[k];
        *loss = s * invm;
    }
}

inline int grid_for(long items) { return stream_grid(ceil_div(items, THREADS)); }
inline bool al16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
inline bool bn_ok(long M, int C) { return M >= 1 && M < (1L << 31) && C >= 4 && C % 4 == 0 && C <= 64 && THREADS % C == 0; }

}  // namespace

extern "C" int dsspk_relu_bwd(void* stream, float* dy, const float* a, long n) {
    if (!dy || !a || n < 0 || !al16(dy) || !al16(a)) return -1;
    hipLaunchKernelGGL(relu_bwd_kernel, dim3(grid_for(n / 4)), dim3(THREADS), 0, (hipStream_t)stream, dy, a, n / 4, n);
    return DSSPK_LAUNCH_RC();
}

extern "C" int dsspk_add(void* stream, float* out, const float* in, long n) {
    if (!out || !in || n < 0 || !al16(out) || !al16(in)) return -1;
    hipLaunchKernelGGL(add_kernel, dim3(grid_for(n / 4)), dim3(THREADS), 0, (hipStream_t)stream, out, in, n / 4, n);
    return DSSPK_LAUNCH_RC();
}

extern "C" int dsspk_maxpool_fwd(void* stream, const float* x, float* y, uint8_t* arg, int N, int H, int W, int C) {
    if (!x || !y || !arg || N < 1 || H < 3 || W < 3 || C < 1) return -1;
    const int Ho = (H - 3) / 2 + 1, Wo = (W - 3) / 2 + 1;
    if (C % 4 == 0 && (long)N * H * W * C < (1L << 31) && al16(x) && al16(y) && (reinterpret_cast<uintptr_t>(arg) & 3) == 0) {
        const long total = (long)N * Ho * Wo * (C / 4);
        hipLaunchKernelGGL(maxpool_fwd4_kernel, dim3(grid_for(total)), dim3(THREADS), 0, (hipStream_t)stream,
                           reinterpret_cast<const float4*>(x), reinterpret_cast<float4*>(y), reinterpret_cast<uchar4*>(arg), H, W, C / 4,
                           Ho, Wo, (unsigned)total);
        return DSSPK_LAUNCH_RC();
    }
    hipLaunchKernelGGL(maxpool_fwd_kernel, dim3(grid_for((long)N * Ho * Wo * C)), dim3(THREADS), 0, (hipStream_t)stream,
                       x, y, arg, N, H, W, C, Ho, Wo);
    return DSSPK_LAUNCH_RC();
}

extern "C" int dsspk_maxpool_bwd_relu(void* stream, const float* dy, const uint8_t* arg, const float* a, float* dx, int N, int H,
                                      int W, int C) {
    if (!dy || !dx || !arg || N < 1 || H < 3 || W < 3 || C < 1) return -1;
    const int Ho = (H - 3) / 2 + 1, Wo = (W - 3) / 2 + 1;
    hipStream_t s = (hipStream_t)stream;
    if (C % 4 == 0 && (long)N * H * W * C < (1L << 31) && al16(dy) && al16(dx) && (!a || al16(a)) && (reinterpret_cast<uintptr_t>(arg) & 3) == 0) {
        const long total = (long)N * H * W * (C / 4);
        const float4* a4 = reinterpret_cast<const float4*>(a);
        if (a)
            hipLaunchKernelGGL((maxpool_bwd4_kernel<true>), dim3(grid_for(total)), dim3(THREADS), 0, s, reinterpret_cast<const float4*>(dy),
                               reinterpret_cast<const uchar4*>(arg), a4, reinterpret_cast<float4*>(dx), H, W, C / 4, Ho, Wo, (unsigned)total);
        else
            hipLaunchKernelGGL((maxpool_bwd4_kernel<false>), dim3(grid_for(total)), dim3(THREADS), 0, s, reinterpret_cast<const float4*>(dy),
                               reinterpret_cast<const uchar4*>(arg), a4, reinterpret_cast<float4*>(dx), H, W, C / 4, Ho, Wo, (unsigned)total);
        return DSSPK_LAUNCH_RC();
    }
    hipLaunchKernelGGL(maxpool_bwd_kernel, dim3(grid_for((long)N * H * W * C)), dim3(THREADS), 0, s, dy, arg, dx, N, H, W, C, Ho, Wo);
    if (int rc = DSSPK_LAUNCH_RC()) return rc;
    return a ? dsspk_relu_bwd(stream, dx, a, (long)N * H * W * C) : 0;
}

extern "C" int dsspk_maxpool_bwd(void* stream, const float* dy, const uint8_t* arg, float* dx, int N, int H, int W, int C) {
    return dsspk_maxpool_bwd_relu(stream, dy, arg, nullptr, dx, N, H, W, C);
}

extern "C" size_t dsspk_bn_scratch_floats(long M, int C) {
    if (!bn_ok(M, C)) return 0;
    return (size_t)32 * THREADS * 2;          // room for the largest number of records a merge accepts: 32 per lane
}

// Workgroups of the elementwise BN kernels: each one repeats the merge of the slab results, so keep
// their number moderate and let them stride over the rows.
inline int bn_elem_grid(long M, int C) { return stream_grid(ceil_div(M * (C / 4), THREADS * 4L), 1024); }

extern "C" int dsspk_bn_fwd(void* stream, const float* x, const float* gamma, const float* beta, float* y,
                            float* stats, float* scratch, long M, int C, float eps, int relu,
                            int shortcut_mode, const float* sc, int sc_n, int sc_ho, int sc_wo, int conv_parts) {
    if (!x || !gamma || !beta || !y || !stats || !scratch || !bn_ok(M, C)) return -1;
    if (!al16(x) || !al16(y) || !al16(gamma) || !al16(beta) || !al16(stats)) return -1;
    if (shortcut_mode < 0 || shortcut_mode > 2 || (shortcut_mode && (!sc || !al16(sc)))) return -1;
    if (shortcut_mode == 2 && ((long)sc_n * sc_ho * sc_wo != M || C % 8)) return -1;
    hipStream_t s = (hipStream_t)stream;
    BnLayout L = bn_layout(M, C);
    if (conv_parts > 0) {           // scratch already holds conv_parts records of M / conv_parts rows each
        if (M % conv_parts || conv_parts > 32 * (THREADS / C)) return -1;
        L.G = conv_parts;
        L.rows_per_block = M / conv_parts;
    } else {
        hipLaunchKernelGGL(bn_stats_partial_kernel, dim3(L.G), dim3(THREADS), 0, s, x, scratch, M, C, L);
    }
    const int grid = bn_elem_grid(M, C);
    if (shortcut_mode == 0)
        hipLaunchKernelGGL((bn_apply_kernel<0>), dim3(grid), dim3(THREADS), 0, s, x, gamma, beta, scratch, stats, y, M, C, eps, relu, sc, sc_ho, sc_wo, L);
    else if (shortcut_mode == 1)
        hipLaunchKernelGGL((bn_apply_kernel<1>), dim3(grid), dim3(THREADS), 0, s, x, gamma, beta, scratch, stats, y, M, C, eps, relu, sc, sc_ho, sc_wo, L);
    else
        hipLaunchKernelGGL((bn_apply_kernel<2>), dim3(grid), dim3(THREADS), 0, s, x, gamma, beta, scratch, stats, y, M, C, eps, relu, sc, sc_ho, sc_wo, L);
    return DSSPK_LAUNCH_RC();
}

static bool bn_bwd_args_ok(const float* x, const float* gamma, const float* stats, const float* da, const float* out,
                           const float* dx, const float* dgamma, const float* dbeta, const float* scratch, long M, int C) {
    if (!x || !gamma || !stats || !da || !dx || !dgamma || !dbeta || !scratch || !bn_ok(M, C)) return false;
    if (!al16(x) || !al16(da) || !al16(dx) || !al16(gamma) || !al16(stats)) return false;
    return !out || al16(out);
}

extern "C" int dsspk_bn_bwd_reduce(void* stream, const float* x, const float* stats, float* da, const float* out,
                                   float* scratch, long M, int C) {
    if (!bn_bwd_args_ok(x, x, stats, da, out, da, x, x, scratch, M, C)) return -1;
    const BnLayout L = bn_layout(M, C);
    hipLaunchKernelGGL(bn_bwd_partial_kernel, dim3(L.G), dim3(THREADS), 0, (hipStream_t)stream, x, stats, da, out, scratch, M, C, L);
    return DSSPK_LAUNCH_RC();
}

extern "C" int dsspk_bn_bwd_dx(void* stream, const float* x, const float* gamma, const float* stats, const float* dz,
                               float* dx, float* dgamma, float* dbeta, const float* scratch, long M, int C, int conv_parts) {
    if (!bn_bwd_args_ok(x, gamma, stats, dz, nullptr, dx, dgamma, dbeta, scratch, M, C)) return -1;
    BnLayout Lr = bn_layout(M, C);
    if (conv_parts > 0) {           // records written by a convolution epilogue, one per tile
        if (M % conv_parts || conv_parts > 32 * (THREADS / C)) return -1;
        Lr.G = conv_parts;
        Lr.rows_per_block = M / conv_parts;
    }
    hipLaunchKernelGGL(bn_bwd_dx_kernel, dim3(bn_elem_grid(M, C)), dim3(THREADS), 0, (hipStream_t)stream,
                       x, gamma, stats, dz, scratch, dgamma, dbeta, dx, M, C, Lr);
    return DSSPK_LAUNCH_RC();
}

extern "C" int dsspk_bn_bwd(void* stream, const float* x, const float* gamma, const float* stats, float* da,
                            const float* out, float* dx, float* dgamma, float* dbeta, float* scratch, long M, int C) {
    if (!bn_bwd_args_ok(x, gamma, stats, da, out, dx, dgamma, dbeta, scratch, M, C)) return -1;
    if (int rc = dsspk_bn_bwd_reduce(stream, x, stats, da, out, scratch, M, C)) return rc;
    return dsspk_bn_bwd_dx(stream, x, gamma, stats, da, dx, dgamma, dbeta, scratch, M, C, 0);
}

extern "C" int dsspk_shortcut_bwd_acc(void* stream, const float* dy, float* dx, int N, int Ho, int Wo, int C) {
    if (!dy || !dx || N < 1 || Ho < 1 || Wo < 1 || C < 8 || C % 8 || !al16(dy) || !al16(dx)) return -1;
    hipLaunchKernelGGL(shortcut_bwd_acc_kernel, dim3(grid_for((long)N * Ho * Wo * (C / 8))), dim3(THREADS), 0,
                       (hipStream_t)stream, dy, dx, N, Ho, Wo, C);
    return DSSPK_LAUNCH_RC();
}

extern "C" int dsspk_gap_fwd(void* stream, const float* x, float* y, int N, int HW, int C) {
    if (!x || !y || N < 1 || HW < 1 || C < 1) return -1;
    hipLaunchKernelGGL(gap_fwd_kernel, dim3(ceil_div((long)N * C, THREADS)), dim3(THREADS), 0, (hipStream_t)stream, x, y, N, HW, C);
    return DSSPK_LAUNCH_RC();
}

extern "C" int dsspk_gap_bwd(void* stream, const float* dy, float* dx, int N, int HW, int C) {
    if (!dy || !dx || N < 1 || HW < 1 || C < 1) return -1;
    hipLaunchKernelGGL(gap_bwd_kernel, dim3(grid_for((long)N * HW * C)), dim3(THREADS), 0, (hipStream_t)stream, dy, dx, N, HW, C);
    return DSSPK_LAUNCH_RC();
}

extern "C" int dsspk_softmax_xent(void* stream, const float* z, const int32_t* y, float* dz, float* loss, int m, int C) {
    if (!z || !y || !dz || m < 1 || m > 1024 || C < 1 || C > 1024) return -1;
    const int threads = m >= 16 ? 1024 : 64 * m;          // one wavefront per sample, at most 16 at a time
    hipLaunchKernelGGL(softmax_xent_kernel, dim3(1), dim3(threads), sizeof(float) * m, (hipStream_t)stream, z, y, dz, loss, m, C);
    return DSSPK_LAUNCH_RC();
}
