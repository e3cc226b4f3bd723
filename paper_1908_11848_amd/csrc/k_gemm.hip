// Fully connected layers: C = op(A) * op(B) (+ bias) (ReLU), fp32 on the matrix cores.
// One workgroup (4 wavefronts) owns a 64 x 64 tile of C; wavefront w owns the 32 x 32
// quadrant (w / 2, w % 2).  Operands come in through generic strides, so the same kernel
// serves y = x W (+b), dx = dy W^T and dW = x^T dy of Alg. 1's worker gradient.
#include <mutex>

#include "mma.hpp"
#include "../../include/dssp_kernels.h"

namespace {

constexpr int BM = 64, BN = 64, THREADS = 256;

// A_FAST_K: op(A) is k-contiguous in memory (a_cs == 1); otherwise row-contiguous (a_rs == 1).
// B_FAST_N: op(B) is column-contiguous (b_cs == 1); otherwise k-contiguous (b_rs == 1).
// The flags only select which index runs across neighbouring lanes so that loads coalesce.
template <bool A_FAST_K, bool B_FAST_N>
__global__ __launch_bounds__(THREADS) void gemm_kernel(const float* __restrict__ A, long a_rs, long a_cs,
                                                       const float* __restrict__ B, long b_rs, long b_cs,
                                                       float* __restrict__ C, long ldc, int M, int N, int K,
                                                       const float* __restrict__ bias, int relu, int k_per_layer) {
    __shared__ __attribute__((aligned(16))) float As[2][BM * mma::LDK];
    __shared__ __attribute__((aligned(16))) float Bs[2][BN * mma::LDK];      // stored [col][k]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    // split-K: layer z of the grid takes the reduction indices [z * k_per_layer, (z + 1) * k_per_layer) and writes its
    // partial product to the z-th [M][N] slab of C (the caller passes scratch, no bias, no ReLU)
    const int k_lo = blockIdx.z * k_per_layer;
    K = min(K, k_lo + k_per_layer);
    C += (long)blockIdx.z * M * N;
    floatx4 acc[2][2];
    mma::zero(acc);
    float ra[4], rb[4];
    auto load = [&](int k0) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int idx = tid + e * THREADS;                     // 0 .. 1023
            const int i = A_FAST_K ? idx / 16 : idx % 64, k = A_FAST_K ? idx % 16 : idx / 64;
            ra[e] = (m0 + i < M && k0 + k < K) ? A[(long)(m0 + i) * a_rs + (long)(k0 + k) * a_cs] : 0.f;
            const int j = B_FAST_N ? idx % 64 : idx / 16, kb = B_FAST_N ? idx / 64 : idx % 16;
            rb[e] = (n0 + j < N && k0 + kb < K) ? B[(long)(k0 + kb) * b_rs + (long)(n0 + j) * b_cs] : 0.f;
        }
    };
    auto store = [&](int buf) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int idx = tid + e * THREADS;
            const int i = A_FAST_K ? idx / 16 : idx % 64, k = A_FAST_K ? idx % 16 : idx / 64;
            As[buf][i * mma::LDK + k] = ra[e];
            const int j = B_FAST_N ? idx % 64 : idx / 16, kb = B_FAST_N ? idx / 64 : idx % 16;
            Bs[buf][j * mma::LDK + kb] = rb[e];
        }
    };
    const int nk = (K - k_lo + mma::KC - 1) / mma::KC;
    load(k_lo);
    for (int kc = 0; kc < nk; ++kc) {
        const int buf = kc & 1;
        store(buf);
        __syncthreads();
        if (kc + 1 < nk) load(k_lo + (kc + 1) * mma::KC);
        mma::chunk16<2, 2, false, true>(As[buf], mma::LDK, Bs[buf], mma::LDK, 32 * (wave >> 1), 32 * (wave & 1), acc, lane);
    }
    mma::drain();
    const int l16 = lane & 15, q = lane >> 4;
#pragma unroll
    for (int wm = 0; wm < 2; ++wm)
#pragma unroll
        for (int wn = 0; wn < 2; ++wn) {
            const int col = n0 + 32 * (wave & 1) + 16 * wn + l16;
            if (col >= N) continue;
            const float bv = bias ? bias[col] : 0.f;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = m0 + 32 * (wave >> 1) + 16 * wm + 4 * q + v;
                if (row >= M) continue;
                float x = acc[wm][wn][v] + bv;
                if (relu) x = fmaxf(x, 0.f);
                C[(long)row * ldc + col] = x;
            }
        }
}

// out[slab][j] = sum over the rows i of the slab of X[i][j]: a workgroup owns 64 columns and one slab of rows
// (blockIdx.y), four row lanes each adding every fourth row of the slab in ascending order, eight loads in flight.
// Tall matrices take two passes (slab sums into scratch, then the sum of the slabs), short ones a single slab.
__global__ __launch_bounds__(256) void colsum_kernel(const float* __restrict__ X, float* __restrict__ out, long M, int N,
                                                     long rows_per_slab) {
    __shared__ float part[4][64];
    const int c = threadIdx.x & 63, g = threadIdx.x >> 6;
    const int col = blockIdx.x * 64 + c;
    const long r0 = (long)blockIdx.y * rows_per_slab;
    const long r1 = r0 + rows_per_slab < M ? r0 + rows_per_slab : M;
    float s = 0.f;
    if (col < N) {
        long i = r0 + g;
        for (; i + 28 < r1; i += 32) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = X[(i + 4 * u) * N + col];
#pragma unroll
            for (int u = 0; u < 8; ++u) s += v[u];
        }
        for (; i < r1; i += 4) s += X[i * N + col];
    }
    part[g][c] = s;
    __syncthreads();
    if (g == 0 && col < N) out[(long)blockIdx.y * N + col] = (part[0][c] + part[1][c]) + (part[2][c] + part[3][c]);
}

constexpr int COLSUM_SLABS = 256;

// C[i][j] = sum over the layers, in order, of partial[layer][i][j] (+ bias[j]) (ReLU)
__global__ __launch_bounds__(256) void splitk_sum_kernel(const float* __restrict__ partial, float* __restrict__ C, long ldc, int M,
                                                         int N, int layers, const float* __restrict__ bias, int relu) {
    const long e = (long)blockIdx.x * 256 + threadIdx.x;
    if (e >= (long)M * N) return;
    float s = 0.f;
    for (int l = 0; l < layers; ++l) s += partial[(long)l * M * N + e];
    const int col = (int)(e % N);
    if (bias) s += bias[col];
    if (relu) s = fmaxf(s, 0.f);
    C[(e / N) * ldc + col] = s;
}

int launch_gemm(hipStream_t s, const float* A, long a_rs, long a_cs, const float* B, long b_rs, long b_cs, float* C, long ldc,
                int M, int N, int K, const float* bias, int relu, int layers) {
    const int chunks = ceil_div(K, mma::KC);
    const int k_per_layer = ceil_div(chunks, layers) * mma::KC;
    dim3 grid(ceil_div(N, BN), ceil_div(M, BM), ceil_div(K, k_per_layer));
    const bool ak = a_cs == 1, bn = b_cs == 1;
#define GO(AK, BNF) hipLaunchKernelGGL((gemm_kernel<AK, BNF>), grid, dim3(THREADS), 0, s, A, a_rs, a_cs, B, b_rs, b_cs, C, ldc, M, N, K, bias, relu, k_per_layer)
    if (ak && bn) GO(true, true);
    else if (ak) GO(true, false);
    else if (bn) GO(false, true);
    else GO(false, false);
#undef GO
    return (int)grid.z;
}

}  // namespace

extern "C" int dsspk_gemm(void* stream, const float* A, long a_rs, long a_cs, const float* B, long b_rs, long b_cs,
                          float* C, long ldc, int M, int N, int K, const float* bias, int relu) {
    if (!A || !B || !C || M < 1 || N < 1 || K < 1) return -1;
    launch_gemm((hipStream_t)stream, A, a_rs, a_cs, B, b_rs, b_cs, C, ldc, M, N, K, bias, relu, 1);
    return DSSPK_LAUNCH_RC();
}

// Layers worth splitting K into (K of 1024 and more, fewer than 128 output tiles): enough workgroups to cover the
// chip, at least 8 k-chunks of work per layer.
extern "C" int dsspk_gemm_splitk_layers(int M, int N, int K) {
    if (M < 1 || N < 1 || K < 1) return 0;
    const int tiles = ceil_div(N, BN) * ceil_div(M, BM), chunks = ceil_div(K, mma::KC);
    if (tiles >= 128 || chunks < 64) return 1;
    const int want = ceil_div(384, tiles), most = chunks / 8;
    const int layers = want < most ? want : most;
    // as launched: the last layers may be empty once k_per_layer is rounded to whole chunks
    return ceil_div(K, ceil_div(chunks, layers) * mma::KC);
}

extern "C" int dsspk_gemm_splitk(void* stream, const float* A, long a_rs, long a_cs, const float* B, long b_rs, long b_cs,
                                 float* C, long ldc, int M, int N, int K, const float* bias, int relu, float* scratch, int layers) {
    if (!A || !B || !C || M < 1 || N < 1 || K < 1 || layers < 1) return -1;
    if (layers == 1) return dsspk_gemm(stream, A, a_rs, a_cs, B, b_rs, b_cs, C, ldc, M, N, K, bias, relu);
    if (!scratch) return -1;
    hipStream_t s = (hipStream_t)stream;
    const int launched = launch_gemm(s, A, a_rs, a_cs, B, b_rs, b_cs, scratch, N, M, N, K, nullptr, 0, layers);
    const long n = (long)M * N;
    hipLaunchKernelGGL(splitk_sum_kernel, dim3((unsigned)ceil_div(n, 256L)), dim3(256), 0, s, scratch, C, ldc, M, N, launched, bias, relu);
    return DSSPK_LAUNCH_RC();
}

extern "C" size_t dsspk_colsum_scratch_floats(long M, int N) {
    return M > 1024 && N >= 1 ? (size_t)COLSUM_SLABS * N : 0;
}

extern "C" int dsspk_colsum(void* stream, const float* X, float* out, float* scratch, long M, int N) {
    if (!X || !out || M < 1 || N < 1) return -1;
    hipStream_t s = (hipStream_t)stream;
    if (dsspk_colsum_scratch_floats(M, N) == 0) {
        hipLaunchKernelGGL(colsum_kernel, dim3(ceil_div(N, 64), 1), dim3(256), 0, s, X, out, M, N, M);
        return DSSPK_LAUNCH_RC();
    }
    if (!scratch) return -1;
    const long rps = (M + COLSUM_SLABS - 1) / COLSUM_SLABS;
    const int slabs = ceil_div(M, rps);
    hipLaunchKernelGGL(colsum_kernel, dim3(ceil_div(N, 64), slabs), dim3(256), 0, s, X, scratch, M, N, rps);
    hipLaunchKernelGGL(colsum_kernel, dim3(ceil_div(N, 64), 1), dim3(256), 0, s, scratch, out, (long)slabs, N, (long)slabs);
    return DSSPK_LAUNCH_RC();
}

// ---- dsspk_colsum for callers that may not allocate: the slab sums go to device memory that is part of the library image
namespace {

constexpr int NOALLOC_MAX_N = DSSPK_COLSUM_NOALLOC_MAX_N;
constexpr int MAX_DEVICES = 64;

// One copy per GPU the library is loaded on, kept until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress: the device address it resolves to (per device) is what kernels and copies are given.
static __device__ __align__(256) float colsum_scratch[(size_t)COLSUM_SLABS * NOALLOC_MAX_N];

std::mutex scratch_mutex;
float* scratch_ptr[MAX_DEVICES];        // device address of colsum_scratch on each device, resolved on first use there

int resolve_scratch(float** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return DSSPK_NOALLOC_EHIP;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(colsum_scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return DSSPK_NOALLOC_EHIP;
        }
        scratch_ptr[dev] = static_cast<float*>(ptr);
    }
    *out = scratch_ptr[dev];
    return 0;
}

}  // namespace

extern "C" int dsspk_colsum_noalloc(void* stream, const float* X, float* out, long M, int N) {
    if (!X || !out || M < 1 || N < 1) return -1;
    if (N > NOALLOC_MAX_N) return DSSPK_NOALLOC_ETOOBIG;
    float* scratch = nullptr;
    if (int rc = resolve_scratch(&scratch)) return rc;
    // every slab row the second pass reads is written by the first pass of the same call, so nothing has to be cleared
    return dsspk_colsum(stream, X, out, scratch, M, N);
}
