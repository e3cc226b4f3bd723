// fp32 matrix-core building block for gfx950, shared by the GEMM and convolution kernels.
//
// v_mfma_f32_16x16x4_f32: one wavefront (64 lanes) multiplies a 16x4 A block by a 4x16 B block
// and accumulates into a 16x16 fp32 tile.  Lane l supplies A[l % 16][l / 16] and
// B[l / 16][l % 16]; afterwards lane l holds D[4 * (l / 16) + v][l % 16] in accumulator
// register v (v = 0..3).
//
// A k-chunk of 16 is consumed by four such instructions.  Which of the 16 k-indices goes to
// which instruction is free as long as A and B agree, so lane group q = l / 16 takes
// k = 4q .. 4q+3, one per instruction: a lane then needs four *consecutive* k values of one
// row, i.e. a single 16-byte LDS read when the tile is stored k-contiguous.
#pragma once
#include "common.hpp"

namespace mma {

constexpr int KC = 16;          // k-chunk per LDS stage
constexpr int LDK = KC + 4;     // row pitch (floats) of a k-contiguous tile: keeps 16-byte alignment,
                                // and 20 floats per row spreads rows over the LDS banks

// acc[wm][wn] += A_tile * B_tile for one k-chunk.
//   A_KM = false: As[row * lda + k]  (k-contiguous, lda = LDK)      true: As[k * lda + row]
//   B_NK = true : Bs[col * ldb + k]  (k-contiguous, ldb = LDK)      false: Bs[k * ldb + col]
// row0 / col0: first row / column of this wavefront's (16*WM) x (16*WN) tile inside the LDS tiles.
template <int WM, int WN, bool A_KM, bool B_NK>
__device__ __forceinline__ void chunk16(const float* __restrict__ As, int lda, const float* __restrict__ Bs, int ldb,
                                        int row0, int col0, floatx4 (&acc)[WM][WN], int lane) {
    const int l16 = lane & 15, q = lane >> 4;
    float a[WM][4], b[WN][4];
#pragma unroll
    for (int wm = 0; wm < WM; ++wm) {
        const int row = row0 + 16 * wm + l16;
        if constexpr (!A_KM) {
            const float4 v = *reinterpret_cast<const float4*>(As + row * lda + 4 * q);
            a[wm][0] = v.x; a[wm][1] = v.y; a[wm][2] = v.z; a[wm][3] = v.w;
        } else {
#pragma unroll
            for (int s = 0; s < 4; ++s) a[wm][s] = As[(4 * q + s) * lda + row];
        }
    }
#pragma unroll
    for (int wn = 0; wn < WN; ++wn) {
        const int col = col0 + 16 * wn + l16;
        if constexpr (B_NK) {
            const float4 v = *reinterpret_cast<const float4*>(Bs + col * ldb + 4 * q);
            b[wn][0] = v.x; b[wn][1] = v.y; b[wn][2] = v.z; b[wn][3] = v.w;
        } else {
#pragma unroll
            for (int s = 0; s < 4; ++s) b[wn][s] = Bs[(4 * q + s) * ldb + col];
        }
    }
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int wm = 0; wm < WM; ++wm)
#pragma unroll
            for (int wn = 0; wn < WN; ++wn)
                acc[wm][wn] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[wm][s], b[wn][s], acc[wm][wn], 0, 0, 0);
}

// Call between the last MFMA of a kernel and the first read of its accumulators.  A matrix-core instruction delivers
// its result several passes after issue and software has to keep dependent reads far enough behind; the compiler
// counts those wait states within a basic block.  One earlier build of the 3x3 kernel had the last MFMA of its product
// loop and the first accumulator read in different basic blocks (a data-dependent branch sat right behind the loop) and
// read one accumulator register too early on the short side of that branch (caught by the element-wise parity test).  The present kernels, built with the present compiler, pass every test without this
// guard too, so it is a precaution, not a necessity: 32 idle cycles per wavefront and call site (13 ns at 2.4 GHz,
// against kernels of 5 us and more), fenced against instruction scheduling, which cover the longest fp32 MFMA on
// every path.
__device__ __forceinline__ void drain() {
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

template <int WM, int WN>
__device__ __forceinline__ void zero(floatx4 (&acc)[WM][WN]) {
#pragma unroll
    for (int wm = 0; wm < WM; ++wm)
#pragma unroll
        for (int wn = 0; wn < WN; ++wn) acc[wm][wn] = floatx4{0.f, 0.f, 0.f, 0.f};
}

}  // namespace mma
