// 3x3, stride 1, pad 1 convolutions with Cin = Cout = C (the 106 inner convolutions of
// ResNet-110): forward and gradient w.r.t. the input as ONE kernel.
//
// A workgroup owns a band of R output rows of one image (the whole 8x8 image in the last
// stage) and CN of the C output channels.  It loads the (R+2) x (HW+2) x C input halo tile
// (zero borders) into LDS once; everything else is served from LDS, so every input element
// is read from memory once per band instead of nine times.  The filter never passes through
// LDS: a wavefront owns ONE tile of 16 output channels and keeps that tile's 9 x C filter
// values in registers (9 * C / 16 float4 per lane, fetched straight from the cached filter
// while the halo tile is still in flight).  LDS therefore holds the halo tile only (about
// 27 KB in every stage), which lets workgroups of several kernels share a compute unit.
//
// The arithmetic is Winograd's minimal filtering F(2x2, 3x3) (Lavin & Gray, "Fast Algorithms for
// Convolutional Neural Networks"): per 2x2 output tile and channel pair 16 multiplications instead of 36,
// Y = A^T [ (G g G^T) .* (B^T d B) ] A with the element-wise products summed over the input channels - which
// is a matrix product per position of the transformed 4x4 patch, M_xi[tile][co] = sum_k V_xi[tile][k] U_xi[k][co].
// Those 16 products run on the matrix cores: v_mfma_f32_16x16x4_f32, 16 tiles x 16 output channels per wavefront,
// with the k-permutation of mma.hpp (both operands k-contiguous per lane: one float4 feeds four MFMAs).  Patch and
// filter transforms are float4 additions in registers (no multiplications but the halvings of G), so the matrix
// cores do 4/9 of the direct form's work; in fp32 the result differs from the direct form by a few ulps.
//
// Gradient w.r.t. the input of such a convolution is the same operation on dy with the filter
// taps reversed and its two channel indices swapped; only the filter fetch differs.
#include "mma.hpp"
#include "bn_merge.hpp"
#include "jobs.hpp"
#include "../../include/dssp_kernels.h"

namespace {

constexpr int THREADS = 256;

// Workgroups are handed to the 8 XCDs round-robin (workgroup b runs on XCD b mod 8) and every XCD has an L2 of its
// own.  Tiles that are neighbours in memory share data - halo rows between the bands of an image, the whole input
// tile between the channel splits of a band, dy between the input-channel slices of the last stage's d-filter
// kernel - so consecutive tiles go to ONE XCD: workgroup b takes tile (b mod 8) * (n / 8) + b / 8, and what the
// first of them fetched is in that L2 for the next (without this, halo rows and shared tiles come over the fabric
// once per XCD that touches them: 1.1x to 1.7x the operands' bytes).  Needs n to be a multiple of 8.
__device__ __forceinline__ int xcd_tile(int block, int n_blocks) {
    constexpr int XCDS = 8;
    return n_blocks % XCDS ? block : (block % XCDS) * (n_blocks / XCDS) + block / XCDS;
}

// ---- gradient w.r.t. the filter by minimal filtering F(3x3, 2x2):
//      dw[tap][ci][co] = sum over pixels x[pixel + tap][ci] dy[pixel][co]; per 2x2 tile of dy and its 4x4 patch of x,
//      dw += A^T [ (B^T x B) .* (G dy G^T) ] A with B^T = [1 0 -1 0; 0 1 1 0; 0 -1 1 0; 0 -1 0 1],
//      G = [1 0; .5 .5; .5 -.5; 0 1], A^T = [1 1 1 0; 0 1 -1 0; 0 1 1 1].  The sum over tiles is taken in the
//      transformed domain by the matrix cores, M_xi[ci][co] += sum over tiles XT_xi[ci][tile] DT_xi[tile][co]
//      (16 products instead of 36 per tile), and A^T M A is applied once at the end.
// One run of 16 tiles: the lane (l16, q) transforms, as scalars, the patch (its input channel) and the dy tile (its
// output channel) of tile 4q + s for each of the four MFMA steps s.  at(tile) locates a tile once; x_at(o, r, c) and
// d_at(o, i, j) fetch the patch and dy elements from there.
template <class At, class XAt, class DAt>
__device__ __forceinline__ void dfilter_run(floatx4 (&M)[16], int q, At at, XAt x_at, DAt d_at) {
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const auto tile = at(4 * q + s);
        float XT[16], DT[16];
        {
            float t[4][4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                float x[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) x[r] = x_at(tile, r, c);
                t[0][c] = x[0] - x[2]; t[1][c] = x[1] + x[2]; t[2][c] = x[2] - x[1]; t[3][c] = x[3] - x[1];
            }
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                XT[4 * a] = t[a][0] - t[a][2]; XT[4 * a + 1] = t[a][1] + t[a][2];
                XT[4 * a + 2] = t[a][2] - t[a][1]; XT[4 * a + 3] = t[a][3] - t[a][1];
            }
        }
        {
            float u[4][2];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const float d0 = d_at(tile, 0, j), d1 = d_at(tile, 1, j);
                u[0][j] = d0; u[1][j] = 0.5f * (d0 + d1); u[2][j] = 0.5f * (d0 - d1); u[3][j] = d1;
            }
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                DT[4 * a] = u[a][0]; DT[4 * a + 1] = 0.5f * (u[a][0] + u[a][1]);
                DT[4 * a + 2] = 0.5f * (u[a][0] - u[a][1]); DT[4 * a + 3] = u[a][1];
            }
        }
#pragma unroll
        for (int xi = 0; xi < 16; ++xi) M[xi] = __builtin_amdgcn_mfma_f32_16x16x4f32(XT[xi], DT[xi], M[xi], 0, 0, 0);
    }
}

// dw = A^T M A; call after mma::drain().
__device__ __forceinline__ void dfilter_finish(const floatx4 (&M)[16], floatx4 (&dw)[9]) {
    floatx4 S[3][4];
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        S[0][b] = M[b] + M[4 + b] + M[8 + b];
        S[1][b] = M[4 + b] - M[8 + b];
        S[2][b] = M[4 + b] + M[8 + b] + M[12 + b];
    }
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        dw[3 * r] = S[r][0] + S[r][1] + S[r][2];
        dw[3 * r + 1] = S[r][1] - S[r][2];
        dw[3 * r + 2] = S[r][1] + S[r][2] + S[r][3];
    }
}

template <int C, int HW, int R, int NSPLIT>
struct Cfg {
    static constexpr int CN = C / NSPLIT;          // output channels per workgroup
    static constexpr int LDC = C + 4;              // pitch of one pixel in LDS (floats)
    static constexpr int TW = HW + 2;              // halo tile width
    static constexpr int XS = (R + 2) * TW * LDC;  // floats
    static constexpr int RUNS = R * HW / 16;       // output pixels of the band / 16
    static constexpr int WAVES_N = CN / 16;        // wavefronts side by side over the output channels
    static constexpr int WAVES_M = 4 / WAVES_N;    // ... and over the runs
    static constexpr int WM = RUNS / WAVES_M;      // accumulator tiles (16 pixels x 16 channels) a wavefront finishes
    static constexpr int KC = C / 16;              // 16-wide chunks of the reduction channel
    static constexpr int SS = 8 * CN;              // per-wavefront column sums (batch-norm records, two components)
    static constexpr int PS = THREADS + 2 * C;     // merge of the input's batch-norm records: tree + (mean, invstd)
    // A run is 16 tiles of 2x2 outputs; every wavefront works on one run.  If the band has fewer runs than
    // WAVES_M (last stage: 16 tiles per image), KS wavefronts share a run and split the input channels; they swap
    // halves of their partial results through LDS and each finishes its half.
    static constexpr int WRUNS = (R / 2) * (HW / 2) / 16;      // runs per band
    static constexpr int KS = WAVES_M / WRUNS;                 // wavefronts per run, each with 1/KS of the channels
    static constexpr int KCW = KC / KS;                        // k-chunks per wavefront
    static constexpr size_t LDS_BYTES = (size_t)(XS + SS + PS) * sizeof(float);
    static constexpr size_t LDS_BYTES_WG = LDS_BYTES + (size_t)XS * sizeof(float);   // + the x halo tile of the fused d-filter
    static_assert(WAVES_N == 1 || WAVES_N == 2 || WAVES_N == 4, "one 16-channel tile per wavefront");
    static_assert(RUNS % WAVES_M == 0 && WM >= 1, "band must give every wavefront at least one run");
    static_assert(WRUNS * KS == WAVES_M && (KS == 1 || KS == 2) && WM * KS == 4 && KCW * KS == KC,
                  "one run of 16 tiles per wavefront, 16 / KS outputs per lane");
};

// Normalisation applied to the input while it is loaded (PRE != 0): the kernel then computes
//   a = ReLU(gamma * (src - mean) * invstd + beta (+ shortcut))   and   dst = conv(a),
// i.e. the batch norm + ReLU that separates two convolutions never runs as a pass of its own.
// mean / invstd come from the statistics records of src, merged by a one-workgroup kernel launched just
// before (they are also what the backward pass needs); the workgroups write `a` (their own rows).
struct PreBn {
    const float* records;      // statistics records of src
    bnm::BnLayout L;           // their layout
    long M;                    // rows of src (= N * HW * HW)
    const float* gamma;
    const float* beta;
    float eps;
    const float* shortcut;     // PRE == 2: added before the ReLU, same shape as src
    float* act_out;            // a
    float* stats_out;          // mean[C], invstd[C]
};

// Backward of the ReLU + batch norm that FOLLOWS in the backward direction, started in the epilogue (POST):
// the result r (gradient w.r.t. a post-ReLU activation) is masked, dz = r * [mask_src > 0], dz is what gets
// stored, and the per-tile sums (sum dz, sum dz * xhat) with xhat = (xc - mean) * invstd are written as
// records for the batch norm's dx kernel.  This replaces that batch norm's stand-alone reduction pass.
struct PostBn {
    const float* mask_src;     // the saved post-ReLU activation
    const float* xc;           // the batch norm's input (convolution output)
    const float* stats;        // its mean[C], invstd[C]
    float* records;            // out: (sum dz, sum dz * xhat) per tile and channel
};

// Batch-norm backward applied to the input while it is loaded (PRE == 3, d-input convolutions): src is dz, the
// masked gradient at the batch norm's output, and the convolution runs on
//   dx = gamma * invstd * (dz - sum(dz) / M - xhat * sum(dz * xhat) / M),   xhat = (xc - mean) * invstd,
// the gradient w.r.t. the batch norm's input xc; the workgroups also write dx (their own rows) for the
// d-filter kernel.  The two sums come from the records of the epilogue that produced dz (TotalsJob).
struct BwdBn {
    const float* xc;           // the batch norm's input
    const float* stats;        // its mean[C], invstd[C]
    const float* gamma;
    const float* totals;       // sum dz [C], sum dz * xhat [C]
    float inv_m;               // 1 / (N * HW * HW)
    float* dx_out;
};

// Gradient w.r.t. the filter in the same kernel (WG, only with PRE == 3 and all channels in one workgroup): the
// dx tile the loader has just built in LDS is the d-filter convolution's dy, so only the convolution's input x
// (halo tile, a second LDS buffer) has to be fetched; dx itself never goes to memory.  After the d-input MFMA
// loop the wavefronts accumulate, as wgrad3x3_kernel does, dw[tap][ci][co] += x[pixel + tap][ci] * dx[pixel][co]
// over the band's pixels and store the workgroup's partial result; the sum over workgroups is a carried job of
// a later kernel.
struct WgradFused {
    const float* x_in;         // input of the convolution (post-ReLU activation of the layer below); it is also the
                               // source of the epilogue's ReLU mask, which is then taken from the LDS tile
    float* partial;            // out: [workgroup][9][C][C]
};

// add and dst may be the same buffer (every element is read and written by the same lane); with PRE == 3
// dst must differ from src, whose halo rows other workgroups still read.
// Registers: with the Winograd form the compiler would keep all 16 accumulator tiles in flight and the kernel
// at 2-3 wavefronts per SIMD; told how many should fit, it orders the work row by row instead (no spills).
template <int C, bool TRANSPOSED, bool WG>
constexpr int min_waves() { return C == 16 ? (WG ? 2 : TRANSPOSED ? 3 : 4) : C == 32 ? 2 : 1; }

template <int C, int HW, int R, int NSPLIT, bool TRANSPOSED, int PRE, bool POST = false, bool WG = false>
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(min_waves<C, TRANSPOSED, WG>()))) void conv3x3_kernel(const float* __restrict__ src, const float* __restrict__ wgt,
                                                          const float* add, float* dst,
                                                          float* __restrict__ bn_partial, PreBn pre, PostBn post, BwdBn bwd,
                                                          int conv_blocks, jobs::ReduceJob rj, WgradFused wg) {
    using K = Cfg<C, HW, R, NSPLIT>;
    static_assert(!WG || (PRE == 3 && NSPLIT == 1 && TRANSPOSED && (C == 16 || C == 32)), "fused d-filter: d-input form, whole channel range");
    extern __shared__ __attribute__((aligned(16))) float lds[];
    if ((int)blockIdx.x >= conv_blocks) {           // workgroups behind the convolution's own carry the reduction job
        jobs::wgrad_reduce(rj, blockIdx.x - conv_blocks, lds);
        return;
    }
    float* Xs = lds;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, q = lane >> 4;
    const int wave_n = wave % K::WAVES_N, wave_m = wave / K::WAVES_N;
    constexpr int BANDS = HW / R;
    const int tile = xcd_tile(blockIdx.x, conv_blocks);
    const int split = tile % NSPLIT;
    const int band = (tile / NSPLIT) % BANDS;
    const int n = tile / (NSPLIT * BANDS);
    const int r_base = band * R;                    // first output row of the band
    const int co_base = split * K::CN;
    const int co = co_base + 16 * wave_n + l16;     // this lane's output channel (column of the MFMA tile)

    // ---- input halo tile, zero outside the image.  The raw loads are issued first; with PRE the merge of
    //      the statistics records (a latency chain of its own) then runs while they are in flight.
    constexpr int V = C / 4;
    constexpr int NL = ((R + 2) * K::TW * V + THREADS - 1) / THREADS;
    float* Sh = PRE == 3 ? lds + K::XS + K::SS                  // five per-channel vectors (PRE == 3)
                         : lds + K::XS + K::SS + THREADS;       // mean[C], invstd[C] of the input (PRE == 1, 2)
    float4 val[NL], scv[PRE >= 2 ? NL : 1], xin[WG ? NL : 1];
    float* Xs2 = lds + K::XS + K::SS + K::PS;                   // x halo tile (WG)
#pragma unroll
    for (int e = 0; e < NL; ++e) {
        const int idx = tid + e * THREADS;
        const int v = idx % V;
        const int pc = (idx / V) % K::TW, pr = idx / (V * K::TW);
        const int h = r_base + pr - 1, w = pc - 1;
        val[e] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (pr < R + 2 && h >= 0 && h < HW && w >= 0 && w < HW) {
            const long off = (((long)n * HW + h) * HW + w) * C + 4 * v;
            val[e] = *reinterpret_cast<const float4*>(src + off);
            if constexpr (PRE == 2) scv[e] = *reinterpret_cast<const float4*>(pre.shortcut + off);
            if constexpr (PRE == 3) scv[e] = *reinterpret_cast<const float4*>(bwd.xc + off);
        }
        if constexpr (WG) {
            xin[e] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (pr < R + 2 && h >= 0 && h < HW && w >= 0 && w < HW)
                xin[e] = *reinterpret_cast<const float4*>(wg.x_in + (((long)n * HW + h) * HW + w) * C + 4 * v);
        }
    }
    if constexpr (PRE == 1 || PRE == 2) {   // mean / invstd of the input, merged from its records by records_merge_kernel
        if (tid < 2 * C) Sh[tid] = pre.stats_out[tid];
        __syncthreads();
    }
    if constexpr (PRE == 3) {               // mean, invstd, gamma * invstd, sum(dz) / M, sum(dz * xhat) / M
        if (tid < C) {
            const float is = bwd.stats[C + tid];
            Sh[tid] = bwd.stats[tid];
            Sh[C + tid] = is;
            Sh[2 * C + tid] = bwd.gamma[tid] * is;
            Sh[3 * C + tid] = bwd.totals[tid] * bwd.inv_m;
            Sh[4 * C + tid] = bwd.totals[C + tid] * bwd.inv_m;
        }
        __syncthreads();
    }
#pragma unroll
    for (int e = 0; e < NL; ++e) {
        const int idx = tid + e * THREADS;
        const int v = idx % V;
        const int pc = (idx / V) % K::TW, pr = idx / (V * K::TW);
        const int h = r_base + pr - 1, w = pc - 1;
        if (pr >= R + 2) continue;
        if constexpr (PRE == 3) {
            if (h >= 0 && h < HW && w >= 0 && w < HW) {
                const float4 mu = *reinterpret_cast<const float4*>(Sh + 4 * v);
                const float4 is = *reinterpret_cast<const float4*>(Sh + C + 4 * v);
                const float4 gi = *reinterpret_cast<const float4*>(Sh + 2 * C + 4 * v);
                const float4 db = *reinterpret_cast<const float4*>(Sh + 3 * C + 4 * v);
                const float4 dg = *reinterpret_cast<const float4*>(Sh + 4 * C + 4 * v);
                float4 o;
                o.x = gi.x * (val[e].x - db.x - (scv[e].x - mu.x) * is.x * dg.x);
                o.y = gi.y * (val[e].y - db.y - (scv[e].y - mu.y) * is.y * dg.y);
                o.z = gi.z * (val[e].z - db.z - (scv[e].z - mu.z) * is.z * dg.z);
                o.w = gi.w * (val[e].w - db.w - (scv[e].w - mu.w) * is.w * dg.w);
                val[e] = o;
                if (!WG && split == 0 && pr >= 1 && pr <= R)
                    *reinterpret_cast<float4*>(bwd.dx_out + (((long)n * HW + h) * HW + w) * C + 4 * v) = o;
            }
        }
        if constexpr (WG) *reinterpret_cast<float4*>(&Xs2[(pr * K::TW + pc) * K::LDC + 4 * v]) = xin[e];
        if constexpr (PRE == 1 || PRE == 2) {
            if (h >= 0 && h < HW && w >= 0 && w < HW) {
                const float4 mu = *reinterpret_cast<const float4*>(Sh + 4 * v);
                const float4 is = *reinterpret_cast<const float4*>(Sh + C + 4 * v);
                const float4 ga = *reinterpret_cast<const float4*>(pre.gamma + 4 * v);
                const float4 be = *reinterpret_cast<const float4*>(pre.beta + 4 * v);
                float4 o = val[e];
                o.x = fmaf((o.x - mu.x) * is.x, ga.x, be.x);
                o.y = fmaf((o.y - mu.y) * is.y, ga.y, be.y);
                o.z = fmaf((o.z - mu.z) * is.z, ga.z, be.z);
                o.w = fmaf((o.w - mu.w) * is.w, ga.w, be.w);
                if constexpr (PRE == 2) { o.x += scv[e].x; o.y += scv[e].y; o.z += scv[e].z; o.w += scv[e].w; }
                o.x = fmaxf(o.x, 0.f); o.y = fmaxf(o.y, 0.f); o.z = fmaxf(o.z, 0.f); o.w = fmaxf(o.w, 0.f);
                val[e] = o;
                // the band's own rows (not the halo rows) are this workgroup's part of `a`
                if (split == 0 && pr >= 1 && pr <= R)
                    *reinterpret_cast<float4*>(pre.act_out + (((long)n * HW + h) * HW + w) * C + 4 * v) = o;
            }
        }
        *reinterpret_cast<float4*>(&Xs[(pr * K::TW + pc) * K::LDC + 4 * v]) = val[e];
    }
    // ---- filter values of this wavefront's 16 output channels, B[k][co] with k = 16 kc + 4 q + {0..3}:
    //      forward : w[tap][k][co]           (four loads, C floats apart)
    //      d-input : w[8 - tap][co][k]       (one 16-byte load, taps reversed)
    const int wrun = wave_m / K::KS, ks = wave_m % K::KS;      // this wavefront's run and share of the channels
    const int k0 = 16 * K::KCW * ks + 4 * q;                   // its first reduction channel
    float4 bf[9][K::KCW];
#pragma unroll
    for (int tap = 0; tap < 9; ++tap)
#pragma unroll
        for (int kc = 0; kc < K::KCW; ++kc) {
            if constexpr (TRANSPOSED) {
                bf[tap][kc] = *reinterpret_cast<const float4*>(wgt + ((long)(8 - tap) * C + co) * C + k0 + 16 * kc);
            } else {
                const float* wp = wgt + ((long)tap * C + k0 + 16 * kc) * C + co;
                bf[tap][kc] = make_float4(wp[0], wp[C], wp[2 * C], wp[3 * C]);
            }
        }
    __syncthreads();

    floatx4 acc[K::WM];
    // band-local pixel (row-major) of accumulator element (wm, v)
    auto pixel = [&](int wm, int v) {   // tile 4q + v of the wavefront's run, output (e / 2, e % 2) of its 2x2
        const int g = wrun * 16 + 4 * q + v, e = ks * K::WM + wm;
        return (2 * (g / (HW / 2)) + (e >> 1)) * HW + 2 * (g % (HW / 2)) + (e & 1);
    };
    {
        // ---- Winograd F(2x2, 3x3), Y = A^T [ (G g G^T) .* (B^T d B) ] A per tile and channel pair, the products
        //      summed over the input channels by the matrix cores: for each of the 16 positions of the transformed
        //      4x4 patch, M[tile][co] += V[tile][k] U[k][co].  A lane transforms the patch of tile l16 (channels
        //      16 kc + 4q ..) and the filter of output channel `co` (same channels), both element-wise on float4.
        constexpr int TXN = HW / 2;
        const int g = wrun * 16 + l16;
        const int base = (2 * (g / TXN) * K::TW + 2 * (g % TXN)) * K::LDC + k0;
        // Row a of the transformed patch at a time (4 of the 16 positions), so that only its four accumulators,
        // its four U and V values and the running A^T M sums are live: s0 = M0 + M1 + M2, s1 = M1 - M2 - M3.
        floatx4 s0[4], s1[4];
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            floatx4 m[4];
#pragma unroll
            for (int b = 0; b < 4; ++b) m[b] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kc = 0; kc < K::KCW; ++kc) {
                float4 U[4];           // row a of G g G^T, G = [1 0 0; .5 .5 .5; .5 -.5 .5; 0 0 1]
                {
                    float4 u[3];
#pragma unroll
                    for (int j = 0; j < 3; ++j) {
                        const float4 g0 = bf[j][kc], g1 = bf[3 + j][kc], g2 = bf[6 + j][kc];
                        u[j] = a == 0 ? g0 : a == 3 ? g2 : a == 1 ? (g0 + g2) * 0.5f + g1 * 0.5f : (g0 + g2) * 0.5f - g1 * 0.5f;
                    }
                    const float4 e = (u[0] + u[2]) * 0.5f, o = u[1] * 0.5f;
                    U[0] = u[0]; U[1] = e + o; U[2] = e - o; U[3] = u[2];
                }
                float4 V[4];           // row a of B^T d B, B^T = [1 0 -1 0; 0 1 1 0; 0 -1 1 0; 0 1 0 -1]
                {
                    constexpr int RA[4] = {0, 1, 2, 1}, RB[4] = {2, 2, 1, 3};      // t[a] = +-d[RA] +- d[RB]
                    float4 t[4];
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const float4 da = *reinterpret_cast<const float4*>(&Xs[base + (RA[a] * K::TW + c) * K::LDC + 16 * kc]);
                        const float4 db = *reinterpret_cast<const float4*>(&Xs[base + (RB[a] * K::TW + c) * K::LDC + 16 * kc]);
                        t[c] = a == 1 ? da + db : da - db;
                    }
                    V[0] = t[0] - t[2]; V[1] = t[1] + t[2]; V[2] = t[2] - t[1]; V[3] = t[1] - t[3];
                }
#pragma unroll
                for (int b = 0; b < 4; ++b) m[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(V[b].x, U[b].x, m[b], 0, 0, 0);
#pragma unroll
                for (int b = 0; b < 4; ++b) m[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(V[b].y, U[b].y, m[b], 0, 0, 0);
#pragma unroll
                for (int b = 0; b < 4; ++b) m[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(V[b].z, U[b].z, m[b], 0, 0, 0);
#pragma unroll
                for (int b = 0; b < 4; ++b) m[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(V[b].w, U[b].w, m[b], 0, 0, 0);
            }
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                if (a == 0) s0[b] = m[b];
                if (a == 1) { s0[b] += m[b]; s1[b] = m[b]; }
                if (a == 2) { s0[b] += m[b]; s1[b] -= m[b]; }
                if (a == 3) s1[b] -= m[b];
            }
        }
        mma::drain();
        // (A^T M) A, A^T = [1 1 1 0; 0 1 -1 -1]: element v of every accumulator belongs to tile 4q + v
        floatx4 y[4];
        y[0] = s0[0] + s0[1] + s0[2]; y[1] = s0[1] - s0[2] - s0[3];
        y[2] = s1[0] + s1[1] + s1[2]; y[3] = s1[1] - s1[2] - s1[3];
        if constexpr (K::KS == 1) {
#pragma unroll
            for (int wm = 0; wm < 4; ++wm) acc[wm] = y[wm];
        } else {
            // the two wavefronts of a run hold partial sums over their halves of the input channels: each hands
            // the other the two accumulators it will not finish and adds what it receives (first half + second half)
            __syncthreads();                               // every wavefront has read the tile for the last time
            float* Ex = lds;                               // [wavefront][2][4][64]
#pragma unroll
            for (int wm = 0; wm < 2; ++wm)
#pragma unroll
                for (int v = 0; v < 4; ++v) Ex[((wave * 2 + wm) * 4 + v) * 64 + lane] = ks == 0 ? y[2 + wm][v] : y[wm][v];
            __syncthreads();
            const int partner = (wave_m ^ 1) * K::WAVES_N + wave_n;
#pragma unroll
            for (int wm = 0; wm < 2; ++wm)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float other = Ex[((partner * 2 + wm) * 4 + v) * 64 + lane];
                    const float own = ks == 0 ? y[wm][v] : y[2 + wm][v];
                    acc[wm][v] = ks == 0 ? own + other : other + own;
                }
        }
    }

    mma::drain();
    // ---- store: lane holds the elements acc[wm][v] of pixels pixel(wm, v), all of output channel co
    float sum_dz = 0.f, sum_dzx = 0.f, mu_c = 0.f, is_c = 0.f;
    if constexpr (POST) {
        mu_c = post.stats[co];
        is_c = post.stats[C + co];
    }
    // all loads of the epilogue first (dst may alias add, so the compiler cannot move them across the stores itself)
    float addv[K::WM][4], maskv[POST ? K::WM : 1][4], xcv[POST ? K::WM : 1][4];
    auto out_off = [&](int wm, int v) {
        const int p = pixel(wm, v);
        return (((long)n * HW + r_base + p / HW) * HW + p % HW) * C + co;
    };
#pragma unroll
    for (int wm = 0; wm < K::WM; ++wm)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const long off = out_off(wm, v);
            addv[wm][v] = add ? add[off] : 0.f;
            if constexpr (POST) {
                if constexpr (WG) {     // the mask source is the convolution's input, whose tile is in LDS
                    const int p = pixel(wm, v);
                    maskv[wm][v] = Xs2[((p / HW + 1) * K::TW + (p % HW + 1)) * K::LDC + co];
                } else {
                    maskv[wm][v] = post.mask_src[off];
                }
                xcv[wm][v] = post.xc[off];
            }
        }
    if constexpr (WG) {
        // ---- d-filter of the same layer from the two LDS tiles, while the epilogue's operands are in flight (see
        //      dfilter_run): x patches from Xs2, dx tiles from the interior of Xs.
        //      C = 16: one 16x16 tile of (ci, co), the four wavefronts take one run each and are summed in a fixed
        //      order; C = 32: wavefront w owns tile (w / 2, w % 2) and walks both runs.
        constexpr bool SPLIT_K = (C == 16);
        constexpr int TXN = HW / 2;
        const int cit = SPLIT_K ? 0 : wave >> 1, cot = SPLIT_K ? 0 : wave & 1;
        floatx4 M[16];
#pragma unroll
        for (int xi = 0; xi < 16; ++xi) M[xi] = floatx4{0.f, 0.f, 0.f, 0.f};
        for (int run = SPLIT_K ? wave : 0; run < K::WRUNS; run += SPLIT_K ? 4 : 1) {
            dfilter_run(M, q,
                        [&](int tile) {                 // the patch's corner in both halo tiles
                            const int g = run * 16 + tile;
                            return (2 * (g / TXN) * K::TW + 2 * (g % TXN)) * K::LDC;
                        },
                        [&](int o, int r, int c) { return Xs2[o + (r * K::TW + c) * K::LDC + 16 * cit + l16]; },
                        [&](int o, int i, int j) { return Xs[o + ((i + 1) * K::TW + j + 1) * K::LDC + 16 * cot + l16]; });
        }
        mma::drain();
        floatx4 dwa[9];
        dfilter_finish(M, dwa);
        float* pout = wg.partial + (long)tile * 9 * C * C;
        if constexpr (SPLIT_K) {
            static_assert(!SPLIT_K || 4 * 9 * C * C <= 2 * K::XS + K::SS + K::PS, "room for the four partial sums");
            __syncthreads();                              // both tiles are no longer needed: reuse LDS for the 4 partial sums
            float* Red = lds;
#pragma unroll
            for (int t = 0; t < 9; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v) Red[wave * 9 * C * C + (t * C + 4 * q + v) * C + l16] = dwa[t][v];
            __syncthreads();
            for (int idx = tid; idx < 9 * C * C; idx += THREADS)
                pout[idx] = (Red[idx] + Red[9 * C * C + idx]) + (Red[2 * 9 * C * C + idx] + Red[3 * 9 * C * C + idx]);
            __syncthreads();                              // before the epilogue's sums use LDS again
        } else {
#pragma unroll
            for (int t = 0; t < 9; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v) pout[(t * C + 16 * cit + 4 * q + v) * C + 16 * cot + l16] = dwa[t][v];
        }
    }
#pragma unroll
    for (int wm = 0; wm < K::WM; ++wm)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float r = acc[wm][v] + addv[wm][v];
            if constexpr (POST) {
                r = maskv[wm][v] > 0.f ? r : 0.f;
                const float xh = (xcv[wm][v] - mu_c) * is_c;
                sum_dz += r;
                sum_dzx = fmaf(r, xh, sum_dzx);
            }
            dst[out_off(wm, v)] = r;
        }
    // per-channel totals over the workgroup's tile: lanes of a wavefront by shuffles, then the WAVES_M
    // wavefronts that share the channel tile through LDS, in a fixed order
    float* Ss = lds + K::XS;
    const int cl = 16 * wave_n + l16;                // channel inside the workgroup's CN
    auto tile_total = [&](const float* S) {
        float t = S[cl];
#pragma unroll
        for (int m = 1; m < K::WAVES_M; ++m) t += S[m * K::CN + cl];
        return t;
    };
    if constexpr (POST) {
        float a_ = sum_dz, b_ = sum_dzx;
        a_ += __shfl_xor(a_, 16); a_ += __shfl_xor(a_, 32);
        b_ += __shfl_xor(b_, 16); b_ += __shfl_xor(b_, 32);
        if (q == 0) { Ss[wave_m * K::CN + cl] = a_; Ss[4 * K::CN + wave_m * K::CN + cl] = b_; }
        __syncthreads();
        if (wave_m == 0 && q == 0)
            *reinterpret_cast<float2*>(post.records + ((long)(n * BANDS + band) * C + co) * 2) =
                make_float2(tile_total(Ss), tile_total(Ss + 4 * K::CN));
    }

    // ---- optional: batch-norm statistics of this workgroup's output tile, per channel:
    //      mean over its R*HW pixels and the sum of squared deviations from that mean
    //      (bn_partial[(g*C + c)*2 + {0,1}], g = image * bands + band), merged later like row slabs.
    if (bn_partial) {
        constexpr float inv_n = 1.0f / (float)(R * HW);
        float mean_t = 0.f;
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            float s_ = 0.f;
#pragma unroll
            for (int wm = 0; wm < K::WM; ++wm)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float d = pass == 0 ? acc[wm][v] : acc[wm][v] - mean_t;
                    s_ += pass == 0 ? d : d * d;
                }
            s_ += __shfl_xor(s_, 16);
            s_ += __shfl_xor(s_, 32);
            if (q == 0) Ss[wave_m * K::CN + cl] = s_;
            __syncthreads();
            const float tot = tile_total(Ss);
            if (pass == 0) mean_t = tot * inv_n;
            else if (wave_m == 0 && q == 0)
                *reinterpret_cast<float2*>(bn_partial + ((long)(n * BANDS + band) * C + co) * 2) = make_float2(mean_t, tot);
            __syncthreads();
        }
    }
}

// Statistics records -> mean[C], invstd[C].  One workgroup per 4 channels, 64 lanes per channel, so a lane
// fetches at most 8 records (all in flight together) and the kernel is a few microseconds of latency on
// C/4 CUs; cheaper than letting every workgroup of the consumer repeat the merge.  The arithmetic is the
// fixed-order merge of bn_merge.hpp: mean = sum n_g mean_g / M, M2 = sum (M2_g + n_g (mean_g - mean)^2).
__global__ __launch_bounds__(THREADS) void records_merge_kernel(const float* __restrict__ records, int G, long rows_per_record,
                                                                long M, int C, float eps, float* __restrict__ stats) {
    __shared__ float red[THREADS];
    constexpr int CW = 4, SUB = THREADS / CW;
    const int cl = threadIdx.x % CW, sub = threadIdx.x / CW;
    const int c = blockIdx.x * CW + cl;
    float2 pv[8];
    float nn[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int g = sub + u * SUB;
        const int gc = min(g, G - 1);
        pv[u] = *reinterpret_cast<const float2*>(records + ((long)gc * C + c) * 2);
        const long lo = (long)gc * rows_per_record;
        nn[u] = g < G ? (float)(min(M, lo + rows_per_record) - lo) : 0.f;
    }
    float s_ = 0.f;
#pragma unroll
    for (int u = 0; u < 8; ++u) s_ = fmaf(nn[u], pv[u].x, s_);
    const float mean = bnm::reduce_sub(s_, red, cl, sub, SUB, CW) / (float)M;
    float m2 = 0.f;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const float d = pv[u].x - mean;
        m2 += nn[u] > 0.f ? pv[u].y + nn[u] * d * d : 0.f;
    }
    m2 = bnm::reduce_sub(m2, red, cl, sub, SUB, CW);
    if (sub == 0) {
        stats[c] = mean;
        stats[C + c] = 1.0f / sqrtf(m2 / (float)M + eps);
    }
}

template <int C, int HW, int R, int NSPLIT, bool T, int PRE = 0, bool POST = false, bool WG = false>
int launch(hipStream_t s, const float* src, const float* w, const float* add, float* dst, float* bn_partial, int N,
           const PreBn& pre = PreBn(), const PostBn& post = PostBn(), const BwdBn& bwd = BwdBn(),
           const jobs::ReduceJob& rj = jobs::ReduceJob(), const WgradFused& wg = WgradFused()) {
    using K = Cfg<C, HW, R, NSPLIT>;
    constexpr size_t LDS_BYTES = WG ? K::LDS_BYTES_WG : K::LDS_BYTES;
    static_assert(LDS_BYTES >= jobs::LDS_FLOATS * sizeof(float), "room for a carried job");
    static bool attr_set = false;       // raise the dynamic-LDS limit once per instantiation
    auto kern = conv3x3_kernel<C, HW, R, NSPLIT, T, PRE, POST, WG>;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)LDS_BYTES) != hipSuccess)
            return -1;
        attr_set = true;
    }
    const int conv_blocks = N * (HW / R) * NSPLIT;
    hipLaunchKernelGGL(kern, dim3(conv_blocks + rj.blocks), dim3(THREADS), LDS_BYTES, s, src, w, add, dst, bn_partial, pre, post,
                       bwd, conv_blocks, rj, wg);
    return DSSPK_LAUNCH_RC();
}

}  // namespace

// dst = conv(src) (+ add, element-wise, if add != NULL).  Returns -2 if the shape is not one of the
// specialised ones (the caller then uses the generic kernel).
int conv3x3_tiled(hipStream_t s, const float* src, const float* w, const float* add, float* dst, float* bn_partial,
                   int N, int HW, int C, bool transposed) {
    if (C == 16 && HW == 32) return transposed ? launch<16, 32, 8, 1, true>(s, src, w, add, dst, bn_partial, N) : launch<16, 32, 8, 1, false>(s, src, w, add, dst, bn_partial, N);
    if (C == 32 && HW == 16) return transposed ? launch<32, 16, 8, 1, true>(s, src, w, add, dst, bn_partial, N) : launch<32, 16, 8, 1, false>(s, src, w, add, dst, bn_partial, N);
    if (C == 64 && HW == 8) return transposed ? launch<64, 8, 8, 2, true>(s, src, w, add, dst, bn_partial, N) : launch<64, 8, 8, 2, false>(s, src, w, add, dst, bn_partial, N);
    return -2;
}

// Forward convolution of a = ReLU(BN(src) (+ shortcut)), see PreBn.  in_parts: number of equal-sized
// statistics records of src in `records` (as emitted by the forward kernel for the same shape).
int conv3x3_tiled_prebn(hipStream_t s, const float* src, const float* records, int in_parts, const float* gamma,
                         const float* beta, float eps, const float* shortcut, float* act_out, float* stats_out,
                         const float* w, float* dst, float* bn_partial, int N, int HW, int C) {
    PreBn pre;
    pre.records = records;
    pre.M = (long)N * HW * HW;
    if (in_parts < 1 || pre.M % in_parts || in_parts > 32 * (THREADS / C)) return -1;
    pre.L = bnm::bn_layout(pre.M, C);
    pre.L.G = in_parts;
    pre.L.rows_per_block = pre.M / in_parts;
    pre.gamma = gamma; pre.beta = beta; pre.eps = eps;
    pre.shortcut = shortcut; pre.act_out = act_out; pre.stats_out = stats_out;
    if (C != 16 && C != 32 && C != 64) return -2;
    if (in_parts > 8 * (THREADS / 4)) return -1;
    hipLaunchKernelGGL(records_merge_kernel, dim3(C / 4), dim3(THREADS), 0, s, records, in_parts, pre.L.rows_per_block, pre.M, C, eps, stats_out);
    if (C == 16 && HW == 32)
        return shortcut ? launch<16, 32, 8, 1, false, 2>(s, src, w, nullptr, dst, bn_partial, N, pre)
                        : launch<16, 32, 8, 1, false, 1>(s, src, w, nullptr, dst, bn_partial, N, pre);
    if (C == 32 && HW == 16)
        return shortcut ? launch<32, 16, 8, 1, false, 2>(s, src, w, nullptr, dst, bn_partial, N, pre)
                        : launch<32, 16, 8, 1, false, 1>(s, src, w, nullptr, dst, bn_partial, N, pre);
    if (C == 64 && HW == 8)
        return shortcut ? launch<64, 8, 8, 2, false, 2>(s, src, w, nullptr, dst, bn_partial, N, pre)
                        : launch<64, 8, 8, 2, false, 1>(s, src, w, nullptr, dst, bn_partial, N, pre);
    return -2;
}

// d-input of the convolution (+ add) followed, in the same kernel, by the ReLU mask and the record sums of the
// batch norm that comes next in the backward direction, see PostBn.
int conv3x3_tiled_dgrad_post(hipStream_t s, const float* dy, const float* w, const float* add, float* dz,
                              const float* mask_src, const float* xc, const float* stats, float* records, int N, int HW, int C) {
    PostBn post;
    post.mask_src = mask_src; post.xc = xc; post.stats = stats; post.records = records;
    if (C == 16 && HW == 32) return launch<16, 32, 8, 1, true, 0, true>(s, dy, w, add, dz, nullptr, N, PreBn(), post);
    if (C == 32 && HW == 16) return launch<32, 16, 8, 1, true, 0, true>(s, dy, w, add, dz, nullptr, N, PreBn(), post);
    if (C == 64 && HW == 8) return launch<64, 8, 8, 2, true, 0, true>(s, dy, w, add, dz, nullptr, N, PreBn(), post);
    return -2;
}

// d-input convolution of dx = batch-norm backward of dz (see BwdBn), with the epilogue of conv3x3_tiled_dgrad_post;
// optionally carries the second stage of an earlier d-filter convolution (red_partial != NULL).
int conv3x3_tiled_dgrad_bn(hipStream_t s, const float* dz, const float* xc, const float* stats, const float* gamma,
                            const float* totals, float* dx_out, const float* w, const float* add, float* out,
                            const float* mask_src, const float* xc_post, const float* stats_post, float* records,
                            const float* red_partial, float* red_dw, int red_E, int red_chunks, int N, int HW, int C) {
    BwdBn bwd;
    bwd.xc = xc; bwd.stats = stats; bwd.gamma = gamma; bwd.totals = totals; bwd.dx_out = dx_out;
    bwd.inv_m = 1.0f / (float)((long)N * HW * HW);
    PostBn post;
    post.mask_src = mask_src; post.xc = xc_post; post.stats = stats_post; post.records = records;
    jobs::ReduceJob rj = jobs::ReduceJob();
    if (red_partial) {
        rj.partial = red_partial; rj.dw = red_dw; rj.E = red_E; rj.chunks = red_chunks;
        const int groups = jobs::reduce_groups(red_E, red_chunks);
        rj.blocks = groups < 288 ? groups : 288;
    }
    if (C == 16 && HW == 32) return launch<16, 32, 8, 1, true, 3, true>(s, dz, w, add, out, nullptr, N, PreBn(), post, bwd, rj);
    if (C == 32 && HW == 16) return launch<32, 16, 8, 1, true, 3, true>(s, dz, w, add, out, nullptr, N, PreBn(), post, bwd, rj);
    if (C == 64 && HW == 8) return launch<64, 8, 8, 2, true, 3, true>(s, dz, w, add, out, nullptr, N, PreBn(), post, bwd, rj);
    return -2;
}

// conv3x3_tiled_dgrad_bn with the d-filter convolution of the same layer in the same kernel (see WgradFused);
// dx is not stored.  Returns -2 for shapes the fused form does not cover (then the two-kernel form applies).
int conv3x3_tiled_dgrad_bn_wgrad(hipStream_t s, const float* dz, const float* xc, const float* stats, const float* gamma,
                                  const float* totals, const float* w, const float* add, float* out,
                                  const float* xc_post, const float* stats_post, float* records,
                                  const float* x_in, float* partial, const float* red_partial, float* red_dw, int red_E,
                                  int red_chunks, int N, int HW, int C) {
    BwdBn bwd;
    bwd.xc = xc; bwd.stats = stats; bwd.gamma = gamma; bwd.totals = totals; bwd.dx_out = nullptr;
    bwd.inv_m = 1.0f / (float)((long)N * HW * HW);
    PostBn post;
    post.mask_src = x_in; post.xc = xc_post; post.stats = stats_post; post.records = records;
    jobs::ReduceJob rj = jobs::ReduceJob();
    if (red_partial) {
        rj.partial = red_partial; rj.dw = red_dw; rj.E = red_E; rj.chunks = red_chunks;
        const int groups = jobs::reduce_groups(red_E, red_chunks);
        rj.blocks = groups < 288 ? groups : 288;
    }
    WgradFused wg;
    wg.x_in = x_in; wg.partial = partial;
    if (C == 16 && HW == 32) return launch<16, 32, 8, 1, true, 3, true, true>(s, dz, w, add, out, nullptr, N, PreBn(), post, bwd, rj, wg);
    if (C == 32 && HW == 16) return launch<32, 16, 8, 1, true, 3, true, true>(s, dz, w, add, out, nullptr, N, PreBn(), post, bwd, rj, wg);
    return -2;
}

// Number of per-workgroup statistics records (tiles of equal size) the forward kernel emits, 0 if the
// shape is not covered by it.
int conv3x3_tiled_stat_parts(int N, int HW, int C) {
    if (C == 16 && HW == 32) return N * 4;
    if (C == 32 && HW == 16) return N * 2;
    if (C == 64 && HW == 8) return N;
    return 0;
}

// ---------------------------------------------------------------------------------------------
// Gradient w.r.t. the filter of the same convolutions, stage 1 of 2: one workgroup per band of
// R rows of one image; the x halo tile and the dy tile sit in LDS and all nine taps
//   dw[tap][ci][co] += sum_{pixels of the band} x[pixel + tap][ci] * dy[pixel][co]
// are accumulated from them (x and dy are read from memory once), by minimal filtering (dfilter_run).  The
// matrix-core tile is 16 (ci) x 16 (co), the reduction runs over tiles of 2x2 pixels in runs of 16.
//   C = 16: one (ci, co) tile; the four wavefronts take one run each and are summed in a fixed order at the end.
//   C = 32: four (ci, co) tiles; wavefront w owns tile (w / 2, w % 2) and walks both runs.
// Output: partial[workgroup][tap][ci][co]; stage 2 (wgrad_reduce_kernel) sums over workgroups.
namespace {

template <int C, int HW, int R>
struct WCfg {
    static constexpr int LDC = C + 4;
    static constexpr int TW = HW + 2;
    static constexpr int XS = (R + 2) * TW * LDC;
    static constexpr int DS = R * HW * LDC;
    static constexpr bool SPLIT_K = (C == 16);
    static_assert(!SPLIT_K || (R / 2) * (HW / 2) == 64, "one run of 16 tiles per wavefront");
    static constexpr int RED = SPLIT_K ? 4 * 9 * C * C : 0;
    static constexpr size_t LDS_BYTES = (size_t)((XS + DS) > RED ? (XS + DS) : RED) * sizeof(float);
};

template <int C, int HW, int R>
__global__ __launch_bounds__(THREADS) void wgrad3x3_kernel(const float* __restrict__ x, const float* __restrict__ dy,
                                                           float* __restrict__ partial, int own_blocks, jobs::TotalsJob tj) {
    using K = WCfg<C, HW, R>;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    if ((int)blockIdx.x >= own_blocks) {            // workgroups behind the kernel's own carry the batch-norm sums job
        jobs::bn_totals(tj, blockIdx.x - own_blocks, lds);
        return;
    }
    float* Xs = lds;
    float* Ds = lds + K::XS;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int BANDS = HW / R;
    const int tile = xcd_tile(blockIdx.x, own_blocks);
    const int band = tile % BANDS, n = tile / BANDS;
    const int r_base = band * R;
    constexpr int V = C / 4;
    for (int idx = tid; idx < (R + 2) * K::TW * V; idx += THREADS) {
        const int v = idx % V;
        const int pc = (idx / V) % K::TW, pr = idx / (V * K::TW);
        const int h = r_base + pr - 1, w = pc - 1;
        float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
        if (h >= 0 && h < HW && w >= 0 && w < HW)
            val = *reinterpret_cast<const float4*>(x + (((long)n * HW + h) * HW + w) * C + 4 * v);
        *reinterpret_cast<float4*>(&Xs[(pr * K::TW + pc) * K::LDC + 4 * v]) = val;
    }
    const float* dyb = dy + ((long)n * HW + r_base) * HW * C;
    for (int idx = tid; idx < R * HW * V; idx += THREADS) {
        const int v = idx % V, p = idx / V;
        *reinterpret_cast<float4*>(&Ds[p * K::LDC + 4 * v]) = *reinterpret_cast<const float4*>(dyb + (long)p * C + 4 * v);
    }
    __syncthreads();

    const int l16 = lane & 15, q = lane >> 4;
    const int cit = K::SPLIT_K ? 0 : wave >> 1, cot = K::SPLIT_K ? 0 : wave & 1;
    constexpr int TXN = HW / 2, WRUNS = (R / 2) * TXN / 16;
    floatx4 M[16];
#pragma unroll
    for (int xi = 0; xi < 16; ++xi) M[xi] = floatx4{0.f, 0.f, 0.f, 0.f};
    for (int run = K::SPLIT_K ? wave : 0; run < WRUNS; run += K::SPLIT_K ? 4 : 1) {
        dfilter_run(M, q,
                    [&](int tile) { return make_int2(2 * ((run * 16 + tile) / TXN), 2 * ((run * 16 + tile) % TXN)); },
                    [&](int2 o, int r, int c) { return Xs[((o.x + r) * K::TW + o.y + c) * K::LDC + 16 * cit + l16]; },
                    [&](int2 o, int i, int j) { return Ds[((o.x + i) * HW + o.y + j) * K::LDC + 16 * cot + l16]; });
    }
    mma::drain();
    floatx4 acc[9];
    dfilter_finish(M, acc);
    float* out = partial + (long)tile * 9 * C * C;
    if constexpr (K::SPLIT_K) {
        __syncthreads();                              // tiles no longer needed: reuse LDS for the 4 partial sums
        float* Red = lds;
#pragma unroll
        for (int t = 0; t < 9; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) Red[wave * 9 * C * C + (t * C + 4 * q + v) * C + l16] = acc[t][v];
        __syncthreads();
        for (int idx = tid; idx < 9 * C * C; idx += THREADS)
            out[idx] = (Red[idx] + Red[9 * C * C + idx]) + (Red[2 * 9 * C * C + idx] + Red[3 * 9 * C * C + idx]);
    } else {
#pragma unroll
        for (int t = 0; t < 9; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) out[(t * C + 16 * cit + 4 * q + v) * C + 16 * cot + l16] = acc[t][v];
    }
}

// The same for the last stage (64 channels, 8x8 images), where one image is only four pixel chunks and the
// result is as large as 9 x 64 x 64: a workgroup owns 16 of the input channels (wavefront w: output channels
// 16w..16w+15, the 16 accumulator tiles of the transformed domain) and IMGS whole images, one after the other; the next image's
// x halo tile (its 16 channels only) and dy tile are fetched into registers while the matrix cores work on the
// current one (two LDS buffers, one barrier per image).  Output: partial[image group][tap][ci][co], the
// workgroup's 16 ci rows of it.
template <int IMGS>
__global__ __launch_bounds__(THREADS) void wgrad3x3_wide_kernel(const float* __restrict__ x, const float* __restrict__ dy,
                                                                float* __restrict__ partial, int N, int own_blocks,
                                                                jobs::TotalsJob tj) {
    constexpr int C = 64, HW = 8, TW = HW + 2, CIW = 16, LDA = CIW + 4, LDB = C + 4;
    constexpr int XS = TW * TW * LDA, DS = HW * HW * LDB, BUF = XS + DS;
    constexpr int XV = (TW * TW * (CIW / 4) + THREADS - 1) / THREADS, DV = HW * HW * (C / 4) / THREADS;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    if ((int)blockIdx.x >= own_blocks) {
        jobs::bn_totals(tj, blockIdx.x - own_blocks, lds);
        return;
    }
    const int tid = threadIdx.x, lane = tid & 63, cot = tid >> 6;
    const int l16 = lane & 15, q = lane >> 4;
    const int tile = xcd_tile(blockIdx.x, own_blocks);
    const int cit = tile % (C / CIW), grp = tile / (C / CIW);
    const int n0 = grp * IMGS;
    const int nimg = min(IMGS, N - n0);
    float4 rx[XV], rd[DV];
#pragma unroll
    for (int e = 0; e < XV; ++e) rx[e] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int e = 0; e < DV; ++e) rd[e] = make_float4(0.f, 0.f, 0.f, 0.f);
    // written out as macros: with lambdas that capture the two arrays the compiler kept rd in scratch memory
#define WIDE_FETCH(n)                                                                                                      \
    _Pragma("unroll") for (int e = 0; e < XV; ++e) {                                                                       \
        const int idx = tid + e * THREADS;                                                                                 \
        const int v = idx % (CIW / 4), pix = idx / (CIW / 4);                                                              \
        const int h = pix / TW - 1, w = pix % TW - 1;                                                                      \
        rx[e] = make_float4(0.f, 0.f, 0.f, 0.f);                                                                           \
        if (pix < TW * TW && h >= 0 && h < HW && w >= 0 && w < HW)                                                         \
            rx[e] = *reinterpret_cast<const float4*>(x + (((long)(n) * HW + h) * HW + w) * C + CIW * cit + 4 * v);         \
    }                                                                                                                      \
    _Pragma("unroll") for (int e = 0; e < DV; ++e)                                                                         \
        rd[e] = *reinterpret_cast<const float4*>(dy + (long)(n) * HW * HW * C + 4 * (long)(tid + e * THREADS));
#define WIDE_STAGE(buf)                                                                                                    \
    {                                                                                                                      \
        float* Xw = lds + (buf) * BUF;                                                                                     \
        float* Dw = Xw + XS;                                                                                               \
        _Pragma("unroll") for (int e = 0; e < XV; ++e) {                                                                   \
            const int idx = tid + e * THREADS;                                                                             \
            if (idx < TW * TW * (CIW / 4)) *reinterpret_cast<float4*>(&Xw[(idx / (CIW / 4)) * LDA + 4 * (idx % (CIW / 4))]) = rx[e]; \
        }                                                                                                                  \
        _Pragma("unroll") for (int e = 0; e < DV; ++e) {                                                                   \
            const int idx = tid + e * THREADS;                                                                             \
            *reinterpret_cast<float4*>(&Dw[(idx / (C / 4)) * LDB + 4 * (idx % (C / 4))]) = rd[e];                          \
        }                                                                                                                  \
    }
    floatx4 M[16];
#pragma unroll
    for (int xi = 0; xi < 16; ++xi) M[xi] = floatx4{0.f, 0.f, 0.f, 0.f};
    WIDE_FETCH(n0)
    for (int i = 0; i < nimg; ++i) {
        WIDE_STAGE(i & 1)
        __syncthreads();
        if (i + 1 < nimg) { WIDE_FETCH(n0 + i + 1) }
        const float* Xs = lds + (i & 1) * BUF;
        const float* Ds = Xs + XS;
        // the image is one run: 4 x 4 tiles of 2x2 pixels
        dfilter_run(M, q,
                    [&](int tile) { return make_int2(2 * (tile / 4), 2 * (tile % 4)); },
                    [&](int2 o, int r, int c) { return Xs[((o.x + r) * TW + o.y + c) * LDA + l16]; },
                    [&](int2 o, int i_, int j) { return Ds[((o.x + i_) * HW + o.y + j) * LDB + 16 * cot + l16]; });
    }
#undef WIDE_FETCH
#undef WIDE_STAGE
    mma::drain();
    floatx4 acc[9];
    dfilter_finish(M, acc);
    float* out = partial + (long)grp * 9 * C * C;
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) out[(t * C + CIW * cit + 4 * q + v) * C + 16 * cot + l16] = acc[t][v];
}

template <int IMGS>
int launch_wgrad_wide(hipStream_t s, const float* x, const float* dy, float* partial, int N, const jobs::TotalsJob& tj) {
    constexpr size_t bytes = (size_t)2 * (10 * 10 * 20 + 8 * 8 * 68) * sizeof(float);
    static_assert(bytes >= jobs::LDS_FLOATS * sizeof(float), "room for a carried job");
    static bool attr_set = false;
    auto kern = wgrad3x3_wide_kernel<IMGS>;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess)
            return -1;
        attr_set = true;
    }
    const int own = (N + IMGS - 1) / IMGS * 4;
    hipLaunchKernelGGL(kern, dim3(own + tj.blocks), dim3(THREADS), bytes, s, x, dy, partial, N, own, tj);
    return DSSPK_LAUNCH_RC();
}

template <int C, int HW, int R>
int launch_wgrad(hipStream_t s, const float* x, const float* dy, float* partial, int N, const jobs::TotalsJob& tj) {
    using K = WCfg<C, HW, R>;
    static_assert(K::LDS_BYTES >= jobs::LDS_FLOATS * sizeof(float), "room for a carried job");
    static bool attr_set = false;
    auto kern = wgrad3x3_kernel<C, HW, R>;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)K::LDS_BYTES) != hipSuccess)
            return -1;
        attr_set = true;
    }
    const int own = N * (HW / R);
    hipLaunchKernelGGL(kern, dim3(own + tj.blocks), dim3(THREADS), K::LDS_BYTES, s, x, dy, partial, own, tj);
    return DSSPK_LAUNCH_RC();
}

}  // namespace

constexpr int WIDE_IMGS = 2;          // images per workgroup of the last stage's d-filter kernel

// Number of partial results the specialised d-filter kernel writes, 0 if the shape is not covered.
int wgrad3x3_tiled_parts(int N, int HW, int C) {
    if (C == 16 && HW == 32) return N * 4;
    if (C == 32 && HW == 16) return N * 2;
    if (C == 64 && HW == 8) return (N + WIDE_IMGS - 1) / WIDE_IMGS;
    return 0;
}

int wgrad3x3_tiled(hipStream_t s, const float* x, const float* dy, float* partial, int N, int HW, int C, const jobs::TotalsJob& tj) {
    if (C == 16 && HW == 32) return launch_wgrad<16, 32, 8>(s, x, dy, partial, N, tj);
    if (C == 32 && HW == 16) return launch_wgrad<32, 16, 8>(s, x, dy, partial, N, tj);
    if (C == 64 && HW == 8) return launch_wgrad_wide<WIDE_IMGS>(s, x, dy, partial, N, tj);
    return -2;
}
