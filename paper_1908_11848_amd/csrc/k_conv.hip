// Convolution forward, gradient w.r.t. the input and gradient w.r.t. the filter, as implicit
// GEMMs on the fp32 matrix cores (the dense contractions of Alg. 1's worker gradient).
//
//   forward : y[pixel][co]  = sum_{tap,ci} x[src(pixel,tap)][ci] * w[tap][ci][co]
//   d-input : dx[pixel][ci] = sum_{tap,co} dy[src'(pixel,tap)][co] * w[tap][ci][co]
//   d-filter: dw[tap][ci][co] = sum_{pixel} x[src(pixel,tap)][ci] * dy[pixel][co]
//
// Activations are [N][H][W][C]: the C values of a pixel are contiguous, so a k-chunk of 16
// channels of one filter tap is one 64-byte run per pixel and neighbouring pixels of an image
// row are neighbouring runs.  A workgroup of 4 wavefronts stages a BM-pixel x 16 slice of the
// gathered operand and the matching 16 x C slice of the filter in LDS (double buffered, next
// slice prefetched into registers while the matrix cores work on the current one).
#include "mma.hpp"
#include "jobs.hpp"
#include "../../include/dssp_kernels.h"

// Specialised 3x3 / stride 1 / Cin = Cout kernels (k_conv3x3.hip); -2 = shape not covered.
int conv3x3_tiled(hipStream_t s, const float* src, const float* w, const float* add, float* dst, float* bn_partial,
                   int N, int HW, int C, bool transposed);
int conv3x3_tiled_stat_parts(int N, int HW, int C);
int conv3x3_tiled_dgrad_post(hipStream_t s, const float* dy, const float* w, const float* add, float* dz,
                              const float* mask_src, const float* xc, const float* stats, float* records, int N, int HW, int C);
int conv3x3_tiled_prebn(hipStream_t s, const float* src, const float* records, int in_parts, const float* gamma,
                         const float* beta, float eps, const float* shortcut, float* act_out, float* stats_out,
                         const float* w, float* dst, float* bn_partial, int N, int HW, int C);
int wgrad3x3_tiled_parts(int N, int HW, int C);
int wgrad3x3_tiled(hipStream_t s, const float* x, const float* dy, float* partial, int N, int HW, int C, const jobs::TotalsJob& tj);
int conv3x3_tiled_dgrad_bn(hipStream_t s, const float* dz, const float* xc, const float* stats, const float* gamma,
                            const float* totals, float* dx_out, const float* w, const float* add, float* out,
                            const float* mask_src, const float* xc_post, const float* stats_post, float* records,
                            const float* red_partial, float* red_dw, int red_E, int red_chunks, int N, int HW, int C);
int conv3x3_tiled_dgrad_bn_wgrad(hipStream_t s, const float* dz, const float* xc, const float* stats, const float* gamma,
                                  const float* totals, const float* w, const float* add, float* out,
                                  const float* xc_post, const float* stats_post, float* records,
                                  const float* x_in, float* partial, const float* red_partial, float* red_dw, int red_E,
                                  int red_chunks, int N, int HW, int C);

namespace {

constexpr int THREADS = 256;

struct ConvGeom {
    int N, OH, OW;      // pixel grid of the GEMM's rows
    int SH, SW;         // spatial size of the gathered tensor
    int IC, OC;         // channels of the gathered tensor (reduction) / of the result (columns)
    int KH, KW, stride, pad;
    long M;             // N * OH * OW
};

// Row m of the GEMM -> (image, output row, output column).  M < 2^31 (checked when the geometry is built), so the
// divisions are 32-bit: a 64-bit division per gathered element costs more than the element's memory traffic.
__device__ __forceinline__ void row_pixel(const ConvGeom& g, long m, int& n, int& oh, int& ow) {
    const unsigned mu = (unsigned)m, W = (unsigned)g.OW, H = (unsigned)g.OH;
    const unsigned r = mu / W;
    ow = (int)(mu - r * W);
    n = (int)(r / H);
    oh = (int)(r - (unsigned)n * H);
}

// Source pixel of row-pixel (oh, ow) for filter tap (kh, kw); false if it falls into the padding
// (forward) or between the strides (d-input).
template <bool DGRAD>
__device__ __forceinline__ bool src_pixel(const ConvGeom& g, int oh, int ow, int kh, int kw, int& sh, int& sw) {
    if constexpr (!DGRAD) {
        sh = oh * g.stride + kh - g.pad;
        sw = ow * g.stride + kw - g.pad;
        return sh >= 0 && sh < g.SH && sw >= 0 && sw < g.SW;
    } else {
        const int hs = oh + g.pad - kh, ws = ow + g.pad - kw;
        if (hs < 0 || ws < 0) return false;
        if (g.stride == 1) { sh = hs; sw = ws; }
        else {
            if ((hs % g.stride) | (ws % g.stride)) return false;
            sh = hs / g.stride; sw = ws / g.stride;
        }
        return sh < g.SH && sw < g.SW;
    }
}

// ---------------------------------------------------------------------------------------------
// forward / d-input.  BM rows (pixels) x BN columns per workgroup, BN = OC (16, 32 or 64; wider
// results take several column tiles).  wavefront w owns rows [w*BM/4, (w+1)*BM/4).
//   DGRAD: gather from dy and use the filter transposed.
//   VEC  : IC is a multiple of 16 (one k-chunk = 16 channels of one tap, 16-byte loads);
//          otherwise the reduction index (tap, ci) is flattened and loaded element-wise.
//   KS   : k-chunks of 16 per LDS stage (VEC only; IC a multiple of 16 * KS).  A stage is one barrier, one round of
//          address arithmetic and one round of global loads, so wide layers take KS = 2: half the barriers and
//          half the vector instructions per MFMA (fp32 MFMA and vector arithmetic do not overlap on this chip).
template <int BM, int BN, bool DGRAD, bool VEC, int KS = 1>
__global__ __launch_bounds__(THREADS) void conv_igemm_kernel(const float* __restrict__ src, const float* __restrict__ wgt,
                                                             const float* __restrict__ bias, const float* __restrict__ add,
                                                             float* __restrict__ dst, ConvGeom g, int relu) {
    static_assert(KS == 1 || VEC, "several k-chunks per stage only with 16-byte gathers");
    constexpr int WM = BM / 64, WN = BN / 16;
    constexpr int KST = mma::KC * KS;                              // reduction indices per stage
    constexpr int LDA = KST + 4;                                   // pitch of a k-contiguous row: 16-byte aligned, 4 (mod 8) quads
    constexpr int LDB = DGRAD ? LDA : BN + 4;
    constexpr int BS = DGRAD ? BN * LDA : KST * (BN + 4);
    constexpr int RPT = BM / 64;                                   // gathered rows per thread (VEC)
    constexpr int BV = KST * BN / 4 / THREADS > 0 ? KST * BN / 4 / THREADS : 1;     // 16-byte filter loads per thread and stage
    extern __shared__ __attribute__((aligned(16))) float igemm_lds[];      // As[2][BM * LDA], then Bs[2][BS]
    float (*As)[BM * LDA] = reinterpret_cast<float (*)[BM * LDA]>(igemm_lds);
    float (*Bs)[BS] = reinterpret_cast<float (*)[BS]>(igemm_lds + 2 * BM * LDA);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long m0 = (long)blockIdx.x * BM;
    const int n0 = blockIdx.y * BN;
    const int taps = g.KH * g.KW;

    floatx4 acc[WM][WN];
    mma::zero(acc);

    // per-thread rows of the gathered tile
    int rn[VEC ? RPT : 1], roh[VEC ? RPT : 1], row_w[VEC ? RPT : 1];
    bool rvalid[VEC ? RPT : 1];
    const int part = tid & 3;                                      // which float4 of the 16-channel chunk
    if constexpr (VEC) {
#pragma unroll
        for (int e = 0; e < RPT; ++e) {
            const long m = m0 + (tid >> 2) + 64 * e;
            rvalid[e] = m < g.M;
            const long mm = rvalid[e] ? m : 0;
            row_pixel(g, mm, rn[e], roh[e], row_w[e]);
        }
    }

    // element-wise gather (!VEC): thread t loads reduction index t % 16 of rows t / 16 + 16 e, the same rows in every chunk
    constexpr int EPT = BM * mma::KC / THREADS;
    int sn[VEC ? 1 : EPT], soh[VEC ? 1 : EPT], sow[VEC ? 1 : EPT];
    if constexpr (!VEC) {
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            const long m = m0 + (tid >> 4) + 16 * e;
            const long mm = m < g.M ? m : 0;
            row_pixel(g, mm, sn[e], soh[e], sow[e]);
            if (m >= g.M) sn[e] = -1;
        }
    }
    float4 ra[VEC ? RPT * KS : 1];
    float ras[VEC ? 1 : BM * mma::KC / THREADS];
    float4 rb[BV];
#pragma unroll
    for (int e = 0; e < BV; ++e) rb[e] = make_float4(0.f, 0.f, 0.f, 0.f);
    const int ktot = taps * g.IC;
    const int nchunks = VEC ? taps * (g.IC / KST) : (ktot + mma::KC - 1) / mma::KC;

    auto load = [&](int chunk) {
        if constexpr (VEC) {
            const int cpt = g.IC / KST;
            const int tap = chunk / cpt, c0 = (chunk - tap * cpt) * KST;
            const int kh = tap / g.KW, kw = tap - kh * g.KW;
#pragma unroll
            for (int e = 0; e < RPT; ++e) {
                int sh, sw;
                const bool ok = rvalid[e] && src_pixel<DGRAD>(g, roh[e], row_w[e], kh, kw, sh, sw);
                const float* sp = src + (((long)rn[e] * g.SH + sh) * g.SW + sw) * g.IC + c0 + 4 * part;
#pragma unroll
                for (int u = 0; u < KS; ++u)
                    ra[e * KS + u] = ok ? *reinterpret_cast<const float4*>(sp + mma::KC * u) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int e = 0; e < BV; ++e) {
                const int idx = tid + e * THREADS;
                if (idx < KST * BN / 4) {
                    if constexpr (!DGRAD) {   // rows k = channel c0+k of this tap, BN columns
                        const int k = idx / (BN / 4), j4 = idx % (BN / 4);
                        rb[e] = *reinterpret_cast<const float4*>(wgt + ((long)tap * g.IC + c0 + k) * g.OC + n0 + 4 * j4);
                    } else {                  // rows j = result channel, KST contiguous reduction channels
                        const int j = idx / (KST / 4), k4 = idx % (KST / 4);
                        rb[e] = *reinterpret_cast<const float4*>(wgt + ((long)tap * g.OC + n0 + j) * g.IC + c0 + 4 * k4);
                    }
                }
            }
        } else {
            const int k0 = chunk * mma::KC;
            const int kk = k0 + (tid & 15);
            const int tap = kk / g.IC, ci = kk - tap * g.IC;
            const int kh = tap / g.KW, kw = tap - kh * g.KW;
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                float v = 0.f;
                int sh, sw;
                if (sn[e] >= 0 && kk < ktot && src_pixel<DGRAD>(g, soh[e], sow[e], kh, kw, sh, sw))
                    v = src[(((long)sn[e] * g.SH + sh) * g.SW + sw) * g.IC + ci];
                ras[e] = v;
            }
            if (tid < 4 * BN) {               // forward only: filter rows are the flattened (tap, ci)
                const int k = tid / (BN / 4), j4 = tid % (BN / 4);
                rb[0] = (k0 + k < ktot) ? *reinterpret_cast<const float4*>(wgt + (long)(k0 + k) * g.OC + n0 + 4 * j4)
                                        : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
    };
    auto store = [&](int buf) {
        if constexpr (VEC) {
#pragma unroll
            for (int e = 0; e < RPT; ++e)
#pragma unroll
                for (int u = 0; u < KS; ++u)
                    *reinterpret_cast<float4*>(&As[buf][((tid >> 2) + 64 * e) * LDA + mma::KC * u + 4 * part]) = ra[e * KS + u];
        } else {
#pragma unroll
            for (int e = 0; e < BM * mma::KC / THREADS; ++e) {
                const int idx = tid + e * THREADS;
                As[buf][(idx / mma::KC) * LDA + idx % mma::KC] = ras[e];
            }
        }
        if constexpr (VEC) {
#pragma unroll
            for (int e = 0; e < BV; ++e) {
                const int idx = tid + e * THREADS;
                if (idx < KST * BN / 4) {
                    if constexpr (!DGRAD) {
                        const int k = idx / (BN / 4), j4 = idx % (BN / 4);
                        *reinterpret_cast<float4*>(&Bs[buf][k * LDB + 4 * j4]) = rb[e];
                    } else {
                        const int j = idx / (KST / 4), k4 = idx % (KST / 4);
                        *reinterpret_cast<float4*>(&Bs[buf][j * LDB + 4 * k4]) = rb[e];
                    }
                }
            }
        } else if (tid < 4 * BN) {
            const int k = tid / (BN / 4), j4 = tid % (BN / 4);
            *reinterpret_cast<float4*>(&Bs[buf][k * LDB + 4 * j4]) = rb[0];
        }
    };

    load(0);
    for (int c = 0; c < nchunks; ++c) {
        const int buf = c & 1;
        store(buf);
        __syncthreads();
        if (c + 1 < nchunks) load(c + 1);
#pragma unroll
        for (int u = 0; u < KS; ++u)
            mma::chunk16<WM, WN, false, DGRAD>(As[buf] + mma::KC * u, LDA, Bs[buf] + (DGRAD ? mma::KC * u : mma::KC * u * LDB), LDB,
                                               wave * (BM / 4), 0, acc, lane);
    }

    mma::drain();
    const int l16 = lane & 15, q = lane >> 4;
#pragma unroll
    for (int wm = 0; wm < WM; ++wm)
#pragma unroll
        for (int wn = 0; wn < WN; ++wn) {
            const int col = n0 + 16 * wn + l16;
            const float bv = bias ? bias[col] : 0.f;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const long m = m0 + wave * (BM / 4) + 16 * wm + 4 * q + v;
                if (m >= g.M) continue;
                float x = acc[wm][wn][v] + bv;
                if (add) x += add[m * g.OC + col];
                if (relu) x = fmaxf(x, 0.f);
                dst[m * g.OC + col] = x;
            }
        }
}

// ---------------------------------------------------------------------------------------------
// d-filter, stage 1.  Workgroup (chunk, tap) reduces `stages` slices of 64 output pixels for one
// filter tap and writes a partial [CIP][COP] block; wavefront w takes pixels [16w, 16w+16) of
// every slice, the four wavefronts' tiles are summed in a fixed order at the end.
//   VEC  : Cin is a multiple of 16, rows of the tile are the channels of tap blockIdx.y.
//   !VEC : rows are the flattened (tap, ci) index (first layer, Cin = 3), blockIdx.y = 0.
// Layers wider than one tile (more than 16 * CI_T input or 16 * CO_T output channels) are cut into channel slices,
// one per blockIdx.z: slice z covers input channels [ci0, ci0 + CIP) (VEC only) and output channels [co0, co0 + COP).
template <int CI_T, int CO_T, bool VEC>
__global__ __launch_bounds__(THREADS) void conv_wgrad_kernel(const float* __restrict__ x, const float* __restrict__ dy,
                                                             float* __restrict__ partial, ConvGeom g, int stages, int rows_total) {
    constexpr int CIP = 16 * CI_T, COP = 16 * CO_T;
    constexpr int LDA = CIP + 4, LDB = COP + 4;
    constexpr int PIX = 64;
    __shared__ __attribute__((aligned(16))) float Xs[PIX * LDA];
    __shared__ __attribute__((aligned(16))) float Ds[PIX * LDB];
    __shared__ __attribute__((aligned(16))) float Red[CIP * COP];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tap = blockIdx.y;
    const int kh = tap / g.KW, kw = tap - kh * g.KW;
    const long p_begin = (long)blockIdx.x * stages * PIX;
    const int ci_slices = VEC ? g.IC / CIP : 1;
    const int ci0 = ((int)blockIdx.z % ci_slices) * CIP, co0 = ((int)blockIdx.z / ci_slices) * COP;

    floatx4 acc[CI_T][CO_T];
    mma::zero(acc);

    for (int st = 0; st < stages; ++st) {
        const long p0 = p_begin + (long)st * PIX;
        if (p0 >= g.M) break;
        __syncthreads();                                            // previous slice fully consumed
        if constexpr (VEC) {
            for (int idx = tid; idx < PIX * (CIP / 4); idx += THREADS) {
                const int pix = idx / (CIP / 4), c4 = idx % (CIP / 4);
                const long m = p0 + pix;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (m < g.M) {
                    int n, oh, ow;
                    row_pixel(g, m, n, oh, ow);
                    int sh, sw;
                    if (src_pixel<false>(g, oh, ow, kh, kw, sh, sw))
                        v = *reinterpret_cast<const float4*>(x + (((long)n * g.SH + sh) * g.SW + sw) * g.IC + ci0 + 4 * c4);
                }
                *reinterpret_cast<float4*>(&Xs[pix * LDA + 4 * c4]) = v;
            }
        } else {
            for (int idx = tid; idx < PIX * CIP; idx += THREADS) {
                const int pix = idx / CIP, kk = idx % CIP;
                const long m = p0 + pix;
                float v = 0.f;
                if (m < g.M && kk < rows_total) {
                    const int t2 = kk / g.IC, ci = kk - t2 * g.IC;
                    const int kh2 = t2 / g.KW, kw2 = t2 - kh2 * g.KW;
                    int n, oh, ow;
                    row_pixel(g, m, n, oh, ow);
                    int sh, sw;
                    if (src_pixel<false>(g, oh, ow, kh2, kw2, sh, sw))
                        v = x[(((long)n * g.SH + sh) * g.SW + sw) * g.IC + ci];
                }
                Xs[pix * LDA + kk] = v;
            }
        }
        for (int idx = tid; idx < PIX * (COP / 4); idx += THREADS) {
            const int pix = idx / (COP / 4), c4 = idx % (COP / 4);
            const long m = p0 + pix;
            const float4 v = m < g.M ? *reinterpret_cast<const float4*>(dy + m * g.OC + co0 + 4 * c4) : make_float4(0.f, 0.f, 0.f, 0.f);
            *reinterpret_cast<float4*>(&Ds[pix * LDB + 4 * c4]) = v;
        }
        __syncthreads();
        mma::chunk16<CI_T, CO_T, true, false>(Xs + 16 * wave * LDA, LDA, Ds + 16 * wave * LDB, LDB, 0, 0, acc, lane);
    }

    mma::drain();
    // ((w0 + w1) + w2) + w3, element by element
    const int l16 = lane & 15, q = lane >> 4;
    for (int w = 0; w < 4; ++w) {
        __syncthreads();
        if (wave == w) {
#pragma unroll
            for (int a = 0; a < CI_T; ++a)
#pragma unroll
                for (int b = 0; b < CO_T; ++b)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int idx = (16 * a + 4 * q + v) * COP + 16 * b + l16;
                        Red[idx] = (w == 0 ? 0.f : Red[idx]) + acc[a][b][v];
                    }
        }
    }
    __syncthreads();
    // partial[chunk][row][co]; VEC: row = tap*Cin + ci, else row = flattened (tap, ci)
    const int rows = VEC ? CIP : rows_total;
    float* out = partial + ((long)blockIdx.x * rows_total + (VEC ? (long)tap * g.IC + ci0 : 0)) * g.OC + co0;
    for (int idx = tid; idx < rows * COP; idx += THREADS) {
        const int rr = idx / COP, co = idx - rr * COP;
        out[(long)rr * g.OC + co] = Red[rr * COP + co];
    }
}

// d-filter, stage 1, for wide layers (at least four 16x16 tiles per tap).  Same work split over
// (pixel chunk, tap) workgroups, but each wavefront owns a block of the Cin x Cout result and walks
// all 64 pixels of every slice (no cross-wavefront sum), and the next slice is prefetched into
// registers while the matrix cores work on the current one (two LDS buffers, one barrier per slice).
template <int CI_T, int CO_T>
__global__ __launch_bounds__(THREADS) void conv_wgrad_tile_kernel(const float* __restrict__ x, const float* __restrict__ dy,
                                                                  float* __restrict__ partial, ConvGeom g, int stages,
                                                                  int own_x, jobs::TotalsJob tj) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    if ((int)blockIdx.x >= own_x) {                 // columns of workgroups behind the kernel's own carry the batch-norm sums job
        const int jb = ((int)blockIdx.x - own_x) * gridDim.y + blockIdx.y;
        if (jb < tj.blocks) jobs::bn_totals(tj, jb, lds);
        return;
    }
    constexpr int CIP = 16 * CI_T, COP = 16 * CO_T;
    constexpr int LDA = CIP + 4, LDB = COP + 4;
    constexpr int PIX = 64;
    constexpr int WR = CI_T >= 2 ? 2 : 1, WC = 4 / WR;           // wavefront grid over the result
    constexpr int TM = CI_T / WR, TN = CO_T / WC;                // tiles per wavefront
    static_assert(CI_T % WR == 0 && CO_T % WC == 0 && TM >= 1 && TN >= 1, "tile split");
    constexpr int XV = PIX * (CIP / 4) / THREADS, DV = PIX * (COP / 4) / THREADS;
    float* Xs = lds;                                   // [2][PIX * LDA]
    float* Ds = lds + 2 * PIX * LDA;                   // [2][PIX * LDB]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tap = blockIdx.y;
    const int kh = tap / g.KW, kw = tap - kh * g.KW;
    const long p_begin = (long)blockIdx.x * stages * PIX;
    int nst = stages;
    if (p_begin + (long)nst * PIX > g.M) nst = (int)((g.M - p_begin + PIX - 1) / PIX);

    floatx4 acc[TM][TN];
    mma::zero(acc);
    float4 rx[XV], rd[DV];
    auto load = [&](int st) {
        const long p0 = p_begin + (long)st * PIX;
#pragma unroll
        for (int e = 0; e < XV; ++e) {
            const int idx = tid + e * THREADS;
            const int pix = idx / (CIP / 4), c4 = idx % (CIP / 4);
            const long m = p0 + pix;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (m < g.M) {
                int n, oh, ow;
                    row_pixel(g, m, n, oh, ow);
                int sh, sw;
                if (src_pixel<false>(g, oh, ow, kh, kw, sh, sw))
                    v = *reinterpret_cast<const float4*>(x + (((long)n * g.SH + sh) * g.SW + sw) * g.IC + 4 * c4);
            }
            rx[e] = v;
        }
#pragma unroll
        for (int e = 0; e < DV; ++e) {
            const int idx = tid + e * THREADS;
            const int pix = idx / (COP / 4), c4 = idx % (COP / 4);
            const long m = p0 + pix;
            rd[e] = m < g.M ? *reinterpret_cast<const float4*>(dy + m * g.OC + 4 * c4) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    auto store = [&](int buf) {
#pragma unroll
        for (int e = 0; e < XV; ++e) {
            const int idx = tid + e * THREADS;
            *reinterpret_cast<float4*>(&Xs[buf * PIX * LDA + (idx / (CIP / 4)) * LDA + 4 * (idx % (CIP / 4))]) = rx[e];
        }
#pragma unroll
        for (int e = 0; e < DV; ++e) {
            const int idx = tid + e * THREADS;
            *reinterpret_cast<float4*>(&Ds[buf * PIX * LDB + (idx / (COP / 4)) * LDB + 4 * (idx % (COP / 4))]) = rd[e];
        }
    };
    const int row0 = 16 * TM * (wave / WC), col0 = 16 * TN * (wave % WC);
    if (nst > 0) load(0);
    for (int st = 0; st < nst; ++st) {
        const int buf = st & 1;
        store(buf);
        __syncthreads();
        if (st + 1 < nst) load(st + 1);
#pragma unroll
        for (int c = 0; c < PIX / 16; ++c)
            mma::chunk16<TM, TN, true, false>(Xs + buf * PIX * LDA + 16 * c * LDA, LDA, Ds + buf * PIX * LDB + 16 * c * LDB, LDB,
                                              row0, col0, acc, lane);
    }
    mma::drain();
    const int l16 = lane & 15, q = lane >> 4;
    float* out = partial + ((long)blockIdx.x * g.KH * g.KW * g.IC + (long)tap * g.IC) * g.OC;
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                out[(row0 + 16 * a + 4 * q + v) * g.OC + col0 + 16 * b + l16] = acc[a][b][v];
}

template <int CI_T, int CO_T>
int launch_wgrad_tile(hipStream_t s, const float* x, const float* dy, float* scratch, const ConvGeom& g, int stages, dim3 grid,
                      const jobs::TotalsJob& tj) {
    constexpr size_t bytes = (size_t)2 * 64 * ((16 * CI_T + 4) + (16 * CO_T + 4)) * sizeof(float);
    static_assert(bytes >= jobs::LDS_FLOATS * sizeof(float), "room for a carried job");
    const int own_x = grid.x;
    grid.x += (tj.blocks + grid.y - 1) / grid.y;
    static bool attr_set = false;
    auto kern = conv_wgrad_tile_kernel<CI_T, CO_T>;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess)
            return -1;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(THREADS), bytes, s, x, dy, scratch, g, stages, own_x, tj);
    return DSSPK_LAUNCH_RC();
}

// d-filter, stage 2 as a kernel of its own: dw[e] = sum over chunks of partial[chunk][e] (jobs::wgrad_reduce).
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(jobs::ReduceJob j) {
    __shared__ __attribute__((aligned(16))) float lds[jobs::LDS_FLOATS];
    jobs::wgrad_reduce(j, blockIdx.x, lds);
}

// Batch-norm backward sums as a kernel of its own (jobs::bn_totals).
__global__ __launch_bounds__(256) void bn_totals_kernel(jobs::TotalsJob j) {
    __shared__ __attribute__((aligned(16))) float lds[jobs::LDS_FLOATS];
    jobs::bn_totals(j, blockIdx.x, lds);
}

int launch_reduce(hipStream_t s, const float* partial, float* dw, int E, int chunks) {
    jobs::ReduceJob j;
    j.partial = partial; j.dw = dw; j.E = E; j.chunks = chunks; j.blocks = jobs::reduce_groups(E, chunks);
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3(j.blocks), dim3(256), 0, s, j);
    return DSSPK_LAUNCH_RC();
}

bool geom(ConvGeom& g, int N, int H, int W, int Cin, int Cout, int KH, int KW, int stride, int pad) {
    if (N < 1 || H < 1 || W < 1 || Cin < 1 || Cout < 1 || KH < 1 || KW < 1 || stride < 1 || pad < 0) return false;
    if (H + 2 * pad < KH || W + 2 * pad < KW) return false;
    g.N = N; g.KH = KH; g.KW = KW; g.stride = stride; g.pad = pad;
    g.SH = H; g.SW = W; g.IC = Cin; g.OC = Cout;
    g.OH = (H + 2 * pad - KH) / stride + 1;
    g.OW = (W + 2 * pad - KW) / stride + 1;
    g.M = (long)N * g.OH * g.OW;
    return g.M < (1L << 31);
}

int wgrad_stages(const ConvGeom& g, int grid_y) {
    // about 288 workgroups; four times as many where the gather is scalar (Cin not a multiple of 16: the loads of a
    // slice are many and narrow, so more of them have to be in flight)
    long s = g.M * grid_y / (64L * (g.IC % 16 ? 1152L : 288L));
    if (s < 1) s = 1;
    if (s > 16) s = 16;
    return (int)s;
}

// LDS of an instantiation (floats), as laid out in the kernel
template <int BM, int BN, bool DGRAD, int KS>
constexpr size_t igemm_lds_bytes() {
    constexpr int KST = mma::KC * KS, LDA = KST + 4;
    return sizeof(float) * 2 * ((size_t)BM * LDA + (DGRAD ? (size_t)BN * LDA : (size_t)KST * (BN + 4)));
}

template <int BM, int BN, bool DGRAD, bool VEC, int KS>
int igemm_launch(dim3 grid, hipStream_t s, const float* src, const float* w, const float* bias, const float* add, float* dst,
                 const ConvGeom& g, int relu) {
    constexpr size_t bytes = igemm_lds_bytes<BM, BN, DGRAD, KS>();
    auto kern = conv_igemm_kernel<BM, BN, DGRAD, VEC, KS>;
    static bool attr_set = false;       // raise the dynamic-LDS limit once per instantiation
    if (!attr_set) {
        if (bytes > 48 * 1024 &&
            hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess)
            return -1;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(THREADS), bytes, s, src, w, bias, add, dst, g, relu);
    return 0;
}

template <bool DGRAD, bool VEC>
int launch_igemm(hipStream_t s, const float* src, const float* w, const float* bias, const float* add, float* dst, const ConvGeom& g, int relu) {
    // output-channel tile: the widest of 64, 32, 16 that divides the layer
    const int bn = g.OC % 64 == 0 ? 64 : g.OC % 32 == 0 ? 32 : g.OC % 16 == 0 ? 16 : 0;
    if (!bn) return -1;
    // small problems take 64-pixel tiles so that the grid still covers the chip
    const bool small = g.M < 128L * 512;
    dim3 grid(ceil_div(g.M, small ? 64 : 128), g.OC / bn);
#define GO(BM, BN) do { if (igemm_launch<BM, BN, DGRAD, VEC, 1>(grid, s, src, w, bias, add, dst, g, relu)) return -1; } while (0)
#define GOK(BM, BN, KS) do { if (igemm_launch<BM, BN, DGRAD, VEC, KS>(grid, s, src, w, bias, add, dst, g, relu)) return -1; } while (0)
    if constexpr (VEC) {
        if (bn == 64 && g.IC % 64 == 0 && small) {      // wide layers: several k-chunks per stage
            GOK(64, 64, 4);
            return DSSPK_LAUNCH_RC();
        }
        if (bn == 64 && g.IC % 32 == 0) {
            if (small) GOK(64, 64, 2); else GOK(128, 64, 2);
            return DSSPK_LAUNCH_RC();
        }
    }
    if (small) { if (bn == 16) GO(64, 16); else if (bn == 32) GO(64, 32); else GO(64, 64); }
    else       { if (bn == 16) GO(128, 16); else if (bn == 32) GO(128, 32); else GO(128, 64); }
#undef GOK
#undef GO
    return DSSPK_LAUNCH_RC();
}

}  // namespace

extern "C" int dsspk_conv_fwd_stat_parts(int N, int H, int W, int Cin, int Cout, int KH, int KW, int stride, int pad) {
    if (KH == 3 && KW == 3 && stride == 1 && pad == 1 && Cin == Cout && H == W) return conv3x3_tiled_stat_parts(N, H, Cin);
    return 0;
}

extern "C" int dsspk_conv_fwd(void* stream, const float* x, const float* w, const float* bias, float* y,
                              int N, int H, int W, int Cin, int Cout, int KH, int KW, int stride, int pad, int relu,
                              float* bn_partial) {
    ConvGeom g;
    if (!x || !w || !y || !geom(g, N, H, W, Cin, Cout, KH, KW, stride, pad)) return -1;
    if (bn_partial && (bias || relu || dsspk_conv_fwd_stat_parts(N, H, W, Cin, Cout, KH, KW, stride, pad) == 0)) return -1;
    if (KH == 3 && KW == 3 && stride == 1 && pad == 1 && Cin == Cout && H == W && !bias && !relu) {
        const int rc = conv3x3_tiled((hipStream_t)stream, x, w, nullptr, y, bn_partial, N, H, Cin, false);
        if (rc != -2) return rc;
    }
    if (Cin % 16 == 0) return launch_igemm<false, true>((hipStream_t)stream, x, w, bias, nullptr, y, g, relu);
    return launch_igemm<false, false>((hipStream_t)stream, x, w, bias, nullptr, y, g, relu);
}

extern "C" int dsspk_conv_fwd_prebn(void* stream, const float* src, const float* records, int in_parts, const float* gamma,
                                    const float* beta, float eps, const float* shortcut, float* act_out, float* stats_out,
                                    const float* w, float* y, float* bn_partial, int N, int H, int C) {
    if (!src || !records || !gamma || !beta || !act_out || !stats_out || !w || !y || N < 1) return -1;
    if (conv3x3_tiled_stat_parts(N, H, C) == 0) return -1;
    const int rc = conv3x3_tiled_prebn((hipStream_t)stream, src, records, in_parts, gamma, beta, eps, shortcut, act_out, stats_out,
                                        w, y, bn_partial, N, H, C);
    return rc == -2 ? -1 : rc;
}

extern "C" int dsspk_conv_bwd_data_post(void* stream, const float* dy, const float* w, const float* add, float* dz,
                                        const float* mask_src, const float* xc, const float* stats, float* records,
                                        int N, int H, int C) {
    if (!dy || !w || !dz || !mask_src || !xc || !stats || !records || N < 1) return -1;
    const int rc = conv3x3_tiled_dgrad_post((hipStream_t)stream, dy, w, add, dz, mask_src, xc, stats, records, N, H, C);
    return rc == -2 ? -1 : rc;
}

extern "C" int dsspk_conv_bwd_data(void* stream, const float* dy, const float* w, const float* add, float* dx,
                                   int N, int H, int W, int Cin, int Cout, int KH, int KW, int stride, int pad) {
    ConvGeom f;
    if (!dy || !w || !dx || !geom(f, N, H, W, Cin, Cout, KH, KW, stride, pad)) return -1;
    if (Cout % 16) return -1;
    if (KH == 3 && KW == 3 && stride == 1 && pad == 1 && Cin == Cout && H == W) {
        const int rc = conv3x3_tiled((hipStream_t)stream, dy, w, add, dx, nullptr, N, H, Cin, true);
        if (rc != -2) return rc;
    }
    ConvGeom g = f;                       // rows: input pixels; gathered tensor: dy
    g.OH = H; g.OW = W; g.SH = f.OH; g.SW = f.OW; g.IC = Cout; g.OC = Cin;
    g.M = (long)N * H * W;
    if (g.M >= (1L << 31)) return -1;
    return launch_igemm<true, true>((hipStream_t)stream, dy, w, nullptr, add, dx, g, 0);
}

extern "C" size_t dsspk_conv_wgrad_scratch_floats(int N, int H, int W, int Cin, int Cout, int KH, int KW, int stride, int pad) {
    ConvGeom g;
    if (!geom(g, N, H, W, Cin, Cout, KH, KW, stride, pad)) return 0;
    const int gy = (Cin % 16 == 0) ? KH * KW : 1;
    const int stages = wgrad_stages(g, gy);
    long chunks = ceil_div(g.M, 64L * stages);
    if (KH == 3 && KW == 3 && stride == 1 && pad == 1 && Cin == Cout && H == W) {
        const long parts = wgrad3x3_tiled_parts(N, H, Cin);
        if (parts > chunks) chunks = parts;
    }
    return (size_t)chunks * KH * KW * Cin * Cout;
}

// Stage 1 of the d-filter convolution: partial[chunk][KH*KW*Cin*Cout] in scratch, *chunks_out chunks.
// tj.blocks > 0 asks the kernel to carry the batch-norm sums job (only the specialised 3x3 and the tile kernels can).
static int wgrad_stage1(hipStream_t s, const float* x, const float* dy, float* scratch, const ConvGeom& g, int N, int H, int W,
                        int Cin, int Cout, int KH, int KW, int stride, int pad, const jobs::TotalsJob& tj, int* chunks_out) {
    if (Cout < 16 || Cout % 16) return -1;
    const bool vec = Cin % 16 == 0;
    const int rows_total = KH * KW * Cin;
    if (KH == 3 && KW == 3 && stride == 1 && pad == 1 && Cin == Cout && H == W) {
        const int parts = wgrad3x3_tiled_parts(N, H, Cin);
        if (parts > 0) {
            *chunks_out = parts;
            return wgrad3x3_tiled(s, x, dy, scratch, N, H, Cin, tj);
        }
    }
    const int gy = vec ? KH * KW : 1;
    const int stages = wgrad_stages(g, gy);
    const int chunks = ceil_div(g.M, 64L * stages);
    *chunks_out = chunks;
    dim3 grid(chunks, gy);
    // channel slices of the widest tile that divides the layer: 64, 32 or 16 channels
    const int cop = Cout % 64 == 0 ? 64 : Cout % 32 == 0 ? 32 : 16;
    const int cip = !vec ? 0 : Cin % 64 == 0 ? 64 : Cin % 32 == 0 ? 32 : 16;
    const bool sliced = Cout > 64 || (vec && Cin > 64);
#define GO(CI, CO, V) hipLaunchKernelGGL((conv_wgrad_kernel<CI, CO, V>), grid, dim3(THREADS), 0, s, x, dy, scratch, g, stages, rows_total)
#define GO_CO(CI, V) do { if (cop == 16) GO(CI, 1, V); else if (cop == 32) GO(CI, 2, V); else GO(CI, 4, V); } while (0)
    if (sliced) {
        if (tj.blocks) return -1;
        grid.z = (unsigned)((Cout / cop) * (vec ? Cin / cip : 1));
    }
    if (!sliced && vec && (Cin / 16) * (Cout / 16) >= 4 && Cout >= 32 && (Cin == 16 || Cin == 32 || Cin == 64)) {
        if (Cin == 64 && Cout == 64) return launch_wgrad_tile<4, 4>(s, x, dy, scratch, g, stages, grid, tj);
        if (Cin == 32 && Cout == 64) return launch_wgrad_tile<2, 4>(s, x, dy, scratch, g, stages, grid, tj);
        if (Cin == 32 && Cout == 32) return launch_wgrad_tile<2, 2>(s, x, dy, scratch, g, stages, grid, tj);
        if (Cin == 64 && Cout == 32) return launch_wgrad_tile<4, 2>(s, x, dy, scratch, g, stages, grid, tj);
        return launch_wgrad_tile<1, 4>(s, x, dy, scratch, g, stages, grid, tj);
    }
    if (tj.blocks) return -1;
    if (vec) {
        if (cip == 16) GO_CO(1, true); else if (cip == 32) GO_CO(2, true); else GO_CO(4, true);
    } else {
        const int tiles = ceil_div(rows_total, 16);
        if (tiles <= 2) GO_CO(2, false); else if (tiles <= 5) GO_CO(5, false); else return -1;
    }
#undef GO_CO
#undef GO
    return DSSPK_LAUNCH_RC();
}

extern "C" int dsspk_conv_bwd_weight(void* stream, const float* x, const float* dy, float* dw, float* scratch,
                                     int N, int H, int W, int Cin, int Cout, int KH, int KW, int stride, int pad) {
    ConvGeom g;
    if (!x || !dy || !dw || !scratch || !geom(g, N, H, W, Cin, Cout, KH, KW, stride, pad)) return -1;
    int chunks = 0;
    const int rc = wgrad_stage1((hipStream_t)stream, x, dy, scratch, g, N, H, W, Cin, Cout, KH, KW, stride, pad, jobs::TotalsJob(), &chunks);
    if (rc) return rc;
    return launch_reduce((hipStream_t)stream, scratch, dw, KH * KW * Cin * Cout, chunks);
}

static bool totals_job(jobs::TotalsJob& tj, const float* records, int G, int C, float* totals, float* dgamma, float* dbeta) {
    tj = jobs::TotalsJob();
    if (!records) return true;
    if (!totals || !dgamma || !dbeta || G < 1 || C < 4 || C % 4) return false;
    tj.records = records; tj.G = G; tj.C = C; tj.totals = totals; tj.dgamma = dgamma; tj.dbeta = dbeta; tj.blocks = C / 4;
    return true;
}

extern "C" int dsspk_conv_bwd_weight_parts(void* stream, const float* x, const float* dy, float* scratch,
                                           int N, int H, int W, int Cin, int Cout, int KH, int KW, int stride, int pad,
                                           const float* records, int G, int C, float* totals, float* dgamma, float* dbeta,
                                           int* chunks_out) {
    ConvGeom g;
    jobs::TotalsJob tj;
    if (!x || !dy || !scratch || !chunks_out || !geom(g, N, H, W, Cin, Cout, KH, KW, stride, pad)) return -1;
    if (!totals_job(tj, records, G, C, totals, dgamma, dbeta)) return -1;
    return wgrad_stage1((hipStream_t)stream, x, dy, scratch, g, N, H, W, Cin, Cout, KH, KW, stride, pad, tj, chunks_out);
}

extern "C" int dsspk_wgrad_reduce(void* stream, const float* partial, float* dw, int E, int chunks) {
    if (!partial || !dw || E < 4 || E % 4 || chunks < 1) return -1;
    return launch_reduce((hipStream_t)stream, partial, dw, E, chunks);
}

extern "C" int dsspk_bn_bwd_totals(void* stream, const float* records, int G, int C, float* totals, float* dgamma, float* dbeta) {
    jobs::TotalsJob tj;
    if (!records || !totals_job(tj, records, G, C, totals, dgamma, dbeta)) return -1;
    hipLaunchKernelGGL(bn_totals_kernel, dim3(tj.blocks), dim3(256), 0, (hipStream_t)stream, tj);
    return DSSPK_LAUNCH_RC();
}

extern "C" int dsspk_conv_bwd_data_bn(void* stream, const float* dz, const float* xc, const float* stats, const float* gamma,
                                      const float* totals, float* dx, const float* w, const float* add, float* out,
                                      const float* mask_src, const float* xc_post, const float* stats_post, float* records,
                                      const float* red_partial, float* red_dw, int red_E, int red_chunks, int N, int H, int C) {
    if (!dz || !xc || !stats || !gamma || !totals || !dx || !w || !out || !mask_src || !xc_post || !stats_post || !records || N < 1)
        return -1;
    if (out == dz || dx == dz || dx == out) return -1;
    if (red_partial && (!red_dw || red_E < 4 || red_E % 4 || red_chunks < 1)) return -1;
    const int rc = conv3x3_tiled_dgrad_bn((hipStream_t)stream, dz, xc, stats, gamma, totals, dx, w, add, out, mask_src, xc_post,
                                           stats_post, records, red_partial, red_dw, red_E, red_chunks, N, H, C);
    return rc == -2 ? -1 : rc;
}

extern "C" int dsspk_conv_bwd_fused_chunks(int N, int H, int C) {
    if ((C == 16 && H == 32) || (C == 32 && H == 16)) return wgrad3x3_tiled_parts(N, H, C);
    return 0;
}

extern "C" int dsspk_conv_bwd_data_bn_wgrad(void* stream, const float* dz, const float* xc, const float* stats, const float* gamma,
                                            const float* totals, const float* w, const float* add, float* out,
                                            const float* xc_post, const float* stats_post, float* records,
                                            const float* x_in, float* partial, const float* red_partial, float* red_dw,
                                            int red_E, int red_chunks, int N, int H, int C) {
    if (!dz || !xc || !stats || !gamma || !totals || !w || !out || !xc_post || !stats_post || !records || !x_in ||
        !partial || N < 1)
        return -1;
    if (out == dz || partial == red_partial) return -1;
    if (red_partial && (!red_dw || red_E < 4 || red_E % 4 || red_chunks < 1)) return -1;
    if (dsspk_conv_bwd_fused_chunks(N, H, C) == 0) return -1;
    const int rc = conv3x3_tiled_dgrad_bn_wgrad((hipStream_t)stream, dz, xc, stats, gamma, totals, w, add, out, xc_post,
                                                 stats_post, records, x_in, partial, red_partial, red_dw, red_E, red_chunks, N, H, C);
    return rc == -2 ? -1 : rc;
}
