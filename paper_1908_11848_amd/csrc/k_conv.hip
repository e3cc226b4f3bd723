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
constexpr int IGEMM_IMG_MAX = 2048;                 // floats of the staged input rows (element-wise forward gather)
constexpr int IGEMM_STAGED = 1, IGEMM_PARITY = 2;   // gather modes of conv_igemm_kernel

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
        else if (g.stride == 2) {                      // the usual down-sampling stride: no division per gathered row
            if ((hs | ws) & 1) return false;
            sh = hs >> 1; sw = ws >> 1;
        } else {
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
                                                             float* __restrict__ dst, ConvGeom g, int relu, int mode) {
    static_assert(KS == 1 || VEC, "several k-chunks per stage only with 16-byte gathers");
    constexpr int WM = BM / 64, WN = BN / 16;
    constexpr int KST = mma::KC * KS;                              // reduction indices per stage
    constexpr int LDA = KST + 4;                                   // pitch of a k-contiguous row: 16-byte aligned, 4 (mod 8) quads
    constexpr int LDB = DGRAD ? LDA : BN + 4;
    constexpr int BS = DGRAD ? BN * LDA : KST * (BN + 4);
    constexpr int RPT = BM / 64;                                   // gathered rows per thread (VEC)
    constexpr int BV = KST * BN / 4 / THREADS > 0 ? KST * BN / 4 / THREADS : 1;     // 16-byte filter loads per thread and stage
    extern __shared__ __attribute__((aligned(16))) float igemm_lds[];      // As[2][BM * LDA], then Bs[2][BS], then the staged rows
    float (*As)[BM * LDA] = reinterpret_cast<float (*)[BM * LDA]>(igemm_lds);
    float (*Bs)[BS] = reinterpret_cast<float (*)[BS]>(igemm_lds + 2 * BM * LDA);
    const float* Img = igemm_lds + 2 * BM * LDA + 2 * BS;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bool staged = !VEC && mode == IGEMM_STAGED;
    const int n0 = blockIdx.y * BN;
    const int taps = g.KH * g.KW;
    // IGEMM_PARITY (d-input of a stride-2 layer, even H and W): the rows are ordered by the parity class (h % 2, w % 2) of
    // the pixel, a workgroup's rows are of one class, and it walks only the taps that reach a dy pixel from that class
    // (kh = (h + pad) mod 2, +2, ...): a quarter of the (pixel, tap) pairs, the others would multiply zeros.
    const bool parity = DGRAD && mode == IGEMM_PARITY;
    long m0 = (long)blockIdx.x * BM, Mrows = g.M;
    ConvGeom gr = g;                                               // pixel grid the rows are decomposed on
    int ph = 0, pw = 0, kh0 = 0, kw0 = 0, nkw = g.KW, ntaps = taps;
    if (parity) {
        const int tiles = gridDim.x >> 2, cls = blockIdx.x / tiles;
        m0 = (long)(blockIdx.x - cls * tiles) * BM;
        ph = cls >> 1; pw = cls & 1;
        kh0 = (ph + g.pad) & 1; kw0 = (pw + g.pad) & 1;
        nkw = (g.KW - kw0 + 1) >> 1;
        ntaps = ((g.KH - kh0 + 1) >> 1) * nkw;
        gr.OH = g.OH >> 1; gr.OW = g.OW >> 1;
        Mrows = (long)g.N * gr.OH * gr.OW;
    }

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
            rvalid[e] = m < Mrows;
            const long mm = rvalid[e] ? m : 0;
            row_pixel(gr, mm, rn[e], roh[e], row_w[e]);
            if (parity) { roh[e] = 2 * roh[e] + ph; row_w[e] = 2 * row_w[e] + pw; }
        }
    }

    // element-wise gather (!VEC): thread t loads reduction index t % 16 of rows t / 16 + 16 e, the same rows in every chunk.
    // staged (forward, stride 1, the tile is whole rows of one image): the input rows the tile touches are copied to LDS
    // with their zero padding once, in coalesced loads, and every chunk gathers from that copy; sow[] then holds the
    // offset of the row's pixel in the copy.
    constexpr int EPT = BM * mma::KC / THREADS;
    int sn[VEC ? 1 : EPT], soh[VEC ? 1 : EPT], sow[VEC ? 1 : EPT];
    const int twi = g.SW + 2 * g.pad;
    if constexpr (!VEC) {
        if (staged) {
            const unsigned per_image = (unsigned)(g.OH * g.OW);
            const unsigned n = (unsigned)m0 / per_image;
            const int oh0 = (int)(((unsigned)m0 - n * per_image) / (unsigned)g.OW);
            const float* xin = src + (long)n * g.SH * g.SW * g.IC;
            const int row_len = twi * g.IC, img_rows = BM / g.OW + g.KH - 1;
            float* img = igemm_lds + 2 * BM * LDA + 2 * BS;
            for (int idx = tid; idx < img_rows * row_len; idx += THREADS) {
                const int r = idx / row_len, rest = idx - r * row_len;
                const int sh = oh0 - g.pad + r, col = rest - g.pad * g.IC;       // col = sw * IC + ci
                img[idx] = (sh >= 0 && sh < g.SH && col >= 0 && col < g.SW * g.IC) ? xin[((long)sh * g.SW) * g.IC + col] : 0.f;
            }
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                const int pix = (tid >> 4) + 16 * e;
                const int r = pix / g.OW, c = pix - r * g.OW;
                sn[e] = 0; soh[e] = 0;
                sow[e] = (r * twi + c) * g.IC;
            }
            __syncthreads();
        } else {
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                const long m = m0 + (tid >> 4) + 16 * e;
                const long mm = m < g.M ? m : 0;
                row_pixel(g, mm, sn[e], soh[e], sow[e]);
                if (m >= g.M) sn[e] = -1;
            }
        }
    }
    float4 ra[VEC ? RPT * KS : 1];
    float ras[VEC ? 1 : BM * mma::KC / THREADS];
    float4 rb[BV];
#pragma unroll
    for (int e = 0; e < BV; ++e) rb[e] = make_float4(0.f, 0.f, 0.f, 0.f);
    const int ktot = taps * g.IC;
    const int nchunks = VEC ? ntaps * (g.IC / KST) : (ktot + mma::KC - 1) / mma::KC;

    auto load = [&](int chunk) {
        if constexpr (VEC) {
            const int cpt = g.IC / KST;
            const int tap_i = chunk / cpt, c0 = (chunk - tap_i * cpt) * KST;
            int kh, kw;
            if (parity) { const int ikh = tap_i / nkw; kh = kh0 + 2 * ikh; kw = kw0 + 2 * (tap_i - ikh * nkw); }
            else { kh = tap_i / g.KW; kw = tap_i - kh * g.KW; }
            const int tap = kh * g.KW + kw;
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
            if (staged) {
                const int tap_off = (kh * twi + kw) * g.IC + ci;
#pragma unroll
                for (int e = 0; e < EPT; ++e) ras[e] = kk < ktot ? Img[sow[e] + tap_off] : 0.f;
            } else {
#pragma unroll
                for (int e = 0; e < EPT; ++e) {
                    float v = 0.f;
                    int sh, sw;
                    if (sn[e] >= 0 && kk < ktot && src_pixel<DGRAD>(g, soh[e], sow[e], kh, kw, sh, sw))
                        v = src[(((long)sn[e] * g.SH + sh) * g.SW + sw) * g.IC + ci];
                    ras[e] = v;
                }
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

    if (nchunks > 0) load(0);          // a parity class that no tap reaches has no chunk at all: its rows are zero (+ add)
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
                const long r = m0 + wave * (BM / 4) + 16 * wm + 4 * q + v;
                if (r >= Mrows) continue;
                long m = r;
                if (parity) {
                    int pn, phh, pww;
                    row_pixel(gr, r, pn, phh, pww);
                    m = ((long)pn * g.OH + 2 * phh + ph) * g.OW + 2 * pww + pw;
                }
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
//   IMG  : (!VEC, stride 1, a slice is whole rows of one image) the input rows a slice touches are staged in LDS with their
//          zero padding first, in coalesced loads, and the (pixel, tap, ci) operand is gathered from that copy through
//          offsets each thread works out once: the element-wise gather from global memory costs far more than the MFMAs.
constexpr int WGRAD_IMG_MAX = 2048;                 // floats of the staged input rows
template <int CI_T, int CO_T, bool VEC, bool IMG = false>
__global__ __launch_bounds__(THREADS) void conv_wgrad_kernel(const float* __restrict__ x, const float* __restrict__ dy,
                                                             float* __restrict__ partial, ConvGeom g, int stages, int rows_total) {
    static_assert(!(VEC && IMG), "staged rows serve the element-wise gather only");
    constexpr int CIP = 16 * CI_T, COP = 16 * CO_T;
    constexpr int LDA = CIP + 4, LDB = COP + 4;
    constexpr int PIX = 64;
    static_assert(CIP * COP <= PIX * LDA, "the cross-wavefront sum reuses the operand tile");
    __shared__ __attribute__((aligned(16))) float Xs[PIX * LDA];
    __shared__ __attribute__((aligned(16))) float Ds[PIX * LDB];
    __shared__ __attribute__((aligned(16))) float Img[IMG ? WGRAD_IMG_MAX : 4];
    float* Red = Xs;                                                // used after the last slice has been consumed
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tap = blockIdx.y;
    const int kh = tap / g.KW, kw = tap - kh * g.KW;
    const long p_begin = (long)blockIdx.x * stages * PIX;
    const int ci_slices = VEC ? g.IC / CIP : 1;
    const int ci0 = ((int)blockIdx.z % ci_slices) * CIP, co0 = ((int)blockIdx.z / ci_slices) * COP;

    floatx4 acc[CI_T][CO_T];
    mma::zero(acc);

    // IMG: the staged copy holds rows [oh0 - pad, oh0 + PIX / OW + KH - 1 - pad) of the image, TWI = SW + 2 pad columns each
    constexpr int EPT = PIX * CIP / THREADS;
    int img_off[IMG ? EPT : 1];
    const int twi = g.SW + 2 * g.pad, row_len = twi * g.IC, img_rows = PIX / g.OW + g.KH - 1;
    if constexpr (IMG) {
        // offset of (tap, ci) within the copy, one division pair per reduction index; OW is a power of two here
        int* tap_off = reinterpret_cast<int*>(Ds);
        if (tid < CIP) {
            const int t2 = tid / g.IC, ci = tid - t2 * g.IC;
            const int kh2 = t2 / g.KW, kw2 = t2 - kh2 * g.KW;
            tap_off[tid] = tid < rows_total ? (kh2 * twi + kw2) * g.IC + ci : -1;
        }
        __syncthreads();
        const int lw = __ffs(g.OW) - 1;
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            const int idx = tid + e * THREADS;
            const int pix = idx / CIP, kk = idx % CIP;
            const int t = tap_off[kk];
            img_off[e] = t >= 0 ? t + ((pix >> lw) * twi + (pix & (g.OW - 1))) * g.IC : -1;
        }
    }

    if constexpr (IMG) {
        // global -> registers -> LDS, the next slice's loads in flight while the matrix cores work on the current one
        constexpr int IV = WGRAD_IMG_MAX / THREADS, DV = PIX * (COP / 4) / THREADS;
        static_assert(DV >= 1 && THREADS % (COP / 4) == 0, "dy rows per thread");
        int img_rc[IV];                                             // (row << 16 | position in the row) of the thread's staged elements
#pragma unroll
        for (int e = 0; e < IV; ++e) {
            const int idx = tid + e * THREADS;
            const int r = idx / row_len;
            img_rc[e] = idx < img_rows * row_len ? (r << 16) | (idx - r * row_len) : -1;
        }
        float ri[IV];
        float4 rd[DV];
        auto fetch = [&](long p0) {
            const unsigned per_image = (unsigned)(g.OH * g.OW);
            const unsigned n = (unsigned)p0 / per_image;
            const int oh0 = (int)(((unsigned)p0 - n * per_image) / (unsigned)g.OW);
            const float* xin = x + (long)n * g.SH * g.SW * g.IC;
#pragma unroll
            for (int e = 0; e < IV; ++e) {
                const int sh = oh0 - g.pad + (img_rc[e] >> 16), col = (img_rc[e] & 0xffff) - g.pad * g.IC;     // col = sw * IC + ci
                ri[e] = (img_rc[e] >= 0 && sh >= 0 && sh < g.SH && col >= 0 && col < g.SW * g.IC) ? xin[sh * g.SW * g.IC + col] : 0.f;
            }
#pragma unroll
            for (int e = 0; e < DV; ++e) {
                const int idx = tid + e * THREADS;
                rd[e] = *reinterpret_cast<const float4*>(dy + (p0 + idx / (COP / 4)) * g.OC + co0 + 4 * (idx % (COP / 4)));   // M is a multiple of PIX here
            }
        };
        int nst = stages;
        if (p_begin + (long)nst * PIX > g.M) nst = p_begin < g.M ? (int)((g.M - p_begin) / PIX) : 0;
        if (nst > 0) fetch(p_begin);
        for (int st = 0; st < nst; ++st) {
            __syncthreads();                                        // previous slice fully consumed
#pragma unroll
            for (int e = 0; e < IV; ++e)
                if (img_rc[e] >= 0) Img[tid + e * THREADS] = ri[e];
#pragma unroll
            for (int e = 0; e < DV; ++e) {
                const int idx = tid + e * THREADS;
                *reinterpret_cast<float4*>(&Ds[(idx / (COP / 4)) * LDB + 4 * (idx % (COP / 4))]) = rd[e];
            }
            __syncthreads();                                        // staged rows complete
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                const int idx = tid + e * THREADS;
                Xs[(idx / CIP) * LDA + idx % CIP] = img_off[e] >= 0 ? Img[img_off[e]] : 0.f;
            }
            if (st + 1 < nst) fetch(p_begin + (long)(st + 1) * PIX);
            __syncthreads();
            mma::chunk16<CI_T, CO_T, true, false>(Xs + 16 * wave * LDA, LDA, Ds + 16 * wave * LDB, LDB, 0, 0, acc, lane);
        }
    } else
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
    // The pixels a thread gathers move on by PIX from slice to slice: (image, row, column) are decomposed once and then
    // stepped with carries, since a division per gathered row and slice costs as many cycles as the slice's MFMAs.
    int pn[XV], poh[XV], pw[XV];
#pragma unroll
    for (int e = 0; e < XV; ++e) row_pixel(g, p_begin + (tid + e * THREADS) / (CIP / 4), pn[e], poh[e], pw[e]);
    int step_n, step_h, step_w;
    row_pixel(g, PIX, step_n, step_h, step_w);
    long dy_row = p_begin + tid / (COP / 4);                       // first of the thread's dy rows; the others follow at THREADS / (COP / 4)
    auto load = [&](int) {
#pragma unroll
        for (int e = 0; e < XV; ++e) {
            const int c4 = (tid + e * THREADS) % (CIP / 4);
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            int sh, sw;
            if (pn[e] < g.N && src_pixel<false>(g, poh[e], pw[e], kh, kw, sh, sw))
                v = *reinterpret_cast<const float4*>(x + (long)((pn[e] * g.SH + sh) * g.SW + sw) * g.IC + 4 * c4);
            rx[e] = v;
            pw[e] += step_w;
            if (pw[e] >= g.OW) { pw[e] -= g.OW; ++poh[e]; }
            poh[e] += step_h;
            if (poh[e] >= g.OH) { poh[e] -= g.OH; ++pn[e]; }
            pn[e] += step_n;
        }
#pragma unroll
        for (int e = 0; e < DV; ++e) {
            const long m = dy_row + e * (THREADS / (COP / 4));
            const int c4 = tid % (COP / 4);
            rd[e] = m < g.M ? *reinterpret_cast<const float4*>(dy + m * g.OC + 4 * c4) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        dy_row += PIX;
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
    return g.M < (1L << 31) && (long)N * H * W < (1L << 31);      // pixel indices are 32-bit in the kernels
}

// d-filter, element-wise gather: 64-pixel slices are whole rows of one image and the rows they touch fit the staged copy
bool wgrad_staged(const ConvGeom& g) {
    return g.IC % 16 != 0 && g.stride == 1 && g.OW <= 64 && 64 % g.OW == 0 && ((long)g.OH * g.OW) % 64 == 0 &&
           (long)(64 / g.OW + g.KH - 1) * (g.SW + 2 * g.pad) * g.IC <= WGRAD_IMG_MAX;
}

// d-filter: layers of at least four 16x16 tiles per tap go to conv_wgrad_tile_kernel
bool wgrad_tiled(const ConvGeom& g) {
    const int Cin = g.IC, Cout = g.OC;
    return (Cout == 64 && (Cin == 16 || Cin == 32 || Cin == 64)) || (Cout == 32 && (Cin == 32 || Cin == 64));     // its instantiations
}

// Slices of 64 pixels per workgroup.
int wgrad_stages(const ConvGeom& g, int grid_y) {
    const long slices = (g.M + 63) / 64;
    long s;
    if (wgrad_tiled(g)) {
        // the tile kernel overlaps a slice's loads with the previous slice's MFMAs and LDS lets two workgroups share a CU:
        // at most one round of 512 workgroups, however many slices that takes (a second, partly filled round costs a fifth)
        long chunks = 512L / grid_y;
        if (chunks < 1) chunks = 1;
        s = (slices + chunks - 1) / chunks;
    } else {
        // the plain kernel does not overlap them, so several workgroups per compute unit have to: about 1152 workgroups,
        // half as many with the staged gather, whose set-up per workgroup costs more
        s = slices * grid_y / (wgrad_staged(g) ? 576L : 1152L);
        if (s > 16) s = 16;
    }
    return (int)(s < 1 ? 1 : s);
}


// LDS of an instantiation's operand tiles (bytes), as laid out in the kernel
template <int BM, int BN, bool DGRAD, int KS>
constexpr size_t igemm_lds_bytes() {
    constexpr int KST = mma::KC * KS, LDA = KST + 4;
    return sizeof(float) * 2 * ((size_t)BM * LDA + (DGRAD ? (size_t)BN * LDA : (size_t)KST * (BN + 4)));
}

template <int BM, int BN, bool DGRAD, bool VEC, int KS>
int igemm_launch(dim3 grid, hipStream_t s, const float* src, const float* w, const float* bias, const float* add, float* dst,
                 const ConvGeom& g, int relu, bool parity) {
    // staged gather: forward, element-wise, stride 1, tiles of whole rows of one image, the rows they touch within the LDS budget
    const bool staged = !VEC && !DGRAD && g.stride == 1 && g.OW <= BM && BM % g.OW == 0 && ((long)g.OH * g.OW) % BM == 0 &&
                        (long)(BM / g.OW + g.KH - 1) * (g.SW + 2 * g.pad) * g.IC <= IGEMM_IMG_MAX;
    const size_t bytes = igemm_lds_bytes<BM, BN, DGRAD, KS>() + (staged ? sizeof(float) * IGEMM_IMG_MAX : 0);
    auto kern = conv_igemm_kernel<BM, BN, DGRAD, VEC, KS>;
    static bool attr_set = false;       // raise the dynamic-LDS limit once per instantiation
    if (!attr_set) {
        constexpr size_t most = igemm_lds_bytes<BM, BN, DGRAD, KS>() + (VEC ? 0 : sizeof(float) * IGEMM_IMG_MAX);
        if (most > 48 * 1024 &&
            hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)most) != hipSuccess)
            return -1;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(THREADS), bytes, s, src, w, bias, add, dst, g, relu, staged ? IGEMM_STAGED : parity ? IGEMM_PARITY : 0);
    return 0;
}

template <bool DGRAD, bool VEC>
int launch_igemm(hipStream_t s, const float* src, const float* w, const float* bias, const float* add, float* dst, const ConvGeom& g, int relu) {
    // output-channel tile: the widest of 64, 32, 16 that divides the layer
    const int bn = g.OC % 64 == 0 ? 64 : g.OC % 32 == 0 ? 32 : g.OC % 16 == 0 ? 16 : 0;
    if (!bn) return -1;
    // small problems take 64-pixel tiles so that the grid still covers the chip
    const bool small = g.M < 128L * 512;
    // d-input of a stride-2 layer on an even pixel grid: four parity classes of rows, each with its own tiles
    const bool parity = DGRAD && VEC && g.stride == 2 && g.OH % 2 == 0 && g.OW % 2 == 0;
    dim3 grid(parity ? 4 * ceil_div(g.M / 4, small ? 64 : 128) : ceil_div(g.M, small ? 64 : 128), g.OC / bn);
#define GO(BM, BN) do { if (igemm_launch<BM, BN, DGRAD, VEC, 1>(grid, s, src, w, bias, add, dst, g, relu, parity)) return -1; } while (0)
#define GOK(BM, BN, KS) do { if (igemm_launch<BM, BN, DGRAD, VEC, KS>(grid, s, src, w, bias, add, dst, g, relu, parity)) return -1; } while (0)
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
    // element-wise layers whose 64-pixel slices are whole rows of one image gather from a staged copy of those rows
    const bool img = wgrad_staged(g);
    const int gy = vec ? KH * KW : 1;
    const int stages = wgrad_stages(g, gy);
    const int chunks = ceil_div(g.M, 64L * stages);
    *chunks_out = chunks;
    dim3 grid(chunks, gy);
    // channel slices of the widest tile that divides the layer: 64, 32 or 16 channels
    const int cop = Cout % 64 == 0 ? 64 : Cout % 32 == 0 ? 32 : 16;
    const int cip = !vec ? 0 : Cin % 64 == 0 ? 64 : Cin % 32 == 0 ? 32 : 16;
    const bool sliced = !wgrad_tiled(g) && (Cout > cop || (vec && Cin > cip));
#define GO(CI, CO, V) do { if (!V && img) hipLaunchKernelGGL((conv_wgrad_kernel<CI, CO, V, !V>), grid, dim3(THREADS), 0, s, x, dy, scratch, g, stages, rows_total); \
                           else hipLaunchKernelGGL((conv_wgrad_kernel<CI, CO, V, false>), grid, dim3(THREADS), 0, s, x, dy, scratch, g, stages, rows_total); } while (0)
#define GO_CO(CI, V) do { if (cop == 16) GO(CI, 1, V); else if (cop == 32) GO(CI, 2, V); else GO(CI, 4, V); } while (0)
    if (sliced) {
        if (tj.blocks) return -1;
        grid.z = (unsigned)((Cout / cop) * (vec ? Cin / cip : 1));
    }
    if (wgrad_tiled(g)) {
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
