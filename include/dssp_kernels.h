/* Raw kernel launchers of libdssp (layer L0): one extern "C" function per kernel family,
 * plain device pointers and sizes, a hipStream_t passed as void*.  They enqueue and return
 * the HIP error code of the launch (0 = success, -1 = shape not supported).  The library's
 * own worker step is built from exactly these; they are exported so that each kernel can be
 * checked on its own.  Every operation is a step of Alg. 1: the worker's mini-batch gradient
 * (worker step 4) or the server's weight update (server step 2) / the worker's pull (worker
 * steps 2-3).
 *
 * Layouts: activations [N][H][W][C] fp32, filters [KH][KW][Cin][Cout], FC weights [in][out].
 */
#ifndef DSSP_KERNELS_H
#define DSSP_KERNELS_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

/* Server step 2: w[i] -= scale * g[i], i < n; *stamp_dev = version. */
int dsspk_apply(void* stream, float* w_dev, const float* g_dev, int64_t n, float scale,
                uint64_t* stamp_dev, uint64_t version);
/* Worker steps 2-3: dst[i] = w[i]; *dst_stamp_dev = *stamp_dev. */
int dsspk_pull(void* stream, float* dst_dev, const float* w_dev, int64_t n,
               uint64_t* dst_stamp_dev, const uint64_t* stamp_dev);
/* apply and pull in one pass (16 B/param): w -= scale * g, the new w also written to dst_dev, both stamps = version.
 * Results are bit-identical to dsspk_apply followed by dsspk_pull.  dst_stamp_dev may be NULL. */
int dsspk_apply_pull(void* stream, float* w_dev, const float* g_dev, float* dst_dev, int64_t n, float scale,
                     uint64_t* stamp_dev, uint64_t* dst_stamp_dev, uint64_t version);
/* Server step 2 for m pushes that arrived at the same time ("aggregated before updating"), in one pass over w:
 *   w_j = w_{j-1} - scale * g[j-1], j = 1..m (w_0 = w on entry), w = w_m on return, *stamp_dev = version_first + m - 1,
 * bit-identical to m calls of dsspk_apply in that order.  Snapshot d (d < n_dst) receives w_{dst_after[d]} - the
 * weights after that many gradients - and *dst_stamp_dev[d] = version_first + dst_after[d] - 1, as dsspk_pull would
 * have copied between two of the single applies.  g, dst, dst_after, dst_stamp_dev are HOST arrays (of device
 * pointers / ints); dst_after must be ascending, in [1, m]; the snapshots must be distinct buffers other than w;
 * dst_stamp_dev or any entry of it may be NULL.  m <= DSSPK_APPLY_MANY_MAX, n_dst <= DSSPK_APPLY_MANY_MAX_DST (-1 beyond). */
#define DSSPK_APPLY_MANY_MAX 16
#define DSSPK_APPLY_MANY_MAX_DST 32
int dsspk_apply_many(void* stream, float* w_dev, int m, const float* const* g_dev, int64_t n, float scale, int n_dst,
                     float* const* dst_dev, const int* dst_after, uint64_t* const* dst_stamp_dev, uint64_t* stamp_dev,
                     uint64_t version_first);

/* C[M][N] = op(A)[M][K] * op(B)[K][N] (+ bias[N]) (ReLU if relu).  Element (i,k) of op(A) is
 * A[i*a_rs + k*a_cs], element (k,j) of op(B) is B[k*b_rs + j*b_cs]; C is row-major with
 * leading dimension ldc.  bias_dev may be NULL. */
int dsspk_gemm(void* stream, const float* A_dev, long a_rs, long a_cs, const float* B_dev, long b_rs, long b_cs,
               float* C_dev, long ldc, int M, int N, int K, const float* bias_dev, int relu);
/* The same product with the reduction index K split over `layers` layers of workgroups, for products with few
 * output tiles and a long K (the forward pass of a wide fully connected layer at a small batch would otherwise
 * occupy a dozen compute units): every layer writes its partial product to scratch_dev ([layers][M][N] floats), a
 * second kernel adds the layers in order and applies bias / ReLU.  dsspk_gemm_splitk_layers proposes the number of
 * layers (1: the plain kernel is used and scratch_dev may be NULL). */
int dsspk_gemm_splitk_layers(int M, int N, int K);
int dsspk_gemm_splitk(void* stream, const float* A_dev, long a_rs, long a_cs, const float* B_dev, long b_rs, long b_cs,
                      float* C_dev, long ldc, int M, int N, int K, const float* bias_dev, int relu,
                      float* scratch_dev, int layers);
/* out[j] = sum_i X[i][j], X is [M][N] row-major.  Fixed summation order (row slabs, then the slabs). */
int dsspk_colsum(void* stream, const float* X_dev, float* out_dev, float* scratch_dev, long M, int N);
/* Floats of scratch_dev dsspk_colsum needs for an [M][N] matrix (0 for short matrices: scratch_dev may be NULL). */
size_t dsspk_colsum_scratch_floats(long M, int N);
/* dsspk_colsum for callers that cannot allocate device memory or bring a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  The slab sums go to a fixed buffer that is part of the
 * library image on every GPU (DSSPK_COLSUM_NOALLOC_MAX_N * 256 floats = 4 MiB, held until the process ends); the call
 * allocates and frees nothing and gives the same bits as dsspk_colsum.  X_dev and out_dev are the caller's, as above.
 * Returns 0, -1 (null pointer, M < 1 or N < 1), DSSPK_NOALLOC_ETOOBIG (N > DSSPK_COLSUM_NOALLOC_MAX_N: the matrix has
 * more columns than the fixed buffer holds slab sums for; use dsspk_colsum with a workspace) or DSSPK_NOALLOC_EHIP (the
 * buffer's address could not be resolved on the current device), else the HIP error code of the launch.
 * All calls on one GPU share that GPU's buffer: calls that overlap in time on one GPU (different streams) race; calls on
 * one stream, or otherwise ordered, are safe.  Nothing needs clearing between calls (every slab sum read was written
 * by the same call). */
#define DSSPK_COLSUM_NOALLOC_MAX_N 4096
#define DSSPK_NOALLOC_ETOOBIG (-2)
#define DSSPK_NOALLOC_EHIP (-3)
int dsspk_colsum_noalloc(void* stream, const float* X_dev, float* out_dev, long M, int N);

/* Convolution (cross-correlation, zero padding), implicit GEMM on fp32 MFMA.
 * Ho = (H + 2*pad - KH)/stride + 1.  bias_dev may be NULL; relu applies max(.,0) to the output.
 * bn_partial_dev (may be NULL): the kernel also writes, per workgroup tile, the mean and the sum of
 * squared deviations of every output channel (dsspk_conv_fwd_stat_parts(...) records of
 * N*Ho*Wo / parts rows each, the layout dsspk_bn_fwd merges when given conv_parts); only for shapes
 * where dsspk_conv_fwd_stat_parts(...) > 0, without bias / relu. */
int dsspk_conv_fwd(void* stream, const float* x_dev, const float* w_dev, const float* bias_dev, float* y_dev,
                   int N, int H, int W, int Cin, int Cout, int KH, int KW, int stride, int pad, int relu,
                   float* bn_partial_dev);
int dsspk_conv_fwd_stat_parts(int N, int H, int W, int Cin, int Cout, int KH, int KW, int stride, int pad);
/* 3x3 / stride 1 / pad 1 / C -> C convolution of a = ReLU(BN(src) (+ shortcut)) without a separate batch-norm
 * pass: the kernel normalises src while loading it.  src is [N][H][H][C]; records_dev holds in_parts statistics
 * records of src as written by dsspk_conv_fwd(..., bn_partial_dev) for the same shape; shortcut_dev (may be
 * NULL) has src's shape.  Side outputs: act_out_dev = a, stats_out_dev = mean[C], invstd[C] (what dsspk_bn_fwd
 * would have produced).  bn_partial_dev (may be NULL): statistics records of y, which must not be the buffer
 * records_dev points to.  Only shapes with dsspk_conv_fwd_stat_parts(...) > 0; returns -1 otherwise. */
int dsspk_conv_fwd_prebn(void* stream, const float* src_dev, const float* records_dev, int in_parts,
                         const float* gamma_dev, const float* beta_dev, float eps, const float* shortcut_dev,
                         float* act_out_dev, float* stats_out_dev, const float* w_dev, float* y_dev,
                         float* bn_partial_dev, int N, int H, int C);
/* dx = transpose of the above applied to dy (gradient w.r.t. the input), plus add_dev element-wise if it
 * is not NULL (the gradient arriving through a residual shortcut; add_dev has dx's shape, may not alias dx). */
int dsspk_conv_bwd_data(void* stream, const float* dy_dev, const float* w_dev, const float* add_dev, float* dx_dev,
                        int N, int H, int W, int Cin, int Cout, int KH, int KW, int stride, int pad);
/* 3x3 / stride 1 / pad 1 / C -> C only (shapes with dsspk_conv_fwd_stat_parts > 0, -1 otherwise): d-input as
 * above, then in the same kernel the first half of the backward pass of the ReLU + batch norm whose output fed
 * this convolution: dz = (dx + add) * [mask_src > 0] is what is stored to dz_dev, and per tile and channel
 * (sum dz, sum dz * xhat), xhat = (xc - mean) * invstd with mean / invstd from stats_dev, go to records_dev
 * (dsspk_conv_fwd_stat_parts(...) records; consumed by dsspk_bn_bwd_dx with conv_parts).  mask_src_dev: the
 * saved post-ReLU activation, xc_dev: that batch norm's input; both have dx's shape. */
int dsspk_conv_bwd_data_post(void* stream, const float* dy_dev, const float* w_dev, const float* add_dev, float* dz_dev,
                             const float* mask_src_dev, const float* xc_dev, const float* stats_dev, float* records_dev,
                             int N, int H, int C);
/* dsspk_conv_bwd_data_post with the batch norm that PRECEDES it in the backward direction folded into its loader:
 * the convolution runs on
 *   dx = gamma * invstd * (dz - totals[c] / M - xhat * totals[C + c] / M),  xhat = (xc - mean) * invstd,  M = N*H*H,
 * computed from dz_dev (masked gradient at that batch norm's output), xc_dev (its input), stats_dev (its
 * mean[C], invstd[C]), gamma_dev and totals_dev (sum dz [C], sum dz * xhat [C], see dsspk_bn_bwd_totals); dx is
 * also stored to dx_dev for the d-filter convolution.  The epilogue is that of dsspk_conv_bwd_data_post
 * (mask_src_dev, xc_post_dev, stats_post_dev, records_dev); out_dev may be add_dev itself (in place) but
 * neither dz_dev nor dx_dev.  red_partial_dev != NULL: the kernel also carries the second stage of an earlier
 * d-filter convolution, red_dw_dev[e] = sum over red_chunks of red_partial_dev[chunk][e], e < red_E (as extra
 * workgroups, result identical to dsspk_wgrad_reduce). */
int dsspk_conv_bwd_data_bn(void* stream, const float* dz_dev, const float* xc_dev, const float* stats_dev,
                           const float* gamma_dev, const float* totals_dev, float* dx_dev, const float* w_dev,
                           const float* add_dev, float* out_dev, const float* mask_src_dev, const float* xc_post_dev,
                           const float* stats_post_dev, float* records_dev, const float* red_partial_dev,
                           float* red_dw_dev, int red_E, int red_chunks, int N, int H, int C);
/* dsspk_conv_bwd_data_bn and stage 1 of the d-filter convolution of the same layer in ONE kernel: dx is used from
 * LDS for both and never stored.  x_in_dev: the convolution's input [N][H][H][C], a post-ReLU activation, which is
 * also the source of the epilogue's ReLU mask (there is no separate mask_src_dev); partial_dev receives
 * dsspk_conv_bwd_fused_chunks(N, H, C) partial results of 9*C*C floats (to be summed by dsspk_wgrad_reduce or a
 * later call's red_* job; must not be the buffer red_partial_dev points to).  Only where
 * dsspk_conv_bwd_fused_chunks(...) > 0 (C = 16 at 32x32, C = 32 at 16x16), -1 otherwise. */
int dsspk_conv_bwd_data_bn_wgrad(void* stream, const float* dz_dev, const float* xc_dev, const float* stats_dev,
                                 const float* gamma_dev, const float* totals_dev, const float* w_dev,
                                 const float* add_dev, float* out_dev,
                                 const float* xc_post_dev, const float* stats_post_dev, float* records_dev,
                                 const float* x_in_dev, float* partial_dev, const float* red_partial_dev,
                                 float* red_dw_dev, int red_E, int red_chunks, int N, int H, int C);
int dsspk_conv_bwd_fused_chunks(int N, int H, int C);
/* dw[kh][kw][ci][co] = sum over batch and output pixels of x * dy.  Two stages (partial sums per
 * pixel chunk, then a fixed-order reduction).  scratch_dev: dsspk_conv_wgrad_scratch_floats(...) floats. */
int dsspk_conv_bwd_weight(void* stream, const float* x_dev, const float* dy_dev, float* dw_dev, float* scratch_dev,
                          int N, int H, int W, int Cin, int Cout, int KH, int KW, int stride, int pad);
/* The two stages of dsspk_conv_bwd_weight on their own.  Stage 1 leaves *chunks_out (host memory) partial
 * results of KH*KW*Cin*Cout floats each in scratch_dev; stage 2 sums them in a fixed order.  With records_dev
 * != NULL stage 1 also carries, as extra workgroups, the sums dsspk_bn_bwd_totals computes (3x3 / stride 1 /
 * Cin = Cout in {16, 32, 64} shapes only, -1 otherwise). */
int dsspk_conv_bwd_weight_parts(void* stream, const float* x_dev, const float* dy_dev, float* scratch_dev,
                                int N, int H, int W, int Cin, int Cout, int KH, int KW, int stride, int pad,
                                const float* records_dev, int G, int C, float* totals_dev, float* dgamma_dev,
                                float* dbeta_dev, int* chunks_out);
int dsspk_wgrad_reduce(void* stream, const float* partial_dev, float* dw_dev, int E, int chunks);
size_t dsspk_conv_wgrad_scratch_floats(int N, int H, int W, int Cin, int Cout, int KH, int KW, int stride, int pad);

/* dy[i] = a[i] > 0 ? dy[i] : 0 (in place). */
int dsspk_relu_bwd(void* stream, float* dy_dev, const float* a_dev, long n);
/* out[i] += in[i]. */
int dsspk_add(void* stream, float* out_dev, const float* in_dev, long n);

/* Max pooling 3x3 stride 2, no padding, floor.  arg: chosen window position kh*3+kw (first
 * maximum in scan order). */
int dsspk_maxpool_fwd(void* stream, const float* x_dev, float* y_dev, uint8_t* arg_dev, int N, int H, int W, int C);
int dsspk_maxpool_bwd(void* stream, const float* dy_dev, const uint8_t* arg_dev, float* dx_dev, int N, int H, int W, int C);
/* dsspk_maxpool_bwd followed by the backward pass of the ReLU in front of the pooling, in one kernel:
 * dx = a > 0 ? (gathered gradient) : 0, a_dev = the pooling's input (post-ReLU, dx's shape); a_dev == NULL: no mask. */
int dsspk_maxpool_bwd_relu(void* stream, const float* dy_dev, const uint8_t* arg_dev, const float* a_dev, float* dx_dev,
                           int N, int H, int W, int C);

/* Batch normalisation over the M rows of x[M][C], batch statistics, biased variance, eps inside
 * the root.  stats: mean[C] then invstd[C] (written by fwd, read by bwd).
 * fwd: y = gamma*(x-mean)*invstd + beta (+ shortcut) (ReLU if relu).
 *   shortcut_mode 0: none; 1: sc_dev has y's shape; 2: sc_dev is [N][2Ho][2Wo][C/2], subsampled by
 *   2 in h and w, channels >= C/2 read as zero (Ho, Wo, N given by sc_n, sc_ho, sc_wo).
 * conv_parts > 0: scratch_dev already holds that many statistics records written by dsspk_conv_fwd
 *   (the pass over x that computes them is skipped); 0: they are computed here.
 * scratch_dev: dsspk_bn_scratch_floats(M, C) floats (per-slab partial results; one buffer serves one stream at a time). */
int dsspk_bn_fwd(void* stream, const float* x_dev, const float* gamma_dev, const float* beta_dev, float* y_dev,
                 float* stats_dev, float* scratch_dev, long M, int C, float eps, int relu,
                 int shortcut_mode, const float* sc_dev, int sc_n, int sc_ho, int sc_wo, int conv_parts);
/* Backward of ReLU(BN(x) [+ shortcut]) w.r.t. x, gamma, beta.
 *   da_dev    gradient w.r.t. the (post-ReLU) output; overwritten IN PLACE by dz = da * [out > 0]
 *             when out_dev != NULL (out_dev = the saved forward output), left as is otherwise
 *   dx_dev    gamma*invstd*(dz - mean(dz) - xhat*mean(dz*xhat)) */
int dsspk_bn_bwd(void* stream, const float* x_dev, const float* gamma_dev, const float* stats_dev,
                 float* da_dev, const float* out_dev, float* dx_dev, float* dgamma_dev, float* dbeta_dev,
                 float* scratch_dev, long M, int C);
/* The two kernels of dsspk_bn_bwd on their own: the per-slab sums (and the ReLU mask written into da), then dx. */
int dsspk_bn_bwd_reduce(void* stream, const float* x_dev, const float* stats_dev, float* da_dev, const float* out_dev,
                        float* scratch_dev, long M, int C);
/* conv_parts > 0: scratch_dev holds that many (sum dz, sum dz*xhat) records written by dsspk_conv_bwd_data_post. */
int dsspk_bn_bwd_dx(void* stream, const float* x_dev, const float* gamma_dev, const float* stats_dev, const float* dz_dev,
                    float* dx_dev, float* dgamma_dev, float* dbeta_dev, const float* scratch_dev, long M, int C, int conv_parts);
/* Sums of G records of C channels, records_dev[(g * C + c) * 2 + {0, 1}] = (sum dz, sum dz * xhat) of one tile
 * as written by dsspk_conv_bwd_data_post / _bn:  totals_dev[c] = dbeta_dev[c] = sum dz,
 * totals_dev[C + c] = dgamma_dev[c] = sum dz * xhat.  C a multiple of 4; fixed summation order. */
int dsspk_bn_bwd_totals(void* stream, const float* records_dev, int G, int C, float* totals_dev, float* dgamma_dev,
                        float* dbeta_dev);
size_t dsspk_bn_scratch_floats(long M, int C);

/* dx[n][2ho][2wo][c] += dy[n][ho][wo][c] for c < C/2 (transpose of shortcut_mode 2). */
int dsspk_shortcut_bwd_acc(void* stream, const float* dy_dev, float* dx_dev, int N, int Ho, int Wo, int C);

/* y[n][c] = mean over hw of x[n][hw][c];  dx[n][hw][c] = dy[n][c] / HW. */
int dsspk_gap_fwd(void* stream, const float* x_dev, float* y_dev, int N, int HW, int C);
int dsspk_gap_bwd(void* stream, const float* dy_dev, float* dx_dev, int N, int HW, int C);

/* loss = mean_i(logsumexp(z_i) - z_i[y_i]); dz = (softmax(z) - onehot(y)) / m.  loss_dev may be NULL.
 * m <= 1024, C <= 1024. */
int dsspk_softmax_xent(void* stream, const float* z_dev, const int32_t* y_dev, float* dz_dev, float* loss_dev, int m, int C);

/* Device-side time (the push timestamps of Alg. 2 as real times; a slower worker of Sec. V-C's unequal cluster).
 * Ticks are those of the GPU's constant-rate wall clock (hipDeviceAttributeWallClockRate, in kHz).
 * dsspk_clock_stamp: a one-lane kernel stores the current tick to out_a and out_b (either may be NULL, not both).
 * dsspk_clock_stretch: a one-lane kernel reads *start_dev (a tick stored earlier on the same stream), notes the tick
 * it starts at (arrival: everything enqueued before it has finished) and holds the stream until
 * clock - start >= permille / 1000 * (arrival - start), but never longer than max_extra_ticks and never more than about
 * 0.2 s (a bounded number of sleeps); permille <= 1000 does not wait.  arrival_out / left_out (either may be NULL, not
 * both) receive the tick of arrival and the tick at which it left.  The out pointers may be device memory or pinned
 * host memory (stores are system-scope releases). */
int dsspk_clock_khz(void);      /* ticks per millisecond of the current device's wall clock; -1 on failure */
int dsspk_clock_stamp(void* stream, uint64_t* out_a, uint64_t* out_b);
int dsspk_clock_stretch(void* stream, const uint64_t* start_dev, int permille, uint64_t max_extra_ticks,
                        uint64_t* arrival_out, uint64_t* left_out);

#ifdef __cplusplus
}
#endif
#endif
