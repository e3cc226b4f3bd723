/* Oracle, part 2a: fp64 layer forward / backward, written as the defining sums.
 *
 * TEST INFRASTRUCTURE ONLY.  Used by the tests, the smoke check and the
 * benchmark's CPU-baseline leg; never by the product path.  Shares nothing
 * with the HIP library.
 *
 * The worker's gradient is the mean over the mini-batch of the per-sample
 * loss gradients (Alg. 1, worker step 4); the loss is softmax cross-entropy
 * of the network output.  Each function below is one layer's definition (or
 * the chain rule applied to it), as plain loops, all in double precision.
 *
 * Layouts: activations are [N][H][W][C] (channels last), convolution filters
 * [KH][KW][Cin][Cout], fully connected weights [in][out].
 *
 * OpenMP is used only across independent outputs (each output element is
 * produced by exactly one thread, with its own fixed summation order), so
 * results do not depend on the thread count.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#define IDX4(n, h, w, c, H, W, C) ((((size_t)(n) * (H) + (h)) * (W) + (w)) * (C) + (c))

/* y[n,ho,wo,co] = b[co] + sum_{kh,kw,ci} x[n, ho*s+kh-p, wo*s+kw-p, ci] * w[kh,kw,ci,co]
 * (cross-correlation, zero padding).  b may be NULL. */
void conv2d_fwd(const double* x, const double* w, const double* b, double* y,
                int N, int H, int W, int Cin, int Cout, int KH, int KW, int stride, int pad)
{
    const int Ho = (H + 2 * pad - KH) / stride + 1, Wo = (W + 2 * pad - KW) / stride + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int ho = 0; ho < Ho; ++ho)
            for (int wo = 0; wo < Wo; ++wo) {
                double* yo = y + IDX4(n, ho, wo, 0, Ho, Wo, Cout);
                for (int co = 0; co < Cout; ++co) yo[co] = b ? b[co] : 0.0;
                for (int kh = 0; kh < KH; ++kh) {
                    const int hi = ho * stride + kh - pad;
                    if (hi < 0 || hi >= H) continue;
                    for (int kw = 0; kw < KW; ++kw) {
                        const int wi = wo * stride + kw - pad;
                        if (wi < 0 || wi >= W) continue;
                        const double* xi = x + IDX4(n, hi, wi, 0, H, W, Cin);
                        const double* wk = w + ((size_t)(kh * KW + kw) * Cin) * Cout;
                        for (int ci = 0; ci < Cin; ++ci) {
                            const double xv = xi[ci];
                            for (int co = 0; co < Cout; ++co) yo[co] += xv * wk[(size_t)ci * Cout + co];
                        }
                    }
                }
            }
}

/* dx[n,hi,wi,ci] = sum over every (ho,wo,kh,kw,co) whose input tap is (hi,wi):
 *                  dy[n,ho,wo,co] * w[kh,kw,ci,co]. */
void conv2d_bwd_data(const double* w, const double* dy, double* dx,
                     int N, int H, int W, int Cin, int Cout, int KH, int KW, int stride, int pad)
{
    const int Ho = (H + 2 * pad - KH) / stride + 1, Wo = (W + 2 * pad - KW) / stride + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int hi = 0; hi < H; ++hi)
            for (int wi = 0; wi < W; ++wi) {
                double* dxi = dx + IDX4(n, hi, wi, 0, H, W, Cin);
                for (int ci = 0; ci < Cin; ++ci) dxi[ci] = 0.0;
                for (int kh = 0; kh < KH; ++kh) {
                    const int hs = hi + pad - kh;
                    if (hs < 0 || hs % stride) continue;
                    const int ho = hs / stride;
                    if (ho >= Ho) continue;
                    for (int kw = 0; kw < KW; ++kw) {
                        const int ws = wi + pad - kw;
                        if (ws < 0 || ws % stride) continue;
                        const int wo = ws / stride;
                        if (wo >= Wo) continue;
                        const double* dyo = dy + IDX4(n, ho, wo, 0, Ho, Wo, Cout);
                        const double* wk = w + ((size_t)(kh * KW + kw) * Cin) * Cout;
                        for (int ci = 0; ci < Cin; ++ci) {
                            double acc = 0.0;
                            for (int co = 0; co < Cout; ++co) acc += dyo[co] * wk[(size_t)ci * Cout + co];
                            dxi[ci] += acc;
                        }
                    }
                }
            }
}

/* dw[kh,kw,ci,co] = sum_{n,ho,wo} x[n, ho*s+kh-p, wo*s+kw-p, ci] * dy[n,ho,wo,co]
 * db[co]          = sum_{n,ho,wo} dy[n,ho,wo,co]            (db may be NULL) */
void conv2d_bwd_weight(const double* x, const double* dy, double* dw, double* db,
                       int N, int H, int W, int Cin, int Cout, int KH, int KW, int stride, int pad)
{
    const int Ho = (H + 2 * pad - KH) / stride + 1, Wo = (W + 2 * pad - KW) / stride + 1;
#pragma omp parallel for collapse(3) schedule(static)
    for (int kh = 0; kh < KH; ++kh)
        for (int kw = 0; kw < KW; ++kw)
            for (int ci = 0; ci < Cin; ++ci) {
                double* dwo = dw + ((size_t)(kh * KW + kw) * Cin + ci) * Cout;
                for (int co = 0; co < Cout; ++co) dwo[co] = 0.0;
                for (int n = 0; n < N; ++n)
                    for (int ho = 0; ho < Ho; ++ho) {
                        const int hi = ho * stride + kh - pad;
                        if (hi < 0 || hi >= H) continue;
                        for (int wo = 0; wo < Wo; ++wo) {
                            const int wi = wo * stride + kw - pad;
                            if (wi < 0 || wi >= W) continue;
                            const double xv = x[IDX4(n, hi, wi, ci, H, W, Cin)];
                            const double* dyo = dy + IDX4(n, ho, wo, 0, Ho, Wo, Cout);
                            for (int co = 0; co < Cout; ++co) dwo[co] += xv * dyo[co];
                        }
                    }
            }
    if (db) {
#pragma omp parallel for schedule(static)
        for (int co = 0; co < Cout; ++co) {
            double acc = 0.0;
            for (size_t i = 0; i < (size_t)N * Ho * Wo; ++i) acc += dy[i * Cout + co];
            db[co] = acc;
        }
    }
}

/* y[i,o] = b[o] + sum_k x[i,k] * w[k,o] */
void fc_fwd(const double* x, const double* w, const double* b, double* y, int m, int in, int out)
{
#pragma omp parallel for schedule(static)
    for (int i = 0; i < m; ++i) {
        double* yo = y + (size_t)i * out;
        for (int o = 0; o < out; ++o) yo[o] = b ? b[o] : 0.0;
        for (int k = 0; k < in; ++k) {
            const double xv = x[(size_t)i * in + k];
            const double* wk = w + (size_t)k * out;
            for (int o = 0; o < out; ++o) yo[o] += xv * wk[o];
        }
    }
}

/* dx[i,k] = sum_o dy[i,o] w[k,o];  dw[k,o] = sum_i x[i,k] dy[i,o];  db[o] = sum_i dy[i,o] */
void fc_bwd(const double* x, const double* w, const double* dy, double* dx, double* dw, double* db,
            int m, int in, int out)
{
    if (dx) {
#pragma omp parallel for schedule(static)
        for (int i = 0; i < m; ++i)
            for (int k = 0; k < in; ++k) {
                double acc = 0.0;
                for (int o = 0; o < out; ++o) acc += dy[(size_t)i * out + o] * w[(size_t)k * out + o];
                dx[(size_t)i * in + k] = acc;
            }
    }
#pragma omp parallel for schedule(static)
    for (int k = 0; k < in; ++k) {
        double* dwo = dw + (size_t)k * out;
        for (int o = 0; o < out; ++o) dwo[o] = 0.0;
        for (int i = 0; i < m; ++i) {
            const double xv = x[(size_t)i * in + k];
            for (int o = 0; o < out; ++o) dwo[o] += xv * dy[(size_t)i * out + o];
        }
    }
    if (db)
        for (int o = 0; o < out; ++o) {
            double acc = 0.0;
            for (int i = 0; i < m; ++i) acc += dy[(size_t)i * out + o];
            db[o] = acc;
        }
}

/* ReLU.  active[i] in: -1 = decide here (z > 0), 0 / 1 = forced by the caller
 * (a tie-break; the Python wrapper only allows it where |z| is below its
 * ambiguity threshold).  out: the decision taken (0 / 1). */
void relu_fwd(const double* z, double* a, int8_t* active, size_t n)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
        int on = active[i] < 0 ? (z[i] > 0.0) : active[i];
        active[i] = (int8_t)on;
        a[i] = on ? (z[i] > 0.0 ? z[i] : 0.0) : 0.0;
    }
}

void relu_bwd(const double* da, const int8_t* active, double* dz, size_t n)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) dz[i] = active[i] ? da[i] : 0.0;
}

/* Max pooling k x k, stride s, no padding, floor:  Ho = (H-k)/s + 1.
 * arg[n,ho,wo,c] in: -1 = decide here (first maximum in (kh,kw) scan order),
 * otherwise a forced window position kh*k+kw (tie-break, validated by the
 * wrapper).  out: the position taken.  gap[...] = max - runner-up (the margin
 * of the decision; +inf for a 1-element window). */
void maxpool_fwd(const double* x, double* y, int32_t* arg, double* gap,
                 int N, int H, int W, int C, int k, int s)
{
    const int Ho = (H - k) / s + 1, Wo = (W - k) / s + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int ho = 0; ho < Ho; ++ho)
            for (int wo = 0; wo < Wo; ++wo)
                for (int c = 0; c < C; ++c) {
                    double best = -INFINITY, second = -INFINITY;
                    int bi = 0;
                    for (int kh = 0; kh < k; ++kh)
                        for (int kw = 0; kw < k; ++kw) {
                            const double v = x[IDX4(n, ho * s + kh, wo * s + kw, c, H, W, C)];
                            if (v > best) { second = best; best = v; bi = kh * k + kw; }
                            else if (v > second) second = v;
                        }
                    const size_t o = IDX4(n, ho, wo, c, Ho, Wo, C);
                    gap[o] = best - second;
                    if (arg[o] >= 0) bi = arg[o];
                    arg[o] = bi;
                    y[o] = x[IDX4(n, ho * s + bi / k, wo * s + bi % k, c, H, W, C)];
                }
}

void maxpool_bwd(const double* dy, const int32_t* arg, double* dx,
                 int N, int H, int W, int C, int k, int s)
{
    const int Ho = (H - k) / s + 1, Wo = (W - k) / s + 1;
    for (size_t i = 0; i < (size_t)N * H * W * C; ++i) dx[i] = 0.0;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)   /* windows of one image only touch that image */
        for (int ho = 0; ho < Ho; ++ho)
            for (int wo = 0; wo < Wo; ++wo)
                for (int c = 0; c < C; ++c) {
                    const size_t o = IDX4(n, ho, wo, c, Ho, Wo, C);
                    const int bi = arg[o];
                    dx[IDX4(n, ho * s + bi / k, wo * s + bi % k, c, H, W, C)] += dy[o];
                }
}

/* Batch normalisation, training mode, over the M = N*H*W rows of x[M][C]:
 * mean_c = (1/M) sum x, var_c = (1/M) sum (x - mean)^2 (biased),
 * xhat = (x - mean) / sqrt(var + eps),  y = gamma * xhat + beta. */
void bn_fwd(const double* x, const double* gamma, const double* beta, double* y,
            double* mean, double* invstd, size_t M, int C, double eps)
{
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        double s = 0.0;
        for (size_t i = 0; i < M; ++i) s += x[i * C + c];
        const double mu = s / (double)M;
        double v = 0.0;
        for (size_t i = 0; i < M; ++i) { const double d = x[i * C + c] - mu; v += d * d; }
        mean[c] = mu;
        invstd[c] = 1.0 / sqrt(v / (double)M + eps);
    }
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < M; ++i)
        for (int c = 0; c < C; ++c)
            y[i * C + c] = gamma[c] * (x[i * C + c] - mean[c]) * invstd[c] + beta[c];
}

/* Chain rule through the definition above (mean and var depend on x):
 * dbeta = sum dy, dgamma = sum dy*xhat,
 * dx = gamma*invstd * (dy - dbeta/M - xhat*dgamma/M). */
void bn_bwd(const double* x, const double* gamma, const double* mean, const double* invstd,
            const double* dy, double* dx, double* dgamma, double* dbeta, size_t M, int C)
{
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        double sb = 0.0, sg = 0.0;
        for (size_t i = 0; i < M; ++i) {
            const double xh = (x[i * C + c] - mean[c]) * invstd[c];
            sb += dy[i * C + c];
            sg += dy[i * C + c] * xh;
        }
        dbeta[c] = sb;
        dgamma[c] = sg;
    }
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < M; ++i)
        for (int c = 0; c < C; ++c) {
            const double xh = (x[i * C + c] - mean[c]) * invstd[c];
            dx[i * C + c] = gamma[c] * invstd[c] *
                            (dy[i * C + c] - dbeta[c] / (double)M - xh * dgamma[c] / (double)M);
        }
}

/* Global average pooling: y[n,c] = mean over (h,w) of x[n,h,w,c]. */
void gap_fwd(const double* x, double* y, int N, int HW, int C)
{
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            double s = 0.0;
            for (int i = 0; i < HW; ++i) s += x[((size_t)n * HW + i) * C + c];
            y[(size_t)n * C + c] = s / (double)HW;
        }
}

void gap_bwd(const double* dy, double* dx, int N, int HW, int C)
{
    for (int n = 0; n < N; ++n)
        for (int i = 0; i < HW; ++i)
            for (int c = 0; c < C; ++c)
                dx[((size_t)n * HW + i) * C + c] = dy[(size_t)n * C + c] / (double)HW;
}

/* Parameter-free shortcut for a block that halves the resolution and widens
 * the channels: y[n,ho,wo,c] = x[n,2ho,2wo,c] for c < Cin, 0 for c >= Cin. */
void shortcut_pad_fwd(const double* x, double* y, int N, int H, int W, int Cin, int Cout)
{
    const int Ho = (H + 1) / 2, Wo = (W + 1) / 2;
    for (int n = 0; n < N; ++n)
        for (int ho = 0; ho < Ho; ++ho)
            for (int wo = 0; wo < Wo; ++wo)
                for (int c = 0; c < Cout; ++c)
                    y[IDX4(n, ho, wo, c, Ho, Wo, Cout)] =
                        c < Cin ? x[IDX4(n, 2 * ho, 2 * wo, c, H, W, Cin)] : 0.0;
}

/* dx += transpose of the map above applied to dy. */
void shortcut_pad_bwd_acc(const double* dy, double* dx, int N, int H, int W, int Cin, int Cout)
{
    const int Ho = (H + 1) / 2, Wo = (W + 1) / 2;
    for (int n = 0; n < N; ++n)
        for (int ho = 0; ho < Ho; ++ho)
            for (int wo = 0; wo < Wo; ++wo)
                for (int c = 0; c < Cin; ++c)
                    dx[IDX4(n, 2 * ho, 2 * wo, c, H, W, Cin)] += dy[IDX4(n, ho, wo, c, Ho, Wo, Cout)];
}

/* loss = (1/m) sum_i [ log sum_j exp(z_ij) - z_{i,y_i} ]  (max subtracted first);
 * dz_ij = (softmax(z_i)_j - [j == y_i]) / m. */
double softmax_xent(const double* z, const int32_t* label, double* dz, int m, int C)
{
    double loss = 0.0;
    for (int i = 0; i < m; ++i) {
        const double* zi = z + (size_t)i * C;
        double mx = zi[0];
        for (int j = 1; j < C; ++j) if (zi[j] > mx) mx = zi[j];
        double se = 0.0;
        for (int j = 0; j < C; ++j) se += exp(zi[j] - mx);
        loss += log(se) + mx - zi[label[i]];
        for (int j = 0; j < C; ++j)
            dz[(size_t)i * C + j] = (exp(zi[j] - mx) / se - (j == label[i] ? 1.0 : 0.0)) / (double)m;
    }
    return loss / (double)m;
}
