/*
 * CPU oracle, layer arithmetic -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct definitions of the layers that make up a block function
 * f_k(h_k; x_k) of the paper's problem statement (Section 2, Eq. (1)) and of the
 * vector-Jacobian products the chain rule of Eq. (2) needs.  The paper does not restate
 * these textbook layers; each routine below is the definition written out as loops:
 * fp64, NCHW, no blocking, no fusion.  OpenMP splits only the outermost independent loop,
 * so every sum is taken in one fixed order whatever the thread count.
 *
 * Nothing in the product path may link or call this file.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#define IDX4(n, c, h, w, C, H, W) ((((size_t)(n) * (C) + (c)) * (H) + (h)) * (W) + (w))

static int out_dim(int in, int k, int stride, int pad) { return (in + 2 * pad - k) / stride + 1; }

/* Range [lo, hi) of output positions o whose tap o*stride + t - pad falls inside [0, in). */
static void tap_range(int in, int out, int t, int stride, int pad, int* lo, int* hi)
{
    int l = 0, h = out;
    while (l < out && l * stride + t - pad < 0) ++l;
    while (h > l && (h - 1) * stride + t - pad >= in) --h;
    *lo = l;
    *hi = h;
}

/* y[n,co,ho,wo] = sum_{ci,r,s} x[n,ci,ho*st+r-pad,wo*st+s-pad] * w[co,ci,r,s]   (zero padding) */
void oracle_conv2d_forward(const double* x, const double* w, double* y, int N, int C, int H, int W, int K,
                           int R, int S, int stride, int pad)
{
    const int Ho = out_dim(H, R, stride, pad), Wo = out_dim(W, S, stride, pad);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int co = 0; co < K; ++co) {
            double* yp = y + IDX4(n, co, 0, 0, K, Ho, Wo);
            memset(yp, 0, sizeof(double) * (size_t)Ho * Wo);
            for (int ci = 0; ci < C; ++ci)
                for (int r = 0; r < R; ++r)
                    for (int s = 0; s < S; ++s) {
                        const double wv = w[(((size_t)co * C + ci) * R + r) * S + s];
                        int wlo, whi;
                        tap_range(W, Wo, s, stride, pad, &wlo, &whi);
                        for (int ho = 0; ho < Ho; ++ho) {
                            const int hi = ho * stride + r - pad;
                            if (hi < 0 || hi >= H) continue;
                            const double* xp = x + IDX4(n, ci, hi, 0, C, H, W);
                            for (int wo = wlo; wo < whi; ++wo)
                                yp[(size_t)ho * Wo + wo] += xp[wo * stride + s - pad] * wv;
                        }
                    }
        }
}

/* dx[n,ci,hi,wi] = sum over every (co,r,s,ho,wo) whose forward term read x[n,ci,hi,wi] of dy*w */
void oracle_conv2d_backward_data(const double* dy, const double* w, double* dx, int N, int C, int H, int W,
                                 int K, int R, int S, int stride, int pad)
{
    const int Ho = out_dim(H, R, stride, pad), Wo = out_dim(W, S, stride, pad);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        memset(dx + IDX4(n, 0, 0, 0, C, H, W), 0, sizeof(double) * (size_t)C * H * W);
        for (int co = 0; co < K; ++co) {
            const double* gp = dy + IDX4(n, co, 0, 0, K, Ho, Wo);
            for (int ci = 0; ci < C; ++ci)
                for (int r = 0; r < R; ++r)
                    for (int s = 0; s < S; ++s) {
                        const double wv = w[(((size_t)co * C + ci) * R + r) * S + s];
                        int wlo, whi;
                        tap_range(W, Wo, s, stride, pad, &wlo, &whi);
                        for (int ho = 0; ho < Ho; ++ho) {
                            const int hi = ho * stride + r - pad;
                            if (hi < 0 || hi >= H) continue;
                            double* dxp = dx + IDX4(n, ci, hi, 0, C, H, W);
                            for (int wo = wlo; wo < whi; ++wo)
                                dxp[wo * stride + s - pad] += gp[(size_t)ho * Wo + wo] * wv;
                        }
                    }
        }
    }
}

/* dw[co,ci,r,s] = sum_{n,ho,wo} dy[n,co,ho,wo] * x[n,ci,ho*st+r-pad,wo*st+s-pad] */
void oracle_conv2d_backward_weight(const double* x, const double* dy, double* dw, int N, int C, int H, int W,
                                   int K, int R, int S, int stride, int pad)
{
    const int Ho = out_dim(H, R, stride, pad), Wo = out_dim(W, S, stride, pad);
#pragma omp parallel for schedule(static) collapse(2)
    for (int co = 0; co < K; ++co)
        for (int ci = 0; ci < C; ++ci)
            for (int r = 0; r < R; ++r)
                for (int s = 0; s < S; ++s) {
                    double acc = 0.0;
                    int wlo, whi;
                    tap_range(W, Wo, s, stride, pad, &wlo, &whi);
                    for (int n = 0; n < N; ++n) {
                        const double* gp = dy + IDX4(n, co, 0, 0, K, Ho, Wo);
                        for (int ho = 0; ho < Ho; ++ho) {
                            const int hi = ho * stride + r - pad;
                            if (hi < 0 || hi >= H) continue;
                            const double* xp = x + IDX4(n, ci, hi, 0, C, H, W);
                            for (int wo = wlo; wo < whi; ++wo)
                                acc += gp[(size_t)ho * Wo + wo] * xp[wo * stride + s - pad];
                        }
                    }
                    dw[(((size_t)co * C + ci) * R + r) * S + s] = acc;
                }
}

/*
 * Batch normalisation in training mode, per channel over (N, H, W):
 *   mu = mean(x), var = mean((x-mu)^2) (biased), xhat = (x-mu)/sqrt(var+eps), y = gamma*xhat + beta.
 * mean[] and invstd[] (= 1/sqrt(var+eps)) are returned for the backward pass.
 */
void oracle_bn_forward(const double* x, const double* gamma, const double* beta, double eps, double* y,
                       double* mean, double* invstd, int N, int C, int HW)
{
    const double M = (double)N * HW;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        double s = 0.0;
        for (int n = 0; n < N; ++n)
            for (int i = 0; i < HW; ++i) s += x[((size_t)n * C + c) * HW + i];
        const double mu = s / M;
        double v = 0.0;
        for (int n = 0; n < N; ++n)
            for (int i = 0; i < HW; ++i) {
                const double d = x[((size_t)n * C + c) * HW + i] - mu;
                v += d * d;
            }
        const double is = 1.0 / sqrt(v / M + eps);
        mean[c] = mu;
        invstd[c] = is;
        for (int n = 0; n < N; ++n)
            for (int i = 0; i < HW; ++i) {
                const size_t j = ((size_t)n * C + c) * HW + i;
                y[j] = gamma[c] * ((x[j] - mu) * is) + beta[c];
            }
    }
}

/*
 * VJP of the map above (statistics are functions of x):
 *   dbeta = sum dy, dgamma = sum dy*xhat,
 *   dx = gamma*invstd * (dy - dbeta/M - xhat*dgamma/M).
 */
void oracle_bn_backward(const double* dy, const double* x, const double* gamma, const double* mean,
                        const double* invstd, double* dx, double* dgamma, double* dbeta, int N, int C, int HW)
{
    const double M = (double)N * HW;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        double sb = 0.0, sg = 0.0;
        for (int n = 0; n < N; ++n)
            for (int i = 0; i < HW; ++i) {
                const size_t j = ((size_t)n * C + c) * HW + i;
                sb += dy[j];
                sg += dy[j] * ((x[j] - mean[c]) * invstd[c]);
            }
        dbeta[c] = sb;
        dgamma[c] = sg;
        for (int n = 0; n < N; ++n)
            for (int i = 0; i < HW; ++i) {
                const size_t j = ((size_t)n * C + c) * HW + i;
                const double xh = (x[j] - mean[c]) * invstd[c];
                dx[j] = gamma[c] * invstd[c] * (dy[j] - sb / M - xh * sg / M);
            }
    }
}

/* Max pooling, padding value -inf; argmax[] keeps the flat (h*W+w) source of each output (first max wins). */
void oracle_maxpool_forward(const double* x, double* y, int32_t* argmax, int N, int C, int H, int W, int k,
                            int stride, int pad)
{
    const int Ho = out_dim(H, k, stride, pad), Wo = out_dim(W, k, stride, pad);
#pragma omp parallel for schedule(static)
    for (int nc = 0; nc < N * C; ++nc) {
        const double* xp = x + (size_t)nc * H * W;
        for (int ho = 0; ho < Ho; ++ho)
            for (int wo = 0; wo < Wo; ++wo) {
                double best = -INFINITY;
                int arg = -1;
                for (int r = 0; r < k; ++r)
                    for (int s = 0; s < k; ++s) {
                        const int hi = ho * stride + r - pad, wi = wo * stride + s - pad;
                        if (hi < 0 || hi >= H || wi < 0 || wi >= W) continue;
                        if (xp[hi * W + wi] > best) { best = xp[hi * W + wi]; arg = hi * W + wi; }
                    }
                y[((size_t)nc * Ho + ho) * Wo + wo] = best;
                argmax[((size_t)nc * Ho + ho) * Wo + wo] = arg;
            }
    }
}

void oracle_maxpool_backward(const double* dy, const int32_t* argmax, double* dx, int N, int C, int H, int W,
                             int Ho, int Wo)
{
#pragma omp parallel for schedule(static)
    for (int nc = 0; nc < N * C; ++nc) {
        double* dxp = dx + (size_t)nc * H * W;
        memset(dxp, 0, sizeof(double) * (size_t)H * W);
        for (int i = 0; i < Ho * Wo; ++i) {
            const int a = argmax[(size_t)nc * Ho * Wo + i];
            if (a >= 0) dxp[a] += dy[(size_t)nc * Ho * Wo + i];
        }
    }
}
