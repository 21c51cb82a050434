/*
 * CPU checker ("oracle") for the CNN layer-chain hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct definitions of every layer the HIP library
 * executes, written as direct loop nests in the style of the paper's
 * "Reference: standard C++" pooling kernel (Sec. IV, Listing "AveragePooling
 * layer in DFP description").  The paper treats layer semantics as those of
 * the unmodified framework it wraps (Sec. V, evaluation set-up), so the
 * definitions are the textbook ones: cross-correlation convolution with zero
 * padding, floor-mode pooling, batch-norm with eps inside the square root.
 *
 * Everything is fp64, logical layout: activations [N][C][H][W], convolution
 * weights [K][C][R][S], linear weights [Out][In].  There is no blocking, no
 * fusion, no reordering; OpenMP is applied to the outermost loops only.
 * Nothing here is shared with, derived from, or used by the HIP path; only
 * tests, the smoke check and the benchmark's CPU-baseline leg may call it.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define IDX4(n, c, h, w, C, H, W) ((((size_t)(n) * (C) + (c)) * (H) + (h)) * (W) + (w))

/* floor-mode output extent of a sliding window (convolution and pooling alike) */
int orc_out_size(int in, int k, int s, int p) { return (in + 2 * p - k) / s + 1; }

/* ------------------------------------------------------------------ forward ---- */

/* y[n,k,p,q] = bias[k] + sum_{c,r,s} x[n,c,p*sh+r-ph,q*sw+s-pw] * w[k,c,r,s]; x outside = 0 */
void orc_conv2d(const double *x, const double *w, const double *bias, double *y, int N, int C, int H,
                int W, int K, int R, int S, int sh, int sw, int ph, int pw) {
    const int Ho = orc_out_size(H, R, sh, ph), Wo = orc_out_size(W, S, sw, pw);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; n++)
        for (int k = 0; k < K; k++)
            for (int p = 0; p < Ho; p++)
                for (int q = 0; q < Wo; q++) {
                    double acc = bias ? bias[k] : 0.0;
                    for (int c = 0; c < C; c++)
                        for (int r = 0; r < R; r++)
                            for (int s = 0; s < S; s++) {
                                const int ih = p * sh + r - ph, iw = q * sw + s - pw;
                                if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                                acc += x[IDX4(n, c, ih, iw, C, H, W)] * w[IDX4(k, c, r, s, C, R, S)];
                            }
                    y[IDX4(n, k, p, q, K, Ho, Wo)] = acc;
                }
}

/* Depthwise convolution (as many groups as channels; the paper's optimizer hands exactly this case to its fused
 * loop-nest module instead of a library, Sec. III-A): every channel is filtered on its own,
 * y[n,c,p,q] = bias[c] + sum_{r,s} x[n,c,p*sh+r-ph,q*sw+s-pw] * w[c,r,s]; x outside = 0 */
void orc_dwconv2d(const double *x, const double *w, const double *bias, double *y, int N, int C, int H, int W,
                  int R, int S, int sh, int sw, int ph, int pw) {
    const int Ho = orc_out_size(H, R, sh, ph), Wo = orc_out_size(W, S, sw, pw);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; n++)
        for (int c = 0; c < C; c++)
            for (int p = 0; p < Ho; p++)
                for (int q = 0; q < Wo; q++) {
                    double acc = bias ? bias[c] : 0.0;
                    for (int r = 0; r < R; r++)
                        for (int s = 0; s < S; s++) {
                            const int ih = p * sh + r - ph, iw = q * sw + s - pw;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                            acc += x[IDX4(n, c, ih, iw, C, H, W)] * w[((size_t)c * R + r) * S + s];
                        }
                    y[IDX4(n, c, p, q, C, Ho, Wo)] = acc;
                }
}

/* the same definition evaluated at a list of output coordinates (n,k,p,q) only */
void orc_conv2d_points(const double *x, const double *w, const double *bias, const int32_t *coords,
                       int npts, double *out, int N, int C, int H, int W, int K, int R, int S, int sh,
                       int sw, int ph, int pw) {
    (void)N; (void)K;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < npts; i++) {
        const int n = coords[4 * i], k = coords[4 * i + 1], p = coords[4 * i + 2], q = coords[4 * i + 3];
        double acc = bias ? bias[k] : 0.0;
        for (int c = 0; c < C; c++)
            for (int r = 0; r < R; r++)
                for (int s = 0; s < S; s++) {
                    const int ih = p * sh + r - ph, iw = q * sw + s - pw;
                    if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                    acc += x[IDX4(n, c, ih, iw, C, H, W)] * w[IDX4(k, c, r, s, C, R, S)];
                }
        out[i] = acc;
    }
}

/* inference batch-norm, unfolded: y = gamma * (x - mean) / sqrt(var + eps) + beta */
void orc_bn_infer(const double *x, const double *gamma, const double *beta, const double *mean,
                  const double *var, double eps, double *y, int N, int C, int HW) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; n++)
        for (int c = 0; c < C; c++)
            for (int i = 0; i < HW; i++) {
                const size_t o = ((size_t)n * C + c) * HW + i;
                y[o] = gamma[c] * (x[o] - mean[c]) / sqrt(var[c] + eps) + beta[c];
            }
}

/* the same map applied to a list of scalars, element i belonging to channel ch[i] */
void orc_bn_infer_points(const double *x, const int32_t *ch, const double *gamma, const double *beta,
                         const double *mean, const double *var, double eps, double *y, int n) {
    for (int i = 0; i < n; i++) {
        const int c = ch[i];
        y[i] = gamma[c] * (x[i] - mean[c]) / sqrt(var[c] + eps) + beta[c];
    }
}

/* training batch-norm: per-channel mean and biased variance over (N,H,W) */
void orc_bn_train(const double *x, const double *gamma, const double *beta, double eps, double *y,
                  double *mean_out, double *var_out, int N, int C, int HW) {
    const double M = (double)N * HW;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; c++) {
        double s = 0.0;
        for (int n = 0; n < N; n++)
            for (int i = 0; i < HW; i++) s += x[((size_t)n * C + c) * HW + i];
        const double mu = s / M;
        double v = 0.0;
        for (int n = 0; n < N; n++)
            for (int i = 0; i < HW; i++) {
                const double d = x[((size_t)n * C + c) * HW + i] - mu;
                v += d * d;
            }
        v /= M;
        mean_out[c] = mu;
        var_out[c] = v;
        for (int n = 0; n < N; n++)
            for (int i = 0; i < HW; i++) {
                const size_t o = ((size_t)n * C + c) * HW + i;
                y[o] = gamma[c] * (x[o] - mu) / sqrt(v + eps) + beta[c];
            }
    }
}

void orc_relu(const double *x, double *y, size_t n) {
    for (size_t i = 0; i < n; i++) y[i] = x[i] > 0.0 ? x[i] : 0.0;
}

void orc_add(const double *a, const double *b, double *y, size_t n) {
    for (size_t i = 0; i < n; i++) y[i] = a[i] + b[i];
}

/* max-pool; padding acts as -inf; window scanned row-major, replaced only on strict '>',
 * so among equal maxima the first (lowest logical index ih*W+iw) wins.  argmax may be NULL. */
void orc_maxpool(const double *x, double *y, int32_t *argmax, int N, int C, int H, int W, int kh,
                 int kw, int sh, int sw, int ph, int pw) {
    const int Ho = orc_out_size(H, kh, sh, ph), Wo = orc_out_size(W, kw, sw, pw);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; n++)
        for (int c = 0; c < C; c++)
            for (int p = 0; p < Ho; p++)
                for (int q = 0; q < Wo; q++) {
                    double best = -INFINITY;
                    int32_t bi = -1;
                    for (int r = 0; r < kh; r++)
                        for (int s = 0; s < kw; s++) {
                            const int ih = p * sh + r - ph, iw = q * sw + s - pw;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                            const double v = x[IDX4(n, c, ih, iw, C, H, W)];
                            if (bi < 0 || v > best) { best = v; bi = ih * W + iw; }
                        }
                    y[IDX4(n, c, p, q, C, Ho, Wo)] = best;
                    if (argmax) argmax[IDX4(n, c, p, q, C, Ho, Wo)] = bi;
                }
}

/* average pool: window sum divided by the window area (count_pad) or by the number of
 * in-range elements (!count_pad) -- the two divisors of the paper's K.area(isCountPadding) */
void orc_avgpool(const double *x, double *y, int N, int C, int H, int W, int kh, int kw, int sh,
                 int sw, int ph, int pw, int count_pad) {
    const int Ho = orc_out_size(H, kh, sh, ph), Wo = orc_out_size(W, kw, sw, pw);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; n++)
        for (int c = 0; c < C; c++)
            for (int p = 0; p < Ho; p++)
                for (int q = 0; q < Wo; q++) {
                    double sum = 0.0;
                    int cnt = 0;
                    for (int r = 0; r < kh; r++)
                        for (int s = 0; s < kw; s++) {
                            const int ih = p * sh + r - ph, iw = q * sw + s - pw;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                            sum += x[IDX4(n, c, ih, iw, C, H, W)];
                            cnt++;
                        }
                    y[IDX4(n, c, p, q, C, Ho, Wo)] = sum / (count_pad ? (double)(kh * kw) : (double)cnt);
                }
}

/* global average pool: mean over H*W */
void orc_gap(const double *x, double *y, int N, int C, int HW) {
    for (int n = 0; n < N; n++)
        for (int c = 0; c < C; c++) {
            double s = 0.0;
            for (int i = 0; i < HW; i++) s += x[((size_t)n * C + c) * HW + i];
            y[(size_t)n * C + c] = s / HW;
        }
}

/* y[m,o] = b[o] + sum_i x[m,i] * w[o,i] */
void orc_linear(const double *x, const double *w, const double *b, double *y, int M, int I, int O) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int m = 0; m < M; m++)
        for (int o = 0; o < O; o++) {
            double acc = b ? b[o] : 0.0;
            for (int i = 0; i < I; i++) acc += x[(size_t)m * I + i] * w[(size_t)o * I + i];
            y[(size_t)m * O + o] = acc;
        }
}

/* round to the nearest bf16 value (8 exponent bits, 8 significant bits), ties to even */
double orc_bf16(double v) {
    if (v == 0.0 || isnan(v) || isinf(v)) return v;
    int e;
    frexp(v, &e);            /* |v| = f * 2^e, f in [0.5,1)  ->  floor(log2|v|) = e-1 */
    int ex = e - 1;
    if (ex < -126) ex = -126; /* subnormal range shares the quantum of the smallest normal */
    const double quantum = ldexp(1.0, ex - 7);
    double r = nearbyint(v / quantum) * quantum; /* default rounding mode: ties to even */
    if (fabs(r) > 0x1.FEp127) r = v > 0 ? INFINITY : -INFINITY;
    return r;
}

void orc_round_bf16(double *x, size_t n) {
    for (size_t i = 0; i < n; i++) x[i] = orc_bf16(x[i]);
}

/* ----------------------------------------------------------------- backward ---- */

/* dx[n,c,ih,iw] = sum over all (k,p,q,r,s) that read that input element of dy * w */
void orc_conv2d_dgrad(const double *dy, const double *w, double *dx, int N, int C, int H, int W,
                      int K, int R, int S, int sh, int sw, int ph, int pw) {
    const int Ho = orc_out_size(H, R, sh, ph), Wo = orc_out_size(W, S, sw, pw);
    memset(dx, 0, sizeof(double) * (size_t)N * C * H * W);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; n++)
        for (int c = 0; c < C; c++)
            for (int k = 0; k < K; k++)
                for (int p = 0; p < Ho; p++)
                    for (int q = 0; q < Wo; q++) {
                        const double g = dy[IDX4(n, k, p, q, K, Ho, Wo)];
                        for (int r = 0; r < R; r++)
                            for (int s = 0; s < S; s++) {
                                const int ih = p * sh + r - ph, iw = q * sw + s - pw;
                                if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                                dx[IDX4(n, c, ih, iw, C, H, W)] += g * w[IDX4(k, c, r, s, C, R, S)];
                            }
                    }
}

/* dw[k,c,r,s] = sum_{n,p,q} dy[n,k,p,q] * x[n,c,p*sh+r-ph,q*sw+s-pw];  db[k] = sum dy (may be NULL) */
void orc_conv2d_wgrad(const double *x, const double *dy, double *dw, double *db, int N, int C, int H,
                      int W, int K, int R, int S, int sh, int sw, int ph, int pw) {
    const int Ho = orc_out_size(H, R, sh, ph), Wo = orc_out_size(W, S, sw, pw);
#pragma omp parallel for collapse(2) schedule(static)
    for (int k = 0; k < K; k++)
        for (int c = 0; c < C; c++)
            for (int r = 0; r < R; r++)
                for (int s = 0; s < S; s++) {
                    double acc = 0.0;
                    for (int n = 0; n < N; n++)
                        for (int p = 0; p < Ho; p++)
                            for (int q = 0; q < Wo; q++) {
                                const int ih = p * sh + r - ph, iw = q * sw + s - pw;
                                if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                                acc += dy[IDX4(n, k, p, q, K, Ho, Wo)] * x[IDX4(n, c, ih, iw, C, H, W)];
                            }
                    dw[IDX4(k, c, r, s, C, R, S)] = acc;
                }
    if (db)
        for (int k = 0; k < K; k++) {
            double acc = 0.0;
            for (int n = 0; n < N; n++)
                for (int i = 0; i < Ho * Wo; i++) acc += dy[((size_t)n * K + k) * Ho * Wo + i];
            db[k] = acc;
        }
}

/* batch-stat BN backward.  xhat = (x-mean)/sigma, sigma = sqrt(var+eps):
 * dbeta = sum dy, dgamma = sum dy*xhat,
 * dx = gamma/sigma * (dy - dbeta/M - xhat*dgamma/M) */
void orc_bn_train_bwd(const double *x, const double *dy, const double *gamma, const double *mean,
                      const double *var, double eps, double *dx, double *dgamma, double *dbeta, int N,
                      int C, int HW) {
    const double M = (double)N * HW;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; c++) {
        const double sigma = sqrt(var[c] + eps);
        double sb = 0.0, sg = 0.0;
        for (int n = 0; n < N; n++)
            for (int i = 0; i < HW; i++) {
                const size_t o = ((size_t)n * C + c) * HW + i;
                sb += dy[o];
                sg += dy[o] * (x[o] - mean[c]) / sigma;
            }
        dbeta[c] = sb;
        dgamma[c] = sg;
        for (int n = 0; n < N; n++)
            for (int i = 0; i < HW; i++) {
                const size_t o = ((size_t)n * C + c) * HW + i;
                const double xh = (x[o] - mean[c]) / sigma;
                dx[o] = gamma[c] / sigma * (dy[o] - sb / M - xh * sg / M);
            }
    }
}

/* ReLU backward from the forward OUTPUT: gradient passes where y > 0 */
void orc_relu_bwd(const double *y, const double *dy, double *dx, size_t n) {
    for (size_t i = 0; i < n; i++) dx[i] = y[i] > 0.0 ? dy[i] : 0.0;
}

/* max-pool backward: scatter-add every output gradient to its argmax input element */
void orc_maxpool_bwd(const double *dy, const int32_t *argmax, double *dx, int N, int C, int H, int W,
                     int Ho, int Wo) {
    memset(dx, 0, sizeof(double) * (size_t)N * C * H * W);
    for (int n = 0; n < N; n++)
        for (int c = 0; c < C; c++)
            for (int i = 0; i < Ho * Wo; i++) {
                const size_t o = ((size_t)n * C + c) * Ho * Wo + i;
                dx[((size_t)n * C + c) * H * W + argmax[o]] += dy[o];
            }
}

void orc_avgpool_bwd(const double *dy, double *dx, int N, int C, int H, int W, int kh, int kw, int sh,
                     int sw, int ph, int pw, int count_pad) {
    const int Ho = orc_out_size(H, kh, sh, ph), Wo = orc_out_size(W, kw, sw, pw);
    memset(dx, 0, sizeof(double) * (size_t)N * C * H * W);
    for (int n = 0; n < N; n++)
        for (int c = 0; c < C; c++)
            for (int p = 0; p < Ho; p++)
                for (int q = 0; q < Wo; q++) {
                    int cnt = 0;
                    for (int r = 0; r < kh; r++)
                        for (int s = 0; s < kw; s++) {
                            const int ih = p * sh + r - ph, iw = q * sw + s - pw;
                            if (ih >= 0 && ih < H && iw >= 0 && iw < W) cnt++;
                        }
                    const double g = dy[IDX4(n, c, p, q, C, Ho, Wo)] / (count_pad ? (double)(kh * kw) : (double)cnt);
                    for (int r = 0; r < kh; r++)
                        for (int s = 0; s < kw; s++) {
                            const int ih = p * sh + r - ph, iw = q * sw + s - pw;
                            if (ih >= 0 && ih < H && iw >= 0 && iw < W) dx[IDX4(n, c, ih, iw, C, H, W)] += g;
                        }
                }
}

void orc_gap_bwd(const double *dy, double *dx, int N, int C, int HW) {
    for (int n = 0; n < N; n++)
        for (int c = 0; c < C; c++)
            for (int i = 0; i < HW; i++) dx[((size_t)n * C + c) * HW + i] = dy[(size_t)n * C + c] / HW;
}

/* dx = dy W,  dW = dy^T x,  db = column sums of dy */
void orc_linear_bwd(const double *x, const double *w, const double *dy, double *dx, double *dw,
                    double *db, int M, int I, int O) {
    for (int m = 0; m < M; m++)
        for (int i = 0; i < I; i++) {
            double acc = 0.0;
            for (int o = 0; o < O; o++) acc += dy[(size_t)m * O + o] * w[(size_t)o * I + i];
            dx[(size_t)m * I + i] = acc;
        }
#pragma omp parallel for schedule(static)
    for (int o = 0; o < O; o++) {
        for (int i = 0; i < I; i++) {
            double acc = 0.0;
            for (int m = 0; m < M; m++) acc += dy[(size_t)m * O + o] * x[(size_t)m * I + i];
            dw[(size_t)o * I + i] = acc;
        }
        double sb = 0.0;
        for (int m = 0; m < M; m++) sb += dy[(size_t)m * O + o];
        db[o] = sb;
    }
}

/* loss = mean_n( -log softmax(z_n)[label_n] ), max-subtracted; dz = (softmax - onehot) / N */
double orc_softmax_ce(const double *z, const int32_t *labels, double *dz, int N, int K) {
    double loss = 0.0;
    for (int n = 0; n < N; n++) {
        const double *zn = z + (size_t)n * K;
        double mx = zn[0];
        for (int k = 1; k < K; k++) mx = zn[k] > mx ? zn[k] : mx;
        double se = 0.0;
        for (int k = 0; k < K; k++) se += exp(zn[k] - mx);
        loss += -(zn[labels[n]] - mx - log(se));
        if (dz)
            for (int k = 0; k < K; k++)
                dz[(size_t)n * K + k] = (exp(zn[k] - mx) / se - (k == labels[n] ? 1.0 : 0.0)) / N;
    }
    return loss / N;
}

/* SGD with momentum: v <- mu*v + g ; w <- w - lr*v */
void orc_sgd(double *w, double *v, const double *g, double lr, double mu, size_t n) {
    for (size_t i = 0; i < n; i++) {
        v[i] = mu * v[i] + g[i];
        w[i] -= lr * v[i];
    }
}
