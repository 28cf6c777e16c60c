/*
 * CPU oracle for the layer-wise CNN training step of vDNN (arxiv 1602.08124).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what each
 * layer computes.  It is used by the tests, the smoke check and the cpu_baseline
 * leg of the benchmark; the product path never calls it and shares no code with it.
 *
 * Everything is fp64, NCHW, direct nested loops in the order of the defining sums.
 * There is no blocking, no im2col, no reordering.  OpenMP only splits the outermost
 * independent loop (each thread owns whole output elements, so results do not depend
 * on the thread count).
 *
 * What the paper fixes (Section 2.2 "DNN training", Eq. bwdprop / chain_rule): a layer
 * maps X to Y in forward propagation; in backward propagation dX = dY * dY/dX and the
 * weight gradients follow from the same chain rule.  The paper names the layer types
 * (CONV, ACTV, POOL, FC, a loss) but not their formulas; the formulas below are the
 * textbook ones, with these readings where the paper is silent:
 *   - CONV is cross-correlation with zero padding and no bias;
 *   - ACTV is ReLU, computed in place, its gradient masked by (Y > 0);
 *   - max-pool picks the first maximum in row-major window order; padded cells never win;
 *     overlapping windows accumulate into dX;
 *   - the loss is softmax cross-entropy, mean over the batch.
 */
#include <math.h>
#include <stddef.h>
#include <string.h>

#define IDX4(n, c, h, w, C, H, W) ((((size_t)(n) * (C) + (c)) * (H) + (h)) * (W) + (w))

static int out_dim(int in, int k, int stride, int pad) { return (in + 2 * pad - k) / stride + 1; }

int oracle_out_dim(int in, int k, int stride, int pad) { return out_dim(in, k, stride, pad); }

/* Y[n,k,p,q] = sum_{c,r,s} X[n,c,p*st+r-pad,q*st+s-pad] * W[k,c,r,s]   (Section 2.2, forward propagation of a CONV layer) */
void oracle_conv_fwd(const double* X, const double* Wt, double* Y, int N, int C, int H, int W, int K, int R, int S,
                     int stride, int pad) {
    const int P = out_dim(H, R, stride, pad), Q = out_dim(W, S, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double acc = 0.0;
                    for (int c = 0; c < C; ++c)
                        for (int r = 0; r < R; ++r) {
                            const int h = p * stride + r - pad;
                            if (h < 0 || h >= H) continue;
                            for (int s = 0; s < S; ++s) {
                                const int w = q * stride + s - pad;
                                if (w < 0 || w >= W) continue;
                                acc += X[IDX4(n, c, h, w, C, H, W)] * Wt[IDX4(k, c, r, s, C, R, S)];
                            }
                        }
                    Y[IDX4(n, k, p, q, K, P, Q)] = acc;
                }
}

/* dX[n,c,h,w] = sum_{k,p,q,r,s : p*st+r-pad==h, q*st+s-pad==w} dY[n,k,p,q] * W[k,c,r,s]
 * (Eq. chain_rule applied to the CONV definition).  Written as a scatter of every
 * forward term into the input it touched, so the index relation is literally the forward one. */
void oracle_conv_bwd_data(const double* dY, const double* Wt, double* dX, int N, int C, int H, int W, int K, int R,
                          int S, int stride, int pad) {
    const int P = out_dim(H, R, stride, pad), Q = out_dim(W, S, stride, pad);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        memset(dX + (size_t)n * C * H * W, 0, sizeof(double) * (size_t)C * H * W);
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    const double g = dY[IDX4(n, k, p, q, K, P, Q)];
                    for (int c = 0; c < C; ++c)
                        for (int r = 0; r < R; ++r) {
                            const int h = p * stride + r - pad;
                            if (h < 0 || h >= H) continue;
                            for (int s = 0; s < S; ++s) {
                                const int w = q * stride + s - pad;
                                if (w < 0 || w >= W) continue;
                                dX[IDX4(n, c, h, w, C, H, W)] += g * Wt[IDX4(k, c, r, s, C, R, S)];
                            }
                        }
                }
    }
}

/* dW[k,c,r,s] = sum_{n,p,q} dY[n,k,p,q] * X[n,c,p*st+r-pad,q*st+s-pad]   (Eq. chain_rule, weight gradients) */
void oracle_conv_bwd_filter(const double* X, const double* dY, double* dW, int N, int C, int H, int W, int K, int R,
                            int S, int stride, int pad) {
    const int P = out_dim(H, R, stride, pad), Q = out_dim(W, S, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
    for (int k = 0; k < K; ++k)
        for (int c = 0; c < C; ++c)
            for (int r = 0; r < R; ++r)
                for (int s = 0; s < S; ++s) {
                    double acc = 0.0;
                    for (int n = 0; n < N; ++n)
                        for (int p = 0; p < P; ++p) {
                            const int h = p * stride + r - pad;
                            if (h < 0 || h >= H) continue;
                            for (int q = 0; q < Q; ++q) {
                                const int w = q * stride + s - pad;
                                if (w < 0 || w >= W) continue;
                                acc += dY[IDX4(n, k, p, q, K, P, Q)] * X[IDX4(n, c, h, w, C, H, W)];
                            }
                        }
                    dW[IDX4(k, c, r, s, C, R, S)] = acc;
                }
}

/* In-place activation (Section 2.2 footnote on in-place ACTV layers): Y <- max(Y, 0). */
void oracle_relu_fwd(double* Y, size_t count) {
    for (size_t i = 0; i < count; ++i) Y[i] = Y[i] > 0.0 ? Y[i] : 0.0;
}

/* dY <- dY where the activation OUTPUT is positive, else 0 (only Y and dY exist for an in-place layer). */
void oracle_relu_bwd(const double* Y, double* dY, size_t count) {
    for (size_t i = 0; i < count; ++i) dY[i] = Y[i] > 0.0 ? dY[i] : 0.0;
}

/* POOL layer, max: Y[n,c,p,q] = max over the k x k window at (p*st-pad, q*st-pad); cells outside the image never win. */
void oracle_maxpool_fwd(const double* X, double* Y, int N, int C, int H, int W, int k, int stride, int pad) {
    const int P = out_dim(H, k, stride, pad), Q = out_dim(W, k, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double best = -INFINITY;
                    for (int r = 0; r < k; ++r)
                        for (int s = 0; s < k; ++s) {
                            const int h = p * stride + r - pad, w = q * stride + s - pad;
                            if (h < 0 || h >= H || w < 0 || w >= W) continue;
                            const double v = X[IDX4(n, c, h, w, C, H, W)];
                            if (v > best) best = v;
                        }
                    Y[IDX4(n, c, p, q, C, P, Q)] = best;
                }
}

/* Max-pool backward: each dY element is routed to the first maximum of its window (strict > scan, row-major);
 * windows that overlap add up. */
void oracle_maxpool_bwd(const double* X, const double* dY, double* dX, int N, int C, int H, int W, int k, int stride,
                        int pad) {
    const int P = out_dim(H, k, stride, pad), Q = out_dim(W, k, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            double* dx = dX + IDX4(n, c, 0, 0, C, H, W);
            for (int i = 0; i < H * W; ++i) dx[i] = 0.0;
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double best = -INFINITY;
                    int bh = -1, bw = -1;
                    for (int r = 0; r < k; ++r)
                        for (int s = 0; s < k; ++s) {
                            const int h = p * stride + r - pad, w = q * stride + s - pad;
                            if (h < 0 || h >= H || w < 0 || w >= W) continue;
                            const double v = X[IDX4(n, c, h, w, C, H, W)];
                            if (v > best) { best = v; bh = h; bw = w; }
                        }
                    if (bh >= 0) dx[bh * W + bw] += dY[IDX4(n, c, p, q, C, P, Q)];
                }
        }
}

/* POOL layer, average: window mean with the divisor k*k (padded cells count as zeros). */
void oracle_avgpool_fwd(const double* X, double* Y, int N, int C, int H, int W, int k, int stride, int pad) {
    const int P = out_dim(H, k, stride, pad), Q = out_dim(W, k, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double acc = 0.0;
                    for (int r = 0; r < k; ++r)
                        for (int s = 0; s < k; ++s) {
                            const int h = p * stride + r - pad, w = q * stride + s - pad;
                            if (h < 0 || h >= H || w < 0 || w >= W) continue;
                            acc += X[IDX4(n, c, h, w, C, H, W)];
                        }
                    Y[IDX4(n, c, p, q, C, P, Q)] = acc / (double)(k * k);
                }
}

void oracle_avgpool_bwd(const double* dY, double* dX, int N, int C, int H, int W, int k, int stride, int pad) {
    const int P = out_dim(H, k, stride, pad), Q = out_dim(W, k, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            double* dx = dX + IDX4(n, c, 0, 0, C, H, W);
            for (int i = 0; i < H * W; ++i) dx[i] = 0.0;
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    const double g = dY[IDX4(n, c, p, q, C, P, Q)] / (double)(k * k);
                    for (int r = 0; r < k; ++r)
                        for (int s = 0; s < k; ++s) {
                            const int h = p * stride + r - pad, w = q * stride + s - pad;
                            if (h < 0 || h >= H || w < 0 || w >= W) continue;
                            dx[h * W + w] += g;
                        }
                }
        }
}

/* FC layer on the flattened NCHW vector: Y[n,o] = sum_i X[n,i] * W[o,i]. */
void oracle_fc_fwd(const double* X, const double* Wt, double* Y, int N, int I, int O) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int o = 0; o < O; ++o) {
            double acc = 0.0;
            for (int i = 0; i < I; ++i) acc += X[(size_t)n * I + i] * Wt[(size_t)o * I + i];
            Y[(size_t)n * O + o] = acc;
        }
}

/* dX[n,i] = sum_o dY[n,o] * W[o,i] */
void oracle_fc_bwd_data(const double* dY, const double* Wt, double* dX, int N, int I, int O) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int i = 0; i < I; ++i) {
            double acc = 0.0;
            for (int o = 0; o < O; ++o) acc += dY[(size_t)n * O + o] * Wt[(size_t)o * I + i];
            dX[(size_t)n * I + i] = acc;
        }
}

/* dW[o,i] = sum_n dY[n,o] * X[n,i] */
void oracle_fc_bwd_filter(const double* X, const double* dY, double* dW, int N, int I, int O) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int o = 0; o < O; ++o)
        for (int i = 0; i < I; ++i) {
            double acc = 0.0;
            for (int n = 0; n < N; ++n) acc += dY[(size_t)n * O + o] * X[(size_t)n * I + i];
            dW[(size_t)o * I + i] = acc;
        }
}

/* Loss (Eq. bwdprop: the gradient of the loss w.r.t. the last layer's output starts backward propagation).
 * loss = (1/N) sum_n [ log sum_j exp(z[n,j]) - z[n,label_n] ],  dz = (softmax(z) - onehot) / N.
 * The maximum is subtracted before exponentiation; that does not change the value. */
double oracle_softmax_ce(const double* Z, const int* labels, double* dZ, int N, int classes) {
    double loss = 0.0;
    for (int n = 0; n < N; ++n) {
        const double* z = Z + (size_t)n * classes;
        double m = z[0];
        for (int j = 1; j < classes; ++j) if (z[j] > m) m = z[j];
        double sum = 0.0;
        for (int j = 0; j < classes; ++j) sum += exp(z[j] - m);
        const double lse = m + log(sum);
        loss += lse - z[labels[n]];
        if (dZ) {
            double* dz = dZ + (size_t)n * classes;
            for (int j = 0; j < classes; ++j) dz[j] = exp(z[j] - lse) / (double)N;
            dz[labels[n]] -= 1.0 / (double)N;
        }
    }
    return loss / (double)N;
}
