/*
 * CPU oracle for the library's other functions (paper, Section 2.2 "Other functions"):
 * the three neuron activations (sigmoid, rectified linear, hyperbolic tangent), forward
 * and backward; softmax, computed the numerically stable way (every element shifted by
 * the maximum before exponentiation), per image over (feature map, height, width) or per
 * spatial location over the feature maps; max and average pooling; and the addition of
 * tensors with optional broadcasting.  TEST INFRASTRUCTURE ONLY: used by the tests, the
 * smoke check and the bench's baseline leg; the HIP library never calls it and shares no
 * code with it.
 *
 * Each function is the plain definition, element by element, in double precision;
 * tensors are logical (N,C,H,W) arrays addressed through four element strides; results
 * are blended as out = alpha * value + beta * old (Section 2.1.1's accumulate form).
 * Nothing is tiled, fused or reordered.
 */
#include <math.h>
#include <stddef.h>

enum { ACT_SIGMOID = 0, ACT_RELU = 1, ACT_TANH = 2 };
enum { SOFTMAX_INSTANCE = 0, SOFTMAX_CHANNEL = 1 };
enum { POOL_MAX = 0, POOL_AVERAGE = 1 };

static long long at(const long long *s, int n, int c, int h, int w)
{
    return n * s[0] + c * s[1] + h * s[2] + w * s[3];
}

static double act_value(int mode, double x)
{
    if (mode == ACT_SIGMOID) return 1.0 / (1.0 + exp(-x));
    if (mode == ACT_RELU) return x > 0.0 ? x : 0.0;
    return tanh(x);
}

/* y = alpha * f(x) + beta * y_old */
int pointwise_oracle_activation_forward(int mode, const float *x, const long long *xs,
                                        int N, int C, int H, int W, double alpha, double beta,
                                        const double *y_old, double *y, const long long *ys)
{
    if (mode < 0 || mode > 2 || N < 1 || C < 1 || H < 1 || W < 1) return -1;
    if (beta != 0.0 && y_old == NULL) return -2;
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w) {
                    long long o = at(ys, n, c, h, w);
                    double v = alpha * act_value(mode, (double)x[at(xs, n, c, h, w)]);
                    if (beta != 0.0) v += beta * y_old[o];
                    y[o] = v;
                }
    return 0;
}

/* dx = alpha * dy * f'(.) + beta * dx_old, with f' written in terms of the forward output
 * y = f(x) for sigmoid (y(1-y)) and tanh (1-y^2), and of the input x for the rectifier
 * (1 where x > 0, else 0). */
int pointwise_oracle_activation_backward(int mode, const float *y, const long long *ys,
                                         const float *dy, const long long *dys,
                                         const float *x, const long long *xs,
                                         int N, int C, int H, int W, double alpha, double beta,
                                         const double *dx_old, double *dx, const long long *dxs)
{
    if (mode < 0 || mode > 2 || N < 1 || C < 1 || H < 1 || W < 1) return -1;
    if (beta != 0.0 && dx_old == NULL) return -2;
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w) {
                    double yy = (double)y[at(ys, n, c, h, w)];
                    double g = (double)dy[at(dys, n, c, h, w)];
                    double d;
                    if (mode == ACT_SIGMOID) d = yy * (1.0 - yy);
                    else if (mode == ACT_RELU) d = (double)x[at(xs, n, c, h, w)] > 0.0 ? 1.0 : 0.0;
                    else d = 1.0 - yy * yy;
                    long long o = at(dxs, n, c, h, w);
                    double v = alpha * g * d;
                    if (beta != 0.0) v += beta * dx_old[o];
                    dx[o] = v;
                }
    return 0;
}

/* y = alpha * b + beta * y_old, b broadcast along every dimension in which it has size 1. */
int pointwise_oracle_add_tensor(const float *b, const long long *bs, int bN, int bC, int bH, int bW,
                                int N, int C, int H, int W, double alpha, double beta,
                                const double *y_old, double *y, const long long *ys)
{
    if (N < 1 || C < 1 || H < 1 || W < 1) return -1;
    if ((bN != 1 && bN != N) || (bC != 1 && bC != C) || (bH != 1 && bH != H) || (bW != 1 && bW != W)) return -3;
    if (beta != 0.0 && y_old == NULL) return -2;
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w) {
                    long long o = at(ys, n, c, h, w);
                    double v = alpha * (double)b[at(bs, bN == 1 ? 0 : n, bC == 1 ? 0 : c, bH == 1 ? 0 : h, bW == 1 ? 0 : w)];
                    if (beta != 0.0) v += beta * y_old[o];
                    y[o] = v;
                }
    return 0;
}

/* Softmax over a group of elements: INSTANCE: all (c,h,w) of one image; CHANNEL: all c of
 * one (n,h,w).  Stable form: m = max over the group, y = exp(x - m) / sum exp(x - m). */
int pointwise_oracle_softmax_forward(int mode, const float *x, const long long *xs,
                                     int N, int C, int H, int W, double alpha, double beta,
                                     const double *y_old, double *y, const long long *ys)
{
    if (mode < 0 || mode > 1 || N < 1 || C < 1 || H < 1 || W < 1) return -1;
    if (beta != 0.0 && y_old == NULL) return -2;
    for (int n = 0; n < N; ++n) {
        int groups_h = mode == SOFTMAX_INSTANCE ? 1 : H, groups_w = mode == SOFTMAX_INSTANCE ? 1 : W;
        for (int gh = 0; gh < groups_h; ++gh)
            for (int gw = 0; gw < groups_w; ++gw) {
                int h0 = mode == SOFTMAX_INSTANCE ? 0 : gh, h1 = mode == SOFTMAX_INSTANCE ? H : gh + 1;
                int w0 = mode == SOFTMAX_INSTANCE ? 0 : gw, w1 = mode == SOFTMAX_INSTANCE ? W : gw + 1;
                double m = -INFINITY, sum = 0.0;
                for (int c = 0; c < C; ++c)
                    for (int h = h0; h < h1; ++h)
                        for (int w = w0; w < w1; ++w) {
                            double v = (double)x[at(xs, n, c, h, w)];
                            if (v > m) m = v;
                        }
                for (int c = 0; c < C; ++c)
                    for (int h = h0; h < h1; ++h)
                        for (int w = w0; w < w1; ++w) sum += exp((double)x[at(xs, n, c, h, w)] - m);
                for (int c = 0; c < C; ++c)
                    for (int h = h0; h < h1; ++h)
                        for (int w = w0; w < w1; ++w) {
                            long long o = at(ys, n, c, h, w);
                            double v = alpha * (exp((double)x[at(xs, n, c, h, w)] - m) / sum);
                            if (beta != 0.0) v += beta * y_old[o];
                            y[o] = v;
                        }
            }
    }
    return 0;
}

/* Pooling over windows of win_h x win_w input elements, window (p,q) starting at
 * (p*u - pad_h, q*v - pad_w); output size as eq. 1 of the convolution with the window in
 * place of the filter.  Elements outside the image do not take part: the maximum runs
 * over the in-image elements, the average divides by their number.  A window with no
 * in-image element (possible only with pad >= window) is rejected. */
int pointwise_oracle_pooling_forward(int mode, const float *x, const long long *xs,
                                     int N, int C, int H, int W, int win_h, int win_w,
                                     int pad_h, int pad_w, int u, int v, double alpha, double beta,
                                     const double *y_old, double *y, const long long *ys, int P, int Q)
{
    if (mode < 0 || mode > 1 || N < 1 || C < 1 || H < 1 || W < 1) return -1;
    if (win_h < 1 || win_w < 1 || u < 1 || v < 1 || pad_h < 0 || pad_w < 0) return -4;
    if (pad_h >= win_h || pad_w >= win_w) return -5;
    if (H + 2 * pad_h < win_h || W + 2 * pad_w < win_w) return -6;
    if (P != (H + 2 * pad_h - win_h) / u + 1 || Q != (W + 2 * pad_w - win_w) / v + 1) return -7;
    if (beta != 0.0 && y_old == NULL) return -2;
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double m = -INFINITY, sum = 0.0;
                    int count = 0;
                    for (int r = 0; r < win_h; ++r)
                        for (int s = 0; s < win_w; ++s) {
                            int h = p * u + r - pad_h, w = q * v + s - pad_w;
                            if (h < 0 || h >= H || w < 0 || w >= W) continue;
                            double val = (double)x[at(xs, n, c, h, w)];
                            if (val > m) m = val;
                            sum += val;
                            ++count;
                        }
                    if (count == 0) return -8;
                    long long o = at(ys, n, c, p, q);
                    double val = alpha * (mode == POOL_MAX ? m : sum / count);
                    if (beta != 0.0) val += beta * y_old[o];
                    y[o] = val;
                }
    return 0;
}

/* Softmax backward.  With y the forward result of a group and dy the gradient with respect
 * to y, the Jacobian dy_j/dx_i = y_j (delta_ij - y_i) gives
 *     dx_i = y_i * (dy_i - sum_j dy_j y_j),   j over the group (see the forward function). */
int pointwise_oracle_softmax_backward(int mode, const float *y, const long long *ys,
                                      const float *dy, const long long *dys,
                                      int N, int C, int H, int W, double alpha, double beta,
                                      const double *dx_old, double *dx, const long long *dxs)
{
    if (mode < 0 || mode > 1 || N < 1 || C < 1 || H < 1 || W < 1) return -1;
    if (beta != 0.0 && dx_old == NULL) return -2;
    for (int n = 0; n < N; ++n) {
        int groups_h = mode == SOFTMAX_INSTANCE ? 1 : H, groups_w = mode == SOFTMAX_INSTANCE ? 1 : W;
        for (int gh = 0; gh < groups_h; ++gh)
            for (int gw = 0; gw < groups_w; ++gw) {
                int h0 = mode == SOFTMAX_INSTANCE ? 0 : gh, h1 = mode == SOFTMAX_INSTANCE ? H : gh + 1;
                int w0 = mode == SOFTMAX_INSTANCE ? 0 : gw, w1 = mode == SOFTMAX_INSTANCE ? W : gw + 1;
                double dot = 0.0;
                for (int c = 0; c < C; ++c)
                    for (int h = h0; h < h1; ++h)
                        for (int w = w0; w < w1; ++w)
                            dot += (double)dy[at(dys, n, c, h, w)] * (double)y[at(ys, n, c, h, w)];
                for (int c = 0; c < C; ++c)
                    for (int h = h0; h < h1; ++h)
                        for (int w = w0; w < w1; ++w) {
                            long long o = at(dxs, n, c, h, w);
                            double v = alpha * ((double)y[at(ys, n, c, h, w)] * ((double)dy[at(dys, n, c, h, w)] - dot));
                            if (beta != 0.0) v += beta * dx_old[o];
                            dx[o] = v;
                        }
            }
    }
    return 0;
}

/* Pooling backward: the gradient dy of every window goes back to the input elements the
 * window's value came from.  AVERAGE: each in-image element of the window receives
 * dy / (number of in-image elements) - the transpose of the forward map.  MAX: the
 * in-image element holding the maximum receives dy; among equal maxima the first in scan
 * order (rows, then columns, of the window).  An element covered by several windows sums
 * their contributions.  `scratch` holds N*C*H*W doubles (packed N,C,H,W) for the raw sum. */
int pointwise_oracle_pooling_backward(int mode, const float *x, const long long *xs,
                                      const float *dy, const long long *dys,
                                      int N, int C, int H, int W, int win_h, int win_w,
                                      int pad_h, int pad_w, int u, int v, double alpha, double beta,
                                      const double *dx_old, double *dx, const long long *dxs, int P, int Q,
                                      double *scratch)
{
    if (mode < 0 || mode > 1 || N < 1 || C < 1 || H < 1 || W < 1) return -1;
    if (win_h < 1 || win_w < 1 || u < 1 || v < 1 || pad_h < 0 || pad_w < 0) return -4;
    if (pad_h >= win_h || pad_w >= win_w) return -5;
    if (H + 2 * pad_h < win_h || W + 2 * pad_w < win_w) return -6;
    if (P != (H + 2 * pad_h - win_h) / u + 1 || Q != (W + 2 * pad_w - win_w) / v + 1) return -7;
    if (beta != 0.0 && dx_old == NULL) return -2;
    if (scratch == NULL) return -3;
    for (long long i = 0; i < (long long)N * C * H * W; ++i) scratch[i] = 0.0;
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            double *g = scratch + ((long long)n * C + c) * H * W;
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double grad = (double)dy[at(dys, n, c, p, q)];
                    double m = -INFINITY;
                    int count = 0, mh = -1, mw = -1;
                    for (int r = 0; r < win_h; ++r)
                        for (int s = 0; s < win_w; ++s) {
                            int h = p * u + r - pad_h, w = q * v + s - pad_w;
                            if (h < 0 || h >= H || w < 0 || w >= W) continue;
                            double val = (double)x[at(xs, n, c, h, w)];
                            if (count == 0 || val > m) { m = val; mh = h; mw = w; }
                            ++count;
                        }
                    if (count == 0) return -8;
                    if (mode == POOL_MAX) {
                        g[mh * W + mw] += grad;
                    } else {
                        for (int r = 0; r < win_h; ++r)
                            for (int s = 0; s < win_w; ++s) {
                                int h = p * u + r - pad_h, w = q * v + s - pad_w;
                                if (h < 0 || h >= H || w < 0 || w >= W) continue;
                                g[h * W + w] += grad / count;
                            }
                    }
                }
        }
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w) {
                    long long o = at(dxs, n, c, h, w);
                    double val = alpha * scratch[(((long long)n * C + c) * H + h) * W + w];
                    if (beta != 0.0) val += beta * dx_old[o];
                    dx[o] = val;
                }
    return 0;
}
