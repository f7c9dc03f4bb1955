/* Driver for a build of the C oracles under AddressSanitizer and UndefinedBehaviorSanitizer (test
 * infrastructure, like the oracles themselves): calls every oracle function on a few dozen small random
 * problems whose buffers are allocated at exactly the size the strides span, so that an access outside a
 * tensor, a signed overflow or a misaligned read in the oracle's C code ends the run with a report.  The values
 * computed are not checked here (the pins in tests/ do that on the ordinary build).  Prints "oracle check ok". */
#include <stdio.h>
#include <stdlib.h>

long long conv_oracle_output_dim(long long H, long long R, long long u, long long pad);
int conv_oracle_forward(const float *x, const long long *xs, int N, int C, int H, int W, const float *w, int K, int R, int S,
                        int pad_h, int pad_w, int u, int v, int mode, double alpha, double beta, const double *y_old,
                        double *y, const long long *ys, int P, int Q, int nthreads);
int conv_oracle_backward_data(const float *w, int K, int C, int R, int S, const float *dy, const long long *dys, int N, int P,
                              int Q, int pad_h, int pad_w, int u, int v, int mode, double alpha, double beta,
                              const double *dx_old, double *dx, const long long *dxs, int H, int W, int nthreads);
int conv_oracle_backward_filter(const float *x, const long long *xs, int N, int C, int H, int W, const float *dy,
                                const long long *dys, int K, int P, int Q, int pad_h, int pad_w, int u, int v, int mode,
                                double alpha, double beta, const double *dw_old, double *dw, int R, int S, int nthreads);
int pointwise_oracle_activation_forward(int mode, const float *x, const long long *xs, int N, int C, int H, int W, double alpha,
                                        double beta, const double *y_old, double *y, const long long *ys);
int pointwise_oracle_activation_backward(int mode, const float *y, const long long *ys, const float *dy, const long long *dys,
                                         const float *x, const long long *xs, int N, int C, int H, int W, double alpha,
                                         double beta, const double *dx_old, double *dx, const long long *dxs);
int pointwise_oracle_add_tensor(const float *b, const long long *bs, int bN, int bC, int bH, int bW, int N, int C, int H, int W,
                                double alpha, double beta, const double *y_old, double *y, const long long *ys);
int pointwise_oracle_bias_backward(const float *dy, const long long *dys, int N, int C, int H, int W, double alpha, double beta,
                                   const double *db_old, double *db);
int pointwise_oracle_softmax_forward(int mode, const float *x, const long long *xs, int N, int C, int H, int W, double alpha,
                                     double beta, const double *y_old, double *y, const long long *ys);
int pointwise_oracle_softmax_backward(int mode, const float *y, const long long *ys, const float *dy, const long long *dys, int N,
                                      int C, int H, int W, double alpha, double beta, const double *dx_old, double *dx,
                                      const long long *dxs);
int pointwise_oracle_pooling_forward(int mode, const float *x, const long long *xs, int N, int C, int H, int W, int win_h,
                                     int win_w, int pad_h, int pad_w, int u, int v, double alpha, double beta,
                                     const double *y_old, double *y, const long long *ys, int P, int Q);
int pointwise_oracle_pooling_backward(int mode, const float *x, const long long *xs, const float *dy, const long long *dys, int N,
                                      int C, int H, int W, int win_h, int win_w, int pad_h, int pad_w, int u, int v,
                                      double alpha, double beta, const double *dx_old, double *dx, const long long *dxs, int P,
                                      int Q, double *scratch);

static unsigned long long state = 14100759ull;
static int draw(int lo, int hi) /* uniform in lo..hi */
{
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return lo + (int)((state >> 33) % (unsigned long long)(hi - lo + 1));
}

static float *floats(long long n)
{
    float *p = (float *)malloc((size_t)n * sizeof(float));
    if (!p) exit(3);
    for (long long i = 0; i < n; ++i) p[i] = (float)draw(-8, 8) / 8.0f;
    return p;
}

static double *doubles(long long n)
{
    double *p = (double *)malloc((size_t)n * sizeof(double));
    if (!p) exit(3);
    for (long long i = 0; i < n; ++i) p[i] = (double)draw(-8, 8) / 8.0;
    return p;
}

/* strides n,c,h,w of a packed tensor with the channel index slowest-but-one (layout 0) or fastest (layout 1) */
static void strides(long long *s, int C, int H, int W, int layout)
{
    if (layout == 0) { s[0] = (long long)C * H * W; s[1] = (long long)H * W; s[2] = W; s[3] = 1; }
    else { s[0] = (long long)C * H * W; s[1] = 1; s[2] = (long long)W * C; s[3] = C; }
}

#define CHECK(call) do { int rc_ = (call); if (rc_ != 0) { fprintf(stderr, "%s returned %d (case %d)\n", #call, rc_, it); return 1; } } while (0)

int main(void)
{
    for (int it = 0; it < 60; ++it) {
        const int N = draw(1, 3), C = draw(1, 6), K = draw(1, 7), R = draw(1, 5), S = draw(1, 5);
        const int pad_h = draw(0, R - 1), pad_w = draw(0, S - 1), u = draw(1, 3), v = draw(1, 3), mode = draw(0, 1);
        const int H = draw(R > 2 * pad_h ? R - 2 * pad_h : 1, 12), W = draw(S > 2 * pad_w ? S - 2 * pad_w : 1, 12);
        const int P = (int)conv_oracle_output_dim(H, R, u, pad_h), Q = (int)conv_oracle_output_dim(W, S, v, pad_w);
        const int layout = draw(0, 1);
        long long xs[4], ys[4];
        strides(xs, C, H, W, layout);
        strides(ys, K, P, Q, layout);
        const long long nx = (long long)N * C * H * W, ny = (long long)N * K * P * Q, nw = (long long)K * C * R * S;
        float *x = floats(nx), *w = floats(nw), *dy = floats(ny);
        double *y = doubles(ny), *y_old = doubles(ny), *dx = doubles(nx), *dx_old = doubles(nx), *dw = doubles(nw), *dw_old = doubles(nw);
        CHECK(conv_oracle_forward(x, xs, N, C, H, W, w, K, R, S, pad_h, pad_w, u, v, mode, 0.5, -1.5, y_old, y, ys, P, Q, 2));
        CHECK(conv_oracle_forward(x, xs, N, C, H, W, w, K, R, S, pad_h, pad_w, u, v, mode, 1.0, 0.0, NULL, y, ys, P, Q, 1));
        CHECK(conv_oracle_backward_data(w, K, C, R, S, dy, ys, N, P, Q, pad_h, pad_w, u, v, mode, 0.5, -1.5, dx_old, dx, xs, H, W, 2));
        CHECK(conv_oracle_backward_filter(x, xs, N, C, H, W, dy, ys, K, P, Q, pad_h, pad_w, u, v, mode, 0.5, -1.5, dw_old, dw, R, S, 2));
        /* the other functions on the x-shaped tensors */
        float *x2 = floats(nx), *x3 = floats(nx);
        for (int m = 0; m < 3; ++m) {
            CHECK(pointwise_oracle_activation_forward(m, x, xs, N, C, H, W, 1.0, 0.5, dx_old, dx, xs));
            CHECK(pointwise_oracle_activation_backward(m, x, xs, x2, xs, x3, xs, N, C, H, W, 1.0, 0.5, dx_old, dx, xs));
        }
        for (int m = 0; m < 2; ++m) {
            CHECK(pointwise_oracle_softmax_forward(m, x, xs, N, C, H, W, 1.0, 0.5, dx_old, dx, xs));
            CHECK(pointwise_oracle_softmax_backward(m, x, xs, x2, xs, N, C, H, W, 1.0, 0.5, dx_old, dx, xs));
        }
        {   /* a bias-shaped operand broadcast over n, h, w */
            long long bs[4] = {C, 1, 1, 1};
            float *b = floats(C);
            CHECK(pointwise_oracle_add_tensor(b, bs, 1, C, 1, 1, N, C, H, W, 2.0, 1.0, dx_old, dx, xs));
            free(b);
            double *db = doubles(C), *db_old = doubles(C);   /* and the gradient with respect to it */
            CHECK(pointwise_oracle_bias_backward(x, xs, N, C, H, W, 1.0, 0.5, db_old, db));
            free(db);
            free(db_old);
        }
        {   /* pooling with the convolution's window geometry */
            long long ps[4];
            strides(ps, C, P, Q, layout);
            const long long np_ = (long long)N * C * P * Q;
            float *pdy = floats(np_);
            double *py = doubles(np_), *py_old = doubles(np_), *scratch = doubles(nx);
            for (int m = 0; m < 2; ++m) {
                CHECK(pointwise_oracle_pooling_forward(m, x, xs, N, C, H, W, R, S, pad_h, pad_w, u, v, 1.0, 0.5, py_old, py, ps, P, Q));
                CHECK(pointwise_oracle_pooling_backward(m, x, xs, pdy, ps, N, C, H, W, R, S, pad_h, pad_w, u, v, 1.0, 0.5, dx_old, dx,
                                                        xs, P, Q, scratch));
            }
            free(pdy); free(py); free(py_old); free(scratch);
        }
        free(x); free(w); free(dy); free(y); free(y_old); free(dx); free(dx_old); free(dw); free(dw_old); free(x2); free(x3);
    }
    printf("oracle check ok\n");
    return 0;
}
